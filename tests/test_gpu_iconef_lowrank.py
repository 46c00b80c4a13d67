"""GPU parity tests of improved contractive error feedback, version 1 (Algorithm 3, the quantiser twice) around the
rank-r compressor: the library through the C ABI against oracle/iconef_ref.c, free-running over several steps, in
the kernel families for whole blocks with rank 2/4/8 and for any shape, both gradient types; the bf16 matrix-core
family (rank 32) has a test of its own below, with the criteria of the plain step's matrix-core tests.

Per step and matrix: the gradient buffer is left as it was; the factors agree with the oracle's step from the same
state to 1e-5; and both new vectors are, bit for bit, the oracle's two error steps applied to the
residual formed from the library's own factors (the fp32 fma chain is the same on both sides, so nothing is left to
tolerance there).  The oracle then continues from the library's state."""
import numpy as np
import pytest

from paper_2312_08538_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from oracle import conef_ref as R
    from paper_2312_08538_amd import binding as B
    import parity_util as U

    B.lib()
    return R, B, U, torch


CASES = [
    # (layout, rank, bits, block)
    ([(128, 256), (64, 512), (300, 128)], 4, 4, 128),          # whole blocks, rank 4: the lane-per-octet kernels
    ([(64, 147), (37, 53), (130, 129)], 4, 4, 128),            # odd shapes: the kernels for any layout
    ([(96, 512), (200, 1024)], 8, 2, 256),
    ([(100, 192), (33, 64)], 2, 8, 64),
    ([(70, 200), (256, 384)], 12, 4, 200),                     # a rank outside 2/4/8 and an odd block length
    ([(500, 768), (64, 147)], 8, 8, 128),                      # both families in one model
    # bf16 gradients: the packed-split P and Q+ passes on the bf16 matrix cores, each vector's share in a launch of its own
    ([(300, 256), (77, 384), (1100, 128)], 4, 4, 128),         # an odd number of column blocks, partial sums of Q+
    ([(130, 1536), (520, 512)], 2, 2, 512),
]


@pytest.mark.parametrize("case", range(len(CASES)))
@pytest.mark.parametrize("gdt", [wl.F32, wl.BF16])
def test_iconef_with_the_rank_r_compressor(env, case, gdt):
    R, B, U, torch = env
    import test_gpu_sketch as S

    layout, rank, bits, block = CASES[case]
    seed, W = 3100 + case, 32 // bits
    model = B.Model(layout, rank, bits, block, gdt, seed)
    buf = model.alloc()
    codes2, scales2 = torch.zeros_like(buf["codes"]), torch.zeros_like(buf["scales"])
    rng = np.random.default_rng([case, 31])
    state = []
    for l, (n, m) in enumerate(layout):
        N = n * m
        Q0 = rng.standard_normal((m, rank)).astype(np.float32)
        state.append([np.zeros(R.n_words(N, bits), np.uint32), np.zeros(R.n_blocks(N, block), np.float32),
                      np.zeros(R.n_words(N, bits), np.uint32), np.zeros(R.n_blocks(N, block), np.float32), Q0])
        o = model.offsets[l]
        buf["Q"][o["q_off"]:o["q_off"] + Q0.size] = torch.from_numpy(Q0.ravel()).to("cuda:0")
    second_live = False
    for t in range(4):
        grads = [S._grad(rng, n, m, gdt) for n, m in layout]
        S._to_dev_grads(torch, model, buf, grads)
        g_before = buf["grads"].clone()
        print(f"[iconef rank-r case {case} gdt {gdt}] step {t}: launching", flush=True)
        B.conef_i_step(model.ctx, buf["grads"], buf["codes"], buf["scales"], codes2, scales2, buf["Q"], buf["P"], buf["Q"],
                       buf["ws"], t, model.stream_handle())
        torch.cuda.synchronize()
        for l, (n, m) in enumerate(layout):
            N, o = n * m, model.offsets[l]
            c1, s1, c2, s2, Q = state[l]
            tag = f"case {case} mat {l} step {t}"
            P_gpu = buf["P"][o["p_off"]:o["p_off"] + n * rank].cpu().numpy().reshape(n, rank)
            Q_gpu = buf["Q"][o["q_off"]:o["q_off"] + m * rank].cpu().numpy().reshape(m, rank)
            # the oracle's two error steps on the residual from the library's own factors: bit for bit
            p = R.i_form_p(grads[l], c1, s1, c2, s2, bits, block).reshape(n, m)
            own = [c1.copy(), s1.copy(), c2.copy(), s2.copy()]
            R.i_error(R.residual(p, P_gpu, Q_gpu), *own, bits, block, seed, l, t)
            # the oracle's whole step from the same state: factors to 1e-5
            Ph, Qn = R.i_step_matrix(grads[l], c1, s1, c2, s2, Q, rank, bits, block, seed, l, t)
            assert U.rel_err(P_gpu, Ph) <= 1e-5, f"{tag}: P^ {U.rel_err(P_gpu, Ph)}"
            assert U.rel_err(Q_gpu, Qn) <= 1e-5, f"{tag}: Q+ {U.rel_err(Q_gpu, Qn)}"
            got = [buf["codes"][o["word_off"]:o["word_off"] + c1.size].cpu().numpy().view(np.uint32),
                   buf["scales"][o["scale_off"]:o["scale_off"] + s1.size].cpu().numpy(),
                   codes2[o["word_off"]:o["word_off"] + c2.size].cpu().numpy().view(np.uint32),
                   scales2[o["scale_off"]:o["scale_off"] + s2.size].cpu().numpy()]
            for name, g_, w_ in zip(("first codes", "first scales", "second codes", "second scales"), got, own):
                assert np.array_equal(g_.view(np.uint32), w_.view(np.uint32)), \
                    f"{tag}: {name} differ in {(g_.view(np.uint32) != w_.view(np.uint32)).sum()} of {w_.size}"
            second_live = second_live or bool(np.any(got[2] != 0))
            # the oracle goes on from the library's state
            state[l] = [got[0].copy(), got[1].copy(), got[2].copy(), got[3].copy(), Q_gpu.copy()]
        assert torch.equal(buf["grads"], g_before)          # the gradients are read only
    assert second_live
    model.close()


def test_staged_calls_give_the_fused_step(env):
    R, B, U, torch = env
    layout, rank, bits, block = [(128, 256), (64, 147)], 4, 4, 128
    rng = np.random.default_rng(5)
    outs = []
    for staged in (False, True):
        model = B.Model(layout, rank, bits, block, wl.F32, 9)
        buf = model.alloc()
        c2, s2 = torch.zeros_like(buf["codes"]), torch.zeros_like(buf["scales"])
        r2 = np.random.default_rng(6)
        buf["Q"].copy_(torch.from_numpy(r2.standard_normal(buf["Q"].numel()).astype(np.float32)).to("cuda:0"))
        for t in range(3):
            buf["grads"].copy_(torch.from_numpy(r2.standard_normal(buf["grads"].numel()).astype(np.float32)).to("cuda:0"))
            a = (model.ctx, buf["grads"], buf["codes"], buf["scales"])
            if staged:
                B.conef_i_step_p(*a, c2, s2, buf["Q"], buf["P"], buf["ws"])
                B.conef_orthonormalise(model.ctx, buf["P"], buf["ws"])
                B.conef_i_step_q(*a, c2, s2, buf["P"], buf["Q"], buf["ws"])
                B.conef_i_step_err(*a, c2, s2, buf["P"], buf["Q"], buf["ws"], t)
            else:
                B.conef_i_step(*a, c2, s2, buf["Q"], buf["P"], buf["Q"], buf["ws"], t)
        torch.cuda.synchronize()
        outs.append([x.clone() for x in (buf["codes"], buf["scales"], c2, s2, buf["Q"], buf["P"])])
        model.close()
    for a, b in zip(*outs):
        assert torch.equal(a, b)


MFMA_LAYOUTS = [
    [(300, 256), (2200, 128), (45, 384)],           # ragged 128-row and 16-row tiles, more than one row tile of the Q+ pass
    [(421, 1536), (128, 2304)],                     # runs of column blocks that are not a whole 16, an odd number of blocks
]


@pytest.mark.parametrize("case", range(len(MFMA_LAYOUTS)))
def test_iconef_with_the_rank_r_compressor_on_the_matrix_cores(env, case):
    """The bf16 matrix-core family (rank 32, bf16 gradients, 4-bit codes, blocks of 128).  Its factors are fp32 sums of
    exact bf16 products, so, as for the plain step, nothing is bit for bit: per step and matrix the factors agree with
    the oracle's step from the same state; the first vector is the oracle's quantisation of the residual formed from
    the library's own factors, scales to 1e-6 (of the larger of the scale and the terms of the reconstruction) and
    codes under the boundary rule; the second vector is judged the same way against the oracle's quantisation (random
    stream mat | 2^31) of that residual minus the LIBRARY's decoded first vector, so that a first code excused at a
    boundary does not count again (the block's largest element leaves a difference of the size of its own rounding
    error there, so the windows of the second vector are relative to the first vector's magnitudes).  The oracle then
    continues from the library's state."""
    R, B, U, torch = env
    import test_gpu_sketch as S

    layout, rank, bits, block = MFMA_LAYOUTS[case], 32, 4, 128
    seed = 4100 + case
    model = B.Model(layout, rank, bits, block, wl.BF16, seed)
    buf = model.alloc()
    codes2, scales2 = torch.zeros_like(buf["codes"]), torch.zeros_like(buf["scales"])
    rng = np.random.default_rng([case, 41])
    state = []
    for l, (n, m) in enumerate(layout):
        N = n * m
        Q0 = rng.standard_normal((m, rank)).astype(np.float32)
        state.append([np.zeros(R.n_words(N, bits), np.uint32), np.zeros(R.n_blocks(N, block), np.float32),
                      np.zeros(R.n_words(N, bits), np.uint32), np.zeros(R.n_blocks(N, block), np.float32), Q0])
        o = model.offsets[l]
        buf["Q"][o["q_off"]:o["q_off"] + Q0.size] = torch.from_numpy(Q0.ravel()).to("cuda:0")
    excused, second_live = 0, False
    for t in range(3):
        grads = [S._grad(rng, n, m, wl.BF16) for n, m in layout]
        S._to_dev_grads(torch, model, buf, grads)
        g_before = buf["grads"].clone()
        print(f"[iconef rank-32 case {case}] step {t}: launching", flush=True)
        B.conef_i_step(model.ctx, buf["grads"], buf["codes"], buf["scales"], codes2, scales2, buf["Q"], buf["P"], buf["Q"],
                       buf["ws"], t, model.stream_handle())
        torch.cuda.synchronize()
        for l, (n, m) in enumerate(layout):
            N, o = n * m, model.offsets[l]
            c1, s1, c2, s2, Q = state[l]
            tag = f"rank-32 case {case} mat {l} step {t}"
            P_gpu = buf["P"][o["p_off"]:o["p_off"] + n * rank].cpu().numpy().reshape(n, rank)
            Q_gpu = buf["Q"][o["q_off"]:o["q_off"] + m * rank].cpu().numpy().reshape(m, rank)
            got = [buf["codes"][o["word_off"]:o["word_off"] + c1.size].cpu().numpy().view(np.uint32),
                   buf["scales"][o["scale_off"]:o["scale_off"] + s1.size].cpu().numpy(),
                   codes2[o["word_off"]:o["word_off"] + c2.size].cpu().numpy().view(np.uint32),
                   scales2[o["scale_off"]:o["scale_off"] + s2.size].cpu().numpy()]
            Ph, Qn = R.i_step_matrix(grads[l], c1.copy(), s1.copy(), c2.copy(), s2.copy(), Q, rank, bits, block, seed, l, t)
            assert U.rel_err(P_gpu, Ph) <= 1e-4, f"{tag}: P^ {U.rel_err(P_gpu, Ph)}"
            assert U.rel_err(Q_gpu, Qn) <= 1e-4, f"{tag}: Q+ {U.rel_err(Q_gpu, Qn)}"
            p = R.i_form_p(grads[l], c1, s1, c2, s2, bits, block).reshape(n, m)
            x = R.residual(p, P_gpu, Q_gpu).ravel()
            rec = (np.abs(P_gpu).astype(np.float64) @ np.abs(Q_gpu).astype(np.float64).T).astype(np.float32).ravel()
            blk_rec = rec.reshape(-1, block).max(1)
            # first error step
            w1, ws1 = R.quantise(x, bits, block, seed, l, t)
            assert np.all(np.abs(got[1] - ws1) <= 1e-6 * np.maximum(ws1, blk_rec)), f"{tag}: first scales"
            excused += U.check_codes(got[0], w1, x, N, bits, block, seed, l, t, tag + " first", rec_oracle=rec)
            # second error step, from the library's own first vector
            x2 = x - R.decode(got[0], got[1], N, bits, block).ravel()
            w2, ws2 = R.quantise(x2, bits, block, seed, l | 0x80000000, t)
            # ... whose argument is a difference of terms as large as the residual itself (about 7 of its own levels):
            # the 1e-6 windows are taken relative to the largest term, here the first vector's block max-norm, and
            # doubled, the argument being two fp32 roundings away from those terms (the residual, then the subtraction)
            terms = 2.0 * np.maximum(rec, np.abs(x))
            assert np.all(np.abs(got[3] - ws2) <= 1e-6 * np.maximum(ws2, terms.reshape(-1, block).max(1))), f"{tag}: second scales"
            excused += U.check_codes(got[2], w2, x2, N, bits, block, seed, l | 0x80000000, t, tag + " second", rec_oracle=terms)
            second_live = second_live or bool(np.any(got[2] != 0))
            state[l] = [got[0].copy(), got[1].copy(), got[2].copy(), got[3].copy(), Q_gpu.copy()]
        assert torch.equal(buf["grads"], g_before)
    assert second_live
    print(f"[iconef rank-32 case {case}] excused codes: {excused}", flush=True)
    model.close()


def test_staged_calls_give_the_fused_step_on_the_matrix_cores(env):
    R, B, U, torch = env
    layout = [(300, 256), (2100, 128)]
    outs = []
    for staged in (False, True):
        model = B.Model(layout, 32, 4, 128, wl.BF16, 9)
        buf = model.alloc()
        c2, s2 = torch.zeros_like(buf["codes"]), torch.zeros_like(buf["scales"])
        r2 = np.random.default_rng(6)
        buf["Q"].copy_(torch.from_numpy(r2.standard_normal(buf["Q"].numel()).astype(np.float32)).to("cuda:0"))
        for t in range(3):
            g = torch.from_numpy(r2.standard_normal(buf["grads"].numel()).astype(np.float32)).to("cuda:0")
            buf["grads"].copy_(g.to(buf["grads"].dtype))
            a = (model.ctx, buf["grads"], buf["codes"], buf["scales"])
            if staged:
                B.conef_i_step_p(*a, c2, s2, buf["Q"], buf["P"], buf["ws"])
                B.conef_orthonormalise(model.ctx, buf["P"], buf["ws"])
                B.conef_i_step_q(*a, c2, s2, buf["P"], buf["Q"], buf["ws"])
                buf["ws"].zero_()           # the err stage call relies on nothing left in the workspace
                B.conef_i_step_err(*a, c2, s2, buf["P"], buf["Q"], buf["ws"], t)
            else:
                B.conef_i_step(*a, c2, s2, buf["Q"], buf["P"], buf["Q"], buf["ws"], t)
        torch.cuda.synchronize()
        outs.append([x.clone() for x in (buf["codes"], buf["scales"], c2, s2, buf["Q"], buf["P"])])
        assert bool(torch.any(c2 != 0))
        model.close()
    for a, b in zip(*outs):
        assert torch.equal(a, b)


def test_rank_r_iconef_calls_reject_what_they_cannot_serve(env):
    R, B, U, torch = env
    m = B.Model([(64, 64)], 4, 4, 64, wl.F32, 1)
    buf = m.alloc()
    c2, s2 = torch.zeros_like(buf["codes"]), torch.zeros_like(buf["scales"])
    B.conef_set_beta(m.ctx, 0.5)
    with pytest.raises(B.ConefError) as e:          # Algorithm 3 has no partial update
        B.conef_i_step(m.ctx, buf["grads"], buf["codes"], buf["scales"], c2, s2, buf["Q"], buf["P"], buf["Q"], buf["ws"], 0)
    assert e.value.code == B.ESTATE
    B.conef_set_beta(m.ctx, 0.0)
    with pytest.raises(B.ConefError) as e:          # the two vectors in one buffer
        B.conef_i_step(m.ctx, buf["grads"], buf["codes"], buf["scales"], buf["codes"], s2, buf["Q"], buf["P"], buf["Q"], buf["ws"], 0)
    assert e.value.code == B.EINVAL
    m.close()
    sk = B.SketchModel([(64, 64)], [16], 4, 0.0, 0, wl.F32, 1)
    sb = sk.alloc()
    with pytest.raises(B.ConefError) as e:
        B.conef_i_step_p(sk.ctx, sb["grads"], sb["table"], sb["table"], sb["P"], sb["P"], sb["Q"], sb["P"], sb["ws"])
    assert e.value.code == B.ESTATE
    sk.close()


@pytest.mark.parametrize("name", ["lm", "translation"])
def test_whole_model_second_step_against_the_oracle(env, name):
    """Every matrix of the `lm` (123.5 M fp32 elements, rank 4) and `translation` (209.7 M bf16 elements, rank 8, 2-bit
    codes) workloads, whole, in the launch configuration `bench.py` times for this step: the library's second step
    against the oracle started from the state the library held before it."""
    R, B, U, torch = env
    w = wl.WORKLOADS[name]
    bits, block, rank, seed, W = w.bits, w.block, w.rank, w.lib_seed, 32 // w.bits
    model = B.Model(w.layout, rank, bits, block, w.grad_dtype, seed)
    buf = model.alloc()
    codes2, scales2 = torch.zeros_like(buf["codes"]), torch.zeros_like(buf["scales"])
    goffs = [o["grad_off"] for o in model.offsets]
    wl.device_q0(w, buf["Q"], [o["q_off"] for o in model.offsets])

    def step(t):
        print(f"[iconef rank-r {name}] step {t}: launching", flush=True)
        B.conef_i_step(model.ctx, buf["grads"], buf["codes"], buf["scales"], codes2, scales2, buf["Q"], buf["P"], buf["Q"],
                       buf["ws"], t, model.stream_handle())
        torch.cuda.synchronize()

    def download():
        return [buf["codes"].cpu().numpy().view(np.uint32), buf["scales"].cpu().numpy(),
                codes2.cpu().numpy().view(np.uint32), scales2.cpu().numpy()]

    wl.device_fill_gradients(w, 0, buf["grads"], goffs)
    step(0)
    before, Q0 = download(), buf["Q"].cpu().numpy()
    wl.device_fill_gradients(w, 1, buf["grads"], goffs)
    g_dev = buf["grads"].view(torch.int16) if w.grad_dtype == wl.BF16 else buf["grads"]
    g_all = g_dev.cpu().numpy().view(np.uint16 if w.grad_dtype == wl.BF16 else np.float32)
    step(1)
    after, P1, Q1 = download(), buf["P"].cpu().numpy(), buf["Q"].cpu().numpy()
    assert np.any(before[2] != 0)
    for l, (n, m) in enumerate(w.layout):
        o, N = model.offsets[l], n * m
        nw, nb = -(-N // W), -(-N // block)
        g = g_all[o["grad_off"]:o["grad_off"] + N].reshape(n, m)
        st = [before[i][(o["word_off"] if i % 2 == 0 else o["scale_off"]):][:(nw if i % 2 == 0 else nb)].copy() for i in range(4)]
        P_gpu = P1[o["p_off"]:o["p_off"] + n * rank].reshape(n, rank)
        Q_gpu = Q1[o["q_off"]:o["q_off"] + m * rank].reshape(m, rank)
        own = [a.copy() for a in st]
        R.i_error(R.residual(R.i_form_p(g, *st, bits, block).reshape(n, m), P_gpu, Q_gpu), *own, bits, block, seed, l, 1)
        Ph, Qn = R.i_step_matrix(g, *st, Q0[o["q_off"]:o["q_off"] + m * rank].reshape(m, rank), rank, bits, block, seed, l, 1)
        tag = f"{name} mat {l} ({n}x{m})"
        assert U.rel_err(P_gpu, Ph) <= 1e-5 and U.rel_err(Q_gpu, Qn) <= 1e-5, f"{tag}: factors"
        for i, what in enumerate(("first codes", "first scales", "second codes", "second scales")):
            off, cnt = (o["word_off"], nw) if i % 2 == 0 else (o["scale_off"], nb)
            got = after[i][off:off + cnt]
            assert np.array_equal(got.view(np.uint32), own[i].view(np.uint32)), \
                f"{tag}: {what} differ in {(got.view(np.uint32) != own[i].view(np.uint32)).sum()} of {cnt}"
    print(f"[iconef rank-r {name}] all {len(w.layout)} matrices: both error vectors bit for bit", flush=True)
    model.close()


def test_large_whole_model_second_step_on_the_matrix_cores(env):
    """Every matrix of `large` (1.31 G bf16 elements, rank 32), whole, in the launch configuration `bench.py` times for
    this step: the library's second iConEF step against the oracle started from the state the library held before it.
    Criteria of the matrix-core family (see the test above): factors to 1e-4, both vectors under the boundary rule, the
    second one against the oracle's second error step on the residual minus the library's own decoded first vector."""
    R, B, U, torch = env
    w = wl.WORKLOADS["large"]
    bits, block, rank, seed, W = w.bits, w.block, w.rank, w.lib_seed, 32 // w.bits
    model = B.Model(w.layout, rank, bits, block, w.grad_dtype, seed)
    buf = model.alloc()
    codes2, scales2 = torch.zeros_like(buf["codes"]), torch.zeros_like(buf["scales"])
    goffs = [o["grad_off"] for o in model.offsets]
    wl.device_q0(w, buf["Q"], [o["q_off"] for o in model.offsets])

    def step(t):
        print(f"[iconef rank-32 large] step {t}: launching", flush=True)
        B.conef_i_step(model.ctx, buf["grads"], buf["codes"], buf["scales"], codes2, scales2, buf["Q"], buf["P"], buf["Q"],
                       buf["ws"], t, model.stream_handle())
        torch.cuda.synchronize()

    def download():
        return [buf["codes"].cpu().numpy().view(np.uint32), buf["scales"].cpu().numpy(),
                codes2.cpu().numpy().view(np.uint32), scales2.cpu().numpy()]

    wl.device_fill_gradients(w, 0, buf["grads"], goffs)
    step(0)
    before, Q0 = download(), buf["Q"].cpu().numpy()
    wl.device_fill_gradients(w, 1, buf["grads"], goffs)
    g_all = buf["grads"].view(torch.int16).cpu().numpy().view(np.uint16)
    step(1)
    after, P1, Q1 = download(), buf["P"].cpu().numpy(), buf["Q"].cpu().numpy()
    assert np.any(before[2] != 0)
    excused, stats = 0, {}
    for l, (n, m) in enumerate(w.layout):
        o, N = model.offsets[l], n * m
        nw, nb = -(-N // W), -(-N // block)
        g = g_all[o["grad_off"]:o["grad_off"] + N].reshape(n, m)
        st = [before[i][(o["word_off"] if i % 2 == 0 else o["scale_off"]):][:(nw if i % 2 == 0 else nb)].copy() for i in range(4)]
        got = [after[i][(o["word_off"] if i % 2 == 0 else o["scale_off"]):][:(nw if i % 2 == 0 else nb)] for i in range(4)]
        P_gpu = P1[o["p_off"]:o["p_off"] + n * rank].reshape(n, rank)
        Q_gpu = Q1[o["q_off"]:o["q_off"] + m * rank].reshape(m, rank)
        tag = f"large mat {l} ({n}x{m})"
        Ph, Qn = R.i_step_matrix(g, *[a.copy() for a in st], Q0[o["q_off"]:o["q_off"] + m * rank].reshape(m, rank), rank, bits,
                                 block, seed, l, 1)
        assert U.rel_err(P_gpu, Ph) <= 1e-4 and U.rel_err(Q_gpu, Qn) <= 1e-4, f"{tag}: factors"
        x = R.residual(R.i_form_p(g, *st, bits, block).reshape(n, m), P_gpu, Q_gpu).ravel()
        rec = (np.abs(P_gpu).astype(np.float64) @ np.abs(Q_gpu).astype(np.float64).T).astype(np.float32).ravel()
        w1, ws1 = R.quantise(x, bits, block, seed, l, 1)
        assert np.all(np.abs(got[1] - ws1) <= 1e-6 * np.maximum(ws1, rec.reshape(-1, block).max(1))), f"{tag}: first scales"
        excused += U.check_codes_sparse(got[0], w1, lambda: x, N, bits, block, seed, l, 1, tag + " first", rec_of=lambda: rec,
                                        stats=stats)
        x2 = x - R.decode(got[0], got[1], N, bits, block).ravel()
        w2, ws2 = R.quantise(x2, bits, block, seed, l | 0x80000000, 1)
        terms = 2.0 * np.maximum(rec, np.abs(x))          # (see the test above)
        assert np.all(np.abs(got[3] - ws2) <= 1e-6 * np.maximum(ws2, terms.reshape(-1, block).max(1))), f"{tag}: second scales"
        excused += U.check_codes_sparse(got[2], w2, lambda: x2, N, bits, block, seed, l | 0x80000000, 1, tag + " second",
                                        rec_of=lambda: terms, stats=stats)
        if l < 3:
            print(f"[iconef rank-32 large] {tag}: within the criteria", flush=True)
    print(f"[iconef rank-32 large] all {len(w.layout)} matrices; codes excused at a rounding boundary: {excused} of "
          f"{2 * w.elements} ({stats})", flush=True)
    assert excused <= 1e-5 * 2 * w.elements
    model.close()
