"""GPU parity tests of improved contractive error feedback, version 1 (Algorithm 3) with the quantiser twice and the
element-wise gradient compressors: the library, called through the C ABI, against oracle/iconef_ref.c on the same
seeded inputs, free-running over several steps (so the second vector written by one step is read by the next).
Every operation is element-wise fp32 arithmetic in a fixed order: kept values, sign words and both pairs of codes
and scales are compared bit for bit (the scaled sign's c to one unit in the last place, see test_gpu_scaledsign)."""
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
    import test_gpu_sketch as S

    B.lib()
    return R, B, S, torch


CASES = [
    # (layout, bits, block, kept fraction)
    ([(64, 128), (40, 512), (256, 96)], 4, 128, 0.1),          # whole power-of-two blocks: the wave-per-run kernel
    ([(64, 147), (37, 53), (128, 576)], 4, 128, 0.1),          # odd sizes: the kernel for any layout
    ([(32, 512), (100, 1024)], 2, 256, 0.25),
    ([(96, 160), (33, 129)], 8, 8, 0.5),
    ([(16, 64), (8, 8)], 4, 200, 1.0),                          # the whole matrix is kept: both vectors stay empty
    ([(77, 768), (5, 128), (129, 64)], 8, 64, 0.1),             # whole blocks, short last runs of 512
    ([(2000, 1024)], 4, 128, 0.01),                             # many items and partial sums
]


def _fresh(R, layout, bits, block):
    return [[np.zeros(R.n_words(n * m, bits), np.uint32), np.zeros(R.n_blocks(n * m, block), np.float32),
             np.zeros(R.n_words(n * m, bits), np.uint32), np.zeros(R.n_blocks(n * m, block), np.float32)] for n, m in layout]


def _second_buffers(torch, buf):
    return torch.zeros_like(buf["codes"]), torch.zeros_like(buf["scales"])


def _compare_state(buf, codes2, scales2, o, st, tag):
    c1, s1, c2, s2 = st
    for name, dev, want in (("first codes", buf["codes"], c1), ("second codes", codes2, c2)):
        got = dev[o["word_off"]:o["word_off"] + want.size].cpu().numpy().view(np.uint32)
        assert np.array_equal(got, want), f"{tag}: {name} differ in {(got != want).sum()} words"
    for name, dev, want in (("first scales", buf["scales"], s1), ("second scales", scales2, s2)):
        got = dev[o["scale_off"]:o["scale_off"] + want.size].cpu().numpy()
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), f"{tag}: {name}"


@pytest.mark.parametrize("case", range(len(CASES)))
@pytest.mark.parametrize("gdt", [wl.F32, wl.BF16])
def test_iconef_with_the_random_block_is_bit_exact(env, case, gdt):
    R, B, S, torch = env
    layout, bits, block, frac = CASES[case]
    seed = 1500 + case
    keep = wl.random_block_keep(layout, frac)
    model = B.Model(layout, 4, bits, block, gdt, seed)
    B.conef_rb_configure(model.ctx, keep)
    buf = model.alloc()
    codes2, scales2 = _second_buffers(torch, buf)
    delta = torch.zeros(B.conef_rb_sizes(model.ctx)["delta_elems"], dtype=torch.float32, device="cuda:0")
    rng = np.random.default_rng([case, gdt, 15])
    states = _fresh(R, layout, bits, block)
    live = False
    for t in range(4):
        grads = [S._grad(rng, n, m, gdt) for n, m in layout]
        S._to_dev_grads(torch, model, buf, grads)
        delta.fill_(float("nan"))
        print(f"[iconef random block case {case} gdt {gdt}] step {t}: launching", flush=True)
        B.conef_i_rb_step(model.ctx, buf["grads"], buf["codes"], buf["scales"], codes2, scales2, delta, t, model.stream_handle())
        torch.cuda.synchronize()
        for l, (n, m) in enumerate(layout):
            c1, s1, c2, s2 = states[l]
            want = R.i_rb_step_matrix(grads[l], c1, s1, c2, s2, keep[l], bits, block, seed, l, t)
            ro = B.conef_rb_offsets(model.ctx, l)
            got = delta[ro["delta_off"]:ro["delta_off"] + keep[l]].cpu().numpy()
            tag = f"case {case} mat {l} step {t}"
            assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), f"{tag}: kept values"
            _compare_state(buf, codes2, scales2, model.offsets[l], states[l], tag)
            live = live or bool(np.any(c2 != 0))
    assert live or frac == 1.0          # the second vector carried something from step to step
    model.close()


@pytest.mark.parametrize("case", [0, 1, 2, 3, 5, 6])
@pytest.mark.parametrize("gdt", [wl.F32, wl.BF16])
def test_iconef_with_the_scaled_sign(env, case, gdt):
    R, B, S, torch = env
    layout, bits, block, _ = CASES[case]
    seed = 1600 + case
    model = B.Model(layout, 4, bits, block, gdt, seed)
    buf = model.alloc()
    codes2, scales2 = _second_buffers(torch, buf)
    signs = torch.zeros(B.conef_ss_sizes(model.ctx)["sign_words"], dtype=torch.int32, device="cuda:0")
    cs = torch.zeros(len(layout), dtype=torch.float32, device="cuda:0")
    rng = np.random.default_rng([case, gdt, 16])
    states = _fresh(R, layout, bits, block)
    for t in range(4):
        grads = [S._grad(rng, n, m, gdt) for n, m in layout]
        S._to_dev_grads(torch, model, buf, grads)
        signs.fill_(-1)
        print(f"[iconef scaled sign case {case} gdt {gdt}] step {t}: launching", flush=True)
        B.conef_i_ss_step(model.ctx, buf["grads"], buf["codes"], buf["scales"], codes2, scales2, signs, cs, buf["ws"], t,
                          model.stream_handle())
        torch.cuda.synchronize()
        for l, (n, m) in enumerate(layout):
            c1, s1, c2, s2 = states[l]
            words, c = R.i_ss_step_matrix(grads[l], c1, s1, c2, s2, bits, block, seed, l, t)
            tag = f"case {case} mat {l} step {t}"
            o = model.offsets[l]
            got_c = cs[l].item()
            assert abs(float(got_c) - float(c)) <= float(np.spacing(np.float32(c))), f"{tag}: scale {got_c} vs {c}"
            if np.float32(got_c) != np.float32(c):
                # a last-bit difference of the scale changes every argument: go on from the library's state
                for dev, off, arr in ((buf["codes"], "word_off", c1), (buf["scales"], "scale_off", s1),
                                      (codes2, "word_off", c2), (scales2, "scale_off", s2)):
                    host = dev[o[off]:o[off] + arr.size].cpu().numpy()
                    arr[:] = host.view(arr.dtype)
                continue
            so = B.conef_ss_offsets(model.ctx, l)["sign_off"]
            N = n * m
            got = signs[so:so + words.size].cpu().numpy().view(np.uint32).copy()
            if N % 32:
                got[-1] &= np.uint32((1 << (N % 32)) - 1)
            assert np.array_equal(got, words), f"{tag}: sign bits"
            _compare_state(buf, codes2, scales2, o, states[l], tag)
    model.close()


def test_iconef_calls_reject_what_algorithm_3_does_not_define(env):
    R, B, S, torch = env
    qm = B.Model([(64, 64)], 4, 4, 64, wl.F32, 1)
    sk = B.SketchModel([(64, 64)], [16], 4, 0.0, 0, wl.F32, 1)
    qb, sb = qm.alloc(), sk.alloc()
    c2, s2 = _second_buffers(torch, qb)
    d = torch.zeros(4096, dtype=torch.float32, device="cuda:0")
    signs = torch.zeros(B.conef_ss_sizes(qm.ctx)["sign_words"], dtype=torch.int32, device="cuda:0")
    cs = torch.zeros(1, dtype=torch.float32, device="cuda:0")

    def rb(ctx=qm.ctx, codes2=c2, scales2=s2):
        B.conef_i_rb_step(ctx, qb["grads"], qb["codes"], qb["scales"], codes2, scales2, d, 0)

    def ss(ctx=qm.ctx, codes2=c2, scales2=s2):
        B.conef_i_ss_step(ctx, qb["grads"], qb["codes"], qb["scales"], codes2, scales2, signs, cs, qb["ws"], 0)

    with pytest.raises(B.ConefError) as e:          # before conef_rb_configure
        rb()
    assert e.value.code == B.ESTATE
    B.conef_rb_configure(qm.ctx, [100])
    B.conef_rb_configure(sk.ctx, [100])
    for call in (rb, ss):
        with pytest.raises(B.ConefError) as e:      # a count-sketch context
            call(ctx=sk.ctx)
        assert e.value.code == B.ESTATE
        with pytest.raises(B.ConefError) as e:      # the two vectors in one buffer
            call(codes2=qb["codes"])
        assert e.value.code == B.EINVAL
        with pytest.raises(B.ConefError) as e:
            call(scales2=qb["scales"])
        assert e.value.code == B.EINVAL
        B.conef_set_beta(qm.ctx, 0.5)               # Algorithm 3 has no partial update
        with pytest.raises(B.ConefError) as e:
            call()
        assert e.value.code == B.ESTATE
        B.conef_set_beta(qm.ctx, 0.0)
        call()
    torch.cuda.synchronize()
    assert np.isfinite(qb["scales"].cpu().numpy()).all() and np.isfinite(s2.cpu().numpy()).all()
    qm.close()
    sk.close()


@pytest.mark.parametrize("which", ["scaled_sign", "iconef_scaled_sign", "iconef_random_block", "random_k", "iconef_random_k"])
def test_stream_steps_replayed_from_a_hip_graph_equal_the_eager_steps(env, which):
    """The steps with an element-wise gradient compressor enqueue kernels only (the sign words that are set with
    atomic ORs are cleared by a kernel, not a memset), so they can be captured in a HIP graph.  Every replay, with
    eager work and synchronisations between the replays, must give the bits of the eager step."""
    R, B, S, torch = env
    layout, bits, block = [(64, 147), (128, 512), (37, 53)], 4, 128        # both kernel families
    model = B.Model(layout, 4, bits, block, wl.F32, 77)
    B.conef_rb_configure(model.ctx, wl.random_block_keep(layout, 0.1))
    B.conef_rk_configure(model.ctx, [10, 10, 7])
    buf = model.alloc()
    codes2, scales2 = _second_buffers(torch, buf)
    delta = torch.zeros(max(B.conef_rb_sizes(model.ctx)["delta_elems"], B.conef_rk_sizes(model.ctx)["delta_elems"]),
                        dtype=torch.float32, device="cuda:0")
    signs = torch.zeros(B.conef_ss_sizes(model.ctx)["sign_words"], dtype=torch.int32, device="cuda:0")
    cs = torch.zeros(len(layout), dtype=torch.float32, device="cuda:0")
    rng = np.random.default_rng(3)

    def launch(t, stream):
        a = (model.ctx, buf["grads"], buf["codes"], buf["scales"])
        if which == "scaled_sign":
            B.conef_ss_step(*a, signs, cs, buf["ws"], t, stream)
        elif which == "iconef_scaled_sign":
            B.conef_i_ss_step(*a, codes2, scales2, signs, cs, buf["ws"], t, stream)
        elif which == "iconef_random_block":
            B.conef_i_rb_step(*a, codes2, scales2, delta, t, stream)
        elif which == "random_k":
            B.conef_rk_step(*a, delta, t, stream)
        else:
            B.conef_i_rk_step(*a, codes2, scales2, delta, t, stream)

    state = {"codes": buf["codes"], "scales": buf["scales"], "codes2": codes2, "scales2": scales2}
    outs = dict(state, delta=delta, signs=signs, cs=cs)
    S._to_dev_grads(torch, model, buf, [S._grad(rng, n, m, wl.F32) for n, m in layout])
    launch(0, model.stream_handle())                 # also uploads the work tables
    torch.cuda.synchronize()
    before = {k: v.clone() for k, v in state.items()}
    S._to_dev_grads(torch, model, buf, [S._grad(rng, n, m, wl.F32) for n, m in layout])
    delta.fill_(float("nan"))                        # what the step does not write stays NaN
    launch(1, model.stream_handle())
    torch.cuda.synchronize()
    want = {k: v.clone() for k, v in outs.items()}
    s = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    for k in before:
        state[k].copy_(before[k])
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=s):
        launch(1, s.cuda_stream)
    for replay in range(3):
        for k in before:
            state[k].copy_(before[k])                # eager work between the replays
        delta.fill_(float("nan"))
        signs.fill_(-1)
        cs.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in want:
            if k == "delta":
                if "sign" in which:
                    continue                         # not written by these steps
                kept = ~torch.isnan(want[k])
                assert torch.equal(outs[k][kept], want[k][kept]), (which, replay, k)
            elif k == "signs" and "sign" in which:
                # bits beyond a matrix's last entry and the padding between matrices are unspecified
                for l, (n, m) in enumerate(layout):
                    so, full = B.conef_ss_offsets(model.ctx, l)["sign_off"], (n * m) // 32
                    assert torch.equal(outs[k][so:so + full], want[k][so:so + full]), (which, replay, k, l)
            elif k != "signs":
                assert torch.equal(outs[k], want[k]), (which, replay, k)
    model.close()
