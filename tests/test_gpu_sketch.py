"""GPU parity tests of the count-sketch mode (Section 4.2.2, Algorithm 4): the library, called through
the C ABI, against oracle/sketch_ref.c on the same seeded inputs.

  * update stage (Algorithm 4 line 9) from identical inputs: the table bit for bit (all of it is fp32
    arithmetic in a fixed order, rounded once to the table's type);
  * estimate of the error: bit for bit;
  * P and Q+ stages: fp64 sums of exact products rounded once -> relative error <= 1e-6;
  * whole steps, each from the oracle's state: factors to 1e-5; a table entry to 2e-6 of the size of
    the terms it is the sum of (fp32), plus one unit in the last place on at most 5e-3 of the entries
    (fp16): the factors the update sees may differ from the oracle's in their last bit.
"""
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


def _grad(rng, n, m, dtype, scale=0.05):
    x = (rng.standard_normal((n, m)) * scale).astype(np.float32)
    return x if dtype == wl.F32 else wl.f32_to_bf16_bits(x)


def _to_dev_grads(torch, model, buf, grads):
    for l, g in enumerate(grads):
        off = model.offsets[l]["grad_off"]
        if model.grad_dtype == wl.F32:
            t = torch.from_numpy(np.ascontiguousarray(g, np.float32).ravel())
        else:
            t = torch.from_numpy(np.ascontiguousarray(g, np.uint16).ravel().view(np.int16)).view(torch.bfloat16)
        buf["grads"][off:off + t.numel()] = t.to(buf["grads"].device)


def _set_table(torch, model, buf, l, table):
    off = model.offsets[l]["table_off"]
    if table.dtype == np.uint16:
        t = torch.from_numpy(table.ravel().view(np.int16)).view(torch.float16)
    else:
        t = torch.from_numpy(table.ravel())
    buf["table"][off:off + t.numel()] = t.to(buf["table"].device)


def _get_table(model, buf, l):
    off = model.offsets[l]["table_off"]
    w, m = model.sketch_rows[l], model.layout[l][1]
    t = buf["table"][off:off + w * m].cpu()
    if model.table_dtype == 1:
        return t.view(dtype=__import__("torch").int16).numpy().view(np.uint16).reshape(w, m)
    return t.numpy().reshape(w, m)


def _set_factor(torch, buf, key, off, a):
    t = torch.from_numpy(np.ascontiguousarray(a, np.float32).ravel())
    buf[key][off:off + t.numel()] = t.to(buf[key].device)


def _get_factor(buf, key, off, rows, r):
    return buf[key][off:off + rows * r].cpu().numpy().reshape(rows, r)


def _random_table(rng, w, m, fp16):
    t = (rng.standard_normal((w, m)) * 0.05).astype(np.float32)
    return t.astype(np.float16).view(np.uint16) if fp16 else t


def _linear_form(rank, gdt, fp16, m):
    """Matrices that the library updates in the sketch's linear form (rank 32, bf16 gradients, fp16 table, columns a
    multiple of 128: S+ = (beta + (1 - beta)|b|) S + C(g) - U Q+^T): other rounding points than the per-element form the
    oracle follows, so a table entry may come out one fp16 unit in the last place away."""
    return rank == 32 and gdt == wl.BF16 and fp16 and m % 128 == 0


def _one_fp16_ulp(got, want, max_frac, what):
    g16, w16 = got.view(np.uint16).astype(np.int32).ravel(), want.view(np.uint16).astype(np.int32).ravel()
    diff = np.nonzero(g16 != w16)[0]
    assert diff.size <= max(2, int(max_frac * w16.size)), f"{what}: {diff.size} of {w16.size} entries differ"
    gv, wv = got.view(np.float16).ravel().astype(np.float64), want.view(np.float16).ravel().astype(np.float64)
    ulp = np.spacing(np.abs(want.view(np.float16).ravel()[diff]).astype(np.float16)).astype(np.float64)
    assert np.all(np.abs(gv[diff] - wv[diff]) <= ulp), f"{what}: an entry differs by more than one unit in the last place"


LAYOUTS = [
    # (layout, sketch rows, rank)
    ([(37, 11), (64, 8), (300, 256)], [5, 64, 60], 4),
    ([(64, 147), (128, 576), (20, 33)], [13, 26, 1], 3),          # odd column counts, one bucket for a whole matrix
    ([(200, 520), (96, 1024)], [40, 77], 8),
    ([(130, 300), (70, 260)], [50, 70], 32),
    ([(48, 96)], [48], 12),                                        # as many buckets as rows: some stay empty
    ([(130, 304), (70, 264), (40, 2048)], [50, 70, 9], 32),        # whole octets per row: the matrix-core path at rank 32
    ([(100, 136), (333, 640)], [30, 100], 16),
    ([(1000, 1160), (64, 4608)], [200, 51], 4),                    # several row tiles and column chunks, ragged ends
    ([(700, 72)], [1], 2),                                         # one bucket: a long list of rows
]


@pytest.mark.parametrize("case", range(len(LAYOUTS)))
@pytest.mark.parametrize("gdt", [wl.F32, wl.BF16])
@pytest.mark.parametrize("fp16", [False, True])
@pytest.mark.parametrize("beta", [0.0, 0.9])
def test_update_stage_and_estimate_are_bit_exact(env, case, gdt, fp16, beta):
    R, B, U, torch = env
    layout, ws, rank = LAYOUTS[case]
    seed = 1000 + case
    rng = np.random.default_rng([case, gdt, int(fp16)])
    model = B.SketchModel(layout, ws, rank, beta, int(fp16), gdt, seed)
    B.conef_check_plan(model.ctx)
    buf = model.alloc()
    grads = [_grad(rng, n, m, gdt) for n, m in layout]
    tables = [_random_table(rng, w, m, fp16) for w, (_, m) in zip(ws, layout)]
    Phs = [rng.standard_normal((n, rank)).astype(np.float32) / np.float32(np.sqrt(n)) for n, _ in layout]
    Qns = [(rng.standard_normal((m, rank)) * 0.1).astype(np.float32) for _, m in layout]
    _to_dev_grads(torch, model, buf, grads)
    Qdev = torch.zeros_like(buf["Q"])
    for l in range(len(layout)):
        _set_table(torch, model, buf, l, tables[l])
        _set_factor(torch, buf, "P", model.offsets[l]["p_off"], Phs[l])
        _set_factor(torch, {"Q": Qdev}, "Q", model.offsets[l]["q_off"], Qns[l])
    # estimate of the error
    e_dev = torch.zeros(model.sizes["grad_elems"], dtype=torch.float32, device="cuda:0")
    B.conef_cs_decode_error(model.ctx, buf["table"], e_dev, B.Model.stream_handle())
    torch.cuda.synchronize()
    print(f"[sketch update case {case} gdt {gdt} fp16 {fp16} beta {beta}] launching", flush=True)
    B.conef_cs_step_err(model.ctx, buf["grads"], buf["table"], buf["P"], Qdev, buf["ws"], B.Model.stream_handle())
    torch.cuda.synchronize()
    for l, (n, m) in enumerate(layout):
        b, s = R.cs_hash(seed, l, n, ws[l])
        off = model.offsets[l]["grad_off"]
        e = e_dev[off:off + n * m].cpu().numpy().reshape(n, m)
        assert np.array_equal(e.view(np.uint32), R.cs_decode(tables[l], b, s, n).view(np.uint32)), f"estimate, mat {l}"
        p = R.cs_form_p(grads[l], tables[l], b, s, beta)
        x = R.residual(p, Phs[l], Qns[l])
        want = tables[l].copy()
        R.cs_update(x, b, s, beta, want)
        got = _get_table(model, buf, l)
        if _linear_form(rank, gdt, fp16, m):
            _one_fp16_ulp(got, want, 5e-3, f"table of mat {l} ({n}x{m}, {ws[l]} buckets)")
            continue
        assert np.array_equal(got.view(np.uint16 if fp16 else np.uint32), want.view(np.uint16 if fp16 else np.uint32)), \
            f"table of mat {l} ({n}x{m}, {ws[l]} buckets) differs in {(got != want).sum()} entries"


@pytest.mark.parametrize("case", range(len(LAYOUTS)))
@pytest.mark.parametrize("gdt,fp16", [(wl.F32, False), (wl.BF16, True)])
def test_factor_stages_match_the_oracle(env, case, gdt, fp16):
    R, B, U, torch = env
    layout, ws, rank = LAYOUTS[case]
    seed, beta = 2000 + case, 0.75
    rng = np.random.default_rng([7, case, gdt])
    model = B.SketchModel(layout, ws, rank, beta, int(fp16), gdt, seed)
    buf = model.alloc()
    grads = [_grad(rng, n, m, gdt) for n, m in layout]
    tables = [_random_table(rng, w, m, fp16) for w, (_, m) in zip(ws, layout)]
    Qs = [rng.standard_normal((m, rank)).astype(np.float32) for _, m in layout]
    _to_dev_grads(torch, model, buf, grads)
    for l in range(len(layout)):
        _set_table(torch, model, buf, l, tables[l])
        _set_factor(torch, buf, "Q", model.offsets[l]["q_off"], Qs[l])
    st = B.Model.stream_handle()
    print(f"[sketch factors case {case} gdt {gdt}] launching", flush=True)
    B.conef_cs_step_p(model.ctx, buf["grads"], buf["table"], buf["Q"], buf["P"], buf["ws"], st)
    torch.cuda.synchronize()
    ps, Phs = [], []
    for l, (n, m) in enumerate(layout):
        b, s = R.cs_hash(seed, l, n, ws[l])
        p = R.cs_form_p(grads[l], tables[l], b, s, beta)
        ps.append(p)
        assert U.rel_err(_get_factor(buf, "P", model.offsets[l]["p_off"], n, rank), R.lowrank_P(p, Qs[l])) <= 1e-6
        # the Q+ stage is given the oracle's orthonormal factor
        Phs.append(R.orthonormalise(R.lowrank_P(p, Qs[l])))
        _set_factor(torch, buf, "P", model.offsets[l]["p_off"], Phs[l])
    Qout = torch.zeros_like(buf["Q"])
    B.conef_cs_step_q(model.ctx, buf["grads"], buf["table"], buf["P"], Qout, buf["ws"], st)
    torch.cuda.synchronize()
    for l, (n, m) in enumerate(layout):
        got = _get_factor({"Q": Qout}, "Q", model.offsets[l]["q_off"], m, rank)
        assert U.rel_err(got, R.lowrank_Q(ps[l], Phs[l])) <= 1e-6


@pytest.mark.parametrize("case", range(len(LAYOUTS)))
@pytest.mark.parametrize("gdt,fp16,beta", [(wl.F32, False, 0.0), (wl.F32, True, 0.9), (wl.BF16, True, 0.85)])
def test_steps_match_the_oracle(env, case, gdt, fp16, beta):
    """Four whole steps; before each, the library's state (table, Q) is set to the oracle's, so that every
    step is compared on identical inputs."""
    R, B, U, torch = env
    layout, ws, rank = LAYOUTS[case]
    seed = 3000 + case
    rng = np.random.default_rng([11, case, gdt, int(fp16)])
    model = B.SketchModel(layout, ws, rank, beta, int(fp16), gdt, seed)
    buf = model.alloc()
    states = [R.SketchState.fresh(n, m, w, fp16, rng.standard_normal((m, rank)).astype(np.float32))
              for (n, m), w in zip(layout, ws)]
    for t in range(4):
        grads = [_grad(rng, n, m, gdt) for n, m in layout]
        _to_dev_grads(torch, model, buf, grads)
        for l, stt in enumerate(states):
            _set_table(torch, model, buf, l, stt.table)
            _set_factor(torch, buf, "Q", model.offsets[l]["q_off"], stt.Q)
        print(f"[sketch steps case {case} gdt {gdt} fp16 {fp16} beta {beta}] step {t}: launching", flush=True)
        model.step(buf)
        torch.cuda.synchronize()
        for l, ((n, m), stt) in enumerate(zip(layout, states)):
            before = stt.table.copy()
            Ph, Qn = R.cs_step_matrix(grads[l], stt, rank, beta, seed, l)
            tag = f"case {case} mat {l} step {t}"
            assert U.rel_err(_get_factor(buf, "P", model.offsets[l]["p_off"], n, rank), Ph) <= 1e-5, tag
            assert U.rel_err(_get_factor(buf, "Q", model.offsets[l]["q_off"], m, rank), Qn) <= 1e-5, tag
            # size of the terms a table entry is the sum of: beta |S| + sum over its bucket of |x| (a last-bit
            # difference in a factor moves every term by ~1e-7 of its size, whatever the sum cancels to)
            b, sg = R.cs_hash(seed, l, n, ws[l])
            x = R.residual(R.cs_form_p(grads[l], before, b, sg, beta), Ph, Qn)
            mag = np.zeros((ws[l], m), np.float32)
            R.cs_update(np.abs(x), b, np.ones(n, np.int8), 0.0, mag)
            bf = before.view(np.float16).astype(np.float32) if fp16 else before
            mag = mag.astype(np.float64) + beta * np.abs(bf) + np.abs(Ph).max() * np.abs(Qn).max() * rank
            got = _get_table(model, buf, l)
            gf = got.view(np.float16).astype(np.float32) if fp16 else got
            wf = stt.table.view(np.float16).astype(np.float32) if fp16 else stt.table
            diff = np.abs(gf.astype(np.float64) - wf.astype(np.float64))
            if fp16:
                # one unit in the last place of fp16 where the two roundings fall on different sides, rarely
                assert np.all(diff <= np.abs(wf) * 2.0 ** -10 + 2.0 ** -24 + 2e-6 * mag), f"{tag}: table"
                assert (got != stt.table).mean() <= 5e-3, f"{tag}: {(got != stt.table).mean()} of the table differs"
            else:
                assert np.all(diff <= 2e-6 * mag), f"{tag}: table differs by {diff.max()}"


def test_quantiser_calls_refuse_a_sketch_context_and_back(env):
    R, B, U, torch = env
    sk = B.SketchModel([(64, 64)], [16], 4, 0.5, 0, wl.F32, 1)
    qm = B.Model([(64, 64)], 4, 4, 64, wl.F32, 1)
    sb, qb = sk.alloc(), qm.alloc()
    with pytest.raises(B.ConefError) as e1:
        B.conef_step(sk.ctx, sb["grads"], sb["table"], sb["table"], sb["Q"], sb["P"], sb["Q"], sb["ws"], 0)
    assert e1.value.code == B.ESTATE
    with pytest.raises(B.ConefError) as e2:
        B.conef_cs_step(qm.ctx, qb["grads"], qb["codes"], qb["Q"], qb["P"], qb["Q"], qb["ws"])
    assert e2.value.code == B.ESTATE
    # the calls shared by both kinds of context work on a sketch context
    B.conef_orthonormalise(sk.ctx, sb["P"], sb["ws"])
    x = torch.zeros(sk.sizes["grad_elems"], dtype=torch.float32, device="cuda:0")
    B.conef_decompress(sk.ctx, sb["P"], sb["Q"], x)
    torch.cuda.synchronize()


def test_sketch_step_is_reproducible_and_replays_from_a_hip_graph(env):
    """After the first call on a context a count-sketch step only enqueues kernels, in a fixed summation
    order: two runs give the same bits, and a captured step replayed three times (with eager work and
    synchronisations in between) gives the bits of the eager step on the same inputs."""
    R, B, U, torch = env
    for layout, ws, rank, gdt, fp16 in [([(300, 256), (130, 384)], [60, 26], 32, wl.BF16, True),
                                        ([(64, 147), (128, 576)], [13, 26], 4, wl.F32, True),
                                        ([(200, 512)], [40], 8, wl.BF16, False)]:
        rng = np.random.default_rng(77)
        model = B.SketchModel(layout, ws, rank, 0.9, int(fp16), gdt, 31)
        b = model.alloc()
        for l, (n, m) in enumerate(layout):
            _set_factor(torch, b, "Q", model.offsets[l]["q_off"], rng.standard_normal((m, rank)).astype(np.float32))
        grads = [[_grad(rng, n, m, gdt) for n, m in layout] for _ in range(2)]
        _to_dev_grads(torch, model, b, grads[0]); model.step(b)          # also uploads the work tables
        before = {k: b[k].clone() for k in ("table", "Q")}
        _to_dev_grads(torch, model, b, grads[1]); model.step(b)
        torch.cuda.synchronize()
        want = {k: b[k].clone() for k in ("table", "Q", "P")}
        s = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        for k in before:
            b[k].copy_(before[k])
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=s):
            model.step(b)
        for replay in range(3):
            for k in before:
                b[k].copy_(before[k])            # eager work between the replays
            b["P"].zero_()
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for k in want:
                assert torch.equal(b[k].view(torch.uint8), want[k].view(torch.uint8)), (layout, replay, k)
        model.close()


def test_set_beta_on_a_sketch_context_equals_a_context_made_with_that_beta(env):
    R, B, U, torch = env
    layout, ws, rank = [(200, 520), (64, 147)], [40, 13], 4
    rng = np.random.default_rng(99)
    grads = [_grad(rng, n, m, wl.F32) for n, m in layout]
    tables = [_random_table(rng, w, m, True) for w, (_, m) in zip(ws, layout)]
    Qs = [rng.standard_normal((m, rank)).astype(np.float32) for _, m in layout]
    results = []
    for make in ("init", "set"):
        model = B.SketchModel(layout, ws, rank, 0.9 if make == "init" else 0.25, 1, wl.F32, 7)
        if make == "set":
            B.conef_set_beta(model.ctx, 0.9)
        buf = model.alloc()
        _to_dev_grads(torch, model, buf, grads)
        for l in range(len(layout)):
            _set_table(torch, model, buf, l, tables[l])
            _set_factor(torch, buf, "Q", model.offsets[l]["q_off"], Qs[l])
        model.step(buf)
        torch.cuda.synchronize()
        results.append({k: buf[k].clone() for k in ("table", "Q", "P")})
        model.close()
    for k in results[0]:
        assert torch.equal(results[0][k].view(torch.uint8), results[1][k].view(torch.uint8)), k
