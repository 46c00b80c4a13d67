"""GPU parity tests of the count sketch in the column form of the tensor trick (Section 5.3, "row or column"): the
library through the C ABI (conef_csc_init and the conef_cs_* step calls) against oracle/sketch_col_ref.c on the same
seeded inputs.  Estimate and update stage from identical inputs: bit for bit (element-wise fp32 arithmetic in a fixed
order); P and Q+ stages: 1e-6 relative (fp64 sums of exact products in another order); whole steps, each started from
the oracle's state: factors 1e-5, table entries within 2e-6 of the size of the terms they sum (plus one fp16 unit in the
last place for fp16 tables, rarely)."""
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
    import test_gpu_sketch as S

    B.lib()
    return R, B, U, S, torch


LAYOUTS = [
    # (layout, buckets per matrix (of its columns), rank)
    ([(37, 11), (64, 8), (300, 256)], [5, 8, 60], 4),              # as many buckets as columns: some stay empty
    ([(64, 147), (128, 576), (20, 33)], [13, 120, 1], 3),           # odd column counts, one bucket for a whole matrix
    ([(200, 520), (96, 1024)], [104, 200], 8),
    ([(130, 304), (40, 2048)], [60, 410], 32),
    ([(700, 72), (5, 4608)], [15, 922], 2),                         # more columns than threads of a workgroup several times over
]


def _table(rng, n, w, fp16):
    t = (rng.standard_normal((n, w)) * 0.05).astype(np.float32)
    return t.astype(np.float16).view(np.uint16) if fp16 else t


def _set_table(torch, model, buf, l, table):
    off = model.offsets[l]["table_off"]
    t = torch.from_numpy(table.ravel().view(np.int16)).view(torch.float16) if table.dtype == np.uint16 else torch.from_numpy(table.ravel())
    buf["table"][off:off + t.numel()] = t.to(buf["table"].device)


def _get_table(model, buf, l, n, w):
    off = model.offsets[l]["table_off"]
    t = buf["table"][off:off + n * w].cpu()
    if model.table_dtype == 1:
        return t.view(dtype=__import__("torch").int16).numpy().view(np.uint16).reshape(n, w)
    return t.numpy().reshape(n, w)


@pytest.mark.parametrize("case", range(len(LAYOUTS)))
@pytest.mark.parametrize("gdt", [wl.F32, wl.BF16])
@pytest.mark.parametrize("fp16", [False, True])
@pytest.mark.parametrize("beta", [0.0, 0.9])
def test_update_stage_and_estimate_are_bit_exact(env, case, gdt, fp16, beta):
    R, B, U, S, torch = env
    layout, ws, rank = LAYOUTS[case]
    seed = 6000 + case
    rng = np.random.default_rng([case, gdt, int(fp16), 60])
    model = B.SketchModel(layout, ws, rank, beta, int(fp16), gdt, seed, columns=True)
    B.conef_check_plan(model.ctx)
    buf = model.alloc()
    grads = [S._grad(rng, n, m, gdt) for n, m in layout]
    tables = [_table(rng, n, w, fp16) for w, (n, _) in zip(ws, layout)]
    Phs = [rng.standard_normal((n, rank)).astype(np.float32) / np.float32(np.sqrt(n)) for n, _ in layout]
    Qns = [(rng.standard_normal((m, rank)) * 0.1).astype(np.float32) for _, m in layout]
    S._to_dev_grads(torch, model, buf, grads)
    Qdev = torch.zeros_like(buf["Q"])
    for l in range(len(layout)):
        _set_table(torch, model, buf, l, tables[l])
        S._set_factor(torch, buf, "P", model.offsets[l]["p_off"], Phs[l])
        S._set_factor(torch, {"Q": Qdev}, "Q", model.offsets[l]["q_off"], Qns[l])
    e_dev = torch.zeros(model.sizes["grad_elems"], dtype=torch.float32, device="cuda:0")
    B.conef_cs_decode_error(model.ctx, buf["table"], e_dev, B.Model.stream_handle())
    torch.cuda.synchronize()
    print(f"[column sketch update case {case} gdt {gdt} fp16 {fp16} beta {beta}] launching", flush=True)
    B.conef_cs_step_err(model.ctx, buf["grads"], buf["table"], buf["P"], Qdev, buf["ws"], B.Model.stream_handle())
    torch.cuda.synchronize()
    for l, (n, m) in enumerate(layout):
        b, s = R.cs_hash(seed, l, m, ws[l])
        hb, hs = B.conef_cs_hash(model.ctx, l, m)
        assert np.array_equal(hb, b) and np.array_equal(hs, s) and model.offsets[l]["sketch_rows"] == ws[l]
        off = model.offsets[l]["grad_off"]
        e = e_dev[off:off + n * m].cpu().numpy().reshape(n, m)
        assert np.array_equal(e.view(np.uint32), R.csc_decode(tables[l], b, s, m).view(np.uint32)), f"estimate, mat {l}"
        x = R.residual(R.csc_form_p(grads[l], tables[l], b, s, beta), Phs[l], Qns[l])
        want = tables[l].copy()
        R.csc_update(x, b, s, beta, want)
        got = _get_table(model, buf, l, n, ws[l])
        assert np.array_equal(got.view(np.uint16 if fp16 else np.uint32), want.view(np.uint16 if fp16 else np.uint32)), \
            f"table of mat {l} ({n}x{m}, {ws[l]} buckets) differs in {(got != want).sum()} entries"
    model.close()


@pytest.mark.parametrize("case", range(len(LAYOUTS)))
@pytest.mark.parametrize("gdt,fp16", [(wl.F32, False), (wl.BF16, True)])
def test_factor_stages_match_the_oracle(env, case, gdt, fp16):
    R, B, U, S, torch = env
    layout, ws, rank = LAYOUTS[case]
    seed, beta = 7000 + case, 0.75
    rng = np.random.default_rng([7, case, gdt, 70])
    model = B.SketchModel(layout, ws, rank, beta, int(fp16), gdt, seed, columns=True)
    buf = model.alloc()
    grads = [S._grad(rng, n, m, gdt) for n, m in layout]
    tables = [_table(rng, n, w, fp16) for w, (n, _) in zip(ws, layout)]
    Qs = [rng.standard_normal((m, rank)).astype(np.float32) for _, m in layout]
    S._to_dev_grads(torch, model, buf, grads)
    for l in range(len(layout)):
        _set_table(torch, model, buf, l, tables[l])
        S._set_factor(torch, buf, "Q", model.offsets[l]["q_off"], Qs[l])
    st = B.Model.stream_handle()
    print(f"[column sketch factors case {case} gdt {gdt}] launching", flush=True)
    B.conef_cs_step_p(model.ctx, buf["grads"], buf["table"], buf["Q"], buf["P"], buf["ws"], st)
    torch.cuda.synchronize()
    ps, Phs = [], []
    for l, (n, m) in enumerate(layout):
        b, s = R.cs_hash(seed, l, m, ws[l])
        p = R.csc_form_p(grads[l], tables[l], b, s, beta)
        ps.append(p)
        assert U.rel_err(S._get_factor(buf, "P", model.offsets[l]["p_off"], n, rank), R.lowrank_P(p, Qs[l])) <= 1e-6
        Phs.append(R.orthonormalise(R.lowrank_P(p, Qs[l])))
        S._set_factor(torch, buf, "P", model.offsets[l]["p_off"], Phs[l])
    Qout = torch.zeros_like(buf["Q"])
    B.conef_cs_step_q(model.ctx, buf["grads"], buf["table"], buf["P"], Qout, buf["ws"], st)
    torch.cuda.synchronize()
    for l, (n, m) in enumerate(layout):
        got = S._get_factor({"Q": Qout}, "Q", model.offsets[l]["q_off"], m, rank)
        assert U.rel_err(got, R.lowrank_Q(ps[l], Phs[l])) <= 1e-6
    model.close()


@pytest.mark.parametrize("case", range(len(LAYOUTS)))
@pytest.mark.parametrize("gdt,fp16,beta", [(wl.F32, False, 0.0), (wl.BF16, True, 0.85)])
def test_steps_match_the_oracle(env, case, gdt, fp16, beta):
    """Four whole fused steps; before each, the library's state (table, Q) is set to the oracle's."""
    R, B, U, S, torch = env
    layout, ws, rank = LAYOUTS[case]
    seed = 8000 + case
    rng = np.random.default_rng([11, case, gdt, int(fp16), 80])
    model = B.SketchModel(layout, ws, rank, beta, int(fp16), gdt, seed, columns=True)
    buf = model.alloc()
    tables = [np.zeros((n, w), np.uint16 if fp16 else np.float32) for (n, _), w in zip(layout, ws)]
    Qs = [rng.standard_normal((m, rank)).astype(np.float32) for _, m in layout]
    for t in range(4):
        grads = [S._grad(rng, n, m, gdt) for n, m in layout]
        S._to_dev_grads(torch, model, buf, grads)
        for l in range(len(layout)):
            _set_table(torch, model, buf, l, tables[l])
            S._set_factor(torch, buf, "Q", model.offsets[l]["q_off"], Qs[l])
        print(f"[column sketch steps case {case} gdt {gdt} fp16 {fp16} beta {beta}] step {t}: launching", flush=True)
        model.step(buf)
        torch.cuda.synchronize()
        for l, (n, m) in enumerate(layout):
            before = tables[l].copy()
            Ph, Qn = R.csc_step_matrix(grads[l], tables[l], Qs[l], rank, beta, seed, l)
            Qs[l] = Qn
            tag = f"case {case} mat {l} step {t}"
            assert U.rel_err(S._get_factor(buf, "P", model.offsets[l]["p_off"], n, rank), Ph) <= 1e-5, tag
            assert U.rel_err(S._get_factor(buf, "Q", model.offsets[l]["q_off"], m, rank), Qn) <= 1e-5, tag
            # size of the terms a table entry is the sum of (a last-bit difference in a factor moves every term by ~1e-7 of its size)
            b, sg = R.cs_hash(seed, l, m, ws[l])
            x = R.residual(R.csc_form_p(grads[l], before, b, sg, beta), Ph, Qn)
            mag = np.zeros((n, ws[l]), np.float32)
            R.csc_update(np.abs(x), b, np.ones(m, np.int8), 0.0, mag)
            bf = before.view(np.float16).astype(np.float32) if fp16 else before
            mag = mag.astype(np.float64) + beta * np.abs(bf) + np.abs(Ph).max() * np.abs(Qn).max() * rank
            got = _get_table(model, buf, l, n, ws[l])
            gf = got.view(np.float16).astype(np.float32) if fp16 else got
            wf = tables[l].view(np.float16).astype(np.float32) if fp16 else tables[l]
            diff = np.abs(gf.astype(np.float64) - wf.astype(np.float64))
            if fp16:
                assert np.all(diff <= np.abs(wf) * 2.0 ** -10 + 2.0 ** -24 + 2e-6 * mag), f"{tag}: table"
                assert (got != tables[l]).mean() <= 5e-3, f"{tag}: {(got != tables[l]).mean()} of the table differs"
            else:
                assert np.all(diff <= 2e-6 * mag), f"{tag}: table differs by {diff.max()}"
    assert any(np.any(t != 0) for t in tables)
    model.close()


def test_column_form_refuses_what_it_cannot_serve(env):
    R, B, U, S, torch = env
    with pytest.raises(B.ConefError) as e:                       # more buckets than columns
        B.conef_csc_init([(64, 64)], [65], 4, 0.5, 0, wl.F32, 1)
    assert e.value.code == B.EINVAL
    with pytest.raises(B.ConefError) as e:                       # a row of the residual has to fit the workgroup's LDS
        B.conef_csc_init([(8, 16392)], [100], 4, 0.5, 0, wl.F32, 1)
    assert e.value.code == B.EINVAL
    sk = B.SketchModel([(64, 64)], [16], 4, 0.5, 0, wl.F32, 1, columns=True)
    sb = sk.alloc()
    B.conef_rb_configure(sk.ctx, [100])
    B.conef_rk_configure(sk.ctx, [10])
    d = torch.zeros(4096, dtype=torch.float32, device="cuda:0")
    for call in (lambda: B.conef_cs_rb_step(sk.ctx, sb["grads"], sb["table"], d, 0),
                 lambda: B.conef_cs_rk_step(sk.ctx, sb["grads"], sb["table"], d, 0)):
        with pytest.raises(B.ConefError) as e:
            call()
        assert e.value.code == B.ESTATE
    sk.close()
