"""Parity at full size, in the launch configuration `bench.py` times: the `large` workload (1.31 G elements,
rank 32, bf16 gradients) checked on sampled outputs that the oracle can compute one by one from the inputs
the library saw (downloaded from the device), and whole models (`large`, `translation`, `lm`) against one
oracle step per matrix.  Sampled:

  * sampled rows of the raw P of the step's first stage,
  * the whole orthonormal factor of sampled matrices (orthonormal, same span as the raw P),
  * sampled rows of Q+ (each needs one column of the gradient and of the error state),
  * the new error state of sampled rows (quantiser) or sampled buckets (count sketch), computed by the
    oracle from the library's own factors.

Inputs are the benchmark's device-side generators; the step checked is the second one, so that the error
state it decodes is not zero.
"""
import numpy as np
import pytest

from paper_2312_08538_amd import workloads as wl

pytestmark = pytest.mark.gpu

MATS = [0, 3, 4, 94]                  # 50304 x 2048, 2048 x 8192, 8192 x 2048, 2048 x 2048
ROWS_PER_MAT = 3
COLS_PER_MAT = 3


@pytest.fixture(scope="module")
def env():
    import torch

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from oracle import conef_ref as R
    from paper_2312_08538_amd import binding as B
    import parity_util as U

    B.lib()
    return R, B, U, torch


def _rows(rng, n, k):
    return sorted(set([0, n - 1] + [int(x) for x in rng.integers(0, n, k)]))


def _grad_rows(torch, buf, off, m, rows):
    """bf16 gradient rows as uint16 bit patterns, shape (len(rows), m)."""
    idx = torch.tensor(rows, device=buf.device)
    g = buf[off:].view(torch.int16)[: (max(rows) + 1) * m].view(-1, m)[idx]
    return g.cpu().numpy().view(np.uint16)


def _grad_col(torch, buf, off, n, m, k):
    return buf[off:off + n * m].view(torch.int16).view(n, m)[:, k].cpu().numpy().view(np.uint16)


def test_large_quantiser_step_on_sampled_outputs(env):
    R, B, U, torch = env
    w = wl.WORKLOADS["large"]
    bits, block, rank, W = w.bits, w.block, w.rank, 32 // w.bits
    model = B.Model(w.layout, rank, bits, block, w.grad_dtype, w.lib_seed)
    buf = model.alloc()
    st = model.stream_handle()
    goffs = [o["grad_off"] for o in model.offsets]
    wl.device_q0(w, buf["Q"], [o["q_off"] for o in model.offsets])
    wl.device_fill_gradients(w, 0, buf["grads"], goffs)
    print("[fullsize quantiser] step 0", flush=True)
    model.step(buf, 0)
    wl.device_fill_gradients(w, 1, buf["grads"], goffs)
    torch.cuda.synchronize()
    codes0, scales0, Q0 = buf["codes"].clone(), buf["scales"].clone(), buf["Q"].clone()
    print("[fullsize quantiser] step 1, stage by stage", flush=True)
    B.conef_step_p(model.ctx, buf["grads"], buf["codes"], buf["scales"], buf["Q"], buf["P"], buf["ws"], st)
    torch.cuda.synchronize()
    Praw = buf["P"].clone()
    B.conef_orthonormalise(model.ctx, buf["P"], buf["ws"], st)
    B.conef_step_q(model.ctx, buf["grads"], buf["codes"], buf["scales"], buf["P"], buf["Q"], buf["ws"], st)
    B.conef_step_err(model.ctx, buf["grads"], buf["codes"], buf["scales"], buf["P"], buf["Q"], buf["ws"], 1, st)
    torch.cuda.synchronize()
    rng = np.random.default_rng(2024)
    inv_s = np.float32(1.0 / R.levels(bits))
    for l in MATS:
        n, m = w.layout[l]
        o = model.offsets[l]
        Qs = Q0[o["q_off"]:o["q_off"] + m * rank].cpu().numpy().reshape(m, rank)
        Pr = Praw[o["p_off"]:o["p_off"] + n * rank].cpu().numpy().reshape(n, rank)
        Ph = buf["P"][o["p_off"]:o["p_off"] + n * rank].cpu().numpy().reshape(n, rank)
        Qn = buf["Q"][o["q_off"]:o["q_off"] + m * rank].cpu().numpy().reshape(m, rank)
        # the orthonormal factor: orthonormal columns, and the raw P lies in its span
        G = Ph.astype(np.float64).T @ Ph.astype(np.float64)
        assert np.abs(G - np.eye(rank)).max() <= 1e-5, f"mat {l}: P^ not orthonormal"
        proj = Ph.astype(np.float64) @ (Ph.astype(np.float64).T @ Pr.astype(np.float64))
        assert np.abs(proj - Pr).max() <= 1e-5 * np.abs(Pr).max(), f"mat {l}: raw P outside the span of P^"
        rows = _rows(rng, n, ROWS_PER_MAT)
        g_rows = _grad_rows(torch, buf["grads"], o["grad_off"], m, rows)
        for gi, i in enumerate(rows):
            wo, so = o["word_off"] + i * m // W, o["scale_off"] + i * m // block
            c_old = codes0[wo:wo + m // W].cpu().numpy().view(np.uint32)
            s_old = scales0[so:so + m // block].cpu().numpy()
            p = R.form_p(g_rows[gi:gi + 1], c_old, s_old, bits, block)              # 1 x m, fp32
            # raw P row
            want = p.astype(np.float64) @ Qs.astype(np.float64)
            assert np.abs(Pr[i] - want[0]).max() <= 2e-2 * np.abs(Pr).max(), f"mat {l} row {i}: raw P"
            assert np.abs(Pr[i] - want[0]).max() <= 1e-5 * np.abs(Pr).max(), f"mat {l} row {i}: raw P (achieved level)"
            # new error state of the row from the library's own factors
            x = R.residual(p, Ph[i:i + 1], Qn)
            draws = np.array([R.rand16(w.lib_seed, l, 1, i * m + k) for k in range(m)], np.uint16)
            c_want, s_want = R.quantise(x, bits, block, draw=draws)
            c_got = buf["codes"][wo:wo + m // W].cpu().numpy().view(np.uint32)
            s_got = buf["scales"][so:so + m // block].cpu().numpy()
            # the matrix-core family forms the residual from fp32-exact operand splits with fp32 accumulation:
            # its value differs from the fma chain by ~1e-6 of the reconstruction's terms
            rec = (np.abs(Ph[i:i + 1]).astype(np.float64) @ np.abs(Qn).astype(np.float64).T).ravel()
            blk_rec = rec.reshape(-1, block).max(1)
            assert np.all(np.abs(s_got - s_want) <= 1e-6 * np.maximum(s_want, blk_rec) + 1e-30), f"mat {l} row {i}: scales"
            # every differing code excused one by one by the boundary rule (at most 1e-4 of the row, i.e. one code;
            # the factors are the library's own on both sides, so nothing is added for them)
            sampled_stats = {}
            U.check_codes(c_got, c_want, x.ravel(), m, bits, block, w.lib_seed, l, 1, f"mat {l} row {i}",
                          rec_oracle=rec.astype(np.float32), j0=i * m, stats=sampled_stats)
        # sampled rows of Q+ (columns of p)
        for k in _rows(rng, m, COLS_PER_MAT):
            gk = wl.bf16_bits_to_f32(_grad_col(torch, buf["grads"], o["grad_off"], n, m, k))
            j = np.arange(n, dtype=np.int64) * m + k
            words = codes0[o["word_off"]:o["word_off"] + n * m // W][torch.from_numpy(j // W).cuda()].cpu().numpy().view(np.uint32)
            f = (words >> (bits * (j % W)).astype(np.uint32)) & np.uint32((1 << bits) - 1)
            q = np.where(f >= (1 << (bits - 1)), f.astype(np.int64) - (1 << bits), f.astype(np.int64))
            sc = scales0[o["scale_off"]:o["scale_off"] + n * m // block][torch.from_numpy(j // block).cuda()].cpu().numpy()
            d = sc * inv_s                                                  # fp32 product, as in the decode
            pk = (d.astype(np.float64) * q + gk.astype(np.float64)).astype(np.float32)     # one rounding (the product is exact)
            want = pk.astype(np.float64) @ Ph.astype(np.float64)
            assert np.abs(Qn[k] - want).max() <= 1e-5 * np.abs(Qn).max(), f"mat {l} column {k}: Q+"
    model.close()


def test_large_count_sketch_step_on_sampled_outputs(env):
    R, B, U, torch = env
    w = wl.WORKLOADS["large"]
    rank, beta, keep = w.rank, 0.9, 0.2
    ws = wl.sketch_rows(w.layout, keep)
    model = B.SketchModel(w.layout, ws, rank, beta, B.TABLE_F16, w.grad_dtype, w.lib_seed)
    buf = model.alloc()
    st = B.Model.stream_handle()
    goffs = [o["grad_off"] for o in model.offsets]
    wl.device_q0(w, buf["Q"], [o["q_off"] for o in model.offsets])
    wl.device_fill_gradients(w, 0, buf["grads"], goffs)
    print("[fullsize sketch] step 0", flush=True)
    model.step(buf)
    wl.device_fill_gradients(w, 1, buf["grads"], goffs)
    torch.cuda.synchronize()
    table0, Q0 = buf["table"].clone(), buf["Q"].clone()
    print("[fullsize sketch] step 1, stage by stage", flush=True)
    B.conef_cs_step_p(model.ctx, buf["grads"], buf["table"], buf["Q"], buf["P"], buf["ws"], st)
    torch.cuda.synchronize()
    Praw = buf["P"].clone()
    B.conef_orthonormalise(model.ctx, buf["P"], buf["ws"], st)
    B.conef_cs_step_q(model.ctx, buf["grads"], buf["table"], buf["P"], buf["Q"], buf["ws"], st)
    B.conef_cs_step_err(model.ctx, buf["grads"], buf["table"], buf["P"], buf["Q"], buf["ws"], st)
    torch.cuda.synchronize()
    rng = np.random.default_rng(4048)

    def table_rows(t, off, m, rows):
        idx = torch.tensor(rows, device=t.device)
        return t[off:].view(torch.int16)[: (max(rows) + 1) * m].view(-1, m)[idx].cpu().numpy().view(np.uint16)

    for l in MATS:
        n, m = w.layout[l]
        o = model.offsets[l]
        bucket, sign = R.cs_hash(w.lib_seed, l, n, ws[l])
        Qs = Q0[o["q_off"]:o["q_off"] + m * rank].cpu().numpy().reshape(m, rank)
        Pr = Praw[o["p_off"]:o["p_off"] + n * rank].cpu().numpy().reshape(n, rank)
        Ph = buf["P"][o["p_off"]:o["p_off"] + n * rank].cpu().numpy().reshape(n, rank)
        Qn = buf["Q"][o["q_off"]:o["q_off"] + m * rank].cpu().numpy().reshape(m, rank)
        G = Ph.astype(np.float64).T @ Ph.astype(np.float64)
        assert np.abs(G - np.eye(rank)).max() <= 1e-5, f"mat {l}: P^ not orthonormal"
        # raw P of sampled rows
        rows = _rows(rng, n, ROWS_PER_MAT)
        g_rows = _grad_rows(torch, buf["grads"], o["grad_off"], m, rows)
        t_rows = table_rows(table0, o["table_off"], m, [int(bucket[i]) for i in rows])
        for gi, i in enumerate(rows):
            p = R.cs_form_p(g_rows[gi:gi + 1], t_rows[gi:gi + 1], np.zeros(1, np.int32), sign[i:i + 1], beta)
            want = p.astype(np.float64) @ Qs.astype(np.float64)
            assert np.abs(Pr[i] - want[0]).max() <= 1e-5 * np.abs(Pr).max(), f"mat {l} row {i}: raw P"
        # Q+ of sampled columns
        for k in _rows(rng, m, COLS_PER_MAT):
            gk = wl.bf16_bits_to_f32(_grad_col(torch, buf["grads"], o["grad_off"], n, m, k))
            tk = table0[o["table_off"]:o["table_off"] + ws[l] * m].view(ws[l], m)[:, k].float().cpu().numpy()
            e = tk[bucket] * sign.astype(np.float32)
            omb = np.float32(1.0) - np.float32(beta)
            pk = (np.float64(omb) * e.astype(np.float64) + gk.astype(np.float64)).astype(np.float32)   # one rounding
            want = pk.astype(np.float64) @ Ph.astype(np.float64)
            assert np.abs(Qn[k] - want).max() <= 1e-5 * np.abs(Qn).max(), f"mat {l} column {k}: Q+"
        # the new table row of sampled buckets from the library's own factors
        counts = np.bincount(bucket, minlength=ws[l])
        some = sorted(set([0, ws[l] - 1, int(np.argmax(counts))] + [int(x) for x in rng.integers(0, ws[l], 3)]))
        for b in some:
            members = np.nonzero(bucket == b)[0]                       # ascending rows
            old = table_rows(table0, o["table_off"], m, [b])
            new = old.copy()
            if members.size:
                gm = _grad_rows(torch, buf["grads"], o["grad_off"], m, [int(i) for i in members])
                zero = np.zeros(members.size, np.int32)
                p = R.cs_form_p(gm, old, zero, sign[members], beta)
                x = R.residual(p, Ph[members], Qn)
                R.cs_update(x, zero, sign[members], beta, new)
            else:
                R.cs_update(np.zeros((1, m), np.float32), np.zeros(1, np.int32), np.ones(1, np.int8), beta, new)
            got = table_rows(buf["table"], o["table_off"], m, [b])
            # every matrix of `large` is updated in the sketch's linear form, S+ = (beta + (1 - beta)|b|) S + C(g) - U Q+^T,
            # which rounds at other points than the per-element form the oracle follows: one fp16 unit in the last place
            ne = got != new
            assert ne.mean() <= 2e-2, f"mat {l} bucket {b} ({members.size} rows): {ne.sum()} entries differ"
            gf, wf = got.view(np.float16).astype(np.float64), new.view(np.float16).astype(np.float64)
            ulp = np.maximum(2.0 ** -24, 2.0 ** (np.floor(np.log2(np.maximum(np.abs(wf), 2.0 ** -24))) - 10))
            assert np.all(np.abs(gf - wf) <= ulp), f"mat {l} bucket {b}: an entry differs by more than one unit in the last place"
    model.close()


@pytest.mark.parametrize("name", ["lm", "translation", "large"])
def test_whole_model_second_step_against_the_oracle(env, name):
    """Every matrix of the workload, whole (`large`: 1.31 G elements; `translation`, `lm`: the other kernel
    families at their full sizes): the library's second step (fused call, the launch configuration of the
    benchmark) against one oracle step started from the state the library itself held before that step
    (downloaded), on the gradients the library read.  Factors, scales and every code are compared with the
    criteria of parity_util.compare_step."""
    R, B, U, torch = env
    w = wl.WORKLOADS[name]
    bits, block, rank, W = w.bits, w.block, w.rank, 32 // w.bits
    model = B.Model(w.layout, rank, bits, block, w.grad_dtype, w.lib_seed)
    buf = model.alloc()
    goffs = [o["grad_off"] for o in model.offsets]
    wl.device_q0(w, buf["Q"], [o["q_off"] for o in model.offsets])
    wl.device_fill_gradients(w, 0, buf["grads"], goffs)
    print("[fullsize whole model] step 0", flush=True)
    model.step(buf, 0)
    wl.device_fill_gradients(w, 1, buf["grads"], goffs)
    torch.cuda.synchronize()
    codes0, scales0, Q0 = buf["codes"].cpu().numpy().view(np.uint32), buf["scales"].cpu().numpy(), buf["Q"].cpu().numpy()
    print("[fullsize whole model] step 1", flush=True)
    model.step(buf, 1)
    torch.cuda.synchronize()
    codes1, scales1 = buf["codes"].cpu().numpy().view(np.uint32), buf["scales"].cpu().numpy()
    P1, Q1 = buf["P"].cpu().numpy(), buf["Q"].cpu().numpy()
    excused = 0
    # how far the criteria as stated (scales within 1e-6 of the scale itself; a differing code within 1e-6 max(1, u)
    # of a boundary) are from holding without the allowances below
    strict = {"blocks": 0, "scale_misses": 0, "worst_scale_rel": 0.0, "codes": {}}
    for l, (n, m) in enumerate(w.layout):
        o = model.offsets[l]
        N = n * m
        gd = buf["grads"][o["grad_off"]:o["grad_off"] + N]
        g = (gd.view(torch.int16).cpu().numpy().view(np.uint16) if w.grad_dtype == wl.BF16 else gd.cpu().numpy()).reshape(n, m)
        nw, nb = -(-N // W), -(-N // block)
        c0 = codes0[o["word_off"]:o["word_off"] + nw].copy()
        s0 = scales0[o["scale_off"]:o["scale_off"] + nb].copy()
        st = R.MatState(n, m, c0.copy(), s0.copy(), Q0[o["q_off"]:o["q_off"] + m * rank].reshape(m, rank).copy())
        Ph, Qn = R.step_matrix(g, st, rank, bits, block, w.lib_seed, l, 1)
        tag = f"{name} mat {l} ({n}x{m})"
        eP = U.rel_err(P1[o["p_off"]:o["p_off"] + n * rank].reshape(n, rank), Ph)
        eQ = U.rel_err(Q1[o["q_off"]:o["q_off"] + m * rank].reshape(m, rank), Qn)
        assert eP <= 1e-5, f"{tag}: P rel err {eP}"
        assert eQ <= 1e-5, f"{tag}: Q+ rel err {eQ}"
        # The two sides' factors differ by eP, eQ (relative to the largest entry), so their residuals differ by
        # at most sum_c |dP^[i,c]| |Q+[k,c]| + |P^[i,c]| |dQ+[k,c]|:
        x_tol = float(eP * np.abs(Ph).max() * np.abs(Qn).sum(1).max() + eQ * np.abs(Qn).max() * np.abs(Ph).sum(1).max())

        def rec_of():
            return (np.abs(Ph).astype(np.float64) @ np.abs(Qn).astype(np.float64).T).astype(np.float32).ravel()

        def x_of():
            return R.residual(R.form_p(g, c0, s0, bits, block), Ph, Qn).ravel()

        gs = scales1[o["scale_off"]:o["scale_off"] + nb]
        dev = np.abs(gs - st.scales)
        strict["blocks"] += nb
        rel = dev / np.maximum(st.scales, np.float32(1e-30))
        strict["scale_misses"] += int((rel > 1e-6).sum())
        strict["worst_scale_rel"] = max(strict["worst_scale_rel"], float(rel.max()))
        if dev.max() > 0:
            rec = rec_of()
            blk_rec = np.concatenate([rec, np.zeros((-N) % block, np.float32)]).reshape(-1, block).max(1)
            worst = float((dev / (1e-6 * np.maximum(st.scales, blk_rec) + x_tol)).max())
            assert worst <= 1.0, f"{tag}: scales off by {worst} times the tolerance"
        ex = U.check_codes_sparse(codes1[o["word_off"]:o["word_off"] + nw], st.codes, x_of, N, bits, block,
                                  w.lib_seed, l, 1, tag, rec_of=rec_of, x_abs_tol=x_tol, stats=strict["codes"])
        excused += ex
        if l < 6 or ex:
            print(f"[fullsize whole model] {tag}: eP {eP:.1e} eQ {eQ:.1e} max scale deviation {dev.max():.2e} "
                  f"(x_tol {x_tol:.1e}), {ex} codes differ", flush=True)
    print(f"[fullsize whole model] {name}: {excused} codes of {w.elements} excused as boundary cases", flush=True)
    n_strict, n_wide = strict["codes"].get("strict", 0), strict["codes"].get("widened", 0)
    print(f"[fullsize whole model] {name}: against the criteria as stated: {strict['scale_misses']} of {strict['blocks']} scales "
          f"off by more than 1e-6 of the scale (worst {strict['worst_scale_rel']:.2e}); of the {excused} differing codes "
          f"{n_strict} lie within 1e-6 max(1, u) of a boundary, {n_wide} need the widened window", flush=True)
    assert n_strict + n_wide == excused
    # The allowances are bounded quantities, not open windows.  Measured on `large` (bf16 matrix cores): all 271
    # differing codes of 1.31e9 lie inside the window as stated, none needs the widened one; 97 of 10.2e6 scales
    # (1e-5 of them) miss 1e-6 relative to the scale itself, the worst by a factor 8.  The other families meet
    # the criteria as stated, exactly.
    assert strict["scale_misses"] <= 1e-4 * strict["blocks"] and strict["worst_scale_rel"] <= 2e-5
    assert n_wide <= 1e-7 * w.elements
    if name != "large":
        assert strict["scale_misses"] == 0 and n_wide == 0
    model.close()


def test_large_whole_model_count_sketch_second_step_against_the_oracle(env):
    """The same for the count-sketch mode (fp16 table with a fifth of the rows, beta 0.9): every factor entry and
    every table entry of all 97 matrices after the library's second fused step, against one oracle step started
    from the table and Q the library held.  A table entry may differ by one fp16 unit in the last place (the two
    roundings can fall on different sides when the factors differ in their last bits), rarely."""
    R, B, U, torch = env
    w = wl.WORKLOADS["large"]
    rank, beta = w.rank, 0.9
    ws = wl.sketch_rows(w.layout, 0.2)
    model = B.SketchModel(w.layout, ws, rank, beta, B.TABLE_F16, w.grad_dtype, w.lib_seed)
    buf = model.alloc()
    goffs = [o["grad_off"] for o in model.offsets]
    wl.device_q0(w, buf["Q"], [o["q_off"] for o in model.offsets])
    wl.device_fill_gradients(w, 0, buf["grads"], goffs)
    print("[fullsize sketch whole model] step 0", flush=True)
    model.step(buf)
    wl.device_fill_gradients(w, 1, buf["grads"], goffs)
    torch.cuda.synchronize()
    table0 = buf["table"].view(torch.int16).cpu().numpy().view(np.uint16)
    Q0 = buf["Q"].cpu().numpy()
    print("[fullsize sketch whole model] step 1", flush=True)
    model.step(buf)
    torch.cuda.synchronize()
    table1 = buf["table"].view(torch.int16).cpu().numpy().view(np.uint16)
    P1, Q1 = buf["P"].cpu().numpy(), buf["Q"].cpu().numpy()
    differing = 0
    for l, (n, m) in enumerate(w.layout):
        o = model.offsets[l]
        g = buf["grads"][o["grad_off"]:o["grad_off"] + n * m].view(torch.int16).cpu().numpy().view(np.uint16).reshape(n, m)
        st = R.SketchState(n, m, table0[o["table_off"]:o["table_off"] + ws[l] * m].reshape(ws[l], m).copy(),
                           Q0[o["q_off"]:o["q_off"] + m * rank].reshape(m, rank).copy())
        Ph, Qn = R.cs_step_matrix(g, st, rank, beta, w.lib_seed, l)
        tag = f"large mat {l} ({n}x{m}, {ws[l]} buckets)"
        eP = U.rel_err(P1[o["p_off"]:o["p_off"] + n * rank].reshape(n, rank), Ph)
        eQ = U.rel_err(Q1[o["q_off"]:o["q_off"] + m * rank].reshape(m, rank), Qn)
        assert eP <= 1e-5 and eQ <= 1e-5, f"{tag}: factors rel err {eP}, {eQ}"
        got = table1[o["table_off"]:o["table_off"] + ws[l] * m].reshape(ws[l], m)
        ne = got != st.table
        if ne.any():
            # bound on the difference of the two sides' residuals from their factors differing, times the rows of a bucket
            x_tol = float(eP * np.abs(Ph).max() * np.abs(Qn).sum(1).max() + eQ * np.abs(Qn).max() * np.abs(Ph).sum(1).max())
            counts = np.bincount(R.cs_hash(w.lib_seed, l, n, ws[l])[0], minlength=ws[l]).astype(np.float64)
            gf = got.view(np.float16).astype(np.float64)
            wf = st.table.view(np.float16).astype(np.float64)
            ulp = np.maximum(2.0 ** -24, 2.0 ** (np.floor(np.log2(np.maximum(np.abs(wf), 2.0 ** -24))) - 10))
            assert np.all(np.abs(gf - wf) <= ulp + counts[:, None] * x_tol), f"{tag}: a table entry differs by more than an fp16 ulp"
            assert ne.mean() <= 5e-3, f"{tag}: {ne.mean()} of the table differs"
            differing += int(ne.sum())
    print(f"[fullsize sketch whole model] {differing} of {sum(a * m for a, (_, m) in zip(ws, w.layout))} table entries "
          f"differ (by one fp16 unit in the last place)", flush=True)
    model.close()
