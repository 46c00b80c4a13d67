"""CPU-side tests of the C ABI: the library loads, exports every function the header declares,
validates its arguments, and plans buffer layouts as documented.  No kernel is launched."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2312_08538_amd import binding as B
from paper_2312_08538_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_function():
    header = open(os.path.join(ROOT, "include", "conef.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = sorted(set(re.findall(r"\b(conef_[a-z0-9_]+)\s*\(", header)))
    assert declared, "no declarations found"
    L = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(L, name), f"{name} is declared in conef.h but not exported"
    assert sorted(B.EXPORTS) == declared          # the binding covers the same set


def test_init_rejects_bad_arguments():
    ok = [(64, 64)]
    bad = [
        (ok, 0, 4, 128), (ok, 33, 4, 128), (ok, 65, 4, 128),      # rank
        (ok, 4, 3, 128), (ok, 4, 16, 128), (ok, 4, 0, 128),       # bits
        (ok, 4, 4, 0), (ok, 4, 4, 12), (ok, 4, 4, -8), (ok, 4, 8, 6), (ok, 4, 2, 8), (ok, 4, 4, 1 << 21),  # block
        ([(0, 64)], 1, 4, 128), ([(64, -1)], 1, 4, 128),          # dims
        ([(3, 64)], 4, 4, 128), ([(64, 2)], 4, 4, 128),           # rank > min(rows, cols)
        ([(1 << 20, 1 << 15)], 4, 4, 128),                        # rows*cols >= 2^35
        ([], 4, 4, 128),
    ]
    for layout, rank, bits, block in bad:
        with pytest.raises(B.ConefError) as e:
            B.conef_init(layout, rank, bits, block, B.F32, 0)
        assert e.value.code == B.EINVAL
    with pytest.raises(B.ConefError):
        B.conef_init(ok, 4, 4, 128, 7, 0)                          # dtype
    assert B.lib().conef_init(None, None, 1, 4, 4, 128, 0, 0) == B.EINVAL
    ctx = ctypes.c_void_p()
    assert B.lib().conef_init(ctypes.byref(ctx), None, 1, 4, 4, 128, 0, 0) == B.EINVAL


def test_null_and_misaligned_pointers_are_rejected_before_any_launch():
    ctx = B.conef_init([(64, 64)], 4, 4, 128, B.F32, 0)
    L = B.lib()
    assert L.conef_step(ctx, 0, 0, 0, 0, 0, 0, 0, 0, 0) == B.EINVAL
    assert L.conef_step(ctx, 256, 256, 256, 0, 256, 256, 256, 0, 0) == B.EINVAL       # null Q_state
    assert L.conef_step(ctx, 260, 256, 256, 256, 256, 256, 256, 0, 0) == B.EINVAL     # grads not 16-byte aligned
    assert L.conef_step(ctx, 256, 256, 256, 256, 256, 256, 128, 0, 0) == B.EINVAL     # workspace not 256-byte aligned
    assert L.conef_step_err(ctx, 256, 256, 258, 256, 256, 256, 0, 0) == B.EINVAL           # scales not 4-byte aligned
    assert L.conef_step(None, 256, 256, 256, 256, 256, 256, 256, 0, 0) == B.EINVAL
    assert L.conef_reset_error(ctx, 0, 0, 0) == B.EINVAL
    assert L.conef_decode_error(ctx, 256, 256, 0, 0) == B.EINVAL
    assert L.conef_sizes(None, None, None, None, None, None, None) == B.EINVAL
    assert L.conef_offsets(ctx, 1, None, None, None, None, None) == B.EINVAL
    assert L.conef_offsets(ctx, -1, None, None, None, None, None) == B.EINVAL
    ms = (ctypes.c_float * 4)()
    assert L.conef_get_timing(ctx, ms) == B.ESTATE                                     # timing never switched on
    assert B.lib().conef_strerror(B.EINVAL) == b"invalid argument"
    B.conef_destroy(ctx)
    B.conef_destroy(None)


@pytest.mark.parametrize("name", list(wl.WORKLOADS))
def test_sizes_and_offsets_follow_the_documented_layout(name):
    w = wl.WORKLOADS[name]
    m = B.Model(w.layout, w.rank, w.bits, w.block, w.grad_dtype, w.lib_seed)
    W = 32 // w.bits
    ru = lambda v: (v + 63) // 64 * 64
    g = c = s = p = q = 0
    for l, (n, mm) in enumerate(w.layout):
        o = m.offsets[l]
        assert (o["grad_off"], o["word_off"], o["scale_off"], o["p_off"], o["q_off"]) == (g, c, s, p, q)
        N = n * mm
        g += ru(N); c += ru(-(-N // W)); s += ru(-(-N // w.block)); p += ru(n * w.rank); q += ru(mm * w.rank)
    sz = m.sizes
    assert (sz["grad_elems"], sz["code_words"], sz["n_scales"], sz["p_elems"], sz["q_elems"]) == (g, c, s, p, q)
    assert sz["workspace_bytes"] % 256 == 0 and sz["workspace_bytes"] > 0
    m.close()


def test_state_memory_matches_the_closed_form():
    """Compressed error vs an fp32 error vector: 1 - (b + 32/B)/32 up to padding."""
    w = wl.WORKLOADS["lm"]
    m = B.Model(w.layout, w.rank, w.bits, w.block, w.grad_dtype, 0)
    kept = 4 * (m.sizes["code_words"] + m.sizes["n_scales"])
    saving = 1 - kept / (4 * w.elements)
    assert abs(saving - (1 - (w.bits + 32 / w.block) / 32)) < 1e-3
    m.close()


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "libconef.so"))
    with pytest.raises(RuntimeError):
        B.lib()


PLAN_CASES = [
    # (layout, rank, bits, block, dtype): every kernel family, ragged tiles, short last blocks
    ([(256, 128)], 2, 8, 64, B.F32),
    ([(64, 147), (64, 576), (512, 4608), (1000, 512)], 4, 4, 128, B.F32),
    ([(32768, 1024), (1024, 4096), (4096, 1024), (77, 1024)], 8, 2, 256, B.BF16),
    ([(50304, 2048), (2048, 8192), (8192, 2048), (2200, 128), (300, 2304), (45, 384)], 32, 4, 128, B.BF16),
    ([(64, 147), (5, 3), (2, 67), (130, 2), (33, 129), (2, 1000), (257, 64)], 2, 4, 8, B.F32),
    ([(96, 160), (40, 512), (300, 33)], 16, 4, 32, B.F32),
    ([(640, 192), (65, 64), (129, 320)], 4, 8, 64, B.BF16),
    ([(3000, 512), (100, 1536)], 8, 4, 512, B.F32),
]


@pytest.mark.parametrize("case", range(len(PLAN_CASES)))
def test_work_tables_cover_every_matrix_exactly_once(case):
    """The planner's work tables (which workgroup does which rows and columns in each of the three
    passes, per kernel family), its reduction / orthonormalisation items and its workspace map."""
    layout, rank, bits, block, dtype = PLAN_CASES[case]
    ctx = B.conef_init(layout, rank, bits, block, dtype, 1)
    try:
        B.conef_check_plan(ctx)
    finally:
        B.conef_destroy(ctx)


def test_static_workspace_step_checks_the_size_on_the_host():
    """conef_step_static refuses a model whose workspace exceeds the library's static array before it looks at
    a pointer or at the device (so the check runs without a GPU), and a context with nothing uploaded yet."""
    w = wl.WORKLOADS["large"]
    big = B.conef_init(list(w.layout), w.rank, w.bits, w.block, w.grad_dtype, w.lib_seed)
    assert B.conef_sizes(big)["workspace_bytes"] > B.STATIC_WORKSPACE_BYTES
    fake = ctypes.c_void_p(0x1000)
    assert B.lib().conef_step_static(big, fake, fake, fake, fake, fake, fake, 0, None) == B.ETOOBIG
    B.conef_destroy(big)
    small = B.conef_init([(64, 64)], 4, 4, 64, B.F32, 0)
    assert B.conef_sizes(small)["workspace_bytes"] <= B.STATIC_WORKSPACE_BYTES
    assert B.lib().conef_step_static(small, fake, fake, fake, fake, fake, fake, 0, None) == B.ESTATE
    assert B.lib().conef_step_static(None, fake, fake, fake, fake, fake, fake, 0, None) == B.EINVAL
    assert b"static workspace" in B.lib().conef_strerror(B.ETOOBIG)
    B.conef_destroy(small)


def test_full_workloads_plan_consistently():
    for w in wl.WORKLOADS.values():
        ctx = B.conef_init(list(w.layout), w.rank, w.bits, w.block, w.grad_dtype, w.lib_seed)
        try:
            B.conef_check_plan(ctx)
        finally:
            B.conef_destroy(ctx)


# ------------------------------------------------------------------ count-sketch mode (host side)
def test_sketch_init_rejects_bad_arguments():
    lay = [(64, 64), (30, 20)]
    bad = [
        dict(sketch_rows=[0, 5]), dict(sketch_rows=[65, 5]), dict(sketch_rows=[8, 31]),   # 1 <= w <= rows
        dict(beta=1.0), dict(beta=-0.01), dict(beta=float("nan")),
        dict(table_dtype=2), dict(table_dtype=-1), dict(rank=0), dict(rank=21), dict(grad_dtype=5),
    ]
    for b in bad:
        kw = dict(sketch_rows=[16, 30], rank=4, beta=0.9, table_dtype=B.TABLE_F16, grad_dtype=B.F32)
        kw.update(b)
        with pytest.raises(B.ConefError) as e:
            B.conef_cs_init(lay, kw["sketch_rows"], kw["rank"], kw["beta"], kw["table_dtype"], kw["grad_dtype"], 0)
        assert e.value.code == B.EINVAL, b
    ctx = ctypes.c_void_p()
    arr = (B.conef_mat * 1)()
    arr[0].rows, arr[0].cols = 8, 8
    assert B.lib().conef_cs_init(ctypes.byref(ctx), arr, None, 1, 2, 0.5, 0, 0, 0) == B.EINVAL     # null sketch_rows


def test_column_sketch_init_plan_and_hash(ref):
    """The column form of the count sketch (host side): argument checks, table sizes and offsets (rows x buckets), the
    hash of the columns against the oracle's, the plan's self-check."""
    L = B.lib()
    layout = [(64, 147), (300, 256), (3, 5)]
    buckets = [30, 256, 1]
    seed = 0xFEED5
    ctx = B.conef_csc_init(layout, buckets, 2, 0.5, B.TABLE_F16, B.BF16, seed)
    B.conef_check_plan(ctx)
    off = 0
    for l, (n, m) in enumerate(layout):
        o = B.conef_cs_offsets(ctx, l)
        assert (o["table_off"], o["sketch_rows"]) == (off, buckets[l])
        off += (n * buckets[l] + 63) // 64 * 64
        b, s = B.conef_cs_hash(ctx, l, m)
        rb, rs = ref.cs_hash(seed, l, m, buckets[l])
        assert np.array_equal(b, rb) and np.array_equal(s, rs)
    assert B.conef_cs_sizes(ctx)["table_elems"] == off
    A = 512
    assert L.conef_cs_rb_step(ctx, A, A, A, 0, 0) == B.ESTATE
    assert L.conef_cs_ss_step(ctx, A, A, A, A, A, 0) == B.ESTATE
    assert L.conef_step(ctx, A, A, A, A, A, A, A, 0, 0) == B.ESTATE         # a sketch context all the same
    B.conef_destroy(ctx)
    for bad_layout, bad_buckets in (([(64, 64)], [65]), ([(64, 64)], [0]), ([(8, 16392)], [10])):
        with pytest.raises(B.ConefError) as e:
            B.conef_csc_init(bad_layout, bad_buckets, 2, 0.5, B.TABLE_F32, B.F32, 1)
        assert e.value.code == B.EINVAL


def test_sketch_and_quantiser_contexts_refuse_each_others_calls():
    sk = B.conef_cs_init([(64, 64)], [16], 4, 0.5, B.TABLE_F32, B.F32, 0)
    qc = B.conef_init([(64, 64)], 4, 4, 64, B.F32, 0)
    L = B.lib()
    assert L.conef_step(sk, 256, 256, 256, 256, 256, 256, 256, 0, 0) == B.ESTATE
    assert L.conef_step_p(sk, 256, 256, 256, 256, 256, 256, 0) == B.ESTATE
    assert L.conef_decode_error(sk, 256, 256, 256, 0) == B.ESTATE
    assert L.conef_reset_error(sk, 256, 256, 0) == B.ESTATE
    assert L.conef_cs_step(qc, 256, 256, 256, 256, 256, 256, 0) == B.ESTATE
    assert L.conef_cs_step_err(qc, 256, 256, 256, 256, 256, 0) == B.ESTATE
    assert L.conef_cs_decode_error(qc, 256, 256, 0) == B.ESTATE
    assert L.conef_cs_sizes(qc, None) == B.ESTATE
    assert L.conef_cs_step(sk, 256, 0, 256, 256, 256, 256, 0) == B.EINVAL              # null table
    assert L.conef_cs_step(sk, 256, 264, 256, 256, 256, 256, 0) == B.EINVAL            # table not 16-byte aligned
    assert L.conef_cs_offsets(sk, 1, None, None) == B.EINVAL
    assert B.conef_sizes(sk)["code_words"] == 0 and B.conef_sizes(sk)["n_scales"] == 0
    B.conef_destroy(sk)
    B.conef_destroy(qc)


SKETCH_PLAN_CASES = [
    ([(37, 11), (64, 8), (300, 256)], [5, 64, 60], 4),
    ([(64, 147), (128, 576), (20, 33)], [13, 26, 1], 3),
    ([(2000, 520), (96, 1024)], [400, 96], 8),
    ([(130, 300), (70, 2600)], [50, 7], 32),
]


@pytest.mark.parametrize("case", range(len(SKETCH_PLAN_CASES)))
def test_sketch_plan_tables_hash_and_bucket_lists(case, ref):
    """Table offsets as documented; the library's hash is the oracle's; the bucket lists hold every row once
    in ascending order and the update's work items cover every table entry once (the plan's self-check)."""
    layout, ws, rank = SKETCH_PLAN_CASES[case]
    m = B.SketchModel(layout, ws, rank, 0.9, B.TABLE_F16, B.BF16, 0xABCDEF0123)
    B.conef_check_plan(m.ctx)
    t = 0
    for l, (n, mm) in enumerate(layout):
        assert m.offsets[l]["table_off"] == t and m.offsets[l]["sketch_rows"] == ws[l]
        t += (ws[l] * mm + 63) // 64 * 64
        b, s = B.conef_cs_hash(m.ctx, l, n)
        rb, rs = ref.cs_hash(0xABCDEF0123, l, n, ws[l])
        assert np.array_equal(b, rb) and np.array_equal(s, rs)
    assert m.sizes["table_elems"] == t
    m.close()


def test_sketch_plans_of_the_full_workloads_are_consistent():
    for w in wl.WORKLOADS.values():
        for keep in (0.2, 0.8):
            m = B.SketchModel(w.layout, wl.sketch_rows(w.layout, keep), w.rank, 0.9, B.TABLE_F16, w.grad_dtype, w.lib_seed)
            B.conef_check_plan(m.ctx)
            m.close()


def test_set_beta_validates_its_argument():
    ctx = B.conef_init([(64, 64)], 4, 4, 64, B.F32, 0)
    L = B.lib()
    for bad in (-0.1, 1.0, 1.5, float("nan")):
        assert L.conef_set_beta(ctx, bad) == B.EINVAL
    assert L.conef_set_beta(None, 0.5) == B.EINVAL
    for good in (0.0, 0.5, 0.999):
        assert L.conef_set_beta(ctx, good) == B.OK
    B.conef_destroy(ctx)


# ------------------------------------------------------------------ random-block gradient compressor (host side)
def test_random_block_layout_and_start_match_the_oracle(ref):
    layout = [(64, 147), (512, 1024), (3, 5)]
    keep = wl.random_block_keep(layout, 0.1)
    assert keep == [940, 52428, 1]
    for ctx in (B.conef_init(layout, 2, 4, 128, B.BF16, 0xC0FFEE123),
                B.conef_cs_init(layout, [8, 100, 3], 2, 0.5, B.TABLE_F16, B.BF16, 0xC0FFEE123)):
        L = B.lib()
        assert L.conef_rb_sizes(ctx, None) == B.ESTATE                      # not configured yet
        B.conef_rb_configure(ctx, keep)
        off = 0
        for l, (n, m) in enumerate(layout):
            o = B.conef_rb_offsets(ctx, l)
            assert (o["delta_off"], o["keep"]) == (off, keep[l])
            off += (keep[l] + 63) // 64 * 64
            for step in (0, 1, 7, 2 ** 33 + 1):
                s = B.conef_rb_start(ctx, l, step)
                assert s == ref.rb_start(0xC0FFEE123, l, step, n * m, keep[l])
                assert 0 <= s <= n * m - keep[l]
        assert B.conef_rb_sizes(ctx)["delta_elems"] == off
        B.conef_check_plan(ctx)
        for bad in ([0, 1, 1], [1, 1, 16]):
            with pytest.raises(B.ConefError) as e:
                B.conef_rb_configure(ctx, bad)
            assert e.value.code == B.EINVAL
        assert L.conef_rb_configure(ctx, None) == B.EINVAL
        B.conef_destroy(ctx)


def test_random_k_layout_and_kept_coordinates_match_the_oracle(ref):
    layout = [(64, 147), (512, 1024), (3, 5)]
    group = [10, 16, 4]
    for ctx in (B.conef_init(layout, 2, 4, 128, B.BF16, 0xC0FFEE123),
                B.conef_cs_init(layout, [8, 100, 3], 2, 0.5, B.TABLE_F16, B.BF16, 0xC0FFEE123)):
        L = B.lib()
        assert L.conef_rk_sizes(ctx, None) == B.ESTATE                      # not configured yet
        B.conef_rk_configure(ctx, group)
        off = 0
        for l, (n, m) in enumerate(layout):
            N, G = n * m, group[l]
            keep = -(-N // G)
            o = B.conef_rk_offsets(ctx, l)
            assert (o["delta_off"], o["keep"]) == (off, keep) and keep == ref.rk_count(N, G)
            off += (keep + 63) // 64 * 64
            for step in (0, 7, 2 ** 33 + 1):
                want = ref.rk_indices(0xC0FFEE123, l, step, N, G)
                for i in (0, 1, keep // 2, keep - 1):
                    assert B.conef_rk_index(ctx, l, step, i) == want[i]
            with pytest.raises(B.ConefError) as e:
                B.conef_rk_index(ctx, l, 0, keep)
            assert e.value.code == B.EINVAL
        assert B.conef_rk_sizes(ctx)["delta_elems"] == off
        B.conef_check_plan(ctx)
        for bad in ([0, 1, 1], [1, 1, 16], [-3, 1, 1]):
            with pytest.raises(B.ConefError) as e:
                B.conef_rk_configure(ctx, bad)
            assert e.value.code == B.EINVAL
        assert L.conef_rk_configure(ctx, None) == B.EINVAL
        B.conef_destroy(ctx)
    # a matrix of 2^32 coordinates or more is refused (the kernels index a matrix with 32 bits here)
    ctx = B.conef_init([(65536, 65536)], 2, 4, 128, B.BF16, 1)
    with pytest.raises(B.ConefError) as e:
        B.conef_rk_configure(ctx, [10])
    assert e.value.code == B.EINVAL
    B.conef_destroy(ctx)


def test_uniform_random_k_layout_and_slots_match_the_oracle(ref):
    """The uniformly drawn k-subset (host side): sizes, offsets, the coordinate of every slot (the inverse of the keyed
    permutation), and that the coordinates of the k slots are distinct."""
    layout = [(64, 147), (512, 1024), (3, 5), (256, 256), (1, 1)]
    keep = [941, 52429, 15, 1, 1]
    seed = 0xC0FFEE123
    for ctx in (B.conef_init(layout, 1, 4, 128, B.BF16, seed),
                B.conef_cs_init(layout, [8, 100, 3, 7, 1], 1, 0.5, B.TABLE_F16, B.BF16, seed)):
        L = B.lib()
        assert L.conef_rk_sizes(ctx, None) == B.ESTATE
        B.conef_rk_configure_uniform(ctx, keep)
        off = 0
        for l, (n, m) in enumerate(layout):
            N, k = n * m, keep[l]
            o = B.conef_rk_offsets(ctx, l)
            assert (o["delta_off"], o["keep"]) == (off, k)
            off += (k + 63) // 64 * 64
            for step in (0, 7, 2 ** 33 + 1):
                want = ref.rk_indices(seed, l, step, N, -k)
                assert len(set(want.tolist())) == k and want.min() >= 0 and want.max() < N
                for i in sorted({0, 1 % k, k // 2, k - 1}):
                    j = B.conef_rk_index(ctx, l, step, i)
                    assert j == want[i] and ref.rku_perm(seed, l, step, N, j) == i
            with pytest.raises(B.ConefError) as e:
                B.conef_rk_index(ctx, l, 0, k)
            assert e.value.code == B.EINVAL
        assert B.conef_rk_sizes(ctx)["delta_elems"] == off
        B.conef_check_plan(ctx)
        for bad in ([0, 1, 1, 1, 1], [1, 1, 16, 1, 1], [-3, 1, 1, 1, 1]):
            with pytest.raises(B.ConefError) as e:
                B.conef_rk_configure_uniform(ctx, bad)
            assert e.value.code == B.EINVAL
        assert L.conef_rk_configure_uniform(ctx, None) == B.EINVAL
        # the stratified form replaces it, and the other way round
        B.conef_rk_configure(ctx, [10, 16, 4, 3, 1])
        assert B.conef_rk_offsets(ctx, 0)["keep"] == -(-64 * 147 // 10)
        B.conef_check_plan(ctx)
        B.conef_rk_configure_uniform(ctx, keep)
        assert B.conef_rk_offsets(ctx, 0)["keep"] == keep[0]
        B.conef_check_plan(ctx)
        B.conef_destroy(ctx)
    ctx = B.conef_init([(65536, 65536)], 2, 4, 128, B.BF16, 1)
    with pytest.raises(B.ConefError) as e:
        B.conef_rk_configure_uniform(ctx, [10])
    assert e.value.code == B.EINVAL
    B.conef_destroy(ctx)


def test_kernel_family_of_a_matrix_is_reported(monkeypatch):
    """conef_matrix_family: which matrices accumulate their factors in fp64 (families 0 and 1) and which on the bf16 matrix
    cores (2: rank 32; 3: packed splits at ranks 2, 4, 8), and that CONEF_PACK=0 keeps family 1."""
    layout = [(64, 147), (300, 512), (40, 256), (128, 128)]
    cases = [  # rank, bits, block, dtype -> families
        (8, 2, 256, B.BF16, [0, 3, 3, 0]),           # 128 columns do not hold a block of 256
        (8, 2, 256, B.F32, [0, 1, 1, 0]),
        (4, 4, 128, B.BF16, [0, 3, 3, 3]),
        (4, 8, 128, B.BF16, [0, 1, 1, 1]),           # 8-bit codes stay on the octet family
        (4, 4, 64, B.BF16, [0, 1, 1, 1]),            # so do blocks below 128
        (32, 4, 128, B.BF16, [0, 2, 2, 2]),
        (16, 4, 128, B.BF16, [0, 0, 0, 0]),
    ]
    for rank, bits, block, dt, want in cases:
        ctx = B.conef_init(layout, rank, bits, block, dt, 5)
        assert [B.conef_matrix_family(ctx, l) for l in range(len(layout))] == want, (rank, bits, block, dt)
        B.conef_check_plan(ctx)
        with pytest.raises(B.ConefError) as e:
            B.conef_matrix_family(ctx, len(layout))
        assert e.value.code == B.EINVAL
        B.conef_destroy(ctx)
    monkeypatch.setenv("CONEF_PACK", "0")
    ctx = B.conef_init(layout, 8, 2, 256, B.BF16, 5)
    assert [B.conef_matrix_family(ctx, l) for l in range(len(layout))] == [0, 1, 1, 0]
    B.conef_check_plan(ctx)
    B.conef_destroy(ctx)
    sk = B.conef_cs_init(layout, [8, 100, 8, 16], 8, 0.5, B.TABLE_F16, B.BF16, 5)
    assert all(B.conef_matrix_family(sk, l) in (0, 1) for l in range(len(layout)))
    B.conef_destroy(sk)


def test_first_error_vector_layout_and_start_match_the_oracle(ref):
    """Algorithm 3, version 2: sizes, offsets and block starts of the first error vectors (host side)."""
    layout = [(64, 147), (512, 1024), (3, 5)]
    keep_e = [470, 0, 15]
    seed = 0xC0FFEE123
    ctx = B.conef_init(layout, 2, 4, 128, B.BF16, seed)
    L = B.lib()
    assert L.conef_i2_sizes(ctx, None) == B.ESTATE                          # not configured yet
    assert L.conef_i2_rb_step(ctx, 512, 512, 1024, 512, 512, 512, 0, 0) == B.ESTATE
    B.conef_i2_configure(ctx, keep_e)
    off = 0
    for l, (n, m) in enumerate(layout):
        o = B.conef_i2_offsets(ctx, l)
        assert (o["e_off"], o["keep_e"]) == (off, keep_e[l])
        off += (keep_e[l] + 63) // 64 * 64
        for step in (0, 1, 7, 2 ** 33 + 1, 2 ** 64 - 1):
            s = B.conef_i2_start(ctx, l, step)
            assert s == ref.i2_start(seed, l, step, n * m, keep_e[l]) and 0 <= s <= n * m - keep_e[l]
    assert B.conef_i2_sizes(ctx)["e_elems"] == off
    B.conef_check_plan(ctx)
    for bad in ([-1, 1, 1], [1, 1, 16]):
        with pytest.raises(B.ConefError) as e:
            B.conef_i2_configure(ctx, bad)
        assert e.value.code == B.EINVAL
    assert L.conef_i2_configure(ctx, None) == B.EINVAL
    # null, misaligned and doubled buffers (after the gradient compressor is configured, before any launch)
    B.conef_rb_configure(ctx, [10, 10, 1])
    A = 512
    assert L.conef_i2_rb_step(ctx, A, 0, 1024, A, A, A, 0, 0) == B.EINVAL
    assert L.conef_i2_rb_step(ctx, A, A, A, A, A, A, 0, 0) == B.EINVAL
    assert L.conef_i2_rb_step(ctx, A, 514, 1024, A, A, A, 0, 0) == B.EINVAL
    assert L.conef_i2_rk_step(ctx, A, A, 1024, A, A, A, 0, 0) == B.ESTATE     # random-k not configured
    B.conef_destroy(ctx)
    sk = B.conef_cs_init(layout, [8, 100, 3], 2, 0.5, B.TABLE_F16, B.BF16, seed)
    assert L.conef_i2_configure(sk, (ctypes.c_int64 * 3)(1, 1, 1)) == B.ESTATE
    B.conef_destroy(sk)
    # all zero: the buffer is still a valid allocation
    ctx = B.conef_init([(8, 8)], 2, 4, 8, B.F32, 1)
    B.conef_i2_configure(ctx, [0])
    assert B.conef_i2_sizes(ctx)["e_elems"] == 64
    B.conef_destroy(ctx)


def test_element_wise_and_iconef_calls_validate_their_arguments_before_any_launch():
    """Every check below returns before the library touches the GPU, so it runs here."""
    L = B.lib()
    q = B.conef_init([(64, 64)], 4, 4, 128, B.F32, 0)
    qb = B.conef_init([(64, 64)], 4, 4, 128, B.BF16, 0)
    sk = B.conef_cs_init([(64, 64)], [16], 4, 0.0, B.TABLE_F32, B.F32, 0)
    A = 256                                                    # any aligned non-null address
    # not configured yet
    assert L.conef_rb_step(q, A, A, A, A, 0, 0) == B.ESTATE
    assert L.conef_rk_step(q, A, A, A, A, 0, 0) == B.ESTATE
    assert L.conef_i_rb_step(q, A, A, A, 512, 512, A, 0, 0) == B.ESTATE
    assert L.conef_i_rk_step(q, A, A, A, 512, 512, A, 0, 0) == B.ESTATE
    assert L.conef_cs_rk_step(sk, A, A, A, 0, 0) == B.ESTATE
    for ctx in (q, qb, sk):
        B.conef_rb_configure(ctx, [100])
        B.conef_rk_configure(ctx, [10])
    # the wrong kind of context
    assert L.conef_rb_step(sk, A, A, A, A, 0, 0) == B.ESTATE
    assert L.conef_rk_step(sk, A, A, A, A, 0, 0) == B.ESTATE
    assert L.conef_ss_step(sk, A, A, A, A, A, A, 0, 0) == B.ESTATE
    assert L.conef_i_ss_step(sk, A, A, A, 512, 512, A, A, A, 0, 0) == B.ESTATE
    assert L.conef_cs_rb_step(q, A, A, A, 0, 0) == B.ESTATE
    assert L.conef_cs_rk_step(q, A, A, A, 0, 0) == B.ESTATE
    assert L.conef_cs_ss_step(q, A, A, A, A, A, 0) == B.ESTATE
    assert L.conef_i_step(sk, A, A, A, 512, 512, A, A, A, A, 0, 0) == B.ESTATE
    # null and misaligned pointers, the two vectors in one buffer
    assert L.conef_rk_step(q, 0, A, A, A, 0, 0) == B.EINVAL
    assert L.conef_rk_step(q, 260, A, A, A, 0, 0) == B.EINVAL
    assert L.conef_rk_step(q, A, A, A, 258, 0, 0) == B.EINVAL
    assert L.conef_i_rb_step(q, A, A, A, 0, 512, A, 0, 0) == B.EINVAL
    assert L.conef_i_rb_step(q, A, A, A, A, 512, A, 0, 0) == B.EINVAL                   # codes twice
    assert L.conef_i_rk_step(q, A, A, A, 512, A, A, 0, 0) == B.EINVAL                   # scales twice
    assert L.conef_i_ss_step(q, A, A, A, 512, 512, A, A, 128, 0, 0) == B.EINVAL         # workspace not 256-byte aligned
    assert L.conef_i_step(q, A, A, A, A, 512, A, A, A, A, 0, 0) == B.EINVAL
    assert L.conef_i_step(q, A, A, A, 512, 512, A, A, A, 128, 0, 0) == B.EINVAL
    assert L.conef_i_step_err(q, A, A, A, 512, 512, 0, A, A, 0, 0) == B.EINVAL
    assert L.conef_i_step_err(q, A, A, A, 512, 512, A, A, 0, 0, 0) == B.EINVAL            # no workspace
    assert L.conef_i_step_p(q, 260, A, A, 512, 512, A, A, A, 0) == B.EINVAL
    assert L.conef_i_step_q(q, A, A, A, 512, 512, A, A, 128, 0) == B.EINVAL
    assert L.conef_i_step_q(qb, A, A, A, A, 512, A, A, A, 0) == B.EINVAL
    # Algorithm 3 has no partial update
    B.conef_set_beta(q, 0.25)
    assert L.conef_i_rb_step(q, A, A, A, 512, 512, A, 0, 0) == B.ESTATE
    assert L.conef_i_ss_step(q, A, A, A, 512, 512, A, A, A, 0, 0) == B.ESTATE
    assert L.conef_i_rk_step(q, A, A, A, 512, 512, A, 0, 0) == B.ESTATE
    assert L.conef_i_step(q, A, A, A, 512, 512, A, A, A, A, 0, 0) == B.ESTATE
    for ctx in (q, qb, sk):
        B.conef_destroy(ctx)
