"""ctypes face of the CPU oracle: oracle/conef_ref.c (the step of Algorithm 2), sketch_ref.c (count sketch, partial
update), randblock_ref.c (random block, scaled sign), iconef_ref.c (Algorithm 3, version 1), randk_ref.c (random-k) and
iconef2_ref.c (Algorithm 3, version 2) and sketch_col_ref.c (count sketch, column form), built into one shared library
with gcc.

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg.  The product package never imports this module.

Every function takes and returns numpy arrays; the arithmetic is all in the C
file (Algorithm 2: accumulate, compress, error; eq. (3) with the block max-norm; the rank-r
factorisation of Section 5.2).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conef_ref.c")
_SRC_SKETCH = os.path.join(_HERE, "sketch_ref.c")
_SRC_RB = os.path.join(_HERE, "randblock_ref.c")
_SRC_I = os.path.join(_HERE, "iconef_ref.c")
_SRC_RK = os.path.join(_HERE, "randk_ref.c")
_SRC_I2 = os.path.join(_HERE, "iconef2_ref.c")
_SRC_CSC = os.path.join(_HERE, "sketch_col_ref.c")
_LIB = os.path.join(_HERE, "libconef_ref.so")

F32, BF16 = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  -ffp-contract=off: every fused multiply-add
    in the source is an explicit fmaf(), nothing else may be contracted."""
    newest = max(os.path.getmtime(f) for f in (_SRC, _SRC_SKETCH, _SRC_RB, _SRC_I, _SRC_RK, _SRC_I2, _SRC_CSC))
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-mfma", "-Wall", "-Wextra", "-o", _LIB, _SRC, _SRC_SKETCH, _SRC_RB, _SRC_I, _SRC_RK, _SRC_I2, _SRC_CSC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        vp, i64, i32, u64, u32 = (ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_uint64,
                                  ctypes.c_uint32)
        L.ref_philox4x32_10.argtypes = [vp, vp, vp]
        L.ref_philox4x32_10.restype = None
        L.ref_rand16.argtypes = [u64, u32, u64, u64]
        L.ref_rand16.restype = u32
        L.ref_get_code.argtypes = [vp, i64, i32]
        L.ref_get_code.restype = ctypes.c_int32
        L.ref_decode.argtypes = [vp, vp, i64, i32, i32, vp]
        L.ref_decode.restype = None
        L.ref_form_p.argtypes = [vp, i32, vp, vp, i64, i32, i32, vp]
        L.ref_form_p.restype = None
        L.ref_form_p_partial.argtypes = [vp, i32, vp, vp, i64, i32, i32, ctypes.c_float, vp]
        L.ref_form_p_partial.restype = None
        L.ref_step_matrix_partial.argtypes = [vp, i32, i64, i64, i32, i32, i32, ctypes.c_float, u64, u32, u64,
                                              vp, vp, vp, vp, vp, vp]
        L.ref_step_matrix_partial.restype = None
        L.ref_lowrank_P.argtypes = [vp, i64, i64, vp, i32, vp]
        L.ref_lowrank_P.restype = None
        L.ref_orthonormalise.argtypes = [vp, i64, i32]
        L.ref_orthonormalise.restype = None
        L.ref_lowrank_Q.argtypes = [vp, i64, i64, vp, i32, vp]
        L.ref_lowrank_Q.restype = None
        L.ref_residual.argtypes = [vp, i64, i64, vp, vp, i32, vp]
        L.ref_residual.restype = None
        L.ref_decompress.argtypes = [i64, i64, vp, vp, i32, vp]
        L.ref_decompress.restype = None
        L.ref_apply_update.argtypes = [vp, i64, i64, vp, vp, i32]
        L.ref_apply_update.restype = None
        L.ref_quantise.argtypes = [vp, i64, i32, i32, u64, u32, u64, vp, vp, vp]
        L.ref_quantise.restype = None
        L.ref_step_matrix.argtypes = [vp, i32, i64, i64, i32, i32, i32, u64, u32, u64,
                                      vp, vp, vp, vp, vp, vp]
        L.ref_step_matrix.restype = None
        L.ref_step_matrix_efsgd.argtypes = [vp, i64, i64, i32, vp, vp, vp, vp, vp]
        L.ref_step_matrix_efsgd.restype = None
        f32 = ctypes.c_float
        L.ref_f16_to_f32.argtypes = [ctypes.c_uint16]
        L.ref_f16_to_f32.restype = f32
        L.ref_f32_to_f16.argtypes = [f32]
        L.ref_f32_to_f16.restype = ctypes.c_uint16
        L.ref_cs_hash.argtypes = [u64, u32, i64, i64, vp, vp]
        L.ref_cs_hash.restype = None
        L.ref_cs_decode.argtypes = [vp, i32, i64, i64, vp, vp, vp]
        L.ref_cs_decode.restype = None
        L.ref_cs_form_p.argtypes = [vp, i32, vp, i32, i64, i64, vp, vp, f32, vp]
        L.ref_cs_form_p.restype = None
        L.ref_cs_update.argtypes = [vp, i64, i64, vp, vp, i64, f32, vp, i32]
        L.ref_cs_update.restype = None
        L.ref_cs_step_matrix.argtypes = [vp, i32, i64, i64, i32, i64, f32, u64, u32, vp, i32, vp, vp, vp, vp]
        L.ref_cs_step_matrix.restype = None
        L.ref_rb_start.argtypes = [u64, u32, u64, i64, i64]
        L.ref_rb_start.restype = i64
        L.ref_rb_step_matrix.argtypes = [vp, i32, i64, i64, i32, i32, f32, u64, u32, u64, vp, vp, vp, vp]
        L.ref_rb_step_matrix.restype = None
        L.ref_cs_rb_step_matrix.argtypes = [vp, i32, i64, i64, i64, i64, f32, u64, u32, u64, vp, i32, vp, vp]
        L.ref_cs_rb_step_matrix.restype = None
        L.ref_ss_step_matrix.argtypes = [vp, i32, i64, i32, i32, f32, u64, u32, u64, vp, vp, vp, vp]
        L.ref_ss_step_matrix.restype = f32
        L.ref_cs_ss_step_matrix.argtypes = [vp, i32, i64, i64, i64, f32, u64, u32, vp, i32, vp, vp]
        L.ref_cs_ss_step_matrix.restype = f32
        L.ref_i_form_p.argtypes = [vp, i32, vp, vp, vp, vp, i64, i32, i32, vp, vp]
        L.ref_i_form_p.restype = None
        L.ref_i_rb_step_matrix.argtypes = [vp, i32, i64, i64, i32, i32, u64, u32, u64, vp, vp, vp, vp, vp, vp]
        L.ref_i_rb_step_matrix.restype = None
        L.ref_i_ss_step_matrix.argtypes = [vp, i32, i64, i32, i32, u64, u32, u64, vp, vp, vp, vp, vp, vp]
        L.ref_i_ss_step_matrix.restype = f32
        L.ref_rk_count.argtypes = [i64, i64]
        L.ref_rk_count.restype = i64
        L.ref_rku_perm.argtypes = [u64, u32, u64, i64, i64]
        L.ref_rku_perm.restype = i64
        L.ref_rku_inverse.argtypes = [u64, u32, u64, i64, i64]
        L.ref_rku_inverse.restype = i64
        L.ref_rk_indices.argtypes = [u64, u32, u64, i64, i64, vp]
        L.ref_rk_indices.restype = None
        L.ref_rk_step_matrix.argtypes = [vp, i32, i64, i64, i32, i32, f32, u64, u32, u64, vp, vp, vp, vp]
        L.ref_rk_step_matrix.restype = None
        L.ref_cs_rk_step_matrix.argtypes = [vp, i32, i64, i64, i64, i64, f32, u64, u32, u64, vp, i32, vp, vp]
        L.ref_cs_rk_step_matrix.restype = None
        L.ref_i_rk_step_matrix.argtypes = [vp, i32, i64, i64, i32, i32, u64, u32, u64, vp, vp, vp, vp, vp, vp]
        L.ref_i_rk_step_matrix.restype = None
        L.ref_csc_decode.argtypes = [vp, i32, i64, i64, i64, vp, vp, vp]
        L.ref_csc_decode.restype = None
        L.ref_csc_form_p.argtypes = [vp, i32, vp, i32, i64, i64, i64, vp, vp, f32, vp]
        L.ref_csc_form_p.restype = None
        L.ref_csc_update.argtypes = [vp, i64, i64, vp, vp, i64, f32, vp, i32]
        L.ref_csc_update.restype = None
        L.ref_csc_step_matrix.argtypes = [vp, i32, i64, i64, i32, i64, f32, u64, u32, vp, i32, vp, vp, vp, vp]
        L.ref_csc_step_matrix.restype = None
        L.ref_i2_start.argtypes = [u64, u32, u64, i64, i64]
        L.ref_i2_start.restype = i64
        L.ref_i2_rb_step_matrix.argtypes = [vp, i32, i64, i64, i64, i32, i32, u64, u32, u64, vp, vp, vp, vp, vp]
        L.ref_i2_rb_step_matrix.restype = None
        L.ref_i2_rk_step_matrix.argtypes = [vp, i32, i64, i64, i64, i32, i32, u64, u32, u64, vp, vp, vp, vp, vp]
        L.ref_i2_rk_step_matrix.restype = None
        L.ref_i_error.argtypes = [vp, i64, i32, i32, u64, u32, u64, vp, vp, vp, vp, vp]
        L.ref_i_error.restype = None
        L.ref_i_step_matrix.argtypes = [vp, i32, i64, i64, i32, i32, i32, u64, u32, u64, vp, vp, vp, vp, vp, vp, vp, vp]
        L.ref_i_step_matrix.restype = None
        L.ref_num_threads.argtypes = []
        L.ref_num_threads.restype = i32
        _lib = L
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


def levels(bits: int) -> int:
    return (1 << (bits - 1)) - 1


def n_words(N: int, bits: int) -> int:
    W = 32 // bits
    return (N + W - 1) // W


def n_blocks(N: int, block: int) -> int:
    return (N + block - 1) // block


def num_threads() -> int:
    return int(lib().ref_num_threads())


# ---------------------------------------------------------------- random bits
def philox4x32_10(ctr, key) -> np.ndarray:
    c, k = _c(ctr, np.uint32), _c(key, np.uint32)
    out = np.zeros(4, np.uint32)
    lib().ref_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def rand16(seed: int, mat: int, step: int, j: int) -> int:
    return int(lib().ref_rand16(seed, mat, step, j))


# ---------------------------------------------------------------- codec
def grad_array(g: np.ndarray):
    """Returns (contiguous array, dtype tag).  bf16 gradients travel as uint16 bit patterns."""
    if g.dtype == np.float32:
        return np.ascontiguousarray(g), F32
    if g.dtype == np.uint16:
        return np.ascontiguousarray(g), BF16
    raise TypeError("gradient must be float32 or uint16 (bf16 bits)")


def unpack_codes(codes: np.ndarray, N: int, bits: int) -> np.ndarray:
    c = _c(codes, np.uint32)
    return np.array([lib().ref_get_code(_p(c), j, bits) for j in range(N)], np.int32)


def decode(codes, scales, N: int, bits: int, block: int) -> np.ndarray:
    c, s = _c(codes, np.uint32), _c(scales, np.float32)
    e = np.empty(N, np.float32)
    lib().ref_decode(_p(c), _p(s), N, bits, block, _p(e))
    return e


def form_p(g, codes, scales, bits: int, block: int) -> np.ndarray:
    ga, dt = grad_array(g)
    N = ga.size
    c, s = _c(codes, np.uint32), _c(scales, np.float32)
    p = np.empty(N, np.float32)
    lib().ref_form_p(_p(ga), dt, _p(c), _p(s), N, bits, block, _p(p))
    return p.reshape(g.shape)


def form_p_partial(g, codes, scales, bits: int, block: int, beta: float) -> np.ndarray:
    """The accumulation step of Algorithm 4: g + (1 - beta) decode(codes, scales)."""
    ga, dt = grad_array(g)
    N = ga.size
    c, s = _c(codes, np.uint32), _c(scales, np.float32)
    p = np.empty(N, np.float32)
    lib().ref_form_p_partial(_p(ga), dt, _p(c), _p(s), N, bits, block, beta, _p(p))
    return p.reshape(g.shape)


def quantise(x, bits: int, block: int, seed: int = 0, mat: int = 0, step: int = 0, draw=None):
    """eq. (3) with block max-norm.  Returns (codes uint32[n_words], scales float32[n_blocks])."""
    xa = _c(x, np.float32).ravel()
    N = xa.size
    assert block % (32 // bits) == 0
    codes = np.zeros(n_words(N, bits), np.uint32)
    scales = np.zeros(n_blocks(N, block), np.float32)
    d = None if draw is None else _c(draw, np.uint16).ravel()
    lib().ref_quantise(_p(xa), N, bits, block, seed, mat, step,
                       None if d is None else _p(d), _p(codes), _p(scales))
    return codes, scales


# ---------------------------------------------------------------- rank-r compressor
def lowrank_P(p, Q) -> np.ndarray:
    pa, Qa = _c(p, np.float32), _c(Q, np.float32)
    n, m = pa.shape
    r = Qa.shape[1]
    assert Qa.shape[0] == m and r <= 64
    P = np.empty((n, r), np.float32)
    lib().ref_lowrank_P(_p(pa), n, m, _p(Qa), r, _p(P))
    return P


def orthonormalise(P) -> np.ndarray:
    Pa = np.array(P, dtype=np.float32, order="C", copy=True)
    n, r = Pa.shape
    lib().ref_orthonormalise(_p(Pa), n, r)
    return Pa


def lowrank_Q(p, Phat) -> np.ndarray:
    pa, Pa = _c(p, np.float32), _c(Phat, np.float32)
    n, m = pa.shape
    r = Pa.shape[1]
    Qn = np.empty((m, r), np.float32)
    lib().ref_lowrank_Q(_p(pa), n, m, _p(Pa), r, _p(Qn))
    return Qn


def residual(p, Phat, Qn) -> np.ndarray:
    pa, Pa, Qa = _c(p, np.float32), _c(Phat, np.float32), _c(Qn, np.float32)
    n, m = pa.shape
    x = np.empty((n, m), np.float32)
    lib().ref_residual(_p(pa), n, m, _p(Pa), _p(Qa), Pa.shape[1], _p(x))
    return x


def decompress(Phat, Qn) -> np.ndarray:
    """Delta = Phat Qn^T (the aggregated compressed gradient of Algorithm 2, for one worker), each entry an fp32 fma chain over c."""
    Pa, Qa = _c(Phat, np.float32), _c(Qn, np.float32)
    n, m = Pa.shape[0], Qa.shape[0]
    delta = np.empty((n, m), np.float32)
    lib().ref_decompress(n, m, _p(Pa), _p(Qa), Pa.shape[1], _p(delta))
    return delta


def apply_update(x, Phat, Qn) -> np.ndarray:
    """x - Phat Qn^T (the update step of Algorithm 2); returns a new array."""
    xa = np.array(x, np.float32, order="C", copy=True)
    Pa, Qa = _c(Phat, np.float32), _c(Qn, np.float32)
    n, m = xa.shape
    lib().ref_apply_update(_p(xa), n, m, _p(Pa), _p(Qa), Pa.shape[1])
    return xa


# ---------------------------------------------------------------- whole step
@dataclass
class MatState:
    """Per-matrix persistent state of the path: compressed error and the warm-started Q."""
    n: int
    m: int
    codes: np.ndarray
    scales: np.ndarray
    Q: np.ndarray

    @staticmethod
    def fresh(n: int, m: int, bits: int, block: int, Q0: np.ndarray) -> "MatState":
        N = n * m
        return MatState(n, m, np.zeros(n_words(N, bits), np.uint32),
                        np.zeros(n_blocks(N, block), np.float32),
                        np.array(Q0, np.float32, order="C", copy=True))


def step_matrix(g, st: MatState, rank: int, bits: int, block: int, seed: int, mat: int, step: int):
    """Runs one ConEF step on one matrix; updates `st` in place; returns (Phat, Qn)."""
    ga, dt = grad_array(g)
    n, m = st.n, st.m
    assert ga.size == n * m and st.Q.shape == (m, rank)
    P = np.empty((n, rank), np.float32)
    Qn = np.empty((m, rank), np.float32)
    work = np.empty(2 * n * m, np.float32)
    lib().ref_step_matrix(_p(ga), dt, n, m, rank, bits, block, seed, mat, step,
                          _p(st.codes), _p(st.scales), _p(st.Q), _p(P), _p(Qn), _p(work))
    st.Q = Qn
    return P, Qn


def step_matrix_partial(g, st: MatState, rank: int, bits: int, block: int, beta: float, seed: int, mat: int, step: int):
    """One partial-ConEF step (Algorithm 4) with the quantiser; updates `st`; returns (Phat, Qn)."""
    ga, dt = grad_array(g)
    n, m = st.n, st.m
    assert ga.size == n * m and st.Q.shape == (m, rank)
    P = np.empty((n, rank), np.float32)
    Qn = np.empty((m, rank), np.float32)
    work = np.empty(2 * n * m, np.float32)
    lib().ref_step_matrix_partial(_p(ga), dt, n, m, rank, bits, block, beta, seed, mat, step,
                                  _p(st.codes), _p(st.scales), _p(st.Q), _p(P), _p(Qn), _p(work))
    st.Q = Qn
    return P, Qn


def step_matrix_efsgd(g, e, Q):
    """Algorithm 1 (uncompressed error) with the same rank-r compressor. e updated in place."""
    ga = _c(g, np.float32)
    n, m = ga.shape
    Qa = _c(Q, np.float32)
    r = Qa.shape[1]
    assert e.dtype == np.float32 and e.flags.c_contiguous and e.shape == (n, m)
    P = np.empty((n, r), np.float32)
    Qn = np.empty((m, r), np.float32)
    work = np.empty(n * m, np.float32)
    lib().ref_step_matrix_efsgd(_p(ga), n, m, r, _p(e), _p(Qa), _p(P), _p(Qn), _p(work))
    return P, Qn


# ---------------------------------------------------------------- count sketch (oracle/sketch_ref.c)
TABLE_F32, TABLE_F16 = 0, 1


def f32_to_f16(x: float) -> int:
    return int(lib().ref_f32_to_f16(float(np.float32(x))))


def f16_to_f32(h: int) -> float:
    return float(lib().ref_f16_to_f32(int(h)))


def table_array(table: np.ndarray):
    """Returns (contiguous array, type tag).  fp16 tables travel as uint16 bit patterns."""
    if table.dtype == np.float32:
        return np.ascontiguousarray(table), TABLE_F32
    if table.dtype == np.uint16:
        return np.ascontiguousarray(table), TABLE_F16
    raise TypeError("table must be float32 or uint16 (fp16 bits)")


def cs_hash(seed: int, mat: int, n: int, w: int):
    """Bucket (0..w-1) and sign (+1/-1) of every row of matrix `mat` (Section 4.2.2, row tensor trick)."""
    bucket, sign = np.empty(n, np.int32), np.empty(n, np.int8)
    lib().ref_cs_hash(seed, mat, n, w, _p(bucket), _p(sign))
    return bucket, sign


def cs_decode(table, bucket, sign, n: int) -> np.ndarray:
    ta, tt = table_array(table)
    m = ta.shape[1]
    b, s = _c(bucket, np.int32), _c(sign, np.int8)
    e = np.empty((n, m), np.float32)
    lib().ref_cs_decode(_p(ta), tt, n, m, _p(b), _p(s), _p(e))
    return e


def cs_form_p(g, table, bucket, sign, beta: float) -> np.ndarray:
    ga, dt = grad_array(g)
    ta, tt = table_array(table)
    n, m = g.shape
    b, s = _c(bucket, np.int32), _c(sign, np.int8)
    p = np.empty((n, m), np.float32)
    lib().ref_cs_form_p(_p(ga), dt, _p(ta), tt, n, m, _p(b), _p(s), beta, _p(p))
    return p


def cs_update(x, bucket, sign, beta: float, table) -> None:
    """table <- beta * table + sketch(x), in place (the error step of Algorithm 4, by linearity)."""
    xa = _c(x, np.float32)
    n, m = xa.shape
    assert table.flags.c_contiguous and table.shape[1] == m
    _, tt = table_array(table)
    b, s = _c(bucket, np.int32), _c(sign, np.int8)
    lib().ref_cs_update(_p(xa), n, m, _p(b), _p(s), table.shape[0], beta, _p(table), tt)


@dataclass
class SketchState:
    """Per-matrix persistent state of ConEF-CS: the w x m table and the warm-started Q."""
    n: int
    m: int
    table: np.ndarray
    Q: np.ndarray

    @staticmethod
    def fresh(n: int, m: int, w: int, fp16: bool, Q0: np.ndarray) -> "SketchState":
        return SketchState(n, m, np.zeros((w, m), np.uint16 if fp16 else np.float32),
                           np.array(Q0, np.float32, order="C", copy=True))


def cs_step_matrix(g, st: SketchState, rank: int, beta: float, seed: int, mat: int):
    """Runs one partial-ConEF step with the count sketch on one matrix; updates `st`; returns (Phat, Qn)."""
    ga, dt = grad_array(g)
    n, m = st.n, st.m
    assert ga.size == n * m and st.Q.shape == (m, rank) and st.table.flags.c_contiguous
    _, tt = table_array(st.table)
    P = np.empty((n, rank), np.float32)
    Qn = np.empty((m, rank), np.float32)
    work = np.empty(2 * n * m, np.float32)
    lib().ref_cs_step_matrix(_p(ga), dt, n, m, rank, st.table.shape[0], beta, seed, mat,
                             _p(st.table), tt, _p(st.Q), _p(P), _p(Qn), _p(work))
    st.Q = Qn
    return P, Qn


# ---------------------------------------------------------------- random-block gradient compressor (oracle/randblock_ref.c)
def rb_start(seed: int, mat: int, step: int, N: int, k: int) -> int:
    return int(lib().ref_rb_start(seed, mat, step, N, k))


def rb_step_matrix(g, codes, scales, k: int, bits: int, block: int, beta: float, seed: int, mat: int, step: int):
    """One step with the random-block compressor and the quantiser; codes/scales updated in place; returns Delta (k values)."""
    ga, dt = grad_array(g)
    N = ga.size
    assert codes.dtype == np.uint32 and scales.dtype == np.float32 and codes.flags.c_contiguous and scales.flags.c_contiguous
    delta = np.empty(k, np.float32)
    work = np.empty(2 * N, np.float32)
    lib().ref_rb_step_matrix(_p(ga), dt, N, k, bits, block, beta, seed, mat, step, _p(codes), _p(scales), _p(delta), _p(work))
    return delta


def cs_rb_step_matrix(g, table, k: int, beta: float, seed: int, mat: int, step: int):
    """The same with the count sketch; `table` (w x m) updated in place; returns Delta."""
    ga, dt = grad_array(g)
    n, m = g.shape
    _, tt = table_array(table)
    assert table.flags.c_contiguous and table.shape[1] == m
    delta = np.empty(k, np.float32)
    work = np.empty(n * m, np.float32)
    lib().ref_cs_rb_step_matrix(_p(ga), dt, n, m, k, table.shape[0], beta, seed, mat, step, _p(table), tt, _p(delta), _p(work))
    return delta


# ---------------------------------------------------------------- scaled-sign gradient compressor (oracle/randblock_ref.c)
def ss_step_matrix(g, codes, scales, bits: int, block: int, beta: float, seed: int, mat: int, step: int):
    """One step with the scaled-sign compressor and the quantiser; codes/scales updated in place.
    Returns (sign words uint32[ceil(N/32)], c)."""
    ga, dt = grad_array(g)
    N = ga.size
    assert codes.dtype == np.uint32 and scales.dtype == np.float32 and codes.flags.c_contiguous and scales.flags.c_contiguous
    words = np.empty((N + 31) // 32, np.uint32)
    work = np.empty(2 * N, np.float32)
    c = lib().ref_ss_step_matrix(_p(ga), dt, N, bits, block, beta, seed, mat, step, _p(codes), _p(scales), _p(words), _p(work))
    return words, np.float32(c)


def cs_ss_step_matrix(g, table, beta: float, seed: int, mat: int):
    """The same with the count sketch; `table` (w x m) updated in place.  Returns (sign words, c)."""
    ga, dt = grad_array(g)
    n, m = g.shape
    _, tt = table_array(table)
    assert table.flags.c_contiguous and table.shape[1] == m
    words = np.empty((n * m + 31) // 32, np.uint32)
    work = np.empty(n * m, np.float32)
    c = lib().ref_cs_ss_step_matrix(_p(ga), dt, n, m, table.shape[0], beta, seed, mat, _p(table), tt, _p(words), _p(work))
    return words, np.float32(c)


# ---------------------------------------------------------------- iConEF version 1 (oracle/iconef_ref.c)
def _check_state(*arrays):
    for a in arrays:
        assert a.flags.c_contiguous and a.dtype in (np.uint32, np.float32)


def i_form_p(g, codes, scales, codes2, scales2, bits: int, block: int) -> np.ndarray:
    """p = g + e~ + q (Algorithm 3, accumulation), flat fp32."""
    ga, dt = grad_array(g)
    N = ga.size
    _check_state(codes, scales, codes2, scales2)
    tmp, p = np.empty(N, np.float32), np.empty(N, np.float32)
    lib().ref_i_form_p(_p(ga), dt, _p(codes), _p(scales), _p(codes2), _p(scales2), N, bits, block, _p(tmp), _p(p))
    return p


def i_rb_step_matrix(g, codes, scales, codes2, scales2, k: int, bits: int, block: int, seed: int, mat: int, step: int):
    """One iConEF-v1 step with the random-block compressor; both vectors updated in place; returns Delta (k values)."""
    ga, dt = grad_array(g)
    N = ga.size
    _check_state(codes, scales, codes2, scales2)
    delta = np.empty(k, np.float32)
    work = np.empty(2 * N, np.float32)
    lib().ref_i_rb_step_matrix(_p(ga), dt, N, k, bits, block, seed, mat, step, _p(codes), _p(scales), _p(codes2),
                               _p(scales2), _p(delta), _p(work))
    return delta


def i_ss_step_matrix(g, codes, scales, codes2, scales2, bits: int, block: int, seed: int, mat: int, step: int):
    """One iConEF-v1 step with the scaled-sign compressor; both vectors updated in place; returns (sign words, c)."""
    ga, dt = grad_array(g)
    N = ga.size
    _check_state(codes, scales, codes2, scales2)
    words = np.empty((N + 31) // 32, np.uint32)
    work = np.empty(2 * N, np.float32)
    c = lib().ref_i_ss_step_matrix(_p(ga), dt, N, bits, block, seed, mat, step, _p(codes), _p(scales), _p(codes2),
                                   _p(scales2), _p(words), _p(work))
    return words, np.float32(c)


# ---------------------------------------------------------------- random-k gradient compressor, stratified (oracle/randk_ref.c)
def rk_count(N: int, G: int) -> int:
    return int(lib().ref_rk_count(N, G))


def rku_perm(seed: int, mat: int, step: int, N: int, j: int) -> int:
    """pi(j) of the uniformly drawn subset's keyed permutation (kept iff below k; the slot of the kept value)."""
    return int(lib().ref_rku_perm(seed, mat, step, N, j))


def rku_inverse(seed: int, mat: int, step: int, N: int, i: int) -> int:
    return int(lib().ref_rku_inverse(seed, mat, step, N, i))


def rk_indices(seed: int, mat: int, step: int, N: int, G: int) -> np.ndarray:
    """Kept coordinate of every stratum (int64, ascending); G < 0: the coordinates of the uniformly drawn subset of -G,
    in slot order.  Every rk step routine below takes G < 0 in that sense."""
    idx = np.empty(rk_count(N, G), np.int64)
    lib().ref_rk_indices(seed, mat, step, N, G, _p(idx))
    return idx


def rk_step_matrix(g, codes, scales, G: int, bits: int, block: int, beta: float, seed: int, mat: int, step: int):
    """One step with the random-k compressor and the quantiser; codes/scales updated in place; returns Delta (k values)."""
    ga, dt = grad_array(g)
    N = ga.size
    _check_state(codes, scales)
    delta = np.empty(rk_count(N, G), np.float32)
    work = np.empty(2 * N, np.float32)
    lib().ref_rk_step_matrix(_p(ga), dt, N, G, bits, block, beta, seed, mat, step, _p(codes), _p(scales), _p(delta), _p(work))
    return delta


def cs_rk_step_matrix(g, table, G: int, beta: float, seed: int, mat: int, step: int):
    """The same with the count sketch; `table` (w x m) updated in place; returns Delta."""
    ga, dt = grad_array(g)
    n, m = g.shape
    _, tt = table_array(table)
    assert table.flags.c_contiguous and table.shape[1] == m
    delta = np.empty(rk_count(n * m, G), np.float32)
    work = np.empty(n * m, np.float32)
    lib().ref_cs_rk_step_matrix(_p(ga), dt, n, m, G, table.shape[0], beta, seed, mat, step, _p(table), tt, _p(delta), _p(work))
    return delta


def i_rk_step_matrix(g, codes, scales, codes2, scales2, G: int, bits: int, block: int, seed: int, mat: int, step: int):
    """One iConEF-v1 step with the random-k compressor; both vectors updated in place; returns Delta."""
    ga, dt = grad_array(g)
    N = ga.size
    _check_state(codes, scales, codes2, scales2)
    delta = np.empty(rk_count(N, G), np.float32)
    work = np.empty(2 * N, np.float32)
    lib().ref_i_rk_step_matrix(_p(ga), dt, N, G, bits, block, seed, mat, step, _p(codes), _p(scales), _p(codes2),
                               _p(scales2), _p(delta), _p(work))
    return delta


# ---------------------------------------------------------------- count sketch, column form (oracle/sketch_col_ref.c)
# The table is n x w; bucket / sign come from cs_hash(seed, mat, m, w): one hash per column.
def csc_decode(table, bucket, sign, m: int) -> np.ndarray:
    ta, tt = table_array(table)
    n, w = ta.shape
    b, s = _c(bucket, np.int32), _c(sign, np.int8)
    e = np.empty((n, m), np.float32)
    lib().ref_csc_decode(_p(ta), tt, n, m, w, _p(b), _p(s), _p(e))
    return e


def csc_form_p(g, table, bucket, sign, beta: float) -> np.ndarray:
    ga, dt = grad_array(g)
    ta, tt = table_array(table)
    n, m = g.shape
    assert ta.shape[0] == n
    b, s = _c(bucket, np.int32), _c(sign, np.int8)
    p = np.empty((n, m), np.float32)
    lib().ref_csc_form_p(_p(ga), dt, _p(ta), tt, n, m, ta.shape[1], _p(b), _p(s), beta, _p(p))
    return p


def csc_update(x, bucket, sign, beta: float, table) -> None:
    """table (n x w) <- beta * table + column sketch of x, in place."""
    xa = _c(x, np.float32)
    n, m = xa.shape
    assert table.flags.c_contiguous and table.shape[0] == n
    _, tt = table_array(table)
    b, s = _c(bucket, np.int32), _c(sign, np.int8)
    lib().ref_csc_update(_p(xa), n, m, _p(b), _p(s), table.shape[1], beta, _p(table), tt)


def csc_step_matrix(g, table, Q, rank: int, beta: float, seed: int, mat: int):
    """One partial-ConEF step with the column count sketch on one matrix; `table` (n x w) updated in place; returns
    (Phat, Qn)."""
    ga, dt = grad_array(g)
    n, m = g.shape
    assert table.flags.c_contiguous and table.shape[0] == n
    _, tt = table_array(table)
    Qs = np.ascontiguousarray(Q, np.float32)
    P, Qn = np.empty((n, rank), np.float32), np.empty((m, rank), np.float32)
    work = np.empty(2 * n * m, np.float32)
    lib().ref_csc_step_matrix(_p(ga), dt, n, m, rank, table.shape[1], beta, seed, mat, _p(table), tt, _p(Qs), _p(P), _p(Qn),
                              _p(work))
    return P, Qn


# ---------------------------------------------------------------- iConEF version 2 (oracle/iconef2_ref.c)
def i2_start(seed: int, mat: int, step: int, N: int, ke: int) -> int:
    """First coordinate of the block the first error compressor keeps when it runs at `step` (step taken mod 2^64)."""
    return int(lib().ref_i2_start(seed, mat, step % (1 << 64), N, ke))


def _i2_step(fn, g, e_vals, codes, scales, arg, n_delta: int, bits: int, block: int, seed: int, mat: int, step: int):
    ga, dt = grad_array(g)
    N = ga.size
    _check_state(codes, scales)
    assert e_vals.dtype == np.float32 and e_vals.flags.c_contiguous and 0 <= e_vals.size <= N
    delta = np.empty(n_delta, np.float32)
    work = np.empty(N, np.float32)
    fn(_p(ga), dt, N, arg, e_vals.size, bits, block, seed, mat, step, _p(e_vals), _p(codes), _p(scales), _p(delta), _p(work))
    return delta


def i2_rb_step_matrix(g, e_vals, codes, scales, k: int, bits: int, block: int, seed: int, mat: int, step: int):
    """One iConEF-v2 step, random block of k as gradient compressor, random block of e_vals.size as first error
    compressor; e_vals, codes, scales updated in place; returns Delta (k values)."""
    return _i2_step(lib().ref_i2_rb_step_matrix, g, e_vals, codes, scales, k, k, bits, block, seed, mat, step)


def i2_rk_step_matrix(g, e_vals, codes, scales, G: int, bits: int, block: int, seed: int, mat: int, step: int):
    """The same with the stratified random-k gradient compressor (strata of G); returns Delta."""
    return _i2_step(lib().ref_i2_rk_step_matrix, g, e_vals, codes, scales, G, rk_count(np.asarray(g).size, G), bits, block,
                    seed, mat, step)


def i_error(x, codes, scales, codes2, scales2, bits: int, block: int, seed: int, mat: int, step: int) -> None:
    """The two error steps of Algorithm 3 on x = p - Delta (flat fp32, left unchanged): both vectors replaced."""
    xa = np.ascontiguousarray(x, np.float32).ravel().copy()
    _check_state(codes, scales, codes2, scales2)
    tmp = np.empty(xa.size, np.float32)
    lib().ref_i_error(_p(xa), xa.size, bits, block, seed, mat, step, _p(codes), _p(scales), _p(codes2), _p(scales2), _p(tmp))


def i_step_matrix(g, codes, scales, codes2, scales2, Q, rank: int, bits: int, block: int, seed: int, mat: int, step: int):
    """One iConEF-v1 step with the rank-r compressor; both vectors updated in place; returns (P^, Q+)."""
    ga, dt = grad_array(g)
    n, m = g.shape
    _check_state(codes, scales, codes2, scales2)
    Qs = np.ascontiguousarray(Q, np.float32)
    assert Qs.shape == (m, rank)
    P_out, Q_out = np.empty((n, rank), np.float32), np.empty((m, rank), np.float32)
    work = np.empty(3 * n * m, np.float32)
    lib().ref_i_step_matrix(_p(ga), dt, n, m, rank, bits, block, seed, mat, step, _p(codes), _p(scales), _p(codes2),
                            _p(scales2), _p(Qs), _p(P_out), _p(Q_out), _p(work))
    return P_out, Q_out
