"""Thin ctypes face of libconef.so: the functions of include/conef.h under the same names,
plus `Model`, a holder of one context with its buffer sizes and offsets.  Argument
marshalling only -- every step of the path runs in the library's HIP kernels.  There is no
fallback: if the compiled library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Sequence, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libconef.so")

F32, BF16 = 0, 1
TABLE_F32, TABLE_F16 = 0, 1
OK, EINVAL, ENOMEM, EHIP, ESTATE, ETOOBIG = 0, -1, -2, -3, -4, -5
STATIC_WORKSPACE_BYTES = 32 << 20

EXPORTS = ["conef_init", "conef_sizes", "conef_offsets", "conef_step", "conef_step_static", "conef_step_p",
           "conef_orthonormalise", "conef_step_q", "conef_step_err", "conef_reset_error",
           "conef_decode_error", "conef_set_timing", "conef_get_timing", "conef_check_plan", "conef_matrix_family", "conef_decompress",
           "conef_apply_update", "conef_destroy",
           "conef_strerror", "conef_set_beta",
           "conef_ss_sizes", "conef_ss_offsets", "conef_ss_step", "conef_cs_ss_step",
           "conef_rb_configure", "conef_rb_sizes", "conef_rb_offsets", "conef_rb_start", "conef_rb_step", "conef_cs_rb_step",
           "conef_i_rb_step", "conef_i_ss_step", "conef_i_rk_step", "conef_i_step_p", "conef_i_step_q", "conef_i_step_err", "conef_i_step",
           "conef_i2_configure", "conef_i2_sizes", "conef_i2_offsets", "conef_i2_start", "conef_i2_rb_step", "conef_i2_rk_step",
           "conef_rk_configure", "conef_rk_configure_uniform", "conef_rk_sizes", "conef_rk_offsets", "conef_rk_index", "conef_rk_step", "conef_cs_rk_step",
           "conef_cs_init", "conef_csc_init", "conef_cs_sizes", "conef_cs_offsets", "conef_cs_hash", "conef_cs_step",
           "conef_cs_step_p", "conef_cs_step_q", "conef_cs_step_err", "conef_cs_decode_error"]


class conef_mat(ctypes.Structure):
    _fields_ = [("rows", ctypes.c_int64), ("cols", ctypes.c_int64)]


_lib = None


def lib() -> ctypes.CDLL:
    """Loads libconef.so (built by paper_2312_08538_amd.build / __graft_entry__.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2312_08538_amd.build`; "
                           "there is no fallback path")
    L = ctypes.CDLL(LIB_PATH)
    vp, sz, u64, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_uint64, ctypes.c_int
    szp = ctypes.POINTER(sz)
    L.conef_init.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(conef_mat), i32, i32, i32, i32, i32, u64]
    L.conef_sizes.argtypes = [vp, szp, szp, szp, szp, szp, szp]
    L.conef_offsets.argtypes = [vp, i32, szp, szp, szp, szp, szp]
    L.conef_step.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, u64, vp]
    L.conef_step_static.argtypes = [vp, vp, vp, vp, vp, vp, vp, u64, vp]
    L.conef_step_p.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp]
    L.conef_orthonormalise.argtypes = [vp, vp, vp, vp]
    L.conef_step_q.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp]
    L.conef_step_err.argtypes = [vp, vp, vp, vp, vp, vp, vp, u64, vp]
    L.conef_reset_error.argtypes = [vp, vp, vp, vp]
    L.conef_decode_error.argtypes = [vp, vp, vp, vp, vp]
    L.conef_set_timing.argtypes = [vp, i32]
    L.conef_get_timing.argtypes = [vp, ctypes.POINTER(ctypes.c_float)]
    L.conef_check_plan.argtypes = [vp]
    L.conef_matrix_family.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_int)]
    L.conef_set_beta.argtypes = [vp, ctypes.c_float]
    L.conef_ss_sizes.argtypes = [vp, szp]
    L.conef_ss_offsets.argtypes = [vp, i32, szp]
    L.conef_ss_step.argtypes = [vp, vp, vp, vp, vp, vp, vp, u64, vp]
    L.conef_cs_ss_step.argtypes = [vp, vp, vp, vp, vp, vp, vp]
    L.conef_rb_configure.argtypes = [vp, ctypes.POINTER(ctypes.c_int64)]
    L.conef_rb_sizes.argtypes = [vp, szp]
    L.conef_rb_offsets.argtypes = [vp, i32, szp, ctypes.POINTER(ctypes.c_int64)]
    L.conef_rb_start.argtypes = [vp, i32, u64, ctypes.POINTER(ctypes.c_int64)]
    L.conef_rb_step.argtypes = [vp, vp, vp, vp, vp, u64, vp]
    L.conef_i_rb_step.argtypes = [vp, vp, vp, vp, vp, vp, vp, u64, vp]
    L.conef_i_rk_step.argtypes = [vp, vp, vp, vp, vp, vp, vp, u64, vp]
    L.conef_i_step_p.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    L.conef_i_step_q.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    L.conef_i_step_err.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, u64, vp]
    L.conef_i_step.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, u64, vp]
    L.conef_i2_configure.argtypes = [vp, ctypes.POINTER(ctypes.c_int64)]
    L.conef_i2_sizes.argtypes = [vp, szp]
    L.conef_i2_offsets.argtypes = [vp, i32, szp, ctypes.POINTER(ctypes.c_int64)]
    L.conef_i2_start.argtypes = [vp, i32, u64, ctypes.POINTER(ctypes.c_int64)]
    L.conef_i2_rb_step.argtypes = [vp, vp, vp, vp, vp, vp, vp, u64, vp]
    L.conef_i2_rk_step.argtypes = [vp, vp, vp, vp, vp, vp, vp, u64, vp]
    L.conef_rk_configure.argtypes = [vp, ctypes.POINTER(ctypes.c_int64)]
    L.conef_rk_configure_uniform.argtypes = [vp, ctypes.POINTER(ctypes.c_int64)]
    L.conef_rk_sizes.argtypes = [vp, szp]
    L.conef_rk_offsets.argtypes = [vp, i32, szp, ctypes.POINTER(ctypes.c_int64)]
    L.conef_rk_index.argtypes = [vp, i32, u64, ctypes.c_int64, ctypes.POINTER(ctypes.c_int64)]
    L.conef_rk_step.argtypes = [vp, vp, vp, vp, vp, u64, vp]
    L.conef_cs_rk_step.argtypes = [vp, vp, vp, vp, u64, vp]
    L.conef_i_ss_step.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, u64, vp]
    L.conef_cs_rb_step.argtypes = [vp, vp, vp, vp, u64, vp]
    L.conef_decompress.argtypes = [vp, vp, vp, vp, vp]
    L.conef_apply_update.argtypes = [vp, vp, vp, vp, vp]
    L.conef_cs_init.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(conef_mat), ctypes.POINTER(ctypes.c_int64), i32, i32,
                                ctypes.c_float, i32, i32, u64]
    L.conef_csc_init.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(conef_mat), ctypes.POINTER(ctypes.c_int64), i32, i32,
                                ctypes.c_float, i32, i32, u64]
    L.conef_cs_sizes.argtypes = [vp, szp]
    L.conef_cs_offsets.argtypes = [vp, i32, szp, ctypes.POINTER(ctypes.c_int64)]
    L.conef_cs_hash.argtypes = [vp, i32, vp, vp]
    L.conef_cs_step.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp]
    L.conef_cs_step_p.argtypes = [vp, vp, vp, vp, vp, vp, vp]
    L.conef_cs_step_q.argtypes = [vp, vp, vp, vp, vp, vp, vp]
    L.conef_cs_step_err.argtypes = [vp, vp, vp, vp, vp, vp, vp]
    L.conef_cs_decode_error.argtypes = [vp, vp, vp, vp]
    L.conef_destroy.argtypes = [vp]
    L.conef_destroy.restype = None
    L.conef_strerror.argtypes = [i32]
    L.conef_strerror.restype = ctypes.c_char_p
    for name in EXPORTS:
        if name not in ("conef_destroy", "conef_strerror"):
            getattr(L, name).restype = i32
    _lib = L
    return L


class ConefError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {lib().conef_strerror(code).decode()} ({code})")


def _check(code: int, where: str) -> None:
    if code != OK:
        raise ConefError(code, where)


def _ptr(t) -> int:
    """Device (or host) address of a torch tensor / numpy array / raw int."""
    if t is None:
        return 0
    if isinstance(t, int):
        return t
    if hasattr(t, "data_ptr"):
        return t.data_ptr()
    return t.ctypes.data


# ------------------------------------------------------------------ plain functions, C names
def conef_init(layout: Sequence[Tuple[int, int]], rank: int, bits: int, block: int, grad_dtype: int, seed: int):
    arr = (conef_mat * max(1, len(layout)))()
    for i, (n, m) in enumerate(layout):
        arr[i].rows, arr[i].cols = n, m
    ctx = ctypes.c_void_p()
    _check(lib().conef_init(ctypes.byref(ctx), arr, len(layout), rank, bits, block, grad_dtype, seed), "conef_init")
    return ctx


def conef_sizes(ctx) -> dict:
    v = [ctypes.c_size_t() for _ in range(6)]
    _check(lib().conef_sizes(ctx, *[ctypes.byref(x) for x in v]), "conef_sizes")
    keys = ["grad_elems", "code_words", "n_scales", "p_elems", "q_elems", "workspace_bytes"]
    return {k: int(x.value) for k, x in zip(keys, v)}


# scaled-sign gradient compressor
def conef_ss_sizes(ctx) -> dict:
    v = ctypes.c_size_t()
    _check(lib().conef_ss_sizes(ctx, ctypes.byref(v)), "conef_ss_sizes")
    return {"sign_words": int(v.value)}


def conef_ss_offsets(ctx, mat: int) -> dict:
    v = ctypes.c_size_t()
    _check(lib().conef_ss_offsets(ctx, mat, ctypes.byref(v)), "conef_ss_offsets")
    return {"sign_off": int(v.value)}


def conef_ss_step(ctx, grads, err_codes, err_scales, sign_out, scale_out, workspace, step: int, stream=0):
    _check(lib().conef_ss_step(ctx, _ptr(grads), _ptr(err_codes), _ptr(err_scales), _ptr(sign_out), _ptr(scale_out),
                               _ptr(workspace), step, stream), "conef_ss_step")


def conef_cs_ss_step(ctx, grads, table, sign_out, scale_out, workspace, stream=0):
    _check(lib().conef_cs_ss_step(ctx, _ptr(grads), _ptr(table), _ptr(sign_out), _ptr(scale_out), _ptr(workspace), stream),
           "conef_cs_ss_step")


# random-block gradient compressor
def conef_rb_configure(ctx, keep: Sequence[int]) -> None:
    arr = (ctypes.c_int64 * max(1, len(keep)))(*[int(x) for x in keep])
    _check(lib().conef_rb_configure(ctx, arr), "conef_rb_configure")


def conef_rb_sizes(ctx) -> dict:
    v = ctypes.c_size_t()
    _check(lib().conef_rb_sizes(ctx, ctypes.byref(v)), "conef_rb_sizes")
    return {"delta_elems": int(v.value)}


def conef_rb_offsets(ctx, mat: int) -> dict:
    off, k = ctypes.c_size_t(), ctypes.c_int64()
    _check(lib().conef_rb_offsets(ctx, mat, ctypes.byref(off), ctypes.byref(k)), "conef_rb_offsets")
    return {"delta_off": int(off.value), "keep": int(k.value)}


def conef_rb_start(ctx, mat: int, step: int) -> int:
    v = ctypes.c_int64()
    _check(lib().conef_rb_start(ctx, mat, step, ctypes.byref(v)), "conef_rb_start")
    return int(v.value)


def conef_rb_step(ctx, grads, err_codes, err_scales, delta_out, step: int, stream=0):
    _check(lib().conef_rb_step(ctx, _ptr(grads), _ptr(err_codes), _ptr(err_scales), _ptr(delta_out), step, stream),
           "conef_rb_step")


def conef_cs_rb_step(ctx, grads, table, delta_out, step: int, stream=0):
    _check(lib().conef_cs_rb_step(ctx, _ptr(grads), _ptr(table), _ptr(delta_out), step, stream), "conef_cs_rb_step")


# improved contractive error feedback, version 1 (two compressed error vectors)
def conef_i_rb_step(ctx, grads, err_codes, err_scales, err2_codes, err2_scales, delta_out, step: int, stream=0):
    _check(lib().conef_i_rb_step(ctx, _ptr(grads), _ptr(err_codes), _ptr(err_scales), _ptr(err2_codes), _ptr(err2_scales),
                                 _ptr(delta_out), step, stream), "conef_i_rb_step")


def conef_i_ss_step(ctx, grads, err_codes, err_scales, err2_codes, err2_scales, sign_out, scale_out, workspace, step: int,
                    stream=0):
    _check(lib().conef_i_ss_step(ctx, _ptr(grads), _ptr(err_codes), _ptr(err_scales), _ptr(err2_codes), _ptr(err2_scales),
                                 _ptr(sign_out), _ptr(scale_out), _ptr(workspace), step, stream), "conef_i_ss_step")


def conef_i_rk_step(ctx, grads, err_codes, err_scales, err2_codes, err2_scales, delta_out, step: int, stream=0):
    _check(lib().conef_i_rk_step(ctx, _ptr(grads), _ptr(err_codes), _ptr(err_scales), _ptr(err2_codes), _ptr(err2_scales),
                                 _ptr(delta_out), step, stream), "conef_i_rk_step")


def conef_i_step_p(ctx, grads, err_codes, err_scales, err2_codes, err2_scales, Q_state, P_raw_out, workspace, stream=0):
    _check(lib().conef_i_step_p(ctx, _ptr(grads), _ptr(err_codes), _ptr(err_scales), _ptr(err2_codes), _ptr(err2_scales),
                                _ptr(Q_state), _ptr(P_raw_out), _ptr(workspace), stream), "conef_i_step_p")


def conef_i_step_q(ctx, grads, err_codes, err_scales, err2_codes, err2_scales, P_hat, Q_out, workspace, stream=0):
    _check(lib().conef_i_step_q(ctx, _ptr(grads), _ptr(err_codes), _ptr(err_scales), _ptr(err2_codes), _ptr(err2_scales),
                                _ptr(P_hat), _ptr(Q_out), _ptr(workspace), stream), "conef_i_step_q")


def conef_i_step_err(ctx, grads, err_codes, err_scales, err2_codes, err2_scales, P_hat, Q_new, workspace, step: int, stream=0):
    _check(lib().conef_i_step_err(ctx, _ptr(grads), _ptr(err_codes), _ptr(err_scales), _ptr(err2_codes), _ptr(err2_scales),
                                  _ptr(P_hat), _ptr(Q_new), _ptr(workspace), step, stream), "conef_i_step_err")


def conef_i_step(ctx, grads, err_codes, err_scales, err2_codes, err2_scales, Q_state, P_out, Q_out, workspace, step: int,
                 stream=0):
    _check(lib().conef_i_step(ctx, _ptr(grads), _ptr(err_codes), _ptr(err_scales), _ptr(err2_codes), _ptr(err2_scales),
                              _ptr(Q_state), _ptr(P_out), _ptr(Q_out), _ptr(workspace), step, stream), "conef_i_step")


# random-k gradient compressor (stratified: one coordinate kept per stratum of group[l] consecutive ones)
def conef_rk_configure(ctx, group: Sequence[int]) -> None:
    arr = (ctypes.c_int64 * max(1, len(group)))(*[int(x) for x in group])
    _check(lib().conef_rk_configure(ctx, arr), "conef_rk_configure")


def conef_rk_configure_uniform(ctx, keep: Sequence[int]) -> None:
    """random-k as a uniformly drawn subset of keep[l] coordinates of matrix l (replaces the strata for the context)"""
    arr = (ctypes.c_int64 * max(1, len(keep)))(*[int(x) for x in keep])
    _check(lib().conef_rk_configure_uniform(ctx, arr), "conef_rk_configure_uniform")


def conef_rk_sizes(ctx) -> dict:
    v = ctypes.c_size_t()
    _check(lib().conef_rk_sizes(ctx, ctypes.byref(v)), "conef_rk_sizes")
    return {"delta_elems": int(v.value)}


def conef_rk_offsets(ctx, mat: int) -> dict:
    off, keep = ctypes.c_size_t(), ctypes.c_int64()
    _check(lib().conef_rk_offsets(ctx, mat, ctypes.byref(off), ctypes.byref(keep)), "conef_rk_offsets")
    return {"delta_off": int(off.value), "keep": int(keep.value)}


def conef_rk_index(ctx, mat: int, step: int, stratum: int) -> int:
    v = ctypes.c_int64()
    _check(lib().conef_rk_index(ctx, mat, step, stratum, ctypes.byref(v)), "conef_rk_index")
    return int(v.value)


def conef_rk_step(ctx, grads, err_codes, err_scales, delta_out, step: int, stream=0):
    _check(lib().conef_rk_step(ctx, _ptr(grads), _ptr(err_codes), _ptr(err_scales), _ptr(delta_out), step, stream),
           "conef_rk_step")


def conef_cs_rk_step(ctx, grads, table, delta_out, step: int, stream=0):
    _check(lib().conef_cs_rk_step(ctx, _ptr(grads), _ptr(table), _ptr(delta_out), step, stream), "conef_cs_rk_step")


# improved contractive error feedback, version 2: the first error vector is a random block kept as it is
def conef_i2_configure(ctx, keep_e: Sequence[int]) -> None:
    arr = (ctypes.c_int64 * max(1, len(keep_e)))(*[int(x) for x in keep_e])
    _check(lib().conef_i2_configure(ctx, arr), "conef_i2_configure")


def conef_i2_sizes(ctx) -> dict:
    v = ctypes.c_size_t()
    _check(lib().conef_i2_sizes(ctx, ctypes.byref(v)), "conef_i2_sizes")
    return {"e_elems": int(v.value)}


def conef_i2_offsets(ctx, mat: int) -> dict:
    off, keep = ctypes.c_size_t(), ctypes.c_int64()
    _check(lib().conef_i2_offsets(ctx, mat, ctypes.byref(off), ctypes.byref(keep)), "conef_i2_offsets")
    return {"e_off": int(off.value), "keep_e": int(keep.value)}


def conef_i2_start(ctx, mat: int, step: int) -> int:
    v = ctypes.c_int64()
    _check(lib().conef_i2_start(ctx, mat, step % (1 << 64), ctypes.byref(v)), "conef_i2_start")
    return int(v.value)


def conef_i2_rb_step(ctx, grads, e_in, e_out, err_codes, err_scales, delta_out, step: int, stream=0):
    _check(lib().conef_i2_rb_step(ctx, _ptr(grads), _ptr(e_in), _ptr(e_out), _ptr(err_codes), _ptr(err_scales), _ptr(delta_out),
                                  step, stream), "conef_i2_rb_step")


def conef_i2_rk_step(ctx, grads, e_in, e_out, err_codes, err_scales, delta_out, step: int, stream=0):
    _check(lib().conef_i2_rk_step(ctx, _ptr(grads), _ptr(e_in), _ptr(e_out), _ptr(err_codes), _ptr(err_scales), _ptr(delta_out),
                                  step, stream), "conef_i2_rk_step")


def conef_set_beta(ctx, beta: float) -> None:
    _check(lib().conef_set_beta(ctx, beta), "conef_set_beta")


def conef_check_plan(ctx) -> None:
    _check(lib().conef_check_plan(ctx), "conef_check_plan")


FAMILY_GENERIC, FAMILY_OCTET, FAMILY_MFMA, FAMILY_PACKED = 0, 1, 2, 3


def conef_matrix_family(ctx, mat: int) -> int:
    """kernel family of a matrix: 0 generic, 1 octet (both accumulate the factors in fp64), 2 rank-32 matrix cores,
    3 octet with the packed-split P and Q+ passes on the bf16 matrix cores (fp32 sums)"""
    v = ctypes.c_int()
    _check(lib().conef_matrix_family(ctx, mat, ctypes.byref(v)), "conef_matrix_family")
    return v.value


def conef_offsets(ctx, mat: int) -> dict:
    v = [ctypes.c_size_t() for _ in range(5)]
    _check(lib().conef_offsets(ctx, mat, *[ctypes.byref(x) for x in v]), "conef_offsets")
    keys = ["grad_off", "word_off", "scale_off", "p_off", "q_off"]
    return {k: int(x.value) for k, x in zip(keys, v)}


def conef_step(ctx, grads, err_codes, err_scales, Q_state, P_out, Q_out, workspace, step: int, stream=0):
    _check(lib().conef_step(ctx, _ptr(grads), _ptr(err_codes), _ptr(err_scales), _ptr(Q_state), _ptr(P_out),
                            _ptr(Q_out), _ptr(workspace), step, stream), "conef_step")


def conef_step_static(ctx, grads, err_codes, err_scales, Q_state, P_out, Q_out, step: int, stream=0):
    _check(lib().conef_step_static(ctx, _ptr(grads), _ptr(err_codes), _ptr(err_scales), _ptr(Q_state), _ptr(P_out),
                                   _ptr(Q_out), step, stream), "conef_step_static")


def conef_step_p(ctx, grads, err_codes, err_scales, Q_state, P_raw_out, workspace, stream=0):
    _check(lib().conef_step_p(ctx, _ptr(grads), _ptr(err_codes), _ptr(err_scales), _ptr(Q_state), _ptr(P_raw_out),
                              _ptr(workspace), stream), "conef_step_p")


def conef_orthonormalise(ctx, P_inout, workspace, stream=0):
    _check(lib().conef_orthonormalise(ctx, _ptr(P_inout), _ptr(workspace), stream), "conef_orthonormalise")


def conef_step_q(ctx, grads, err_codes, err_scales, P_hat, Q_out, workspace, stream=0):
    _check(lib().conef_step_q(ctx, _ptr(grads), _ptr(err_codes), _ptr(err_scales), _ptr(P_hat), _ptr(Q_out),
                              _ptr(workspace), stream), "conef_step_q")


def conef_step_err(ctx, grads, err_codes, err_scales, P_hat, Q_new, workspace, step: int, stream=0):
    _check(lib().conef_step_err(ctx, _ptr(grads), _ptr(err_codes), _ptr(err_scales), _ptr(P_hat), _ptr(Q_new),
                                _ptr(workspace), step, stream), "conef_step_err")


def conef_reset_error(ctx, err_codes, err_scales, stream=0):
    _check(lib().conef_reset_error(ctx, _ptr(err_codes), _ptr(err_scales), stream), "conef_reset_error")


def conef_decode_error(ctx, err_codes, err_scales, e_out, stream=0):
    _check(lib().conef_decode_error(ctx, _ptr(err_codes), _ptr(err_scales), _ptr(e_out), stream),
           "conef_decode_error")


def conef_decompress(ctx, P_hat, Q_new, delta_out, stream=0):
    _check(lib().conef_decompress(ctx, _ptr(P_hat), _ptr(Q_new), _ptr(delta_out), stream), "conef_decompress")


def conef_apply_update(ctx, P_hat, Q_new, params, stream=0):
    _check(lib().conef_apply_update(ctx, _ptr(P_hat), _ptr(Q_new), _ptr(params), stream), "conef_apply_update")


# count-sketch mode
def conef_cs_init(layout: Sequence[Tuple[int, int]], sketch_rows: Sequence[int], rank: int, beta: float,
                  table_dtype: int, grad_dtype: int, seed: int, columns: bool = False):
    """columns: the column form (conef_csc_init; sketch_rows then holds the buckets per matrix, at most its columns)."""
    arr = (conef_mat * max(1, len(layout)))()
    for i, (n, m) in enumerate(layout):
        arr[i].rows, arr[i].cols = n, m
    w = (ctypes.c_int64 * max(1, len(sketch_rows)))(*[int(x) for x in sketch_rows])
    ctx = ctypes.c_void_p()
    fn, name = (lib().conef_csc_init, "conef_csc_init") if columns else (lib().conef_cs_init, "conef_cs_init")
    _check(fn(ctypes.byref(ctx), arr, w, len(layout), rank, beta, table_dtype, grad_dtype, seed), name)
    return ctx


def conef_csc_init(layout, sketch_cols, rank: int, beta: float, table_dtype: int, grad_dtype: int, seed: int):
    return conef_cs_init(layout, sketch_cols, rank, beta, table_dtype, grad_dtype, seed, columns=True)


def conef_cs_sizes(ctx) -> dict:
    v = ctypes.c_size_t()
    _check(lib().conef_cs_sizes(ctx, ctypes.byref(v)), "conef_cs_sizes")
    return {"table_elems": int(v.value)}


def conef_cs_offsets(ctx, mat: int) -> dict:
    off, w = ctypes.c_size_t(), ctypes.c_int64()
    _check(lib().conef_cs_offsets(ctx, mat, ctypes.byref(off), ctypes.byref(w)), "conef_cs_offsets")
    return {"table_off": int(off.value), "sketch_rows": int(w.value)}


def conef_cs_hash(ctx, mat: int, rows: int):
    """(bucket int32[rows], sign int8[rows]) of the rows of matrix `mat`."""
    import numpy as np

    bucket, sign = np.empty(rows, np.int32), np.empty(rows, np.int8)
    _check(lib().conef_cs_hash(ctx, mat, bucket.ctypes.data, sign.ctypes.data), "conef_cs_hash")
    return bucket, sign


def conef_cs_step(ctx, grads, table, Q_state, P_out, Q_out, workspace, stream=0):
    _check(lib().conef_cs_step(ctx, _ptr(grads), _ptr(table), _ptr(Q_state), _ptr(P_out), _ptr(Q_out),
                               _ptr(workspace), stream), "conef_cs_step")


def conef_cs_step_p(ctx, grads, table, Q_state, P_raw_out, workspace, stream=0):
    _check(lib().conef_cs_step_p(ctx, _ptr(grads), _ptr(table), _ptr(Q_state), _ptr(P_raw_out), _ptr(workspace),
                                 stream), "conef_cs_step_p")


def conef_cs_step_q(ctx, grads, table, P_hat, Q_out, workspace, stream=0):
    _check(lib().conef_cs_step_q(ctx, _ptr(grads), _ptr(table), _ptr(P_hat), _ptr(Q_out), _ptr(workspace), stream),
           "conef_cs_step_q")


def conef_cs_step_err(ctx, grads, table, P_hat, Q_new, workspace, stream=0):
    _check(lib().conef_cs_step_err(ctx, _ptr(grads), _ptr(table), _ptr(P_hat), _ptr(Q_new), _ptr(workspace), stream),
           "conef_cs_step_err")


def conef_cs_decode_error(ctx, table, e_out, stream=0):
    _check(lib().conef_cs_decode_error(ctx, _ptr(table), _ptr(e_out), stream), "conef_cs_decode_error")


def conef_set_timing(ctx, on: bool):
    _check(lib().conef_set_timing(ctx, 1 if on else 0), "conef_set_timing")


def conef_get_timing(ctx) -> List[float]:
    ms = (ctypes.c_float * 4)()
    _check(lib().conef_get_timing(ctx, ms), "conef_get_timing")
    return [float(x) for x in ms]


def conef_destroy(ctx):
    lib().conef_destroy(ctx)


# ------------------------------------------------------------------ holder
class Model:
    """One context plus its sizes and per-matrix offsets.  `alloc(device)` returns zeroed torch
    buffers of the right lengths (device memory management is all torch is used for)."""

    def __init__(self, layout, rank, bits, block, grad_dtype, seed):
        self.layout = [tuple(x) for x in layout]
        self.rank, self.bits, self.block, self.grad_dtype, self.seed = rank, bits, block, grad_dtype, seed
        self.ctx = conef_init(self.layout, rank, bits, block, grad_dtype, seed)
        self.sizes = conef_sizes(self.ctx)
        self.offsets = [conef_offsets(self.ctx, l) for l in range(len(self.layout))]

    def close(self):
        if self.ctx is not None:
            conef_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def alloc(self, device="cuda:0"):
        import torch

        s = self.sizes
        gdt = torch.float32 if self.grad_dtype == F32 else torch.bfloat16
        return {
            "grads": torch.zeros(s["grad_elems"], dtype=gdt, device=device),
            "codes": torch.zeros(s["code_words"], dtype=torch.int32, device=device),
            "scales": torch.zeros(s["n_scales"], dtype=torch.float32, device=device),
            "Q": torch.zeros(s["q_elems"], dtype=torch.float32, device=device),
            "P": torch.zeros(s["p_elems"], dtype=torch.float32, device=device),
            "ws": torch.zeros(max(256, s["workspace_bytes"]), dtype=torch.uint8, device=device),
        }

    @staticmethod
    def stream_handle() -> int:
        import torch

        return torch.cuda.current_stream().cuda_stream

    def step(self, buf, step: int, Q_out=None):
        conef_step(self.ctx, buf["grads"], buf["codes"], buf["scales"], buf["Q"], buf["P"],
                   buf["Q"] if Q_out is None else Q_out, buf["ws"], step, self.stream_handle())


class SketchModel:
    """One count-sketch context plus its sizes and per-matrix offsets (see Model)."""

    def __init__(self, layout, sketch_rows, rank, beta, table_dtype, grad_dtype, seed, columns=False):
        self.layout = [tuple(x) for x in layout]
        self.sketch_rows = [int(x) for x in sketch_rows]
        self.rank, self.beta, self.table_dtype, self.grad_dtype, self.seed = rank, beta, table_dtype, grad_dtype, seed
        self.columns = columns
        self.ctx = conef_cs_init(self.layout, self.sketch_rows, rank, beta, table_dtype, grad_dtype, seed, columns)
        self.sizes = conef_sizes(self.ctx)
        self.sizes.update(conef_cs_sizes(self.ctx))
        self.offsets = [dict(conef_offsets(self.ctx, l), **conef_cs_offsets(self.ctx, l))
                        for l in range(len(self.layout))]

    def close(self):
        if self.ctx is not None:
            conef_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def alloc(self, device="cuda:0"):
        import torch

        s = self.sizes
        gdt = torch.float32 if self.grad_dtype == F32 else torch.bfloat16
        tdt = torch.float32 if self.table_dtype == TABLE_F32 else torch.float16
        return {
            "grads": torch.zeros(s["grad_elems"], dtype=gdt, device=device),
            "table": torch.zeros(s["table_elems"], dtype=tdt, device=device),
            "Q": torch.zeros(s["q_elems"], dtype=torch.float32, device=device),
            "P": torch.zeros(s["p_elems"], dtype=torch.float32, device=device),
            "ws": torch.zeros(max(256, s["workspace_bytes"]), dtype=torch.uint8, device=device),
        }

    def step(self, buf, Q_out=None):
        conef_cs_step(self.ctx, buf["grads"], buf["table"], buf["Q"], buf["P"],
                      buf["Q"] if Q_out is None else Q_out, buf["ws"], Model.stream_handle())
