"""Helpers of the GPU parity tests: run the oracle and the library on the same seeded inputs
and compare element by element with the tolerances of the agreement criteria:
  P, Q      relative error <= 1e-4 (fp32 gradients) / 2e-2 (bf16 gradients)
  scales    <= 1e-6 relative
  codes     bit-exact, except where the oracle's pre-rounding value lies within 1e-6 of a
            rounding boundary: there a difference of one level is excused, for at most 1e-4
            of all codes.
"""
from __future__ import annotations

import numpy as np

from oracle import conef_ref as R
from paper_2312_08538_amd import binding as B


def rel_err(got: np.ndarray, want: np.ndarray) -> float:
    """max |got - want| over the matrix, relative to the largest entry of `want`."""
    den = float(np.abs(want).max())
    if den == 0.0:
        return float(np.abs(got).max())
    return float(np.abs(got.astype(np.float64) - want.astype(np.float64)).max()) / den


def unpack(codes: np.ndarray, N: int, bits: int) -> np.ndarray:
    """Vectorised unpack of LSB-first two's-complement fields (layout checked against the oracle's
    own accessor in the CPU tests)."""
    W = 32 // bits
    idx = np.arange(N)
    f = (codes[idx // W].astype(np.uint64) >> (bits * (idx % W)).astype(np.uint64)) & np.uint64((1 << bits) - 1)
    f = f.astype(np.int64)
    return np.where(f >= (1 << (bits - 1)), f - (1 << bits), f).astype(np.int32)


def unpack_at(codes: np.ndarray, idx: np.ndarray, bits: int) -> np.ndarray:
    """Signed fields of the elements `idx` only."""
    W = 32 // bits
    f = (codes[idx // W].astype(np.uint64) >> (bits * (idx % W)).astype(np.uint64)) & np.uint64((1 << bits) - 1)
    f = f.astype(np.int64)
    return np.where(f >= (1 << (bits - 1)), f - (1 << bits), f).astype(np.int32)


def _excuse(bad, g_bad, w_bad, x_oracle, N, bits, block, seed, mat, step, what, rec_oracle, max_frac=1e-4, x_abs_tol=0.0,
            j0=0, stats=None):
    """The boundary rule for the elements `bad` (codes g_bad on the GPU, w_bad in the oracle).  x_abs_tol: a
    bound on the absolute difference of the two sides' residuals that comes from their factors differing
    (whole steps on large matrices), added to the window.  j0: flat index (within the matrix) of element 0 of
    x_oracle, when only a piece of the matrix is looked at.  stats (a dict): counts the differing codes that the
    strict rule (window 1e-6 max(1, u), nothing added) already excuses under "strict" and the others, which need
    the widened window, under "widened"."""
    s = R.levels(bits)
    assert bad.size <= max(1, int(max_frac * N)), f"{what}: {bad.size} of {N} codes differ"
    for j, gj, wj in zip(bad, g_bad, w_bad):
        assert abs(int(gj) - int(wj)) == 1, f"{what}: code {j} differs by more than one level"
        b0 = (j // block) * block
        xb = x_oracle[b0:min(N, b0 + block)]
        a = np.abs(xb).max()
        inv = np.float32(s) / np.float32(a)
        u = np.float32(np.abs(x_oracle[j]) * inv)
        f = float(u - np.floor(u))
        xi = R.rand16(seed, mat, step, int(j0 + j)) / 65536.0
        tol = 1e-6 * max(1.0, float(u))
        if stats is not None:
            strict = abs(f + xi - 1.0) <= tol or abs(float(u) - round(float(u))) <= tol
            stats["strict" if strict else "widened"] = stats.get("strict" if strict else "widened", 0) + 1
        if rec_oracle is not None:
            tol *= max(1.0, float(np.abs(rec_oracle[b0:min(N, b0 + block)]).max()) / float(a))
        tol += x_abs_tol * float(inv)
        near_draw = abs(f + xi - 1.0) <= tol          # rounded up exactly when fraction + draw / 2^16 >= 1
        near_grid = abs(float(u) - round(float(u))) <= tol
        assert near_draw or near_grid, (f"{what}: code {j} differs although the pre-rounding value is not near a "
                                        f"boundary (u={u}, f={f}, xi={xi})")
    return int(bad.size)


def check_codes(got_codes, want_codes, x_oracle, N, bits, block, seed, mat, step, what="", rec_oracle=None, j0=0,
                stats=None):
    """Applies the boundary rule.  x_oracle: the oracle's residual (fp32, flat).  Returns the number
    of excused mismatches.  rec_oracle (flat, sum_c |P^[i,c]| |Q+[k,c]|: the size of the terms of
    the reconstruction) is given for the matrix-core family only: there the factors carry fp32
    rounding, so the residual p - P^ Q+^T has an absolute error of ~1e-6 of those terms, and the
    1e-6 window is taken relative to max(a, rec_block) instead of the block max-norm a."""
    g = unpack(np.asarray(got_codes), N, bits)
    w = unpack(np.asarray(want_codes), N, bits)
    bad = np.nonzero(g != w)[0]
    if bad.size == 0:
        return 0
    return _excuse(bad, g[bad], w[bad], x_oracle, N, bits, block, seed, mat, step, what, rec_oracle, j0=j0, stats=stats)


def check_codes_sparse(got_codes, want_codes, x_of, N, bits, block, seed, mat, step, what="", rec_of=None, x_abs_tol=0.0,
                       stats=None):
    """check_codes for large matrices: code words are compared packed, and only the fields of differing
    words are unpacked; x_of() / rec_of() are called only if something differs."""
    got_codes, want_codes = np.asarray(got_codes), np.asarray(want_codes)
    diffw = np.nonzero(got_codes != want_codes)[0]
    if diffw.size == 0:
        return 0
    W = 32 // bits
    idx = (diffw[:, None].astype(np.int64) * W + np.arange(W, dtype=np.int64)[None, :]).ravel()
    idx = idx[idx < N]
    g, w = unpack_at(got_codes, idx, bits), unpack_at(want_codes, idx, bits)
    sel = g != w
    return _excuse(idx[sel], g[sel], w[sel], x_of(), N, bits, block, seed, mat, step, what,
                   rec_of() if rec_of is not None else None, x_abs_tol=x_abs_tol, stats=stats)


class OracleModel:
    """The oracle run over a list of matrices, keeping per-matrix state."""

    def __init__(self, layout, rank, bits, block, seed, Q0s, beta=0.0):
        self.layout, self.rank, self.bits, self.block, self.seed, self.beta = layout, rank, bits, block, seed, beta
        self.states = [R.MatState.fresh(n, m, bits, block, Q0) for (n, m), Q0 in zip(layout, Q0s)]

    def step(self, grads, step):
        """grads: list of per-matrix arrays.  Returns per matrix (Phat, Qn, residual x)."""
        out = []
        for l, (g, st) in enumerate(zip(grads, self.states)):
            p = R.form_p(g.reshape(st.n, st.m), st.codes, st.scales, self.bits, self.block)      # g + e
            if self.beta == 0.0:
                Ph, Qn = R.step_matrix(g, st, self.rank, self.bits, self.block, self.seed, l, step)
            else:
                Ph, Qn = R.step_matrix_partial(g, st, self.rank, self.bits, self.block, self.beta, self.seed, l, step)
            x = R.residual(p, Ph, Qn).ravel()
            out.append((Ph, Qn, x))
        return out


class GpuModel:
    """The library run over the same list of matrices through the C ABI."""

    def __init__(self, layout, rank, bits, block, dtype, seed, Q0s, device="cuda:0", beta=0.0):
        import torch

        self.torch = torch
        self.m = B.Model(layout, rank, bits, block, dtype, seed)
        if beta != 0.0:
            B.conef_set_beta(self.m.ctx, beta)
        self.buf = self.m.alloc(device)
        self.dtype = dtype
        for l, Q0 in enumerate(Q0s):
            off = self.m.offsets[l]["q_off"]
            self.buf["Q"][off:off + Q0.size] = torch.from_numpy(np.ascontiguousarray(Q0, np.float32).ravel()).to(device)

    def set_grads(self, grads):
        torch = self.torch
        for l, g in enumerate(grads):
            off = self.m.offsets[l]["grad_off"]
            if self.dtype == B.F32:
                t = torch.from_numpy(np.ascontiguousarray(g, np.float32).ravel())
            else:
                t = torch.from_numpy(np.ascontiguousarray(g, np.uint16).ravel().view(np.int16)).view(torch.bfloat16)
            self.buf["grads"][off:off + t.numel()] = t.to(self.buf["grads"].device)

    def step(self, step):
        self.m.step(self.buf, step)
        self.torch.cuda.synchronize()

    def fp32_factors(self, l=None):
        """Does matrix l (any matrix, if None) take a kernel family whose P and Q+ passes add up in fp32 on the bf16
        matrix cores (about 1e-6 relative) instead of in fp64 (last-bit agreement with the oracle)?"""
        mats = range(len(self.m.layout)) if l is None else [l]
        return any(B.conef_matrix_family(self.m.ctx, i) in (B.FAMILY_MFMA, B.FAMILY_PACKED) for i in mats)

    def mat_P(self, l):
        n, _ = self.m.layout[l]
        off = self.m.offsets[l]["p_off"]
        return self.buf["P"][off:off + n * self.m.rank].cpu().numpy().reshape(n, self.m.rank)

    def mat_Q(self, l):
        _, m = self.m.layout[l]
        off = self.m.offsets[l]["q_off"]
        return self.buf["Q"][off:off + m * self.m.rank].cpu().numpy().reshape(m, self.m.rank)

    def mat_codes(self, l):
        n, m = self.m.layout[l]
        off = self.m.offsets[l]["word_off"]
        return self.buf["codes"][off:off + R.n_words(n * m, self.m.bits)].cpu().numpy().view(np.uint32)

    def mat_scales(self, l):
        n, m = self.m.layout[l]
        off = self.m.offsets[l]["scale_off"]
        return self.buf["scales"][off:off + R.n_blocks(n * m, self.m.block)].cpu().numpy()

    def set_Q(self, l, Q):
        off = self.m.offsets[l]["q_off"]
        t = self.torch.from_numpy(np.ascontiguousarray(Q, np.float32).ravel())
        self.buf["Q"][off:off + t.numel()] = t.to(self.buf["Q"].device)

    def set_state(self, l, codes, scales):
        torch = self.torch
        dev = self.buf["codes"].device
        o = self.m.offsets[l]
        self.buf["codes"][o["word_off"]:o["word_off"] + codes.size] = torch.from_numpy(codes.view(np.int32)).to(dev)
        self.buf["scales"][o["scale_off"]:o["scale_off"] + scales.size] = torch.from_numpy(scales).to(dev)


def compare_step(gpu: GpuModel, oracle_out, oracle: OracleModel, step, pq_tol, what="", fp32_factors=None):
    """Compares P, Q, scales and codes of every matrix after a step; returns total excused codes.
    fp32_factors: the path under test accumulates the factors in fp32 (matrix cores), see check_codes; None: asked of
    the library, matrix by matrix."""
    excused = 0
    ask = fp32_factors is None
    for l, (Ph, Qn, x) in enumerate(oracle_out):
        if ask:
            fp32_factors = gpu.fp32_factors(l)
        st = oracle.states[l]
        N = st.n * st.m
        tag = f"{what} mat {l} ({st.n}x{st.m}) step {step}"
        eP = rel_err(gpu.mat_P(l), Ph)
        eQ = rel_err(gpu.mat_Q(l), Qn)
        assert eP <= pq_tol, f"{tag}: P rel err {eP}"
        assert eQ <= pq_tol, f"{tag}: Q rel err {eQ}"
        gs = gpu.mat_scales(l)
        rec = None
        ref_mag = np.abs(st.scales)
        if fp32_factors:
            # magnitude of the terms of the reconstruction: sum_c |P^[i,c]| |Q+[k,c]|
            rec = (np.abs(Ph).astype(np.float64) @ np.abs(Qn).astype(np.float64).T).astype(np.float32).ravel()
            pad = (-N) % oracle.block
            blk_rec = np.abs(np.concatenate([rec, np.zeros(pad, np.float32)])).reshape(-1, oracle.block).max(1)
            ref_mag = np.maximum(ref_mag, blk_rec)
        assert np.all(np.abs(gs - st.scales) <= 1e-6 * ref_mag), f"{tag}: scales differ"
        excused += check_codes(gpu.mat_codes(l), st.codes, x, N, oracle.bits, oracle.block, oracle.seed, l, step, tag,
                               rec_oracle=rec)
    return excused
