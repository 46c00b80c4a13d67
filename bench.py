#!/usr/bin/env python3
"""Benchmark of the ConEF per-worker step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload large|lm|translation|cnn|tiny]

One "step" is one conef_step call: the whole hot path (decode + add, P = pQ, orthonormalise,
Q+ = p^T P^, residual, stochastic quantise + pack) over every matrix of the workload, inputs
resident in HBM.  Prints ONE JSON line: gradient GB/s processed (metric), the roofline of the
dominant kernel from HIP events recorded on the launch stream inside the timed region, and
the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X HBM3E, published peak
STAGES = ["p", "orthonormalise", "q", "err"]
KERNEL_OF_STAGE = {"p": "pass_p (P = (g+e) Q)", "orthonormalise": "gram + cholesky + apply",
                   "q": "pass_q (Q+ = (g+e)^T P^)", "err": "pass_err (residual + quantise + pack)"}


def stage_bytes(w, stage: str) -> float:
    """Algorithmic HBM bytes of one launch of a stage's main kernel over the whole workload:
    per element the gradient (G bytes), b/8 bytes of codes and 4/B bytes of scales are read once
    (and codes + scales written once by the err pass), plus the P and Q factors it touches."""
    G = 4 if w.grad_dtype == 0 else 2
    per_elem_read = G + w.bits / 8 + 4.0 / w.block
    tot = 0.0
    for n, m in w.layout:
        N = n * m
        if stage == "p":
            tot += N * per_elem_read + (m + n) * w.rank * 4
        elif stage == "q":
            tot += N * per_elem_read + (n + m) * w.rank * 4
        elif stage == "err":
            tot += N * per_elem_read + N * (w.bits / 8 + 4.0 / w.block) + (n + m) * w.rank * 4
        else:  # orthonormalise: read P for the Gram matrix, read + write it for the apply
            tot += 3 * n * w.rank * 4
    return tot


def run_gpu(w, steps: int, warmup: int):
    import torch

    from paper_2312_08538_amd import binding as B
    from paper_2312_08538_amd import workloads as wl

    dev = "cuda:0"
    model = B.Model(w.layout, w.rank, w.bits, w.block, w.grad_dtype, w.lib_seed)
    buf = model.alloc(dev)
    goffs = [o["grad_off"] for o in model.offsets]
    qoffs = [o["q_off"] for o in model.offsets]
    # gradient sets to rotate through, so that a small workload is not served from the last-level
    # cache left by the previous step: enough sets to exceed 512 MiB, at least 2, at most 8
    n_sets = max(2, min(8, int(512 * 2**20 // max(1, w.grad_bytes)) + 1))
    gsets = [buf["grads"]] + [torch.empty_like(buf["grads"]) for _ in range(n_sets - 1)]
    for i, g in enumerate(gsets):
        wl.device_fill_gradients(w, i, g, goffs)
    wl.device_q0(w, buf["Q"], qoffs)
    torch.cuda.synchronize()
    st = model.stream_handle()

    def one_step(t):
        B.conef_step(model.ctx, gsets[t % n_sets], buf["codes"], buf["scales"], buf["Q"], buf["P"], buf["Q"],
                     buf["ws"], t, st)

    # the error state grows from step to step on iid synthetic gradients (no decay as in real
    # training); a reset every 16 steps keeps every value finite for any K.  It is a fill kernel
    # of the state buffers on the same stream and is part of the timed work when it happens.
    def maybe_reset(t):
        if t > 0 and t % 16 == 0:
            B.conef_reset_error(model.ctx, buf["codes"], buf["scales"], st)

    for t in range(warmup):
        maybe_reset(t)
        one_step(t)
    # The timed region: exactly `steps` steps, bracketed by synchronisation; one event pair per step on the
    # launch stream (torch's current stream, the one the library is given) for the median and the minimum.
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i, t in enumerate(range(warmup, warmup + steps)):
        maybe_reset(t)
        ev[i][0].record()
        one_step(t)
        ev[i][1].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    per_step = sorted(e0.elapsed_time(e1) for e0, e1 in ev)
    stats = {"median_ms": round(per_step[len(per_step) // 2] if len(per_step) % 2 else
                                0.5 * (per_step[len(per_step) // 2 - 1] + per_step[len(per_step) // 2]), 4),
             "min_ms": round(per_step[0], 4), "max_ms": round(per_step[-1], 4)}
    # Stage durations: the same steps again with the library's stage events on (the events sit between the
    # kernels of a step, so these steps are kept out of the timed region above).
    B.conef_set_timing(model.ctx, True)
    for t in range(warmup + steps, warmup + 2 * steps):
        maybe_reset(t)
        one_step(t)
    torch.cuda.synchronize()
    stage_ms = B.conef_get_timing(model.ctx)
    B.conef_set_timing(model.ctx, False)
    finite = bool(torch.isfinite(buf["P"]).all()) and bool(torch.isfinite(buf["Q"]).all())
    model.close()
    del buf, gsets
    torch.cuda.empty_cache()
    return (t1 - t0) * 1e3 / steps, dict(zip(STAGES, stage_ms)), finite, stats


def run_update(w, reps: int = 10):
    """Times the decompress-and-apply call that follows a step (Algorithm 2 lines 7-8, x <- x - P^ Q+^T)
    on fp32 parameters of the workload's layout, with HIP events on the launch stream.  Not part of
    `value`: the headline step is the compression path; this is reported beside it."""
    import torch

    from paper_2312_08538_amd import binding as B
    from paper_2312_08538_amd import workloads as wl

    model = B.Model(w.layout, w.rank, w.bits, w.block, w.grad_dtype, w.lib_seed)
    P = torch.randn(model.sizes["p_elems"], dtype=torch.float32, device="cuda:0")
    Q = torch.randn(model.sizes["q_elems"], dtype=torch.float32, device="cuda:0") * 1e-3
    x = torch.zeros(model.sizes["grad_elems"], dtype=torch.float32, device="cuda:0")
    st = model.stream_handle()
    for _ in range(2):
        B.conef_apply_update(model.ctx, P, Q, x, st)
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for e0, e1 in ev:                       # the library launches on torch's current stream, where these events go
        e0.record()
        B.conef_apply_update(model.ctx, P, Q, x, st)
        e1.record()
    torch.cuda.synchronize()
    ms = sum(e0.elapsed_time(e1) for e0, e1 in ev) / reps
    finite = bool(torch.isfinite(x).all())
    model.close()
    del P, Q, x
    torch.cuda.empty_cache()
    nbytes = 8 * w.elements + 4 * w.rank * sum(n + m for n, m in w.layout)       # read + write x, read the factors
    return {"ms": round(ms, 4), "bytes": int(nbytes), "GB/s": round(nbytes / (ms * 1e-3) / 1e9, 1),
            "frac_of_peak": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4), "finite": finite}


def sketch_bytes(w, keep: float, table_bytes: int = 2) -> int:
    """Algorithmic HBM bytes of one count-sketch step: the gradient is read three times, the table (keep x
    the matrix, `table_bytes` per entry) three times and written once, plus the factors as in the
    quantiser's step."""
    from paper_2312_08538_amd import workloads as wl

    G = 4 if w.grad_dtype == 0 else 2
    tot = 0.0
    for (n, m), ws in zip(w.layout, wl.sketch_rows(w.layout, keep)):
        tot += n * m * 3 * G + ws * m * 4 * table_bytes + (5 * n + 3 * m) * w.rank * 4
    return int(tot)


def run_sketch(w, keep: float, beta: float, steps: int = 10, warmup: int = 3, columns: bool = False):
    """Times the step with the count sketch as the error compressor (Section 4.2.2, Algorithm 4) on the
    workload's layout: fp16 table of `keep` x rows buckets per matrix (columns: the column form of Section 5.3, `keep` x
    cols buckets), HIP events around the stages."""
    import torch

    from paper_2312_08538_amd import binding as B
    from paper_2312_08538_amd import workloads as wl

    buckets = [max(1, int(m * keep)) for _, m in w.layout] if columns else wl.sketch_rows(w.layout, keep)
    model = B.SketchModel(w.layout, buckets, w.rank, beta, B.TABLE_F16, w.grad_dtype, w.lib_seed, columns=columns)
    buf = model.alloc("cuda:0")
    goffs = [o["grad_off"] for o in model.offsets]
    n_sets = max(2, min(8, int(512 * 2**20 // max(1, w.grad_bytes)) + 1))
    gsets = [buf["grads"]] + [torch.empty_like(buf["grads"]) for _ in range(n_sets - 1)]
    for i, g in enumerate(gsets):
        wl.device_fill_gradients(w, i, g, goffs)
    wl.device_q0(w, buf["Q"], [o["q_off"] for o in model.offsets])
    torch.cuda.synchronize()
    st = B.Model.stream_handle()

    def one_step(t):
        B.conef_cs_step(model.ctx, gsets[t % n_sets], buf["table"], buf["Q"], buf["P"], buf["Q"], buf["ws"], st)

    for t in range(warmup):
        one_step(t)
    torch.cuda.synchronize()
    B.conef_set_timing(model.ctx, True)
    t0 = time.perf_counter()
    for t in range(warmup, warmup + steps):
        one_step(t)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    stage_ms = dict(zip(STAGES, B.conef_get_timing(model.ctx)))
    finite = bool(torch.isfinite(buf["P"]).all()) and bool(torch.isfinite(buf["table"].float()).all())
    model.close()
    del buf, gsets
    torch.cuda.empty_cache()
    nbytes = sketch_bytes(w, keep)
    return {"ms_per_step": round(ms, 4), "grad_GB/s": round(w.grad_bytes / (ms * 1e-3) / 1e9, 2),
            "bytes_per_step": nbytes, "model_hbm_frac": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "stage_ms": {k: round(v, 4) for k, v in stage_ms.items()}, "finite": finite}


def run_random_block(w, fraction: float = 0.1, reps: int = 10):
    """Times one step with the unscaled random-block gradient compressor (Section 5.3: a tenth of the coordinates
    kept) in place of the rank-r one: with the workload's quantiser (beta = 0) and with the count sketch (fp16
    table, keep 0.2, beta 0.9).  One streaming pass each; HIP events on the launch stream."""
    import torch

    from paper_2312_08538_amd import binding as B
    from paper_2312_08538_amd import workloads as wl

    keep = wl.random_block_keep(w.layout, fraction)
    G = 4 if w.grad_dtype == 0 else 2
    out = {}
    for kind in ("quantiser", "count_sketch"):
        if kind == "quantiser":
            model = B.Model(w.layout, w.rank, w.bits, w.block, w.grad_dtype, w.lib_seed)
            state_bytes = sum(n * m * (w.bits / 8 + 4.0 / w.block) for n, m in w.layout)
        else:
            ws = wl.sketch_rows(w.layout, 0.2)
            model = B.SketchModel(w.layout, ws, w.rank, 0.9, B.TABLE_F16, w.grad_dtype, w.lib_seed)
            state_bytes = sum(a * m * 2 for a, (_, m) in zip(ws, w.layout))
        B.conef_rb_configure(model.ctx, keep)
        buf = model.alloc("cuda:0")
        delta = torch.zeros(B.conef_rb_sizes(model.ctx)["delta_elems"], dtype=torch.float32, device="cuda:0")
        wl.device_fill_gradients(w, 0, buf["grads"], [o["grad_off"] for o in model.offsets])
        st = B.Model.stream_handle()

        def one(t):
            if kind == "quantiser":
                B.conef_rb_step(model.ctx, buf["grads"], buf["codes"], buf["scales"], delta, t, st)
            else:
                B.conef_cs_rb_step(model.ctx, buf["grads"], buf["table"], delta, t, st)

        for t in range(2):
            one(t)
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for t, (e0, e1) in enumerate(ev):
            e0.record()
            one(2 + t)
            e1.record()
            if kind == "count_sketch" and t % 8 == 7:
                buf["table"].zero_()        # outside the timed spans; see run_scaled_sign
        torch.cuda.synchronize()
        ms = sum(e0.elapsed_time(e1) for e0, e1 in ev) / reps
        nbytes = int(w.elements * G + 2 * state_bytes + 4 * sum(keep))      # gradient, state read + written, kept values
        out[kind] = {"ms": round(ms, 4), "bytes": nbytes, "GB/s": round(nbytes / (ms * 1e-3) / 1e9, 1),
                     "frac_of_peak": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                     "finite": bool(torch.isfinite(delta).all())}
        model.close()
        del buf, delta
        torch.cuda.empty_cache()
    return out


def run_scaled_sign(w, reps: int = 10):
    """Times one step with the scaled-sign gradient compressor (Section 5.1) in place of the rank-r one, with the
    workload's quantiser (beta = 0) and with the count sketch (fp16 table, keep 0.2, beta 0.9): two passes over
    the gradient and the error state.  HIP events on the launch stream."""
    import torch

    from paper_2312_08538_amd import binding as B
    from paper_2312_08538_amd import workloads as wl

    G = 4 if w.grad_dtype == 0 else 2
    out = {}
    for kind in ("quantiser", "count_sketch"):
        if kind == "quantiser":
            model = B.Model(w.layout, w.rank, w.bits, w.block, w.grad_dtype, w.lib_seed)
            state_bytes = sum(n * m * (w.bits / 8 + 4.0 / w.block) for n, m in w.layout)
        else:
            ws = wl.sketch_rows(w.layout, 0.2)
            model = B.SketchModel(w.layout, ws, w.rank, 0.9, B.TABLE_F16, w.grad_dtype, w.lib_seed)
            state_bytes = sum(a * m * 2 for a, (_, m) in zip(ws, w.layout))
        buf = model.alloc("cuda:0")
        signs = torch.zeros(B.conef_ss_sizes(model.ctx)["sign_words"], dtype=torch.int32, device="cuda:0")
        cs = torch.zeros(len(w.layout), dtype=torch.float32, device="cuda:0")
        wl.device_fill_gradients(w, 0, buf["grads"], [o["grad_off"] for o in model.offsets])
        st = B.Model.stream_handle()

        def one(t):
            if kind == "quantiser":
                B.conef_ss_step(model.ctx, buf["grads"], buf["codes"], buf["scales"], signs, cs, buf["ws"], t, st)
            else:
                B.conef_cs_ss_step(model.ctx, buf["grads"], buf["table"], signs, cs, buf["ws"], st)

        for t in range(2):
            one(t)
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for t, (e0, e1) in enumerate(ev):
            e0.record()
            one(2 + t)
            e1.record()
            if kind == "count_sketch" and t % 8 == 7:
                # With one hash per row, bucket b of the table feeds back into itself with the factor
                # beta + (1 - beta) |b| per step (|b| rows share it: 5 on average here, so 1.4); only the gradient
                # compressor's Delta holds against that.  The rank-r Delta does; an element-wise one on the SAME
                # gradient step after step does not, and the fp16 table overflows after some twenty steps.  The
                # kernels' work does not depend on the values: start again from an empty table, outside the timed spans.
                buf["table"].zero_()
        torch.cuda.synchronize()
        ms = sum(e0.elapsed_time(e1) for e0, e1 in ev) / reps
        # gradient and state read twice, state written once, one sign bit per entry written
        nbytes = int(2 * w.elements * G + 3 * state_bytes + w.elements / 8)
        out[kind] = {"ms": round(ms, 4), "bytes": nbytes, "GB/s": round(nbytes / (ms * 1e-3) / 1e9, 1),
                     "frac_of_peak": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                     "finite": bool(torch.isfinite(cs).all())}
        model.close()
        del buf, signs
        torch.cuda.empty_cache()
    return out


def run_random_k(w, group: int = 10, reps: int = 10, uniform: bool = False):
    """Times one step with the random-k gradient compressor (stratified: one coordinate kept of every `group`
    consecutive ones; uniform: a uniformly drawn subset of the same size, one evaluation of a keyed permutation per
    coordinate) in place of the rank-r one: with the workload's quantiser (beta = 0), with the count sketch (fp16
    table, keep 0.2, beta 0.9), with iConEF-v1 (the quantiser twice) and with iConEF-v2 (first error vector: a random block
    of 5 % of every matrix kept in fp32, as large as the appendix experiment's; second: the quantiser).  One streaming pass
    each; HIP events on the launch stream."""
    import torch

    from paper_2312_08538_amd import binding as B
    from paper_2312_08538_amd import workloads as wl

    G = 4 if w.grad_dtype == 0 else 2
    kept = sum(-(-(n * m) // group) for n, m in w.layout)
    out = {}
    for kind in ("quantiser", "count_sketch", "iconef_v1", "iconef_v2"):
        if kind == "count_sketch":
            ws = wl.sketch_rows(w.layout, 0.2)
            model = B.SketchModel(w.layout, ws, w.rank, 0.9, B.TABLE_F16, w.grad_dtype, w.lib_seed)
            state_bytes = sum(a * m * 2 for a, (_, m) in zip(ws, w.layout))
        else:
            model = B.Model(w.layout, w.rank, w.bits, w.block, w.grad_dtype, w.lib_seed)
            state_bytes = sum(n * m * (w.bits / 8 + 4.0 / w.block) for n, m in w.layout) * (2 if kind == "iconef_v1" else 1)
        if uniform:
            B.conef_rk_configure_uniform(model.ctx, [-(-(n * m) // group) for n, m in w.layout])
        else:
            B.conef_rk_configure(model.ctx, [group] * len(w.layout))
        buf = model.alloc("cuda:0")
        delta = torch.zeros(B.conef_rk_sizes(model.ctx)["delta_elems"], dtype=torch.float32, device="cuda:0")
        if kind == "iconef_v1":
            codes2, scales2 = torch.zeros_like(buf["codes"]), torch.zeros_like(buf["scales"])
        if kind == "iconef_v2":
            keep_e = [max(1, (n * m) // 20) for n, m in w.layout]
            B.conef_i2_configure(model.ctx, keep_e)
            e_bufs = [torch.zeros(B.conef_i2_sizes(model.ctx)["e_elems"], dtype=torch.float32, device="cuda:0") for _ in range(2)]
            state_bytes += 4 * sum(keep_e)
        wl.device_fill_gradients(w, 0, buf["grads"], [o["grad_off"] for o in model.offsets])
        st = B.Model.stream_handle()

        def one(t):
            if kind == "quantiser":
                B.conef_rk_step(model.ctx, buf["grads"], buf["codes"], buf["scales"], delta, t, st)
            elif kind == "count_sketch":
                B.conef_cs_rk_step(model.ctx, buf["grads"], buf["table"], delta, t, st)
            elif kind == "iconef_v1":
                B.conef_i_rk_step(model.ctx, buf["grads"], buf["codes"], buf["scales"], codes2, scales2, delta, t, st)
            else:
                B.conef_i2_rk_step(model.ctx, buf["grads"], e_bufs[t % 2], e_bufs[(t + 1) % 2], buf["codes"], buf["scales"],
                                   delta, t, st)

        for t in range(2):
            one(t)
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for t, (e0, e1) in enumerate(ev):
            e0.record()
            one(2 + t)
            e1.record()
            if kind == "count_sketch" and t % 8 == 7:
                buf["table"].zero_()        # outside the timed spans; see run_scaled_sign
        torch.cuda.synchronize()
        ms = sum(e0.elapsed_time(e1) for e0, e1 in ev) / reps
        nbytes = int(w.elements * G + 2 * state_bytes + 4 * kept)       # gradient, state read + written, kept values
        out[kind] = {"ms": round(ms, 4), "bytes": nbytes, "GB/s": round(nbytes / (ms * 1e-3) / 1e9, 1),
                     "frac_of_peak": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                     "finite": bool(torch.isfinite(delta).all())}
        model.close()
        del buf, delta
        if kind == "iconef_v1":
            del codes2, scales2
        if kind == "iconef_v2":
            del e_bufs
        torch.cuda.empty_cache()
    return out


def run_iconef(w, fraction: float = 0.1, reps: int = 10):
    """Times one step of improved contractive error feedback, version 1 (Algorithm 3: two compressed error vectors, the
    workload's quantiser twice) with the random-block (a tenth kept) and the scaled-sign gradient compressors.  HIP
    events on the launch stream."""
    import torch

    from paper_2312_08538_amd import binding as B
    from paper_2312_08538_amd import workloads as wl

    keep = wl.random_block_keep(w.layout, fraction)
    G = 4 if w.grad_dtype == 0 else 2
    state_bytes = sum(n * m * (w.bits / 8 + 4.0 / w.block) for n, m in w.layout)      # one of the two vectors
    model = B.Model(w.layout, w.rank, w.bits, w.block, w.grad_dtype, w.lib_seed)
    B.conef_rb_configure(model.ctx, keep)
    buf = model.alloc("cuda:0")
    codes2, scales2 = torch.zeros_like(buf["codes"]), torch.zeros_like(buf["scales"])
    delta = torch.zeros(B.conef_rb_sizes(model.ctx)["delta_elems"], dtype=torch.float32, device="cuda:0")
    signs = torch.zeros(B.conef_ss_sizes(model.ctx)["sign_words"], dtype=torch.int32, device="cuda:0")
    cs = torch.zeros(len(w.layout), dtype=torch.float32, device="cuda:0")
    wl.device_fill_gradients(w, 0, buf["grads"], [o["grad_off"] for o in model.offsets])
    st = B.Model.stream_handle()
    out = {}
    for kind in ("random_block", "scaled_sign"):
        def one(t):
            if kind == "random_block":
                B.conef_i_rb_step(model.ctx, buf["grads"], buf["codes"], buf["scales"], codes2, scales2, delta, t, st)
            else:
                B.conef_i_ss_step(model.ctx, buf["grads"], buf["codes"], buf["scales"], codes2, scales2, signs, cs,
                                  buf["ws"], t, st)

        for t in range(2):
            one(t)
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for t, (e0, e1) in enumerate(ev):
            e0.record()
            one(2 + t)
            e1.record()
        torch.cuda.synchronize()
        ms = sum(e0.elapsed_time(e1) for e0, e1 in ev) / reps
        if kind == "random_block":      # gradient, both vectors read and written, kept values
            nbytes = int(w.elements * G + 4 * state_bytes + 4 * sum(keep))
        else:                           # gradient and both vectors read twice, both written once, one sign bit per entry
            nbytes = int(2 * w.elements * G + 6 * state_bytes + w.elements / 8)
        out[kind] = {"ms": round(ms, 4), "bytes": nbytes, "GB/s": round(nbytes / (ms * 1e-3) / 1e9, 1),
                     "frac_of_peak": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                     "finite": bool(torch.isfinite(delta).all() and torch.isfinite(cs).all()
                                    and torch.isfinite(scales2).all())}
    model.close()
    del buf, codes2, scales2, delta, signs
    torch.cuda.empty_cache()
    return out


def run_iconef_lowrank(w, reps: int = 10):
    """Times one iConEF-v1 step around the rank-r compressor (the three passes of the plain step, each decoding both
    error vectors, and the second rounding in the err pass)."""
    import torch

    from paper_2312_08538_amd import binding as B
    from paper_2312_08538_amd import workloads as wl

    G = 4 if w.grad_dtype == 0 else 2
    model = B.Model(w.layout, w.rank, w.bits, w.block, w.grad_dtype, w.lib_seed)
    buf = model.alloc("cuda:0")
    codes2, scales2 = torch.zeros_like(buf["codes"]), torch.zeros_like(buf["scales"])
    wl.device_q0(w, buf["Q"], [o["q_off"] for o in model.offsets])
    wl.device_fill_gradients(w, 0, buf["grads"], [o["grad_off"] for o in model.offsets])
    st = B.Model.stream_handle()

    def one(t):
        B.conef_i_step(model.ctx, buf["grads"], buf["codes"], buf["scales"], codes2, scales2, buf["Q"], buf["P"], buf["Q"],
                       buf["ws"], t, st)

    for t in range(2):
        one(t)
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for t, (e0, e1) in enumerate(ev):
        e0.record()
        one(2 + t)
        e1.record()
    torch.cuda.synchronize()
    ms = sum(e0.elapsed_time(e1) for e0, e1 in ev) / reps
    state = sum(n * m * (w.bits / 8 + 4.0 / w.block) for n, m in w.layout)          # one of the two vectors
    nbytes = int(w.elements * G * 3 + state * 8)        # three passes read the gradient and both vectors; the last writes both
    out = {"ms_per_step": round(ms, 4), "bytes": nbytes, "model_hbm_frac": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
           "finite": bool(torch.isfinite(buf["Q"]).all() and torch.isfinite(scales2).all())}
    model.close()
    del buf, codes2, scales2
    torch.cuda.empty_cache()
    return out


def run_oracle_sample(w, budget_s: float = 20.0):
    """Times the oracle (as it stands) on the workload's matrices in layout order, one step from
    zero error, until about `budget_s` seconds of CPU work are spent or the whole model is done.
    To bound host-side generation, one gradient is drawn per distinct matrix shape and shared by
    the matrices of that shape (every matrix still has its own state, Q and random draws)."""
    from oracle import conef_ref as R
    from paper_2312_08538_amd import workloads as wl

    R.lib()
    by_shape = {}
    spent, tot, used = 0.0, 0, 0
    for l, (n, m) in enumerate(w.layout):
        if (n, m) not in by_shape:
            by_shape[(n, m)] = wl.host_gradient(w, 0, l)
        stt = R.MatState.fresh(n, m, w.bits, w.block, wl.host_q0(w, l))
        t0 = time.perf_counter()
        R.step_matrix(by_shape[(n, m)], stt, w.rank, w.bits, w.block, w.lib_seed, l, 0)
        spent += time.perf_counter() - t0
        tot += n * m
        used += 1
        if spent >= budget_s:
            break
    G = 4 if w.grad_dtype == 0 else 2
    sample = (f"the first {used} of {len(w.layout)} matrices of the workload in layout order ({tot} elements, "
              f"{100.0 * tot / w.elements:.1f} % of it), one step from zero error, {spent:.1f} s of oracle time")
    return tot * G / spent / 1e9, R.num_threads(), sample


def calibrate_copy(w):
    """One launch of the library's plain decode kernel over the workload's (zero) state: it reads
    every code word and scale once and writes one fp32 value per element, nothing else, so the
    byte counters of this launch give the scale of FETCH_SIZE / WRITE_SIZE."""
    import torch

    from paper_2312_08538_amd import binding as B

    model = B.Model(w.layout, w.rank, w.bits, w.block, w.grad_dtype, w.lib_seed)
    codes = torch.zeros(model.sizes["code_words"], dtype=torch.int32, device="cuda:0")
    scales = torch.zeros(model.sizes["n_scales"], dtype=torch.float32, device="cuda:0")
    e = torch.zeros(model.sizes["grad_elems"], dtype=torch.float32, device="cuda:0")   # also evicts the state from the caches
    torch.cuda.synchronize()
    B.conef_decode_error(model.ctx, codes, scales, e, model.stream_handle())
    torch.cuda.synchronize()
    rd = 4 * (sum(-(-n * m // (32 // w.bits)) for n, m in w.layout) + sum(-(-n * m // w.block) for n, m in w.layout))
    print(f"calibration launch k_decode: reads {rd} bytes, writes {4 * w.elements} bytes", file=sys.stderr)
    model.close()
    # and a plain device-to-device copy of 1 GiB (the runtime's copy kernel), src not cache resident
    src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")
    dst = torch.empty_like(src)
    e.zero_()
    torch.cuda.synchronize()
    dst.copy_(src)
    torch.cuda.synchronize()
    print(f"calibration copy (runtime copy kernel): reads {src.numel() * 4} bytes, writes {src.numel() * 4} bytes",
          file=sys.stderr)


MFMA_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 matrix-core peak, published


def kernels_digest(w) -> str:
    """Digest of the sources that the pass kernels of this workload's kernel family and their launch tables are built from:
    counter values measured on other sources are not this build's (profiles/hbm_traffic.json records the digest of the
    run it was measured on)."""
    if w.rank == 32 and w.grad_dtype == 1 and w.bits == 4 and w.block == 128:
        family = ("kernels_mfma.hip", "mfma_common.h")
    elif w.rank in (2, 4, 8) and w.grad_dtype == 1 and w.bits in (2, 4) and w.block >= 128:
        family = ("kernels_octet.hip", "kernels_pack.hip", "mfma_common.h")        # packed-split P and Q+, the octet family's err pass
    elif w.rank in (2, 4, 8):
        family = ("kernels_octet.hip",)
    else:
        family = ("kernels_generic.hip",)
    d = os.path.join(ROOT, "paper_2312_08538_amd", "csrc")
    h = hashlib.sha256()
    for name in (*family, "device_common.h", "kernels.h", "plan.h", "plan.cpp"):
        h.update(name.encode())
        h.update(open(os.path.join(d, name), "rb").read())
    return h.hexdigest()[:16]


def load_counters(w, stage: str):
    """What the committed rocprofv3 --pmc summaries hold for the dominant kernel of this workload
    (profiles/hbm_traffic.json: HBM bytes per launch, matrix-core busy fraction), if they were measured on the kernel
    sources of this build; else None, with the reason."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if not os.path.exists(path):
        return None, "no counter summary committed"
    try:
        rec = json.load(open(path)).get(w.name)
    except Exception:
        return None, "counter summary unreadable"
    if not rec or rec.get("stage") != stage:
        return None, "no counter summary for this workload's dominant kernel"
    if rec.get("kernels_digest") != kernels_digest(w):
        return None, f"counter summary measured on other kernel sources ({rec.get('kernels_digest')})"
    return rec, None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="large")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the short runs of the other workloads")
    ap.add_argument("--columns", action="store_true", help="with --count-sketch: the column form of the sketch")
    ap.add_argument("--count-sketch", action="store_true",
                    help="time only the step with the count sketch as the error compressor (fp16 table, keep 0.2, "
                         "beta 0.9) on --workload and print its line; for profiling that mode on its own")
    ap.add_argument("--random-block", action="store_true",
                    help="time only the step with the random-block gradient compressor (a tenth of the coordinates "
                         "kept; quantiser and count-sketch error compressors) on --workload and print its line")
    ap.add_argument("--scaled-sign", action="store_true",
                    help="time only the step with the scaled-sign gradient compressor (quantiser and count-sketch error "
                         "compressors) on --workload and print its line")
    ap.add_argument("--random-k", action="store_true",
                    help="time only the step with the random-k gradient compressor (stratified, one coordinate of every "
                         "ten kept; quantiser, count sketch, iConEF-v1 and iConEF-v2) on --workload and print its line")
    ap.add_argument("--uniform", action="store_true",
                    help="with --random-k: the uniformly drawn subset of a tenth of every matrix instead of the strata")
    ap.add_argument("--iconef", action="store_true",
                    help="time only the iConEF-v1 step (two compressed error vectors, the quantiser twice) with the "
                         "random-block and scaled-sign gradient compressors on --workload and print its line")
    ap.add_argument("--iconef-rank-r", action="store_true",
                    help="time only the iConEF-v1 step around the rank-r compressor on --workload and print its line")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain streaming kernel of known size (k_decode: reads the codes and "
                         "scales, writes 4 bytes per element) for scaling rocprofv3 byte counters")
    a = ap.parse_args()
    if a.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is one worker's share of the method on ONE GPU; it has no collectives "
              "and no sharding, so --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    if a.steps < 1 or a.steps > 64:
        print("bench.py: --steps must be in 1..64 (one event set per timed step is kept)", file=sys.stderr)
        sys.exit(2)

    from paper_2312_08538_amd import workloads as wl

    w = wl.WORKLOADS[a.workload]
    if a.calibrate_copy:
        calibrate_copy(w)
    if a.scaled_sign:
        r = run_scaled_sign(w, a.steps)
        print(json.dumps({"metric": "scaled-sign ConEF step throughput: gradient GB/s processed",
                          "value": round(w.grad_bytes / (r["quantiser"]["ms"] * 1e-3) / 1e9, 2), "unit": "GB/s", "n_gpus": 1,
                          "steps": a.steps, "config": {"workload": w.name}, **r}), flush=True)
        return
    if a.iconef_rank_r:
        r = run_iconef_lowrank(w, a.steps)
        print(json.dumps({"metric": "iConEF-v1 rank-r step throughput: gradient GB/s processed",
                          "value": round(w.grad_bytes / (r["ms_per_step"] * 1e-3) / 1e9, 2), "unit": "GB/s", "n_gpus": 1,
                          "steps": a.steps, "config": {"workload": w.name, "rank": w.rank}, **r}), flush=True)
        return
    if a.random_k:
        r = run_random_k(w, 10, a.steps, a.uniform)
        print(json.dumps({"metric": ("uniform-subset" if a.uniform else "stratified") + " random-k ConEF step throughput: gradient GB/s processed",
                          "value": round(w.grad_bytes / (r["quantiser"]["ms"] * 1e-3) / 1e9, 2), "unit": "GB/s", "n_gpus": 1,
                          "steps": a.steps, "config": {"workload": w.name, "group": 10}, **r}), flush=True)
        return
    if a.iconef:
        r = run_iconef(w, 0.1, a.steps)
        print(json.dumps({"metric": "iConEF-v1 step throughput (random block): gradient GB/s processed",
                          "value": round(w.grad_bytes / (r["random_block"]["ms"] * 1e-3) / 1e9, 2), "unit": "GB/s", "n_gpus": 1,
                          "steps": a.steps, "config": {"workload": w.name, "fraction": 0.1}, **r}), flush=True)
        return
    if a.random_block:
        r = run_random_block(w, 0.1, a.steps)
        print(json.dumps({"metric": "random-block ConEF step throughput: gradient GB/s processed",
                          "value": round(w.grad_bytes / (r["quantiser"]["ms"] * 1e-3) / 1e9, 2), "unit": "GB/s", "n_gpus": 1,
                          "steps": a.steps, "config": {"workload": w.name, "fraction": 0.1}, **r}), flush=True)
        return
    if a.count_sketch:
        r = run_sketch(w, 0.2, 0.9, a.steps, a.warmup, columns=a.columns)
        print(json.dumps({"metric": "ConEF-CS step throughput: gradient GB/s processed", "value": r["grad_GB/s"],
                          "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
                          "config": {"workload": w.name, "rank": w.rank, "keep": 0.2, "beta": 0.9, "table": "f16",
                                     "form": "column" if a.columns else "row"},
                          **r}), flush=True)
        return
    ms, stage_ms, finite, stats = run_gpu(w, a.steps, a.warmup)
    if not finite:
        print("bench.py: non-finite factors after the timed run", file=sys.stderr)
        sys.exit(1)
    value = w.grad_bytes / (ms * 1e-3) / 1e9
    dom = max(("p", "q", "err"), key=lambda s: stage_ms[s])
    dom_bytes = stage_bytes(w, dom)
    achieved = dom_bytes / (stage_ms[dom] * 1e-3) / 1e9
    counters, why_not = load_counters(w, dom)
    out = {
        "metric": "ConEF step throughput: gradient GB/s processed",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(ms, 4), "step_ms": stats, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if w.grad_dtype == 0 else "bf16->f32",
        "data": "synthetic",
        "config": {"workload": w.name, "matrices": len(w.layout), "elements": w.elements,
                   "grad_dtype": "f32" if w.grad_dtype == 0 else "bf16", "rank": w.rank, "bits": w.bits,
                   "block": w.block, "dist": w.dist},
        "model_hbm": {"bytes_per_step": w.model_bytes(),
                      "GB/s": round(w.model_bytes() / (ms * 1e-3) / 1e9, 1),
                      "frac_of_peak": round(w.model_bytes() / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
        "stage_ms": {k: round(v, 4) for k, v in stage_ms.items()},
        "roofline": {"kernel": KERNEL_OF_STAGE[dom], "bound": "hbm", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "bytes_per_launch": int(dom_bytes), "ms_per_launch": round(stage_ms[dom], 4),
                     "traffic": counters["bytes"] if counters else None},
        "kernels_digest": kernels_digest(w),
    }
    if counters:
        out["roofline"]["traffic_source"] = {"kernel": counters["kernel"], "kernels_digest": counters["kernels_digest"]}
    else:
        out["roofline"]["traffic_note"] = why_not
    if w.rank == 32 and w.grad_dtype == 1 and w.bits == 4 and w.block == 128:
        # the bf16 matrix-core kernels: every pass multiplies three bf16 splits of a factor with the gradient and with the
        # codes, 6 products of 2 * 32 flops per element
        flops = 384.0 * w.elements
        tf = flops / (stage_ms[dom] * 1e-3) / 1e12
        out["roofline"]["mfma"] = {"flops_per_launch": int(flops), "achieved": round(tf, 1), "peak": MFMA_PEAK_TFLOPS,
                                   "unit": "TFLOP/s", "frac": round(tf / MFMA_PEAK_TFLOPS, 4),
                                   "busy_frac": counters.get("mfma_busy_frac") if counters else None}
    if not a.no_extra:
        out["apply_update"] = run_update(w)
        extra = {}
        for name in ("cnn", "lm", "translation", "large"):
            if name == w.name:
                continue
            ww = wl.WORKLOADS[name]
            ms2, st2, _, stats2 = run_gpu(ww, 10, 3)
            extra[name] = {"ms_per_step": round(ms2, 4), "grad_GB/s": round(ww.grad_bytes / (ms2 * 1e-3) / 1e9, 2),
                           "model_hbm_frac": round(ww.model_bytes() / (ms2 * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                           "step_ms": stats2, "stage_ms": {k: round(v, 4) for k, v in st2.items()}}
        out["other_workloads"] = extra
        # the count sketch as the error compressor (fp16 table with a fifth of the rows: 90 % of an fp32 error
        # vector saved, beta = 0.9, the setting of Section 5.2), beside the step, not inside `value`
        out["count_sketch"] = {"keep": 0.2, "beta": 0.9, "table": "f16",
                               "column_form": {name: run_sketch(wl.WORKLOADS[name], 0.2, 0.9, columns=True)
                                               for name in ("cnn", "lm")},
                               "workloads": {name: run_sketch(wl.WORKLOADS[name], 0.2, 0.9)
                                             for name in ("cnn", "lm", "translation", "large")}}
        # the unscaled random-block gradient compressor in place of the rank-r one (a tenth of the coordinates kept)
        out["random_block"] = {"fraction": 0.1, "workloads": {name: run_random_block(wl.WORKLOADS[name])
                                                              for name in ("cnn", "lm", "translation", "large")}}
        out["scaled_sign"] = {"workloads": {name: run_scaled_sign(wl.WORKLOADS[name])
                                            for name in ("cnn", "lm", "translation", "large")}}
        out["random_k"] = {"group": 10, "workloads": {name: run_random_k(wl.WORKLOADS[name])
                                                      for name in ("cnn", "lm", "translation", "large")}}
        # ... as a uniformly drawn subset of the same size (a keyed permutation evaluated for every coordinate)
        out["random_k_uniform"] = {"fraction": 0.1, "workloads": {name: run_random_k(wl.WORKLOADS[name], uniform=True)
                                                                  for name in ("lm", "large")}}
        # improved contractive error feedback, version 1: a second compressed vector, the quantiser twice
        out["iconef_v1"] = {"fraction": 0.1, "workloads": {name: run_iconef(wl.WORKLOADS[name])
                                                           for name in ("cnn", "lm", "translation", "large")}}
        # ... and around the rank-r compressor
        out["iconef_v1_rank_r"] = {"workloads": {name: run_iconef_lowrank(wl.WORKLOADS[name])
                                                 for name in ("cnn", "lm", "translation", "large")}}
    if not a.no_cpu_baseline:
        v, cores, sample = run_oracle_sample(w)
        out["cpu_baseline"] = {"value": round(v, 4), "unit": "GB/s", "cores": cores, "kind": "oracle",
                               "sample": sample}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
