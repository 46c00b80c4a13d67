"""GPU parity tests of the packed-split P and Q+ passes (ranks 2, 4, 8 with bf16 gradients, 2- or 4-bit codes, blocks of
128 to 512: three exact bf16 splits of a factor row side by side in one matrix-core operand): the library, called
through the C ABI, against the oracle on the same seeded inputs.  The factors carry fp32 sums (one scale block or 64 rows
at a time, fp64 beyond), so the comparison is the one of the rank-32 matrix-core family: P^ and Q+ within the stated
tolerance, scales within 1e-6, codes bit for bit except within the boundary rule's window, every step from the oracle's
state (see test_gpu_parity._run_model)."""
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
    return R, B, U


SHAPES = [
    # one block of columns (a pair without a second block), a row tail; an odd number of column blocks and a code line
    # that ends early; several row tiles of the Q+ pass (partial sums) with a tail; whole lines of 2-bit codes
    # (columns for blocks of 512; halved for 256, quartered for 128)
    (300, 512), (77, 1536), (1100, 1024), (130, 2048), (16, 512), (520, 3 * 512),
]


def _layout(block):
    out = []
    for n, m in SHAPES:
        m = m if block == 512 else m // 4 if block == 128 else m // 2
        if m % block == 0 and m % 64 == 0:
            out.append((n, m))
    return out


@pytest.mark.parametrize("rank,bits,block", [(8, 2, 256), (8, 4, 128), (4, 2, 128), (4, 4, 256), (2, 2, 512), (8, 4, 512), (2, 4, 128)])
@pytest.mark.parametrize("beta", [0.0, 0.5])
def test_packed_split_passes_against_the_oracle(env, rank, bits, block, beta):
    import test_gpu_parity as T

    R, B, U = env
    layout = _layout(block)
    w = wl.Workload("pack", 11, tuple(layout), rank, bits, block, wl.BF16, "normal", 1.0, 0x9AC4ED + rank + bits)
    probe = B.Model(layout, rank, bits, block, wl.BF16, 1)
    fam = [B.conef_matrix_family(probe.ctx, l) for l in range(len(layout))]
    B.conef_check_plan(probe.ctx)
    probe.close()
    assert fam == [B.FAMILY_PACKED] * len(layout), (fam, layout)
    T._run_model((R, B, U), w, layout, 3, f"pack-r{rank}-b{bits}-B{block}-beta{beta}", beta=beta)


def test_factors_agree_with_the_oracle_to_fp32_sums(env):
    """P^ and Q+ of the first step (no error state) and of a step from the oracle's state: relative error against the
    oracle's fp64 factors well inside 1e-5 (the family's own figure; the stated tolerance is 2e-2 for bf16 gradients)."""
    R, B, U = env
    layout = [(1100, 1024), (300, 2048)]
    w = wl.Workload("pack", 12, tuple(layout), 8, 2, 256, wl.BF16, "normal", 1e-3, 0x51DE)
    Q0s = [wl.host_q0(w, l, shape=layout[l]) for l in range(len(layout))]
    gpu = U.GpuModel(layout, w.rank, w.bits, w.block, w.grad_dtype, w.lib_seed, Q0s)
    ora = U.OracleModel(layout, w.rank, w.bits, w.block, w.lib_seed, Q0s)
    for t in range(3):
        grads = [wl.host_gradient(w, t, l, shape=layout[l]) for l in range(len(layout))]
        gpu.set_grads(grads)
        for l, st in enumerate(ora.states):
            gpu.set_state(l, st.codes, st.scales)
            gpu.set_Q(l, st.Q)
        print(f"[pack factors] step {t}: launching", flush=True)
        gpu.step(t)
        out = ora.step(grads, t)
        for l, (Ph, Qn, _) in enumerate(out):
            eP, eQ = U.rel_err(gpu.mat_P(l), Ph), U.rel_err(gpu.mat_Q(l), Qn)
            print(f"  mat {l} step {t}: P^ {eP:.2e} Q+ {eQ:.2e}", flush=True)
            assert eP <= 1e-5 and eQ <= 1e-5, (l, t, eP, eQ)


def test_the_octet_passes_still_serve_these_matrices_when_asked(env, monkeypatch):
    """CONEF_PACK=0 before conef_init keeps the octet family's own P and Q+ passes (fp64 sums): three free-running steps
    agree with the oracle bit for bit, nothing excused."""
    import test_gpu_parity as T

    R, B, U = env
    monkeypatch.setenv("CONEF_PACK", "0")
    layout = _layout(256)
    w = wl.Workload("nopack", 13, tuple(layout), 8, 2, 256, wl.BF16, "normal", 1.0, 0x0C7E7)
    probe = B.Model(layout, 8, 2, 256, wl.BF16, 1)
    assert [B.conef_matrix_family(probe.ctx, l) for l in range(len(layout))] == [B.FAMILY_OCTET] * len(layout)
    probe.close()
    assert T._run_model((R, B, U), w, layout, 3, "octet passes, CONEF_PACK=0") == 0
