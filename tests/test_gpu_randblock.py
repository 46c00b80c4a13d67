"""GPU parity tests of the random-block gradient compressor (Section 5.3) with either error compressor: the
library, called through the C ABI, against oracle/randblock_ref.c on the same seeded inputs, free-running over
several steps.  Every operation is element-wise fp32 arithmetic in a fixed order, so the kept values, the codes
and scales (quantiser) and the table (count sketch) are compared bit for bit."""
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


QUANTISER_CASES = [
    # (layout, rank (unused by this path), bits, block, fraction)
    ([(64, 128), (40, 512), (256, 96)], 4, 4, 128, 0.1),          # whole power-of-two blocks: the wave-per-run kernel
    ([(64, 147), (37, 53), (128, 576)], 4, 4, 128, 0.1),          # odd sizes: the kernel for any layout
    ([(32, 512), (100, 1024)], 8, 2, 256, 0.25),
    ([(96, 160), (33, 129)], 2, 8, 8, 0.5),
    ([(16, 64), (8, 8)], 2, 4, 200, 1.0),                          # the whole matrix is kept
    ([(300, 256), (160, 384)], 32, 4, 128, 0.001),                 # a block of a few coordinates
    ([(77, 768), (5, 128), (129, 64)], 4, 4, 128, 0.1),            # whole blocks, short last runs of 512
]


@pytest.mark.parametrize("case", range(len(QUANTISER_CASES)))
@pytest.mark.parametrize("gdt", [wl.F32, wl.BF16])
@pytest.mark.parametrize("beta", [0.0, 0.75])
def test_random_block_with_the_quantiser_is_bit_exact(env, case, gdt, beta):
    R, B, U, S, torch = env
    layout, rank, bits, block, frac = QUANTISER_CASES[case]
    seed = 500 + case
    keep = wl.random_block_keep(layout, frac)
    model = B.Model(layout, rank, bits, block, gdt, seed)
    B.conef_set_beta(model.ctx, beta)
    B.conef_rb_configure(model.ctx, keep)
    buf = model.alloc()
    delta = torch.zeros(B.conef_rb_sizes(model.ctx)["delta_elems"], dtype=torch.float32, device="cuda:0")
    rng = np.random.default_rng([case, gdt])
    states = [(np.zeros(R.n_words(n * m, bits), np.uint32), np.zeros(R.n_blocks(n * m, block), np.float32)) for n, m in layout]
    for t in range(4):
        grads = [S._grad(rng, n, m, gdt) for n, m in layout]
        S._to_dev_grads(torch, model, buf, grads)
        delta.fill_(float("nan"))
        print(f"[random block quantiser case {case} gdt {gdt} beta {beta}] step {t}: launching", flush=True)
        B.conef_rb_step(model.ctx, buf["grads"], buf["codes"], buf["scales"], delta, t, model.stream_handle())
        torch.cuda.synchronize()
        for l, (n, m) in enumerate(layout):
            codes, scales = states[l]
            want = R.rb_step_matrix(grads[l], codes, scales, keep[l], bits, block, beta, seed, l, t)
            assert B.conef_rb_start(model.ctx, l, t) == R.rb_start(seed, l, t, n * m, keep[l])
            o = model.offsets[l]
            ro = B.conef_rb_offsets(model.ctx, l)
            assert ro["keep"] == keep[l]
            got = delta[ro["delta_off"]:ro["delta_off"] + keep[l]].cpu().numpy()
            tag = f"case {case} mat {l} step {t}"
            assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), f"{tag}: kept values"
            gc = buf["codes"][o["word_off"]:o["word_off"] + codes.size].cpu().numpy().view(np.uint32)
            gs = buf["scales"][o["scale_off"]:o["scale_off"] + scales.size].cpu().numpy()
            assert np.array_equal(gs.view(np.uint32), scales.view(np.uint32)), f"{tag}: scales"
            assert np.array_equal(gc, codes), f"{tag}: codes"
    model.close()


SKETCH_CASES = [
    # (layout, sketch rows, fraction)
    ([(37, 11), (64, 8), (300, 256)], [5, 64, 60], 0.1),
    ([(64, 147), (128, 576), (20, 33)], [13, 26, 1], 0.1),
    ([(1000, 1160), (64, 4608)], [200, 51], 0.25),
    ([(48, 96)], [48], 1.0),
]


@pytest.mark.parametrize("case", range(len(SKETCH_CASES)))
@pytest.mark.parametrize("gdt,fp16", [(wl.F32, False), (wl.F32, True), (wl.BF16, True)])
@pytest.mark.parametrize("beta", [0.0, 0.9])
def test_random_block_with_the_count_sketch_is_bit_exact(env, case, gdt, fp16, beta):
    R, B, U, S, torch = env
    layout, ws, frac = SKETCH_CASES[case]
    seed = 700 + case
    keep = wl.random_block_keep(layout, frac)
    model = B.SketchModel(layout, ws, 1, beta, int(fp16), gdt, seed)
    B.conef_rb_configure(model.ctx, keep)
    buf = model.alloc()
    delta = torch.zeros(B.conef_rb_sizes(model.ctx)["delta_elems"], dtype=torch.float32, device="cuda:0")
    rng = np.random.default_rng([3, case, gdt])
    tables = [np.zeros((w, m), np.uint16 if fp16 else np.float32) for w, (_, m) in zip(ws, layout)]
    for t in range(4):
        grads = [S._grad(rng, n, m, gdt) for n, m in layout]
        S._to_dev_grads(torch, model, buf, grads)
        delta.fill_(float("nan"))
        print(f"[random block sketch case {case} gdt {gdt} fp16 {fp16} beta {beta}] step {t}: launching", flush=True)
        B.conef_cs_rb_step(model.ctx, buf["grads"], buf["table"], delta, t, B.Model.stream_handle())
        torch.cuda.synchronize()
        for l, (n, m) in enumerate(layout):
            want = R.cs_rb_step_matrix(grads[l], tables[l], keep[l], beta, seed, l, t)
            ro = B.conef_rb_offsets(model.ctx, l)
            got = delta[ro["delta_off"]:ro["delta_off"] + keep[l]].cpu().numpy()
            tag = f"case {case} mat {l} step {t}"
            assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), f"{tag}: kept values"
            gt = S._get_table(model, buf, l)
            assert np.array_equal(gt.view(np.uint16 if fp16 else np.uint32), tables[l].view(np.uint16 if fp16 else np.uint32)), \
                f"{tag}: table differs in {(gt != tables[l]).sum()} entries"
    model.close()


def test_random_block_calls_need_configuration_and_the_right_kind_of_context(env):
    R, B, U, S, torch = env
    qm = B.Model([(64, 64)], 4, 4, 64, wl.F32, 1)
    sk = B.SketchModel([(64, 64)], [16], 4, 0.5, 0, wl.F32, 1)
    qb, sb = qm.alloc(), sk.alloc()
    d = torch.zeros(4096, dtype=torch.float32, device="cuda:0")
    for call in (lambda: B.conef_rb_step(qm.ctx, qb["grads"], qb["codes"], qb["scales"], d, 0),
                 lambda: B.conef_cs_rb_step(sk.ctx, sb["grads"], sb["table"], d, 0),
                 lambda: B.conef_rb_sizes(qm.ctx)):
        with pytest.raises(B.ConefError) as e:
            call()
        assert e.value.code == B.ESTATE
    B.conef_rb_configure(qm.ctx, [100])
    B.conef_rb_configure(sk.ctx, [100])
    with pytest.raises(B.ConefError) as e:
        B.conef_cs_rb_step(qm.ctx, qb["grads"], qb["codes"], d, 0)
    assert e.value.code == B.ESTATE
    with pytest.raises(B.ConefError) as e:
        B.conef_rb_step(sk.ctx, sb["grads"], sb["table"], sb["table"], d, 0)
    assert e.value.code == B.ESTATE
    for bad in ([0], [4097], [-1]):
        with pytest.raises(B.ConefError) as e:
            B.conef_rb_configure(qm.ctx, bad)
        assert e.value.code == B.EINVAL
    # the low-rank step still works on a context that has been configured for the random block
    qm.step(qb, 0)
    torch.cuda.synchronize()
