"""GPU parity tests of the scaled-sign gradient compressor (Section 5.1) with either error compressor: the library,
called through the C ABI, against oracle/randblock_ref.c (second part) on the same seeded inputs, free-running.
The scale c = ||p||_1 / N comes from fp64 partial sums in the library's fixed order and from a sum in index order
in the oracle: it must agree to one unit in the last place of fp32, and where it is equal (in practice always)
sign words, codes, scales and tables are compared bit for bit."""
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
    import test_gpu_sketch as S

    B.lib()
    return R, B, S, torch


def _check_scale(got, want, tag):
    assert abs(float(got) - float(want)) <= float(np.spacing(np.float32(want))), f"{tag}: scale {got} vs {want}"
    return np.float32(got) == np.float32(want)


QUANTISER_CASES = [
    ([(64, 128), (40, 512), (256, 96)], 4, 4, 128),          # whole power-of-two blocks: the wave-per-run kernel
    ([(64, 147), (37, 53), (128, 576)], 4, 4, 128),          # odd sizes: the kernel for any layout, atomic sign bits
    ([(32, 512), (100, 1024)], 8, 2, 256),
    ([(96, 160), (33, 129)], 2, 8, 8),
    ([(77, 768), (5, 128), (129, 64)], 4, 4, 128),           # short last runs
    ([(2000, 1024)], 4, 4, 128),                              # many partial sums
]


@pytest.mark.parametrize("case", range(len(QUANTISER_CASES)))
@pytest.mark.parametrize("gdt", [wl.F32, wl.BF16])
@pytest.mark.parametrize("beta", [0.0, 0.75])
def test_scaled_sign_with_the_quantiser(env, case, gdt, beta):
    R, B, S, torch = env
    layout, rank, bits, block = QUANTISER_CASES[case]
    seed = 900 + case
    model = B.Model(layout, rank, bits, block, gdt, seed)
    B.conef_set_beta(model.ctx, beta)
    buf = model.alloc()
    signs = torch.zeros(B.conef_ss_sizes(model.ctx)["sign_words"], dtype=torch.int32, device="cuda:0")
    cs = torch.zeros(len(layout), dtype=torch.float32, device="cuda:0")
    rng = np.random.default_rng([case, gdt, 5])
    states = [(np.zeros(R.n_words(n * m, bits), np.uint32), np.zeros(R.n_blocks(n * m, block), np.float32)) for n, m in layout]
    for t in range(4):
        grads = [S._grad(rng, n, m, gdt) for n, m in layout]
        S._to_dev_grads(torch, model, buf, grads)
        signs.fill_(-1)                      # whatever the buffer held must not show through
        print(f"[scaled sign quantiser case {case} gdt {gdt} beta {beta}] step {t}: launching", flush=True)
        B.conef_ss_step(model.ctx, buf["grads"], buf["codes"], buf["scales"], signs, cs, buf["ws"], t, model.stream_handle())
        torch.cuda.synchronize()
        for l, (n, m) in enumerate(layout):
            codes, scales = states[l]
            words, c = R.ss_step_matrix(grads[l], codes, scales, bits, block, beta, seed, l, t)
            tag = f"case {case} mat {l} step {t}"
            o = model.offsets[l]
            if not _check_scale(cs[l].item(), c, tag):
                # a last-bit difference of the scale changes every argument: take the library's state as the oracle's
                codes[:] = buf["codes"][o["word_off"]:o["word_off"] + codes.size].cpu().numpy().view(np.uint32)
                scales[:] = buf["scales"][o["scale_off"]:o["scale_off"] + scales.size].cpu().numpy()
                continue
            so = B.conef_ss_offsets(model.ctx, l)["sign_off"]
            N = n * m
            got = signs[so:so + words.size].cpu().numpy().view(np.uint32).copy()
            if N % 32:
                got[-1] &= np.uint32((1 << (N % 32)) - 1)          # bits beyond the last entry are not part of the result
            assert np.array_equal(got, words), f"{tag}: sign bits"
            gc = buf["codes"][o["word_off"]:o["word_off"] + codes.size].cpu().numpy().view(np.uint32)
            gs = buf["scales"][o["scale_off"]:o["scale_off"] + scales.size].cpu().numpy()
            assert np.array_equal(gs.view(np.uint32), scales.view(np.uint32)), f"{tag}: scales"
            assert np.array_equal(gc, codes), f"{tag}: codes"
    model.close()


SKETCH_CASES = [
    ([(37, 11), (64, 8), (300, 256)], [5, 64, 60]),
    ([(64, 147), (128, 576), (20, 33)], [13, 26, 1]),
    ([(1000, 1160), (64, 4608)], [200, 51]),
]


@pytest.mark.parametrize("case", range(len(SKETCH_CASES)))
@pytest.mark.parametrize("gdt,fp16", [(wl.F32, False), (wl.F32, True), (wl.BF16, True)])
@pytest.mark.parametrize("beta", [0.0, 0.9])
def test_scaled_sign_with_the_count_sketch(env, case, gdt, fp16, beta):
    R, B, S, torch = env
    layout, ws = SKETCH_CASES[case]
    seed = 950 + case
    model = B.SketchModel(layout, ws, 1, beta, int(fp16), gdt, seed)
    buf = model.alloc()
    signs = torch.zeros(B.conef_ss_sizes(model.ctx)["sign_words"], dtype=torch.int32, device="cuda:0")
    cs = torch.zeros(len(layout), dtype=torch.float32, device="cuda:0")
    rng = np.random.default_rng([6, case, gdt])
    tables = [np.zeros((w, m), np.uint16 if fp16 else np.float32) for w, (_, m) in zip(ws, layout)]
    for t in range(4):
        grads = [S._grad(rng, n, m, gdt) for n, m in layout]
        S._to_dev_grads(torch, model, buf, grads)
        signs.fill_(-1)
        print(f"[scaled sign sketch case {case} gdt {gdt} fp16 {fp16} beta {beta}] step {t}: launching", flush=True)
        B.conef_cs_ss_step(model.ctx, buf["grads"], buf["table"], signs, cs, buf["ws"], B.Model.stream_handle())
        torch.cuda.synchronize()
        for l, (n, m) in enumerate(layout):
            words, c = R.cs_ss_step_matrix(grads[l], tables[l], beta, seed, l)
            tag = f"case {case} mat {l} step {t}"
            gt = S._get_table(model, buf, l)
            if not _check_scale(cs[l].item(), c, tag):
                tables[l][:] = gt
                continue
            so = B.conef_ss_offsets(model.ctx, l)["sign_off"]
            N = n * m
            got = signs[so:so + words.size].cpu().numpy().view(np.uint32).copy()
            if N % 32:
                got[-1] &= np.uint32((1 << (N % 32)) - 1)
            assert np.array_equal(got, words), f"{tag}: sign bits"
            assert np.array_equal(gt.view(np.uint16 if fp16 else np.uint32), tables[l].view(np.uint16 if fp16 else np.uint32)), \
                f"{tag}: table differs in {(gt != tables[l]).sum()} entries"
    model.close()


def test_scaled_sign_calls_refuse_the_other_kind_of_context(env):
    R, B, S, torch = env
    qm = B.Model([(64, 64)], 4, 4, 64, wl.F32, 1)
    sk = B.SketchModel([(64, 64)], [16], 4, 0.5, 0, wl.F32, 1)
    qb, sb = qm.alloc(), sk.alloc()
    sg = torch.zeros(256, dtype=torch.int32, device="cuda:0")
    c = torch.zeros(1, dtype=torch.float32, device="cuda:0")
    with pytest.raises(B.ConefError) as e:
        B.conef_cs_ss_step(qm.ctx, qb["grads"], qb["codes"], sg, c, qb["ws"])
    assert e.value.code == B.ESTATE
    with pytest.raises(B.ConefError) as e:
        B.conef_ss_step(sk.ctx, sb["grads"], sb["table"], sb["table"], sg, c, sb["ws"], 0)
    assert e.value.code == B.ESTATE
    assert B.lib().conef_ss_step(qm.ctx, 256, 256, 256, 0, 256, 256, 0, 0) == B.EINVAL      # null sign buffer
