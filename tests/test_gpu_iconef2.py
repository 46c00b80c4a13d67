"""GPU parity tests of improved contractive error feedback, version 2 (Algorithm 3 with e~+ = Q(p - Delta), the first
error vector a random block kept as it is, the second the quantiser's) around the random-block and the random-k
gradient compressors: the library, called through the C ABI, against oracle/iconef2_ref.c on the same seeded inputs,
free-running over several steps with the two buffers of first error vectors swapped from step to step.  Every
operation is element-wise fp32 arithmetic in a fixed order: kept values, first error vectors, codes and scales are
compared bit for bit."""
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


CASES = [
    # (layout, bits, block, fraction kept by the gradient compressor / stratum length, fraction kept by e~)
    ([(64, 128), (40, 512), (256, 96)], 4, 128, 0.1, 0.05),          # whole power-of-two blocks: the wave-per-run kernel
    ([(64, 147), (37, 53), (128, 576)], 4, 128, 0.1, 0.05),          # odd sizes: the kernel for any layout
    ([(32, 512), (100, 1024)], 2, 256, 0.25, 0.3),
    ([(96, 160), (33, 129)], 8, 8, 0.5, 0.9),                        # the two blocks overlap at every step
    ([(16, 64), (8, 8)], 4, 200, 0.1, 1.0),                          # e~ keeps all that Delta leaves: q stays empty
    ([(77, 768), (5, 128), (129, 64)], 8, 64, 0.1, 0.0),             # nothing kept in e~: the plain step
    ([(2000, 1024)], 4, 128, 0.01, 0.05),                            # many items
]


def _run(env, case, gdt, strata):
    R, B, S, torch = env
    layout, bits, block, frac, frac_e = CASES[case]
    seed = 2500 + case
    keep = wl.random_block_keep(layout, frac)
    group = [max(1, round(1.0 / frac))] * len(layout)
    keep_e = [int(round(frac_e * n * m)) for n, m in layout]
    model = B.Model(layout, 4, bits, block, gdt, seed)
    if strata:
        B.conef_rk_configure(model.ctx, group)
        n_delta = B.conef_rk_sizes(model.ctx)["delta_elems"]
    else:
        B.conef_rb_configure(model.ctx, keep)
        n_delta = B.conef_rb_sizes(model.ctx)["delta_elems"]
    B.conef_i2_configure(model.ctx, keep_e)
    buf = model.alloc()
    n_e = B.conef_i2_sizes(model.ctx)["e_elems"]
    e_bufs = [torch.zeros(n_e, dtype=torch.float32, device="cuda:0") for _ in range(2)]
    delta = torch.zeros(n_delta, dtype=torch.float32, device="cuda:0")
    rng = np.random.default_rng([case, gdt, 25, int(strata)])
    states = [[np.zeros(keep_e[l], np.float32), np.zeros(R.n_words(n * m, bits), np.uint32),
               np.zeros(R.n_blocks(n * m, block), np.float32)] for l, (n, m) in enumerate(layout)]
    live = False
    for t in range(4):
        grads = [S._grad(rng, n, m, gdt) for n, m in layout]
        S._to_dev_grads(torch, model, buf, grads)
        delta.fill_(float("nan"))
        e_in, e_out = e_bufs[t % 2], e_bufs[(t + 1) % 2]
        e_out.fill_(float("nan"))
        print(f"[iconef v2 {'random-k' if strata else 'random block'} case {case} gdt {gdt}] step {t}: launching", flush=True)
        (B.conef_i2_rk_step if strata else B.conef_i2_rb_step)(model.ctx, buf["grads"], e_in, e_out, buf["codes"], buf["scales"],
                                                               delta, t, model.stream_handle())
        torch.cuda.synchronize()
        for l, (n, m) in enumerate(layout):
            e, c, s = states[l]
            tag = f"case {case} mat {l} step {t}"
            if strata:
                want = R.i2_rk_step_matrix(grads[l], e, c, s, group[l], bits, block, seed, l, t)
                ro = B.conef_rk_offsets(model.ctx, l)
            else:
                want = R.i2_rb_step_matrix(grads[l], e, c, s, keep[l], bits, block, seed, l, t)
                ro = B.conef_rb_offsets(model.ctx, l)
            got = delta[ro["delta_off"]:ro["delta_off"] + want.size].cpu().numpy()
            assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), f"{tag}: kept values"
            eo = B.conef_i2_offsets(model.ctx, l)
            assert eo["keep_e"] == keep_e[l] and B.conef_i2_start(model.ctx, l, t) == R.i2_start(seed, l, t, n * m, keep_e[l])
            got_e = e_out[eo["e_off"]:eo["e_off"] + keep_e[l]].cpu().numpy()
            assert np.array_equal(got_e.view(np.uint32), e.view(np.uint32)), \
                f"{tag}: first error vector differs in {(got_e.view(np.uint32) != e.view(np.uint32)).sum()} of {e.size}"
            o = model.offsets[l]
            got_c = buf["codes"][o["word_off"]:o["word_off"] + c.size].cpu().numpy().view(np.uint32)
            got_s = buf["scales"][o["scale_off"]:o["scale_off"] + s.size].cpu().numpy()
            assert np.array_equal(got_c, c), f"{tag}: codes differ in {(got_c != c).sum()} words"
            assert np.array_equal(got_s.view(np.uint32), s.view(np.uint32)), f"{tag}: scales"
            live = live or bool(np.any(e != 0))
    assert live or frac_e == 0.0
    model.close()


@pytest.mark.parametrize("case", range(len(CASES)))
@pytest.mark.parametrize("gdt", [wl.F32, wl.BF16])
def test_iconef_v2_with_the_random_block_is_bit_exact(env, case, gdt):
    _run(env, case, gdt, False)


@pytest.mark.parametrize("case", range(len(CASES)))
@pytest.mark.parametrize("gdt", [wl.F32, wl.BF16])
def test_iconef_v2_with_random_k_is_bit_exact(env, case, gdt):
    _run(env, case, gdt, True)


def test_v2_calls_reject_what_they_cannot_serve(env):
    R, B, S, torch = env
    m = B.Model([(64, 64)], 4, 4, 64, wl.F32, 1)
    buf = m.alloc()
    e = [torch.zeros(4096, dtype=torch.float32, device="cuda:0") for _ in range(2)]
    d = torch.zeros(4096, dtype=torch.float32, device="cuda:0")
    a = (m.ctx, buf["grads"])
    with pytest.raises(B.ConefError) as ex:                      # not configured
        B.conef_i2_rb_step(*a, e[0], e[1], buf["codes"], buf["scales"], d, 0)
    assert ex.value.code == B.ESTATE
    B.conef_i2_configure(m.ctx, [100])
    with pytest.raises(B.ConefError) as ex:                      # no gradient compressor configured
        B.conef_i2_rb_step(*a, e[0], e[1], buf["codes"], buf["scales"], d, 0)
    assert ex.value.code == B.ESTATE
    B.conef_rb_configure(m.ctx, [400])
    with pytest.raises(B.ConefError) as ex:                      # one buffer for both first error vectors
        B.conef_i2_rb_step(*a, e[0], e[0], buf["codes"], buf["scales"], d, 0)
    assert ex.value.code == B.EINVAL
    with pytest.raises(B.ConefError) as ex:                      # random-k not configured
        B.conef_i2_rk_step(*a, e[0], e[1], buf["codes"], buf["scales"], d, 0)
    assert ex.value.code == B.ESTATE
    B.conef_set_beta(m.ctx, 0.5)
    with pytest.raises(B.ConefError) as ex:                      # Algorithm 3 has no partial update
        B.conef_i2_rb_step(*a, e[0], e[1], buf["codes"], buf["scales"], d, 0)
    assert ex.value.code == B.ESTATE
    B.conef_set_beta(m.ctx, 0.0)
    with pytest.raises(B.ConefError) as ex:
        B.conef_i2_configure(m.ctx, [64 * 64 + 1])
    assert ex.value.code == B.EINVAL
    B.conef_i2_rb_step(*a, e[0], e[1], buf["codes"], buf["scales"], d, 0)
    torch.cuda.synchronize()
    m.close()
