"""msrl_gae on the GPU against the oracle's reverse recurrence, element by element."""
import numpy as np
import pytest

from oracle import ref
from paper_2210_00882_amd import synth
from helpers import TOL_F32, assert_close

pytestmark = pytest.mark.gpu


def gpu_gae(r, v, d, gamma, lam):
    import torch
    from paper_2210_00882_amd import binding as B
    rt, vt, dt = (torch.from_numpy(np.ascontiguousarray(x)).cuda() for x in (r, v, d))
    adv = torch.full_like(rt, -77.0)
    ret = torch.full_like(rt, -77.0)
    B.msrl_gae(rt, vt, dt, gamma, lam, adv, ret)
    torch.cuda.synchronize()
    return adv.cpu().numpy(), ret.cpu().numpy()


@pytest.mark.parametrize("T,M,ep", [
    (1, 1, 1), (3, 5, 2), (7, 64, 3), (8, 65, 4), (9, 193, 5), (100, 192, 25),      # below / around one unroll block
    (128, 12288, 25), (17, 1000, 1), (33, 4099, 50),                                # ragged column counts, scalar path
    (20, 262144, 7), (21, 262148, 50),                                              # vector path (M % 4 == 0, large)
    (19, 262146, 6),                                                                # large but not a multiple of 4
])
def test_gae_matches_oracle(T, M, ep):
    r, v, d = synth.make_gae_inputs(T, M, ep, seed=T * 1000 + M)
    adv, ret = gpu_gae(r, v, d, 0.99, 0.95)
    oa, orr = ref.gae(r, v, d, 0.99, 0.95)
    assert_close(adv, oa, TOL_F32, "adv")
    assert_close(ret, orr, TOL_F32, "ret")


def test_gae_other_discounts_and_all_done():
    T, M = 40, 777
    r, v, d = synth.make_gae_inputs(T, M, 9, seed=5)
    for gamma, lam in [(1.0, 1.0), (0.9, 0.0), (0.0, 0.5)]:
        adv, ret = gpu_gae(r, v, d, gamma, lam)
        oa, orr = ref.gae(r, v, d, gamma, lam)
        assert_close(adv, oa, TOL_F32, f"adv gamma {gamma} lambda {lam}")
        assert_close(ret, orr, TOL_F32, "ret")
    ones = np.ones_like(d)
    adv, _ = gpu_gae(r, v, ones, 0.99, 0.95)
    assert_close(adv, r - v[:T], TOL_F32, "every step terminal: A = r - V")


def test_gae_empty_is_a_noop():
    import torch
    from paper_2210_00882_amd import binding as B
    e = torch.empty((0, 16), device="cuda")
    B.msrl_gae(e, torch.empty((1, 16), device="cuda"), e.to(torch.uint8), 0.99, 0.95, e.clone(), e.clone())
    torch.cuda.synchronize()


def test_gae_benchmark_size_sampled_columns():
    # cfg5's [200, 655360] in the launch configuration the benchmark uses; oracle on sampled columns
    cfg = synth.CONFIGS[5]
    import torch
    from paper_2210_00882_amd import binding as B
    T, M = cfg.T, cfg.M
    gen = torch.Generator(device="cuda").manual_seed(3)
    r = -torch.rand((T, M), device="cuda", generator=gen) * 5
    v = torch.randn((T + 1, M), device="cuda", generator=gen)
    d = (((torch.arange(T, device="cuda")[:, None] + 1) % cfg.episode_len) == 0).to(torch.uint8).expand(T, M).contiguous()
    adv = torch.empty_like(r)
    ret = torch.empty_like(r)
    B.msrl_gae(r, v, d, cfg.gamma, cfg.lam, adv, ret)
    torch.cuda.synchronize()
    cols = np.unique(np.concatenate([np.arange(0, 2048), np.arange(M - 2048, M), np.arange(0, M, 1021)]))
    ct = torch.from_numpy(cols).cuda()
    oa, orr = ref.gae(r[:, ct].cpu().numpy(), v[:, ct].cpu().numpy(), d[:, ct].cpu().numpy(), cfg.gamma, cfg.lam)
    assert_close(adv[:, ct].cpu().numpy(), oa, TOL_F32, "adv")
    assert_close(ret[:, ct].cpu().numpy(), orr, TOL_F32, "ret")
    assert float((ret - (adv + v[:T])).abs().max()) < 1e-4 * max(1.0, float(ret.abs().max()))
