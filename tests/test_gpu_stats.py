"""GPU parity of the per-head statistics (Eq. 3 sparsity rate, Eq. 4 redundancy rate)."""
import sys

import numpy as np
import pytest
import torch

import ems_inputs
from gpu_util import dev_tensor
from oracle import ems_ref
from oracle.ems_ref import RefParams
from paper_2412_08521_amd import binding as B

pytestmark = pytest.mark.gpu


def _log(*a):
    print("[case]", *a, file=sys.stderr, flush=True)


@pytest.mark.parametrize("zeta", [0.5, 0.9, 0.99, 1.0])
@pytest.mark.parametrize("bh_n", [(3, 700), (2, 5000), (1, 40000)])
def test_sparsity_rate_matches_oracle(bh_n, zeta):
    bh, n = bh_n
    _log("sparsity", bh_n, zeta)
    rng = np.random.default_rng(n)
    g = rng.gamma(0.3, 1.0, (1, bh, n)).astype(np.float32)
    l = rng.gamma(0.3, 0.02, (1, bh, n)).astype(np.float32)
    l[..., ::23] *= 300
    p = B.EmsParams(1, bh, bh, 64, n, 8)
    rate, nk = B.ems_sparsity_rate(p, zeta, torch.from_numpy(g).cuda(), torch.from_numpy(l).cuda())
    rp = RefParams(1, bh, bh, 64, n, 8)
    o_rate, o_nk = ems_ref.sparsity(rp, zeta, g, l)
    nk = nk.cpu().numpy()
    for h in range(bh):
        # the count may differ only where the threshold is met within float32 noise of the total
        c = l[0, h].astype(np.float64).sum() / g[0, h].astype(np.float64).sum()
        s = np.sort(np.maximum(g[0, h].astype(np.float64) * c, l[0, h].astype(np.float64)))[::-1]
        cs, thr = np.cumsum(s), zeta * s.sum()
        k = int(nk[0, h])
        assert 1 <= k <= n
        assert cs[k - 1] >= thr * (1 - 2e-5), (h, k, o_nk[0, h])
        assert k == 1 or cs[k - 2] < thr * (1 + 2e-5), (h, k, o_nk[0, h])
        if zeta < 1.0:
            assert abs(k - int(o_nk[0, h])) <= max(2, n // 2000), (k, o_nk[0, h])
    np.testing.assert_allclose(rate.cpu().numpy(), 1 - nk / n, rtol=1e-6, atol=1e-7)
    if zeta < 1.0:
        np.testing.assert_allclose(rate.cpu().numpy(), o_rate, atol=max(2, n // 2000) / n + 1e-6)


def test_sparsity_closed_forms_on_gpu():
    n = 4096
    p = B.EmsParams(1, 3, 3, 64, n, 8)
    s = np.zeros((1, 3, n), np.float32)
    s[0, 0] = 0.5                                      # uniform: zeta of the tokens
    s[0, 1, 77] = 2.0                                  # one-hot: one token
    s[0, 2] = 2.0 ** -(np.arange(n) % 64).astype(np.float32)   # 64 groups of equal scores: exact ties
    t = torch.from_numpy(s).cuda()
    rate, nk = B.ems_sparsity_rate(p, 0.75, t, t.clone())
    nk = nk.cpu().numpy()[0]
    assert nk[0] == int(np.ceil(0.75 * n)) and nk[1] == 1
    _, o_nk = ems_ref.sparsity(RefParams(1, 3, 3, 64, n, 8), 0.75, s, s)
    assert nk[2] == o_nk[0, 2]


@pytest.mark.parametrize("mode", [B.EMS_BF16, B.EMS_F32])
@pytest.mark.parametrize("shape", [(1, 2, 64, 700), (2, 1, 128, 1500), (1, 1, 128, 3001)])
def test_redundancy_rate_matches_oracle(shape, mode):
    b, h, d, n = shape
    _log("redundancy", shape, mode)
    inp = ems_inputs.small(b, h, h, d, n, seed=n)
    kf, vf = inp.f32("k").copy(), inp.f32("v").copy()
    rng = np.random.default_rng(7)
    for t in range(20, n, 11):                         # near-copies of earlier tokens
        j = rng.integers(0, t)
        kf[:, :, t] = 0.95 * kf[:, :, j] + 0.2 * kf[:, :, t]
        vf[:, :, t] = 0.9 * vf[:, :, j] + 0.25 * vf[:, :, t]
    kb, vb = ems_inputs.f32_to_bf16_bits(kf), ems_inputs.f32_to_bf16_bits(vf)
    kf, vf = ems_inputs.bf16_bits_to_f32(kb), ems_inputs.bf16_bits_to_f32(vb)
    tau = 0.6
    p = B.EmsParams(b, h, h, d, n, 8, tau=tau, dtype=mode)
    rate, best = B.ems_redundancy_rate(p, dev_tensor(kb, mode), dev_tensor(vb, mode))
    o_rate, o_best = ems_ref.redundancy(RefParams(b, h, h, d, n, 8, tau=tau), kf, vf)
    best = best.cpu().numpy()
    assert (best[..., 0] == -np.inf).all()
    np.testing.assert_allclose(best[..., 1:], o_best[..., 1:], rtol=0, atol=1e-5)
    # the count: tokens whose best redundancy is within float32 noise of tau may fall on either side
    sure = (o_best >= tau + 2e-5).sum(-1)
    maybe = (np.abs(o_best - tau) < 2e-5).sum(-1)
    got = np.rint(rate.cpu().numpy() * n)
    assert (got >= sure).all() and (got <= sure + maybe).all()
    assert 0.02 < o_rate.mean() < 0.5
    # the rate is exactly the count of the kernel's own best values
    np.testing.assert_array_equal(got, (best >= np.float32(tau)).sum(-1))
