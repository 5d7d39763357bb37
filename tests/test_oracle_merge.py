"""Pins for the oracle's offline dual-mask merge (Sec. 3.2, Eqs. 1-5).  CPU only."""
import math

import numpy as np
import pytest
import torch


def bits(t):
    return t.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def f64(b):
    return torch.from_numpy(np.ascontiguousarray(b).astype(np.int16)).view(torch.bfloat16).double().numpy()


def gaussian_pair(n, sigma_i, sigma_j, seed):
    g = torch.Generator().manual_seed(seed)
    return (bits(torch.randn(n, n, generator=g) * sigma_i), bits(torch.randn(n, n, generator=g) * sigma_j))


def lemma31(tau, ratio=1.0):
    """Closed form of Lemma 3.1 (appendix form with sigma_j / sigma_i = ratio)."""
    return 2 / math.pi * (math.atan(ratio * (1 + tau) / (1 - tau)) - math.atan(ratio * (1 - tau) / (1 + tau)))


@pytest.mark.parametrize("tau,ratio", [(0.4, 1.0), (0.2, 1.0), (0.6, 1.0), (0.4, 2.0), (0.3, 0.5)])
def test_similar_fraction_matches_lemma_3_1(oracle, tau, ratio):
    n = 1536
    wi, wj = gaussian_pair(n, 0.02, 0.02 * ratio, seed=int(tau * 100 + ratio * 7))
    one = np.ones(n, dtype=np.float32)
    r = oracle.merge(wi, wj, one, one, tau)
    p = lemma31(tau, ratio)
    frac = r["n_similar"] / n / n
    sigma = math.sqrt(p * (1 - p) / (n * n))
    assert abs(frac - p) < 5 * sigma + 2e-4, (frac, p)          # 2e-4: bf16 grid of the inputs
    assert abs(lemma31(0.4) - 0.48447) < 1e-5
    if ratio == 1.0:
        # Eq. 4: density of each mask = P_sim + (1 - P_sim) / 2
        for m in ("mask0", "mask1"):
            assert abs(float(r[m].mean()) - (p + (1 - p) / 2)) < 2e-3


def test_mask_structure_and_reconstruction_bound(oracle):
    n, tau = 512, 0.4
    wi, wj = gaussian_pair(n, 0.02, 0.02, seed=3)
    g = torch.Generator().manual_seed(5)
    ni = (torch.rand(n, generator=g) + 0.5).numpy().astype(np.float32)
    nj = (torch.rand(n, generator=g) + 0.5).numpy().astype(np.float32)
    r = oracle.merge(wi, wj, ni, nj, tau)
    m0, m1 = r["mask0"].astype(bool), r["mask1"].astype(bool)
    assert np.all(m0 | m1)                                        # never (0, 0): Eq. 4
    a, b, mg = np.abs(f64(wi)), np.abs(f64(wj)), f64(r["merged"])
    sim = m0 & m1
    d, s = np.abs(a - b), a + b
    assert np.all(d[sim] <= tau * s[sim] * (1 + 1e-6)) and np.all(d[~sim] >= tau * s[~sim] * (1 - 1e-6))
    # Eq. 3 with channel norms: on dissimilar elements the kept expert is the more salient one
    sal_i = a.astype(np.float32) * ni[None, :]
    sal_j = b.astype(np.float32) * nj[None, :]
    assert np.array_equal(m0 & ~sim, (sal_i >= sal_j) & ~sim)
    assert np.array_equal(m1 & ~sim, (sal_i < sal_j) & ~sim)
    # Eq. 5: kept magnitude is exact on dissimilar elements, the rounded mean on similar ones
    assert np.array_equal(mg[m0 & ~sim], a[m0 & ~sim]) and np.array_equal(mg[m1 & ~sim], b[m1 & ~sim])
    assert np.all(np.abs(mg[sim] - s[sim] / 2) <= s[sim] / 2 * 2.0 ** -8)
    # Eq. 6 on the merge: |W_hat - W| <= tau (|wi|+|wj|) / 2 (+ bf16 rounding of the mean) where kept
    for w, m, sg in ((wi, m0, "sign0"), (wj, m1, "sign1")):
        what = np.where(r[sg] == 1, -1.0, 1.0) * mg
        err = np.abs(what - f64(w))[m]
        assert np.all(err <= (tau * s / 2)[m] + (s / 2)[m] * 2.0 ** -8)
        assert np.array_equal(r[sg] == 1, f64(w) < 0)             # Eq. 1


def test_special_cases(oracle):
    n = 64
    wi, wj = gaussian_pair(n, 0.02, 0.02, seed=9)
    one = np.ones(n, dtype=np.float32)
    same = oracle.merge(wi, wi, one, one, 0.4)                    # identical experts: everything similar
    assert same["n_similar"] == int((wi & 0x7FFF != 0).sum())
    assert np.array_equal(same["merged"][wi & 0x7FFF != 0], (wi & 0x7FFF)[wi & 0x7FFF != 0])
    all_sim = oracle.merge(wi, wj, one, one, 1.0)                 # tau = 1: d <= s always
    assert all_sim["n_similar"] == int(((wi & 0x7FFF) + (wj & 0x7FFF) != 0).sum())
    none_sim = oracle.merge(wi, wj, one, one, 0.0)                # tau = 0: only equal magnitudes
    assert none_sim["n_similar"] == int((((wi & 0x7FFF) == (wj & 0x7FFF)) & ((wi & 0x7FFF) != 0)).sum())
    # a dominant activation norm on expert j makes j win every dissimilar element
    big = oracle.merge(wi, wj, one, one * 1e6, 0.0)
    nz = (wj & 0x7FFF) != 0
    assert np.all(big["mask1"][nz] == 1)
    # both zero: not similar, expert i kept (tie), merged 0
    z = np.zeros((16, 32), dtype=np.uint16)
    zz = oracle.merge(z, z, np.ones(32, np.float32), np.ones(32, np.float32), 0.4)
    assert zz["n_similar"] == 0 and np.all(zz["merged"] == 0) and np.all(zz["mask0"] == 1) and np.all(zz["mask1"] == 0)


def test_merge_feeds_pack_and_eq6(oracle):
    """merge -> pack -> unpack gives (-1)^S * M * W_merged for both experts."""
    n = 128
    wi, wj = gaussian_pair(n, 0.02, 0.02, seed=13)
    one = np.ones(n, dtype=np.float32)
    r = oracle.merge(wi, wj, one, one, 0.4)
    packed, bad = oracle.pack(r["merged"], r["mask0"], r["mask1"], r["sign0"], r["sign1"])
    assert bad == 0
    mg = f64(r["merged"])
    in_band = (r["merged"] >> 7) >= 112
    for pos in (0, 1):
        want = np.where(r["sign%d" % pos] == 1, -1.0, 1.0) * r["mask%d" % pos] * mg
        got = f64(oracle.unpack(packed, pos))
        assert np.array_equal(got[in_band], want[in_band] + 0.0)
