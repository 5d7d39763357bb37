"""The oracle's integer decisions against the plain fp64 definitions.  CPU only.

Three parts of the oracle decide integers by floating-point comparisons and take them in fp32 so
that the kernel and the oracle agree bit for bit: the masks of the dual-mask merge, the experts a
router picks, the codes of the quantised variant.  fp32 is not what the paper defines.  These
tests evaluate the definitions themselves in fp64 -- with the division in the similarity measure
(display before Eq. 1), the saliency products (Eqs. 2-3), the router's logits as dot products,
the quantiser's quotient magnitude / scale -- and require that a decision of the oracle differs
from the definition's only where the fp64 margin of that decision lies inside the rounding error
of a handful of fp32 operations.  Every count is printed.
"""
import numpy as np
import torch

U24 = 2.0 ** -24          # half an ulp of fp32, relative


def say(msg):
    print(msg, flush=True)


def bits(t):
    return t.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def f64(b):
    return (np.ascontiguousarray(b).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def test_merge_masks_against_fp64_definition(oracle):
    """Similarity: | |wi|-|wj| | / (|wi|+|wj|) <= tau, by division, in fp64.  Saliency: |wi| n_i >=
    |wj| n_j with exact fp64 products (8-bit x 24-bit significands).  The oracle's fp32 decisions
    round the difference, the sum and tau * sum once each (and each saliency product once), so
    they may differ only where the definition's margin is within 4 such roundings."""
    n, tau = 2048, np.float32(0.4)
    g = torch.Generator().manual_seed(21)
    wi = bits(torch.randn(n, n, generator=g) * 0.02)
    wj = bits(torch.randn(n, n, generator=g) * 0.02)
    ni = (torch.rand(n, generator=g) * 3 + 0.25).numpy().astype(np.float32)
    nj = (torch.rand(n, generator=g) * 3 + 0.25).numpy().astype(np.float32)
    r = oracle.merge(wi, wj, ni, nj, float(tau))
    sim_orc = (r["mask0"] == 1) & (r["mask1"] == 1)

    a, b = np.abs(f64(wi)), np.abs(f64(wj))
    s = a + b
    with np.errstate(invalid="ignore", divide="ignore"):
        delta = np.abs(a - b) / s                                # the paper's measure; 0/0 -> nan -> not similar
    sim_def = delta <= float(tau)
    differ = sim_orc != sim_def
    margin = np.abs(delta - float(tau))                          # in units of delta (<= 1)
    bound = 4 * 2 * U24                                          # 4 roundings of half an ulp, doubled for the division by s
    say("merge, %d elements: similarity decisions that differ from the fp64 definition: %d "
        "(%.2e of all); elements whose margin is inside the bound %.1e: %d"
        % (n * n, differ.sum(), differ.mean(), bound, (margin <= bound).sum()))
    assert np.all(margin[differ] <= bound)
    assert differ.mean() < 1e-5
    # the real number 0.4 instead of its fp32 neighbour: the same, the two differ by 1.5e-8 relative
    differ_real = sim_orc != (delta <= 0.4)
    assert np.all(np.abs(delta - 0.4)[differ_real] <= bound + abs(float(tau) - 0.4))

    sal_i, sal_j = a * ni.astype(np.float64)[None, :], b * nj.astype(np.float64)[None, :]
    pick_def = sal_i >= sal_j                                    # Eq. 3, ties to expert i
    dis = ~sim_orc & ~sim_def
    pick_orc = (r["mask0"] == 1)
    differ_s = dis & (pick_orc != pick_def)
    rel = np.abs(sal_i - sal_j) / np.maximum(np.maximum(sal_i, sal_j), 1e-300)
    say("merge: saliency decisions (dissimilar elements) that differ: %d (%.2e); inside 2 roundings: %d"
        % (differ_s.sum(), differ_s.sum() / max(dis.sum(), 1), (dis & (rel <= 2 * U24)).sum()))
    assert np.all(rel[differ_s] <= 2 * U24)
    assert differ_s.sum() / max(dis.sum(), 1) < 1e-5

    # Eq. 5 in fp64: the mean of the two magnitudes, then ONE rounding to bf16.  The oracle forms
    # the sum and its half in fp32 first; both are exact there unless the magnitudes are more than
    # 2^16 apart, which similar elements never are.
    both = sim_orc & sim_def
    mean_bits = np.array([oracle.bf16_from_double(v) for v in (s[both] / 2)[:200000]], dtype=np.uint16)
    assert np.array_equal(r["merged"][both][:200000], mean_bits)


def test_router_choice_against_fp64_logits(oracle):
    """Logits as fp64 dot products.  Every step of the oracle's fp32 fused-multiply-add chain
    rounds the running sum once, so the chain is within 2^-24 * sum_c |partial sum_c| of the
    definition, and its k chosen experts, in order, are those of the definition for every token
    whose first k+1 fp64 logits are further apart than twice that."""
    g = torch.Generator().manual_seed(31)
    T, d, E, k = 768, 2048, 64, 6
    x = torch.randn(T, d, generator=g)
    w = torch.randn(E, d, generator=g) * 0.05
    xb, wb = bits(x), bits(w)
    ids, wts, logits32 = oracle.router_topk(xb, wb, k)
    xd, wd = f64(xb), f64(wb)
    logits = xd @ wd.T
    err_bound = np.empty((T, E))
    for t0 in range(0, T, 64):                                   # partial sums of every chain, in fp64
        part = np.cumsum(xd[t0:t0 + 64, None, :] * wd[None, :, :], axis=2)
        err_bound[t0:t0 + 64] = 1.001 * U24 * np.abs(part).sum(axis=2)
    err = np.abs(logits32.astype(np.float64) - logits)
    assert np.all(err <= err_bound)
    order = np.lexsort((np.broadcast_to(np.arange(E), logits.shape), -logits), axis=1)
    top = np.take_along_axis(logits, order[:, :k + 1], axis=1)
    gap = (top[:, :-1] - top[:, 1:]).min(axis=1)                 # smallest gap among the first k+1
    safe = gap > 2 * err_bound.max(axis=1)
    differ = (ids != order[:, :k].astype(np.int32)).any(axis=1)
    say("router, %d tokens x %d experts, top-%d: tokens whose choice differs from the fp64 definition: %d; "
        "tokens inside the error bound: %d; largest |fp32 chain - fp64 logit| = %.2e (bound %.2e)"
        % (T, E, k, differ.sum(), (~safe).sum(), err.max(), err_bound.max()))
    assert not np.any(differ & safe)
    assert safe.mean() > 0.98
    # a sharper statement with the measured error instead of the worst-case bound
    assert not np.any(differ & (gap > 2 * err.max()))
    assert differ.mean() < 5e-3
    # weights: softmax over the selected fp64 logits
    sel = np.take_along_axis(logits, ids.astype(np.int64), axis=1)
    want = torch.softmax(torch.from_numpy(sel), dim=1).numpy()
    assert np.allclose(wts, want, rtol=0, atol=4 * err.max() + 1e-7)


def test_quantiser_against_fp64_quotients(oracle):
    """Scale: bf16(max / 7) with the quotient in fp64 and ONE rounding to bf16.  Code:
    min(7, round-half-even(magnitude / scale)) with the quotient in fp64.  The oracle rounds each
    quotient to fp32 first, so a scale may differ only where max / 7 is within 2^-24 (relative)
    of the midpoint of two bf16 numbers, and a code only where magnitude / scale is within
    2^-24 (relative) of a half-integer."""
    rng = np.random.RandomState(41)
    rows, cols = 1024, 2048
    mag = (np.abs(rng.randn(rows, cols)) * 0.02).astype(np.float32)
    merged = ((mag.view(np.uint32) + 0x8000) >> 16).astype(np.uint16)
    t = rng.randint(0, 3, size=(rows, cols))
    m0 = ((t == 0) | (t == 2)).astype(np.uint8)
    m1 = ((t == 1) | (t == 2)).astype(np.uint8)
    z = np.zeros_like(m0)
    q = oracle.q_quantise(merged, m0, m1, z, z)
    m = f64(merged)
    mx = m.reshape(rows, cols // 128, 128).max(axis=2)
    quo = mx / 7.0
    scale_def = np.array([oracle.bf16_from_double(v) for v in quo.ravel()], dtype=np.uint16).reshape(quo.shape)
    differ = scale_def != q["scale"]
    # distance of max/7 from the nearest midpoint between neighbouring bf16 numbers, relative
    lo = f64(np.minimum(scale_def, q["scale"]))
    hi = f64(np.maximum(scale_def, q["scale"]))
    mid_rel = np.abs(quo - (lo + hi) / 2) / quo
    say("quantiser, %d groups: scales that differ from the fp64 definition: %d" % (quo.size, differ.sum()))
    assert np.all(mid_rel[differ] <= U24)
    assert differ.mean() < 1e-4

    sc = np.repeat(f64(q["scale"]), 128, axis=1)                 # the scales the oracle stored
    ratio = m / sc
    code_def = np.minimum(7, np.rint(ratio)).astype(np.uint8)    # numpy rint: ties to even
    differ_c = code_def != q["code"]
    half_rel = np.abs(ratio - (np.floor(ratio) + 0.5)) / np.maximum(ratio, 1e-300)
    say("quantiser, %d elements: codes that differ from the fp64 definition: %d (%.2e); "
        "elements within 2^-24 of a half-integer quotient: %d"
        % (m.size, differ_c.sum(), differ_c.mean(), (half_rel <= U24).sum()))
    assert np.all(half_rel[differ_c] <= U24)
    assert differ_c.mean() < 1e-5
