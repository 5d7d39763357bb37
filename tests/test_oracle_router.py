"""Pins for the oracle's router (linear logits, top-k, softmax over the selected).  CPU only."""
import numpy as np
import torch


def bits(t):
    return t.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def test_router_matches_numpy_on_exact_inputs(oracle):
    """Small multiples of 1/4: every product and partial sum is exact in fp32, so the fma chain equals
    numpy's integer matmul and top-k / softmax can be checked against library routines."""
    g = torch.Generator().manual_seed(3)
    T, d, E, k = 37, 64, 12, 4
    x = torch.randint(-2, 3, (T, d), generator=g).float() * 0.25
    w = torch.randint(-2, 3, (E, d), generator=g).float() * 0.25
    ids, wts, logits = oracle.router_topk(bits(x), bits(w), k)
    ref = (x.double() @ w.double().T).numpy()
    assert np.array_equal(logits.astype(np.float64), ref)
    # library top-k with the tie rule "lower index first": sort by (-logit, index)
    order = np.lexsort((np.broadcast_to(np.arange(E), ref.shape), -ref), axis=1)[:, :k]
    assert np.array_equal(ids, order.astype(np.int32))
    sel = np.take_along_axis(ref, order, axis=1)
    want = torch.softmax(torch.from_numpy(sel), dim=1).numpy()
    assert np.allclose(wts, want, rtol=1e-6, atol=1e-9)
    assert np.allclose(wts.sum(1), 1.0, atol=1e-6)


def test_router_ties_and_permutation(oracle):
    T, d, E = 3, 32, 6
    x = torch.ones(T, d)
    w = torch.zeros(E, d)
    w[1, 0] = 2.0; w[4, 0] = 2.0; w[5, 0] = 1.0            # logits: e1 = e4 = 2 > e5 = 1 > others = 0
    ids, wts, _ = oracle.router_topk(bits(x), bits(w), 4)
    assert np.array_equal(ids[0], [1, 4, 5, 0])             # ties resolved towards the lower index
    e = np.exp(np.array([2.0, 2.0, 1.0, 0.0]) - 2.0)
    assert np.allclose(wts[0], e / e.sum(), rtol=1e-6)
    # permuting the experts permutes the ids
    perm = np.array([3, 0, 5, 1, 4, 2])
    g = torch.Generator().manual_seed(5)
    xr = torch.randn(8, d, generator=g)
    wr = torch.randn(E, d, generator=g)
    ids_a, w_a, _ = oracle.router_topk(bits(xr), bits(wr), 2)
    ids_b, w_b, _ = oracle.router_topk(bits(xr), bits(wr[perm]), 2)
    assert np.array_equal(perm[ids_b], ids_a) and np.array_equal(w_a, w_b)
