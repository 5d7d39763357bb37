"""Pins for the quantised-variant oracle (appendix "Combining PuzzleMoE with Quantization").

None of these re-types the oracle's formulas: they check what the appendix and the arithmetic fix
(the bit-width accounting, the digit coding, the quantiser's error bound, exact special cases) and
a reduction of the quantised FFN to the already pinned dense-expert oracle."""
import numpy as np
import pytest

import oracle


def bf16(a):
    """float32 array -> bf16 bits (values chosen to be exactly representable)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    assert not (u & 0xFFFF).any(), "test value is not a bf16"
    return (u >> 16).astype(np.uint16)


def bf16_to_f64(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def random_case(rows, cols, seed, paper_masks=True):
    rng = np.random.RandomState(seed)
    mag = np.abs(rng.randn(rows, cols)).astype(np.float32) * 0.02
    merged = (mag.view(np.uint32) >> 16).astype(np.uint16)       # truncated to bf16: still non-negative
    if paper_masks:                                              # Eq. 4: never both clear
        t = rng.randint(0, 3, size=(rows, cols))
        m0 = ((t == 0) | (t == 2)).astype(np.uint8)
        m1 = ((t == 1) | (t == 2)).astype(np.uint8)
    else:
        m0 = rng.randint(0, 2, size=(rows, cols)).astype(np.uint8)
        m1 = rng.randint(0, 2, size=(rows, cols)).astype(np.uint8)
    s0 = rng.randint(0, 2, size=(rows, cols)).astype(np.uint8)
    s1 = rng.randint(0, 2, size=(rows, cols)).astype(np.uint8)
    return merged, m0, m1, s0, s1


def test_bit_width_accounting():
    """Appendix: (2 sign + 1.58 mask + 3 code + 0.125 scale) / 2 = 3.35.  The stored format spends
    13 bits on 8 base-3 digits (1.625 instead of log2 3), everything else as in the formula."""
    paper = (2 + 1.58 + 3 + 0.125) / 2
    assert round(paper, 2) == 3.35
    ours = oracle.q_bits_per_weight()
    assert ours == pytest.approx((2 + 13 / 8 + 3 + 16 / 128) / 2)
    assert ours - (2 + np.log2(3) + 3 + 0.125) / 2 == pytest.approx((13 / 8 - np.log2(3)) / 2)
    assert 3 ** 8 <= 2 ** 13 < 3 ** 9                            # 13 bits hold exactly 8 digits
    assert ours < 3.4 and ours / 16 < 0.22                       # > 4.7x smaller than bf16 experts


def test_digit_coding_is_a_bijection():
    """Every 13-bit mask number below 3^8 is produced by exactly one combination of 8 masks."""
    rows, cols = 6561 // 16 + 1, 128                             # 411 * 16 records >= 6561
    n_rec = rows * cols // 8
    digits = np.zeros((n_rec, 8), dtype=np.int64)
    vals = np.arange(n_rec) % 6561
    v = vals.copy()
    for e in range(8):
        digits[:, e] = v % 3
        v //= 3
    trit = digits.reshape(rows, cols).astype(np.uint8)
    m0 = ((trit == 0) | (trit == 2)).astype(np.uint8)
    m1 = ((trit == 1) | (trit == 2)).astype(np.uint8)
    merged = bf16(np.full((rows, cols), 0.5, dtype=np.float32))
    zeros = np.zeros((rows, cols), dtype=np.uint8)
    q = oracle.q_quantise(merged, m0, m1, zeros, zeros)
    assert (q["trit"] == trit).all()
    rec = oracle.q_records(q).reshape(-1)
    assert ((rec >> np.uint64(40)) == vals.astype(np.uint64)).all()
    assert len(set((rec[:6561] >> np.uint64(40)).tolist())) == 6561
    assert (rec >> np.uint64(53) == 0).all()                     # nothing above bit 52
    # masks recovered from the records' digits: expert p uses the element iff digit is p or 2
    for pos in (0, 1):
        w = oracle.q_dequantise(q, pos)
        assert ((w != 0) == ((trit == 2) | (trit == pos))).all()


def test_record_fields():
    """Field positions of one hand-built record: codes at 3e, S0 at 24+e, S1 at 32+e."""
    merged = bf16(np.array([[1, 2, 3, 4, 5, 6, 7, 0] + [0] * 120], dtype=np.float32))
    ones = np.ones((1, 128), dtype=np.uint8)
    s0 = np.zeros((1, 128), dtype=np.uint8); s0[0, 1] = 1
    s1 = np.zeros((1, 128), dtype=np.uint8); s1[0, 6] = 1
    q = oracle.q_quantise(merged, ones, ones, s0, s1)
    assert bf16_to_f64(q["scale"])[0, 0] == 1.0                  # max 7 / 7
    assert q["code"][0, :8].tolist() == [1, 2, 3, 4, 5, 6, 7, 0]
    rec = int(oracle.q_records(q)[0, 0])
    assert rec & 0xFFFFFF == sum(c << (3 * e) for e, c in enumerate([1, 2, 3, 4, 5, 6, 7, 0]))
    assert (rec >> 24) & 0xFF == 1 << 1 and (rec >> 32) & 0xFF == 1 << 6
    assert rec >> 40 == 6560                                     # all eight digits 2: 3^8 - 1


@pytest.mark.parametrize("paper_masks", [True, False])
def test_quantiser_error_bound_and_extremes(paper_masks):
    merged, m0, m1, s0, s1 = random_case(32, 512, seed=11, paper_masks=paper_masks)
    q = oracle.q_quantise(merged, m0, m1, s0, s1)
    assert q["n_bad"] == 0 and q["code"].max() <= 7
    mag = bf16_to_f64(merged)
    used = (m0 | m1).astype(bool)
    scale = np.repeat(bf16_to_f64(q["scale"]), 128, axis=1)
    recon = q["code"].astype(np.float64) * scale
    # nearest-level rounding: half a step, plus the fp32 rounding of the quotient
    inner = used & (q["code"] < 7)
    assert (np.abs(recon - mag)[inner] <= scale[inner] * (0.5 + 1e-6)).all()
    # a clamped element lies above the last decision level
    top = used & (q["code"] == 7)
    assert (mag[top] >= 6.5 * scale[top] * (1 - 1e-6)).all()
    # unused elements cost nothing and the group maximum reaches the top code
    assert (q["code"][~used] == 0).all()
    gmax = np.where(used, mag, 0).reshape(32, 4, 128).max(axis=2)
    gcode = np.where(used, q["code"], 0).reshape(32, 4, 128).max(axis=2)
    assert (gcode[gmax > 0] == 7).all()
    # the scale is the group maximum over 7, to bf16 precision
    assert np.allclose(bf16_to_f64(q["scale"]), gmax / 7, rtol=2 ** -8)
    # signs and masks pass through; both experts reconstruct with their own sign
    w0, w1 = oracle.q_dequantise(q, 0), oracle.q_dequantise(q, 1)
    assert (np.sign(w0)[m0.astype(bool) & (q["code"] > 0)] == (1 - 2.0 * s0)[m0.astype(bool) & (q["code"] > 0)]).all()
    assert (w0[~m0.astype(bool) & used] == 0).all() and (w1[~m1.astype(bool) & used] == 0).all()
    assert (np.abs(w0)[m0.astype(bool)] == recon[m0.astype(bool)]).all()


def test_exact_when_magnitudes_are_multiples_of_a_power_of_two():
    """Weights k * 2^-6 (k = 0..7, one 7 per group): scale 2^-6, codes k, reconstruction exact."""
    rng = np.random.RandomState(5)
    k = rng.randint(0, 8, size=(16, 256))
    k[:, 0] = 7; k[:, 128] = 7
    merged = bf16((k * 2.0 ** -6).astype(np.float32))
    ones = np.ones(k.shape, dtype=np.uint8)
    s0 = rng.randint(0, 2, size=k.shape).astype(np.uint8)
    q = oracle.q_quantise(merged, ones, ones, s0, 1 - s0)
    assert (q["code"] == k).all() and (bf16_to_f64(q["scale"]) == 2.0 ** -6).all()
    assert (oracle.q_dequantise(q, 0) == (1 - 2.0 * s0) * k * 2.0 ** -6).all()
    assert (oracle.q_dequantise(q, 1) == -(1 - 2.0 * s0) * k * 2.0 ** -6).all()


def test_zero_group_and_ties():
    merged = bf16(np.zeros((16, 128), dtype=np.float32))
    ones = np.ones((16, 128), dtype=np.uint8)
    q = oracle.q_quantise(merged, ones, ones, ones, ones)
    assert (q["scale"] == 0).all() and (q["code"] == 0).all()
    assert (oracle.q_dequantise(q, 0) == 0).all()
    # ties to even: scale 1 (max 7): 0.5 -> 0, 1.5 -> 2, 2.5 -> 2, 6.5 -> 6
    vals = np.zeros((1, 128), dtype=np.float32)
    vals[0, :5] = [7, 0.5, 1.5, 2.5, 6.5]
    q = oracle.q_quantise(bf16(vals), np.ones((1, 128), np.uint8), np.ones((1, 128), np.uint8),
                          np.zeros((1, 128), np.uint8), np.zeros((1, 128), np.uint8))
    assert q["code"][0, :5].tolist() == [7, 0, 2, 2, 6]


def test_ffn_reduces_to_the_dense_expert_oracle():
    """With weights that the quantiser reproduces exactly and that are bf16 numbers, the quantised
    layer's FFN (fp64 weights) must equal the bf16 oracle's FFN over the same experts kept dense."""
    rng = np.random.RandomState(9)
    d, f, E, T, k = 128, 256, 4, 5, 2

    def matrix(rows, cols):
        kk = rng.randint(0, 8, size=(rows, cols)); kk[:, ::128] = 7
        sgn = rng.randint(0, 2, size=(rows, cols)).astype(np.uint8)
        return kk, sgn

    experts64, dense_bits = [], []
    for e in range(0, E, 2):
        mats = []
        for rows, cols in ((f, d), (f, d), (d, f)):
            kk, sgn = matrix(rows, cols)
            t = rng.randint(0, 3, size=(rows, cols))
            m0 = ((t == 0) | (t == 2)).astype(np.uint8); m1 = ((t == 1) | (t == 2)).astype(np.uint8)
            q = oracle.q_quantise(bf16((kk * 2.0 ** -5).astype(np.float32)), m0, m1, sgn, 1 - sgn)
            mats.append((oracle.q_dequantise(q, 0), oracle.q_dequantise(q, 1)))
        for pos in (0, 1):
            experts64.append(tuple(m[pos] for m in mats))
            dense_bits.append(tuple(bf16(m[pos].astype(np.float32)) for m in mats))
    x = bf16((rng.randint(-8, 9, size=(T, d)) / 16.0).astype(np.float32))
    ids = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    w = rng.rand(T, k).astype(np.float32)
    y_q = oracle.ffn_dense64(x, ids, w, [e[0] for e in experts64], [e[1] for e in experts64], [e[2] for e in experts64])
    pair = np.array([-1 - j for j in range(E)], dtype=np.int32)
    y_d, _ = oracle.moe_ffn(x, ids, w, pair, np.zeros(E, np.uint8), [], [], [], dense=dense_bits)
    assert np.array_equal(y_q, y_d)
