"""Pins for the oracle's bf16 helpers, pack (Sec. 3.3.2) and unpack (Algorithm 1).  CPU only."""
import os

import numpy as np
import torch

HERE = os.path.dirname(os.path.abspath(__file__))


def closed_form_value(word, pos):
    """Independent arithmetic meaning of a packed word: (-1)^s m 2^(e5-15) (1 + mant/128)."""
    word = word.astype(np.int64)
    m = (word >> (13 - pos)) & 1
    s = (word >> (15 - pos)) & 1
    e5 = (word >> 7) & 31
    mant = word & 127
    return np.where(s == 1, -1.0, 1.0) * m * np.ldexp(1.0 + mant / 128.0, e5 - 15)


def bits_to_f64(bits):
    return torch.from_numpy(bits.astype(np.int16)).view(torch.bfloat16).double().numpy()


def test_bf16_rounding_matches_library_on_float32(oracle):
    g = torch.Generator().manual_seed(7)
    v = torch.randn(20000, generator=g) * torch.exp(torch.randn(20000, generator=g) * 8)
    # exact ties and near-ties in float32
    base = torch.tensor([1.0, 1.5, 0.02, 3e-39, 1e-40, 65280.0, 3.38e38], dtype=torch.float32)
    ties = torch.cat([base * (1 + 2.0 ** -8), base * (1 + 3 * 2.0 ** -8), -base * (1 + 2.0 ** -8)])
    v = torch.cat([v, ties, torch.tensor([0.0, -0.0, float("inf"), -float("inf")])])
    want = v.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([oracle.bf16_from_double(float(a)) for a in v.double()], dtype=np.uint16)
    assert np.array_equal(got, want)


def test_bf16_rounding_is_direct_from_double(oracle):
    # 1 + 2^-8 is a tie -> even (1.0); a hair above the tie must round up, which a
    # double -> float -> bf16 chain gets wrong (the float stage lands on the tie).
    assert oracle.bf16_from_double(1.0 + 2.0 ** -8) == 0x3F80
    assert oracle.bf16_from_double(1.0 + 2.0 ** -8 + 2.0 ** -40) == 0x3F81
    assert oracle.bf16_from_double(1.0 + 3 * 2.0 ** -8) == 0x3F82      # tie -> even upwards
    assert oracle.bf16_from_double(-(1.0 + 2.0 ** -8 + 2.0 ** -40)) == 0xBF81
    assert oracle.bf16_to_double(0x3F81) == 1.0078125


def test_algorithm1_truth_table_exhaustive(oracle):
    words = np.arange(65536, dtype=np.uint16)
    for pos in (0, 1):
        got = bits_to_f64(oracle.unpack(words, pos))
        assert np.array_equal(got, closed_form_value(words, pos))
        # masked-out elements are +0, never -0 (Algorithm 1 assigns 0 before the sign)
        out = oracle.unpack(words, pos)
        masked = ((words >> (13 - pos)) & 1) == 0
        assert np.all(out[masked] == 0)


def test_pack_unpack_equals_eq6_all_bf16_all_flags(oracle):
    mags = np.arange(32768, dtype=np.uint16)
    exps = mags >> 7
    ok = exps <= 143
    for flags in range(16):
        s0, s1, m0, m1 = [(np.full(mags.shape, (flags >> b) & 1, dtype=np.uint8)) for b in (3, 2, 1, 0)]
        packed, bad = oracle.pack(mags, m0, m1, s0, s1)
        assert bad == int((~ok).sum())
        # canon(W): exponent raised to 112 with the mantissa kept; Eq. 6 on that value
        canon = np.where(exps < 112, (112 << 7) | (mags & 0x7F), mags).astype(np.uint16)
        canon_val = np.where(mags == 0, 0.0, bits_to_f64(canon))
        for pos, s, m in ((0, s0, m0), (1, s1, m1)):
            with np.errstate(invalid="ignore"):
                want = np.where(s == 1, -1.0, 1.0) * m * canon_val
            got = bits_to_f64(oracle.unpack(packed, pos))
            assert np.array_equal(got[ok], want[ok] + 0.0)
            # inside the band the round trip reproduces the input magnitude itself
            band = (exps >= 112) & ok
            assert np.array_equal(np.abs(got[band]), bits_to_f64(mags)[band] * m[band])
            assert np.all(got[~ok] == 0)


def test_golden_examples(oracle):
    rows = []
    with open(os.path.join(HERE, "golden", "alg1_examples.txt")) as fh:
        for line in fh:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append([int(tok, 0) for tok in line.split()])
    assert len(rows) >= 10
    for merged, s0, s1, m0, m1, word, d0, d1 in rows:
        a = lambda v, t: np.array([v], dtype=t)
        packed, bad = oracle.pack(a(merged, np.uint16), a(m0, np.uint8), a(m1, np.uint8),
                                  a(s0, np.uint8), a(s1, np.uint8))
        assert bad == 0 and packed[0] == word, hex(packed[0])
        assert oracle.unpack(packed, 0)[0] == d0
        assert oracle.unpack(packed, 1)[0] == d1


def test_out_of_range_and_input_sign(oracle):
    one = np.ones(4, dtype=np.uint8)
    zero = np.zeros(4, dtype=np.uint8)
    merged = np.array([0x4800, 0x7F80, 0x7FC0, 0x47FF], dtype=np.uint16)   # 2^17, inf, nan, max ok
    packed, bad = oracle.pack(merged, one, one, zero, zero)
    assert bad == 3
    assert np.all(oracle.unpack(packed, 0)[:3] == 0) and oracle.unpack(packed, 0)[3] == 0x47FF
    pos_in, _ = oracle.pack(np.array([0x3CA4] * 4, dtype=np.uint16), one, one, zero, one)
    neg_in, _ = oracle.pack(np.array([0xBCA4] * 4, dtype=np.uint16), one, one, zero, one)
    assert np.array_equal(pos_in, neg_in)


def test_synthetic_weights_stay_in_band(oracle):
    from paper_2511_04805_amd import synth
    cfg = synth.CONFIGS["tiny"]
    m = synth.pair_matrix(cfg, 0, synth.GATE, shape=(1024, 1024))
    packed, bad = oracle.pack(m["merged"], m["mask0"], m["mask1"], m["sign0"], m["sign1"])
    assert bad == 0 and packed.nbytes == m["merged"].size * 2          # no metadata
    exps = m["merged"] >> 7
    clamp_frac = float((exps < 112).mean())
    # P(|N(0,0.02)| < 2^-15) = 2 pdf(0) 2^-15 / 0.02 ~ 1.22e-3
    assert 0.8e-3 < clamp_frac < 1.7e-3
    assert exps.max() <= 128
    for pos, mk, sg in ((0, "mask0", "sign0"), (1, "mask1", "sign1")):
        got = bits_to_f64(oracle.unpack(packed, pos))
        band = exps >= 112
        want = bits_to_f64(m["merged"]) * m[mk] * np.where(m[sg] == 1, -1.0, 1.0)
        assert np.array_equal(got[band], want[band] + 0.0)
        assert abs(float(m[mk].mean()) - 0.5) < 0.01
