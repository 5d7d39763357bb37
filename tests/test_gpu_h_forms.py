"""The two forms of the SwiGLU output H between the contractions, and the decode behind each.

Packed pairs keep H as one half-precision plane (the down projection then decodes its weights to
half precision) unless a down matrix holds weights of 2^15 and more, or the caller asks for the
wide form (two bf16 planes).  Checked here against the CPU oracle, which knows neither form:
  - the half-precision decode, bit for bit, on every 16-bit word it is defined for;
  - FFN layers whose weights span the format's whole exponent range 112..143 (Sec. 3.3.2), with
    clamped and zero words, in the wide form, and whose down matrices span 112..141 in the
    half-precision form;
  - activations scaled down until H sits in half precision's subnormal range, and scaled up until
    it saturates (counted, finite; the wide form of the same layer stays within the bound);
  - shared (dense bf16) experts on the tiled kernels, whose H is one half-precision plane too and
    whose down matrices are decoded to half precision times a power of two taken from their
    largest exponent: ordinary weights, weights over 30 and over 80 binades, huge and tiny ones,
    two experts of one launch with different ranges, saturation, and the wide form on request.
"""
import numpy as np
import pytest
import torch

from paper_2511_04805_amd import synth
from helpers import bits_to_f64, tolerance_ok

pytestmark = pytest.mark.gpu
W3 = (synth.GATE, synth.UP, synth.DOWN)


def say(msg):
    print(msg, flush=True)


@pytest.fixture(scope="module")
def binding():
    from paper_2511_04805_amd import binding as b
    b.load()
    assert torch.cuda.is_available()
    return b


def test_half_decode_all_words(oracle, binding):
    """Every word whose exponent field is at most 29, both positions: the half-precision decode is
    exactly twice Algorithm 1's bf16 result (and +0 where the mask bit is clear)."""
    words = np.arange(65536, dtype=np.uint16).reshape(64, 1024)
    tiled = np.empty(65536, dtype=np.uint16)
    r, c = np.divmod(np.arange(65536), 1024)
    tiled[((r // 16) * 32 + c // 32) * 512 + (((c % 32) // 8) * 16 + r % 16) * 8 + c % 8] = words.reshape(-1)
    t = torch.from_numpy(tiled.view(np.int16)).cuda()
    defined = ((words >> 7) & 31) <= 29
    assert defined.sum() == 65536 * 30 // 32
    for pos in (0, 1):
        out = binding.pzl_unpack_half_x2(t, pos, 64, 1024)
        torch.cuda.synchronize()
        got_bits = out.view(torch.int16).cpu().numpy().view(np.uint16)
        got = out.double().cpu().numpy()
        want = 2.0 * bits_to_f64(oracle.unpack(words, pos))
        assert np.array_equal(got[defined], want[defined])
        masked = defined & (((words >> (13 - pos)) & 1) == 0)
        assert np.all(got_bits[masked] == 0)                  # +0, not -0


class PlaneCase:
    """A layer built from explicit pack inputs: planes[p][which] = dict(merged, mask0, mask1, sign0, sign1)."""

    def __init__(self, oracle, binding, d, f, planes, wide_h=False, shared=()):
        """shared: (gate [fs, d], up [fs, d], down [d, fs]) bf16 bit patterns (uint16) per shared expert."""
        self.oracle, self.d, self.f = oracle, d, f
        self.shared_cpu = [tuple(np.ascontiguousarray(m) for m in mats) for mats in shared]
        shared_gpu = [tuple(binding.pzl_tile_dense(torch.from_numpy(m.view(np.int16)).cuda()) for m in mats) + (mats[0].shape[0],)
                      for mats in self.shared_cpu]
        P = len(planes)
        self.cpu, gpu = {}, {}
        n_bad = torch.zeros(1, dtype=torch.int32, device="cuda")
        for p in range(P):
            for which in W3:
                pl = planes[p][which]
                dev = {k: torch.from_numpy(v.view(np.int16) if v.dtype == np.uint16 else v).cuda() for k, v in pl.items()}
                gpu[p, which] = binding.pzl_pack(dev["merged"], dev["mask0"], dev["mask1"], dev["sign0"], dev["sign1"],
                                                 n_out_of_range=n_bad)
                self.cpu[p, which], bad = oracle.pack(pl["merged"], pl["mask0"], pl["mask1"], pl["sign0"], pl["sign1"])
                assert bad == 0
                rows, cols = pl["merged"].shape
                got = binding.tiled_to_logical(gpu[p, which].cpu().numpy().view(np.uint16), rows, cols)
                assert np.array_equal(got, self.cpu[p, which])
        assert int(n_bad.item()) == 0
        self.pair = np.repeat(np.arange(P, dtype=np.int32), 2)
        self.pos = np.tile(np.array([0, 1], dtype=np.uint8), P)
        self.P = P
        self.layer = binding.Layer(d, f, self.pair, self.pos, [gpu[p, synth.GATE] for p in range(P)],
                                   [gpu[p, synth.UP] for p in range(P)], [gpu[p, synth.DOWN] for p in range(P)],
                                   shared=shared_gpu, wide_h=wide_h)

    def gpu(self, x, ids, w):
        y = self.layer.pzl_moe_ffn(torch.from_numpy(x.view(np.int16)).cuda(), torch.from_numpy(ids).cuda(),
                                   torch.from_numpy(w).cuda())
        torch.cuda.synchronize()
        return y.view(torch.int16).cpu().numpy().view(np.uint16)

    def ref(self, x, ids, w):
        return self.oracle.moe_ffn(x, ids, w, self.pair, self.pos, [self.cpu[p, synth.GATE] for p in range(self.P)],
                                   [self.cpu[p, synth.UP] for p in range(self.P)],
                                   [self.cpu[p, synth.DOWN] for p in range(self.P)], shared=self.shared_cpu)[0]


def draw_planes(rng, shape, exp_lo, exp_hi, sigma=None):
    """Pack inputs with bf16 exponents uniform over [exp_lo, exp_hi] and random mantissas (or, with
    sigma, magnitudes |N(0, sigma)|), a sprinkle of exact zeros and of values below the band
    (exponent < 112, which pack raises to 112), independent masks and signs."""
    n = shape[0] * shape[1]
    if sigma is None:
        merged = ((rng.randint(exp_lo, exp_hi + 1, size=n) << 7) | rng.randint(0, 128, size=n)).astype(np.uint16)
    else:
        v = np.abs(rng.randn(n) * sigma).astype(np.float32)
        merged = ((v.view(np.uint32) + 0x8000) >> 16).astype(np.uint16)
    special = rng.rand(n)
    merged[special < 0.01] = 0
    below = (special >= 0.01) & (special < 0.03)
    merged[below] = ((rng.randint(90, 112, size=int(below.sum())) << 7) | rng.randint(0, 128, size=int(below.sum()))).astype(np.uint16)
    bits = lambda: rng.randint(0, 2, size=shape).astype(np.uint8)
    return {"merged": merged.reshape(shape), "mask0": bits(), "mask1": bits(), "sign0": bits(), "sign1": bits()}


def batch(rng, T, d, E, k, scale=1.0):
    x = (rng.randn(T, d) * scale).astype(np.float32)
    xb = ((x.view(np.uint32) + 0x8000) >> 16).astype(np.uint16)
    ids = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    w = rng.rand(T, k).astype(np.float32)
    w /= w.sum(1, keepdims=True)
    return xb, ids, w


@pytest.mark.parametrize("T", [24, 200])
def test_whole_exponent_range_wide_form(oracle, binding, T):
    """Every matrix spans exponents 112..143 (stored fields 0..31), with zero and clamped words:
    the library picks the wide form by itself (fields 30 and 31 have no half-precision decode)."""
    rng = np.random.RandomState(501)
    d, f, P = 256, 384, 2
    planes = [{which: draw_planes(rng, synth.matrix_shape(synth.LayerConfig("r", 4, d, f, 2, (1,)), which), 112, 143)
               for which in W3} for _ in range(P)]
    case = PlaneCase(oracle, binding, d, f, planes)
    assert case.layer.h_info()[0] is False
    x, ids, w = batch(rng, T, d, 2 * P, 2, scale=2.0 ** -20)     # keeps y inside fp32 with weights up to 2^17
    y = case.gpu(x, ids, w)
    ok, worst = tolerance_ok(y, case.ref(x, ids, w))
    say("exponents 112..143, wide H, T=%d: worst err / bound = %.3f" % (T, worst))
    assert ok, worst


@pytest.mark.parametrize("T", [24, 200])
def test_down_range_to_field_29_half_form(oracle, binding, T):
    """Down matrices span exponents 112..141 (fields 0..29, the whole range the half-precision
    decode covers), gate/up are ordinary small weights: the half-precision form, no saturation."""
    rng = np.random.RandomState(502)
    d, f, P = 256, 384, 2
    cfg = synth.LayerConfig("r", 4, d, f, 2, (1,))
    planes = [{synth.GATE: draw_planes(rng, synth.matrix_shape(cfg, synth.GATE), 0, 0, sigma=0.05),
               synth.UP: draw_planes(rng, synth.matrix_shape(cfg, synth.UP), 0, 0, sigma=0.05),
               synth.DOWN: draw_planes(rng, synth.matrix_shape(cfg, synth.DOWN), 112, 141)} for _ in range(P)]
    case = PlaneCase(oracle, binding, d, f, planes)
    assert case.layer.h_info() == (True, 0)
    x, ids, w = batch(rng, T, d, 2 * P, 2)
    y = case.gpu(x, ids, w)
    ok, worst = tolerance_ok(y, case.ref(x, ids, w))
    say("down exponents 112..141, half-precision H, T=%d: worst err / bound = %.3f" % (T, worst))
    assert ok, worst
    assert case.layer.h_info() == (True, 0)
    # the same layer forced to the wide form gives the same answer within the same bound
    wide = PlaneCase(oracle, binding, d, f, planes, wide_h=True)
    assert wide.layer.h_info()[0] is False
    ok, worst = tolerance_ok(wide.gpu(x, ids, w), case.ref(x, ids, w))
    assert ok, worst


@pytest.mark.parametrize("T", [16, 150])
def test_small_and_large_activations(oracle, binding, T):
    """Activations scaled by 2^-5 (H around 1e-4..1e-3 and below: half precision's subnormal range
    carries part of it) stay within the bound; scaled by 2^10 (|H| beyond 65504) the half-precision
    form saturates, says so, and stays finite, and the wide form is within the bound."""
    rng = np.random.RandomState(503)
    d, f, P = 256, 512, 2
    cfg = synth.LayerConfig("r", 4, d, f, 2, (1,))
    planes = [{which: draw_planes(rng, synth.matrix_shape(cfg, which), 0, 0, sigma=0.05) for which in W3}
              for _ in range(P)]
    case = PlaneCase(oracle, binding, d, f, planes)
    assert case.layer.h_info() == (True, 0)
    for scale in (1.0, 2.0 ** -5):
        x, ids, w = batch(rng, T, d, 2 * P, 2, scale=scale)
        ok, worst = tolerance_ok(case.gpu(x, ids, w), case.ref(x, ids, w))
        say("half-precision H, T=%d, x scaled by %g: worst err / bound = %.3f" % (T, scale, worst))
        assert ok, worst
    assert case.layer.h_info() == (True, 0)
    x, ids, w = batch(rng, T, d, 2 * P, 2, scale=2.0 ** 10)
    y = case.gpu(x, ids, w)
    assert np.isfinite(bits_to_f64(y)).all()
    assert case.layer.h_info()[1] > 0                            # saturation was counted
    wide = PlaneCase(oracle, binding, d, f, planes, wide_h=True)
    ok, worst = tolerance_ok(wide.gpu(x, ids, w), case.ref(x, ids, w))
    say("wide H, T=%d, x scaled by 2^10: worst err / bound = %.3f" % (T, worst))
    assert ok, worst


def dense_bits(rng, shape, exp_lo=None, exp_hi=None, sigma=None):
    """bf16 bit patterns: exponents uniform over [exp_lo, exp_hi] with random mantissas, or N(0, sigma); random
    signs, a sprinkle of exact zeros."""
    n = shape[0] * shape[1]
    if sigma is None:
        bits = ((rng.randint(exp_lo, exp_hi + 1, size=n) << 7) | rng.randint(0, 128, size=n)).astype(np.uint16)
    else:
        v = np.abs(rng.randn(n) * sigma).astype(np.float32)
        bits = ((v.view(np.uint32) + 0x8000) >> 16).astype(np.uint16)
    bits[rng.rand(n) < 0.01] = 0
    bits |= (rng.randint(0, 2, size=n).astype(np.uint16) << 15)
    return bits.reshape(shape)


@pytest.mark.parametrize("T", [80, 300])
def test_shared_experts_half_form_weight_ranges(oracle, binding, T):
    """Three shared experts on the tiled kernels (65 tokens and more).  The two of width 256 share a
    launch and hence a scale: one has ordinary down weights, the other's span 30 binades up to 2^73
    (everything of the first then sits far below the common top and is flushed -- the oracle's sum
    is dominated by the second in the same way).  The third, of width 128, spans 80 binades."""
    rng = np.random.RandomState(504)
    d, f, P = 256, 128, 1
    cfg = synth.LayerConfig("r", 2, d, f, 1, (1,))
    planes = [{which: draw_planes(rng, synth.matrix_shape(cfg, which), 0, 0, sigma=0.05) for which in W3}]
    for spans in (((None, None, 0.05), (None, None, 0.04), (None, None, 0.06)),     # ordinary weights, three experts
                  ((None, None, 0.05), (170, 200, None), (40, 120, None)),            # huge next to ordinary; 80 binades
                  ((20, 50, None), (20, 50, None), (1, 29, None))):                   # tiny: below half precision's own range
        shared = []
        for (lo, hi, sg), fs in zip(spans, (256, 256, 128)):
            shared.append((dense_bits(rng, (fs, d), sigma=0.05), dense_bits(rng, (fs, d), sigma=0.05),
                           dense_bits(rng, (d, fs), lo, hi, sg)))
        x, ids, w = batch(rng, T, d, 2, 1)
        ref = None
        for wide in (False, True):
            case = PlaneCase(oracle, binding, d, f, planes, wide_h=wide, shared=shared)
            ref = case.ref(x, ids, w) if ref is None else ref
            assert np.isfinite(ref).all()
            ok, worst = tolerance_ok(case.gpu(x, ids, w), ref)
            say("shared experts, down spans %s, %s H, T=%d: worst err / bound = %.3f" % (
                [sp[:2] if sp[2] is None else "N(0,%g)" % sp[2] for sp in spans], "wide" if wide else "half-precision", T, worst))
            assert ok, worst
            assert case.layer.h_info()[1] == 0


def test_shared_expert_saturation_is_counted(oracle, binding):
    """Packed pairs with small gate/up weights (their H stays small) and a shared expert with large
    ones: with activations scaled up, only the shared expert's H passes 65504.  The half-precision
    form saturates and counts it; the wide form of the same layer is within the bound.  Below 65
    tokens the shared experts run on the streaming kernels, which keep H wide: no saturation."""
    rng = np.random.RandomState(505)
    d, f, P = 256, 128, 1
    cfg = synth.LayerConfig("r", 2, d, f, 1, (1,))
    planes = [{which: draw_planes(rng, synth.matrix_shape(cfg, which), 0, 0, sigma=0.01) for which in W3}]
    shared = [(dense_bits(rng, (256, d), sigma=2.0), dense_bits(rng, (256, d), sigma=2.0), dense_bits(rng, (d, 256), sigma=0.05))]
    case = PlaneCase(oracle, binding, d, f, planes, shared=shared)
    x, ids, w = batch(rng, 100, d, 2, 1, scale=64.0)
    y = case.gpu(x, ids, w)
    assert np.isfinite(bits_to_f64(y)).all()
    assert case.layer.h_info()[1] > 0
    wide = PlaneCase(oracle, binding, d, f, planes, wide_h=True, shared=shared)
    ref = case.ref(x, ids, w)
    ok, worst = tolerance_ok(wide.gpu(x, ids, w), ref)
    say("shared expert, |H| beyond 65504, wide H: worst err / bound = %.3f" % worst)
    assert ok, worst
    assert wide.layer.h_info()[1] == 0
    small = PlaneCase(oracle, binding, d, f, planes, shared=shared)
    ok, worst = tolerance_ok(small.gpu(x[:40], ids[:40], w[:40]), ref[:40])
    say("shared expert, |H| beyond 65504, 40 tokens (streaming kernels): worst err / bound = %.3f" % worst)
    assert ok, worst
    assert small.layer.h_info()[1] == 0
