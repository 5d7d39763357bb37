"""GPU parity of the quantised variant (appendix "Combining PuzzleMoE with Quantization"):
the HIP codec through its C ABI against the CPU oracle, bit-exact (codes, scales, signs and the
base-3 mask numbers are integers; code * scale is exact in fp32)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def binding():
    from paper_2511_04805_amd import binding as b
    b.load()
    assert torch.cuda.is_available()
    return b


def say(msg):
    print(msg, flush=True)


def make_case(rows, cols, seed, paper_masks):
    rng = np.random.RandomState(seed)
    mag = np.abs(rng.randn(rows, cols)).astype(np.float32) * 0.02
    merged = (mag.view(np.uint32) >> 16).astype(np.uint16)
    if paper_masks:
        t = rng.randint(0, 3, size=(rows, cols))
        m0 = ((t == 0) | (t == 2)).astype(np.uint8)
        m1 = ((t == 1) | (t == 2)).astype(np.uint8)
    else:
        m0 = rng.randint(0, 2, size=(rows, cols)).astype(np.uint8)
        m1 = rng.randint(0, 2, size=(rows, cols)).astype(np.uint8)
    s0 = rng.randint(0, 2, size=(rows, cols)).astype(np.uint8)
    s1 = rng.randint(0, 2, size=(rows, cols)).astype(np.uint8)
    return merged, m0, m1, s0, s1


@pytest.mark.parametrize("shape,paper_masks", [((16, 128), True), ((48, 384), False), ((256, 1024), True),
                                               ((1408, 2048), False)])
def test_q_pack_unpack_bit_exact(oracle, binding, shape, paper_masks):
    say("q_pack/q_unpack shape=%s paper_masks=%s" % (shape, paper_masks))
    rows, cols = shape
    merged, m0, m1, s0, s1 = make_case(rows, cols, seed=rows + cols, paper_masks=paper_masks)
    # corner cases in the first group: an all-zero second row group, Inf and NaN magnitudes, a
    # negative input sign (ignored), exact ties of the quotient
    flat = merged.reshape(-1)
    flat[:6] = np.array([0x0000, 0x7F80, 0x7FC1, 0xBCA4, 0x3C00, 0x0001], dtype=np.uint16)
    m0.reshape(-1)[:6] = 1
    if cols >= 256:
        merged[0, 128:256] = 0
    dev = [torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).cuda() for a in (merged, m0, m1, s0, s1)]
    n_bad = torch.zeros(1, dtype=torch.int32, device="cuda")
    records, scales = binding.pzl_q_pack(*dev, n_non_finite=n_bad)
    torch.cuda.synchronize()
    q = oracle.q_quantise(merged, m0, m1, s0, s1)
    assert int(n_bad.item()) == q["n_bad"] == 2
    assert records.numel() == (rows // 16) * (cols // 32) * 424 + 8
    got_rec = binding.q_records_to_logical(records.cpu().numpy(), rows, cols)
    assert np.array_equal(got_rec, oracle.q_records(q))
    got_sc = binding.q_scales_to_logical(scales.cpu().numpy().view(np.uint16), rows, cols)
    assert np.array_equal(got_sc, q["scale"])
    for pos in (0, 1):
        out = binding.pzl_q_unpack(records, scales, pos, rows, cols)
        torch.cuda.synchronize()
        want = oracle.q_dequantise(q, pos)
        got = out.cpu().numpy().astype(np.float64)
        assert np.array_equal(got, want)
    # size of the stored pair against the 16-bit format: (424*8/512 + 16/128) / 16 bits
    stored = (records.numel() - 8) + scales.numel() * 2
    assert stored * 8 / (rows * cols) == pytest.approx(2 * oracle.q_bits_per_weight())


def test_q_pack_rejects_bad_shapes(binding):
    for rows, cols in ((16, 96), (8, 128), (0, 128)):
        merged = torch.zeros(max(rows, 1), max(cols, 1), dtype=torch.int16, device="cuda")
        planes = [torch.zeros(max(rows, 1), max(cols, 1), dtype=torch.uint8, device="cuda") for _ in range(4)]
        merged = merged[:rows, :cols].contiguous() if rows and cols else merged
        with pytest.raises((ValueError, binding.PzlError)):
            binding.pzl_q_pack(merged.reshape(rows, cols) if rows and cols else merged[:0].reshape(0, 128), *[
                p[:rows, :cols].contiguous() if rows and cols else p[:0].reshape(0, 128) for p in planes])


# ---------- the expert FFN over quantised pairs ----------

from paper_2511_04805_amd import synth                      # noqa: E402
from helpers import tolerance_ok                             # noqa: E402

W3 = (synth.GATE, synth.UP, synth.DOWN)


class QCase:
    """One quantised layer: the oracle's reconstructed fp64 experts and the library's Layer."""

    def __init__(self, cfg, oracle, binding, needed_experts=None):
        self.cfg, self.oracle, self.binding = cfg, oracle, binding
        self.emap = synth.expert_map(cfg, "adjacent")
        pair_of, pos_of = self.emap
        needed = set(range(cfg.n_experts)) if needed_experts is None else set(needed_experts)
        dev = {}
        self.w64 = {}                                        # (expert, which) -> fp64 matrix
        for p in range(cfg.n_pairs):
            for which in W3:
                pl = synth.pair_matrix(cfg, p, which)
                t = {k: torch.from_numpy(v.view(np.int16) if v.dtype == np.uint16 else v).cuda() for k, v in pl.items()}
                dev[p, which] = binding.pzl_q_pack(t["merged"], t["mask0"], t["mask1"], t["sign0"], t["sign1"])
                experts = [e for e in range(cfg.n_experts) if pair_of[e] == p and e in needed]
                if experts:
                    q = oracle.q_quantise(pl["merged"], pl["mask0"], pl["mask1"], pl["sign0"], pl["sign1"])
                    for e in experts:
                        self.w64[e, which] = oracle.q_dequantise(q, int(pos_of[e]))
        P = cfg.n_pairs
        self.layer = binding.Layer(cfg.d_model, cfg.d_ffn, pair_of, pos_of,
                                   [dev[p, synth.GATE] for p in range(P)], [dev[p, synth.UP] for p in range(P)],
                                   [dev[p, synth.DOWN] for p in range(P)], quantised=True)

    def gpu(self, x, ids, w):
        xt = torch.from_numpy(x.view(np.int16)).cuda()
        y = self.layer.pzl_moe_ffn(xt, torch.from_numpy(ids).cuda(), torch.from_numpy(w).cuda())
        torch.cuda.synchronize()
        return y.view(torch.int16).cpu().numpy().view(np.uint16)

    def ref(self, x, ids, w):
        any_e = next(iter(self.w64))[0]
        mats = [[self.w64.get((e, which), self.w64[any_e, which]) for e in range(self.cfg.n_experts)] for which in W3]
        return self.oracle.ffn_dense64(x, ids, w, *mats)


@pytest.fixture(scope="module")
def small_q(oracle, binding):
    cfg = synth.LayerConfig("quant_small", 8, 256, 512, 2, (64,), seed=4242)
    return QCase(cfg, oracle, binding)


@pytest.mark.parametrize("T", [1, 7, 33, 64, 150])
def test_q_ffn_small(small_q, T):
    """Element-wise parity over several token tiles, a ragged tail and (T = 150) several passes."""
    say("quantised FFN, small layer, T=%d" % T)
    cfg = small_q.cfg
    x = synth.tokens(cfg, T)
    ids, w = synth.routing(cfg, T)
    y = small_q.gpu(x, ids, w)
    y64 = small_q.ref(x, ids, w)
    ok, worst = tolerance_ok(y, y64)
    say("  worst err / bound = %.3f" % worst)
    assert ok, worst


def test_q_ffn_skewed_and_empty(small_q):
    """All tokens on one expert (many passes for one pair, none for the others); zero tokens."""
    cfg = small_q.cfg
    T = 70
    x = synth.tokens(cfg, T)
    ids = np.tile(np.array([[3, 3]], dtype=np.int32), (T, 1))            # duplicate ids add up
    w = np.full((T, 2), 0.5, dtype=np.float32)
    y = small_q.gpu(x, ids, w)
    ok, worst = tolerance_ok(y, small_q.ref(x, ids, w))
    assert ok, worst
    y0 = small_q.layer.pzl_moe_ffn(torch.empty(0, cfg.d_model, dtype=torch.bfloat16, device="cuda"),
                                   torch.empty(0, 2, dtype=torch.int32, device="cuda"),
                                   torch.empty(0, 2, dtype=torch.float32, device="cuda"))
    assert y0.shape == (0, cfg.d_model)


def test_q_ffn_refuses_batches_beyond_two_sweeps(small_q, binding):
    """No tiled kernel for the quantised format: a batch of more than 64 (token, choice) entries per
    expert on average is refused (PZL_EINVAL) instead of re-streaming the weights many times."""
    cfg = small_q.cfg                                   # 8 experts, top-2: the limit is 256 tokens
    for T, ok in ((256, True), (257, False), (4096, False)):
        x = torch.zeros(T, cfg.d_model, dtype=torch.bfloat16, device="cuda")
        ids = torch.zeros(T, 2, dtype=torch.int32, device="cuda")
        ids[:, 1] = 1
        w = torch.full((T, 2), 0.5, dtype=torch.float32, device="cuda")
        if ok:
            small_q.layer.pzl_moe_ffn(x, ids, w)
            torch.cuda.synchronize()
        else:
            with pytest.raises(binding.PzlError) as e:
                small_q.layer.pzl_moe_ffn(x, ids, w)
            assert e.value.rc == binding.PZL_EINVAL


def test_q_layer_rejects_bad_shapes(binding):
    """d_model / d_ffn must be multiples of 128 for the quantised format."""
    dummy = (torch.zeros(8, dtype=torch.uint8, device="cuda"), torch.zeros(8, dtype=torch.int16, device="cuda"))
    with pytest.raises((ValueError, binding.PzlError)):
        binding.Layer(96, 256, [0, 0], [0, 1], [dummy], [dummy], [dummy], quantised=True)


def test_q_ffn_mixtral_shaped_decode(oracle, binding):
    """The benchmark's layer shape and batch (Mixtral-8x7B-shaped, T = 64) in the quantised format,
    in the launch configuration bench.py times.  The oracle runs on rows picked from the call's own
    routing tables: of every expert its first, middle and last slot and the slots on either side
    of its 16-token fragment borders (every expert is reconstructed in fp64: 0.47 GB per matrix)."""
    from test_gpu_configs import rows_reaching_every_tile
    cfg = synth.CONFIGS["mixtral_decode"]
    T = 64
    x = synth.tokens(cfg, T)
    ids, w = synth.routing(cfg, T)
    case = QCase(cfg, oracle, binding)
    y = case.gpu(x, ids, w)
    rows, units, covered = rows_reaching_every_tile(case.layer.routing_tables(T, cfg.top_k), T)
    say("quantised FFN, %s T=%d: %d streamed experts, all reached at their edges by %d rows" % (cfg.name, T, units, len(rows)))
    assert units == cfg.n_experts and covered == units and len(rows) >= 12
    y64 = case.ref(x[rows], ids[rows], w[rows])
    ok, worst = tolerance_ok(y[rows], y64)
    say("  worst err / bound = %.3f" % worst)
    assert ok, worst
    assert np.isfinite((y.astype(np.uint32) << 16).view(np.float32)).all()


def test_q_ffn_mixed_layer_with_unmerged_and_shared_experts(oracle, binding):
    """Quantised pairs next to routed experts kept unmerged (25 % compression, Sec. 4.1) and a
    dense shared expert: the routed part against the fp64-weights oracle, the shared part
    against the bf16 oracle's dense path, summed."""
    cfg = synth.LayerConfig("quant_mixed", 6, 256, 384, 2, (40,), shared_d_ffn=(256,), seed=77, n_unmerged=2)
    pair_of, pos_of = synth.expert_map(cfg, "adjacent")
    T = 40
    x = synth.tokens(cfg, T)
    ids, w = synth.routing(cfg, T)
    qdev, w64 = {}, {}
    for p in range(cfg.n_pairs):
        for which in W3:
            pl = synth.pair_matrix(cfg, p, which)
            t = {k: torch.from_numpy(v.view(np.int16) if v.dtype == np.uint16 else v).cuda() for k, v in pl.items()}
            qdev[p, which] = binding.pzl_q_pack(t["merged"], t["mask0"], t["mask1"], t["sign0"], t["sign1"])
            q = oracle.q_quantise(pl["merged"], pl["mask0"], pl["mask1"], pl["sign0"], pl["sign1"])
            for e in range(cfg.n_experts):
                if pair_of[e] == p:
                    w64[e, which] = oracle.q_dequantise(q, int(pos_of[e]))
    dense_gpu = []
    for j in range(cfg.n_unmerged):
        mats = [synth.unmerged_matrix_t(cfg, j, which) for which in W3]
        dense_gpu.append(tuple(binding.pzl_tile_dense(m.cuda()) for m in mats))
        e = [e for e in range(cfg.n_experts) if pair_of[e] == -1 - j][0]
        for which, m in zip(W3, mats):
            w64[e, which] = (synth._np_bits(m).astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    shared_mats = [synth.shared_matrix_t(cfg, 0, which) for which in W3]
    shared_gpu = [tuple(binding.pzl_tile_dense(m.cuda()) for m in shared_mats) + (cfg.shared_d_ffn[0],)]
    P = cfg.n_pairs
    layer = binding.Layer(cfg.d_model, cfg.d_ffn, pair_of, pos_of,
                          [qdev[p, synth.GATE] for p in range(P)], [qdev[p, synth.UP] for p in range(P)],
                          [qdev[p, synth.DOWN] for p in range(P)], shared=shared_gpu, dense=dense_gpu,
                          quantised=True)
    y = layer.pzl_moe_ffn(torch.from_numpy(x.view(np.int16)).cuda(), torch.from_numpy(ids).cuda(),
                          torch.from_numpy(w).cuda())
    torch.cuda.synchronize()
    y = y.view(torch.int16).cpu().numpy().view(np.uint16)
    y_routed = oracle.ffn_dense64(x, ids, w, *[[w64[e, which] for e in range(cfg.n_experts)] for which in W3])
    no_ids = np.zeros((T, 0), dtype=np.int32)
    y_shared, _ = oracle.moe_ffn(x, no_ids, np.zeros((T, 0), dtype=np.float32),
                                 np.full(cfg.n_experts, -1, dtype=np.int32), np.zeros(cfg.n_experts, np.uint8),
                                 [], [], [], shared=[tuple(synth._np_bits(m) for m in shared_mats)])
    ok, worst = tolerance_ok(y, y_routed + y_shared)
    say("mixed quantised layer: worst err / bound = %.3f" % worst)
    assert ok, worst
