"""GPU parity: the HIP library through its C ABI against the CPU oracle.

Bit-exact for pack / unpack (integer work); |y - y_ref| <= 1e-2 * max(|y_ref|, rms of the row)
for the FFN (bf16 x bf16 products, fp32 accumulation, H kept as hi+lo bf16, y rounded to bf16
once, against the oracle's fp64).  The rounding of y alone is up to 2^-8 relative, i.e. 0.39 of
the bound.
"""
import numpy as np
import pytest
import torch

from paper_2511_04805_amd import synth
from helpers import Case, bits_to_f64, tolerance_ok

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def binding():
    from paper_2511_04805_amd import binding as b
    b.load()
    assert torch.cuda.is_available()
    return b


def say(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("shape", [(16, 32), (48, 96), (256, 128), (1408, 2048)])
def test_pack_unpack_bit_exact(oracle, binding, shape):
    say("pack/unpack shape=%s" % (shape,))
    cfg = synth.LayerConfig("codec", 2, 32, 32, 1, (1,), seed=77)
    pl = synth.pair_matrix(cfg, 0, synth.GATE, shape=shape)
    # sprinkle the corner cases: zero, below the band, top of the band, out of range, negative input
    flat = pl["merged"].reshape(-1)
    flat[:8] = np.array([0x0000, 0x0001, 0x3581, 0x37FF, 0x47FF, 0x4800, 0x7F80, 0xBCA4], dtype=np.uint16)
    dev = {k: torch.from_numpy(v.view(np.int16) if v.dtype == np.uint16 else v).cuda() for k, v in pl.items()}
    n_bad = torch.zeros(1, dtype=torch.int32, device="cuda")
    packed = binding.pzl_pack(dev["merged"], dev["mask0"], dev["mask1"], dev["sign0"], dev["sign1"],
                              n_out_of_range=n_bad)
    torch.cuda.synchronize()
    want, bad = oracle.pack(pl["merged"], pl["mask0"], pl["mask1"], pl["sign0"], pl["sign1"])
    assert int(n_bad.item()) == bad == 2
    assert packed.numel() * 2 == binding.pzl_packed_bytes(*shape)
    got = binding.tiled_to_logical(packed.cpu().numpy().view(np.uint16), *shape)
    assert np.array_equal(got, want)
    for pos in (0, 1):
        out = binding.pzl_unpack(packed, pos, *shape)
        torch.cuda.synchronize()
        assert np.array_equal(out.view(torch.int16).cpu().numpy().view(np.uint16), oracle.unpack(want, pos))


def test_unpack_all_words(oracle, binding):
    """Every 16-bit word through the GPU decode, both positions (Algorithm 1 is total)."""
    words = np.arange(65536, dtype=np.uint16).reshape(64, 1024)
    # lay the words out so that logical order == value order
    tiled = np.empty(65536, dtype=np.uint16)
    r, c = np.divmod(np.arange(65536), 1024)
    tiled[((r // 16) * 32 + c // 32) * 512 + (((c % 32) // 8) * 16 + r % 16) * 8 + c % 8] = words.reshape(-1)
    t = torch.from_numpy(tiled.view(np.int16)).cuda()
    for pos in (0, 1):
        out = binding.pzl_unpack(t, pos, 64, 1024)
        torch.cuda.synchronize()
        assert np.array_equal(out.view(torch.int16).cpu().numpy().view(np.uint16), oracle.unpack(words, pos))


def test_tile_dense_roundtrip(binding):
    a = torch.arange(64 * 96, dtype=torch.int16, device="cuda").reshape(64, 96)
    t = binding.pzl_tile_dense(a)
    torch.cuda.synchronize()
    assert np.array_equal(binding.tiled_to_logical(t.cpu().numpy(), 64, 96), a.cpu().numpy())


def check(case, T, label, ids=None, w=None, x=None, ref_rows=None):
    cfg = case.cfg
    say("moe_ffn %s T=%d" % (label, T))
    x = synth.tokens(cfg, T) if x is None else x
    if ids is None:
        ids, w = synth.routing(cfg, T)
    y = case.gpu(x, ids, w)
    rows = np.arange(T) if ref_rows is None else np.asarray(ref_rows)
    y64, _ = case.ref(x[rows], ids[rows], w[rows])
    ok, worst = tolerance_ok(y[rows], y64)
    say("  worst err / bound = %.3f" % worst)
    assert ok, worst
    return y, y64


def test_tiny_config(oracle, binding):
    case = Case(synth.CONFIGS["tiny"], oracle, binding)
    y, y64 = check(case, 8, "tiny")
    assert np.abs(y64).max() > 0


SMALL = synth.LayerConfig("small", 6, 192, 352, 2, (40,), shared_d_ffn=(96, 160), seed=31)


@pytest.fixture(scope="module")
def small_case(oracle, binding):
    return Case(SMALL, oracle, binding, emap_mode="random")


@pytest.mark.parametrize("T", [1, 2, 7, 16, 17, 40, 100, 300])
def test_small_layer_token_counts(small_case, T):
    """Ragged tails, one/several token tiles per expert, several passes, shared experts."""
    check(small_case, T, "small")


def test_edge_cases(small_case, binding):
    cfg, case = SMALL, small_case
    T = 24
    x = synth.tokens(cfg, T)
    ids, w = synth.routing(cfg, T)
    # an expert with no tokens, a pair with no tokens
    ids0 = ids.copy(); ids0[ids0 == 3] = 0
    check(case, T, "expert-empty", ids=ids0, w=w, x=x)
    emap = case.emap
    only = np.array([e for e in range(cfg.n_experts) if emap[0][e] == 0], dtype=np.int32)
    ids1 = np.tile(only[None, :], (T, 1)).astype(np.int32)
    check(case, T, "single-pair", ids=ids1, w=w, x=x)
    # duplicate ids within a token add up
    ids2 = np.repeat(ids[:, :1], 2, axis=1).copy()
    check(case, T, "duplicates", ids=ids2, w=w, x=x)
    # ids outside [0,E) are ignored
    ids3 = ids.copy(); ids3[::3, 1] = cfg.n_experts + 5; ids3[1::3, 1] = -1
    y = case.gpu(x, ids3, w)
    w3 = w.copy(); w3[::3, 1] = 0; w3[1::3, 1] = 0
    y64, _ = case.ref(x, np.where((ids3 < 0) | (ids3 >= cfg.n_experts), 0, ids3).astype(np.int32), w3)
    assert tolerance_ok(y, y64)[0]
    # k = 0: no routed expert at all, y is the sum of the shared experts
    ids4 = np.zeros((T, 0), dtype=np.int32); w4 = np.zeros((T, 0), dtype=np.float32)
    y = case.layer.pzl_moe_ffn(torch.from_numpy(x.view(np.int16)).cuda(), torch.from_numpy(ids4).cuda(),
                               torch.from_numpy(w4).cuda())
    torch.cuda.synchronize()
    y64, _ = case.ref(x, ids4, w4)
    assert np.abs(y64).max() > 0 and tolerance_ok(y.view(torch.int16).cpu().numpy().view(np.uint16), y64)[0]
    # T = 0 is a no-op, and results are reproducible bit for bit
    empty = case.layer.pzl_moe_ffn(torch.empty(0, cfg.d_model, dtype=torch.bfloat16, device="cuda"),
                                   torch.empty(0, 2, dtype=torch.int32, device="cuda"),
                                   torch.empty(0, 2, dtype=torch.float32, device="cuda"))
    assert empty.shape == (0, cfg.d_model)
    ya = case.gpu(x, ids, w); yb = case.gpu(x, ids, w)
    assert np.array_equal(ya, yb)
    # token-permutation equivariance, exactly
    perm = np.random.RandomState(0).permutation(T)
    yp = case.gpu(x[perm], ids[perm], w[perm])
    assert np.array_equal(yp, ya[perm])


def test_error_codes(small_case, binding):
    cfg, case = SMALL, small_case
    lib = binding.load()
    x = torch.zeros(4, cfg.d_model, dtype=torch.bfloat16, device="cuda")
    ids = torch.zeros(4, 2, dtype=torch.int32, device="cuda")
    w = torch.zeros(4, 2, dtype=torch.float32, device="cuda")
    small_ws = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(binding.PzlError) as ei:
        case.layer.pzl_moe_ffn(x, ids, w, workspace=small_ws)
    assert ei.value.rc == binding.PZL_ENOSPC
    with pytest.raises(binding.PzlError) as ei:
        binding.pzl_unpack(torch.zeros(16 * 32, dtype=torch.int16, device="cuda"), 2, 16, 32)
    assert ei.value.rc == binding.PZL_EINVAL
    with pytest.raises(binding.PzlError) as ei:
        binding.pzl_unpack(torch.zeros(15 * 32, dtype=torch.int16, device="cuda"), 0, 15, 32)
    assert ei.value.rc == binding.PZL_EINVAL
    with pytest.raises(binding.PzlError):      # pair map that is not a 2-to-1 cover
        binding.Layer(cfg.d_model, cfg.d_ffn, [0, 0, 0, 1, 2, 2], [0, 1, 0, 1, 0, 1],
                      [case.packed_gpu[p, synth.GATE] for p in range(3)],
                      [case.packed_gpu[p, synth.UP] for p in range(3)],
                      [case.packed_gpu[p, synth.DOWN] for p in range(3)])
    assert lib.pzl_moe_ffn_workspace_bytes(case.layer._h, -1, 2) == 0
    # a workspace sized for max_tokens serves every smaller batch: the size never shrinks with T
    sizes = [lib.pzl_moe_ffn_workspace_bytes(case.layer._h, T, 2) for T in range(0, 1200)]
    assert all(b >= a for a, b in zip(sizes, sizes[1:])) and sizes[1] > 0
    # a batch beyond the documented size limits (T * k * d_ffn < 2^30) is refused, not mis-addressed
    too_many = (1 << 30) // (2 * cfg.d_ffn) + 1
    assert lib.pzl_moe_ffn_workspace_bytes(case.layer._h, too_many, 2) == 0
    assert lib.pzl_moe_ffn_workspace_bytes(case.layer._h, too_many - 2, 2) > 0
    rc = lib.pzl_moe_ffn(case.layer._h, x.data_ptr(), ids.data_ptr(), w.data_ptr(), too_many, 2,
                         x.data_ptr(), small_ws.data_ptr(), 256, None)
    assert rc == binding.PZL_EINVAL


@pytest.mark.parametrize("shape,tau", [((64, 96), 0.4), ((256, 512), 0.4), ((1408, 2048), 0.25)])
def test_merge_pack_bit_exact(oracle, binding, shape, tau):
    """Offline dual-mask merge fused with pack (Eqs. 1-5 -> packed word) against oracle merge + pack."""
    say("merge_pack shape=%s tau=%s" % (shape, tau))
    rows, cols = shape
    g = torch.Generator().manual_seed(rows + cols)
    to_bits = lambda t: t.to(torch.bfloat16).view(torch.int16)
    wi = to_bits(torch.randn(rows, cols, generator=g) * 0.02)
    wj = to_bits(torch.randn(rows, cols, generator=g) * 0.02)
    # corner cases: both zero, equal magnitudes with opposite sign, one zero, -0
    wi.view(-1)[:6] = torch.tensor([0, 0x3CA4, 0x3CA4, 0, -32768, 0x0001], dtype=torch.int16)
    wj.view(-1)[:6] = torch.tensor([0, -17244, 0x3CA5, 0x3CA4, 0x3CA4, 0x0001], dtype=torch.int16)   # -17244 = 0xBCA4
    ni = (torch.rand(cols, generator=g) + 0.5).float()
    nj = (torch.rand(cols, generator=g) + 0.5).float()
    ref = oracle.merge(wi.numpy().view(np.uint16), wj.numpy().view(np.uint16), ni.numpy(), nj.numpy(), tau)
    want, bad = oracle.pack(ref["merged"], ref["mask0"], ref["mask1"], ref["sign0"], ref["sign1"])
    n_sim = torch.zeros(1, dtype=torch.int32, device="cuda")
    n_bad = torch.zeros(1, dtype=torch.int32, device="cuda")
    packed = binding.pzl_merge_pack(wi.cuda(), wj.cuda(), ni.cuda(), nj.cuda(), tau, n_similar=n_sim,
                                    n_out_of_range=n_bad)
    torch.cuda.synchronize()
    got = binding.tiled_to_logical(packed.cpu().numpy().view(np.uint16), rows, cols)
    assert np.array_equal(got, want)
    assert int(n_sim.item()) == ref["n_similar"] and int(n_bad.item()) == bad == 0
    # and the packed pair decodes to each expert's reconstruction (Eq. 6)
    for pos in (0, 1):
        out = binding.pzl_unpack(packed, pos, rows, cols)
        torch.cuda.synchronize()
        assert np.array_equal(out.view(torch.int16).cpu().numpy().view(np.uint16), oracle.unpack(want, pos))


# A layer whose sizes allow the tiled (MFMA) path: d and f multiples of 64.
TILED = synth.LayerConfig("tiled", 4, 256, 384, 2, (600,), shared_d_ffn=(128,), seed=41)


@pytest.fixture(scope="module")
def tiled_case(oracle, binding):
    return Case(TILED, oracle, binding, emap_mode="random")


@pytest.mark.parametrize("T", [192, 200, 333, 600, 1100])
def test_tiled_path_token_counts(tiled_case, T):
    """>= 96 slots per expert: tiled kernels; ragged token tiles, several tiles per expert; the
    dense shared expert runs on the tiled kernels too (from 96 tokens), its tokens cut into several
    small tiles with a ragged last one."""
    check(tiled_case, T, "tiled")


@pytest.mark.parametrize("T", [70, 100, 180])
def test_hybrid_path_mixed_pair_sizes(tiled_case, T):
    """From 20 slots per expert on average both paths are launched and the grouping kernel assigns
    each PAIR to one of them (tiled kernels if one of its experts has more than 32 tokens).
    Routing is set by hand: one pair holds a hot expert (T tokens, several token tiles) and a
    partner with a few tokens (a small tile); the other pair holds an expert with T/8 tokens and an
    empty one and stays with the streaming kernels."""
    cfg = TILED
    pair_of = np.asarray(tiled_case.emap[0])
    a, b = np.where(pair_of == 0)[0]
    c, d = np.where(pair_of == 1)[0]
    x = synth.tokens(cfg, T)
    _, w = synth.routing(cfg, T)
    ids = np.empty((T, 2), dtype=np.int32)
    ids[:, 0] = a                                                # hot expert
    ids[:, 1] = np.where(np.arange(T) % 8 == 0, c, np.where(np.arange(T) % 8 == 1, b, a))
    counts = np.bincount(ids.ravel(), minlength=cfg.n_experts)
    assert T * cfg.top_k >= 20 * cfg.n_experts
    assert counts[a] > 64 and 0 < counts[b] < 33 and 0 < counts[c] < 33 and counts[d] == 0
    check(tiled_case, T, "hybrid", ids=ids, w=w, x=x)


# wide and shallow: 88 row groups in the gate/up stage, so that a handful of token tiles fills the chip
WIDE = synth.LayerConfig("wide", 8, 128, 11264, 2, (256,), seed=43)


@pytest.fixture(scope="module")
def wide_case(oracle, binding):
    return Case(WIDE, oracle, binding, emap_mode="random")


@pytest.mark.parametrize("counts", [(40, 50, 64, 1, 33, 33, 20, 7), (96, 96, 97, 5, 48, 2, 1, 60),
                                    (33, 1, 30, 31, 0, 50, 10, 10), (100, 64, 0, 90, 64, 16, 17, 15)])
def test_tiled_path_pair_tiles(wide_case, counts):
    """A tiled pair both of whose experts have 1..96 tokens gets ONE token tile for both (the
    packed words are loaded once and decoded for both positions) if that shortens the launch
    enough; 97 tokens, or an empty partner, give ordinary tiles, and in the last case too few pairs
    qualify, so none shares a tile.  Expert loads are set by hand: counts = (pair 0 pos 0, pair 0
    pos 1, pair 1 pos 0, ...)."""
    cfg, case = WIDE, wide_case
    pair_of, pos_of = np.asarray(case.emap[0]), np.asarray(case.emap[1])
    experts = [int(np.where((pair_of == p) & (pos_of == q))[0][0]) for p in range(4) for q in (0, 1)]
    flat = np.concatenate([np.full(c, e, dtype=np.int32) for e, c in zip(experts, counts)])
    if flat.size % 2:
        flat = np.concatenate([flat, np.array([-1], dtype=np.int32)])       # an ignored id pads the last token
    np.random.RandomState(sum(counts)).shuffle(flat)
    T = flat.size // 2
    ids = flat.reshape(T, 2)
    x = synth.tokens(cfg, T)
    _, w = synth.routing(cfg, T)
    assert flat.size >= 20 * cfg.n_experts and max(counts) >= 33          # both paths launched, pairs tiled
    y = case.gpu(x, ids, w)
    y64, _ = case.ref(x, np.where(ids < 0, 0, ids).astype(np.int32), np.where(ids < 0, 0.0, w).astype(np.float32))
    ok, worst = tolerance_ok(y, y64)
    say("  pair tiles %s: worst err / bound = %.3f" % (counts, worst))
    assert ok, worst


def _ids_with_counts(cfg, counts, seed):
    """A (T, 2) id table in which expert e appears exactly counts[e] times (a token may name an
    expert twice; an ignored id pads an odd total)."""
    flat = np.concatenate([np.full(c, e, dtype=np.int32) for e, c in enumerate(counts)])
    if flat.size % 2:
        flat = np.concatenate([flat, np.array([-1], dtype=np.int32)])
    np.random.RandomState(seed).shuffle(flat)
    return flat.reshape(flat.size // 2, 2)


def _check_counts(case, counts, label):
    cfg = case.cfg
    ids = _ids_with_counts(cfg, counts, sum(counts))
    T = ids.shape[0]
    x = synth.tokens(cfg, T)
    _, w = synth.routing(cfg, T)
    y = case.gpu(x, ids, w)
    y64, _ = case.ref(x, np.where(ids < 0, 0, ids).astype(np.int32), np.where(ids < 0, 0.0, w).astype(np.float32))
    ok, worst = tolerance_ok(y, y64)
    say("  %s %s: worst err / bound = %.3f" % (label, counts, worst))
    assert ok, worst


@pytest.mark.parametrize("counts", [(140, 170, 200, 270), (272, 129, 233, 144), (257, 161, 193, 225), (280, 150, 190, 0)])
def test_tiled_path_odd_fragment_counts(tiled_case, counts):
    """Tiles of 9, 11, 13, 15 and 17 token fragments have loops of their own that leave out the
    matrix instructions of the padding fragment: expert loads set by hand so that every one of them
    (and, last case, their even neighbours 18, 10, 12) runs in both stages, first and last token of
    the last fragment included."""
    frags = sorted((c + 15) // 16 for c in counts if c)
    assert counts[3] == 0 or all(f % 2 == 1 and f >= 9 for f in frags), frags
    _check_counts(tiled_case, counts, "odd tiles")


def test_odd_fragment_counts_two_plane_h_and_unmerged_experts(oracle, binding):
    """The same for the two-plane form of H (two groups per fragment and K step in the down stage)
    and for routed experts kept unmerged (dense weights, identity decode)."""
    cfg = synth.LayerConfig("odd_wide", 6, 256, 384, 2, (600,), shared_d_ffn=(128,), seed=77, n_unmerged=2)
    case = Case(cfg, oracle, binding, emap_mode="random", wide_h=True)
    _check_counts(case, (140, 170, 200, 270, 233, 129), "odd tiles, wide H, unmerged")


def test_persistent_launches_odd_fragment_counts(oracle, binding):
    """The same loops in the persistent launch form (32 routing keys or more, about one tile per
    expert): a few experts with 129-272 tokens among many small ones."""
    cfg = synth.LayerConfig("many_odd", 32, 128, 256, 2, (64,), seed=73)
    case = Case(cfg, oracle, binding, emap_mode="random")
    counts = [3] * 32
    for e, c in ((1, 136), (6, 175), (7, 201), (12, 239), (20, 262), (21, 272), (30, 130), (31, 96)):
        counts[e] = c
    plan = binding.pzl_moe_ffn_plan(cfg.n_experts, cfg.d_model, cfg.d_ffn, (sum(counts) + 1) // 2, 2)
    assert plan["hybrid"] and plan["persistent"], plan
    _check_counts(case, tuple(counts), "persistent odd tiles")


def test_tiled_path_skewed_routing(tiled_case):
    """One hot expert (several full token tiles), one expert with a single token, one with none."""
    cfg = TILED
    T = 700
    x = synth.tokens(cfg, T)
    ids, w = synth.routing(cfg, T)
    ids[:, 0] = 2
    ids[:, 1] = 0
    ids[5, 1] = 1                    # expert 1: one token; expert 3: none
    check(tiled_case, T, "tiled-skewed", ids=ids.astype(np.int32), w=w, x=x)


def test_merged_layer_end_to_end(oracle, binding):
    """The paper's pipeline on synthetic experts: dense pair -> dual-mask merge (tau = 0.4) -> packed
    pair -> routed FFN.  Masks have the paper's structure: never both clear, density ~0.74."""
    cfg = synth.LayerConfig("merged", 8, 256, 448, 2, (300,), seed=53)
    case = Case(cfg, oracle, binding, emap_mode="random", from_merge=0.4)
    n_elems = cfg.n_pairs * 3 * cfg.d_model * cfg.d_ffn
    assert abs(case.n_similar / n_elems - 0.4845) < 0.005            # Lemma 3.1 at tau = 0.4
    words = case.packed_cpu[0, synth.GATE]
    m0, m1 = (words >> 13) & 1, (words >> 12) & 1
    assert np.all((m0 | m1) == 1) and abs(float(m0.mean()) - 0.742) < 0.01
    for T in (5, 40, 500):                                           # streaming and tiled kernels
        check(case, T, "merged-layer")


# 25 % compression (Sec. 4.1): only half of the routed experts are merged, the rest stay dense.
MIXED = synth.LayerConfig("mixed", 8, 256, 384, 2, (64,), shared_d_ffn=(128,), seed=61, n_unmerged=4)


@pytest.fixture(scope="module")
def mixed_case(oracle, binding):
    assert MIXED.n_pairs == 2
    return Case(MIXED, oracle, binding, emap_mode="random")


@pytest.mark.parametrize("T", [1, 9, 64, 150, 800, 1100])
def test_mixed_layer_unmerged_experts(mixed_case, T):
    """Packed pairs and unmerged dense experts in one layer, on the streaming kernels (T <= 150)
    and on the tiled kernels (T >= 800)."""
    check(mixed_case, T, "mixed")


def test_many_experts_mixed_layer_persistent_launches(oracle, binding):
    """40 routed experts, 8 of them kept unmerged: with 32 or more expert slots and about one tile
    per expert the tiled launches are persistent (workgroups draw their tiles), for the packed pairs
    and for the dense experts alike.  Zipf routing gives a few busy experts (tiled) and many idle
    ones (streamed or empty); the tiled kernels run on the layer's tile stream."""
    cfg = synth.LayerConfig("many_mixed", 40, 128, 384, 3, (300,), shared_d_ffn=(128,), routing="zipf",
                            seed=71, n_unmerged=8)
    case = Case(cfg, oracle, binding, emap_mode="random")
    for T in (120, 300, 700):
        ids, _ = synth.routing(cfg, T)
        counts = np.bincount(ids.ravel(), minlength=cfg.n_experts)
        assert T * cfg.top_k >= 8 * cfg.n_experts and counts.max() >= 33
        check(case, T, "many-mixed")


def test_grouping_inside_the_gateup_kernel_at_its_limits(oracle, binding):
    """Small streaming-only batches have no grouping kernel: the gate/up kernel sorts the (token,
    choice) list itself (at most 512 entries, 128 routing keys).  30 experts with 4 kept unmerged
    (whose launch reads the tables the packed launch wrote): 512 entries (the limit), 514 (one
    over: the grouping kernel runs), ids out of range and every token on one expert."""
    cfg = synth.LayerConfig("group_in_kernel", 30, 128, 256, 2, (256,), shared_d_ffn=(128,), seed=79, n_unmerged=4)
    case = Case(cfg, oracle, binding, emap_mode="random")
    for T, fused in ((256, 1), (257, 0), (3, 1)):
        plan = binding.pzl_moe_ffn_plan(cfg.n_experts, cfg.d_model, cfg.d_ffn, T, cfg.top_k,
                                        shared_d_ffn=cfg.shared_d_ffn, n_unmerged=cfg.n_unmerged)
        assert plan["grouping_in_kernel"] == fused and not plan["hybrid"]
        check(case, T, "grouping in the gate/up kernel" if fused else "grouping kernel")
        tab = case.layer.routing_tables(T, cfg.top_k)            # stable: a key's slots are in ascending flat order
        ids, _ = synth.routing(cfg, T)
        if fused:
            flat_of_slot = np.empty(T * cfg.top_k, dtype=np.int64)
            flat_of_slot[tab["slot_of"].ravel()] = np.arange(T * cfg.top_k)
            for q in range(tab["n_keys"]):
                seg = flat_of_slot[tab["first_slot"][q]:tab["first_slot"][q + 1]]
                assert np.all(np.diff(seg) > 0)
    T = 200
    x = synth.tokens(cfg, T)
    ids, w = synth.routing(cfg, T)
    ids[::7, 1] = cfg.n_experts + 3                               # ignored ids
    ids[5, 0] = -1
    y = case.gpu(x, ids, w)
    tab = case.layer.routing_tables(T, cfg.top_k)
    assert np.array_equal(tab["slot_of"] < 0, (ids < 0) | (ids >= cfg.n_experts))
    keep = (ids >= 0) & (ids < cfg.n_experts)
    y64, _ = case.ref(x, np.where(keep, ids, 0), np.where(keep, w, 0.0).astype(np.float32))
    ok, worst = tolerance_ok(y, y64)
    say("  ignored ids: worst err / bound = %.3f" % worst)
    assert ok, worst
    ids1 = np.zeros((T, 2), dtype=np.int32)
    ids1[:, 1] = 1 + (np.arange(T) % 3)                           # expert 0 gets every token: 200 tokens, 7 sweeps
    check(case, T, "one busy expert", ids=ids1, w=w, x=x)


def test_many_experts_small_batch_hot_expert(oracle, binding):
    """Small batches of a 64-expert layer (fewer than 6 slots per expert on average: streaming
    kernels only) in which every token picks the same first expert: its pair needs 2 to 4 sweeps of
    32 tokens, which the launch spreads over 2 or 3 workgroups per row block (the first of them
    takes sweeps 0 and 3 at 100 tokens), next to pairs and unmerged experts with one sweep or none."""
    cfg = synth.LayerConfig("many_hot", 64, 128, 384, 3, (100,), shared_d_ffn=(128,), routing="zipf",
                            seed=73, n_unmerged=8)
    case = Case(cfg, oracle, binding, emap_mode="random")
    pair = np.asarray(case.emap[0])
    hot_packed = int(np.where(pair >= 0)[0][0])
    hot_dense = int(np.where(pair < 0)[0][0])
    for T, hot in ((48, hot_packed), (100, hot_packed), (100, hot_dense)):
        assert T * cfg.top_k < 6 * cfg.n_experts
        x = synth.tokens(cfg, T)
        ids, w = synth.routing(cfg, T)
        for t in range(T):                              # the hot expert first, the others kept distinct from it
            ids[t, 0] = hot
            for j in range(1, cfg.top_k):
                if ids[t, j] == hot:
                    ids[t, j] = (hot + 1 + j) % cfg.n_experts
        counts = np.bincount(ids.ravel(), minlength=cfg.n_experts)
        assert counts[hot] == T
        check(case, T, "many-hot", ids=ids, w=w, x=x)


def test_router_topk_nonfinite_logits(oracle, binding):
    """A token with a NaN logit and infinite ones, and a token with one infinite logit: the
    chosen experts still equal the oracle's scan (nothing is larger than a NaN and a NaN is larger
    than nothing); the other tokens are unaffected."""
    T, d, E, k = 12, 256, 16, 3
    g = torch.Generator().manual_seed(5)
    x = torch.randn(T, d, generator=g).to(torch.bfloat16)
    wr = (torch.randn(E, d, generator=g) * 0.05).to(torch.bfloat16)
    # (a chain of finite inputs can overflow to +-inf but never yields a NaN: the product inside an
    # fma is not rounded; so the NaN comes from an infinite input)
    x[2, 0] = float("inf"); wr[0, 0] = 0.0               # token 2: expert 0 NaN (inf * 0), the others +-inf
    bx, bw = 1.0e38, 1.0e36                              # bx * bw overflows fp32; N(0,1) * bw and bx * 0.05 do not
    x[7, 3] = bx; wr[9, 3] = bw                          # token 7, expert 9: +inf; other tokens: large but finite
    ids, w = binding.pzl_router_topk(x.cuda(), wr.cuda(), k)
    torch.cuda.synchronize()
    ids_ref, w_ref, logits = oracle.router_topk(x.view(torch.int16).numpy().view(np.uint16),
                                                wr.view(torch.int16).numpy().view(np.uint16), k)
    assert np.isnan(logits[2, 0]) and np.isinf(logits[2, 5]) and np.isinf(logits[7, 9]) and np.isfinite(logits[7, 0])
    assert np.array_equal(ids.cpu().numpy(), ids_ref)
    fin = np.isfinite(w_ref).all(axis=1)
    assert fin.sum() >= T - 2
    assert np.allclose(w.cpu().numpy()[fin], w_ref[fin], rtol=2e-6, atol=1e-9)
    assert np.array_equal(np.isnan(w.cpu().numpy()), np.isnan(w_ref))


@pytest.mark.parametrize("T", [33, 80, 333])
def test_short_contraction_dims(oracle, binding, T):
    """d_ffn = 32 and shared widths of 96: the down stage contracts over 1 to 3 k-blocks, fewer
    than the K splits that a launch of so few workgroups would otherwise get (no split may be left
    without a k-block); d_model = 96 gives the gate/up stage an odd number of k-blocks."""
    cfg = synth.LayerConfig("short_k", 6, 96, 32, 4, (80,), shared_d_ffn=(96, 96), routing="zipf", seed=83)
    case = Case(cfg, oracle, binding)
    check(case, T, "short-k")


def test_all_experts_unmerged(oracle, binding):
    """No pair at all: every routed expert dense (the degenerate end of the compression range)."""
    cfg = synth.LayerConfig("unmerged", 3, 128, 192, 2, (40,), seed=67, n_unmerged=3)
    case = Case(cfg, oracle, binding)
    for T in (3, 40, 400):
        check(case, T, "all-unmerged")


@pytest.mark.parametrize("T,d,E,k", [(1, 4096, 8, 2), (64, 4096, 8, 2), (300, 2048, 60, 4), (2048, 2048, 64, 6),
                                     (5, 520, 3, 1), (37, 1032, 20, 5), (9, 264, 130, 7), (3, 136, 256, 64),
                                     (2100, 264, 33, 3)])
def test_router_topk(oracle, binding, T, d, E, k):
    """Router logits as one fp32 fma chain: expert ids must equal the oracle's exactly."""
    say("router T=%d d=%d E=%d k=%d" % (T, d, E, k))
    g = torch.Generator().manual_seed(T + E)
    x = torch.randn(T, d, generator=g).to(torch.bfloat16)
    wr = (torch.randn(E, d, generator=g) * 0.05).to(torch.bfloat16)
    if T > 1:
        x[1] = x[0]                                    # duplicate token: identical decision
    wr[E - 1] = wr[0]                                  # duplicate expert: a tie on every token
    ids, w = binding.pzl_router_topk(x.cuda(), wr.cuda(), k)
    torch.cuda.synchronize()
    ids_ref, w_ref, _ = oracle.router_topk(x.view(torch.int16).numpy().view(np.uint16),
                                           wr.view(torch.int16).numpy().view(np.uint16), k)
    assert np.array_equal(ids.cpu().numpy(), ids_ref)
    assert np.allclose(w.cpu().numpy(), w_ref, rtol=2e-6, atol=1e-9)
    # the router's output feeds moe_ffn as is
    assert ids.dtype == torch.int32 and w.dtype == torch.float32 and ids.shape == (T, k)
