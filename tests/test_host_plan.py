"""The host-side launch plan of pzl_moe_ffn (pzl_moe_ffn_plan): pure host arithmetic, checked
without a GPU.  The kernels rely on these properties: their launches reject, or would misbehave
on, a plan that breaks them (a K split without a k-block made the read-ahead of a tiny layer leave
its buffers once)."""
import itertools

import pytest

from paper_2511_04805_amd import binding


def plan(*a, **kw):
    return binding.pzl_moe_ffn_plan(*a, **kw)


SHAPES = [  # n_experts, d_model, d_ffn, top_k, shared widths, unmerged
    (8, 4096, 14336, 2, (), 0),
    (60, 2048, 1408, 4, (5632,), 0),
    (64, 2048, 1408, 6, (1408, 1408), 0),
    (6, 96, 32, 4, (96, 96), 0),
    (2, 32, 32, 1, (32,), 0),
    (40, 128, 384, 3, (128,), 8),
    (12, 256, 64, 4, (64, 160), 4),
    (256, 64, 96, 8, (), 0),
]
TOKENS = [0, 1, 2, 31, 32, 33, 47, 48, 64, 65, 80, 96, 100, 128, 200, 256, 288, 289, 333, 500, 1024, 4096, 20000]


@pytest.mark.parametrize("shape", SHAPES)
def test_plan_invariants(shape):
    E, d, f, k, shared, D = shape
    for T, quant in itertools.product(TOKENS, (False, True)):
        if quant and (d % 128 or f % 128):
            continue
        p = plan(E, d, f, T, k, shared_d_ffn=shared, n_unmerged=D, quantised=quant)
        N = T * k
        # every K split holds at least one k-block (one 128-column group in the quantised format)
        assert 1 <= p["ksplit"] <= min(8, f // (128 if quant else 32)), (T, quant, p)
        if shared:
            assert 1 <= p["ksplit_shared"] <= min(8, min(shared) // 32), (T, p)
        # quantised layers have no tiled kernels
        assert not (quant and p["hybrid"])
        # both paths from 20 slots per expert on average (6 with 32 experts or more)
        assert bool(p["hybrid"]) == (not quant and N >= (6 if E >= 32 else 20) * E), (T, p)
        assert p["tile_min"] == (33 if p["hybrid"] else 0)
        # persistent launches and the tile stream only where tiled kernels are launched
        assert not (p["persistent"] and not p["hybrid"]) and not (p["tile_stream"] and not p["hybrid"])
        if p["persistent"]:
            assert 2 * ((E - D) // 2 + D) >= 32 and N <= 256 * 2 * ((E - D) // 2 + D)
        # sweeps of the streaming kernels: one workgroup where the tiled kernels take the busy pairs,
        # else one per 32 (64) tokens that an expert can get, at most 3
        if p["hybrid"]:
            assert p["sweep_wgs_packed"] == 1 and p["sweep_wgs_unmerged"] == 1
        else:
            assert p["sweep_wgs_packed"] == max(1, min(3, -(-T // 32)))
            assert p["sweep_wgs_unmerged"] == max(1, min(3, -(-T // 64)))
        # the gate/up kernel groups the list itself exactly where only it needs the tables first: a
        # streaming-only batch of packed pairs that fits its limits (512 entries, 128 routing keys)
        n_keys = 2 * ((E - D) // 2 + D)
        assert bool(p["grouping_in_kernel"]) == (not quant and not p["hybrid"] and E > D and 1 <= N <= 512 and n_keys <= 128), (T, p)
        # shared experts: tiled from 65 tokens; the tiles cover the batch, hold 16..288 tokens in
        # whole fragments, and experts of equal width (one launch) agree
        assert bool(p["tiled_shared"]) == (len(shared) > 0 and T >= 65)
        assert bool(p["shared_stream"]) == (len(shared) > 0 and N > 0)
        for s, fs in enumerate(shared):
            tiles, tok = p["shared_token_tiles"][s], p["shared_tile_tokens"][s]
            if not p["tiled_shared"]:
                assert tiles == 0 and tok == 0
                continue
            assert tok % 16 == 0 and 16 <= tok <= 288 and tiles * tok >= T > (tiles - 1) * tok, (T, p)
            assert tiles == -(-T // 288) or tok >= 48, (T, p)          # never below 48 tokens unless forced
            if s and shared[s - 1] == fs:
                assert (tiles, tok) == (p["shared_token_tiles"][s - 1], p["shared_tile_tokens"][s - 1])


def test_plan_of_the_benchmark_shapes():
    """The decisions that the measured configurations rely on."""
    p = plan(8, 4096, 14336, 64, 2)                           # decode: streaming only, down split 4 ways
    assert not p["hybrid"] and p["ksplit"] == 4 and p["sweep_wgs_packed"] == 2 and p["grouping_in_kernel"]
    p = plan(8, 4096, 14336, 4096, 2)                         # prefill: one workgroup per tile, no K split
    assert p["hybrid"] and not p["persistent"] and not p["tile_stream"] and p["ksplit"] == 1
    p = plan(60, 2048, 1408, 256, 4, shared_d_ffn=(5632,))    # persistent tiles on the third stream, 4 x 64 shared tokens
    assert p["hybrid"] and p["persistent"] and p["tile_stream"] and p["shared_stream"]
    assert p["shared_token_tiles"] == [4] and p["shared_tile_tokens"] == [64]
    p = plan(64, 2048, 1408, 2048, 6, shared_d_ffn=(1408, 1408))
    assert p["hybrid"] and p["persistent"] and not p["tile_stream"]
    assert p["shared_token_tiles"] == [8, 8] and p["shared_tile_tokens"] == [256, 256]
    p = plan(6, 96, 32, 80, 4, shared_d_ffn=(96, 96))         # one k-block in the down stage: no split
    assert p["ksplit"] == 1 and p["ksplit_shared"] == 1


def test_plan_rejects_bad_arguments():
    for bad in (dict(n_experts=0), dict(n_experts=257), dict(d_model=48), dict(d_ffn=0), dict(n_unmerged=1),
                dict(shared_d_ffn=(40,)), dict(T=-1), dict(k=-1), dict(shared_d_ffn=(32,) * 17)):
        kw = dict(n_experts=8, d_model=128, d_ffn=256, T=10, k=2, shared_d_ffn=(), n_unmerged=0)
        kw.update(bad)
        with pytest.raises(binding.PzlError):
            plan(kw["n_experts"], kw["d_model"], kw["d_ffn"], kw["T"], kw["k"], shared_d_ffn=kw["shared_d_ffn"],
                 n_unmerged=kw["n_unmerged"])
