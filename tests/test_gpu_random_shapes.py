"""Seeded random layer shapes and batch sizes through pzl_moe_ffn against the CPU oracle.

The named tests pick their shapes by hand; this one draws them: 2 to 64 experts, some kept
unmerged, model and expert widths from 32 up (so contractions as short as one k-block and odd
numbers of k-blocks occur), top-1 to top-6, no, one or two shared experts, even or skewed routing,
a hot expert now and then, 1 to 500 tokens.  Same bar as everywhere: every element within
1e-2 * max(|y_ref|, rms of its row).
"""
import random

import numpy as np
import pytest
import torch

from paper_2511_04805_amd import synth
from helpers import Case, tolerance_ok

pytestmark = pytest.mark.gpu

N_CASES = 16


def draw(ci):
    rng = random.Random(9000 + ci)
    E = rng.choice([2, 4, 6, 8, 12, 24, 40, 64])
    D = rng.choice([0, 0, 2, 4]) if E >= 6 else 0
    d = rng.choice([32, 64, 96, 128, 160, 256])
    f = rng.choice([32, 64, 96, 160, 256, 352, 512])
    k = rng.randint(1, min(E, 6))
    shared = rng.choice([(), (), (64,), (96, 96), (160, 64)])
    routing = rng.choice(["gaussian", "zipf"])
    Ts = rng.sample([1, 3, 17, 33, 48, 65, 80, 100, 129, 200, 333, 500], 3)
    cfg = synth.LayerConfig("random%d" % ci, E, d, f, k, tuple(Ts), shared_d_ffn=shared, routing=routing,
                            seed=9000 + ci, n_unmerged=D)
    return cfg, Ts, rng


@pytest.mark.parametrize("ci", range(N_CASES))
def test_random_layer(oracle, ci):
    from paper_2511_04805_amd import binding
    binding.load()
    cfg, Ts, rng = draw(ci)
    print("random layer %d: E=%d unmerged=%d d=%d f=%d k=%d shared=%s routing=%s T=%s" % (
        ci, cfg.n_experts, cfg.n_unmerged, cfg.d_model, cfg.d_ffn, cfg.top_k, cfg.shared_d_ffn, cfg.routing, Ts),
        flush=True)
    case = Case(cfg, oracle, binding, emap_mode=rng.choice(["adjacent", "random"]))
    for T in Ts:
        x = synth.tokens(cfg, T)
        ids, w = synth.routing(cfg, T)
        if rng.random() < 0.3:
            ids[:, 0] = rng.randrange(cfg.n_experts)          # a hot expert (duplicates within a token add up)
        y = case.gpu(x, ids, w)
        y64, _ = case.ref(x, ids, w)
        ok, worst = tolerance_ok(y, y64)
        print("   T=%d worst err / bound = %.3f" % (T, worst), flush=True)
        assert ok, (T, worst)


FORCED = [(-1, -1, -1), (0, -1, -1), (1, 0, 0), (1, 0, 1), (1, 1, 0), (1, 1, 1)]


@pytest.mark.parametrize("shape", [(8, 0, 128, 256, 2, (), "gaussian"), (40, 2, 96, 160, 4, (64,), "zipf"),
                                   (64, 0, 64, 96, 6, (96, 96), "zipf")])
def test_forced_plans(oracle, shape):
    """pzl_layer_force_plan: every launch plan the library could choose (streaming kernels only; tiled
    kernels as one workgroup per tile or as a persistent launch, on the caller's stream or on the
    layer's own) gives the same y within the bound, at batch sizes on both sides of the library's own
    thresholds; releasing the override gives the library's choice back."""
    from paper_2511_04805_amd import binding
    binding.load()
    E, D, d, f, k, shared, routing = shape
    cfg = synth.LayerConfig("forced", E, d, f, k, (1,), shared_d_ffn=shared, routing=routing, seed=9100 + E, n_unmerged=D)
    case = Case(cfg, oracle, binding, emap_mode="random")
    with pytest.raises(binding.PzlError):
        case.layer.pzl_layer_force_plan(2, 0, 0)
    for T in (5, 70, 300):
        x = synth.tokens(cfg, T)
        ids, w = synth.routing(cfg, T)
        y64, _ = case.ref(x, ids, w)
        for force in FORCED:
            case.layer.pzl_layer_force_plan(*force)
            print("   E=%d T=%d forced %s" % (E, T, force), flush=True)
            ok, worst = tolerance_ok(case.gpu(x, ids, w), y64)
            assert ok, (T, force, worst)
    case.layer.pzl_layer_force_plan(-1, -1, -1)


@pytest.mark.parametrize("T", [420, 1040, 1100])
def test_wide_experts_gathered_x(oracle, T):
    """Experts of 8192 features or more, in a batch that the tiled kernels take: x is gathered into
    fragment order in front of the gate/up stage (and H is kept in it), tiles of one to four token
    fragments short of full included, tiles of 17 fragments among them (1040 tokens); same bar."""
    from paper_2511_04805_amd import binding
    binding.load()
    cfg = synth.LayerConfig("wide8192", 4, 64, 8192, 2, (T,), seed=9200)
    case = Case(cfg, oracle, binding, emap_mode="random")
    x = synth.tokens(cfg, T)
    ids, w = synth.routing(cfg, T)
    y64, _ = case.ref(x, ids, w)
    ok, worst = tolerance_ok(case.gpu(x, ids, w), y64)
    print("   T=%d worst err / bound = %.3f" % (T, worst), flush=True)
    assert ok, (T, worst)
