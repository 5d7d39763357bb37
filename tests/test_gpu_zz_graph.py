"""pzl_moe_ffn under HIP graph capture.

The call only enqueues work (kernels, and event record / wait pairs that fork to and join from the
layer's own streams), allocates nothing and clears its counters in its own kernels, so a caller may
capture it into a graph.  Each replay is compared bit for bit with an eager call on the same inputs
(the path is deterministic), with eager work and synchronisation between the replays.
"""
import numpy as np
import pytest
import torch

from paper_2511_04805_amd import synth
from helpers import Case, tolerance_ok

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def binding():
    from paper_2511_04805_amd import binding as b
    b.load()
    assert torch.cuda.is_available()
    return b


def _dev(x, ids, w):
    return (torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16), torch.from_numpy(ids).cuda(),
            torch.from_numpy(w).cuda())


@pytest.mark.parametrize("name,T", [("small", 40), ("many", 120), ("many", 700)])
def test_graph_replays_match_eager_calls(oracle, binding, name, T):
    """small: streaming kernels + two shared experts on the second stream.  many (40 experts, 8
    unmerged, skewed routing): streaming and persistent tiled kernels, the latter on the third
    stream at 120 tokens, + a shared expert."""
    print("graph %s T=%d" % (name, T), flush=True)
    if name == "small":
        cfg = synth.LayerConfig("small", 6, 192, 352, 2, (40,), shared_d_ffn=(96, 160), seed=31)
    else:
        cfg = synth.LayerConfig("many_mixed", 40, 128, 384, 3, (300,), shared_d_ffn=(128,), routing="zipf",
                                seed=71, n_unmerged=8)
    case = Case(cfg, oracle, binding, emap_mode="random", check_pack=False)
    layer = case.layer

    def inputs(variant):
        x = synth.tokens(cfg, T)
        ids, w = synth.routing(cfg, T)
        if variant:                                     # other tokens, other routing
            x = np.roll(x, variant, axis=0).copy()
            ids = ((ids + variant) % cfg.n_experts).astype(np.int32)
            w = np.ascontiguousarray(w[::-1])
        return x, ids, w

    x0, ids0, w0 = inputs(0)
    xs, ids_s, ws_ = _dev(x0, ids0, w0)                 # the graph's fixed input and output buffers
    ys = torch.empty(T, cfg.d_model, dtype=torch.bfloat16, device="cuda")
    work = torch.empty(layer.pzl_moe_ffn_workspace_bytes(T, cfg.top_k), dtype=torch.uint8, device="cuda")
    layer.pzl_moe_ffn(xs, ids_s, ws_, y=ys, workspace=work)        # eager warm-up (one-time kernel attributes)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.graph(graph, stream=side):
        layer.pzl_moe_ffn(xs, ids_s, ws_, y=ys, workspace=work)
    torch.cuda.synchronize()

    for variant in (0, 3, 7, 0):
        x, ids, w = inputs(variant)
        xe, ide, we = _dev(x, ids, w)
        y_eager = layer.pzl_moe_ffn(xe, ide, we)        # eager, own buffers and the layer's own workspace
        torch.cuda.synchronize()
        xs.copy_(xe); ids_s.copy_(ide); ws_.copy_(we)
        ys.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(ys.view(torch.int16), y_eager.view(torch.int16)), "replay differs (variant %d)" % variant
    # and the last replay against the oracle
    y64, _ = case.ref(x, ids, w)
    ok, worst = tolerance_ok(ys.view(torch.int16).cpu().numpy().view(np.uint16), y64)
    assert ok, worst
