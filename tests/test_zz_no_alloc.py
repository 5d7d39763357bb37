"""pzl_moe_ffn_static, the entry point that allocates nothing, against pzl_moe_ffn.

The static variant runs the same kernels on the library's static scratch array instead of a
caller workspace, so its output must equal pzl_moe_ffn's bit for bit (which is stronger than the
1e-2 bound the FFN is held to against the CPU oracle; the oracle comparison of the same layer shape
lives in test_gpu_parity.py).  Two calls in a row, the second with a smaller batch: the array keeps
the first call's contents and the second call must not be disturbed by them.  Collected last: it
leaves the shared array dirty on purpose.
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
    return (torch.from_numpy(x.view(np.int16)).cuda(), torch.from_numpy(ids).cuda(), torch.from_numpy(w).cuda())


def test_static_scratch_matches_workspace_call(oracle, binding):
    cfg = synth.LayerConfig("static_scratch", 8, 1024, 2048, 2, (96, 24), shared_d_ffn=(512,), seed=1077)
    case = Case(cfg, oracle, binding)
    layer = case.layer
    assert binding.pzl_moe_ffn_static_max_bytes() == 32 << 20
    for T in (96, 24):                                    # the second call is smaller than the first
        print("pzl_moe_ffn_static: T=%d" % T, flush=True)
        assert layer.pzl_moe_ffn_workspace_bytes(T, cfg.top_k) <= binding.pzl_moe_ffn_static_max_bytes()
        x, (ids, w) = synth.tokens(cfg, T), synth.routing(cfg, T)
        xt, idt, wt = _dev(x, ids, w)
        y_ws = layer.pzl_moe_ffn(xt, idt, wt)
        torch.cuda.synchronize()
        y_st = torch.full((T, cfg.d_model), float("nan"), dtype=torch.bfloat16, device="cuda")
        layer.pzl_moe_ffn_static(xt, idt, wt, y_st)
        torch.cuda.synchronize()
        a = y_ws.view(torch.int16).cpu().numpy().view(np.uint16)
        b = y_st.view(torch.int16).cpu().numpy().view(np.uint16)
        assert np.array_equal(a, b), "T=%d: %d elements differ" % (T, int((a != b).sum()))
        y64, _ = case.ref(x, ids, w)                      # and both within the FFN's bound of the oracle
        ok, worst = tolerance_ok(b, y64)
        print("  worst err / bound vs the oracle = %.3f" % worst, flush=True)
        assert ok, worst


def test_static_scratch_refuses_what_does_not_fit(oracle, binding):
    cfg = synth.LayerConfig("static_scratch_big", 4, 512, 1024, 2, (8,), seed=1078)
    case = Case(cfg, oracle, binding)
    T = 4096                                              # workspace far beyond 32 MiB
    assert case.layer.pzl_moe_ffn_workspace_bytes(T, cfg.top_k) > binding.pzl_moe_ffn_static_max_bytes()
    x, (ids, w) = synth.tokens(cfg, T), synth.routing(cfg, T)
    xt, idt, wt = _dev(x, ids, w)
    y = torch.zeros(T, cfg.d_model, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(binding.PzlError) as e:
        case.layer.pzl_moe_ffn_static(xt, idt, wt, y)
    assert e.value.rc == binding.PZL_ENOSPC
    torch.cuda.synchronize()
    assert not y.any()                                    # nothing was launched
    # ... and a batch that fits still works afterwards
    x, (ids, w) = synth.tokens(cfg, 8), synth.routing(cfg, 8)
    xt, idt, wt = _dev(x, ids, w)
    y8 = torch.empty(8, cfg.d_model, dtype=torch.bfloat16, device="cuda")
    case.layer.pzl_moe_ffn_static(xt, idt, wt, y8)
    y_ws = case.layer.pzl_moe_ffn(xt, idt, wt)
    torch.cuda.synchronize()
    assert torch.equal(y8.view(torch.int16), y_ws.view(torch.int16))
