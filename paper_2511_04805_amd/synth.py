"""Seeded synthetic workloads shaped like the paper's MoE layers.

This module only *draws inputs*: merged magnitudes, mask and sign planes, dense
shared-expert weights, token activations and router decisions.  It contains none
of the method's arithmetic (no pack, no decode, no FFN) so that the CPU oracle and
the HIP library can both be fed from it without sharing any code of their own.

The trained Mixtral-8x7B / Qwen1.5-MoE-A2.7B / DeepSeek-MoE-16B weights the paper
evaluates (Sec. 4.1) are not available offline; these tensors stand in for them:
expert weights are zero-mean Gaussians with one sigma per layer (paper appendix,
"Visualization of MoE Expert Weight Distribution"), which keeps bf16 exponents in
the 112..128 band the paper reports (Sec. 3.3.1).
"""
from dataclasses import dataclass, field
from typing import Tuple

import numpy as np
import torch


@dataclass(frozen=True)
class LayerConfig:
    name: str
    n_experts: int
    d_model: int
    d_ffn: int
    top_k: int
    n_tokens: Tuple[int, ...]
    shared_d_ffn: Tuple[int, ...] = ()
    routing: str = "gaussian"          # "gaussian" | "zipf"
    seed: int = 1000
    sigma: float = 0.02
    mask_density: float = 0.5
    n_unmerged: int = 0                # routed experts kept dense (25 % compression leaves half of them)

    @property
    def n_pairs(self):
        return (self.n_experts - self.n_unmerged) // 2


CONFIGS = {
    "tiny": LayerConfig("tiny", 2, 128, 256, 1, (8,), seed=1000),
    "mixtral_decode": LayerConfig("mixtral_decode", 8, 4096, 14336, 2, (1, 8, 32, 64), seed=1001),
    "mixtral_prefill": LayerConfig("mixtral_prefill", 8, 4096, 14336, 2, (4096,), seed=1001),
    "qwen15_moe": LayerConfig("qwen15_moe", 60, 2048, 1408, 4, (256,), shared_d_ffn=(5632,),
                              seed=1003),
    "deepseek_moe": LayerConfig("deepseek_moe", 64, 2048, 1408, 6, (2048,),
                                shared_d_ffn=(1408, 1408), routing="zipf", seed=1004),
    # Two further layer shapes, not among the paper's models: the library's launch rules were fitted
    # on the three shapes above, and the benchmark's plan study times them on these (16 wide experts
    # top-2; 128 narrow experts top-8, with an even and with a skewed router).
    "wide16": LayerConfig("wide16", 16, 4096, 6400, 2, (256,), seed=1005),
    "narrow128": LayerConfig("narrow128", 128, 2048, 768, 8, (256,), seed=1006),
    "narrow128_zipf": LayerConfig("narrow128_zipf", 128, 2048, 768, 8, (256,), routing="zipf", seed=1006),
}

_GATE, _UP, _DOWN = 0, 1, 2
_PLANES = ("merged", "mask0", "mask1", "sign0", "sign1")


def _gen(cfg, device, *key):
    """One independent generator per tensor, so any tensor can be redrawn alone."""
    g = torch.Generator(device=device)
    s = cfg.seed
    for v in key:
        s = (s * 1000003 + int(v) + 12345) % (2 ** 62)
    g.manual_seed(s)
    return g


def _np_bits(t):
    """torch int16/uint8 tensor -> numpy (uint16 view for 16-bit patterns)."""
    a = t.cpu().numpy()
    return a.view(np.uint16) if a.dtype == np.int16 else a


def matrix_shape(cfg, which, d_ffn=None):
    f = cfg.d_ffn if d_ffn is None else d_ffn
    return (cfg.d_model, f) if which == _DOWN else (f, cfg.d_model)


def pair_matrix_t(cfg, pair, which, shape=None, device="cpu"):
    """Inputs of pack for one matrix of one expert pair, as torch tensors on ``device``.

    dict(merged: int16 view of the bf16 bits of |N(0, sigma)|, mask0, mask1, sign0, sign1: uint8).
    Masks are independent Bernoulli(mask_density) per expert, signs Bernoulli(0.5).  The stream
    of a CPU generator and of a GPU generator differ; each is reproducible on its own device.
    """
    rows, cols = shape if shape is not None else matrix_shape(cfg, which)
    n = rows * cols
    out = {}
    g = _gen(cfg, device, 1, pair, which, 0)
    mag = (torch.randn(n, generator=g, device=device) * cfg.sigma).abs_()
    out["merged"] = mag.to(torch.bfloat16).view(torch.int16).reshape(rows, cols)
    for i, name in enumerate(_PLANES[1:], start=1):
        g = _gen(cfg, device, 1, pair, which, i)
        p = cfg.mask_density if name.startswith("mask") else 0.5
        out[name] = (torch.rand(n, generator=g, device=device) < p).to(torch.uint8).reshape(rows, cols)
    return out


def pair_matrix(cfg, pair, which, shape=None):
    """numpy form of pair_matrix_t on the CPU (merged as uint16)."""
    return {k: _np_bits(v) for k, v in pair_matrix_t(cfg, pair, which, shape).items()}


def shared_matrix_t(cfg, s, which, device="cpu"):
    """Dense bf16 bits (int16 view) of one matrix of shared expert ``s`` (signed N(0, sigma))."""
    rows, cols = matrix_shape(cfg, which, cfg.shared_d_ffn[s])
    g = _gen(cfg, device, 2, s, which)
    w = torch.randn(rows * cols, generator=g, device=device) * cfg.sigma
    return w.to(torch.bfloat16).view(torch.int16).reshape(rows, cols)


def shared_matrix(cfg, s, which):
    return _np_bits(shared_matrix_t(cfg, s, which))


def unmerged_matrix_t(cfg, j, which, device="cpu"):
    """Dense bf16 bits (int16 view) of one matrix of routed expert j that is kept unmerged."""
    rows, cols = matrix_shape(cfg, which)
    g = _gen(cfg, device, 8, j, which)
    w = torch.randn(rows * cols, generator=g, device=device) * cfg.sigma
    return w.to(torch.bfloat16).view(torch.int16).reshape(rows, cols)


def unmerged_pair_t(cfg, pair, which, shape=None, device="cpu"):
    """Inputs of the offline merge for one matrix of one expert pair: two dense experts drawn as
    signed N(0, sigma) bf16 (int16 views) and one positive activation-norm vector per expert
    (uniform in [0.5, 1.5]; stands in for the calibration norms of Eq. 2, which need real data).
    Returns (w_i, w_j, norm_i, norm_j)."""
    rows, cols = shape if shape is not None else matrix_shape(cfg, which)
    out = []
    for e in (0, 1):
        g = _gen(cfg, device, 6, pair, which, e)
        w = torch.randn(rows * cols, generator=g, device=device) * cfg.sigma
        out.append(w.to(torch.bfloat16).view(torch.int16).reshape(rows, cols))
    for e in (0, 1):
        g = _gen(cfg, device, 7, pair, which, e)
        out.append(torch.rand(cols, generator=g, device=device) + 0.5)
    return tuple(out)


def tokens(cfg, T):
    """x [T, d_model] bf16 bits, N(0,1)."""
    g = _gen(cfg, "cpu", 3, T)
    x = torch.randn(T * cfg.d_model, generator=g).to(torch.bfloat16).view(torch.int16)
    return _np_bits(x).reshape(T, cfg.d_model)


def routing(cfg, T):
    """Router decisions (inputs of the path): ids [T,k] int32, weights [T,k] float32.

    gaussian: top-k of N(0,1) logits.  zipf: expert popularity p_r ~ r^-1.1 assigned to
    experts by a seeded permutation; ids are the top-k of log p + Gumbel noise, i.e. k
    experts sampled without replacement in proportion to p.  Weights are the softmax of
    the selected scores.
    """
    g = _gen(cfg, "cpu", 4, T)
    E, k = cfg.n_experts, cfg.top_k
    logits = torch.randn(T, E, generator=g)
    if cfg.routing == "zipf":
        ranks = torch.arange(1, E + 1, dtype=torch.float64)
        p = ranks.pow(-1.1)
        p = (p / p.sum()).to(torch.float32)
        perm = torch.randperm(E, generator=g)
        logp = torch.empty(E)
        logp[perm] = p.log()
        u = torch.rand(T, E, generator=g).clamp_(1e-9, 1 - 1e-9)
        scores = logp[None, :] + (-(-u.log()).log())
        sel, ids = torch.topk(scores, k, dim=1)
        sel = logits.gather(1, ids)
    else:
        sel, ids = torch.topk(logits, k, dim=1)
    w = torch.softmax(sel.float(), dim=1)
    return ids.to(torch.int32).numpy(), w.to(torch.float32).numpy()


def expert_map(cfg, mode="adjacent"):
    """expert -> (pair, position).  adjacent: (e//2, e%2); random: seeded random pairing
    (the paper's default grouping is random, Sec. 3.2 "Pair-wise Experts Grouping").
    Experts kept unmerged get pair = -1 - j (j-th dense routed expert)."""
    E = cfg.n_experts
    if mode == "adjacent":
        order = np.arange(E)
    else:
        order = torch.randperm(E, generator=_gen(cfg, "cpu", 5)).numpy()
    pair = np.empty(E, dtype=np.int32)
    pos = np.empty(E, dtype=np.uint8)
    pair[order] = np.arange(E) // 2
    pos[order] = np.arange(E) % 2
    # the last n_unmerged experts of the order stay dense: pair = -1 - j, position 0
    D = cfg.n_unmerged
    if D:
        pair[order[E - D:]] = -1 - np.arange(D)
        pos[order[E - D:]] = 0
    return pair, pos


GATE, UP, DOWN = _GATE, _UP, _DOWN
