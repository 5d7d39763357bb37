"""Builds the same synthetic layer for the CPU oracle and for the HIP library (tests only)."""
import numpy as np
import torch

from paper_2511_04805_amd import synth

W3 = (synth.GATE, synth.UP, synth.DOWN)


def bits_to_f64(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).astype(np.int16)).view(torch.bfloat16).double().numpy()


def tolerance_ok(y_gpu_bits, y_ref64, rel=1e-2):
    """|y_gpu - y_ref| <= rel * max(|y_ref|, rms of that token's row), element by element.

    Token rows are independent results, so each row is scaled by its own rms: "relative error"
    is undefined at y ~ 0, and an element much smaller than its row is held to the row's scale.
    Returns (ok, worst error / bound)."""
    y = bits_to_f64(y_gpu_bits)
    if y.size == 0:
        return True, 0.0
    rms = np.sqrt(np.mean(y_ref64 ** 2, axis=1, keepdims=True))
    bound = rel * np.maximum(np.abs(y_ref64), rms)
    err = np.abs(y - y_ref64)
    worst = float((err / np.maximum(bound, 1e-300)).max())
    return bool(np.all(err <= bound)), worst


class Case:
    """One layer: oracle-side packed tensors (numpy, logical order) + the library's Layer."""

    def __init__(self, cfg, oracle, binding, device="cuda", emap_mode="adjacent", gen_device=None,
                 check_pack=True, from_merge=None, wide_h=False):
        self.cfg, self.oracle, self.binding = cfg, oracle, binding
        gen_device = gen_device or device
        self.emap = synth.expert_map(cfg, emap_mode)
        self.packed_cpu = {}
        self.packed_gpu = {}
        self.n_bad = torch.zeros(1, dtype=torch.int32, device=device)
        self.n_similar = 0
        for p in range(cfg.n_pairs):
            for which in W3:
                if from_merge is not None:
                    # the paper's own pipeline: two dense experts -> dual-mask merge -> packed pair
                    wi, wj, ni, nj = synth.unmerged_pair_t(cfg, p, which, device=gen_device)
                    self.packed_gpu[p, which] = binding.pzl_merge_pack(wi.to(device), wj.to(device), ni.to(device),
                                                                       nj.to(device), from_merge,
                                                                       n_out_of_range=self.n_bad)
                    ref = oracle.merge(synth._np_bits(wi), synth._np_bits(wj), ni.cpu().numpy(),
                                       nj.cpu().numpy(), from_merge)
                    packed, bad = oracle.pack(ref["merged"], ref["mask0"], ref["mask1"], ref["sign0"],
                                              ref["sign1"])
                    assert bad == 0
                    self.packed_cpu[p, which] = packed
                    self.n_similar += ref["n_similar"]
                    rows, cols = packed.shape
                    got = binding.tiled_to_logical(
                        self.packed_gpu[p, which].cpu().numpy().view(np.uint16), rows, cols)
                    assert np.array_equal(got, packed), "merge_pack mismatch pair %d matrix %d" % (p, which)
                    continue
                pl = synth.pair_matrix_t(cfg, p, which, device=gen_device)
                pl_dev = {k: v.to(device) for k, v in pl.items()}
                self.packed_gpu[p, which] = binding.pzl_pack(pl_dev["merged"], pl_dev["mask0"], pl_dev["mask1"],
                                                             pl_dev["sign0"], pl_dev["sign1"],
                                                             n_out_of_range=self.n_bad)
                host = {k: synth._np_bits(v) for k, v in pl.items()}
                packed, bad = oracle.pack(host["merged"], host["mask0"], host["mask1"], host["sign0"],
                                          host["sign1"])
                assert bad == 0
                self.packed_cpu[p, which] = packed
                if check_pack:
                    rows, cols = packed.shape
                    got = binding.tiled_to_logical(
                        self.packed_gpu[p, which].cpu().numpy().view(np.uint16), rows, cols)
                    assert np.array_equal(got, packed), "pack mismatch pair %d matrix %d" % (p, which)
                del pl, pl_dev, host
        self.shared_cpu, shared_gpu = [], []
        for s, fs in enumerate(cfg.shared_d_ffn):
            mats = [synth.shared_matrix_t(cfg, s, w, device=gen_device) for w in W3]
            self.shared_cpu.append(tuple(synth._np_bits(m) for m in mats))
            shared_gpu.append(tuple(binding.pzl_tile_dense(m.to(device)) for m in mats) + (fs,))
        self.dense_cpu, dense_gpu = [], []
        for j in range(cfg.n_unmerged):                       # routed experts kept unmerged
            mats = [synth.unmerged_matrix_t(cfg, j, w, device=gen_device) for w in W3]
            self.dense_cpu.append(tuple(synth._np_bits(m) for m in mats))
            dense_gpu.append(tuple(binding.pzl_tile_dense(m.to(device)) for m in mats))
        P = cfg.n_pairs
        self.layer = binding.Layer(cfg.d_model, cfg.d_ffn, self.emap[0], self.emap[1],
                                   [self.packed_gpu[p, synth.GATE] for p in range(P)],
                                   [self.packed_gpu[p, synth.UP] for p in range(P)],
                                   [self.packed_gpu[p, synth.DOWN] for p in range(P)], shared=shared_gpu,
                                   dense=dense_gpu, wide_h=wide_h)
        assert int(self.n_bad.item()) == 0
        self.device = device

    def gpu(self, x, ids, w):
        dev = self.device
        xt = torch.from_numpy(x.view(np.int16)).to(dev)
        y = self.layer.pzl_moe_ffn(xt, torch.from_numpy(ids).to(dev), torch.from_numpy(w).to(dev))
        torch.cuda.synchronize()
        return y.view(torch.int16).cpu().numpy().view(np.uint16)

    def ref(self, x, ids, w, **kw):
        P = self.cfg.n_pairs
        return self.oracle.moe_ffn(x, ids, w, self.emap[0], self.emap[1],
                                   [self.packed_cpu[p, synth.GATE] for p in range(P)],
                                   [self.packed_cpu[p, synth.UP] for p in range(P)],
                                   [self.packed_cpu[p, synth.DOWN] for p in range(P)],
                                   shared=self.shared_cpu, dense=self.dense_cpu, **kw)
