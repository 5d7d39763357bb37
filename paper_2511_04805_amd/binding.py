"""ctypes binding of the HIP C-ABI library (include/puzzle_moe.h).

Argument marshalling only: every step of the path runs in the library's kernels.  torch is
used for device memory and streams.  There is no fallback: if the library is not built, or no
GPU is present, the calls raise.
"""
import ctypes
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpuzzle_moe.so")
_lib = None

PZL_OK, PZL_EINVAL, PZL_ENOSPC, PZL_EHIP, PZL_ENOMEM = 0, -1, -2, -3, -4

EXPORTS = ("pzl_abi_version", "pzl_strerror", "pzl_last_hip_error", "pzl_packed_bytes", "pzl_pack",
           "pzl_unpack", "pzl_unpack_half_x2", "pzl_tile_dense", "pzl_merge_pack", "pzl_router_topk",
           "pzl_q_record_bytes", "pzl_q_scale_bytes", "pzl_q_pack", "pzl_q_unpack", "pzl_layer_create", "pzl_layer_destroy",
           "pzl_moe_ffn_plan", "pzl_moe_ffn_workspace_bytes", "pzl_moe_ffn", "pzl_moe_ffn_staged",
           "pzl_moe_ffn_static", "pzl_moe_ffn_static_max_bytes", "pzl_moe_ffn_workspace_layout", "pzl_layer_h_info",
           "pzl_layer_force_plan")

STAGES = ("route", "gateup", "down", "shared", "combine")


class _LayerShape(ctypes.Structure):
    _fields_ = [("n_experts", ctypes.c_int32), ("n_unmerged", ctypes.c_int32), ("d_model", ctypes.c_int32),
                ("d_ffn", ctypes.c_int32), ("n_shared", ctypes.c_int32),
                ("shared_d_ffn", ctypes.POINTER(ctypes.c_int32)), ("pair_format", ctypes.c_int32)]


class _Plan(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("shared_stream", "hybrid", "tile_min", "persistent", "tile_stream",
                                              "ksplit", "ksplit_shared", "tiled_shared", "sweep_wgs_packed",
                                              "sweep_wgs_unmerged")] + \
               [("shared_token_tiles", ctypes.c_int32 * 16), ("shared_tile_tokens", ctypes.c_int32 * 16),
                ("grouping_in_kernel", ctypes.c_int32)]


class _WorkspaceLayout(ctypes.Structure):
    _fields_ = [("n_keys", ctypes.c_int32), ("max_tiles", ctypes.c_int32)] + \
               [(n, ctypes.c_size_t) for n in ("streamed_count", "first_slot", "slot_token", "slot_of", "tile_key",
                                               "tile_first_slot", "tile_tokens", "n_tiles", "total")]


class PzlError(RuntimeError):
    def __init__(self, rc, where):
        self.rc = rc
        lib = load()
        msg = lib.pzl_strerror(rc).decode()
        if rc == PZL_EHIP:
            msg += ": " + lib.pzl_last_hip_error().decode()
        super().__init__("%s failed: %s (rc=%d)" % (where, msg, rc))


class _LayerDesc(ctypes.Structure):
    _fields_ = [("n_experts", ctypes.c_int32), ("d_model", ctypes.c_int32), ("d_ffn", ctypes.c_int32),
                ("expert_pair", ctypes.c_void_p), ("expert_pos", ctypes.c_void_p),
                ("gate", ctypes.c_void_p), ("up", ctypes.c_void_p), ("down", ctypes.c_void_p),
                ("n_shared", ctypes.c_int32), ("shared_d_ffn", ctypes.c_void_p),
                ("shared_gate", ctypes.c_void_p), ("shared_up", ctypes.c_void_p),
                ("shared_down", ctypes.c_void_p),
                ("n_dense", ctypes.c_int32), ("dense_gate", ctypes.c_void_p),
                ("dense_up", ctypes.c_void_p), ("dense_down", ctypes.c_void_p),
                ("pair_format", ctypes.c_int32), ("gate_scale", ctypes.c_void_p),
                ("up_scale", ctypes.c_void_p), ("down_scale", ctypes.c_void_p), ("h_precision", ctypes.c_int32)]


def load():
    """Load the built library; raise if it is missing (build with `python -m paper_2511_04805_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("HIP library not built: %s is missing "
                               "(run `python -m paper_2511_04805_amd.build`)" % LIB_PATH)
        lib = ctypes.CDLL(LIB_PATH)
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
        lib.pzl_abi_version.restype = ctypes.c_int
        lib.pzl_strerror.restype = ctypes.c_char_p
        lib.pzl_strerror.argtypes = [ctypes.c_int]
        lib.pzl_last_hip_error.restype = ctypes.c_char_p
        lib.pzl_packed_bytes.restype = ctypes.c_size_t
        lib.pzl_packed_bytes.argtypes = [i64, i64]
        lib.pzl_pack.restype = ctypes.c_int
        lib.pzl_pack.argtypes = [vp, vp, vp, vp, vp, i64, i64, vp, vp, vp]
        lib.pzl_unpack.restype = ctypes.c_int
        lib.pzl_unpack.argtypes = [vp, ctypes.c_int, i64, i64, vp, vp]
        lib.pzl_unpack_half_x2.restype = ctypes.c_int
        lib.pzl_unpack_half_x2.argtypes = [vp, ctypes.c_int, i64, i64, vp, vp]
        lib.pzl_tile_dense.restype = ctypes.c_int
        lib.pzl_tile_dense.argtypes = [vp, i64, i64, vp, vp]
        lib.pzl_merge_pack.restype = ctypes.c_int
        lib.pzl_merge_pack.argtypes = [vp, vp, vp, vp, i64, i64, ctypes.c_float, vp, vp, vp, vp]
        lib.pzl_router_topk.restype = ctypes.c_int
        lib.pzl_router_topk.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, vp]
        lib.pzl_layer_create.restype = ctypes.c_int
        lib.pzl_layer_create.argtypes = [ctypes.POINTER(_LayerDesc), ctypes.POINTER(vp)]
        lib.pzl_layer_destroy.restype = None
        lib.pzl_layer_destroy.argtypes = [vp]
        lib.pzl_moe_ffn_plan.restype = ctypes.c_int
        lib.pzl_moe_ffn_plan.argtypes = [ctypes.POINTER(_LayerShape), i32, i32, ctypes.POINTER(_Plan)]
        lib.pzl_moe_ffn_workspace_bytes.restype = ctypes.c_size_t
        lib.pzl_moe_ffn_workspace_bytes.argtypes = [vp, i32, i32]
        lib.pzl_moe_ffn.restype = ctypes.c_int
        lib.pzl_moe_ffn.argtypes = [vp, vp, vp, vp, i32, i32, vp, vp, ctypes.c_size_t, vp]
        lib.pzl_moe_ffn_staged.restype = ctypes.c_int
        lib.pzl_moe_ffn_staged.argtypes = [vp, vp, vp, vp, i32, i32, vp, vp, ctypes.c_size_t, vp, vp]
        lib.pzl_layer_force_plan.restype = ctypes.c_int
        lib.pzl_layer_force_plan.argtypes = [vp, i32, i32, i32]
        lib.pzl_layer_h_info.restype = ctypes.c_int
        lib.pzl_layer_h_info.argtypes = [vp, ctypes.POINTER(i32), ctypes.POINTER(i32)]
        lib.pzl_moe_ffn_workspace_layout.restype = ctypes.c_int
        lib.pzl_moe_ffn_workspace_layout.argtypes = [vp, i32, i32, ctypes.POINTER(_WorkspaceLayout)]
        lib.pzl_moe_ffn_static.restype = ctypes.c_int
        lib.pzl_moe_ffn_static.argtypes = [vp, vp, vp, vp, i32, i32, vp, vp]
        lib.pzl_moe_ffn_static_max_bytes.restype = ctypes.c_size_t
        _lib = lib
    return _lib


def _check(rc, where):
    if rc != PZL_OK:
        raise PzlError(rc, where)


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, dtypes, name):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous() and t.dtype in dtypes):
        raise TypeError("%s must be a contiguous CUDA tensor of dtype %s" % (name, dtypes))
    return ctypes.c_void_p(t.data_ptr())


_BITS16 = (torch.int16, torch.bfloat16, torch.uint16)


def pzl_packed_bytes(rows, cols):
    return load().pzl_packed_bytes(rows, cols)


def pzl_pack(merged, mask0, mask1, sign0, sign1, out=None, n_out_of_range=None):
    """pack(merged weights, masks, signs) -> packed tensor (int16, tiled order, rows*cols elements)."""
    rows, cols = merged.shape
    if out is None:
        out = torch.empty(rows * cols, dtype=torch.int16, device=merged.device)
    for m in (mask0, mask1, sign0, sign1):
        if tuple(m.shape) != (rows, cols):
            raise ValueError("mask/sign planes must have the shape of merged")
    cnt = ctypes.c_void_p(0) if n_out_of_range is None else _dev(n_out_of_range, (torch.int32,), "n_out_of_range")
    rc = load().pzl_pack(_dev(merged, _BITS16, "merged"), _dev(mask0, (torch.uint8,), "mask0"),
                         _dev(mask1, (torch.uint8,), "mask1"), _dev(sign0, (torch.uint8,), "sign0"),
                         _dev(sign1, (torch.uint8,), "sign1"), rows, cols, _dev(out, _BITS16, "out"),
                         cnt, _stream())
    _check(rc, "pzl_pack")
    return out


def pzl_unpack(packed, expert_pos, rows, cols, out=None):
    """Algorithm 1 decode of one expert of the pair -> bfloat16 [rows, cols], row-major."""
    if packed.numel() != rows * cols:
        raise ValueError("packed tensor does not hold rows*cols elements")
    if out is None:
        out = torch.empty(rows, cols, dtype=torch.bfloat16, device=packed.device)
    rc = load().pzl_unpack(_dev(packed, _BITS16, "packed"), int(expert_pos), rows, cols,
                           _dev(out, _BITS16, "out"), _stream())
    _check(rc, "pzl_unpack")
    return out


def pzl_unpack_half_x2(packed, expert_pos, rows, cols):
    """The half-precision form of the decode (each weight times 2) -> float16 [rows, cols], row-major."""
    if packed.numel() != rows * cols:
        raise ValueError("packed tensor does not hold rows*cols elements")
    out = torch.empty(rows, cols, dtype=torch.float16, device=packed.device)
    rc = load().pzl_unpack_half_x2(_dev(packed, _BITS16, "packed"), int(expert_pos), rows, cols,
                                   _dev(out, (torch.float16,), "out"), _stream())
    _check(rc, "pzl_unpack_half_x2")
    return out


def pzl_q_pack(merged, mask0, mask1, sign0, sign1, n_non_finite=None):
    """Quantised pack -> (records uint8 [pzl_q_record_bytes], scales int16 bf16 bits [rows/16, cols/128, 16])."""
    rows, cols = merged.shape
    lib = load()
    lib.pzl_q_record_bytes.restype = ctypes.c_size_t
    lib.pzl_q_scale_bytes.restype = ctypes.c_size_t
    nrec = lib.pzl_q_record_bytes(ctypes.c_int64(rows), ctypes.c_int64(cols))
    nsc = lib.pzl_q_scale_bytes(ctypes.c_int64(rows), ctypes.c_int64(cols))
    if nrec == 0:
        raise ValueError("quantised format needs rows % 16 == 0 and cols % 128 == 0")
    records = torch.zeros(nrec, dtype=torch.uint8, device=merged.device)
    scales = torch.empty(nsc // 2, dtype=torch.int16, device=merged.device)
    cnt = ctypes.c_void_p(0) if n_non_finite is None else _dev(n_non_finite, (torch.int32,), "n_non_finite")
    rc = lib.pzl_q_pack(_dev(merged, _BITS16, "merged"), _dev(mask0, (torch.uint8,), "mask0"),
                        _dev(mask1, (torch.uint8,), "mask1"), _dev(sign0, (torch.uint8,), "sign0"),
                        _dev(sign1, (torch.uint8,), "sign1"), ctypes.c_int64(rows), ctypes.c_int64(cols),
                        _dev(records, (torch.uint8,), "records"), _dev(scales, _BITS16, "scales"), cnt, _stream())
    _check(rc, "pzl_q_pack")
    return records, scales


def pzl_q_unpack(records, scales, expert_pos, rows, cols):
    """Reconstructed weights of one expert of a quantised pair -> float32 [rows, cols], row-major."""
    out = torch.empty(rows, cols, dtype=torch.float32, device=records.device)
    rc = load().pzl_q_unpack(_dev(records, (torch.uint8,), "records"), _dev(scales, _BITS16, "scales"),
                             int(expert_pos), ctypes.c_int64(rows), ctypes.c_int64(cols),
                             _dev(out, (torch.float32,), "out"), _stream())
    _check(rc, "pzl_q_unpack")
    return out


def q_records_to_logical(records, rows, cols):
    """Host view of a record array (numpy uint8, as written by pzl_q_pack): the 53-bit records as
    uint64 [rows, cols/8] in plain row-major record order (a layout change only)."""
    import numpy as np
    rec = np.asarray(records, dtype=np.uint8)
    kb_total = cols // 32
    n_tiles = (rows // 16) * kb_total
    out = np.zeros((rows, cols // 8), dtype=np.uint64)
    lanes = np.arange(64)
    byte0 = (53 * lanes) >> 3
    shift = ((53 * lanes) & 7).astype(np.uint64)
    pow8 = (np.uint64(8) * np.arange(8, dtype=np.uint64))
    for t in range(n_tiles):
        base = t * 424
        idx = base + byte0[:, None] + np.arange(8)[None, :]
        v = (rec[idx].astype(np.uint64) << pow8[None, :]).sum(axis=1, dtype=np.uint64)
        v = (v >> shift) & np.uint64((1 << 53) - 1)
        rt, kb = divmod(t, kb_total)
        out[rt * 16 + (lanes & 15), kb * 4 + (lanes >> 4)] = v
    return out


def q_scales_to_logical(scales, rows, cols):
    """Scale array [rows/16, cols/128, 16] -> [rows, cols/128] (a layout change only)."""
    import numpy as np
    s = np.asarray(scales).reshape(rows // 16, cols // 128, 16)
    return np.ascontiguousarray(s.transpose(0, 2, 1)).reshape(rows, cols // 128)


def pzl_tile_dense(dense, out=None):
    rows, cols = dense.shape
    if out is None:
        out = torch.empty(rows * cols, dtype=dense.dtype, device=dense.device)
    rc = load().pzl_tile_dense(_dev(dense, _BITS16, "dense"), rows, cols, _dev(out, _BITS16, "out"), _stream())
    _check(rc, "pzl_tile_dense")
    return out


def pzl_merge_pack(w_i, w_j, norm_i, norm_j, tau_sim, out=None, n_similar=None, n_out_of_range=None):
    """Offline dual-mask merge of two expert matrices fused with pack -> packed pair (tiled order)."""
    rows, cols = w_i.shape
    if tuple(w_j.shape) != (rows, cols) or norm_i.numel() != cols or norm_j.numel() != cols:
        raise ValueError("w_i, w_j must share a shape and the norms must have one entry per column")
    if out is None:
        out = torch.empty(rows * cols, dtype=torch.int16, device=w_i.device)
    opt = lambda t, name: ctypes.c_void_p(0) if t is None else _dev(t, (torch.int32,), name)
    rc = load().pzl_merge_pack(_dev(w_i, _BITS16, "w_i"), _dev(w_j, _BITS16, "w_j"),
                               _dev(norm_i, (torch.float32,), "norm_i"), _dev(norm_j, (torch.float32,), "norm_j"),
                               rows, cols, ctypes.c_float(tau_sim), _dev(out, _BITS16, "out"),
                               opt(n_similar, "n_similar"), opt(n_out_of_range, "n_out_of_range"), _stream())
    _check(rc, "pzl_merge_pack")
    return out


def pzl_moe_ffn_plan(n_experts, d_model, d_ffn, T, k, shared_d_ffn=(), n_unmerged=0, quantised=False):
    """The host-side launch plan of pzl_moe_ffn for this layer and batch shape (no GPU needed) as a dict."""
    sf = (ctypes.c_int32 * max(len(shared_d_ffn), 1))(*shared_d_ffn)
    shape = _LayerShape(int(n_experts), int(n_unmerged), int(d_model), int(d_ffn), len(shared_d_ffn),
                        ctypes.cast(sf, ctypes.POINTER(ctypes.c_int32)), 1 if quantised else 0)
    plan = _Plan()
    _check(load().pzl_moe_ffn_plan(ctypes.byref(shape), int(T), int(k), ctypes.byref(plan)), "pzl_moe_ffn_plan")
    out = {n: int(getattr(plan, n)) for n, _ in _Plan._fields_[:10]}
    out["shared_token_tiles"] = list(plan.shared_token_tiles)[:len(shared_d_ffn)]
    out["shared_tile_tokens"] = list(plan.shared_tile_tokens)[:len(shared_d_ffn)]
    out["grouping_in_kernel"] = int(plan.grouping_in_kernel)
    return out


def pzl_router_topk(x, w_router, k):
    """Linear router + top-k + softmax over the selected logits -> (ids int32 [T,k], weights fp32 [T,k])."""
    T, d = x.shape
    E = w_router.shape[0]
    ids = torch.empty(T, k, dtype=torch.int32, device=x.device)
    w = torch.empty(T, k, dtype=torch.float32, device=x.device)
    rc = load().pzl_router_topk(_dev(x, _BITS16, "x"), _dev(w_router, _BITS16, "w_router"), T, d, E, k,
                                _dev(ids, (torch.int32,), "ids"), _dev(w, (torch.float32,), "w"), _stream())
    _check(rc, "pzl_router_topk")
    return ids, w


def _ptr_table(tensors):
    return (ctypes.c_void_p * max(len(tensors), 1))(*[t.data_ptr() for t in tensors])


class Layer:
    """Owns a pzl_layer handle and keeps the weight tensors it references alive."""

    def __init__(self, d_model, d_ffn, expert_pair, expert_pos, gate, up, down, shared=(), dense=(),
                 quantised=False, wide_h=False):
        """gate/up/down: one packed tensor per pair -- or, with quantised=True, one (records, scales)
        pair of tensors per pair as returned by pzl_q_pack; shared: (gate, up, down, f) tiled dense
        per shared expert; dense: (gate, up, down) tiled dense per routed expert kept unmerged."""
        self.d_model, self.d_ffn = int(d_model), int(d_ffn)
        scales = None
        if quantised:
            scales = [[t[1] for t in ws] for ws in (gate, up, down)]
            gate, up, down = ([t[0] for t in ws] for ws in (gate, up, down))
        self._keep = (list(gate), list(up), list(down), [tuple(s) for s in shared], [tuple(s) for s in dense], scales)
        pair = np.ascontiguousarray(expert_pair, dtype=np.int32)
        pos = np.ascontiguousarray(expert_pos, dtype=np.uint8)
        P = len(gate)
        for name, ws, shape in (("gate", gate, d_ffn * d_model), ("up", up, d_ffn * d_model),
                                ("down", down, d_model * d_ffn)):
            if len(ws) != P:
                raise ValueError("need one %s tensor per pair" % name)
            for t in ws:
                if quantised:
                    _dev(t, (torch.uint8,), name)
                    if t.numel() != shape // 512 * 424 + 8:
                        raise ValueError("%s record array has the wrong size" % name)
                    continue
                _dev(t, _BITS16, name)
                if t.numel() != shape:
                    raise ValueError("%s tensor has the wrong size" % name)
        sf = np.array([int(s[3]) for s in shared], dtype=np.int32)
        for g, u, dn, fs in shared:
            for t in (g, u, dn):
                _dev(t, _BITS16, "shared weight")
                if t.numel() != fs * d_model:
                    raise ValueError("shared weight has the wrong size")
        for g, u, dn in dense:
            for t in (g, u, dn):
                _dev(t, _BITS16, "unmerged expert weight")
                if t.numel() != d_ffn * d_model:
                    raise ValueError("unmerged expert weight has the wrong size")
        self._tables = (pair, pos, sf, _ptr_table(gate), _ptr_table(up), _ptr_table(down),
                        _ptr_table([s[0] for s in shared]), _ptr_table([s[1] for s in shared]),
                        _ptr_table([s[2] for s in shared]),
                        _ptr_table([s[0] for s in dense]), _ptr_table([s[1] for s in dense]),
                        _ptr_table([s[2] for s in dense]))
        d = _LayerDesc()
        d.n_experts, d.d_model, d.d_ffn = int(pair.size), self.d_model, self.d_ffn
        d.expert_pair, d.expert_pos = pair.ctypes.data, pos.ctypes.data
        cast = lambda a: ctypes.cast(a, ctypes.c_void_p)
        d.gate, d.up, d.down = cast(self._tables[3]), cast(self._tables[4]), cast(self._tables[5])
        d.n_shared = len(shared)
        d.shared_d_ffn = sf.ctypes.data if len(shared) else None
        d.shared_gate, d.shared_up, d.shared_down = (cast(self._tables[6]), cast(self._tables[7]),
                                                     cast(self._tables[8]))
        d.n_dense = len(dense)
        d.dense_gate, d.dense_up, d.dense_down = (cast(self._tables[9]), cast(self._tables[10]),
                                                  cast(self._tables[11]))
        if quantised:
            for ws in scales:
                for t in ws:
                    _dev(t, _BITS16, "scale array")
                    if t.numel() != d_ffn * d_model // 128:
                        raise ValueError("scale array has the wrong size")
            self._scale_tables = tuple(_ptr_table(ws) for ws in scales)
            d.pair_format = 1
            d.gate_scale, d.up_scale, d.down_scale = (cast(t) for t in self._scale_tables)
        d.h_precision = 1 if wide_h else 0
        self._h = ctypes.c_void_p()
        _check(load().pzl_layer_create(ctypes.byref(d), ctypes.byref(self._h)), "pzl_layer_create")
        self._ws = None

    def close(self):
        if getattr(self, "_h", None) is not None and self._h:
            if _lib is not None:                 # (None again while the interpreter shuts down)
                _lib.pzl_layer_destroy(self._h)
            self._h = None

    __del__ = close

    def pzl_moe_ffn_workspace_bytes(self, max_tokens, top_k):
        return load().pzl_moe_ffn_workspace_bytes(self._h, int(max_tokens), int(top_k))

    def pzl_layer_force_plan(self, hybrid=-1, persistent=-1, tile_stream=-1):
        """Override (1 / 0) or release (-1) the library's choice of kernels and launch form for later calls."""
        _check(load().pzl_layer_force_plan(self._h, int(hybrid), int(persistent), int(tile_stream)), "pzl_layer_force_plan")

    def h_info(self):
        """(H of the packed pairs is one half-precision plane, wavefronts that saturated a value of H so far)."""
        half, sat = ctypes.c_int32(), ctypes.c_int32()
        _check(load().pzl_layer_h_info(self._h, ctypes.byref(half), ctypes.byref(sat)), "pzl_layer_h_info")
        return bool(half.value), int(sat.value)

    def routing_tables(self, T, k):
        """The routing tables the last pzl_moe_ffn call with this (T, k) left in the layer's own
        workspace, as numpy arrays (a read-back for inspection; synchronises)."""
        lay = _WorkspaceLayout()
        _check(load().pzl_moe_ffn_workspace_layout(self._h, int(T), int(k), ctypes.byref(lay)),
               "pzl_moe_ffn_workspace_layout")
        torch.cuda.synchronize()
        ws = self._ws[:lay.total].cpu().numpy()
        N = T * k

        def tab(off, n):
            return ws[off:off + 4 * n].view(np.int32).copy()
        n_tiles = int(tab(lay.n_tiles, 1)[0])
        return {"n_keys": lay.n_keys, "first_slot": tab(lay.first_slot, lay.n_keys + 1),
                "streamed_count": tab(lay.streamed_count, lay.n_keys),
                "slot_token": tab(lay.slot_token, N), "slot_of": tab(lay.slot_of, N).reshape(T, k),
                "n_tiles": n_tiles, "tile_key": tab(lay.tile_key, n_tiles),
                "tile_first_slot": tab(lay.tile_first_slot, n_tiles), "tile_tokens": tab(lay.tile_tokens, n_tiles)}

    def pzl_moe_ffn_static(self, x, topk_ids, topk_w, y):
        """pzl_moe_ffn on the library's static scratch array: no workspace, no allocation (y is the caller's)."""
        T = x.shape[0]
        k = topk_ids.shape[1] if topk_ids.dim() == 2 else 0
        _check(load().pzl_moe_ffn_static(self._h, _dev(x, _BITS16, "x"), _dev(topk_ids, (torch.int32,), "topk_ids"),
                                         _dev(topk_w, (torch.float32,), "topk_w"), T, k, _dev(y, _BITS16, "y"),
                                         _stream()), "pzl_moe_ffn_static")
        return y

    def pzl_moe_ffn(self, x, topk_ids, topk_w, y=None, workspace=None, stage_events=None):
        """moe_ffn(x, router top-k ids/weights, packed experts) -> y (bfloat16 [T, d_model]).

        stage_events: optional ctypes array of 2*len(STAGES) hipEvent_t handles (0 = skip); when
        given, the call goes through pzl_moe_ffn_staged."""
        T = x.shape[0]
        k = topk_ids.shape[1] if topk_ids.dim() == 2 else 0
        if y is None:
            y = torch.empty(T, self.d_model, dtype=torch.bfloat16, device=x.device)
        if T == 0:
            return y
        if workspace is None:
            need = self.pzl_moe_ffn_workspace_bytes(T, k)
            if self._ws is None or self._ws.numel() < need:
                self._ws = torch.empty(need, dtype=torch.uint8, device=x.device)
            workspace = self._ws
        args = (self._h, _dev(x, _BITS16, "x"), _dev(topk_ids, (torch.int32,), "topk_ids"),
                _dev(topk_w, (torch.float32,), "topk_w"), T, k, _dev(y, _BITS16, "y"),
                _dev(workspace, (torch.uint8,), "workspace"), workspace.numel(), _stream())
        if stage_events is None:
            _check(load().pzl_moe_ffn(*args), "pzl_moe_ffn")
        else:
            _check(load().pzl_moe_ffn_staged(*args, ctypes.cast(stage_events, ctypes.c_void_p)),
                   "pzl_moe_ffn_staged")
        return y


def pzl_moe_ffn_static_max_bytes():
    return load().pzl_moe_ffn_static_max_bytes()


def tiled_to_logical(tiled, rows, cols):
    """Undo the 16x32 tiled order of a packed / tiled tensor (numpy, layout only)."""
    a = np.asarray(tiled).reshape(rows // 16, cols // 32, 4, 16, 8)       # [rt, kb, kgroup, r, j]
    return np.ascontiguousarray(a.transpose(0, 3, 1, 2, 4)).reshape(rows, cols)
