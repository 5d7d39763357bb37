"""CPU oracle for the bit-packed merged-expert MoE FFN.  TEST INFRASTRUCTURE ONLY.

Thin ctypes access to ``puzzle_oracle.c`` (plain C, fp64).  Nothing in the product
package may import this module; only tests, the smoke check and the benchmark's
CPU-baseline leg do.  It shares no code with the HIP library.

Paper passages: Sec. 3.3.2 (packed word, exponent rule), Algorithm 1 (decode),
Eq. 6 (reconstruction).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "puzzle_oracle.c")
_SRC_Q = os.path.join(_HERE, "quant_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force=False):
    """Compile the oracle with gcc (no fast-math: fp64 sums stay in source order)."""
    newest = max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_Q))
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
                               "-o", _LIB, _SRC, _SRC_Q, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        u16p = ctypes.POINTER(ctypes.c_uint16)
        u8p = ctypes.POINTER(ctypes.c_uint8)
        lib.orc_bf16_to_double.restype = ctypes.c_double
        lib.orc_bf16_to_double.argtypes = [ctypes.c_uint16]
        lib.orc_bf16_from_double.restype = ctypes.c_uint16
        lib.orc_bf16_from_double.argtypes = [ctypes.c_double]
        lib.orc_pack.restype = ctypes.c_int64
        lib.orc_pack.argtypes = [u16p, u8p, u8p, u8p, u8p, ctypes.c_int64, u16p]
        lib.orc_unpack.restype = None
        lib.orc_unpack.argtypes = [u16p, ctypes.c_int, ctypes.c_int64, u16p]
        lib.orc_moe_ffn.restype = ctypes.c_int
        f32p = ctypes.POINTER(ctypes.c_float)
        lib.orc_merge.restype = ctypes.c_int64
        lib.orc_merge.argtypes = [u16p, u16p, f32p, f32p, ctypes.c_int64, ctypes.c_int64, ctypes.c_float,
                                  u16p, u8p, u8p, u8p, u8p]
        _lib = lib
    return _lib


def _u16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def _u8(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint8, a.dtype
    return a


def _ptr(a, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def bf16_to_double(bits):
    return _load().orc_bf16_to_double(int(bits))


def bf16_from_double(v):
    return _load().orc_bf16_from_double(float(v))


def pack(merged, mask0, mask1, sign0, sign1):
    """Sec. 3.3.2 pack.  Returns (packed uint16 array of merged's shape, n_out_of_range)."""
    merged = _u16(merged)
    m0, m1, s0, s1 = (_u8(a) for a in (mask0, mask1, sign0, sign1))
    for a in (m0, m1, s0, s1):
        assert a.shape == merged.shape
    out = np.empty_like(merged)
    bad = _load().orc_pack(_ptr(merged, ctypes.c_uint16), _ptr(m0, ctypes.c_uint8),
                           _ptr(m1, ctypes.c_uint8), _ptr(s0, ctypes.c_uint8),
                           _ptr(s1, ctypes.c_uint8), merged.size, _ptr(out, ctypes.c_uint16))
    return out, int(bad)


def unpack(packed, expert_pos):
    """Algorithm 1 on every element.  Returns bf16 bit patterns (uint16)."""
    packed = _u16(packed)
    assert expert_pos in (0, 1)
    out = np.empty_like(packed)
    _load().orc_unpack(_ptr(packed, ctypes.c_uint16), int(expert_pos), packed.size,
                       _ptr(out, ctypes.c_uint16))
    return out


def merge(wi, wj, norm_i, norm_j, tau):
    """Offline dual-mask merge of two expert matrices (Sec. 3.2, Eqs. 1-5).

    wi, wj: [rows, cols] bf16 bits; norm_i, norm_j: [cols] float32 activation norms.
    Returns dict(merged, mask0, mask1, sign0, sign1, n_similar); position 0 is expert i.
    """
    wi, wj = _u16(wi), _u16(wj)
    assert wi.shape == wj.shape and wi.ndim == 2
    rows, cols = wi.shape
    ni = np.ascontiguousarray(norm_i, dtype=np.float32)
    nj = np.ascontiguousarray(norm_j, dtype=np.float32)
    assert ni.shape == (cols,) and nj.shape == (cols,)
    merged = np.empty_like(wi)
    planes = [np.empty(wi.shape, dtype=np.uint8) for _ in range(4)]
    f32p = ctypes.POINTER(ctypes.c_float)
    n_sim = _load().orc_merge(_ptr(wi, ctypes.c_uint16), _ptr(wj, ctypes.c_uint16),
                              ni.ctypes.data_as(f32p), nj.ctypes.data_as(f32p), rows, cols,
                              ctypes.c_float(tau), _ptr(merged, ctypes.c_uint16),
                              *[_ptr(p, ctypes.c_uint8) for p in planes])
    return {"merged": merged, "mask0": planes[0], "mask1": planes[1], "sign0": planes[2],
            "sign1": planes[3], "n_similar": int(n_sim)}


def router_topk(x, w_router, k):
    """Linear router + top-k + softmax over the selected logits.  x [T,d], w_router [E,d] bf16 bits.
    Returns (ids int32 [T,k], weights float32 [T,k], logits float32 [T,E])."""
    x, wr = _u16(x), _u16(w_router)
    T, d = x.shape
    E = wr.shape[0]
    assert wr.shape == (E, d) and 1 <= k <= min(E, 64)
    ids = np.empty((T, k), dtype=np.int32)
    wts = np.empty((T, k), dtype=np.float32)
    logits = np.empty((T, E), dtype=np.float32)
    lib = _load()
    lib.orc_router_topk.restype = ctypes.c_int
    rc = lib.orc_router_topk(ctypes.c_int(T), ctypes.c_int(d), ctypes.c_int(E), ctypes.c_int(k),
                             ctypes.c_void_p(x.ctypes.data), ctypes.c_void_p(wr.ctypes.data),
                             ctypes.c_void_p(ids.ctypes.data), ctypes.c_void_p(wts.ctypes.data),
                             ctypes.c_void_p(logits.ctypes.data))
    if rc != 0:
        raise ValueError("oracle router_topk: bad k")
    return ids, wts, logits


def moe_ffn(x, ids, w, expert_pair, expert_pos, gate, up, down,
            shared=(), stage_h_bf16=False, dense=()):
    """Routed SwiGLU FFN over Eq. 6-decoded experts, fp64.

    x: [T,d] bf16 bits (uint16); ids: [T,k] int32; w: [T,k] float32;
    gate/up: per pair, packed uint16 [f,d] in logical order; down: per pair [d,f];
    shared: sequence of (gate [fs,d], up [fs,d], down [d,fs]) dense bf16 bits.
    dense: routed experts kept unmerged, sequence of (gate [f,d], up [f,d], down [d,f]) dense bf16
    bits; expert e with expert_pair[e] = -1-j uses dense[j].
    Returns (y_f64 [T,d], y_bf16_bits [T,d]).
    """
    lib = _load()
    x = _u16(x)
    T, d = x.shape
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    w = np.ascontiguousarray(w, dtype=np.float32)
    k = ids.shape[1] if ids.ndim == 2 else 0
    assert ids.shape == (T, k) and w.shape == (T, k)
    expert_pair = np.ascontiguousarray(expert_pair, dtype=np.int32)
    expert_pos = np.ascontiguousarray(expert_pos, dtype=np.uint8)
    E = expert_pair.size
    gate = [_u16(a) for a in gate]
    up = [_u16(a) for a in up]
    down = [_u16(a) for a in down]
    P = len(gate)
    dg = [_u16(s_[0]) for s_ in dense]
    du = [_u16(s_[1]) for s_ in dense]
    dd = [_u16(s_[2]) for s_ in dense]
    f = gate[0].shape[0] if P else (dg[0].shape[0] if dg else 0)
    for a, b, c in zip(dg, du, dd):
        assert a.shape == (f, d) and b.shape == (f, d) and c.shape == (d, f)
    for a, b, c in zip(gate, up, down):
        assert a.shape == (f, d) and b.shape == (f, d) and c.shape == (d, f)
    sg = [_u16(s[0]) for s in shared]
    su = [_u16(s[1]) for s in shared]
    sd = [_u16(s[2]) for s in shared]
    sf = np.array([a.shape[0] for a in sg], dtype=np.int32)
    for a, b, c in zip(sg, su, sd):
        assert a.shape[1] == d and b.shape == a.shape and c.shape == (d, a.shape[0])

    def ptr_array(arrs):
        arr_t = ctypes.c_void_p * max(len(arrs), 1)
        return arr_t(*[a.ctypes.data for a in arrs])

    y64 = np.zeros((T, d), dtype=np.float64)
    ybf = np.zeros((T, d), dtype=np.uint16)
    rc = lib.orc_moe_ffn(
        ctypes.c_int(T), ctypes.c_int(k), ctypes.c_int(E), ctypes.c_int(d), ctypes.c_int(f),
        ctypes.c_void_p(x.ctypes.data), ctypes.c_void_p(ids.ctypes.data),
        ctypes.c_void_p(w.ctypes.data), ctypes.c_void_p(expert_pair.ctypes.data),
        ctypes.c_void_p(expert_pos.ctypes.data),
        ptr_array(gate), ptr_array(up), ptr_array(down),
        ctypes.c_int(len(dg)), ptr_array(dg), ptr_array(du), ptr_array(dd),
        ctypes.c_int(len(sg)), ctypes.c_void_p(sf.ctypes.data),
        ptr_array(sg), ptr_array(su), ptr_array(sd),
        ctypes.c_int(1 if stage_h_bf16 else 0),
        ctypes.c_void_p(y64.ctypes.data), ctypes.c_void_p(ybf.ctypes.data))
    if rc != 0:
        raise ValueError("oracle moe_ffn: expert id out of range or allocation failure")
    return y64, ybf


# ---------- quantised variant (appendix "Combining PuzzleMoE with Quantization") ----------

def q_quantise(merged, mask0, mask1, sign0, sign1):
    """3-bit group-128 quantisation of a merged matrix with its masks and signs.

    Returns dict(code, trit, s0, s1 (uint8 [rows, cols]), scale (uint16 bf16 bits [rows, cols/128]),
    n_bad)."""
    merged = _u16(merged)
    rows, cols = merged.shape
    assert cols % 128 == 0
    m0, m1, s0, s1 = (_u8(a) for a in (mask0, mask1, sign0, sign1))
    out = {k: np.empty(merged.shape, dtype=np.uint8) for k in ("code", "trit", "s0", "s1")}
    scale = np.empty((rows, cols // 128), dtype=np.uint16)
    lib = _load()
    lib.orc_q_quantise.restype = ctypes.c_int64
    bad = lib.orc_q_quantise(*[ctypes.c_void_p(a.ctypes.data) for a in (merged, m0, m1, s0, s1)],
                             ctypes.c_int64(rows), ctypes.c_int64(cols),
                             *[ctypes.c_void_p(out[k].ctypes.data) for k in ("code", "trit", "s0", "s1")],
                             ctypes.c_void_p(scale.ctypes.data))
    out["scale"] = scale
    out["n_bad"] = int(bad)
    return out


def q_dequantise(q, pos):
    """Reconstructed weights of expert `pos` of the pair, fp64 [rows, cols] (exact code * scale)."""
    rows, cols = q["code"].shape
    out = np.empty((rows, cols), dtype=np.float64)
    lib = _load()
    lib.orc_q_dequantise.restype = None
    lib.orc_q_dequantise(*[ctypes.c_void_p(q[k].ctypes.data) for k in ("code", "trit", "s0", "s1", "scale")],
                         ctypes.c_int(pos), ctypes.c_int64(rows), ctypes.c_int64(cols),
                         ctypes.c_void_p(out.ctypes.data))
    return out


def q_records(q):
    """The stored 53-bit records, uint64 [rows, cols/8], in plain row-major record order."""
    rows, cols = q["code"].shape
    out = np.empty((rows, cols // 8), dtype=np.uint64)
    lib = _load()
    lib.orc_q_records.restype = None
    lib.orc_q_records(*[ctypes.c_void_p(q[k].ctypes.data) for k in ("code", "trit", "s0", "s1")],
                      ctypes.c_int64(rows), ctypes.c_int64(cols), ctypes.c_void_p(out.ctypes.data))
    return out


def q_bits_per_weight():
    lib = _load()
    lib.orc_q_bits_per_weight.restype = ctypes.c_double
    return lib.orc_q_bits_per_weight()


def ffn_dense64(x, ids, w, gate, up, down):
    """Routed SwiGLU FFN with per-expert fp64 weight matrices (gate/up [f,d], down [d,f])."""
    x = _u16(x)
    T, d = x.shape
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    w = np.ascontiguousarray(w, dtype=np.float32)
    k = ids.shape[1]
    gate = [np.ascontiguousarray(a, dtype=np.float64) for a in gate]
    up = [np.ascontiguousarray(a, dtype=np.float64) for a in up]
    down = [np.ascontiguousarray(a, dtype=np.float64) for a in down]
    E = len(gate)
    f = gate[0].shape[0]
    for a, b, c in zip(gate, up, down):
        assert a.shape == (f, d) and b.shape == (f, d) and c.shape == (d, f)
    arr_t = ctypes.c_void_p * E
    y64 = np.zeros((T, d), dtype=np.float64)
    lib = _load()
    lib.orc_ffn_dense64.restype = ctypes.c_int
    rc = lib.orc_ffn_dense64(ctypes.c_int(T), ctypes.c_int(k), ctypes.c_int(E), ctypes.c_int(d), ctypes.c_int(f),
                             ctypes.c_void_p(x.ctypes.data), ctypes.c_void_p(ids.ctypes.data),
                             ctypes.c_void_p(w.ctypes.data), arr_t(*[a.ctypes.data for a in gate]),
                             arr_t(*[a.ctypes.data for a in up]), arr_t(*[a.ctypes.data for a in down]),
                             ctypes.c_void_p(y64.ctypes.data))
    if rc != 0:
        raise ValueError("oracle ffn_dense64: expert id out of range or allocation failure")
    return y64
