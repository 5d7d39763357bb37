// Weight-streaming decode-GEMM for small token counts per expert pair (decode-time batches).
//
// Sec. 3.3.2: every packed weight is decoded (Algorithm 1) right before it is multiplied, the
// decoded matrix is never materialised, and ONE read of a packed tile produces the outputs of
// both experts of the pair.  On gfx950 that becomes: each wavefront streams 16-row x 32-col
// packed tiles (1 KiB contiguous, one 128-bit load per lane) straight into registers in
// matrix-core operand order, decodes them for position 0 and position 1 with packed 16-bit
// integer ops, and feeds v_mfma_f32_16x16x32_bf16 with the tokens of each expert as the
// other operand.  The kernels are HBM-bound: their job is to keep the load queue full and
// the decode under the VALU budget.
//
// Every wave owns two weight streams: in the gate/up stage the same row tile of the gate and
// of the up matrix (SwiGLU needs both), in the down stage two adjacent row tiles of the down
// matrix.  A workgroup is 8 waves (two per SIMD) sharing the staged activations in LDS
// (double-buffered chunks of k-blocks); 8 waves measured 5-9 % faster than 4 per workgroup.  Token tiles: up to SG_MAX_TILES tiles of 16 tokens per pass, the tiles
// of position 0 first; longer token lists take further passes (re-streaming the weights) —
// only a fallback, large batches belong to the tiled GEMM path.
//
// The SwiGLU output H needs more than bf16's 8 significant bits: one bf16 plane alone would put
// its rounding (2^-9 relative per element) straight into y and leave no margin under the 1e-2
// output tolerance.  Two forms (template parameter HALF):
//   HALF   one plane of IEEE half precision (11 significant bits; values beyond +-65504 saturate and
//          are counted).  The down stage then decodes the packed words to half precision too (the
//          stored 5-bit exponent field is half precision's own, see pzl_decode.h; the weights come
//          out multiplied by 2, the accumulators are halved at the end) and uses the f16 matrix
//          instruction.  For packed pairs whose down matrices hold no exponent field above 29.
//   !HALF  two bf16 planes, hi = bf16(h) and lo = bf16(h - hi), both multiplied by bf16 weights:
//          twice the matrix instructions and LDS traffic in the down stage, any range.
#include <atomic>
#include "pzl_common.h"
#include "pzl_decode.h"

namespace pzl {

#ifndef SG_DEPTH_N
#define SG_DEPTH_N 4
#endif
#ifndef SG_SCHED_BARRIER
#define SG_SCHED_BARRIER 1
#endif
#ifndef SG_DEPTH_GATEUP
#define SG_DEPTH_GATEUP SG_DEPTH_N
#endif
#ifndef SG_DEPTH_QUANT_GATEUP
#define SG_DEPTH_QUANT_GATEUP 4
#endif
#ifndef SG_PLAIN_LOADS
#define SG_PLAIN_LOADS 0
#endif
#ifndef SG_WAVES_N
#define SG_WAVES_N 8
#endif
#if SG_PLAIN_LOADS
#define SG_WLOAD(p) (*(p))
#else
#define SG_WLOAD(p) __builtin_nontemporal_load(p)
#endif
constexpr int SG_WAVES = SG_WAVES_N;
constexpr int SG_THREADS = SG_WAVES * 64;
constexpr int SG_DEPTH = SG_DEPTH_N;   // weight k-blocks in flight per stream
constexpr int SG_MAX_TILES = 4;        // token tiles per pass (both positions together)
constexpr int SG_POS_TILES = 2;        // token tiles per pass per position (routed groups)
constexpr int SG_FRAGS = 32;           // staged 1 KiB fragments per LDS buffer
constexpr int SG_LDS_BYTES = 2 * SG_FRAGS * 64 * 16;   // 64 KiB, two buffers
constexpr int STAGE_GATEUP = 0, STAGE_DOWN = 1;
constexpr int SG_RESIDENT_WGS = 2048 / SG_WAVES;   // 256 CUs x 8 waves

// Routing done by the gate/up kernel itself (FUSE, small batches; see route_in_block).
struct SgRoute {
    const int32_t *ids, *q_of_expert;        // [n_flat] expert ids, [n_experts] expert -> routing key
    int32_t n_flat, k, n_experts, n_keys;
    int32_t *cnt, *off, *slot_tok, *slot_of; // the workspace's routing tables, written by workgroup 0 for the kernels that follow
};

struct SgArgs {
    const uint16_t *const *w_a;
    const uint16_t *const *w_b;
    const uint16_t *const *s_a;  // quantised pairs: scale arrays of w_a / w_b
    const uint16_t *const *s_b;
    int32_t rows, kdim, ksplit, rg_per_wg;
    const uint16_t *act;
    int64_t act_plane_stride;
    int32_t act_is_x, act_slot_base;
    const int32_t *cnt, *off, *slot_tok;
    int32_t group_base;          // routed groups: first group index (q = 2 * (group_base + g) + pos)
    int32_t dense_tokens, dense_slot_base;
    int32_t n_passes;            // workgroups per (group, rows, K split): workgroup p takes the token passes p, p + n_passes, ...
    uint16_t *h_out;
    int64_t h_plane_stride;
    int32_t h_slot_base;
    float *o_out;
    int64_t o_ks_stride;
    int32_t *h_saturated;        // gate/up stage, half-precision H: counts waves that saturated a value (may be null)
    SgRoute route;               // FUSE only
};

// One 16x32 tile (8 elements per lane) decoded for position POS: as bf16, or (HALFW) as half
// precision times 2.  DENSE: the weights are plain bf16 already.
template <int POS, bool DENSE, bool HALFW>
__device__ __forceinline__ u32x4 decode_frag(u32x4 w)
{
    if (DENSE) return w;
    u32x4 o;
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = decode_pair<POS>(w[i], HALFW ? decode_body_half_x2(w[i]) : decode_body(w[i]));
    return o;
}

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 sg_f16x2 __attribute__((ext_vector_type(2)));

// acc += A (16 rows x 32 k) * B (32 k x 16 tokens); operands as raw bits, bf16 or (HALFW) half precision
template <bool HALFW>
__device__ __forceinline__ f32x4 mma16(u32x4 a, u32x4 b, f32x4 acc)
{
    if (HALFW) return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), acc, 0, 0, 0);
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
}

typedef __bf16 sg_bf16x2 __attribute__((ext_vector_type(2)));
typedef float sg_f32x2 __attribute__((ext_vector_type(2)));

// h = silu(g) * u for two elements -> a bf16 pair of leading parts and a bf16 pair of remainders
// (hi = bf16(h), lo = bf16(h - hi); low half = first element).  Reciprocal and exponential are the
// hardware's approximations (1 ulp), the conversions its round-to-nearest-even.
__device__ __forceinline__ void swiglu_split2(float g0, float u0, float g1, float u1, uint32_t &hi, uint32_t &lo)
{
    float h0 = g0 * __builtin_amdgcn_rcpf(1.0f + __expf(-g0)) * u0;
    float h1 = g1 * __builtin_amdgcn_rcpf(1.0f + __expf(-g1)) * u1;
    hi = __builtin_bit_cast(uint32_t, __builtin_convertvector((sg_f32x2){h0, h1}, sg_bf16x2));
    float r0 = h0 - __uint_as_float(hi << 16), r1 = h1 - __uint_as_float(hi & 0xFFFF0000u);
    lo = __builtin_bit_cast(uint32_t, __builtin_convertvector((sg_f32x2){r0, r1}, sg_bf16x2));
}

// h = silu(g) * u for two elements as one pair of half-precision numbers (low half = first
// element), rounded to nearest even; magnitudes beyond the largest half-precision number saturate
// to it (sat is set), NaN stays NaN.
constexpr float HALF_MAX = 65504.0f;
__device__ __forceinline__ uint32_t swiglu_half2(float g0, float u0, float g1, float u1, bool &sat)
{
    float h0 = g0 * __builtin_amdgcn_rcpf(1.0f + __expf(-g0)) * u0;
    float h1 = g1 * __builtin_amdgcn_rcpf(1.0f + __expf(-g1)) * u1;
    const bool s0 = fabsf(h0) > HALF_MAX, s1 = fabsf(h1) > HALF_MAX;
    h0 = s0 ? copysignf(HALF_MAX, h0) : h0;
    h1 = s1 ? copysignf(HALF_MAX, h1) : h1;
    sat |= s0 | s1;
    return __builtin_bit_cast(uint32_t, __builtin_convertvector((sg_f32x2){h0, h1}, sg_f16x2));
}

// ---- quantised pairs (3-bit codes, group scales, base-3 masks) --------------------------------
// The appendix on combining the method with quantisation stores, per element, a 3-bit magnitude
// code, two sign bits and which expert(s) use it; here 8 elements make one 53-bit record (layout
// in quant_codec.hip).  Decoding with arithmetic would cost more vector instructions than the
// packed bytes leave time for, so it is table-driven; the tables live in LDS, built by every
// workgroup at start:
//   lut_t[13-bit mask number] -> the 8 mask bits of position 0 (low byte) and of position 1
//   lut_mask[nibble] -> 2 dwords, 0xFFFF in each half whose bit is set
//   lut_sign[nibble] -> 2 dwords, bit 15 / bit 31 set where the bit is set
//   lut_mag[6 bits: two codes] -> the two codes as bf16 (0..7 are exact)
// The nibble tables are 128 bytes each and the code table 256: every entry has its own LDS banks,
// so 64 lanes reading arbitrary entries do not conflict (a 256-entry table of 16-byte rows did,
// and was the bottleneck of a first version).
// A decoded fragment holds +-code (or 0); the group scale multiplies the accumulated products
// of each 128-column group afterwards, in fp32, so nothing is rounded that the definition
// (code * scale, exactly) does not round.
constexpr int Q_TILE_BYTES = 424;
constexpr int Q_LUT_T = 8192;
constexpr int Q_LUT_BYTES = Q_LUT_T * 2 + 16 * 8 * 2 + 64 * 4;

struct QLuts {
    const uint16_t *t;
    const u32x2 *mask, *sign;
    const uint32_t *mag;
};

__device__ __forceinline__ void q_build_luts(unsigned char *base, QLuts &l)
{
    uint16_t *t = (uint16_t *)base;
    u32x2 *mask = (u32x2 *)(base + Q_LUT_T * 2);
    u32x2 *sign = mask + 16;
    uint32_t *mag = (uint32_t *)(sign + 16);
    for (int v = threadIdx.x; v < Q_LUT_T; v += SG_THREADS) {
        uint32_t r = v, m0 = 0, m1 = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            uint32_t d = r % 3u;
            r /= 3u;
            m0 |= (d != 1u ? 1u : 0u) << e;          // digit 0 or 2: position 0 uses the element
            m1 |= (d != 0u ? 1u : 0u) << e;          // digit 1 or 2: position 1 uses it
        }
        t[v] = (uint16_t)(v < 6561 ? (m0 | m1 << 8) : 0u);
    }
    if (threadIdx.x < 16) {
        uint32_t b = threadIdx.x;
        u32x2 mk, sg;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            uint32_t lo = (b >> (2 * i)) & 1u, hi = (b >> (2 * i + 1)) & 1u;
            mk[i] = (lo ? 0x0000FFFFu : 0u) | (hi ? 0xFFFF0000u : 0u);
            sg[i] = lo << 15 | hi << 31;
        }
        mask[b] = mk;
        sign[b] = sg;
    }
    if (threadIdx.x < 64) {
        uint32_t ca = threadIdx.x & 7u, cb = threadIdx.x >> 3;
        mag[threadIdx.x] = (__float_as_uint((float)ca) >> 16) | (__float_as_uint((float)cb) & 0xFFFF0000u);
    }
    l.t = t; l.mask = mask; l.sign = sign; l.mag = mag;
}

struct QRecord {
    u32x4 mag;
    uint32_t s0, s1, mm;
};

__device__ __forceinline__ QRecord q_split(uint64_t raw, int shift, const QLuts &l)
{
    uint64_t r = raw >> shift;
    uint32_t lo = (uint32_t)r, hi = (uint32_t)(r >> 32);
    QRecord q;
#pragma unroll
    for (int i = 0; i < 4; ++i) q.mag[i] = l.mag[(lo >> (6 * i)) & 63u];
    q.s0 = lo >> 24;
    q.s1 = hi & 0xFFu;
    q.mm = l.t[(hi >> 8) & 0x1FFFu];
    return q;
}

template <int POS>
__device__ __forceinline__ u32x4 q_frag(const QRecord &q, const QLuts &l)
{
    const uint32_t sb = POS ? q.s1 : q.s0;
    const uint32_t mb = POS ? (q.mm >> 8) : q.mm;
    u32x2 sl = l.sign[sb & 15u], sh = l.sign[(sb >> 4) & 15u];
    u32x2 ml = l.mask[mb & 15u], mh = l.mask[(mb >> 4) & 15u];
    u32x4 o;
    o[0] = (q.mag[0] | sl[0]) & ml[0];
    o[1] = (q.mag[1] | sl[1]) & ml[1];
    o[2] = (q.mag[2] | sh[0]) & mh[0];
    o[3] = (q.mag[3] | sh[1]) & mh[1];
    return o;
}

// ---- grouping of the (token, choice) list inside the gate/up kernel (small batches) -----------
// A decode-time batch has a few hundred (token, choice) entries at most.  A separate grouping
// kernel in front of the first weight-streaming kernel costs about 6 us of a 240 us step; instead
// every workgroup of that kernel sorts the list by itself, in LDS, before it starts streaming (all
// workgroups do the same deterministic work and arrive at the same tables), and workgroup 0 also
// writes the tables to the workspace for the kernels that follow.  Counting sort by routing key,
// stable: a key's slots are in ascending (token, choice) order.  Entry i belongs to thread i
// (n_flat <= FR_MAX_N = the workgroup's size); a wave ranks its 64 entries with one ballot per
// distinct key, the waves' counts are combined through a small table in LDS.
constexpr int FR_MAX_N = SG_THREADS;
constexpr int FR_MAX_KEYS = 128;
static_assert(FR_MAX_N == STREAM_FUSED_ROUTE_MAX_FLAT && FR_MAX_KEYS == STREAM_FUSED_ROUTE_MAX_KEYS, "limits the host checks");
constexpr int FR_LDS_INTS = FR_MAX_N + 2 * FR_MAX_KEYS + SG_WAVES * FR_MAX_KEYS;   // slot_tok, cnt, off, per-wave counts

__device__ __forceinline__ void route_in_block(const SgRoute &r, int32_t *lds, const int32_t *&cnt, const int32_t *&off,
                                               const int32_t *&slot_tok)
{
    int32_t *l_tok = lds, *l_cnt = lds + FR_MAX_N, *l_off = l_cnt + FR_MAX_KEYS, *l_wave = l_off + FR_MAX_KEYS;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const bool writer = blockIdx.x == 0;
    for (int i = tid; i < SG_WAVES * FR_MAX_KEYS; i += SG_THREADS) l_wave[i] = 0;
    int key = -1;
    if (tid < r.n_flat) {
        const int e = r.ids[tid];
        if (e >= 0 && e < r.n_experts) key = r.q_of_expert[e];      // ids outside [0, E) are ignored
    }
    __syncthreads();
    // rank among the wave's entries of the same key (ascending lane), and the wave's count per key
    int rank = 0;
    uint64_t todo = __ballot(key >= 0);
    while (todo) {
        const int first = __builtin_ctzll(todo);
        const int v = __builtin_amdgcn_readlane(key, first);
        const uint64_t same = __ballot(key == v);
        if (key == v) rank = __popcll(same & ((1ull << lane) - 1ull));
        if (lane == first) l_wave[wave * FR_MAX_KEYS + v] = __popcll(same);
        todo &= ~same;
    }
    __syncthreads();
    // per key: first slot of each wave's entries (relative to the key's first slot) and the total
    for (int q = tid; q < r.n_keys; q += SG_THREADS) {
        int run = 0;
        for (int w = 0; w < SG_WAVES; ++w) { const int c = l_wave[w * FR_MAX_KEYS + q]; l_wave[w * FR_MAX_KEYS + q] = run; run += c; }
        l_cnt[q] = run;
    }
    __syncthreads();
    if (wave == 0) {                       // exclusive scan of the counts (at most 128 keys: two per lane)
        const int c0 = 2 * lane < r.n_keys ? l_cnt[2 * lane] : 0, c1 = 2 * lane + 1 < r.n_keys ? l_cnt[2 * lane + 1] : 0;
        int inc = c0 + c1;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) { const int u = __shfl_up(inc, d); if (lane >= d) inc += u; }
        const int ex = inc - c0 - c1;
        if (2 * lane < r.n_keys) l_off[2 * lane] = ex;
        if (2 * lane + 1 < r.n_keys) l_off[2 * lane + 1] = ex + c0;
        if (writer && lane == 63) r.off[r.n_keys] = inc;
    }
    __syncthreads();
    if (tid < r.n_flat) {
        int slot = -1;
        if (key >= 0) {
            slot = l_off[key] + l_wave[wave * FR_MAX_KEYS + key] + rank;
            l_tok[slot] = tid / r.k;
            if (writer) r.slot_tok[slot] = tid / r.k;
        }
        if (writer) r.slot_of[tid] = slot;
    }
    if (writer)
        for (int q = tid; q < r.n_keys; q += SG_THREADS) { r.cnt[q] = l_cnt[q]; r.off[q] = l_off[q]; }
    __syncthreads();
    cnt = l_cnt; off = l_off; slot_tok = l_tok;
}

// One pass: NT0 token tiles of position 0 followed by NT1 tiles of position 1.
// DENSE: the weights are plain bf16 (identity decode).  ALLTOK: the group sees every token
// (a shared expert) instead of a routed slot range.
// QUANT: the weights are quantised records (see above) instead of 16-bit words.
template <int STAGE, bool DENSE, bool ALLTOK, bool QUANT, bool HALF, int NT0, int NT1>
__device__ __forceinline__ void stream_pass(const SgArgs &a, const uint16_t *wa, const uint16_t *wb,
                                            const uint16_t *sa, const uint16_t *sb, const QLuts &luts,
                                            int rt0, int rt1, bool active0, bool active1,
                                            int kb0, int kb1, int ks,
                                            int base0, int n0, int tile0, int base1, int n1, int tile1,
                                            u32x4 *xs, int32_t *rowidx, const int32_t *slot_tok)
{
    constexpr int NT = NT0 + NT1;
    static_assert(!HALF || (!DENSE && !QUANT), "half-precision H is for 16-bit packed pairs");
    constexpr bool HALFW = HALF && STAGE == STAGE_DOWN;      // weights and activations of this stage in half precision
    constexpr int PARTS = (STAGE == STAGE_DOWN && !HALF) ? 2 : 1;    // activation planes (hi, lo)
    constexpr int VT = NT * PARTS;                          // staged fragment columns per k-block
    constexpr int KCB = (STAGE == STAGE_DOWN && !HALF) ? 4 : 8;      // k-blocks per staged chunk
    // (a depth of 8 for the 8-byte quantised records measured 7 % slower than 4)
    constexpr int DEPTH = (STAGE == STAGE_DOWN) ? SG_DEPTH : (QUANT ? SG_DEPTH_QUANT_GATEUP : SG_DEPTH_GATEUP);
    static_assert(VT * KCB <= SG_FRAGS, "staged chunk does not fit its LDS buffer");
    static_assert(KCB % DEPTH == 0, "prefetch slots must line up with chunk steps");
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int kb_total = a.kdim / TILE_COLS;

    // rows of the activation matrix behind each staged token column (clamped to a valid one)
    __syncthreads();
    if (tid < NT * 16) {
        int nt = tid >> 4, j = tid & 15;
        int slot;
        if (nt < NT0) slot = base0 + min((tile0 + nt) * 16 + j, n0 - 1);
        else          slot = base1 + min((tile1 + nt - NT0) * 16 + j, n1 - 1);
        int row;
        if (a.act_is_x) row = ALLTOK ? (slot - base0) : slot_tok[slot];
        else            row = slot - a.act_slot_base;
        rowidx[tid] = row;
    }
    __syncthreads();

    f32x4 acc[2][NT];
    f32x4 accg[2][QUANT ? NT : 1];      // QUANT: products of the current 128-column group, unscaled
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int n = 0; n < NT; ++n) {
            acc[m][n] = (f32x4){0.f, 0.f, 0.f, 0.f};
            if (QUANT) accg[m][n] = (f32x4){0.f, 0.f, 0.f, 0.f};
        }

    // The weight pointers come out of a device-side table, so the compiler cannot see that they
    // are global; say so, or it emits flat loads, which also tick the LDS counter.
    typedef const u32x4 __attribute__((address_space(1))) *gvec_ptr;
    gvec_ptr wp[2];
    wp[0] = (gvec_ptr)(uintptr_t)wa + ((int64_t)rt0 * kb_total + kb0) * 64 + lane;
    wp[1] = (gvec_ptr)(uintptr_t)wb + ((int64_t)rt1 * kb_total + kb0) * 64 + lane;
    // QUANT: a tile is 424 bytes; lane l's 53-bit record starts at bit 53*l: one unaligned
    // 8-byte load at byte 53*l/8, shifted right by 53*l%8
    typedef uint64_t __attribute__((aligned(1))) u64_unaligned;
    typedef const u64_unaligned __attribute__((address_space(1))) *gq_ptr;
    typedef const unsigned char __attribute__((address_space(1))) *gbyte_ptr;
    gbyte_ptr qp[2];
    qp[0] = (gbyte_ptr)(uintptr_t)wa + ((int64_t)rt0 * kb_total + kb0) * Q_TILE_BYTES + ((53 * lane) >> 3);
    qp[1] = (gbyte_ptr)(uintptr_t)wb + ((int64_t)rt1 * kb_total + kb0) * Q_TILE_BYTES + ((53 * lane) >> 3);
    const int qshift = (53 * lane) & 7;
    // ... and the scales of the 4 accumulator rows of this lane, one 128-column group ahead
    typedef const u32x2 __attribute__((address_space(1))) *gsc_ptr;
    const int n_qgroups = kb_total / 4;
    gsc_ptr sp[2];
    sp[0] = (gsc_ptr)(uintptr_t)(sa + ((int64_t)rt0 * n_qgroups) * TILE_ROWS + (lane >> 4) * 4);
    sp[1] = (gsc_ptr)(uintptr_t)(sb + ((int64_t)rt1 * n_qgroups) * TILE_ROWS + (lane >> 4) * 4);
    auto load_scale = [&](int m, int kb_abs) {
        int gi = min(kb_abs / 4, n_qgroups - 1);
        return sp[m][gi * (TILE_ROWS * 2 / 8)];                  // 16 bf16 = 4 x 8 bytes per group
    };
    u32x2 sc_cur[2] = {{0u, 0u}, {0u, 0u}}, sc_nxt[2] = {{0u, 0u}, {0u, 0u}};
    if (QUANT) {
#pragma unroll
        for (int m = 0; m < 2; ++m) { sc_cur[m] = load_scale(m, kb0); sc_nxt[m] = load_scale(m, kb0 + 4); }
    }

    // Weight loads are never predicated (a branch per load would make the compiler drain the
    // whole load queue at every barrier): a k-block past the end re-reads the last valid one,
    // and contributes nothing because its staged activations are zero.
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    const int kb_last = kb1 - 1 - kb0;
    u32x4 wbuf[2][QUANT ? 1 : DEPTH];
    uint64_t qbuf[2][QUANT ? DEPTH : 1];
#pragma unroll
    for (int s = 0; s < DEPTH; ++s)
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            if (QUANT) qbuf[m][s] = SG_WLOAD((gq_ptr)(qp[m] + (int64_t)min(s, kb_last) * Q_TILE_BYTES));
            else       wbuf[m][s] = SG_WLOAD(wp[m] + (int64_t)min(s, kb_last) * 64);
        }

    // activation fragments this thread stages per chunk: fragment f = wave + 4*i,
    // (column, k-block) = (f / KCB, f % KCB), column = tile * PARTS + plane
    constexpr int XPT = VT * KCB / SG_WAVES;
    u32x4 xr[XPT];
    const uint16_t *xrow[XPT];
#pragma unroll
    for (int i = 0; i < XPT; ++i) {
        int col = (wave + SG_WAVES * i) / KCB;
        xrow[i] = a.act + (col % PARTS) * a.act_plane_stride +
                  (int64_t)rowidx[(col / PARTS) * 16 + (lane & 15)] * a.kdim + (lane >> 4) * 8;
    }
    // The loaded registers are only touched again in stage_store, a whole chunk later, so the
    // loads stay in flight behind the weight stream; k-blocks past the end are stored as zeros.
    auto stage_load = [&](int kbc) {
#pragma unroll
        for (int i = 0; i < XPT; ++i) {
            int kb = kbc + (wave + SG_WAVES * i) % KCB;
            xr[i] = *(const u32x4 *)(xrow[i] + min(kb, kb1 - 1) * TILE_COLS);
        }
    };
    auto stage_store = [&](int buf, int kbc) {
#pragma unroll
        for (int i = 0; i < XPT; ++i) {
            int f = wave + SG_WAVES * i;
            xs[(buf * SG_FRAGS + f) * 64 + lane] = (kbc + f % KCB < kb1) ? xr[i] : zero4;
        }
    };

    stage_load(kb0);
    stage_store(0, kb0);
    __syncthreads();

    int buf = 0;
    for (int kb = kb0; kb < kb1; kb += KCB) {
        const bool has_next = kb + KCB < kb1;
        if (has_next) stage_load(kb + KCB);
#pragma unroll
        for (int s = 0; s < KCB; ++s) {
            u32x4 wv[2];
            QRecord qr[2];
#pragma unroll
            for (int m = 0; m < 2; ++m) {
                if (QUANT) qr[m] = q_split(qbuf[m][s % DEPTH], qshift, luts);
                else       wv[m] = wbuf[m][s % DEPTH];
            }
            const u32x4 *xf = xs + (buf * SG_FRAGS + s) * 64 + lane;
            if (NT0 > 0) {
                u32x4 wd[2];
#pragma unroll
                for (int m = 0; m < 2; ++m) wd[m] = QUANT ? q_frag<0>(qr[m], luts) : decode_frag<0, DENSE, HALFW>(wv[m]);
#pragma unroll
                for (int c = 0; c < NT0 * PARTS; ++c) {
                    const u32x4 b = xf[c * KCB * 64];
#pragma unroll
                    for (int m = 0; m < 2; ++m) {
                        f32x4 &dst = QUANT ? accg[m][QUANT ? c / PARTS : 0] : acc[m][c / PARTS];
                        dst = mma16<HALFW>(wd[m], b, dst);
                    }
                }
            }
            if (NT1 > 0) {
                u32x4 wd[2];
#pragma unroll
                for (int m = 0; m < 2; ++m) wd[m] = QUANT ? q_frag<1>(qr[m], luts) : decode_frag<1, DENSE, HALFW>(wv[m]);
#pragma unroll
                for (int c = NT0 * PARTS; c < VT; ++c) {
                    const u32x4 b = xf[c * KCB * 64];
#pragma unroll
                    for (int m = 0; m < 2; ++m) {
                        f32x4 &dst = QUANT ? accg[m][QUANT ? c / PARTS : 0] : acc[m][c / PARTS];
                        dst = mma16<HALFW>(wd[m], b, dst);
                    }
                }
            }
            if (QUANT && s % 4 == 3) {
                // end of a 128-column group: scale its products (rows 4*(lane/16)..+3 of the tile)
#pragma unroll
                for (int m = 0; m < 2; ++m) {
                    float f0 = __uint_as_float(sc_cur[m][0] << 16), f1 = __uint_as_float(sc_cur[m][0] & 0xFFFF0000u);
                    float f2 = __uint_as_float(sc_cur[m][1] << 16), f3 = __uint_as_float(sc_cur[m][1] & 0xFFFF0000u);
#pragma unroll
                    for (int n = 0; n < NT; ++n) {
                        f32x4 &g = accg[m][QUANT ? n : 0];
                        acc[m][n][0] = fmaf(f0, g[0], acc[m][n][0]);
                        acc[m][n][1] = fmaf(f1, g[1], acc[m][n][1]);
                        acc[m][n][2] = fmaf(f2, g[2], acc[m][n][2]);
                        acc[m][n][3] = fmaf(f3, g[3], acc[m][n][3]);
                        g = (f32x4){0.f, 0.f, 0.f, 0.f};
                    }
                    sc_cur[m] = sc_nxt[m];
                    sc_nxt[m] = load_scale(m, kb + s + 5);       // the group after the next one
                }
            }
            // refill the slot just consumed
#pragma unroll
            for (int m = 0; m < 2; ++m) {
                int kbn = min(kb + DEPTH + s - kb0, kb_last);
                if (QUANT) qbuf[m][s % DEPTH] = SG_WLOAD((gq_ptr)(qp[m] + (int64_t)kbn * Q_TILE_BYTES));
                else       wbuf[m][s % DEPTH] = SG_WLOAD(wp[m] + (int64_t)kbn * 64);
            }
#if SG_SCHED_BARRIER
            // keep each step's refill inside the step: the scheduler otherwise sinks all loads
            // of a chunk to its end, which exposes the memory latency once per chunk
            __builtin_amdgcn_sched_barrier(0);
#endif
        }
        if (has_next) stage_store(buf ^ 1, kb + KCB);
        __syncthreads();
        buf ^= 1;
    }

    // D layout of the 16x16 MFMA: lane holds rows 4*(lane/16)..+3 of column lane%16.
    const int j = lane & 15;
    bool sat = false;
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        int within = (n < NT0) ? (tile0 + n) * 16 + j : (tile1 + n - NT0) * 16 + j;
        int cnt = (n < NT0) ? n0 : n1;
        if (within >= cnt) continue;
        int slot = ((n < NT0) ? base0 : base1) + within;
        if (STAGE == STAGE_GATEUP && HALF) {
            if (!active0) continue;
            f32x4 g = acc[0][n], u = acc[1][n];
            u32x2 oh = {swiglu_half2(g[0], u[0], g[1], u[1], sat), swiglu_half2(g[2], u[2], g[3], u[3], sat)};
            *(u32x2 *)(a.h_out + (int64_t)(slot - a.h_slot_base) * a.rows + rt0 * 16 + (lane >> 4) * 4) = oh;
        } else if (STAGE == STAGE_GATEUP) {
            if (!active0) continue;
            f32x4 g = acc[0][n], u = acc[1][n];
            uint32_t hi01, lo01, hi23, lo23;
            swiglu_split2(g[0], u[0], g[1], u[1], hi01, lo01);
            swiglu_split2(g[2], u[2], g[3], u[3], hi23, lo23);
            u32x2 ohi = {hi01, hi23}, olo = {lo01, lo23};
            uint16_t *dst = a.h_out + (int64_t)(slot - a.h_slot_base) * a.rows + rt0 * 16 + (lane >> 4) * 4;
            *(u32x2 *)dst = ohi;
            *(u32x2 *)(dst + a.h_plane_stride) = olo;
        } else {
            // (half-precision weights were decoded as 2 w: halve the sums, which is exact)
            float *dst = a.o_out + (int64_t)ks * a.o_ks_stride + (int64_t)slot * a.rows + (lane >> 4) * 4;
            if (active0) *(f32x4 *)(dst + rt0 * 16) = HALFW ? acc[0][n] * 0.5f : acc[0][n];
            if (active1) *(f32x4 *)(dst + rt1 * 16) = HALFW ? acc[1][n] * 0.5f : acc[1][n];
        }
    }
    if (STAGE == STAGE_GATEUP && HALF && a.h_saturated && __any(sat) && lane == 0) atomicAdd(a.h_saturated, 1);
}

// FUSE: the kernel groups the (token, choice) list itself (route_in_block) instead of reading the
// tables of a grouping kernel that ran before it.
template <int STAGE, bool DENSE, bool ALLTOK, bool QUANT, bool HALF, bool FUSE>
__global__ void __launch_bounds__(SG_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2)))
stream_kernel(SgArgs a)
{
    static_assert(!FUSE || (STAGE == STAGE_GATEUP && !ALLTOK && !QUANT), "in-kernel grouping is for the routed gate/up launch");
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    u32x4 *xs = (u32x4 *)lds_raw;
    int32_t *rowidx = (int32_t *)(lds_raw + SG_LDS_BYTES);
    QLuts luts = {nullptr, nullptr, nullptr, nullptr};
    if (QUANT) q_build_luts(lds_raw + SG_LDS_BYTES + SG_MAX_TILES * 16 * sizeof(int32_t), luts);   // visible after the pass's first barrier
    const int32_t *cnt = a.cnt, *off = a.off, *slot_tok = a.slot_tok;
    if (FUSE) route_in_block(a.route, (int32_t *)(lds_raw + SG_LDS_BYTES + SG_MAX_TILES * 16 * sizeof(int32_t)), cnt, off, slot_tok);

    constexpr int RT_PER_WAVE = (STAGE == STAGE_DOWN) ? 2 : 1;
    const int row_tiles = a.rows / TILE_ROWS;
    const int row_groups = (row_tiles + SG_WAVES * RT_PER_WAVE - 1) / (SG_WAVES * RT_PER_WAVE);
    const int rg_blocks = (row_groups + a.rg_per_wg - 1) / a.rg_per_wg;
    int b = blockIdx.x;
    // A shared expert has few row groups (few workgroups) but sees every token: its token passes
    // go to different workgroups (pass index fastest, so the workgroups that read the same
    // weights run at the same time and share them through L2 / the memory-side cache).  Routed
    // groups get n_passes workgroups too where a router that favours some experts may give one
    // more tokens than a pass holds: the busy group's passes then run side by side instead of
    // making its workgroups the last to finish; workgroups with no pass to do leave at once.
    // (The hardware deals consecutive workgroup ids to the XCDs in turn: a routed group's extra
    // workgroups therefore take the ids after all the first ones, not every n-th id, which would
    // leave the first workgroups, the ones that always have work, on a subset of the XCDs.)
    const int per_pass = gridDim.x / a.n_passes;
    const int my_pass = ALLTOK ? b % a.n_passes : b / per_pass;
    b = ALLTOK ? b / a.n_passes : b % per_pass;
    const int ks = b % a.ksplit; b /= a.ksplit;
    const int rgb = b % rg_blocks;
    const int g = b / rg_blocks;

    int base0, n0, base1, n1;
    if (ALLTOK) {
        n0 = a.dense_tokens; n1 = 0;
        base0 = a.dense_slot_base + g * a.dense_tokens; base1 = 0;
    } else {
        const int q0 = 2 * (a.group_base + g);
        n0 = cnt[q0]; n1 = cnt[q0 + 1];
        base0 = off[q0]; base1 = off[q0 + 1];
    }
    if (n0 + n1 == 0) return;

    const int wave = threadIdx.x >> 6;
    const int kb_total = a.kdim / TILE_COLS;
    // K splits: whole k-blocks; for quantised weights whole 128-column groups (4 k-blocks)
    const int kq = QUANT ? 4 : 1;
    const int kb0 = (int)((int64_t)ks * (kb_total / kq) / a.ksplit) * kq;
    const int kb1 = (int)((int64_t)(ks + 1) * (kb_total / kq) / a.ksplit) * kq;
    const uint16_t *wa = a.w_a[g];
    const uint16_t *wb = (STAGE == STAGE_GATEUP) ? a.w_b[g] : wa;
    const uint16_t *sa = QUANT ? a.s_a[g] : nullptr;
    const uint16_t *sb = QUANT ? ((STAGE == STAGE_GATEUP) ? a.s_b[g] : sa) : nullptr;
    constexpr int PT = DENSE ? SG_MAX_TILES : SG_POS_TILES;   // a dense group has one position only
    const int tiles0 = (n0 + 15) >> 4, tiles1 = (n1 + 15) >> 4;
    if (my_pass * PT >= max(tiles0, tiles1)) return;

    for (int rg = rgb * a.rg_per_wg; rg < min(row_groups, (rgb + 1) * a.rg_per_wg); ++rg) {
    int rt0 = (rg * SG_WAVES + wave) * RT_PER_WAVE;
    int rt1 = (STAGE == STAGE_DOWN) ? rt0 + 1 : rt0;
    const bool active0 = rt0 < row_tiles, active1 = rt1 < row_tiles;
    rt0 = min(rt0, row_tiles - 1);      // inactive streams re-read a valid tile and store nothing
    rt1 = min(rt1, row_tiles - 1);
    for (int t0 = my_pass * PT, t1 = t0; t0 < tiles0 || t1 < tiles1; t0 += a.n_passes * PT, t1 = t0) {
        int c0 = min(PT, max(tiles0 - t0, 0));
        int c1 = min(PT, max(tiles1 - t1, 0));
#define PZL_PASS(A, B)                                                                              \
    stream_pass<STAGE, DENSE, ALLTOK, QUANT, HALF, A, B>(a, wa, wb, sa, sb, luts, rt0, rt1, active0, active1, kb0, kb1, ks, \
                                                   base0, n0, t0, base1, n1, t1, xs, rowidx, slot_tok)
        if (DENSE) {
            switch (c0) {
                case 1: PZL_PASS(1, 0); break;
                case 2: PZL_PASS(2, 0); break;
                case 3: PZL_PASS(3, 0); break;
                default: PZL_PASS(4, 0); break;
            }
        } else {
            switch (c0 * 3 + c1) {
                case 1: PZL_PASS(0, 1); break;
                case 2: PZL_PASS(0, 2); break;
                case 3: PZL_PASS(1, 0); break;
                case 4: PZL_PASS(1, 1); break;
                case 5: PZL_PASS(1, 2); break;
                case 6: PZL_PASS(2, 0); break;
                case 7: PZL_PASS(2, 1); break;
                default: PZL_PASS(2, 2); break;
            }
        }
#undef PZL_PASS
    }
    }
}

int stream_row_groups(int rows, bool down_stage)
{
    const int per_wg = SG_WAVES * (down_stage ? 2 : 1);
    return (rows / TILE_ROWS + per_wg - 1) / per_wg;
}

template <bool QUANT, bool FUSE>
static constexpr size_t stream_lds_bytes()
{
    return SG_LDS_BYTES + SG_MAX_TILES * 16 * sizeof(int32_t) + (QUANT ? Q_LUT_BYTES : 0) + (FUSE ? FR_LDS_INTS * sizeof(int32_t) : 0);
}

// The dynamic LDS size beyond 64 KiB is a per-device attribute of the kernel: set once per device
// (bit d of the mask; setting it twice from two threads is harmless).
template <int STAGE, bool DENSE, bool ALLTOK, bool QUANT, bool HALF, bool FUSE = false>
static int set_lds_attribute()
{
    static std::atomic<uint64_t> attr_devices{0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev > 63) dev = 63;       // unknown device: set it every time
    if (dev == 63 || !((attr_devices.load(std::memory_order_relaxed) >> dev) & 1)) {
        hipError_t e = hipFuncSetAttribute((const void *)stream_kernel<STAGE, DENSE, ALLTOK, QUANT, HALF, FUSE>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)stream_lds_bytes<QUANT, FUSE>());
        if (e != hipSuccess) { set_hip_error(e); return PZL_EHIP; }
        if (dev != 63) attr_devices.fetch_or(1ull << dev, std::memory_order_relaxed);
    }
    return PZL_OK;
}

int prepare_stream_kernels()
{
    int rc = PZL_OK;
#define PZL_PREP(S, D, A, Q, H) if (!rc) rc = set_lds_attribute<S, D, A, Q, H>()
    PZL_PREP(STAGE_GATEUP, false, false, false, false); PZL_PREP(STAGE_DOWN, false, false, false, false);
    PZL_PREP(STAGE_GATEUP, false, false, false, true);  PZL_PREP(STAGE_DOWN, false, false, false, true);
    PZL_PREP(STAGE_GATEUP, true, true, false, false);   PZL_PREP(STAGE_DOWN, true, true, false, false);
    PZL_PREP(STAGE_GATEUP, true, false, false, false);  PZL_PREP(STAGE_DOWN, true, false, false, false);
    PZL_PREP(STAGE_GATEUP, false, false, true, false);  PZL_PREP(STAGE_DOWN, false, false, true, false);
#undef PZL_PREP
    if (!rc) rc = set_lds_attribute<STAGE_GATEUP, false, false, false, false, true>();
    if (!rc) rc = set_lds_attribute<STAGE_GATEUP, false, false, false, true, true>();
    return rc;
}

template <int STAGE, bool DENSE, bool ALLTOK, bool QUANT, bool HALF = false, bool FUSE = false>
static int launch(const StreamGroupArgs &g, hipStream_t st)
{
    if (g.n_groups <= 0) return PZL_OK;
    if (FUSE && (!g.route_ids || !g.route_q_of_expert || g.route_n_flat < 1 || g.route_n_flat > FR_MAX_N || g.route_k < 1 ||
                 g.route_n_keys < 2 || g.route_n_keys > FR_MAX_KEYS || !g.route_slot_of))
        return PZL_EINVAL;
    if (g.rows % TILE_ROWS || g.kdim % TILE_COLS || g.ksplit < 1) return PZL_EINVAL;
    // every K split must hold at least one k-block: the kernel clamps its read-ahead to the last
    // k-block of its share, which an empty share does not have
    if (g.ksplit > g.kdim / TILE_COLS) return PZL_EINVAL;
    if (QUANT && (g.kdim % 128 || !g.s_a || (STAGE == STAGE_GATEUP && !g.s_b))) return PZL_EINVAL;
    SgArgs a;
    a.w_a = g.w_a; a.w_b = g.w_b; a.rows = g.rows; a.kdim = g.kdim; a.ksplit = g.ksplit;
    a.s_a = g.s_a; a.s_b = g.s_b;
    if (QUANT && a.ksplit > g.kdim / 128) return PZL_EINVAL;    // a K split holds whole 128-column groups
    a.act = g.act; a.act_plane_stride = g.act_plane_stride;
    a.act_is_x = g.act_is_x; a.act_slot_base = g.act_slot_base;
    a.cnt = g.cnt; a.off = g.off; a.slot_tok = g.slot_tok; a.group_base = g.group_base;
    a.dense_tokens = g.dense_tokens; a.dense_slot_base = g.dense_slot_base;
    a.h_out = g.h_out; a.h_plane_stride = g.h_plane_stride; a.h_slot_base = g.h_slot_base;
    a.o_out = g.o_out; a.o_ks_stride = g.o_ks_stride;
    a.h_saturated = g.h_saturated;
    a.route = SgRoute{g.route_ids, g.route_q_of_expert, g.route_n_flat, g.route_k, g.route_n_experts, g.route_n_keys,
                      const_cast<int32_t *>(g.cnt), const_cast<int32_t *>(g.off), const_cast<int32_t *>(g.slot_tok), g.route_slot_of};
    // One workgroup (8 waves, two per SIMD) fits a compute unit, 256 on the chip.  A launch a little
    // larger than that runs a second, partly empty round; giving each workgroup several row
    // groups instead keeps the launch to one round.
    const int row_groups = stream_row_groups(g.rows, STAGE == STAGE_DOWN);
    const int pass_tokens = SG_MAX_TILES * 16;
    a.n_passes = ALLTOK ? (g.dense_tokens + pass_tokens - 1) / pass_tokens : g.pass_wgs;
    if (a.n_passes < 1) a.n_passes = 1;
    // (a routed group's extra pass workgroups mostly find nothing to do: not counted as work)
    const int64_t units = (int64_t)(g.groups_touched_max > 0 ? g.groups_touched_max : g.n_groups) * row_groups * g.ksplit *
                          (ALLTOK ? a.n_passes : 1);
    int rg_per_wg = (int)((units + SG_RESIDENT_WGS - 1) / SG_RESIDENT_WGS);
    if (rg_per_wg < 1) rg_per_wg = 1;
    if (rg_per_wg > 4) rg_per_wg = 1;            // many rounds anyway: keep the units small
    if (rg_per_wg > row_groups) rg_per_wg = row_groups;
    a.rg_per_wg = rg_per_wg;
    const int64_t blocks = (int64_t)g.n_groups * ((row_groups + rg_per_wg - 1) / rg_per_wg) * g.ksplit * a.n_passes;
    if (blocks > 0x7FFFFFFFLL) return PZL_EINVAL;
    const size_t lds = stream_lds_bytes<QUANT, FUSE>();
    int rc_attr = set_lds_attribute<STAGE, DENSE, ALLTOK, QUANT, HALF, FUSE>();
    if (rc_attr) return rc_attr;
    hipLaunchKernelGGL((stream_kernel<STAGE, DENSE, ALLTOK, QUANT, HALF, FUSE>), dim3((unsigned)blocks), dim3(SG_THREADS), lds, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_hip_error(e); return PZL_EHIP; }
    return PZL_OK;
}

// kind: 0 = packed pairs (routed), 1 = dense experts that see every token (shared),
//       2 = dense routed experts (kept unmerged), 3 = quantised pairs (routed)
int launch_stream_gateup(const StreamGroupArgs &a, int kind, hipStream_t st)
{
    if (kind == 0 && a.route_ids) return a.half_h ? launch<STAGE_GATEUP, false, false, false, true, true>(a, st)
                                                  : launch<STAGE_GATEUP, false, false, false, false, true>(a, st);
    if (kind == 0 && a.half_h) return launch<STAGE_GATEUP, false, false, false, true>(a, st);
    if (kind == 0) return launch<STAGE_GATEUP, false, false, false>(a, st);
    if (kind == 1) return launch<STAGE_GATEUP, true, true, false>(a, st);
    if (kind == 3) return launch<STAGE_GATEUP, false, false, true>(a, st);
    return launch<STAGE_GATEUP, true, false, false>(a, st);
}

int launch_stream_down(const StreamGroupArgs &a, int kind, hipStream_t st)
{
    if (kind == 0 && a.half_h) return launch<STAGE_DOWN, false, false, false, true>(a, st);
    if (kind == 0) return launch<STAGE_DOWN, false, false, false>(a, st);
    if (kind == 1) return launch<STAGE_DOWN, true, true, false>(a, st);
    if (kind == 3) return launch<STAGE_DOWN, false, false, true>(a, st);
    return launch<STAGE_DOWN, true, false, false>(a, st);
}

}  // namespace pzl
