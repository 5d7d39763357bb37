// Weight-streaming decode-GEMM for small token counts per expert pair (decode-time batches).
//
// Sec. 3.3.2: every packed weight is decoded (Algorithm 1) right before it is multiplied, the
// decoded matrix is never materialised, and ONE read of a packed tile produces the outputs of
// both experts of the pair.  On gfx950 that becomes: each wavefront streams 16-row x 32-col
// packed tiles (1 KiB contiguous, one 128-bit load per lane) straight into registers in
// matrix-core operand order, decodes them for position 0 and position 1 with packed 16-bit
// integer ops, and feeds v_mfma_f32_16x16x32_bf16 with the tokens of each expert as the
// other operand.  The kernel is HBM-bound: its job is to keep enough loads in flight and
// to keep the decode under the VALU budget.
//
// Workgroup = 4 waves = 4 adjacent row tiles sharing the staged activations in LDS
// (double-buffered chunks of 8 k-blocks).  Token tiles: up to MAX_TILES tiles of 16 tokens per
// pass, the tiles of position 0 first; longer token lists take further passes (re-streaming
// the weights), which is only the fallback — large batches belong to the tiled GEMM path.
#include "pzl_common.h"

namespace pzl {

constexpr int SG_WAVES = 4;
constexpr int SG_THREADS = SG_WAVES * 64;
constexpr int SG_KCB = 8;            // k-blocks of 32 per staged chunk == weight prefetch depth
constexpr int SG_MAX_TILES = 4;      // token tiles per pass (both positions together)
constexpr int SG_POS_TILES = 2;      // token tiles per pass per position (routed groups)
constexpr int SG_LDS_BYTES = 2 * SG_MAX_TILES * SG_KCB * 64 * 16;   // 64 KiB

struct SgArgs {
    const uint16_t *const *w_a;
    const uint16_t *const *w_b;
    int32_t rows, kdim, ksplit;
    const uint16_t *act;
    int32_t act_is_x, act_slot_base;
    const int32_t *cnt, *off, *slot_tok;
    int32_t dense_tokens, dense_slot_base;
    uint16_t *h_out;
    int32_t h_slot_base;
    float *o_out;
    int64_t o_ks_stride;
};

// ---- Algorithm 1 on two packed elements at a time -------------------------------------------
// body = exponent+112 and mantissa of both halves (no carry can cross: 0x0FFF + 0x3800 < 0x8000).
__device__ __forceinline__ uint32_t decode_body(uint32_t x) { return (x & 0x0FFF0FFFu) + 0x38003800u; }

// mask bit (13-pos) of each half -> 0xFFFF / 0x0000 via a packed arithmetic shift;
// sign bit (15-pos) of each half moved to bit 15.
template <int POS>
__device__ __forceinline__ uint32_t decode_pair(uint32_t x, uint32_t body)
{
    uint32_t xs = POS ? (x << 1) : x;
    s16x2 t = __builtin_bit_cast(s16x2, x << (2 + POS));
    t = t >> 15;
    uint32_t m = __builtin_bit_cast(uint32_t, t);
    return ((xs & 0x80008000u) | body) & m;
}

template <int POS, bool DENSE>
__device__ __forceinline__ bf16x8 decode_frag(u32x4 w)
{
    if (DENSE) return __builtin_bit_cast(bf16x8, w);
    u32x4 o;
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = decode_pair<POS>(w[i], decode_body(w[i]));
    return __builtin_bit_cast(bf16x8, o);
}

__device__ __forceinline__ uint32_t f32_to_bf16_rne_sg(float v)
{
    uint32_t u = __float_as_uint(v);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0u;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

__device__ __forceinline__ float silu_f32(float g) { return g / (1.0f + __expf(-g)); }

// One pass: NT0 token tiles of position 0 followed by NT1 tiles of position 1.
// NM = 2: gate and up with the SwiGLU epilogue (H, bf16); NM = 1: down (fp32 partial sums).
template <int NM, bool DENSE, int NT0, int NT1>
__device__ __forceinline__ void stream_pass(const SgArgs &a, const uint16_t *wa, const uint16_t *wb,
                                            int rt, bool active, int kb0, int kb1, int ks,
                                            int base0, int n0, int tile0, int base1, int n1, int tile1,
                                            u32x4 *xs, int32_t *rowidx)
{
    constexpr int NT = NT0 + NT1;
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
        if (a.act_is_x) row = DENSE ? (slot - base0) : a.slot_tok[slot];
        else            row = slot - a.act_slot_base;
        rowidx[tid] = row;
    }
    __syncthreads();

    f32x4 acc[NM][NT];
#pragma unroll
    for (int m = 0; m < NM; ++m)
#pragma unroll
        for (int n = 0; n < NT; ++n) acc[m][n] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // The weight pointers come out of a device-side table, so the compiler cannot see that they
    // are global; say so, or it emits flat loads, which also tick the LDS counter.
    typedef const u32x4 __attribute__((address_space(1))) *gvec_ptr;
    gvec_ptr wp[NM];
    wp[0] = (gvec_ptr)(uintptr_t)wa + ((int64_t)rt * kb_total + kb0) * 64 + lane;
    if (NM == 2) wp[NM - 1] = (gvec_ptr)(uintptr_t)wb + ((int64_t)rt * kb_total + kb0) * 64 + lane;

    // Weight loads are never predicated (a branch per load would make the compiler drain the
    // whole load queue at every barrier): a k-block past the end re-reads the last valid one,
    // and contributes nothing because its staged activations are zero.
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    const int kb_last = kb1 - 1 - kb0;
    u32x4 wbuf[NM][SG_KCB];
#pragma unroll
    for (int s = 0; s < SG_KCB; ++s)
#pragma unroll
        for (int m = 0; m < NM; ++m)
            wbuf[m][s] = __builtin_nontemporal_load(wp[m] + (int64_t)min(s, kb_last) * 64);

    // activation fragments this thread stages per chunk: fragment f = wave + 4*i, (tile, k-block) = (f / KCB, f % KCB)
    constexpr int XPT = NT * SG_KCB / SG_WAVES;
    u32x4 xr[XPT];
    const uint16_t *xrow[XPT];
#pragma unroll
    for (int i = 0; i < XPT; ++i) {
        int f = wave + SG_WAVES * i;
        xrow[i] = a.act + (int64_t)rowidx[(f / SG_KCB) * 16 + (lane & 15)] * a.kdim + (lane >> 4) * 8;
    }
    // The loaded registers are only touched again in stage_store, a whole chunk later, so the
    // loads stay in flight behind the weight stream; k-blocks past the end are stored as zeros.
    auto stage_load = [&](int kbc) {
#pragma unroll
        for (int i = 0; i < XPT; ++i) {
            int kb = kbc + (wave + SG_WAVES * i) % SG_KCB;
            xr[i] = *(const u32x4 *)(xrow[i] + min(kb, kb1 - 1) * TILE_COLS);
        }
    };
    auto stage_store = [&](int buf, int kbc) {
#pragma unroll
        for (int i = 0; i < XPT; ++i) {
            int f = wave + SG_WAVES * i;
            xs[(buf * SG_MAX_TILES * SG_KCB + f) * 64 + lane] = (kbc + f % SG_KCB < kb1) ? xr[i] : zero4;
        }
    };

    stage_load(kb0);
    stage_store(0, kb0);
    __syncthreads();

    int buf = 0;
    for (int kb = kb0; kb < kb1; kb += SG_KCB) {
        const bool has_next = kb + SG_KCB < kb1;
        if (has_next) stage_load(kb + SG_KCB);
#pragma unroll
        for (int s = 0; s < SG_KCB; ++s) {
            u32x4 wv[NM];
#pragma unroll
            for (int m = 0; m < NM; ++m) {
                wv[m] = wbuf[m][s];
                int kbn = min(kb + SG_KCB + s - kb0, kb_last);
                wbuf[m][s] = __builtin_nontemporal_load(wp[m] + (int64_t)kbn * 64);
            }
            const u32x4 *xf = xs + (buf * SG_MAX_TILES * SG_KCB + s) * 64 + lane;
            if (NT0 > 0) {
                bf16x8 wd[NM];
#pragma unroll
                for (int m = 0; m < NM; ++m) wd[m] = decode_frag<0, DENSE>(wv[m]);
#pragma unroll
                for (int n = 0; n < NT0; ++n) {
                    bf16x8 b = __builtin_bit_cast(bf16x8, xf[n * SG_KCB * 64]);
#pragma unroll
                    for (int m = 0; m < NM; ++m)
                        acc[m][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wd[m], b, acc[m][n], 0, 0, 0);
                }
            }
            if (NT1 > 0) {
                bf16x8 wd[NM];
#pragma unroll
                for (int m = 0; m < NM; ++m) wd[m] = decode_frag<1, DENSE>(wv[m]);
#pragma unroll
                for (int n = NT0; n < NT; ++n) {
                    bf16x8 b = __builtin_bit_cast(bf16x8, xf[n * SG_KCB * 64]);
#pragma unroll
                    for (int m = 0; m < NM; ++m)
                        acc[m][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wd[m], b, acc[m][n], 0, 0, 0);
                }
            }
        }
        if (has_next) stage_store(buf ^ 1, kb + SG_KCB);
        __syncthreads();
        buf ^= 1;
    }

    if (!active) return;
    // D layout of the 16x16 MFMA: lane holds rows 4*(lane/16)..+3 of column lane%16.
    const int r0 = rt * 16 + (lane >> 4) * 4;
    const int j = lane & 15;
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        int within = (n < NT0) ? (tile0 + n) * 16 + j : (tile1 + n - NT0) * 16 + j;
        int cnt = (n < NT0) ? n0 : n1;
        if (within >= cnt) continue;
        int slot = ((n < NT0) ? base0 : base1) + within;
        if (NM == 2) {
            f32x4 g = acc[0][n], u = acc[NM - 1][n];
            u32x2 o;
            o.x = f32_to_bf16_rne_sg(silu_f32(g.x) * u.x) | (f32_to_bf16_rne_sg(silu_f32(g.y) * u.y) << 16);
            o.y = f32_to_bf16_rne_sg(silu_f32(g.z) * u.z) | (f32_to_bf16_rne_sg(silu_f32(g.w) * u.w) << 16);
            *(u32x2 *)(a.h_out + (int64_t)(slot - a.h_slot_base) * a.rows + r0) = o;
        } else {
            *(f32x4 *)(a.o_out + (int64_t)ks * a.o_ks_stride + (int64_t)slot * a.rows + r0) = acc[0][n];
        }
    }
}

template <int NM, bool DENSE>
__global__ void __launch_bounds__(SG_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2)))
stream_kernel(SgArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    u32x4 *xs = (u32x4 *)lds_raw;
    int32_t *rowidx = (int32_t *)(lds_raw + SG_LDS_BYTES);

    const int row_tiles = a.rows / TILE_ROWS;
    const int row_groups = (row_tiles + SG_WAVES - 1) / SG_WAVES;
    int b = blockIdx.x;
    const int ks = b % a.ksplit; b /= a.ksplit;
    const int rg = b % row_groups;
    const int g = b / row_groups;

    int base0, n0, base1, n1;
    if (DENSE) {
        n0 = a.dense_tokens; n1 = 0;
        base0 = a.dense_slot_base + g * a.dense_tokens; base1 = 0;
    } else {
        n0 = a.cnt[2 * g]; n1 = a.cnt[2 * g + 1];
        base0 = a.off[2 * g]; base1 = a.off[2 * g + 1];
    }
    if (n0 + n1 == 0) return;

    const int wave = threadIdx.x >> 6;
    int rt = rg * SG_WAVES + wave;
    const bool active = rt < row_tiles;
    if (!active) rt = row_tiles - 1;
    const int kb_total = a.kdim / TILE_COLS;
    const int kb0 = (int)((int64_t)ks * kb_total / a.ksplit);
    const int kb1 = (int)((int64_t)(ks + 1) * kb_total / a.ksplit);
    const uint16_t *wa = a.w_a[g];
    const uint16_t *wb = (NM == 2) ? a.w_b[g] : nullptr;

    constexpr int PT = DENSE ? SG_MAX_TILES : SG_POS_TILES;
    const int tiles0 = (n0 + 15) >> 4, tiles1 = (n1 + 15) >> 4;
    for (int t0 = 0, t1 = 0; t0 < tiles0 || t1 < tiles1; t0 += PT, t1 += PT) {
        int c0 = min(PT, max(tiles0 - t0, 0));
        int c1 = min(PT, max(tiles1 - t1, 0));
#define PZL_PASS(A, B)                                                                               \
    stream_pass<NM, DENSE, A, B>(a, wa, wb, rt, active, kb0, kb1, ks, base0, n0, t0, base1, n1, t1, \
                                 xs, rowidx)
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

template <int NM, bool DENSE>
static int launch(const StreamGroupArgs &g, hipStream_t st)
{
    if (g.n_groups <= 0) return PZL_OK;
    if (g.rows % TILE_ROWS || g.kdim % TILE_COLS || g.ksplit < 1) return PZL_EINVAL;
    SgArgs a;
    a.w_a = g.w_a; a.w_b = g.w_b; a.rows = g.rows; a.kdim = g.kdim; a.ksplit = g.ksplit;
    a.act = g.act; a.act_is_x = g.act_is_x; a.act_slot_base = g.act_slot_base;
    a.cnt = g.cnt; a.off = g.off; a.slot_tok = g.slot_tok;
    a.dense_tokens = g.dense_tokens; a.dense_slot_base = g.dense_slot_base;
    a.h_out = g.h_out; a.h_slot_base = g.h_slot_base; a.o_out = g.o_out; a.o_ks_stride = g.o_ks_stride;
    const int row_tiles = g.rows / TILE_ROWS;
    const int row_groups = (row_tiles + SG_WAVES - 1) / SG_WAVES;
    const int64_t blocks = (int64_t)g.n_groups * row_groups * g.ksplit;
    if (blocks > 0x7FFFFFFFLL) return PZL_EINVAL;
    const size_t lds = SG_LDS_BYTES + SG_MAX_TILES * 16 * sizeof(int32_t);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)stream_kernel<NM, DENSE>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) { set_hip_error(e); return PZL_EHIP; }
        attr_set = true;
    }
    hipLaunchKernelGGL((stream_kernel<NM, DENSE>), dim3((unsigned)blocks), dim3(SG_THREADS), lds, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_hip_error(e); return PZL_EHIP; }
    return PZL_OK;
}

int launch_stream_gateup(const StreamGroupArgs &a, bool dense, hipStream_t st)
{
    return dense ? launch<2, true>(a, st) : launch<2, false>(a, st);
}

int launch_stream_down(const StreamGroupArgs &a, bool dense, hipStream_t st)
{
    return dense ? launch<1, true>(a, st) : launch<1, false>(a, st);
}

}  // namespace pzl
