// Tiled decode-GEMM for large token counts per expert (prefill-sized batches): a dense
// contraction on the matrix cores.
//
// Sec. 3.3.2 asks that every packed weight be decoded (Algorithm 1) right before it is
// multiplied and that the decoded matrix never be materialised in memory.  With hundreds of
// tokens per expert the work is MFMA-bound, so here a workgroup decodes each packed 16x32
// tile ONCE into LDS (as bf16, already in matrix-core operand order) and all four waves
// multiply it with up to 256 tokens: the decode cost is amortised over the token tile, and
// the decoded weights live only in LDS.
//
// Workgroup tile (defaults): up to 256 tokens of one expert x 256 weight rows (gate/up stage: the
// same 128 feature rows of the gate and of the up matrix, so SwiGLU runs on the accumulators;
// down stage: 256 rows of the down matrix, with both planes (hi, lo) of H as the token operand).
// 8 waves as 2 (tokens) x 4 (rows), two per SIMD; a wave accumulates up to 8 token fragments x
// 4 row tiles of v_mfma_f32_16x16x32_bf16 (128 accumulator registers, which keeps the wave inside
// the 256 registers it gets at two waves per SIMD).  K advances 64 (gate/up) or 32 (down) per
// step; the global loads of step k+1 are in flight while step k is multiplied; LDS is
// double-buffered, one barrier per step.
//
// Measured alternatives on the Mixtral-shaped prefill (T = 4096), all slower than the default:
// 4 waves with 256 accumulators each (1 wave per SIMD), 4-wave 256x128 / 128x128 tiles with two
// workgroups per compute unit, weights loaded two steps ahead, three LDS stages with fragment
// read-ahead across the barrier.  The shape macros below are kept so they can be re-measured.
//
// Token tiles are cut per expert into equal parts of at most 256 tokens (rounded up to 16),
// so a 1030-token expert costs 5 x 208 rows rather than 5 x 256.
#include "pzl_common.h"

namespace pzl {

#ifndef TG_WN
#define TG_WN 4            // waves along the weight rows (2 more along the tokens)
#endif
#ifndef TG_RT
#define TG_RT 4            // 16-row weight tiles per wave
#endif
#ifndef TG_KBS_GATEUP
#define TG_KBS_GATEUP 2    // k-blocks of 32 per K step, gate/up stage
#endif
#ifndef TG_DOWN_TOK
#define TG_DOWN_TOK 256    // tokens per down tile (256, or 128: half a gate/up tile)
#endif
#ifndef TG_WPE
#define TG_WPE 2
#endif
constexpr int TG_WAVES = 2 * TG_WN;
constexpr int TG_THREADS = TG_WAVES * 64;
constexpr int TG_MAX_TOK = 256;          // tokens per gate/up tile (16 fragments of 16)
constexpr int TG_ROW_TILES = TG_WN * TG_RT;   // 16-row weight tiles per workgroup
constexpr int TG_STAGE_UNITS = (TG_ROW_TILES + 16) * TG_KBS_GATEUP * 64 > (TG_ROW_TILES + 2 * TG_DOWN_TOK / 16) * 64
                                   ? (TG_ROW_TILES + 16) * TG_KBS_GATEUP * 64
                                   : (TG_ROW_TILES + 2 * TG_DOWN_TOK / 16) * 64;   // 16-byte units per LDS stage
constexpr int TG_LDS_BYTES = 2 * TG_STAGE_UNITS * 16 + TG_MAX_TOK * 4;
constexpr int TSTAGE_GATEUP = 0, TSTAGE_DOWN = 1;
#ifndef TG_BLOCK_M
#define TG_BLOCK_M 8
#endif
#ifndef TG_BLOCK_N
#define TG_BLOCK_N 4
#endif

struct TgArgs {
    const uint16_t *const *w_a;
    const uint16_t *const *w_b;
    int32_t rows, kdim;
    const uint16_t *act;
    int64_t act_plane_stride;
    int32_t act_is_x, act_slot_base;
    const int32_t *slot_tok;
    const int32_t *tile_q, *tile_slot0, *tile_n, *n_tiles;   // routed: device tile list
    int32_t group_lo, group_hi;                              // routed: this launch owns groups [lo, hi)
    int32_t dense_tokens, dense_slot_base, dense_tiles, dense_tile_tokens;   // dense: uniform tiles
    uint16_t *h_out;
    int64_t h_plane_stride;
    int32_t h_slot_base;
    float *o_out;
    int64_t o_ks_stride;
    int32_t max_mtiles, n_ntiles, ksplit;
};

__device__ __forceinline__ uint32_t tg_decode_body(uint32_t x) { return (x & 0x0FFF0FFFu) + 0x38003800u; }

template <int POS>
__device__ __forceinline__ uint32_t tg_decode_pair(uint32_t x)
{
    uint32_t body = tg_decode_body(x);
    uint32_t xs = POS ? (x << 1) : x;
    s16x2 t = __builtin_bit_cast(s16x2, x << (2 + POS));
    t = t >> 15;
    uint32_t m = __builtin_bit_cast(uint32_t, t);
    return ((xs & 0x80008000u) | body) & m;
}

template <int POS, bool DENSE>
__device__ __forceinline__ u32x4 tg_decode(u32x4 w)
{
    if (DENSE) return w;
    u32x4 o;
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = tg_decode_pair<POS>(w[i]);
    return o;
}

__device__ __forceinline__ uint32_t tg_bf16_rne(float v)
{
    uint32_t u = __float_as_uint(v);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0u;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

__device__ __forceinline__ void tg_swiglu_split(float g, float u, uint32_t &hi, uint32_t &lo)
{
    float h = (g / (1.0f + __expf(-g))) * u;
    hi = tg_bf16_rne(h);
    lo = tg_bf16_rne(h - __uint_as_float(hi << 16));
}

// The whole tile for one expert position (POS is the position of the expert inside its pair).
// CNT = token fragments per wave: both token-side waves take ceil(n_frags / 2) fragments, so the
// K loop has no data-dependent branch (a guard per fragment makes the register allocator move
// accumulators between register files); an odd tile costs one padded fragment.
// DENSE: plain bf16 weights (identity decode).  ALLTOK: a shared expert, uniform token tiles
// over every token instead of the routed tile list.
template <int STAGE, bool DENSE, bool ALLTOK, int POS, int CNT>
__device__ __forceinline__ void tile_body(const TgArgs &a, const uint16_t *wa, const uint16_t *wb,
                                          int slot0, int n_tok, int ntile, int ks, u32x4 *lds, int32_t *rowidx)
{
    constexpr int KBS = (STAGE == TSTAGE_DOWN) ? 1 : TG_KBS_GATEUP;   // k-blocks (of 32) per K step
    constexpr int FR = (STAGE == TSTAGE_DOWN) ? TG_DOWN_TOK / 16 : TG_MAX_TOK / 16;   // token fragment slots
    constexpr int PARTS = (STAGE == TSTAGE_DOWN) ? 2 : 1;    // activation planes (hi, lo)
    constexpr int W_UNITS = TG_ROW_TILES * KBS * 64;         // 16-byte units of decoded weights per stage
    constexpr int X_UNITS = PARTS * FR * KBS * 64;
    static_assert(W_UNITS + X_UNITS <= TG_STAGE_UNITS, "stage does not fit");
    constexpr int WPT = TG_ROW_TILES * KBS / TG_WAVES;       // weight tiles each wave loads per step
    constexpr int XPT = PARTS * FR * KBS / TG_WAVES;         // activation fragments each wave loads per step
    constexpr int RT = TG_RT;                                // row tiles per wave

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wm = __builtin_amdgcn_readfirstlane(wave & 1);  // wave position along tokens
    const int wn = __builtin_amdgcn_readfirstlane(wave >> 1); // wave position along rows
    const int kb_total = a.kdim / TILE_COLS;
    // this workgroup's share of K (the down stage may be split over several workgroups)
    const int kb0 = (int)((int64_t)ks * kb_total / a.ksplit);
    const int kb1 = (int)((int64_t)(ks + 1) * kb_total / a.ksplit);
    const int n_steps = (kb1 - kb0 + KBS - 1) / KBS;
    const int frag0 = wm * CNT;                              // fragments frag0 .. frag0+CNT-1 (< 16)
    const int row_tiles = a.rows / TILE_ROWS;

    // activation row behind each token column of the tile (clamped to the last valid token)
    if (tid < TG_MAX_TOK) {
        int slot = slot0 + min(tid, n_tok - 1);
        int row;
        if (a.act_is_x) row = ALLTOK ? (slot - a.dense_slot_base) % a.dense_tokens : a.slot_tok[slot];
        else            row = slot - a.act_slot_base;
        rowidx[tid] = row;
    }
    __syncthreads();

    // ---- what this wave loads each step --------------------------------------------------
    // weights: tile t = wave*WPT + i  ->  (local row tile t / KBS, k-block t % KBS)
    // (the tile base is the same for all lanes: keep it in scalar registers and add the lane)
    typedef const u32x4 __attribute__((address_space(1))) *gvec_ptr;
    uint64_t wbase[WPT];
#pragma unroll
    for (int i = 0; i < WPT; ++i) {
        int t = wave * WPT + i;
        int lrt = t / KBS, kbo = t % KBS;
        int grt;                                              // global row tile, clamped to the matrix
        const uint16_t *base;
        if (STAGE == TSTAGE_GATEUP) {
            constexpr int HALF = TG_ROW_TILES / 2;            // local tiles [0,HALF) gate, [HALF,2*HALF) up
            base = (lrt < HALF) ? wa : wb;
            grt = min(ntile * HALF + (lrt % HALF), row_tiles - 1);
        } else {
            base = wa;
            grt = min(ntile * TG_ROW_TILES + lrt, row_tiles - 1);
        }
        uint64_t p = (uint64_t)(uintptr_t)base + (((int64_t)grt * kb_total + kbo) * 64) * 16;
        uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)p);
        uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(p >> 32));
        wbase[i] = ((uint64_t)hi << 32) | lo;
    }
    // activations: fragment column c = wave*XPT + i -> (plane, token fragment, k-block);
    // 32-bit element offsets from the activation base (every activation buffer is < 2^31 elements)
    uint32_t xoff[XPT];
#pragma unroll
    for (int i = 0; i < XPT; ++i) {
        int c = wave * XPT + i;
        int kbo = c % KBS, fr = (c / KBS) % FR, part = c / (KBS * FR);
        xoff[i] = (uint32_t)(part * a.act_plane_stride) +
                  (uint32_t)rowidx[fr * 16 + (lane & 15)] * (uint32_t)a.kdim + kbo * TILE_COLS + (lane >> 4) * 8;
    }

    u32x4 wreg[WPT], xreg[XPT];
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    auto issue_loads = [&](int step) {
        // a k-block past the end re-reads the last valid one; its activations are stored as zero
#pragma unroll
        for (int i = 0; i < WPT; ++i) {
            int kbo = (wave * WPT + i) % KBS;
            int kb = min(kb0 + step * KBS + kbo, kb1 - 1) - kbo;
            wreg[i] = __builtin_nontemporal_load((gvec_ptr)wbase[i] + (int64_t)kb * 64 + lane);
        }
#pragma unroll
        for (int i = 0; i < XPT; ++i) {
            int kbo = (wave * XPT + i) % KBS;
            int kb = min(kb0 + step * KBS + kbo, kb1 - 1) - kbo;
            xreg[i] = *(const u32x4 *)(a.act + (xoff[i] + (uint32_t)(kb * TILE_COLS)));
        }
    };
    auto store_stage = [&](int stage, int step) {
        u32x4 *ws = lds + stage * TG_STAGE_UNITS;
        u32x4 *xs = ws + W_UNITS;
#pragma unroll
        for (int i = 0; i < WPT; ++i)
            ws[(wave * WPT + i) * 64 + lane] = tg_decode<POS, DENSE>(wreg[i]);
#pragma unroll
        for (int i = 0; i < XPT; ++i) {
            int c = wave * XPT + i;
            bool valid = kb0 + step * KBS + c % KBS < kb1;
            xs[c * 64 + lane] = valid ? xreg[i] : zero4;
        }
    };

    f32x4 acc[RT][CNT];
#pragma unroll
    for (int j = 0; j < RT; ++j)
#pragma unroll
        for (int i = 0; i < CNT; ++i) acc[j][i] = (f32x4){0.f, 0.f, 0.f, 0.f};

    issue_loads(0);
    store_stage(0, 0);
    __syncthreads();

    for (int step = 0; step < n_steps; ++step) {
        const bool has_next = step + 1 < n_steps;
        if (has_next) issue_loads(step + 1);

        const u32x4 *ws = lds + (step & 1) * TG_STAGE_UNITS;
        const u32x4 *xs = ws + W_UNITS;
#pragma unroll
        for (int kbo = 0; kbo < KBS; ++kbo) {
            // this wave's 4 weight row tiles: gate/up stage -> gate tiles wn*2, wn*2+1 and up tiles
            // 4+wn*2, 4+wn*2+1 (same feature rows); down stage -> tiles wn*4..+3
            bf16x8 af[RT];
#pragma unroll
            for (int j = 0; j < RT; ++j) {
                int lrt = (STAGE == TSTAGE_GATEUP) ? ((j < RT / 2) ? wn * (RT / 2) + j : TG_ROW_TILES / 2 + wn * (RT / 2) + (j - RT / 2)) : wn * RT + j;
                af[j] = __builtin_bit_cast(bf16x8, ws[(lrt * KBS + kbo) * 64 + lane]);
            }
#pragma unroll
            for (int i = 0; i < CNT; ++i) {
#pragma unroll
                for (int part = 0; part < PARTS; ++part) {
                    bf16x8 b = __builtin_bit_cast(bf16x8, xs[((part * FR + frag0 + i) * KBS + kbo) * 64 + lane]);
#pragma unroll
                    for (int j = 0; j < RT; ++j)
                        acc[j][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[j], b, acc[j][i], 0, 0, 0);
                }
            }
        }
        if (has_next) store_stage((step + 1) & 1, step + 1);
        __syncthreads();
    }

    // ---- epilogue: lane holds rows 4*(lane/16)..+3 of its row tile for token column lane%16 ----
    const int col = lane & 15, rsub = (lane >> 4) * 4;
#pragma unroll
    for (int i = 0; i < CNT; ++i) {
        int within = (frag0 + i) * 16 + col;
        if (within >= n_tok) continue;
        int slot = slot0 + within;
        if (STAGE == TSTAGE_GATEUP) {
#pragma unroll
            for (int j = 0; j < RT / 2; ++j) {
                int grt = ntile * (TG_ROW_TILES / 2) + wn * (RT / 2) + j;
                if (grt >= row_tiles) continue;
                f32x4 g = acc[j][i], u = acc[j + RT / 2][i];
                uint32_t hi[4], lo[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) tg_swiglu_split(g[r], u[r], hi[r], lo[r]);
                u32x2 ohi = {hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16)};
                u32x2 olo = {lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16)};
                uint16_t *dst = a.h_out + (int64_t)(slot - a.h_slot_base) * a.rows + grt * 16 + rsub;
                *(u32x2 *)dst = ohi;
                *(u32x2 *)(dst + a.h_plane_stride) = olo;
            }
        } else {
#pragma unroll
            for (int j = 0; j < RT; ++j) {
                int grt = ntile * TG_ROW_TILES + wn * RT + j;
                if (grt >= row_tiles) continue;
                *(f32x4 *)(a.o_out + (int64_t)ks * a.o_ks_stride + (int64_t)slot * a.rows + grt * 16 + rsub) = acc[j][i];
            }
        }
    }
}

template <int STAGE, bool DENSE, bool ALLTOK>
__global__ void __launch_bounds__(TG_THREADS) __attribute__((amdgpu_waves_per_eu(TG_WPE, TG_WPE)))
tile_kernel(TgArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    u32x4 *lds = (u32x4 *)lds_raw;
    int32_t *rowidx = (int32_t *)(lds_raw + 2 * TG_STAGE_UNITS * 16);

    // XCD-aware order.  Consecutive workgroup ids go to different XCDs (8 of them, each with its
    // own L2), so give each XCD a contiguous range of logical ids.  The 32 workgroups an XCD runs
    // at a time form a block of 4 token tiles x 8 row tiles that march through K together: each
    // K slice of activations is shared by 8 of them and each slice of weights by 4, instead of
    // 32 workgroups streaming 32 different activation tiles through one L2.
    const int total = gridDim.x;
    const int per_xcd = total / 8;
    int logical = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    const int per_ks = total / a.ksplit;                     // K splits are the slowest index
    const int ks = logical / per_ks;
    logical -= ks * per_ks;
    const int gm_count = (a.max_mtiles + TG_BLOCK_M - 1) / TG_BLOCK_M;
    const int blk = logical / (TG_BLOCK_M * TG_BLOCK_N), r = logical % (TG_BLOCK_M * TG_BLOCK_N);
    const int mt_raw = (blk % gm_count) * TG_BLOCK_M + r % TG_BLOCK_M;
    const int ntile = (blk / gm_count) * TG_BLOCK_N + r / TG_BLOCK_M;
    if (mt_raw >= a.max_mtiles || ntile >= a.n_ntiles) return;

    // the down stage takes a gate/up token tile in two halves of at most TG_DOWN_TOK tokens
    constexpr int HALVES = (STAGE == TSTAGE_DOWN) ? TG_MAX_TOK / TG_DOWN_TOK : 1;
    const int half = mt_raw % HALVES;
    const int mt = mt_raw / HALVES;
    int g, pos, slot0, n_tok;
    if (ALLTOK) {
        if (mt >= a.dense_tiles) return;
        g = mt / ((a.dense_tokens + a.dense_tile_tokens - 1) / a.dense_tile_tokens);
        int t_in = mt % ((a.dense_tokens + a.dense_tile_tokens - 1) / a.dense_tile_tokens);
        pos = 0;
        slot0 = a.dense_slot_base + g * a.dense_tokens + t_in * a.dense_tile_tokens;
        n_tok = min(a.dense_tile_tokens, a.dense_tokens - t_in * a.dense_tile_tokens);
    } else {
        if (mt >= *a.n_tiles) return;
        int q = a.tile_q[mt];
        g = q >> 1; pos = q & 1;
        if (g < a.group_lo || g >= a.group_hi) return;       // another launch's kind of expert
        g -= a.group_lo;
        slot0 = a.tile_slot0[mt];
        n_tok = a.tile_n[mt];
    }
    if (STAGE == TSTAGE_DOWN) {
        slot0 += half * TG_DOWN_TOK;
        n_tok = min(n_tok - half * TG_DOWN_TOK, TG_DOWN_TOK);
        if (n_tok <= 0) return;
    }
    // these are the same for the whole workgroup; say so, or the per-fragment guards below become
    // exec-masked branches and the accumulators get shuffled between register files
    g = __builtin_amdgcn_readfirstlane(g);
    pos = __builtin_amdgcn_readfirstlane(pos);
    slot0 = __builtin_amdgcn_readfirstlane(slot0);
    n_tok = __builtin_amdgcn_readfirstlane(n_tok);
    const uint16_t *wa = a.w_a[g];
    const uint16_t *wb = (STAGE == TSTAGE_GATEUP) ? a.w_b[g] : wa;
    const int cnt = (((n_tok + 15) >> 4) + 1) >> 1;          // 1..8 fragments per wave
#define PZL_TILE(P, C) tile_body<STAGE, DENSE, ALLTOK, P, C>(a, wa, wb, slot0, n_tok, ntile, ks, lds, rowidx)
#define PZL_TILE_CNT(P)                                                         \
    switch (cnt) {                                                              \
        case 1: PZL_TILE(P, 1); break; case 2: PZL_TILE(P, 2); break;           \
        case 3: PZL_TILE(P, 3); break; case 4: PZL_TILE(P, 4); break;           \
        case 5: PZL_TILE(P, 5); break; case 6: PZL_TILE(P, 6); break;           \
        case 7: PZL_TILE(P, 7); break; default: PZL_TILE(P, 8); break;          \
    }
    if (DENSE || pos == 0) { PZL_TILE_CNT(0) } else { PZL_TILE_CNT(1) }
#undef PZL_TILE_CNT
#undef PZL_TILE
}

template <int STAGE, bool DENSE, bool ALLTOK>
static int launch(const TileGemmArgs &t, hipStream_t st)
{
    if (t.max_mtiles <= 0) return PZL_OK;
    if (t.rows % TILE_ROWS || t.kdim % TILE_COLS) return PZL_EINVAL;
    TgArgs a;
    a.w_a = t.w_a; a.w_b = t.w_b; a.rows = t.rows; a.kdim = t.kdim;
    a.act = t.act; a.act_plane_stride = t.act_plane_stride; a.act_is_x = t.act_is_x;
    a.act_slot_base = t.act_slot_base; a.slot_tok = t.slot_tok;
    a.tile_q = t.tile_q; a.tile_slot0 = t.tile_slot0; a.tile_n = t.tile_n; a.n_tiles = t.n_tiles;
    a.group_lo = t.group_lo; a.group_hi = t.group_hi;
    a.dense_tokens = t.dense_tokens; a.dense_slot_base = t.dense_slot_base;
    a.dense_tiles = t.dense_tiles; a.dense_tile_tokens = t.dense_tile_tokens;
    a.h_out = t.h_out; a.h_plane_stride = t.h_plane_stride; a.h_slot_base = t.h_slot_base;
    a.o_out = t.o_out; a.o_ks_stride = t.o_ks_stride;
    a.ksplit = (STAGE == TSTAGE_DOWN && t.ksplit > 1) ? t.ksplit : 1;
    a.max_mtiles = t.max_mtiles * ((STAGE == TSTAGE_DOWN) ? TG_MAX_TOK / TG_DOWN_TOK : 1);
    const int rows_per_wg = (STAGE == TSTAGE_GATEUP) ? TG_ROW_TILES * 8 : TG_ROW_TILES * 16;
    a.n_ntiles = (t.rows + rows_per_wg - 1) / rows_per_wg;
    int64_t blocks = (int64_t)((a.max_mtiles + TG_BLOCK_M - 1) / TG_BLOCK_M) *
                     ((a.n_ntiles + TG_BLOCK_N - 1) / TG_BLOCK_N) * (TG_BLOCK_M * TG_BLOCK_N);
    blocks = (blocks + 7) / 8 * 8 * a.ksplit;
    if (blocks > 0x7FFFFFFFLL) return PZL_EINVAL;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)tile_kernel<STAGE, DENSE, ALLTOK>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, TG_LDS_BYTES);
        if (e != hipSuccess) { set_hip_error(e); return PZL_EHIP; }
        attr_set = true;
    }
    hipLaunchKernelGGL((tile_kernel<STAGE, DENSE, ALLTOK>), dim3((unsigned)blocks), dim3(TG_THREADS), TG_LDS_BYTES, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_hip_error(e); return PZL_EHIP; }
    return PZL_OK;
}

// kind: 0 = packed pairs (routed), 1 = dense experts that see every token (shared),
//       2 = dense routed experts (kept unmerged)
int launch_tile_gateup(const TileGemmArgs &a, int kind, hipStream_t st)
{
    if (kind == 0) return launch<TSTAGE_GATEUP, false, false>(a, st);
    if (kind == 1) return launch<TSTAGE_GATEUP, true, true>(a, st);
    return launch<TSTAGE_GATEUP, true, false>(a, st);
}

int launch_tile_down(const TileGemmArgs &a, int kind, hipStream_t st)
{
    if (kind == 0) return launch<TSTAGE_DOWN, false, false>(a, st);
    if (kind == 1) return launch<TSTAGE_DOWN, true, true>(a, st);
    return launch<TSTAGE_DOWN, true, false>(a, st);
}

}  // namespace pzl
