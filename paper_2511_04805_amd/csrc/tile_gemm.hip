// Tiled decode-GEMM for large token counts per expert (prefill-sized batches): a dense
// contraction on the matrix cores.
//
// Sec. 3.3.2 asks that every packed weight be decoded (Algorithm 1) right before it is
// multiplied and that the decoded matrix never be materialised in memory.  Here the decoded
// weights do not even reach LDS: each wave loads the packed 16x32 tiles of its own weight rows
// straight into registers (the tiled layout is already the A operand of
// v_mfma_f32_16x16x32_bf16), decodes them there and multiplies them with every token of the
// tile, so each packed word is decoded once per up to 288 tokens.
//
// Workgroup tile: up to 288 tokens of one expert x 256 weight rows (gate/up stage: the same 128
// feature rows of the gate and of the up matrix, so SwiGLU runs on the accumulators; down stage:
// 256 rows of the down matrix, with both planes (hi, lo) of H as the token operand).  8 waves,
// all along the weight rows: a wave owns 2 row tiles (gate + up of 16 features, or 2 down tiles)
// and all (up to 18) token fragments, up to 144 accumulator registers, two waves per SIMD.
//
// Token operand: activation rows are gathered by `global_load_lds_dwordx4`, which writes a whole
// fragment (64 lanes x 16 bytes, already in B operand order) into LDS without passing through
// registers.  LDS holds a ring of 4 such stages (36 KiB each: 64 K elements of 288 tokens, or 32
// of both H planes), filled three steps ahead; the weights are loaded two steps ahead into two
// register sets.  One barrier per K step publishes the stage written two steps earlier; no wave
// writes LDS with ds_write at all.  (Measured on this chip: ds_write_b128 sustains about
// 70 B/clk per compute unit against 210 B/clk for ds_read_b128, which is why the earlier design,
// decoded weights staged through LDS by all waves, stalled.)
//
// Memory operations complete in issue order, and every step issues [activation stage s+3,
// weights s+2] in that order; waiting for the weights of step s (which the decode does) therefore
// also covers the activation stage s+1 issued before them, which the barrier at the end of step
// s then makes visible to the other waves.
//
// Token tiles are cut per expert into equal parts of at most 288 tokens (rounded up to 16).  The
// limit is what registers and LDS allow, not a power of two: a tile with few tokens streams the
// same weights as a full one and costs about half as much (measured), so an expert with 1030
// tokens is far better served by 4 tiles of 272 than by 4 of 256 and one of 6, or by 5 of 208.
// For the same reason a pair whose two experts both have few tokens can get one tile for both
// (tile_body with POS = 2): its packed words are loaded once and decoded for both positions.
//
// Launch forms (tile_kernel): one workgroup per tile, or, where the host's bound on the number of
// tiles is loose and tiles are uneven (many experts), 256 persistent workgroups that work through
// the tile list, by fixed stride first and then drawing from a counter.
#include <type_traits>
#include "pzl_common.h"
#include "pzl_decode.h"

namespace pzl {

#ifndef TG_WPE
#define TG_WPE 2
#endif
#ifndef TG_KBS_N
#define TG_KBS_N 1          // k-blocks (of 32) per K step where one activation plane is read (measured: 1 is 5 % faster than 2 where K is 2048, equal at 4096)
#endif
constexpr int TG_WAVES = TG_WAVES_N;
constexpr int TG_THREADS = TG_WAVES * 64;
constexpr int TG_MAX_TOK = TILE_MAX_TOKENS;   // tokens per tile (18 fragments of 16)
constexpr int TG_FRAGS = TG_MAX_TOK / 16;
constexpr int TG_ROW_TILES = 2 * TG_WAVES;    // 16-row weight tiles per workgroup
// 16-byte units per ring stage: 18 fragments x (k-blocks per step) x (activation planes)
template <int STAGE, bool HALF, bool DENSE>
constexpr int tg_stage_units()
{
    return (STAGE == 1 /* down */ && !HALF) ? TG_FRAGS * 2 * 64 : TG_FRAGS * TG_KBS_N * 64;
}
constexpr int TSTAGE_GATEUP = 0, TSTAGE_DOWN = 1;
constexpr int TG_PERSISTENT_WGS = 256 * (8 / TG_WAVES);   // workgroups of a persistent launch: as many as the chip holds (8 waves per compute unit)
// Stages of the activation ring: 8 where a stage is 18 KiB (one activation plane, K step 32), which
// lets a step read the first fragments of the next stage before its closing barrier; else 4.
template <int STAGE, bool HALF, bool DENSE>
constexpr int tg_ring_stages() { return tg_stage_units<STAGE, HALF, DENSE>() * 16 * 8 <= 147456 ? 8 : 4; }
#ifndef TG_QUARTER_LOADS
#define TG_QUARTER_LOADS 1
#endif
constexpr int TG_ODD_MIN_CNT = 5;           // pairs of fragments from which a tile with an odd number of fragments has its own loop
constexpr int TG_BLOCK_WGS = 32;            // workgroups an XCD runs side by side (32 compute units): one block of token tiles x row blocks

// Activations in fragment order.  A tile's token operand is what its K loop reads most often from
// L2: 16 rows x 32 columns per fragment and K step, 64 bytes from each of 16 rows that lie
// wherever the router put them (x) or f elements apart (H) -- half of every 128-byte line fetched
// for nothing.  In a fragment-ordered buffer the 1 KiB that one load instruction moves is
// contiguous: 16 token rows form a block of 16 * K elements, inside it k-block after k-block, each
// as the 64 lanes x 8 elements of the matrix instruction's B operand.  Tile number mt of the
// tile list owns the blocks from row slot0 + 32 * mt on (its slots are contiguous from slot0; a
// tile has at most 31 rows of padding, so the blocks of successive tiles never overlap; the
// buffers hold TILE_FRAG_PAD_ROWS rows per tile of the list's bound beyond the slots).  The gate/up
// stage writes H that way for the down stage at no cost (same 8-byte stores, other addresses); x
// needs a gathering pass in front (gather_x_kernel), which pays for wide experts only.
// Measured on the Mixtral-shaped prefill with both: gate/up -3 %, down -5 %.
__device__ __forceinline__ int tg_frag_row(int slot0, int mt) { return slot0 + TILE_FRAG_PAD_ROWS * mt; }

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
    // Activations in fragment order (see tg_frag_row): the stage's input, if it has such a copy, and
    // (gate/up stage) where H goes in that order.  Tiles that cover both experts of a pair keep the
    // row-major buffers.
    const uint16_t *act_frag;
    uint16_t *h_frag;
    float *o_out;
    int64_t o_ks_stride;
    int32_t max_mtiles, n_ntiles, ksplit;
    int32_t block_m;              // token tiles per block of TG_BLOCK_WGS workgroups (8 or 4; the rest are row blocks)
    int32_t *tile_ctr;
    int32_t *h_saturated;
    float out_scale;              // half-precision down stage: what its sums are multiplied by (the weights' scale undone)
    uint32_t dense_clamp2, dense_bias2;   // ... of dense weights: the constants of dense_pair_to_half_scaled
};

// One packed 16x32 tile decoded for position POS, as raw bits: bf16, or (HALFW) half precision
// times 2 (pzl_decode.h).
template <int POS, bool DENSE, bool HALFW>
__device__ __forceinline__ u32x4 tg_decode(u32x4 w)
{
    u32x4 o;
    if (DENSE) {
        // An identity "decode" still has to produce NEW registers (an opaque copy): if the operand
        // were the load's own registers, the compiler would keep them alive past the refill,
        // rename the refill and copy it back at the loop edge while it is still in flight.
        uint32_t o0, o1, o2, o3;
        asm("v_mov_b32 %0, %4\n\tv_mov_b32 %1, %5\n\tv_mov_b32 %2, %6\n\tv_mov_b32 %3, %7"
            : "=&v"(o0), "=&v"(o1), "=&v"(o2), "=&v"(o3) : "v"(w[0]), "v"(w[1]), "v"(w[2]), "v"(w[3]));
        return (u32x4){o0, o1, o2, o3};
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = decode_pair<POS>(w[i], HALFW ? decode_body_half_x2(w[i]) : decode_body(w[i]));
    return o;
}

typedef _Float16 tg_f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 tg_f16x2 __attribute__((ext_vector_type(2)));

template <bool HALFW>
__device__ __forceinline__ f32x4 tg_mma(u32x4 a, u32x4 b, f32x4 acc)
{
    if (HALFW) return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(tg_f16x8, a), __builtin_bit_cast(tg_f16x8, b), acc, 0, 0, 0);
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
}

typedef __bf16 tg_bf16x2 __attribute__((ext_vector_type(2)));
typedef float tg_f32x2 __attribute__((ext_vector_type(2)));

// silu(g) * u for two elements, split into a bf16 pair of leading parts and a bf16 pair of
// remainders (low half = first element).  Reciprocal and exponential are the hardware's
// approximations (1 ulp), far inside the error budget; the conversions are the hardware's
// round-to-nearest-even.  The tile's epilogue is pure vector arithmetic with no matrix work to
// hide behind, so its instruction count is wall time.
__device__ __forceinline__ void tg_swiglu_split2(float g0, float u0, float g1, float u1, uint32_t &hi, uint32_t &lo)
{
    float h0 = g0 * __builtin_amdgcn_rcpf(1.0f + __expf(-g0)) * u0;
    float h1 = g1 * __builtin_amdgcn_rcpf(1.0f + __expf(-g1)) * u1;
    hi = __builtin_bit_cast(uint32_t, __builtin_convertvector((tg_f32x2){h0, h1}, tg_bf16x2));
    float r0 = h0 - __uint_as_float(hi << 16), r1 = h1 - __uint_as_float(hi & 0xFFFF0000u);
    lo = __builtin_bit_cast(uint32_t, __builtin_convertvector((tg_f32x2){r0, r1}, tg_bf16x2));
}

// The same for the half-precision form of H: one pair of half-precision numbers, round to nearest
// even; magnitudes beyond the largest half-precision number saturate to it (sat is set), NaN stays NaN.
constexpr float TG_HALF_MAX = 65504.0f;
__device__ __forceinline__ uint32_t tg_swiglu_half2(float g0, float u0, float g1, float u1, bool &sat)
{
    float h0 = g0 * __builtin_amdgcn_rcpf(1.0f + __expf(-g0)) * u0;
    float h1 = g1 * __builtin_amdgcn_rcpf(1.0f + __expf(-g1)) * u1;
    const bool s0 = fabsf(h0) > TG_HALF_MAX, s1 = fabsf(h1) > TG_HALF_MAX;
    h0 = s0 ? copysignf(TG_HALF_MAX, h0) : h0;
    h1 = s1 ? copysignf(TG_HALF_MAX, h1) : h1;
    sat |= s0 | s1;
    return __builtin_bit_cast(uint32_t, __builtin_convertvector((tg_f32x2){h0, h1}, tg_f16x2));
}

typedef const u32x4 __attribute__((address_space(1))) *tg_gvec_ptr;
typedef __attribute__((address_space(3))) void *tg_lds_ptr;

// The whole tile for one expert position (POS is the position of the expert inside its pair).
// CNT = pairs of token fragments (the tile has at most 32*CNT tokens): a template parameter so
// that the K loop has no data-dependent branch; an odd tile costs one padded fragment.
// DENSE: plain bf16 weights (identity decode).  ALLTOK: a shared expert, uniform token tiles
// over every token instead of the routed tile list.
// POS = 2: a tile for BOTH experts of a pair (n_tok tokens of position 0 in the first half of the
// fragments, n_tok1 tokens of position 1, whose slots follow, in the second half; CNT pairs of
// fragments each): every packed word is loaded once and decoded for both positions.
// HALF: H is one plane of half precision (written by the gate/up stage with saturation; the down
// stage then decodes its weights to half precision times 2, uses the f16 matrix instruction with
// K steps of 64 like the gate/up stage, and halves its sums), instead of two bf16 planes.
// ODD: the tile's last fragment is padding (an odd number of fragments in use): it keeps its place
// in the step's groups (LDS read, share of the decode and of the loads), so that the fragment
// ring and the load counts are those of the even tile, but its matrix instructions are left out
// and it has no accumulators: at the power cap a matrix instruction not issued is time won
// (tiles of 17 fragments, Mixtral-shaped prefill: -3 % per launch).
template <int STAGE, bool DENSE, bool ALLTOK, bool HALF, int POS, int CNT, bool ODD = false>
__device__ __forceinline__ void tile_body(const TgArgs &a, const uint16_t *wa, const uint16_t *wb,
                                          int slot0, int n_tok, int n_tok1, int ntile, int ks, int mt,
                                          u32x4 *ring, int32_t *rowidx, int32_t *draw_ctr, int32_t *drawn)
{
    constexpr bool FUSED = POS == 2;
    static_assert(!HALF || !DENSE || ALLTOK, "half-precision H: packed pairs and shared experts");
    constexpr bool HALFW = HALF && STAGE == TSTAGE_DOWN;     // this stage's operands are half precision
    constexpr int KBS = (STAGE == TSTAGE_DOWN && !HALF) ? 1 : TG_KBS_N;      // k-blocks (of 32) per K step
    constexpr int PARTS = (STAGE == TSTAGE_DOWN && !HALF) ? 2 : 1;    // activation planes (hi, lo)
    constexpr int NF = (FUSED ? 4 : 2) * CNT;                // token fragments in use
    constexpr int NFH = FUSED ? NF / 2 : NF;                 // ... of which the first expert's
    constexpr int NFR = NF - (ODD ? 1 : 0);                  // ... that hold tokens
    static_assert(!ODD || !FUSED, "tiles that cover a pair come in whole pairs of fragments");
    static_assert(NF <= TG_FRAGS, "fragments");
    constexpr int RT = 2;                                    // row tiles per wave
    constexpr int XTOTAL = PARTS * NF * KBS;                 // activation fragments per stage
    // ... fetched by the 8 waves with the same number of loads each (the hand-written waits count
    // loads): whole fragments, 16 bytes per lane, as far as they divide by the number of waves;
    // 2 or 4 fragments left over are fetched as quarters (the 16 rows of one 8-element column
    // group: 256 bytes, 4 bytes per lane), one or two per wave.  (A whole-fragment load for every
    // wave, most of them fetching the last fragment again, cost a tile of 18 fragments 24 loads
    // per K step for 18 KiB: the loads of a step, not its matrix instructions, are what a
    // step's length grows with beyond 16 fragments.)
    constexpr int XLEFT = XTOTAL % TG_WAVES;
    constexpr bool XQUART = TG_QUARTER_LOADS && PARTS == 1 && TG_WAVES == 8 && (XLEFT == 2 || XLEFT == 4);
    constexpr int XFULL = XQUART ? XTOTAL / TG_WAVES : (XTOTAL + TG_WAVES - 1) / TG_WAVES;   // whole-fragment loads per wave
    constexpr int XQ = XQUART ? XLEFT / 2 : 0;                                               // quarter loads per wave
    constexpr int XPT = XFULL + XQ;                          // loads per wave and stage
    constexpr int TG_XSTAGE_UNITS = tg_stage_units<STAGE, HALF, DENSE>();
    static_assert(PARTS * TG_FRAGS * KBS * 64 == TG_XSTAGE_UNITS, "stage size");

    // (the thread index passes through an empty asm: what is derived from it is then computed per
    // tile, not once per kernel and kept in registers across the tiles of a persistent workgroup,
    // where the largest tiles have none to spare)
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63;
    const uint32_t lane16 = lane * 16u;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kb_total = a.kdim / TILE_COLS;
    // this workgroup's share of K (the down stage may be split over several workgroups)
    const int kb0 = (int)((int64_t)ks * kb_total / a.ksplit);
    const int kb1 = (int)((int64_t)(ks + 1) * kb_total / a.ksplit);
    const int n_steps = (kb1 - kb0 + KBS - 1) / KBS;
    const int row_tiles = a.rows / TILE_ROWS;

    // activation row behind each token column of the tile (clamped to the last valid token)
    auto set_row = [&](int t) {
        int slot = slot0 + min(t, n_tok - 1);
        if (FUSED && t >= NFH * 16) slot = slot0 + n_tok + min(t - NFH * 16, n_tok1 - 1);
        int row;
        if (a.act_is_x) row = ALLTOK ? (slot - a.dense_slot_base) % a.dense_tokens : a.slot_tok[slot];
        else            row = slot - a.act_slot_base;
        rowidx[t] = row;
    };
    if constexpr (TG_THREADS >= TG_MAX_TOK) {
        if (tid < TG_MAX_TOK) set_row(tid);
    } else {                                       // fewer threads than a tile has tokens
        for (int t = tid; t < TG_MAX_TOK; t += TG_THREADS) set_row(t);
    }
    __syncthreads();

    // ---- this wave's weight rows: gate/up -> tile `wave` of the gate and of the up rows of this
    // workgroup (same 16 features); down -> tiles 2*wave, 2*wave+1.  The tile base is the same for
    // all lanes: keep it in scalar registers and add the lane.
    uint64_t wbase[RT];
#pragma unroll
    for (int j = 0; j < RT; ++j) {
        const uint16_t *base = (STAGE == TSTAGE_GATEUP && j == 1) ? wb : wa;
        int grt = (STAGE == TSTAGE_GATEUP) ? ntile * TG_WAVES + wave : ntile * TG_ROW_TILES + wave * RT + j;
        grt = min(grt, row_tiles - 1);                        // clamped to the matrix; never stored
        uint64_t p = (uint64_t)(uintptr_t)base + ((int64_t)grt * kb_total * 64) * 16;
        uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)p);
        uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(p >> 32));
        wbase[j] = ((uint64_t)hi << 32) | lo;
    }
    // ---- the activation fragments this wave fetches each step: fragment c = wave*XPT + i (the
    // last one repeated if the count does not divide) -> (plane, token fragment, k-block);
    // 32-bit byte offsets from the activation base (every activation buffer is < 2^31 elements):
    // uniform base + 32-bit lane offset is the addressing form that needs no 64-bit vector math
    // (frag_in: this tile reads its token operand from the fragment-ordered copy: a k-block is then
    // 1 KiB further on, not 64 bytes, and the lane's place inside it is the lane itself)
    const bool frag_in = !FUSED && PARTS == 1 && a.act_frag != nullptr;
    const uint32_t frag_base = (uint32_t)tg_frag_row(slot0, mt) * (uint32_t)a.kdim;   // elements
    const uint32_t xkstride = frag_in ? 1024u : (uint32_t)(TILE_COLS * 2);           // bytes per k-block
    uint32_t xoff[XPT];
    int xunit[XPT], xkbo[XPT];
#pragma unroll
    for (int i = 0; i < XPT; ++i) {
        if (i < XFULL) {
            int c = min(wave * XFULL + i, XTOTAL - 1);
            int kbo = c % KBS, fr = (c / KBS) % NF, part = c / (KBS * NF);
            xkbo[i] = kbo;
            xunit[i] = ((part * TG_FRAGS + fr) * KBS + kbo) * 64;
            xoff[i] = 2u * ((uint32_t)(part * a.act_plane_stride) +
                            (uint32_t)rowidx[fr * 16 + (lane & 15)] * (uint32_t)a.kdim + (lane >> 4) * 8);
            if (frag_in) xoff[i] = 2u * (frag_base + (uint32_t)fr * 16u * (uint32_t)a.kdim) + lane16;
        } else {
            // quarter qq of the left-over fragments: lane l fetches 4 bytes, the (l % 4)-th of the
            // 16 that lane 16 * quarter + l / 4 of the fragment holds (row l / 4, column group `quarter`)
            const int qq = wave * XQ + (i - XFULL);
            const int c = TG_WAVES * XFULL + qq / 4, quarter = qq % 4;
            const int kbo = c % KBS, fr = (c / KBS) % NF;
            xkbo[i] = kbo;
            xunit[i] = (fr * KBS + kbo) * 64 + quarter * 16;
            xoff[i] = 2u * ((uint32_t)rowidx[fr * 16 + (lane >> 2)] * (uint32_t)a.kdim + quarter * 8) + (lane & 3) * 4u;
            if (frag_in) xoff[i] = 2u * (frag_base + (uint32_t)fr * 16u * (uint32_t)a.kdim) + quarter * 256u + lane * 4u;
        }
    }

    // a k-block past the end re-reads the last valid one; the last step skips its products
    // Both kinds of load are issued from inline assembly, and waited for by hand (wait_w below):
    // the compiler, seeing a direct-to-LDS load, waits for ALL outstanding loads before the next
    // LDS read, which would undo the prefetch.
    const uint64_t act_base = (uint64_t)(uintptr_t)(frag_in ? a.act_frag : a.act);
    auto fetch_x_one = [&](int step, u32x4 *stage, int i) {
        int kb = min(kb0 + step * KBS + xkbo[i], kb1 - 1);
        uint32_t voff = xoff[i] + (uint32_t)kb * xkstride;
        uint32_t lds_addr = (uint32_t)(uintptr_t)(tg_lds_ptr)(stage + xunit[i]);
        if (i < XFULL)
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                         :: "s"(lds_addr), "v"(voff), "s"(act_base) : "memory");
        else
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
                         :: "s"(lds_addr), "v"(voff), "s"(act_base) : "memory");
    };
    auto fetch_x = [&](int step, u32x4 *stage) {
#pragma unroll
        for (int i = 0; i < XPT; ++i) fetch_x_one(step, stage, i);
    };
    auto fetch_w = [&](int step, u32x4 (&raw)[KBS][RT], int kbo) {
        int kb = min(kb0 + step * KBS + kbo, kb1 - 1);
#pragma unroll
        for (int j = 0; j < RT; ++j) {
            uint64_t base = wbase[j] + (uint64_t)kb * 1024u;
            // in/out operand: the load must land in the registers that the wait and the decode of
            // step + 2 will name; as a plain output the compiler may pick other registers and
            // copy them over at the loop edge, while the load is still in flight
            asm volatile("global_load_dwordx4 %0, %1, %2" : "+v"(raw[kbo][j]) : "v"(lane16), "s"(base));
        }
    };
    f32x4 acc[RT][NF];
#pragma unroll
    for (int j = 0; j < RT; ++j)
#pragma unroll
        for (int i = 0; i < NF; ++i) acc[j][i] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // One K step, decode one step ahead.  The vector ALU and the matrix pipes only run side by side
    // when their instructions alternate in the instruction stream (measured: with the decode of a
    // step in one piece in front of its matrix instructions the two co-execute 3 % of the time and
    // their times add up).  So step s multiplies operands that step s-1 decoded, and decodes the
    // operands of step s+1 between its own matrix instructions.
    //   raw_n    packed weights of step s+1 (loaded at the end of step s-2): waited for, decoded
    //            into dn, then refilled with the weights of step s+3
    //   dc / dn  decoded operands of this step / of the next
    // Loads complete in issue order, so waiting for the weights of step s+1 also completes every
    // older load, the activation stages among them, which the step's closing barrier publishes.
    // Two schedules of the activation ring:
    //   DEEP (8 stages)  a step issues [activation stage s+4, weights s+3]; younger than the weights
    //     of s+1 at the step's start: stage s+3, weights s+2 = XPT + KBS*RT loads; older and hence
    //     complete: stage s+2, which the closing barrier of step s publishes -- one step before it is
    //     read, so that step s can read the first fragments of stage s+1 before its own closing
    //     barrier and the matrix pipes do not drain at every step boundary.  The stage's loads are
    //     spread over the step's first groups.  Slot reuse: stage s+4 overwrites stage s-4, which
    //     every wave left before the barrier of step s-1.
    //   else (4 stages)  a step issues [stage s+3 at its start, weights s+3 at its end]; younger than
    //     the weights of s+1: stage s+2, weights s+2, stage s+3 = 2*XPT + KBS*RT; the closing barrier
    //     publishes stage s+1; slot reuse: stage s+3 overwrites stage s-1.
    constexpr int RING = tg_ring_stages<STAGE, HALF, DENSE>();
    constexpr bool DEEP = RING == 8;
    constexpr int LEAD = DEEP ? 4 : 3;
    struct Dec { u32x4 a[KBS][RT]; u32x4 a1[KBS][RT]; };
    auto wait_step = [&](u32x4 (&raw)[KBS][RT], bool all) {
        // the asm takes the registers as in/out operands so that nothing that uses them can be scheduled above the wait
        constexpr int YOUNGER = (DEEP ? XPT : 2 * XPT) + KBS * RT;
        if (KBS == 1) {
            if (all) asm volatile("s_waitcnt vmcnt(0)" : "+v"(raw[0][0]), "+v"(raw[0][1]));
            else     asm volatile("s_waitcnt vmcnt(%2)" : "+v"(raw[0][0]), "+v"(raw[0][1]) : "n"(YOUNGER));
        } else {
            if (all) asm volatile("s_waitcnt vmcnt(0)" : "+v"(raw[0][0]), "+v"(raw[0][1]), "+v"(raw[KBS - 1][0]), "+v"(raw[KBS - 1][1]));
            else     asm volatile("s_waitcnt vmcnt(%4)" : "+v"(raw[0][0]), "+v"(raw[0][1]), "+v"(raw[KBS - 1][0]), "+v"(raw[KBS - 1][1])
                                  : "n"(YOUNGER));
        }
    };
    static_assert(KBS <= 2, "wait_step names the registers of at most two k-blocks");
    // The step's matrix instructions come in groups: one token fragment read from LDS (RA groups
    // ahead), its RT products, and a share of the next step's decode (and, DEEP, of the activation
    // loads), in that order, group after group (a scheduling fence after each keeps the order in
    // the machine code).  Decode units: one 32-bit word (two elements) of a packed tile, or one
    // whole register quad of a dense one.
    constexpr int GROUPS = NF * PARTS * KBS;
    // fragments read ahead: 3, or 1 for the smallest tiles (the read-ahead may reach into the next
    // stage but not beyond it; the ring of RA+1 fragment registers must divide two steps' groups)
    // (the largest tiles, whose accumulators leave the fewest registers, read 2 ahead)
    constexpr int RA = GROUPS < 4 ? 1 : (NF == TG_FRAGS ? 2 : 3);
    static_assert(GROUPS % 2 == 0 && (2 * GROUPS) % (RA + 1) == 0 && RA <= GROUPS, "fragment register ring");
    static_assert(!DEEP || XPT <= GROUPS, "activation loads are spread over the groups");
    constexpr int UNITS = DENSE ? KBS * RT : KBS * RT * 4;
    auto decode_unit = [&](u32x4 (&raw)[KBS][RT], Dec &d, int u, int step) {
        if (DENSE) {
            const int kbo = u / RT, j = u % RT;
            if (HALFW) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    uint32_t v = dense_pair_to_half_scaled(raw[kbo][j][i], a.dense_clamp2, a.dense_bias2);
                    asm volatile("" : "+v"(v));               // stays between this step's matrix instructions (see below)
                    d.a[kbo][j][i] = v;
                }
            } else {
                d.a[kbo][j] = tg_decode<0, true, false>(raw[kbo][j]);
            }
            if (kbo > 0 && !(kb0 + step * KBS + kbo < kb1)) d.a[kbo][j] = (u32x4){0u, 0u, 0u, 0u};
            d.a1[kbo][j] = d.a[kbo][j];
        } else {
            const int kbo = u / (RT * 4), j = (u / 4) % RT, i = u % 4;
            const uint32_t w = raw[kbo][j][i];
            const uint32_t body = HALFW ? decode_body_half_x2(w) : decode_body(w);
            uint32_t v0 = decode_pair<FUSED ? 0 : POS>(w, body);
            uint32_t v1 = FUSED ? decode_pair<1>(w, body) : v0;
            if (kbo > 0 && !(kb0 + step * KBS + kbo < kb1)) { v0 = 0u; v1 = 0u; }   // a k-block past the end: multiply by zero
            // pin the result to this place in the instruction stream (an empty volatile asm that
            // "uses" it): the compiler otherwise sinks the whole decode to its first use, at the
            // top of the next step, in one piece
            if (FUSED) asm volatile("" : "+v"(v0), "+v"(v1)); else asm volatile("" : "+v"(v0));
            d.a[kbo][j][i] = v0;
            d.a1[kbo][j][i] = FUSED ? v1 : v0;
        }
    };
    // stage of step s
    auto stage = [&](int step) { return ring + (step & (RING - 1)) * TG_XSTAGE_UNITS; };
    auto frag_of = [&](const u32x4 *st, int g) {                 // B fragment of group g of a stage
        const int kbo = g / (NF * PARTS), i = (g % (NF * PARTS)) / PARTS, part = g % PARTS;
        return st[((part * TG_FRAGS + i) * KBS + kbo) * 64 + lane];
    };
    u32x4 bq[RA + 1];                                            // fragments in flight; DEEP: carried across steps
    // PH: the step's parity (two steps per loop trip), which fixes where in the fragment ring it starts
    auto full_step = [&](auto ph, u32x4 (&raw_n)[KBS][RT], const Dec &dc, Dec &dn, int step) {
        constexpr int PH = decltype(ph)::value;
        const u32x4 *cur = stage(step), *nxt = stage(step + 1);
        u32x4 *fill = stage(step + LEAD);
        if (!DEEP) fetch_x(step + LEAD, fill);
        wait_step(raw_n, false);
        __builtin_amdgcn_sched_barrier(0);
        if (!DEEP) {
#pragma unroll
            for (int f = 0; f < RA; ++f) bq[f % (RA + 1)] = frag_of(cur, f);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int g = 0; g < GROUPS; ++g) {
            constexpr int BASE = DEEP ? PH * GROUPS : 0;
            if (g + RA < GROUPS) bq[(BASE + g + RA) % (RA + 1)] = frag_of(cur, g + RA);
            else if (DEEP)       bq[(BASE + g + RA) % (RA + 1)] = frag_of(nxt, g + RA - GROUPS);
            const int kbo = g / (NF * PARTS), i = (g % (NF * PARTS)) / PARTS;
            if (i < NFR) {
#pragma unroll
                for (int j = 0; j < RT; ++j)
                    acc[j][i] = tg_mma<HALFW>((FUSED && i >= NFH) ? dc.a1[kbo][j] : dc.a[kbo][j], bq[(BASE + g) % (RA + 1)], acc[j][i]);
            }
#pragma unroll
            for (int u = g * UNITS / GROUPS; u < (g + 1) * UNITS / GROUPS; ++u) decode_unit(raw_n, dn, u, step + 1);
            if (DEEP && g < XPT) fetch_x_one(step + LEAD, fill, g);
            __builtin_amdgcn_sched_barrier(0);
        }
        // refill the registers just decoded with the weights of step s+3 (in/out operands: the
        // loads cannot be scheduled above the decode that reads the registers)
#pragma unroll
        for (int kbo = 0; kbo < KBS; ++kbo) fetch_w(step + 3, raw_n, kbo);
        // A bare barrier (no fence): the only LDS writes are the direct loads, whose completion
        // the wait above covers.  Nothing may be scheduled across it.
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
    };
    u32x4 raw0[KBS][RT] = {}, raw1[KBS][RT] = {};      // packed weights of the even / of the odd steps
    Dec dec0, dec1;                                    // decoded operands of the even / of the odd steps
#pragma unroll
    for (int st = 0; st < LEAD; ++st) fetch_x(st, stage(st));
#pragma unroll
    for (int kbo = 0; kbo < KBS; ++kbo) fetch_w(0, raw0, kbo);
#pragma unroll
    for (int kbo = 0; kbo < KBS; ++kbo) fetch_w(1, raw1, kbo);
    wait_step(raw0, true);                 // everything landed (this wave's share of the stages too)
    wait_step(raw1, true);
#pragma unroll
    for (int u = 0; u < UNITS; ++u) decode_unit(raw0, dec0, u, 0);
#pragma unroll
    for (int kbo = 0; kbo < KBS; ++kbo) fetch_w(2, raw0, kbo);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    if (DEEP) {                            // the first fragments of stage 0
#pragma unroll
        for (int f = 0; f < RA; ++f) bq[f % (RA + 1)] = frag_of(stage(0), f);
    }

    // Every step is the same code, the last ones included: their refills are clamped re-reads
    // and their decodes operands that nobody uses, their barrier is harmless.
    for (int step = 0;; step += 2) {
        full_step(std::integral_constant<int, 0>{}, raw1, dec0, dec1, step);
        if (step + 1 >= n_steps) break;
        full_step(std::integral_constant<int, 1>{}, raw0, dec1, dec0, step + 1);
        if (step + 2 >= n_steps) break;
    }
    // No load of this wave is in flight past this point: the refills of the last steps still
    // write the (now dead) weight registers, so nothing may be scheduled above this wait that
    // could be given one of them.
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_waitcnt vmcnt(0) ; end of K loop" ::: "memory");     // (the comment is what the machine-code check looks for)
    __builtin_amdgcn_sched_barrier(0);

    // Draw this workgroup's next tile now (see tile_kernel): the counter's answer travels while
    // the epilogue computes, and is waited for before the epilogue's stores pile up behind it.
    int next_draw = 0;
    if (draw_ctr && tid == 0) next_draw = atomicAdd(draw_ctr, 1);

    // ---- epilogue: lane holds rows 4*(lane/16)..+3 of its row tile for token column lane%16 ----
    const int col = lane & 15, rsub = (lane >> 4) * 4;
    bool sat = false;
#pragma unroll
    for (int i = 0; i < NFR; ++i) {
        int within = i * 16 + col, slot;
        if (FUSED && i >= NFH) {
            within -= NFH * 16;
            if (within >= n_tok1) continue;
            slot = slot0 + n_tok + within;
        } else {
            if (within >= n_tok) continue;
            slot = slot0 + within;
        }
        if (STAGE == TSTAGE_GATEUP && HALF) {
            int grt = ntile * TG_WAVES + wave;
            if (grt >= row_tiles) continue;
            f32x4 g = acc[0][i], u = acc[1][i];
            u32x2 oh = {tg_swiglu_half2(g[0], u[0], g[1], u[1], sat), tg_swiglu_half2(g[2], u[2], g[3], u[3], sat)};
            if (!FUSED && a.h_frag) {
                // fragment order for the down stage: features grt*16 + rsub .. +3 of token `col` of
                // fragment i are elements rsub % 8 .. +3 of lane ((feature % 32) / 8) * 16 + col of
                // k-block feature / 32
                const int feat = grt * 16 + rsub;
                *(u32x2 *)(a.h_frag + ((int64_t)tg_frag_row(slot0, mt) + 16 * i) * a.rows + (feat >> 5) * 512 +
                           ((((feat & 31) >> 3) * 16 + col) * 8) + (feat & 7)) = oh;
            } else {
                *(u32x2 *)(a.h_out + (int64_t)(slot - a.h_slot_base) * a.rows + grt * 16 + rsub) = oh;
            }
        } else if (STAGE == TSTAGE_GATEUP) {
            int grt = ntile * TG_WAVES + wave;
            if (grt >= row_tiles) continue;
            f32x4 g = acc[0][i], u = acc[1][i];
            uint32_t hi01, lo01, hi23, lo23;
            tg_swiglu_split2(g[0], u[0], g[1], u[1], hi01, lo01);
            tg_swiglu_split2(g[2], u[2], g[3], u[3], hi23, lo23);
            u32x2 ohi = {hi01, hi23}, olo = {lo01, lo23};
            uint16_t *dst = a.h_out + (int64_t)(slot - a.h_slot_base) * a.rows + grt * 16 + rsub;
            *(u32x2 *)dst = ohi;
            *(u32x2 *)(dst + a.h_plane_stride) = olo;
        } else {
#pragma unroll
            for (int j = 0; j < RT; ++j) {
                int grt = ntile * TG_ROW_TILES + wave * RT + j;
                if (grt >= row_tiles) continue;
                // (half-precision weights were decoded times a power of two: undo it, which is exact)
                *(f32x4 *)(a.o_out + (int64_t)ks * a.o_ks_stride + (int64_t)slot * a.rows + grt * 16 + rsub) =
                    HALFW ? acc[j][i] * a.out_scale : acc[j][i];
            }
        }
    }
    if (STAGE == TSTAGE_GATEUP && HALF && a.h_saturated && __any(sat) && lane == 0) atomicAdd(a.h_saturated, 1);
    if (draw_ctr && tid == 0) *drawn = next_draw;
}

// One token tile x one block of weight rows, given its logical id (see tile_kernel for the order).
// Returns whether the tile ran (and, if asked to, drew the workgroup's next id into *drawn).
template <int STAGE, bool DENSE, bool ALLTOK, bool PERSIST, bool HALF>
__device__ __forceinline__ bool tile_run(const TgArgs &a, int logical, int n_mt, int gm_count, int per_ks,
                                         u32x4 *ring, int32_t *rowidx, int32_t *draw_ctr, int32_t *drawn)
{
    const int ks = logical / per_ks;
    logical -= ks * per_ks;
    const int bm = a.block_m, bn = TG_BLOCK_WGS / bm;
    const int blk = logical / TG_BLOCK_WGS, r = logical % TG_BLOCK_WGS;
    const int mt = (blk % gm_count) * bm + r % bm;
    const int ntile = (blk / gm_count) * bn + r / bm;
    if (mt >= n_mt || ntile >= a.n_ntiles) return false;

    int g, pos, slot0, n_tok, n_tok1 = 0;
    bool fused = false;
    if (ALLTOK) {
        g = mt / ((a.dense_tokens + a.dense_tile_tokens - 1) / a.dense_tile_tokens);
        int t_in = mt % ((a.dense_tokens + a.dense_tile_tokens - 1) / a.dense_tile_tokens);
        pos = 0;
        slot0 = a.dense_slot_base + g * a.dense_tokens + t_in * a.dense_tile_tokens;
        n_tok = min(a.dense_tile_tokens, a.dense_tokens - t_in * a.dense_tile_tokens);
    } else {
        int q = a.tile_q[mt];
        fused = (q & TILE_FUSED_FLAG) != 0;
        q &= ~TILE_FUSED_FLAG;
        g = q >> 1; pos = q & 1;
        if (g < a.group_lo || g >= a.group_hi) return false;  // another launch's kind of expert
        g -= a.group_lo;
        slot0 = a.tile_slot0[mt];
        n_tok = a.tile_n[mt];
        if (fused) { n_tok1 = n_tok >> 16; n_tok &= 0xFFFF; }
    }
    // these are the same for the whole workgroup; say so, or the per-fragment guards below become
    // exec-masked branches and the accumulators get shuffled between register files
    g = __builtin_amdgcn_readfirstlane(g);
    pos = __builtin_amdgcn_readfirstlane(pos);
    slot0 = __builtin_amdgcn_readfirstlane(slot0);
    n_tok = __builtin_amdgcn_readfirstlane(n_tok);
    n_tok1 = __builtin_amdgcn_readfirstlane(n_tok1);
    const uint16_t *wa = a.w_a[g];
    const uint16_t *wb = (STAGE == TSTAGE_GATEUP) ? a.w_b[g] : wa;
    const int frags = (n_tok + 15) >> 4;
    const int cnt = (frags + 1) >> 1;                        // 1..9 pairs of token fragments
    // (an odd number of fragments has its own loop from TG_ODD_MIN_CNT pairs on: smaller tiles are
    // not bound by their matrix instructions)
    const bool odd = (frags & 1) && cnt >= TG_ODD_MIN_CNT;
#define PZL_TILE(P, C) tile_body<STAGE, DENSE, ALLTOK, HALF, P, C>(a, wa, wb, slot0, n_tok, n_tok1, ntile, ks, mt, ring, rowidx, draw_ctr, drawn)
#define PZL_TILE_ODD(P, C) tile_body<STAGE, DENSE, ALLTOK, HALF, P, C, true>(a, wa, wb, slot0, n_tok, n_tok1, ntile, ks, mt, ring, rowidx, draw_ctr, drawn)
    // tiles that cover a pair, in either launch form (60 experts top-4, even router, 1024 tokens,
    // persistent launches: 282 -> 261 us; a skewed router has few such pairs and loses nothing)
    if constexpr (!DENSE && !ALLTOK) {
        if (__builtin_amdgcn_readfirstlane((int)fused)) {
            static_assert(TILE_FUSED_MAX_TOKENS <= 96, "a tile for both experts holds at most 3 pairs of fragments per expert");
            const int c2 = (max(n_tok, n_tok1) + 31) >> 5;       // 1..3 pairs of fragments per expert
            switch (c2) {
                case 1: PZL_TILE(2, 1); break; case 2: PZL_TILE(2, 2); break;
                default: PZL_TILE(2, 3); break;
            }
            return true;
        }
    }
#define PZL_TILE_CNT(P)                                                         \
    switch (cnt) {                                                              \
        case 1: PZL_TILE(P, 1); break; case 2: PZL_TILE(P, 2); break;           \
        case 3: PZL_TILE(P, 3); break; case 4: PZL_TILE(P, 4); break;           \
        case 5: PZL_TILE(P, 5); break; case 6: PZL_TILE(P, 6); break;           \
        case 7: PZL_TILE(P, 7); break; case 8: PZL_TILE(P, 8); break;           \
        default: PZL_TILE(P, 9); break;                                         \
    }
#define PZL_TILE_CNT_ODD(P)                                                     \
    switch (cnt) {                                                              \
        case 5: PZL_TILE_ODD(P, 5); break; case 6: PZL_TILE_ODD(P, 6); break;   \
        case 7: PZL_TILE_ODD(P, 7); break; case 8: PZL_TILE_ODD(P, 8); break;   \
        default: PZL_TILE_ODD(P, 9); break;                                     \
    }
    static_assert(TG_ODD_MIN_CNT == 5, "the switch above lists the odd tiles from 5 pairs of fragments on");
    if (odd) {
        if (DENSE || pos == 0) { PZL_TILE_CNT_ODD(0) } else { PZL_TILE_CNT_ODD(1) }
    } else {
        if (DENSE || pos == 0) { PZL_TILE_CNT(0) } else { PZL_TILE_CNT(1) }
    }
#undef PZL_TILE_CNT_ODD
#undef PZL_TILE_CNT
#undef PZL_TILE_ODD
#undef PZL_TILE
    return true;
}

template <int STAGE, bool DENSE, bool ALLTOK, bool PERSIST, bool HALF>
__global__ void __launch_bounds__(TG_THREADS) __attribute__((amdgpu_waves_per_eu(TG_WPE, TG_WPE)))
tile_kernel(TgArgs a)
{
    __shared__ u32x4 ring[tg_ring_stages<STAGE, HALF, DENSE>() * tg_stage_units<STAGE, HALF, DENSE>()];
    __shared__ int32_t rowidx[TG_MAX_TOK];
    __shared__ int32_t drawn;

    // XCD-aware order.  Consecutive workgroup ids go to different XCDs (8 of them, each with its
    // own L2), so give each XCD a contiguous range of logical ids.  The 32 workgroups an XCD runs
    // at a time form a block of 4 token tiles x 8 row tiles that march through K together: each
    // K slice of activations is shared by 8 of them and each slice of weights by 4, instead of
    // 32 workgroups streaming 32 different activation tiles through one L2.
    // The logical ids are laid out over the tiles that exist, so that every XCD gets the same
    // share of real work (laid out over the upper bound, some XCDs end a whole round of
    // workgroups short).
    // Routed experts: the number of tiles is only known on the device.  Where the upper bound is
    // close (few experts, many tokens each) the grid is the upper bound, one tile per workgroup.
    // Where it can be many times too large (many experts: one more tile per expert than the token
    // count alone would give; a launch of workgroups that find nothing to do still costs 5-10 us,
    // and tiles of very different sizes want to be handed out one by one) the launch is
    // persistent: one workgroup per compute unit, each working through its XCD's range of ids.
    // Shared experts: the host knows the tiles, one workgroup each.
    const int xcd = blockIdx.x % 8;
    const int n_mt = ALLTOK ? a.dense_tiles : min(*a.n_tiles, a.max_mtiles);
    const int block_n = TG_BLOCK_WGS / a.block_m;
    const int gm_count = (n_mt + a.block_m - 1) / a.block_m;
    const int gn_count = (a.n_ntiles + block_n - 1) / block_n;
    const int per_ks = gm_count * gn_count * TG_BLOCK_WGS;   // K splits are the slowest index
    const int total = per_ks * a.ksplit;
    const int per_xcd = (total + 7) / 8;
    // A persistent workgroup takes its first tiles by fixed stride (half of an even
    // share: the workgroups of an XCD then stay in step on one block of tiles) and draws the rest
    // from its XCD's counter, which evens out what tiles of different sizes left uneven.  A tile
    // draws its successor between its K loop and its epilogue, so that the counter's answer
    // travels while the epilogue computes.
    constexpr bool persistent = PERSIST;        // a template parameter: the one-shot kernel compiles without the loop
    const int wg = blockIdx.x / 8, wgs = gridDim.x / 8;
    const int fixed_rounds = per_xcd / wgs / 2;
    int32_t *ctr = persistent ? a.tile_ctr + xcd : nullptr;
    bool have_draw = false;
    for (int round = 0;; ++round) {
        int i;
        if (!persistent) {
            if (round > 0) return;
            i = wg;
        } else if (round < fixed_rounds) {
            // every wave is past the previous tile here (its loads have landed, its LDS reads
            // are done), so the next tile may overwrite the ring and the row indices
            __syncthreads();
            i = round * wgs + wg;
        } else {
            if (!have_draw && threadIdx.x == 0) drawn = atomicAdd(ctr, 1);
            __syncthreads();
            i = fixed_rounds * wgs + __builtin_amdgcn_readfirstlane(drawn);
        }
        if (i >= per_xcd || xcd * per_xcd + i >= total) return;
        // the tile after this one is drawn by this one unless it is a fixed one
        const bool draw = persistent && round + 1 >= fixed_rounds;
        have_draw = tile_run<STAGE, DENSE, ALLTOK, PERSIST, HALF>(a, xcd * per_xcd + i, n_mt, gm_count, per_ks, ring, rowidx,
                                                   draw ? ctr : nullptr, &drawn) && draw;
        if (persistent && !have_draw) __syncthreads();     // everyone has read `drawn` before it is written again
    }
}

template <int STAGE, bool DENSE, bool ALLTOK, bool HALF = false>
static int launch(const TileGemmArgs &t, hipStream_t st)
{
    if (t.max_mtiles <= 0) return PZL_OK;
    if (t.rows % TILE_ROWS || t.kdim % TILE_COLS) return PZL_EINVAL;
    // every K split must hold at least one k-block: the kernel clamps its read-ahead to the last
    // k-block of its share, which an empty share does not have
    if (STAGE == TSTAGE_DOWN && t.ksplit > t.kdim / TILE_COLS) return PZL_EINVAL;
    TgArgs a;
    a.w_a = t.w_a; a.w_b = t.w_b; a.rows = t.rows; a.kdim = t.kdim;
    a.act = t.act; a.act_plane_stride = t.act_plane_stride; a.act_is_x = t.act_is_x;
    a.act_slot_base = t.act_slot_base; a.slot_tok = t.slot_tok;
    a.tile_q = t.tile_q; a.tile_slot0 = t.tile_slot0; a.tile_n = t.tile_n; a.n_tiles = t.n_tiles;
    a.group_lo = t.group_lo; a.group_hi = t.group_hi;
    a.dense_tokens = t.dense_tokens; a.dense_slot_base = t.dense_slot_base;
    a.dense_tiles = t.dense_tiles; a.dense_tile_tokens = t.dense_tile_tokens;
    a.h_out = t.h_out; a.h_plane_stride = t.h_plane_stride; a.h_slot_base = t.h_slot_base;
    a.act_frag = (!DENSE && HALF) ? t.act_frag : nullptr;
    a.h_frag = (!DENSE && HALF && STAGE == TSTAGE_GATEUP) ? t.h_frag : nullptr;
    a.o_out = t.o_out; a.o_ks_stride = t.o_ks_stride;
    a.ksplit = (STAGE == TSTAGE_DOWN && t.ksplit > 1) ? t.ksplit : 1;
    a.max_mtiles = t.max_mtiles;
    const int rows_per_wg = (STAGE == TSTAGE_GATEUP) ? TILE_WG_FEATURES : TILE_WG_DOWN_ROWS;
    a.n_ntiles = (t.rows + rows_per_wg - 1) / rows_per_wg;
    // Blocks of 8 token tiles x 4 row blocks, or of 4 x 8 where the caller expects about four token
    // tiles per expert (the tiles of one expert are of one size and keep step; measured, 8 experts of
    // about 1024 tokens: -3 %; with 8 tiles per expert +1 %) and the row blocks divide by 8 (laid out
    // over a count that does not, the XCDs get uneven shares: 11 row blocks, +17 %).
    a.block_m = (t.block_m == 4 && a.n_ntiles % 8 == 0) ? 4 : 8;
    const int block_n = TG_BLOCK_WGS / a.block_m;
    int64_t blocks = (int64_t)((a.max_mtiles + a.block_m - 1) / a.block_m) *
                     ((a.n_ntiles + block_n - 1) / block_n) * TG_BLOCK_WGS;
    blocks = (blocks + 7) / 8 * 8 * a.ksplit;
    if (blocks > 0x7FFFFFFFLL) return PZL_EINVAL;
    a.tile_ctr = nullptr;
    if (!ALLTOK && t.tile_ctr) {                  // persistent: one workgroup per compute unit, tiles are drawn
        a.tile_ctr = t.tile_ctr;
        if (blocks > TG_PERSISTENT_WGS) blocks = TG_PERSISTENT_WGS;
    }
    a.h_saturated = t.h_saturated;
    a.out_scale = 0.5f; a.dense_clamp2 = 0; a.dense_bias2 = 0;
    if (DENSE && HALF) {
        const int B = t.dense_half_bias;
        if (B < 0 || B > 224) return PZL_EINVAL;
        a.out_scale = ldexpf(1.0f, B - 112);
        a.dense_clamp2 = ((uint32_t)B << 7) * 0x00010001u;
        a.dense_bias2 = (((uint32_t)B << 10) & 0xFFFFu) * 0x00010001u;
    }
    if (a.tile_ctr) hipLaunchKernelGGL((tile_kernel<STAGE, DENSE, ALLTOK, !ALLTOK, HALF>), dim3((unsigned)blocks), dim3(TG_THREADS), 0, st, a);
    else            hipLaunchKernelGGL((tile_kernel<STAGE, DENSE, ALLTOK, false, HALF>), dim3((unsigned)blocks), dim3(TG_THREADS), 0, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_hip_error(e); return PZL_EHIP; }
    return PZL_OK;
}

// x in fragment order for the tiles of the list: one workgroup per (tile, token fragment), a wave
// per k-block in turn; every lane moves the 16 bytes that the tile's gate/up stage will want in
// its place (columns past the tile's last token repeat that token, as the kernel's own gather does).
__global__ void __launch_bounds__(256)
gather_x_kernel(const uint16_t *__restrict__ x, int32_t d, const int32_t *__restrict__ slot_tok,
                const int32_t *__restrict__ tile_q, const int32_t *__restrict__ tile_slot0,
                const int32_t *__restrict__ tile_n, const int32_t *__restrict__ n_tiles, uint16_t *__restrict__ x_frag)
{
    const int mt = blockIdx.x / TG_FRAGS, fr = blockIdx.x % TG_FRAGS;   // blockIdx.y: a quarter of the k-blocks (more loads in flight per compute unit)
    if (mt >= *n_tiles) return;
    if (tile_q[mt] & TILE_FUSED_FLAG) return;                  // such tiles read x itself
    const int n = tile_n[mt], slot0 = tile_slot0[mt];
    const int nfrag = 2 * ((((n + 15) >> 4) + 1) >> 1);        // fragments come in pairs
    if (fr >= nfrag) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row = slot_tok[slot0 + min(fr * 16 + (lane & 15), n - 1)];
    const u32x4 *src = (const u32x4 *)(x + (int64_t)row * d + (lane >> 4) * 8);
    u32x4 *dst = (u32x4 *)(x_frag + ((int64_t)tg_frag_row(slot0, mt) + 16 * fr) * d) + lane;
    const int kbs = d / TILE_COLS, per = (kbs + (int)gridDim.y - 1) / (int)gridDim.y;
    const int kb_end = min(kbs, ((int)blockIdx.y + 1) * per);
    for (int kb = (int)blockIdx.y * per + wave; kb < kb_end; kb += 4) dst[kb * 64] = src[kb * (TILE_COLS / 8)];
}

int launch_gather_x(const uint16_t *x, int32_t d, const int32_t *slot_tok, const int32_t *tile_q, const int32_t *tile_slot0,
                    const int32_t *tile_n, const int32_t *n_tiles, int32_t max_mtiles, uint16_t *x_frag, hipStream_t st)
{
    if (max_mtiles <= 0) return PZL_OK;
    if (d % TILE_COLS) return PZL_EINVAL;
    hipLaunchKernelGGL(gather_x_kernel, dim3((unsigned)max_mtiles * TG_FRAGS, 4), dim3(256), 0, st, x, d, slot_tok, tile_q, tile_slot0,
                       tile_n, n_tiles, x_frag);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_hip_error(e); return PZL_EHIP; }
    return PZL_OK;
}

// kind: 0 = packed pairs (routed), 1 = dense experts that see every token (shared),
//       2 = dense routed experts (kept unmerged)
int launch_tile_gateup(const TileGemmArgs &a, int kind, hipStream_t st)
{
    if (kind == 0 && a.half_h) return launch<TSTAGE_GATEUP, false, false, true>(a, st);
    if (kind == 0) return launch<TSTAGE_GATEUP, false, false>(a, st);
    if (kind == 1 && a.half_h) return launch<TSTAGE_GATEUP, true, true, true>(a, st);
    if (kind == 1) return launch<TSTAGE_GATEUP, true, true>(a, st);
    return launch<TSTAGE_GATEUP, true, false>(a, st);
}

int launch_tile_down(const TileGemmArgs &a, int kind, hipStream_t st)
{
    if (kind == 0 && a.half_h) return launch<TSTAGE_DOWN, false, false, true>(a, st);
    if (kind == 0) return launch<TSTAGE_DOWN, false, false>(a, st);
    if (kind == 1 && a.half_h) return launch<TSTAGE_DOWN, true, true, true>(a, st);
    if (kind == 1) return launch<TSTAGE_DOWN, true, true>(a, st);
    return launch<TSTAGE_DOWN, true, false>(a, st);
}

}  // namespace pzl

