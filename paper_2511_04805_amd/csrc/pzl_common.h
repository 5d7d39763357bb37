// Internal declarations shared by the library's HIP translation units (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/puzzle_moe.h"

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x2 __attribute__((ext_vector_type(2)));

namespace pzl {

// 16x32 tiled order: one tile is 512 elements = 64 lanes x 8 elements; lane = (c%32)/8*16 + r%16.
constexpr int TILE_ROWS = 16;
constexpr int TILE_COLS = 32;
constexpr int TILE_ELEMS = TILE_ROWS * TILE_COLS;

// Routing tables in the workspace (all int32).  Experts are renumbered q = 2*pair + pos so
// that the two experts of a pair own adjacent slot ranges.
struct RouteTables {
    int32_t *cnt;        // [Q]    tokens routed to expert q that the streaming kernels handle (0 if the expert is tiled)
    int32_t *off;        // [Q+1]  first slot of expert q
    int32_t *slot_tok;   // [N]    token index of each slot (slots grouped by q; order inside a group is arbitrary)
    int32_t *slot_of;    // [N]    slot of flat index t*k+j, or -1 for an id outside [0,E)
    // token tiles of the tiled GEMM path: each expert's slots cut into equal parts of <= TILE_MAX_TOKENS
    int32_t *tile_q;     // [max_tiles] expert q of the tile
    int32_t *tile_slot0; // [max_tiles] first slot
    int32_t *tile_n;     // [max_tiles] tokens in the tile
    int32_t *n_tiles;    // [64]: [0] number of tiles; [8..39] work counters of the tiled launches, zeroed by the grouping kernel
};
constexpr int TILE_MAX_TOKENS = 288;
// A pair both of whose experts have between 1 and TILE_FUSED_MAX_TOKENS tokens gets ONE tile that
// covers both (tile_q = 2*pair | TILE_FUSED_FLAG, tile_slot0 = first slot of the pair,
// tile_n = n0 | n1 << 16; the two experts' slots are adjacent): the packed weights are then read
// once for both, as in the streaming kernels, instead of once per expert.
constexpr int TILE_FUSED_FLAG = 1 << 30;
#ifndef PZL_FUSED_MAX
#define PZL_FUSED_MAX 96
#endif
constexpr int TILE_FUSED_MAX_TOKENS = PZL_FUSED_MAX;
constexpr int TILE_HALF_TOKENS = TILE_MAX_TOKENS / 2;   // tile size of launches that would not fill the chip once
inline int max_token_tiles(int64_t n_flat, int n_experts) { return (int)(n_flat / TILE_MAX_TOKENS) + n_experts; }

void set_hip_error(hipError_t e);

// codec.hip
int launch_pack(const uint16_t *merged, const uint8_t *m0, const uint8_t *m1, const uint8_t *s0,
                const uint8_t *s1, int64_t rows, int64_t cols, uint16_t *out, int32_t *n_bad,
                hipStream_t st);
int launch_unpack(const uint16_t *packed, int pos, int64_t rows, int64_t cols, uint16_t *out, bool half_x2,
                  hipStream_t st);
int launch_tile_dense(const uint16_t *in, int64_t rows, int64_t cols, uint16_t *out, hipStream_t st);
int launch_merge_pack(const uint16_t *wi, const uint16_t *wj, const float *norm_i, const float *norm_j,
                      int64_t rows, int64_t cols, float tau, uint16_t *out, int32_t *n_similar,
                      int32_t *n_bad, hipStream_t st);

int launch_max_exp_bf16(const uint16_t *w, int64_t n_elems, int32_t *max_out, hipStream_t st);   // atomicMax of the bf16 exponent fields of the non-zero elements
int launch_max_exp_field(const uint16_t *packed, int64_t rows, int64_t cols, int32_t *max_out, hipStream_t st);

// quant_codec.hip
size_t q_record_bytes(int64_t rows, int64_t cols);
size_t q_scale_bytes(int64_t rows, int64_t cols);
int launch_q_pack(const uint16_t *merged, const uint8_t *m0, const uint8_t *m1, const uint8_t *s0,
                  const uint8_t *s1, int64_t rows, int64_t cols, uint8_t *records, uint16_t *scales,
                  int32_t *n_bad, hipStream_t st);
int launch_q_unpack(const uint8_t *records, const uint16_t *scales, int pos, int64_t rows, int64_t cols,
                    float *out, hipStream_t st);

// route.hip
// tile_min: a pair one of whose experts has at least that many tokens gets token tiles (tiled
// kernels) and counts as empty for the streaming kernels; the other pairs the other way round.
// row_groups: workgroups per token tile in the gate/up stage (decides whether pairs share tiles;
// 0: never)
int launch_route(const int32_t *ids, int32_t n_flat, int32_t k, int32_t n_experts, int32_t n_slots_q, const int32_t *q_of_expert,
                 RouteTables rt, int32_t tile_min, int32_t row_groups, int32_t launch_rows, hipStream_t st);
int prepare_route_kernel();   // per-device kernel attribute; called at layer creation and (cheaply) by launch_route
int launch_router_topk(const uint16_t *x, const uint16_t *w_router, int32_t T, int32_t d, int32_t E, int32_t k,
                       int32_t *ids_out, float *w_out, hipStream_t st);
int launch_combine(const float *opart, int32_t ksplit, int32_t ksplit_shared, int64_t ks_stride, const RouteTables &rt,
                   const float *topk_w, int32_t T, int32_t k, int32_t d, int32_t n_shared,
                   uint16_t *y, hipStream_t st);

// stream_gemm.hip: weight-streaming decode-GEMM for small token counts per pair.
struct StreamGroupArgs {
    const uint16_t *const *w_a;   // device array [n_groups]: gate (gate/up stage) or down (down stage)
    const uint16_t *const *w_b;   // device array [n_groups]: up, or nullptr in the down stage
    const uint16_t *const *s_a;   // quantised pairs only: the scale arrays of w_a / w_b
    const uint16_t *const *s_b;
    int32_t n_groups;
    int32_t groups_touched_max;   // upper bound on groups that can have tokens (0 = all)
    int32_t rows;                 // output features of the stage (f or d)
    int32_t kdim;                 // contracted dimension (d or f)
    const uint16_t *act;          // activations [*, kdim] bf16 row-major (x, or the hi plane of H)
    int64_t act_plane_stride;     // down stage: elements from the hi plane of H to its lo plane
    int32_t act_is_x;             // 1: row = slot_tok[slot] (or the token itself if dense); 0: row = slot - act_slot_base
    int32_t act_slot_base;
    const int32_t *cnt;           // routed: RouteTables.cnt, dense: nullptr
    int32_t group_base;           // routed: index of the first group (q = 2 * (group_base + g) + pos)
    const int32_t *off;
    const int32_t *slot_tok;
    int32_t dense_tokens;         // dense groups: every group sees tokens 0..dense_tokens-1
    int32_t dense_slot_base;      // dense groups: slot of (group g, token t) = base + g*dense_tokens + t
    uint16_t *h_out;              // gate/up stage: H hi plane [slots, rows] bf16, row index = slot - h_slot_base
    int64_t h_plane_stride;       // elements from the hi plane to the lo plane
    int32_t h_slot_base;
    float *o_out;                 // down stage: partial sums [ksplit][slots][rows] fp32
    int64_t o_ks_stride;          // elements between k-splits
    int32_t ksplit;
    int32_t pass_wgs;             // routed groups: workgroups that share a group's token passes (0 = 1)
    int32_t half_h;               // packed pairs only: H is one half-precision plane (see stream_gemm.hip)
    int32_t *h_saturated;         // ... and this device counter is bumped when a value of H saturates (may be null)
    // Gate/up launch of packed pairs in a small batch: the kernel groups the (token, choice) list
    // itself and writes cnt / off / slot_tok (above) and slot_of for the kernels that follow; no
    // grouping kernel runs before it.  route_ids == nullptr: the tables were written beforehand.
    const int32_t *route_ids, *route_q_of_expert;
    int32_t route_n_flat, route_k, route_n_experts, route_n_keys;
    int32_t *route_slot_of;
};
constexpr int STREAM_FUSED_ROUTE_MAX_FLAT = 512;   // (token, choice) entries the gate/up kernel can group by itself
constexpr int STREAM_FUSED_ROUTE_MAX_KEYS = 128;   // ... and routing keys
int stream_row_groups(int rows, bool down_stage);   // row groups (workgroup units) along the output rows
#ifndef SG_WAVES_N
#define SG_WAVES_N 8
#endif
constexpr int STREAM_RESIDENT_WGS = 2048 / SG_WAVES_N;             // workgroups the chip holds at once (256 CUs x 2)
// kind: 0 packed pairs, 1 dense experts seeing every token (shared), 2 dense routed experts
constexpr int KIND_PACKED = 0, KIND_SHARED = 1, KIND_UNMERGED = 2, KIND_QUANT = 3;
int launch_stream_gateup(const StreamGroupArgs &a, int kind, hipStream_t st);
// Sets the dynamic-LDS attribute of every streaming kernel for the current device (not a stream
// operation; the launches would otherwise do it on their first call per device).
int prepare_stream_kernels();
int launch_stream_down(const StreamGroupArgs &a, int kind, hipStream_t st);

// tile_gemm.hip: LDS-staged decode-GEMM on the matrix cores for large token counts per expert.
#ifndef TG_WAVES_N
#define TG_WAVES_N 8
#endif
constexpr int TILE_WG_FEATURES = TG_WAVES_N * 16;    // gate/up stage: features (rows of gate and of up) per workgroup
constexpr int TILE_WG_DOWN_ROWS = TG_WAVES_N * 32;   // down stage: weight rows per workgroup
constexpr int TILE_WGS_PER_CU = 8 / TG_WAVES_N;      // workgroups a compute unit holds (8 waves)
struct TileGemmArgs {
    const uint16_t *const *w_a;   // device array: gate (gate/up stage) or down (down stage)
    const uint16_t *const *w_b;   // device array: up, or nullptr
    int32_t rows, kdim;
    const uint16_t *act;          // x, or the hi plane of H
    int64_t act_plane_stride;
    int32_t act_is_x, act_slot_base;
    const int32_t *slot_tok;
    const int32_t *tile_q, *tile_slot0, *tile_n, *n_tiles;   // routed groups: RouteTables tile list
    int32_t group_lo, group_hi;                              // routed: groups [lo, hi) belong to this launch
    int32_t dense_tokens, dense_slot_base, dense_tiles, dense_tile_tokens;   // dense group: uniform tiles
    uint16_t *h_out;
    int64_t h_plane_stride;
    int32_t h_slot_base;
    float *o_out;                 // down stage: [ksplit][slots][rows] fp32
    int64_t o_ks_stride;
    int32_t ksplit;               // down stage only: workgroups sharing one output tile along K
    int32_t max_mtiles;           // upper bound on token tiles (grid size)
    int32_t block_m;              // 4: about four token tiles per expert are expected (see launch() in tile_gemm.hip); else 0
    // packed pairs with half-precision H only: fragment-ordered buffers (tile_gemm.hip, tg_frag_row), or null
    const uint16_t *act_frag;     // this stage's token operand in fragment order (x gathered by launch_gather_x; H written by the gate/up stage)
    uint16_t *h_frag;             // gate/up stage: where H goes in fragment order
    int32_t *tile_ctr;            // routed groups: 8 zeroed counters (one per XCD) for a persistent launch that draws its tiles, or nullptr
    int32_t half_h;               // H is one half-precision plane (packed pairs; shared experts with dense_half_bias >= 0)
    int32_t dense_half_bias;      // dense weights of a half_h launch: largest exponent field of the down matrices - 30, at least 0
    int32_t *h_saturated;         // ... and this device counter is bumped when a value of H saturates (may be null)
};
// rows that a fragment-ordered buffer holds per tile of the tile list's bound, beyond the slots
constexpr int TILE_FRAG_PAD_ROWS = 32;
inline size_t tile_frag_rows(int64_t n_flat, int n_keys) { return (size_t)n_flat + (size_t)TILE_FRAG_PAD_ROWS * ((size_t)max_token_tiles(n_flat, n_keys) + 1); }
// x in fragment order for the token tiles of the list (tiles that cover a pair are left out)
int launch_gather_x(const uint16_t *x, int32_t d, const int32_t *slot_tok, const int32_t *tile_q, const int32_t *tile_slot0,
                    const int32_t *tile_n, const int32_t *n_tiles, int32_t max_mtiles, uint16_t *x_frag, hipStream_t st);
int launch_tile_gateup(const TileGemmArgs &a, int kind, hipStream_t st);
int launch_tile_down(const TileGemmArgs &a, int kind, hipStream_t st);

}  // namespace pzl
