// C ABI of the library (see include/puzzle_moe.h): argument checks, the layer object, workspace
// carving and the launch sequence of pzl_moe_ffn.  No kernel lives here.
#include "pzl_common.h"

#include <algorithm>
#include <mutex>
#include <new>
#include <string.h>
#include <vector>

// Scratch memory of pzl_moe_ffn_static, the entry point for callers that cannot allocate: one
// array per GPU, part of the loaded code object, held until the process ends.  In host code the
// name below is only a handle for hipGetSymbolAddress: the device address is looked up once per
// device (static_scratch_of) and that pointer is what kernels and copies get.
static __device__ __align__(256) unsigned char scratch[PZL_STATIC_SCRATCH_BYTES];

namespace pzl {

static thread_local char g_hip_error[256] = "no HIP error recorded";

void set_hip_error(hipError_t e)
{
    const char *s = hipGetErrorString(e);
    strncpy(g_hip_error, s ? s : "unknown HIP error", sizeof(g_hip_error) - 1);
    g_hip_error[sizeof(g_hip_error) - 1] = 0;
}

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Device address of this GPU's copy of `scratch`; looked up on the first call per device (with
// that device current) and kept.  Returns nullptr (and records the HIP error) on failure.
static void *static_scratch_of_current_device()
{
    static std::mutex mu;
    static void *ptr_of[64] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= 64) { set_hip_error(e != hipSuccess ? e : hipErrorInvalidDevice); return nullptr; }
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr_of[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) { set_hip_error(e != hipSuccess ? e : hipErrorInvalidSymbol); return nullptr; }
        ptr_of[dev] = p;
    }
    return ptr_of[dev];
}

}  // namespace pzl

struct pzl_layer {
    int32_t n_experts, n_pairs, n_dense, d_model, d_ffn, n_shared;
    int32_t n_q;                           // routing keys: 2 per pair, then 2 per unmerged expert (its position 1 stays empty)
    std::vector<int32_t> shared_f;
    // device tables
    int32_t *d_q_of_expert;                // [E] expert -> 2*pair + pos
    const uint16_t **d_gate, **d_up, **d_down;            // [P]
    int32_t pair_format;                   // 0: 16-bit packed words, 1: quantised records
    const uint16_t **d_gscale, **d_uscale, **d_dscale;    // [P] scale arrays (quantised format)
    const uint16_t **d_dgate, **d_dup, **d_ddown;         // [n_dense] routed experts kept unmerged
    const uint16_t **d_sgate, **d_sup, **d_sdown;         // [n_shared]
    void *d_block;                         // the one allocation holding all of the above
    // Shared experts do not depend on the routing: they run on a second stream next to the routed
    // kernels (fork after the caller's stream reaches the call, join before the combine).
    hipStream_t aux_stream;            // shared experts
    hipEvent_t ev_fork, ev_join;
    hipStream_t tile_stream;           // tiled kernels of the routed experts, next to the streaming ones
    hipEvent_t ev_tfork, ev_tjoin;
    void *static_scratch;              // this device's copy of the library's static scratch array (pzl_moe_ffn_static)
    // Form of the SwiGLU output H of the packed pairs (stream_gemm.hip): one half-precision plane if
    // no down matrix holds an exponent field above 29 (and the caller did not ask for the wide
    // form), else two bf16 planes.  Unmerged, shared and quantised experts always use two planes.
    bool half_h;
    std::vector<int> shared_max_exp;   // per shared expert: largest bf16 exponent field of its down matrix, or -1 (keep H wide)
    int32_t *d_counters;               // [0] largest exponent field of the down matrices, [1] waves that saturated a value of H
    // pzl_layer_force_plan: -1 leaves the decision to make_plan, 0 / 1 overrides it (measurement only)
    int32_t force_hybrid = -1, force_persistent = -1, force_tile_stream = -1;
};

namespace pzl {

#ifndef PZL_TILED_MIN_TPE
#define PZL_TILED_MIN_TPE 96
#endif
#ifndef PZL_TILED_MIN_SHARED
#define PZL_TILED_MIN_SHARED 65
#endif
#ifndef PZL_SHARED_TILE_WGS
#define PZL_SHARED_TILE_WGS 168
#endif
#ifndef PZL_SHARED_TILE_MIN_TOKENS
#define PZL_SHARED_TILE_MIN_TOKENS 48
#endif
#ifndef PZL_SHARED_TILE_MIN_TOKENS_IDLE
#define PZL_SHARED_TILE_MIN_TOKENS_IDLE 36
#endif
constexpr int TILED_MIN_TOKENS_PER_EXPERT = PZL_TILED_MIN_TPE;   // average tokens per expert from which the K split is sized for the tiled kernels
#ifndef PZL_HYBRID_MIN_TPE
#define PZL_HYBRID_MIN_TPE 20
#endif
#ifndef PZL_HYBRID_MIN_TPE_MANY
#define PZL_HYBRID_MIN_TPE_MANY 6
#endif
#ifndef PZL_HYBRID_TILE_MIN
#define PZL_HYBRID_TILE_MIN 33
#endif
constexpr int HYBRID_MIN_TOKENS_PER_EXPERT = PZL_HYBRID_MIN_TPE;  // average from which both paths are launched
constexpr int HYBRID_MIN_TOKENS_PER_EXPERT_MANY = PZL_HYBRID_MIN_TPE_MANY;   // ... in a layer with 32 experts or more
constexpr int HYBRID_TILE_MIN_TOKENS = PZL_HYBRID_TILE_MIN;       // ... and a pair with an expert of this many tokens is tiled
// a dense expert sees every token: beyond one 64-token sweep of its weights the tiled kernels win,
// given token tiles of the right size (shared_token_parts).  Measured, 60 experts + 1 shared
// expert of 5632: 64 tokens 120 us streamed / 135 tiled, 96 tokens 156 / 139, 256 tokens 192 / 166
constexpr int TILED_MIN_TOKENS_SHARED = PZL_TILED_MIN_SHARED;
constexpr int QUANT_MAX_SLOTS_PER_EXPERT = 64;   // quantised layers: largest average of (token, choice) entries per expert that a call accepts
constexpr int FRAG_X_MIN_FFN = 8192;   // expert width from which x is gathered into fragment order for the tiled gate/up stage
constexpr int MAX_KSPLIT = 8;   // upper bound on the k-splits of the down stage (sizes the workspace)

struct WorkspaceLayout {
    size_t cnt, off, slot_tok, slot_of, tile_q, tile_slot0, tile_n, n_tiles, h_routed, h_frag, x_frag, h_shared, opart, total;
    bool has_h_frag, has_x_frag;   // fragment-ordered copies of H and of x for the tiled kernels (tile_gemm.hip, tg_frag_row)
    int64_t o_ks_stride;      // elements between k-splits of the partial-sum buffer
    // H is held as two bf16 planes (hi, lo), the lo plane right after the hi plane
    size_t h_shared_each(const pzl_layer *L, int32_t T, int s) const
    {
        return align_up((size_t)2 * T * L->shared_f[s] * 2, 256);
    }
};

// Tiled down stage: workgroups = token tiles x rows/256, one per compute unit at a time.  Splitting
// K over `ks` workgroups fills idle compute units when there are few tiles, but every split writes
// its own fp32 partial sums, which the combine step then reads back.  Pick the split with the
// lowest estimated time: rounds of 256 workgroups (at least one) x (K steps x time per step +
// fixed cost per tile) + traffic of the partial sums.  In effect: split only until the launch
// fills the chip once (measured on the Mixtral-shaped layer at 1024-8192 tokens, every further
// split lost 3-10 %).  Constants: 1.8 us per K step for a full 288-token tile, about half of
// that for a nearly empty one, 10 us of prologue and epilogue, 5 TB/s for the partial sums; only
// their ratios matter.
static int choose_tile_ksplit(int64_t token_tiles, int64_t slots, int rows, int kdim, int min_steps = 8)
{
    if (token_tiles < 1) token_tiles = 1;
    const double wgs = (double)token_tiles * ((rows + TILE_WG_DOWN_ROWS - 1) / TILE_WG_DOWN_ROWS) / TILE_WGS_PER_CU;
    const double steps = kdim / TILE_COLS;
    double fill = (double)slots / ((double)token_tiles * TILE_MAX_TOKENS);
    if (fill > 1.0) fill = 1.0;
    const double us_per_step = 1.8 * (0.5 + 0.5 * fill);
    const double us_partials = (double)slots * rows * 8.0 / 5.0e6;      // written once, read once
    int best = 1;
    double best_us = 0.0;
    for (int ks = 1; ks <= MAX_KSPLIT; ++ks) {
        if (ks > 1 && steps / ks < (double)min_steps) break;
        double rounds = wgs * ks / 256.0;          // workgroups are handed out as compute units free up:
        if (rounds < 1.0) rounds = 1.0;            // measured, whole rounds are not the right granularity
        const double us = rounds * (steps / ks * us_per_step + 10.0) + ks * us_partials;
        if (ks == 1 || us < best_us) { best_us = us; best = ks; }
    }
    return best;
}

// Token tiles per shared expert in the tiled kernels (`n_same` experts of width f share a launch).
// The largest tiles (288 tokens) do the least work per token, but a shared expert has few row
// tiles, and a few large tiles are then the longest-running workgroups of the step while compute
// units idle.  So the tokens are cut into more, smaller tiles (48 tokens at least) until the
// gate/up launch has about `target_wgs` workgroups (the down launch splits K to match); the
// caller sets the target by what runs next to the shared experts (shared_target_wgs).
// Measured, 60 experts top-4 + 1 shared expert of 5632 (44 workgroups per token tile), whole step
// in us by tokens per tile: 128 tokens: 128 -> 168, 64 -> 155; 256 tokens: 288 -> 207, 128 -> 174,
// 64 -> 166; 512 tokens: 288 -> 271, 192 -> 252, 128 -> 237, 96 -> 267, 64 -> 254; 768 tokens:
// 288 -> 291, 192 -> 273, 128 -> 303; from 1024 tokens 288 is best (176 workgroups or more).
// 64 experts top-6 + 2 shared experts of 1408 (22 per token tile): within 2 % from 64 to 288.
static int shared_token_parts(int32_t T, int n_same, int f, int target_wgs, bool chip_busy)
{
    int parts = (T + TILE_MAX_TOKENS - 1) / TILE_MAX_TOKENS;
    const int per_part = n_same * ((f + TILE_WG_FEATURES - 1) / TILE_WG_FEATURES) / TILE_WGS_PER_CU;   // gate/up workgroups (in units of a compute unit's share) per token tile
    int want = (target_wgs + per_part / 2) / per_part;
    // at least 48 tokens per tile; 36 (rounded up to 48 by the fragment size) next to routed
    // kernels that leave compute units idle, which lets 72-95 tokens be two tiles (60 experts +
    // 1 shared expert, 72 / 80 / 88 tokens: 147 / 149 / 153 -> 141 / 142 / 142 us)
    const int most = T / (chip_busy ? PZL_SHARED_TILE_MIN_TOKENS : PZL_SHARED_TILE_MIN_TOKENS_IDLE);
    if (want > most) want = most;
    return want > parts ? want : parts;
}

// Workgroups that the shared experts' gate/up launch should have.  Next to routed kernels that
// leave compute units idle (streaming launches, short one-shot tile lists): two thirds of the
// chip.  Next to persistent tiled launches, which occupy every compute unit: in proportion to the
// shared experts' part of the step's matrix work, with the same allowance (a shared expert as
// heavy as the routed top-k gets two thirds, two narrow ones next to top-6 get a third).
static int shared_target_wgs(const pzl_layer *L, int32_t k, bool chip_busy)
{
    if (!chip_busy) return PZL_SHARED_TILE_WGS;
    double fs = 0.0;
    for (int s = 0; s < L->n_shared; ++s) fs += L->shared_f[s];
    const double share = fs / (fs + (double)k * L->d_ffn);
    return (int)(2.0 * PZL_SHARED_TILE_WGS * share);
}

// Workgroups per routed group and row block in the streaming kernels.  A sweep of a pair's
// weights serves 32 tokens per expert (64 for an expert kept unmerged); an expert with more takes
// further sweeps.  Where the tiled kernels are launched too, such pairs are theirs and one
// workgroup is enough.  Otherwise (small batches) a router that favours some experts can still
// hand one of them up to T tokens, and its pair's workgroups would run two or three sweeps in a
// row while the rest of the chip has finished: give every group that many workgroups, each taking
// every n-th sweep; those that find no sweep to do leave at once.
#ifndef PZL_STREAM_PASS_WGS_MAX
#define PZL_STREAM_PASS_WGS_MAX 3
#endif
static int stream_pass_wgs(int32_t T, int kind, int tile_min)
{
    const int most = T < tile_min - 1 ? T : tile_min - 1;      // tokens of one expert that can come to the streaming kernels
    const int per_sweep = kind == KIND_UNMERGED ? 64 : 32;
    const int n = (most + per_sweep - 1) / per_sweep;
    return n < 1 ? 1 : n > PZL_STREAM_PASS_WGS_MAX ? PZL_STREAM_PASS_WGS_MAX : n;
}

static int choose_ksplit(int groups_touched_max, int rows)
{
    // The down projection has only rows/128 workgroups per pair; split its long K so that the
    // launch fills the chip once (about one resident round of workgroups).
    int64_t wgs = (int64_t)groups_touched_max * stream_row_groups(rows, true);
    int ks = (int)(STREAM_RESIDENT_WGS / (wgs > 0 ? wgs : 1));
    if (ks < 1) ks = 1;
    if (ks > MAX_KSPLIT) ks = MAX_KSPLIT;
    return ks;
}

// The host-side decisions of one pzl_moe_ffn call; they depend on the layer's shape and on the
// batch shape only (the routing is known to the device alone).  The reasons and the measurements
// behind each rule stand where pzl_moe_ffn uses it.
struct Plan {
    bool overlap;          // shared experts on the layer's second stream
    bool hybrid;           // tiled kernels launched next to the streaming ones; the grouping kernel picks per pair
    bool mostly_tiled;     // the K split of the routed down stage is sized for the tiled kernels
    bool tiled_shared;     // shared experts on the tiled kernels
    bool persistent;       // tiled launches of the routed experts draw their tiles
    bool tile_overlap;     // ... and run on the layer's third stream
    int tile_min;          // tokens of an expert from which its pair is tiled
    int ksplit, ksplit_shared;
    int shared_wgs;        // workgroups aimed at for the shared experts' tiled gate/up launch
    bool fused_route;      // no grouping kernel: the streaming gate/up kernel of the packed pairs groups the list itself
    int tiles_per_expert;  // token tiles of an expert with the average number of tokens
    bool frag_h, frag_x;   // the tiled kernels of the packed pairs keep H / read x in fragment order
};

static Plan make_plan(const pzl_layer *L, int32_t T, int32_t k, bool staged)
{
    Plan pl;
    const int64_t N = (int64_t)T * k;
    const int64_t E64 = L->n_experts;
    pl.overlap = L->n_shared > 0 && !staged && N > 0;
    pl.hybrid = L->pair_format == 0 &&
        N >= (int64_t)(E64 >= 32 ? HYBRID_MIN_TOKENS_PER_EXPERT_MANY : HYBRID_MIN_TOKENS_PER_EXPERT) * E64;
    if (L->force_hybrid >= 0 && L->pair_format == 0) pl.hybrid = L->force_hybrid != 0;
    pl.tile_min = pl.hybrid ? HYBRID_TILE_MIN_TOKENS : 0x7FFFFFFF;
    pl.tiles_per_expert = (int)((N / E64 + TILE_MAX_TOKENS - 1) / TILE_MAX_TOKENS);
    // Fragment-ordered H costs nothing (the gate/up stage stores it there instead); fragment-ordered
    // x costs a pass that reads and writes N x d elements in front of a gate/up stage that gets
    // about 3 % shorter: by the two kernels' rates that pays from f of about 7000 on, in batches
    // where the tiled kernels do most of the work.
    const int64_t frag_cells = (int64_t)tile_frag_rows(N, L->n_q) * (L->d_ffn > L->d_model ? L->d_ffn : L->d_model);
    pl.frag_h = pl.hybrid && L->half_h && L->pair_format == 0 && L->n_pairs > 0 && frag_cells < (1LL << 31);
    pl.frag_x = pl.frag_h && L->d_ffn >= FRAG_X_MIN_FFN && N >= (int64_t)TILED_MIN_TOKENS_PER_EXPERT * E64;
    pl.mostly_tiled = pl.hybrid && N >= (int64_t)TILED_MIN_TOKENS_PER_EXPERT * E64;
    pl.tiled_shared = T >= TILED_MIN_TOKENS_SHARED;
    pl.persistent = L->n_q >= 32 && N <= (int64_t)256 * L->n_q;
    if (L->force_persistent >= 0) pl.persistent = L->force_persistent != 0;
    pl.tile_overlap = pl.hybrid && !staged && E64 >= 32 && N < 40 * E64;
    if (L->force_tile_stream >= 0) pl.tile_overlap = pl.hybrid && !staged && L->force_tile_stream != 0;
    // Small batches that only stream (no token tiles to cut): a grouping kernel in front of the first
    // weight-streaming kernel is 5-6 us of a 120-240 us step; the gate/up kernel of the packed pairs
    // sorts the few hundred entries itself instead (stream_gemm.hip, route_in_block).
    pl.fused_route = !pl.hybrid && L->pair_format == 0 && L->n_pairs > 0 && N >= 1 &&
                     N <= STREAM_FUSED_ROUTE_MAX_FLAT && L->n_q <= STREAM_FUSED_ROUTE_MAX_KEYS;

    const int ns = L->n_shared > 0 ? L->n_shared : 1;
    pl.shared_wgs = shared_target_wgs(L, k, pl.hybrid && pl.persistent);
    int ksplit_shared = choose_ksplit(ns * ((T + 63) / 64), L->d_model);
    if (pl.tiled_shared) {
        ksplit_shared = MAX_KSPLIT;
        for (int s = 0; s < L->n_shared; ++s) {
            int ks = choose_tile_ksplit((int64_t)ns * shared_token_parts(T, ns, L->shared_f[s], pl.shared_wgs, pl.hybrid && pl.persistent), (int64_t)ns * T,
                                        L->d_model, L->shared_f[s], pl.overlap ? 32 : 8);
            if (ks < ksplit_shared) ksplit_shared = ks;
        }
    }
    // Next to the routed kernels (own stream) the shared experts need not fill the chip by
    // themselves, and every split is another set of partial sums for the combine step: at most 3
    // (60 experts + 1 shared expert of 5632: 256 tokens 166 -> 164 us, 1024 tokens 318 -> 306;
    // 64 experts + 2 shared of 1408: within 1 %)
    // and a split keeps at least 32 K steps (choose_tile_ksplit above): two narrow shared experts of
    // 1408 stay unsplit (64 experts top-6, 1024 / 2048 tokens: 392 / 572 -> 379 / 559 us)
    if (pl.overlap && pl.tiled_shared && ksplit_shared > 3) ksplit_shared = 3;
    for (int s = 0; s < L->n_shared; ++s)                                          // no split without a k-block
        if (ksplit_shared > L->shared_f[s] / TILE_COLS) ksplit_shared = L->shared_f[s] / TILE_COLS;
    pl.ksplit_shared = ksplit_shared;

    const int routed_groups = L->n_pairs + L->n_dense;
    const int groups_max = (int)(N < routed_groups ? N : routed_groups);           // groups that can have tokens
    int ksplit = pl.mostly_tiled ? choose_tile_ksplit(N / TILE_MAX_TOKENS + L->n_experts / 2, N, L->d_model, L->d_ffn)
                                 : choose_ksplit(groups_max > 0 ? groups_max : 1, L->d_model);
    if (L->pair_format == 1 && ksplit > L->d_ffn / 128) ksplit = L->d_ffn / 128;   // whole 128-column groups per split
    if (ksplit > L->d_ffn / TILE_COLS) ksplit = L->d_ffn / TILE_COLS;              // no split without a k-block (tiny layers)
    pl.ksplit = ksplit;
    return pl;
}

static WorkspaceLayout carve(const pzl_layer *L, int32_t T, int32_t k)
{
    WorkspaceLayout w;
    const size_t N = (size_t)T * k;
    const size_t slots = N + (size_t)L->n_shared * T;
    size_t p = 0;
    w.cnt = p;       p += align_up((size_t)L->n_q * 4, 256);
    w.off = p;       p += align_up(((size_t)L->n_q + 1) * 4, 256);
    w.slot_tok = p;  p += align_up(N * 4, 256);
    w.slot_of = p;   p += align_up(N * 4, 256);
    const size_t mt = (size_t)max_token_tiles((int64_t)N, L->n_q);
    w.tile_q = p;     p += align_up(mt * 4, 256);
    w.tile_slot0 = p; p += align_up(mt * 4, 256);
    w.tile_n = p;     p += align_up(mt * 4, 256);
    w.n_tiles = p;    p += 256;
    // routed H: two bf16 planes, or one half-precision plane if every routed expert is a packed pair in that form
    const size_t h_planes = (L->half_h && L->n_dense == 0) ? 1 : 2;
    w.h_routed = p;  p += align_up(h_planes * N * L->d_ffn * 2, 256);
    // fragment-ordered H (written by the tiled gate/up stage for the tiled down stage) and x (gathered)
    const Plan pl = make_plan(L, T, k, false);
    const size_t frag_rows = tile_frag_rows((int64_t)N, L->n_q);
    w.has_h_frag = pl.frag_h; w.has_x_frag = pl.frag_x;
    w.h_frag = p;    if (w.has_h_frag) p += align_up(frag_rows * L->d_ffn * 2, 256);
    w.x_frag = p;    if (w.has_x_frag) p += align_up(frag_rows * L->d_model * 2, 256);
    w.h_shared = p;
    for (int s = 0; s < L->n_shared; ++s) p += w.h_shared_each(L, T, s);
    w.o_ks_stride = (int64_t)slots * L->d_model;
    w.opart = p;     p += align_up((size_t)MAX_KSPLIT * slots * L->d_model * 4, 256);
    w.total = p;
    return w;
}

}  // namespace pzl

using namespace pzl;

extern "C" {

int pzl_abi_version(void) { return PZL_ABI_VERSION; }

const char *pzl_strerror(int rc)
{
    switch (rc) {
        case PZL_OK: return "ok";
        case PZL_EINVAL: return "invalid argument (null pointer, bad shape, bad position or pair map)";
        case PZL_ENOSPC: return "workspace too small (pzl_moe_ffn_static: the batch needs more than the static scratch array holds)";
        case PZL_EHIP: return "HIP call or kernel launch failed (see pzl_last_hip_error)";
        case PZL_ENOMEM: return "device allocation failed";
        default: return "unknown error code";
    }
}

const char *pzl_last_hip_error(void) { return g_hip_error; }

size_t pzl_packed_bytes(int64_t rows, int64_t cols)
{
    if (rows <= 0 || cols <= 0) return 0;
    return (size_t)rows * (size_t)cols * 2;
}

int pzl_pack(const uint16_t *merged, const uint8_t *mask0, const uint8_t *mask1, const uint8_t *sign0,
             const uint8_t *sign1, int64_t rows, int64_t cols, uint16_t *packed_out,
             int32_t *n_out_of_range, void *stream)
{
    return launch_pack(merged, mask0, mask1, sign0, sign1, rows, cols, packed_out, n_out_of_range,
                       (hipStream_t)stream);
}

int pzl_unpack(const uint16_t *packed, int expert_pos, int64_t rows, int64_t cols, uint16_t *out,
               void *stream)
{
    return launch_unpack(packed, expert_pos, rows, cols, out, false, (hipStream_t)stream);
}

int pzl_unpack_half_x2(const uint16_t *packed, int expert_pos, int64_t rows, int64_t cols, uint16_t *out,
                       void *stream)
{
    return launch_unpack(packed, expert_pos, rows, cols, out, true, (hipStream_t)stream);
}

size_t pzl_q_record_bytes(int64_t rows, int64_t cols) { return q_record_bytes(rows, cols); }
size_t pzl_q_scale_bytes(int64_t rows, int64_t cols) { return q_scale_bytes(rows, cols); }

int pzl_q_pack(const uint16_t *merged, const uint8_t *mask0, const uint8_t *mask1, const uint8_t *sign0,
               const uint8_t *sign1, int64_t rows, int64_t cols, uint8_t *records_out,
               uint16_t *scales_out, int32_t *n_non_finite, void *stream)
{
    if ((uintptr_t)records_out & 7) return PZL_EINVAL;
    return launch_q_pack(merged, mask0, mask1, sign0, sign1, rows, cols, records_out, scales_out,
                         n_non_finite, (hipStream_t)stream);
}

int pzl_q_unpack(const uint8_t *records, const uint16_t *scales, int expert_pos, int64_t rows,
                 int64_t cols, float *out, void *stream)
{
    return launch_q_unpack(records, scales, expert_pos, rows, cols, out, (hipStream_t)stream);
}

int pzl_tile_dense(const uint16_t *dense_rowmajor, int64_t rows, int64_t cols, uint16_t *tiled_out,
                   void *stream)
{
    return launch_tile_dense(dense_rowmajor, rows, cols, tiled_out, (hipStream_t)stream);
}

int pzl_merge_pack(const uint16_t *w_i, const uint16_t *w_j, const float *norm_i, const float *norm_j,
                   int64_t rows, int64_t cols, float tau_sim, uint16_t *packed_out, int32_t *n_similar,
                   int32_t *n_out_of_range, void *stream)
{
    return launch_merge_pack(w_i, w_j, norm_i, norm_j, rows, cols, tau_sim, packed_out, n_similar,
                             n_out_of_range, (hipStream_t)stream);
}

int pzl_router_topk(const uint16_t *x, const uint16_t *w_router, int32_t T, int32_t d_model, int32_t n_experts,
                    int32_t k, int32_t *topk_ids, float *topk_w, void *stream)
{
    return launch_router_topk(x, w_router, T, d_model, n_experts, k, topk_ids, topk_w, (hipStream_t)stream);
}

int pzl_layer_create(const pzl_layer_desc *desc, pzl_layer **out)
{
    if (!desc || !out) return PZL_EINVAL;
    *out = nullptr;
    const int E = desc->n_experts, d = desc->d_model, f = desc->d_ffn, S = desc->n_shared, D = desc->n_dense;
    if (E < 1 || E > 256 || D < 0 || D > E || ((E - D) & 1) || d <= 0 || f <= 0 || d % TILE_COLS || f % TILE_COLS)
        return PZL_EINVAL;
    const int P = (E - D) / 2;
    if (!desc->expert_pair || !desc->expert_pos) return PZL_EINVAL;
    if (P > 0 && (!desc->gate || !desc->up || !desc->down)) return PZL_EINVAL;
    if (D > 0 && (!desc->dense_gate || !desc->dense_up || !desc->dense_down)) return PZL_EINVAL;
    const int fmt = desc->pair_format;
    if (fmt != 0 && fmt != 1) return PZL_EINVAL;
    if (fmt == 1 && P > 0 && (d % 128 || f % 128 || !desc->gate_scale || !desc->up_scale || !desc->down_scale))
        return PZL_EINVAL;
    if (desc->h_precision != 0 && desc->h_precision != 1) return PZL_EINVAL;
    if (S < 0 || S > 16) return PZL_EINVAL;
    if (S > 0 && (!desc->shared_d_ffn || !desc->shared_gate || !desc->shared_up || !desc->shared_down))
        return PZL_EINVAL;
    // every (pair, position) and every unmerged expert must be named exactly once
    std::vector<int32_t> q_of(E);
    std::vector<char> seen(2 * (P + D), 0);
    for (int e = 0; e < E; ++e) {
        int p = desc->expert_pair[e], pos = desc->expert_pos[e];
        int q;
        if (p >= 0) {
            if (p >= P || pos < 0 || pos > 1) return PZL_EINVAL;
            q = 2 * p + pos;
        } else {
            int j = -1 - p;
            if (j >= D) return PZL_EINVAL;
            q = 2 * (P + j);
        }
        if (seen[q]) return PZL_EINVAL;
        seen[q] = 1;
        q_of[e] = q;
    }
    for (int p = 0; p < P; ++p) {
        if (!desc->gate[p] || !desc->up[p] || !desc->down[p]) return PZL_EINVAL;
        if (fmt == 1 && (!desc->gate_scale[p] || !desc->up_scale[p] || !desc->down_scale[p])) return PZL_EINVAL;
    }
    for (int j = 0; j < D; ++j)
        if (!desc->dense_gate[j] || !desc->dense_up[j] || !desc->dense_down[j]) return PZL_EINVAL;
    for (int s = 0; s < S; ++s) {
        int fs = desc->shared_d_ffn[s];
        if (fs <= 0 || fs % TILE_COLS || !desc->shared_gate[s] || !desc->shared_up[s] || !desc->shared_down[s])
            return PZL_EINVAL;
    }

    pzl_layer *L = new (std::nothrow) pzl_layer();
    if (!L) return PZL_ENOMEM;
    L->n_experts = E; L->n_pairs = P; L->n_dense = D; L->d_model = d; L->d_ffn = f; L->n_shared = S;
    L->n_q = 2 * (P + D);
    L->pair_format = fmt;
    L->shared_f.assign(desc->shared_d_ffn, desc->shared_d_ffn + S);

    const size_t sz_q = align_up((size_t)E * 4, 256);
    const size_t sz_p = align_up((size_t)(P > 0 ? P : 1) * sizeof(void *), 256);
    const size_t sz_s = align_up((size_t)(S > 0 ? S : 1) * sizeof(void *), 256);
    const size_t sz_d = align_up((size_t)(D > 0 ? D : 1) * sizeof(void *), 256);
    const size_t sz_c = 256;                                   // counters (see pzl_layer.d_counters)
    const size_t total = sz_q + 6 * sz_p + 3 * sz_s + 3 * sz_d + sz_c;
    std::vector<unsigned char> host(total, 0);
    size_t o = 0;
    memcpy(&host[o], q_of.data(), (size_t)E * 4);                     size_t o_q = o;  o += sz_q;
    size_t o_g = o; if (P) memcpy(&host[o], desc->gate, (size_t)P * sizeof(void *)); o += sz_p;
    size_t o_u = o; if (P) memcpy(&host[o], desc->up, (size_t)P * sizeof(void *));   o += sz_p;
    size_t o_d = o; if (P) memcpy(&host[o], desc->down, (size_t)P * sizeof(void *)); o += sz_p;
    const bool q = fmt == 1 && P > 0;
    size_t o_gs = o; if (q) memcpy(&host[o], desc->gate_scale, (size_t)P * sizeof(void *)); o += sz_p;
    size_t o_us = o; if (q) memcpy(&host[o], desc->up_scale, (size_t)P * sizeof(void *));   o += sz_p;
    size_t o_ds = o; if (q) memcpy(&host[o], desc->down_scale, (size_t)P * sizeof(void *)); o += sz_p;
    size_t o_dg = o; if (D) memcpy(&host[o], desc->dense_gate, (size_t)D * sizeof(void *)); o += sz_d;
    size_t o_du = o; if (D) memcpy(&host[o], desc->dense_up, (size_t)D * sizeof(void *));   o += sz_d;
    size_t o_dd = o; if (D) memcpy(&host[o], desc->dense_down, (size_t)D * sizeof(void *)); o += sz_d;
    size_t o_sg = o; if (S) memcpy(&host[o], desc->shared_gate, (size_t)S * sizeof(void *)); o += sz_s;
    size_t o_su = o; if (S) memcpy(&host[o], desc->shared_up, (size_t)S * sizeof(void *));   o += sz_s;
    size_t o_sd = o; if (S) memcpy(&host[o], desc->shared_down, (size_t)S * sizeof(void *)); o += sz_s;
    const size_t o_c = o; o += sz_c;

    hipError_t e = hipMalloc(&L->d_block, total);
    if (e != hipSuccess) { set_hip_error(e); delete L; return PZL_ENOMEM; }
    e = hipMemcpy(L->d_block, host.data(), total, hipMemcpyHostToDevice);
    if (e != hipSuccess) { set_hip_error(e); (void)hipFree(L->d_block); delete L; return PZL_EHIP; }
    unsigned char *base = (unsigned char *)L->d_block;
    L->d_q_of_expert = (int32_t *)(base + o_q);
    L->d_gate = (const uint16_t **)(base + o_g);
    L->d_up = (const uint16_t **)(base + o_u);
    L->d_down = (const uint16_t **)(base + o_d);
    L->d_gscale = (const uint16_t **)(base + o_gs);
    L->d_uscale = (const uint16_t **)(base + o_us);
    L->d_dscale = (const uint16_t **)(base + o_ds);
    L->d_dgate = (const uint16_t **)(base + o_dg);
    L->d_dup = (const uint16_t **)(base + o_du);
    L->d_ddown = (const uint16_t **)(base + o_dd);
    L->d_sgate = (const uint16_t **)(base + o_sg);
    L->d_sup = (const uint16_t **)(base + o_su);
    L->d_sdown = (const uint16_t **)(base + o_sd);
    L->d_counters = (int32_t *)(base + o_c);
    // Half-precision H needs every used exponent field of the down matrices to be at most 29
    // (weights below 2^15): scan them once (device work on the null stream, then one blocking copy).
    L->half_h = false;
    if (fmt == 0 && P > 0 && desc->h_precision == 0) {
        int rc_scan = PZL_OK;
        for (int p = 0; p < P && !rc_scan; ++p) rc_scan = launch_max_exp_field(desc->down[p], d, f, L->d_counters, nullptr);
        int32_t mx = 31;
        if (!rc_scan) {
            e = hipMemcpy(&mx, L->d_counters, sizeof(mx), hipMemcpyDeviceToHost);
            if (e != hipSuccess) { set_hip_error(e); rc_scan = PZL_EHIP; }
        }
        if (rc_scan) { pzl_layer_destroy(L); return rc_scan; }
        L->half_h = mx <= 29;
    }
    // The shared experts' down matrices likewise: with their largest exponent field known, the tiled
    // kernels decode them to half precision times a power of two that puts the largest weights at
    // the top of its range, and H can be one half-precision plane for them too.  Not with an
    // infinity or a NaN among them (field 255), and not if the caller asked for wide H.
    L->shared_max_exp.assign(S, -1);
    if (S > 0 && desc->h_precision == 0) {
        for (int sdx = 0; sdx < S; ++sdx) {
            int32_t mx = 255;
            e = hipMemset(L->d_counters, 0, sizeof(int32_t));
            int rc_scan = e == hipSuccess ? launch_max_exp_bf16(desc->shared_down[sdx], (int64_t)d * desc->shared_d_ffn[sdx], L->d_counters, nullptr) : PZL_EHIP;
            if (e == hipSuccess && !rc_scan) e = hipMemcpy(&mx, L->d_counters, sizeof(mx), hipMemcpyDeviceToHost);
            if (e != hipSuccess) { set_hip_error(e); rc_scan = PZL_EHIP; }
            if (rc_scan) { pzl_layer_destroy(L); return rc_scan; }
            L->shared_max_exp[sdx] = mx <= 254 ? mx : -1;
        }
    }
    L->aux_stream = nullptr; L->ev_fork = nullptr; L->ev_join = nullptr;
    if (S > 0) {                                               // default priority, as every stream here
        e = hipStreamCreateWithFlags(&L->aux_stream, hipStreamNonBlocking);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&L->ev_fork, hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&L->ev_join, hipEventDisableTiming);
        if (e != hipSuccess) { set_hip_error(e); pzl_layer_destroy(L); return PZL_EHIP; }
    }
    // set-up work that is not a stream operation, done here so that the FFN calls need none of it:
    // the address of this device's static scratch array and the kernels' dynamic-LDS attribute
    L->static_scratch = static_scratch_of_current_device();
    if (!L->static_scratch) { pzl_layer_destroy(L); return PZL_EHIP; }
    { int rc_prep = prepare_stream_kernels(); if (!rc_prep) rc_prep = prepare_route_kernel(); if (rc_prep) { pzl_layer_destroy(L); return rc_prep; } }
    L->tile_stream = nullptr; L->ev_tfork = nullptr; L->ev_tjoin = nullptr;
    if (L->pair_format == 0) {
        e = hipStreamCreateWithFlags(&L->tile_stream, hipStreamNonBlocking);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&L->ev_tfork, hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&L->ev_tjoin, hipEventDisableTiming);
        if (e != hipSuccess) { set_hip_error(e); pzl_layer_destroy(L); return PZL_EHIP; }
    }
    *out = L;
    return PZL_OK;
}

void pzl_layer_destroy(pzl_layer *layer)
{
    if (!layer) return;
    if (layer->ev_fork) (void)hipEventDestroy(layer->ev_fork);
    if (layer->ev_join) (void)hipEventDestroy(layer->ev_join);
    if (layer->aux_stream) (void)hipStreamDestroy(layer->aux_stream);
    if (layer->ev_tfork) (void)hipEventDestroy(layer->ev_tfork);
    if (layer->ev_tjoin) (void)hipEventDestroy(layer->ev_tjoin);
    if (layer->tile_stream) (void)hipStreamDestroy(layer->tile_stream);
    if (layer->d_block) (void)hipFree(layer->d_block);
    delete layer;
}

// The kernels address x, H (two planes) and the shared experts' H with 32-bit byte offsets.
static bool batch_fits(const pzl_layer *L, int64_t T, int64_t k)
{
    if (T * L->d_model >= (1LL << 31) || T * k * L->d_ffn >= (1LL << 30)) return false;
    for (int s = 0; s < L->n_shared; ++s)
        if ((int64_t)L->n_shared * T * L->shared_f[s] >= (1LL << 30)) return false;
    return true;
}

int pzl_moe_ffn_plan(const pzl_layer_shape *shape, int32_t T, int32_t k, pzl_plan *out)
{
    if (!shape || !out || T < 0 || k < 0) return PZL_EINVAL;
    const int E = shape->n_experts, D = shape->n_unmerged, S = shape->n_shared;
    if (E < 1 || E > 256 || D < 0 || D > E || ((E - D) & 1) || shape->d_model <= 0 || shape->d_ffn <= 0 ||
        shape->d_model % TILE_COLS || shape->d_ffn % TILE_COLS || S < 0 || S > 16 || (S > 0 && !shape->shared_d_ffn) ||
        (shape->pair_format != 0 && shape->pair_format != 1))
        return PZL_EINVAL;
    for (int s = 0; s < S; ++s)
        if (shape->shared_d_ffn[s] <= 0 || shape->shared_d_ffn[s] % TILE_COLS) return PZL_EINVAL;
    pzl_layer L = {};                                        // the host fields only: make_plan reads nothing else
    L.n_experts = E; L.n_dense = D; L.n_pairs = (E - D) / 2; L.n_q = 2 * (L.n_pairs + D);
    L.d_model = shape->d_model; L.d_ffn = shape->d_ffn; L.n_shared = S; L.pair_format = shape->pair_format;
    L.shared_f.assign(shape->shared_d_ffn, shape->shared_d_ffn + S);
    const Plan pl = make_plan(&L, T, k, false);
    *out = pzl_plan{};
    out->shared_stream = pl.overlap; out->hybrid = pl.hybrid; out->tile_min = pl.hybrid ? pl.tile_min : 0;
    out->persistent = pl.hybrid && pl.persistent; out->tile_stream = pl.tile_overlap;
    out->ksplit = pl.ksplit; out->ksplit_shared = S > 0 ? pl.ksplit_shared : 0; out->tiled_shared = S > 0 && pl.tiled_shared;
    out->grouping_in_kernel = pl.fused_route;
    out->sweep_wgs_packed = stream_pass_wgs(T, L.pair_format == 1 ? KIND_QUANT : KIND_PACKED, pl.tile_min);
    out->sweep_wgs_unmerged = stream_pass_wgs(T, KIND_UNMERGED, pl.tile_min);
    for (int s = 0; s < S;) {                                // experts of equal width share a launch
        int nb = 1;
        while (s + nb < S && L.shared_f[s + nb] == L.shared_f[s]) ++nb;
        int tiles = 0, tokens = 0;
        if (pl.tiled_shared) {
            const int parts = shared_token_parts(T, nb, L.shared_f[s], pl.shared_wgs, pl.hybrid && pl.persistent);
            tokens = ((T + parts - 1) / parts + 15) & ~15;
            tiles = (T + tokens - 1) / tokens;
        }
        for (int j = 0; j < nb; ++j) { out->shared_token_tiles[s + j] = tiles; out->shared_tile_tokens[s + j] = tokens; }
        s += nb;
    }
    return PZL_OK;
}

size_t pzl_moe_ffn_workspace_bytes(const pzl_layer *layer, int32_t max_tokens, int32_t top_k)
{
    if (!layer || max_tokens < 0 || top_k < 0) return 0;
    if ((int64_t)max_tokens * top_k > 0x3FFFFFFF || !batch_fits(layer, max_tokens, top_k)) return 0;
    // every buffer grows with T, so the layout at max_tokens bounds all smaller batches
    return carve(layer, max_tokens, top_k).total;
}

int pzl_moe_ffn_workspace_layout(const pzl_layer *layer, int32_t T, int32_t k, pzl_workspace_layout *out)
{
    if (!layer || !out || T < 0 || k < 0) return PZL_EINVAL;
    if ((int64_t)T * k > 0x3FFFFFFF || !batch_fits(layer, T, k)) return PZL_EINVAL;
    const WorkspaceLayout w = carve(layer, T, k);
    *out = pzl_workspace_layout{};
    out->n_keys = layer->n_q;
    out->max_tiles = max_token_tiles((int64_t)T * k, layer->n_q);
    out->streamed_count = w.cnt; out->first_slot = w.off; out->slot_token = w.slot_tok; out->slot_of = w.slot_of;
    out->tile_key = w.tile_q; out->tile_first_slot = w.tile_slot0; out->tile_tokens = w.tile_n; out->n_tiles = w.n_tiles;
    out->total = w.total;
    return PZL_OK;
}

int pzl_moe_ffn(const pzl_layer *L, const uint16_t *x, const int32_t *topk_ids, const float *topk_w,
                int32_t T, int32_t k, uint16_t *y, void *workspace, size_t workspace_bytes, void *stream)
{
    return pzl_moe_ffn_staged(L, x, topk_ids, topk_w, T, k, y, workspace, workspace_bytes, stream, nullptr);
}

int pzl_moe_ffn_static(const pzl_layer *L, const uint16_t *x, const int32_t *topk_ids, const float *topk_w,
                       int32_t T, int32_t k, uint16_t *y, void *stream)
{
    if (!L || T < 0 || k < 0) return PZL_EINVAL;
    if (T == 0) return PZL_OK;
    if ((int64_t)T * k > 0x3FFFFFFF || !batch_fits(L, T, k)) return PZL_EINVAL;
    if (carve(L, T, k).total > (size_t)PZL_STATIC_SCRATCH_BYTES) return PZL_ENOSPC;
    // L->static_scratch is the device address found at pzl_layer_create; never the array's name
    return pzl_moe_ffn_staged(L, x, topk_ids, topk_w, T, k, y, L->static_scratch, PZL_STATIC_SCRATCH_BYTES, stream, nullptr);
}

int pzl_layer_h_info(const pzl_layer *layer, int32_t *half_precision, int32_t *saturated)
{
    if (!layer) return PZL_EINVAL;
    if (half_precision) *half_precision = layer->half_h ? 1 : 0;
    if (saturated) {
        hipError_t e = hipMemcpy(saturated, layer->d_counters + 1, sizeof(int32_t), hipMemcpyDeviceToHost);
        if (e != hipSuccess) { set_hip_error(e); return PZL_EHIP; }
    }
    return PZL_OK;
}

int pzl_layer_force_plan(pzl_layer *layer, int32_t hybrid, int32_t persistent, int32_t tile_stream)
{
    if (!layer || hybrid < -1 || hybrid > 1 || persistent < -1 || persistent > 1 || tile_stream < -1 || tile_stream > 1)
        return PZL_EINVAL;
    layer->force_hybrid = hybrid; layer->force_persistent = persistent; layer->force_tile_stream = tile_stream;
    return PZL_OK;
}

size_t pzl_moe_ffn_static_max_bytes(void) { return (size_t)PZL_STATIC_SCRATCH_BYTES; }

int pzl_moe_ffn_staged(const pzl_layer *L, const uint16_t *x, const int32_t *topk_ids, const float *topk_w,
                       int32_t T, int32_t k, uint16_t *y, void *workspace, size_t workspace_bytes,
                       void *stream, void *const *stage_events)
{
    // records the caller's events around a stage; a failed record is reported like a failed launch
    auto mark = [&](int stage, int end) -> int {
        if (!stage_events || !stage_events[2 * stage + end]) return PZL_OK;
        hipError_t e = hipEventRecord((hipEvent_t)stage_events[2 * stage + end], (hipStream_t)stream);
        if (e != hipSuccess) { set_hip_error(e); return PZL_EHIP; }
        return PZL_OK;
    };
    if (!L || T < 0 || k < 0) return PZL_EINVAL;
    if (T == 0) return PZL_OK;
    if (!x || !y || (k > 0 && (!topk_ids || !topk_w)) || !workspace) return PZL_EINVAL;
    if ((int64_t)T * k > 0x3FFFFFFF || ((uintptr_t)workspace & 255)) return PZL_EINVAL;
    if (!batch_fits(L, T, k)) return PZL_EINVAL;
    // Quantised pairs have no tiled kernel: the streaming kernels serve 32 tokens of an expert per
    // sweep of its pair's weights and sweep again for every 32 more.  Batches that would, on
    // average, sweep more than twice are refused rather than served at a fraction of the speed
    // (the caller splits them, or keeps such layers in the 16-bit format).
    if (L->pair_format == 1 && (int64_t)T * k > (int64_t)QUANT_MAX_SLOTS_PER_EXPERT * L->n_experts) return PZL_EINVAL;
    const WorkspaceLayout w = carve(L, T, k);
    if (workspace_bytes < w.total) return PZL_ENOSPC;
    hipStream_t st = (hipStream_t)stream;
    unsigned char *ws = (unsigned char *)workspace;
    const int32_t N = T * k;
    // Shared experts on the layer's second stream, unless the caller times stages (then every
    // stage runs alone on the caller's stream) or there is nothing to run next to.
    const Plan pl = make_plan(L, T, k, stage_events != nullptr);
    const bool overlap = pl.overlap;
    hipStream_t sst = overlap ? L->aux_stream : st;
    if (overlap) {
        hipError_t e = hipEventRecord(L->ev_fork, st);
        if (e == hipSuccess) e = hipStreamWaitEvent(L->aux_stream, L->ev_fork, 0);
        if (e != hipSuccess) { set_hip_error(e); return PZL_EHIP; }
    }

    RouteTables rt;
    rt.cnt = (int32_t *)(ws + w.cnt);
    rt.off = (int32_t *)(ws + w.off);
    rt.slot_tok = (int32_t *)(ws + w.slot_tok);
    rt.slot_of = (int32_t *)(ws + w.slot_of);
    rt.tile_q = (int32_t *)(ws + w.tile_q);
    rt.tile_slot0 = (int32_t *)(ws + w.tile_slot0);
    rt.tile_n = (int32_t *)(ws + w.tile_n);
    rt.n_tiles = (int32_t *)(ws + w.n_tiles);
    uint16_t *h_routed = (uint16_t *)(ws + w.h_routed);
    uint16_t *h_frag = w.has_h_frag ? (uint16_t *)(ws + w.h_frag) : nullptr;
    uint16_t *x_frag = w.has_x_frag ? (uint16_t *)(ws + w.x_frag) : nullptr;
    float *opart = (float *)(ws + w.opart);

    // Path choice.  With few tokens per expert the layer is bound by streaming the packed weights
    // once (streaming kernels); with many it is a dense contraction (tiled kernels on the matrix
    // cores).  The streaming kernels take 32 tokens per expert in one sweep of a pair's weights
    // and need another sweep, in sequence, for every 32 more; measured over the Mixtral-, Qwen-
    // and DeepSeek-shaped layers the tiled kernels win as soon as a second sweep would be needed.
    // The host only knows the batch shape, not how the router spread the tokens: from an average
    // of HYBRID_MIN_TOKENS_PER_EXPERT both paths are launched and the grouping kernel decides
    // per pair (tile_min).  Below that average only the streaming kernels are launched (two
    // empty tiled launches would cost the decode step 3 %).  With many experts the average is
    // set low: a router that favours some experts gives them several sweeps' worth of tokens
    // long before the average says so (64 experts, top-6, skewed: 96-192 tokens 272-464 us
    // streamed, 201-246 us with the busy pairs tiled), while two launches that find no tile cost
    // 10-20 us (60 experts, top-4, even routing, 128-192 tokens: 155-171 -> 178-182 us).  With
    // few experts the counts stay near their average.  (6 rather than 8 slots per expert: with
    // the tiled launches on their own stream an even router pays 3-4 % between the two, 60 experts
    // top-4 at 96-112 tokens, a skewed one gains 3-12 %, 64 experts top-6 at 64-80 tokens.)
    // (quantised pairs have no tiled kernel: they always stream)
    const int tile_min = pl.tile_min;
    const bool tiled = pl.hybrid, streamed = true;
    const bool tiled_shared = pl.tiled_shared;

    // Many experts with at most about one full tile each: the tile list is far shorter than its
    // bound and its tiles are uneven, so the tiled launches are persistent and draw their tiles
    // (counters zeroed by the grouping kernel).  Otherwise one workgroup per tile of the bound.
    // Measured (whole step, persistent vs not): 64 experts top-6 at 512-2048 tokens -9 %, at 4096
    // +4 %; 60 experts top-4 at 2048 -3 %, at 4096 +3 %; 8 experts top-2 at 2048-4096 +5-7 %.
    const bool persistent = pl.persistent;
    // one k-split count for all shared experts (the combine step sums that many partials); sized
    // for the usual case, all of them of one width and hence in one launch per stage
    const int shared_wgs = pl.shared_wgs;
    const int ksplit_shared = pl.ksplit_shared;
    // Shared experts of equal width go into one launch per stage (group index = expert), so that
    // the launch has enough workgroups; their H rows sit back to back, slot = N + s*T + t.
    auto launch_shared = [&]() -> int {
        int rc;
        size_t h_off = w.h_shared;
        for (int s = 0; s < L->n_shared;) {
            int nb = 1;
            while (s + nb < L->n_shared && L->shared_f[s + nb] == L->shared_f[s]) ++nb;
            uint16_t *h_s = (uint16_t *)(ws + h_off);
            for (int j = 0; j < nb; ++j) h_off += w.h_shared_each(L, T, s + j);
            const int32_t slot_base = N + s * T;
            const int64_t hs_plane = (int64_t)nb * T * L->shared_f[s];
            if (tiled_shared) {
                TileGemmArgs a = {};
                const int parts = shared_token_parts(T, nb, L->shared_f[s], shared_wgs, pl.hybrid && pl.persistent);
                a.dense_tokens = T; a.dense_slot_base = slot_base;
                a.dense_tile_tokens = ((T + parts - 1) / parts + 15) & ~15;
                a.dense_tiles = nb * ((T + a.dense_tile_tokens - 1) / a.dense_tile_tokens);
                a.max_mtiles = a.dense_tiles;
                a.w_a = L->d_sgate + s; a.w_b = L->d_sup + s;
                a.rows = L->shared_f[s]; a.kdim = L->d_model;
                a.act = x; a.act_is_x = 1;
                a.h_out = h_s; a.h_slot_base = slot_base; a.h_plane_stride = hs_plane;
                // half-precision H if every expert of the launch allows it, with their common scale
                int mx = 0;
                bool half_ok = true;
                for (int j = 0; j < nb; ++j) { half_ok = half_ok && L->shared_max_exp[s + j] >= 0; mx = std::max(mx, L->shared_max_exp[s + j]); }
                a.half_h = half_ok; a.dense_half_bias = std::max(mx - 30, 0); a.h_saturated = L->d_counters + 1;
                rc = launch_tile_gateup(a, KIND_SHARED, sst);
                if (rc) return rc;
                a.w_a = L->d_sdown + s; a.w_b = nullptr;
                a.rows = L->d_model; a.kdim = L->shared_f[s];
                a.act = h_s; a.act_is_x = 0; a.act_slot_base = slot_base; a.act_plane_stride = hs_plane;
                a.h_out = nullptr; a.o_out = opart; a.o_ks_stride = w.o_ks_stride; a.ksplit = ksplit_shared;
                rc = launch_tile_down(a, KIND_SHARED, sst);
                if (rc) return rc;
                s += nb;
                continue;
            }
            StreamGroupArgs a = {};
            a.n_groups = nb;
            a.dense_tokens = T; a.dense_slot_base = slot_base;
            a.w_a = L->d_sgate + s; a.w_b = L->d_sup + s;
            a.rows = L->shared_f[s]; a.kdim = L->d_model; a.ksplit = 1;
            a.act = x; a.act_is_x = 1; a.act_slot_base = 0;
            a.h_out = h_s; a.h_slot_base = slot_base; a.h_plane_stride = hs_plane;
            rc = launch_stream_gateup(a, KIND_SHARED, sst);
            if (rc) return rc;
            a.w_a = L->d_sdown + s; a.w_b = nullptr;
            a.rows = L->d_model; a.kdim = L->shared_f[s]; a.ksplit = ksplit_shared;
            a.act = h_s; a.act_is_x = 0; a.act_slot_base = slot_base; a.act_plane_stride = hs_plane;
            a.h_out = nullptr; a.o_out = opart; a.o_ks_stride = w.o_ks_stride;
            rc = launch_stream_down(a, KIND_SHARED, sst);
            if (rc) return rc;
            s += nb;
        }
        return PZL_OK;
    };
    // The shared experts do not depend on the routing: with a stream of their own they are
    // enqueued first, so that they can start with the grouping kernel and not when the host gets
    // to them after the routed launches (no difference in a loop of calls, where the host runs
    // ahead of the device anyway; it matters to a caller that waits for each call).
    if (overlap) {
        int rc_shared = launch_shared();
        if (rc_shared) return rc_shared;
    }

    int rc = mark(PZL_STAGE_ROUTE, 0);
    if (rc) return rc;
    // both experts of a pair may get one tile (the row groups of gate/up tell the grouping kernel
    // how long the launch is)
    if (!pl.fused_route) {
        rc = launch_route(topk_ids, N, k, L->n_experts, L->n_q, L->d_q_of_expert, rt, tile_min,
                          (L->d_ffn + 127) / 128, (L->d_ffn + 127) / 128, st);   // (in units of a compute unit's share of a launch)
        if (rc) return rc;
    }
    if ((rc = mark(PZL_STAGE_ROUTE, 1))) return rc;
    // The tiled and the streaming kernels of the routed experts work on disjoint pairs (the
    // grouping kernel gave each pair to one of them), so the tiled ones run on a stream of their
    // own, forked here and joined before the combine: a launch that finds no tile then costs
    // nothing, and where both have work they fill the chip together (64 experts, top-6, skewed,
    // 128-256 tokens: -12..-15 %).  The two cross-stream waits cost 5-10 us, so only where a
    // mixture is likely: many experts and fewer than 40 tokens per expert on average (beyond
    // that nearly every pair is tiled); and not when the caller times stages.  Between 32 and 40
    // the routing decides: skewed (64 experts top-6, 384 tokens) 288 -> 238 us, even (60 experts
    // top-4, 512 tokens, every pair tiled) 238 -> 250 us.
    const bool tile_overlap = pl.tile_overlap;
    hipStream_t tst = tile_overlap ? L->tile_stream : st;
    if (tile_overlap) {
        hipError_t e = hipEventRecord(L->ev_tfork, st);
        if (e == hipSuccess) e = hipStreamWaitEvent(L->tile_stream, L->ev_tfork, 0);
        if (e != hipSuccess) { set_hip_error(e); return PZL_EHIP; }
    }

    // one k-split count for all routed slots (the combine step sums that many partials)
    const int ksplit = pl.ksplit;
    const int64_t h_plane = (int64_t)N * L->d_ffn;
    // Routed experts come in two kinds that differ only in the decode: packed pairs (groups
    // [0, P)) and experts kept unmerged (dense bf16, groups [P, P + D), position 0 only).  Both
    // kinds, and both paths, write disjoint slots of the same H and partial-sum buffers.
    for (int stage = 0; stage < 2 && N > 0; ++stage) {
        const int stage_id = stage == 0 ? PZL_STAGE_GATEUP : PZL_STAGE_DOWN;
        if ((rc = mark(stage_id, 0))) return rc;
        for (int pass = 0; pass < 2; ++pass) {
            const bool unmerged = pass == 1;
            const int n_groups = unmerged ? L->n_dense : L->n_pairs;
            if (n_groups == 0) continue;
            const int kind = unmerged ? KIND_UNMERGED : (L->pair_format == 1 ? KIND_QUANT : KIND_PACKED);
            const uint16_t *const *wg = unmerged ? L->d_dgate : L->d_gate;
            const uint16_t *const *wu = unmerged ? L->d_dup : L->d_up;
            const uint16_t *const *wd = unmerged ? L->d_ddown : L->d_down;
            const int group_base = unmerged ? L->n_pairs : 0;
            if (tiled) {
                TileGemmArgs a = {};
                a.slot_tok = rt.slot_tok;
                a.tile_q = rt.tile_q; a.tile_slot0 = rt.tile_slot0; a.tile_n = rt.tile_n; a.n_tiles = rt.n_tiles;
                a.group_lo = group_base; a.group_hi = group_base + n_groups;
                a.max_mtiles = max_token_tiles(N, L->n_q);
                a.block_m = pl.tiles_per_expert <= 4 ? 4 : 0;
                a.half_h = kind == KIND_PACKED && L->half_h; a.h_saturated = L->d_counters + 1;
                a.tile_ctr = persistent ? rt.n_tiles + 8 + (pass * 2 + stage) * 8 : nullptr;
                const bool frag = kind == KIND_PACKED && L->half_h;    // fragment-ordered copies, where the workspace has them
                if (stage == 0) {
                    a.w_a = wg; a.w_b = wu;
                    a.rows = L->d_ffn; a.kdim = L->d_model;
                    a.act = x; a.act_is_x = 1;
                    a.h_out = h_routed; a.h_slot_base = 0; a.h_plane_stride = h_plane;
                    if (frag && x_frag) {
                        rc = launch_gather_x(x, L->d_model, rt.slot_tok, rt.tile_q, rt.tile_slot0, rt.tile_n, rt.n_tiles,
                                             a.max_mtiles, x_frag, tst);
                        if (rc) return rc;
                        a.act_frag = x_frag;
                    }
                    a.h_frag = frag ? h_frag : nullptr;
                    rc = launch_tile_gateup(a, kind, tst);
                } else {
                    a.w_a = wd; a.w_b = nullptr;
                    a.rows = L->d_model; a.kdim = L->d_ffn;
                    a.act = h_routed; a.act_is_x = 0; a.act_slot_base = 0; a.act_plane_stride = h_plane;
                    a.act_frag = frag ? h_frag : nullptr;
                    a.o_out = opart; a.o_ks_stride = w.o_ks_stride; a.ksplit = ksplit;
                    rc = launch_tile_down(a, kind, tst);
                }
                if (rc) return rc;
            }
            if (streamed) {
                StreamGroupArgs a = {};
                a.n_groups = n_groups; a.group_base = group_base;
                a.groups_touched_max = (int)((int64_t)N < n_groups ? N : n_groups);
                a.cnt = rt.cnt; a.off = rt.off; a.slot_tok = rt.slot_tok;
                a.pass_wgs = stream_pass_wgs(T, kind, tile_min);
                a.half_h = kind == KIND_PACKED && L->half_h; a.h_saturated = L->d_counters + 1;
                if (stage == 0) {                        // gate/up + SwiGLU -> H
                    a.w_a = wg; a.w_b = wu;
                    if (kind == KIND_QUANT) { a.s_a = L->d_gscale; a.s_b = L->d_uscale; }
                    a.rows = L->d_ffn; a.kdim = L->d_model; a.ksplit = 1;
                    a.act = x; a.act_is_x = 1; a.act_slot_base = 0;
                    a.h_out = h_routed; a.h_slot_base = 0; a.h_plane_stride = h_plane;
                    if (pl.fused_route && kind == KIND_PACKED) {      // this launch groups the list and writes the tables
                        a.route_ids = topk_ids; a.route_q_of_expert = L->d_q_of_expert;
                        a.route_n_flat = N; a.route_k = k; a.route_n_experts = L->n_experts; a.route_n_keys = L->n_q;
                        a.route_slot_of = rt.slot_of;
                    }
                    rc = launch_stream_gateup(a, kind, st);
                } else {                                 // down -> partial sums
                    a.w_a = wd; a.w_b = nullptr;
                    if (kind == KIND_QUANT) { a.s_a = L->d_dscale; a.s_b = nullptr; }
                    a.rows = L->d_model; a.kdim = L->d_ffn; a.ksplit = ksplit;
                    a.act = h_routed; a.act_is_x = 0; a.act_slot_base = 0; a.act_plane_stride = h_plane;
                    a.o_out = opart; a.o_ks_stride = w.o_ks_stride;
                    rc = launch_stream_down(a, kind, st);
                }
                if (rc) return rc;
            }
        }
        if ((rc = mark(stage_id, 1))) return rc;
    }

    if ((rc = mark(PZL_STAGE_SHARED, 0))) return rc;
    if (!overlap && (rc = launch_shared())) return rc;

    if (tile_overlap) {
        hipError_t e = hipEventRecord(L->ev_tjoin, L->tile_stream);
        if (e == hipSuccess) e = hipStreamWaitEvent(st, L->ev_tjoin, 0);
        if (e != hipSuccess) { set_hip_error(e); return PZL_EHIP; }
    }
    if (overlap) {
        hipError_t e = hipEventRecord(L->ev_join, L->aux_stream);
        if (e == hipSuccess) e = hipStreamWaitEvent(st, L->ev_join, 0);
        if (e != hipSuccess) { set_hip_error(e); return PZL_EHIP; }
    }
    if ((rc = mark(PZL_STAGE_SHARED, 1))) return rc;
    if ((rc = mark(PZL_STAGE_COMBINE, 0))) return rc;
    rc = launch_combine(opart, ksplit, ksplit_shared, w.o_ks_stride, rt, topk_w, T, k, L->d_model, L->n_shared, y, st);
    if (rc) return rc;
    return mark(PZL_STAGE_COMBINE, 1);
}

}  // extern "C"
