/*
 * puzzle_moe.h — C ABI of the MI355X (gfx950) bit-packed merged-expert MoE FFN library.
 *
 * The library implements the inference hot path of PuzzleMoE: two experts of an MoE layer
 * share one merged, non-negative bf16 tensor whose freed exponent bits and unused sign bit
 * hold each expert's mask and sign bit (Sec. 3.3.2 "System Co-design"); an activated
 * expert's weights are rebuilt element by element as (-1)^S * M * W_merged (Eq. 6) by the
 * bit-level decode of Algorithm 1, inside the expert matmuls, without ever materialising
 * the decoded matrix and with one read of the packed tensor serving both experts
 * (Sec. 3.3.2, decode-GEMM).
 *
 * Conventions for every call
 *   - Pointers are DEVICE pointers unless the comment says "host".
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls enqueue
 *     work and return without synchronising; results are valid after the stream is
 *     synchronised.
 *   - No call keeps a reference to caller memory after it returns, except that a
 *     pzl_layer keeps the weight pointers it was created with (the weights stay
 *     caller-owned and must outlive the layer).
 *   - pzl_moe_ffn allocates nothing; everything it needs beyond inputs and outputs is in
 *     the caller's workspace.
 *   - Return value: PZL_OK (0) or a negative PZL_E* code; nothing throws across the ABI.
 *
 * Packed word (16 bits per element, no side metadata; bit positions are those Algorithm 1
 * reads):   15: S0   14: S1   13: M0   12: M1   11..7: exponent-112   6..0: mantissa
 * where S_p / M_p are the sign / mask bit of the expert at position p of the pair.
 *
 * Physical order of a packed (or tiled dense) [rows, cols] matrix.  The paper fixes the
 * word, not the element order in memory; this library stores 16x32 tiles so that one
 * 64-lane wavefront reads 1 KiB contiguously and receives its matrix-core operand
 * directly: rows % 16 == 0 and cols % 32 == 0 are required, and logical element (r, c)
 * lives at 16-bit index
 *     ((r/16) * (cols/32) + c/32) * 512  +  (((c%32)/8) * 16 + r%16) * 8  +  c%8 .
 * pzl_unpack returns the logical row-major matrix.
 */
#ifndef PUZZLE_MOE_H
#define PUZZLE_MOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PZL_ABI_VERSION 6

#define PZL_OK       0
#define PZL_EINVAL  -1   /* null pointer, bad shape, position not 0/1, pair map not a 2-to-1 cover */
#define PZL_ENOSPC  -2   /* workspace too small */
#define PZL_EHIP    -3   /* a HIP call or kernel launch failed; see pzl_last_hip_error() */
#define PZL_ENOMEM  -4   /* pzl_layer_create could not allocate its tables */

int pzl_abi_version(void);
/* Static description of a return code. */
const char *pzl_strerror(int rc);
/* Text of the last HIP error seen by this library on the calling thread (static storage). */
const char *pzl_last_hip_error(void);

/* Size of a packed [rows, cols] tensor: rows*cols*2 bytes, the size of the bf16 tensor it
 * replaces (Sec. 3.3.2: masks and signs are embedded "without additional storage"). */
size_t pzl_packed_bytes(int64_t rows, int64_t cols);

/*
 * pack — Sec. 3.3.2: clamp each exponent to >= 112, subtract 112, and put S0,S1,M0,M1 in the
 * four freed top bits.  Readings where the paper is silent: the mantissa is kept when the
 * exponent is raised; an exactly-zero magnitude is stored with both mask bits cleared; an
 * exponent above 143 (incl. Inf/NaN) is stored as a fully masked word and counted.
 *   merged      [rows, cols] row-major bf16 bit patterns; the sign bit is ignored (Eq. 5)
 *   mask0/1     [rows, cols] row-major bytes, non-zero = element kept for position 0 / 1
 *   sign0/1     [rows, cols] row-major bytes, non-zero = negative (Eq. 1)
 *   packed_out  pzl_packed_bytes(rows, cols) bytes, caller-owned, tiled order (see above)
 *   n_out_of_range  optional int32 on the device; the kernel ADDS the number of
 *               out-of-range elements to it (zero it first).  May be NULL.
 */
int pzl_pack(const uint16_t *merged, const uint8_t *mask0, const uint8_t *mask1,
             const uint8_t *sign0, const uint8_t *sign1, int64_t rows, int64_t cols,
             uint16_t *packed_out, int32_t *n_out_of_range, void *stream);

/*
 * unpack — Algorithm 1 on every element: the weights of the expert at `expert_pos` (0 or 1).
 *   packed  tiled packed tensor written by pzl_pack
 *   out     [rows, cols] row-major bf16 bit patterns, caller-owned
 * Masked-out elements are +0.  Bit-exact by definition.
 */
int pzl_unpack(const uint16_t *packed, int expert_pos, int64_t rows, int64_t cols,
               uint16_t *out, void *stream);

/*
 * The same decode in the second form the library's matmuls use: IEEE half precision, every weight
 * multiplied by 2 (Algorithm 1's exponent field is half precision's own biased exponent; the factor
 * makes field 0 a normal number), as the down projection of a layer with half-precision H runs it.
 * Exact, i.e. out = 2 * pzl_unpack(...) as numbers, for every word whose exponent field is at most
 * 29; words with field 30 or 31 (|w| >= 2^15) have no half-precision form and such tensors are
 * never decoded this way (pzl_layer_create checks).  For inspection and tests.
 *   out     [rows, cols] row-major half-precision bit patterns, caller-owned
 */
int pzl_unpack_half_x2(const uint16_t *packed, int expert_pos, int64_t rows, int64_t cols,
                       uint16_t *out, void *stream);

/*
 * Re-order a dense row-major bf16 matrix (an unmerged shared expert, "other modules
 * unchanged", Sec. 4.1) into the same 16x32 tiled order.  Values are not changed.
 */
int pzl_tile_dense(const uint16_t *dense_rowmajor, int64_t rows, int64_t cols,
                   uint16_t *tiled_out, void *stream);

/*
 * merge_pack — the offline dual-mask merge of two experts (Sec. 3.2, Eqs. 1-5) fused with pack:
 * from the two experts' bf16 matrices straight to the packed pair, position 0 = expert i.
 *   similarity mask   | |wi|-|wj| | / (|wi|+|wj|) <= tau_sim  (evaluated without the division, in
 *                     fp32 with one rounding per operation; 0/0 is "not similar")
 *   sign bits (Eq. 1) w < 0
 *   saliency (Eqs. 2-3)  |wi| * norm_i[c] >= |wj| * norm_j[c] keeps expert i on dissimilar elements
 *   masks (Eq. 4)     saliency OR similarity;   merged (Eq. 5) mean magnitude where similar (fp32
 *                     mean rounded to bf16, nearest even), else the kept expert's magnitude
 *   w_i, w_j    [rows, cols] row-major bf16 bit patterns
 *   norm_i/j    [cols] fp32, the l2 norm of each input channel's calibration activations
 *   tau_sim     in [0, 1] (the paper uses 0.4)
 *   packed_out  pzl_packed_bytes(rows, cols) bytes, tiled order
 *   n_similar, n_out_of_range  optional int32 counters on the device, ADDED to (zero them first)
 */
int pzl_merge_pack(const uint16_t *w_i, const uint16_t *w_j, const float *norm_i, const float *norm_j,
                   int64_t rows, int64_t cols, float tau_sim, uint16_t *packed_out,
                   int32_t *n_similar, int32_t *n_out_of_range, void *stream);

/*
 * Description of one MoE layer.  Host struct; the small tables are copied at create time,
 * the weight tensors are referenced, not copied.
 */
typedef struct pzl_layer_desc {
    int32_t n_experts;              /* E routed experts = 2 * n_pairs + n_dense */
    int32_t d_model;                /* d, multiple of 32 */
    int32_t d_ffn;                  /* f of the routed experts, multiple of 32 */
    const int32_t *expert_pair;     /* host [E]: pair index in [0, n_pairs) for a merged expert,
                                       or -1-j for routed expert j kept unmerged (the paper's
                                       25 % compression setting merges only half of the experts,
                                       Sec. 4.1)                                              */
    const uint8_t *expert_pos;      /* host [E]: position 0|1 inside the pair (0 for unmerged);
                                       every (pair, position) and every unmerged index must be
                                       named exactly once (pair-wise grouping, Sec. 3.2)      */
    const uint16_t *const *gate;    /* host [n_pairs] of device ptrs, packed [d_ffn, d_model] */
    const uint16_t *const *up;      /* host [n_pairs] of device ptrs, packed [d_ffn, d_model] */
    const uint16_t *const *down;    /* host [n_pairs] of device ptrs, packed [d_model, d_ffn] */
    int32_t n_shared;               /* dense experts applied to every token with weight 1 */
    const int32_t *shared_d_ffn;    /* host [n_shared], each a multiple of 32             */
    const uint16_t *const *shared_gate;   /* host [n_shared] of device ptrs, tiled dense  */
    const uint16_t *const *shared_up;     /*   bf16 [fs, d_model] (pzl_tile_dense)        */
    const uint16_t *const *shared_down;   /*   bf16 [d_model, fs]                         */
    int32_t n_dense;                /* routed experts kept unmerged (0 at 50 % compression) */
    const uint16_t *const *dense_gate;    /* host [n_dense] of device ptrs, tiled dense   */
    const uint16_t *const *dense_up;      /*   bf16 [d_ffn, d_model] (pzl_tile_dense)     */
    const uint16_t *const *dense_down;    /*   bf16 [d_model, d_ffn]                      */
    int32_t pair_format;            /* 0: 16-bit packed words (pzl_pack / pzl_merge_pack);
                                       1: quantised records (pzl_q_pack): gate/up/down then point
                                       to the record arrays and the three tables below to the
                                       scale arrays; d_model and d_ffn must be multiples of 128 */
    const uint16_t *const *gate_scale;    /* host [n_pairs] of device ptrs, or NULL (format 0) */
    const uint16_t *const *up_scale;
    const uint16_t *const *down_scale;
    int32_t h_precision;            /* form of the SwiGLU output H of the packed pairs (format 0) and of the shared experts:
                                       0: automatic -- one plane of IEEE half precision if no used
                                          element of any down matrix has an exponent field above 29
                                          (|w| < 2^15; pzl_layer_create scans them), else as 1
                                          (shared experts: see pzl_moe_ffn);
                                       1: always two bf16 planes (hi + lo, about 16 significant bits,
                                          bf16's range): twice the matrix work in the down stage   */
} pzl_layer_desc;

typedef struct pzl_layer pzl_layer;

/* Validates the description and builds the layer's device tables (the only allocation the
 * library performs; it also sets the kernels' launch attributes and looks up the static scratch
 * array of pzl_moe_ffn_static).  The device current at the call is the layer's device.  The layer also
 * owns up to two further streams (default priority) with two events each: pzl_moe_ffn runs the
 * shared experts on one and, for batches that use both kinds of kernel, the tiled kernels of
 * the routed experts on the other, next to the rest of the call, forked from and joined back
 * into the caller's stream inside the call.  Calls on one layer must therefore not overlap in
 * time on different streams (calls queued on one stream are fine). */
int pzl_layer_create(const pzl_layer_desc *desc, pzl_layer **out);
void pzl_layer_destroy(pzl_layer *layer);
/* Which form of H the layer's packed pairs use (*half_precision = 1: one half-precision plane) and
 * how many wavefronts have saturated a value of H to +-65504 since the layer was created (a
 * blocking copy from the device; 0 in any sane model: |silu(g) * u| would have to exceed 65504).
 * Either pointer may be NULL.  Host pointers. */
int pzl_layer_h_info(const pzl_layer *layer, int32_t *half_precision, int32_t *saturated);

/*
 * moe_ffn_plan — what pzl_moe_ffn decides on the host for a layer of this shape and a batch of T
 * tokens with k choices each (the decode-GEMM of Sec. 3.3.2 runs as weight-streaming kernels for
 * small batches and as tiled matrix-core kernels for large ones; the host knows the batch shape,
 * the device the routing).  Pure host arithmetic: no layer, no device and no stream is needed, so
 * a caller can inspect, and a test can check, the launch plan of any shape.  Host pointers.
 */
typedef struct pzl_layer_shape {
    int32_t n_experts;            /* routed experts, 1..256 */
    int32_t n_unmerged;           /* of which kept unmerged (n_experts - n_unmerged is even) */
    int32_t d_model, d_ffn;       /* multiples of 32 */
    int32_t n_shared;             /* 0..16 */
    const int32_t *shared_d_ffn;  /* [n_shared] multiples of 32 */
    int32_t pair_format;          /* 0: 16-bit packed words, 1: quantised records */
} pzl_layer_shape;

typedef struct pzl_plan {
    int32_t shared_stream;        /* shared experts run on the layer's second stream */
    int32_t hybrid;               /* tiled kernels are launched next to the streaming ones */
    int32_t tile_min;             /* hybrid: a pair with an expert of this many tokens is tiled; else 0 */
    int32_t persistent;           /* the routed tiled launches draw their tiles (256 workgroups) */
    int32_t tile_stream;          /* ... and run on the layer's third stream */
    int32_t ksplit;               /* K splits of the routed down stage (partial sums per slot) */
    int32_t ksplit_shared;        /* ... of the shared experts' down stage */
    int32_t tiled_shared;         /* shared experts run on the tiled kernels */
    int32_t sweep_wgs_packed;     /* streaming kernels: workgroups per (pair, row block) sharing its sweeps */
    int32_t sweep_wgs_unmerged;   /* ... per unmerged expert */
    int32_t shared_token_tiles[16];   /* tiled_shared: token tiles per shared expert ... */
    int32_t shared_tile_tokens[16];   /* ... and tokens per tile (a multiple of 16, at most 288) */
    int32_t grouping_in_kernel;   /* small streaming-only batches: no grouping kernel is launched, the gate/up
                                     kernel of the packed pairs groups the (token, choice) list itself */
} pzl_plan;

/* Returns PZL_OK, or PZL_EINVAL for a null pointer, a negative T or k, or a shape that
 * pzl_layer_create would reject. */
int pzl_moe_ffn_plan(const pzl_layer_shape *shape, int32_t T, int32_t k, pzl_plan *out);

/* For measurement: overrides, for every later call on this layer, three of the decisions that
 * pzl_moe_ffn_plan reports (hybrid, persistent, tile_stream): 1 or 0 forces the decision, -1 leaves
 * it to the library (the state of a new layer).  Every combination computes the same y; what
 * changes is which kernels run (Sec. 3.3.2's decode-GEMM as streaming or as tiled kernels) and how
 * they are launched, so a benchmark can time the library's choice against the alternatives on any
 * layer shape.  Call it before pzl_moe_ffn_workspace_bytes: the workspace size follows the plan.
 * hybrid is ignored for quantised layers (they have no tiled kernel).  Not for use while calls on
 * the layer are in flight.  PZL_EINVAL for a null layer or a value outside -1..1. */
int pzl_layer_force_plan(pzl_layer *layer, int32_t hybrid, int32_t persistent, int32_t tile_stream);

/* Bytes of workspace pzl_moe_ffn needs for any T <= max_tokens at this top_k (0 on bad
 * arguments).  The workspace must be 256-byte aligned device memory. */
size_t pzl_moe_ffn_workspace_bytes(const pzl_layer *layer, int32_t max_tokens, int32_t top_k);

/*
 * Where pzl_moe_ffn keeps its routing tables inside the workspace, for inspection after a call (a
 * test that wants to know which token landed in which token tile; a debugger).  Byte offsets from
 * the start of the workspace; every table is int32.  Routing keys: 2 * pair + position for a merged
 * expert, 2 * (n_pairs + j) for unmerged expert j.  Slots are the (token, choice) entries grouped by
 * key.  The layout depends on (layer, T, k) only.  Host pointers; no device work.
 */
typedef struct pzl_workspace_layout {
    int32_t n_keys;             /* routing keys of the layer */
    int32_t max_tiles;          /* capacity of the three tile tables */
    size_t streamed_count;      /* [n_keys]   slots of the key handled by the streaming kernels (0 if its pair is tiled) */
    size_t first_slot;          /* [n_keys+1] first slot of each key */
    size_t slot_token;          /* [T*k]      token of each slot */
    size_t slot_of;             /* [T*k]      slot of flat index t*k+j, -1 for an ignored id */
    size_t tile_key;            /* [max_tiles] key of each token tile of the tiled kernels; bit 30 set:
                                   the tile covers both experts of the pair */
    size_t tile_first_slot;     /* [max_tiles] */
    size_t tile_tokens;         /* [max_tiles] tokens in the tile (n0 | n1 << 16 for a tile that covers a pair) */
    size_t n_tiles;             /* [1]        number of token tiles */
    size_t total;               /* pzl_moe_ffn_workspace_bytes(layer, T, k) */
} pzl_workspace_layout;
int pzl_moe_ffn_workspace_layout(const pzl_layer *layer, int32_t T, int32_t k, pzl_workspace_layout *out);

/*
 * moe_ffn — the routed expert FFN over Eq. 6-decoded weights:
 *   y[t,:] = sum_j topk_w[t,j] * FFN_{topk_ids[t,j]}(x[t,:])  +  sum_s FFN_shared_s(x[t,:])
 *   FFN_e(x) = Wdown_e ( silu(Wgate_e x) * (Wup_e x) ),   silu(g) = g / (1 + exp(-g))
 * with every routed W_e decoded on the fly from its pair's packed tensor (Algorithm 1), or, for a
 * layer in the quantised format, reconstructed on the fly as (-1)^S * M * code * scale (the group
 * scale is applied to the fp32 partial sums of each 128-column group, so code * scale is never
 * rounded).  Quantised layers always take the weight-streaming kernels, which serve 32 tokens of an
 * expert per sweep of its pair's weights: a call with more than 64 (token, choice) entries per
 * expert on average (T * k > 64 * n_experts) is refused with PZL_EINVAL (split the batch, or keep
 * layers that see prefill-sized batches in the 16-bit format).
 * Products are accumulated in fp32 and y is rounded to bf16 once at the end.  Between the two
 * contractions the SwiGLU output h needs more than bf16's 8 significant bits to keep y within 1e-2:
 * packed pairs keep it as one IEEE half-precision number (11 bits; the down projection then decodes
 * its weights to half precision, exactly, and runs on the f16 matrix instruction; |h| beyond 65504
 * saturates and is counted, |h| below 6e-5 keeps an absolute precision of 3e-8), or, where a down
 * matrix holds weights of 2^15 and more or the layer asks for it (h_precision), as two bf16 numbers
 * (hi = bf16(h), lo = bf16(h - hi)) that the down projection both multiplies, as unmerged and
 * quantised experts always do.  Shared experts keep h in half precision too where they run on the
 * tiled kernels (65 tokens and more) unless h_precision asks otherwise or a shared down matrix holds
 * an infinity or a NaN: their bf16 down weights are then decoded to half precision times a power of
 * two chosen from the largest weight of the launch's matrices (weights more than 2^30 below it
 * count as zero), and the sums are scaled back.
 *   x         [T, d_model] bf16 bits, row-major
 *   topk_ids  [T, k] int32 expert ids in [0, E); duplicates within a token add up; ids
 *             outside the range are ignored (contribute nothing)
 *   topk_w    [T, k] fp32 routing weights
 *   y         [T, d_model] bf16 bits, overwritten
 *   workspace at least pzl_moe_ffn_workspace_bytes(layer, T, k) bytes; contents are scratch
 * Size limits of one call (the kernels address activations with 32-bit byte offsets; larger
 * batches are to be split by the caller): T * d_model < 2^31, T * k * d_ffn < 2^30, and for the
 * shared experts n_shared * T * f_shared < 2^30; PZL_EINVAL beyond them.
 * T == 0 is a no-op.  Calls on one layer must not overlap in time on different streams (see
 * pzl_layer_create); calls queued on one stream are fine.
 * Graph capture: the call only enqueues kernels and event record / wait pairs (the fork to and the
 * join from the layer's own streams), allocates nothing, synchronises nothing and clears its
 * counters inside its kernels, so it may be made on a capturing stream; replays are bit-identical
 * to eager calls.  Make one eager call with the same shapes first: the first launch of each kernel
 * sets a function attribute, which is not a stream operation.
 */
int pzl_moe_ffn(const pzl_layer *layer, const uint16_t *x, const int32_t *topk_ids,
                const float *topk_w, int32_t T, int32_t k, uint16_t *y,
                void *workspace, size_t workspace_bytes, void *stream);

/*
 * moe_ffn_static — pzl_moe_ffn for callers that cannot allocate and have no workspace to pass: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs,
 * same outputs, same kernels and the same results bit for bit as pzl_moe_ffn; the workspace is a
 * static array of PZL_STATIC_SCRATCH_BYTES in device memory that belongs to the library (every GPU
 * the library runs on holds its own copy until the process ends; its address on the layer's
 * device is looked up once, in pzl_layer_create).  The call allocates and frees nothing.
 *   - A batch whose workspace (pzl_moe_ffn_workspace_bytes(layer, T, k)) exceeds the array is
 *     refused with PZL_ENOSPC and nothing is launched.  32 MiB hold a Mixtral-8x7B-shaped layer
 *     up to 76 tokens at top-2 (the batches that the streaming kernels serve alone); larger
 *     batches take pzl_moe_ffn with a caller workspace.
 *   - All calls on one GPU share that GPU's array, on whatever layer and stream: calls that
 *     overlap in time on one GPU race.  Calls queued on one stream are fine.  The array keeps the
 *     previous call's contents; the call clears what it needs cleared inside its kernels.
 */
#define PZL_STATIC_SCRATCH_BYTES (32u << 20)
int pzl_moe_ffn_static(const pzl_layer *layer, const uint16_t *x, const int32_t *topk_ids,
                       const float *topk_w, int32_t T, int32_t k, uint16_t *y, void *stream);
/* PZL_STATIC_SCRATCH_BYTES as the loaded library was built with. */
size_t pzl_moe_ffn_static_max_bytes(void);

/*
 * router_topk — the step in front of pzl_moe_ffn, so that a whole MoE block runs on the device.
 * The paper keeps the router as it is in the model ("the other modules unchanged", Sec. 4.1); this
 * is the usual linear router: logits = x W_r^T, the k largest logits per token in descending order
 * (ties: lower expert index first), weights = softmax over those k logits.
 * Each logit is one fp32 fused-multiply-add chain over the channels in order, which makes the
 * chosen experts exactly reproducible.
 *   x         [T, d_model] bf16 bits;  w_router  [n_experts, d_model] bf16 bits, row-major
 *   topk_ids  [T, k] int32 out;        topk_w    [T, k] fp32 out
 * d_model % 8 == 0, n_experts <= 256, k <= min(n_experts, 64).
 */
int pzl_router_topk(const uint16_t *x, const uint16_t *w_router, int32_t T, int32_t d_model,
                    int32_t n_experts, int32_t k, int32_t *topk_ids, float *topk_w, void *stream);

/*
 * Quantised variant of the packed pair (appendix "Combining PuzzleMoE with Quantization": the
 * merged weights quantised uniformly to 3 bits in groups of 128 with a symmetric scheme, stored
 * with the two sign bits and the mask, whose three possible values cost log2(3) bits; the
 * appendix's accounting is (2 + 1.58 + 3 + 0.125) / 2 = 3.35 bits per original weight).
 *
 * The appendix fixes neither a rounding rule nor a storage layout.  This library's readings:
 * codes are unsigned magnitudes 0..7; groups are 128 consecutive columns of one row;
 * scale = bf16(max / 7) over the magnitudes some expert uses, code = min(7, round-to-nearest-even
 * (magnitude / scale)), both divisions correctly rounded in fp32; an element no expert uses is
 * stored as code 0; reconstruction is (-1)^S * M * code * scale with no further rounding.
 * Stored form: per 16x32 tile (same element order as the 16-bit format) 64 records of 53 bits,
 * packed back to back (424 bytes): codes (3 bits x 8 elements), S0 x 8, S1 x 8, and the 8 masks
 * as one base-3 number in 13 bits (digit 0: position 0 only, 1: position 1 only, 2: both); the
 * scales in a separate array [rows/16][cols/128][16] of bf16.  3.375 bits per original weight.
 * rows % 16 == 0 and cols % 128 == 0 are required.
 */
/* Bytes of the record array (includes 8 bytes of padding that the last record's 8-byte load may
 * touch) and of the scale array; 0 for a bad shape. */
size_t pzl_q_record_bytes(int64_t rows, int64_t cols);
size_t pzl_q_scale_bytes(int64_t rows, int64_t cols);
/*
 * q_pack: quantise and store.  Inputs as for pzl_pack (row-major, logical order).
 *   records_out  pzl_q_record_bytes(rows, cols) bytes, 8-byte aligned, caller-owned
 *   scales_out   pzl_q_scale_bytes(rows, cols) bytes, caller-owned
 *   n_non_finite optional int32 on the device; the kernel ADDS the number of used elements whose
 *                magnitude is Inf/NaN (stored as code 0).  May be NULL.
 */
int pzl_q_pack(const uint16_t *merged, const uint8_t *mask0, const uint8_t *mask1,
               const uint8_t *sign0, const uint8_t *sign1, int64_t rows, int64_t cols,
               uint8_t *records_out, uint16_t *scales_out, int32_t *n_non_finite, void *stream);
/*
 * q_unpack: the reconstructed weights of the expert at `expert_pos` (0 or 1) as fp32, row-major
 * [rows, cols]; code * scale is exact in fp32, so this is bit-exact by definition.
 */
int pzl_q_unpack(const uint8_t *records, const uint16_t *scales, int expert_pos, int64_t rows,
                 int64_t cols, float *out, void *stream);

/*
 * Measurement variant of pzl_moe_ffn: the same launches on the same stream, and in addition the
 * caller's hipEvent_t handles are recorded around each stage, so that a benchmark can time one
 * kernel of the path with events on the stream the kernel really runs on.
 *   stage_events  host array of 2*PZL_N_STAGES hipEvent_t (as void*), created by the caller
 *                 with timing enabled; [2*s] is recorded before and [2*s+1] after stage s.
 *                 NULL entries are skipped; a NULL array makes the call identical to
 *                 pzl_moe_ffn.
 * Stages: the token grouping, the routed gate/up decode-GEMM with SwiGLU (the kernel the
 * decode-time roofline is quoted on), the routed down decode-GEMM, all shared-expert work,
 * and the weighted combine.
 */
#define PZL_STAGE_ROUTE   0
#define PZL_STAGE_GATEUP  1
#define PZL_STAGE_DOWN    2
#define PZL_STAGE_SHARED  3
#define PZL_STAGE_COMBINE 4
#define PZL_N_STAGES      5
int pzl_moe_ffn_staged(const pzl_layer *layer, const uint16_t *x, const int32_t *topk_ids,
                       const float *topk_w, int32_t T, int32_t k, uint16_t *y,
                       void *workspace, size_t workspace_bytes, void *stream,
                       void *const *stage_events);

#ifdef __cplusplus
}
#endif
#endif /* PUZZLE_MOE_H */
