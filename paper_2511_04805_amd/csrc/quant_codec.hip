// Codec of the quantised variant (appendix "Combining PuzzleMoE with Quantization"): the merged
// magnitudes as 3-bit codes with one bf16 scale per 128 columns of a row, the two sign bits, and
// the mask as a base-3 digit (an element belongs to expert 0, to expert 1 or to both).
//
// Stored form (this library's; the appendix gives only the bit accounting).  A 16x32 tile is 64
// records of 53 bits, record l for row l%16 and columns (l/16)*8..+7 of the tile -- the element
// order of a matrix-core A operand, as in the 16-bit format -- packed back to back:
//     bits 0..23  codes (element e at 3e)     24..31  S0 bits     32..39  S1 bits
//     bits 40..52 sum_e digit_e 3^e  (digit 0: expert 0 only, 1: expert 1 only, 2: both)
// so a tile is 424 bytes and lane l finds its record with one unaligned 8-byte load at byte
// 53*l/8, shifted right by 53*l%8.  Tiles follow each other in [row tile][k-block] order; the
// scales are a separate array [row tile][group of 128 columns][16 rows].  (2 + 13/8 + 3) bits per
// element position plus 16/128 for the scale: 3.375 bits per original weight.
#include "pzl_common.h"

namespace pzl {

constexpr int Q_GROUP = 128;              // columns per scale
constexpr int Q_TILE_BYTES = 424;         // 64 records x 53 bits
constexpr int Q_TILE_WORDS = Q_TILE_BYTES / 4;

__device__ __forceinline__ uint32_t q_bf16_rne(float v)
{
    uint32_t u = __float_as_uint(v);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0u;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

// One workgroup per (row tile, group of 128 columns): 4 k-blocks x 64 records.
__global__ void __launch_bounds__(256)
q_pack_kernel(const uint16_t *merged, const uint8_t *m0, const uint8_t *m1, const uint8_t *s0,
              const uint8_t *s1, int64_t rows, int64_t cols, uint8_t *records, uint16_t *scales,
              int32_t *n_bad)
{
    __shared__ uint32_t row_max[TILE_ROWS];
    __shared__ uint32_t bits[4][Q_TILE_WORDS];
    const int tid = threadIdx.x, kbl = tid >> 6, lane = tid & 63;
    const int64_t groups = cols / Q_GROUP, kb_total = cols / TILE_COLS;
    const int64_t rt = blockIdx.x / groups, g = blockIdx.x % groups;
    const int row = lane & 15;
    const int64_t kb = g * 4 + kbl;
    const int64_t e0 = (rt * TILE_ROWS + row) * cols + kb * TILE_COLS + (lane >> 4) * 8;

    if (tid < TILE_ROWS) row_max[tid] = 0u;
    for (int i = tid; i < 4 * Q_TILE_WORDS; i += 256) (&bits[0][0])[i] = 0u;
    __syncthreads();

    // the 8 elements of this record
    u32x4 mw = *(const u32x4 *)(merged + e0);
    u32x2 a0 = *(const u32x2 *)(m0 + e0), a1 = *(const u32x2 *)(m1 + e0);
    u32x2 b0 = *(const u32x2 *)(s0 + e0), b1 = *(const u32x2 *)(s1 + e0);
    float mag[8];
    bool k0[8], k1[8], n0[8], n1[8];
    uint32_t local_max = 0u;
    int bad = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        uint32_t h = (mw[e >> 1] >> (16 * (e & 1))) & 0x7FFFu;          // sign of the input ignored
        k0[e] = ((a0[e >> 2] >> (8 * (e & 3))) & 0xFFu) != 0;
        k1[e] = ((a1[e >> 2] >> (8 * (e & 3))) & 0xFFu) != 0;
        n0[e] = ((b0[e >> 2] >> (8 * (e & 3))) & 0xFFu) != 0;
        n1[e] = ((b1[e >> 2] >> (8 * (e & 3))) & 0xFFu) != 0;
        const bool used = k0[e] || k1[e];
        const bool finite = h < 0x7F80u;
        mag[e] = __uint_as_float(h << 16);
        if (used && !finite) ++bad;
        if (used && finite) local_max = max(local_max, h << 16);         // non-negative floats order as integers
    }
    atomicMax(&row_max[row], local_max);
    if (bad && n_bad) atomicAdd(n_bad, bad);
    __syncthreads();

    // scale = bf16(max / 7), one correctly rounded fp32 division
    const float mx = __uint_as_float(row_max[row]);
    const uint32_t sc_bits = q_bf16_rne(__fdiv_rn(mx, 7.0f));
    const float sc = __uint_as_float(sc_bits << 16);
    if (kbl == 0 && lane < TILE_ROWS) scales[(rt * groups + g) * TILE_ROWS + row] = (uint16_t)sc_bits;

    uint64_t rec = 0, digits = 0, p3 = 1;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const bool used = k0[e] || k1[e];
        const bool finite = __float_as_uint(mag[e]) < 0x7F800000u;
        uint32_t q = 0;
        if (used && finite && sc > 0.0f) {
            float rq = rintf(__fdiv_rn(mag[e], sc));                     // nearest integer, ties to even
            q = rq > 7.0f ? 7u : (uint32_t)rq;
        }
        const uint32_t digit = (k0[e] && k1[e]) ? 2u : (k1[e] ? 1u : (k0[e] ? 0u : 2u));
        rec |= (uint64_t)q << (3 * e);
        rec |= (uint64_t)(n0[e] ? 1u : 0u) << (24 + e);
        rec |= (uint64_t)(n1[e] ? 1u : 0u) << (32 + e);
        digits += digit * p3;
        p3 *= 3;
    }
    rec |= digits << 40;

    // 53 bits at bit offset 53*lane of this k-block's tile
    const int bo = 53 * lane, w = bo >> 5, sh = bo & 31;
    atomicOr(&bits[kbl][w], (uint32_t)(rec << sh));
    atomicOr(&bits[kbl][w + 1], (uint32_t)(sh ? (rec >> (32 - sh)) : (rec >> 32)));
    if (sh + 53 > 64) atomicOr(&bits[kbl][w + 2], (uint32_t)(rec >> (64 - sh)));
    __syncthreads();

    uint32_t *dst = (uint32_t *)(records + (rt * kb_total + g * 4) * Q_TILE_BYTES);   // 4 tiles, contiguous
    for (int i = tid; i < 4 * Q_TILE_WORDS; i += 256) dst[i] = (&bits[0][0])[i];
}

// One thread per record: out[r, c..c+7] = (-1)^S * M * code * scale as fp32 (exact: 3 x 8 bits).
__global__ void __launch_bounds__(256)
q_unpack_kernel(const uint8_t *records, const uint16_t *scales, int pos, int64_t rows, int64_t cols, float *out)
{
    const int64_t rec_id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t n_rec = rows * cols / 8;
    if (rec_id >= n_rec) return;
    const int64_t tile = rec_id >> 6;
    const int lane = (int)(rec_id & 63);
    const int64_t kb_total = cols / TILE_COLS, groups = cols / Q_GROUP;
    const int64_t rt = tile / kb_total, kb = tile % kb_total;
    const uint8_t *p = records + tile * Q_TILE_BYTES + ((53 * lane) >> 3);
    uint64_t v = 0;
#pragma unroll
    for (int b = 0; b < 8; ++b) v |= (uint64_t)p[b] << (8 * b);
    v >>= (53 * lane) & 7;
    const uint32_t codes = (uint32_t)v & 0xFFFFFFu;
    const uint32_t sg = (uint32_t)(v >> (pos ? 32 : 24)) & 0xFFu;
    uint32_t t = (uint32_t)(v >> 40) & 0x1FFFu;
    const int row = lane & 15;
    const float sc = __uint_as_float((uint32_t)scales[(rt * groups + kb / 4) * TILE_ROWS + row] << 16);
    float *dst = out + (rt * TILE_ROWS + row) * cols + kb * TILE_COLS + (lane >> 4) * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const uint32_t digit = t % 3u;
        t /= 3u;
        const bool keep = digit == 2u || digit == (uint32_t)pos;
        float val = (float)((codes >> (3 * e)) & 7u) * sc;
        if ((sg >> e) & 1u) val = -val;
        dst[e] = keep ? val : 0.0f;
    }
}

static bool q_shape_ok(int64_t rows, int64_t cols)
{
    return rows > 0 && cols > 0 && rows % TILE_ROWS == 0 && cols % Q_GROUP == 0 &&
           rows * cols / 8 / 256 < 0x7FFFFFFFLL;
}

size_t q_record_bytes(int64_t rows, int64_t cols)
{
    if (!q_shape_ok(rows, cols)) return 0;
    return (size_t)(rows / TILE_ROWS) * (size_t)(cols / TILE_COLS) * Q_TILE_BYTES + 8;   // + the last record's load
}

size_t q_scale_bytes(int64_t rows, int64_t cols)
{
    if (!q_shape_ok(rows, cols)) return 0;
    return (size_t)rows * (size_t)(cols / Q_GROUP) * 2;
}

int launch_q_pack(const uint16_t *merged, const uint8_t *m0, const uint8_t *m1, const uint8_t *s0,
                  const uint8_t *s1, int64_t rows, int64_t cols, uint8_t *records, uint16_t *scales,
                  int32_t *n_bad, hipStream_t st)
{
    if (!merged || !m0 || !m1 || !s0 || !s1 || !records || !scales || !q_shape_ok(rows, cols)) return PZL_EINVAL;
    const int64_t blocks = (rows / TILE_ROWS) * (cols / Q_GROUP);
    if (blocks > 0x7FFFFFFFLL) return PZL_EINVAL;
    hipLaunchKernelGGL(q_pack_kernel, dim3((unsigned)blocks), dim3(256), 0, st, merged, m0, m1, s0, s1,
                       rows, cols, records, scales, n_bad);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_hip_error(e); return PZL_EHIP; }
    return PZL_OK;
}

int launch_q_unpack(const uint8_t *records, const uint16_t *scales, int pos, int64_t rows, int64_t cols,
                    float *out, hipStream_t st)
{
    if (!records || !scales || !out || (pos != 0 && pos != 1) || !q_shape_ok(rows, cols)) return PZL_EINVAL;
    const int64_t n_rec = rows * cols / 8;
    hipLaunchKernelGGL(q_unpack_kernel, dim3((unsigned)((n_rec + 255) / 256)), dim3(256), 0, st,
                       records, scales, pos, rows, cols, out);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_hip_error(e); return PZL_EHIP; }
    return PZL_OK;
}

}  // namespace pzl
