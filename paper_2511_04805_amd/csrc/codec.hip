// pack / unpack / tile_dense: element-wise codec kernels (HBM-bound, offline or test use).
// pack: Sec. 3.3.2 exponent clamp-and-shift + flag bits; unpack: Algorithm 1.
#include "pzl_common.h"

namespace pzl {

// One thread owns one lane-chunk of a tile: 8 consecutive columns of one row.
__device__ __forceinline__ void chunk_coords(int64_t chunk, int64_t col_tiles, int64_t &row, int64_t &col)
{
    int64_t tile = chunk >> 6;
    int lane = (int)(chunk & 63);
    int64_t rt = tile / col_tiles, kb = tile - rt * col_tiles;
    row = rt * TILE_ROWS + (lane & 15);
    col = kb * TILE_COLS + (lane >> 4) * 8;
}

__global__ void __launch_bounds__(256)
pack_kernel(const uint16_t *__restrict__ merged, const uint8_t *__restrict__ m0,
            const uint8_t *__restrict__ m1, const uint8_t *__restrict__ s0,
            const uint8_t *__restrict__ s1, int64_t rows, int64_t cols,
            uint16_t *__restrict__ out, int32_t *__restrict__ n_bad)
{
    int64_t n_chunks = rows * cols / 8;
    int64_t chunk = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (chunk >= n_chunks) return;
    int64_t row, col;
    chunk_coords(chunk, cols / TILE_COLS, row, col);
    int64_t src = row * cols + col;
    u32x4 w = *(const u32x4 *)(merged + src);
    u32x2 vm0 = *(const u32x2 *)(m0 + src), vm1 = *(const u32x2 *)(m1 + src);
    u32x2 vs0 = *(const u32x2 *)(s0 + src), vs1 = *(const u32x2 *)(s1 + src);
    uint32_t res[4];
    int bad = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        uint32_t mag = (w[i >> 1] >> ((i & 1) * 16)) & 0x7FFFu;     // input sign ignored
        uint32_t fm0 = (vm0[i >> 2] >> ((i & 3) * 8)) & 0xFFu, fm1 = (vm1[i >> 2] >> ((i & 3) * 8)) & 0xFFu;
        uint32_t fs0 = (vs0[i >> 2] >> ((i & 3) * 8)) & 0xFFu, fs1 = (vs1[i >> 2] >> ((i & 3) * 8)) & 0xFFu;
        uint32_t exponent = mag >> 7, mantissa = mag & 0x7Fu;
        uint32_t flags = (fs0 ? 0x8000u : 0u) | (fs1 ? 0x4000u : 0u);
        uint32_t word;
        if (exponent > 143u) {            // does not fit five bits: fully masked, counted
            ++bad;
            word = flags;
        } else if (mag == 0u) {           // exact zero: fully masked so that Eq. 6 gives 0
            word = flags;
        } else {
            if (exponent < 112u) exponent = 112u;                   // raised, mantissa kept
            word = flags | (fm0 ? 0x2000u : 0u) | (fm1 ? 0x1000u : 0u) | ((exponent - 112u) << 7) | mantissa;
        }
        if (i & 1) res[i >> 1] |= word << 16; else res[i >> 1] = word;
    }
    u32x4 o = {res[0], res[1], res[2], res[3]};
    *(u32x4 *)(out + chunk * 8) = o;
    if (bad && n_bad) atomicAdd(n_bad, bad);
}

__device__ __forceinline__ uint32_t decode16(uint32_t W, int pos)
{
    // Algorithm 1, one element.
    uint32_t mask_bit = (W >> (13 - pos)) & 1u;
    if (mask_bit == 0u) return 0u;
    uint32_t sign_bit = (W >> (15 - pos)) & 1u;
    uint32_t exp_field = (W & 0x0F80u) + (112u << 7);
    return (sign_bit << 15) | exp_field | (W & 0x007Fu);
}

__global__ void __launch_bounds__(256)
unpack_kernel(const uint16_t *__restrict__ packed, int pos, int64_t rows, int64_t cols,
              uint16_t *__restrict__ out)
{
    int64_t n_chunks = rows * cols / 8;
    int64_t chunk = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (chunk >= n_chunks) return;
    int64_t row, col;
    chunk_coords(chunk, cols / TILE_COLS, row, col);
    u32x4 w = *(const u32x4 *)(packed + chunk * 8);
    u32x4 o;
#pragma unroll
    for (int i = 0; i < 4; ++i)
        o[i] = decode16(w[i] & 0xFFFFu, pos) | (decode16(w[i] >> 16, pos) << 16);
    *(u32x4 *)(out + row * cols + col) = o;
}

__global__ void __launch_bounds__(256)
tile_dense_kernel(const uint16_t *__restrict__ in, int64_t rows, int64_t cols, uint16_t *__restrict__ out)
{
    int64_t n_chunks = rows * cols / 8;
    int64_t chunk = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (chunk >= n_chunks) return;
    int64_t row, col;
    chunk_coords(chunk, cols / TILE_COLS, row, col);
    *(u32x4 *)(out + chunk * 8) = *(const u32x4 *)(in + row * cols + col);
}

static bool shape_ok(int64_t rows, int64_t cols)
{
    return rows > 0 && cols > 0 && rows % TILE_ROWS == 0 && cols % TILE_COLS == 0 &&
           rows * cols / 8 / 256 < 0x7FFFFFFFLL;
}

static int finish_launch()
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_hip_error(e); return PZL_EHIP; }
    return PZL_OK;
}

int launch_pack(const uint16_t *merged, const uint8_t *m0, const uint8_t *m1, const uint8_t *s0,
                const uint8_t *s1, int64_t rows, int64_t cols, uint16_t *out, int32_t *n_bad,
                hipStream_t st)
{
    if (!merged || !m0 || !m1 || !s0 || !s1 || !out || !shape_ok(rows, cols)) return PZL_EINVAL;
    int64_t n_chunks = rows * cols / 8;
    unsigned blocks = (unsigned)((n_chunks + 255) / 256);
    hipLaunchKernelGGL(pack_kernel, dim3(blocks), dim3(256), 0, st, merged, m0, m1, s0, s1, rows, cols, out, n_bad);
    return finish_launch();
}

int launch_unpack(const uint16_t *packed, int pos, int64_t rows, int64_t cols, uint16_t *out, hipStream_t st)
{
    if (!packed || !out || (pos != 0 && pos != 1) || !shape_ok(rows, cols)) return PZL_EINVAL;
    int64_t n_chunks = rows * cols / 8;
    unsigned blocks = (unsigned)((n_chunks + 255) / 256);
    hipLaunchKernelGGL(unpack_kernel, dim3(blocks), dim3(256), 0, st, packed, pos, rows, cols, out);
    return finish_launch();
}

int launch_tile_dense(const uint16_t *in, int64_t rows, int64_t cols, uint16_t *out, hipStream_t st)
{
    if (!in || !out || !shape_ok(rows, cols)) return PZL_EINVAL;
    int64_t n_chunks = rows * cols / 8;
    unsigned blocks = (unsigned)((n_chunks + 255) / 256);
    hipLaunchKernelGGL(tile_dense_kernel, dim3(blocks), dim3(256), 0, st, in, rows, cols, out);
    return finish_launch();
}

}  // namespace pzl
