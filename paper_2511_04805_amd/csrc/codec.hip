// pack / unpack / tile_dense: element-wise codec kernels (HBM-bound, offline or test use).
// pack: Sec. 3.3.2 exponent clamp-and-shift + flag bits; unpack: Algorithm 1 (pzl_decode.h).
#include "pzl_common.h"
#include "pzl_decode.h"

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

// Sec. 3.3.2 word for one element: exponent raised to >= 112 and shifted by -112, flags on top.
__device__ __forceinline__ uint32_t pack_word(uint32_t mag, uint32_t m0, uint32_t m1, uint32_t s0, uint32_t s1, int &bad)
{
    uint32_t exponent = mag >> 7, mantissa = mag & 0x7Fu;
    uint32_t flags = (s0 ? 0x8000u : 0u) | (s1 ? 0x4000u : 0u);
    if (exponent > 143u) { ++bad; return flags; }      // does not fit five bits: fully masked, counted
    if (mag == 0u) return flags;                        // exact zero: fully masked so that Eq. 6 gives 0
    if (exponent < 112u) exponent = 112u;               // raised, mantissa kept
    return flags | (m0 ? 0x2000u : 0u) | (m1 ? 0x1000u : 0u) | ((exponent - 112u) << 7) | mantissa;
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
        uint32_t word = pack_word(mag, fm0, fm1, fs0, fs1, bad);
        if (i & 1) res[i >> 1] |= word << 16; else res[i >> 1] = word;
    }
    u32x4 o = {res[0], res[1], res[2], res[3]};
    *(u32x4 *)(out + chunk * 8) = o;
    if (bad && n_bad) atomicAdd(n_bad, bad);
}

__device__ __forceinline__ uint32_t f32_to_bf16_rne_codec(float v)
{
    uint32_t u = __float_as_uint(v);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

// Offline dual-mask merge of two experts (Sec. 3.2, Eqs. 1-5) fused with pack: reads the two bf16
// matrices and the per-input-channel activation norms, writes the packed pair (tiled order).
// Mask decisions are fp32 comparisons, one rounding per operation:
//   similar:  | |wi|-|wj| | <= tau * (|wi|+|wj|), and not both zero   (the paper's ratio test,
//             written without the division);
//   salient:  |wi| * norm_i[c] >= |wj| * norm_j[c] keeps expert i (ties to i, Eq. 3).
__global__ void __launch_bounds__(256)
merge_pack_kernel(const uint16_t *__restrict__ wi, const uint16_t *__restrict__ wj,
                  const float *__restrict__ norm_i, const float *__restrict__ norm_j, int64_t rows,
                  int64_t cols, float tau, uint16_t *__restrict__ out, int32_t *__restrict__ n_similar,
                  int32_t *__restrict__ n_bad)
{
    int64_t n_chunks = rows * cols / 8;
    int64_t chunk = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (chunk >= n_chunks) return;
    int64_t row, col;
    chunk_coords(chunk, cols / TILE_COLS, row, col);
    int64_t src = row * cols + col;
    u32x4 vi = *(const u32x4 *)(wi + src), vj = *(const u32x4 *)(wj + src);
    f32x4 ni0 = *(const f32x4 *)(norm_i + col), ni1 = *(const f32x4 *)(norm_i + col + 4);
    f32x4 nj0 = *(const f32x4 *)(norm_j + col), nj1 = *(const f32x4 *)(norm_j + col + 4);
    uint32_t res[4];
    int bad = 0, sim_count = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        uint32_t bi = (vi[i >> 1] >> ((i & 1) * 16)) & 0xFFFFu, bj = (vj[i >> 1] >> ((i & 1) * 16)) & 0xFFFFu;
        float a = __uint_as_float((bi & 0x7FFFu) << 16), b = __uint_as_float((bj & 0x7FFFu) << 16);
        float cn_i = (i < 4) ? ni0[i & 3] : ni1[i & 3], cn_j = (i < 4) ? nj0[i & 3] : nj1[i & 3];
        float diff = fabsf(__fsub_rn(a, b));
        float sum = __fadd_rn(a, b);
        float thr = __fmul_rn(tau, sum);
        bool sim = (sum > 0.0f) && (diff <= thr);
        bool pick_i = __fmul_rn(a, cn_i) >= __fmul_rn(b, cn_j);
        float mag = sim ? __fmul_rn(sum, 0.5f) : (pick_i ? a : b);
        uint32_t s_i = (bi & 0x8000u) && (bi & 0x7FFFu), s_j = (bj & 0x8000u) && (bj & 0x7FFFu);
        uint32_t word = pack_word(f32_to_bf16_rne_codec(mag), sim || pick_i, sim || !pick_i, s_i, s_j, bad);
        sim_count += sim;
        if (i & 1) res[i >> 1] |= word << 16; else res[i >> 1] = word;
    }
    u32x4 o = {res[0], res[1], res[2], res[3]};
    *(u32x4 *)(out + chunk * 8) = o;
    if (n_similar) {
        // one atomic per wavefront
        for (int off = 32; off > 0; off >>= 1) sim_count += __shfl_down(sim_count, off);
        if ((threadIdx.x & 63) == 0 && sim_count) atomicAdd(n_similar, sim_count);
    }
    if (bad && n_bad) atomicAdd(n_bad, bad);
}

// unpack: the library's one decode routine (pzl_decode.h), written out to memory.
// HALFW: the half-precision form of the decode (each weight times 2), as the down stage of a
// layer with half-precision H runs it.
template <int POS, bool HALFW>
__global__ void __launch_bounds__(256)
unpack_kernel(const uint16_t *__restrict__ packed, int64_t rows, int64_t cols, uint16_t *__restrict__ out)
{
    int64_t n_chunks = rows * cols / 8;
    int64_t chunk = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (chunk >= n_chunks) return;
    int64_t row, col;
    chunk_coords(chunk, cols / TILE_COLS, row, col);
    u32x4 w = *(const u32x4 *)(packed + chunk * 8);
    u32x4 o;
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = decode_pair<POS>(w[i], HALFW ? decode_body_half_x2(w[i]) : decode_body(w[i]));
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

// Largest stored exponent field (0..31) among the words that at least one expert uses, added to
// *max_out by atomicMax.  pzl_layer_create runs it over the down matrices: a tensor whose largest
// field is at most 29 can be decoded to half precision (pzl_decode.h).
__global__ void __launch_bounds__(256)
max_exp_field_kernel(const uint16_t *__restrict__ packed, int64_t n_chunks, int32_t *__restrict__ max_out)
{
    uint32_t mx = 0;
    for (int64_t chunk = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; chunk < n_chunks; chunk += (int64_t)gridDim.x * blockDim.x) {
        u32x4 w = *(const u32x4 *)(packed + chunk * 8);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t lo = w[i] & 0xFFFFu, hi = w[i] >> 16;
            if (lo & 0x3000u) mx = max(mx, (lo >> 7) & 31u);
            if (hi & 0x3000u) mx = max(mx, (hi >> 7) & 31u);
        }
    }
    for (int off = 32; off > 0; off >>= 1) mx = max(mx, (uint32_t)__shfl_down((int)mx, off));
    if ((threadIdx.x & 63) == 0 && mx) atomicMax(max_out, (int32_t)mx);
}

// Largest bf16 exponent field among the non-zero elements of a dense matrix (any element order):
// what decides whether, and with which scale, its weights can be decoded to half precision.
__global__ void __launch_bounds__(256)
max_exp_bf16_kernel(const uint16_t *__restrict__ w, int64_t n_chunks, int32_t *__restrict__ max_out)
{
    uint32_t mx = 0;
    for (int64_t chunk = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; chunk < n_chunks; chunk += (int64_t)gridDim.x * blockDim.x) {
        u32x4 v = *(const u32x4 *)(w + chunk * 8);
#pragma unroll
        for (int i = 0; i < 4; ++i) mx = max(mx, max((v[i] >> 7) & 255u, (v[i] >> 23) & 255u));
    }
    for (int off = 32; off > 0; off >>= 1) mx = max(mx, (uint32_t)__shfl_down((int)mx, off));
    if ((threadIdx.x & 63) == 0 && mx) atomicMax(max_out, (int32_t)mx);
}

int launch_max_exp_bf16(const uint16_t *w, int64_t n_elems, int32_t *max_out, hipStream_t st)
{
    if (!w || !max_out || n_elems <= 0 || n_elems % 8) return PZL_EINVAL;
    hipLaunchKernelGGL(max_exp_bf16_kernel, dim3(1024), dim3(256), 0, st, w, n_elems / 8, max_out);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_hip_error(e); return PZL_EHIP; }
    return PZL_OK;
}

int launch_max_exp_field(const uint16_t *packed, int64_t rows, int64_t cols, int32_t *max_out, hipStream_t st)
{
    if (!packed || !max_out || rows <= 0 || cols <= 0 || (rows * cols) % 8) return PZL_EINVAL;
    hipLaunchKernelGGL(max_exp_field_kernel, dim3(2048), dim3(256), 0, st, packed, rows * cols / 8, max_out);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_hip_error(e); return PZL_EHIP; }
    return PZL_OK;
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

int launch_unpack(const uint16_t *packed, int pos, int64_t rows, int64_t cols, uint16_t *out, bool half_x2, hipStream_t st)
{
    if (!packed || !out || (pos != 0 && pos != 1) || !shape_ok(rows, cols)) return PZL_EINVAL;
    int64_t n_chunks = rows * cols / 8;
    unsigned blocks = (unsigned)((n_chunks + 255) / 256);
    if (half_x2) {
        if (pos == 0) hipLaunchKernelGGL((unpack_kernel<0, true>), dim3(blocks), dim3(256), 0, st, packed, rows, cols, out);
        else          hipLaunchKernelGGL((unpack_kernel<1, true>), dim3(blocks), dim3(256), 0, st, packed, rows, cols, out);
    } else {
        if (pos == 0) hipLaunchKernelGGL((unpack_kernel<0, false>), dim3(blocks), dim3(256), 0, st, packed, rows, cols, out);
        else          hipLaunchKernelGGL((unpack_kernel<1, false>), dim3(blocks), dim3(256), 0, st, packed, rows, cols, out);
    }
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

int launch_merge_pack(const uint16_t *wi, const uint16_t *wj, const float *norm_i, const float *norm_j,
                      int64_t rows, int64_t cols, float tau, uint16_t *out, int32_t *n_similar,
                      int32_t *n_bad, hipStream_t st)
{
    if (!wi || !wj || !norm_i || !norm_j || !out || !shape_ok(rows, cols) || !(tau >= 0.0f && tau <= 1.0f))
        return PZL_EINVAL;
    int64_t n_chunks = rows * cols / 8;
    unsigned blocks = (unsigned)((n_chunks + 255) / 256);
    hipLaunchKernelGGL(merge_pack_kernel, dim3(blocks), dim3(256), 0, st, wi, wj, norm_i, norm_j, rows, cols,
                       tau, out, n_similar, n_bad);
    return finish_launch();
}

}  // namespace pzl
