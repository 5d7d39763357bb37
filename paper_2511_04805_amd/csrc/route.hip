// Token-to-expert grouping and the weighted top-k combine.
// Neither is in the paper (it leaves routing to the host framework, Sec. 4.1 "other modules
// unchanged"); they are the glue that lets one packed-pair read serve both experts'
// token blocks, as the decode-GEMM of Sec. 3.3.2 requires.
#include "pzl_common.h"
#include <atomic>

namespace pzl {

constexpr int ROUTE_THREADS = 1024;
constexpr int ROUTE_WAVES = ROUTE_THREADS / 64;
constexpr int ROUTE_QMAX = 512;
constexpr int ROUTE_EMAX = 256;                     // routed experts of a layer (pzl_layer_create's bound)
constexpr int ROUTE_KEEP = 4;                       // trips of 256 ids that a wave keeps in registers

__device__ __forceinline__ bool pair_is_fused(int c0, int c1)
{
    return c0 >= 1 && c1 >= 1 && c0 <= TILE_FUSED_MAX_TOKENS && c1 <= TILE_FUSED_MAX_TOKENS;
}

// Counting sort of the flat (token, choice) list by q = 2*pair + pos, one workgroup.
// Wave w owns the contiguous index range [w*chunk, (w+1)*chunk) and its own histogram row, so
// the only contended atomics are LDS atomics inside one wave.
__global__ void __launch_bounds__(ROUTE_THREADS)
route_kernel(const int32_t *__restrict__ ids, int32_t n_flat, int32_t k, int32_t n_experts,
             const int32_t *__restrict__ q_of_expert, int32_t Q, int32_t *__restrict__ cnt,
             int32_t *__restrict__ off, int32_t *__restrict__ slot_tok, int32_t *__restrict__ slot_of,
             int32_t *__restrict__ tile_q, int32_t *__restrict__ tile_slot0, int32_t *__restrict__ tile_n,
             int32_t *__restrict__ n_tiles, int32_t tile_min, int32_t row_groups, int32_t launch_rows,
             int32_t sorted_cap)
{
    __shared__ int32_t hist[ROUTE_WAVES][ROUTE_QMAX];
    __shared__ int32_t total[ROUTE_QMAX];
    __shared__ bool tiled_pair[ROUTE_QMAX];
    __shared__ int16_t q_of[ROUTE_EMAX];              // expert -> routing key, staged: the lookups below are LDS reads
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    for (int i = tid; i < ROUTE_WAVES * ROUTE_QMAX; i += ROUTE_THREADS) (&hist[0][0])[i] = 0;
    for (int e = tid; e < n_experts; e += ROUTE_THREADS) q_of[e] = (int16_t)q_of_expert[e];

    int chunk = (n_flat + ROUTE_WAVES - 1) / ROUTE_WAVES;
    chunk = (chunk + 63) & ~63;
    const int lo = wave * chunk;
    const int hi = min(n_flat, lo + chunk);

    // Four ids per lane and trip (one 16-byte load when the range allows).  The kernel is bound by
    // the latency of its loads, not by their number: the first ROUTE_KEEP trips of a wave (1024
    // ids; all of them up to 16384 entries) are loaded at once, before anything waits for them,
    // and stay in registers for the scatter pass.
    const bool vec_ok = ((uintptr_t)ids & 15) == 0;      // lo is a multiple of 64 ids
    auto load4 = [&](int idx, int (&e4)[4]) {
        e4[0] = e4[1] = e4[2] = e4[3] = -1;
        if (vec_ok && idx + 3 < hi) {
            const int4 v = *(const int4 *)(ids + idx);
            e4[0] = v.x; e4[1] = v.y; e4[2] = v.z; e4[3] = v.w;
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) if (idx + j < hi) e4[j] = ids[idx + j];
        }
    };
    int kept[ROUTE_KEEP][4];
#pragma unroll
    for (int r = 0; r < ROUTE_KEEP; ++r) load4(lo + r * 256 + lane * 4, kept[r]);
    __syncthreads();                                     // hist is zero, q_of is there

#pragma unroll
    for (int r = 0; r < ROUTE_KEEP; ++r)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (kept[r][j] >= 0 && kept[r][j] < n_experts) atomicAdd(&hist[wave][q_of[kept[r][j]]], 1);
    for (int i = lo + ROUTE_KEEP * 256; i < hi; i += 256) {
        int e4[4];
        load4(i + lane * 4, e4);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (e4[j] >= 0 && e4[j] < n_experts) atomicAdd(&hist[wave][q_of[e4[j]]], 1);
    }
    __syncthreads();
    // per-q totals, then turn hist[w][q] into the first slot of (q, wave w)
    for (int q = tid; q < Q; q += ROUTE_THREADS) {
        int s = 0;
        for (int w = 0; w < ROUTE_WAVES; ++w) s += hist[w][q];
        total[q] = s;
    }
    __syncthreads();
    // A pair one of whose experts has at least tile_min tokens belongs to the tiled kernels (token
    // tiles below) and is empty for the streaming kernels; the decision is per pair so that a
    // pair's weights are swept by one path only.  If at least half of the pairs that have tokens
    // are such pairs, all of them go to the tiled kernels: two half-empty launches one after the
    // other are slower than either path alone.
    //
    // One tile for both experts of a pair (see pair_is_fused) saves a second pass over the pair's
    // weights but does the work of two tiles in one workgroup.  Measured on the three layer shapes
    // it pays when the launch (tiles x row_groups workgroups, 256 at a time) gets shorter by well
    // over a third, counting a launch that does not fill the chip as one that just does; it costs
    // when it only thins out a launch that was already short.
    //
    // The sums over the pairs behind these decisions are taken by wave 0 with shuffles (every thread
    // adding to one LDS word took 60 cycles per pair and sum, 12 000 cycles with 32 pairs).
    __shared__ int32_t scan_c[ROUTE_QMAX], scan_t[ROUTE_QMAX], n_slots_sh;
    __shared__ int32_t all_tiled_sh, tiles_plain, tiles_half, pairs_fusable, tiled_max, tiled_sum, tiled_experts;
    if (wave == 0) {
        auto wave_sum = [](int v) {
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d);
            return v;
        };
        auto wave_max = [](int v) {
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) v = max(v, __shfl_xor(v, d));
            return v;
        };
        int act = 0, big = 0;
        for (int g = lane; g < Q / 2; g += 64) {
            const int m = max(total[2 * g], total[2 * g + 1]);
            act += m > 0; big += m >= tile_min;
        }
        act = wave_sum(act); big = wave_sum(big);
        const bool all = big > 0 && 2 * big >= act;
        int tp = 0, th = 0, pf = 0, tm = 0, ts = 0, te = 0;
        for (int g = lane; g < Q / 2; g += 64) {
            const int c0 = total[2 * g], c1 = total[2 * g + 1];
            if (all || max(c0, c1) >= tile_min) {
                tp += (c0 + TILE_MAX_TOKENS - 1) / TILE_MAX_TOKENS + (c1 + TILE_MAX_TOKENS - 1) / TILE_MAX_TOKENS;
                th += (c0 + TILE_HALF_TOKENS - 1) / TILE_HALF_TOKENS + (c1 + TILE_HALF_TOKENS - 1) / TILE_HALF_TOKENS;
                pf += pair_is_fused(c0, c1);
                tm = max(tm, max(c0, c1));
                ts += c0 + c1;
                te += (c0 > 0) + (c1 > 0);
            }
        }
        tp = wave_sum(tp); th = wave_sum(th); pf = wave_sum(pf); tm = wave_max(tm); ts = wave_sum(ts); te = wave_sum(te);
        if (lane == 0) {
            all_tiled_sh = all; tiles_plain = tp; tiles_half = th; pairs_fusable = pf;
            tiled_max = tm; tiled_sum = ts; tiled_experts = te;
        }
    }
    __syncthreads();
    const bool all_tiled = all_tiled_sh != 0;
    // A launch of a few rounds of workgroups ends with its largest tiles: a busy expert's 281
    // tokens as one tile keep 11 workgroups running twice as long as the tiles of the others.
    // Such a launch, if its busiest expert has at least twice the tokens of the average tiled
    // expert, cuts its tiles at half the size (the tile list's bound, sized for full tiles plus
    // one per expert, must still hold them).  Measured (whole step): 64 experts top-6, skewed,
    // 192-768 tokens -10..-24 %; with an even router the smaller tiles only cost (60 experts top-4,
    // 2048 tokens: +6 % when cut regardless of the spread).
#ifndef PZL_HALF_TILE_WGS
#define PZL_HALF_TILE_WGS 768
#endif
    const bool spread = (int64_t)tiled_max * tiled_experts >= 2 * (int64_t)tiled_sum;
    const int tile_cap = (spread && (int64_t)tiles_plain * launch_rows <= PZL_HALF_TILE_WGS && tiles_half <= n_flat / TILE_MAX_TOKENS + Q)
                             ? TILE_HALF_TOKENS : TILE_MAX_TOKENS;
    const int64_t wgs_plain = max((int64_t)tiles_plain * row_groups, (int64_t)256);
    const int64_t wgs_fused = max((int64_t)(tiles_plain - pairs_fusable) * row_groups, (int64_t)256);
    const bool fuse = row_groups > 0 && pairs_fusable > 0 && 17 * wgs_fused < 10 * wgs_plain;
    // per expert: its count and its number of token tiles (equal parts of at most TILE_MAX_TOKENS,
    // rounded up to whole fragments of 16) ...
    for (int q = tid; q < ROUTE_QMAX; q += ROUTE_THREADS) {
        int c = q < Q ? total[q] : 0;
        bool t = q < Q && (all_tiled || max(total[q & ~1], total[q | 1]) >= tile_min);   // Q is even: q | 1 < Q
        int parts = (c + tile_cap - 1) / tile_cap;
        int size = parts ? (((c + parts - 1) / parts + 15) & ~15) : 0;
        scan_c[q] = c;
        scan_t[q] = t && c ? (c + size - 1) / size : 0;
        // a tiled pair whose experts both have a few tokens gets one tile for both (counted for the
        // even expert), so that its weights are read once
        if (t && fuse && pair_is_fused(total[q & ~1], total[q | 1])) scan_t[q] = (q & 1) ? 0 : 1;
        if (q < Q) { tiled_pair[q] = t; cnt[q] = t ? 0 : c; }
    }
    __syncthreads();
    // ... turned into first slot and first tile by an inclusive scan over the ROUTE_QMAX entries
    // (wave 0: every lane sums its 8 consecutive entries, a shuffle scan over the lanes, then the
    // lane walks its entries again)
    if (wave == 0) {
        constexpr int PER = ROUTE_QMAX / 64;
        int sc = 0, st = 0;
#pragma unroll
        for (int i = 0; i < PER; ++i) { sc += scan_c[lane * PER + i]; st += scan_t[lane * PER + i]; }
        int ic = sc, it = st;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            int uc = __shfl_up(ic, d), ut = __shfl_up(it, d);
            if (lane >= d) { ic += uc; it += ut; }
        }
        int run_c = ic - sc, run_t = it - st;                        // exclusive prefix of this lane
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            int q = lane * PER + i;
            int c = scan_c[q], t = scan_t[q];
            scan_c[q] = run_c; scan_t[q] = run_t;
            run_c += c; run_t += t;
        }
        if (lane == 63) { off[Q] = run_c; *n_tiles = run_t; n_slots_sh = run_c; }
        if (lane >= 8 && lane < 40) n_tiles[lane] = 0;               // work counters of the tiled launches
    }
    __syncthreads();
    for (int q = tid; q < Q; q += ROUTE_THREADS) {
        const int c = total[q], first = scan_c[q];
        off[q] = first;
        if (tiled_pair[q] && fuse && pair_is_fused(total[q & ~1], total[q | 1])) {
            if (!(q & 1)) {
                const int nt = scan_t[q];
                tile_q[nt] = q | TILE_FUSED_FLAG; tile_slot0[nt] = first; tile_n[nt] = c | (total[q | 1] << 16);
            }
        } else if (tiled_pair[q] && c > 0) {
            int parts = (c + tile_cap - 1) / tile_cap;
            int size = ((c + parts - 1) / parts + 15) & ~15;
            int nt = scan_t[q];
            for (int s0 = 0; s0 < c; s0 += size, ++nt) {
                tile_q[nt] = q; tile_slot0[nt] = first + s0; tile_n[nt] = min(size, c - s0);
            }
        }
    }
    __syncthreads();
    for (int q = tid; q < Q; q += ROUTE_THREADS) total[q] = scan_c[q];
    __syncthreads();
    for (int q = tid; q < Q; q += ROUTE_THREADS) {
        int run = total[q];
        for (int w = 0; w < ROUTE_WAVES; ++w) { int c = hist[w][q]; hist[w][q] = run; run += c; }
    }
    __syncthreads();

    // scatter: the rank inside (q, wave) comes from an LDS atomic.  Which lane gets which rank is
    // up to the hardware, so the order of slots inside one expert is not fixed; nothing
    // downstream depends on it (every slot is computed on its own and the combine adds a
    // token's choices in choice order).
    // slot -> token goes through LDS where the list fits (sorted_cap entries of dynamic LDS): written
    // straight to memory it is one scattered 4-byte store per entry, a cache line each, from a single
    // compute unit (14 000 cycles for 12 288 entries); from LDS it leaves as whole lines.
    extern __shared__ int32_t sorted_tok[];
    const bool via_lds = n_flat <= sorted_cap;
    auto scatter4 = [&](int idx, const int (&e4)[4]) {
        int slot4[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            slot4[j] = -1;
            if (idx + j < hi && e4[j] >= 0 && e4[j] < n_experts) {
                const int slot = atomicAdd(&hist[wave][q_of[e4[j]]], 1);
                if (via_lds) sorted_tok[slot] = (idx + j) / k;
                else         slot_tok[slot] = (idx + j) / k;
                slot4[j] = slot;
            }
        }
        if ((((uintptr_t)slot_of) & 15) == 0 && idx + 3 < hi) {
            *(int4 *)(slot_of + idx) = make_int4(slot4[0], slot4[1], slot4[2], slot4[3]);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) if (idx + j < hi) slot_of[idx + j] = slot4[j];
        }
    };
#pragma unroll
    for (int r = 0; r < ROUTE_KEEP; ++r) scatter4(lo + r * 256 + lane * 4, kept[r]);
    for (int i = lo + ROUTE_KEEP * 256; i < hi; i += 256) {
        int e4[4];
        load4(i + lane * 4, e4);
        scatter4(i + lane * 4, e4);
    }
    if (via_lds) {
        __syncthreads();
        for (int i = tid; i < n_slots_sh; i += ROUTE_THREADS) slot_tok[i] = sorted_tok[i];
    }
}

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float v)
{
    uint32_t u = __float_as_uint(v);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0u;          // NaN
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

// y[t, c] = bf16( sum_j w[t,j] * sum_ks O[ks][slot_of(t,j)][c]  +  sum_s sum_ks O[ks][N + s*T + t][c] )
// Fixed summation order (j ascending, k-splits ascending inside), so results are reproducible.
__global__ void __launch_bounds__(256)
combine_kernel(const float *__restrict__ opart, int32_t ksplit, int32_t ksplit_shared, int64_t ks_stride,
               const int32_t *__restrict__ slot_of, const float *__restrict__ topk_w, int32_t T,
               int32_t k, int32_t d, int32_t n_shared, uint16_t *__restrict__ y)
{
    const int t = blockIdx.x;
    const int c = (blockIdx.y * 256 + threadIdx.x) * 4;
    if (c >= d) return;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    const int n_flat = T * k;
    for (int j = 0; j < k; ++j) {
        int slot = slot_of[t * k + j];
        if (slot < 0) continue;
        float w = topk_w[t * k + j];
        const float *p = opart + (int64_t)slot * d + c;
        f32x4 s = *(const f32x4 *)p;
        for (int ks = 1; ks < ksplit; ++ks) s += *(const f32x4 *)(p + ks * ks_stride);
        acc += w * s;
    }
    for (int sh = 0; sh < n_shared; ++sh) {
        const float *p = opart + (int64_t)(n_flat + sh * T + t) * d + c;
        f32x4 s = *(const f32x4 *)p;
        for (int ks = 1; ks < ksplit_shared; ++ks) s += *(const f32x4 *)(p + ks * ks_stride);
        acc += s;
    }
    u32x2 o;
    o.x = f32_to_bf16_rne(acc.x) | (f32_to_bf16_rne(acc.y) << 16);
    o.y = f32_to_bf16_rne(acc.z) | (f32_to_bf16_rne(acc.w) << 16);
    *(u32x2 *)(y + (int64_t)t * d + c) = o;
}

// Router in front of the experts (not in the paper, which leaves the rest of the model unchanged,
// Sec. 4.1): logits = x W_r^T, top-k, softmax over the selected logits.  A lane owns one (token,
// expert) logit and accumulates it as ONE fused-multiply-add chain over the channels in order,
// so the logits, and with them the chosen experts, are reproducible bit for bit by a CPU that
// does the same.  Ties go to the lower expert index.
// The chain is the time: d dependent steps of three vector operations (two bf16 -> fp32
// conversions and the fma), whatever the number of lanes in use, so nothing else may hold it up.
// Thread = token * e_pad + expert (e_pad: the power of two >= E, at least 8), 256 / e_pad tokens
// per workgroup.  The lanes of a wave want 16 bytes each of DIFFERENT rows of W_r, which as a
// global load costs one cache line per lane and instruction; instead the workgroup copies W_r in
// chunks of CH channels (contiguous pieces of each row) into LDS, one chunk ahead of the chains
// (a chunk is long enough to cover the latency of the next one's loads), and every lane reads its
// row from there (row pitch CH*2 + 16 bytes).  x is read directly (the lanes of a token share the
// address), one chunk ahead as well.
constexpr int ROUTER_MAX_E = 256;
constexpr int ROUTER_MAX_K = 64;
constexpr int ROUTER_THREADS = 256;
constexpr int ROUTER_MAX_TPB = ROUTER_THREADS / 8; // tokens per workgroup at e_pad = 8

// The selection that ends both router kernels: `logit` holds the workgroup's logits (thread
// tid's at [tid], a token's e_pad logits side by side), e / ts / t are this thread's expert, token
// slot and token.
__device__ __forceinline__ void router_select(float *logit, float (*sel)[ROUTER_MAX_K], int tid, int e, int ts, int t,
                                              int T, int E, int k, int e_pad, int32_t *__restrict__ ids_out,
                                              float *__restrict__ w_out)
{
    // k selection passes: the largest logit not yet taken, ties to the lower expert index.
    // A token whose experts sit in one wave (e_pad <= 64) and whose logits are all numbers takes
    // each pass as a butterfly over its e_pad lanes on (value, index); otherwise one thread scans
    // the logits in LDS in index order, as the CPU side does (which also fixes what happens with
    // a NaN logit: it is never larger than anything, and nothing is larger than it).
    bool scan = e_pad > 64;
    if (!scan) {
        const float v = logit[tid];
        float nanf_ = (e < E && v != v) ? 1.0f : 0.0f;
        for (int off = e_pad / 2; off >= 1; off >>= 1) nanf_ = fmaxf(nanf_, __shfl_xor(nanf_, off, 64));
        scan = nanf_ != 0.0f;                               // the same for all lanes of the token
        if (!scan) {
            bool taken = e >= E;
            for (int j = 0; j < k; ++j) {
                float bv = taken ? -INFINITY : v;
                int bi = taken ? 0x7FFFFFFF : e;
                for (int off = e_pad / 2; off >= 1; off >>= 1) {
                    const float ov = __shfl_xor(bv, off, 64);
                    const int oi = __shfl_xor(bi, off, 64);
                    if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
                }
                if (e == bi) taken = true;
                if (e == 0 && t < T) {
                    ids_out[(int64_t)t * k + j] = bi;
                    sel[ts][j] = bv;
                }
            }
        }
    }
    if (e == 0 && t < T) {
        if (scan) {
            // a taken expert is marked by clearing its slot after the pass has recorded it
            float *lg = logit + ts * e_pad;
            for (int j = 0; j < k; ++j) {
                int best = -1;
                float bv = 0.0f;
                for (int i = 0; i < E; ++i) {
                    float v = lg[i];
                    bool free_slot = !(__float_as_uint(v) == 0xFF800001u);  // marker, see below
                    if (free_slot && (best < 0 || v > bv)) { best = i; bv = v; }
                }
                ids_out[(int64_t)t * k + j] = best;
                sel[ts][j] = bv;
                lg[best] = __uint_as_float(0xFF800001u);                    // a NaN pattern no fma chain of finite bf16 yields
            }
        }
        float mx = sel[ts][0], sum = 0.0f;
        for (int j = 0; j < k; ++j) sum += expf(sel[ts][j] - mx);
        for (int j = 0; j < k; ++j) w_out[(int64_t)t * k + j] = expf(sel[ts][j] - mx) / sum;
    }
}

// Few experts (e_pad <= 32): a wave holds 64 / e_pad tokens, so its lanes want only a few
// different rows of x and of W_r per load, and loading both operands directly, two sets of
// ROUTER_U 16-byte loads ahead of the chain, beats the copy through LDS below (8 experts, d = 4096:
// 39 us against 54 at 64 tokens, 42 against 56 at 4096).  One wave per workgroup.
constexpr int ROUTER_U = 6;

__global__ void __launch_bounds__(64)
router_topk_direct_kernel(const uint16_t *__restrict__ x, const uint16_t *__restrict__ w_router, int32_t T, int32_t d,
                          int32_t E, int32_t k, int32_t e_pad, int32_t *__restrict__ ids_out, float *__restrict__ w_out)
{
    __shared__ float logit[64];
    __shared__ float sel[ROUTER_MAX_TPB][ROUTER_MAX_K];
    const int tid = threadIdx.x;
    const int tpb = 64 / e_pad;
    const int e = tid % e_pad, ts = tid / e_pad;
    const int t = blockIdx.x * tpb + ts;
    {
        // lanes beyond the batch or the expert count run the chain of a valid (token, expert) and drop it
        const u32x4 *xr = (const u32x4 *)(x + (int64_t)min(t, T - 1) * d);
        const u32x4 *wr = (const u32x4 *)(w_router + (int64_t)min(e, E - 1) * d);
        const int n8 = d / 8;
        float acc = 0.0f;
        u32x4 xa[ROUTER_U], wa[ROUTER_U], xb[ROUTER_U], wb[ROUTER_U];
        auto load = [&](int c0, u32x4 (&xv)[ROUTER_U], u32x4 (&wv)[ROUTER_U]) {
#pragma unroll
            for (int u = 0; u < ROUTER_U; ++u) {
                const int c = min(c0 + u, n8 - 1);        // past the end: a re-read nobody uses
                xv[u] = xr[c];
                wv[u] = wr[c];
            }
        };
        auto chain = [&](int c0, const u32x4 (&xv)[ROUTER_U], const u32x4 (&wv)[ROUTER_U]) {
#pragma unroll
            for (int u = 0; u < ROUTER_U; ++u) {
                if (c0 + u >= n8) break;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    acc = __fmaf_rn(__uint_as_float(xv[u][i] << 16), __uint_as_float(wv[u][i] << 16), acc);
                    acc = __fmaf_rn(__uint_as_float(xv[u][i] & 0xFFFF0000u), __uint_as_float(wv[u][i] & 0xFFFF0000u), acc);
                }
            }
        };
        load(0, xa, wa);
        for (int c0 = 0; c0 < n8; c0 += 2 * ROUTER_U) {
            load(c0 + ROUTER_U, xb, wb);
            chain(c0, xa, wa);
            load(c0 + 2 * ROUTER_U, xa, wa);
            chain(c0 + ROUTER_U, xb, wb);
        }
        logit[tid] = acc;
    }
    __syncthreads();
    router_select(logit, sel, tid, e, ts, t, T, E, k, e_pad, ids_out, w_out);
}

template <int CH, int EROWS>                        // channels per chunk, rows of W_r the buffers hold
__global__ void __launch_bounds__(ROUTER_THREADS)
router_topk_kernel(const uint16_t *__restrict__ x, const uint16_t *__restrict__ w_router, int32_t T, int32_t d,
                   int32_t E, int32_t k, int32_t e_pad, int32_t *__restrict__ ids_out, float *__restrict__ w_out)
{
    constexpr int PITCH = CH * 2 + 16;              // bytes per row of a chunk in LDS
    constexpr int UNITS = CH / 8;                   // 16-byte units per row and chunk
    constexpr int WLOADS = EROWS * UNITS / ROUTER_THREADS;
    static_assert(EROWS * UNITS % ROUTER_THREADS == 0, "copy loop");
    __shared__ __attribute__((aligned(16))) unsigned char wbuf[2][EROWS * PITCH];
    __shared__ float logit[ROUTER_THREADS];
    __shared__ float sel[ROUTER_MAX_TPB][ROUTER_MAX_K];
    const int tid = threadIdx.x;
    const int tpb = ROUTER_THREADS / e_pad;
    const int e = tid % e_pad, ts = tid / e_pad;
    const int t = blockIdx.x * tpb + ts;
    {
        // lanes beyond the batch or the expert count run the chain of a valid (token, expert) and drop it
        const u32x4 *xr = (const u32x4 *)(x + (int64_t)min(t, T - 1) * d);
        const unsigned char *my_row = &wbuf[0][0] + min(e, E - 1) * PITCH;
        const int n8 = d / 8;                             // 16-byte units per row; the last chunk may hold fewer than UNITS
        const int n_chunks = (d + CH - 1) / CH;
        u32x4 wreg[WLOADS], xreg[UNITS];
        // unit v of a chunk = (row v / UNITS, 16-byte part v % UNITS); thread tid copies units tid, tid + 256, ...
        auto fetch_w = [&](int chunk) {
#pragma unroll
            for (int i = 0; i < WLOADS; ++i) {
                const int v = tid + i * ROUTER_THREADS;
                if (v < E * UNITS && chunk * UNITS + v % UNITS < n8)
                    wreg[i] = *(const u32x4 *)(w_router + (int64_t)(v / UNITS) * d + chunk * CH + (v % UNITS) * 8);
            }
        };
        auto store_w = [&](int buf) {
#pragma unroll
            for (int i = 0; i < WLOADS; ++i) {
                const int v = tid + i * ROUTER_THREADS;
                if (v < E * UNITS) *(u32x4 *)(&wbuf[buf][0] + (v / UNITS) * PITCH + (v % UNITS) * 16) = wreg[i];
            }
        };
        auto fetch_x = [&](int chunk) {
#pragma unroll
            for (int u = 0; u < UNITS; ++u) xreg[u] = xr[min(chunk * UNITS + u, n8 - 1)];
        };
        float acc = 0.0f;
        fetch_w(0);
        fetch_x(0);
        store_w(0);
        __syncthreads();
        for (int c = 0; c < n_chunks; ++c) {
            const bool more = c + 1 < n_chunks;
            u32x4 xv[UNITS];
#pragma unroll
            for (int u = 0; u < UNITS; ++u) xv[u] = xreg[u];
            if (more) { fetch_w(c + 1); fetch_x(c + 1); }
            const unsigned char *row = my_row + (c & 1) * (EROWS * PITCH);
            // a whole chunk is straight-line code (the LDS reads can then run ahead of the chain);
            // only the last chunk of a row that is not a multiple of CH long checks its units
            auto unit = [&](int u) {
                const u32x4 wv = *(const u32x4 *)(row + u * 16);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    acc = __fmaf_rn(__uint_as_float(xv[u][i] << 16), __uint_as_float(wv[i] << 16), acc);
                    acc = __fmaf_rn(__uint_as_float(xv[u][i] & 0xFFFF0000u), __uint_as_float(wv[i] & 0xFFFF0000u), acc);
                }
            };
            if ((c + 1) * UNITS <= n8) {
#pragma unroll
                for (int u = 0; u < UNITS; ++u) unit(u);
            } else {
#pragma unroll
                for (int u = 0; u < UNITS; ++u) if (c * UNITS + u < n8) unit(u);
            }
            if (more) store_w((c + 1) & 1);               // last read two chunks ago, before the previous barrier
            __syncthreads();
        }
        logit[tid] = acc;
    }
    __syncthreads();
    router_select(logit, sel, tid, e, ts, t, T, E, k, e_pad, ids_out, w_out);
}

int launch_router_topk(const uint16_t *x, const uint16_t *w_router, int32_t T, int32_t d, int32_t E, int32_t k,
                       int32_t *ids_out, float *w_out, hipStream_t st)
{
    if (T < 0 || d <= 0 || d % 8 || E < 1 || E > ROUTER_MAX_E || k < 1 || k > E || k > ROUTER_MAX_K) return PZL_EINVAL;
    if (T == 0) return PZL_OK;
    if (!x || !w_router || !ids_out || !w_out) return PZL_EINVAL;
    int e_pad = 8;
    while (e_pad < E) e_pad *= 2;
    if (e_pad <= 32) {
        const int tpw = 64 / e_pad;
        hipLaunchKernelGGL(router_topk_direct_kernel, dim3((unsigned)((T + tpw - 1) / tpw)), dim3(64), 0, st, x, w_router,
                           T, d, E, k, e_pad, ids_out, w_out);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) { set_hip_error(e); return PZL_EHIP; }
        return PZL_OK;
    }
    const int tpb = ROUTER_THREADS / e_pad;
    const dim3 grid((unsigned)((T + tpb - 1) / tpb)), block(ROUTER_THREADS);
    // chunks as long as two buffers of E rows allow (about 17-20 KiB each); with more than two
    // workgroups per compute unit shorter chunks, whose registers let four workgroups share one
    // (64 experts, d = 2048: 2048 tokens 46 us with 128 channels per chunk / 47 with 64, 4096
    // tokens 88 / 71)
    if (e_pad <= 64 && grid.x > 512)
        hipLaunchKernelGGL((router_topk_kernel<64, 64>), grid, block, 0, st, x, w_router, T, d, E, k, e_pad, ids_out, w_out);
    else if (e_pad <= 64)
        hipLaunchKernelGGL((router_topk_kernel<128, 64>), grid, block, 0, st, x, w_router, T, d, E, k, e_pad, ids_out, w_out);
    else if (e_pad == 128)
        hipLaunchKernelGGL((router_topk_kernel<64, 128>), grid, block, 0, st, x, w_router, T, d, E, k, e_pad, ids_out, w_out);
    else
        hipLaunchKernelGGL((router_topk_kernel<32, 256>), grid, block, 0, st, x, w_router, T, d, E, k, e_pad, ids_out, w_out);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_hip_error(e); return PZL_EHIP; }
    return PZL_OK;
}

// Dynamic LDS of the grouping kernel: the slot -> token list of batches up to this many entries
constexpr int ROUTE_SORTED_CAP = 16384;

// more than 64 KiB of LDS in all: a per-device attribute of the kernel, set once per device (layer
// creation does it, so that no call under stream capture has to)
int prepare_route_kernel()
{
    static std::atomic<uint64_t> attr_devices{0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev > 63) dev = 63;       // unknown device: set it every time
    if (dev == 63 || !((attr_devices.load(std::memory_order_relaxed) >> dev) & 1)) {
        hipError_t e = hipFuncSetAttribute((const void *)route_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           ROUTE_SORTED_CAP * (int)sizeof(int32_t));
        if (e != hipSuccess) { set_hip_error(e); return PZL_EHIP; }
        if (dev != 63) attr_devices.fetch_or(1ull << dev, std::memory_order_relaxed);
    }
    return PZL_OK;
}

int launch_route(const int32_t *ids, int32_t n_flat, int32_t k, int32_t n_experts, int32_t n_slots_q,
                 const int32_t *q_of_expert, RouteTables rt, int32_t tile_min, int32_t row_groups, int32_t launch_rows,
                 hipStream_t st)
{
    int Q = n_slots_q;
    if (Q > ROUTE_QMAX || n_experts > ROUTE_EMAX) return PZL_EINVAL;
    int rc = prepare_route_kernel();
    if (rc) return rc;
    const int sorted_cap = n_flat <= ROUTE_SORTED_CAP ? ((n_flat + 63) & ~63) : 0;
    hipLaunchKernelGGL(route_kernel, dim3(1), dim3(ROUTE_THREADS), sorted_cap * sizeof(int32_t), st, ids, n_flat, k, n_experts,
                       q_of_expert, Q, rt.cnt, rt.off, rt.slot_tok, rt.slot_of, rt.tile_q, rt.tile_slot0,
                       rt.tile_n, rt.n_tiles, tile_min, row_groups, launch_rows, sorted_cap);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_hip_error(e); return PZL_EHIP; }
    return PZL_OK;
}

int launch_combine(const float *opart, int32_t ksplit, int32_t ksplit_shared, int64_t ks_stride, const RouteTables &rt,
                   const float *topk_w, int32_t T, int32_t k, int32_t d, int32_t n_shared,
                   uint16_t *y, hipStream_t st)
{
    dim3 grid((unsigned)T, (unsigned)((d / 4 + 255) / 256));
    hipLaunchKernelGGL(combine_kernel, grid, dim3(256), 0, st, opart, ksplit, ksplit_shared, ks_stride, rt.slot_of,
                       topk_w, T, k, d, n_shared, y);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_hip_error(e); return PZL_EHIP; }
    return PZL_OK;
}

}  // namespace pzl
