/*
 * CPU oracle for the quantised variant of the merged-expert format.  TEST INFRASTRUCTURE ONLY:
 * shares no code with the HIP library, and nothing in the product path may call it.
 *
 * Paper: appendix "Combining PuzzleMoE with Quantization".  After merging, the (non-negative)
 * merged weights are quantised uniformly in groups of 128 with a symmetric scheme (no zero point)
 * to 3 bits and stored alongside the two sign bits and the mask; the mask of an element is one of
 * {01, 10, 11} and therefore costs log2(3) ~ 1.58 bits; with a 16-bit scale per group the
 * appendix's average is (2 + 1.58 + 3 + 0.125) / 2 = 3.35 bits per original weight.
 *
 * The appendix gives the bit accounting, not a storage format or a rounding rule.  Readings taken
 * here (all listed in the design notes):
 *   - the three quantisation bits are magnitude bits (signs are stored separately), so a code is
 *     an unsigned integer 0..7 and the dequantised magnitude is code * scale;
 *   - groups run along the input dimension (the columns of a [rows, cols] weight), 128 consecutive
 *     columns of one row;
 *   - scale = bf16( max_group / 7 ), max over the magnitudes of the group that at least one expert
 *     uses; code = min(7, rint(magnitude / scale)) with magnitude, scale and the quotient in fp32
 *     (one correctly rounded division, ties to even) -- an integer decided by floating point, so
 *     both sides take it in this precision; a group whose maximum is 0 has scale 0 and codes 0;
 *   - an element that no expert uses (mask 00, which Eq. 4 never produces but the generic format
 *     allows) is stored as code 0 with mask 11: it reconstructs to 0 for both experts either way;
 *   - the mask is stored as a base-3 digit: 0 -> expert 0 only, 1 -> expert 1 only, 2 -> both;
 *     eight digits make one 13-bit number (3^8 = 6561 <= 2^13), 1.625 bits per element instead
 *     of the entropy bound 1.58;
 *   - reconstruction: W_p = (-1)^(S_p) * M_p * code * scale, exactly (no rounding of the product).
 *
 * Logical arrays (row-major [rows, cols], one byte per field and element) are what this oracle
 * produces and consumes; orc_q_records lays them out as the 53-bit records the format stores
 * (codes 24 bits, S0 8, S1 8, mask number 13, for the 8 elements of one row inside a 32-column
 * block) in plain row-major record order.  The tiled order in device memory is the GPU library's
 * business; the tests map one to the other.
 *
 * Pins (tests, CPU only): the digit coding is a bijection on 0..6560; the appendix's bit-width
 * formula against the size of the stored format; |W - code*scale| <= scale/2 wherever the code
 * is below 7, and the group maximum gets code 7; exact reconstruction when the magnitudes are
 * integer multiples of a power-of-two step; the FFN against the bf16 oracle's dense-expert path
 * on such exactly representable weights.
 * Parity unpinned (paper silent, no second source): that the codes are unsigned, the rounding
 * rule of scale and code, and the treatment of an element that no expert uses.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define QGROUP 128

static float bf16_bits_to_float(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* fp32 -> bf16, round to nearest even (finite, non-negative inputs only are used here) */
static uint16_t float_to_bf16_rne(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

/*
 * Quantise.  merged: bf16 bits (sign ignored), mask0/mask1/sign0/sign1: 0/1 bytes, all [rows, cols].
 * Out: code[rows*cols] in 0..7, trit[rows*cols] in 0..2, s0/s1 copied as 0/1,
 *      scale[rows * cols/128] bf16 bits.  Returns the number of non-finite magnitudes (stored as 0).
 */
int64_t orc_q_quantise(const uint16_t *merged, const uint8_t *mask0, const uint8_t *mask1,
                       const uint8_t *sign0, const uint8_t *sign1, int64_t rows, int64_t cols,
                       uint8_t *code, uint8_t *trit, uint8_t *s0, uint8_t *s1, uint16_t *scale)
{
    int64_t bad = 0;
    const int64_t groups = cols / QGROUP;
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t g = 0; g < groups; ++g) {
            const int64_t base = r * cols + g * QGROUP;
            volatile float mx = 0.0f;
            for (int c = 0; c < QGROUP; ++c) {
                int64_t i = base + c;
                int used = (mask0[i] != 0) || (mask1[i] != 0);
                float m = bf16_bits_to_float(merged[i] & 0x7FFF);
                if (!isfinite(m)) { if (used) ++bad; continue; }
                if (used && m > mx) mx = m;
            }
            volatile float sc_f = mx / 7.0f;                     /* one rounded fp32 division */
            uint16_t sc_bits = float_to_bf16_rne(sc_f);
            float sc = bf16_bits_to_float(sc_bits);
            scale[r * groups + g] = sc_bits;
            for (int c = 0; c < QGROUP; ++c) {
                int64_t i = base + c;
                int m0 = mask0[i] != 0, m1 = mask1[i] != 0;
                float m = bf16_bits_to_float(merged[i] & 0x7FFF);
                int q = 0;
                if ((m0 || m1) && isfinite(m) && sc > 0.0f) {
                    volatile float quo = m / sc;                 /* one rounded fp32 division */
                    float rq = rintf(quo);                       /* ties to even */
                    q = rq > 7.0f ? 7 : (int)rq;
                }
                code[i] = (uint8_t)q;
                trit[i] = (uint8_t)((m0 && m1) ? 2 : (m1 ? 1 : (m0 ? 0 : 2)));
                if (!m0 && !m1) code[i] = 0;
                s0[i] = sign0[i] != 0;
                s1[i] = sign1[i] != 0;
            }
        }
    }
    return bad;
}

/* Reconstruct expert `pos` (0 or 1): out[i] = (-1)^S * M * code * scale, exact in fp64. */
void orc_q_dequantise(const uint8_t *code, const uint8_t *trit, const uint8_t *s0, const uint8_t *s1,
                      const uint16_t *scale, int pos, int64_t rows, int64_t cols, double *out)
{
    const int64_t groups = cols / QGROUP;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) {
            int64_t i = r * cols + c;
            int t = trit[i];
            int m = (t == 2) || (t == pos);
            int s = pos ? s1[i] : s0[i];
            double v = (double)code[i] * (double)bf16_bits_to_float(scale[r * groups + c / QGROUP]);
            out[i] = m ? (s ? -v : v) : 0.0;
        }
}

/*
 * The stored records, in plain row-major record order: record (r, c/8) covers the 8 elements
 * (r, 8*(c/8) .. +7) and is the 53-bit number
 *   codes (element e at bits 3e..3e+2) | S0 bits << 24 | S1 bits << 32 | (sum_e trit_e 3^e) << 40.
 * out: one uint64 per record.
 */
void orc_q_records(const uint8_t *code, const uint8_t *trit, const uint8_t *s0, const uint8_t *s1,
                   int64_t rows, int64_t cols, uint64_t *out)
{
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t b = 0; b < cols / 8; ++b) {
            uint64_t rec = 0, t = 0, p3 = 1;
            for (int e = 0; e < 8; ++e) {
                int64_t i = r * cols + b * 8 + e;
                rec |= (uint64_t)(code[i] & 7) << (3 * e);
                rec |= (uint64_t)(s0[i] & 1) << (24 + e);
                rec |= (uint64_t)(s1[i] & 1) << (32 + e);
                t += (uint64_t)trit[i] * p3;
                p3 *= 3;
            }
            out[r * (cols / 8) + b] = rec | (t << 40);
        }
}

/* Stored bits per original expert weight: 53 bits per 8 element positions plus a 16-bit scale per
 * 128, shared by the two experts of the pair. */
double orc_q_bits_per_weight(void)
{
    return (53.0 / 8.0 + 16.0 / QGROUP) / 2.0;
}

/* ---------- routed SwiGLU expert FFN on reconstructed weights (fp64, plain definition) ---------- */

static double silu(double g) { return g / (1.0 + exp(-g)); }

static void matvec64(const double *W, int rows, int cols, const double *v, double *out)
{
#pragma omp parallel for schedule(static)
    for (int r = 0; r < rows; ++r) {
        const double *row = W + (int64_t)r * cols;
        double acc = 0.0;
        for (int c = 0; c < cols; ++c) acc += row[c] * v[c];
        out[r] = acc;
    }
}

/*
 * y[t,:] = sum_j w[t,j] * Wdown_e ( silu(Wgate_e x_t) * (Wup_e x_t) ),  e = ids[t,j],
 * with the experts' reconstructed weights given as fp64 matrices (gate/up [f,d], down [d,f]).
 * x: bf16 bits.  Returns 0, or -1 on a bad id / allocation failure.
 */
int orc_ffn_dense64(int T, int k, int E, int d, int f, const uint16_t *x, const int32_t *ids,
                    const float *w, const double *const *gate, const double *const *up,
                    const double *const *down, double *y64)
{
    double *xv = malloc(sizeof(double) * d), *g = malloc(sizeof(double) * f);
    double *u = malloc(sizeof(double) * f), *h = malloc(sizeof(double) * f);
    double *o = malloc(sizeof(double) * d);
    int rc = 0;
    if (!xv || !g || !u || !h || !o) { rc = -1; goto done; }
    for (int t = 0; t < T; ++t) {
        for (int c = 0; c < d; ++c) xv[c] = (double)bf16_bits_to_float(x[(int64_t)t * d + c]);
        for (int c = 0; c < d; ++c) y64[(int64_t)t * d + c] = 0.0;
        for (int j = 0; j < k; ++j) {
            int e = ids[(int64_t)t * k + j];
            if (e < 0 || e >= E) { rc = -1; goto done; }
            matvec64(gate[e], f, d, xv, g);
            matvec64(up[e], f, d, xv, u);
            for (int r = 0; r < f; ++r) h[r] = silu(g[r]) * u[r];
            matvec64(down[e], d, f, h, o);
            double wt = (double)w[(int64_t)t * k + j];
            for (int c = 0; c < d; ++c) y64[(int64_t)t * d + c] += wt * o[c];
        }
    }
done:
    free(xv); free(g); free(u); free(h); free(o);
    return rc;
}
