/*
 * CPU oracle for the bit-packed merged-expert MoE FFN (PuzzleMoE inference path).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * HIP library is checked against.  It shares no code, header, table or helper
 * with the GPU path, and nothing in the product path may call it.
 *
 * What follows the paper, and where:
 *   - packed 16-bit word and exponent rule ... Sec. 3.3.2 "System Co-design"
 *   - orc_unpack .............................. Algorithm 1 (weight decoding)
 *   - reconstruction identity ................. Eq. 6
 *   - orc_moe_ffn ............................. Eq. 6 weights inside an ordinary
 *     routed SwiGLU expert FFN ("other modules unchanged", Sec. 4.1); the FFN
 *     itself (gate/up/down, silu, weighted top-k sum, shared experts added with
 *     weight 1) is not in the paper and follows the standard definition.
 *
 * Readings where the paper is silent (all listed in the design notes):
 *   - an exponent below 112 is raised to 112 and the mantissa is kept;
 *   - an exactly-zero magnitude is stored with both mask bits cleared, so
 *     that Eq. 6 still gives 0;
 *   - an exponent above 143 (this includes Inf/NaN) cannot be stored in five
 *     bits: it is counted as out of range and stored as a fully masked word;
 *   - a masked-out element decodes to +0 (Algorithm 1 assigns 0 before any
 *     sign handling);
 *   - sign bits are stored as given even where the mask is 0; the sign bit of
 *     the merged input is ignored (Eq. 5 makes W_merged non-negative).
 *
 * Parity pins (tests, CPU only): exhaustive Algorithm-1 truth table against
 * the closed form (-1)^s m 2^(e5-15)(1+mant/128); pack->unpack against Eq. 6
 * over every non-negative bf16 and all 16 flag combinations; a hand-derived
 * golden example; the FFN against an independent dense numpy evaluation and
 * against special cases that reduce to a textbook dense SwiGLU FFN.
 * Unpinned (paper silent, no second source): the three readings above that
 * concern exponents < 112, zero, and exponents > 143.
 *
 * orc_router_topk (the router in front of the experts; not in the paper, which keeps
 * "the other modules unchanged", Sec. 4.1): a textbook linear router, top-k, softmax over
 * the selected logits.  The logits decide integers (which experts), so they are computed
 * in fp32 as one fused multiply-add chain over the channels in order, exactly as the GPU
 * kernel does; ties go to the lower expert index.  Pinned by brute force against numpy on
 * inputs whose products and sums are exact in fp32, and by permutation / tie cases.
 *
 * Arithmetic: integer for pack/unpack; fp64 everywhere in the FFN; a single
 * round-to-nearest-even to bf16 at the very end.
 *
 * orc_merge (the offline dual-mask merge, Sec. 3.2, Eqs. 1-5) decides two masks by
 * floating-point comparisons.  Those decisions are taken in fp32, one rounding per
 * operation and no fused multiply-add, which is the precision the GPU kernel uses:
 * a mask bit is an integer result and both sides must take it the same way.
 * Pinned by Lemma 3.1's closed form on Gaussian inputs, the structure Eq. 4 implies
 * (never both masks clear), the reconstruction error bound, and special cases.
 * Unpinned: 0/0 in the similarity measure is read as "not similar".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---------- bf16 helpers (bf16 = 1 sign, 8 exponent, 7 mantissa bits; Sec. 3.3.1) ---------- */

double orc_bf16_to_double(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* Round a double to the nearest bf16, ties to even, directly (no float stage). */
uint16_t orc_bf16_from_double(double v)
{
    if (isnan(v)) return 0x7FC0;
    uint16_t sign = signbit(v) ? 0x8000 : 0;
    double a = fabs(v);
    if (a == 0.0) return sign;
    if (isinf(a)) return sign | 0x7F80;
    double r;                              /* the rounded magnitude, exactly representable */
    const double min_normal = ldexp(1.0, -126);
    if (a < min_normal) {
        const double quantum = ldexp(1.0, -133);           /* bf16 subnormal spacing */
        r = nearbyint(a / quantum) * quantum;
    } else {
        int e;
        double m = frexp(a, &e);                           /* a = m 2^e, m in [0.5,1) */
        double q = nearbyint(m * 256.0);                   /* 8 significant bits, RNE */
        r = ldexp(q, e - 8);
    }
    float f = (float)r;                                    /* exact, or overflow to inf */
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    return sign | (uint16_t)(u >> 16);
}

/* ---------- pack: Sec. 3.3.2 exponent rule + the bit positions Algorithm 1 reads ---------- */

/*
 * word = S0<<15 | S1<<14 | M0<<13 | M1<<12 | (exponent-112)<<7 | mantissa
 * Returns the number of elements whose exponent does not fit (exponent > 143).
 */
int64_t orc_pack(const uint16_t *merged, const uint8_t *mask0, const uint8_t *mask1,
                 const uint8_t *sign0, const uint8_t *sign1, int64_t n, uint16_t *packed)
{
    int64_t bad = 0;
    for (int64_t i = 0; i < n; ++i) {
        uint16_t mag = merged[i] & 0x7FFF;                 /* input sign ignored */
        int exponent = mag >> 7;
        int mantissa = mag & 0x7F;
        int m0 = mask0[i] ? 1 : 0, m1 = mask1[i] ? 1 : 0;
        int s0 = sign0[i] ? 1 : 0, s1 = sign1[i] ? 1 : 0;
        if (exponent > 143) {                              /* not representable in 5 bits */
            ++bad;
            packed[i] = (uint16_t)(s0 << 15 | s1 << 14);
            continue;
        }
        if (mag == 0) {                                    /* exact zero: mask it out */
            packed[i] = (uint16_t)(s0 << 15 | s1 << 14);
            continue;
        }
        if (exponent < 112) exponent = 112;                /* raised to 112, mantissa kept */
        packed[i] = (uint16_t)(s0 << 15 | s1 << 14 | m0 << 13 | m1 << 12 |
                               (exponent - 112) << 7 | mantissa);
    }
    return bad;
}

/* ---------- unpack: Algorithm 1 ---------- */

static uint16_t decode_word(uint16_t W, int expert_pos)
{
    int mask_bit = (W >> (13 - expert_pos)) & 1;
    if (mask_bit == 0) return 0;
    int sign_bit = (W >> (15 - expert_pos)) & 1;
    int exp_field = (W & 0x0F80) + (112 << 7);
    return (uint16_t)(sign_bit << 15 | exp_field | (W & 0x007F));
}

void orc_unpack(const uint16_t *packed, int expert_pos, int64_t n, uint16_t *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = decode_word(packed[i], expert_pos);
}

/* ---------- routed SwiGLU expert FFN on decoded weights ---------- */

static double silu(double g) { return g / (1.0 + exp(-g)); }

/* out[r] = sum_c decode(Wp[r,c]) * v[c]   (rows x cols, row-major, fp64, left to right) */
static void matvec_packed(const uint16_t *Wp, int pos, int rows, int cols,
                          const double *v, double *out)
{
#pragma omp parallel for schedule(static)
    for (int r = 0; r < rows; ++r) {
        const uint16_t *row = Wp + (int64_t)r * cols;
        double acc = 0.0;
        for (int c = 0; c < cols; ++c)
            acc += orc_bf16_to_double(decode_word(row[c], pos)) * v[c];
        out[r] = acc;
    }
}

static void matvec_dense(const uint16_t *Wd, int rows, int cols, const double *v, double *out)
{
#pragma omp parallel for schedule(static)
    for (int r = 0; r < rows; ++r) {
        const uint16_t *row = Wd + (int64_t)r * cols;
        double acc = 0.0;
        for (int c = 0; c < cols; ++c) acc += orc_bf16_to_double(row[c]) * v[c];
        out[r] = acc;
    }
}

/*
 * y[t,:] = sum_j w[t,j] * FFN_{ids[t,j]}(x[t,:])  +  sum_s FFN_shared_s(x[t,:])
 * FFN_e(x) = Wdown_e ( silu(Wgate_e x) * (Wup_e x) ).
 * Expert e with expert_pair[e] = p >= 0 is merged: W_e = Eq. 6 decode of pair p's packed tensor at
 * position expert_pos[e].  Expert e with expert_pair[e] = -1-j is routed dense expert j, kept
 * unmerged (the 25 % compression setting of Sec. 4.1 leaves half of the experts as they are).
 * gate/up are [f,d], down is [d,f], row-major, in the *logical* element order.
 *
 * stage_h_bf16 = 0: the definition (h kept in fp64).
 * stage_h_bf16 = 1: h rounded to bf16 before the down projection (diagnostic only).
 * y64 (optional) receives the unrounded sums, ybf16 (optional) their bf16 rounding.
 * Returns 0, or -1 on an id outside [0,E) or allocation failure.
 */
int orc_moe_ffn(int T, int k, int E, int d, int f,
                const uint16_t *x, const int32_t *ids, const float *w,
                const int32_t *expert_pair, const uint8_t *expert_pos,
                const uint16_t *const *gate, const uint16_t *const *up,
                const uint16_t *const *down,
                int n_dense, const uint16_t *const *dgate, const uint16_t *const *dup,
                const uint16_t *const *ddown,
                int n_shared, const int32_t *shared_f,
                const uint16_t *const *sgate, const uint16_t *const *sup,
                const uint16_t *const *sdown,
                int stage_h_bf16, double *y64, uint16_t *ybf16)
{
    int fmax = f;
    for (int s = 0; s < n_shared; ++s) if (shared_f[s] > fmax) fmax = shared_f[s];
    double *xv = malloc(sizeof(double) * d);
    double *g = malloc(sizeof(double) * fmax);
    double *u = malloc(sizeof(double) * fmax);
    double *h = malloc(sizeof(double) * fmax);
    double *o = malloc(sizeof(double) * d);
    double *acc = malloc(sizeof(double) * d);
    int rc = 0;
    if (!xv || !g || !u || !h || !o || !acc) { rc = -1; goto done; }

    for (int t = 0; t < T; ++t) {
        for (int c = 0; c < d; ++c) xv[c] = orc_bf16_to_double(x[(int64_t)t * d + c]);
        for (int c = 0; c < d; ++c) acc[c] = 0.0;

        for (int j = 0; j < k; ++j) {
            int e = ids[(int64_t)t * k + j];
            if (e < 0 || e >= E) { rc = -1; goto done; }
            int p = expert_pair[e], pos = expert_pos[e];
            if (p >= 0) {
                matvec_packed(gate[p], pos, f, d, xv, g);
                matvec_packed(up[p], pos, f, d, xv, u);
            } else {
                int dj = -1 - p;
                if (dj >= n_dense) { rc = -1; goto done; }
                matvec_dense(dgate[dj], f, d, xv, g);
                matvec_dense(dup[dj], f, d, xv, u);
            }
            for (int r = 0; r < f; ++r) {
                h[r] = silu(g[r]) * u[r];
                if (stage_h_bf16) h[r] = orc_bf16_to_double(orc_bf16_from_double(h[r]));
            }
            if (p >= 0) matvec_packed(down[p], pos, d, f, h, o);
            else        matvec_dense(ddown[-1 - p], d, f, h, o);
            double wt = (double)w[(int64_t)t * k + j];
            for (int c = 0; c < d; ++c) acc[c] += wt * o[c];
        }
        for (int s = 0; s < n_shared; ++s) {
            int fs = shared_f[s];
            matvec_dense(sgate[s], fs, d, xv, g);
            matvec_dense(sup[s], fs, d, xv, u);
            for (int r = 0; r < fs; ++r) {
                h[r] = silu(g[r]) * u[r];
                if (stage_h_bf16) h[r] = orc_bf16_to_double(orc_bf16_from_double(h[r]));
            }
            matvec_dense(sdown[s], d, fs, h, o);
            for (int c = 0; c < d; ++c) acc[c] += o[c];
        }
        for (int c = 0; c < d; ++c) {
            if (y64) y64[(int64_t)t * d + c] = acc[c];
            if (ybf16) ybf16[(int64_t)t * d + c] = orc_bf16_from_double(acc[c]);
        }
    }
done:
    free(xv); free(g); free(u); free(h); free(o); free(acc);
    return rc;
}

/* ---------- offline dual-mask merge of two experts: Sec. 3.2, Eqs. 1-5 ---------- */

static float bf16_to_float(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/*
 * wi, wj: [rows, cols] bf16 bit patterns of the two experts' matrices (row-major, the
 * contracted/input dimension along cols).  norm_i, norm_j: [cols] the l2 norm of each input
 * channel's calibration activations (Eq. 2 multiplies |W| by it, channel-wise).
 * Outputs, all [rows, cols]: merged (bf16 bits, >= 0), mask_i, mask_j, sign_i, sign_j (0/1).
 *
 *   similarity (unnumbered display before Eq. 1):  | |wi|-|wj| | / (|wi|+|wj|) <= tau,
 *       evaluated division-free as  | |wi|-|wj| |  <=  tau * (|wi|+|wj|)  in fp32;
 *       both magnitudes zero (0/0) counts as not similar;
 *   signs (Eq. 1): w < 0;  saliency (Eqs. 2, 3): |wi|*norm_i >= |wj|*norm_j picks i, ties to i;
 *   masks (Eq. 4): saliency mask OR similarity mask;
 *   merged (Eq. 5): mean magnitude where similar, else the salient expert's magnitude;
 *       the mean is formed in fp32 and rounded to bf16 to nearest even.
 * Returns the number of similar elements.
 */
int64_t orc_merge(const uint16_t *wi, const uint16_t *wj, const float *norm_i, const float *norm_j,
                  int64_t rows, int64_t cols, float tau,
                  uint16_t *merged, uint8_t *mask_i, uint8_t *mask_j, uint8_t *sign_i, uint8_t *sign_j)
{
    int64_t n_sim = 0;
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t c = 0; c < cols; ++c) {
            int64_t k = r * cols + c;
            float a = fabsf(bf16_to_float(wi[k])), b = fabsf(bf16_to_float(wj[k]));
            volatile float diff = fabsf(a - b);            /* volatile: one rounding per operation, */
            volatile float sum = a + b;                    /* never contracted into an fma          */
            volatile float thr = tau * sum;
            int sim = (sum > 0.0f) && (diff <= thr);
            volatile float sal_i = a * norm_i[c];
            volatile float sal_j = b * norm_j[c];
            int pick_i = sal_i >= sal_j;
            float mag;
            if (sim) { volatile float half = sum * 0.5f; mag = half; }
            else     mag = pick_i ? a : b;
            merged[k] = orc_bf16_from_double((double)mag);
            mask_i[k] = (uint8_t)(sim || pick_i);
            mask_j[k] = (uint8_t)(sim || !pick_i);
            sign_i[k] = (uint8_t)((wi[k] & 0x8000) && (wi[k] & 0x7FFF));   /* w < 0: -0 is not negative */
            sign_j[k] = (uint8_t)((wj[k] & 0x8000) && (wj[k] & 0x7FFF));
            n_sim += sim;
        }
    }
    return n_sim;
}

/* ---------- router: logits, top-k, softmax over the selected logits ---------- */

/*
 * x [T,d] bf16 bits, w_router [E,d] bf16 bits (row-major).  logits[t,e] = sum_c x[t,c]*w[e,c]
 * as acc = fmaf(x, w, acc) for c = 0..d-1 in fp32.  ids[t,0..k) are the k largest logits in
 * descending order (ties: lower expert first); weights[t,:] = softmax of those k logits,
 * computed in fp64 from the fp32 logits and returned as fp32.  Optionally returns the logits.
 */
int orc_router_topk(int T, int d, int E, int k, const uint16_t *x, const uint16_t *w_router,
                    int32_t *ids, float *weights, float *logits_out)
{
    if (k > E || k < 1) return -1;
    float *logit = malloc(sizeof(float) * E);
    char *taken = malloc(E);
    if (!logit || !taken) { free(logit); free(taken); return -1; }
    for (int t = 0; t < T; ++t) {
        for (int e = 0; e < E; ++e) {
            float acc = 0.0f;
            for (int c = 0; c < d; ++c)
                acc = fmaf(bf16_to_float(x[(int64_t)t * d + c]), bf16_to_float(w_router[(int64_t)e * d + c]), acc);
            logit[e] = acc;
            if (logits_out) logits_out[(int64_t)t * E + e] = acc;
        }
        memset(taken, 0, E);
        double sel[64];
        for (int j = 0; j < k; ++j) {
            int best = -1;
            for (int e = 0; e < E; ++e)
                if (!taken[e] && (best < 0 || logit[e] > logit[best])) best = e;   /* strict >: lower index wins ties */
            taken[best] = 1;
            ids[(int64_t)t * k + j] = best;
            if (j < 64) sel[j] = (double)logit[best];
        }
        double mx = sel[0], sum = 0.0;
        for (int j = 0; j < k && j < 64; ++j) sum += exp(sel[j] - mx);
        for (int j = 0; j < k && j < 64; ++j) weights[(int64_t)t * k + j] = (float)(exp(sel[j] - mx) / sum);
    }
    free(logit); free(taken);
    return 0;
}
