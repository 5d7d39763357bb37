/*
 * Drives every entry point of the CPU oracle on small inputs held in exactly-sized heap
 * buffers.  Built by tests/test_oracle_sanitizers.py together with the sources under oracle/ under
 * -fsanitize=address,undefined: an out-of-bounds access, a signed overflow or a bad shift in
 * the oracle ends the program with a report.  Test infrastructure only.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int64_t orc_pack(const uint16_t *, const uint8_t *, const uint8_t *, const uint8_t *, const uint8_t *, int64_t, uint16_t *);
void orc_unpack(const uint16_t *, int, int64_t, uint16_t *);
uint16_t orc_bf16_from_double(double);
double orc_bf16_to_double(uint16_t);
int orc_moe_ffn(int, int, int, int, int, const uint16_t *, const int32_t *, const float *, const int32_t *,
                const uint8_t *, const uint16_t *const *, const uint16_t *const *, const uint16_t *const *, int,
                const uint16_t *const *, const uint16_t *const *, const uint16_t *const *, int, const int32_t *,
                const uint16_t *const *, const uint16_t *const *, const uint16_t *const *, int, double *, uint16_t *);
int64_t orc_merge(const uint16_t *, const uint16_t *, const float *, const float *, int64_t, int64_t, float,
                  uint16_t *, uint8_t *, uint8_t *, uint8_t *, uint8_t *);
int orc_router_topk(int, int, int, int, const uint16_t *, const uint16_t *, int32_t *, float *, float *);
int64_t orc_q_quantise(const uint16_t *, const uint8_t *, const uint8_t *, const uint8_t *, const uint8_t *, int64_t,
                       int64_t, uint8_t *, uint8_t *, uint8_t *, uint8_t *, uint16_t *);
void orc_q_dequantise(const uint8_t *, const uint8_t *, const uint8_t *, const uint8_t *, const uint16_t *, int,
                      int64_t, int64_t, double *);
void orc_q_records(const uint8_t *, const uint8_t *, const uint8_t *, const uint8_t *, int64_t, int64_t, uint64_t *);
int orc_ffn_dense64(int, int, int, int, int, const uint16_t *, const int32_t *, const float *, const double *const *,
                    const double *const *, const double *const *, double *);

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(void)
{
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
    return (uint32_t)(rng_state >> 32);
}
static double rnd_unit(void) { return (double)rnd() / 4294967296.0 - 0.5; }

static uint16_t *rand_bf16(size_t n, double scale)
{
    uint16_t *p = malloc(n * sizeof *p);
    for (size_t i = 0; i < n; ++i) p[i] = orc_bf16_from_double(rnd_unit() * scale);
    return p;
}
static uint8_t *rand_bits(size_t n)
{
    uint8_t *p = malloc(n);
    for (size_t i = 0; i < n; ++i) p[i] = rnd() & 1;
    return p;
}

int main(void)
{
    /* pack / unpack over every 16-bit pattern as the merged input, every flag combination */
    enum { NW = 65536 };
    uint16_t *all = malloc(NW * sizeof *all), *packed = malloc(NW * sizeof *packed), *dec = malloc(NW * sizeof *dec);
    uint8_t *m0 = rand_bits(NW), *m1 = rand_bits(NW), *s0 = rand_bits(NW), *s1 = rand_bits(NW);
    for (int i = 0; i < NW; ++i) all[i] = (uint16_t)i;
    int64_t bad = orc_pack(all, m0, m1, s0, s1, NW, packed);
    orc_unpack(packed, 0, NW, dec);
    orc_unpack(all, 1, NW, dec);                    /* every word as a packed word too */
    (void)orc_bf16_from_double(1e300); (void)orc_bf16_from_double(-1e-300); (void)orc_bf16_from_double(0.0 / 1.0);
    free(all); free(dec); free(m0); free(m1); free(s0); free(s1);

    /* a small layer: 2 pairs + 1 unmerged expert + 1 shared expert */
    const int d = 64, f = 96, fs = 32, T = 5, k = 3, E = 5;
    const size_t nfd = (size_t)f * d;
    uint16_t *g[2], *u[2], *dn[2];
    for (int p = 0; p < 2; ++p) {
        uint16_t **dst[3] = {&g[p], &u[p], &dn[p]};
        for (int w = 0; w < 3; ++w) {
            uint16_t *mg = rand_bf16(nfd, 0.08);
            uint8_t *a = rand_bits(nfd), *b = rand_bits(nfd), *c = rand_bits(nfd), *e = rand_bits(nfd);
            *dst[w] = malloc(nfd * sizeof(uint16_t));
            bad += orc_pack(mg, a, b, c, e, (int64_t)nfd, *dst[w]);
            free(mg); free(a); free(b); free(c); free(e);
        }
    }
    uint16_t *dg = rand_bf16(nfd, 0.08), *du = rand_bf16(nfd, 0.08), *dd = rand_bf16(nfd, 0.08);
    uint16_t *sg = rand_bf16((size_t)fs * d, 0.08), *su = rand_bf16((size_t)fs * d, 0.08), *sd = rand_bf16((size_t)fs * d, 0.08);
    uint16_t *x = rand_bf16((size_t)T * d, 2.0);
    int32_t *ids = malloc(sizeof(int32_t) * T * k);
    float *w = malloc(sizeof(float) * T * k);
    for (int i = 0; i < T * k; ++i) { ids[i] = (int32_t)(rnd() % E); w[i] = (float)(rnd_unit() + 0.5); }
    const int32_t pair[5] = {0, 1, -1, 1, 0};
    const uint8_t pos[5] = {0, 1, 0, 0, 1};
    const uint16_t *gp[2] = {g[0], g[1]}, *up[2] = {u[0], u[1]}, *dp[2] = {dn[0], dn[1]};
    const uint16_t *dgp[1] = {dg}, *dup_[1] = {du}, *ddp[1] = {dd}, *sgp[1] = {sg}, *sup[1] = {su}, *sdp[1] = {sd};
    const int32_t shared_f[1] = {fs};
    double *y64 = malloc(sizeof(double) * T * d);
    uint16_t *ybf = malloc(sizeof(uint16_t) * T * d);
    int rc = 0;
    for (int stage = 0; stage < 2; ++stage)
        rc |= orc_moe_ffn(T, k, E, d, f, x, ids, w, pair, pos, gp, up, dp, 1, dgp, dup_, ddp, 1, shared_f, sgp, sup, sdp,
                          stage, y64, ybf);
    ids[1] = E;                                     /* an id out of range must be refused, not read */
    if (orc_moe_ffn(T, k, E, d, f, x, ids, w, pair, pos, gp, up, dp, 1, dgp, dup_, ddp, 1, shared_f, sgp, sup, sdp,
                    0, y64, ybf) == 0) rc |= 2;
    ids[1] = 0;

    /* merge */
    const int64_t mr = 48, mc = 64;
    uint16_t *wi = rand_bf16((size_t)(mr * mc), 0.08), *wj = rand_bf16((size_t)(mr * mc), 0.08);
    wi[3] = 0; wj[3] = 0x8000; wi[7] = 0x7F80; wj[9] = 0x7FC1;   /* zeros, an infinity, a NaN */
    float *ni = malloc(sizeof(float) * mc), *nj = malloc(sizeof(float) * mc);
    for (int c = 0; c < mc; ++c) { ni[c] = (float)(rnd_unit() + 1.0); nj[c] = (float)(rnd_unit() + 1.0); }
    uint16_t *mg = malloc(sizeof(uint16_t) * mr * mc);
    uint8_t *pl[4];
    for (int i = 0; i < 4; ++i) pl[i] = malloc((size_t)(mr * mc));
    (void)orc_merge(wi, wj, ni, nj, mr, mc, 0.4f, mg, pl[0], pl[1], pl[2], pl[3]);

    /* router */
    const int RE = 7, rk = 3;
    uint16_t *wr = rand_bf16((size_t)RE * d, 0.2);
    int32_t *rid = malloc(sizeof(int32_t) * T * rk);
    float *rw = malloc(sizeof(float) * T * rk), *rl = malloc(sizeof(float) * T * RE);
    rc |= orc_router_topk(T, d, RE, rk, x, wr, rid, rw, rl);
    if (orc_router_topk(T, d, RE, RE + 1, x, wr, rid, rw, NULL) == 0) rc |= 4;   /* k > E is refused before any write */

    /* quantised variant */
    const int64_t qr = 32, qc = 256;
    uint16_t *qm = rand_bf16((size_t)(qr * qc), 0.08);
    qm[5] = 0x7F80;
    uint8_t *qa = rand_bits((size_t)(qr * qc)), *qb = rand_bits((size_t)(qr * qc)), *qs0 = rand_bits((size_t)(qr * qc)),
            *qs1 = rand_bits((size_t)(qr * qc));
    uint8_t *code = malloc((size_t)(qr * qc)), *trit = malloc((size_t)(qr * qc)), *o0 = malloc((size_t)(qr * qc)),
            *o1 = malloc((size_t)(qr * qc));
    uint16_t *scale = malloc(sizeof(uint16_t) * qr * (qc / 128));
    (void)orc_q_quantise(qm, qa, qb, qs0, qs1, qr, qc, code, trit, o0, o1, scale);
    double *deq = malloc(sizeof(double) * qr * qc);
    orc_q_dequantise(code, trit, o0, o1, scale, 0, qr, qc, deq);
    orc_q_dequantise(code, trit, o0, o1, scale, 1, qr, qc, deq);
    uint64_t *rec = malloc(sizeof(uint64_t) * qr * (qc / 8));
    orc_q_records(code, trit, o0, o1, qr, qc, rec);

    /* dense fp64 FFN */
    double *Wg = malloc(sizeof(double) * nfd), *Wu = malloc(sizeof(double) * nfd), *Wd = malloc(sizeof(double) * nfd);
    for (size_t i = 0; i < nfd; ++i) { Wg[i] = rnd_unit(); Wu[i] = rnd_unit(); Wd[i] = rnd_unit(); }
    const double *Wgp[2] = {Wg, Wu}, *Wup[2] = {Wu, Wd}, *Wdp[2] = {Wd, Wg};
    for (int i = 0; i < T * k; ++i) ids[i] = (int32_t)(rnd() % 2);
    rc |= orc_ffn_dense64(T, k, 2, d, f, x, ids, w, Wgp, Wup, Wdp, y64);

    for (int p = 0; p < 2; ++p) { free(g[p]); free(u[p]); free(dn[p]); }
    free(packed); free(dg); free(du); free(dd); free(sg); free(su); free(sd); free(x); free(ids); free(w);
    free(y64); free(ybf); free(wi); free(wj); free(ni); free(nj); free(mg);
    for (int i = 0; i < 4; ++i) free(pl[i]);
    free(wr); free(rid); free(rw); free(rl); free(qm); free(qa); free(qb); free(qs0); free(qs1);
    free(code); free(trit); free(o0); free(o1); free(scale); free(deq); free(rec); free(Wg); free(Wu); free(Wd);
    printf("oracle sanitizer drive: rc=%d out_of_range=%lld\n", rc, (long long)bad);
    return rc;
}
