/*
 * Host-side sanitizer driver (TEST INFRASTRUCTURE): linked with oracle/nsml_oracle.c and the
 * host C of the library (csrc/nsml_ctl.c), all built with -fsanitize=address,undefined, and
 * run as a plain process (no Python inside it).  Every output buffer is allocated at exactly
 * the size the layout functions report, so an overrun of one byte is caught.  Exit status 0 =
 * no finding and every cross-check held.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "nsml.h"

uint64_t orc_k(double ratio, uint64_t n);
int orc_layout(const uint64_t *off, uint32_t B, double ratio, int bits, uint32_t chunk,
               uint64_t *k_b, uint64_t *K, uint64_t *val_bytes, uint64_t *n_scales);
int orc_compress(const float *g, float *r, uint64_t n, const uint64_t *off, uint32_t B, double ratio,
                 int bits, uint32_t chunk, uint32_t *idx, void *val, float *scales, int nthreads);
int orc_decompress(const uint32_t *idx, const void *val, const float *scales, uint64_t n,
                   const uint64_t *off, uint32_t B, double ratio, int bits, uint32_t chunk,
                   float *dense, int nthreads);
int orc_compress_pruned(const float *g, float *r, const float *w, uint64_t n, const uint64_t *off,
                        uint32_t B, double ratio, int bits, uint32_t chunk, uint32_t *idx,
                        void *val, float *scales, int nthreads);
int orc_decompress_accumulate(const uint32_t *idx, const void *val, const float *scales, uint64_t n,
                              const uint64_t *off, uint32_t B, double ratio, int bits,
                              uint32_t chunk, float *dense);
double orc_l2norm(const float *g, const uint64_t *off, uint32_t B, double *per_bucket);

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(void)
{
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
    return (uint32_t)(rng_state >> 32);
}
static float rndf(void) { return ((float)(rnd() % 2001) - 1000.0f) * 1e-4f; }   /* many ties, zeros */

#define CHECK(c) do { if (!(c)) { fprintf(stderr, "sanitize_driver: %s failed at line %d\n", #c, __LINE__); return 1; } } while (0)

static void *exact(size_t bytes) { return malloc(bytes ? bytes : 1); }

static int one_case(const uint64_t *off, uint32_t B, double ratio, int bits, uint32_t chunk, int pruned)
{
    const uint64_t n = off[B];
    uint64_t K = 0, vb = 0, ns = 0, K2 = 0, vb2 = 0, ns2 = 0;
    uint64_t *kb = (uint64_t *)exact(B * sizeof(uint64_t)), *kb2 = (uint64_t *)exact(B * sizeof(uint64_t));
    CHECK(orc_layout(off, B, ratio, bits, chunk, kb, &K, &vb, &ns) == 0);
    CHECK(nsml_payload_layout(off, B, ratio, bits, chunk, kb2, &K2, &vb2, &ns2) == NSML_OK);
    CHECK(K == K2 && vb == vb2 && ns == ns2 && memcmp(kb, kb2, B * sizeof(uint64_t)) == 0);
    float *g = (float *)exact(n * 4), *r = (float *)exact(n * 4), *w = (float *)exact(n * 4);
    float *acc = (float *)exact(n * 4), *dense = (float *)exact(n * 4);
    for (uint64_t i = 0; i < n; ++i) { g[i] = rndf(); r[i] = rndf(); w[i] = rndf(); acc[i] = g[i] + r[i]; }
    uint32_t *idx = (uint32_t *)exact(K * 4);
    uint8_t *val = (uint8_t *)exact(vb);
    float *sc = (float *)exact(ns * 4);
    int rc = pruned ? orc_compress_pruned(g, r, w, n, off, B, ratio, bits, chunk, idx, val, sc, 2)
                    : orc_compress(g, r, n, off, B, ratio, bits, chunk, idx, val, sc, 2);
    CHECK(rc == 0);
    CHECK(orc_decompress(idx, val, sc, n, off, B, ratio, bits, chunk, dense, 2) == 0);
    /* conservation law, element by element */
    for (uint64_t i = 0; i < n; ++i) { volatile float s = dense[i] + r[i]; CHECK(s == acc[i]); }
    /* indices ascending and inside each bucket */
    uint64_t p = 0;
    for (uint32_t b = 0; b < B; ++b)
        for (uint64_t j = 0; j < kb[b]; ++j, ++p) {
            CHECK(idx[p] < off[b + 1] - off[b]);
            if (j) CHECK(idx[p] > idx[p - 1]);
        }
    CHECK(p == K);
    /* receiver side: twice the payload on top of a constant */
    for (uint64_t i = 0; i < n; ++i) acc[i] = 0.5f;
    CHECK(orc_decompress_accumulate(idx, val, sc, n, off, B, ratio, bits, chunk, acc) == 0);
    for (uint64_t i = 0; i < n; ++i) { volatile float s = 0.5f + dense[i]; CHECK(acc[i] == s); }
    double *per = (double *)exact(B * sizeof(double));
    const double tot = orc_l2norm(g, off, B, per);
    double sq = 0.0;
    for (uint32_t b = 0; b < B; ++b) sq += per[b] * per[b];
    CHECK(fabs(sqrt(sq) - tot) <= 1e-9 * (tot + 1e-30));
    free(kb); free(kb2); free(g); free(r); free(w); free(acc); free(dense); free(idx); free(val); free(sc); free(per);
    return 0;
}

static int controller(int win_bw, int win_rt, int steps)
{
    nsml_ctl_params p;
    CHECK(nsml_ctl_default_params(&p) == NSML_OK);
    p.win_bw = win_bw; p.win_rt = win_rt;
    nsml_ctl_state *s = (nsml_ctl_state *)exact(sizeof *s);     /* heap: red zones on both sides */
    CHECK(nsml_ctl_init(s, &p) == NSML_OK);
    double bytes = 0.0, secs = 0.0;
    for (int i = 0; i < steps; ++i) {
        double ratio = 0.0; int bits = 0;
        CHECK(nsml_choose_ratio(s, bytes, secs, 1e8, (i % 3) ? -1.0 : 2.5, &ratio, &bits) == NSML_OK);
        CHECK(ratio > 0.0 && ratio <= 1.0 && (bits == 4 || bits == 8 || bits == 16 || bits == 32));
        bytes = ratio * 1e8 * (4.0 + bits / 8.0);
        secs = 0.01 + bytes / (1e8 * (1.0 + (double)(rnd() % 100)));
    }
    /* the state is plain data: a copy continues identically */
    nsml_ctl_state *c = (nsml_ctl_state *)exact(sizeof *c);
    memcpy(c, s, sizeof *s);
    double r1, r2; int b1, b2;
    CHECK(nsml_choose_ratio(s, bytes, secs, 1e8, -1.0, &r1, &b1) == NSML_OK);
    CHECK(nsml_choose_ratio(c, bytes, secs, 1e8, -1.0, &r2, &b2) == NSML_OK);
    CHECK(r1 == r2 && b1 == b2);
    p.win_bw = NSML_CTL_MAX_WIN + 1;
    CHECK(nsml_ctl_init(c, &p) == NSML_EINVAL);
    free(s); free(c);
    return 0;
}

int main(void)
{
    /* ragged layouts: empty buckets, n = 1, odd survivor counts (4-bit tail), unaligned starts */
    const uint64_t l1[] = {0, 1};
    const uint64_t l2[] = {0, 0, 5, 5, 6, 4103, 4103};
    const uint64_t l3[] = {0, 3, 1003, 1010, 9999};
    const uint64_t l4[] = {0, 17};
    const struct { const uint64_t *off; uint32_t B; } layouts[] = {{l1, 1}, {l2, 6}, {l3, 4}, {l4, 1}};
    const double ratios[] = {1.0, 0.5, 0.3, 0.05, 0.001};
    const int widths[] = {4, 8, 16, 32};
    const uint32_t chunks[] = {8, 64, 2048};
    int cases = 0;
    for (unsigned a = 0; a < sizeof layouts / sizeof layouts[0]; ++a)
        for (unsigned b = 0; b < sizeof ratios / sizeof ratios[0]; ++b)
            for (unsigned c = 0; c < sizeof widths / sizeof widths[0]; ++c)
                for (unsigned d = 0; d < sizeof chunks / sizeof chunks[0]; ++d)
                    for (int pruned = 0; pruned < 2; ++pruned, ++cases)
                        if (one_case(layouts[a].off, layouts[a].B, ratios[b], widths[c], chunks[d], pruned)) return 1;
    /* argument errors are returned, nothing is touched */
    uint64_t K;
    if (nsml_payload_layout(l3, 4, 0.0, 8, 2048, NULL, &K, NULL, NULL) != NSML_EINVAL) return 1;
    if (nsml_payload_layout(l3, 4, 0.5, 8, 12, NULL, &K, NULL, NULL) != NSML_EINVAL) return 1;
    if (nsml_payload_layout(l3, 4, 0.5, 7, 2048, NULL, &K, NULL, NULL) != NSML_EINVAL) return 1;
    if (controller(10, 100, 700) || controller(0, 0, 700) || controller(NSML_CTL_MAX_WIN, NSML_CTL_MAX_WIN, 1000) ||
        controller(1, 1, 300))
        return 1;
    printf("sanitize_driver: %d compress/decompress cases and 4 controller runs clean\n", cases);
    return 0;
}
