/*
 * nsml_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain, slow, single-pass-per-definition CPU statement of what one
 * NetSenseML worker does to its own gradient before communication
 * (Algorithm 2 Step 3, the sparsification step, with the local accumulation of
 * the filtered part described in Sec. 4.2 Step 3), plus
 * the low-bit value coding, the index/value/scale payload and the inverse
 * decompress-and-scatter that the build contract adds around it.
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may load
 * this library.  It shares no source, header, table or helper with the HIP
 * path and is never used to produce a product result.
 *
 * Top-k here is the definition itself: a full sort of every element of a
 * bucket by (magnitude key descending, index ascending) and a cut after k.
 * There is no blocking, no histogram, no selection algorithm.
 *
 * Arithmetic: every floating-point step is one IEEE-754 binary32 operation
 * (add, divide, multiply, subtract, round-to-nearest-even to integer), no
 * fused multiply-add, subnormals kept.  Build with
 *   gcc -O2 -fno-fast-math -ffp-contract=off -fopenmp -shared -fPIC
 *
 * Parity pins live in tests/ (-m "not gpu"): rank-definition brute force,
 * exhaustive tie patterns, identity at ratio=1/bits=32, the error-feedback
 * conservation law, quantizer error bounds, numpy's binary16 conversion.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_EINVAL (-1)
#define ORC_ENOMEM (-5)

/* ---------------------------------------------------------------- helpers */

static uint32_t f32_bits(float x) { uint32_t u; memcpy(&u, &x, 4); return u; }
static float bits_f32(uint32_t u) { float x; memcpy(&x, &u, 4); return x; }

/* Magnitude key: the binary32 pattern with the sign cleared.  For finite
 * values the unsigned order of keys is the order of |x|; +0 and -0 tie. */
static uint32_t mag_key(float x) { return f32_bits(x) & 0x7FFFFFFFu; }

static int qmax_of(int bits) { return bits == 8 ? 127 : (bits == 4 ? 7 : 0); }

/* binary32 -> binary16, round to nearest even, written out by cases
 * (Sec. 4.2 Step 1: the paper's quantizer is the 32-bit to 16-bit float cast). */
static uint16_t f32_to_f16(float x)
{
    uint32_t u = f32_bits(x);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    uint32_t a = u & 0x7FFFFFFFu;
    if (a > 0x7F800000u) return (uint16_t)(sign | 0x7E00u);           /* NaN */
    if (a >= 0x477FF000u) return (uint16_t)(sign | 0x7C00u);          /* >= 65520 -> inf (incl. inf) */
    if (a < 0x33000000u) return sign;                                 /* < 2^-25 -> 0 */
    int e = (int)(a >> 23) - 127;                                     /* unbiased exponent */
    uint32_t man = (a & 0x007FFFFFu) | 0x00800000u;                   /* 24-bit significand */
    int shift;                                                        /* bits dropped from man */
    uint32_t base;                                                    /* half pattern before adding kept bits */
    if (e >= -14) { shift = 13; base = (uint32_t)(e + 15) << 10; man &= 0x007FFFFFu; }
    else          { shift = 13 + (-14 - e); base = 0; }               /* subnormal half */
    uint32_t kept = man >> shift;
    uint32_t rem  = man & ((1u << shift) - 1u);
    uint32_t half = 1u << (shift - 1);
    uint32_t h = base + kept;
    if (rem > half || (rem == half && (kept & 1u))) h += 1u;          /* carries propagate correctly */
    return (uint16_t)(sign | h);
}

static float f16_to_f32(uint16_t h)
{
    uint32_t sign = ((uint32_t)h & 0x8000u) << 16;
    uint32_t e = (h >> 10) & 0x1Fu, m = h & 0x3FFu;
    if (e == 0x1Fu) return bits_f32(sign | 0x7F800000u | (m << 13));
    if (e == 0) {
        if (m == 0) return bits_f32(sign);
        float v = ldexpf((float)m, -24);                              /* exact */
        return sign ? -v : v;
    }
    return bits_f32(sign | ((e + 112u) << 23) | (m << 13));
}

/* ------------------------------------------------------------------ sizes */

/* Algorithm 2, Step 3: top_k(grads, ratio) keeps k = ceil(ratio * n) entries,
 * at least one, at most n.  The product is an IEEE double product. */
uint64_t orc_k(double ratio, uint64_t n)
{
    if (n == 0) return 0;
    double kd = ceil(ratio * (double)n);
    uint64_t k = kd < 1.0 ? 1u : (kd >= (double)n ? n : (uint64_t)kd);
    return k;
}

static uint64_t val_bytes_of(uint64_t k, int bits)
{
    switch (bits) {
    case 32: return 4 * k;
    case 16: return 2 * k;
    case 8:  return k;
    case 4:  return (k + 1) / 2;
    default: return 0;
    }
}

/* Payload geometry for a bucketed gradient.  Every bucket's value region
 * starts on a byte boundary; scales exist only for the integer codes, one per
 * `chunk` consecutive survivors of a bucket. */
int orc_layout(const uint64_t *off, uint32_t B, double ratio, int bits, uint32_t chunk,
               uint64_t *k_b, uint64_t *K, uint64_t *val_bytes, uint64_t *n_scales)
{
    if (!off || B == 0 || chunk == 0) return ORC_EINVAL;
    if (!(ratio > 0.0 && ratio <= 1.0)) return ORC_EINVAL;
    if (bits != 4 && bits != 8 && bits != 16 && bits != 32) return ORC_EINVAL;
    uint64_t Ks = 0, vb = 0, ns = 0;
    for (uint32_t b = 0; b < B; ++b) {
        if (off[b + 1] < off[b]) return ORC_EINVAL;
        uint64_t nb = off[b + 1] - off[b];
        uint64_t k = orc_k(ratio, nb);
        if (k_b) k_b[b] = k;
        Ks += k;
        vb += val_bytes_of(k, bits);
        if (bits == 8 || bits == 4) ns += (k + chunk - 1) / chunk;
    }
    if (K) *K = Ks;
    if (val_bytes) *val_bytes = vb;
    if (n_scales) *n_scales = ns;
    return ORC_OK;
}

/* ----------------------------------------------------------- one bucket */

typedef struct { uint32_t key; uint32_t idx; } keyed;

static int by_key_desc_then_idx_asc(const void *pa, const void *pb)
{
    const keyed *a = (const keyed *)pa, *b = (const keyed *)pb;
    if (a->key != b->key) return a->key > b->key ? -1 : 1;
    if (a->idx != b->idx) return a->idx < b->idx ? -1 : 1;
    return 0;
}

static int by_u32_asc(const void *pa, const void *pb)
{
    uint32_t a = *(const uint32_t *)pa, b = *(const uint32_t *)pb;
    return a < b ? -1 : (a > b ? 1 : 0);
}

/*
 * Compress one bucket of n elements.
 *   g      gradient, read only
 *   r      residual, in: what earlier steps did not send; out: what this step
 *          does not send (Sec. 4.2 Step 3: the filtered gradients are
 *          accumulated locally for later aggregation)
 *   idx    k bucket-local indices, ascending
 *   val    k values: f32 (bits 32), binary16 patterns (16), int8 codes (8),
 *          two's-complement nibbles two per byte, even survivor in the low
 *          nibble (4)
 *   scales one f32 per chunk of `chunk` consecutive survivors (bits 8 and 4)
 * Returns k (>= 0) or a negative error.
 */
int64_t orc_compress_bucket(const float *g, float *r, uint64_t n, double ratio, int bits,
                            uint32_t chunk, uint32_t *idx, void *val, float *scales)
{
    if (n == 0) return 0;
    if (!g || !r || !idx || !val || n > 0xFFFFFFFFull || chunk == 0) return ORC_EINVAL;
    if (!(ratio > 0.0 && ratio <= 1.0)) return ORC_EINVAL;
    if (bits != 4 && bits != 8 && bits != 16 && bits != 32) return ORC_EINVAL;
    if ((bits == 4 || bits == 8) && !scales) return ORC_EINVAL;

    /* 1. error-feedback accumulation: a = g + r, one binary32 add per element */
    for (uint64_t i = 0; i < n; ++i) {
        volatile float a = g[i] + r[i];
        r[i] = a;
    }

    /* 2. k */
    uint64_t k = orc_k(ratio, n);

    /* 3. select: full sort by (|a| descending, index ascending), keep the first
     *    k, then list them by ascending index */
    keyed *order = (keyed *)malloc(n * sizeof(keyed));
    if (!order) return ORC_ENOMEM;
    for (uint64_t i = 0; i < n; ++i) { order[i].key = mag_key(r[i]); order[i].idx = (uint32_t)i; }
    qsort(order, n, sizeof(keyed), by_key_desc_then_idx_asc);
    for (uint64_t j = 0; j < k; ++j) idx[j] = order[j].idx;
    free(order);
    qsort(idx, k, sizeof(uint32_t), by_u32_asc);

    /* 4.-6. gather, code the values, leave the coding error in the residual */
    const int qmax = qmax_of(bits);
    uint64_t n_chunks = (k + chunk - 1) / chunk;
    if (bits == 4) memset(val, 0, (k + 1) / 2);
    for (uint64_t c = 0; c < n_chunks; ++c) {
        uint64_t j0 = c * (uint64_t)chunk;
        uint64_t j1 = j0 + chunk < k ? j0 + chunk : k;
        float scale = 0.0f;
        if (qmax) {
            float m = 0.0f;
            for (uint64_t j = j0; j < j1; ++j) {
                float av = bits_f32(mag_key(r[idx[j]]));
                if (av > m) m = av;
            }
            volatile float s = m / (float)qmax;       /* IEEE binary32 divide */
            scale = (m == 0.0f) ? 0.0f : s;
            scales[c] = scale;
        }
        for (uint64_t j = j0; j < j1; ++j) {
            float v = r[idx[j]];
            float deq;
            if (bits == 32) {
                ((float *)val)[j] = v;
                deq = v;
            } else if (bits == 16) {
                uint16_t h = f32_to_f16(v);
                ((uint16_t *)val)[j] = h;
                deq = f16_to_f32(h);
            } else {
                int q = 0;
                if (scale != 0.0f) {
                    volatile float t = v / scale;     /* IEEE binary32 divide */
                    float rt = rintf(t);              /* ties to even (default mode) */
                    if (rt > (float)qmax) rt = (float)qmax;
                    if (rt < (float)-qmax) rt = (float)-qmax;
                    q = (int)rt;
                }
                if (bits == 8) ((int8_t *)val)[j] = (int8_t)q;
                else {
                    uint8_t nib = (uint8_t)(q & 0xF);
                    uint8_t *p = (uint8_t *)val + (j >> 1);
                    *p = (j & 1) ? (uint8_t)(*p | (nib << 4)) : (uint8_t)(*p | nib);
                }
                volatile float d = (float)q * scale;  /* one binary32 multiply */
                deq = d;
            }
            volatile float res = v - deq;             /* one binary32 subtract */
            r[idx[j]] = res;
        }
    }
    return (int64_t)k;
}

/* ------------------------------------------------- with model pruning */

/* Algorithm 2 Step 2: pruning_rate = 0.5 * (1 - ratio); the parameters with the smallest
 * |weight| are pruned and their gradients take no part in the sparsification that follows.
 * Reading taken here: floor(rate * n) parameters of the bucket are pruned; the kept set is the
 * n - floor(rate * n) largest |weight| with the same tie rule as the gradient selection (equal
 * magnitudes: lower index kept first); pruned parameters are not removed for good -- their
 * accumulated gradient stays in the residual and they may come back in a later step. */
uint64_t orc_pruned_count(double ratio, uint64_t n)
{
    double np = floor(0.5 * (1.0 - ratio) * (double)n);
    if (np < 0.0) np = 0.0;
    return (uint64_t)np;
}

/* eligible[i] = 1 for the kept parameters of one bucket */
int orc_keep_mask(const float *w, uint64_t n, double ratio, uint8_t *eligible)
{
    if (n == 0) return ORC_OK;
    if (!w || !eligible || n > 0xFFFFFFFFull) return ORC_EINVAL;
    uint64_t m = n - orc_pruned_count(ratio, n);
    keyed *order = (keyed *)malloc(n * sizeof(keyed));
    if (!order) return ORC_ENOMEM;
    for (uint64_t i = 0; i < n; ++i) { order[i].key = mag_key(w[i]); order[i].idx = (uint32_t)i; }
    qsort(order, n, sizeof(keyed), by_key_desc_then_idx_asc);
    memset(eligible, 0, n);
    for (uint64_t j = 0; j < m; ++j) eligible[order[j].idx] = 1;
    free(order);
    return ORC_OK;
}

/* As orc_compress_bucket, but only the parameters kept by the pruning step can be selected. */
int64_t orc_compress_bucket_pruned(const float *g, float *r, const float *w, uint64_t n,
                                   double ratio, int bits, uint32_t chunk, uint32_t *idx,
                                   void *val, float *scales)
{
    if (n == 0) return 0;
    if (!g || !r || !w || !idx || !val || n > 0xFFFFFFFFull || chunk == 0) return ORC_EINVAL;
    if (!(ratio > 0.0 && ratio <= 1.0)) return ORC_EINVAL;
    uint8_t *eligible = (uint8_t *)malloc(n);
    if (!eligible) return ORC_ENOMEM;
    int rc = orc_keep_mask(w, n, ratio, eligible);
    if (rc != ORC_OK) { free(eligible); return rc; }

    /* accumulate, then select among the kept parameters only */
    for (uint64_t i = 0; i < n; ++i) { volatile float acc = g[i] + r[i]; r[i] = acc; }
    uint64_t k = orc_k(ratio, n), m = 0;
    keyed *order = (keyed *)malloc(n * sizeof(keyed));
    if (!order) { free(eligible); return ORC_ENOMEM; }
    for (uint64_t i = 0; i < n; ++i)
        if (eligible[i]) { order[m].key = mag_key(r[i]); order[m].idx = (uint32_t)i; ++m; }
    free(eligible);
    if (m < k) { free(order); return ORC_EINVAL; }      /* cannot happen: kept >= (1 + ratio) n / 2 >= k */
    qsort(order, m, sizeof(keyed), by_key_desc_then_idx_asc);
    for (uint64_t j = 0; j < k; ++j) idx[j] = order[j].idx;
    free(order);
    qsort(idx, k, sizeof(uint32_t), by_u32_asc);

    /* from here on nothing differs from the unpruned path: code the gathered values and leave
     * the coding error in the residual.  Done by handing the survivors to the plain routine on
     * a compact copy: a bucket that consists of exactly the survivors, at ratio 1. */
    float *gv = (float *)malloc(k * sizeof(float)), *rv = (float *)calloc(k, sizeof(float));
    uint32_t *tmp_idx = (uint32_t *)malloc(k * sizeof(uint32_t));
    if (!gv || !rv || !tmp_idx) { free(gv); free(rv); free(tmp_idx); return ORC_ENOMEM; }
    for (uint64_t j = 0; j < k; ++j) gv[j] = r[idx[j]];
    int64_t kk = orc_compress_bucket(gv, rv, k, 1.0, bits, chunk, tmp_idx, val, scales);
    if (kk == (int64_t)k)
        for (uint64_t j = 0; j < k; ++j) r[idx[j]] = rv[j];
    free(gv); free(rv); free(tmp_idx);
    return kk == (int64_t)k ? (int64_t)k : ORC_EINVAL;
}

int orc_compress_pruned(const float *g, float *r, const float *w, uint64_t n, const uint64_t *off,
                        uint32_t B, double ratio, int bits, uint32_t chunk, uint32_t *idx,
                        void *val, float *scales, int nthreads)
{
    if (!off || B == 0 || off[0] != 0 || off[B] != n) return ORC_EINVAL;
    uint64_t *P = (uint64_t *)malloc(3 * (size_t)(B + 1) * sizeof(uint64_t));
    if (!P) return ORC_ENOMEM;
    uint64_t *V = P + (B + 1), *S = V + (B + 1);
    P[0] = V[0] = S[0] = 0;
    for (uint32_t b = 0; b < B; ++b) {
        if (off[b + 1] < off[b]) { free(P); return ORC_EINVAL; }
        uint64_t k = orc_k(ratio, off[b + 1] - off[b]);
        P[b + 1] = P[b] + k;
        V[b + 1] = V[b] + val_bytes_of(k, bits);
        S[b + 1] = S[b] + ((bits == 8 || bits == 4) ? (k + chunk - 1) / chunk : 0);
    }
    int err = ORC_OK;
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
    for (int64_t b = 0; b < (int64_t)B; ++b) {
        int64_t rc = orc_compress_bucket_pruned(g + off[b], r + off[b], w + off[b], off[b + 1] - off[b],
                                                ratio, bits, chunk, idx + P[b], (uint8_t *)val + V[b],
                                                scales ? scales + S[b] : NULL);
        if (rc < 0) {
#pragma omp critical
            err = (int)rc;
        }
    }
    free(P);
    return err;
}

/* Inverse: dense[i] = +0 everywhere, dense[idx[j]] = decoded value j. */
int orc_decompress_bucket(const uint32_t *idx, const void *val, const float *scales, uint64_t k,
                          uint64_t n, int bits, uint32_t chunk, float *dense)
{
    if (n == 0) return ORC_OK;
    if (!dense || chunk == 0 || k > n) return ORC_EINVAL;
    if (bits != 4 && bits != 8 && bits != 16 && bits != 32) return ORC_EINVAL;
    for (uint64_t i = 0; i < n; ++i) dense[i] = 0.0f;
    for (uint64_t j = 0; j < k; ++j) {
        if (idx[j] >= n) return ORC_EINVAL;
        float d;
        if (bits == 32) d = ((const float *)val)[j];
        else if (bits == 16) d = f16_to_f32(((const uint16_t *)val)[j]);
        else {
            int q;
            if (bits == 8) q = ((const int8_t *)val)[j];
            else {
                uint8_t byte = ((const uint8_t *)val)[j >> 1];
                int nib = (j & 1) ? (byte >> 4) : (byte & 0xF);
                q = nib >= 8 ? nib - 16 : nib;
            }
            volatile float t = (float)q * scales[j / chunk];
            d = t;
        }
        dense[idx[j]] = d;
    }
    return ORC_OK;
}

/* ------------------------------------------------- bucketed whole gradient */

/* Buckets are independent (the hook of Sec. 5.1 is called once per bucket);
 * the only parallelism here is one bucket per thread. */
int orc_compress(const float *g, float *r, uint64_t n, const uint64_t *off, uint32_t B,
                 double ratio, int bits, uint32_t chunk, uint32_t *idx, void *val, float *scales,
                 int nthreads)
{
    if (!off || B == 0 || off[0] != 0 || off[B] != n) return ORC_EINVAL;
    uint64_t *P = (uint64_t *)malloc(3 * (size_t)(B + 1) * sizeof(uint64_t));
    if (!P) return ORC_ENOMEM;
    uint64_t *V = P + (B + 1), *S = V + (B + 1);
    P[0] = V[0] = S[0] = 0;
    for (uint32_t b = 0; b < B; ++b) {
        if (off[b + 1] < off[b]) { free(P); return ORC_EINVAL; }
        uint64_t k = orc_k(ratio, off[b + 1] - off[b]);
        P[b + 1] = P[b] + k;
        V[b + 1] = V[b] + val_bytes_of(k, bits);
        S[b + 1] = S[b] + ((bits == 8 || bits == 4) ? (k + chunk - 1) / chunk : 0);
    }
    int err = ORC_OK;
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
    for (int64_t b = 0; b < (int64_t)B; ++b) {
        int64_t rc = orc_compress_bucket(g + off[b], r + off[b], off[b + 1] - off[b], ratio, bits,
                                         chunk, idx + P[b], (uint8_t *)val + V[b],
                                         scales ? scales + S[b] : NULL);
        if (rc < 0) {
#pragma omp critical
            err = (int)rc;
        }
    }
    free(P);
    return err;
}

int orc_decompress(const uint32_t *idx, const void *val, const float *scales, uint64_t n,
                   const uint64_t *off, uint32_t B, double ratio, int bits, uint32_t chunk,
                   float *dense, int nthreads)
{
    if (!off || B == 0 || off[0] != 0 || off[B] != n) return ORC_EINVAL;
    uint64_t *P = (uint64_t *)malloc(3 * (size_t)(B + 1) * sizeof(uint64_t));
    if (!P) return ORC_ENOMEM;
    uint64_t *V = P + (B + 1), *S = V + (B + 1);
    P[0] = V[0] = S[0] = 0;
    for (uint32_t b = 0; b < B; ++b) {
        uint64_t k = orc_k(ratio, off[b + 1] - off[b]);
        P[b + 1] = P[b] + k;
        V[b + 1] = V[b] + val_bytes_of(k, bits);
        S[b + 1] = S[b] + ((bits == 8 || bits == 4) ? (k + chunk - 1) / chunk : 0);
    }
    int err = ORC_OK;
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
    for (int64_t b = 0; b < (int64_t)B; ++b) {
        int rc = orc_decompress_bucket(idx + P[b], (const uint8_t *)val + V[b],
                                       scales ? scales + S[b] : NULL, P[b + 1] - P[b],
                                       off[b + 1] - off[b], bits, chunk, dense + off[b]);
        if (rc < 0) {
#pragma omp critical
            err = rc;
        }
    }
    free(P);
    return err;
}

/* Receiver side of an all-gather of sparse payloads (Sec. 5.3 reports AllGather as the pattern
 * for TopK): dense[idx[j]] += decoded value j, one binary32 add per survivor; everything else
 * in dense is left alone. */
int orc_decompress_accumulate(const uint32_t *idx, const void *val, const float *scales, uint64_t n,
                              const uint64_t *off, uint32_t B, double ratio, int bits,
                              uint32_t chunk, float *dense)
{
    if (!off || B == 0 || off[0] != 0 || off[B] != n || !dense) return ORC_EINVAL;
    float *tmp = (float *)malloc((size_t)(n ? n : 1) * sizeof(float));
    if (!tmp) return ORC_ENOMEM;
    /* decode into a scratch dense vector with the plain decompressor, then add where a survivor sits */
    int rc = orc_decompress(idx, val, scales, n, off, B, ratio, bits, chunk, tmp, 1);
    if (rc == ORC_OK) {
        uint64_t p = 0;
        for (uint32_t b = 0; b < B; ++b) {
            uint64_t k = orc_k(ratio, off[b + 1] - off[b]);
            for (uint64_t j = 0; j < k; ++j, ++p) {
                uint64_t i = off[b] + idx[p];
                volatile float sum = dense[i] + tmp[i];
                dense[i] = sum;
            }
        }
    }
    free(tmp);
    return rc;
}

/* Algorithm 2 Step 1: calculate_L2_norm(grads), in double, in index order.  per_bucket (B
 * entries) may be NULL.  Returns the norm of the whole gradient. */
double orc_l2norm(const float *g, const uint64_t *off, uint32_t B, double *per_bucket)
{
    double total = 0.0;
    for (uint32_t b = 0; b < B; ++b) {
        double s = 0.0;
        for (uint64_t i = off[b]; i < off[b + 1]; ++i) s += (double)g[i] * (double)g[i];
        if (per_bucket) per_bucket[b] = sqrt(s);
        total += s;
    }
    return sqrt(total);
}

/* Exposed so tests can pin the conversions against numpy's binary16. */
uint16_t orc_f32_to_f16(float x) { return f32_to_f16(x); }
float orc_f16_to_f32(uint16_t h) { return f16_to_f32(h); }
