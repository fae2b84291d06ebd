/*
 * libnsml device code, part 1: constants, device-resident tables, geometry, set-up kernels, histogram helpers.
 * Included by nsml_kernels.hip (one translation unit); not a public header.
 */
#ifndef NSML_DEVICE_COMMON_HPP
#define NSML_DEVICE_COMMON_HPP

namespace {

constexpr int WG = 256;
constexpr int TILE = 4096;        /* elements per tile */
constexpr int WTILE = 1024;       /* elements one wavefront covers per iteration in ef_emit */
constexpr int NB0 = 4096, NB1 = 4096, NB2 = 128;
constexpr int SUB_DIGITS = 4, SUB_BITS = 6, NBS = SUB_DIGITS << SUB_BITS;   /* finer histogram of a few level-0 digits: 64 bins each */
constexpr int SHS = 19 - SUB_BITS;   /* key >> SHS : level-0 digit and the 6 bits below it */
constexpr int SH0 = 19;   /* key >> 19         : level-0 digit (sign-less exponent + 4 mantissa bits) */
constexpr int SH1 = 7;    /* (key >> 7) & 4095 : level-1 digit;  key & 127 : level-2 digit */
constexpr int MAX_SPAN_TILES = 16;
constexpr uint32_t NONE = 0xFFFFFFFFu;
constexpr uint32_t SAMPLE_ALL_BELOW = 262144;  /* buckets smaller than this are sampled in full */
constexpr uint32_t SAMPLE_STRIDE = 64;         /* larger ones: 32 elements out of every 2048 */
constexpr uint32_t RUNS_PER_WG = 128;          /* sample runs (32 elements each) per workgroup */

/* Diagnostic: why the plan sent a bucket to the dense passes (bits; 0 when it did not). */
enum Why : uint32_t { WHY_NO_GUESS = 1, WHY_OVERFLOW = 2, WHY_TOO_FEW = 4, WHY_NO_ROOM = 8, WHY_OUTSIDE_BAND = 16, WHY_NONZEROS = 32 };

/* How a bucket's survivors are found once the streaming pass is done. */
enum Path : uint32_t {
    PATH_DENSE = 0,   /* the staged elements cannot decide: every step over the dense accumulator */
    PATH_CAND = 1,    /* staged = everything from L up: threshold and survivors from the staged entries alone */
    PATH_BAND = 2,    /* staged = a band of keys around the threshold: threshold from the band, survivors from the dense accumulator */
    PATH_ZERO = 3     /* more survivors than non-zero elements: threshold key 0, known from the counts alone */
};

enum KernelId {
    KID_SETUP = 0, KID_SPANMAP, KID_CLEAR, KID_SAMPLE, KID_PREDICT, KID_EF_EMIT, KID_PLAN,
    KID_SELECT, KID_FINISH, KID_ENCODE, KID_HARD, KID_QUANT,
    KID_TILESTART, KID_DECOMP, KID_DECOMP_ACC,
    KID_WHIST, KID_WPLAN, KID_WMASK, KID_WHARD, KID_N
};
const char *const kKernelNames[KID_N] = {
    "setup", "spanmap", "clear", "sample", "predict", "ef_emit", "plan",
    "select_count", "select_finish", "encode", "hard", "quant",
    "tilestart", "decomp", "decomp_acc",
    "whist", "wplan", "wmask", "whard"
};
static_assert(KID_N <= NSML_MAX_KERNELS, "raise NSML_MAX_KERNELS");

/* Device-resident tables.  Layout part: fixed by the bucket offsets.  Call part: fixed by
 * (ratio, bits).  State part: rewritten by every compress call. */
struct Tables {
    const uint64_t *off;     /* B+1 bucket offsets */
    const uint32_t *tile0;   /* B+1 prefix of tile counts */
    const uint32_t *span0;   /* B+1 prefix of span counts */
    const uint32_t *samp0;   /* B+1 prefix of sample workgroups */
    const uint32_t *span_b;  /* n_spans: bucket of each span */
    uint32_t *k;             /* B   survivors per bucket */
    uint64_t *P;             /* B+1 prefix of k */
    uint64_t *V;             /* B+1 prefix of value bytes */
    uint64_t *S;             /* B+1 prefix of scale counts */
    uint64_t *C;             /* B+1 prefix of chunk counts (all widths) */
    uint32_t *T;             /* B   threshold key, refined level by level */
    uint32_t *need;          /* B   how many more to take at the current level */
    uint32_t *L;             /* B   the streaming pass stages the elements with L <= key < H (L = NONE: none) */
    uint32_t *H;             /* B   NONE: no upper bound (everything from L up is staged: "candidates");
                              *     else a band is staged and the elements with key >= H are counted per segment.
                              *     L == H == 1: nothing is staged, non-zero and zero keys are counted per segment */
    uint32_t *fast;          /* B   how the bucket is decided (PATH_*); the weight stage uses 0 / 1 only */
    uint32_t *subLo;         /* B   first of the SUB_DIGITS level-0 digits whose next 6 key bits the streaming pass
                              *     also counts (NONE: none) */
    uint32_t *sh;            /* B   T holds the key bits from this position up (19: the level-0 digit only; 13: six more) */
    uint32_t *margin;        /* B   what the bucket has learned about its sample: factor on k_predict's margin (kept across calls) */
    uint32_t *why;           /* B   diagnostic: why the plan did not take the staged elements (WHY_* bits, 0 if it did) */
    uint32_t *ovf;           /* B   a staging segment of the bucket overflowed */
    uint32_t *fspan0;        /* B+1 prefix of the spans of fallback buckets */
    uint32_t *nhard;         /* 1   buckets of this call that are not on PATH_CAND (their kernels leave at once when 0) */
    uint32_t *kw;            /* B   parameters the pruning step keeps (only with weights) */
    const uint32_t *pmask;   /* with Algorithm 2 Step 2: the pruning bitmap, 128 words per tile, bit = pruned; else NULL */
    uint32_t B;
    uint32_t n_spans;
    uint32_t spanT;          /* tiles per span */
    uint32_t segSh;          /* log2 of the staging segments per span (= wavefronts of the streaming pass) */
    uint32_t chunk;
    uint32_t chunkSh;        /* log2(chunk) when chunk is a power of two, else NONE */
    uint32_t dencSpans;      /* spans per work unit of the one-pass dense encode (2 on large gradients: fewer chunks straddle units; 1 on smaller ones: more units than workgroups) */
};

/* Candidate staging: segment ss = (span << segSh) + wavefront owns entries [ss * cap, ss * cap + cnt[ss]) */
struct Cand {
    uint32_t *idx;   /* bucket-local index */
    float *val;      /* accumulator value */
    uint32_t *cnt;   /* entries per segment */
    uint32_t *G;     /* per segment: #(key > T), later its exclusive prefix inside the bucket */
    uint32_t *E;     /* per segment: #(key == T), later its exclusive prefix */
    uint32_t cap;    /* entries per segment: a quarter of the elements it covers */
};

typedef float f4 __attribute__((ext_vector_type(4)));   /* one aligned 16-byte access */

__device__ __forceinline__ uint32_t keyof(float x) { return __float_as_uint(x) & 0x7FFFFFFFu; }

/* largest b with pre[b] <= x; pre has B+1 non-decreasing entries and pre[B] > x */
template <typename T>
__device__ __forceinline__ uint32_t find_bucket(const T *__restrict__ pre, uint32_t B, T x)
{
    uint32_t lo = 0, hi = B;
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (pre[mid] <= x) lo = mid; else hi = mid;
    }
    return lo;
}

/* The same search done by a whole workgroup of 256 threads, 256 ways at a time: one or two
 * rounds of independent probes instead of a chain of dependent ones.  Every thread must call
 * it; sh is one word of LDS; returns the same value in every thread. */
template <typename T>
__device__ __forceinline__ uint32_t find_bucket_wg(const T *__restrict__ pre, uint32_t B, T x, uint32_t *sh)
{
    uint32_t lo = 0, hi = B;                 /* pre[lo] <= x < pre[hi] */
    while (hi - lo > 1) {
        const uint32_t step = (hi - lo + 255u) / 256u;
        const uint32_t p = lo + threadIdx.x * step, q = p + step;
        /* thread t owns [p, q) clipped to hi; exactly one thread's range holds the answer */
        if (p < hi && pre[p] <= x && (q >= hi || x < pre[q])) *sh = p;
        __syncthreads();
        const uint32_t np = *sh;
        __syncthreads();
        lo = np;
        hi = np + step < hi ? np + step : hi;
    }
    return lo;
}

struct SpanGeo {
    uint32_t b;        /* bucket */
    uint32_t ntiles;   /* tiles in this span */
    uint32_t tile_g;   /* global id of the first tile */
    uint64_t lo, hi;   /* bucket range */
    uint64_t base;     /* aligned global element index where the first tile starts */
};

/* span number si of bucket b */
__device__ __forceinline__ SpanGeo span_geo_b(const Tables &t, uint32_t b, uint32_t si)
{
    SpanGeo g;
    g.b = b;
    g.lo = t.off[b];
    g.hi = t.off[b + 1];
    const uint32_t tiles_b = t.tile0[b + 1] - t.tile0[b];
    const uint32_t first = si * t.spanT;
    g.ntiles = min(t.spanT, tiles_b - first);
    g.tile_g = t.tile0[b] + first;
    g.base = (g.lo & ~3ull) + (uint64_t)first * TILE;
    return g;
}

/* global span s */
__device__ __forceinline__ SpanGeo span_geo(const Tables &t, uint32_t s)
{
    const uint32_t b = t.span_b[s];
    return span_geo_b(t, b, s - t.span0[b]);
}

/* The four pruning bits of quad `quad` (0..1023) of tile `tile_abs`. */
__device__ __forceinline__ uint32_t pruned_bits(const uint32_t *__restrict__ pm, uint32_t tile_abs, uint32_t quad)
{
    return (pm[(uint64_t)tile_abs * (TILE / 32) + (quad >> 3)] >> ((quad & 7u) * 4u)) & 0xFu;
}

/* Load the quad at aligned element index gi, masking what lies outside [lo, hi).
 * Returns the 4-bit validity mask. */
__device__ __forceinline__ uint32_t load_quad(const float *__restrict__ p, uint64_t gi,
                                              uint64_t lo, uint64_t hi, float (&x)[4])
{
    if (gi >= lo && gi + 4 <= hi) {
        const f4 v = *reinterpret_cast<const f4 *>(p + gi);
        x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
        return 0xFu;
    }
    uint32_t m = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        x[j] = 0.0f;
        if (gi + j >= lo && gi + j < hi) { x[j] = p[gi + j]; m |= 1u << j; }
    }
    return m;
}

/* ------------------------------------------------------------------ setup / clear */

__device__ __forceinline__ uint64_t survivors_dev(double ratio, uint64_t nb)
{
    if (nb == 0) return 0;
    const double want = ceil(ratio * (double)nb);   /* one IEEE double product, then ceil */
    if (want < 1.0) return 1;
    if (want >= (double)nb) return nb;
    return (uint64_t)want;
}

/* One workgroup: k_b and the four prefix tables for (ratio, bits, chunk). */
__global__ __launch_bounds__(WG) void k_setup(Tables t, double ratio, int bits)
{
    __shared__ uint64_t part[4][WG];
    const uint32_t tid = threadIdx.x;
    const uint32_t per = (t.B + WG - 1) / WG;
    const uint32_t b0 = min(t.B, tid * per), b1 = min(t.B, b0 + per);
    uint64_t sk = 0, sv = 0, ss = 0, sc = 0;
    for (uint32_t b = b0; b < b1; ++b) {
        const uint64_t k = survivors_dev(ratio, t.off[b + 1] - t.off[b]);
        const uint64_t ch = (k + t.chunk - 1) / t.chunk;
        sk += k;
        sv += bits == 32 ? 4 * k : bits == 16 ? 2 * k : bits == 8 ? k : (k + 1) / 2;
        ss += bits <= 8 ? ch : 0;
        sc += ch;
    }
    part[0][tid] = sk; part[1][tid] = sv; part[2][tid] = ss; part[3][tid] = sc;
    __syncthreads();
    if (tid < 4) {
        uint64_t run = 0;
        for (int i = 0; i < WG; ++i) { const uint64_t x = part[tid][i]; part[tid][i] = run; run += x; }
    }
    __syncthreads();
    uint64_t pk = part[0][tid], pv = part[1][tid], ps = part[2][tid], pc = part[3][tid];
    for (uint32_t b = b0; b < b1; ++b) {
        const uint64_t k = survivors_dev(ratio, t.off[b + 1] - t.off[b]);
        const uint64_t ch = (k + t.chunk - 1) / t.chunk;
        t.k[b] = (uint32_t)k;
        {   /* Algorithm 2 Step 2: floor(0.5 * (1 - ratio) * n_b) parameters are pruned */
            const uint64_t nb = t.off[b + 1] - t.off[b];
            const double np = floor(0.5 * (1.0 - ratio) * (double)nb);
            t.kw[b] = (uint32_t)(nb - (uint64_t)(np < 0.0 ? 0.0 : np));
        }
        t.P[b] = pk; t.V[b] = pv; t.S[b] = ps; t.C[b] = pc;
        pk += k;
        pv += bits == 32 ? 4 * k : bits == 16 ? 2 * k : bits == 8 ? k : (k + 1) / 2;
        ps += bits <= 8 ? ch : 0;
        pc += ch;
        if (b == t.B - 1) { t.P[t.B] = pk; t.V[t.B] = pv; t.S[t.B] = ps; t.C[t.B] = pc; }
    }
}

/* span -> bucket map, once per bucket layout */
__global__ __launch_bounds__(WG) void k_spanmap(const uint32_t *__restrict__ span0, uint32_t B,
                                                uint32_t n_spans, uint32_t *__restrict__ span_b)
{
    const uint32_t s = blockIdx.x * WG + threadIdx.x;
    if (s < n_spans) span_b[s] = find_bucket<uint32_t>(span0, B, s);
}

__global__ __launch_bounds__(WG) void k_clear(uint32_t *__restrict__ p, uint64_t n)
{
    const uint64_t stride = (uint64_t)gridDim.x * WG;
    for (uint64_t i = (uint64_t)blockIdx.x * WG + threadIdx.x; i < n; i += stride) p[i] = 0u;
}

/* Plain 16-byte copy, the yardstick for the profiler's HBM byte counters. */
__global__ __launch_bounds__(WG) void k_calib_copy(const f4 *__restrict__ src, f4 *__restrict__ dst, uint64_t n16)
{
    const uint64_t stride = (uint64_t)gridDim.x * WG;
    for (uint64_t i = (uint64_t)blockIdx.x * WG + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

/* Streaming yardsticks in the shape of the library's own passes: 1024 threads, every wavefront
 * on its own contiguous 16 KiB (16 rows of 64 lanes x 16 bytes), one such block per workgroup. */
template <bool NT>
__device__ __forceinline__ f4 calib_ld(const f4 *p) { return NT ? __builtin_nontemporal_load(p) : *p; }
template <bool NT>
__device__ __forceinline__ void calib_st(f4 *p, f4 v) { if (NT) __builtin_nontemporal_store(v, p); else *p = v; }
__device__ __forceinline__ uint64_t calib_base()
{
    return ((uint64_t)blockIdx.x * 16u + (threadIdx.x >> 6)) * 1024u + (threadIdx.x & 63u);   /* in 16-byte units */
}
template <bool NT>
__global__ __launch_bounds__(1024) void k_calib_read(const f4 *__restrict__ a, f4 *__restrict__ out)
{
    const uint64_t base = calib_base();
    f4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < 16; ++u) { const f4 v = calib_ld<NT>(a + base + u * 64); acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w; }
    /* keep the loads alive: one store per workgroup at most (never taken for ordinary data) */
    if (acc.x + acc.y + acc.z + acc.w == 12345.678f && threadIdx.x == 0) out[blockIdx.x] = acc;
}
template <bool NT>
__global__ __launch_bounds__(1024) void k_calib_fill(f4 *__restrict__ b)
{
    const uint64_t base = calib_base();
    const f4 z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < 16; ++u) calib_st<NT>(b + base + u * 64, z);
}
template <bool NT>
__global__ __launch_bounds__(1024) void k_calib_add(const f4 *__restrict__ a, f4 *__restrict__ b)
{
    const uint64_t base = calib_base();
#pragma unroll
    for (int h = 0; h < 4; ++h) {
        f4 x[4], y[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) { x[u] = calib_ld<NT>(a + base + (h * 4 + u) * 64); y[u] = calib_ld<NT>(b + base + (h * 4 + u) * 64); }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            f4 r; r.x = x[u].x + y[u].x; r.y = x[u].y + y[u].y; r.z = x[u].z + y[u].z; r.w = x[u].w + y[u].w;
            calib_st<NT>(b + base + (h * 4 + u) * 64, r);
        }
    }
}
template <bool NT>
__global__ __launch_bounds__(1024) void k_calib_copy2(const f4 *__restrict__ a, f4 *__restrict__ b)
{
    const uint64_t base = calib_base();
#pragma unroll
    for (int h = 0; h < 4; ++h) {
        f4 x[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) x[u] = calib_ld<NT>(a + base + (h * 4 + u) * 64);
#pragma unroll
        for (int u = 0; u < 4; ++u) calib_st<NT>(b + base + (h * 4 + u) * 64, x[u]);
    }
}

/* ------------------------------------------------------------------ histograms */

/* Add the four level digits of a quad to an LDS histogram.  When every lane of the wavefront
 * carries the same digit in all four slots (runs of zeros, saturated buckets) one lane adds
 * the whole count: same-address LDS atomics of a wavefront serialise.  All 64 lanes must be
 * active. */
__device__ __forceinline__ void hist_quad_full(uint32_t *h, uint32_t d0, uint32_t d1,
                                               uint32_t d2, uint32_t d3)
{
    const uint32_t f = __builtin_amdgcn_readfirstlane(d0);
    const bool same = (d0 == f) & (d1 == f) & (d2 == f) & (d3 == f);
    if (__all(same)) {
        if ((threadIdx.x & 63) == 0) atomicAdd(&h[f], 256u);
    } else {
        atomicAdd(&h[d0], 1u); atomicAdd(&h[d1], 1u); atomicAdd(&h[d2], 1u); atomicAdd(&h[d3], 1u);
    }
}

__device__ __forceinline__ void hist_flush(const uint32_t *h, uint32_t *__restrict__ dst, int nb,
                                           int nthreads = WG)
{
    for (int i = threadIdx.x; i < nb; i += nthreads) {
        const uint32_t c = h[i];
        if (c) atomicAdd(&dst[i], c);
    }
}

/* Inclusive scan over the 256 threads of a workgroup: shuffles inside each wavefront, one
 * exchange of the four wavefront totals through LDS.  tmp needs WG words; on return
 * tmp[WG - 1] holds the grand total (callers read it, then synchronise before reusing tmp). */
__device__ __forceinline__ uint32_t block_incl_scan(uint32_t x, uint32_t *tmp)
{
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t y = __shfl_up(x, d, 64);
        if (lane >= (uint32_t)d) x += y;
    }
    if (lane == 63) tmp[wave] = x;
    __syncthreads();
    uint32_t add = 0;
#pragma unroll
    for (int w = 0; w < WG / 64; ++w) add += (uint32_t)w < wave ? tmp[w] : 0u;
    const uint32_t total = tmp[0] + tmp[1] + tmp[2] + tmp[3];
    __syncthreads();
    x += add;
    if (tid == WG - 1) tmp[WG - 1] = total;
    __syncthreads();
    return x;
}

/* A histogram row seen from the top digit down: thread 0 owns the highest digits. */
template <int NB>
struct DigitWalk {
    static constexpr int PER = NB >= WG ? NB / WG : 1;
    uint32_t c[PER];
    uint32_t sum, incl, total;
    int top;

    /* every thread of the workgroup must call this (it synchronises) */
    __device__ __forceinline__ void load(const uint32_t *__restrict__ hb, uint32_t *tmp)
    {
        top = NB - 1 - (int)threadIdx.x * PER;
        sum = 0;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int d = top - i;
            c[i] = d >= 0 ? hb[d] : 0u;
            sum += c[i];
        }
        incl = block_incl_scan(sum, tmp);
        total = tmp[WG - 1];
        __syncthreads();
    }
    /* Zero the row again once it has been read (every thread its own digits): the histograms
     * of a call are left clean for the next one, which saves a fill kernel per call. */
    __device__ __forceinline__ void clear(uint32_t *__restrict__ hb) const
    {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int d = top - i;
            if (d >= 0) hb[d] = 0u;
        }
    }
    /* The digit holding the want-th largest entry (1 <= want <= total): exactly one thread
     * returns true, with the digit, the number of entries in higher digits, and the number
     * in the digit itself. */
    __device__ __forceinline__ bool find(uint32_t want, uint32_t &digit, uint32_t &above,
                                         uint32_t &at) const
    {
        const uint32_t before = incl - sum;
        if (!(before < want && want <= incl)) return false;
        uint32_t acc = before;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            if (acc + c[i] >= want) { digit = (uint32_t)(top - i); above = acc; at = c[i]; return true; }
            acc += c[i];
        }
        return false;
    }
};

}  // namespace

#endif
