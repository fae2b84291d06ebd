/*
 * libnsml GPU path for gfx950 (MI355X): hand-written HIP kernels and their C-ABI entry points.
 *
 * One compress call = error-feedback accumulation, exact top-k by magnitude per bucket
 * (Sec. 4.2 Step 3 / Algorithm 2 Step 3), value coding and payload packing; one decompress
 * call = payload -> dense gradient.  Nothing here is a dense contraction: every kernel is a
 * streaming pass bound by HBM bandwidth, so the work is organised around coalesced 16-byte
 * accesses, LDS histograms and 64-lane ballots, not MFMA.
 *
 * Selection is an exact radix select on the 31-bit magnitude key (binary32 pattern with the
 * sign cleared), digits of 12 + 12 + 7 bits, arranged so that the gradient is read ONCE:
 *
 *   sample    level-0 histogram of a 1/64 sample of grad + residual (small buckets: all of it)
 *   predict   per bucket: a level-0 digit whose lower edge L_b is, with a wide margin, below
 *             the k-th largest key
 *   ef_emit   acc = grad + residual (written over residual), exact level-0 histogram, and
 *             every element with key >= L_b appended, in index order, to a per-wavefront
 *             staging segment ("candidates")                                  12 B/element
 *   plan      per bucket: exact level-0 digit b0 of the k-th key; the candidates (exactly
 *             the elements with key >= L_b) decide the bucket iff there are at least k of
 *             them and no staging segment overflowed
 *   refine1/2, pick1/2   remaining digits from the candidates only -> threshold key T_b and
 *             e_b = how many elements equal to T_b are admitted (lowest indices first)
 *   count, scan, write   survivors to their final, index-ordered slots
 *   fallback  buckets whose candidates cannot decide (huge groups of equal keys, ratio near
 *             1, an unlucky sample) take the same steps over the dense accumulator instead,
 *             in the last workgroups of the same launches: four more reads of that bucket
 *             only.  Results are identical.
 *   quant     per chunk of survivors: absmax scale, codes, packing, residual update
 *   tilestart, decomp    payload -> dense, each output line written once, tile staged in LDS
 *
 * Geometry: a bucket [lo, hi) is cut into tiles of 4096 elements starting at lo rounded down
 * to a multiple of 4, so every 16-byte access is aligned; elements of an edge tile outside
 * [lo, hi) are masked.  A workgroup owns a span of up to 16 consecutive tiles of one bucket.
 * Workgroups have 256 threads, except in the streaming pass, which runs one wavefront per
 * tile (512 or 1024 threads) on spans of 8 and 16 tiles.
 */
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#include <new>
#include <vector>

#include "nsml.h"

namespace {

constexpr int WG = 256;
constexpr int TILE = 4096;        /* elements per tile */
constexpr int WTILE = 1024;       /* elements one wavefront covers per iteration in ef_emit */
constexpr int NB0 = 4096, NB1 = 4096, NB2 = 128;
constexpr int SH0 = 19;   /* key >> 19         : level-0 digit (sign-less exponent + 4 mantissa bits) */
constexpr int SH1 = 7;    /* (key >> 7) & 4095 : level-1 digit;  key & 127 : level-2 digit */
constexpr int MAX_SPAN_TILES = 16;
constexpr uint32_t NONE = 0xFFFFFFFFu;
constexpr uint32_t SAMPLE_ALL_BELOW = 262144;  /* buckets smaller than this are sampled in full */
constexpr uint32_t SAMPLE_STRIDE = 64;         /* larger ones: 32 elements out of every 2048 */
constexpr uint32_t RUNS_PER_WG = 128;          /* sample runs (32 elements each) per workgroup */
constexpr uint32_t SIDE_GRID = 2048;           /* workgroups of the kernels that walk work lists */
constexpr uint32_t AGG_GRID = 1024;            /* workgroups of the candidate refine that aggregates in LDS */

enum KernelId {
    KID_SETUP = 0, KID_SPANMAP, KID_CLEAR, KID_SAMPLE, KID_PREDICT, KID_EF_EMIT, KID_PLAN, KID_FB_PLAN,
    KID_REFINE1, KID_PICK1, KID_REFINE2, KID_PICK2, KID_COUNT, KID_SCAN, KID_WRITE,
    KID_QUANT, KID_TILESTART, KID_DECOMP, KID_DECOMP_ACC, KID_WHIST, KID_WPLAN, KID_WMASK, KID_N
};
const char *const kKernelNames[KID_N] = {
    "setup", "spanmap", "clear", "sample", "predict", "ef_emit", "plan", "fb_plan",
    "refine1", "pick1", "refine2", "pick2", "count", "scan", "write",
    "quant", "tilestart", "decomp", "decomp_acc", "whist", "wplan", "wmask"
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
    uint32_t *L;             /* B   candidates are the elements with key >= L (NONE: no candidates) */
    uint32_t *fast;          /* B   1: the candidates decide the bucket, 0: the dense fallback does */
    uint32_t *ovf;           /* B   a staging segment of the bucket overflowed */
    uint32_t *fspan0;        /* B+1 prefix of the spans of fallback buckets */
    uint32_t *margin;        /* B   history mode: how far below the last threshold key L is placed */
    uint32_t *kw;            /* B   parameters the pruning step keeps (only with weights) */
    const float *w;          /* weights when Algorithm 2 Step 2 is on, else NULL */
    const uint32_t *wT;      /* B   with weights: threshold key of |w|; NONE: the bucket's mask is in the bitmap */
    const uint32_t *wcut;    /* B   with weights: among parameters with key(w) == wT, those up to this
                              *     bucket-local index are kept (kept: key > wT, or key == wT and index <= wcut) */
    const uint32_t *pmask;   /* pruning bitmap, 128 words per tile, bit = pruned (buckets with wT = NONE) */
    uint32_t B;
    uint32_t n_spans;
    uint32_t spanT;          /* tiles per span */
    uint32_t segSh;          /* log2 of the staging segments per span (= wavefronts of the streaming pass) */
    uint32_t chunk;
};

/* Candidate staging: segment ss = (span << segSh) + wavefront owns entries [ss * cap, ss * cap + cnt[ss]) */
struct Cand {
    uint32_t *idx;   /* bucket-local index */
    float *val;      /* accumulator value */
    uint32_t *cnt;   /* entries per segment */
    uint32_t *G;     /* per segment: #(key > T), later its exclusive prefix inside the bucket */
    uint32_t *E;     /* per segment: #(key == T), later its exclusive prefix */
    uint32_t cap;    /* entries per segment: a quarter of the elements it covers */
    uint32_t splitSh; /* log2 of the wavefronts that share a chunk of 64 segments in the candidate kernels */
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

/* The four pruning bits (1 = pruned) of the quad at aligned element index gi, which is quad
 * `quad` of tile `tile_abs`, in a bucket [lo, hi) whose weight threshold is wT and whose last
 * kept index among the weights equal to the threshold is cut. */
__device__ __forceinline__ uint32_t pruned_quad(const Tables &t, uint32_t wT, uint32_t cut, uint32_t tile_abs,
                                                uint32_t quad, uint64_t gi, uint64_t lo, uint64_t hi)
{
    if (wT == 0xFFFFFFFFu) return pruned_bits(t.pmask, tile_abs, quad);
    float x[4];
    load_quad(t.w, gi, lo, hi, x);
    const uint32_t li = (uint32_t)(gi - lo);        /* meaningless below lo: those lanes are masked anyway */
    uint32_t bits = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t key = __float_as_uint(x[j]) & 0x7FFFFFFFu;
        bits |= ((key < wT || (key == wT && li + j > cut)) ? 1u : 0u) << j;
    }
    return bits;
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

__global__ __launch_bounds__(WG) void k_fill_u32(uint32_t *__restrict__ p, uint32_t n, uint32_t v)
{
    const uint32_t i = blockIdx.x * WG + threadIdx.x;
    if (i < n) p[i] = v;
}

/* Plain 16-byte copy, the yardstick for the profiler's HBM byte counters. */
__global__ __launch_bounds__(WG) void k_calib_copy(const f4 *__restrict__ src, f4 *__restrict__ dst, uint64_t n16)
{
    const uint64_t stride = (uint64_t)gridDim.x * WG;
    for (uint64_t i = (uint64_t)blockIdx.x * WG + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
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

/* ------------------------------------------------------------------ sample / predict */

/* Level-0 histogram of a sample of acc = grad + residual: runs of 32 consecutive elements,
 * every run of a small bucket, one run in 64 of a large one. */
template <bool SUM>   /* SUM: keys of g + r; else keys of g alone (the weight stage) */
__global__ __launch_bounds__(WG) void k_sample(const float *__restrict__ g, const float *__restrict__ r,
                                               Tables t, uint32_t *__restrict__ hist_s)
{
    __shared__ uint32_t h[NB0];
    const uint32_t tid = threadIdx.x;
    for (int i = tid; i < NB0; i += WG) h[i] = 0;
    const uint32_t b = find_bucket<uint32_t>(t.samp0, t.B, blockIdx.x);
    const uint32_t wi = blockIdx.x - t.samp0[b];
    const uint64_t lo = t.off[b], hi = t.off[b + 1];
    const uint64_t a0 = lo & ~3ull;
    const uint64_t stride = (hi - lo) < SAMPLE_ALL_BELOW ? 1 : SAMPLE_STRIDE;
    const uint64_t run_elems = 32ull * stride;
    const uint64_t n_runs = (hi - a0 + run_elems - 1) / run_elems;
    __syncthreads();
#pragma unroll 4
    for (uint32_t i = 0; i < RUNS_PER_WG / 32; ++i) {
        const uint64_t run = (uint64_t)wi * RUNS_PER_WG + i * 32 + (tid >> 3);
        if (run < n_runs) {
            const uint64_t gi = a0 + run * run_elems + (tid & 7u) * 4;
            float x[4], y[4];
            uint32_t m = load_quad(g, gi, lo, hi, x);
            if (SUM) load_quad(r, gi, lo, hi, y);
            if (SUM && t.w) {
                const uint64_t rel = gi - a0;
                m &= ~pruned_quad(t, t.wT[b], t.wcut[b], t.tile0[b] + (uint32_t)(rel / TILE),
                                  (uint32_t)(rel % TILE) / 4, gi, lo, hi);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if ((m >> j) & 1u) atomicAdd(&h[keyof(SUM ? __fadd_rn(x[j], y[j]) : x[j]) >> SH0], 1u);
        }
    }
    __syncthreads();
    hist_flush(h, hist_s + (uint64_t)b * NB0, NB0);
}

/* Per bucket: choose the candidate bound L_b from the sample histogram.  The sample count
 * above the true k-th key is binomial with mean ks = k * m / n; asking for ks + 4 sqrt(ks) + 4
 * sampled entries above L_b leaves the candidates short of k only a few times in 1e5 buckets,
 * and then the dense fallback still gives the exact result. */
__global__ __launch_bounds__(WG) void k_predict(Tables t, const uint32_t *__restrict__ hist_s,
                                                int force_dense)
{
    __shared__ uint32_t tmp[WG];
    const uint32_t b = blockIdx.x, tid = threadIdx.x;
    const uint64_t nb = t.off[b + 1] - t.off[b];
    const uint32_t k = t.k[b];
    if (nb == 0 || force_dense) {
        if (tid == 0) t.L[b] = NONE;
        return;
    }
    DigitWalk<NB0> w;
    w.load(hist_s + (uint64_t)b * NB0, tmp);
    const uint32_t m = w.total;
    const bool exact = nb < SAMPLE_ALL_BELOW;
    /* the sample was drawn from the parameters that can be selected: all of them, or the
     * ones the pruning step kept */
    const double pop = t.w ? (double)t.kw[b] : (double)nb;
    const double ks = (double)k * (double)m / pop;
    const double want_d = exact ? (double)k : ceil(ks + 4.0 * sqrt(ks) + 4.0);
    const double cap_b = (double)(t.span0[b + 1] - t.span0[b]) * 4.0 * (double)t.spanT * 256.0;
    if (m == 0 || want_d > (double)m || (double)k > 0.5 * cap_b) {
        /* not enough sample above any bound, or k too large for the staging area */
        if (tid == 0) t.L[b] = NONE;
        return;
    }
    uint32_t digit, above, at;
    if (w.find((uint32_t)want_d, digit, above, at)) {
        const double est = (double)(above + at) * pop / (double)m;
        t.L[b] = est <= 0.8 * cap_b ? (digit << SH0) : NONE;
    }
}

/* ------------------------------------------------------------------ the streaming pass */

/* Append the flagged elements of a row (64 lanes x 4 consecutive elements) to the wavefront's
 * staging segment, in index order: ranks come from ballots, nothing crosses wavefronts.  Every
 * lane of the wavefront must call this. */
__device__ __forceinline__ void emit_quad(const bool (&f)[4], const float (&a)[4], uint32_t li, const Cand &c,
                                          uint64_t cbase, uint32_t &wcount)
{
    if (__ballot(f[0] | f[1] | f[2] | f[3]) == 0ull) return;
    uint64_t bal[4];
    uint32_t pos = wcount;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        bal[j] = __ballot(f[j]);
        /* flagged entries in lower lanes */
        pos = __builtin_amdgcn_mbcnt_hi((uint32_t)(bal[j] >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal[j], pos));
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if (f[j]) {
            if (pos < c.cap) { c.idx[cbase + pos] = li + j; c.val[cbase + pos] = a[j]; }
            ++pos;
        }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) wcount += __popcll(bal[j]);
}

/* One row of the streaming pass: 64 lanes x 4 consecutive elements (one contiguous 1 KiB).
 * a[] is the accumulator quad of this lane, m its validity mask, li the bucket-local index
 * of a[0].  Stores the accumulator, counts its level-0 digits and appends candidates. */
template <bool INTERIOR, bool EMIT, int NT, bool PRUNE>
__device__ __forceinline__ void ef_row(float *__restrict__ r, uint64_t gi, const float (&a)[4],
                                       uint32_t m, uint32_t cm, uint32_t li, uint32_t *h, uint32_t L,
                                       const Cand &c, uint64_t cbase, uint32_t &wcount)
{
    uint32_t key[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) key[j] = keyof(a[j]);
    if (INTERIOR) {
        f4 v; v.x = a[0]; v.y = a[1]; v.z = a[2]; v.w = a[3];
        if (NT & 4) __builtin_nontemporal_store(v, reinterpret_cast<f4 *>(r + gi));
        else *reinterpret_cast<f4 *>(r + gi) = v;
        if (!PRUNE || __all(cm == 0xFu)) {
            hist_quad_full(h, key[0] >> SH0, key[1] >> SH0, key[2] >> SH0, key[3] >> SH0);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if ((cm >> j) & 1u) atomicAdd(&h[key[j] >> SH0], 1u);
        }
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if ((m >> j) & 1u) r[gi + j] = a[j];               /* the accumulator is always stored */
            if ((cm >> j) & 1u) atomicAdd(&h[key[j] >> SH0], 1u);
        }
    }
    if (EMIT) {
        bool f[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) f[j] = ((cm >> j) & 1u) && key[j] >= L;
        emit_quad(f, a, li, c, cbase, wcount);
    }
}

/* acc = grad + residual over a span, written over residual (Sec. 4.2 Step 3: what top-k
 * filters out is accumulated locally; the add is that), the exact level-0 histogram, and the
 * candidates.  Each wavefront owns a contiguous share of the span and its own staging
 * segment, so candidates come out in index order without any cross-wavefront exchange.
 * Launched with 64 << segSh threads: large spans run 8 or 16 wavefronts per workgroup (one
 * or two tiles each), which keeps more loads in flight per compute unit than four do. */
constexpr uint32_t MAX_SEG_WAVES = 16;
template <bool EMIT, int NT, bool PRUNE>
__global__ __launch_bounds__(64 * MAX_SEG_WAVES) void k_ef_emit(const float *__restrict__ g, float *__restrict__ r,
                                                Tables t, uint32_t *__restrict__ hist0, Cand c,
                                                double *__restrict__ span_sq)
{
    __shared__ uint32_t h[NB0];
    __shared__ double sq_w[MAX_SEG_WAVES];
    double sq = 0.0;                     /* sum of grad^2 over this thread's elements */
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t nthreads = 64u << t.segSh;
    for (uint32_t i = tid; i < NB0; i += nthreads) h[i] = 0;
    const SpanGeo s = span_geo(t, blockIdx.x);
    const uint32_t L = EMIT ? t.L[s.b] : NONE;
    const uint32_t wT = PRUNE ? t.wT[s.b] : 0u;          /* NONE: this bucket's mask is in the bitmap */
    const uint32_t wcut = PRUNE ? t.wcut[s.b] : 0u;
    const uint32_t ss = (blockIdx.x << t.segSh) + wave;
    const uint64_t cbase = (uint64_t)ss * c.cap;
    uint32_t wcount = 0;
    __syncthreads();
    /* this wavefront's wave-tiles: [wave * per, (wave + 1) * per) of the span's 4 * ntiles */
    const uint32_t per = (t.spanT * 4u) >> t.segSh;
    const uint32_t wt0 = wave * per;
    const uint32_t wt1 = min(s.ntiles * 4u, wt0 + per);
    for (uint32_t wt = wt0; wt < wt1; ++wt) {
        const uint64_t wb = s.base + (uint64_t)wt * WTILE;
        if (wb >= s.lo && wb + WTILE <= s.hi) {
            f4 gv[4], rv[4], wv[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint64_t gi = wb + (uint64_t)(u * 64 + lane) * 4;
                gv[u] = (NT & 1) ? __builtin_nontemporal_load(reinterpret_cast<const f4 *>(g + gi))
                                 : *reinterpret_cast<const f4 *>(g + gi);
                rv[u] = (NT & 2) ? __builtin_nontemporal_load(reinterpret_cast<const f4 *>(r + gi))
                                 : *reinterpret_cast<const f4 *>(r + gi);
                if (PRUNE && wT != NONE) wv[u] = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(t.w + gi));
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint64_t gi = wb + (uint64_t)(u * 64 + lane) * 4;
                float a[4];
                a[0] = __fadd_rn(gv[u].x, rv[u].x); a[1] = __fadd_rn(gv[u].y, rv[u].y);
                a[2] = __fadd_rn(gv[u].z, rv[u].z); a[3] = __fadd_rn(gv[u].w, rv[u].w);
                sq += (double)(__fmaf_rn(gv[u].x, gv[u].x, __fmul_rn(gv[u].y, gv[u].y)) +
                               __fmaf_rn(gv[u].z, gv[u].z, __fmul_rn(gv[u].w, gv[u].w)));
                uint32_t cm = 0xFu;
                if (PRUNE) {
                    if (wT != NONE) {
                        const uint32_t li = (uint32_t)(gi - s.lo);
                        const uint32_t kx = keyof(wv[u].x), ky = keyof(wv[u].y), kz = keyof(wv[u].z), kq = keyof(wv[u].w);
                        cm = ((kx > wT || (kx == wT && li <= wcut)) ? 1u : 0u) |
                             ((ky > wT || (ky == wT && li + 1 <= wcut)) ? 2u : 0u) |
                             ((kz > wT || (kz == wT && li + 2 <= wcut)) ? 4u : 0u) |
                             ((kq > wT || (kq == wT && li + 3 <= wcut)) ? 8u : 0u);
                    } else
                        cm &= ~pruned_bits(t.pmask, s.tile_g + (wt >> 2), (wt & 3u) * WG + u * 64 + lane);
                }
                ef_row<true, EMIT, NT, PRUNE>(r, gi, a, 0xFu, cm, (uint32_t)(gi - s.lo), h, L, c, cbase, wcount);
            }
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint64_t gi = wb + (uint64_t)(u * 64 + lane) * 4;
                float x[4], y[4], a[4];
                const uint32_t m = load_quad(g, gi, s.lo, s.hi, x);
                load_quad(r, gi, s.lo, s.hi, y);
#pragma unroll
                for (int j = 0; j < 4; ++j) { a[j] = __fadd_rn(x[j], y[j]); sq += (double)__fmul_rn(x[j], x[j]); }
                uint32_t cm = m;
                if (PRUNE) cm &= ~pruned_quad(t, wT, wcut, s.tile_g + (wt >> 2), (wt & 3u) * WG + u * 64 + lane, gi, s.lo, s.hi);
                ef_row<false, EMIT, NT, PRUNE>(r, gi, a, m, cm, (uint32_t)(gi - s.lo), h, L, c, cbase, wcount);
            }
        }
    }
    if (EMIT && lane == 0) {
        c.cnt[ss] = min(wcount, c.cap);
        if (wcount > c.cap) t.ovf[s.b] = 1u;
    }
    /* the span's share of |grad|^2 (by-product for the density test of Algorithm 2 Step 1):
     * fixed reduction tree, so the sum does not depend on scheduling */
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) sq += __shfl_xor(sq, d, 64);
    if (lane == 0) sq_w[wave] = sq;
    __syncthreads();
    if (tid == 0) {
        double tot = 0.0;
        for (uint32_t w = 0; w < (1u << t.segSh); w += 4) tot += (sq_w[w] + sq_w[w + 1]) + (sq_w[w + 2] + sq_w[w + 3]);
        span_sq[blockIdx.x] = tot;
    }
    hist_flush(h, hist0 + (uint64_t)s.b * NB0, NB0, (int)nthreads);
}

constexpr uint32_t MARGIN_INIT = 1u << 20;   /* 1/8 octave below the last threshold */
constexpr uint32_t MARGIN_MIN = 1u << 15, MARGIN_MAX = 1u << 22;

/* Per bucket: exact level-0 digit of the k-th largest key, and whether the candidates can
 * decide the bucket: they are exactly the elements with key >= L_b, so they contain the k
 * largest iff there are at least k of them (and no staging segment overflowed).  In history
 * mode the distance between L_b and the threshold is steered by how many candidates came. */
__global__ __launch_bounds__(WG) void k_plan(Tables t, const uint32_t *__restrict__ hist0,
                                             const uint32_t *__restrict__ cand_cnt, int have_cand,
                                             const double *__restrict__ span_sq, double *__restrict__ l2sq)
{
    __shared__ uint32_t tmp[WG];
    __shared__ double red[WG / 64];
    __shared__ uint32_t redc[WG / 64];
    const uint32_t b = blockIdx.x, tid = threadIdx.x;
    uint32_t n_cand = 0;
    {   /* |grad|^2 of the bucket: strided partial sums, then a fixed tree; candidates likewise */
        double acc = 0.0;
        for (uint32_t s = t.span0[b] + tid; s < t.span0[b + 1]; s += WG) acc += span_sq[s];
        uint32_t cc = 0;
        if (have_cand)
            for (uint32_t ss = (t.span0[b] << t.segSh) + tid; ss < (t.span0[b + 1] << t.segSh); ss += WG) cc += cand_cnt[ss];
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) { acc += __shfl_xor(acc, d, 64); cc += __shfl_xor(cc, d, 64); }
        if ((tid & 63) == 0) { red[tid >> 6] = acc; redc[tid >> 6] = cc; }
        __syncthreads();
        if (tid == 0) l2sq[b] = (red[0] + red[1]) + (red[2] + red[3]);
        n_cand = redc[0] + redc[1] + redc[2] + redc[3];
    }
    const uint32_t want = t.k[b];
    if (want == 0) {                       /* empty bucket: nothing can match */
        if (tid == 0) { t.T[b] = NONE; t.need[b] = 0; t.fast[b] = 1u; }
        return;
    }
    DigitWalk<NB0> w;
    w.load(hist0 + (uint64_t)b * NB0, tmp);
    uint32_t digit, above, at;
    if (w.find(want, digit, above, at)) {
        t.T[b] = digit;
        t.need[b] = want - above;
        const uint32_t L = t.L[b];
        const bool valid = have_cand && L != NONE && n_cand >= want && !t.ovf[b];
        t.fast[b] = valid ? 1u : 0u;
        /* margin control for the next call */
        uint32_t mg = t.margin[b];
        if (L != NONE) {
            if (!valid) mg = min(MARGIN_MAX, mg * 4u);
            else if ((uint64_t)n_cand * 5u > (uint64_t)want * 8u) mg = max(MARGIN_MIN, mg - mg / 4u);   /* > 1.6 k */
            else if ((uint64_t)n_cand * 20u < (uint64_t)want * 23u) mg = min(MARGIN_MAX, mg + mg / 4u); /* < 1.15 k */
        }
        t.margin[b] = mg;
    }
}

/* One workgroup: the list of spans that belong to fallback buckets.  (Kept as its own small
 * launch: doing it in the last workgroup of k_plan needs a device-scope fence in every
 * workgroup, which on this multi-die GPU writes back each L2 and costs more than a launch.) */
__global__ __launch_bounds__(WG) void k_fb_plan(Tables t)
{
    __shared__ uint32_t tmp[WG];
    const uint32_t tid = threadIdx.x;
    uint32_t carry = 0;
    for (uint32_t base = 0; base < t.B; base += WG) {
        const uint32_t bb = base + tid;
        const bool fb = bb < t.B && !t.fast[bb];
        const uint32_t x = fb ? t.span0[bb + 1] - t.span0[bb] : 0u;
        const uint32_t incl = block_incl_scan(x, tmp);
        const uint32_t tot = tmp[WG - 1];
        __syncthreads();
        if (bb < t.B) t.fspan0[bb] = carry + incl - x;
        carry += tot;
    }
    if (tid == 0) t.fspan0[t.B] = carry;
}

/* ------------------------------------------------------------------ candidate path */

/* The candidate kernels walk the staging segments, 64 consecutive ones per wavefront at a
 * time.  Lane l first fetches what describes segment 64 * chunk + l (bucket, entry count,
 * threshold): one round of look-ups for 64 segments.  Then the wavefront goes through them
 * 64 / GROUP at a time, GROUP lanes per segment, taking each description from the lane that
 * holds it.  GROUP is 4 or 16 when segments are short (low ratios), 64 otherwise.  Entries are
 * fetched four per lane before any is used, so a segment costs about one memory round trip.
 * When there are fewer chunks than wavefronts, 2^splitSh wavefronts share a chunk and take
 * every 2^splitSh-th round of it. */
struct SegMeta {
    uint32_t ss, b, cnt;
    uint32_t T;          /* the bucket's threshold key / prefix so far */
    bool in_range, active;
};

__device__ __forceinline__ SegMeta seg_meta(const Tables &t, const Cand &c, uint32_t chunk)
{
    SegMeta m;
    m.ss = chunk * 64 + (threadIdx.x & 63);
    m.in_range = m.ss < (t.n_spans << t.segSh);
    /* independent loads first (segment -> bucket, entry count), then the bucket's state */
    m.b = m.in_range ? t.span_b[m.ss >> t.segSh] : 0u;
    const uint32_t cnt = m.in_range ? c.cnt[m.ss] : 0u;
    m.T = t.T[m.b];
    m.active = m.in_range && t.fast[m.b] != 0u;
    m.cnt = m.active ? cnt : 0u;
    return m;
}

__device__ __forceinline__ uint32_t seg_chunks(const Tables &t) { return ((t.n_spans << t.segSh) + 63u) / 64u; }

constexpr uint32_t CU = 4;   /* entries a lane fetches ahead */

/* Next-digit histogram over the candidates that carry the prefix found so far (LEVEL 1:
 * 12-bit prefix, digit = key bits 18..7; LEVEL 2: 24-bit prefix, digit = bits 6..0).  The
 * matching entries are few, so they go straight to global atomics. */
template <int LEVEL, uint32_t GROUP>
__device__ __forceinline__ void crefine_body(const Tables &t, const Cand &c, uint32_t *__restrict__ hist,
                                             uint32_t bid, uint32_t nblk)
{
    constexpr int NB = LEVEL == 1 ? NB1 : NB2;
    constexpr int PSH = LEVEL == 1 ? SH0 : SH1;
    constexpr int DSH = LEVEL == 1 ? SH1 : 0;
    constexpr uint32_t SPR = 64 / GROUP;             /* segments per round */
    const uint32_t lane = threadIdx.x & 63, sub = lane / GROUP, gl = lane % GROUP;
    const uint32_t n_chunks = seg_chunks(t);
    const uint32_t split = 1u << c.splitSh;
    for (uint32_t v = bid * 4 + (threadIdx.x >> 6); v < (n_chunks << c.splitSh); v += nblk * 4) {
        const uint32_t chunk = v >> c.splitSh;
        const SegMeta m = seg_meta(t, c, chunk);
        if (__ballot(m.cnt != 0u) == 0ull) continue;
        for (uint32_t rd = v & (split - 1u); rd < GROUP; rd += split) {
            const uint32_t src = rd * SPR + sub;
            const uint32_t cnt = __shfl(m.cnt, src, 64);
            if (__ballot(cnt != 0u) == 0ull) continue;
            const uint32_t prefix = __shfl(m.T, src, 64), b = __shfl(m.b, src, 64);
            const uint64_t base = (uint64_t)(chunk * 64 + src) * c.cap;
            for (uint32_t i0 = gl; i0 < cnt; i0 += CU * GROUP) {
                float x[CU];
#pragma unroll
                for (uint32_t u = 0; u < CU; ++u) {
                    const uint32_t i = i0 + u * GROUP;
                    x[u] = i < cnt ? c.val[base + i] : 0.0f;
                }
#pragma unroll
                for (uint32_t u = 0; u < CU; ++u) {
                    const uint32_t key = keyof(x[u]);
                    if (i0 + u * GROUP < cnt && (key >> PSH) == prefix)
                        atomicAdd(&hist[(uint64_t)b * NB + ((key >> DSH) & (NB - 1))], 1u);
                }
            }
        }
    }
}

/* The same histogram when a large share of the staged elements carries the prefix (the weight
 * stage: a whole level-0 digit of the weights): a workgroup walks a contiguous range of
 * chunks, which almost always lies inside one bucket, counts in LDS and adds its histogram to
 * the bucket's once.  Groups of chunks that straddle two buckets count straight into global
 * memory.  h: NB words of LDS. */
template <int LEVEL, uint32_t GROUP>
__device__ __forceinline__ void crefine_agg_body(const Tables &t, const Cand &c, uint32_t *__restrict__ hist,
                                                 uint32_t *h, uint32_t bid, uint32_t nblk)
{
    constexpr int NB = LEVEL == 1 ? NB1 : NB2;
    constexpr int PSH = LEVEL == 1 ? SH0 : SH1;
    constexpr int DSH = LEVEL == 1 ? SH1 : 0;
    constexpr uint32_t SPR = 64 / GROUP;
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, sub = lane / GROUP, gl = lane % GROUP;
    const uint32_t n_segs = t.n_spans << t.segSh;
    const uint32_t n_chunks = seg_chunks(t);
    const uint32_t per = (n_chunks + nblk - 1) / nblk;
    const uint32_t start = min(n_chunks, bid * per), end = min(n_chunks, start + per);
    for (int i = tid; i < NB; i += WG) h[i] = 0;
    __syncthreads();
    uint32_t cur_b = NONE;               /* bucket whose counts sit in LDS (same in every thread) */
    for (uint32_t g0 = start; g0 < end; g0 += 4) {
        /* the segments of this group of up to four chunks: one bucket or several? */
        const uint32_t seg_a = g0 * 64, seg_z = min(n_segs, min(end, g0 + 4) * 64) - 1u;
        const uint32_t b_a = t.span_b[seg_a >> t.segSh], b_z = t.span_b[seg_z >> t.segSh];
        const bool one = b_a == b_z;
        if (one && b_a != cur_b) {
            __syncthreads();
            if (cur_b != NONE) hist_flush(h, hist + (uint64_t)cur_b * NB, NB);
            __syncthreads();
            for (int i = tid; i < NB; i += WG) h[i] = 0;
            __syncthreads();
            cur_b = b_a;
        }
        const uint32_t chunk = g0 + wave;
        if (chunk >= end) continue;
        const SegMeta m = seg_meta(t, c, chunk);
        if (__ballot(m.cnt != 0u) == 0ull) continue;
        for (uint32_t rd = 0; rd < GROUP; ++rd) {
            const uint32_t src = rd * SPR + sub;
            const uint32_t cnt = __shfl(m.cnt, src, 64);
            if (__ballot(cnt != 0u) == 0ull) continue;
            const uint32_t prefix = __shfl(m.T, src, 64), b = __shfl(m.b, src, 64);
            const uint64_t base = (uint64_t)(chunk * 64 + src) * c.cap;
            for (uint32_t i0 = gl; i0 < cnt; i0 += CU * GROUP) {
                float x[CU];
#pragma unroll
                for (uint32_t u = 0; u < CU; ++u) {
                    const uint32_t i = i0 + u * GROUP;
                    x[u] = i < cnt ? c.val[base + i] : 0.0f;
                }
#pragma unroll
                for (uint32_t u = 0; u < CU; ++u) {
                    const uint32_t key = keyof(x[u]);
                    if (i0 + u * GROUP < cnt && (key >> PSH) == prefix) {
                        const uint32_t d = (key >> DSH) & (NB - 1);
                        if (one) atomicAdd(&h[d], 1u);
                        else atomicAdd(&hist[(uint64_t)b * NB + d], 1u);
                    }
                }
            }
        }
    }
    __syncthreads();
    if (cur_b != NONE) hist_flush(h, hist + (uint64_t)cur_b * NB, NB);
}

/* Per bucket, levels 1 and 2: walk the level's histogram (the candidates' one or the dense
 * fallback's, whichever path the bucket is on) to the digit holding the need-th entry and
 * append it to the prefix. */
template <int LEVEL>
__global__ __launch_bounds__(WG) void k_pick(Tables t, const uint32_t *__restrict__ hist_c,
                                             const uint32_t *__restrict__ hist_f, uint32_t *__restrict__ err,
                                             int write_next, uint32_t *__restrict__ wT_out = nullptr)
{
    constexpr int NB = LEVEL == 2 ? NB2 : NB1;
    constexpr int BITS = LEVEL == 2 ? 7 : 12;
    __shared__ uint32_t tmp[WG];
    const uint32_t b = blockIdx.x, tid = threadIdx.x;
    const uint32_t want = t.need[b];
    if (want == 0) {
        /* empty bucket */
        if (LEVEL == 2 && wT_out && tid == 0) wT_out[b] = 0u;
        return;
    }
    const uint32_t *hist = t.fast[b] ? hist_c : hist_f;
    DigitWalk<NB> w;
    w.load(hist + (uint64_t)b * NB, tmp);
    if (w.total < want) {                  /* cannot happen: the level above counted them */
        if (tid == 0) err[0] = 1u;
        return;
    }
    uint32_t digit, above, at;
    if (w.find(want, digit, above, at)) {
        const uint32_t T = (t.T[b] << BITS) | digit;
        t.T[b] = T;
        t.need[b] = want - above;
        /* weight stage: buckets decided from the candidates hand the gradient kernels the
         * threshold itself (and, next, the last kept index among equal weights); the others a
         * bitmap */
        if (LEVEL == 2 && wT_out) wT_out[b] = t.fast[b] ? T : NONE;
        if (LEVEL == 2 && write_next) {
            /* history mode: next call's candidate bound sits a margin below this threshold */
            const double cap_b = (double)(t.span0[b + 1] - t.span0[b]) * 4.0 * (double)t.spanT * 256.0;
            const uint32_t mg = t.margin[b];
            /* elements with key >= T: the k survivors plus the equal ones left out */
            const double ge_T = (double)t.k[b] - (double)(want - above) + (double)at;
            t.L[b] = ((double)t.k[b] > 0.5 * cap_b || ge_T > 0.8 * cap_b) ? NONE : (T > mg ? T - mg : 0u);
        }
    }
}

/* Per segment: how many candidates exceed the threshold, how many equal it.  The counts of
 * a chunk's 64 segments are gathered back into the lanes that described them and stored
 * side by side. */
template <uint32_t GROUP>
__device__ __forceinline__ void ccount_body(const Tables &t, const Cand &c, uint32_t bid, uint32_t nblk)
{
    constexpr uint32_t SPR = 64 / GROUP;
    const uint32_t lane = threadIdx.x & 63, sub = lane / GROUP, gl = lane % GROUP;
    const uint32_t n_chunks = seg_chunks(t);
    const uint32_t split = 1u << c.splitSh;
    for (uint32_t v = bid * 4 + (threadIdx.x >> 6); v < (n_chunks << c.splitSh); v += nblk * 4) {
        const uint32_t chunk = v >> c.splitSh, part = v & (split - 1u);
        const SegMeta m = seg_meta(t, c, chunk);
        if (__ballot(m.active) == 0ull) continue;
        uint32_t my_g = 0, my_e = 0;             /* results for segment 64 * chunk + lane */
        for (uint32_t rd = part; rd < GROUP; rd += split) {
            const uint32_t src = rd * SPR + sub;
            const uint32_t cnt = __shfl(m.cnt, src, 64);
            if (__ballot(cnt != 0u) == 0ull) continue;
            const uint32_t T = __shfl(m.T, src, 64);
            const uint64_t base = (uint64_t)(chunk * 64 + src) * c.cap;
            uint32_t ng = 0, ne = 0;
            for (uint32_t i0 = gl; i0 < cnt; i0 += CU * GROUP) {
                float x[CU];
#pragma unroll
                for (uint32_t u = 0; u < CU; ++u) {
                    const uint32_t i = i0 + u * GROUP;
                    x[u] = i < cnt ? c.val[base + i] : 0.0f;
                }
#pragma unroll
                for (uint32_t u = 0; u < CU; ++u) {
                    const uint32_t key = keyof(x[u]);
                    const bool in = i0 + u * GROUP < cnt;
                    ng += (in && key > T) ? 1u : 0u;
                    ne += (in && key == T) ? 1u : 0u;
                }
            }
#pragma unroll
            for (int d = GROUP / 2; d >= 1; d >>= 1) { ng += __shfl_xor(ng, d, 64); ne += __shfl_xor(ne, d, 64); }
            /* segment rd * SPR + j was counted by the group of lanes starting at j * GROUP */
            const uint32_t from = (lane % SPR) * GROUP;
            const uint32_t got_g = __shfl(ng, from, 64), got_e = __shfl(ne, from, 64);
            if (lane / SPR == rd) { my_g = got_g; my_e = got_e; }
        }
        /* this wavefront took the rounds congruent to `part` */
        if (m.active && ((lane / SPR) & (split - 1u)) == part) { c.G[m.ss] = my_g; c.E[m.ss] = my_e; }
    }
}

/* Per bucket: exclusive scan, in place, of per-unit counts (units: the bucket's staging
 * segments on the candidate path, its tiles on the fallback path).  Both counts of a unit
 * travel as one 64-bit word (neither total can reach 2^32: a bucket has fewer elements), and
 * every thread takes four consecutive units, so a round covers 1024 units with one scan. */
__global__ __launch_bounds__(WG) void k_scan(Tables t, uint32_t *__restrict__ cG, uint32_t *__restrict__ cE,
                                             uint32_t *__restrict__ tG, uint32_t *__restrict__ tE)
{
    __shared__ uint64_t tmp[WG / 64];
    const uint32_t b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t mode = t.fast[b];
    uint32_t *G = mode ? cG : tG, *E = mode ? cE : tE;
    const uint32_t t0 = mode ? t.span0[b] << t.segSh : t.tile0[b];
    const uint32_t t1 = mode ? t.span0[b + 1] << t.segSh : t.tile0[b + 1];
    uint64_t carry = 0;
    for (uint32_t base = t0; base < t1; base += WG * 4) {
        const uint32_t i0 = base + tid * 4;
        uint64_t v[4], x = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            v[j] = i0 + j < t1 ? ((uint64_t)G[i0 + j] << 32) | (uint64_t)E[i0 + j] : 0ull;
            x += v[j];
        }
        const uint64_t own = x;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t hi = __shfl_up((uint32_t)(x >> 32), d, 64), lo = __shfl_up((uint32_t)x, d, 64);
            if (lane >= (uint32_t)d) x += ((uint64_t)hi << 32) | (uint64_t)lo;
        }
        if (lane == 63) tmp[wave] = x;
        __syncthreads();
        uint64_t before = carry, total = 0;
#pragma unroll
        for (uint32_t w = 0; w < WG / 64; ++w) { before += w < wave ? tmp[w] : 0ull; total += tmp[w]; }
        __syncthreads();
        uint64_t run = before + x - own;         /* exclusive prefix of this thread's first unit */
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (i0 + j < t1) { G[i0 + j] = (uint32_t)(run >> 32); E[i0 + j] = (uint32_t)run; }
            run += v[j];
        }
        carry += total;
    }
}

/* Per segment: copy the admitted candidates (key > T, or key == T and among the first e_b
 * equal ones of the bucket in index order) to their final slots. */
template <uint32_t GROUP, bool CUT = false>   /* CUT (weight stage): only record, per bucket in idx_out[b],
                                               * the index of the last admitted entry equal to the threshold */
__device__ __forceinline__ void cwrite_body(const Tables &t, const Cand &c, uint32_t *__restrict__ idx_out,
                                            float *__restrict__ v_out, uint32_t bid, uint32_t nblk)
{
    constexpr uint32_t SPR = 64 / GROUP;
    const uint32_t lane = threadIdx.x & 63, sub = lane / GROUP, gl = lane % GROUP;
    const uint32_t shift = sub * GROUP;
    const uint64_t below = (1ull << gl) - 1ull;
    const uint64_t gmask = GROUP == 64 ? ~0ull : ((1ull << (GROUP % 64)) - 1ull);
    const uint32_t n_chunks = seg_chunks(t);
    const uint32_t split = 1u << c.splitSh;
    for (uint32_t v = bid * 4 + (threadIdx.x >> 6); v < (n_chunks << c.splitSh); v += nblk * 4) {
        const uint32_t chunk = v >> c.splitSh;
        const SegMeta m = seg_meta(t, c, chunk);
        if (__ballot(m.cnt != 0u) == 0ull) continue;
        const uint32_t m_g = m.in_range ? c.G[m.ss] : 0u, m_e = m.in_range ? c.E[m.ss] : 0u;
        const uint32_t m_need = t.need[m.b];
        const uint64_t m_P = t.P[m.b];
        for (uint32_t rd = v & (split - 1u); rd < GROUP; rd += split) {
            const uint32_t src = rd * SPR + sub;
            const uint32_t cnt = __shfl(m.cnt, src, 64);
            /* the groups of the wavefront advance together: ballots need every lane */
            uint32_t maxcnt = cnt;
#pragma unroll
            for (int d = 32; d >= (int)GROUP; d >>= 1) maxcnt = max(maxcnt, (uint32_t)__shfl_xor(maxcnt, d, 64));
            if (maxcnt == 0u) continue;
            const uint32_t T = __shfl(m.T, src, 64), e_b = __shfl(m_need, src, 64);
            uint32_t run_g = __shfl(m_g, src, 64), run_e = __shfl(m_e, src, 64);
            const uint64_t Pb = ((uint64_t)__shfl((uint32_t)(m_P >> 32), src, 64) << 32) |
                                (uint64_t)__shfl((uint32_t)m_P, src, 64);
            const uint32_t bkt = __shfl(m.b, src, 64);
            const uint64_t base = (uint64_t)(chunk * 64 + src) * c.cap;
            for (uint32_t i0 = 0; i0 < maxcnt; i0 += CU * GROUP) {
                float x[CU];
                uint32_t li[CU];
#pragma unroll
                for (uint32_t u = 0; u < CU; ++u) {
                    const uint32_t i = i0 + u * GROUP + gl;
                    x[u] = i < cnt ? c.val[base + i] : 0.0f;
                    li[u] = i < cnt ? c.idx[base + i] : 0u;
                }
#pragma unroll
                for (uint32_t u = 0; u < CU; ++u) {
                    const uint32_t key = keyof(x[u]);
                    const bool in = i0 + u * GROUP + gl < cnt;
                    const bool isg = in && key > T, ise = in && key == T;
                    const uint64_t bg = (__ballot(isg) >> shift) & gmask;
                    const uint64_t be = (__ballot(ise) >> shift) & gmask;
                    const uint32_t pg = run_g + __popcll(bg & below), pe = run_e + __popcll(be & below);
                    if (CUT) {
                        if (ise && pe + 1u == e_b) idx_out[bkt] = li[u];
                    } else if (isg || (ise && pe < e_b)) {
                        const uint64_t pos = Pb + pg + min(e_b, pe);
                        idx_out[pos] = li[u];
                        v_out[pos] = x[u];
                    }
                    run_g += __popcll(bg);
                    run_e += __popcll(be);
                }
            }
        }
    }
}

/* ------------------------------------------------------------------ dense fallback path */

/* Histogram of the next digit over the dense accumulator of the fallback buckets. */
template <int LEVEL>
__device__ __forceinline__ void fb_refine_body(const float *__restrict__ r, const Tables &t,
                                               uint32_t *__restrict__ hist, uint32_t *h,
                                               uint32_t bid, uint32_t nblk)
{
    constexpr int NB = LEVEL == 1 ? NB1 : NB2;
    constexpr int PSH = LEVEL == 1 ? SH0 : SH1;          /* key >> PSH is the prefix */
    constexpr int DSH = LEVEL == 1 ? SH1 : 0;
    constexpr uint32_t DMASK = NB - 1;
    const uint32_t tid = threadIdx.x;
    const uint32_t total = t.fspan0[t.B];
    for (uint32_t fs = bid; fs < total; fs += nblk) {
        const uint32_t b = find_bucket<uint32_t>(t.fspan0, t.B, fs);
        const SpanGeo s = span_geo_b(t, b, fs - t.fspan0[b]);
        const uint32_t prefix = t.T[b];
        for (int i = tid; i < NB; i += WG) h[i] = 0;
        __syncthreads();
        for (uint32_t ti = 0; ti < s.ntiles; ++ti) {
            const uint64_t tb = s.base + (uint64_t)ti * TILE;
            const bool interior = tb >= s.lo && tb + TILE <= s.hi;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint64_t gi = tb + (uint64_t)(u * WG + tid) * 4;
                float x[4];
                uint32_t m = load_quad(r, gi, s.lo, s.hi, x);
                if (t.w) m &= ~pruned_quad(t, t.wT[b], t.wcut[b], s.tile_g + ti, u * WG + tid, gi, s.lo, s.hi);
                uint32_t d[4];
                uint32_t hit = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t key = keyof(x[j]);
                    d[j] = (key >> DSH) & DMASK;
                    if (((m >> j) & 1u) && (key >> PSH) == prefix) hit |= 1u << j;
                }
                if (interior) {
                    /* all lanes active here: whole-wavefront shortcut for runs of equal keys */
                    const uint32_t f = __builtin_amdgcn_readfirstlane(d[0]);
                    const bool same = hit == 0xFu && d[0] == f && d[1] == f && d[2] == f && d[3] == f;
                    if (__all(same)) {
                        if ((tid & 63) == 0) atomicAdd(&h[f], 256u);
                        continue;
                    }
                }
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if ((hit >> j) & 1u) atomicAdd(&h[d[j]], 1u);
            }
        }
        __syncthreads();
        hist_flush(h, hist + (uint64_t)b * NB, NB);
        __syncthreads();
    }
}

/* Per tile of a fallback bucket: how many keys exceed the threshold, how many equal it. */
__device__ __forceinline__ void fb_count_body(const float *__restrict__ r, const Tables &t,
                                              uint32_t *__restrict__ tG, uint32_t *__restrict__ tE,
                                              uint32_t (*cnt)[2], uint32_t bid, uint32_t nblk)
{
    const uint32_t tid = threadIdx.x;
    const uint32_t total = t.fspan0[t.B];
    for (uint32_t fs = bid; fs < total; fs += nblk) {
        const uint32_t b = find_bucket<uint32_t>(t.fspan0, t.B, fs);
        const SpanGeo s = span_geo_b(t, b, fs - t.fspan0[b]);
        const uint32_t T = t.T[b];
        if (tid < MAX_SPAN_TILES * 2) (&cnt[0][0])[tid] = 0;
        __syncthreads();
        for (uint32_t ti = 0; ti < s.ntiles; ++ti) {
            const uint64_t tb = s.base + (uint64_t)ti * TILE;
            uint32_t ng = 0, ne = 0;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint64_t gi = tb + (uint64_t)(u * WG + tid) * 4;
                float x[4];
                uint32_t m = load_quad(r, gi, s.lo, s.hi, x);
                if (t.w) m &= ~pruned_quad(t, t.wT[b], t.wcut[b], s.tile_g + ti, u * WG + tid, gi, s.lo, s.hi);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t key = keyof(x[j]);
                    const bool ok = (m >> j) & 1u;
                    ng += (ok && key > T) ? 1u : 0u;
                    ne += (ok && key == T) ? 1u : 0u;
                }
            }
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) {
                ng += __shfl_xor(ng, d, 64);
                ne += __shfl_xor(ne, d, 64);
            }
            if ((tid & 63) == 0) { atomicAdd(&cnt[ti][0], ng); atomicAdd(&cnt[ti][1], ne); }
        }
        __syncthreads();
        if (tid < s.ntiles) { tG[s.tile_g + tid] = cnt[tid][0]; tE[s.tile_g + tid] = cnt[tid][1]; }
        __syncthreads();
    }
}

/* Per tile of a fallback bucket: write the survivors to their final slots, in ascending
 * index order.  Inside a tile, thread t owns the quads (u*256 + t)*4, u = 0..3. */
template <bool MASKOUT>
__device__ __forceinline__ void fb_write_body(const float *__restrict__ r, const Tables &t,
                                              const uint32_t *__restrict__ tG,
                                              const uint32_t *__restrict__ tE,
                                              uint32_t *__restrict__ idx_out,
                                              float *__restrict__ v_out, uint32_t (*tot)[2],
                                              uint32_t *bitmap, uint32_t *__restrict__ mask_out,
                                              uint32_t bid, uint32_t nblk)
{
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint64_t lt = (1ull << lane) - 1ull;
    const uint32_t total = t.fspan0[t.B];
    for (uint32_t fs = bid; fs < total; fs += nblk) {
        const uint32_t b = find_bucket<uint32_t>(t.fspan0, t.B, fs);
        const SpanGeo s = span_geo_b(t, b, fs - t.fspan0[b]);
        const uint32_t T = t.T[b], e_b = t.need[b];
        const uint64_t Pb = t.P[b];
        for (uint32_t ti = 0; ti < s.ntiles; ++ti) {
            const uint64_t tb = s.base + (uint64_t)ti * TILE;
            const uint32_t gpre = tG[s.tile_g + ti], epre = tE[s.tile_g + ti];
            float x[4][4];
            uint32_t fg[4], fe[4], gb[4], eb[4], vm[4] = {0, 0, 0, 0};
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint64_t gi = tb + (uint64_t)(u * WG + tid) * 4;
                uint32_t m = load_quad(r, gi, s.lo, s.hi, x[u]);
                if (!MASKOUT && t.w) m &= ~pruned_quad(t, t.wT[b], t.wcut[b], s.tile_g + ti, u * WG + tid, gi, s.lo, s.hi);
                fg[u] = fe[u] = 0;
                if (MASKOUT) {
                    vm[u] = m;
                    if (u == 0 && tid < TILE / 32) bitmap[tid] = 0u;
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t key = keyof(x[u][j]);
                    if (((m >> j) & 1u) && key > T) fg[u] |= 1u << j;
                    if (((m >> j) & 1u) && key == T) fe[u] |= 1u << j;
                }
                uint32_t cg = 0, ce = 0, wg = 0, we = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint64_t bg = __ballot((fg[u] >> j) & 1u);
                    const uint64_t be = __ballot((fe[u] >> j) & 1u);
                    cg += __popcll(bg & lt); wg += __popcll(bg);
                    ce += __popcll(be & lt); we += __popcll(be);
                }
                gb[u] = cg; eb[u] = ce;
                if (lane == 0) { tot[u * 4 + wave][0] = wg; tot[u * 4 + wave][1] = we; }
            }
            __syncthreads();
            uint32_t run_g = 0, run_e = 0;
            int sl = 0;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int mine = u * 4 + (int)wave;
                for (; sl < mine; ++sl) { run_g += tot[sl][0]; run_e += tot[sl][1]; }
                uint32_t pg = gpre + run_g + gb[u];
                uint32_t pe = epre + run_e + eb[u];
                const uint64_t gi = tb + (uint64_t)(u * WG + tid) * 4;
                uint32_t kept = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const bool isg = (fg[u] >> j) & 1u, ise = (fe[u] >> j) & 1u;
                    if (isg || (ise && pe < e_b)) {
                        if (MASKOUT) {
                            kept |= 1u << j;
                        } else {
                            const uint64_t pos = Pb + pg + min(e_b, pe);
                            idx_out[pos] = (uint32_t)(gi + j - s.lo);
                            v_out[pos] = x[u][j];
                        }
                    }
                    pg += isg ? 1u : 0u;
                    pe += ise ? 1u : 0u;
                }
                if (MASKOUT) {
                    /* pruned = inside the bucket and not kept; 8 quads share a bitmap word */
                    const uint32_t q = u * WG + tid;
                    const uint32_t bits = vm[u] & ~kept;
                    if (bits) atomicOr(&bitmap[q >> 3], bits << ((q & 7u) * 4u));
                }
            }
            __syncthreads();
            if (MASKOUT && tid < TILE / 32) mask_out[(uint64_t)(s.tile_g + ti) * (TILE / 32) + tid] = bitmap[tid];
        }
    }
}

/* ------------------------------------------------------------------ merged stages */

/* Each selection stage is one launch: the first cgrid workgroups walk the candidate segments,
 * the others walk the dense spans of the fallback buckets (usually none: they read the empty
 * list and leave). */
template <int LEVEL, uint32_t GROUP, bool AGG = false>
__global__ __launch_bounds__(WG) void k_refine(const float *__restrict__ r, Tables t, Cand c,
                                               uint32_t *__restrict__ hist_c, uint32_t *__restrict__ hist_f,
                                               uint32_t cgrid)
{
    __shared__ uint32_t h[LEVEL == 1 ? NB1 : NB2];
    if (blockIdx.x < cgrid) {
        if (AGG) crefine_agg_body<LEVEL, GROUP>(t, c, hist_c, h, blockIdx.x, cgrid);
        else crefine_body<LEVEL, GROUP>(t, c, hist_c, blockIdx.x, cgrid);
    } else fb_refine_body<LEVEL>(r, t, hist_f, h, blockIdx.x - cgrid, gridDim.x - cgrid);
}

template <uint32_t GROUP>
__global__ __launch_bounds__(WG) void k_count(const float *__restrict__ r, Tables t, Cand c,
                                              uint32_t *__restrict__ tG, uint32_t *__restrict__ tE,
                                              uint32_t cgrid)
{
    __shared__ uint32_t cnt[MAX_SPAN_TILES][2];
    if (blockIdx.x < cgrid) ccount_body<GROUP>(t, c, blockIdx.x, cgrid);
    else fb_count_body(r, t, tG, tE, cnt, blockIdx.x - cgrid, gridDim.x - cgrid);
}

template <uint32_t GROUP>
__global__ __launch_bounds__(WG) void k_write(const float *__restrict__ r, Tables t, Cand c,
                                              const uint32_t *__restrict__ tG, const uint32_t *__restrict__ tE,
                                              uint32_t *__restrict__ idx_out, float *__restrict__ v_out,
                                              uint32_t cgrid)
{
    __shared__ uint32_t tot[16][2];      /* slot = u * 4 + wavefront */
    if (blockIdx.x < cgrid) cwrite_body<GROUP>(t, c, idx_out, v_out, blockIdx.x, cgrid);
    else fb_write_body<false>(r, t, tG, tE, idx_out, v_out, tot, nullptr, nullptr, blockIdx.x - cgrid,
                              gridDim.x - cgrid);
}

/* ------------------------------------------------------------------ model pruning (optional) */

/* Algorithm 2 Step 2 on the GPU: the kept parameters of a bucket are its n_b - floor(0.5 (1 -
 * ratio) n_b) largest |weight| (ties: lower index kept).  The kept set is more than half of
 * the bucket, so "candidates above a bound" would be most of it; instead the threshold is
 * bracketed: a sample of |w| gives a band of level-0 digits that holds the kw-th largest key
 * with a wide margin, one pass over the weights builds the exact level-0 histogram and stages
 * the elements inside the band, and the remaining digits, the threshold key T and the index
 * of the last kept element among those equal to T come from the staged elements alone.  The
 * gradient kernels then decide "kept" from the weight itself as they stream it (key > T, or
 * key == T and index <= cut).  A bucket whose band missed or overflowed (a sample that was
 * unlucky, a huge group of equal weights) takes the dense ordered passes instead, which leave
 * a bitmap (1 = pruned).  Either way pruned parameters are neither counted nor emitted, and
 * their accumulated gradient is still written to the residual: pruning is not permanent. */

/* Per bucket: the band of keys [lo, hi) to stage, from the sample histogram of |w|. */
__global__ __launch_bounds__(WG) void k_wpredict(Tables t, const uint32_t *__restrict__ hist_s,
                                                 uint32_t *__restrict__ wLo, uint32_t *__restrict__ wHi,
                                                 int force_dense, uint32_t *__restrict__ werr)
{
    __shared__ uint32_t tmp[WG];
    __shared__ uint32_t res[6];          /* digit, above, at for the upper and the lower rank */
    const uint32_t b = blockIdx.x, tid = threadIdx.x;
    if (b == 0 && tid == 0) werr[0] = 0u;        /* the weight stage's own consistency flag */
    const uint64_t nb = t.off[b + 1] - t.off[b];
    const uint32_t k = t.k[b];
    if (nb == 0 || k == 0 || force_dense) {
        if (tid == 0) { wLo[b] = NONE; wHi[b] = 0u; }
        return;
    }
    DigitWalk<NB0> w;
    w.load(hist_s + (uint64_t)b * NB0, tmp);
    const uint32_t m = w.total;
    if (m == 0) {
        if (tid == 0) { wLo[b] = NONE; wHi[b] = 0u; }
        return;
    }
    const bool exact = nb < SAMPLE_ALL_BELOW;
    const double ks = (double)k * (double)m / (double)nb;      /* sample rank of the threshold, from the top */
    const double dev = exact ? 0.0 : 4.0 * sqrt(ks) + 4.0;
    double r_up = floor(ks - dev), r_dn = ceil(ks + dev);
    if (r_up < 1.0) r_up = 1.0;
    if (r_dn < 1.0) r_dn = 1.0;
    if (r_dn > (double)m) r_dn = (double)m;
    if (r_up > (double)m) r_up = (double)m;
    uint32_t digit, above, at;
    if (w.find((uint32_t)r_up, digit, above, at)) { res[0] = digit; res[1] = above; res[2] = at; }
    if (w.find((uint32_t)r_dn, digit, above, at)) { res[3] = digit; res[4] = above; res[5] = at; }
    __syncthreads();
    if (tid == 0) {
        /* sample entries inside the band -> expected staged elements */
        const double in_band = (double)(res[4] + res[5]) - (double)res[1];
        const double est = in_band * (double)nb / (double)m;
        const double cap_b = (double)(t.span0[b + 1] - t.span0[b]) * 4.0 * (double)t.spanT * 256.0;
        /* a bucket sampled in full whose kept set is all of it needs no band either way */
        if (est <= 0.8 * cap_b) { wLo[b] = res[3] << SH0; wHi[b] = (res[0] + 1u) << SH0; }
        else { wLo[b] = NONE; wHi[b] = 0u; }
    }
}

/* One pass over the weights: exact level-0 histogram of |w|, and every element whose key lies
 * in the bucket's band appended, in index order, to its wavefront's staging segment.  Same
 * geometry as the streaming pass of the gradient (64 << segSh threads, one contiguous share
 * of the span per wavefront). */
__global__ __launch_bounds__(64 * MAX_SEG_WAVES) void k_whist(const float *__restrict__ w, Tables t,
                                                              uint32_t *__restrict__ hist0, Cand c,
                                                              const uint32_t *__restrict__ wLo,
                                                              const uint32_t *__restrict__ wHi)
{
    __shared__ uint32_t h[NB0];
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t nthreads = 64u << t.segSh;
    for (uint32_t i = tid; i < NB0; i += nthreads) h[i] = 0;
    const SpanGeo s = span_geo(t, blockIdx.x);
    const uint32_t lo_k = wLo[s.b], hi_k = wHi[s.b];       /* NONE, 0: nothing is staged */
    const uint32_t ss = (blockIdx.x << t.segSh) + wave;
    const uint64_t cbase = (uint64_t)ss * c.cap;
    uint32_t wcount = 0;
    __syncthreads();
    const uint32_t per = (t.spanT * 4u) >> t.segSh;
    const uint32_t wt0 = wave * per;
    const uint32_t wt1 = min(s.ntiles * 4u, wt0 + per);
    for (uint32_t wt = wt0; wt < wt1; ++wt) {
        const uint64_t wb = s.base + (uint64_t)wt * WTILE;
        if (wb >= s.lo && wb + WTILE <= s.hi) {
            f4 wv[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                wv[u] = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(w + wb + (uint64_t)(u * 64 + lane) * 4));
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint64_t gi = wb + (uint64_t)(u * 64 + lane) * 4;
                const float a[4] = {wv[u].x, wv[u].y, wv[u].z, wv[u].w};
                uint32_t key[4];
                bool f[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) { key[j] = keyof(a[j]); f[j] = key[j] >= lo_k && key[j] < hi_k; }
                hist_quad_full(h, key[0] >> SH0, key[1] >> SH0, key[2] >> SH0, key[3] >> SH0);
                emit_quad(f, a, (uint32_t)(gi - s.lo), c, cbase, wcount);
            }
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint64_t gi = wb + (uint64_t)(u * 64 + lane) * 4;
                float a[4];
                const uint32_t m = load_quad(w, gi, s.lo, s.hi, a);
                bool f[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t key = keyof(a[j]);
                    const bool in = (m >> j) & 1u;
                    if (in) atomicAdd(&h[key >> SH0], 1u);
                    f[j] = in && key >= lo_k && key < hi_k;
                }
                emit_quad(f, a, (uint32_t)(gi - s.lo), c, cbase, wcount);
            }
        }
    }
    if (lane == 0) {
        c.cnt[ss] = min(wcount, c.cap);
        if (wcount > c.cap) t.ovf[s.b] = 1u;
    }
    __syncthreads();
    hist_flush(h, hist0 + (uint64_t)s.b * NB0, NB0, (int)nthreads);
}

/* Per bucket: level-0 digit of the kw-th largest |weight|, and whether the staged band can
 * decide the rest: it holds every element of that digit iff the digit lies inside the band
 * and no staging segment overflowed. */
__global__ __launch_bounds__(WG) void k_wplan(Tables t, const uint32_t *__restrict__ hist0,
                                              const uint32_t *__restrict__ wLo, const uint32_t *__restrict__ wHi)
{
    __shared__ uint32_t tmp[WG];
    const uint32_t b = blockIdx.x, tid = threadIdx.x;
    const uint32_t want = t.k[b];
    if (want == 0) {
        if (tid == 0) { t.T[b] = NONE; t.need[b] = 0; t.fast[b] = 1u; }
        return;
    }
    DigitWalk<NB0> w;
    w.load(hist0 + (uint64_t)b * NB0, tmp);
    uint32_t digit, above, at;
    if (w.find(want, digit, above, at)) {
        t.T[b] = digit;
        t.need[b] = want - above;
        const uint32_t lo_k = wLo[b], hi_k = wHi[b];
        const bool valid = lo_k != NONE && (lo_k >> SH0) <= digit && digit < (hi_k >> SH0) && !t.ovf[b];
        t.fast[b] = valid ? 1u : 0u;
    }
}

/* Last stage of the weight select.  Candidate role: per bucket, the index of the last kept
 * element among those equal to the threshold.  Fallback role: the bitmap of a bucket that
 * went through the dense passes. */
template <uint32_t GROUP>
__global__ __launch_bounds__(WG) void k_wfinish(const float *__restrict__ w, Tables t, Cand c,
                                                const uint32_t *__restrict__ tG, const uint32_t *__restrict__ tE,
                                                uint32_t *__restrict__ wcut, uint32_t *__restrict__ mask_out,
                                                uint32_t cgrid)
{
    __shared__ uint32_t tot[16][2];
    __shared__ uint32_t bitmap[TILE / 32];
    if (blockIdx.x < cgrid) cwrite_body<GROUP, true>(t, c, wcut, nullptr, blockIdx.x, cgrid);
    else fb_write_body<true>(w, t, tG, tE, nullptr, nullptr, tot, bitmap, mask_out, blockIdx.x - cgrid,
                             gridDim.x - cgrid);
}

/* ------------------------------------------------------------------ value coding */

/* One workgroup per chunk of `chunk` consecutive survivors of one bucket: absmax, scale,
 * codes, packing, and the coding error left in the residual.  Every floating-point step is a
 * single correctly rounded binary32 operation (divide, round-to-nearest-even, multiply,
 * subtract); nothing may be contracted into an fma. */
template <int BITS>
__global__ __launch_bounds__(WG) void k_quant(const float *__restrict__ v, const uint32_t *__restrict__ idx,
                                              Tables t, float *__restrict__ r, void *__restrict__ val,
                                              float *__restrict__ scales)
{
    __shared__ float red[WG / 64];
    const uint32_t tid = threadIdx.x;
    const uint64_t c = blockIdx.x;
    const uint32_t b = find_bucket<uint64_t>(t.C, t.B, c);
    const uint64_t cb = c - t.C[b];
    const uint64_t j0 = cb * t.chunk;                         /* first survivor of the chunk, bucket-local */
    const uint32_t cnt = (uint32_t)min((uint64_t)t.chunk, (uint64_t)t.k[b] - j0);
    const uint64_t jg = t.P[b] + j0;                          /* same, global */
    const uint64_t lo = t.off[b];
    float scale = 0.0f;
    if (BITS <= 8) {
        constexpr float QMAX = BITS == 8 ? 127.0f : 7.0f;
        float m = 0.0f;
        for (uint32_t i = tid; i < cnt; i += WG) m = fmaxf(m, fabsf(v[jg + i]));
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) m = fmaxf(m, __shfl_xor(m, d, 64));
        if ((tid & 63) == 0) red[tid >> 6] = m;
        __syncthreads();
        m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        scale = m == 0.0f ? 0.0f : __fdiv_rn(m, QMAX);
        if (tid == 0) scales[t.S[b] + cb] = scale;
    }
    uint8_t *vb = reinterpret_cast<uint8_t *>(val) + t.V[b];
    /* two survivors per thread per round, so a 4-bit pair is one byte store */
    for (uint32_t p = tid; 2 * p < cnt; p += WG) {
        float res[2];
        int q[2] = {0, 0};
        const uint32_t i0 = 2 * p;
        const int have = (i0 + 1 < cnt) ? 2 : 1;
        for (int h = 0; h < have; ++h) {
            const float x = v[jg + i0 + h];
            float deq;
            if (BITS == 32) {
                deq = x;
            } else if (BITS == 16) {
                const __half hv = __float2half_rn(x);
                reinterpret_cast<__half *>(vb)[j0 + i0 + h] = hv;
                deq = __half2float(hv);
            } else {
                constexpr float QMAX = BITS == 8 ? 127.0f : 7.0f;
                if (scale != 0.0f) {
                    float tq = rintf(__fdiv_rn(x, scale));
                    tq = fminf(fmaxf(tq, -QMAX), QMAX);
                    q[h] = (int)tq;
                }
                deq = __fmul_rn((float)q[h], scale);
                if (BITS == 8) reinterpret_cast<int8_t *>(vb)[j0 + i0 + h] = (int8_t)q[h];
            }
            res[h] = __fsub_rn(x, deq);
        }
        if (BITS == 4) vb[(j0 >> 1) + p] = (uint8_t)((q[0] & 0xF) | ((q[1] & 0xF) << 4));
        for (int h = 0; h < have; ++h) r[lo + idx[jg + i0 + h]] = res[h];
    }
}

/* ------------------------------------------------------------------ decompress */

template <int BITS>
__device__ __forceinline__ float decode(const uint8_t *__restrict__ vb, const float *__restrict__ sc,
                                        uint64_t j, uint32_t chunk)
{
    if (BITS == 32) return reinterpret_cast<const float *>(vb)[j];
    if (BITS == 16) return __half2float(reinterpret_cast<const __half *>(vb)[j]);
    int q;
    if (BITS == 8) q = reinterpret_cast<const int8_t *>(vb)[j];
    else {
        const uint32_t byte = vb[j >> 1];
        const int nib = (j & 1) ? (int)(byte >> 4) : (int)(byte & 0xFu);
        q = nib >= 8 ? nib - 16 : nib;
    }
    return __fmul_rn((float)q, sc[j / chunk]);
}

/* Where each tile's survivors start in its bucket's ascending index list: ts[tile0[b] + b + i]
 * = number of survivors of bucket b with an index below tile i (i = 0..tiles_b).  A thread
 * takes TS_PER consecutive survivors (8 for long payloads, 2 for short ones, which need the
 * threads more); a survivor whose tile differs from its predecessor's writes the entries of
 * the tiles that begin between the two, and the last survivor of a bucket also closes the
 * bucket's remaining tiles. */

__device__ __forceinline__ void tilestart_one(const uint32_t *__restrict__ idx, const Tables &t, uint32_t b,
                                              uint64_t j, uint32_t *__restrict__ ts)
{
    const uint32_t tiles_b = t.tile0[b + 1] - t.tile0[b];
    const uint32_t kb = t.k[b];
    const uint32_t jj = (uint32_t)(j - t.P[b]);
    uint32_t *tsb = ts + t.tile0[b] + b;
    const uint32_t head = (uint32_t)(t.off[b] & 3ull);
    /* tile of a local index; indices beyond the bucket (invalid payload) count as the last tile */
    uint32_t tcur = (uint32_t)(((uint64_t)idx[j] + head) / TILE);
    tcur = min(tcur, tiles_b - 1);
    uint32_t tfrom = 0;                         /* first tile this survivor fills */
    if (jj > 0) {
        uint32_t tprev = (uint32_t)(((uint64_t)idx[j - 1] + head) / TILE);
        tprev = min(tprev, tiles_b - 1);
        tfrom = tprev + 1;
    }
    for (uint32_t tt = tfrom; tt <= tcur; ++tt) tsb[tt] = jj;
    if (jj == kb - 1)
        for (uint32_t tt = tcur + 1; tt <= tiles_b; ++tt) tsb[tt] = kb;
}

template <uint32_t TS_PER>
__global__ __launch_bounds__(WG) void k_tilestart(const uint32_t *__restrict__ idx, Tables t,
                                                  uint64_t K, uint32_t *__restrict__ ts)
{
    constexpr uint32_t LDS_B = 2047;
    __shared__ uint64_t sP[LDS_B + 1];
    const bool in_lds = t.B <= LDS_B;
    if (in_lds) {
        for (uint32_t i = threadIdx.x; i <= t.B; i += WG) sP[i] = t.P[i];
        __syncthreads();
    }
    const uint64_t stride = (uint64_t)gridDim.x * WG * TS_PER;
    for (uint64_t j0 = ((uint64_t)blockIdx.x * WG + threadIdx.x) * TS_PER; j0 < K; j0 += stride) {
        const uint32_t b = in_lds ? find_bucket<uint64_t>(sP, t.B, j0) : find_bucket<uint64_t>(t.P, t.B, j0);
        const uint64_t Pb = t.P[b], Pn = t.P[b + 1];
        if (j0 > Pb && j0 + TS_PER < Pn) {
            /* all of them inside one bucket, none its first or last survivor: only tile changes matter */
            const uint32_t tiles_b = t.tile0[b + 1] - t.tile0[b];
            const uint32_t head = (uint32_t)(t.off[b] & 3ull);
            uint32_t *tsb = ts + t.tile0[b] + b;
            uint32_t v[TS_PER + 1];
#pragma unroll
            for (uint32_t i = 0; i <= TS_PER; ++i) v[i] = idx[j0 - 1 + i];
#pragma unroll
            for (uint32_t i = 0; i <= TS_PER; ++i) v[i] = min((uint32_t)(((uint64_t)v[i] + head) / TILE), tiles_b - 1);
            if (v[0] != v[TS_PER]) {
                const uint32_t jj0 = (uint32_t)(j0 - Pb);
#pragma unroll
                for (uint32_t i = 1; i <= TS_PER; ++i)
                    for (uint32_t tt = v[i - 1] + 1; tt <= v[i]; ++tt) tsb[tt] = jj0 + i - 1;
            }
        } else {
            for (uint64_t j = j0; j < min(K, j0 + TS_PER); ++j) {
                const uint32_t bj = j < Pn ? b : (in_lds ? find_bucket<uint64_t>(sP, t.B, j) : find_bucket<uint64_t>(t.P, t.B, j));
                tilestart_one(idx, t, bj, j, ts);
            }
        }
    }
}

/* Dense output for a span of tiles: each tile is assembled in LDS (zeros, then the decoded
 * survivors that fall inside it, found through the tile-start table) and written out once with
 * aligned 16-byte stores, so no output line is touched twice and no atomics are needed.  The
 * loads of the next tile's survivors are issued before the current tile is written out. */
template <int BITS, bool NTS>
__global__ __launch_bounds__(WG) void k_decomp(const uint32_t *__restrict__ idx, const void *__restrict__ val,
                                               const float *__restrict__ scales, Tables t,
                                               const uint32_t *__restrict__ ts, float *__restrict__ dense)
{
    __shared__ float tile[TILE];
    __shared__ uint32_t sts[MAX_SPAN_TILES + 1];
    const uint32_t tid = threadIdx.x;
    const SpanGeo s = span_geo(t, blockIdx.x);
    const uint32_t kb = t.k[s.b];
    const uint32_t *ib = idx + t.P[s.b];
    const uint8_t *vb = reinterpret_cast<const uint8_t *>(val) + t.V[s.b];
    const float *sb = BITS <= 8 ? scales + t.S[s.b] : nullptr;
    const uint32_t nb = (uint32_t)(s.hi - s.lo);
    const uint32_t first = s.tile_g - t.tile0[s.b];
    if (tid <= s.ntiles) sts[tid] = min(ts[t.tile0[s.b] + s.b + first + tid], kb);
    __syncthreads();

    /* survivor number j0 + tid of a tile, if it exists: local index and decoded value */
    uint32_t p_li = NONE;
    float p_x = 0.0f;
    auto fetch = [&](uint32_t ti) {
        p_li = NONE;
        if (ti < s.ntiles) {
            const uint32_t j0 = sts[ti], j1 = sts[ti + 1];
            const uint64_t j = (uint64_t)j0 + tid;
            if (j < j1) { p_li = ib[j]; p_x = decode<BITS>(vb, sb, j, t.chunk); }
        }
    };
    fetch(0);
    for (uint32_t ti = 0; ti < s.ntiles; ++ti) {
        const uint64_t tb = s.base + (uint64_t)ti * TILE;
        const uint64_t shift = s.lo - tb;                   /* slot = local index + lo - tb (mod 2^64) */
#pragma unroll
        for (int u = 0; u < 4; ++u)
            *reinterpret_cast<f4 *>(&tile[(u * WG + tid) * 4]) = f4{0.f, 0.f, 0.f, 0.f};
        __syncthreads();
        if (p_li < nb) {
            const uint64_t slot = (uint64_t)p_li + shift;
            if (slot < TILE) tile[slot] = p_x;
        }
        /* more than 256 survivors in the tile (ratio above 6 %) */
        const uint32_t j0 = sts[ti], j1 = sts[ti + 1];
        for (uint64_t j = (uint64_t)j0 + WG + tid; j < j1; j += WG) {
            const uint32_t li = ib[j];
            const uint64_t slot = (uint64_t)li + shift;
            if (li < nb && slot < TILE) tile[slot] = decode<BITS>(vb, sb, j, t.chunk);
        }
        fetch(ti + 1);
        __syncthreads();
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t sl = (u * WG + tid) * 4;
            const uint64_t gi = tb + sl;
            if (gi >= s.lo && gi + 4 <= s.hi) {
                const f4 v = *reinterpret_cast<const f4 *>(&tile[sl]);
                if (NTS) __builtin_nontemporal_store(v, reinterpret_cast<f4 *>(dense + gi));
                else *reinterpret_cast<f4 *>(dense + gi) = v;
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (gi + j >= s.lo && gi + j < s.hi) dense[gi + j] = tile[sl + j];
            }
        }
    }
}

/* Receiver side of an all-gather of payloads: add one worker's decoded survivors into a dense
 * gradient that is being accumulated (nothing else is touched).  One thread per survivor;
 * the indices of a payload are distinct, so plain read-modify-write needs no atomics. */
template <int BITS>
__global__ __launch_bounds__(WG) void k_decomp_acc(const uint32_t *__restrict__ idx, const void *__restrict__ val,
                                                   const float *__restrict__ scales, Tables t, uint64_t K,
                                                   float *__restrict__ dense)
{
    constexpr uint32_t LDS_B = 2047;
    __shared__ uint64_t sP[LDS_B + 1];
    const bool in_lds = t.B <= LDS_B;
    if (in_lds) {
        for (uint32_t i = threadIdx.x; i <= t.B; i += WG) sP[i] = t.P[i];
        __syncthreads();
    }
    const uint64_t stride = (uint64_t)gridDim.x * WG;
    for (uint64_t j = (uint64_t)blockIdx.x * WG + threadIdx.x; j < K; j += stride) {
        const uint32_t b = in_lds ? find_bucket<uint64_t>(sP, t.B, j) : find_bucket<uint64_t>(t.P, t.B, j);
        const uint64_t lo = t.off[b], nb = t.off[b + 1] - lo;
        const uint64_t jj = j - t.P[b];
        const uint32_t li = idx[j];
        if (li >= nb) continue;                       /* invalid payload: never leave the bucket */
        const uint8_t *vb = reinterpret_cast<const uint8_t *>(val) + t.V[b];
        const float *sb = BITS <= 8 ? scales + t.S[b] : nullptr;
        const float x = decode<BITS>(vb, sb, jj, t.chunk);
        dense[lo + li] = __fadd_rn(dense[lo + li], x);
    }
}

}  // namespace

/* ====================================================================== host side */

struct nsml_ctx {
    int device;
    uint64_t max_n;
    uint32_t max_buckets;
    uint32_t chunk;
    int last_hip;
    uint64_t ws_bytes;
    uint32_t max_tiles;
    uint64_t max_cand;     /* staging entries */

    /* device workspace */
    uint64_t *d_off, *d_P, *d_V, *d_S, *d_C;
    uint32_t *d_tile0, *d_span0, *d_samp0, *d_span_b, *d_k, *d_T, *d_need, *d_L, *d_fast, *d_fspan0;
    uint32_t *d_zero;      /* cleared by every compress call: histograms and overflow flags */
    uint32_t *d_tG, *d_tE; /* per tile (fallback path) */
    uint32_t *d_ccnt, *d_cG, *d_cE, *d_cidx;   /* candidate staging */
    float *d_cval;
    float *d_v;            /* survivor values in final order (not used for bits == 32) */
    uint32_t *d_ts;        /* decompress: where each tile's survivors start */
    uint32_t *d_pmask;     /* pruning bitmap, 128 words per tile */
    uint32_t *d_kw, *d_Tw, *d_needw;              /* pruning stage: kept counts, threshold search state */
    uint32_t *d_wT, *d_wcut, *d_wfast;            /* pruning stage: threshold key and cut index per bucket; path taken */
    uint32_t *d_wLo, *d_wHi;                      /* pruning stage: band of keys staged per bucket */
    uint32_t *d_werr;                             /* pruning stage: consistency flag (1 word) */
    bool have_prune;                              /* the last compress call had weights */
    double *d_span_sq;     /* per span: sum of grad^2 */
    double *d_l2sq;        /* per bucket: sum of grad^2 of the last compress call */
    bool have_l2;

    /* host copies / caches */
    std::vector<uint64_t> h_off;
    uint32_t B;
    uint64_t n;
    uint32_t n_tiles, n_spans, n_samp, spanT, segSh;
    bool tables_valid;
    double t_ratio; int t_bits;       /* what d_k/d_P/... were computed for */
    uint64_t K, NC;                   /* totals for (layout, t_ratio, t_bits) */
    void *pinned; size_t pinned_bytes;
    int span_override;
    int seg_override;      /* wavefronts per workgroup of the streaming pass (0: by span size) */
    int group_override;    /* lanes per staging segment in the candidate kernels (0: by ratio) */
    int agg_override;      /* level-1 candidate histogram aggregated in LDS: 1 always, 0 never, -1 by size */
    int force_dense;
    int nt_mode;
    int nt_dense;          /* non-temporal stores for the dense output of decompress */
    int use_history;       /* place the candidate bound from the previous call's thresholds */
    bool hist_ready; double hist_ratio; bool hist_pruned;
    uint32_t *d_margin;

    /* profiling */
    bool prof;
    struct Rec { int kid; hipEvent_t a, b; };
    std::vector<Rec> recs;
    std::vector<hipEvent_t> pool;
};

namespace {

struct DeviceGuard {
    int prev; bool ok;
    explicit DeviceGuard(int dev) : prev(-1), ok(false) {
        if (hipGetDevice(&prev) != hipSuccess) prev = -1;
        ok = hipSetDevice(dev) == hipSuccess;
    }
    ~DeviceGuard() { if (prev >= 0) (void)hipSetDevice(prev); }
};

#define NSML_HIP(ctx, call)                                                        \
    do {                                                                           \
        hipError_t e_ = (call);                                                    \
        if (e_ != hipSuccess) { (ctx)->last_hip = (int)e_; return NSML_EHIP; }     \
    } while (0)

template <typename T>
int dev_alloc(nsml_ctx *c, T **p, uint64_t count)
{
    const uint64_t bytes = (count ? count : 1) * sizeof(T);
    NSML_HIP(c, hipMalloc(reinterpret_cast<void **>(p), bytes));
    c->ws_bytes += bytes;
    return NSML_OK;
}

/* words of the per-call zeroed area: hist0, sample hist, candidate level 1/2, fallback level
 * 1/2 histograms, overflow flags */
uint64_t zero_words(uint64_t B) { return B * (uint64_t)(NB0 + NB0 + NB1 + NB2 + NB1 + NB2 + 1) + 16; }

struct Hists { uint32_t *h0, *hs, *c1, *c2, *f1, *f2, *ovf, *ticket, *err; };
Hists hists_of(const nsml_ctx *c, uint32_t B)
{
    Hists h;
    h.h0 = c->d_zero;
    h.hs = h.h0 + (uint64_t)B * NB0;
    h.c1 = h.hs + (uint64_t)B * NB0;
    h.c2 = h.c1 + (uint64_t)B * NB1;
    h.f1 = h.c2 + (uint64_t)B * NB2;
    h.f2 = h.f1 + (uint64_t)B * NB1;
    h.ovf = h.f2 + (uint64_t)B * NB2;
    h.ticket = h.ovf + B;
    h.err = h.ticket + 1;
    return h;
}

Tables tables_of(const nsml_ctx *c)
{
    Tables t;
    t.off = c->d_off; t.tile0 = c->d_tile0; t.span0 = c->d_span0; t.samp0 = c->d_samp0;
    t.span_b = c->d_span_b;
    t.k = c->d_k; t.P = c->d_P; t.V = c->d_V; t.S = c->d_S; t.C = c->d_C;
    t.T = c->d_T; t.need = c->d_need; t.L = c->d_L; t.fast = c->d_fast;
    t.ovf = hists_of(c, c->B).ovf; t.fspan0 = c->d_fspan0;
    t.kw = c->d_kw; t.w = nullptr; t.wT = nullptr; t.wcut = nullptr; t.pmask = nullptr; t.margin = c->d_margin;
    t.B = c->B; t.n_spans = c->n_spans; t.spanT = c->spanT; t.segSh = c->segSh; t.chunk = c->chunk;
    return t;
}

Cand cand_of(const nsml_ctx *c)
{
    Cand k;
    k.idx = c->d_cidx; k.val = c->d_cval; k.cnt = c->d_ccnt; k.G = c->d_cG; k.E = c->d_cE;
    k.cap = (c->spanT * (TILE / 4)) >> c->segSh;
    k.splitSh = 0;
    return k;
}

/* Profiling brackets */
int prof_begin(nsml_ctx *c, int kid, hipStream_t st)
{
    if (!c->prof || c->recs.size() >= 4096) return NSML_OK;
    nsml_ctx::Rec r; r.kid = kid;
    for (hipEvent_t *e : {&r.a, &r.b}) {
        if (!c->pool.empty()) { *e = c->pool.back(); c->pool.pop_back(); }
        else NSML_HIP(c, hipEventCreate(e));
    }
    NSML_HIP(c, hipEventRecord(r.a, st));
    c->recs.push_back(r);
    return NSML_OK;
}
int prof_end(nsml_ctx *c, int kid, hipStream_t st)
{
    if (!c->prof || c->recs.empty() || c->recs.back().kid != kid) return NSML_OK;
    NSML_HIP(c, hipEventRecord(c->recs.back().b, st));
    return NSML_OK;
}

#define LAUNCHB(ctx, kid, st, kernel, grid, block, ...)                             \
    do {                                                                            \
        int rc_ = prof_begin(ctx, kid, st);                                         \
        if (rc_) return rc_;                                                        \
        hipLaunchKernelGGL(kernel, dim3(grid), dim3(block), 0, st, __VA_ARGS__);    \
        NSML_HIP(ctx, hipGetLastError());                                           \
        rc_ = prof_end(ctx, kid, st);                                               \
        if (rc_) return rc_;                                                        \
    } while (0)
#define LAUNCH(ctx, kid, st, kernel, grid, ...) LAUNCHB(ctx, kid, st, kernel, grid, WG, __VA_ARGS__)

bool aligned(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

/* Tiles per span (one span = one workgroup of the streaming kernels, four candidate
 * segments).  Small spans stream a few per cent faster, large spans mean fewer segments for
 * the candidate kernels to walk; measured on 25 M .. 6.7 G elements the totals favour this. */
uint32_t pick_span_tiles(uint32_t n_tiles, int override_)
{
    if (override_ >= 1 && override_ <= MAX_SPAN_TILES) return (uint32_t)override_;
    if (n_tiles >= 16u * 4096u) return 16;
    if (n_tiles >= 8u * 2048u) return 8;
    if (n_tiles >= 4u * 1024u) return 4;
    if (n_tiles >= 2u * 512u) return 2;
    return 1;
}

/* log2 of the wavefronts per workgroup of the streaming pass (= staging segments per span):
 * one wavefront per tile for spans of 8 and 16 tiles, four wavefronts otherwise.  Every
 * wavefront gets at least one wave-tile. */
uint32_t pick_seg_shift(uint32_t spanT, int override_)
{
    uint32_t w = override_ > 0 ? (uint32_t)override_ : (spanT > 4 ? spanT : 4u);
    const uint32_t hi = spanT * 4u < MAX_SEG_WAVES ? spanT * 4u : MAX_SEG_WAVES;
    if (w > hi) w = hi;
    uint32_t sh = 2;
    while ((2u << sh) <= w) ++sh;
    return sh;
}

/* Validate a bucket layout; (re)build the layout tables if it differs from the cached one. */
int ensure_layout(nsml_ctx *c, uint64_t n, const uint64_t *off, uint32_t B, hipStream_t st)
{
    if (!off || B == 0 || n == 0) return NSML_EINVAL;
    if (B > c->max_buckets || n > c->max_n) return NSML_ECAP;
    if (off[0] != 0 || off[B] != n) return NSML_EINVAL;
    for (uint32_t b = 0; b < B; ++b) {
        if (off[b + 1] < off[b]) return NSML_EINVAL;
        if (off[b + 1] - off[b] > 0xFFFFFFFFull) return NSML_EINVAL;
    }
    if (c->B == B && c->n == n && c->h_off.size() == (size_t)B + 1 &&
        memcmp(c->h_off.data(), off, sizeof(uint64_t) * ((size_t)B + 1)) == 0)
        return NSML_OK;

    /* new layout: tiles start at the bucket start rounded down to a multiple of 4 */
    const size_t B1 = (size_t)B + 1;
    std::vector<uint32_t> tile0(B1), span0(B1), samp0(B1);
    uint64_t nt = 0, nsamp = 0;
    for (uint32_t b = 0; b < B; ++b) {
        tile0[b] = (uint32_t)nt;
        samp0[b] = (uint32_t)nsamp;
        const uint64_t lo = off[b], hi = off[b + 1];
        if (hi > lo) {
            const uint64_t len = hi - (lo & ~3ull);
            nt += (len + TILE - 1) / TILE;
            const uint64_t run_elems = 32ull * ((hi - lo) < SAMPLE_ALL_BELOW ? 1 : SAMPLE_STRIDE);
            const uint64_t runs = (len + run_elems - 1) / run_elems;
            nsamp += (runs + RUNS_PER_WG - 1) / RUNS_PER_WG;
        }
        if (nt > c->max_tiles) return NSML_ECAP;
    }
    tile0[B] = (uint32_t)nt;
    samp0[B] = (uint32_t)nsamp;
    const uint32_t spanT = pick_span_tiles((uint32_t)nt, c->span_override);
    uint64_t ns = 0;
    for (uint32_t b = 0; b < B; ++b) {
        span0[b] = (uint32_t)ns;
        ns += (tile0[b + 1] - tile0[b] + spanT - 1) / spanT;
    }
    span0[B] = (uint32_t)ns;
    if (ns * 4ull * spanT * 256ull > c->max_cand) return NSML_ECAP;

    /* the stream may still be using the old tables */
    NSML_HIP(c, hipStreamSynchronize(st));
    c->tables_valid = false;
    c->B = 0;
    const size_t need = sizeof(uint64_t) * B1 + 3 * sizeof(uint32_t) * B1;
    if (need > c->pinned_bytes) return NSML_ECAP;
    uint8_t *hp = static_cast<uint8_t *>(c->pinned);
    uint8_t *hp_t = hp + sizeof(uint64_t) * B1;
    uint8_t *hp_s = hp_t + sizeof(uint32_t) * B1;
    uint8_t *hp_m = hp_s + sizeof(uint32_t) * B1;
    memcpy(hp, off, sizeof(uint64_t) * B1);
    memcpy(hp_t, tile0.data(), sizeof(uint32_t) * B1);
    memcpy(hp_s, span0.data(), sizeof(uint32_t) * B1);
    memcpy(hp_m, samp0.data(), sizeof(uint32_t) * B1);
    NSML_HIP(c, hipMemcpyAsync(c->d_off, hp, sizeof(uint64_t) * B1, hipMemcpyHostToDevice, st));
    NSML_HIP(c, hipMemcpyAsync(c->d_tile0, hp_t, sizeof(uint32_t) * B1, hipMemcpyHostToDevice, st));
    NSML_HIP(c, hipMemcpyAsync(c->d_span0, hp_s, sizeof(uint32_t) * B1, hipMemcpyHostToDevice, st));
    NSML_HIP(c, hipMemcpyAsync(c->d_samp0, hp_m, sizeof(uint32_t) * B1, hipMemcpyHostToDevice, st));
    LAUNCH(c, KID_SPANMAP, st, k_spanmap, (uint32_t)((ns + WG - 1) / WG), (const uint32_t *)c->d_span0, B,
           (uint32_t)ns, c->d_span_b);
    LAUNCH(c, KID_SPANMAP, st, k_fill_u32, (B + WG - 1) / WG, c->d_margin, B, MARGIN_INIT);
    c->hist_ready = false;
    NSML_HIP(c, hipStreamSynchronize(st));

    c->h_off.assign(off, off + B + 1);
    c->B = B; c->n = n;
    c->n_tiles = (uint32_t)nt; c->n_spans = (uint32_t)ns; c->n_samp = (uint32_t)nsamp; c->spanT = spanT;
    c->segSh = pick_seg_shift(spanT, c->seg_override);
    return NSML_OK;
}

/* Make d_k / d_P / d_V / d_S / d_C match (ratio, bits) for the cached layout. */
int ensure_tables(nsml_ctx *c, double ratio, int bits, hipStream_t st)
{
    if (!(ratio > 0.0 && ratio <= 1.0)) return NSML_EINVAL;
    if (bits != 4 && bits != 8 && bits != 16 && bits != 32) return NSML_EINVAL;
    if (c->tables_valid && c->t_ratio == ratio && c->t_bits == bits) return NSML_OK;
    uint64_t K = 0, nc = 0;
    {
        std::vector<uint64_t> kb(c->B);
        int rc = nsml_payload_layout(c->h_off.data(), c->B, ratio, bits, c->chunk, kb.data(), &K, nullptr, nullptr);
        if (rc) return rc;
        for (uint32_t b = 0; b < c->B; ++b) nc += (kb[b] + c->chunk - 1) / c->chunk;
    }
    if (nc >= 0x7FFFFFFFull) return NSML_ECAP;
    LAUNCH(c, KID_SETUP, st, k_setup, 1, tables_of(c), ratio, bits);
    c->K = K; c->NC = nc;
    c->t_ratio = ratio; c->t_bits = bits;
    c->tables_valid = true;
    return NSML_OK;
}

}  // namespace

extern "C" {

int nsml_create(nsml_ctx **out, int device, uint64_t max_n, uint32_t max_buckets, uint32_t chunk)
{
    if (!out || max_n == 0 || max_buckets == 0 || chunk == 0 || chunk % 8 != 0) return NSML_EINVAL;
    *out = nullptr;
    nsml_ctx *c = new (std::nothrow) nsml_ctx();
    if (!c) return NSML_ENOMEM;
    c->device = device; c->max_n = max_n; c->max_buckets = max_buckets; c->chunk = chunk;
    c->last_hip = 0; c->ws_bytes = 0; c->B = 0; c->n = 0; c->tables_valid = false;
    c->prof = false; c->pinned = nullptr; c->pinned_bytes = 0;
    c->d_off = c->d_P = c->d_V = c->d_S = c->d_C = nullptr;
    c->d_tile0 = c->d_span0 = c->d_samp0 = c->d_span_b = c->d_k = c->d_T = c->d_need = nullptr;
    c->d_L = c->d_fast = c->d_fspan0 = c->d_zero = c->d_tG = c->d_tE = nullptr;
    c->d_ccnt = c->d_cG = c->d_cE = c->d_cidx = nullptr;
    c->d_cval = nullptr; c->d_v = nullptr; c->d_ts = nullptr; c->d_span_sq = c->d_l2sq = nullptr; c->have_l2 = false;
    c->d_pmask = c->d_kw = c->d_Tw = c->d_needw = c->d_wT = c->d_wfast = c->d_wcut = c->d_wLo = c->d_wHi = c->d_werr = nullptr;
    c->have_prune = false;
    const char *so = getenv("NSML_SPAN_TILES");
    c->span_override = so ? atoi(so) : 0;
    const char *sw = getenv("NSML_SEG_WAVES");
    c->seg_override = sw ? atoi(sw) : 0;
    c->segSh = 2;
    const char *ao = getenv("NSML_AGG");
    c->agg_override = ao ? (atoi(ao) != 0 ? 1 : 0) : -1;
    const char *go = getenv("NSML_GROUP");
    c->group_override = go ? atoi(go) : 0;
    const char *fd = getenv("NSML_FORCE_DENSE");
    c->force_dense = (fd && atoi(fd) != 0) ? 1 : 0;
    const char *ntm = getenv("NSML_NT");
    c->nt_mode = ntm ? atoi(ntm) : 7;
    const char *nd = getenv("NSML_NT_DENSE");
    c->nt_dense = nd ? (atoi(nd) != 0) : 1;
    const char *hs = getenv("NSML_HISTORY");
    /* off by default: while error feedback is still building up, thresholds climb from step to
     * step and bounds taken from the previous step let in about twice the candidates a fresh
     * sample does; the sample costs 1 % of a step */
    c->use_history = hs ? (atoi(hs) != 0) : 0;
    c->hist_ready = false; c->hist_ratio = 0.0; c->hist_pruned = false; c->d_margin = nullptr;

    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || device < 0 || device >= ndev) {
        c->last_hip = (int)hipErrorInvalidDevice;
        delete c;
        return NSML_EHIP;
    }
    DeviceGuard guard(device);
    if (!guard.ok) { delete c; return NSML_EHIP; }

    /* every bucket can add one partial tile at each end */
    const uint64_t mt = max_n / TILE + 2ull * max_buckets + 2;
    if (mt >= 0x3FFFFFFFull) { delete c; return NSML_ECAP; }
    c->max_tiles = (uint32_t)mt;
    /* staging: a quarter of the elements every span covers; a span is at most 16 tiles and
     * every bucket can leave one span partly filled */
    c->max_cand = (mt + (uint64_t)MAX_SPAN_TILES * max_buckets) * (TILE / 4);
    const uint64_t B1 = (uint64_t)max_buckets + 1;
    int rc = NSML_OK;
    auto A = [&](int r) { if (rc == NSML_OK) rc = r; };
    A(dev_alloc(c, &c->d_off, B1)); A(dev_alloc(c, &c->d_P, B1)); A(dev_alloc(c, &c->d_V, B1));
    A(dev_alloc(c, &c->d_S, B1)); A(dev_alloc(c, &c->d_C, B1));
    A(dev_alloc(c, &c->d_tile0, B1)); A(dev_alloc(c, &c->d_span0, B1)); A(dev_alloc(c, &c->d_samp0, B1));
    A(dev_alloc(c, &c->d_k, B1)); A(dev_alloc(c, &c->d_T, B1)); A(dev_alloc(c, &c->d_need, B1));
    A(dev_alloc(c, &c->d_L, B1)); A(dev_alloc(c, &c->d_fast, B1)); A(dev_alloc(c, &c->d_fspan0, B1));
    A(dev_alloc(c, &c->d_span_b, mt));
    A(dev_alloc(c, &c->d_zero, zero_words(max_buckets)));
    A(dev_alloc(c, &c->d_tG, mt)); A(dev_alloc(c, &c->d_tE, mt));
    /* segments: at most 4 per tile-sized span, or one per tile plus a partly filled span per bucket */
    const uint64_t msg = 4 * mt + (uint64_t)MAX_SEG_WAVES * B1;
    A(dev_alloc(c, &c->d_ccnt, msg)); A(dev_alloc(c, &c->d_cG, msg)); A(dev_alloc(c, &c->d_cE, msg));
    A(dev_alloc(c, &c->d_cidx, c->max_cand)); A(dev_alloc(c, &c->d_cval, c->max_cand));
    A(dev_alloc(c, &c->d_v, max_n));
    A(dev_alloc(c, &c->d_ts, mt + B1 + 1));
    A(dev_alloc(c, &c->d_span_sq, mt)); A(dev_alloc(c, &c->d_l2sq, B1));
    A(dev_alloc(c, &c->d_pmask, mt * (TILE / 32)));
    A(dev_alloc(c, &c->d_kw, B1)); A(dev_alloc(c, &c->d_Tw, B1)); A(dev_alloc(c, &c->d_needw, B1));
    A(dev_alloc(c, &c->d_margin, B1));
    A(dev_alloc(c, &c->d_wT, B1)); A(dev_alloc(c, &c->d_wfast, B1)); A(dev_alloc(c, &c->d_wcut, B1));
    A(dev_alloc(c, &c->d_wLo, B1)); A(dev_alloc(c, &c->d_wHi, B1)); A(dev_alloc(c, &c->d_werr, 1));
    if (rc == NSML_OK) {
        c->pinned_bytes = B1 * 20;
        hipError_t e = hipHostMalloc(&c->pinned, c->pinned_bytes, hipHostMallocDefault);
        if (e != hipSuccess) { c->last_hip = (int)e; rc = NSML_EHIP; }
    }
    if (rc != NSML_OK) { nsml_destroy(c); return rc; }
    *out = c;
    return NSML_OK;
}

int nsml_destroy(nsml_ctx *c)
{
    if (!c) return NSML_EINVAL;
    DeviceGuard guard(c->device);
    (void)hipDeviceSynchronize();
    void *ptrs[] = {c->d_off, c->d_P, c->d_V, c->d_S, c->d_C, c->d_tile0, c->d_span0, c->d_samp0,
                    c->d_span_b, c->d_k, c->d_T, c->d_need, c->d_L, c->d_fast, c->d_fspan0,
                    c->d_zero, c->d_tG, c->d_tE, c->d_ccnt, c->d_cG, c->d_cE, c->d_cidx,
                    c->d_cval, c->d_v, c->d_ts, c->d_span_sq, c->d_l2sq, c->d_pmask, c->d_kw,
                    c->d_Tw, c->d_needw, c->d_margin, c->d_wT, c->d_wfast, c->d_wcut,
                    c->d_wLo, c->d_wHi, c->d_werr};
    for (void *p : ptrs) if (p) (void)hipFree(p);
    if (c->pinned) (void)hipHostFree(c->pinned);
    for (auto &r : c->recs) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    for (auto e : c->pool) (void)hipEventDestroy(e);
    delete c;
    return NSML_OK;
}

int nsml_last_hip_error(const nsml_ctx *c) { return c ? c->last_hip : 0; }
uint64_t nsml_workspace_bytes(const nsml_ctx *c) { return c ? c->ws_bytes : 0; }

/* Shared body of nsml_compress and nsml_compress_pruned (weights == NULL: no pruning). */
static int compress_impl(nsml_ctx *c, const float *grad, float *residual, const float *weights,
                         uint64_t n, const uint64_t *bucket_off, uint32_t B, double ratio, int bits,
                         uint32_t *idx, void *val, float *scales, void *stream)
{
    if (!c || !grad || !residual || !idx || !val) return NSML_EINVAL;
    if ((bits == 8 || bits == 4) && !scales) return NSML_EINVAL;
    if (!aligned(grad, 16) || !aligned(residual, 16) || !aligned(idx, 4) || !aligned(val, 4) ||
        !aligned(scales, 4) || !aligned(weights, 16))
        return NSML_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    DeviceGuard guard(c->device);
    if (!guard.ok) { c->last_hip = (int)hipErrorInvalidDevice; return NSML_EHIP; }
    int rc = ensure_layout(c, n, bucket_off, B, st);
    if (rc) return rc;
    rc = ensure_tables(c, ratio, bits, st);
    if (rc) return rc;

    Tables t = tables_of(c);
    const Cand cd0 = cand_of(c);
    const Hists h = hists_of(c, B);
    const uint64_t zw = zero_words(B);
    const uint32_t clear_grid = (uint32_t)((zw + WG * 8 - 1) / (WG * 8));
    float *vdst = bits == 32 ? static_cast<float *>(val) : c->d_v;
    const uint32_t n_ss = c->n_spans << c->segSh;
    const uint32_t eblock = 64u << c->segSh;
    const uint32_t fgrid = c->n_spans < SIDE_GRID ? c->n_spans : SIDE_GRID;

    if (weights) {
        /* Algorithm 2 Step 2: threshold and cut of |w| per bucket (bitmap for the buckets that
         * had to take the dense passes), on its own set of tables */
        Tables tw = t;
        tw.k = c->d_kw; tw.T = c->d_Tw; tw.need = c->d_needw; tw.fast = c->d_wfast;
        Cand cdw = cd0;
        const uint32_t n_chunks_w = (n_ss + 63) / 64;
        while (cdw.splitSh < 6u && ((uint64_t)n_chunks_w << cdw.splitSh) < 4ull * SIDE_GRID) ++cdw.splitSh;
        const uint64_t wwaves = (uint64_t)n_chunks_w << cdw.splitSh;
        const uint32_t cgw = c->force_dense ? 0u : (uint32_t)((wwaves + 3) / 4 < SIDE_GRID ? (wwaves + 3) / 4 : SIDE_GRID);
        LAUNCH(c, KID_CLEAR, st, k_clear, clear_grid < 2048 ? clear_grid : 2048, c->d_zero, zw);
        if (!c->force_dense)
            LAUNCH(c, KID_SAMPLE, st, k_sample<false>, c->n_samp, weights, (const float *)nullptr, tw, h.hs);
        LAUNCH(c, KID_WPLAN, st, k_wpredict, B, tw, (const uint32_t *)h.hs, c->d_wLo, c->d_wHi, c->force_dense,
               c->d_werr);
        LAUNCHB(c, KID_WHIST, st, k_whist, c->n_spans, eblock, weights, tw, h.h0, cdw,
                (const uint32_t *)c->d_wLo, (const uint32_t *)c->d_wHi);
        LAUNCH(c, KID_WPLAN, st, k_wplan, B, tw, (const uint32_t *)h.h0, (const uint32_t *)c->d_wLo,
               (const uint32_t *)c->d_wHi);
        LAUNCH(c, KID_FB_PLAN, st, k_fb_plan, 1, tw);
        if (cgw && (c->agg_override > 0 || (c->agg_override < 0 && n_chunks_w >= 8u * SIDE_GRID)))
            LAUNCH(c, KID_REFINE1, st, (k_refine<1, 64, true>), cgw + fgrid, weights, tw, cdw, h.c1, h.f1, cgw);
        else
            LAUNCH(c, KID_REFINE1, st, (k_refine<1, 64>), cgw + fgrid, weights, tw, cdw, h.c1, h.f1, cgw);
        LAUNCH(c, KID_PICK1, st, k_pick<1>, B, tw, (const uint32_t *)h.c1, (const uint32_t *)h.f1, c->d_werr, 0);
        LAUNCH(c, KID_REFINE2, st, (k_refine<2, 64>), cgw + fgrid, weights, tw, cdw, h.c2, h.f2, cgw);
        LAUNCH(c, KID_PICK2, st, k_pick<2>, B, tw, (const uint32_t *)h.c2, (const uint32_t *)h.f2, c->d_werr, 0, c->d_wT);
        LAUNCH(c, KID_COUNT, st, k_count<64>, cgw + fgrid, weights, tw, cdw, c->d_tG, c->d_tE, cgw);
        LAUNCH(c, KID_SCAN, st, k_scan, B, tw, cdw.G, cdw.E, c->d_tG, c->d_tE);
        LAUNCH(c, KID_WMASK, st, k_wfinish<64>, cgw + fgrid, weights, tw, cdw, (const uint32_t *)c->d_tG,
               (const uint32_t *)c->d_tE, c->d_wcut, c->d_pmask, cgw);
        t.w = weights;
        t.wT = c->d_wT;
        t.wcut = c->d_wcut;
        t.pmask = c->d_pmask;
    }

    /* where the candidate bounds L_b come from: the thresholds of the previous call when it had
     * the same layout, ratio and pruning (k_pick<2> left them in place), else a sample of
     * this gradient */
    const bool pruned = weights != nullptr;
    const bool from_history = c->use_history && !c->force_dense && c->hist_ready &&
                              c->hist_ratio == ratio && c->hist_pruned == pruned;
    const int write_next = (c->use_history && !c->force_dense) ? 1 : 0;
    c->hist_ready = false;
    LAUNCH(c, KID_CLEAR, st, k_clear, clear_grid < 2048 ? clear_grid : 2048, c->d_zero, zw);
    if (!from_history) {
        if (!c->force_dense)
            LAUNCH(c, KID_SAMPLE, st, k_sample<true>, c->n_samp, grad, (const float *)residual, t, h.hs);
        LAUNCH(c, KID_PREDICT, st, k_predict, B, t, (const uint32_t *)h.hs, c->force_dense);
    }
    if (c->force_dense) {
        if (weights) LAUNCHB(c, KID_EF_EMIT, st, (k_ef_emit<false, 7, true>), c->n_spans, eblock, grad, residual, t, h.h0, cd0, c->d_span_sq);
        else LAUNCHB(c, KID_EF_EMIT, st, (k_ef_emit<false, 7, false>), c->n_spans, eblock, grad, residual, t, h.h0, cd0, c->d_span_sq);
    } else if (weights) {
        LAUNCHB(c, KID_EF_EMIT, st, (k_ef_emit<true, 7, true>), c->n_spans, eblock, grad, residual, t, h.h0, cd0, c->d_span_sq);
    } else {
        switch (c->nt_mode) {
        case 1:  LAUNCHB(c, KID_EF_EMIT, st, (k_ef_emit<true, 1, false>), c->n_spans, eblock, grad, residual, t, h.h0, cd0, c->d_span_sq); break;
        case 3:  LAUNCHB(c, KID_EF_EMIT, st, (k_ef_emit<true, 3, false>), c->n_spans, eblock, grad, residual, t, h.h0, cd0, c->d_span_sq); break;
        case 5:  LAUNCHB(c, KID_EF_EMIT, st, (k_ef_emit<true, 5, false>), c->n_spans, eblock, grad, residual, t, h.h0, cd0, c->d_span_sq); break;
        default: LAUNCHB(c, KID_EF_EMIT, st, (k_ef_emit<true, 7, false>), c->n_spans, eblock, grad, residual, t, h.h0, cd0, c->d_span_sq); break;
        }
    }
    LAUNCH(c, KID_PLAN, st, k_plan, B, t, (const uint32_t *)h.h0, (const uint32_t *)cd0.cnt,
           c->force_dense ? 0 : 1, (const double *)c->d_span_sq, c->d_l2sq);
    LAUNCH(c, KID_FB_PLAN, st, k_fb_plan, 1, t);
    /* every stage serves both kinds of bucket: candidate segments first, then the dense
     * spans of the buckets the candidates could not decide */
    const float *acc = residual;
    /* lanes per candidate segment: a segment is expected to hold about 1.5 * ratio of the
     * elements it covers, and a group of lanes fetches 4 entries per lane at a time */
    const double per_seg = 1.5 * ratio * (double)((c->spanT * TILE) >> c->segSh);
    uint32_t group = per_seg < 7.0 ? 4u : per_seg < 48.0 ? 16u : 64u;
    if (c->group_override == 4 || c->group_override == 16 || c->group_override == 64) group = (uint32_t)c->group_override;
    /* wavefronts of the candidate role: one per chunk of 64 segments, or several per chunk
     * (each taking a share of its rounds) while that does not fill the grid */
    Cand cd = cd0;
    const uint32_t n_chunks = (n_ss + 63) / 64;
    const uint32_t max_split = group == 4 ? 2u : group == 16 ? 4u : 6u;   /* log2 of the rounds per chunk */
    cd.splitSh = 0;
    while (cd.splitSh < max_split && ((uint64_t)n_chunks << cd.splitSh) < 4ull * SIDE_GRID) ++cd.splitSh;
    const uint64_t cwaves = (uint64_t)n_chunks << cd.splitSh;
    const uint32_t cgrid = (uint32_t)((cwaves + 3) / 4 < SIDE_GRID ? (cwaves + 3) / 4 : SIDE_GRID);
    const uint32_t cg = c->force_dense ? 0u : cgrid;
#define NSML_BY_GROUP(kid, K, ...)                                                          \
    do {                                                                                    \
        if (group == 4) LAUNCH(c, kid, st, (K(4)), cg + fgrid, __VA_ARGS__);                \
        else if (group == 16) LAUNCH(c, kid, st, (K(16)), cg + fgrid, __VA_ARGS__);         \
        else LAUNCH(c, kid, st, (K(64)), cg + fgrid, __VA_ARGS__);                          \
    } while (0)
#define NSML_K_REFINE1(G) k_refine<1, G>
#define NSML_K_REFINE2(G) k_refine<2, G>
#define NSML_K_COUNT(G) k_count<G>
#define NSML_K_WRITE(G) k_write<G>
    if (cg && (c->agg_override > 0 || (c->agg_override < 0 && n_chunks >= 8u * AGG_GRID))) {
        /* many segments per workgroup: count the level-1 digits in LDS over a contiguous range
         * of chunks and add each bucket's histogram once (a third of the global atomics) */
        const uint32_t ag = AGG_GRID;
        if (group == 4) LAUNCH(c, KID_REFINE1, st, (k_refine<1, 4, true>), ag + fgrid, acc, t, cd, h.c1, h.f1, ag);
        else if (group == 16) LAUNCH(c, KID_REFINE1, st, (k_refine<1, 16, true>), ag + fgrid, acc, t, cd, h.c1, h.f1, ag);
        else LAUNCH(c, KID_REFINE1, st, (k_refine<1, 64, true>), ag + fgrid, acc, t, cd, h.c1, h.f1, ag);
    } else {
        NSML_BY_GROUP(KID_REFINE1, NSML_K_REFINE1, acc, t, cd, h.c1, h.f1, cg);
    }
    LAUNCH(c, KID_PICK1, st, k_pick<1>, B, t, (const uint32_t *)h.c1, (const uint32_t *)h.f1, h.err, 0);
    NSML_BY_GROUP(KID_REFINE2, NSML_K_REFINE2, acc, t, cd, h.c2, h.f2, cg);
    LAUNCH(c, KID_PICK2, st, k_pick<2>, B, t, (const uint32_t *)h.c2, (const uint32_t *)h.f2, h.err, write_next);
    NSML_BY_GROUP(KID_COUNT, NSML_K_COUNT, acc, t, cd, c->d_tG, c->d_tE, cg);
    LAUNCH(c, KID_SCAN, st, k_scan, B, t, cd.G, cd.E, c->d_tG, c->d_tE);
    NSML_BY_GROUP(KID_WRITE, NSML_K_WRITE, acc, t, cd, (const uint32_t *)c->d_tG, (const uint32_t *)c->d_tE,
                  idx, vdst, cg);
#undef NSML_BY_GROUP
#undef NSML_K_REFINE1
#undef NSML_K_REFINE2
#undef NSML_K_COUNT
#undef NSML_K_WRITE
    const uint32_t qgrid = (uint32_t)c->NC;
    switch (bits) {
    case 32: LAUNCH(c, KID_QUANT, st, k_quant<32>, qgrid, (const float *)vdst, (const uint32_t *)idx, t, residual, val, scales); break;
    case 16: LAUNCH(c, KID_QUANT, st, k_quant<16>, qgrid, (const float *)vdst, (const uint32_t *)idx, t, residual, val, scales); break;
    case 8:  LAUNCH(c, KID_QUANT, st, k_quant<8>,  qgrid, (const float *)vdst, (const uint32_t *)idx, t, residual, val, scales); break;
    default: LAUNCH(c, KID_QUANT, st, k_quant<4>,  qgrid, (const float *)vdst, (const uint32_t *)idx, t, residual, val, scales); break;
    }
    c->have_l2 = true;
    c->have_prune = pruned;
    c->hist_ready = write_next != 0;
    c->hist_ratio = ratio;
    c->hist_pruned = pruned;
    return NSML_OK;
}

int nsml_compress(nsml_ctx *c, const float *grad, float *residual, uint64_t n,
                  const uint64_t *bucket_off, uint32_t B, double ratio, int bits,
                  uint32_t *idx, void *val, float *scales, void *stream)
{
    return compress_impl(c, grad, residual, nullptr, n, bucket_off, B, ratio, bits, idx, val, scales, stream);
}

int nsml_compress_pruned(nsml_ctx *c, const float *grad, float *residual, const float *weights,
                         uint64_t n, const uint64_t *bucket_off, uint32_t B, double ratio, int bits,
                         uint32_t *idx, void *val, float *scales, void *stream)
{
    if (!weights) return NSML_EINVAL;
    return compress_impl(c, grad, residual, weights, n, bucket_off, B, ratio, bits, idx, val, scales, stream);
}

int nsml_decompress(nsml_ctx *c, const uint32_t *idx, const void *val, const float *scales,
                    uint64_t n, const uint64_t *bucket_off, uint32_t B, double ratio, int bits,
                    float *dense_out, void *stream)
{
    if (!c || !idx || !val || !dense_out) return NSML_EINVAL;
    if ((bits == 8 || bits == 4) && !scales) return NSML_EINVAL;
    if (!aligned(dense_out, 16) || !aligned(idx, 4) || !aligned(val, 4) || !aligned(scales, 4))
        return NSML_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    DeviceGuard guard(c->device);
    if (!guard.ok) { c->last_hip = (int)hipErrorInvalidDevice; return NSML_EHIP; }
    int rc = ensure_layout(c, n, bucket_off, B, st);
    if (rc) return rc;
    rc = ensure_tables(c, ratio, bits, st);
    if (rc) return rc;
    const Tables t = tables_of(c);
    if (c->K >= (4ull << 20)) {
        const uint64_t want = (c->K + (uint64_t)WG * 8 - 1) / ((uint64_t)WG * 8);
        LAUNCH(c, KID_TILESTART, st, k_tilestart<8>, (uint32_t)(want < 16384 ? want : 16384), idx, t, c->K, c->d_ts);
    } else {
        const uint64_t want = (c->K + (uint64_t)WG * 2 - 1) / ((uint64_t)WG * 2);
        LAUNCH(c, KID_TILESTART, st, k_tilestart<2>, (uint32_t)want, idx, t, c->K, c->d_ts);
    }
    const uint32_t *ts = c->d_ts;
    if (c->nt_dense) {
        switch (bits) {
        case 32: LAUNCH(c, KID_DECOMP, st, (k_decomp<32, true>), c->n_spans, idx, val, scales, t, ts, dense_out); break;
        case 16: LAUNCH(c, KID_DECOMP, st, (k_decomp<16, true>), c->n_spans, idx, val, scales, t, ts, dense_out); break;
        case 8:  LAUNCH(c, KID_DECOMP, st, (k_decomp<8, true>),  c->n_spans, idx, val, scales, t, ts, dense_out); break;
        default: LAUNCH(c, KID_DECOMP, st, (k_decomp<4, true>),  c->n_spans, idx, val, scales, t, ts, dense_out); break;
        }
    } else {
        switch (bits) {
        case 32: LAUNCH(c, KID_DECOMP, st, (k_decomp<32, false>), c->n_spans, idx, val, scales, t, ts, dense_out); break;
        case 16: LAUNCH(c, KID_DECOMP, st, (k_decomp<16, false>), c->n_spans, idx, val, scales, t, ts, dense_out); break;
        case 8:  LAUNCH(c, KID_DECOMP, st, (k_decomp<8, false>),  c->n_spans, idx, val, scales, t, ts, dense_out); break;
        default: LAUNCH(c, KID_DECOMP, st, (k_decomp<4, false>),  c->n_spans, idx, val, scales, t, ts, dense_out); break;
        }
    }
    return NSML_OK;
}

int nsml_decompress_accumulate(nsml_ctx *c, const uint32_t *idx, const void *val, const float *scales,
                               uint64_t n, const uint64_t *bucket_off, uint32_t B, double ratio,
                               int bits, float *dense_inout, void *stream)
{
    if (!c || !idx || !val || !dense_inout) return NSML_EINVAL;
    if ((bits == 8 || bits == 4) && !scales) return NSML_EINVAL;
    if (!aligned(dense_inout, 16) || !aligned(idx, 4) || !aligned(val, 4) || !aligned(scales, 4))
        return NSML_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    DeviceGuard guard(c->device);
    if (!guard.ok) { c->last_hip = (int)hipErrorInvalidDevice; return NSML_EHIP; }
    int rc = ensure_layout(c, n, bucket_off, B, st);
    if (rc) return rc;
    rc = ensure_tables(c, ratio, bits, st);
    if (rc) return rc;
    const Tables t = tables_of(c);
    const uint64_t want = (c->K + WG - 1) / WG;
    const uint32_t grid = (uint32_t)(want < 32768 ? want : 32768);
    switch (bits) {
    case 32: LAUNCH(c, KID_DECOMP_ACC, st, k_decomp_acc<32>, grid, idx, val, scales, t, c->K, dense_inout); break;
    case 16: LAUNCH(c, KID_DECOMP_ACC, st, k_decomp_acc<16>, grid, idx, val, scales, t, c->K, dense_inout); break;
    case 8:  LAUNCH(c, KID_DECOMP_ACC, st, k_decomp_acc<8>,  grid, idx, val, scales, t, c->K, dense_inout); break;
    default: LAUNCH(c, KID_DECOMP_ACC, st, k_decomp_acc<4>,  grid, idx, val, scales, t, c->K, dense_inout); break;
    }
    return NSML_OK;
}

int nsml_last_l2norm(nsml_ctx *c, double *total, double *per_bucket)
{
    if (!c || !total) return NSML_EINVAL;
    *total = 0.0;
    if (!c->have_l2 || c->B == 0) return NSML_EINVAL;
    DeviceGuard guard(c->device);
    NSML_HIP(c, hipDeviceSynchronize());
    std::vector<double> sq(c->B);
    NSML_HIP(c, hipMemcpy(sq.data(), c->d_l2sq, sizeof(double) * c->B, hipMemcpyDeviceToHost));
    double sum = 0.0;
    for (uint32_t b = 0; b < c->B; ++b) {
        const double v = c->h_off[b + 1] > c->h_off[b] ? sq[b] : 0.0;
        sum += v;
        if (per_bucket) per_bucket[b] = sqrt(v);
    }
    *total = sqrt(sum);
    return NSML_OK;
}

int nsml_profile_enable(nsml_ctx *c, int on)
{
    if (!c) return NSML_EINVAL;
    c->prof = on != 0;
    return NSML_OK;
}

int nsml_profile_read(nsml_ctx *c, uint32_t *launches, double *total_ms)
{
    if (!c || !launches || !total_ms) return NSML_EINVAL;
    DeviceGuard guard(c->device);
    for (int i = 0; i < NSML_MAX_KERNELS; ++i) { launches[i] = 0; total_ms[i] = 0.0; }
    int rc = NSML_OK;
    for (auto &r : c->recs) {
        float ms = 0.f;
        hipError_t e = hipEventSynchronize(r.b);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, r.a, r.b);
        if (e != hipSuccess) { c->last_hip = (int)e; rc = NSML_EHIP; }
        else { launches[r.kid] += 1; total_ms[r.kid] += (double)ms; }
        c->pool.push_back(r.a); c->pool.push_back(r.b);
    }
    c->recs.clear();
    return rc;
}

int nsml_path_stats(nsml_ctx *c, uint32_t *fast_buckets, uint32_t *fallback_buckets)
{
    if (!c || !fast_buckets || !fallback_buckets) return NSML_EINVAL;
    *fast_buckets = *fallback_buckets = 0;
    if (c->B == 0) return NSML_OK;
    DeviceGuard guard(c->device);
    NSML_HIP(c, hipDeviceSynchronize());
    std::vector<uint32_t> f(c->B);
    NSML_HIP(c, hipMemcpy(f.data(), c->d_fast, sizeof(uint32_t) * c->B, hipMemcpyDeviceToHost));
    for (uint32_t b = 0; b < c->B; ++b) {
        if (c->h_off[b + 1] == c->h_off[b]) continue;
        if (f[b]) *fast_buckets += 1; else *fallback_buckets += 1;
    }
    uint32_t err = 0;
    NSML_HIP(c, hipMemcpy(&err, hists_of(c, c->B).err, sizeof(uint32_t), hipMemcpyDeviceToHost));
    return err ? NSML_EINTERNAL : NSML_OK;
}

int nsml_prune_stats(nsml_ctx *c, uint32_t *band_buckets, uint32_t *dense_buckets)
{
    if (!c || !band_buckets || !dense_buckets) return NSML_EINVAL;
    *band_buckets = *dense_buckets = 0;
    if (c->B == 0 || !c->have_prune) return NSML_OK;
    DeviceGuard guard(c->device);
    NSML_HIP(c, hipDeviceSynchronize());
    std::vector<uint32_t> f(c->B);
    NSML_HIP(c, hipMemcpy(f.data(), c->d_wfast, sizeof(uint32_t) * c->B, hipMemcpyDeviceToHost));
    for (uint32_t b = 0; b < c->B; ++b) {
        if (c->h_off[b + 1] == c->h_off[b]) continue;
        if (f[b]) *band_buckets += 1; else *dense_buckets += 1;
    }
    uint32_t err = 0;
    NSML_HIP(c, hipMemcpy(&err, c->d_werr, sizeof(uint32_t), hipMemcpyDeviceToHost));
    return err ? NSML_EINTERNAL : NSML_OK;
}

int nsml_calibration_copy(const void *src, void *dst, uint64_t bytes, void *stream)
{
    if (!src || !dst || bytes == 0 || bytes % 16 != 0 || !aligned(src, 16) || !aligned(dst, 16))
        return NSML_EINVAL;
    const uint64_t n16 = bytes / 16;
    const uint64_t want = (n16 + WG - 1) / WG;
    const uint32_t grid = (uint32_t)(want < 65536 ? want : 65536);
    hipLaunchKernelGGL(k_calib_copy, dim3(grid), dim3(WG), 0, static_cast<hipStream_t>(stream),
                       static_cast<const f4 *>(src), static_cast<f4 *>(dst), n16);
    return hipGetLastError() == hipSuccess ? NSML_OK : NSML_EHIP;
}

const char *nsml_kernel_name(int id) { return (id >= 0 && id < KID_N) ? kKernelNames[id] : nullptr; }

}  // extern "C"
