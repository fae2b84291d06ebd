/*
 * libnsml GPU path for gfx950 (MI355X): hand-written HIP kernels and their C-ABI entry points.
 *
 * One compress call = error-feedback accumulation, exact top-k by magnitude per bucket
 * (Sec. 4.2 Step 3 / Algorithm 2 Step 3), value coding and payload packing; one decompress
 * call = payload -> dense gradient.  Nothing here is a dense contraction: every kernel is a
 * streaming pass bound by HBM bandwidth, so the work is organised around coalesced 16-byte
 * accesses, LDS histograms and 64-lane ballots, not MFMA.
 *
 * Selection is a three-level radix select on the 31-bit magnitude key
 * (binary32 pattern with the sign cleared):  12 + 12 + 7 bits.
 *   ef_hist   acc = grad + residual (written over residual) + level-0 histogram   12 B/elem
 *   pick0     per bucket: level-0 bin that holds the k-th largest key
 *   refine1/2 histogram of the next digit over elements inside the chosen bin      4 B/elem each
 *   pick1/2   -> exact threshold key T_b and the number e_b of elements equal to T_b to admit
 *   count     per 4096-element tile: #(key > T), #(key == T)                       4 B/elem
 *   scan      per bucket exclusive scan of the tile counts
 *   write     survivors to their final, index-ordered slots (idx, value)           4 B/elem
 *   quant     per chunk of survivors: absmax scale, codes, packing, residual update
 *   decomp    payload -> dense, each output line written once, tile staged in LDS  4 B/elem
 *
 * Geometry: a bucket [lo, hi) is cut into tiles of 4096 elements starting at lo rounded down
 * to a multiple of 4, so every 16-byte access is aligned; elements of an edge tile outside
 * [lo, hi) are masked.  A workgroup (256 threads = 4 wavefronts) owns a span of consecutive
 * tiles of one bucket.  Inside a tile, thread t owns the four quads (u*256 + t)*4, u = 0..3,
 * which makes every load instruction of a wavefront one contiguous 1 KiB run.
 */
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#include <new>
#include <vector>

#include "nsml.h"

namespace {

constexpr int WG = 256;
constexpr int TILE = 4096;
constexpr int NB0 = 4096, NB1 = 4096, NB2 = 128;
constexpr int SH0 = 19;   /* key >> 19         : level-0 digit (sign-less exponent + 4 mantissa bits) */
constexpr int SH1 = 7;    /* (key >> 7) & 4095 : level-1 digit;  key & 127 : level-2 digit */
constexpr int MAX_SPAN_TILES = 16;

enum KernelId {
    KID_SETUP = 0, KID_CLEAR, KID_EF_HIST, KID_PICK0, KID_REFINE1, KID_PICK1, KID_REFINE2,
    KID_PICK2, KID_COUNT, KID_SCAN, KID_WRITE, KID_QUANT, KID_DECOMP, KID_N
};
const char *const kKernelNames[KID_N] = {
    "setup", "clear", "ef_hist", "pick0", "refine1", "pick1", "refine2",
    "pick2", "count", "scan", "write", "quant", "decomp"
};
static_assert(KID_N <= NSML_MAX_KERNELS, "raise NSML_MAX_KERNELS");

/* Device-resident tables of one (bucket layout, ratio, bits) combination. */
struct Tables {
    const uint64_t *off;    /* B+1 bucket offsets */
    const uint32_t *tile0;  /* B+1 prefix of tile counts */
    const uint32_t *span0;  /* B+1 prefix of span counts */
    uint32_t *k;            /* B   survivors per bucket */
    uint64_t *P;            /* B+1 prefix of k */
    uint64_t *V;            /* B+1 prefix of value bytes */
    uint64_t *S;            /* B+1 prefix of scale counts */
    uint64_t *C;            /* B+1 prefix of chunk counts (all widths) */
    uint32_t *T;            /* B   threshold key, refined level by level */
    uint32_t *need;         /* B   how many more to take at the current level */
    uint32_t B;
    uint32_t spanT;         /* tiles per span */
    uint32_t chunk;
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

__device__ __forceinline__ SpanGeo span_geo(const Tables &t, uint32_t s)
{
    SpanGeo g;
    g.b = find_bucket<uint32_t>(t.span0, t.B, s);
    const uint32_t si = s - t.span0[g.b];
    g.lo = t.off[g.b];
    g.hi = t.off[g.b + 1];
    const uint32_t tiles_b = t.tile0[g.b + 1] - t.tile0[g.b];
    const uint32_t first = si * t.spanT;
    g.ntiles = min(t.spanT, tiles_b - first);
    g.tile_g = t.tile0[g.b] + first;
    g.base = (g.lo & ~3ull) + (uint64_t)first * TILE;
    return g;
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
        t.P[b] = pk; t.V[b] = pv; t.S[b] = ps; t.C[b] = pc;
        pk += k;
        pv += bits == 32 ? 4 * k : bits == 16 ? 2 * k : bits == 8 ? k : (k + 1) / 2;
        ps += bits <= 8 ? ch : 0;
        pc += ch;
        if (b == t.B - 1) { t.P[t.B] = pk; t.V[t.B] = pv; t.S[t.B] = ps; t.C[t.B] = pc; }
    }
}

__global__ __launch_bounds__(WG) void k_clear(uint32_t *__restrict__ p, uint64_t n)
{
    const uint64_t stride = (uint64_t)gridDim.x * WG;
    for (uint64_t i = (uint64_t)blockIdx.x * WG + threadIdx.x; i < n; i += stride) p[i] = 0u;
}

/* ------------------------------------------------------------------ histograms */

/* Add the four level digits of a quad to an LDS histogram.  When every lane of the wavefront
 * carries the same digit in all four slots (runs of zeros, saturated buckets) one lane adds
 * the whole count: same-address LDS atomics of a wavefront serialise. */
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

__device__ __forceinline__ void hist_flush(const uint32_t *h, uint32_t *__restrict__ dst, int nb)
{
    for (int i = threadIdx.x; i < nb; i += WG) {
        const uint32_t c = h[i];
        if (c) atomicAdd(&dst[i], c);
    }
}

/* acc = grad + residual over a span, written over residual, plus the level-0 histogram.
 * (Sec. 4.2 Step 3: what top-k filters out is accumulated locally; the add is that.) */
__global__ __launch_bounds__(WG) void k_ef_hist(const float *__restrict__ g, float *__restrict__ r,
                                                Tables t, uint32_t *__restrict__ hist0)
{
    __shared__ uint32_t h[NB0];
    const uint32_t tid = threadIdx.x;
    for (int i = tid; i < NB0; i += WG) h[i] = 0;
    const SpanGeo s = span_geo(t, blockIdx.x);
    __syncthreads();
    for (uint32_t ti = 0; ti < s.ntiles; ++ti) {
        const uint64_t tb = s.base + (uint64_t)ti * TILE;
        if (tb >= s.lo && tb + TILE <= s.hi) {
            f4 gv[4], rv[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint64_t gi = tb + (uint64_t)(u * WG + tid) * 4;
                gv[u] = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(g + gi));
                rv[u] = *reinterpret_cast<const f4 *>(r + gi);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint64_t gi = tb + (uint64_t)(u * WG + tid) * 4;
                f4 a;
                a.x = __fadd_rn(gv[u].x, rv[u].x); a.y = __fadd_rn(gv[u].y, rv[u].y);
                a.z = __fadd_rn(gv[u].z, rv[u].z); a.w = __fadd_rn(gv[u].w, rv[u].w);
                *reinterpret_cast<f4 *>(r + gi) = a;
                hist_quad_full(h, keyof(a.x) >> SH0, keyof(a.y) >> SH0, keyof(a.z) >> SH0,
                               keyof(a.w) >> SH0);
            }
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint64_t gi = tb + (uint64_t)(u * WG + tid) * 4;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint64_t i = gi + j;
                    if (i >= s.lo && i < s.hi) {
                        const float a = __fadd_rn(g[i], r[i]);
                        r[i] = a;
                        atomicAdd(&h[keyof(a) >> SH0], 1u);
                    }
                }
            }
        }
    }
    __syncthreads();
    hist_flush(h, hist0 + (uint64_t)s.b * NB0, NB0);
}

/* Histogram of the next digit over the elements whose higher digits equal the prefix found
 * so far (LEVEL 1: 12-bit prefix in T, digit = bits 18..7; LEVEL 2: 24-bit prefix, bits 6..0). */
template <int LEVEL>
__global__ __launch_bounds__(WG) void k_refine(const float *__restrict__ r, Tables t,
                                               uint32_t *__restrict__ hist)
{
    constexpr int NB = LEVEL == 1 ? NB1 : NB2;
    constexpr int PSH = LEVEL == 1 ? SH0 : SH1;          /* key >> PSH is the prefix */
    constexpr int DSH = LEVEL == 1 ? SH1 : 0;
    constexpr uint32_t DMASK = NB - 1;
    __shared__ uint32_t h[NB];
    const uint32_t tid = threadIdx.x;
    for (int i = tid; i < NB; i += WG) h[i] = 0;
    const SpanGeo s = span_geo(t, blockIdx.x);
    const uint32_t prefix = t.T[s.b];
    __syncthreads();
    for (uint32_t ti = 0; ti < s.ntiles; ++ti) {
        const uint64_t tb = s.base + (uint64_t)ti * TILE;
        const bool interior = tb >= s.lo && tb + TILE <= s.hi;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint64_t gi = tb + (uint64_t)(u * WG + tid) * 4;
            float x[4];
            const uint32_t m = load_quad(r, gi, s.lo, s.hi, x);
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
    hist_flush(h, hist + (uint64_t)s.b * NB, NB);
}

/* Inclusive scan over the 256 threads of a workgroup (tmp: 256 words of LDS). */
__device__ __forceinline__ uint32_t block_incl_scan(uint32_t x, uint32_t *tmp)
{
    const uint32_t tid = threadIdx.x;
    tmp[tid] = x;
    __syncthreads();
#pragma unroll
    for (int d = 1; d < WG; d <<= 1) {
        const uint32_t y = tid >= (uint32_t)d ? tmp[tid - d] : 0u;
        __syncthreads();
        x += y;
        tmp[tid] = x;
        __syncthreads();
    }
    return x;
}

/* Per bucket: walk one level's histogram from the top digit down to the digit that holds the
 * want-th largest key; append it to the prefix; what is still wanted inside it goes to need. */
template <int LEVEL>
__global__ __launch_bounds__(WG) void k_pick(Tables t, const uint32_t *__restrict__ hist)
{
    constexpr int NB = LEVEL == 2 ? NB2 : NB0;
    constexpr int PER = NB >= WG ? NB / WG : 1;
    constexpr int BITS = LEVEL == 2 ? 7 : 12;
    __shared__ uint32_t tmp[WG];
    const uint32_t b = blockIdx.x, tid = threadIdx.x;
    const uint32_t want = LEVEL == 0 ? t.k[b] : t.need[b];
    if (want == 0) {                       /* empty bucket: nothing can match */
        if (tid == 0) { t.T[b] = 0xFFFFFFFFu; t.need[b] = 0; }
        return;
    }
    const uint32_t *hb = hist + (uint64_t)b * NB;
    /* thread 0 owns the highest digits */
    const int top = NB - 1 - (int)tid * PER;
    uint32_t c[PER];
    uint32_t sum = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int d = top - i;
        c[i] = d >= 0 ? hb[d] : 0u;
        sum += c[i];
    }
    const uint32_t incl = block_incl_scan(sum, tmp);
    const uint32_t above = incl - sum;
    if (above < want && want <= incl) {
        uint32_t acc = above;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            if (acc + c[i] >= want) {
                const uint32_t d = (uint32_t)(top - i);
                t.T[b] = LEVEL == 0 ? d : ((t.T[b] << BITS) | d);
                t.need[b] = want - acc;
                break;
            }
            acc += c[i];
        }
    }
}

/* ------------------------------------------------------------------ compaction */

/* Per tile: how many keys exceed the threshold, how many equal it. */
__global__ __launch_bounds__(WG) void k_count(const float *__restrict__ r, Tables t,
                                              uint32_t *__restrict__ tG, uint32_t *__restrict__ tE)
{
    __shared__ uint32_t cnt[MAX_SPAN_TILES][2];
    const uint32_t tid = threadIdx.x;
    if (tid < MAX_SPAN_TILES * 2) (&cnt[0][0])[tid] = 0;
    const SpanGeo s = span_geo(t, blockIdx.x);
    const uint32_t T = t.T[s.b];
    __syncthreads();
    for (uint32_t ti = 0; ti < s.ntiles; ++ti) {
        const uint64_t tb = s.base + (uint64_t)ti * TILE;
        uint32_t ng = 0, ne = 0;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint64_t gi = tb + (uint64_t)(u * WG + tid) * 4;
            float x[4];
            const uint32_t m = load_quad(r, gi, s.lo, s.hi, x);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t key = keyof(x[j]);
                const bool ok = (m >> j) & 1u;
                ng += (ok && key > T) ? 1u : 0u;
                ne += (ok && key == T) ? 1u : 0u;
            }
        }
        /* wavefront sum by shuffles, then one LDS atomic per wavefront */
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            ng += __shfl_xor(ng, d, 64);
            ne += __shfl_xor(ne, d, 64);
        }
        if ((tid & 63) == 0) { atomicAdd(&cnt[ti][0], ng); atomicAdd(&cnt[ti][1], ne); }
    }
    __syncthreads();
    if (tid < s.ntiles) { tG[s.tile_g + tid] = cnt[tid][0]; tE[s.tile_g + tid] = cnt[tid][1]; }
}

/* Per bucket: exclusive scan, in place, of the per-tile counts. */
__global__ __launch_bounds__(WG) void k_scan(Tables t, uint32_t *__restrict__ tG,
                                             uint32_t *__restrict__ tE)
{
    __shared__ uint32_t tmp[WG];
    const uint32_t b = blockIdx.x, tid = threadIdx.x;
    const uint32_t t0 = t.tile0[b], t1 = t.tile0[b + 1];
    uint32_t carry_g = 0, carry_e = 0;
    for (uint32_t base = t0; base < t1; base += WG) {
        const uint32_t i = base + tid;
        const uint32_t g = i < t1 ? tG[i] : 0u, e = i < t1 ? tE[i] : 0u;
        const uint32_t ig = block_incl_scan(g, tmp);
        const uint32_t tot_g = tmp[WG - 1];
        __syncthreads();
        const uint32_t ie = block_incl_scan(e, tmp);
        const uint32_t tot_e = tmp[WG - 1];
        __syncthreads();
        if (i < t1) { tG[i] = carry_g + ig - g; tE[i] = carry_e + ie - e; }
        carry_g += tot_g;
        carry_e += tot_e;
    }
}

/* Per tile: write the survivors (key > T, or key == T and among the first e_b equal ones of
 * the bucket in index order) to their final slots, in ascending index order. */
__global__ __launch_bounds__(WG) void k_write(const float *__restrict__ r, Tables t,
                                              const uint32_t *__restrict__ tG,
                                              const uint32_t *__restrict__ tE,
                                              uint32_t *__restrict__ idx_out,
                                              float *__restrict__ v_out)
{
    __shared__ uint32_t tot[16][2];      /* slot = u * 4 + wavefront */
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint64_t lt = (1ull << lane) - 1ull;
    const SpanGeo s = span_geo(t, blockIdx.x);
    const uint32_t T = t.T[s.b], e_b = t.need[s.b];
    const uint64_t Pb = t.P[s.b];
    for (uint32_t ti = 0; ti < s.ntiles; ++ti) {
        const uint64_t tb = s.base + (uint64_t)ti * TILE;
        const uint32_t gpre = tG[s.tile_g + ti], epre = tE[s.tile_g + ti];
        float x[4][4];
        uint32_t fg[4], fe[4], gb[4], eb[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint64_t gi = tb + (uint64_t)(u * WG + tid) * 4;
            const uint32_t m = load_quad(r, gi, s.lo, s.hi, x[u]);
            fg[u] = fe[u] = 0;
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
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bool isg = (fg[u] >> j) & 1u, ise = (fe[u] >> j) & 1u;
                if (isg || (ise && pe < e_b)) {
                    const uint64_t pos = Pb + pg + min(e_b, pe);
                    idx_out[pos] = (uint32_t)(gi + j - s.lo);
                    v_out[pos] = x[u][j];
                }
                pg += isg ? 1u : 0u;
                pe += ise ? 1u : 0u;
            }
        }
        __syncthreads();
    }
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

/* Dense output for a span of tiles: each tile is assembled in LDS (zeros, then the decoded
 * survivors that fall inside it) and written out once with aligned 16-byte stores, so no
 * output line is touched twice and no atomics are needed.  The survivors of a span are a
 * contiguous run of the bucket's ascending index list: its start is found by a 256-ary
 * search, after that a running cursor follows the tiles. */
template <int BITS>
__global__ __launch_bounds__(WG) void k_decomp(const uint32_t *__restrict__ idx, const void *__restrict__ val,
                                               const float *__restrict__ scales, Tables t,
                                               float *__restrict__ dense)
{
    __shared__ float tile[TILE];
    const uint32_t tid = threadIdx.x;
    const SpanGeo s = span_geo(t, blockIdx.x);
    const uint32_t kb = t.k[s.b];
    const uint32_t *ib = idx + t.P[s.b];
    const uint8_t *vb = reinterpret_cast<const uint8_t *>(val) + t.V[s.b];
    const float *sb = BITS <= 8 ? scales + t.S[s.b] : nullptr;

    /* first survivor whose local index is >= the first local index of the span */
    const uint64_t first_g = s.base > s.lo ? s.base : s.lo;
    const uint32_t L0 = (uint32_t)(first_g - s.lo);
    uint32_t a = 0, bnd = kb;                      /* answer in [a, bnd] */
    while (bnd - a > WG) {
        const uint32_t step = (bnd - a + WG - 1) / WG;
        const uint64_t p = (uint64_t)a + (uint64_t)tid * step;
        const int below = (p < bnd) && (ib[p] < L0);
        const uint32_t c = __syncthreads_count(below);   /* flags are a prefix: idx ascending */
        const uint64_t na = c ? (uint64_t)a + (uint64_t)(c - 1) * step + 1 : a;
        const uint64_t nb = min((uint64_t)bnd, (uint64_t)a + (uint64_t)c * step);
        a = (uint32_t)na; bnd = (uint32_t)nb;
    }
    {
        const uint32_t p = a + tid;
        const int below = (p < bnd) && (ib[p] < L0);
        a += __syncthreads_count(below);
    }
    uint32_t cur = a;

    for (uint32_t ti = 0; ti < s.ntiles; ++ti) {
        const uint64_t tb = s.base + (uint64_t)ti * TILE;
        /* local index one past the tile's last valid element */
        const uint64_t tend_g = tb + TILE < s.hi ? tb + TILE : s.hi;
        const uint32_t L1 = (uint32_t)(tend_g - s.lo);      /* may be 2^32 - 0? no: n_b < 2^32 */
        const uint64_t shift = s.lo - tb;                   /* slot = local index + lo - tb (mod 2^64) */
#pragma unroll
        for (int u = 0; u < 4; ++u)
            *reinterpret_cast<f4 *>(&tile[(u * WG + tid) * 4]) = f4{0.f, 0.f, 0.f, 0.f};
        __syncthreads();
        for (;;) {
            const uint64_t j = (uint64_t)cur + tid;
            int in = 0;
            if (j < kb) {
                const uint32_t li = ib[j];
                if (li < L1) {
                    const uint64_t slot = (uint64_t)li + shift;
                    if (slot < TILE) { tile[slot] = decode<BITS>(vb, sb, j, t.chunk); }
                    in = 1;
                }
            }
            const uint32_t c = __syncthreads_count(in);
            cur += c;
            if (c < WG) break;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t sl = (u * WG + tid) * 4;
            const uint64_t gi = tb + sl;
            if (gi >= s.lo && gi + 4 <= s.hi) {
                *reinterpret_cast<f4 *>(dense + gi) = *reinterpret_cast<const f4 *>(&tile[sl]);
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (gi + j >= s.lo && gi + j < s.hi) dense[gi + j] = tile[sl + j];
            }
        }
        __syncthreads();
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

    /* device workspace */
    uint64_t *d_off, *d_P, *d_V, *d_S, *d_C;
    uint32_t *d_tile0, *d_span0, *d_k, *d_T, *d_need;
    uint32_t *d_hist;      /* B * (NB0 + NB1 + NB2) */
    uint32_t *d_tG, *d_tE; /* per tile */
    float *d_v;            /* survivor values in final order (not used for bits == 32) */

    /* host copies / caches */
    std::vector<uint64_t> h_off;
    uint32_t B;
    uint64_t n;
    uint32_t n_tiles, n_spans, spanT;
    bool tables_valid;
    double t_ratio; int t_bits;       /* what d_k/d_P/... were computed for */
    uint64_t K, NC;                   /* totals for (layout, t_ratio, t_bits) */
    void *pinned; size_t pinned_bytes;
    int span_override;

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

Tables tables_of(const nsml_ctx *c)
{
    Tables t;
    t.off = c->d_off; t.tile0 = c->d_tile0; t.span0 = c->d_span0;
    t.k = c->d_k; t.P = c->d_P; t.V = c->d_V; t.S = c->d_S; t.C = c->d_C;
    t.T = c->d_T; t.need = c->d_need;
    t.B = c->B; t.spanT = c->spanT; t.chunk = c->chunk;
    return t;
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

#define LAUNCH(ctx, kid, st, kernel, grid, ...)                                     \
    do {                                                                            \
        int rc_ = prof_begin(ctx, kid, st);                                         \
        if (rc_) return rc_;                                                        \
        hipLaunchKernelGGL(kernel, dim3(grid), dim3(WG), 0, st, __VA_ARGS__);       \
        NSML_HIP(ctx, hipGetLastError());                                           \
        rc_ = prof_end(ctx, kid, st);                                               \
        if (rc_) return rc_;                                                        \
    } while (0)

bool aligned(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

uint32_t pick_span_tiles(uint32_t n_tiles, int override_)
{
    if (override_ >= 1 && override_ <= MAX_SPAN_TILES) return (uint32_t)override_;
    if (n_tiles >= 16u * 4096u) return 16;
    if (n_tiles >= 8u * 2048u) return 8;
    if (n_tiles >= 4u * 1024u) return 4;
    if (n_tiles >= 2u * 512u) return 2;
    return 1;
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
    std::vector<uint32_t> tile0((size_t)B + 1), span0((size_t)B + 1);
    uint64_t nt = 0;
    for (uint32_t b = 0; b < B; ++b) {
        tile0[b] = (uint32_t)nt;
        const uint64_t lo = off[b], hi = off[b + 1];
        if (hi > lo) nt += (hi - (lo & ~3ull) + TILE - 1) / TILE;
        if (nt > c->max_tiles) return NSML_ECAP;
    }
    tile0[B] = (uint32_t)nt;
    const uint32_t spanT = pick_span_tiles((uint32_t)nt, c->span_override);
    uint64_t ns = 0;
    for (uint32_t b = 0; b < B; ++b) {
        span0[b] = (uint32_t)ns;
        ns += (tile0[b + 1] - tile0[b] + spanT - 1) / spanT;
    }
    span0[B] = (uint32_t)ns;

    /* the stream may still be using the old tables */
    NSML_HIP(c, hipStreamSynchronize(st));
    c->tables_valid = false;
    c->B = 0;
    const size_t need = sizeof(uint64_t) * ((size_t)B + 1) + 2 * sizeof(uint32_t) * ((size_t)B + 1);
    if (need > c->pinned_bytes) return NSML_ECAP;
    uint8_t *hp = static_cast<uint8_t *>(c->pinned);
    memcpy(hp, off, sizeof(uint64_t) * ((size_t)B + 1));
    uint8_t *hp_t = hp + sizeof(uint64_t) * ((size_t)B + 1);
    memcpy(hp_t, tile0.data(), sizeof(uint32_t) * ((size_t)B + 1));
    uint8_t *hp_s = hp_t + sizeof(uint32_t) * ((size_t)B + 1);
    memcpy(hp_s, span0.data(), sizeof(uint32_t) * ((size_t)B + 1));
    NSML_HIP(c, hipMemcpyAsync(c->d_off, hp, sizeof(uint64_t) * ((size_t)B + 1), hipMemcpyHostToDevice, st));
    NSML_HIP(c, hipMemcpyAsync(c->d_tile0, hp_t, sizeof(uint32_t) * ((size_t)B + 1), hipMemcpyHostToDevice, st));
    NSML_HIP(c, hipMemcpyAsync(c->d_span0, hp_s, sizeof(uint32_t) * ((size_t)B + 1), hipMemcpyHostToDevice, st));
    NSML_HIP(c, hipStreamSynchronize(st));

    c->h_off.assign(off, off + B + 1);
    c->B = B; c->n = n;
    c->n_tiles = (uint32_t)nt; c->n_spans = (uint32_t)ns; c->spanT = spanT;
    return NSML_OK;
}

/* Make d_k / d_P / d_V / d_S / d_C match (ratio, bits) for the cached layout. */
int ensure_tables(nsml_ctx *c, double ratio, int bits, hipStream_t st)
{
    if (!(ratio > 0.0 && ratio <= 1.0)) return NSML_EINVAL;
    if (bits != 4 && bits != 8 && bits != 16 && bits != 32) return NSML_EINVAL;
    if (c->tables_valid && c->t_ratio == ratio && c->t_bits == bits) return NSML_OK;
    uint64_t K = 0;
    int rc = nsml_payload_layout(c->h_off.data(), c->B, ratio, bits, c->chunk, nullptr, &K, nullptr, nullptr);
    if (rc) return rc;
    /* chunk count over all buckets (for every width) */
    uint64_t nc = 0;
    {
        std::vector<uint64_t> kb(c->B);
        rc = nsml_payload_layout(c->h_off.data(), c->B, ratio, bits, c->chunk, kb.data(), nullptr, nullptr, nullptr);
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
    c->d_tile0 = c->d_span0 = c->d_k = c->d_T = c->d_need = c->d_hist = c->d_tG = c->d_tE = nullptr;
    c->d_v = nullptr;
    const char *so = getenv("NSML_SPAN_TILES");
    c->span_override = so ? atoi(so) : 0;

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
    if (mt >= 0xFFFFFFFFull) { delete c; return NSML_ECAP; }
    c->max_tiles = (uint32_t)mt;
    const uint64_t B1 = (uint64_t)max_buckets + 1;
    int rc = NSML_OK;
    auto A = [&](int r) { if (rc == NSML_OK) rc = r; };
    A(dev_alloc(c, &c->d_off, B1)); A(dev_alloc(c, &c->d_P, B1)); A(dev_alloc(c, &c->d_V, B1));
    A(dev_alloc(c, &c->d_S, B1)); A(dev_alloc(c, &c->d_C, B1));
    A(dev_alloc(c, &c->d_tile0, B1)); A(dev_alloc(c, &c->d_span0, B1));
    A(dev_alloc(c, &c->d_k, B1)); A(dev_alloc(c, &c->d_T, B1)); A(dev_alloc(c, &c->d_need, B1));
    A(dev_alloc(c, &c->d_hist, (uint64_t)max_buckets * (NB0 + NB1 + NB2)));
    A(dev_alloc(c, &c->d_tG, mt)); A(dev_alloc(c, &c->d_tE, mt));
    A(dev_alloc(c, &c->d_v, max_n));
    if (rc == NSML_OK) {
        c->pinned_bytes = B1 * 16;
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
    void *ptrs[] = {c->d_off, c->d_P, c->d_V, c->d_S, c->d_C, c->d_tile0, c->d_span0, c->d_k,
                    c->d_T, c->d_need, c->d_hist, c->d_tG, c->d_tE, c->d_v};
    for (void *p : ptrs) if (p) (void)hipFree(p);
    if (c->pinned) (void)hipHostFree(c->pinned);
    for (auto &r : c->recs) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    for (auto e : c->pool) (void)hipEventDestroy(e);
    delete c;
    return NSML_OK;
}

int nsml_last_hip_error(const nsml_ctx *c) { return c ? c->last_hip : 0; }
uint64_t nsml_workspace_bytes(const nsml_ctx *c) { return c ? c->ws_bytes : 0; }

int nsml_compress(nsml_ctx *c, const float *grad, float *residual, uint64_t n,
                  const uint64_t *bucket_off, uint32_t B, double ratio, int bits,
                  uint32_t *idx, void *val, float *scales, void *stream)
{
    if (!c || !grad || !residual || !idx || !val) return NSML_EINVAL;
    if ((bits == 8 || bits == 4) && !scales) return NSML_EINVAL;
    if (!aligned(grad, 16) || !aligned(residual, 16) || !aligned(idx, 4) || !aligned(val, 4) ||
        !aligned(scales, 4))
        return NSML_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    DeviceGuard guard(c->device);
    if (!guard.ok) { c->last_hip = (int)hipErrorInvalidDevice; return NSML_EHIP; }
    int rc = ensure_layout(c, n, bucket_off, B, st);
    if (rc) return rc;
    rc = ensure_tables(c, ratio, bits, st);
    if (rc) return rc;

    const Tables t = tables_of(c);
    uint32_t *h0 = c->d_hist;
    uint32_t *h1 = h0 + (uint64_t)B * NB0;
    uint32_t *h2 = h1 + (uint64_t)B * NB1;
    const uint64_t hist_words = (uint64_t)B * (NB0 + NB1 + NB2);
    const uint32_t clear_grid = (uint32_t)((hist_words + WG * 8 - 1) / (WG * 8));
    float *vdst = bits == 32 ? static_cast<float *>(val) : c->d_v;

    LAUNCH(c, KID_CLEAR, st, k_clear, clear_grid < 2048 ? clear_grid : 2048, c->d_hist, hist_words);
    LAUNCH(c, KID_EF_HIST, st, k_ef_hist, c->n_spans, grad, residual, t, h0);
    LAUNCH(c, KID_PICK0, st, k_pick<0>, B, t, (const uint32_t *)h0);
    LAUNCH(c, KID_REFINE1, st, k_refine<1>, c->n_spans, (const float *)residual, t, h1);
    LAUNCH(c, KID_PICK1, st, k_pick<1>, B, t, (const uint32_t *)h1);
    LAUNCH(c, KID_REFINE2, st, k_refine<2>, c->n_spans, (const float *)residual, t, h2);
    LAUNCH(c, KID_PICK2, st, k_pick<2>, B, t, (const uint32_t *)h2);
    LAUNCH(c, KID_COUNT, st, k_count, c->n_spans, (const float *)residual, t, c->d_tG, c->d_tE);
    LAUNCH(c, KID_SCAN, st, k_scan, B, t, c->d_tG, c->d_tE);
    LAUNCH(c, KID_WRITE, st, k_write, c->n_spans, (const float *)residual, t,
           (const uint32_t *)c->d_tG, (const uint32_t *)c->d_tE, idx, vdst);
    const uint32_t qgrid = (uint32_t)c->NC;
    switch (bits) {
    case 32: LAUNCH(c, KID_QUANT, st, k_quant<32>, qgrid, (const float *)vdst, (const uint32_t *)idx, t, residual, val, scales); break;
    case 16: LAUNCH(c, KID_QUANT, st, k_quant<16>, qgrid, (const float *)vdst, (const uint32_t *)idx, t, residual, val, scales); break;
    case 8:  LAUNCH(c, KID_QUANT, st, k_quant<8>,  qgrid, (const float *)vdst, (const uint32_t *)idx, t, residual, val, scales); break;
    default: LAUNCH(c, KID_QUANT, st, k_quant<4>,  qgrid, (const float *)vdst, (const uint32_t *)idx, t, residual, val, scales); break;
    }
    return NSML_OK;
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
    switch (bits) {
    case 32: LAUNCH(c, KID_DECOMP, st, k_decomp<32>, c->n_spans, idx, val, scales, t, dense_out); break;
    case 16: LAUNCH(c, KID_DECOMP, st, k_decomp<16>, c->n_spans, idx, val, scales, t, dense_out); break;
    case 8:  LAUNCH(c, KID_DECOMP, st, k_decomp<8>,  c->n_spans, idx, val, scales, t, dense_out); break;
    default: LAUNCH(c, KID_DECOMP, st, k_decomp<4>,  c->n_spans, idx, val, scales, t, dense_out); break;
    }
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

const char *nsml_kernel_name(int id) { return (id >= 0 && id < KID_N) ? kKernelNames[id] : nullptr; }

}  // extern "C"
