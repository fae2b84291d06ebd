/*
 * libnsml device code, part 2: the selection path: sample, candidate bound, the streaming pass, the candidate
 * and dense-fallback stages of the radix select.
 * Included by nsml_kernels.hip (one translation unit); not a public header.
 */
#ifndef NSML_SELECT_HPP
#define NSML_SELECT_HPP

namespace {

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

}  // namespace

#endif
