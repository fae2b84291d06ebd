/*
 * libnsml device code, part 2: the head of the selection: sample, what to stage, the streaming
 * pass, the plan, and the radix steps over the dense accumulator that the fallback uses.
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
            if (SUM && t.pmask) {
                const uint64_t rel = gi - a0;
                m &= ~pruned_bits(t.pmask, t.tile0[b] + (uint32_t)(rel / TILE), (uint32_t)(rel % TILE) / 4);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if ((m >> j) & 1u) atomicAdd(&h[keyof(SUM ? __fadd_rn(x[j], y[j]) : x[j]) >> SH0], 1u);
        }
    }
    __syncthreads();
    hist_flush(h, hist_s + (uint64_t)b * NB0, NB0);
}

/* Per bucket: what the streaming pass stages, from the sample histogram.  The sample count
 * above the true k-th key is binomial with mean ks = k * m / n.
 *   candidates  k at most an eighth of the bucket: L_b = lower edge of the digit that has
 *               ks + 4 sqrt(ks) + 4 sampled keys above it; everything from L_b up is staged and
 *               contains the k largest unless the sample was very unlucky
 *   band        larger k (ratios towards 1): staging everything above a bound would be most of
 *               the bucket, so only the level-0 digits between the ranks ks +- (4 sqrt(ks) + 4)
 *               are staged, [L_b, H_b); the elements above H_b are survivors for certain and are
 *               only counted
 *   zero        even the optimistic rank lies among keys below 2^19 (in practice: exact zeros,
 *               as in an embedding whose rows were not touched), or k is the whole bucket: the
 *               threshold key is 0, nothing is staged, non-zero and zero keys are counted
 * A bucket for which none of this fits (or whose guess turns out wrong once the exact histogram
 * is known) takes the dense passes and still gets the exact result. */
__global__ __launch_bounds__(WG) void k_predict(Tables t, uint32_t *__restrict__ hist_s,
                                                int force_dense)
{
    __shared__ uint32_t tmp[WG];
    __shared__ uint32_t res[9];          /* digit, above, at for three ranks */
    const uint32_t b = blockIdx.x, tid = threadIdx.x;
    const uint64_t nb = t.off[b + 1] - t.off[b];
    const uint32_t k = t.k[b];
    if (b == 0 && tid < 4) t.nhard[tid] = 0u;      /* counted anew by this call's plan ([1]: the barrier of k_hard) */
    if (nb == 0 || force_dense) {
        if (tid == 0) { t.L[b] = NONE; t.H[b] = NONE; t.subLo[b] = NONE; }
        return;
    }
    if ((uint64_t)k == nb) {             /* everything is sent: all keys >= 1, and the zeros as ties of key 0 */
        if (tid == 0) { t.L[b] = 1u; t.H[b] = 1u; t.subLo[b] = NONE; }
        for (int i = tid; i < NB0; i += WG) hist_s[(uint64_t)b * NB0 + i] = 0u;     /* left clean for the next call */
        return;
    }
    DigitWalk<NB0> w;
    w.load(hist_s + (uint64_t)b * NB0, tmp);
    w.clear(hist_s + (uint64_t)b * NB0);
    const uint32_t m = w.total;
    if (m == 0) {
        if (tid == 0) { t.L[b] = NONE; t.H[b] = NONE; t.subLo[b] = NONE; }
        return;
    }
    const bool exact = nb < SAMPLE_ALL_BELOW;
    /* the sample was drawn from the parameters that can be selected: all of them, or the
     * ones the pruning step kept */
    const double pop = t.pmask ? (double)t.kw[b] : (double)nb;
    const double ks = (double)k * (double)m / pop;
    /* the margin: four standard deviations of a binomial sample, times what the bucket has
     * learned (a sample of 32-element runs of a gradient whose large values come in runs has far
     * fewer independent draws than entries; a bucket whose guess missed widens its margin) */
    const double widen = (double)(t.margin[b] & 0xFFu ? t.margin[b] & 0xFFu : 1u);
    const double dev = exact ? 0.0 : (4.0 * sqrt(ks) + 4.0) * widen;
    const double want_d = exact ? (double)k : ceil(ks + dev);
    const double cap_b = (double)(t.span0[b + 1] - t.span0[b]) * 4.0 * (double)t.spanT * 256.0;
    double r_up = floor(ks - dev), r_dn = ceil(ks + dev);
    r_up = r_up < 1.0 ? 1.0 : (r_up > (double)m ? (double)m : r_up);
    r_dn = r_dn < 1.0 ? 1.0 : (r_dn > (double)m ? (double)m : r_dn);
    const double r_c = want_d > (double)m ? (double)m : (want_d < 1.0 ? 1.0 : want_d);
    uint32_t digit, above, at;
    if (w.find((uint32_t)r_c, digit, above, at)) { res[0] = digit; res[1] = above; res[2] = at; }
    if (w.find((uint32_t)r_up, digit, above, at)) { res[3] = digit; res[4] = above; res[5] = at; }
    if (w.find((uint32_t)r_dn, digit, above, at)) { res[6] = digit; res[7] = above; res[8] = at; }
    __syncthreads();
    if (tid != 0) return;
    uint32_t L = NONE, H = NONE;
    bool done = false;
    if (want_d <= (double)m && (double)k <= 0.5 * cap_b) {
        const double est = (double)(res[1] + res[2]) * pop / (double)m;
        if (est <= 0.8 * cap_b) { L = res[0] << SH0; done = true; }
    }
    if (!done) {
        const uint32_t dig_up = res[3], dig_dn = res[6];
        if (dig_up == 0u) {
            L = 1u; H = 1u;
        } else {
            /* a pessimistic rank among the zeros (digit 0) while the optimistic one is not: the band
             * starts at key 1, zeros are only counted, and the plan decides between a zero
             * threshold and one inside the band */
            const double in_band = (double)res[7] + (dig_dn != 0u ? (double)res[8] : 0.0) - (double)res[4];
            const double est = in_band * pop / (double)m;
            if (est <= 0.8 * cap_b) { L = dig_dn != 0u ? dig_dn << SH0 : 1u; H = (dig_up + 1u) << SH0; }
        }
    }
    t.L[b] = L;
    t.H[b] = H;
    /* the k-th key lies, very likely, in one of the level-0 digits between the two ranks: the
     * streaming pass counts six more key bits inside them, so that the plan knows the threshold to
     * 18 bits and only 1/64 of such a digit stays undecided.  (With error feedback the
     * accumulators pile up just below the threshold: one level-0 digit there can hold 4 % of a
     * bucket.) */
    t.subLo[b] = (L != NONE && L != H) ? res[6] : NONE;
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
                                       uint32_t m, uint32_t cm, uint32_t li, uint32_t *h, uint32_t *hb, uint32_t subLo,
                                       uint32_t L, uint32_t H,
                                       const Cand &c, uint64_t cbase, uint32_t &wcount, uint32_t &n_hi, uint32_t &n_lo)
{
    uint32_t key[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) key[j] = keyof(a[j]);
    if (EMIT) {
        /* the finer histogram of the few digits around the expected threshold */
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t dd = (key[j] >> SH0) - subLo;
            if (((cm >> j) & 1u) && dd < (uint32_t)SUB_DIGITS)
                atomicAdd(&hb[(dd << SUB_BITS) | ((key[j] >> SHS) & ((1u << SUB_BITS) - 1u))], 1u);
        }
    }
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
        for (int j = 0; j < 4; ++j) f[j] = ((cm >> j) & 1u) && key[j] >= L && key[j] < H;
        emit_quad(f, a, li, c, cbase, wcount);
        if (H != NONE) {
            /* a band is staged: count what lies above it (survivors for certain) and below it */
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                n_hi += __popcll(__ballot(((cm >> j) & 1u) && key[j] >= H));
                n_lo += __popcll(__ballot(((cm >> j) & 1u) && key[j] < L));
            }
        }
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
                                                Tables t, uint32_t *__restrict__ hist0, uint32_t *__restrict__ hist0b,
                                                Cand c, double *__restrict__ span_sq)
{
    __shared__ uint32_t h[NB0];
    __shared__ uint32_t hb[NBS];
    __shared__ double sq_w[MAX_SEG_WAVES];
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t nthreads = 64u << t.segSh;
    /* a workgroup takes a contiguous share of the spans (one span each when the grid has as many
     * workgroups as there are spans); the LDS histogram is flushed when the bucket changes */
    const uint32_t share = (t.n_spans + gridDim.x - 1) / gridDim.x;
    const uint32_t sp0 = blockIdx.x * share, sp1 = min(t.n_spans, sp0 + share);
    uint32_t cur_b = NONE;
    for (uint32_t span = sp0; span < sp1; ++span) {
    double sq = 0.0;                     /* sum of grad^2 over this thread's elements */
    const SpanGeo s = span_geo(t, span);
    /* this wavefront's wave-tiles: [wave * per, (wave + 1) * per) of the span's 4 * ntiles.  The
     * rows of a wave-tile that lies wholly inside the bucket are requested half a wave-tile
     * ahead: the first two before the histograms are set up, each further pair before the pair at
     * hand is worked on, so a wavefront always has loads in flight. */
    constexpr int FR = 2;                /* rows of 1 KiB per operand and request */
    const uint32_t per = (t.spanT * 4u) >> t.segSh;
    const uint32_t wt0 = wave * per;
    const uint32_t wt1 = min(s.ntiles * 4u, wt0 + per);
    f4 gn[FR], rn[FR];
    auto whole = [&](uint32_t wt) {
        const uint64_t wb = s.base + (uint64_t)wt * WTILE;
        return wt < wt1 && wb >= s.lo && wb + WTILE <= s.hi;
    };
    auto fetch = [&](uint32_t wt, int half) {
        const uint64_t wb = s.base + (uint64_t)wt * WTILE;
#pragma unroll
        for (int v = 0; v < FR; ++v) {
            const uint64_t gi = wb + (uint64_t)((half * FR + v) * 64 + lane) * 4;
            gn[v] = (NT & 1) ? __builtin_nontemporal_load(reinterpret_cast<const f4 *>(g + gi))
                             : *reinterpret_cast<const f4 *>(g + gi);
            rn[v] = (NT & 2) ? __builtin_nontemporal_load(reinterpret_cast<const f4 *>(r + gi))
                             : *reinterpret_cast<const f4 *>(r + gi);
        }
    };
    if (whole(wt0)) fetch(wt0, 0);
    if (s.b != cur_b) {
        if (cur_b != NONE) {
            __syncthreads();
            hist_flush(h, hist0 + (uint64_t)cur_b * NB0, NB0, (int)nthreads);
            if (EMIT) hist_flush(hb, hist0b + (uint64_t)cur_b * NBS, NBS, (int)nthreads);
            __syncthreads();
        }
        for (uint32_t i = tid; i < NB0; i += nthreads) h[i] = 0;
        if (EMIT) for (uint32_t i = tid; i < NBS; i += nthreads) hb[i] = 0;
        cur_b = s.b;
    }
    uint32_t subLo = EMIT ? t.subLo[s.b] : NONE;
    if (subLo == NONE) subLo = 0x80000000u;              /* no digit is within reach of it */
    const uint32_t L = EMIT ? t.L[s.b] : NONE;
    const uint32_t H = EMIT ? t.H[s.b] : NONE;           /* NONE: no upper bound */
    uint32_t n_hi = 0, n_lo = 0;                          /* band mode: elements above / below the band */
    const uint32_t ss = (span << t.segSh) + wave;
    const uint64_t cbase = (uint64_t)ss * c.cap;
    uint32_t wcount = 0;
    __syncthreads();
    for (uint32_t wt = wt0; wt < wt1; ++wt) {
        const uint64_t wb = s.base + (uint64_t)wt * WTILE;
        if (whole(wt)) {
            {
#pragma unroll
            for (int half = 0; half < 4 / FR; ++half) {
                /* the sums first: they free the registers the next rows arrive in */
                float acc[FR][4];
#pragma unroll
                for (int v = 0; v < FR; ++v) {
                    acc[v][0] = __fadd_rn(gn[v].x, rn[v].x); acc[v][1] = __fadd_rn(gn[v].y, rn[v].y);
                    acc[v][2] = __fadd_rn(gn[v].z, rn[v].z); acc[v][3] = __fadd_rn(gn[v].w, rn[v].w);
                    sq += (double)(__fmaf_rn(gn[v].x, gn[v].x, __fmul_rn(gn[v].y, gn[v].y)) +
                                   __fmaf_rn(gn[v].z, gn[v].z, __fmul_rn(gn[v].w, gn[v].w)));
                }
                if (half + 1 < 4 / FR) fetch(wt, half + 1);
                else if (whole(wt + 1)) fetch(wt + 1, 0);
#pragma unroll
                for (int v = 0; v < FR; ++v) {
                    const int u = half * FR + v;
                    const uint64_t gi = wb + (uint64_t)(u * 64 + lane) * 4;
                    const float (&a)[4] = acc[v];
                    uint32_t cm = 0xFu;
                    if (PRUNE) cm &= ~pruned_bits(t.pmask, s.tile_g + (wt >> 2), (wt & 3u) * WG + u * 64 + lane);
                    ef_row<true, EMIT, NT, PRUNE>(r, gi, a, 0xFu, cm, (uint32_t)(gi - s.lo), h, hb, subLo, L, H, c, cbase, wcount, n_hi, n_lo);
                }
            }
            }
        } else {
            if (whole(wt + 1)) fetch(wt + 1, 0);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint64_t gi = wb + (uint64_t)(u * 64 + lane) * 4;
                float x[4], y[4], a[4];
                const uint32_t m = load_quad(g, gi, s.lo, s.hi, x);
                load_quad(r, gi, s.lo, s.hi, y);
#pragma unroll
                for (int j = 0; j < 4; ++j) { a[j] = __fadd_rn(x[j], y[j]); sq += (double)__fmul_rn(x[j], x[j]); }
                uint32_t cm = m;
                if (PRUNE) cm &= ~pruned_bits(t.pmask, s.tile_g + (wt >> 2), (wt & 3u) * WG + u * 64 + lane);
                ef_row<false, EMIT, NT, PRUNE>(r, gi, a, m, cm, (uint32_t)(gi - s.lo), h, hb, subLo, L, H, c, cbase, wcount, n_hi, n_lo);
            }
        }
    }
    if (EMIT && lane == 0) {
        /* the true count: more than the segment holds means "read this segment from the dense
         * accumulator" to the kernels that follow */
        c.cnt[ss] = wcount;
        if (wcount > c.cap) t.ovf[s.b] = 1u;
        if (H != NONE) { c.G[ss] = n_hi; c.E[ss] = n_lo; }
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
        span_sq[span] = tot;
    }
    }
    __syncthreads();
    if (cur_b != NONE) {
        hist_flush(h, hist0 + (uint64_t)cur_b * NB0, NB0, (int)nthreads);
        if (EMIT) hist_flush(hb, hist0b + (uint64_t)cur_b * NBS, NBS, (int)nthreads);
    }
}

/* Per bucket: exact level-0 digit of the k-th largest key, the gradient's |.|^2, and how the
 * bucket is decided (PATH_*).  The staged elements can decide it when they are known to hold
 * every element of that digit: in candidate mode they are exactly the elements with key >= L_b,
 * so they do iff there are at least k of them; in band mode iff the digit lies inside the band;
 * in both only if no staging segment overflowed and the undecided keys of the digit are few
 * enough to fit the free part of the staging area (k_select_count parks them there).  In zero mode
 * the counts settle everything: fewer non-zero elements than k means threshold key 0. */
__global__ __launch_bounds__(WG) void k_plan(Tables t, uint32_t *__restrict__ hist0, uint32_t *__restrict__ hist0b,
                                             Cand c, int have_cand,
                                             const double *__restrict__ span_sq, double *__restrict__ l2sq)
{
    __shared__ uint32_t tmp[WG];
    __shared__ uint32_t fnd[4];          /* digit, above, at of the k-th key; whether any thread found it */
    __shared__ double red[WG / 64];
    __shared__ uint32_t redc[WG / 64], redh[WG / 64];
    const uint32_t b = blockIdx.x, tid = threadIdx.x;
    const uint32_t L = t.L[b], H = t.H[b];
    uint32_t n_cand = 0, n_hi = 0;
    {   /* |grad|^2 of the bucket: strided partial sums, then a fixed tree; staged counts likewise */
        double acc = 0.0;
        for (uint32_t s = t.span0[b] + tid; s < t.span0[b + 1]; s += WG) acc += span_sq[s];
        uint32_t cc = 0, ch = 0;
        if (have_cand && L != NONE)
            for (uint32_t ss = (t.span0[b] << t.segSh) + tid; ss < (t.span0[b + 1] << t.segSh); ss += WG) {
                cc += c.cnt[ss];
                if (H != NONE) ch += c.G[ss];
            }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) { acc += __shfl_xor(acc, d, 64); cc += __shfl_xor(cc, d, 64); ch += __shfl_xor(ch, d, 64); }
        if ((tid & 63) == 0) { red[tid >> 6] = acc; redc[tid >> 6] = cc; redh[tid >> 6] = ch; }
        __syncthreads();
        if (tid == 0) l2sq[b] = (red[0] + red[1]) + (red[2] + red[3]);
        n_cand = redc[0] + redc[1] + redc[2] + redc[3];
        n_hi = redh[0] + redh[1] + redh[2] + redh[3];
    }
    const uint32_t want = t.k[b];
    if (want == 0) {                       /* empty bucket: nothing can match */
        if (tid == 0) { t.T[b] = NONE; t.need[b] = 0; t.fast[b] = PATH_CAND; }
        return;
    }
    DigitWalk<NB0> w;
    w.load(hist0 + (uint64_t)b * NB0, tmp);
    w.clear(hist0 + (uint64_t)b * NB0);        /* left clean for the next call, like the overflow flag below */
    const uint32_t ovf = t.ovf[b];
    if (tid == 0 && ovf) t.ovf[b] = 0u;
    /* the finer counts of the digits around the expected threshold: fetched by the first
     * wavefront (64 bins of whichever digit it turns out to be), zeroed again for the next call */
    const uint32_t subLo = t.subLo[b];
    uint32_t subrow[SUB_DIGITS];
#pragma unroll
    for (int d = 0; d < SUB_DIGITS; ++d) {
        uint32_t *p = hist0b + (uint64_t)b * NBS + (d << SUB_BITS) + ((1u << SUB_BITS) - 1u - tid);   /* top bin first */
        subrow[d] = 0u;
        if (tid < (1u << SUB_BITS) && subLo != NONE) { subrow[d] = *p; if (subrow[d]) *p = 0u; }
    }
    if (tid == 0) fnd[3] = 0u;
    __syncthreads();
    {
        uint32_t digit, above, at;
        if (w.find(want, digit, above, at)) { fnd[0] = digit; fnd[1] = above; fnd[2] = at; fnd[3] = 1u; }
    }
    __syncthreads();
    if (tid < 64 && fnd[3]) {
        const uint32_t digit = fnd[0], above = fnd[1];
        uint32_t at = fnd[2];
        uint32_t path = PATH_DENSE, T = digit, need = want - above, sh = SH0;
        /* six more bits of the threshold from the finer counts, when the digit is among them and
         * the counts add up (they do unless the digit was not covered) */
        bool fine = false;
        uint32_t T18 = 0, need18 = 0, at18 = 0;
        if (subLo != NONE && digit - subLo < (uint32_t)SUB_DIGITS) {
            uint32_t mine = 0;
#pragma unroll
            for (int d = 0; d < SUB_DIGITS; ++d) mine = (digit - subLo == (uint32_t)d) ? subrow[d] : mine;
            uint32_t incl = mine;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const uint32_t y = __shfl_up(incl, d, 64);
                if (tid >= (uint32_t)d) incl += y;
            }
            const uint32_t total = __shfl(incl, 63, 64);
            const bool here = incl - mine < need && need <= incl;      /* lane = 63 - (the six bits) */
            const uint64_t bal = __ballot(here);
            if (total == at && bal) {
                const uint32_t ln = (uint32_t)__builtin_ctzll(bal);
                T18 = (digit << SUB_BITS) | (63u - ln);
                need18 = need - (__shfl(incl, ln, 64) - __shfl(mine, ln, 64));
                at18 = __shfl(mine, ln, 64);
                fine = true;
            }
        }
        if (tid != 0) return;
        uint32_t why = 0u;
        if (!have_cand || L == NONE) why = WHY_NO_GUESS;
        else {
            /* a staging segment that overflowed is read from the dense accumulator by the kernels
             * that find the threshold; the survivors of such a bucket are then taken from the dense
             * accumulator as well (PATH_BAND), since the staged entries cannot supply them all */
            const uint64_t cap_b = (uint64_t)((t.span0[b + 1] - t.span0[b]) << t.segSh) * c.cap;
            if (fine) at = at18;
            const bool room = (uint64_t)n_cand <= cap_b && (uint64_t)at * 2u <= cap_b - (uint64_t)n_cand;     /* for the undecided keys in the tails */
            if (H == NONE) {
                if (n_cand >= want && room) path = ovf ? PATH_BAND : PATH_CAND;
                else why = n_cand < want ? WHY_TOO_FEW : WHY_NO_ROOM;
            } else if (L == H) {
                /* n_hi = non-zero keys among the selectable elements: if they are no more than k,
                 * all of them survive and zeros (lowest indices first) fill the rest */
                if (n_hi <= want) { path = PATH_ZERO; T = 0u; need = want - n_hi; }
                else why = WHY_NONZEROS;
            } else if (L == 1u && n_hi + n_cand <= want) {
                /* the band starts at key 1 and everything non-zero is still not enough: zero threshold */
                path = PATH_ZERO; T = 0u; need = want - (n_hi + n_cand);
            } else if ((digit << SH0) >= L && ((digit + 1u) << SH0) <= H) {
                if (room) path = PATH_BAND;
                else why = WHY_NO_ROOM;
            } else why = WHY_OUTSIDE_BAND;
            if (fine && (path == PATH_CAND || path == PATH_BAND)) { T = T18; need = need18; sh = SHS; }
        }
        t.why[b] = why;
        {
            /* low byte: factor on the margin of k_predict (1, 2, 4, 8, 16); above it: calls since it last grew.
             * A guess that missed doubles it, 64 calls without a miss halve it. */
            const uint32_t mg = t.margin[b];
            uint32_t f = mg & 0xFFu ? mg & 0xFFu : 1u, age = mg >> 8;
            if (why == WHY_TOO_FEW || why == WHY_OUTSIDE_BAND) { f = f < 16u ? f * 2u : 16u; age = 0u; }
            else if (++age >= 64u) { f = f > 1u ? f / 2u : 1u; age = 0u; }
            t.margin[b] = (age << 8) | f;
        }
        t.T[b] = T;
        t.need[b] = need;
        t.sh[b] = sh;
        t.fast[b] = path;
        if (path != PATH_CAND) atomicAdd(t.nhard, 1u);
        if (path == PATH_DENSE) atomicAdd(t.nhard + 2, 1u);
    }
}

/* One workgroup: the list of spans that belong to fallback buckets.  (Kept as its own small
 * launch: doing it in the last workgroup of k_plan needs a device-scope fence in every
 * workgroup, which on this multi-die GPU writes back each L2 and costs more than a launch.) */
__device__ __forceinline__ void fb_plan_body(const Tables &t)
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

constexpr uint32_t CU = 4;   /* entries a lane fetches ahead */

template <int LEVEL>
__device__ __forceinline__ void pick_body(const Tables &t, const uint32_t *__restrict__ hist_c,
                                          const uint32_t *__restrict__ hist_f, uint32_t *__restrict__ err,
                                          uint32_t *__restrict__ wT_out, int only_fb, uint32_t b)
{
    constexpr int NB = LEVEL == 2 ? NB2 : NB1;
    constexpr int BITS = LEVEL == 2 ? 7 : 12;
    __shared__ uint32_t tmp[WG];
    const uint32_t tid = threadIdx.x;
    if (only_fb && t.fast[b]) return;          /* decided from its staged elements */
    const uint32_t want = t.need[b];
    if (want == 0) {
        /* empty bucket */
        if (LEVEL == 2 && wT_out && tid == 0) wT_out[b] = 0u;
        return;
    }
    const uint32_t *hist = t.fast[b] ? hist_c : hist_f;
    DigitWalk<NB> w;
    w.load(hist + (uint64_t)b * NB, tmp);
    if (only_fb) w.clear(const_cast<uint32_t *>(hist) + (uint64_t)b * NB);     /* left clean for the next call */
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
    }
}

/* Per bucket: exclusive scan, in place, of per-unit counts (units: the bucket's staging
 * segments on the candidate path, its tiles on the fallback path).  Both counts of a unit
 * travel as one 64-bit word (neither total can reach 2^32: a bucket has fewer elements), and
 * every thread takes four consecutive units, so a round covers 1024 units with one scan. */
__device__ __forceinline__ void scan_body(const Tables &t, uint32_t *__restrict__ cG, uint32_t *__restrict__ cE,
                                          uint32_t *__restrict__ tG, uint32_t *__restrict__ tE, int only_fb, uint32_t b)
{
    __shared__ uint64_t tmp[WG / 64];
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t mode = t.fast[b];
    if (only_fb) {
        /* gradient stage: only the buckets on the dense passes, whose counts are per segment too */
        if (mode != PATH_DENSE) return;
        mode = 1u;
    }
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
                if (t.pmask) m &= ~pruned_bits(t.pmask, s.tile_g + ti, u * WG + tid);
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

}  // namespace

#endif
