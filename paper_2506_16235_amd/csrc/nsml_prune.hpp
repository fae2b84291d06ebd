/*
 * libnsml device code, part 3: weight-magnitude pruning (Algorithm 2 Step 2).
 * Included by nsml_kernels.hip (one translation unit); not a public header.
 */
#ifndef NSML_PRUNE_HPP
#define NSML_PRUNE_HPP

namespace {

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
    (void)werr;
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

}  // namespace

#endif
