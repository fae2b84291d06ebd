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
 * bracketed by a band of keys [lo, hi) that holds the kw-th largest key: from a sample of |w|
 * with a wide margin, or, from the second call on, a narrow one around the threshold the call
 * before found (weights move little between steps).  One pass over the weights stages the
 * elements inside the band, counts those above it and writes the pruning bitmap (1 = pruned)
 * for everything outside it; the threshold key T and the number e of admitted elements equal to
 * T come from the staged elements alone (k_select_count / k_select_finish), and k_wfix sets the
 * bits of the band elements that turn out pruned.  A bucket whose band missed or overflowed
 * repeats the pass with an exact histogram and takes the dense ordered passes (k_whard), which
 * write its bitmap.  The gradient kernels read one bit per parameter.  Pruned parameters are
 * neither counted nor emitted, and their accumulated gradient is still written to the residual:
 * pruning is not permanent. */

/* Per bucket: the band of keys [lo, hi) to stage, from the sample histogram of |w|. */
__global__ __launch_bounds__(WG) void k_wpredict(Tables t, const uint32_t *__restrict__ hist_s,
                                                 uint32_t *__restrict__ wLo, uint32_t *__restrict__ wHi,
                                                 int force_dense, int miss,
                                                 const uint32_t *__restrict__ prevT, const uint32_t *__restrict__ prevHw)
{
    __shared__ uint32_t tmp[WG];
    __shared__ uint32_t res[6];          /* digit, above, at for the upper and the lower rank */
    const uint32_t b = blockIdx.x, tid = threadIdx.x;
    const uint64_t nb = t.off[b + 1] - t.off[b];
    const uint32_t k = t.k[b];
    if (b == 0 && tid < 4) t.nhard[tid] = 0u;      /* counted anew by k_wplan ([1]: the barrier of k_whard) */
    if (nb == 0 || k == 0 || force_dense) {
        if (tid == 0) { wLo[b] = NONE; wHi[b] = 0u; }
        return;
    }
    if (prevT && prevT[b] != NONE && !miss) {
        /* weights move little from one step to the next: a narrow band around the threshold the
         * last call found (k_wremember chose its width); if it misses, the pass is repeated */
        if (tid == 0) {
            const uint32_t T = prevT[b], hw = prevHw[b];
            wLo[b] = T > hw ? T - hw : 0u;
            wHi[b] = (uint32_t)min((uint64_t)T + hw + 1ull, 0x7FFFFFFFull);
        }
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
        /* diagnostic: a band of two digits above the right one, so that the threshold is missed */
        if (miss && wLo[b] != NONE) { wLo[b] = (res[0] + 1u) << SH0; wHi[b] = (res[0] + 3u) << SH0; }
    }
}

/* One pass over the weights.  For a bucket with a band [lo, hi): every element whose key lies in
 * the band is appended, in index order, to its wavefront's staging segment and counted in the
 * level-0 histogram (of the band only); the elements above the band are only counted, per
 * segment (c.G); and the pruning bitmap gets a first version: 1 for the elements below the band
 * (pruned for certain), 0 for the rest (the few band elements that end up pruned are set later by
 * k_wfix).  Hardly any element touches LDS, so the pass runs at the speed of reading w.
 * For a bucket without a band (no usable sample, or the dense passes were asked for) the exact
 * level-0 histogram of all its elements is built instead and nothing else is written.
 * second != 0: the repeat for the buckets whose band turned out not to hold the threshold
 * (redo[b] set by k_wplan): only those, treated as buckets without a band.
 * Same geometry as the streaming pass of the gradient (64 << segSh threads, one contiguous share
 * of the span per wavefront). */
/* (two workgroups of sixteen wavefronts per compute unit: one streams while the other starts or ends) */
__global__ __launch_bounds__(64 * MAX_SEG_WAVES, 8) void k_whist(const float *__restrict__ w, Tables t,
                                                              uint32_t *__restrict__ hist0, Cand c,
                                                              const uint32_t *__restrict__ wLo,
                                                              const uint32_t *__restrict__ wHi,
                                                              uint32_t *__restrict__ pmask,
                                                              const uint32_t *__restrict__ redo, int second)
{
    __shared__ uint32_t h[NB0];
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t nthreads = 64u << t.segSh;
    const SpanGeo s = span_geo(t, blockIdx.x);
    if (second && !redo[s.b]) return;                     /* same for the whole workgroup */
    for (uint32_t i = tid; i < NB0; i += nthreads) h[i] = 0;
    uint32_t lo_k = wLo[s.b], hi_k = wHi[s.b];             /* NONE, 0: no band */
    if (second) { lo_k = NONE; hi_k = 0u; }
    const bool band = lo_k != NONE;
    const uint32_t ss = (blockIdx.x << t.segSh) + wave;
    const uint64_t cbase = (uint64_t)ss * c.cap;
    uint32_t wcount = 0, above = 0;
    __syncthreads();
    const uint32_t per = (t.spanT * 4u) >> t.segSh;
    const uint32_t wt0 = wave * per;
    const uint32_t wt1 = min(s.ntiles * 4u, wt0 + per);
    for (uint32_t wt = wt0; wt < wt1; ++wt) {
        const uint64_t wb = s.base + (uint64_t)wt * WTILE;
        const bool interior = wb >= s.lo && wb + WTILE <= s.hi;
        f4 wv[4];
        if (interior) {
#pragma unroll
            for (int u = 0; u < 4; ++u)
                wv[u] = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(w + wb + (uint64_t)(u * 64 + lane) * 4));
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint64_t gi = wb + (uint64_t)(u * 64 + lane) * 4;
            float a[4];
            uint32_t m = 0xFu;
            if (interior) { a[0] = wv[u].x; a[1] = wv[u].y; a[2] = wv[u].z; a[3] = wv[u].w; }
            else m = load_quad(w, gi, s.lo, s.hi, a);
            uint32_t key[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) key[j] = keyof(a[j]);
            if (!band) {
                if (interior) hist_quad_full(h, key[0] >> SH0, key[1] >> SH0, key[2] >> SH0, key[3] >> SH0);
                else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if ((m >> j) & 1u) atomicAdd(&h[key[j] >> SH0], 1u);
                }
                continue;
            }
            bool f[4];
            uint32_t bits = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bool in = (m >> j) & 1u;
                const bool below = key[j] < lo_k, over = key[j] >= hi_k;
                f[j] = in && !below && !over;
                above += (in && over) ? 1u : 0u;
                bits |= ((in && below) ? 1u : 0u) << j;
            }
            if (f[0] | f[1] | f[2] | f[3]) {              /* rare: the band is narrow */
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (f[j]) atomicAdd(&h[key[j] >> SH0], 1u);
            }
            emit_quad(f, a, (uint32_t)(gi - s.lo), c, cbase, wcount);
            /* eight lanes share a word of the bitmap (four bits per quad): lane 8g collects the
             * words of lanes 8g .. 8g+7 by shifts inside its row of 16 lanes */
            uint32_t word = bits << ((lane & 7u) * 4u);
            word |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)word, 0x101, 0xF, 0xF, true);     /* from lane + 1 */
            word |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)word, 0x102, 0xF, 0xF, true);     /* from lane + 2 */
            word |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)word, 0x104, 0xF, 0xF, true);     /* from lane + 4 */
            if ((lane & 7u) == 0u)
                pmask[(uint64_t)(s.tile_g + (wt >> 2)) * (TILE / 32) + (wt & 3u) * (WG / 8) + u * 8 + (lane >> 3)] = word;
        }
    }
    if (band) {
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) above += __shfl_xor(above, d, 64);
        if (lane == 0) {
            c.cnt[ss] = min(wcount, c.cap);
            c.G[ss] = above;
            if (wcount > c.cap) t.ovf[s.b] = 1u;
        }
    } else if (lane == 0 && !second) {
        c.cnt[ss] = 0u;
        c.G[ss] = 0u;
    }
    __syncthreads();
    hist_flush(h, hist0 + (uint64_t)s.b * NB0, NB0, (int)nthreads);
}

/* Per bucket: level-0 digit of the kw-th largest |weight|.  With a band: from the counts of the
 * elements above the band and the histogram of the band; the staged band can decide the rest iff
 * the kw-th largest lies inside it and no staging segment overflowed, otherwise the bucket is
 * marked for the repeat of the pass (redo) and its histogram is cleared for it.  Without a band,
 * and in the second round (after the repeat): from the exact histogram, dense passes. */
__global__ __launch_bounds__(WG) void k_wplan(Tables t, uint32_t *__restrict__ hist0, Cand c,
                                              const uint32_t *__restrict__ wLo, const uint32_t *__restrict__ wHi,
                                              uint32_t *__restrict__ redo, uint32_t *__restrict__ nband_out, int second)
{
    __shared__ uint32_t tmp[WG];
    __shared__ uint32_t red[2][WG / 64];
    const uint32_t b = blockIdx.x, tid = threadIdx.x;
    const uint32_t want = t.k[b];
    if (second && !redo[b]) return;
    if (want == 0) {
        if (tid == 0) { t.T[b] = NONE; t.need[b] = 0; t.fast[b] = PATH_BAND; t.sh[b] = SH0; redo[b] = 0u; }
        return;
    }
    const bool band = !second && wLo[b] != NONE;
    uint32_t n_above = 0, n_band = 0;
    if (band) {
        uint32_t ca = 0, cb = 0;
        for (uint32_t ss = (t.span0[b] << t.segSh) + tid; ss < (t.span0[b + 1] << t.segSh); ss += WG) { ca += c.G[ss]; cb += c.cnt[ss]; }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) { ca += __shfl_xor(ca, d, 64); cb += __shfl_xor(cb, d, 64); }
        if ((tid & 63) == 0) { red[0][tid >> 6] = ca; red[1][tid >> 6] = cb; }
        __syncthreads();
        n_above = red[0][0] + red[0][1] + red[0][2] + red[0][3];
        n_band = red[1][0] + red[1][1] + red[1][2] + red[1][3];
        if (tid == 0) nband_out[b] = n_band;
    }
    DigitWalk<NB0> w;
    w.load(hist0 + (uint64_t)b * NB0, tmp);
    const bool inside = band && !t.ovf[b] && want > n_above && want - n_above <= n_band;
    if (band && !inside) {
        /* the band missed (or overflowed): the pass is repeated for this bucket with the full histogram */
        w.clear(hist0 + (uint64_t)b * NB0);
        if (tid == 0) { redo[b] = 1u; t.fast[b] = PATH_DENSE; }
        return;
    }
    if (tid == 0 && !second) redo[b] = 0u;
    uint32_t digit, above, at;
    if (w.find(inside ? want - n_above : want, digit, above, at)) {
        t.T[b] = digit;
        t.need[b] = (inside ? want - n_above : want) - above;
        t.sh[b] = SH0;
        t.fast[b] = inside ? PATH_BAND : PATH_DENSE;
        if (!inside) atomicAdd(t.nhard + 2, 1u);         /* k_whard has work */
    }
}

/* What the next call's band is built from, per bucket: the threshold key this call found, and a
 * half-width that would have staged about 0.2 % of the bucket (at least 4096 elements) at the
 * density of keys this call's band had.  A bucket that took the dense passes remembers nothing. */
__global__ __launch_bounds__(WG) void k_wremember(Tables t, const uint32_t *__restrict__ wT,
                                                  const uint32_t *__restrict__ wLo, const uint32_t *__restrict__ wHi,
                                                  const uint32_t *__restrict__ nband, uint32_t *__restrict__ prevT,
                                                  uint32_t *__restrict__ prevHw)
{
    const uint32_t b = blockIdx.x * WG + threadIdx.x;
    if (b >= t.B) return;
    const uint64_t nb = t.off[b + 1] - t.off[b];
    if (!t.fast[b] || t.k[b] == 0u || wT[b] == NONE || wLo[b] == NONE) { prevT[b] = NONE; return; }
    const uint64_t width = (uint64_t)wHi[b] - wLo[b];
    const uint64_t target = nb / 512 > 4096 ? nb / 512 : 4096;
    uint64_t hw = nband[b] ? width * target / (2ull * nband[b]) : width;
    hw = hw < 256 ? 256 : (hw > (1ull << 24) ? (1ull << 24) : hw);
    prevT[b] = wT[b];
    prevHw[b] = (uint32_t)hw;
}

}  // namespace

#endif
