/*
 * libnsml device code, part 5: the tail of the selection.
 * Included by nsml_kernels.hip (one translation unit); not a public header.
 *
 * What the tail knows when it starts (left by the streaming pass and the plan): for every
 * bucket the leading bits b0 of its k-th largest key (the level-0 digit, or 18 bits when the
 * finer histogram covered it) and how many of the keys that share them are still wanted; for
 * every staging segment its entries (index, value) in index order.  Entries above b0 are
 * survivors, entries below it are not, the ones that share it are the only undecided ones, and
 * they are few.
 *
 *   k_select_count   per segment: entries above b0; the keys of the undecided entries go to a list
 *                    per workgroup (read back with coalesced loads) and, as a fallback, into the
 *                    unused tail of the segment's own staging area
 *   k_select_finish  per bucket, one workgroup of 1024 threads: threshold key T and tie allowance
 *                    e from those few keys (the remaining bits, histograms in LDS); per segment
 *                    the number of survivors and of threshold ties that precede it in the bucket;
 *                    per chunk of the payload the segment that holds its first survivor
 *   k_encode         PATH_CAND, per chunk of `chunk` consecutive survivors: gathers them in index
 *                    order from the staged entries into LDS, then scale, codes, packing, indices
 *                    and the residual update, all from LDS
 *   k_hard           PATH_BAND / PATH_ZERO (survivors too many to stage: a band of keys around
 *                    the threshold was staged instead, or the threshold is key 0): survivors
 *                    taken from the dense accumulator and coded in one streaming pass;
 *                    PATH_DENSE: every radix step over the dense accumulator, barriers between
 *   k_quant          codes the chunks k_hard wrote uncoded
 *   k_wfix, k_whard  the same machinery for the pruning bitmap of the weight stage
 * Every small kernel here is a handful of dependent memory round trips long, which is what a
 * small kernel costs on this GPU; tables that a kernel would otherwise search for (workgroup ->
 * segments, chunk -> bucket, chunk -> first segment) are therefore prepared by the kernel before.
 */
#ifndef NSML_TAIL_HPP
#define NSML_TAIL_HPP

namespace {

constexpr uint32_t SEL_THREADS = 1024;     /* k_select_finish workgroup: 16 wavefronts */
constexpr uint32_t SEL_WAVES = SEL_THREADS / 64;
constexpr uint32_t SEL_SEGS_PER_WAVE = 4;
constexpr uint32_t ENC_BLK = WG * 8;       /* survivors gathered in LDS at a time */

/* Inclusive scan of 64-bit values over a workgroup of NW wavefronts; tmp: NW words of LDS. */
template <uint32_t NW>
__device__ __forceinline__ uint64_t block_incl_scan64(uint64_t x, uint64_t *tmp, uint64_t &total)
{
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t hi = __shfl_up((uint32_t)(x >> 32), d, 64), lo = __shfl_up((uint32_t)x, d, 64);
        if (lane >= (uint32_t)d) x += ((uint64_t)hi << 32) | (uint64_t)lo;
    }
    if (lane == 63) tmp[wave] = x;
    __syncthreads();
    uint64_t before = 0;
    total = 0;
#pragma unroll
    for (uint32_t w = 0; w < NW; ++w) { const uint64_t v = tmp[w]; before += w < wave ? v : 0ull; total += v; }
    __syncthreads();
    return x + before;
}

/* The digit of an LDS histogram of NB bins that holds the want-th entry counted from the top
 * digit down (1 <= want <= number of entries).  Every thread of the NW-wavefront workgroup must
 * call it; res (3 words of LDS) receives digit, entries in higher digits, entries in the digit.
 * Returns false (in every thread) when the histogram holds fewer than `want` entries. */
template <int NB, uint32_t NW>
__device__ __forceinline__ bool find_digit_lds(const uint32_t *h, uint32_t want, uint64_t *tmp, uint32_t *res)
{
    constexpr int NT = NW * 64;
    constexpr int PER = NB >= NT ? NB / NT : 1;
    const int top = NB - 1 - (int)threadIdx.x * PER;
    uint32_t cnt[PER], sum = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) { const int d = top - i; cnt[i] = d >= 0 ? h[d] : 0u; sum += cnt[i]; }
    uint64_t total;
    const uint32_t incl = (uint32_t)block_incl_scan64<NW>((uint64_t)sum, tmp, total);
    const uint32_t before = incl - sum;
    if (before < want && want <= incl) {
        uint32_t acc = before;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            if (acc + cnt[i] >= want) { res[0] = (uint32_t)(top - i); res[1] = acc; res[2] = cnt[i]; break; }
            acc += cnt[i];
        }
    }
    __syncthreads();
    return (uint32_t)total >= want;
}

/* Largest i in [lo, hi) with f(i) <= x, for a non-decreasing f with f(lo) <= x; the whole
 * workgroup of 256 threads searches, 256 probes a round.  sh: one word of LDS. */
template <typename F>
__device__ __forceinline__ uint32_t wg_search_le(uint32_t lo, uint32_t hi, uint64_t x, F f, uint32_t *sh)
{
    while (hi - lo > 1) {
        const uint32_t step = (hi - lo + 255u) / 256u;
        const uint32_t p = lo + threadIdx.x * step, q = p + step;
        if (p < hi && f(p) <= x && (q >= hi || x < f(q))) *sh = p;
        __syncthreads();
        const uint32_t np = *sh;
        __syncthreads();
        lo = np;
        hi = np + step < hi ? np + step : hi;
    }
    return lo;
}

/* Inclusive prefix sum over the 64 lanes of a wavefront with data-parallel moves: shifts by 1, 2,
 * 4, 8 lanes inside each row of 16 (lanes shifted in from outside a row read 0), then lane 15 of
 * rows 0 and 2 added to rows 1 and 3, then lane 31 added to rows 2 and 3. */
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v)
{
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xF, 0xF, true);
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xF, 0xF, true);
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xF, 0xF, true);
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xF, 0xF, true);
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xA, 0xF, false);
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xC, 0xF, false);
    return v;
}

/* ------------------------------------------------------------------ k_select_count */

constexpr uint32_t SELC_WAVES = WG / 64;
constexpr uint32_t SELC_SEGS = SELC_WAVES * SEL_SEGS_PER_WAVE;     /* segments per workgroup of k_select_count */

/* Work list of k_select_count, fixed by the bucket layout: workgroup w takes segments
 * [x.y, x.z) of bucket x.x. */
__global__ __launch_bounds__(WG) void k_selmap(const uint32_t *__restrict__ sel0, const uint32_t *__restrict__ span0,
                                               uint32_t B, uint32_t n_sel, uint32_t segSh, uint4 *__restrict__ selw)
{
    const uint32_t w = blockIdx.x * WG + threadIdx.x;
    if (w >= n_sel) return;
    const uint32_t b = find_bucket<uint32_t>(sel0, B, w);
    const uint32_t seg_lo = span0[b] << segSh, seg_hi = span0[b + 1] << segSh;
    const uint32_t s0 = seg_lo + (w - sel0[b]) * SELC_SEGS;
    selw[w] = make_uint4(b, s0, min(seg_hi, s0 + SELC_SEGS), 0u);
}

/* chunk -> bucket, fixed by the layout and (ratio, bits) */
__global__ __launch_bounds__(WG) void k_chunkmap(const uint64_t *__restrict__ C, uint32_t B, uint64_t NC,
                                                 uint32_t *__restrict__ chunk_b)
{
    const uint64_t c = (uint64_t)blockIdx.x * WG + threadIdx.x;
    if (c < NC) chunk_b[c] = find_bucket<uint64_t>(C, B, c);
}

constexpr uint32_t LCAP = SELC_SEGS * 128;            /* list entries per workgroup of k_select_count */
/* a list entry: the 19 key bits below the level-0 digit, and above them the segment's number inside the workgroup */
__device__ __forceinline__ uint32_t list_entry(uint32_t key, uint32_t segl) { return (segl << SH0) | (key & ((1u << SH0) - 1u)); }

/* A staging segment that overflowed (more staged elements than a quarter of what it covers: its
 * count says so) is read from the dense accumulator instead: the elements its wavefront of the
 * streaming pass covered, in index order, minus the pruned ones.  This is their range. */
struct DenseSeg {
    uint64_t e0;         /* first element (global index) */
    uint32_t len;
};
__device__ __forceinline__ DenseSeg dense_seg(const Tables &t, uint32_t b, uint32_t ss)
{
    const uint32_t span = ss >> t.segSh, wv = ss & ((1u << t.segSh) - 1u);
    const SpanGeo s = span_geo_b(t, b, span - t.span0[b]);
    const uint32_t per = (t.spanT * 4u) >> t.segSh;
    const uint32_t wt0 = wv * per, wt1 = min(s.ntiles * 4u, wt0 + per);
    DenseSeg d;
    d.e0 = 0; d.len = 0;
    if (wt1 > wt0) {
        const uint64_t a = max(s.lo, s.base + (uint64_t)wt0 * WTILE), z = min(s.hi, s.base + (uint64_t)wt1 * WTILE);
        if (z > a) { d.e0 = a; d.len = (uint32_t)(z - a); }
    }
    return d;
}
/* whether element e (global index) of a bucket whose first tile is tile0b and starts at lo_al
 * (its offset rounded down to a multiple of 4) is pruned */
__device__ __forceinline__ bool pruned_elem(const uint32_t *__restrict__ pmask, uint32_t tile0b, uint64_t lo_al, uint64_t e)
{
    const uint64_t pos = e - lo_al;
    return (pmask[(uint64_t)(tile0b + (uint32_t)(pos / TILE)) * (TILE / 32) + (uint32_t)((pos % TILE) >> 5)] >> (pos & 31u)) & 1u;
}
struct DenseSrc {
    const float *r;              /* the dense accumulator */
    const uint32_t *pmask;       /* NULL: nothing is pruned */
    uint32_t tile0b;
    uint64_t lo_al;
};

/* One wavefront's four segments of k_select_count, GROUP lanes per segment (16: all four at
 * once, 64: one after the other).  mlen != 0 in the lane that describes a segment: the segment
 * overflowed and is read from the dense accumulator (me0, mlen). */
template <uint32_t GROUP, bool DENSE>      /* DENSE: some segment of this wavefront is read from the accumulator */
__device__ __forceinline__ void select_count_wave(const Cand &c, uint32_t b0, uint32_t sh, uint32_t wseg0, uint32_t mcnt,
                                                  uint64_t me0, uint32_t mlen, const DenseSrc &ds,
                                                  uint32_t segl0, uint32_t *lk, uint32_t *lcur,
                                                  uint32_t &my_g, uint32_t &my_b)
{
    constexpr uint32_t SPR = 64 / GROUP;             /* segments per round */
    constexpr uint32_t ROUNDS = SEL_SEGS_PER_WAVE / SPR;
    const uint32_t lane = threadIdx.x & 63, sub = lane / GROUP, gl = lane % GROUP;
    const uint32_t shift = sub * GROUP;
    const uint64_t below = (1ull << gl) - 1ull;
    const uint64_t gmask = GROUP == 64 ? ~0ull : ((1ull << (GROUP % 64)) - 1ull);
    uint32_t *cvalu = reinterpret_cast<uint32_t *>(c.val);
#pragma unroll
    for (uint32_t rd = 0; rd < ROUNDS; ++rd) {
        const uint32_t src = rd * SPR + sub;
        const uint32_t staged = __shfl(mcnt, src, 64);
        const uint32_t dlen = DENSE ? __shfl(mlen, src, 64) : 0u;
        const bool dense = DENSE && dlen != 0u;
        const uint64_t e0 = DENSE ? ((uint64_t)__shfl((uint32_t)(me0 >> 32), src, 64) << 32) | (uint64_t)__shfl((uint32_t)me0, src, 64) : 0ull;
        const uint32_t cnt = dense ? dlen : staged;
        uint32_t maxcnt = cnt;
#pragma unroll
        for (int d = 32; d >= (int)GROUP; d >>= 1) maxcnt = max(maxcnt, (uint32_t)__shfl_xor(maxcnt, d, 64));
        const uint64_t base = (uint64_t)(wseg0 + src) * c.cap;
        const float *p = dense ? ds.r + e0 : c.val + base;
        uint32_t run_g = 0, run_b = 0;
        for (uint32_t i0 = 0; i0 < maxcnt; i0 += 2 * CU * GROUP) {
            float x[2 * CU];
#pragma unroll
            for (uint32_t u = 0; u < 2 * CU; ++u) {
                const uint32_t i = i0 + u * GROUP + gl;
                x[u] = i < cnt ? p[i] : 0.0f;
            }
#pragma unroll
            for (uint32_t u = 0; u < 2 * CU; ++u) {
                const uint32_t key = keyof(x[u]);
                const uint32_t i = i0 + u * GROUP + gl;
                bool in = i < cnt;
                if (dense && ds.pmask && in) in = !pruned_elem(ds.pmask, ds.tile0b, ds.lo_al, e0 + i);
                const bool isg = in && (key >> sh) > b0, isb = in && (key >> sh) == b0;
                const uint64_t ball = __ballot(isb);
                const uint64_t bg = (__ballot(isg) >> shift) & gmask;
                const uint64_t bb = (ball >> shift) & gmask;
                if (ball) {
                    /* undecided keys: to the tail of the segment's area (last slot first) and to the
                     * workgroup's list, whose slots are handed out per wavefront */
                    uint32_t lbase = 0;
                    if (lane == 0) lbase = atomicAdd(lcur, (uint32_t)__popcll(ball));
                    lbase = __builtin_amdgcn_readfirstlane(lbase);
                    if (isb) {
                        const uint32_t pos = run_b + __popcll(bb & below);
                        if (!dense && cnt + pos < c.cap) cvalu[base + c.cap - 1u - pos] = key;
                        const uint32_t lp = lbase + __popcll(ball & ((1ull << lane) - 1ull));
                        if (lp < LCAP) lk[lp] = list_entry(key, segl0 + src);
                    }
                }
                run_g += __popcll(bg);
                run_b += __popcll(bb);
            }
        }
        /* segment rd * SPR + j was counted by the group of lanes starting at j * GROUP */
        const uint32_t from = (lane % SPR) * GROUP;
        const uint32_t got_g = __shfl(run_g, from, 64), got_b = __shfl(run_b, from, 64);
        if (lane / SPR == rd) { my_g = got_g; my_b = got_b; }
    }
}

/* Per staging segment of the buckets decided from staged elements (PATH_CAND, PATH_BAND), with
 * b0 the level-0 digit of the bucket's k-th key: G = entries above digit b0 (plus, in band mode,
 * the elements above the band the streaming pass counted), E = entries inside digit b0.  The keys of those undecided entries go to two places: the unused tail of the segment's
 * staging area, last slot first (as long as there is room), and a list per workgroup (the
 * undecided key bits and the segment's number in one word, in no particular order) that k_select_finish reads with coalesced loads; the
 * list is left out (lcnt = NONE) when the workgroup has more than LCAP of them.
 * A workgroup takes 16 consecutive segments, a wavefront four of them, with 16 lanes per
 * segment, or all 64 on one segment after the other when a segment is long. */
__global__ __launch_bounds__(WG) void k_select_count(Tables t, Cand c, const uint4 *__restrict__ selw,
                                                     uint32_t *__restrict__ tail_ovf, uint32_t *__restrict__ lcnt,
                                                     uint32_t *__restrict__ lkey, const float *__restrict__ r)
{
    __shared__ uint32_t lk[LCAP];
    __shared__ uint32_t lcur;
    const uint4 wk = selw[blockIdx.x];
    const uint32_t b = wk.x, s0 = wk.y, s1 = wk.z;
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t wseg0 = s0 + wave * SEL_SEGS_PER_WAVE;
    /* lane l < 4 describes segment wseg0 + l; issued before the bucket's state is known */
    const uint32_t ms = wseg0 + (lane & (SEL_SEGS_PER_WAVE - 1));
    const bool mine = lane < SEL_SEGS_PER_WAVE && ms < s1;
    const uint32_t mcnt = mine ? c.cnt[ms] : 0u;
    uint32_t mg0 = mine ? c.G[ms] : 0u;              /* band mode: elements above the band, counted by the streaming pass */
    const uint32_t path = t.fast[b], b0 = t.T[b], sh = t.sh[b];     /* b0: the key bits from position sh up */
    if (path != PATH_CAND && path != PATH_BAND) return;      /* same for the whole workgroup */
    if (t.H[b] == NONE) mg0 = 0u;                    /* no band was staged: nothing was counted above it */
    if (tid == 0) lcur = 0u;
    __syncthreads();
    /* an overflowed segment is read from the dense accumulator, where nothing is missing */
    uint64_t me0 = 0;
    uint32_t mlen = 0;
    if (mine && mcnt > c.cap) {
        const DenseSeg d = dense_seg(t, b, ms);
        me0 = d.e0; mlen = d.len;
        mg0 = 0u;                                    /* its elements above the band are counted here as well */
    }
    DenseSrc ds;
    ds.r = r; ds.pmask = t.pmask; ds.tile0b = t.tile0[b]; ds.lo_al = t.off[b] & ~3ull;
    uint32_t mx = mlen ? mlen : mcnt;
#pragma unroll
    for (int d = 2; d >= 1; d >>= 1) mx = max(mx, (uint32_t)__shfl_xor(mx, d, 64));
    mx = __builtin_amdgcn_readfirstlane(mx);
    uint32_t my_g = 0, my_b = 0;
    if (__any(mlen != 0u)) {
        if (mx > 2 * CU * 16) select_count_wave<64, true>(c, b0, sh, wseg0, mcnt, me0, mlen, ds, wave * SEL_SEGS_PER_WAVE, lk, &lcur, my_g, my_b);
        else if (mx) select_count_wave<16, true>(c, b0, sh, wseg0, mcnt, me0, mlen, ds, wave * SEL_SEGS_PER_WAVE, lk, &lcur, my_g, my_b);
    } else {
        if (mx > 2 * CU * 16) select_count_wave<64, false>(c, b0, sh, wseg0, mcnt, me0, mlen, ds, wave * SEL_SEGS_PER_WAVE, lk, &lcur, my_g, my_b);
        else if (mx) select_count_wave<16, false>(c, b0, sh, wseg0, mcnt, me0, mlen, ds, wave * SEL_SEGS_PER_WAVE, lk, &lcur, my_g, my_b);
    }
    if (mine) {
        c.G[ms] = mg0 + my_g;
        c.E[ms] = my_b;
        /* a tail that did not fit (or a segment without one): k_select_finish filters the entries again
         * if it cannot use the lists */
        if (my_b != 0u && (mlen != 0u || mcnt + my_b > c.cap)) tail_ovf[b] = 1u;
    }
    __syncthreads();
    const uint32_t total = lcur;
    if (tid == 0) lcnt[blockIdx.x] = total > LCAP ? NONE : total;
    if (total <= LCAP) {
        const uint64_t lb = (uint64_t)blockIdx.x * LCAP;
        for (uint32_t i = tid; i < total; i += WG) lkey[lb + i] = lk[i];
    }
}

/* ------------------------------------------------------------------ k_select_finish */

/* The undecided keys of one segment: the tail list k_select_count wrote, or, when some tail did
 * not fit (`rescan`), the segment's staged entries filtered again. */
struct KeySource {
    const uint32_t *cvalu;
    const uint32_t *cnt;
    uint32_t cap, b0, sh;
    bool rescan;
    const Tables *t;             /* for the segments that overflowed: they are read from the dense accumulator */
    const float *r;
    uint32_t b;
    __device__ __forceinline__ bool wanted(uint32_t key) const { return !rescan || (key >> sh) == b0; }
    /* f(key) for every undecided key of segment s, eight loads in flight at a time */
    template <typename F>
    __device__ __forceinline__ void for_each(uint32_t s, uint32_t bcnt, F f) const
    {
        const uint32_t staged = cnt[s];
        if (rescan && staged > cap) {
            const DenseSeg d = dense_seg(*t, b, s);
            const uint32_t tile0b = t->tile0[b];
            const uint64_t lo_al = t->off[b] & ~3ull;
            for (uint32_t i = 0; i < d.len; i += 8) {
                uint32_t kk[8];
#pragma unroll
                for (uint32_t u = 0; u < 8; ++u) kk[u] = i + u < d.len ? keyof(r[d.e0 + i + u]) : 0u;
#pragma unroll
                for (uint32_t u = 0; u < 8; ++u)
                    if (i + u < d.len && wanted(kk[u]) && !(t->pmask && pruned_elem(t->pmask, tile0b, lo_al, d.e0 + i + u))) f(kk[u]);
            }
            return;
        }
        const uint32_t nw = rescan ? staged : bcnt;
        const uint64_t base = (uint64_t)s * cap;
        for (uint32_t i = 0; i < nw; i += 8) {
            uint32_t kk[8];
#pragma unroll
            for (uint32_t u = 0; u < 8; ++u)
                kk[u] = i + u < nw ? (rescan ? (cvalu[base + i + u] & 0x7FFFFFFFu) : cvalu[base + cap - 1u - (i + u)]) : 0u;
#pragma unroll
            for (uint32_t u = 0; u < 8; ++u)
                if (i + u < nw && wanted(kk[u])) f(kk[u]);
        }
    }
};

/* LDS of k_select_finish, one pool carved by both variants below (u32 words):
 *   [0, 4096)        level-1 histogram; later, with [4096, 8192), the per-segment counts (lists) /
 *   [4096, 8192)     per-segment key counts as u16 (tails)
 *   [8192, 11264)    undecided keys kept in LDS
 *   [11264, 12800)   their segment numbers as u16 (lists)
 *   [12800, 13826)   exclusive prefix of the list lengths (lists) */
constexpr uint32_t FIN_POOL = 13826;
constexpr uint32_t FIN_KEYS_LDS = 3072;    /* undecided keys kept in LDS */
constexpr uint32_t FIN_MAX_SEGS = 8192;    /* segments whose counts fit the pool */
constexpr uint32_t RQ = FIN_MAX_SEGS / SEL_THREADS;

struct FinShared {
    uint32_t *pool;      /* FIN_POOL words */
    uint32_t *h2;        /* NB2 */
    uint64_t *tmp;       /* SEL_WAVES */
    uint32_t *res;       /* 4 */
};

/* Last part of both variants: exclusive prefixes of (elements above T, elements equal to T) over
 * the bucket's segments, in place over the per-segment counts, and for every chunk of the
 * payload the segment that holds its first survivor.  count(r, s, g, q) adds to g and q what
 * segment s (round r) holds above / equal to T among its undecided keys. */
template <typename F>
__device__ __forceinline__ void finish_prefixes(const Tables &t, const Cand &c, uint32_t b, uint32_t seg_lo,
                                                uint32_t seg_hi, uint32_t T, uint32_t e_b, uint32_t kb,
                                                uint32_t *__restrict__ chunk_seg, uint64_t *tmp,
                                                uint32_t *__restrict__ err, F count)
{
    const uint32_t tid = threadIdx.x;
    const uint32_t rounds = (seg_hi - seg_lo + SEL_THREADS - 1) / SEL_THREADS;
    const uint64_t Cb = t.C[b];
    const uint32_t chunk = t.chunk;
    uint64_t run = 0;
    uint32_t g_next = seg_lo + tid < seg_hi ? c.G[seg_lo + tid] : 0u;
    for (uint32_t r = 0; r < rounds; ++r) {
        const uint32_t s = seg_lo + r * SEL_THREADS + tid;
        const bool in = s < seg_hi;
        uint32_t g = g_next, q = 0;
        if (r + 1 < rounds) g_next = s + SEL_THREADS < seg_hi ? c.G[s + SEL_THREADS] : 0u;   /* fetched under this round's work */
        count(r, s, g, q);
        const uint64_t v = ((uint64_t)g << 32) | (uint64_t)q;
        uint64_t tt;
        const uint64_t incl = block_incl_scan64<SEL_WAVES>(v, tmp, tt);
        const uint64_t excl = run + incl - v;
        if (in) {
            const uint32_t Gp = (uint32_t)(excl >> 32), Ep = (uint32_t)excl;
            c.G[s] = Gp;
            c.E[s] = Ep;
            /* survivors of this segment have ranks [r0, r1): the chunks that start among them */
            const uint64_t r0 = (uint64_t)Gp + min(e_b, Ep);
            const uint64_t r1 = (uint64_t)Gp + g + min((uint64_t)e_b, (uint64_t)Ep + q);
            if (chunk_seg)                           /* not for the weight stage: its ranks are no payload positions */
                for (uint64_t cb = (r0 + chunk - 1) / chunk; cb * chunk < r1; ++cb) chunk_seg[Cb + cb] = s;
        }
        run += tt;
    }
    if (tid == 0) {
        t.T[b] = T;
        t.need[b] = e_b;
        /* above + admitted ties must be exactly k */
        const uint32_t above = (uint32_t)(run >> 32), ties = (uint32_t)run;
        if (above + e_b != kb || e_b > ties) err[0] = 1u;
    }
}

/* Variant 1 (the usual one): the undecided keys come from the lists of the bucket's
 * k_select_count workgroups ("units"), read with coalesced loads, eight per thread in flight.
 * Two passes over them when they do not fit in LDS: level-1 digits; then, knowing the level-1
 * digit d1 of the threshold, everything above d1 is tallied per segment at once and the few
 * keys inside d1 are set aside in LDS for the last 7 bits. */
__device__ __forceinline__ void finish_from_lists(const Tables &t, const Cand &c, uint32_t b, uint32_t b0, uint32_t sh,
                                                  uint32_t need0, uint32_t kb, uint32_t seg_lo, uint32_t seg_hi,
                                                  uint32_t u0, uint32_t nun, uint32_t my_cnt,
                                                  const uint32_t *__restrict__ lkey,
                                                  uint32_t *__restrict__ chunk_seg, const FinShared &sm,
                                                  uint32_t *__restrict__ err)
{
    const uint32_t tid = threadIdx.x;
    uint32_t *h1 = sm.pool, *cnts = sm.pool, *keys = sm.pool + 8192, *uoff = sm.pool + 12800;
    uint16_t *segs = reinterpret_cast<uint16_t *>(sm.pool + 11264);
    for (uint32_t i = tid; i < NB1; i += SEL_THREADS) h1[i] = 0u;
    if (tid < NB2) sm.h2[tid] = 0u;
    if (tid == 0) sm.res[3] = 0u;                      /* entries set aside */
    uint64_t tot64;
    const uint32_t incl = (uint32_t)block_incl_scan64<SEL_WAVES>((uint64_t)my_cnt, sm.tmp, tot64);
    if (tid < nun) uoff[tid] = incl - my_cnt;
    if (tid == 0) uoff[nun] = (uint32_t)tot64;
    __syncthreads();
    const uint32_t nkeys = (uint32_t)tot64;
    const bool resident = nkeys <= FIN_KEYS_LDS;
    const uint32_t m1 = (1u << (sh - SH1)) - 1u;       /* level-1 digit: key bits sh-1 .. 7 (12 or 6 bits) */
    /* f(i, entry, segment number inside the bucket) for every list entry of the bucket */
    auto for_keys = [&](auto f) {
        for (uint32_t i0 = tid; i0 < nkeys; i0 += 8 * SEL_THREADS) {
            uint32_t kk[8], un[8];
#pragma unroll
            for (uint32_t u = 0; u < 8; ++u) {
                const uint32_t i = i0 + u * SEL_THREADS;
                kk[u] = 0; un[u] = 0;
                if (i < nkeys) {
                    uint32_t lo = 0, hi = nun;         /* uoff[lo] <= i < uoff[hi] */
                    while (hi - lo > 1) { const uint32_t mid = (lo + hi) >> 1; if (uoff[mid] <= i) lo = mid; else hi = mid; }
                    un[u] = lo;
                    kk[u] = lkey[(uint64_t)(u0 + lo) * LCAP + (i - uoff[lo])];
                }
            }
#pragma unroll
            for (uint32_t u = 0; u < 8; ++u)
                if (i0 + u * SEL_THREADS < nkeys) f(i0 + u * SEL_THREADS, kk[u], un[u] * SELC_SEGS + (kk[u] >> SH0));
        }
    };
    /* pass 1: level-1 digits (key bits 18..7); entries and segment numbers to LDS if they fit */
    for_keys([&](uint32_t i, uint32_t e, uint32_t seg) {
        atomicAdd(&h1[(e >> SH1) & m1], 1u);
        if (resident) { keys[i] = e; segs[i] = (uint16_t)seg; }
    });
    __syncthreads();
    if (!find_digit_lds<NB1, SEL_WAVES>(h1, need0, sm.tmp, sm.res)) { if (tid == 0) err[0] = 1u; return; }
    const uint32_t d1 = sm.res[0];
    const uint32_t need1 = need0 - sm.res[1];
    __syncthreads();
    /* pass 2: per segment, entries above digit d1 (high half of the count); level-2 digits (key
     * bits 6..0) of the entries inside d1, which are set aside when they came from memory */
    const uint32_t nseg = seg_hi - seg_lo;
    for (uint32_t i = tid; i < nseg; i += SEL_THREADS) cnts[i] = 0u;       /* takes the place of the level-1 histogram */
    __syncthreads();
    auto pass2 = [&](uint32_t e, uint32_t seg, bool collect) {
        const uint32_t d = (e >> SH1) & m1;
        if (d > d1) atomicAdd(&cnts[seg], 1u << 16);
        else if (d == d1) {
            atomicAdd(&sm.h2[e & (NB2 - 1)], 1u);
            if (collect) {
                const uint32_t at = atomicAdd(&sm.res[3], 1u);
                if (at < FIN_KEYS_LDS) { keys[at] = e; segs[at] = (uint16_t)seg; }
            }
        }
    };
    if (resident) {
        for (uint32_t i = tid; i < nkeys; i += SEL_THREADS) pass2(keys[i], segs[i], false);
    } else {
        for_keys([&](uint32_t, uint32_t e, uint32_t seg) { pass2(e, seg, true); });
    }
    __syncthreads();
    if (!find_digit_lds<NB2, SEL_WAVES>(sm.h2, need1, sm.tmp, sm.res)) { if (tid == 0) err[0] = 1u; return; }
    const uint32_t d2 = sm.res[0];
    const uint32_t T = (b0 << sh) | (d1 << SH1) | d2;
    const uint32_t e_b = need1 - sm.res[1];            /* ties admitted: 1 <= e_b <= keys equal to T */
    const uint32_t aside = sm.res[3];
    __syncthreads();
    /* pass 3: the entries inside d1 against the last digit: above T, or equal to T (low half) */
    auto pass3 = [&](uint32_t e, uint32_t seg) {
        if (((e >> SH1) & m1) != d1) return;
        const uint32_t d = e & (NB2 - 1);
        if (d > d2) atomicAdd(&cnts[seg], 1u << 16);
        else if (d == d2) atomicAdd(&cnts[seg], 1u);
    };
    if (resident) {
        for (uint32_t i = tid; i < nkeys; i += SEL_THREADS) pass3(keys[i], segs[i]);
    } else if (aside <= FIN_KEYS_LDS) {
        for (uint32_t i = tid; i < aside; i += SEL_THREADS) pass3(keys[i], segs[i]);
    } else {
        for_keys([&](uint32_t, uint32_t e, uint32_t seg) { pass3(e, seg); });      /* too many were inside d1 */
    }
    __syncthreads();
    finish_prefixes(t, c, b, seg_lo, seg_hi, T, e_b, kb, chunk_seg, sm.tmp, err,
                    [&](uint32_t, uint32_t s, uint32_t &g, uint32_t &q) {
                        if (s < seg_hi) { const uint32_t v = cnts[s - seg_lo]; g += v >> 16; q += v & 0xFFFFu; }
                    });
}

/* Variant 2: the undecided keys of a segment come from the tail of its staging area, or, when
 * some tail did not fit (`rescan`), from the staged entries filtered again; one thread per
 * segment.  Taken when a list was left out (a workgroup with more than LCAP undecided keys) or
 * the bucket has more segments than the LDS tables of variant 1 hold; slower, same result. */
__device__ __forceinline__ void finish_from_tails(const Tables &t, const Cand &c, uint32_t b, uint32_t b0, uint32_t sh,
                                                  uint32_t need0, uint32_t kb, uint32_t seg_lo, uint32_t seg_hi,
                                                  bool rescan, uint32_t *__restrict__ chunk_seg,
                                                  const FinShared &sm, uint32_t *__restrict__ err,
                                                  const float *__restrict__ r)
{
    const uint32_t tid = threadIdx.x;
    uint32_t *h1 = sm.pool, *keys = sm.pool + 8192;
    uint16_t *sbc = reinterpret_cast<uint16_t *>(sm.pool + 4096);
    KeySource ks;
    ks.cvalu = reinterpret_cast<const uint32_t *>(c.val); ks.cnt = c.cnt; ks.cap = c.cap; ks.b0 = b0; ks.sh = sh;
    ks.rescan = rescan; ks.t = &t; ks.r = r; ks.b = b;
    const uint32_t m1 = (1u << (sh - SH1)) - 1u;       /* level-1 digit: key bits sh-1 .. 7 */
    const uint32_t rounds = (seg_hi - seg_lo + SEL_THREADS - 1) / SEL_THREADS;
    for (uint32_t i = tid; i < NB1; i += SEL_THREADS) h1[i] = 0u;
    if (tid < NB2) sm.h2[tid] = 0u;
    for (uint32_t r = 0; r < RQ; ++r) {
        const uint32_t s = seg_lo + r * SEL_THREADS + tid;
        sbc[r * SEL_THREADS + tid] = (uint16_t)((r < rounds && s < seg_hi) ? c.E[s] : 0u);
    }
    auto bc_of = [&](uint32_t r, uint32_t s) -> uint32_t {
        return r < RQ ? (uint32_t)sbc[r * SEL_THREADS + tid] : (s < seg_hi ? c.E[s] : 0u);
    };
    uint64_t tot64;
    {
        uint32_t mine = 0;
        for (uint32_t r = 0; r < rounds; ++r) mine += bc_of(r, seg_lo + r * SEL_THREADS + tid);
        block_incl_scan64<SEL_WAVES>((uint64_t)mine, sm.tmp, tot64);
    }
    const bool resident = !ks.rescan && tot64 <= (uint64_t)FIN_KEYS_LDS;
    const uint32_t nkeys = (uint32_t)tot64;
    uint32_t carry = 0;
    for (uint32_t r = 0; r < rounds; ++r) {
        const uint32_t s = seg_lo + r * SEL_THREADS + tid;
        const uint32_t bc = bc_of(r, s);
        uint32_t off = 0;
        if (resident) {
            uint64_t tt;
            off = carry + (uint32_t)block_incl_scan64<SEL_WAVES>((uint64_t)bc, sm.tmp, tt) - bc;
            carry += (uint32_t)tt;
        }
        uint32_t kept = 0;
        if (s < seg_hi)
            ks.for_each(s, bc, [&](uint32_t key) {
                atomicAdd(&h1[(key >> SH1) & m1], 1u);
                if (resident) keys[off + kept] = key;
                ++kept;
            });
    }
    __syncthreads();
    if (!find_digit_lds<NB1, SEL_WAVES>(h1, need0, sm.tmp, sm.res)) { if (tid == 0) err[0] = 1u; return; }
    const uint32_t prefix24 = (b0 << (sh - SH1)) | sm.res[0];     /* the key bits from position 7 up */
    const uint32_t need1 = need0 - sm.res[1];
    __syncthreads();
    if (resident) {
        for (uint32_t i = tid; i < nkeys; i += SEL_THREADS) {
            const uint32_t key = keys[i];
            if ((key >> SH1) == prefix24) atomicAdd(&sm.h2[key & (NB2 - 1)], 1u);
        }
    } else {
        for (uint32_t r = 0; r < rounds; ++r) {
            const uint32_t s = seg_lo + r * SEL_THREADS + tid;
            if (s < seg_hi)
                ks.for_each(s, bc_of(r, s), [&](uint32_t key) {
                    if ((key >> SH1) == prefix24) atomicAdd(&sm.h2[key & (NB2 - 1)], 1u);
                });
        }
    }
    __syncthreads();
    if (!find_digit_lds<NB2, SEL_WAVES>(sm.h2, need1, sm.tmp, sm.res)) { if (tid == 0) err[0] = 1u; return; }
    const uint32_t T = (prefix24 << 7) | sm.res[0];
    const uint32_t e_b = need1 - sm.res[1];
    __syncthreads();
    carry = 0;
    finish_prefixes(t, c, b, seg_lo, seg_hi, T, e_b, kb, chunk_seg, sm.tmp, err,
                    [&](uint32_t r, uint32_t s, uint32_t &g, uint32_t &q) {
                        const uint32_t bc = bc_of(r, s);
                        if (resident) {
                            uint64_t tt;
                            const uint32_t off = carry + (uint32_t)block_incl_scan64<SEL_WAVES>((uint64_t)bc, sm.tmp, tt) - bc;
                            carry += (uint32_t)tt;
                            for (uint32_t i = 0; i < bc; ++i) {
                                const uint32_t key = keys[off + i];
                                g += key > T ? 1u : 0u;
                                q += key == T ? 1u : 0u;
                            }
                        } else if (s < seg_hi) {
                            ks.for_each(s, bc, [&](uint32_t key) {
                                g += key > T ? 1u : 0u;
                                q += key == T ? 1u : 0u;
                            });
                        }
                    });
}

/* One workgroup of 1024 threads per bucket decided from staged elements: the threshold key T and
 * the tie allowance e from the few undecided keys (12 + 7 remaining bits, histograms in LDS),
 * then every segment's place in the survivor order.  PATH_ZERO buckets arrive with T = 0 and e
 * known and only get the prefixes. */
__global__ __launch_bounds__(SEL_THREADS) void k_select_finish(Tables t, Cand c, const uint32_t *__restrict__ sel0,
                                                               uint32_t *__restrict__ tail_ovf,
                                                               const uint32_t *__restrict__ lcnt,
                                                               const uint32_t *__restrict__ lkey,
                                                               uint32_t *__restrict__ chunk_seg,
                                                               uint32_t *__restrict__ err, int force_rescan,
                                                               const float *__restrict__ r)
{
    __shared__ uint32_t pool[FIN_POOL];
    __shared__ uint32_t h2[NB2];
    __shared__ uint64_t tmp[SEL_WAVES];
    __shared__ uint32_t res[4];
    const uint32_t b = blockIdx.x, tid = threadIdx.x;
    const uint32_t path = t.fast[b], kb = t.k[b];
    const uint32_t u0 = sel0[b], u1 = sel0[b + 1];
    const uint32_t ovf = tail_ovf[b];
    if (tid == 0 && ovf) tail_ovf[b] = 0u;           /* left clean for the next call */
    /* this unit's list length, fetched before the bucket's state is known */
    const uint32_t my_cnt = (tid < u1 - u0 && tid < SEL_THREADS) ? lcnt[u0 + tid] : 0u;
    if (path == PATH_DENSE || kb == 0u) return;
    const uint32_t seg_lo = t.span0[b] << t.segSh, seg_hi = t.span0[b + 1] << t.segSh;
    const uint32_t b0 = t.T[b];                      /* the key bits from position sh up; PATH_ZERO: the full key (0) */
    const uint32_t need0 = t.need[b], sh = t.sh[b];
    FinShared sm;
    sm.pool = pool; sm.h2 = h2; sm.tmp = tmp; sm.res = res;
    if (path == PATH_ZERO) {
        /* the streaming pass counted non-zero (G) and zero (E) keys per segment; when a band from
         * key 1 up was staged as well, G holds the keys above the band and the staged ones add to it */
        const bool mixed = t.L[b] != t.H[b];
        finish_prefixes(t, c, b, seg_lo, seg_hi, 0u, need0, kb, chunk_seg, tmp, err,
                        [&](uint32_t, uint32_t s, uint32_t &g, uint32_t &q) {
                            if (s < seg_hi) { q += c.E[s]; if (mixed) g += c.cnt[s]; }
                        });
        return;
    }
    const uint32_t nun = u1 - u0;
    const int no_list = __syncthreads_or(my_cnt == NONE);
    /* the lists hold every undecided key whenever none of them was left out; the tails are the
     * fallback, and when a tail did not fit either (or a segment has none: it overflowed), the
     * segments are filtered again */
    if (no_list || force_rescan || nun > SEL_THREADS || seg_hi - seg_lo > FIN_MAX_SEGS)
        finish_from_tails(t, c, b, b0, sh, need0, kb, seg_lo, seg_hi, ovf != 0u || force_rescan, chunk_seg, sm, err, r);
    else
        finish_from_lists(t, c, b, b0, sh, need0, kb, seg_lo, seg_hi, u0, nun, my_cnt, lkey, chunk_seg, sm, err);
}

/* ------------------------------------------------------------------ k_encode */

/* The segments whose descriptions sit in LDS (mc entries, mg / me running counts before them),
 * numbers 0 .. m-1 of the block that starts at segment sblk: their survivors with ranks in
 * [j0, j0 + n) go to sv / si.  GROUP lanes work on one segment at a time; returns how many
 * survivors this thread placed. */
template <uint32_t GROUP>
__device__ __forceinline__ uint32_t gather_block(const Cand &c, uint32_t sblk, uint32_t m, uint32_t T, uint32_t e_b,
                                                 uint32_t j0, uint32_t n, float *sv, uint32_t *si,
                                                 const uint32_t *mc, const uint32_t *mg, const uint32_t *me)
{
    constexpr uint32_t SPR = 64 / GROUP;
    constexpr uint32_t SLOTS = (WG / 64) * SPR;      /* segments the workgroup works on at a time */
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6, sub = lane / GROUP, gl = lane % GROUP;
    const uint32_t shift = sub * GROUP;
    const uint64_t below = (1ull << gl) - 1ull;
    const uint64_t gmask = GROUP == 64 ? ~0ull : ((1ull << (GROUP % 64)) - 1ull);
    uint32_t got = 0;
    /* the first batch of entries of a segment is fetched while the previous segment is worked on */
    auto first_batch = [&](uint32_t q, float (&x)[CU], uint32_t (&li)[CU]) {
        const uint32_t cnt = q < m ? mc[q] : 0u;
        const uint64_t base = (uint64_t)(sblk + q) * c.cap;
#pragma unroll
        for (uint32_t u = 0; u < CU; ++u) {
            const uint32_t i = u * GROUP + gl;
            x[u] = i < cnt ? c.val[base + i] : 0.0f;
            li[u] = i < cnt ? c.idx[base + i] : 0u;
        }
    };
    const uint32_t qend = ((m + SLOTS - 1) / SLOTS) * SLOTS;
    float xn[CU];
    uint32_t lin[CU];
    first_batch(wave * SPR + sub, xn, lin);
    for (uint32_t q = wave * SPR + sub; q < qend; q += SLOTS) {
        const bool live = q < m;
        const uint32_t cnt = live ? mc[q] : 0u;
        uint32_t run_g = live ? mg[q] : 0u, run_e = live ? me[q] : 0u;
        uint32_t maxcnt = cnt;
#pragma unroll
        for (int d = 32; d >= (int)GROUP; d >>= 1) maxcnt = max(maxcnt, (uint32_t)__shfl_xor(maxcnt, d, 64));
        const uint64_t base = (uint64_t)(sblk + q) * c.cap;
        float x[CU];
        uint32_t li[CU];
#pragma unroll
        for (uint32_t u = 0; u < CU; ++u) { x[u] = xn[u]; li[u] = lin[u]; }
        if (q + SLOTS < qend) first_batch(q + SLOTS, xn, lin);
        for (uint32_t i0 = 0; i0 < maxcnt; i0 += CU * GROUP) {
            if (i0 != 0) {
#pragma unroll
                for (uint32_t u = 0; u < CU; ++u) {
                    const uint32_t i = i0 + u * GROUP + gl;
                    x[u] = i < cnt ? c.val[base + i] : 0.0f;
                    li[u] = i < cnt ? c.idx[base + i] : 0u;
                }
            }
#pragma unroll
            for (uint32_t u = 0; u < CU; ++u) {
                const uint32_t key = keyof(x[u]);
                const bool in = i0 + u * GROUP + gl < cnt;
                const bool isg = in && key > T, ise = in && key == T;
                const uint64_t bg = (__ballot(isg) >> shift) & gmask;
                const uint64_t be = (__ballot(ise) >> shift) & gmask;
                const uint32_t pg = run_g + __popcll(bg & below), pe = run_e + __popcll(be & below);
                if (isg || (ise && pe < e_b)) {
                    const uint64_t slot = (uint64_t)pg + (uint64_t)min(e_b, pe) - (uint64_t)j0;   /* wraps below j0 */
                    if (slot < (uint64_t)n) { sv[slot] = x[u]; si[slot] = li[u]; ++got; }
                }
                run_g += __popcll(bg);
                run_e += __popcll(be);
            }
        }
    }
    return got;
}

/* Gather survivors number [j0, j0 + n) of a PATH_CAND bucket (n <= ENC_BLK), in index order,
 * into LDS: sv their accumulator values, si their bucket-local indices; sA = the segment that
 * holds survivor j0.  Survivor ranks come from the per-segment prefixes k_select_finish left: an
 * entry above T, or an admitted tie, has rank G + min(e, E), with G / E the running counts of
 * entries above / equal to T before it.  The descriptions of up to 256 segments are fetched in
 * one go into LDS (mc, mg, me); how many lanes then share a segment follows the longest of them. */
__device__ __forceinline__ void gather_survivors(const Cand &c, uint32_t sA, uint32_t seg_hi, uint32_t T,
                                                 uint32_t e_b, uint32_t j0, uint32_t n, float *sv, uint32_t *si,
                                                 uint32_t *mc, uint32_t *mg, uint32_t *me, uint32_t *mxc,
                                                 uint32_t *filled)
{
    const uint32_t tid = threadIdx.x, lane = tid & 63;
    const uint64_t jend = (uint64_t)j0 + n;
    uint32_t got = 0;
    for (uint32_t sblk = sA; sblk < seg_hi; sblk += WG) {
        /* descriptions of segments sblk .. sblk + 255; the ones whose first survivor lies before
         * jend form a prefix of them */
        const uint32_t s = sblk + tid;
        uint32_t d_c = 0, d_g = 0, d_e = 0;
        if (s < seg_hi) { d_c = c.cnt[s]; d_g = c.G[s]; d_e = c.E[s]; }
        __syncthreads();                             /* the previous block's descriptions are consumed */
        mc[tid] = d_c; mg[tid] = d_g; me[tid] = d_e;
        if (tid == 0) *mxc = 0u;
        const bool need = s < seg_hi && (uint64_t)d_g + min(e_b, d_e) < jend;
        const uint32_t m = __syncthreads_count(need);
        if (need && d_c) atomicMax(mxc, d_c);
        __syncthreads();
        const uint32_t longest = *mxc;
        if (longest > 8 * CU * 4) got += gather_block<64>(c, sblk, m, T, e_b, j0, n, sv, si, mc, mg, me);
        else if (longest > 2 * CU * 4) got += gather_block<16>(c, sblk, m, T, e_b, j0, n, sv, si, mc, mg, me);
        else got += gather_block<4>(c, sblk, m, T, e_b, j0, n, sv, si, mc, mg, me);
        if (m < WG) break;                           /* same value in every thread */
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) got += __shfl_xor(got, d, 64);
    if (lane == 0 && got) atomicAdd(filled, got);
}

/* One workgroup per chunk of `chunk` consecutive survivors of a PATH_CAND bucket: gather,
 * absmax, scale, codes, packing, indices, and the coding error left in the residual.  Every
 * floating-point step is a single correctly rounded binary32 operation.  A chunk longer than
 * ENC_BLK is gathered block by block, once for its absmax and once more for the codes. */
template <int BITS>
__global__ __launch_bounds__(WG) void k_encode(Tables t, Cand c, const uint32_t *__restrict__ chunk_b,
                                               const uint32_t *__restrict__ chunk_seg, float *__restrict__ r,
                                               uint32_t *__restrict__ idx_out, void *__restrict__ val,
                                               float *__restrict__ scales, uint32_t *__restrict__ err,
                                               uint64_t n_chunks, uint32_t cpw)
{
    __shared__ float sv[ENC_BLK];
    __shared__ uint32_t si[ENC_BLK];
    __shared__ uint32_t mc[WG], mg[WG], me[WG];
    __shared__ float red[WG / 64];
    __shared__ uint32_t sh, filled, mxc;
    constexpr float QMAX = BITS == 8 ? 127.0f : 7.0f;
    const uint32_t tid = threadIdx.x;
    /* a workgroup takes cpw consecutive chunks (one, unless the payload has very many) */
    const uint64_t cend = min(n_chunks, ((uint64_t)blockIdx.x + 1) * cpw);
    if (cpw > 1) {
        /* all of them in one bucket that is not coded here: nothing to do */
        const uint32_t bf = chunk_b[(uint64_t)blockIdx.x * cpw], bl = chunk_b[cend - 1];
        if (bf == bl && t.fast[bf] != PATH_CAND) return;
    }
    for (uint64_t cid = (uint64_t)blockIdx.x * cpw; cid < cend; ++cid) {
    const uint32_t b = chunk_b[cid];
    const uint32_t sFirst = chunk_seg[cid];          /* meaningful for PATH_CAND buckets only */
    if (t.fast[b] != PATH_CAND) continue;
    const uint64_t cb = cid - t.C[b];
    const uint64_t j0c = cb * t.chunk;                         /* first survivor of the chunk, bucket-local */
    const uint32_t cnt_c = (uint32_t)min((uint64_t)t.chunk, (uint64_t)t.k[b] - j0c);
    const uint32_t T = t.T[b], e_b = t.need[b];
    const uint32_t seg_lo = t.span0[b] << t.segSh, seg_hi = t.span0[b + 1] << t.segSh;
    const uint64_t lo = t.off[b], Pb = t.P[b];
    uint8_t *vb = reinterpret_cast<uint8_t *>(val) + t.V[b];

    auto block_absmax = [&](uint32_t n) {
        float m = 0.0f;
        for (uint32_t i = tid; i < n; i += WG) m = fmaxf(m, fabsf(sv[i]));
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) m = fmaxf(m, __shfl_xor(m, d, 64));
        __syncthreads();
        if ((tid & 63) == 0) red[tid >> 6] = m;
        __syncthreads();
        return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    };
    auto gather = [&](uint32_t blk0, uint32_t n) {
        __syncthreads();                                       /* the previous block has been consumed */
        if (tid == 0) filled = 0u;
        const uint32_t j0 = (uint32_t)j0c + blk0;
        uint32_t sA = sFirst;
        if (blk0 != 0) {
            /* a later block of a long chunk: the last segment whose first survivor is not beyond j0 */
            auto rank0 = [&](uint32_t s) { return (uint64_t)c.G[s] + (uint64_t)min(e_b, c.E[s]); };
            sA = wg_search_le(seg_lo, seg_hi, (uint64_t)j0, rank0, &sh);
        }
        __syncthreads();
        gather_survivors(c, sA, seg_hi, T, e_b, j0, n, sv, si, mc, mg, me, &mxc, &filled);
        __syncthreads();
        if (tid == 0 && filled != n) err[0] = 1u;              /* the prefixes and the entries disagree */
    };

    float m = 0.0f;
    const bool long_chunk = cnt_c > ENC_BLK;
    if (BITS <= 8 && long_chunk)
        for (uint32_t blk0 = 0; blk0 < cnt_c; blk0 += ENC_BLK) {
            const uint32_t n = min(ENC_BLK, cnt_c - blk0);
            gather(blk0, n);
            m = fmaxf(m, block_absmax(n));
        }
    for (uint32_t blk0 = 0; blk0 < cnt_c; blk0 += ENC_BLK) {
        const uint32_t n = min(ENC_BLK, cnt_c - blk0);
        gather(blk0, n);
        float scale = 0.0f;
        if (BITS <= 8) {
            if (!long_chunk) m = block_absmax(n);
            scale = m == 0.0f ? 0.0f : __fdiv_rn(m, QMAX);
            if (tid == 0 && blk0 == 0) scales[t.S[b] + cb] = scale;
        }
        const uint64_t jb = j0c + blk0;                        /* bucket-local number of the block's first survivor */
        /* a thread takes pairs of consecutive survivors (a 4-bit pair is one byte) */
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t i0 = 2 * (tid + u * WG);
            if (i0 >= n) continue;
            const int have = (i0 + 1 < n) ? 2 : 1;
            float res[2] = {0.0f, 0.0f};
            int q[2] = {0, 0};
            uint32_t li[2] = {si[i0], have == 2 ? si[i0 + 1] : 0u};
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                if (hh >= have) continue;
                const float xv = sv[i0 + hh];
                float deq;
                if (BITS == 32) {
                    reinterpret_cast<float *>(vb)[jb + i0 + hh] = xv;
                    deq = xv;
                } else if (BITS == 16) {
                    const __half hv = __float2half_rn(xv);
                    reinterpret_cast<__half *>(vb)[jb + i0 + hh] = hv;
                    deq = __half2float(hv);
                } else {
                    if (scale != 0.0f) {
                        float tq = rintf(__fdiv_rn(xv, scale));
                        tq = fminf(fmaxf(tq, -QMAX), QMAX);
                        q[hh] = (int)tq;
                    }
                    deq = __fmul_rn((float)q[hh], scale);
                    if (BITS == 8) reinterpret_cast<int8_t *>(vb)[jb + i0 + hh] = (int8_t)q[hh];
                }
                res[hh] = __fsub_rn(xv, deq);
                idx_out[Pb + jb + i0 + hh] = li[hh];
            }
            if (BITS == 4) vb[(jb + i0) >> 1] = (uint8_t)((q[0] & 0xF) | ((q[1] & 0xF) << 4));
#pragma unroll
            for (int hh = 0; hh < 2; ++hh)
                if (hh < have) r[lo + li[hh]] = res[hh];
        }
    }
    }
}

/* ------------------------------------------------------------------ k_hard */

/* Ordered write for the buckets whose survivors are taken from the dense accumulator (PATH_BAND,
 * PATH_ZERO, and PATH_DENSE once its own passes have left T, e and the per-segment prefixes):
 * one wavefront per staging segment walks the elements the segment covers, in index order, and writes the
 * survivors' indices and values to their final slots.  Ranks inside a row of 64 lanes x 4
 * elements come from ballots; nothing crosses wavefronts.  which: bit p set = serve PATH p. */
template <bool DIRECT>   /* DIRECT (32-bit values): v_out is the payload itself and the survivors' residual is zero */
__device__ __forceinline__ void write_dense_body(float *__restrict__ r, const Tables &t, const Cand &c,
                                                 uint32_t *__restrict__ idx_out, float *__restrict__ v_out,
                                                 uint32_t which, uint32_t bid, uint32_t nblk)
{
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t n_seg = t.n_spans << t.segSh;
    for (uint32_t ss = bid * (WG / 64) + wave; ss < n_seg; ss += nblk * (WG / 64)) {
    const uint32_t span = ss >> t.segSh, wslot = ss & ((1u << t.segSh) - 1u);
    const uint32_t b = t.span_b[span];
    const uint32_t path = t.fast[b];
    if (!((which >> path) & 1u) || t.k[b] == 0u) continue;
    const SpanGeo s = span_geo_b(t, b, span - t.span0[b]);
    const uint32_t T = t.T[b], e_b = t.need[b];
    const uint64_t Pb = t.P[b];
    uint32_t run_g = c.G[ss], run_e = c.E[ss];
    const uint64_t lt = (1ull << lane) - 1ull;
    const uint32_t per = (t.spanT * 4u) >> t.segSh;
    const uint32_t wt0 = wslot * per, wt1 = min(s.ntiles * 4u, wt0 + per);
    /* the next wave-tile (64 lanes x 4 rows x 4 elements) is fetched while this one is written */
    float xn[4][4];
    uint32_t mn[4];
    auto fetch = [&](uint32_t wt) {
        const uint64_t wb = s.base + (uint64_t)wt * WTILE;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint64_t gi = wb + (uint64_t)(u * 64 + lane) * 4;
            mn[u] = load_quad(r, gi, s.lo, s.hi, xn[u]);
            if (t.pmask) mn[u] &= ~pruned_bits(t.pmask, s.tile_g + (wt >> 2), (wt & 3u) * WG + u * 64 + lane);
        }
    };
    if (wt0 < wt1) fetch(wt0);
    for (uint32_t wt = wt0; wt < wt1; ++wt) {
        const uint64_t wb = s.base + (uint64_t)wt * WTILE;
        float x[4][4];
        uint32_t m[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            m[u] = mn[u];
#pragma unroll
            for (int j = 0; j < 4; ++j) x[u][j] = xn[u][j];
        }
        if (wt + 1 < wt1) fetch(wt + 1);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint64_t gi = wb + (uint64_t)(u * 64 + lane) * 4;
            uint32_t fg = 0, fe = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t key = keyof(x[u][j]);
                if ((m[u] >> j) & 1u) { fg |= (key > T ? 1u : 0u) << j; fe |= (key == T ? 1u : 0u) << j; }
            }
            /* entries of lower lanes come first, then this lane's own four in order */
            uint32_t pg = run_g, pe = run_e, tg = 0, te = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint64_t bg = __ballot((fg >> j) & 1u), be = __ballot((fe >> j) & 1u);
                pg += __popcll(bg & lt); pe += __popcll(be & lt);
                tg += __popcll(bg); te += __popcll(be);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bool isg = (fg >> j) & 1u, ise = (fe >> j) & 1u;
                if (isg || (ise && pe < e_b)) {
                    const uint64_t pos = Pb + pg + min(e_b, pe);
                    idx_out[pos] = (uint32_t)(gi + j - s.lo);
                    v_out[pos] = x[u][j];
                    if (DIRECT) r[gi + j] = 0.0f;    /* value - value: nothing is left behind */
                }
                pg += isg ? 1u : 0u;
                pe += ise ? 1u : 0u;
            }
            run_g += tg;
            run_e += te;
        }
    }
    }
}

/* PATH_DENSE buckets, after their own passes have found T and e: elements above and equal to T
 * per staging segment (one wavefront per segment), the counts the scan turns into prefixes. */
__device__ __forceinline__ void segcount_dense_body(const float *__restrict__ r, const Tables &t, const Cand &c,
                                                    uint32_t bid, uint32_t nblk)
{
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t n_seg = t.n_spans << t.segSh;
    for (uint32_t ss = bid * (WG / 64) + wave; ss < n_seg; ss += nblk * (WG / 64)) {
    const uint32_t span = ss >> t.segSh, wslot = ss & ((1u << t.segSh) - 1u);
    const uint32_t b = t.span_b[span];
    if (t.fast[b] != PATH_DENSE || t.k[b] == 0u) continue;
    const SpanGeo s = span_geo_b(t, b, span - t.span0[b]);
    const uint32_t T = t.T[b];
    const uint32_t per = (t.spanT * 4u) >> t.segSh;
    const uint32_t wt0 = wslot * per, wt1 = min(s.ntiles * 4u, wt0 + per);
    uint32_t ng = 0, ne = 0;
    for (uint32_t wt = wt0; wt < wt1; ++wt) {
        const uint64_t wb = s.base + (uint64_t)wt * WTILE;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint64_t gi = wb + (uint64_t)(u * 64 + lane) * 4;
            float x[4];
            uint32_t m = load_quad(r, gi, s.lo, s.hi, x);
            if (t.pmask) m &= ~pruned_bits(t.pmask, s.tile_g + (wt >> 2), (wt & 3u) * WG + u * 64 + lane);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t key = keyof(x[j]);
                const bool ok = (m >> j) & 1u;
                ng += (ok && key > T) ? 1u : 0u;
                ne += (ok && key == T) ? 1u : 0u;
            }
        }
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) { ng += __shfl_xor(ng, d, 64); ne += __shfl_xor(ne, d, 64); }
    if (lane == 0) { c.G[ss] = ng; c.E[ss] = ne; }
    }
}

/* The buckets whose staged elements could not decide them (PATH_DENSE: an unlucky sample, a
 * staging segment that overflowed, a huge group of equal keys), in ONE launch of a fixed, small
 * grid whose workgroups meet at barriers between the steps: list of their spans, level-1
 * histogram over the dense accumulator, digit, level-2 histogram, digit, counts per segment,
 * prefixes, ordered write.  In the usual case there is no such bucket: each workgroup reads one
 * word and leaves, so the whole chain costs a single empty launch per call.
 * A barrier is an arrival counter in memory: every wavefront waits for its own stores, one thread
 * per workgroup then makes them visible device wide, counts the workgroup in and waits until all
 * have arrived, and drops what the caches hold afterwards.  The grid is small enough to be
 * resident at once; the wait is bounded by a clock all the same, and running out raises the
 * consistency flag. */
constexpr unsigned long long HARD_SPIN_TICKS = 500000000ull;      /* 5 s of the 100 MHz wall clock */

__device__ __forceinline__ void grid_barrier(uint32_t *bar, uint32_t target, uint32_t *__restrict__ err)
{
    __builtin_amdgcn_s_waitcnt(0);                   /* this wavefront's stores have reached the L2 */
    __syncthreads();
    if (threadIdx.x == 0) {
        __threadfence();                             /* write the L2 back: visible to the other dies */
        __hip_atomic_fetch_add(bar, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const unsigned long long t0 = wall_clock64();
        while (__hip_atomic_load(bar, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            __builtin_amdgcn_s_sleep(32);
            if (wall_clock64() - t0 > HARD_SPIN_TICKS) { err[0] = 1u; break; }
        }
        __threadfence();                             /* and nothing stale is read afterwards */
    }
    __syncthreads();
}

/* Ordered write and value coding in one pass, for the buckets whose survivors are taken from the
 * dense accumulator and whose threshold is known (PATH_BAND, PATH_ZERO), with chunks of at most
 * DENC_MAX_CHUNK survivors.  Survivors are dense here (ratios from an eighth up, or an
 * embedding whose few non-zero rows all survive), so the work is laid out by elements: a
 * workgroup streams a unit of one or two (dencSpans) consecutive spans, 4096 elements at a time (one
 * wave-tile per wavefront); ranks come from ballots and a prefix over the four wavefronts; the
 * survivors are put into LDS in rank order behind the ones still waiting for their chunk to
 * fill up; every chunk that is complete is coded from LDS by one wavefront (absmax, scale,
 * codes, indices, and the coding error scattered into the accumulator lines the workgroup has
 * just read, which are still in the cache).  A chunk that reaches across the unit's ends (or a
 * bucket's spans of another unit) is written uncoded to idx / v_out, and k_quant codes exactly
 * those afterwards (same test, see chunk_coded_by_stream).  16-bit values need no chunk and are
 * all coded here. */
constexpr uint32_t DENC_SMALL_CHUNK = 256;         /* up to here a wavefront codes a chunk */
constexpr uint32_t DENC_MAX_CHUNK = 2048;
constexpr uint32_t denc_cap(bool big) { return TILE + (big ? DENC_MAX_CHUNK : DENC_SMALL_CHUNK); }

template <int BITS, bool BIG>       /* BIG: chunks of more than DENC_SMALL_CHUNK survivors */
__device__ __forceinline__ void dense_encode_body(float *__restrict__ r, const Tables &t, const Cand &c,
                                                  uint32_t *__restrict__ idx_out, float *__restrict__ v_out,
                                                  void *__restrict__ val, float *__restrict__ scales,
                                                  float *sv, uint32_t *si, uint32_t *wtot, uint32_t *__restrict__ err,
                                                  uint32_t bid, uint32_t nblk)
{
    constexpr float QMAX = BITS == 8 ? 127.0f : 7.0f;     /* (unused for 16 / 32 bits) */
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t chunk = t.chunk;
    const uint32_t n_units = (t.n_spans + t.dencSpans - 1) / t.dencSpans;
    for (uint32_t unit = bid; unit < n_units; unit += nblk) {
        uint32_t cur_b = NONE;
        /* state of the stream: one bucket's consecutive spans inside the unit */
        uint32_t T = 0, e_b = 0, kb = 0, run_g = 0, run_e = 0, carry = 0, Rbase = 0;
        uint64_t Pb = 0, lo = 0;
        uint8_t *vb = nullptr;
        uint64_t Sb = 0;
        bool head = false;
        /* what is left in LDS when a stream ends belongs to a chunk that goes on elsewhere */
        auto flush = [&]() {
            for (uint32_t i = tid; i < carry; i += WG) {
                idx_out[Pb + Rbase + i] = si[i];
                v_out[Pb + Rbase + i] = sv[i];
            }
            carry = 0;
            __syncthreads();
        };
        const uint32_t sp1 = min(t.n_spans, (unit + 1) * t.dencSpans);
        for (uint32_t span = unit * t.dencSpans; span < sp1; ++span) {
            const uint32_t b = t.span_b[span];
            const uint32_t path = t.fast[b];
            if ((path != PATH_BAND && path != PATH_ZERO) || t.k[b] == 0u) {
                if (cur_b != NONE) { flush(); cur_b = NONE; }
                continue;
            }
            const SpanGeo s = span_geo_b(t, b, span - t.span0[b]);
            if (b != cur_b) {
                if (cur_b != NONE) flush();
                cur_b = b;
                T = t.T[b]; e_b = t.need[b]; kb = t.k[b]; Pb = t.P[b]; lo = s.lo;
                vb = reinterpret_cast<uint8_t *>(val) + t.V[b];
                Sb = t.S[b];
                const uint32_t ss0 = span << t.segSh;
                run_g = c.G[ss0]; run_e = c.E[ss0];
                Rbase = run_g + min(e_b, run_e);
                carry = 0;
                head = BITS <= 8 && (Rbase % chunk) != 0u;
            }
            else if (tid == 0 && (run_g != c.G[span << t.segSh] || run_e != c.E[span << t.segSh]))
                err[0] = 1u;                         /* the prefixes and the elements disagree */
                    const uint32_t nwt = s.ntiles * 4u;
            /* the next 4096 elements are fetched while the survivors of these are coded */
            float xn[4][4];
            uint32_t mn[4];
            auto fetch = [&](uint32_t wt_base) {
                const uint32_t wt = wt_base + wave;
                const uint64_t wb = s.base + (uint64_t)wt * WTILE;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const uint64_t gi = wb + (uint64_t)(u * 64 + lane) * 4;
                    mn[u] = 0;
#pragma unroll
                    for (int j = 0; j < 4; ++j) xn[u][j] = 0.0f;
                    if (wt < nwt) {
                        if (wb >= s.lo && wb + WTILE <= s.hi) {          /* the whole wave-tile lies inside the bucket */
                            const f4 v = *reinterpret_cast<const f4 *>(r + gi);
                            xn[u][0] = v.x; xn[u][1] = v.y; xn[u][2] = v.z; xn[u][3] = v.w;
                            mn[u] = 0xFu;
                        } else {
                            mn[u] = load_quad(r, gi, s.lo, s.hi, xn[u]);
                        }
                        if (t.pmask) mn[u] &= ~pruned_bits(t.pmask, s.tile_g + (wt >> 2), (wt & 3u) * WG + u * 64 + lane);
                    }
                }
            };
            fetch(0);
            for (uint32_t wt_base = 0; wt_base < nwt; wt_base += WG / 64) {
                const uint32_t wt = wt_base + wave;
                const uint64_t wb = s.base + (uint64_t)wt * WTILE;
                float x[4][4];
                uint32_t fg[4], fe[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    fg[u] = fe[u] = 0;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        x[u][j] = xn[u][j];
                        const uint32_t key = keyof(x[u][j]);
                        if ((mn[u] >> j) & 1u) { fg[u] |= (key > T ? 1u : 0u) << j; fe[u] |= (key == T ? 1u : 0u) << j; }
                    }
                }
                /* ranks: a lane's elements of a row are consecutive, so the elements before one are
                 * those of the lower lanes of its row, of the earlier rows and of the earlier
                 * wavefronts.  Counts of elements above T (low half) and equal to T (high half)
                 * travel in one word; 4096 elements cannot carry from one half into the other. */
                uint32_t ex[4], wsum = 0;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const uint32_t cnt = (uint32_t)__popc(fg[u]) | ((uint32_t)__popc(fe[u]) << 16);
                    const uint32_t incl = wave_incl_scan(cnt);
                    ex[u] = wsum + incl - cnt;
                    wsum += __builtin_amdgcn_readlane(incl, 63);
                }
                if (lane == 0) wtot[wave] = wsum;
                __syncthreads();
                uint32_t woff = 0, all = 0;
#pragma unroll
                for (uint32_t w = 0; w < WG / 64; ++w) {
                    if (w < wave) woff += wtot[w];
                    all += wtot[w];
                }
                const uint32_t all_g = all & 0xFFFFu, all_e = all >> 16;
                const uint32_t Rnext = run_g + min(e_b, run_e);               /* rank of the next survivor = Rbase + carry */
                const uint32_t nsurv = (run_g + all_g + min(e_b, run_e + all_e)) - Rnext;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const uint64_t gi = wb + (uint64_t)(u * 64 + lane) * 4;
                    const uint32_t before = woff + ex[u];
                    uint32_t pe = run_e + (before >> 16);
                    /* a lane's survivors are consecutive in rank: one slot computed, then counted on */
                    uint32_t slot = carry + (run_g + (before & 0xFFFFu) + min(e_b, pe) - Rnext);
                    const uint32_t li0 = (uint32_t)(gi - s.lo);
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const bool ise = (fe[u] >> j) & 1u;
                        const bool take = ((fg[u] >> j) & 1u) || (ise && pe < e_b);
                        if (take) { sv[slot] = x[u][j]; si[slot] = li0 + j; }
                        slot += take ? 1u : 0u;
                        pe += ise ? 1u : 0u;
                    }
                }
                run_g += all_g;
                run_e += all_e;
                __syncthreads();
                if (wt_base + WG / 64 < nwt) fetch(wt_base + WG / 64);
                /* consume what is complete */
                const uint32_t total = carry + nsurv;
                uint32_t p = 0;
                if (BITS >= 16) {
                    /* no scale to wait for: every survivor is final at once */
                    for (uint32_t i = tid; i < total; i += WG) {
                        const float xv = sv[i];
                        const uint32_t li = si[i];
                        idx_out[Pb + Rbase + i] = li;
                        if (BITS == 16) {
                            const __half hv = __float2half_rn(xv);
                            reinterpret_cast<__half *>(vb)[Rbase + i] = hv;
                            r[lo + li] = __fsub_rn(xv, __half2float(hv));
                        } else {
                            reinterpret_cast<float *>(vb)[Rbase + i] = xv;
                            r[lo + li] = 0.0f;       /* value - value: nothing is left behind */
                        }
                    }
                    p = total;
                } else {
                    if (head) {
                        /* up to the next chunk boundary: part of a chunk that began before this stream */
                        const uint32_t to_edge = chunk - (Rbase % chunk);
                        const uint32_t nh = min(total, to_edge);
                        for (uint32_t i = tid; i < nh; i += WG) {
                            idx_out[Pb + Rbase + i] = si[i];
                            v_out[Pb + Rbase + i] = sv[i];
                        }
                        p = nh;
                        if (nh == to_edge) head = false;
                    }
                    if (!head) {
                        const uint32_t avail = total - p;
                        const uint32_t nfull = avail / chunk, rem = avail - nfull * chunk;
                        const uint32_t ncode = nfull + ((rem != 0u && Rbase + total == kb) ? 1u : 0u);   /* the bucket's last chunk may be short */
                        /* one pair of consecutive survivors of a chunk: codes, index, coding error */
                        auto code_pair = [&](uint32_t rank0, uint32_t i0, uint32_t cnt, float scale, const float (&xv)[2],
                                             const uint32_t (&li)[2]) {
                            const int have = (i0 + 1 < cnt) ? 2 : 1;
                            int qq[2] = {0, 0};
                            float res[2] = {0.0f, 0.0f};
#pragma unroll
                            for (int hh = 0; hh < 2; ++hh) {
                                if (hh >= have) continue;
                                if (scale != 0.0f) {
                                    float tq = rintf(__fdiv_rn(xv[hh], scale));
                                    tq = fminf(fmaxf(tq, -QMAX), QMAX);
                                    qq[hh] = (int)tq;
                                }
                                res[hh] = __fsub_rn(xv[hh], __fmul_rn((float)qq[hh], scale));
                                if (BITS == 8) reinterpret_cast<int8_t *>(vb)[rank0 + i0 + hh] = (int8_t)qq[hh];
                                idx_out[Pb + rank0 + i0 + hh] = li[hh];
                            }
                            if (BITS == 4) vb[(rank0 + i0) >> 1] = (uint8_t)((qq[0] & 0xF) | ((qq[1] & 0xF) << 4));
#pragma unroll
                            for (int hh = 0; hh < 2; ++hh)
                                if (hh < have) r[lo + li[hh]] = res[hh];
                        };
                        if (!BIG) {
                            /* chunks of up to 256: a wavefront each, two pairs per lane */
                            for (uint32_t q = wave; q < ncode; q += WG / 64) {
                                const uint32_t base = p + q * chunk;
                                const uint32_t cnt = min(chunk, total - base);
                                const uint32_t rank0 = Rbase + base;
                                float xv[2][2];
                                uint32_t li[2][2];
#pragma unroll
                                for (int u = 0; u < 2; ++u)
#pragma unroll
                                    for (int hh = 0; hh < 2; ++hh) {
                                        const uint32_t i = 2 * (lane + u * 64) + hh;
                                        xv[u][hh] = i < cnt ? sv[base + i] : 0.0f;
                                        li[u][hh] = i < cnt ? si[base + i] : 0u;
                                    }
                                float mx = fmaxf(fmaxf(fabsf(xv[0][0]), fabsf(xv[0][1])), fmaxf(fabsf(xv[1][0]), fabsf(xv[1][1])));
#pragma unroll
                                for (int d = 32; d >= 1; d >>= 1) mx = fmaxf(mx, __shfl_xor(mx, d, 64));
                                const float scale = mx == 0.0f ? 0.0f : __fdiv_rn(mx, QMAX);
                                if (lane == 0) scales[Sb + rank0 / chunk] = scale;
#pragma unroll
                                for (int u = 0; u < 2; ++u) {
                                    const uint32_t i0 = 2 * (lane + u * 64);
                                    if (i0 < cnt) code_pair(rank0, i0, cnt, scale, xv[u], li[u]);
                                }
                            }
                        } else {
                            /* longer chunks: the whole workgroup on one chunk after the other */
                            for (uint32_t q = 0; q < ncode; ++q) {
                                const uint32_t base = p + q * chunk;
                                const uint32_t cnt = min(chunk, total - base);
                                const uint32_t rank0 = Rbase + base;
                                float mx = 0.0f;
                                for (uint32_t i = tid; i < cnt; i += WG) mx = fmaxf(mx, fabsf(sv[base + i]));
#pragma unroll
                                for (int d = 32; d >= 1; d >>= 1) mx = fmaxf(mx, __shfl_xor(mx, d, 64));
                                float *red = reinterpret_cast<float *>(wtot);
                                if (lane == 0) red[wave] = mx;
                                __syncthreads();
                                mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
                                const float scale = mx == 0.0f ? 0.0f : __fdiv_rn(mx, QMAX);
                                if (tid == 0) scales[Sb + rank0 / chunk] = scale;
                                for (uint32_t i0 = 2 * tid; i0 < cnt; i0 += 2 * WG) {
                                    const float xv[2] = {sv[base + i0], i0 + 1 < cnt ? sv[base + i0 + 1] : 0.0f};
                                    const uint32_t li[2] = {si[base + i0], i0 + 1 < cnt ? si[base + i0 + 1] : 0u};
                                    code_pair(rank0, i0, cnt, scale, xv, li);
                                }
                                __syncthreads();
                            }
                        }
                        p += min(avail, ncode * chunk);
                    }
                }
                __syncthreads();
                /* the rest waits at the front for the next elements */
                const uint32_t left = total - p;
                constexpr uint32_t KEEP = (BIG ? DENC_MAX_CHUNK : DENC_SMALL_CHUNK) / WG;
                float keep_v[KEEP];
                uint32_t keep_i[KEEP];
#pragma unroll
                for (uint32_t u = 0; u < KEEP; ++u) {
                    const uint32_t i = tid + u * WG;
                    keep_v[u] = 0.0f; keep_i[u] = 0u;
                    if (i < left) { keep_v[u] = sv[p + i]; keep_i[u] = si[p + i]; }
                }
                __syncthreads();
#pragma unroll
                for (uint32_t u = 0; u < KEEP; ++u) {
                    const uint32_t i = tid + u * WG;
                    if (i < left) { sv[i] = keep_v[u]; si[i] = keep_i[u]; }
                }
                Rbase += p;
                carry = left;
            }
        }
        if (cur_b != NONE) flush();
        __syncthreads();
    }
}

/* Whether chunk cb (bucket-local) of a PATH_BAND / PATH_ZERO bucket b was coded by
 * dense_encode_body: its first survivor lies in segment s, and all of its survivors lie in the
 * spans of b inside the unit of dencSpans spans that holds s. */
__device__ __forceinline__ bool chunk_coded_by_stream(const Tables &t, const Cand &c, uint32_t b, uint64_t cb, uint32_t s)
{
    const uint32_t kb = t.k[b], e_b = t.need[b];
    const uint64_t end = min((cb + 1) * (uint64_t)t.chunk, (uint64_t)kb);
    const uint32_t next_span = ((s >> t.segSh) / t.dencSpans + 1u) * t.dencSpans;
    uint64_t r1 = kb;
    if (next_span < t.span0[b + 1]) {
        const uint32_t sn = next_span << t.segSh;
        r1 = (uint64_t)c.G[sn] + min(e_b, c.E[sn]);
    }
    return end <= r1;
}

/* workgroups of k_hard per compute unit: what its LDS allows (all of them must be resident) */
constexpr uint32_t hard_wg_per_cu(bool big) { return big ? 3u : 4u; }
constexpr uint32_t hard_lds(bool big) { return 2 * denc_cap(big) + 2 * (WG / 64); }    /* words; also holds the level-1 histogram */

template <int BITS, bool BIG>
__global__ __launch_bounds__(WG, hard_wg_per_cu(BIG)) void k_hard(float *__restrict__ r, Tables t, Cand c, uint32_t *__restrict__ f1,
                                             uint32_t *__restrict__ f2, uint32_t *__restrict__ idx,
                                             float *__restrict__ vdst, void *__restrict__ val,
                                             float *__restrict__ scales, uint32_t *__restrict__ err, int stream_coding, uint32_t team)
{
    static_assert(hard_lds(BIG) >= NB1, "the pool must hold the level-1 histogram");
    __shared__ uint32_t pool[hard_lds(BIG)];
    if (t.nhard[0] == 0u) return;                    /* every bucket was decided and coded from its staged elements */
    const uint32_t bid = blockIdx.x;
    uint32_t nblk = gridDim.x;
    /* band and zero-threshold buckets: survivors from the dense accumulator, threshold known */
    if (stream_coding)
        dense_encode_body<BITS, BIG>(r, t, c, idx, vdst, val, scales, reinterpret_cast<float *>(pool),
                                     pool + denc_cap(BIG), pool + 2 * denc_cap(BIG), err, bid, nblk);
    else
        write_dense_body<BITS == 32>(r, t, c, idx, vdst, (1u << PATH_BAND) | (1u << PATH_ZERO), bid, nblk);
    /* the dense passes: the first `team` workgroups only.  They are dispatched before the others
     * of this launch, and the team is small enough (one workgroup per compute unit) to be
     * resident at once even next to the teams of other contexts; a barrier that still cannot
     * complete runs into its time limit and raises the consistency flag. */
    if (t.nhard[2] == 0u || bid >= team) return;
    __syncthreads();
    nblk = team;
    uint32_t *h = pool;
    uint32_t *bar = t.nhard + 1;
    uint32_t arrivals = 0;
    if (bid == 0) fb_plan_body(t);
    grid_barrier(bar, arrivals += nblk, err);
    fb_refine_body<1>(r, t, f1, h, bid, nblk);
    grid_barrier(bar, arrivals += nblk, err);
    for (uint32_t b = bid; b < t.B; b += nblk) { __syncthreads(); pick_body<1>(t, f1, f1, err, nullptr, 1, b); }
    grid_barrier(bar, arrivals += nblk, err);
    fb_refine_body<2>(r, t, f2, h, bid, nblk);
    grid_barrier(bar, arrivals += nblk, err);
    for (uint32_t b = bid; b < t.B; b += nblk) { __syncthreads(); pick_body<2>(t, f2, f2, err, nullptr, 1, b); }
    grid_barrier(bar, arrivals += nblk, err);
    segcount_dense_body(r, t, c, bid, nblk);
    grid_barrier(bar, arrivals += nblk, err);
    for (uint32_t b = bid; b < t.B; b += nblk) { __syncthreads(); scan_body(t, c.G, c.E, nullptr, nullptr, 1, b); }
    grid_barrier(bar, arrivals += nblk, err);
    write_dense_body<BITS == 32>(r, t, c, idx, vdst, 1u << PATH_DENSE, bid, nblk);
}

/* Value coding of the survivors the ordered writes above left uncoded in idx / vdst: every chunk
 * of a PATH_DENSE bucket, and of the band / zero-threshold buckets the chunks that the one-pass
 * coding could not complete (all of them when it was not used).  Leaves at once when every
 * bucket was coded from its staged elements.  Chunks of up to 256 survivors: a wavefront per
 * chunk, QUANT_PER_WAVE chunks per wavefront; longer chunks: a workgroup each. */
constexpr uint32_t QUANT_WAVE_CHUNK = 256;
constexpr uint32_t QUANT_BIG_PER_WG = 8;
template <int BITS>
__global__ __launch_bounds__(WG) void k_quant(const float *__restrict__ v, const uint32_t *__restrict__ idx, Tables t,
                                              Cand c, float *__restrict__ r, void *__restrict__ val,
                                              float *__restrict__ scales, const uint32_t *__restrict__ chunk_b,
                                              const uint32_t *__restrict__ chunk_seg, uint64_t n_chunks, int stream_coding)
{
    if (t.nhard[0] == 0u) return;
    if (t.chunk <= QUANT_WAVE_CHUNK) {
        /* which of the workgroup's chunks are still to be coded: one lane per chunk */
        constexpr uint32_t PER_WG = (WG / 64) * QUANT_PER_WAVE;
        __shared__ uint32_t todo_sh;
        const uint64_t cw = (uint64_t)blockIdx.x * PER_WG;
        if (threadIdx.x < 64) {
            const uint64_t cid = cw + threadIdx.x;
            bool todo = false;
            if (threadIdx.x < PER_WG && cid < n_chunks) {
                const uint32_t b = chunk_b[cid];
                const uint32_t path = t.fast[b];
                todo = path != PATH_CAND;
                if (todo && stream_coding && path != PATH_DENSE)
                    todo = BITS <= 8 && !chunk_coded_by_stream(t, c, b, cid - t.C[b], chunk_seg[cid]);
            }
            const uint64_t bal = __ballot(todo);
            if (threadIdx.x == 0) todo_sh = (uint32_t)bal;
        }
        __syncthreads();
        const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        const uint32_t mine = (todo_sh >> (wave * QUANT_PER_WAVE)) & ((1u << QUANT_PER_WAVE) - 1u);
        if (mine) quant_wave<BITS>(v, idx, t, r, val, scales, chunk_b, cw + wave * QUANT_PER_WAVE, mine);
    } else {
        /* longer chunks: QUANT_BIG_PER_WG chunks per workgroup, one after the other; which of them
         * are still to be coded is found by one lane per chunk first */
        __shared__ uint32_t todo_big;
        const uint64_t cw = (uint64_t)blockIdx.x * QUANT_BIG_PER_WG;
        if (threadIdx.x < 64) {
            const uint64_t cid = cw + threadIdx.x;
            bool todo = false;
            if (threadIdx.x < QUANT_BIG_PER_WG && cid < n_chunks) {
                const uint32_t b = chunk_b[cid];
                const uint32_t path = t.fast[b];
                todo = path != PATH_CAND;
                if (todo && stream_coding && path != PATH_DENSE)
                    todo = BITS <= 8 && !chunk_coded_by_stream(t, c, b, cid - t.C[b], chunk_seg[cid]);
            }
            const uint64_t bal = __ballot(todo);
            if (threadIdx.x == 0) todo_big = (uint32_t)bal;
        }
        __syncthreads();
        uint32_t mask = todo_big;
        while (mask) {
            const uint32_t q = (uint32_t)__builtin_ctz(mask);
            mask &= mask - 1u;
            __syncthreads();                         /* the previous chunk's use of LDS is over */
            quant_body<BITS>(v, idx, t, r, val, scales, chunk_b, cw + q);
        }
    }
}

/* ------------------------------------------------------------------ weight stage: the bitmap */

/* The staged band elements of a bucket decided from its band that are pruned get their bit in the
 * bitmap (k_whist left 0 for the whole band): below the threshold key, or equal to it and not
 * among the first e equal ones in index order (k_select_finish left T, e and, per segment, the
 * number of equal keys before it).  Sixteen lanes per staging segment, four segments per
 * wavefront. */
__global__ __launch_bounds__(WG) void k_wfix(Tables t, Cand c, uint32_t *__restrict__ pmask)
{
    const uint32_t lane = threadIdx.x & 63, sub = lane >> 4, gl = lane & 15u;
    const uint32_t n_seg = t.n_spans << t.segSh;
    const uint32_t ss = (blockIdx.x * (WG / 64) + (threadIdx.x >> 6)) * 4u + sub;
    uint32_t cnt = 0, T = 0, e_b = 0, run_e = 0, b = 0, head = 0;
    if (ss < n_seg) {
        b = t.span_b[ss >> t.segSh];
        if (t.fast[b] == PATH_BAND && t.k[b] != 0u) {
            cnt = c.cnt[ss];
            T = t.T[b]; e_b = t.need[b]; run_e = c.E[ss];
            head = (uint32_t)(t.off[b] & 3ull);
        }
    }
    uint32_t maxcnt = cnt;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) maxcnt = max(maxcnt, (uint32_t)__shfl_xor(maxcnt, d, 64));
    const uint64_t base = (uint64_t)ss * c.cap;
    for (uint32_t i0 = 0; i0 < maxcnt; i0 += 16) {
        const uint32_t i = i0 + gl;
        const bool in = i < cnt;
        const uint32_t key = in ? keyof(c.val[base + i]) : 0u;
        const uint32_t li = in ? c.idx[base + i] : 0u;
        const bool ise = in && key == T;
        const uint32_t be = (uint32_t)(__ballot(ise) >> (sub * 16u)) & 0xFFFFu;
        const uint32_t pe = run_e + __popc(be & ((1u << gl) - 1u));
        if (in && (key < T || (ise && pe >= e_b))) {
            const uint64_t e = (uint64_t)li + head;          /* position counted from the bucket's first tile */
            const uint32_t tile = t.tile0[b] + (uint32_t)(e / TILE);
            const uint32_t inq = (uint32_t)(e % TILE);
            atomicOr(&pmask[(uint64_t)tile * (TILE / 32) + (inq >> 5)], 1u << (inq & 31u));
        }
        run_e += __popc(be);
    }
}

/* Bitmap of a bucket that went through the dense passes (T, e and the per-segment prefixes are
 * known): one wavefront per staging segment walks the weights it covers in index order; a weight
 * is kept when its key exceeds T or equals it among the first e such, everything else gets its
 * bit.  Every word of the bucket's tiles is written. */
__device__ __forceinline__ void mask_dense_body(const float *__restrict__ w, const Tables &t, const Cand &c,
                                                uint32_t *__restrict__ pmask, uint32_t bid, uint32_t nblk)
{
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t n_seg = t.n_spans << t.segSh;
    const uint64_t lt = (1ull << lane) - 1ull;
    for (uint32_t ss = bid * (WG / 64) + wave; ss < n_seg; ss += nblk * (WG / 64)) {
        const uint32_t span = ss >> t.segSh, wslot = ss & ((1u << t.segSh) - 1u);
        const uint32_t b = t.span_b[span];
        if (t.fast[b] != PATH_DENSE || t.k[b] == 0u) continue;
        const SpanGeo s = span_geo_b(t, b, span - t.span0[b]);
        const uint32_t T = t.T[b], e_b = t.need[b];
        uint32_t run_e = c.E[ss];
        const uint32_t per = (t.spanT * 4u) >> t.segSh;
        const uint32_t wt0 = wslot * per, wt1 = min(s.ntiles * 4u, wt0 + per);
        for (uint32_t wt = wt0; wt < wt1; ++wt) {
            const uint64_t wb = s.base + (uint64_t)wt * WTILE;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint64_t gi = wb + (uint64_t)(u * 64 + lane) * 4;
                float x[4];
                const uint32_t m = load_quad(w, gi, s.lo, s.hi, x);
                uint32_t fe = 0, bits = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t key = keyof(x[j]);
                    if ((m >> j) & 1u) { fe |= (key == T ? 1u : 0u) << j; bits |= (key < T ? 1u : 0u) << j; }
                }
                uint32_t pe = run_e, te = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint64_t be = __ballot((fe >> j) & 1u);
                    pe += __popcll(be & lt);
                    te += __popcll(be);
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const bool ise = (fe >> j) & 1u;
                    if (ise && pe >= e_b) bits |= 1u << j;
                    pe += ise ? 1u : 0u;
                }
                run_e += te;
                uint32_t word = bits << ((lane & 7u) * 4u);
                word |= __shfl_xor(word, 1, 64);
                word |= __shfl_xor(word, 2, 64);
                word |= __shfl_xor(word, 4, 64);
                if ((lane & 7u) == 0u)
                    pmask[(uint64_t)(s.tile_g + (wt >> 2)) * (TILE / 32) + (wt & 3u) * (WG / 8) + u * 8 + (lane >> 3)] = word;
            }
        }
    }
}

/* The weight buckets on the dense passes (no usable band, or a band that missed twice over), in
 * one launch of a small resident grid with barriers between the steps, like k_hard: spans,
 * level-1 histogram of |w|, digit, level-2 histogram, digit, counts per segment, prefixes,
 * bitmap.  Leaves at once when there is no such bucket. */
__global__ __launch_bounds__(WG) void k_whard(const float *__restrict__ w, Tables t, Cand c, uint32_t *__restrict__ f1,
                                              uint32_t *__restrict__ f2, uint32_t *__restrict__ pmask,
                                              uint32_t *__restrict__ err)
{
    __shared__ uint32_t h[NB1];
    if (t.nhard[2] == 0u) return;
    const uint32_t bid = blockIdx.x, nblk = gridDim.x;
    uint32_t *bar = t.nhard + 1;
    uint32_t arrivals = 0;
    if (bid == 0) fb_plan_body(t);
    grid_barrier(bar, arrivals += nblk, err);
    fb_refine_body<1>(w, t, f1, h, bid, nblk);
    grid_barrier(bar, arrivals += nblk, err);
    for (uint32_t b = bid; b < t.B; b += nblk) { __syncthreads(); pick_body<1>(t, f1, f1, err, nullptr, 1, b); }
    grid_barrier(bar, arrivals += nblk, err);
    fb_refine_body<2>(w, t, f2, h, bid, nblk);
    grid_barrier(bar, arrivals += nblk, err);
    for (uint32_t b = bid; b < t.B; b += nblk) { __syncthreads(); pick_body<2>(t, f2, f2, err, nullptr, 1, b); }
    grid_barrier(bar, arrivals += nblk, err);
    segcount_dense_body(w, t, c, bid, nblk);
    grid_barrier(bar, arrivals += nblk, err);
    for (uint32_t b = bid; b < t.B; b += nblk) { __syncthreads(); scan_body(t, c.G, c.E, nullptr, nullptr, 1, b); }
    grid_barrier(bar, arrivals += nblk, err);
    mask_dense_body(w, t, c, pmask, bid, nblk);
}

}  // namespace

#endif
