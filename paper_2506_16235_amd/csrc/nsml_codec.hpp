/*
 * libnsml device code, part 4: value coding of the survivors and the decompress kernels.
 * Included by nsml_kernels.hip (one translation unit); not a public header.
 */
#ifndef NSML_CODEC_HPP
#define NSML_CODEC_HPP

namespace {

/* ------------------------------------------------------------------ value coding */

/* The coding of quant_body (below) for chunks of at most 256 survivors, one wavefront per chunk and QUANT_PER_WAVE
 * chunks per wavefront, all of whose values and indices are fetched before any is used (with a
 * workgroup per small chunk the step is bound by the latency of its chain of dependent loads,
 * not by bandwidth).  A lane takes up to two pairs of consecutive survivors of each chunk. */
constexpr uint32_t QUANT_PER_WAVE = 4;
template <int BITS>
__device__ __forceinline__ void quant_wave(const float *__restrict__ v, const uint32_t *__restrict__ idx,
                                           const Tables &t, float *__restrict__ r, void *__restrict__ val,
                                           float *__restrict__ scales, const uint32_t *__restrict__ chunk_b,
                                           uint64_t c0, uint32_t todo)
{
    constexpr float QMAX = BITS == 8 ? 127.0f : 7.0f;
    const uint32_t lane = threadIdx.x & 63;
    uint32_t bq[QUANT_PER_WAVE], cnt[QUANT_PER_WAVE];
    uint64_t j0[QUANT_PER_WAVE], jg[QUANT_PER_WAVE], cbq[QUANT_PER_WAVE];
#pragma unroll
    for (uint32_t q = 0; q < QUANT_PER_WAVE; ++q) bq[q] = ((todo >> q) & 1u) ? chunk_b[c0 + q] : NONE;   /* bit q: chunk c0 + q is to be coded */
#pragma unroll
    for (uint32_t q = 0; q < QUANT_PER_WAVE; ++q) {
        cnt[q] = 0; j0[q] = jg[q] = cbq[q] = 0;
        if (bq[q] != NONE) {
            cbq[q] = c0 + q - t.C[bq[q]];
            j0[q] = cbq[q] * t.chunk;
            cnt[q] = (uint32_t)min((uint64_t)t.chunk, (uint64_t)t.k[bq[q]] - j0[q]);
            jg[q] = t.P[bq[q]] + j0[q];
        }
    }
    float x[QUANT_PER_WAVE][2][2];
    uint32_t li[QUANT_PER_WAVE][2][2];
#pragma unroll
    for (uint32_t q = 0; q < QUANT_PER_WAVE; ++q)
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                const uint32_t i = 2 * (lane + u * 64) + hh;
                x[q][u][hh] = i < cnt[q] ? v[jg[q] + i] : 0.0f;
                li[q][u][hh] = i < cnt[q] ? idx[jg[q] + i] : 0u;
            }
#pragma unroll
    for (uint32_t q = 0; q < QUANT_PER_WAVE; ++q) {
        if (cnt[q] == 0) continue;                             /* same for the whole wavefront */
        const uint32_t b = bq[q];
        const uint64_t lo = t.off[b];
        uint8_t *vb = reinterpret_cast<uint8_t *>(val) + t.V[b];
        float scale = 0.0f;
        if (BITS <= 8) {
            float m = fmaxf(fmaxf(fabsf(x[q][0][0]), fabsf(x[q][0][1])), fmaxf(fabsf(x[q][1][0]), fabsf(x[q][1][1])));
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) m = fmaxf(m, __shfl_xor(m, d, 64));
            scale = m == 0.0f ? 0.0f : __fdiv_rn(m, QMAX);
            if (lane == 0) scales[t.S[b] + cbq[q]] = scale;
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const uint32_t i0 = 2 * (lane + u * 64);
            if (i0 >= cnt[q]) continue;
            const int have = (i0 + 1 < cnt[q]) ? 2 : 1;
            float res[2] = {0.0f, 0.0f};
            int qq[2] = {0, 0};
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                if (hh >= have) continue;
                const float xv = x[q][u][hh];
                float deq;
                if (BITS == 32) {
                    deq = xv;
                } else if (BITS == 16) {
                    const __half hv = __float2half_rn(xv);
                    reinterpret_cast<__half *>(vb)[j0[q] + i0 + hh] = hv;
                    deq = __half2float(hv);
                } else {
                    if (scale != 0.0f) {
                        float tq = rintf(__fdiv_rn(xv, scale));
                        tq = fminf(fmaxf(tq, -QMAX), QMAX);
                        qq[hh] = (int)tq;
                    }
                    deq = __fmul_rn((float)qq[hh], scale);
                    if (BITS == 8) reinterpret_cast<int8_t *>(vb)[j0[q] + i0 + hh] = (int8_t)qq[hh];
                }
                res[hh] = __fsub_rn(xv, deq);
            }
            if (BITS == 4) vb[(j0[q] + i0) >> 1] = (uint8_t)((qq[0] & 0xF) | ((qq[1] & 0xF) << 4));
#pragma unroll
            for (int hh = 0; hh < 2; ++hh)
                if (hh < have) r[lo + li[q][u][hh]] = res[hh];
        }
    }
}

/* A workgroup's work on one chunk of `chunk` consecutive survivors of a bucket whose survivors
 * were written by k_hard's ordered pass (not PATH_CAND): absmax, scale,
 * codes, packing, and the coding error left in the residual.  Every floating-point step is a
 * single correctly rounded binary32 operation (divide, round-to-nearest-even, multiply,
 * subtract); nothing may be contracted into an fma. */
template <int BITS>
__device__ __forceinline__ void quant_body(const float *__restrict__ v, const uint32_t *__restrict__ idx,
                                           const Tables &t, float *__restrict__ r, void *__restrict__ val,
                                           float *__restrict__ scales, const uint32_t *__restrict__ chunk_b,
                                           uint64_t c)
{
    __shared__ float red[WG / 64];
    const uint32_t tid = threadIdx.x;
    const uint32_t b = chunk_b[c];
    if (t.fast[b] == PATH_CAND) return;                     /* coded by k_encode */
    const uint64_t cb = c - t.C[b];
    const uint64_t j0 = cb * t.chunk;                         /* first survivor of the chunk, bucket-local */
    const uint32_t cnt = (uint32_t)min((uint64_t)t.chunk, (uint64_t)t.k[b] - j0);
    const uint64_t jg = t.P[b] + j0;                          /* same, global */
    const uint64_t lo = t.off[b];
    uint8_t *vb = reinterpret_cast<uint8_t *>(val) + t.V[b];
    /* A thread takes pairs of consecutive survivors (so a 4-bit pair is one byte store), up to
     * four pairs per block of 2048; the values and indices of a block are fetched before any is
     * used.  A chunk of up to 2048 is one block and its values are read once; a longer chunk
     * first takes its absmax in a pass of its own. */
    constexpr uint32_t BLK = WG * 8;
    const bool one_block = cnt <= BLK;
    float scale = 0.0f;
    if (BITS <= 8 && !one_block) {
        float m = 0.0f;
        for (uint32_t i = tid; i < cnt; i += WG) m = fmaxf(m, fabsf(v[jg + i]));
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) m = fmaxf(m, __shfl_xor(m, d, 64));
        if ((tid & 63) == 0) red[tid >> 6] = m;
        __syncthreads();
        m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        constexpr float QMAX = BITS == 8 ? 127.0f : 7.0f;
        scale = m == 0.0f ? 0.0f : __fdiv_rn(m, QMAX);
        if (tid == 0) scales[t.S[b] + cb] = scale;
    }
    for (uint32_t b0 = 0; b0 < cnt; b0 += BLK) {
        float x[4][2];
        uint32_t li[4][2];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                const uint32_t i = b0 + 2 * (tid + u * WG) + hh;
                x[u][hh] = i < cnt ? v[jg + i] : 0.0f;
                li[u][hh] = i < cnt ? idx[jg + i] : 0u;
            }
        }
        if (BITS <= 8 && one_block) {
            float m = 0.0f;
#pragma unroll
            for (int u = 0; u < 4; ++u) m = fmaxf(m, fmaxf(fabsf(x[u][0]), fabsf(x[u][1])));   /* absent ones are 0 */
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) m = fmaxf(m, __shfl_xor(m, d, 64));
            if ((tid & 63) == 0) red[tid >> 6] = m;
            __syncthreads();
            m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
            constexpr float QMAX = BITS == 8 ? 127.0f : 7.0f;
            scale = m == 0.0f ? 0.0f : __fdiv_rn(m, QMAX);
            if (tid == 0) scales[t.S[b] + cb] = scale;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t i0 = b0 + 2 * (tid + u * WG);
            if (i0 >= cnt) continue;
            const int have = (i0 + 1 < cnt) ? 2 : 1;
            float res[2] = {0.0f, 0.0f};
            int q[2] = {0, 0};
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                if (hh >= have) continue;
                const float xv = x[u][hh];
                float deq;
                if (BITS == 32) {
                    deq = xv;
                } else if (BITS == 16) {
                    const __half hv = __float2half_rn(xv);
                    reinterpret_cast<__half *>(vb)[j0 + i0 + hh] = hv;
                    deq = __half2float(hv);
                } else {
                    constexpr float QMAX = BITS == 8 ? 127.0f : 7.0f;
                    if (scale != 0.0f) {
                        float tq = rintf(__fdiv_rn(xv, scale));
                        tq = fminf(fmaxf(tq, -QMAX), QMAX);
                        q[hh] = (int)tq;
                    }
                    deq = __fmul_rn((float)q[hh], scale);
                    if (BITS == 8) reinterpret_cast<int8_t *>(vb)[j0 + i0 + hh] = (int8_t)q[hh];
                }
                res[hh] = __fsub_rn(xv, deq);
            }
            if (BITS == 4) vb[(j0 + i0) >> 1] = (uint8_t)((q[0] & 0xF) | ((q[1] & 0xF) << 4));
#pragma unroll
            for (int hh = 0; hh < 2; ++hh)
                if (hh < have) r[lo + li[u][hh]] = res[hh];
        }
    }
}

/* ------------------------------------------------------------------ decompress */

template <int BITS>
__device__ __forceinline__ float decode(const uint8_t *__restrict__ vb, const float *__restrict__ sc,
                                        uint64_t j, uint32_t chunk, uint32_t chunkSh)
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
    /* the usual chunk lengths are powers of two: a shift instead of a 64-bit division */
    return __fmul_rn((float)q, sc[chunkSh < 64u ? (j >> chunkSh) : j / chunk]);
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

/* The same table by binary search, one thread per tile: cheaper than walking the whole index
 * list once a tile holds many survivors (high ratios).  An index list that is not ascending (an
 * invalid payload) gives entries that are wrong but still within [0, k_b]. */
__global__ __launch_bounds__(WG) void k_tilestart_search(const uint32_t *__restrict__ idx, Tables t, uint32_t n_tiles,
                                                         uint32_t *__restrict__ ts)
{
    const uint32_t g = blockIdx.x * WG + threadIdx.x;
    if (g >= n_tiles) return;
    const uint32_t b = find_bucket<uint32_t>(t.tile0, t.B, g);
    const uint32_t i = g - t.tile0[b], tiles_b = t.tile0[b + 1] - t.tile0[b];
    const uint32_t kb = t.k[b];
    const uint32_t *ib = idx + t.P[b];
    const uint64_t head = t.off[b] & 3ull;
    const uint64_t edge = (uint64_t)i * TILE;           /* survivors with index + head below this come first */
    uint32_t lo = 0, hi = kb;                           /* first j in [0, kb] with ib[j] + head >= edge */
    while (lo < hi) {
        const uint32_t mid = lo + ((hi - lo) >> 1);
        if ((uint64_t)ib[mid] + head < edge) lo = mid + 1; else hi = mid;
    }
    uint32_t *tsb = ts + t.tile0[b] + b;
    tsb[i] = lo;
    if (i + 1 == tiles_b) tsb[tiles_b] = kb;
}

/* Dense output for a span of tiles, the variant for gradients of up to a few hundred million
 * elements and for any gradient whose tiles hold many survivors (256 threads): each tile is
 * assembled in LDS (zeros, then the decoded survivors that fall inside it, found through the
 * tile-start table) and written out once with aligned 16-byte stores, so no output line is
 * touched twice and no atomics are needed.  The loads of the next tile's first survivors are
 * issued before the current tile is written out; a very crowded tile is read four consecutive
 * survivors per thread and load.  A bucket of which every element was sent needs neither LDS
 * nor its index list: its output is the decoded value stream. */
template <int BITS, bool NTS>
__global__ __launch_bounds__(WG) void k_decomp_lds(const uint32_t *__restrict__ idx, const void *__restrict__ val,
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
    if (kb == nb) {
        /* every element of the bucket was sent (ratio 1, or a bucket of one element): survivor j is
         * element j, so the index list (which can only be 0 .. n_b - 1) is not read and the
         * output is a plain decode of the value stream */
        for (uint32_t ti = 0; ti < s.ntiles; ++ti) {
            const uint64_t tb = s.base + (uint64_t)ti * TILE;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint64_t gi = tb + (uint64_t)(u * WG + tid) * 4;
                float x[4];
                if ((BITS == 8 || BITS == 32) && gi >= s.lo && gi + 4 <= s.hi) {
                    /* four consecutive values in one load (the value stream of a bucket starts at
                     * any byte, so the address is not aligned; global loads need not be) */
                    const uint64_t j0 = gi - s.lo;
                    if (BITS == 32) {
                        f4 v;
                        __builtin_memcpy(&v, vb + 4 * j0, 16);
                        x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
                    } else {
                        uint32_t w4;
                        __builtin_memcpy(&w4, vb + j0, 4);
                        const uint64_t c0 = t.chunkSh < 64u ? (j0 >> t.chunkSh) : j0 / t.chunk;
                        const uint64_t c3 = t.chunkSh < 64u ? ((j0 + 3) >> t.chunkSh) : (j0 + 3) / t.chunk;
                        const float s0 = sb[c0], s3 = c3 == c0 ? s0 : sb[c3];
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const int q = (int)(int8_t)(w4 >> (8 * j));
                            const uint64_t cj = t.chunkSh < 64u ? ((j0 + j) >> t.chunkSh) : (j0 + j) / t.chunk;
                            x[j] = __fmul_rn((float)q, cj == c0 ? s0 : s3);
                        }
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        x[j] = (gi + j >= s.lo && gi + j < s.hi) ? decode<BITS>(vb, sb, gi + j - s.lo, t.chunk, t.chunkSh) : 0.0f;
                }
                if (gi >= s.lo && gi + 4 <= s.hi) {
                    const f4 v = {x[0], x[1], x[2], x[3]};
                    if (NTS) __builtin_nontemporal_store(v, reinterpret_cast<f4 *>(dense + gi));
                    else *reinterpret_cast<f4 *>(dense + gi) = v;
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (gi + j >= s.lo && gi + j < s.hi) dense[gi + j] = x[j];
                }
            }
        }
        return;
    }
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
            if (j < j1) { p_li = ib[j]; p_x = decode<BITS>(vb, sb, j, t.chunk, t.chunkSh); }
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
        /* more than 256 survivors in the tile (ratio above 6 %): a thread takes four consecutive
         * ones at a time, indices and codes each in one load (the addresses are not aligned; global
         * loads need not be), two such groups in flight; the last few of a tile one by one */
        const uint32_t j0 = sts[ti], j1 = sts[ti + 1];
        const uint64_t jA = (uint64_t)j0 + WG;
        /* (groups of four only when there is at least one for every thread: otherwise a survivor per thread keeps more of them busy) */
        const uint64_t ngrp = j1 >= jA + 4 * WG ? (j1 - jA) / 4 : 0;      /* whole groups of four */
        for (uint64_t g0 = 0; g0 < ngrp; g0 += 2 * WG) {
            uint32_t li4[2][4];
            float x4[2][4];
#pragma unroll
            for (int v = 0; v < 2; ++v) {
                const uint64_t g = g0 + (uint64_t)v * WG + tid;
#pragma unroll
                for (int u = 0; u < 4; ++u) { li4[v][u] = NONE; x4[v][u] = 0.0f; }
                if (g < ngrp) {
                    const uint64_t j = jA + 4 * g;
                    uint4 iv;
                    __builtin_memcpy(&iv, ib + j, 16);
                    li4[v][0] = iv.x; li4[v][1] = iv.y; li4[v][2] = iv.z; li4[v][3] = iv.w;
                    if (BITS == 8) {
                        uint32_t w4;
                        __builtin_memcpy(&w4, vb + j, 4);
                        const uint64_t c0 = t.chunkSh < 64u ? (j >> t.chunkSh) : j / t.chunk;
                        const uint64_t c3 = t.chunkSh < 64u ? ((j + 3) >> t.chunkSh) : (j + 3) / t.chunk;
                        const float s0 = sb[c0], s3 = c3 == c0 ? s0 : sb[c3];
#pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            const uint64_t cu = t.chunkSh < 64u ? ((j + u) >> t.chunkSh) : (j + u) / t.chunk;
                            x4[v][u] = __fmul_rn((float)(int)(int8_t)(w4 >> (8 * u)), cu == c0 ? s0 : s3);
                        }
                    } else if (BITS == 32) {
                        f4 fv;
                        __builtin_memcpy(&fv, vb + 4 * j, 16);
                        x4[v][0] = fv.x; x4[v][1] = fv.y; x4[v][2] = fv.z; x4[v][3] = fv.w;
                    } else {
#pragma unroll
                        for (int u = 0; u < 4; ++u) x4[v][u] = decode<BITS>(vb, sb, j + u, t.chunk, t.chunkSh);
                    }
                }
            }
#pragma unroll
            for (int v = 0; v < 2; ++v)
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const uint64_t slot = (uint64_t)li4[v][u] + shift;
                    if (li4[v][u] < nb && slot < TILE) tile[slot] = x4[v][u];
                }
        }
        /* what is left (at most three after the groups; everything beyond the first 256 of a less crowded tile) */
        for (uint64_t jb = jA + 4 * ngrp; jb < j1; jb += 4 * WG) {
            uint32_t li1[4];
            float x1[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint64_t j = jb + (uint64_t)u * WG + tid;
                li1[u] = NONE;
                x1[u] = 0.0f;
                if (j < j1) { li1[u] = ib[j]; x1[u] = decode<BITS>(vb, sb, j, t.chunk, t.chunkSh); }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint64_t slot = (uint64_t)li1[u] + shift;
                if (li1[u] < nb && slot < TILE) tile[slot] = x1[u];
            }
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

/* Dense output for a span of tiles, the variant for the largest gradients: one wavefront per
 * tile, 16 wavefronts per workgroup (one span of 16 tiles, two of 8, ...).  A wavefront
 * first fetches its tile's survivors (found through the tile-start table), then writes the
 * tile's 16 KiB of zeros with aligned 16-byte stores, one contiguous KiB per instruction, waits
 * for those stores, and drops the decoded survivors into place.  Both writes to a survivor's
 * line meet in the cache, so the memory sees each output line once; no LDS, no atomics.  (The
 * wait is what orders the two stores to one address: they come from different lanes.) */
template <int BITS, bool NTS>
__global__ __launch_bounds__(64 * MAX_SEG_WAVES) void k_decomp(const uint32_t *__restrict__ idx, const void *__restrict__ val,
                                                               const float *__restrict__ scales, Tables t,
                                                               const uint32_t *__restrict__ ts, float *__restrict__ dense)
{
    constexpr int U = 2;                     /* survivors per lane fetched ahead of the zeros */
    /* a workgroup of 16 wavefronts takes as many whole spans as it has a wavefront per tile for */
    const uint32_t tid = threadIdx.x, lane = tid & 63;
    const uint32_t per_wg = max(1u, (uint32_t)MAX_SEG_WAVES / t.spanT);
    const uint32_t sub = (tid >> 6) / t.spanT;
    const uint32_t span = blockIdx.x * per_wg + min(sub, per_wg - 1u);
    const uint32_t wave = (tid >> 6) - min(sub, per_wg - 1u) * t.spanT;       /* wavefront within its span */
    const uint32_t n_waves = per_wg > 1u ? t.spanT : (uint32_t)(blockDim.x >> 6);
    if (span >= t.n_spans || (per_wg > 1u && sub >= per_wg)) return;
    const SpanGeo s = span_geo(t, span);
    const uint32_t kb = t.k[s.b];
    const uint32_t *ib = idx + t.P[s.b];
    const uint8_t *vb = reinterpret_cast<const uint8_t *>(val) + t.V[s.b];
    const float *sb = BITS <= 8 ? scales + t.S[s.b] : nullptr;
    const uint32_t nb = (uint32_t)(s.hi - s.lo);
    const uint32_t *tsb = ts + t.tile0[s.b] + s.b + (s.tile_g - t.tile0[s.b]);
    const f4 z = {0.f, 0.f, 0.f, 0.f};
    for (uint32_t ti = wave; ti < s.ntiles; ti += n_waves) {
        const uint64_t tb = s.base + (uint64_t)ti * TILE;
        const uint64_t shift = s.lo - tb;                   /* slot in the tile = local index + lo - tb (mod 2^64) */
        const uint32_t j0 = min(tsb[ti], kb), j1 = min(tsb[ti + 1], kb);
        uint32_t p_li[U];
        float p_x[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint64_t j = (uint64_t)j0 + lane + 64u * u;
            p_li[u] = NONE;
            p_x[u] = 0.0f;
            if (j < j1) { p_li[u] = ib[j]; p_x[u] = decode<BITS>(vb, sb, j, t.chunk, t.chunkSh); }
        }
        if (tb >= s.lo && tb + TILE <= s.hi) {
#pragma unroll
            for (int u = 0; u < TILE / 256; ++u) {
                f4 *a = reinterpret_cast<f4 *>(dense + tb + (uint64_t)(u * 64 + lane) * 4);
                if (NTS) __builtin_nontemporal_store(z, a);
                else *a = z;
            }
        } else {
            for (int u = 0; u < TILE / 256; ++u) {
                const uint64_t gi = tb + (uint64_t)(u * 64 + lane) * 4;
                if (gi >= s.lo && gi + 4 <= s.hi) {
                    *reinterpret_cast<f4 *>(dense + gi) = z;
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (gi + j >= s.lo && gi + j < s.hi) dense[gi + j] = 0.0f;
                }
            }
        }
        /* the zeros must have landed before a survivor is stored over one of them */
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_s_waitcnt(0);
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int u = 0; u < U; ++u) {
            /* an index outside the bucket or outside this tile (invalid payload) is dropped */
            const uint64_t slot = (uint64_t)p_li[u] + shift;
            if (p_li[u] < nb && slot < TILE) dense[s.lo + p_li[u]] = p_x[u];
        }
        for (uint64_t j = (uint64_t)j0 + 64u * U + lane; j < j1; j += 64) {
            const uint32_t li = ib[j];
            const uint64_t slot = (uint64_t)li + shift;
            if (li < nb && slot < TILE) dense[s.lo + li] = decode<BITS>(vb, sb, j, t.chunk, t.chunkSh);
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
        const float x = decode<BITS>(vb, sb, jj, t.chunk, t.chunkSh);
        dense[lo + li] = __fadd_rn(dense[lo + li], x);
    }
}

}  // namespace

#endif
