/*
 * libnsml GPU path for gfx950 (MI355X): hand-written HIP kernels and their C-ABI entry points.
 *
 * One compress call = error-feedback accumulation, exact top-k by magnitude per bucket
 * (Sec. 4.2 Step 3 / Algorithm 2 Step 3), value coding and payload packing; one decompress
 * call = payload -> dense gradient.  Nothing here is a dense contraction: every kernel is a
 * streaming pass bound by HBM bandwidth (or, for the small ones, by launch and dependent-load
 * latency), so the work is organised around coalesced 16-byte accesses, LDS histograms, 64-lane
 * ballots and as few dependent launches as possible, not MFMA.
 *
 * Selection is an exact radix select on the 31-bit magnitude key (binary32 pattern with the
 * sign cleared), digits of 12 + 12 + 7 bits, arranged so that the gradient is read ONCE:
 *
 *   sample    level-0 histogram of a 1/64 sample of grad + residual (small buckets: all of it)
 *   predict   per bucket, what the streaming pass stages: everything from a key L_b up that lies,
 *             with a wide margin, below the k-th largest ("candidates", ratios up to an eighth);
 *             a band [L_b, H_b) of keys around the k-th largest (larger ratios); nothing, when
 *             the k-th largest is a zero (sparse embeddings, ratio 1)
 *   ef_emit   acc = grad + residual (written over residual), exact level-0 histogram, a finer
 *             histogram of the four level-0 digits around the expected threshold, and the staged
 *             elements appended, in index order, to per-wavefront segments       12 B/element
 *   plan      per bucket: exact level-0 digit of the k-th key (18 bits of it when the finer
 *             histogram covers it) and the path: PATH_CAND, PATH_BAND, PATH_ZERO when the staged
 *             elements and the counts can decide it, else PATH_DENSE
 *   select_count, select_finish   the staged entries against those bits: counts per segment, the
 *             few undecided keys set aside, then per bucket (one workgroup of 1024 threads) the
 *             remaining bits in LDS -> threshold key T_b, e_b = how many elements equal to T_b
 *             are admitted (lowest indices first), and every segment's place in the survivor order
 *   encode    PATH_CAND: one workgroup per chunk of survivors gathers them from the segments and
 *             codes them (absmax scale, codes, packing, indices, coding error into the residual)
 *   hard      usually one empty launch.  PATH_BAND / PATH_ZERO: survivors taken from the dense
 *             accumulator and coded in one streaming pass; PATH_DENSE (an unlucky sample, a
 *             staging segment that overflowed, huge groups of equal keys): all radix steps over
 *             the dense accumulator, in a small resident grid with barriers between the steps
 *   quant     codes what hard left uncoded (chunks that straddle its work units; PATH_DENSE)
 *   tilestart, decomp    payload -> dense, each output line written once
 * Every path gives the same bytes.
 *
 * With weights (Algorithm 2 Step 2) a weight pass comes first: sample of |w| -> band around the
 * threshold of the kept set (from the second call on: around the threshold the call before
 * found) -> one pass over w that stages the band, counts what lies above it and writes the
 * pruning bitmap for everything outside the band -> threshold and ties from the band with the
 * same select_count / select_finish -> bitmap bits of the band; the gradient kernels then read
 * one bit per element instead of the weight.
 *
 * Geometry: a bucket [lo, hi) is cut into tiles of 4096 elements starting at lo rounded down
 * to a multiple of 4, so every 16-byte access is aligned; elements of an edge tile outside
 * [lo, hi) are masked.  A workgroup owns a span of up to 16 consecutive tiles of one bucket.
 * Workgroups have 256 threads, except in the streaming passes, which run one wavefront per
 * staging segment (256 to 1024 threads), and in select_finish.
 *
 * One translation unit: the device code lives in nsml_device_common.hpp (tables, geometry,
 * histogram helpers), nsml_select.hpp (sample .. plan, the radix steps over the dense
 * accumulator), nsml_prune.hpp (weight pass), nsml_codec.hpp (value coding of leftover chunks,
 * decompress) and nsml_tail.hpp (select_count .. quant, the bitmap kernels); this file holds
 * the context, the launch sequences and the C-ABI entry points.
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

#include "nsml_device_common.hpp"
#include "nsml_select.hpp"
#include "nsml_prune.hpp"
#include "nsml_codec.hpp"
#include "nsml_tail.hpp"

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
    uint32_t *d_sel0;      /* B+1 prefix of the workgroups per bucket of k_select_count */
    uint4 *d_selw;         /* per workgroup of k_select_count: bucket, first and last segment */
    uint32_t *d_chunk_b;   /* per chunk of the payload: its bucket (fixed by layout, ratio, bits) */
    uint32_t *d_chunk_seg; /* per chunk: the staging segment that holds its first survivor */
    uint32_t *d_H, *d_subLo, *d_sh, *d_why, *d_margin, *d_wredo, *d_wprevT, *d_wprevHw, *d_wnband;
    uint32_t *d_lcnt, *d_lkey;   /* k_select_count: lists of undecided keys per workgroup */
    uint64_t max_chunks; uint32_t max_sel;
    uint32_t *d_zero;      /* cleared by every compress call: histograms and overflow flags */
    uint32_t *d_ccnt, *d_cG, *d_cE, *d_cidx;   /* candidate staging */
    float *d_cval;
    float *d_v;            /* survivor values in final order (not used for bits == 32) */
    uint32_t *d_ts;        /* decompress: where each tile's survivors start */
    uint32_t *d_pmask;     /* pruning bitmap, 128 words per tile */
    uint32_t *d_kw, *d_Tw, *d_needw;              /* pruning stage: kept counts, threshold search state */
    uint32_t *d_wfast;                            /* pruning stage: how each bucket was decided */
    uint32_t *d_wLo, *d_wHi;                      /* pruning stage: band of keys staged per bucket */
    uint32_t *h_flags;     /* pinned, mapped: [0] consistency flag of the selection, [1] of the pruning stage */
    uint32_t *d_flags;     /* the same two words as the kernels see them */
    double max_ratio;      /* largest ratio the survivor-value buffer was sized for */
    bool have_prune;                              /* the last compress call had weights */
    double *d_span_sq;     /* per span: sum of grad^2 */
    double *d_l2sq;        /* per bucket: sum of grad^2 of the last compress call */
    bool have_l2;

    /* host copies / caches */
    std::vector<uint64_t> h_off;
    uint32_t B;
    uint64_t n;
    uint32_t n_tiles, n_spans, n_samp, n_sel, spanT, segSh;
    bool tables_valid;
    double t_ratio; int t_bits;       /* what d_k/d_P/... were computed for */
    uint64_t K, NC;                   /* totals for (layout, t_ratio, t_bits) */
    void *pinned; size_t pinned_bytes;
    int span_override;
    int seg_override;      /* wavefronts per workgroup of the streaming pass (0: by span size) */
    int force_dense;
    bool zero_clean; uint32_t zero_B;   /* the per-call histograms and flags were left zeroed (for this many buckets) */
    int persist;           /* workgroups per compute unit of the streaming pass (0: one workgroup per span) */
    int decomp_variant;    /* decompress: 1 direct stores, 0 tiles assembled in LDS, -1 by gradient size */
    int n_cu;
    int hard_occ[2];       /* workgroups of k_hard that fit a compute unit at once (short / long chunks) */
    int whistory;          /* the weight band follows the threshold of the last call (1, default) or always comes from a sample (0) */
    int wband_miss;        /* diagnostic: the weight band is placed beside the threshold, so every bucket takes the repeat */
    int force_rescan;      /* diagnostic: k_select_finish filters the staged entries again instead of using the tails */
    int nt_mode;
    int nt_dense;          /* non-temporal stores for the dense output of decompress: 1, 0, or -1 = by variant */

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
        if (e_ != hipSuccess) { if (ctx) (ctx)->last_hip = (int)e_; return NSML_EHIP; } \
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
uint64_t zero_words(uint64_t B) { return B * (uint64_t)(NB0 + NB0 + NB1 + NB2 + NB1 + NB2 + NBS + 2) + 16; }   /* 16 spare words: counters */

struct Hists { uint32_t *h0, *hs, *c1, *c2, *f1, *f2, *h0b, *ovf, *tail_ovf, *nhard; };
Hists hists_of(const nsml_ctx *c, uint32_t B)
{
    Hists h;
    h.h0 = c->d_zero;
    h.hs = h.h0 + (uint64_t)B * NB0;
    h.c1 = h.hs + (uint64_t)B * NB0;
    h.c2 = h.c1 + (uint64_t)B * NB1;
    h.f1 = h.c2 + (uint64_t)B * NB2;
    h.f2 = h.f1 + (uint64_t)B * NB1;
    h.h0b = h.f2 + (uint64_t)B * NB2;       /* finer counts of a few level-0 digits */
    h.ovf = h.h0b + (uint64_t)B * NBS;
    h.tail_ovf = h.ovf + B;        /* k_select_count: a segment's tail could not hold its undecided keys */
    h.nhard = h.tail_ovf + B;      /* k_plan: buckets not on the candidate path */
    return h;
}

static uint32_t chunk_shift(uint32_t chunk)
{
    if (chunk == 0 || (chunk & (chunk - 1)) != 0) return NONE;
    uint32_t sh = 0;
    while ((1u << sh) != chunk) ++sh;
    return sh;
}

Tables tables_of(const nsml_ctx *c)
{
    Tables t;
    t.off = c->d_off; t.tile0 = c->d_tile0; t.span0 = c->d_span0; t.samp0 = c->d_samp0;
    t.span_b = c->d_span_b;
    t.k = c->d_k; t.P = c->d_P; t.V = c->d_V; t.S = c->d_S; t.C = c->d_C;
    t.T = c->d_T; t.need = c->d_need; t.L = c->d_L; t.H = c->d_H; t.fast = c->d_fast; t.subLo = c->d_subLo; t.sh = c->d_sh; t.why = c->d_why; t.margin = c->d_margin;
    t.ovf = hists_of(c, c->B).ovf; t.fspan0 = c->d_fspan0; t.nhard = hists_of(c, c->B).nhard;
    t.kw = c->d_kw; t.pmask = nullptr;
    t.B = c->B; t.n_spans = c->n_spans; t.spanT = c->spanT; t.segSh = c->segSh; t.chunk = c->chunk; t.chunkSh = chunk_shift(c->chunk);
    t.dencSpans = c->n_spans >= 16u * (uint32_t)c->n_cu ? 2u : 1u;
    return t;
}

Cand cand_of(const nsml_ctx *c)
{
    Cand k;
    k.idx = c->d_cidx; k.val = c->d_cval; k.cnt = c->d_ccnt; k.G = c->d_cG; k.E = c->d_cE;
    k.cap = (c->spanT * (TILE / 4)) >> c->segSh;
    return k;
}

/* Profiling brackets */
int prof_begin(nsml_ctx *c, int kid, hipStream_t st, bool *recorded)
{
    *recorded = false;
    if (!c || !c->prof || c->recs.size() >= 4096) return NSML_OK;
    nsml_ctx::Rec r; r.kid = kid;
    for (hipEvent_t *e : {&r.a, &r.b}) {
        if (!c->pool.empty()) { *e = c->pool.back(); c->pool.pop_back(); }
        else NSML_HIP(c, hipEventCreate(e));
    }
    NSML_HIP(c, hipEventRecord(r.a, st));
    c->recs.push_back(r);
    *recorded = true;
    return NSML_OK;
}
/* closes the record prof_begin opened for this launch (and only if it opened one) */
int prof_end(nsml_ctx *c, bool recorded, hipStream_t st)
{
    if (!recorded) return NSML_OK;
    NSML_HIP(c, hipEventRecord(c->recs.back().b, st));
    return NSML_OK;
}

#define LAUNCHB(ctx, kid, st, kernel, grid, block, ...)                             \
    do {                                                                            \
        bool rec_ = false;                                                          \
        int rc_ = prof_begin(ctx, kid, st, &rec_);                                  \
        if (rc_) return rc_;                                                        \
        hipLaunchKernelGGL(kernel, dim3(grid), dim3(block), 0, st, __VA_ARGS__);    \
        NSML_HIP(ctx, hipGetLastError());                                           \
        rc_ = prof_end(ctx, rec_, st);                                              \
        if (rc_) return rc_;                                                        \
    } while (0)
#define LAUNCH(ctx, kid, st, kernel, grid, ...) LAUNCHB(ctx, kid, st, kernel, grid, WG, __VA_ARGS__)

bool aligned(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

/* Tiles per span (one span = one workgroup of the streaming kernels, with four to sixteen
 * staging segments).  Small spans stream a few per cent faster, large spans mean fewer segments
 * for the candidate kernels to walk; measured on 25 M .. 6.7 G elements the totals favour this.
 * (Spans of 16 tiles, one workgroup of 16 wavefronts per compute unit, lose 1 - 8 % to spans of 8
 * with two workgroups of 8: while one of the two ends and its successor starts, the other keeps
 * streaming.) */
uint32_t pick_span_tiles(uint32_t n_tiles, int override_)
{
    if (override_ >= 1 && override_ <= MAX_SPAN_TILES) return (uint32_t)override_;
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
    std::vector<uint32_t> tile0(B1), span0(B1), samp0(B1), sel0(B1);
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
    /* k_select_count: one workgroup per SELC_SEGS staging segments of a bucket */
    const uint32_t segSh = pick_seg_shift(spanT, c->seg_override);
    uint64_t nsel = 0;
    for (uint32_t b = 0; b < B; ++b) {
        sel0[b] = (uint32_t)nsel;
        const uint64_t segs = (uint64_t)(span0[b + 1] - span0[b]) << segSh;
        nsel += (segs + SELC_SEGS - 1) / SELC_SEGS;
    }
    sel0[B] = (uint32_t)nsel;
    if (nsel > c->max_sel) return NSML_ECAP;

    /* the stream may still be using the old tables */
    NSML_HIP(c, hipStreamSynchronize(st));
    c->tables_valid = false;
    c->B = 0;
    const size_t need = sizeof(uint64_t) * B1 + 4 * sizeof(uint32_t) * B1;
    if (need > c->pinned_bytes) return NSML_ECAP;
    uint8_t *hp = static_cast<uint8_t *>(c->pinned);
    uint8_t *hp_t = hp + sizeof(uint64_t) * B1;
    uint8_t *hp_s = hp_t + sizeof(uint32_t) * B1;
    uint8_t *hp_m = hp_s + sizeof(uint32_t) * B1;
    uint8_t *hp_l = hp_m + sizeof(uint32_t) * B1;
    memcpy(hp_l, sel0.data(), sizeof(uint32_t) * B1);
    memcpy(hp, off, sizeof(uint64_t) * B1);
    memcpy(hp_t, tile0.data(), sizeof(uint32_t) * B1);
    memcpy(hp_s, span0.data(), sizeof(uint32_t) * B1);
    memcpy(hp_m, samp0.data(), sizeof(uint32_t) * B1);
    NSML_HIP(c, hipMemcpyAsync(c->d_off, hp, sizeof(uint64_t) * B1, hipMemcpyHostToDevice, st));
    NSML_HIP(c, hipMemcpyAsync(c->d_tile0, hp_t, sizeof(uint32_t) * B1, hipMemcpyHostToDevice, st));
    NSML_HIP(c, hipMemcpyAsync(c->d_span0, hp_s, sizeof(uint32_t) * B1, hipMemcpyHostToDevice, st));
    NSML_HIP(c, hipMemcpyAsync(c->d_samp0, hp_m, sizeof(uint32_t) * B1, hipMemcpyHostToDevice, st));
    NSML_HIP(c, hipMemcpyAsync(c->d_sel0, hp_l, sizeof(uint32_t) * B1, hipMemcpyHostToDevice, st));
    LAUNCH(c, KID_SPANMAP, st, k_spanmap, (uint32_t)((ns + WG - 1) / WG), (const uint32_t *)c->d_span0, B,
           (uint32_t)ns, c->d_span_b);
    if (nsel)
        LAUNCH(c, KID_SPANMAP, st, k_selmap, (uint32_t)((nsel + WG - 1) / WG), (const uint32_t *)c->d_sel0,
               (const uint32_t *)c->d_span0, B, (uint32_t)nsel, segSh, c->d_selw);
    NSML_HIP(c, hipMemsetAsync(c->d_wprevT, 0xFF, sizeof(uint32_t) * B1, st));     /* other buckets: nothing remembered */
    NSML_HIP(c, hipMemsetAsync(c->d_margin, 0, sizeof(uint32_t) * B1, st));
    NSML_HIP(c, hipStreamSynchronize(st));

    c->h_off.assign(off, off + B + 1);
    c->B = B; c->n = n;
    c->n_tiles = (uint32_t)nt; c->n_spans = (uint32_t)ns; c->n_samp = (uint32_t)nsamp; c->spanT = spanT;
    c->segSh = segSh;
    c->n_sel = (uint32_t)nsel;
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
    if (nc >= 0x7FFFFFFFull || nc > c->max_chunks) return NSML_ECAP;
    LAUNCH(c, KID_SETUP, st, k_setup, 1, tables_of(c), ratio, bits);
    if (nc) LAUNCH(c, KID_SETUP, st, k_chunkmap, (uint32_t)((nc + WG - 1) / WG), (const uint64_t *)c->d_C, c->B, nc, c->d_chunk_b);
    c->K = K; c->NC = nc;
    c->t_ratio = ratio; c->t_bits = bits;
    c->tables_valid = true;
    return NSML_OK;
}

/* A device-side consistency check that tripped during an earlier call is reported once, by the
 * next GPU entry point (the kernels raise the flag in host memory they can reach; reading it
 * needs no synchronisation, so the report comes one call late). */
bool pending_internal_error(nsml_ctx *c)
{
    volatile uint32_t *f = c->h_flags;
    if (!f || (f[0] | f[1]) == 0u) return false;
    f[0] = 0u; f[1] = 0u;
    c->zero_clean = false;
    return true;
}

}  // namespace

extern "C" {

int nsml_create(nsml_ctx **out, int device, uint64_t max_n, uint32_t max_buckets, uint32_t chunk)
{
    return nsml_create_ex(out, device, max_n, max_buckets, chunk, 1.0);
}

int nsml_create_ex(nsml_ctx **out, int device, uint64_t max_n, uint32_t max_buckets, uint32_t chunk,
                   double max_ratio)
{
    if (!out || max_n == 0 || max_buckets == 0 || chunk == 0 || chunk % 8 != 0) return NSML_EINVAL;
    if (!(max_ratio > 0.0 && max_ratio <= 1.0)) return NSML_EINVAL;
    *out = nullptr;
    nsml_ctx *c = new (std::nothrow) nsml_ctx();
    if (!c) return NSML_ENOMEM;
    c->device = device; c->max_n = max_n; c->max_buckets = max_buckets; c->chunk = chunk;
    c->last_hip = 0; c->ws_bytes = 0; c->B = 0; c->n = 0; c->tables_valid = false;
    c->prof = false; c->pinned = nullptr; c->pinned_bytes = 0;
    c->d_off = c->d_P = c->d_V = c->d_S = c->d_C = nullptr;
    c->d_tile0 = c->d_span0 = c->d_samp0 = c->d_span_b = c->d_k = c->d_T = c->d_need = nullptr;
    c->d_L = c->d_fast = c->d_fspan0 = c->d_zero = nullptr;
    c->d_sel0 = nullptr; c->d_selw = nullptr; c->d_chunk_b = c->d_chunk_seg = c->d_H = c->d_subLo = c->d_sh = c->d_why = c->d_margin = c->d_wredo = c->d_wprevT = c->d_wprevHw = c->d_wnband = nullptr;
    c->d_lcnt = c->d_lkey = nullptr;
    c->d_ccnt = c->d_cG = c->d_cE = c->d_cidx = nullptr;
    c->d_cval = nullptr; c->d_v = nullptr; c->d_ts = nullptr; c->d_span_sq = c->d_l2sq = nullptr; c->have_l2 = false;
    c->d_pmask = c->d_kw = c->d_Tw = c->d_needw = c->d_wfast = c->d_wLo = c->d_wHi = nullptr;
    c->h_flags = c->d_flags = nullptr;
    c->have_prune = false;
    c->max_ratio = max_ratio;
    /* tuning switches: the measured defaults (see nsml_set_option) */
    c->span_override = 0; c->seg_override = 0; c->segSh = 2;
    c->zero_clean = false; c->zero_B = 0;
    c->persist = 0; c->decomp_variant = -1; c->n_cu = 256;
    c->force_dense = 0; c->force_rescan = 0; c->wband_miss = 0; c->whistory = 1; c->nt_mode = 7; c->nt_dense = -1;

    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || device < 0 || device >= ndev) {
        c->last_hip = (int)hipErrorInvalidDevice;
        delete c;
        return NSML_EHIP;
    }
    DeviceGuard guard(device);
    if (!guard.ok) { delete c; return NSML_EHIP; }
    {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) == hipSuccess && cus > 0) c->n_cu = cus;
        /* k_hard's workgroups meet at barriers, so its grid must fit the device at once: ask the
         * runtime how many of them a compute unit holds (the variants per width use the same LDS) */
        int occ = 0;
        c->hard_occ[0] = c->hard_occ[1] = 1;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, k_hard<8, false>, (int)WG, 0) == hipSuccess && occ > 0)
            c->hard_occ[0] = occ < (int)hard_wg_per_cu(false) ? occ : (int)hard_wg_per_cu(false);
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, k_hard<8, true>, (int)WG, 0) == hipSuccess && occ > 0)
            c->hard_occ[1] = occ < (int)hard_wg_per_cu(true) ? occ : (int)hard_wg_per_cu(true);
        (void)hipGetLastError();
    }

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
    A(dev_alloc(c, &c->d_sel0, B1)); A(dev_alloc(c, &c->d_H, B1)); A(dev_alloc(c, &c->d_subLo, B1)); A(dev_alloc(c, &c->d_sh, B1)); A(dev_alloc(c, &c->d_why, B1)); A(dev_alloc(c, &c->d_margin, B1));
    A(dev_alloc(c, &c->d_span_b, mt));
    A(dev_alloc(c, &c->d_zero, zero_words(max_buckets)));
    /* segments: at most 4 per tile-sized span, or one per tile plus a partly filled span per bucket */
    const uint64_t msg = 4 * mt + (uint64_t)MAX_SEG_WAVES * B1;
    A(dev_alloc(c, &c->d_ccnt, msg)); A(dev_alloc(c, &c->d_cG, msg)); A(dev_alloc(c, &c->d_cE, msg));
    /* k_select_count workgroups: 16 segments each; the geometries the library picks itself have
     * at most one segment per tile from 16384 tiles up */
    c->max_sel = (uint32_t)(((mt > 16384 ? mt : 16384) + (uint64_t)MAX_SEG_WAVES * B1) / SELC_SEGS + B1);
    A(dev_alloc(c, &c->d_selw, c->max_sel));
    A(dev_alloc(c, &c->d_lcnt, c->max_sel));
    A(dev_alloc(c, &c->d_lkey, (uint64_t)c->max_sel * LCAP));
    A(dev_alloc(c, &c->d_cidx, c->max_cand)); A(dev_alloc(c, &c->d_cval, c->max_cand));
    {   /* survivor values in final order: ceil(ratio * n_b) per bucket, at most one more than
         * ratio * n_b each */
        uint64_t mv = (uint64_t)ceil(max_ratio * (double)max_n) + max_buckets;
        if (mv > max_n) mv = max_n;
        A(dev_alloc(c, &c->d_v, mv));
        /* chunks of the payload: every bucket can end with a short one */
        c->max_chunks = mv / chunk + max_buckets + 1;
        A(dev_alloc(c, &c->d_chunk_b, c->max_chunks)); A(dev_alloc(c, &c->d_chunk_seg, c->max_chunks));
    }
    A(dev_alloc(c, &c->d_ts, mt + B1 + 1));
    A(dev_alloc(c, &c->d_span_sq, mt)); A(dev_alloc(c, &c->d_l2sq, B1));
    A(dev_alloc(c, &c->d_pmask, mt * (TILE / 32)));
    A(dev_alloc(c, &c->d_kw, B1)); A(dev_alloc(c, &c->d_Tw, B1)); A(dev_alloc(c, &c->d_needw, B1));
    A(dev_alloc(c, &c->d_wfast, B1));
    A(dev_alloc(c, &c->d_wLo, B1)); A(dev_alloc(c, &c->d_wHi, B1));
    A(dev_alloc(c, &c->d_wredo, B1));
    A(dev_alloc(c, &c->d_wprevT, B1)); A(dev_alloc(c, &c->d_wprevHw, B1)); A(dev_alloc(c, &c->d_wnband, B1));
    if (rc == NSML_OK) {
        hipError_t e = hipMemset(c->d_wredo, 0, sizeof(uint32_t) * B1);
        if (e == hipSuccess) e = hipMemset(c->d_margin, 0, sizeof(uint32_t) * B1);
        if (e == hipSuccess) e = hipMemset(c->d_wprevT, 0xFF, sizeof(uint32_t) * B1);   /* nothing remembered */
        if (e != hipSuccess) { c->last_hip = (int)e; rc = NSML_EHIP; }
    }
    if (rc == NSML_OK) {
        c->pinned_bytes = B1 * 24;
        hipError_t e = hipHostMalloc(&c->pinned, c->pinned_bytes, hipHostMallocDefault);
        if (e != hipSuccess) { c->last_hip = (int)e; rc = NSML_EHIP; }
    }
    if (rc == NSML_OK) {
        /* two words the kernels write only when a consistency check fails; the host reads them
         * at the start of the next call, without waiting for anything */
        void *hp = nullptr, *dp = nullptr;
        hipError_t e = hipHostMalloc(&hp, 64, hipHostMallocMapped);
        if (e == hipSuccess) {
            c->h_flags = static_cast<uint32_t *>(hp);
            c->h_flags[0] = c->h_flags[1] = 0u;
            e = hipHostGetDevicePointer(&dp, hp, 0);
        }
        if (e != hipSuccess) { c->last_hip = (int)e; rc = NSML_EHIP; }
        else c->d_flags = static_cast<uint32_t *>(dp);
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
                    c->d_zero, c->d_ccnt, c->d_cG, c->d_cE, c->d_cidx,
                    c->d_cval, c->d_v, c->d_ts, c->d_span_sq, c->d_l2sq, c->d_pmask, c->d_kw,
                    c->d_Tw, c->d_needw, c->d_wfast,
                    c->d_wLo, c->d_wHi, c->d_sel0, c->d_selw, c->d_chunk_b, c->d_chunk_seg, c->d_H, c->d_lcnt, c->d_lkey, c->d_subLo, c->d_sh, c->d_why, c->d_margin, c->d_wredo, c->d_wprevT, c->d_wprevHw, c->d_wnband};
    for (void *p : ptrs) if (p) (void)hipFree(p);
    if (c->pinned) (void)hipHostFree(c->pinned);
    if (c->h_flags) (void)hipHostFree(c->h_flags);
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
    if (ratio > c->max_ratio) return NSML_ECAP;
    if (pending_internal_error(c)) return NSML_EINTERNAL;
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
    uint32_t egrid = c->n_spans;         /* streaming pass: one workgroup per span, or a fixed number per compute unit */
    if (c->persist > 0 && (uint32_t)(c->persist * c->n_cu) < egrid) egrid = (uint32_t)(c->persist * c->n_cu);

    if (weights) {
        /* Algorithm 2 Step 2: threshold and cut of |w| per bucket (bitmap for the buckets that
         * had to take the dense passes), on its own set of tables */
        Tables tw = t;
        tw.k = c->d_kw; tw.T = c->d_Tw; tw.need = c->d_needw; tw.fast = c->d_wfast;
        tw.L = c->d_wLo; tw.H = c->d_wHi;              /* the staged band of weight keys (H is never NONE here) */
        const Cand cdw = cd0;
        LAUNCH(c, KID_CLEAR, st, k_clear, clear_grid < 2048 ? clear_grid : 2048, c->d_zero, zw);
        if (!c->force_dense)
            LAUNCH(c, KID_SAMPLE, st, k_sample<false>, c->n_samp, weights, (const float *)nullptr, tw, h.hs);
        LAUNCH(c, KID_WPLAN, st, k_wpredict, B, tw, (const uint32_t *)h.hs, c->d_wLo, c->d_wHi, c->force_dense,
               c->wband_miss, c->whistory ? (const uint32_t *)c->d_wprevT : (const uint32_t *)nullptr,
               (const uint32_t *)c->d_wprevHw);
        LAUNCHB(c, KID_WHIST, st, k_whist, c->n_spans, eblock, weights, tw, h.h0, cdw,
                (const uint32_t *)c->d_wLo, (const uint32_t *)c->d_wHi, c->d_pmask, (const uint32_t *)c->d_wredo, 0);
        LAUNCH(c, KID_WPLAN, st, k_wplan, B, tw, h.h0, cdw, (const uint32_t *)c->d_wLo,
               (const uint32_t *)c->d_wHi, c->d_wredo, c->d_wnband, 0);
        /* the buckets whose band missed the threshold (rare): the pass again, exact histogram */
        LAUNCHB(c, KID_WHIST, st, k_whist, c->n_spans, eblock, weights, tw, h.h0, cdw,
                (const uint32_t *)c->d_wLo, (const uint32_t *)c->d_wHi, c->d_pmask, (const uint32_t *)c->d_wredo, 1);
        LAUNCH(c, KID_WPLAN, st, k_wplan, B, tw, h.h0, cdw, (const uint32_t *)c->d_wLo,
               (const uint32_t *)c->d_wHi, c->d_wredo, c->d_wnband, 1);
        /* buckets decided from their band: undecided keys, threshold key and tie count, the pruned
         * band elements' bits; buckets on the dense passes: everything in one resident launch */
        if (!c->force_dense) {
            LAUNCH(c, KID_SELECT, st, k_select_count, c->n_sel, tw, cdw, (const uint4 *)c->d_selw, h.tail_ovf, c->d_lcnt, c->d_lkey, weights);
            LAUNCHB(c, KID_FINISH, st, k_select_finish, B, SEL_THREADS, tw, cdw, (const uint32_t *)c->d_sel0, h.tail_ovf,
                    (const uint32_t *)c->d_lcnt, (const uint32_t *)c->d_lkey, (uint32_t *)nullptr, c->d_flags + 1,
                    c->force_rescan, weights);
            LAUNCH(c, KID_WMASK, st, k_wfix, (n_ss + 15) / 16, tw, cdw, c->d_pmask);
        }
        LAUNCH(c, KID_WHARD, st, k_whard, (uint32_t)c->n_cu, weights, tw, cdw, h.f1, h.f2, c->d_pmask, c->d_flags + 1);
        LAUNCH(c, KID_WPLAN, st, k_wremember, (B + WG - 1) / WG, tw, (const uint32_t *)c->d_Tw, (const uint32_t *)c->d_wLo,
               (const uint32_t *)c->d_wHi, (const uint32_t *)c->d_wnband, c->d_wprevT, c->d_wprevHw);
        t.pmask = c->d_pmask;
    }

    const bool pruned = weights != nullptr;
    /* the kernels below zero what they have read of the per-call histograms and flags, so a fill
     * is only needed after something else used the area: the weight stage, another bucket
     * count, a call that did not get to its end */
    if (pruned || !c->zero_clean || c->zero_B != B)
        LAUNCH(c, KID_CLEAR, st, k_clear, clear_grid < 2048 ? clear_grid : 2048, c->d_zero, zw);
    c->zero_clean = false;
    if (!c->force_dense)
        LAUNCH(c, KID_SAMPLE, st, k_sample<true>, c->n_samp, grad, (const float *)residual, t, h.hs);
    LAUNCH(c, KID_PREDICT, st, k_predict, B, t, h.hs, c->force_dense);
    if (c->force_dense) {
        if (weights) LAUNCHB(c, KID_EF_EMIT, st, (k_ef_emit<false, 7, true>), egrid, eblock, grad, residual, t, h.h0, h.h0b, cd0, c->d_span_sq);
        else LAUNCHB(c, KID_EF_EMIT, st, (k_ef_emit<false, 7, false>), egrid, eblock, grad, residual, t, h.h0, h.h0b, cd0, c->d_span_sq);
    } else if (weights) {
        LAUNCHB(c, KID_EF_EMIT, st, (k_ef_emit<true, 7, true>), egrid, eblock, grad, residual, t, h.h0, h.h0b, cd0, c->d_span_sq);
    } else {
        switch (c->nt_mode) {
        case 1:  LAUNCHB(c, KID_EF_EMIT, st, (k_ef_emit<true, 1, false>), egrid, eblock, grad, residual, t, h.h0, h.h0b, cd0, c->d_span_sq); break;
        case 3:  LAUNCHB(c, KID_EF_EMIT, st, (k_ef_emit<true, 3, false>), egrid, eblock, grad, residual, t, h.h0, h.h0b, cd0, c->d_span_sq); break;
        case 5:  LAUNCHB(c, KID_EF_EMIT, st, (k_ef_emit<true, 5, false>), egrid, eblock, grad, residual, t, h.h0, h.h0b, cd0, c->d_span_sq); break;
        default: LAUNCHB(c, KID_EF_EMIT, st, (k_ef_emit<true, 7, false>), egrid, eblock, grad, residual, t, h.h0, h.h0b, cd0, c->d_span_sq); break;
        }
    }
    LAUNCH(c, KID_PLAN, st, k_plan, B, t, h.h0, h.h0b, cd0, c->force_dense ? 0 : 1,
           (const double *)c->d_span_sq, c->d_l2sq);
    const uint32_t qgrid = (uint32_t)c->NC;
    if (!c->force_dense) {
        /* buckets decided from their staged elements: undecided keys set apart, threshold and
         * survivor order per bucket, then the payload of the candidate-path buckets */
        const uint4 *selw = c->d_selw;
        LAUNCH(c, KID_SELECT, st, k_select_count, c->n_sel, t, cd0, selw, h.tail_ovf, c->d_lcnt, c->d_lkey, (const float *)residual);
        LAUNCHB(c, KID_FINISH, st, k_select_finish, B, SEL_THREADS, t, cd0, (const uint32_t *)c->d_sel0, h.tail_ovf,
                (const uint32_t *)c->d_lcnt, (const uint32_t *)c->d_lkey, c->d_chunk_seg, c->d_flags,
                c->force_rescan, (const float *)residual);
        {
            const uint32_t *cb_ = c->d_chunk_b, *cs_ = c->d_chunk_seg;
            const uint64_t nc64e = c->NC;
            const uint32_t cpw = c->NC > (1ull << 14) ? 16u : 1u;     /* very many chunks: fewer, longer-lived workgroups */
            const uint32_t egrid2 = (uint32_t)((c->NC + cpw - 1) / cpw);
            switch (bits) {
            case 32: LAUNCH(c, KID_ENCODE, st, k_encode<32>, egrid2, t, cd0, cb_, cs_, residual, idx, val, scales, c->d_flags, nc64e, cpw); break;
            case 16: LAUNCH(c, KID_ENCODE, st, k_encode<16>, egrid2, t, cd0, cb_, cs_, residual, idx, val, scales, c->d_flags, nc64e, cpw); break;
            case 8:  LAUNCH(c, KID_ENCODE, st, k_encode<8>, egrid2, t, cd0, cb_, cs_, residual, idx, val, scales, c->d_flags, nc64e, cpw); break;
            default: LAUNCH(c, KID_ENCODE, st, k_encode<4>, egrid2, t, cd0, cb_, cs_, residual, idx, val, scales, c->d_flags, nc64e, cpw); break;
            }
        }
    }
    /* the buckets whose survivors come from the dense accumulator (usually none: the workgroups
     * read one word and leave): a fixed grid, resident at once, that streams the band and
     * zero-threshold buckets (ordered write and coding in one pass) and then does all the steps of
     * the buckets on the dense passes with barriers between; then the value coding of what those
     * left uncoded */
    {
        const bool big = c->chunk > DENC_SMALL_CHUNK;
        const uint32_t hgrid = (uint32_t)(c->hard_occ[big ? 1 : 0] * c->n_cu);
        /* the workgroups that meet at barriers: one per compute unit, so that the teams of two or
         * three contexts working at the same time still fit the device together */
        const uint32_t team = (uint32_t)c->n_cu < hgrid ? (uint32_t)c->n_cu : hgrid;
        const uint32_t *cb_ = c->d_chunk_b, *cs_ = c->d_chunk_seg;
        const int stream_coding = c->chunk <= DENC_MAX_CHUNK ? 1 : 0;
#define NSML_HARD(BITS_, BIG_) LAUNCH(c, KID_HARD, st, (k_hard<BITS_, BIG_>), hgrid, residual, t, cd0, h.f1, h.f2, idx, vdst, val, scales, c->d_flags, stream_coding, team)
        switch (bits) {
        case 32: NSML_HARD(32, false); break;
        case 16: if (big) NSML_HARD(16, true); else NSML_HARD(16, false); break;
        case 8:  if (big) NSML_HARD(8, true); else NSML_HARD(8, false); break;
        default: if (big) NSML_HARD(4, true); else NSML_HARD(4, false); break;
        }
#undef NSML_HARD
        const uint32_t per_wg = (WG / 64) * QUANT_PER_WAVE;
        const uint32_t ngrid = c->chunk <= QUANT_WAVE_CHUNK ? (qgrid + per_wg - 1) / per_wg
                                                            : (qgrid + QUANT_BIG_PER_WG - 1) / QUANT_BIG_PER_WG;
        const uint64_t nc64 = c->NC;
        switch (bits) {
        case 32: break;        /* the ordered write left values and residual in their final state */
        case 16: LAUNCH(c, KID_QUANT, st, k_quant<16>, ngrid, (const float *)vdst, (const uint32_t *)idx, t, cd0, residual, val, scales, cb_, cs_, nc64, stream_coding); break;
        case 8:  LAUNCH(c, KID_QUANT, st, k_quant<8>,  ngrid, (const float *)vdst, (const uint32_t *)idx, t, cd0, residual, val, scales, cb_, cs_, nc64, stream_coding); break;
        default: LAUNCH(c, KID_QUANT, st, k_quant<4>,  ngrid, (const float *)vdst, (const uint32_t *)idx, t, cd0, residual, val, scales, cb_, cs_, nc64, stream_coding); break;
        }
    }
    c->have_l2 = true;
    c->have_prune = pruned;
    c->zero_clean = true;
    c->zero_B = B;
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

/* The launches of one decompress: tile-start table, then the dense output.  c may be NULL
 * (the entry point without a context): then nothing is profiled and no error code is kept. */
static int launch_decompress(nsml_ctx *c, hipStream_t st, const Tables &t, uint64_t K, uint32_t n_spans, uint32_t n_tiles,
                             uint32_t *d_ts, int nt_dense, int variant, const uint32_t *idx, const void *val,
                             const float *scales, int bits, float *dense_out)
{
    const bool crowded = K >= 64ull * n_tiles;           /* many survivors per tile */
    if (crowded) {
        LAUNCH(c, KID_TILESTART, st, k_tilestart_search, (n_tiles + WG - 1) / WG, idx, t, n_tiles, d_ts);
    } else if (K >= (4ull << 20)) {
        const uint64_t want = (K + (uint64_t)WG * 8 - 1) / ((uint64_t)WG * 8);
        LAUNCH(c, KID_TILESTART, st, k_tilestart<8>, (uint32_t)(want < 16384 ? want : 16384), idx, t, K, d_ts);
    } else {
        const uint64_t want = (K + (uint64_t)WG * 2 - 1) / ((uint64_t)WG * 2);
        LAUNCH(c, KID_TILESTART, st, k_tilestart<2>, (uint32_t)want, idx, t, K, d_ts);
    }
    const uint32_t *ts = d_ts;
    if (variant > 0 || (variant < 0 && n_tiles >= 16u * 4096u && !crowded)) {
        /* the largest gradients at low ratios: one wavefront per tile, direct stores (plain unless asked
         * otherwise); 16 wavefronts per workgroup, which take 16 / spanT whole spans */
        const uint32_t dblock = 64u * MAX_SEG_WAVES;
        const uint32_t per_wg = MAX_SEG_WAVES / t.spanT ? MAX_SEG_WAVES / t.spanT : 1u;
        n_spans = (n_spans + per_wg - 1) / per_wg;
        if (nt_dense > 0) {
            switch (bits) {
            case 32: LAUNCHB(c, KID_DECOMP, st, (k_decomp<32, true>), n_spans, dblock, idx, val, scales, t, ts, dense_out); break;
            case 16: LAUNCHB(c, KID_DECOMP, st, (k_decomp<16, true>), n_spans, dblock, idx, val, scales, t, ts, dense_out); break;
            case 8:  LAUNCHB(c, KID_DECOMP, st, (k_decomp<8, true>),  n_spans, dblock, idx, val, scales, t, ts, dense_out); break;
            default: LAUNCHB(c, KID_DECOMP, st, (k_decomp<4, true>),  n_spans, dblock, idx, val, scales, t, ts, dense_out); break;
            }
        } else {
            switch (bits) {
            case 32: LAUNCHB(c, KID_DECOMP, st, (k_decomp<32, false>), n_spans, dblock, idx, val, scales, t, ts, dense_out); break;
            case 16: LAUNCHB(c, KID_DECOMP, st, (k_decomp<16, false>), n_spans, dblock, idx, val, scales, t, ts, dense_out); break;
            case 8:  LAUNCHB(c, KID_DECOMP, st, (k_decomp<8, false>),  n_spans, dblock, idx, val, scales, t, ts, dense_out); break;
            default: LAUNCHB(c, KID_DECOMP, st, (k_decomp<4, false>),  n_spans, dblock, idx, val, scales, t, ts, dense_out); break;
            }
        }
    } else if (nt_dense != 0) {
        /* smaller gradients: tiles assembled in LDS, non-temporal stores unless asked otherwise */
        switch (bits) {
        case 32: LAUNCH(c, KID_DECOMP, st, (k_decomp_lds<32, true>), n_spans, idx, val, scales, t, ts, dense_out); break;
        case 16: LAUNCH(c, KID_DECOMP, st, (k_decomp_lds<16, true>), n_spans, idx, val, scales, t, ts, dense_out); break;
        case 8:  LAUNCH(c, KID_DECOMP, st, (k_decomp_lds<8, true>),  n_spans, idx, val, scales, t, ts, dense_out); break;
        default: LAUNCH(c, KID_DECOMP, st, (k_decomp_lds<4, true>),  n_spans, idx, val, scales, t, ts, dense_out); break;
        }
    } else {
        switch (bits) {
        case 32: LAUNCH(c, KID_DECOMP, st, (k_decomp_lds<32, false>), n_spans, idx, val, scales, t, ts, dense_out); break;
        case 16: LAUNCH(c, KID_DECOMP, st, (k_decomp_lds<16, false>), n_spans, idx, val, scales, t, ts, dense_out); break;
        case 8:  LAUNCH(c, KID_DECOMP, st, (k_decomp_lds<8, false>),  n_spans, idx, val, scales, t, ts, dense_out); break;
        default: LAUNCH(c, KID_DECOMP, st, (k_decomp_lds<4, false>),  n_spans, idx, val, scales, t, ts, dense_out); break;
        }
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
    if (pending_internal_error(c)) return NSML_EINTERNAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    DeviceGuard guard(c->device);
    if (!guard.ok) { c->last_hip = (int)hipErrorInvalidDevice; return NSML_EHIP; }
    int rc = ensure_layout(c, n, bucket_off, B, st);
    if (rc) return rc;
    rc = ensure_tables(c, ratio, bits, st);
    if (rc) return rc;
    return launch_decompress(c, st, tables_of(c), c->K, c->n_spans, c->n_tiles, c->d_ts, c->nt_dense, c->decomp_variant, idx, val, scales,
                             bits, dense_out);
}

/* ---------------------------------------------------------------- no-allocation decompress */

}  // extern "C"

/* Scratch of nsml_decompress_static: the layout tables and the tile-start table of one call.
 * One copy per GPU, at its own address on each; host code never uses this name as a pointer,
 * only what hipGetSymbolAddress returns for the current device. */
static __device__ __align__(256) unsigned char scratch[NSML_STATIC_SCRATCH_BYTES];

namespace {

constexpr int STATIC_MAX_DEVICES = 64;
void *g_scratch_ptr[STATIC_MAX_DEVICES];        /* per device, resolved on the first call there */

constexpr uint32_t STATIC_B1 = NSML_STATIC_MAX_BUCKETS + 1;
constexpr uint64_t STATIC_MAX_TILES = NSML_STATIC_MAX_N / TILE + 2ull * NSML_STATIC_MAX_BUCKETS + 2;

struct StaticOffsets { uint64_t off[STATIC_B1]; };      /* travels as a kernel argument */

/* where each table sits inside the scratch array */
struct StaticScratch {
    uint64_t *off, *P, *V, *S, *C;
    uint32_t *tile0, *span0, *k, *kw, *span_b, *ts;
};
StaticScratch carve(void *base)
{
    StaticScratch m;
    uint64_t *q = static_cast<uint64_t *>(base);
    m.off = q; q += STATIC_B1;
    m.P = q; q += STATIC_B1;
    m.V = q; q += STATIC_B1;
    m.S = q; q += STATIC_B1;
    m.C = q; q += STATIC_B1;
    uint32_t *w = reinterpret_cast<uint32_t *>(q);
    m.tile0 = w; w += STATIC_B1 + 1;
    m.span0 = w; w += STATIC_B1 + 1;
    m.k = w; w += STATIC_B1 + 1;
    m.kw = w; w += STATIC_B1 + 1;
    m.span_b = w; w += STATIC_MAX_TILES;
    m.ts = w; w += STATIC_MAX_TILES + STATIC_B1 + 1;
    return m;
}
static_assert(5 * STATIC_B1 * 8 + 4 * (STATIC_B1 + 1) * 4 + (2 * STATIC_MAX_TILES + STATIC_B1 + 1) * 4
                  <= NSML_STATIC_SCRATCH_BYTES, "scratch array too small for its tables");
static_assert(sizeof(StaticOffsets) <= 3072, "bucket offsets must fit the kernel argument block");

/* One workgroup: bucket offsets (handed over by value) and the tile / span prefixes they imply. */
__global__ __launch_bounds__(WG) void k_static_layout(StaticOffsets so, uint32_t B, uint32_t spanT,
                                                      uint64_t *__restrict__ off, uint32_t *__restrict__ tile0,
                                                      uint32_t *__restrict__ span0)
{
    for (uint32_t b = threadIdx.x; b <= B; b += WG) off[b] = so.off[b];
    if (threadIdx.x == 0) {
        uint32_t nt = 0, ns = 0;
        for (uint32_t b = 0; b < B; ++b) {
            tile0[b] = nt; span0[b] = ns;
            const uint64_t lo = so.off[b], hi = so.off[b + 1];
            const uint32_t tb = hi > lo ? (uint32_t)((hi - (lo & ~3ull) + TILE - 1) / TILE) : 0u;
            nt += tb;
            ns += (tb + spanT - 1) / spanT;
        }
        tile0[B] = nt; span0[B] = ns;
    }
}

}  // namespace

extern "C" {

int nsml_decompress_static(const uint32_t *idx, const void *val, const float *scales, uint64_t n,
                           const uint64_t *bucket_off, uint32_t B, double ratio, int bits,
                           uint32_t chunk, float *dense_out, void *stream)
{
    if (!idx || !val || !dense_out || !bucket_off || B == 0 || n == 0) return NSML_EINVAL;
    if ((bits == 8 || bits == 4) && !scales) return NSML_EINVAL;
    if (!aligned(dense_out, 16) || !aligned(idx, 4) || !aligned(val, 4) || !aligned(scales, 4))
        return NSML_EINVAL;
    if (B > NSML_STATIC_MAX_BUCKETS || n > NSML_STATIC_MAX_N) return NSML_ECAP;
    if (bucket_off[0] != 0 || bucket_off[B] != n) return NSML_EINVAL;
    uint64_t K = 0;
    int rc = nsml_payload_layout(bucket_off, B, ratio, bits, chunk, nullptr, &K, nullptr, nullptr);
    if (rc) return rc;                      /* also rejects descending offsets, bad ratio / bits / chunk */
    /* the same geometry a context would build, computed without any table on the host */
    uint64_t nt = 0, ns = 0;
    for (uint32_t b = 0; b < B; ++b) {
        const uint64_t lo = bucket_off[b], hi = bucket_off[b + 1];
        if (hi > lo) nt += (hi - (lo & ~3ull) + TILE - 1) / TILE;
    }
    if (nt > STATIC_MAX_TILES) return NSML_ECAP;
    const uint32_t spanT = pick_span_tiles((uint32_t)nt, 0);
    StaticOffsets so;
    for (uint32_t b = 0; b < B; ++b) {
        const uint64_t lo = bucket_off[b], hi = bucket_off[b + 1];
        const uint64_t tb = hi > lo ? (hi - (lo & ~3ull) + TILE - 1) / TILE : 0;
        ns += (tb + spanT - 1) / spanT;
        so.off[b] = lo;
    }
    so.off[B] = n;
    for (uint32_t b = B + 1; b < STATIC_B1; ++b) so.off[b] = n;

    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= STATIC_MAX_DEVICES) return NSML_EHIP;
    void *base = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
    if (!base) {
        /* this GPU's copy of the array; the symbol's own name is no device address on the host */
        if (hipGetSymbolAddress(&base, HIP_SYMBOL(scratch)) != hipSuccess || !base) return NSML_EHIP;
        __atomic_store_n(&g_scratch_ptr[dev], base, __ATOMIC_RELEASE);
    }
    const StaticScratch m = carve(base);
    hipStream_t st = static_cast<hipStream_t>(stream);
    nsml_ctx *none = nullptr;

    Tables t;
    memset(&t, 0, sizeof t);
    t.off = m.off; t.tile0 = m.tile0; t.span0 = m.span0; t.span_b = m.span_b;
    t.k = m.k; t.kw = m.kw; t.P = m.P; t.V = m.V; t.S = m.S; t.C = m.C;
    t.B = B; t.n_spans = (uint32_t)ns; t.spanT = spanT; t.segSh = 2; t.chunk = chunk; t.chunkSh = chunk_shift(chunk); t.dencSpans = 1;
    LAUNCH(none, KID_SETUP, st, k_static_layout, 1, so, B, spanT, m.off, m.tile0, m.span0);
    LAUNCH(none, KID_SETUP, st, k_setup, 1, t, ratio, bits);
    LAUNCH(none, KID_SPANMAP, st, k_spanmap, (uint32_t)((ns + WG - 1) / WG), (const uint32_t *)m.span0, B,
           (uint32_t)ns, m.span_b);
    return launch_decompress(none, st, t, K, (uint32_t)ns, (uint32_t)nt, m.ts, -1, -1, idx, val, scales, bits, dense_out);
}

int nsml_decompress_accumulate(nsml_ctx *c, const uint32_t *idx, const void *val, const float *scales,
                               uint64_t n, const uint64_t *bucket_off, uint32_t B, double ratio,
                               int bits, float *dense_inout, void *stream)
{
    if (!c || !idx || !val || !dense_inout) return NSML_EINVAL;
    if ((bits == 8 || bits == 4) && !scales) return NSML_EINVAL;
    if (!aligned(dense_inout, 16) || !aligned(idx, 4) || !aligned(val, 4) || !aligned(scales, 4))
        return NSML_EINVAL;
    if (pending_internal_error(c)) return NSML_EINTERNAL;
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
    return *(volatile uint32_t *)&c->h_flags[0] ? NSML_EINTERNAL : NSML_OK;
}

int nsml_bucket_state(nsml_ctx *c, uint32_t b, uint32_t *out8)
{
    if (!c || !out8 || b >= c->B) return NSML_EINVAL;
    DeviceGuard guard(c->device);
    NSML_HIP(c, hipDeviceSynchronize());
    const uint32_t *src[8] = {c->d_fast, c->d_why, c->d_L, c->d_H, c->d_T, c->d_need, c->d_sh, c->d_k};
    for (int i = 0; i < 8; ++i)
        NSML_HIP(c, hipMemcpy(out8 + i, src[i] + b, sizeof(uint32_t), hipMemcpyDeviceToHost));
    return NSML_OK;
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
    return *(volatile uint32_t *)&c->h_flags[1] ? NSML_EINTERNAL : NSML_OK;
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

int nsml_set_option(nsml_ctx *c, const char *name, int value)
{
    if (!c || !name) return NSML_EINVAL;
    auto is = [&](const char *s) { return strcmp(name, s) == 0; };
    if (is("span_tiles")) {
        if (value < 0 || value > MAX_SPAN_TILES) return NSML_EINVAL;
        c->span_override = value;
        c->B = 0;                              /* the geometry changes: rebuild the layout tables */
        c->tables_valid = false;
    } else if (is("seg_waves")) {
        if (value != 0 && value != 4 && value != 8 && value != 16) return NSML_EINVAL;
        c->seg_override = value;
        c->B = 0;
        c->tables_valid = false;
    } else if (is("force_dense")) {
        if (value != 0 && value != 1) return NSML_EINVAL;
        c->force_dense = value;
    } else if (is("nt")) {
        if (value != 1 && value != 3 && value != 5 && value != 7) return NSML_EINVAL;
        c->nt_mode = value;
    } else if (is("nt_dense")) {
        if (value < -1 || value > 1) return NSML_EINVAL;
        c->nt_dense = value;
    } else if (is("persist")) {
        if (value < 0 || value > 8) return NSML_EINVAL;
        c->persist = value;
    } else if (is("decomp_variant")) {
        if (value < -1 || value > 1) return NSML_EINVAL;
        c->decomp_variant = value;
    } else if (is("rescan")) {
        if (value != 0 && value != 1) return NSML_EINVAL;
        c->force_rescan = value;
    } else if (is("whistory")) {
        if (value != 0 && value != 1) return NSML_EINVAL;
        c->whistory = value;
    } else if (is("wband_miss")) {
        if (value != 0 && value != 1) return NSML_EINVAL;
        c->wband_miss = value;
    } else if (is("trip_check")) {
        if (value != 1) return NSML_EINVAL;
        *(volatile uint32_t *)&c->h_flags[0] = 1u;
    } else {
        return NSML_EINVAL;
    }
    return NSML_OK;
}

int nsml_calibration_stream(int mode, const void *a, void *b, uint64_t bytes, int nontemporal, void *stream)
{
    constexpr uint64_t PER_WG = 16ull * 16384ull;      /* 16 wavefronts x 16 KiB */
    if (!a || !b || bytes == 0 || bytes % PER_WG != 0 || !aligned(a, 16) || !aligned(b, 16)) return NSML_EINVAL;
    if (mode < 0 || mode > 3) return NSML_EINVAL;
    const uint64_t wgs = bytes / PER_WG;
    if (wgs > 0x7FFFFFFFull) return NSML_ECAP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const f4 *pa = static_cast<const f4 *>(a);
    f4 *pb = static_cast<f4 *>(b);
    const dim3 grid((uint32_t)wgs), block(1024);
    switch (mode * 2 + (nontemporal ? 1 : 0)) {
    case 0: hipLaunchKernelGGL((k_calib_read<false>), grid, block, 0, st, pa, pb); break;
    case 1: hipLaunchKernelGGL((k_calib_read<true>), grid, block, 0, st, pa, pb); break;
    case 2: hipLaunchKernelGGL((k_calib_fill<false>), grid, block, 0, st, pb); break;
    case 3: hipLaunchKernelGGL((k_calib_fill<true>), grid, block, 0, st, pb); break;
    case 4: hipLaunchKernelGGL((k_calib_add<false>), grid, block, 0, st, pa, pb); break;
    case 5: hipLaunchKernelGGL((k_calib_add<true>), grid, block, 0, st, pa, pb); break;
    case 6: hipLaunchKernelGGL((k_calib_copy2<false>), grid, block, 0, st, pa, pb); break;
    default: hipLaunchKernelGGL((k_calib_copy2<true>), grid, block, 0, st, pa, pb); break;
    }
    return hipGetLastError() == hipSuccess ? NSML_OK : NSML_EHIP;
}

const char *nsml_kernel_name(int id) { return (id >= 0 && id < KID_N) ? kKernelNames[id] : nullptr; }

}  // extern "C"
