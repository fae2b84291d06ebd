/*
 * nsml.h -- C ABI of libnsml: the per-step gradient data-reduction pipeline that one
 * data-parallel NetSenseML worker runs on its own gradient before communication,
 * for AMD MI355X (gfx950).
 *
 *   nsml_choose_ratio   host   Algorithm 1 + Eq. (1)-(3): network sensing -> ratio;
 *                              Algorithm 2 Step 1: the value width for the step
 *   nsml_compress       GPU    Sec. 4.2 Step 3 / Algorithm 2 Step 3: local accumulation
 *                              (error feedback), exact top-k by magnitude, then the value
 *                              coding and index/value/scale payload of the build contract
 *   nsml_decompress     GPU    receiver side of Algorithm 2 Step 3's transmission:
 *                              payload -> dense gradient
 *
 * Conventions
 *   - Every function returns int: NSML_OK (0) or a negative NSML_E* code.  Nothing throws,
 *     aborts or prints.
 *   - "dev" pointers are device memory on the context's GPU, allocated and owned by the
 *     caller; "host" pointers are ordinary host memory.  The library allocates only its own
 *     workspace, once, in nsml_create.
 *   - GPU entry points enqueue work on the caller's HIP stream and return without waiting.
 *     A context serves one stream at a time: calls that use the same context must be
 *     ordered on one stream (or separated by a synchronisation).
 *   - A gradient of n fp32 elements is split into B consecutive buckets by the host array
 *     bucket_off[0..B], bucket_off[0] = 0, bucket_off[B] = n, non-decreasing.  Buckets are
 *     compressed independently (the DDP hook of Sec. 5.1 is called per bucket); a bucket has
 *     fewer than 2^32 elements; empty buckets are allowed.
 *   - grad, residual and dense_out must be 16-byte aligned, idx/scales/val 4-byte aligned.
 *     No two of the buffers passed to one call may overlap.
 */
#ifndef NSML_H
#define NSML_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define NSML_OK        0
#define NSML_EINVAL   (-1)  /* null pointer, n == 0, ratio outside (0,1], bits not in {4,8,16,32},
                               offsets not ascending or not covering [0,n), bucket >= 2^32,
                               chunk not a positive multiple of 8, misaligned buffer */
#define NSML_ECAP     (-2)  /* n, B or chunk exceed what the context was created for */
#define NSML_EHIP     (-3)  /* a HIP call failed; see nsml_last_hip_error */
#define NSML_ENOTIMPL (-4)
#define NSML_ENOMEM   (-5)  /* host allocation failed */
#define NSML_EINTERNAL (-6) /* a device-side consistency check of the selection tripped during an
                               earlier call on this context (a bug in the library): that call's
                               outputs are not valid.  Returned once, by the next GPU entry point
                               called on the context (which then enqueues nothing), and by
                               nsml_path_stats / nsml_prune_stats */

const char *nsml_strerror(int code);

/* ------------------------------------------------------------------ controller (host) */

/* Parameters of Algorithm 1 / Eq. (3) and of the gate of Algorithm 2 Step 1.
 * The paper prints alpha = 0.5, beta2 = 0.01, the initial ratio 0.01, the floor 0.005, the cap 1
 * and the trigger 0.9 * BDP; the remaining defaults are this library's readings. */
typedef struct nsml_ctl_params {
    double alpha;       /* 0.5   multiplicative decrease, Eq. (3) */
    double beta1;       /* 0.1   start-up increment, Algorithm 1 Step 1 (value not printed) */
    double beta2;       /* 0.01  additive increase, Eq. (3) */
    double floor;       /* 0.005 lower bound of the ratio, Eq. (3) */
    double cap;         /* 1.0   upper bound of the ratio, Eq. (3) */
    double init;        /* 0.01  initial ratio, Algorithm 1 Step 1 */
    double bdp_frac;    /* 0.9   congestion trigger as a fraction of BDP, Eq. (3) */
    double rtt_excess;  /* 2.0   start-up ends when the last transmission time exceeds this
                                 multiple of RTprop (the RTT criterion of Sec. 4.1) */
    double tr_q;        /* 0.1   Algorithm 2 Step 1: quantize when ratio < tr_q ... */
    double tr_q4;       /* 0.01  ... with 4-bit codes when ratio < tr_q4 (quant_mode 0) */
    double tr_d;        /* 0.0   ... and the gradient L2 norm exceeds tr_d */
    int32_t startup_max;/* 10    start-up lasts at most this many increments */
    int32_t win_bw;     /* 10    BtlBw = max EBB over the last win_bw intervals; 0 = all time */
    int32_t win_rt;     /* 100   RTprop = min RTT over the last win_rt intervals; 0 = all time */
    int32_t quant_mode; /* 0: int8 / int4 codes; 1: binary16, the paper's own cast; 2: never */
} nsml_ctl_params;

#define NSML_CTL_MAX_WIN 128

/* Controller state: plain data, can be copied, saved and restored with memcpy. */
typedef struct nsml_ctl_state {
    nsml_ctl_params p;
    double ratio;        /* the controller's own ratio (before the gate's doubling) */
    double btlbw;        /* bytes / second, max EBB in the window */
    double rtprop;       /* seconds, min transmission time in the window */
    double bdp;          /* bytes, Eq. (2) */
    double all_max_ebb;  /* running extremes for window 0 */
    double all_min_rtt;
    double ebb[NSML_CTL_MAX_WIN];   /* ring buffers, newest at (count - 1) % NSML_CTL_MAX_WIN */
    double rtt[NSML_CTL_MAX_WIN];
    int64_t count;       /* measurements seen */
    int32_t phase;       /* 0 start-up, 1 NetSense */
    int32_t startup_steps;
} nsml_ctl_state;

/* Fill *p with the defaults listed above. */
int nsml_ctl_default_params(nsml_ctl_params *p);

/* Start a controller: ratio = p->init, start-up phase.  p == NULL uses the defaults.
 * NSML_EINVAL if a window exceeds NSML_CTL_MAX_WIN or a bound is inconsistent. */
int nsml_ctl_init(nsml_ctl_state *s, const nsml_ctl_params *p);

/* One decision before a transmission (Algorithm 1, one iteration).
 *   last_payload_bytes, last_tx_seconds  size and transmission time of the interval just
 *       finished (data_size_{i-1}, RTT_{i-1}); both <= 0 means "nothing measured yet" and
 *       leaves the ratio unchanged.
 *   dense_bytes   size of the uncompressed gradient; informational (ignored by the update).
 *   last_l2norm   L2 norm of the gradient for the density test of Algorithm 2 Step 1;
 *                 negative = unknown, which passes the test.
 *   ratio_out     ratio to hand to nsml_compress (already doubled when values are quantized)
 *   bits_out      32, 16, 8 or 4
 * Host only, O(window). */
int nsml_choose_ratio(nsml_ctl_state *s, double last_payload_bytes, double last_tx_seconds,
                      double dense_bytes, double last_l2norm, double *ratio_out, int *bits_out);

/* ------------------------------------------------------------------ payload geometry */

/* Pure host function.  k_b = min(n_b, max(1, ceil(ratio * n_b))) survivors per non-empty
 * bucket (Algorithm 2 Step 3).  Payload of a call:
 *   idx     uint32[K]           bucket-local indices, ascending inside each bucket, buckets
 *                               in order (bucket b starts at sum of k_b' for b' < b)
 *   val     val_bytes bytes     per bucket, byte-aligned: bits 32: float[k_b]; 16: binary16[k_b];
 *                               8: int8[k_b]; 4: ceil(k_b/2) bytes, survivor 2t in the low
 *                               nibble of byte t, survivor 2t+1 in the high nibble, two's
 *                               complement, unused high nibble of an odd tail = 0
 *   scales  float[n_scales]     bits 8/4 only: one per `chunk` consecutive survivors of a
 *                               bucket (last chunk of a bucket may be short); scale =
 *                               absmax / 127 (8) or / 7 (4); n_scales = 0 for bits 16/32
 * Any of k_b (host, B entries), K, val_bytes, n_scales may be NULL. */
int nsml_payload_layout(const uint64_t *bucket_off, uint32_t B, double ratio, int bits,
                        uint32_t chunk, uint64_t *k_b, uint64_t *K, uint64_t *val_bytes,
                        uint64_t *n_scales);

/* ------------------------------------------------------------------ GPU path */

typedef struct nsml_ctx nsml_ctx;

/* Allocate a context and its device workspace on GPU `device` for gradients of up to max_n
 * elements in up to max_buckets buckets, quantized in chunks of `chunk` survivors (2048 in
 * the benchmark configurations; a positive multiple of 8).  Workspace: about 6.3 bytes per
 * element of max_n (4 for survivor values at ratio 1, 2 for the staging segments, 0.3 for the
 * lists of undecided keys, the pruning bitmap and the per-tile tables) plus 200 KiB per bucket.  NSML_EHIP if the device or its memory is not
 * available (there is no CPU fallback).
 * A context serialises nothing itself: its calls share the workspace and the cached tables, so
 * they must not overlap, neither from several host threads nor on different streams (use one
 * context per stream).  Several contexts may work at the same time; the rare buckets that take the
 * dense passes use a small resident team of workgroups with barriers between its steps (one per
 * compute unit), sized so that the teams of a few concurrent contexts fit the device together; a
 * barrier that cannot complete within five seconds (the device held by something else for that
 * long) raises the consistency flag instead of waiting on.  A change of bucket layout between calls makes the next call wait for
 * the stream once, to rebuild the tables; a change of (ratio, bits) costs one small kernel. */
int nsml_create(nsml_ctx **ctx, int device, uint64_t max_n, uint32_t max_buckets, uint32_t chunk);
/* As nsml_create for callers that never exceed a ratio: the buffer of survivor values is sized
 * for max_ratio in (0, 1] instead of 1 (nsml_create is nsml_create_ex with max_ratio = 1), which
 * brings the workspace to about 2.3 + 4 * max_ratio bytes per element.  A compress call with a
 * larger ratio returns NSML_ECAP. */
int nsml_create_ex(nsml_ctx **ctx, int device, uint64_t max_n, uint32_t max_buckets, uint32_t chunk,
                   double max_ratio);
int nsml_destroy(nsml_ctx *ctx);

/* Tuning and diagnostic switches of a context.  The defaults are what the library measures as
 * best; results are identical for every setting (the tests run the path under each of them).
 * Takes effect from the next call; waits for nothing.  NSML_EINVAL for an unknown name or a value
 * outside the listed range.
 *   "span_tiles"   tiles of 4096 elements per workgroup of the streaming kernels: 1..16, 0 = by
 *                  gradient size
 *   "seg_waves"    wavefronts per workgroup of the streaming pass (4, 8 or 16), 0 = by span size
 *   "persist"      workgroups per compute unit of the streaming pass, each taking a contiguous
 *                  share of the spans: 1..8, 0 (default) = one workgroup per span
 *   "decomp_variant"  decompress: 1 = one wavefront per tile with direct stores, 0 = tiles assembled
 *                  in LDS, -1 (default) = by gradient size and survivors per tile
 *   "force_dense"  1: decide every bucket by the dense passes over the accumulator (the path a
 *                  bucket takes when its staged elements cannot decide it), 0: default
 *   "nt"           bit mask of non-temporal hints in the streaming pass (1 grad loads, 2 residual
 *                  loads, 4 accumulator stores); default 7
 *   "nt_dense"     non-temporal stores of the dense output of decompress: 1, 0, -1 = by variant
 *   "rescan"       diagnostic: 1 makes the threshold search read the undecided keys from the
 *                  staged entries again (the path taken when a staging segment has no room left
 *                  for its copy of them), 0: default
 *   "whistory"     pruning step: 1 (default) stages a narrow band of weight magnitudes around the
 *                  threshold the previous call on this context found for the bucket (weights move
 *                  little between steps; a band that misses costs a repeat of the weight pass, the
 *                  result is the same), 0: the band always comes from a sample of the weights
 *   "wband_miss"   diagnostic: 1 places the band of weight magnitudes that the pruning step stages
 *                  beside the threshold, so that every bucket takes the repeat of the weight pass
 *                  (the path of a band that missed), 0: default
 *   "trip_check"   diagnostic: 1 raises the flag a failed device-side consistency check raises,
 *                  so the error reporting of the next call can be exercised without a failure */
int nsml_set_option(nsml_ctx *ctx, const char *name, int value);

/* hipError_t of the last failed HIP call made through this context (0 = none). */
int nsml_last_hip_error(const nsml_ctx *ctx);
/* Bytes of device workspace the context holds. */
uint64_t nsml_workspace_bytes(const nsml_ctx *ctx);

/* Compress one gradient.
 *   grad      dev, const, float[n]
 *   residual  dev, in/out, float[n]: on entry what earlier steps did not send, on return what
 *             this step does not send: residual'[i] = grad[i] + residual[i] for elements not
 *             selected, and (value - decoded value) for selected ones, so that
 *             decompressed + residual' == grad + residual element by element
 *   n, bucket_off (host, B+1), B   the bucketed gradient
 *   ratio     in (0, 1]; k_b as in nsml_payload_layout.  Survivors of a bucket are its k_b
 *             largest |grad + residual|; equal magnitudes (+0 and -0 are equal) go to the
 *             lower index; exactly k_b are kept, zeros included if needed
 *   bits      32, 16, 8 or 4
 *   idx, val, scales  dev, out, sized by nsml_payload_layout (scales may be NULL for 16/32)
 *   stream    hipStream_t (NULL = the default stream)
 * Errors found while enqueuing are returned; the outputs are complete when the stream
 * reaches the end of the enqueued work. */
int nsml_compress(nsml_ctx *ctx, const float *grad, float *residual, uint64_t n,
                  const uint64_t *bucket_off, uint32_t B, double ratio, int bits,
                  uint32_t *idx, void *val, float *scales, void *stream);

/* As nsml_compress, preceded by the model-pruning step of Algorithm 2 Step 2.
 *   weights   dev, const, float[n]: the parameters the gradient belongs to, same bucketing.
 * Per bucket, floor(0.5 * (1 - ratio) * n_b) parameters with the smallest |weight| are pruned
 * for this step (equal magnitudes: the higher index is pruned first, so the kept set is the
 * top n_b - floor(...) by |weight| under the tie rule of the gradient selection); the k_b
 * survivors are chosen among the kept parameters only.  Pruning is not permanent: a pruned
 * parameter's accumulated gradient is written to the residual like any other unsent element
 * and competes again in later steps.  Outputs, payload layout and errors as nsml_compress.
 * Costs about two extra reads of `weights` per call (five for a bucket in which a huge group
 * of equal weights surrounds the pruning threshold). */
int nsml_compress_pruned(nsml_ctx *ctx, const float *grad, float *residual, const float *weights,
                         uint64_t n, const uint64_t *bucket_off, uint32_t B, double ratio,
                         int bits, uint32_t *idx, void *val, float *scales, void *stream);

/* Decompress a payload produced with the same (bucket_off, B, ratio, bits, chunk):
 *   dense_out  dev, out, float[n], fully overwritten: +0 everywhere except
 *              dense_out[bucket_off[b] + idx[j]] = decoded value j
 * The indices of each bucket must be ascending and inside the bucket, as nsml_compress
 * writes them; other index lists give unspecified values in dense_out (never an access
 * outside dense_out). */
int nsml_decompress(nsml_ctx *ctx, const uint32_t *idx, const void *val, const float *scales,
                    uint64_t n, const uint64_t *bucket_off, uint32_t B, double ratio, int bits,
                    float *dense_out, void *stream);

/* nsml_decompress for callers that cannot allocate device memory or create a context: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  It needs no
 * nsml_ctx and calls no allocating routine: its tables (bucket geometry, where each tile's
 * survivors start) live in a fixed device array inside the library, NSML_STATIC_SCRATCH_BYTES
 * per GPU, held until the process ends.  Same arguments, payload format and result as
 * nsml_decompress, plus the chunk size; runs on the current device.
 *   limits   n <= NSML_STATIC_MAX_N, B <= NSML_STATIC_MAX_BUCKETS, else NSML_ECAP
 * Every call on a GPU uses that GPU's one array: calls that overlap in time on one GPU (two
 * streams, two threads) race and give unspecified values; order them on one stream.  The array
 * keeps the last call's contents; every entry a call reads is written by that call first. */
#define NSML_STATIC_MAX_N        (1ull << 28)
#define NSML_STATIC_MAX_BUCKETS  320u
#define NSML_STATIC_SCRATCH_BYTES (1u << 20)
int nsml_decompress_static(const uint32_t *idx, const void *val, const float *scales, uint64_t n,
                           const uint64_t *bucket_off, uint32_t B, double ratio, int bits,
                           uint32_t chunk, float *dense_out, void *stream);

/* Receiver side of an all-gather of payloads (the communication pattern the paper reports for
 * sparsified gradients, Sec. 5.3): add one payload into a dense gradient that is being
 * accumulated.  dense_inout[bucket_off[b] + idx[j]] += decoded value j; no other element is
 * read or written.  Same arguments as nsml_decompress.  Calling it once per peer on a zeroed
 * buffer sums the peers' sparse gradients. */
int nsml_decompress_accumulate(nsml_ctx *ctx, const uint32_t *idx, const void *val,
                               const float *scales, uint64_t n, const uint64_t *bucket_off,
                               uint32_t B, double ratio, int bits, float *dense_inout, void *stream);

/* L2 norm of the gradient handed to the last nsml_compress of the context: a by-product of its
 * streaming pass (no extra memory traffic), for the density test of Algorithm 2 Step 1
 * (pass it as last_l2norm to nsml_choose_ratio).  total: norm over the whole gradient;
 * per_bucket: host array of B norms, or NULL.  The sums are accumulated in double over a fixed
 * reduction tree (binary32 products inside groups of four), so the value does not depend on
 * scheduling.  Synchronises the device.  NSML_EINVAL before the first compress. */
int nsml_last_l2norm(nsml_ctx *ctx, double *total, double *per_bucket);

/* ------------------------------------------------------------------ measurement */

#define NSML_MAX_KERNELS 32

/* When enabled, every kernel launch of the context is bracketed by HIP events on the caller's
 * stream.  nsml_profile_read synchronises those events and returns, for each kernel id,
 * the number of launches and their summed duration in milliseconds since the last read
 * (arrays of NSML_MAX_KERNELS entries), then resets the record.  At most 4096 launches are
 * kept between reads. */
int nsml_profile_enable(nsml_ctx *ctx, int on);
int nsml_profile_read(nsml_ctx *ctx, uint32_t *launches, double *total_ms);
/* Diagnostics for the last nsml_compress of the context: how many non-empty buckets were
 * decided from the single streaming pass (fast) and how many needed the extra dense passes
 * (fallback).  Both give identical results.  Synchronises the device.  NSML_EINTERNAL if the
 * call tripped a device-side consistency check (its outputs are then not valid). */
int nsml_path_stats(nsml_ctx *ctx, uint32_t *fast_buckets, uint32_t *fallback_buckets);
/* Diagnostics: the selection state of bucket b after the last nsml_compress of the context, eight
 * words to out8 (host): how it was decided (0 dense passes, 1 candidates, 2 band, 3 zero
 * threshold), why the dense passes were taken (bits: 1 the sample gave no usable guess, 2 not
 * used (a staging segment that overflows is read from the dense accumulator instead), 4 fewer
 * staged elements than k, 8 no room for the undecided keys,
 * 16 the threshold lies outside the staged band, 32 more non-zero elements than k in zero mode),
 * the staged key range [L, H) (0xFFFFFFFF: none / no upper bound), the threshold key, the number
 * of admitted elements equal to it, the bit position the threshold was known to before the
 * finish, and k_b.  Synchronises the device.  NSML_EINVAL for a bucket out of range. */
int nsml_bucket_state(nsml_ctx *ctx, uint32_t b, uint32_t *out8);
/* The same for the weight-pruning stage of the last nsml_compress_pruned (zeros if the last
 * compress call had no weights): how many non-empty buckets got their pruning threshold from
 * the band of weights staged in one pass, and how many needed the dense ordered passes (a
 * sample that missed, a huge group of equal weights).  Identical results either way.
 * Synchronises the device.  NSML_EINTERNAL as above. */
int nsml_prune_stats(nsml_ctx *ctx, uint32_t *band_buckets, uint32_t *dense_buckets);
/* Measurement aid: a plain device-to-device copy kernel ("k_calib_copy") of `bytes` bytes
 * (a multiple of 16, both pointers 16-byte aligned, dev) on `stream`, on the current device.
 * A profiler's HBM byte counters are scaled by what they report for this copy of known size. */
int nsml_calibration_copy(const void *src, void *dst, uint64_t bytes, void *stream);
/* Measurement aid: plain streaming kernels of the shape of the library's own streaming passes
 * (1024 threads, every wavefront on its own contiguous 16 KiB), to find what this machine
 * sustains for each access pattern.  a, b: dev, 16-byte aligned, `bytes` a multiple of 262144.
 *   mode 0 "k_calib_read"  reads a (b receives one word per workgroup)       bytes moved: bytes
 *   mode 1 "k_calib_fill"  writes zeros to b                                              bytes
 *   mode 2 "k_calib_add"   b = a + b (the access pattern of the accumulation)         3 * bytes
 *   mode 3 "k_calib_copy2" b = a                                                      2 * bytes
 * nontemporal != 0 uses non-temporal loads and stores. */
int nsml_calibration_stream(int mode, const void *a, void *b, uint64_t bytes, int nontemporal, void *stream);
/* Name of kernel id (NULL beyond the last). */
const char *nsml_kernel_name(int id);

#ifdef __cplusplus
}
#endif
#endif /* NSML_H */
