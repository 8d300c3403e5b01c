/*
 * covap.h -- C ABI of libcovap: the per-iteration gradient-compression hot
 * path of COVAP (arXiv 2311.04499) as hand-written HIP kernels for gfx950
 * (MI355X), plus the host-side planner and ratio policy around it.
 *
 * One worker's iteration, as the paper states it:
 *   1. error feedback      A = G + c * residual            Algorithm 1, line 2;
 *                                                          c from the scheduler
 *                                                          of Sec. III-D
 *   2. coarse filter       shard s is sent at iteration t iff (s + t) mod I == 0
 *                                                          Sec. III-A, Definition 1
 *   3. pack                selected shards, ascending, contiguous in `send`
 *   4. residual            selected: 0, otherwise A        Algorithm 1, line 4
 *   5. exchange + mean     out = (sum over N workers' payloads) / N, unpacked to
 *                          the dense layout, 0 where nothing was sent
 *                                                          Sec. II-A, Sec. III-B
 * Steps 1-4 are covap_compress (one kernel), step 5 is covap_decompress (one
 * kernel).  The exchange itself (AllReduce) is not part of this library: the
 * caller hands covap_decompress the N payload rows, or, after a sum-AllReduce,
 * hands covap_decompress_reduced the one summed row.
 *
 * Conventions
 *  - Pointers marked [device] are HIP device pointers owned by the caller; the
 *    library never allocates or frees device memory in a hot-path call and
 *    never keeps a pointer after the call returns.  [host] pointers are
 *    ordinary host memory.
 *  - Device buffers must be 16-byte aligned.  Elements are fp32, or bf16 stored
 *    as 16-bit patterns (computed in fp32, rounded to nearest-even once); with
 *    COVAP_BF16_RES32 the residual buffer alone is fp32; with COVAP_F32_PAY16 the
 *    payload buffers alone are 16-bit (IEEE half).
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Hot-path calls are asynchronous: COVAP_OK means "enqueued".
 *  - Indexing is 0-based for tensors, shards, buckets and iterations.
 *  - Every function returns a status (or a plain value for pure queries) and
 *    never aborts; covap_last_error() gives the text of this thread's last
 *    failure.
 *  - A plan is immutable after creation and may be shared by threads.  The
 *    interval I is fixed for the life of a plan (the paper fixes it once, early
 *    in training); a new I needs a new plan.
 */
#ifndef COVAP_H
#define COVAP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct covap_plan_s covap_plan_t; /* opaque, owned by the library */

typedef enum {
    COVAP_OK = 0,
    COVAP_EINVAL = 1,       /* bad argument (null, misaligned, out of range) */
    COVAP_ENOMEM = 2,       /* host or device allocation failed (plan creation only) */
    COVAP_EHIP = 3,         /* a HIP call or kernel launch failed */
    COVAP_ERANGE = 4,       /* index (tensor, shard, bucket) out of range */
    COVAP_EUNSUPPORTED = 5  /* valid request this build does not implement */
} covap_status_t;

typedef enum {
    COVAP_F32 = 0,        /* gradients, residual, payload, dense output: fp32 */
    COVAP_BF16 = 1,       /* all four bf16 (computed in fp32, rounded once) */
    /* gradients, payload and dense output bf16, residual fp32: Algorithm 1 with the
     * bf16 rounding as the quantiser of line 3 -- a sent element leaves
     * residual = A - bf16(A) (exact), a kept element leaves residual = A. */
    COVAP_BF16_RES32 = 2,
    /* gradients, residual and dense output fp32, payload IEEE half precision: the
     * coarse filter combined with the FP16 scheme of Table II as the quantiser of
     * Algorithm 1 line 3 -- a sent element travels as fp16(A) (round to nearest
     * even, overflow to Inf) and leaves residual = A - fp16(A); a kept element
     * leaves residual = A.  The mean is taken in fp32 over the widened halves.
     * Shard sizes and row strides count elements and must be multiples of 8. */
    COVAP_F32_PAY16 = 3
} covap_dtype_t;

typedef enum {
    /* The arena is cut into shards of `shard_elems` elements regardless of
     * tensor boundaries; the last shard is short.  Buckets are greedy runs of
     * shards under `bucket_cap_bytes`. */
    COVAP_SHARD_FIXED = 0,
    /* Sec. III-C: whole tensors are grouped, in order, into buckets
     * (communication tensors) of about `bucket_cap_bytes`; a bucket holding at
     * least twice the reference element count (the median of the bucket sizes, or
     * `ref_elems` when > 0) is cut evenly into floor(numel/ref) pieces, at most I.
     * Every piece is one shard for the filter; shards have different lengths.
     * Each bucket starts on a 1 KiB boundary of the arena -- 256 elements for
     * COVAP_F32, 512 for the other element types, see covap_plan_align_elems() --
     * (so total_elems may exceed the sum of the tensor counts by padding elements
     * that no call reads or writes), pieces are multiples of that unit, and in the
     * packed layout every sent shard starts on such a boundary too (elements in
     * the gaps are never written or read). */
    COVAP_SHARD_MEDIAN = 1
} covap_shard_mode_t;

typedef struct {
    int32_t dtype;            /* covap_dtype_t */
    int32_t mode;             /* covap_shard_mode_t */
    int64_t shard_elems;      /* FIXED mode: 1..2^30, multiple of 4 (fp32) or 8 (bf16) */
    int64_t bucket_cap_bytes; /* > 0; the paper's default is 25 MiB (Sec. III-A) */
    int64_t ref_elems;        /* MEDIAN mode: reference count, 0 = use the median */
    int32_t K;                /* the interval I >= 1 (1 = no compression) */
    int32_t reserved;         /* must be 0 */
} covap_plan_opts_t;

/* ---- planning (host) --------------------------------------------------- */

/* Lay `n_tensors` tensors (element counts in tensor_numel [host]) end to end
 * in one flat arena, cut it into shards and buckets, and fix the interval.
 * The arena offset of each tensor is the plan's to assign: ask for it with
 * covap_plan_tensor_offset.
 * On success *out receives a plan to be released with covap_plan_free.
 * EINVAL: null argument, n_tensors < 1, a negative count, K < 1, bad shard
 * size or cap, more than 2^33 elements in all (alignment padding included). */
covap_status_t covap_plan(const int64_t *tensor_numel, int32_t n_tensors,
                          const covap_plan_opts_t *opts, covap_plan_t **out);
void covap_plan_free(covap_plan_t *plan);

/* Pure queries; a null plan gives -1. */
int64_t covap_plan_total_elems(const covap_plan_t *plan);
int32_t covap_plan_num_tensors(const covap_plan_t *plan);
int32_t covap_plan_num_shards(const covap_plan_t *plan);
int32_t covap_plan_num_buckets(const covap_plan_t *plan);
int32_t covap_plan_interval(const covap_plan_t *plan);
/* Alignment unit, in elements, of shard starts in the arena and in the packed
 * layout: the 16-byte vector for COVAP_SHARD_FIXED (where no padding ever
 * appears), 1 KiB of the narrowest buffer for COVAP_SHARD_MEDIAN.  Row strides
 * that are multiples of 1 KiB keep every payload row aligned alike (faster). */
int32_t covap_plan_align_elems(const covap_plan_t *plan);
/* Arena offset (elements) of tensor i, or -1 when i is out of range. */
int64_t covap_plan_tensor_offset(const covap_plan_t *plan, int32_t i);
/* Arena offset, length and bucket of shard s; any out pointer may be null. */
covap_status_t covap_plan_shard(const covap_plan_t *plan, int32_t s, int64_t *off,
                                int64_t *len, int32_t *bucket);
/* Shard range [*sh_lo, *sh_hi) of bucket b. */
covap_status_t covap_plan_bucket(const covap_plan_t *plan, int32_t b, int32_t *sh_lo,
                                 int32_t *sh_hi);
/* 1 if shard s is sent at iteration `step`, 0 if not, -1 on a bad argument. */
int32_t covap_plan_is_selected(const covap_plan_t *plan, uint64_t step, int32_t s);
/* Ids of the shards sent at `step`, ascending, into shard_ids[cap] [host]
 * (may be null to only count).  Returns how many there are. */
int32_t covap_plan_selected(const covap_plan_t *plan, uint64_t step, int32_t *shard_ids,
                            int32_t cap);
/* Extent, in elements, of the packed range that bucket b's sent shards occupy
 * at `step` (b = -1: the whole payload); 0 if it sends nothing.  With
 * fixed-size shards this is the number of elements sent. */
int64_t covap_plan_packed_elems(const covap_plan_t *plan, uint64_t step, int32_t bucket);
/* Offset in the step's packed layout at which bucket b's payload starts
 * (meaningful when covap_plan_packed_elems(step, b) > 0). */
int64_t covap_plan_packed_base(const covap_plan_t *plan, uint64_t step, int32_t bucket);
/* Largest covap_plan_packed_elems(step, -1) over all steps: the size to give
 * send buffers and the row stride of receive buffers. */
int64_t covap_plan_packed_elems_max(const covap_plan_t *plan);

/* Replays, on the host, the launches that a hot-path call would make -- the same
 * index arithmetic the kernels run on their workgroup index, compiled for the host
 * -- and lists the tiles they resolve to, in launch and workgroup order: tile i
 * covers n[i] elements from arena offset off[i]; sel[i] is 1 if its shard is sent at
 * `step`, and then poff[i] is where the tile starts in the packed layout.  For
 * checking the launch geometry without a GPU; no hot-path call uses it.
 *   tile_elems  elements per workgroup: a power of two, 256..8192
 *   sent_only   0: every shard of the call, as covap_compress and covap_decompress
 *               launch; 1: only the sent shards, as covap_compress_aliased launches
 *   cap         capacity of the four arrays [host], any of which may be null; tiles
 *               beyond cap are counted but not stored
 *   n_launches, n_workgroups  [host, may be null] kernel launches of the call and
 *               workgroups in all (some return at once without a tile)
 * Returns the number of tiles, or -1 on a bad argument. */
int64_t covap_plan_trace(const covap_plan_t *plan, uint64_t step, int32_t bucket, int32_t tile_elems,
                         int32_t sent_only, int64_t cap, int64_t *off, int64_t *poff, int32_t *n,
                         uint8_t *sel, int32_t *n_launches, int64_t *n_workgroups);

/* ---- ratio policy and error-feedback scheduler (host) ------------------- */

/* I = ceil(CCR), never below 1 (Sec. III-B).  EINVAL unless 0 < ccr < 2^31. */
covap_status_t covap_ratio_from_ccr(double ccr, int32_t *K);
/* CCR = t_comm / t_comp (Sec. II-A), then as above.  Both times > 0, finite. */
covap_status_t covap_ratio_from_times(double t_comm, double t_comp, int32_t *K);
/* Compensation coefficient of the error-feedback scheduler (Sec. III-D):
 *   min(init_value + floor(num_steps / ascend_steps) * ascend_range, 1),
 * evaluated in double from the fp32 parameters and rounded to fp32.
 * EINVAL: ascend_steps == 0, non-finite parameter, null out. */
covap_status_t covap_ef_coeff(float init_value, uint64_t num_steps, uint64_t ascend_steps,
                              float ascend_range, float *coeff);

/* ---- hot path (device) ------------------------------------------------- */

/* Steps 1-4 for bucket `bucket` (-1 = the whole arena in one launch) at
 * iteration `step`.
 *   grad      [device] const, whole arena (total_elems elements), read only
 *   residual  [device] whole arena, read and overwritten with the new residual
 *   send      [device] the step's packed layout, indexed from its start: a
 *             per-bucket call writes only [packed_base, packed_base + packed_elems)
 *   send_cap_elems     capacity of `send` in elements; EINVAL if the range
 *                      this call writes does not fit
 *   ef_coeff  the scheduler's coefficient c; A = fma(c, residual, grad)
 * `grad`, `residual` and `send` must not overlap.  Selected residual elements
 * become +0.0 whatever A was (COVAP_BF16_RES32: A - bf16(A); COVAP_F32_PAY16:
 * A - fp16(A)). */
covap_status_t covap_compress(const covap_plan_t *plan, uint64_t step, int32_t bucket,
                              const void *grad, void *residual, void *send,
                              int64_t send_cap_elems, float ef_coeff, void *stream);

/* covap_compress on a grid of at most `max_workgroups` workgroups (>= 1) that walk
 * the call's tiles with a grid stride.  Same arguments otherwise, same result bits.
 * For running under a compute-bound kernel of another stream, the way the method
 * hides compression behind backward propagation (Sec. II-B): a few resident waves
 * per compute unit move the data while the other kernel keeps the rest of the unit.
 * On an idle GPU it is slower than covap_compress unless max_workgroups is in the
 * tens of thousands. */
covap_status_t covap_compress_bounded(const covap_plan_t *plan, uint64_t step, int32_t bucket,
                                      const void *grad, void *residual, void *send,
                                      int64_t send_cap_elems, float ef_coeff,
                                      int32_t max_workgroups, void *stream);

/* Aliased-residual form of steps 1-4, for callers whose gradient-accumulation
 * buffer doubles as the residual: the producer adds every new gradient into
 * `accum` (that addition IS Algorithm 1 line 2 with c = 1), and this call only
 * moves the sent shards of `accum` to `send` and clears them; shards that are
 * not sent are neither read nor written, so the call touches 3 * packed_elems
 * elements instead of 3 * total + packed.  Same packed layout and the same bits
 * as covap_compress(ef_coeff = 1) fed with the last gradient and the previous
 * residual.  Not available for COVAP_BF16_RES32 and COVAP_F32_PAY16
 * (EUNSUPPORTED), nor for c != 1.
 *   accum  [device] whole arena, read and written (sent shards only)
 *   send   [device] as in covap_compress */
covap_status_t covap_compress_aliased(const covap_plan_t *plan, uint64_t step, int32_t bucket,
                                      void *accum, void *send, int64_t send_cap_elems,
                                      void *stream);

/* Step 5 for bucket `bucket` (-1 = all) at iteration `step`.
 *   recv       [device] const, n_workers rows of stride_elems elements each;
 *              row w is worker w's `send` buffer of this step
 *   dense_out  [device] whole arena; this call writes every element of the
 *              bucket's shards: the mean where the shard was sent, +0.0 elsewhere
 * The sum runs over w = 0, 1, ..., n_workers-1 in that order in fp32 and is
 * divided by n_workers (IEEE division).  EINVAL: n_workers < 1, stride smaller
 * than the packed range read, stride not a multiple of 4 (fp32) / 8 (bf16)
 * elements when n_workers > 1.  dense_out must not overlap recv. */
covap_status_t covap_decompress(const covap_plan_t *plan, uint64_t step, int32_t bucket,
                                const void *recv, int32_t n_workers, int64_t stride_elems,
                                void *dense_out, void *stream);

/* Step 5 when the exchange is a sum-AllReduce, as the paper runs it (Sec. II-A:
 * AllReduce, then the average; Sec. III-B: COVAP keeps AllReduce because every
 * worker sends the same shards): the collective has already added the workers'
 * payloads, and what is left is the division and the unpack.
 *   summed     [device] const, ONE payload row in covap_compress's layout for
 *              this step: the element-wise sum of the n_workers payloads, in the
 *              payload's element type (the order and precision of that sum are
 *              the collective's); at least packed_base + packed_elems elements
 *              for the bucket
 *   n_workers  the divisor
 *   dense_out  [device] as in covap_decompress: summed / n_workers where the
 *              shard was sent (widened to fp32, IEEE division, one rounding
 *              back for bf16), +0.0 elsewhere
 * Reads packed_elems and writes the bucket's elements, whatever n_workers is.
 * Same bits as covap_decompress on one row holding that sum with the divisor
 * n_workers.  EINVAL: n_workers < 1, null/misaligned/overlapping pointers. */
covap_status_t covap_decompress_reduced(const covap_plan_t *plan, uint64_t step, int32_t bucket,
                                        const void *summed, int32_t n_workers, void *dense_out,
                                        void *stream);

/* ---- fine-grained top-k sparsifier (contrast point; Sec. I, Table II) --- */

/* Bytes of device workspace topk_compress needs for n elements of `dtype`
 * (0 for n < 0 or an element type topk_compress does not take). */
size_t topk_workspace_bytes(int64_t n, int32_t dtype);

/* A = fma(c, residual, grad) over n fp32 elements; keep the k entries of
 * largest magnitude.  Magnitudes are ordered by the bit pattern of |A| read as
 * an unsigned integer; among equal magnitudes the lowest index is kept.
 *   out_vals [device] k values, out_idx [device] k indices, ascending index
 *   residual [device] becomes A with the kept entries set to +0.0
 *   workspace [device] at least topk_workspace_bytes(n) bytes, 256-byte aligned
 * EINVAL: k < 0, k > n, n >= 2^32, null/misaligned pointer, small workspace.
 * EUNSUPPORTED: dtype other than COVAP_F32. */
covap_status_t topk_compress(const void *grad, void *residual, int64_t n, int64_t k,
                             int32_t dtype, float ef_coeff, void *out_vals,
                             uint32_t *out_idx, void *workspace, size_t ws_bytes,
                             void *stream);

/* topk_compress for callers that cannot allocate device memory or carry a
 * workspace around: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments (without the workspace), same kernels and
 * the same result bits as topk_compress; the workspace is a fixed array inside the
 * library's code object (about 6.2 MB on every GPU the library runs on, held until
 * the process ends), whose device address is looked up once per device on the first
 * call made with that device current.  The call allocates nothing and frees nothing.
 *   n at most topk_static_max_elems() = 2^24 elements; EINVAL beyond that (use
 *   topk_compress with a caller-owned workspace for larger inputs)
 *   the device that owns `stream` and the buffers must be the current device
 * All calls on one GPU share that GPU's array: calls that may overlap in time on one
 * GPU (different streams, different threads) race and give unspecified results (but
 * touch nothing outside the array and the caller's buffers); calls on one stream are
 * ordered and need nothing else.  The array keeps the previous call's contents; the
 * first kernel of every call resets the parts that are accumulated into, so no
 * clearing is needed between calls. */
int64_t topk_static_max_elems(void);
covap_status_t topk_compress_static(const void *grad, void *residual, int64_t n, int64_t k,
                                    int32_t dtype, float ef_coeff, void *out_vals,
                                    uint32_t *out_idx, void *stream);

/* ---- further contrast points without data dependencies (Sec. II-C, Table III) --- */

/* Random-k sparsifier with error feedback.  The k coordinates are the caller's
 * to draw (from a seed all workers share, so every worker sends the same set):
 *   idx [device] k indices, all distinct, each < n
 *   A = fma(c, residual, grad) over n fp32 elements; out_vals[j] = A[idx[j]];
 *   residual [device] becomes A with the sent coordinates set to +0.0
 * EINVAL: k < 0, k > n, n >= 2^32, null or misaligned pointer. */
covap_status_t randk_compress(const void *grad, void *residual, int64_t n, const uint32_t *idx,
                              int64_t k, float ef_coeff, void *out_vals, void *stream);

/* FP16 quantiser with error feedback over n fp32 elements:
 *   A = fma(c, residual, grad); out_half[i] = fp16(A[i]) (round to nearest even);
 *   residual[i] = A[i] - fp16(A[i]).  All pointers [device], 16-byte aligned. */
covap_status_t fp16_compress(const void *grad, void *residual, int64_t n, float ef_coeff,
                             void *out_half, void *stream);

/* Mean of n_workers fp16 payload rows (row w at recv + w * stride_elems halves):
 *   dense_out[i] = (sum over w = 0..n_workers-1, in that order, in fp32) / n_workers
 * dense_out [device] n fp32 elements.  EINVAL: stride < n, stride not a
 * multiple of 8 when n_workers > 1, null or misaligned pointer. */
covap_status_t fp16_decompress(const void *recv, int32_t n_workers, int64_t stride_elems,
                               int64_t n, void *dense_out, void *stream);

/* Mean of n_workers sparse payloads, k (value, index) pairs each (row w at
 * vals + w * stride_elems and idx + w * stride_elems), as produced by
 * topk_compress or randk_compress:
 *   dense_out = 0; for w = 0..n_workers-1 in order: dense_out[idx] += val;
 *   dense_out /= n_workers
 * Indices inside one row must be distinct (rows may overlap freely).  The
 * additions into one element happen in worker order, so the result is
 * deterministic.  dense_out [device] n fp32 elements, fully written. */
covap_status_t sparse_decompress(const void *vals, const uint32_t *idx, int32_t n_workers,
                                 int64_t k, int64_t stride_elems, int64_t n, void *dense_out,
                                 void *stream);

/* The same mean for payloads whose indices ascend inside every row (what
 * topk_compress writes; Random-k payloads qualify if the caller drew or sorted
 * its coordinates in ascending order): one pass over dense_out instead of one
 * launch per worker.  Same arguments, same result bits.  Rows that are not
 * ascending give an unspecified result (but no access outside the buffers).
 * More than 64 workers are handed to sparse_decompress.  n < 2^32 - 16. */
covap_status_t sparse_decompress_sorted(const void *vals, const uint32_t *idx, int32_t n_workers,
                                        int64_t k, int64_t stride_elems, int64_t n, void *dense_out,
                                        void *stream);

/* ---- measurement helpers ------------------------------------------------ */

/* Plain streaming kernels used to measure the achievable HBM rate next to the
 * hot path and to calibrate hardware byte counters: dst = src (16-byte
 * vectors; `bytes` a multiple of 16), and a = b + s*c over n fp32 elements
 * (n a multiple of 4).  All pointers [device], 16-byte aligned. */
covap_status_t covap_probe_copy(void *dst, const void *src, size_t bytes, void *stream);
covap_status_t covap_probe_triad(float *a, const float *b, const float *c, float s, int64_t n,
                                 void *stream);

/* A compute-only kernel for overlap measurements: `workgroups` workgroups of 256
 * threads, each wave issuing 4 * iters matrix-core instructions on registers, with
 * `lds_bytes` of (unused) LDS reserved per workgroup to set its occupancy; one store
 * per thread at the end into out [device, workgroups * 256 floats]. */
covap_status_t covap_probe_mfma(float *out, int32_t workgroups, int32_t iters, int32_t lds_bytes,
                                void *stream);

/* Launch-shape knobs for tuning sweeps (the defaults are the measured best on
 * MI355X).  Keys and allowed values:
 *   "compress_threads", "decompress_threads"  workgroup size: 64, 256
 *   "compress_unroll"    16-byte vectors per thread per tile: 1, 2, 4
 *   "decompress_tile"    16-byte vectors per thread per tile: 1, 2, 4
 *   "decompress_unroll"  payload rows loaded before they are summed: 1, 2, 4
 *   "nontemporal"        streaming cache hints on loads and stores: 0, 1
 *   "decompress_lds_pad" bytes of unused LDS reserved per decompress workgroup, which
 *                        caps its occupancy: 0, 6144, 8192, 24576, 32768, 49152
 *   "topk_pass1_waves"   waves that share a 1024-element tile in the first pass of
 *                        topk_compress: 1, 2, 4
 *   "topk_pass1_lds_pad" as decompress_lds_pad, for that pass: 0, 6144, 8192, 24576
 * Value -1 returns a knob to "never set".  While "decompress_threads",
 * "decompress_tile" and "decompress_lds_pad" are all in that state, a decompress
 * call that reads fewer payload elements than it writes dense ones (few rows:
 * covap_decompress_reduced always, covap_decompress with n_workers below about the
 * interval) is bound by its stores and runs in the shape that fills memory fastest:
 * 256-thread workgroups, one 16-byte store per thread (fixed-size shards) or two and
 * a 32 KiB reservation (variable-length shards).  covap_tune_get reports the many-row
 * values.
 * No knob changes any result bit.  EINVAL for an unknown key or value.  For
 * tuning sweeps and tests only: the knobs are global to the process (every plan and
 * every later call sees a change).  Stores and loads are atomic and a hot-path call
 * reads the knobs once, so a change made while another thread is inside a call
 * takes effect for that thread's next call, never in the middle of one. */
covap_status_t covap_tune_set(const char *key, int32_t value);
int32_t covap_tune_get(const char *key);

/* Text of the calling thread's most recent error ("" if none). */
const char *covap_last_error(void);
/* Library version, "major.minor.patch". */
const char *covap_version(void);

#ifdef __cplusplus
}
#endif
#endif /* COVAP_H */
