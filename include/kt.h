/*
 * kt -- per-GPU reduction stage of a load-adaptive data-parallel step on
 * AMD MI355X (gfx950).
 *
 * Setting (KAITIAN, Sec. III): under synchronous data parallelism every device
 * computes gradients on its share of the global mini-batch; DDP flattens the
 * per-parameter gradients into buckets and the K peer copies of each bucket are
 * combined by the gradient AllReduce.  With the load-adaptive shares of
 * Sec. III-C (b_i proportional to the device score, sum b_i = B_global) the
 * devices hold means over different sample counts, so the copies combine with
 * weights w_k = b_k / B into the global-batch mean.  This library is that
 * stage on one GPU: plan shares, pack gradients into buckets, K-way weighted
 * reduce, scale and unpack.  The K peer buffers are resident in device memory.
 *
 * Conventions
 *  - Plain C ABI.  Every call returns a kt_status; on error the out-parameters
 *    are untouched and kt_last_error() describes the failure (thread-local).
 *  - "host" pointers are ordinary process memory; "device" pointers are HIP
 *    device memory owned by the caller, which must stay valid until the work
 *    enqueued on the stream has finished.  The library owns only the plan.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Device calls are asynchronous: they enqueue kernels and return.
 *  - Device calls use the calling thread's current HIP device; a plan binds to
 *    the device of its first device call.
 *  - Arrays indexed "by bucket" have kt_plan_num_buckets() entries and are
 *    indexed by bucket id also when a single bucket is processed.  The whole
 *    host array is copied on every call (all entries must be initialised;
 *    NULL is fine for buckets not selected); only the selected buckets'
 *    pointers are checked and dereferenced on the device.  Passing the same
 *    array contents on successive calls lets the library reuse its resident
 *    device copy instead of uploading it again.
 *  - HIP graphs: a device call may be recorded under stream capture once the
 *    same call (same plan, same pointer arrays) has been made outside capture,
 *    so that the plan's tables and the pointer table are resident; under
 *    capture the library enqueues its kernel and nothing else.  Otherwise the
 *    call returns KT_EUNSUPPORTED.  A pointer table read by a recorded call is
 *    set aside for the graph and stays resident until the plan is destroyed
 *    (one table per distinct pointer set: a chained step records three, pack,
 *    reduce and unpack; tables of eager calls are not affected).
 *    Everything passed by value is frozen into the recorded kernel node: the K
 *    weights, scale, lr, momentum, weight_decay and first_step.  After new
 *    shares (kt_replan_shares) or a learning-rate change a replayed graph
 *    still applies the old values: record the step again, or update the
 *    kernel node's parameters.  Or keep them out of the recording: record
 *    kt_weighted_reduce / kt_fused_step with weights == NULL and change the
 *    weights with kt_plan_set_weights; record kt_bucket_unpack_sgd_resident
 *    (or kt_fused_step_sgd_resident) and change scale, lr, momentum and
 *    weight_decay with kt_plan_set_sgd.
 *    A recorded first_step != 0 would reset the momentum on every replay, so
 *    the SGD calls refuse it under capture (KT_EUNSUPPORTED).
 *  - Large launches (K >= 4, hundreds of MiB per peer) of kt_weighted_reduce and
 *    kt_fused_step issue their stores in bursts that every workgroup times by
 *    the device-wide clock (1.2 us in every 12 us), which the memory system
 *    rewards when the launch has the GPU to itself.  The environment variable
 *    KT_STORE_WINDOW_NS, read once per process, sets the period in nanoseconds;
 *    0 switches the bursts off.  Results do not depend on it.
 *  - Streams passed to device calls should outlive the plan.  If the stream of
 *    an earlier call has been destroyed, the library waits for the whole
 *    device instead of that stream when it recycles a pointer table.
 */
#ifndef KT_H
#define KT_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* The entry points below are the only symbols the shared library exports. */
#define KT_API __attribute__((visibility("default")))

typedef struct kt_plan kt_plan;

typedef enum { KT_F32 = 0, KT_BF16 = 1 } kt_dtype;

typedef enum {
    KT_OK = 0,
    KT_EINVAL = 1,        /* bad argument (NULL, range, non-finite, overlap)   */
    KT_EALIGN = 2,        /* pointer not aligned to the element size           */
    KT_ENOMEM = 3,        /* host or device allocation failed                  */
    KT_EHIP = 4,          /* a HIP runtime call or kernel launch failed        */
    KT_EUNSUPPORTED = 5   /* valid request outside the supported range         */
} kt_status;

#define KT_MAX_PEERS 64
#define KT_ALL_BUCKETS (-1)

/* Library version string, static storage. */
KT_API const char *kt_version(void);

/* Text for a status code, static storage. */
KT_API const char *kt_status_string(kt_status s);

/* Message of the last failing call on this thread, static storage ("" if none). */
KT_API const char *kt_last_error(void);

/*
 * Load-adaptive batch shares (Sec. III-C, phase 2: the display equation and
 * the rounding sentence after it).  Host only; touches no GPU.
 *
 *   thr[K]     host, in : device throughputs (samples per unit time), finite
 *                         and > 0.  score_i = thr_i / max thr; the common
 *                         factor cancels, so any positive scale is accepted.
 *   B          in       : global batch size, 0 <= B <= 2^40.
 *   shares[K]  host, out: integers b_i >= 0 with sum b_i = B.  Quota
 *                         q_i = (thr_i / sum thr) * B in IEEE double
 *                         (left-to-right sum); b_i = floor(q_i), then +1 for
 *                         the B - sum floor entries with the largest
 *                         fractional part, ties to the lowest index.
 *   weights[K] host, out: optional (may be NULL).  w_k = (float)b_k /
 *                         (float)B, one binary32 division; requires B > 0.
 * Errors: KT_EINVAL for NULL thr/shares, K < 1, K > KT_MAX_PEERS, B out of
 * range, a throughput that is not finite and positive, weights with B == 0.
 */
KT_API kt_status kt_plan_shares(const double *thr, int K, int64_t B,
                         int64_t *shares, float *weights);

/*
 * Online adaptation of the shares (Sec. III-C phase 1, "Online Adaptation":
 * monitor the computation time per batch during training and adjust the
 * scores).  Host only.  Device k processed shares_used[k] samples in
 * step_time[k] (any time unit); its time per sample tau_k = t_k / b_k enters
 *     ema[k] <- alpha * tau_k + (1 - alpha) * ema[k]
 * (ema[k] <= 0 means "no estimate yet" and is replaced by tau_k; a device that
 * processed no samples keeps its estimate), all in IEEE double.  The new
 * shares are kt_plan_shares(1 / ema, B); weights as there (may be NULL).
 *   ema[K] host, in/out; alpha in (0, 1].
 * Errors: KT_EINVAL (NULL, ranges, a device with samples but a time that is
 * not finite and positive, a device without any estimate); on error nothing
 * is written.
 */
KT_API kt_status kt_replan_shares(const double *step_time, const int64_t *shares_used,
                           double *ema, double alpha, int K, int64_t B,
                           int64_t *shares, float *weights);

/*
 * Weights for a two-level combination (Sec. III-A: reduction inside each group
 * of homogeneous accelerators, then across groups through host memory).  Host
 * only.  With B_g the sum of the shares of group g and B the sum of all shares:
 *   w_intra[k] = (float)b_k / (float)B_g   (k's weight inside its group),
 *   w_inter[g] = (float)B_g / (float)B     (the group's weight across groups),
 * so that a group's result is the mean gradient over the group's samples and
 * the product of the two weights is the flat weight b_k / B.  The two levels
 * are two kt_weighted_reduce calls; the second one may read the other groups'
 * results from device-accessible pinned host memory.
 *
 *   group_of[K]    host, in : group index of each device, in [0, G).
 *   group_batch[G] host, out: optional (may be NULL), the B_g.
 * Errors: KT_EINVAL (NULL, ranges, a group without samples).
 */
KT_API kt_status kt_plan_group_weights(const int64_t *shares, int K,
                                const int *group_of, int G, float *w_intra,
                                float *w_inter, int64_t *group_batch);

/*
 * Load-adaptive sampler partition (Sec. III-C phase 2: portions of every
 * global mini-batch go to device i in proportion to its score; Sec. IV-A: the
 * DistributedSampler override).  Host only.
 *
 * The epoch ordering of the N dataset indices is the identity (shuffle == 0)
 * or a Fisher-Yates shuffle (i = N-1..1, swap with a uniform j <= i) driven by
 * SplitMix64 started at state seed + epoch * 0x9E3779B97F4A7C15, bounded draws
 * by multiply-high with rejection.  The ordering is cut into global batches of
 * B; in every batch device `rank` takes the contiguous slice of shares[rank]
 * indices starting at shares[0] + ... + shares[rank-1].  If B does not divide
 * N the last batch is dropped (drop_last != 0) or completed by wrapping around
 * to the start of the ordering.
 *
 *   shares[K] host, in : integers >= 0 summing to B (e.g. from kt_plan_shares).
 *   out       host, out: the rank's indices for the epoch, steps * shares[rank]
 *                        entries; capacity is the size of `out` in entries.
 *   count     host, out: entries written (may be NULL in kt_sampler_epoch).
 * Errors: KT_EINVAL (arguments, capacity too small), KT_ENOMEM.
 */
KT_API kt_status kt_sampler_epoch_size(int64_t N, int64_t B, const int64_t *shares,
                                int K, int rank, int drop_last, int64_t *count);
KT_API kt_status kt_sampler_epoch(int64_t N, int64_t B, const int64_t *shares, int K,
                           uint64_t seed, uint64_t epoch, int shuffle, int rank,
                           int drop_last, int64_t *out, int64_t capacity,
                           int64_t *count);

/*
 * Bucket plan: the flattening DDP applies before the gradient AllReduce
 * (Sec. III).  Host only until the first device call, which uploads the
 * plan's tables to the current device.
 *
 *   numel[T]     host, in: element count of each gradient tensor, >= 0, in the
 *                          caller's order (kept).
 *   T            in      : number of tensors, >= 0.
 *   dt           in      : element type of tensors and buckets.
 *   cap_bytes    in      : bucket size cap; 0 = one bucket.  A bucket closes
 *                          before a tensor whose aligned end would exceed the
 *                          cap; tensors are never split (an oversize tensor
 *                          sits alone).
 *   align_bytes  in      : every tensor starts at a multiple of this inside
 *                          its bucket and the bucket length is rounded up to
 *                          it.  Power of two, multiple of the element size,
 *                          <= 16384.  16 gives the fast vector path; the
 *                          element size gives dense packing; 16384 (the
 *                          kernels' tile) makes every tensor start on a tile
 *                          boundary, so that tensor-side addresses are as
 *                          well aligned as the tensors' own base addresses.
 *   out          out     : new plan, to be released with kt_plan_destroy.
 * Errors: KT_EINVAL (arguments), KT_ENOMEM, KT_EUNSUPPORTED (the plan would
 * need 2^24 or more 16 KiB tiles, i.e. 256 GiB per peer).
 */
KT_API kt_status kt_plan_create(const int64_t *numel, int T, kt_dtype dt,
                         int64_t cap_bytes, int align_bytes, kt_plan **out);

/* Releases host tables and, if uploaded, the device tables (waits for the
 * device to go idle first).  NULL is accepted. */
KT_API kt_status kt_plan_destroy(kt_plan *plan);

/* Number of buckets / tensors; -1 for a NULL plan. */
KT_API int kt_plan_num_buckets(const kt_plan *plan);
KT_API int kt_plan_num_tensors(const kt_plan *plan);

/* Bucket b: length in elements (padding included; the caller allocates
 * n_elems * element size bytes per bucket buffer), first tensor, tensor
 * count.  Any out-pointer may be NULL. */
KT_API kt_status kt_plan_bucket_info(const kt_plan *plan, int b, int64_t *n_elems,
                              int *first_tensor, int *n_tensors);

/* Tensor t: its bucket and element offset inside it.  Out-pointers may be NULL. */
KT_API kt_status kt_plan_tensor_info(const kt_plan *plan, int t, int *bucket,
                              int64_t *elem_offset);

/*
 * Tile table introspection (for checks).  The device kernels process a bucket
 * in fixed tiles of 16 KiB, one workgroup each.  Tile i (0 <= i <
 * kt_plan_num_tiles) covers elements [tile_in_bucket * E, min((tile_in_bucket
 * + 1) * E, n_elems)) of `bucket`, E = 16384 / element size.  Tensors
 * first_tensor .. first_tensor + n_tensors - 1 are the only ones that may own
 * elements of the tile; n_tensors == 0 marks a tile wholly inside tensor
 * first_tensor.  Out-pointers may be NULL.
 */
KT_API int64_t kt_plan_num_tiles(const kt_plan *plan);
KT_API kt_status kt_plan_tile_info(const kt_plan *plan, int64_t i, int *bucket,
                            int64_t *tile_in_bucket, int *first_tensor,
                            int *n_tensors);

/*
 * Pack: bucket_b[off_t + i] = tensor_t[i] for every tensor of the selected
 * bucket(s); padding elements are written as zero bits.  A raw copy: bit
 * patterns are preserved.
 *
 *   bucket       in      : bucket id, or KT_ALL_BUCKETS for one batched launch.
 *   tensor_ptrs  host, in: T device pointers (contiguous tensors), indexed by
 *                          tensor id; entries of zero-size tensors may be NULL.
 *   bucket_bufs  host, in: device pointers by bucket; only selected buckets
 *                          are written on the device.
 * Pointers must be aligned to the element size (KT_EALIGN otherwise); 16-byte
 * aligned pointers take the vector path, others a slower correct one.
 * Tensors and buckets must not overlap.
 */
KT_API kt_status kt_bucket_pack(kt_plan *plan, int bucket,
                         const void *const *tensor_ptrs,
                         void *const *bucket_bufs, void *stream);

/*
 * K-way weighted reduce: out_b[i] = sum_{k=0}^{K-1} w_k * peer_{b,k}[i] over
 * the whole bucket length, evaluated per element in binary32 as
 * acc = w_0 * x_0 (rounded product), then acc = fma(w_k, x_k, acc) for
 * k = 1..K-1 in ascending k.  bf16 buckets are widened exactly, accumulated in
 * binary32 and rounded to nearest-even once at the end.
 *
 *   peer_bufs  host, in: device pointers, entry [b * K + k] = peer k's copy of
 *                        bucket b (num_buckets * K entries).
 *   K          in      : 1 <= K <= KT_MAX_PEERS.
 *   weights    host, in: K binary32 weights (copied during the call), or NULL
 *                        for the weights set with kt_plan_set_weights.
 *   out_bufs   host, in: device pointers by bucket.  out_b may be identical to
 *                        one peer_{b,k} (in place); any other overlap is an
 *                        error where detected (equal ranges are; partial
 *                        overlaps are undefined).
 */
KT_API kt_status kt_weighted_reduce(kt_plan *plan, int bucket,
                             const void *const *peer_bufs, int K,
                             const float *weights, void *const *out_bufs,
                             void *stream);

/*
 * Device-resident weights, for recorded graphs that must follow new shares
 * (Sec. III-C phase 1, online adaptation).  kt_plan_set_weights copies K weights
 * into device memory owned by the plan, on `stream`, ordered behind the work
 * already enqueued there.  kt_weighted_reduce, kt_fused_step and
 * kt_fused_step_noalloc called with weights == NULL read these K weights from
 * device memory when their kernel runs, instead of freezing K values into the
 * launch: a graph recorded with weights == NULL applies, on every replay,
 * whatever the last kt_plan_set_weights on the replaying stream (or one
 * synchronised with it) has written.  The arithmetic is the same.
 *
 *   weights host, in: K binary32 weights (copied before the call returns).
 * Errors: KT_EINVAL (arguments); KT_EUNSUPPORTED under stream capture (the
 * copy cannot be recorded; call it outside capture); a device call with
 * weights == NULL fails with KT_EINVAL if no weights were set or K differs.
 */
KT_API kt_status kt_plan_set_weights(kt_plan *plan, const float *weights, int K,
                                     void *stream);

/*
 * Unpack with scale: tensor_t[i] = scale * bucket_b[off_t + i] for every
 * tensor of the selected bucket(s), one binary32 multiplication per element
 * (bf16: widen, multiply, round to nearest-even).  Padding is not read into
 * any tensor and nothing outside the tensors is written.
 */
KT_API kt_status kt_bucket_unpack_scale(kt_plan *plan, int bucket,
                                 const void *const *bucket_bufs, float scale,
                                 void *const *tensor_ptrs, void *stream);

/*
 * Fused single pass over the same data: for every tensor t of the selected
 * bucket(s)
 *     out_t[i] = scale * R( w_0 * local_t[i] + sum_{k=1}^{K-1} w_k * peer_{b,k}[off_t + i] )
 * where R rounds the binary32 accumulator to the storage type (identity for
 * fp32, nearest-even for bf16).  The local device's gradients (peer 0) are read
 * in place from the tensors instead of being packed first, and the result goes
 * straight to the output tensors: the arithmetic and its rounding order are
 * those of kt_bucket_pack -> kt_weighted_reduce -> kt_bucket_unpack_scale, so
 * results are bit-identical to that chain, while (K+1) instead of (K+5)
 * element sizes move per element.  This is the form a DDP gradient hook wants
 * (Sec. III: gradient AllReduce per bucket, followed by the copy back).
 *
 *   local_tensor_ptrs host, in: T device pointers, peer 0's gradients.
 *   peer_bufs         host, in: device pointers, entry [b * (K-1) + (k-1)] =
 *                               peer k's copy of bucket b, k = 1..K-1 (ignored
 *                               when K == 1).
 *   out_tensor_ptrs   host, in: T device pointers; out_t may be identical to
 *                               local_t (in place); any other overlap with
 *                               inputs is rejected where detected.
 * Padding positions of the peer buckets are not read into any output.
 */
KT_API kt_status kt_fused_step(kt_plan *plan, int bucket,
                        const void *const *local_tensor_ptrs,
                        const void *const *peer_bufs, int K,
                        const float *weights, float scale,
                        void *const *out_tensor_ptrs, void *stream);

/*
 * Unpack fused with the optimizer of the paper's runs (Sec. IV-B: SGD with
 * momentum 0.9 and weight decay 5e-4): the reduced gradient is consumed from
 * the bucket and never written.  For every tensor t of the selected bucket(s)
 * and element i, with g = scale * bucket_b[off_t + i] (one binary32 product;
 * bf16 buckets are widened exactly first):
 *     g' = fma(weight_decay, p, g)
 *     v' = g'                       if first_step != 0
 *          fma(momentum, v, g')     otherwise
 *     p' = fma(-lr, v', p)
 * p (parameters) and v (momentum) are binary32 tensors updated in place; on the
 * first step v is written without being read.
 *
 *   param_ptrs, momentum_ptrs host, in: T device pointers each (binary32,
 *                                       numel[t] elements), 4-byte aligned;
 *                                       16-byte alignment gives the vector path.
 * Parameters, momentum and buckets must not overlap.
 */
KT_API kt_status kt_bucket_unpack_sgd(kt_plan *plan, int bucket,
                               const void *const *bucket_bufs, float scale,
                               void *const *param_ptrs,
                               void *const *momentum_ptrs, float lr,
                               float momentum, float weight_decay,
                               int first_step, void *stream);

/*
 * kt_bucket_unpack_sgd for mixed-precision training (the bf16 workload): the
 * parameters updated in binary32 are the master copy; every updated value is
 * also written, rounded to nearest-even, to a bf16 model-parameter tensor, the
 * copy that the next forward and backward pass read.  Same arithmetic as
 * kt_bucket_unpack_sgd for p' and v' (Sec. IV-B's optimizer), plus
 *     model_t[i] = bf16(p')
 * Buckets may be of either element type; 2 more bytes per element are written.
 *
 *   master_ptrs, momentum_ptrs host, in: T device pointers each, binary32.
 *   model_ptrs                 host, in: T device pointers, bf16, numel[t]
 *                                        elements, 2-byte aligned (8-byte
 *                                        alignment gives the vector path);
 *                                        written only.
 * Master parameters, momentum, model parameters and buckets must not overlap.
 */
KT_API kt_status kt_bucket_unpack_sgd_master(kt_plan *plan, int bucket,
                                             const void *const *bucket_bufs,
                                             float scale, void *const *master_ptrs,
                                             void *const *momentum_ptrs,
                                             void *const *model_ptrs, float lr,
                                             float momentum, float weight_decay,
                                             int first_step, void *stream);

/*
 * Device-resident optimizer scalars, for recorded graphs that must follow a
 * learning-rate schedule (Sec. IV-B trains with a stepped learning rate).
 * kt_plan_set_sgd copies scale, lr, momentum and weight_decay into device
 * memory owned by the plan, on `stream`, ordered behind the work already
 * enqueued there.  kt_bucket_unpack_sgd_resident is kt_bucket_unpack_sgd
 * (model_ptrs == NULL) or kt_bucket_unpack_sgd_master (model_ptrs != NULL)
 * with these four values read from device memory when the kernel runs; the
 * arithmetic is the same, and a graph recorded with it applies, on every
 * replay, whatever the last kt_plan_set_sgd on the replaying stream (or one
 * synchronised with it) has written.
 *
 * Errors: kt_plan_set_sgd: KT_EINVAL (NULL plan), KT_EUNSUPPORTED under stream
 * capture (the copy cannot be recorded).  kt_bucket_unpack_sgd_resident: as
 * kt_bucket_unpack_sgd[_master], and KT_EINVAL if no scalars were set.
 */
KT_API kt_status kt_plan_set_sgd(kt_plan *plan, float scale, float lr,
                                 float momentum, float weight_decay,
                                 void *stream);
KT_API kt_status kt_bucket_unpack_sgd_resident(kt_plan *plan, int bucket,
                                               const void *const *bucket_bufs,
                                               void *const *param_ptrs,
                                               void *const *momentum_ptrs,
                                               void *const *model_ptrs,
                                               int first_step, void *stream);

/*
 * The single pass from K gradient copies to updated parameters: kt_fused_step
 * and kt_bucket_unpack_sgd[_master] in one kernel.  Per element of every
 * tensor of the selected bucket(s)
 *     r  = round(w_0 * local_t[i] + sum_{k=1}^{K-1} w_k * peer_{b,k}[off_t + i])
 * with the arithmetic and rounding of kt_weighted_reduce (r in the bucket's
 * element type), then the update of kt_bucket_unpack_sgd on g = scale * r
 * (Sec. IV-B's optimizer).  The results are bit-identical to kt_bucket_pack ->
 * kt_weighted_reduce -> kt_bucket_unpack_sgd[_master]; the reduced gradient is
 * never written, so (K-1)*s + s + 16 bytes per element move instead of
 * (K+1)*s + s + 16 for kt_fused_step followed by an optimizer pass.
 *
 *   local_tensor_ptrs host, in: T device pointers, this device's gradients
 *                               (peer 0), read only.
 *   peer_bufs         host, in: device pointers, entry [b * (K-1) + (k-1)] =
 *                               peer k's copy of bucket b, k = 1..K-1
 *                               (ignored when K == 1).
 *   weights           host, in: K weights, or NULL for the weights set with
 *                               kt_plan_set_weights.
 *   param_ptrs, momentum_ptrs host, in: T device pointers each, binary32,
 *                               updated in place (momentum is written without
 *                               being read when first_step != 0).
 *   model_ptrs        host, in: NULL, or T device pointers to bf16 tensors that
 *                               receive every updated parameter rounded to
 *                               nearest-even (mixed precision).
 * Gradients, parameters, momentum, model parameters and peer buckets must not
 * overlap.  16-byte aligned addresses (8 for the model copy) take the vector
 * path.  kt_fused_step_sgd_resident reads the weights (kt_plan_set_weights) and
 * scale, lr, momentum, weight_decay (kt_plan_set_sgd) from the plan's device
 * memory when the kernel runs, for recorded graphs; KT_EINVAL if either was not
 * set.  A first step is refused under stream capture (KT_EUNSUPPORTED).
 */
KT_API kt_status kt_fused_step_sgd(kt_plan *plan, int bucket,
                                   const void *const *local_tensor_ptrs,
                                   const void *const *peer_bufs, int K,
                                   const float *weights, float scale,
                                   void *const *param_ptrs,
                                   void *const *momentum_ptrs,
                                   void *const *model_ptrs, float lr,
                                   float momentum, float weight_decay,
                                   int first_step, void *stream);
KT_API kt_status kt_fused_step_sgd_resident(kt_plan *plan, int bucket,
                                            const void *const *local_tensor_ptrs,
                                            const void *const *peer_bufs, int K,
                                            void *const *param_ptrs,
                                            void *const *momentum_ptrs,
                                            void *const *model_ptrs,
                                            int first_step, void *stream);

/*
 * kt_fused_step for callers that cannot allocate device memory: code that runs
 * under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, same kernels and bit-identical results, but the
 * plan's tables and the call's pointer table live in a device array of fixed
 * size that is part of the library's code object (one copy per GPU, held until
 * the process ends) instead of in memory the library allocates.  The call
 * allocates and frees nothing on the device and creates no events.
 *
 * Limits: tables (16 bytes per 16 KiB tile, 16 per tensor, 8 per bucket) plus
 * the pointer table must fit 4 MiB, and the pointer table (2 T + (K-1) *
 * num_buckets entries) 65536 entries; devices 0..15.  Beyond that the call
 * returns KT_EUNSUPPORTED and does nothing.
 *
 * All calls on one GPU share the array.  It keeps the tables of the last call:
 * a call with the same plan and the same pointers uploads nothing and only
 * enqueues its kernel (such a call may be recorded under stream capture); any
 * other call copies its tables into the array on `stream`, ordered behind the
 * work already enqueued there, and waits for those copies to finish before it
 * returns.  Calls that overlap in time on one GPU (different streams or
 * threads, or a graph replay of an earlier call against a new call) with
 * different plans or pointers race on the array: serialise them.  Nothing in
 * the array needs to start at zero.
 */
KT_API kt_status kt_fused_step_noalloc(kt_plan *plan, int bucket,
                                const void *const *local_tensor_ptrs,
                                const void *const *peer_bufs, int K,
                                const float *weights, float scale,
                                void *const *out_tensor_ptrs, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* KT_H */
