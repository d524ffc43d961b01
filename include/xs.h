/*
 * xs - fused gradient synchronisation for CrossoverScheduler (arXiv 2103.07974)
 *      on AMD Instinct MI355X (gfx950).  C99 interface of libxs.so.
 *
 * One synchronisation of one training task is
 *     pack      every worker's per-layer gradient tensors into one fused bucket
 *               (Section 2.1, tensor fusion; Algorithm 1 "Fuse all gradient into
 *               one group"),
 *     reduce    the W workers' buckets in worker order 0..W-1 and average them
 *               (Algorithm 1 "Receive averaged gradients"),
 *     update    the parameters with momentum SGD in the same pass
 *               (Algorithm 1 "Model Update", x <- SGD(x, g)),
 *     unpack    the updated parameter bucket into the per-layer tensors,
 * and the scheduler alternates one task's gradient computation with another
 * task's synchronisation on two HIP streams (Algorithm 1; Section 2.1).
 *
 * All W workers' gradients are resident on one GPU (that GPU's share of the
 * reduction); the library performs no communication.
 *
 * General rules
 *  - Every function returns an xs_status (0 = success, negative = error) and never
 *    throws or aborts.  Arguments are validated before anything is launched; on
 *    error nothing has been enqueued.  xs_last_error() gives a thread-local
 *    description of the last failure in the calling thread.
 *  - "device" pointers are HIP device addresses; "host" pointers are ordinary
 *    process memory that is read during the call only.
 *  - The caller owns every data buffer (tensors, pointer tables, buckets,
 *    parameters, momentum, flags).  The library owns only what *_create returns.
 *  - hip_stream is a hipStream_t passed as void* (NULL = the default stream).
 *    The four hot calls (xs_fuse_pack, xs_fused_reduce_sgd, xs_fuse_unpack,
 *    xs_crossover_step) only enqueue work and return; they allocate no memory
 *    and do not synchronise.  Execution errors surface at the caller's next
 *    synchronisation.
 *  - Calls act on the calling thread's current HIP device; every device pointer, stream and
 *    handle passed to one call must belong to that device.
 *  - Same inputs give bit-identical outputs on every call.
 */
#ifndef XS_H
#define XS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define XS_MAX_REPLICAS 32   /* largest W accepted by xs_fused_reduce_sgd */

typedef enum {
    XS_OK = 0,
    XS_ERR_INVALID_ARG = -1,  /* NULL required pointer, W out of range, bad handle, aliasing */
    XS_ERR_ALIGNMENT   = -2,  /* a bucket / parameter / momentum pointer is not 16-byte aligned */
    XS_ERR_SIZE        = -3,  /* offsets not monotone, overlap, sizes inconsistent */
    XS_ERR_UNSUPPORTED = -4,  /* unknown dtype or option */
    XS_ERR_HIP         = -5,  /* a HIP runtime call failed; see xs_last_error() */
    XS_ERR_NOMEM       = -6,  /* host or device allocation failed in a *_create call */
    XS_ERR_STATE       = -7   /* crossover call out of order (nothing to synchronise, or
                                 gradients that would be overwritten) */
} xs_status;

typedef enum { XS_F32 = 0, XS_F16 = 1, XS_BF16 = 2 } xs_dtype;   /* element types */

/* Static string for a status code. */
const char *xs_status_string(int status);
/* Thread-local detail of the last error in this thread ("" if none). */
const char *xs_last_error(void);

/* ------------------------------------------------------------------------
 * Bucket layout (Section 2.1: all tensors of one model form one united tensor).
 * offsets_out[0] = 0; offsets_out[t+1] = offsets_out[t] + numel[t] rounded up to
 * a multiple of align_elems; offsets_out[n_tensors] is the bucket length in
 * elements.  align_elems = 1 is plain concatenation.  Host pointers.
 * Errors: NULL pointer (n_tensors > 0), align_elems == 0.
 */
int xs_bucket_layout(const uint64_t *numel, uint32_t n_tensors, uint64_t align_elems,
                     uint64_t *offsets_out /* n_tensors + 1 */);

/* Where to put a task's flat buffers (the W replica buckets, the parameters, the momentum):
 * in ONE device allocation, each buffer starting at a multiple of XS_POOL_ALIGN bytes.  On
 * MI355X the fused reduce + SGD streams 4-7 % faster over such a pool than over W + 2 separate
 * allocations of the same sizes (measured; the library works with either).
 * offsets_out[i] = byte offset of buffer i from a base that is itself a multiple of
 * XS_POOL_ALIGN; offsets_out[n_buffers] = bytes needed behind that base.  Allocate
 * offsets_out[n_buffers] + XS_POOL_ALIGN bytes and round the returned address up.
 * Host pointers.  Errors: NULL pointer (n_buffers > 0), total overflowing 64 bits. */
#define XS_POOL_ALIGN (2u << 20)
int xs_pool_layout(const uint64_t *nbytes, uint32_t n_buffers, uint64_t *offsets_out);

/* ------------------------------------------------------------------------
 * Plan: device-resident description of one tensor list's place in its bucket.
 * numel[t], offsets[t] (host, read during the call): tensor t occupies bucket
 * elements [offsets[t], offsets[t]+numel[t]); offsets has n_tensors+1 entries,
 * offsets[0] == 0, offsets[t]+numel[t] <= offsets[t+1], and offsets[n_tensors]
 * is the bucket length.  Elements between a tensor's end and the next offset
 * are padding.  dtype is the element type moved by pack/unpack with this plan.
 * xs_plan_create allocates small device tables and synchronises once.  A plan must outlive
 * every kernel that was enqueued with it (destroy it after the stream has drained).
 * n_tensors == 0 and numel[t] == 0 are valid.
 */
typedef struct xs_plan xs_plan;
int xs_plan_create(const uint64_t *numel, const uint64_t *offsets, uint32_t n_tensors,
                   int dtype, xs_plan **out);
int xs_plan_destroy(xs_plan *plan);                 /* NULL is accepted */
uint64_t xs_plan_bucket_elems(const xs_plan *plan); /* offsets[n_tensors]; 0 for NULL */
uint32_t xs_plan_n_tensors(const xs_plan *plan);

/* ------------------------------------------------------------------------
 * Pack (Algorithm 1, "Fuse all gradient into one group"): bit copy of every
 * tensor into the bucket at its offset; padding elements are written as +0.
 *   tensor_ptrs  device array of n_tensors device pointers (element-aligned;
 *                any further alignment is handled), owned by the caller and
 *                read by the kernel when it runs
 *   bucket       device, 16-byte aligned, xs_plan_bucket_elems() elements
 *   found_inf    device int32, may be NULL; set to 1 by the kernel if any
 *                copied element is +-inf or NaN (never cleared by the library)
 * The bucket must not overlap any tensor.
 */
int xs_fuse_pack(const xs_plan *plan, const void *const *tensor_ptrs, void *bucket,
                 int32_t *found_inf, void *hip_stream);

/* The same for n (pointer table, bucket) pairs of one plan in a single launch - the W workers'
 * packs of one synchronisation.  tensor_ptr_tables and buckets are host arrays of n device
 * pointers; n <= XS_MAX_REPLICAS; n == 0 is a no-op. */
int xs_fuse_pack_many(const xs_plan *plan, const void *const *const *tensor_ptr_tables,
                      void *const *buckets, uint32_t n, int32_t *found_inf, void *hip_stream);

/* xs_fuse_pack for callers that cannot allocate device memory or create a plan first: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Takes the
 * layout as xs_plan_create does (numel, offsets: host arrays read during the call) and
 * everything else as xs_fuse_pack does.  The device tables that a plan would own are
 * rewritten, on hip_stream and in front of the pack, inside a fixed device array of the
 * library (about 41 KiB per GPU, held until the process ends) by small kernels that carry the
 * entries in their arguments; the call allocates nothing and copies nothing from host memory.
 *   - n_tensors > XS_STATIC_MAX_TENSORS returns XS_ERR_SIZE.
 *   - Every call on a GPU uses that GPU's one array: calls on one stream are ordered and
 *     correct; calls that may overlap in time on one GPU (different streams or threads) race
 *     on the tables and must be serialised by the caller.
 *   - The first call on a device resolves the array's address (a host-side lookup).
 */
#define XS_STATIC_MAX_TENSORS 2048
int xs_fuse_pack_static(const uint64_t *numel, const uint64_t *offsets, uint32_t n_tensors,
                        int dtype, const void *const *tensor_ptrs, void *bucket,
                        int32_t *found_inf, void *hip_stream);

/* Unpack: inverse of pack.  Copies each tensor's range of the bucket to
 * tensor_ptrs[t]; padding is ignored.  Same pointer conventions as pack. */
int xs_fuse_unpack(const xs_plan *plan, const void *bucket, void *const *tensor_ptrs,
                   void *hip_stream);

/* ------------------------------------------------------------------------
 * Fused reduce + average + momentum-SGD (Algorithm 1, "Receive averaged
 * gradients" and "Model Update"), one pass over memory.  For every j < n_elems
 *     s = g_0[j] + g_1[j] + ... + g_{W-1}[j]     (left to right, fp32;
 *                                                 fp16 / bf16 gradients widened first)
 *     g = s * (inv_loss_scale * (1/W))
 *     d = g + weight_decay * x[j];  v[j] = momentum * v[j] + d;  x[j] -= lr * v[j]
 * every operation rounded to fp32 separately (no fused multiply-add).
 *
 *   replica_buckets  host array of W device pointers, each 16-byte aligned and
 *                    holding n_elems elements of grad_dtype; replicas may alias
 *                    one another but not the parameter or momentum buffers
 *   params, momentum device fp32, 16-byte aligned, n_elems each
 *   params_out, momentum_out   both NULL: update in place.  Both non-NULL
 *                    (16-byte aligned, n_elems, overlapping nothing else):
 *                    results are written there and the inputs are left intact.
 *   found_inf        device int32, may be NULL.  If non-NULL and nonzero when the
 *                    kernel starts, the kernel writes nothing (step skipped).
 *                    In the out-of-place form the kernel additionally sets it to
 *                    1 when any gradient element in [0, n_elems) is +-inf or
 *                    NaN; the caller then discards the outputs.  The in-place
 *                    form relies on xs_fuse_pack having raised the flag on the
 *                    same stream, since an in-place pass cannot be undone.
 * W in [1, XS_MAX_REPLICAS].  n_elems == 0 is a no-op.
 */
typedef struct {
    float lr;
    float momentum;
    float weight_decay;
    float inv_loss_scale;   /* 1.0f when no loss scaling is used */
} xs_sgd_hparams;

int xs_fused_reduce_sgd(const void *const *replica_buckets, uint32_t W, int grad_dtype,
                        uint64_t n_elems, float *params, float *momentum,
                        float *params_out, float *momentum_out,
                        const xs_sgd_hparams *hp, int32_t *found_inf, void *hip_stream);

/* Mixed-precision outputs (beyond the paper: the practical surface around SGD(x, g) when the
 * model computes in half precision and the optimizer keeps fp32 master weights).
 *   model_copy        xs_fused_reduce_sgd_mp only: device, 16-byte aligned, n_elems half-
 *                     precision elements in bucket layout, or NULL.  Receives the updated
 *                     parameters rounded to nearest even, in the same pass (+2 bytes/element).
 *                     XS_ERR_UNSUPPORTED together with in-kernel overflow detection
 *                     (out-of-place outputs and found_inf both given): the copy is the live
 *                     model, and a pass that is still deciding whether the step is skipped
 *                     must not overwrite part of it.
 *   model_copy_dtype  XS_F16 or XS_BF16.
 *   view_dtype        xs_fused_gather_reduce_sgd_mp only: element type of the per-layer views
 *                     that param_tensor_ptrs point to: XS_F32, XS_F16 or XS_BF16.
 * A NULL xs_mp_options pointer means: no model copy, fp32 views.
 */
typedef struct {
    void *model_copy;
    int model_copy_dtype;
    int view_dtype;
} xs_mp_options;

int xs_fused_reduce_sgd_mp(const void *const *replica_buckets, uint32_t W, int grad_dtype,
                           uint64_t n_elems, float *params, float *momentum,
                           float *params_out, float *momentum_out,
                           const xs_sgd_hparams *hp, int32_t *found_inf,
                           const xs_mp_options *mp, void *hip_stream);

/* ------------------------------------------------------------------------
 * The same pass without materialised buckets (Section 2.1 fuses the tensors only
 * because the fused tensor has to be sent; on one GPU the layout alone suffices):
 * element j of the bucket layout of gradient_plan is read from worker w's tensor
 * that covers j, padding contributes +0, and the result is bit-identical to
 * xs_fuse_pack x W + xs_fused_reduce_sgd (+ xs_fuse_unpack).
 *   grad_ptrs          device array of n_tensors*W device pointers, laid out
 *                      [tensor][worker]; element-aligned tensors of the plan's dtype
 *   params, momentum, params_out, momentum_out, hp, found_inf   as in
 *                      xs_fused_reduce_sgd, bucket layout, xs_plan_bucket_elems() long
 *   param_tensor_ptrs  device array of n_tensors device pointers to fp32 per-layer
 *                      parameter tensors, or NULL.  If given, the updated parameters
 *                      are also written there in the same pass (no separate unpack).
 *                      XS_ERR_UNSUPPORTED together with in-kernel overflow detection
 *                      (out-of-place outputs and found_inf both given).
 * No xs_fuse_pack runs in this form, so nothing raises found_inf before an in-place
 * pass; mixed-precision callers use the out-of-place form and commit by swapping
 * pointers when the flag is still zero.
 */
int xs_fused_gather_reduce_sgd(const xs_plan *gradient_plan, const void *const *grad_ptrs,
                               uint32_t W, float *params, float *momentum,
                               float *params_out, float *momentum_out,
                               void *const *param_tensor_ptrs, const xs_sgd_hparams *hp,
                               int32_t *found_inf, void *hip_stream);
/* As above with mixed-precision options: mp->view_dtype selects half-precision views;
 * mp->model_copy must be NULL here (XS_ERR_UNSUPPORTED otherwise). */
int xs_fused_gather_reduce_sgd_mp(const xs_plan *gradient_plan, const void *const *grad_ptrs,
                                  uint32_t W, float *params, float *momentum,
                                  float *params_out, float *momentum_out,
                                  void *const *param_tensor_ptrs, const xs_sgd_hparams *hp,
                                  int32_t *found_inf, const xs_mp_options *mp, void *hip_stream);

/* ------------------------------------------------------------------------
 * Hyper-parameters per tensor (beyond the paper, whose "Model Update" is a bare SGD(x, g):
 * optimizers apply it with parameter groups - no weight decay on biases and normalisation
 * layers, a learning rate per group).  One 16-byte record per tensor of the plan, in a device
 * array the caller owns.  Record t governs bucket elements offsets[t] .. offsets[t+1]-1, i.e.
 * tensor t and the padding behind it; the arithmetic per element is that of
 * xs_fused_reduce_sgd with the record's values in place of hp's, and inv_loss_scale stays
 * one value for the whole bucket.
 */
typedef struct {
    float lr;
    float momentum;
    float weight_decay;
    float reserved;          /* pads the record to 16 bytes; not read */
} xs_tensor_hparams;

/* xs_fused_reduce_sgd_mp with a record per tensor.  The replica buckets, params and momentum
 * have the layout of gradient_plan (whose dtype is the gradients' and whose
 * xs_plan_bucket_elems() is the element count); everything else as in xs_fused_reduce_sgd_mp.
 *   tensor_hp   device, 16-byte aligned, xs_plan_n_tensors() records; read by the kernel, so
 *               it must stay valid and unchanged until the pass has run.
 */
int xs_fused_reduce_sgd_pt(const xs_plan *gradient_plan, const void *const *replica_buckets,
                           uint32_t W, float *params, float *momentum,
                           float *params_out, float *momentum_out,
                           const xs_tensor_hparams *tensor_hp, float inv_loss_scale,
                           int32_t *found_inf, const xs_mp_options *mp, void *hip_stream);

/* xs_fused_gather_reduce_sgd_mp with a record per tensor; tensor_hp as above. */
int xs_fused_gather_reduce_sgd_pt(const xs_plan *gradient_plan, const void *const *grad_ptrs,
                                  uint32_t W, float *params, float *momentum,
                                  float *params_out, float *momentum_out,
                                  void *const *param_tensor_ptrs,
                                  const xs_tensor_hparams *tensor_hp, float inv_loss_scale,
                                  int32_t *found_inf, const xs_mp_options *mp, void *hip_stream);

/* ------------------------------------------------------------------------
 * xs_fused_reduce_sgd (in place) with the unpack fused in: the updated parameters are also
 * written to the per-layer tensors in the same pass, which saves the separate unpack's read
 * of the parameter bucket (Section 2.1 fuses the tensors so that they can be sent; the way
 * back to the layers needs no pass of its own).  The replica buckets, params and momentum
 * have the layout of gradient_plan, whose dtype is the gradients'.
 *   param_tensor_ptrs  device array of xs_plan_n_tensors() device pointers to the per-layer
 *                      parameter tensors (element-aligned); element type fp32, or
 *                      mp->view_dtype (XS_F16 / XS_BF16: half-precision model weights
 *                      rounded to nearest even from the fp32 master update)
 *   hp                 lr / momentum / weight_decay for the whole bucket when tensor_hp is
 *                      NULL; inv_loss_scale always
 *   tensor_hp          device, one record per tensor, or NULL (see xs_tensor_hparams below)
 *   found_inf          as in the in-place xs_fused_reduce_sgd: if raised when the kernel
 *                      starts nothing is written, the views keep the unchanged parameters
 *   mp                 may be NULL; mp->model_copy is honoured as in xs_fused_reduce_sgd_mp
 * Bit-identical to xs_fused_reduce_sgd(_pt) followed by xs_fuse_unpack.
 */
int xs_fused_reduce_sgd_unpack(const xs_plan *gradient_plan, const void *const *replica_buckets,
                               uint32_t W, float *params, float *momentum,
                               void *const *param_tensor_ptrs, const xs_sgd_hparams *hp,
                               const xs_tensor_hparams *tensor_hp, int32_t *found_inf,
                               const xs_mp_options *mp, void *hip_stream);

/* ------------------------------------------------------------------------
 * Launch settings.  xs_tuning_set changes the process-wide values that every call outside an
 * xs_app reads (one consistent snapshot per call; setting a value while another thread
 * launches is safe, that launch sees the old or the new value).  A task that must be
 * launched differently from the rest of the process - e.g. paced so that it runs beside
 * another task's computation - carries its own values in xs_app_desc.tuning instead.
 * The defaults are the measured best for a synchronisation that has MI355X to itself.
 * Returns XS_ERR_INVALID_ARG for an unknown key or an out-of-range value.
 */
typedef enum {
    XS_TUNE_REDUCE_WG_PER_CU = 0,   /* reduce kernels: workgroups per compute unit for a grid-stride
                                       launch; 0 (default) = one 16-byte vector per lane, no loop */
    XS_TUNE_COPY_WG_PER_CU = 1,     /* pack/unpack: workgroups per compute unit of a persistent grid;
                                       0 (default) = one KiB row of the bucket per wavefront, dispatched
                                       in bucket order */
    XS_TUNE_NT_GRADS = 2,           /* bucket-form reduce: non-temporal gradient loads (0/1, default 1) */
    XS_TUNE_NT_STATE = 3,           /* bucket-form reduce: non-temporal parameter/momentum accesses (0/1, default 1) */
    XS_TUNE_REDUCE_LDS_RESERVE = 4, /* bytes of LDS reserved per reduce workgroup; the kernel uses no
                                       LDS, the reservation caps how many workgroups share a compute
                                       unit; -1 (default) = 16384: ten one-wave workgroups per compute unit
                                       (20480 to 28672, eight to five, for most instances with the
                                       unpack fused in and for 16 half-precision replicas with
                                       per-tensor records) */
    XS_TUNE_REDUCE_MAX_WG = 5,      /* absolute cap on reduce workgroups, 0 = none */
    XS_TUNE_COPY_MAX_WG = 6,        /* absolute cap on pack/unpack workgroups, 0 = none */
    XS_TUNE_COPY_NT = 7,            /* pack/unpack: non-temporal accesses (0/1, default 1) */
    XS_TUNE_GATHER_LDS_RESERVE = 8, /* as 4 for the gathering form; -1 = 8192 to 12288 fp32, 10240 to
                                       16384 half, by W */
    XS_TUNE_COPY_LDS_RESERVE = 9,   /* pack/unpack: bytes of LDS reserved per workgroup (the kernel uses
                                       none; caps the workgroups per compute unit); -1 (default) = 0 */
    XS_TUNE_REDUCE_WAVES_PER_WG = 10, /* gathering form and the generic-W bucket-form kernel (any W outside
                                       2/4/8/16, or XS_TUNE_REDUCE_SMALL): wavefronts per workgroup, 1
                                       (default), 2 or 4; the four wavefronts of a 4-wave workgroup land
                                       on the four SIMDs of one compute unit.  The W-specialised
                                       bucket-form kernels always use one-wavefront workgroups */
    XS_TUNE_REDUCE_SMALL = 11,      /* bucket-form reduce: 0 (default) = the kernel specialised for W with all
                                       W + 2 loads in flight (54 to 85 registers per lane); 1 = the
                                       generic-W kernel whatever W is: four replica loads in flight at a
                                       time, 28 (fp32) to 47 (fp16) registers per lane, same arithmetic */
    XS_TUNE_COPY_WAVES_PER_WG = 12, /* pack/unpack: wavefronts per workgroup, 1 (default), 2 or 4; each
                                       wavefront moves one KiB row of the bucket */
    XS_TUNE_COUNT = 13
} xs_tuning_key;
int xs_tuning_set(int key, int value);
int xs_tuning_get(int key, int *value_out);

/* Fills values_out[XS_TUNE_COUNT] with a named set of launch settings for xs_app_desc.tuning.
 *   XS_PRESET_ALONE           the defaults: the synchronisation has the GPU to itself
 *   XS_PRESET_BESIDE_COMPUTE  the synchronisation shares every compute unit with another
 *                             task's kernels (Section 2.1): one 4-wave workgroup per compute
 *                             unit at a time (one wavefront per SIMD, at most 48 registers
 *                             per lane in the bucket form) holding an LDS reservation of
 *                             82 KiB, so that a second synchronisation workgroup never fits
 *                             while 78 KiB of LDS, 7/8 of the wave slots and 29/32 of the
 *                             register file stay free for the other task's workgroups at
 *                             all times
 *   XS_PRESET_LEAVE_WAVE_SLOTS  as ALONE, but pack and unpack hold a 16 KiB LDS reservation per
 *                             one-wave workgroup: ten per compute unit instead of every wave
 *                             slot (their stand-alone rate falls from 6.4 to 4.1 TB/s).  The
 *                             reduce kernels keep that much room by default.  For a task whose
 *                             neighbour launches few long-lived workgroups: dispatched while
 *                             copies fill every wave slot they land on whichever compute
 *                             units have room first and stay unevenly spread.  Beside kernels
 *                             that own whole compute units (GEMM macro-tiles) the slower copies
 *                             only hold the compute units longer: use the defaults there
 * XS_ERR_INVALID_ARG for an unknown preset or a NULL pointer.
 */
typedef enum { XS_PRESET_ALONE = 0, XS_PRESET_BESIDE_COMPUTE = 1, XS_PRESET_LEAVE_WAVE_SLOTS = 2 } xs_tuning_preset_id;
int xs_tuning_preset(int preset, int32_t *values_out /* XS_TUNE_COUNT */);

/* ------------------------------------------------------------------------
 * Training task ("distributed task i" of Algorithm 1) as seen by the scheduler.
 * All pointers in the descriptor are copied or referenced as stated and must
 * stay valid until xs_app_destroy.
 */
typedef void (*xs_compute_fn)(void *user_ctx, void *hip_stream);
/* Enqueues the task's gradient computation (forward + backward) on hip_stream and
 * returns without blocking; it must leave worker w's gradients in the tensors
 * that grad_tensor_ptrs[w] points to. */

typedef struct {
    const xs_plan *gradient_plan;            /* layout in the gradient dtype          */
    const xs_plan *parameter_plan;           /* same layout, dtype XS_F32             */
    uint32_t W;                              /* workers resident on this GPU          */
    const void *const *const *grad_tensor_ptrs; /* host array of W device pointer tables  */
    void *const *replica_buckets;            /* host array of W device buckets        */
    float *params;                           /* device, bucket layout, fp32           */
    float *momentum;                         /* device, bucket layout, fp32           */
    void *const *param_tensor_ptrs;          /* device pointer table of parameter views */
    xs_sgd_hparams hp;
    int32_t *found_inf;                      /* device, may be NULL; see below        */
    xs_compute_fn compute;                   /* may be NULL (no compute enqueued)     */
    void *compute_ctx;
    uint32_t flags;                          /* XS_APP_* bits                         */
    const void *const *grad_ptrs_tw;         /* device [n_tensors][W] table; required
                                                with XS_APP_FUSED_GATHER, else may be NULL */
    const xs_tensor_hparams *tensor_hp;      /* device, one record per tensor, or NULL:
                                                hp's lr/momentum/weight_decay for all     */
    const int32_t *tuning;                   /* host, XS_TUNE_COUNT launch settings copied at
                                                xs_app_create (see xs_tuning_preset), or NULL:
                                                the process-wide settings at every call   */
} xs_app_desc;

/* Synchronise with xs_fused_gather_reduce_sgd (gradients read from the per-layer tensors,
 * parameters written to the views in the same pass) instead of W packs + reduce + unpack.
 * replica_buckets and grad_tensor_ptrs are then unused and may be NULL.  No pack runs in this
 * form, so nothing could raise found_inf before the in-place pass: xs_app_create returns
 * XS_ERR_UNSUPPORTED when found_inf is given together with this flag. */
#define XS_APP_FUSED_GATHER 1u

/* Synchronise with W packs (one launch) + xs_fused_reduce_sgd_unpack: the buckets exist, as
 * they must where the fused tensor is what gets sent, but the unpack has no pass of its own. */
#define XS_APP_FUSED_UNPACK 2u

/* xs_app_desc.found_inf - loss-scale overflow inside the scheduler (beyond the paper).
 * The W packs of a synchronisation raise the flag when any gradient element of any worker is
 * +-inf or NaN; the reduce + SGD enqueued behind them then leaves parameters and momentum
 * untouched, and the unpack hands the unchanged parameters back.  The library never clears
 * the flag: while it is up every later synchronisation of the task is skipped as well.
 * The caller clears it on the SYNC stream (a one-word fill kernel or copy enqueued there is
 * ordered after the synchronisation that read it and before the next one), typically right
 * after it has looked at the flag's value behind sync_done (xs_app_wait_sync) to rescale
 * the loss.  A caller that never looks keeps the enqueue-only contract of Algorithm 1 and
 * simply loses every step after the first overflow. */

typedef struct xs_app xs_app;
int xs_app_create(const xs_app_desc *desc, xs_app **out);   /* creates two HIP events */
int xs_app_destroy(xs_app *app);                            /* NULL is accepted */

/* The whole synchronisation of one task on one stream: W packs, fused
 * reduce + SGD in place, unpack of the parameters.  Enqueue only. */
int xs_app_sync(xs_app *app, void *hip_stream);

/* One inner step of Algorithm 1 for two tasks: compute_app's gradient computation
 * is enqueued on compute_stream (after its own previous synchronisation, so that
 * it sees updated parameters) while sync_app's synchronisation is enqueued on
 * sync_stream (after the computation that produced its gradients).  sync_app ==
 * NULL is the first-iteration bypass of Section 2.2.  Returns XS_ERR_STATE if
 * sync_app has no gradients outstanding, or if compute_app still has: its gradient
 * tensors would be overwritten before they were synchronised.  Enqueue only; no host
 * synchronisation.
 */
int xs_crossover_step(xs_app *compute_app, xs_app *sync_app,
                      void *compute_stream, void *sync_stream);

/* The additional synchronisation phase after the last iteration (Section 2.2):
 * synchronises app's outstanding gradients on sync_stream.  XS_ERR_STATE if none. */
int xs_crossover_drain(xs_app *app, void *sync_stream);

/* One outer iteration of Algorithm 1 over N tasks ("for i = 1..N"): apps[i] computes while
 * the task of the previous inner step (apps[i-1]; apps[N-1] of the previous call for i = 0)
 * is synchronised, if its gradients are outstanding - they are not at the very first inner
 * step (the bypass of Section 2.2).  Every synchronisation thus has the N-1 computations that
 * follow it to hide under before its own task computes again.  n_apps == 1 degenerates to
 * compute, then synchronise.  The same array, in the same order, is expected on every call.
 * Enqueue only; stops at the first error and returns it.
 */
int xs_crossover_iteration(xs_app *const *apps, uint32_t n_apps,
                           void *compute_stream, void *sync_stream);

/* The additional synchronisation phase after the last iteration for N tasks: synchronises
 * every app of the array whose gradients are still outstanding, in array order.  XS_OK if
 * none is. */
int xs_crossover_finish(xs_app *const *apps, uint32_t n_apps, void *sync_stream);

/* Makes hip_stream wait for app's last enqueued synchronisation (no-op if none). */
int xs_app_wait_sync(xs_app *app, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* XS_H */
