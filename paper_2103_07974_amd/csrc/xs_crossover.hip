// Two-stream crossover driver (arXiv 2103.07974, Algorithm 1 and Section 2.1).
//
// A task's gradient computation runs on the compute stream; its synchronisation
// (the W packs in one launch, fused reduce + SGD, unpack; the last two in one pass with
// XS_APP_FUSED_UNPACK; or the single gathering kernel when the task was created with
// XS_APP_FUSED_GATHER) runs on the sync stream.  Two events per
// task carry the only dependencies the algorithm has:
//   grads_ready  recorded on the compute stream after the task's computation;
//                the task's synchronisation waits for it ("Send ... for gradient
//                synchronization" follows "Gradient computation");
//   sync_done    recorded on the sync stream after the task's unpack; the task's
//                next computation waits for it, so it sees the updated model
//                ("Model Update" precedes the next "Gradient computation" of the
//                same task).
// Nothing else orders the two streams, so one task's synchronisation overlaps the
// other task's computation, and no call blocks the host.
#include <new>
#include <vector>

#include "xs_internal.h"

struct xs_app {
    uint32_t magic;
    const xs_plan *gplan;
    const xs_plan *pplan;
    uint32_t W;
    std::vector<const void *const *> grad_tables;   // W device pointer tables
    std::vector<void *> buckets;                    // W device buckets
    float *params;
    float *momentum;
    void *const *param_table;
    const void *const *gather_table;   // device [T][W], fused-gather mode
    uint32_t flags;
    xs_sgd_hparams hp;
    const xs_tensor_hparams *tensor_hp;   // device records per tensor, or nullptr
    int32_t *found_inf;
    xs_compute_fn compute;
    void *compute_ctx;
    hipEvent_t grads_ready;
    hipEvent_t sync_done;
    bool grads_outstanding;   // grads_ready recorded and not yet consumed by a sync
    bool has_sync;            // sync_done has been recorded at least once
    bool own_tuning;          // launch settings of its own (xs_app_desc.tuning)
    xs::Tuning tuning;
};

using namespace xs;

static bool is_app(const xs_app *a) { return a && a->magic == XS_APP_MAGIC; }

extern "C" int xs_app_create(const xs_app_desc *d, xs_app **out)
{
    if (!out) return fail(XS_ERR_INVALID_ARG, "xs_app_create: out is NULL");
    *out = nullptr;
    if (!d) return fail(XS_ERR_INVALID_ARG, "xs_app_create: desc is NULL");
    if (!d->gradient_plan || d->gradient_plan->magic != XS_PLAN_MAGIC || !d->parameter_plan ||
        d->parameter_plan->magic != XS_PLAN_MAGIC)
        return fail(XS_ERR_INVALID_ARG, "xs_app_create: gradient_plan/parameter_plan is not a plan");
    if (d->parameter_plan->dtype != XS_F32)
        return fail(XS_ERR_UNSUPPORTED, "xs_app_create: parameter_plan must have dtype XS_F32");
    if (d->gradient_plan->bucket_elems != d->parameter_plan->bucket_elems ||
        d->gradient_plan->n_tensors != d->parameter_plan->n_tensors)
        return fail(XS_ERR_SIZE, "xs_app_create: gradient and parameter plans differ in layout");
    if (d->W == 0 || d->W > XS_MAX_REPLICAS)
        return fail(XS_ERR_INVALID_ARG, "xs_app_create: W = %u outside [1, %d]", d->W, XS_MAX_REPLICAS);
    const bool empty = d->gradient_plan->bucket_elems == 0;
    if (d->flags & ~(XS_APP_FUSED_GATHER | XS_APP_FUSED_UNPACK))
        return fail(XS_ERR_UNSUPPORTED, "xs_app_create: unknown flags 0x%x", d->flags);
    if ((d->flags & XS_APP_FUSED_GATHER) && (d->flags & XS_APP_FUSED_UNPACK))
        return fail(XS_ERR_UNSUPPORTED, "xs_app_create: XS_APP_FUSED_GATHER and XS_APP_FUSED_UNPACK exclude each other");
    const bool gather = (d->flags & XS_APP_FUSED_GATHER) != 0;
    if (!empty && (!d->params || !d->momentum || !d->param_tensor_ptrs))
        return fail(XS_ERR_INVALID_ARG, "xs_app_create: a required pointer is NULL");
    if (!empty && gather && !d->grad_ptrs_tw)
        return fail(XS_ERR_INVALID_ARG, "xs_app_create: XS_APP_FUSED_GATHER needs grad_ptrs_tw");
    if (gather && d->found_inf)
        return fail(XS_ERR_UNSUPPORTED,
                    "xs_app_create: found_inf cannot be honoured with XS_APP_FUSED_GATHER: no pack runs "
                    "that could raise the flag before the in-place pass");
    Tuning tuning = {};
    if (d->tuning) {
        const int rc = tuning_check(d->tuning, &tuning);
        if (rc != XS_OK) return rc;
    }
    if (!empty && !gather && (!d->grad_tensor_ptrs || !d->replica_buckets))
        return fail(XS_ERR_INVALID_ARG, "xs_app_create: a required pointer is NULL");
    if (!empty) {
        if (!aligned16(d->params) || !aligned16(d->momentum))
            return fail(XS_ERR_ALIGNMENT, "xs_app_create: params/momentum must be 16-byte aligned");
        if (d->tensor_hp && !aligned16(d->tensor_hp))
            return fail(XS_ERR_ALIGNMENT, "xs_app_create: tensor_hp must be 16-byte aligned");
        for (uint32_t w = 0; !gather && w < d->W; ++w) {
            if (!d->grad_tensor_ptrs[w] || !d->replica_buckets[w])
                return fail(XS_ERR_INVALID_ARG, "xs_app_create: worker %u has a NULL table or bucket", w);
            if (!aligned16(d->replica_buckets[w]))
                return fail(XS_ERR_ALIGNMENT, "xs_app_create: replica_buckets[%u] is not 16-byte aligned", w);
        }
    }
    xs_app *a = new (std::nothrow) xs_app();
    if (!a) return fail(XS_ERR_NOMEM, "xs_app_create: host allocation failed");
    a->magic = XS_APP_MAGIC;
    a->gplan = d->gradient_plan;
    a->pplan = d->parameter_plan;
    a->W = d->W;
    if (!empty && !gather) {
        try {
            a->grad_tables.assign(d->grad_tensor_ptrs, d->grad_tensor_ptrs + d->W);
            a->buckets.assign(d->replica_buckets, d->replica_buckets + d->W);
        } catch (const std::bad_alloc &) {
            delete a;
            return fail(XS_ERR_NOMEM, "xs_app_create: host allocation failed");
        }
    }
    a->gather_table = d->grad_ptrs_tw;
    a->flags = d->flags;
    a->params = d->params;
    a->momentum = d->momentum;
    a->param_table = d->param_tensor_ptrs;
    a->hp = d->hp;
    a->tensor_hp = d->tensor_hp;
    a->found_inf = d->found_inf;
    a->compute = d->compute;
    a->compute_ctx = d->compute_ctx;
    a->grads_outstanding = false;
    a->has_sync = false;
    a->own_tuning = d->tuning != nullptr;
    a->tuning = tuning;
    a->grads_ready = nullptr;
    a->sync_done = nullptr;
    hipError_t e = hipEventCreateWithFlags(&a->grads_ready, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&a->sync_done, hipEventDisableTiming);
    if (e != hipSuccess) {
        if (a->grads_ready) (void)hipEventDestroy(a->grads_ready);
        delete a;
        return fail_hip(e, "hipEventCreateWithFlags");
    }
    *out = a;
    return XS_OK;
}

extern "C" int xs_app_destroy(xs_app *a)
{
    if (!a) return XS_OK;
    if (!is_app(a)) return fail(XS_ERR_INVALID_ARG, "xs_app_destroy: not an app");
    a->magic = 0;
    hipError_t e1 = hipEventDestroy(a->grads_ready);
    hipError_t e2 = hipEventDestroy(a->sync_done);
    delete a;
    if (e1 != hipSuccess) return fail_hip(e1, "hipEventDestroy");
    if (e2 != hipSuccess) return fail_hip(e2, "hipEventDestroy");
    return XS_OK;
}

// Algorithm 1: fuse, synchronise (average), update; then hand the model back per layer.
static int enqueue_sync(xs_app *a, hipStream_t s)
{
    if (a->gplan->bucket_elems == 0) return XS_OK;
    const Tuning tn = a->own_tuning ? a->tuning : tuning_now();
    if (a->flags & XS_APP_FUSED_GATHER)
        return gather_reduce_sgd_impl(tn, a->gplan, a->gather_table, a->W, a->params, a->momentum,
                                      nullptr, nullptr, a->param_table, &a->hp, a->tensor_hp,
                                      nullptr, nullptr, s);
    int rc = fuse_pack_many_impl(tn, a->gplan, a->grad_tables.data(), a->buckets.data(), a->W,
                                 a->found_inf, s);
    if (rc != XS_OK) return rc;
    if (a->flags & XS_APP_FUSED_UNPACK)
        return reduce_sgd_unpack_impl(tn, a->gplan, (const void *const *)a->buckets.data(), a->W,
                                      a->params, a->momentum, a->param_table, &a->hp, a->tensor_hp,
                                      a->found_inf, nullptr, s);
    if (a->tensor_hp)
        rc = reduce_sgd_pt_impl(tn, a->gplan, (const void *const *)a->buckets.data(), a->W, a->params,
                                a->momentum, nullptr, nullptr, a->tensor_hp, a->hp.inv_loss_scale,
                                a->found_inf, nullptr, s);
    else
        rc = reduce_sgd_impl(tn, nullptr, nullptr, (const void *const *)a->buckets.data(), a->W,
                             a->gplan->dtype, a->gplan->bucket_elems, a->params, a->momentum, nullptr,
                             nullptr, &a->hp, a->found_inf, nullptr, nullptr, s);
    if (rc != XS_OK) return rc;
    return fuse_unpack_impl(tn, a->pplan, a->params, a->param_table, s);
}

extern "C" int xs_app_sync(xs_app *a, void *hip_stream)
{
    if (!is_app(a)) return fail(XS_ERR_INVALID_ARG, "xs_app_sync: app is NULL or not an app");
    return enqueue_sync(a, (hipStream_t)hip_stream);
}

static int sync_on_stream(xs_app *y, hipStream_t ss)
{
    XS_HIP_TRY(hipStreamWaitEvent(ss, y->grads_ready, 0));
    int rc = enqueue_sync(y, ss);
    if (rc != XS_OK) return rc;
    XS_HIP_TRY(hipEventRecord(y->sync_done, ss));
    y->has_sync = true;
    y->grads_outstanding = false;
    return XS_OK;
}

static int compute_on_stream(xs_app *x, hipStream_t cs)
{
    if (x->has_sync) XS_HIP_TRY(hipStreamWaitEvent(cs, x->sync_done, 0));
    if (x->compute) x->compute(x->compute_ctx, (void *)cs);
    XS_HIP_TRY(hipEventRecord(x->grads_ready, cs));
    x->grads_outstanding = true;
    return XS_OK;
}

extern "C" int xs_crossover_step(xs_app *x, xs_app *y, void *compute_stream, void *sync_stream)
{
    if (!is_app(x)) return fail(XS_ERR_INVALID_ARG, "xs_crossover_step: compute_app is NULL or not an app");
    if (y && !is_app(y)) return fail(XS_ERR_INVALID_ARG, "xs_crossover_step: sync_app is not an app");
    hipStream_t cs = (hipStream_t)compute_stream, ss = (hipStream_t)sync_stream;
    if (x->grads_outstanding)
        return fail(XS_ERR_STATE, "xs_crossover_step: compute_app's previous gradients have not been "
                                  "synchronised; computing again would overwrite them");
    if (y == x) {
        // a single task degenerates to compute, then synchronise, in order
        int rc = compute_on_stream(x, cs);
        if (rc != XS_OK) return rc;
        return sync_on_stream(x, ss);
    }
    if (y && !y->grads_outstanding)
        return fail(XS_ERR_STATE, "xs_crossover_step: sync_app has no gradients outstanding");
    // the synchronisation is enqueued first: its few launches reach the GPU while the
    // host is still issuing the computation
    if (y) {
        int rc = sync_on_stream(y, ss);
        if (rc != XS_OK) return rc;
    }
    return compute_on_stream(x, cs);
}

extern "C" int xs_crossover_drain(xs_app *a, void *sync_stream)
{
    if (!is_app(a)) return fail(XS_ERR_INVALID_ARG, "xs_crossover_drain: app is NULL or not an app");
    if (!a->grads_outstanding)
        return fail(XS_ERR_STATE, "xs_crossover_drain: app has no gradients outstanding");
    return sync_on_stream(a, (hipStream_t)sync_stream);
}

// Algorithm 1, the inner loop "for i = 1..N" of one outer iteration.
extern "C" int xs_crossover_iteration(xs_app *const *apps, uint32_t n_apps, void *compute_stream,
                                      void *sync_stream)
{
    if (n_apps == 0) return XS_OK;
    if (!apps) return fail(XS_ERR_INVALID_ARG, "xs_crossover_iteration: apps is NULL");
    for (uint32_t i = 0; i < n_apps; ++i) {
        if (!is_app(apps[i]))
            return fail(XS_ERR_INVALID_ARG, "xs_crossover_iteration: apps[%u] is NULL or not an app", i);
        for (uint32_t k = 0; k < i; ++k)
            if (apps[k] == apps[i])
                return fail(XS_ERR_INVALID_ARG, "xs_crossover_iteration: apps[%u] and apps[%u] are the same app", k, i);
    }
    for (uint32_t i = 0; i < n_apps; ++i) {
        xs_app *x = apps[i];
        xs_app *y = n_apps == 1 ? x : apps[(i + n_apps - 1) % n_apps];
        if (y != x && !y->grads_outstanding) y = nullptr;      // first-iteration bypass
        const int rc = xs_crossover_step(x, y, compute_stream, sync_stream);
        if (rc != XS_OK) return rc;
    }
    return XS_OK;
}

extern "C" int xs_crossover_finish(xs_app *const *apps, uint32_t n_apps, void *sync_stream)
{
    if (n_apps == 0) return XS_OK;
    if (!apps) return fail(XS_ERR_INVALID_ARG, "xs_crossover_finish: apps is NULL");
    for (uint32_t i = 0; i < n_apps; ++i)
        if (!is_app(apps[i]))
            return fail(XS_ERR_INVALID_ARG, "xs_crossover_finish: apps[%u] is NULL or not an app", i);
    for (uint32_t i = 0; i < n_apps; ++i) {
        if (!apps[i]->grads_outstanding) continue;
        const int rc = sync_on_stream(apps[i], (hipStream_t)sync_stream);
        if (rc != XS_OK) return rc;
    }
    return XS_OK;
}

extern "C" int xs_app_wait_sync(xs_app *a, void *hip_stream)
{
    if (!is_app(a)) return fail(XS_ERR_INVALID_ARG, "xs_app_wait_sync: app is NULL or not an app");
    if (a->has_sync) XS_HIP_TRY(hipStreamWaitEvent((hipStream_t)hip_stream, a->sync_done, 0));
    return XS_OK;
}
