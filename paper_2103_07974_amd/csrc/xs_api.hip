// Host side of libxs.so: status strings, error text, bucket layout, plans, tuning,
// and the argument validation of the three data-moving entry points.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <atomic>
#include <new>
#include <vector>

#include "xs_internal.h"

namespace xs {

static thread_local char t_error[512] = "";

int fail(int status, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(t_error, sizeof t_error, fmt, ap);
    va_end(ap);
    return status;
}

int fail_hip(hipError_t e, const char *what)
{
    snprintf(t_error, sizeof t_error, "%s: %s", what, hipGetErrorString(e));
    return XS_ERR_HIP;
}

void clear_error() { t_error[0] = '\0'; }

int compute_units()
{
    // one cached value per device ordinal; a benign race writes the same number twice
    constexpr int kMaxDevices = 64;
    static int cached[kMaxDevices] = {};
    int dev = 0, cus = 0;
    XS_HIP_TRY(hipGetDevice(&dev));
    if (dev >= 0 && dev < kMaxDevices && cached[dev] > 0) return cached[dev];
    XS_HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    if (cus <= 0) return fail(XS_ERR_HIP, "device reports %d compute units", cus);
    if (dev >= 0 && dev < kMaxDevices) cached[dev] = cus;
    return cus;
}

// process-wide launch settings; -1 = chosen per gradient dtype at launch
static const int kTuningDefault[XS_TUNE_COUNT] = {/*reduce_wg_per_cu*/ 0, /*copy_wg_per_cu*/ 0,
                                                 /*nt_grads*/ 1, /*nt_state*/ 1,
                                                 /*reduce_lds_reserve*/ -1, /*reduce_max_wg*/ 0,
                                                 /*copy_max_wg*/ 0, /*copy_nt*/ 1,
                                                 /*gather_lds_reserve*/ -1, /*copy_lds_reserve*/ -1,
                                                 /*reduce_waves_per_wg*/ 1, /*reduce_small*/ 0,
                                                 /*copy_waves_per_wg*/ 1};
struct TuningRange {
    int lo, hi;
};
static const TuningRange kTuningRange[XS_TUNE_COUNT] = {
    {0, 64},          // XS_TUNE_REDUCE_WG_PER_CU
    {0, 4096},        // XS_TUNE_COPY_WG_PER_CU
    {0, 1},           // XS_TUNE_NT_GRADS
    {0, 1},           // XS_TUNE_NT_STATE
    {-1, 131072},     // XS_TUNE_REDUCE_LDS_RESERVE
    {0, 0x7fffffff},  // XS_TUNE_REDUCE_MAX_WG
    {0, 0x7fffffff},  // XS_TUNE_COPY_MAX_WG
    {0, 1},           // XS_TUNE_COPY_NT
    {-1, 131072},     // XS_TUNE_GATHER_LDS_RESERVE
    {-1, 131072},     // XS_TUNE_COPY_LDS_RESERVE
    {1, 4},           // XS_TUNE_REDUCE_WAVES_PER_WG (1, 2 or 4)
    {0, 1},           // XS_TUNE_REDUCE_SMALL
    {1, 4},           // XS_TUNE_COPY_WAVES_PER_WG (1, 2 or 4)
};
static std::atomic<int> g_tuning[XS_TUNE_COUNT] = {
    {kTuningDefault[0]}, {kTuningDefault[1]}, {kTuningDefault[2]}, {kTuningDefault[3]},
    {kTuningDefault[4]}, {kTuningDefault[5]}, {kTuningDefault[6]}, {kTuningDefault[7]},
    {kTuningDefault[8]}, {kTuningDefault[9]}, {kTuningDefault[10]}, {kTuningDefault[11]},
    {kTuningDefault[12]}};

static bool tuning_value_ok(int key, int value)
{
    if (value < kTuningRange[key].lo || value > kTuningRange[key].hi) return false;
    return (key != XS_TUNE_REDUCE_WAVES_PER_WG && key != XS_TUNE_COPY_WAVES_PER_WG) || value != 3;
}

Tuning tuning_now()
{
    Tuning t;
    for (int k = 0; k < XS_TUNE_COUNT; ++k) t.v[k] = g_tuning[k].load(std::memory_order_relaxed);
    return t;
}

int tuning_check(const int32_t *values, Tuning *out)
{
    for (int k = 0; k < XS_TUNE_COUNT; ++k) {
        if (!tuning_value_ok(k, values[k]))
            return fail(XS_ERR_INVALID_ARG, "launch setting %d = %d is outside [%d, %d]", k, values[k],
                        kTuningRange[k].lo, kTuningRange[k].hi);
        out->v[k] = values[k];
    }
    return XS_OK;
}

}  // namespace xs

using namespace xs;

extern "C" const char *xs_status_string(int status)
{
    switch (status) {
    case XS_OK: return "XS_OK";
    case XS_ERR_INVALID_ARG: return "XS_ERR_INVALID_ARG";
    case XS_ERR_ALIGNMENT: return "XS_ERR_ALIGNMENT";
    case XS_ERR_SIZE: return "XS_ERR_SIZE";
    case XS_ERR_UNSUPPORTED: return "XS_ERR_UNSUPPORTED";
    case XS_ERR_HIP: return "XS_ERR_HIP";
    case XS_ERR_NOMEM: return "XS_ERR_NOMEM";
    case XS_ERR_STATE: return "XS_ERR_STATE";
    default: return "XS_ERR_UNKNOWN";
    }
}

extern "C" const char *xs_last_error(void) { return t_error; }

extern "C" int xs_tuning_set(int key, int value)
{
    if (key < 0 || key >= XS_TUNE_COUNT)
        return fail(XS_ERR_INVALID_ARG, "xs_tuning_set: unknown key %d", key);
    if (!tuning_value_ok(key, value))
        return fail(XS_ERR_INVALID_ARG, "xs_tuning_set: value %d out of range [%d, %d] for key %d",
                    value, kTuningRange[key].lo, kTuningRange[key].hi, key);
    g_tuning[key].store(value, std::memory_order_relaxed);
    return XS_OK;
}

extern "C" int xs_tuning_get(int key, int *value_out)
{
    if (!value_out) return fail(XS_ERR_INVALID_ARG, "xs_tuning_get: value_out is NULL");
    if (key < 0 || key >= XS_TUNE_COUNT)
        return fail(XS_ERR_INVALID_ARG, "xs_tuning_get: unknown key %d", key);
    *value_out = g_tuning[key].load(std::memory_order_relaxed);
    return XS_OK;
}

// Launch settings for a synchronisation that shares the compute units with another task's
// kernels (Section 2.1).  MI355X: 160 KiB of LDS per compute unit; a reservation of 82 KiB
// admits exactly one synchronisation workgroup per compute unit and leaves 78 KiB to the other task.
extern "C" int xs_tuning_preset(int preset, int32_t *values_out)
{
    if (!values_out) return fail(XS_ERR_INVALID_ARG, "xs_tuning_preset: values_out is NULL");
    for (int k = 0; k < XS_TUNE_COUNT; ++k) values_out[k] = kTuningDefault[k];
    switch (preset) {
    case XS_PRESET_ALONE: return XS_OK;
    case XS_PRESET_BESIDE_COMPUTE:
        values_out[XS_TUNE_REDUCE_WAVES_PER_WG] = 4;
        values_out[XS_TUNE_REDUCE_LDS_RESERVE] = 82 * 1024;
        values_out[XS_TUNE_GATHER_LDS_RESERVE] = 82 * 1024;
        values_out[XS_TUNE_COPY_LDS_RESERVE] = 82 * 1024;
        values_out[XS_TUNE_REDUCE_SMALL] = 1;   // 28-47 registers per lane
        values_out[XS_TUNE_COPY_WAVES_PER_WG] = 4;
        return XS_OK;
    case XS_PRESET_LEAVE_WAVE_SLOTS:
        values_out[XS_TUNE_COPY_LDS_RESERVE] = 16 * 1024;
        return XS_OK;
    default: return fail(XS_ERR_INVALID_ARG, "xs_tuning_preset: unknown preset %d", preset);
    }
}

// Section 2.1, tensor fusion: tensors laid end to end, each start rounded up.
extern "C" int xs_bucket_layout(const uint64_t *numel, uint32_t n_tensors, uint64_t align_elems,
                                uint64_t *offsets_out)
{
    if (!offsets_out) return fail(XS_ERR_INVALID_ARG, "xs_bucket_layout: offsets_out is NULL");
    if (n_tensors > 0 && !numel) return fail(XS_ERR_INVALID_ARG, "xs_bucket_layout: numel is NULL");
    if (align_elems == 0) return fail(XS_ERR_INVALID_ARG, "xs_bucket_layout: align_elems is 0");
    uint64_t pos = 0;
    offsets_out[0] = 0;
    for (uint32_t t = 0; t < n_tensors; ++t) {
        if (numel[t] > UINT64_MAX - pos - align_elems)
            return fail(XS_ERR_SIZE, "xs_bucket_layout: bucket length overflows 64 bits");
        pos += numel[t];
        pos = (pos + align_elems - 1) / align_elems * align_elems;
        offsets_out[t + 1] = pos;
    }
    return XS_OK;
}

// One allocation for a task's flat buffers, each at a multiple of XS_POOL_ALIGN.
extern "C" int xs_pool_layout(const uint64_t *nbytes, uint32_t n_buffers, uint64_t *offsets_out)
{
    if (!offsets_out) return fail(XS_ERR_INVALID_ARG, "xs_pool_layout: offsets_out is NULL");
    if (n_buffers > 0 && !nbytes) return fail(XS_ERR_INVALID_ARG, "xs_pool_layout: nbytes is NULL");
    const uint64_t a = XS_POOL_ALIGN;
    uint64_t pos = 0;
    offsets_out[0] = 0;
    for (uint32_t i = 0; i < n_buffers; ++i) {
        if (nbytes[i] > UINT64_MAX - pos - a)
            return fail(XS_ERR_SIZE, "xs_pool_layout: pool size overflows 64 bits");
        pos = (pos + nbytes[i] + a - 1) / a * a;
        offsets_out[i + 1] = pos;
    }
    return XS_OK;
}

static int elem_size_of(int dtype)
{
    switch (dtype) {
    case XS_F32: return 4;
    case XS_F16: return 2;
    case XS_BF16: return 2;
    default: return 0;
    }
}

extern "C" int xs_plan_create(const uint64_t *numel, const uint64_t *offsets, uint32_t n_tensors,
                              int dtype, xs_plan **out)
{
    if (!out) return fail(XS_ERR_INVALID_ARG, "xs_plan_create: out is NULL");
    *out = nullptr;
    if (!offsets || (n_tensors > 0 && !numel))
        return fail(XS_ERR_INVALID_ARG, "xs_plan_create: numel/offsets is NULL");
    const int es = elem_size_of(dtype);
    if (es == 0) return fail(XS_ERR_UNSUPPORTED, "xs_plan_create: unknown dtype %d", dtype);
    if (offsets[0] != 0) return fail(XS_ERR_SIZE, "xs_plan_create: offsets[0] must be 0");
    if (n_tensors >= UINT32_MAX - 1) return fail(XS_ERR_SIZE, "xs_plan_create: too many tensors");

    xs_plan *p = nullptr;
    try {
        std::vector<uint32_t> prefix(n_tensors + 1, 0);
        uint64_t chunks = 0;
        for (uint32_t t = 0; t < n_tensors; ++t) {
            if (offsets[t + 1] < offsets[t] || numel[t] > offsets[t + 1] - offsets[t])
                return fail(XS_ERR_SIZE,
                            "xs_plan_create: tensor %u (numel %llu at offset %llu) overruns the next offset %llu",
                            t, (unsigned long long)numel[t], (unsigned long long)offsets[t],
                            (unsigned long long)offsets[t + 1]);
            if (offsets[t + 1] > (UINT64_MAX >> 4))
                return fail(XS_ERR_SIZE, "xs_plan_create: bucket too large");
            const uint64_t seg_bytes = (offsets[t + 1] - offsets[t]) * (uint64_t)es;
            prefix[t] = (uint32_t)chunks;
            chunks += (seg_bytes + kChunkBytes - 1) / kChunkBytes;
            if (chunks > 0x7fffffffull) return fail(XS_ERR_SIZE, "xs_plan_create: bucket too large");
        }
        prefix[n_tensors] = (uint32_t)chunks;

        p = new (std::nothrow) xs_plan();
        if (!p) return fail(XS_ERR_NOMEM, "xs_plan_create: host allocation failed");
        p->magic = XS_PLAN_MAGIC;
        p->n_tensors = n_tensors;
        p->dtype = dtype;
        p->elem_size = (uint32_t)es;
        p->bucket_elems = offsets[n_tensors];
        p->n_chunks = (uint32_t)chunks;
        p->dev_blob = nullptr;

        // rows of kRowBytes of this dtype: which tensor's segment holds each row's first element
        const uint64_t row_elems = kRowBytes / (uint64_t)es;
        const uint64_t n_rows = (offsets[n_tensors] + row_elems - 1) / row_elems;
        if (n_rows > 0x7fffffffull) { delete p; return fail(XS_ERR_SIZE, "xs_plan_create: bucket too large"); }
        p->n_rows = n_rows;
        std::vector<uint32_t> row_first((size_t)n_rows, 0);
        {
            uint32_t t = 0;
            for (uint64_t r = 0; r < n_rows; ++r) {
                const uint64_t j = r * row_elems;
                while (t + 1 < n_tensors && offsets[t + 1] <= j) ++t;
                row_first[(size_t)r] = t;
            }
        }

        // one device blob: offsets | numel | chunk_prefix | row_first
        const size_t off_bytes = (size_t)(n_tensors + 1) * 8;
        const size_t num_bytes = (size_t)n_tensors * 8;
        const size_t pre_bytes = (size_t)(n_tensors + 1) * 4;
        const size_t row_bytes = (size_t)n_rows * 4;
        std::vector<unsigned char> host(off_bytes + num_bytes + pre_bytes + row_bytes);
        memcpy(host.data(), offsets, off_bytes);
        if (n_tensors) memcpy(host.data() + off_bytes, numel, num_bytes);
        memcpy(host.data() + off_bytes + num_bytes, prefix.data(), pre_bytes);
        if (n_rows) memcpy(host.data() + off_bytes + num_bytes + pre_bytes, row_first.data(), row_bytes);
        hipError_t e = hipMalloc(&p->dev_blob, host.size());
        if (e != hipSuccess) {
            delete p;
            fail_hip(e, "hipMalloc(plan tables)");
            return e == hipErrorOutOfMemory ? XS_ERR_NOMEM : XS_ERR_HIP;
        }
        e = hipMemcpy(p->dev_blob, host.data(), host.size(), hipMemcpyHostToDevice);
        if (e != hipSuccess) {
            (void)hipFree(p->dev_blob);
            delete p;
            return fail_hip(e, "hipMemcpy(plan tables)");
        }
        unsigned char *d = (unsigned char *)p->dev_blob;
        p->tables.offsets = (const uint64_t *)d;
        p->tables.numel = (const uint64_t *)(d + off_bytes);
        p->tables.chunk_prefix = (const uint32_t *)(d + off_bytes + num_bytes);
        p->tables.row_first = (const uint32_t *)(d + off_bytes + num_bytes + pre_bytes);
        *out = p;
        return XS_OK;
    } catch (const std::bad_alloc &) {      // the host-side tables (one word per KiB of bucket)
        delete p;
        return fail(XS_ERR_NOMEM, "xs_plan_create: host allocation failed");
    }
}

extern "C" int xs_plan_destroy(xs_plan *plan)
{
    if (!plan) return XS_OK;
    if (plan->magic != XS_PLAN_MAGIC) return fail(XS_ERR_INVALID_ARG, "xs_plan_destroy: not a plan");
    plan->magic = 0;
    hipError_t e = plan->dev_blob ? hipFree(plan->dev_blob) : hipSuccess;
    delete plan;
    if (e != hipSuccess) return fail_hip(e, "hipFree(plan tables)");
    return XS_OK;
}

extern "C" uint64_t xs_plan_bucket_elems(const xs_plan *plan)
{
    return (plan && plan->magic == XS_PLAN_MAGIC) ? plan->bucket_elems : 0;
}

extern "C" uint32_t xs_plan_n_tensors(const xs_plan *plan)
{
    return (plan && plan->magic == XS_PLAN_MAGIC) ? plan->n_tensors : 0;
}

// ---- Algorithm 1, "Fuse all gradient into one group" -----------------------------
extern "C" int xs_fuse_pack(const xs_plan *plan, const void *const *tensor_ptrs, void *bucket,
                            int32_t *found_inf, void *hip_stream)
{
    if (!plan || plan->magic != XS_PLAN_MAGIC)
        return fail(XS_ERR_INVALID_ARG, "xs_fuse_pack: plan is NULL or not a plan");
    if (plan->n_chunks == 0) return XS_OK;
    if (!bucket) return fail(XS_ERR_INVALID_ARG, "xs_fuse_pack: bucket is NULL");
    if (!tensor_ptrs) return fail(XS_ERR_INVALID_ARG, "xs_fuse_pack: tensor_ptrs is NULL");
    if (!aligned16(bucket)) return fail(XS_ERR_ALIGNMENT, "xs_fuse_pack: bucket is not 16-byte aligned");
    if (found_inf && ((uintptr_t)found_inf & 3u))
        return fail(XS_ERR_ALIGNMENT, "xs_fuse_pack: found_inf is not 4-byte aligned");
    const void *table = tensor_ptrs;
    return launch_pack(tuning_now(), plan, &table, &bucket, 1, found_inf, (hipStream_t)hip_stream);
}

// The W workers' packs of one synchronisation in a single launch.
int xs::fuse_pack_many_impl(const Tuning &tn, const xs_plan *plan,
                            const void *const *const *tensor_ptr_tables, void *const *buckets,
                            uint32_t n, int32_t *found_inf, hipStream_t stream)
{
    if (!plan || plan->magic != XS_PLAN_MAGIC)
        return fail(XS_ERR_INVALID_ARG, "xs_fuse_pack_many: plan is NULL or not a plan");
    if (n > XS_MAX_REPLICAS)
        return fail(XS_ERR_INVALID_ARG, "xs_fuse_pack_many: n = %u exceeds %d", n, XS_MAX_REPLICAS);
    if (n == 0 || plan->n_chunks == 0) return XS_OK;
    if (!tensor_ptr_tables || !buckets)
        return fail(XS_ERR_INVALID_ARG, "xs_fuse_pack_many: tensor_ptr_tables/buckets is NULL");
    if (found_inf && ((uintptr_t)found_inf & 3u))
        return fail(XS_ERR_ALIGNMENT, "xs_fuse_pack_many: found_inf is not 4-byte aligned");
    for (uint32_t i = 0; i < n; ++i) {
        if (!tensor_ptr_tables[i] || !buckets[i])
            return fail(XS_ERR_INVALID_ARG, "xs_fuse_pack_many: entry %u is NULL", i);
        if (!aligned16(buckets[i]))
            return fail(XS_ERR_ALIGNMENT, "xs_fuse_pack_many: buckets[%u] is not 16-byte aligned", i);
    }
    return launch_pack(tn, plan, (const void *const *)tensor_ptr_tables, buckets, n, found_inf, stream);
}

extern "C" int xs_fuse_pack_many(const xs_plan *plan, const void *const *const *tensor_ptr_tables,
                                 void *const *buckets, uint32_t n, int32_t *found_inf,
                                 void *hip_stream)
{
    return fuse_pack_many_impl(tuning_now(), plan, tensor_ptr_tables, buckets, n, found_inf,
                               (hipStream_t)hip_stream);
}

int xs::fuse_unpack_impl(const Tuning &tn, const xs_plan *plan, const void *bucket,
                         void *const *tensor_ptrs, hipStream_t stream)
{
    if (!plan || plan->magic != XS_PLAN_MAGIC)
        return fail(XS_ERR_INVALID_ARG, "xs_fuse_unpack: plan is NULL or not a plan");
    if (plan->n_chunks == 0) return XS_OK;
    if (!bucket) return fail(XS_ERR_INVALID_ARG, "xs_fuse_unpack: bucket is NULL");
    if (!tensor_ptrs) return fail(XS_ERR_INVALID_ARG, "xs_fuse_unpack: tensor_ptrs is NULL");
    if (!aligned16(bucket)) return fail(XS_ERR_ALIGNMENT, "xs_fuse_unpack: bucket is not 16-byte aligned");
    return launch_unpack(tn, plan, bucket, tensor_ptrs, stream);
}

extern "C" int xs_fuse_unpack(const xs_plan *plan, const void *bucket, void *const *tensor_ptrs,
                              void *hip_stream)
{
    return fuse_unpack_impl(tuning_now(), plan, bucket, tensor_ptrs, (hipStream_t)hip_stream);
}

// ---- Algorithm 1, "Receive averaged gradients" + "Model Update" ----------------------
static bool overlaps(const void *a, uint64_t a_bytes, const void *b, uint64_t b_bytes)
{
    const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a0 < b0 + b_bytes && b0 < a0 + a_bytes;
}

static bool is_half_dtype(int dtype) { return dtype == XS_F16 || dtype == XS_BF16; }

// plan + tensor_hp: per-tensor records (both NULL for the single-triple entry points)
int xs::reduce_sgd_impl(const Tuning &tn, const xs_plan *plan, const xs_tensor_hparams *tensor_hp,
                        const void *const *replica_buckets, uint32_t W, int grad_dtype,
                        uint64_t n_elems, float *params, float *momentum,
                        float *params_out, float *momentum_out,
                        const xs_sgd_hparams *hp, int32_t *found_inf,
                        const xs_mp_options *mp, void *const *param_tensor_ptrs, hipStream_t stream)
{
    void *model_copy = mp ? mp->model_copy : nullptr;
    const int view_dtype = (mp && param_tensor_ptrs) ? mp->view_dtype : XS_F32;
    if (view_dtype != XS_F32 && !is_half_dtype(view_dtype))
        return fail(XS_ERR_UNSUPPORTED, "xs_fused_reduce_sgd: unknown view_dtype %d", view_dtype);
    if (param_tensor_ptrs && (!plan || params_out || momentum_out))
        return fail(XS_ERR_UNSUPPORTED,
                    "xs_fused_reduce_sgd: parameter views are written by the in-place form only");
    const int model_copy_dtype = mp ? mp->model_copy_dtype : XS_F16;
    if (model_copy && !is_half_dtype(model_copy_dtype))
        return fail(XS_ERR_UNSUPPORTED, "xs_fused_reduce_sgd: model_copy_dtype %d is not XS_F16 or XS_BF16",
                    model_copy_dtype);
    if (model_copy && !aligned16(model_copy))
        return fail(XS_ERR_ALIGNMENT, "xs_fused_reduce_sgd: model_copy is not 16-byte aligned");
    const int es = elem_size_of(grad_dtype);
    if (es == 0) return fail(XS_ERR_UNSUPPORTED, "xs_fused_reduce_sgd: unknown grad_dtype %d", grad_dtype);
    if (W == 0 || W > XS_MAX_REPLICAS)
        return fail(XS_ERR_INVALID_ARG, "xs_fused_reduce_sgd: W = %u outside [1, %d]", W, XS_MAX_REPLICAS);
    if (!hp) return fail(XS_ERR_INVALID_ARG, "xs_fused_reduce_sgd: hp is NULL");
    if ((params_out == nullptr) != (momentum_out == nullptr))
        return fail(XS_ERR_INVALID_ARG,
                    "xs_fused_reduce_sgd: params_out and momentum_out must both be NULL or both be given");
    if (n_elems == 0) return XS_OK;
    if (n_elems > (UINT64_MAX >> 4)) return fail(XS_ERR_SIZE, "xs_fused_reduce_sgd: n_elems too large");
    if (!replica_buckets || !params || !momentum)
        return fail(XS_ERR_INVALID_ARG, "xs_fused_reduce_sgd: replica_buckets/params/momentum is NULL");
    const bool out_of_place = params_out != nullptr;
    if (model_copy && out_of_place && found_inf)
        return fail(XS_ERR_UNSUPPORTED,
                    "xs_fused_reduce_sgd: model_copy cannot be written by a pass that is still deciding "
                    "whether the step is skipped (out-of-place outputs with found_inf)");
    if (!aligned16(params) || !aligned16(momentum) ||
        (out_of_place && (!aligned16(params_out) || !aligned16(momentum_out))))
        return fail(XS_ERR_ALIGNMENT, "xs_fused_reduce_sgd: params/momentum pointers must be 16-byte aligned");
    if (found_inf && ((uintptr_t)found_inf & 3u))
        return fail(XS_ERR_ALIGNMENT, "xs_fused_reduce_sgd: found_inf is not 4-byte aligned");
    const uint64_t sbytes = n_elems * 4, gbytes = n_elems * (uint64_t)es;
    const void *state[4] = {params, momentum, params_out, momentum_out};
    const int n_state = out_of_place ? 4 : 2;
    for (int a = 0; a < n_state; ++a)
        for (int b = a + 1; b < n_state; ++b)
            if (overlaps(state[a], sbytes, state[b], sbytes))
                return fail(XS_ERR_INVALID_ARG, "xs_fused_reduce_sgd: params/momentum buffers overlap");
    for (uint32_t w = 0; w < W; ++w) {
        if (!replica_buckets[w])
            return fail(XS_ERR_INVALID_ARG, "xs_fused_reduce_sgd: replica_buckets[%u] is NULL", w);
        if (!aligned16(replica_buckets[w]))
            return fail(XS_ERR_ALIGNMENT, "xs_fused_reduce_sgd: replica_buckets[%u] is not 16-byte aligned", w);
        for (int a = 0; a < n_state; ++a)
            if (overlaps(replica_buckets[w], gbytes, state[a], sbytes))
                return fail(XS_ERR_INVALID_ARG,
                            "xs_fused_reduce_sgd: replica_buckets[%u] overlaps a parameter/momentum buffer", w);
    }
    if (model_copy) {
        for (int a = 0; a < n_state; ++a)
            if (overlaps(model_copy, n_elems * 2, state[a], sbytes))
                return fail(XS_ERR_INVALID_ARG, "xs_fused_reduce_sgd: model_copy overlaps a parameter/momentum buffer");
        for (uint32_t w = 0; w < W; ++w)
            if (overlaps(model_copy, n_elems * 2, replica_buckets[w], gbytes))
                return fail(XS_ERR_INVALID_ARG, "xs_fused_reduce_sgd: model_copy overlaps replica_buckets[%u]", w);
    }
    if (tensor_hp) {
        const uint64_t hbytes = (uint64_t)plan->n_tensors * sizeof(xs_tensor_hparams);
        for (int a = (out_of_place ? 2 : 0); a < n_state; ++a)
            if (overlaps(tensor_hp, hbytes, state[a], sbytes))
                return fail(XS_ERR_INVALID_ARG, "xs_fused_reduce_sgd_pt: tensor_hp overlaps an output buffer");
    }
    return launch_reduce_sgd(tn, replica_buckets, W, grad_dtype, n_elems, params, momentum,
                             out_of_place ? params_out : params,
                             out_of_place ? momentum_out : momentum, *hp, found_inf,
                             /*detect=*/out_of_place && found_inf != nullptr, model_copy,
                             model_copy_dtype, (tensor_hp || param_tensor_ptrs) ? plan : nullptr, tensor_hp,
                             param_tensor_ptrs, view_dtype, stream);
}

extern "C" int xs_fused_reduce_sgd_mp(const void *const *replica_buckets, uint32_t W, int grad_dtype,
                                      uint64_t n_elems, float *params, float *momentum,
                                      float *params_out, float *momentum_out,
                                      const xs_sgd_hparams *hp, int32_t *found_inf,
                                      const xs_mp_options *mp, void *hip_stream)
{
    return reduce_sgd_impl(tuning_now(), nullptr, nullptr, replica_buckets, W, grad_dtype, n_elems,
                           params, momentum, params_out, momentum_out, hp, found_inf, mp, nullptr,
                           (hipStream_t)hip_stream);
}

// One (lr, momentum, weight decay) record per tensor of the plan the buckets were packed with.
int xs::reduce_sgd_pt_impl(const Tuning &tn, const xs_plan *gradient_plan,
                           const void *const *replica_buckets, uint32_t W, float *params,
                           float *momentum, float *params_out, float *momentum_out,
                           const xs_tensor_hparams *tensor_hp, float inv_loss_scale,
                           int32_t *found_inf, const xs_mp_options *mp, hipStream_t stream)
{
    if (!gradient_plan || gradient_plan->magic != XS_PLAN_MAGIC)
        return fail(XS_ERR_INVALID_ARG, "xs_fused_reduce_sgd_pt: plan is NULL or not a plan");
    if (gradient_plan->bucket_elems == 0) return XS_OK;
    if (!tensor_hp) return fail(XS_ERR_INVALID_ARG, "xs_fused_reduce_sgd_pt: tensor_hp is NULL");
    if (!aligned16(tensor_hp))
        return fail(XS_ERR_ALIGNMENT, "xs_fused_reduce_sgd_pt: tensor_hp is not 16-byte aligned");
    const xs_sgd_hparams hp = {0.f, 0.f, 0.f, inv_loss_scale};
    return reduce_sgd_impl(tn, gradient_plan, tensor_hp, replica_buckets, W, gradient_plan->dtype,
                           gradient_plan->bucket_elems, params, momentum, params_out,
                           momentum_out, &hp, found_inf, mp, nullptr, stream);
}

// "Receive averaged gradients" + "Model Update" + the way back to the per-layer tensors, one pass.
int xs::reduce_sgd_unpack_impl(const Tuning &tn, const xs_plan *gradient_plan,
                               const void *const *replica_buckets, uint32_t W, float *params,
                               float *momentum, void *const *param_tensor_ptrs,
                               const xs_sgd_hparams *hp, const xs_tensor_hparams *tensor_hp,
                               int32_t *found_inf, const xs_mp_options *mp, hipStream_t stream)
{
    if (!gradient_plan || gradient_plan->magic != XS_PLAN_MAGIC)
        return fail(XS_ERR_INVALID_ARG, "xs_fused_reduce_sgd_unpack: plan is NULL or not a plan");
    if (!hp) return fail(XS_ERR_INVALID_ARG, "xs_fused_reduce_sgd_unpack: hp is NULL");
    if (gradient_plan->bucket_elems == 0) return XS_OK;
    if (!param_tensor_ptrs)
        return fail(XS_ERR_INVALID_ARG, "xs_fused_reduce_sgd_unpack: param_tensor_ptrs is NULL");
    if (tensor_hp && !aligned16(tensor_hp))
        return fail(XS_ERR_ALIGNMENT, "xs_fused_reduce_sgd_unpack: tensor_hp is not 16-byte aligned");
    return reduce_sgd_impl(tn, gradient_plan, tensor_hp, replica_buckets, W, gradient_plan->dtype,
                           gradient_plan->bucket_elems, params, momentum, nullptr, nullptr, hp,
                           found_inf, mp, param_tensor_ptrs, stream);
}

extern "C" int xs_fused_reduce_sgd_unpack(const xs_plan *gradient_plan, const void *const *replica_buckets,
                                          uint32_t W, float *params, float *momentum,
                                          void *const *param_tensor_ptrs, const xs_sgd_hparams *hp,
                                          const xs_tensor_hparams *tensor_hp, int32_t *found_inf,
                                          const xs_mp_options *mp, void *hip_stream)
{
    return reduce_sgd_unpack_impl(tuning_now(), gradient_plan, replica_buckets, W, params, momentum,
                                  param_tensor_ptrs, hp, tensor_hp, found_inf, mp,
                                  (hipStream_t)hip_stream);
}

extern "C" int xs_fused_reduce_sgd_pt(const xs_plan *gradient_plan, const void *const *replica_buckets,
                                      uint32_t W, float *params, float *momentum,
                                      float *params_out, float *momentum_out,
                                      const xs_tensor_hparams *tensor_hp, float inv_loss_scale,
                                      int32_t *found_inf, const xs_mp_options *mp, void *hip_stream)
{
    return reduce_sgd_pt_impl(tuning_now(), gradient_plan, replica_buckets, W, params, momentum,
                              params_out, momentum_out, tensor_hp, inv_loss_scale, found_inf, mp,
                              (hipStream_t)hip_stream);
}

extern "C" int xs_fused_reduce_sgd(const void *const *replica_buckets, uint32_t W, int grad_dtype,
                                   uint64_t n_elems, float *params, float *momentum,
                                   float *params_out, float *momentum_out,
                                   const xs_sgd_hparams *hp, int32_t *found_inf, void *hip_stream)
{
    return xs_fused_reduce_sgd_mp(replica_buckets, W, grad_dtype, n_elems, params, momentum,
                                  params_out, momentum_out, hp, found_inf, nullptr, hip_stream);
}

// ---- the same pass reading the per-layer gradient tensors directly ----------------------
int xs::gather_reduce_sgd_impl(const Tuning &tn, const xs_plan *gradient_plan,
                               const void *const *grad_ptrs, uint32_t W, float *params,
                               float *momentum, float *params_out, float *momentum_out,
                               void *const *param_tensor_ptrs, const xs_sgd_hparams *hp,
                               const xs_tensor_hparams *tensor_hp, int32_t *found_inf,
                               const xs_mp_options *mp, hipStream_t stream)
{
    const int view_dtype = mp ? mp->view_dtype : XS_F32;
    if (view_dtype != XS_F32 && !is_half_dtype(view_dtype))
        return fail(XS_ERR_UNSUPPORTED, "xs_fused_gather_reduce_sgd: unknown view_dtype %d", view_dtype);
    if (mp && mp->model_copy)
        return fail(XS_ERR_UNSUPPORTED,
                    "xs_fused_gather_reduce_sgd: model_copy is not available in the gathering form; "
                    "use half-precision parameter views (view_dtype)");
    if (!gradient_plan || gradient_plan->magic != XS_PLAN_MAGIC)
        return fail(XS_ERR_INVALID_ARG, "xs_fused_gather_reduce_sgd: plan is NULL or not a plan");
    if (W == 0 || W > XS_MAX_REPLICAS)
        return fail(XS_ERR_INVALID_ARG, "xs_fused_gather_reduce_sgd: W = %u outside [1, %d]", W, XS_MAX_REPLICAS);
    if (!hp) return fail(XS_ERR_INVALID_ARG, "xs_fused_gather_reduce_sgd: hp is NULL");
    if ((params_out == nullptr) != (momentum_out == nullptr))
        return fail(XS_ERR_INVALID_ARG,
                    "xs_fused_gather_reduce_sgd: params_out and momentum_out must both be NULL or both be given");
    const uint64_t n = gradient_plan->bucket_elems;
    if (n == 0) return XS_OK;
    if (!grad_ptrs || !params || !momentum)
        return fail(XS_ERR_INVALID_ARG, "xs_fused_gather_reduce_sgd: grad_ptrs/params/momentum is NULL");
    const bool out_of_place = params_out != nullptr;
    if (!aligned16(params) || !aligned16(momentum) ||
        (out_of_place && (!aligned16(params_out) || !aligned16(momentum_out))))
        return fail(XS_ERR_ALIGNMENT,
                    "xs_fused_gather_reduce_sgd: params/momentum pointers must be 16-byte aligned");
    if (found_inf && ((uintptr_t)found_inf & 3u))
        return fail(XS_ERR_ALIGNMENT, "xs_fused_gather_reduce_sgd: found_inf is not 4-byte aligned");
    const bool detect = out_of_place && found_inf != nullptr;
    if (detect && param_tensor_ptrs)
        return fail(XS_ERR_UNSUPPORTED,
                    "xs_fused_gather_reduce_sgd: parameter views cannot be written in a pass that is "
                    "still deciding whether the step is skipped");
    const uint64_t sbytes = n * 4;
    const void *state[4] = {params, momentum, params_out, momentum_out};
    const int n_state = out_of_place ? 4 : 2;
    for (int a = 0; a < n_state; ++a)
        for (int b = a + 1; b < n_state; ++b)
            if (overlaps(state[a], sbytes, state[b], sbytes))
                return fail(XS_ERR_INVALID_ARG, "xs_fused_gather_reduce_sgd: params/momentum buffers overlap");
    if (tensor_hp) {
        if (!aligned16(tensor_hp))
            return fail(XS_ERR_ALIGNMENT, "xs_fused_gather_reduce_sgd_pt: tensor_hp is not 16-byte aligned");
        const uint64_t hbytes = (uint64_t)gradient_plan->n_tensors * sizeof(xs_tensor_hparams);
        for (int a = (out_of_place ? 2 : 0); a < n_state; ++a)
            if (overlaps(tensor_hp, hbytes, state[a], sbytes))
                return fail(XS_ERR_INVALID_ARG, "xs_fused_gather_reduce_sgd_pt: tensor_hp overlaps an output buffer");
    }
    return launch_gather_reduce_sgd(tn, gradient_plan, grad_ptrs, W, params, momentum,
                                    out_of_place ? params_out : params,
                                    out_of_place ? momentum_out : momentum, param_tensor_ptrs,
                                    view_dtype, *hp, tensor_hp, found_inf, detect, stream);
}

extern "C" int xs_fused_gather_reduce_sgd_mp(const xs_plan *gradient_plan, const void *const *grad_ptrs,
                                             uint32_t W, float *params, float *momentum,
                                             float *params_out, float *momentum_out,
                                             void *const *param_tensor_ptrs, const xs_sgd_hparams *hp,
                                             int32_t *found_inf, const xs_mp_options *mp,
                                             void *hip_stream)
{
    return gather_reduce_sgd_impl(tuning_now(), gradient_plan, grad_ptrs, W, params, momentum,
                                  params_out, momentum_out, param_tensor_ptrs, hp, nullptr, found_inf,
                                  mp, (hipStream_t)hip_stream);
}

extern "C" int xs_fused_gather_reduce_sgd_pt(const xs_plan *gradient_plan, const void *const *grad_ptrs,
                                             uint32_t W, float *params, float *momentum,
                                             float *params_out, float *momentum_out,
                                             void *const *param_tensor_ptrs,
                                             const xs_tensor_hparams *tensor_hp, float inv_loss_scale,
                                             int32_t *found_inf, const xs_mp_options *mp,
                                             void *hip_stream)
{
    if (gradient_plan && gradient_plan->magic == XS_PLAN_MAGIC && gradient_plan->bucket_elems != 0 &&
        !tensor_hp)
        return fail(XS_ERR_INVALID_ARG, "xs_fused_gather_reduce_sgd_pt: tensor_hp is NULL");
    const xs_sgd_hparams hp = {0.f, 0.f, 0.f, inv_loss_scale};
    return gather_reduce_sgd_impl(tuning_now(), gradient_plan, grad_ptrs, W, params, momentum,
                                  params_out, momentum_out, param_tensor_ptrs, &hp, tensor_hp,
                                  found_inf, mp, (hipStream_t)hip_stream);
}

extern "C" int xs_fused_gather_reduce_sgd(const xs_plan *gradient_plan, const void *const *grad_ptrs,
                                          uint32_t W, float *params, float *momentum,
                                          float *params_out, float *momentum_out,
                                          void *const *param_tensor_ptrs, const xs_sgd_hparams *hp,
                                          int32_t *found_inf, void *hip_stream)
{
    return xs_fused_gather_reduce_sgd_mp(gradient_plan, grad_ptrs, W, params, momentum, params_out,
                                         momentum_out, param_tensor_ptrs, hp, found_inf, nullptr,
                                         hip_stream);
}
