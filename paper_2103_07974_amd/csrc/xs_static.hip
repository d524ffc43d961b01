// xs_fuse_pack_static: the pack of xs_fuse_pack for callers that cannot allocate device
// memory (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).
//
// xs_fuse_pack reads the tensor list's layout from device tables that xs_plan_create
// allocates.  Here the same tables live in one fixed device array of the library, `scratch`,
// and are rewritten on the caller's stream in front of every pack by small kernels that
// receive the table entries through their kernel arguments (no host-to-device copy, no
// allocation, nothing that a capture could not record).  The pack itself is the chunk-form
// copy kernel of xs_copy.hip, whose tables are O(tensors) and fit the array; the result is
// bit-identical to xs_fuse_pack's.
//
// Every call on a GPU shares that GPU's array: the array keeps the last call's tables, each
// call overwrites the part it uses, and two calls that overlap in time on one GPU (different
// streams, or different threads) race on it.
#include <atomic>

#include "xs_device.h"
#include "xs_internal.h"

namespace xs {

constexpr uint32_t kStaticMaxTensors = XS_STATIC_MAX_TENSORS;
// offsets[kStaticMaxTensors + 1] | numel[kStaticMaxTensors] | chunk_prefix[kStaticMaxTensors + 1]
constexpr size_t kOffBytes = (size_t)(kStaticMaxTensors + 1) * 8;
constexpr size_t kNumBytes = (size_t)kStaticMaxTensors * 8;
constexpr size_t kPreBytes = (size_t)(kStaticMaxTensors + 1) * 4;
constexpr size_t kScratchBytes = (kOffBytes + kNumBytes + kPreBytes + 255) / 256 * 256;

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// `scratch` names the array in device code only; host code uses the address that
// hipGetSymbolAddress returns for the current device (each GPU has its own copy).
constexpr int kMaxDevices = 64;
static std::atomic<unsigned char *> g_scratch_ptr[kMaxDevices];

static int scratch_for_current_device(unsigned char **out)
{
    int dev = 0;
    XS_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(XS_ERR_UNSUPPORTED, "xs_fuse_pack_static: device ordinal %d", dev);
    unsigned char *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        void *sym = nullptr;
        XS_HIP_TRY(hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)));
        if (!sym) return fail(XS_ERR_HIP, "xs_fuse_pack_static: hipGetSymbolAddress returned NULL");
        p = (unsigned char *)sym;
        g_scratch_ptr[dev].store(p, std::memory_order_release);   // every thread resolves the same address
    }
    *out = p;
    return XS_OK;
}

constexpr uint32_t kBatch = 128;   // table entries per writer launch (2.6 KB of kernel arguments)
struct TableBatch {
    uint64_t offsets[kBatch];
    uint64_t numel[kBatch];
    uint32_t prefix[kBatch];
    uint32_t first, count;
    uint32_t n_tensors;       // the last batch also writes offsets[n_tensors], chunk_prefix[n_tensors]
    uint32_t end_prefix;
    uint64_t end_offset;
    uint32_t is_last;
};

__global__ __launch_bounds__(kBatch) void table_write_kernel(unsigned char *tables, TableBatch b)
{
    uint64_t *offsets = (uint64_t *)tables;
    uint64_t *numel = (uint64_t *)(tables + kOffBytes);
    uint32_t *prefix = (uint32_t *)(tables + kOffBytes + kNumBytes);
    const uint32_t i = threadIdx.x;
    if (i < b.count) {
        offsets[b.first + i] = b.offsets[i];
        numel[b.first + i] = b.numel[i];
        prefix[b.first + i] = b.prefix[i];
    }
    if (b.is_last && i == 0) {
        offsets[b.n_tensors] = b.end_offset;
        prefix[b.n_tensors] = b.end_prefix;
    }
}

}  // namespace xs

using namespace xs;

extern "C" int xs_fuse_pack_static(const uint64_t *numel, const uint64_t *offsets, uint32_t n_tensors,
                                   int dtype, const void *const *tensor_ptrs, void *bucket,
                                   int32_t *found_inf, void *hip_stream)
{
    if (n_tensors > kStaticMaxTensors)
        return fail(XS_ERR_SIZE, "xs_fuse_pack_static: %u tensors exceed the limit of %u (XS_STATIC_MAX_TENSORS); "
                                 "use xs_plan_create + xs_fuse_pack",
                    n_tensors, kStaticMaxTensors);
    if (!offsets || (n_tensors > 0 && !numel))
        return fail(XS_ERR_INVALID_ARG, "xs_fuse_pack_static: numel/offsets is NULL");
    const int es = dtype == XS_F32 ? 4 : (dtype == XS_F16 || dtype == XS_BF16) ? 2 : 0;
    if (es == 0) return fail(XS_ERR_UNSUPPORTED, "xs_fuse_pack_static: unknown dtype %d", dtype);
    if (offsets[0] != 0) return fail(XS_ERR_SIZE, "xs_fuse_pack_static: offsets[0] must be 0");

    // the chunk-count prefix of xs_plan_create, on the stack
    uint32_t prefix[kStaticMaxTensors + 1];
    uint64_t chunks = 0;
    for (uint32_t t = 0; t < n_tensors; ++t) {
        if (offsets[t + 1] < offsets[t] || numel[t] > offsets[t + 1] - offsets[t])
            return fail(XS_ERR_SIZE, "xs_fuse_pack_static: tensor %u (numel %llu at offset %llu) overruns the next offset %llu",
                        t, (unsigned long long)numel[t], (unsigned long long)offsets[t],
                        (unsigned long long)offsets[t + 1]);
        if (offsets[t + 1] > (UINT64_MAX >> 4)) return fail(XS_ERR_SIZE, "xs_fuse_pack_static: bucket too large");
        prefix[t] = (uint32_t)chunks;
        chunks += ((offsets[t + 1] - offsets[t]) * (uint64_t)es + kChunkBytes - 1) / kChunkBytes;
        if (chunks > 0x7fffffffull) return fail(XS_ERR_SIZE, "xs_fuse_pack_static: bucket too large");
    }
    prefix[n_tensors] = (uint32_t)chunks;
    if (chunks == 0) return XS_OK;
    if (!bucket) return fail(XS_ERR_INVALID_ARG, "xs_fuse_pack_static: bucket is NULL");
    if (!tensor_ptrs) return fail(XS_ERR_INVALID_ARG, "xs_fuse_pack_static: tensor_ptrs is NULL");
    if (!aligned16(bucket)) return fail(XS_ERR_ALIGNMENT, "xs_fuse_pack_static: bucket is not 16-byte aligned");
    if (found_inf && ((uintptr_t)found_inf & 3u))
        return fail(XS_ERR_ALIGNMENT, "xs_fuse_pack_static: found_inf is not 4-byte aligned");

    unsigned char *tables = nullptr;
    int rc = scratch_for_current_device(&tables);
    if (rc != XS_OK) return rc;
    hipStream_t stream = (hipStream_t)hip_stream;

    for (uint32_t first = 0; first < n_tensors; first += kBatch) {
        TableBatch b;
        b.first = first;
        b.count = n_tensors - first < kBatch ? n_tensors - first : kBatch;
        for (uint32_t i = 0; i < b.count; ++i) {
            b.offsets[i] = offsets[first + i];
            b.numel[i] = numel[first + i];
            b.prefix[i] = prefix[first + i];
        }
        b.n_tensors = n_tensors;
        b.end_prefix = prefix[n_tensors];
        b.end_offset = offsets[n_tensors];
        b.is_last = first + kBatch >= n_tensors;
        hipLaunchKernelGGL(table_write_kernel, dim3(1), dim3(kBatch), 0, stream, tables, b);
        XS_HIP_TRY(hipGetLastError());
    }

    xs_plan plan = {};
    plan.magic = XS_PLAN_MAGIC;
    plan.n_tensors = n_tensors;
    plan.dtype = dtype;
    plan.elem_size = (uint32_t)es;
    plan.bucket_elems = offsets[n_tensors];
    plan.n_chunks = (uint32_t)chunks;
    plan.n_rows = 0;
    plan.dev_blob = nullptr;
    plan.tables.offsets = (const uint64_t *)tables;
    plan.tables.numel = (const uint64_t *)(tables + kOffBytes);
    plan.tables.chunk_prefix = (const uint32_t *)(tables + kOffBytes + kNumBytes);
    plan.tables.row_first = nullptr;   // pack does not read it
    const void *table = tensor_ptrs;
    return launch_pack(tuning_now(), &plan, &table, &bucket, 1, found_inf, stream);
}
