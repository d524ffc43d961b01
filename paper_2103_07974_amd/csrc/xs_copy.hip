// Pack / unpack between a list of per-layer tensors and one fused bucket on gfx950
// (arXiv 2103.07974, Section 2.1 tensor fusion; Algorithm 1 "Fuse all gradient into
// one group" and its inverse).
//
// One launch moves the whole list, however many small tensors it has.  The bucket
// is cut into chunks of kChunkBytes of one tensor's segment (tensor + trailing
// padding); by default every workgroup takes one chunk, in bucket order (a persistent
// grid striding over the chunk ids can be asked for instead).  Each workgroup copies the
// per-tensor chunk-count prefix table into LDS once and finds the tensor of its chunk by
// binary search there (the table is uniform across the workgroup, so the LDS reads are
// broadcasts).  Inside a chunk each lane moves
// 16-byte vectors: the bucket side is always 16-byte aligned, the tensor side is
// accessed with element-aligned 16-byte loads/stores (gfx950 global memory
// instructions do not need natural alignment), so tight layouts and odd tensor
// addresses stay on the vector path.  Only the partial vectors at a chunk's two
// ends and at the tensor/padding boundary go element by element.
//
// HBM-bound: 2*s bytes per element (read once, written once); no arithmetic
// except the exponent test that raises the overflow flag while packing.
#include "xs_device.h"
#include "xs_internal.h"

namespace xs {

// Tensor addresses arrive as integers; the global address space on them (gbyte, gvec) makes
// the copies compile to global_* rather than flat_* instructions.

template <int ALIGN>
struct __attribute__((packed, aligned(ALIGN))) LooseVec {
    u32x4 v;
};

// 16-byte accesses with or without the non-temporal hint.  The element-aligned ("loose")
// forms go through a packed struct so that the compiler may assume only ES-byte alignment;
// the non-temporal builtin needs a naturally typed pointer, so those forms move four dwords
// (fp32) through it only when the hint is asked for and the address happens to be aligned.
template <bool NT>
__device__ __forceinline__ u32x4 load_vec(const gvec *p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}
template <bool NT>
__device__ __forceinline__ void store_vec(gvec *p, u32x4 v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}
template <bool NT, int ES>
__device__ __forceinline__ u32x4 load_loose(const __attribute__((address_space(1))) LooseVec<ES> *p)
{
    if constexpr (NT) {
        if (((uintptr_t)p & 15u) == 0) return __builtin_nontemporal_load((const gvec *)p);
    }
    return p->v;
}
template <bool NT, int ES>
__device__ __forceinline__ void store_loose(__attribute__((address_space(1))) LooseVec<ES> *p, u32x4 v)
{
    if constexpr (NT) {
        if (((uintptr_t)p & 15u) == 0) { __builtin_nontemporal_store(v, (gvec *)p); return; }
    }
    p->v = v;
}

constexpr int kTrips = (kChunkBytes / 16 + 1 + kCopyThreads - 1) / kCopyThreads;   // 5

// first index in table[0..count) whose value is > key, minus one
template <typename Table>
__device__ __forceinline__ uint32_t find_tensor(Table table, uint32_t count, uint32_t key)
{
    uint32_t lo = 0, hi = count;          // invariant: table[lo-1] <= key < table[hi]
    while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        if (table[mid] <= key) lo = mid + 1;
        else hi = mid;
    }
    return lo - 1;
}

template <int ES>
struct Elem;
template <>
struct Elem<4> { typedef uint32_t type; };
template <>
struct Elem<2> { typedef uint16_t type; };

// UNPACK = false: tensors -> bucket (padding zero-filled, optional overflow flag)
// UNPACK = true : bucket -> tensors (padding skipped)
// DT: element type of the plan (XS_F32 / XS_F16 / XS_BF16); it matters only for the overflow test.
// One launch can serve several (pointer table, bucket) pairs of the same plan - the W
// workers' packs of one synchronisation: work item = (pair, chunk), pair-major.
struct CopyPairs {
    const uintptr_t *tables[XS_MAX_REPLICAS];
    unsigned char *buckets[XS_MAX_REPLICAS];
};

template <bool UNPACK, bool DETECT, int DT, bool LDS_TABLE, bool NT>
__global__ __launch_bounds__(kCopyThreads) void copy_kernel(
    PlanTables tb, uint32_t n_tensors, uint32_t n_chunks, uint32_t n_pairs, CopyPairs pairs,
    int32_t *found_inf)
{
    constexpr int ES = Grad<DT>::ES;
    typedef typename Elem<ES>::type elem_t;
    typedef __attribute__((address_space(1))) elem_t gelem;
    extern __shared__ uint32_t s_prefix[];
    if constexpr (LDS_TABLE) {
        for (uint32_t i = threadIdx.x; i <= n_tensors; i += kCopyThreads) s_prefix[i] = tb.chunk_prefix[i];
        __syncthreads();
    }
    bool bad = false;

    const uint64_t n_items = (uint64_t)n_pairs * n_chunks;
    for (uint64_t item = blockIdx.x; item < n_items; item += gridDim.x) {
        const uint32_t pair = (uint32_t)(item / n_chunks);
        const uint32_t c = (uint32_t)(item - (uint64_t)pair * n_chunks);
        const uintptr_t *tensor_ptrs = pairs.tables[pair];
        unsigned char *bucket = pairs.buckets[pair];
        uint32_t t, first_chunk;
        if constexpr (LDS_TABLE) {
            t = find_tensor(s_prefix, n_tensors + 1, c);
            t = (uint32_t)__builtin_amdgcn_readfirstlane((int)t);
            first_chunk = s_prefix[t];
        } else {
            t = find_tensor(tb.chunk_prefix, n_tensors + 1, c);
            t = (uint32_t)__builtin_amdgcn_readfirstlane((int)t);
            first_chunk = tb.chunk_prefix[t];
        }
        const uint64_t seg_begin = tb.offsets[t] * ES;
        const uint64_t seg_bytes = tb.offsets[t + 1] * ES - seg_begin;
        const uint64_t val_bytes = tb.numel[t] * ES;
        const uint64_t k0 = (uint64_t)(c - first_chunk) * kChunkBytes;
        const uint64_t left = seg_bytes - k0;
        const int32_t len = (int32_t)(left < kChunkBytes ? left : kChunkBytes);       // bytes in this chunk
        const int32_t vlen = val_bytes <= k0 ? 0
                             : (int32_t)((val_bytes - k0) < (uint64_t)len ? (val_bytes - k0) : (uint64_t)len);
        gbyte *b = (gbyte *)bucket + seg_begin + k0;                // bucket side of the chunk
        gbyte *q = (gbyte *)tensor_ptrs[t] + k0;                    // tensor side of the chunk
        const int32_t skew = (int32_t)((uintptr_t)b & 15u);         // bucket vectors start at b - skew
        const int32_t nvec = (skew + len + 15) >> 4;

        u32x4 r[kTrips];
        bool fast[kTrips];
#pragma unroll
        for (int u = 0; u < kTrips; ++u) {
            const int32_t j = (int32_t)threadIdx.x + u * (int32_t)kCopyThreads;
            const int32_t lo = j * 16 - skew;                       // byte offset inside the chunk
            fast[u] = j < nvec && lo >= 0 && lo + 16 <= vlen;
            if (fast[u]) {
                if constexpr (UNPACK) r[u] = load_vec<NT>((const gvec *)(b + lo));
                else r[u] = load_loose<NT, ES>((const __attribute__((address_space(1))) LooseVec<ES> *)(q + lo));
            }
        }
#pragma unroll
        for (int u = 0; u < kTrips; ++u) {
            const int32_t j = (int32_t)threadIdx.x + u * (int32_t)kCopyThreads;
            const int32_t lo = j * 16 - skew;
            if (fast[u]) {
                if constexpr (UNPACK) store_loose<NT, ES>((__attribute__((address_space(1))) LooseVec<ES> *)(q + lo), r[u]);
                else {
                    store_vec<NT>((gvec *)(b + lo), r[u]);
                    if constexpr (DETECT)
                        bad = bad || Grad<DT>::nonfinite(r[u][0]) || Grad<DT>::nonfinite(r[u][1]) ||
                              Grad<DT>::nonfinite(r[u][2]) || Grad<DT>::nonfinite(r[u][3]);
                }
            } else if (j < nvec) {
                const int32_t e0 = lo < 0 ? 0 : lo;
                const int32_t e1 = lo + 16 < len ? lo + 16 : len;
                for (int32_t e = e0; e < e1; e += ES) {
                    if (e < vlen) {
                        if constexpr (UNPACK) *(gelem *)(q + e) = *(const gelem *)(b + e);
                        else {
                            const elem_t bits = *(const gelem *)(q + e);
                            *(gelem *)(b + e) = bits;
                            if constexpr (DETECT) bad |= Grad<DT>::nonfinite_elem(bits);
                        }
                    } else if constexpr (!UNPACK) {
                        *(gelem *)(b + e) = (elem_t)0;
                    }
                }
            }
        }
    }

    if constexpr (DETECT) {
        raise_flag_if(bad, found_inf);
    }
}

template <bool UNPACK, bool DETECT, int DT>
static int launch_copy(const Tuning &tn, const xs_plan *plan, const void *const *tables, void *const *buckets,
                       uint32_t n_pairs, int32_t *found_inf, hipStream_t stream)
{
    const int cus = compute_units();
    if (cus < 0) return cus;
    CopyPairs pairs;
    for (uint32_t i = 0; i < XS_MAX_REPLICAS; ++i) {
        pairs.tables[i] = i < n_pairs ? (const uintptr_t *)tables[i] : nullptr;
        pairs.buckets[i] = i < n_pairs ? (unsigned char *)buckets[i] : nullptr;
    }
    const uint64_t n_items = (uint64_t)n_pairs * plan->n_chunks;
    const bool lds = plan->n_tensors + 1 <= kLdsPrefixCap;
    const size_t lds_bytes = lds ? (size_t)(plan->n_tensors + 1) * 4 : 0;
    // Measured on MI355X: one chunk per workgroup, dispatched in bucket order as earlier
    // workgroups retire, moves 8-9 % more than a persistent grid of 16 workgroups per compute
    // unit striding over the chunks (as for the reduce kernels, the DRAM access front stays
    // tight).  Every workgroup stages the chunk-prefix table in LDS first, so lists with a table
    // beyond 4 KiB give each workgroup one more chunk per further 4 KiB to amortise that.
    uint64_t blocks;
    if (tn.copy_wg_per_cu() > 0) {
        blocks = (uint64_t)cus * (uint64_t)tn.copy_wg_per_cu();
    } else {
        const uint64_t per_wg = lds_bytes > 4096 ? (lds_bytes + 4095) / 4096 : 1;
        blocks = (n_items + per_wg - 1) / per_wg;
    }
    if (tn.copy_max_wg() > 0 && blocks > (uint64_t)tn.copy_max_wg())
        blocks = (uint64_t)tn.copy_max_wg();
    if (blocks > n_items) blocks = n_items;
    if (blocks > 0x7fffffffull) blocks = 0x7fffffffull;   // the loop covers the rest
    const bool nt = tn.copy_nt();
    const dim3 grid((unsigned)blocks), block(kCopyThreads);
    // Measured on MI355X: five 256-lane workgroups per compute unit (32 KiB of LDS each, only the
    // table's share of it used) copy 6 % faster than the eight that fit otherwise, and they leave
    // wave slots on every compute unit, so that another task's workgroups dispatched meanwhile
    // spread evenly instead of piling up on the few compute units that happen to have room.
    const size_t reserve = tn.copy_lds_reserve() < 0 ? 32768 : (size_t)tn.copy_lds_reserve();
    const size_t lds_launch = (lds_bytes > reserve ? lds_bytes : reserve);
#define XS_COPY_LAUNCH(LDS, NT)                                                                   \
    hipLaunchKernelGGL((copy_kernel<UNPACK, DETECT, DT, LDS, NT>), grid, block, lds_launch,        \
                       stream, plan->tables, plan->n_tensors, plan->n_chunks, n_pairs, pairs, found_inf)
    if (lds) { if (nt) XS_COPY_LAUNCH(true, true); else XS_COPY_LAUNCH(true, false); }
    else     { if (nt) XS_COPY_LAUNCH(false, true); else XS_COPY_LAUNCH(false, false); }
#undef XS_COPY_LAUNCH
    XS_HIP_TRY(hipGetLastError());
    return XS_OK;
}

int launch_pack(const Tuning &tn, const xs_plan *plan, const void *const *tables, void *const *buckets,
                uint32_t n_pairs, int32_t *found_inf, hipStream_t stream)
{
    if (!found_inf)   // a plain copy: only the element size matters
        return plan->elem_size == 4
                   ? launch_copy<false, false, XS_F32>(tn, plan, tables, buckets, n_pairs, nullptr, stream)
                   : launch_copy<false, false, XS_F16>(tn, plan, tables, buckets, n_pairs, nullptr, stream);
    switch (plan->dtype) {
    case XS_F16: return launch_copy<false, true, XS_F16>(tn, plan, tables, buckets, n_pairs, found_inf, stream);
    case XS_BF16: return launch_copy<false, true, XS_BF16>(tn, plan, tables, buckets, n_pairs, found_inf, stream);
    default: return launch_copy<false, true, XS_F32>(tn, plan, tables, buckets, n_pairs, found_inf, stream);
    }
}

int launch_unpack(const Tuning &tn, const xs_plan *plan, const void *bucket, void *const *tensor_ptrs,
                  hipStream_t stream)
{
    const void *table = tensor_ptrs;
    void *b = const_cast<void *>(bucket);
    if (plan->elem_size == 4)
        return launch_copy<true, false, XS_F32>(tn, plan, &table, &b, 1, nullptr, stream);
    return launch_copy<true, false, XS_F16>(tn, plan, &table, &b, 1, nullptr, stream);
}

}  // namespace xs
