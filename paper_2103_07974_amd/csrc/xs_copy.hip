// Pack / unpack between a list of per-layer tensors and one fused bucket on gfx950
// (arXiv 2103.07974, Section 2.1 tensor fusion; Algorithm 1 "Fuse all gradient into
// one group" and its inverse).
//
// One launch moves the whole list (or the W workers' lists), however many small tensors
// it has.  HBM-bound: 2*s bytes per element (read once, written once); no arithmetic except
// the exponent test that raises the overflow flag while packing.
//
// row_copy_kernel - the form every plan-based call uses.  The bucket is cut into rows of one
// KiB; a one-wavefront workgroup moves one row, one 16-byte vector per lane, and rows are
// dispatched in bucket order with nothing capping how many share a compute unit: this is
// the launch shape at which a plain 1:1 copy reaches its best rate on MI355X (6.5 TB/s; one
// KiB in flight per wavefront needs every wave slot).  The plan's row table names the tensor
// that holds a row's first element; when the whole row lies in that tensor's segment (the
// rule) its offset, size and address come through four scalar loads and every lane copies its
// vector; rows that cross tensors step forward per lane.  The bucket side is always accessed
// with aligned 16-byte vectors, the tensor side with element-aligned ones (gfx950 global
// memory instructions need no natural alignment), so tight layouts and odd tensor addresses
// stay on the vector path; only vectors that touch padding or span tensors go element by
// element.
//
// copy_kernel - the earlier form, kept for xs_fuse_pack_static, whose layout tables must be
// small enough to travel in kernel arguments (this form needs O(tensors) of table, the row
// form one word per KiB of bucket): 16 KiB chunks of one tensor's segment per 256-lane
// workgroup, the tensor of a chunk found by binary search in an LDS copy of the per-tensor
// chunk-count prefix table.
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

// ---- the row form ---------------------------------------------------------------------------
struct RowCopyArgs {
    PlanTables tb;
    uint32_t n_tensors;
    uint32_t n_pairs;
    uint64_t n_rows;
    uint64_t n_bucket;     // bucket length in elements
    CopyPairs pairs;
    int32_t *found_inf;
};

typedef const __attribute__((address_space(4))) uint32_t cu32;
typedef const __attribute__((address_space(4))) uint64_t cu64;
typedef const __attribute__((address_space(4))) uintptr_t cuptr;

// One 16-byte vector of the bucket starting at bucket element j, which lies in the segment of
// a tensor that starts at bucket element `off`, has `num` valid elements and lives at `base`.
template <bool UNPACK, bool DETECT, int DT, bool NT>
__device__ __forceinline__ void copy_vector(gbyte *bucket, gbyte *base, uint64_t j, uint64_t off,
                                            uint64_t num, uint64_t n_bucket, bool &bad)
{
    constexpr int ES = Grad<DT>::ES;
    constexpr int VEC = 16 / ES;
    typedef typename Elem<ES>::type elem_t;
    typedef __attribute__((address_space(1))) elem_t gelem;
    typedef __attribute__((address_space(1))) LooseVec<ES> gloose;
    const uint64_t k = j - off;
    gbyte *b = bucket + j * ES;
    gbyte *q = base + k * ES;
    if (k + VEC <= num) {
        if constexpr (UNPACK) {
            store_loose<NT, ES>((gloose *)q, load_vec<NT>((const gvec *)b));
        } else {
            const u32x4 r = load_loose<NT, ES>((const gloose *)q);
            store_vec<NT>((gvec *)b, r);
            if constexpr (DETECT)
                bad = bad || Grad<DT>::nonfinite(r[0]) || Grad<DT>::nonfinite(r[1]) ||
                      Grad<DT>::nonfinite(r[2]) || Grad<DT>::nonfinite(r[3]);
        }
        return;
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        if (j + e >= n_bucket) break;
        if (k + e < num) {
            if constexpr (UNPACK) ((gelem *)q)[e] = ((const gelem *)b)[e];
            else {
                const elem_t bits = ((const gelem *)q)[e];
                ((gelem *)b)[e] = bits;
                if constexpr (DETECT) bad |= Grad<DT>::nonfinite_elem(bits);
            }
        } else if constexpr (!UNPACK) {
            ((gelem *)b)[e] = (elem_t)0;       // padding behind the tensor
        }
    }
}

template <bool UNPACK, bool DETECT, int DT, bool NT>
__global__ __launch_bounds__(kMaxReduceThreads) void row_copy_kernel(RowCopyArgs a)
{
    constexpr int ES = Grad<DT>::ES;
    constexpr int VEC = 16 / ES;
    constexpr uint64_t ROW = (uint64_t)kWave * VEC;
    typedef typename Elem<ES>::type elem_t;
    typedef __attribute__((address_space(1))) elem_t gelem;
    const uint32_t waves = blockDim.x / kWave, wave = threadIdx.x / kWave, lane = threadIdx.x & (kWave - 1);
    bool bad = false;
    // grid: x over the rows of one (pointer table, bucket) pair, y over the pairs
    gbyte *bucket = (gbyte *)a.pairs.buckets[blockIdx.y];
    const uintptr_t *tensor_ptrs = a.pairs.tables[blockIdx.y];

    for (uint64_t row = (uint64_t)blockIdx.x * waves + wave; row < a.n_rows; row += (uint64_t)gridDim.x * waves) {
        // wave-uniform look-ups through the scalar cache (the tables are not written while the
        // kernel runs): the row's first tensor, its segment and its address
        const uint32_t t_row = (uint32_t)__builtin_amdgcn_readfirstlane((int)((cu32 *)a.tb.row_first)[row]);
        const uint64_t off = ((cu64 *)a.tb.offsets)[t_row];
        const uint64_t seg_end = ((cu64 *)a.tb.offsets)[t_row + 1];
        const uint64_t num = ((cu64 *)a.tb.numel)[t_row];
        gbyte *base = (gbyte *)((cuptr *)tensor_ptrs)[t_row];
        const uint64_t row_begin = row * ROW;
        const uint64_t row_end = row_begin + ROW < a.n_bucket ? row_begin + ROW : a.n_bucket;
        const uint64_t j = row_begin + (uint64_t)lane * VEC;
        if (j >= a.n_bucket) continue;
        if (seg_end >= row_end) {                    // the rule: the whole row is in one segment
            copy_vector<UNPACK, DETECT, DT, NT>(bucket, base, j, off, num, a.n_bucket, bad);
            continue;
        }
        // the row crosses tensors: each lane finds the tensor of its vector's first element
        uint32_t t = t_row;
        while (t + 1 < a.n_tensors && a.tb.offsets[t + 1] <= j) ++t;
        const uint64_t offl = a.tb.offsets[t], numl = a.tb.numel[t];
        if (j - offl + VEC <= numl || j + VEC <= a.tb.offsets[t + 1]) {
            // wholly valid, or valid elements and padding of this one tensor
            copy_vector<UNPACK, DETECT, DT, NT>(bucket, (gbyte *)tensor_ptrs[t], j, offl, numl, a.n_bucket, bad);
            continue;
        }
        // the vector itself spans tensors (tight layouts): element by element, stepping forward
        for (int e = 0; e < VEC; ++e) {
            const uint64_t je = j + e;
            if (je >= a.n_bucket) break;
            while (t + 1 < a.n_tensors && a.tb.offsets[t + 1] <= je) ++t;
            const uint64_t ke = je - a.tb.offsets[t];
            gelem *b = (gelem *)(bucket + je * ES);
            if (ke < a.tb.numel[t]) {
                gelem *q = (gelem *)((gbyte *)tensor_ptrs[t] + ke * ES);
                if constexpr (UNPACK) *q = *b;
                else {
                    const elem_t bits = *q;
                    *b = bits;
                    if constexpr (DETECT) bad |= Grad<DT>::nonfinite_elem(bits);
                }
            } else if constexpr (!UNPACK) {
                *b = (elem_t)0;
            }
        }
    }

    if constexpr (DETECT) {
        raise_flag_if(bad, a.found_inf);
    }
}

template <bool UNPACK, bool DETECT, int DT>
static int launch_row_copy(const Tuning &tn, const xs_plan *plan, const void *const *tables,
                           void *const *buckets, uint32_t n_pairs, int32_t *found_inf, hipStream_t stream)
{
    const int cus = compute_units();
    if (cus < 0) return cus;
    RowCopyArgs a;
    a.tb = plan->tables;
    a.n_tensors = plan->n_tensors;
    a.n_pairs = n_pairs;
    a.n_rows = plan->n_rows;
    a.n_bucket = plan->bucket_elems;
    for (uint32_t i = 0; i < XS_MAX_REPLICAS; ++i) {
        a.pairs.tables[i] = i < n_pairs ? (const uintptr_t *)tables[i] : nullptr;
        a.pairs.buckets[i] = i < n_pairs ? (unsigned char *)buckets[i] : nullptr;
    }
    a.found_inf = found_inf;
    const uint64_t waves = (uint64_t)tn.copy_waves_per_wg();
    uint64_t blocks = (plan->n_rows + waves - 1) / waves;      // per pair
    if (tn.copy_wg_per_cu() > 0) {
        const uint64_t cap = ((uint64_t)cus * (uint64_t)tn.copy_wg_per_cu() + n_pairs - 1) / n_pairs;
        if (blocks > cap) blocks = cap;
    }
    if (tn.copy_max_wg() > 0) {
        const uint64_t cap = ((uint64_t)tn.copy_max_wg() + n_pairs - 1) / n_pairs;
        if (blocks > cap) blocks = cap;
    }
    if (blocks > 0x7fffffffull) blocks = 0x7fffffffull;   // the loop covers the rest
    // Measured on MI355X: no occupancy cap is the optimum here (6.45-6.55 TB/s; an 8 KiB
    // reservation per wavefront, i.e. 20 per compute unit, already costs a quarter)
    const unsigned lds = (unsigned)(tn.copy_lds_reserve() < 0 ? 0 : tn.copy_lds_reserve());
    const dim3 grid((unsigned)blocks, n_pairs), block((unsigned)(waves * kWave));
    if (tn.copy_nt())
        hipLaunchKernelGGL((row_copy_kernel<UNPACK, DETECT, DT, true>), grid, block, lds, stream, a);
    else
        hipLaunchKernelGGL((row_copy_kernel<UNPACK, DETECT, DT, false>), grid, block, lds, stream, a);
    XS_HIP_TRY(hipGetLastError());
    return XS_OK;
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
    const bool rows = plan->tables.row_first != nullptr;   // plans of xs_plan_create; not the static tables
    if (!found_inf) {   // a plain copy: only the element size matters
        if (rows)
            return plan->elem_size == 4
                       ? launch_row_copy<false, false, XS_F32>(tn, plan, tables, buckets, n_pairs, nullptr, stream)
                       : launch_row_copy<false, false, XS_F16>(tn, plan, tables, buckets, n_pairs, nullptr, stream);
        return plan->elem_size == 4
                   ? launch_copy<false, false, XS_F32>(tn, plan, tables, buckets, n_pairs, nullptr, stream)
                   : launch_copy<false, false, XS_F16>(tn, plan, tables, buckets, n_pairs, nullptr, stream);
    }
    if (rows) {
        switch (plan->dtype) {
        case XS_F16: return launch_row_copy<false, true, XS_F16>(tn, plan, tables, buckets, n_pairs, found_inf, stream);
        case XS_BF16: return launch_row_copy<false, true, XS_BF16>(tn, plan, tables, buckets, n_pairs, found_inf, stream);
        default: return launch_row_copy<false, true, XS_F32>(tn, plan, tables, buckets, n_pairs, found_inf, stream);
        }
    }
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
    if (plan->tables.row_first != nullptr) {
        if (plan->elem_size == 4)
            return launch_row_copy<true, false, XS_F32>(tn, plan, &table, &b, 1, nullptr, stream);
        return launch_row_copy<true, false, XS_F16>(tn, plan, &table, &b, 1, nullptr, stream);
    }
    if (plan->elem_size == 4)
        return launch_copy<true, false, XS_F32>(tn, plan, &table, &b, 1, nullptr, stream);
    return launch_copy<true, false, XS_F16>(tn, plan, &table, &b, 1, nullptr, stream);
}

}  // namespace xs
