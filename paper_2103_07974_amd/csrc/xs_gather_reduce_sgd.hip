// Gathering form of the fused reduce + average + momentum-SGD pass for gfx950.
//
// Same arithmetic and order as reduce_sgd_kernel (Algorithm 1 of arXiv 2103.07974,
// "Receive averaged gradients" and "Model Update"), but the W workers' gradients are read
// straight from their per-layer tensors through the bucket layout of Section 2.1 instead of
// from W packed buckets, and the updated parameters can be written to the per-layer views in
// the same pass.  On one GPU, where the fused bucket never has to leave the device, this
// removes the W packs and the unpack: (W*s + 16) bytes per element are read/written once
// (+4 with views) instead of (3*W*s + 24).
//
// Work unit: one row of 1 KiB of gradient data per replica = one 16-byte vector per lane of
// a one-wavefront workgroup, dispatched in bucket order (the launch shape that measured
// fastest for the bucket form).  The plan's row table gives the tensor that holds the row's
// first element; lanes step forward from there (rows that cross tensor boundaries are the
// exception: 64-element layers are the smallest in the workloads).  When the whole wavefront
// sits in one tensor, the W tensor addresses come through scalar loads; otherwise each lane
// fetches its own.  A vector that lies wholly inside a tensor's valid range takes the vector
// path (element-aligned 16-byte loads from the tensors); vectors that touch padding or
// straddle tensors (tight layouts) go element by element, with padding contributing +0
// exactly as a packed bucket would.
#include "xs_internal.h"

namespace xs {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) unsigned char gbyte;
typedef __attribute__((address_space(1))) u32x4 gvec;

template <int ALIGN>
struct __attribute__((packed, aligned(ALIGN))) LooseVec {
    u32x4 v;
};

constexpr int kLanes = 64;

template <bool NT, int ES>
__device__ __forceinline__ u32x4 load_tensor_vec(const gbyte *p)
{
    if constexpr (NT) {
        if (((uintptr_t)p & 15u) == 0) return __builtin_nontemporal_load((const gvec *)p);
    }
    return ((const __attribute__((address_space(1))) LooseVec<ES> *)p)->v;
}

template <bool NT>
__device__ __forceinline__ void store_tensor_vec(gbyte *p, f32x4 v)
{
    const u32x4 bits = __builtin_bit_cast(u32x4, v);
    if constexpr (NT) {
        if (((uintptr_t)p & 15u) == 0) { __builtin_nontemporal_store(bits, (gvec *)p); return; }
    }
    ((__attribute__((address_space(1))) LooseVec<4> *)p)->v = bits;
}

template <bool NT>
__device__ __forceinline__ f32x4 load_state(const f32x4 *p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}
template <bool NT>
__device__ __forceinline__ void store_state(f32x4 *p, f32x4 v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

__device__ __forceinline__ float g_half_lo(uint32_t w)
{
    return (float)__builtin_bit_cast(_Float16, (uint16_t)(w & 0xffffu));
}
__device__ __forceinline__ float g_half_hi(uint32_t w)
{
    return (float)__builtin_bit_cast(_Float16, (uint16_t)(w >> 16));
}
__device__ __forceinline__ bool g_nonfinite_f32(uint32_t w) { return (w & 0x7f800000u) == 0x7f800000u; }
__device__ __forceinline__ bool g_nonfinite_f16x2(uint32_t w)
{
    return (((w & 0x7c007c00u) + 0x04000400u) & 0x80008000u) != 0u;
}

__device__ __forceinline__ void g_sgd(float g_sum, float c, float &x, float &v, float lr, float mu,
                                      float wd)
{
    const float g = g_sum * c;
    const float wx = wd * x;
    const float d = g + wx;
    const float mv = mu * v;
    const float vn = mv + d;
    const float lv = lr * vn;
    v = vn;
    x = x - lv;
}

struct GatherArgs {
    PlanTables tb;
    uint32_t n_tensors;
    uint32_t W;               // run-time copy of the replica count
    uint64_t n_bucket;
    uint64_t n_rows;
    const uintptr_t *grad_ptrs;    // device [n_tensors][W]
    const float *x_in, *v_in;
    float *x_out, *v_out;
    const uintptr_t *param_ptrs;   // device [n_tensors] or nullptr
    float lr, mu, wd, c;
    int32_t *found_inf;
};

// The vector path for one lane.  `t` is either wave-uniform (scalar address loads) or per lane.
// SHUF (fp16 gradients, whole wavefront in one tensor, complete row): lanes take state
// vectors `lane` and `64 + lane` of the row instead of the two under their own gradient
// vector, and receive the matching gradient sums through the LDS crossbar, so that every
// state access of the wavefront is one contiguous kilobyte.
template <int W, bool F16, bool DETECT, bool VIEWS, bool NTG, bool NTS, bool NTX, bool SHUF>
__device__ __forceinline__ void vector_path(const GatherArgs &a, uint32_t t, uint64_t j, uint64_t k,
                                            bool &bad)
{
    constexpr int ES = F16 ? 2 : 4;
    constexpr int VEC = 16 / ES;
    constexpr int SV = VEC / 4;
    u32x4 g[W];
#pragma unroll
    for (int w = 0; w < W; ++w)
        g[w] = load_tensor_vec<NTG, ES>((const gbyte *)a.grad_ptrs[(uint64_t)t * W + w] + k * ES);
    // state vector q of this lane starts at bucket element sj[q] = tensor element sk[q]
    uint64_t sj[SV], sk[SV];
#pragma unroll
    for (int q = 0; q < SV; ++q) {
        if constexpr (SHUF) {
            const uint64_t lane_off = (uint64_t)threadIdx.x * VEC;       // j = row start + lane_off
            const uint64_t d = (uint64_t)q * 4 * kLanes + 4 * threadIdx.x;
            sj[q] = j - lane_off + d;
            sk[q] = k - lane_off + d;
        } else {
            sj[q] = j + 4 * q;
            sk[q] = k + 4 * q;
        }
    }
    f32x4 x[SV], v[SV];
#pragma unroll
    for (int q = 0; q < SV; ++q) {
        x[q] = load_state<NTX>((const f32x4 *)(a.x_in + sj[q]));
        v[q] = load_state<NTX>((const f32x4 *)(a.v_in + sj[q]));
    }
    float s[VEC];
#pragma unroll
    for (int w = 0; w < W; ++w) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t bits = g[w][q];
            if constexpr (F16) {
                if constexpr (DETECT) bad |= g_nonfinite_f16x2(bits);
                const float lo = g_half_lo(bits), hi = g_half_hi(bits);
                if (w == 0) { s[2 * q] = lo; s[2 * q + 1] = hi; }
                else { s[2 * q] = s[2 * q] + lo; s[2 * q + 1] = s[2 * q + 1] + hi; }
            } else {
                if constexpr (DETECT) bad |= g_nonfinite_f32(bits);
                const float f = __builtin_bit_cast(float, bits);
                if (w == 0) s[q] = f;
                else s[q] = s[q] + f;
            }
        }
    }
    if constexpr (SHUF) {
        // element 4L+e of the row sits in lane L>>1, slot (L&1)*4+e; element 256+4L+e in lane
        // 32+(L>>1), same slot
        const int src0 = (int)((threadIdx.x >> 1) << 2);
        const int src1 = (int)((32u + (threadIdx.x >> 1)) << 2);
        const bool odd = (threadIdx.x & 1u) != 0u;
        float t2[VEC];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int lo = __builtin_bit_cast(int, s[e]), hi = __builtin_bit_cast(int, s[4 + e]);
            const int a_lo = __builtin_amdgcn_ds_bpermute(src0, lo);
            const int a_hi = __builtin_amdgcn_ds_bpermute(src0, hi);
            const int b_lo = __builtin_amdgcn_ds_bpermute(src1, lo);
            const int b_hi = __builtin_amdgcn_ds_bpermute(src1, hi);
            t2[e] = __builtin_bit_cast(float, odd ? a_hi : a_lo);
            t2[4 + e] = __builtin_bit_cast(float, odd ? b_hi : b_lo);
        }
#pragma unroll
        for (int e = 0; e < VEC; ++e) s[e] = t2[e];
    }
#pragma unroll
    for (int q = 0; q < SV; ++q) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float xe = x[q][e], ve = v[q][e];
            g_sgd(s[4 * q + e], a.c, xe, ve, a.lr, a.mu, a.wd);
            x[q][e] = xe;
            v[q][e] = ve;
        }
        store_state<NTS>((f32x4 *)(a.x_out + sj[q]), x[q]);
        store_state<NTS>((f32x4 *)(a.v_out + sj[q]), v[q]);
    }
    if constexpr (VIEWS) {
        gbyte *dst = (gbyte *)a.param_ptrs[t];
#pragma unroll
        for (int q = 0; q < SV; ++q) store_tensor_vec<NTS>(dst + sk[q] * 4, x[q]);
    }
}

template <int W, bool F16, bool DETECT, bool VIEWS, bool NTG, bool NTS, bool NTX>
__global__ __launch_bounds__(kLanes) void gather_reduce_sgd_kernel(GatherArgs a)
{
    constexpr int ES = F16 ? 2 : 4;
    constexpr int VEC = 16 / ES;
    constexpr uint64_t ROW = (uint64_t)kLanes * VEC;
    if (a.found_inf != nullptr && *(volatile int32_t *)a.found_inf != 0) return;
    bool bad = false;

    for (uint64_t row = blockIdx.x; row < a.n_rows; row += gridDim.x) {
        const uint64_t j = row * ROW + (uint64_t)threadIdx.x * VEC;    // lane's first bucket element
        if (j >= a.n_bucket) continue;
        const uint32_t t_row = a.tb.row_first[row];
        uint32_t t = t_row;
        while (t + 1 < a.n_tensors && a.tb.offsets[t + 1] <= j) ++t;
        const uint64_t k = j - a.tb.offsets[t];
        const bool full = k + VEC <= a.tb.numel[t];

        const bool wave_in_row_tensor = __builtin_amdgcn_ballot_w64(t != t_row || !full) == 0ull;
        if (wave_in_row_tensor) {
            // every active lane is a full vector of tensor t_row: scalar address loads
            const uint32_t tu = (uint32_t)__builtin_amdgcn_readfirstlane((int)t_row);
            const uint64_t ku = j - a.tb.offsets[tu];
            if (F16 && (row + 1) * ROW <= a.n_bucket)      // complete row: all 64 lanes are here
                vector_path<W, F16, DETECT, VIEWS, NTG, NTS, NTX, F16>(a, tu, j, ku, bad);
            else
                vector_path<W, F16, DETECT, VIEWS, NTG, NTS, NTX, false>(a, tu, j, ku, bad);
        } else if (full) {
            vector_path<W, F16, DETECT, VIEWS, NTG, NTS, NTX, false>(a, t, j, k, bad);
        } else {
            // element by element: padding contributes +0, elements may belong to later tensors
            uint32_t te = t;
            for (int e = 0; e < VEC; ++e) {
                const uint64_t je = j + e;
                if (je >= a.n_bucket) break;
                while (te + 1 < a.n_tensors && a.tb.offsets[te + 1] <= je) ++te;
                const uint64_t ke = je - a.tb.offsets[te];
                const bool valid = ke < a.tb.numel[te];
                float s = 0.f;
                if (valid) {
#pragma unroll
                    for (int w = 0; w < W; ++w) {
                        const gbyte *p = (const gbyte *)a.grad_ptrs[(uint64_t)te * W + w] + ke * ES;
                        float f;
                        if constexpr (F16) {
                            const uint16_t h = *(const __attribute__((address_space(1))) uint16_t *)p;
                            if constexpr (DETECT) bad |= (h & 0x7c00u) == 0x7c00u;
                            f = (float)__builtin_bit_cast(_Float16, h);
                        } else {
                            const uint32_t b = *(const __attribute__((address_space(1))) uint32_t *)p;
                            if constexpr (DETECT) bad |= g_nonfinite_f32(b);
                            f = __builtin_bit_cast(float, b);
                        }
                        s = (w == 0) ? f : s + f;
                    }
                }
                float xe = a.x_in[je], ve = a.v_in[je];
                g_sgd(s, a.c, xe, ve, a.lr, a.mu, a.wd);
                a.x_out[je] = xe;
                a.v_out[je] = ve;
                if constexpr (VIEWS) {
                    if (valid)
                        *(__attribute__((address_space(1))) float *)((gbyte *)a.param_ptrs[te] + ke * 4) = xe;
                }
            }
        }
    }

    if constexpr (DETECT) {
        if (__builtin_amdgcn_ballot_w64(bad) != 0ull && (threadIdx.x & 63u) == 0u)
            atomicOr(a.found_inf, 1);
    }
}

// Any W: replicas accumulated one after the other (run-time trip count).
template <bool F16, bool DETECT, bool VIEWS>
__global__ __launch_bounds__(kLanes) void gather_reduce_sgd_anyw_kernel(GatherArgs a)
{
    constexpr int ES = F16 ? 2 : 4;
    constexpr int VEC = 16 / ES;
    constexpr uint64_t ROW = (uint64_t)kLanes * VEC;
    if (a.found_inf != nullptr && *(volatile int32_t *)a.found_inf != 0) return;
    bool bad = false;
    for (uint64_t row = blockIdx.x; row < a.n_rows; row += gridDim.x) {
        const uint64_t j = row * ROW + (uint64_t)threadIdx.x * VEC;
        if (j >= a.n_bucket) continue;
        uint32_t te = a.tb.row_first[row];
        for (int e = 0; e < VEC; ++e) {
            const uint64_t je = j + e;
            if (je >= a.n_bucket) break;
            while (te + 1 < a.n_tensors && a.tb.offsets[te + 1] <= je) ++te;
            const uint64_t ke = je - a.tb.offsets[te];
            const bool valid = ke < a.tb.numel[te];
            float s = 0.f;
            if (valid) {
                for (uint32_t w = 0; w < a.W; ++w) {
                    const gbyte *p = (const gbyte *)a.grad_ptrs[(uint64_t)te * a.W + w] + ke * ES;
                    float f;
                    if constexpr (F16) {
                        const uint16_t h = *(const __attribute__((address_space(1))) uint16_t *)p;
                        if constexpr (DETECT) bad |= (h & 0x7c00u) == 0x7c00u;
                        f = (float)__builtin_bit_cast(_Float16, h);
                    } else {
                        const uint32_t b = *(const __attribute__((address_space(1))) uint32_t *)p;
                        if constexpr (DETECT) bad |= g_nonfinite_f32(b);
                        f = __builtin_bit_cast(float, b);
                    }
                    s = (w == 0) ? f : s + f;
                }
            }
            float xe = a.x_in[je], ve = a.v_in[je];
            g_sgd(s, a.c, xe, ve, a.lr, a.mu, a.wd);
            a.x_out[je] = xe;
            a.v_out[je] = ve;
            if constexpr (VIEWS) {
                if (valid)
                    *(__attribute__((address_space(1))) float *)((gbyte *)a.param_ptrs[te] + ke * 4) = xe;
            }
        }
    }
    if constexpr (DETECT) {
        if (__builtin_amdgcn_ballot_w64(bad) != 0ull && (threadIdx.x & 63u) == 0u)
            atomicOr(a.found_inf, 1);
    }
}

// ---- dispatch ---------------------------------------------------------------------------
template <int W, bool F16, bool DETECT, bool VIEWS>
static void launch_g(const GatherArgs &a, dim3 grid, unsigned lds, hipStream_t stream)
{
    // cache hints as in the bucket form: every stream non-temporal
    hipLaunchKernelGGL((gather_reduce_sgd_kernel<W, F16, DETECT, VIEWS, true, true, true>), grid,
                       dim3(kLanes), lds, stream, a);
}

template <int W>
static void launch_gw(const GatherArgs &a, bool f16, bool detect, bool views, dim3 grid,
                      unsigned lds, hipStream_t stream)
{
    if (f16) {
        if (detect) launch_g<W, true, true, false>(a, grid, lds, stream);
        else if (views) launch_g<W, true, false, true>(a, grid, lds, stream);
        else launch_g<W, true, false, false>(a, grid, lds, stream);
    } else {
        if (detect) launch_g<W, false, true, false>(a, grid, lds, stream);
        else if (views) launch_g<W, false, false, true>(a, grid, lds, stream);
        else launch_g<W, false, false, false>(a, grid, lds, stream);
    }
}

template <bool F16>
static void launch_ganyw(const GatherArgs &a, bool detect, bool views, dim3 grid, unsigned lds,
                         hipStream_t stream)
{
    if (detect)
        hipLaunchKernelGGL((gather_reduce_sgd_anyw_kernel<F16, true, false>), grid, dim3(kLanes), lds, stream, a);
    else if (views)
        hipLaunchKernelGGL((gather_reduce_sgd_anyw_kernel<F16, false, true>), grid, dim3(kLanes), lds, stream, a);
    else
        hipLaunchKernelGGL((gather_reduce_sgd_anyw_kernel<F16, false, false>), grid, dim3(kLanes), lds, stream, a);
}

int launch_gather_reduce_sgd(const xs_plan *plan, const void *const *grad_ptrs, uint32_t W,
                             const float *x_in, const float *v_in, float *x_out, float *v_out,
                             void *const *param_ptrs, const xs_sgd_hparams &hp,
                             int32_t *found_inf, bool detect, hipStream_t stream)
{
    const int cus = compute_units();
    if (cus < 0) return cus;
    const bool f16 = plan->dtype == XS_F16;
    GatherArgs a;
    a.tb = plan->tables;
    a.n_tensors = plan->n_tensors;
    a.W = W;
    a.n_bucket = plan->bucket_elems;
    a.n_rows = plan->n_rows;
    a.grad_ptrs = (const uintptr_t *)grad_ptrs;
    a.x_in = x_in; a.v_in = v_in; a.x_out = x_out; a.v_out = v_out;
    a.param_ptrs = (const uintptr_t *)param_ptrs;
    a.lr = hp.lr; a.mu = hp.momentum; a.wd = hp.weight_decay;
    volatile float one_over_w = 1.0f / (float)W;
    a.c = hp.inv_loss_scale * one_over_w;
    a.found_inf = found_inf;

    uint64_t blocks = plan->n_rows;
    if (g_tuning.reduce_wg_per_cu > 0) {
        const uint64_t cap = (uint64_t)cus * (uint64_t)g_tuning.reduce_wg_per_cu;
        if (blocks > cap) blocks = cap;
    }
    if (g_tuning.reduce_max_wg > 0 && blocks > (uint64_t)g_tuning.reduce_max_wg)
        blocks = (uint64_t)g_tuning.reduce_max_wg;
    if (blocks > 0x7fffffffull) blocks = 0x7fffffffull;
    const dim3 grid((unsigned)blocks);
    // the address look-ups in front of the loads want about twice the residency of the
    // bucket form: 20 one-wave workgroups per compute unit for fp32, 10 for fp16 (measured)
    const int lds_auto = f16 ? 16384 : 8192;
    const unsigned lds = (unsigned)(g_tuning.gather_lds_reserve < 0 ? lds_auto : g_tuning.gather_lds_reserve);
    const bool views = param_ptrs != nullptr;

    switch (W) {
    case 1: launch_gw<1>(a, f16, detect, views, grid, lds, stream); break;
    case 2: launch_gw<2>(a, f16, detect, views, grid, lds, stream); break;
    case 4: launch_gw<4>(a, f16, detect, views, grid, lds, stream); break;
    case 8: launch_gw<8>(a, f16, detect, views, grid, lds, stream); break;
    case 16: launch_gw<16>(a, f16, detect, views, grid, lds, stream); break;
    default:
        if (f16) launch_ganyw<true>(a, detect, views, grid, lds, stream);
        else launch_ganyw<false>(a, detect, views, grid, lds, stream);
    }
    XS_HIP_TRY(hipGetLastError());
    return XS_OK;
}

}  // namespace xs
