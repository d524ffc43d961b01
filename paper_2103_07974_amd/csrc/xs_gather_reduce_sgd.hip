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
// first element.  When the row is a complete row of valid elements of that tensor (the rule:
// 64-element layers are the smallest in the workloads) that is decided from three scalar
// look-ups and the W tensor addresses come through scalar loads too; otherwise lanes step
// forward from the row's first tensor and each fetches its own.  A vector that lies wholly inside a tensor's valid range takes the vector
// path (element-aligned 16-byte loads from the tensors); vectors that touch padding or
// straddle tensors (tight layouts) go element by element, with padding contributing +0
// exactly as a packed bucket would.
#include "xs_device.h"
#include "xs_internal.h"

namespace xs {

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
    int view_dtype;                // dtype of the views param_ptrs point to
    float lr, mu, wd, c;
    const f32x4 *tensor_hp;        // device [n_tensors] records (lr, mu, wd, -), kernels with PT only
    int32_t *found_inf;
};

// The vector path for one lane.  `t` is either wave-uniform (scalar address loads) or per lane.
// EXCH (half-precision gradients, whole wavefront in one tensor, complete row): lanes take
// state vectors `lane` and `64 + lane` of the row instead of the two under their own gradient
// vector, and receive the matching gradient sums through the LDS crossbar, so that every
// state access of the wavefront is one contiguous kilobyte.
template <int W, int GT, bool DETECT, bool VIEWS, bool PT, bool EXCH>
__device__ __forceinline__ void vector_path(const GatherArgs &a, uint32_t t, uint64_t j, uint64_t k,
                                            bool &bad)
{
    constexpr int ES = Grad<GT>::ES;
    constexpr int VEC = 16 / ES;
    constexpr int SV = VEC / 4;
    u32x4 g[W];
#pragma unroll
    for (int w = 0; w < W; ++w)
        g[w] = load_tensor_vec<ES>((const gbyte *)a.grad_ptrs[(uint64_t)t * W + w] + k * ES);
    // state vector q of this lane starts at bucket element sj[q] = tensor element sk[q]
    uint64_t sj[SV], sk[SV];
#pragma unroll
    for (int q = 0; q < SV; ++q) {
        if constexpr (EXCH) {
            const uint32_t lane = threadIdx.x & (kWave - 1);
            const uint64_t lane_off = (uint64_t)lane * VEC;               // j = row start + lane_off
            const uint64_t d = (uint64_t)q * 4 * kWave + 4 * lane;
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
        x[q] = load16f<true>((const f32x4 *)(a.x_in + sj[q]));
        v[q] = load16f<true>((const f32x4 *)(a.v_in + sj[q]));
    }
    // every state vector handled here lies in tensor t (EXCH: the whole row does)
    const f32x4 rec = PT ? a.tensor_hp[t] : f32x4{a.lr, a.mu, a.wd, 0.f};
    float s[VEC];
#pragma unroll
    for (int w = 0; w < W; ++w) accumulate<GT, DETECT>(g[w], w == 0, s, bad);
    if constexpr (EXCH) exchange_half_row(s);
#pragma unroll
    for (int q = 0; q < SV; ++q) {
        sgd_update4(s + 4 * q, a.c, x[q], v[q], rec);
        store16f<true>((f32x4 *)(a.x_out + sj[q]), x[q]);
        store16f<true>((f32x4 *)(a.v_out + sj[q]), v[q]);
    }
    if constexpr (VIEWS) {
        gbyte *view = (gbyte *)a.param_ptrs[t];
#pragma unroll
        for (int q = 0; q < SV; ++q) store_view4(view, sk[q], x[q], a.view_dtype);
    }
}

// One bucket element at a time: padding contributes +0, consecutive elements may belong to
// different tensors.  `te` is carried along so that the search only ever moves forward.
template <int GT, bool DETECT, bool VIEWS, bool PT>
__device__ __forceinline__ void element_path(const GatherArgs &a, uint32_t &te, uint64_t je, bool &bad)
{
    constexpr int ES = Grad<GT>::ES;
    while (te + 1 < a.n_tensors && a.tb.offsets[te + 1] <= je) ++te;
    const uint64_t ke = je - a.tb.offsets[te];
    const bool valid = ke < a.tb.numel[te];
    float s = 0.f;
    if (valid) {
        for (uint32_t w = 0; w < a.W; ++w) {
            const gbyte *p = (const gbyte *)a.grad_ptrs[(uint64_t)te * a.W + w] + ke * ES;
            uint32_t e;
            if constexpr (Grad<GT>::HALF) e = *(const __attribute__((address_space(1))) uint16_t *)p;
            else e = *(const __attribute__((address_space(1))) uint32_t *)p;
            if constexpr (DETECT) bad |= Grad<GT>::nonfinite_elem(e);
            const float f = Grad<GT>::lo(e);
            s = (w == 0) ? f : s + f;
        }
    }
    float xe = a.x_in[je], ve = a.v_in[je];
    float lr = a.lr, mu = a.mu, wd = a.wd;
    if constexpr (PT) {
        const f32x4 rec = a.tensor_hp[te];     // padding follows the tensor in front of it
        lr = rec[0]; mu = rec[1]; wd = rec[2];
    }
    sgd_update(s, a.c, xe, ve, lr, mu, wd);
    a.x_out[je] = xe;
    a.v_out[je] = ve;
    if constexpr (VIEWS) {
        if (valid) store_view1((gbyte *)a.param_ptrs[te], ke, xe, a.view_dtype);
    }
}

template <int W, int GT, bool DETECT, bool VIEWS, bool PT>
__global__ __launch_bounds__(kMaxReduceThreads) void gather_reduce_sgd_kernel(GatherArgs a)
{
    constexpr int VEC = 16 / Grad<GT>::ES;
    constexpr uint64_t ROW = (uint64_t)kWave * VEC;
    if (a.found_inf != nullptr && *(volatile int32_t *)a.found_inf != 0) return;
    bool bad = false;

    // each wavefront of the workgroup owns one row per trip
    const uint32_t waves = blockDim.x / kWave, wave = threadIdx.x / kWave, lane = threadIdx.x & (kWave - 1);
    for (uint64_t row = (uint64_t)blockIdx.x * waves + wave; row < a.n_rows; row += (uint64_t)gridDim.x * waves) {
        const uint64_t j = row * ROW + (uint64_t)lane * VEC;           // lane's first bucket element
        if (j >= a.n_bucket) continue;
        {
            // The rule: a complete row of valid elements of one tensor.  Decided from three
            // wave-uniform look-ups through the scalar cache (the tables are not written while
            // the kernel runs); the tensor addresses follow the same way.
            typedef const __attribute__((address_space(4))) uint32_t cu32;
            typedef const __attribute__((address_space(4))) uint64_t cu64;
            const uint32_t ts = (uint32_t)__builtin_amdgcn_readfirstlane((int)((cu32 *)a.tb.row_first)[row]);
            const uint64_t off = ((cu64 *)a.tb.offsets)[ts];
            const uint64_t num = ((cu64 *)a.tb.numel)[ts];
            const uint64_t row_end = (row + 1) * ROW;
            if (off + num >= row_end && row_end <= a.n_bucket) {
                vector_path<W, GT, DETECT, VIEWS, PT, Grad<GT>::HALF>(a, ts, j, j - off, bad);
                continue;
            }
        }
        // rows that cross tensors, touch padding or end the bucket: per-lane look-ups
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
            if (Grad<GT>::HALF && (row + 1) * ROW <= a.n_bucket)      // complete row: all 64 lanes here
                vector_path<W, GT, DETECT, VIEWS, PT, Grad<GT>::HALF>(a, tu, j, ku, bad);
            else
                vector_path<W, GT, DETECT, VIEWS, PT, false>(a, tu, j, ku, bad);
        } else if (full) {
            vector_path<W, GT, DETECT, VIEWS, PT, false>(a, t, j, k, bad);
        } else {
            uint32_t te = t;
            for (int e = 0; e < VEC; ++e) {
                if (j + e >= a.n_bucket) break;
                element_path<GT, DETECT, VIEWS, PT>(a, te, j + e, bad);
            }
        }
    }

    if constexpr (DETECT) {
        raise_flag_if(bad, a.found_inf);
    }
}

// Any W: element by element with a run-time replica count.
template <int GT, bool DETECT, bool VIEWS, bool PT>
__global__ __launch_bounds__(kMaxReduceThreads) void gather_reduce_sgd_anyw_kernel(GatherArgs a)
{
    constexpr int VEC = 16 / Grad<GT>::ES;
    constexpr uint64_t ROW = (uint64_t)kWave * VEC;
    if (a.found_inf != nullptr && *(volatile int32_t *)a.found_inf != 0) return;
    bool bad = false;
    const uint32_t waves = blockDim.x / kWave, wave = threadIdx.x / kWave, lane = threadIdx.x & (kWave - 1);
    for (uint64_t row = (uint64_t)blockIdx.x * waves + wave; row < a.n_rows; row += (uint64_t)gridDim.x * waves) {
        const uint64_t j = row * ROW + (uint64_t)lane * VEC;
        if (j >= a.n_bucket) continue;
        uint32_t te = a.tb.row_first[row];
        for (int e = 0; e < VEC; ++e) {
            if (j + e >= a.n_bucket) break;
            element_path<GT, DETECT, VIEWS, PT>(a, te, j + e, bad);
        }
    }
    if constexpr (DETECT) {
        raise_flag_if(bad, a.found_inf);
    }
}

// ---- dispatch ---------------------------------------------------------------------------
template <int W, int GT, bool PT>
static void launch_g(const GatherArgs &a, bool detect, bool views, dim3 grid, dim3 block, unsigned lds,
                     hipStream_t stream)
{
    if (detect)
        hipLaunchKernelGGL((gather_reduce_sgd_kernel<W, GT, true, false, PT>), grid, block, lds, stream, a);
    else if (views)
        hipLaunchKernelGGL((gather_reduce_sgd_kernel<W, GT, false, true, PT>), grid, block, lds, stream, a);
    else
        hipLaunchKernelGGL((gather_reduce_sgd_kernel<W, GT, false, false, PT>), grid, block, lds, stream, a);
}

template <int GT, bool PT>
static void launch_ganyw(const GatherArgs &a, bool detect, bool views, dim3 grid, dim3 block, unsigned lds,
                         hipStream_t stream)
{
    if (detect)
        hipLaunchKernelGGL((gather_reduce_sgd_anyw_kernel<GT, true, false, PT>), grid, block, lds, stream, a);
    else if (views)
        hipLaunchKernelGGL((gather_reduce_sgd_anyw_kernel<GT, false, true, PT>), grid, block, lds, stream, a);
    else
        hipLaunchKernelGGL((gather_reduce_sgd_anyw_kernel<GT, false, false, PT>), grid, block, lds, stream, a);
}

template <int GT, bool PT>
static void launch_w(const GatherArgs &a, bool detect, bool views, dim3 grid, dim3 block, unsigned lds,
                     hipStream_t stream)
{
    switch (a.W) {
    case 2: launch_g<2, GT, PT>(a, detect, views, grid, block, lds, stream); break;
    case 4: launch_g<4, GT, PT>(a, detect, views, grid, block, lds, stream); break;
    case 8: launch_g<8, GT, PT>(a, detect, views, grid, block, lds, stream); break;
    case 16: launch_g<16, GT, PT>(a, detect, views, grid, block, lds, stream); break;
    default: launch_ganyw<GT, PT>(a, detect, views, grid, block, lds, stream); break;
    }
}

template <int GT>
static void launch_gt(const GatherArgs &a, bool detect, bool views, dim3 grid, dim3 block, unsigned lds,
                      hipStream_t stream)
{
    if (a.tensor_hp != nullptr) launch_w<GT, true>(a, detect, views, grid, block, lds, stream);
    else launch_w<GT, false>(a, detect, views, grid, block, lds, stream);
}

int launch_gather_reduce_sgd(const Tuning &tn, const xs_plan *plan, const void *const *grad_ptrs, uint32_t W,
                             const float *x_in, const float *v_in, float *x_out, float *v_out,
                             void *const *param_ptrs, int view_dtype, const xs_sgd_hparams &hp,
                             const xs_tensor_hparams *tensor_hp, int32_t *found_inf, bool detect,
                             hipStream_t stream)
{
    const int cus = compute_units();
    if (cus < 0) return cus;
    const bool half = plan->dtype != XS_F32;
    GatherArgs a;
    a.tb = plan->tables;
    a.n_tensors = plan->n_tensors;
    a.W = W;
    a.n_bucket = plan->bucket_elems;
    a.n_rows = plan->n_rows;
    a.grad_ptrs = (const uintptr_t *)grad_ptrs;
    a.x_in = x_in; a.v_in = v_in; a.x_out = x_out; a.v_out = v_out;
    a.param_ptrs = (const uintptr_t *)param_ptrs;
    a.view_dtype = view_dtype;
    a.lr = hp.lr; a.mu = hp.momentum; a.wd = hp.weight_decay;
    volatile float one_over_w = 1.0f / (float)W;
    a.c = hp.inv_loss_scale * one_over_w;
    a.tensor_hp = (const f32x4 *)tensor_hp;
    a.found_inf = found_inf;

    const uint64_t waves = (uint64_t)tn.reduce_waves_per_wg();
    uint64_t blocks = (plan->n_rows + waves - 1) / waves;
    if (tn.reduce_wg_per_cu() > 0) {
        const uint64_t cap = (uint64_t)cus * (uint64_t)tn.reduce_wg_per_cu();
        if (blocks > cap) blocks = cap;
    }
    if (tn.reduce_max_wg() > 0 && blocks > (uint64_t)tn.reduce_max_wg())
        blocks = (uint64_t)tn.reduce_max_wg();
    if (blocks > 0x7fffffffull) blocks = 0x7fffffffull;
    const dim3 grid((unsigned)blocks), block((unsigned)(waves * kWave));
    // The look-ups in front of the loads want more resident wavefronts than the bucket form,
    // the fewer the more bytes a wavefront has in flight.  Measured optimum (one-wave
    // workgroups per compute unit, VGG-16- and BERT-large-shaped sets):
    //   fp32: W = 8: 13 (12 KiB), W = 4: 16 (10 KiB), W = 2: 20 (8 KiB)
    //   half: W = 16: 8-10 (16-20 KiB), W = 8: 13, W = 4 and 2: 16
    int lds_auto = half ? 16384 : 8192;
    if (W == 2 || W == 4 || W == 8 || W == 16) {
        if (!half) lds_auto = W >= 8 ? 12288 : (W == 4 ? 10240 : 8192);
        else lds_auto = W >= 16 ? 16384 : (W == 8 ? 12288 : 10240);
    }
    const unsigned lds = (unsigned)(tn.gather_lds_reserve() < 0 ? lds_auto : tn.gather_lds_reserve());
    const bool views = param_ptrs != nullptr;

    switch (plan->dtype) {
    case XS_F16: launch_gt<XS_F16>(a, detect, views, grid, block, lds, stream); break;
    case XS_BF16: launch_gt<XS_BF16>(a, detect, views, grid, block, lds, stream); break;
    default: launch_gt<XS_F32>(a, detect, views, grid, block, lds, stream); break;
    }
    XS_HIP_TRY(hipGetLastError());
    return XS_OK;
}

}  // namespace xs
