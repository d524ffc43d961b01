// Fused reduce + average + momentum-SGD for gfx950 (Algorithm 1 of arXiv 2103.07974,
// steps "Receive averaged gradients" and "Model Update").
//
// The pass is element-wise and streams (W*s + 16) bytes per element exactly once
// (W gradient replicas of s bytes read, parameters and momentum read and written),
// so HBM bandwidth is the only bound and there is nothing for MFMA to do.
//
//  * One 16-byte vector of every stream per lane: all W+2 loads (fp16: W+4) are issued as
//    global_load_dwordx4 before the first add; replicas are added in worker order 0..W-1 with
//    every operation rounded to fp32 separately (-ffp-contract=off): bit-reproducible.
//  * One-wavefront workgroups, one vector per lane, no loop in the default launch: workgroups
//    are dispatched in address order as earlier ones retire, which keeps the DRAM access
//    front tight (a strided persistent grid measured 25 % slower on MI355X).  The generic-W
//    kernel (any W; also chosen by XS_TUNE_REDUCE_SMALL for its small register footprint)
//    can be launched with 2 or 4 wavefronts per workgroup instead, each wavefront still
//    owning one row of 64 vectors: a 4-wave workgroup puts one wavefront on every SIMD of
//    its compute unit, which is how a synchronisation shares the compute units with another
//    task's kernels.  The W-specialised kernels always run as one-wavefront workgroups.
//  * The launch reserves LDS the kernel never touches, to cap how many wavefronts share a
//    compute unit: about 100-120 KB of loads in flight per compute unit is the optimum.
//  * Every stream is touched once, so loads and stores carry the non-temporal hint.
//  * fp16 gradients: lanes exchange their gradient sums through the LDS crossbar so that the
//    fp32 state accesses of a wavefront are contiguous (see the main loop).
//  * The only cross-lane quantity besides that is the overflow flag: a wavefront ballot, then
//    one atomic per wavefront that saw a non-finite gradient.
#include "xs_device.h"
#include "xs_internal.h"

namespace xs {

constexpr int kThreads = kWave;   // one row = one wavefront = 64 gradient vectors

template <int N>
struct ReplicaPtrs {
    const void *p[N];
};

struct ReduceArgs {
    uint64_t n;
    const float *x_in, *v_in;
    float *x_out, *v_out;
    float lr, mu, wd, c;
    int32_t *found_inf;
    void *model_copy;       // half-precision copy of the updated parameters, or nullptr
    int model_copy_dtype;   // XS_F16 or XS_BF16
    TensorHp thp;           // layout tables (PT or VIEWS) and per-tensor records (PT only)
    const uint64_t *numel;        // device [n_tensors]                     (VIEWS only)
    const uintptr_t *param_ptrs;  // device [n_tensors]: per-layer views    (VIEWS only)
    int view_dtype;               // element type of the views
};

// One element of the ragged tail (fewer than VEC elements at the end of the bucket).
template <int GT, bool DETECT, bool PT, bool VIEWS, typename Reps>
__device__ __forceinline__ void tail_element(const Reps &reps, uint32_t W, const ReduceArgs &a,
                                             uint64_t j, bool &bad)
{
    float s = 0.f;
    for (uint32_t w = 0; w < W; ++w) {
        uint32_t e;
        if constexpr (Grad<GT>::HALF) e = ((const uint16_t *)reps.p[w])[j];
        else e = ((const uint32_t *)reps.p[w])[j];
        if constexpr (DETECT) bad |= Grad<GT>::nonfinite_elem(e);
        const float f = Grad<GT>::lo(e);
        s = (w == 0) ? f : s + f;
    }
    float xe = a.x_in[j], ve = a.v_in[j];
    float lr = a.lr, mu = a.mu, wd = a.wd;
    if constexpr (PT) {
        uint32_t t = a.thp.row_first[j / ((uint64_t)kThreads * (16 / Grad<GT>::ES))];
        seek_tensor(a.thp, t, j);
        const f32x4 rec = a.thp.rec[t];
        lr = rec[0]; mu = rec[1]; wd = rec[2];
    }
    sgd_update(s, a.c, xe, ve, lr, mu, wd);
    a.x_out[j] = xe;
    a.v_out[j] = ve;
    if (a.model_copy) ((uint16_t *)a.model_copy)[j] = to_half1(xe, a.model_copy_dtype);
    if constexpr (VIEWS) {
        uint32_t t = a.thp.row_first[j / ((uint64_t)kThreads * (16 / Grad<GT>::ES))];
        seek_tensor(a.thp, t, j);
        const uint64_t k = j - a.thp.offsets[t];
        if (k < a.numel[t]) store_view1((gbyte *)a.param_ptrs[t], k, xe, a.view_dtype);
    }
}

// The state vectors of one row of kThreads gradient vectors under per-tensor records: the
// row's first tensor and, when the whole row lies in that tensor's segment (the rule: the
// smallest layers of the workloads are a quarter of a row), its record through scalar loads.
struct RowHp {
    uint32_t t_first;
    bool uniform;
    f32x4 rec;
};
// The three look-ups go through the constant address space with wave-uniform indices, i.e.
// through the scalar cache: they neither queue behind the streaming vector loads nor hold up
// their issue.  (The tables are written once, at plan creation and by the caller before the
// launch, and never by a kernel.)
typedef const __attribute__((address_space(4))) uint32_t cu32;
typedef const __attribute__((address_space(4))) uint64_t cu64;
typedef const __attribute__((address_space(4))) f32x4 cf32x4;

template <int VEC>
__device__ __forceinline__ RowHp row_hp(const TensorHp &h, uint64_t first_vec, uint64_t n)
{
    constexpr uint64_t ROW = (uint64_t)kThreads * VEC;
    const uint32_t row = (uint32_t)__builtin_amdgcn_readfirstlane((int)(first_vec / kThreads));
    RowHp r;
    r.t_first = (uint32_t)__builtin_amdgcn_readfirstlane((int)((cu32 *)h.row_first)[row]);
    const uint64_t row_end = ((uint64_t)row + 1) * ROW < n ? ((uint64_t)row + 1) * ROW : n;
    r.uniform = ((cu64 *)h.offsets)[r.t_first + 1] >= row_end;
    r.rec = ((cf32x4 *)h.rec)[r.t_first];
    return r;
}

// The unpack fused into the pass (Section 2.1 read backwards: the per-layer tensors receive
// the updated parameters): where a row's first element lives, and - when every element of
// the row is a valid element of that one tensor, the rule - that tensor's offset and view
// address through scalar loads.
struct RowView {
    uint32_t t_first;
    bool uniform;
    uint64_t off;
    gbyte *view;
};
typedef const __attribute__((address_space(4))) uintptr_t cuptr;

template <int VEC>
__device__ __forceinline__ RowView row_view(const ReduceArgs &a, uint64_t first_vec)
{
    constexpr uint64_t ROW = (uint64_t)kThreads * VEC;
    const uint32_t row = (uint32_t)__builtin_amdgcn_readfirstlane((int)(first_vec / kThreads));
    RowView r;
    r.t_first = (uint32_t)__builtin_amdgcn_readfirstlane((int)((cu32 *)a.thp.row_first)[row]);
    const uint64_t row_end = ((uint64_t)row + 1) * ROW < a.n ? ((uint64_t)row + 1) * ROW : a.n;
    r.off = ((cu64 *)a.thp.offsets)[r.t_first];
    r.uniform = r.off + ((cu64 *)a.numel)[r.t_first] >= row_end;
    r.view = (gbyte *)((cuptr *)a.param_ptrs)[r.t_first];
    return r;
}

// four updated parameters that start at bucket element j go to their place in the views
__device__ __forceinline__ void store_views4(const ReduceArgs &a, const RowView &rv, uint64_t j, f32x4 x)
{
    if (rv.uniform) {
        store_view4(rv.view, j - rv.off, x, a.view_dtype);
        return;
    }
    uint32_t t = rv.t_first;
    seek_tensor(a.thp, t, j);
    const uint64_t k = j - a.thp.offsets[t];
    if (k + 4 <= a.numel[t]) {
        store_view4((gbyte *)a.param_ptrs[t], k, x, a.view_dtype);
        return;
    }
    // the vector touches padding or spans several tensors (tight layouts): element by element
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        if (j + q >= a.n) break;
        seek_tensor(a.thp, t, j + q);
        const uint64_t ke = j + q - a.thp.offsets[t];
        if (ke < a.numel[t]) store_view1((gbyte *)a.param_ptrs[t], ke, x[q], a.view_dtype);
    }
}

// VEC elements per lane per trip: 4 (fp32 gradients) or 8 (fp16 / bf16 gradients), so that
// every gradient load is 16 bytes wide.
template <int W, int GT, bool DETECT, bool NTG, bool NTS, bool PT, bool VIEWS>
__global__ __launch_bounds__(kThreads) void reduce_sgd_kernel(ReplicaPtrs<W> reps, ReduceArgs a)
{
    constexpr bool HALF = Grad<GT>::HALF;
    constexpr int VEC = 16 / Grad<GT>::ES;
    constexpr int SV = VEC / 4;   // fp32 state vectors per gradient vector
    if (a.found_inf != nullptr && *(volatile int32_t *)a.found_inf != 0) return;

    const uint64_t nvec = a.n / VEC;
    const uint64_t stride = (uint64_t)gridDim.x * kThreads;
    const uint32_t lane = threadIdx.x;             // always launched with one-wavefront workgroups
    bool bad = false;

    for (uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x; i < nvec; i += stride) {
        u32x4 g[W];
#pragma unroll
        for (int w = 0; w < W; ++w) g[w] = load16<NTG>((const u32x4 *)reps.p[w] + i);
        // Which fp32 state vectors this lane updates.  fp32 gradients: the one under its
        // gradient vector.  Half-precision gradients: a lane's 8 elements would be two
        // neighbouring state vectors, i.e. 32-byte strides per load instruction; in a full row
        // of 64 lanes the lanes instead take state vectors `lane` and `64 + lane` of the row,
        // so that every state load and store of the wavefront is one contiguous kilobyte, and
        // the gradient sums are moved to the owning lanes through the LDS crossbar afterwards.
        uint64_t sx[SV];
        bool exchanged = false;
        if constexpr (HALF) {
            const uint64_t row0 = i - lane;                        // vector index of lane 0
            exchanged = row0 + (kThreads - 1) < nvec;              // uniform: the whole row is live
            sx[0] = exchanged ? row0 * 2 + lane : i * 2;
            sx[1] = exchanged ? row0 * 2 + kThreads + lane : i * 2 + 1;
        } else {
            sx[0] = i;
        }
        f32x4 x[SV], v[SV];
#pragma unroll
        for (int k = 0; k < SV; ++k) {
            x[k] = load16f<NTS>((const f32x4 *)a.x_in + sx[k]);
            v[k] = load16f<NTS>((const f32x4 *)a.v_in + sx[k]);
        }
        RowHp rh;
        if constexpr (PT) rh = row_hp<VEC>(a.thp, i - lane, a.n);
        else rh.rec = f32x4{a.lr, a.mu, a.wd, 0.f};
        RowView rv;
        if constexpr (VIEWS) rv = row_view<VEC>(a, i - lane);
        float s[VEC];
#pragma unroll
        for (int w = 0; w < W; ++w) accumulate<GT, DETECT>(g[w], w == 0, s, bad);
        if constexpr (HALF) {
            if (exchanged) exchange_half_row(s);
        }
        uint32_t t = PT ? rh.t_first : 0u;
#pragma unroll
        for (int k = 0; k < SV; ++k) {
            if (!PT || rh.uniform) sgd_update4(s + 4 * k, a.c, x[k], v[k], rh.rec);
            else sgd_update4_per_tensor(a.thp, t, sx[k] * 4, s + 4 * k, a.c, x[k], v[k]);
            store16f<NTS>((f32x4 *)a.x_out + sx[k], x[k]);
            store16f<NTS>((f32x4 *)a.v_out + sx[k], v[k]);
            if (a.model_copy)
                store8<NTS>((u32x2 *)a.model_copy + sx[k], to_half4(x[k], a.model_copy_dtype));
            if constexpr (VIEWS) store_views4(a, rv, sx[k] * 4, x[k]);
        }
    }

    // ragged tail: fewer than VEC elements, one lane each, in workgroup 0
    const uint32_t rem = (uint32_t)(a.n - nvec * VEC);
    if (blockIdx.x == 0 && threadIdx.x < rem)
        tail_element<GT, DETECT, PT, VIEWS>(reps, (uint32_t)W, a, nvec * VEC + threadIdx.x, bad);

    if constexpr (DETECT) {
        raise_flag_if(bad, a.found_inf);
    }
}

// Any W up to XS_MAX_REPLICAS: replica loop with a run-time trip count, four loads in flight
// at a time.  Same arithmetic and order as the specialised kernels; plain lane mapping.
template <int GT, bool DETECT, bool PT, bool VIEWS>
__global__ __launch_bounds__(kMaxReduceThreads) void reduce_sgd_anyw_kernel(
    ReplicaPtrs<XS_MAX_REPLICAS> reps, uint32_t W, ReduceArgs a)
{
    constexpr int ES = Grad<GT>::ES;
    constexpr int VEC = 16 / ES;
    constexpr int SV = VEC / 4;
    if (a.found_inf != nullptr && *(volatile int32_t *)a.found_inf != 0) return;
    const uint64_t nvec = a.n / VEC;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    const uint32_t lane = threadIdx.x & (kThreads - 1);
    bool bad = false;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += stride) {
        RowHp rh;
        if constexpr (PT) rh = row_hp<VEC>(a.thp, i - lane, a.n);
        else rh.rec = f32x4{a.lr, a.mu, a.wd, 0.f};
        RowView rv;
        if constexpr (VIEWS) rv = row_view<VEC>(a, i - lane);
        float s[VEC];
        accumulate<GT, DETECT>(*((const u32x4 *)reps.p[0] + i), true, s, bad);
#pragma unroll 4
        for (uint32_t w = 1; w < W; ++w)
            accumulate<GT, DETECT>(*((const u32x4 *)reps.p[w] + i), false, s, bad);
        uint32_t t = PT ? rh.t_first : 0u;
#pragma unroll
        for (int k = 0; k < SV; ++k) {
            f32x4 x = ((const f32x4 *)a.x_in)[i * SV + k], v = ((const f32x4 *)a.v_in)[i * SV + k];
            if (!PT || rh.uniform) sgd_update4(s + 4 * k, a.c, x, v, rh.rec);
            else sgd_update4_per_tensor(a.thp, t, (i * SV + k) * 4, s + 4 * k, a.c, x, v);
            ((f32x4 *)a.x_out)[i * SV + k] = x;
            ((f32x4 *)a.v_out)[i * SV + k] = v;
            if (a.model_copy) ((u32x2 *)a.model_copy)[i * SV + k] = to_half4(x, a.model_copy_dtype);
            if constexpr (VIEWS) store_views4(a, rv, (i * SV + k) * 4, x);
        }
    }
    const uint32_t rem = (uint32_t)(a.n - nvec * VEC);
    if (blockIdx.x == 0 && threadIdx.x < rem)
        tail_element<GT, DETECT, PT, VIEWS>(reps, W, a, nvec * VEC + threadIdx.x, bad);
    if constexpr (DETECT) {
        raise_flag_if(bad, a.found_inf);
    }
}

// ---- dispatch --------------------------------------------------------------------
struct Launch {
    const void *const *replicas;
    ReduceArgs a;
    dim3 grid, block;   // the generic-W kernel: `block` lanes per workgroup
    dim3 grid1;         // the W-specialised kernels: one wavefront per workgroup
    unsigned lds_reserve;
    hipStream_t stream;
};

template <int W, int GT, bool DETECT, bool NTG, bool NTS, bool PT, bool VIEWS>
static void launch_one(const Launch &l)
{
    ReplicaPtrs<W> r;
    for (int w = 0; w < W; ++w) r.p[w] = l.replicas[w];
    hipLaunchKernelGGL((reduce_sgd_kernel<W, GT, DETECT, NTG, NTS, PT, VIEWS>), l.grid1, dim3(kThreads),
                       l.lds_reserve, l.stream, r, l.a);
}

template <int W, int GT, bool DETECT, bool NTG, bool NTS>
static void launch_pt(const Launch &l)
{
    if (l.a.thp.rec != nullptr) launch_one<W, GT, DETECT, NTG, NTS, true, false>(l);
    else launch_one<W, GT, DETECT, NTG, NTS, false, false>(l);
}

template <int W, int GT, bool DETECT>
static void launch_nt(const Launch &l, bool ntg, bool nts)
{
    if (ntg) { if (nts) launch_pt<W, GT, DETECT, true, true>(l); else launch_pt<W, GT, DETECT, true, false>(l); }
    else     { if (nts) launch_pt<W, GT, DETECT, false, true>(l); else launch_pt<W, GT, DETECT, false, false>(l); }
}

template <int W, int GT>
static void launch_gt(const Launch &l, bool detect, bool ntg, bool nts)
{
    if (l.a.param_ptrs != nullptr) {
        // with the unpack fused in: in place, no in-kernel detection, every stream non-temporal
        if (l.a.thp.rec != nullptr) launch_one<W, GT, false, true, true, true, true>(l);
        else launch_one<W, GT, false, true, true, false, true>(l);
        return;
    }
    if (detect) launch_nt<W, GT, true>(l, ntg, nts);
    else launch_nt<W, GT, false>(l, ntg, nts);
}

template <int W>
static void launch_w(const Launch &l, int dtype, bool detect, bool ntg, bool nts)
{
    switch (dtype) {
    case XS_F16: launch_gt<W, XS_F16>(l, detect, ntg, nts); break;
    case XS_BF16: launch_gt<W, XS_BF16>(l, detect, ntg, nts); break;
    default: launch_gt<W, XS_F32>(l, detect, ntg, nts); break;
    }
}

template <int GT, bool DETECT, bool PT, bool VIEWS>
static void launch_anyw_one(const Launch &l, uint32_t W)
{
    ReplicaPtrs<XS_MAX_REPLICAS> r;
    for (uint32_t w = 0; w < XS_MAX_REPLICAS; ++w) r.p[w] = w < W ? l.replicas[w] : nullptr;
    hipLaunchKernelGGL((reduce_sgd_anyw_kernel<GT, DETECT, PT, VIEWS>), l.grid, l.block, l.lds_reserve,
                       l.stream, r, W, l.a);
}

template <int GT>
static void launch_anyw(const Launch &l, uint32_t W, bool detect)
{
    const bool pt = l.a.thp.rec != nullptr;
    if (l.a.param_ptrs != nullptr) {
        if (pt) launch_anyw_one<GT, false, true, true>(l, W); else launch_anyw_one<GT, false, false, true>(l, W);
        return;
    }
    if (detect) { if (pt) launch_anyw_one<GT, true, true, false>(l, W); else launch_anyw_one<GT, true, false, false>(l, W); }
    else        { if (pt) launch_anyw_one<GT, false, true, false>(l, W); else launch_anyw_one<GT, false, false, false>(l, W); }
}

int launch_reduce_sgd(const Tuning &tn, const void *const *replicas, uint32_t W, int dtype, uint64_t n,
                      const float *x_in, const float *v_in, float *x_out, float *v_out,
                      const xs_sgd_hparams &hp, int32_t *found_inf, bool detect,
                      void *model_copy, int model_copy_dtype, const xs_plan *plan,
                      const xs_tensor_hparams *tensor_hp, void *const *param_ptrs, int view_dtype,
                      hipStream_t stream)
{
    const int cus = compute_units();
    if (cus < 0) return cus;
    const bool half = dtype != XS_F32;
    const uint64_t vec = half ? 8 : 4;
    const uint64_t threads = (uint64_t)kThreads * (uint64_t)tn.reduce_waves_per_wg();
    auto grid_for = [&](uint64_t lanes_per_wg) {
        uint64_t blocks = (n / vec + lanes_per_wg - 1) / lanes_per_wg;
        if (blocks == 0) blocks = 1;   // tail only
        if (tn.reduce_wg_per_cu() > 0) {
            const uint64_t cap = (uint64_t)cus * (uint64_t)tn.reduce_wg_per_cu();
            if (blocks > cap) blocks = cap;
        }
        if (tn.reduce_max_wg() > 0 && blocks > (uint64_t)tn.reduce_max_wg())
            blocks = (uint64_t)tn.reduce_max_wg();
        if (blocks > 0x7fffffffull) blocks = 0x7fffffffull;   // the loop covers the rest
        return blocks;
    };
    const uint64_t blocks = grid_for(threads), blocks1 = grid_for(kThreads);

    Launch l;
    l.replicas = replicas;
    l.a.n = n;
    l.a.x_in = x_in; l.a.v_in = v_in; l.a.x_out = x_out; l.a.v_out = v_out;
    l.a.lr = hp.lr; l.a.mu = hp.momentum; l.a.wd = hp.weight_decay;
    // one constant for averaging and loss scale: inv_loss_scale * (1/W), rounded to fp32 twice
    volatile float one_over_w = 1.0f / (float)W;
    l.a.c = hp.inv_loss_scale * one_over_w;
    l.a.found_inf = found_inf;
    l.a.model_copy = model_copy;
    l.a.model_copy_dtype = model_copy_dtype;
    // per-tensor records need the layout (plan) that the buckets were packed with
    l.a.thp.rec = (plan && tensor_hp) ? (const f32x4 *)tensor_hp : nullptr;
    l.a.thp.offsets = plan ? plan->tables.offsets : nullptr;
    l.a.thp.row_first = plan ? plan->tables.row_first : nullptr;
    l.a.thp.n_tensors = plan ? plan->n_tensors : 0;
    // the unpack fused in needs the layout as well (plan) and is never combined with `detect`
    l.a.numel = plan ? plan->tables.numel : nullptr;
    l.a.param_ptrs = (plan && param_ptrs && !detect) ? (const uintptr_t *)param_ptrs : nullptr;
    l.a.view_dtype = view_dtype;
    l.grid = dim3((unsigned)blocks);
    l.block = dim3((unsigned)threads);
    l.grid1 = dim3((unsigned)blocks1);
    l.stream = stream;
    // Measured on MI355X: the pass is fastest with 10 one-wave workgroups per compute unit
    // (fp32 W = 8: 12 loads per lane, about 120 KB in flight per compute unit; fp16 W = 16:
    // 20 loads per lane); more wavefronts than that only disorder the DRAM access stream,
    // fewer expose the latency of the kernel's prologue.  The LDS reservation (unused by the
    // kernel) is what caps the residency.
    // The W-specialised instances that look the row's tensor up want fewer, not more, resident
    // wavefronts than the plain kernel (measured on the VGG-16- and BERT-large-shaped sets, state
    // in one pool; GB/s at the reservation below against 16 KiB):
    //   unpack fused in, fp32:  W = 8: 6646 vs 6352 (5 per compute unit); W = 4: 6645 vs 6580 (8)
    //   unpack fused in, half:  W = 16: 6447 vs 6202 (5); W = 8: 6407 vs 6311 (6); W = 4: 6496 vs
    //                           6318 (6); W = 2: 6509 vs 6431 (8)
    //   per-tensor records only, half, W = 16: 6573 vs 6293 (5); every other case is flat
    const bool views = l.a.param_ptrs != nullptr, records = l.a.thp.rec != nullptr;
    const bool specialised = !tn.reduce_small() && (W == 2 || W == 4 || W == 8 || W == 16);
    int lds_auto = 16384;
    if (specialised && views) {
        if (!half) lds_auto = W >= 8 ? 28672 : (W == 4 ? 20480 : 16384);
        else lds_auto = W >= 16 ? 28672 : (W >= 4 ? 24576 : 20480);
    } else if (specialised && records && half && W == 16) {
        lds_auto = 28672;
    }
    l.lds_reserve = (unsigned)(tn.reduce_lds_reserve() < 0 ? lds_auto : tn.reduce_lds_reserve());
    const bool ntg = tn.nt_grads(), nts = tn.nt_state();

    switch (tn.reduce_small() ? 0u : W) {
    case 2: launch_w<2>(l, dtype, detect, ntg, nts); break;
    case 4: launch_w<4>(l, dtype, detect, ntg, nts); break;
    case 8: launch_w<8>(l, dtype, detect, ntg, nts); break;
    case 16: launch_w<16>(l, dtype, detect, ntg, nts); break;
    default:
        switch (dtype) {
        case XS_F16: launch_anyw<XS_F16>(l, W, detect); break;
        case XS_BF16: launch_anyw<XS_BF16>(l, W, detect); break;
        default: launch_anyw<XS_F32>(l, W, detect); break;
        }
    }
    XS_HIP_TRY(hipGetLastError());
    return XS_OK;
}

}  // namespace xs
