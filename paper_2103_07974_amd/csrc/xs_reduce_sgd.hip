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
//    front tight (a strided persistent grid measured 25 % slower on MI355X).
//  * The launch reserves LDS the kernel never touches, to cap how many wavefronts share a
//    compute unit: about 100-120 KB of loads in flight per compute unit is the optimum.
//  * Every stream is touched once, so loads and stores carry the non-temporal hint.
//  * fp16 gradients: lanes exchange their gradient sums through the LDS crossbar so that the
//    fp32 state accesses of a wavefront are contiguous (see the main loop).
//  * The only cross-lane quantity besides that is the overflow flag: a wavefront ballot, then
//    one atomic per wavefront that saw a non-finite gradient.
#include "xs_internal.h"

namespace xs {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 64;   // one wavefront per workgroup: finest dispatch grain

template <int N>
struct ReplicaPtrs {
    const void *p[N];
};

template <bool NT>
__device__ __forceinline__ u32x4 load_g(const u32x4 *p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}

template <bool NT>
__device__ __forceinline__ f32x4 load_s(const f32x4 *p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}

template <bool NT>
__device__ __forceinline__ void store_s(f32x4 *p, f32x4 v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

__device__ __forceinline__ float half_lo(uint32_t w)
{
    return (float)__builtin_bit_cast(_Float16, (uint16_t)(w & 0xffffu));
}
__device__ __forceinline__ float half_hi(uint32_t w)
{
    return (float)__builtin_bit_cast(_Float16, (uint16_t)(w >> 16));
}

// non-finite tests on raw bits: exponent field all ones
__device__ __forceinline__ bool nonfinite_f32(uint32_t w) { return (w & 0x7f800000u) == 0x7f800000u; }
__device__ __forceinline__ bool nonfinite_f16x2(uint32_t w)
{
    // adding one exponent step carries into bit 15 only from an all-ones exponent
    return (((w & 0x7c007c00u) + 0x04000400u) & 0x80008000u) != 0u;
}

__device__ __forceinline__ void sgd(float g_sum, float c, float &x, float &v, float lr, float mu,
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

// VEC elements per lane per trip: 4 (fp32 gradients) or 8 (fp16 gradients), so that
// every gradient load is 16 bytes wide.
template <int W, bool F16, bool DETECT, bool NTL, bool NTS, bool NTX, bool SHUF>
__global__ __launch_bounds__(kThreads) void reduce_sgd_kernel(
    ReplicaPtrs<W> reps, uint64_t n, const float *x_in, const float *v_in,
    float *x_out, float *v_out, float lr, float mu, float wd, float c,
    int32_t *found_inf)
{
    constexpr int VEC = F16 ? 8 : 4;
    constexpr int SV = VEC / 4;   // fp32 state vectors per gradient vector
    if (found_inf != nullptr && *(volatile int32_t *)found_inf != 0) return;

    const uint64_t nvec = n / VEC;
    const uint64_t stride = (uint64_t)gridDim.x * kThreads;
    bool bad = false;

    for (uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x; i < nvec; i += stride) {
        u32x4 g[W];
#pragma unroll
        for (int w = 0; w < W; ++w) g[w] = load_g<NTL>((const u32x4 *)reps.p[w] + i);
        // Which fp32 state vectors this lane updates.  fp32 gradients: the one under its
        // gradient vector.  fp16 gradients: a lane's 8 elements would be two neighbouring state
        // vectors, i.e. 32-byte strides per load instruction; in a full row of 64 lanes the
        // lanes instead take state vectors `lane` and `64 + lane` of the row, so that every
        // state load and store of the wavefront is one contiguous kilobyte, and the gradient
        // sums are moved to the owning lanes through the LDS crossbar afterwards.
        uint64_t sx[SV];
        bool shuffled = false;
        if constexpr (F16) {
            const uint64_t row0 = i - threadIdx.x;            // vector index of lane 0 (kThreads == 64)
            shuffled = SHUF && row0 + (kThreads - 1) < nvec;   // uniform: every lane of the row is live
            sx[0] = shuffled ? row0 * 2 + threadIdx.x : i * 2;
            sx[1] = shuffled ? row0 * 2 + kThreads + threadIdx.x : i * 2 + 1;
        } else {
            sx[0] = i;
        }
        f32x4 x[SV], v[SV];
#pragma unroll
        for (int k = 0; k < SV; ++k) {
            x[k] = load_s<NTX>((const f32x4 *)x_in + sx[k]);
            v[k] = load_s<NTX>((const f32x4 *)v_in + sx[k]);
        }
        float s[VEC];
#pragma unroll
        for (int w = 0; w < W; ++w) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t bits = g[w][q];
                if constexpr (F16) {
                    if constexpr (DETECT) bad |= nonfinite_f16x2(bits);
                    const float lo = half_lo(bits), hi = half_hi(bits);
                    if (w == 0) { s[2 * q] = lo; s[2 * q + 1] = hi; }
                    else { s[2 * q] = s[2 * q] + lo; s[2 * q + 1] = s[2 * q + 1] + hi; }
                } else {
                    if constexpr (DETECT) bad |= nonfinite_f32(bits);
                    const float f = __builtin_bit_cast(float, bits);
                    if (w == 0) s[q] = f;
                    else s[q] = s[q] + f;
                }
            }
        }
        if constexpr (F16) {
            if (shuffled) {
                // element 4L+e of the row sits in lane L>>1, slot (L&1)*4+e; element 256+4L+e in
                // lane 32+(L>>1), same slot
                const int src0 = (int)((threadIdx.x >> 1) << 2);
                const int src1 = (int)((32u + (threadIdx.x >> 1)) << 2);
                const bool odd = (threadIdx.x & 1u) != 0u;
                float t[VEC];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int lo = __builtin_bit_cast(int, s[e]), hi = __builtin_bit_cast(int, s[4 + e]);
                    const int a_lo = __builtin_amdgcn_ds_bpermute(src0, lo);
                    const int a_hi = __builtin_amdgcn_ds_bpermute(src0, hi);
                    const int b_lo = __builtin_amdgcn_ds_bpermute(src1, lo);
                    const int b_hi = __builtin_amdgcn_ds_bpermute(src1, hi);
                    t[e] = __builtin_bit_cast(float, odd ? a_hi : a_lo);
                    t[4 + e] = __builtin_bit_cast(float, odd ? b_hi : b_lo);
                }
#pragma unroll
                for (int e = 0; e < VEC; ++e) s[e] = t[e];
            }
        }
#pragma unroll
        for (int k = 0; k < SV; ++k) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float xe = x[k][q], ve = v[k][q];
                sgd(s[4 * k + q], c, xe, ve, lr, mu, wd);
                x[k][q] = xe;
                v[k][q] = ve;
            }
            store_s<NTS>((f32x4 *)x_out + sx[k], x[k]);
            store_s<NTS>((f32x4 *)v_out + sx[k], v[k]);
        }
    }

    // ragged tail: fewer than VEC elements, one lane each, in workgroup 0
    const uint32_t rem = (uint32_t)(n - nvec * VEC);
    if (blockIdx.x == 0 && threadIdx.x < rem) {
        const uint64_t j = nvec * VEC + threadIdx.x;
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < W; ++w) {
            float f;
            if constexpr (F16) {
                const uint16_t h = ((const uint16_t *)reps.p[w])[j];
                if constexpr (DETECT) bad |= (h & 0x7c00u) == 0x7c00u;
                f = (float)__builtin_bit_cast(_Float16, h);
            } else {
                const uint32_t b = ((const uint32_t *)reps.p[w])[j];
                if constexpr (DETECT) bad |= nonfinite_f32(b);
                f = __builtin_bit_cast(float, b);
            }
            s = (w == 0) ? f : s + f;
        }
        float xe = x_in[j], ve = v_in[j];
        sgd(s, c, xe, ve, lr, mu, wd);
        x_out[j] = xe;
        v_out[j] = ve;
    }

    if constexpr (DETECT) {
        // wavefront-level vote, then at most one atomic per wavefront
        if (__builtin_amdgcn_ballot_w64(bad) != 0ull && (threadIdx.x & 63u) == 0u)
            atomicOr(found_inf, 1);
    }
}

// Any W up to XS_MAX_REPLICAS: replica loop with a run-time trip count, four loads
// in flight at a time.  Same arithmetic and order as the specialised kernels.
template <bool F16, bool DETECT>
__global__ __launch_bounds__(kThreads) void reduce_sgd_anyw_kernel(
    ReplicaPtrs<XS_MAX_REPLICAS> reps, uint32_t W, uint64_t n, const float *x_in,
    const float *v_in, float *x_out, float *v_out, float lr,
    float mu, float wd, float c, int32_t *found_inf)
{
    constexpr int VEC = F16 ? 8 : 4;
    if (found_inf != nullptr && *(volatile int32_t *)found_inf != 0) return;
    const uint64_t stride = (uint64_t)gridDim.x * kThreads * VEC;
    bool bad = false;
    // element-granular with a guarded last vector: simple, and only used for unusual W
    for (uint64_t base = ((uint64_t)blockIdx.x * kThreads + threadIdx.x) * VEC; base < n;
         base += stride) {
        const int cnt = (n - base) < (uint64_t)VEC ? (int)(n - base) : VEC;
        float s[VEC];
        if (cnt == VEC) {
            const uint64_t byte_off = base * (F16 ? 2 : 4);
            {
                const u32x4 g = *(const u32x4 *)((const char *)reps.p[0] + byte_off);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint32_t bits = g[q];   // a scalar copy: bit_cast of a vector element misreads
                    if constexpr (F16) {
                        if constexpr (DETECT) bad |= nonfinite_f16x2(bits);
                        s[2 * q] = half_lo(bits);
                        s[2 * q + 1] = half_hi(bits);
                    } else {
                        if constexpr (DETECT) bad |= nonfinite_f32(bits);
                        s[q] = __builtin_bit_cast(float, bits);
                    }
                }
            }
#pragma unroll 4
            for (uint32_t w = 1; w < W; ++w) {
                const u32x4 g = *(const u32x4 *)((const char *)reps.p[w] + byte_off);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint32_t bits = g[q];
                    if constexpr (F16) {
                        if constexpr (DETECT) bad |= nonfinite_f16x2(bits);
                        s[2 * q] = s[2 * q] + half_lo(bits);
                        s[2 * q + 1] = s[2 * q + 1] + half_hi(bits);
                    } else {
                        if constexpr (DETECT) bad |= nonfinite_f32(bits);
                        s[q] = s[q] + __builtin_bit_cast(float, bits);
                    }
                }
            }
        } else {
            for (int e = 0; e < cnt; ++e) {
                float acc = 0.f;
                for (uint32_t w = 0; w < W; ++w) {
                    float f;
                    if constexpr (F16) {
                        const uint16_t h = ((const uint16_t *)reps.p[w])[base + e];
                        if constexpr (DETECT) bad |= (h & 0x7c00u) == 0x7c00u;
                        f = (float)__builtin_bit_cast(_Float16, h);
                    } else {
                        const uint32_t b = ((const uint32_t *)reps.p[w])[base + e];
                        if constexpr (DETECT) bad |= nonfinite_f32(b);
                        f = __builtin_bit_cast(float, b);
                    }
                    acc = (w == 0) ? f : acc + f;
                }
                s[e] = acc;
            }
        }
        for (int e = 0; e < cnt; ++e) {
            float xe = x_in[base + e], ve = v_in[base + e];
            sgd(s[e], c, xe, ve, lr, mu, wd);
            x_out[base + e] = xe;
            v_out[base + e] = ve;
        }
    }
    if constexpr (DETECT) {
        if (__builtin_amdgcn_ballot_w64(bad) != 0ull && (threadIdx.x & 63u) == 0u)
            atomicOr(found_inf, 1);
    }
}

// ---- dispatch --------------------------------------------------------------------
struct LaunchArgs {
    const void *const *replicas;
    uint64_t n;
    const float *x_in, *v_in;
    float *x_out, *v_out;
    float lr, mu, wd, c;
    int32_t *found_inf;
    dim3 grid;
    unsigned lds_reserve;
    bool shuffle;
    hipStream_t stream;
};

template <int W, bool F16, bool DETECT, bool NTL, bool NTS, bool NTX>
static void launch_one(const LaunchArgs &a)
{
    ReplicaPtrs<W> r;
    for (int w = 0; w < W; ++w) r.p[w] = a.replicas[w];
    if (F16 && a.shuffle)
        hipLaunchKernelGGL((reduce_sgd_kernel<W, F16, DETECT, NTL, NTS, NTX, F16>), a.grid,
                           dim3(kThreads), a.lds_reserve, a.stream, r, a.n, a.x_in, a.v_in, a.x_out,
                           a.v_out, a.lr, a.mu, a.wd, a.c, a.found_inf);
    else
        hipLaunchKernelGGL((reduce_sgd_kernel<W, F16, DETECT, NTL, NTS, NTX, false>), a.grid,
                           dim3(kThreads), a.lds_reserve, a.stream, r, a.n, a.x_in, a.v_in, a.x_out,
                           a.v_out, a.lr, a.mu, a.wd, a.c, a.found_inf);
}

template <int W, bool F16, bool DETECT>
static void launch_nt(const LaunchArgs &a, int nt)
{
    switch (nt & 7) {
    case 0: launch_one<W, F16, DETECT, false, false, false>(a); break;
    case 1: launch_one<W, F16, DETECT, true, false, false>(a); break;
    case 2: launch_one<W, F16, DETECT, false, true, false>(a); break;
    case 3: launch_one<W, F16, DETECT, true, true, false>(a); break;
    case 4: launch_one<W, F16, DETECT, false, false, true>(a); break;
    case 5: launch_one<W, F16, DETECT, true, false, true>(a); break;
    case 6: launch_one<W, F16, DETECT, false, true, true>(a); break;
    default: launch_one<W, F16, DETECT, true, true, true>(a); break;
    }
}

template <int W>
static void launch_w(const LaunchArgs &a, bool f16, bool detect, int nt)
{
    if (f16) { if (detect) launch_nt<W, true, true>(a, nt); else launch_nt<W, true, false>(a, nt); }
    else     { if (detect) launch_nt<W, false, true>(a, nt); else launch_nt<W, false, false>(a, nt); }
}

template <bool F16, bool DETECT>
static void launch_anyw(const LaunchArgs &a, uint32_t W)
{
    ReplicaPtrs<XS_MAX_REPLICAS> r;
    for (uint32_t w = 0; w < XS_MAX_REPLICAS; ++w) r.p[w] = w < W ? a.replicas[w] : nullptr;
    hipLaunchKernelGGL((reduce_sgd_anyw_kernel<F16, DETECT>), a.grid, dim3(kThreads), a.lds_reserve, a.stream,
                       r, W, a.n, a.x_in, a.v_in, a.x_out, a.v_out, a.lr, a.mu, a.wd, a.c,
                       a.found_inf);
}

int launch_reduce_sgd(const void *const *replicas, uint32_t W, int dtype, uint64_t n,
                      const float *x_in, const float *v_in, float *x_out, float *v_out,
                      const xs_sgd_hparams &hp, int32_t *found_inf, bool detect,
                      hipStream_t stream)
{
    const int cus = compute_units();
    if (cus < 0) return cus;
    const bool f16 = dtype == XS_F16;
    const uint64_t vec = f16 ? 8 : 4;
    uint64_t blocks = (n / vec + kThreads - 1) / kThreads;
    if (blocks == 0) blocks = 1;   // tail only
    if (g_tuning.reduce_wg_per_cu > 0) {
        const uint64_t cap = (uint64_t)cus * (uint64_t)g_tuning.reduce_wg_per_cu;
        if (blocks > cap) blocks = cap;
    }
    if (g_tuning.reduce_max_wg > 0 && blocks > (uint64_t)g_tuning.reduce_max_wg)
        blocks = (uint64_t)g_tuning.reduce_max_wg;
    if (blocks > 0x7fffffffull) blocks = 0x7fffffffull;   // the loop covers the rest

    LaunchArgs a;
    a.replicas = replicas;
    a.n = n;
    a.x_in = x_in; a.v_in = v_in; a.x_out = x_out; a.v_out = v_out;
    a.lr = hp.lr; a.mu = hp.momentum; a.wd = hp.weight_decay;
    // one constant for averaging and loss scale: inv_loss_scale * (1/W), rounded to fp32 twice
    volatile float one_over_w = 1.0f / (float)W;
    a.c = hp.inv_loss_scale * one_over_w;
    a.found_inf = found_inf;
    a.grid = dim3((unsigned)blocks);
    a.stream = stream;
    // Measured on MI355X: the pass is fastest with about 100-120 KB of loads in flight per
    // compute unit; more wavefronts than that only disorder the DRAM access stream.  The
    // LDS reservation (unused by the kernel) caps residency at 10 one-wave workgroups per
    // compute unit for fp32 gradients (12 loads per lane) and 5 for fp16 (20 loads per lane).
    // Every stream is touched once per lane -> all non-temporal (fp16 without the lane
    // exchange: a lane's two state vectors share cache lines with its neighbours', so state
    // loads stay cacheable there).
    const int lds_auto = f16 ? 32768 : 16384;
    a.lds_reserve = (unsigned)(g_tuning.reduce_lds_reserve < 0 ? lds_auto : g_tuning.reduce_lds_reserve);
    a.shuffle = g_tuning.f16_state_shuffle != 0;
    const int ntl = g_tuning.nt_loads < 0 ? 1 : g_tuning.nt_loads;
    const int nts = g_tuning.nt_stores < 0 ? 1 : g_tuning.nt_stores;
    const int ntx = g_tuning.nt_state_loads < 0 ? ((f16 && !a.shuffle) ? 0 : 1) : g_tuning.nt_state_loads;
    const int nt = (ntl ? 1 : 0) | (nts ? 2 : 0) | (ntx ? 4 : 0);

    switch (W) {
    case 1: launch_w<1>(a, f16, detect, nt); break;
    case 2: launch_w<2>(a, f16, detect, nt); break;
    case 4: launch_w<4>(a, f16, detect, nt); break;
    case 8: launch_w<8>(a, f16, detect, nt); break;
    case 16: launch_w<16>(a, f16, detect, nt); break;
    default:
        if (f16) { if (detect) launch_anyw<true, true>(a, W); else launch_anyw<true, false>(a, W); }
        else     { if (detect) launch_anyw<false, true>(a, W); else launch_anyw<false, false>(a, W); }
    }
    XS_HIP_TRY(hipGetLastError());
    return XS_OK;
}

}  // namespace xs
