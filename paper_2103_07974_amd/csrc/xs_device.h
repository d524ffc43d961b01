// Device-side pieces shared by the reduce kernels of libxs.so (bucket form and gathering
// form): gradient element types, the update arithmetic, conversions, cache-hinted accesses.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "xs.h"

namespace xs {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(1))) unsigned char gbyte;
typedef __attribute__((address_space(1))) u32x4 gvec;

constexpr int kWave = 64;
constexpr int kMaxReduceThreads = 256;   // reduce kernels: 1, 2 or 4 wavefronts per workgroup

// ---- gradient element types ------------------------------------------------------------
// GT = XS_F32 (0): one element per 32-bit word.  XS_F16 (1) / XS_BF16 (2): two per word.
template <int GT>
struct Grad;

template <>
struct Grad<0> {
    static constexpr int ES = 4;
    static constexpr bool HALF = false;
    static __device__ __forceinline__ float lo(uint32_t w) { return __builtin_bit_cast(float, w); }
    static __device__ __forceinline__ float hi(uint32_t w) { return 0.f; }
    static __device__ __forceinline__ bool nonfinite(uint32_t w) { return (w & 0x7f800000u) == 0x7f800000u; }
    static __device__ __forceinline__ bool nonfinite_elem(uint32_t e) { return nonfinite(e); }
};

template <>
struct Grad<1> {   // IEEE binary16
    static constexpr int ES = 2;
    static constexpr bool HALF = true;
    static __device__ __forceinline__ float lo(uint32_t w)
    {
        return (float)__builtin_bit_cast(_Float16, (uint16_t)(w & 0xffffu));
    }
    static __device__ __forceinline__ float hi(uint32_t w)
    {
        return (float)__builtin_bit_cast(_Float16, (uint16_t)(w >> 16));
    }
    // adding one exponent step carries into bit 15 only from an all-ones exponent
    static __device__ __forceinline__ bool nonfinite(uint32_t w)
    {
        return (((w & 0x7c007c00u) + 0x04000400u) & 0x80008000u) != 0u;
    }
    static __device__ __forceinline__ bool nonfinite_elem(uint32_t e) { return (e & 0x7c00u) == 0x7c00u; }
};

template <>
struct Grad<2> {   // bfloat16: the upper half of an IEEE single
    static constexpr int ES = 2;
    static constexpr bool HALF = true;
    static __device__ __forceinline__ float lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
    static __device__ __forceinline__ float hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xffff0000u); }
    static __device__ __forceinline__ bool nonfinite(uint32_t w)
    {
        return (((w & 0x7f807f80u) + 0x00800080u) & 0x80008000u) != 0u;
    }
    static __device__ __forceinline__ bool nonfinite_elem(uint32_t e) { return (e & 0x7f80u) == 0x7f80u; }
};

// ---- Algorithm 1, "Model Update": d = g + wd*x; v = mu*v + d; x = x - lr*v ----------------
// g = g_sum * c with c = inv_loss_scale * (1/W); every operation rounded to fp32 separately.
__device__ __forceinline__ void sgd_update(float g_sum, float c, float &x, float &v, float lr,
                                           float mu, float wd)
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

// ---- hyper-parameters per tensor ----------------------------------------------------------
// One 16-byte record (lr, momentum, weight decay, unused) per tensor; record t governs the
// bucket elements offsets[t] .. offsets[t+1]-1 (tensor t and the padding behind it).
struct TensorHp {
    const f32x4 *rec;          // device [n_tensors], or nullptr: one triple for the bucket
    const uint64_t *offsets;   // device [n_tensors + 1]
    const uint32_t *row_first; // device [n_rows]: tensor whose segment holds a row's first element
    uint32_t n_tensors;
};

// the tensor whose segment holds bucket element j; t must not be past it (forward search)
__device__ __forceinline__ void seek_tensor(const TensorHp &h, uint32_t &t, uint64_t j)
{
    while (t + 1 < h.n_tensors && h.offsets[t + 1] <= j) ++t;
}

__device__ __forceinline__ void sgd_update4(const float *s, float c, f32x4 &x, f32x4 &v, f32x4 rec)
{
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        float xe = x[q], ve = v[q];
        sgd_update(s[q], c, xe, ve, rec[0], rec[1], rec[2]);
        x[q] = xe;
        v[q] = ve;
    }
}

// One 4-element state vector starting at bucket element j, which may span several segments
// (tight layouts).  t as for seek_tensor; it is left at the tensor of the vector's first element.
__device__ __forceinline__ void sgd_update4_per_tensor(const TensorHp &h, uint32_t &t, uint64_t j,
                                                       const float *s, float c, f32x4 &x, f32x4 &v)
{
    seek_tensor(h, t, j);
    if (j + 4 <= h.offsets[t + 1]) {
        sgd_update4(s, c, x, v, h.rec[t]);
        return;
    }
    uint32_t te = t;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        seek_tensor(h, te, j + q);
        const f32x4 rec = h.rec[te];
        float xe = x[q], ve = v[q];
        sgd_update(s[q], c, xe, ve, rec[0], rec[1], rec[2]);
        x[q] = xe;
        v[q] = ve;
    }
}

// ---- fp32 -> half-precision copies of the parameters (round to nearest even) ---------------
__device__ __forceinline__ uint32_t to_f16_bits(float x)
{
    return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)x);
}
__device__ __forceinline__ uint32_t to_bf16_bits(float x)
{
    uint32_t b = __builtin_bit_cast(uint32_t, x);
    if ((b & 0x7fffffffu) > 0x7f800000u) return (b >> 16) | 0x0040u;   // NaN stays NaN
    b += 0x7fffu + ((b >> 16) & 1u);
    return b >> 16;
}
// four fp32 values -> four half-precision values in two words; dtype is XS_F16 or XS_BF16
__device__ __forceinline__ u32x2 to_half4(f32x4 x, int dtype)
{
    u32x2 r;
    if (dtype == 1) {
        r[0] = to_f16_bits(x[0]) | (to_f16_bits(x[1]) << 16);
        r[1] = to_f16_bits(x[2]) | (to_f16_bits(x[3]) << 16);
    } else {
        r[0] = to_bf16_bits(x[0]) | (to_bf16_bits(x[1]) << 16);
        r[1] = to_bf16_bits(x[2]) | (to_bf16_bits(x[3]) << 16);
    }
    return r;
}
__device__ __forceinline__ uint16_t to_half1(float x, int dtype)
{
    return (uint16_t)(dtype == 1 ? to_f16_bits(x) : to_bf16_bits(x));
}

// ---- cache-hinted 16-byte accesses --------------------------------------------------------
template <bool NT>
__device__ __forceinline__ u32x4 load16(const u32x4 *p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}
template <bool NT>
__device__ __forceinline__ f32x4 load16f(const f32x4 *p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}
template <bool NT>
__device__ __forceinline__ void store16f(f32x4 *p, f32x4 v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}
template <bool NT>
__device__ __forceinline__ void store8(u32x2 *p, u32x2 v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// ---- element-aligned vector accesses to per-layer tensors and views --------------------------
template <int ALIGN>
struct __attribute__((packed, aligned(ALIGN))) LooseVec16 {
    u32x4 v;
};
struct __attribute__((packed, aligned(2))) LooseVec8 {
    u32x2 v;
};

// element-aligned 16-byte load from a gradient tensor (non-temporal when it happens to be aligned)
template <int ES>
__device__ __forceinline__ u32x4 load_tensor_vec(const gbyte *p)
{
    if (((uintptr_t)p & 15u) == 0) return __builtin_nontemporal_load((const gvec *)p);
    return ((const __attribute__((address_space(1))) LooseVec16<ES> *)p)->v;
}

// four updated parameters to a per-layer view: fp32 (16 bytes) or half precision (8 bytes)
__device__ __forceinline__ void store_view4(gbyte *view, uint64_t elem, f32x4 x, int view_dtype)
{
    if (view_dtype == XS_F32) {
        gbyte *p = view + elem * 4;
        const u32x4 bits = __builtin_bit_cast(u32x4, x);
        if (((uintptr_t)p & 15u) == 0) __builtin_nontemporal_store(bits, (gvec *)p);
        else ((__attribute__((address_space(1))) LooseVec16<4> *)p)->v = bits;
    } else {
        ((__attribute__((address_space(1))) LooseVec8 *)(view + elem * 2))->v = to_half4(x, view_dtype);
    }
}
__device__ __forceinline__ void store_view1(gbyte *view, uint64_t elem, float x, int view_dtype)
{
    if (view_dtype == XS_F32) *(__attribute__((address_space(1))) float *)(view + elem * 4) = x;
    else *(__attribute__((address_space(1))) uint16_t *)(view + elem * 2) = to_half1(x, view_dtype);
}

// ---- fp16/bf16 gradients: move gradient sums to the lanes that own the state vectors ---------
// Before: lane L holds s[0..7] = sums of row elements 8L..8L+7.  After: s[0..3] = elements
// 4L..4L+3 and s[4..7] = elements 256+4L..256+4L+3, i.e. the lane's state vectors `L` and
// `64+L` of the row.  Element 4L+e sits in lane L>>1, slot (L&1)*4+e; element 256+4L+e in lane
// 32+(L>>1), same slot.  All 64 lanes must be active.
__device__ __forceinline__ void exchange_half_row(float (&s)[8])
{
    const uint32_t lane = threadIdx.x & 63u;
    const int src0 = (int)((lane >> 1) << 2);
    const int src1 = (int)((32u + (lane >> 1)) << 2);
    const bool odd = (lane & 1u) != 0u;
    float t[8];
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
    for (int e = 0; e < 8; ++e) s[e] = t[e];
}

// ---- overflow flag ---------------------------------------------------------------------------
// Wavefront-level vote, then at most one atomic per wavefront that saw a non-finite value -
// and none once the flag is up: with many such wavefronts (0.1 % of the elements non-finite
// puts one in nearly every workgroup) the atomics on the one address would otherwise queue up
// behind each other in L2.
__device__ __forceinline__ void raise_flag_if(bool bad, int32_t *found_inf)
{
    if (__builtin_amdgcn_ballot_w64(bad) != 0ull && (threadIdx.x & 63u) == 0u) {
        if (*(volatile int32_t *)found_inf == 0) atomicOr(found_inf, 1);
    }
}

// Accumulate one replica's 16-byte gradient vector into the per-lane sums, in worker order.
template <int GT, bool DETECT>
__device__ __forceinline__ void accumulate(const u32x4 &g, bool first, float *s, bool &bad)
{
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint32_t bits = g[q];   // a scalar copy: bit_cast of a vector element misreads
        if constexpr (DETECT) bad |= Grad<GT>::nonfinite(bits);
        if constexpr (Grad<GT>::HALF) {
            const float lo = Grad<GT>::lo(bits), hi = Grad<GT>::hi(bits);
            s[2 * q] = first ? lo : s[2 * q] + lo;
            s[2 * q + 1] = first ? hi : s[2 * q + 1] + hi;
        } else {
            const float f = Grad<GT>::lo(bits);
            s[q] = first ? f : s[q] + f;
        }
    }
}

}  // namespace xs
