// Helpers of bench.py that are NOT part of libxs.so: the compute side of the crossover
// measurements (arXiv 2103.07974, Section 2.1: one task computes while the other task's
// gradients are synchronised) and the stream set-up those measurements need.
//
//   bs_gemm_*        the configured compute stand-in, a chain of bf16 GEMMs, issued through
//                    hipBLASLt's C interface with an explicit choice among the algorithms its
//                    heuristic offers (the library's first choice launches exactly one
//                    workgroup per compute unit, which cannot be placed on a stream that owns
//                    fewer compute units)
//   bs_alu           an arithmetic-only kernel of ordinary occupancy and no memory traffic
//   bs_stream_*      streams restricted to a set of compute units (hipExtStreamCreateWithCUMask)
//   bs_census        which compute units the workgroups of a stream actually land on
//   bs_copy / bs_mix / bs_read  plain streaming kernels (1:1 copy; 10 reads : 2 writes; 10 reads) that give the
//                    chip's attainable HBM rate for the access mix of pack/unpack and of the
//                    fused reduce + SGD, beside which the library's kernels are reported
#include <hip/hip_runtime.h>
#include <hipblaslt/hipblaslt.h>
#include <stdarg.h>
#include <stdint.h>
#include <stdio.h>

#include <new>
#include <vector>

namespace {

thread_local char t_error[512] = "";

int fail(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(t_error, sizeof t_error, fmt, ap);
    va_end(ap);
    return -1;
}

#define BS_HIP(expr)                                                                     \
    do {                                                                                 \
        hipError_t e_ = (expr);                                                          \
        if (e_ != hipSuccess) return fail("%s: %s", #expr, hipGetErrorString(e_));       \
    } while (0)
#define BS_LT(expr)                                                                      \
    do {                                                                                 \
        hipblasStatus_t s_ = (expr);                                                     \
        if (s_ != HIPBLAS_STATUS_SUCCESS) return fail("%s: hipblas status %d", #expr, (int)s_); \
    } while (0)

__global__ __launch_bounds__(256) void alu_kernel(float *sink, uint32_t iters, float a, float b)
{
    float x0 = threadIdx.x * 1e-3f, x1 = x0 + 1, x2 = x0 + 2, x3 = x0 + 3, x4 = x0 + 4, x5 = x0 + 5,
          x6 = x0 + 6, x7 = x0 + 7;
    for (uint32_t i = 0; i < iters; ++i) {
        x0 = x0 * a + b; x1 = x1 * a + b; x2 = x2 * a + b; x3 = x3 * a + b;
        x4 = x4 * a + b; x5 = x5 * a + b; x6 = x6 * a + b; x7 = x7 * a + b;
    }
    const float s = x0 + x1 + x2 + x3 + x4 + x5 + x6 + x7;
    if (s == 1.2345f) sink[threadIdx.x] = s;   // keeps the loop alive; practically never taken
}

// One wavefront per workgroup reports where it runs: XCC_ID (hardware register 20, bits 3:0)
// and HW_ID (register 4: CU_ID bits 11:8, SH_ID bit 12, SE_ID bits 15:13), then idles for
// `spin` ticks of the clock counter (at most 2^20) so that the workgroups of one launch spread over every compute unit the
// stream may use instead of all retiring on the first few.
__global__ __launch_bounds__(64) void census_kernel(uint32_t *out, uint32_t spin)
{
    const uint32_t xcc = __builtin_amdgcn_s_getreg(20 | (3 << 11)) & 0xfu;
    const uint32_t hw = __builtin_amdgcn_s_getreg(4 | (31 << 11));
    const uint64_t t0 = __builtin_readcyclecounter();
    while (__builtin_readcyclecounter() - t0 < spin) {}
    if (threadIdx.x == 0)
        out[blockIdx.x] = (xcc << 16) | (((hw >> 13) & 7u) << 8) | (((hw >> 12) & 1u) << 4) | ((hw >> 8) & 0xfu);
}

// The same with a chosen register footprint: the empty asm statement names the highest
// vector register as clobbered, which makes the kernel allocate V + 1 registers per lane
// without using them.  Each workgroup also records when it started (clock counter ticks).
#define BS_FOOTPRINT_KERNEL(V)                                                              \
    __global__ __launch_bounds__(256) void footprint_v##V(uint32_t *out, uint64_t *t_start,   \
                                                          uint32_t spin)                      \
    {                                                                                       \
        asm volatile("" ::: "v" #V);                                                        \
        const uint64_t t0 = __builtin_readcyclecounter();                                   \
        while (__builtin_readcyclecounter() - t0 < spin) {}                                 \
        if (threadIdx.x == 0) {                                                             \
            const uint32_t xcc = __builtin_amdgcn_s_getreg(20 | (3 << 11)) & 0xfu;          \
            const uint32_t hw = __builtin_amdgcn_s_getreg(4 | (31 << 11));                  \
            out[blockIdx.x] = (xcc << 16) | (((hw >> 13) & 7u) << 8) | (((hw >> 12) & 1u) << 4) | ((hw >> 8) & 0xfu); \
            t_start[blockIdx.x] = t0;                                                       \
        }                                                                                   \
    }
BS_FOOTPRINT_KERNEL(23)
BS_FOOTPRINT_KERNEL(47)
BS_FOOTPRINT_KERNEL(63)
BS_FOOTPRINT_KERNEL(71)
BS_FOOTPRINT_KERNEL(95)
BS_FOOTPRINT_KERNEL(127)
BS_FOOTPRINT_KERNEL(191)
BS_FOOTPRINT_KERNEL(255)

typedef float f32x4 __attribute__((ext_vector_type(4)));

// 1:1 streaming copy, one 16-byte vector per lane, one-wavefront workgroups in address order
__global__ __launch_bounds__(64) void copy_kernel(const f32x4 *src, f32x4 *dst, uint64_t nvec)
{
    const uint64_t i = (uint64_t)blockIdx.x * 64 + threadIdx.x;
    if (i < nvec) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

struct Mix10 {
    const f32x4 *r[10];
};
// 10 streams read, 2 written, per 16-byte vector: the access mix of the fused reduce + SGD at
// W = 8 fp32 with the arithmetic reduced to adds
__global__ __launch_bounds__(64) void mix_kernel(Mix10 m, f32x4 *o0, f32x4 *o1, uint64_t nvec)
{
    const uint64_t i = (uint64_t)blockIdx.x * 64 + threadIdx.x;
    if (i >= nvec) return;
    f32x4 g[10];
#pragma unroll
    for (int k = 0; k < 10; ++k) g[k] = __builtin_nontemporal_load(m.r[k] + i);
    f32x4 s = g[0];
#pragma unroll
    for (int k = 1; k < 8; ++k) s = s + g[k];
    __builtin_nontemporal_store(s + g[8], o0 + i);
    __builtin_nontemporal_store(s + g[9], o1 + i);
}

// 10 streams read, nothing written (a wavefront that finds an all-ones sum, which random data
// never gives, writes one word, so that the loads cannot be dropped): the read-only limit
__global__ __launch_bounds__(64) void read_kernel(Mix10 m, uint32_t *sink, uint64_t nvec)
{
    const uint64_t i = (uint64_t)blockIdx.x * 64 + threadIdx.x;
    if (i >= nvec) return;
    f32x4 g[10];
#pragma unroll
    for (int k = 0; k < 10; ++k) g[k] = __builtin_nontemporal_load(m.r[k] + i);
    f32x4 s = g[0];
#pragma unroll
    for (int k = 1; k < 10; ++k) s = s + g[k];
    if (__float_as_uint(s[0]) == 0xffffffffu && __float_as_uint(s[3]) == 0xffffffffu) sink[0] = 1u;
}

struct Gemm {
    hipblasLtHandle_t lt = nullptr;
    hipblasLtMatmulDesc_t desc = nullptr;
    hipblasLtMatrixLayout_t layout = nullptr;
    hipblasLtMatmulPreference_t pref = nullptr;
    std::vector<hipblasLtMatmulHeuristicResult_t> algos;
    void *workspace = nullptr;
    size_t workspace_bytes = 0;
    uint32_t n = 0;
};

}  // namespace

extern "C" const char *bs_last_error(void) { return t_error; }

extern "C" int bs_alu(uint32_t workgroups, uint32_t iters, float *sink, void *stream)
{
    if (!sink || workgroups == 0 || workgroups > (1u << 20)) return fail("bs_alu: bad argument");
    hipLaunchKernelGGL(alu_kernel, dim3(workgroups), dim3(256), 0, (hipStream_t)stream, sink, iters,
                       1.0000001f, 1e-7f);
    BS_HIP(hipGetLastError());
    return 0;
}

// out: device, n_workgroups words; word = xcc << 16 | se << 8 | sh << 4 | cu
extern "C" int bs_census(uint32_t *out, uint32_t n_workgroups, uint32_t spin, void *stream)
{
    if (!out || n_workgroups == 0 || n_workgroups > (1u << 20) || spin > (1u << 20))
        return fail("bs_census: bad argument");
    hipLaunchKernelGGL(census_kernel, dim3(n_workgroups), dim3(64), 0, (hipStream_t)stream, out, spin);
    BS_HIP(hipGetLastError());
    return 0;
}

// A launch of n_workgroups workgroups of `threads` lanes (64..256) that each allocate `vgprs`
// registers per lane (24, 48, 64, 72, 96, 128, 192 or 256) and lds_bytes of LDS, idle for `spin`
// ticks and record their place (as bs_census) and start tick: which footprint fits beside
// the workgroups of another kernel.
extern "C" int bs_footprint(uint32_t *out, uint64_t *t_start, uint32_t n_workgroups, uint32_t threads,
                            uint32_t lds_bytes, uint32_t vgprs, uint32_t spin, void *stream)
{
    if (!out || !t_start || n_workgroups == 0 || n_workgroups > (1u << 20) || spin > (1u << 20) ||
        threads < 64 || threads > 256 || (threads & 63u) || lds_bytes > 160 * 1024)
        return fail("bs_footprint: bad argument");
    void (*k)(uint32_t *, uint64_t *, uint32_t) = nullptr;
    switch (vgprs) {
    case 24: k = footprint_v23; break;
    case 48: k = footprint_v47; break;
    case 64: k = footprint_v63; break;
    case 72: k = footprint_v71; break;
    case 96: k = footprint_v95; break;
    case 128: k = footprint_v127; break;
    case 192: k = footprint_v191; break;
    case 256: k = footprint_v255; break;
    default: return fail("bs_footprint: no kernel with %u registers", vgprs);
    }
    if (lds_bytes > 65536)
        BS_HIP(hipFuncSetAttribute((const void *)k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes));
    hipLaunchKernelGGL(k, dim3(n_workgroups), dim3(threads), lds_bytes, (hipStream_t)stream, out, t_start, spin);
    BS_HIP(hipGetLastError());
    return 0;
}

// words[i] bit b = compute unit 32 i + b of the device's mask numbering; default priority
extern "C" int bs_stream_create_masked(const uint32_t *words, uint32_t n_words, void **stream_out)
{
    if (!words || !stream_out || n_words == 0) return fail("bs_stream_create_masked: bad argument");
    hipStream_t s = nullptr;
    BS_HIP(hipExtStreamCreateWithCUMask(&s, n_words, words));
    *stream_out = (void *)s;
    return 0;
}

extern "C" int bs_stream_destroy(void *stream)
{
    BS_HIP(hipStreamDestroy((hipStream_t)stream));
    return 0;
}

extern "C" int bs_copy(const void *src, void *dst, uint64_t bytes, uint32_t lds_reserve, void *stream)
{
    if (!src || !dst || (bytes & 15u) || lds_reserve > 160 * 1024) return fail("bs_copy: bad argument");
    const uint64_t nvec = bytes / 16, blocks = (nvec + 63) / 64;
    if (blocks == 0) return 0;
    if (blocks > 0x7fffffffull) return fail("bs_copy: too large");
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(64), lds_reserve, (hipStream_t)stream,
                       (const f32x4 *)src, (f32x4 *)dst, nvec);
    BS_HIP(hipGetLastError());
    return 0;
}

// reads: host array of 10 device pointers; every buffer `bytes` long
extern "C" int bs_mix(const void *const *reads, void *out0, void *out1, uint64_t bytes,
                      uint32_t lds_reserve, void *stream)
{
    if (!reads || !out0 || !out1 || (bytes & 15u) || lds_reserve > 160 * 1024) return fail("bs_mix: bad argument");
    Mix10 m;
    for (int k = 0; k < 10; ++k) {
        if (!reads[k]) return fail("bs_mix: reads[%d] is NULL", k);
        m.r[k] = (const f32x4 *)reads[k];
    }
    const uint64_t nvec = bytes / 16, blocks = (nvec + 63) / 64;
    if (blocks == 0) return 0;
    if (blocks > 0x7fffffffull) return fail("bs_mix: too large");
    hipLaunchKernelGGL(mix_kernel, dim3((unsigned)blocks), dim3(64), lds_reserve, (hipStream_t)stream, m,
                       (f32x4 *)out0, (f32x4 *)out1, nvec);
    BS_HIP(hipGetLastError());
    return 0;
}

// reads: host array of 10 device pointers; every buffer `bytes` long; sink: one device word
extern "C" int bs_read(const void *const *reads, void *sink, uint64_t bytes, uint32_t lds_reserve, void *stream)
{
    if (!reads || !sink || (bytes & 15u) || lds_reserve > 160 * 1024) return fail("bs_read: bad argument");
    Mix10 m;
    for (int k = 0; k < 10; ++k) {
        if (!reads[k]) return fail("bs_read: reads[%d] is NULL", k);
        m.r[k] = (const f32x4 *)reads[k];
    }
    const uint64_t nvec = bytes / 16, blocks = (nvec + 63) / 64;
    if (blocks == 0) return 0;
    if (blocks > 0x7fffffffull) return fail("bs_read: too large");
    hipLaunchKernelGGL(read_kernel, dim3((unsigned)blocks), dim3(64), lds_reserve, (hipStream_t)stream, m,
                       (uint32_t *)sink, nvec);
    BS_HIP(hipGetLastError());
    return 0;
}

// Square bf16 GEMM C = A @ B (row-major, fp32 accumulation), n x n each, with up to
// max_algos of the algorithms hipBLASLt's heuristic returns for it, best estimate first.
extern "C" int bs_gemm_create(uint32_t n, uint32_t max_algos, uint64_t workspace_bytes, void **out)
{
    if (!out || n == 0 || max_algos == 0 || max_algos > 4096) return fail("bs_gemm_create: bad argument");
    *out = nullptr;
    Gemm *g = new (std::nothrow) Gemm();
    if (!g) return fail("bs_gemm_create: out of host memory");
    g->n = n;
    g->workspace_bytes = (size_t)workspace_bytes;
    int rc = [&]() -> int {
        BS_LT(hipblasLtCreate(&g->lt));
        BS_LT(hipblasLtMatmulDescCreate(&g->desc, HIPBLAS_COMPUTE_32F, HIP_R_32F));
        const hipblasOperation_t op = HIPBLAS_OP_N;
        BS_LT(hipblasLtMatmulDescSetAttribute(g->desc, HIPBLASLT_MATMUL_DESC_TRANSA, &op, sizeof op));
        BS_LT(hipblasLtMatmulDescSetAttribute(g->desc, HIPBLASLT_MATMUL_DESC_TRANSB, &op, sizeof op));
        BS_LT(hipblasLtMatrixLayoutCreate(&g->layout, HIP_R_16BF, n, n, n));
        BS_LT(hipblasLtMatmulPreferenceCreate(&g->pref));
        BS_LT(hipblasLtMatmulPreferenceSetAttribute(g->pref, HIPBLASLT_MATMUL_PREF_MAX_WORKSPACE_BYTES,
                                                    &g->workspace_bytes, sizeof g->workspace_bytes));
        if (g->workspace_bytes) BS_HIP(hipMalloc(&g->workspace, g->workspace_bytes));
        g->algos.resize(max_algos);
        int returned = 0;
        BS_LT(hipblasLtMatmulAlgoGetHeuristic(g->lt, g->desc, g->layout, g->layout, g->layout, g->layout,
                                              g->pref, (int)max_algos, g->algos.data(), &returned));
        g->algos.resize(returned > 0 ? (size_t)returned : 0);
        if (g->algos.empty()) return fail("bs_gemm_create: the heuristic returned no algorithm");
        return 0;
    }();
    if (rc != 0) {
        if (g->workspace) (void)hipFree(g->workspace);
        delete g;
        return rc;
    }
    *out = g;
    return 0;
}

extern "C" int bs_gemm_algo_count(void *handle) { return handle ? (int)((Gemm *)handle)->algos.size() : 0; }

// Row-major C = A @ B is, read column-major, C' = B' @ A' on the same memory.
extern "C" int bs_gemm_run(void *handle, int algo, const void *A, const void *B, void *C, void *stream)
{
    Gemm *g = (Gemm *)handle;
    if (!g || !A || !B || !C) return fail("bs_gemm_run: bad argument");
    if (algo < 0 || algo >= (int)g->algos.size()) return fail("bs_gemm_run: algorithm %d of %zu", algo, g->algos.size());
    const float alpha = 1.f, beta = 0.f;
    BS_LT(hipblasLtMatmul(g->lt, g->desc, &alpha, B, g->layout, A, g->layout, &beta, C, g->layout, C,
                          g->layout, &g->algos[(size_t)algo].algo, g->workspace, g->workspace_bytes,
                          (hipStream_t)stream));
    return 0;
}

extern "C" int bs_gemm_destroy(void *handle)
{
    Gemm *g = (Gemm *)handle;
    if (!g) return 0;
    if (g->pref) (void)hipblasLtMatmulPreferenceDestroy(g->pref);
    if (g->layout) (void)hipblasLtMatrixLayoutDestroy(g->layout);
    if (g->desc) (void)hipblasLtMatmulDescDestroy(g->desc);
    if (g->lt) (void)hipblasLtDestroy(g->lt);
    if (g->workspace) (void)hipFree(g->workspace);
    delete g;
    return 0;
}
