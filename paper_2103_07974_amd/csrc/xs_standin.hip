// Arithmetic-only compute stand-in for overlap measurements of the crossover schedule
// (arXiv 2103.07974, Section 2.1: one task computes while the other synchronises).
// Not part of the synchronisation path: it plays the role of a task's forward + backward
// when no model is attached, and touches no memory, so whatever it slows down by when a
// synchronisation runs beside it is pure compute-unit sharing.
#include "xs_internal.h"

namespace xs {

__global__ __launch_bounds__(256) void standin_alu_kernel(float *sink, uint32_t iters, float a, float b)
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

}  // namespace xs

extern "C" int xs_standin_alu(uint32_t workgroups, uint32_t iters, float *sink, void *hip_stream)
{
    using namespace xs;
    if (!sink) return fail(XS_ERR_INVALID_ARG, "xs_standin_alu: sink is NULL");
    if (workgroups == 0 || workgroups > (1u << 20))
        return fail(XS_ERR_INVALID_ARG, "xs_standin_alu: workgroups = %u outside [1, 2^20]", workgroups);
    hipLaunchKernelGGL(standin_alu_kernel, dim3(workgroups), dim3(256), 0, (hipStream_t)hip_stream,
                       sink, iters, 1.0000001f, 1e-7f);
    XS_HIP_TRY(hipGetLastError());
    return XS_OK;
}
