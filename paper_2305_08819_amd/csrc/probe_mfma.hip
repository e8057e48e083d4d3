// Measurement aid, not an operator: a register-only v_mfma_f32_32x32x2_f32 loop, optionally with
// ordinary vector-ALU instructions between the matrix instructions.  It gives the matrix rate this
// chip sustains at its actual clock (what "% of measured peak" in the bench refers to) and shows
// that fp32 MFMA and VALU instructions share a SIMD's issue cycles - the fact the convolution
// kernels' loops are built around.
#include "../../include/mi355conv.h"
#include "conv_internal.h"

namespace mi355conv {

typedef float float16v __attribute__((ext_vector_type(16)));

// NV vector-ALU instructions (dependent fp32 FMAs) per 8 MFMAs, spread evenly between them.
template <int NV>
__global__ __launch_bounds__(kThreads) void mfma_rate_kernel(float *out, int iters, float seed)
{
    float16v acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    const float a = seed + 1e-3f * (float)threadIdx.x, b = 1.f - seed;
    float y = a;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            acc[u & 3] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[u & 3], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);   // keeps the vector instructions between the matrix ones
#pragma unroll
            for (int v = 0; v < NV / 8; ++v) y = __builtin_fmaf(y, b, a);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    float s = y;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    out[(size_t)blockIdx.x * kThreads + threadIdx.x] = s;
}

}  // namespace mi355conv

using namespace mi355conv;

extern "C" int conv2d_probe_mfma_rate(int valu_per_8_mfma, int workgroups, int iters, float *out, void *stream)
{
    if (!out) return MI355CONV_ERR_NULL_PTR;
    if (workgroups <= 0 || iters <= 0) return MI355CONV_ERR_BAD_DIM;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)workgroups), block(kThreads);
    switch (valu_per_8_mfma) {
    case 0: hipLaunchKernelGGL(mfma_rate_kernel<0>, grid, block, 0, st, out, iters, 0.25f); break;
    case 16: hipLaunchKernelGGL(mfma_rate_kernel<16>, grid, block, 0, st, out, iters, 0.25f); break;
    case 48: hipLaunchKernelGGL(mfma_rate_kernel<48>, grid, block, 0, st, out, iters, 0.25f); break;
    case 96: hipLaunchKernelGGL(mfma_rate_kernel<96>, grid, block, 0, st, out, iters, 0.25f); break;
    default: return MI355CONV_ERR_UNSUPPORTED;
    }
    return hipGetLastError() == hipSuccess ? MI355CONV_OK : MI355CONV_ERR_HIP;
}
