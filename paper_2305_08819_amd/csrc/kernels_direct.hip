// Direct (one thread per output element) kernels and the slice-reduce kernel.
//
// The direct kernels take any shape the ABI accepts; the host picks them when the MFMA
// variants' divisibility conditions do not hold (e.g. the 3-channel first layer) or when a
// test forces them.  They follow the operator definitions literally (paper Sec. III
// Layer-1 / Sec. IV name the operators; layouts from Table I) with fp32 FMAs.
#include "conv_internal.h"

namespace mi355conv {

__global__ __launch_bounds__(256) void direct_fwd_kernel(const float *__restrict__ X,
                                                         const float *__restrict__ W,
                                                         float *__restrict__ Y, Shape s)
{
    long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    long long total = (long long)s.N * s.OH * s.OW * s.OC;
    if (idx >= total) return;
    int oc = (int)(idx % s.OC);
    long long m = idx / s.OC;
    int ow = (int)(m % s.OW);
    long long t = m / s.OW;
    int oh = (int)(t % s.OH);
    int n = (int)(t / s.OH);
    float acc = 0.f;
    for (int fh = 0; fh < s.FH; ++fh) {
        int ih = oh * s.sh - s.ph + fh;
        if ((unsigned)ih >= (unsigned)s.IH) continue;
        for (int fw = 0; fw < s.FW; ++fw) {
            int iw = ow * s.sw - s.pw + fw;
            if ((unsigned)iw >= (unsigned)s.IW) continue;
            const float *x = X + (((long long)n * s.IH + ih) * s.IW + iw) * s.IC;
            const float *w = W + (((long long)oc * s.FH + fh) * s.FW + fw) * s.IC;
            for (int ic = 0; ic < s.IC; ++ic) acc = fmaf(x[ic], w[ic], acc);
        }
    }
    Y[idx] = acc;
}

__global__ __launch_bounds__(256) void direct_bwd_data_kernel(const float *__restrict__ G,
                                                              const float *__restrict__ W,
                                                              float *__restrict__ dX, Shape s)
{
    long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    long long total = (long long)s.N * s.IH * s.IW * s.IC;
    if (idx >= total) return;
    int ic = (int)(idx % s.IC);
    long long m = idx / s.IC;
    int iw = (int)(m % s.IW);
    long long t = m / s.IW;
    int ih = (int)(t % s.IH);
    int n = (int)(t / s.IH);
    float acc = 0.f;
    for (int fh = 0; fh < s.FH; ++fh) {
        int th = ih + s.ph - fh;
        if (th < 0 || th % s.sh != 0) continue;
        int oh = th / s.sh;
        if (oh >= s.OH) continue;
        for (int fw = 0; fw < s.FW; ++fw) {
            int tw = iw + s.pw - fw;
            if (tw < 0 || tw % s.sw != 0) continue;
            int ow = tw / s.sw;
            if (ow >= s.OW) continue;
            const float *g = G + (((long long)n * s.OH + oh) * s.OW + ow) * s.OC;
            const float *w = W + ((long long)fh * s.FW + fw) * s.IC + ic;
            long long wstride = (long long)s.FH * s.FW * s.IC;
            for (int oc = 0; oc < s.OC; ++oc) acc = fmaf(g[oc], w[oc * wstride], acc);
        }
    }
    dX[idx] = acc;
}

// One workgroup per dW element.  Each thread sums a strided subset of the N*OH*OW rows;
// its running sum is folded into a second accumulator every 512 terms so that no fp32
// chain is longer than that, then the 256 partial sums are combined by a fixed LDS tree.
__global__ __launch_bounds__(256) void direct_bwd_weight_kernel(const float *__restrict__ X,
                                                                const float *__restrict__ G,
                                                                float *__restrict__ dW, Shape s)
{
    __shared__ float red[256];
    long long e = blockIdx.x;
    int ic = (int)(e % s.IC);
    long long t = e / s.IC;
    int fw = (int)(t % s.FW);
    t /= s.FW;
    int fh = (int)(t % s.FH);
    int oc = (int)(t / s.FH);
    long long M = (long long)s.N * s.OH * s.OW;
    float acc = 0.f, acc2 = 0.f;
    int chain = 0;
    for (long long m = threadIdx.x; m < M; m += 256) {
        int ow = (int)(m % s.OW);
        long long r = m / s.OW;
        int oh = (int)(r % s.OH);
        int n = (int)(r / s.OH);
        int ih = oh * s.sh - s.ph + fh, iw = ow * s.sw - s.pw + fw;
        if ((unsigned)ih < (unsigned)s.IH && (unsigned)iw < (unsigned)s.IW)
            acc = fmaf(G[m * s.OC + oc], X[(((long long)n * s.IH + ih) * s.IW + iw) * s.IC + ic], acc);
        if (++chain == 512) {
            acc2 += acc;
            acc = 0.f;
            chain = 0;
        }
    }
    red[threadIdx.x] = acc2 + acc;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) dW[e] = red[0];
}

// out[i] = sum_s ws[s*stride + i].  The partials are fp32; they are added in fp64 in a fixed
// order and rounded once, so the result is reproducible and the combine step adds no error of
// its own beyond the final rounding.  A workgroup owns 256/G float4 columns; G thread groups
// each add every G-th slice, then the G group sums are combined by halving (group g takes
// group g + w for w = G/2, G/4, ... 1) through LDS - a fixed tree, whatever the timing.
// Optional epilogue (cols > 0): out = act(sum + bias[column]), act(v) = v > 0 ? v : slope * v, the
// same fp32 arithmetic as the epilogue of an unsliced launch.
__device__ __forceinline__ float bias_act(float v, long long index, const float *bias, float slope, int cols)
{
    if (cols > 0) {
        if (bias) v += bias[index % cols];
        v = v > 0.f ? v : v * slope;
    }
    return v;
}

template <int G>
__global__ __launch_bounds__(256) void slice_reduce_kernel(const float *__restrict__ ws,
                                                           float *__restrict__ out,
                                                           long long count4, int split, long long stride4,
                                                           const float *__restrict__ bias, float slope, int cols)
{
    constexpr int COLS = 256 / G;
    __shared__ double red[G > 1 ? 256 * 4 : 1];
    const int c = threadIdx.x % COLS, g = threadIdx.x / COLS;
    const long long i = (long long)blockIdx.x * COLS + c;
    double a0 = 0, a1 = 0, a2 = 0, a3 = 0;
    if (i < count4) {
        const float4 *p = reinterpret_cast<const float4 *>(ws) + i;
        int s = g;
        // four loads in flight, added in slice order
        for (; s + 3 * G < split; s += 4 * G) {
            const float4 v0 = p[s * stride4], v1 = p[(s + G) * stride4], v2 = p[(s + 2 * G) * stride4],
                         v3 = p[(s + 3 * G) * stride4];
            a0 += v0.x; a1 += v0.y; a2 += v0.z; a3 += v0.w;
            a0 += v1.x; a1 += v1.y; a2 += v1.z; a3 += v1.w;
            a0 += v2.x; a1 += v2.y; a2 += v2.z; a3 += v2.w;
            a0 += v3.x; a1 += v3.y; a2 += v3.z; a3 += v3.w;
        }
        for (; s < split; s += G) {
            const float4 v = p[s * stride4];
            a0 += v.x; a1 += v.y; a2 += v.z; a3 += v.w;
        }
    }
    if (G > 1) {
        double *mine = red + (g * COLS + c) * 4;
        mine[0] = a0; mine[1] = a1; mine[2] = a2; mine[3] = a3;
        __syncthreads();
#pragma unroll
        for (int w = G / 2; w >= 1; w /= 2) {
            if (g < w) {
                const double *other = red + ((g + w) * COLS + c) * 4;
                mine[0] += other[0]; mine[1] += other[1]; mine[2] += other[2]; mine[3] += other[3];
            }
            __syncthreads();
        }
        a0 = mine[0]; a1 = mine[1]; a2 = mine[2]; a3 = mine[3];
    }
    if (g == 0 && i < count4)
        reinterpret_cast<float4 *>(out)[i] =
            make_float4(bias_act((float)a0, 4 * i, bias, slope, cols), bias_act((float)a1, 4 * i + 1, bias, slope, cols),
                        bias_act((float)a2, 4 * i + 2, bias, slope, cols), bias_act((float)a3, 4 * i + 3, bias, slope, cols));
}

// scalar tail (count % 4 elements) of the reduce
__global__ void slice_reduce_tail_kernel(const float *__restrict__ ws, float *__restrict__ out,
                                         long long first, long long count, int split, long long stride,
                                         const float *__restrict__ bias, float slope, int cols)
{
    const long long j = first + threadIdx.x;
    if (j < count) {
        double a = 0;
        for (int s = 0; s < split; ++s) a += ws[s * stride + j];
        out[j] = bias_act((float)a, j, bias, slope, cols);
    }
}

__global__ __launch_bounds__(256) void bias_act_kernel(float *__restrict__ out, long long count,
                                                       const float *__restrict__ bias, float slope, int cols)
{
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i < count) out[i] = bias_act(out[i], i, bias, slope, cols);
}

static inline unsigned blocks_for(long long n) { return (unsigned)((n + 255) / 256); }

hipError_t launch_direct_fwd(const float *X, const float *W, float *Y, const Shape &s, hipStream_t st)
{
    long long total = (long long)s.N * s.OH * s.OW * s.OC;
    hipLaunchKernelGGL(direct_fwd_kernel, dim3(blocks_for(total)), dim3(256), 0, st, X, W, Y, s);
    return hipGetLastError();
}

hipError_t launch_direct_bwd_data(const float *G, const float *W, float *dX, const Shape &s, hipStream_t st)
{
    long long total = (long long)s.N * s.IH * s.IW * s.IC;
    hipLaunchKernelGGL(direct_bwd_data_kernel, dim3(blocks_for(total)), dim3(256), 0, st, G, W, dX, s);
    return hipGetLastError();
}

hipError_t launch_direct_bwd_weight(const float *X, const float *G, float *dW, const Shape &s, hipStream_t st)
{
    long long total = (long long)s.OC * s.FH * s.FW * s.IC;
    hipLaunchKernelGGL(direct_bwd_weight_kernel, dim3((unsigned)total), dim3(256), 0, st, X, G, dW, s);
    return hipGetLastError();
}

hipError_t launch_bias_act(float *out, long long count, const float *bias, float slope, int cols, hipStream_t st)
{
    hipLaunchKernelGGL(bias_act_kernel, dim3(blocks_for(count)), dim3(256), 0, st, out, count, bias, slope, cols);
    return hipGetLastError();
}

hipError_t launch_slice_reduce(const float *ws, float *out, long long count, int split,
                               long long stride, hipStream_t st, const float *bias, float slope, int cols)
{
    // stride is a multiple of 4 (the host pads it), so float4 loads of every slice are aligned
    const long long count4 = count >> 2;
    if (count4 > 0) {
        // more thread groups per column when there are few columns and many slices
        // at least 8 float4 columns (128 bytes) of a slice per workgroup row: a narrower strip would pull a
        // whole cache line for every 16 bytes it uses
        int G = 1;
        while (G < 32 && G * 2 <= split && count4 * G < (1 << 17)) G *= 2;
        const long long perWg = 256 / G;   // float4 columns per workgroup
        const unsigned grid = (unsigned)((count4 + perWg - 1) / perWg);
        const long long stride4 = stride >> 2;
#define MI355CONV_SR(G_)                                                                                  \
    case G_:                                                                                              \
        hipLaunchKernelGGL(slice_reduce_kernel<G_>, dim3(grid), dim3(256), 0, st, ws, out, count4, split, \
                           stride4, bias, slope, cols);                                                   \
        break;
        switch (G) {
            MI355CONV_SR(1) MI355CONV_SR(2) MI355CONV_SR(4) MI355CONV_SR(8) MI355CONV_SR(16)
        default:
            hipLaunchKernelGGL(slice_reduce_kernel<32>, dim3(grid), dim3(256), 0, st, ws, out, count4, split, stride4,
                               bias, slope, cols);
            break;
        }
#undef MI355CONV_SR
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (count4 * 4 < count)
        hipLaunchKernelGGL(slice_reduce_tail_kernel, dim3(1), dim3(4), 0, st, ws, out, count4 * 4, count, split, stride,
                           bias, slope, cols);
    return hipGetLastError();
}

}  // namespace mi355conv
