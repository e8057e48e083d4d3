// Backward-data for layers with very few input channels (the first layer of a CIFAR network:
// dX has 3 channels), unit stride.
//
// Treating dX[M x IC] = dY-patches[M x (taps*OC)] * W' as a GEMM wastes the matrix unit: its
// narrowest tile is 32 columns wide and only IC of them are real.  Instead the products are
// grouped the other way round:
//   P[pixel of dY][(fh,fw,ic)] = sum_oc dY[pixel, oc] * W[oc, fh, fw, ic]        (a dense GEMM with
//                                 K = OC and N = FH*FW*IC <= 32: 27 of 32 columns real for 3x3x3)
//   dX[n, ih, iw, ic]          = sum_{fh,fw} P[(ih+ph-fh, iw+pw-fw)][(fh,fw,ic)]  (col2im gather)
// which is the same sum in another order and 9x fewer MFMAs.  A workgroup owns kTR x 32 pixels of
// one image of dX; it computes P for those pixels' halo ((kTR+FH-1) x (32+FW-1) dY pixels, at most
// 224) with v_mfma_f32_32x32x2_f32 into LDS and then gathers.  dY pixels outside the map get an
// out-of-range buffer offset, read zeros and give zero rows of P, so the gather needs no test.
#include <hip/hip_runtime.h>
#include "gather_common.h"

namespace mi355conv {

namespace {
constexpr int kTR = 4, kTC = 32;          // dX tile: rows x columns of one image
constexpr int kPRows = 224;               // P rows held (7 MFMA row blocks)
constexpr int kLDP = 33;                  // P row pitch (floats): odd, so the gather's strided reads spread over banks
}  // namespace

__global__ __launch_bounds__(kThreads, 2) void bwd_data_small_ic_kernel(const SmallIcParams p)
{
    extern __shared__ f4 smem_raw[];
    float *As = reinterpret_cast<float *>(smem_raw);          // [kPRows][LDA], later P as [kPRows][kLDP]
    float *Bs = As + kPRows * LDA;                            // [32 columns (fh,fw,ic)][LDA] (k = oc contiguous)

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, lh = lane >> 5;
    const int tilesW = (p.IW + kTC - 1) / kTC, tilesH = (p.IH + kTR - 1) / kTR;
    int bid = blockIdx.x;
    const int tw = bid % tilesW;
    bid /= tilesW;
    const int th = bid % tilesH;
    const int n = bid / tilesH;
    const int ih0 = th * kTR, iw0 = tw * kTC;
    const int PR = kTR + p.FH - 1, PC = kTC + p.FW - 1;       // halo of dY pixels; PR * PC <= kPRows (host checks)
    const int ohBase = ih0 + p.ph - (p.FH - 1), owBase = iw0 + p.pw - (p.FW - 1);
    const int Kp = p.FH * p.FW * p.IC;                        // real columns of P (<= 32)

    constexpr int kOutOfRange = (int)0x80000000;
    const __amdgpu_buffer_rsrc_t rsrcG =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(p.G), 0, (int)p.gBytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrcW =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(p.W), 0, (int)p.wBytes, 0x00020000);

    // A loader: 224 rows x 8 segments of 16 bytes per 32-channel chunk = 7 loads per thread
    constexpr int kPA = kPRows * 8 / kThreads;
    const int aSeg = tid & 7, aRow = tid >> 3;
    int aOff[kPA];
#pragma unroll
    for (int i = 0; i < kPA; ++i) {
        const int q = aRow + 32 * i;
        const int pr = q / PC, pc = q - pr * PC;
        const int oh = ohBase + pr, ow = owBase + pc;
        const bool ok = q < PR * PC && (unsigned)oh < (unsigned)p.OH && (unsigned)ow < (unsigned)p.OW;
        aOff[i] = ok ? (((n * p.OH + oh) * p.OW + ow) * p.OC + aSeg * 4) * 4 : kOutOfRange;
    }
    // B loader: Bs[col][k] = W[oc = c0 + k][col], 32 x 32 elements, 4 per thread
    int bOff[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int idx = tid + kThreads * i;
        const int col = idx >> 5, k = idx & 31;
        bOff[i] = col < Kp ? (k * Kp + col) * 4 : kOutOfRange;
    }

    f4 ga[kPA];
    float gb[4];
    auto gload = [&](int chunk) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < kPA; ++i)
            ga[i] = __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(rsrcG, aOff[i], chunk * kBK * 4, 0));
#pragma unroll
        for (int i = 0; i < 4; ++i)
            gb[i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrcW, bOff[i], chunk * kBK * Kp * 4, 0));
    };
    auto lds_store = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < kPA; ++i) *reinterpret_cast<f4 *>(As + (aRow + 32 * i) * LDA + aSeg * 4) = ga[i];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int idx = tid + kThreads * i;
            Bs[(idx >> 5) * LDA + (idx & 31)] = gb[i];
        }
    };

    // wave w owns P row blocks w and w + 4 (block 7 does not exist)
    float16v acc[2];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[b][r] = 0.f;
    const bool second = wave + 4 < kPRows / 32;

    const int chunks = p.OC / kBK;
    gload(0);
    for (int c = 0; c < chunks; ++c) {
        lds_store();
        __syncthreads();
        if (c + 1 < chunks) gload(c + 1);
#pragma unroll
        for (int g = 0; g < kBK / 8; ++g) {
            const f4 fb = *reinterpret_cast<const f4 *>(Bs + l32 * LDA + g * 8 + lh * 4);
            const f4 fa0 = *reinterpret_cast<const f4 *>(As + (wave * 32 + l32) * LDA + g * 8 + lh * 4);
            f4 fa1 = f4{0.f, 0.f, 0.f, 0.f};
            if (second) fa1 = *reinterpret_cast<const f4 *>(As + ((wave + 4) * 32 + l32) * LDA + g * 8 + lh * 4);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa0[t], fb[t], acc[0], 0, 0, 0);
                if (second) acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa1[t], fb[t], acc[1], 0, 0, 0);
            }
        }
        __syncthreads();   // everyone is done reading this chunk's tiles
    }

    // P into LDS (over the A tile): accumulator register r of lane l is row 8*(r/4)+4*(l/32)+r%4, column l%32
    float *Ps = As;
#pragma unroll
    for (int b = 0; b < 2; ++b)
        if (b == 0 || second) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = (wave + 4 * b) * 32 + 8 * (r / 4) + 4 * lh + (r % 4);
                Ps[row * kLDP + l32] = acc[b][r];
            }
        }
    __syncthreads();

    // col2im: one thread per dX pixel of the tile
    if (tid < kTR * kTC) {
        const int r = tid / kTC, cc = tid - r * kTC;
        const int ih = ih0 + r, iw = iw0 + cc;
        if (ih < p.IH && iw < p.IW) {
            float sum[4] = {0.f, 0.f, 0.f, 0.f};
            for (int fh = 0; fh < p.FH; ++fh)
                for (int fw = 0; fw < p.FW; ++fw) {
                    const float *row = Ps + ((r + p.FH - 1 - fh) * PC + (cc + p.FW - 1 - fw)) * kLDP + (fh * p.FW + fw) * p.IC;
#pragma unroll
                    for (int ic = 0; ic < 4; ++ic)
                        if (ic < p.IC) sum[ic] += row[ic];
                }
            float *dst = p.dX + (((long long)n * p.IH + ih) * p.IW + iw) * p.IC;
#pragma unroll
            for (int ic = 0; ic < 4; ++ic)
                if (ic < p.IC) dst[ic] = sum[ic];
        }
    }
}

hipError_t launch_bwd_data_small_ic(const SmallIcParams &p, hipStream_t st)
{
    const int PR = kTR + p.FH - 1, PC = kTC + p.FW - 1;
    if (PR * PC > kPRows || p.FH * p.FW * p.IC > 32 || p.IC > 4 || p.OC % kBK != 0) return hipErrorInvalidValue;
    const size_t smem = (size_t)(kPRows * LDA + 32 * LDA) * sizeof(float);
    static_assert(kPRows * kLDP <= kPRows * LDA, "P fits over the A tile");
    auto kern = bwd_data_small_ic_kernel;
    static bool attrSet[16] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 16 || !attrSet[dev]) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        if (dev >= 0 && dev < 16) attrSet[dev] = true;
    }
    const int grid = p.N * ((p.IH + kTR - 1) / kTR) * ((p.IW + kTC - 1) / kTC);
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kThreads), smem, st, p);
    return hipGetLastError();
}

}  // namespace mi355conv
