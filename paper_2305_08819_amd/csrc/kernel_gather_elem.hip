// Element-wise gather-GEMM for forward convolution and backward-data with channel counts the
// 16-byte loader cannot take (e.g. the 3-channel first layer, 16 output channels).
//
// Same GEMM view, tiles, MFMA layout and epilogue as gather_gemm_kernel, but the reduction
// index k = (tap, channel) is walked as one flat range in stages of kBK and every operand
// element is fetched with its own 4-byte load and its own bounds test, so any IC, OC, filter
// and stride works.  Meant for short reductions (the 3-channel layer has ONE stage): single
// LDS buffer, two barriers per stage, no tap skipping.
#include "gather_common.h"

namespace mi355conv {

template <int BM, int BN, int WAVES_M, bool BWD>
__global__ __launch_bounds__(kThreads, 2) void gather_elem_kernel(const GatherGemmParams p)
{
    using T = GG<BM, BN, WAVES_M, BWD>;
    extern __shared__ f4 smem_raw[];
    float *As = reinterpret_cast<float *>(smem_raw);
    float *Bs = As + T::A_STAGE;
    int *rowBase = reinterpret_cast<int *>(Bs + T::B_STAGE);
    int *rowY = rowBase + BM;
    int *rowX = rowY + BM;
    int *outRow = rowX + BM;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    BalancePrefetch pre = balance_prefetch(p.runs, p.posOrder);
    balance_prefetch_classes(pre, p.classes);
    const GatherTile tile = gather_tile_setup<BM, BN, BWD>(p, pre, rowBase, rowY, rowX, outRow);
    const int slice = tile.slice, n0 = tile.n0;

    const int Ktot = p.FH * p.FW * p.SC;
    const int nIter = (Ktot + kBK - 1) / kBK;
    const int it0 = (int)((long long)slice * nIter / p.split);
    const int it1 = (int)((long long)(slice + 1) * nIter / p.split);

    const int aSeg = tid & 7, aRow = tid >> 3;
    int rBase[T::PA], rY[T::PA], rX[T::PA];
#pragma unroll
    for (int i = 0; i < T::PA; ++i) {
        const int r = aRow + 32 * i;
        rBase[i] = rowBase[r];
        rY[i] = rowY[r];
        rX[i] = rowX[r];
    }
    const int bSeg = tid % T::B_TPR, bRow = tid / T::B_TPR;
    const long long wRowStride = (long long)p.FH * p.FW * (BWD ? p.DC : p.SC);

    float16v acc[T::MB][T::NB];
#pragma unroll
    for (int i = 0; i < T::MB; ++i)
#pragma unroll
        for (int j = 0; j < T::NB; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int wm = wave / T::WAVES_N, wn = wave % T::WAVES_N;
    const int l32 = lane & 31, lh = lane >> 5;

    for (int it = it0; it < it1; ++it) {
        // ---- this thread's four reduction elements of the A tile (same for all its rows)
        int eOff[4], eDy[4], eDx[4];
        bool eOk[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int k = it * kBK + aSeg * 4 + e;
            const int tap = k / p.SC, c = k - tap * p.SC;
            const int fh = tap / p.FW, fw = tap - fh * p.FW;
            eOk[e] = k < Ktot;
            if (BWD) {
                eOk[e] = eOk[e] && (fh % p.sh) == tile.ra && (fw % p.sw) == tile.rb;
                eDy[e] = -(fh / p.sh);
                eDx[e] = -(fw / p.sw);
            } else {
                eDy[e] = fh;
                eDx[e] = fw;
            }
            eOff[e] = (eDy[e] * p.SW + eDx[e]) * p.SC + c;
        }
        f4 ga[T::PA], gb[T::PB];
#pragma unroll
        for (int i = 0; i < T::PA; ++i)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float v = 0.f;
                if (eOk[e] && (unsigned)(rY[i] + eDy[e]) < (unsigned)p.SH &&
                    (unsigned)(rX[i] + eDx[e]) < (unsigned)p.SW)
                    v = p.A[(long long)(rBase[i] + eOff[e])];
                ga[i][e] = v;
            }
#pragma unroll
        for (int i = 0; i < T::PB; ++i) {
            const int r = bRow + T::B_RPP * i;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float v = 0.f;
                if (BWD) {
                    // B tile [k][col]: k = (tap, oc), col = ic
                    const int k = it * kBK + r, col = n0 + bSeg * 4 + e;
                    if (r < kBK && k < Ktot && col < p.DC) {
                        const int tap = k / p.SC, c = k - tap * p.SC;
                        v = p.B[(long long)c * wRowStride + (long long)tap * p.DC + col];
                    }
                } else {
                    // B tile [col][k]: col = oc, k contiguous in W
                    const int k = it * kBK + bSeg * 4 + e, col = n0 + r;
                    if (r < BN && k < Ktot && col < p.DC) v = p.B[(long long)col * wRowStride + k];
                }
                gb[i][e] = v;
            }
        }
        __syncthreads();   // previous stage's MFMAs have read the single LDS buffer
#pragma unroll
        for (int i = 0; i < T::PA; ++i)
            *reinterpret_cast<f4 *>(As + (aRow + 32 * i) * LDA + aSeg * 4) = ga[i];
#pragma unroll
        for (int i = 0; i < T::PB; ++i) {
            const int r = bRow + T::B_RPP * i;
            if (r < T::B_ROWS) *reinterpret_cast<f4 *>(Bs + r * T::LDB + bSeg * 4) = gb[i];
        }
        __syncthreads();

        const float *a = As + (wm * T::WTM + l32) * LDA + lh * 4;
        const float *b = BWD ? Bs + (lh * 4) * T::LDB + wn * T::WTN + l32
                             : Bs + (wn * T::WTN + l32) * T::LDB + lh * 4;
#pragma unroll
        for (int jj = 0; jj < kBK / 8; ++jj) {
            f4 fa[T::MB], fb[T::NB];
#pragma unroll
            for (int i = 0; i < T::MB; ++i) fa[i] = *reinterpret_cast<const f4 *>(a + i * 32 * LDA + jj * 8);
#pragma unroll
            for (int j = 0; j < T::NB; ++j) {
                if (BWD) {
                    const float *q = b + (jj * 8) * T::LDB + j * 32;
                    fb[j] = f4{q[0], q[T::LDB], q[2 * T::LDB], q[3 * T::LDB]};
                } else {
                    fb[j] = *reinterpret_cast<const f4 *>(b + j * 32 * T::LDB + jj * 8);
                }
            }
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int i = 0; i < T::MB; ++i)
#pragma unroll
                    for (int j = 0; j < T::NB; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i][t], fb[j][t], acc[i][j], 0, 0, 0);
        }
    }

    gather_tile_store<T>(p, slice, n0, outRow, acc, wm, wn, l32, lh);
}

template <int BM, int BN, int WAVES_M, bool BWD>
static hipError_t launch_elem(const GatherGemmParams &p, int grid, hipStream_t st)
{
    using T = GG<BM, BN, WAVES_M, BWD>;
    constexpr size_t smem = (T::A_STAGE + T::B_STAGE + T::TABLE_INTS) * sizeof(float);
    static_assert(smem <= 64 * 1024, "single-buffered tiles fit the default LDS limit");
    hipLaunchKernelGGL((gather_elem_kernel<BM, BN, WAVES_M, BWD>), dim3((unsigned)grid), dim3(kThreads), smem, st, p);
    return hipGetLastError();
}

hipError_t launch_gather_elem(const GatherGemmParams &p, bool bwdData, int bm, int bn, int grid, hipStream_t st)
{
    if (!gather_elem_accepts(bm, bn)) return hipErrorInvalidValue;
#define MI355_GE_CASE(BM_, BN_, WM_)                                                     \
    if (bm == BM_ && bn == BN_)                                                          \
        return bwdData ? launch_elem<BM_, BN_, WM_, true>(p, grid, st)                   \
                       : launch_elem<BM_, BN_, WM_, false>(p, grid, st);
    MI355_GE_CASE(128, 64, 2)
    MI355_GE_CASE(64, 64, 2)
    MI355_GE_CASE(128, 32, 4)
#undef MI355_GE_CASE
    return hipErrorInvalidValue;
}

}  // namespace mi355conv
