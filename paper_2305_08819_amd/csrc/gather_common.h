// Pieces shared by the two gather-GEMM kernels (16-byte channel-chunk loader and the
// element-wise loader): tile geometry, per-tile row tables, fragment reads + MFMAs, epilogue.
#pragma once
#include "conv_internal.h"

namespace mi355conv {

typedef float float16v __attribute__((ext_vector_type(16)));
typedef float f4 __attribute__((ext_vector_type(4)));   // native vector: stays in registers

constexpr int LDA = kBK + 4;   // LDS row pitch (floats) of a [row][k] tile: 16-byte aligned, bank-skewed
constexpr int kInvalidCoord = -(1 << 28);

template <int BM, int BN, int WAVES_M, bool BWD>
struct GG {
    static constexpr int WAVES_N = 4 / WAVES_M;
    static constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;   // wave tile
    static constexpr int MB = WTM / 32, NB = WTN / 32;             // 32x32 MFMA blocks per wave
    static constexpr int PA = BM / 32;                             // A loader passes (32 rows each)
    // forward: B tile is [BN cols][kBK] (k contiguous, like A); backward-data: [kBK][BN] (col contiguous)
    static constexpr int LDB = BWD ? (BN + 8) : LDA;
    static constexpr int B_TPR = BWD ? BN / 4 : 8;                 // threads per B tile row
    static constexpr int B_RPP = kThreads / B_TPR;                 // B rows per pass
    static constexpr int B_ROWS = BWD ? kBK : BN;
    static constexpr int PB = (B_ROWS + B_RPP - 1) / B_RPP;
    static constexpr int A_STAGE = BM * LDA;
    static constexpr int B_STAGE = B_ROWS * LDB;
    static constexpr int TABLE_INTS = 4 * BM + 4;
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be whole 32x32 blocks");
    static_assert(B_ROWS % B_RPP == 0 || B_ROWS < B_RPP, "B loader passes");
};

struct GatherTile {
    int slice;                  // reduction slice of this workgroup
    int n0;                     // first output column
    int ra, rb;                 // stride-phase residues (backward-data)
    unsigned long long tapMask; // taps that land inside the source image for at least one row
};

// Decodes the workgroup id into (row tile, column tile, slice, phase), fills the per-row
// tables (source base offset, source y0/x0, destination pixel index or -1) and ORs the rows'
// in-range tap sets.  All threads must call it; it contains two barriers.
template <int BM, int BN, bool BWD>
__device__ __forceinline__ GatherTile gather_tile_setup(const GatherGemmParams &p, int *rowBase, int *rowY,
                                                        int *rowX, int *outRow, unsigned *tapMaskS)
{
    const int tid = threadIdx.x;
    int bid = xcd_remap(blockIdx.x, gridDim.x, p.xcdUnit);
    const int tn = bid % p.tilesN;
    bid /= p.tilesN;
    const int slice = bid % p.split;
    const int tmGlobal = bid / p.split;
    int phase = 0;
    while (phase + 1 < p.nPhases && tmGlobal >= p.phaseTileStart[phase + 1]) ++phase;
    const int tmLocal = tmGlobal - p.phaseTileStart[phase];
    const int ra = p.phaseRa[phase], rb = p.phaseRb[phase];
    const int PY0 = p.phaseY0[phase], PX0 = p.phaseX0[phase];
    const int PDH = p.phaseDH[phase], PDW = p.phaseDW[phase];
    const int Mphase = p.Nimg * PDH * PDW;

    if (tid < 2) tapMaskS[tid] = 0u;
    __syncthreads();

    if (tid < BM) {   // one thread per tile row
        const int m = tmLocal * BM + tid;
        int base = 0, y0 = kInvalidCoord, x0 = kInvalidCoord, orow = -1;
        if (m < Mphase) {
            int n, i, j;
            if (p.posMajor) {
                n = m % p.Nimg;
                const int pos = m / p.Nimg;
                i = pos / PDW;
                j = pos - i * PDW;
            } else {
                const int hw = PDH * PDW;
                n = m / hw;
                const int r = m - n * hw;
                i = r / PDW;
                j = r - i * PDW;
            }
            int dyc, dxc;
            if (BWD) {
                dyc = PY0 + i * p.sh;
                dxc = PX0 + j * p.sw;
                y0 = (PY0 + p.ph) / p.sh + i;
                x0 = (PX0 + p.pw) / p.sw + j;
            } else {
                dyc = i;
                dxc = j;
                y0 = i * p.sh - p.ph;
                x0 = j * p.sw - p.pw;
            }
            orow = (n * p.DH + dyc) * p.DW + dxc;
            base = ((n * p.SH + y0) * p.SW + x0) * p.SC;
        }
        unsigned lo = 0u, hi = 0u;
        int t = 0;
        for (int fh = 0; fh < p.FH; ++fh) {
            bool okh;
            int sy;
            if (BWD) {
                okh = (fh % p.sh) == ra;
                sy = y0 - fh / p.sh;
            } else {
                okh = true;
                sy = y0 + fh;
            }
            okh = okh && (unsigned)sy < (unsigned)p.SH;
            for (int fw = 0; fw < p.FW; ++fw, ++t) {
                bool okw;
                int sx;
                if (BWD) {
                    okw = (fw % p.sw) == rb;
                    sx = x0 - fw / p.sw;
                } else {
                    okw = true;
                    sx = x0 + fw;
                }
                okw = okw && (unsigned)sx < (unsigned)p.SW;
                if (okh && okw && t < kMaxTaps) {
                    if (t < 32) lo |= 1u << t;
                    else hi |= 1u << (t - 32);
                }
            }
        }
        if (lo) atomicOr(&tapMaskS[0], lo);
        if (hi) atomicOr(&tapMaskS[1], hi);
        rowBase[tid] = base;
        rowY[tid] = y0;
        rowX[tid] = x0;
        outRow[tid] = orow;
    }
    __syncthreads();

    GatherTile t;
    t.slice = slice;
    t.n0 = tn * BN;
    t.ra = ra;
    t.rb = rb;
    t.tapMask = (unsigned long long)tapMaskS[0] | ((unsigned long long)tapMaskS[1] << 32);
    return t;
}

// Epilogue: rows of a 32x32 block are spread over accumulator registers, columns over lanes.
template <class T>
__device__ __forceinline__ void gather_tile_store(const GatherGemmParams &p, int slice, int n0, const int *outRow,
                                                  const float16v (&acc)[T::MB][T::NB], int wm, int wn, int l32,
                                                  int lh)
{
    float *C = p.C + (long long)slice * p.sliceStride;
#pragma unroll
    for (int i = 0; i < T::MB; ++i)
#pragma unroll
        for (int j = 0; j < T::NB; ++j) {
            const int col = n0 + wn * T::WTN + j * 32 + l32;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = wm * T::WTM + i * 32 + 8 * (r / 4) + 4 * lh + (r % 4);
                const int orow = outRow[row];
                if (orow >= 0 && col < p.DC) C[(long long)orow * p.DC + col] = acc[i][j][r];
            }
        }
}

}  // namespace mi355conv
