// Pieces shared by the two gather-GEMM kernels (16-byte channel-chunk loader and the
// element-wise loader): tile geometry, per-tile row tables, fragment reads + MFMAs, epilogue.
#pragma once
#include "conv_internal.h"

namespace mi355conv {

typedef float float16v __attribute__((ext_vector_type(16)));
typedef float f4 __attribute__((ext_vector_type(4)));   // native vector: stays in registers
typedef const volatile __attribute__((address_space(3))) float *lds_cvptr;

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
    int uLo, uHi, vLo, vHi;     // bounding rectangle of the taps (u,v) that land inside the
                                // source image for at least one row; empty if uHi < uLo
};

// Decodes the workgroup id into (row tile, column tile, slice, phase) and fills the per-row
// tables (source base offset, source y0/x0, destination pixel index or -1).  The tile's tap
// rectangle is computed from the tile's first and last row alone (uniform, no cross-thread
// reduction): a row's valid taps along each axis form an interval whose ends are monotone in
// the row's source coordinate, and the rows of a tile are contiguous in (n,y,x) or (y,x,n)
// order.  Where a tile wraps over image rows or images the rectangle is widened to the full
// range, which only adds taps whose operands load as zeros.  All threads must call it; it
// contains one barrier.
template <int BM, int BN, bool BWD, class P>
__device__ __forceinline__ GatherTile gather_tile_setup(const P &p, const BalancePrefetch &pre, int *rowBase, int *rowY,
                                                        int *rowX, int *outRow)
{
    const int tid = threadIdx.x;
    int tn, tmGlobal, slice;
    if (p.regional) {
        // region-wise order: the XCD (hardware id % 8) fixes the spatial region, the image group and the
        // group of (slice, column tile) pairs; the id's place on the XCD is the tile's rank there
        int xcd, posRank, inner;
        region_wise_place(p, (int)blockIdx.x, &xcd, &posRank, &inner);
        region_wise_tile(p, xcd, balance_order(pre, posRank), inner, &tmGlobal, &tn, &slice);
    } else {
    int bid = p.balance && p.runsN ? balanced_rank(blockIdx.x, p.grid, pre)
                                    : xcd_remap_fast(blockIdx.x, p.xcdWhole, p.xcdUnit, p.divXcdUnit);
    if (p.balance && p.classesN) {
        // class-wise enumeration: (slice, column tile) slow, (position, row tile) fast - see BalanceClasses
        int firstUnit, inner, row;
        balance_class_decode(pre, bid, &firstUnit, &inner, &row);
        slice = (int)fast_div((unsigned)inner, p.divTilesN);
        tn = inner - slice * p.tilesN;
        const int unit = (int)fast_div((unsigned)row, p.divRowTilesPerPos);
        tmGlobal = balance_order(pre, firstUnit + unit) * p.rowTilesPerPos + (row - unit * p.rowTilesPerPos);
    } else {
        const int rest = (int)fast_div((unsigned)bid, p.divTilesN);
        tn = bid - rest * p.tilesN;
        tmGlobal = (int)fast_div((unsigned)rest, p.divSplit);
        slice = rest - tmGlobal * p.split;
        if (p.balance) {   // row tiles are enumerated by position rank
            const int rank = (int)fast_div((unsigned)tmGlobal, p.divRowTilesPerPos);
            tmGlobal = balance_order(pre, rank) * p.rowTilesPerPos + (tmGlobal - rank * p.rowTilesPerPos);
        }
    }
    }
    // Forward and unit-stride backward-data have one phase that holds all pixels and all taps: its
    // record is made up from the scalar arguments.  Only strided backward-data
    // fetches the record of the tile's phase, a load that depends on the decoded tile.
    GatherPhase ph;
    if (!BWD || (p.sh == 1 && p.sw == 1)) {
        ph.tileStart = 0; ph.ra = 0; ph.rb = 0; ph.y0 = 0; ph.x0 = 0;
        ph.dh = p.DH; ph.dw = p.DW; ph.nU = p.FH; ph.nV = p.FW;
        ph.divHW = p.divDHW; ph.divW = p.divDW;
    } else {   // phase starts are ascending: the phase is the number of starts not above this tile
        int phase = 0;
#pragma unroll
        for (int i = 1; i < kMaxPhases; ++i) phase += tmGlobal >= p.phaseStart[i] ? 1 : 0;
        ph = p.phase[phase];
    }
    const int tmLocal = tmGlobal - ph.tileStart;
    const int hw = ph.dh * ph.dw;
    const int Mphase = p.Nimg * hw;
    const int yBase = BWD ? (ph.y0 + p.ph) / p.sh : -p.ph;   // source y of destination index i = 0
    const int xBase = BWD ? (ph.x0 + p.pw) / p.sw : -p.pw;
    const int yStep = BWD ? 1 : p.sh, xStep = BWD ? 1 : p.sw;

    if (tid < BM) {   // one thread per tile row
        const int m = tmLocal * BM + tid;
        int base = 0, y0 = kInvalidCoord, x0 = kInvalidCoord, orow = -1;
        if (m < Mphase) {
            int n, i, j;
            if (p.posMajor) {
                const int pos = (int)fast_div((unsigned)m, p.divN);
                n = m - pos * p.Nimg;
                i = (int)fast_div((unsigned)pos, ph.divW);
                j = pos - i * ph.dw;
            } else {
                n = (int)fast_div((unsigned)m, ph.divHW);
                const int r = m - n * hw;
                i = (int)fast_div((unsigned)r, ph.divW);
                j = r - i * ph.dw;
            }
            const int dyc = BWD ? ph.y0 + i * p.sh : i;
            const int dxc = BWD ? ph.x0 + j * p.sw : j;
            y0 = yBase + i * yStep;
            x0 = xBase + j * xStep;
            orow = (n * p.DH + dyc) * p.DW + dxc;
            base = ((n * p.SH + y0) * p.SW + x0) * p.SC;
        }
        rowBase[tid] = base;
        rowY[tid] = y0;
        rowX[tid] = x0;
        outRow[tid] = orow;
    }

    // ---- tap rectangle from the first and last row of the tile (uniform) ----------------
    GatherTile t;
    t.slice = slice;
    t.n0 = tn * BN;
    t.ra = ph.ra;
    t.rb = ph.rb;
    t.uLo = t.vLo = 0;
    t.uHi = t.vHi = -1;
    const int m0 = tmLocal * BM;
    if (m0 < Mphase) {
        const int m1 = (m0 + BM < Mphase ? m0 + BM : Mphase) - 1;
        int i0, i1, j0, j1;
        bool wrap;
        int r0, r1;
        if (p.posMajor) {
            r0 = (int)fast_div((unsigned)m0, p.divN);
            r1 = (int)fast_div((unsigned)m1, p.divN);
            wrap = false;
        } else {
            const int n0 = (int)fast_div((unsigned)m0, ph.divHW), n1 = (int)fast_div((unsigned)m1, ph.divHW);
            r0 = m0 - n0 * hw;
            r1 = m1 - n1 * hw;
            wrap = n0 != n1;
        }
        if (wrap) {
            i0 = 0; i1 = ph.dh - 1; j0 = 0; j1 = ph.dw - 1;
        } else {
            i0 = (int)fast_div((unsigned)r0, ph.divW);
            i1 = (int)fast_div((unsigned)r1, ph.divW);
            j0 = r0 - i0 * ph.dw;
            j1 = r1 - i1 * ph.dw;
            if (i0 != i1) { j0 = 0; j1 = ph.dw - 1; }
        }
        const int yMin = yBase + i0 * yStep, yMax = yBase + i1 * yStep;
        const int xMin = xBase + j0 * xStep, xMax = xBase + j1 * xStep;
        if (BWD) {   // source row y - u in [0, SH): u in [max(0, y-SH+1), min(nU-1, y)], both rising with y
            t.uLo = max(0, yMin - p.SH + 1);
            t.uHi = min(ph.nU - 1, yMax);
            t.vLo = max(0, xMin - p.SW + 1);
            t.vHi = min(ph.nV - 1, xMax);
        } else {     // source row y + u in [0, SH): u in [max(0, -y), min(nU-1, SH-1-y)], both falling with y
            t.uLo = max(0, -yMax);
            t.uHi = min(ph.nU - 1, p.SH - 1 - yMin);
            t.vLo = max(0, -xMax);
            t.vHi = min(ph.nV - 1, p.SW - 1 - xMin);
        }
        if (t.uHi < t.uLo || t.vHi < t.vLo) { t.uHi = -1; t.uLo = 0; t.vHi = -1; t.vLo = 0; }
    }
    __syncthreads();
    return t;
}

// Epilogue: rows of a 32x32 block are spread over accumulator registers, columns over lanes.
// With `scratch` (32 x kLDT floats of LDS owned by the calling wave) and a destination whose
// channel count is a multiple of 4, each block is turned in LDS so that a lane holds four
// neighbouring columns of one row: four 16-byte stores per block, each covering eight 128-byte
// row segments, instead of sixteen 4-byte stores covering two.  Otherwise the 16
// destination-pixel indices of a block are fetched with four 16-byte LDS reads and every
// accumulator register is stored on its own.  Output offsets fit 32 bits because every tensor
// holds fewer than 2^31 elements.
constexpr int kLDT = 36;   // pitch of the turning buffer: 16-byte aligned rows, bank-skewed
template <class T, class P>
__device__ __forceinline__ void gather_tile_store(const P &p, int slice, int n0, const int *outRow,
                                                  const float16v (&acc)[T::MB][T::NB], int wm, int wn, int l32,
                                                  int lh, float *scratch = nullptr)
{
    typedef int i4 __attribute__((ext_vector_type(4)));
    float *C = p.C + (long long)slice * p.sliceStride;
    const bool epi = p.epilogue && p.split == 1;   // sliced launches leave it to the combine pass
    const float slope = epi ? p.slope : 1.f;
    const int lane = lh * 32 + l32;
#pragma unroll
    for (int i = 0; i < T::MB; ++i) {
#pragma unroll
        for (int j = 0; j < T::NB; ++j) {
            const int colBase = n0 + wn * T::WTN + j * 32;
            if (scratch && (p.DC & 3) == 0 && colBase + 32 <= p.DC) {   // uniform
                if (epi) {   // uniform: the plain operator pays no vector arithmetic here
                    const float b = p.bias ? p.bias[colBase + l32] : 0.f;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        float v = acc[i][j][r] + b;
                        v = v > 0.f ? v : v * slope;
                        scratch[(8 * (r / 4) + 4 * lh + (r % 4)) * kLDT + l32] = v;
                    }
                } else {
#pragma unroll
                    for (int r = 0; r < 16; ++r) scratch[(8 * (r / 4) + 4 * lh + (r % 4)) * kLDT + l32] = acc[i][j][r];
                }
                // the LDS pipeline keeps a wave's accesses in order; no other wave touches this buffer
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int row = q * 8 + (lane >> 3), seg = lane & 7;
                    const f4 v = *reinterpret_cast<const f4 *>(scratch + row * kLDT + seg * 4);
                    const int o = outRow[wm * T::WTM + i * 32 + row];
                    if (o >= 0) *reinterpret_cast<f4 *>(C + o * p.DC + colBase + seg * 4) = v;
                }
            } else {
                i4 orow[4];
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    orow[g] = *reinterpret_cast<const i4 *>(outRow + wm * T::WTM + i * 32 + 8 * g + 4 * lh);
                const int col = colBase + l32;
                if (col < p.DC) {
                    const float b = epi && p.bias ? p.bias[col] : 0.f;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int o = orow[r / 4][r % 4];
                        float v = acc[i][j][r] + b;
                        v = v > 0.f ? v : v * slope;
                        if (o >= 0) C[o * p.DC + col] = v;
                    }
                }
            }
        }
    }
}

}  // namespace mi355conv
