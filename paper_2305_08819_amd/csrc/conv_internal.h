// Internal declarations shared by the host API and the HIP kernels of libmi355conv.
// Nothing here is part of the public ABI (see include/mi355conv.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace mi355conv {

struct Shape {
    int N, IH, IW, IC, OC, FH, FW, sh, sw, ph, pw;
    int OH, OW;
};

constexpr int kThreads = 256;     // every MFMA kernel runs 4 wavefronts per workgroup
constexpr int kBK = 32;           // reduction elements staged per LDS stage
constexpr int kMaxTaps = 64;      // FH*FW limit of the MFMA variants (tap set is a 64-bit mask)
constexpr int kMaxPhases = 16;    // sh*sw limit of the MFMA backward-data variant

// ---- gather-GEMM (forward and backward-data) ------------------------------------------
// C[row, col] = sum over taps t of the tile's tap set, channels c:
//                 A[n, y0(row)+dy(t), x0(row)+dx(t), c] * Wt(t, c, col)
// Forward : A = X,  rows = output pixels,  cols = oc, c = ic, dy = fh,      phases = 1.
// Bwd-data: A = dY, rows = input pixels of one stride phase, cols = ic, c = oc,
//           dy = -(fh / sh) for the taps with fh % sh == phase residue.
struct GatherGemmParams {
    const float *A;
    const float *B;
    float *C;             // output tensor, or workspace base when split > 1
    int Nimg;
    int SH, SW, SC;       // source map height, width, channels (SC = reduction channels per tap)
    int DH, DW, DC;       // destination map height, width, channels (DC = GEMM columns)
    int FH, FW;
    int sh, sw, ph, pw;
    int posMajor;         // rows ordered (y, x, n) instead of (n, y, x)
    int split;            // reduction slices
    long long sliceStride;// elements between consecutive partial outputs in the workspace
    int tilesN;
    int xcdUnit;          // consecutive logical workgroup ids kept on one XCD
    int nPhases;
    int phaseTileStart[kMaxPhases + 1];
    // per phase: residues, first destination row/col, destination rows/cols in the phase
    short phaseRa[kMaxPhases], phaseRb[kMaxPhases];
    short phaseY0[kMaxPhases], phaseX0[kMaxPhases];
    int phaseDH[kMaxPhases], phaseDW[kMaxPhases];
};

// ---- backward-weight ---------------------------------------------------------------------
// dW[oc, col] = sum over rows m=(n,oh,ow): G[m, oc] * X[n, oh*sh-ph+fh(col), ow*sw-pw+fw(col), ic(col)]
// with col = (fh*FW + fw)*IC + ic.  The row range is cut into `split` slices.
struct WgradParams {
    const float *X;
    const float *G;
    float *C;             // dW, or workspace base when split > 1
    int N, IH, IW, IC, OC, OH, OW, FH, FW;
    int sh, sw, ph, pw;
    int posMajor;
    int split;
    long long sliceStride;
    int tilesN;           // tiles along the K' = FH*FW*IC axis
    int xcdUnit;          // consecutive logical workgroup ids kept on one XCD
    int M;                // N*OH*OW
    int flushChunks;      // fold the running accumulator into a second one every this many stages
};

// MI355X spreads consecutive workgroup ids round-robin over its 8 XCDs, each with its own
// L2.  Map the hardware id to a logical id so that `unit` consecutive logical ids (workgroups
// that share operand tiles) run on one XCD, while units are still dealt round-robin so every
// XCD gets the same mix of long and short tiles.  Ids past the last whole group of 8 units
// keep their value.  A bijection on [0, grid).
__device__ __forceinline__ int xcd_remap(int bid, int grid, int unit)
{
    constexpr int kXcds = 8;
    const int span = kXcds * unit;
    const int whole = (grid / span) * span;
    if (bid >= whole) return bid;
    const int x = bid % kXcds, q = bid / kXcds;
    return ((q / unit) * kXcds + x) * unit + q % unit;
}

hipError_t launch_direct_fwd(const float *X, const float *W, float *Y, const Shape &s, hipStream_t st);
hipError_t launch_direct_bwd_data(const float *G, const float *W, float *dX, const Shape &s, hipStream_t st);
hipError_t launch_direct_bwd_weight(const float *X, const float *G, float *dW, const Shape &s, hipStream_t st);

// out[i] = sum_{s<split} ws[s*stride + i], combined pairwise in a fixed order.
hipError_t launch_slice_reduce(const float *ws, float *out, long long count, int split,
                               long long stride, hipStream_t st);

// bm/bn select the compiled tile; returns hipErrorInvalidValue for an unknown pair.
hipError_t launch_gather_gemm(const GatherGemmParams &p, bool bwdData, int bm, int bn, int grid,
                              hipStream_t st);
// same tiles (except 128x128), element-wise loader: any channel counts
hipError_t launch_gather_elem(const GatherGemmParams &p, bool bwdData, int bm, int bn, int grid, hipStream_t st);
hipError_t launch_wgrad(const WgradParams &p, int bm, int bn, bool xElem, int grid, hipStream_t st);

}  // namespace mi355conv
