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
constexpr int kMaxPhases = 16;    // sh*sw limit of the MFMA backward-data variant
constexpr int kMaxBalancedPositions = 256;
constexpr int kMaxBalancedTaps = 128;
constexpr int kMaxBalanceRuns = 48;

// Load balancing for launches whose workgroups differ in length (small maps in (y,x,n) order,
// where a tile's stage count is the number of filter taps / output positions inside the
// image).  Work items are ranked by descending length; the host deals them to the 256 CUs
// longest-first (workgroup ids 256 apart share a CU while the whole grid is resident) and
// writes the resulting permutation as runs: slots [idStart[r], idStart[r+1]) (see balance_slot)
// take the ranks rankStart[r], rankStart[r]+1, ...  n = 0: no dealing, ranks in id order.
struct BalanceRuns {
    int n;
    int idStart[kMaxBalanceRuns];
    int rankStart[kMaxBalanceRuns];
};

// Work items of equal length form a class (a contiguous range of ranks).  Inside a class the ranks
// enumerate the items with the operand-sharing index slowest: consecutive ranks - which the dealing
// keeps on one XCD - differ in the pixel position / row tile and share the filter slice, so a slice
// of W is fetched into an XCD's L2 once for all positions instead of once per position.
constexpr int kMaxBalanceClasses = 32;
struct BalanceClasses;   // defined after FastDiv

// Division by a launch-invariant divisor with one multiply-high and two shifts (round-up
// method of Granlund & Montgomery, "Division by invariant integers using multiplication").
// Exact for every 32-bit unsigned n and 1 <= d < 2^31.
struct FastDiv {
    unsigned mul, sh1, sh2, d;
};
inline FastDiv make_fastdiv(unsigned d)
{
    unsigned l = 0;
    while ((1ull << l) < d) ++l;                               // ceil(log2 d)
    FastDiv f;
    f.mul = (unsigned)(((1ull << 32) * ((1ull << l) - d)) / d + 1);
    f.sh1 = l < 1 ? l : 1;
    f.sh2 = l > 1 ? l - 1 : 0;
    f.d = d;
    return f;
}
__host__ __device__ inline unsigned fast_div(unsigned n, const FastDiv &f)
{
#if defined(__HIP_DEVICE_COMPILE__)
    const unsigned t = __umulhi(f.mul, n);
#else
    const unsigned t = (unsigned)(((unsigned long long)f.mul * n) >> 32);
#endif
    return (t + ((n - t) >> f.sh1)) >> f.sh2;
}

struct BalanceClasses {
    int n;                                  // 0: ranks enumerate unit by unit (no class-wise order)
    int rankStart[kMaxBalanceClasses];      // first rank of the class; INT_MAX for unused entries
    int firstUnit[kMaxBalanceClasses];      // first unit (position rank) of the class
    FastDiv divRows[kMaxBalanceClasses];    // by units of the class * row tiles per unit
};

// ---- gather-GEMM (forward and backward-data) ------------------------------------------
// C[row, col] = sum over taps t of the tile's tap set, channels c:
//                 A[n, y0(row)+dy(t), x0(row)+dx(t), c] * Wt(t, c, col)
// Forward : A = X,  rows = output pixels,  cols = oc, c = ic, taps (u,v) = (fh,fw), dy = u.
// Bwd-data: A = dY, rows = input pixels of one stride phase (ra,rb), cols = ic, c = oc,
//           taps fh = ra + sh*u, fw = rb + sw*v, dy = -u, dx = -v.
struct GatherPhase {
    int tileStart;        // first row tile of the phase
    int ra, rb;           // residues of (ih+ph) % sh, (iw+pw) % sw   (0 for forward)
    int y0, x0;           // first destination row / column of the phase
    int dh, dw;           // destination rows / columns in the phase
    int nU, nV;           // taps of the phase along h and w
    int pad_[3];
    FastDiv divHW, divW;  // by dh*dw and by dw
};

struct GatherGemmParams {
    const float *A;
    const float *B;
    float *C;             // output tensor, or workspace base when split > 1
    unsigned aBytes, bBytes;  // sizes of A and B in bytes (both below 2^31): buffer-load range checks
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
    // Load balancing for (y,x,n) row order on small maps, where a tile's work is the number of
    // taps inside the image at its position (4, 6 or 9 of 9 for a padded 3x3 filter): the
    // workgroup id is mapped to a rank (runs), and ranks enumerate the row tiles position by
    // position in posOrder (most taps first).  0 = off.
    int balance;
    int rowTilesPerPos;   // Nimg / BM
    // epilogue of the unsliced launch: out = act(acc + bias[col]); epilogue == 0: plain store
    int epilogue;
    float slope;
    const float *bias;    // may be null
    FastDiv divN;         // by Nimg
    FastDiv divTilesN, divSplit, divRowTilesPerPos, divChunksPerTap;   // chunks per tap = SC / kBK
    FastDiv divDHW, divDW;   // by DH*DW and DW: the row decode of single-phase launches (forward, unit-stride backward-data)
    FastDiv divXcdUnit;      // by xcdUnit
    int xcdWhole;            // workgroup ids below this are remapped (a whole number of 8 * xcdUnit)
    int grid;                // workgroups of the launch
    int runsN;               // runs.n, among the scalars fetched first
    int classesN;            // classes.n, likewise
    // Region-wise order ((y,x,n) rows, one phase): XCD x = hardware id % 8 owns the product of a spatial
    // region of the map (halves or quarters, mirrored so that every region looks like the first), a group
    // of row tiles (images) and a group of (slice, column tile) pairs; regLut holds one byte per XCD:
    // bits 0-2 column group, 3-5 image group, 6 mirrored in x, 7 mirrored in y.  Inside an XCD the tiles
    // are ranked position by position (posOrder: positions of the first region, most taps first) and,
    // while the whole launch is resident, dealt to its 32 CUs in a snake (ranks 0..31, 63..32, ...).
    int regional;
    int regSnake;
    int regLocal;            // workgroups per XCD = grid / 8
    int regPerPos;           // tiles per position inside one XCD = regRowTiles * regCsPer
    int regCsPer;            // (slice, column tile) pairs per XCD
    int regRowTiles;         // row tiles per position and image group
    int regW;                // width of a region in positions
    unsigned regLutLo, regLutHi;
    FastDiv divRegPerPos, divRegCsPer, divRegW;
    // > 0: slice s walks the source-channel chunks [s*chunksPerSlice, (s+1)*chunksPerSlice) of every tap
    // (slices differ in channels, so a slice reads a 1/split part of both operands); 0: the list of
    // stages (tap-major) is cut into split equal parts.
    int chunksPerSlice;
    int phaseStart[kMaxPhases];   // first row tile of each phase; INT_MAX past the last phase
    GatherPhase phase[kMaxPhases];
    BalanceRuns runs;
    unsigned char posOrder[kMaxBalancedPositions];
    BalanceClasses classes;
};

static_assert(sizeof(GatherGemmParams) <= 4096, "kernel arguments are limited to 4 KB");

// The scalar fields of GatherGemmParams held in SGPRs from the kernel's first instructions on:
// the compiler otherwise fetches each kernel argument where it is first used, one dependent
// scalar load after the other all through the prologue.  Field names match GatherGemmParams, so
// code templated on the parameter type takes either.
struct GatherView {
    const float *A;
    const float *B;
    float *C;
    unsigned aBytes, bBytes;
    int Nimg, SH, SW, SC, DH, DW, DC, FH, FW, sh, sw, ph, pw;
    int posMajor, split;
    long long sliceStride;
    int tilesN, xcdUnit, nPhases, balance, rowTilesPerPos, epilogue;
    float slope;
    const float *bias;
    FastDiv divN, divTilesN, divSplit, divRowTilesPerPos, divChunksPerTap, divDHW, divDW, divXcdUnit;
    int xcdWhole, grid, runsN, classesN;
    int regional, regSnake, regLocal, regPerPos, regCsPer, regRowTiles, regW;
    unsigned regLutLo, regLutHi;
    FastDiv divRegPerPos, divRegCsPer, divRegW;
    int chunksPerSlice;
    const int *phaseStart;
    const GatherPhase *phase;
    const BalanceRuns &runs;
    const unsigned char *posOrder;
};
#if defined(__HIPCC__)
#define MI355CONV_PIN(x) asm volatile("" : "+s"(x))
__device__ __forceinline__ GatherView gather_view(const GatherGemmParams &p)
{
    GatherView v{p.A, p.B, p.C, p.aBytes, p.bBytes, p.Nimg, p.SH, p.SW, p.SC, p.DH, p.DW, p.DC, p.FH, p.FW,
                 p.sh, p.sw, p.ph, p.pw, p.posMajor, p.split, p.sliceStride, p.tilesN, p.xcdUnit, p.nPhases,
                 p.balance, p.rowTilesPerPos, p.epilogue, p.slope, p.bias, p.divN, p.divTilesN, p.divSplit, p.divRowTilesPerPos,
                 p.divChunksPerTap, p.divDHW, p.divDW, p.divXcdUnit, p.xcdWhole, p.grid, p.runsN, p.classesN,
                 p.regional, p.regSnake, p.regLocal, p.regPerPos, p.regCsPer, p.regRowTiles, p.regW, p.regLutLo, p.regLutHi,
                 p.divRegPerPos, p.divRegCsPer, p.divRegW, p.chunksPerSlice, p.phaseStart, p.phase, p.runs, p.posOrder};
    MI355CONV_PIN(v.A); MI355CONV_PIN(v.B); MI355CONV_PIN(v.C);
    MI355CONV_PIN(v.aBytes); MI355CONV_PIN(v.bBytes);
    MI355CONV_PIN(v.Nimg); MI355CONV_PIN(v.SH); MI355CONV_PIN(v.SW); MI355CONV_PIN(v.SC);
    MI355CONV_PIN(v.DH); MI355CONV_PIN(v.DW); MI355CONV_PIN(v.DC); MI355CONV_PIN(v.FH); MI355CONV_PIN(v.FW);
    MI355CONV_PIN(v.sh); MI355CONV_PIN(v.sw); MI355CONV_PIN(v.ph); MI355CONV_PIN(v.pw);
    MI355CONV_PIN(v.posMajor); MI355CONV_PIN(v.split); MI355CONV_PIN(v.sliceStride);
    MI355CONV_PIN(v.tilesN); MI355CONV_PIN(v.xcdUnit); MI355CONV_PIN(v.nPhases);
    MI355CONV_PIN(v.balance); MI355CONV_PIN(v.rowTilesPerPos);
    MI355CONV_PIN(v.divN.mul); MI355CONV_PIN(v.divN.sh1); MI355CONV_PIN(v.divN.sh2);
    MI355CONV_PIN(v.divTilesN.mul); MI355CONV_PIN(v.divTilesN.sh1); MI355CONV_PIN(v.divTilesN.sh2);
    MI355CONV_PIN(v.divSplit.mul); MI355CONV_PIN(v.divSplit.sh1); MI355CONV_PIN(v.divSplit.sh2);
    MI355CONV_PIN(v.divChunksPerTap.mul); MI355CONV_PIN(v.divChunksPerTap.sh1); MI355CONV_PIN(v.divChunksPerTap.sh2);
    MI355CONV_PIN(v.divRowTilesPerPos.mul); MI355CONV_PIN(v.divRowTilesPerPos.sh1); MI355CONV_PIN(v.divRowTilesPerPos.sh2);
    MI355CONV_PIN(v.divDHW.mul); MI355CONV_PIN(v.divDHW.sh1); MI355CONV_PIN(v.divDHW.sh2);
    MI355CONV_PIN(v.divDW.mul); MI355CONV_PIN(v.divDW.sh1); MI355CONV_PIN(v.divDW.sh2);
    MI355CONV_PIN(v.divXcdUnit.mul); MI355CONV_PIN(v.divXcdUnit.sh1); MI355CONV_PIN(v.divXcdUnit.sh2);
    MI355CONV_PIN(v.xcdWhole); MI355CONV_PIN(v.grid); MI355CONV_PIN(v.runsN); MI355CONV_PIN(v.classesN);
    MI355CONV_PIN(v.regional); MI355CONV_PIN(v.regSnake); MI355CONV_PIN(v.regLocal); MI355CONV_PIN(v.regPerPos);
    MI355CONV_PIN(v.regCsPer); MI355CONV_PIN(v.regRowTiles); MI355CONV_PIN(v.regW);
    MI355CONV_PIN(v.regLutLo); MI355CONV_PIN(v.regLutHi);
    MI355CONV_PIN(v.divRegPerPos.mul); MI355CONV_PIN(v.divRegPerPos.sh1); MI355CONV_PIN(v.divRegPerPos.sh2);
    MI355CONV_PIN(v.divRegCsPer.mul); MI355CONV_PIN(v.divRegCsPer.sh1); MI355CONV_PIN(v.divRegCsPer.sh2);
    MI355CONV_PIN(v.divRegW.mul); MI355CONV_PIN(v.divRegW.sh1); MI355CONV_PIN(v.divRegW.sh2);
    MI355CONV_PIN(v.chunksPerSlice);
    return v;
}
#endif

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
    // fast variant only
    unsigned xBytes, gBytes;          // tensor sizes in bytes (below 2^31): buffer-load range checks
    FastDiv divOHOW, divOW, divN;     // by OH*OW, OW and N
    FastDiv divIC, divFW, divTilesN, divSplit;
    // (oh,ow,n) order: a tile's live stages are the output positions at which its filter tap is
    // inside the image.  With balance set (needs IC % BN == 0: one tap per tile) ranks enumerate
    // the tiles tap by tap in tapOrder (most positions first); see BalanceRuns.
    int balance;
    int tilesPerTap;      // IC / BN
    int tilesM;
    FastDiv divTilesPerTap, divPerTap;   // by tilesPerTap and by tilesPerTap * tilesM * split
    int grid;             // workgroups of the launch
    int runsN;            // runs.n, among the scalars fetched first
    int xcdWhole;         // workgroup ids below this are remapped (a whole number of 8 * xcdUnit)
    FastDiv divXcdUnit;
    // Group-wise order of the (oh,ow,n) launches: XCD x = hardware id % 8 owns a group of output-channel
    // tiles (x % A), of input-channel tiles ((x / A) % B) and of slices (x / (A*B)), A*B*S = 8, all powers
    // of two, for every tap; regShift = log2 A | log2 B << 8.  Inside an XCD the tiles are ranked tap by
    // tap (tapOrder) and dealt to its 32 CUs through `runs` (slots = place of the id on the XCD).
    // divPerTap then divides by the tiles of a tap on one XCD.
    int regional;
    int regShift;
    int regOcTiles;       // output-channel tiles per group
    FastDiv divRegIc, divRegSplit;   // by input-channel tiles per group, by slices per group
    BalanceRuns runs;
    unsigned char tapOrder[256];   // kMaxBalancedTaps entries used; sized for one 4-byte load per lane
};

// Scalar fields of WgradParams in SGPRs from the kernel's first instructions on (see GatherView).
struct WgradView {
    const float *X;
    const float *G;
    float *C;
    int N, IH, IW, IC, OC, OH, OW, FH, FW, sh, sw, ph, pw;
    int posMajor, split;
    long long sliceStride;
    int tilesN, xcdUnit, M, flushChunks;
    unsigned xBytes, gBytes;
    FastDiv divOHOW, divOW, divN, divIC, divFW, divTilesN, divSplit;
    int balance, tilesPerTap, tilesM;
    FastDiv divTilesPerTap, divPerTap;
    int grid, runsN, xcdWhole;
    FastDiv divXcdUnit;
    int regional, regShift, regOcTiles;
    FastDiv divRegIc, divRegSplit;
    const BalanceRuns &runs;
    const unsigned char *tapOrder;
};
#if defined(__HIPCC__)
__device__ __forceinline__ void pin_fastdiv(FastDiv &f)
{
    MI355CONV_PIN(f.mul); MI355CONV_PIN(f.sh1); MI355CONV_PIN(f.sh2);
}
__device__ __forceinline__ WgradView wgrad_view(const WgradParams &p)
{
    WgradView v{p.X, p.G, p.C, p.N, p.IH, p.IW, p.IC, p.OC, p.OH, p.OW, p.FH, p.FW, p.sh, p.sw, p.ph, p.pw,
                p.posMajor, p.split, p.sliceStride, p.tilesN, p.xcdUnit, p.M, p.flushChunks, p.xBytes, p.gBytes,
                p.divOHOW, p.divOW, p.divN, p.divIC, p.divFW, p.divTilesN, p.divSplit, p.balance, p.tilesPerTap,
                p.tilesM, p.divTilesPerTap, p.divPerTap, p.grid, p.runsN, p.xcdWhole, p.divXcdUnit,
                p.regional, p.regShift, p.regOcTiles, p.divRegIc, p.divRegSplit, p.runs, p.tapOrder};
    MI355CONV_PIN(v.X); MI355CONV_PIN(v.G); MI355CONV_PIN(v.C);
    MI355CONV_PIN(v.N); MI355CONV_PIN(v.IH); MI355CONV_PIN(v.IW); MI355CONV_PIN(v.IC); MI355CONV_PIN(v.OC);
    MI355CONV_PIN(v.OH); MI355CONV_PIN(v.OW); MI355CONV_PIN(v.FH); MI355CONV_PIN(v.FW);
    MI355CONV_PIN(v.sh); MI355CONV_PIN(v.sw); MI355CONV_PIN(v.ph); MI355CONV_PIN(v.pw);
    MI355CONV_PIN(v.posMajor); MI355CONV_PIN(v.split); MI355CONV_PIN(v.sliceStride);
    MI355CONV_PIN(v.tilesN); MI355CONV_PIN(v.xcdUnit); MI355CONV_PIN(v.M); MI355CONV_PIN(v.flushChunks);
    MI355CONV_PIN(v.xBytes); MI355CONV_PIN(v.gBytes);
    pin_fastdiv(v.divOHOW); pin_fastdiv(v.divOW); pin_fastdiv(v.divN); pin_fastdiv(v.divIC);
    pin_fastdiv(v.divFW); pin_fastdiv(v.divTilesN); pin_fastdiv(v.divSplit);
    MI355CONV_PIN(v.balance); MI355CONV_PIN(v.tilesPerTap); MI355CONV_PIN(v.tilesM);
    pin_fastdiv(v.divTilesPerTap); pin_fastdiv(v.divPerTap); pin_fastdiv(v.divXcdUnit);
    MI355CONV_PIN(v.grid); MI355CONV_PIN(v.runsN); MI355CONV_PIN(v.xcdWhole);
    MI355CONV_PIN(v.regional); MI355CONV_PIN(v.regShift); MI355CONV_PIN(v.regOcTiles);
    pin_fastdiv(v.divRegIc); pin_fastdiv(v.divRegSplit);
    MI355CONV_PIN(v.divPerTap.d); MI355CONV_PIN(v.divRegIc.d); MI355CONV_PIN(v.divRegSplit.d);
    return v;
}
#endif

// ---- backward-data for very few input channels (kernel_small_ic.hip) ----------------------------
struct SmallIcParams {
    const float *G;       // dY [N, OH, OW, OC]
    const float *W;       // [OC, FH, FW, IC]
    float *dX;            // [N, IH, IW, IC]; the forward kernel writes Y [N, OH, OW, OC] through it
    unsigned gBytes, wBytes;
    int N, IH, IW, IC, OC, OH, OW, FH, FW, ph, pw;
    // backward-weight only
    const float *X;       // [N, IH, IW, IC]
    float *C;             // dW, or workspace base when split > 1
    unsigned xBytes;
    int sh, sw, split, M;
    long long sliceStride;
    FastDiv divOHOW, divOW, divIC, divFW;
    // forward only: X holds unsigned bytes, converted on load as (float)byte * scale
    int u8;
    float scale;
    // forward only: out = act(acc + bias[oc]) before the store (epilogue == 0: plain store)
    int epilogue;
    float slope;
    const float *bias;    // may be null
};

// MI355X spreads consecutive workgroup ids round-robin over its 8 XCDs, each with its own
// L2.  Map the hardware id to a logical id so that `unit` consecutive logical ids (workgroups
// that share operand tiles) run on one XCD, while units are still dealt round-robin so every
// XCD gets the same mix of long and short tiles.  Ids past the last whole group of 8 units
// keep their value.  A bijection on [0, grid).
// Column of the dealing that hardware workgroup id `bid` belongs to, as an id: within every
// whole lap of 256 ids the 32 ids that run on one XCD (bid % 8 equal) become neighbours, so
// that a run of consecutive ranks - tiles that share operand rows - stays on one XCD and its
// L2.  Ids of the last, partial lap keep their value.  The host uses the same function.
__host__ __device__ __forceinline__ int balance_slot(int bid, int grid)
{
    const int lap = bid >> 8;
    if ((lap + 1) * 256 > grid) return bid;
    const int c = bid & 255;
    return (lap << 8) + (c & 7) * 32 + (c >> 3);
}

// ---- region-wise / group-wise orders: the arithmetic between workgroup id and tile ------------------
// Shared by the kernels and by the host (conv2d_query_tile, which the CPU tests sweep over shapes to
// check that every plan maps the workgroup ids one-to-one onto the tiles).  P is GatherGemmParams /
// GatherView resp. WgradParams / WgradView.

// Gather operators, first half: hardware id -> XCD, rank of the tile's position on that XCD (index
// into posOrder) and place among that position's tiles.
template <class P>
__host__ __device__ inline void region_wise_place(const P &p, int bid, int *xcd, int *posRank, int *inner)
{
    const int q = bid >> 3;
    int lr = q;
    if (p.regSnake) {   // ids 32 apart share a CU: every other lap of 32 is dealt backwards
        const int lap = q >> 5;
        int c = q & 31;
        const int left = p.regLocal - (lap << 5);
        const int w = left < 32 ? left : 32;
        if (lap & 1) c = w - 1 - c;
        lr = (lap << 5) + c;
    }
    *xcd = bid & 7;
    *posRank = (int)fast_div((unsigned)lr, p.divRegPerPos);
    *inner = lr - *posRank * p.regPerPos;
}
// Second half: lpos = posOrder[posRank], a position of the first region -> row tile, column tile, slice.
template <class P>
__host__ __device__ inline void region_wise_tile(const P &p, int xcd, int lpos, int inner, int *tmGlobal, int *tn, int *slice)
{
    const int ly = (int)fast_div((unsigned)lpos, p.divRegW);
    const int lx = lpos - ly * p.regW;
    const unsigned lut = ((xcd < 4 ? p.regLutLo : p.regLutHi) >> ((xcd & 3) * 8)) & 255u;
    const int y = (lut & 128u) ? p.DH - 1 - ly : ly;
    const int x = (lut & 64u) ? p.DW - 1 - lx : lx;
    const int rt = (int)fast_div((unsigned)inner, p.divRegCsPer);
    const int cs = (int)(lut & 7u) * p.regCsPer + (inner - rt * p.regCsPer);
    *slice = (int)fast_div((unsigned)cs, p.divTilesN);
    *tn = cs - *slice * p.tilesN;
    *tmGlobal = (y * p.DW + x) * p.rowTilesPerPos + (int)((lut >> 3) & 7u) * p.regRowTiles + rt;
}
// Backward-weight: XCD and rank on that XCD (after the dealing) -> rank of the tap (index into
// tapOrder), input-channel tile inside the tap, output-channel tile, slice.
template <class P>
__host__ __device__ inline void group_wise_tile(const P &p, int xcd, int lr, int *tapRank, int *icTile, int *tmo, int *slice)
{
    const int perTap = (int)p.divPerTap.d, icTiles = (int)p.divRegIc.d, slices = (int)p.divRegSplit.d;
    *tapRank = (int)fast_div((unsigned)lr, p.divPerTap);
    const int inner = lr - *tapRank * perTap;
    const int r2 = (int)fast_div((unsigned)inner, p.divRegIc);
    const int lgA = p.regShift & 255, lgB = p.regShift >> 8;
    const int ga = xcd & ((1 << lgA) - 1), gb = (xcd >> lgA) & ((1 << lgB) - 1), gs = xcd >> (lgA + lgB);
    *icTile = gb * icTiles + (inner - r2 * icTiles);
    const int ocl = (int)fast_div((unsigned)r2, p.divRegSplit);
    *tmo = ga * p.regOcTiles + ocl;
    *slice = gs * slices + (r2 - ocl * slices);
}

#if defined(__HIPCC__)   // device-side decode of the workgroup id
// Rank of workgroup id `bid` under the host's longest-first dealing.  Lane i looks at run i
// (there are fewer than 64): the run is the last one that starts at or before the slot.
__device__ __forceinline__ int balanced_rank(int bid, int grid, const BalanceRuns &b)
{
    static_assert(kMaxBalanceRuns < 64, "one lane per run");
    const int slot = balance_slot(bid, grid);
    const int lane = threadIdx.x & 63;
    const int start = lane < b.n ? b.idStart[lane] : 0x7fffffff;
    const int r = __popcll(__ballot(slot >= start)) - 1;   // idStart[0] == 0
    return b.rankStart[r] + (slot - b.idStart[r]);
}

// The per-lane pieces of the workgroup-id decode (run table of the dealing, order of positions
// or taps), requested by every wave with its very first instructions so that they travel
// together with the scalar kernel arguments instead of one dependent load after the other.
// Unused run entries hold idStart = INT_MAX (the host fills them), so no count is needed.
struct BalancePrefetch {
    int runId, runRank;   // lane i: run i
    unsigned order4;      // lane i: entries 4i .. 4i+3 of the 256-entry order table
    int clsRank, clsFirst;                      // lane i: class i
    unsigned clsMul, clsSh1, clsSh2, clsD;      // lane i: class i's divisor
};
__device__ __forceinline__ BalancePrefetch balance_prefetch(const BalanceRuns &runs, const unsigned char *order)
{
    static_assert(kMaxBalanceRuns < 64, "one lane per run");
    const int lane = threadIdx.x & 63;
    BalancePrefetch b;
    b.runId = lane < kMaxBalanceRuns ? runs.idStart[lane] : 0x7fffffff;
    b.runRank = lane < kMaxBalanceRuns ? runs.rankStart[lane] : 0;
    b.order4 = reinterpret_cast<const unsigned *>(order)[lane];
    b.clsRank = 0x7fffffff;
    b.clsFirst = 0;
    b.clsMul = b.clsSh1 = b.clsSh2 = b.clsD = 0;
    return b;
}
__device__ __forceinline__ void balance_prefetch_classes(BalancePrefetch &b, const BalanceClasses &c)
{
    static_assert(kMaxBalanceClasses <= 64, "one lane per class");
    const int lane = threadIdx.x & 63;
    if (lane < kMaxBalanceClasses) {
        b.clsRank = c.rankStart[lane];
        b.clsFirst = c.firstUnit[lane];
        b.clsMul = c.divRows[lane].mul; b.clsSh1 = c.divRows[lane].sh1; b.clsSh2 = c.divRows[lane].sh2; b.clsD = c.divRows[lane].d;
    }
}
// Class of a rank and, from there, the rank's place inside it: q = rank - first rank of the class,
// inner = q / rows (rows = units of the class * row tiles per unit), row = q % rows.
__device__ __forceinline__ void balance_class_decode(const BalancePrefetch &b, int rank, int *firstUnit, int *inner, int *row)
{
    const int c = __popcll(__ballot(rank >= b.clsRank)) - 1;   // rankStart[0] == 0, unused entries INT_MAX
    const int q = rank - __builtin_amdgcn_readlane(b.clsRank, c);
    FastDiv f;
    f.mul = (unsigned)__builtin_amdgcn_readlane((int)b.clsMul, c);
    f.sh1 = (unsigned)__builtin_amdgcn_readlane((int)b.clsSh1, c);
    f.sh2 = (unsigned)__builtin_amdgcn_readlane((int)b.clsSh2, c);
    f.d = (unsigned)__builtin_amdgcn_readlane((int)b.clsD, c);
    *firstUnit = __builtin_amdgcn_readlane(b.clsFirst, c);
    *inner = (int)fast_div((unsigned)q, f);
    *row = q - *inner * (int)f.d;
}
__device__ __forceinline__ int balanced_rank(int bid, int grid, const BalancePrefetch &b)
{
    const int slot = balance_slot(bid, grid);
    const int r = __popcll(__ballot(slot >= b.runId)) - 1;   // idStart[0] == 0
    return __builtin_amdgcn_readlane(b.runRank, r) + (slot - __builtin_amdgcn_readlane(b.runId, r));
}
// The same look-up for a dealing inside one XCD: the slot is the id's place on the XCD (id / 8).
__device__ __forceinline__ int balanced_rank_local(int slot, const BalancePrefetch &b)
{
    const int r = __popcll(__ballot(slot >= b.runId)) - 1;   // idStart[0] == 0
    return __builtin_amdgcn_readlane(b.runRank, r) + (slot - __builtin_amdgcn_readlane(b.runId, r));
}
__device__ __forceinline__ int balance_order(const BalancePrefetch &b, int rank)   // rank < 256, uniform
{
    return (int)((__builtin_amdgcn_readlane((int)b.order4, rank >> 2) >> ((rank & 3) * 8)) & 255u);
}

// xcd_remap with the division by `unit` and the remapped range precomputed on the host
__device__ __forceinline__ int xcd_remap_fast(int bid, int whole, int unit, const FastDiv &divUnit)
{
    if (bid >= whole) return bid;
    const int x = bid & 7, q = bid >> 3;
    const int g = (int)fast_div((unsigned)q, divUnit);
    return (g * 8 + x) * unit + (q - g * unit);
}

__device__ __forceinline__ int xcd_remap(int bid, int grid, int unit)
{
    constexpr int kXcds = 8;
    const int span = kXcds * unit;
    const int whole = (grid / span) * span;
    if (bid >= whole) return bid;
    const int x = bid % kXcds, q = bid / kXcds;
    return ((q / unit) * kXcds + x) * unit + q % unit;
}
#endif   // __HIPCC__

// ---- what each launcher takes, as host-side predicates ---------------------------------------
// The planner checks every plan against the same predicate that the launcher applies, so a plan
// that a launcher would refuse is caught on the host before any HIP call (and by a CPU test
// that sweeps shapes through conv2d_query_plan).
inline bool gather_gemm_accepts(int srcC, int dstC, bool bwdData, int bm, int bn)
{
    if (srcC % 4 != 0) return false;
    if (bwdData && dstC % 4 != 0) return bm == 128 && bn == 32;   // filter columns by 4-byte loads
    return (bm == 128 && (bn == 128 || bn == 64 || bn == 32)) || (bm == 64 && bn == 64);
}
inline bool gather_elem_accepts(int bm, int bn)
{
    return (bm == 128 && (bn == 64 || bn == 32)) || (bm == 64 && bn == 64);
}
// Generic backward-weight kernel: (oh,ow,n) order needs stages that sit on one output position.
inline bool wgrad_accepts(int N, int IC, int OC, int posMajor, bool xElem, int bm, int bn)
{
    if (OC % 4 != 0) return false;
    if (xElem) return !posMajor && bn == 64 && (bm == 64 || bm == 128);
    if (IC % 4 != 0) return false;
    if (posMajor && N % kBK != 0) return false;
    return (bm == 128 || bm == 64) && (bn == 128 || bn == 64);
}
// Fast backward-weight kernel: "aligned" maps only - OW divides 32 and OH*OW divides or is a multiple
// of 32, or OW is a multiple of 32 (wide rows; (n,oh,ow) order only).  (oh,ow,n) order keeps a 64-bit
// mask of output positions and needs N to be a multiple of 32.
inline bool wgrad_fast_accepts(int N, int OH, int OW, int IC, int OC, int posMajor, int bm, int bn)
{
    const int ohow = OH * OW;
    const bool narrow = kBK % OW == 0 && (ohow % kBK == 0 || kBK % ohow == 0);
    const bool wide = OW > kBK && OW % kBK == 0;
    if (!narrow && !wide) return false;
    if (IC % 4 != 0 || OC % 4 != 0) return false;
    if (posMajor && (wide || N % kBK != 0 || ohow > 64)) return false;
    return ((bm == 128 || bm == 64) && (bn == 128 || bn == 64)) || (bm == 32 && bn == 128);
}
inline bool bwd_data_small_ic_accepts(int IC, int OC, int FH, int FW, int sh, int sw)
{
    return sh == 1 && sw == 1 && IC <= 4 && FH * FW * IC <= 32 && OC % kBK == 0 && (4 + FH - 1) * (32 + FW - 1) <= 224;
}
inline bool patch_small_ic_accepts(int IC, int FH, int FW) { return FH * FW * IC <= 32; }   // forward, backward-weight

// Once per device, outside any stream capture: raise the dynamic-LDS limit of the kernel
// instantiations whose tiles exceed the 64 KB a kernel gets by default.
hipError_t prepare_gather_gemm();
hipError_t prepare_wgrad();
hipError_t prepare_wgrad_fast();

hipError_t launch_direct_fwd(const float *X, const float *W, float *Y, const Shape &s, hipStream_t st);
hipError_t launch_direct_bwd_data(const float *G, const float *W, float *dX, const Shape &s, hipStream_t st);
hipError_t launch_direct_bwd_weight(const float *X, const float *G, float *dW, const Shape &s, hipStream_t st);

// out[i] = sum_{s<split} ws[s*stride + i], combined pairwise in a fixed order.
// With bias / slope (cols = channel count of the output's last axis, cols > 0):
// out[i] = act(sum + bias[i % cols]).
hipError_t launch_slice_reduce(const float *ws, float *out, long long count, int split,
                               long long stride, hipStream_t st, const float *bias = nullptr,
                               float slope = 1.f, int cols = 0);
// out[i] = act(out[i] + bias[i % cols]) in place (after the direct forward kernel)
hipError_t launch_bias_act(float *out, long long count, const float *bias, float slope, int cols, hipStream_t st);

// bm/bn select the compiled tile; returns hipErrorInvalidValue for an unknown pair.
hipError_t launch_gather_gemm(const GatherGemmParams &p, bool bwdData, int bm, int bn, int grid,
                              hipStream_t st);
// same tiles (except 128x128), element-wise loader: any channel counts
hipError_t launch_gather_elem(const GatherGemmParams &p, bool bwdData, int bm, int bn, int grid, hipStream_t st);
hipError_t launch_wgrad(const WgradParams &p, int bm, int bn, bool xElem, int grid, hipStream_t st);
// Aligned maps (OW divides 32 and OH*OW divides or is a multiple of 32; or OW a multiple of 32, row-major
// order only), IC % 4 == 0, OC % 4 == 0,
// tensors below 2^31 bytes.
hipError_t launch_wgrad_fast(const WgradParams &p, int bm, int bn, int grid, hipStream_t st);
// unit stride, FH*FW*IC <= 32, IC <= 4, OC % 32 == 0, (4+FH-1)*(32+FW-1) <= 224, tensors below 2^31 bytes
hipError_t launch_bwd_data_small_ic(const SmallIcParams &p, hipStream_t st);
// FH*FW*IC <= 32, any stride; grid = ceil(OC / 64) * split
hipError_t launch_wgrad_small_ic(const SmallIcParams &p, hipStream_t st);
// FH*FW*IC <= 32, any stride, any OC; X, W, dX (= Y), M, strides, divisors set
hipError_t launch_fwd_small_ic(const SmallIcParams &p, hipStream_t st);

}  // namespace mi355conv
