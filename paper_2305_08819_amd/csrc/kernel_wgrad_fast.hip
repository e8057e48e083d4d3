// Backward-weight, fast variant for "aligned" feature maps (every CIFAR-pyramid shape).
//
// Same GEMM view and MFMA operand scheme as wgrad_kernel:
//   dW[oc, col] = sum_m G[m, oc] * Xg[m, col],  col = (fh*FW + fw)*IC + ic,
// both LDS tiles are [k = m][channel], operands read with 4-byte LDS loads.
//
// What makes it fast: on this chip fp32 MFMA and VALU instructions share the SIMD's issue
// cycles, so the loop is built to contain almost no VALU work.
//  * A stage is kBK = 32 consecutive rows m.  When OW divides 32 and OH*OW divides (or is a
//    multiple of) 32, row r of a stage is always the same (image offset, row offset, column)
//    relative to the stage's first pixel.  Each thread's part of the X address and its
//    column validity are therefore fixed for the whole kernel; per stage only the uniform
//    (n0, oh0) changes, which costs one add, two compares and a select per 16-byte load.
//  * G rows are consecutive in memory: fixed VGPR offset + per-stage SGPR offset, no VALU.
//  * Loads are raw buffer loads: rows past the end or in the padding get an out-of-range
//    offset and read zeros, so there is no branch and no zero-select.
//  * With (oh,ow,n) row order (maps of at most 64 positions) a stage sits on one output
//    position; each thread keeps a 64-bit mask of the positions where its filter tap is inside
//    the image, and whole stages that are padding for every tap of the tile are skipped with
//    a find-first-set on the tile's mask (small-feature-map operator, Sec. IV).
//  * The row order is a template parameter, so the loop carries no branch on it.
//  * Loads run two stages ahead through two register sets; memory instructions are spread
//    between MFMA steps; fragments are read three MFMA steps ahead; one barrier per stage.
// Accuracy: the accumulator is folded into a second one every `flushChunks` stages (512
// products), so no fp32 chain is longer than that however long the slice is.
#include <hip/hip_runtime.h>
#include "gather_common.h"

namespace mi355conv {

namespace {
template <int BM, int BN>
struct WF {
    static constexpr int WAVES_M = BM >= 64 ? 2 : 1, WAVES_N = 4 / WAVES_M;   // a 32-row tile is one block row
    static constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
    static constexpr int MB = WTM / 32, NB = WTN / 32;
    static constexpr int LDG = BM + 8, LDX = BN + 8;
    static constexpr int G_TPR = BM / 4, G_RPP = kThreads / G_TPR, PG = kBK / G_RPP;
    static constexpr int X_TPR = BN / 4, X_RPP = kThreads / X_TPR, PX = kBK / X_RPP;
    static constexpr int G_STAGE = kBK * LDG, X_STAGE = kBK * LDX;
    static constexpr size_t SMEM_BYTES = 2 * (G_STAGE + X_STAGE) * sizeof(float);
};
}  // namespace

// PM: rows in (oh, ow, n) order with N a multiple of 32 and OH*OW <= 64, so that a stage sits on
// one output position and positions fit 64-bit masks.
// WIDE (with PM false): OW is a multiple of 32 instead of a divisor, so a stage is 32 neighbouring
// pixels of one output row that starts at column ow0 = 0, 32, 64, ...: the column validity of a
// thread's tap then depends on ow0 and is tested per stage (two more VALU per load).
template <int BM, int BN, bool PM, bool WIDE = false>
__global__ __launch_bounds__(kThreads, (BM * BN >= 128 * 128) ? 1 : (BM * BN <= 64 * 64) ? 4 : 2) void wgrad_fast_kernel(const WgradParams params)
{
    using T = WF<BM, BN>;
    extern __shared__ f4 smem_raw[];
    float *Gs = reinterpret_cast<float *>(smem_raw);
    float *Xs = Gs + 2 * T::G_STAGE;

    const BalancePrefetch pre = balance_prefetch(params.runs, params.tapOrder);   // in flight with the scalar arguments
    const WgradView p = wgrad_view(params);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int tn, tmo, slice;
    if (PM && p.regional) {
        // group-wise order: the XCD fixes the groups of output-channel tiles, input-channel tiles and
        // slices; the id's place on the XCD gives the tile's rank there (tap by tap, longest taps first)
        const int xcd = blockIdx.x & 7, q = blockIdx.x >> 3;
        const int lr = p.runsN ? balanced_rank_local(q, pre) : q;
        int tapRank, icTile;
        group_wise_tile(p, xcd, lr, &tapRank, &icTile, &tmo, &slice);
        tn = balance_order(pre, tapRank) * p.tilesPerTap + icTile;
    } else if (PM && p.balance) {   // tiles enumerated tap by tap, taps with the most live positions first
        const int rank = p.runsN ? balanced_rank(blockIdx.x, p.grid, pre) : (int)blockIdx.x;
        const int tapRank = (int)fast_div((unsigned)rank, p.divPerTap);
        const int inner = rank - tapRank * (p.tilesPerTap * p.tilesM * p.split);
        const int r2 = (int)fast_div((unsigned)inner, p.divTilesPerTap);
        tn = balance_order(pre, tapRank) * p.tilesPerTap + (inner - r2 * p.tilesPerTap);
        tmo = (int)fast_div((unsigned)r2, p.divSplit);
        slice = r2 - tmo * p.split;
    } else {
        const int bid = xcd_remap_fast(blockIdx.x, p.xcdWhole, p.xcdUnit, p.divXcdUnit);
        const int rest = (int)fast_div((unsigned)bid, p.divTilesN);
        tn = bid - rest * p.tilesN;
        tmo = (int)fast_div((unsigned)rest, p.divSplit);
        slice = rest - tmo * p.split;
    }
    const int oc0 = tmo * BM, col0 = tn * BN;
    const int Ktot = p.FH * p.FW * p.IC;
    const int ohow = p.OH * p.OW;

    const int chunksTotal = (p.M + kBK - 1) / kBK;
    int ch0 = slice * chunksTotal / p.split;          // (oh,ow,n) order: replaced below by a cut of the live stages
    int ch1 = (slice + 1) * chunksTotal / p.split;

    constexpr int kOutOfRange = (int)0x80000000;
    const __amdgpu_buffer_rsrc_t rsrcX =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(p.X), 0, (int)p.xBytes, 0x00020000);

    // ---- per-thread constants ---------------------------------------------------------------
    const int gSeg = tid % T::G_TPR, gRow = tid / T::G_TPR;
    const int xSeg = tid % T::X_TPR, xRow = tid / T::X_TPR;
    const int gOc = oc0 + gSeg * 4;
    const int xCol = col0 + xSeg * 4;
    const bool xOk = xCol < Ktot;
    const int xTap = xOk ? (int)fast_div((unsigned)xCol, p.divIC) : 0;
    const int xIc = xCol - xTap * p.IC;
    const int xFh = (int)fast_div((unsigned)xTap, p.divFW), xFw = xTap - xFh * p.FW;

    int gVoff[T::PG];                       // bytes, fixed
#pragma unroll
    for (int i = 0; i < T::PG; ++i) {
        const int r = gRow + T::G_RPP * i;
        const int pixel = PM ? r * ohow : r;   // (oh,ow,n) order: row r of a stage is image nb + r
        gVoff[i] = gOc < p.OC ? (pixel * p.OC + gOc) * 4 : kOutOfRange;
    }
    // X: element offset of the thread's part of the address; validity inputs.
    // Rows past the last image need no test: their X addresses lie past the end of X (whole offset
    // in the VGPR), and G is read through a per-stage window that ends with the tensor.
    int xPart[T::PX];
    int xWBase[WIDE ? T::PX : 1];           // WIDE: input column of the thread's tap when the stage starts at ow0 = 0
    int xHBase[T::PX];                      // !PM: input row relative to the stage's first one; far out of range
                                            //      where the thread's column is never inside the image
    unsigned long long liveMask = 0ull;     // PM: positions at which this thread's tap is inside the image
    unsigned long long tileLive = ~0ull;    // PM: positions at which any tap of the tile is (uniform)
    if constexpr (PM) {
#pragma unroll
        for (int i = 0; i < T::PX; ++i) {
            const int r = xRow + T::X_RPP * i;
            xPart[i] = (r * p.IH * p.IW + xFh * p.IW + xFw) * p.IC + xIc;
            xHBase[i] = 0;
        }
        unsigned long long wMask = 0ull;
        for (int ow = 0; ow < p.OW; ++ow)
            if ((unsigned)(ow * p.sw - p.pw + xFw) < (unsigned)p.IW) wMask |= 1ull << ow;
        for (int oh = 0; oh < p.OH; ++oh)
            if (xOk && (unsigned)(oh * p.sh - p.ph + xFh) < (unsigned)p.IH) liveMask |= wMask << (oh * p.OW);
        // every wave holds all column segments of the tile in its first X_TPR lanes
        unsigned lo = 0u, hi = 0u;
#pragma unroll
        for (int l = 0; l < T::X_TPR; ++l) {
            lo |= (unsigned)__builtin_amdgcn_readlane((int)(unsigned)liveMask, l);
            hi |= (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(liveMask >> 32), l);
        }
        tileLive = ((unsigned long long)hi << 32) | lo;
        // Slices cut the tile's LIVE stages evenly, not its rows: a slice of the first output rows
        // would otherwise be nearly empty for a tap that reaches up, and the slices of one tile
        // would differ in length by several times.  Live stage q sits at the (q / cpp)-th live
        // position, chunk q % cpp of it (cpp = chunks per position).
        const int cpp = p.N / kBK;
        const int liveQ = __popcll(tileLive) * cpp;
        auto chunk_of = [&](int q) __attribute__((always_inline)) -> int {
            if (q >= liveQ) return chunksTotal;
            const int idx = q / cpp;
            unsigned long long m = tileLive;
            for (int k = 0; k < idx; ++k) m &= m - 1;     // drop the idx lowest live positions
            return __builtin_ctzll(m) * cpp + (q - idx * cpp);
        };
        ch0 = chunk_of((int)((long long)slice * liveQ / p.split));
        ch1 = chunk_of((int)((long long)(slice + 1) * liveQ / p.split));
    } else {
#pragma unroll
        for (int i = 0; i < T::PX; ++i) {
            const int r = xRow + T::X_RPP * i;
            int dn = 0, rr = r;
            if (ohow < kBK) {
                dn = (int)fast_div((unsigned)r, p.divOHOW);
                rr = r - dn * ohow;
            }
            const int doh = (int)fast_div((unsigned)rr, p.divOW), ow = rr - doh * p.OW;
            const int iw = ow * p.sw - p.pw + xFw;
            xHBase[i] = doh * p.sh - p.ph + xFh;
            xPart[i] = ((dn * p.IH + xHBase[i]) * p.IW + iw) * p.IC + xIc;   // may be negative
            if (WIDE) {
                xWBase[i] = iw;
                if (!xOk) xHBase[i] = kInvalidCoord;
            } else if (!(xOk && (unsigned)iw < (unsigned)p.IW)) {
                xHBase[i] = kInvalidCoord;
            }
        }
    }

    // First stage at or after ch that has work for this tile (uniform, branch-free).
    const int chunksPerPos = p.N / kBK;
    auto next_live = [&](int ch) __attribute__((always_inline)) -> int {
        if constexpr (!PM) {
            return ch < ch1 ? ch : ch1;
        } else {
            int pos = (int)fast_div((unsigned)(ch * kBK), p.divN);
            pos = pos < 63 ? pos : 63;
            const unsigned long long rem = tileLive >> pos;
            const int skip = rem ? __builtin_ctzll(rem) : 64;
            const int nch = skip == 0 ? ch : (pos + skip) * chunksPerPos;
            return nch < ch1 ? nch : ch1;
        }
    };

    // ---- stage cursor for the loads: uniform part of the addresses ------------------------------
    // Computed in four pieces, so that the steady-state loop can spread them over four MFMA steps
    // instead of leaving one long run of ALU work between two MFMAs.
    int gSoff = 0;                 // bytes
    int xVoff[T::PX];              // bytes, recomputed per stage
    int curA = 0, curB = 0, curUni = 0, curW = 0;   // uniform intermediates handed from piece to piece
    auto set_piece = [&](int piece, int ch) __attribute__((always_inline)) {
        if constexpr (PM) {
            if (piece == 0) {
                const int m0 = ch * kBK;
                curA = (int)fast_div((unsigned)m0, p.divN);          // output position
                curB = m0 - curA * p.N;                               // first image of the stage
            } else if (piece == 1) {
                const int oh = (int)fast_div((unsigned)curA, p.divOW), ow = curA - oh * p.OW;
                gSoff = (curB * ohow + curA) * p.OC * 4;
                curUni = ((curB * p.IH + oh * p.sh - p.ph) * p.IW + ow * p.sw - p.pw) * p.IC;
            } else {
                const bool live = ((liveMask >> curA) & 1ull) != 0;
#pragma unroll
                for (int i = 0; i < T::PX; ++i)
                    if ((i < T::PX / 2) == (piece == 2)) {
                        const int off = (xPart[i] + curUni) * 4;
                        xVoff[i] = live ? off : kOutOfRange;
                    }
            }
        } else {
            if (piece == 0) {
                const int m0 = ch * kBK;
                gSoff = m0 * p.OC * 4;
                curA = (int)fast_div((unsigned)m0, p.divOHOW);       // image
                curB = m0 - curA * ohow;                              // first output pixel inside it
            } else if (piece == 1) {
                const int oh0 = (int)fast_div((unsigned)curB, p.divOW);
                if (WIDE) curW = (curB - oh0 * p.OW) * p.sw;          // ow0 * sw: the stage's column shift
                curB = oh0 * p.sh;
                curUni = ((curA * p.IH + curB) * p.IW + (WIDE ? curW : 0)) * p.IC;
            } else {
#pragma unroll
                for (int i = 0; i < T::PX; ++i)
                    if ((i < T::PX / 2) == (piece == 2)) {
                        const int off = (xPart[i] + curUni) * 4;
                        bool ok = (unsigned)(curB + xHBase[i]) < (unsigned)p.IH;
                        if (WIDE) ok = ok && (unsigned)(curW + xWBase[i]) < (unsigned)p.IW;
                        xVoff[i] = ok ? off : kOutOfRange;
                    }
            }
        }
    };
    auto set_stage = [&](int ch) __attribute__((always_inline)) {
#pragma unroll
        for (int piece = 0; piece < 4; ++piece) set_piece(piece, ch);
    };

    f4 ggS[2][T::PG], gxS[2][T::PX];
    constexpr int kItems = T::PG + T::PX;
    auto gload_item = [&](int q, f4 *gg, f4 *gx) __attribute__((always_inline)) {
        // The stage's rows of G are addressed through a descriptor that starts at the stage's first
        // row and ends with the tensor: the range check of a raw buffer load covers the VGPR
        // offset only, never the scalar offset, so a window that moves with the stage is what
        // makes rows past the last one (a partial last stage) read zeros.  Scalar work only.
        // gSoff is uniform; saying so keeps it in SGPRs instead of a per-lane loop over its values.
        if (q < T::PG) {
            const unsigned soff = (unsigned)__builtin_amdgcn_readfirstlane(gSoff);
            const __amdgpu_buffer_rsrc_t rsrcG = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<char *>(reinterpret_cast<const char *>(p.G)) + soff, 0, (int)(p.gBytes - soff), 0x00020000);
            gg[q] = __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(rsrcG, gVoff[q], 0, 0));
        } else gx[q - T::PG] = __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(rsrcX, xVoff[q - T::PG], 0, 0));
    };
    auto lds_store_item = [&](int q, int buf, const f4 *gg, const f4 *gx) __attribute__((always_inline)) {
        if (q < T::PG)
            *reinterpret_cast<f4 *>(Gs + buf * T::G_STAGE + (gRow + T::G_RPP * q) * T::LDG + gSeg * 4) = gg[q];
        else
            *reinterpret_cast<f4 *>(Xs + buf * T::X_STAGE + (xRow + T::X_RPP * (q - T::PG)) * T::LDX + xSeg * 4) = gx[q - T::PG];
    };

    float16v acc[T::MB][T::NB], acc2[T::MB][T::NB];
#pragma unroll
    for (int i = 0; i < T::MB; ++i)
#pragma unroll
        for (int j = 0; j < T::NB; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                acc[i][j][r] = 0.f;
                acc2[i][j][r] = 0.f;
            }
    int sinceFlush = 0;
    auto maybe_flush = [&]() __attribute__((always_inline)) {
        if (++sinceFlush == p.flushChunks) {
            sinceFlush = 0;
#pragma unroll
            for (int i = 0; i < T::MB; ++i)
#pragma unroll
                for (int j = 0; j < T::NB; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        acc2[i][j][r] += acc[i][j][r];
                        acc[i][j][r] = 0.f;
                    }
        }
    };

    const int wm = wave / T::WAVES_N, wn = wave % T::WAVES_N;
    const int l32 = lane & 31, lh = lane >> 5;

    // Fragment ring: the LDS reads of MFMA step s+kAhead are issued before the MFMAs of step s, so a
    // wave alone on its SIMD still feeds the matrix pipe back to back.  The stage's barrier sits
    // kAhead steps before the stage's end: by then every wave has read all of this buffer into
    // registers and stored its share of the next one, and the last steps' MFMAs run while the
    // first fragments of the next buffer arrive.
    // volatile: the compiler would otherwise pair the reads into two-address LDS reads, each pair
    // needing a VALU add for its base - and VALU instructions cost matrix time, LDS reads do not
    constexpr int kSteps = kBK / 2, kRing = 4, kAhead = kRing - 1;
    static_assert(kSteps % kRing == 0, "ring slots must line up across stages");
    float fa[kRing][T::MB], fb[kRing][T::NB];
    const float *gFrag = Gs + (lh * 4) * T::LDG + wm * T::WTM + l32;
    const float *xFrag = Xs + (lh * 4) * T::LDX + wn * T::WTN + l32;
    auto read_step = [&](int buf, int s, float *a, float *b) __attribute__((always_inline)) {
        const int row = (s / 4) * 8 + s % 4;   // the lane's upper half adds 4: both operands use the same rows
        lds_cvptr g = (lds_cvptr)(gFrag + buf * T::G_STAGE + row * T::LDG);
        lds_cvptr x = (lds_cvptr)(xFrag + buf * T::X_STAGE + row * T::LDX);
#pragma unroll
        for (int i = 0; i < T::MB; ++i) a[i] = g[i * 32];
#pragma unroll
        for (int j = 0; j < T::NB; ++j) b[j] = x[j * 32];
    };

    // One stage: MFMAs from LDS buffer `buf`; between MFMA steps the wave issues its share of
    // the loads of the chunk two stages ahead (register set ld) and of the LDS stores of set st.
    // Ends with the fragments of the first kAhead steps of buffer buf^1 in flight.
    constexpr int kSlots = kSteps - kAhead;   // memory items go before the barrier
    static_assert(kItems <= kSlots, "one memory item per MFMA step");
    // With adv, the last four steps also move the load cursor to chunk advCh (the loads of this
    // stage have been issued by then).
    constexpr int kAdvStep = kSteps - 4;
    static_assert((kItems - 1) * kSlots / kItems < kAdvStep, "cursor pieces come after the last load");
    int advCh = 0;
    auto stage = [&](int buf, bool doLoad, int ld, bool doStore, int st, bool adv) __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < kSteps; ++s) {
            if (s == kSlots) __syncthreads();
            const int sp = s + kAhead;
            if (sp < kSteps) read_step(buf, sp, fa[sp % kRing], fb[sp % kRing]);
            else read_step(buf ^ 1, sp - kSteps, fa[sp % kRing], fb[sp % kRing]);
#pragma unroll
            for (int q = 0; q < kItems; ++q)
                if (q * kSlots / kItems == s) {
                    if (doLoad) gload_item(q, ggS[ld], gxS[ld]);
                    if (doStore) lds_store_item(q, buf ^ 1, ggS[st], gxS[st]);
                }
            if (adv && s >= kAdvStep) set_piece(s - kAdvStep, advCh);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < T::MB; ++i)
#pragma unroll
                for (int j = 0; j < T::NB; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[s % kRing][i], fb[s % kRing][j], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- main loop over the live stages of this slice --------------------------------------------
    // c0 is multiplied now, c1 sits in registers (other set), c2 is loaded during this stage.
    int c0 = next_live(ch0);
    if (c0 < ch1) {
        set_stage(c0);
#pragma unroll
        for (int q = 0; q < kItems; ++q) gload_item(q, ggS[0], gxS[0]);
        int c1 = next_live(c0 + 1);
        if (c1 < ch1) {
            set_stage(c1);
#pragma unroll
            for (int q = 0; q < kItems; ++q) gload_item(q, ggS[1], gxS[1]);
        }
#pragma unroll
        for (int q = 0; q < kItems; ++q) lds_store_item(q, 0, ggS[0], gxS[0]);
        __syncthreads();
#pragma unroll
        for (int s = 0; s < kAhead; ++s) read_step(0, s, fa[s], fb[s]);
        // c0 is in LDS buffer 0, c1 in register set 1, c2 is the chunk the next stage loads (its
        // offsets are set), c3 the one after.
        int c2 = next_live(c1 + 1);
        if (c2 < ch1) set_stage(c2);
        int c3 = next_live(c2 + 1);
        for (;;) {
            // two stages per trip so that buffer and register-set indices are compile-time
            if (c3 < ch1) {   // steady state: no branch around memory instructions
                const int c4 = next_live(c3 + 1);
                advCh = c3;
                stage(0, true, 0, true, 1, true);    // loads c2, then moves the cursor to c3
                maybe_flush();
                advCh = c4;                          // past the end: offsets nobody loads from
                stage(1, true, 1, true, 0, true);    // loads c3
                maybe_flush();
                c1 = c3;
                c2 = c4;
                c3 = next_live(c4 + 1);
                continue;
            }
            // tail: c0 (in LDS 0), maybe c1 (registers 1), maybe c2
            if (c2 < ch1) set_stage(c2);
            stage(0, c2 < ch1, 0, c1 < ch1, 1, false);
            maybe_flush();
            if (c1 >= ch1) break;
            stage(1, false, 1, c2 < ch1, 0, false);
            maybe_flush();
            if (c2 >= ch1) break;
            stage(0, false, 0, false, 1, false);
            break;
        }
    }

    float *C = p.C + (long long)slice * p.sliceStride;
#pragma unroll
    for (int i = 0; i < T::MB; ++i)
#pragma unroll
        for (int j = 0; j < T::NB; ++j) {
            const int col = col0 + wn * T::WTN + j * 32 + l32;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int oc = oc0 + wm * T::WTM + i * 32 + 8 * (r / 4) + 4 * lh + (r % 4);
                if (oc < p.OC && col < Ktot) C[oc * Ktot + col] = acc2[i][j][r] + acc[i][j][r];
            }
        }
}

template <int BM, int BN, bool PM, bool WIDE = false>
static hipError_t launch_fast_one(const WgradParams &p, int grid, hipStream_t st)
{
    constexpr size_t kSmemBytes = WF<BM, BN>::SMEM_BYTES;
    hipLaunchKernelGGL((wgrad_fast_kernel<BM, BN, PM, WIDE>), dim3((unsigned)grid), dim3(kThreads), kSmemBytes, st, p);
    return hipGetLastError();
}

// Tiles that need more LDS than a kernel gets by default (64 KB): limit raised once per device,
// outside any stream capture (see prepare_device in the host API).
template <int BM, int BN>
static hipError_t raise_lds_limit()
{
    constexpr size_t bytes = WF<BM, BN>::SMEM_BYTES;
    if (bytes <= 64 * 1024) return hipSuccess;
    const void *kerns[3] = {reinterpret_cast<const void *>(wgrad_fast_kernel<BM, BN, false, false>),
                            reinterpret_cast<const void *>(wgrad_fast_kernel<BM, BN, true, false>),
                            reinterpret_cast<const void *>(wgrad_fast_kernel<BM, BN, false, true>)};
    for (const void *k : kerns) {
        const hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t prepare_wgrad_fast()
{
    hipError_t e = raise_lds_limit<128, 128>();
    if (e == hipSuccess) e = raise_lds_limit<64, 128>();
    if (e == hipSuccess) e = raise_lds_limit<128, 64>();
    if (e == hipSuccess) e = raise_lds_limit<64, 64>();
    if (e == hipSuccess) e = raise_lds_limit<32, 128>();
    return e;
}

hipError_t launch_wgrad_fast(const WgradParams &p, int bm, int bn, int grid, hipStream_t st)
{
    if (!wgrad_fast_accepts(p.N, p.OH, p.OW, p.IC, p.OC, p.posMajor, bm, bn)) return hipErrorInvalidValue;
    const bool wide = p.OW > kBK;   // then a multiple of 32, (n,oh,ow) order only
#define MI355CONV_WF(BM_, BN_)                                                        \
    if (bm == BM_ && bn == BN_) {                                                     \
        if (wide) return launch_fast_one<BM_, BN_, false, true>(p, grid, st);         \
        return p.posMajor ? launch_fast_one<BM_, BN_, true>(p, grid, st)              \
                          : launch_fast_one<BM_, BN_, false>(p, grid, st);            \
    }
    MI355CONV_WF(128, 128)
    MI355CONV_WF(64, 128)
    MI355CONV_WF(64, 64)
    MI355CONV_WF(128, 64)
    MI355CONV_WF(32, 128)
#undef MI355CONV_WF
    return hipErrorInvalidValue;
}

}  // namespace mi355conv
