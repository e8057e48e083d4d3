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
//  * With (oh,ow,n) row order a stage sits on one output position; each thread keeps a 64-bit
//    mask of the positions where its filter tap is inside the image, and whole stages that
//    are padding for every tap of the tile are skipped (small-feature-map operator, Sec. IV).
//  * Loads run two stages ahead through two register sets; memory instructions are spread
//    between MFMA groups; one barrier per stage.
// Accuracy: the accumulator is folded into a second one every `flushChunks` stages (512
// products), so no fp32 chain is longer than that however long the slice is.
#include <hip/hip_runtime.h>
#if defined(EXP_STAMPS)
namespace mi355conv { __device__ unsigned long long g_wstamps[16384 * 8]; }
#define STAMP(i) do { if (threadIdx.x == 0 && blockIdx.x < 16384) mi355conv::g_wstamps[blockIdx.x * 8 + (i)] = wall_clock64(); } while (0)
#endif
#include "gather_common.h"

namespace mi355conv {

namespace {
template <int BM, int BN>
struct WF {
    static constexpr int WTM = BM / 2, WTN = BN / 2;
    static constexpr int MB = WTM / 32, NB = WTN / 32;
    static constexpr int LDG = BM + 8, LDX = BN + 8;
    static constexpr int G_TPR = BM / 4, G_RPP = kThreads / G_TPR, PG = kBK / G_RPP;
    static constexpr int X_TPR = BN / 4, X_RPP = kThreads / X_TPR, PX = kBK / X_RPP;
    static constexpr int G_STAGE = kBK * LDG, X_STAGE = kBK * LDX;
    static constexpr size_t SMEM_BYTES = 2 * (G_STAGE + X_STAGE) * sizeof(float);
};
}  // namespace

template <int BM, int BN>
__global__ __launch_bounds__(kThreads, (BM * BN >= 128 * 128) ? 1 : (BM * BN <= 64 * 64) ? 4 : 2) void wgrad_fast_kernel(const WgradParams p)
{
    using T = WF<BM, BN>;
    extern __shared__ f4 smem_raw[];
    float *Gs = reinterpret_cast<float *>(smem_raw);
    float *Xs = Gs + 2 * T::G_STAGE;

    STAMP(0);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int bid = xcd_remap(blockIdx.x, gridDim.x, p.xcdUnit);
    const int rest = (int)fast_div((unsigned)bid, p.divTilesN);
    const int tn = bid - rest * p.tilesN;
    const int tmo = (int)fast_div((unsigned)rest, p.divSplit);
    const int slice = rest - tmo * p.split;
    const int oc0 = tmo * BM, col0 = tn * BN;
    const int Ktot = p.FH * p.FW * p.IC;
    const int ohow = p.OH * p.OW;

    const int chunksTotal = (p.M + kBK - 1) / kBK;
    const int ch0 = slice * chunksTotal / p.split;
    const int ch1 = (slice + 1) * chunksTotal / p.split;

    constexpr int kOutOfRange = (int)0x80000000;
    const __amdgpu_buffer_rsrc_t rsrcG =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(p.G), 0, (int)p.gBytes, 0x00020000);
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
        const int pixel = p.posMajor ? r * ohow : r;   // (y,x,n) order: row r of a stage is image nb + r
        gVoff[i] = gOc < p.OC ? (pixel * p.OC + gOc) * 4 : kOutOfRange;
    }
    // X: element offset of the thread's part, row-validity inputs
    int xPart[T::PX], xHBase[T::PX], xDn[T::PX];   // xHBase = far out of range where the column is never valid
    // (y,x,n) order: output rows / columns at which this thread's tap is inside the image
    unsigned long long hMask = 0ull, wMask = 0ull;
    if (p.posMajor) {
#pragma unroll
        for (int i = 0; i < T::PX; ++i) {
            const int r = xRow + T::X_RPP * i;
            xPart[i] = (r * p.IH * p.IW + xFh * p.IW + xFw) * p.IC + xIc;
            xHBase[i] = 0;
            xDn[i] = 0;
        }
        for (int oh = 0; oh < p.OH; ++oh)
            if ((unsigned)(oh * p.sh - p.ph + xFh) < (unsigned)p.IH) hMask |= 1ull << oh;
        for (int ow = 0; ow < p.OW; ++ow)
            if ((unsigned)(ow * p.sw - p.pw + xFw) < (unsigned)p.IW) wMask |= 1ull << ow;
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
            xDn[i] = dn;
            xPart[i] = ((dn * p.IH + xHBase[i]) * p.IW + iw) * p.IC + xIc;   // may be negative
            if (!(xOk && (unsigned)iw < (unsigned)p.IW)) xHBase[i] = kInvalidCoord;
        }
    }

    // taps covered by this tile (for the stage-skip test)
    const int tapLo = (int)fast_div((unsigned)col0, p.divIC);
    const int lastCol = (col0 + BN - 1 < Ktot - 1) ? col0 + BN - 1 : Ktot - 1;
    const int tapHi = (int)fast_div((unsigned)lastCol, p.divIC);
    auto stage_live = [&](int ch) __attribute__((always_inline)) -> bool {
        if (!p.posMajor) return true;
        const int pos = (int)fast_div((unsigned)(ch * kBK), p.divN);
        const int oh = (int)fast_div((unsigned)pos, p.divOW), ow = pos - oh * p.OW;
        for (int t = tapLo; t <= tapHi; ++t) {
            const int fh = (int)fast_div((unsigned)t, p.divFW), fw = t - fh * p.FW;
            if ((unsigned)(oh * p.sh - p.ph + fh) < (unsigned)p.IH && (unsigned)(ow * p.sw - p.pw + fw) < (unsigned)p.IW)
                return true;
        }
        return false;
    };
    auto next_live = [&](int ch) __attribute__((always_inline)) -> int {
        while (ch < ch1 && !stage_live(ch)) ++ch;
        return ch;
    };

    // ---- stage cursor for the loads: uniform part of the addresses ------------------------------
    int gSoff = 0;                 // bytes
    int xVoff[T::PX];              // bytes, recomputed per stage (4 VALU each)
    auto set_stage = [&](int ch) __attribute__((always_inline)) {
        const int m0 = ch * kBK;
        if (p.posMajor) {
            const int pos = (int)fast_div((unsigned)m0, p.divN);
            const int nb = m0 - pos * p.N;
            const int oh = (int)fast_div((unsigned)pos, p.divOW), ow = pos - oh * p.OW;
            gSoff = (nb * ohow + pos) * p.OC * 4;
            const int uni = ((nb * p.IH + oh * p.sh - p.ph) * p.IW + ow * p.sw - p.pw) * p.IC;
            const bool live = ((hMask >> oh) & (wMask >> ow) & 1ull) != 0;
#pragma unroll
            for (int i = 0; i < T::PX; ++i) xVoff[i] = (live && xOk) ? (xPart[i] + uni) * 4 : kOutOfRange;
        } else {
            gSoff = m0 * p.OC * 4;
            const int n0 = (int)fast_div((unsigned)m0, p.divOHOW);
            const int r0 = m0 - n0 * ohow;
            const int oh0 = (int)fast_div((unsigned)r0, p.divOW);
            const int ohs = oh0 * p.sh;
            const int uni = (n0 * p.IH + ohs) * p.IW * p.IC;
#pragma unroll
            for (int i = 0; i < T::PX; ++i) {
                const bool ok = (unsigned)(ohs + xHBase[i]) < (unsigned)p.IH && n0 + xDn[i] < p.N;
                xVoff[i] = ok ? (xPart[i] + uni) * 4 : kOutOfRange;
            }
        }
    };

    f4 ggS[2][T::PG], gxS[2][T::PX];
    constexpr int kItems = T::PG + T::PX;
    constexpr int kGroups = kBK / 8;
    auto gload_item = [&](int q, f4 *gg, f4 *gx) __attribute__((always_inline)) {
        // gSoff is uniform; saying so keeps it in an SGPR instead of a per-lane loop over its values
        if (q < T::PG)
            gg[q] = __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(rsrcG, gVoff[q],
                                                                                __builtin_amdgcn_readfirstlane(gSoff), 0));
        else gx[q - T::PG] = __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(rsrcX, xVoff[q - T::PG], 0, 0));
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

    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, lh = lane >> 5;

    // volatile: the compiler would otherwise pair these into two-address LDS reads, each pair
    // needing a VALU add for its base - and VALU instructions cost matrix time, LDS reads do not
    auto load_frag = [&](const float *g, const float *x, int jj, f4 *fa, f4 *fb) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < T::MB; ++i) {
            lds_cvptr q = (lds_cvptr)(g + (jj * 8) * T::LDG + i * 32);
            fa[i] = f4{q[0], q[T::LDG], q[2 * T::LDG], q[3 * T::LDG]};
        }
#pragma unroll
        for (int j = 0; j < T::NB; ++j) {
            lds_cvptr q = (lds_cvptr)(x + (jj * 8) * T::LDX + j * 32);
            fb[j] = f4{q[0], q[T::LDX], q[2 * T::LDX], q[3 * T::LDX]};
        }
    };

    // One stage: MFMAs from LDS buffer `buf`; between MFMA groups the wave issues its share of
    // the loads of chunk `chLoad` (register set ld) and of the LDS stores of set st.
    auto stage = [&](int buf, bool doLoad, int ld, bool doStore, int st) __attribute__((always_inline)) {
        const float *g = Gs + buf * T::G_STAGE + (lh * 4) * T::LDG + wm * T::WTM + l32;
        const float *x = Xs + buf * T::X_STAGE + (lh * 4) * T::LDX + wn * T::WTN + l32;
        constexpr bool kTwoFrags = BM * BN < 128 * 128 && BM * BN > 64 * 64;   // register budget of the smallest and largest tile
        f4 fa[kTwoFrags ? 2 : 1][T::MB], fb[kTwoFrags ? 2 : 1][T::NB];
        if (kTwoFrags) load_frag(g, x, 0, fa[0], fb[0]);
#pragma unroll
        for (int jj = 0; jj < kGroups; ++jj) {
            const int cur = kTwoFrags ? (jj & 1) : 0;
            if (kTwoFrags) {
                if (jj + 1 < kGroups) load_frag(g, x, jj + 1, fa[cur ^ 1], fb[cur ^ 1]);
            } else {
                load_frag(g, x, jj, fa[0], fb[0]);
            }
#pragma unroll
            for (int q = 0; q < kItems; ++q)
                if (q % kGroups == jj) {
                    if (doLoad) gload_item(q, ggS[ld], gxS[ld]);
                    if (doStore) lds_store_item(q, buf ^ 1, ggS[st], gxS[st]);
                }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int i = 0; i < T::MB; ++i)
#pragma unroll
                    for (int j = 0; j < T::NB; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[cur][i][t], fb[cur][j][t], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- main loop over the live stages of this slice --------------------------------------------
    // c0 is multiplied now, c1 sits in registers (other set), c2 is loaded during this stage.
    STAMP(1);
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
        STAMP(2);
        for (;;) {
            // two stages per trip so that buffer and register-set indices are compile-time
            int c2 = c1 < ch1 ? next_live(c1 + 1) : ch1;
            int c3 = c2 < ch1 ? next_live(c2 + 1) : ch1;
            if (c3 < ch1) {   // steady state: no branch around memory instructions
                set_stage(c2);
                stage(0, true, 0, true, 1);
                maybe_flush();
                __syncthreads();
                set_stage(c3);
                stage(1, true, 1, true, 0);
                maybe_flush();
                __syncthreads();
                c0 = c2;
                c1 = c3;
                continue;
            }
            // tail: c0 (in LDS 0), maybe c1 (registers 1), maybe c2
            if (c2 < ch1) set_stage(c2);
            stage(0, c2 < ch1, 0, c1 < ch1, 1);
            maybe_flush();
            __syncthreads();
            if (c1 >= ch1) break;
            stage(1, false, 1, c2 < ch1, 0);
            maybe_flush();
            __syncthreads();
            if (c2 >= ch1) break;
            stage(0, false, 0, false, 1);
            break;
        }
    }

    STAMP(3);
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
    STAMP(4);
}

#if defined(EXP_STAMPS)
extern "C" int exp_read_wstamps(unsigned long long *host, size_t count)
{
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_wstamps), count * sizeof(unsigned long long));
}
#endif

template <int BM, int BN>
static hipError_t launch_fast_one(const WgradParams &p, int grid, hipStream_t st)
{
    using T = WF<BM, BN>;
    auto kern = wgrad_fast_kernel<BM, BN>;
    static bool attrSet[16] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 16 || !attrSet[dev]) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)T::SMEM_BYTES);
        if (e != hipSuccess) return e;
        if (dev >= 0 && dev < 16) attrSet[dev] = true;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kThreads), T::SMEM_BYTES, st, p);
    return hipGetLastError();
}

hipError_t launch_wgrad_fast(const WgradParams &p, int bm, int bn, int grid, hipStream_t st)
{
    if (bm == 128 && bn == 128) return launch_fast_one<128, 128>(p, grid, st);
    if (bm == 64 && bn == 128) return launch_fast_one<64, 128>(p, grid, st);
    if (bm == 64 && bn == 64) return launch_fast_one<64, 64>(p, grid, st);
    if (bm == 128 && bn == 64) return launch_fast_one<128, 64>(p, grid, st);
    return hipErrorInvalidValue;
}

}  // namespace mi355conv
