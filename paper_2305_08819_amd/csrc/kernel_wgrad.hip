// Backward-weight on v_mfma_f32_32x32x2_f32 for gfx950.
//
// GEMM view: dW[oc, col] = sum_m G[m, oc] * Xg[m, col], m = (n, oh, ow) over N*OH*OW rows,
// col = (fh*FW + fw)*IC + ic, Xg the input pixel that tap (fh,fw) reads for output pixel m
// (zero outside the image).  The output is small and the reduction is long, so the row
// range is always cut into slices (grid = tiles x slices); slice partials go to the
// workspace and a separate kernel adds them in a fixed order.
//
// Both operands arrive with the reduction index m as the SLOW memory index (NHWC rows are
// channel-contiguous), so both LDS tiles are [k = m][channel] and MFMA operands are read
// with 4-byte LDS loads: lane l takes k = 8*jj + 4*(l/32) + t for t = 0..3 and channel l%32.
//
// Accuracy: an fp32 accumulator is folded into a second one every `flushChunks` stages, so
// no running sum is longer than flushChunks*kBK products however long the slice is.
//
// Small maps (paper Sec. IV): with rows ordered (oh, ow, n) a stage of kBK rows sits on one
// output position; stages whose position lies in the padding for every tap of the tile are
// skipped outright.
#include "conv_internal.h"

namespace mi355conv {

typedef float float16v __attribute__((ext_vector_type(16)));
typedef float f4 __attribute__((ext_vector_type(4)));   // native vector: stays in registers

namespace {
template <int BM, int BN>
struct WG {
    static constexpr int WTM = BM / 2, WTN = BN / 2;
    static constexpr int MB = WTM / 32, NB = WTN / 32;
    static constexpr int LDG = BM + 8, LDX = BN + 8;
    static constexpr int G_TPR = BM / 4, G_RPP = kThreads / G_TPR, PG = kBK / G_RPP;
    static constexpr int X_TPR = BN / 4, X_RPP = kThreads / X_TPR, PX = kBK / X_RPP;
    static constexpr int G_STAGE = kBK * LDG, X_STAGE = kBK * LDX;
    static constexpr size_t SMEM_BYTES = 2 * (G_STAGE + X_STAGE) * sizeof(float);
};
}  // namespace

// XELEM: the input-channel count is not a multiple of 4, so a 4-column segment of the X tile
// can straddle filter taps; its four elements are then fetched one by one, each with its own
// tap.  (Row order must be (n,oh,ow) in that mode.)
template <int BM, int BN, bool XELEM>
__global__ __launch_bounds__(kThreads, 2) void wgrad_kernel(const WgradParams p)
{
    using T = WG<BM, BN>;
    extern __shared__ f4 smem_raw[];
    float *Gs = reinterpret_cast<float *>(smem_raw);
    float *Xs = Gs + 2 * T::G_STAGE;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int bid = xcd_remap(blockIdx.x, gridDim.x, p.xcdUnit);
    const int tn = bid % p.tilesN;
    bid /= p.tilesN;
    const int slice = bid % p.split;
    const int tmo = bid / p.split;
    const int oc0 = tmo * BM, col0 = tn * BN;
    const int Ktot = p.FH * p.FW * p.IC;

    const int chunksTotal = (p.M + kBK - 1) / kBK;
    const int ch0 = (int)((long long)slice * chunksTotal / p.split);
    const int ch1 = (int)((long long)(slice + 1) * chunksTotal / p.split);

    // loader roles: fixed channel segment, rows vary per stage
    const int gSeg = tid % T::G_TPR, gRow = tid / T::G_TPR;
    const int xSeg = tid % T::X_TPR, xRow = tid / T::X_TPR;
    const int gOc = oc0 + gSeg * 4;
    const bool gOk = gOc < p.OC;
    const int xCol = col0 + xSeg * 4;
    const bool xOk = xCol < Ktot;
    const int xTap = xOk ? xCol / p.IC : 0;
    const int xIc = xCol - xTap * p.IC;
    const int xFh = xTap / p.FW, xFw = xTap - xFh * p.FW;
    int eFh[4], eFw[4], eIc[4];   // XELEM: tap and channel of each of the four columns
    bool eOk[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int col = xCol + e;
        eOk[e] = col < Ktot;
        const int tap = eOk[e] ? col / p.IC : 0;
        eIc[e] = col - tap * p.IC;
        eFh[e] = tap / p.FW;
        eFw[e] = tap - eFh[e] * p.FW;
    }
    const int ohow = p.OH * p.OW;

    // taps covered by this tile (for the stage-skip test)
    const int tapLo = col0 / p.IC;
    const int lastCol = (col0 + BN - 1 < Ktot - 1) ? col0 + BN - 1 : Ktot - 1;
    const int tapHi = lastCol / p.IC;

    auto stage_live = [&](int ch) __attribute__((always_inline)) -> bool {
        if (!p.posMajor) return true;
        const int pos = (ch * kBK) / p.N;   // all kBK rows of the stage share this position
        const int oh = pos / p.OW, ow = pos - oh * p.OW;
        for (int t = tapLo; t <= tapHi; ++t) {
            const int fh = t / p.FW, fw = t - fh * p.FW;
            if ((unsigned)(oh * p.sh - p.ph + fh) < (unsigned)p.IH &&
                (unsigned)(ow * p.sw - p.pw + fw) < (unsigned)p.IW)
                return true;
        }
        return false;
    };
    auto next_live = [&](int ch) __attribute__((always_inline)) -> int {
        while (ch < ch1 && !stage_live(ch)) ++ch;
        return ch;
    };

    f4 gg[T::PG], gx[T::PX];
    const f4 zero4 = {0.f, 0.f, 0.f, 0.f};

    // (n, oh, ow) of this thread's X rows.  With (n,oh,ow) row order consecutive stages are
    // kBK rows apart, so the triple advances by a fixed (dn, dh, dw) with at most one carry
    // per digit and no division in the loop.
    int rn[T::PX], rh[T::PX], rw[T::PX];
    const int stepN = kBK / ohow, stepRem = kBK - stepN * ohow;
    const int stepH = stepRem / p.OW, stepW = stepRem - stepH * p.OW;
    auto seek_rows = [&](int ch) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < T::PX; ++i) {
            const int m = ch * kBK + xRow + T::X_RPP * i;
            rn[i] = m / ohow;
            const int r = m - rn[i] * ohow;
            rh[i] = r / p.OW;
            rw[i] = r - rh[i] * p.OW;
        }
    };
    auto step_rows = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < T::PX; ++i) {
            rw[i] += stepW;
            rh[i] += stepH;
            rn[i] += stepN;
            if (rw[i] >= p.OW) { rw[i] -= p.OW; ++rh[i]; }
            if (rh[i] >= p.OH) { rh[i] -= p.OH; ++rn[i]; }
        }
    };

    auto gload = [&](int ch) __attribute__((always_inline)) {
        if (p.posMajor) {
            // a stage sits on one output position; rows differ only in n
            const int m0 = ch * kBK;
            const int pos = m0 / p.N, nb = m0 - pos * p.N;
            const int oh = pos / p.OW, ow = pos - oh * p.OW;
            const int ih = oh * p.sh - p.ph + xFh, iw = ow * p.sw - p.pw + xFw;
            const bool live = xOk && (unsigned)ih < (unsigned)p.IH && (unsigned)iw < (unsigned)p.IW;
#pragma unroll
            for (int i = 0; i < T::PG; ++i) {
                gg[i] = zero4;
                const int n = nb + gRow + T::G_RPP * i;
                if (gOk) gg[i] = *reinterpret_cast<const f4 *>(p.G + ((long long)n * ohow + pos) * p.OC + gOc);
            }
#pragma unroll
            for (int i = 0; i < T::PX; ++i) {
                gx[i] = zero4;
                const int n = nb + xRow + T::X_RPP * i;
                if (live)
                    gx[i] = *reinterpret_cast<const f4 *>(
                        p.X + ((long long)(n * p.IH + ih) * p.IW + iw) * p.IC + xIc);
            }
        } else {
#pragma unroll
            for (int i = 0; i < T::PG; ++i) {
                gg[i] = zero4;
                const int m = ch * kBK + gRow + T::G_RPP * i;
                if (gOk && m < p.M) gg[i] = *reinterpret_cast<const f4 *>(p.G + (long long)m * p.OC + gOc);
            }
#pragma unroll
            for (int i = 0; i < T::PX; ++i) {
                gx[i] = zero4;
                if (XELEM) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int ih = rh[i] * p.sh - p.ph + eFh[e], iw = rw[i] * p.sw - p.pw + eFw[e];
                        if (eOk[e] && rn[i] < p.N && (unsigned)ih < (unsigned)p.IH && (unsigned)iw < (unsigned)p.IW)
                            gx[i][e] = p.X[((long long)(rn[i] * p.IH + ih) * p.IW + iw) * p.IC + eIc[e]];
                    }
                } else {
                    const int ih = rh[i] * p.sh - p.ph + xFh, iw = rw[i] * p.sw - p.pw + xFw;
                    if (xOk && rn[i] < p.N && (unsigned)ih < (unsigned)p.IH && (unsigned)iw < (unsigned)p.IW)
                        gx[i] = *reinterpret_cast<const f4 *>(
                            p.X + ((long long)(rn[i] * p.IH + ih) * p.IW + iw) * p.IC + xIc);
                }
            }
            step_rows();
        }
    };
    auto lds_store = [&](int buf) __attribute__((always_inline)) {
        float *g = Gs + buf * T::G_STAGE, *x = Xs + buf * T::X_STAGE;
#pragma unroll
        for (int i = 0; i < T::PG; ++i)
            *reinterpret_cast<f4 *>(g + (gRow + T::G_RPP * i) * T::LDG + gSeg * 4) = gg[i];
#pragma unroll
        for (int i = 0; i < T::PX; ++i)
            *reinterpret_cast<f4 *>(x + (xRow + T::X_RPP * i) * T::LDX + xSeg * 4) = gx[i];
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

    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, lh = lane >> 5;

    auto load_frag = [&](const float *g, const float *x, int jj, f4 *fa, f4 *fb) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < T::MB; ++i) {
            const float *q = g + (jj * 8) * T::LDG + i * 32;
            fa[i] = f4{q[0], q[T::LDG], q[2 * T::LDG], q[3 * T::LDG]};
        }
#pragma unroll
        for (int j = 0; j < T::NB; ++j) {
            const float *q = x + (jj * 8) * T::LDX + j * 32;
            fb[j] = f4{q[0], q[T::LDX], q[2 * T::LDX], q[3 * T::LDX]};
        }
    };

    // fragments of group jj+1 are requested before the MFMAs of group jj are issued
    auto compute = [&](int buf) __attribute__((always_inline)) {
        const float *g = Gs + buf * T::G_STAGE + (lh * 4) * T::LDG + wm * T::WTM + l32;
        const float *x = Xs + buf * T::X_STAGE + (lh * 4) * T::LDX + wn * T::WTN + l32;
        f4 fa[2][T::MB], fb[2][T::NB];
        load_frag(g, x, 0, fa[0], fb[0]);
#pragma unroll
        for (int jj = 0; jj < kBK / 8; ++jj) {
            const int cur = jj & 1;
            if (jj + 1 < kBK / 8) load_frag(g, x, jj + 1, fa[cur ^ 1], fb[cur ^ 1]);
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
    auto flush = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < T::MB; ++i)
#pragma unroll
            for (int j = 0; j < T::NB; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    acc2[i][j][r] += acc[i][j][r];
                    acc[i][j][r] = 0.f;
                }
    };

    int cur = next_live(ch0);
    if (cur < ch1) {
        if (!p.posMajor) seek_rows(cur);
        gload(cur);
        lds_store(0);
        __syncthreads();
        int buf = 0, sinceFlush = 0;
        while (cur < ch1) {
            const int nxt = next_live(cur + 1);
            if (nxt < ch1) gload(nxt);
            compute(buf);
            if (++sinceFlush == p.flushChunks) {
                flush();
                sinceFlush = 0;
            }
            if (nxt < ch1) lds_store(buf ^ 1);
            __syncthreads();
            buf ^= 1;
            cur = nxt;
        }
    }
    flush();

    float *C = p.C + (long long)slice * p.sliceStride;
#pragma unroll
    for (int i = 0; i < T::MB; ++i)
#pragma unroll
        for (int j = 0; j < T::NB; ++j) {
            const int col = col0 + wn * T::WTN + j * 32 + l32;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int oc = oc0 + wm * T::WTM + i * 32 + 8 * (r / 4) + 4 * lh + (r % 4);
                if (oc < p.OC && col < Ktot) C[(long long)oc * Ktot + col] = acc2[i][j][r];
            }
        }
}

template <int BM, int BN, bool XELEM>
static hipError_t launch_one(const WgradParams &p, int grid, hipStream_t st)
{
    constexpr size_t kSmemBytes = WG<BM, BN>::SMEM_BYTES;
    hipLaunchKernelGGL((wgrad_kernel<BM, BN, XELEM>), dim3((unsigned)grid), dim3(kThreads), kSmemBytes, st, p);
    return hipGetLastError();
}

// Tiles that need more LDS than a kernel gets by default (64 KB): limit raised once per device,
// outside any stream capture (see prepare_device in the host API).
template <int BM, int BN, bool XELEM>
static hipError_t raise_lds_limit()
{
    constexpr size_t bytes = WG<BM, BN>::SMEM_BYTES;
    if (bytes <= 64 * 1024) return hipSuccess;
    return hipFuncSetAttribute(reinterpret_cast<const void *>(wgrad_kernel<BM, BN, XELEM>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

hipError_t prepare_wgrad()
{
    hipError_t e = raise_lds_limit<128, 128, false>();
    if (e == hipSuccess) e = raise_lds_limit<64, 128, false>();
    if (e == hipSuccess) e = raise_lds_limit<128, 64, false>();
    if (e == hipSuccess) e = raise_lds_limit<64, 64, false>();
    if (e == hipSuccess) e = raise_lds_limit<128, 64, true>();
    if (e == hipSuccess) e = raise_lds_limit<64, 64, true>();
    return e;
}

hipError_t launch_wgrad(const WgradParams &p, int bm, int bn, bool xElem, int grid, hipStream_t st)
{
    if (!wgrad_accepts(p.N, p.IC, p.OC, p.posMajor, xElem, bm, bn)) return hipErrorInvalidValue;
    if (xElem) {   // narrow-channel layers: small tiles only
        if (bm == 64 && bn == 64) return launch_one<64, 64, true>(p, grid, st);
        if (bm == 128 && bn == 64) return launch_one<128, 64, true>(p, grid, st);
        return hipErrorInvalidValue;
    }
    if (bm == 128 && bn == 128) return launch_one<128, 128, false>(p, grid, st);
    if (bm == 64 && bn == 128) return launch_one<64, 128, false>(p, grid, st);
    if (bm == 64 && bn == 64) return launch_one<64, 64, false>(p, grid, st);
    if (bm == 128 && bn == 64) return launch_one<128, 64, false>(p, grid, st);
    return hipErrorInvalidValue;
}

}  // namespace mi355conv
