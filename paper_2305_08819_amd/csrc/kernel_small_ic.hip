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
    static_assert(kTR == 4 && kTC == 32 && kPRows == 224, "bwd_data_small_ic_accepts() states these tile sizes");
    if (PR * PC > kPRows || !bwd_data_small_ic_accepts(p.IC, p.OC, p.FH, p.FW, 1, 1)) return hipErrorInvalidValue;
    const size_t smem = (size_t)(kPRows * LDA + 32 * LDA) * sizeof(float);
    static_assert(kPRows * kLDP <= kPRows * LDA, "P fits over the A tile");
    static_assert((size_t)(kPRows * LDA + 32 * LDA) * sizeof(float) <= 64 * 1024, "within the default dynamic LDS limit");
    const int grid = p.N * ((p.IH + kTR - 1) / kTR) * ((p.IW + kTC - 1) / kTC);
    hipLaunchKernelGGL(bwd_data_small_ic_kernel, dim3((unsigned)grid), dim3(kThreads), smem, st, p);
    return hipGetLastError();
}

// ---- forward for very few input channels -------------------------------------------------------
// Y[m, oc] = sum_k patch[m, k] * W[oc, k] with k = (fh,fw,ic) and at most 32 patch columns: the
// whole reduction is one MFMA stage.  A workgroup gathers the patch rows of 128 output pixels
// element by element (a thread owns one row; the tap of column k is uniform, so its address
// part is a scalar), 64 filter rows, multiplies once and stores.  Bound by writing Y.
// U8: X holds unsigned bytes (pixels); each is converted on load, x = (float)byte * p.scale.
template <bool U8>
__global__ __launch_bounds__(kThreads, 2) void fwd_small_ic_kernel(const SmallIcParams p)
{
    constexpr int BMf = 128, BNf = 64, LDf = 33;      // odd pitch: both the stores (lane = row) and the
                                                      // fragment reads (lane = row, 4 bytes) spread over banks
    __shared__ __attribute__((aligned(16))) float sm[BMf * LDf + BNf * LDf];
    float *As = sm, *Bs = sm + BMf * LDf;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, lh = lane >> 5;
    const int tilesN = (p.OC + BNf - 1) / BNf;
    const int tn = blockIdx.x % tilesN, tm = blockIdx.x / tilesN;
    const int m0 = tm * BMf, oc0 = tn * BNf;
    const int Kp = p.FH * p.FW * p.IC, ohow = p.OH * p.OW;

    constexpr int kOutOfRange = (int)0x80000000;
    const __amdgpu_buffer_rsrc_t rsrcX =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(p.X), 0, (int)p.xBytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrcW =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(p.W), 0, (int)p.wBytes, 0x00020000);

    // filter tile: Bs[oc][k], 64 x 32 elements, 8 per thread (k fastest: coalesced rows of W)
    float wv[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int idx = tid + kThreads * i;
        const int oc = idx >> 5, k = idx & 31;
        const int off = (k < Kp && oc0 + oc < p.OC) ? ((oc0 + oc) * Kp + k) * 4 : kOutOfRange;
        wv[i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrcW, off, 0, 0));
    }
    // patch tile: thread owns row (tid & 127) and the columns of one half (16 each)
    const int row = tid & (BMf - 1), khalf = tid >> 7;
    const int m = m0 + row;
    const int n = (int)fast_div((unsigned)m, p.divOHOW);
    const int r = m - n * ohow;
    const int oh = (int)fast_div((unsigned)r, p.divOW), ow = r - oh * p.OW;
    const int ihBase = oh * p.sh - p.ph, iwBase = ow * p.sw - p.pw;
    constexpr int kElem = U8 ? 1 : 4;                                       // bytes per element of X
    const int pixBase = ((n * p.IH + ihBase) * p.IW + iwBase) * p.IC * kElem;   // bytes; may be negative
    float xv[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int k = khalf * 16 + i;                                     // uniform per instruction
        const int tap = (int)fast_div((unsigned)k, p.divIC), ic = k - tap * p.IC;
        const int fh = (int)fast_div((unsigned)tap, p.divFW), fw = tap - fh * p.FW;
        const bool ok = k < Kp && m < p.M && (unsigned)(ihBase + fh) < (unsigned)p.IH &&
                        (unsigned)(iwBase + fw) < (unsigned)p.IW;
        const int off = ok ? pixBase + ((fh * p.IW + fw) * p.IC + ic) * kElem : kOutOfRange;
        if (U8) xv[i] = (float)__builtin_amdgcn_raw_buffer_load_b8(rsrcX, off, 0, 0) * p.scale;
        else xv[i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrcX, off, 0, 0));
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int idx = tid + kThreads * i;
        Bs[(idx >> 5) * LDf + (idx & 31)] = wv[i];
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) As[row * LDf + khalf * 16 + i] = xv[i];
    __syncthreads();

    // wave w: rows 32w .. 32w+31, all 64 columns
    float16v acc[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[j][q] = 0.f;
    const float *a = As + (wave * 32 + l32) * LDf + lh;
    const float *b = Bs + l32 * LDf + lh;
#pragma unroll
    for (int step = 0; step < 16; ++step) {
        const float fa = a[2 * step];
#pragma unroll
        for (int j = 0; j < 2; ++j)
            acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa, b[j * 32 * LDf + 2 * step], acc[j], 0, 0, 0);
    }
    // accumulator register q of lane l is row 8*(q/4)+4*(l/32)+q%4, column l%32
    if (p.epilogue) {   // uniform: bias add and leaky-ReLU in the accumulator registers
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int col = oc0 + j * 32 + l32;
            const float b = p.bias && col < p.OC ? p.bias[col] : 0.f;
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const float v = acc[j][q] + b;
                acc[j][q] = v > 0.f ? v : v * p.slope;
            }
        }
    }
    if ((p.OC & 3) == 0) {
        // the kernel is bound by writing Y: turn each 32x32 block through LDS (the tiles are done
        // with) so that a lane stores 16 bytes and a store instruction covers eight 128-byte runs
        static_assert(4 * 32 * kLDT <= BMf * LDf + BNf * LDf, "four turning buffers fit over the tiles");
        __syncthreads();                       // every wave has read its last fragments
        float *scratch = sm + wave * 32 * kLDT;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int colBase = oc0 + j * 32;
            if (colBase < p.OC) {              // uniform; OC % 4 == 0, so 16-byte groups are in or out as a whole
#pragma unroll
                for (int q = 0; q < 16; ++q) scratch[(8 * (q / 4) + 4 * lh + (q % 4)) * kLDT + l32] = acc[j][q];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int rowT = t * 8 + (lane >> 3), seg = lane & 7;
                    const f4 v = *reinterpret_cast<const f4 *>(scratch + rowT * kLDT + seg * 4);
                    const int mm = m0 + wave * 32 + rowT;
                    if (mm < p.M && colBase + seg * 4 < p.OC)
                        *reinterpret_cast<f4 *>(p.dX + (long long)mm * p.OC + colBase + seg * 4) = v;
                }
            }
        }
        return;
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int col = oc0 + j * 32 + l32;
        if (col < p.OC) {
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const int mm = m0 + wave * 32 + 8 * (q / 4) + 4 * lh + (q % 4);
                if (mm < p.M) p.dX[(long long)mm * p.OC + col] = acc[j][q];
            }
        }
    }
}

hipError_t launch_fwd_small_ic(const SmallIcParams &p, hipStream_t st)
{
    if (!patch_small_ic_accepts(p.IC, p.FH, p.FW)) return hipErrorInvalidValue;
    const int grid = ((p.M + 127) / 128) * ((p.OC + 63) / 64);
    if (p.u8) hipLaunchKernelGGL(fwd_small_ic_kernel<true>, dim3((unsigned)grid), dim3(kThreads), 0, st, p);
    else hipLaunchKernelGGL(fwd_small_ic_kernel<false>, dim3((unsigned)grid), dim3(kThreads), 0, st, p);
    return hipGetLastError();
}

// ---- backward-weight for very few input channels ----------------------------------------------
// dW[oc, (fh,fw,ic)] = sum_m dY[m, oc] * patch[m, (fh,fw,ic)] with at most 32 columns: one 64 x 32
// output tile per 64 output channels, the rows m = (n, oh, ow) cut into `split` slices.  The
// kernel is bound by reading dY once, so it moves in macro-stages of 4 x 32 rows: all loads of a
// macro-stage are in flight together (dY with 16-byte loads, the patch matrix element by element
// - each thread owns one column, so its filter tap is fixed), and the next macro-stage is
// requested before the current one is multiplied.  The four waves are 2 (oc halves) x 2 (halves
// of a 32-row stage's 16 MFMA steps); the two step halves are added through LDS at the end.
namespace {
constexpr int kSub = 4;                                   // 32-row stages per macro-stage
constexpr int kWsLDG = 64 + 8, kWsLDX = 32 + 8;
constexpr int kWsGStage = kBK * kWsLDG, kWsXStage = kBK * kWsLDX;
}  // namespace

__global__ __launch_bounds__(kThreads, 2) void wgrad_small_ic_kernel(const SmallIcParams p)
{
    constexpr int LDG = kWsLDG, LDX = kWsLDX, G_STAGE = kWsGStage, X_STAGE = kWsXStage;
    extern __shared__ f4 smem_raw[];
    float *Gs = reinterpret_cast<float *>(smem_raw);       // [kSub][32 rows][LDG]
    float *Xs = Gs + kSub * G_STAGE;                       // [kSub][32 rows][LDX]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, lh = lane >> 5;
    const int slice = blockIdx.x % p.split, tmo = blockIdx.x / p.split;
    const int oc0 = tmo * 64;
    const int Kp = p.FH * p.FW * p.IC, ohow = p.OH * p.OW;
    const int chunksTotal = (p.M + kBK - 1) / kBK;
    const int ch0 = (int)((long long)slice * chunksTotal / p.split), ch1 = (int)((long long)(slice + 1) * chunksTotal / p.split);

    constexpr int kOutOfRange = (int)0x80000000;
    const __amdgpu_buffer_rsrc_t rsrcX =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(p.X), 0, (int)p.xBytes, 0x00020000);

    // dY loader: 32 rows x 16 segments per stage, 2 per thread; rows past M read zeros (see gload)
    const int gSeg = tid & 15, gRow = tid >> 4;
    int gOff[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
        gOff[i] = oc0 + gSeg * 4 < p.OC ? ((gRow + 16 * i) * p.OC + oc0 + gSeg * 4) * 4 : kOutOfRange;
    // patch loader: thread owns column xCol (its tap is fixed) and rows xRow + 8*i of every stage
    const int xCol = tid & 31, xRow = tid >> 5;
    const bool colOk = xCol < Kp;
    const int tap = colOk ? (int)fast_div((unsigned)xCol, p.divIC) : 0;
    const int ic = xCol - tap * p.IC;
    const int fh = (int)fast_div((unsigned)tap, p.divFW), fw = tap - fh * p.FW;

    f4 gg[kSub][2];
    float gx[kSub][4];
    auto gload = [&](int chBase) __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < kSub; ++s) {
            const int ch = chBase + s;
            const bool live = ch < ch1;      // uniform; stages past the slice load zeros
            const int m0 = ch * kBK;
            // dY through a window that starts at the stage's first row and ends with the tensor (empty
            // for stages past the slice): the range check of a raw buffer load covers the VGPR offset
            // only, so this is what makes the rows past M of a partial last stage read zeros
            const unsigned gStart = live ? (unsigned)m0 * (unsigned)p.OC * 4u : p.gBytes;
            const __amdgpu_buffer_rsrc_t rsrcG = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<char *>(reinterpret_cast<const char *>(p.G)) + gStart, 0, (int)(p.gBytes - gStart), 0x00020000);
#pragma unroll
            for (int i = 0; i < 2; ++i)
                gg[s][i] = __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(rsrcG, gOff[i], 0, 0));
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int m = m0 + xRow + 8 * i;
                const int n = (int)fast_div((unsigned)m, p.divOHOW);
                const int r = m - n * ohow;
                const int oh = (int)fast_div((unsigned)r, p.divOW), ow = r - oh * p.OW;
                const int ih = oh * p.sh - p.ph + fh, iw = ow * p.sw - p.pw + fw;
                const bool ok = live && colOk && m < p.M && (unsigned)ih < (unsigned)p.IH && (unsigned)iw < (unsigned)p.IW;
                const int off = ok ? (((n * p.IH + ih) * p.IW + iw) * p.IC + ic) * 4 : kOutOfRange;
                gx[s][i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrcX, off, 0, 0));
            }
        }
    };
    auto lds_store = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < kSub; ++s) {
#pragma unroll
            for (int i = 0; i < 2; ++i)
                *reinterpret_cast<f4 *>(Gs + s * G_STAGE + (gRow + 16 * i) * LDG + gSeg * 4) = gg[s][i];
#pragma unroll
            for (int i = 0; i < 4; ++i) Xs[s * X_STAGE + (xRow + 8 * i) * LDX + xCol] = gx[s][i];
        }
    };

    float16v acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    const int wo = wave >> 1, wk = wave & 1;   // oc half, half of a stage's MFMA steps

    if (ch0 < ch1) {
        gload(ch0);
        for (int ch = ch0; ch < ch1; ch += kSub) {
            lds_store();
            __syncthreads();
            if (ch + kSub < ch1) gload(ch + kSub);
            // lane (l32, lh) supplies row k = 2*step + lh of a stage: G^T as A, patch as B
#pragma unroll
            for (int s = 0; s < kSub; ++s) {
                const float *g = Gs + s * G_STAGE + lh * LDG + wo * 32 + l32;
                const float *x = Xs + s * X_STAGE + lh * LDX + l32;
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    const int step = wk * 8 + t;
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(g[2 * step * LDG], x[2 * step * LDX], acc, 0, 0, 0);
                }
            }
            __syncthreads();   // all waves are done with this macro-stage's tiles
        }
    }

    // add the two step halves: waves with wk = 1 hand their block to the wave with the same oc half
    float *red = Gs;   // 64 x 33 floats, the stage buffers are free now
    if (wk == 1) {
#pragma unroll
        for (int r = 0; r < 16; ++r) red[(wo * 32 + 8 * (r / 4) + 4 * lh + (r % 4)) * 33 + l32] = acc[r];
    }
    __syncthreads();
    if (wk == 0) {
        float *C = p.C + (long long)slice * p.sliceStride;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = 8 * (r / 4) + 4 * lh + (r % 4);
            const int oc = oc0 + wo * 32 + row;
            if (oc < p.OC && l32 < Kp) C[oc * Kp + l32] = acc[r] + red[(wo * 32 + row) * 33 + l32];
        }
    }
}

hipError_t launch_wgrad_small_ic(const SmallIcParams &p, hipStream_t st)
{
    if (!patch_small_ic_accepts(p.IC, p.FH, p.FW) || p.split < 1) return hipErrorInvalidValue;
    constexpr size_t smem = (size_t)kSub * (kWsGStage + kWsXStage) * sizeof(float);
    static_assert(64 * 33 <= kSub * kWsGStage, "the reduction buffer fits over the dY stages");
    static_assert(smem <= 64 * 1024, "within the default dynamic LDS limit");
    const int grid = ((p.OC + 63) / 64) * p.split;
    hipLaunchKernelGGL(wgrad_small_ic_kernel, dim3((unsigned)grid), dim3(kThreads), smem, st, p);
    return hipGetLastError();
}

}  // namespace mi355conv
