// Implicit-GEMM ("gather-GEMM") kernel for forward convolution and backward-data on
// v_mfma_f32_32x32x2_f32, written for gfx950 (wave64, 4 waves per workgroup).
//
// GEMM view (never materialised): rows = pixels of the tensor being produced, columns =
// its channels, reduction = (filter tap, source channel).  A workgroup owns a BM x BN
// output tile and walks the reduction in stages of kBK source channels of one tap:
//   global (NHWC, 16-byte loads along the channel axis) -> registers -> LDS -> MFMA.
// Global loads run two stages ahead through two register sets and land in the other LDS
// buffer one stage later; one barrier per stage.
//
// Two things make it a small-feature-map operator (paper Sec. IV: special conv\deconv
// operators that cut the work more the smaller the map is):
//  * every tile first ORs, over its rows, the set of filter taps that fall inside the
//    source image, and only walks that set.  With rows ordered (y, x, n) a tile sits on one
//    pixel position, so at 2x2/4x4/8x8 maps with a padded 3x3 filter only 44/69/84 % of the
//    taps are ever multiplied;
//  * backward-data is split into sh*sw stride phases; a tile belongs to one phase and its
//    tap set holds only the taps congruent to that phase, so no inserted zero is multiplied
//    and pixels no tap reaches are written as 0 by tiles with an empty tap set.
//
// MFMA operand layout used below (AMD CDNA3/4 ISA, v_mfma_f32_32x32x2_f32): lane l holds
// A[i = l%32][k = l/32] and B[k = l/32][j = l%32]; accumulator register r of lane l is
// D[i = 8*(r/4) + 4*(l/32) + r%4][j = l%32].  The order in which reduction elements are fed
// is free as long as A and B agree, so a lane reads FOUR consecutive k (one 16-byte LDS
// read at k = 8*jj + 4*(l/32)) and uses them in four successive MFMAs.
#include <hip/hip_runtime.h>
#include "gather_common.h"

namespace mi355conv {

// BELEM (backward-data only): the destination channel count is not a multiple of 4, so a
// 16-byte load of four filter columns would be misaligned; the B tile is fetched with four
// 4-byte loads per thread instead (e.g. the first layer's dX with 3 channels).
// RAGGED: the source channel count is a multiple of 4 but not of 32, so the last 32-channel
// stage of every tap is partly empty; its surplus 16-byte loads get an out-of-range offset
// (one select per load and stage, which the aligned instantiation does not pay).
template <int BM, int BN, int WAVES_M, bool BWD, bool BELEM = false, bool RAGGED = false>
__global__ __launch_bounds__(kThreads, 2) void gather_gemm_kernel(const GatherGemmParams params)
{
    BalancePrefetch pre = balance_prefetch(params.runs, params.posOrder);   // in flight with the scalar arguments
    balance_prefetch_classes(pre, params.classes);
    const GatherView p = gather_view(params);
    using T = GG<BM, BN, WAVES_M, BWD>;
    extern __shared__ f4 smem_raw[];
    float *smem = reinterpret_cast<float *>(smem_raw);
    float *As = smem;
    float *Bs = As + 2 * T::A_STAGE;
    int *rowBase = reinterpret_cast<int *>(Bs + 2 * T::B_STAGE);
    int *rowY = rowBase + BM;
    int *rowX = rowY + BM;
    int *outRow = rowX + BM;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;

    const GatherTile tile = gather_tile_setup<BM, BN, BWD>(p, pre, rowBase, rowY, rowX, outRow);
    const int slice = tile.slice, n0 = tile.n0;

    // taps walked by this tile: the rectangle [uLo,uHi] x [vLo,vHi]
    const int uCnt = tile.uHi >= tile.uLo ? tile.uHi - tile.uLo + 1 : 0;
    const int vCnt = tile.vHi >= tile.vLo ? tile.vHi - tile.vLo + 1 : 0;
    const int chunksPerTap = RAGGED ? (p.SC + kBK - 1) / kBK : p.SC / kBK;
    const int lastValid = p.SC - (chunksPerTap - 1) * kBK;   // source channels in a tap's last stage
    // This slice's part of the reduction: either the chunks [cLo, cHi) of every tap (slices differ in
    // source channels), or the stages [it0, it1) of the tap-major list of all stages.
    int cLo = 0, cHi = chunksPerTap, it0 = 0, it1;
    if (p.chunksPerSlice) {
        cLo = slice * p.chunksPerSlice;
        cHi = cLo + p.chunksPerSlice;
        it1 = uCnt * vCnt * p.chunksPerSlice;
    } else {
        const int nIter = uCnt * vCnt * chunksPerTap;
        it0 = (int)fast_div((unsigned)(slice * nIter), p.divSplit);          // nIter * split is far below 2^31
        it1 = (int)fast_div((unsigned)((slice + 1) * nIter), p.divSplit);
    }

    // ---- per-thread loader state --------------------------------------------------------
    // Operands are fetched with raw buffer loads: address = base + VGPR byte offset + SGPR byte
    // offset, and an offset past the tensor's size returns zeros.  The VGPR offsets change only
    // when the tap changes (rows whose source pixel is padding get an out-of-range offset);
    // the position inside the tap is the SGPR offset.  Steady-state stages therefore issue
    // their loads with no vector-ALU instruction at all - on this chip fp32 MFMA and VALU
    // instructions share the SIMD's issue cycles, so every VALU instruction in the loop is
    // taken from the matrix rate.
    const __amdgpu_buffer_rsrc_t rsrcA =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(p.A), 0, (int)p.aBytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrcB =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(p.B), 0, (int)p.bBytes, 0x00020000);
    constexpr int kOutOfRange = (int)0x80000000;   // tensors are below 2^31 bytes
    const int aSeg = tid & 7, aRow = tid >> 3;
    int rBase[T::PA], rY[T::PA], rX[T::PA];
#pragma unroll
    for (int i = 0; i < T::PA; ++i) {
        const int r = aRow + 32 * i;
        rBase[i] = (rowBase[r] + aSeg * 4) * 4;   // bytes; may be negative before the tap offset is added
        rY[i] = rowY[r];
        rX[i] = rowX[r];
    }
    const int bSeg = tid % T::B_TPR, bRow = tid / T::B_TPR;
    const int wRowStride = p.FH * p.FW * (BWD ? p.DC : p.SC);  // floats per oc in W
    static_assert(!BELEM || BWD, "element-wise B loads exist for backward-data only");
    int bOff[T::PB];   // fixed for the whole kernel
    int bOffE[BELEM ? T::PB : 1][4];
#pragma unroll
    for (int i = 0; i < T::PB; ++i) {
        const int r = bRow + T::B_RPP * i;
        if (BWD) bOff[i] = (r < kBK && n0 + bSeg * 4 < p.DC) ? (r * wRowStride + n0 + bSeg * 4) * 4 : kOutOfRange;
        else bOff[i] = (r < BN && n0 + r < p.DC) ? ((n0 + r) * wRowStride + bSeg * 4) * 4 : kOutOfRange;
        if (BELEM) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int col = n0 + bSeg * 4 + e;
                bOffE[i][e] = (r < kBK && col < p.DC) ? (r * wRowStride + col) * 4 : kOutOfRange;
            }
        }
    }

    // ragged last stage: which of this thread's loads fall inside it
    const bool aLastOk = aSeg * 4 < lastValid;
    bool bLastOk[T::PB];
#pragma unroll
    for (int i = 0; i < T::PB; ++i) bLastOk[i] = BWD ? bRow + T::B_RPP * i < lastValid : bSeg * 4 < lastValid;

    // reduction cursor: current tap (u,v) and chunk within the tap
    int chunk = cLo, tapU = tile.uLo, tapV = tile.vLo;
    if (it0 > 0 && it0 < it1) {   // only stage-list slices after the first start inside the tap list
        const int tapIdx = (int)fast_div((unsigned)it0, p.divChunksPerTap);
        chunk = it0 - tapIdx * chunksPerTap;
        const int du = tapIdx / vCnt;
        tapU += du;
        tapV += tapIdx - du * vCnt;
    }
    int tapOffB = 0;      // floats, uniform
    int aOff[T::PA];      // byte offsets of this thread's A rows for the current tap

    auto set_tap = [&]() __attribute__((always_inline)) {
        int t, dy, dx;
        if (BWD) {
            dy = -tapU;
            dx = -tapV;
            t = (tile.ra + p.sh * tapU) * p.FW + tile.rb + p.sw * tapV;
            tapOffB = t * p.DC;
        } else {
            dy = tapU;
            dx = tapV;
            t = tapU * p.FW + tapV;
            tapOffB = t * p.SC;
        }
        const int tapBytesA = (dy * p.SW + dx) * p.SC * 4;
        if (p.posMajor) {
            // (y,x,n) rows: the tile sits on one pixel position (the batch is a multiple of the row tile),
            // so its tap rectangle holds exactly the taps inside the image - no row needs a test
#pragma unroll
            for (int i = 0; i < T::PA; ++i) aOff[i] = rBase[i] + tapBytesA;
        } else {
#pragma unroll
            for (int i = 0; i < T::PA; ++i) {
                const bool ok = (unsigned)(rY[i] + dy) < (unsigned)p.SH && (unsigned)(rX[i] + dx) < (unsigned)p.SW;
                aOff[i] = ok ? rBase[i] + tapBytesA : kOutOfRange;
            }
        }
    };

    // two register sets: the loads of stage t+2 are in flight while stage t is multiplied
    f4 gaS[2][T::PA], gbS[2][T::PB];

    // item q of a stage: q < PA is A-tile pass q, otherwise B-tile pass q - PA
    constexpr int kItems = T::PA + T::PB;
    auto gload_item = [&](int q, f4 *ga, f4 *gb) __attribute__((always_inline)) {
        const int c0 = chunk * kBK;
        const bool lastChunk = RAGGED && chunk == chunksPerTap - 1;   // uniform
        if (q < T::PA) {
            const int voff = (lastChunk && !aLastOk) ? kOutOfRange : aOff[q];
            ga[q] = __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(rsrcA, voff, c0 * 4, 0));
        } else {
            const int i = q - T::PA;
            const int soff = BWD ? (c0 * wRowStride + tapOffB) * 4 : (tapOffB + c0) * 4;
            const bool drop = lastChunk && !bLastOk[i];
            if (BELEM) {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    gb[i][e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                                                             rsrcB, drop ? kOutOfRange : bOffE[i][e], soff, 0));
            } else {
                gb[i] = __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(rsrcB, drop ? kOutOfRange : bOff[i],
                                                                                    soff, 0));
            }
        }
    };
    auto gload = [&](f4 *ga, f4 *gb) __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < kItems; ++q) gload_item(q, ga, gb);
    };

    auto advance = [&]() __attribute__((always_inline)) {
        if (++chunk == cHi) {
            chunk = cLo;
            if (++tapV > tile.vHi) {
                tapV = tile.vLo;
                ++tapU;
            }
            if (tapU <= tile.uHi) set_tap();
        }
    };

    auto lds_store_item = [&](int q, int buf, const f4 *ga, const f4 *gb) __attribute__((always_inline)) {
        if (q < T::PA) {
            float *a = As + buf * T::A_STAGE;
            *reinterpret_cast<f4 *>(a + (aRow + 32 * q) * LDA + aSeg * 4) = ga[q];
        } else {
            const int i = q - T::PA;
            float *b = Bs + buf * T::B_STAGE;
            const int r = bRow + T::B_RPP * i;
            if (T::B_ROWS % T::B_RPP == 0 || r < T::B_ROWS) *reinterpret_cast<f4 *>(b + r * T::LDB + bSeg * 4) = gb[i];
        }
    };
    auto lds_store = [&](int buf, const f4 *ga, const f4 *gb) __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < kItems; ++q) lds_store_item(q, buf, ga, gb);
    };

    // ---- accumulators -------------------------------------------------------------------
    float16v acc[T::MB][T::NB];
#pragma unroll
    for (int i = 0; i < T::MB; ++i)
#pragma unroll
        for (int j = 0; j < T::NB; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int wm = wave / T::WAVES_N, wn = wave % T::WAVES_N;
    const int l32 = lane & 31, lh = lane >> 5;

    // LDS -> register fragments.  A group is kGK MFMA steps: each half-wave reads kGK consecutive
    // reduction elements with one LDS read per 32 tile rows (16 bytes; 8 bytes for the largest
    // tile, whose registers only hold two small fragment sets).
    constexpr int kGK = BM * BN >= 128 * 128 ? 2 : 4;
    constexpr int kGroups = kBK / (2 * kGK);
    static_assert(kGroups % 2 == 0, "fragment sets alternate across stages");
    typedef float fragv __attribute__((ext_vector_type(kGK)));
    fragv fa[2][T::MB], fb[2][T::NB];
    const float *aFrag = As + (wm * T::WTM + l32) * LDA + lh * kGK;
    const float *bFrag = BWD ? Bs + (lh * kGK) * T::LDB + wn * T::WTN + l32
                             : Bs + (wn * T::WTN + l32) * T::LDB + lh * kGK;
    auto read_group = [&](int buf, int g, fragv *ra, fragv *rb) __attribute__((always_inline)) {
        const float *a = aFrag + buf * T::A_STAGE + g * 2 * kGK;
#pragma unroll
        for (int i = 0; i < T::MB; ++i) ra[i] = *reinterpret_cast<const fragv *>(a + i * 32 * LDA);
#pragma unroll
        for (int j = 0; j < T::NB; ++j) {
            if (BWD) {
                // volatile LDS pointer: keeps single reads with immediate offsets; paired
                // two-address reads would each need a VALU add, which costs matrix time
                lds_cvptr q = (lds_cvptr)(bFrag + buf * T::B_STAGE + (g * 2 * kGK) * T::LDB + j * 32);
#pragma unroll
                for (int t = 0; t < kGK; ++t) rb[j][t] = q[t * T::LDB];
            } else {
                rb[j] = *reinterpret_cast<const fragv *>(bFrag + buf * T::B_STAGE + j * 32 * T::LDB + g * 2 * kGK);
            }
        }
    };

    // One stage.  MFMAs run from LDS buffer `buf` in kGroups groups.  Before the MFMAs of group
    // g are issued the wave requests the fragments of group g+1 and issues its share of
    //   - the global loads of the stage two ahead, into register set `ld` (when doLoad),
    //   - the LDS stores of the next stage, from register set `st` into the other buffer
    //     (when doStore),
    // so memory instructions are spread between MFMAs instead of starving the matrix pipe in
    // a burst at the stage boundary.  The stage's barrier sits before its LAST group: by then
    // every wave holds that group's fragments in registers and has stored its share of the
    // next buffer, so the first fragments of the next stage are requested right after the
    // barrier and arrive while the last group is multiplied - a wave alone on its SIMD does
    // not wait for LDS at the stage boundary.
    constexpr int kSlots = kGroups - 1;
    auto stage = [&](int buf, bool doLoad, int ld, bool doStore, int st) __attribute__((always_inline)) {
#pragma unroll
        for (int g = 0; g < kGroups; ++g) {
            const int cur = g & 1;
            if (g + 1 < kGroups) {
                read_group(buf, g + 1, fa[cur ^ 1], fb[cur ^ 1]);
            } else {
                __syncthreads();
                read_group(buf ^ 1, 0, fa[cur ^ 1], fb[cur ^ 1]);
            }
#pragma unroll
            for (int q = 0; q < kItems; ++q)
                if (q % kSlots == g) {
                    if (doLoad) gload_item(q, gaS[ld], gbS[ld]);
                    if (doStore) lds_store_item(q, buf ^ 1, gaS[st], gbS[st]);
                }
            if (g + 1 == kGroups && doLoad) advance();
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int t = 0; t < kGK; ++t) {
#pragma unroll
                for (int i = 0; i < T::MB; ++i)
#pragma unroll
                    for (int j = 0; j < T::NB; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[cur][i][t], fb[cur][j][t], acc[i][j], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- main loop ----------------------------------------------------------------------
    // Stage t is multiplied from LDS buffer t&1.  Register set t&1 (whose data went to LDS one
    // stage ago) receives the global loads of stage t+2; register set (t+1)&1, loaded one stage
    // ago, moves to the other LDS buffer.  One barrier per stage (inside it).
    if (it0 < it1) {
        const int n = it1 - it0;
        set_tap();
        gload(gaS[0], gbS[0]);
        advance();
        if (n > 1) {
            gload(gaS[1], gbS[1]);
            advance();
        }
        lds_store(0, gaS[0], gbS[0]);
        __syncthreads();
        read_group(0, 0, fa[0], fb[0]);
        int t = 0;
        // steady state: no branch around memory instructions, so every wait is an exact count
        for (; t + 3 < n; t += 2) {
            stage(0, true, 0, true, 1);
            stage(1, true, 1, true, 0);
        }
        // tail: at most three stages left
        for (; t < n; t += 2) {
            stage(0, t + 2 < n, 0, t + 1 < n, 1);
            if (t + 1 >= n) break;
            stage(1, t + 3 < n, 1, t + 2 < n, 0);
        }
    }

    // the stage buffers are free now (every wave read its last fragments before the last barrier;
    // what is still read from them is never used): each wave turns its blocks in its own part
    static_assert(4 * 32 * kLDT <= 2 * T::A_STAGE, "four turning buffers fit over the A stages");
    gather_tile_store<T>(p, slice, n0, outRow, acc, wm, wn, l32, lh, As + wave * 32 * kLDT);
}

template <int BM, int BN, int WAVES_M, bool BWD>
constexpr size_t gather_smem_bytes()
{
    using T = GG<BM, BN, WAVES_M, BWD>;
    return (2 * (T::A_STAGE + T::B_STAGE) + T::TABLE_INTS) * sizeof(float);
}

template <int BM, int BN, int WAVES_M, bool BWD, bool BELEM = false, bool RAGGED = false>
static hipError_t launch_one(const GatherGemmParams &p, int grid, hipStream_t st)
{
    constexpr size_t kSmemBytes = gather_smem_bytes<BM, BN, WAVES_M, BWD>();
    hipLaunchKernelGGL((gather_gemm_kernel<BM, BN, WAVES_M, BWD, BELEM, RAGGED>), dim3((unsigned)grid), dim3(kThreads),
                       kSmemBytes, st, p);
    return hipGetLastError();
}

// Instantiations whose tiles need more LDS than a kernel gets by default (64 KB): the limit is
// raised once per device, outside any stream capture (see prepare_device in the host API).
template <int BM, int BN, int WAVES_M, bool BWD, bool RAGGED>
static hipError_t raise_lds_limit()
{
    constexpr size_t bytes = gather_smem_bytes<BM, BN, WAVES_M, BWD>();
    if (bytes <= 64 * 1024) return hipSuccess;
    return hipFuncSetAttribute(reinterpret_cast<const void *>(gather_gemm_kernel<BM, BN, WAVES_M, BWD, false, RAGGED>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

hipError_t prepare_gather_gemm()
{
    hipError_t e = hipSuccess;
#define MI355_GG_PREP(BM_, BN_, WM_)                                                    \
    if (e == hipSuccess) e = raise_lds_limit<BM_, BN_, WM_, false, false>();            \
    if (e == hipSuccess) e = raise_lds_limit<BM_, BN_, WM_, false, true>();             \
    if (e == hipSuccess) e = raise_lds_limit<BM_, BN_, WM_, true, false>();             \
    if (e == hipSuccess) e = raise_lds_limit<BM_, BN_, WM_, true, true>();
    MI355_GG_PREP(128, 128, 2)
    MI355_GG_PREP(128, 64, 2)
    MI355_GG_PREP(64, 64, 2)
    MI355_GG_PREP(128, 32, 4)
#undef MI355_GG_PREP
    static_assert(gather_smem_bytes<128, 32, 4, true>() <= 64 * 1024, "the 4-byte filter loader's tile fits the default limit");
    return e;
}

hipError_t launch_gather_gemm(const GatherGemmParams &p, bool bwdData, int bm, int bn, int grid,
                              hipStream_t st)
{
    if (!gather_gemm_accepts(p.SC, p.DC, bwdData, bm, bn)) return hipErrorInvalidValue;
    if (bwdData && p.DC % 4 != 0) {   // filter columns by 4-byte loads: on the narrow tile only
        if (bm == 128 && bn == 32) return launch_one<128, 32, 4, true, true, true>(p, grid, st);
        return hipErrorInvalidValue;
    }
    const bool ragged = p.SC % kBK != 0;
#define MI355_GG_CASE(BM_, BN_, WM_)                                                                 \
    if (bm == BM_ && bn == BN_) {                                                                    \
        if (ragged)                                                                                  \
            return bwdData ? launch_one<BM_, BN_, WM_, true, false, true>(p, grid, st)               \
                           : launch_one<BM_, BN_, WM_, false, false, true>(p, grid, st);             \
        return bwdData ? launch_one<BM_, BN_, WM_, true>(p, grid, st)                                \
                       : launch_one<BM_, BN_, WM_, false>(p, grid, st);                              \
    }
    MI355_GG_CASE(128, 128, 2)
    MI355_GG_CASE(128, 64, 2)
    MI355_GG_CASE(64, 64, 2)
    MI355_GG_CASE(128, 32, 4)
#undef MI355_GG_CASE
    return hipErrorInvalidValue;
}

}  // namespace mi355conv
