// Host side of libmi355conv: argument checks, variant/tile/split selection, launches.
// The selection logic is the analogue of the paper's Layer-2 (Sec. III) "logics and
// strategies" above the native kernels, including the size threshold below which the
// small-feature-map operators are chosen (Sec. IV).
#include "../../include/mi355conv.h"
#include "conv_internal.h"

#include <algorithm>
#include <atomic>
#include <cstdio>
#include <cstring>
#include <functional>
#include <mutex>
#include <unordered_map>

using namespace mi355conv;

// Device memory of the library's own for conv2d_bwd_weight_noalloc: the slice partials of callers
// that cannot bring (or allocate) a workspace.  Every GPU the library runs on holds its own copy
// until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; the address of each device's copy is looked up once and kept
// (prepare_device), and only that address is ever handed to kernels.
constexpr size_t kScratchBytes = (size_t)32 << 20;
#if !defined(__HIPCC__)   // host-only sanitizer build (plain C++ compiler): the two HIP spellings below, as that compiler needs them
#define __align__(n) __attribute__((aligned(n)))
#define HIP_SYMBOL(x) (&(x))
#endif
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

std::atomic<int> g_forceVariant{MI355CONV_VARIANT_AUTO};
std::atomic<int> g_forceSplit{0};
std::atomic<int> g_forceBM{0}, g_forceBN{0}, g_forcePosMajor{-1};
std::atomic<int> g_regionalOrder{1};   // 0: region-wise workgroup order off (conv2d_set_order)
thread_local char t_hipError[256] = "";

constexpr long long kMaxElems = (1LL << 31) - 1;
constexpr int kSmallMapPixels = 64;      // maps of at most 8x8 outputs use position-major rows
constexpr int kMaxSplit = 1024;

struct Plan {
    int variant = MI355CONV_VARIANT_DIRECT;
    int bm = 0, bn = 0;
    int split = 1;
    int posMajor = 0;
    int elem = 0;          // element-wise loader (channel counts the 16-byte loader cannot take)
    int fast = 0;          // backward-weight: aligned-map kernel
    int smallIc = 0;       // backward-data: patch-gradient GEMM + col2im kernel for very few input channels
    int grid = 0;
    int tilesM = 0, tilesN = 0;
    int flushChunks = 16;
    long long outElems = 0;
    long long sliceStride = 0;
    size_t wsBytes = 0;
    // backward-data phase table
    int nPhases = 1;
    GatherPhase phase[kMaxPhases] = {};
    // load balancing of unequal tiles (small maps in position-major order)
    int balance = 0;
    int itemsPerClassUnit = 0;   // workgroups per position (gather) / per tap (backward-weight)
    BalanceRuns runs = {};
    unsigned char order[256] = {};   // rank -> position (gather) or tap (backward-weight)
    unsigned char unitWork[256] = {}; // length of unit u (taps / live positions), by rank
    // classes of units of equal length (gather operators): first unit and unit count of each
    int nClasses = 0;
    int classFirstUnit[kMaxBalanceClasses] = {};
    int classUnits[kMaxBalanceClasses] = {};
    // region-wise order of the gather operators (see GatherGemmParams::regional); uses order / unitWork
    int regional = 0, regSnake = 0, regPerPos = 0, regCsPer = 0, regRowTiles = 0, regW = 0;
    unsigned char regLut[8] = {};
    // group-wise order of the (oh,ow,n) backward-weight launches (see WgradParams::regional)
    int regShiftA = 0, regShiftB = 0, regOcTiles = 0, regIcTiles = 0, regSlices = 0;
    int chunksPerSlice = 0;   // gather operators: slices by source channels (0: by stages)
};

int out_extent(int in, int pad, int f, int stride)
{
    long long span = (long long)in + 2LL * pad - f;
    if (span < 0) return 0;
    return (int)(span / stride) + 1;
}

int check_desc(const conv2d_desc *d, Shape *s)
{
    if (!d) return MI355CONV_ERR_NULL_PTR;
    if (d->N <= 0 || d->IH <= 0 || d->IW <= 0 || d->IC <= 0 || d->OC <= 0 || d->FH <= 0 || d->FW <= 0 ||
        d->sh <= 0 || d->sw <= 0 || d->ph < 0 || d->pw < 0)
        return MI355CONV_ERR_BAD_DIM;
    if (d->ph > (1 << 20) || d->pw > (1 << 20)) return MI355CONV_ERR_BAD_DIM;
    const int OH = out_extent(d->IH, d->ph, d->FH, d->sh), OW = out_extent(d->IW, d->pw, d->FW, d->sw);
    if (OH <= 0 || OW <= 0) return MI355CONV_ERR_BAD_DIM;
    const long long xe = (long long)d->N * d->IH * d->IW;
    const long long ye = (long long)d->N * OH * OW;
    const long long we = (long long)d->OC * d->FH * d->FW;
    if (xe > kMaxElems / d->IC || ye > kMaxElems / d->OC || we > kMaxElems / d->IC) return MI355CONV_ERR_BAD_DIM;
    *s = Shape{d->N, d->IH, d->IW, d->IC, d->OC, d->FH, d->FW, d->sh, d->sw, d->ph, d->pw, OH, OW};
    return MI355CONV_OK;
}

inline long long pad4(long long v) { return (v + 3) & ~3LL; }
inline int ceil_div(long long a, long long b) { return (int)((a + b - 1) / b); }

// Source-index headroom of the 32-bit offsets used by the gather-GEMM kernel.
bool offsets_fit_32bit(long long srcElems, const Shape &s, int srcW, int srcC)
{
    const long long halo = ((long long)(s.FH + s.ph + 1) * srcW + s.FW + s.pw + 1) * srcC;
    return srcElems + halo < kMaxElems && halo < (1 << 27);
}

// Both operands of the buffer-load kernels must lie below 2^31 bytes, halo included.
bool buffer_addressable(const Shape &s, long long srcElems, int srcW, int srcC)
{
    const long long halo = ((long long)(s.FH + s.ph + 1) * srcW + s.FW + s.pw + 1) * srcC;
    const long long wElems = (long long)s.OC * s.FH * s.FW * s.IC;
    return (srcElems + halo) * 4 < (1LL << 31) && wElems * 4 < (1LL << 31);
}

// ---- cost model ------------------------------------------------------------------------
// Picks tile and slice count by a small analytic model instead of fixed thresholds.  A launch
// whose workgroups are all resident at once lasts as long as its busiest CU (the grid is
// quantised to the 256 CUs); a larger one divides its work evenly over the CUs and then
// drains; the reduce pass is added when the reduction is sliced.  Only ratios matter.
struct TileCand { int bm, bn; double eff; int resident; };

// Constants of the model, chosen to minimise the regret of the planner's pick over tile x split
// x row-order sweeps of the benchmark layers on MI355X (separately for the gather-GEMM and the
// backward-weight kernel).
struct CostParams {
    double loneEff;        // efficiency factor when a workgroup has a CU to itself
    double fewEff;         // ... when two or three share it
    double refillEff;      // ... when finished workgroups are replaced by waiting ones (desynchronised)
    double mix;            // weight of the other workgroups on the busiest CU (they are not all the longest)
    double tail;           // drain of the last workgroups, in units of one resident set
    double fixedUs;        // launch + prologue + epilogue
    double reduceUs;       // launch + ramp of the slice-reduce kernel
    double reduceBytesPerUs;
};
constexpr CostParams kGatherCost = {0.85, 0.95, 1.0, 1.0, 0.25, 4.0, 0.5, 8.0e6};
constexpr CostParams kWgradCost = {0.80, 0.95, 1.03, 0.56, 0.20, 4.0, 10.0, 6.2e6};

constexpr double kCuFlopPerUs = 157.3e6 / 256.0;   // fp32 MFMA FLOP per microsecond per CU
constexpr size_t kMaxWorkspace = (size_t)1 << 30;

// balanced: long and short workgroups are dealt evenly to the CUs (see GatherGemmParams::balance)
// exactBusiestStages >= 0 (ranking of slice counts only, see best_split): the stages of the busiest CU as
// the host's own dealing leaves them, in place of the estimate from average and longest workgroup, plus
// wgUs per workgroup on that CU for the part of a workgroup's prologue and epilogue that nothing hides.
double launch_cost(const CostParams &k, const TileCand &c, long long tiles, double avgStages, double maxStages,
                   int split, long long outElems, bool balanced = false, double exactBusiestStages = -1.0,
                   double wgUs = 0.0)
{
    const long long grid = tiles * split;
    const int cus = 256;
    const long long slots = (long long)cus * c.resident;
    // time of one workgroup that has the CU's matrix pipes to itself at full efficiency
    const double unit = (2.0 * c.bm * c.bn * kBK) / kCuFlopPerUs;
    const double avgWg = avgStages / split * unit, maxWg = maxStages / split * unit;
    double t;
    if (grid <= slots) {
        // everything is resident at once: the busiest CU holds ceil(grid / 256) workgroups
        const long long perCu = (grid + cus - 1) / cus;
        const double eff = c.eff * (perCu == 1 ? k.loneEff : perCu <= 3 ? k.fewEff : 1.0);
        double busiest = (double)perCu * avgWg;
        const double withLongest = balanced && grid >= 2 * cus
                                       ? busiest + (maxWg - avgWg) * 2.0 / (double)perCu   // what pairing cannot even out
                                       : maxWg + (double)(perCu - 1) * avgWg * k.mix;
        if (withLongest > busiest) busiest = withLongest;
        if (exactBusiestStages >= 0) busiest = exactBusiestStages * unit + (double)perCu * wgUs * eff;
        t = busiest / eff;
    } else {
        // finished workgroups are replaced at once: work divides evenly, plus the drain
        t = ((double)grid / cus * avgWg + k.tail * c.resident * avgWg) / (c.eff * k.refillEff);
    }
    t += k.fixedUs;
    if (split > 1) t += k.reduceUs + (2.0 * split + 1.0) * (double)outElems * 4.0 / k.reduceBytesPerUs;
    return t;
}

// Best slice count for one candidate; returns the cost.
// busiestFn (optional): stages of the busiest CU for a slice count under the order the launch will use, or a
// negative value where unknown.  Where it is known for every candidate slice count, the slice count is
// ranked with it; the cost returned - what tiles and row orders are compared by - stays the estimate.
double best_split(const CostParams &k, const TileCand &c, long long tiles, double avgStages, double maxStages,
                  long long outElems, int *splitOut, int minS = 1, bool balanced = false,
                  const std::function<double(int)> *busiestFn = nullptr, int chunksPerTap = 0)
{
    // Gather operators (chunksPerTap > 0): a slice count that divides the 32-channel chunks of a tap cuts
    // the reduction by source channels, so a slice reads a 1/split part of both operands; any other
    // count cuts the tap-major list of stages and measured 3-8 % slower than its even neighbours.
    auto uneven = [&](int sp) { return chunksPerTap > 0 && sp > 1 && chunksPerTap % sp != 0 ? 1.04 : 1.0; };
    const int forced = g_forceSplit.load();
    int maxS = (int)(avgStages / 2.0);              // keep >= 2 stages per slice on average
    if (maxS > kMaxSplit) maxS = kMaxSplit;
    const long long wsPerSlice = pad4(outElems) * 4;
    if ((long long)maxS * wsPerSlice > (long long)kMaxWorkspace) maxS = (int)(kMaxWorkspace / wsPerSlice);
    if (maxS < minS) maxS = minS;
    if (forced > 0) {
        *splitOut = forced < maxS ? forced : maxS;
        if (*splitOut < minS) *splitOut = minS;
        return launch_cost(k, c, tiles, avgStages, maxStages, *splitOut, outElems, balanced);
    }
    double best = 1e300;
    int bestS = 1;
    for (int sp = minS; sp <= maxS; ++sp) {
        const double t = launch_cost(k, c, tiles, avgStages, maxStages, sp, outElems, balanced) * uneven(sp);
        if (t < best) { best = t; bestS = sp; }
    }
    if (busiestFn) {   // second opinion on the slice count from the dealing itself
        constexpr double kWgUs = 0.7;
        double bestExact = 1e300;
        int exactS = 0;
        bool pickKnown = false;
        for (int sp = minS; sp <= maxS; ++sp) {
            const double stages = (*busiestFn)(sp);
            if (stages < 0) continue;   // not resident at once, or another order: no opinion
            if (sp == bestS) pickKnown = true;
            const double t = launch_cost(k, c, tiles, avgStages, maxStages, sp, outElems, balanced, stages, kWgUs) * uneven(sp);
            if (t < bestExact) { bestExact = t; exactS = sp; }
        }
        if (exactS && pickKnown) {
            bestS = exactS;
            best = launch_cost(k, c, tiles, avgStages, maxStages, bestS, outElems, balanced) * uneven(bestS);
        }
    }
    *splitOut = bestS;
    return best;
}

void finish_plan(Plan &pl, int split)
{
    pl.split = split;
    pl.grid = pl.tilesM * pl.tilesN * pl.split;
    pl.sliceStride = pad4(pl.outElems);
    pl.wsBytes = pl.split > 1 ? (size_t)pl.split * (size_t)pl.sliceStride * sizeof(float) : 0;
}

bool tile_compiled(int bm, int bn, bool gather)
{
    if (gather) return (bm == 128 && (bn == 128 || bn == 64 || bn == 32)) || (bm == 64 && bn == 64);
    return ((bm == 128 || bm == 64) && (bn == 128 || bn == 64)) || (bm == 32 && bn == 128);
}

const TileCand kGatherTiles[] = {{128, 128, 0.88, 2}, {128, 64, 0.93, 2}, {64, 64, 0.945, 4}, {128, 32, 0.80, 3}};
const TileCand kWgradTiles[] = {{128, 128, 0.80, 1}, {64, 128, 0.93, 2}, {128, 64, 0.94, 2}, {64, 64, 0.98, 4},
                                {32, 128, 0.90, 3}};

bool forced_tile(int *bm, int *bn, bool gather)
{
    const int fm = g_forceBM.load(), fn = g_forceBN.load();
    if (fm > 0 && fn > 0 && tile_compiled(fm, fn, gather)) {
        *bm = fm;
        *bn = fn;
        return true;
    }
    return false;
}

int resolve_order(int wanted, bool allowed)
{
    const int f = g_forcePosMajor.load();
    if (f == 0) return 0;
    if (f == 1) return allowed ? 1 : 0;
    return wanted && allowed;
}

bool plan_regional_gather(const Shape &s, Plan &pl, bool bwd);

// Stages of the busiest CU of a (y,x,n)-row forward / unit-stride backward-data launch with the given
// tile and slice count under the region-wise order: the dealing is carried out as the kernels will
// see it (XCD = id % 8, ids 32 apart on an XCD share a CU).  Negative where that order does not apply
// or the launch is not resident at once.
double regional_busiest_stages(const Shape &s, bool bwd, int bm, int bn, int split, int chunksPerTap);

// Forward convolution has a single "phase": all output pixels, all taps.
void set_forward_phase(Plan &pl, const Shape &s)
{
    pl.nPhases = 1;
    GatherPhase &g = pl.phase[0];
    g = GatherPhase{};
    g.dh = s.OH;
    g.dw = s.OW;
    g.nU = s.FH;
    g.nV = s.FW;
    g.divHW = make_fastdiv((unsigned)(s.OH * s.OW));
    g.divW = make_fastdiv((unsigned)s.OW);
}

// Tile and slice count for the element-wise gather kernel (tiles 128x64, 64x64, 128x32).
void plan_elem_tiles(Plan &pl, long long rows, int cols, double stages)
{
    int fbm = 0, fbn = 0;
    const bool haveForced = forced_tile(&fbm, &fbn, true) && !(fbm == 128 && fbn == 128);
    double best = 1e300;
    for (const TileCand &c0 : kGatherTiles) {
        TileCand c = c0;
        if (c.bm == 128 && c.bn == 128) continue;
        if (haveForced) {
            if (c.bm != fbm || c.bn != fbn) continue;
        } else {
            if (c.bn > 32 && c.bn / 2 >= cols) continue;
            if (c.bn == 32 && cols > 32) continue;
        }
        c.eff *= 0.5;   // 4-byte loads, single LDS buffer
        const long long tiles = (long long)ceil_div(rows, c.bm) * ceil_div(cols, c.bn);
        int sp = 1;
        const double t = best_split(kGatherCost, c, tiles, stages, stages, pl.outElems, &sp);
        if (t < best) {
            best = t;
            pl.bm = c.bm;
            pl.bn = c.bn;
            pl.split = sp;
        }
    }
    pl.posMajor = 0;
    pl.tilesM = ceil_div(rows, pl.bm);
    pl.tilesN = ceil_div(cols, pl.bn);
}

// Taps of a padded filter that land inside a map of `in` pixels for output index o.
int taps_in_range(int o, int stride, int pad, int f, int in)
{
    int c = 0;
    for (int t = 0; t < f; ++t) c += (unsigned)(o * stride - pad + t) < (unsigned)in;
    return c;
}

Plan plan_fwd(const Shape &s)
{
    Plan pl;
    pl.outElems = (long long)s.N * s.OH * s.OW * s.OC;
    const int forced = g_forceVariant.load();
    const bool fits = offsets_fit_32bit((long long)s.N * s.IH * s.IW * s.IC, s, s.IW, s.IC);
    // the 16-byte loader addresses both operands with 32-bit byte offsets
    // 16-byte loads along the channel axis; a tap's last 32-channel stage may be partly empty
    const bool chunked = s.IC % 4 == 0 && buffer_addressable(s, (long long)s.N * s.IH * s.IW * s.IC, s.IW, s.IC);
    if (forced == MI355CONV_VARIANT_DIRECT || !fits) return pl;
    pl.variant = MI355CONV_VARIANT_MFMA;
    const long long M = (long long)s.N * s.OH * s.OW;
    int ftm = 0, ftn = 0;
    if (s.FH * s.FW * s.IC <= 32 && (s.IC % 4 != 0 || s.IC <= 4) && g_forceSplit.load() == 0 &&
        !forced_tile(&ftm, &ftn, true) && (long long)s.N * s.IH * s.IW * s.IC * 4 < (1LL << 31) &&
        pl.outElems * 4 < (1LL << 31)) {
        // very few input channels (first layer): the whole reduction is one MFMA stage
        pl.smallIc = 1;
        pl.bm = 128;
        pl.bn = 64;
        pl.tilesM = ceil_div(M, 128);
        pl.tilesN = ceil_div(s.OC, 64);
        finish_plan(pl, 1);
        return pl;
    }
    if (!chunked) {   // element-wise loader: flat reduction range, no tap skipping
        pl.elem = 1;
        const double stages = (double)ceil_div((long long)s.FH * s.FW * s.IC, kBK);
        plan_elem_tiles(pl, M, s.OC, stages);
        set_forward_phase(pl, s);
        finish_plan(pl, pl.split);
        return pl;
    }
    const int chunksPerTap = ceil_div(s.IC, kBK);
    // taps per output position (what a position-major tile walks)
    double avgTapsPos = 0;
    int maxTapsPos = 0;
    for (int oh = 0; oh < s.OH; ++oh)
        for (int ow = 0; ow < s.OW; ++ow) {
            const int t = taps_in_range(oh, s.sh, s.ph, s.FH, s.IH) * taps_in_range(ow, s.sw, s.pw, s.FW, s.IW);
            avgTapsPos += t;
            if (t > maxTapsPos) maxTapsPos = t;
        }
    avgTapsPos /= (double)s.OH * s.OW;
    // position-major rows pay off whenever some taps fall into the padding
    const bool padded = avgTapsPos < s.FH * s.FW;

    int fbm = 0, fbn = 0;
    const bool haveForced = forced_tile(&fbm, &fbn, true);
    double best = 1e300;
    for (const TileCand &c0 : kGatherTiles) {
        TileCand c = c0;
        if (haveForced) {
            if (c.bm != fbm || c.bn != fbn) continue;
        } else {
            // no column tile wider than needed, and the narrow tile only for narrow outputs
            if (c.bn > 32 && c.bn / 2 >= s.OC) continue;
            // the narrow tile: narrow outputs, or a channel count whose last 64-wide tile would be at most half used
            if (c.bn == 32 && s.OC > 32 && !(s.OC % 64 != 0 && s.OC % 64 <= 32)) continue;
        }
        const long long tiles = (long long)ceil_div(M, c.bm) * ceil_div(s.OC, c.bn);
        for (int order = 0; order < 2; ++order) {
            if (resolve_order(order, s.N % c.bm == 0) != order) continue;
            if (order && !padded && g_forcePosMajor.load() != 1) continue;
            const double avgStages = (order ? avgTapsPos : s.FH * s.FW) * chunksPerTap;
            const double maxStages = (order ? maxTapsPos : s.FH * s.FW) * chunksPerTap;
            int sp = 1;
            const bool balanced = order && s.OH * s.OW <= kMaxBalancedPositions;
            const std::function<double(int)> busiest = [&](int split) {
                return order ? regional_busiest_stages(s, false, c.bm, c.bn, split, chunksPerTap) : -1.0;
            };
            const double t = best_split(kGatherCost, c, tiles, avgStages, maxStages, pl.outElems, &sp, 1, balanced,
                                        order ? &busiest : nullptr, chunksPerTap);
            if (t < best) {
                best = t;
                pl.bm = c.bm;
                pl.bn = c.bn;
                pl.posMajor = order;
                pl.split = sp;
            }
        }
    }
    pl.tilesN = ceil_div(s.OC, pl.bn);
    pl.tilesM = ceil_div(M, pl.bm);
    set_forward_phase(pl, s);
    finish_plan(pl, pl.split);
    return pl;
}

// Phase table of backward-data for row tile bm; returns total row tiles.
int build_phases(const Shape &s, int bm, Plan &pl, double *avgTaps, int *maxTaps)
{
    // phases ordered by decreasing tap count so the long tiles are dispatched first
    struct Ph { int ra, rb, taps; };
    Ph ph[kMaxPhases];
    int np = 0;
    for (int ra = 0; ra < s.sh; ++ra)
        for (int rb = 0; rb < s.sw; ++rb) {
            int th = 0, tw = 0;
            for (int fh = 0; fh < s.FH; ++fh) th += (fh % s.sh) == ra;
            for (int fw = 0; fw < s.FW; ++fw) tw += (fw % s.sw) == rb;
            ph[np++] = Ph{ra, rb, th * tw};
        }
    for (int i = 1; i < np; ++i)   // insertion sort, stable
        for (int j = i; j > 0 && ph[j].taps > ph[j - 1].taps; --j) {
            Ph t = ph[j]; ph[j] = ph[j - 1]; ph[j - 1] = t;
        }
    int tiles = 0, k = 0;
    double tapTiles = 0;
    *maxTaps = 0;
    for (int i = 0; i < np; ++i) {
        // destination rows ih with (ih + ph) % sh == ra:  ih = y0, y0 + sh, ...
        const int y0 = ((ph[i].ra - s.ph) % s.sh + s.sh) % s.sh;
        const int x0 = ((ph[i].rb - s.pw) % s.sw + s.sw) % s.sw;
        const int dh = y0 < s.IH ? (s.IH - 1 - y0) / s.sh + 1 : 0;
        const int dw = x0 < s.IW ? (s.IW - 1 - x0) / s.sw + 1 : 0;
        if (dh == 0 || dw == 0) continue;
        GatherPhase &g = pl.phase[k];
        g = GatherPhase{};
        g.tileStart = tiles;
        g.ra = ph[i].ra;
        g.rb = ph[i].rb;
        g.y0 = y0;
        g.x0 = x0;
        g.dh = dh;
        g.dw = dw;
        g.nU = ph[i].ra < s.FH ? (s.FH - 1 - ph[i].ra) / s.sh + 1 : 0;
        g.nV = ph[i].rb < s.FW ? (s.FW - 1 - ph[i].rb) / s.sw + 1 : 0;
        g.divHW = make_fastdiv((unsigned)(dh * dw));
        g.divW = make_fastdiv((unsigned)dw);
        const int t = ceil_div((long long)s.N * dh * dw, bm);
        tiles += t;
        tapTiles += (double)t * ph[i].taps;
        if (ph[i].taps > *maxTaps) *maxTaps = ph[i].taps;
        ++k;
    }
    pl.nPhases = k;
    *avgTaps = tiles ? tapTiles / tiles : 0;
    return tiles;
}

Plan plan_bwd_data(const Shape &s)
{
    Plan pl;
    pl.outElems = (long long)s.N * s.IH * s.IW * s.IC;
    const int forced = g_forceVariant.load();
    const bool fits = s.sh * s.sw <= kMaxPhases &&
                      offsets_fit_32bit((long long)s.N * s.OH * s.OW * s.OC, s, s.OW, s.OC) &&
                      pl.outElems < kMaxElems;
    // up to 32 input channels of any count go through the narrow tile with 4-byte filter loads
    const bool chunked = s.OC % 4 == 0 && (s.IC % 4 == 0 || s.IC <= 32) &&
                         buffer_addressable(s, (long long)s.N * s.OH * s.OW * s.OC, s.OW, s.OC);
    if (forced == MI355CONV_VARIANT_DIRECT || !fits) return pl;
    pl.variant = MI355CONV_VARIANT_MFMA;
    // very few input channels (first layer): P = dY x W as a dense GEMM, then a col2im gather
    int ftm = 0, ftn = 0;
    if (s.sh == 1 && s.sw == 1 && s.IC <= 4 && s.FH * s.FW * s.IC <= 32 && s.OC % kBK == 0 &&
        (4 + s.FH - 1) * (32 + s.FW - 1) <= 224 && g_forceSplit.load() == 0 && !forced_tile(&ftm, &ftn, true) &&
        (long long)s.N * s.OH * s.OW * s.OC * 4 < (1LL << 31) && pl.outElems * 4 < (1LL << 31)) {
        pl.smallIc = 1;
        pl.bm = 128;     // 4 x 32 pixels of dX per workgroup
        pl.bn = 32;
        pl.tilesM = s.N * ceil_div(s.IH, 4) * ceil_div(s.IW, 32);
        pl.tilesN = 1;
        finish_plan(pl, 1);
        return pl;
    }
    if (!chunked) {
        pl.elem = 1;
        // every phase walks the whole flat (tap, oc) range; taps of other phases multiply zeros
        const double stages = (double)ceil_div((long long)s.FH * s.FW * s.OC, kBK);
        plan_elem_tiles(pl, (long long)s.N * s.IH * s.IW, s.IC, stages);
        double avgTaps = 0;
        int maxTaps = 0;
        pl.tilesM = build_phases(s, pl.bm, pl, &avgTaps, &maxTaps);
        int sp = 1;
        TileCand c = {pl.bm, pl.bn, 0.35, 2};
        best_split(kGatherCost, c, (long long)pl.tilesM * pl.tilesN, stages, stages, pl.outElems, &sp);
        finish_plan(pl, sp);
        return pl;
    }
    const int chunksPerTap = ceil_div(s.OC, kBK);
    const bool unitStride = s.sh == 1 && s.sw == 1;
    // stride 1: taps reaching input position (ih, iw) = taps of the flipped filter with pad F-1-p
    double avgTapsPos = 0;
    int maxTapsPos = 0;
    if (unitStride) {
        for (int ih = 0; ih < s.IH; ++ih)
            for (int iw = 0; iw < s.IW; ++iw) {
                int th = 0, tw = 0;
                for (int fh = 0; fh < s.FH; ++fh) th += (unsigned)(ih + s.ph - fh) < (unsigned)s.OH;
                for (int fw = 0; fw < s.FW; ++fw) tw += (unsigned)(iw + s.pw - fw) < (unsigned)s.OW;
                avgTapsPos += th * tw;
                if (th * tw > maxTapsPos) maxTapsPos = th * tw;
            }
        avgTapsPos /= (double)s.IH * s.IW;
    }
    const bool padded = unitStride && avgTapsPos < s.FH * s.FW;

    int fbm = 0, fbn = 0;
    const bool haveForced = forced_tile(&fbm, &fbn, true);
    double best = 1e300;
    for (const TileCand &c0 : kGatherTiles) {
        TileCand c = c0;
        if (s.IC % 4 != 0) {   // 4-byte filter loads exist for the narrow tile only
            if (c.bn != 32) continue;
        } else if (haveForced) {
            if (c.bm != fbm || c.bn != fbn) continue;
        } else {
            if (c.bn > 32 && c.bn / 2 >= s.IC) continue;
            if (c.bn == 32 && s.IC > 32 && !(s.IC % 64 != 0 && s.IC % 64 <= 32)) continue;
        }
        Plan trial = pl;
        double avgTaps = 0;
        int maxTaps = 0;
        const int tilesM = build_phases(s, c.bm, trial, &avgTaps, &maxTaps);
        const long long tiles = (long long)tilesM * ceil_div(s.IC, c.bn);
        for (int order = 0; order < 2; ++order) {
            if (resolve_order(order, s.N % c.bm == 0) != order) continue;
            if (order && !padded && g_forcePosMajor.load() != 1) continue;
            const double a = order && unitStride ? avgTapsPos : avgTaps;
            const double m = order && unitStride ? (double)maxTapsPos : (double)maxTaps;
            int sp = 1;
            const bool balanced = order && unitStride && s.IH * s.IW <= kMaxBalancedPositions;
            const std::function<double(int)> busiest = [&](int split) {
                return regional_busiest_stages(s, true, c.bm, c.bn, split, chunksPerTap);
            };
            const double t = best_split(kGatherCost, c, tiles, a * chunksPerTap, m * chunksPerTap, pl.outElems, &sp, 1,
                                        balanced, order && unitStride ? &busiest : nullptr, chunksPerTap);
            if (t < best) {
                best = t;
                trial.bm = c.bm;
                trial.bn = c.bn;
                trial.posMajor = order;
                trial.split = sp;
                trial.tilesM = tilesM;
                trial.tilesN = ceil_div(s.IC, c.bn);
                pl = trial;
            }
        }
    }
    finish_plan(pl, pl.split);
    return pl;
}

Plan plan_bwd_weight(const Shape &s)
{
    Plan pl;
    pl.outElems = (long long)s.OC * s.FH * s.FW * s.IC;
    const int forced = g_forceVariant.load();
    const long long M = (long long)s.N * s.OH * s.OW;
    const bool eligible = s.OC % 4 == 0 && M < kMaxElems - kBK && (long long)s.N * s.IH * s.IW < kMaxElems;
    if (forced == MI355CONV_VARIANT_DIRECT || !eligible) return pl;
    pl.variant = MI355CONV_VARIANT_MFMA;
    int ftm = 0, ftn = 0;
    if (s.FH * s.FW * s.IC <= 32 && !forced_tile(&ftm, &ftn, false) &&
        (long long)s.N * s.IH * s.IW * s.IC * 4 < (1LL << 31) && M * s.OC * 4 < (1LL << 31)) {
        // very few input channels (first layer): one 64 x 32 tile per 64 output channels, rows sliced
        pl.smallIc = 1;
        pl.bm = 64;
        pl.bn = 32;
        pl.tilesM = ceil_div(s.OC, 64);
        pl.tilesN = 1;
        const int chunks = ceil_div(M, kBK);
        int sp = g_forceSplit.load();
        if (sp <= 0) {   // about two workgroups per CU, at least 4 stages each
            sp = 512 / pl.tilesM;
            if (sp > chunks / 4) sp = chunks / 4;
        }
        if (sp > chunks) sp = chunks;
        if (sp > kMaxSplit) sp = kMaxSplit;
        if (sp < 1) sp = 1;
        finish_plan(pl, sp);
        return pl;
    }
    pl.elem = s.IC % 4 != 0;
    const int chunksAll = ceil_div(M, kBK);
    const int ohow = s.OH * s.OW;
    // fast kernel: rows of a 32-row stage always sit at the same place relative to its first pixel
    const bool aligned = (kBK % s.OW == 0 && (ohow % kBK == 0 || kBK % ohow == 0)) || s.OW % kBK == 0;
    pl.fast = !pl.elem && aligned && chunksAll >= 1 &&
              (long long)s.N * s.IH * s.IW * s.IC * 4 < (1LL << 31) && M * s.OC * 4 < (1LL << 31);
    // the fast kernel keeps a 64-bit mask of output positions in (oh,ow,n) order
    const bool smallMap = (s.ph > 0 || s.pw > 0) && s.OH * s.OW <= kSmallMapPixels;
    // ... and takes (oh,ow,n) order only where an output row is at most one stage long
    const int posMajor = resolve_order(smallMap, s.N % kBK == 0 && !pl.elem && (!pl.fast || (ohow <= 64 && s.OW <= kBK)));
    const long long Ktot = (long long)s.FH * s.FW * s.IC;
    const int chunks = ceil_div(M, kBK);
    // fraction of (position, tap) pairs inside the image = share of stages a tile keeps
    double live = 1.0;
    if (posMajor) {
        double inside = 0;
        for (int oh = 0; oh < s.OH; ++oh)
            for (int ow = 0; ow < s.OW; ++ow)
                inside += taps_in_range(oh, s.sh, s.ph, s.FH, s.IH) * taps_in_range(ow, s.sw, s.pw, s.FW, s.IW);
        live = inside / ((double)s.OH * s.OW * s.FH * s.FW);
    }
    int fbm = 0, fbn = 0;
    const bool haveForced = forced_tile(&fbm, &fbn, false);
    double best = 1e300;
    for (int pass = 0; pass < 2 && pl.bm == 0; ++pass) {   // second pass: the forced tile does not apply here
        for (const TileCand &c : kWgradTiles) {
            if (pl.elem && c.bn != 64) continue;   // element-wise X loader is compiled for 64-wide tiles
            // one block row (fast kernel only): narrow outputs, or a channel count whose last 64-row tile
            // would be at most half used
            if (c.bm == 32 && (!pl.fast || (s.OC > 32 && !(s.OC % 64 != 0 && s.OC % 64 <= 32)))) continue;
            if (pass == 0 && haveForced && !(pl.elem && fbn != 64)) {
                if (c.bm != fbm || c.bn != fbn) continue;
            } else {
                if (c.bm > 64 && c.bm / 2 >= s.OC) continue;
                if (c.bn > 64 && c.bn / 2 >= Ktot && c.bm != 32) continue;
            }
            const long long tiles = (long long)ceil_div(s.OC, c.bm) * ceil_div(Ktot, c.bn);
            int sp = 1;
            const double t = best_split(kWgradCost, c, tiles, chunks * live, (double)chunks, pl.outElems, &sp);
            if (t < best) {
                best = t;
                pl.bm = c.bm;
                pl.bn = c.bn;
                pl.split = sp;
            }
        }
    }
    pl.posMajor = posMajor;
    pl.tilesM = ceil_div(s.OC, pl.bm);
    pl.tilesN = ceil_div(Ktot, pl.bn);
    // A grid barely above one lap of 256 leaves most CUs with one workgroup and a few with two whole
    // ones; two slices per tile halve the items, and the dealing then fills the CUs to 3 halves at most
    // (measured on 288 tiles: 43 -> 38 us).  The model's whole-number quantisation does not see this.
    if (posMajor && pl.fast && pl.split == 1 && g_forceSplit.load() == 0 && s.IC % pl.bn == 0) {
        const long long tiles = (long long)pl.tilesM * pl.tilesN;
        if (tiles > 256 && tiles < 384 && chunks * live >= 8) pl.split = 2;
    }
    pl.flushChunks = M > 150000 ? 8 : 16;   // fp32 chains of at most 512 products (256 for very long reductions)
    finish_plan(pl, pl.split);
    return pl;
}

int hip_fail(hipError_t e)
{
    snprintf(t_hipError, sizeof t_hipError, "%s", hipGetErrorString(e));
    return MI355CONV_ERR_HIP;
}

// ---- per-device set-up -------------------------------------------------------------------
constexpr int kMaxDevices = 64;
std::mutex g_deviceMutex;
std::atomic<int> g_deviceReady[kMaxDevices];
void *g_scratchPtr[kMaxDevices];

// Once per device, with that device current and no stream capture under way: raises the LDS limit
// of the large-tile kernels and looks up the device's scratch array.
int prepare_device(int *devOut)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev < 0 || dev >= kMaxDevices) return hip_fail(hipErrorInvalidDevice);
    if (devOut) *devOut = dev;
    if (g_deviceReady[dev].load(std::memory_order_acquire)) return MI355CONV_OK;
    std::lock_guard<std::mutex> lock(g_deviceMutex);
    if (g_deviceReady[dev].load(std::memory_order_relaxed)) return MI355CONV_OK;
    e = prepare_gather_gemm();
    if (e == hipSuccess) e = prepare_wgrad();
    if (e == hipSuccess) e = prepare_wgrad_fast();
    void *ptr = nullptr;
    if (e == hipSuccess) e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_fail(e);
    if (!ptr) return hip_fail(hipErrorInvalidSymbol);
    g_scratchPtr[dev] = ptr;
    g_deviceReady[dev].store(1, std::memory_order_release);
    return MI355CONV_OK;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_buffers(const void *a, const void *b, const void *c, const Plan &pl, const void *ws, size_t wsBytes)
{
    if (!a || !b || !c) return MI355CONV_ERR_NULL_PTR;
    if (!aligned16(a) || !aligned16(b) || !aligned16(c)) return MI355CONV_ERR_ALIGNMENT;
    if (pl.wsBytes > 0) {
        if (!ws || wsBytes < pl.wsBytes) return MI355CONV_ERR_WORKSPACE;
        if (!aligned16(ws)) return MI355CONV_ERR_ALIGNMENT;
    }
    return MI355CONV_OK;
}

void fill_gather_params(GatherGemmParams &g, const Plan &pl)
{
    g.posMajor = pl.posMajor;
    g.split = pl.split;
    g.sliceStride = pl.sliceStride;
    g.tilesN = pl.tilesN;
    g.xcdUnit = pl.tilesN * pl.split * 2;   // both column tiles, all slices, two neighbouring row tiles
    g.nPhases = pl.nPhases;
    for (int i = 0; i < kMaxPhases; ++i) {
        g.phase[i] = pl.phase[i];
        g.phaseStart[i] = i < pl.nPhases ? pl.phase[i].tileStart : 0x7fffffff;
    }
    g.divTilesN = make_fastdiv((unsigned)pl.tilesN);
    g.divSplit = make_fastdiv((unsigned)pl.split);
    g.divXcdUnit = make_fastdiv((unsigned)g.xcdUnit);
    const int span = 8 * g.xcdUnit;
    g.xcdWhole = (pl.grid / span) * span;
    g.grid = pl.grid;
    g.runsN = 0;
    g.classesN = 0;
    for (int c = 0; c < kMaxBalanceClasses; ++c) g.classes.rankStart[c] = 0x7fffffff;   // unused classes never match
    for (int i = 0; i < kMaxBalanceRuns; ++i) g.runs.idStart[i] = 0x7fffffff;   // unused run entries never match
}

// Longest-first dealing of a launch's workgroups to the 256 CUs.  unitWork[u] is the length of
// the workgroups of unit u (a position or a tap), each unit holding perUnit workgroups; units
// come ranked by descending length.  While the whole grid is resident, workgroup ids 256 apart
// share a CU, so CU c holds ids c, c + 256, ...: every item goes to the least loaded CU that
// still has a free id, CUs with equal contents are made neighbours, and the permutation comes
// out as a few runs.  Returns false (identity order, still longest first) when the grid is
// not resident at once or the runs do not fit.
bool build_balance_runs(const int *unitWork, int nUnits, int perUnit, int grid, int resident, BalanceRuns *out,
                        bool oneXcd = false)
{
    // oneXcd: the same dealing for the workgroups of a single XCD (32 CUs; slots are the ids' places on
    // that XCD, so the columns of a partial last lap are simply its first ones)
    out->n = 0;
    constexpr int kCus = 256;
    const int cus = oneXcd ? 32 : kCus;
    if (grid <= cus || grid > cus * resident || resident > 8 || nUnits > 256) return false;
    const int laps = grid / cus, extra = grid % cus;
    struct Deal {
        int load[kCus], cnt[kCus];
        short cls[kCus][8];
        int worst;
    };
    auto fresh = [&](Deal &d) {
        for (int c = 0; c < cus; ++c) {
            d.load[c] = 0;
            d.cnt[c] = 0;
            for (int l = 0; l < 8; ++l) d.cls[c][l] = -1;
        }
    };
    auto finish = [&](Deal &d) {
        d.worst = 0;
        for (int c = 0; c < cus; ++c)
            if (d.load[c] > d.worst) d.worst = d.load[c];
    };
    // Columns are slots (balance_slot): column j of the last, partial lap exists iff some id
    // 256 * laps + c with c < extra has j as its slot in the whole laps - ids of the partial lap
    // keep their value, so those are the columns c' with slot-inverse below `extra`.
    bool roomy[kCus];
    for (int j = 0; j < cus; ++j) roomy[j] = false;
    for (int c = 0; c < extra; ++c) roomy[oneXcd ? c : (c & 7) * 32 + (c >> 3)] = true;
    // Two dealings, the better one is kept.  The roomy columns hold one item more than the
    // others: (a) give them the lightest items up front, then deal the rest to the other
    // columns; (b) deal everything to all columns, the roomy ones last among equals.
    auto lpt = [&](Deal &d, const int *take, int pass) -> bool {   // pass 0: roomy only, 1: others only, 2: all
        for (int u = 0; u < nUnits; ++u)
            for (int j = 0; j < take[u]; ++j) {
                int best = -1;
                for (int phase = 0; phase < 2; ++phase)     // non-roomy columns win ties
                    for (int c = 0; c < cus; ++c) {
                        if (roomy[c] != (phase == 1)) continue;
                        if (pass == 0 && !roomy[c]) continue;
                        if (pass == 1 && roomy[c]) continue;
                        const int cap = laps + (roomy[c] ? 1 : 0);
                        if (d.cnt[c] < cap && (best < 0 || d.load[c] < d.load[best])) best = c;
                    }
                if (best < 0) return false;
                d.cls[best][d.cnt[best]++] = (short)u;
                d.load[best] += unitWork[u];
            }
        return true;
    };
    static thread_local Deal a, bdeal;
    int light[256], heavy[256], all[256];
    {
        long long need = (long long)(laps + 1) * extra;
        for (int u = nUnits - 1; u >= 0; --u) {
            const int t = (int)(need < perUnit ? need : perUnit);
            light[u] = t;
            heavy[u] = perUnit - t;
            all[u] = perUnit;
            need -= t;
        }
    }
    fresh(a);
    const bool okA = lpt(a, light, 0) && lpt(a, heavy, 1);
    if (okA) finish(a);
    fresh(bdeal);
    const bool okB = lpt(bdeal, all, 2);
    if (okB) finish(bdeal);
    if (!okA && !okB) return false;
    Deal &d = (okA && (!okB || a.worst <= bdeal.worst)) ? a : bdeal;
    short (*cls)[8] = d.cls;
    // neighbours with equal contents: within each capacity group the columns' contents are
    // reassigned in sorted order (column j takes the contents of abstract column col[j])
    int col[kCus], idxRoomy[kCus], idxPlain[kCus], nr = 0, np_ = 0;
    for (int c = 0; c < cus; ++c) (roomy[c] ? idxRoomy[nr++] : idxPlain[np_++]) = c;
    auto less = [&](int x, int y) {   // by the lengths of the contents, longest first
        for (int l = 0; l < 8; ++l) {
            const int wx = cls[x][l] < 0 ? -1 : unitWork[cls[x][l]], wy = cls[y][l] < 0 ? -1 : unitWork[cls[y][l]];
            if (wx != wy) return wx > wy;
        }
        return false;
    };
    {
        int tmp[kCus];
        for (int i = 0; i < nr; ++i) tmp[i] = idxRoomy[i];
        std::stable_sort(tmp, tmp + nr, less);
        for (int i = 0; i < nr; ++i) col[idxRoomy[i]] = tmp[i];
        for (int i = 0; i < np_; ++i) tmp[i] = idxPlain[i];
        std::stable_sort(tmp, tmp + np_, less);
        for (int i = 0; i < np_; ++i) col[idxPlain[i]] = tmp[i];
    }
    // emit runs in slot order; items of units of equal length are interchangeable, and such
    // units are neighbours in the ranking, so a class of them is one range of ranks
    int classOf[256], classBase[256], emitted[256], nClasses = 0;
    for (int u = 0; u < nUnits; ++u) {
        if (u == 0 || unitWork[u] != unitWork[u - 1]) {
            classBase[nClasses] = u * perUnit;
            emitted[nClasses] = 0;
            ++nClasses;
        }
        classOf[u] = nClasses - 1;
    }
    int n = 0, prevClass = -1;
    for (int l = 0; l <= laps; ++l) {
        const int width = l < laps ? cus : extra;
        for (int c = 0; c < width; ++c) {
            // whole laps are walked by slot; in the partial lap id c sits in column slot(c)
            const int column = (l < laps || oneXcd) ? c : (c & 7) * 32 + (c >> 3);
            const int u = cls[col[column]][l];
            if (u < 0) return false;
            const int k = classOf[u];
            if (k != prevClass) {
                if (n == kMaxBalanceRuns) { out->n = 0; return false; }
                out->idStart[n] = l * cus + c;
                out->rankStart[n] = classBase[k] + emitted[k];
                ++n;
                prevClass = k;
            }
            ++emitted[k];
        }
    }
    out->n = n;
    return true;
}

// (y,x,n) row order on a small map: rank the positions by the number of taps inside the image
// (= stages of their tiles), most first.  Only for the single-phase cases (forward, unit-stride
// backward-data), where a row tile lies on one position.
void plan_balance_gather(const Shape &s, Plan &pl, bool bwd)
{
    pl.balance = 0;
    if (!pl.posMajor || pl.elem || pl.nPhases != 1 || s.N % pl.bm != 0) return;
    if (bwd && (s.sh != 1 || s.sw != 1)) return;
    const int dh = bwd ? s.IH : s.OH, dw = bwd ? s.IW : s.OW;
    const int nPos = dh * dw;
    if (nPos > kMaxBalancedPositions || pl.grid <= 256) return;
    int taps[kMaxBalancedPositions];
    int lo = 1 << 30, hi = 0;
    for (int i = 0; i < dh; ++i)
        for (int j = 0; j < dw; ++j) {
            int th = 0, tw = 0;
            for (int f = 0; f < s.FH; ++f)
                th += bwd ? (unsigned)(i + s.ph - f) < (unsigned)s.OH : (unsigned)(i * s.sh - s.ph + f) < (unsigned)s.IH;
            for (int f = 0; f < s.FW; ++f)
                tw += bwd ? (unsigned)(j + s.pw - f) < (unsigned)s.OW : (unsigned)(j * s.sw - s.pw + f) < (unsigned)s.IW;
            const int t = th * tw;
            taps[i * dw + j] = t;
            if (t < lo) lo = t;
            if (t > hi) hi = t;
        }
    if (lo == hi) return;
    int order[kMaxBalancedPositions];
    for (int i = 0; i < nPos; ++i) order[i] = i;
    std::stable_sort(order, order + nPos, [&](int a, int b) { return taps[a] > taps[b]; });
    int work[kMaxBalancedPositions];
    for (int i = 0; i < nPos; ++i) {
        pl.order[i] = (unsigned char)order[i];
        work[i] = taps[order[i]];
        pl.unitWork[i] = (unsigned char)(work[i] < 255 ? work[i] : 255);
    }
    pl.itemsPerClassUnit = (s.N / pl.bm) * pl.tilesN * pl.split;
    const int resident = pl.bm * pl.bn <= 64 * 64 ? 4 : 2;
    build_balance_runs(work, nPos, pl.itemsPerClassUnit, pl.grid, resident, &pl.runs);
    pl.balance = 1;
    // Classes of positions with equal tap counts (neighbours in the ranking).  The class-wise rank
    // order keeps a filter slice on one XCD at the price of spreading a row tile's column tiles over
    // XCDs, so it is used where the filter is the larger operand and does not fit an XCD's 4 MB L2.
    pl.nClasses = 0;
    const long long wBytes = 4LL * s.OC * s.FH * s.FW * s.IC;
    const long long aBytes = 4LL * s.N * (bwd ? (long long)s.OH * s.OW * s.OC : (long long)s.IH * s.IW * s.IC);
    const bool filterHeavy = wBytes > (2LL << 20) && wBytes >= aBytes;
    for (int i = 0; i < nPos && filterHeavy; ++i) {
        if (i == 0 || work[i] != work[i - 1]) {
            if (pl.nClasses == kMaxBalanceClasses) { pl.nClasses = 0; break; }   // too many: unit-wise order
            pl.classFirstUnit[pl.nClasses] = i;
            pl.classUnits[pl.nClasses] = 0;
            ++pl.nClasses;
        }
        ++pl.classUnits[pl.nClasses - 1];
    }
}

// Region-wise order for (y,x,n) launches of one phase.  Workgroup ids go round-robin to the 8 XCDs, each with
// its own L2, so the tiles of a launch are divided among the XCDs as a product of (spatial regions) x
// (image groups) x (groups of (slice, column tile) pairs), the factors chosen for the fewest bytes
// fetched: a spatial region re-reads only its halo of the gathered tensor, an image group shares
// nothing with the others, and a (slice, column) group reads its own part of the filter (and, with
// slices by channels, its own channels of the gathered tensor).  Regions are halves / quarters of the
// map mirrored onto the first one, which needs even extents and tap counts that mirror.
bool plan_regional_gather(const Shape &s, Plan &pl, bool bwd)
{
    pl.regional = 0;
    if (!pl.posMajor || pl.elem || pl.nPhases != 1 || s.N % pl.bm != 0) return false;
    if (bwd && (s.sh != 1 || s.sw != 1)) return false;
    if (pl.grid < 256 || pl.grid % 8 != 0) return false;
    const int dh = bwd ? s.IH : s.OH, dw = bwd ? s.IW : s.OW;
    const int srcH = bwd ? s.OH : s.IH, srcW = bwd ? s.OW : s.IW, srcC = bwd ? s.OC : s.IC;
    const int yStep = bwd ? 1 : s.sh, xStep = bwd ? 1 : s.sw;
    if ((long long)dh * dw > 1024) return false;
    int taps[1024];
    for (int i = 0; i < dh; ++i)
        for (int j = 0; j < dw; ++j) {
            int th = 0, tw = 0;
            for (int f = 0; f < s.FH; ++f)
                th += bwd ? (unsigned)(i + s.ph - f) < (unsigned)s.OH : (unsigned)(i * s.sh - s.ph + f) < (unsigned)s.IH;
            for (int f = 0; f < s.FW; ++f)
                tw += bwd ? (unsigned)(j + s.pw - f) < (unsigned)s.OW : (unsigned)(j * s.sw - s.pw + f) < (unsigned)s.IW;
            taps[i * dw + j] = th * tw;
        }
    bool symY = dh % 2 == 0, symX = dw % 2 == 0;
    for (int i = 0; i < dh; ++i)
        for (int j = 0; j < dw; ++j) {
            if (taps[(dh - 1 - i) * dw + j] != taps[i * dw + j]) symY = false;
            if (taps[i * dw + dw - 1 - j] != taps[i * dw + j]) symX = false;
        }
    // measured: an XCD whose tiles cover the whole map runs 2-5 % slower than under the chip-wide dealing,
    // whatever the other two factors are, so without a spatial split the older order stays
    if (!symY && !symX) return false;
    const int rtpp = s.N / pl.bm, cs = pl.tilesN * pl.split;
    const double aBytes = 4.0 * s.N * srcH * srcW * srcC, wBytes = 4.0 * s.OC * s.FH * s.FW * s.IC;
    double bestCost = 0;
    int bRy = 0, bRx = 0, bG = 0, bC = 0;
    for (int Ry = 2; Ry >= 1; --Ry)          // ties go to the split along y (regions of whole rows)
        for (int Rx = 1; Rx <= 2; ++Rx)
            for (int G = 1; G <= 8; G *= 2) {
                if ((Ry == 2 && !symY) || (Rx == 2 && !symX) || rtpp % G != 0) continue;
                if (Ry * Rx == 1) continue;   // see above
                const int RG = Ry * Rx * G;
                if (8 % RG != 0) continue;
                const int C = 8 / RG;
                if (cs % C != 0 || (dh / Ry) * (dw / Rx) > kMaxBalancedPositions) continue;
                const int needY = Ry == 1 ? srcH : std::min(srcH, (dh / Ry - 1) * yStep + s.FH);
                const int needX = Rx == 1 ? srcW : std::min(srcW, (dw / Rx - 1) * xStep + s.FW);
                const int csPer = cs / C;
                const int slices = std::min(pl.split, (csPer + pl.tilesN - 1) / pl.tilesN + (csPer > pl.tilesN && csPer % pl.tilesN ? 1 : 0));
                const double chanFrac = pl.chunksPerSlice ? (double)slices / pl.split : 1.0;
                const double aTot = 8.0 * aBytes * ((double)needY / srcH) * ((double)needX / srcW) / G * chanFrac;
                const double wTot = wBytes * RG;
                if (!bRy || aTot + wTot < bestCost) {
                    bestCost = aTot + wTot;
                    bRy = Ry; bRx = Rx; bG = G; bC = C;
                }
            }
    if (!bRy) return false;
    const int rh = dh / bRy, rw = dw / bRx, nPos = rh * rw;
    int order[kMaxBalancedPositions];
    for (int i = 0; i < nPos; ++i) order[i] = i;
    auto tapsAt = [&](int l) { return taps[(l / rw) * dw + l % rw]; };
    std::stable_sort(order, order + nPos, [&](int a, int b) { return tapsAt(a) > tapsAt(b); });
    for (int i = 0; i < nPos; ++i) {
        pl.order[i] = (unsigned char)order[i];
        const int t = tapsAt(order[i]);
        pl.unitWork[i] = (unsigned char)(t < 255 ? t : 255);
    }
    for (int x = 0; x < 8; ++x) {
        const int c = x % bC, g = (x / bC) % bG, r = x / (bC * bG);
        pl.regLut[x] = (unsigned char)(c | (g << 3) | ((r % bRx) << 6) | ((r / bRx) << 7));
    }
    pl.regCsPer = cs / bC;
    pl.regRowTiles = rtpp / bG;
    pl.regPerPos = pl.regRowTiles * pl.regCsPer;
    pl.regW = rw;
    pl.itemsPerClassUnit = pl.regPerPos;
    const int resident = pl.bm * pl.bn <= 64 * 64 ? 4 : 2;
    pl.regSnake = pl.grid / 8 <= 32 * resident;
    pl.regional = 1;
    return true;
}

double regional_busiest_stages(const Shape &s, bool bwd, int bm, int bn, int split, int chunksPerTap)
{
    if (!g_regionalOrder.load() || s.N % bm != 0) return -1.0;
    Plan t;
    t.variant = MI355CONV_VARIANT_MFMA;
    t.bm = bm;
    t.bn = bn;
    t.posMajor = 1;
    t.nPhases = 1;
    t.split = split;
    const int dh = bwd ? s.IH : s.OH, dw = bwd ? s.IW : s.OW;
    t.tilesM = ceil_div((long long)s.N * dh * dw, bm);
    t.tilesN = ceil_div(bwd ? s.IC : s.OC, bn);
    t.grid = t.tilesM * t.tilesN * split;
    if (split > 1 && chunksPerTap % split == 0) t.chunksPerSlice = chunksPerTap / split;
    if (!plan_regional_gather(s, t, bwd) || !t.regSnake) return -1.0;
    int load[32] = {};
    const int local = t.grid / 8;
    for (int q = 0; q < local; ++q) {
        const int lap = q >> 5, left = local - (lap << 5), w = left < 32 ? left : 32;
        int c = q & 31;
        if (lap & 1) c = w - 1 - c;
        load[q & 31] += t.unitWork[((lap << 5) + c) / t.regPerPos];
    }
    int worst = 0;
    for (int c = 0; c < 32; ++c)
        if (load[c] > worst) worst = load[c];
    return (double)worst * chunksPerTap / split;
}

// Slicing and workgroup order of a gather-operator plan.
void plan_order_gather(const Shape &s, Plan &pl, bool bwd)
{
    pl.balance = 0;
    pl.regional = 0;
    pl.chunksPerSlice = 0;
    if (pl.smallIc) return;
    const int chunks = ceil_div(bwd ? s.OC : s.IC, kBK);
    if (!pl.elem && pl.split > 1 && chunks % pl.split == 0) pl.chunksPerSlice = chunks / pl.split;
    if (g_regionalOrder.load() && plan_regional_gather(s, pl, bwd)) return;
    plan_balance_gather(s, pl, bwd);
}

// Backward-weight in (oh,ow,n) order: rank the taps by the number of output positions at which
// they are inside the image.
void plan_balance_wgrad(const Shape &s, Plan &pl)
{
    pl.balance = 0;
    const int nTaps = s.FH * s.FW;
    if (!pl.posMajor || !pl.fast || s.IC % pl.bn != 0 || nTaps > kMaxBalancedTaps || pl.grid <= 256) return;
    int live[kMaxBalancedTaps];
    int lo = 1 << 30, hi = 0;
    for (int fh = 0; fh < s.FH; ++fh)
        for (int fw = 0; fw < s.FW; ++fw) {
            int lh = 0, lw = 0;
            for (int oh = 0; oh < s.OH; ++oh) lh += (unsigned)(oh * s.sh - s.ph + fh) < (unsigned)s.IH;
            for (int ow = 0; ow < s.OW; ++ow) lw += (unsigned)(ow * s.sw - s.pw + fw) < (unsigned)s.IW;
            const int t = lh * lw;
            live[fh * s.FW + fw] = t;
            if (t < lo) lo = t;
            if (t > hi) hi = t;
        }
    if (lo == hi) return;
    int order[kMaxBalancedTaps];
    for (int i = 0; i < nTaps; ++i) order[i] = i;
    std::stable_sort(order, order + nTaps, [&](int a, int b) { return live[a] > live[b]; });
    int work[kMaxBalancedTaps];
    for (int i = 0; i < nTaps; ++i) {
        pl.order[i] = (unsigned char)order[i];
        work[i] = live[order[i]];
        pl.unitWork[i] = (unsigned char)(work[i] < 255 ? work[i] : 255);
    }
    const int resident = pl.bm * pl.bn <= 64 * 64 ? 4 : pl.bm * pl.bn >= 128 * 128 ? 1 : 2;
    pl.balance = 1;
    // Group-wise order: the 8 XCDs (workgroup id % 8, one L2 each) divide the tiles as (A groups of
    // output-channel tiles) x (B groups of input-channel tiles) x (S groups of slices), A*B*S = 8; an
    // XCD then reads 1/(A*S) of dY and about 1/(B*S) of X (a slice group's rows plus the rows its taps
    // reach beyond them), so dY is fetched B times and X A times over.  Powers of two only.
    pl.regional = 0;
    const int icTiles = s.IC / pl.bn;
    if (g_regionalOrder.load() && pl.grid % 8 == 0) {
        const double gBytes = 4.0 * s.N * s.OH * s.OW * s.OC, xBytes = 4.0 * s.N * s.IH * s.IW * s.IC;
        const int ohow = s.OH * s.OW;
        double bestCost = 0;
        int bA = 0, bB = 0, bS = 0;
        for (int A = 1; A <= 8; A *= 2)
            for (int B = 1; A * B <= 8; B *= 2) {
                const int S = 8 / (A * B);
                if (pl.tilesM % A != 0 || icTiles % B != 0 || pl.split % S != 0) continue;
                // positions a slice group covers, and those its taps reach on either side
                const double len = (double)ohow / S, reach = (s.FH / 2) * s.OW + s.FW / 2;
                const double halo = S == 1 ? 1.0 : std::min((double)S, (len + 2 * reach) / len);
                const double cost = gBytes * B + xBytes * A * halo;
                if (!bA || cost < bestCost) {
                    bestCost = cost;
                    bA = A; bB = B; bS = S;
                }
            }
        if (bA) {
            int lgA = 0, lgB = 0;
            while ((1 << lgA) < bA) ++lgA;
            while ((1 << lgB) < bB) ++lgB;
            pl.regional = 1;
            pl.regShiftA = lgA;
            pl.regShiftB = lgB;
            pl.regOcTiles = pl.tilesM / bA;
            pl.regIcTiles = icTiles / bB;
            pl.regSlices = pl.split / bS;
            pl.itemsPerClassUnit = pl.regOcTiles * pl.regIcTiles * pl.regSlices;
            build_balance_runs(work, nTaps, pl.itemsPerClassUnit, pl.grid / 8, resident, &pl.runs, true);
            return;
        }
    }
    pl.itemsPerClassUnit = icTiles * pl.tilesM * pl.split;
    build_balance_runs(work, nTaps, pl.itemsPerClassUnit, pl.grid, resident, &pl.runs);
}

// The plan against the preconditions of the launcher it names (the same predicates the launchers
// apply).  A plan that fails here is a defect of the planner; the entry points then report
// MI355CONV_ERR_UNSUPPORTED before any HIP call instead of a launch error.
bool plan_launchable(int op, const Shape &s, const Plan &pl)
{
    if (pl.variant != MI355CONV_VARIANT_MFMA) return true;
    if (pl.bm <= 0 || pl.bn <= 0 || pl.split < 1 || pl.grid < 1) return false;
    if (op == MI355CONV_OP_BWD_WEIGHT) {
        if (pl.smallIc) return patch_small_ic_accepts(s.IC, s.FH, s.FW) && pl.bm == 64 && pl.bn == 32;
        if (pl.fast) return wgrad_fast_accepts(s.N, s.OH, s.OW, s.IC, s.OC, pl.posMajor, pl.bm, pl.bn);
        return wgrad_accepts(s.N, s.IC, s.OC, pl.posMajor, pl.elem != 0, pl.bm, pl.bn);
    }
    const bool bwd = op == MI355CONV_OP_BWD_DATA;
    if (pl.smallIc)
        return bwd ? bwd_data_small_ic_accepts(s.IC, s.OC, s.FH, s.FW, s.sh, s.sw) : patch_small_ic_accepts(s.IC, s.FH, s.FW);
    if (pl.posMajor && s.N % pl.bm != 0) return false;   // a row tile sits on one pixel position
    if (pl.elem) return gather_elem_accepts(pl.bm, pl.bn);
    return gather_gemm_accepts(bwd ? s.OC : s.IC, bwd ? s.IC : s.OC, bwd, pl.bm, pl.bn);
}

// Plans depend on the descriptor and the tuning overrides only; they are kept in a hash map so
// that the enqueue path does not repeat the search (and the longest-first dealing, which takes
// a good fraction of a millisecond) on every call.
struct PlanKey {
    int v[18];
    bool operator==(const PlanKey &o) const { return memcmp(v, o.v, sizeof v) == 0; }
};
struct PlanKeyHash {
    size_t operator()(const PlanKey &k) const
    {
        unsigned h = 2166136261u;
        for (int i = 0; i < 18; ++i) h = (h ^ (unsigned)k.v[i]) * 16777619u;
        return h;
    }
};
constexpr size_t kMaxCachedPlans = 4096;   // the map is emptied when it grows past this
std::mutex g_planMutex;
std::unordered_map<PlanKey, Plan, PlanKeyHash> *g_planMap = nullptr;   // allocated on first use, never freed

int make_plan(int op, const Shape &s, Plan *pl)
{
    if (op != MI355CONV_OP_FWD && op != MI355CONV_OP_BWD_DATA && op != MI355CONV_OP_BWD_WEIGHT)
        return MI355CONV_ERR_UNSUPPORTED;
    PlanKey k;
    const int vals[18] = {op, s.N, s.IH, s.IW, s.IC, s.OC, s.FH, s.FW, s.sh, s.sw, s.ph, s.pw,
                          g_forceVariant.load(), g_forceSplit.load(), g_forceBM.load(), g_forceBN.load(),
                          g_forcePosMajor.load(), g_regionalOrder.load()};
    memcpy(k.v, vals, sizeof vals);
    {
        std::lock_guard<std::mutex> lock(g_planMutex);
        if (g_planMap) {
            auto it = g_planMap->find(k);
            if (it != g_planMap->end()) {
                *pl = it->second;
                return MI355CONV_OK;
            }
        }
    }
    switch (op) {
    case MI355CONV_OP_FWD:
        *pl = plan_fwd(s);
        if (pl->variant == MI355CONV_VARIANT_MFMA) plan_order_gather(s, *pl, false);
        break;
    case MI355CONV_OP_BWD_DATA:
        *pl = plan_bwd_data(s);
        if (pl->variant == MI355CONV_VARIANT_MFMA) plan_order_gather(s, *pl, true);
        break;
    default:
        *pl = plan_bwd_weight(s);
        if (pl->variant == MI355CONV_VARIANT_MFMA) plan_balance_wgrad(s, *pl);
        break;
    }
    if (!plan_launchable(op, s, *pl)) return MI355CONV_ERR_UNSUPPORTED;
    {
        std::lock_guard<std::mutex> lock(g_planMutex);
        if (!g_planMap) g_planMap = new std::unordered_map<PlanKey, Plan, PlanKeyHash>();
        if (g_planMap->size() >= kMaxCachedPlans) g_planMap->clear();
        (*g_planMap)[k] = *pl;
    }
    return MI355CONV_OK;
}

struct Epilogue {
    bool on = false;
    const float *bias = nullptr;
    float slope = 1.f;
};

// Everything in the kernel arguments of a gather-operator launch that follows from the shape and the
// plan (no pointers, no epilogue): also what conv2d_query_tile decodes workgroup ids with.
void fill_gather_geometry(GatherGemmParams &g, const Shape &s, const Plan &pl, bool bwd)
{
    memset(&g, 0, sizeof g);
    g.Nimg = s.N;
    if (bwd) {
        g.SH = s.OH; g.SW = s.OW; g.SC = s.OC;
        g.DH = s.IH; g.DW = s.IW; g.DC = s.IC;
    } else {
        g.SH = s.IH; g.SW = s.IW; g.SC = s.IC;
        g.DH = s.OH; g.DW = s.OW; g.DC = s.OC;
    }
    g.FH = s.FH; g.FW = s.FW;
    g.sh = s.sh; g.sw = s.sw; g.ph = s.ph; g.pw = s.pw;
    g.divN = make_fastdiv((unsigned)s.N);
    g.divChunksPerTap = make_fastdiv((unsigned)ceil_div(g.SC, kBK));
    g.divDHW = make_fastdiv((unsigned)(g.DH * g.DW));
    g.divDW = make_fastdiv((unsigned)g.DW);
    g.aBytes = (unsigned)((long long)g.Nimg * g.SH * g.SW * g.SC * 4);
    g.bBytes = (unsigned)((long long)s.OC * s.FH * s.FW * s.IC * 4);
    fill_gather_params(g, pl);
    g.balance = pl.balance;
    g.rowTilesPerPos = 1;
    if (pl.balance) {
        g.rowTilesPerPos = s.N / pl.bm;
        g.runs.n = g.runsN = pl.runs.n;
        for (int i = 0; i < pl.runs.n; ++i) {
            g.runs.idStart[i] = pl.runs.idStart[i];
            g.runs.rankStart[i] = pl.runs.rankStart[i];
        }
        memcpy(g.posOrder, pl.order, sizeof g.posOrder);
        g.classes.n = g.classesN = pl.nClasses;
        for (int c = 0; c < pl.nClasses; ++c) {
            g.classes.rankStart[c] = pl.classFirstUnit[c] * pl.itemsPerClassUnit;
            g.classes.firstUnit[c] = pl.classFirstUnit[c];
            g.classes.divRows[c] = make_fastdiv((unsigned)(pl.classUnits[c] * g.rowTilesPerPos));
        }
    }
    g.chunksPerSlice = pl.chunksPerSlice;
    if (pl.regional) {
        g.regional = 1;
        g.rowTilesPerPos = s.N / pl.bm;
        g.regSnake = pl.regSnake;
        g.regLocal = pl.grid / 8;
        g.regPerPos = pl.regPerPos;
        g.regCsPer = pl.regCsPer;
        g.regRowTiles = pl.regRowTiles;
        g.regW = pl.regW;
        g.regLutLo = (unsigned)pl.regLut[0] | ((unsigned)pl.regLut[1] << 8) | ((unsigned)pl.regLut[2] << 16) | ((unsigned)pl.regLut[3] << 24);
        g.regLutHi = (unsigned)pl.regLut[4] | ((unsigned)pl.regLut[5] << 8) | ((unsigned)pl.regLut[6] << 16) | ((unsigned)pl.regLut[7] << 24);
        g.divRegPerPos = make_fastdiv((unsigned)pl.regPerPos);
        g.divRegCsPer = make_fastdiv((unsigned)pl.regCsPer);
        g.divRegW = make_fastdiv((unsigned)pl.regW);
        memcpy(g.posOrder, pl.order, sizeof g.posOrder);
    }
    g.divRowTilesPerPos = make_fastdiv((unsigned)g.rowTilesPerPos);
}

// The shape- and plan-dependent part of the backward-weight kernel arguments (no pointers).
void fill_wgrad_geometry(WgradParams &w, const Shape &s, const Plan &pl)
{
    memset(&w, 0, sizeof w);
    w.N = s.N; w.IH = s.IH; w.IW = s.IW; w.IC = s.IC; w.OC = s.OC; w.OH = s.OH; w.OW = s.OW;
    w.FH = s.FH; w.FW = s.FW; w.sh = s.sh; w.sw = s.sw; w.ph = s.ph; w.pw = s.pw;
    w.posMajor = pl.posMajor;
    w.split = pl.split;
    w.sliceStride = pl.sliceStride;
    w.tilesN = pl.tilesN;
    w.xcdUnit = pl.tilesN;   // the column tiles of one slice read the same G and X rows
    w.M = s.N * s.OH * s.OW;
    w.flushChunks = pl.flushChunks;
    w.xBytes = (unsigned)((long long)s.N * s.IH * s.IW * s.IC * 4);
    w.gBytes = (unsigned)((long long)w.M * s.OC * 4);
    w.divOHOW = make_fastdiv((unsigned)(s.OH * s.OW));
    w.divOW = make_fastdiv((unsigned)s.OW);
    w.divN = make_fastdiv((unsigned)s.N);
    w.divIC = make_fastdiv((unsigned)s.IC);
    w.divFW = make_fastdiv((unsigned)s.FW);
    w.divTilesN = make_fastdiv((unsigned)pl.tilesN);
    w.divSplit = make_fastdiv((unsigned)pl.split);
    w.balance = pl.balance;
    w.tilesM = pl.tilesM;
    w.grid = pl.grid;
    w.divXcdUnit = make_fastdiv((unsigned)w.xcdUnit);
    w.xcdWhole = (pl.grid / (8 * w.xcdUnit)) * (8 * w.xcdUnit);
    w.divTilesPerTap = w.divPerTap = make_fastdiv(1u);
    for (int i = 0; i < kMaxBalanceRuns; ++i) w.runs.idStart[i] = 0x7fffffff;   // unused run entries never match
    if (pl.balance) {
        w.tilesPerTap = s.IC / pl.bn;
        w.divTilesPerTap = make_fastdiv((unsigned)w.tilesPerTap);
        w.divPerTap = make_fastdiv((unsigned)(w.tilesPerTap * pl.tilesM * pl.split));
        if (pl.regional) {
            w.regional = 1;
            w.regShift = pl.regShiftA | (pl.regShiftB << 8);
            w.regOcTiles = pl.regOcTiles;
            w.divRegIc = make_fastdiv((unsigned)pl.regIcTiles);
            w.divRegSplit = make_fastdiv((unsigned)pl.regSlices);
            w.divPerTap = make_fastdiv((unsigned)pl.itemsPerClassUnit);
        }
        w.runs.n = w.runsN = pl.runs.n;
        for (int i = 0; i < pl.runs.n; ++i) {
            w.runs.idStart[i] = pl.runs.idStart[i];
            w.runs.rankStart[i] = pl.runs.rankStart[i];
        }
        static_assert(sizeof pl.order >= kMaxBalancedTaps && sizeof w.tapOrder >= kMaxBalancedTaps, "tap order fits");
        memcpy(w.tapOrder, pl.order, kMaxBalancedTaps);
    }
}

int run_gather(const float *A, const float *B, float *out, const Shape &s, const Plan &pl, bool bwd,
               void *ws, hipStream_t st, const Epilogue &epi = Epilogue())
{
    GatherGemmParams g;
    fill_gather_geometry(g, s, pl, bwd);
    g.A = A;
    g.B = B;
    g.C = pl.split > 1 ? static_cast<float *>(ws) : out;
    g.epilogue = epi.on ? 1 : 0;
    g.bias = epi.bias;
    g.slope = epi.slope;
    hipError_t e = pl.elem ? launch_gather_elem(g, bwd, pl.bm, pl.bn, pl.grid, st)
                           : launch_gather_gemm(g, bwd, pl.bm, pl.bn, pl.grid, st);
    if (e != hipSuccess) return hip_fail(e);
    if (pl.split > 1) {
        e = launch_slice_reduce(static_cast<const float *>(ws), out, pl.outElems, pl.split, pl.sliceStride, st,
                                epi.bias, epi.slope, epi.on ? g.DC : 0);
        if (e != hipSuccess) return hip_fail(e);
    }
    return MI355CONV_OK;
}

}  // namespace

extern "C" {

size_t conv2d_workspace_bytes(int op, const conv2d_desc *d)
{
    Shape s;
    Plan pl;
    if (check_desc(d, &s) != MI355CONV_OK || make_plan(op, s, &pl) != MI355CONV_OK) return 0;
    return pl.wsBytes;
}

int conv2d_query_plan(int op, const conv2d_desc *d, conv2d_plan_info *info)
{
    if (!info) return MI355CONV_ERR_NULL_PTR;
    Shape s;
    Plan pl;
    int rc = check_desc(d, &s);
    if (rc != MI355CONV_OK) return rc;
    rc = make_plan(op, s, &pl);
    if (rc != MI355CONV_OK) return rc;
    info->variant = pl.variant;
    info->tile_m = pl.bm;
    info->tile_n = pl.bn;
    info->split = pl.split;
    info->pos_major = pl.posMajor;
    info->grid = pl.grid;
    info->workspace_bytes = pl.wsBytes;
    if (pl.variant == MI355CONV_VARIANT_DIRECT) info->kernel = MI355CONV_KERNEL_DIRECT;
    else if (pl.smallIc) info->kernel = MI355CONV_KERNEL_FIRST_LAYER;
    else if (op == MI355CONV_OP_BWD_WEIGHT) info->kernel = pl.fast ? MI355CONV_KERNEL_WGRAD_FAST : MI355CONV_KERNEL_WGRAD;
    else info->kernel = pl.elem ? MI355CONV_KERNEL_GATHER_ELEM : MI355CONV_KERNEL_GATHER;
    info->order = pl.regional ? MI355CONV_ORDER_REGIONS : pl.balance ? MI355CONV_ORDER_LONGEST : MI355CONV_ORDER_PLAIN;
    return MI355CONV_OK;
}

int conv2d_query_workgroup(int op, const conv2d_desc *d, int workgroup, int *rank, int *work)
{
    if (!rank || !work) return MI355CONV_ERR_NULL_PTR;
    Shape s;
    Plan pl;
    int rc = check_desc(d, &s);
    if (rc != MI355CONV_OK) return rc;
    rc = make_plan(op, s, &pl);
    if (rc != MI355CONV_OK) return rc;
    if (workgroup < 0 || workgroup >= pl.grid) return MI355CONV_ERR_BAD_DIM;
    *rank = workgroup;
    *work = 1;
    if (pl.regional && op == MI355CONV_OP_BWD_WEIGHT) {   // group-wise: dealing inside the XCD through the run table
        const int q = workgroup >> 3;
        int lr = q;
        if (pl.runs.n) {
            int r = 0;
            for (int i = 1; i < pl.runs.n; ++i)
                if (q >= pl.runs.idStart[i]) r = i;
            lr = pl.runs.rankStart[r] + (q - pl.runs.idStart[r]);
        }
        *rank = lr * 8 + (workgroup & 7);
        *work = pl.unitWork[lr / pl.itemsPerClassUnit];
        return MI355CONV_OK;
    }
    if (pl.regional) {   // the kernels' region-wise decode: XCD = id % 8, place on the XCD = id / 8
        const int q = workgroup >> 3, local = pl.grid / 8;
        int lr = q;
        if (pl.regSnake) {
            const int lap = q >> 5, left = local - (lap << 5), w = left < 32 ? left : 32;
            int c = q & 31;
            if (lap & 1) c = w - 1 - c;
            lr = (lap << 5) + c;
        }
        *rank = lr * 8 + (workgroup & 7);
        *work = pl.unitWork[lr / pl.regPerPos];
        return MI355CONV_OK;
    }
    if (!pl.balance) return MI355CONV_OK;
    if (pl.runs.n) {   // the same lookup as the kernels' balanced_rank()
        const int slot = balance_slot(workgroup, pl.grid);
        int r = 0;
        for (int i = 1; i < pl.runs.n; ++i)
            if (slot >= pl.runs.idStart[i]) r = i;
        *rank = pl.runs.rankStart[r] + (slot - pl.runs.idStart[r]);
    }
    *work = pl.unitWork[*rank / pl.itemsPerClassUnit];
    return MI355CONV_OK;
}

int conv2d_query_tile(int op, const conv2d_desc *d, int workgroup, int *row_tile, int *col_tile, int *slice)
{
    if (!row_tile || !col_tile || !slice) return MI355CONV_ERR_NULL_PTR;
    Shape s;
    Plan pl;
    int rc = check_desc(d, &s);
    if (rc != MI355CONV_OK) return rc;
    rc = make_plan(op, s, &pl);
    if (rc != MI355CONV_OK) return rc;
    if (workgroup < 0 || workgroup >= pl.grid) return MI355CONV_ERR_BAD_DIM;
    if (!pl.regional) return MI355CONV_ERR_UNSUPPORTED;
    // the kernels' own decode functions, fed with the same argument block the launch would get
    if (op == MI355CONV_OP_BWD_WEIGHT) {
        static thread_local WgradParams w;
        fill_wgrad_geometry(w, s, pl);
        const int q = workgroup >> 3;
        int lr = q;
        if (w.runsN) {
            int r = 0;
            for (int i = 1; i < kMaxBalanceRuns; ++i)
                if (q >= w.runs.idStart[i]) r = i;
            lr = w.runs.rankStart[r] + (q - w.runs.idStart[r]);
        }
        int tapRank, icTile;
        group_wise_tile(w, workgroup & 7, lr, &tapRank, &icTile, row_tile, slice);
        *col_tile = w.tapOrder[tapRank] * w.tilesPerTap + icTile;
        return MI355CONV_OK;
    }
    static thread_local GatherGemmParams g;
    fill_gather_geometry(g, s, pl, op == MI355CONV_OP_BWD_DATA);
    int xcd, posRank, inner;
    region_wise_place(g, workgroup, &xcd, &posRank, &inner);
    region_wise_tile(g, xcd, g.posOrder[posRank], inner, row_tile, col_tile, slice);
    return MI355CONV_OK;
}

int conv2d_set_tuning(int variant, int split)
{
    if (variant < MI355CONV_VARIANT_AUTO || variant > MI355CONV_VARIANT_MFMA || split < 0)
        return MI355CONV_ERR_UNSUPPORTED;
    g_forceVariant.store(variant);
    g_forceSplit.store(split);
    return MI355CONV_OK;
}

int conv2d_set_tile(int tile_m, int tile_n, int pos_major)
{
    if (tile_m < 0 || tile_n < 0 || pos_major < -1 || pos_major > 1 || (tile_m == 0) != (tile_n == 0))
        return MI355CONV_ERR_UNSUPPORTED;
    if (tile_m && !tile_compiled(tile_m, tile_n, true) && !tile_compiled(tile_m, tile_n, false))
        return MI355CONV_ERR_UNSUPPORTED;
    g_forceBM.store(tile_m);
    g_forceBN.store(tile_n);
    g_forcePosMajor.store(pos_major);
    return MI355CONV_OK;
}



int conv2d_set_order(int region_wise)
{
    if (region_wise < 0 || region_wise > 1) return MI355CONV_ERR_UNSUPPORTED;
    g_regionalOrder.store(region_wise);
    return MI355CONV_OK;
}

static int fwd_impl(const float *X, const float *W, float *Y, const conv2d_desc *d, void *ws, size_t ws_bytes,
                    void *stream, const Epilogue &epi, const unsigned char *X8 = nullptr, float scale = 1.f)
{
    Shape s;
    Plan pl;
    int rc = check_desc(d, &s);
    if (rc != MI355CONV_OK) return rc;
    rc = make_plan(MI355CONV_OP_FWD, s, &pl);
    if (rc != MI355CONV_OK) return rc;
    if (X8) {   // bytes: only the first-layer kernel converts on load
        if (!W || !Y) return MI355CONV_ERR_NULL_PTR;
        if ((reinterpret_cast<uintptr_t>(W) | reinterpret_cast<uintptr_t>(Y)) & 15u) return MI355CONV_ERR_ALIGNMENT;
        if (!pl.smallIc) return MI355CONV_ERR_UNSUPPORTED;
    } else {
        rc = check_buffers(X, W, Y, pl, ws, ws_bytes);
        if (rc != MI355CONV_OK) return rc;
    }
    rc = prepare_device(nullptr);
    if (rc != MI355CONV_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (pl.variant == MI355CONV_VARIANT_DIRECT) {
        hipError_t e = launch_direct_fwd(X, W, Y, s, st);
        if (e == hipSuccess && epi.on)
            e = launch_bias_act(Y, (long long)s.N * s.OH * s.OW * s.OC, epi.bias, epi.slope, s.OC, st);
        return e == hipSuccess ? MI355CONV_OK : hip_fail(e);
    }
    if (pl.smallIc) {
        SmallIcParams q;
        memset(&q, 0, sizeof q);
        q.X = X8 ? reinterpret_cast<const float *>(X8) : X;
        q.W = W; q.dX = Y;
        q.u8 = X8 ? 1 : 0;
        q.scale = scale;
        q.xBytes = (unsigned)((long long)s.N * s.IH * s.IW * s.IC * (X8 ? 1 : 4));
        q.wBytes = (unsigned)((long long)s.OC * s.FH * s.FW * s.IC * 4);
        q.N = s.N; q.IH = s.IH; q.IW = s.IW; q.IC = s.IC; q.OC = s.OC; q.OH = s.OH; q.OW = s.OW;
        q.FH = s.FH; q.FW = s.FW; q.ph = s.ph; q.pw = s.pw; q.sh = s.sh; q.sw = s.sw;
        q.M = s.N * s.OH * s.OW;
        q.divOHOW = make_fastdiv((unsigned)(s.OH * s.OW));
        q.divOW = make_fastdiv((unsigned)s.OW);
        q.divIC = make_fastdiv((unsigned)s.IC);
        q.divFW = make_fastdiv((unsigned)s.FW);
        q.epilogue = epi.on ? 1 : 0;
        q.bias = epi.bias;
        q.slope = epi.slope;
        hipError_t e = launch_fwd_small_ic(q, st);
        return e == hipSuccess ? MI355CONV_OK : hip_fail(e);
    }
    return run_gather(X, W, Y, s, pl, false, ws, st, epi);
}

int conv2d_fwd(const float *X, const float *W, float *Y, const conv2d_desc *d, void *ws, size_t ws_bytes,
               void *stream)
{
    return fwd_impl(X, W, Y, d, ws, ws_bytes, stream, Epilogue());
}

int conv2d_fwd_u8(const unsigned char *X8, float scale, const float *W, float *Y, const conv2d_desc *d, void *stream)
{
    if (!X8) return MI355CONV_ERR_NULL_PTR;
    if (!(scale == scale)) return MI355CONV_ERR_UNSUPPORTED;   // NaN
    return fwd_impl(nullptr, W, Y, d, nullptr, 0, stream, Epilogue(), X8, scale);
}

int conv2d_fwd_bias_act(const float *X, const float *W, const float *bias, float *Y, const conv2d_desc *d,
                        float negative_slope, void *ws, size_t ws_bytes, void *stream)
{
    if (bias && (reinterpret_cast<uintptr_t>(bias) & 3u)) return MI355CONV_ERR_ALIGNMENT;
    if (!(negative_slope == negative_slope)) return MI355CONV_ERR_UNSUPPORTED;   // NaN
    Epilogue epi;
    epi.on = true;
    epi.bias = bias;
    epi.slope = negative_slope;
    return fwd_impl(X, W, Y, d, ws, ws_bytes, stream, epi);
}

int conv2d_bwd_data(const float *dY, const float *W, float *dX, const conv2d_desc *d, void *ws,
                    size_t ws_bytes, void *stream)
{
    Shape s;
    Plan pl;
    int rc = check_desc(d, &s);
    if (rc != MI355CONV_OK) return rc;
    rc = make_plan(MI355CONV_OP_BWD_DATA, s, &pl);
    if (rc != MI355CONV_OK) return rc;
    rc = check_buffers(dY, W, dX, pl, ws, ws_bytes);
    if (rc != MI355CONV_OK) return rc;
    rc = prepare_device(nullptr);
    if (rc != MI355CONV_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (pl.variant == MI355CONV_VARIANT_DIRECT) {
        hipError_t e = launch_direct_bwd_data(dY, W, dX, s, st);
        return e == hipSuccess ? MI355CONV_OK : hip_fail(e);
    }
    if (pl.smallIc) {
        SmallIcParams q;
        memset(&q, 0, sizeof q);
        q.G = dY; q.W = W; q.dX = dX;
        q.gBytes = (unsigned)((long long)s.N * s.OH * s.OW * s.OC * 4);
        q.wBytes = (unsigned)((long long)s.OC * s.FH * s.FW * s.IC * 4);
        q.N = s.N; q.IH = s.IH; q.IW = s.IW; q.IC = s.IC; q.OC = s.OC; q.OH = s.OH; q.OW = s.OW;
        q.FH = s.FH; q.FW = s.FW; q.ph = s.ph; q.pw = s.pw;
        hipError_t e = launch_bwd_data_small_ic(q, st);
        return e == hipSuccess ? MI355CONV_OK : hip_fail(e);
    }
    return run_gather(dY, W, dX, s, pl, true, ws, st);
}

int deconv2d(const float *dY, const float *W, float *dX, const conv2d_desc *d, void *ws, size_t ws_bytes,
             void *stream)
{
    return conv2d_bwd_data(dY, W, dX, d, ws, ws_bytes, stream);
}

// ownWorkspace: the slice partials go to the library's per-device scratch array instead of a
// caller workspace (conv2d_bwd_weight_noalloc)
static int bwd_weight_impl(const float *X, const float *dY, float *dW, const conv2d_desc *d, void *ws,
                           size_t ws_bytes, void *stream, bool ownWorkspace)
{
    Shape s;
    Plan pl;
    int rc = check_desc(d, &s);
    if (rc != MI355CONV_OK) return rc;
    rc = make_plan(MI355CONV_OP_BWD_WEIGHT, s, &pl);
    if (rc != MI355CONV_OK) return rc;
    if (ownWorkspace) {
        if (pl.wsBytes > kScratchBytes) return MI355CONV_ERR_WORKSPACE;   // before any HIP call
        if (!X || !dY || !dW) return MI355CONV_ERR_NULL_PTR;
        if (!aligned16(X) || !aligned16(dY) || !aligned16(dW)) return MI355CONV_ERR_ALIGNMENT;
    } else {
        rc = check_buffers(X, dY, dW, pl, ws, ws_bytes);
        if (rc != MI355CONV_OK) return rc;
    }
    int dev = 0;
    rc = prepare_device(&dev);
    if (rc != MI355CONV_OK) return rc;
    if (ownWorkspace) ws = g_scratchPtr[dev];   // the device's copy of `scratch`, never the array's name
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (pl.variant == MI355CONV_VARIANT_DIRECT) {
        hipError_t e = launch_direct_bwd_weight(X, dY, dW, s, st);
        return e == hipSuccess ? MI355CONV_OK : hip_fail(e);
    }
    if (pl.smallIc) {
        SmallIcParams q;
        memset(&q, 0, sizeof q);
        q.G = dY; q.X = X;
        q.C = pl.split > 1 ? static_cast<float *>(ws) : dW;
        q.gBytes = (unsigned)((long long)s.N * s.OH * s.OW * s.OC * 4);
        q.xBytes = (unsigned)((long long)s.N * s.IH * s.IW * s.IC * 4);
        q.N = s.N; q.IH = s.IH; q.IW = s.IW; q.IC = s.IC; q.OC = s.OC; q.OH = s.OH; q.OW = s.OW;
        q.FH = s.FH; q.FW = s.FW; q.ph = s.ph; q.pw = s.pw; q.sh = s.sh; q.sw = s.sw;
        q.split = pl.split;
        q.M = s.N * s.OH * s.OW;
        q.sliceStride = pl.sliceStride;
        q.divOHOW = make_fastdiv((unsigned)(s.OH * s.OW));
        q.divOW = make_fastdiv((unsigned)s.OW);
        q.divIC = make_fastdiv((unsigned)s.IC);
        q.divFW = make_fastdiv((unsigned)s.FW);
        hipError_t e = launch_wgrad_small_ic(q, st);
        if (e != hipSuccess) return hip_fail(e);
        if (pl.split > 1) {
            e = launch_slice_reduce(static_cast<const float *>(ws), dW, pl.outElems, pl.split, pl.sliceStride, st);
            if (e != hipSuccess) return hip_fail(e);
        }
        return MI355CONV_OK;
    }
    WgradParams w;
    fill_wgrad_geometry(w, s, pl);
    w.X = X;
    w.G = dY;
    w.C = pl.split > 1 ? static_cast<float *>(ws) : dW;
    hipError_t e = pl.fast ? launch_wgrad_fast(w, pl.bm, pl.bn, pl.grid, st)
                           : launch_wgrad(w, pl.bm, pl.bn, pl.elem != 0, pl.grid, st);
    if (e != hipSuccess) return hip_fail(e);
    if (pl.split > 1) {
        e = launch_slice_reduce(static_cast<const float *>(ws), dW, pl.outElems, pl.split, pl.sliceStride, st);
        if (e != hipSuccess) return hip_fail(e);
    }
    return MI355CONV_OK;
}

int conv2d_bwd_weight(const float *X, const float *dY, float *dW, const conv2d_desc *d, void *ws,
                      size_t ws_bytes, void *stream)
{
    return bwd_weight_impl(X, dY, dW, d, ws, ws_bytes, stream, false);
}

int conv2d_bwd_weight_noalloc(const float *X, const float *dY, float *dW, const conv2d_desc *d, void *stream)
{
    return bwd_weight_impl(X, dY, dW, d, nullptr, 0, stream, true);
}

size_t conv2d_noalloc_scratch_bytes(void) { return kScratchBytes; }

int conv2d_init(void) { return prepare_device(nullptr); }

// The matrix multiplies of a fully-connected layer as the 1x1 operators on a 1x1 map: the rows of the
// left matrix are the "images".
static int matmul_desc(int kind, int M, int N, int K, conv2d_desc *d, int *op)
{
    if (M <= 0 || N <= 0 || K <= 0) return MI355CONV_ERR_BAD_DIM;
    conv2d_desc t = {0, 1, 1, 0, 0, 1, 1, 1, 1, 0, 0};
    switch (kind) {
    case MI355CONV_MATMUL_NT: t.N = M; t.IC = K; t.OC = N; *op = MI355CONV_OP_FWD; break;         // Y[M,N] = X[M,K] W[N,K]^T
    case MI355CONV_MATMUL_NN: t.N = M; t.IC = N; t.OC = K; *op = MI355CONV_OP_BWD_DATA; break;    // dX[M,N] = dY[M,K] W[K,N]
    case MI355CONV_MATMUL_TN: t.N = K; t.IC = N; t.OC = M; *op = MI355CONV_OP_BWD_WEIGHT; break;  // dW[M,N] = dY[K,M]^T X[K,N]
    default: return MI355CONV_ERR_UNSUPPORTED;
    }
    *d = t;
    return MI355CONV_OK;
}

size_t matmul_workspace_bytes(int kind, int M, int N, int K)
{
    conv2d_desc d;
    int op = 0;
    if (matmul_desc(kind, M, N, K, &d, &op) != MI355CONV_OK) return 0;
    return conv2d_workspace_bytes(op, &d);
}

int matmul_f32(int kind, const float *A, const float *B, float *C, int M, int N, int K, void *ws, size_t ws_bytes,
               void *stream)
{
    conv2d_desc d;
    int op = 0;
    const int rc = matmul_desc(kind, M, N, K, &d, &op);
    if (rc != MI355CONV_OK) return rc;
    if (op == MI355CONV_OP_FWD) return conv2d_fwd(A, B, C, &d, ws, ws_bytes, stream);
    if (op == MI355CONV_OP_BWD_DATA) return conv2d_bwd_data(A, B, C, &d, ws, ws_bytes, stream);
    return conv2d_bwd_weight(B, A, C, &d, ws, ws_bytes, stream);   // (X, dY, dW) = (B, A, C)
}

const char *conv2d_status_string(int status)
{
    switch (status) {
    case MI355CONV_OK: return "ok";
    case MI355CONV_ERR_NULL_PTR: return "null pointer";
    case MI355CONV_ERR_BAD_DIM: return "bad dimension";
    case MI355CONV_ERR_WORKSPACE: return "workspace missing or too small";
    case MI355CONV_ERR_ALIGNMENT: return "pointer not 16-byte aligned";
    case MI355CONV_ERR_UNSUPPORTED: return "unsupported argument";
    case MI355CONV_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
    }
}

const char *conv2d_last_hip_error(void) { return t_hipError; }

}  // extern "C"
