// Host side of the convolution entry points: validation, tile/split selection, workspace layout, launches.
#include <algorithm>

#include "conv_kernels.h"

namespace rn50 {

int conv_check(const char *who, const rn50_conv_desc *d)
{
    RN50_REQUIRE(d, RN50_EINVAL, "%s: null descriptor", who);
    RN50_REQUIRE(d->n > 0 && d->c > 0 && d->h > 0 && d->w > 0 && d->k > 0 && d->r > 0 && d->s > 0 && d->stride > 0 && d->pad >= 0,
                 RN50_EINVAL, "%s: non-positive dimension", who);
    RN50_REQUIRE(d->layout == RN50_LAYOUT_NHWC, RN50_EUNSUPPORTED, "%s: only the NHWC/KRSC layout has kernels", who);
    RN50_REQUIRE(d->in_dtype == RN50_DTYPE_F32 || d->in_dtype == RN50_DTYPE_BF16 || d->in_dtype == RN50_DTYPE_BF16_ACT ||
                     d->in_dtype == RN50_DTYPE_BF16_ACT_F32IN,
                 RN50_EUNSUPPORTED, "%s: unknown operand dtype", who);
    RN50_REQUIRE(d->h + 2 * d->pad >= d->r && d->w + 2 * d->pad >= d->s, RN50_EINVAL, "%s: filter larger than the padded input", who);
    RN50_REQUIRE(d->pad < d->r && d->pad < d->s, RN50_EUNSUPPORTED, "%s: padding must be smaller than the filter", who);
    RN50_REQUIRE((long)d->h * d->w < (1L << 24) && d->c < (1 << 24) && d->k < (1 << 24), RN50_EUNSUPPORTED,
                 "%s: H*W, C and K must be below 2^24 (24-bit multiplies in the gather)", who);
    const long P = (d->h + 2 * d->pad - d->r) / d->stride + 1, Q = (d->w + 2 * d->pad - d->s) / d->stride + 1;
    RN50_REQUIRE((long)d->n * d->h * d->w * d->c < (1L << 31) && (long)d->n * P * Q * d->k < (1L << 31) &&
                     (long)d->n * d->h * d->w < (1L << 27) && (long)d->k * d->r * d->s * d->c < (1L << 31),
                 RN50_EUNSUPPORTED, "%s: tensor too large for 32-bit indexing", who);
    return RN50_OK;
}

// Storage of the activation tensors a call reads and writes: 0 fp32, 1 bfloat16 bits, 2 bfloat16 bits except the layer
// input x, which is fp32 (the network's first layer).  Both bf16 forms multiply on the bf16 MFMA.
static int act_of(const rn50_conv_desc *d)
{
    return d->in_dtype == RN50_DTYPE_BF16_ACT ? 1 : d->in_dtype == RN50_DTYPE_BF16_ACT_F32IN ? 2 : 0;
}
static bool bf16_of(const rn50_conv_desc *d) { return d->in_dtype != RN50_DTYPE_F32; }
// Reduction elements per LDS stage of the implicit GEMM: 64 for bf16 operands through the vector gather when a stage of 64 stays
// inside one filter tap (cin = channels of the gathered tensor), else 32.
static int igemm_bk(bool bf16, int act, int cin) { return bf16 && act != 2 && cin % (2 * kBK) == 0 ? 2 * kBK : kBK; }

struct Geom { int P, Q; long Mout, Min; int Kdim; };
static Geom geom(const rn50_conv_desc *d)
{
    Geom g;
    g.P = (d->h + 2 * d->pad - d->r) / d->stride + 1;
    g.Q = (d->w + 2 * d->pad - d->s) / d->stride + 1;
    g.Mout = (long)d->n * g.P * g.Q;
    g.Min = (long)d->n * d->h * d->w;
    g.Kdim = d->r * d->s * d->c;
    return g;
}

// ---- tile and split selection ------------------------------------------------------------------------
constexpr double kCUs = 256.0;
constexpr double kBytesPerClk = 8e12 / 2.4e9;  // HBM bytes per core clock, whole chip
constexpr double kLaunchClks = 6000.0;         // one extra kernel launch, in core clocks

struct GemmPlan { int bm, bn, split, chunks_per_split; };

// Plans measured on the MI355X for the ResNet-50 layer shapes: {op, n, c, h, k, r, stride, pad, bm, bn, split}.
// Other shapes use the cost model below.
static const PlanRow kTuned[] = {
#include "conv_plans.inc"
    {-1, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}};
// The same for bf16 activations in memory, where most layers are bound by memory traffic and other tiles win; consulted first
// for that storage (shapes it does not list fall through to the table above).
static const PlanRow kTunedAct[] = {
#include "conv_plans_bf16act.inc"
    {-1, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}};

static bool plan_matches(const PlanRow &t, const rn50_conv_desc *d, int op)
{
    return t.op == op && t.n == d->n && t.c == d->c && t.h == d->h && d->w == d->h && t.k == d->k && t.r == d->r && d->s == d->r &&
           t.stride == d->stride && t.pad == d->pad;
}

// Rows set with rn50_set_option("plan_overrides") go before the table (a tuning aid: plans tried inside a whole step).
static bool tuned_plan(const Config &cfg, const rn50_conv_desc *d, int op, GemmPlan *pl)
{
    for (const PlanRow &t : cfg.overrides)
        if (plan_matches(t, d, op)) {
            pl->bm = t.bm; pl->bn = t.bn; pl->split = t.split;
            return true;
        }
    if (cfg.no_tuned) return false;
    if (act_of(d))
        for (const PlanRow &t : kTunedAct)
            if (plan_matches(t, d, op)) {
                pl->bm = t.bm; pl->bn = t.bn; pl->split = t.split;
                return true;
            }
    for (const PlanRow &t : kTuned)
        if (plan_matches(t, d, op)) {
            pl->bm = t.bm; pl->bn = t.bn; pl->split = t.split;
            return true;
        }
    return false;
}

static bool forced_plan(bool has, const int v[3], GemmPlan *pl)
{
    if (!has) return false;
    pl->bm = v[0]; pl->bn = v[1]; pl->split = v[2];
    return true;
}

static double tile_eff(int bm, int bn) { return bm == 128 && bn == 128 ? 1.0 : (bm == 64 && bn == 64 ? 0.72 : 0.86); }

// Persistent implicit-GEMM launch: G workgroups; the first full_items tiles whole, the last tail_tiles tiles cut
// into tail_split pieces of tail_chunks reduction chunks each.
struct IgemmPlan { int bm, bn, grid, full_items, tail_tiles, tail_split, tail_chunks; size_t ws_floats; };


static IgemmPlan make_igemm_plan(int bm, int bn, long M, int Nout, int kchunks, int want_split, bool allow_split)
{
    IgemmPlan pl;
    pl.bm = bm; pl.bn = bn;
    const int tiles = ceil_div(M, bm) * ceil_div(Nout, bn);
    const int Gmax = (int)kCUs * igemm_occupancy(bm, bn);
    pl.full_items = tiles / Gmax * Gmax;
    pl.tail_tiles = tiles - pl.full_items;
    int sp = allow_split ? want_split : 1;
    if (sp > kchunks) sp = kchunks;
    if (sp < 1) sp = 1;
    pl.tail_chunks = ceil_div(kchunks, sp);
    pl.tail_split = pl.tail_tiles ? ceil_div(kchunks, pl.tail_chunks) : 1;
    const int items = pl.full_items + pl.tail_tiles * pl.tail_split;
    pl.grid = pl.full_items ? Gmax : std::min(Gmax, (items + 7) / 8 * 8);
    pl.ws_floats = pl.tail_split > 1 ? (size_t)pl.tail_tiles * pl.tail_split * bm * bn : 0;
    return pl;
}

// modelled time in core clocks
static double igemm_cost(const IgemmPlan &pl, long M, int Nout, int kchunks, int bk)
{
    const double chunk_clks = 4096.0 * (bk / (double)kBK) * (pl.bm * pl.bn / 16384.0) / tile_eff(pl.bm, pl.bn);
    const int occ = igemm_occupancy(pl.bm, pl.bn);
    const double full_rounds = pl.full_items / (kCUs * occ);
    double t = full_rounds * occ * (kchunks + 2.0) * chunk_clks;
    if (pl.tail_tiles) {
        const double pieces = (double)pl.tail_tiles * pl.tail_split;
        const double per_cu = ceil(pieces / kCUs);
        t += per_cu * (pl.tail_chunks + 3.0) * chunk_clks / (per_cu >= 2.0 ? 1.0 : 0.65);
        if (pl.tail_split > 1) t += kLaunchClks + (pl.tail_split + 1.0) * pl.tail_tiles * pl.bm * pl.bn * 4.0 / kBytesPerClk;
    }
    (void)M; (void)Nout;
    return t;
}

// out[M][Nout] with reduction length Kdim (in elements)
// cin: channels of the gathered tensor (the forward pass gathers x, the data gradient dy)
static IgemmPlan plan_igemm(const rn50_conv_desc *d, int op, long M, int Nout, int Kdim, bool allow_split, int cin)
{
    const int bk = igemm_bk(bf16_of(d), act_of(d), cin);
    const int kchunks = ceil_div(Kdim, bk);
    GemmPlan forced;
    const std::shared_ptr<const Config> cfg = config();
    if (forced_plan(cfg->has_igemm_plan, cfg->igemm_plan, &forced) || tuned_plan(*cfg, d, op, &forced))
        return make_igemm_plan(forced.bm, forced.bn, M, Nout, kchunks, forced.split, allow_split);
    IgemmPlan best{};
    double best_cost = 1e300;
    static const int splits[] = {1, 2, 3, 4, 6, 8, 12, 16, 24, 32};
    for (int bm = 128; bm >= 64; bm -= 64)
        for (int bn = 128; bn >= 64; bn -= 64) {
            if (bn == 128 && Nout <= 64) continue;
            if (bm == 128 && M <= 64) continue;
            for (int sp : splits) {
                if (sp > 1 && (!allow_split || kchunks / sp < 2)) break;
                const IgemmPlan pl = make_igemm_plan(bm, bn, M, Nout, kchunks, sp, allow_split);
                const double cost = igemm_cost(pl, M, Nout, kchunks, bk);
                if (cost < best_cost) { best_cost = cost; best = pl; }
            }
        }
    return best;
}

// The filter-gradient kernels take two stages per trip of their loop: a range of an odd number of stages ends with a stage of
// zeros, so ranges are cut at even counts where there is more than one range.
static int even_stages(int cps, int pchunks) { return cps < pchunks ? cps + (cps & 1) : cps; }

// dw[Kout][Jdim] with the reduction over Mpix pixels, split into `split` ranges of chunks_per_split stages
static GemmPlan plan_wgrad_any_tile(const rn50_conv_desc *d, int Kout, int Jdim, long Mpix);

static GemmPlan plan_wgrad(const rn50_conv_desc *d, int Kout, int Jdim, long Mpix)
{
    GemmPlan pl = plan_wgrad_any_tile(d, Kout, Jdim, Mpix);
    if (act_of(d) && (pl.bm != 64 || pl.bn != 64)) {
        // the bf16-activation kernel has 64x64 tiles only: as many workgroups as the chosen plan by a matching split
        const int pchunks = ceil_div(Mpix, kBK);
        const long wgs = (long)ceil_div(Kout, pl.bm) * ceil_div(Jdim, pl.bn) * pl.split;
        int split = std::max(1, (int)(wgs / ((long)ceil_div(Kout, 64) * ceil_div(Jdim, 64))));
        if (split > pchunks) split = pchunks;
        pl.bm = pl.bn = 64;
        pl.chunks_per_split = even_stages(ceil_div(pchunks, split), pchunks);
        pl.split = ceil_div(pchunks, pl.chunks_per_split);
    }
    return pl;
}

static GemmPlan plan_wgrad_any_tile(const rn50_conv_desc *d, int Kout, int Jdim, long Mpix)
{
    const int pchunks = ceil_div(Mpix, kBK);
    GemmPlan best{64, 64, 1, pchunks};
    GemmPlan forced;
    const std::shared_ptr<const Config> cfg = config();
    if (forced_plan(cfg->has_wgrad_plan, cfg->wgrad_plan, &forced) || tuned_plan(*cfg, d, RN50_OP_BWD_WEIGHT, &forced)) {
        if (forced.split > pchunks) forced.split = pchunks;
        forced.chunks_per_split = even_stages(ceil_div(pchunks, forced.split), pchunks);
        forced.split = ceil_div(pchunks, forced.chunks_per_split);
        return forced;
    }
    double best_cost = 1e300;
    for (int bm = 128; bm >= 64; bm -= 64)
        for (int bn = 128; bn >= 64; bn -= 64) {
            if (bm == 128 && Kout <= 64) continue;
            if (bn == 128 && Jdim <= 64) continue;
            const double tiles = (double)ceil_div(Kout, bm) * ceil_div(Jdim, bn);
            const int occ = wgrad_occupancy(bm, bn);
            const double chunk_clks = 4096.0 * (bm * bn / 16384.0);
            for (int s = 1; s <= 2048; s = (s < 8 ? s + 1 : s + s / 4)) {
                if (s > 1 && pchunks / s < 2) break;
                const int cps = even_stages(ceil_div(pchunks, s), pchunks);
                const int sp = ceil_div(pchunks, cps);
                const double wgs = tiles * sp;
                const double per_cu = ceil(wgs / kCUs);            // workgroups the busiest CU runs
                const double conc = std::min((double)occ, per_cu);  // of which this many at a time
                // a stage costs its MFMA time, but no less than what the load latency allows at this concurrency
                const double stage = std::max(chunk_clks, 3000.0 / conc);
                const double cost = per_cu * (cps + 3.0) * stage + kLaunchClks + (sp + 1.0) * Kout * Jdim * 4.0 / kBytesPerClk;
                if (cost < best_cost) { best_cost = cost; best = GemmPlan{bm, bn, sp, cps}; }
            }
        }
    return best;
}

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

template <int MODE, bool BF, bool INAFF, int ACT, bool STATS, int BK>
static void launch_igemm_bk(const IgemmPlan &pl, const IgemmP &p, hipStream_t st)
{
    const dim3 grid(pl.grid), block(kConvThreads);
    if (pl.bm == 128 && pl.bn == 128) hipLaunchKernelGGL((igemm_kernel<128, 128, MODE, BF, INAFF, ACT, STATS, BK>), grid, block, 0, st, p);
    else if (pl.bm == 128) hipLaunchKernelGGL((igemm_kernel<128, 64, MODE, BF, INAFF, ACT, STATS, BK>), grid, block, 0, st, p);
    else if (pl.bn == 128) hipLaunchKernelGGL((igemm_kernel<64, 128, MODE, BF, INAFF, ACT, STATS, BK>), grid, block, 0, st, p);
    else hipLaunchKernelGGL((igemm_kernel<64, 64, MODE, BF, INAFF, ACT, STATS, BK>), grid, block, 0, st, p);
}

// p.kchunks counts stages of igemm_bk() elements: the instantiation with that stage length
template <int MODE, bool BF, bool INAFF = false, int ACT = 0, bool STATS = false>
static void launch_igemm_mode(const IgemmPlan &pl, const IgemmP &p, hipStream_t st)
{
    if constexpr (BF && MODE <= 1) {
        if (igemm_bk(true, ACT, p.Cin) == 2 * kBK) {
            launch_igemm_bk<MODE, BF, INAFF, ACT, STATS, 2 * kBK>(pl, p, st);
            return;
        }
    }
    launch_igemm_bk<MODE, BF, INAFF, ACT, STATS, kBK>(pl, p, st);
}

// The forward launches that also gather the output's statistics (p.stat_mean set): no dilation, so the vector gather
// (MODE 0) or the scalar one (MODE 2).
static void launch_igemm_stats(const IgemmPlan &pl, const IgemmP &p, bool bf16, int act, hipStream_t st)
{
    const bool fast = p.Cin % kBK == 0 && act != 2;
    if (act == 1) {
        if (p.in_scale) launch_igemm_mode<0, true, true, 1, true>(pl, p, st);
        else if (fast) launch_igemm_mode<0, true, false, 1, true>(pl, p, st);
        else launch_igemm_mode<2, true, false, 1, true>(pl, p, st);
    } else if (act == 2) {
        launch_igemm_mode<2, true, false, 2, true>(pl, p, st);
    } else if (p.in_scale) {
        if (bf16) launch_igemm_mode<0, true, true, 0, true>(pl, p, st);
        else launch_igemm_mode<0, false, true, 0, true>(pl, p, st);
    } else if (bf16) {
        if (fast) launch_igemm_mode<0, true, false, 0, true>(pl, p, st);
        else launch_igemm_mode<2, true, false, 0, true>(pl, p, st);
    } else {
        if (fast) launch_igemm_mode<0, false, false, 0, true>(pl, p, st);
        else launch_igemm_mode<2, false, false, 0, true>(pl, p, st);
    }
}

template <bool O16>
static void launch_tail_reduce(const IgemmPlan &pl, const IgemmP &p, hipStream_t st)
{
    const dim3 grid(ceil_div(pl.bm * pl.bn / 4, 256), pl.tail_tiles), block(256);
    if (pl.bm == 128 && pl.bn == 128) hipLaunchKernelGGL((igemm_tail_reduce_kernel<128, 128, O16>), grid, block, 0, st, p);
    else if (pl.bm == 128) hipLaunchKernelGGL((igemm_tail_reduce_kernel<128, 64, O16>), grid, block, 0, st, p);
    else if (pl.bn == 128) hipLaunchKernelGGL((igemm_tail_reduce_kernel<64, 128, O16>), grid, block, 0, st, p);
    else hipLaunchKernelGGL((igemm_tail_reduce_kernel<64, 64, O16>), grid, block, 0, st, p);
}

template <bool O16>
static void launch_tail_reduce_stats(const IgemmPlan &pl, const IgemmP &p, hipStream_t st)
{
    const dim3 grid(pl.bn / 32, pl.tail_tiles), block(256);
    if (pl.bm == 128 && pl.bn == 128) hipLaunchKernelGGL((igemm_tail_reduce_stats_kernel<128, 128, O16>), grid, block, 0, st, p);
    else if (pl.bm == 128) hipLaunchKernelGGL((igemm_tail_reduce_stats_kernel<128, 64, O16>), grid, block, 0, st, p);
    else if (pl.bn == 128) hipLaunchKernelGGL((igemm_tail_reduce_stats_kernel<64, 128, O16>), grid, block, 0, st, p);
    else hipLaunchKernelGGL((igemm_tail_reduce_stats_kernel<64, 64, O16>), grid, block, 0, st, p);
}

// Runs out[M][Nout] (+ optional stride-2 scatter) and, when tail tiles are split, the ordered sum of their pieces.
// act: storage of the gathered operand and of the output (see act_of)
static void run_igemm(IgemmP p, const IgemmPlan &pl, float *out, float *partials, bool bf16, int act, hipStream_t st)
{
    const bool fast = p.Cin % kBK == 0 && act != 2;  // an fp32 input beside bf16 activations goes through the scalar gather
    p.kchunks = ceil_div(p.Kdim, fast ? igemm_bk(bf16, act, p.Cin) : kBK);
    p.tiles_m = ceil_div(p.M, pl.bm);
    p.tiles_n = ceil_div(p.Nout, pl.bn);
    p.full_items = pl.full_items;
    p.tail_tiles = pl.tail_tiles;
    p.tail_split = pl.tail_split;
    p.tail_chunks = pl.tail_chunks;
    p.out = out;
    p.partial = partials;
    p.div_ohw = make_fastdiv(p.OH * p.OW);
    p.div_ow = make_fastdiv(p.OW);
    p.div_cin = make_fastdiv(p.Cin);
    p.div_s = make_fastdiv(p.S);
    if (p.stat_mean) {
        launch_igemm_stats(pl, p, bf16, act, st);  // callers have checked: a forward pass (sd == 1)
    } else if (act == 1) {
        if (p.in_scale) launch_igemm_mode<0, true, true, 1>(pl, p, st);
        else if (fast && p.sd == 1) launch_igemm_mode<0, true, false, 1>(pl, p, st);
        else if (fast) launch_igemm_mode<1, true, false, 1>(pl, p, st);
        else launch_igemm_mode<2, true, false, 1>(pl, p, st);
    } else if (act == 2) {
        launch_igemm_mode<2, true, false, 2>(pl, p, st);
    } else if (p.in_scale) {  // callers have checked: Cin % 32 == 0 and no dilation
        if (bf16) launch_igemm_mode<0, true, true>(pl, p, st);
        else launch_igemm_mode<0, false, true>(pl, p, st);
    } else if (bf16) {
        if (fast && p.sd == 1) launch_igemm_mode<0, true>(pl, p, st);
        else if (fast) launch_igemm_mode<1, true>(pl, p, st);
        else launch_igemm_mode<2, true>(pl, p, st);
    } else {
        if (fast && p.sd == 1) launch_igemm_mode<0, false>(pl, p, st);
        else if (fast) launch_igemm_mode<1, false>(pl, p, st);
        else launch_igemm_mode<2, false>(pl, p, st);
    }
    if (pl.tail_split > 1) {
        if (p.stat_mean) {
            if (act) launch_tail_reduce_stats<true>(pl, p, st);
            else launch_tail_reduce_stats<false>(pl, p, st);
        } else {
            if (act) launch_tail_reduce<true>(pl, p, st);
            else launch_tail_reduce<false>(pl, p, st);
        }
    }
}

// data gradient of a 1x1 stride-2 convolution on an even-sized input: a GEMM whose rows are scattered
static bool is_scatter2(const rn50_conv_desc *d)
{
    return d->r == 1 && d->s == 1 && d->stride == 2 && d->pad == 0 && d->h % 2 == 0 && d->w % 2 == 0;
}

struct BwdDataPlan { IgemmPlan g; bool scatter; size_t wt_bytes, part_bytes; };
static BwdDataPlan plan_bwd_data(const rn50_conv_desc *d)
{
    const Geom ge = geom(d);
    BwdDataPlan b;
    b.scatter = is_scatter2(d);
    const long M = b.scatter ? ge.Mout : ge.Min;
    const int Kd = d->r * d->s * d->k;
    b.g = plan_igemm(d, RN50_OP_BWD_DATA, M, d->c, Kd, true, d->k);
    b.wt_bytes = align_up((size_t)d->k * d->r * d->s * d->c * sizeof(float), 256);
    b.part_bytes = b.g.ws_floats * sizeof(float);
    return b;
}

// Forward pass that also gathers the output's batch statistics: workspace = [the forward pass's own][statistics region].
// The region holds mean and squared deviations per (row tile, output channel), or, for a shape whose forward pass does not
// run through the tiled kernel, the band partials of the separate statistics pass; it is sized for both.
struct FwdStatsPlan { IgemmPlan g; int tiles_m; size_t conv_bytes, stat_bytes; };
static FwdStatsPlan plan_fwd_stats(const rn50_conv_desc *d)
{
    const Geom ge = geom(d);
    FwdStatsPlan f;
    f.g = plan_igemm(d, RN50_OP_FWD, ge.Mout, d->k, ge.Kdim, true, d->c);
    f.tiles_m = ceil_div(ge.Mout, f.g.bm);
    f.conv_bytes = align_up(f.g.ws_floats * sizeof(float), 256);
    f.stat_bytes = align_up(std::max((size_t)2 * f.tiles_m * d->k * sizeof(float), rn50_bn_workspace_bytes(d->n, d->k, ge.P, ge.Q)), 256);
    return f;
}

}  // namespace rn50

using namespace rn50;

// Workgroups of the first layer's own filter-gradient kernel (0: the layer goes through the general kernel).
static int stem_wgrad_grid(const rn50_conv_desc *d, const Geom &ge)
{
    if (!(d->c == 3 && d->r == 7 && d->s == 7 && d->stride == 2 && d->pad == 3 && d->k == 64 && d->in_dtype == RN50_DTYPE_F32 &&
          (long)d->n * d->h * d->w * 3 < (1l << 31)) || config()->no_stem_kernel)
        return 0;
    const int ntiles = d->n * ceil_div(ge.P, kStemTH) * ceil_div(ge.Q, kStemTW);
    return std::min(ntiles, 2 * (int)kCUs);
}

extern "C" size_t rn50_conv_workspace_bytes(const rn50_conv_desc *d, int op)
{
    if (conv_check("rn50_conv_workspace_bytes", d) != RN50_OK) return 0;
    const Geom ge = geom(d);
    if (op == RN50_OP_FWD) {
        return plan_igemm(d, RN50_OP_FWD, ge.Mout, d->k, ge.Kdim, true, d->c).ws_floats * sizeof(float);
    }
    if (op == RN50_OP_BWD_DATA) {
        const BwdDataPlan b = plan_bwd_data(d);
        return b.wt_bytes + b.part_bytes;
    }
    if (op == RN50_OP_BWD_WEIGHT) {
        if (stem_wgrad_grid(d, ge)) return (size_t)stem_wgrad_grid(d, ge) * d->k * ge.Kdim * sizeof(float);
        const GemmPlan pl = plan_wgrad(d, d->k, ge.Kdim, ge.Mout);
        return (size_t)pl.split * d->k * ge.Kdim * sizeof(float);
    }
    if (op == RN50_OP_BWD_DATA_FLIPPED) return plan_bwd_data(d).part_bytes;
    if (op == RN50_OP_FWD_BNSTATS) {
        const FwdStatsPlan f = plan_fwd_stats(d);
        return f.conv_bytes + f.stat_bytes;
    }
    return 0;
}

extern "C" int rn50_conv_plan(const rn50_conv_desc *d, int op, int *bm, int *bn, int *split, int *workgroups)
{
    if (int rc = conv_check("rn50_conv_plan", d)) return rc;
    const Geom ge = geom(d);
    int v[4];
    if (op == RN50_OP_FWD || op == RN50_OP_FWD_BNSTATS || op == RN50_OP_BWD_DATA || op == RN50_OP_BWD_DATA_FLIPPED) {
        const IgemmPlan pl = (op == RN50_OP_FWD || op == RN50_OP_FWD_BNSTATS) ? plan_igemm(d, RN50_OP_FWD, ge.Mout, d->k, ge.Kdim, true, d->c) : plan_bwd_data(d).g;
        v[0] = pl.bm; v[1] = pl.bn; v[2] = pl.tail_tiles ? pl.tail_split : 1; v[3] = pl.grid;
        if ((op == RN50_OP_FWD || op == RN50_OP_FWD_BNSTATS) && stem_wgrad_grid(d, ge)) {
            // the first layer's own forward kernel (same shapes as its filter-gradient kernel): tiles of 8 x 16 pixels x 64 filters
            v[0] = kStemTH * kStemTW; v[1] = 64; v[2] = 1;
            v[3] = std::min(d->n * ceil_div(ge.P, kStemTH) * ceil_div(ge.Q, kStemTW), 3 * (int)kCUs);
        }
    } else if (op == RN50_OP_BWD_WEIGHT) {
        const GemmPlan pl = plan_wgrad(d, d->k, ge.Kdim, ge.Mout);
        v[0] = pl.bm; v[1] = pl.bn; v[2] = pl.split; v[3] = ceil_div(d->k, pl.bm) * ceil_div(ge.Kdim, pl.bn) * pl.split;
        if (const int sgrid = stem_wgrad_grid(d, ge)) {  // the first layer's own kernel: 64 filters x 160 filter elements, one partial per workgroup
            v[0] = 64; v[1] = 160; v[2] = sgrid; v[3] = sgrid;
        }
    } else {
        return fail(RN50_EINVAL, "rn50_conv_plan: unknown operation %d", op);
    }
    if (bm) *bm = v[0];
    if (bn) *bn = v[1];
    if (split) *split = v[2];
    if (workgroups) *workgroups = v[3];
    return RN50_OK;
}

// stats (may be null): [2][row tiles][K] floats for the output's per-tile statistics; *gathered tells whether they were left
static int conv_fwd_impl(const char *who, const rn50_conv_desc *d, const float *x, const float *in_scale, const float *in_shift,
                         const float *w, float *y, void *ws, size_t ws_bytes, void *stream, float *stats = nullptr, bool *gathered = nullptr);

extern "C" int conv2d_fwd(const rn50_conv_desc *d, const float *x, const float *w, float *y, void *ws, size_t ws_bytes,
                          void *stream)
{
    return conv_fwd_impl("conv2d_fwd", d, x, nullptr, nullptr, w, y, ws, ws_bytes, stream);
}

extern "C" int conv2d_fwd_bnrelu_input(const rn50_conv_desc *d, const float *x, const float *in_scale, const float *in_shift,
                                       const float *w, float *y, void *ws, size_t ws_bytes, void *stream)
{
    RN50_REQUIRE(in_scale && in_shift && aligned16(in_scale) && aligned16(in_shift), RN50_EINVAL,
                 "conv2d_fwd_bnrelu_input: scale and shift must be non-null and 16-byte aligned");
    RN50_REQUIRE(d && d->c % kBK == 0, RN50_EUNSUPPORTED, "conv2d_fwd_bnrelu_input: the channel count must be a multiple of 32");
    return conv_fwd_impl("conv2d_fwd_bnrelu_input", d, x, in_scale, in_shift, w, y, ws, ws_bytes, stream);
}

static int conv_fwd_impl(const char *who, const rn50_conv_desc *d, const float *x, const float *in_scale, const float *in_shift,
                         const float *w, float *y, void *ws, size_t ws_bytes, void *stream, float *stats, bool *gathered)
{
    if (gathered) *gathered = false;
    if (int rc = conv_check(who, d)) return rc;
    RN50_REQUIRE(x && w && y, RN50_EINVAL, "%s: null pointer", who);
    RN50_REQUIRE(aligned16(x) && aligned16(w) && aligned16(y) && aligned16(ws), RN50_EINVAL, "%s: pointers must be 16-byte aligned", who);
    const Geom ge = geom(d);
    const IgemmPlan pl = plan_igemm(d, RN50_OP_FWD, ge.Mout, d->k, ge.Kdim, true, d->c);
    const size_t need = pl.ws_floats * sizeof(float);
    RN50_REQUIRE(ws_bytes >= need && (need == 0 || ws), RN50_EWORKSPACE, "%s: workspace too small (%zu < %zu)", who, ws_bytes, need);
    RN50_REQUIRE(!in_scale || act_of(d) != 2, RN50_EUNSUPPORTED, "%s: the fused input transform needs a bf16 or fp32 input of the variant's own type", who);
    if (d->c == 3 && d->r == 7 && d->s == 7 && d->stride == 2 && d->pad == 3 && d->k == 64 && d->in_dtype == RN50_DTYPE_F32 && !in_scale &&
        (long)d->n * d->h * d->w * 3 < (1l << 31) && !config()->no_stem_kernel) {
        // the network's first layer has a kernel of its own (input tile and filter in LDS)
        StemP sp{};
        sp.x = x; sp.w = w; sp.y = y;
        sp.N = d->n; sp.IH = d->h; sp.IW = d->w; sp.OH = ge.P; sp.OW = ge.Q;
        sp.tiles_h = ceil_div(ge.P, kStemTH); sp.tiles_w = ceil_div(ge.Q, kStemTW);
        sp.ntiles = d->n * sp.tiles_h * sp.tiles_w;
        hipLaunchKernelGGL(stem_fwd_kernel, dim3(std::min(sp.ntiles, 3 * (int)kCUs)), dim3(kConvThreads), 0, (hipStream_t)stream, sp);
        return launch_status(who);
    }
    IgemmP p{};
    p.a = x; p.b = w; p.in_scale = in_scale; p.in_shift = in_shift;
    p.IH = d->h; p.IW = d->w; p.Cin = d->c; p.OH = ge.P; p.OW = ge.Q; p.Nout = d->k; p.R = d->r; p.S = d->s;
    p.so = d->stride; p.off = -d->pad; p.sd = 1; p.M = (int)ge.Mout; p.Kdim = ge.Kdim; p.scatter2 = 0;
    if (stats) {
        p.stat_mean = stats;
        p.stat_m2 = stats + (size_t)ceil_div(ge.Mout, pl.bm) * d->k;
        if (gathered) *gathered = true;
    }
    run_igemm(p, pl, y, (float *)ws, bf16_of(d), act_of(d), (hipStream_t)stream);
    return launch_status(who);
}

extern "C" int conv2d_fwd_bnstats(const rn50_conv_desc *d, const float *x, const float *in_scale_or_null, const float *in_shift_or_null,
                                  const float *w, float *y, const float *gamma, const float *beta, float eps, float *save_mean,
                                  float *save_invstd, float *scale, float *shift, void *ws, size_t ws_bytes, void *stream)
{
    const char *who = "conv2d_fwd_bnstats";
    if (int rc = conv_check(who, d)) return rc;
    RN50_REQUIRE(gamma && beta && save_mean && save_invstd && scale && shift, RN50_EINVAL, "%s: null pointer", who);
    RN50_REQUIRE(aligned16(gamma) && aligned16(beta) && aligned16(save_mean) && aligned16(save_invstd) && aligned16(scale) && aligned16(shift),
                 RN50_EINVAL, "%s: pointers must be 16-byte aligned", who);
    RN50_REQUIRE((in_scale_or_null == nullptr) == (in_shift_or_null == nullptr), RN50_EINVAL, "%s: scale and shift of the input go together", who);
    RN50_REQUIRE(aligned16(in_scale_or_null) && aligned16(in_shift_or_null), RN50_EINVAL, "%s: pointers must be 16-byte aligned", who);
    RN50_REQUIRE(!in_scale_or_null || d->c % kBK == 0, RN50_EUNSUPPORTED, "%s: with a fused input transform the channel count must be a multiple of 32", who);
    RN50_REQUIRE(d->k % 4 == 0, RN50_EUNSUPPORTED, "%s: K must be a multiple of 4", who);
    RN50_REQUIRE(eps >= 0.f, RN50_EINVAL, "%s: negative eps", who);
    const Geom ge = geom(d);
    const FwdStatsPlan f = plan_fwd_stats(d);
    RN50_REQUIRE(ws && aligned16(ws) && ws_bytes >= f.conv_bytes + f.stat_bytes, RN50_EWORKSPACE, "%s: workspace too small (%zu < %zu)", who,
                 ws_bytes, f.conv_bytes + f.stat_bytes);
    float *stats = (float *)((char *)ws + f.conv_bytes);
    bool gathered = false;
    if (int rc = conv_fwd_impl(who, d, x, in_scale_or_null, in_shift_or_null, w, y, ws, f.conv_bytes, stream, stats, &gathered)) return rc;
    if (gathered) {
        bn_finalize_partials(ge.Mout, d->k, f.tiles_m, f.g.bm, stats, stats + (size_t)f.tiles_m * d->k, gamma, beta, eps, save_mean, save_invstd,
                             scale, shift, (hipStream_t)stream);
        return launch_status(who);
    }
    // no tiled kernel ran: the separate pass over y
    if (act_of(d))
        return bn_stats_scale_shift_bf16(d->n, d->k, ge.P, ge.Q, RN50_LAYOUT_NHWC, (const uint16_t *)y, gamma, beta, eps, save_mean, save_invstd,
                                         scale, shift, stats, f.stat_bytes, stream);
    return bn_stats_scale_shift(d->n, d->k, ge.P, ge.Q, RN50_LAYOUT_NHWC, y, gamma, beta, eps, save_mean, save_invstd, scale, shift, stats,
                                f.stat_bytes, stream);
}

// Data gradient with the filter already flipped and transposed (wt[c][R-1-r][S-1-s][k] = w[k][r][s][c]): a
// forward-type gather over dy.  ws = the implicit GEMM's partial tiles only.
int rn50::conv_bwd_data_pretransposed(const rn50_conv_desc *d, const float *dy, const float *wt, float *dx, void *ws,
                                      size_t ws_bytes, hipStream_t st)
{
    const Geom ge = geom(d);
    const BwdDataPlan b = plan_bwd_data(d);
    RN50_REQUIRE(act_of(d) != 2, RN50_EUNSUPPORTED, "conv2d_bwd_data: RN50_DTYPE_BF16_ACT_F32IN is for the forward pass and the filter gradient");
    RN50_REQUIRE(ws_bytes >= b.part_bytes && (b.part_bytes == 0 || ws), RN50_EWORKSPACE,
                 "conv2d_bwd_data: workspace too small (%zu < %zu)", ws_bytes, b.part_bytes);
    IgemmP p{};
    p.a = dy; p.b = wt;
    p.IH = ge.P; p.IW = ge.Q; p.Cin = d->k; p.Nout = d->c; p.R = d->r; p.S = d->s;
    p.Kdim = d->r * d->s * d->k;
    if (b.scatter) {
        // dx[n,2p,2q,:] = dy[n,p,q,:] * W, the other three pixels of each 2x2 cell receive no tap
        p.OH = ge.P; p.OW = ge.Q; p.so = 1; p.off = 0; p.sd = 1; p.M = (int)ge.Mout; p.scatter2 = 1;
    } else {
        p.OH = d->h; p.OW = d->w; p.so = 1; p.off = d->pad - (d->r - 1); p.sd = d->stride; p.M = (int)ge.Min; p.scatter2 = 0;
        if (d->stride == 2 && d->h % 2 == 0 && d->w % 2 == 0 && d->k % kBK == 0) {
            // rows grouped by the parity class of their pixel: a tile inside one class skips the taps that never reach it
            p.OH = d->h / 2; p.OW = d->w / 2; p.scatter2 = 2;
            p.div_class = make_fastdiv(p.M / 4);
        }
    }
    run_igemm(p, b.g, dx, (float *)ws, bf16_of(d), act_of(d), st);
    return launch_status("conv2d_bwd_data");
}

size_t rn50::conv_bwd_data_pretransposed_ws(const rn50_conv_desc *d) { return plan_bwd_data(d).part_bytes; }

void rn50::launch_filter_flip_batched(const void *jobs, int njobs, int nblocks, const float *theta, float *wt, hipStream_t st)
{
    hipLaunchKernelGGL(filter_flip_batched_kernel, dim3(nblocks), dim3(256), 0, st, (const FlipJob *)jobs, njobs, theta, wt);
}

void rn50::launch_filter_flip(int K, int C, int RS, const float *w, float *wt, hipStream_t st)
{
    hipLaunchKernelGGL(filter_flip_transpose_kernel, dim3(ceil_div(C, kFlipTile), ceil_div(K, kFlipTile), RS), dim3(256), 0, st, K, C, RS, w, wt);
}

extern "C" int conv2d_bwd_data(const rn50_conv_desc *d, const float *dy, const float *w, float *dx, void *ws,
                               size_t ws_bytes, void *stream)
{
    if (int rc = conv_check("conv2d_bwd_data", d)) return rc;
    RN50_REQUIRE(dy && w && dx, RN50_EINVAL, "conv2d_bwd_data: null pointer");
    RN50_REQUIRE(d->r == d->s, RN50_EUNSUPPORTED, "conv2d_bwd_data: non-square filters are not supported");
    RN50_REQUIRE(aligned16(dy) && aligned16(w) && aligned16(dx) && aligned16(ws), RN50_EINVAL,
                 "conv2d_bwd_data: pointers must be 16-byte aligned");
    RN50_REQUIRE(act_of(d) != 2, RN50_EUNSUPPORTED, "conv2d_bwd_data: RN50_DTYPE_BF16_ACT_F32IN is for the forward pass and the filter gradient");
    const BwdDataPlan b = plan_bwd_data(d);
    RN50_REQUIRE(ws && ws_bytes >= b.wt_bytes + b.part_bytes, RN50_EWORKSPACE, "conv2d_bwd_data: workspace too small (%zu < %zu)",
                 ws_bytes, b.wt_bytes + b.part_bytes);
    hipStream_t st = (hipStream_t)stream;
    // workspace = [flipped filter][partial tiles]
    float *wt = (float *)ws;
    launch_filter_flip(d->k, d->c, d->r * d->s, w, wt, st);
    return conv_bwd_data_pretransposed(d, dy, wt, dx, (char *)ws + b.wt_bytes, b.part_bytes, st);
}

extern "C" int conv2d_filter_flip(const rn50_conv_desc *d, const float *w, float *wt, void *stream)
{
    if (int rc = conv_check("conv2d_filter_flip", d)) return rc;
    RN50_REQUIRE(w && wt && w != wt, RN50_EINVAL, "conv2d_filter_flip: null pointer or in-place call");
    RN50_REQUIRE(aligned16(w) && aligned16(wt), RN50_EINVAL, "conv2d_filter_flip: pointers must be 16-byte aligned");
    launch_filter_flip(d->k, d->c, d->r * d->s, w, wt, (hipStream_t)stream);
    return launch_status("conv2d_filter_flip");
}

extern "C" int conv2d_bwd_data_flipped(const rn50_conv_desc *d, const float *dy, const float *wt, float *dx, void *ws,
                                       size_t ws_bytes, void *stream)
{
    if (int rc = conv_check("conv2d_bwd_data_flipped", d)) return rc;
    RN50_REQUIRE(dy && wt && dx, RN50_EINVAL, "conv2d_bwd_data_flipped: null pointer");
    RN50_REQUIRE(d->r == d->s, RN50_EUNSUPPORTED, "conv2d_bwd_data_flipped: non-square filters are not supported");
    RN50_REQUIRE(aligned16(dy) && aligned16(wt) && aligned16(dx) && aligned16(ws), RN50_EINVAL,
                 "conv2d_bwd_data_flipped: pointers must be 16-byte aligned");
    RN50_REQUIRE(act_of(d) != 2, RN50_EUNSUPPORTED, "conv2d_bwd_data_flipped: RN50_DTYPE_BF16_ACT_F32IN is for the forward pass and the filter gradient");
    const size_t need = plan_bwd_data(d).part_bytes;
    RN50_REQUIRE(ws_bytes >= need && (need == 0 || ws), RN50_EWORKSPACE, "conv2d_bwd_data_flipped: workspace too small (%zu < %zu)",
                 ws_bytes, need);
    return conv_bwd_data_pretransposed(d, dy, wt, dx, ws, ws_bytes, (hipStream_t)stream);
}

static int conv_bwd_weight_impl(const char *who, const rn50_conv_desc *d, const float *x, const float *in_scale, const float *in_shift,
                                const float *dy, float *dw, void *ws, size_t ws_bytes, void *stream);

extern "C" int conv2d_bwd_weight(const rn50_conv_desc *d, const float *x, const float *dy, float *dw, void *ws,
                                 size_t ws_bytes, void *stream)
{
    return conv_bwd_weight_impl("conv2d_bwd_weight", d, x, nullptr, nullptr, dy, dw, ws, ws_bytes, stream);
}

extern "C" int conv2d_bwd_weight_bnrelu_input(const rn50_conv_desc *d, const float *x, const float *in_scale, const float *in_shift,
                                              const float *dy, float *dw, void *ws, size_t ws_bytes, void *stream)
{
    RN50_REQUIRE(in_scale && in_shift && aligned16(in_scale) && aligned16(in_shift), RN50_EINVAL,
                 "conv2d_bwd_weight_bnrelu_input: scale and shift must be non-null and 16-byte aligned");
    RN50_REQUIRE(d && d->c % 4 == 0, RN50_EUNSUPPORTED, "conv2d_bwd_weight_bnrelu_input: the channel count must be a multiple of 4");
    return conv_bwd_weight_impl("conv2d_bwd_weight_bnrelu_input", d, x, in_scale, in_shift, dy, dw, ws, ws_bytes, stream);
}

static int conv_bwd_weight_impl(const char *who, const rn50_conv_desc *d, const float *x, const float *in_scale, const float *in_shift,
                                const float *dy, float *dw, void *ws, size_t ws_bytes, void *stream)
{
    if (int rc = conv_check(who, d)) return rc;
    RN50_REQUIRE(x && dy && dw, RN50_EINVAL, "%s: null pointer", who);
    RN50_REQUIRE(aligned16(x) && aligned16(dy) && aligned16(dw) && aligned16(ws), RN50_EINVAL, "%s: pointers must be 16-byte aligned", who);
    RN50_REQUIRE(d->k % 4 == 0, RN50_EUNSUPPORTED, "%s: K must be a multiple of 4", who);
    const Geom ge = geom(d);
    const bool vec = d->c % 4 == 0;
    if (const int sgrid = in_scale ? 0 : stem_wgrad_grid(d, ge)) {
        // the network's first layer has a kernel of its own (input tile and dy tile in LDS, one partial per workgroup)
        const size_t sneed = (size_t)sgrid * d->k * ge.Kdim * sizeof(float);
        RN50_REQUIRE(ws && ws_bytes >= sneed, RN50_EWORKSPACE, "%s: workspace too small (%zu < %zu)", who, ws_bytes, sneed);
        StemWP sp{};
        sp.x = x; sp.dy = dy; sp.part = (float *)ws;
        sp.N = d->n; sp.IH = d->h; sp.IW = d->w; sp.OH = ge.P; sp.OW = ge.Q;
        sp.tiles_h = ceil_div(ge.P, kStemTH); sp.tiles_w = ceil_div(ge.Q, kStemTW);
        sp.ntiles = d->n * sp.tiles_h * sp.tiles_w;
        hipLaunchKernelGGL(stem_wgrad_kernel, dim3(sgrid), dim3(kConvThreads), 0, (hipStream_t)stream, sp);
        const long scount4 = (long)d->k * ge.Kdim / 4;
        hipLaunchKernelGGL(splitk_reduce_kernel, dim3(ceil_div(scount4, 64)), dim3(256), 0, (hipStream_t)stream, scount4, sgrid,
                           (long)d->k * ge.Kdim, (const float *)ws, dw);
        return launch_status(who);
    }
    const GemmPlan pl = plan_wgrad(d, d->k, ge.Kdim, ge.Mout);
    const size_t need = (size_t)pl.split * d->k * ge.Kdim * sizeof(float);
    RN50_REQUIRE(ws && ws_bytes >= need, RN50_EWORKSPACE, "%s: workspace too small (%zu < %zu)", who, ws_bytes, need);
    RN50_REQUIRE(((long)d->k * ge.Kdim) % 4 == 0, RN50_EUNSUPPORTED, "%s: filter size must be a multiple of 4", who);
    const int act = act_of(d);
    RN50_REQUIRE(!act || d->k % 8 == 0, RN50_EUNSUPPORTED, "%s: with bf16 activations K must be a multiple of 8", who);
    RN50_REQUIRE(act != 1 || d->c % 8 == 0, RN50_EUNSUPPORTED, "%s: with bf16 activations C must be a multiple of 8", who);
    RN50_REQUIRE(!in_scale || act != 2, RN50_EUNSUPPORTED, "%s: the fused input transform needs an input of the variant's own type", who);
    WgradP p{};
    p.dy = dy; p.x = x; p.out = (float *)ws; p.in_scale = in_scale; p.in_shift = in_shift;
    wgrad_fill(p, d, ge.P, ge.Q, pl.bm, pl.bn, pl.split, pl.chunks_per_split);
    const int grid = p.tiles_k * p.tiles_j * pl.split;
    hipStream_t st = (hipStream_t)stream;
    const bool bf16 = bf16_of(d);
    if (act) {  // 64x64 tiles (plan_wgrad keeps to them)
        if (act == 2) hipLaunchKernelGGL((wgrad_act_kernel<true, false>), dim3(grid), dim3(kConvThreads), 0, st, p);
        else if (in_scale) hipLaunchKernelGGL((wgrad_act_kernel<false, true>), dim3(grid), dim3(kConvThreads), 0, st, p);
        else hipLaunchKernelGGL((wgrad_act_kernel<false, false>), dim3(grid), dim3(kConvThreads), 0, st, p);
    } else {
#define RN50_WG(BM_, BN_)                                                                                              \
    do {                                                                                                               \
        if (in_scale && bf16) hipLaunchKernelGGL((wgrad_kernel<BM_, BN_, true, true, true>), dim3(grid), dim3(kConvThreads), 0, st, p); \
        else if (in_scale) hipLaunchKernelGGL((wgrad_kernel<BM_, BN_, true, false, true>), dim3(grid), dim3(kConvThreads), 0, st, p);   \
        else if (bf16 && vec) hipLaunchKernelGGL((wgrad_kernel<BM_, BN_, true, true>), dim3(grid), dim3(kConvThreads), 0, st, p);   \
        else if (bf16) hipLaunchKernelGGL((wgrad_kernel<BM_, BN_, false, true>), dim3(grid), dim3(kConvThreads), 0, st, p);    \
        else if (vec) hipLaunchKernelGGL((wgrad_kernel<BM_, BN_, true, false>), dim3(grid), dim3(kConvThreads), 0, st, p);     \
        else hipLaunchKernelGGL((wgrad_kernel<BM_, BN_, false, false>), dim3(grid), dim3(kConvThreads), 0, st, p);             \
    } while (0)
    if (pl.bm == 128 && pl.bn == 128) RN50_WG(128, 128);
    else if (pl.bm == 128) RN50_WG(128, 64);
    else if (pl.bn == 128) RN50_WG(64, 128);
    else RN50_WG(64, 64);
#undef RN50_WG
    }
    const long count4 = p.split_stride / 4;
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3(ceil_div(count4, 64)), dim3(256), 0, st, count4, pl.split, p.split_stride,
                       (const float *)ws, dw);
    return launch_status(who);
}
