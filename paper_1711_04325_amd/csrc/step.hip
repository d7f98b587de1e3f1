// One GPU's share of a synchronous data-parallel ResNet-50 training step: forward, loss, backward, half-precision
// gradient buffer, update rule.  Host-side orchestration only: a static schedule of kernel launches on one stream
// over tensors planned inside the caller's arena.  No allocation, no synchronisation.
//
// Network: ResNet-50 of He et al. 2016 (the model the paper trains, Section 1), stride of a stage's first block on its
// first 1x1 convolution ("v1") or on its 3x3 convolution ("v1.5"; same parameters, larger 1x1 inputs); batch
// normalization with current-minibatch statistics only (Section 2); fp32 compute, fp16 communication buffer
// (Section 3); update rule of Appendix A.1.
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <string>
#include <vector>

#include "common.h"

namespace rn50 {

struct ConvL {
    std::string name;
    int c, k, r, stride, pad, hin, hout;
    size_t w_off, g_off, b_off;  // offsets in the flat parameter arenas
    int block_pos;               // 0 stem, 1 a, 2 b, 3 c, 4 projection
};
struct ParamE { std::string name; size_t off, count; int dims[4]; int kind; };

struct Net {
    std::vector<ConvL> convs;
    std::vector<ParamE> table;
    size_t fcw_off, fcb_off, count;
};

static Net build_net(int variant)
{
        Net t;
        size_t off = 0;
        auto add_conv = [&](const std::string &nm, int c, int k, int r, int stride, int pad, int hin, int pos) {
            ConvL l{nm, c, k, r, stride, pad, hin, (hin + 2 * pad - r) / stride + 1, 0, 0, 0, pos};
            l.w_off = off;
            t.table.push_back(ParamE{nm + ".w", off, (size_t)k * r * r * c, {k, r, r, c}, RN50_KIND_CONV_W});
            off += (size_t)k * r * r * c;
            l.g_off = off;
            t.table.push_back(ParamE{nm + ".g", off, (size_t)k, {k, 1, 1, 1}, RN50_KIND_BN_G});
            off += k;
            l.b_off = off;
            t.table.push_back(ParamE{nm + ".beta", off, (size_t)k, {k, 1, 1, 1}, RN50_KIND_BN_B});
            off += k;
            t.convs.push_back(l);
        };
        add_conv("stem", 3, 64, 7, 2, 3, 224, 0);
        static const int widths[4] = {64, 128, 256, 512}, nblocks[4] = {3, 4, 6, 3};
        int cin = 64, h = 56;
        for (int s = 0; s < 4; ++s)
            for (int b = 0; b < nblocks[s]; ++b) {
                const int stride = (b == 0 && s > 0) ? 2 : 1, wd = widths[s];
                char nm[32];
                snprintf(nm, sizeof nm, "s%d.b%d", s + 2, b);
                const int sa = variant == RN50_VARIANT_V1 ? stride : 1, sb = stride / sa;  // where the block's stride sits
                add_conv(std::string(nm) + ".a", cin, wd, 1, sa, 0, h, 1);
                add_conv(std::string(nm) + ".b", wd, wd, 3, sb, 1, h / sa, 2);
                add_conv(std::string(nm) + ".c", wd, 4 * wd, 1, 1, 0, h / stride, 3);
                if (b == 0) add_conv(std::string(nm) + ".p", cin, 4 * wd, 1, stride, 0, h, 4);
                cin = 4 * wd;
                h /= stride;
            }
        t.fcw_off = off;
        t.table.push_back(ParamE{"fc.w", off, (size_t)1000 * 2048, {1000, 2048, 1, 1}, RN50_KIND_FC_W});
        off += (size_t)1000 * 2048;
        t.fcb_off = off;
        t.table.push_back(ParamE{"fc.b", off, 1000, {1000, 1, 1, 1}, RN50_KIND_FC_B});
        off += 1000;
        t.count = off;
        return t;
}

// Parameter table, offsets and count are the same for both variants; only strides and spatial sizes differ.
static const Net &net(int variant = RN50_VARIANT_V1)
{
    static const Net v1 = build_net(RN50_VARIANT_V1), v15 = build_net(RN50_VARIANT_V15);
    return variant == RN50_VARIANT_V15 ? v15 : v1;
}

static rn50_conv_desc desc_of(const ConvL &l, int batch, int in_dtype = RN50_DTYPE_F32)
{
    rn50_conv_desc d;
    d.n = batch; d.c = l.c; d.h = l.hin; d.w = l.hin; d.k = l.k; d.r = l.r; d.s = l.r; d.stride = l.stride; d.pad = l.pad;
    d.layout = RN50_LAYOUT_NHWC; d.in_dtype = in_dtype;
    return d;
}

struct Plan {
    size_t total = 0;
    size_t mask_off, pool_out, pool_arg, feat, logits, dlogits, dfeat, ws_conv, ws_bn;
    size_t ws_conv_bytes, ws_bn_bytes;
    size_t gbuf[6];
    size_t dconv[3];             // ring of BN-input gradients: the filter gradient of one layer reads its buffer on the
                                 // side stream while the main stream already fills the next
    size_t ws_conv2;             // the side stream's convolution workspace
    size_t ws_conv3, ws_bn2;     // workspaces of the projection-branch stream
    size_t dconv_p, gbuf_p;      // projection branch of the backward pass: BN-input gradient and block-input gradient
    size_t flip_jobs, wt_arena;  // job table and destination of the one-launch filter flip of the backward pass
    int flip_blocks;
    std::vector<FlipJobHost> jobs;
    std::vector<size_t> conv_out, bn_out, mean, invstd, wt;  // wt: float offset of a layer's flipped filter in wt_arena
    std::vector<size_t> scale, shift;                        // per-channel scale and shift of a layer's BN (BN(x) = x*scale + shift)
    std::vector<size_t> relu_mask;                           // c layers: one byte per four channels, [block output > 0]
    // Grouped filter gradients: every layer's BN-input gradient keeps a buffer of its own until the launch that covers its
    // group has read it; one workspace for the partial sums (the groups run one after the other) and room for the plans.
    std::vector<size_t> dconv_l;
    size_t ws_group, ws_group_bytes, group_tables, group_tables_bytes;
};

constexpr int kGroupMinStages = 16;  // the workspace is planned for work items of at least this many stages

// One layer of a grouped filter-gradient launch, described without pointers (null pointers are not accepted by the checks,
// so sizes are asked for with a stand-in that is never dereferenced).
static rn50_wgrad_group_item group_item(const rn50_conv_desc &d)
{
    rn50_wgrad_group_item it{};
    it.desc = d;
    it.x = it.dy = reinterpret_cast<const float *>(uintptr_t(256));
    return it;
}

static size_t take(size_t &cur, size_t bytes)
{
    const size_t o = cur;
    cur += (bytes + 255) / 256 * 256;
    return o;
}

static Plan make_plan(int batch, int variant)
{
    const Net &n = net(variant);
    Plan p;
    size_t cur = 0;
    p.mask_off = take(cur, (n.count + RN50_WD_GROUP - 1) / RN50_WD_GROUP);
    size_t max_act = 0, wsc = 0, wsb = 0;
    for (const ConvL &l : n.convs) {
        const size_t cnt = (size_t)batch * l.hout * l.hout * l.k;
        p.conv_out.push_back(take(cur, cnt * 4));
        p.bn_out.push_back(take(cur, cnt * 4));
        p.mean.push_back(take(cur, (size_t)l.k * 4));
        p.invstd.push_back(take(cur, (size_t)l.k * 4));
        p.relu_mask.push_back(l.block_pos == 3 ? take(cur, cnt / 4) : 0);
        p.scale.push_back(take(cur, (size_t)l.k * 4));
        p.shift.push_back(take(cur, (size_t)l.k * 4));
        max_act = std::max(max_act, cnt);
        max_act = std::max(max_act, (size_t)batch * l.hin * l.hin * l.c);
        // workspaces sized for every operand storage a context may be created with (the filter gradient's plan depends on it)
        const bool first = &l == &n.convs[0];
        for (int dt : {RN50_DTYPE_F32, first ? RN50_DTYPE_BF16_ACT_F32IN : RN50_DTYPE_BF16_ACT}) {
            const rn50_conv_desc d = desc_of(l, batch, dt);
            wsc = std::max(wsc, rn50_conv_workspace_bytes(&d, RN50_OP_FWD));
            wsc = std::max(wsc, rn50_conv_workspace_bytes(&d, RN50_OP_FWD_BNSTATS));
            wsc = std::max(wsc, rn50_conv_workspace_bytes(&d, RN50_OP_BWD_WEIGHT));
            if (dt != RN50_DTYPE_BF16_ACT_F32IN) wsc = std::max(wsc, conv_bwd_data_pretransposed_ws(&d));
        }
        wsb = std::max(wsb, rn50_bn_workspace_bytes(batch, l.k, l.hout, l.hout));
    }
    // flipped filters of every convolution whose data gradient is needed (all but the stem)
    size_t wt_floats = 0;
    int blocks = 0;
    p.wt.assign(n.convs.size(), 0);
    for (size_t i = 1; i < n.convs.size(); ++i) {
        const ConvL &l = n.convs[i];
        FlipJobHost j;
        j.K = l.k; j.C = l.c; j.RS = l.r * l.r;
        j.tiles_c = (l.c + kFlipTileHost - 1) / kFlipTileHost; j.tiles_k = (l.k + kFlipTileHost - 1) / kFlipTileHost;
        j.block_begin = blocks;
        j.src_off = (long)l.w_off; j.dst_off = (long)wt_floats;
        p.jobs.push_back(j);
        p.wt[i] = wt_floats;
        blocks += j.RS * j.tiles_c * j.tiles_k;
        wt_floats += (size_t)l.k * l.r * l.r * l.c;
    }
    p.flip_blocks = blocks;
    p.flip_jobs = take(cur, p.jobs.size() * sizeof(FlipJobHost));
    p.wt_arena = take(cur, wt_floats * 4);
    const size_t pool_cnt = (size_t)batch * 56 * 56 * 64;
    p.pool_out = take(cur, pool_cnt * 4);
    p.pool_arg = take(cur, pool_cnt);
    p.feat = take(cur, (size_t)batch * 2048 * 4);
    p.logits = take(cur, (size_t)batch * 1000 * 4);
    p.dlogits = take(cur, (size_t)batch * 1000 * 4);
    p.dfeat = take(cur, (size_t)batch * 2048 * 4);
    for (int i = 0; i < 6; ++i) p.gbuf[i] = take(cur, max_act * 4);
    for (int i = 0; i < 3; ++i) p.dconv[i] = take(cur, max_act * 4);
    p.ws_conv_bytes = wsc;
    p.ws_bn_bytes = wsb;
    p.ws_conv = take(cur, wsc);
    p.ws_conv2 = take(cur, wsc);
    p.ws_conv3 = take(cur, wsc);
    p.ws_bn = take(cur, wsb);
    p.ws_bn2 = take(cur, wsb);
    p.dconv_p = take(cur, max_act * 4);
    p.gbuf_p = take(cur, max_act * 4);
    std::vector<rn50_wgrad_group_item> items;
    p.dconv_l.assign(n.convs.size(), 0);
    for (size_t i = 1; i < n.convs.size(); ++i) {
        const ConvL &l = n.convs[i];
        p.dconv_l[i] = take(cur, (size_t)batch * l.hout * l.hout * l.k * 4);
        items.push_back(group_item(desc_of(l, batch)));
    }
    p.ws_group_bytes = wgrad_group_ws_bytes((int)items.size(), items.data(), kGroupMinStages);
    p.ws_group = take(cur, p.ws_group_bytes);
    // every layer a group of its own is the most room the plans can take
    p.group_tables_bytes = items.size() * ((wgrad_group_table_bytes(1) + 255) / 256 * 256);
    p.group_tables = take(cur, p.group_tables_bytes);
    p.total = cur;
    return p;
}

}  // namespace rn50

using namespace rn50;

struct rn50_ctx {
    int batch;
    char *arena;
    Plan plan;
    int variant = RN50_VARIANT_V1;
    // RN50_DTYPE_F32 / RN50_DTYPE_BF16: operand precision of the convolutions (sums and all other steps are fp32).
    // RN50_DTYPE_BF16_ACT: every activation and activation gradient the step keeps in memory is bfloat16 (parameters, their
    // gradients, BN statistics, pooled features, logits and all sums stay fp32); the buffers are planned at their fp32 size.
    int conv_dtype = RN50_DTYPE_F32;
    // The BN + ReLU behind the stem and behind the a and b convolutions of a block has ONE consumer each (the max pooling, the
    // next convolution): it is applied by that consumer as it loads (and again by the consumer's filter gradient) instead
    // of by a kernel of its own, and its output is never written.  Option "fuse_bn" = 0 at rn50_create switches this off.
    // Bits: 1 = stem -> max pooling, 2 = b -> c (a 1x1 consumer), 4 = a -> b (a 3x3 consumer, which would apply it nine times).
    int fuse_bn = 3;
    // The BN backward of a block's c layer takes its ReLU mask from one byte per four channels that the forward pass wrote
    // beside the block output, instead of from the output itself.  Option "relu_mask" = 0 at rn50_create switches this off.
    bool relu_mask = true;
    // The forward convolutions gather the BN statistics of their output as they write it (conv2d_fwd_bnstats) instead of a
    // separate pass over the tensor.  Option "conv_bn_stats" = 0 at rn50_create switches this off.
    bool conv_bn_stats = true;
    std::vector<char> bn_out_stale;   // fused layers whose BN output buffer does not hold the last step's values (rn50_peek fills it)
    // Filter gradients run on a side stream, forked from and joined to the caller's stream with events: they are off
    // the critical path of the backward pass (only the data gradient feeds the next layer) and fill the CUs that the
    // tail of a data-gradient kernel leaves idle.
    bool use_side = false;
    hipStream_t side = nullptr;
    hipEvent_t ready[3] = {nullptr, nullptr, nullptr}, done[3] = {nullptr, nullptr, nullptr};
    // The projection shortcut of a stage's first block is independent of the block's a-b chain in both passes: it runs on
    // a third stream between a fork and a join event.
    hipStream_t side2 = nullptr;
    hipEvent_t pfork = nullptr, pjoin = nullptr;
    // The flipped/transposed filters of the backward pass depend only on the parameters: they are produced on the side
    // stream while the forward pass runs.
    hipEvent_t entry = nullptr, flipped = nullptr;
    // Filter gradients in grouped launches (option "wgrad_group" = blocks per group at rn50_create; fp32 contexts): the layers
    // of that many consecutive blocks go into one launch once the last of their BN-input gradients is written.  A group
    // launches after the layers of its last block in backward order.
    struct Group { int first_block, last_block; std::vector<int> layers; std::vector<char> host; size_t dev_off; };
    std::vector<Group> groups;
    hipEvent_t pbn = nullptr, gdone = nullptr;  // projection branch's BN backward done; last group launched so far done
};

// The blocks of the network: index of the a convolution and whether a projection shortcut follows the c convolution.
struct BlockL { int first; bool proj; };
static std::vector<BlockL> blocks_of(const Net &n)
{
    std::vector<BlockL> v;
    const int L = (int)n.convs.size();
    for (int li = 1; li < L;) {
        const bool proj = li + 3 < L && n.convs[li + 3].block_pos == 4;
        v.push_back(BlockL{li, proj});
        li += proj ? 4 : 3;
    }
    return v;
}

// Builds the grouped filter-gradient plans of a context and uploads them (rn50_create).
static int build_groups(rn50_ctx *c, const Config &cfg)
{
    const Net &n = net(c->variant);
    const Plan &pl = c->plan;
    char *A = c->arena;
    auto F = [&](size_t off) { return (const float *)(A + off); };
    const std::vector<BlockL> blocks = blocks_of(n);
    const int fuse = c->fuse_bn;
    auto fused_out = [&](int li) {
        const int pos = n.convs[li].block_pos;
        return (pos == 0 && (fuse & 1)) || (pos == 2 && (fuse & 2)) || (pos == 1 && (fuse & 4));
    };
    // groups in backward order: blocks from the last to the first, wgrad_group of them to a group
    std::vector<rn50_ctx::Group> groups;
    for (int b = (int)blocks.size() - 1; b >= 0; --b) {
        const bool start = groups.empty() || groups.back().first_block - groups.back().last_block + 1 >= cfg.wgrad_group;
        if (start) groups.push_back(rn50_ctx::Group{b, b, {}, {}, 0});
        groups.back().last_block = b;
        const int li = blocks[b].first;
        groups.back().layers.push_back(li + 2);
        if (blocks[b].proj) groups.back().layers.push_back(li + 3);
        groups.back().layers.push_back(li + 1);
        groups.back().layers.push_back(li);
    }
    const int stages = std::max(cfg.wgrad_group_stages, kGroupMinStages);
    size_t dev_off = pl.group_tables;
    for (rn50_ctx::Group &g : groups) {
        std::vector<rn50_wgrad_group_item> items;
        for (int li : g.layers) {
            const ConvL &l = n.convs[li];
            int b = 0;
            while (b + 1 < (int)blocks.size() && blocks[b + 1].first <= li) ++b;
            const float *block_in = b == 0 ? F(pl.pool_out) : F(pl.bn_out[blocks[b - 1].first + 2]);
            rn50_wgrad_group_item it{};
            it.desc = desc_of(l, c->batch);
            const int prod = (l.block_pos == 2 || l.block_pos == 3) ? li - 1 : -1;  // the layer whose BN + ReLU output is the input
            if (prod >= 0 && fused_out(prod)) {
                it.x = F(pl.conv_out[prod]);
                it.in_scale = F(pl.scale[prod]);
                it.in_shift = F(pl.shift[prod]);
            } else {
                it.x = prod >= 0 ? F(pl.bn_out[prod]) : block_in;
            }
            it.dy = F(pl.dconv_l[li]);
            it.dw_offset = l.w_off;
            items.push_back(it);
        }
        g.host.resize(wgrad_group_table_bytes((int)items.size()));
        g.dev_off = dev_off;
        dev_off += (g.host.size() + 255) / 256 * 256;
        if (dev_off > pl.group_tables + pl.group_tables_bytes) return fail(RN50_EWORKSPACE, "rn50_create: no room for the grouped plans");
        if (int rc = wgrad_group_plan((int)items.size(), items.data(), A + pl.ws_group, pl.ws_group_bytes, g.host.data(), g.host.size(), stages,
                                      cfg.wgrad_group_bm, cfg.wgrad_group_bn, cfg.wgrad_group_wgs_per_cu))
            return rc;
        if (hipMemcpy(A + g.dev_off, g.host.data(), g.host.size(), hipMemcpyHostToDevice) != hipSuccess)
            return fail(RN50_EHIP, "rn50_create: upload of a grouped plan failed");
    }
    c->groups = std::move(groups);
    return RN50_OK;
}

extern "C" size_t rn50_param_count(void) { return net().count; }
extern "C" int rn50_param_table_size(void) { return (int)net().table.size(); }

extern "C" int rn50_param_table(int idx, const char **name, size_t *offset, size_t *count, int dims[4], int *kind)
{
    const Net &n = net();
    RN50_REQUIRE(idx >= 0 && idx < (int)n.table.size(), RN50_EINVAL, "rn50_param_table: index out of range");
    const ParamE &e = n.table[idx];
    if (name) *name = e.name.c_str();
    if (offset) *offset = e.off;
    if (count) *count = e.count;
    if (dims) memcpy(dims, e.dims, sizeof e.dims);
    if (kind) *kind = e.kind;
    return RN50_OK;
}

extern "C" size_t rn50_activation_bytes(int batch, int variant)
{
    if (batch <= 0 || batch > 1024 || (variant != RN50_VARIANT_V1 && variant != RN50_VARIANT_V15)) return 0;
    return make_plan(batch, variant).total;
}

extern "C" int rn50_create(rn50_ctx **out, int batch, int variant, int conv_dtype, void *act_arena, size_t act_bytes)
{
    RN50_REQUIRE(out, RN50_EINVAL, "rn50_create: null output pointer");
    *out = nullptr;
    RN50_REQUIRE(batch > 0 && batch <= 1024, RN50_EINVAL, "rn50_create: batch must be in [1, 1024]");
    RN50_REQUIRE(variant == RN50_VARIANT_V1 || variant == RN50_VARIANT_V15, RN50_EINVAL,
                 "rn50_create: variant must be RN50_VARIANT_V1 or RN50_VARIANT_V15");
    RN50_REQUIRE(conv_dtype == RN50_DTYPE_F32 || conv_dtype == RN50_DTYPE_BF16 || conv_dtype == RN50_DTYPE_BF16_ACT, RN50_EINVAL,
                 "rn50_create: conv_dtype must be RN50_DTYPE_F32, RN50_DTYPE_BF16 or RN50_DTYPE_BF16_ACT");
    RN50_REQUIRE(act_arena && (reinterpret_cast<uintptr_t>(act_arena) & 255u) == 0, RN50_EINVAL,
                 "rn50_create: the arena must be non-null and 256-byte aligned");
    rn50_ctx *c = new rn50_ctx{batch, (char *)act_arena, make_plan(batch, variant)};
    c->variant = variant;
    c->conv_dtype = conv_dtype;
    if (act_bytes < c->plan.total) {
        const size_t need = c->plan.total;
        delete c;
        return fail(RN50_EWORKSPACE, "rn50_create: arena too small (%zu < %zu)", act_bytes, need);
    }
    // weight-decay mask: decay applies to convolution and FC weights, not to BN scale/shift or the FC bias
    const Net &n = net();
    std::vector<uint8_t> mask((n.count + RN50_WD_GROUP - 1) / RN50_WD_GROUP, 0);
    for (const ParamE &e : n.table)
        if (e.kind == RN50_KIND_CONV_W || e.kind == RN50_KIND_FC_W)
            for (size_t g = e.off / RN50_WD_GROUP; g < (e.off + e.count + RN50_WD_GROUP - 1) / RN50_WD_GROUP; ++g) mask[g] = 1;
    hipError_t e = hipMemcpy(c->arena + c->plan.mask_off, mask.data(), mask.size(), hipMemcpyHostToDevice);
    if (e == hipSuccess)
        e = hipMemcpy(c->arena + c->plan.flip_jobs, c->plan.jobs.data(), c->plan.jobs.size() * sizeof(FlipJobHost), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        delete c;
        return fail(RN50_EHIP, "rn50_create: upload failed: %s", hipGetErrorString(e));
    }
    const std::shared_ptr<const Config> cfg = config();  // the context keeps the switches it was created under
    // with 2-byte activations the transform on the way into LDS (widen, multiply-add, maximum, round, pack, eight values per
    // load) costs a 1x1 consumer more than the normalising pass it saves: only the max pooling fuses there
    c->fuse_bn = cfg->fuse_bn >= 0 ? cfg->fuse_bn : (conv_dtype == RN50_DTYPE_BF16_ACT ? 1 : 3);
    c->relu_mask = cfg->relu_mask;
    c->conv_bn_stats = cfg->conv_bn_stats;
    c->bn_out_stale.assign(n.convs.size(), 0);
    if (cfg->side_stream) {
        bool ok = hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking) == hipSuccess &&
                  hipStreamCreateWithFlags(&c->side2, hipStreamNonBlocking) == hipSuccess &&
                  hipEventCreateWithFlags(&c->pfork, hipEventDisableTiming) == hipSuccess &&
                  hipEventCreateWithFlags(&c->pjoin, hipEventDisableTiming) == hipSuccess &&
                  hipEventCreateWithFlags(&c->entry, hipEventDisableTiming) == hipSuccess &&
                  hipEventCreateWithFlags(&c->flipped, hipEventDisableTiming) == hipSuccess &&
                  hipEventCreateWithFlags(&c->pbn, hipEventDisableTiming) == hipSuccess &&
                  hipEventCreateWithFlags(&c->gdone, hipEventDisableTiming) == hipSuccess;
        for (int i = 0; i < 3 && ok; ++i)
            ok = hipEventCreateWithFlags(&c->ready[i], hipEventDisableTiming) == hipSuccess &&
                 hipEventCreateWithFlags(&c->done[i], hipEventDisableTiming) == hipSuccess;
        if (!ok) {
            rn50_destroy(c);
            return fail(RN50_EHIP, "rn50_create: could not create the side stream or its events");
        }
        c->use_side = true;
    }
    if (cfg->wgrad_group > 0 && conv_dtype == RN50_DTYPE_F32) {
        if (int rc = build_groups(c, *cfg)) {
            rn50_destroy(c);
            return rc;
        }
    }
    *out = c;
    return RN50_OK;
}

extern "C" void rn50_destroy(rn50_ctx *ctx)
{
    if (!ctx) return;
    for (int i = 0; i < 3; ++i) {
        if (ctx->ready[i]) (void)hipEventDestroy(ctx->ready[i]);
        if (ctx->done[i]) (void)hipEventDestroy(ctx->done[i]);
    }
    if (ctx->pfork) (void)hipEventDestroy(ctx->pfork);
    if (ctx->pjoin) (void)hipEventDestroy(ctx->pjoin);
    if (ctx->entry) (void)hipEventDestroy(ctx->entry);
    if (ctx->flipped) (void)hipEventDestroy(ctx->flipped);
    if (ctx->pbn) (void)hipEventDestroy(ctx->pbn);
    if (ctx->gdone) (void)hipEventDestroy(ctx->gdone);
    if (ctx->side) (void)hipStreamDestroy(ctx->side);
    if (ctx->side2) (void)hipStreamDestroy(ctx->side2);
    delete ctx;
}

#define RN50_TRY_(call) \
    do { if (int rc_ = (call)) return rc_; } while (0)

extern "C" int rn50_filter_flip_all(rn50_ctx *ctx, const float *theta, void *stream)
{
    RN50_REQUIRE(ctx && theta, RN50_EINVAL, "rn50_filter_flip_all: null pointer");
    const Plan &pl = ctx->plan;
    char *A = (char *)ctx->arena;
    launch_filter_flip_batched(A + pl.flip_jobs, (int)pl.jobs.size(), pl.flip_blocks, theta, (float *)(A + pl.wt_arena), (hipStream_t)stream);
    return launch_status("rn50_filter_flip_all");
}

extern "C" int rn50_wgrad_groups_run(rn50_ctx *ctx, float *grad, void *stream)
{
    RN50_REQUIRE(ctx && grad, RN50_EINVAL, "rn50_wgrad_groups_run: null pointer");
    for (const rn50_ctx::Group &g : ctx->groups)
        RN50_TRY_(conv2d_bwd_weight_group(g.host.data(), ctx->arena + g.dev_off, grad, stream));
    return (int)ctx->groups.size();
}

extern "C" const float *rn50_peek(rn50_ctx *ctx, int layer, int what, size_t *count, void *stream)
{
    if (!ctx) return nullptr;
    const Plan &pl = ctx->plan;
    const size_t N = ctx->batch;
    size_t off, c;
    if (what >= 4) {
        switch (what) {
        case 4: off = pl.pool_out; c = N * 56 * 56 * 64; break;
        case 5: off = pl.pool_arg; c = N * 56 * 56 * 64; break;  // bytes
        case 6: off = pl.feat; c = N * 2048; break;
        case 7: off = pl.logits; c = N * 1000; break;
        case 8: off = pl.dlogits; c = N * 1000; break;
        default: return nullptr;
        }
    } else {
        if (layer < 0 || layer >= (int)net(ctx->variant).convs.size()) return nullptr;
        const ConvL &l = net(ctx->variant).convs[layer];
        const size_t cnt = N * l.hout * l.hout * l.k;
        switch (what) {
        case 0: off = pl.conv_out[layer]; c = cnt; break;
        case 1:
            off = pl.bn_out[layer];
            c = cnt;
            if (ctx->bn_out_stale[layer]) {
                // a fused layer: its BN + ReLU output was never written; enqueue the kernel that produces it
                const int rc = ctx->conv_dtype == RN50_DTYPE_BF16_ACT
                                   ? bn_apply_scale_shift_bf16((int)N, l.k, l.hout, l.hout, (const uint16_t *)(ctx->arena + pl.conv_out[layer]),
                                                               (const float *)(ctx->arena + pl.scale[layer]),
                                                               (const float *)(ctx->arena + pl.shift[layer]), 1,
                                                               (uint16_t *)(ctx->arena + off), (hipStream_t)stream)
                                   : bn_apply_scale_shift((int)N, l.k, l.hout, l.hout, (const float *)(ctx->arena + pl.conv_out[layer]),
                                                          (const float *)(ctx->arena + pl.scale[layer]),
                                                          (const float *)(ctx->arena + pl.shift[layer]), 1, (float *)(ctx->arena + off),
                                                          (hipStream_t)stream);
                if (rc != RN50_OK) return nullptr;
                ctx->bn_out_stale[layer] = 0;
            }
            break;
        case 2: off = pl.mean[layer]; c = l.k; break;
        case 3: off = pl.invstd[layer]; c = l.k; break;
        default: return nullptr;
        }
    }
    if (count) *count = c;
    return (const float *)(ctx->arena + off);
}

#define RN50_TRY(call) \
    do { if (int rc_ = (call)) return rc_; } while (0)

// Validation-side forward (Section 2): every BN normalises with the statistics the context holds, i.e. those the last
// training forward saved (with several workers: after averaging them, which bn_stats_average does on gathered sets and
// rn50_set_bn_stats stores back).  Overwrites the stored activations of the last training step.
extern "C" int rn50_forward_eval(rn50_ctx *ctx, const float *images, const float *theta, float *logits_out, void *stream)
{
    RN50_REQUIRE(ctx && images && theta && logits_out, RN50_EINVAL, "rn50_forward_eval: null pointer");
    RN50_REQUIRE(aligned16(images) && aligned16(theta) && aligned16(logits_out), RN50_EINVAL,
                 "rn50_forward_eval: pointers must be 16-byte aligned");
    RN50_REQUIRE(ctx->conv_dtype != RN50_DTYPE_BF16_ACT, RN50_EUNSUPPORTED,
                 "rn50_forward_eval: not built for contexts with bf16 activations");
    const Net &n = net(ctx->variant);
    const Plan &pl = ctx->plan;
    const int N = ctx->batch;
    char *A = ctx->arena;
    auto F = [&](size_t off) { return (float *)(A + off); };
    void *wsc = A + pl.ws_conv, *wsb = A + pl.ws_bn;
    const int L = (int)n.convs.size();
    auto conv_bn = [&](int li, const float *x, const float *residual, int relu) -> int {
        const ConvL &l = n.convs[li];
        const rn50_conv_desc d = desc_of(l, N, ctx->conv_dtype);
        RN50_TRY(conv2d_fwd(&d, x, theta + l.w_off, F(pl.conv_out[li]), wsc, pl.ws_conv_bytes, stream));
        ctx->bn_out_stale[li] = 0;  // every BN output is written here
        return bn_fwd_inference(N, l.k, l.hout, l.hout, RN50_LAYOUT_NHWC, F(pl.conv_out[li]), theta + l.g_off, theta + l.b_off,
                                F(pl.mean[li]), F(pl.invstd[li]), residual, relu, F(pl.bn_out[li]), wsb, pl.ws_bn_bytes, stream);
    };
    RN50_TRY(conv_bn(0, images, nullptr, 1));
    RN50_TRY(maxpool3x3s2_fwd(N, 64, 112, 112, F(pl.bn_out[0]), F(pl.pool_out), (uint8_t *)(A + pl.pool_arg), stream));
    const float *h = F(pl.pool_out);
    for (int li = 1; li < L;) {
        const bool proj = li + 3 < L && n.convs[li + 3].block_pos == 4;
        const float *shortcut = h;
        if (proj) {
            RN50_TRY(conv_bn(li + 3, h, nullptr, 0));
            shortcut = F(pl.bn_out[li + 3]);
        }
        RN50_TRY(conv_bn(li, h, nullptr, 1));
        RN50_TRY(conv_bn(li + 1, F(pl.bn_out[li]), nullptr, 1));
        RN50_TRY(conv_bn(li + 2, F(pl.bn_out[li + 1]), shortcut, 1));
        h = F(pl.bn_out[li + 2]);
        li += proj ? 4 : 3;
    }
    RN50_TRY(avgpool_fwd(N, 2048, 7, 7, h, F(pl.feat), stream));
    return fc_fwd(N, 2048, 1000, F(pl.feat), theta + n.fcw_off, theta + n.fcb_off, logits_out, stream);
}

// Replaces the statistics of BN layer `layer` held by the context (device-to-device copies on the stream): the way averaged
// or otherwise externally produced statistics reach rn50_forward_eval.
extern "C" int rn50_set_bn_stats(rn50_ctx *ctx, int layer, const float *mean, const float *invstd, void *stream)
{
    RN50_REQUIRE(ctx && mean && invstd, RN50_EINVAL, "rn50_set_bn_stats: null pointer");
    const Net &n = net(ctx->variant);
    RN50_REQUIRE(layer >= 0 && layer < (int)n.convs.size(), RN50_EINVAL, "rn50_set_bn_stats: layer out of range");
    const size_t bytes = (size_t)n.convs[layer].k * sizeof(float);
    hipError_t e = hipMemcpyAsync(ctx->arena + ctx->plan.mean[layer], mean, bytes, hipMemcpyDeviceToDevice, (hipStream_t)stream);
    if (e == hipSuccess)
        e = hipMemcpyAsync(ctx->arena + ctx->plan.invstd[layer], invstd, bytes, hipMemcpyDeviceToDevice, (hipStream_t)stream);
    if (e != hipSuccess) return fail(RN50_EHIP, "rn50_set_bn_stats: %s", hipGetErrorString(e));
    return RN50_OK;
}

// pending_stem: when non-null and the side stream is in use, the call returns with the stem's filter gradient (the last
// one of the pass) possibly still running on the side stream and stores the event that follows it; everything else is
// joined.  The caller must make `stream` wait for that event before it reads the stem's filter gradient.
static int forward_backward_impl(rn50_ctx *ctx, const float *images, const int32_t *labels, const float *theta, float *grad,
                                 float bn_eps, float *loss_out, void *stream, hipEvent_t *pending_stem)
{
    RN50_REQUIRE(ctx && images && labels && theta && grad && loss_out, RN50_EINVAL, "rn50_forward_backward: null pointer");
    RN50_REQUIRE(aligned16(images) && aligned16(theta) && aligned16(grad), RN50_EINVAL,
                 "rn50_forward_backward: pointers must be 16-byte aligned");
    const Net &n = net(ctx->variant);
    const Plan &pl = ctx->plan;
    const int N = ctx->batch;
    char *A = ctx->arena;
    auto F = [&](size_t off) { return (float *)(A + off); };
    void *wsc = A + pl.ws_conv, *wsb = A + pl.ws_bn;
    const int L = (int)n.convs.size();

    hipStream_t main_st = (hipStream_t)stream;
#define RN50_HIP(call)                                                                                   \
    do {                                                                                                 \
        const hipError_t e_ = (call);                                                                    \
        if (e_ != hipSuccess) return fail(RN50_EHIP, "rn50_forward_backward: %s", hipGetErrorString(e_)); \
    } while (0)

    // conv -> BN(batch statistics) [+ residual] [ReLU], on the caller's stream or on the projection-branch stream
    // prod >= 0: the input is the BN + ReLU of layer prod's convolution output, applied as it is loaded (x is ignored).
    // The stem and the a and b layers of a block only get their statistics here when the context fuses: their consumer
    // normalises.
    const int fuse = ctx->fuse_bn;
    auto fused_out = [&](int li) {  // is the BN + ReLU behind layer li applied by its consumer?
        const int pos = n.convs[li].block_pos;
        return (pos == 0 && (fuse & 1)) || (pos == 2 && (fuse & 2)) || (pos == 1 && (fuse & 4));
    };
    const bool a16 = ctx->conv_dtype == RN50_DTYPE_BF16_ACT;  // activations in memory are bfloat16
    auto H = [](const float *q) { return reinterpret_cast<const uint16_t *>(q); };
    auto HW_ = [](float *q) { return reinterpret_cast<uint16_t *>(q); };
    // the first layer reads the fp32 image whatever the activation storage
    auto dtype_of = [&](int li) { return a16 && li == 0 ? RN50_DTYPE_BF16_ACT_F32IN : ctx->conv_dtype; };
    auto conv_bn = [&](int li, const float *x, const float *residual, int relu, bool branch = false, int prod = -1) -> int {
        const ConvL &l = n.convs[li];
        const rn50_conv_desc d = desc_of(l, N, dtype_of(li));
        void *st = branch ? (void *)ctx->side2 : stream;
        if (ctx->conv_bn_stats) {
            // statistics gathered by the convolution itself; what is left of the BN is the normalising pass, where the
            // consumer does not normalise as it loads
            RN50_TRY(conv2d_fwd_bnstats(&d, prod >= 0 ? F(pl.conv_out[prod]) : x, prod >= 0 ? F(pl.scale[prod]) : nullptr,
                                        prod >= 0 ? F(pl.shift[prod]) : nullptr, theta + l.w_off, F(pl.conv_out[li]), theta + l.g_off,
                                        theta + l.b_off, bn_eps, F(pl.mean[li]), F(pl.invstd[li]), F(pl.scale[li]), F(pl.shift[li]),
                                        branch ? A + pl.ws_conv3 : wsc, pl.ws_conv_bytes, st));
            ctx->bn_out_stale[li] = fused_out(li) ? 1 : 0;
            if (fused_out(li)) return RN50_OK;
            uint8_t *mask = l.block_pos == 3 && ctx->relu_mask ? (uint8_t *)(A + pl.relu_mask[li]) : nullptr;
            if (a16)
                return bn_fwd_apply_bf16(N, l.k, l.hout, l.hout, RN50_LAYOUT_NHWC, H(F(pl.conv_out[li])), F(pl.scale[li]), F(pl.shift[li]),
                                         H(residual), relu, HW_(F(pl.bn_out[li])), mask, st);
            return bn_fwd_apply(N, l.k, l.hout, l.hout, RN50_LAYOUT_NHWC, F(pl.conv_out[li]), F(pl.scale[li]), F(pl.shift[li]), residual, relu,
                                F(pl.bn_out[li]), mask, st);
        }
        if (prod >= 0)
            RN50_TRY(conv2d_fwd_bnrelu_input(&d, F(pl.conv_out[prod]), F(pl.scale[prod]), F(pl.shift[prod]), theta + l.w_off,
                                             F(pl.conv_out[li]), branch ? A + pl.ws_conv3 : wsc, pl.ws_conv_bytes, st));
        else
            RN50_TRY(conv2d_fwd(&d, x, theta + l.w_off, F(pl.conv_out[li]), branch ? A + pl.ws_conv3 : wsc, pl.ws_conv_bytes, st));
        if (fused_out(li)) {
            ctx->bn_out_stale[li] = 1;
            if (a16)
                return bn_stats_scale_shift_bf16(N, l.k, l.hout, l.hout, RN50_LAYOUT_NHWC, H(F(pl.conv_out[li])), theta + l.g_off,
                                                 theta + l.b_off, bn_eps, F(pl.mean[li]), F(pl.invstd[li]), F(pl.scale[li]),
                                                 F(pl.shift[li]), branch ? A + pl.ws_bn2 : wsb, pl.ws_bn_bytes, st);
            return bn_stats_scale_shift(N, l.k, l.hout, l.hout, RN50_LAYOUT_NHWC, F(pl.conv_out[li]), theta + l.g_off, theta + l.b_off,
                                        bn_eps, F(pl.mean[li]), F(pl.invstd[li]), F(pl.scale[li]), F(pl.shift[li]),
                                        branch ? A + pl.ws_bn2 : wsb, pl.ws_bn_bytes, st);
        }
        ctx->bn_out_stale[li] = 0;
        if (a16)
            return bn_fwd_batchstats_bf16(N, l.k, l.hout, l.hout, RN50_LAYOUT_NHWC, H(F(pl.conv_out[li])), theta + l.g_off, theta + l.b_off,
                                          bn_eps, H(residual), relu, HW_(F(pl.bn_out[li])),
                                          l.block_pos == 3 && ctx->relu_mask ? (uint8_t *)(A + pl.relu_mask[li]) : nullptr, F(pl.mean[li]),
                                          F(pl.invstd[li]), branch ? A + pl.ws_bn2 : wsb, pl.ws_bn_bytes, st);
        if (l.block_pos == 3 && ctx->relu_mask)  // the block output: the backward pass reads a byte mask instead of it
            return bn_fwd_batchstats_mask(N, l.k, l.hout, l.hout, RN50_LAYOUT_NHWC, F(pl.conv_out[li]), theta + l.g_off, theta + l.b_off,
                                          bn_eps, residual, F(pl.bn_out[li]), (uint8_t *)(A + pl.relu_mask[li]), F(pl.mean[li]),
                                          F(pl.invstd[li]), branch ? A + pl.ws_bn2 : wsb, pl.ws_bn_bytes, st);
        return bn_fwd_batchstats(N, l.k, l.hout, l.hout, RN50_LAYOUT_NHWC, F(pl.conv_out[li]), theta + l.g_off, theta + l.b_off,
                                 bn_eps, residual, relu, F(pl.bn_out[li]), F(pl.mean[li]), F(pl.invstd[li]),
                                 branch ? A + pl.ws_bn2 : wsb, pl.ws_bn_bytes, st);
    };

    // every filter flipped and transposed for the data gradients, in one launch: beside the forward pass when there is a
    // side stream (after everything already enqueued on the caller's stream, which may still read the previous copy)
    if (ctx->use_side) {
        RN50_HIP(hipEventRecord(ctx->entry, main_st));
        RN50_HIP(hipStreamWaitEvent(ctx->side, ctx->entry, 0));
        launch_filter_flip_batched(A + pl.flip_jobs, (int)pl.jobs.size(), pl.flip_blocks, theta, F(pl.wt_arena), ctx->side);
        RN50_HIP(hipEventRecord(ctx->flipped, ctx->side));
    }

    // ---------------- forward ----------------
    RN50_TRY(conv_bn(0, images, nullptr, 1));
    if (a16)
        RN50_TRY(maxpool3x3s2_fwd_bf16(N, 64, 112, 112, H(F(fused_out(0) ? pl.conv_out[0] : pl.bn_out[0])),
                                       fused_out(0) ? F(pl.scale[0]) : nullptr, fused_out(0) ? F(pl.shift[0]) : nullptr,
                                       HW_(F(pl.pool_out)), (uint8_t *)(A + pl.pool_arg), stream));
    else if (fused_out(0))
        RN50_TRY(maxpool3x3s2_fwd_bnrelu_input(N, 64, 112, 112, F(pl.conv_out[0]), F(pl.scale[0]), F(pl.shift[0]), F(pl.pool_out),
                                               (uint8_t *)(A + pl.pool_arg), stream));
    else
        RN50_TRY(maxpool3x3s2_fwd(N, 64, 112, 112, F(pl.bn_out[0]), F(pl.pool_out), (uint8_t *)(A + pl.pool_arg), stream));
    const float *h = F(pl.pool_out);
    std::vector<const float *> block_in;  // input activation of each block
    std::vector<int> block_first;         // index of its 'a' convolution
    for (int li = 1; li < L;) {
        const bool proj = li + 3 < L && n.convs[li + 3].block_pos == 4;
        block_in.push_back(h);
        block_first.push_back(li);
        const float *shortcut = h;
        if (proj) {
            // the projection shortcut only needs the block input: it runs beside the a and b layers
            if (ctx->use_side) {
                RN50_HIP(hipEventRecord(ctx->pfork, main_st));
                RN50_HIP(hipStreamWaitEvent(ctx->side2, ctx->pfork, 0));
            }
            RN50_TRY(conv_bn(li + 3, h, nullptr, 0, ctx->use_side));
            if (ctx->use_side) RN50_HIP(hipEventRecord(ctx->pjoin, ctx->side2));
            shortcut = F(pl.bn_out[li + 3]);
        }
        RN50_TRY(conv_bn(li, h, nullptr, 1));
        RN50_TRY(conv_bn(li + 1, F(pl.bn_out[li]), nullptr, 1, false, fused_out(li) ? li : -1));
        if (proj && ctx->use_side) RN50_HIP(hipStreamWaitEvent(main_st, ctx->pjoin, 0));
        RN50_TRY(conv_bn(li + 2, F(pl.bn_out[li + 1]), shortcut, 1, false, fused_out(li + 1) ? li + 1 : -1));
        h = F(pl.bn_out[li + 2]);
        li += proj ? 4 : 3;
    }
    if (a16) RN50_TRY(avgpool_fwd_bf16(N, 2048, 7, 7, H(h), F(pl.feat), stream));
    else RN50_TRY(avgpool_fwd(N, 2048, 7, 7, h, F(pl.feat), stream));
    RN50_TRY(fc_fwd(N, 2048, 1000, F(pl.feat), theta + n.fcw_off, theta + n.fcb_off, F(pl.logits), stream));
    RN50_TRY(softmax_ce(N, 1000, F(pl.logits), labels, loss_out, F(pl.dlogits), stream));

    // ---------------- backward ----------------
    RN50_TRY(fc_bwd(N, 2048, 1000, F(pl.feat), theta + n.fcw_off, F(pl.dlogits), F(pl.dfeat), grad + n.fcw_off, grad + n.fcb_off, stream));
    if (ctx->use_side) RN50_HIP(hipStreamWaitEvent(main_st, ctx->flipped, 0));
    else launch_filter_flip_batched(A + pl.flip_jobs, (int)pl.jobs.size(), pl.flip_blocks, theta, F(pl.wt_arena), main_st);
    float *T2 = F(pl.gbuf[1]);
    float *setO[2] = {F(pl.gbuf[2]), F(pl.gbuf[4])}, *setR[2] = {F(pl.gbuf[3]), F(pl.gbuf[5])};
    float *ring[3] = {F(pl.dconv[0]), F(pl.dconv[1]), F(pl.dconv[2])};
    int cur = 0;
    if (a16) RN50_TRY(avgpool_bwd_bf16(N, 2048, 7, 7, F(pl.dfeat), HW_(setO[cur]), stream));
    else RN50_TRY(avgpool_bwd(N, 2048, 7, 7, F(pl.dfeat), setO[cur], stream));
    const float *in1 = setO[cur], *in2 = nullptr;
    int calls = 0;  // BN/conv backward calls issued so far: call i uses ring[i % 3]
    const bool grouped = !ctx->groups.empty();
    bool group_launched = false;

    // BN backward of layer li (incoming gradient g1 (+ g2)) into a ring buffer, then the filter gradient (side stream)
    // and the data gradient (main stream)
    // x_prod >= 0: the layer's input is the BN + ReLU of layer x_prod's convolution output, which the filter gradient
    // applies as it loads (x_in is ignored)
    auto bn_conv_bwd = [&](int li, const float *x_in, const float *g1, const float *g2, int relu, float *dres,
                           float *dx_or_null, int x_prod = -1) -> int {
        const ConvL &l = n.convs[li];
        const rn50_conv_desc d = desc_of(l, N, dtype_of(li));
        const bool in_group = grouped && li > 0;  // its filter gradient belongs to a grouped launch
        const int slot = grouped ? 0 : calls % 3;
        float *dconv = in_group ? F(pl.dconv_l[li]) : ring[slot];
        // the filter gradient that read this buffer three calls ago must have finished
        if (ctx->use_side && !grouped && calls >= 3) RN50_HIP(hipStreamWaitEvent(main_st, ctx->done[slot], 0));
        if (a16) {
            // mask source: rebuilt from the BN input (no residual), the byte mask (block outputs), else the stored output
            const bool xm = relu && !g2 && !dres, bm = relu && !xm && l.block_pos == 3 && ctx->relu_mask;
            RN50_TRY(bn_bwd_batchstats_bf16(N, l.k, l.hout, l.hout, RN50_LAYOUT_NHWC, H(F(pl.conv_out[li])), H(g1), H(g2),
                                            relu && !xm && !bm ? H(F(pl.bn_out[li])) : nullptr,
                                            bm ? (const uint8_t *)(A + pl.relu_mask[li]) : nullptr, theta + l.g_off,
                                            xm ? theta + l.b_off : nullptr, F(pl.mean[li]), F(pl.invstd[li]), relu, HW_(dconv), HW_(dres),
                                            grad + l.g_off, grad + l.b_off, wsb, pl.ws_bn_bytes, stream));
        } else if (relu && !g2 && !dres)  // BN -> ReLU with no residual (a and b layers, stem): the mask is rebuilt from the BN input
            RN50_TRY(bn_bwd_batchstats_xmask(N, l.k, l.hout, l.hout, RN50_LAYOUT_NHWC, F(pl.conv_out[li]), g1, theta + l.g_off,
                                             theta + l.b_off, F(pl.mean[li]), F(pl.invstd[li]), dconv, grad + l.g_off, grad + l.b_off,
                                             wsb, pl.ws_bn_bytes, stream));
        else if (relu && l.block_pos == 3 && ctx->relu_mask)
            RN50_TRY(bn_bwd_batchstats_mask(N, l.k, l.hout, l.hout, RN50_LAYOUT_NHWC, F(pl.conv_out[li]), g1, g2,
                                            (const uint8_t *)(A + pl.relu_mask[li]), theta + l.g_off, F(pl.mean[li]), F(pl.invstd[li]),
                                            dconv, dres, grad + l.g_off, grad + l.b_off, wsb, pl.ws_bn_bytes, stream));
        else
            RN50_TRY(bn_bwd_batchstats(N, l.k, l.hout, l.hout, RN50_LAYOUT_NHWC, F(pl.conv_out[li]), g1, g2,
                                       relu ? F(pl.bn_out[li]) : nullptr, theta + l.g_off, F(pl.mean[li]), F(pl.invstd[li]), relu, dconv,
                                       dres, grad + l.g_off, grad + l.b_off, wsb, pl.ws_bn_bytes, stream));
        auto wgrad = [&](void *ws, void *st) -> int {
            if (x_prod >= 0)
                return conv2d_bwd_weight_bnrelu_input(&d, F(pl.conv_out[x_prod]), F(pl.scale[x_prod]), F(pl.shift[x_prod]), dconv,
                                                      grad + l.w_off, ws, pl.ws_conv_bytes, st);
            return conv2d_bwd_weight(&d, x_in, dconv, grad + l.w_off, ws, pl.ws_conv_bytes, st);
        };
        if (in_group) {
            // the launch of its group follows the last layer of the group; the event is for a projection branch that starts here
            if (ctx->use_side) RN50_HIP(hipEventRecord(ctx->ready[slot], main_st));
        } else if (ctx->use_side && grouped) {
            // the first layer, beside the last grouped launch: on the projection-branch stream, which is idle by now
            RN50_HIP(hipEventRecord(ctx->ready[slot], main_st));
            RN50_HIP(hipStreamWaitEvent(ctx->side2, ctx->ready[slot], 0));
            RN50_TRY(wgrad(A + pl.ws_conv3, ctx->side2));
            RN50_HIP(hipEventRecord(ctx->done[slot], ctx->side2));
        } else if (ctx->use_side) {
            RN50_HIP(hipEventRecord(ctx->ready[slot], main_st));
            RN50_HIP(hipStreamWaitEvent(ctx->side, ctx->ready[slot], 0));
            RN50_TRY(wgrad(A + pl.ws_conv2, ctx->side));
            RN50_HIP(hipEventRecord(ctx->done[slot], ctx->side));
        } else {
            RN50_TRY(wgrad(wsc, stream));
        }
        if (dx_or_null)
            RN50_TRY(conv_bwd_data_pretransposed(&d, dconv, F(pl.wt_arena) + pl.wt[li], dx_or_null, wsc, pl.ws_conv_bytes, main_st));
        ++calls;
        return RN50_OK;
    };

    // Projection branch of a block on its own stream: BN backward (no ReLU) of the shortcut gradient, filter gradient and
    // data gradient, between the event that follows the c layer's BN backward and the join before the block-input
    // gradient is consumed.
    auto proj_bwd_branch = [&](int lp, const float *x_in, const float *dshortcut, hipEvent_t after) -> int {
        const ConvL &l = n.convs[lp];
        const rn50_conv_desc d = desc_of(l, N, dtype_of(lp));
        float *dconv = grouped ? F(pl.dconv_l[lp]) : F(pl.dconv_p);
        RN50_HIP(hipStreamWaitEvent(ctx->side2, after, 0));
        if (a16)
            RN50_TRY(bn_bwd_batchstats_bf16(N, l.k, l.hout, l.hout, RN50_LAYOUT_NHWC, H(F(pl.conv_out[lp])), H(dshortcut), nullptr, nullptr,
                                            nullptr, theta + l.g_off, nullptr, F(pl.mean[lp]), F(pl.invstd[lp]), 0, HW_(dconv), nullptr,
                                            grad + l.g_off, grad + l.b_off, A + pl.ws_bn2, pl.ws_bn_bytes, ctx->side2));
        else
        RN50_TRY(bn_bwd_batchstats(N, l.k, l.hout, l.hout, RN50_LAYOUT_NHWC, F(pl.conv_out[lp]), dshortcut, nullptr, nullptr,
                                   theta + l.g_off, F(pl.mean[lp]), F(pl.invstd[lp]), 0, dconv, nullptr, grad + l.g_off,
                                   grad + l.b_off, A + pl.ws_bn2, pl.ws_bn_bytes, ctx->side2));
        RN50_TRY(conv_bwd_data_pretransposed(&d, dconv, F(pl.wt_arena) + pl.wt[lp], F(pl.gbuf_p), A + pl.ws_conv3, pl.ws_conv_bytes,
                                             ctx->side2));
        RN50_HIP(hipEventRecord(ctx->pjoin, ctx->side2));
        if (grouped) {  // its filter gradient is part of the block's grouped launch, which waits for this BN backward
            RN50_HIP(hipEventRecord(ctx->pbn, ctx->side2));
            return RN50_OK;
        }
        // the filter gradient is needed only at the end of the pass: after the join point
        return conv2d_bwd_weight(&d, x_in, dconv, grad + l.w_off, A + pl.ws_conv3, pl.ws_conv_bytes, ctx->side2);
    };
    // The grouped launch that ends with block b, once every BN-input gradient of its layers is enqueued.
    auto launch_group_after = [&](int b) -> int {
        for (const rn50_ctx::Group &g : ctx->groups) {
            if (g.last_block != b) continue;
            void *st = stream;
            if (ctx->use_side) {
                RN50_HIP(hipEventRecord(ctx->ready[1], main_st));
                RN50_HIP(hipStreamWaitEvent(ctx->side, ctx->ready[1], 0));
                bool has_proj = false;
                for (int li : g.layers) has_proj = has_proj || n.convs[li].block_pos == 4;
                if (has_proj) RN50_HIP(hipStreamWaitEvent(ctx->side, ctx->pbn, 0));
                st = ctx->side;
            }
            RN50_TRY(conv2d_bwd_weight_group(g.host.data(), A + g.dev_off, grad, st));
            if (ctx->use_side) RN50_HIP(hipEventRecord(ctx->gdone, ctx->side));
            group_launched = true;
        }
        return RN50_OK;
    };
    bool pending_join = false;

    for (int b = (int)block_first.size() - 1; b >= 0; --b) {
        const int li = block_first[b];
        const bool proj = li + 3 < L && n.convs[li + 3].block_pos == 4;
        const int nxt = 1 - cur;
        if (pending_join) {  // in2 comes from the projection-branch stream
            RN50_HIP(hipStreamWaitEvent(main_st, ctx->pjoin, 0));
            pending_join = false;
        }
        // c: gradient of the block output is in1 (+ in2); dres = masked gradient = gradient of the shortcut
        RN50_TRY(bn_conv_bwd(li + 2, F(pl.bn_out[li + 1]), in1, in2, 1, setR[nxt], T2, fused_out(li + 1) ? li + 1 : -1));
        if (proj && ctx->use_side) {
            RN50_TRY(proj_bwd_branch(li + 3, block_in[b], setR[nxt], ctx->ready[grouped ? 0 : (calls - 1) % 3]));
            pending_join = true;
        }
        RN50_TRY(bn_conv_bwd(li + 1, F(pl.bn_out[li]), T2, nullptr, 1, nullptr, T2, fused_out(li) ? li : -1));
        RN50_TRY(bn_conv_bwd(li, block_in[b], T2, nullptr, 1, nullptr, setO[nxt]));
        if (proj && ctx->use_side) {
            in2 = F(pl.gbuf_p);
        } else if (proj) {
            // projection branch: BN without ReLU; its input gradient overwrites the shortcut-gradient buffer once consumed
            RN50_TRY(bn_conv_bwd(li + 3, block_in[b], setR[nxt], nullptr, 0, nullptr, T2));
            in2 = T2;
            // T2 is reused by the next block as scratch: move the pair member out of the way by swapping roles
            std::swap(T2, setR[nxt]);
        } else {
            in2 = setR[nxt];
        }
        in1 = setO[nxt];
        cur = nxt;
        if (grouped) RN50_TRY(launch_group_after(b));
    }
    float *dpool = F(pl.gbuf[0]);
    if (pending_join) RN50_HIP(hipStreamWaitEvent(main_st, ctx->pjoin, 0));
    if (a16) RN50_TRY(maxpool3x3s2_bwd_bf16(N, 64, 112, 112, H(in1), H(in2), (const uint8_t *)(A + pl.pool_arg), HW_(dpool), stream));
    else RN50_TRY(maxpool3x3s2_bwd(N, 64, 112, 112, in1, in2, (const uint8_t *)(A + pl.pool_arg), dpool, stream));
    // stem: the gradient with respect to the images is never needed
    RN50_TRY(bn_conv_bwd(0, images, dpool, nullptr, 1, nullptr, nullptr));
    // join: every filter gradient still in flight on the side stream
    if (pending_stem) *pending_stem = nullptr;
    if (ctx->use_side && grouped) {
        if (group_launched) RN50_HIP(hipStreamWaitEvent(main_st, ctx->gdone, 0));
        if (pending_stem) *pending_stem = ctx->done[0];
        else RN50_HIP(hipStreamWaitEvent(main_st, ctx->done[0], 0));
    } else if (ctx->use_side) {
        const int stem_slot = (calls - 1) % 3;
        for (int i = 0; i < 3 && i < calls; ++i) {
            if (pending_stem && i == stem_slot) continue;
            RN50_HIP(hipStreamWaitEvent(main_st, ctx->done[i], 0));
        }
        if (pending_stem) *pending_stem = ctx->done[stem_slot];
        // ... and the projection branch's last filter gradient
        RN50_HIP(hipEventRecord(ctx->pfork, ctx->side2));
        RN50_HIP(hipStreamWaitEvent(main_st, ctx->pfork, 0));
    }
#undef RN50_HIP
    return RN50_OK;
}

extern "C" int rn50_forward_backward(rn50_ctx *ctx, const float *images, const int32_t *labels, const float *theta,
                                     float *grad, float bn_eps, float *loss_out, void *stream)
{
    return forward_backward_impl(ctx, images, labels, theta, grad, bn_eps, loss_out, stream, nullptr);
}

extern "C" int rn50_step(rn50_ctx *ctx, const float *images, const int32_t *labels, float *theta, float *grad, float *delta,
                         float *m, uint16_t *grad16, const rn50_opt_hparams *hp, float bn_eps, float *loss_out, void *stream)
{
    RN50_REQUIRE(ctx && delta && m && grad16 && hp, RN50_EINVAL, "rn50_step: null pointer");
    RN50_REQUIRE(aligned16(delta) && aligned16(m) && aligned16(grad16), RN50_EINVAL, "rn50_step: pointers must be 16-byte aligned");
    hipEvent_t stem_done = nullptr;
    RN50_TRY(forward_backward_impl(ctx, images, labels, theta, grad, bn_eps, loss_out, stream, &stem_done));
    const Net &n = net(ctx->variant);
    const size_t count = n.count;
    const uint8_t *mask = (const uint8_t *)(ctx->arena + ctx->plan.mask_off);
    // Half-precision communication buffer, then the update from it; with one worker the all-reduce between pack and unpack
    // is the identity.  Two buckets: everything behind the stem's three tensors first, while the stem's filter gradient
    // (the last kernel of the backward pass) may still be running on the side stream, then the stem.
    const size_t head = stem_done ? n.convs[1].w_off : 0;  // a multiple of RN50_WD_GROUP and of 8
    RN50_TRY(grad_pack_fp16(count - head, grad + head, grad16 + head, stream));
    RN50_TRY(opt_update(count - head, theta + head, delta + head, m + head, nullptr, grad16 + head, mask + head / RN50_WD_GROUP, hp, stream));
    if (head) {
        if (hipStreamWaitEvent((hipStream_t)stream, stem_done, 0) != hipSuccess) return fail(RN50_EHIP, "rn50_step: event wait failed");
        RN50_TRY(grad_pack_fp16(head, grad, grad16, stream));
        RN50_TRY(opt_update(head, theta, delta, m, nullptr, grad16, mask, hp, stream));
    }
    return RN50_OK;
}
