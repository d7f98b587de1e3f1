// Filter gradients of several convolution layers in one launch: host side (plan blob, launches).
//
// A plan is a blob the caller keeps twice, in host memory and (the same bytes) in device memory: a header, one WgradJob per
// layer for the kernel that forms the partial sums and one ReduceJob per layer for the kernel that adds them in order.
// Planning touches no device memory; launching reads the header from the host copy and hands the device copy to the kernels.
#include <string.h>

#include <algorithm>

#include "conv_kernels.h"

namespace rn50 {

struct GroupHeader {
    uint32_t magic;
    int njobs, items, reduce_blocks, bm, bn;
    size_t bytes, ws_bytes;
    const void *ws;       // the workspace the partials of this plan live in
    int lds_pad;          // unused LDS added to every workgroup, so that no more than the wanted number share a CU
    int reserved[3];
};
static_assert(sizeof(GroupHeader) == 64, "header of a grouped filter-gradient plan");
constexpr uint32_t kGroupMagic = 0x47573035u;

static size_t blob_bytes(int count) { return sizeof(GroupHeader) + (size_t)count * (sizeof(WgradJob) + sizeof(ReduceJob)); }

struct JobPlan { int P, Q, split, cps; size_t part_floats; };

// Pixel ranges of about `stages` LDS stages each (a work item then lasts about as long whatever its layer).
static JobPlan plan_job(const rn50_conv_desc *d, int stages)
{
    JobPlan j;
    j.P = (d->h + 2 * d->pad - d->r) / d->stride + 1;
    j.Q = (d->w + 2 * d->pad - d->s) / d->stride + 1;
    const int pchunks = ceil_div((long)d->n * j.P * j.Q, kBK);
    const int want = std::max(1, (pchunks + stages / 2) / stages);
    j.cps = ceil_div(pchunks, want);
    if (j.cps < pchunks) j.cps += j.cps & 1;  // two stages per trip of the kernel's loop: an odd range would end with a stage of zeros
    j.split = ceil_div(pchunks, j.cps);
    j.part_floats = ((size_t)j.split * d->k * d->r * d->s * d->c + 63) / 64 * 64;
    return j;
}

static int check_items(const char *who, int count, const rn50_wgrad_group_item *items)
{
    RN50_REQUIRE(count > 0 && count <= 4096 && items, RN50_EINVAL, "%s: between 1 and 4096 layers", who);
    for (int i = 0; i < count; ++i) {
        const rn50_conv_desc *d = &items[i].desc;
        if (int rc = conv_check(who, d)) return rc;
        RN50_REQUIRE(d->in_dtype == RN50_DTYPE_F32, RN50_EUNSUPPORTED, "%s: fp32 operands only", who);
        RN50_REQUIRE(d->c % 4 == 0 && d->k % 4 == 0, RN50_EUNSUPPORTED, "%s: C and K must be multiples of 4", who);
    }
    return RN50_OK;
}

size_t wgrad_group_table_bytes(int count) { return count > 0 && count <= 4096 ? blob_bytes(count) : 0; }

size_t wgrad_group_ws_bytes(int count, const rn50_wgrad_group_item *items, int stages)
{
    if (check_items("rn50_wgrad_group_workspace_bytes", count, items) != RN50_OK) return 0;
    size_t floats = 0;
    for (int i = 0; i < count; ++i) floats += plan_job(&items[i].desc, stages).part_floats;
    return floats * sizeof(float);
}

int wgrad_group_plan(int count, const rn50_wgrad_group_item *items, void *ws, size_t ws_bytes, void *table_host, size_t table_bytes,
                     int stages, int bm, int bn, int wgs_per_cu)
{
    if (int rc = check_items("rn50_wgrad_group_plan", count, items)) return rc;
    RN50_REQUIRE(table_host && table_bytes >= blob_bytes(count), RN50_EINVAL, "rn50_wgrad_group_plan: table buffer too small");
    RN50_REQUIRE(ws && aligned16(ws), RN50_EINVAL, "rn50_wgrad_group_plan: the workspace must be non-null and 16-byte aligned");
    GroupHeader h{};
    h.magic = kGroupMagic;
    h.njobs = count;
    h.bm = bm;
    h.bn = bn;
    h.bytes = blob_bytes(count);
    h.ws = ws;
    {
        // a CU has 160 KB of LDS: workgroups that each take more than 160/(k+1) KB are at most k to a CU, which leaves wave slots
        // and registers to the kernels of other streams; a launch may ask for up to 64 KB
        const int own = kBK * (bm + 4 + bn + 4) * (int)sizeof(float);
        const int want = wgs_per_cu > 0 ? (160 * 1024) / (wgs_per_cu + 1) + 256 : 0;
        h.lds_pad = std::max(0, std::min(want, 64 * 1024) - own) / 256 * 256;
    }
    char *blob = (char *)table_host;
    WgradJob *jobs = reinterpret_cast<WgradJob *>(blob + sizeof(GroupHeader));
    ReduceJob *red = reinterpret_cast<ReduceJob *>(blob + sizeof(GroupHeader) + (size_t)count * sizeof(WgradJob));
    memset(blob, 0, h.bytes);
    size_t floats = 0;
    long items_total = 0, blocks = 0;
    for (int i = 0; i < count; ++i) {
        const rn50_wgrad_group_item &it = items[i];
        const rn50_conv_desc *d = &it.desc;
        RN50_REQUIRE(it.x && it.dy && aligned16(it.x) && aligned16(it.dy), RN50_EINVAL,
                     "rn50_wgrad_group_plan: x and dy must be non-null and 16-byte aligned (layer %d)", i);
        RN50_REQUIRE(!it.in_scale == !it.in_shift && aligned16(it.in_scale) && aligned16(it.in_shift), RN50_EINVAL,
                     "rn50_wgrad_group_plan: scale and shift come together, 16-byte aligned (layer %d)", i);
        RN50_REQUIRE(it.dw_offset % 4 == 0, RN50_EINVAL, "rn50_wgrad_group_plan: gradient offsets must be multiples of 4 elements (layer %d)", i);
        const JobPlan jp = plan_job(d, stages);
        WgradP &p = jobs[i].p;
        p.dy = it.dy; p.x = it.x; p.in_scale = it.in_scale; p.in_shift = it.in_shift;
        p.out = (float *)ws + floats;
        wgrad_fill(p, d, jp.P, jp.Q, h.bm, h.bn, jp.split, jp.cps);
        jobs[i].item_begin = (int)items_total;
        items_total += (long)p.tiles_k * p.tiles_j * jp.split;
        red[i].count4 = p.split_stride / 4;
        red[i].stride = p.split_stride;
        red[i].part = p.out;
        red[i].out_off = (long)it.dw_offset;
        red[i].split = jp.split;
        red[i].block_begin = (int)blocks;
        blocks += ceil_div(red[i].count4, 64);
        floats += jp.part_floats;
        RN50_REQUIRE(items_total < (1L << 30) && blocks < (1L << 30), RN50_EUNSUPPORTED, "rn50_wgrad_group_plan: too many work items");
    }
    h.items = (int)items_total;
    h.reduce_blocks = (int)blocks;
    h.ws_bytes = floats * sizeof(float);
    RN50_REQUIRE(ws_bytes >= h.ws_bytes, RN50_EWORKSPACE, "rn50_wgrad_group_plan: workspace too small (%zu < %zu)", ws_bytes, h.ws_bytes);
    memcpy(blob, &h, sizeof h);
    return RN50_OK;
}

}  // namespace rn50

using namespace rn50;

extern "C" size_t rn50_wgrad_group_table_bytes(int count) { return wgrad_group_table_bytes(count); }

extern "C" size_t rn50_wgrad_group_workspace_bytes(int count, const rn50_wgrad_group_item *items)
{
    return wgrad_group_ws_bytes(count, items, config()->wgrad_group_stages);
}

extern "C" int rn50_wgrad_group_plan(int count, const rn50_wgrad_group_item *items, void *ws, size_t ws_bytes, void *table_host,
                                     size_t table_bytes)
{
    const std::shared_ptr<const Config> cfg = config();
    return wgrad_group_plan(count, items, ws, ws_bytes, table_host, table_bytes, cfg->wgrad_group_stages, cfg->wgrad_group_bm,
                            cfg->wgrad_group_bn, cfg->wgrad_group_wgs_per_cu);
}

extern "C" int conv2d_bwd_weight_group(const void *table_host, const void *table_device, float *dw_base, void *stream)
{
    RN50_REQUIRE(table_host && table_device && dw_base, RN50_EINVAL, "conv2d_bwd_weight_group: null pointer");
    RN50_REQUIRE(aligned16(table_device) && aligned16(dw_base), RN50_EINVAL, "conv2d_bwd_weight_group: pointers must be 16-byte aligned");
    GroupHeader h;
    memcpy(&h, table_host, sizeof h);
    RN50_REQUIRE(h.magic == kGroupMagic && h.njobs > 0 && h.bytes == blob_bytes(h.njobs) && h.items > 0 && h.reduce_blocks > 0,
                 RN50_EINVAL, "conv2d_bwd_weight_group: not a plan written by rn50_wgrad_group_plan");
    RN50_REQUIRE(h.lds_pad >= 0 && h.lds_pad <= 64 * 1024, RN50_EINVAL, "conv2d_bwd_weight_group: damaged plan");
    const char *dev = (const char *)table_device;
    const WgradJob *jobs = reinterpret_cast<const WgradJob *>(dev + sizeof(GroupHeader));
    const ReduceJob *red = reinterpret_cast<const ReduceJob *>(dev + sizeof(GroupHeader) + (size_t)h.njobs * sizeof(WgradJob));
    hipStream_t st = (hipStream_t)stream;
    const dim3 grid(h.items), block(kConvThreads);
    if (h.bm == 128 && h.bn == 128) hipLaunchKernelGGL((wgrad_group_kernel<128, 128>), grid, block, h.lds_pad, st, jobs, h.njobs);
    else if (h.bm == 128) hipLaunchKernelGGL((wgrad_group_kernel<128, 64>), grid, block, h.lds_pad, st, jobs, h.njobs);
    else if (h.bn == 128) hipLaunchKernelGGL((wgrad_group_kernel<64, 128>), grid, block, h.lds_pad, st, jobs, h.njobs);
    else if (h.bm == 64 && h.bn == 64) hipLaunchKernelGGL((wgrad_group_kernel<64, 64>), grid, block, h.lds_pad, st, jobs, h.njobs);
    else return fail(RN50_EINVAL, "conv2d_bwd_weight_group: plan names an unknown tile");
    hipLaunchKernelGGL(splitk_reduce_group_kernel, dim3(h.reduce_blocks), dim3(256), 0, st, red, h.njobs, dw_base);
    return launch_status("conv2d_bwd_weight_group");
}
