// Tuning and test switches of the library: one immutable snapshot that every call reads, replaced as a whole by
// rn50_set_option.  The environment is consulted exactly once, when the first snapshot is built; no entry point calls
// getenv afterwards.
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <mutex>

#include "common.h"

namespace rn50 {

static bool parse_plan(const char *v, int out[3])
{
    int a, b, c;
    if (!v || sscanf(v, "%d,%d,%d", &a, &b, &c) != 3) return false;
    if ((a != 64 && a != 128) || (b != 64 && b != 128) || c < 1) return false;
    out[0] = a; out[1] = b; out[2] = c;
    return true;
}

// "op,n,c,h,k,r,stride,pad,bm,bn,split;...": rows that do not parse or do not name a tile shape are skipped
static std::vector<PlanRow> parse_rows(const char *v)
{
    std::vector<PlanRow> rows;
    for (const char *q = v; q && *q;) {
        PlanRow t;
        if (sscanf(q, "%d,%d,%d,%d,%d,%d,%d,%d,%d,%d,%d", &t.op, &t.n, &t.c, &t.h, &t.k, &t.r, &t.stride, &t.pad, &t.bm, &t.bn, &t.split) == 11 &&
            (t.bm == 64 || t.bm == 128) && (t.bn == 64 || t.bn == 128) && t.split >= 1)
            rows.push_back(t);
        q = strchr(q, ';');
        if (q) ++q;
    }
    return rows;
}

// Applies one (name, value) pair to c.  value == nullptr or "" restores the built-in default.
static bool apply_option(Config &c, const char *name, const char *value)
{
    const bool unset = !value || !*value;
    const Config def;
    if (!strcmp(name, "side_stream")) c.side_stream = unset ? def.side_stream : atoi(value) != 0;
    else if (!strcmp(name, "fuse_bn")) c.fuse_bn = unset ? def.fuse_bn : (atoi(value) & 7);
    else if (!strcmp(name, "relu_mask")) c.relu_mask = unset ? def.relu_mask : atoi(value) != 0;
    else if (!strcmp(name, "no_tuned")) c.no_tuned = unset ? false : atoi(value) != 0;
    else if (!strcmp(name, "no_stem_kernel")) c.no_stem_kernel = unset ? false : atoi(value) != 0;
    else if (!strcmp(name, "conv_bn_stats")) c.conv_bn_stats = unset ? def.conv_bn_stats : atoi(value) != 0;
    else if (!strcmp(name, "wgrad_group")) c.wgrad_group = unset ? def.wgrad_group : std::max(0, std::min(64, atoi(value)));
    else if (!strcmp(name, "wgrad_group_stages")) c.wgrad_group_stages = unset ? def.wgrad_group_stages : std::max(2, atoi(value));
    else if (!strcmp(name, "wgrad_group_wgs_per_cu")) c.wgrad_group_wgs_per_cu = unset ? def.wgrad_group_wgs_per_cu : std::max(0, std::min(8, atoi(value)));
    else if (!strcmp(name, "wgrad_group_tile")) {
        int t[3];
        char buf[48];
        snprintf(buf, sizeof buf, "%s,1", unset ? "0,0" : value);
        if (unset) { c.wgrad_group_bm = def.wgrad_group_bm; c.wgrad_group_bn = def.wgrad_group_bn; }
        else if (parse_plan(buf, t)) { c.wgrad_group_bm = t[0]; c.wgrad_group_bn = t[1]; }
        else return false;
    }
    else if (!strcmp(name, "igemm_plan")) {
        c.has_igemm_plan = false;
        if (!unset && !(c.has_igemm_plan = parse_plan(value, c.igemm_plan))) return false;
    } else if (!strcmp(name, "wgrad_plan")) {
        c.has_wgrad_plan = false;
        if (!unset && !(c.has_wgrad_plan = parse_plan(value, c.wgrad_plan))) return false;
    } else if (!strcmp(name, "plan_overrides")) c.overrides = unset ? std::vector<PlanRow>() : parse_rows(value);
    else return false;
    return true;
}

static std::mutex g_mu;
static std::shared_ptr<const Config> g_cfg;

static std::shared_ptr<const Config> from_environment()
{
    static const char *const names[] = {"side_stream", "fuse_bn", "relu_mask", "no_tuned", "no_stem_kernel", "conv_bn_stats", "igemm_plan", "wgrad_plan", "wgrad_group",
                                        "wgrad_group_stages", "wgrad_group_tile", "wgrad_group_wgs_per_cu",
                                        "plan_overrides"};
    auto c = std::make_shared<Config>();
    for (const char *n : names) {
        char var[64] = "RN50_";
        size_t j = strlen(var);
        for (const char *p = n; *p && j + 1 < sizeof var; ++p) var[j++] = (char)(*p >= 'a' && *p <= 'z' ? *p - 32 : *p);
        var[j] = 0;
        const char *v = getenv(var);
        if (v && *v) {
            Config trial = *c;
            if (apply_option(trial, n, v)) *c = trial;  // a value that does not parse leaves the default
        }
    }
    return c;
}

std::shared_ptr<const Config> config()
{
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_cfg) g_cfg = from_environment();
    return g_cfg;
}

}  // namespace rn50

extern "C" int rn50_set_option(const char *name, const char *value_or_null)
{
    using namespace rn50;
    RN50_REQUIRE(name, RN50_EINVAL, "rn50_set_option: null name");
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_cfg) g_cfg = from_environment();
    auto next = std::make_shared<Config>(*g_cfg);
    if (!apply_option(*next, name, value_or_null))
        return fail(RN50_EINVAL, "rn50_set_option: unknown option or malformed value (%s = %s)", name, value_or_null ? value_or_null : "(null)");
    g_cfg = next;
    return RN50_OK;
}
