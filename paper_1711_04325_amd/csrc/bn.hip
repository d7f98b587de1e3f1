// Batch normalization with the statistics of the current minibatch only (Section 2, "Batch
// Normalization without Moving Averages"), NHWC, fp32, with the residual add and ReLU of the
// bottleneck block fused in.  Bandwidth-bound: the tensor is an [M][C] matrix (M = N*H*W rows,
// channels contiguous), a workgroup owns a band of rows and up to 1024 channels, every access is a
// 16-byte load or store of four neighbouring channels.
//
// Forward  : (1) per-band (mean, M2) by shifted sums, merged with Chan's formula inside the workgroup
//            (2) one small kernel merges the bands in a fixed order -> mean, invstd, scale, shift
//            (3) y = x*scale + shift [+ residual] [ReLU]
// Backward : (1) per-band sums of dz and dz*xhat  (2) fixed-order merge -> dgamma, dbeta and the three
//            coefficients of dx  (3) dx = a*dz + b*x + c per channel.
// All merges run in a fixed order, so results are bit-identical from call to call.
#include <mutex>

#include "common.h"

namespace rn50 {

constexpr int kBnThreads = 256;

// Scratch of bn_fwd_batchstats_static, the entry point for callers that cannot allocate: band partials and per-channel
// coefficients of ONE call.  Every GPU the library runs on holds its own copy until the process ends.  In host code the
// array's name is only a handle for hipGetSymbolAddress: kernels get the address that call returns, per device.
static __device__ __align__(256) unsigned char scratch[RN50_BN_STATIC_SCRATCH_BYTES];

struct BnGeom {
    int M, C, C4;
    int cols;        // float4 columns per workgroup (power of two, <= 256)
    int row_lanes;   // 256 / cols
    int col_blocks;  // grid.y
    int bands;       // grid.x
    int rows_per_band;
};

static BnGeom bn_geom(int n, int c, int h, int w)
{
    BnGeom g;
    g.M = n * h * w;
    g.C = c;
    g.C4 = c / 4;
    int cols = 1;
    while (cols < g.C4 && cols < kBnThreads) cols <<= 1;
    g.cols = cols;
    g.row_lanes = kBnThreads / cols;
    g.col_blocks = ceil_div(g.C4, cols);
    // aim at ~2048 workgroups, at least 4 rows per thread, at most 512 bands
    int bands = 2048 / g.col_blocks;
    const int max_bands = ceil_div(g.M, (long)g.row_lanes * 4);
    if (bands > max_bands) bands = max_bands;
    if (bands > 512) bands = 512;
    if (bands < 1) bands = 1;
    g.rows_per_band = ceil_div(g.M, bands);
    g.bands = ceil_div(g.M, g.rows_per_band);
    return g;
}

// The element-wise passes have no partial results to merge and take a finer cut of the rows than the reductions: up to 8192
// workgroups of at least four rows per thread (a 100 MB tensor in 512 workgroups leaves the memory system under-subscribed).
static BnGeom bn_apply_geom(BnGeom g)
{
    int bands = 8192 / g.col_blocks;
    const int most = ceil_div(g.M, (long)g.row_lanes * 4);
    if (bands > most) bands = most;
    if (bands < 1) bands = 1;
    g.rows_per_band = ceil_div(g.M, bands);
    g.bands = ceil_div(g.M, g.rows_per_band);
    return g;
}

// workspace: [2][bands][C] partials, then [4][C] per-channel coefficients
static size_t bn_ws_floats(const BnGeom &g) { return (size_t)2 * g.bands * g.C + (size_t)4 * g.C; }

__device__ inline float4 f4(float v) { return make_float4(v, v, v, v); }
__device__ inline float4 operator+(float4 a, float4 b) { return make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w); }
__device__ inline float4 operator-(float4 a, float4 b) { return make_float4(a.x - b.x, a.y - b.y, a.z - b.z, a.w - b.w); }
__device__ inline float4 operator*(float4 a, float4 b) { return make_float4(a.x * b.x, a.y * b.y, a.z * b.z, a.w * b.w); }
__device__ inline float4 fma4(float4 a, float4 b, float4 c)
{
    return make_float4(fmaf(a.x, b.x, c.x), fmaf(a.y, b.y, c.y), fmaf(a.z, b.z, c.z), fmaf(a.w, b.w, c.w));
}

// A thread's rows r, r+step, ... < r1 in groups of kRowGroup: load(row, slot) for the whole group first, so that the
// group's loads are in flight together, then use(row, slot) in row order (the order of a plain loop, so sums keep their
// value).  A thread with one row in flight waits a full memory round trip per row, which the few resident workgroups of a
// reduction do not hide; groups of two measured best inside the training step (groups of three and four are equal on a
// kernel alone and slow the step down, with or without a predicated last group).
constexpr int kRowGroup = 2;
template <int GROUP, class Load, class Use>
__device__ inline void for_rows(int r, int r1, int step, Load load, Use use)
{
    for (; r + (GROUP - 1) * step < r1; r += GROUP * step) {
#pragma unroll
        for (int u = 0; u < GROUP; ++u) load(r + u * step, u);
#pragma unroll
        for (int u = 0; u < GROUP; ++u) use(r + u * step, u);
    }
    for (; r < r1; r += step) {
        load(r, 0);
        use(r, 0);
    }
}

// ---- merging the row lanes of a workgroup --------------------------------------------------------------------------------
// A workgroup is `cols` float4 columns x 256/cols row lanes, thread = lane_row*cols + column.  When cols < 64 several row
// lanes share a wavefront and are merged with lane shuffles (a butterfly over the lane bits above the column bits; both
// partners form the merge of (lower lane, upper lane) in that operand order, so they hold the same bits); what is left, at
// most four groups, goes through LDS once and is merged in group order by the threads of row lane 0.  The order is fixed
// by the geometry alone.
__device__ inline float4 shfl_xor4(float4 v, int off)
{
    return make_float4(__shfl_xor(v.x, off, 64), __shfl_xor(v.y, off, 64), __shfl_xor(v.z, off, 64), __shfl_xor(v.w, off, 64));
}
__device__ inline int row_groups(int cols, int row_lanes) { return cols < 64 ? kBnThreads / 64 : row_lanes; }

// Chan et al.: (mean, M2, count) of the union of two sample sets A and B
__device__ inline void chan_merge(float4 &mean, float4 &m2, float &n, float4 mean_b, float4 m2_b, float nb)
{
    if (nb > 0.f) {
        const float nt = n + nb;
        const float4 d = mean_b - mean;
        mean = fma4(d, f4(nb / nt), mean);
        m2 = m2 + m2_b + d * d * f4(n * nb / nt);
        n = nt;
    }
}

// sums a and b over the row lanes; valid afterwards in the threads of row lane 0 (tid < cols)
__device__ inline void merge_rows_sum(float4 &a, float4 &b, int cols, int row_lanes, float4 *s_a, float4 *s_b)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int off = cols; off < 64; off <<= 1) {
        const float4 pa = shfl_xor4(a, off), pb = shfl_xor4(b, off);
        const bool lower = (lane & off) == 0;
        a = lower ? a + pa : pa + a;
        b = lower ? b + pb : pb + b;
    }
    const int groups = row_groups(cols, row_lanes);
    if (groups == 1) return;
    if (cols < 64) {
        if (lane < cols) {
            s_a[wave * cols + lane] = a;
            s_b[wave * cols + lane] = b;
        }
    } else {
        s_a[tid] = a;
        s_b[tid] = b;
    }
    __syncthreads();
    if (tid < cols) {
        a = s_a[tid];
        b = s_b[tid];
        for (int g = 1; g < groups; ++g) {
            a = a + s_a[g * cols + tid];
            b = b + s_b[g * cols + tid];
        }
    }
}

// ---- forward, pass 1: per-band mean and M2 = sum (x-mean)^2 -------------------------------------
template <class T>
__global__ __launch_bounds__(kBnThreads) void bn_stats_kernel(BnGeom g, const T *__restrict__ x,
                                                              float *__restrict__ part_mean, float *__restrict__ part_m2)
{
    __shared__ float4 s_mean[kBnThreads];
    __shared__ float4 s_m2[kBnThreads];
    __shared__ float s_n[kBnThreads];
    const int tid = threadIdx.x;
    const int col = blockIdx.y * g.cols + tid % g.cols;
    const int lane_row = tid / g.cols;
    const int r0 = blockIdx.x * g.rows_per_band;
    const int r1 = min(g.M, r0 + g.rows_per_band);
    const bool active = col < g.C4;
    float4 mean = f4(0.f), m2 = f4(0.f);
    float cnt = 0.f;
    if (active && r0 + lane_row < r1) {
        // sums of (x - shift) with shift = the first sample: no catastrophic cancellation in M2
        const float4 shift = ld4(x, (size_t)(r0 + lane_row) * g.C4 + col);
        float4 s = f4(0.f), ss = f4(0.f);
        float4 xv[kRowGroup];
        for_rows<kRowGroup>(
            r0 + lane_row, r1, g.row_lanes, [&](int r, int u) { xv[u] = ld4(x, (size_t)r * g.C4 + col); },
            [&](int, int u) {
                const float4 d = xv[u] - shift;
                s = s + d;
                ss = fma4(d, d, ss);
                cnt += 1.f;
            });
        const float inv = 1.f / cnt;
        mean = fma4(s, f4(inv), shift);
        m2 = ss - s * s * f4(inv);
    }
    // Chan et al. merge across the row lanes: inside a wavefront by shuffles, then the (at most four) groups through LDS
    const int lane = tid & 63, wave = tid >> 6;
    for (int off = g.cols; off < 64; off <<= 1) {
        const float4 pm = shfl_xor4(mean, off), p2 = shfl_xor4(m2, off);
        const float pn = __shfl_xor(cnt, off, 64);
        if ((lane & off) == 0) {
            chan_merge(mean, m2, cnt, pm, p2, pn);
        } else {  // the same merge(lower, upper) as the partner forms
            float4 am = pm, a2 = p2;
            float an = pn;
            chan_merge(am, a2, an, mean, m2, cnt);
            mean = am; m2 = a2; cnt = an;
        }
    }
    const int groups = row_groups(g.cols, g.row_lanes);
    if (groups > 1) {
        if (g.cols < 64) {
            if (lane < g.cols) {
                s_mean[wave * g.cols + lane] = mean;
                s_m2[wave * g.cols + lane] = m2;
                s_n[wave * g.cols + lane] = cnt;
            }
        } else {
            s_mean[tid] = mean;
            s_m2[tid] = m2;
            s_n[tid] = cnt;
        }
        __syncthreads();
        if (tid < g.cols) {
            mean = s_mean[tid]; m2 = s_m2[tid]; cnt = s_n[tid];
            for (int q = 1; q < groups; ++q) chan_merge(mean, m2, cnt, s_mean[q * g.cols + tid], s_m2[q * g.cols + tid], s_n[q * g.cols + tid]);
        }
    }
    if (lane_row == 0 && active) {
        reinterpret_cast<float4 *>(part_mean + (size_t)blockIdx.x * g.C)[col] = mean;
        reinterpret_cast<float4 *>(part_m2 + (size_t)blockIdx.x * g.C)[col] = m2;
    }
}

// ---- forward, pass 2: merge the bands; workgroup = 4 channels x 64 slices of the band range ------------------
// Thread = (slice, channel) with the channel in the two low lane bits: the four channels of a slice are one 16-byte access.
// Each thread merges its slice of bands in increasing order; the 16 slices of a wavefront are merged by a shuffle butterfly
// (both partners form merge(lower lane, upper lane)), the four wavefronts through LDS in wavefront order: a fixed order,
// independent of scheduling.
constexpr int kFinCh = 4, kFinSl = 64;

// Eight workgroups of four channels share every 128-byte line of the partials: xcd_contiguous() hands each XCD a contiguous
// range of channel groups so that a line is fetched into one L2, not eight.

__device__ inline void chan_merge1(float &mean, float &m2, float &n, float mean_b, float m2_b, float nb)
{
    if (nb > 0.f) {
        const float nt = n + nb;
        const float d = mean_b - mean;
        mean = fmaf(d, nb / nt, mean);
        m2 = m2 + m2_b + d * d * (n * nb / nt);
        n = nt;
    }
}

// SL slices per workgroup: 64 (four wavefronts), or 256 (sixteen) when there are many partials per channel, as after a
// convolution that left one per 64-row tile of a large tensor: a thread's serial run of merges is a quarter as long.
template <int SL>
__global__ __launch_bounds__(kFinCh * SL) void bn_stats_finalize_kernel(
    BnGeom g, const float *__restrict__ part_mean, const float *__restrict__ part_m2, const float *__restrict__ gamma,
    const float *__restrict__ beta, float eps, float *__restrict__ save_mean, float *__restrict__ save_invstd,
    float *__restrict__ scale, float *__restrict__ shift)
{
    constexpr int NW = kFinCh * SL / 64;  // wavefronts
    __shared__ float s_mean[NW][kFinCh], s_m2[NW][kFinCh], s_n[NW][kFinCh];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int cl = threadIdx.x % kFinCh, sl = threadIdx.x / kFinCh;
    const int c = xcd_contiguous(blockIdx.x, gridDim.x) * kFinCh + cl;
    const int per = (g.bands + SL - 1) / SL;
    const int b0 = sl * per, b1 = min(g.bands, b0 + per);
    float mean = 0.f, m2 = 0.f, na = 0.f;
    if (c < g.C) {
#pragma unroll 4
        for (int b = b0; b < b1; ++b) {
            const float nb = (float)(min(g.M, (b + 1) * g.rows_per_band) - b * g.rows_per_band);
            const float nt = na + nb;
            const float d = part_mean[(size_t)b * g.C + c] - mean;
            mean = fmaf(d, nb / nt, mean);
            m2 = m2 + part_m2[(size_t)b * g.C + c] + d * d * (na * nb / nt);
            na = nt;
        }
    }
    for (int off = kFinCh; off < 64; off <<= 1) {
        const float pm = __shfl_xor(mean, off, 64), p2 = __shfl_xor(m2, off, 64), pn = __shfl_xor(na, off, 64);
        if ((lane & off) == 0) {
            chan_merge1(mean, m2, na, pm, p2, pn);
        } else {
            float am = pm, a2 = p2, an = pn;
            chan_merge1(am, a2, an, mean, m2, na);
            mean = am; m2 = a2; na = an;
        }
    }
    if (lane < kFinCh) {
        s_mean[wave][lane] = mean;
        s_m2[wave][lane] = m2;
        s_n[wave][lane] = na;
    }
    __syncthreads();
    if (threadIdx.x < kFinCh && c < g.C) {
        for (int w = 1; w < NW; ++w) chan_merge1(mean, m2, na, s_mean[w][cl], s_m2[w][cl], s_n[w][cl]);
        const float var = m2 / (float)g.M;
        const float invstd = 1.0f / sqrtf(var + eps);
        save_mean[c] = mean;
        save_invstd[c] = invstd;
        const float a = gamma[c] * invstd;
        scale[c] = a;
        shift[c] = fmaf(-mean, a, beta[c]);
    }
}

// ---- forward, pass 3: normalise ----------------------------------------------------------------------
template <class T, bool RES, bool RELU>
__global__ __launch_bounds__(kBnThreads) void bn_apply_kernel(BnGeom g, const T *__restrict__ x,
                                                              const float *__restrict__ scale, const float *__restrict__ shift,
                                                              const T *__restrict__ residual, T *__restrict__ y,
                                                              uint8_t *__restrict__ relu_mask)
{
    const int tid = threadIdx.x;
    const int col = blockIdx.y * g.cols + tid % g.cols;
    if (col >= g.C4) return;
    const int lane_row = tid / g.cols;
    const int r0 = blockIdx.x * g.rows_per_band;
    const int r1 = min(g.M, r0 + g.rows_per_band);
    const float4 a = reinterpret_cast<const float4 *>(scale)[col];
    const float4 b = reinterpret_cast<const float4 *>(shift)[col];
    float4 xv[kRowGroup], rv[kRowGroup];
    for_rows<kRowGroup>(
        r0 + lane_row, r1, g.row_lanes,
        [&](int r, int u) {
            const size_t o = (size_t)r * g.C4 + col;
            xv[u] = ld4(x, o);
            if (RES) rv[u] = ld4(residual, o);
        },
        [&](int r, int u) {
            const size_t o = (size_t)r * g.C4 + col;
            float4 v = fma4(xv[u], a, b);
            if (RES) v = v + rv[u];
            if (RELU) v = make_float4(fmaxf(v.x, 0.f), fmaxf(v.y, 0.f), fmaxf(v.z, 0.f), fmaxf(v.w, 0.f));
            st4(y, o, v);
            // one byte per four channels, bit e = [y > 0] of channel 4*col + e, of y as stored: what the backward pass needs of y
            if (RELU && relu_mask) {
                const float4 w = as_stored(y, v);
                relu_mask[o] = (uint8_t)((w.x > 0.f) | ((w.y > 0.f) << 1) | ((w.z > 0.f) << 2) | ((w.w > 0.f) << 3));
            }
        });
}

// ---- validation side: given statistics ---------------------------------------------------------------
// scale = gamma * invstd, shift = beta - mean * scale: the same two expressions as at the end of the training forward
__global__ __launch_bounds__(256) void bn_scale_shift_kernel(int C, const float *__restrict__ gamma, const float *__restrict__ beta,
                                                             const float *__restrict__ mean, const float *__restrict__ invstd,
                                                             float *__restrict__ scale, float *__restrict__ shift)
{
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= C) return;
    const float a = gamma[c] * invstd[c];
    scale[c] = a;
    shift[c] = fmaf(-mean[c], a, beta[c]);
}

// mean_out = average of the sets' means; invstd_out = 1/sqrt(average of the sets' variances + eps), the variance of a
// set recovered from its saved invstd.  Sets are added in index order.
__global__ __launch_bounds__(256) void bn_stats_average_kernel(int C, int n_sets, const float *__restrict__ means,
                                                               const float *__restrict__ invstds, float eps,
                                                               float *__restrict__ mean_out, float *__restrict__ invstd_out)
{
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= C) return;
    float sm = 0.f, sv = 0.f;
    for (int i = 0; i < n_sets; ++i) {
        const float is = invstds[(size_t)i * C + c];
        sm += means[(size_t)i * C + c];
        sv += 1.0f / (is * is) - eps;
    }
    mean_out[c] = sm / (float)n_sets;
    invstd_out[c] = 1.0f / sqrtf(fmaxf(sv / (float)n_sets, 0.f) + eps);
}

// ---- backward --------------------------------------------------------------------------------------
// mask: when non-null the ReLU mask comes from one byte per four channels (bit e = [y > 0]) instead of y itself
// The operands of dz = (dy [+ dy2]) * [y > 0] for one float4: loaded first (DzRaw), combined later, so that several rows'
// loads can be in flight before the first is used.
struct DzRaw {
    float4 d, d2, yy;
    unsigned b;
};
template <class T, bool RELU, bool DY2>
__device__ inline void load_dz_raw(DzRaw &q, const T *__restrict__ dy, const T *__restrict__ dy2, const T *__restrict__ y,
                                   const uint8_t *__restrict__ mask, size_t o)
{
    q.d = ld4(dy, o);
    if (DY2) q.d2 = ld4(dy2, o);
    if (RELU) {
        if (mask) q.b = mask[o];
        else q.yy = ld4(y, o);
    }
}
template <bool RELU, bool DY2>
__device__ inline float4 finish_dz(const DzRaw &q, bool from_mask)
{
    float4 d = q.d;
    if (DY2) d = d + q.d2;
    if (RELU) {
        if (from_mask) {
            d.x = (q.b & 1u) ? d.x : 0.f;
            d.y = (q.b & 2u) ? d.y : 0.f;
            d.z = (q.b & 4u) ? d.z : 0.f;
            d.w = (q.b & 8u) ? d.w : 0.f;
        } else {
            d.x = q.yy.x > 0.f ? d.x : 0.f;
            d.y = q.yy.y > 0.f ? d.y : 0.f;
            d.z = q.yy.z > 0.f ? d.z : 0.f;
            d.w = q.yy.w > 0.f ? d.w : 0.f;
        }
    }
    return d;
}

// pass 1: per-band sums of dz and dz*xhat; optionally stores dz (the gradient of the residual input)
template <class T, bool RELU, bool DY2, bool WRITE_DZ>
__global__ __launch_bounds__(kBnThreads) void bn_bwd_reduce_kernel(BnGeom g, const T *__restrict__ x,
                                                                   const T *__restrict__ dy, const T *__restrict__ dy2,
                                                                   const T *__restrict__ y, const uint8_t *__restrict__ mask,
                                                                   const float *__restrict__ save_mean,
                                                                   const float *__restrict__ save_invstd, T *__restrict__ dz_out,
                                                                   float *__restrict__ part_db, float *__restrict__ part_dg)
{
    main_chain_priority();  // these run beside the filter gradients of the layer before (see igemm_kernel)
    __shared__ float4 s_db[kBnThreads];
    __shared__ float4 s_dg[kBnThreads];
    const int tid = threadIdx.x;
    const int col = blockIdx.y * g.cols + tid % g.cols;
    const int lane_row = tid / g.cols;
    const int r0 = blockIdx.x * g.rows_per_band;
    const int r1 = min(g.M, r0 + g.rows_per_band);
    const bool active = col < g.C4;
    float4 db = f4(0.f), dg = f4(0.f);
    if (active) {
        const float4 mean = reinterpret_cast<const float4 *>(save_mean)[col];
        const float4 inv = reinterpret_cast<const float4 *>(save_invstd)[col];
        DzRaw q[kRowGroup];
        float4 xv[kRowGroup];
        for_rows<kRowGroup>(
            r0 + lane_row, r1, g.row_lanes,
            [&](int r, int u) {
                const size_t o = (size_t)r * g.C4 + col;
                load_dz_raw<T, RELU, DY2>(q[u], dy, dy2, y, mask, o);
                xv[u] = ld4(x, o);
            },
            [&](int r, int u) {
                float4 dz = finish_dz<RELU, DY2>(q[u], mask != nullptr);
                // a stored dz is what the third pass and the shortcut branch read: the sums use the stored value too
                if (WRITE_DZ) dz = as_stored(dz_out, dz);
                const float4 xhat = (xv[u] - mean) * inv;
                db = db + dz;
                dg = fma4(dz, xhat, dg);
                if (WRITE_DZ) st4(dz_out, (size_t)r * g.C4 + col, dz);
            });
    }
    merge_rows_sum(db, dg, g.cols, g.row_lanes, s_db, s_dg);
    if (lane_row == 0 && active) {
        reinterpret_cast<float4 *>(part_db + (size_t)blockIdx.x * g.C)[col] = db;
        reinterpret_cast<float4 *>(part_dg + (size_t)blockIdx.x * g.C)[col] = dg;
    }
}

// pass 2: dgamma, dbeta and the coefficients of dx = ca*dz + cb*x + cc (same fixed-order merge)
__global__ __launch_bounds__(kFinCh * kFinSl) void bn_bwd_finalize_kernel(
    BnGeom g, const float *__restrict__ part_db, const float *__restrict__ part_dg, const float *__restrict__ gamma,
    const float *__restrict__ save_mean, const float *__restrict__ save_invstd, float *__restrict__ dgamma,
    float *__restrict__ dbeta, float *__restrict__ ca, float *__restrict__ cb, float *__restrict__ cc)
{
    main_chain_priority();  // these run beside the filter gradients of the layer before (see igemm_kernel)
    __shared__ float s_db[4][kFinCh], s_dg[4][kFinCh];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int cl = threadIdx.x % kFinCh, sl = threadIdx.x / kFinCh;
    const int c = xcd_contiguous(blockIdx.x, gridDim.x) * kFinCh + cl;
    const int per = (g.bands + kFinSl - 1) / kFinSl;
    const int b0 = sl * per, b1 = min(g.bands, b0 + per);
    float db = 0.f, dg = 0.f;
    if (c < g.C) {
#pragma unroll 4
        for (int b = b0; b < b1; ++b) {
            db += part_db[(size_t)b * g.C + c];
            dg += part_dg[(size_t)b * g.C + c];
        }
    }
    for (int off = kFinCh; off < 64; off <<= 1) {
        const float pb = __shfl_xor(db, off, 64), pg = __shfl_xor(dg, off, 64);
        const bool lower = (lane & off) == 0;
        db = lower ? db + pb : pb + db;
        dg = lower ? dg + pg : pg + dg;
    }
    if (lane < kFinCh) {
        s_db[wave][lane] = db;
        s_dg[wave][lane] = dg;
    }
    __syncthreads();
    if (threadIdx.x < kFinCh && c < g.C) {
        for (int w = 1; w < 4; ++w) {
            db += s_db[w][cl];
            dg += s_dg[w][cl];
        }
        dgamma[c] = dg;
        dbeta[c] = db;
        // dx = gamma*inv*(dz - db/M - xhat*dg/M),  xhat = (x-mean)*inv
        const float inv = save_invstd[c], mean = save_mean[c];
        const float a = gamma[c] * inv;
        const float invM = 1.0f / (float)g.M;
        const float bx = -a * inv * dg * invM;
        ca[c] = a;
        cb[c] = bx;
        cc[c] = fmaf(-bx, mean, -a * db * invM);
    }
}

// pass 3: dx.  DZ_IN: read dz stored by pass 1 instead of rebuilding it from dy, dy2, y.
template <class T, bool RELU, bool DY2, bool DZ_IN>
__global__ __launch_bounds__(kBnThreads) void bn_bwd_apply_kernel(BnGeom g, const T *__restrict__ x,
                                                                  const T *__restrict__ dy, const T *__restrict__ dy2,
                                                                  const T *__restrict__ y, const uint8_t *__restrict__ mask,
                                                                  const float *__restrict__ ca,
                                                                  const float *__restrict__ cb, const float *__restrict__ cc,
                                                                  T *__restrict__ dx)
{
    main_chain_priority();  // these run beside the filter gradients of the layer before (see igemm_kernel)
    const int tid = threadIdx.x;
    const int col = blockIdx.y * g.cols + tid % g.cols;
    if (col >= g.C4) return;
    const int lane_row = tid / g.cols;
    const int r0 = blockIdx.x * g.rows_per_band;
    const int r1 = min(g.M, r0 + g.rows_per_band);
    const float4 a = reinterpret_cast<const float4 *>(ca)[col];
    const float4 b = reinterpret_cast<const float4 *>(cb)[col];
    const float4 c = reinterpret_cast<const float4 *>(cc)[col];
    DzRaw q[kRowGroup];
    float4 xv[kRowGroup];
    for_rows<kRowGroup>(
        r0 + lane_row, r1, g.row_lanes,
        [&](int r, int u) {
            const size_t o = (size_t)r * g.C4 + col;
            if (DZ_IN) q[u].d = ld4(dy, o);
            else load_dz_raw<T, RELU, DY2>(q[u], dy, dy2, y, mask, o);
            xv[u] = ld4(x, o);
        },
        [&](int r, int u) {
            const float4 dz = DZ_IN ? q[u].d : finish_dz<RELU, DY2>(q[u], mask != nullptr);
            st4(dx, (size_t)r * g.C4 + col, fma4(a, dz, fma4(b, xv[u], c)));
        });
}

// ---- backward of BN + ReLU without a residual, the mask rebuilt from x ------------------------------------
// Without a residual the forward output is max(0, fma(x, scale, shift)) with scale = gamma*invstd and
// shift = fma(-mean, scale, beta): the same three roundings here give the same sign, so y need not be read
// (8 of the 28 bytes per element of the two passes).
template <class T>
__device__ inline float4 relu_mask_from_x(const T *like, float4 dz, float4 xv, float4 sc, float4 sh)
{
    // the forward output as it was stored (a bf16 store can round a tiny positive value to zero)
    const float4 pre = as_stored(like, fma4(xv, sc, sh));
    return make_float4(pre.x > 0.f ? dz.x : 0.f, pre.y > 0.f ? dz.y : 0.f, pre.z > 0.f ? dz.z : 0.f, pre.w > 0.f ? dz.w : 0.f);
}

template <class T>
__global__ __launch_bounds__(kBnThreads) void bn_bwd_reduce_xmask_kernel(BnGeom g, const T *__restrict__ x, const T *__restrict__ dy,
                                                                         const float *__restrict__ gamma, const float *__restrict__ beta,
                                                                         const float *__restrict__ save_mean,
                                                                         const float *__restrict__ save_invstd,
                                                                         float *__restrict__ part_db, float *__restrict__ part_dg)
{
    main_chain_priority();  // these run beside the filter gradients of the layer before (see igemm_kernel)
    __shared__ float4 s_db[kBnThreads];
    __shared__ float4 s_dg[kBnThreads];
    const int tid = threadIdx.x;
    const int col = blockIdx.y * g.cols + tid % g.cols;
    const int lane_row = tid / g.cols;
    const int r0 = blockIdx.x * g.rows_per_band;
    const int r1 = min(g.M, r0 + g.rows_per_band);
    const bool active = col < g.C4;
    float4 db = f4(0.f), dg = f4(0.f);
    if (active) {
        const float4 mean = reinterpret_cast<const float4 *>(save_mean)[col];
        const float4 inv = reinterpret_cast<const float4 *>(save_invstd)[col];
        const float4 sc = reinterpret_cast<const float4 *>(gamma)[col] * inv;
        const float4 sh = fma4(f4(0.f) - mean, sc, reinterpret_cast<const float4 *>(beta)[col]);
        float4 xv[kRowGroup], dv[kRowGroup];
        for_rows<kRowGroup>(
            r0 + lane_row, r1, g.row_lanes,
            [&](int r, int u) {
                const size_t o = (size_t)r * g.C4 + col;
                xv[u] = ld4(x, o);
                dv[u] = ld4(dy, o);
            },
            [&](int, int u) {
                const float4 dz = relu_mask_from_x(x, dv[u], xv[u], sc, sh);
                db = db + dz;
                dg = fma4(dz, (xv[u] - mean) * inv, dg);
            });
    }
    merge_rows_sum(db, dg, g.cols, g.row_lanes, s_db, s_dg);
    if (lane_row == 0 && active) {
        reinterpret_cast<float4 *>(part_db + (size_t)blockIdx.x * g.C)[col] = db;
        reinterpret_cast<float4 *>(part_dg + (size_t)blockIdx.x * g.C)[col] = dg;
    }
}

template <class T>
__global__ __launch_bounds__(kBnThreads) void bn_bwd_apply_xmask_kernel(BnGeom g, const T *__restrict__ x, const T *__restrict__ dy,
                                                                        const float *__restrict__ gamma, const float *__restrict__ beta,
                                                                        const float *__restrict__ save_mean,
                                                                        const float *__restrict__ save_invstd, const float *__restrict__ ca,
                                                                        const float *__restrict__ cb, const float *__restrict__ cc,
                                                                        T *__restrict__ dx)
{
    main_chain_priority();  // these run beside the filter gradients of the layer before (see igemm_kernel)
    const int tid = threadIdx.x;
    const int col = blockIdx.y * g.cols + tid % g.cols;
    if (col >= g.C4) return;
    const int lane_row = tid / g.cols;
    const int r0 = blockIdx.x * g.rows_per_band;
    const int r1 = min(g.M, r0 + g.rows_per_band);
    const float4 a = reinterpret_cast<const float4 *>(ca)[col];
    const float4 b = reinterpret_cast<const float4 *>(cb)[col];
    const float4 c = reinterpret_cast<const float4 *>(cc)[col];
    const float4 sc = reinterpret_cast<const float4 *>(gamma)[col] * reinterpret_cast<const float4 *>(save_invstd)[col];
    const float4 sh = fma4(f4(0.f) - reinterpret_cast<const float4 *>(save_mean)[col], sc, reinterpret_cast<const float4 *>(beta)[col]);
    float4 xv[kRowGroup], dv[kRowGroup];
    for_rows<kRowGroup>(
        r0 + lane_row, r1, g.row_lanes,
        [&](int r, int u) {
            const size_t o = (size_t)r * g.C4 + col;
            xv[u] = ld4(x, o);
            dv[u] = ld4(dy, o);
        },
        [&](int r, int u) {
            const float4 dz = relu_mask_from_x(x, dv[u], xv[u], sc, sh);
            st4(dx, (size_t)r * g.C4 + col, fma4(a, dz, fma4(b, xv[u], c)));
        });
}

static int bn_check(const char *who, int n, int c, int h, int w, int layout)
{
    RN50_REQUIRE(n > 0 && c > 0 && h > 0 && w > 0, RN50_EINVAL, "%s: non-positive dimension", who);
    RN50_REQUIRE(layout == RN50_LAYOUT_NHWC, RN50_EUNSUPPORTED, "%s: only the NHWC layout has kernels", who);
    RN50_REQUIRE(c % 4 == 0, RN50_EUNSUPPORTED, "%s: channel count must be a multiple of 4", who);
    RN50_REQUIRE((long)n * h * w < (1L << 31) / 4, RN50_EUNSUPPORTED, "%s: N*H*W too large", who);
    return RN50_OK;
}

}  // namespace rn50

using namespace rn50;

// ---- host side, written once for both activation storage types (T = float, or bf16_t for bfloat16 bits) -----------------

template <class T>
static void launch_bn_apply(const BnGeom &ga, bool res, bool relu, const T *x, const float *scale, const float *shift, const T *residual,
                            T *y, uint8_t *relu_mask, hipStream_t st)
{
    const dim3 grid(ga.bands, ga.col_blocks), block(kBnThreads);
    if (res && relu) hipLaunchKernelGGL((bn_apply_kernel<T, true, true>), grid, block, 0, st, ga, x, scale, shift, residual, y, relu_mask);
    else if (res) hipLaunchKernelGGL((bn_apply_kernel<T, true, false>), grid, block, 0, st, ga, x, scale, shift, residual, y, relu_mask);
    else if (relu) hipLaunchKernelGGL((bn_apply_kernel<T, false, true>), grid, block, 0, st, ga, x, scale, shift, residual, y, relu_mask);
    else hipLaunchKernelGGL((bn_apply_kernel<T, false, false>), grid, block, 0, st, ga, x, scale, shift, residual, y, relu_mask);
}

template <class T>
static int bn_apply_scale_shift_t(int n, int c, int h, int w, const T *x, const float *scale, const float *shift, int relu, T *y, hipStream_t st)
{
    launch_bn_apply<T>(bn_apply_geom(bn_geom(n, c, h, w)), false, relu != 0, x, scale, shift, nullptr, y, nullptr, st);
    return launch_status("bn_apply_scale_shift");
}

int rn50::bn_apply_scale_shift(int n, int c, int h, int w, const float *x, const float *scale, const float *shift, int relu, float *y,
                               hipStream_t st)
{
    return bn_apply_scale_shift_t<float>(n, c, h, w, x, scale, shift, relu, y, st);
}
int rn50::bn_apply_scale_shift_bf16(int n, int c, int h, int w, const uint16_t *x, const float *scale, const float *shift, int relu,
                                    uint16_t *y, hipStream_t st)
{
    return bn_apply_scale_shift_t<bf16_t>(n, c, h, w, x, scale, shift, relu, y, st);
}

void rn50::bn_finalize_partials(long M, int C, int bands, int rows_per_band, const float *part_mean, const float *part_m2,
                                const float *gamma, const float *beta, float eps, float *save_mean, float *save_invstd, float *scale,
                                float *shift, hipStream_t st)
{
    BnGeom g{};  // the merge reads the row count, the channel count and the cut of the rows into bands only
    g.M = (int)M; g.C = C; g.C4 = C / 4; g.bands = bands; g.rows_per_band = rows_per_band;
    if (bands > 1024)
        hipLaunchKernelGGL(bn_stats_finalize_kernel<256>, dim3(ceil_div(C, kFinCh)), dim3(kFinCh * 256), 0, st, g, part_mean, part_m2, gamma,
                           beta, eps, save_mean, save_invstd, scale, shift);
    else
        hipLaunchKernelGGL(bn_stats_finalize_kernel<kFinSl>, dim3(ceil_div(C, kFinCh)), dim3(kFinCh * kFinSl), 0, st, g, part_mean, part_m2,
                           gamma, beta, eps, save_mean, save_invstd, scale, shift);
}

template <class T>
static int bn_fwd_apply_impl(const char *who, int n, int c, int h, int w, int layout, const T *x, const float *scale, const float *shift,
                             const T *residual_or_null, int relu, T *y, uint8_t *relu_mask_or_null, void *stream)
{
    if (int rc = bn_check(who, n, c, h, w, layout)) return rc;
    RN50_REQUIRE(x && scale && shift && y, RN50_EINVAL, "%s: null pointer", who);
    RN50_REQUIRE(aligned16(x) && aligned16(scale) && aligned16(shift) && aligned16(residual_or_null) && aligned16(y), RN50_EINVAL,
                 "%s: pointers must be 16-byte aligned", who);
    RN50_REQUIRE(!relu_mask_or_null || relu, RN50_EINVAL, "%s: the mask is the ReLU's", who);
    launch_bn_apply<T>(bn_apply_geom(bn_geom(n, c, h, w)), residual_or_null != nullptr, relu != 0, x, scale, shift, residual_or_null, y,
                       relu_mask_or_null, (hipStream_t)stream);
    return launch_status(who);
}

extern "C" int bn_fwd_apply(int n, int c, int h, int w, int layout, const float *x, const float *scale, const float *shift,
                            const float *residual_or_null, int relu, float *y, uint8_t *relu_mask_or_null, void *stream)
{
    return bn_fwd_apply_impl<float>("bn_fwd_apply", n, c, h, w, layout, x, scale, shift, residual_or_null, relu, y, relu_mask_or_null, stream);
}

extern "C" int bn_fwd_apply_bf16(int n, int c, int h, int w, int layout, const uint16_t *x, const float *scale, const float *shift,
                                 const uint16_t *residual_or_null, int relu, uint16_t *y, uint8_t *relu_mask_or_null, void *stream)
{
    return bn_fwd_apply_impl<bf16_t>("bn_fwd_apply_bf16", n, c, h, w, layout, x, scale, shift, residual_or_null, relu, y, relu_mask_or_null,
                                     stream);
}

extern "C" size_t rn50_bn_workspace_bytes(int n, int c, int h, int w)
{
    if (n <= 0 || c <= 0 || h <= 0 || w <= 0 || c % 4) return 0;
    return bn_ws_floats(bn_geom(n, c, h, w)) * sizeof(float);
}

// Forward: statistics, merge, normalise.  y == nullptr stops after the merge (the consumer normalises); then scale_out and
// shift_out receive the per-channel coefficients instead of the workspace.
template <class T>
static int bn_fwd_impl(const char *who, int n, int c, int h, int w, int layout, const T *x, const float *gamma, const float *beta, float eps,
                       const T *residual_or_null, int relu, T *y, uint8_t *relu_mask, float *save_mean, float *save_invstd,
                       float *scale_out, float *shift_out, void *ws, size_t ws_bytes, void *stream)
{
    if (int rc = bn_check(who, n, c, h, w, layout)) return rc;
    RN50_REQUIRE(x && gamma && beta && save_mean && save_invstd && ws && (y || (scale_out && shift_out)), RN50_EINVAL, "%s: null pointer", who);
    RN50_REQUIRE(aligned16(x) && aligned16(gamma) && aligned16(beta) && aligned16(y) && aligned16(save_mean) && aligned16(save_invstd) &&
                     aligned16(residual_or_null) && aligned16(scale_out) && aligned16(shift_out) && aligned16(ws),
                 RN50_EINVAL, "%s: pointers must be 16-byte aligned", who);
    RN50_REQUIRE(eps >= 0.f, RN50_EINVAL, "%s: negative eps", who);
    const BnGeom g = bn_geom(n, c, h, w);
    RN50_REQUIRE(ws_bytes >= bn_ws_floats(g) * sizeof(float), RN50_EWORKSPACE, "%s: workspace too small", who);
    float *part_mean = (float *)ws, *part_m2 = part_mean + (size_t)g.bands * g.C;
    float *scale = y ? part_m2 + (size_t)g.bands * g.C : scale_out, *shift = y ? scale + g.C : shift_out;
    hipStream_t st = (hipStream_t)stream;
    hipLaunchKernelGGL((bn_stats_kernel<T>), dim3(g.bands, g.col_blocks), dim3(kBnThreads), 0, st, g, x, part_mean, part_m2);
    hipLaunchKernelGGL(bn_stats_finalize_kernel<kFinSl>, dim3(ceil_div(c, kFinCh)), dim3(kFinCh * kFinSl), 0, st, g, part_mean, part_m2, gamma,
                       beta, eps, save_mean, save_invstd, scale, shift);
    if (y) launch_bn_apply<T>(bn_apply_geom(g), residual_or_null != nullptr, relu != 0, x, scale, shift, residual_or_null, y, relu_mask, st);
    return launch_status(who);
}

extern "C" int bn_fwd_batchstats(int n, int c, int h, int w, int layout, const float *x, const float *gamma,
                                 const float *beta, float eps, const float *residual_or_null, int relu, float *y,
                                 float *save_mean, float *save_invstd, void *ws, size_t ws_bytes, void *stream)
{
    RN50_REQUIRE(y, RN50_EINVAL, "bn_fwd_batchstats: null pointer");
    return bn_fwd_impl<float>("bn_fwd_batchstats", n, c, h, w, layout, x, gamma, beta, eps, residual_or_null, relu, y, nullptr, save_mean,
                              save_invstd, nullptr, nullptr, ws, ws_bytes, stream);
}

// Device address of `scratch` on the current device, looked up once per device (with that device current) and kept.
static int static_scratch(void **out)
{
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void *ptrs[kMaxDevices] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(RN50_EHIP, "bn_fwd_batchstats_static: hipGetDevice: %s", hipGetErrorString(e));
    RN50_REQUIRE(dev >= 0 && dev < kMaxDevices, RN50_EUNSUPPORTED, "bn_fwd_batchstats_static: device ordinal %d out of range", dev);
    std::lock_guard<std::mutex> lk(mu);
    if (!ptrs[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return fail(RN50_EHIP, "bn_fwd_batchstats_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
        ptrs[dev] = p;
    }
    *out = ptrs[dev];
    return RN50_OK;
}

extern "C" int bn_fwd_batchstats_static(int n, int c, int h, int w, int layout, const float *x, const float *gamma, const float *beta,
                                        float eps, const float *residual_or_null, int relu, float *y, float *save_mean,
                                        float *save_invstd, void *stream)
{
    if (int rc = bn_check("bn_fwd_batchstats_static", n, c, h, w, layout)) return rc;
    const size_t need = bn_ws_floats(bn_geom(n, c, h, w)) * sizeof(float);
    RN50_REQUIRE(need <= (size_t)RN50_BN_STATIC_SCRATCH_BYTES, RN50_EWORKSPACE,
                 "bn_fwd_batchstats_static: this shape needs %zu bytes of scratch, the built-in buffer has %zu (use bn_fwd_batchstats with "
                 "a workspace)", need, (size_t)RN50_BN_STATIC_SCRATCH_BYTES);
    RN50_REQUIRE(x && gamma && beta && y && save_mean && save_invstd, RN50_EINVAL, "bn_fwd_batchstats_static: null pointer");
    void *ws = nullptr;
    if (int rc = static_scratch(&ws)) return rc;
    // every partial and coefficient the kernels read is written earlier in the same call: nothing has to start at zero
    return bn_fwd_impl<float>("bn_fwd_batchstats_static", n, c, h, w, layout, x, gamma, beta, eps, residual_or_null, relu, y, nullptr,
                              save_mean, save_invstd, nullptr, nullptr, ws, RN50_BN_STATIC_SCRATCH_BYTES, stream);
}

extern "C" int bn_fwd_batchstats_mask(int n, int c, int h, int w, int layout, const float *x, const float *gamma, const float *beta,
                                      float eps, const float *residual_or_null, float *y, uint8_t *relu_mask, float *save_mean,
                                      float *save_invstd, void *ws, size_t ws_bytes, void *stream)
{
    RN50_REQUIRE(relu_mask && y, RN50_EINVAL, "bn_fwd_batchstats_mask: null pointer");
    return bn_fwd_impl<float>("bn_fwd_batchstats_mask", n, c, h, w, layout, x, gamma, beta, eps, residual_or_null, 1, y, relu_mask, save_mean,
                              save_invstd, nullptr, nullptr, ws, ws_bytes, stream);
}

extern "C" int bn_stats_scale_shift(int n, int c, int h, int w, int layout, const float *x, const float *gamma, const float *beta,
                                    float eps, float *save_mean, float *save_invstd, float *scale, float *shift, void *ws,
                                    size_t ws_bytes, void *stream)
{
    RN50_REQUIRE(scale && shift, RN50_EINVAL, "bn_stats_scale_shift: null pointer");
    return bn_fwd_impl<float>("bn_stats_scale_shift", n, c, h, w, layout, x, gamma, beta, eps, nullptr, 0, nullptr, nullptr, save_mean,
                              save_invstd, scale, shift, ws, ws_bytes, stream);
}

extern "C" int bn_fwd_batchstats_bf16(int n, int c, int h, int w, int layout, const uint16_t *x, const float *gamma, const float *beta,
                                      float eps, const uint16_t *residual_or_null, int relu, uint16_t *y, uint8_t *relu_mask_or_null,
                                      float *save_mean, float *save_invstd, void *ws, size_t ws_bytes, void *stream)
{
    RN50_REQUIRE(y, RN50_EINVAL, "bn_fwd_batchstats_bf16: null pointer");
    RN50_REQUIRE(!relu_mask_or_null || relu, RN50_EINVAL, "bn_fwd_batchstats_bf16: the mask is the ReLU's");
    return bn_fwd_impl<bf16_t>("bn_fwd_batchstats_bf16", n, c, h, w, layout, x, gamma, beta, eps, residual_or_null, relu, y, relu_mask_or_null,
                               save_mean, save_invstd, nullptr, nullptr, ws, ws_bytes, stream);
}

extern "C" int bn_stats_scale_shift_bf16(int n, int c, int h, int w, int layout, const uint16_t *x, const float *gamma, const float *beta,
                                         float eps, float *save_mean, float *save_invstd, float *scale, float *shift, void *ws,
                                         size_t ws_bytes, void *stream)
{
    RN50_REQUIRE(scale && shift, RN50_EINVAL, "bn_stats_scale_shift_bf16: null pointer");
    return bn_fwd_impl<bf16_t>("bn_stats_scale_shift_bf16", n, c, h, w, layout, x, gamma, beta, eps, nullptr, 0, nullptr, nullptr, save_mean,
                               save_invstd, scale, shift, ws, ws_bytes, stream);
}

extern "C" int bn_fwd_inference(int n, int c, int h, int w, int layout, const float *x, const float *gamma, const float *beta,
                                const float *mean, const float *invstd, const float *residual_or_null, int relu, float *y,
                                void *ws, size_t ws_bytes, void *stream)
{
    if (int rc = bn_check("bn_fwd_inference", n, c, h, w, layout)) return rc;
    RN50_REQUIRE(x && gamma && beta && mean && invstd && y && ws, RN50_EINVAL, "bn_fwd_inference: null pointer");
    RN50_REQUIRE(aligned16(x) && aligned16(gamma) && aligned16(beta) && aligned16(mean) && aligned16(invstd) && aligned16(y) &&
                     aligned16(residual_or_null) && aligned16(ws),
                 RN50_EINVAL, "bn_fwd_inference: pointers must be 16-byte aligned");
    const BnGeom g = bn_geom(n, c, h, w);
    RN50_REQUIRE(ws_bytes >= bn_ws_floats(g) * sizeof(float), RN50_EWORKSPACE, "bn_fwd_inference: workspace too small");
    float *scale = (float *)ws, *shift = scale + g.C;
    hipStream_t st = (hipStream_t)stream;
    hipLaunchKernelGGL(bn_scale_shift_kernel, dim3(ceil_div(c, 256)), dim3(256), 0, st, c, gamma, beta, mean, invstd, scale, shift);
    launch_bn_apply<float>(bn_apply_geom(g), residual_or_null != nullptr, relu != 0, x, scale, shift, residual_or_null, y, nullptr, st);
    return launch_status("bn_fwd_inference");
}

extern "C" int bn_stats_average(int c, int n_sets, const float *means, const float *invstds, float eps, float *mean_out,
                                float *invstd_out, void *stream)
{
    RN50_REQUIRE(c > 0 && n_sets > 0, RN50_EINVAL, "bn_stats_average: non-positive size");
    RN50_REQUIRE(means && invstds && mean_out && invstd_out, RN50_EINVAL, "bn_stats_average: null pointer");
    RN50_REQUIRE(eps >= 0.f, RN50_EINVAL, "bn_stats_average: negative eps");
    hipLaunchKernelGGL(bn_stats_average_kernel, dim3(ceil_div(c, 256)), dim3(256), 0, (hipStream_t)stream, c, n_sets, means, invstds,
                       eps, mean_out, invstd_out);
    return launch_status("bn_stats_average");
}

// Backward.  The ReLU mask comes from y, else from the byte mask, else (beta given) it is rebuilt from x.
template <class T>
static int bn_bwd_impl(const char *who, int n, int c, int h, int w, int layout, const T *x, const T *dy, const T *dy2_or_null,
                       const T *y_or_null, const uint8_t *mask, const float *gamma, const float *beta_for_xmask, const float *save_mean,
                       const float *save_invstd, int relu, T *dx, T *dresidual_or_null, float *dgamma, float *dbeta, void *ws,
                       size_t ws_bytes, void *stream)
{
    if (int rc = bn_check(who, n, c, h, w, layout)) return rc;
    RN50_REQUIRE(x && dy && gamma && save_mean && save_invstd && dx && dgamma && dbeta && ws, RN50_EINVAL, "%s: null pointer", who);
    const bool xmask = relu && !y_or_null && !mask;
    RN50_REQUIRE(!xmask || (beta_for_xmask && !dy2_or_null && !dresidual_or_null), RN50_EINVAL,
                 "%s: the ReLU mask needs the forward output y, a byte mask, or (one gradient, no residual) beta to rebuild it from x", who);
    RN50_REQUIRE(aligned16(x) && aligned16(dy) && aligned16(dy2_or_null) && aligned16(y_or_null) && aligned16(gamma) &&
                     aligned16(beta_for_xmask) && aligned16(save_mean) && aligned16(save_invstd) && aligned16(dx) &&
                     aligned16(dresidual_or_null) && aligned16(dgamma) && aligned16(dbeta) && aligned16(ws),
                 RN50_EINVAL, "%s: pointers must be 16-byte aligned", who);
    const BnGeom g = bn_geom(n, c, h, w);
    const BnGeom ga = bn_apply_geom(g);
    RN50_REQUIRE(ws_bytes >= bn_ws_floats(g) * sizeof(float), RN50_EWORKSPACE, "%s: workspace too small", who);
    float *part_db = (float *)ws, *part_dg = part_db + (size_t)g.bands * g.C;
    float *ca = part_dg + (size_t)g.bands * g.C, *cb = ca + g.C, *cc = cb + g.C;
    hipStream_t st = (hipStream_t)stream;
    const dim3 grid(g.bands, g.col_blocks), agrid(ga.bands, ga.col_blocks), block(kBnThreads);
    const dim3 fgrid(ceil_div(c, kFinCh)), fblock(kFinCh * kFinSl);
    if (xmask) {
        hipLaunchKernelGGL((bn_bwd_reduce_xmask_kernel<T>), grid, block, 0, st, g, x, dy, gamma, beta_for_xmask, save_mean, save_invstd, part_db, part_dg);
        hipLaunchKernelGGL(bn_bwd_finalize_kernel, fgrid, fblock, 0, st, g, part_db, part_dg, gamma, save_mean, save_invstd, dgamma, dbeta, ca, cb, cc);
        hipLaunchKernelGGL((bn_bwd_apply_xmask_kernel<T>), agrid, block, 0, st, ga, x, dy, gamma, beta_for_xmask, save_mean, save_invstd, ca, cb, cc, dx);
        return launch_status(who);
    }
    const bool two = dy2_or_null != nullptr, wdz = dresidual_or_null != nullptr;
#define RN50_BN_REDUCE(R, D, W)                                                                                            \
    hipLaunchKernelGGL((bn_bwd_reduce_kernel<T, R, D, W>), grid, block, 0, st, g, x, dy, dy2_or_null, y_or_null, mask, save_mean, \
                       save_invstd, dresidual_or_null, part_db, part_dg)
    if (relu) {
        if (two) { if (wdz) RN50_BN_REDUCE(true, true, true); else RN50_BN_REDUCE(true, true, false); }
        else     { if (wdz) RN50_BN_REDUCE(true, false, true); else RN50_BN_REDUCE(true, false, false); }
    } else {
        if (two) { if (wdz) RN50_BN_REDUCE(false, true, true); else RN50_BN_REDUCE(false, true, false); }
        else     { if (wdz) RN50_BN_REDUCE(false, false, true); else RN50_BN_REDUCE(false, false, false); }
    }
#undef RN50_BN_REDUCE
    hipLaunchKernelGGL(bn_bwd_finalize_kernel, fgrid, fblock, 0, st, g, part_db, part_dg, gamma, save_mean, save_invstd, dgamma, dbeta, ca, cb, cc);
    if (wdz) {
        // dz was stored by the reduce pass: read it back instead of dy, dy2 and y
        hipLaunchKernelGGL((bn_bwd_apply_kernel<T, false, false, true>), agrid, block, 0, st, ga, x, (const T *)dresidual_or_null, (const T *)nullptr,
                           (const T *)nullptr, (const uint8_t *)nullptr, ca, cb, cc, dx);
    } else {
#define RN50_BN_APPLY(R, D) \
    hipLaunchKernelGGL((bn_bwd_apply_kernel<T, R, D, false>), agrid, block, 0, st, ga, x, dy, dy2_or_null, y_or_null, mask, ca, cb, cc, dx)
        if (relu) { if (two) RN50_BN_APPLY(true, true); else RN50_BN_APPLY(true, false); }
        else      { if (two) RN50_BN_APPLY(false, true); else RN50_BN_APPLY(false, false); }
#undef RN50_BN_APPLY
    }
    return launch_status(who);
}

extern "C" int bn_bwd_batchstats(int n, int c, int h, int w, int layout, const float *x, const float *dy,
                                 const float *dy2_or_null, const float *y_or_null, const float *gamma,
                                 const float *save_mean, const float *save_invstd, int relu, float *dx,
                                 float *dresidual_or_null, float *dgamma, float *dbeta, void *ws, size_t ws_bytes,
                                 void *stream)
{
    RN50_REQUIRE(!relu || y_or_null, RN50_EINVAL, "bn_bwd_batchstats: the ReLU mask needs the forward output y");
    return bn_bwd_impl<float>("bn_bwd_batchstats", n, c, h, w, layout, x, dy, dy2_or_null, y_or_null, nullptr, gamma, nullptr, save_mean,
                              save_invstd, relu, dx, dresidual_or_null, dgamma, dbeta, ws, ws_bytes, stream);
}

extern "C" int bn_bwd_batchstats_mask(int n, int c, int h, int w, int layout, const float *x, const float *dy, const float *dy2_or_null,
                                      const uint8_t *relu_mask, const float *gamma, const float *save_mean, const float *save_invstd,
                                      float *dx, float *dresidual_or_null, float *dgamma, float *dbeta, void *ws, size_t ws_bytes,
                                      void *stream)
{
    RN50_REQUIRE(relu_mask, RN50_EINVAL, "bn_bwd_batchstats_mask: null mask pointer");
    return bn_bwd_impl<float>("bn_bwd_batchstats_mask", n, c, h, w, layout, x, dy, dy2_or_null, nullptr, relu_mask, gamma, nullptr, save_mean,
                              save_invstd, 1, dx, dresidual_or_null, dgamma, dbeta, ws, ws_bytes, stream);
}

extern "C" int bn_bwd_batchstats_xmask(int n, int c, int h, int w, int layout, const float *x, const float *dy, const float *gamma,
                                      const float *beta, const float *save_mean, const float *save_invstd, float *dx, float *dgamma,
                                      float *dbeta, void *ws, size_t ws_bytes, void *stream)
{
    RN50_REQUIRE(beta, RN50_EINVAL, "bn_bwd_batchstats_xmask: null pointer");
    return bn_bwd_impl<float>("bn_bwd_batchstats_xmask", n, c, h, w, layout, x, dy, nullptr, nullptr, nullptr, gamma, beta, save_mean,
                              save_invstd, 1, dx, nullptr, dgamma, dbeta, ws, ws_bytes, stream);
}

extern "C" int bn_bwd_batchstats_bf16(int n, int c, int h, int w, int layout, const uint16_t *x, const uint16_t *dy,
                                      const uint16_t *dy2_or_null, const uint16_t *y_or_null, const uint8_t *relu_mask_or_null,
                                      const float *gamma, const float *beta_or_null, const float *save_mean, const float *save_invstd,
                                      int relu, uint16_t *dx, uint16_t *dresidual_or_null, float *dgamma, float *dbeta, void *ws,
                                      size_t ws_bytes, void *stream)
{
    return bn_bwd_impl<bf16_t>("bn_bwd_batchstats_bf16", n, c, h, w, layout, x, dy, dy2_or_null, y_or_null, relu_mask_or_null, gamma,
                               beta_or_null, save_mean, save_invstd, relu, dx, dresidual_or_null, dgamma, dbeta, ws, ws_bytes, stream);
}
