// Internal helpers shared by the translation units of librn50.so (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdint.h>
#include <stdio.h>

#include <memory>
#include <vector>

#include "rn50.h"

namespace rn50 {

int fail(int code, const char *fmt, ...);  // records the message for rn50_last_error() and returns code

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// After a kernel launch: turn a launch error into RN50_EHIP.
inline int launch_status(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(RN50_EHIP, "%s: %s", what, hipGetErrorString(e));
    return RN50_OK;
}

// Tuning and test switches (rn50_set_option; initial values from the RN50_* environment variables, read once).
struct PlanRow { int op, n, c, h, k, r, stride, pad, bm, bn, split; };
struct Config {
    bool side_stream = true;   // rn50_create: filter gradients and projection shortcuts on helper streams
    int fuse_bn = -1;          // rn50_create: which BN + ReLU outputs are applied by their consumer (bit mask); -1: 3, with bf16 activations 1
    bool relu_mask = true;     // rn50_create: byte mask instead of the block output in the c layers' BN backward
    bool no_tuned = false;     // ignore the measured plan table (cost model only)
    bool no_stem_kernel = false;  // first layer through the implicit GEMM
    bool conv_bn_stats = true;    // rn50_create: forward convolutions gather the BN statistics of their output
    int wgrad_group = 0;          // rn50_create: filter gradients launched per layer (0) or grouped, this many blocks to a launch
    int wgrad_group_wgs_per_cu = 0;  // grouped filter gradients: at most this many workgroups of theirs per CU (0: what fits)
    int wgrad_group_stages = 48;  // grouped filter gradients: LDS stages (of 32 pixels) per work item
    int wgrad_group_bm = 64, wgrad_group_bn = 64;  // ... and their tile
    bool has_igemm_plan = false, has_wgrad_plan = false;
    int igemm_plan[3] = {0, 0, 0}, wgrad_plan[3] = {0, 0, 0};  // bm, bn, split forced for every call
    std::vector<PlanRow> overrides;                            // rows that go before the measured table
};
std::shared_ptr<const Config> config();  // the current snapshot (immutable; a call keeps the one it started with)

inline int ceil_div(long a, long b) { return (int)((a + b - 1) / b); }

constexpr int kWave = 64;

// Sum over the 64 lanes of a wavefront (result valid in every lane).
__device__ inline float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ inline float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// ---- activation storage: fp32, or bfloat16 bits (round to nearest even on store) ------------------------------------
typedef uint16_t bf16_t;

// fp32 -> bfloat16 bits, round to nearest, ties to even (NaN stays NaN): gfx950 converts in hardware, two values per
// instruction (v_cvt_pk_bf16_f32); in integer arithmetic the same rounding costs about five instructions per value, in
// kernels that round every operand on its way into LDS.  Written as the instruction itself: the compiler emits it for a
// conversion of a two-element vector too, but building that vector from elements of two register arrays made it keep the
// arrays in scratch memory in the filter-gradient kernels.
__device__ inline uint32_t bf16_pack2(float lo, float hi)
{
    uint32_t r;
    asm("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(r) : "v"(lo), "v"(hi));
    return r;
}
__device__ inline uint32_t bf16_rne(float f) { return bf16_pack2(f, f) & 0xffffu; }
__device__ inline float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }          // element in the low half of a word
__device__ inline float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }  // element in the high half
__device__ inline float bf16_round(float f) { return __uint_as_float(bf16_rne(f) << 16); }

// Elements 4*i4 .. 4*i4+3 of a tensor as floats, and the store of four floats (the bf16 store rounds).
__device__ inline float4 ld4(const float *p, size_t i4) { return reinterpret_cast<const float4 *>(p)[i4]; }
__device__ inline float4 ld4(const bf16_t *p, size_t i4)
{
    const uint2 u = reinterpret_cast<const uint2 *>(p)[i4];
    return make_float4(bf16_lo(u.x), bf16_hi(u.x), bf16_lo(u.y), bf16_hi(u.y));
}
__device__ inline void st4(float *p, size_t i4, float4 v) { reinterpret_cast<float4 *>(p)[i4] = v; }
__device__ inline void st4(bf16_t *p, size_t i4, float4 v)
{
    reinterpret_cast<uint2 *>(p)[i4] = make_uint2(bf16_pack2(v.x, v.y), bf16_pack2(v.z, v.w));
}
// What a store of v leaves in memory, as floats (the forward output's sign decides the ReLU mask: it is taken after rounding).
__device__ inline float4 as_stored(const float *, float4 v) { return v; }
__device__ inline float4 as_stored(const bf16_t *, float4 v) { return make_float4(bf16_round(v.x), bf16_round(v.y), bf16_round(v.z), bf16_round(v.w)); }

// Issue priority of the calling wavefront among the wavefronts of its SIMD (0 = default = lowest, 3 = highest); see igemm_kernel.
__device__ inline void main_chain_priority() { __builtin_amdgcn_s_setprio(3); }

// Consecutive workgroups are dispatched to different XCDs, each with an L2 of its own.  Workgroup b of n does the work of
// index xcd_contiguous(b, n): the eight XCDs then each cover one contiguous range of the index space, so that neighbouring
// work items, which read the same cache lines, share an L2.
__device__ inline int xcd_contiguous(int b, int n)
{
    const int n8 = n & ~7;
    return b < n8 ? (b & 7) * (n8 >> 3) + (b >> 3) : b;
}

}  // namespace rn50

namespace rn50 {
// Internal entry points used by the whole-step schedule (csrc/conv.hip).
int conv_check(const char *who, const rn50_conv_desc *d);  // argument checks shared by the convolution entry points
int conv_bwd_data_pretransposed(const rn50_conv_desc *d, const float *dy, const float *wt, float *dx, void *ws, size_t ws_bytes,
                                hipStream_t st);
size_t conv_bwd_data_pretransposed_ws(const rn50_conv_desc *d);
void launch_filter_flip(int K, int C, int RS, const float *w, float *wt, hipStream_t st);
// One launch for many filters; `jobs` is a device array of FlipJobHost records (same layout as the kernel's).
struct FlipJobHost {
    int K, C, RS, tiles_c, tiles_k, block_begin;
    long src_off, dst_off;
};
// y = x*scale[c] + shift[c] [ReLU] over an N x H x W x C tensor (the normalising kernel of the BN forward alone).
int bn_apply_scale_shift(int n, int c, int h, int w, const float *x, const float *scale, const float *shift, int relu, float *y,
                         hipStream_t st);
int bn_apply_scale_shift_bf16(int n, int c, int h, int w, const uint16_t *x, const float *scale, const float *shift, int relu,
                              uint16_t *y, hipStream_t st);
// Merge of per-row-tile statistics gathered by a convolution: `bands` tiles of rows_per_band rows each (the last one
// ragged) left mean and squared deviations at part_mean / part_m2 [band][C]; writes what the BN forward's merge writes.
void bn_finalize_partials(long M, int C, int bands, int rows_per_band, const float *part_mean, const float *part_m2,
                          const float *gamma, const float *beta, float eps, float *save_mean, float *save_invstd, float *scale,
                          float *shift, hipStream_t st);
// Filter gradients of several layers in one launch (csrc/conv_group.hip): the extern "C" calls with the tuning values spelled out.
size_t wgrad_group_table_bytes(int count);
size_t wgrad_group_ws_bytes(int count, const rn50_wgrad_group_item *items, int stages);
int wgrad_group_plan(int count, const rn50_wgrad_group_item *items, void *ws, size_t ws_bytes, void *table_host, size_t table_bytes,
                     int stages, int bm, int bn, int wgs_per_cu);
constexpr int kFlipTileHost = 64;  // tile edge of the filter flip kernels (a job counts its workgroups with it)
void launch_filter_flip_batched(const void *jobs, int njobs, int nblocks, const float *theta, float *wt, hipStream_t st);
}  // namespace rn50

#define RN50_REQUIRE(cond, code, ...) \
    do { if (!(cond)) return rn50::fail(code, __VA_ARGS__); } while (0)
