// fp32-MFMA implicit-GEMM kernels for the ResNet-50 convolutions (device code; included by conv.hip).
//
// Two kernels cover the three directions:
//   igemm_kernel : out[m][j] = sum_kk A[m][kk] * B[j][kk], both operands contiguous along the
//                  reduction index kk = (r,s,c).  A is gathered on the fly from an NHWC tensor
//                  (im2col never exists in memory), B is a K x (R*S*C) filter matrix.  Used for the
//                  forward pass and, with flipped/transposed filters, for the data gradient.
//   wgrad_kernel : dw[k][(r,s,c)] = sum_pix dy[pix][k] * xcol[pix][(r,s,c)], both operands contiguous
//                  along the OUTPUT index; the reduction runs over pixels and is split over workgroups
//                  into partial sums that a second kernel adds in a fixed order.
// Tiles are staged through LDS and multiplied with v_mfma_f32_32x32x2_f32 (the paper computes in
// single precision).  256 threads = 4 wavefronts in a 2x2 arrangement; each wavefront owns
// (BM/2) x (BN/2) outputs as 32x32 MFMA blocks.
#pragma once
#include "common.h"

namespace rn50 {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kConvThreads = 256;
constexpr int kBK = 32;        // reduction elements per LDS stage
constexpr int kLDK = kBK + 4;  // padded row length: 16-byte aligned rows, conflict-free 128-bit fragment reads
constexpr int kLDH = kBK + 8;  // the same for rows of 16-bit elements (80 bytes)

// Division of a 32-bit unsigned number by a divisor fixed at launch, as multiply-high and shifts (Granlund and
// Montgomery's round-up method): exact for every 32-bit dividend.  A hardware-less integer division would cost
// some forty vector instructions, and the pixel -> (image, row, column) decode sits in the inner loops.
struct FastDiv {
    uint32_t d, m, s1, s2;
};
inline FastDiv make_fastdiv(uint32_t d)
{
    FastDiv f;
    f.d = d;
    uint32_t l = 0;
    while ((1ull << l) < d) ++l;  // ceil(log2 d)
    f.m = (uint32_t)(((1ull << 32) * ((1ull << l) - d)) / d + 1);
    f.s1 = l < 1 ? l : 1;
    f.s2 = l > 0 ? l - 1 : 0;
    return f;
}
__device__ inline uint32_t fdiv(uint32_t n, const FastDiv &f)
{
    const uint32_t t = __umulhi(f.m, n);
    return (t + ((n - t) >> f.s1)) >> f.s2;
}

// Geometry of the gathered operand.  Output row m = (n, oh, ow); for filter tap (r, s) the input
// coordinate is ih = (oh*so + r + off)/sd and exists only when the numerator is a non-negative
// multiple of sd and ih < IH (same for iw).  Forward: so = stride, off = -pad, sd = 1.  Data gradient:
// so = 1, off = pad-(R-1), sd = stride, with the filter flipped.
//
// Work decomposition.  The grid is persistent: G workgroups (a multiple of 8, sized to what the chip holds
// at once) each take work items g, g+G, g+2G, ...  The first `full_items` items (a multiple of G) are whole
// output tiles.  The remaining `tail_tiles` tiles would fill only part of the machine, so each is cut into
// `tail_split` pieces along the reduction; a piece writes its partial tile to scratch and a second kernel adds
// the pieces of each tile in a fixed order.  Stores are not waited for, so the write-out of one tile overlaps
// the loads and MFMAs of the next item.
struct IgemmP {
    const float *a;
    const float *b;
    float *out;
    float *partial;        // [tail_tiles][tail_split][BM*BN], tile-local row-major
    // INAFF kernels: the gathered operand is max(0, a*in_scale[c] + in_shift[c]) per input channel c, computed on the way
    // into LDS (the BN + ReLU that produced the layer's input, never written to memory); padding stays zero.
    const float *in_scale;
    const float *in_shift;
    // Batch statistics of the output, gathered as it is written (null: off): row tile tm leaves the mean of its rows and the
    // sum of their squared deviations from it, per output column, at [tm * Nout + column] (values as stored; a ragged last
    // tile counts its own rows only).  A later kernel merges the row tiles in tile order.
    float *stat_mean;
    float *stat_m2;
    int IH, IW, Cin;
    int OH, OW;
    int Nout;
    int R, S;
    int so, off, sd;
    int M;      // N*OH*OW
    int Kdim;   // R*S*Cin
    int kchunks;
    int tiles_m, tiles_n;
    int full_items, tail_tiles, tail_split, tail_chunks;  // tail_chunks = reduction chunks per piece
    // Row order of the output matrix.  0: row m is pixel m.  1: row m = (n, oh, ow) goes to pixel (n, 2*oh, 2*ow) of an
    // N x 2OH x 2OW x Nout tensor and its three siblings are zeroed (data gradient of a 1x1 stride-2 convolution).
    // 2: rows are grouped by the parity class (oh%2, ow%2) of their pixel in that tensor: row m = (class, n, oh, ow) is
    // pixel (n, 2*oh + class/2, 2*ow + class%2).  For the data gradient of a stride-2 convolution every row of a class
    // receives the same subset of filter taps, so a tile inside one class skips the other taps instead of multiplying
    // gathered zeros (OH, OW are the half sizes here, M = 4*N*OH*OW).
    int scatter2;
    FastDiv div_ohw, div_ow, div_cin, div_s;  // by OH*OW, OW, Cin, S
    FastDiv div_class;                        // by M/4 (row order 2)
};

__device__ inline float4 ldg4(const float *p) { return *reinterpret_cast<const float4 *>(p); }
typedef const float __attribute__((address_space(1))) *gcfp;  // pointers known to point to global memory
typedef float __attribute__((address_space(1))) *gfp;
__device__ inline float4 ldg4(gcfp p)
{
    typedef float f4 __attribute__((ext_vector_type(4)));
    const f4 v = *reinterpret_cast<const f4 __attribute__((address_space(1))) *>(p);
    return make_float4(v.x, v.y, v.z, v.w);
}

// Row m of the GEMM -> first element of its output row (stride-2 scatter of the 1x1/2 data gradient included).
// row m -> (class, image, row, column) with the half sizes of row order 2 (class = 0 for the other orders)
__device__ inline void decode_row(const IgemmP &p, int m, int &cls, int &n, int &oh, int &ow)
{
    cls = 0;
    if (p.scatter2 == 2) {
        cls = (int)fdiv(m, p.div_class);
        m -= cls * (p.M >> 2);
    }
    n = (int)fdiv(m, p.div_ohw);
    const int rem = m - n * (p.OH * p.OW);
    oh = (int)fdiv(rem, p.div_ow);
    ow = rem - oh * p.OW;
}

__device__ inline long out_row_index(const IgemmP &p, int m)
{
    if (!p.scatter2) return m;
    int cls, n, oh, ow;
    decode_row(p, m, cls, n, oh, ow);
    return ((long)n * 2 * p.OH + 2 * oh + (cls >> 1)) * (2 * p.OW) + 2 * ow + (cls & 1);
}

template <bool O16 = false>
__device__ inline void store_out(const IgemmP &p, long row, int col, float v)
{
    if (O16) {  // the output tensor holds bfloat16 bits
        bf16_t *o = reinterpret_cast<bf16_t *>(p.out);
        o[row * p.Nout + col] = (bf16_t)bf16_rne(v);
        if (p.scatter2 == 1) {
            o[(row + 1) * p.Nout + col] = 0;
            o[(row + 2 * p.OW) * p.Nout + col] = 0;
            o[(row + 2 * p.OW + 1) * p.Nout + col] = 0;
        }
        return;
    }
    p.out[row * p.Nout + col] = v;
    if (p.scatter2 == 1) {
        p.out[(row + 1) * p.Nout + col] = 0.f;
        p.out[(row + 2 * p.OW) * p.Nout + col] = 0.f;
        p.out[(row + 2 * p.OW + 1) * p.Nout + col] = 0.f;
    }
}

// Workgroups of the implicit-GEMM kernel that one CU holds at once (= wavefronts per SIMD, since a workgroup puts
// one wavefront on each SIMD).  The launch bounds make the compiler keep the register count within this, and the
// host sizes the persistent grid with the same number.
constexpr int igemm_occupancy(int bm, int bn) { return (bm == 128 && bn == 128) ? 2 : (bm == 64 && bn == 64) ? 4 : 3; }

// MODE 0: Cin % 32 == 0, sd == 1.  MODE 1: Cin % 32 == 0, sd > 1.  MODE 2: any Cin and sd (scalar gather).
// BF = false: fp32 operands, v_mfma_f32_32x32x2_f32 (the paper's single precision).
// BF = true : operands are rounded to bfloat16 (RNE) on their way into LDS and multiplied with
//             v_mfma_f32_32x32x16_bf16; accumulation and outputs stay fp32.
// INAFF (MODE 0 only): per-channel scale, shift and ReLU applied to the gathered operand (see IgemmP::in_scale).
// ACT (BF only): storage of the activation tensors.  0: fp32.  1: the gathered operand `a` and the output hold bfloat16
//             bits (activations kept as bf16 in memory; a thread gathers eight elements per 16-byte load).  2: `a` is fp32,
//             the output bf16 (the network's first layer, whose input is the image).  The filter operand `b` is fp32 always.
// STATS: the kernel also leaves the per-tile batch statistics of its output (IgemmP::stat_mean, which must be set).
// BK: reduction elements per LDS stage.  32, or 64 for bf16 operands through the vector gather: the stage then has the bytes of an
// fp32 stage of 32 (same LDS footprint), twice the MFMAs between two barriers, and needs Cin % 64 == 0 (p.kchunks counts stages of BK).
template <int BM, int BN, int MODE, bool BF, bool INAFF = false, int ACT = 0, bool STATS = false, int BK = kBK>
__global__ __launch_bounds__(kConvThreads, igemm_occupancy(BM, BN)) void igemm_kernel(IgemmP p)
{
    static_assert(BK == kBK || (BK == 2 * kBK && BF && MODE <= 1), "long stages exist for bf16 operands through the vector gather");
    constexpr int LDH = BK + 8;                // row of 16-bit elements: 80 or 144 bytes (the latter = an fp32 row of 32 + 4)
    constexpr int TPR = BK / 4, ROWS = kConvThreads / TPR;  // threads per row of a stage with 16-byte loads of fp32, rows per pass
    static_assert(!INAFF || MODE == 0, "the fused input transform exists for the vector gather only");
    static_assert(ACT == 0 || BF, "bf16 activations are multiplied on the bf16 MFMA");
    constexpr bool A16 = ACT == 1, O16 = ACT != 0;
    constexpr bool AV16 = A16 && MODE <= 1;    // vector gather of bf16: 8 elements per load, 4 loads per row of a stage
    constexpr int WTM = BM / 2, WTN = BN / 2, MI = WTM / 32, NI = WTN / 32;
    constexpr int ATPR = AV16 ? BK / 8 : TPR;  // threads per gathered row (eight bf16 or four fp32 elements per load)
    constexpr int AROWS = kConvThreads / ATPR;  // rows of the gathered tile one pass of the workgroup's loads covers
    constexpr int RA = BM / AROWS, RB = BN / ROWS;  // rows per thread of each operand tile
    static_assert(BM % AROWS == 0 && BN % ROWS == 0, "whole passes");
    __shared__ __attribute__((aligned(16))) float As[BM * kLDK];
    __shared__ __attribute__((aligned(16))) float Bs[BN * kLDK];
    __shared__ float s_stat[2][STATS ? BN : 1];  // column statistics of a tile's second row half, on their way to the first half's wavefronts

    // The kernels of the step's main chain (forward pass, data gradients, BN backward) raise the issue priority of their
    // wavefronts; the filter gradients, which run beside them on another stream and are needed only at the end of the pass, keep
    // the default (lowest).  Where wavefronts of both share a SIMD the chain's instructions go first.
    main_chain_priority();
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int kq = tid % TPR, row_in = tid / TPR;
    const int akq = tid % ATPR, arow = tid / ATPR;  // this thread's piece of a gathered row, and its row
    const bf16_t *a16 = reinterpret_cast<const bf16_t *>(p.a);
    const int G = gridDim.x;
    const int n_items = p.full_items + p.tail_tiles * p.tail_split;
    // MFMA operand for lane l: row l%32 of the block, reduction element l/32 of the current pair.  A lane
    // reads four consecutive reduction elements at once; pairing element e of lanes 0-31 with element e
    // of lanes 32-63 is a permutation of the reduction order, applied identically to both operands.
    const int frag_off = (lane & 31) * kLDK + (lane >> 5) * 4;

    for (int item = blockIdx.x; item < n_items; item += G) {
        int tile, kc_begin, kc_end;
        float *part = nullptr;
        if (item < p.full_items) {
            // within a round of G items, consecutive workgroups sit on different XCDs (round-robin dispatch):
            // give each XCD a contiguous range of tiles so that tiles sharing activations share an L2
            const int round = item / G, i = item - round * G;
            tile = round * G + (i & 7) * (G >> 3) + (i >> 3);
            kc_begin = 0;
            kc_end = p.kchunks;
        } else {
            const int piece = item - p.full_items;
            const int tt = piece / p.tail_split, sp = piece - tt * p.tail_split;
            tile = p.full_items + tt;
            kc_begin = sp * p.tail_chunks;
            kc_end = min(p.kchunks, kc_begin + p.tail_chunks);
            if (p.tail_split > 1) part = p.partial + (long)piece * (BM * BN);
        }
        const int tm = tile / p.tiles_n, tn = tile - tm * p.tiles_n;
        const int m0 = tm * BM, n0 = tn * BN;

        // per-row geometry of the gathered operand
        // Offsets into the gathered tensor are 32-bit element counts (every tensor has fewer than 2^31 elements) built
        // with 24-bit multiplies (rows*columns and the channel count are below 2^24): the 64-bit and full 32-bit integer
        // multiplies run at a quarter of the rate and sit in the inner loop.
        int hn[RA], wnum[RA];
        int abase[RA];
#pragma unroll
        for (int i = 0; i < RA; ++i) {
            const int m = m0 + arow + AROWS * i;
            if (m < p.M) {
                int cls, n, oh, ow;
                decode_row(p, m, cls, n, oh, ow);
                if (p.scatter2 == 2) {
                    oh = 2 * oh + (cls >> 1);
                    ow = 2 * ow + (cls & 1);
                }
                hn[i] = oh * p.so + p.off;
                wnum[i] = ow * p.so + p.off;
                abase[i] = n * (p.IH * p.IW * p.Cin);
            } else {
                hn[i] = -(1 << 28);  // every tap falls outside
                wnum[i] = 0;
                abase[i] = 0;
            }
        }

        float4 ra[RA], rb[RB];
        uint4 ra16[RA];                                                 // AV16: eight bf16 elements per register
        float4 in_sc = make_float4(0.f, 0.f, 0.f, 0.f), in_sh = in_sc;  // INAFF: scale and shift of this thread's four channels
        float4 in_sc2 = in_sc, in_sh2 = in_sc;                          // INAFF with AV16: of the next four
        unsigned in_ok = 0;                                             // INAFF: bit i set when ra[i] was loaded (not padding)
        auto load_chunk = [&](int kc) {
            const int k0 = kc * BK;
            if (MODE <= 1) {
                const int tap = (int)fdiv(k0, p.div_cin);
                const int c0 = k0 - tap * p.Cin + akq * (AV16 ? 8 : 4);
                const int r = (int)fdiv(tap, p.div_s), s = tap - r * p.S;
                if (INAFF) {
                    in_sc = ldg4(p.in_scale + c0);
                    in_sh = ldg4(p.in_shift + c0);
                    if (AV16) {
                        in_sc2 = ldg4(p.in_scale + c0 + 4);
                        in_sh2 = ldg4(p.in_shift + c0 + 4);
                    }
                    in_ok = 0;
                }
#pragma unroll
                for (int i = 0; i < RA; ++i) {
                    int ih = hn[i] + r, iw = wnum[i] + s;
                    bool ok = ih >= 0 && iw >= 0;
                    if (MODE == 1) {
                        if (p.sd == 2) {  // the common dilation: no integer division in the inner loop
                            ok = ok && ((ih | iw) & 1) == 0;
                            ih >>= 1;
                            iw >>= 1;
                        } else {
                            ok = ok && (ih % p.sd == 0) && (iw % p.sd == 0);
                            ih /= p.sd;
                            iw /= p.sd;
                        }
                    }
                    ok = ok && ih < p.IH && iw < p.IW;
                    const unsigned aoff = (unsigned)(abase[i] + (int)__umul24(__umul24(ih, p.IW) + iw, p.Cin) + c0);
                    if (AV16) ra16[i] = ok ? *reinterpret_cast<const uint4 *>(a16 + aoff) : make_uint4(0u, 0u, 0u, 0u);
                    else ra[i] = ok ? ldg4(p.a + aoff) : make_float4(0.f, 0.f, 0.f, 0.f);
                    if (INAFF && ok) in_ok |= 1u << i;
                }
#pragma unroll
                for (int i = 0; i < RB; ++i) {
                    const int j = n0 + row_in + ROWS * i;
                    rb[i] = j < p.Nout ? ldg4(p.b + (long)j * p.Kdim + k0 + kq * 4) : make_float4(0.f, 0.f, 0.f, 0.f);
                }
            } else {
                float va[RA][4], vb[RB][4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int k = k0 + kq * 4 + e;
                    const bool kin = k < p.Kdim;
                    const int tap = (int)fdiv(k, p.div_cin), c = k - tap * p.Cin;
                    const int r = (int)fdiv(tap, p.div_s), s = tap - r * p.S;
#pragma unroll
                    for (int i = 0; i < RA; ++i) {
                        int ih = hn[i] + r, iw = wnum[i] + s;
                        bool ok = kin && ih >= 0 && iw >= 0;
                        if (p.sd != 1) {  // forward passes (sd == 1) pay no integer division here
                            ok = ok && (ih % p.sd == 0) && (iw % p.sd == 0);
                            ih /= p.sd;
                            iw /= p.sd;
                        }
                        ok = ok && ih < p.IH && iw < p.IW;
                        const unsigned aoff = (unsigned)(abase[i] + (int)__umul24(__umul24(ih, p.IW) + iw, p.Cin) + c);
                        if (A16) va[i][e] = ok ? bf16_lo(a16[aoff]) : 0.f;
                        else va[i][e] = ok ? p.a[aoff] : 0.f;
                    }
#pragma unroll
                    for (int i = 0; i < RB; ++i) {
                        const int j = n0 + row_in + ROWS * i;
                        vb[i][e] = (kin && j < p.Nout) ? p.b[(long)j * p.Kdim + k] : 0.f;
                    }
                }
#pragma unroll
                for (int i = 0; i < RA; ++i) ra[i] = make_float4(va[i][0], va[i][1], va[i][2], va[i][3]);
#pragma unroll
                for (int i = 0; i < RB; ++i) rb[i] = make_float4(vb[i][0], vb[i][1], vb[i][2], vb[i][3]);
            }
        };
        auto store_chunk = [&]() {
            if (AV16) {
                uint16_t *ah = reinterpret_cast<uint16_t *>(As), *bh = reinterpret_cast<uint16_t *>(Bs);
#pragma unroll
                for (int i = 0; i < RA; ++i) {
                    uint4 v = ra16[i];
                    if (INAFF && (in_ok & (1u << i))) {
                        // the BN + ReLU output as the normalising kernel would have stored it: fp32 arithmetic, one rounding
                        v.x = bf16_pack2(fmaxf(fmaf(bf16_lo(v.x), in_sc.x, in_sh.x), 0.f), fmaxf(fmaf(bf16_hi(v.x), in_sc.y, in_sh.y), 0.f));
                        v.y = bf16_pack2(fmaxf(fmaf(bf16_lo(v.y), in_sc.z, in_sh.z), 0.f), fmaxf(fmaf(bf16_hi(v.y), in_sc.w, in_sh.w), 0.f));
                        v.z = bf16_pack2(fmaxf(fmaf(bf16_lo(v.z), in_sc2.x, in_sh2.x), 0.f), fmaxf(fmaf(bf16_hi(v.z), in_sc2.y, in_sh2.y), 0.f));
                        v.w = bf16_pack2(fmaxf(fmaf(bf16_lo(v.w), in_sc2.z, in_sh2.z), 0.f), fmaxf(fmaf(bf16_hi(v.w), in_sc2.w, in_sh2.w), 0.f));
                    }
                    *reinterpret_cast<uint4 *>(&ah[(arow + AROWS * i) * LDH + akq * 8]) = v;
                }
#pragma unroll
                for (int i = 0; i < RB; ++i)
                    *reinterpret_cast<uint2 *>(&bh[(row_in + ROWS * i) * LDH + kq * 4]) =
                        make_uint2(bf16_pack2(rb[i].x, rb[i].y), bf16_pack2(rb[i].z, rb[i].w));
                return;
            }
            if (INAFF) {
#pragma unroll
                for (int i = 0; i < RA; ++i)
                    if (in_ok & (1u << i)) {
                        ra[i].x = fmaxf(fmaf(ra[i].x, in_sc.x, in_sh.x), 0.f);
                        ra[i].y = fmaxf(fmaf(ra[i].y, in_sc.y, in_sh.y), 0.f);
                        ra[i].z = fmaxf(fmaf(ra[i].z, in_sc.z, in_sh.z), 0.f);
                        ra[i].w = fmaxf(fmaf(ra[i].w, in_sc.w, in_sh.w), 0.f);
                    }
            }
            if (BF) {
                uint16_t *ah = reinterpret_cast<uint16_t *>(As), *bh = reinterpret_cast<uint16_t *>(Bs);
#pragma unroll
                for (int i = 0; i < RA; ++i)
                    *reinterpret_cast<uint2 *>(&ah[(row_in + ROWS * i) * LDH + kq * 4]) =
                        make_uint2(bf16_pack2(ra[i].x, ra[i].y), bf16_pack2(ra[i].z, ra[i].w));
#pragma unroll
                for (int i = 0; i < RB; ++i)
                    *reinterpret_cast<uint2 *>(&bh[(row_in + ROWS * i) * LDH + kq * 4]) =
                        make_uint2(bf16_pack2(rb[i].x, rb[i].y), bf16_pack2(rb[i].z, rb[i].w));
                return;
            }
#pragma unroll
            for (int i = 0; i < RA; ++i) *reinterpret_cast<float4 *>(&As[(row_in + ROWS * i) * kLDK + kq * 4]) = ra[i];
#pragma unroll
            for (int i = 0; i < RB; ++i) *reinterpret_cast<float4 *>(&Bs[(row_in + ROWS * i) * kLDK + kq * 4]) = rb[i];
        };

        floatx16 acc[MI][NI];
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

        // Row order 2, tile inside one parity class (ph, pw): tap (r, s) reaches a row only when ph + off + r and
        // pw + off + s are multiples of the dilation (2): the other chunks are skipped.  Uniform over the workgroup.
        int skip_ph = -1, skip_pw = 0;
        if (MODE == 1 && p.scatter2 == 2) {
            const int mq = p.M >> 2, c0 = m0 / mq, c1 = min(m0 + BM - 1, p.M - 1) / mq;
            if (c0 == c1) {
                skip_ph = c0 >> 1;
                skip_pw = c0 & 1;
            }
        }
        auto next_chunk = [&](int kc) {
            if (MODE != 1 || skip_ph < 0) return kc;
            for (; kc < kc_end; ++kc) {
                const int tap = (int)fdiv(kc * BK, p.div_cin);
                const int r = (int)fdiv(tap, p.div_s), sx = tap - r * p.S;
                if ((((skip_ph + p.off + r) | (skip_pw + p.off + sx)) & 1) == 0) break;
            }
            return kc;
        };
        int kc = next_chunk(kc_begin);
        if (kc < kc_end) {
            load_chunk(kc);
            store_chunk();  // the previous item's last reads of LDS are fenced by the barrier that ended its loop
            __syncthreads();
        }
        while (kc < kc_end) {
            const int kc_next = next_chunk(kc + 1);
            const bool more = kc_next < kc_end;
            if (more) load_chunk(kc_next);  // in flight while the current stage is multiplied
            __builtin_amdgcn_s_setprio(3);  // a wavefront that multiplies goes before one that computes addresses
            if (BF) {
                // lane l: row l%32 of the block, eight consecutive reduction elements (l/32)*8.. of the 16 of one MFMA
                const uint16_t *ah = reinterpret_cast<const uint16_t *>(As), *bh = reinterpret_cast<const uint16_t *>(Bs);
                const int hoff = (lane & 31) * LDH + (lane >> 5) * 8;
#pragma unroll
                for (int ks = 0; ks < BK / 16; ++ks) {
                    bf16x8 ah8[MI], bh8[NI];
#pragma unroll
                    for (int i = 0; i < MI; ++i) ah8[i] = *reinterpret_cast<const bf16x8 *>(&ah[(wm * WTM + i * 32) * LDH + hoff + ks * 16]);
#pragma unroll
                    for (int j = 0; j < NI; ++j) bh8[j] = *reinterpret_cast<const bf16x8 *>(&bh[(wn * WTN + j * 32) * LDH + hoff + ks * 16]);
#pragma unroll
                    for (int i = 0; i < MI; ++i)
#pragma unroll
                        for (int j = 0; j < NI; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah8[i], bh8[j], acc[i][j], 0, 0, 0);
                }
            } else if constexpr (BM == 128 && BN == 64) {
                // no registers to spare for a second fragment set here (it spills)
#pragma unroll
                for (int kg = 0; kg < kBK / 8; ++kg) {
                    float4 af[MI], bf[NI];
#pragma unroll
                    for (int i = 0; i < MI; ++i) af[i] = *reinterpret_cast<const float4 *>(&As[(wm * WTM + i * 32) * kLDK + frag_off + kg * 8]);
#pragma unroll
                    for (int j = 0; j < NI; ++j) bf[j] = *reinterpret_cast<const float4 *>(&Bs[(wn * WTN + j * 32) * kLDK + frag_off + kg * 8]);
#pragma unroll
                    for (int e = 0; e < 4; ++e)
#pragma unroll
                        for (int i = 0; i < MI; ++i)
#pragma unroll
                            for (int j = 0; j < NI; ++j) {
                                const float av = e == 0 ? af[i].x : e == 1 ? af[i].y : e == 2 ? af[i].z : af[i].w;
                                const float bv = e == 0 ? bf[j].x : e == 1 ? bf[j].y : e == 2 ? bf[j].z : bf[j].w;
                                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[i][j], 0, 0, 0);
                            }
                }
            } else {
                // The fragments of group kg+1 are read from LDS while the MFMAs of group kg run (two register sets); the
                // scheduling hints keep that order: read, then multiply, group by group.  Read and used back to back, every
                // group would start with the latency of its LDS reads.
                float4 af[2][MI], bf[2][NI];
                auto load_frag = [&](int set, int kg) {
#pragma unroll
                    for (int i = 0; i < MI; ++i) af[set][i] = *reinterpret_cast<const float4 *>(&As[(wm * WTM + i * 32) * kLDK + frag_off + kg * 8]);
#pragma unroll
                    for (int j = 0; j < NI; ++j) bf[set][j] = *reinterpret_cast<const float4 *>(&Bs[(wn * WTN + j * 32) * kLDK + frag_off + kg * 8]);
                };
                load_frag(0, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, MI + NI, 0);
#pragma unroll
                for (int kg = 0; kg < kBK / 8; ++kg) {
                    if (kg + 1 < kBK / 8) {
                        load_frag((kg + 1) & 1, kg + 1);
                        __builtin_amdgcn_sched_group_barrier(0x100, MI + NI, 0);
                    }
                    // consecutive MFMAs go to different accumulators
#pragma unroll
                    for (int e = 0; e < 4; ++e)
#pragma unroll
                        for (int i = 0; i < MI; ++i)
#pragma unroll
                            for (int j = 0; j < NI; ++j) {
                                const float4 a4 = af[kg & 1][i], b4 = bf[kg & 1][j];
                                const float av = e == 0 ? a4.x : e == 1 ? a4.y : e == 2 ? a4.z : a4.w;
                                const float bv = e == 0 ? b4.x : e == 1 ? b4.y : e == 2 ? b4.z : b4.w;
                                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[i][j], 0, 0, 0);
                            }
                    __builtin_amdgcn_sched_group_barrier(0x008, 4 * MI * NI, 0);
                }
            }
            __syncthreads();
            __builtin_amdgcn_s_setprio(2);
            if (more) {
                store_chunk();
                __syncthreads();
            }
            kc = kc_next;
        }

        // Column statistics of the tile (whole tiles only: the pieces of a split tile are added up by another kernel, which
        // gathers them there), before the tile is written out: the wavefronts have just left the loop's last barrier together, so
        // the barrier below costs little here, and the write-out that follows stays unsynchronised (behind the stores it would
        // make every wavefront wait for the slowest one's).  A wavefront holds WTM rows of its columns, 16 per block in each
        // half-wave: mean and squared deviations of those in two passes over the registers, then the two row halves of the tile
        // are merged with the pairwise update of Chan et al. by the wavefronts of the first half.  Uniform over the workgroup.
        if (STATS && !part) {
            const int valid = min(WTM, p.M - (m0 + wm * WTM));  // rows of this wavefront inside the matrix (may be <= 0)
            // element e of block i is row i*32 + 8*(e/4) + e%4 + 4*(lane/32) of the wavefront: inside when the lane-free part
            // is below vlim (one register, against compile-time constants)
            const int vlim = valid - 4 * (lane >> 5);
            float cmean[NI], cm2[NI];
            if (O16) {  // the statistics are those of the tensor as stored (rounding is idempotent: the stores below round again)
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int j = 0; j < NI; ++j)
#pragma unroll
                        for (int e = 0; e < 16; ++e) acc[i][j][e] = bf16_round(acc[i][j][e]);
            }
            const bool whole = valid == WTM;  // uniform over the wavefront: no row needs masking
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                float sum = 0.f;
                if (whole) {
#pragma unroll
                    for (int i = 0; i < MI; ++i)
#pragma unroll
                        for (int e = 0; e < 16; ++e) sum += acc[i][j][e];
                } else {
#pragma unroll
                    for (int i = 0; i < MI; ++i)
#pragma unroll
                        for (int e = 0; e < 16; ++e) sum += i * 32 + 8 * (e >> 2) + (e & 3) < vlim ? acc[i][j][e] : 0.f;
                }
                sum += __shfl_xor(sum, 32, 64);
                const float mean = valid > 0 ? sum / (float)valid : 0.f;
                float dev = 0.f;
                if (whole) {
#pragma unroll
                    for (int i = 0; i < MI; ++i)
#pragma unroll
                        for (int e = 0; e < 16; ++e) {
                            const float d = acc[i][j][e] - mean;
                            dev = fmaf(d, d, dev);
                        }
                } else {
#pragma unroll
                    for (int i = 0; i < MI; ++i)
#pragma unroll
                        for (int e = 0; e < 16; ++e) {
                            const float d = acc[i][j][e] - mean;
                            dev = i * 32 + 8 * (e >> 2) + (e & 3) < vlim ? fmaf(d, d, dev) : dev;
                        }
                }
                dev += __shfl_xor(dev, 32, 64);
                cmean[j] = mean;
                cm2[j] = dev;
                if (wm == 1 && lane < 32) {
                    s_stat[0][wn * WTN + j * 32 + lane] = mean;
                    s_stat[1][wn * WTN + j * 32 + lane] = dev;
                }
            }
            __syncthreads();  // the next write of s_stat comes after the barriers of the next item's loop
            if (wm == 0 && lane < 32) {
                const float na = (float)valid, nb = (float)max(0, min(WTM, p.M - (m0 + WTM)));
#pragma unroll
                for (int j = 0; j < NI; ++j) {
                    const int cl = wn * WTN + j * 32 + lane, col = n0 + cl;
                    float mean = cmean[j], m2 = cm2[j];
                    if (nb > 0.f) {
                        const float nt = na + nb, d = s_stat[0][cl] - mean;
                        mean = fmaf(d, nb / nt, mean);
                        m2 = m2 + s_stat[1][cl] + d * d * (na * nb / nt);
                    }
                    if (col < p.Nout) {
                        p.stat_mean[(long)tm * p.Nout + col] = mean;
                        p.stat_m2[(long)tm * p.Nout + col] = m2;
                    }
                }
            }
        }
        // Epilogue.  Accumulator element e of lane l is row 8*(e/4) + 4*(l/32) + e%4, column l%32 of its block.
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int rl = wm * WTM + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                if (part) {
#pragma unroll
                    for (int j = 0; j < NI; ++j) part[rl * BN + wn * WTN + j * 32 + (lane & 31)] = acc[i][j][e];
                } else {
                    const int m = m0 + rl;
                    if (m >= p.M) continue;
                    const long row = out_row_index(p, m);
#pragma unroll
                    for (int j = 0; j < NI; ++j) {
                        const int col = n0 + wn * WTN + j * 32 + (lane & 31);
                        if (col < p.Nout) store_out<O16>(p, row, col, acc[i][j][e]);
                    }
                }
            }

    }
}

// Adds the pieces of every tail tile in piece order and writes the tile (one thread per four columns).
template <int BM, int BN, bool O16 = false>
__global__ __launch_bounds__(256) void igemm_tail_reduce_kernel(IgemmP p)
{
    main_chain_priority();
    constexpr int V = BM * BN / 4;
    const int tt = blockIdx.y;
    const int v = blockIdx.x * 256 + threadIdx.x;
    if (v >= V) return;
    const float *src = p.partial + (long)tt * p.tail_split * (BM * BN);
    // pieces are added in piece order; four loads are in flight at once (one at a time is a chain of memory round trips)
    float4 acc = reinterpret_cast<const float4 *>(src)[v];
    int s = 1;
    for (; s + 3 < p.tail_split; s += 4) {
        float4 t[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) t[u] = reinterpret_cast<const float4 *>(src + (long)(s + u) * (BM * BN))[v];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            acc.x += t[u].x; acc.y += t[u].y; acc.z += t[u].z; acc.w += t[u].w;
        }
    }
    for (; s < p.tail_split; ++s) {
        const float4 t = reinterpret_cast<const float4 *>(src + (long)s * (BM * BN))[v];
        acc.x += t.x; acc.y += t.y; acc.z += t.z; acc.w += t.w;
    }
    const int tile = p.full_items + tt;
    const int tm = tile / p.tiles_n, tn = tile - tm * p.tiles_n;
    const int rl = (v * 4) / BN, cl = (v * 4) - rl * BN;
    const int m = tm * BM + rl;
    if (m >= p.M) return;
    const long row = out_row_index(p, m);
    const int col = tn * BN + cl;
    if (!p.scatter2 && (p.Nout & 3) == 0) {  // rows of whole 16-byte groups
        if (col < p.Nout) {
            if (O16) st4(reinterpret_cast<bf16_t *>(p.out), (size_t)(row * p.Nout + col) / 4, acc);
            else *reinterpret_cast<float4 *>(&p.out[row * p.Nout + col]) = acc;
        }
        return;
    }
    const float vals[4] = {acc.x, acc.y, acc.z, acc.w};
#pragma unroll
    for (int e = 0; e < 4; ++e)
        if (col + e < p.Nout) store_out<O16>(p, row, col + e, vals[e]);
}

// The same sum for a launch that gathers the output's batch statistics (IgemmP::stat_mean): a workgroup owns 32 columns of one
// tail tile, thread = (row lane, four columns), so that the rows of a column meet in one workgroup: the column sums and then
// the squared deviations from the column mean are merged over the row lanes by shuffles inside a wavefront and through LDS
// across the four wavefronts, in a fixed order.  grid = (BN / 32, tail tiles).
template <int BM, int BN, bool O16 = false>
__global__ __launch_bounds__(256) void igemm_tail_reduce_stats_kernel(IgemmP p)
{
    main_chain_priority();
    constexpr int RPT = BM / 32;  // rows per thread: row lane, row lane + 32, ...
    __shared__ float4 s_red[4][8];
    const int tt = blockIdx.y, cgrp = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c4 = tid & 7, rlane = tid >> 3;
    const int tile = p.full_items + tt;
    const int tm = tile / p.tiles_n, tn = tile - tm * p.tiles_n;
    const int cl = cgrp * 32 + c4 * 4, col = tn * BN + cl;
    const float *src = p.partial + (long)tt * p.tail_split * (BM * BN);
    float4 acc[RPT];
#pragma unroll
    for (int u = 0; u < RPT; ++u) acc[u] = *reinterpret_cast<const float4 *>(src + (rlane + 32 * u) * BN + cl);
    for (int s = 1; s < p.tail_split; ++s) {  // piece order; the rows of a piece are in flight together
        float4 t[RPT];
#pragma unroll
        for (int u = 0; u < RPT; ++u) t[u] = *reinterpret_cast<const float4 *>(src + (long)s * (BM * BN) + (rlane + 32 * u) * BN + cl);
#pragma unroll
        for (int u = 0; u < RPT; ++u) {
            acc[u].x += t[u].x; acc[u].y += t[u].y; acc[u].z += t[u].z; acc[u].w += t[u].w;
        }
    }
    const int valid = min(BM, p.M - tm * BM);  // rows of the tile inside the matrix (>= 1)
#pragma unroll
    for (int u = 0; u < RPT; ++u) {
        const int rl = rlane + 32 * u;
        if (rl >= valid) continue;
        const long row = out_row_index(p, tm * BM + rl);
        if (!p.scatter2 && (p.Nout & 3) == 0) {
            if (col < p.Nout) {
                if (O16) st4(reinterpret_cast<bf16_t *>(p.out), (size_t)(row * p.Nout + col) / 4, acc[u]);
                else *reinterpret_cast<float4 *>(&p.out[row * p.Nout + col]) = acc[u];
            }
        } else {
            const float vals[4] = {acc[u].x, acc[u].y, acc[u].z, acc[u].w};
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (col + e < p.Nout) store_out<O16>(p, row, col + e, vals[e]);
        }
        if (O16) acc[u] = make_float4(bf16_round(acc[u].x), bf16_round(acc[u].y), bf16_round(acc[u].z), bf16_round(acc[u].w));
    }
    // sum of v over the workgroup's row lanes, valid in every thread: lane bits 3-5 by a butterfly (both partners add lower
    // lane + upper lane), the wavefronts in wavefront order
    auto column_total = [&](float4 v) {
#pragma unroll
        for (int off = 8; off < 64; off <<= 1) {
            const float4 q = make_float4(__shfl_xor(v.x, off, 64), __shfl_xor(v.y, off, 64), __shfl_xor(v.z, off, 64), __shfl_xor(v.w, off, 64));
            const bool lower = (lane & off) == 0;
            v = lower ? make_float4(v.x + q.x, v.y + q.y, v.z + q.z, v.w + q.w) : make_float4(q.x + v.x, q.y + v.y, q.z + v.z, q.w + v.w);
        }
        __syncthreads();  // the previous total has been read by everyone
        if (lane < 8) s_red[wave][lane] = v;
        __syncthreads();
        float4 t = s_red[0][c4];
#pragma unroll
        for (int w = 1; w < 4; ++w) {
            const float4 q = s_red[w][c4];
            t = make_float4(t.x + q.x, t.y + q.y, t.z + q.z, t.w + q.w);
        }
        return t;
    };
    float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int u = 0; u < RPT; ++u)
        if (rlane + 32 * u < valid) sum = make_float4(sum.x + acc[u].x, sum.y + acc[u].y, sum.z + acc[u].z, sum.w + acc[u].w);
    sum = column_total(sum);
    const float inv = 1.f / (float)valid;
    const float4 mean = make_float4(sum.x * inv, sum.y * inv, sum.z * inv, sum.w * inv);
    float4 dev = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int u = 0; u < RPT; ++u)
        if (rlane + 32 * u < valid) {
            const float dx = acc[u].x - mean.x, dy = acc[u].y - mean.y, dz = acc[u].z - mean.z, dw = acc[u].w - mean.w;
            dev = make_float4(fmaf(dx, dx, dev.x), fmaf(dy, dy, dev.y), fmaf(dz, dz, dev.z), fmaf(dw, dw, dev.w));
        }
    dev = column_total(dev);
    if (tid < 8) {
        const float m4[4] = {mean.x, mean.y, mean.z, mean.w}, d4[4] = {dev.x, dev.y, dev.z, dev.w};
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (col + e < p.Nout) {
                p.stat_mean[(long)tm * p.Nout + col + e] = m4[e];
                p.stat_m2[(long)tm * p.Nout + col + e] = d4[e];
            }
    }
}

// ---------------------------------------------------------------------------------------------------
// Forward convolution of the network's first layer (3 input channels, 7x7, stride 2, pad 3, 64 filters).  With three
// channels the implicit GEMM's gather is one scalar load per element and decodes (r, s, c) for each of them.  Here a
// workgroup owns a tile of 8 x 16 output pixels: the 21 x 37 input pixels under it are loaded once, row by row and
// coalesced, into LDS, the whole filter lives in LDS for the life of the workgroup, and the MFMA operands are read from
// LDS at computed offsets.  The 7 taps x 3 channels of a filter row are 21 consecutive floats of an image row; a patch row
// keeps them in order with one unused float after every second input pixel, so that neighbouring output pixels are 7 floats
// apart instead of 6 and the 32 pixels of a wavefront (2 rows x 16 columns, rows 2*pitch apart) read 32 different LDS banks:
// pixel (r, c) of the tile and element j of filter row fr sit at patch[(2r + fr)*pitch + 7c + j + j/6].
// Reduction index: (fr, j) with j < 22, the 22nd element carrying a zero weight; lanes 0-31 take even j, lanes 32-63 odd j.
struct StemP {
    const float *x;  // N x IH x IW x 3
    const float *w;  // 64 x 7 x 7 x 3
    float *y;        // N x OH x OW x 64
    int N, IH, IW, OH, OW;
    int tiles_h, tiles_w, ntiles;
};
constexpr int kStemTH = 8, kStemTW = 16;
constexpr int kStemRows = 2 * kStemTH + 5;           // 21 input rows under a tile
constexpr int kStemCols = (2 * kStemTW + 5) * 3;     // 111 floats of each
constexpr int kStemPitch = 136;                      // 37 pixels x 3 + 18 unused floats, rounded up to 8 mod 16
constexpr int kStemLoads = (kStemRows * kStemCols + kConvThreads - 1) / kConvThreads;

static __global__ __launch_bounds__(kConvThreads, 3) void stem_fwd_kernel(StemP p)
{
    __shared__ float patch[kStemRows * kStemPitch];
    __shared__ float wl[7 * 11 * 2 * 64];  // [filter row][pair of elements][element of the pair][filter]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // the filter is read in its own order (coalesced) and scattered into the LDS layout; the 22nd element of each row is zero
    for (int i = tid; i < 64 * 147; i += kConvThreads) {
        const int n = i / 147, rem = i - n * 147;
        const int fr = rem / 21, j = rem - fr * 21;
        wl[((fr * 11 + (j >> 1)) * 2 + (j & 1)) * 64 + n] = p.w[i];
    }
    for (int i = tid; i < 7 * 64; i += kConvThreads) wl[(((i >> 6) * 11 + 10) * 2 + 1) * 64 + (i & 63)] = 0.f;
    // the floats the loads never write (the unused ones and the one the zero-weight element reads) must not hold NaNs
    for (int i = tid; i < kStemRows * kStemPitch; i += kConvThreads) patch[i] = 0.f;
    __syncthreads();

    const int pix = lane & 31, half = lane >> 5;
    const int tr = 2 * wave + (pix >> 4), tc = pix & 15;  // this lane's pixel of the tile, as the A operand's row
    const int abase = 2 * tr * kStemPitch + 7 * tc + half;
    const int bbase = half * 64 + pix;

    // the patch of the next tile is loaded into registers while the current tile is multiplied
    float v[kStemLoads];
    auto load_patch = [&](int tile) {
        const int n = tile / (p.tiles_h * p.tiles_w), rem = tile - n * (p.tiles_h * p.tiles_w);
        const int th = rem / p.tiles_w, tw = rem - th * p.tiles_w;
        const int ih0 = 2 * th * kStemTH - 3, if0 = (2 * tw * kStemTW - 3) * 3;  // first input row; first float of the input rows
#pragma unroll
        for (int u = 0; u < kStemLoads; ++u) {
            const int i = tid + u * kConvThreads;
            const int pr = i / kStemCols, pc = i - pr * kStemCols;
            const int ih = ih0 + pr, f = if0 + pc;
            const bool ok = i < kStemRows * kStemCols && ih >= 0 && ih < p.IH && f >= 0 && f < p.IW * 3;
            v[u] = ok ? p.x[((long)n * p.IH + ih) * (p.IW * 3) + f] : 0.f;
        }
    };
    if ((int)blockIdx.x < p.ntiles) load_patch(blockIdx.x);
    for (int tile = blockIdx.x; tile < p.ntiles; tile += gridDim.x) {
        const int n = tile / (p.tiles_h * p.tiles_w), rem = tile - n * (p.tiles_h * p.tiles_w);
        const int th = rem / p.tiles_w, tw = rem - th * p.tiles_w;
        const int oh0 = th * kStemTH, ow0 = tw * kStemTW;
#pragma unroll
        for (int u = 0; u < kStemLoads; ++u) {
            const int i = tid + u * kConvThreads;
            const int pr = i / kStemCols, pc = i - pr * kStemCols;
            const int px = pc / 3;  // input pixel of the patch row
            if (i < kStemRows * kStemCols) patch[pr * kStemPitch + pc + (px >> 1)] = v[u];
        }
        __syncthreads();
        if (tile + (int)gridDim.x < p.ntiles) load_patch(tile + gridDim.x);

        floatx16 acc[2];
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
        // the operands of filter row fr+1 are read from LDS while the 22 MFMAs of row fr run (two register sets; the scheduling
        // hints keep that order)
        float av[2][11], bv[2][11][2];
        auto load_row = [&](int set, int fr) {
#pragma unroll
            for (int t = 0; t < 11; ++t) {
                av[set][t] = patch[abase + fr * kStemPitch + 2 * t + (2 * t) / 6];
                bv[set][t][0] = wl[(fr * 11 + t) * 128 + bbase];
                bv[set][t][1] = wl[(fr * 11 + t) * 128 + 32 + bbase];
            }
        };
        load_row(0, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 22, 0);
#pragma unroll
        for (int fr = 0; fr < 7; ++fr) {
            if (fr + 1 < 7) {
                load_row((fr + 1) & 1, fr + 1);
                __builtin_amdgcn_sched_group_barrier(0x100, 22, 0);
            }
#pragma unroll
            for (int t = 0; t < 11; ++t) {
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[fr & 1][t], bv[fr & 1][t][0], acc[0], 0, 0, 0);
                acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[fr & 1][t], bv[fr & 1][t][1], acc[1], 0, 0, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, 22, 0);
        }
        // accumulator element e of lane l: row 8*(e/4) + 4*(l/32) + e%4 of the wavefront's 32 pixels, column l%32 of its block
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int q = 8 * (e >> 2) + 4 * half + (e & 3);
            const int oh = oh0 + 2 * wave + (q >> 4), ow = ow0 + (q & 15);
            if (oh < p.OH && ow < p.OW) {
                float *o = p.y + (((long)n * p.OH + oh) * p.OW + ow) * 64 + pix;
                o[0] = acc[0][e];
                o[32] = acc[1][e];
            }
        }
        __syncthreads();  // every wavefront is done with the patch before the next tile overwrites it
    }
}

// ---------------------------------------------------------------------------------------------------
// Filter gradient of the network's first layer (3 channels, 7x7, stride 2, pad 3, 64 filters): dw[k][fr][j] = sum over output
// pixels of dy[pixel][k] * x[2*oh + fr - 3][(2*ow - 3)*3 + j], j = 0..20 the 7 taps x 3 channels of a filter row, which are 21
// consecutive floats of an image row.  Same tiling as stem_fwd_kernel: a workgroup takes 8 x 16 output pixels at a time, the 21 x 37
// input pixels under them go to LDS once (same bank layout), and so do the tile's 128 x 64 values of dy.  The product is
// [64 filters] x [128 pixels] x [147 -> 160 filter elements]: ten 32x32 blocks, reduced over pixel pairs; each wavefront takes the
// 32 pixels of two tile rows for all ten blocks (160 accumulator registers) and keeps accumulating over every tile of the
// persistent workgroup, so the four wavefronts' sums meet only once, at the end, through LDS in wavefront order.  The workgroup
// leaves one partial [64][147]; the ordered sum over workgroups is splitk_reduce_kernel's.
struct StemWP {
    const float *x;   // N x IH x IW x 3
    const float *dy;  // N x OH x OW x 64
    float *part;      // [workgroups][64][147]
    int N, IH, IW, OH, OW;
    int tiles_h, tiles_w, ntiles;
};
constexpr int kStemDyLoads = kStemTH * kStemTW * 64 / 4 / kConvThreads;  // 16-byte loads of dy per thread and tile

static __global__ __launch_bounds__(kConvThreads, 2) void stem_wgrad_kernel(StemWP p)
{
    __shared__ float patch[kStemRows * kStemPitch];
    __shared__ __attribute__((aligned(16))) float dyl[kStemTH * kStemTW * 64];  // [pixel of the tile][filter]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, half = lane >> 5;
    for (int i = tid; i < kStemRows * kStemPitch; i += kConvThreads) patch[i] = 0.f;  // the floats no load writes must not hold NaNs
    // filter element 32*nb + col of this lane in block nb: its place in a patch relative to the pixel's (see stem_fwd_kernel's layout)
    int cj[5];
#pragma unroll
    for (int nb = 0; nb < 5; ++nb) {
        const int c = min(32 * nb + col, 146), fr = c / 21, j = c - fr * 21;
        cj[nb] = fr * kStemPitch + j + ((j / 3) >> 1);
    }
    floatx16 acc[2][5];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < 5; ++nb)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[mb][nb][e] = 0.f;
    __syncthreads();

    for (int tile = blockIdx.x; tile < p.ntiles; tile += gridDim.x) {
        const int n = tile / (p.tiles_h * p.tiles_w), rem = tile - n * (p.tiles_h * p.tiles_w);
        const int th = rem / p.tiles_w, tw = rem - th * p.tiles_w;
        const int oh0 = th * kStemTH, ow0 = tw * kStemTW;
        const int ih0 = 2 * oh0 - 3, if0 = (2 * ow0 - 3) * 3;
        float v[kStemLoads];
        float4 g[kStemDyLoads];
#pragma unroll
        for (int u = 0; u < kStemLoads; ++u) {
            const int i = tid + u * kConvThreads;
            const int pr = i / kStemCols, pc = i - pr * kStemCols;
            const int ih = ih0 + pr, f = if0 + pc;
            const bool ok = i < kStemRows * kStemCols && ih >= 0 && ih < p.IH && f >= 0 && f < p.IW * 3;
            v[u] = ok ? p.x[((long)n * p.IH + ih) * (p.IW * 3) + f] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < kStemDyLoads; ++u) {
            const int i = tid + u * kConvThreads;      // float4 index: pixel i / 16, filters 4 * (i % 16) ..
            const int q = i >> 4, oh = oh0 + (q >> 4), ow = ow0 + (q & 15);
            // a pixel outside the output contributes nothing: its dy is zero (the patch under it holds finite values)
            g[u] = (oh < p.OH && ow < p.OW) ? ldg4(p.dy + (((long)n * p.OH + oh) * p.OW + ow) * 64 + 4 * (i & 15)) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        __syncthreads();  // every wavefront is done with the previous tile
#pragma unroll
        for (int u = 0; u < kStemLoads; ++u) {
            const int i = tid + u * kConvThreads;
            const int pr = i / kStemCols, pc = i - pr * kStemCols;
            if (i < kStemRows * kStemCols) patch[pr * kStemPitch + pc + ((pc / 3) >> 1)] = v[u];
        }
#pragma unroll
        for (int u = 0; u < kStemDyLoads; ++u) *reinterpret_cast<float4 *>(&dyl[4 * (tid + u * kConvThreads)]) = g[u];
        __syncthreads();
        // pixel pairs 16*wave .. +15: lane half h multiplies pixel 2t + h
#pragma unroll 4
        for (int t = 0; t < 16; ++t) {
            const int q = 32 * wave + 2 * t + half;
            const int pb = 2 * (q >> 4) * kStemPitch + 7 * (q & 15);
            const float a0 = dyl[q * 64 + col], a1 = dyl[q * 64 + 32 + col];
            float b[5];
#pragma unroll
            for (int nb = 0; nb < 5; ++nb) b[nb] = patch[pb + cj[nb]];
#pragma unroll
            for (int nb = 0; nb < 5; ++nb) {
                acc[0][nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b[nb], acc[0][nb], 0, 0, 0);
                acc[1][nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b[nb], acc[1][nb], 0, 0, 0);
            }
        }
    }
    // the four wavefronts' sums, added in wavefront order through LDS, one half of the filters at a time (5 x 16 x 64 floats = 20 KB)
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
        for (int w = 1; w < 4; ++w) {
            __syncthreads();
            if (wave == w) {
#pragma unroll
                for (int nb = 0; nb < 5; ++nb)
#pragma unroll
                    for (int e = 0; e < 16; ++e) dyl[(nb * 16 + e) * 64 + lane] = acc[mb][nb][e];
            }
            __syncthreads();
            if (wave == 0) {
#pragma unroll
                for (int nb = 0; nb < 5; ++nb)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc[mb][nb][e] += dyl[(nb * 16 + e) * 64 + lane];
            }
        }
    if (wave == 0) {
        float *out = p.part + (long)blockIdx.x * (64 * 147);
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int nb = 0; nb < 5; ++nb) {
                const int c = 32 * nb + col;
                if (c < 147) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) out[(32 * mb + 8 * (e >> 2) + 4 * half + (e & 3)) * 147 + c] = acc[mb][nb][e];
                }
            }
    }
}

// ---------------------------------------------------------------------------------------------------
struct WgradP {
    const float *dy;  // [Mpix][Kout]
    const float *x;   // N x IH x IW x Cin
    float *out;       // partials: [split][Kout][R*S*Cin]
    // INAFF kernels: the layer's input is max(0, x*in_scale[c] + in_shift[c]), computed on the way into LDS
    const float *in_scale;
    const float *in_shift;
    int IH, IW, Cin, OH, OW, Kout, R, S, stride, pad;
    int Mpix;         // N*OH*OW
    int Jdim;         // R*S*Cin
    int tiles_k, tiles_j;  // tiles along Kout and along the flat filter index j = (r*S + s)*Cin + c
    int split, pix_per_split;
    long split_stride;
    FastDiv div_ohw, div_ow;  // by OH*OW and OW
    // Advance of one stage (kBK pixels) of the gathered input: kBK = (d_n*OH + d_oh)*OW + d_ow.
    int adv_iw, adv_ih;       // d_ow*stride, d_oh*stride
    int lim_iw, lim_ih;       // OW*stride, OH*stride
    unsigned adv_off;         // element offset of (d_n images, d_oh*stride rows, d_ow*stride columns)
    unsigned carry_row;       // one output row on, OW output columns back
    unsigned carry_img;       // one image on, OH output rows back
    unsigned adv_dy;          // kBK*Kout
};

// Fills everything of a filter gradient's launch parameters but the pointers: tiles of bm x bn, the pixels cut into `split`
// ranges of chunks_per_split stages.  P, Q: output height and width.
inline void wgrad_fill(WgradP &p, const rn50_conv_desc *d, int P, int Q, int bm, int bn, int split, int chunks_per_split)
{
    const int Jdim = d->r * d->s * d->c;
    p.IH = d->h; p.IW = d->w; p.Cin = d->c; p.OH = P; p.OW = Q; p.Kout = d->k; p.R = d->r; p.S = d->s;
    p.stride = d->stride; p.pad = d->pad; p.Mpix = d->n * P * Q; p.Jdim = Jdim;
    p.tiles_k = (d->k + bm - 1) / bm;
    p.tiles_j = (Jdim + bn - 1) / bn;
    p.split = split;
    p.pix_per_split = chunks_per_split * kBK;
    p.split_stride = (long)d->k * Jdim;
    p.div_ohw = make_fastdiv(P * Q);
    p.div_ow = make_fastdiv(Q);
    const int d_ow = kBK % Q, rows = kBK / Q, d_oh = rows % P, d_n = rows / P;
    const unsigned colsz = (unsigned)d->stride * d->c, rowsz = (unsigned)d->stride * d->w * d->c, imgsz = (unsigned)d->h * d->w * d->c;
    p.adv_iw = d_ow * d->stride;
    p.adv_ih = d_oh * d->stride;
    p.lim_iw = Q * d->stride;
    p.lim_ih = P * d->stride;
    p.adv_off = d_n * imgsz + d_oh * rowsz + d_ow * colsz;
    p.carry_row = rowsz - (unsigned)Q * colsz;   // modulo 2^32, like every offset sum in the kernel
    p.carry_img = imgsz - (unsigned)P * rowsz;
    p.adv_dy = (unsigned)kBK * d->k;
}

// Workgroups per CU the launch bounds allow for (register budget); small tiles do little MFMA work per stage and
// need more resident workgroups to cover the latency of their loads.
constexpr int wgrad_occupancy(int bm, int bn) { return (bm == 128 && bn == 128) ? 2 : (bm == 64 && bn == 64) ? 4 : 3; }

// A tile is BM output channels x BN consecutive flat filter indices (it may span several taps).
// VEC = true : Cin % 4 == 0, so four consecutive indices share a tap and are one 16-byte load.
// VEC = false: any Cin (the 3-channel stem): one float at a time.
// Loads run two stages ahead of the MFMAs (two register stages), because a stage of a small tile is too short
// to cover the latency of a load issued only one stage earlier.
// BF = true : both operands are rounded to bf16 (nearest even) on the way into LDS, which then holds
// [output index][pixel] rows of 16-bit elements, and the products run on the bf16 MFMA; sums stay fp32.
// INAFF (VEC only): per-channel scale, shift and ReLU applied to the gathered input (see WgradP::in_scale).
// One work item of a filter gradient: the BM x BN tile `item % ntiles` of dw over the pixel range `item / ntiles`, written as
// a partial to p.out.  As and Bs are the workgroup's LDS stages (kBK x (BM + 4) and kBK x (BN + 4) floats).
template <int BM, int BN, bool VEC, bool BF, bool INAFF>
__device__ __forceinline__ void wgrad_tile(const WgradP &p, const int item, float *__restrict__ As, float *__restrict__ Bs)
{
    static_assert(!INAFF || VEC, "the fused input transform exists for the vector gather only");
    constexpr int MI = BM / 64, NI = BN / 64;      // 32x32 blocks per wavefront along each side
    constexpr int LDA = BM + 4, LDB = BN + 4;
    constexpr int CA = BM / 4, CB = BN / 4;        // float4 columns per pixel row
    constexpr int PA = kConvThreads / CA, PB = kConvThreads / CB;  // pixel rows per pass
    constexpr int RA = kBK / PA, RB = kBK / PB;
    constexpr int LDW = kBK / 2 + 2;               // bf16 rows: 32 pixels as 16 words, padded to 72 bytes
    static_assert(RA % 2 == 0 && RB % 2 == 0, "bf16 staging pairs neighbouring pixels");

    // the pointers as global-memory pointers: read from a job table they would otherwise be generic, and every load a flat one
    const gcfp g_dy = (gcfp)p.dy, g_x = (gcfp)p.x, g_sc = (gcfp)p.in_scale, g_sh = (gcfp)p.in_shift;
    const int ntiles = p.tiles_k * p.tiles_j;
    const int split = item / ntiles;
    const int tile = item - split * ntiles;
    const int tk = tile / p.tiles_j, tj = tile - tk * p.tiles_j;
    const int k0 = tk * BM, j0 = tj * BN;
    const int pix_begin = split * p.pix_per_split;
    const int pix_end = min(p.Mpix, pix_begin + p.pix_per_split);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int ca = tid % CA, pa = tid / CA;
    const int cb = tid % CB, pb = tid / CB;

    // filter tap and channel of this thread's columns, decoded once
    int gr[4], gs[4], gc[4];
    bool gok[4];
#pragma unroll
    for (int e = 0; e < (VEC ? 1 : 4); ++e) {
        const int j = j0 + cb * 4 + e;
        gok[e] = j < p.Jdim;
        gr[e] = j / (p.S * p.Cin);
        const int rem = j - gr[e] * (p.S * p.Cin);
        gs[e] = rem / p.Cin;
        gc[e] = rem - gs[e] * p.Cin;
    }
    const bool a_ok = k0 + ca * 4 < p.Kout;
    // INAFF: this thread's four input channels are the same for every pixel
    float4 in_sc = make_float4(0.f, 0.f, 0.f, 0.f), in_sh = in_sc;
    if (INAFF && gok[0]) {
        in_sc = ldg4(g_sc + gc[0]);
        in_sh = ldg4(g_sh + gc[0]);
    }

    // Running state of this thread's loads.  Consecutive stages are kBK pixels apart, so the pixel -> (image, row, column)
    // decode is done once, here, and then advanced with additions and two carries per stage (the advance of kBK pixels
    // in rows and columns and the matching offset steps are launch constants): the multiply-high divisions and the 64-bit
    // multiplies of a fresh decode would otherwise sit in the inner loop of a kernel that has only 16-64 MFMAs per stage.
    // Offsets are 32-bit element counts (every tensor has fewer than 2^31 elements).
    int apix[RA], bpix[RB], bih[RB], biw[RB];
    unsigned aoff[RA], boff[RB];
#pragma unroll
    for (int i = 0; i < RA; ++i) {
        apix[i] = pix_begin + (BF ? 2 * pa + (i & 1) + 2 * PA * (i >> 1) : pa + PA * i);
        aoff[i] = (unsigned)apix[i] * (unsigned)p.Kout + (unsigned)(k0 + ca * 4);
    }
#pragma unroll
    for (int i = 0; i < RB; ++i) {
        const int pix = pix_begin + (BF ? 2 * pb + (i & 1) + 2 * PB * (i >> 1) : pb + PB * i);
        const int n = (int)fdiv(pix, p.div_ohw);
        const int rem = pix - n * (p.OH * p.OW);
        const int oh = (int)fdiv(rem, p.div_ow), ow = rem - oh * p.OW;
        bpix[i] = pix;
        bih[i] = oh * p.stride;   // input row and column of filter tap (pad, pad)
        biw[i] = ow * p.stride;
        boff[i] = ((unsigned)(n * p.IH + bih[i]) * (unsigned)p.IW + (unsigned)biw[i]) * (unsigned)p.Cin;
    }
    // this thread's filter tap(s) relative to that position
    int th[4], tw[4], toff[4];
#pragma unroll
    for (int e = 0; e < (VEC ? 1 : 4); ++e) {
        th[e] = gr[e] - p.pad;
        tw[e] = gs[e] - p.pad;
        toff[e] = (th[e] * p.IW + tw[e]) * p.Cin + gc[e];
    }

    // loads the stage the running state points at, then advances the state by kBK pixels
    auto load_chunk = [&](float4 (&ra)[RA], float4 (&rb)[RB], unsigned &okb) {
        okb = 0;
#pragma unroll
        for (int i = 0; i < RA; ++i) {
            ra[i] = (a_ok && apix[i] < pix_end) ? ldg4(g_dy + aoff[i]) : make_float4(0.f, 0.f, 0.f, 0.f);
            apix[i] += kBK;
            aoff[i] += p.adv_dy;
        }
#pragma unroll
        for (int i = 0; i < RB; ++i) {
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (VEC) {
                // one condition, one branch: nested tests make the compiler clear the destination once per level
                const int ih = bih[i] + th[0], iw = biw[i] + tw[0];
                const bool ok = (bpix[i] < pix_end) & gok[0] & ((unsigned)ih < (unsigned)p.IH) & ((unsigned)iw < (unsigned)p.IW);
                if (ok) {
                    v = ldg4(g_x + (boff[i] + (unsigned)toff[0]));
                    if (INAFF) okb |= 1u << i;
                }
            } else if (bpix[i] < pix_end) {
                {
                    float t[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int ih = bih[i] + th[e], iw = biw[i] + tw[e];
                        const bool ok = gok[e] && (unsigned)ih < (unsigned)p.IH && (unsigned)iw < (unsigned)p.IW;
                        t[e] = ok ? g_x[boff[i] + (unsigned)toff[e]] : 0.f;
                    }
                    v = make_float4(t[0], t[1], t[2], t[3]);
                }
            }
            rb[i] = v;
            // kBK pixels on: columns first, a carry into the rows, rows, a carry into the images
            bpix[i] += kBK;
            biw[i] += p.adv_iw;
            boff[i] += p.adv_off;
            if (biw[i] >= p.lim_iw) {
                biw[i] -= p.lim_iw;
                bih[i] += p.stride;
                boff[i] += p.carry_row;
            }
            bih[i] += p.adv_ih;
            if (bih[i] >= p.lim_ih) {
                bih[i] -= p.lim_ih;
                boff[i] += p.carry_img;
            }
        }
    };
    uint32_t *Aw = reinterpret_cast<uint32_t *>(As), *Bw = reinterpret_cast<uint32_t *>(Bs);
    auto store_chunk = [&](const float4 (&ra)[RA], float4 (&rb)[RB], unsigned okb) {
        if (INAFF) {
#pragma unroll
            for (int i = 0; i < RB; ++i)
                if (okb & (1u << i)) {  // padding stays zero
                    rb[i].x = fmaxf(fmaf(rb[i].x, in_sc.x, in_sh.x), 0.f);
                    rb[i].y = fmaxf(fmaf(rb[i].y, in_sc.y, in_sh.y), 0.f);
                    rb[i].z = fmaxf(fmaf(rb[i].z, in_sc.z, in_sh.z), 0.f);
                    rb[i].w = fmaxf(fmaf(rb[i].w, in_sc.w, in_sh.w), 0.f);
                }
        }
        if (BF) {
            // registers 2i and 2i+1 hold neighbouring pixels: one word per output index
#pragma unroll
            for (int i = 0; i < RA / 2; ++i) {
                uint32_t *d = Aw + (ca * 4) * LDW + pa + PA * i;
                d[0] = bf16_pack2(ra[2 * i].x, ra[2 * i + 1].x);
                d[LDW] = bf16_pack2(ra[2 * i].y, ra[2 * i + 1].y);
                d[2 * LDW] = bf16_pack2(ra[2 * i].z, ra[2 * i + 1].z);
                d[3 * LDW] = bf16_pack2(ra[2 * i].w, ra[2 * i + 1].w);
            }
#pragma unroll
            for (int i = 0; i < RB / 2; ++i) {
                uint32_t *d = Bw + (cb * 4) * LDW + pb + PB * i;
                d[0] = bf16_pack2(rb[2 * i].x, rb[2 * i + 1].x);
                d[LDW] = bf16_pack2(rb[2 * i].y, rb[2 * i + 1].y);
                d[2 * LDW] = bf16_pack2(rb[2 * i].z, rb[2 * i + 1].z);
                d[3 * LDW] = bf16_pack2(rb[2 * i].w, rb[2 * i + 1].w);
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < RA; ++i) *reinterpret_cast<float4 *>(&As[(pa + PA * i) * LDA + ca * 4]) = ra[i];
#pragma unroll
        for (int i = 0; i < RB; ++i) *reinterpret_cast<float4 *>(&Bs[(pb + PB * i) * LDB + cb * 4]) = rb[i];
    };

    floatx16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // Lane l supplies output index MI*(l%32)+i for block i (interleaved, so that one 8-byte LDS read feeds
    // both blocks) and reduction element l/32 of the current pixel pair.
    const int fa = (lane >> 5) * LDA + wm * (BM / 2) + (lane & 31) * MI;
    const int fb = (lane >> 5) * LDB + wn * (BN / 2) + (lane & 31) * NI;
    // bf16: lane l supplies output index 32*i + l%32 of block i and the eight pixels 8*(l/32) .. +7 of each
    // half of the chunk (two 8-byte reads; rows are 72 bytes apart)
    const int ha = (wm * (BM / 2) + (lane & 31)) * LDW + (lane >> 5) * 4;
    const int hb = (wn * (BN / 2) + (lane & 31)) * LDW + (lane >> 5) * 4;
    auto compute = [&]() {
        if (BF) {
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                union { uint2 u[2]; bf16x8 v; } a8[MI], b8[NI];
#pragma unroll
                for (int i = 0; i < MI; ++i) {
                    a8[i].u[0] = *reinterpret_cast<const uint2 *>(&Aw[ha + i * 32 * LDW + ks * 8]);
                    a8[i].u[1] = *reinterpret_cast<const uint2 *>(&Aw[ha + i * 32 * LDW + ks * 8 + 2]);
                }
#pragma unroll
                for (int j = 0; j < NI; ++j) {
                    b8[j].u[0] = *reinterpret_cast<const uint2 *>(&Bw[hb + j * 32 * LDW + ks * 8]);
                    b8[j].u[1] = *reinterpret_cast<const uint2 *>(&Bw[hb + j * 32 * LDW + ks * 8 + 2]);
                }
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int j = 0; j < NI; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a8[i].v, b8[j].v, acc[i][j], 0, 0, 0);
            }
            return;
        }
        if constexpr (MI * NI > 1) {
            // the larger tiles have no registers to spare for a second fragment set (it spills); a pixel pair feeds 2-4 MFMAs here
#pragma unroll
            for (int kp = 0; kp < kBK / 2; ++kp) {
                float af[MI], bf[NI];
                if (MI == 2) {
                    const float2 t = *reinterpret_cast<const float2 *>(&As[kp * 2 * LDA + fa]);
                    af[0] = t.x;
                    af[MI - 1] = t.y;
                } else {
                    af[0] = As[kp * 2 * LDA + fa];
                }
                if (NI == 2) {
                    const float2 t = *reinterpret_cast<const float2 *>(&Bs[kp * 2 * LDB + fb]);
                    bf[0] = t.x;
                    bf[NI - 1] = t.y;
                } else {
                    bf[0] = Bs[kp * 2 * LDB + fb];
                }
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int j = 0; j < NI; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i], bf[j], acc[i][j], 0, 0, 0);
            }
            return;
        }
        // 64x64 tiles (one MFMA per pixel pair and wavefront).  Pixel pairs in groups of kFragGroup: the fragments of group g+1 are read from LDS while the MFMAs of group g run
        // (two register sets; the scheduling hints keep the order read, multiply, group by group).  Read and used pair by
        // pair, every one or two MFMAs would wait for the latency of an LDS read.
        constexpr int kFragGroup = INAFF ? 2 : 4, kGroups = kBK / 2 / kFragGroup;
        float af[2][kFragGroup][MI], bf[2][kFragGroup][NI];
        auto load_group = [&](int set, int g) {
#pragma unroll
            for (int t = 0; t < kFragGroup; ++t) {
                const int kp = g * kFragGroup + t;
                if (MI == 2) {
                    const float2 v = *reinterpret_cast<const float2 *>(&As[kp * 2 * LDA + fa]);
                    af[set][t][0] = v.x;
                    af[set][t][MI - 1] = v.y;
                } else {
                    af[set][t][0] = As[kp * 2 * LDA + fa];
                }
                if (NI == 2) {
                    const float2 v = *reinterpret_cast<const float2 *>(&Bs[kp * 2 * LDB + fb]);
                    bf[set][t][0] = v.x;
                    bf[set][t][NI - 1] = v.y;
                } else {
                    bf[set][t][0] = Bs[kp * 2 * LDB + fb];
                }
            }
        };
        load_group(0, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2 * kFragGroup, 0);
#pragma unroll
        for (int g = 0; g < kGroups; ++g) {
            if (g + 1 < kGroups) {
                load_group((g + 1) & 1, g + 1);
                __builtin_amdgcn_sched_group_barrier(0x100, 2 * kFragGroup, 0);
            }
#pragma unroll
            for (int t = 0; t < kFragGroup; ++t)
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int j = 0; j < NI; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[g & 1][t][i], bf[g & 1][t][j], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, kFragGroup * MI * NI, 0);
        }
    };

    // LDS holds stage c; r0 holds stage c+1, r1 holds stage c+2 (loads past the end of the range return zeros
    // without touching memory)
    float4 ra0[RA], rb0[RB], ra1[RA], rb1[RB];
    unsigned ok0 = 0, ok1 = 0;
    load_chunk(ra0, rb0, ok0);
    store_chunk(ra0, rb0, ok0);
    load_chunk(ra0, rb0, ok0);
    load_chunk(ra1, rb1, ok1);
    __syncthreads();
    // Two stages per trip and no way out of the loop but its end: with exits between the stages the compiler keeps the
    // accumulators in different registers at different points of the loop and copies them, behind a drained MFMA pipe, on
    // every trip.  A range with an odd number of stages multiplies one stage of zeros at its end (loads past the end of the
    // range return zeros), which is why the launch plans cut ranges of an even number of stages.
    const int pairs = (pix_end - pix_begin + 2 * kBK - 1) / (2 * kBK);
    for (int it = 0; it < pairs; ++it) {
        __builtin_amdgcn_s_setprio(1);  // a wavefront that multiplies goes before one that computes addresses (both below the main chain's)
        compute();
        __syncthreads();
        __builtin_amdgcn_s_setprio(0);
        store_chunk(ra0, rb0, ok0);
        load_chunk(ra0, rb0, ok0);
        __syncthreads();
        __builtin_amdgcn_s_setprio(1);
        compute();
        __syncthreads();
        __builtin_amdgcn_s_setprio(0);
        store_chunk(ra1, rb1, ok1);
        load_chunk(ra1, rb1, ok1);
        __syncthreads();
    }

    gfp out = (gfp)p.out + (long)split * p.split_stride;
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int brow = 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
            const int k = k0 + wm * (BM / 2) + (BF ? i * 32 + brow : brow * MI + i);
            if (k >= p.Kout) continue;
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                const int col = j0 + wn * (BN / 2) + (BF ? j * 32 + (lane & 31) : (lane & 31) * NI + j);
                if (col < p.Jdim) out[(long)k * p.Jdim + col] = acc[i][j][e];
            }
        }
}

template <int BM, int BN, bool VEC, bool BF, bool INAFF = false>
__global__ __launch_bounds__(kConvThreads, wgrad_occupancy(BM, BN)) void wgrad_kernel(WgradP p)
{
    __shared__ __attribute__((aligned(16))) float As[kBK * (BM + 4)];
    __shared__ __attribute__((aligned(16))) float Bs[kBK * (BN + 4)];
    // Work item = (pixel range, tile), the tiles of one pixel range adjacent: they read the same rows of dy and x.  Consecutive
    // workgroups are dispatched to different XCDs, so each XCD takes a contiguous run of items and the tiles of a range meet in
    // one L2 instead of being fetched into eight.
    wgrad_tile<BM, BN, VEC, BF, INAFF>(p, xcd_contiguous(blockIdx.x, gridDim.x), As, Bs);
}

// The filter gradients of several layers in ONE launch.  Job j owns the work items [item_begin, next job's item_begin) of
// the launch (its pixel ranges x tiles, as in wgrad_kernel); a job with in_scale set applies the fused input transform.
// fp32 operands through the vector gather (Cin % 4 == 0).  A layer-sized launch starts all its workgroups together, so they load,
// multiply and store in lock step and every layer pays a ramp and a tail; here a finished workgroup is replaced by the next
// item (of the same or the next layer) while its neighbours on the CU are in the middle of theirs.
struct WgradJob {
    WgradP p;
    int item_begin;
    int pad_;
};
template <int BM, int BN>
__global__ __launch_bounds__(kConvThreads, wgrad_occupancy(BM, BN)) void wgrad_group_kernel(const WgradJob *__restrict__ jobs, int njobs)
{
    __shared__ __attribute__((aligned(16))) float As[kBK * (BM + 4)];
    __shared__ __attribute__((aligned(16))) float Bs[kBK * (BN + 4)];
    const int item = xcd_contiguous(blockIdx.x, gridDim.x);
    int lo = 0, hi = njobs - 1;  // the last job whose item_begin <= item
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (jobs[mid].item_begin <= item) lo = mid;
        else hi = mid - 1;
    }
    const int j = __builtin_amdgcn_readfirstlane(lo);
    const WgradP p = jobs[j].p;
    const int local = item - jobs[j].item_begin;
    if (p.in_scale) wgrad_tile<BM, BN, true, false, true>(p, local, As, Bs);
    else wgrad_tile<BM, BN, true, false, false>(p, local, As, Bs);
}

// The ordered sums of the partials of several filter gradients in one launch: job j owns workgroups [block_begin, next
// job's block_begin), each 64 float4 columns of its gradient (same order of additions as splitk_reduce_kernel).
struct ReduceJob {
    long count4, stride;  // float4 elements of the gradient; floats between two partials
    const float *part;
    long out_off;         // element offset of the gradient from the launch's dw_base
    int split, block_begin;
};
static __global__ __launch_bounds__(256) void splitk_reduce_group_kernel(const ReduceJob *__restrict__ jobs, int njobs, float *__restrict__ dw_base)
{
    __shared__ float4 red[4][64];
    int lo = 0, hi = njobs - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (jobs[mid].block_begin <= (int)blockIdx.x) lo = mid;
        else hi = mid - 1;
    }
    const ReduceJob job = jobs[__builtin_amdgcn_readfirstlane(lo)];
    const int c = threadIdx.x & 63, q = threadIdx.x >> 6;
    const long i = (long)((int)blockIdx.x - job.block_begin) * 64 + c;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i < job.count4) {
#pragma unroll 4
        for (int s = q; s < job.split; s += 4) {
            const float4 v = reinterpret_cast<const float4 *>(job.part + (long)s * job.stride)[i];
            acc.x += v.x;
            acc.y += v.y;
            acc.z += v.z;
            acc.w += v.w;
        }
    }
    red[q][c] = acc;
    __syncthreads();
    if (q == 0 && i < job.count4) {
        float4 r = red[0][c];
#pragma unroll
        for (int t = 1; t < 4; ++t) {
            r.x += red[t][c].x;
            r.y += red[t][c].y;
            r.z += red[t][c].z;
            r.w += red[t][c].w;
        }
        reinterpret_cast<float4 *>(dw_base + job.out_off)[i] = r;
    }
}

// ---------------------------------------------------------------------------------------------------
// Filter gradient with the activation tensors kept as bfloat16 in memory: dy holds bf16 bits; x holds bf16 bits (XF32 = false)
// or fp32 (XF32 = true: the network's first layer, whose input is the image; any channel count, scalar gather).  Tiles of
// 64 output channels x 64 flat filter indices, products on the bf16 MFMA, sums and the output partials in fp32, same split
// of the pixel range and same ordered reduction as wgrad_kernel.
// Half of the workgroup loads dy, the other half x: a thread owns eight neighbouring output indices (one 16-byte load of
// bf16) of two neighbouring pixels and writes eight LDS words, each the pair (pixel 2q, pixel 2q+1) of one index, which is
// the [index][pixel] order the MFMA operands are read in.  Loads run two stages ahead, as in wgrad_kernel.
// INAFF (XF32 = false only): x is max(0, x*in_scale[c] + in_shift[c]) rounded to bf16, i.e. the BN + ReLU output as stored.
template <bool XF32, bool INAFF>
__global__ __launch_bounds__(kConvThreads, 4) void wgrad_act_kernel(WgradP p)
{
    static_assert(!(XF32 && INAFF), "the fused input transform exists for bf16 inputs only");
    constexpr int BM = 64, BN = 64;
    constexpr int LDW = kBK / 2 + 2;  // rows of 16 words (32 pixels), padded to 72 bytes
    __shared__ __attribute__((aligned(16))) uint32_t Aw[BM * LDW];
    __shared__ __attribute__((aligned(16))) uint32_t Bw[BN * LDW];

    const int ntiles = p.tiles_k * p.tiles_j;
    const int item = xcd_contiguous(blockIdx.x, gridDim.x);
    const int split = item / ntiles;
    const int tile = item - split * ntiles;
    const int tk = tile / p.tiles_j, tj = tile - tk * p.tiles_j;
    const int k0 = tk * BM, j0 = tj * BN;
    const int pix_begin = split * p.pix_per_split;
    const int pix_end = min(p.Mpix, pix_begin + p.pix_per_split);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const bool is_dy = tid < 128;          // uniform per wavefront
    const int t = tid & 127, c8 = t & 7, pp = t >> 3;   // eight indices c8*8.., pixel pair pp of the stage
    const bf16_t *dy16 = reinterpret_cast<const bf16_t *>(p.dy);
    const bf16_t *x16 = reinterpret_cast<const bf16_t *>(p.x);

    // x side: filter tap and channel of this thread's indices, decoded once (bf16 input: the eight share a tap, Cin % 8 == 0)
    constexpr int NE = XF32 ? 8 : 1;
    int th[NE], tw[NE], toff[NE];
    bool gok[NE];
#pragma unroll
    for (int e = 0; e < NE; ++e) {
        const int j = j0 + c8 * 8 + e;
        gok[e] = j < p.Jdim;
        const int r = j / (p.S * p.Cin);
        const int rem = j - r * (p.S * p.Cin);
        const int sx = rem / p.Cin, c = rem - sx * p.Cin;
        th[e] = r - p.pad;
        tw[e] = sx - p.pad;
        toff[e] = (th[e] * p.IW + tw[e]) * p.Cin + c;
    }
    float4 in_sc = make_float4(0.f, 0.f, 0.f, 0.f), in_sh = in_sc, in_sc2 = in_sc, in_sh2 = in_sc;
    if (INAFF && !is_dy && gok[0]) {
        const int j = j0 + c8 * 8;
        const int c = j % p.Cin;
        in_sc = ldg4(p.in_scale + c);
        in_sh = ldg4(p.in_shift + c);
        in_sc2 = ldg4(p.in_scale + c + 4);
        in_sh2 = ldg4(p.in_shift + c + 4);
    }
    const bool a_ok = k0 + c8 * 8 < p.Kout;

    // running state of the two pixels of this thread (see wgrad_kernel: decoded once, then advanced by kBK pixels per stage)
    int pix[2], bih[2], biw[2];
    unsigned off[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        pix[u] = pix_begin + 2 * pp + u;
        if (is_dy) {
            off[u] = (unsigned)pix[u] * (unsigned)p.Kout + (unsigned)(k0 + c8 * 8);
            bih[u] = biw[u] = 0;
        } else {
            const int n = (int)fdiv(pix[u], p.div_ohw);
            const int rem = pix[u] - n * (p.OH * p.OW);
            const int oh = (int)fdiv(rem, p.div_ow), ow = rem - oh * p.OW;
            bih[u] = oh * p.stride;
            biw[u] = ow * p.stride;
            off[u] = ((unsigned)(n * p.IH + bih[u]) * (unsigned)p.IW + (unsigned)biw[u]) * (unsigned)p.Cin;
        }
    }

    struct Stage {
        uint4 q[2];          // bf16 loads
        float xf[2][NE];     // fp32 input: one float per index
        unsigned ok;         // INAFF: bit u set when q[u] was loaded (not padding)
    };
    auto load_chunk = [&](Stage &sg) {
        sg.ok = 0;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            sg.q[u] = make_uint4(0u, 0u, 0u, 0u);
            if (is_dy) {
                if (a_ok && pix[u] < pix_end) sg.q[u] = *reinterpret_cast<const uint4 *>(dy16 + off[u]);
                off[u] += p.adv_dy;
            } else {
                if (XF32) {
#pragma unroll
                    for (int e = 0; e < NE; ++e) {
                        const int ih = bih[u] + th[e], iw = biw[u] + tw[e];
                        const bool ok = pix[u] < pix_end && gok[e] && (unsigned)ih < (unsigned)p.IH && (unsigned)iw < (unsigned)p.IW;
                        sg.xf[u][e] = ok ? p.x[off[u] + (unsigned)toff[e]] : 0.f;
                    }
                } else {
                    const int ih = bih[u] + th[0], iw = biw[u] + tw[0];
                    if (pix[u] < pix_end && gok[0] && (unsigned)ih < (unsigned)p.IH && (unsigned)iw < (unsigned)p.IW) {
                        sg.q[u] = *reinterpret_cast<const uint4 *>(x16 + (off[u] + (unsigned)toff[0]));
                        sg.ok |= 1u << u;
                    }
                }
                // kBK pixels on: columns first, a carry into the rows, rows, a carry into the images
                biw[u] += p.adv_iw;
                off[u] += p.adv_off;
                if (biw[u] >= p.lim_iw) {
                    biw[u] -= p.lim_iw;
                    bih[u] += p.stride;
                    off[u] += p.carry_row;
                }
                bih[u] += p.adv_ih;
                if (bih[u] >= p.lim_ih) {
                    bih[u] -= p.lim_ih;
                    off[u] += p.carry_img;
                }
            }
            pix[u] += kBK;
        }
    };
    auto store_chunk = [&](Stage &sg) {
        uint32_t *dst = (is_dy ? Aw : Bw) + (c8 * 8) * LDW + pp;
        if (XF32 && !is_dy) {
#pragma unroll
            for (int e = 0; e < NE; ++e) dst[e * LDW] = bf16_pack2(sg.xf[0][e], sg.xf[1][e]);
            return;
        }
        if (INAFF && !is_dy) {
#pragma unroll
            for (int u = 0; u < 2; ++u)
                if (sg.ok & (1u << u)) {  // padding stays zero
                    uint4 v = sg.q[u];
                    v.x = bf16_pack2(fmaxf(fmaf(bf16_lo(v.x), in_sc.x, in_sh.x), 0.f), fmaxf(fmaf(bf16_hi(v.x), in_sc.y, in_sh.y), 0.f));
                    v.y = bf16_pack2(fmaxf(fmaf(bf16_lo(v.y), in_sc.z, in_sh.z), 0.f), fmaxf(fmaf(bf16_hi(v.y), in_sc.w, in_sh.w), 0.f));
                    v.z = bf16_pack2(fmaxf(fmaf(bf16_lo(v.z), in_sc2.x, in_sh2.x), 0.f), fmaxf(fmaf(bf16_hi(v.z), in_sc2.y, in_sh2.y), 0.f));
                    v.w = bf16_pack2(fmaxf(fmaf(bf16_lo(v.w), in_sc2.z, in_sh2.z), 0.f), fmaxf(fmaf(bf16_hi(v.w), in_sc2.w, in_sh2.w), 0.f));
                    sg.q[u] = v;
                }
        }
        // word e = (index e of the first pixel, index e of the second): low and high halves of the two loads' words
        const uint32_t a[4] = {sg.q[0].x, sg.q[0].y, sg.q[0].z, sg.q[0].w}, b[4] = {sg.q[1].x, sg.q[1].y, sg.q[1].z, sg.q[1].w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            dst[(2 * c) * LDW] = (a[c] & 0xffffu) | (b[c] << 16);
            dst[(2 * c + 1) * LDW] = (a[c] >> 16) | (b[c] & 0xffff0000u);
        }
    };

    floatx16 acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
    // lane l supplies output index l%32 of its block and the eight pixels 8*(l/32) .. +7 of each half of the stage
    const int ha = (wm * (BM / 2) + (lane & 31)) * LDW + (lane >> 5) * 4;
    const int hb = (wn * (BN / 2) + (lane & 31)) * LDW + (lane >> 5) * 4;
    auto compute = [&]() {
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            union { uint2 u[2]; bf16x8 v; } a8, b8;
            a8.u[0] = *reinterpret_cast<const uint2 *>(&Aw[ha + ks * 8]);
            a8.u[1] = *reinterpret_cast<const uint2 *>(&Aw[ha + ks * 8 + 2]);
            b8.u[0] = *reinterpret_cast<const uint2 *>(&Bw[hb + ks * 8]);
            b8.u[1] = *reinterpret_cast<const uint2 *>(&Bw[hb + ks * 8 + 2]);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a8.v, b8.v, acc, 0, 0, 0);
        }
    };

    // LDS holds stage c; s0 holds stage c+1, s1 holds stage c+2 (loads past the end of the range return zeros without
    // touching memory)
    Stage s0, s1;
    load_chunk(s0);
    store_chunk(s0);
    load_chunk(s0);
    load_chunk(s1);
    __syncthreads();
    // two stages per trip and no exit between them (see wgrad_tile): an odd range ends with a stage of zeros
    const int pairs = (pix_end - pix_begin + 2 * kBK - 1) / (2 * kBK);
    for (int it = 0; it < pairs; ++it) {
        __builtin_amdgcn_s_setprio(1);  // as in wgrad_tile: multiplying goes before address arithmetic, both below the main chain
        compute();
        __syncthreads();
        __builtin_amdgcn_s_setprio(0);
        store_chunk(s0);
        load_chunk(s0);
        __syncthreads();
        __builtin_amdgcn_s_setprio(1);
        compute();
        __syncthreads();
        __builtin_amdgcn_s_setprio(0);
        store_chunk(s1);
        load_chunk(s1);
        __syncthreads();
    }

    float *out = p.out + (long)split * p.split_stride;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const int k = k0 + wm * (BM / 2) + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
        const int col = j0 + wn * (BN / 2) + (lane & 31);
        if (k < p.Kout && col < p.Jdim) out[(long)k * p.Jdim + col] = acc[e];
    }
}

// out[i] = sum_s part[s][i].  Workgroup = 64 float4 columns x 4 lanes over the splits; lane q adds splits q, q+4, ...
// in increasing order (several loads in flight), then the four lane sums are added in lane order through LDS.
// The order is fixed by (split count, position), so the result is bit-identical from call to call.
static __global__ __launch_bounds__(256) void splitk_reduce_kernel(long count4, int split, long stride, const float *__restrict__ part,
                                                            float *__restrict__ out)
{
    __shared__ float4 red[4][64];
    const int c = threadIdx.x & 63, q = threadIdx.x >> 6;
    const long i = (long)blockIdx.x * 64 + c;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i < count4) {
#pragma unroll 4
        for (int s = q; s < split; s += 4) {
            const float4 v = reinterpret_cast<const float4 *>(part + (long)s * stride)[i];
            acc.x += v.x;
            acc.y += v.y;
            acc.z += v.z;
            acc.w += v.w;
        }
    }
    red[q][c] = acc;
    __syncthreads();
    if (q == 0 && i < count4) {
        float4 r = red[0][c];
#pragma unroll
        for (int t = 1; t < 4; ++t) {
            r.x += red[t][c].x;
            r.y += red[t][c].y;
            r.z += red[t][c].z;
            r.w += red[t][c].w;
        }
        reinterpret_cast<float4 *>(out)[i] = r;
    }
}

// Filter of the data gradient: wt[c][R-1-r][S-1-s][k] = w[k][r][s][c].  One workgroup transposes a 64 (k) x 64 (c) tile
// of one filter tap through LDS; when K and C are multiples of 4 both sides move 16 bytes per lane (rows of 256 bytes).
constexpr int kFlipTile = 64;
__device__ inline void flip_tile(int K, int C, int RS, int tap, int k0, int c0, const float *__restrict__ w, float *__restrict__ wt,
                                 float (*t)[kFlipTile + 1])
{
    const int tid = threadIdx.x;
    const int tap_t = RS - 1 - tap;  // flipping r and s together reverses the flat tap index
    if (((K | C) & 3) == 0) {
        const int q = tid & 15, row = tid >> 4;  // 16 float4 columns x 16 rows per pass
#pragma unroll
        for (int i = 0; i < kFlipTile / 16; ++i) {
            const int kl = row + 16 * i, k = k0 + kl, c = c0 + q * 4;
            const float4 v = (k < K && c < C) ? ldg4(w + ((long)k * RS + tap) * C + c) : make_float4(0.f, 0.f, 0.f, 0.f);
            t[kl][q * 4 + 0] = v.x;
            t[kl][q * 4 + 1] = v.y;
            t[kl][q * 4 + 2] = v.z;
            t[kl][q * 4 + 3] = v.w;
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < kFlipTile / 16; ++i) {
            const int cl = row + 16 * i, c = c0 + cl, k = k0 + q * 4;
            if (c < C && k < K)
                *reinterpret_cast<float4 *>(wt + ((long)c * RS + tap_t) * K + k) =
                    make_float4(t[q * 4 + 0][cl], t[q * 4 + 1][cl], t[q * 4 + 2][cl], t[q * 4 + 3][cl]);
        }
    } else {
        const int tx = tid & 63, ty = tid >> 6;  // 64 x 4
        for (int i = ty; i < kFlipTile; i += 4) {
            const int k = k0 + i, c = c0 + tx;
            t[i][tx] = (k < K && c < C) ? w[((long)k * RS + tap) * C + c] : 0.f;
        }
        __syncthreads();
        for (int i = ty; i < kFlipTile; i += 4) {
            const int c = c0 + i, k = k0 + tx;
            if (k < K && c < C) wt[((long)c * RS + tap_t) * K + k] = t[tx][i];
        }
    }
}

static __global__ __launch_bounds__(256) void filter_flip_transpose_kernel(int K, int C, int RS, const float *__restrict__ w,
                                                                    float *__restrict__ wt)
{
    __shared__ float t[kFlipTile][kFlipTile + 1];
    flip_tile(K, C, RS, blockIdx.z, blockIdx.y * kFlipTile, blockIdx.x * kFlipTile, w, wt, t);
}

// The same for many filters in one launch (all layers of a network at the start of its backward pass): job j owns
// workgroups [block_begin, next job's block_begin); src/dst are offsets into one parameter arena and one arena of
// flipped filters.
struct FlipJob {
    int K, C, RS, tiles_c, tiles_k, block_begin;
    long src_off, dst_off;
};
static __global__ __launch_bounds__(256) void filter_flip_batched_kernel(const FlipJob *__restrict__ jobs, int njobs,
                                                                  const float *__restrict__ theta, float *__restrict__ wt)
{
    __shared__ float t[kFlipTile][kFlipTile + 1];
    int j = 0;
    while (j + 1 < njobs && (int)blockIdx.x >= jobs[j + 1].block_begin) ++j;
    const FlipJob job = jobs[j];
    int local = blockIdx.x - job.block_begin;
    const int tap = local / (job.tiles_c * job.tiles_k);
    local -= tap * (job.tiles_c * job.tiles_k);
    flip_tile(job.K, job.C, job.RS, tap, (local / job.tiles_c) * kFlipTile, (local % job.tiles_c) * kFlipTile, theta + job.src_off,
              wt + job.dst_off, t);
}

}  // namespace rn50
