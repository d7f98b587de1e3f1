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

constexpr int kConvThreads = 256;
constexpr int kBK = 32;        // reduction elements per LDS stage
constexpr int kLDK = kBK + 4;  // padded row length: 16-byte aligned rows, conflict-free 128-bit fragment reads

// Geometry of the gathered operand.  Output row m = (n, oh, ow); for filter tap (r, s) the input
// coordinate is ih = (oh*so + r + off)/sd and exists only when the numerator is a non-negative
// multiple of sd and ih < IH (same for iw).  Forward: so = stride, off = -pad, sd = 1.  Data gradient:
// so = 1, off = pad-(R-1), sd = stride, with the filter flipped.
struct IgemmP {
    const float *a;
    const float *b;
    float *out;
    int IH, IW, Cin;
    int OH, OW;
    int Nout;
    int R, S;
    int so, off, sd;
    int M;      // N*OH*OW
    int Kdim;   // R*S*Cin
    int kchunks;
    int split_k, chunks_per_split;
    int tiles_m, tiles_n, tiles_per_xcd;
    int scatter2;          // rows go to pixel (n, 2*oh, 2*ow) of an N x 2OH x 2OW x Nout tensor, siblings are zeroed
    long out_split_stride; // elements between the partial outputs of consecutive splits
};

// Workgroup id -> logical tile: consecutive ids land on different XCDs (round-robin dispatch), so give
// each XCD a contiguous range of logical tiles; tiles that share activations then share an L2.
__device__ inline int xcd_remap(int wg, int tiles_per_xcd) { return (wg & 7) * tiles_per_xcd + (wg >> 3); }

__device__ inline float4 ldg4(const float *p) { return *reinterpret_cast<const float4 *>(p); }

// MODE 0: Cin % 32 == 0, sd == 1.  MODE 1: Cin % 32 == 0, sd > 1.  MODE 2: any Cin and sd (scalar gather).
template <int BM, int BN, int MODE>
__global__ __launch_bounds__(kConvThreads, 2) void igemm_kernel(IgemmP p)
{
    constexpr int WTM = BM / 2, WTN = BN / 2, MI = WTM / 32, NI = WTN / 32;
    constexpr int RA = BM / 32, RB = BN / 32;  // rows per thread of each operand tile
    __shared__ __attribute__((aligned(16))) float As[BM * kLDK];
    __shared__ __attribute__((aligned(16))) float Bs[BN * kLDK];

    const int ntiles = p.tiles_m * p.tiles_n;
    const int wg = blockIdx.x;
    const int split = wg / (p.tiles_per_xcd * 8);
    const int tile = xcd_remap(wg - split * p.tiles_per_xcd * 8, p.tiles_per_xcd);
    if (tile >= ntiles) return;
    const int tm = tile / p.tiles_n, tn = tile - tm * p.tiles_n;
    const int m0 = tm * BM, n0 = tn * BN;
    const int kc_begin = split * p.chunks_per_split;
    const int kc_end = min(p.kchunks, kc_begin + p.chunks_per_split);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int kq = tid & 7, row_in = tid >> 3;

    // per-row geometry of the gathered operand
    int hn[RA], wnum[RA];
    long abase[RA];
#pragma unroll
    for (int i = 0; i < RA; ++i) {
        const int m = m0 + row_in + 32 * i;
        if (m < p.M) {
            const int n = m / (p.OH * p.OW);
            const int rem = m - n * (p.OH * p.OW);
            const int oh = rem / p.OW, ow = rem - oh * p.OW;
            hn[i] = oh * p.so + p.off;
            wnum[i] = ow * p.so + p.off;
            abase[i] = (long)n * p.IH * p.IW * p.Cin;
        } else {
            hn[i] = -(1 << 28);  // every tap falls outside
            wnum[i] = 0;
            abase[i] = 0;
        }
    }

    float4 ra[RA], rb[RB];
    auto load_chunk = [&](int kc) {
        const int k0 = kc * kBK;
        if (MODE <= 1) {
            const int tap = k0 / p.Cin;
            const int c0 = k0 - tap * p.Cin + kq * 4;
            const int r = tap / p.S, s = tap - r * p.S;
#pragma unroll
            for (int i = 0; i < RA; ++i) {
                int ih = hn[i] + r, iw = wnum[i] + s;
                bool ok = ih >= 0 && iw >= 0;
                if (MODE == 1) {
                    ok = ok && (ih % p.sd == 0) && (iw % p.sd == 0);
                    ih /= p.sd;
                    iw /= p.sd;
                }
                ok = ok && ih < p.IH && iw < p.IW;
                ra[i] = ok ? ldg4(p.a + abase[i] + ((long)ih * p.IW + iw) * p.Cin + c0) : make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
            for (int i = 0; i < RB; ++i) {
                const int j = n0 + row_in + 32 * i;
                rb[i] = j < p.Nout ? ldg4(p.b + (long)j * p.Kdim + k0 + kq * 4) : make_float4(0.f, 0.f, 0.f, 0.f);
            }
        } else {
            float va[RA][4], vb[RB][4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int k = k0 + kq * 4 + e;
                const bool kin = k < p.Kdim;
                const int r = k / (p.S * p.Cin);
                const int rem = k - r * (p.S * p.Cin);
                const int s = rem / p.Cin, c = rem - s * p.Cin;
#pragma unroll
                for (int i = 0; i < RA; ++i) {
                    int ih = hn[i] + r, iw = wnum[i] + s;
                    bool ok = kin && ih >= 0 && iw >= 0 && (ih % p.sd == 0) && (iw % p.sd == 0);
                    ih /= p.sd;
                    iw /= p.sd;
                    ok = ok && ih < p.IH && iw < p.IW;
                    va[i][e] = ok ? p.a[abase[i] + ((long)ih * p.IW + iw) * p.Cin + c] : 0.f;
                }
#pragma unroll
                for (int i = 0; i < RB; ++i) {
                    const int j = n0 + row_in + 32 * i;
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
#pragma unroll
        for (int i = 0; i < RA; ++i) *reinterpret_cast<float4 *>(&As[(row_in + 32 * i) * kLDK + kq * 4]) = ra[i];
#pragma unroll
        for (int i = 0; i < RB; ++i) *reinterpret_cast<float4 *>(&Bs[(row_in + 32 * i) * kLDK + kq * 4]) = rb[i];
    };

    floatx16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    if (kc_begin < kc_end) {
        load_chunk(kc_begin);
        store_chunk();
    }
    __syncthreads();
    // MFMA operand for lane l: row l%32 of the block, reduction element l/32 of the current pair.  A lane
    // reads four consecutive reduction elements at once; pairing element e of lanes 0-31 with element e
    // of lanes 32-63 is a permutation of the reduction order, applied identically to both operands.
    const int frag_off = (lane & 31) * kLDK + (lane >> 5) * 4;
    for (int kc = kc_begin; kc < kc_end; ++kc) {
        const bool more = kc + 1 < kc_end;
        if (more) load_chunk(kc + 1);  // in flight while the current stage is multiplied
#pragma unroll
        for (int kg = 0; kg < kBK / 8; ++kg) {
            float4 af[MI], bf[NI];
#pragma unroll
            for (int i = 0; i < MI; ++i) af[i] = *reinterpret_cast<const float4 *>(&As[(wm * WTM + i * 32) * kLDK + frag_off + kg * 8]);
#pragma unroll
            for (int j = 0; j < NI; ++j) bf[j] = *reinterpret_cast<const float4 *>(&Bs[(wn * WTN + j * 32) * kLDK + frag_off + kg * 8]);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j) {
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i].x, bf[j].x, acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i].y, bf[j].y, acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i].z, bf[j].z, acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i].w, bf[j].w, acc[i][j], 0, 0, 0);
                }
        }
        __syncthreads();
        if (more) store_chunk();
        __syncthreads();
    }

    // Epilogue.  Accumulator element e of lane l is row 8*(e/4) + 4*(l/32) + e%4, column l%32 of its block.
    float *out = p.out + (long)split * p.out_split_stride;
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int m = m0 + wm * WTM + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
            if (m >= p.M) continue;
            long row = m;
            if (p.scatter2) {
                const int n = m / (p.OH * p.OW);
                const int rem = m - n * (p.OH * p.OW);
                const int oh = rem / p.OW, ow = rem - oh * p.OW;
                row = ((long)n * 2 * p.OH + 2 * oh) * (2 * p.OW) + 2 * ow;
            }
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                const int col = n0 + wn * WTN + j * 32 + (lane & 31);
                if (col >= p.Nout) continue;
                out[row * p.Nout + col] = acc[i][j][e];
                if (p.scatter2) {
                    out[(row + 1) * p.Nout + col] = 0.f;
                    out[(row + 2 * p.OW) * p.Nout + col] = 0.f;
                    out[(row + 2 * p.OW + 1) * p.Nout + col] = 0.f;
                }
            }
        }
}

// ---------------------------------------------------------------------------------------------------
struct WgradP {
    const float *dy;  // [Mpix][Kout]
    const float *x;   // N x IH x IW x Cin
    float *out;       // partials: [split][Kout][R*S*Cin]
    int IH, IW, Cin, OH, OW, Kout, R, S, stride, pad;
    int Mpix;         // N*OH*OW
    int Jdim;         // R*S*Cin
    int tiles_k, tiles_j;  // tiles along Kout and along the filter index (taps x channel blocks, or flat for GENERIC)
    int cblocks;           // channel blocks per tap
    int split, pix_per_split;
    long split_stride;
};

// GENERIC = false: Cin % 4 == 0, a tile's columns are BN consecutive channels of one tap.
// GENERIC = true : any Cin; columns are BN consecutive flat filter indices (r,s,c), gathered one float at a time.
template <int BM, int BN, bool GENERIC>
__global__ __launch_bounds__(kConvThreads, 2) void wgrad_kernel(WgradP p)
{
    constexpr int MI = BM / 64, NI = BN / 64;      // 32x32 blocks per wavefront along each side
    constexpr int LDA = BM + 4, LDB = BN + 4;
    constexpr int CA = BM / 4, CB = BN / 4;        // float4 columns per pixel row
    constexpr int PA = kConvThreads / CA, PB = kConvThreads / CB;  // pixel rows per pass
    constexpr int RA = kBK / PA, RB = kBK / PB;
    __shared__ __attribute__((aligned(16))) float As[kBK * LDA];
    __shared__ __attribute__((aligned(16))) float Bs[kBK * LDB];

    const int ntiles = p.tiles_k * p.tiles_j;
    const int split = blockIdx.x / ntiles;
    const int tile = blockIdx.x - split * ntiles;
    const int tk = tile / p.tiles_j, tj = tile - tk * p.tiles_j;
    const int k0 = tk * BM;
    int tap = 0, c0 = 0, j0 = 0;
    if (GENERIC) {
        j0 = tj * BN;
    } else {
        tap = tj / p.cblocks;
        c0 = (tj - tap * p.cblocks) * BN;
        j0 = tap * p.Cin + c0;
    }
    const int fr = tap / p.S, fs = tap - fr * p.S;
    const int pix_begin = split * p.pix_per_split;
    const int pix_end = min(p.Mpix, pix_begin + p.pix_per_split);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int ca = tid % CA, pa = tid / CA;
    const int cb = tid % CB, pb = tid / CB;

    // GENERIC: the four filter indices of this thread's columns, decoded once
    int gr[4], gs[4], gc[4];
    bool gok[4];
    if (GENERIC) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int j = j0 + cb * 4 + e;
            gok[e] = j < p.Jdim;
            gr[e] = j / (p.S * p.Cin);
            const int rem = j - gr[e] * (p.S * p.Cin);
            gs[e] = rem / p.Cin;
            gc[e] = rem - gs[e] * p.Cin;
        }
    }

    float4 ra[RA], rb[RB];
    auto load_chunk = [&](int pix0) {
#pragma unroll
        for (int i = 0; i < RA; ++i) {
            const int pix = pix0 + pa + PA * i;
            const bool ok = pix < pix_end && k0 + ca * 4 < p.Kout;
            ra[i] = ok ? ldg4(p.dy + (long)pix * p.Kout + k0 + ca * 4) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int i = 0; i < RB; ++i) {
            const int pix = pix0 + pb + PB * i;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (pix < pix_end) {
                const int n = pix / (p.OH * p.OW);
                const int rem = pix - n * (p.OH * p.OW);
                const int oh = rem / p.OW, ow = rem - oh * p.OW;
                const long nb = (long)n * p.IH * p.IW * p.Cin;
                if (!GENERIC) {
                    const int ih = oh * p.stride + fr - p.pad, iw = ow * p.stride + fs - p.pad;
                    if (ih >= 0 && ih < p.IH && iw >= 0 && iw < p.IW && c0 + cb * 4 < p.Cin)
                        v = ldg4(p.x + nb + ((long)ih * p.IW + iw) * p.Cin + c0 + cb * 4);
                } else {
                    float t[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int ih = oh * p.stride + gr[e] - p.pad, iw = ow * p.stride + gs[e] - p.pad;
                        const bool ok = gok[e] && ih >= 0 && ih < p.IH && iw >= 0 && iw < p.IW;
                        t[e] = ok ? p.x[nb + ((long)ih * p.IW + iw) * p.Cin + gc[e]] : 0.f;
                    }
                    v = make_float4(t[0], t[1], t[2], t[3]);
                }
            }
            rb[i] = v;
        }
    };
    auto store_chunk = [&]() {
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

    if (pix_begin < pix_end) {
        load_chunk(pix_begin);
        store_chunk();
    }
    __syncthreads();
    // Lane l supplies output index MI*(l%32)+i for block i (interleaved, so that one 8-byte LDS read feeds
    // both blocks) and reduction element l/32 of the current pixel pair.
    const int fa = (lane >> 5) * LDA + wm * (BM / 2) + (lane & 31) * MI;
    const int fb = (lane >> 5) * LDB + wn * (BN / 2) + (lane & 31) * NI;
    for (int pix0 = pix_begin; pix0 < pix_end; pix0 += kBK) {
        const bool more = pix0 + kBK < pix_end;
        if (more) load_chunk(pix0 + kBK);
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
        __syncthreads();
        if (more) store_chunk();
        __syncthreads();
    }

    float *out = p.out + (long)split * p.split_stride;
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int brow = 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
            const int k = k0 + wm * (BM / 2) + brow * MI + i;
            if (k >= p.Kout) continue;
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                const int col = wn * (BN / 2) + (lane & 31) * NI + j;
                const bool ok = GENERIC ? (j0 + col < p.Jdim) : (c0 + col < p.Cin);
                if (ok) out[(long)k * p.Jdim + j0 + col] = acc[i][j][e];
            }
        }
}

// out[i] = sum_s part[s][i], s in increasing order (fixed order: bit-identical from call to call)
__global__ __launch_bounds__(256) void splitk_reduce_kernel(long count4, int split, long stride, const float *__restrict__ part,
                                                            float *__restrict__ out)
{
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= count4) return;
    float4 acc = reinterpret_cast<const float4 *>(part)[i];
    for (int s = 1; s < split; ++s) {
        const float4 v = reinterpret_cast<const float4 *>(part + (long)s * stride)[i];
        acc.x += v.x;
        acc.y += v.y;
        acc.z += v.z;
        acc.w += v.w;
    }
    reinterpret_cast<float4 *>(out)[i] = acc;
}

// Filter of the data gradient: wt[c][R-1-r][S-1-s][k] = w[k][r][s][c]  (32x32 tiles through LDS)
__global__ __launch_bounds__(256) void filter_flip_transpose_kernel(int K, int C, int RS, const float *__restrict__ w,
                                                                    float *__restrict__ wt)
{
    __shared__ float t[32][33];
    const int tap = blockIdx.z;
    const int k0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
    for (int i = ty; i < 32; i += 8) {
        const int k = k0 + i, c = c0 + tx;
        t[i][tx] = (k < K && c < C) ? w[((long)k * RS + tap) * C + c] : 0.f;
    }
    __syncthreads();
    const int tap_t = RS - 1 - tap;  // flipping r and s together reverses the flat tap index
    for (int i = ty; i < 32; i += 8) {
        const int c = c0 + i, k = k0 + tx;
        if (k < K && c < C) wt[((long)c * RS + tap_t) * K + k] = t[tx][i];
    }
}

}  // namespace rn50
