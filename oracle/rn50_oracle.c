/*
 * CPU oracle for one GPU's share of the ResNet-50 training step of
 * "Extremely Large Minibatch SGD: Training ResNet-50 on ImageNet in 15 Minutes".
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call this file:
 * only the tests, the smoke check and the cpu_baseline leg of the benchmark do.
 * It shares no code, header, table or helper with the HIP library.
 *
 * Everything is the plain definition of the result, evaluated in double
 * precision with nested loops.  No blocking, no fusion beyond what the
 * definition states.  OpenMP is applied to the outermost independent loops
 * only.  Tensors are dense, logical order NCHW for activations and KCRS for
 * filters (the textbook order); the tests transpose to the device layout.
 *
 * Passages followed:
 *   - model: ResNet-50 (Section 1 names it; layer geometry from He et al. 2016,
 *     Table 1, which the paper cites);
 *   - batch normalization with the statistics of the current minibatch only,
 *     no moving averages (Section 2, "Batch Normalization without Moving
 *     Averages");
 *   - single-precision compute, half-precision communication (Section 3,
 *     "Software");
 *   - update rule, hyper-parameters and schedules (Appendix A.1, A.2).
 *
 * Parity pins: every function below is pinned by a test in
 * tests/test_oracle_*.py (closed forms, brute force in pure Python, library
 * matmul on special cases, finite differences, adjoint identities, numpy's
 * float16 conversion).  The end-to-end composition of the whole network has no
 * value printed in the paper: it is "parity unpinned" beyond those per-function
 * pins, the architecture totals (25,557,032 parameters) and the initial loss
 * being close to ln(1000).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define IDX4(a, b, c, d, B, C, D) ((((size_t)(a) * (B) + (b)) * (C) + (c)) * (D) + (d))

/* threads the parallel loops use (reported next to the timing of the cpu baseline) */
int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static int out_size(int in, int r, int stride, int pad) { return (in + 2 * pad - r) / stride + 1; }

/* ------------------------------------------------------------------ */
/* Convolution (cross-correlation, zero padding, no bias).             */
/* y[n,k,p,q] = sum_{c,r,s} x[n,c,p*st+r-pad,q*st+s-pad] * w[k,c,r,s]   */
/* ------------------------------------------------------------------ */
void orc_conv2d_fwd(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                    const double *x, const double *w, double *y)
{
    const int P = out_size(H, R, stride, pad), Q = out_size(W, S, stride, pad);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k) {
            double *yp = y + IDX4(n, k, 0, 0, K, P, Q);
            for (int i = 0; i < P * Q; ++i) yp[i] = 0.0;
            for (int c = 0; c < C; ++c)
                for (int r = 0; r < R; ++r)
                    for (int s = 0; s < S; ++s) {
                        const double wv = w[IDX4(k, c, r, s, C, R, S)];
                        for (int p = 0; p < P; ++p) {
                            const int h = p * stride + r - pad;
                            if (h < 0 || h >= H) continue;
                            for (int q = 0; q < Q; ++q) {
                                const int ww = q * stride + s - pad;
                                if (ww < 0 || ww >= W) continue;
                                yp[p * Q + q] += x[IDX4(n, c, h, ww, C, H, W)] * wv;
                            }
                        }
                    }
        }
}

/* dx[n,c,h,w] = sum over (k,r,s,p,q) with h=p*st+r-pad, w=q*st+s-pad of dy[n,k,p,q]*w[k,c,r,s].
 * Every dx element is written (zero where no tap lands). */
void orc_conv2d_bwd_data(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                         const double *dy, const double *w, double *dx)
{
    const int P = out_size(H, R, stride, pad), Q = out_size(W, S, stride, pad);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c) {
            double *dxp = dx + IDX4(n, c, 0, 0, C, H, W);
            for (int i = 0; i < H * W; ++i) dxp[i] = 0.0;
            for (int k = 0; k < K; ++k)
                for (int r = 0; r < R; ++r)
                    for (int s = 0; s < S; ++s) {
                        const double wv = w[IDX4(k, c, r, s, C, R, S)];
                        for (int p = 0; p < P; ++p) {
                            const int h = p * stride + r - pad;
                            if (h < 0 || h >= H) continue;
                            for (int q = 0; q < Q; ++q) {
                                const int ww = q * stride + s - pad;
                                if (ww < 0 || ww >= W) continue;
                                dxp[h * W + ww] += dy[IDX4(n, k, p, q, K, P, Q)] * wv;
                            }
                        }
                    }
        }
}

/* dw[k,c,r,s] = sum_{n,p,q} dy[n,k,p,q] * x[n,c,p*st+r-pad,q*st+s-pad]; dw is overwritten. */
void orc_conv2d_bwd_weight(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                           const double *x, const double *dy, double *dw)
{
    const int P = out_size(H, R, stride, pad), Q = out_size(W, S, stride, pad);
#pragma omp parallel for collapse(2) schedule(static)
    for (int k = 0; k < K; ++k)
        for (int c = 0; c < C; ++c)
            for (int r = 0; r < R; ++r)
                for (int s = 0; s < S; ++s) {
                    double acc = 0.0;
                    for (int n = 0; n < N; ++n)
                        for (int p = 0; p < P; ++p) {
                            const int h = p * stride + r - pad;
                            if (h < 0 || h >= H) continue;
                            for (int q = 0; q < Q; ++q) {
                                const int ww = q * stride + s - pad;
                                if (ww < 0 || ww >= W) continue;
                                acc += dy[IDX4(n, k, p, q, K, P, Q)] * x[IDX4(n, c, h, ww, C, H, W)];
                            }
                        }
                    dw[IDX4(k, c, r, s, C, R, S)] = acc;
                }
}

/* ------------------------------------------------------------------ */
/* Batch normalization with the current minibatch's statistics only.   */
/* mean_c = (1/M) sum x, var_c = (1/M) sum (x-mean_c)^2 (two passes),   */
/* invstd_c = 1/sqrt(var_c+eps), y = gamma*(x-mean)*invstd + beta,      */
/* then optionally + residual, then optionally ReLU.  The saved mean    */
/* and invstd are the "last minibatch" statistics; no running average   */
/* exists anywhere.                                                     */
/* ------------------------------------------------------------------ */
void orc_bn_fwd(int N, int C, int H, int W, const double *x, const double *gamma, const double *beta,
                double eps, const double *residual /* or NULL */, int relu,
                double *y, double *save_mean, double *save_invstd)
{
    const size_t HW = (size_t)H * W;
    const double M = (double)N * (double)HW;
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        double sum = 0.0;
        for (int n = 0; n < N; ++n)
            for (size_t i = 0; i < HW; ++i) sum += x[((size_t)n * C + c) * HW + i];
        const double mean = sum / M;
        double ss = 0.0;
        for (int n = 0; n < N; ++n)
            for (size_t i = 0; i < HW; ++i) {
                const double d = x[((size_t)n * C + c) * HW + i] - mean;
                ss += d * d;
            }
        const double var = ss / M;
        const double invstd = 1.0 / sqrt(var + eps);
        save_mean[c] = mean;
        save_invstd[c] = invstd;
        for (int n = 0; n < N; ++n)
            for (size_t i = 0; i < HW; ++i) {
                const size_t o = ((size_t)n * C + c) * HW + i;
                double v = gamma[c] * (x[o] - mean) * invstd + beta[c];
                if (residual) v += residual[o];
                if (relu && !(v > 0.0)) v = 0.0;
                y[o] = v;
            }
    }
}

/* Backward of the above.  dz = dy * [y > 0] when ReLU was applied (the mask comes from the stored
 * forward output y, derivative at exactly 0 taken as 0), else dz = dy.
 * dbeta = sum dz, dgamma = sum dz*xhat, dx = gamma*invstd*(dz - dbeta/M - xhat*dgamma/M),
 * and, when a residual was added in the forward, dresidual = dz. */
void orc_bn_bwd(int N, int C, int H, int W, const double *x, const double *dy, const double *y /* or NULL */,
                const double *gamma, const double *save_mean, const double *save_invstd, int relu,
                double *dx, double *dresidual /* or NULL */, double *dgamma, double *dbeta)
{
    const size_t HW = (size_t)H * W;
    const double M = (double)N * (double)HW;
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        const double mean = save_mean[c], invstd = save_invstd[c];
        double db = 0.0, dg = 0.0;
        for (int n = 0; n < N; ++n)
            for (size_t i = 0; i < HW; ++i) {
                const size_t o = ((size_t)n * C + c) * HW + i;
                const double dz = (relu && !(y[o] > 0.0)) ? 0.0 : dy[o];
                db += dz;
                dg += dz * (x[o] - mean) * invstd;
            }
        dbeta[c] = db;
        dgamma[c] = dg;
        for (int n = 0; n < N; ++n)
            for (size_t i = 0; i < HW; ++i) {
                const size_t o = ((size_t)n * C + c) * HW + i;
                const double dz = (relu && !(y[o] > 0.0)) ? 0.0 : dy[o];
                const double xhat = (x[o] - mean) * invstd;
                dx[o] = gamma[c] * invstd * (dz - db / M - xhat * dg / M);
                if (dresidual) dresidual[o] = dz;
            }
    }
}

/* ------------------------------------------------------------------ */
/* Pooling.                                                            */
/* ------------------------------------------------------------------ */
/* Max pooling; padding never wins (treated as -inf).  argmax[n,c,p,q] is the flat h*W+w index of
 * the first maximal element in row-major window order. */
void orc_maxpool_fwd(int N, int C, int H, int W, int R, int stride, int pad,
                     const double *x, double *y, int32_t *argmax)
{
    const int P = out_size(H, R, stride, pad), Q = out_size(W, R, stride, pad);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    double best = -INFINITY;
                    int bi = -1;
                    for (int r = 0; r < R; ++r)
                        for (int s = 0; s < R; ++s) {
                            const int h = p * stride + r - pad, ww = q * stride + s - pad;
                            if (h < 0 || h >= H || ww < 0 || ww >= W) continue;
                            const double v = x[IDX4(n, c, h, ww, C, H, W)];
                            if (bi < 0 || v > best) { best = v; bi = h * W + ww; }
                        }
                    y[IDX4(n, c, p, q, C, P, Q)] = best;
                    argmax[IDX4(n, c, p, q, C, P, Q)] = bi;
                }
}

/* dx[arg-max position] += dy; overlapping windows accumulate. */
void orc_maxpool_bwd(int N, int C, int H, int W, int R, int stride, int pad,
                     const double *dy, const int32_t *argmax, double *dx)
{
    const int P = out_size(H, R, stride, pad), Q = out_size(W, R, stride, pad);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c) {
            double *dxp = dx + IDX4(n, c, 0, 0, C, H, W);
            for (int i = 0; i < H * W; ++i) dxp[i] = 0.0;
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    const size_t o = IDX4(n, c, p, q, C, P, Q);
                    dxp[argmax[o]] += dy[o];
                }
        }
}

/* Global average pooling: y[n,c] = mean over H*W. */
void orc_avgpool_fwd(int N, int C, int H, int W, const double *x, double *y)
{
    const size_t HW = (size_t)H * W;
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c) {
            double s = 0.0;
            for (size_t i = 0; i < HW; ++i) s += x[((size_t)n * C + c) * HW + i];
            y[(size_t)n * C + c] = s / (double)HW;
        }
}

void orc_avgpool_bwd(int N, int C, int H, int W, const double *dy, double *dx)
{
    const size_t HW = (size_t)H * W;
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (size_t i = 0; i < HW; ++i) dx[((size_t)n * C + c) * HW + i] = dy[(size_t)n * C + c] / (double)HW;
}

/* ------------------------------------------------------------------ */
/* Fully connected layer: y[n,k] = sum_j f[n,j]*w[k,j] + b[k].          */
/* ------------------------------------------------------------------ */
void orc_fc_fwd(int N, int J, int K, const double *f, const double *w, const double *b, double *y)
{
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k) {
            double acc = 0.0;
            for (int j = 0; j < J; ++j) acc += f[(size_t)n * J + j] * w[(size_t)k * J + j];
            y[(size_t)n * K + k] = acc + b[k];
        }
}

void orc_fc_bwd(int N, int J, int K, const double *f, const double *w, const double *dy,
                double *df, double *dw, double *db)
{
#pragma omp parallel for schedule(static)
    for (int k = 0; k < K; ++k) {
        double sb = 0.0;
        for (int n = 0; n < N; ++n) sb += dy[(size_t)n * K + k];
        db[k] = sb;
        for (int j = 0; j < J; ++j) {
            double acc = 0.0;
            for (int n = 0; n < N; ++n) acc += dy[(size_t)n * K + k] * f[(size_t)n * J + j];
            dw[(size_t)k * J + j] = acc;
        }
    }
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int j = 0; j < J; ++j) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k) acc += dy[(size_t)n * K + k] * w[(size_t)k * J + j];
            df[(size_t)n * J + j] = acc;
        }
}

/* ------------------------------------------------------------------ */
/* Softmax cross-entropy, mean over the local batch.                   */
/* loss = -(1/N) sum_n log softmax(logits_n)[label_n]                   */
/* dlogits = (softmax - onehot)/N                                       */
/* ------------------------------------------------------------------ */
double orc_softmax_ce(int N, int K, const double *logits, const int32_t *labels, double *dlogits /* or NULL */)
{
    double loss = 0.0;
    for (int n = 0; n < N; ++n) {
        const double *z = logits + (size_t)n * K;
        double mx = z[0];
        for (int k = 1; k < K; ++k) if (z[k] > mx) mx = z[k];
        double se = 0.0;
        for (int k = 0; k < K; ++k) se += exp(z[k] - mx);
        const double lse = mx + log(se);
        loss += lse - z[labels[n]];
        if (dlogits)
            for (int k = 0; k < K; ++k)
                dlogits[(size_t)n * K + k] = (exp(z[k] - lse) - (k == labels[n] ? 1.0 : 0.0)) / (double)N;
    }
    return loss / (double)N;
}

/* ------------------------------------------------------------------ */
/* Half-precision communication buffer.                                */
/* fp32 -> IEEE binary16, round to nearest, ties to even, by integer   */
/* bit manipulation: overflow -> +-inf, gradual underflow to           */
/* subnormals, signed zero kept, NaN -> a quiet NaN.                   */
/* ------------------------------------------------------------------ */
static uint16_t f32_to_f16_rne(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    const uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    const uint32_t a = u & 0x7fffffffu;
    if (a > 0x7f800000u) return (uint16_t)(sign | 0x7e00u);       /* NaN */
    if (a == 0x7f800000u) return (uint16_t)(sign | 0x7c00u);      /* inf */
    const int e = (int)(a >> 23) - 127;                           /* unbiased exponent */
    uint32_t man = a & 0x7fffffu;
    if (e > 15) return (uint16_t)(sign | 0x7c00u);                /* >= 2^16: overflow */
    if (e >= -14) {
        /* normal half: keep 10 mantissa bits, round on the 13 dropped ones */
        uint32_t h = ((uint32_t)(e + 15) << 10) | (man >> 13);
        const uint32_t rem = man & 0x1fffu;
        if (rem > 0x1000u || (rem == 0x1000u && (h & 1u))) h += 1u; /* carry may reach the exponent, even to inf */
        return (uint16_t)(sign | h);
    }
    if (e < -25) return sign;                                     /* below half of the smallest subnormal */
    /* subnormal half: value = m * 2^-24 with m = round(1.man * 2^(e+24)) */
    man |= 0x800000u;                                             /* 24-bit significand, value man*2^(e-23) */
    const int shift = -e - 1;                                     /* man*2^(e-23) / 2^-24 = man >> (-e-1); shift in 14..24 */
    uint32_t h = man >> shift;
    const uint32_t rem = man & ((1u << shift) - 1u);
    const uint32_t half = 1u << (shift - 1);
    if (rem > half || (rem == half && (h & 1u))) h += 1u;
    return (uint16_t)(sign | h);
}

static double f16_to_f64(uint16_t h)
{
    const int sign = (h >> 15) & 1, e = (h >> 10) & 0x1f, man = h & 0x3ff;
    double v;
    if (e == 0) v = ldexp((double)man, -24);
    else if (e == 31) v = man ? NAN : INFINITY;
    else v = ldexp((double)(man | 0x400), e - 25);
    return sign ? -v : v;
}

void orc_grad_pack_fp16(size_t count, const float *g, uint16_t *out16)
{
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < count; ++i) out16[i] = f32_to_f16_rne(g[i]);
}

/* g[i] = value(in16[i]) * scale, in double.  For a power-of-two scale and |result| in fp32's
 * normal range the product is exact, so rounding it to fp32 loses nothing. */
void orc_grad_unpack_fp16(size_t count, const uint16_t *in16, double scale, double *g)
{
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < count; ++i) g[i] = f16_to_f64(in16[i]) * scale;
}

/* ------------------------------------------------------------------ */
/* Update rule (Appendix A.1), one element at a time, in this order:   */
/*   m     <- mu2*m + (1-mu2)*g^2                                       */
/*   Delta <- mu1*Delta - (a_sgd + a_rms/(sqrt(m)+eps))*g               */
/*   theta <- theta + eta*Delta                                         */
/* with the new m used for Delta and the new Delta used for theta.     */
/* Weight decay is not in the paper's equations; when decay[i] != 0    */
/* (or decay == NULL and wd != 0) g is first replaced by g + wd*theta. */
/* ------------------------------------------------------------------ */
void orc_opt_update(size_t count, double *theta, double *delta, double *m, const double *g,
                    const uint8_t *decay /* per element, or NULL = all */,
                    double eta, double mu1, double mu2, double eps, double a_sgd, double a_rms, double wd)
{
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < count; ++i) {
        double gi = g[i];
        if (wd != 0.0 && (!decay || decay[i])) gi += wd * theta[i];
        m[i] = mu2 * m[i] + (1.0 - mu2) * gi * gi;
        delta[i] = mu1 * delta[i] - (a_sgd + a_rms / (sqrt(m[i]) + eps)) * gi;
        theta[i] = theta[i] + eta * delta[i];
    }
}

/* ------------------------------------------------------------------ */
/* Schedules (Appendix A.1, A.2), host scalars.                        */
/* ------------------------------------------------------------------ */
/* alpha_SGD(epoch): exponential rise to 1/2 at `center`, then linear up to 1 at center+period/2, then 1.
 * The printed middle branch has slope 2/period, which would give 1.5 at center+period/2 and
 * contradicts the text (reaches 1 there, ELU-like i.e. smooth at the joint).  as_printed == 0 uses
 * the slope 1/period that satisfies the text; as_printed != 0 evaluates the printed formula
 * clipped to 1. */
double orc_alpha_sgd(double epoch, double center, double period, int as_printed)
{
    if (epoch < center) return 0.5 * exp(2.0 * (epoch - center) / period);
    if (epoch < center + 0.5 * period) {
        const double slope = as_printed ? 2.0 : 1.0;
        const double v = 0.5 + slope * (epoch - center) / period;
        return v < 1.0 ? v : 1.0;
    }
    return 1.0;
}

/* The transition functions Appendix A.1 says were examined and rejected.  The paper only names them (a sudden switch, a
 * linear and a sigmoid function); each is written here as the plainest function of that name that passes 1/2 at the centre
 * and, where it has a slope there, has the ELU-like function's slope 1/period:
 *   kind 1, linear : 1/2 + (epoch-center)/period clipped to [0,1]   (starts abruptly at center - period/2)
 *   kind 2, sigmoid: 1 / (1 + exp(-4 (epoch-center)/period))
 *   kind 3, sudden : 0 before the centre, 1 from it on
 * kind 0 is the paper's own function above. */
double orc_alpha_sgd_transition(double epoch, double center, double period, int kind)
{
    const double t = (epoch - center) / period;
    if (kind == 0) return orc_alpha_sgd(epoch, center, period, 0);
    if (kind == 1) {
        const double v = 0.5 + t;
        return v < 0.0 ? 0.0 : (v > 1.0 ? 1.0 : v);
    }
    if (kind == 2) return 1.0 / (1.0 + exp(-4.0 * t));
    if (kind == 3) return epoch < center ? 0.0 : 1.0;
    return NAN;
}

/* alpha_RMSprop = (1 - alpha_SGD) * eta_RMSprop / eta_SGD */
double orc_alpha_rmsprop(double a_sgd, double eta_rmsprop, double eta_sgd) { return (1.0 - a_sgd) * eta_rmsprop / eta_sgd; }

/* eta_base = 0.1 * n * b_local / 256 */
double orc_lr_base(int n_workers, int b_local) { return 0.1 * (double)n_workers * (double)b_local / 256.0; }

/* Slow-start schedule: 0.5 eta_base for epochs [0,40), 0.075 for [40,70), 0.01 for [70,85), 0.001 after. */
double orc_lr_slow_start(double epoch, int n_workers, int b_local)
{
    const double base = orc_lr_base(n_workers, b_local);
    if (epoch < 40.0) return 0.5 * base;
    if (epoch < 70.0) return 0.075 * base;
    if (epoch < 85.0) return 0.01 * base;
    return 0.001 * base;
}
