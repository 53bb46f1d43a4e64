/*
 * CPU oracle for one pipeline stage's layer arithmetic.  TEST INFRASTRUCTURE ONLY:
 * it exists to check the HIP library and to be timed beside it as a baseline; the
 * product never calls it, and it shares no code with the HIP path.
 *
 * The paper (BaPipe, Sec. III-A/III-B) treats a stage as "forward and backward
 * propagation of a contiguous subset of layers" of VGG-16 / ResNet-50 and gives no
 * layer mathematics of its own, so every function here is the plain textbook
 * definition of the layer and of its adjoint, written as direct loops:
 *   convolution = cross-correlation with zero padding, Ho = floor((H+2p-k)/s)+1 ;
 *   ReLU backward passes the gradient where the forward output is > 0 ;
 *   max-pool keeps the first maximum in row-major window order (padded positions are not
 *   candidates; overlapping windows that pick the same input add their gradients) ;
 *   average pool is the mean of a k x k window, stride k, its adjoint spreads dy / k^2 ;
 *   batch-norm uses biased per-channel statistics of the given (micro-)batch ;
 *   the LSTM layer (the sequence-to-sequence workload's layer, Sec. IV-A) is the standard cell with
 *   gates in the order input, forget, cell candidate, output, zero initial state ;
 *   the loss is softmax cross-entropy scaled by a caller-given factor ;
 *   the update is plain SGD (the paper's 2*w weights memory leaves no optimiser state).
 * All tensors are double, activations NCHW, conv weights OIHW, linear weights [out][in].
 * Loops are ordered so that the innermost one has no loop-carried dependency where
 * possible; each output still receives its terms in (ci, r, s) order.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <omp.h>

#define IDX4(n, c, h, w, C, H, W) ((((size_t)(n) * (C) + (c)) * (H) + (h)) * (W) + (w))

int orc_num_threads(void) { return omp_get_max_threads(); }

/* Nearest-even rounding of a double to the bf16 grid (1 sign, 8 exponent, 7 fraction
 * bits, fp32 exponent range, gradual underflow), result returned as double. */
static double round_bf16_one(double v)
{
    if (v != v || isinf(v)) return v;
    double a = fabs(v);
    if (a < 0x1p-126) {                       /* subnormal range: grid step 2^-133 */
        double q = nearbyint(a * 0x1p133) * 0x1p-133;
        return v < 0 ? -q : q;
    }
    uint64_t u;
    memcpy(&u, &v, 8);
    const int drop = 52 - 7;                  /* fraction bits that do not fit */
    uint64_t lsb = (u >> drop) & 1u;
    u += ((uint64_t)1 << (drop - 1)) - 1 + lsb;
    u &= ~(((uint64_t)1 << drop) - 1);
    double r;
    memcpy(&r, &u, 8);
    if (fabs(r) > 0x1.FEp127) r = (v < 0) ? -INFINITY : INFINITY;
    return r;
}

void orc_round_bf16(double *a, size_t n)
{
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) a[i] = round_bf16_one(a[i]);
}


/* Output columns q in [lo, hi) are those whose tap column q*st+s-pad lies inside [0, W). */
static inline void tap_range(int W, int Wo, int s, int st, int pad, int *lo, int *hi)
{
    int a = pad - s, l = a > 0 ? (a + st - 1) / st : 0;
    int b = W - 1 + pad - s, h = b < 0 ? 0 : b / st + 1;
    *lo = l;
    *hi = h < Wo ? h : Wo;
}

/* y[n,co,p,q] = b[co] + sum_{ci,r,s} w[co,ci,r,s] * x[n,ci,p*st+r-pad,q*st+s-pad]  */
void orc_conv2d_fwd(const double *x, const double *w, const double *b, double *y,
                    int N, int Cin, int H, int W, int Cout, int kh, int kw, int st, int pad)
{
    const int Ho = (H + 2 * pad - kh) / st + 1, Wo = (W + 2 * pad - kw) / st + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int co = 0; co < Cout; ++co) {
            double *yo = y + IDX4(n, co, 0, 0, Cout, Ho, Wo);
            const double b0 = b ? b[co] : 0.0;
            for (int i = 0; i < Ho * Wo; ++i) yo[i] = b0;
            for (int ci = 0; ci < Cin; ++ci)
                for (int r = 0; r < kh; ++r)
                    for (int s = 0; s < kw; ++s) {
                        const double wv = w[IDX4(co, ci, r, s, Cin, kh, kw)];
                        int qlo, qhi;
                        tap_range(W, Wo, s, st, pad, &qlo, &qhi);
                        for (int p = 0; p < Ho; ++p) {
                            const int ih = p * st + r - pad;
                            if (ih < 0 || ih >= H) continue;
                            const double *xr = x + IDX4(n, ci, ih, 0, Cin, H, W) + (s - pad);
                            double *yr = yo + (size_t)p * Wo;
                            for (int q = qlo; q < qhi; ++q) yr[q] += wv * xr[q * st];
                        }
                    }
        }
}

/* Adjoint of orc_conv2d_fwd in x: every product w*dy is scattered to the input
 * position it was read from.  dx is overwritten. */
void orc_conv2d_dgrad(const double *dy, const double *w, double *dx,
                      int N, int Cin, int H, int W, int Cout, int kh, int kw, int st, int pad)
{
    const int Ho = (H + 2 * pad - kh) / st + 1, Wo = (W + 2 * pad - kw) / st + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int ci = 0; ci < Cin; ++ci) {
            double *dxo = dx + IDX4(n, ci, 0, 0, Cin, H, W);
            for (int i = 0; i < H * W; ++i) dxo[i] = 0.0;
            for (int co = 0; co < Cout; ++co)
                for (int r = 0; r < kh; ++r)
                    for (int s = 0; s < kw; ++s) {
                        const double wv = w[IDX4(co, ci, r, s, Cin, kh, kw)];
                        int qlo, qhi;
                        tap_range(W, Wo, s, st, pad, &qlo, &qhi);
                        for (int p = 0; p < Ho; ++p) {
                            const int ih = p * st + r - pad;
                            if (ih < 0 || ih >= H) continue;
                            const double *gr = dy + IDX4(n, co, p, 0, Cout, Ho, Wo);
                            double *dr = dxo + (size_t)ih * W + (s - pad);
                            for (int q = qlo; q < qhi; ++q) dr[q * st] += wv * gr[q];
                        }
                    }
        }
}

/* dw[co,ci,r,s] += sum_{n,p,q} dy[n,co,p,q] * x[n,ci,p*st+r-pad,q*st+s-pad] ;
 * db[co] += sum_{n,p,q} dy[n,co,p,q].  Both ACCUMULATE (weights gradients are summed
 * over the micro-batches of a mini-batch, paper Sec. III-B-1). db may be NULL. */
void orc_conv2d_wgrad(const double *x, const double *dy, double *dw, double *db,
                      int N, int Cin, int H, int W, int Cout, int kh, int kw, int st, int pad)
{
    const int Ho = (H + 2 * pad - kh) / st + 1, Wo = (W + 2 * pad - kw) / st + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int co = 0; co < Cout; ++co)
        for (int ci = 0; ci < Cin; ++ci)
            for (int r = 0; r < kh; ++r)
                for (int s = 0; s < kw; ++s) {
                    double acc = 0.0;
                    int qlo, qhi;
                    tap_range(W, Wo, s, st, pad, &qlo, &qhi);
                    for (int n = 0; n < N; ++n)
                        for (int p = 0; p < Ho; ++p) {
                            const int ih = p * st + r - pad;
                            if (ih < 0 || ih >= H) continue;
                            const double *xr = x + IDX4(n, ci, ih, 0, Cin, H, W) + (s - pad);
                            const double *gr = dy + IDX4(n, co, p, 0, Cout, Ho, Wo);
                            double rowacc = 0.0;
#pragma omp simd reduction(+ : rowacc)
                            for (int q = qlo; q < qhi; ++q) rowacc += gr[q] * xr[q * st];
                            acc += rowacc;
                        }
                    dw[IDX4(co, ci, r, s, Cin, kh, kw)] += acc;
                }
    if (db) {
#pragma omp parallel for schedule(static)
        for (int co = 0; co < Cout; ++co) {
            double acc = 0.0;
            for (int n = 0; n < N; ++n) {
                const double *g = dy + IDX4(n, co, 0, 0, Cout, Ho, Wo);
                for (int i = 0; i < Ho * Wo; ++i) acc += g[i];
            }
            db[co] += acc;
        }
    }
}

/* y = max(x, 0) */
void orc_relu_fwd(const double *x, double *y, size_t n)
{
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) y[i] = x[i] > 0.0 ? x[i] : 0.0;
}

/* dx = dy where the forward OUTPUT y is > 0, else 0 */
void orc_relu_bwd(const double *y, const double *dy, double *dx, size_t n)
{
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) dx[i] = y[i] > 0.0 ? dy[i] : 0.0;
}

/* Max-pool over kh x kw windows, stride st, implicit -inf padding `pad`.
 * idx = dh*kw+dw of the first maximum met scanning the window row-major
 * (a later element replaces the current one only if strictly greater). */
void orc_maxpool_fwd(const double *x, double *y, uint8_t *idx,
                     int N, int C, int H, int W, int kh, int kw, int st, int pad)
{
    const int Ho = (H + 2 * pad - kh) / st + 1, Wo = (W + 2 * pad - kw) / st + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int p = 0; p < Ho; ++p)
                for (int q = 0; q < Wo; ++q) {
                    double best = -INFINITY;
                    int bi = -1;
                    for (int dh = 0; dh < kh; ++dh)
                        for (int dw = 0; dw < kw; ++dw) {
                            const int ih = p * st + dh - pad, iw = q * st + dw - pad;
                            if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                            const double v = x[IDX4(n, c, ih, iw, C, H, W)];
                            if (bi < 0 || v > best) { best = v; bi = dh * kw + dw; }
                        }
                    y[IDX4(n, c, p, q, C, Ho, Wo)] = best;
                    idx[IDX4(n, c, p, q, C, Ho, Wo)] = (uint8_t)bi;
                }
}

/* dx is zero except dx[argmax position of each window] += dy[window]. */
void orc_maxpool_bwd(const double *dy, const uint8_t *idx, double *dx,
                     int N, int C, int H, int W, int kh, int kw, int st, int pad)
{
    const int Ho = (H + 2 * pad - kh) / st + 1, Wo = (W + 2 * pad - kw) / st + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c) {
            double *d = dx + IDX4(n, c, 0, 0, C, H, W);
            for (int i = 0; i < H * W; ++i) d[i] = 0.0;
            for (int p = 0; p < Ho; ++p)
                for (int q = 0; q < Wo; ++q) {
                    const int bi = idx[IDX4(n, c, p, q, C, Ho, Wo)];
                    const int ih = p * st + bi / kw - pad, iw = q * st + bi % kw - pad;
                    d[(size_t)ih * W + iw] += dy[IDX4(n, c, p, q, C, Ho, Wo)];
                }
        }
}

/* y[n,c,p,q] = mean of the kh x kw window at (p*kh, q*kw): stride = window, no padding;
 * rows / columns beyond the last full window are ignored. */
void orc_avgpool_fwd(const double *x, double *y, int N, int C, int H, int W, int kh, int kw)
{
    const int Ho = H / kh, Wo = W / kw;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int p = 0; p < Ho; ++p)
                for (int q = 0; q < Wo; ++q) {
                    double s = 0.0;
                    for (int dh = 0; dh < kh; ++dh)
                        for (int dw = 0; dw < kw; ++dw)
                            s += x[IDX4(n, c, p * kh + dh, q * kw + dw, C, H, W)];
                    y[IDX4(n, c, p, q, C, Ho, Wo)] = s / (double)(kh * kw);
                }
}

/* Adjoint of the above: every input of a window receives dy / (kh*kw); inputs outside all
 * windows receive zero. */
void orc_avgpool_bwd(const double *dy, double *dx, int N, int C, int H, int W, int kh, int kw)
{
    const int Ho = H / kh, Wo = W / kw;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int h = 0; h < H; ++h)
                for (int w = 0; w < W; ++w) {
                    const int p = h / kh, q = w / kw;
                    dx[IDX4(n, c, h, w, C, H, W)] =
                        (p < Ho && q < Wo) ? dy[IDX4(n, c, p, q, C, Ho, Wo)] / (double)(kh * kw) : 0.0;
                }
}

/* LSTM layer over sequences of T steps.  x is [N][In][T] (the sequence axis is the H axis of an
 * NCHW tensor of width 1), y is [N][Hd][T].  w is [4*Hd][In+Hd]: row k of gate block q (q = 0..3
 * for input, forget, candidate, output; k = q*Hd + j) holds the In input weights, then the Hd
 * recurrent weights; b is [4*Hd] or NULL.  With h_{-1} = c_{-1} = 0:
 *   P_t   = W_x x_t + b                              (input projection, all steps)
 *   a_t   = P_t + W_h h_{t-1}
 *   i,f,o = sigmoid(a_t[0], a_t[1], a_t[3]) ; g = tanh(a_t[2])
 *   c_t   = f*c_{t-1} + i*g ; h_t = o*tanh(c_t) ; y[:, :, t] = h_t
 * gates [N][T][4*Hd] (i, f, g, o after their non-linearities) and cells [N][T][Hd] are returned
 * for the backward pass.  round16 != 0 rounds P_t and h_t to bf16 where an implementation with
 * 16-bit storage keeps them (P is a stored GEMM output, h_t is the layer output). */
static double sigm(double v) { return 1.0 / (1.0 + exp(-v)); }

void orc_lstm_fwd(const double *x, const double *w, const double *b, double *y, double *gates,
                  double *cells, int N, int In, int Hd, int T, int round16)
{
    const int G = 4 * Hd, ld = In + Hd;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        double *a = (double *)malloc(sizeof(double) * (size_t)(G + 2 * Hd));
        double *hp = a + G, *cp = hp + Hd;
        for (int j = 0; j < Hd; ++j) hp[j] = cp[j] = 0.0;
        for (int t = 0; t < T; ++t) {
            for (int k = 0; k < G; ++k) {
                double p = b ? b[k] : 0.0;
                for (int c = 0; c < In; ++c) p += w[(size_t)k * ld + c] * x[((size_t)n * In + c) * T + t];
                if (round16) p = round_bf16_one(p);
                double r = 0.0;
                for (int j = 0; j < Hd; ++j) r += w[(size_t)k * ld + In + j] * hp[j];
                a[k] = p + r;
            }
            double *gt = gates + ((size_t)n * T + t) * G, *ct = cells + ((size_t)n * T + t) * Hd;
            for (int j = 0; j < Hd; ++j) {
                const double ig = sigm(a[j]), fg = sigm(a[Hd + j]), gg = tanh(a[2 * Hd + j]), og = sigm(a[3 * Hd + j]);
                gt[j] = ig; gt[Hd + j] = fg; gt[2 * Hd + j] = gg; gt[3 * Hd + j] = og;
                ct[j] = fg * cp[j] + ig * gg;
            }
            for (int j = 0; j < Hd; ++j) {
                double h = gt[3 * Hd + j] * tanh(ct[j]);
                if (round16) h = round_bf16_one(h);
                cp[j] = ct[j];
                hp[j] = h;
                y[((size_t)n * Hd + j) * T + t] = h;
            }
        }
        free(a);
    }
}

/* Back-propagation through time of the layer above.  With dh_t = dy_t + W_h^T D_{t+1} and
 * dc_t = dh_t*o*(1-tanh(c_t)^2) + dc_{t+1}*f_{t+1}, the gradient w.r.t. the pre-activations is
 *   D_t = ( dc_t*g*i(1-i), dc_t*c_{t-1}*f(1-f), dc_t*i*(1-g^2), dh_t*tanh(c_t)*o(1-o) )
 * and dx_t = W_x^T D_t, dW_x += D_t x_t^T, dW_h += D_t h_{t-1}^T, db += D_t.
 * round16 != 0 rounds D_t to bf16 (it is stored as the operand of those products).
 * dx may be NULL; dw [4*Hd][In+Hd] and db (may be NULL) are accumulated into.  y is the forward
 * output (h_t), D is scratch of N*T*4*Hd doubles supplied by the caller. */
void orc_lstm_bwd(const double *x, const double *y, const double *w, const double *gates,
                  const double *cells, const double *dy, double *dx, double *dw, double *db, double *D,
                  int N, int In, int Hd, int T, int round16)
{
    const int G = 4 * Hd, ld = In + Hd;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        double *r = (double *)malloc(sizeof(double) * (size_t)(2 * Hd));
        double *dcn = r + Hd;                          /* dc_{t+1} * f_{t+1} */
        for (int j = 0; j < Hd; ++j) r[j] = dcn[j] = 0.0;
        for (int t = T - 1; t >= 0; --t) {
            const double *gt = gates + ((size_t)n * T + t) * G, *ct = cells + ((size_t)n * T + t) * Hd;
            double *Dt = D + ((size_t)n * T + t) * G;
            for (int j = 0; j < Hd; ++j) {
                const double ig = gt[j], fg = gt[Hd + j], gg = gt[2 * Hd + j], og = gt[3 * Hd + j];
                const double th = tanh(ct[j]);
                const double cprev = t > 0 ? ct[j - Hd] : 0.0;
                const double dh = dy[((size_t)n * Hd + j) * T + t] + r[j];
                const double dc = dh * og * (1.0 - th * th) + dcn[j];
                Dt[j] = dc * gg * ig * (1.0 - ig);
                Dt[Hd + j] = dc * cprev * fg * (1.0 - fg);
                Dt[2 * Hd + j] = dc * ig * (1.0 - gg * gg);
                Dt[3 * Hd + j] = dh * th * og * (1.0 - og);
                dcn[j] = dc * fg;
            }
            if (round16)
                for (int k = 0; k < G; ++k) Dt[k] = round_bf16_one(Dt[k]);
            for (int j = 0; j < Hd; ++j) {
                double s = 0.0;
                for (int k = 0; k < G; ++k) s += Dt[k] * w[(size_t)k * ld + In + j];
                r[j] = s;
            }
            if (dx)
                for (int c = 0; c < In; ++c) {
                    double s = 0.0;
                    for (int k = 0; k < G; ++k) s += Dt[k] * w[(size_t)k * ld + c];
                    dx[((size_t)n * In + c) * T + t] = s;
                }
        }
        free(r);
    }
#pragma omp parallel for schedule(static)
    for (int k = 0; k < G; ++k) {
        for (int n = 0; n < N; ++n)
            for (int t = 0; t < T; ++t) {
                const double d = D[((size_t)n * T + t) * G + k];
                for (int c = 0; c < In; ++c) dw[(size_t)k * ld + c] += d * x[((size_t)n * In + c) * T + t];
                if (t > 0)
                    for (int j = 0; j < Hd; ++j) dw[(size_t)k * ld + In + j] += d * y[((size_t)n * Hd + j) * T + t - 1];
                if (db) db[k] += d;
            }
    }
}

/* Training-mode batch-norm over (N,H,W) per channel:
 *   mu = mean(x), var = mean((x-mu)^2)  (biased), inv = 1/sqrt(var+eps),
 *   xhat = (x-mu)*inv, y = gamma*xhat + beta.  mean[] and invstd[] are returned. */
void orc_bn_fwd(const double *x, const double *gamma, const double *beta, double eps,
                double *y, double *mean, double *invstd, int N, int C, int HW)
{
    const double m = (double)N * HW;
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        double s = 0.0;
        for (int n = 0; n < N; ++n)
            for (int i = 0; i < HW; ++i) s += x[((size_t)n * C + c) * HW + i];
        const double mu = s / m;
        double v = 0.0;
        for (int n = 0; n < N; ++n)
            for (int i = 0; i < HW; ++i) {
                const double d = x[((size_t)n * C + c) * HW + i] - mu;
                v += d * d;
            }
        const double inv = 1.0 / sqrt(v / m + eps);
        mean[c] = mu;
        invstd[c] = inv;
        for (int n = 0; n < N; ++n)
            for (int i = 0; i < HW; ++i) {
                const size_t o = ((size_t)n * C + c) * HW + i;
                y[o] = gamma[c] * ((x[o] - mu) * inv) + beta[c];
            }
    }
}

/* dbeta += sum dy ; dgamma += sum dy*xhat ;
 * dx = gamma*inv*(dy - sum(dy)/m - xhat*sum(dy*xhat)/m)   (sums of THIS batch only). */
void orc_bn_bwd(const double *x, const double *dy, const double *gamma, const double *mean,
                const double *invstd, double *dx, double *dgamma, double *dbeta,
                int N, int C, int HW)
{
    const double m = (double)N * HW;
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        double s1 = 0.0, s2 = 0.0;
        for (int n = 0; n < N; ++n)
            for (int i = 0; i < HW; ++i) {
                const size_t o = ((size_t)n * C + c) * HW + i;
                s1 += dy[o];
                s2 += dy[o] * ((x[o] - mean[c]) * invstd[c]);
            }
        dbeta[c] += s1;
        dgamma[c] += s2;
        for (int n = 0; n < N; ++n)
            for (int i = 0; i < HW; ++i) {
                const size_t o = ((size_t)n * C + c) * HW + i;
                const double xh = (x[o] - mean[c]) * invstd[c];
                dx[o] = gamma[c] * invstd[c] * (dy[o] - s1 / m - xh * s2 / m);
            }
    }
}

/* y[n,o] = b[o] + sum_i x[n,i]*w[o,i] */
void orc_linear_fwd(const double *x, const double *w, const double *b, double *y,
                    int N, int In, int Out)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int o = 0; o < Out; ++o) {
            double acc = 0.0;
#pragma omp simd reduction(+ : acc)
            for (int i = 0; i < In; ++i) acc += x[(size_t)n * In + i] * w[(size_t)o * In + i];
            y[(size_t)n * Out + o] = acc + (b ? b[o] : 0.0);
        }
}

/* dx[n,i] = sum_o dy[n,o]*w[o,i]  (overwritten) */
void orc_linear_dgrad(const double *dy, const double *w, double *dx, int N, int In, int Out)
{
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        double *d = dx + (size_t)n * In;
        for (int i = 0; i < In; ++i) d[i] = 0.0;
        for (int o = 0; o < Out; ++o) {
            const double g = dy[(size_t)n * Out + o];
            const double *wr = w + (size_t)o * In;
            for (int i = 0; i < In; ++i) d[i] += g * wr[i];
        }
    }
}

/* dw[o,i] += sum_n dy[n,o]*x[n,i] ; db[o] += sum_n dy[n,o]  (accumulate) */
void orc_linear_wgrad(const double *x, const double *dy, double *dw, double *db,
                      int N, int In, int Out)
{
#pragma omp parallel for schedule(static)
    for (int o = 0; o < Out; ++o) {
        double *dr = dw + (size_t)o * In;
        double sb = 0.0;
        for (int n = 0; n < N; ++n) {
            const double g = dy[(size_t)n * Out + o];
            const double *xr = x + (size_t)n * In;
            for (int i = 0; i < In; ++i) dr[i] += g * xr[i];
            sb += g;
        }
        if (db) db[o] += sb;
    }
}

/* p = softmax(z) row-wise, computed after subtracting the row maximum. */
void orc_softmax_fwd(const double *z, double *p, int N, int K)
{
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        const double *zr = z + (size_t)n * K;
        double *pr = p + (size_t)n * K;
        double mx = zr[0];
        for (int k = 1; k < K; ++k) mx = zr[k] > mx ? zr[k] : mx;
        double s = 0.0;
        for (int k = 0; k < K; ++k) { pr[k] = exp(zr[k] - mx); s += pr[k]; }
        for (int k = 0; k < K; ++k) pr[k] /= s;
    }
}

/* loss = -scale * sum_n log p[n,label_n] (returned) ; dz = scale*(p - onehot(label)). */
double orc_xent_bwd(const double *z, const int32_t *label, double scale, double *dz, int N, int K)
{
    double loss = 0.0;
    for (int n = 0; n < N; ++n) {
        const double *zr = z + (size_t)n * K;
        double mx = zr[0];
        for (int k = 1; k < K; ++k) mx = zr[k] > mx ? zr[k] : mx;
        double s = 0.0;
        for (int k = 0; k < K; ++k) s += exp(zr[k] - mx);
        const double lse = mx + log(s);
        loss += -(zr[label[n]] - lse);
        for (int k = 0; k < K; ++k)
            dz[(size_t)n * K + k] = scale * (exp(zr[k] - lse) - (k == label[n] ? 1.0 : 0.0));
    }
    return scale * loss;
}

/* w <- w - lr*g */
void orc_sgd_step(double *w, const double *g, double lr, size_t n)
{
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) w[i] -= lr * g[i];
}
