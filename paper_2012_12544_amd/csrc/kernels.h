// Host-callable launchers of the stage's HIP kernels.  Internal to the library: the public
// interface is include/bapipe_stage.h.  All tensors are NHWC in HBM; `dtype` selects the
// storage type (0 = float, 1 = bf16) of activations, activation gradients and working
// weights; master weights, weight gradients, statistics and losses are always float.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace bapipe {

enum { DT_F32 = 0, DT_BF16 = 1 };
inline size_t dt_size(int dt) { return dt == DT_F32 ? 4 : 2; }

// out[n,oh,ow,ko] = sum_{r,s,ki} in[n,ih,iw,ki] * wt[ko][r][s][ki]  (+ bias[ko]),
// ih = (oh*s_out + r - pad_h) / s_in when divisible and inside [0,Hi), same for iw.
//   forward conv : in = x,  s_out = stride, s_in = 1,      pad = pad,       wt = w [K][R][S][C]
//   dgrad        : in = dy, s_out = 1,      s_in = stride, pad = R-1-pad,   wt = flipped,
//                  channel-transposed copy [C][R][S][K]
struct GatherConv {
    int N, Hi, Wi, Ci, Ho, Wo, Co, R, S, s_out, s_in, pad_h, pad_w;
    // Hint for the tile plan: kernels of other streams run beside this launch.  Alone on the chip a launch wants
    // every compute unit busy; beside others, units it leaves idle are not lost, and fewer, larger blocks (less
    // operand traffic per FLOP) are the better neighbour.  Only the pixel tile may depend on it: every output
    // element is still one sum over K in the same order, so results do not change by a bit.
    int beside = 0;
};

// Forward-convolution geometry (x: N,H,W,C ; y: N,P,Q,K ; filter R x S).
struct ConvShape {
    int N, H, W, C, P, Q, K, R, S, stride, pad;
};

// Epilogue options of kernels that write an activation gradient (see grad_out()).
struct GradEpi {
    const void *gate;  // forward values deciding the producer's fused-ReLU mask, or NULL
    int accum;         // add to what is already stored
    // With accum: the stored value is read from here (same layout as the destination) instead of from the
    // destination itself - the other contribution to a gradient with two sources, taken where it already lies
    // instead of being copied first.  Honoured by the MFMA gather convolution; NULL everywhere else.
    const void *accum_from = nullptr;
};

// ---- direct (CUDA-core style) convolution: fp32 stages and shapes the MFMA path skips
hipError_t conv_gather_direct(int dt, const void *in, const void *wt, const float *bias, void *out,
                              int relu, GradEpi epi, const GatherConv &g, hipStream_t s);
size_t conv_wgrad_direct_workspace(const ConvShape &c);
hipError_t conv_wgrad_direct(int dt, const void *x, const void *dy, float *dw, void *workspace,
                             const ConvShape &c, hipStream_t s);

// ---- bf16 MFMA implicit-GEMM convolution (kernels_conv_mfma.hip)
bool conv_gather_mfma_supported(const GatherConv &g);
size_t conv_gather_mfma_workspace(const GatherConv &g);      // split-K partials (0 if K is not split)
// bn_x / bn_stats (optional, gradient epilogue, with stat_part): the output is the gradient of a batch-norm's
// output; stat_part then receives the per-tile sums of dy and dy*xhat (xhat from bn_x and the saved mean, 1/std)
// stat_part (optional): the kernel also leaves, per pixel tile, the per-channel sum and sum of squares of
// the values it stores - [2][chunks][Co] floats with chunks = conv_gather_mfma_stat_chunks(g) - which is what
// bn_fwd would otherwise compute in a pass of its own; only where that function returns a non-zero count
int conv_gather_mfma_stat_chunks(const GatherConv &g);
hipError_t conv_gather_mfma(const void *in, const void *wt, const float *bias, void *out, int relu,
                            GradEpi epi, const GatherConv &g, void *workspace, hipStream_t s,
                            float *stat_part = nullptr, const void *bn_x = nullptr, const float *bn_stats = nullptr);
// 3x3 / stride 1 / pad 1 with the input halo of a 16x16 output patch resident in LDS
// (kernels_conv_halo.hip); conv_gather_mfma routes to it when it applies
bool conv3x3_halo_supported(const GatherConv &g);
hipError_t conv3x3_halo_mfma(const void *in, const void *wt, const float *bias, void *out, int relu,
                             GradEpi epi, const GatherConv &g, hipStream_t s);
// forward of a 3x3 / stride 1 / pad 1 conv whose input has 8 channels in memory (the padded RGB stage input)
bool conv3x3_c8_supported(const GatherConv &g);
hipError_t conv3x3_c8_mfma(const void *in, const void *wt, const float *bias, void *out, int relu,
                           const GatherConv &g, hipStream_t s);
// same convolution with a 2x2 stride-2 max-pool fused into the epilogue: writes the pooled output
// [N][H/2][W/2][Co] and the arg-max indices (one byte each, same layout); the conv output is not stored
hipError_t conv3x3_halo_pool_mfma(const void *in, const void *wt, const float *bias, int relu, void *pool_out,
                                  uint8_t *pool_idx, const GatherConv &g, hipStream_t s);
// The same implicit GEMM leaving raw fp32 sums: part[split][pixel][co], *splits partial results the
// caller adds up (no bias, no epilogue, no rounding).  Used for the recurrent products of the LSTM.
size_t conv_gather_mfma_raw_workspace(const GatherConv &g);
hipError_t conv_gather_mfma_raw(const void *in, const void *wt, const GatherConv &g, float *part, int *splits,
                                hipStream_t s);
bool wgrad3x3_halo_supported(const ConvShape &c);
size_t wgrad3x3_halo_workspace(const ConvShape &c);
hipError_t wgrad3x3_halo_mfma(const void *x, const void *dy, float *dw, float *db, void *workspace,
                              const ConvShape &c, hipStream_t s);
// weight gradient of a 3x3 / stride 1 / pad 1 conv whose input has 8 channels in memory (the padded RGB stage input)
bool wgrad3x3_c8_supported(const ConvShape &c);
size_t wgrad3x3_c8_workspace(const ConvShape &c);
hipError_t wgrad3x3_c8_mfma(const void *x, const void *dy, float *dw, float *db, void *workspace, const ConvShape &c,
                            hipStream_t s);
bool conv_wgrad_mfma_supported(const ConvShape &c);
size_t conv_wgrad_mfma_workspace(const ConvShape &c);
// dw += dy^T x over all pixels; db (may be null) += column sums of dy
hipError_t conv_wgrad_mfma(const void *x, const void *dy, float *dw, float *db, void *workspace,
                           const ConvShape &c, hipStream_t s);

// ---- column sums over a [rows][C] matrix: out[c] += sum_r a[r][c]  (bias gradient)
size_t colsum_workspace(int rows, int C);
hipError_t colsum_accumulate(int dt, const void *a, int rows, int C, float *out, void *workspace,
                             hipStream_t s);

// ---- element-wise / pooling / normalisation
hipError_t relu_fwd(int dt, const void *x, void *y, size_t n, hipStream_t s);
hipError_t relu_bwd(int dt, const void *y, const void *dy, void *dx, GradEpi epi, size_t n, hipStream_t s);
hipError_t maxpool2x2_fwd(int dt, const void *x, void *y, uint8_t *idx, int N, int H, int W, int C,
                          hipStream_t s);
// gate (if any) is indexed like dy (the pooled tensor), not like dx.
hipError_t maxpool2x2_bwd(int dt, const void *dy, const uint8_t *idx, void *dx, GradEpi epi_pooled_gate,
                          int N, int H, int W, int C, hipStream_t s);
// any window / stride / padding (kh*kw <= 255): idx = dh*kw + dw of the first maximum inside the
// padded window; backward adds the gradients of all windows that chose an input (fixed order)
hipError_t maxpool_fwd(int dt, const void *x, void *y, uint8_t *idx, int N, int H, int W, int C, int kh,
                       int kw, int stride, int pad, hipStream_t s);
hipError_t maxpool_bwd(int dt, const void *dy, const uint8_t *idx, void *dx, GradEpi epi_pooled_gate, int N,
                       int H, int W, int C, int kh, int kw, int stride, int pad, hipStream_t s);
// mean over kh x kw windows at stride (kh, kw), no padding; gate (if any) indexed like dx
hipError_t avgpool_fwd(int dt, const void *x, void *y, int N, int H, int W, int C, int kh, int kw, hipStream_t s);
hipError_t avgpool_bwd(int dt, const void *dy, void *dx, GradEpi epi, int N, int H, int W, int C, int kh, int kw,
                       hipStream_t s);
// dx[n,h,w,:] (+)= t[n,h/stride,w/stride,:] at multiples of the stride, zero elsewhere (t: [N][Ho][Wo][C])
hipError_t upsample_grad(int dt, const void *t, void *dx, GradEpi epi, int N, int H, int W, int Ho, int Wo, int C,
                         int stride, hipStream_t s);
hipError_t add_fwd(int dt, const void *a, const void *b, void *y, int relu, size_t n, hipStream_t s);
// dx (+)= dy with the epilogue of grad_out
hipError_t grad_copy(int dt, const void *dy, void *dx, GradEpi epi, size_t n, hipStream_t s);

// ---- LSTM cell, one time step t over all N sequences (gate order i, f, g, o; H = hidden size)
// P: input projection incl. bias [N][T][4H] (storage type); gh: S partial recurrent sums [S][N][4H]
// (S = 0 at t = 0); writes gates [N][T][4H] and cells [N][T][H] (float), h [N][T][H] and the
// one-step-delayed copy hs (hs[:, t+1] = h[:, t], hs[:, 0] = 0) in the storage type.
hipError_t lstm_cell_fwd(int dt, const void *P, const float *gh, int S, float *gates, float *cells, void *h,
                         void *hs, int N, int T, int H, int t, hipStream_t s);
// dy: gradient of h [N][T][H]; r: S partial sums of W_h^T D_{t+1} [S][N][H] (S = 0 at t = T-1);
// dcn [N][H] carries dc_{t+1}*f_{t+1} between steps; writes D[:, t] (pre-activation gradients,
// [N][T][4H], storage type).
hipError_t lstm_cell_bwd(int dt, const void *dy, const float *r, int S, const float *gates, const float *cells,
                         float *dcn, void *D, int N, int T, int H, int t, hipStream_t s);

size_t bn_workspace(int rows, int C);
// stats: [2][C] floats (mean, invstd)
// pre_chunks > 0: the workspace already holds [2][pre_chunks][C] partial sums of x and x^2 (left there by
// the kernel that produced x) and the first pass over x is skipped
// res: the other input of a residual ADD fed only by this layer - y = [relu_sum](round(bn(x)) + res) in one pass
hipError_t bn_fwd(int dt, const void *x, const float *gamma, const float *beta, float eps, void *y,
                  float *stats, int relu, int rows, int C, void *workspace, hipStream_t s, int pre_chunks = 0,
                  const void *res = nullptr, int relu_sum = 0);
// pre_chunks > 0: the workspace already holds [2][pre_chunks][C] partial sums of dy and dy*xhat
hipError_t bn_bwd(int dt, const void *x, const void *dy, const float *gamma, const float *stats,
                  void *dx, float *dgamma, float *dbeta, GradEpi epi, int rows, int C,
                  void *workspace, hipStream_t s, int pre_chunks = 0);

// p = softmax(z) rows of K classes (float out)
hipError_t softmax_fwd(int dt, const void *z, float *p, int rows, int K, hipStream_t s);
// dz = scale*(p - onehot), loss[0] = -scale*sum_n log p[n,label]
hipError_t xent_bwd(int dt, const float *p, const int32_t *labels, float scale, void *dz, float *loss,
                    int rows, int K, hipStream_t s);

// ---- parameters
// w <- w - lr*g ; g <- 0 ; work <- storage(w)   (work may be NULL for float vectors)
hipError_t sgd_step(int dt, float *w, float *g, float lr, void *work, size_t n, hipStream_t s);
hipError_t recast(int dt, const float *w, void *work, size_t n, hipStream_t s);
// wt[c][R-1-r][S-1-s][k] = work(w[k][r][s][c])   (dgrad filter)
hipError_t make_dgrad_filter(int dt, const float *w, void *wt, int K, int R, int S, int C, hipStream_t s);
hipError_t fill_f32(float *p, float v, size_t n, hipStream_t s);

// ---- boundary layout conversion NCHW <-> NHWC (same storage type); optional ReLU gate.
// The NHWC side has Cp >= C physical channels (zero padded); nhwc_repad changes the channel
// count of an NHWC tensor (zero fill or truncation).
hipError_t nchw_to_nhwc(int dt, const void *src, void *dst, GradEpi epi, int N, int C, int H, int W,
                        int Cp, hipStream_t s);
hipError_t nhwc_to_nchw(int dt, const void *src, void *dst, int N, int C, int H, int W, int Cp,
                        hipStream_t s);
hipError_t nhwc_repad(int dt, const void *src, void *dst, size_t rows, int Cs, int Cd, hipStream_t s);
hipError_t nhwc_to_nchw_u8(const uint8_t *src, uint8_t *dst, int N, int C, int H, int W, hipStream_t s);

}  // namespace bapipe
