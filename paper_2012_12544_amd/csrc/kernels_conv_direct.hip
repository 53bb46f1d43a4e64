// Direct (vector-ALU) convolution kernels: the arithmetic path of fp32 stages, whose 1e-4
// parity bound needs true fp32 products, and of the few bf16 shapes the MFMA kernels do not
// take (channel counts that are not a multiple of 8).  One thread per output element, fp32
// accumulation in the order (r, s, ci).
#include "dev_common.h"
#include "kernels.h"

namespace bapipe {
namespace {

constexpr int TPB = 256;

template <class T>
__global__ void k_conv_gather(const T *__restrict__ in, const T *__restrict__ wt,
                              const float *__restrict__ bias, T *out, const T *__restrict__ gate,
                              int accum, int relu, int is_grad, GatherConv g)
{
    size_t i = (size_t)blockIdx.x * TPB + threadIdx.x;
    size_t total = (size_t)g.N * g.Ho * g.Wo * g.Co;
    if (i >= total) return;
    int ko = (int)(i % g.Co);
    size_t t = i / g.Co;
    int ow = (int)(t % g.Wo);
    t /= g.Wo;
    int oh = (int)(t % g.Ho);
    int n = (int)(t / g.Ho);
    float acc = bias ? bias[ko] : 0.0f;
    for (int r = 0; r < g.R; ++r) {
        int hn = oh * g.s_out + r - g.pad_h;
        if (hn < 0 || hn % g.s_in) continue;
        int ih = hn / g.s_in;
        if (ih >= g.Hi) continue;
        for (int s = 0; s < g.S; ++s) {
            int wn = ow * g.s_out + s - g.pad_w;
            if (wn < 0 || wn % g.s_in) continue;
            int iw = wn / g.s_in;
            if (iw >= g.Wi) continue;
            const T *ip = in + (((size_t)n * g.Hi + ih) * g.Wi + iw) * g.Ci;
            const T *wp = wt + (((size_t)ko * g.R + r) * g.S + s) * g.Ci;
            for (int c = 0; c < g.Ci; ++c) acc = fmaf(to_f32(ip[c]), to_f32(wp[c]), acc);
        }
    }
    if (relu) acc = fmaxf(acc, 0.0f);
    if (is_grad) {
        T old = from_f32<T>(0.0f), gt = old;
        if (accum) old = out[i];
        if (gate) gt = gate[i];
        out[i] = grad_out<T>(acc, accum != 0, old, gate != nullptr, gt);
    } else {
        out[i] = from_f32<T>(acc);
    }
}

// part[chunk][k][r][s][c] = sum over the chunk's output rows (n,p) and all q of
//   dy[n,p,q,k] * x[n, p*stride+r-pad, q*stride+s-pad, c] ;  chunk = blockIdx.y
template <class T>
__global__ void k_conv_wgrad_partial(const T *__restrict__ x, const T *__restrict__ dy,
                                     float *__restrict__ part, ConvShape c, int rows_per_chunk)
{
    size_t i = (size_t)blockIdx.x * TPB + threadIdx.x;
    size_t total = (size_t)c.K * c.R * c.S * c.C;
    if (i >= total) return;
    int ci = (int)(i % c.C);
    size_t t = i / c.C;
    int s = (int)(t % c.S);
    t /= c.S;
    int r = (int)(t % c.R);
    int k = (int)(t / c.R);
    int row0 = blockIdx.y * rows_per_chunk, row1 = row0 + rows_per_chunk;
    if (row1 > c.N * c.P) row1 = c.N * c.P;
    float acc = 0.0f;
    for (int row = row0; row < row1; ++row) {
        int n = row / c.P, p = row % c.P;
        int ih = p * c.stride + r - c.pad;
        if (ih < 0 || ih >= c.H) continue;
        for (int q = 0; q < c.Q; ++q) {
            int iw = q * c.stride + s - c.pad;
            if (iw < 0 || iw >= c.W) continue;
            acc = fmaf(to_f32(dy[(((size_t)n * c.P + p) * c.Q + q) * c.K + k]),
                       to_f32(x[(((size_t)n * c.H + ih) * c.W + iw) * c.C + ci]), acc);
        }
    }
    part[(size_t)blockIdx.y * total + i] = acc;
}

// dw[i] += sum_chunk part[chunk][i], chunks added in index order (bit-reproducible)
__global__ void k_wgrad_reduce(const float *__restrict__ part, float *dw, size_t total, int chunks)
{
    size_t i = (size_t)blockIdx.x * TPB + threadIdx.x;
    if (i >= total) return;
    float acc = 0.0f;
    for (int k = 0; k < chunks; ++k) acc += part[(size_t)k * total + i];
    dw[i] += acc;
}

inline int direct_wgrad_chunks(const ConvShape &c)
{
    size_t total = (size_t)c.K * c.R * c.S * c.C;
    int rows = c.N * c.P;
    size_t cap = ((size_t)16 << 20) / (total ? total : 1);    // <= 64 MiB of partials
    int chunks = rows < 1024 ? rows : 1024;
    if ((size_t)chunks > cap) chunks = (int)cap;
    return chunks < 1 ? 1 : chunks;
}

}  // namespace

hipError_t conv_gather_direct(int dt, const void *in, const void *wt, const float *bias, void *out,
                              int relu, GradEpi epi, const GatherConv &g, hipStream_t s)
{
    size_t total = (size_t)g.N * g.Ho * g.Wo * g.Co;
    if (total == 0) return hipSuccess;
    unsigned nb = (unsigned)((total + TPB - 1) / TPB);
    int is_grad = (epi.gate != nullptr || epi.accum) ? 1 : 0;
    if (dt == DT_F32)
        hipLaunchKernelGGL((k_conv_gather<float>), dim3(nb), dim3(TPB), 0, s, (const float *)in,
                           (const float *)wt, bias, (float *)out, (const float *)epi.gate, epi.accum, relu,
                           is_grad, g);
    else
        hipLaunchKernelGGL((k_conv_gather<bf16_t>), dim3(nb), dim3(TPB), 0, s, (const bf16_t *)in,
                           (const bf16_t *)wt, bias, (bf16_t *)out, (const bf16_t *)epi.gate, epi.accum,
                           relu, is_grad, g);
    return hipGetLastError();
}

size_t conv_wgrad_direct_workspace(const ConvShape &c)
{
    return (size_t)direct_wgrad_chunks(c) * c.K * c.R * c.S * c.C * sizeof(float);
}

hipError_t conv_wgrad_direct(int dt, const void *x, const void *dy, float *dw, void *workspace,
                             const ConvShape &c, hipStream_t s)
{
    size_t total = (size_t)c.K * c.R * c.S * c.C;
    if (total == 0 || c.N * c.P == 0) return hipSuccess;
    unsigned nb = (unsigned)((total + TPB - 1) / TPB);
    int chunks = direct_wgrad_chunks(c);
    int rpc = (c.N * c.P + chunks - 1) / chunks;
    chunks = (c.N * c.P + rpc - 1) / rpc;
    float *part = (float *)workspace;
    if (dt == DT_F32)
        hipLaunchKernelGGL((k_conv_wgrad_partial<float>), dim3(nb, chunks), dim3(TPB), 0, s,
                           (const float *)x, (const float *)dy, part, c, rpc);
    else
        hipLaunchKernelGGL((k_conv_wgrad_partial<bf16_t>), dim3(nb, chunks), dim3(TPB), 0, s,
                           (const bf16_t *)x, (const bf16_t *)dy, part, c, rpc);
    hipLaunchKernelGGL(k_wgrad_reduce, dim3(nb), dim3(TPB), 0, s, part, dw, total, chunks);
    return hipGetLastError();
}

}  // namespace bapipe
