// HBM-bound kernels of a stage: ReLU, 2x2 max-pool, residual add, training-mode batch-norm,
// softmax cross-entropy, SGD update, bias-gradient column sums and boundary layout changes.
// All activations are NHWC, so the channel index is the fastest one: threads own V = 16/sizeof(T)
// consecutive channels (one 16-byte access) and neighbouring threads neighbouring channel
// groups, which keeps every wavefront's HBM access contiguous.
#include "dev_common.h"
#include "kernels.h"

namespace bapipe {
namespace {

constexpr int TPB = 256;

inline unsigned blocks_for(size_t n, int per_block = TPB)
{
    size_t b = (n + per_block - 1) / per_block;
    return (unsigned)(b == 0 ? 1 : b);
}

template <class T> constexpr int vec_width() { return 16 / (int)sizeof(T); }

inline bool aligned16(const void *p) { return (((uintptr_t)p) & 15u) == 0; }

// ------------------------------------------------------------------ flat element-wise
template <class T, int V>
__global__ void k_relu_fwd(const T *__restrict__ x, T *__restrict__ y, size_t nvec)
{
    size_t i = (size_t)blockIdx.x * TPB + threadIdx.x;
    if (i >= nvec) return;
    vec_t<T, V> a = reinterpret_cast<const vec_t<T, V> *>(x)[i], r;
#pragma unroll
    for (int j = 0; j < V; ++j) r.e[j] = from_f32<T>(fmaxf(to_f32(a.e[j]), 0.0f));
    reinterpret_cast<vec_t<T, V> *>(y)[i] = r;
}

template <class T, int V>
__global__ void k_add_fwd(const T *__restrict__ a, const T *__restrict__ b, T *__restrict__ y, int relu,
                          size_t nvec)
{
    size_t i = (size_t)blockIdx.x * TPB + threadIdx.x;
    if (i >= nvec) return;
    vec_t<T, V> va = reinterpret_cast<const vec_t<T, V> *>(a)[i];
    vec_t<T, V> vb = reinterpret_cast<const vec_t<T, V> *>(b)[i], r;
#pragma unroll
    for (int j = 0; j < V; ++j) {
        float v = to_f32(va.e[j]) + to_f32(vb.e[j]);
        if (relu) v = fmaxf(v, 0.0f);
        r.e[j] = from_f32<T>(v);
    }
    reinterpret_cast<vec_t<T, V> *>(y)[i] = r;
}

// dx (+)= dy, gated.  With own_gate the kernel is a stand-alone ReLU backward: the value is
// first zeroed where own_gate <= 0 (own_gate = that ReLU's output).
template <class T, int V>
__global__ void k_grad_copy(const T *__restrict__ dy, const T *__restrict__ own_gate, T *dx,
                            const T *__restrict__ gate, int accum, size_t nvec)
{
    size_t i = (size_t)blockIdx.x * TPB + threadIdx.x;
    if (i >= nvec) return;
    vec_t<T, V> g = reinterpret_cast<const vec_t<T, V> *>(dy)[i];
    vec_t<T, V> og, old, gt, r;
    if (own_gate) og = reinterpret_cast<const vec_t<T, V> *>(own_gate)[i];
    if (accum) old = reinterpret_cast<const vec_t<T, V> *>(dx)[i];
    if (gate) gt = reinterpret_cast<const vec_t<T, V> *>(gate)[i];
#pragma unroll
    for (int j = 0; j < V; ++j) {
        float v = to_f32(g.e[j]);
        if (own_gate && !(to_f32(og.e[j]) > 0.0f)) v = 0.0f;
        r.e[j] = grad_out<T>(v, accum != 0, old.e[j], gate != nullptr, gt.e[j]);
    }
    reinterpret_cast<vec_t<T, V> *>(dx)[i] = r;
}

// dx[n,h,w,:] (+)= t[n,h/s,w/s,:] where h and w are multiples of s (and inside t), zero elsewhere: the input
// gradient of a 1x1 convolution with stride s, whose product with the filter was taken at the strided
// resolution.  Same epilogue as every gradient write.
template <class T, int V>
__global__ void k_upsample_grad(const T *__restrict__ t, T *dx, const T *__restrict__ gate, int accum, int N,
                                int H, int W, int Ho, int Wo, int CV, int stride)
{
    size_t i = (size_t)blockIdx.x * TPB + threadIdx.x;
    if (i >= (size_t)N * H * W * CV) return;
    const int cv = (int)(i % CV);
    size_t r = i / CV;
    const int w = (int)(r % W);
    r /= W;
    const int h = (int)(r % H), n = (int)(r / H);
    const int p = h / stride, q = w / stride;
    const bool hit = p * stride == h && q * stride == w && p < Ho && q < Wo;
    vec_t<T, V> g, old, gt, o;
    if (hit) g = reinterpret_cast<const vec_t<T, V> *>(t)[(((size_t)n * Ho + p) * Wo + q) * CV + cv];
    if (accum) old = reinterpret_cast<const vec_t<T, V> *>(dx)[i];
    if (gate) gt = reinterpret_cast<const vec_t<T, V> *>(gate)[i];
#pragma unroll
    for (int j = 0; j < V; ++j)
        o.e[j] = grad_out<T>(hit ? to_f32(g.e[j]) : 0.0f, accum != 0, old.e[j], gate != nullptr, gt.e[j]);
    reinterpret_cast<vec_t<T, V> *>(dx)[i] = o;
}

// ------------------------------------------------------------------ 2x2 stride-2 max-pool
template <class T, int V>
__global__ void k_pool_fwd(const T *__restrict__ x, T *__restrict__ y, uint8_t *__restrict__ idx, int N,
                           int H, int W, int CV)
{
    const int Ho = H / 2, Wo = W / 2;
    size_t i = (size_t)blockIdx.x * TPB + threadIdx.x;
    size_t total = (size_t)N * Ho * Wo * CV;
    if (i >= total) return;
    int cv = (int)(i % CV);
    size_t t = i / CV;
    int q = (int)(t % Wo);
    t /= Wo;
    int p = (int)(t % Ho);
    int n = (int)(t / Ho);
    const vec_t<T, V> *xv = reinterpret_cast<const vec_t<T, V> *>(x);
    size_t base = (((size_t)n * H + 2 * p) * W + 2 * q) * CV + cv;
    vec_t<T, V> a[4];
    a[0] = xv[base];
    a[1] = xv[base + CV];
    a[2] = xv[base + (size_t)W * CV];
    a[3] = xv[base + (size_t)W * CV + CV];
    vec_t<T, V> r;
    vec_t<uint8_t, V> ri;
#pragma unroll
    for (int j = 0; j < V; ++j) {
        float best = to_f32(a[0].e[j]);
        int bi = 0;
#pragma unroll
        for (int k = 1; k < 4; ++k) {
            float v = to_f32(a[k].e[j]);
            if (v > best) {                       // strictly greater: the first maximum wins
                best = v;
                bi = k;
            }
        }
        r.e[j] = from_f32<T>(best);
        ri.e[j] = (uint8_t)bi;
    }
    reinterpret_cast<vec_t<T, V> *>(y)[i] = r;
    reinterpret_cast<vec_t<uint8_t, V> *>(idx)[i] = ri;
}

template <class T, int V>
__global__ void k_pool_bwd(const T *__restrict__ dy, const uint8_t *__restrict__ idx, T *dx,
                           const T *__restrict__ gate, int accum, int N, int H, int W, int CV)
{
    const int Ho = H / 2, Wo = W / 2;
    size_t i = (size_t)blockIdx.x * TPB + threadIdx.x;
    size_t total = (size_t)N * Ho * Wo * CV;
    if (i >= total) return;
    int cv = (int)(i % CV);
    size_t t = i / CV;
    int q = (int)(t % Wo);
    t /= Wo;
    int p = (int)(t % Ho);
    int n = (int)(t / Ho);
    vec_t<T, V> g = reinterpret_cast<const vec_t<T, V> *>(dy)[i];
    vec_t<uint8_t, V> ix = reinterpret_cast<const vec_t<uint8_t, V> *>(idx)[i];
    vec_t<T, V> gt;
    if (gate) gt = reinterpret_cast<const vec_t<T, V> *>(gate)[i];
    vec_t<T, V> *dxv = reinterpret_cast<vec_t<T, V> *>(dx);
    size_t base = (((size_t)n * H + 2 * p) * W + 2 * q) * CV + cv;
    const size_t off[4] = {0, (size_t)CV, (size_t)W * CV, (size_t)W * CV + CV};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        vec_t<T, V> old, r;
        if (accum) old = dxv[base + off[k]];
#pragma unroll
        for (int j = 0; j < V; ++j) {
            float v = (ix.e[j] == k) ? to_f32(g.e[j]) : 0.0f;
            r.e[j] = grad_out<T>(v, accum != 0, old.e[j], gate != nullptr, gt.e[j]);
        }
        dxv[base + off[k]] = r;
    }
}

// ------------------------------------------------------------------ windowed pooling (any window / stride / pad)
struct PoolWin {
    int N, H, W, CV, Ho, Wo, kh, kw, stride, pad;
};

// Max over the in-image part of each window, first maximum in row-major window order; the index
// stored is dh*kw + dw of the winner inside the (padded) window.
template <class T, int V>
__global__ void k_poolw_fwd(const T *__restrict__ x, T *__restrict__ y, uint8_t *__restrict__ idx, PoolWin g)
{
    size_t i = (size_t)blockIdx.x * TPB + threadIdx.x;
    size_t total = (size_t)g.N * g.Ho * g.Wo * g.CV;
    if (i >= total) return;
    int cv = (int)(i % g.CV);
    size_t t = i / g.CV;
    int q = (int)(t % g.Wo);
    t /= g.Wo;
    int p = (int)(t % g.Ho);
    int n = (int)(t / g.Ho);
    const vec_t<T, V> *xv = reinterpret_cast<const vec_t<T, V> *>(x);
    float best[V];
    int bi[V];
#pragma unroll
    for (int j = 0; j < V; ++j) { best[j] = 0.0f; bi[j] = -1; }
    for (int dh = 0; dh < g.kh; ++dh) {
        const int ih = p * g.stride + dh - g.pad;
        if (ih < 0 || ih >= g.H) continue;
        for (int dw = 0; dw < g.kw; ++dw) {
            const int iw = q * g.stride + dw - g.pad;
            if (iw < 0 || iw >= g.W) continue;
            vec_t<T, V> a = xv[(((size_t)n * g.H + ih) * g.W + iw) * g.CV + cv];
#pragma unroll
            for (int j = 0; j < V; ++j) {
                float v = to_f32(a.e[j]);
                if (bi[j] < 0 || v > best[j]) { best[j] = v; bi[j] = dh * g.kw + dw; }
            }
        }
    }
    vec_t<T, V> r;
    vec_t<uint8_t, V> ri;
#pragma unroll
    for (int j = 0; j < V; ++j) {
        r.e[j] = from_f32<T>(best[j]);
        ri.e[j] = (uint8_t)(bi[j] < 0 ? 0 : bi[j]);
    }
    reinterpret_cast<vec_t<T, V> *>(y)[i] = r;
    reinterpret_cast<vec_t<uint8_t, V> *>(idx)[i] = ri;
}

// One thread per INPUT position: it visits the windows that contain the position (in (p,q)
// order, so the sum is reproducible) and adds the gradient of those whose arg-max it is.
// `gate`, indexed like dy, holds the pooled forward values: a window whose maximum is not
// positive passes nothing (its winner was zeroed by the producer's ReLU).
template <class T, int V>
__global__ void k_poolw_bwd(const T *__restrict__ dy, const uint8_t *__restrict__ idx, T *dx,
                            const T *__restrict__ gate, int accum, PoolWin g)
{
    size_t i = (size_t)blockIdx.x * TPB + threadIdx.x;
    size_t total = (size_t)g.N * g.H * g.W * g.CV;
    if (i >= total) return;
    int cv = (int)(i % g.CV);
    size_t t = i / g.CV;
    int w = (int)(t % g.W);
    t /= g.W;
    int h = (int)(t % g.H);
    int n = (int)(t / g.H);
    const int hp = h + g.pad, wp = w + g.pad;
    int p0 = hp - g.kh + 1, q0 = wp - g.kw + 1;
    p0 = p0 <= 0 ? 0 : (p0 + g.stride - 1) / g.stride;
    q0 = q0 <= 0 ? 0 : (q0 + g.stride - 1) / g.stride;
    int p1 = hp / g.stride, q1 = wp / g.stride;
    p1 = p1 < g.Ho - 1 ? p1 : g.Ho - 1;
    q1 = q1 < g.Wo - 1 ? q1 : g.Wo - 1;
    float acc[V];
#pragma unroll
    for (int j = 0; j < V; ++j) acc[j] = 0.0f;
    for (int p = p0; p <= p1; ++p)
        for (int q = q0; q <= q1; ++q) {
            const size_t o = (((size_t)n * g.Ho + p) * g.Wo + q) * g.CV + cv;
            const int want = (hp - p * g.stride) * g.kw + (wp - q * g.stride);
            vec_t<uint8_t, V> ix = reinterpret_cast<const vec_t<uint8_t, V> *>(idx)[o];
            vec_t<T, V> gv = reinterpret_cast<const vec_t<T, V> *>(dy)[o], gt;
            if (gate) gt = reinterpret_cast<const vec_t<T, V> *>(gate)[o];
#pragma unroll
            for (int j = 0; j < V; ++j) {
                bool take = ix.e[j] == want;
                if (gate) take = take && to_f32(gt.e[j]) > 0.0f;
                acc[j] += take ? to_f32(gv.e[j]) : 0.0f;
            }
        }
    vec_t<T, V> *dxv = reinterpret_cast<vec_t<T, V> *>(dx);
    vec_t<T, V> old, r;
    if (accum) old = dxv[i];
#pragma unroll
    for (int j = 0; j < V; ++j) r.e[j] = grad_out<T>(acc[j], accum != 0, old.e[j], false, old.e[j]);
    dxv[i] = r;
}

// Mean over kh x kw windows at stride (kh, kw), no padding.
template <class T, int V>
__global__ void k_avgpool_fwd(const T *__restrict__ x, T *__restrict__ y, PoolWin g)
{
    size_t i = (size_t)blockIdx.x * TPB + threadIdx.x;
    size_t total = (size_t)g.N * g.Ho * g.Wo * g.CV;
    if (i >= total) return;
    int cv = (int)(i % g.CV);
    size_t t = i / g.CV;
    int q = (int)(t % g.Wo);
    t /= g.Wo;
    int p = (int)(t % g.Ho);
    int n = (int)(t / g.Ho);
    const vec_t<T, V> *xv = reinterpret_cast<const vec_t<T, V> *>(x);
    float acc[V];
#pragma unroll
    for (int j = 0; j < V; ++j) acc[j] = 0.0f;
    for (int dh = 0; dh < g.kh; ++dh)
        for (int dw = 0; dw < g.kw; ++dw) {
            vec_t<T, V> a = xv[(((size_t)n * g.H + p * g.kh + dh) * g.W + q * g.kw + dw) * g.CV + cv];
#pragma unroll
            for (int j = 0; j < V; ++j) acc[j] += to_f32(a.e[j]);
        }
    const float cnt = (float)(g.kh * g.kw);
    vec_t<T, V> r;
#pragma unroll
    for (int j = 0; j < V; ++j) r.e[j] = from_f32<T>(acc[j] / cnt);
    reinterpret_cast<vec_t<T, V> *>(y)[i] = r;
}

// dx = dy / (kh*kw) for every input of a window, zero outside all windows; gate indexed like dx.
template <class T, int V>
__global__ void k_avgpool_bwd(const T *__restrict__ dy, T *dx, const T *__restrict__ gate, int accum, PoolWin g)
{
    size_t i = (size_t)blockIdx.x * TPB + threadIdx.x;
    size_t total = (size_t)g.N * g.H * g.W * g.CV;
    if (i >= total) return;
    int cv = (int)(i % g.CV);
    size_t t = i / g.CV;
    int w = (int)(t % g.W);
    t /= g.W;
    int h = (int)(t % g.H);
    int n = (int)(t / g.H);
    const int p = h / g.kh, q = w / g.kw;
    const bool inside = p < g.Ho && q < g.Wo;
    vec_t<T, V> gv, gt, old, r;
    if (inside) gv = reinterpret_cast<const vec_t<T, V> *>(dy)[(((size_t)n * g.Ho + p) * g.Wo + q) * g.CV + cv];
    if (gate) gt = reinterpret_cast<const vec_t<T, V> *>(gate)[i];
    vec_t<T, V> *dxv = reinterpret_cast<vec_t<T, V> *>(dx);
    if (accum) old = dxv[i];
    const float cnt = (float)(g.kh * g.kw);
#pragma unroll
    for (int j = 0; j < V; ++j) {
        float v = inside ? to_f32(gv.e[j]) / cnt : 0.0f;
        r.e[j] = grad_out<T>(v, accum != 0, old.e[j], gate != nullptr, gt.e[j]);
    }
    dxv[i] = r;
}

// ------------------------------------------------------------------ column reductions
// A [rows][C] matrix is cut into `chunks` row ranges; block (bx, chunk) owns up to TPB channel
// groups... each block reduces its rows for CGB channel groups with RY row lanes, the lanes are
// combined through LDS, and one partial per (chunk, channel, quantity) goes to the workspace.
// A second tiny kernel adds the partials in double.  Fixed partition => bit-reproducible.
struct ColPlan {
    int CV, CGB, RY, chunks, rows_per_chunk, gx;
};

inline ColPlan col_plan(int rows, int C, int V)
{
    ColPlan p;
    p.CV = C / V;
    p.CGB = p.CV < TPB ? p.CV : TPB;
    p.RY = TPB / p.CGB;
    p.gx = (p.CV + p.CGB - 1) / p.CGB;
    int want = (rows + p.RY * 16 - 1) / (p.RY * 16);      // 16 rows per thread: fewer, longer partial blocks measured faster than 8 or 4
    int cap = 1024 / p.gx;
    if (cap < 1) cap = 1;
    p.chunks = want < 1 ? 1 : (want > cap ? cap : want);
    p.rows_per_chunk = (rows + p.chunks - 1) / p.chunks;
    p.chunks = (rows + p.rows_per_chunk - 1) / p.rows_per_chunk;
    if (p.chunks < 1) p.chunks = 1;
    return p;
}

inline int col_vec(int dt, int C, const void *a, const void *b = nullptr, const void *c = nullptr)
{
    int V = dt == DT_F32 ? 4 : 8;
    bool ok = (C % V == 0) && aligned16(a) && aligned16(b) && aligned16(c);
    return ok ? V : 1;
}

// NQ quantities per element computed by functor F(row, channel-vector index, out[NQ][V])
template <class T, int V, int NQ, class F>
__device__ __forceinline__ void col_partial_body(F f, int rows, ColPlan p, float *__restrict__ part, int C)
{
    __shared__ float red[NQ * V * TPB];
    const int cx = threadIdx.x % p.CGB, ry = threadIdx.x / p.CGB;
    const int cg = blockIdx.x * p.CGB + cx;
    const int chunk = blockIdx.y;
    float acc[NQ][V];
#pragma unroll
    for (int qn = 0; qn < NQ; ++qn)
#pragma unroll
        for (int j = 0; j < V; ++j) acc[qn][j] = 0.0f;
    const bool active = ry < p.RY && cg < p.CV;
    if (active) {
        int r0 = chunk * p.rows_per_chunk, r1 = r0 + p.rows_per_chunk;
        if (r1 > rows) r1 = rows;
        // four rows per trip, all loads first (row index clamped, contribution masked): the trip costs one
        // memory round trip instead of four
        for (int r = r0 + ry; r < r1; r += 4 * p.RY) {
            float v[4][NQ][V];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int rr = r + u * p.RY;
                f(rr < r1 ? rr : r1 - 1, cg, v[u]);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float keep = r + u * p.RY < r1 ? 1.0f : 0.0f;
#pragma unroll
                for (int qn = 0; qn < NQ; ++qn)
#pragma unroll
                    for (int j = 0; j < V; ++j) acc[qn][j] += keep * v[u][qn][j];
            }
        }
    }
#pragma unroll
    for (int qn = 0; qn < NQ; ++qn)
#pragma unroll
        for (int j = 0; j < V; ++j) red[(qn * V + j) * TPB + threadIdx.x] = acc[qn][j];
    __syncthreads();
    if (active && ry == 0) {
#pragma unroll
        for (int qn = 0; qn < NQ; ++qn)
#pragma unroll
            for (int j = 0; j < V; ++j) {
                float s = 0.0f;
                for (int k = 0; k < p.RY; ++k) s += red[(qn * V + j) * TPB + k * p.CGB + cx];
                part[((size_t)qn * p.chunks + chunk) * C + cg * V + j] = s;
            }
    }
}

template <class T, int V>
__global__ void k_colsum_partial(const T *__restrict__ a, int rows, int C, ColPlan p, float *part)
{
    const vec_t<T, V> *av = reinterpret_cast<const vec_t<T, V> *>(a);
    auto f = [&](int r, int cg, float(&v)[1][V]) {
        vec_t<T, V> x = av[(size_t)r * p.CV + cg];
#pragma unroll
        for (int j = 0; j < V; ++j) v[0][j] = to_f32(x.e[j]);
    };
    col_partial_body<T, V, 1>(f, rows, p, part, C);
}

// Final pass over the per-chunk partials: a block owns 4 channels, 64 lanes per channel walk
// the chunks with stride 64, and the lanes are combined through LDS in lane order, so the
// result does not depend on scheduling.  Returns true in the lane that holds the totals.
constexpr int FIN_CH = 4, FIN_LANES = TPB / FIN_CH;
template <int NQ>
__device__ __forceinline__ bool col_final_sums(const float *__restrict__ part, int chunks, int C, int &c,
                                               double (&tot)[NQ])
{
    __shared__ double red[NQ][FIN_LANES][FIN_CH];
    const int cc = threadIdx.x % FIN_CH, cl = threadIdx.x / FIN_CH;
    c = blockIdx.x * FIN_CH + cc;
    double s[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) s[q] = 0.0;
    if (c < C)
        for (int k = cl; k < chunks; k += 4 * FIN_LANES) {      // four independent loads per quantity and trip
            float v[4][NQ];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int kk = k + u * FIN_LANES;
#pragma unroll
                for (int q = 0; q < NQ; ++q) v[u][q] = kk < chunks ? part[((size_t)q * chunks + kk) * C + c] : 0.0f;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int q = 0; q < NQ; ++q) s[q] += (double)v[u][q];
        }
#pragma unroll
    for (int q = 0; q < NQ; ++q) red[q][cl][cc] = s[q];
    __syncthreads();
    if (cl != 0 || c >= C) return false;
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        double t = 0.0;
        for (int k = 0; k < FIN_LANES; ++k) t += red[q][k][cc];
        tot[q] = t;
    }
    return true;
}

inline unsigned final_blocks(int C) { return (unsigned)((C + FIN_CH - 1) / FIN_CH); }

__global__ void k_colsum_final(const float *__restrict__ part, int chunks, int C, float *out)
{
    int c;
    double t[1];
    if (col_final_sums<1>(part, chunks, C, c, t)) out[c] += (float)t[0];
}

// ------------------------------------------------------------------ batch-norm
template <class T, int V>
__global__ void k_bn_stat_partial(const T *__restrict__ x, int rows, int C, ColPlan p, float *part)
{
    const vec_t<T, V> *xv = reinterpret_cast<const vec_t<T, V> *>(x);
    auto f = [&](int r, int cg, float(&v)[2][V]) {
        vec_t<T, V> a = xv[(size_t)r * p.CV + cg];
#pragma unroll
        for (int j = 0; j < V; ++j) {
            float t = to_f32(a.e[j]);
            v[0][j] = t;
            v[1][j] = t * t;
        }
    };
    col_partial_body<T, V, 2>(f, rows, p, part, C);
}

__global__ void k_bn_stat_final(const float *__restrict__ part, int chunks, int C, int rows, float eps,
                                float *stats)
{
    int c;
    double t[2];
    if (!col_final_sums<2>(part, chunks, C, c, t)) return;
    double m = (double)rows, mu = t[0] / m, var = t[1] / m - mu * mu;
    if (var < 0.0) var = 0.0;
    stats[c] = (float)mu;
    stats[C + c] = (float)(1.0 / sqrt(var + (double)eps));
}

// Normalisation pass.  A thread keeps ONE channel group for its whole life (its V means, inverse
// deviations, gammas and betas sit in registers) and walks down the rows, so that per 16 bytes
// of activations there is one 16-byte load and one 16-byte store and nothing else.  Two rows per
// thread: these launches last a few microseconds, and many short blocks ramp up and drain faster
// than fewer long ones (8 rows per thread cost the ResNet stage 4 %).
constexpr int BN_ROWS_PER_THREAD = 2;

template <class T, int V>
__global__ void k_bn_apply(const T *__restrict__ x, const float *__restrict__ gamma,
                           const float *__restrict__ beta, const float *__restrict__ stats,
                           T *__restrict__ y, int relu, int rows, int C, ColPlan p,
                           const T *__restrict__ res, int relu_sum)
{
    // res: the other input of a residual ADD that only this layer's output feeds - y = [relu](q(bn(x)) + res),
    // the normalised value rounded to storage first, as the stand-alone ADD would have read it
    const int cx = threadIdx.x % p.CGB, ry = threadIdx.x / p.CGB;
    const int cg = blockIdx.x * p.CGB + cx;
    if (ry >= p.RY || cg >= p.CV) return;
    float mu[V], inv[V], ga[V], be[V];
#pragma unroll
    for (int j = 0; j < V; ++j) {
        mu[j] = stats[cg * V + j];
        inv[j] = stats[C + cg * V + j];
        ga[j] = gamma[cg * V + j];
        be[j] = beta[cg * V + j];
    }
    const vec_t<T, V> *xv = reinterpret_cast<const vec_t<T, V> *>(x);
    vec_t<T, V> *yv = reinterpret_cast<vec_t<T, V> *>(y);
    const int r0 = blockIdx.y * (p.RY * BN_ROWS_PER_THREAD);
    int r1 = r0 + p.RY * BN_ROWS_PER_THREAD;
    if (r1 > rows) r1 = rows;
    vec_t<T, V> a[BN_ROWS_PER_THREAD], b[BN_ROWS_PER_THREAD];
#pragma unroll
    for (int u = 0; u < BN_ROWS_PER_THREAD; ++u) {            // all loads of the thread first
        const int r = r0 + ry + u * p.RY;
        a[u] = xv[(size_t)(r < r1 ? r : r1 - 1) * p.CV + cg];
        if (res) b[u] = reinterpret_cast<const vec_t<T, V> *>(res)[(size_t)(r < r1 ? r : r1 - 1) * p.CV + cg];
    }
#pragma unroll
    for (int u = 0; u < BN_ROWS_PER_THREAD; ++u) {
        const int r = r0 + ry + u * p.RY;
        if (r >= r1) break;
        vec_t<T, V> o;
#pragma unroll
        for (int j = 0; j < V; ++j) {
            float xh = (to_f32(a[u].e[j]) - mu[j]) * inv[j];
            float v = ga[j] * xh + be[j];
            if (relu) v = fmaxf(v, 0.0f);
            if (res) {
                v = round_to<T>(v) + to_f32(b[u].e[j]);
                if (relu_sum) v = fmaxf(v, 0.0f);
            }
            o.e[j] = from_f32<T>(v);
        }
        yv[(size_t)r * p.CV + cg] = o;
    }
}

template <class T, int V>
__global__ void k_bn_bwd_partial(const T *__restrict__ x, const T *__restrict__ dy,
                                 const float *__restrict__ stats, int rows, int C, ColPlan p, float *part)
{
    const vec_t<T, V> *xv = reinterpret_cast<const vec_t<T, V> *>(x);
    const vec_t<T, V> *gv = reinterpret_cast<const vec_t<T, V> *>(dy);
    int cg0 = blockIdx.x * p.CGB + threadIdx.x % p.CGB;
    if (cg0 >= p.CV) cg0 = p.CV - 1;
    float mu[V], inv[V];
#pragma unroll
    for (int j = 0; j < V; ++j) {
        mu[j] = stats[cg0 * V + j];
        inv[j] = stats[C + cg0 * V + j];
    }
    auto f = [&](int r, int cg, float(&v)[2][V]) {
        vec_t<T, V> a = xv[(size_t)r * p.CV + cg];
        vec_t<T, V> g = gv[(size_t)r * p.CV + cg];
#pragma unroll
        for (int j = 0; j < V; ++j) {
            float gg = to_f32(g.e[j]);
            float xh = (to_f32(a.e[j]) - mu[j]) * inv[j];
            v[0][j] = gg;
            v[1][j] = gg * xh;
        }
    };
    col_partial_body<T, V, 2>(f, rows, p, part, C);
}

// sums[c] = (sum dy, sum dy*xhat) of this micro-batch; dbeta/dgamma accumulate over micro-batches
__global__ void k_bn_bwd_final(const float *__restrict__ part, int chunks, int C, float *sums,
                               float *dgamma, float *dbeta)
{
    int c;
    double t[2];
    if (!col_final_sums<2>(part, chunks, C, c, t)) return;
    sums[c] = (float)t[0];
    sums[C + c] = (float)t[1];
    dbeta[c] += (float)t[0];
    dgamma[c] += (float)t[1];
}

template <class T, int V>
__global__ void k_bn_bwd_apply(const T *__restrict__ x, const T *__restrict__ dy,
                               const float *__restrict__ gamma, const float *__restrict__ stats,
                               const float *__restrict__ sums, T *dx, const T *__restrict__ gate,
                               int accum, float inv_m, int rows, int C, ColPlan p)
{
    const int cx = threadIdx.x % p.CGB, ry = threadIdx.x / p.CGB;
    const int cg = blockIdx.x * p.CGB + cx;
    if (ry >= p.RY || cg >= p.CV) return;
    float mu[V], inv[V], gi[V], m1[V], m2[V];          // mean, 1/std, gamma/std, sum(dy)/m, sum(dy*xhat)/m
#pragma unroll
    for (int j = 0; j < V; ++j) {
        mu[j] = stats[cg * V + j];
        inv[j] = stats[C + cg * V + j];
        gi[j] = gamma[cg * V + j] * inv[j];
        m1[j] = sums[cg * V + j] * inv_m;
        m2[j] = sums[C + cg * V + j] * inv_m;
    }
    const vec_t<T, V> *xv = reinterpret_cast<const vec_t<T, V> *>(x);
    const vec_t<T, V> *gv = reinterpret_cast<const vec_t<T, V> *>(dy);
    const vec_t<T, V> *tv = reinterpret_cast<const vec_t<T, V> *>(gate);
    vec_t<T, V> *dv = reinterpret_cast<vec_t<T, V> *>(dx);
    const int r0 = blockIdx.y * (p.RY * BN_ROWS_PER_THREAD);
    int r1 = r0 + p.RY * BN_ROWS_PER_THREAD;
    if (r1 > rows) r1 = rows;
    constexpr int HALF = BN_ROWS_PER_THREAD / 2;
#pragma unroll
    for (int h = 0; h < 2; ++h) {                               // four rows at a time: loads first, then stores
        vec_t<T, V> a[HALF], g[HALF], old[HALF], gt[HALF];
#pragma unroll
        for (int u = 0; u < HALF; ++u) {
            const int r = r0 + ry + (h * HALF + u) * p.RY;
            const size_t i = (size_t)(r < r1 ? r : r1 - 1) * p.CV + cg;
            a[u] = xv[i];
            g[u] = gv[i];
            if (accum) old[u] = dv[i];
            if (gate) gt[u] = tv[i];
        }
#pragma unroll
        for (int u = 0; u < HALF; ++u) {
            const int r = r0 + ry + (h * HALF + u) * p.RY;
            if (r >= r1) break;
            vec_t<T, V> o;
#pragma unroll
            for (int j = 0; j < V; ++j) {
                float xh = (to_f32(a[u].e[j]) - mu[j]) * inv[j];
                float v = gi[j] * (to_f32(g[u].e[j]) - m1[j] - xh * m2[j]);
                o.e[j] = grad_out<T>(v, accum != 0, old[u].e[j], gate != nullptr, gt[u].e[j]);
            }
            dv[(size_t)r * p.CV + cg] = o;
        }
    }
}

// ------------------------------------------------------------------ batch-norm in one launch
// For tensors of up to 2048 rows one block owns ONE group of V = 4 channels over ALL rows: every thread keeps its R rows in registers, the block
// reduces the statistics (wave butterflies, then the 16 wave results added in double in wave
// order: fixed order, bit-reproducible), and the same registers are normalised and stored.  The
// activations are read once, nothing goes through a workspace and there is no second launch.
// Neighbouring blocks read neighbouring pieces of the same cache lines: poor use of the load
// path, acceptable only because tensors this small are bound by launch latency.
constexpr int OP_NT = 1024, OP_WAVES = OP_NT / 64;

// Makes the compiler forget what it knows about a register-resident vector (so that values derived
// from it before a reduction are recomputed after it instead of being kept alive in registers).
template <class T, int V>
__device__ __forceinline__ void forget(vec_t<T, V> &a)
{
    static_assert(sizeof(a) % 4 == 0, "whole dwords");
    uint32_t *w = reinterpret_cast<uint32_t *>(&a);
#pragma unroll
    for (int i = 0; i < (int)sizeof(a) / 4; ++i) asm volatile("" : "+v"(w[i]));
}

template <int NQV>
__device__ __forceinline__ void block_sums(float (&v)[NQV], float (*wpart)[NQV], double *tot)
{
#pragma unroll
    for (int q = 0; q < NQV; ++q) v[q] = wave_sum(v[q]);
    if ((threadIdx.x & 63) == 0) {
#pragma unroll
        for (int q = 0; q < NQV; ++q) wpart[threadIdx.x >> 6][q] = v[q];
    }
    __syncthreads();
    if (threadIdx.x < NQV) {
        double t = 0.0;
        for (int w = 0; w < OP_WAVES; ++w) t += (double)wpart[w][threadIdx.x];
        tot[threadIdx.x] = t;
    }
    __syncthreads();
}

template <class T, int V, int R>
__global__ __launch_bounds__(OP_NT) void k_bn_fwd_onepass(const T *__restrict__ x, const float *__restrict__ gamma,
                                                          const float *__restrict__ beta, float eps,
                                                          T *__restrict__ y, float *__restrict__ stats, int relu,
                                                          int rows, int C, const T *__restrict__ res, int relu_sum)
{
    __shared__ float wpart[OP_WAVES][2 * V];
    __shared__ double tot[2 * V];
    __shared__ float mi[2 * V];
    const int CV = C / V, cg = blockIdx.x;
    const vec_t<T, V> *xv = reinterpret_cast<const vec_t<T, V> *>(x);
    vec_t<T, V> *yv = reinterpret_cast<vec_t<T, V> *>(y);
    vec_t<T, V> a[R];
#pragma unroll
    for (int u = 0; u < R; ++u) {
        const int r = threadIdx.x + u * OP_NT;
        a[u] = xv[(size_t)(r < rows ? r : rows - 1) * CV + cg];
    }
    float acc[2 * V];
#pragma unroll
    for (int j = 0; j < 2 * V; ++j) acc[j] = 0.0f;
#pragma unroll
    for (int u = 0; u < R; ++u) {
        const bool in = threadIdx.x + u * OP_NT < rows;
#pragma unroll
        for (int j = 0; j < V; ++j) {
            const float t = in ? to_f32(a[u].e[j]) : 0.0f;
            acc[j] += t;
            acc[V + j] += t * t;
        }
    }
    block_sums<2 * V>(acc, wpart, tot);
    if (threadIdx.x < V) {
        const double m = (double)rows, mu = tot[threadIdx.x] / m;
        double var = tot[V + threadIdx.x] / m - mu * mu;
        if (var < 0.0) var = 0.0;
        const float fm = (float)mu, fi = (float)(1.0 / sqrt(var + (double)eps));
        mi[threadIdx.x] = fm;
        mi[V + threadIdx.x] = fi;
        stats[cg * V + threadIdx.x] = fm;
        stats[C + cg * V + threadIdx.x] = fi;
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < R; ++u) forget(a[u]);
    float mu[V], inv[V], ga[V], be[V];
#pragma unroll
    for (int j = 0; j < V; ++j) {
        mu[j] = mi[j];
        inv[j] = mi[V + j];
        ga[j] = gamma[cg * V + j];
        be[j] = beta[cg * V + j];
    }
#pragma unroll
    for (int u = 0; u < R; ++u) {
        const int r = threadIdx.x + u * OP_NT;
        if (r >= rows) break;
        vec_t<T, V> o, b;
        if (res) b = reinterpret_cast<const vec_t<T, V> *>(res)[(size_t)r * CV + cg];
#pragma unroll
        for (int j = 0; j < V; ++j) {
            float xh = (to_f32(a[u].e[j]) - mu[j]) * inv[j];
            float v = ga[j] * xh + be[j];
            if (relu) v = fmaxf(v, 0.0f);
            if (res) {                                   // residual ADD behind this layer, see k_bn_apply
                v = round_to<T>(v) + to_f32(b.e[j]);
                if (relu_sum) v = fmaxf(v, 0.0f);
            }
            o.e[j] = from_f32<T>(v);
        }
        yv[(size_t)r * CV + cg] = o;
    }
}

template <class T, int V, int R>
__global__ __launch_bounds__(OP_NT) void k_bn_bwd_onepass(const T *__restrict__ x, const T *__restrict__ dy,
                                                          const float *__restrict__ gamma,
                                                          const float *__restrict__ stats, T *dx,
                                                          const T *__restrict__ gate, int accum, float *dgamma,
                                                          float *dbeta, float inv_m, int rows, int C)
{
    __shared__ float wpart[OP_WAVES][2 * V];
    __shared__ double tot[2 * V];
    const int CV = C / V, cg = blockIdx.x;
    const vec_t<T, V> *xv = reinterpret_cast<const vec_t<T, V> *>(x);
    const vec_t<T, V> *gv = reinterpret_cast<const vec_t<T, V> *>(dy);
    vec_t<T, V> a[R], g[R];
#pragma unroll
    for (int u = 0; u < R; ++u) {
        const int r = threadIdx.x + u * OP_NT;
        const size_t i = (size_t)(r < rows ? r : rows - 1) * CV + cg;
        a[u] = xv[i];
        g[u] = gv[i];
    }
    float mu[V], inv[V];
#pragma unroll
    for (int j = 0; j < V; ++j) {
        mu[j] = stats[cg * V + j];
        inv[j] = stats[C + cg * V + j];
    }
    float acc[2 * V];
#pragma unroll
    for (int j = 0; j < 2 * V; ++j) acc[j] = 0.0f;
#pragma unroll
    for (int u = 0; u < R; ++u) {
        const bool in = threadIdx.x + u * OP_NT < rows;
#pragma unroll
        for (int j = 0; j < V; ++j) {
            const float gg = in ? to_f32(g[u].e[j]) : 0.0f;
            const float xh = (to_f32(a[u].e[j]) - mu[j]) * inv[j];
            acc[j] += gg;
            acc[V + j] += gg * xh;
        }
    }
    block_sums<2 * V>(acc, wpart, tot);
    if (threadIdx.x < V) {
        dbeta[cg * V + threadIdx.x] += (float)tot[threadIdx.x];
        dgamma[cg * V + threadIdx.x] += (float)tot[V + threadIdx.x];
    }
    if (!dx) return;
#pragma unroll
    for (int u = 0; u < R; ++u) {
        forget(a[u]);
        forget(g[u]);
    }
    float gi[V], m1[V], m2[V];
#pragma unroll
    for (int j = 0; j < V; ++j) {
        gi[j] = gamma[cg * V + j] * inv[j];
        m1[j] = (float)tot[j] * inv_m;
        m2[j] = (float)tot[V + j] * inv_m;
    }
    const vec_t<T, V> *tv = reinterpret_cast<const vec_t<T, V> *>(gate);
    vec_t<T, V> *dv = reinterpret_cast<vec_t<T, V> *>(dx);
    constexpr int G = R < 2 ? R : 2;
#pragma unroll
    for (int h = 0; h < R / G; ++h) {
        vec_t<T, V> old[G], gt[G];
#pragma unroll
        for (int u = 0; u < G; ++u) {
            const int r = threadIdx.x + (h * G + u) * OP_NT;
            const size_t i = (size_t)(r < rows ? r : rows - 1) * CV + cg;
            if (accum) old[u] = dv[i];
            if (gate) gt[u] = tv[i];
        }
#pragma unroll
        for (int u = 0; u < G; ++u) {
            const int r = threadIdx.x + (h * G + u) * OP_NT;
            if (r < rows) {
                vec_t<T, V> o;
#pragma unroll
                for (int j = 0; j < V; ++j) {
                    float xh = (to_f32(a[h * G + u].e[j]) - mu[j]) * inv[j];
                    float v = gi[j] * (to_f32(g[h * G + u].e[j]) - m1[j] - xh * m2[j]);
                    o.e[j] = grad_out<T>(v, accum != 0, old[u].e[j], gate != nullptr, gt[u].e[j]);
                }
                dv[(size_t)r * CV + cg] = o;
            }
        }
    }
}

// ------------------------------------------------------------------ LSTM cell
__device__ __forceinline__ float sigmoidf(float v) { return 1.0f / (1.0f + expf(-v)); }

template <class T>
__global__ void k_lstm_cell_fwd(const T *__restrict__ P, const float *__restrict__ gh, int S,
                                float *__restrict__ gates, float *__restrict__ cells, T *__restrict__ h,
                                T *__restrict__ hs, int N, int Tn, int H, int t)
{
    const size_t i = (size_t)blockIdx.x * TPB + threadIdx.x;
    if (i >= (size_t)N * H) return;
    const int n = (int)(i / H), j = (int)(i % H);
    const size_t row = (size_t)n * Tn + t;
    float a[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        a[q] = to_f32(P[row * 4 * H + (size_t)q * H + j]);
        float rsum = 0.0f;
        for (int sp = 0; sp < S; ++sp) rsum += gh[((size_t)sp * N + n) * 4 * H + (size_t)q * H + j];
        a[q] += rsum;
    }
    const float ig = sigmoidf(a[0]), fg = sigmoidf(a[1]), gg = tanhf(a[2]), og = sigmoidf(a[3]);
    const float cprev = t > 0 ? cells[(row - 1) * H + j] : 0.0f;
    const float c = fg * cprev + ig * gg;
    float *gt = gates + row * 4 * H + j;
    gt[0] = ig;
    gt[H] = fg;
    gt[2 * (size_t)H] = gg;
    gt[3 * (size_t)H] = og;
    cells[row * H + j] = c;
    const T hv = from_f32<T>(og * tanhf(c));
    h[row * H + j] = hv;
    if (t + 1 < Tn) hs[(row + 1) * H + j] = hv;
    if (t == 0) hs[row * H + j] = from_f32<T>(0.0f);
}

template <class T>
__global__ void k_lstm_cell_bwd(const T *__restrict__ dy, const float *__restrict__ r, int S,
                                const float *__restrict__ gates, const float *__restrict__ cells,
                                float *__restrict__ dcn, T *__restrict__ D, int N, int Tn, int H, int t)
{
    const size_t i = (size_t)blockIdx.x * TPB + threadIdx.x;
    if (i >= (size_t)N * H) return;
    const int n = (int)(i / H), j = (int)(i % H);
    const size_t row = (size_t)n * Tn + t;
    float dh = to_f32(dy[row * H + j]);
    float rsum = 0.0f;
    for (int sp = 0; sp < S; ++sp) rsum += r[((size_t)sp * N + n) * H + j];
    dh += rsum;
    const float *gt = gates + row * 4 * H + j;
    const float ig = gt[0], fg = gt[H], gg = gt[2 * (size_t)H], og = gt[3 * (size_t)H];
    const float th = tanhf(cells[row * H + j]);
    const float cprev = t > 0 ? cells[(row - 1) * H + j] : 0.0f;
    const float carry = t + 1 < Tn ? dcn[i] : 0.0f;
    const float dc = dh * og * (1.0f - th * th) + carry;
    T *d = D + row * 4 * H + j;
    d[0] = from_f32<T>(dc * gg * ig * (1.0f - ig));
    d[H] = from_f32<T>(dc * cprev * fg * (1.0f - fg));
    d[2 * (size_t)H] = from_f32<T>(dc * ig * (1.0f - gg * gg));
    d[3 * (size_t)H] = from_f32<T>(dh * th * og * (1.0f - og));
    dcn[i] = dc * fg;
}

// ------------------------------------------------------------------ softmax cross-entropy
template <class T>
__global__ void k_softmax_fwd(const T *__restrict__ z, float *__restrict__ p, int K)
{
    __shared__ float sh[TPB / 64];
    __shared__ float bc;
    const T *zr = z + (size_t)blockIdx.x * K;
    float *pr = p + (size_t)blockIdx.x * K;
    float mx = -INFINITY;
    for (int k = threadIdx.x; k < K; k += TPB) mx = fmaxf(mx, to_f32(zr[k]));
    mx = wave_max(mx);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
        float m = sh[0];
        for (int i = 1; i < TPB / 64; ++i) m = fmaxf(m, sh[i]);
        bc = m;
    }
    __syncthreads();
    mx = bc;
    float s = 0.0f;
    for (int k = threadIdx.x; k < K; k += TPB) s += expf(to_f32(zr[k]) - mx);
    s = wave_sum(s);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = 0.0f;
        for (int i = 0; i < TPB / 64; ++i) t += sh[i];
        bc = t;
    }
    __syncthreads();
    float inv = 1.0f / bc;
    for (int k = threadIdx.x; k < K; k += TPB) pr[k] = expf(to_f32(zr[k]) - mx) * inv;
}

template <class T>
__global__ void k_xent_dz(const float *__restrict__ p, const int32_t *__restrict__ labels, float scale,
                          T *__restrict__ dz, int K)
{
    const int n = blockIdx.x;
    const int lab = labels[n];
    for (int k = threadIdx.x; k < K; k += TPB) {
        float v = scale * (p[(size_t)n * K + k] - (k == lab ? 1.0f : 0.0f));
        dz[(size_t)n * K + k] = from_f32<T>(v);
    }
}

// one block: loss = -scale * sum_n log p[n, label_n]   (labels outside [0,K) contribute 0)
__global__ void k_xent_loss(const float *__restrict__ p, const int32_t *__restrict__ labels, float scale,
                            float *loss, int rows, int K)
{
    __shared__ float sh[TPB / 64];
    float s = 0.0f;
    for (int n = threadIdx.x; n < rows; n += TPB) {
        int lab = labels[n];
        if (lab >= 0 && lab < K) s -= logf(fmaxf(p[(size_t)n * K + lab], 1e-37f));
    }
    s = wave_sum(s);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = 0.0f;
        for (int i = 0; i < TPB / 64; ++i) t += sh[i];
        loss[0] = scale * t;
    }
}

// ------------------------------------------------------------------ parameters
template <class T, bool HAS_WORK>
__global__ void k_sgd(float *__restrict__ w, float *__restrict__ g, float lr, T *__restrict__ work, size_t n)
{
    size_t i = (size_t)blockIdx.x * TPB + threadIdx.x;
    if (i >= n) return;
    float v = w[i] - lr * g[i];
    w[i] = v;
    g[i] = 0.0f;
    if (HAS_WORK) work[i] = from_f32<T>(v);
}

template <class T> __global__ void k_recast(const float *__restrict__ w, T *__restrict__ work, size_t n)
{
    size_t i = (size_t)blockIdx.x * TPB + threadIdx.x;
    if (i < n) work[i] = from_f32<T>(w[i]);
}

// wt[c][r][s][k] = w[k][R-1-r][S-1-s][c] in storage type: per tap a K x C -> C x K transpose, done
// on 64 x 64 tiles through LDS so that both the fp32 reads (along c) and the writes (along k) are
// contiguous.  grid: (C tiles, K tiles, R*S)
template <class T>
__global__ void k_dgrad_filter(const float *__restrict__ w, T *__restrict__ wt, int K, int R, int S, int C)
{
    __shared__ float tile[64][65];
    const int c0 = blockIdx.x * 64, k0 = blockIdx.y * 64;
    const int tap = blockIdx.z, r = tap / S, q = tap - r * S;
    const int src_tap = (R - 1 - r) * S + (S - 1 - q);
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;          // 64 x 4
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int k = k0 + ty + 4 * i, c = c0 + tx;
        tile[ty + 4 * i][tx] = (k < K && c < C) ? w[((size_t)k * R * S + src_tap) * C + c] : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int c = c0 + ty + 4 * i, k = k0 + tx;
        if (c < C && k < K) wt[((size_t)c * R * S + tap) * K + k] = from_f32<T>(tile[tx][ty + 4 * i]);
    }
}

__global__ void k_fill(float *p, float v, size_t n)
{
    size_t i = (size_t)blockIdx.x * TPB + threadIdx.x;
    if (i < n) p[i] = v;
}

// ------------------------------------------------------------------ layout changes
// NCHW (C channels) -> NHWC with Cp >= C physical channels, the extra ones zero
template <class T>
__global__ void k_nchw_to_nhwc(const T *__restrict__ src, T *dst, const T *__restrict__ gate, int accum,
                               int N, int C, int H, int W, int Cp)
{
    size_t i = (size_t)blockIdx.x * TPB + threadIdx.x;       // index into dst (NHWC)
    size_t total = (size_t)N * Cp * H * W;
    if (i >= total) return;
    int c = (int)(i % Cp);
    size_t t = i / Cp;
    int w = (int)(t % W);
    t /= W;
    int h = (int)(t % H);
    int n = (int)(t / H);
    T v = from_f32<T>(0.0f);
    if (c < C) v = src[(((size_t)n * C + c) * H + h) * W + w];
    if (gate || accum) {
        T old = v, gt = v;
        if (accum) old = dst[i];
        if (gate) gt = gate[i];
        v = grad_out<T>(to_f32(v), accum != 0, old, gate != nullptr, gt);
    }
    dst[i] = v;
}

// NHWC with Cp physical channels -> NCHW with the first C of them
template <class T>
__global__ void k_nhwc_to_nchw(const T *__restrict__ src, T *__restrict__ dst, int N, int C, int H, int W,
                               int Cp)
{
    size_t i = (size_t)blockIdx.x * TPB + threadIdx.x;       // index into dst (NCHW)
    size_t total = (size_t)N * C * H * W;
    if (i >= total) return;
    int w = (int)(i % W);
    size_t t = i / W;
    int h = (int)(t % H);
    t /= H;
    int c = (int)(t % C);
    int n = (int)(t / C);
    dst[i] = src[(((size_t)n * H + h) * W + w) * Cp + c];
}

// rows x Cs -> rows x Cd (zero fill when Cd > Cs, truncate when Cd < Cs)
template <class T>
__global__ void k_repad(const T *__restrict__ src, T *__restrict__ dst, size_t rows, int Cs, int Cd)
{
    size_t i = (size_t)blockIdx.x * TPB + threadIdx.x;
    if (i >= rows * Cd) return;
    int c = (int)(i % Cd);
    size_t r = i / Cd;
    dst[i] = c < Cs ? src[r * Cs + c] : from_f32<T>(0.0f);
}

// the common case (RGB input padded to 8 bf16 channels): one thread builds one 16-byte pixel
template <int CS>
__global__ void k_repad_to8(const uint16_t *__restrict__ src, uint4 *__restrict__ dst, size_t rows)
{
    size_t r = (size_t)blockIdx.x * TPB + threadIdx.x;
    if (r >= rows) return;
    uint16_t v[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) v[c] = c < CS ? src[r * CS + c] : (uint16_t)0;
    uint4 o;
    o.x = v[0] | ((uint32_t)v[1] << 16);
    o.y = v[2] | ((uint32_t)v[3] << 16);
    o.z = v[4] | ((uint32_t)v[5] << 16);
    o.w = v[6] | ((uint32_t)v[7] << 16);
    dst[r] = o;
}

#define DISPATCH_T(dt, ...)                        \
    do {                                           \
        if ((dt) == DT_F32) {                      \
            using T = float;                       \
            __VA_ARGS__                            \
        } else {                                   \
            using T = bf16_t;                      \
            __VA_ARGS__                            \
        }                                          \
    } while (0)

#define DISPATCH_TV(dt, vec, ...)                  \
    do {                                           \
        if ((dt) == DT_F32) {                      \
            using T = float;                       \
            if (vec) {                             \
                constexpr int V = 4;               \
                __VA_ARGS__                        \
            } else {                               \
                constexpr int V = 1;               \
                __VA_ARGS__                        \
            }                                      \
        } else {                                   \
            using T = bf16_t;                      \
            if (vec) {                             \
                constexpr int V = 8;               \
                __VA_ARGS__                        \
            } else {                               \
                constexpr int V = 1;               \
                __VA_ARGS__                        \
            }                                      \
        }                                          \
    } while (0)

inline bool flat_vec(int dt, size_t n, const void *a, const void *b = nullptr, const void *c = nullptr,
                     const void *d = nullptr)
{
    size_t V = dt == DT_F32 ? 4 : 8;
    return n % V == 0 && aligned16(a) && aligned16(b) && aligned16(c) && aligned16(d);
}

}  // namespace

// ====================================================================== launchers
hipError_t relu_fwd(int dt, const void *x, void *y, size_t n, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    bool vec = flat_vec(dt, n, x, y);
    DISPATCH_TV(dt, vec, {
        size_t nv = n / V;
        hipLaunchKernelGGL((k_relu_fwd<T, V>), dim3(blocks_for(nv)), dim3(TPB), 0, s, (const T *)x, (T *)y, nv);
    });
    return hipGetLastError();
}

hipError_t relu_bwd(int dt, const void *y, const void *dy, void *dx, GradEpi epi, size_t n, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    bool vec = flat_vec(dt, n, y, dy, dx, epi.gate);
    DISPATCH_TV(dt, vec, {
        size_t nv = n / V;
        hipLaunchKernelGGL((k_grad_copy<T, V>), dim3(blocks_for(nv)), dim3(TPB), 0, s, (const T *)dy,
                           (const T *)y, (T *)dx, (const T *)epi.gate, epi.accum, nv);
    });
    return hipGetLastError();
}

hipError_t grad_copy(int dt, const void *dy, void *dx, GradEpi epi, size_t n, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    bool vec = flat_vec(dt, n, dy, dx, epi.gate);
    DISPATCH_TV(dt, vec, {
        size_t nv = n / V;
        hipLaunchKernelGGL((k_grad_copy<T, V>), dim3(blocks_for(nv)), dim3(TPB), 0, s, (const T *)dy,
                           (const T *)nullptr, (T *)dx, (const T *)epi.gate, epi.accum, nv);
    });
    return hipGetLastError();
}

hipError_t upsample_grad(int dt, const void *t, void *dx, GradEpi epi, int N, int H, int W, int Ho, int Wo, int C,
                         int stride, hipStream_t s)
{
    if (stride < 1 || (long long)(Ho - 1) * stride >= H || (long long)(Wo - 1) * stride >= W) return hipErrorInvalidValue;
    const size_t n = (size_t)N * H * W * C;
    if (n == 0) return hipSuccess;
    const int Vw = dt == DT_F32 ? 4 : 8;
    const bool vec = C % Vw == 0 && aligned16(t) && aligned16(dx) && aligned16(epi.gate);
    DISPATCH_TV(dt, vec, {
        hipLaunchKernelGGL((k_upsample_grad<T, V>), dim3(blocks_for(n / V)), dim3(TPB), 0, s, (const T *)t, (T *)dx,
                           (const T *)epi.gate, epi.accum, N, H, W, Ho, Wo, C / V, stride);
    });
    return hipGetLastError();
}

hipError_t add_fwd(int dt, const void *a, const void *b, void *y, int relu, size_t n, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    bool vec = flat_vec(dt, n, a, b, y);
    DISPATCH_TV(dt, vec, {
        size_t nv = n / V;
        hipLaunchKernelGGL((k_add_fwd<T, V>), dim3(blocks_for(nv)), dim3(TPB), 0, s, (const T *)a,
                           (const T *)b, (T *)y, relu, nv);
    });
    return hipGetLastError();
}

hipError_t maxpool2x2_fwd(int dt, const void *x, void *y, uint8_t *idx, int N, int H, int W, int C,
                          hipStream_t s)
{
    size_t outs = (size_t)N * (H / 2) * (W / 2) * C;
    if (outs == 0) return hipSuccess;
    int Vw = dt == DT_F32 ? 4 : 8;
    bool vec = (C % Vw == 0) && aligned16(x) && aligned16(y) && ((uintptr_t)idx % 8 == 0);
    DISPATCH_TV(dt, vec, {
        size_t nv = outs / V;
        hipLaunchKernelGGL((k_pool_fwd<T, V>), dim3(blocks_for(nv)), dim3(TPB), 0, s, (const T *)x, (T *)y,
                           idx, N, H, W, C / V);
    });
    return hipGetLastError();
}

hipError_t maxpool2x2_bwd(int dt, const void *dy, const uint8_t *idx, void *dx, GradEpi epi, int N, int H,
                          int W, int C, hipStream_t s)
{
    size_t outs = (size_t)N * (H / 2) * (W / 2) * C;
    if (((H | W) & 1) && !epi.accum) {   // odd sizes: the last row/column gets no gradient
        size_t bytes = (size_t)N * H * W * C * dt_size(dt);
        hipLaunchKernelGGL(k_fill, dim3(blocks_for(bytes / 4)), dim3(TPB), 0, s, (float *)dx, 0.0f, bytes / 4);
        if (bytes % 4) return hipErrorInvalidValue;
    }
    if (outs == 0) return hipGetLastError();
    int Vw = dt == DT_F32 ? 4 : 8;
    bool vec = (C % Vw == 0) && aligned16(dy) && aligned16(dx) && aligned16(epi.gate) &&
               ((uintptr_t)idx % 8 == 0);
    DISPATCH_TV(dt, vec, {
        size_t nv = outs / V;
        hipLaunchKernelGGL((k_pool_bwd<T, V>), dim3(blocks_for(nv)), dim3(TPB), 0, s, (const T *)dy, idx,
                           (T *)dx, (const T *)epi.gate, epi.accum, N, H, W, C / V);
    });
    return hipGetLastError();
}

static PoolWin pool_win(int N, int H, int W, int C, int V, int kh, int kw, int stride, int pad)
{
    PoolWin g{N, H, W, C / V, (H + 2 * pad - kh) / stride + 1, (W + 2 * pad - kw) / stride + 1, kh, kw, stride, pad};
    return g;
}

hipError_t maxpool_fwd(int dt, const void *x, void *y, uint8_t *idx, int N, int H, int W, int C, int kh,
                       int kw, int stride, int pad, hipStream_t s)
{
    if (kh < 1 || kw < 1 || kh * kw > 255 || stride < 1 || pad < 0 || pad >= kh || pad >= kw ||
        H + 2 * pad < kh || W + 2 * pad < kw)
        return hipErrorInvalidValue;
    if (kh == 2 && kw == 2 && stride == 2 && pad == 0) return maxpool2x2_fwd(dt, x, y, idx, N, H, W, C, s);
    int Vw = dt == DT_F32 ? 4 : 8;
    bool vec = (C % Vw == 0) && aligned16(x) && aligned16(y) && ((uintptr_t)idx % 8 == 0);
    DISPATCH_TV(dt, vec, {
        PoolWin g = pool_win(N, H, W, C, V, kh, kw, stride, pad);
        size_t nv = (size_t)N * g.Ho * g.Wo * g.CV;
        if (nv == 0) return hipSuccess;
        hipLaunchKernelGGL((k_poolw_fwd<T, V>), dim3(blocks_for(nv)), dim3(TPB), 0, s, (const T *)x, (T *)y, idx, g);
    });
    return hipGetLastError();
}

hipError_t maxpool_bwd(int dt, const void *dy, const uint8_t *idx, void *dx, GradEpi epi, int N, int H, int W,
                       int C, int kh, int kw, int stride, int pad, hipStream_t s)
{
    if (kh < 1 || kw < 1 || kh * kw > 255 || stride < 1 || pad < 0 || pad >= kh || pad >= kw ||
        H + 2 * pad < kh || W + 2 * pad < kw)
        return hipErrorInvalidValue;
    if (kh == 2 && kw == 2 && stride == 2 && pad == 0) return maxpool2x2_bwd(dt, dy, idx, dx, epi, N, H, W, C, s);
    int Vw = dt == DT_F32 ? 4 : 8;
    bool vec = (C % Vw == 0) && aligned16(dy) && aligned16(dx) && aligned16(epi.gate) && ((uintptr_t)idx % 8 == 0);
    DISPATCH_TV(dt, vec, {
        PoolWin g = pool_win(N, H, W, C, V, kh, kw, stride, pad);
        size_t nv = (size_t)N * H * W * g.CV;
        if (nv == 0) return hipSuccess;
        hipLaunchKernelGGL((k_poolw_bwd<T, V>), dim3(blocks_for(nv)), dim3(TPB), 0, s, (const T *)dy, idx, (T *)dx,
                           (const T *)epi.gate, epi.accum, g);
    });
    return hipGetLastError();
}

hipError_t avgpool_fwd(int dt, const void *x, void *y, int N, int H, int W, int C, int kh, int kw, hipStream_t s)
{
    if (kh < 1 || kw < 1 || kh > H || kw > W) return hipErrorInvalidValue;
    int Vw = dt == DT_F32 ? 4 : 8;
    bool vec = (C % Vw == 0) && aligned16(x) && aligned16(y);
    DISPATCH_TV(dt, vec, {
        PoolWin g{N, H, W, C / V, H / kh, W / kw, kh, kw, 0, 0};
        size_t nv = (size_t)N * g.Ho * g.Wo * g.CV;
        if (nv == 0) return hipSuccess;
        hipLaunchKernelGGL((k_avgpool_fwd<T, V>), dim3(blocks_for(nv)), dim3(TPB), 0, s, (const T *)x, (T *)y, g);
    });
    return hipGetLastError();
}

hipError_t avgpool_bwd(int dt, const void *dy, void *dx, GradEpi epi, int N, int H, int W, int C, int kh, int kw,
                       hipStream_t s)
{
    if (kh < 1 || kw < 1 || kh > H || kw > W) return hipErrorInvalidValue;
    int Vw = dt == DT_F32 ? 4 : 8;
    bool vec = (C % Vw == 0) && aligned16(dy) && aligned16(dx) && aligned16(epi.gate);
    DISPATCH_TV(dt, vec, {
        PoolWin g{N, H, W, C / V, H / kh, W / kw, kh, kw, 0, 0};
        size_t nv = (size_t)N * H * W * g.CV;
        if (nv == 0) return hipSuccess;
        hipLaunchKernelGGL((k_avgpool_bwd<T, V>), dim3(blocks_for(nv)), dim3(TPB), 0, s, (const T *)dy, (T *)dx,
                           (const T *)epi.gate, epi.accum, g);
    });
    return hipGetLastError();
}

size_t colsum_workspace(int rows, int C)
{
    ColPlan p = col_plan(rows, C, 1);           // V = 1 gives the largest chunk count bound
    ColPlan p8 = col_plan(rows, C, (C % 8 == 0) ? 8 : 1);
    ColPlan p4 = col_plan(rows, C, (C % 4 == 0) ? 4 : 1);
    int chunks = p.chunks > p8.chunks ? p.chunks : p8.chunks;
    chunks = chunks > p4.chunks ? chunks : p4.chunks;
    return (size_t)2 * chunks * C * sizeof(float) + 4 * (size_t)C * sizeof(float);
}

size_t bn_workspace(int rows, int C) { return colsum_workspace(rows, C); }

hipError_t colsum_accumulate(int dt, const void *a, int rows, int C, float *out, void *workspace,
                             hipStream_t s)
{
    if (rows <= 0 || C <= 0) return hipSuccess;
    int Vsel = col_vec(dt, C, a);
    float *part = (float *)workspace;
    DISPATCH_TV(dt, Vsel > 1, {
        ColPlan p = col_plan(rows, C, V);
        hipLaunchKernelGGL((k_colsum_partial<T, V>), dim3(p.gx, p.chunks), dim3(TPB), 0, s, (const T *)a, rows,
                           C, p, part);
        hipLaunchKernelGGL(k_colsum_final, dim3(final_blocks(C)), dim3(TPB), 0, s, part, p.chunks, C, out);
    });
    return hipGetLastError();
}

// The one-launch kernels pay for their strided 8-byte loads (measured: 3x slower than the three
// coalesced launches at 6272 rows), so they are used only where launch latency is all there is:
// 16-byte aligned tensors of at most OP_R rows per thread and at least 32 channel groups.
constexpr int OP_R = 2;
static bool bn_onepass(int Vsel, int rows, int C) { return Vsel > 1 && rows <= OP_R * OP_NT && C / 4 >= 32; }

// channels per block of the one-launch kernels: 8 bytes of bf16 / 16 bytes of float per row
constexpr int OP_V = 4;
#define BN_FWD_OP(T_, R_)                                                                                        \
    hipLaunchKernelGGL((k_bn_fwd_onepass<T_, OP_V, R_>), dim3(C / OP_V), dim3(OP_NT), 0, s, (const T_ *)x, gamma, \
                       beta, eps, (T_ *)y, stats, relu, rows, C, (const T_ *)res, relu_sum)
#define BN_BWD_OP(T_, R_)                                                                                        \
    hipLaunchKernelGGL((k_bn_bwd_onepass<T_, OP_V, R_>), dim3(C / OP_V), dim3(OP_NT), 0, s, (const T_ *)x,        \
                       (const T_ *)dy, gamma, stats, (T_ *)dx, (const T_ *)epi.gate, epi.accum, dgamma, dbeta,    \
                       1.0f / (float)rows, rows, C)

hipError_t bn_fwd(int dt, const void *x, const float *gamma, const float *beta, float eps, void *y,
                  float *stats, int relu, int rows, int C, void *workspace, hipStream_t s, int pre_chunks,
                  const void *res, int relu_sum)
{
    if (rows <= 0 || C <= 0) return hipSuccess;
    if (res && relu) return hipErrorInvalidValue;          // the layer's own ReLU and a residual behind it exclude each other
    int Vsel = col_vec(dt, C, x, y, res);
    float *part = (float *)workspace;
    if (pre_chunks > 0) {                 // statistics partials came with x: final pass and normalisation only
        hipLaunchKernelGGL(k_bn_stat_final, dim3(final_blocks(C)), dim3(TPB), 0, s, part, pre_chunks, C, rows, eps, stats);
        DISPATCH_TV(dt, Vsel > 1, {
            ColPlan p = col_plan(rows, C, V);
            const int rpb = p.RY * BN_ROWS_PER_THREAD;
            hipLaunchKernelGGL((k_bn_apply<T, V>), dim3(p.gx, (rows + rpb - 1) / rpb), dim3(TPB), 0, s, (const T *)x,
                               gamma, beta, stats, (T *)y, relu, rows, C, p, (const T *)res, relu_sum);
        });
        return hipGetLastError();
    }
    if (bn_onepass(Vsel, rows, C)) {
        if (dt == DT_F32) BN_FWD_OP(float, OP_R);
        else BN_FWD_OP(bf16_t, OP_R);
        return hipGetLastError();
    }
    DISPATCH_TV(dt, Vsel > 1, {
        ColPlan p = col_plan(rows, C, V);
        hipLaunchKernelGGL((k_bn_stat_partial<T, V>), dim3(p.gx, p.chunks), dim3(TPB), 0, s, (const T *)x,
                           rows, C, p, part);
        hipLaunchKernelGGL(k_bn_stat_final, dim3(final_blocks(C)), dim3(TPB), 0, s, part, p.chunks, C, rows,
                           eps, stats);
        const int rpb = p.RY * BN_ROWS_PER_THREAD;
        hipLaunchKernelGGL((k_bn_apply<T, V>), dim3(p.gx, (rows + rpb - 1) / rpb), dim3(TPB), 0, s, (const T *)x,
                           gamma, beta, stats, (T *)y, relu, rows, C, p, (const T *)res, relu_sum);
    });
    return hipGetLastError();
}

hipError_t bn_bwd(int dt, const void *x, const void *dy, const float *gamma, const float *stats, void *dx,
                  float *dgamma, float *dbeta, GradEpi epi, int rows, int C, void *workspace,
                  hipStream_t s, int pre_chunks)
{
    if (rows <= 0 || C <= 0) return hipSuccess;
    int Vsel = col_vec(dt, C, x, dy, dx);
    if (!aligned16(epi.gate)) Vsel = 1;
    float *part = (float *)workspace;
    if (pre_chunks > 0) {                 // the sums over dy came with dy: final pass and the dx pass only
        float *sums = part + (size_t)2 * pre_chunks * C;
        hipLaunchKernelGGL(k_bn_bwd_final, dim3(final_blocks(C)), dim3(TPB), 0, s, part, pre_chunks, C, sums, dgamma, dbeta);
        if (dx) {
            DISPATCH_TV(dt, Vsel > 1, {
                ColPlan p = col_plan(rows, C, V);
                const int rpb = p.RY * BN_ROWS_PER_THREAD;
                hipLaunchKernelGGL((k_bn_bwd_apply<T, V>), dim3(p.gx, (rows + rpb - 1) / rpb), dim3(TPB), 0, s,
                                   (const T *)x, (const T *)dy, gamma, stats, sums, (T *)dx, (const T *)epi.gate,
                                   epi.accum, 1.0f / (float)rows, rows, C, p);
            });
        }
        return hipGetLastError();
    }
    if (bn_onepass(Vsel, rows, C)) {
        if (dt == DT_F32) BN_BWD_OP(float, OP_R);
        else BN_BWD_OP(bf16_t, OP_R);
        return hipGetLastError();
    }
    DISPATCH_TV(dt, Vsel > 1, {
        ColPlan p = col_plan(rows, C, V);
        float *sums = part + (size_t)2 * p.chunks * C;
        hipLaunchKernelGGL((k_bn_bwd_partial<T, V>), dim3(p.gx, p.chunks), dim3(TPB), 0, s, (const T *)x,
                           (const T *)dy, stats, rows, C, p, part);
        hipLaunchKernelGGL(k_bn_bwd_final, dim3(final_blocks(C)), dim3(TPB), 0, s, part, p.chunks, C, sums,
                           dgamma, dbeta);
        if (dx) {
            const int rpb = p.RY * BN_ROWS_PER_THREAD;
            hipLaunchKernelGGL((k_bn_bwd_apply<T, V>), dim3(p.gx, (rows + rpb - 1) / rpb), dim3(TPB), 0, s,
                               (const T *)x, (const T *)dy, gamma, stats, sums, (T *)dx, (const T *)epi.gate,
                               epi.accum, 1.0f / (float)rows, rows, C, p);
        }
    });
    return hipGetLastError();
}

hipError_t lstm_cell_fwd(int dt, const void *P, const float *gh, int S, float *gates, float *cells, void *h,
                         void *hs, int N, int Tn, int H, int t, hipStream_t s)
{
    if (N <= 0 || H <= 0 || t < 0 || t >= Tn || S < 0 || (t == 0 && S != 0)) return hipErrorInvalidValue;
    DISPATCH_T(dt, {
        hipLaunchKernelGGL((k_lstm_cell_fwd<T>), dim3(blocks_for((size_t)N * H)), dim3(TPB), 0, s, (const T *)P, gh, S,
                           gates, cells, (T *)h, (T *)hs, N, Tn, H, t);
    });
    return hipGetLastError();
}

hipError_t lstm_cell_bwd(int dt, const void *dy, const float *r, int S, const float *gates, const float *cells,
                         float *dcn, void *D, int N, int Tn, int H, int t, hipStream_t s)
{
    if (N <= 0 || H <= 0 || t < 0 || t >= Tn || S < 0 || (t == Tn - 1 && S != 0)) return hipErrorInvalidValue;
    DISPATCH_T(dt, {
        hipLaunchKernelGGL((k_lstm_cell_bwd<T>), dim3(blocks_for((size_t)N * H)), dim3(TPB), 0, s, (const T *)dy, r, S,
                           gates, cells, dcn, (T *)D, N, Tn, H, t);
    });
    return hipGetLastError();
}

hipError_t softmax_fwd(int dt, const void *z, float *p, int rows, int K, hipStream_t s)
{
    if (rows <= 0) return hipSuccess;
    DISPATCH_T(dt, { hipLaunchKernelGGL((k_softmax_fwd<T>), dim3(rows), dim3(TPB), 0, s, (const T *)z, p, K); });
    return hipGetLastError();
}

hipError_t xent_bwd(int dt, const float *p, const int32_t *labels, float scale, void *dz, float *loss,
                    int rows, int K, hipStream_t s)
{
    if (rows <= 0) return hipSuccess;
    DISPATCH_T(dt, {
        hipLaunchKernelGGL((k_xent_dz<T>), dim3(rows), dim3(TPB), 0, s, p, labels, scale, (T *)dz, K);
    });
    hipLaunchKernelGGL(k_xent_loss, dim3(1), dim3(TPB), 0, s, p, labels, scale, loss, rows, K);
    return hipGetLastError();
}

hipError_t sgd_step(int dt, float *w, float *g, float lr, void *work, size_t n, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    if (!work) {
        hipLaunchKernelGGL((k_sgd<float, false>), dim3(blocks_for(n)), dim3(TPB), 0, s, w, g, lr, (float *)nullptr, n);
    } else {
        DISPATCH_T(dt, {
            hipLaunchKernelGGL((k_sgd<T, true>), dim3(blocks_for(n)), dim3(TPB), 0, s, w, g, lr, (T *)work, n);
        });
    }
    return hipGetLastError();
}

hipError_t recast(int dt, const float *w, void *work, size_t n, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    DISPATCH_T(dt, { hipLaunchKernelGGL((k_recast<T>), dim3(blocks_for(n)), dim3(TPB), 0, s, w, (T *)work, n); });
    return hipGetLastError();
}

hipError_t make_dgrad_filter(int dt, const float *w, void *wt, int K, int R, int S, int C, hipStream_t s)
{
    size_t n = (size_t)K * R * S * C;
    if (n == 0) return hipSuccess;
    DISPATCH_T(dt, {
        hipLaunchKernelGGL((k_dgrad_filter<T>), dim3((unsigned)((C + 63) / 64), (unsigned)((K + 63) / 64), (unsigned)(R * S)),
                           dim3(256), 0, s, w, (T *)wt, K, R, S, C);
    });
    return hipGetLastError();
}

hipError_t fill_f32(float *p, float v, size_t n, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(k_fill, dim3(blocks_for(n)), dim3(TPB), 0, s, p, v, n);
    return hipGetLastError();
}

hipError_t nchw_to_nhwc(int dt, const void *src, void *dst, GradEpi epi, int N, int C, int H, int W,
                        int Cp, hipStream_t s)
{
    size_t n = (size_t)N * Cp * H * W;
    if (n == 0) return hipSuccess;
    DISPATCH_T(dt, {
        hipLaunchKernelGGL((k_nchw_to_nhwc<T>), dim3(blocks_for(n)), dim3(TPB), 0, s, (const T *)src, (T *)dst,
                           (const T *)epi.gate, epi.accum, N, C, H, W, Cp);
    });
    return hipGetLastError();
}

hipError_t nhwc_to_nchw(int dt, const void *src, void *dst, int N, int C, int H, int W, int Cp,
                        hipStream_t s)
{
    size_t n = (size_t)N * C * H * W;
    if (n == 0) return hipSuccess;
    DISPATCH_T(dt, {
        hipLaunchKernelGGL((k_nhwc_to_nchw<T>), dim3(blocks_for(n)), dim3(TPB), 0, s, (const T *)src, (T *)dst,
                           N, C, H, W, Cp);
    });
    return hipGetLastError();
}

hipError_t nhwc_repad(int dt, const void *src, void *dst, size_t rows, int Cs, int Cd, hipStream_t s)
{
    size_t n = rows * Cd;
    if (n == 0) return hipSuccess;
    if (dt == DT_BF16 && Cd == 8 && aligned16(dst) && (Cs == 3 || Cs == 1 || Cs == 4)) {
#define REPAD8(CS_) \
    hipLaunchKernelGGL((k_repad_to8<CS_>), dim3(blocks_for(rows)), dim3(TPB), 0, s, (const uint16_t *)src, (uint4 *)dst, rows)
        if (Cs == 3) REPAD8(3);
        else if (Cs == 1) REPAD8(1);
        else REPAD8(4);
#undef REPAD8
        return hipGetLastError();
    }
    DISPATCH_T(dt, {
        hipLaunchKernelGGL((k_repad<T>), dim3(blocks_for(n)), dim3(TPB), 0, s, (const T *)src, (T *)dst, rows, Cs, Cd);
    });
    return hipGetLastError();
}

hipError_t nhwc_to_nchw_u8(const uint8_t *src, uint8_t *dst, int N, int C, int H, int W, hipStream_t s)
{
    size_t n = (size_t)N * C * H * W;
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL((k_nhwc_to_nchw<uint8_t>), dim3(blocks_for(n)), dim3(TPB), 0, s, src, dst, N, C, H, W, C);
    return hipGetLastError();
}

}  // namespace bapipe
