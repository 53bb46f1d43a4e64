// Host side of libbapipe_stage: the C ABI of include/bapipe_stage.h, shape inference over the
// layer list, the 1F1B micro-batch bookkeeping with its bounded activation-stash ring
// (paper Sec. III-B-1, Table I/II "Features memory"), the HBM memory plan, the per-layer
// kernel sequencing for forward / backward / update, and the layer profiler (Sec. III-A).
//
// Memory plan (all HBM, one allocation each, obtained through the caller's allocator):
//   params    fp32 master w,b | fp32 accumulators dw,db | working copies (storage type):
//             w [K][R][S][C] for forward, flipped channel-transposed [C][R][S][K] for dgrad
//   stash     depth x slot ; a slot holds, for one in-flight micro-batch, exactly the tensors
//             backward reads again: layer inputs of conv/linear/BN, ReLU gates, pool indices,
//             BN statistics, softmax output.  depth = min(M, N-i+1) (x2 for 1F1B-SO).
//   transient forward tensors nobody reads in backward (reused by every micro-batch)
//   grads     one buffer per tensor that receives an activation gradient (reused)
//   workspace split-K / column-reduction partials
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/bapipe_stage.h"
#include "kernels.h"

using namespace bapipe;

namespace {

thread_local std::string g_create_error;      // message of the calling thread's last failed create (the one piece of
                                              // state that is not in a handle: there is no handle to keep it in)
constexpr size_t kTapMaxEvents = 2 * (1u << 18);   // event pairs the measurement tap may hold

size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

struct Tensor {
    int C = 0, H = 0, W = 0;
    int Cp = 0;            // channels as laid out in HBM (>= C: a narrow stage input is zero-padded)
    size_t elems = 0;      // per micro-batch, physical (Cp channels)
    size_t esize = 0;      // bytes per element
    int root = -1;         // storage owner (FLATTEN outputs alias their input)
    int producer = -1;     // layer index, -1 for the stage input
    bool stashed = false;  // kept per in-flight micro-batch
    bool need_grad = false;
    bool gated = false;    // producer applies a fused ReLU (or is a ReLU layer)
    size_t off = 0;        // byte offset in the stash slot or in the transient arena
    size_t goff = 0;       // byte offset in the gradient arena
    int galias = -1;       // tensor whose gradient IS this tensor's gradient (an un-gated input of an ADD that
                           // nobody else reads: the sum's gradient passes through unchanged, no copy is made)
    std::vector<int> consumers;
    // Input / output gradient of a linear layer whose weight gradient is deferred: the tensor (its gradient) lives
    // in that layer's per-mini-batch buffer, one copy per micro-batch, so that nothing has to be copied there.
    char *mb_store = nullptr, *gmb_store = nullptr;
    // Gradient with two sources, a residual ADD (processed first in backward) and a conv: the ADD's share is not
    // copied, the conv's input-gradient epilogue reads it where it lies (GradEpi::accum_from).  Layer index of
    // that conv, or -1.
    int fanout_conv = -1;
    size_t bytes() const { return elems * esize; }
};

struct Layer {
    bapipe_layer_desc_t d;
    int a = -1, b = -1, o = -1;   // tensor ids (0 = stage input, i+1 = output of layer i)
    size_t w_elems = 0, b_elems = 0;
    float *w = nullptr, *bias = nullptr, *dw = nullptr, *db = nullptr;
    void *w_work = nullptr, *w_t = nullptr;
    size_t aux_off = 0, aux_bytes = 0;   // pool indices / BN statistics inside the slot
    int cin_p = 0;                       // input channels as laid out in HBM (conv / linear)
    // deferred weight gradient (linear layers): the layer's input and gated output gradient of every
    // micro-batch are kept and ONE wgrad GEMM over all of them runs at step time, so that dW
    // (hundreds of MB for the VGG classifier) is touched once per mini-batch instead of M times
    bool deferred = false;
    char *def_x = nullptr, *def_g = nullptr;
    size_t def_x_bytes = 0, def_g_bytes = 0;     // per micro-batch
    // conv whose output only feeds a 2x2 max-pool: the pool runs in the conv kernel's epilogue and
    // the conv output is never stored (fuse_pool = index of that pool layer; fused marks the pool)
    int fuse_pool = -1;
    bool fused = false;
    // conv directly followed by the batch-norm that is its only reader: the conv kernel leaves the per-tile
    // statistics partials in the workspace (stat_chunks of them) and the batch-norm skips its first pass
    int stat_chunks = 0;
    bool stats_given = false;
    // conv whose input is the output of the batch-norm right before it (its only reader): the conv's
    // input-gradient kernel leaves the per-tile sums of dy and dy*xhat for that batch-norm's backward
    int bnb_chunks = 0;
    bool bwd_sums_given = false;
    // 1x1 conv with a stride: its input gradient is non-zero only at multiples of the stride, so the product
    // with the filter is taken at the output's resolution into the workspace (at up_off) and spread from there
    bool strided_1x1 = false;
    size_t up_off = 0;
    int fuse_add = -1;     // batch-norm: the residual ADD (layer index) whose sum this layer's normalisation pass stores
    // LSTM: per in-flight micro-batch the slot keeps the gates and cell states (float), the delayed
    // copy of h that the recurrent products read, the buffer shared by the input projection
    // (forward) and the pre-activation gradients (backward) and the cell-gradient carry
    size_t off_gates = 0, off_cells = 0, off_hs = 0, off_pd = 0, off_dcn = 0;
    bool permute_in = false;             // LINEAR fed by a flattened (C,H,W) tensor
    int pc = 0, ph = 0, pw = 0;
};

}  // namespace

struct bapipe_stage {
    std::vector<Layer> layers;
    std::vector<Tensor> tensors;
    bapipe_stage_opts_t opts;
    int dt = DT_F32;
    int mb = 0, M = 0, depth = 0;
    float loss_scale = 0.f;
    hipStream_t stream = nullptr;
    // with a backward stream (bapipe_stage_set_streams) the backward passes run beside the forward passes of
    // later micro-batches: stream_f / work_f are the handle's own stream and workspace, stream_b / work_b those of the
    // backward passes, `stream` / `work` whichever the pass being enqueued uses.  Events order the two:
    // forward m -> backward m (its features), backward m -> forward m + depth (which reuses its ring slot)
    hipStream_t stream_f = nullptr, stream_b = nullptr;
    // with a weight-gradient stream the wgrad kernels of a backward pass run beside its input-gradient kernels (they
    // only need the layer's output gradient, marked by ev_g, and stashed features); the pass's own stream waits for
    // them at the end of the pass (ev_w_end), so "pass complete" keeps covering them
    hipStream_t stream_w = nullptr;
    char *work_w = nullptr;
    hipEvent_t ev_g = nullptr, ev_w_end = nullptr;
    bool w_used = false;
    char *work_f = nullptr, *work_b = nullptr;
    std::vector<hipEvent_t> ev_fwd, ev_bwd;
    // arenas
    char *params = nullptr, *stash = nullptr, *transient = nullptr, *grads = nullptr, *work = nullptr;
    char *deferred = nullptr;
    size_t deferred_bytes = 0;
    int flushed = 0;                         // micro-batches whose deferred weight gradients are already in dw
    float *losses = nullptr;
    size_t params_bytes = 0, slot_bytes = 0, transient_bytes = 0, grads_bytes = 0, work_bytes = 0;
    size_t accum_off = 0, accum_bytes = 0;   // the dw/db region inside params (zeroed together)
    // schedule
    int n_fwd = 0, n_bwd = 0;
    std::vector<char> loss_valid;
    std::string err;
    // measurement tap: event pairs around launches of one kernel class
    int tap_class = -1;
    std::vector<hipEvent_t> tap_events;
    size_t tap_used = 0;
    double tap_flop = 0.0, tap_bytes = 0.0;
    size_t tap_dropped = 0;                  // launches of the class that found no event pair (pool limit reached)
    hipStream_t tap_stream = nullptr;        // stream of the launch being bracketed
    bool tap_begin(int cls, hipStream_t on = nullptr)
    {
        if (cls != tap_class) return false;
        tap_stream = on ? on : stream;
        if (tap_used + 2 > tap_events.size()) {              // grow the pool: host-side objects only
            const size_t grow = 2 * 1024;
            if (tap_events.size() + grow > kTapMaxEvents) { ++tap_dropped; return false; }
            for (size_t i = 0; i < grow; ++i) {
                hipEvent_t e;
                if (hipEventCreate(&e) != hipSuccess) { (void)hipGetLastError(); ++tap_dropped; return false; }
                tap_events.push_back(e);
            }
        }
        (void)hipEventRecord(tap_events[tap_used], tap_stream);
        return true;
    }
    void tap_end(bool on, double flop, double bytes)
    {
        if (!on) return;
        (void)hipEventRecord(tap_events[tap_used + 1], tap_stream);
        tap_used += 2;
        tap_flop += flop;
        tap_bytes += bytes;
    }

    void *dev_alloc(size_t bytes)
    {
        if (bytes == 0) bytes = 256;
        if (opts.mem.alloc) return opts.mem.alloc(bytes, opts.mem.ctx);
        void *p = nullptr;
        if (hipMalloc(&p, bytes) != hipSuccess) {
            (void)hipGetLastError();
            return nullptr;
        }
        return p;
    }
    void dev_free(void *p)
    {
        if (!p) return;
        if (opts.mem.alloc) {
            if (opts.mem.free) opts.mem.free(p, opts.mem.ctx);
        } else {
            (void)hipFree(p);
        }
    }
    int fail(int code, const char *fmt, ...)
    {
        char buf[512];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof buf, fmt, ap);
        va_end(ap);
        err = buf;
        return code;
    }
    char *slot(int mbid) { return stash + (size_t)(mbid % depth) * slot_bytes; }
    void *tptr(int t, int mbid)
    {
        const Tensor &T = tensors[tensors[t].root];
        if (T.mb_store) return T.mb_store + (size_t)mbid * T.bytes();
        return (T.stashed ? slot(mbid) : transient) + T.off;
    }
    void *gptr(int t) { return grads + tensors[tensors[t].root].goff; }
};

namespace {

int create_fail(int code, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_create_error = buf;
    return code;
}

hipError_t sync_streams(bapipe_stage *st)
{
    hipError_t e = hipStreamSynchronize(st->stream);
    if (e == hipSuccess && st->stream_b) e = hipStreamSynchronize(st->stream_b);
    if (e == hipSuccess && st->stream_w) e = hipStreamSynchronize(st->stream_w);
    return e;
}

bool has_params(int kind)
{
    return kind == BAPIPE_CONV2D || kind == BAPIPE_LINEAR || kind == BAPIPE_BATCHNORM2D || kind == BAPIPE_LSTM;
}
bool has_matrix(int kind) { return kind == BAPIPE_CONV2D || kind == BAPIPE_LINEAR || kind == BAPIPE_LSTM; }

GatherConv fwd_geom(const bapipe_stage *st, const Layer &L)
{
    const Tensor &A = st->tensors[L.a], &O = st->tensors[L.o];
    GatherConv g;
    g.N = st->mb;
    if (L.d.kind == BAPIPE_LINEAR) {
        g.Hi = g.Wi = g.Ho = g.Wo = 1;
        g.Ci = L.d.cin;
        g.Co = L.d.cout;
        g.R = g.S = 1;
        g.s_out = g.s_in = 1;
        g.pad_h = g.pad_w = 0;
        return g;
    }
    g.Hi = A.H; g.Wi = A.W; g.Ci = A.Cp;
    g.Ho = O.H; g.Wo = O.W; g.Co = O.C;
    g.R = L.d.kh; g.S = L.d.kw;
    g.s_out = L.d.stride; g.s_in = 1;
    g.pad_h = g.pad_w = L.d.pad;
    return g;
}

GatherConv dgrad_geom(const bapipe_stage *st, const Layer &L)
{
    GatherConv f = fwd_geom(st, L), g;
    g.N = f.N;
    g.Hi = f.Ho; g.Wi = f.Wo; g.Ci = f.Co;
    g.Ho = f.Hi; g.Wo = f.Wi; g.Co = f.Ci;
    g.R = f.R; g.S = f.S;
    g.s_out = 1; g.s_in = f.s_out;
    g.pad_h = f.R - 1 - f.pad_h;
    g.pad_w = f.S - 1 - f.pad_w;
    return g;
}

ConvShape conv_shape(const bapipe_stage *st, const Layer &L)
{
    GatherConv f = fwd_geom(st, L);
    ConvShape c;
    c.N = f.N; c.H = f.Hi; c.W = f.Wi; c.C = f.Ci;
    c.P = f.Ho; c.Q = f.Wo; c.K = f.Co;
    c.R = f.R; c.S = f.S; c.stride = f.s_out; c.pad = f.pad_h;
    return c;
}

double conv_flop(const GatherConv &f, int logical_ci)
{
    return 2.0 * (double)f.N * f.Ho * f.Wo * f.Co * f.R * f.S * logical_ci;
}

bool use_mfma_gather(const bapipe_stage *st, const GatherConv &g) { return st->dt == DT_BF16 && conv_gather_mfma_supported(g); }
bool use_mfma_wgrad(const bapipe_stage *st, const ConvShape &c) { return st->dt == DT_BF16 && conv_wgrad_mfma_supported(c); }

#define HIPCHK(call)                                                                   \
    do {                                                                               \
        hipError_t e_ = (call);                                                        \
        if (e_ != hipSuccess) return st->fail(BAPIPE_E_DEVICE, "%s: %s", #call, hipGetErrorString(e_)); \
    } while (0)

// OIHW (or [out][in] with NCHW-flattened in) host weights <-> internal [K][R][S][C]
void to_internal(const Layer &L, const float *src, float *dst)
{
    const int K = L.d.cout;
    if (L.d.kind == BAPIPE_LSTM) {       // [4H][In+H] rows -> the input block [4H][In], then the recurrent block [4H][H]
        const int In = L.d.cin, H = L.d.cout, G = 4 * H;
        for (int k = 0; k < G; ++k) {
            memcpy(dst + (size_t)k * In, src + (size_t)k * (In + H), sizeof(float) * In);
            memcpy(dst + (size_t)G * In + (size_t)k * H, src + (size_t)k * (In + H) + In, sizeof(float) * H);
        }
        return;
    }
    if (L.d.kind == BAPIPE_LINEAR) {
        const int In = L.d.cin;
        if (!L.permute_in) {
            memcpy(dst, src, sizeof(float) * (size_t)K * In);
            return;
        }
        for (int k = 0; k < K; ++k)
            for (int c = 0; c < L.pc; ++c)
                for (int h = 0; h < L.ph; ++h)
                    for (int w = 0; w < L.pw; ++w)
                        dst[(size_t)k * In + ((size_t)h * L.pw + w) * L.pc + c] =
                            src[(size_t)k * In + ((size_t)c * L.ph + h) * L.pw + w];
        return;
    }
    const int C = L.d.cin, Cp = L.cin_p, R = L.d.kh, S = L.d.kw;
    memset(dst, 0, sizeof(float) * L.w_elems);
    for (int k = 0; k < K; ++k)
        for (int c = 0; c < C; ++c)
            for (int r = 0; r < R; ++r)
                for (int s = 0; s < S; ++s)
                    dst[(((size_t)k * R + r) * S + s) * Cp + c] = src[(((size_t)k * C + c) * R + r) * S + s];
}

void from_internal(const Layer &L, const float *src, float *dst)
{
    const int K = L.d.cout;
    if (L.d.kind == BAPIPE_LSTM) {
        const int In = L.d.cin, H = L.d.cout, G = 4 * H;
        for (int k = 0; k < G; ++k) {
            memcpy(dst + (size_t)k * (In + H), src + (size_t)k * In, sizeof(float) * In);
            memcpy(dst + (size_t)k * (In + H) + In, src + (size_t)G * In + (size_t)k * H, sizeof(float) * H);
        }
        return;
    }
    if (L.d.kind == BAPIPE_LINEAR) {
        const int In = L.d.cin;
        if (!L.permute_in) {
            memcpy(dst, src, sizeof(float) * (size_t)K * In);
            return;
        }
        for (int k = 0; k < K; ++k)
            for (int c = 0; c < L.pc; ++c)
                for (int h = 0; h < L.ph; ++h)
                    for (int w = 0; w < L.pw; ++w)
                        dst[(size_t)k * In + ((size_t)c * L.ph + h) * L.pw + w] =
                            src[(size_t)k * In + ((size_t)h * L.pw + w) * L.pc + c];
        return;
    }
    const int C = L.d.cin, Cp = L.cin_p, R = L.d.kh, S = L.d.kw;
    for (int k = 0; k < K; ++k)
        for (int c = 0; c < C; ++c)
            for (int r = 0; r < R; ++r)
                for (int s = 0; s < S; ++s)
                    dst[(((size_t)k * C + c) * R + r) * S + s] = src[(((size_t)k * R + r) * S + s) * Cp + c];
}

// working copies of one layer's weights from its fp32 master
// channel-transposed (and flipped) copy of the master weights that the input-gradient GEMMs read
hipError_t refresh_transposed(bapipe_stage *st, Layer &L)
{
    if (L.d.kind == BAPIPE_LSTM) {       // [In][4H] for dx, then [H][4H] for the recurrent gradient
        const int In = L.d.cin, H = L.d.cout, G = 4 * H;
        const size_t es = dt_size(st->dt);
        hipError_t e = make_dgrad_filter(st->dt, L.w, L.w_t, G, 1, 1, In, st->stream);
        if (e != hipSuccess) return e;
        return make_dgrad_filter(st->dt, L.w + (size_t)G * In, (char *)L.w_t + (size_t)G * In * es, G, 1, 1, H, st->stream);
    }
    int R = L.d.kind == BAPIPE_LINEAR ? 1 : L.d.kh, S = L.d.kind == BAPIPE_LINEAR ? 1 : L.d.kw;
    return make_dgrad_filter(st->dt, L.w, L.w_t, L.d.cout, R, S, L.cin_p, st->stream);
}

hipError_t refresh_work(bapipe_stage *st, Layer &L)
{
    if (!has_matrix(L.d.kind)) return hipSuccess;
    hipError_t e = recast(st->dt, L.w, L.w_work, L.w_elems, st->stream);
    if (e != hipSuccess) return e;
    return refresh_transposed(st, L);
}

// ---------------------------------------------------------------- LSTM layer (sequence axis = H, W = 1)
// GEMM over all N*T rows of a [N][T][ci] tensor: out[row][co] = sum in[row][ci] * wt[co][ci]
GatherConv rows_geom(int N, int T, int ci, int co)
{
    GatherConv g;
    g.N = N; g.Hi = T; g.Wi = 1; g.Ci = ci;
    g.Ho = T; g.Wo = 1; g.Co = co;
    g.R = g.S = 1; g.s_out = g.s_in = 1; g.pad_h = g.pad_w = 0;
    return g;
}
// the same product restricted to the rows (n, t) of every sequence: one output row per sequence
GatherConv step_geom(int N, int T, int ci, int co, int t)
{
    GatherConv g = rows_geom(N, T, ci, co);
    g.Ho = 1;
    g.pad_h = -t;                      // output row 0 reads input row t
    return g;
}

// fp32 sums of one recurrent product: *S partial results [S][N][co] in the workspace
int step_product(bapipe_stage *st, const void *in, const void *wt, const GatherConv &g, int *S)
{
    if (st->dt == DT_BF16) {
        HIPCHK(conv_gather_mfma_raw(in, wt, g, (float *)st->work, S, st->stream));
    } else {
        GradEpi none{nullptr, 0};
        HIPCHK(conv_gather_direct(st->dt, in, wt, nullptr, st->work, 0, none, g, st->stream));
        *S = 1;
    }
    return BAPIPE_OK;
}

int lstm_forward(bapipe_stage *st, Layer &L, const void *x, void *h, int mbid)
{
    const Tensor &A = st->tensors[L.a];
    const int N = st->mb, T = A.H, In = A.Cp, H = L.d.cout, G = 4 * H;
    hipStream_t s = st->stream;
    char *slot = st->slot(mbid);
    void *P = slot + L.off_pd, *hs = slot + L.off_hs;
    float *gates = (float *)(slot + L.off_gates), *cells = (float *)(slot + L.off_cells);
    const char *w_hh = (const char *)L.w_work + (size_t)G * In * dt_size(st->dt);
    GradEpi none{nullptr, 0};
    const GatherConv gx = rows_geom(N, T, In, G);
    const bool tp = st->tap_begin(st->dt == DT_BF16 ? BAPIPE_KC_CONV_GATHER_MFMA : BAPIPE_KC_CONV_DIRECT);
    if (st->dt == DT_BF16)
        HIPCHK(conv_gather_mfma(x, L.w_work, L.bias, P, 0, none, gx, st->work, s));
    else
        HIPCHK(conv_gather_direct(st->dt, x, L.w_work, L.bias, P, 0, none, gx, s));
    for (int t = 0; t < T; ++t) {
        int S = 0;
        if (t > 0) {                                   // W_h h_{t-1}: row t of the delayed copy
            int rc = step_product(st, hs, w_hh, step_geom(N, T, H, G, t), &S);
            if (rc != BAPIPE_OK) return rc;
        }
        HIPCHK(lstm_cell_fwd(st->dt, P, (const float *)st->work, S, gates, cells, h, hs, N, T, H, t, s));
    }
    // x and W_x once, W_h once per step, P written and read, h written
    st->tap_end(tp, 2.0 * N * T * (double)G * (L.d.cin + H),
                dt_size(st->dt) * ((double)N * T * (In + 2.0 * G + H) + (double)G * In + (double)(T - 1) * G * H));
    return BAPIPE_OK;
}

// dy: gradient of the layer output [N][T][H]; dx (may be NULL) receives W_x^T D through the epilogue e
int lstm_backward(bapipe_stage *st, Layer &L, const void *x, const void *dy, void *dx, GradEpi e, int mbid)
{
    const Tensor &A = st->tensors[L.a];
    const int N = st->mb, T = A.H, In = A.Cp, H = L.d.cout, G = 4 * H;
    const size_t es = dt_size(st->dt);
    hipStream_t s = st->stream;
    char *slot = st->slot(mbid);
    void *D = slot + L.off_pd;
    const void *hs = slot + L.off_hs;
    const float *gates = (const float *)(slot + L.off_gates), *cells = (const float *)(slot + L.off_cells);
    float *dcn = (float *)(slot + L.off_dcn);
    const char *wt_x = (const char *)L.w_t, *wt_h = wt_x + (size_t)G * In * es;
    const bool mf = st->dt == DT_BF16;
    bool tp = st->tap_begin(mf ? BAPIPE_KC_CONV_GATHER_MFMA : BAPIPE_KC_CONV_DIRECT);
    for (int t = T - 1; t >= 0; --t) {
        int S = 0;
        if (t + 1 < T) {                               // W_h^T D_{t+1}
            int rc = step_product(st, D, wt_h, step_geom(N, T, G, H, t + 1), &S);
            if (rc != BAPIPE_OK) return rc;
        }
        HIPCHK(lstm_cell_bwd(st->dt, dy, (const float *)st->work, S, gates, cells, dcn, D, N, T, H, t, s));
    }
    double flop = 2.0 * N * (T - 1) * (double)G * H;
    if (dx) {
        const GatherConv gd = rows_geom(N, T, G, In);
        if (mf)
            HIPCHK(conv_gather_mfma(D, wt_x, nullptr, dx, 0, e, gd, st->work, s));
        else
            HIPCHK(conv_gather_direct(st->dt, D, wt_x, nullptr, dx, 0, e, gd, s));
        flop += 2.0 * N * T * (double)G * L.d.cin;
    }
    st->tap_end(tp, flop, dt_size(st->dt) * ((double)N * T * (H + 2.0 * G + (dx ? In : 0)) + (double)G * In +
                                             (double)(T - 1) * G * H));
    // dW_x += D^T x (the bias gradient rides along), dW_h += D^T (delayed h)
    ConvShape cx{N, T, 1, In, T, 1, G, 1, 1, 1, 0}, ch{N, T, 1, H, T, 1, G, 1, 1, 1, 0};
    float *dw_h = L.dw + (size_t)G * In;
    tp = st->tap_begin(mf ? BAPIPE_KC_CONV_WGRAD_MFMA : BAPIPE_KC_CONV_DIRECT);
    if (mf) {
        HIPCHK(conv_wgrad_mfma(x, D, L.dw, L.db, st->work, cx, s));
        HIPCHK(conv_wgrad_mfma(hs, D, dw_h, nullptr, st->work, ch, s));
    } else {
        HIPCHK(conv_wgrad_direct(st->dt, x, D, L.dw, st->work, cx, s));
        HIPCHK(conv_wgrad_direct(st->dt, hs, D, dw_h, st->work, ch, s));
        if (L.db) HIPCHK(colsum_accumulate(st->dt, D, N * T, G, L.db, st->work, s));
    }
    st->tap_end(tp, 2.0 * N * T * (double)G * (L.d.cin + H),
                dt_size(st->dt) * (double)N * T * (In + H + 2.0 * G) + 8.0 * L.w_elems);
    return BAPIPE_OK;
}

// ---------------------------------------------------------------- per-layer forward
// xin: pointer used for tensor 0 when it is not stashed (caller's NHWC buffer)
struct FwdCtx {
    int mbid;
    const void *x_direct;
    bool profiling = false;      // layers are timed one at a time: nothing may rely on what the previous layer left behind
};

const void *in_ptr(bapipe_stage *st, int t, const FwdCtx &c)
{
    int r = st->tensors[t].root;
    if (r == 0 && c.x_direct) return c.x_direct;
    return st->tptr(t, c.mbid);
}

int layer_forward(bapipe_stage *st, int li, const FwdCtx &c)
{
    Layer &L = st->layers[li];
    const Tensor &O = st->tensors[L.o];
    const void *a = in_ptr(st, L.a, c);
    void *o = st->tptr(L.o, c.mbid);
    hipStream_t s = st->stream;
    const int dt = st->dt;
    switch (L.d.kind) {
    case BAPIPE_CONV2D:
    case BAPIPE_LINEAR: {
        GatherConv g = fwd_geom(st, L);
        // the number of statistics chunks a conv leaves for its batch-norm was fixed at creation: same plan here
        g.beside = st->stream_b && !c.profiling && !L.stat_chunks;
        GradEpi none{nullptr, 0};
        const bool mf = use_mfma_gather(st, g);
        const bool tp = st->tap_begin(mf ? BAPIPE_KC_CONV_GATHER_MFMA : BAPIPE_KC_CONV_DIRECT);
        if (L.fuse_pool >= 0) {
            const Layer &P = st->layers[L.fuse_pool];
            HIPCHK(conv3x3_halo_pool_mfma(a, L.w_work, L.bias, L.d.fuse_relu, st->tptr(P.o, c.mbid),
                                          (uint8_t *)(st->slot(c.mbid) + P.aux_off), g, s));
        } else if (mf)
            HIPCHK(conv_gather_mfma(a, L.w_work, L.bias, o, L.d.fuse_relu, none, g, st->work, s,
                                    (L.stat_chunks && !c.profiling) ? (float *)st->work : nullptr));
        else
            HIPCHK(conv_gather_direct(dt, a, L.w_work, L.bias, o, L.d.fuse_relu, none, g, s));
        // algorithmic bytes: input and filter read once, output (or pooled output + indices) written once
        const double wbytes = (double)L.w_elems * dt_size(dt);
        const double obytes = L.fuse_pool >= 0 ? (double)st->tensors[st->layers[L.fuse_pool].o].bytes() +
                                                     (double)st->tensors[st->layers[L.fuse_pool].o].elems
                                               : (double)O.bytes();
        st->tap_end(tp, conv_flop(g, L.d.cin), (double)st->tensors[L.a].bytes() + wbytes + obytes);
        break;
    }
    case BAPIPE_RELU: {
        const bool tp = st->tap_begin(BAPIPE_KC_ELEMENTWISE);
        HIPCHK(relu_fwd(dt, a, o, O.elems, s));
        st->tap_end(tp, 0.0, 2.0 * O.bytes());
        break;
    }
    case BAPIPE_MAXPOOL2D: {
        if (L.fused) break;                       // done in the producing conv's epilogue
        const Tensor &A = st->tensors[L.a];
        const bool tp = st->tap_begin(BAPIPE_KC_POOL);
        HIPCHK(maxpool_fwd(dt, a, o, (uint8_t *)(st->slot(c.mbid) + L.aux_off), st->mb, A.H, A.W, A.C, L.d.kh, L.d.kw,
                           L.d.stride, L.d.pad, s));
        st->tap_end(tp, 0.0, (double)A.bytes() + O.bytes() + O.elems);           // read x, write y + idx
        break;
    }
    case BAPIPE_AVGPOOL2D: {
        const Tensor &A = st->tensors[L.a];
        const bool tp = st->tap_begin(BAPIPE_KC_POOL);
        HIPCHK(avgpool_fwd(dt, a, o, st->mb, A.H, A.W, A.C, L.d.kh, L.d.kw, s));
        st->tap_end(tp, 0.0, (double)A.bytes() + O.bytes());
        break;
    }
    case BAPIPE_BATCHNORM2D: {
        const Tensor &A = st->tensors[L.a];
        const bool tp = st->tap_begin(BAPIPE_KC_BATCHNORM);
        // the partials of the producing conv are only there when that conv has just run (not when the
        // profiler times this layer alone)
        const int pre = (L.stats_given && !c.profiling) ? st->layers[li - 1].stat_chunks : 0;
        if (L.fuse_add >= 0) {                       // y of the ADD behind this layer, in the same pass
            const Layer &S = st->layers[L.fuse_add];
            const void *other = in_ptr(st, S.a == L.o ? S.b : S.a, c);
            HIPCHK(bn_fwd(dt, a, L.w, L.bias, L.d.eps, st->tptr(S.o, c.mbid), (float *)(st->slot(c.mbid) + L.aux_off), 0,
                          st->mb * A.H * A.W, A.C, st->work, s, pre, other, S.d.fuse_relu));
            st->tap_end(tp, 0.0, 4.0 * A.bytes());                               // x twice, the other summand, y
            break;
        }
        HIPCHK(bn_fwd(dt, a, L.w, L.bias, L.d.eps, o, (float *)(st->slot(c.mbid) + L.aux_off), L.d.fuse_relu,
                      st->mb * A.H * A.W, A.C, st->work, s, pre));
        st->tap_end(tp, 0.0, 3.0 * A.bytes());                                   // read x twice, write y
        break;
    }
    case BAPIPE_ADD: {
        if (L.fused) break;                       // stored by the batch-norm that feeds it
        const bool tp = st->tap_begin(BAPIPE_KC_ELEMENTWISE);
        HIPCHK(add_fwd(dt, a, in_ptr(st, L.b, c), o, L.d.fuse_relu, O.elems, s));
        st->tap_end(tp, 0.0, 3.0 * O.bytes());
        break;
    }
    case BAPIPE_FLATTEN:
        break;   // alias of its input
    case BAPIPE_LSTM: {
        int rc = lstm_forward(st, L, a, o, c.mbid);
        if (rc != BAPIPE_OK) return rc;
        break;
    }
    case BAPIPE_SOFTMAX_XENT:
        HIPCHK(softmax_fwd(dt, a, (float *)o, st->mb, O.C, s));
        break;
    default:
        return st->fail(BAPIPE_E_UNSUPPORTED, "layer %d: kind %d", li, L.d.kind);
    }
    return BAPIPE_OK;
}

// ---------------------------------------------------------------- per-layer backward
struct BwdCtx {
    int mbid;
    const void *x_direct;          // unused in backward (stage input is stashed when needed)
    const void *dy_direct;         // caller's NHWC gradient used in place of grads[last]
    void *dx_direct;               // caller's NHWC buffer used in place of grads[0]
    const int32_t *labels;
    std::vector<char> written;
    std::vector<const void *> pending;   // per tensor: an ADD's share of its gradient that the tensor's conv will add (fanout_conv)
    bool profiling = false;        // profiler: run every kernel of the layer now (no deferral)
    int bn_sums_ready = -1;        // batch-norm layer whose backward sums the last conv left in the workspace
};

void *grad_ptr(bapipe_stage *st, int t, BwdCtx &c)
{
    int r = st->tensors[t].root;
    if (st->tensors[r].galias >= 0) return grad_ptr(st, st->tensors[r].galias, c);
    if (r == 0 && c.dx_direct) return c.dx_direct;
    if (r == st->tensors[(int)st->tensors.size() - 1].root && c.dy_direct) return const_cast<void *>(c.dy_direct);
    if (st->tensors[r].gmb_store) return st->tensors[r].gmb_store + (size_t)c.mbid * st->tensors[r].bytes();
    return st->gptr(t);
}

// epilogue for a write into the gradient of tensor t; pool_gate_t >= 0: the writer is a max-pool
// whose own output (tensor pool_gate_t) carries the same sign information per window
GradEpi epi_for(bapipe_stage *st, int t, BwdCtx &c, int pool_gate_t = -1)
{
    int r = st->tensors[t].root;
    GradEpi e{nullptr, 0};
    if (st->tensors[r].gated) e.gate = st->tptr(pool_gate_t >= 0 ? pool_gate_t : r, c.mbid);
    e.accum = c.written[r] ? 1 : 0;
    c.written[r] = 1;
    return e;
}

int layer_backward(bapipe_stage *st, int li, BwdCtx &c)
{
    Layer &L = st->layers[li];
    const Tensor &A = st->tensors[L.a];
    const Tensor &O = st->tensors[L.o];
    hipStream_t s = st->stream;
    const int dt = st->dt;
    const bool a_grad = st->tensors[A.root].need_grad;
    switch (L.d.kind) {
    case BAPIPE_CONV2D:
    case BAPIPE_LINEAR: {
        const void *g = grad_ptr(st, L.o, c);
        const void *x = st->tptr(L.a, c.mbid);
        ConvShape cs = conv_shape(st, L);
        const double flop = conv_flop(fwd_geom(st, L), L.d.cin);
        bool bias_done = false;
        if (L.deferred && !c.profiling) {
            // nothing to copy where the tensor already lives in the layer's buffer
            char *xk = L.def_x + (size_t)c.mbid * L.def_x_bytes, *gk = L.def_g + (size_t)c.mbid * L.def_g_bytes;
            if (x != xk) HIPCHK(hipMemcpyAsync(xk, x, L.def_x_bytes, hipMemcpyDeviceToDevice, s));
            if (g != gk) HIPCHK(hipMemcpyAsync(gk, g, L.def_g_bytes, hipMemcpyDeviceToDevice, s));
            bias_done = true;                             // the column sums of dy ride along in the deferred GEMM
        } else {
            const bool mf = use_mfma_wgrad(st, cs);
            // a layer without an input gradient ends the pass's kernel chain: its weight gradient would only delay
            // the end of the pass from the other stream
            const bool side = mf && st->stream_w && !c.profiling && a_grad;
            hipStream_t ws = s;
            char *wwork = st->work;
            if (side) {                                   // g is complete on the backward stream at this point
                HIPCHK(hipEventRecord(st->ev_g, s));
                HIPCHK(hipStreamWaitEvent(st->stream_w, st->ev_g, 0));
                ws = st->stream_w;
                wwork = st->work_w;
                st->w_used = true;
            }
            const bool tp = st->tap_begin(mf ? BAPIPE_KC_CONV_WGRAD_MFMA : BAPIPE_KC_CONV_DIRECT, ws);
            if (mf)
                HIPCHK(conv_wgrad_mfma(x, g, L.dw, L.db, wwork, cs, ws));      // bias gradient rides along
            else
                HIPCHK(conv_wgrad_direct(dt, x, g, L.dw, st->work, cs, s));
            st->tap_end(tp, flop, (double)A.bytes() + O.bytes() + 8.0 * L.w_elems);   // x, dy read; fp32 dw read and written
            bias_done = mf;
        }
        if (L.db && !bias_done) {
            const bool tp = st->tap_begin(BAPIPE_KC_ELEMENTWISE);
            HIPCHK(colsum_accumulate(dt, g, cs.N * cs.P * cs.Q, cs.K, L.db, st->work, s));
            st->tap_end(tp, 0.0, (double)O.bytes());
        }
        if (a_grad) {
            GatherConv dg = dgrad_geom(st, L);
            dg.beside = st->stream_b && !c.profiling && !L.bnb_chunks && !L.strided_1x1;
            GradEpi e = epi_for(st, L.a, c);
            if (c.pending[A.root]) {                      // the residual ADD's share, added here instead of copied there
                e.accum_from = c.pending[A.root];
                c.pending[A.root] = nullptr;
            }
            void *dx = grad_ptr(st, L.a, c);
            const bool mf = use_mfma_gather(st, dg);
            const bool tp = st->tap_begin(mf ? BAPIPE_KC_CONV_GATHER_MFMA : BAPIPE_KC_CONV_DIRECT);
            if (mf && L.strided_1x1) {
                GatherConv dense = dg;                       // dy as the image, one output pixel per dy pixel
                dense.Ho = dg.Hi; dense.Wo = dg.Wi; dense.s_in = 1;
                GradEpi none{nullptr, 0};
                void *tmp = st->work + L.up_off;
                HIPCHK(conv_gather_mfma(g, L.w_t, nullptr, tmp, 0, none, dense, st->work, s));
                HIPCHK(upsample_grad(dt, tmp, dx, e, dg.N, dg.Ho, dg.Wo, dg.Hi, dg.Wi, dg.Co, L.d.stride, s));
            } else if (mf && L.bnb_chunks && !c.profiling && (e.gate || e.accum)) {
                const Layer &B = st->layers[li - 1];
                HIPCHK(conv_gather_mfma(g, L.w_t, nullptr, dx, 0, e, dg, st->work, s, (float *)st->work,
                                        st->tptr(B.a, c.mbid), (const float *)(st->slot(c.mbid) + B.aux_off)));
                c.bn_sums_ready = li - 1;
            } else if (mf)
                HIPCHK(conv_gather_mfma(g, L.w_t, nullptr, dx, 0, e, dg, st->work, s));
            else
                HIPCHK(conv_gather_direct(dt, g, L.w_t, nullptr, dx, 0, e, dg, s));
            // dy and filter read, dx written, plus the gate and the previous dx where the epilogue uses them
            st->tap_end(tp, flop, (double)O.bytes() + (double)L.w_elems * dt_size(dt) +
                                      (double)A.bytes() * (1.0 + (e.gate ? 1.0 : 0.0) + (e.accum ? 1.0 : 0.0)));
        }
        break;
    }
    case BAPIPE_RELU:
        if (a_grad) {
            GradEpi e = epi_for(st, L.a, c);
            const bool tp = st->tap_begin(BAPIPE_KC_ELEMENTWISE);
            HIPCHK(relu_bwd(dt, st->tptr(L.o, c.mbid), grad_ptr(st, L.o, c), grad_ptr(st, L.a, c), e, O.elems, s));
            st->tap_end(tp, 0.0, 3.0 * O.bytes());
        }
        break;
    case BAPIPE_MAXPOOL2D:
        if (a_grad) {
            GradEpi e = epi_for(st, L.a, c, L.o);
            const bool tp = st->tap_begin(BAPIPE_KC_POOL);
            HIPCHK(maxpool_bwd(dt, grad_ptr(st, L.o, c), (const uint8_t *)(st->slot(c.mbid) + L.aux_off),
                               grad_ptr(st, L.a, c), e, st->mb, A.H, A.W, A.C, L.d.kh, L.d.kw, L.d.stride, L.d.pad, s));
            st->tap_end(tp, 0.0, (double)O.bytes() + O.elems + A.bytes() + (e.gate ? O.bytes() : 0));
        }
        break;
    case BAPIPE_AVGPOOL2D:
        if (a_grad) {
            GradEpi e = epi_for(st, L.a, c);
            const bool tp = st->tap_begin(BAPIPE_KC_POOL);
            HIPCHK(avgpool_bwd(dt, grad_ptr(st, L.o, c), grad_ptr(st, L.a, c), e, st->mb, A.H, A.W, A.C, L.d.kh, L.d.kw, s));
            st->tap_end(tp, 0.0, (double)O.bytes() + A.bytes() * (e.gate ? 2.0 : 1.0));
        }
        break;
    case BAPIPE_BATCHNORM2D: {
        GradEpi e{nullptr, 0};
        void *dx = nullptr;
        if (a_grad) {
            e = epi_for(st, L.a, c);
            dx = grad_ptr(st, L.a, c);
        }
        const bool tp = st->tap_begin(BAPIPE_KC_BATCHNORM);
        const int pre = (L.bwd_sums_given && c.bn_sums_ready == li) ? st->layers[li + 1].bnb_chunks : 0;
        HIPCHK(bn_bwd(dt, st->tptr(L.a, c.mbid), grad_ptr(st, L.o, c), L.w,
                      (const float *)(st->slot(c.mbid) + L.aux_off), dx, L.dw, L.db, e, st->mb * A.H * A.W, A.C,
                      st->work, s, pre));
        st->tap_end(tp, 0.0, 5.0 * A.bytes());                                   // x, dy twice each; dx once
        break;
    }
    case BAPIPE_ADD: {
        const void *g = grad_ptr(st, L.o, c);
        const bool tp = st->tap_begin(BAPIPE_KC_ELEMENTWISE);
        double bytes = 0.0;
        if (a_grad && st->tensors[A.root].galias == L.o) {
            c.written[A.root] = 1;
        } else if (a_grad && st->tensors[A.root].fanout_conv >= 0 && !c.profiling && !c.written[A.root]) {
            c.pending[A.root] = g;                        // taken by that conv's input-gradient epilogue
            c.written[A.root] = 1;
        } else if (a_grad) {
            GradEpi e = epi_for(st, L.a, c);
            HIPCHK(grad_copy(dt, g, grad_ptr(st, L.a, c), e, O.elems, s));
            bytes += 2.0 * O.bytes();
        }
        const int rb = st->tensors[L.b].root;
        if (st->tensors[rb].need_grad && st->tensors[rb].galias == L.o) {
            c.written[rb] = 1;
        } else if (st->tensors[rb].need_grad && st->tensors[rb].fanout_conv >= 0 && !c.profiling && !c.written[rb]) {
            c.pending[rb] = g;
            c.written[rb] = 1;
        } else if (st->tensors[rb].need_grad) {
            GradEpi e = epi_for(st, L.b, c);
            HIPCHK(grad_copy(dt, g, grad_ptr(st, L.b, c), e, O.elems, s));
            bytes += 2.0 * O.bytes();
        }
        st->tap_end(tp, 0.0, bytes);
        break;
    }
    case BAPIPE_FLATTEN:
        break;
    case BAPIPE_LSTM: {
        GradEpi e{nullptr, 0};
        void *dx = nullptr;
        if (a_grad) {
            e = epi_for(st, L.a, c);
            dx = grad_ptr(st, L.a, c);
        }
        int rc = lstm_backward(st, L, st->tptr(L.a, c.mbid), grad_ptr(st, L.o, c), dx, e, c.mbid);
        if (rc != BAPIPE_OK) return rc;
        break;
    }
    case BAPIPE_SOFTMAX_XENT:
        if (a_grad) {
            c.written[A.root] = 1;
            HIPCHK(xent_bwd(dt, (const float *)st->tptr(L.o, c.mbid), c.labels, st->loss_scale,
                            grad_ptr(st, L.a, c), st->losses + c.mbid, st->mb, O.C, s));
        }
        break;
    default:
        return st->fail(BAPIPE_E_UNSUPPORTED, "layer %d: kind %d", li, L.d.kind);
    }
    return BAPIPE_OK;
}

// weight gradients of the deferred layers for micro-batches [flushed, n_bwd): one GEMM per layer
int flush_deferred(bapipe_stage *st)
{
    const int n = st->n_bwd - st->flushed;
    if (n <= 0) return BAPIPE_OK;
    // the copies these GEMMs read were enqueued by the backward passes, possibly on their own stream
    if (st->stream_b) HIPCHK(hipStreamWaitEvent(st->stream, st->ev_bwd[st->n_bwd - 1], 0));
    for (auto &L : st->layers) {
        if (!L.deferred) continue;
        ConvShape cs = conv_shape(st, L);
        cs.N = st->mb * n;
        const char *x = L.def_x + (size_t)st->flushed * L.def_x_bytes;
        const char *g = L.def_g + (size_t)st->flushed * L.def_g_bytes;
        const bool tp = st->tap_begin(BAPIPE_KC_CONV_WGRAD_MFMA);
        HIPCHK(conv_wgrad_mfma(x, g, L.dw, L.db, st->work, cs, st->stream));
        st->tap_end(tp, conv_flop(fwd_geom(st, L), L.d.cin) * n, (double)n * (L.def_x_bytes + L.def_g_bytes) + 8.0 * L.w_elems);
    }
    st->flushed = st->n_bwd;
    return BAPIPE_OK;
}

}  // namespace

// ---------------------------------------------------------------- statically allocated workspace
// Workspace of bapipe_stage_backward_static: lives in the code object, one copy per GPU that loads the
// library, held until the process ends.  `scratch` itself is only a host-side stand-in for the symbol;
// the device address of each GPU's copy comes from hipGetSymbolAddress, once per device, and only that
// pointer is ever handed to a kernel.
static __device__ __align__(256) unsigned char scratch[BAPIPE_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
char *g_scratch_ptr[kMaxDevices] = {};

// device address of the current device's copy of `scratch` (looked up on the first call per device)
hipError_t static_scratch(char **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        g_scratch_ptr[dev] = (char *)p;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace

// ======================================================================== C ABI
extern "C" {

const char *bapipe_last_error(const bapipe_stage_t *st) { return st ? st->err.c_str() : g_create_error.c_str(); }

void bapipe_stage_destroy(bapipe_stage_t *st)
{
    if (!st) return;
    (void)hipStreamSynchronize(st->stream);                              // the caller's streams: drained, not destroyed
    if (st->stream_b) (void)hipStreamSynchronize(st->stream_b);
    if (st->stream_w) (void)hipStreamSynchronize(st->stream_w);
    for (hipEvent_t e : st->ev_fwd) if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : st->ev_bwd) if (e) (void)hipEventDestroy(e);
    st->dev_free(st->work_b);
    if (st->ev_g) (void)hipEventDestroy(st->ev_g);
    if (st->ev_w_end) (void)hipEventDestroy(st->ev_w_end);
    st->dev_free(st->work_w);
    st->dev_free(st->params);
    st->dev_free(st->stash);
    st->dev_free(st->transient);
    st->dev_free(st->grads);
    st->dev_free(st->work);
    st->dev_free(st->losses);
    st->dev_free(st->deferred);
    for (hipEvent_t e : st->tap_events) (void)hipEventDestroy(e);
    delete st;
}

int bapipe_stage_create(const bapipe_layer_desc_t *layers, int n_layers, int micro_batch, int n_micro,
                        const bapipe_stage_opts_t *opts, bapipe_stage_t **out)
{
    if (!layers || !opts || !out) return create_fail(BAPIPE_E_INVALID, "NULL argument");
    if (n_layers <= 0 || micro_batch <= 0 || n_micro <= 0)
        return create_fail(BAPIPE_E_INVALID, "n_layers, micro_batch and n_micro must be positive");
    if (opts->dtype != BAPIPE_FP32 && opts->dtype != BAPIPE_BF16) return create_fail(BAPIPE_E_INVALID, "bad dtype");
    if (opts->io_layout != BAPIPE_NCHW && opts->io_layout != BAPIPE_NHWC)
        return create_fail(BAPIPE_E_INVALID, "bad io_layout");
    if (opts->schedule != BAPIPE_SCHED_1F1B && opts->schedule != BAPIPE_SCHED_1F1B_SO)
        return create_fail(BAPIPE_E_INVALID, "bad schedule");
    if (opts->n_stages < 1 || opts->stage_index < 1 || opts->stage_index > opts->n_stages)
        return create_fail(BAPIPE_E_INVALID, "need 1 <= stage_index <= n_stages");
    if (opts->in_c <= 0 || opts->in_h <= 0 || opts->in_w <= 0) return create_fail(BAPIPE_E_INVALID, "bad input shape");
    if ((opts->mem.alloc == nullptr) != (opts->mem.free == nullptr))
        return create_fail(BAPIPE_E_INVALID, "allocator needs both alloc and free");

    bapipe_stage *st = new bapipe_stage();
    struct Guard {
        bapipe_stage *s;
        ~Guard() { if (s) bapipe_stage_destroy(s); }
    } guard{st};
    st->opts = *opts;
    st->dt = opts->dtype == BAPIPE_FP32 ? DT_F32 : DT_BF16;
    st->mb = micro_batch;
    st->M = n_micro;
    st->stream = (hipStream_t)opts->hip_stream;
    int live = opts->n_stages - opts->stage_index + 1;           // Table I/II: (N-i+1) micro-batches
    if (opts->schedule == BAPIPE_SCHED_1F1B_SO) live *= 2;       // doubled warm-up (Table II)
    st->depth = live < n_micro ? live : n_micro;
    st->loss_scale = opts->loss_scale > 0.f ? opts->loss_scale : 1.0f / ((float)micro_batch * (float)n_micro);
    st->loss_valid.assign(n_micro, 0);
    const size_t es = dt_size(st->dt);

    // ---- shape inference
    st->tensors.resize(n_layers + 1);
    {
        Tensor &T = st->tensors[0];
        T.C = T.Cp = opts->in_c; T.H = opts->in_h; T.W = opts->in_w;
        // a bf16 stage input with a channel count that is not a multiple of 8 (e.g. RGB) is
        // zero-padded to 8 in HBM when only convolutions read it, so that they can take the MFMA path
        bool only_convs = true;
        for (int i = 0; i < n_layers; ++i)
            if ((layers[i].src0 == -1 && layers[i].kind != BAPIPE_CONV2D) ||
                (layers[i].kind == BAPIPE_ADD && layers[i].src1 == -1))
                only_convs = false;
        if (st->dt == DT_BF16 && T.C % 8 != 0 && only_convs) T.Cp = (T.C + 7) / 8 * 8;
        T.elems = (size_t)micro_batch * T.Cp * T.H * T.W;
        T.esize = es; T.root = 0; T.producer = -1;
    }
    st->layers.resize(n_layers);
    for (int i = 0; i < n_layers; ++i) {
        Layer &L = st->layers[i];
        L.d = layers[i];
        const bapipe_layer_desc_t &d = L.d;
        if (d.src0 < -1 || d.src0 >= i) return create_fail(BAPIPE_E_SHAPE, "layer %d: src0=%d must name an earlier layer or -1", i, d.src0);
        L.a = d.src0 + 1;
        L.o = i + 1;
        const Tensor A = st->tensors[L.a];
        Tensor &O = st->tensors[L.o];
        O.esize = es; O.root = L.o; O.producer = i;
        if (A.esize != es) return create_fail(BAPIPE_E_SHAPE, "layer %d: consumes the softmax output", i);
        switch (d.kind) {
        case BAPIPE_CONV2D: {
            if (d.kh <= 0 || d.kw <= 0 || d.stride <= 0 || d.pad < 0 || d.cin <= 0 || d.cout <= 0)
                return create_fail(BAPIPE_E_INVALID, "layer %d: bad conv parameters", i);
            if (d.kh != d.kw) return create_fail(BAPIPE_E_UNSUPPORTED, "layer %d: non-square filter", i);
            if (d.pad > d.kh - 1) return create_fail(BAPIPE_E_UNSUPPORTED, "layer %d: pad > k-1", i);
            if (A.C != d.cin) return create_fail(BAPIPE_E_SHAPE, "layer %d: cin=%d but input has %d channels", i, d.cin, A.C);
            int ho = (A.H + 2 * d.pad - d.kh) / d.stride + 1, wo = (A.W + 2 * d.pad - d.kw) / d.stride + 1;
            if (A.H + 2 * d.pad < d.kh || A.W + 2 * d.pad < d.kw || ho <= 0 || wo <= 0)
                return create_fail(BAPIPE_E_SHAPE, "layer %d: filter larger than padded input", i);
            O.C = d.cout; O.H = ho; O.W = wo;
            L.cin_p = A.Cp;
            L.w_elems = (size_t)d.cout * d.kh * d.kw * L.cin_p;
            L.b_elems = d.has_bias ? d.cout : 0;
            break;
        }
        case BAPIPE_LINEAR: {
            if (d.cin <= 0 || d.cout <= 0) return create_fail(BAPIPE_E_INVALID, "layer %d: bad linear parameters", i);
            if ((size_t)A.C * A.H * A.W != (size_t)d.cin)
                return create_fail(BAPIPE_E_SHAPE, "layer %d: cin=%d but input has %zu features", i, d.cin, (size_t)A.C * A.H * A.W);
            O.C = d.cout; O.H = O.W = 1;
            L.cin_p = d.cin;
            L.w_elems = (size_t)d.cout * d.cin;
            L.b_elems = d.has_bias ? d.cout : 0;
            const Tensor &R = st->tensors[A.root];
            if (R.H * R.W > 1) { L.permute_in = true; L.pc = R.C; L.ph = R.H; L.pw = R.W; }
            break;
        }
        case BAPIPE_LSTM: {
            if (d.cin <= 0 || d.cout <= 0) return create_fail(BAPIPE_E_INVALID, "layer %d: bad LSTM parameters", i);
            if (A.C != d.cin) return create_fail(BAPIPE_E_SHAPE, "layer %d: cin=%d but input has %d channels", i, d.cin, A.C);
            if (A.W != 1) return create_fail(BAPIPE_E_SHAPE, "layer %d: LSTM input must be (cin, T, 1)", i);
            if (A.Cp != A.C) return create_fail(BAPIPE_E_UNSUPPORTED, "layer %d: LSTM input with padded channels", i);
            if (opts->dtype == BAPIPE_BF16 && (d.cin % 8 || d.cout % 8))
                return create_fail(BAPIPE_E_UNSUPPORTED, "layer %d: bf16 LSTM needs cin and cout that are multiples of 8", i);
            O.C = d.cout; O.H = A.H; O.W = 1;
            L.cin_p = A.Cp;
            L.w_elems = (size_t)4 * d.cout * (d.cin + d.cout);
            L.b_elems = d.has_bias ? (size_t)4 * d.cout : 0;
            break;
        }
        case BAPIPE_RELU:
            O.C = A.C; O.H = A.H; O.W = A.W;
            break;
        case BAPIPE_MAXPOOL2D:
            if (d.kh <= 0 || d.kw <= 0 || d.stride <= 0 || d.pad < 0)
                return create_fail(BAPIPE_E_INVALID, "layer %d: bad pool parameters", i);
            if (d.kh * d.kw > 255) return create_fail(BAPIPE_E_UNSUPPORTED, "layer %d: pool window above 255 positions", i);
            if (d.pad >= d.kh || d.pad >= d.kw)           // a window must never lie wholly in the padding
                return create_fail(BAPIPE_E_UNSUPPORTED, "layer %d: pool padding must be smaller than the window", i);
            if (A.H + 2 * d.pad < d.kh || A.W + 2 * d.pad < d.kw)
                return create_fail(BAPIPE_E_SHAPE, "layer %d: pool input smaller than window", i);
            O.C = A.C;
            O.H = (A.H + 2 * d.pad - d.kh) / d.stride + 1;
            O.W = (A.W + 2 * d.pad - d.kw) / d.stride + 1;
            break;
        case BAPIPE_AVGPOOL2D:
            if (d.kh <= 0 || d.kw <= 0) return create_fail(BAPIPE_E_INVALID, "layer %d: bad pool parameters", i);
            if (d.kh != d.kw || d.stride != d.kh || d.pad != 0)
                return create_fail(BAPIPE_E_UNSUPPORTED, "layer %d: average pool needs a square window, stride = window, no padding", i);
            if (A.H < d.kh || A.W < d.kw) return create_fail(BAPIPE_E_SHAPE, "layer %d: pool input smaller than window", i);
            O.C = A.C; O.H = A.H / d.kh; O.W = A.W / d.kw;
            break;
        case BAPIPE_BATCHNORM2D:
            if (d.cin != A.C || d.cout != A.C) return create_fail(BAPIPE_E_SHAPE, "layer %d: batch-norm over %d channels, input has %d", i, d.cin, A.C);
            if (!(d.eps > 0.f)) return create_fail(BAPIPE_E_INVALID, "layer %d: eps must be positive", i);
            O.C = A.C; O.H = A.H; O.W = A.W;
            L.w_elems = A.C; L.b_elems = A.C;
            break;
        case BAPIPE_ADD: {
            if (d.src1 < -1 || d.src1 >= i) return create_fail(BAPIPE_E_SHAPE, "layer %d: src1=%d must name an earlier layer or -1", i, d.src1);
            L.b = d.src1 + 1;
            const Tensor &B = st->tensors[L.b];
            if (B.C != A.C || B.H != A.H || B.W != A.W) return create_fail(BAPIPE_E_SHAPE, "layer %d: add of different shapes", i);
            if (L.a == L.b) return create_fail(BAPIPE_E_UNSUPPORTED, "layer %d: add of a tensor with itself", i);
            O.C = A.C; O.H = A.H; O.W = A.W;
            break;
        }
        case BAPIPE_FLATTEN:
            O.C = A.C * A.H * A.W; O.H = O.W = 1;
            O.root = A.root;
            break;
        case BAPIPE_SOFTMAX_XENT:
            if (i != n_layers - 1) return create_fail(BAPIPE_E_SHAPE, "layer %d: softmax cross-entropy must be last", i);
            if (A.H * A.W != 1) return create_fail(BAPIPE_E_SHAPE, "layer %d: softmax needs a (K,1,1) input", i);
            O.C = A.C; O.H = O.W = 1;
            O.esize = sizeof(float);
            break;
        default:
            return create_fail(BAPIPE_E_INVALID, "layer %d: unknown kind %d", i, d.kind);
        }
        O.Cp = O.C;
        O.elems = (size_t)micro_batch * O.C * O.H * O.W;
        st->tensors[L.a].consumers.push_back(i);
        if (L.b >= 0) st->tensors[L.b].consumers.push_back(i);
    }
    const int nt = n_layers + 1, last_t = n_layers;
    // the MFMA kernels address their operands with 32-bit byte offsets; larger tensors have no tested kernel
    for (int t = 0; t < nt; ++t)
        if (st->tensors[t].bytes() >= ((size_t)1 << 31))
            return create_fail(BAPIPE_E_UNSUPPORTED, "%s: %zu bytes per micro-batch; tensors of 2 GiB or more are not supported",
                               t ? "a layer output" : "the stage input", st->tensors[t].bytes());
    for (int i = 0; i < n_layers; ++i)
        if (st->layers[i].w_elems * 4 >= ((size_t)1 << 31))
            return create_fail(BAPIPE_E_UNSUPPORTED, "layer %d: weight matrix of 2 GiB or more", i);
    for (int t = 1; t < nt - 1; ++t)
        if (st->tensors[t].consumers.empty())
            return create_fail(BAPIPE_E_SHAPE, "layer %d: output is never used", t - 1);

    // ---- what backward needs
    for (int t = 1; t < nt; ++t) {
        const Layer &P = st->layers[t - 1];
        Tensor &T = st->tensors[t];
        T.gated = (P.d.kind == BAPIPE_RELU) ||
                  (P.d.fuse_relu && (P.d.kind == BAPIPE_CONV2D || P.d.kind == BAPIPE_LINEAR ||
                                     P.d.kind == BAPIPE_BATCHNORM2D || P.d.kind == BAPIPE_ADD));
        if (P.d.kind == BAPIPE_FLATTEN) T.gated = false;
    }
    // gate of an aliased tensor is the gate of its root
    st->tensors[0].need_grad = opts->need_input_grad != 0;
    for (int t = 1; t < nt; ++t) {
        const Layer &P = st->layers[t - 1];
        bool ng = has_params(P.d.kind) || st->tensors[st->tensors[P.a].root].need_grad;
        if (P.b >= 0) ng = ng || st->tensors[st->tensors[P.b].root].need_grad;
        st->tensors[t].need_grad = ng;
    }
    auto root_of = [&](int t) { return st->tensors[t].root; };
    // gradient aliasing at ADD layers
    for (int i = 0; i < n_layers; ++i) {
        const Layer &L = st->layers[i];
        if (L.d.kind != BAPIPE_ADD) continue;
        for (int src : {L.a, L.b}) {
            Tensor &S = st->tensors[src];
            if (src != 0 && S.root == src && !S.gated && S.need_grad && S.consumers.size() == 1) S.galias = L.o;
        }
    }
    for (int i = 0; i < n_layers; ++i) {
        const Layer &L = st->layers[i];
        Tensor &RA = st->tensors[root_of(L.a)];
        switch (L.d.kind) {
        case BAPIPE_CONV2D: case BAPIPE_LINEAR: case BAPIPE_BATCHNORM2D: case BAPIPE_LSTM:
            RA.stashed = true;
            break;
        case BAPIPE_RELU: case BAPIPE_SOFTMAX_XENT:
            st->tensors[L.o].stashed = true;
            break;
        case BAPIPE_MAXPOOL2D:
            if (RA.gated && RA.need_grad) st->tensors[L.o].stashed = true;   // pooled values gate the window
            break;
        default:
            break;
        }
        // a gated tensor is read again by every non-pool layer that writes its gradient
        if (L.d.kind != BAPIPE_MAXPOOL2D && L.d.kind != BAPIPE_FLATTEN) {
            if (RA.gated && RA.need_grad) RA.stashed = true;
            if (L.b >= 0) {
                Tensor &RB = st->tensors[root_of(L.b)];
                if (RB.gated && RB.need_grad) RB.stashed = true;
            }
        }
    }
    if (st->tensors[root_of(last_t)].gated) st->tensors[root_of(last_t)].stashed = true;   // gates the caller's dy
    if (st->layers[n_layers - 1].d.kind == BAPIPE_SOFTMAX_XENT) {
        const Tensor &Z = st->tensors[root_of(st->layers[n_layers - 1].a)];
        if (Z.gated || Z.consumers.size() > 1)
            return create_fail(BAPIPE_E_UNSUPPORTED, "softmax input must be an un-gated tensor used only by the loss");
    }

    // ---- memory plan
    size_t slot = 0, trans = 0, gr = 0;
    for (int t = 0; t < nt; ++t) {
        Tensor &T = st->tensors[t];
        if (T.root != t) continue;
        if (T.stashed) { T.off = slot; slot += align_up(T.bytes()); }
        else { T.off = trans; trans += align_up(T.bytes()); }
        if (T.need_grad && t != last_t) { T.goff = gr; gr += align_up(T.bytes()); }
    }
    {   // gradient of the stage output (ingest target when the caller's dy cannot be used in place)
        Tensor &T = st->tensors[root_of(last_t)];
        if (st->layers[n_layers - 1].d.kind != BAPIPE_SOFTMAX_XENT && root_of(last_t) == last_t) { T.goff = gr; gr += align_up(T.bytes()); }
    }
    // conv -> max-pool fusion (bf16, halo kernel shapes): the conv output must be a transient tensor
    // read by that pool only
    for (int i = 0; i < n_layers; ++i) {
        Layer &L = st->layers[i];
        const Tensor &O = st->tensors[L.o];
        if (L.d.kind != BAPIPE_CONV2D || st->dt != DT_BF16 || L.o == last_t || O.stashed || O.consumers.size() != 1) continue;
        Layer &P = st->layers[O.consumers[0]];
        if (P.d.kind != BAPIPE_MAXPOOL2D || P.a != L.o) continue;
        if (P.d.kh != 2 || P.d.kw != 2 || P.d.stride != 2 || P.d.pad != 0) continue;
        if (!conv3x3_halo_supported(fwd_geom(st, L)) || (O.H & 1) || (O.W & 1)) continue;
        L.fuse_pool = O.consumers[0];
        P.fused = true;
    }
    // batch-norm -> residual ADD: where the later-produced summand is a batch-norm output (no ReLU of its own) that
    // only the ADD reads, that layer's normalisation pass stores the sum and the ADD launches nothing
    for (int i = 0; i < n_layers; ++i) {
        Layer &S = st->layers[i];
        if (S.d.kind != BAPIPE_ADD) continue;
        const int t = S.a > S.b ? S.a : S.b;                  // the summand produced last
        if (t == 0 || root_of(t) != t || root_of(S.a) != S.a || root_of(S.b) != S.b) continue;
        Layer &Bn = st->layers[t - 1];
        const Tensor &T = st->tensors[t];
        if (Bn.d.kind != BAPIPE_BATCHNORM2D || Bn.d.fuse_relu || T.consumers.size() != 1 || T.stashed || t == last_t) continue;
        Bn.fuse_add = i;
        S.fused = true;
    }
    size_t work = 256;
    for (int i = 0; i < n_layers; ++i) {
        Layer &L = st->layers[i];
        const Tensor &A = st->tensors[L.a];
        if (L.d.kind == BAPIPE_MAXPOOL2D) { L.aux_off = slot; L.aux_bytes = st->tensors[L.o].elems; slot += align_up(L.aux_bytes); }
        if (L.d.kind == BAPIPE_BATCHNORM2D) {
            L.aux_off = slot; L.aux_bytes = 2 * sizeof(float) * A.C; slot += align_up(L.aux_bytes);
            size_t w = bn_workspace(micro_batch * A.H * A.W, A.C);
            work = w > work ? w : work;
        }
        if (L.d.kind == BAPIPE_LSTM) {
            const int N = micro_batch, T = A.H, In = A.Cp, H = L.d.cout, G = 4 * H;
            const size_t rows = (size_t)N * T;
            L.aux_off = slot;
            L.off_gates = slot; slot += align_up(rows * G * sizeof(float));
            L.off_cells = slot; slot += align_up(rows * H * sizeof(float));
            L.off_hs = slot; slot += align_up(rows * H * es);
            L.off_pd = slot; slot += align_up(rows * G * es);
            L.off_dcn = slot; slot += align_up((size_t)N * H * sizeof(float));
            L.aux_bytes = slot - L.aux_off;
            size_t w = 0, v;
            const ConvShape cx{N, T, 1, In, T, 1, G, 1, 1, 1, 0}, ch{N, T, 1, H, T, 1, G, 1, 1, 1, 0};
            if (st->dt == DT_BF16) {
                // the widest request among the whole-sequence products and one step of either recurrence
                v = conv_gather_mfma_workspace(rows_geom(N, T, In, G)); w = v > w ? v : w;
                v = conv_gather_mfma_workspace(rows_geom(N, T, G, In)); w = v > w ? v : w;
                v = conv_gather_mfma_raw_workspace(step_geom(N, T, H, G, 1)); w = v > w ? v : w;
                v = conv_gather_mfma_raw_workspace(step_geom(N, T, G, H, 1)); w = v > w ? v : w;
                v = conv_wgrad_mfma_workspace(cx); w = v > w ? v : w;
                v = conv_wgrad_mfma_workspace(ch); w = v > w ? v : w;
            } else {
                w = (size_t)N * G * sizeof(float);
                v = conv_wgrad_direct_workspace(cx); w = v > w ? v : w;
                v = conv_wgrad_direct_workspace(ch); w = v > w ? v : w;
                v = colsum_workspace(N * T, G); w = v > w ? v : w;
            }
            work = w > work ? w : work;
        }
        if (L.d.kind == BAPIPE_CONV2D && st->dt == DT_BF16 && i + 1 < n_layers && L.o != last_t && L.fuse_pool < 0) {
            Layer &B = st->layers[i + 1];
            const Tensor &O = st->tensors[L.o];
            const GatherConv g = fwd_geom(st, L);
            const int rows = micro_batch * O.H * O.W;
            // the one-launch batch-norm of tiny tensors reads x once anyway
            if (B.d.kind == BAPIPE_BATCHNORM2D && B.a == L.o && O.consumers.size() == 1 && !L.d.fuse_relu &&
                rows > 2048 && use_mfma_gather(st, g)) {
                const int chunks = conv_gather_mfma_stat_chunks(g);
                if (chunks > 0) {
                    L.stat_chunks = chunks;
                    B.stats_given = true;
                    const size_t w = (size_t)2 * chunks * O.C * sizeof(float) + 4 * (size_t)O.C * sizeof(float);
                    work = w > work ? w : work;
                }
            }
        }
        if (L.d.kind == BAPIPE_CONV2D && st->dt == DT_BF16 && i > 0 && L.a == i) {      // input = output of layer i-1
            Layer &B = st->layers[i - 1];
            const Tensor &X = st->tensors[L.a];
            const GatherConv dg = dgrad_geom(st, L);
            const int rows = micro_batch * X.H * X.W;
            if (B.d.kind == BAPIPE_BATCHNORM2D && X.root == L.a && X.consumers.size() == 1 && X.need_grad &&
                st->tensors[st->tensors[B.a].root].need_grad && rows > 2048 && use_mfma_gather(st, dg)) {
                const int chunks = conv_gather_mfma_stat_chunks(dg);
                if (chunks > 0) {
                    L.bnb_chunks = chunks;
                    B.bwd_sums_given = true;
                    const size_t w = (size_t)2 * chunks * X.C * sizeof(float) + 4 * (size_t)X.C * sizeof(float);
                    work = w > work ? w : work;
                }
            }
        }
        if (L.d.kind == BAPIPE_CONV2D && st->dt == DT_BF16 && L.d.kh == 1 && L.d.kw == 1 && L.d.stride > 1 && L.d.pad == 0 &&
            st->tensors[st->tensors[L.a].root].need_grad) {
            const GatherConv dg = dgrad_geom(st, L);
            GatherConv dense = dg;
            dense.Ho = dg.Hi; dense.Wo = dg.Wi; dense.s_in = 1;
            if (use_mfma_gather(st, dg) && use_mfma_gather(st, dense)) {
                L.strided_1x1 = true;
                L.bnb_chunks = 0;
                L.up_off = align_up(conv_gather_mfma_workspace(dense));
                const size_t w = L.up_off + align_up((size_t)dense.N * dense.Ho * dense.Wo * dense.Co * es);
                work = w > work ? w : work;
            }
        }
        if (L.d.kind == BAPIPE_CONV2D || L.d.kind == BAPIPE_LINEAR) {
            ConvShape cs = conv_shape(st, L);
            if (L.d.kind == BAPIPE_LINEAR && n_micro > 1 && use_mfma_wgrad(st, cs)) {
                ConvShape all = cs;
                all.N = micro_batch * n_micro;
                if (use_mfma_wgrad(st, all)) {
                    L.deferred = true;
                    L.def_x_bytes = st->tensors[st->tensors[L.a].root].bytes();
                    L.def_g_bytes = st->tensors[L.o].bytes();
                    size_t wd = conv_wgrad_mfma_workspace(all);
                    work = wd > work ? wd : work;
                }
            }
            size_t w = use_mfma_wgrad(st, cs) ? conv_wgrad_mfma_workspace(cs) : conv_wgrad_direct_workspace(cs);
            work = w > work ? w : work;
            w = colsum_workspace(cs.N * cs.P * cs.Q, cs.K);
            work = w > work ? w : work;
            GatherConv fg = fwd_geom(st, L), dg = dgrad_geom(st, L);
            if (use_mfma_gather(st, fg)) { w = conv_gather_mfma_workspace(fg); work = w > work ? w : work; }
            if (use_mfma_gather(st, dg)) { w = conv_gather_mfma_workspace(dg); work = w > work ? w : work; }
            // the plans these launches take beside kernels of further streams (bapipe_stage_set_streams)
            fg.beside = dg.beside = 1;
            if (use_mfma_gather(st, fg)) { w = conv_gather_mfma_workspace(fg); work = w > work ? w : work; }
            if (use_mfma_gather(st, dg)) { w = conv_gather_mfma_workspace(dg); work = w > work ? w : work; }
        }
    }
    // residual fan-out: a tensor read by exactly one conv (MFMA gather input gradient, plain epilogue) and, later in
    // the list, one ADD
    for (int t = 0; t < nt; ++t) {
        Tensor &T = st->tensors[t];
        if (st->dt != DT_BF16 || T.root != t || !T.need_grad || T.galias >= 0 || T.consumers.size() != 2) continue;
        const int ic = T.consumers[0], ia = T.consumers[1];
        const Layer &Lc = st->layers[ic], &La = st->layers[ia];
        if (ic >= ia || Lc.d.kind != BAPIPE_CONV2D || La.d.kind != BAPIPE_ADD || Lc.a != t || (La.a != t && La.b != t)) continue;
        const GatherConv dg = dgrad_geom(st, Lc);
        if (!use_mfma_gather(st, dg) || conv3x3_halo_supported(dg) || Lc.strided_1x1 || Lc.bnb_chunks) continue;
        T.fanout_conv = ic;
    }
    st->slot_bytes = align_up(slot);
    st->transient_bytes = trans;
    st->grads_bytes = gr;
    st->work_bytes = work;

    size_t pb = 0;
    std::vector<size_t> o_w(n_layers), o_b(n_layers), o_dw(n_layers), o_db(n_layers), o_ww(n_layers), o_wt(n_layers);
    for (int i = 0; i < n_layers; ++i) { const Layer &L = st->layers[i]; o_w[i] = pb; pb += align_up(L.w_elems * 4); o_b[i] = pb; pb += align_up(L.b_elems * 4); }
    st->accum_off = pb;
    for (int i = 0; i < n_layers; ++i) { const Layer &L = st->layers[i]; o_dw[i] = pb; pb += align_up(L.w_elems * 4); o_db[i] = pb; pb += align_up(L.b_elems * 4); }
    st->accum_bytes = pb - st->accum_off;
    for (int i = 0; i < n_layers; ++i) {
        const Layer &L = st->layers[i];
        bool mat = has_matrix(L.d.kind);
        o_ww[i] = pb; pb += mat ? align_up(L.w_elems * es) : 0;
        o_wt[i] = pb; pb += mat ? align_up(L.w_elems * es) : 0;
    }
    st->params_bytes = pb;

    size_t defb = 0;
    for (auto &L : st->layers)
        if (L.deferred) defb += align_up(L.def_x_bytes * n_micro) + align_up(L.def_g_bytes * n_micro);
    st->deferred_bytes = defb;
    if (hipSuccess != hipGetLastError()) { /* clear stale error state */ }
    st->params = (char *)st->dev_alloc(st->params_bytes);
    st->stash = (char *)st->dev_alloc(st->slot_bytes * st->depth);
    st->transient = (char *)st->dev_alloc(st->transient_bytes);
    st->grads = (char *)st->dev_alloc(st->grads_bytes);
    st->work = (char *)st->dev_alloc(st->work_bytes);
    st->losses = (float *)st->dev_alloc(sizeof(float) * n_micro);
    if (defb) st->deferred = (char *)st->dev_alloc(defb);
    st->stream_f = st->stream;
    st->work_f = st->work;
    if (!st->params || !st->stash || !st->transient || !st->grads || !st->work || !st->losses || (defb && !st->deferred))
        return create_fail(BAPIPE_E_OOM, "device allocation failed (params %zu, stash %zu x %d, transient %zu, grads %zu, work %zu bytes)",
                           st->params_bytes, st->slot_bytes, st->depth, st->transient_bytes, st->grads_bytes, st->work_bytes);
    {
        size_t off = 0;
        for (auto &L : st->layers)
            if (L.deferred) {
                L.def_x = st->deferred + off; off += align_up(L.def_x_bytes * n_micro);
                L.def_g = st->deferred + off; off += align_up(L.def_g_bytes * n_micro);
                Tensor &RA = st->tensors[root_of(L.a)];
                if (RA.stashed && !RA.mb_store && RA.bytes() == L.def_x_bytes) RA.mb_store = L.def_x;
                const int ro = root_of(L.o);
                Tensor &RO = st->tensors[ro];
                if (ro != 0 && ro != root_of(last_t) && RO.galias < 0 && RO.need_grad && !RO.gmb_store && RO.bytes() == L.def_g_bytes)
                    RO.gmb_store = L.def_g;
            }
    }
    for (int i = 0; i < n_layers; ++i) {
        Layer &L = st->layers[i];
        if (!L.w_elems) continue;
        L.w = (float *)(st->params + o_w[i]);
        L.dw = (float *)(st->params + o_dw[i]);
        if (L.b_elems) { L.bias = (float *)(st->params + o_b[i]); L.db = (float *)(st->params + o_db[i]); }
        if (L.d.kind != BAPIPE_BATCHNORM2D) { L.w_work = st->params + o_ww[i]; L.w_t = st->params + o_wt[i]; }
    }
    // parameters start at zero (gamma at one); all of it through kernels on the stage's stream
    hipError_t e = fill_f32((float *)st->params, 0.f, st->params_bytes / 4, st->stream);
    for (int i = 0; i < n_layers && e == hipSuccess; ++i)
        if (st->layers[i].d.kind == BAPIPE_BATCHNORM2D) e = fill_f32(st->layers[i].w, 1.f, st->layers[i].w_elems, st->stream);
    if (e == hipSuccess) e = fill_f32(st->losses, 0.f, n_micro, st->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(st->stream);
    if (e != hipSuccess) return create_fail(BAPIPE_E_DEVICE, "initialisation: %s", hipGetErrorString(e));
    guard.s = nullptr;
    *out = st;
    return BAPIPE_OK;
}

int bapipe_stage_forward(bapipe_stage_t *st, int mb_id, const void *x_dev, void *y_dev)
{
    if (!st || !x_dev) return st ? st->fail(BAPIPE_E_INVALID, "forward: NULL argument") : BAPIPE_E_INVALID;
    if (mb_id != st->n_fwd || mb_id >= st->M)
        return st->fail(BAPIPE_E_ORDER, "forward: expected micro-batch %d of %d, got %d", st->n_fwd, st->M, mb_id);
    if (st->n_fwd - st->n_bwd >= st->depth)
        return st->fail(BAPIPE_E_ORDER, "forward: %d micro-batches already in flight (stash depth %d)", st->n_fwd - st->n_bwd, st->depth);
    const Tensor &In = st->tensors[0];
    const int dt = st->dt;
    hipStream_t s = st->stream;
    if (mb_id == 0) st->loss_valid.assign(st->M, 0);       // a new mini-batch: the previous one's losses are gone
    if (st->stream_b && mb_id >= st->depth) HIPCHK(hipStreamWaitEvent(s, st->ev_bwd[mb_id - st->depth], 0));
    FwdCtx c{mb_id, nullptr};
    GradEpi none{nullptr, 0};
    if (st->opts.io_layout == BAPIPE_NCHW) {
        HIPCHK(nchw_to_nhwc(dt, x_dev, st->tptr(0, mb_id), none, st->mb, In.C, In.H, In.W, In.Cp, s));
    } else if (In.Cp != In.C) {
        HIPCHK(nhwc_repad(dt, x_dev, st->tptr(0, mb_id), (size_t)st->mb * In.H * In.W, In.C, In.Cp, s));
    } else if (In.stashed) {
        HIPCHK(hipMemcpyAsync(st->tptr(0, mb_id), x_dev, In.bytes(), hipMemcpyDeviceToDevice, s));
    } else {
        c.x_direct = x_dev;
    }
    for (int i = 0; i < (int)st->layers.size(); ++i) {
        int rc = layer_forward(st, i, c);
        if (rc != BAPIPE_OK) return rc;
    }
    if (y_dev) {
        const int last = (int)st->tensors.size() - 1;
        const Tensor &O = st->tensors[last];
        const Tensor &R = st->tensors[O.root];
        const void *src = in_ptr(st, last, c);
        // a flattened view of a spatial tensor is indexed c*H*W + h*W + w whatever the boundary layout is
        const bool flat_of_spatial = O.root != last && R.H * R.W > 1;
        if (O.esize == dt_size(dt) && ((st->opts.io_layout == BAPIPE_NCHW && R.H * R.W > 1) || flat_of_spatial))
            HIPCHK(nhwc_to_nchw(dt, src, y_dev, st->mb, R.C, R.H, R.W, R.Cp, s));
        else
            HIPCHK(hipMemcpyAsync(y_dev, src, O.bytes(), hipMemcpyDeviceToDevice, s));
    }
    if (st->stream_b) HIPCHK(hipEventRecord(st->ev_fwd[mb_id], s));
    st->n_fwd++;
    return BAPIPE_OK;
}

int bapipe_stage_backward(bapipe_stage_t *st, int mb_id, const void *dy_dev_or_labels, void *dx_dev)
{
    if (!st || !dy_dev_or_labels) return st ? st->fail(BAPIPE_E_INVALID, "backward: NULL argument") : BAPIPE_E_INVALID;
    if (mb_id != st->n_bwd || mb_id >= st->n_fwd)
        return st->fail(BAPIPE_E_ORDER, "backward: expected micro-batch %d (forwarded so far: %d), got %d", st->n_bwd, st->n_fwd, mb_id);
    const int nl = (int)st->layers.size(), last = nl;
    const int dt = st->dt;
    struct Lane {           // the backward pass runs on its own stream and workspace when there is one
        bapipe_stage *st;
        explicit Lane(bapipe_stage *s_) : st(s_) { if (st->stream_b) { st->stream = st->stream_b; st->work = st->work_b; } }
        ~Lane() { st->stream = st->stream_f; st->work = st->work_f; }
    } lane(st);
    hipStream_t s = st->stream;
    if (st->stream_b) HIPCHK(hipStreamWaitEvent(s, st->ev_fwd[mb_id], 0));
    const bool nhwc = st->opts.io_layout == BAPIPE_NHWC;
    BwdCtx c;
    c.mbid = mb_id;
    c.x_direct = nullptr;
    c.dy_direct = nullptr;
    c.dx_direct = nullptr;
    c.labels = nullptr;
    c.written.assign(st->tensors.size(), 0);
    c.pending.assign(st->tensors.size(), nullptr);
    const Tensor &In = st->tensors[0];
    const bool want_dx = In.need_grad && dx_dev != nullptr;
    if (want_dx && (nhwc || In.H * In.W == 1) && In.Cp == In.C) c.dx_direct = dx_dev;
    if (st->layers[nl - 1].d.kind == BAPIPE_SOFTMAX_XENT) {
        c.labels = (const int32_t *)dy_dev_or_labels;
    } else {
        const int r = st->tensors[last].root;
        const Tensor &O = st->tensors[last];
        const Tensor &R = st->tensors[r];
        GradEpi e{nullptr, 0};
        if (st->tensors[r].gated) e.gate = st->tptr(r, mb_id);
        const bool flat_of_spatial = r != last && R.H * R.W > 1;      // dy arrives indexed c*H*W + h*W + w
        if ((!nhwc && R.H * R.W > 1) || flat_of_spatial) {
            HIPCHK(nchw_to_nhwc(dt, dy_dev_or_labels, st->gptr(last), e, st->mb, R.C, R.H, R.W, R.Cp, s));
        } else if (e.gate || r == 0) {
            HIPCHK(grad_copy(dt, dy_dev_or_labels, st->gptr(last), e, O.elems, s));
        } else {
            c.dy_direct = dy_dev_or_labels;
        }
        c.written[r] = 1;
    }
    for (int i = nl - 1; i >= 0; --i) {
        int rc = layer_backward(st, i, c);
        if (rc != BAPIPE_OK) return rc;
    }
    for (const void *p : c.pending)
        if (p) return st->fail(BAPIPE_E_DEVICE, "backward: a residual gradient was left for a conv that never took it");
    if (want_dx && !c.dx_direct) {
        if (nhwc)
            HIPCHK(nhwc_repad(dt, st->gptr(0), dx_dev, (size_t)st->mb * In.H * In.W, In.Cp, In.C, s));
        else
            HIPCHK(nhwc_to_nchw(dt, st->gptr(0), dx_dev, st->mb, In.C, In.H, In.W, In.Cp, s));
    }
    if (c.labels) st->loss_valid[mb_id] = 1;
    if (st->w_used) {                                   // the pass is complete when its weight-gradient kernels are
        HIPCHK(hipEventRecord(st->ev_w_end, st->stream_w));
        HIPCHK(hipStreamWaitEvent(s, st->ev_w_end, 0));
        st->w_used = false;
    }
    if (st->stream_b) HIPCHK(hipEventRecord(st->ev_bwd[mb_id], s));
    st->n_bwd++;
    return BAPIPE_OK;
}

int bapipe_stage_set_streams(bapipe_stage_t *st, void *hip_stream_backward, void *hip_stream_wgrad)
{
    if (!st) return BAPIPE_E_INVALID;
    if (st->n_fwd != 0 || st->n_bwd != 0)
        return st->fail(BAPIPE_E_ORDER, "set_streams: only between mini-batches (after create or step)");
    HIPCHK(sync_streams(st));
    hipStream_t sb = (hipStream_t)hip_stream_backward, sw = (hipStream_t)hip_stream_wgrad;
    if (sb == st->stream_f) sb = nullptr;
    if (sw && (sw == st->stream_f || sw == sb))
        return st->fail(BAPIPE_E_INVALID, "set_streams: the weight-gradient stream must differ from the other streams");
    // workspaces and events are created on first use and stay for the next time
    if (sb && !st->work_b) {
        st->work_b = (char *)st->dev_alloc(st->work_bytes);
        if (!st->work_b) return st->fail(BAPIPE_E_OOM, "set_streams: %zu bytes of workspace", st->work_bytes);
    }
    if (sw && !st->work_w) {
        st->work_w = (char *)st->dev_alloc(st->work_bytes);
        if (!st->work_w) return st->fail(BAPIPE_E_OOM, "set_streams: %zu bytes of workspace", st->work_bytes);
    }
    if (sb && st->ev_fwd.empty()) {
        std::vector<hipEvent_t> ev(2 * (size_t)st->M, nullptr);
        for (auto &e : ev)
            if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) {
                for (hipEvent_t d : ev) if (d) (void)hipEventDestroy(d);
                return st->fail(BAPIPE_E_DEVICE, "set_streams: hipEventCreate failed");
            }
        st->ev_fwd.assign(ev.begin(), ev.begin() + st->M);
        st->ev_bwd.assign(ev.begin() + st->M, ev.end());
    }
    if (sw && !st->ev_g) {
        HIPCHK(hipEventCreateWithFlags(&st->ev_g, hipEventDisableTiming));
        HIPCHK(hipEventCreateWithFlags(&st->ev_w_end, hipEventDisableTiming));
    }
    st->stream_b = sb;
    st->stream_w = sw;
    return BAPIPE_OK;
}

int bapipe_stage_backward_static(bapipe_stage_t *st, int mb_id, const void *dy_dev_or_labels, void *dx_dev)
{
    if (!st) return BAPIPE_E_INVALID;
    if (st->work_bytes > (size_t)BAPIPE_STATIC_SCRATCH_BYTES)
        return st->fail(BAPIPE_E_UNSUPPORTED, "backward_static: the stage's kernels need %zu bytes of workspace, the static one holds %zu",
                        st->work_bytes, (size_t)BAPIPE_STATIC_SCRATCH_BYTES);
    char *ws = nullptr;
    HIPCHK(static_scratch(&ws));
    // every kernel of the backward pass writes its partial results before a later kernel of the same pass reads
    // them (no atomics, nothing accumulates in the workspace), so what the previous call left there needs no clearing
    char *own_f = st->work_f, *own_b = st->work_b;
    hipStream_t own_w = st->stream_w;
    st->work = st->work_f = ws;
    if (st->work_b) st->work_b = ws;
    st->stream_w = nullptr;              // one array: the weight-gradient kernels of this pass stay on the pass's stream
    const int rc = bapipe_stage_backward(st, mb_id, dy_dev_or_labels, dx_dev);
    st->stream_w = own_w;
    st->work_f = own_f;
    st->work_b = own_b;
    st->work = own_f;
    return rc;
}

int bapipe_stage_step(bapipe_stage_t *st, float lr)
{
    if (!st) return BAPIPE_E_INVALID;
    if (st->n_bwd != st->M)
        return st->fail(BAPIPE_E_ORDER, "step: %d of %d backward passes done", st->n_bwd, st->M);
    if (st->stream_b) HIPCHK(hipStreamWaitEvent(st->stream, st->ev_bwd[st->M - 1], 0));
    {
        int rc = flush_deferred(st);
        if (rc != BAPIPE_OK) return rc;
    }
    for (auto &L : st->layers) {
        if (!L.w_elems) continue;
        const bool mat = L.d.kind != BAPIPE_BATCHNORM2D;
        HIPCHK(sgd_step(st->dt, L.w, L.dw, lr, mat ? L.w_work : nullptr, L.w_elems, st->stream));
        if (L.b_elems) HIPCHK(sgd_step(st->dt, L.bias, L.db, lr, nullptr, L.b_elems, st->stream));
        if (mat) HIPCHK(refresh_transposed(st, L));
    }
    st->n_fwd = st->n_bwd = 0;
    st->flushed = 0;
    return BAPIPE_OK;
}

int bapipe_stage_set_params(bapipe_stage_t *st, int layer, const float *w_host, const float *b_host)
{
    if (!st) return BAPIPE_E_INVALID;
    if (layer < 0 || layer >= (int)st->layers.size() || !st->layers[layer].w_elems)
        return st->fail(BAPIPE_E_INVALID, "set_params: layer %d has no parameters", layer);
    Layer &L = st->layers[layer];
    HIPCHK(sync_streams(st));
    if (w_host) {
        if (L.d.kind == BAPIPE_BATCHNORM2D) {
            HIPCHK(hipMemcpy(L.w, w_host, L.w_elems * 4, hipMemcpyHostToDevice));
        } else {
            std::vector<float> tmp(L.w_elems);
            to_internal(L, w_host, tmp.data());
            HIPCHK(hipMemcpy(L.w, tmp.data(), L.w_elems * 4, hipMemcpyHostToDevice));
            HIPCHK(refresh_work(st, L));
            HIPCHK(sync_streams(st));
        }
    }
    if (b_host) {
        if (!L.b_elems) return st->fail(BAPIPE_E_INVALID, "set_params: layer %d has no bias", layer);
        HIPCHK(hipMemcpy(L.bias, b_host, L.b_elems * 4, hipMemcpyHostToDevice));
    }
    return BAPIPE_OK;
}

static int get_vectors(bapipe_stage_t *st, int layer, float *w_host, float *b_host, bool grads, const char *what)
{
    if (!st) return BAPIPE_E_INVALID;
    if (layer < 0 || layer >= (int)st->layers.size() || !st->layers[layer].w_elems)
        return st->fail(BAPIPE_E_INVALID, "%s: layer %d has no parameters", what, layer);
    Layer &L = st->layers[layer];
    if (grads) {
        int rc = flush_deferred(st);
        if (rc != BAPIPE_OK) return rc;
    }
    HIPCHK(sync_streams(st));
    if (w_host) {
        const float *src = grads ? L.dw : L.w;
        if (L.d.kind == BAPIPE_BATCHNORM2D) {
            HIPCHK(hipMemcpy(w_host, src, L.w_elems * 4, hipMemcpyDeviceToHost));
        } else {
            std::vector<float> tmp(L.w_elems);
            HIPCHK(hipMemcpy(tmp.data(), src, L.w_elems * 4, hipMemcpyDeviceToHost));
            from_internal(L, tmp.data(), w_host);
        }
    }
    if (b_host) {
        if (!L.b_elems) return st->fail(BAPIPE_E_INVALID, "%s: layer %d has no bias", what, layer);
        HIPCHK(hipMemcpy(b_host, grads ? L.db : L.bias, L.b_elems * 4, hipMemcpyDeviceToHost));
    }
    return BAPIPE_OK;
}

int bapipe_stage_get_params(bapipe_stage_t *st, int layer, float *w_host, float *b_host)
{
    return get_vectors(st, layer, w_host, b_host, false, "get_params");
}

int bapipe_stage_get_grads(bapipe_stage_t *st, int layer, float *dw_host, float *db_host)
{
    return get_vectors(st, layer, dw_host, db_host, true, "get_grads");
}

int bapipe_stage_get_pool_indices(bapipe_stage_t *st, int layer, int mb_id, uint8_t *idx_host)
{
    if (!st || !idx_host) return st ? st->fail(BAPIPE_E_INVALID, "get_pool_indices: NULL argument") : BAPIPE_E_INVALID;
    if (layer < 0 || layer >= (int)st->layers.size() || st->layers[layer].d.kind != BAPIPE_MAXPOOL2D)
        return st->fail(BAPIPE_E_INVALID, "get_pool_indices: layer %d is not a max-pool", layer);
    if (mb_id < st->n_bwd || mb_id >= st->n_fwd)
        return st->fail(BAPIPE_E_ORDER, "get_pool_indices: micro-batch %d is not in flight", mb_id);
    const Layer &L = st->layers[layer];
    const Tensor &O = st->tensors[L.o];
    // NHWC on the device -> NCHW for the caller, through the workspace if it is large enough
    std::vector<uint8_t> tmp(O.elems);
    HIPCHK(sync_streams(st));
    HIPCHK(hipMemcpy(tmp.data(), st->slot(mb_id) + L.aux_off, O.elems, hipMemcpyDeviceToHost));
    const int N = st->mb, C = O.C, H = O.H, W = O.W;
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int h = 0; h < H; ++h)
                for (int w = 0; w < W; ++w)
                    idx_host[(((size_t)n * C + c) * H + h) * W + w] = tmp[(((size_t)n * H + h) * W + w) * C + c];
    return BAPIPE_OK;
}

int bapipe_stage_get_loss(bapipe_stage_t *st, int mb_id, float *loss_host)
{
    if (!st || !loss_host) return st ? st->fail(BAPIPE_E_INVALID, "get_loss: NULL argument") : BAPIPE_E_INVALID;
    if (st->layers.back().d.kind != BAPIPE_SOFTMAX_XENT) return st->fail(BAPIPE_E_ORDER, "get_loss: stage has no loss layer");
    if (mb_id < 0 || mb_id >= st->M || !st->loss_valid[mb_id])
        return st->fail(BAPIPE_E_ORDER, "get_loss: micro-batch %d has not been backwarded", mb_id);
    HIPCHK(sync_streams(st));
    HIPCHK(hipMemcpy(loss_host, st->losses + mb_id, sizeof(float), hipMemcpyDeviceToHost));
    return BAPIPE_OK;
}

int bapipe_stage_stash_bytes(const bapipe_stage_t *st, uint64_t *per_mb, int *depth)
{
    if (!st) return BAPIPE_E_INVALID;
    // the inputs / output gradients that the linear layers keep of ALL M micro-batches for their one weight-gradient
    // GEMM per mini-batch are spread over the ring slots, so that per_mb x depth covers everything the stage holds
    if (per_mb) *per_mb = st->slot_bytes + (st->deferred_bytes + st->depth - 1) / st->depth;
    if (depth) *depth = st->depth;
    return BAPIPE_OK;
}

int bapipe_stage_kernel_timing(bapipe_stage_t *st, int kernel_class)
{
    if (!st) return BAPIPE_E_INVALID;
    if (kernel_class >= BAPIPE_KC_COUNT) return st->fail(BAPIPE_E_INVALID, "kernel_timing: class %d", kernel_class);
    HIPCHK(sync_streams(st));
    if (kernel_class >= 0 && st->tap_events.empty()) {
        st->tap_events.resize(2 * 4096);
        for (auto &e : st->tap_events) HIPCHK(hipEventCreate(&e));
    }
    st->tap_class = kernel_class < 0 ? -1 : kernel_class;
    st->tap_used = 0;
    st->tap_dropped = 0;
    st->tap_flop = st->tap_bytes = 0.0;
    return BAPIPE_OK;
}

int bapipe_stage_kernel_timing_read(bapipe_stage_t *st, double *total_ms, uint64_t *launches, double *flop,
                                    double *bytes)
{
    if (!st) return BAPIPE_E_INVALID;
    HIPCHK(sync_streams(st));
    double ms = 0.0;
    for (size_t i = 0; i + 1 < st->tap_used; i += 2) {
        float t = 0.f;
        HIPCHK(hipEventElapsedTime(&t, st->tap_events[i], st->tap_events[i + 1]));
        ms += t;
    }
    const size_t dropped = st->tap_dropped;
    st->tap_dropped = 0;
    if (dropped) {
        st->tap_used = 0;
        st->tap_flop = st->tap_bytes = 0.0;
        return st->fail(BAPIPE_E_UNSUPPORTED, "kernel_timing_read: %zu launches were not recorded (more than %zu between reads)",
                        dropped, kTapMaxEvents / 2);
    }
    if (total_ms) *total_ms = ms;
    if (launches) *launches = st->tap_used / 2;
    if (flop) *flop = st->tap_flop;
    if (bytes) *bytes = st->tap_bytes;
    st->tap_used = 0;
    st->tap_flop = st->tap_bytes = 0.0;
    return BAPIPE_OK;
}

int bapipe_profile_layers(bapipe_stage_t *st, int warmup, int iters, bapipe_layer_profile_t *out, int cap, int *n)
{
    if (!st || !out || !n || iters <= 0 || warmup < 0) return st ? st->fail(BAPIPE_E_INVALID, "profile: bad argument") : BAPIPE_E_INVALID;
    const int nl = (int)st->layers.size();
    if (cap < nl) return st->fail(BAPIPE_E_INVALID, "profile: %d records needed, cap is %d", nl, cap);
    if (st->n_fwd != 0) return st->fail(BAPIPE_E_ORDER, "profile: only between mini-batches (after create or step)");
    hipStream_t s = st->stream;
    // defined (zero) scratch data in slot 0, the transient arena and the gradient buffers
    HIPCHK(fill_f32((float *)st->slot(0), 0.f, st->slot_bytes / 4, s));
    HIPCHK(fill_f32((float *)st->transient, 0.f, st->transient_bytes / 4, s));
    HIPCHK(fill_f32((float *)st->grads, 0.f, st->grads_bytes / 4, s));
    hipEvent_t e0, e1;
    HIPCHK(hipEventCreate(&e0));
    HIPCHK(hipEventCreate(&e1));
    int rc = BAPIPE_OK;
    FwdCtx fc{0, nullptr, true};
    std::vector<int32_t> zero_labels(st->mb, 0);
    int32_t *labels_dev = (int32_t *)st->work;   // xent reads labels only; no kernel of that layer uses the workspace
    for (int i = 0; i < nl && rc == BAPIPE_OK; ++i) {
        Layer &L = st->layers[i];
        const Tensor &O = st->tensors[L.o];
        float ms = 0.f;
        for (int k = 0; k < warmup && rc == BAPIPE_OK; ++k) rc = layer_forward(st, i, fc);
        if (rc != BAPIPE_OK) break;
        (void)hipEventRecord(e0, s);
        for (int k = 0; k < iters && rc == BAPIPE_OK; ++k) rc = layer_forward(st, i, fc);
        (void)hipEventRecord(e1, s);
        if (hipEventSynchronize(e1) != hipSuccess) { rc = st->fail(BAPIPE_E_DEVICE, "profile: event sync failed"); break; }
        (void)hipEventElapsedTime(&ms, e0, e1);
        out[i].fwd_ms = L.fused ? 0.0 : ms / iters;          // done by the layer before it: only the empty event pair was timed

        BwdCtx bc;
        bc.mbid = 0; bc.x_direct = bc.dy_direct = nullptr; bc.dx_direct = nullptr; bc.labels = nullptr;
        bc.profiling = true;
        if (L.d.kind == BAPIPE_SOFTMAX_XENT) {
            if (hipMemcpyAsync(labels_dev, zero_labels.data(), sizeof(int32_t) * st->mb, hipMemcpyHostToDevice, s) != hipSuccess) { rc = st->fail(BAPIPE_E_DEVICE, "profile: label upload"); break; }
            (void)hipStreamSynchronize(s);
            bc.labels = labels_dev;
        }
        for (int k = 0; k < warmup + iters && rc == BAPIPE_OK; ++k) {
            if (k == warmup) (void)hipEventRecord(e0, s);
            bc.written.assign(st->tensors.size(), 0);
            bc.pending.assign(st->tensors.size(), nullptr);
            rc = layer_backward(st, i, bc);
        }
        (void)hipEventRecord(e1, s);
        if (hipEventSynchronize(e1) != hipSuccess) { rc = st->fail(BAPIPE_E_DEVICE, "profile: event sync failed"); break; }
        (void)hipEventElapsedTime(&ms, e0, e1);
        out[i].bwd_ms = ms / iters;
        out[i].weight_bytes = (uint64_t)(L.w_elems + L.b_elems) * 4;
        out[i].out_feature_bytes = (uint64_t)O.bytes();
        uint64_t sb = L.aux_bytes;
        if (O.root == L.o && O.stashed) sb += O.bytes();
        if (L.deferred)            // kept for all M micro-batches, not only the in-flight ones: spread over the ring depth
            sb += ((uint64_t)(L.def_x_bytes + L.def_g_bytes) * st->M + st->depth - 1) / st->depth;
        out[i].stash_bytes = sb;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    // the timed backward passes added into the accumulators: restore zeros and the loss slots
    if (rc == BAPIPE_OK) {
        HIPCHK(fill_f32((float *)(st->params + st->accum_off), 0.f, st->accum_bytes / 4, s));
        HIPCHK(fill_f32(st->losses, 0.f, st->M, s));
        HIPCHK(hipStreamSynchronize(s));
        *n = nl;
    }
    return rc;
}

int bapipe_profile_sweep(const bapipe_layer_desc_t *layers, int n_layers, const int *micro_batches, int n_sizes,
                         const bapipe_stage_opts_t *opts, int warmup, int iters, bapipe_layer_profile_t *out)
{
    if (!layers || n_layers <= 0 || !micro_batches || n_sizes <= 0 || !opts || !out) return BAPIPE_E_INVALID;
    std::vector<bapipe_layer_profile_t> all((size_t)n_sizes * n_layers);
    for (int k = 0; k < n_sizes; ++k) {
        bapipe_stage_t *st = nullptr;
        int rc = bapipe_stage_create(layers, n_layers, micro_batches[k], 1, opts, &st);
        if (rc != BAPIPE_OK) return rc;
        int n = 0;
        rc = bapipe_profile_layers(st, warmup, iters, all.data() + (size_t)k * n_layers, n_layers, &n);
        bapipe_stage_destroy(st);
        if (rc != BAPIPE_OK) return rc;
    }
    for (size_t i = 0; i < all.size(); ++i) out[i] = all[i];
    return BAPIPE_OK;
}

}  // extern "C"
