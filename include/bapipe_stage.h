/*
 * bapipe_stage.h - C ABI of one pipeline stage's forward/backward engine on one MI355X.
 *
 * A stage is the contiguous subset of a network's layers that pipeline parallelism places
 * on one accelerator (paper Sec. I, Sec. III-A).  A mini-batch is split into M micro-batches
 * (Sec. II-B); the stage runs forward and backward of each micro-batch with the same
 * weights, alternating them in the 1F1B steady state, and updates its weights once per
 * mini-batch after the last backward (Sec. III-B-1).  Between forward and backward of a
 * micro-batch the stage keeps that micro-batch's features; under 1F1B at most N-i+1
 * micro-batches are in flight at stage i of N (Table I / II, "Features memory"), twice that
 * with doubled warm-up (1F1B-SO, Table II).  The profiler call returns what the paper's
 * "DNN profile" step collects per layer: forward time, backward time, weights size and
 * features size (Sec. III-A).
 *
 * Conventions
 *  - Every function returns a bapipe_status_t.  Output arguments are written only on
 *    BAPIPE_OK.  No exception crosses this boundary.
 *  - "dev" pointers are device (HBM) addresses on the current HIP device, owned by the
 *    caller; "host" pointers are ordinary host memory.  The library never frees caller
 *    memory and does not keep x_dev / dy_dev after the call has enqueued its work.
 *  - forward / backward / step only ENQUEUE kernels on opts->hip_stream and return without
 *    synchronising; get_* / profile calls synchronise that stream.
 *  - Weights, gradient accumulators, the activation stash ring and workspaces are owned by
 *    the handle and obtained through opts->mem (NULL callbacks: hipMalloc / hipFree).
 *  - A handle is not thread-safe; distinct handles are independent.  The library keeps two
 *    pieces of state outside handles: the message of the calling thread's last failed
 *    bapipe_stage_create (thread-local, read with bapipe_last_error(NULL)) and the statically
 *    allocated workspace of bapipe_stage_backward_static (one per GPU, see there).
 *  - Storage types.  BAPIPE_FP32: activations, gradients and weights are float.
 *    BAPIPE_BF16: activations, activation gradients and working weights are bfloat16
 *    (round-to-nearest-even), accumulation is fp32, master weights and weight gradients are
 *    fp32.  Boundary tensors (x, y, dy, dx) have the stage's storage type and the layout
 *    opts->io_layout; softmax outputs and losses are always float.
 *  - Parameter layouts at this boundary follow the PyTorch conventions: conv weights OIHW,
 *    linear weights [out][in] where `in` indexes the NCHW flattening (c*H*W + h*W + w) of
 *    the producing tensor, batch-norm w = gamma, b = beta.  LSTM (the layer of the paper's
 *    sequence-to-sequence workload, Sec. IV-A; hidden size cout, zero initial state, gates in
 *    the order input, forget, candidate, output): w is [4*cout][cin+cout], row q*cout + j =
 *    gate q of unit j, first the cin input weights, then the cout recurrent ones; b is
 *    [4*cout] (the sum of PyTorch's two bias vectors).
 */
#ifndef BAPIPE_STAGE_H
#define BAPIPE_STAGE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct bapipe_stage bapipe_stage_t; /* opaque; created by _create, freed by _destroy */

typedef enum {
    BAPIPE_OK = 0,
    BAPIPE_E_INVALID = 1,     /* NULL / out-of-range argument                         */
    BAPIPE_E_SHAPE = 2,       /* layer list does not type-check (channels, sizes)      */
    BAPIPE_E_ORDER = 3,       /* call violates the micro-batch schedule; nothing done  */
    BAPIPE_E_OOM = 4,         /* allocator returned NULL; nothing leaked               */
    BAPIPE_E_DEVICE = 5,      /* a HIP call failed                                     */
    BAPIPE_E_UNSUPPORTED = 6  /* valid request this build has no kernel for            */
} bapipe_status_t;

typedef enum {
    BAPIPE_CONV2D = 0,       /* y = x (*) w + b, cross-correlation, zero padding            */
    BAPIPE_RELU = 1,         /* y = max(x,0)                                                */
    BAPIPE_MAXPOOL2D = 2,    /* kh x kw window, first maximum wins (row-major scan)         */
    BAPIPE_BATCHNORM2D = 3,  /* training mode: biased statistics of the micro-batch         */
    BAPIPE_ADD = 4,          /* y = src0 + src1                                             */
    BAPIPE_FLATTEN = 5,      /* (C,H,W) -> (C*H*W,1,1)                                      */
    BAPIPE_LINEAR = 6,       /* y = x W^T + b                                               */
    BAPIPE_SOFTMAX_XENT = 7, /* last layer only: p = softmax(z); loss from labels in bwd    */
    BAPIPE_AVGPOOL2D = 8,    /* mean of k x k windows, stride = k, pad = 0 (k = H: global)  */
    BAPIPE_LSTM = 9          /* LSTM over the H axis of a (cin, T, 1) tensor -> (cout, T, 1) */
} bapipe_layer_kind_t;

/* One layer of the stage.  src0/src1: index of the producing layer in the list, -1 = the
 * stage input; producers must precede consumers.  fuse_relu applies max(.,0) to the output
 * of CONV2D / BATCHNORM2D / ADD / LINEAR.  cin/cout: channels (features for LINEAR;
 * BATCHNORM2D needs cin == cout == channels of its input). */
typedef struct {
    int32_t kind;
    int32_t cin, cout;
    int32_t kh, kw, stride, pad;
    int32_t has_bias;
    int32_t fuse_relu;
    int32_t src0, src1;
    float eps;
} bapipe_layer_desc_t;

typedef struct {
    void *(*alloc)(size_t bytes, void *ctx); /* returns a device pointer (256-byte aligned) or NULL */
    void (*free)(void *dev_ptr, void *ctx);
    void *ctx;
} bapipe_allocator_t;

enum { BAPIPE_FP32 = 0, BAPIPE_BF16 = 1 };
enum { BAPIPE_NCHW = 0, BAPIPE_NHWC = 1 };
enum { BAPIPE_SCHED_1F1B = 0, BAPIPE_SCHED_1F1B_SO = 1 };

typedef struct {
    int32_t dtype;               /* BAPIPE_FP32 | BAPIPE_BF16                                   */
    int32_t in_c, in_h, in_w;    /* per-sample shape of the stage input                         */
    int32_t io_layout;           /* layout of x, y, dy, dx: BAPIPE_NCHW | BAPIPE_NHWC           */
    int32_t stage_index;         /* i, 1-based position of this stage (Sec. III-B-1)            */
    int32_t n_stages;            /* N, number of pipeline stages                                */
    int32_t schedule;            /* stash depth min(M, N-i+1) (1F1B) or min(M, 2(N-i+1)) (SO)   */
    int32_t need_input_grad;     /* 0: the stage is first in the network, dx is never produced  */
    float loss_scale;            /* s in loss = -s*sum log p[label]; <=0: 1/(micro_batch*M)     */
    void *hip_stream;            /* hipStream_t all work is enqueued on (NULL: default stream)  */
    bapipe_allocator_t mem;
} bapipe_stage_opts_t;

typedef struct {
    double fwd_ms;               /* mean time of the layer's forward kernels, one micro-batch     */
    double bwd_ms;               /* mean time of its backward kernels (dgrad + wgrad + masks)     */
    uint64_t weight_bytes;       /* fp32 master weights + bias of the layer                      */
    uint64_t out_feature_bytes;  /* bytes of the layer's output for one micro-batch               */
    uint64_t stash_bytes;        /* bytes the layer keeps per in-flight micro-batch for backward  */
} bapipe_layer_profile_t;

/* Build a stage from a layer list (Sec. I: a stage is "consecutive layers"), the
 * micro-batch size and the number M of micro-batches per mini-batch (Sec. II-B).
 * layers: host array of n_layers descriptors (copied).  opts: host, copied.
 * Parameters start at zero (gamma at one); load them with bapipe_stage_set_params.
 * Errors: E_INVALID (NULL, n_layers<=0, sizes<=0, bad enum), E_SHAPE (list does not
 * type-check; bapipe_last_error(NULL) names the layer), E_UNSUPPORTED, E_OOM, E_DEVICE. */
int bapipe_stage_create(const bapipe_layer_desc_t *layers, int n_layers, int micro_batch,
                        int n_micro, const bapipe_stage_opts_t *opts, bapipe_stage_t **out);

/* Forward pass of micro-batch mb_id (Sec. III-B-1).  x_dev: device, micro_batch x (in_c,
 * in_h,in_w) in io_layout and the stage's storage type.  y_dev: device, receives the last
 * layer's output (softmax probabilities as float for SOFTMAX_XENT); may be NULL.
 * Legal order within a mini-batch: ids 0..M-1 ascending, and at most `depth` micro-batches
 * forwarded but not yet backwarded; otherwise E_ORDER and nothing is enqueued. */
int bapipe_stage_forward(bapipe_stage_t *st, int mb_id, const void *x_dev, void *y_dev);

/* Backward pass of micro-batch mb_id: consumes its stashed features, adds its weight
 * gradients into the fp32 accumulators and releases its stash slot.  (For LINEAR layers the
 * library may keep the micro-batch's layer input and output gradient instead and form the
 * weight gradient of all micro-batches with one GEMM inside bapipe_stage_step /
 * bapipe_stage_get_grads: same sums, different summation order.)
 * dy_dev_or_labels: device; gradient w.r.t. the stage output (layout/type as y), or, when
 * the last layer is SOFTMAX_XENT, micro_batch int32 class labels.
 * dx_dev: device, receives the gradient w.r.t. the stage input (layout/type as x); may be
 * NULL; ignored when need_input_grad == 0.
 * Legal order: ids ascending, each after its own forward; otherwise E_ORDER. */
int bapipe_stage_backward(bapipe_stage_t *st, int mb_id, const void *dy_dev_or_labels,
                          void *dx_dev);

/* Overlap of independent work on further streams.  By default every kernel is enqueued on
 * opts->hip_stream, one after the other.  Two kinds of work do not depend on each other:
 *  - In the 1F1B steady state the forward pass of one micro-batch and the backward pass of an
 *    earlier one alternate (Sec. III-B-1): they touch different ring slots, and weights only
 *    change in the update.  With hip_stream_backward every backward pass is enqueued on that
 *    stream instead, beside the forward passes of later micro-batches.
 *  - Inside a backward pass a layer's weight gradient needs the layer's output gradient and its
 *    stashed input, nothing the remaining input-gradient kernels produce.  With
 *    hip_stream_wgrad the weight-gradient kernels of conv layers are enqueued on that stream,
 *    beside the input-gradient chain.
 * Kernels of different streams share the compute units, so each fills what the others leave
 * idle while they ramp up, drain, or wait for memory.  Both streams are caller-owned, on the
 * stage's device, of default priority, and distinct from each other and from opts->hip_stream;
 * either may be NULL (that kind of work then stays where it was).  The library orders the streams
 * with events: backward(m) starts after forward(m); forward(m + depth), which reuses the ring
 * slot of micro-batch m, after backward(m); a weight-gradient kernel after the kernels that
 * complete its layer's output gradient; the backward pass's own stream waits for the pass's
 * weight-gradient kernels before the pass counts as complete; bapipe_stage_step runs after the
 * last backward pass; get_* / set_* / profile calls synchronise all streams.  Results are the same
 * bit for bit.  What changes for the caller: dx_dev and the loss of a micro-batch are complete
 * when the stream of the BACKWARD passes has run the pass, and dy_dev_or_labels must be complete
 * on (or before) that stream and stay untouched until then.  A stage with a ring of depth 1
 * cannot overlap passes and only pays for the event hand-overs of a backward stream.
 * bapipe_stage_backward_static keeps its weight-gradient kernels on the pass's stream (there is
 * one static workspace).  Only between mini-batches (after create or step), else E_ORDER.  The
 * first use of each stream allocates one more kernel workspace through opts->mem and a few
 * events: E_OOM, E_DEVICE.  E_INVALID if hip_stream_wgrad equals one of the other streams. */
int bapipe_stage_set_streams(bapipe_stage_t *st, void *hip_stream_backward, void *hip_stream_wgrad);

/* bapipe_stage_backward for callers that must not allocate device memory while they run (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same arguments,
 * same schedule rules, same results bit for bit, but the kernels' workspace (split-K partial
 * sums of the weight-gradient and linear-layer GEMMs, column-reduction partials of batch-norm and
 * bias gradients, the dense product of a strided 1x1 input gradient) is a statically allocated
 * device array of BAPIPE_STATIC_SCRATCH_BYTES inside the library instead of the workspace the
 * handle obtained from its allocator.  The call allocates and frees nothing on the device.  Every
 * GPU the library runs on holds one copy of the array until the process ends, and all handles on
 * a GPU share it: two calls that overlap in time on one GPU (different streams or threads) race
 * on it; calls on one stream are ordered and safe.  The current HIP device must be the stage's.
 * E_UNSUPPORTED (nothing enqueued) if the stage's kernels need more workspace than the array
 * holds; otherwise the errors of bapipe_stage_backward. */
#define BAPIPE_STATIC_SCRATCH_BYTES (64u << 20)
int bapipe_stage_backward_static(bapipe_stage_t *st, int mb_id, const void *dy_dev_or_labels,
                                 void *dx_dev);

/* Weight update after the M backward passes of the mini-batch (Sec. III-B-1): plain SGD
 * w <- w - lr * g on the fp32 masters (weights memory is 2w, Table I: no optimiser state),
 * refresh of the working copies, zeroing of the accumulators, and reset of the micro-batch
 * bookkeeping.  E_ORDER unless exactly M backwards have run since the last step. */
int bapipe_stage_step(bapipe_stage_t *st, float lr);

/* Per-layer profile (Sec. III-A "DNN profile"; Sec. III-B-2 asks for it per batch size, which
 * is the micro_batch the stage was created with).  Runs each layer's forward and backward
 * kernels in isolation on scratch data, `warmup` untimed then `iters` timed repetitions,
 * timed with HIP events on the stage's stream.  Does not change weights, gradients, stash
 * or schedule state; E_ORDER if micro-batches are in flight.  out: host array of `cap`
 * records; *n receives the number of layers; E_INVALID if cap < n_layers.
 * Where the stage runs two layers as one kernel, the time is reported on the layer that launches
 * it and the other reports 0: a max-pool done in the epilogue of the conv before it (forward),
 * a residual ADD whose sum is stored by the batch-norm before it (forward).  Linear layers, whose
 * weight gradient the stage defers to `step`, are timed with that GEMM run per micro-batch: an
 * upper bound for what the schedule pays. */
int bapipe_profile_layers(bapipe_stage_t *st, int warmup, int iters,
                          bapipe_layer_profile_t *out, int cap, int *n);

/* The same profile taken at several micro-batch sizes (Sec. III-B-2: on GPUs small batches may
 * not fill the device, so the profile has to treat the batch size as a variable).  For each of
 * the n_sizes entries of micro_batches a temporary stage is created from the layer list
 * (n_micro = 1, otherwise opts as given), profiled as above and destroyed.  out: host array of
 * n_sizes x n_layers records, row k holding the profile at micro_batches[k].  Errors are those
 * of bapipe_stage_create / bapipe_profile_layers; nothing is left allocated. */
int bapipe_profile_sweep(const bapipe_layer_desc_t *layers, int n_layers, const int *micro_batches,
                         int n_sizes, const bapipe_stage_opts_t *opts, int warmup, int iters,
                         bapipe_layer_profile_t *out);

/* Parameter / result access for checkpoints and parity checks (host buffers, float,
 * PyTorch layouts as described above).  w_host / b_host may be NULL to skip.  Layers
 * without parameters: E_INVALID.  These calls synchronise the stream. */
int bapipe_stage_set_params(bapipe_stage_t *st, int layer, const float *w_host, const float *b_host);
int bapipe_stage_get_params(bapipe_stage_t *st, int layer, float *w_host, float *b_host);
int bapipe_stage_get_grads(bapipe_stage_t *st, int layer, float *dw_host, float *db_host);

/* Arg-max indices (dh*kw+dw, one byte per pooled output, NCHW order) of MAXPOOL2D layer
 * `layer` for a micro-batch that is forwarded and not yet backwarded; else E_ORDER. */
int bapipe_stage_get_pool_indices(bapipe_stage_t *st, int layer, int mb_id, uint8_t *idx_host);

/* Loss of micro-batch mb_id of the current (or just finished) mini-batch; needs a
 * SOFTMAX_XENT last layer and that micro-batch's backward, else E_ORDER. */
int bapipe_stage_get_loss(bapipe_stage_t *st, int mb_id, float *loss_host);

/* Activation-stash accounting: bytes kept per in-flight micro-batch and the ring depth
 * min(M, N-i+1) resp. min(M, 2(N-i+1)) (Table I / II, "Features memory").  LINEAR layers whose
 * weight gradient is formed once per mini-batch keep their input and output gradient of all M
 * micro-batches (beyond the table's (N-i+1) a); that memory is included, divided by depth and
 * rounded up, so that per_mb * depth bounds everything held between a forward and the update.
 * The stash_bytes of bapipe_profile_layers counts it the same way. */
int bapipe_stage_stash_bytes(const bapipe_stage_t *st, uint64_t *per_mb, int *depth);

/* Measurement tap (Sec. III-A profiles layers; this profiles one kernel class inside the real
 * schedule).  While enabled, every launch of the chosen class made by forward / backward is
 * bracketed by two HIP events on the stage's stream.  _read synchronises the stream and
 * returns the summed event time, the number of launches, and the algorithmic work of those
 * launches: FLOP (2 per multiply-accumulate) for the convolution classes, HBM bytes each
 * element must move once for the others.  Reading resets the counters.  The event pool grows
 * as needed up to 262144 launches between reads; beyond that launches go unrecorded and the
 * next _read returns E_UNSUPPORTED instead of an understated sum.  kernel_class < 0 disables
 * the tap.  The events themselves cost a few per cent: time a workload with the tap off. */
enum {
    BAPIPE_KC_CONV_GATHER_MFMA = 0, /* bf16 MFMA forward / dgrad implicit GEMM           */
    BAPIPE_KC_CONV_WGRAD_MFMA = 1,  /* bf16 MFMA wgrad incl. its split-K reduction       */
    BAPIPE_KC_CONV_DIRECT = 2,      /* vector-ALU convolution (fp32 stages, odd channels) */
    BAPIPE_KC_POOL = 3,
    BAPIPE_KC_BATCHNORM = 4,
    BAPIPE_KC_ELEMENTWISE = 5,      /* ReLU, add, gradient copies, bias-gradient sums     */
    BAPIPE_KC_COUNT = 6
};
int bapipe_stage_kernel_timing(bapipe_stage_t *st, int kernel_class);
int bapipe_stage_kernel_timing_read(bapipe_stage_t *st, double *total_ms, uint64_t *launches,
                                    double *flop, double *bytes);

/* Measured ceilings of the current device, for reporting kernel throughput against what this very
 * GPU reaches beside its published peaks (Sec. III-A lists each accelerator's computing power and
 * memory bandwidth among the hardware constraints the framework takes as input): a register-resident
 * bf16 MFMA loop with no memory traffic (TFLOP/s, 2 per multiply-accumulate) and a streaming copy of
 * 256 MiB (GB/s, bytes read + bytes written).  Allocates 0.5 GiB of device memory for the duration
 * of the call, runs on hip_stream and synchronises it.  E_OOM / E_DEVICE on failure. */
int bapipe_measure_peaks(void *hip_stream, double *mfma_bf16_tflops, double *copy_gbs);

/* The third ceiling of the MFMA kernels, which feed the matrix cores from LDS: the rate at which all
 * compute units together read LDS (TB/s, conflict-free addresses, nothing leaves the unit) with
 * ds_read_b128, the fragment load of the forward / input-gradient kernels, and with the transposing
 * ds_read_b64_tr_b16, the fragment load of the weight-gradient kernels (both operands of a weight
 * gradient are contracted over pixels, the dimension that is not contiguous in memory).  A kernel that
 * reads B bytes of fragments per MFMA cannot run the matrix cores above rate / B.  Runs on
 * hip_stream and synchronises it; E_OOM / E_DEVICE on failure. */
int bapipe_measure_lds(void *hip_stream, double *read_b128_tbs, double *read_b64_tr_tbs);

/* Message of the last failed call on this handle (or of the last failed create when st is
 * NULL); valid until the next call on the same handle. */
const char *bapipe_last_error(const bapipe_stage_t *st);

/* Frees everything the handle owns (after synchronising its stream). NULL is allowed. */
void bapipe_stage_destroy(bapipe_stage_t *st);

#ifdef __cplusplus
}
#endif
#endif /* BAPIPE_STAGE_H */
