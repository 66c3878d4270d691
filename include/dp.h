/*
 * dp.h -- C ABI of the per-layer training-compute library for MI355X (gfx950).
 *
 * The operations are the per-layer forward and backward computations whose
 * time, at per-GPU batch B/g, is the planner input comp(i,g) of burst-parallel
 * training (paper, section 4.1 "Computation cost"), for the "Conv, Dense"
 * layer kinds of the evaluated models (paper, Table 1).  The paper treats the
 * layers as black boxes; their arithmetic is the standard deep-learning
 * definition (cross-correlation, zero padding, floor output size).
 *
 * Conventions that hold for every call unless stated otherwise:
 *  - All tensor pointers are DEVICE pointers owned by the caller; the library
 *    never allocates, frees or keeps them (dp_profile_layer is the exception,
 *    see there).  Descriptors and row arrays are HOST pointers.
 *  - Layouts are dense: activations NHWC, conv weights KRSC (K = c_out),
 *    dense-layer weights [out_features, in_features].
 *  - io_dtype DP_BF16: x, w, y, dy, dx are bfloat16 (raw 16-bit), products are
 *    accumulated in fp32 on the matrix cores, y / dx are rounded to bf16
 *    (nearest-even).  io_dtype DP_F32: everything fp32, plain fp32 FMA.
 *    bias, dw, dW, dbias are always fp32.
 *  - Outputs are fully overwritten (no accumulation into dw).
 *  - Calls enqueue work on `hip_stream` (a hipStream_t; NULL = default stream)
 *    and return without synchronising.  Arguments are validated before any
 *    launch, so every error path can be reached on a host without a GPU.
 *  - Tensor pointers must be 16-byte aligned; every tensor must hold fewer than
 *    2^31 elements.
 *  - Results are deterministic: split reductions are summed in a fixed order,
 *    no floating-point atomics are used.
 *  - Return value: DP_OK or an error code; dp_last_error() gives a message for
 *    the calling thread's most recent failure.
 */
#ifndef DP_H
#define DP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DP_OK = 0,
    DP_ERR_NULL = 1,        /* a required pointer is NULL */
    DP_ERR_BAD_DESC = 2,    /* non-positive size, empty output, misaligned pointer, too many elements */
    DP_ERR_UNSUPPORTED = 3, /* unknown dtype / flag / pass */
    DP_ERR_WORKSPACE = 4,   /* workspace missing or smaller than dp_*_workspace_bytes() */
    DP_ERR_HIP = 5          /* a HIP runtime call failed (no device, launch error, ...) */
} dp_status;

typedef enum { DP_F32 = 0, DP_BF16 = 1 } dp_dtype;

enum {
    DP_BIAS = 1u,          /* forward adds bias[c_out] */
    DP_RELU = 2u,          /* forward applies max(.,0) after the bias */
    DP_DETERMINISTIC = 4u, /* results are bitwise reproducible for a given kernel choice in any case (ordered
                              reductions, no float atomics); this flag also keeps the call on the analytic kernel
                              choice when dp_set_autotune is on, so that the choice cannot differ between processes */
    DP_DX_F32 = 8u,        /* bf16 path only: dx is written as fp32 instead of bf16 */
    DP_RELU_IN = 16u       /* the layer's input x is the output of a ReLU: backward-data also applies that ReLU's
                              backward, dx *= [x > 0], in its epilogue (needs the saved input: dp_conv2d_bwd_data_relu,
                              or x in dp_linear_fwd_bwd).  The gradient then reaches the preceding layer already
                              masked, so that layer passes y_saved = NULL and needs no pointwise pass of its own */
};

enum { DP_PASS_FWD = 0, DP_PASS_DGRAD = 1, DP_PASS_WGRAD = 2 };

/* One conv2d layer at per-GPU batch n.  dilation 1, groups 1.
 * Output size: ho = (h + 2*pad_h - r) / stride_h + 1 (floor), same for wo. */
typedef struct {
    int32_t n, h, w, c_in, c_out, r, s, stride_h, stride_w, pad_h, pad_w;
    int32_t io_dtype; /* dp_dtype */
    uint32_t flags;
} dp_conv_desc;

/* One dense layer at per-GPU batch n. */
typedef struct {
    int32_t n, in_features, out_features;
    int32_t io_dtype; /* dp_dtype */
    uint32_t flags;   /* DP_BIAS, DP_RELU, DP_DX_F32, DP_RELU_IN */
} dp_linear_desc;

/* Bytes of device scratch the given pass (DP_PASS_*) of this layer needs.
 * 0 is a valid answer.  Returns 0 for an invalid descriptor. */
size_t dp_conv2d_workspace_bytes(const dp_conv_desc *desc, int pass);
size_t dp_linear_workspace_bytes(const dp_linear_desc *desc);

/* Forward: y[n,p,q,k] = bias[k] + sum_{r,s,c} x[n, p*sh-ph+r, q*sw-pw+s, c] * w[k,r,s,c],
 * then ReLU if DP_RELU.  (Layer forward pass of comp(i,g), paper section 4.1.)
 * x [n,h,w,c_in], w [c_out,r,s,c_in], bias [c_out] fp32 (required iff DP_BIAS),
 * y [n,ho,wo,c_out].  ws: device scratch of >= dp_conv2d_workspace_bytes(desc, DP_PASS_FWD). */
dp_status dp_conv2d_fwd(const dp_conv_desc *desc, const void *x, const void *w, const float *bias,
                        void *y, void *ws, size_t ws_bytes, void *hip_stream);

/* Backward data: dx[n,h,w,c] = sum_{k,r,s} g[n,p,q,k] * w[k,r,s,c] over the (p,q) with
 * p*sh-ph+r == h and q*sw-pw+s == w, where g = dy * [y_saved > 0] if y_saved is given
 * (the layer's stored post-ReLU output), else g = dy.  (Backward pass of comp(i,g),
 * paper section 4.1; "gradients during backward passes", section 4.1 "Communication cost".)
 * dy, y_saved [n,ho,wo,c_out]; dx [n,h,w,c_in] in io_dtype (fp32 if DP_DX_F32). */
dp_status dp_conv2d_bwd_data(const dp_conv_desc *desc, const void *dy, const void *y_saved_or_null,
                             const void *w, void *dx, void *ws, size_t ws_bytes, void *hip_stream);

/* The same with the backward of the ReLU in front of the layer fused into the epilogue (activation work
 * fused into the producing kernel): with DP_RELU_IN in desc->flags, dx[n,h,w,c] is set to 0 where
 * x_saved[n,h,w,c] <= 0.  x_saved [n,h,w,c_in] in io_dtype is the layer's forward input (post-ReLU output
 * of the preceding layer, or its 2x2 max-pooled version: masking the pooled gradient by [pooled > 0] and
 * then routing it through the pooling backward equals routing first and masking by [unpooled > 0]).
 * Without the flag x_saved is ignored and may be NULL; dp_conv2d_bwd_data rejects the flag (no x_saved). */
dp_status dp_conv2d_bwd_data_relu(const dp_conv_desc *desc, const void *dy, const void *y_saved_or_null,
                                  const void *w, const void *x_saved, void *dx, void *ws, size_t ws_bytes,
                                  void *hip_stream);

/* Backward filter: dw[k,r,s,c] = sum_{n,p,q} g[n,p,q,k] * x[n, p*sh-ph+r, q*sw-pw+s, c];
 * dbias[k] = sum_{n,p,q} g[n,p,q,k] if dbias is given.  g as in dp_conv2d_bwd_data.
 * dw [c_out,r,s,c_in] fp32, dbias [c_out] fp32.  These are the per-layer gradients that
 * data-parallel training sums across GPUs (paper section 4.1, sync(i,g)). */
dp_status dp_conv2d_bwd_filter(const dp_conv_desc *desc, const void *x, const void *dy,
                               const void *y_saved_or_null, float *dw, float *dbias_or_null,
                               void *ws, size_t ws_bytes, void *hip_stream);

/* dp_conv2d_bwd_filter for callers that cannot allocate or pass a workspace: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, results and errors, minus ws: split partials,
 * the masked gradient and bias-gradient sums go to a scratch array built into the library (DP_NOALLOC_SCRATCH_BYTES
 * of device memory per GPU, held from the library's load until the process ends).  The call allocates nothing on the
 * device (no hipMalloc / hipFree / events) and always uses the analytic kernel choice (dp_set_autotune is ignored).
 * A layer whose pass needs more scratch than that (dp_conv2d_workspace_bytes(desc, DP_PASS_WGRAD) with the measured
 * choice off) is rejected with DP_ERR_WORKSPACE before any launch.  The first call on a device looks the array's
 * address up on that device (hipGetSymbolAddress, device current) and performs the library's one-time kernel
 * set-up: make it outside a capture.  All calls on one GPU share the one array: calls that overlap on a GPU
 * (different streams or threads) race; serialise them.  Nothing in it has to be cleared between calls. */
#define DP_NOALLOC_SCRATCH_BYTES ((size_t)32 << 20)
dp_status dp_conv2d_bwd_filter_noalloc(const dp_conv_desc *desc, const void *x, const void *dy,
                                       const void *y_saved_or_null, float *dw, float *dbias_or_null,
                                       void *hip_stream);

/* Dense layer, forward and/or backward in one call (paper Table 1 "Dense"; section 4.1):
 *   y = x W^T + bias (ReLU if DP_RELU)                       if y != NULL   (needs x, W)
 *   g = dy * [y_saved > 0] (or dy);  dx = g W; dW = g^T x; dbias = sum_n g
 *                                                            each if its pointer != NULL
 * x [n,in], W [out,in], dy / y / y_saved [n,out], dx [n,in], dW [out,in] fp32, dbias [out] fp32.
 * Backward outputs need dy; dW needs x.  At least one output must be requested.
 * With DP_RELU_IN, dx is multiplied by [x > 0] (needs x). */
dp_status dp_linear_fwd_bwd(const dp_linear_desc *desc, const void *x, const void *W,
                            const float *bias, const void *dy, const void *y_saved_or_null,
                            void *y, void *dx, float *dW, float *dbias,
                            void *ws, size_t ws_bytes, void *hip_stream);

/* ReLU gradient and bias gradient of a [rows, k] activation matrix
 * (the pointwise part of a layer's backward pass, paper section 4.1):
 *   g = dy * [y_saved > 0];  g_out = g (if g_out != NULL, in io_dtype);
 *   dbias[j] = sum_rows g[., j] (if dbias != NULL, fp32).
 * ws: device scratch of >= dp_relu_bias_grad_workspace_bytes(rows, k) when dbias is requested. */
size_t dp_relu_bias_grad_workspace_bytes(int64_t rows, int32_t k);
dp_status dp_relu_bias_grad(int64_t rows, int32_t k, int32_t io_dtype, const void *dy,
                            const void *y_saved, void *g_out_or_null, float *dbias_or_null,
                            void *ws, size_t ws_bytes, void *hip_stream);

/* One row of the time-versus-batch table comp(i,g) the planner consumes
 * (paper section 4.1: each layer is profiled at every per-GPU batch size and the
 * forward and backward times are summed). */
typedef struct {
    int32_t batch;
    float fwd_us, dgrad_us, wgrad_us; /* average time of one launch, microseconds */
    double flops_per_pass;            /* 2*n*ho*wo*c_out*r*s*c_in (2*n*in*out for dense) */
    double min_bytes_fwd, min_bytes_dgrad, min_bytes_wgrad; /* algorithmic HBM bytes */
} dp_profile_row;

/* Time forward, backward-data and backward-filter of one layer at each batch in `batches`.
 * Exactly one of conv / linear is non-NULL; its n field is ignored.  For each batch the
 * call allocates device buffers itself (hipMalloc/hipFree), fills them with a fixed
 * pattern, runs `warmup` untimed and `iters` timed back-to-back launches of each pass
 * between HIP events on `hip_stream`, and synchronises: the only blocking call here.
 * For a dense layer fwd_us is the y pass, dgrad_us the dx pass, wgrad_us the dW+dbias pass.
 * The backward passes mask the incoming gradient with the saved output when the flags have DP_RELU; with
 * DP_RELU_IN as well they run as in a step where each ReLU is differentiated by the layer behind it
 * (y_saved = NULL, dx *= [x > 0]).  One untimed call per pass precedes the warm-up, so the measured kernel
 * choice (dp_set_autotune) never times its candidates inside the timed window, whatever `warmup` is.
 * rows_out: host array of n_batches rows. */
dp_status dp_profile_layer(const dp_conv_desc *conv, const dp_linear_desc *linear,
                           const int32_t *batches, int32_t n_batches, int32_t warmup,
                           int32_t iters, dp_profile_row *rows_out, void *hip_stream);

/* Names the main kernel this pass of the layer would launch, as the profiler prints it
 * (e.g. "k_conv_gemm<0, 128, 128, 32, 2, 2, true, true>"), and its number of reduction
 * splits (> 1 means a second, small reduction kernel follows; < -1: that many splits, summed inside the main kernel
 * by the last block to finish each output tile, so no second kernel follows).  Host-only, no launch.
 * The backward passes are named for a call that passes no saved output (y_saved = NULL, the gradient
 * arrives already masked) and, for the filter gradient, asks for the bias gradient too; a few shapes run
 * another kernel when dy still has to be masked.
 * name: host buffer of name_bytes; either output pointer may be NULL. */
dp_status dp_conv2d_kernel_info(const dp_conv_desc *desc, int pass, char *name, size_t name_bytes,
                                int32_t *splits);

/* Tuning hook: force the tile variant (>= 0) and/or the number of reduction splits (> 0)
 * used by the given pass; -1 / 0 restore the built-in choice.  Process-wide.
 * tile_variant 1000 + v (forward, backward-data): variant v, and if v is a pipelined kernel with a reduction split,
 * the splits are summed inside that kernel (dp_conv2d_kernel_info then reports -splits).  The built-in choice never
 * takes this form: on one GPU it measured no faster than the reduction kernel it saves.  Such launches share a ring
 * of 65536 tile counters, handed out in launch order (at most 1024 per launch): a launch must have finished before
 * 64 later ones of this form are enqueued on other streams. */
dp_status dp_set_override(int pass, int tile_variant, int splits);

/* Measured kernel choice (the paper's layer profiler, Section 3 "profiling", applied to the
 * library's own kernels): enabled != 0 makes the first launch of a pass on a new layer shape time
 * the analytic model's best tile/split candidates on the caller's own buffers and stream (each
 * candidate writes the same result; the stream is drained, so that one call blocks the host) and
 * keeps the fastest for later calls of every thread (a shape is measured once per process; a thread that asks for
 * a shape while another is measuring it waits for that choice).  Workspace queries made while it is on
 * return the largest need of any candidate, so query after switching it on.  No measurement takes
 * place while the stream is being captured (the model's choice is used), with a forced override,
 * or for fp32.  0 (the default) restores the purely analytic choice.  Process-wide.
 * enabled == 2 measures COLD: before every timed launch a kernel reads a 384 MiB buffer (allocated by the library on
 * first use and kept until the process ends), so the candidate finds its operands in HBM rather than in the L2 / memory-side
 * caches -- the state a layer meets inside a training step, where the traffic of the other layers has gone through the
 * caches since its operands were last touched.  Any other non-zero value measures warm (back-to-back launches). */
dp_status dp_set_autotune(int enabled);

/* Per-kernel timing of the calling thread's compute calls, for benchmarks (the measured side of a roofline).
 * Between dp_trace_begin and dp_trace_end every conv / dense pass records three HIP events on the stream it is
 * given: before its first kernel, after its main kernel (the implicit-GEMM kernel; a split-reduce or column-sum
 * kernel may follow) and after its last kernel.  dp_trace_end waits for the events (it blocks until the traced
 * work is done), writes one row per pass in call order (at most max_rows; a dense call yields one row per
 * half it ran) and frees the events.  kernel: the main kernel as the profiler prints it; main_us: first event to
 * second; total_us: first to third.  Tracing creates events: not for use under stream capture.  Passes that
 * the measured kernel choice (dp_set_autotune) uses for its measurement are timed from the end of that measurement. */
typedef struct {
    char kernel[96];
    int32_t pass;   /* DP_PASS_* */
    int32_t splits; /* reduction splits of the plan that ran (> 1: a reduce kernel follows the main kernel; < -1: summed inside it) */
    float main_us, total_us;
} dp_trace_row;
dp_status dp_trace_begin(void);
dp_status dp_trace_end(dp_trace_row *rows, int32_t max_rows, int32_t *n_rows);

/* ---- Glue layers of a whole training step (paper Table 1 counts VGG-16's pooling layers among its 21
 * layers; the paper gives no arithmetic for them).  Pointwise, HBM-bound, asynchronous on hip_stream, no
 * workspace, deterministic.  Device pointers, 16-byte aligned. ---------------------------------------- */

/* 2x2 max pooling at stride 2 without padding, NHWC: y[n,p,q,c] = max of x[n,2p..2p+1,2q..2q+1,c];
 * y is [n, h/2, w/2, c] (a trailing odd row / column of x is dropped; with h < 2 or w < 2 there is no
 * window, y is empty and may be NULL).  io_dtype DP_BF16 or DP_F32. */
dp_status dp_maxpool2x2_fwd(int32_t n, int32_t h, int32_t w, int32_t c, int32_t io_dtype, const void *x, void *y,
                            void *hip_stream);
/* dx[n,h,w,c] = dy of its window if x there is the window's FIRST maximum in row-major order
 * ((0,0),(0,1),(1,0),(1,1)), else 0; every element of dx is written (dy may be NULL when there is no
 * window).  x is the forward input. */
dp_status dp_maxpool2x2_bwd(int32_t n, int32_t h, int32_t w, int32_t c, int32_t io_dtype, const void *x,
                            const void *dy, void *dx, void *hip_stream);

/* Softmax cross-entropy with integer labels: *loss = mean over the n rows of logsumexp(z_r) - z_r[label_r]
 * (fp32, device); dz = (softmax(z) - onehot(label)) / n in io_dtype (may be NULL).  z [n, classes] in
 * io_dtype; labels [n] int32 on the device, each in [0, classes) (a label outside contributes
 * logsumexp only and no one-hot term).  fp32 arithmetic; rows are summed in a fixed order. */
dp_status dp_softmax_xent(int32_t n, int32_t classes, int32_t io_dtype, const void *z, const int32_t *labels,
                          float *loss, void *dz, void *hip_stream);

/* SGD with momentum on fp32 master weights, in place: mom = momentum*mom + grad; w32 -= lr*mom; if
 * w_bf16 is not NULL it receives w32 rounded to nearest-even bf16 (the copy the next forward reads).
 * No dampening, Nesterov term or weight decay.  count elements. */
dp_status dp_sgd_update(int64_t count, float lr, float momentum, const float *grad, float *mom, float *w32,
                        void *w_bf16, void *hip_stream);

/* ---- Burst-parallel plan of a chain of layers (host only: no GPU call, all pointers host) -------
 * Paper section 4.2, algorithm "Search Linear": dynamic programming over two tables,
 *   S[i][g] = earliest finish of layer i when it runs on g GPUs, over the predecessor choices the search admits,
 *   T[i][g] = layer i's own share of that finish time (transition into it + its compute + its gradient sync),
 * admitting a predecessor GPU count h only while its GPU-sec amplification
 *   Amp(i-1,h) = T[i-1][h] * h / comp(i-1,1)
 * is within max(best amplification admitted so far, amp_limit) and S[i-1][h] + comm does not exceed
 * the best so far (ties take the later h; the first h scanned is always admitted).  Layer 0 does not
 * exist: S[0][g] = 0 and Amp(0,h) = 0.  The last layer's GPU count is chosen by the same admission
 * scan with zero transition cost, then the predecessors are traced back.
 * Tables are dense row-major doubles; index a / b runs over gpu_counts. */
typedef struct {
    int32_t n_layers;          /* L >= 1 */
    int32_t n_gpu_counts;      /* G >= 1 */
    const int32_t *gpu_counts; /* [G] strictly ascending, gpu_counts[0] == 1 */
    const double *comp;        /* [L][G] comp(i,g): forward+backward time of layer i on g GPUs, > 0, e.g. the
                                  dp_profile_layer times at per-GPU batch B/g */
    const double *comm;        /* [L][G][G] comm[i][b][a]: transition from layer i-1 on gpu_counts[b] to layer i
                                  on gpu_counts[a] (i = 0: into the first layer); NULL = all zero */
    const double *sync;        /* [L][G] sync(i,g): gradient synchronisation of layer i; NULL = all zero */
    double amp_limit;          /* GPU-sec amplification limit; INFINITY = none (plain shortest path) */
} dp_plan_desc;

/* gpus_per_layer [L]: GPU count of each layer; iteration_time: S[L][g_L]; S_out / T_out: [(L+1)][G]
 * including row 0, either may be NULL.  DP_ERR_NULL / DP_ERR_BAD_DESC on missing or malformed input
 * (non-ascending counts, first count != 1, non-finite or non-positive comp, negative costs). */
dp_status dp_plan_chain(const dp_plan_desc *desc, int32_t *gpus_per_layer, double *iteration_time,
                        double *S_out, double *T_out);

/* Closed-form costs of paper section 4.1 (payload over per-GPU bandwidth plus a propagation delay, full
 * bisection).  act_bytes[i]: bytes of the global batch entering layer i (act_bytes[0], the network input, is
 * never redistributed: comm[0] = 0); param_bytes[i]: gradient bytes of layer i.
 *   comm (g != h) = 2 * (act_bytes * (1/min(g,h) - 1/max(g,h)) / bandwidth + delay)   forward + backward
 *   sync (g > 1)  = 2 * (param_bytes * (g-1)/g / bandwidth + delay)                   reduce-scatter + all-gather
 * comm_out [L][G][G], sync_out [L][G]. */
dp_status dp_plan_cost_tables(int32_t n_layers, int32_t n_gpu_counts, const int32_t *gpu_counts,
                              const double *act_bytes, const double *param_bytes, double bandwidth,
                              double delay, double *comm_out, double *sync_out);

/* ---- Burst-parallel plan of a chain whose edges may be branch/join blocks (host only) -------------
 * Paper section 4.2, paragraph "Multi-chain graph reduction".  Between main layers i-1 (the branching
 * layer) and i (the joining layer) there may be n_branches[i] parallel branches instead of a direct
 * edge.  For every GPU count g of the branching layer each branch is searched as a chain whose layer 0
 * is pinned to g; for every GPU count h of the joining layer each branch's time to reach it is chosen
 * by the chain algorithm's admission scan over the branch's last layer (transition cost join).  The
 * longest branch is critical (first on ties).  Branches run one after another unless moved aside: a
 * non-critical branch with layers is moved to a GPU set of its own (as many GPUs as the largest count
 * on its plan) when time + move[g][h] <= critical time and the block's amplification
 *   (block time + comp(i,h) + sync(i,h)) * (h + GPUs added so far + its own) / one-GPU compute of the
 *   joining layer and all branch layers
 * stays within amp_limit; candidates are tried in branch order.  The block's time tr[g][h] = critical +
 * the branches not moved; it takes the place of comm[i] in the chain algorithm, and the joining layer's
 * amplification counts the added GPUs and the block's one-GPU compute.  Blocks do not nest. */
typedef struct {
    int32_t n_layers;   /* Lb >= 0; 0 = a skip connection whose time is join[g][h] */
    const double *comp; /* [Lb][G], > 0 */
    const double *comm; /* [Lb][G][G]; comm[0][b][a] leaves the branching layer on gpu_counts[b]; NULL = zero */
    const double *sync; /* [Lb][G]; NULL = zero */
    const double *join; /* [G][G] join[b][a]: from the branch's last layer (the branching layer if Lb = 0) on
                           gpu_counts[b] to the joining layer on gpu_counts[a]; NULL = zero */
    const double *move; /* [G][G] move[g][h]: cost of taking the branch's samples to a GPU set of its own and
                           back; entries may be INFINITY; NULL = the branch is never moved */
} dp_plan_branch;

typedef struct {
    dp_plan_desc chain;             /* the main layers; chain.comm[i] is not read where n_branches[i] > 0 */
    const int32_t *n_branches;      /* [L] >= 0, n_branches[0] == 0 */
    const dp_plan_branch *branches; /* the branches of all blocks, in layer order; may be NULL if there are none */
} dp_plan_graph_desc;

/* gpus_per_layer [L]; branch_gpus: GPU count of every branch layer along the chosen plan, branches
 * concatenated in the order of desc->branches (may be NULL); branch_parallel: one byte per branch, 1 =
 * moved aside (may be NULL); critical_branch [L]: index of the critical branch within its block, -1 for a
 * direct edge (may be NULL); S_out / T_out [(L+1)][G] (may be NULL).  Errors as dp_plan_chain. */
dp_status dp_plan_graph(const dp_plan_graph_desc *desc, int32_t *gpus_per_layer, int32_t *branch_gpus,
                        uint8_t *branch_parallel, int32_t *critical_branch, double *iteration_time,
                        double *S_out, double *T_out);

const char *dp_last_error(void); /* thread-local, static storage */
const char *dp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DP_H */
