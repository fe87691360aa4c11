/*
 * dds — one training iteration of data parallelism combined with fully decoupled
 * parallel backpropagation (stale gradients), for one MI355X (gfx950).
 *
 * The network (L layers) is split into K contiguous modules; W data-groups
 * ("replicas") each feed their own mini-batch of B samples per iteration.
 * At iteration t module k0 (zero-based)
 *   - forwards the mini-batch sampled at t-k0 with its current weights,
 *   - back-propagates the mini-batch sampled at t-k0-2*d[k0] with the weights it
 *     held at that batch's forward and the error gradient module k0+1 produced in
 *     an earlier iteration,
 *   - applies  w <- w - lr * (1/W) sum_s g_s  (g_s = mean gradient over replica s's
 *     mini-batch); no update while the backward batch index is negative.
 * (Paper: Section 3.2 forward/backward schedule; Section 3.3 update (a)/(b) with the
 *  mixing matrix P = (1/S) 1 1^T; Algorithm 1, Appendix D.)
 *
 * All pointers named "device" must be device memory of the current HIP device (or
 * host memory the device can address). The library never allocates device memory:
 * the caller provides one arena. All work is enqueued on the stream passed in; side
 * streams used internally are forked from and joined to it with events.
 * Every function returns DDS_OK (0) or a negative error code; dds_last_error()
 * returns a thread-local message for the last failing call. No C++ exceptions cross
 * this boundary. A context is not thread-safe.
 */
#ifndef DDS_H_
#define DDS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  DDS_OK = 0,
  DDS_EINVAL = -1,       /* malformed spec / K / W / delays / arguments */
  DDS_ENOMEM = -2,       /* arena too small */
  DDS_EHIP = -3,         /* a HIP runtime call failed */
  DDS_EUNSUPPORTED = -4  /* valid request the kernels do not cover */
};

/* Layer kinds A_l (Section 2.1: h_l = A_l(h_{l-1}, w_l)). */
enum {
  DDS_OP_CONV2D = 1,    /* cin,cout,ksize,stride,pad; square kernel; has a bias */
  DDS_OP_LINEAR = 2,    /* cin,cout; input must be [N,cin,1,1]; has a bias */
  DDS_OP_RELU = 3,      /* must directly follow CONV2D, LINEAR or RES_ADD */
  DDS_OP_MAXPOOL2 = 4,  /* 2x2 window, stride 2; gradient goes to the first maximum */
  DDS_OP_GAP = 5,       /* global average pool to [N,C,1,1] */
  DDS_OP_RES_BEGIN = 6, /* marks the residual block input x */
  DDS_OP_RES_ADD = 7,   /* y = shortcut(x) + res_scale * y_main. cout == 0: identity
                           shortcut; else a conv(cin,cout,ksize,stride,pad)+bias */
  DDS_OP_SOFTMAX_CE = 8, /* mean softmax cross-entropy; must be the last layer */
  DDS_OP_BATCHNORM = 9  /* cout = channels, res_scale = eps. Training-mode batch normalisation with
                           statistics over each data-group's own mini-batch (biased variance); must
                           directly follow CONV2D or LINEAR, and RES_ADD / RELU may follow it as they
                           follow a convolution. Parameters: gamma [cout] ("weight") then beta [cout]
                           ("bias") in the canonical order, at the position of this layer */
};

enum { DDS_F32 = 0, DDS_BF16_F32MASTER = 1 };
enum { DDS_ACT_STORE = 0, DDS_ACT_RECOMPUTE = 1 };

typedef struct dds_layer {
  int32_t op;
  int32_t cin, cout, ksize, stride, pad;
  float res_scale;
  int32_t reserved;
} dds_layer;

typedef struct dds_spec {
  int32_t n_layers;
  const dds_layer* layers; /* host; n_layers entries */
  const int32_t* bounds;   /* host; K+1 indices: module k0 owns layers[bounds[k0]..bounds[k0+1]) */
  int32_t in_c, in_h, in_w; /* one sample as the caller stores it (NCHW, fp32) */
  int32_t classes;
  int32_t batch;           /* B: samples per replica per iteration */
  int32_t precision;       /* DDS_F32 | DDS_BF16_F32MASTER */
  float lr;                /* default step size (see dds_step) */
  float momentum;          /* 0 = plain SGD; else v <- mu v + g, w <- w - lr v */
  const float* mixing;     /* host; NULL: every data-group mixes with every other with weight 1/W
                              (exact mean, one weight copy per module -- the hot path). Else the
                              W x W row-major matrix P of Section 2.3 (symmetric, rows summing to
                              1, entries in [0,1]); each data-group then keeps its own weights and
                              Section 3.3's update u_s = w_s - lr g_s, w_s <- sum_r P[s][r] u_r runs
                              as written. Read during dds_arena_bytes / dds_create only. */
  int32_t activations;     /* DDS_ACT_STORE | DDS_ACT_RECOMPUTE: what a module with delay d > 0 keeps for the
                              2d iterations between the forward and the backward pass of a mini-batch
                              (Section 3.2: the backward pass at t uses the activations and weights of
                              t - 2d). STORE: every saved tensor, in each of the 2d+1 ring slots. RECOMPUTE:
                              only the module's input and output per slot plus a snapshot of the parameters
                              that forward pass used; the other tensors are rebuilt, bit for bit, by a
                              second forward pass right before the backward pass. Same results, less
                              memory (dds_arena_bytes tells how much; the snapshots cost 4-6 bytes per
                              parameter, slot and weight copy), one more forward per iteration in every
                              module with d > 0. */
} dds_spec;

typedef struct dds_ctx dds_ctx;

/* Integers that drive iteration t (Section 3.2 closed forms). Pure host function, no
 * GPU needed; dds_step executes from the very record this call returns (one function inside the
 * library computes it for both). delays: K per-leg delays d[k0] or NULL for the paper's d[k0] = K-1-k0.
 * out: K records of DDS_SCHED_INTS int32 each:
 *   [0] f = t-k0            mini-batch forwarded (negative: idle)
 *   [1] b = t-k0-2d[k0]     mini-batch back-propagated (negative: idle, no update)
 *   [2] ring depth R = 2d[k0]+1 (saved activations and weight snapshots)
 *   [3] slot written by the forward      = t mod R
 *   [4] slot read by the backward        = (t-2d[k0]) mod R
 *   [5] error-mailbox slot read  (gradient sent by module k0+1), -1 for the last module
 *   [6] error-mailbox slot written (gradient sent to module k0-1), -1 for module 0
 *   [7] label-queue slot read by the last module's forward, -1 otherwise
 *   [8] slot of module k0-1's ring holding this module's input for mini-batch f (module k0-1
 *       forwarded it at iteration f+k0-1; hand-offs are zero-copy), -1 for module 0 or f < 0
 *   [9] the same for mini-batch b, -1 for module 0 or b < 0
 *   [10] label-queue slot of mini-batch b (last module: where its loss gradient starts), -1 otherwise
 *   [11] ring slot that receives the weight snapshot after this iteration's update = (t+1) mod R
 *   [12] label-queue slot the ingest writes = t mod (K + 2d[K-1]) (module 0), -1 otherwise
 * Returns DDS_EINVAL if delays violate d[K-1] >= 0, d[k0] >= d[k0+1]+1. */
#define DDS_SCHED_INTS 13
int dds_schedule(int K, const int* delays, int64_t t, int32_t* out);

/* Bytes of arena dds_create needs for this problem (host computation only). */
int dds_arena_bytes(const dds_spec* spec, int K, int W, const int* delays, size_t* bytes);

/* Builds a context inside the caller's arena (device memory, 256-byte aligned, at
 * least dds_arena_bytes bytes, owned by the caller and kept alive until
 * dds_destroy). Zeroes the arena: all weights are zero until dds_set_params
 * is called. Errors: DDS_EINVAL (spec, K, W in [1,32], delays),
 * DDS_EUNSUPPORTED (layer pattern the kernels do not cover), DDS_ENOMEM, DDS_EHIP. */
int dds_create(const dds_spec* spec, int K, int W, const int* delays, void* arena_device,
               size_t arena_bytes, dds_ctx** out);

int dds_destroy(dds_ctx* ctx);

/* Number of fp32 parameters of a module in canonical order: for every CONV2D /
 * LINEAR / BATCHNORM / RES_ADD-with-projection in layer order, weight [cout,cin,k,k] (linear:
 * [cout,cin]; batch normalisation: gamma [cout]) then bias [cout] (beta). Negative error code
 * on failure. */
int64_t dds_param_count(const dds_ctx* ctx, int module);

/* Copies a module's fp32 master weights to / from dst / src (device-addressable,
 * n_floats == dds_param_count) in canonical order, asynchronously on stream.
 * dds_set_params also refreshes the compute-precision copy and every weight
 * snapshot of the module and clears its momentum; call it before the first step
 * (Algorithm 1 input: the initial weights, identical in every data-group). Every call that
 * reads or writes module state on a stream (these, dds_get_loss, dds_consensus_error) is ordered
 * after the latest dds_step also when that stream is not the one dds_step was given. */
int dds_get_params(dds_ctx* ctx, int module, float* dst_device, size_t n_floats, void* hip_stream);
int dds_set_params(dds_ctx* ctx, int module, const float* src_device, size_t n_floats, void* hip_stream);

/* dds_get_params for the weights of one data-group (Section 3.3: agent (s,k) holds its own
 * w_{s,k}). replica in [0,W). Without a mixing matrix every data-group holds the same
 * weights and this equals dds_get_params; with one, dds_get_params returns data-group 0's
 * and dds_set_params gives all of them the same initial weights. */
int dds_get_params_replica(dds_ctx* ctx, int module, int replica, float* dst_device, size_t n_floats,
                           void* hip_stream);

/* Disagreement between the data-groups' weights as the experiment section measures it:
 * delta = max over layers l and data-groups s of || w_{s,l} - (1/W) sum_r w_{r,l} ||_2, where
 * w_{s,l} is data-group s's weight vector of layer l in the sense of Section 2.1: all parameters
 * of the layer (weight and bias; gamma and beta of a normalisation) as one vector. Accumulated in
 * fp64 from the fp32 master weights. Exactly 0 without a mixing matrix. Synchronises stream. */
int dds_consensus_error(dds_ctx* ctx, double* host_out, void* hip_stream);

/* dds_consensus_error for callers that cannot allocate device memory or hand over a workspace for this
 * call (code under HIP graph capture set-up, tight serving loops, harnesses that forbid allocations): the
 * per-block partial sums of the reduction live in a device array of fixed size inside the library
 * (512 KiB per GPU, held until the process ends) instead of in the arena. Same result as
 * dds_consensus_error, bit for bit. Calls no hipMalloc / hipFree. Limit: every module must satisfy
 * 2 * ceil(parameters of a layer / 1024, summed over layers) * W <= 65536, else DDS_EUNSUPPORTED with a
 * message (nothing is launched). All calls on one GPU share the array: two calls that overlap in time on
 * the same GPU (different streams or threads) race; the array keeps the previous call's contents, which is
 * harmless because the kernel writes every entry that is read back. Synchronises stream. */
int dds_consensus_error_static(dds_ctx* ctx, double* host_out, void* hip_stream);

/* One iteration t of every module (Algorithm 1 loop body for all S*K agents).
 * x_device[s]: replica s's mini-batch, fp32 [B,in_c,in_h,in_w] (NCHW);
 * y_device[s]: its targets, int32 [B], values in [0,classes). Both arrays of
 * pointers are host arrays of W device pointers, borrowed: they are read only by the
 * ingest kernel enqueued by this call. lr: step size for this iteration, or NaN to
 * use spec.lr. Asynchronous on stream: the K module programs run on stream and on internal
 * non-blocking streams (as many streams in all as the runtime has hardware queues, see
 * GPU_MAX_HW_QUEUES; default priority). All of them are joined to stream before the call
 * returns, so work enqueued on stream afterwards sees the whole iteration. A program on an
 * internal stream is ordered after the caller's earlier work on stream in the first
 * iteration and in any iteration that follows a dds_get_params* / dds_set_params /
 * dds_consensus_error / dds_profile call; otherwise (three or more modules) only after the
 * previous iteration of its two neighbour modules, which is all it depends on. stream may
 * differ from call to call: an iteration is then ordered after the previous one by the
 * library. */
int dds_step(dds_ctx* ctx, const float* const* x_device, const int32_t* const* y_device, float lr,
             void* hip_stream);

/* Step-size rules of the experiment section and of the diminishing step-size section, for
 * callers that want eta_t computed the paper's way (pure host function, no GPU needed):
 *   DDS_ETA_CONSTANT     Strategy I : eta_t = eta0 for all t (the paper uses eta0 = 0.1)
 *   DDS_ETA_PIECEWISE    Strategy II: eta0 while t <= 15000, eta0/10 while t <= 30000, eta0/100
 *                        while t <= 40000, eta0/1000 after (0.1, 0.01, 0.001, 0.0001 for eta0 = 0.1)
 *   DDS_ETA_DIMINISHING  eta_t = eta0 / (t + 1)
 * Returns eta_t, or NaN for an unknown rule or t < 0. dds_step's lr multiplies the mean of the
 * data-groups' mean gradients: with W equal partitions the paper's update corresponds to
 * lr = eta_t / W. */
enum { DDS_ETA_CONSTANT = 1, DDS_ETA_PIECEWISE = 2, DDS_ETA_DIMINISHING = 3 };
float dds_step_size(int rule, int64_t t, float eta0);

/* Mean loss of the mini-batch the last module forwarded in the latest step (sampled
 * K-1 iterations earlier): mean over each replica's B samples, then over replicas.
 * Synchronises stream. DDS_EINVAL if no loss exists yet (fewer than K steps). */
int dds_get_loss(dds_ctx* ctx, float* host_out, void* hip_stream);

/* Iterations executed so far. */
int64_t dds_step_count(const dds_ctx* ctx);

/* Introspection for tests and the benchmark (host only): number of kernel launches
 * of the latest step, and per-step algorithmic FLOPs of the conv/linear kernels
 * (2*M*N*K over forward, dgrad and wgrad launches of a steady-state step). */
int64_t dds_launches_last_step(const dds_ctx* ctx);
double dds_gemm_flops_per_step(const dds_ctx* ctx);

/* Per-launch timing of the MFMA kernels for the benchmark's roofline record. While
 * enabled every conv/linear forward, dgrad and wgrad launch is bracketed by HIP events on
 * the stream it is launched on and dds_step synchronises at its end (do not time
 * throughput in this mode). enable = 1: modules stay on their concurrent streams, so a
 * launch's duration includes the time it shares the chip with other modules' kernels;
 * enable = 2: modules run one after another on the caller's stream, so every launch has
 * the chip to itself; 0: off. Enabling also clears the totals.
 * dds_profile_read fills 18 doubles: for each of six classes summed milliseconds, number of
 * launches, summed algorithmic FLOPs (2*M*N*K). Classes 0 forward, 1 dgrad, 2 wgrad launches
 * taken by the generic implicit-GEMM kernels; 3, 4, 5 the same three kinds taken by the
 * asynchronous global->LDS kernels (3x3 stride-1 forward / dgrad; 3x3 and stride-2 wgrad). */
int dds_profile(dds_ctx* ctx, int enable);
int dds_profile_read(const dds_ctx* ctx, double* out18);

/* Test-only raw view of the delay buffers, so that batch assignment and slot indexing of Section 3.2
 * (forward of mini-batch t-k0 into slot t mod R; backward of mini-batch t-k0-2d from slot (t-2d) mod R
 * with the weights of that slot) can be checked bit for bit on the device. Copies one region, as stored,
 * to dst_device (asynchronous on stream, ordered after the latest dds_step); bytes must equal
 * dds_debug_bytes(ctx, what, module, index). Regions:
 *   DDS_DBG_INPUT     module 0, ring slot: the ingested mini-batch, [W*B][H][W][Cpad] in the compute
 *                     precision (Cpad = in_c rounded up to a 16-byte chunk, pad lanes zero)
 *   DDS_DBG_OUTPUT    ring slot: the module's output tensor, same layout (logits of the last module: fp32)
 *   DDS_DBG_ERROR     mailbox slot of the error gradient module+1 sent to this module (layout of its output)
 *   DDS_DBG_LABELS    label-queue slot: int32 [W*B] (module is ignored but must be valid)
 *   DDS_DBG_SNAPSHOT  ring slot, index = the module's layer in canonical order: the weight snapshot the
 *                     backward reads, transposed [cin][k*k][cout rounded up to a 16-byte chunk], compute
 *                     precision; DDS_EINVAL for a layer nothing back-propagates through
 * dds_debug_bytes returns the size in bytes or a negative error code. */
enum { DDS_DBG_INPUT = 0, DDS_DBG_OUTPUT = 1, DDS_DBG_ERROR = 2, DDS_DBG_LABELS = 3, DDS_DBG_SNAPSHOT = 4 };
int64_t dds_debug_bytes(dds_ctx* ctx, int what, int module, int index);
int dds_debug_read(dds_ctx* ctx, int what, int module, int index, int slot, void* dst_device, size_t bytes,
                   void* hip_stream);

const char* dds_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* DDS_H_ */
