/*
 * rev_stack.h -- C ABI of the reversible transformer stack on MI355X (gfx950).
 *
 * One block of the stack is the two-stream reversible map of the paper's Eq. 1
 * (Sec. 3.1), written here with X/Y names (I1->X2, I2->X1, O2->Y1, O1->Y2):
 *
 *      Y1 = X1 + F(X2)          F(x) = Proj(MHA(LN1(x)))      attention branch
 *      Y2 = X2 + G(Y1)          G(x) = fc2(gelu(fc1(LN2(x)))) MLP branch   (Sec. 3.2)
 *
 * and its inverse (Sec. 3.1, one call of F and one of G):
 *
 *      X2 = Y2 - G(Y1)          X1 = Y1 - F(X2)
 *
 * Readings the paper leaves open: LayerNorm sits inside each branch (pre-LN),
 * uses the biased variance and eps = cfg.ln_eps; attention is softmax(q k^T /
 * sqrt(head_dim)) v with no mask and no dropout; GELU is the erf form x*Phi(x)
 * (REV_MODE_FP32 evaluates erf; REV_MODE_BF16 evaluates Phi with a fitted
 * polynomial of absolute error < 6.5e-5 on |x| <= 3.8 and takes exactly 0 / 1
 * beyond); every linear map has a bias.
 *
 * All pointers except `cfg` are DEVICE pointers owned by the caller; the library
 * allocates no device memory, frees none, and keeps no state between calls
 * except a pool of HIP events.  Every call only enqueues work and returns; on
 * return the work is ordered before anything enqueued later on the stream the
 * call was given (for the PaReprop entry: on `stream_grad`).  Inputs are never
 * written.  Outputs and the workspace are fully overwritten; they must not
 * overlap each other or the inputs.  Calls may be issued concurrently from
 * several host threads as long as every call in flight has its own workspace,
 * its own streams and its own outputs (each two-stream call leases its own set
 * of events from the pool); the rev_profile_* calls are the exception and are
 * not thread safe.
 *
 * Layouts.  Activations and cotangents X1, X2, Y1, Y2, dY1, dY2, dX1, dX2 are
 * float32, row-major [batch, seq_len, d_model] (token-major, features
 * contiguous) in BOTH modes.  `params` is one packed vector, block after block,
 * each block holding, in this order (linear weights are [out, in] row-major;
 * the rows of w_qkv are ordered q | k | v, then head, then head_dim):
 *
 *      ln1_g[D] ln1_b[D] w_qkv[3D,D] b_qkv[3D] w_proj[D,D] b_proj[D]
 *      ln2_g[D] ln2_b[D] w_fc1[Dm,D] b_fc1[Dm] w_fc2[D,Dm] b_fc2[D]
 *
 * Element type of `params`: float32 in REV_MODE_FP32, bfloat16 in
 * REV_MODE_BF16.  `dparams` has the same layout, is always float32 and is
 * overwritten (not accumulated into).
 *
 * Modes.  REV_MODE_FP32: all storage and arithmetic float32.  REV_MODE_BF16:
 * parameters and the per-block activations held in the workspace are bf16,
 * the dense contractions run on bf16 matrix cores with float32 accumulation;
 * residual streams, cotangent streams, LayerNorm statistics, softmax
 * statistics and all parameter gradients stay float32.
 *
 * Limits (anything else returns REV_EINVAL before any work is enqueued):
 * all six sizes positive; d_model % n_heads == 0; d_model % 8 == 0;
 * d_mlp % 8 == 0; head_dim % 8 == 0 and head_dim <= 128; d_model <= 8192;
 * d_mlp <= 32768; batch*seq_len <= 4194240 and batch*n_heads <= 65535 (launch-
 * grid limits).
 *
 * Errors.  Every int-returning call returns REV_OK (0) or a negative code; the
 * text of the last failure on the calling thread is returned by
 * rev_last_error().  Nothing throws or aborts across this boundary.
 */
#ifndef REV_STACK_H
#define REV_STACK_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define REV_MODE_FP32 0
#define REV_MODE_BF16 1

#define REV_OK          0
#define REV_EINVAL     -1   /* null pointer, bad size, unsupported shape or mode */
#define REV_EWORKSPACE -2   /* workspace smaller than rev_stack_workspace_bytes  */
#define REV_EHIP       -3   /* a HIP runtime call failed                          */

typedef struct rev_cfg {
    int32_t n_blocks;   /* N: number of reversible blocks                    */
    int32_t d_model;    /* D: width of each residual stream                  */
    int32_t n_heads;    /* H: attention heads, head_dim = D / H              */
    int32_t d_mlp;      /* Dm: hidden width of the MLP branch                */
    int32_t seq_len;    /* T: tokens per sample                              */
    int32_t batch;      /* B: samples                                        */
    int32_t mode;       /* REV_MODE_FP32 or REV_MODE_BF16                    */
    float   ln_eps;     /* LayerNorm epsilon (the paper is silent; 1e-6)     */
} rev_cfg;

/* Validates cfg; REV_OK or REV_EINVAL.  Host only, touches no GPU. */
int rev_stack_check_cfg(const rev_cfg* cfg);

/* Number of elements of the packed parameter vector (N * per-block count), or
 * a negative error code.  Host only. */
int64_t rev_stack_param_count(const rev_cfg* cfg);

/* Element offset of tensor `tensor` (0..11 in the order listed above) of block
 * `block` inside the packed vector, and its element count in *count (nullable).
 * Negative error code on bad arguments.  Host only. */
int64_t rev_stack_param_offset(const rev_cfg* cfg, int32_t block, int32_t tensor, int64_t* count);

/* Bytes of device workspace that is enough for every entry point below
 * (a multiple of 256).  Negative error code on bad cfg.
 * Holds: two activation slots (the per-block intermediates a gradient step
 * consumes; the second slot is what lets block i-1 be recomputed while block i
 * is still being differentiated, Sec. 3.2/3.3), a ring of three residual-stream
 * levels, two cotangent levels, gradient temporaries and the partial sums of
 * the deterministic reductions.  Host only. */
int64_t rev_stack_workspace_bytes(const rev_cfg* cfg);

/* Bytes of the smaller workspace that rev_stack_forward and
 * rev_stack_backward_reprop accept: with one stream nothing of block i-1 is
 * produced while block i is still being consumed, so ONE activation slot, two
 * residual-stream levels and single gradient temporaries suffice.  The
 * difference to rev_stack_workspace_bytes is the extra memory the parallel
 * schedule pays for its speed (Sec. 3.3; memory trends, Sec. 4.2).  Host only. */
int64_t rev_stack_workspace_bytes_reprop(const rev_cfg* cfg);

/* Bytes of one activation slot: the intermediates of ONE block that a gradient
 * step consumes (normalised inputs, QKV, attention output and row statistics,
 * MLP pre-activation and activation).  Backpropagation without recomputation
 * would keep one such slot, plus both residual streams, per block; the
 * reversible schedules keep one (Reprop) or two (PaReprop) in total.  For the
 * memory-versus-batch comparison of Sec. 4.2.  Host only. */
int64_t rev_stack_slot_bytes(const rev_cfg* cfg);

/* Forward map of the whole stack (Eq. 1 applied N times); stores no
 * activations beyond Y1, Y2.  X1, X2 in; Y1, Y2 out (float32 [B,T,D]).
 * `stream` is a hipStream_t (NULL = the default stream). */
int rev_stack_forward(const rev_cfg* cfg, const void* params,
                      const float* X1, const float* X2, float* Y1, float* Y2,
                      void* workspace, int64_t workspace_bytes, void* stream);

/* Reversible backpropagation, sequential schedule ("Reprop", Sec. 3.2): for
 * block N down to 1, on one stream: recompute the block's inputs and
 * intermediates from its outputs (the inverse above), then apply the block's
 * transposed Jacobian to the incoming cotangents.
 *   in : params; Y1, Y2 = outputs of the last block; dY1, dY2 = their cotangents
 *   out: dX1, dX2 = cotangents of the stack inputs; dparams = gradient of every
 *        parameter (float32, packed like params, overwritten);
 *        X1_out, X2_out (nullable) = the reconstructed stack inputs. */
int rev_stack_backward_reprop(const rev_cfg* cfg, const void* params,
                              const float* Y1, const float* Y2,
                              const float* dY1, const float* dY2,
                              float* dX1, float* dX2,
                              float* X1_out, float* X2_out, float* dparams,
                              void* workspace, int64_t workspace_bytes, void* stream);

/* Same inputs, outputs and results -- bit for bit -- as
 * rev_stack_backward_reprop, under the parallel schedule ("PaReprop", Sec. 3.3,
 * Fig. 3 bottom row): the recomputation chain R_N, R_{N-1}, ... runs on
 * `stream_recompute`, the gradient chain V_N, V_{N-1}, ... on `stream_grad`;
 * V_i waits for R_i, and R_{i-2} waits for V_i (which frees the activation
 * slot it will overwrite), so R_{i-1} overlaps V_i.  Within V_i only the
 * input-gradient kernels (the part V_{i-1} depends on) stay on `stream_grad`;
 * its four weight-gradient GEMMs follow R_{i-1} on `stream_recompute` (in bf16
 * mode as one launch, ordered after the kernels that produce their cotangent
 * operands; in float32 mode one by one, each after its own).
 * `stream_recompute` first
 * waits for everything already enqueued on `stream_grad` and is joined back
 * into `stream_grad` before the call returns.  The two streams must differ and
 * must have the same (default) priority.  The call enqueues kernels and event
 * records / waits only, so it may be issued while `stream_grad` is being
 * captured into a HIP graph: `stream_recompute` joins the capture through the
 * fork event and the graph replays the whole two-stream pass. */
int rev_stack_backward_pareprop(const rev_cfg* cfg, const void* params,
                                const float* Y1, const float* Y2,
                                const float* dY1, const float* dY2,
                                float* dX1, float* dX2,
                                float* X1_out, float* X2_out, float* dparams,
                                void* workspace, int64_t workspace_bytes,
                                void* stream_grad, void* stream_recompute);

/* For callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): rev_stack_backward_reprop
 * without the workspace argument.  The workspace is a buffer of
 * REV_STATIC_WORKSPACE_BYTES that is part of the library's device image, so each
 * GPU the library runs on holds it from load until the process ends; the call
 * allocates nothing, on the device or through any library (it creates no events
 * either), and frees nothing.  Same arguments, results (bit for bit), ordering
 * and errors as rev_stack_backward_reprop, plus: REV_EWORKSPACE, before anything
 * is enqueued, if rev_stack_workspace_bytes_reprop(cfg) exceeds
 * REV_STATIC_WORKSPACE_BYTES (the message says what the shape needs).  All calls
 * on one GPU share the one buffer, which keeps the previous call's contents
 * (every region is written before it is read, nothing has to start at zero):
 * two such calls that overlap in time on one GPU race, also from different
 * streams or host threads -- order them on one stream or with events. */
#define REV_STATIC_WORKSPACE_BYTES (64 * 1024 * 1024)
int rev_stack_backward_reprop_static(const rev_cfg* cfg, const void* params,
                                     const float* Y1, const float* Y2,
                                     const float* dY1, const float* dY2,
                                     float* dX1, float* dX2,
                                     float* X1_out, float* X2_out, float* dparams,
                                     void* stream);

/* Optimizer update of a training step: AdamW, the optimizer of the paper's
 * throughput experiments (Sec. 4, experimental setup; the paper gives neither
 * formula nor hyper-parameters, so this is the published update with decoupled
 * weight decay, eps outside the square root, step counter from 1):
 *   m = beta1 m + (1-beta1) g;  v = beta2 v + (1-beta2) g^2;
 *   theta -= lr * ( (m / (1-beta1^step)) / (sqrt(v / (1-beta2^step)) + eps)
 *                   + weight_decay * theta ).
 * All buffers are device memory of n elements, updated in place:
 *   master      float32 weights (in float32 mode these ARE the stack's params);
 *   params_bf16 nullable; if given, receives master rounded to bf16 (nearest
 *               even): the copy the bf16-mode entry points read;
 *   grad        float32 gradient, e.g. dparams of a backward call (not modified);
 *   m, v        float32 moments (zero before step 1).
 * float32 arithmetic throughout.  Enqueues on `stream` and returns.
 * REV_EINVAL on null/misaligned pointers (16 bytes; 8 for params_bf16), n <= 0,
 * step < 1, beta outside [0,1) or a negative lr/eps/weight_decay. */
int rev_adamw_step(int64_t n, float* master, void* params_bf16, const float* grad,
                   float* m, float* v, int32_t step, float lr, float beta1, float beta2,
                   float eps, float weight_decay, void* stream);

/* The same three calls with a key-padding mask, for batches of sequences of
 * different lengths padded to seq_len (the variable-length text batches of the
 * paper's language experiments, Sec. 4.1; the paper does not describe the mask,
 * this is the common one).  key_len: device pointer to `batch` int32 values;
 * in every attention of sample b the keys at positions >= key_len[b] get
 * probability exactly 0.  Values are clamped to [1, seq_len] (a softmax needs
 * one key).  All seq_len query rows of every sample are still computed and
 * returned, padded positions included: they flow through the blocks like any
 * token but no valid position ever reads them, so with cotangents that vanish
 * on the padded positions every result at a valid position and every parameter
 * gradient equals that of the unpadded sequences.  Everything else (arguments,
 * workspace sizes, ordering, errors, bit-identity of the two schedules) is as
 * for the unmasked calls; key_len must not be null here. */
int rev_stack_forward_masked(const rev_cfg* cfg, const void* params,
                             const float* X1, const float* X2, const int32_t* key_len,
                             float* Y1, float* Y2,
                             void* workspace, int64_t workspace_bytes, void* stream);
int rev_stack_backward_reprop_masked(const rev_cfg* cfg, const void* params,
                                     const float* Y1, const float* Y2, const int32_t* key_len,
                                     const float* dY1, const float* dY2,
                                     float* dX1, float* dX2,
                                     float* X1_out, float* X2_out, float* dparams,
                                     void* workspace, int64_t workspace_bytes, void* stream);
int rev_stack_backward_pareprop_masked(const rev_cfg* cfg, const void* params,
                                       const float* Y1, const float* Y2, const int32_t* key_len,
                                       const float* dY1, const float* dY2,
                                       float* dX1, float* dX2,
                                       float* X1_out, float* X2_out, float* dparams,
                                       void* workspace, int64_t workspace_bytes,
                                       void* stream_grad, void* stream_recompute);

/* Plain stochastic gradient descent on the packed vector, theta <- theta - lr * grad
 * (Sec. 4: the paper reports the same behaviour with SGD as with AdamW).
 * Arguments, alignment, in-place update, optional bf16 copy and errors as for
 * rev_adamw_step. */
int rev_sgd_step(int64_t n, float* master, void* params_bf16, const float* grad,
                 float lr, void* stream);

/* Measurement aid for the hidden-recompute fraction: runs only one of the two
 * chains of the backward pass on `stream`.  chain = 0: the recomputation chain
 * R_N..R_1 alone (writes X1_out/X2_out if given).  chain = 1: the gradient
 * chain V_N..V_1 alone, reading whatever the two activation slots and the
 * residual ring currently hold (run a full backward first so they hold finite
 * values); its outputs are meaningful as timings only. */
int rev_stack_backward_chain(const rev_cfg* cfg, const void* params,
                             const float* Y1, const float* Y2,
                             const float* dY1, const float* dY2,
                             float* dX1, float* dX2,
                             float* X1_out, float* X2_out, float* dparams,
                             void* workspace, int64_t workspace_bytes,
                             void* stream, int32_t chain);

/* ---- Stage transition of a hierarchical reversible model ------------------
 *
 * Between two stages of its hierarchical (window-attention) model the paper
 * places a block that first fuses the two residual streams (by averaging, or
 * by a small MLP) and then applies the usual patch merging (Sec. 3.4 and
 * panel (b) of the architecture figure).  The readings built here: fusion by
 * averaging, z0 = (X1 + X2) / 2 (cfg.fusion = REV_FUSION_AVERAGE), or by a small
 * MLP on the concatenated streams, z0 = gelu([X1 | X2] Wa^T + ba) Wb^T + bb with
 * one hidden layer as wide as a stream (REV_FUSION_MLP; the GELU of the blocks);
 * patch merging = concatenate every 2x2 neighbourhood of the token
 * grid along the feature axis (C -> 4C, neighbour (dy, dx) at feature block
 * 2*dy + dx), LayerNorm over the 4C features, bias-free linear map 4C -> 2C;
 * both streams of the next stage start from the result, so the backward pass
 * takes one cotangent per copy and adds them.  The block is not reversible:
 * the caller keeps its inputs (the last stage's outputs) for the backward call.
 *
 * Tokens are stored window by window, on both sides: row
 *   ((b * (grid_h/window) + y/window) * (grid_w/window) + x/window) * window^2
 *     + (y % window) * window + (x % window)
 * holds the token at grid position (y, x) of image b, so that a stage's
 * windows are the contiguous sequences rev_stack_* works on.  The merged map
 * has (grid_h/2) x (grid_w/2) tokens per image in the same order.
 *
 * Packed parameters (element type as in rev_cfg.mode): ln_gamma[4C],
 * ln_beta[4C], W[2C, 4C] row-major, and with REV_FUSION_MLP behind them
 * Wa[C, 2C], ba[C], Wb[C, C], bb[C].  dparams: same layout, float32,
 * overwritten.  X1, X2, dX1, dX2: [batch*grid_h*grid_w, C] float32.  out, dOutA,
 * dOutB: [batch*grid_h*grid_w/4, 2C] float32.  All device pointers, 16-byte
 * aligned; the workspace 256-byte aligned and at least
 * rev_merge_workspace_bytes() long.  Calls enqueue on `stream` and return;
 * nothing is allocated.  Errors as for the rev_stack_* calls. */
#define REV_FUSION_AVERAGE 0
#define REV_FUSION_MLP     1

typedef struct rev_merge_cfg {
    int32_t batch;      /* images                                              */
    int32_t grid_h;     /* token grid of the incoming stage; both sides must   */
    int32_t grid_w;     /*   be multiples of 2 * window                        */
    int32_t window;     /* side of the square attention windows                */
    int32_t d_in;       /* width C of the incoming stage (multiple of 8, <= 2048) */
    int32_t mode;       /* REV_MODE_FP32 or REV_MODE_BF16                      */
    float   ln_eps;
    int32_t fusion;     /* REV_FUSION_AVERAGE or REV_FUSION_MLP                */
} rev_merge_cfg;

int     rev_merge_check_cfg(const rev_merge_cfg* cfg);
int64_t rev_merge_param_count(const rev_merge_cfg* cfg);      /* 8C + 8C^2 (+ 3C^2 + 2C with the MLP fusion) */
int64_t rev_merge_workspace_bytes(const rev_merge_cfg* cfg);
int rev_merge_forward(const rev_merge_cfg* cfg, const void* params,
                      const float* X1, const float* X2, float* out,
                      void* workspace, int64_t workspace_bytes, void* stream);
int rev_merge_backward(const rev_merge_cfg* cfg, const void* params,
                       const float* X1, const float* X2,
                       const float* dOutA, const float* dOutB,
                       float* dX1, float* dX2, float* dparams,
                       void* workspace, int64_t workspace_bytes, void* stream);

/* Per-kernel-family timing.  Between rev_profile_begin() and rev_profile_end()
 * every kernel launch made by the calling process is bracketed by a pair of
 * HIP events on the stream it is launched on.  rev_profile_end() synchronises
 * the device, folds the elapsed times into per-family totals and stops
 * recording.  rev_profile_get() returns, for family `kind` (0 <=
 * kind < rev_profile_kinds()), its name, total milliseconds, launch count and
 * the algorithmic work of those launches (flops for matrix-core families, HBM
 * bytes for the others; see rev_profile_is_flops).  Totals accumulate until
 * rev_profile_begin() is called again.  Not thread safe. */
int         rev_profile_begin(void);
int         rev_profile_end(void);
int         rev_profile_kinds(void);
const char* rev_profile_name(int kind);
int         rev_profile_is_flops(int kind);
int         rev_profile_get(int kind, double* total_ms, int64_t* launches, double* work);

/* Text of the last error reported on this thread ("" if none). */
const char* rev_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* REV_STACK_H */
