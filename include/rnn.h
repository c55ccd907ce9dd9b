/*
 * rnn.h -- C ABI of the MI355X (gfx950) Elman recurrent-network training path.
 *
 * The path is the one the paper's symbolic loop (its "Scan" section) compiles for a simple
 * recurrent language model (its recurrent-network benchmark section): a forward loop over
 * the leading (time) axis, an output layer with a loss, and backpropagation through time
 * that keeps every hidden state (Scan property 1).  The paper prints no equations for the
 * network; the ones used are the textbook Elman equations:
 *
 *     a_t = in_t + Wh h_{t-1} + b          in_t = Wx[x_t,:] (token ids) or Wx x_t (dense)
 *     h_t = act(a_t)                       act  = sigmoid or tanh
 *     z_t = V^T h_t + c
 *     softmax-CE : loss = mean over the T*B rows of ( logsumexp(z) - z[y] )   (natural log)
 *     linear-MSE : loss = mean over the T*B*O entries of (z - Y)^2            (no factor 1/2)
 *
 * Conventions shared by every entry point
 *   - All tensors are float32, row-major and time-major ([T,B,...]); token ids and class
 *     targets are int32.  Every data pointer is a DEVICE pointer unless it says "host";
 *     rnn_dims / rnn_params / rnn_grads structs themselves live in HOST memory.
 *   - Layouts:  Wx [in_dim,H] for token input (row v = input vector of token v) or [H,in_dim]
 *     for dense input;  Wh [H,H] with a[j] = sum_i Wh[j,i] h[i];  b [H];
 *     V [H,out_dim] with z[k] = sum_i h[i] V[i,k] + c[k];  c [out_dim].
 *     Gradients have the layout of their parameter.
 *   - Ownership: the caller owns every buffer including the workspace; the library never
 *     allocates, frees or keeps device memory (the paper's garbage-collection-free linker
 *     keeps buffers alive between calls for the same reason).
 *   - Asynchrony: every call only enqueues kernels on `hip_stream` (a hipStream_t, NULL =
 *     the default stream) and returns, as in the paper's section on asynchronous GPU calls;
 *     flag RNN_FLAG_SYNC makes the call wait for the stream (for profiling).
 *   - Trust: the hot calls do O(1) host-side argument checks and never read device data on
 *     the host; out-of-range token ids are undefined behaviour unless rnn_check_tokens is
 *     used first (the paper's trusted-input switch makes the same trade).
 *   - Call order on one stream with one workspace: rnn_forward -> rnn_loss -> rnn_bptt.
 *     rnn_loss leaves the logits and row statistics in the workspace for rnn_bptt; with
 *     RNN_FLAG_BPTT_RECOMPUTE rnn_bptt recomputes them itself and needs no prior rnn_loss.
 *   - Parameter, gradient, state and workspace pointers must be 16-byte aligned; inputs x,
 *     targets and the loss scalar only 4-byte aligned (so a window may start anywhere in a
 *     longer stream).  No size needs to be a multiple of anything.
 *   - Return value: RNN_OK or a negative RNN_E* code; nothing is printed, nothing aborts.
 *     When a call returns an error nothing has been enqueued, except RNN_EHIP which reports
 *     a failed launch.
 */
#ifndef RNN_MI355X_H
#define RNN_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RNN_OK            0
#define RNN_EINVAL       (-1)  /* bad size, enum, or NULL required pointer            */
#define RNN_EWORKSPACE   (-2)  /* workspace NULL, misaligned or smaller than required */
#define RNN_EUNSUPPORTED (-3)  /* valid request this build has no kernel for          */
#define RNN_EHIP         (-4)  /* a HIP launch or query failed                        */
#define RNN_ETOOLARGE    (-5)  /* problem exceeds the fixed scratch of rnn_window_static */

#define RNN_INPUT_TOKENS 0     /* x is int32 [T,B], values in [0,in_dim)              */
#define RNN_INPUT_DENSE  1     /* x is float32 [T,B,in_dim]                           */
#define RNN_ACT_SIGMOID  0
#define RNN_ACT_TANH     1
#define RNN_LOSS_SOFTMAX_CE 0  /* targets int32 [T,B], values in [0,out_dim)          */
#define RNN_LOSS_LINEAR_MSE 1  /* targets float32 [T,B,out_dim]                       */

#define RNN_FLAG_ACCUMULATE     1u /* gradients are added to the buffers instead of overwriting */
#define RNN_FLAG_SYNC           2u /* hipStreamSynchronize before returning                     */
#define RNN_FLAG_BPTT_RECOMPUTE 4u /* rnn_bptt recomputes logits; no prior rnn_loss needed      */
#define RNN_FLAG_REFERENCE_KERNELS 8u /* use only the shape-agnostic kernels (A/B testing)      */
/* Opt-in reduced-precision output layer: the large products Z = H V + c, dV = H^T dZ, G = dZ V^T
 * (and dWh = Delta^T H_prev, dense-input dWx = Delta^T X) run on the bf16 matrix cores with float32 accumulation, every float32
 * operand split into two bf16 numbers (hi + lo) and each product taken as hi*hi + hi*lo + lo*hi
 * (error per product term below 2^-16 relative; parameters, results and everything else stay
 * float32).  Set it on rnn_workspace_bytes, rnn_loss and rnn_bptt alike (the workspace grows by
 * the bf16 copies of the operands).  Ignored where the column-strip kernels of a short single
 * sequence serve the output layer; rnn_gauss_newton_vec takes it too (its five output-layer
 * products); rejected by rnn_window and rnn_train_stream. */
#define RNN_FLAG_BF16X3_OUTPUT 16u
/* rnn_window only: launch cooperatively (the runtime then guarantees that all workgroups of the
 * launch are resident together, at about 18 us more per launch) instead of the plain launch that
 * relies on the precondition stated at rnn_window. */
#define RNN_FLAG_COOPERATIVE 32u

typedef struct {
    int32_t in_dim;     /* vocabulary size NV for token input, feature count D for dense input */
    int32_t hidden;     /* H                                                                   */
    int32_t out_dim;    /* NV for softmax-CE, O for linear-MSE                                 */
    int32_t seq_len;    /* T, number of time steps of this call (one truncated-BPTT window)     */
    int32_t batch;      /* B, independent sequences                                            */
    int32_t input_kind; /* RNN_INPUT_*                                                         */
    int32_t act;        /* RNN_ACT_*                                                           */
    int32_t loss_kind;  /* RNN_LOSS_*                                                          */
    uint32_t flags;     /* RNN_FLAG_* bits                                                     */
} rnn_dims;

typedef struct { const float *Wx, *Wh, *b, *V, *c; } rnn_params; /* device pointers */
typedef struct { float *dWx, *dWh, *db, *dV, *dc; } rnn_grads;   /* device pointers */

/* Bytes of workspace the three calls below need for these sizes (host-only, no GPU touched).
 * The same workspace must be passed to forward, loss and bptt of one window. */
int rnn_workspace_bytes(const rnn_dims *dims, size_t *bytes);

/*
 * Forward recurrence (the loop of the Scan section, run entirely on the device with no host
 * work per step -- Scan properties 4 and 5; the input term is gathered/projected for all
 * steps outside the loop -- property 8).
 *   x       token ids int32[T,B] or inputs float32[T,B,in_dim]
 *   h0      initial state [B,H], NULL = zeros
 *   h_all   [T+1,B,H] receives h_all[0] = h0 and h_all[t+1] = h_t; NULL = keep no history
 *           (Scan property 6: only a two-slot ring in the workspace is used)
 *   h_last  [B,H] receives h_{T-1}; NULL = not wanted.  h_all and h_last may not both be NULL.
 */
int rnn_forward(const rnn_dims *dims, const rnn_params *params, const void *x,
                const float *h0, float *h_all, float *h_last,
                void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Output projection and loss over all T*B rows at once (matrix-matrix product hoisted out of
 * the loop, Scan property 8), evaluated as a max-subtracted log-sum-exp (the numerically
 * stable form the paper's graph optimiser rewrites to).
 *   h_all    [T+1,B,H] as written by rnn_forward
 *   targets  int32[T,B] (CE) or float32[T,B,out_dim] (MSE)
 *   loss     device float32[1], overwritten
 */
int rnn_loss(const rnn_dims *dims, const rnn_params *params, const float *h_all,
             const void *targets, float *loss,
             void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Backpropagation through time (Scan property 1): gradients of the mean loss of this
 * window, plus <dh_last, h_{T-1}> when dh_last is given, with respect to every parameter.
 *   x, targets as above; h_all [T+1,B,H] from rnn_forward
 *   dh_last  [B,H] gradient arriving at h_{T-1} from a later window, NULL = zeros
 *   grads    all five device pointers required; overwritten, or added to with
 *            RNN_FLAG_ACCUMULATE.  For token input in overwrite mode rows of dWx whose token
 *            does not occur are set to exactly 0; in accumulate mode they are not written.
 *   dh0      [B,H] receives the gradient w.r.t. the initial state; NULL = not wanted
 * Weight-gradient sums are accumulated in float32 in a fixed order (run-to-run identical).
 */
int rnn_bptt(const rnn_dims *dims, const rnn_params *params, const void *x,
             const void *targets, const float *h_all, const float *dh_last,
             const rnn_grads *grads, float *dh0,
             void *workspace, size_t workspace_bytes, void *hip_stream);

/* Opt-in validation: counts ids outside [0,limit) among n int32 ids into bad_count (device
 * int32[1], overwritten).  Asynchronous like the other calls. */
int rnn_check_tokens(const void *ids, int64_t n, int32_t limit, int32_t *bad_count,
                     void *hip_stream);

/*
 * Workspace set-up and the device status word.
 *
 * rnn_workspace_init must be called once on a newly allocated workspace (and again whenever
 * the memory has been used for anything else) before the first rnn_forward / rnn_loss /
 * rnn_bptt with these dims: kernels of one launch pass small results to each other as words
 * that carry a per-launch tag, and a cleared word is what "not written yet" looks like.  The tag
 * itself is a word of the workspace that the kernels advance (device state, nothing of it is
 * baked into a launch's arguments), so calls captured into a HIP graph may be replayed.  The call
 * is asynchronous on hip_stream and also clears the status word.  One workspace serves one stream
 * at a time.
 *
 * Status word: the kernels that wait for other workgroups of their launch do so with a bounded
 * spin; if a wait ever expires (which needs the GPU to be shared in a way that keeps those
 * workgroups from running together) the kernel sets the word to 1, stops waiting, and the
 * results of that call are invalid, as are those of later calls until rnn_workspace_init has run
 * on the workspace again.  rnn_workspace_status copies the word to *status_host and synchronises
 * the stream.
 *
 * rnn_set_wait_limit sets the number of polls such a wait makes before it gives up (host state of
 * the process, read when a call is enqueued; default 2^22, about a second; polls <= 0 restores the
 * default).  For callers that share the GPU and prefer an early status 1 to a long spin, and for
 * tests of the failure path.
 */
int rnn_set_wait_limit(int polls);
int rnn_workspace_init(const rnn_dims *dims, void *workspace, size_t workspace_bytes,
                       void *hip_stream);
int rnn_workspace_status(const rnn_dims *dims, const void *workspace, size_t workspace_bytes,
                         void *hip_stream, int32_t *status_host);

/*
 * Many consecutive truncated-BPTT windows of ONE token stream with a plain SGD update after
 * every window, in a single call and a single persistent launch (callers: training loops that
 * would otherwise pay three launches per window; the paper's function objects offer the same
 * shortcut as a repeat count on the call, returning only the last result).  The paper names
 * no update rule; the plain one is used.  For w = 0 .. n_windows-1:
 *
 *     x = ids[w*T .. w*T+T-1],  y = ids[w*T+1 .. w*T+T]            (next-token targets)
 *     h_all = forward(params, x, h);  losses[w] = loss(params, h_all, y)
 *     params <- params - lr * gradient of that loss (all five tensors; no gradient arrives
 *               from later windows, none is sent to earlier ones)
 *     h <- h_{T-1} of this window (computed with the parameters before the update)
 *
 *   dims     token input, softmax-CE, in_dim == out_dim (else RNN_EUNSUPPORTED); flags:
 *            RNN_FLAG_SYNC only.  ONE persistent launch for batch 1, hidden <= 128, seq_len <= 32,
 *            out_dim <= 32640 (the paper's benchmark shape).  Every other size is served by the
 *            same call as, per window, the launches of rnn_forward, rnn_loss and rnn_bptt plus one
 *            update launch, all enqueued by this call (same results; ids is then int32
 *            [n_windows*T + 1, B], h0 and h_last [B,H], and the parameters are up to date after
 *            every window)
 *   params   device pointers, 16-byte aligned, UPDATED IN PLACE; while the call runs the
 *            buffers are in an intermediate state (the model lives in on-chip memory and is
 *            written back when the last window is done)
 *   ids      device int32[n_windows*T + 1], values in [0, in_dim) (not checked)
 *   h0       [H] initial state, NULL = zeros;  h_last [H] final state, NULL = not wanted
 *   losses   device float32[n_windows], NULL = not wanted
 *   workspace  rnn_train_stream_workspace_bytes() bytes, 256-byte aligned; needs no set-up (the
 *            call clears what it uses) and may be shared with the other calls of this library
 *            on the same stream
 * Asynchronous like the other calls.  The launch is cooperative (1 + ceil(out_dim/128)
 * workgroups that wait for each other with bounded spins; the runtime guarantees that they are
 * resident together); rnn_train_stream_status copies the workspace's status word to *status_host
 * after synchronising the stream: 0 = every wait was met, 1 = a wait expired and the results of
 * that call are invalid.
 */
typedef struct { float *Wx, *Wh, *b, *V, *c; } rnn_params_inout; /* device pointers */
int rnn_train_stream_workspace_bytes(const rnn_dims *dims, size_t *bytes);
int rnn_train_stream(const rnn_dims *dims, const rnn_params_inout *params, const int32_t *ids,
                     int64_t n_windows, float lr, const float *h0, float *h_last, float *losses,
                     void *workspace, size_t workspace_bytes, void *hip_stream);
int rnn_train_stream_status(const void *workspace, void *hip_stream, int32_t *status_host);

/*
 * One truncated-BPTT window in ONE launch: what rnn_forward -> rnn_loss -> rnn_bptt compute
 * together (same equations, same outputs), for callers that step through a stream window by
 * window and would otherwise pay three launches per window.  The one-launch kernel serves the
 * paper's benchmark shape (its recurrent-network benchmark section: batch 1, vocabulary-sized
 * output layer, short windows): token input, softmax-CE, batch 1, hidden <= 128, seq_len <= 32,
 * out_dim <= 32640.  Every other token / softmax-CE size is served by the same call as the
 * launches of the three calls above on a workspace of its own layout (same results, any batch);
 * dense input or the MSE loss return RNN_EUNSUPPORTED.
 *   x, targets  device int32[T,B] (4-byte aligned; a window may start anywhere in a stream)
 *   h0, dh_last [B,H], NULL = zeros;  h_all [T+1,B,H], h_last [B,H], dh0 [B,H]: NULL = not wanted
 *   loss        device float32[1];  grads as in rnn_bptt (RNN_FLAG_ACCUMULATE adds)
 *   workspace   rnn_window_workspace_bytes() bytes, 256-byte aligned, cleared ONCE with
 *               rnn_window_workspace_init before its first use (the workgroups of the launch
 *               exchange words that carry a per-launch tag; cleared memory is "not written yet";
 *               the tag is a word of the workspace that the kernel advances, so a captured call
 *               may be replayed, and a workspace rnn_train_stream has used needs no new set-up)
 * Launch form of the one-launch kernel and its precondition: 1 + ceil(out_dim/128) workgroups that
 * wait for each other with bounded spins.  By default this is a PLAIN launch (a cooperative one costs about 18 us more,
 * the time of a whole window at the benchmark shape), used only when the whole grid fits the chip
 * by itself (checked on the host; otherwise the launch is cooperative): it is correct as long as
 * no other kernel occupies the GPU's compute units while the call runs -- other streams of the
 * process must be idle or hold only kernels that leave room for the grid.  A caller that cannot
 * promise that sets RNN_FLAG_COOPERATIVE.  If the precondition is broken the waits expire
 * (rnn_set_wait_limit), the status word becomes 1 and the outputs of that call are invalid:
 * callers that share the GPU must read rnn_train_stream_status (which reads the status word of
 * this workspace as well) before they trust a window's results.
 */
/* 1: rnn_window serves these sizes with its one-launch kernel; 0: with the launches of the three
 * calls; negative: an error code (sizes it does not serve at all).  Host-only. */
int rnn_window_one_launch(const rnn_dims *dims);
int rnn_window_workspace_bytes(const rnn_dims *dims, size_t *bytes);
int rnn_window_workspace_init(const rnn_dims *dims, void *workspace, size_t workspace_bytes,
                              void *hip_stream);
int rnn_window(const rnn_dims *dims, const rnn_params *params, const int32_t *x,
               const int32_t *targets, const float *h0, const float *dh_last, float *h_all,
               float *h_last, float *loss, const rnn_grads *grads, float *dh0,
               void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * rnn_window for callers that cannot allocate device memory and have no workspace to pass: code
 * under HIP graph capture, tight serving or training loops, harnesses that forbid hipMalloc.  Same
 * computation, same kernels and same outputs as rnn_window; the exchange boxes live in a fixed
 * array inside the library's code object instead (RNN_WINDOW_STATIC_BYTES = 2 MiB per GPU, held by
 * every GPU the library runs on until the process ends).  The call allocates and frees nothing,
 * here or in any library routine it uses.
 *   dims .. dh0   as in rnn_window, for the sizes its one-launch kernel serves
 *                 (rnn_window_one_launch() == 1; others return RNN_EUNSUPPORTED: the launches of the
 *                 three calls need a workspace).  Sizes whose boxes exceed the array (more than
 *                 rnn_window_workspace_bytes() = RNN_WINDOW_STATIC_BYTES) return RNN_ETOOLARGE and
 *                 nothing is enqueued; the paper's benchmark shape (vocabulary 10000, hidden 100,
 *                 windows of 10) needs 0.67 MB.
 *   status        device int32[1], nullable, 4-byte aligned: set to 1 by the kernel if a bounded
 *                 wait expired (results of that call invalid), untouched otherwise; the caller
 *                 clears it.  NULL: the word is kept inside the array and cannot be read.
 * The first call on a device looks the array's device address up and clears the array with a fill
 * kernel on hip_stream, ahead of the window kernel; make that first call outside graph capture.
 * All calls on one GPU share that GPU's array, which keeps the previous call's words (they carry
 * that call's tag, so a later call never mistakes them for its own): calls that overlap in time
 * on one GPU, on whatever streams, race and give undefined results.  Calls on different GPUs are
 * independent.
 */
#define RNN_WINDOW_STATIC_BYTES ((size_t)2 << 20)
int rnn_window_static(const rnn_dims *dims, const rnn_params *params, const int32_t *x,
                      const int32_t *targets, const float *h0, const float *dh_last, float *h_all,
                      float *h_last, float *loss, const rnn_grads *grads, float *dh0,
                      int32_t *status, void *hip_stream);

/*
 * Gauss-Newton matrix times a vector by the R-operator (the paper's section on the R-operator:
 * the forward-mode derivative R{f} = (df/dtheta) gamma carried through the loop next to the
 * states, then a reverse pass, i.e. Lop(f, theta, Rop(f, theta, gamma)) -- two passes over the
 * sequence instead of forming any Jacobian).  f is the matrix of all T*B output rows z; with
 * J = df/dtheta the call returns  J^T M J gamma  for
 *   RNN_GN_METRIC_LOSS      M = Hessian of this library's mean loss w.r.t. z
 *                           (softmax-CE: (diag(p) - p p^T)/N per row; linear-MSE: 2/(N O) I)
 *   RNN_GN_METRIC_IDENTITY  M = I, the paper's literal expression.
 *     R a_t = gin_t + gamma.b + gamma.Wh h_{t-1} + Wh R h_{t-1}    gin_t = gamma.Wx[x_t,:] or gamma.Wx x_t
 *     R h_t = act'(h_t) R a_t,  R h_{-1} = 0 (the initial state is a constant)
 *     R z_t = V^T R h_t + gamma.V^T h_t + gamma.c;   u = M R z;   result = backpropagation of u
 *   params, gamma  the parameters and a direction of the same shapes (device, 16-byte aligned)
 *   x        as in rnn_forward;  h_all [T+1,B,H] from rnn_forward with these parameters
 *   out      five device pointers of the parameters' shapes; overwritten, or added to with
 *            RNN_FLAG_ACCUMULATE (token input: rows of out->dWx as in rnn_bptt)
 *   Rz       [T*B,out_dim] receives R z (the R-operator's own result); NULL = not wanted
 *   workspace  rnn_gauss_newton_workspace_bytes() bytes, 16-byte aligned; its first
 *            rnn_workspace_bytes() bytes are an ordinary workspace and need rnn_workspace_init
 *            once.  The logits rnn_loss left in a workspace do not survive this call.
 * Needs no prior rnn_loss.  Asynchronous like the other calls.  RNN_FLAG_BPTT_RECOMPUTE is
 * rejected (RNN_EINVAL).
 */
#define RNN_GN_METRIC_LOSS     0
#define RNN_GN_METRIC_IDENTITY 1
int rnn_gauss_newton_workspace_bytes(const rnn_dims *dims, size_t *bytes);
int rnn_gauss_newton_vec(const rnn_dims *dims, const rnn_params *params, const rnn_params *gamma,
                         const void *x, const float *h_all, int32_t metric, const rnn_grads *out,
                         float *Rz, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Second workload: training steps of a feed-forward classifier (the paper's neural-network
 * training benchmark: 10-class classification of a 784-dimensional input by logistic regression,
 * one hidden layer of 500 units, or three of 1000; stochastic gradient descent on single
 * examples or mini-batches of 10 and 60; examples per second).  The paper prints no equations
 * and names no hidden non-linearity; the textbook network is used:
 *
 *     a_0 = x;  a_l = act(W_l a_{l-1} + b_l), l = 1..n_hidden;  z = W_L a_{L-1} + b_L
 *     loss = mean over the batch of ( logsumexp(z) - z[y] )                 (natural log)
 *     after every batch:  W_l <- W_l - lr dloss/dW_l,   b_l <- b_l - lr dloss/db_l
 *
 * rnn_mlp_train runs n_batches consecutive batches in one call (the paper's function objects
 * offer the same as a repeat count, "several iterations at once"): nothing returns to the host
 * between batches, every batch is 2 n_hidden + 2 launches on hip_stream (one more with more than
 * 16 classes).
 *   dims     host struct; act = RNN_ACT_* of the hidden layers; flags: RNN_FLAG_SYNC only;
 *            n_hidden + 1 <= RNN_MLP_MAX_LAYERS; batch <= 1024 (else RNN_EUNSUPPORTED)
 *   params   host struct of device pointers, layer l = 0..n_hidden (input side first):
 *            W[l] float32 [fan_out_l, fan_in_l] row-major, b[l] float32 [fan_out_l]; 16-byte
 *            aligned; UPDATED IN PLACE
 *   X        device float32 [n_batches*batch, in_dim], 16-byte aligned;  y device int32
 *            [n_batches*batch], values in [0, out_dim) (not checked)
 *   losses   device float32 [n_batches]: mean loss of every batch, computed with the parameters
 *            before that batch's update; NULL = not wanted
 *   workspace  rnn_mlp_workspace_bytes() bytes, 16-byte aligned, needs no set-up
 * Asynchronous like the other calls; sums run in a fixed order (run-to-run identical results).
 */
#define RNN_MLP_MAX_LAYERS 16
typedef struct {
    int32_t in_dim;     /* width of the input                                  */
    int32_t hidden;     /* width of every hidden layer (ignored if n_hidden=0) */
    int32_t n_hidden;   /* number of hidden layers, 0 = logistic regression    */
    int32_t out_dim;    /* number of classes                                   */
    int32_t batch;      /* examples per update                                 */
    int32_t act;        /* RNN_ACT_* of the hidden layers                      */
    uint32_t flags;     /* RNN_FLAG_SYNC                                       */
} rnn_mlp_dims;
typedef struct { float *W[RNN_MLP_MAX_LAYERS], *b[RNN_MLP_MAX_LAYERS]; } rnn_mlp_params; /* device pointers */
int rnn_mlp_workspace_bytes(const rnn_mlp_dims *dims, size_t *bytes);
int rnn_mlp_train(const rnn_mlp_dims *dims, const rnn_mlp_params *params, const float *X,
                  const int32_t *y, int64_t n_batches, float lr, float *losses,
                  void *workspace, size_t workspace_bytes, void *hip_stream);

/* Static description of an error code (host string, never NULL). */
const char *rnn_strerror(int code);

/* Name of the recurrence kernel family the dispatcher picks for these sizes (host-only; for
 * reports and tests): "wg_resident" (one workgroup per sequence, weights in LDS),
 * "grid_resident" (several cooperating workgroups per sequence), "batch_mfma" (batched,
 * hidden <= 256: one persistent matrix-core workgroup per 4 batch rows, weights in registers),
 * "xcd_mfma" (batched, 256 < hidden <= 1024, batch <= 64, hidden % 4 == 0, at least 10 steps, on
 * a device of 8 x 32 compute units: one persistent launch, 16 groups of 4 batch rows, two groups
 * per XCD),
 * "step_mfma" (other batched sizes: one fused matrix-core launch per step) or "reference". */
const char *rnn_recurrence_variant(const rnn_dims *dims);

/* Number of workgroups (= compute units occupied, one workgroup per unit) of one launch of the
 * forward time-loop kernel for these sizes, or RNN_EINVAL (host-only; roofline reports state
 * the loop's rate against the on-chip bandwidth or matrix rate of exactly these units). */
int rnn_recurrence_workgroups(const rnn_dims *dims);

/*
 * Per-kernel timing for roofline reports (the paper's GPU backend has a synchronous mode for
 * timing each kernel, section on the CUDA backend; this is the asynchronous equivalent).  Between
 * rnn_profile_begin and rnn_profile_end every kernel the library launches is bracketed by two
 * HIP events on its stream (at most max_launches launches are recorded, later ones are not).
 * rnn_profile_end waits for the recorded events and fills counts[k] / total_ms[k] (host arrays
 * of n_kernels >= rnn_profile_kernel_count() entries) per kernel id.  Host state, single
 * thread; the events add a little stream overhead, so time throughput with profiling off.
 */
int rnn_profile_begin(int max_launches);
int rnn_profile_end(int n_kernels, int64_t *counts, double *total_ms);
int rnn_profile_kernel_count(void);
const char *rnn_profile_kernel_name(int kernel_id);

/*
 * Measured ceilings of the device the calling thread has current, for roofline reports beside
 * the published peaks (not an operation of the paper).  Runs four saturating kernels on
 * `stream` and waits for them: results_host[0] = device-memory copy rate in GB/s (bytes read +
 * bytes written), [1] = fp32 matrix-core rate in TFLOP/s (32x32x2 products), [2] = bf16
 * matrix-core rate in TFLOP/s (32x32x16 products), [3] = LDS read rate in GB/s (16-byte reads,
 * all compute units), [4] = device-memory read rate in GB/s.  `scratch` is device memory the caller owns (16-byte aligned, at least
 * 128 MiB; the copy moves min(scratch_bytes / 2, 1 GiB) from its first half to its second, and
 * the contents are overwritten); results_host is a host array of 5 doubles.  Allocates no
 * device memory; creates and destroys two HIP events.  RNN_EINVAL on a null, misaligned or
 * short scratch, RNN_EHIP if a HIP call fails.
 */
int rnn_measure_ceilings(void *scratch, size_t scratch_bytes, double *results_host, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* RNN_MI355X_H */
