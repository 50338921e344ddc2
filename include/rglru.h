/*
 * rglru.h - C ABI of the MI355X (gfx950) library for the hot path of the Griffin/Hawk
 * recurrent block (arxiv 2402.19427): the width-4 temporal Conv1D (Section 2.3,
 * "Recurrent block") feeding the RG-LRU layer (Section 2.4, eqs. 1-4; log-space decay of
 * Appendix A; block-diagonal gate weights of Section 4.1), for whole sequences, for
 * single-token decode (Section 5, Appendix F "Cache sizes") and for the backward pass.
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 * - Every tensor pointer is a DEVICE pointer owned by the caller. The library never
 *   allocates, frees or keeps them. Struct pointers (rglru_shape, rglru_params,
 *   rglru_param_grads) are HOST pointers, read during the call only.
 * - Calls are asynchronous: kernels are enqueued on `stream` (a hipStream_t passed as
 *   void*, NULL = the default stream) and the function returns without synchronising.
 *   A call enqueues kernels only (no memsets, copies, allocations or waits), so calls may be
 *   recorded into a HIP graph by capturing the stream (with rglru_timing_enable(0)).
 * - Scratch memory comes from the caller: `workspace` must hold at least
 *   rglru_workspace_bytes(shape, op) bytes, 256-byte aligned; the library initialises what
 *   it needs on `stream`. Two calls that overlap in time must not share a workspace.
 * - Inputs are read-only. Outputs are overwritten (gradients are NOT accumulated).
 * - Return value: RGLRU_OK, or a negative RGLRU_ERR_* code; rglru_last_error() then
 *   describes the failure (thread-local string). Argument validation happens on the host
 *   before anything is launched, so an error return leaves all outputs untouched.
 *
 * Layouts (row-major, last index fastest; "act" = shape.act_dtype, "w" = shape.w_dtype)
 *   u, y, dy, du, x   [B][T][D]         act
 *   W_a, W_x          [nb][bs][bs]      w     W[g][j][k]: output channel g*bs+j, input
 *                                             channel g*bs+k; bs = D/nb (block-diagonal
 *                                             gate matrices, Section 4.1)
 *   b_a, b_x, Lambda  [D]               f32
 *   conv_w            [4][D]            f32   lag-indexed: conv_w[k] multiplies u_{t-k}
 *   conv_b            [D] or NULL       f32
 *   h0, hT, h, dh0, dhT [B][D]          f32
 *   conv state        [B][3][D]         act   ring buffer: the input at absolute position n
 *                                             lives in slot n mod 3 (mathematical modulo).
 *                                             A NULL incoming state means zero left-padding.
 *
 * What is computed (x_t is the Conv1D output, c = shape.c, sigma = logistic function):
 *   x_t = sum_{k=0..3} conv_w[k] * u_{t-k} (+ conv_b)                     Section 2.3
 *   r_t = sigma(W_a x_t + b_a),  i_t = sigma(W_x x_t + b_x)               eqs. (1), (2)
 *   a_t = sigma(Lambda)^(c r_t)  evaluated as exp(-c softplus(-Lambda) r_t) eq. (3), App. A
 *   h_t = a_t h_{t-1} + sqrt(1 - a_t^2) (i_t x_t),  y_t = h_t             eq. (4)
 * (Appendix A prints softplus(+Lambda); that contradicts a = sigma(Lambda) of Section 2.4,
 * which is what this library follows.)
 *
 * Which kernels run (bf16 storage): gate blocks of 256 channels, or of a multiple of 16 channels
 * from 128 to 240 (e.g. Section 4.1's 16 blocks at width 2560 = 160 channels), run on the fused
 * matrix-core kernels in every call. Any other multiple of 16 (e.g. 352 and 512 channels at
 * widths 5632 and 8192): rglru_forward runs as three matrix-core passes through the workspace
 * (widths that are a multiple of 256), decode steps on a matrix-core kernel of their own
 * (blocks up to 768 channels), the backward as matrix-core passes as well. All other block
 * sizes up to 2048 and fp32 storage run on generic kernels that give the same results far
 * more slowly.
 * rglru_workspace_bytes() accounts for all of it.
 */
#ifndef RGLRU_H
#define RGLRU_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* status codes */
#define RGLRU_OK 0
#define RGLRU_ERR_INVALID_ARG (-1) /* NULL required pointer, non-positive size, D % nb != 0,   */
                                   /* negative position, misaligned pointer                    */
#define RGLRU_ERR_UNSUPPORTED (-2) /* dtype / conv width / block size with no kernel           */
#define RGLRU_ERR_WORKSPACE (-3)   /* workspace NULL or smaller than rglru_workspace_bytes()   */
#define RGLRU_ERR_HIP (-4)         /* a HIP runtime call or kernel launch failed               */
#define RGLRU_ERR_TIMEOUT (-5)     /* rglru_workspace_status(): a bounded wait expired         */

/* element types */
#define RGLRU_F32 0
#define RGLRU_BF16 1

/* operations, for rglru_workspace_bytes() */
#define RGLRU_OP_CONV1D 0
#define RGLRU_OP_FORWARD 1
#define RGLRU_OP_DECODE 2
#define RGLRU_OP_BACKWARD 3
#define RGLRU_OP_SCAN 4
#define RGLRU_OP_FORWARD_MERGE 5
#define RGLRU_OP_BACKWARD_MERGE 6
#define RGLRU_OP_FORWARD_PACKED 7
#define RGLRU_OP_BACKWARD_PACKED 8
#define RGLRU_OP_CG_BACKWARD 9
#define RGLRU_OP_CG_FORWARD 10

typedef struct rglru_shape {
  int32_t B;          /* sequences                                  (>= 1)                 */
  int32_t T;          /* time steps per sequence                    (>= 0; ignored by decode) */
  int32_t D;          /* channels (D_RNN)                           (>= 1)                 */
  int32_t num_blocks; /* gate blocks nb; D % nb == 0                (ignored by conv1d)    */
  int32_t conv_width; /* temporal filter width: 4, or 0 = no Conv1D, the input is already  */
                      /* x_t (the RG-LRU layer of Section 2.4 alone): conv_w, conv_b and   */
                      /* every conv state argument are then ignored and may be NULL, and   */
                      /* dconv_w, dconv_b are not produced. rglru_conv1d takes 4 only.     */
  float c;            /* exponent scale of eq. (3); the paper uses 8                       */
  int32_t act_dtype;  /* RGLRU_F32 or RGLRU_BF16: u, y, dy, du, x, conv state              */
  int32_t w_dtype;    /* RGLRU_F32 or RGLRU_BF16: W_a, W_x. Supported pairs:               */
                      /* (act f32, w f32) and (act bf16, w bf16)                           */
} rglru_shape;

typedef struct rglru_params {
  const void *W_a;     /* [nb][bs][bs] w   recurrence-gate weights, eq. (1) */
  const void *W_x;     /* [nb][bs][bs] w   input-gate weights, eq. (2)      */
  const float *b_a;    /* [D]                                               */
  const float *b_x;    /* [D]                                               */
  const float *Lambda; /* [D]              a = sigma(Lambda), Section 2.4   */
  const float *conv_w; /* [4][D]           Section 2.3                      */
  const float *conv_b; /* [D] or NULL                                       */
} rglru_params;

typedef struct rglru_param_grads {
  float *dW_a;     /* [nb][bs][bs] */
  float *dW_x;     /* [nb][bs][bs] */
  float *db_a;     /* [D]          */
  float *db_x;     /* [D]          */
  float *dLambda;  /* [D]          */
  float *dconv_w;  /* [4][D]       */
  float *dconv_b;  /* [D] or NULL (skipped) */
} rglru_param_grads;

/*
 * Temporal Conv1D alone (Section 2.3): x[b,t,d] = sum_k conv_w[k,d] u[b,t-k,d] (+ conv_b[d]).
 *   u              [B][T][D] act, read.
 *   conv_state_in  ring state holding the inputs at positions pos0-3..pos0-1, or NULL (zeros).
 *   pos0           absolute position of u[:,0,:] (>= 0); selects the ring slots.
 *   x_out          [B][T][D] act, written.
 *   conv_state_out ring state after consuming the T inputs, or NULL (not produced). May alias
 *                  conv_state_in.
 * shape.num_blocks is ignored. T == 0 copies the state through and writes nothing else.
 */
int rglru_conv1d(const rglru_shape *shape, const void *u, const float *conv_w,
                 const float *conv_b, const void *conv_state_in, int64_t pos0, void *x_out,
                 void *conv_state_out, void *stream);

/* flags of rglru_scan() */
#define RGLRU_SCAN_LOG_A 1u          /* `a` holds log a_t (<= 0) instead of a_t            */
#define RGLRU_SCAN_NO_INPUT_SCALE 2u /* h_t = a_t h_{t-1} + g_t, without sqrt(1 - a_t^2)   */
#define RGLRU_SCAN_ADJOINT 4u        /* the adjoint recurrence, backwards in time (below);  */
                                     /* only together with RGLRU_SCAN_NO_INPUT_SCALE        */

/*
 * Eq. (4) alone, as a linear scan over given sequences (Section 4.2, "A custom linear scan";
 * the operation whose runtimes Appendix A.3 reports for batch 8, width 1024):
 *     h_t = a_t h_{t-1} + sqrt(1 - a_t^2) g_t,   h_{-1} = h0
 *   a      [B][T][D] act, read: the decay a_t in [0, 1]; with RGLRU_SCAN_LOG_A its logarithm,
 *          the form Appendix A evaluates it in (then sqrt(1 - a_t^2) = sqrt(-expm1(2 log a_t))).
 *   g      [B][T][D] act, read: the gated input i_t x_t.
 *   h0     [B][D] f32 or NULL (zeros).
 *   h      [B][T][D] act, written; must not overlap a or g.
 *   hT     [B][D] f32 or NULL (not produced): the state after the last step.
 *   workspace: rglru_workspace_bytes(shape, RGLRU_OP_SCAN) bytes.
 * The state is carried in fp32 whatever the storage type. Of `shape`, only B, T (>= 0), D and
 * act_dtype are used (the other fields must still be valid). T == 0 writes hT = h0 only.
 * With RGLRU_SCAN_ADJOINT the call runs the adjoint of the unscaled scan (what training through
 * eq. (4) needs; not printed in the paper): for L = sum_t g_t h_t + h0 . h_{T-1} it returns
 *     delta_t = g_t + a_{t+1} delta_{t+1},   delta_{T-1} = g_{T-1} + h0
 * in `h` (delta_t = dL/db_t for h_t = a_t h_{t-1} + b_t; dL/da_t = delta_t h_{t-1}) and
 * a_0 delta_0 = dL/dh_{-1} in `hT`: `g` carries the upstream gradient, `h0` the gradient
 * reaching the final state (NULL = zeros), `a` is the forward call's array, unshifted.
 */
int rglru_scan(const rglru_shape *shape, const void *a, const void *g, const float *h0,
               unsigned flags, void *h, float *hT, void *workspace, size_t workspace_bytes,
               void *stream);

/*
 * Forward over whole sequences: Conv1D then RG-LRU (Sections 2.3-2.4, eqs. 1-4).
 *   u              [B][T][D] act, read.
 *   h0             [B][D] f32 state before the first step, or NULL (zeros).
 *   conv_state_in / pos0 / conv_state_out  as in rglru_conv1d.
 *   y              [B][T][D] act, written (y_t = h_t, rounded to act).
 *   hT             [B][D] f32 state after the last step (unrounded), or NULL. May alias h0.
 *   workspace      >= rglru_workspace_bytes(shape, RGLRU_OP_FORWARD) bytes. For shapes that run on
 *                  the general kernels (fp32 storage, block sizes no matrix-core kernel takes)
 *                  the scratch is optional: with it the forward runs in two passes parallel
 *                  over time, without it (NULL or too small) in one pass serial in time.
 * A sequence may be fed in pieces: passing hT and conv_state_out of one call as h0 and
 * conv_state_in of the next (with pos0 advanced by T) gives the one-shot result.
 * T == 0 copies h0 to hT and the conv state through.
 */
int rglru_forward(const rglru_shape *shape, const rglru_params *params, const void *u,
                  const float *h0, const void *conv_state_in, int64_t pos0, void *y, float *hT,
                  void *conv_state_out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * rglru_forward without a workspace argument, for callers that cannot allocate device memory or
 * carry a workspace along: code that runs under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc. The scratch rglru_forward takes from its workspace (status
 * word, carry records of sequences sliced in time, W_x in half precision) lives in a static
 * device array of RGLRU_STATIC_SCRATCH_BYTES inside the library instead; each GPU the library
 * runs on holds its own copy until the process ends. The call allocates and frees nothing.
 *   Arguments, results and error codes: as rglru_forward (same kernels, same results bit for bit).
 *   RGLRU_ERR_WORKSPACE if rglru_workspace_bytes(shape, RGLRU_OP_FORWARD) exceeds
 *   RGLRU_STATIC_SCRATCH_BYTES (the five workloads this library is tuned for need 2 - 9 MB);
 *   nothing is launched then.
 * All calls on one GPU share that GPU's array: two calls that overlap in time on the same GPU
 * (different streams or threads) race on it - serialise them, or give the overlapping ones a
 * workspace of their own through rglru_forward. The array keeps the last call's contents; the
 * call clears what must start at zero with a kernel on `stream`, so it may be captured into a
 * HIP graph after one ordinary call on that GPU (the first call on a GPU looks the array's
 * address up).
 */
#define RGLRU_STATIC_SCRATCH_BYTES ((size_t)16 << 20)
int rglru_forward_static(const rglru_shape *shape, const rglru_params *params, const void *u,
                         const float *h0, const void *conv_state_in, int64_t pos0, void *y,
                         float *hT, void *conv_state_out, void *stream);

/*
 * One decode step (Section 5; state sizes of Appendix F): the forward equations for one new
 * token per sequence, with both states updated in place.
 *   u_t        [B][D] act, the new input of every sequence.
 *   h          [B][D] f32, recurrent state: read as h_{t-1}, overwritten with h_t.
 *   conv_state [B][3][D] act ring: slots (pos-1, pos-2, pos-3) mod 3 are read as lags 1..3,
 *              then slot pos mod 3 is overwritten with u_t.
 *   pos        absolute position of the new token (>= 0), one value for the whole batch.
 *   y_t        [B][D] act, written.
 * shape.T is ignored. No workspace is needed.
 */
int rglru_decode_step(const rglru_shape *shape, const rglru_params *params, const void *u_t,
                      float *h, void *conv_state, int64_t pos, void *y_t, void *stream);

/*
 * Backward of rglru_forward for the loss L = sum(dy * y) + sum(dhT * hT): the adjoint of
 * eqs. (1)-(4) and of the Conv1D (the paper prints no backward; it is the reverse-time scan
 * delta_t = dy_t + a_{t+1} delta_{t+1} followed by the pointwise, block-diagonal and
 * convolution adjoints).
 *   u, h0, conv_state_in, pos0   the forward call's inputs.
 *   y          [B][T][D] act, the forward call's output (supplies h_{t-1}).
 *   dy         [B][T][D] act, upstream gradient.
 *   dhT        [B][D] f32 gradient reaching hT, or NULL (zeros).
 *   du         [B][T][D] act, written.
 *   dh0        [B][D] f32, written, or NULL (skipped).
 *   grads      parameter gradients, f32, summed over B and T, overwritten. Every pointer
 *              except dconv_b is required. The carried-in conv state receives no gradient.
 *   workspace  >= rglru_workspace_bytes(shape, RGLRU_OP_BACKWARD) bytes.
 * T must be >= 1.
 */
int rglru_backward(const rglru_shape *shape, const rglru_params *params, const void *u,
                   const float *h0, const void *conv_state_in, int64_t pos0, const void *y,
                   const void *dy, const float *dhT, void *du, float *dh0,
                   const rglru_param_grads *grads, void *workspace, size_t workspace_bytes,
                   void *stream);

/*
 * Forward and backward over packed sequences: a row of the batch may hold several documents
 * back to back. Sections 2.3-2.4 define the Conv1D and the recurrence per sequence and say
 * nothing about packing; the convention here is that NOTHING crosses the first step of a
 * document: at a step t with reset[b][t] != 0 the recurrence starts from h_{t-1} := 0, the
 * Conv1D takes every input before t as zero, and in the backward no gradient flows from the
 * document into the steps (or the incoming states) in front of it. Each document then gets
 * exactly what it would get as a sequence of its own.
 *   reset      [B][T] bytes, read, or NULL (no boundaries: rglru_forward / rglru_backward).
 *              reset[b][0] != 0 makes row b ignore h0 and conv_state_in.
 *   hT, conv_state_out   the states after the last step, those of the row's last document: ring
 *              slots of inputs in front of that document's first step hold zeros.
 *   dh0        zero for a row whose reset[b][0] != 0.
 *   every other argument: as in rglru_forward / rglru_backward; conv_width 0 is accepted.
 *   workspace  rglru_workspace_bytes(shape, RGLRU_OP_FORWARD_PACKED) bytes for the forward,
 *              rglru_workspace_bytes(shape, RGLRU_OP_BACKWARD_PACKED) bytes for the backward.
 * Both calls run on the fused matrix-core kernels of rglru_forward / rglru_backward where those
 * take the shape - the forward for bf16 storage and gate blocks of 128 - 256 channels, the
 * backward for bf16 storage and blocks of 256 channels. The boundaries reach the kernels as bit
 * masks per tile of 32 steps (a prep kernel makes them in the workspace); rglru_workspace_status
 * with RGLRU_OP_FORWARD_PACKED / RGLRU_OP_BACKWARD_PACKED works as for the unpacked calls. Every
 * other shape runs on the library's general kernels (one workgroup per (sequence, gate block),
 * plain fp32 arithmetic for either storage type), where no kernel waits on another.
 */
int rglru_forward_packed(const rglru_shape *shape, const rglru_params *params, const void *u,
                         const uint8_t *reset, const float *h0, const void *conv_state_in,
                         int64_t pos0, void *y, float *hT, void *conv_state_out, void *workspace,
                         size_t workspace_bytes, void *stream);
int rglru_backward_packed(const rglru_shape *shape, const rglru_params *params, const void *u,
                          const uint8_t *reset, const float *h0, const void *conv_state_in,
                          int64_t pos0, const void *y, const void *dy, const float *dhT, void *du,
                          float *dh0, const rglru_param_grads *grads, void *workspace,
                          size_t workspace_bytes, void *stream);

/*
 * Complex-gated LRU (Appendix B, "Complex-Gated Linear Recurrent Unit"): the RG-LRU with the
 * complex diagonal recurrence weight a~ = sigmoid(Lambda) e^{i theta}. The D real channels of
 * x_t (D even) are read as H = D / 2 complex ones, first half real parts, second half
 * imaginary parts; gates, decay and state have H entries:
 *     r_t = sigmoid(W_a x_t + b_a),  i_t = sigmoid(W_x x_t + b_x)            in R^H
 *     a~_t = a~^(c r_t) = exp(c r_t (log sigmoid(Lambda) + i theta))
 *     h~_t = a~_t h~_{t-1} + sqrt(1 - |a~_t|^2) (i_t x~_t),   y_t = [Re h~_t ; Im h~_t]  in R^D
 * The appendix does not say how the block-diagonal gates of Section 4.1 carry over. Here gate
 * block g (of shape.num_blocks; H % num_blocks == 0, hs = H / num_blocks) owns the complex
 * channels g*hs .. (g+1)*hs-1 and sees the real and the imaginary parts of exactly those:
 * W[g] is [hs][2 hs], input k < hs = real channel g*hs + k, input k >= hs = real channel
 * H + g*hs + (k - hs). One block is the appendix's dense H x D matrix. The power is
 * exp(c r_t log a~) with log a~ = log sigmoid(Lambda) + i theta (theta as given, not reduced).
 * States ([B][D] f32) hold [Re h~ ; Im h~] like y_t. The Conv1D in front (shape.conv_width 4,
 * or 0 for none) is the real layer's, on all D channels, with the same ring state.
 */
typedef struct rglru_cg_params {
  const void *W_a;     /* [nb][hs][2 hs] w   recurrence-gate weights */
  const void *W_x;     /* [nb][hs][2 hs] w   input-gate weights      */
  const float *b_a;    /* [H]                                         */
  const float *b_x;    /* [H]                                         */
  const float *Lambda; /* [H]   |a~| = sigmoid(Lambda)                */
  const float *theta;  /* [H]   arg a~                                */
  const float *conv_w; /* [4][D] or NULL with conv_width 0            */
  const float *conv_b; /* [D] or NULL                                 */
} rglru_cg_params;

typedef struct rglru_cg_param_grads {
  float *dW_a;     /* [nb][hs][2 hs] */
  float *dW_x;     /* [nb][hs][2 hs] */
  float *db_a;     /* [H]            */
  float *db_x;     /* [H]            */
  float *dLambda;  /* [H]            */
  float *dtheta;   /* [H]            */
  float *dconv_w;  /* [4][D]; not produced with conv_width 0 */
  float *dconv_b;  /* [D] or NULL (skipped) */
} rglru_cg_param_grads;

/*
 * Forward, decode step and backward of the complex-gated layer. Arguments, layouts, state
 * handling and error codes are those of rglru_forward, rglru_decode_step and rglru_backward
 * (the backward is the adjoint for the real loss L = sum(dy * y) + sum(dhT * hT), derived from
 * the appendix's equations with real and imaginary parts as independent variables; it also
 * returns dtheta; it takes no y: the gradient of the decay multiplies the state's adjoint by
 * conj(h~_{t-1}), which needs more than the 8 bits of a bf16 y, so the backward recomputes the
 * states in fp32 into its workspace). They run on shape-generic kernels (fp32 arithmetic for either storage
 * type); no kernel waits on another. The forward's workspace is optional (NULL, or
 * rglru_workspace_bytes(shape, RGLRU_OP_CG_FORWARD) bytes: with it the forward runs in two passes
 * parallel over time, without it in one pass, a workgroup per (sequence, gate block)); the decode
 * step needs none; the backward needs rglru_workspace_bytes(shape, RGLRU_OP_CG_BACKWARD) bytes.
 * hs may be at most 1024.
 */
int rglru_cg_forward(const rglru_shape *shape, const rglru_cg_params *params, const void *u,
                     const float *h0, const void *conv_state_in, int64_t pos0, void *y, float *hT,
                     void *conv_state_out, void *workspace, size_t workspace_bytes, void *stream);
int rglru_cg_decode_step(const rglru_shape *shape, const rglru_cg_params *params, const void *u_t,
                         float *h, void *conv_state, int64_t pos, void *y_t, void *stream);
int rglru_cg_backward(const rglru_shape *shape, const rglru_cg_params *params, const void *u,
                      const float *h0, const void *conv_state_in, int64_t pos0, const void *dy,
                      const float *dhT, void *du, float *dh0, const rglru_cg_param_grads *grads,
                      void *workspace, size_t workspace_bytes, void *stream);

/* flags of the merge calls */
#define RGLRU_MERGE_GELU_TANH 1u /* GeLU in its tanh form instead of z * Phi(z)             */
#define RGLRU_MERGE_SEPARATE 2u  /* forward: run the merge as a kernel of its own after the  */
                                 /* recurrence instead of as its epilogue (same results up  */
                                 /* to rounding; for measurements)                          */

/*
 * Forward with the recurrent block's merge as its epilogue (Section 2.3, "Recurrent block":
 * the RG-LRU branch is multiplied element by element with GeLU of the block's other branch):
 *   out_t = y_t * GeLU(branch_t),   y = rglru_forward(u, ...).
 * GeLU(z) = z * Phi(z), Phi the standard normal CDF; RGLRU_MERGE_GELU_TANH selects
 * 0.5 z (1 + tanh(sqrt(2/pi) (z + 0.044715 z^3))). The product is formed in fp32 from y_t as
 * stored (rounded to act) and rounded to act. Where it is faster the merge runs as the
 * epilogue of the recurrence kernel (y then never travels through memory unless asked for),
 * else as a streaming kernel after it; the results agree up to rounding.
 *   branch     [B][T][D] act, read: the other branch before its non-linearity.
 *   out        [B][T][D] act, written. Must not alias u, branch or y.
 *   y          [B][T][D] act, written as by rglru_forward, or NULL (skipped). Training keeps
 *              it for rglru_backward_merge; inference passes NULL and saves its write.
 *   the other arguments, the workspace (RGLRU_OP_FORWARD_MERGE) and T == 0: as rglru_forward.
 */
int rglru_forward_merge(const rglru_shape *shape, const rglru_params *params, const void *u,
                        const void *branch, const float *h0, const void *conv_state_in,
                        int64_t pos0, unsigned flags, void *out, void *y, float *hT,
                        void *conv_state_out, void *workspace, size_t workspace_bytes,
                        void *stream);

/*
 * The decode step (Section 5; Conv1D of Section 2.3 feeding eqs. (1)-(4) for one new token)
 * with a position per sequence, for a batch whose sequences are at different lengths: the
 * ring slots of sequence b follow pos[b]; the arithmetic is that of rglru_decode_step.
 *   pos        [B] int64, DEVICE pointer (8-byte aligned), read by the kernels, owned by the
 *              caller: absolute position of the new token of each sequence. Values must be
 *              >= 0; they are not checked on the host, a negative one selects a slot as if it
 *              were taken modulo 3 (never an access outside conv_state).
 *   u_t, h, conv_state, y_t: as in rglru_decode_step (states updated in place).
 * shape.T is ignored. No workspace is needed. Errors: RGLRU_ERR_INVALID_ARG for a NULL or
 * misaligned pointer or an invalid shape; nothing is launched then.
 */
int rglru_decode_step_at(const rglru_shape *shape, const rglru_params *params, const void *u_t,
                         float *h, void *conv_state, const int64_t *pos, void *y_t, void *stream);

/*
 * One decode step with the merge as its epilogue: rglru_decode_step, then
 * out_t = y_t * GeLU(branch_t) is what is written (RGLRU_MERGE_SEPARATE is not accepted).
 *   branch_t   [B][D] act, read.
 *   out_t      [B][D] act, written. Must not alias branch_t or u_t.
 */
int rglru_decode_step_merge(const rglru_shape *shape, const rglru_params *params, const void *u_t,
                            const void *branch_t, float *h, void *conv_state, int64_t pos,
                            unsigned flags, void *out_t, void *stream);

/*
 * Backward of rglru_forward_merge for the loss L = sum(dout * out) + sum(dhT * hT): the
 * adjoint of the merge, dy = dout * GeLU(branch) and dbranch = dout * y * GeLU'(branch),
 * followed by rglru_backward on dy. dy is not rounded to act in between (in bf16 storage it
 * travels as the sum of two bf16 tensors in the workspace, 16 significant bits): the reverse scan
 * accumulates dy over the memory of the recurrence, and an 8-bit dy would move single elements
 * of dW_a by several times the bf16 tolerance.
 *   branch, y  [B][T][D] act: the forward call's input and its saved y.
 *   dout       [B][T][D] act, upstream gradient of out.
 *   dbranch    [B][T][D] act, written. May alias dout or branch.
 *   the other arguments: as rglru_backward; workspace: RGLRU_OP_BACKWARD_MERGE.
 */
int rglru_backward_merge(const rglru_shape *shape, const rglru_params *params, const void *u,
                         const void *branch, const float *h0, const void *conv_state_in,
                         int64_t pos0, unsigned flags, const void *y, const void *dout,
                         const float *dhT, void *du, void *dbranch, float *dh0,
                         const rglru_param_grads *grads, void *workspace,
                         size_t workspace_bytes, void *stream);

/* Bytes of workspace `op` (RGLRU_OP_*) needs for `shape`; 0 if none or if shape is invalid. */
size_t rglru_workspace_bytes(const rglru_shape *shape, int op);

/*
 * Health check of the calls made on a workspace (it synchronises). When sequences are cut into
 * time slices, the workgroups of a launch hand carries to each other through records in
 * `workspace`. Every wait on such a record is bounded. A wait that expires - it would mean that
 * the workgroups of the launch were not all resident at once, which the launch sizes rule out
 * on a GPU the process has to itself - does not hang: it marks the workspace's status word,
 * and from that point on the outputs of that call are filled with NaN, and so are the outputs of
 * every later call on the same workspace (each call looks at the word before it starts), so that
 * the failure cannot go unnoticed downstream. This function waits for `stream`, reads the word
 * left by the calls of `op` (RGLRU_OP_FORWARD, _BACKWARD, _SCAN or a _MERGE variant) that ran
 * with this `shape` and `workspace`, and returns RGLRU_OK, or RGLRU_ERR_TIMEOUT after clearing
 * the word (the next call starts afresh; see rglru_set_max_time_slices for a retry that cannot
 * time out), or RGLRU_ERR_INVALID_ARG / RGLRU_ERR_HIP. Uninitialised workspace memory is never
 * mistaken for the mark (a 16-byte pattern).
 */
int rglru_workspace_status(const rglru_shape *shape, int op, const void *workspace, void *stream);

/*
 * Upper bound on the number of time slices a sequence is cut into (process-wide; 0 = automatic,
 * the default; it also bounds the contiguous windows that the forward of a single long prompt is
 * run in, which exchange nothing while they run and cannot time out). With 1 no kernel ever waits on another workgroup: every (sequence, gate block)
 * pair is walked by a single workgroup, slower for few long sequences but independent of all
 * workgroups of a launch being resident at once. This is the setting to retry with after
 * rglru_workspace_status has reported RGLRU_ERR_TIMEOUT (e.g. when another process occupies part
 * of the GPU). Workspace sizes depend on it: query them again after changing it.
 * Returns RGLRU_OK or RGLRU_ERR_INVALID_ARG (negative value).
 */
int rglru_set_max_time_slices(int max_slices);

/* Description of the last error returned on the calling thread ("" if none). */
const char *rglru_last_error(void);

/*
 * Kernel timing for benchmarks (not part of the method). While enabled on the calling thread,
 * every kernel an entry point launches is bracketed by two HIP events recorded on that call's
 * stream; the library owns the events. rglru_timing_count() is the number of kernels recorded
 * since the last rglru_timing_enable(1) (at most 8192; later launches are not recorded).
 * rglru_timing_get() returns the name of record `index` (a static string) and, once the caller
 * has synchronised the stream, the kernel's duration in milliseconds in *ms.
 * rglru_timing_select(name) restricts the bracketing to the kernels of that name (NULL or ""
 * = every kernel again): two event records per launch are not free, and a run that only needs
 * one kernel's duration should not pay for all of them.
 * Returns RGLRU_OK, RGLRU_ERR_INVALID_ARG (bad index / NULL / name too long) or RGLRU_ERR_HIP.
 */
int rglru_timing_enable(int enable);
int rglru_timing_select(const char *kernel_name);
int rglru_timing_count(void);
int rglru_timing_get(int index, const char **name, float *ms);

/* Library version: major * 10000 + minor * 100 + patch. */
int rglru_version(void);

#ifdef __cplusplus
}
#endif
#endif /* RGLRU_H */
