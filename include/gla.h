/*
 * gla.h - C ABI of the MI355X (gfx950) implementation of the gated-linear-attention
 * (GLA) token mixer used in the DiG diffusion backbone: the forward pass (gla_fwd*),
 * its variants with the gate prologue and output epilogue (gla_fwd_fused) and with
 * several scan orders summed (gla_fwd_multi), the backward pass (gla_bwd*), the same
 * with the full gate matrix alpha_t^T beta_t (gla_fwd_gates, gla_fwd_fused_gates,
 * gla_bwd_gates), and the depth-wise convolution of the DiG block's reorientation
 * module (gla_srem_dwconv).
 *
 * Operation (DiG paper, Sec. 3.1 "Gated Linear Attention Transformer",
 * Eq. (attn_gla), rows 1-3, with the gate G_t reduced to its key-side factor
 * alpha_t, i.e. beta_t = 1, except in the *_gates entry points):
 *
 *     S_t = diag(alpha_t) S_{t-1} + k_t^T v_t ,     o_t = q_t S_t ,     S_0 = 0
 *
 * per (batch, head), S in R^{dk x dv}, evaluated in the chunk-parallel form of
 * Sec. 3.5 ("Efficiency Analysis": the sequence is cut into chunks that are
 * computed on-chip, cost O(T M D + T D^2)).  The tokens of one image form a
 * grid_h x grid_w grid; the recurrence runs along one of the four scan orders
 * that the DiG block obtains by alternately transposing and flipping the token
 * grid (Sec. 3.3, Algorithm 1; operators of the supplementary Algorithms 2-4).
 * The permutation is folded into the kernels' address arithmetic: tensors stay
 * in canonical order and nothing is transposed in memory.
 *
 * Conventions common to every entry point
 * ---------------------------------------
 * Pointers marked DEVICE are device (HBM) addresses owned by the caller; the
 * library never frees, reallocates or retains them.  All tensors are dense,
 * row-major, in canonical token order n = r * grid_w + c for every scan order:
 *
 *     q, k        : [B, H, T, dk]   element type qkv_dtype (bf16 or fp32)
 *     log_alpha   : [B, H, T, dk]   fp32, log(alpha_t) <= 0 (e.g. logsigmoid(z)/tau)
 *     v           : [B, H, T, dv]   element type qkv_dtype
 *     out         : [B, H, T, dv]   element type out_dtype; out[n] = o at token n
 *     final_state : [B, H, dk, dv]  fp32, the state after the last scan step; may be NULL
 *
 * T must equal grid_h * grid_w.  No 1/sqrt(dk) scale is applied (the recurrence
 * has none); scale q beforehand.  Supported head sizes: 1 <= dk <= 64,
 * 1 <= dv <= 128.  T need not be a multiple of the chunk length.
 *
 * Calls enqueue work on `stream` (a hipStream_t passed as void*, NULL = the
 * default stream) and return without synchronising the host; results are valid
 * once the stream reaches that point.  Inputs must stay unmodified until then.
 * Outputs must not alias inputs.  The current HIP device must be the one that
 * owns the buffers.
 *
 * Every function returns a gla_status (0 = success).  An argument error (every
 * status but GLA_ERR_HIP) is found before anything is enqueued: no kernel has
 * run and no output byte has been written.  GLA_ERR_HIP reports a failed runtime
 * call or launch; a call is several kernels, so the earlier ones of that call
 * may already be enqueued and the outputs are then undefined.
 *
 * Preconditions that are not checked: log_alpha <= 0 and finite inputs.  Further
 * limits of the engines (see gla_engine):
 *  - bf16 hi/lo MFMA engine: the summed |log_alpha| over any 64 consecutive scan
 *    steps of one key channel stays below 80 (true for alpha = sigmoid(z)^(1/16)
 *    whenever z > -20).  GLA_ENGINE_RECURRENT has no such limit.
 *  - fp16 MFMA engine (what GLA_ENGINE_AUTO takes for the plain forward pass, and for
 *    gla_fwd_fused without the output epilogue, on bf16 inputs with 17..64 key
 *    channels and more than four chunks): its operands
 *    cover a decay of at most 2^-11 per key channel over 32 consecutive scan steps
 *    (alpha above about 0.79 on average; sigmoid(z)^(1/16) with z > -3.7) and
 *    inputs whose largest |q|, |k| lie in [2^-8, 8] and |v| in [2^-8, 2^14].  This
 *    IS checked, on the device: a (batch, head) sequence outside the range is
 *    recomputed in the same call by the bf16 hi/lo kernel, one work-group walking
 *    the whole sequence - correct, but many times slower for that sequence.
 *    Callers whose gates close faster than that as a rule should select
 *    GLA_ENGINE_MFMA.
 *  - Where the output pass chains the span states itself (gla_carry), a thread
 *    stops adding earlier spans once the decay accumulated on its key channels is
 *    below 2^-40: what is left out is at most 2^-40 of what those earlier states
 *    hold.  The bound is relative to the earlier states, not to the sum so far
 *    (a thread whose sum is still exactly zero, e.g. behind a padded tail of
 *    all-zero k or v, does go on): sequences whose later spans are many orders
 *    of magnitude smaller than the earlier ones lose the decayed remainder of
 *    the earlier ones.  GLA_CARRY_KERNEL has no cut-off.
 *
 * The entry points that take a caller workspace only enqueue kernels, with one
 * exception: the first use of a kernel instantiation on a device raises its
 * dynamic-LDS limit (hipFuncSetAttribute).  Before capturing calls into a HIP
 * graph, or entering a region that must not touch the runtime, run each call
 * once with the same shapes and options.
 */
#ifndef GLA_H_
#define GLA_H_

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    GLA_OK = 0,
    GLA_ERR_NULL = 1,        /* a required pointer is NULL */
    GLA_ERR_SHAPE = 2,       /* non-positive size, grid_h*grid_w != T, or a bad enum value */
    GLA_ERR_UNSUPPORTED = 3, /* dk > 64, dv > 128, or a dtype / engine combination not built */
    GLA_ERR_ALIGN = 4,       /* a base pointer is not 16-byte aligned */
    GLA_ERR_WORKSPACE = 5,   /* workspace NULL or smaller than gla_fwd_workspace_bytes() */
    GLA_ERR_HIP = 6          /* the HIP runtime reported an error (allocation or launch) */
} gla_status;

/* Scan orders (Sec. 3.3 / Algorithm 1).  Scan step s visits canonical token n:
 *   ROW_FWD  n = s                       ROW_REV  n = T-1-s
 *   COL_FWD  n = (s % grid_h) * grid_w + s / grid_h   (down a column, then the next column)
 *   COL_REV  the COL_FWD sequence read from its last step backwards              */
typedef enum { GLA_SCAN_ROW_FWD = 0, GLA_SCAN_ROW_REV = 1,
               GLA_SCAN_COL_FWD = 2, GLA_SCAN_COL_REV = 3 } gla_scan_dir;

typedef enum { GLA_DT_F32 = 0, GLA_DT_BF16 = 1 } gla_dtype;

/* Options for gla_set_option (process-wide, meant for tuning and tests). */
typedef enum {
    GLA_OPT_CHUNKS_PER_SPAN = 0, /* 0 = choose automatically; n > 0 = n 64-token chunks per work-group */
    GLA_OPT_ENGINE = 1,          /* gla_engine */
    GLA_OPT_CARRY = 2,           /* gla_carry */
    GLA_OPT_BWD_SPLIT = 3,       /* 0 = the backward pass computes dk and dv of a chunk in one kernel (MFMA engine);
                                    1 = in two kernels (the forward output pass for dv, the row read for dk) */
    GLA_OPT_RANGE_FALLBACK = 4   /* 1 (default) = after the fp16 engine's passes, the (batch, head) sequences that
                                    left its range are recomputed by the bf16 hi/lo kernel (one more launch, whose
                                    work-groups return at once when no flag is raised); 0 = that launch is skipped
                                    (for callers that know their gates and inputs stay in range, and for
                                    measurements) */
} gla_option;
typedef enum {
    GLA_ENGINE_AUTO = 0,      /* bf16 inputs with dk % 4 == 0 and dv % 8 == 0 -> an MFMA engine (the fp16 one for the
                                 plain forward pass and for gla_fwd_fused without r_pre, with 17..64 key channels
                                 and more than four chunks, else the bf16 hi/lo one), otherwise recurrent */
    GLA_ENGINE_RECURRENT = 1, /* fp32 token-by-token arithmetic inside each span; any dtype, any gates */
    GLA_ENGINE_MFMA = 2,      /* bf16 hi/lo MFMA chunk form (Sec. 3.5) in every pass; bf16 inputs only */
    GLA_ENGINE_MFMA_FP16 = 3  /* fp16 operands in both passes of the plain forward call and of gla_fwd_fused without
                                 r_pre (producer / consumer waves), the bf16 hi/lo kernel as range fallback;
                                 GLA_ERR_UNSUPPORTED where it does not apply (the output epilogue, other entry
                                 points, fp32 inputs, fewer than 17 key channels) */
} gla_engine;

/* Where the states of the spans of one (batch, head) are chained, S_start(r+1) = diag(Gamma_r) S_start(r) + U_r
 * (the recurrence of Eq. (attn_gla) applied span by span). */
typedef enum {
    GLA_CARRY_AUTO = 0,          /* in the output pass when an MFMA engine runs with at most 128 spans per head */
    GLA_CARRY_KERNEL = 1,        /* a kernel of its own between the two passes */
    GLA_CARRY_IN_OUTPUT_PASS = 2 /* each output work-group chains the local states before its span, whatever the
                                    span count (the recurrent engine has no such path and keeps the kernel) */
} gla_carry;

typedef void *gla_stream_t; /* a hipStream_t */

/*
 * gla_fwd - GLA forward for bf16 q/k/v, fp32 log_alpha, fp32 out
 * (Eq. (attn_gla) rows 1-3 along `scan_dir`; chunk form of Sec. 3.5).
 *
 *   q, k, v      DEVICE, bf16, layouts above            (read)
 *   log_alpha    DEVICE, fp32                           (read)
 *   out          DEVICE, fp32 [B,H,T,dv]                (written)
 *   final_state  DEVICE, fp32 [B,H,dk,dv] or NULL       (written if not NULL)
 *
 * Uses a library-owned scratch buffer per device that grows on demand with
 * hipMalloc (which synchronises the device the first time a larger problem is
 * seen) and is kept until the process ends; concurrent calls on different
 * streams of one device would share it and are not supported - use gla_fwd_ex
 * with separate workspaces for that.
 */
int gla_fwd(const void *q, const void *k, const void *v, const float *log_alpha,
            int B, int H, int T, int dk, int dv, int grid_h, int grid_w, int scan_dir,
            float *out, float *final_state, gla_stream_t stream);

/*
 * gla_fwd_static - gla_fwd for callers that cannot allocate device memory: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results and status codes as gla_fwd; the span states live in a static
 * device array of GLA_STATIC_SCRATCH_BYTES that every GPU the library runs on holds
 * until the process ends.  The call itself makes no hipMalloc / hipFree and uses no
 * allocating library routine; the kernels it launches are gla_fwd's.
 *
 * GLA_ERR_WORKSPACE if the launch plan of the problem needs more than the array holds
 * (B * H * spans * (dk * dv + dk + dv) floats, spans = 64-token chunks / chunks per
 * work-group; the DiG-XL/2 shape at 2048 px uses about 7 MiB); nothing is enqueued then.
 * All calls on one GPU share that GPU's array: calls that overlap on one GPU (different
 * streams or threads) race.  Nothing in it needs clearing between calls: every call
 * writes the span states before it reads them.  As for every entry point that takes a
 * workspace, the first call of a kernel variant in the process configures it
 * (hipFuncSetAttribute); make one call outside graph capture before capturing.
 */
#define GLA_STATIC_SCRATCH_BYTES (16u << 20)
int gla_fwd_static(const void *q, const void *k, const void *v, const float *log_alpha,
                   int B, int H, int T, int dk, int dv, int grid_h, int grid_w, int scan_dir,
                   float *out, float *final_state, gla_stream_t stream);

/*
 * gla_fwd_ex - the same operation with explicit element types and a caller-owned
 * workspace; never allocates.
 *
 *   qkv_dtype        gla_dtype of q, k, v
 *   out_dtype        gla_dtype of out (final_state is always fp32)
 *   workspace        DEVICE, 16-byte aligned, at least gla_fwd_workspace_bytes(...) bytes;
 *                    contents on entry are ignored, contents on return are unspecified
 */
int gla_fwd_ex(const void *q, const void *k, const void *v, const float *log_alpha,
               int B, int H, int T, int dk, int dv, int grid_h, int grid_w, int scan_dir,
               int qkv_dtype, int out_dtype, void *out, float *final_state,
               void *workspace, size_t workspace_bytes, gla_stream_t stream);

/* Memory order of q, k, log_alpha ([.., dk]) and v, out ([.., dv]); final_state and initial_state are always
 * [B,H,dk,dv].  BTHD is the (B, T, D) token stream of Algorithm 1 with D = H * d seen per head. */
typedef enum { GLA_LAYOUT_BHTD = 0, GLA_LAYOUT_BTHD = 1 } gla_layout;

/*
 * gla_fwd_layout - gla_fwd_ex for either memory order, starting from a given state
 * (Eq. (attn_gla) row 1 with S_0 = initial_state instead of zero: the recurrence
 * continued from an earlier call's final_state, e.g. a sequence fed in pieces).
 *
 *   layout           gla_layout of q, k, v, log_alpha and out (dense, no padding)
 *   initial_state    DEVICE, fp32 [B,H,dk,dv], 16-byte aligned, or NULL for a zero state   (read)
 *
 * Everything else as gla_fwd_ex; GLA_ERR_SHAPE for an unknown layout.  With the MFMA
 * engine a (batch, head) view must span less than 2 GiB (T * H * max(dk, dv) * 4 bytes
 * in BTHD order), otherwise the call falls back to the recurrent engine.
 */
int gla_fwd_layout(const void *q, const void *k, const void *v, const float *log_alpha,
                   int B, int H, int T, int dk, int dv, int grid_h, int grid_w, int scan_dir,
                   int qkv_dtype, int out_dtype, int layout, const float *initial_state,
                   void *out, float *final_state,
                   void *workspace, size_t workspace_bytes, gla_stream_t stream);

/*
 * gla_fwd_gates - the recurrence with the full gate matrix of Sec. 3.1, G_t = alpha_t^T beta_t
 * (Eq. (gate_gla) for the key side, Eq. (gate_gla_2) for the value side), applied element-wise
 * in Eq. (attn_gla) row 1:   S_t = (alpha_t^T beta_t) * S_{t-1} + k_t^T v_t ,  o_t = q_t S_t.
 *
 *   log_beta         DEVICE, fp32, shaped and laid out like v ([B,H,T,dv] or [B,T,H,dv]), 16-byte
 *                    aligned; log of the value-side gate, <= 0                                  (read)
 *
 * Everything else as gla_fwd_layout (log_beta = 0 gives its result).  bf16 q, k, v with
 * dk % 4 == 0, dv % 8 == 0, dk <= 40 and dv <= 80 run on the MFMA engine (chunk form with both
 * decays factorised: the values are gated like the keys and carried as bf16 hi/lo pairs); every
 * other element type and head size runs on the token-by-token fp32 engine.
 * GLA_ERR_UNSUPPORTED if the engine option forces the MFMA engine
 * onto a case it does not cover, GLA_ERR_NULL for a NULL log_beta.
 */
int gla_fwd_gates(const void *q, const void *k, const void *v, const float *log_alpha, const float *log_beta,
                  int B, int H, int T, int dk, int dv, int grid_h, int grid_w, int scan_dir,
                  int qkv_dtype, int out_dtype, int layout, const float *initial_state,
                  void *out, float *final_state, void *workspace, size_t workspace_bytes, gla_stream_t stream);

/*
 * gla_bwd - gradients of a scalar loss L that depends on `out` of gla_fwd_ex (zero initial
 * state, [B,H,T,d] order) with respect to q, k, v and log_alpha: Eq. (attn_gla) rows 1-3
 * differentiated in reverse mode.  With S_s the state after scan step s and
 * G_s = q_s^T dO_s + diag(alpha_{s+1}) G_{s+1} the gradient that reaches it:
 *   dq_s = S_s dO_s^T,  dk_s = G_s v_s^T,  dv_s = k_s G_s,
 *   dlog_alpha_s = sum over scan steps s' >= s of (q_s' * dq_s' - k_s' * dk_s').
 *
 *   q, k, v, d_out   DEVICE, qkv_dtype (d_out = dL/d out, shaped like v)              (read)
 *   log_alpha        DEVICE, fp32                                                     (read)
 *   dq, dk_grad, dlog_alpha   DEVICE, fp32 [B,H,T,dk];  dv_grad  DEVICE, fp32 [B,H,T,dv]   (written)
 *   workspace        DEVICE, 16-byte aligned, at least gla_bwd_workspace_bytes(...) bytes
 *
 * Same status codes as gla_fwd_ex.  Never allocates.
 */
int gla_bwd(const void *q, const void *k, const void *v, const float *log_alpha, const void *d_out,
            int B, int H, int T, int dk, int dv, int grid_h, int grid_w, int scan_dir, int qkv_dtype,
            float *dq, float *dk_grad, float *dv_grad, float *dlog_alpha,
            void *workspace, size_t workspace_bytes, gla_stream_t stream);
size_t gla_bwd_workspace_bytes(int B, int H, int T, int dk, int dv, int qkv_dtype);

/*
 * gla_bwd_gates - gla_bwd for the recurrence of gla_fwd_gates (two-sided gate alpha_t^T beta_t,
 * zero initial state, [B,H,T,d] order).  The gradient that reaches the state obeys
 * G_s = q_s^T dO_s + (alpha_{s+1}^T beta_{s+1}) * G_{s+1}; dq, dk, dv as in gla_bwd, and
 *   dlog_alpha_s = sum over s' >= s of (q_s' * dq_s' - k_s' * dk_s'),
 *   dlog_beta_s  = sum over s' >= s of (o_s' * dO_s' - v_s' * dv_s')      (o = the forward outputs,
 *                                                                           recomputed in the workspace).
 *
 *   log_beta         DEVICE, fp32 [B,H,T,dv]                                           (read)
 *   out_fwd          DEVICE, fp32 [B,H,T,dv]: `out` of gla_fwd_gates on the same inputs, or NULL
 *                    (the outputs are then recomputed, one more pass over the sequence)          (read)
 *   dlog_beta        DEVICE, fp32 [B,H,T,dv]                                           (written)
 *   workspace        DEVICE, 16-byte aligned, at least gla_bwd_gates_workspace_bytes(...) bytes
 *
 * Everything else as gla_bwd.  Engines as gla_fwd_gates (MFMA chunk form for bf16 rows with
 * dk % 4 == 0, dv % 8 == 0, dk <= 40, dv <= 80; token by token in fp32 otherwise).  Never allocates.
 */
int gla_bwd_gates(const void *q, const void *k, const void *v, const float *log_alpha, const float *log_beta,
                  const void *d_out, const float *out_fwd, int B, int H, int T, int dk, int dv, int grid_h, int grid_w, int scan_dir,
                  int qkv_dtype, float *dq, float *dk_grad, float *dv_grad, float *dlog_alpha, float *dlog_beta,
                  void *workspace, size_t workspace_bytes, gla_stream_t stream);
size_t gla_bwd_gates_workspace_bytes(int B, int H, int T, int dk, int dv, int qkv_dtype);

/*
 * gla_bwd_reuse - gla_bwd that takes the span states of S from the workspace of the forward
 * call instead of recomputing them (one of the two state passes of the backward pass is the
 * state pass of the forward pass).
 *
 *   fwd_workspace        DEVICE, the workspace that gla_fwd_ex / gla_fwd_layout (same layout, no
 *                        initial state) / gla_fwd_multi's last scan order used for the SAME
 *                        q, k, v, log_alpha, sizes and scan_dir, untouched since that call, and
 *                        with the same gla_set_option values in force as then               (read)
 *   fwd_workspace_bytes  its size, at least gla_fwd_workspace_bytes(...)
 *
 * Everything else as gla_bwd; `workspace` must be a different buffer.  The library cannot
 * check that the forward workspace belongs to these tensors: a stale one gives wrong dq.
 */
int gla_bwd_reuse(const void *q, const void *k, const void *v, const float *log_alpha, const void *d_out,
                  int B, int H, int T, int dk, int dv, int grid_h, int grid_w, int scan_dir, int qkv_dtype,
                  const void *fwd_workspace, size_t fwd_workspace_bytes,
                  float *dq, float *dk_grad, float *dv_grad, float *dlog_alpha,
                  void *workspace, size_t workspace_bytes, gla_stream_t stream);

/*
 * gla_bwd_layout - gla_bwd / gla_bwd_reuse for either memory order: the backward pass of
 * gla_fwd_layout with a zero initial state (Eq. (attn_gla) rows 1-3 differentiated).
 *
 *   layout           gla_layout of q, k, v, log_alpha, d_out and of the four gradients
 *   fwd_workspace    as in gla_bwd_reuse, or NULL to recompute the span states (then
 *                    fwd_workspace_bytes is ignored)
 *
 * Everything else as gla_bwd; GLA_ERR_SHAPE for an unknown layout.
 */
int gla_bwd_layout(const void *q, const void *k, const void *v, const float *log_alpha, const void *d_out,
                   int B, int H, int T, int dk, int dv, int grid_h, int grid_w, int scan_dir, int qkv_dtype,
                   int layout, const void *fwd_workspace, size_t fwd_workspace_bytes,
                   float *dq, float *dk_grad, float *dv_grad, float *dlog_alpha,
                   void *workspace, size_t workspace_bytes, gla_stream_t stream);

/*
 * gla_srem_dwconv - the 3x3 depth-wise convolution of the spatial reorient & enhancement
 * module (Sec. 3.3, Algorithm 1: DWConv2d on the 2-D token matrix; every channel has its own
 * 3x3 kernel, zero padding of one token, stride one; the paper initialises it to the identity).
 *   y[b, r, c, d] = bias[d] + sum over dy, dx in {-1,0,1} of weight[d, dy+1, dx+1] * x[b, r+dy, c+dx, d]
 * for orient = 0.  The paper permutes the token sequence between blocks; here tensors stay in
 * canonical row-major order and `orient` (a gla_scan_dir) names the order the paper's sequence
 * would be in, so that the result equals: permute, reshape to 2-D, convolve, flatten, un-permute.
 *
 *   x        DEVICE, x_dtype [B, grid_h*grid_w, D], 16-byte aligned                  (read)
 *   weight   DEVICE, fp32 [D, 3, 3]                                                  (read)
 *   bias     DEVICE, fp32 [D], or NULL                                               (read)
 *   y        DEVICE, y_dtype [B, grid_h*grid_w, D], 16-byte aligned, not x           (written)
 *
 * Status codes as gla_fwd_ex.  Needs no workspace and never allocates.
 */
int gla_srem_dwconv(const void *x, const float *weight, const float *bias, int B, int grid_h, int grid_w, int D,
                    int orient, int x_dtype, int y_dtype, void *y, gla_stream_t stream);

/*
 * gla_fwd_multi - multi-directional scanning (supplement, Algorithms 2 and 3): the sum over
 * several scan orders of the outputs of gla_fwd_ex on the same q, k, v, log_alpha, every
 * term in canonical token order:  out = sum over d in scan_mask of gla_fwd_ex(..., scan_dir = d).
 *
 *   scan_mask   bit d set (d = gla_scan_dir): scan order d takes part; 0x3 is the
 *               bidirectional variant, 0xF the 4-directional one; 1..15
 *   out         DEVICE, fp32 [B,H,T,dv]                                              (written)
 *
 * q, k, v, log_alpha, sizes, workspace (gla_fwd_workspace_bytes) and stream as gla_fwd_ex;
 * no final state is returned (each scan order ends in its own).  The scan orders run one
 * after the other on `stream`; the first writes `out`, the others add to it.  Same status
 * codes as gla_fwd_ex, GLA_ERR_SHAPE for a mask outside 1..15.  Never allocates.
 */
int gla_fwd_multi(const void *q, const void *k, const void *v, const float *log_alpha,
                  int B, int H, int T, int dk, int dv, int grid_h, int grid_w, unsigned scan_mask,
                  int qkv_dtype, float *out, void *workspace, size_t workspace_bytes, gla_stream_t stream);

/*
 * gla_fwd_fused - gla_fwd_ex with the gate computed from its pre-activation inside the kernels
 * and, optionally, the output gate and normalisation applied before the store:
 *   log alpha_t = logsigmoid(z_t) / tau                  (Eq. (gate_gla), alpha = sigmoid(z)^(1/tau))
 *   y_t = Swish(r_t) * LN(o_t),  Swish(x) = x sigmoid(x)  (Eq. (attn_gla) rows 4-5, up to the projection W_O)
 * LN takes mean and (biased) variance over the dv entries of one head's o_t, adds ln_eps
 * under the square root, and applies weight and bias rows of that head.
 *
 *   z_alpha     DEVICE, qkv_dtype [B,H,T,dk]: X W_alpha + b_alpha                         (read)
 *   tau         temperature, > 0 (the DiG configurations use 16)
 *   r_pre       DEVICE, qkv_dtype [B,H,T,dv]: X W_r + b_r, or NULL: no epilogue, `out`
 *               receives o_t as in gla_fwd_ex (the three ln_ arguments are then ignored)    (read)
 *   ln_weight, ln_bias   DEVICE, fp32 [H,dv], or NULL for all ones / all zeros            (read)
 *   ln_eps      >= 0
 *
 * Everything else as gla_fwd_ex ([B,H,T,d] order, zero initial state); same status codes,
 * GLA_ERR_SHAPE also for tau <= 0 or ln_eps < 0.  Never allocates.
 */
int gla_fwd_fused(const void *q, const void *k, const void *v, const void *z_alpha, float tau,
                  const void *r_pre, const float *ln_weight, const float *ln_bias, float ln_eps,
                  int B, int H, int T, int dk, int dv, int grid_h, int grid_w, int scan_dir,
                  int qkv_dtype, int out_dtype, void *out, float *final_state,
                  void *workspace, size_t workspace_bytes, gla_stream_t stream);

/*
 * gla_fwd_fused_gates - gla_fwd_fused with the value-side gate as well, also from its
 * pre-activation (Eq. (gate_gla_2): beta = sigmoid(z_beta)^(1/tau), same temperature):
 * the mixer of Sec. 3.1 from the projections' outputs to the input of W_O in one call.
 *
 *   z_beta      DEVICE, qkv_dtype [B,H,T,dv]: X W_beta + b_beta, 16-byte aligned          (read)
 *
 * Everything else as gla_fwd_fused; engines as gla_fwd_gates.  GLA_ERR_NULL for a NULL z_beta.
 */
int gla_fwd_fused_gates(const void *q, const void *k, const void *v, const void *z_alpha, const void *z_beta, float tau,
                        const void *r_pre, const float *ln_weight, const float *ln_bias, float ln_eps,
                        int B, int H, int T, int dk, int dv, int grid_h, int grid_w, int scan_dir,
                        int qkv_dtype, int out_dtype, void *out, float *final_state,
                        void *workspace, size_t workspace_bytes, gla_stream_t stream);

/* Bytes of workspace gla_fwd_ex / gla_fwd_layout need for this problem (an upper bound over all
 * launch plans, so it does not depend on tuning options).  0 on invalid sizes. */
size_t gla_fwd_workspace_bytes(int B, int H, int T, int dk, int dv, int qkv_dtype);

/*
 * gla_fwd_timed - measurement aid: runs gla_fwd_ex `iters` times on `stream`
 * with HIP events around each of the three phases of the chunk-parallel plan
 * (Sec. 3.5 cut into spans: local span states, carry across spans, outputs) and
 * returns mean milliseconds per call in phase_ms (HOST pointer to 4 floats:
 * span-state kernel, carry kernel, output kernel, whole call).  Synchronises
 * the stream before returning.  Phases a plan skips report 0.
 */
int gla_fwd_timed(const void *q, const void *k, const void *v, const float *log_alpha,
                  int B, int H, int T, int dk, int dv, int grid_h, int grid_w, int scan_dir,
                  int qkv_dtype, int out_dtype, void *out, float *final_state,
                  void *workspace, size_t workspace_bytes, gla_stream_t stream,
                  int iters, float *phase_ms);

/*
 * gla_calibrate_mfma - measurement aid: the rate at which this GPU retires v_mfma_f32_16x16x32_bf16 when nothing
 * else limits it (every wave of a grid that fills the chip runs a loop of eight independent accumulator chains
 * held in registers, no memory traffic), in TFLOP/s (2 flops per multiply-add), written to *tflops (HOST pointer).
 * It is the figure to hold next to the published dense bf16 peak when a kernel's MFMA rate is priced.  Runs on
 * `stream`, synchronises it before returning, allocates 4 KiB of device memory for the duration of the call.
 * GLA_ERR_NULL for a NULL pointer, GLA_ERR_HIP if a runtime call fails.
 */
int gla_calibrate_mfma(double *tflops, gla_stream_t stream);

/* Process-wide tuning knobs; returns GLA_ERR_SHAPE for an unknown option or value.  They are plain process
 * globals read at the start of every call: set them before, not while, other threads call the library. */
int gla_set_option(int option, int value);
int gla_get_option(int option);

/*
 * gla_block_scan_dir - the scan order that DiG block `block` uses (Sec. 3.3, Algorithm 1: after every block the
 * token matrix is transposed, for even block indices, or the sequence flipped, for odd ones; supplement,
 * Algorithm 4 states the same schedule with the parities swapped).  This library leaves the tokens in canonical
 * row-major order and folds those permutations into `scan_dir` of the gla_fwd* / gla_bwd* calls and `orient` of
 * gla_srem_dwconv; this function names the order a block sees:
 *   GLA_SCHEDULE_BLOCK_PROCESS (Algorithm 1):  block 1, 2, 3, 4, 5 ... -> ROW_FWD, ROW_REV, COL_REV, COL_FWD, ROW_FWD ...
 *   GLA_SCHEDULE_BLOCK_SCAN    (Algorithm 4):  block 1, 2, 3, 4, 5 ... -> ROW_FWD, COL_FWD, COL_REV, ROW_REV, ROW_FWD ...
 * (the paper's reshape2d takes a square token matrix; on a grid_h x grid_w grid the orders are those of
 * gla_scan_dir on that grid).  Host only, no GPU work.
 *
 *   block      1-based index of the block (the paper's l)
 *   schedule   a gla_schedule
 * Returns the gla_scan_dir, or -1 for block < 1 or an unknown schedule.
 */
typedef enum { GLA_SCHEDULE_BLOCK_PROCESS = 0, GLA_SCHEDULE_BLOCK_SCAN = 1 } gla_schedule;
int gla_block_scan_dir(int block, int schedule);

/* Static, NUL-terminated description of a status code. */
const char *gla_status_string(int status);

/* Library version: major * 10000 + minor * 100 + patch. */
int gla_version(void);

#ifdef __cplusplus
}
#endif
#endif /* GLA_H_ */
