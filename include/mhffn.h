/*
 * mhffn.h -- C ABI of the MI355X (gfx950) fused Multi-Head FFN library.
 *
 * The operation is the gated Multi-Head FFN of FlashMHF: tokens are split into
 * H heads of width d_h (paper, Preliminary, "Headwise Operation Functions");
 * every head owns E SwiGLU sub-networks of width d_e (Methodology, "Parallel
 * FFN Sub-Networks"); their outputs are mixed with per-token weights
 * R = sigmoid(P) / (sum_e sigmoid(P) + eps), P = q W^h (eq:routing) and the
 * heads are concatenated again:
 *
 *   Y[l, h*d_h + j] = sum_e R[l,h,e] * sum_c SiLU(q.K[h,e,c,:]) * (q.U[h,e,c,:]) * V[h,e,c,j]
 *   with q = X[l, h*d_h : (h+1)*d_h]               (eq:intuitive-ffn, aggregation eq.)
 *
 * The fused entry points evaluate the sum over the intermediate index (e,c)
 * block by block on chip (eq:flash-ffn-loop), so the [N, H, E*d_e] activation
 * never reaches device memory; the backward recomputes it (appendix algorithms
 * "Backward (dQ,dR)" and "Backward (dK,dU,dV)").
 *
 * Conventions for every entry point
 *  - All tensor pointers are DEVICE pointers, 16-byte aligned, owned by the
 *    caller.  `desc` is a HOST pointer.  `hip_stream` is a hipStream_t passed
 *    as void* (NULL = the default stream).
 *  - The library never allocates or frees device memory, never synchronises
 *    and keeps no data between calls: all work is enqueued on `hip_stream`,
 *    which must belong to the calling thread's current device, and the call
 *    returns immediately.  Calls may come from several threads and for
 *    several devices.  Scratch comes from the caller through `workspace` (at
 *    least mhffn_workspace_bytes() bytes, 256-byte aligned; may be NULL when
 *    that size is 0).
 *  - The only host-side state is, per kernel and device, the fact that the
 *    kernel's dynamic-LDS limit has been raised (a function attribute).
 *    mhffn_init() does this for every kernel on the current device; without
 *    it the first launch of each kernel on a device does it, and that first
 *    launch must then happen outside stream capture.
 *  - Outputs are overwritten, never accumulated into.
 *  - Errors are reported by return code only; every argument is validated on
 *    the host before anything is launched, so a non-zero return means nothing
 *    was enqueued (except MHFFN_ERR_LAUNCH, which reports a HIP launch error).
 *
 * Layouts (row-major, innermost index last)
 *   X, Y, dX, dY : [n_tokens][ld]            head h = columns h*d_h .. (h+1)*d_h-1
 *   W_gate (paper K), W_up (U), W_down (V) and their gradients:
 *                  [n_heads][n_sub][d_sub][d_head]   (one row per intermediate neuron)
 *   route, MHFFN_ROUTE_PARAMS : W_r [n_heads][d_head][n_sub], dtype = desc.dtype
 *   route, MHFFN_ROUTE_WEIGHTS: R   [n_tokens][n_heads][n_sub], always fp32
 *   d_route has the shape and dtype of `route` for the mode in use.
 */
#ifndef MHFFN_H
#define MHFFN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MHFFN_OK = 0,
  MHFFN_ERR_NULL = 1,        /* a required pointer is NULL                       */
  MHFFN_ERR_SHAPE = 2,       /* a size is non-positive or a stride is too small  */
  MHFFN_ERR_UNSUPPORTED = 3, /* valid problem, but no kernel for it (see below)  */
  MHFFN_ERR_ALIGN = 4,       /* a pointer or stride breaks the alignment rule    */
  MHFFN_ERR_WORKSPACE = 5,   /* workspace NULL or smaller than required          */
  MHFFN_ERR_LAUNCH = 6,      /* HIP reported an error when launching             */
  MHFFN_ERR_STATIC_SCRATCH = 7 /* mhffn_forward_static: the problem needs more scratch
                                  than MHFFN_STATIC_SCRATCH_BYTES                  */
} mhffn_status;

typedef enum {
  MHFFN_F32 = 0, /* fp32 storage, fp32 arithmetic                         */
  MHFFN_BF16 = 1 /* bf16 storage, bf16 MFMA with fp32 accumulation        */
} mhffn_dtype;

typedef enum {
  MHFFN_ROUTE_PARAMS = 0, /* route = W_r; R is computed in-kernel (eq:routing)          */
  MHFFN_ROUTE_WEIGHTS = 1 /* route = R, used as given (the paper's kernel-level input)  */
} mhffn_route_mode;

typedef enum {
  MHFFN_OP_FORWARD = 0,
  MHFFN_OP_BACKWARD = 1,
  MHFFN_OP_UNFUSED_FORWARD = 2,
  MHFFN_OP_UNFUSED_BACKWARD = 3, /* mhffn_reference_unfused with dY != NULL */
  MHFFN_OP_MODULE_FORWARD = 4,
  MHFFN_OP_MODULE_BACKWARD = 5
} mhffn_op;

typedef struct {
  int64_t n_tokens;  /* N = batch * sequence; any N >= 0, ragged tails are masked    */
  int32_t n_heads;   /* H                                                            */
  int32_t d_head;    /* d_h; d_model = H*d_h                                         */
  int32_t n_sub;     /* E, sub-networks per head                                     */
  int32_t d_sub;     /* d_e, width of one sub-network; d_ff = E*d_e                  */
  int64_t ld_x;      /* row stride of X and dX in elements (>= H*d_h); 0 => H*d_h    */
  int64_t ld_y;      /* row stride of Y and dY in elements (>= H*d_h); 0 => H*d_h    */
  int32_t dtype;     /* mhffn_dtype of X, Y, weights, W_r and all their gradients    */
  int32_t route_mode;/* mhffn_route_mode                                             */
  float eps;         /* epsilon of eq:routing (the paper gives no value)             */
} mhffn_desc;

/*
 * Shape support.
 *   bf16: the fused kernels need d_head in {64, 128, 256}, d_sub % 32 == 0 and
 *         n_sub <= 96 (backward with d_head = 256: n_sub <= 64); other shapes
 *         return MHFFN_ERR_UNSUPPORTED.
 *   fp32: the fused kernels take d_head % 4 == 0 up to 256, any n_sub, d_sub, as long as
 *         their LDS tiles fit.  The backward keeps whole d_head-wide token and weight tiles
 *         and two n_sub-wide rows per token resident: d_head = 256 with up to about 170
 *         sub-networks, d_head = 128 with several hundred.
 *   mhffn_reference_unfused takes any shape with d_head % 8 == 0.
 *   Row strides must keep every row 16-byte aligned.
 */

/* Bytes of caller-provided scratch needed by `op` (an mhffn_op) for `desc`.
 * Returns 0 for an invalid descriptor as well; validate with the entry point.
 * For MHFFN_OP_FORWARD this is 0 whenever the token tiles alone give the chip
 * enough workgroups (d_head = 128 with up to 64 sub-networks: more than 128
 * tiles of 256 tokens x heads, i.e. ceil(n_tokens / 256) * n_heads > 128; the
 * other kernels: at least 384 tiles): the fused forward then touches nothing
 * but its inputs and Y, which is the "intermediate never reaches HBM" property
 * of eq:flash-ffn-loop stated as a number.  For fewer tokens (decode, short
 * prefill) the blocks of eq:flash-ffn-loop are shared out over several
 * workgroups per token tile and their fp32 partial outputs, n_split * N *
 * d_model * 4 bytes (a few output-sized buffers, never d_ff-sized ones), pass
 * through the workspace; ask this function rather than relying on the rule.  For MHFFN_OP_BACKWARD it is the gating weights R and
 * their gradient as [H][E][N] fp32, the partial sums of dW_r, and, for the
 * neuron groups that would otherwise leave CUs idle in the last round of
 * workgroups, fp32 partial weight gradients of a few token segments (a multiple
 * of the parameter count, not of the token count; all summed in a fixed order:
 * results are bit-identical from run to run).  For the unfused ops it is the three
 * materialised [N][H][d_ff] activations plus the [N][H][E] weights, i.e. the
 * O((L*H + d_model)*d_ff) footprint of the naive multi-head FFN. */
size_t mhffn_workspace_bytes(const mhffn_desc* desc, int op);

/* Fused forward (appendix algorithm "SRAMFFN-Forward"; gating of eq:routing is
 * evaluated in the same kernel in MHFFN_ROUTE_PARAMS mode).  Writes Y. */
int mhffn_forward(const mhffn_desc* desc, const void* X, const void* W_gate,
                  const void* W_up, const void* W_down, const void* route,
                  void* Y, void* workspace, size_t workspace_bytes,
                  void* hip_stream);

/* mhffn_forward for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops (decode steps),
 * harnesses that forbid hipMalloc.  Same arguments, kernels and results as
 * mhffn_forward, but the scratch that small token counts need (the fp32
 * partial outputs, see mhffn_workspace_bytes) lies in a device buffer of
 * MHFFN_STATIC_SCRATCH_BYTES that is part of the library's code object: every
 * GPU the library runs on holds one copy until the process ends, and the call
 * allocates nothing (its address on the current device is looked up at the first
 * use there, or by mhffn_init).  A problem whose mhffn_workspace_bytes exceeds
 * that size returns MHFFN_ERR_STATIC_SCRATCH and launches nothing (d_head = 128
 * with up to 64 sub-networks never needs more than 32 MiB, whatever the token
 * count; the kernels of the other shapes can need up to 64 MiB at a few hundred
 * to a few thousand tokens and are then refused).  All calls on one GPU share the buffer: it keeps the last call's
 * partial sums (each call overwrites what it reads, nothing has to start at
 * zero), and two calls that overlap in time on one GPU (different streams) race
 * on it -- serialise them, or use mhffn_forward with workspaces of their own. */
#define MHFFN_STATIC_SCRATCH_BYTES (40u << 20)
int mhffn_forward_static(const mhffn_desc* desc, const void* X, const void* W_gate,
                         const void* W_up, const void* W_down, const void* route,
                         void* Y, void* hip_stream);

/* Fused, recompute-based backward (appendix algorithms "Backward (dQ,dR)" and
 * "Backward (dK,dU,dV)"; the derivative through eq:routing is taken here too).
 * Needs only X, the weights and dY: nothing is saved by the forward.
 * Any of dX, dW_gate, dW_up, dW_down, d_route may be NULL => not computed.
 * d_route is dW_r (PARAMS mode) or dR (WEIGHTS mode). */
int mhffn_backward(const mhffn_desc* desc, const void* X, const void* W_gate,
                   const void* W_up, const void* W_down, const void* route,
                   const void* dY, void* dX, void* dW_gate, void* dW_up,
                   void* dW_down, void* d_route, void* workspace,
                   size_t workspace_bytes, void* hip_stream);

/* mhffn_backward with timing marks, for profiling the phases of the fused
 * backward on the caller's stream without a tracing tool.  The phases are, in
 * launch order (appendix algorithms "Backward (dQ,dR)" and "Backward
 * (dK,dU,dV)"): 0 token-major kernel (dX, R, dp), 1 weight-major kernel
 * (dW_gate, dW_up, dW_down), 2 gating-parameter gradient (dW_r).
 * `phase_events` is a HOST array of `n_phase_events` hipEvent_t handles owned
 * by the caller (entries may be NULL = skipped): event 0 is recorded on
 * `hip_stream` before the first launch, event i after phase i-1; at most 4 are
 * used.  Everything else is exactly mhffn_backward. */
int mhffn_backward_phases(const mhffn_desc* desc, const void* X, const void* W_gate,
                          const void* W_up, const void* W_down, const void* route,
                          const void* dY, void* dX, void* dW_gate, void* dW_up,
                          void* dW_down, void* d_route, void* workspace,
                          size_t workspace_bytes, void* hip_stream,
                          void* const* phase_events, int n_phase_events);

/* Unfused GPU baseline: the naive execution of the same layer (Methodology,
 * "Naive Multi-Head FFN", Limitations: memory pressure).  Separate kernels with
 * a device-memory round trip between them: (i) R, (ii) per-head products
 * G = X_h K^T and U' = X_h U^T, (iii) A = SiLU(G)*U'*R, (iv) Y_h = A_h V;
 * G, U' and A are materialised in `workspace`.  With dY != NULL it also runs
 * the backward from those saved activations and writes the non-NULL
 * gradients.  With dY == NULL the gradient pointers are ignored. */
int mhffn_reference_unfused(const mhffn_desc* desc, const void* X,
                            const void* W_gate, const void* W_up,
                            const void* W_down, const void* route, void* Y,
                            const void* dY, void* dX, void* dW_gate,
                            void* dW_up, void* dW_down, void* d_route,
                            void* workspace, size_t workspace_bytes,
                            void* hip_stream);

/* The whole module around the fused path (Methodology: per-head inputs
 * Q = split_H(X W_in), output O = concat_H(S) W_out, both projections d_model x
 * d_model, no bias):
 *     Q = X W_in;   S = mhffn_forward(Q);   O = S W_out.
 * W_in, W_out: [d_model][d_model] row-major, applied from the right (row i = input
 * feature i), dtype = desc.dtype.  desc.ld_x / ld_y are the row strides of X and O;
 * desc.route_mode must be MHFFN_ROUTE_PARAMS.  Q and S are outputs too, dense
 * [n_tokens][d_model], required: they are what a training step keeps for
 * mhffn_module_backward (two d_model-wide activations; nothing d_ff-wide exists).
 * Shape support is that of mhffn_forward. */
int mhffn_module_forward(const mhffn_desc* desc, const void* X, const void* W_in,
                         const void* W_gate, const void* W_up, const void* W_down,
                         const void* W_r, const void* W_out, void* O, void* Q, void* S,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/* Backward of mhffn_module_forward from X, the weights, the saved Q and S, and dO:
 *     dS = dO W_out^T;  dW_out = S^T dO;  (dQ, dW_gate, dW_up, dW_down, dW_r) =
 *     mhffn_backward(Q, dS);  dW_in = X^T dQ;  dX = dQ W_in^T.
 * Any gradient pointer may be NULL => not computed.  dS and dQ pass through the
 * workspace (MHFFN_OP_MODULE_BACKWARD: two [n_tokens][d_model] buffers plus the
 * fused backward's own scratch): it begins with dS, then dQ, each dense
 * [n_tokens][d_model] in desc.dtype and rounded up to a multiple of 256 bytes; both
 * hold their values when the call has finished (dQ only if dX or dW_in was asked
 * for).  Shape support is that of mhffn_backward. */
int mhffn_module_backward(const mhffn_desc* desc, const void* X, const void* W_in,
                          const void* W_gate, const void* W_up, const void* W_down,
                          const void* W_r, const void* W_out, const void* Q, const void* S,
                          const void* dO, void* dX, void* dW_in, void* dW_gate, void* dW_up,
                          void* dW_down, void* dW_r, void* dW_out, void* workspace,
                          size_t workspace_bytes, void* hip_stream);

/* Optional set-up for the calling thread's current device: raises the
 * dynamic-LDS limit of every kernel of the library there, so that no later call
 * on that device changes a kernel attribute (first calls may then be recorded
 * into a HIP graph).  Idempotent, thread-safe, enqueues nothing.  Returns
 * MHFFN_OK, or MHFFN_ERR_LAUNCH if HIP refused an attribute. */
int mhffn_init(void);

/* Static, human-readable name of a status code. */
const char* mhffn_status_string(int status);

/* Library version string (static storage). */
const char* mhffn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MHFFN_H */
