/*
 * canvas_dag.h -- C ABI of the micro-DAG executor for AMD MI355X (gfx950).
 *
 * A micro-DAG is a kernel built from the fine-grained primitives of
 * "Canvas: End-to-End Kernel Architecture Search" (Section 5, table of
 * primitives): rearrangement (Group, Shift, Unfold), arithmetic
 * (Fully-connected, element-wise, Folding, Softmax) and blending (Broadcast).
 * This library compiles a serialized micro-DAG for a concrete input shape and
 * runs it forward and backward on NCHW feature maps on one GPU.
 *
 * Serialized form ("blob"): UTF-8 text, one node per line, topological order,
 * ids consecutive from 1, %0 is the input [N, C, H, W]:
 *
 *     canvas-dag 1
 *     %1 = unfold %0 kh=3 kw=3
 *     %2 = fc %1 groups=8 out=64
 *     %3 = unary %2 op=gelu            relu | abs | gelu | sin | expclip lo=<f> hi=<f>
 *     %4 = shift %3 dh=0 dw=1 c0=32 c1=64
 *     %5 = binary %0 %4 op=mul         first operand LHS, second RHS; add | sub | mul | min | max [lhs=pixels]
 *     %6 = fold %5 op=avg              sum | avg | max [axis=T | H | W | HW | C [groups=<G>]]
 *     %7 = softmax %6 axis=C           C | T | CT | H | W | HW
 *     %8 = group %7 groups=4           a view [G, C/G] of the channels; groups=C: every channel a group
 *     output %8
 *
 * Tensors are [N, C, T, H, W], contiguous, T = number of unfolded taps (1 when
 * the tensor has none; then the layout is plain NCHW).
 *
 *   unfold   U(n,c,t,h,w) = I(n,c,t_in,h+kh-KH/2,w+kw-KW/2), t = t_in*KH*KW + kh*KW + kw,
 *            zero outside the image (Section 5: U(c,kh,kw,h,w) = I(c,h+kh,w+kw)).
 *   shift    S(n,c,t,h,w) = I(n,c,t,h+dh,w+dw) for c in [c0,c1), zero outside;
 *            other channels pass through (Section 5: U(c,h,w) = I(c,h+1,w)).
 *   fc       y(n,g*Og+o,h,w) = sum_{c'<C/G, t<T} W[g][o][c'*T+t] * x(n,g*(C/G)+c',t,h,w);
 *            contracts channels of a group and all taps, keeps groups apart, no
 *            bias (Section 5, Fully-connected; group rearrangement g*GROUP_SIZE+c).
 *   unary    relu, abs, gelu (erf form), sin, exp(clamp(x,lo,hi)) (Section 5, element-wise).
 *   binary   out = op(tile(LHS), RHS), shape of RHS (Section 5, Broadcast): with
 *            dims [C,T] of both sides, equal C is a common prefix (lhs c = c,
 *            lhs t = t mod T_L); otherwise the LHS is replicated along the
 *            flattened (c*T_R + t) index modulo C_L*T_L.  The LHS size must
 *            divide the RHS size.  op: add, sub (tile(LHS) - RHS), mul, min, max.
 *            With lhs=pixels a pooled LHS of exactly H*W elements is laid over the
 *            pixels instead: out(c,t,h,w) = op(LHS(h*W+w), RHS(c,t,h,w)) (Section 8,
 *            the kernel that pools to [C], maps to H x W with an FC and multiplies x).
 *   softmax  along C (per n,t,h,w), along T (per n,c,h,w) or along both jointly
 *            (axis=CT, per n,h,w); along H (per n,c,t,w), along W (per n,c,t,h) or
 *            over both jointly (axis=HW, per n,c,t) (Section 5, Softmax at any
 *            continuous dims).
 *   fold     sum, avg or max over T; T disappears (Section 5, Folding).  Max
 *            sends its gradient to the first maximal tap.  With axis=HW the
 *            pixels are folded instead (global pooling), with axis=H or axis=W
 *            one spatial dim: the result is [N, C, T, 1, 1], [N, C, T, 1, W] or
 *            [N, C, T, H, 1] (first maximum in the order h, then w); fc, unary,
 *            softmax, the remaining folds and binary accept such a tensor
 *            (unfold and shift do not), and as the LHS of a binary it is
 *            replicated along the dims it has folded onto an RHS that still has
 *            them (an RHS may not have folded a dim that the LHS keeps).  With
 *            axis=C groups=G (default 1) the C/G channels of each of G channel
 *            groups are folded: G channels remain.
 *   group    the Group primitive as a node (Section 5, Group: [.., X, ..] => [.., G, X/G, ..]
 *            or [.., X, 1, ..]): the same data, seen as G channel groups.  The view
 *            travels through unfold, shift, unary, softmax and fold over T / HW; an
 *            fc of a grouped tensor contracts inside each group (its groups= may be
 *            left out, and must equal G when given) and its output keeps the view;
 *            a binary result has the view of its RHS; when both operands of a binary
 *            carry the same view, G is a common leading dim and the Broadcast rule
 *            applies inside each group to [C_L/G, T_L] and [C_R/G, T_R] (Section 5:
 *            [G, x/G, H, W] onto [G, C/G, K_H, H, W]).  fold axis=C drops the view.
 *            An fc without groups= on a tensor without a view has one group.
 *   backward exact vector-Jacobian products of the above; relu'(0) = 0,
 *            sign(0) = 0, expclip has zero gradient outside the open interval; a
 *            tie of binary min / max sends the gradient to the LHS.
 *
 * Threading: a canvas_dag handle may be used by one thread at a time.  All
 * functions return CANVAS_OK (0) or a negative canvas_status; they never throw
 * and never launch work after detecting an error.  canvas_last_error() gives a
 * thread-local message for the last failure.
 */
#ifndef CANVAS_DAG_H
#define CANVAS_DAG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CANVAS_MAX_NODES 64

typedef struct canvas_dag canvas_dag; /* opaque, owned by the library */

typedef enum { CANVAS_F32 = 0, CANVAS_BF16 = 1 } canvas_dtype;

typedef enum {
    CANVAS_OK = 0,
    CANVAS_INVALID_BLOB = -1,       /* syntax error */
    CANVAS_UNKNOWN_OP = -2,
    CANVAS_SHAPE_MISMATCH = -3,     /* groups do not divide, LHS size does not divide RHS size, ... */
    CANVAS_BAD_ARG = -4,            /* null or misaligned pointer, bad enum, bad shape */
    CANVAS_WORKSPACE_TOO_SMALL = -5,
    CANVAS_UNSUPPORTED = -6,
    CANVAS_HIP_ERROR = -7
} canvas_status;

/* Option flags for canvas_dag_compile. */
#define CANVAS_OPT_NO_FUSION 1u /* one kernel per node, fp32 intermediates (reference lowering) */
#define CANVAS_OPT_INFERENCE 2u /* forward-only plan: no backward, weight repacking / widening taken out of
                                   canvas_dag_forward into canvas_dag_prepare (run once per set of weights) */

typedef struct canvas_options {
    uint32_t flags;
    uint32_t reserved[7]; /* must be zero */
} canvas_options;

typedef struct canvas_dag_info {
    int32_t n_nodes;                          /* including node 0, the input */
    int32_t out_node;
    int32_t n_weights;                        /* number of fc nodes */
    int32_t n_launches_fwd, n_launches_bwd;   /* kernels enqueued per call */
    int32_t fused;                            /* 1 when one of the whole-DAG kernel families was chosen, else 0 (lowering by units) */
    int32_t n_launches_prepare;               /* inference plans: kernels canvas_dag_prepare enqueues, else 0 */
    int32_t n_fused_chains;                   /* lowering by units: chains of memory-bound nodes fused into one kernel each */
    int64_t out_shape[5];                     /* N, C, T, H, W */
    int64_t node_shape[CANVAS_MAX_NODES][5];  /* N, C, T, H, W per node */
    int64_t weight_shape[CANVAS_MAX_NODES][3];/* G, C_out/G, (C_in/G)*T per fc node, in node order */
    int32_t weight_node[CANVAS_MAX_NODES];    /* node id of each weight */
    uint64_t workspace_bytes;                 /* device bytes forward/backward need */
    double fc_flops_fwd;                      /* 2*M*C_out*(C_in/G)*T summed over fc nodes (block-diagonal only) */
    double min_bytes_fwd;                     /* x read + y written + weights read, once each */
    double min_bytes_bwd;                     /* x, dy read + dx written + weights read + dW written */
    int32_t n_fused_nodes;                    /* nodes inside those chains (none of them is materialised unless a later unit reads it) */
    int32_t reserved1;
} canvas_dag_info;

typedef struct canvas_launch_desc {
    char name[64];      /* kernel family */
    double bytes;       /* algorithmic bytes this launch must move (each operand once) */
    double flops;       /* algorithmic flops (FC contractions only) */
} canvas_launch_desc;

/* Parse, infer shapes, check legality and plan the lowering.  Host only: needs
 * no GPU.  blob: host pointer, blob_len bytes, not retained.  in_shape: host
 * pointer to N, C, H, W (all >= 1).  dt: element type of x, weights, y, dy, dx
 * (weight gradients are always fp32).  opt: host pointer or NULL.  *out: new
 * handle, released with canvas_dag_destroy.  Errors: INVALID_BLOB, UNKNOWN_OP,
 * SHAPE_MISMATCH, BAD_ARG, UNSUPPORTED (more than CANVAS_MAX_NODES nodes). */
int canvas_dag_compile(const void* blob, size_t blob_len, const int64_t in_shape[4], canvas_dtype dt,
                       const canvas_options* opt, canvas_dag** out);

/* Fill *info (host pointer).  Host only. */
int canvas_dag_query(const canvas_dag* dag, canvas_dag_info* info);

/* Describe launch idx of the forward (backward = 0) or backward (= 1) plan. */
int canvas_dag_launch_desc(const canvas_dag* dag, int backward, int idx, canvas_launch_desc* out);

/* Enqueue the forward pass on `stream` (a hipStream_t, or NULL for the default
 * stream).  Device pointers, owned by the caller, 16-byte aligned, contiguous:
 *   x        [N, C, H, W]           dtype dt, read
 *   weights  host array of n_weights device pointers, each [G, C_out/G, (C_in/G)*T] dtype dt, read
 *   y        [N, C_out, T_out, H, W] dtype dt, written
 *   workspace  workspace_bytes bytes; carries what backward needs, so it must stay
 *            untouched until the matching canvas_dag_backward has run
 * Does not allocate, free or synchronise.  Errors: BAD_ARG,
 * WORKSPACE_TOO_SMALL, HIP_ERROR (launch failure). */
int canvas_dag_forward(canvas_dag* dag, const void* x, const void* const* weights, void* y, void* workspace,
                       size_t workspace_bytes, void* stream);

/* canvas_dag_forward for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): the same kernels, with the workspace taken from a
 * static device array of CANVAS_STATIC_WORKSPACE_BYTES that is part of the library (every GPU the library
 * runs on holds one copy until the process ends).  Calls no hipMalloc / hipFree and no allocating library
 * routine.  x, weights, y, stream as canvas_dag_forward.  An inference plan runs its weight-only launches
 * with every call (nothing is kept in the static workspace between calls), so canvas_dag_prepare is not
 * needed; no canvas_dag_backward can follow, since that reads the workspace of its forward call.
 * All calls on one GPU, of any plan, share the one array: calls that overlap on a GPU (different streams
 * or host threads) race; calls enqueued on one stream are ordered and safe.
 * Errors: WORKSPACE_TOO_SMALL when the plan's workspace_bytes exceeds CANVAS_STATIC_WORKSPACE_BYTES
 * (nothing is launched), BAD_ARG, HIP_ERROR. */
#define CANVAS_STATIC_WORKSPACE_BYTES (64u << 20)
int canvas_dag_forward_static(canvas_dag* dag, const void* x, const void* const* weights, void* y, void* stream);

/* Inference plans (CANVAS_OPT_INFERENCE) only: enqueue the weight-only work of the forward pass
 * (repacking into MFMA operand order, widening) on `stream`; its results live in the workspace, so
 * call it once before the first canvas_dag_forward on that workspace and again whenever the weights
 * change.  A no-op for plans that have no such work.  Errors: BAD_ARG (also: not an inference plan),
 * WORKSPACE_TOO_SMALL, HIP_ERROR.  Callers: serving loops at batch 1-8 where the per-call repacking
 * launches would dominate the latency. */
int canvas_dag_prepare(canvas_dag* dag, const void* const* weights, void* workspace, size_t workspace_bytes, void* stream);

/* Enqueue the backward pass of the preceding canvas_dag_forward on the same
 * x, weights and workspace.
 *   dy       like y, dtype dt, read
 *   dx       like x, dtype dt, written
 *   dweights host array of n_weights device pointers, fp32, shaped like the weights, overwritten
 * Deterministic: no floating-point atomics, two runs give identical bits.
 * Errors as canvas_dag_forward; UNSUPPORTED for an inference plan. */
int canvas_dag_backward(canvas_dag* dag, const void* x, const void* const* weights, const void* dy, void* dx,
                        void* const* dweights, void* workspace, size_t workspace_bytes, void* stream);

/* Benchmark aid.  enable != 0: every kernel launch of later forward/backward calls carries a start and
 * a stop HIP event on the caller's stream (events are created here, not in the hot path), so that
 * canvas_dag_get_timing reports each kernel's own execution time.  enable == 0:
 * events are destroyed.  Needs a GPU.  Errors: BAD_ARG, HIP_ERROR. */
int canvas_dag_set_timing(canvas_dag* dag, int enable);

/* Waits for the last timed forward (backward = 0) or backward (= 1) call and writes the duration of
 * each of its n launches, in milliseconds, to ms (host pointer, n = n_launches_fwd or _bwd).
 * Errors: BAD_ARG (timing not enabled, no call yet, wrong n), HIP_ERROR. */
int canvas_dag_get_timing(canvas_dag* dag, int backward, float* ms, int n);

void canvas_dag_destroy(canvas_dag* dag);

/* Message of the last error on this thread ("" when none).  Host pointer owned by the library. */
const char* canvas_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* CANVAS_DAG_H */
