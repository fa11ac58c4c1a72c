/*
 * msla.h -- C ABI of the MI355X (gfx950) multi-scale linear attention library.
 *
 * The library computes the multi-scale linear attention (MSLA) module of
 * EfficientViT (paper Section 3.1, Fig. 2 right):
 *
 *   x --1x1 projection--> Q/K/V token maps                     (Section 3.1, Eq. (1): Q = x W_Q ...)
 *     --per aggregated scale: depthwise k x k conv + grouped 1x1 conv
 *       (3*heads groups of d channels) --> multi-scale Q/K/V    (Section 3.1, last paragraph)
 *     --per branch, per head: ReLU linear attention             (Eqs. (2), (3))
 *         KV   = sum_n relu(K_n)^T [V_n, 1]            (d x (d+1), once per image/branch/head)
 *         att_n = relu(Q_n) KV[:, :d] / (relu(Q_n) KV[:, d] + eps)
 *     --concatenate branches and heads, 1x1 projection--> out   (Section 3.1, last sentence)
 *
 * General rules for every entry point
 *   - All data pointers are DEVICE pointers (HBM), 16-byte aligned, row-major,
 *     in the storage dtype `dt`; every sum is accumulated in fp32.  `scales`
 *     is a HOST pointer.  `stream` is a hipStream_t passed as void*.
 *   - The caller owns every buffer, including `workspace` (size it with
 *     msla_workspace_bytes).  The library allocates and frees nothing and is
 *     re-entrant as long as concurrent calls use different workspaces and
 *     outputs.  The only state it keeps between calls are per-process caches
 *     of device properties (the compute-unit count of the first device used;
 *     per kernel and device, that its LDS limit has been raised), which do not
 *     depend on any call's arguments.
 *   - Work is enqueued on `stream`; the call returns without synchronising.
 *     Buffers must stay alive and unmodified until the stream has passed it.
 *     Outputs must not alias inputs or the workspace.
 *   - All validation happens on the host before the first launch: a call that
 *     returns MSLA_ERR_INVALID_ARG, _UNSUPPORTED or _WORKSPACE has enqueued
 *     nothing.  No exception, abort or exit crosses this boundary.
 *
 * Shapes.  T = B*H*W tokens, Ct = heads*head_dim, A = n_scales aggregated
 * scales, S = 1 + A branches (branch 0 is the raw Q/K/V map and is always
 * present; branch a+1 is aggregated with a scales[a] x scales[a] kernel; every
 * aggregated branch reads the raw map).
 *   x      [B, H, W, C]            (MSLA_NHWC: a token is one row of C channels), or
 *          [B, C, H, W]            (MSLA_NCHW; turned into the token-major form by a
 *                                  transposition pass of its own before the module runs)
 *   w_qkv  [3*Ct, C]               row o = (h*3 + t)*head_dim + e, t = 0:Q 1:K 2:V,
 *                                  so each (head, Q/K/V) pair is one contiguous group
 *                                  of head_dim channels (the 3*heads groups of Section 3.1)
 *   qkv    [B, H, W, 3*Ct]         same channel order as the rows of w_qkv
 *   w_dw   concat over a of [3*Ct, k_a, k_a]   depthwise filters; stride 1, zero padding
 *                                  (k_a-1)/2, cross-correlation (tap (u,v) reads token
 *                                  (y+u-p, x+v-p))
 *   w_gpw  [A, 3*Ct, head_dim]     grouped 1x1: out channel o, input e of o's own group
 *   w_proj [C, S*Ct]               column m = (s*heads + h)*head_dim + f
 *   att    [B, H, W, S*Ct]         column order as w_proj's columns
 *   out    [B, H, W, C] or [B, C, H, W], as x
 * No bias, normalisation or activation other than the ReLUs of Eq. (2).
 *
 * Supported: head_dim == 16; scales[a] in {3, 5, 7}; n_scales <= 7;
 * C and Ct multiples of 16; with MSLA_NCHW also C <= 2*Ct.  msla_forward (and the
 * workspace query) also take head_dim 8 and 32 (no options).  Heads of 8 run in pairs
 * on the head_dim-16 kernels (the call first writes the weights in that arrangement into
 * the workspace); heads of 32 (with MSLA_NCHW: C <= 3*Ct) have an aggregation kernel of their
 * own for fp16 / bf16 and a plain vector-ALU one for fp32.  Anything else that is
 * otherwise well-formed returns MSLA_ERR_UNSUPPORTED.
 */
#ifndef MSLA_H_
#define MSLA_H_

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MSLA_OK = 0,
    MSLA_ERR_INVALID_ARG = -1,  /* null pointer, non-positive size, even kernel size, eps < 0, bad enum, misaligned pointer */
    MSLA_ERR_UNSUPPORTED = -2,  /* well-formed but outside what the kernels cover (see above) */
    MSLA_ERR_WORKSPACE = -3,    /* workspace_bytes smaller than msla_workspace_bytes reports */
    MSLA_ERR_LAUNCH = -4        /* the HIP runtime reported an error while enqueueing */
} msla_status;

typedef enum { MSLA_F32 = 0, MSLA_F16 = 1, MSLA_BF16 = 2 } msla_dtype;   /* storage type; sums are fp32 */
typedef enum { MSLA_NHWC = 0, MSLA_NCHW = 1 } msla_layout;               /* of x and out */
typedef enum { MSLA_ACT_RELU = 0, MSLA_ACT_HSWISH = 1 } msla_act;        /* hard-swish: a * clip(a + 3, 0, 6) / 6 */

/* Human-readable name of a status code (static storage, never NULL). */
const char* msla_error_string(msla_status status);

/* Bytes of device workspace that any of the calls below needs for this shape
 * (the largest over the entry points).  *bytes is written only on MSLA_OK. */
msla_status msla_workspace_bytes(int B, int C, int H, int W, int heads, int head_dim,
                                 const int* scales, int n_scales, msla_dtype dt,
                                 size_t* bytes);

/* The whole module (Section 3.1, Fig. 2 right): out = MSLA(x).
 * eps is added to the denominator of Eq. (3) in fp32 (the equation has none;
 * a token whose rectified query is all zero then yields exactly 0). */
msla_status msla_forward(const void* x, const void* w_qkv, const void* w_dw,
                         const void* w_gpw, const void* w_proj, void* out,
                         void* workspace, size_t workspace_bytes,
                         int B, int C, int H, int W, int heads, int head_dim,
                         const int* scales, int n_scales,
                         float eps, msla_dtype dt, msla_layout layout, void* stream);

/* msla_forward with a choice of code path (same computation and result contract, Section 3.1).
 * options: bitwise OR of
 *   MSLA_OPT_GENERAL_AGGREGATION  the 16-bit storage types take the general (vector-ALU
 *       depthwise) aggregation kernel instead of the matrix-core one.  msla_forward itself
 *       takes it only for an image whose maps span 2 GiB or more; this is how that path
 *       is reached at ordinary sizes.
 *   MSLA_OPT_STATE_VALU  with n_scales == 0 (no aggregated scale) the Eq. (3) state is accumulated
 *       on the vector ALUs with wavefront shuffles instead of the matrix cores (same result up to
 *       summation order; kept so that the two can be timed against each other).  Ignored otherwise.
 *   MSLA_OPT_STAGE_PROJECT / _AGGREGATE / _FINALIZE / _APPLY  (for profiling) when any of these
 *       is set, only the kernels of the named stages are enqueued: the Q/K/V projection; the
 *       aggregation + partial Eq. (3) states; the fixed-order sum of the partial states; the
 *       fused normalise-and-apply + output projection.  A stage reads what the stages before it
 *       left in `workspace`, so a complete call with the same arguments must have run on that
 *       workspace before; MSLA_NHWC only (else MSLA_ERR_UNSUPPORTED).
 * Any other bit returns MSLA_ERR_INVALID_ARG. */
#define MSLA_OPT_GENERAL_AGGREGATION 1u
#define MSLA_OPT_STAGE_PROJECT 2u
#define MSLA_OPT_STAGE_AGGREGATE 4u
#define MSLA_OPT_STAGE_FINALIZE 8u
#define MSLA_OPT_STAGE_APPLY 16u
#define MSLA_OPT_STATE_VALU 32u
msla_status msla_forward_opts(const void* x, const void* w_qkv, const void* w_dw,
                              const void* w_gpw, const void* w_proj, void* out,
                              void* workspace, size_t workspace_bytes,
                              int B, int C, int H, int W, int heads, int head_dim,
                              const int* scales, int n_scales,
                              float eps, msla_dtype dt, msla_layout layout, void* stream,
                              unsigned options);

/* msla_forward with stage timing (for benchmarks; same computation, Section 3.1).
 * events: HOST array of 5 hipEvent_t created by the caller with timing enabled.  They are
 * recorded on `stream`: [0] before the first kernel, [1] after the Q/K/V projection,
 * [2] after the aggregation kernels (partial states written), [3] after the state
 * finalize kernel, [4] after the fused apply + output projection. */
msla_status msla_forward_profiled(const void* x, const void* w_qkv, const void* w_dw,
                                  const void* w_gpw, const void* w_proj, void* out,
                                  void* workspace, size_t workspace_bytes,
                                  int B, int C, int H, int W, int heads, int head_dim,
                                  const int* scales, int n_scales,
                                  float eps, msla_dtype dt, msla_layout layout, void* stream,
                                  void* const* events);

/* The module without its two projections: multi-scale token aggregation and
 * per-head ReLU linear attention on a given projected map (Section 3.1,
 * Eqs. (2)-(3)): att = concat_s LinearAttention(branch_s(qkv)). */
msla_status msla_core_forward(const void* qkv, const void* w_dw, const void* w_gpw,
                              void* att, void* workspace, size_t workspace_bytes,
                              int B, int H, int W, int heads, int head_dim,
                              const int* scales, int n_scales,
                              float eps, msla_dtype dt, void* stream);

/* Stage: multi-scale aggregation and the once-per-image state of Eq. (3).
 *   q_ms [B, H, W, S*Ct] (storage dtype): the Q tokens of every branch, column
 *        (s*heads + h)*head_dim + e  (branch 0 = the raw Q; may be NULL)
 *   kv   [B, S, heads, head_dim, head_dim+1] fp32:
 *        kv[..., e, f] = sum_n relu(K_n[e]) V_n[f],  kv[..., e, head_dim] = sum_n relu(K_n[e]),
 *        the sum running over the H*W tokens of one image and one branch. */
msla_status msla_multiscale_state(const void* qkv, const void* w_dw, const void* w_gpw,
                                  void* q_ms, float* kv,
                                  void* workspace, size_t workspace_bytes,
                                  int B, int H, int W, int heads, int head_dim,
                                  const int* scales, int n_scales,
                                  msla_dtype dt, void* stream);

/* msla_multiscale_state for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * computation, arguments and results as msla_multiscale_state, except that
 *   - there is no workspace argument: the per-state buffers (partial states of the workgroups, the
 *     summed states, their operand form) live in a device array inside the library, of
 *     MSLA_STATIC_SCRATCH_BYTES on every GPU the library is used on, held until the process ends;
 *   - q_ms must be given (not NULL): the Q tokens of every branch are an output here;
 *   - a shape whose per-state buffers exceed that array returns MSLA_ERR_WORKSPACE with nothing
 *     enqueued.  They take B*S*heads*(1088*(chunks+1) + 2052) bytes plus alignment, chunks being
 *     the number of workgroups one state's reduction is split over (enough to fill the GPU:
 *     2 at B*heads = 128, 32 at B*heads = 8); 8 MiB covers e.g. 1500 states at 2 chunks.
 * It calls no allocating routine.  Every call on a GPU uses that GPU's one array, so calls that
 * overlap on one GPU (different streams, or threads) race: serialise them.  Nothing in the array has
 * to start at zero and nothing in it survives as a result: each call overwrites what it reads. */
#define MSLA_STATIC_SCRATCH_BYTES (8u << 20)
msla_status msla_multiscale_state_static(const void* qkv, const void* w_dw, const void* w_gpw,
                                         void* q_ms, float* kv,
                                         int B, int H, int W, int heads, int head_dim,
                                         const int* scales, int n_scales,
                                         msla_dtype dt, void* stream);

/* The other half of the EfficientViT building block: the FFN with a depthwise convolution inserted
 * (Section 3.1, "we insert a depthwise convolution in each FFN layer"; Fig. 2 left).  The paper's text
 * gives no more than that; this library's declared reading is
 *     h = act(W1 y)   1x1, C -> hidden        g = act(DW3x3(h))   stride 1, zero padding 1, cross-correlation
 *     out = y + W2 g  1x1, hidden -> C, no activation, residual; no bias, no normalisation.
 *   y, out [B, H, W, C] (token-major);  w1 [hidden, C];  w_dw [hidden, 3, 3];  w2 [C, hidden].
 * C and hidden multiples of 16 (else MSLA_ERR_UNSUPPORTED).  out may not alias y.
 * workspace: msla_ffn_workspace_bytes (one [B,H,W,hidden] map: the activated expand result). */
msla_status msla_ffn_workspace_bytes(int B, int C, int H, int W, int hidden, msla_dtype dt, size_t* bytes);
msla_status msla_ffn_forward(const void* y, const void* w1, const void* w_dw, const void* w2, void* out,
                             void* workspace, size_t workspace_bytes,
                             int B, int C, int H, int W, int hidden, msla_act act, msla_dtype dt, void* stream);

/* The whole building block (Fig. 2 left; Section 3.2 puts it in stages 3 and 4 of the backbone):
 *     y = x + MSLA(x)   (msla_forward, MSLA_NHWC)        out = y + FFN(y)   (msla_ffn_forward).
 * Arguments as in those two calls (w_ffn_dw is the FFN's [hidden, 3, 3] filter).  out may not alias x. */
msla_status msla_block_workspace_bytes(int B, int C, int H, int W, int heads, int head_dim,
                                       const int* scales, int n_scales, int hidden, msla_dtype dt, size_t* bytes);
msla_status msla_block_forward(const void* x, const void* w_qkv, const void* w_dw, const void* w_gpw,
                               const void* w_proj, const void* w1, const void* w_ffn_dw, const void* w2,
                               void* out, void* workspace, size_t workspace_bytes,
                               int B, int C, int H, int W, int heads, int head_dim,
                               const int* scales, int n_scales, float eps,
                               int hidden, msla_act act, msla_dtype dt, void* stream);

/* Backward pass of ReLU linear attention: the gradient of Eq. (3) (Section 3.1) with respect to Q, K and V.
 * The paper trains its models (Section 4.1) and prints no gradient, so this is the derivative of the
 * forward definition att_n = relu(Q_n) KV / (relu(Q_n) Ksum + eps), KV|Ksum = sum_n relu(K_n)^T [V_n, 1], per
 * image and head, the rectifier's derivative taken as 0 at 0:
 *   qkv   [B, N, 3*heads*head_dim]  the forward input (channel (h*3 + t)*head_dim + e)
 *   d_att [B, N, heads*head_dim]    dL/d att
 *   d_qkv [B, N, 3*heads*head_dim]  dL/d qkv (written; same channel order)
 * fp32 sums, storage type dt; two passes over the tokens around a second head_dim x (head_dim+1) reduction,
 * summed in a fixed order (reproducible).  head_dim == 16 only.  workspace: the query below (a few KB per state). */
msla_status msla_linear_attention_backward_workspace_bytes(int B, int N, int heads, int head_dim, msla_dtype dt,
                                                           size_t* bytes);
msla_status msla_linear_attention_backward(const void* qkv, const void* d_att, void* d_qkv,
                                           void* workspace, size_t workspace_bytes,
                                           int B, int N, int heads, int head_dim, float eps,
                                           msla_dtype dt, void* stream);

/* Softmax attention, the form the paper's ReLU linear attention replaces (Section 3.1: Eq. (1) with
 * Sim(Q, K) = exp(Q K^T / sqrt(d)); Fig. 3 compares the two): for every image and head
 *     att_i = sum_j exp(Q_i . K_j / sqrt(d)) V_j / sum_j exp(Q_i . K_j / sqrt(d)).
 *   qkv [B, N, 3*heads*head_dim] (channel order as everywhere: (h*3 + t)*head_dim + e)
 *   att [B, N, heads*head_dim]
 * Quadratic in N by definition; here as a measured comparison point (one pass over the keys, nothing of
 * size N x N stored, fp32 sums).  head_dim == 16 only.  No workspace. */
msla_status msla_softmax_attention(const void* qkv, void* att, int B, int N, int heads, int head_dim,
                                   msla_dtype dt, void* stream);

/* Stage: a 1x1 projection of a token map (Section 3.1: Q = x W_Q etc., and the
 * final projection):  y[n, o] = sum_c x[n, c] * w[o, c],
 *   x [n_tokens, c_in], w [c_out, c_in], y [n_tokens, c_out]; c_in, c_out multiples of 16. */
msla_status msla_linear(const void* x, const void* w, void* y,
                        long n_tokens, int c_in, int c_out, msla_dtype dt, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MSLA_H_ */
