// Host-side launchers of the gfx950 kernels (internal to the library; the
// public boundary is include/msla.h).  Every pointer is a device pointer.
// dt: 0 fp32, 1 fp16, 2 bf16 (the values of msla_dtype).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace msla {

// Number of compute units of the current device (queried once per process).
int compute_units();

// y[n, o] = sum_c x[n, c] * w[o, c]
hipError_t launch_linear(int dt, const void* x, const void* w, void* y, long n_tokens, int c_in,
                         int c_out, hipStream_t stream);

// The Q/K/V projection with a split destination: output channel (h*3+t)*16+e goes to
//   t = 0: q_ms[n * q_ms_stride + h*16 + e]       (branch-0 columns of the multi-scale Q map)
//   t > 0: kv_raw[n * kv_tok_stride + h * kv_head_stride + (t-1)*16 + e]
// with (kv_tok_stride, kv_head_stride) = (2*Ct, 32) for a token-major K|V map or (32, P*32) for a
// head-major one whose P >= n_tokens is a multiple of 32 (rows of a ragged last tile fall into the
// padding); kv_span = elements of the whole map, below 2^30 when head-major.
hipError_t launch_qkv_project(int dt, const void* x, const void* w_qkv, void* q_ms, long q_ms_stride,
                              void* kv_raw, long kv_tok_stride, long kv_head_stride, long kv_span,
                              long n_tokens, int c_in, int heads, hipStream_t stream);

struct AggregateArgs {
    // raw Q, K, V maps: element (token n, head h, channel e) of map m lives at
    // m + n * m_ts + h * m_hs + e   (strides in elements)
    const void *q, *k, *v;
    long q_ts, k_ts, v_ts;
    int q_hs, k_hs, v_hs;
    const void* w_dw;        // [3*Ct, ks, ks] of this scale
    const void* w_gpw;       // [3*Ct, 16] of this scale
    void* q_ms;              // [T, S*Ct] multi-scale Q map (written: this branch; branch 0 if copy_raw_q)
    float* partials;         // [B, S, heads, nchunks, 272] per-workgroup partial states
    int B, H, W, heads, S;
    int ks;                  // 3 or 5
    int branch;              // 1 + index of this scale
    int nchunks, tiles_per_chunk;
    int do_raw;              // also accumulate the branch-0 state from the raw K, V
    int copy_raw_q;          // also copy the raw Q into the branch-0 columns of q_ms
    int state_valu = 0;      // raw-state kernel only: vector ALUs + shuffles instead of the matrix cores
};
hipError_t launch_aggregate(int dt, const AggregateArgs& a, hipStream_t stream);

// Same contract for the 16-bit storage types, depthwise convolution on the matrix cores
// (16 x 32-token tiles; needs v == k + 16 elements with equal strides).  Returns
// hipErrorNotSupported without launching when one image's maps span 2^31 bytes or more.
hipError_t launch_aggregate_mfma(int dt, const AggregateArgs& a, hipStream_t stream);

// Two aggregated scales (3x3 and 5x5, either order) of the same module in one launch; hipErrorNotSupported,
// without launching, for anything else (then the caller launches them one by one).
hipError_t launch_aggregate_mfma_pair(int dt, const AggregateArgs& a0, const AggregateArgs& a1, hipStream_t stream);

// The same contract for heads of 32 channels, fp16 / bf16 (k_aggregate32.hip): maps with 32 channels per head and
// kind, w_gpw rows of 32, partial states [.., nchunks, 32*33], 8 x 32-token tiles.  hipErrorNotSupported for fp32.
hipError_t launch_aggregate32(int dt, const AggregateArgs& a, hipStream_t stream);

// Raw-branch-only variant for n_scales == 0 (no convolution): state of branch 0, optional Q copy.
hipError_t launch_raw_state(int dt, const AggregateArgs& a, hipStream_t stream);

// Sums the per-workgroup partial states in a fixed order and emits
//   kv32    [n_states, 16, 17] fp32 (the state of Eq. (3))
//   kvfrag  [n_states, 2, 64, 16 bytes] the state laid out as MFMA operands
//   kvscale [n_states] the power of two the operands were scaled by
// split = 8: a state holds two heads of 8 channels side by side; the operands keep each head's own block of KV
// and, row by row, its own part of Ksum (0: one head of 16)
hipError_t launch_state_finalize(int dt, const float* partials, float* kv32, void* kvfrag, float* kvscale,
                                 int n_states, int nchunks, hipStream_t stream, int split = 0);

// Head size 8 on the head-size-16 kernels: heads 2p and 2p+1 become one head of 16 whose Q, K and V blocks are
// [Q_2p Q_2p+1], [K_2p K_2p+1], [V_2p V_2p+1].  Writes the module's weights in that arrangement: the rows of
// w_qkv [3*Ct, C] and of every scale's w_dw [3*Ct, k, k] permuted, and w_gpw [A, 3*Ct, 8] as block-diagonal
// [A, 3*Ct, 16] (k_generic.hip).  heads8 must be even.
hipError_t launch_pair_head8_weights(int dt, const void* w_qkv, const void* w_dw, const void* w_gpw, void* w_qkv16,
                                     void* w_dw16, void* w_gpw16, int C, int heads8, const int* scales, int n_scales,
                                     hipStream_t stream);

// att[n, m*16 + f] for every head-branch m of q_ms (Eq. (3), last line)
hipError_t launch_apply(int dt, const void* q_ms, const void* kvfrag, const float* kvscale, void* att,
                        long n_tokens, int tokens_per_image, int n_hb, float eps, hipStream_t stream);

// out[n, c] = (res ? res[n, c] : 0) + sum_m att[n, m] * w_proj[c, m] with att produced on the fly; the optional
// residual [n_tokens, c_out] joins the fp32 sums before their one rounding
hipError_t launch_apply_project(int dt, const void* q_ms, const void* kvfrag, const float* kvscale,
                                const void* w_proj, void* out, const void* res, long n_tokens, int tokens_per_image,
                                int n_hb, int c_out, float eps, hipStream_t stream);

// The same three operations for 16-bit storage types with a contraction of 257 .. 1024 slots and
// few enough tokens that the weights are what a workgroup mostly fetches (k_small.hip).  They return
// hipErrorNotSupported, without launching, for anything else.
hipError_t launch_small_linear(int dt, const void* x, const void* w, void* y, long n_tokens, int c_in, int c_out,
                               hipStream_t stream);
hipError_t launch_small_qkv_project(int dt, const void* x, const void* w_qkv, void* q_ms, long q_ms_stride,
                                    void* kv_raw, long kv_tok_stride, long kv_head_stride, long n_tokens, int c_in,
                                    int heads, hipStream_t stream);
hipError_t launch_small_apply_project(int dt, const void* q_ms, const void* kvfrag, const float* kvscale,
                                      const void* w_proj, void* out, const void* res, long n_tokens, int tokens_per_image,
                                      int n_hb, int c_out, float eps, hipStream_t stream);
// whether a [n_tokens x K] by [K x c_out] product is "small" in that sense
inline bool small_product(int dt, long n_tokens, int K, int c_out) {
    return dt != 0 && K > 256 && K <= 1024 && ((n_tokens + 31) / 32) * ((c_out + 127) / 128) <= 8L * compute_units();
}

// The FFN+DWConv half of the building block (k_ffn.hip).  act: 0 ReLU, 1 hard-swish.
//   out[n, c] = res[n, c] + sum_e act(DW3x3(h))[n, e] * w2[c, e]   (one kernel: the depthwise result stays on chip)
hipError_t launch_ffn_dw_project(int dt, const void* h, const void* w_dw, const void* w2, const void* res, void* out, int B,
                                 int H, int W, int E, int c_out, int act, hipStream_t stream);
//   y[n, o] = act(sum_c x[n, c] * w[o, c])   (k_project.hip; the activation is applied to the fp32 sums)
hipError_t launch_linear_act(int dt, const void* x, const void* w, void* y, long n_tokens, int c_in, int c_out, int act,
                             hipStream_t stream);
//   y[n, o] = res[n, o] + sum_c x[n, c] * w[o, c]   (k_project.hip, tiled form; the residual joins the fp32 sums)
hipError_t launch_linear_residual(int dt, const void* x, const void* w, const void* res, void* y, long n_tokens,
                                  int c_in, int c_out, hipStream_t stream);

// Softmax attention per image and head on qkv [B, N, 3*heads*16] -> att [B, N, heads*16] (k_softmax.hip)
hipError_t launch_softmax_attention(int dt, const void* qkv, void* att, int B, int N, int heads, hipStream_t stream);

// Gradient of Eq. (3) (k_backward.hip): d_qkv [B, N, 3*heads*16] from qkv, d_att [B, N, heads*16] and the forward
// states kv32 [B*heads, 16, 17]; partials [B*heads*nchunks*272], ds32 [B*heads*272], frag_scratch [B*heads*2048 bytes]
// and scale_scratch [B*heads] are work buffers.
hipError_t launch_linear_attention_backward(int dt, const void* qkv, const void* d_att, const float* kv32, float* partials,
                                            float* ds32, void* frag_scratch, float* scale_scratch, void* d_qkv, int B,
                                            int N, int heads, int nchunks, int tiles_per_chunk, float eps,
                                            hipStream_t stream);

// The module's core (aggregation, Eq. (3) state, normalise-and-apply) for head sizes 8 and 32 (k_generic.hip):
// att [T, S*heads*head_dim] from the projected map qkv [T, 3*heads*head_dim].
struct GenericArgs {
    const void* qkv;
    const void* w_dw;       // concat over scales of [3*Ct, k, k]
    const void* w_gpw;      // [A, 3*Ct, head_dim]
    void* q_ms;             // [T, S*Ct] work buffer: the Q tokens of every branch
    float* partials;        // [B*S*heads*nchunks, head_dim*(head_dim+1)]
    float* kv32;            // [B*S*heads, head_dim*(head_dim+1)]
    void* att;
    int B, H, W, heads, head_dim;
    int n_scales;
    int scales[8];
    int nchunks;
    float eps;
};
hipError_t launch_generic_core(int dt, const GenericArgs& a, hipStream_t stream);

// dst[b][c][r] = src[b][r][c] for every b < batch: the change between [B, C, H*W] and [B, H*W, C]
hipError_t launch_transpose(int dt, const void* src, void* dst, long batch, int rows, int cols,
                            hipStream_t stream);

// Raises a kernel's dynamic-LDS limit (the CU has 160 KB; the default limit is 48 KB).  The attribute
// sticks to the (kernel, device) pair, so it is set once for each: later launches -- also those
// recorded into a graph -- make no runtime call besides the launch itself.
template <auto Kernel>
inline hipError_t allow_dynamic_lds(int bytes) {
    static bool done[64] = {};      // benign if two threads race to set an entry
    int dev = 0;
    const hipError_t eg = hipGetDevice(&dev);
    if (eg != hipSuccess) return eg;
    if (dev >= 0 && dev < 64 && done[dev]) return hipSuccess;
    const hipError_t e = hipFuncSetAttribute((const void*)Kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess && dev >= 0 && dev < 64) done[dev] = true;
    return e;
}

constexpr int kAggTileH = 8;        // vector-ALU kernel (fp32 storage)
constexpr int kAggTileW = 32;
constexpr int kAggMfmaTileH = 16;   // matrix-core kernel (fp16 / bf16 storage)
constexpr int kAggMfmaTileW = 32;

}  // namespace msla
