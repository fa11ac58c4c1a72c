// Backward pass of ReLU linear attention (the gradient of Eq. (3), Section 3.1; the paper trains its
// models, Section 4.1, and prints nothing about gradients).  Per image and head, with rq = max(Q, 0),
// rk = max(K, 0), the forward state S = sum_n rk_n^T [V_n, 1] and den_n = rq_n . S[:, d] + eps:
//     g_n = dA_n / den_n,   c_n = -(dA_n . att_n) / den_n
//     dS     = sum_n rq_n^T [g_n, c_n]                        (a second reduction over the tokens)
//     dQ_n   = (S[:, :d] g_n + S[:, d] c_n) * [Q_n > 0]
//     dK_n   = (dS[:, :d] V_n + dS[:, d])   * [K_n > 0]
//     dV_n   = rk_n dS[:, :d]
// Like the forward pass it is two passes over the tokens around a d x (d+1) reduction: the forward
// state comes from the library's own state kernels, `backward_state_kernel` accumulates dS per
// workgroup (fixed-order sum afterwards, so results are reproducible), `backward_apply_kernel`
// writes the three gradients.
//
// Every product with a state's d x d part is a 16 x 16 x 16 contraction and runs on the matrix cores in fp32
// (four v_mfma_f32_16x16x4f32 each): the operands -- tokens converted from the storage type, the
// states as the state kernels summed them -- go in exactly, so the pass is fp32 throughout for every
// storage type, with nothing to rescale or to split.  A wave works on 16 tokens at a time, lane
// (token x16, q) holding channels 4q..4q+3 of its token (the fragment convention of the forward
// kernels); a product whose contraction runs over the tokens (dS) takes its operands through a
// multiplication with the identity, which hands lane (channel, q) the tokens 4q..4q+3 of that channel.  What
// involves a state's last column (the denominators, the c terms) is four vector FMAs and two cross-lane adds.
#include "msla_device.h"
#include "msla_kernels.h"

namespace msla {
namespace {

constexpr int kBwdThreads = 256;
constexpr int kStateThreads = 1024;
constexpr int kApplyUnits = 8;      // groups of 16 tokens per workgroup of the apply kernel (the state operands are loaded once)
typedef Traits<float> F32;

__device__ __forceinline__ f32x4 mma(f32x4 c, f32x4 a, f32x4 b) { return F32::mma16(c, a, b); }

// One state [16][17] (fp32, in memory) as matrix-core operands of this lane (x16, q):
//   col[r]  = S[4q+r][x16]   row operand of a product contracted over the state's rows e  (out[f]  = sum_e S[e][f] x[e])
//   row[r]  = S[x16][4q+r]   row operand of a product contracted over its columns f      (out[e]  = sum_f S[e][f] x[f])
//   last[r] = S[4q+r][16]    the state's last column, the four entries that belong to the channels 4q..4q+3 this
//                            lane owns of its token (denominators and the "+ S[:, d] c" terms: vector FMAs)
struct StateOperands {
    f32x4 col, row, last;
};
__device__ __forceinline__ StateOperands state_operands(const float* __restrict__ st) {
    const int x16 = lane_id() & 15, q = lane_id() >> 4;
    StateOperands o;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        o.col[r] = st[(q * 4 + r) * 17 + x16];
        o.row[r] = st[x16 * 17 + q * 4 + r];
        o.last[r] = st[(q * 4 + r) * 17 + 16];
    }
    return o;
}

// What both kernels need of a token: rq = max(Q, 0) (this lane's four channels), g = dA / den (its four
// columns) and c = -(dA . att) / den, from the forward state S.  live: the token exists.
struct TokenGrad {
    f32x4 rq, g;
    float c;
};
// One token's operands as loaded: Q, K, V (K and V only where asked for) and dA, this lane's four channels of
// each.  A token past the end reads token 0 of its image instead (always there) and is zeroed in `widen`, so
// the loads carry no branch and can be issued a group ahead.
template <class T>
struct TokenLoad {
    typename Traits<T>::Frag q, k, v, da;
};
template <class T, bool kWithKV>
__device__ __forceinline__ TokenLoad<T> load_token(const T* row, const T* da_tok) {
    const int q = lane_id() >> 4;
    TokenLoad<T> l;
    l.q = load_frag<T>(row + q * 4);
    l.da = load_frag<T>(da_tok + q * 4);
    if (kWithKV) {
        l.k = load_frag<T>(row + 16 + q * 4);
        l.v = load_frag<T>(row + 32 + q * 4);
    } else {
        l.k = l.v = frag_zero<T>();
    }
    return l;
}
template <class T>
__device__ __forceinline__ f32x4 widen(typename Traits<T>::Frag f, bool live) {
    const f32x4 v = frag_to_f32<T>(f);
    return f32x4{live ? v[0] : 0.f, live ? v[1] : 0.f, live ? v[2] : 0.f, live ? v[3] : 0.f};
}

__device__ __forceinline__ TokenGrad token_grad(f32x4 qf, f32x4 da, const StateOperands& S, float eps, bool live) {
    const f32x4 z = {0.f, 0.f, 0.f, 0.f};
    TokenGrad t;
#pragma unroll
    for (int r = 0; r < 4; ++r) t.rq[r] = fmaxf(qf[r], 0.f);
    const f32x4 num = mma(z, S.col, t.rq);       // lane (token, q): sum_e S[e][4q+r] rq[e]
    float den = 0.f;                             // sum_e S[e][16] rq[e]: this lane's four channels, then the four q
#pragma unroll
    for (int r = 0; r < 4; ++r) den = fmaf(S.last[r], t.rq[r], den);
    den += __shfl_xor(den, 16);
    den += __shfl_xor(den, 32);
    const float inv = live ? 1.0f / (den + eps) : 0.f;
    float dot = 0.f;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        dot = fmaf(da[r], num[r] * inv, dot);
        t.g[r] = da[r] * inv;
    }
    dot += __shfl_xor(dot, 16);
    dot += __shfl_xor(dot, 32);
    t.c = -dot * inv;
    return t;
}

// Both kernels give a workgroup four neighbouring heads, one per wave: a token's Q, K, V of four heads are
// 384 contiguous bytes of its row (three whole 128-byte lines in the 16-bit types), so every line of qkv and
// of d_qkv is touched by one workgroup only.
//
// partial dS of (image b, head h, chunk) -> partials[((b*heads + h)*nchunks + chunk)*272 ...]: sixteen waves, four
// per head, each taking every fourth group of 16 tokens of the chunk; the four are summed in a fixed order
template <class T>
__global__ __launch_bounds__(kStateThreads) void backward_state_kernel(const T* __restrict__ qkv, const T* __restrict__ d_att,
                                                                       const float* __restrict__ kv32,
                                                                       float* __restrict__ partials, int N, int heads,
                                                                       int nchunks, int groups_per_chunk, float eps) {
    __shared__ float red[16 * kStateSize];
    const int quads = (heads + 3) / 4;
    const int lane = lane_id(), wave = threadIdx.x >> 6, x16 = lane & 15, q = lane >> 4;
    const int hw = wave & 3, part = wave >> 2;
    const int h = (blockIdx.x % quads) * 4 + hw;
    const int chunk = (blockIdx.x / quads) % nchunks;
    const int b = blockIdx.x / (quads * nchunks);
    const bool head_live = h < heads;
    const long sid = (long)b * heads + (head_live ? h : 0);
    const StateOperands S = state_operands(kv32 + sid * kStateSize);
    const long ts = 3L * heads * 16;
    const f32x4 z = {0.f, 0.f, 0.f, 0.f};
    f32x4 ident;
#pragma unroll
    for (int r = 0; r < 4; ++r) ident[r] = x16 == q * 4 + r ? 1.0f : 0.0f;
    const typename Traits<T>::Frag ident_t = frag_from_f32<T>(ident);
    f32x4 ds = z, dsc = z;      // lane (f, q): dS[4q+r][f];  lane (e, q): dS[e][16] summed over the tokens 4q+r of every group
    const long n_groups = ((long)N + 15) / 16;
    const long g_begin = (long)chunk * groups_per_chunk;
    const long g_end = g_begin + groups_per_chunk < n_groups ? g_begin + groups_per_chunk : n_groups;
    auto fetch = [&](long g, bool& live) {
        const long n = g * 16 + x16;
        live = n < N;
        const long tok = (long)b * N + (live ? n : 0);
        return load_token<T, false>(qkv + tok * ts + h * 48, d_att + tok * (heads * 16) + h * 16);
    };
    if (head_live && g_begin + part < g_end) {
        bool live, live_next = false;
        TokenLoad<T> cur = fetch(g_begin + part, live), next = cur;
        for (long g = g_begin + part; g < g_end; g += 4) {
            if (g + 4 < g_end) next = fetch(g + 4, live_next);
            const TokenGrad t = token_grad(widen<T>(cur.q, live), widen<T>(cur.da, live), S, eps, live);
            // channel-major forms: lane (channel, q) <- tokens 4q..4q+3 of that channel.  rq is a value of the
            // storage type, so its product with the identity is exact on that type's instruction
            const f32x4 rq_t = Traits<T>::mma16(z, frag_from_f32<T>(t.rq), ident_t);
            const f32x4 g_t = mma(z, t.g, ident);
            ds = mma(ds, rq_t, g_t);         // dS[e][f] += sum_tokens rq[e] g[f]
#pragma unroll
            for (int r = 0; r < 4; ++r) dsc[r] = fmaf(rq_t[r], __shfl(t.c, q * 4 + r), dsc[r]);   // c of token 4q+r
            cur = next;
            live = live_next;
        }
    }
    float last = (dsc[0] + dsc[1]) + (dsc[2] + dsc[3]);     // dS[x16][16]: the four tokens, then the four q
    last += __shfl_xor(last, 16);
    last += __shfl_xor(last, 32);
    float* mine = red + wave * kStateSize;                  // wave = part * 4 + head
#pragma unroll
    for (int r = 0; r < 4; ++r) mine[(q * 4 + r) * 17 + x16] = ds[r];
    if (q == 0) mine[x16 * 17 + 16] = last;
    __syncthreads();
    for (int j = threadIdx.x; j < 4 * kStateSize; j += kStateThreads) {
        const int hh = j / kStateSize, e = j - hh * kStateSize;
        const int head = (blockIdx.x % quads) * 4 + hh;
        if (head < heads)
            partials[(((long)b * heads + head) * nchunks + chunk) * kStateSize + e] =
                (red[hh * kStateSize + e] + red[(4 + hh) * kStateSize + e]) +
                (red[(8 + hh) * kStateSize + e] + red[(12 + hh) * kStateSize + e]);
    }
}

template <class T>
__global__ __launch_bounds__(kBwdThreads) void backward_apply_kernel(const T* __restrict__ qkv, const T* __restrict__ d_att,
                                                                     const float* __restrict__ kv32,
                                                                     const float* __restrict__ ds32, T* __restrict__ d_qkv,
                                                                     int N, int heads, int blocks_per_image, float eps) {
    const int quads = (heads + 3) / 4;
    const int lane = lane_id(), wave = threadIdx.x >> 6, x16 = lane & 15, q = lane >> 4;
    const int h = (blockIdx.x % quads) * 4 + wave;
    const int nb = (blockIdx.x / quads) % blocks_per_image;
    const int b = blockIdx.x / (quads * blocks_per_image);
    if (h >= heads) return;     // no barrier below
    const long sid = (long)b * heads + h;
    const StateOperands S = state_operands(kv32 + sid * kStateSize);
    const StateOperands dS = state_operands(ds32 + sid * kStateSize);
    const long ts = 3L * heads * 16;
    const f32x4 z = {0.f, 0.f, 0.f, 0.f};
    auto fetch = [&](int u, bool& live, long& tok) {
        const long n = ((long)nb * kApplyUnits + u) * 16 + x16;
        live = n < N;
        tok = (long)b * N + (live ? n : 0);
        return load_token<T, true>(qkv + tok * ts + h * 48, d_att + tok * (heads * 16) + h * 16);
    };
    bool live, live_next = false;
    long tok, tok_next = 0;
    TokenLoad<T> cur = fetch(0, live, tok), next = cur;
#pragma unroll
    for (int u = 0; u < kApplyUnits; ++u) {
        if (u + 1 < kApplyUnits) next = fetch(u + 1, live_next, tok_next);
        const f32x4 qf = widen<T>(cur.q, live), kf = widen<T>(cur.k, live), vf = widen<T>(cur.v, live);
        const TokenGrad t = token_grad(qf, widen<T>(cur.da, live), S, eps, live);
        f32x4 rk;
#pragma unroll
        for (int r = 0; r < 4; ++r) rk[r] = fmaxf(kf[r], 0.f);
        // lane (token, q) <- rows 4q..4q+3 of each product
        f32x4 dq = mma(z, S.row, t.g);        // sum_f S[e][f] g[f]
        f32x4 dk = mma(z, dS.row, vf);        // sum_f dS[e][f] V[f]
        const f32x4 dv = mma(z, dS.col, rk);  // sum_e rk[e] dS[e][f]
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            dq[r] = qf[r] > 0.f ? fmaf(S.last[r], t.c, dq[r]) : 0.f;
            dk[r] = kf[r] > 0.f ? dk[r] + dS.last[r] : 0.f;
        }
        if (live) {
            T* out = d_qkv + tok * ts + h * 48 + q * 4;
            store_frag<T>(out, frag_from_f32<T>(dq));
            store_frag<T>(out + 16, frag_from_f32<T>(dk));
            store_frag<T>(out + 32, frag_from_f32<T>(dv));
        }
        cur = next;
        live = live_next;
        tok = tok_next;
    }
}

template <class T>
hipError_t run_backward(const void* qkv, const void* d_att, const float* kv32, float* partials, float* ds32, void* frag_scratch,
                        float* scale_scratch, void* d_qkv, int B, int N, int heads, int nchunks, int tiles_per_chunk,
                        float eps, hipStream_t stream) {
    const long nb1 = (long)B * ((heads + 3) / 4) * nchunks;
    const int bpi = (N + 16 * kApplyUnits - 1) / (16 * kApplyUnits);
    const int quads = (heads + 3) / 4;
    const long nb2 = (long)B * quads * bpi;
    if (nb1 <= 0 || nb1 > 0x7fffffffL || nb2 <= 0 || nb2 > 0x7fffffffL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((backward_state_kernel<T>), dim3((unsigned)nb1), dim3(kStateThreads), 0, stream, (const T*)qkv,
                       (const T*)d_att, kv32, partials, N, heads, nchunks, tiles_per_chunk * 4, eps);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // fixed-order sum of the partial dS (the fp32 form of the state kernel's own second stage; its
    // operand-form outputs go to scratch)
    e = launch_state_finalize(0, partials, ds32, frag_scratch, scale_scratch, B * heads, nchunks, stream);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((backward_apply_kernel<T>), dim3((unsigned)nb2), dim3(kBwdThreads), 0, stream, (const T*)qkv,
                       (const T*)d_att, kv32, ds32, (T*)d_qkv, N, heads, bpi, eps);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_linear_attention_backward(int dt, const void* qkv, const void* d_att, const float* kv32, float* partials,
                                            float* ds32, void* frag_scratch, float* scale_scratch, void* d_qkv, int B,
                                            int N, int heads, int nchunks, int tiles_per_chunk, float eps,
                                            hipStream_t stream) {
    switch (dt) {
        case 0: return run_backward<float>(qkv, d_att, kv32, partials, ds32, frag_scratch, scale_scratch, d_qkv, B, N, heads, nchunks, tiles_per_chunk, eps, stream);
        case 1: return run_backward<_Float16>(qkv, d_att, kv32, partials, ds32, frag_scratch, scale_scratch, d_qkv, B, N, heads, nchunks, tiles_per_chunk, eps, stream);
        case 2: return run_backward<__bf16>(qkv, d_att, kv32, partials, ds32, frag_scratch, scale_scratch, d_qkv, B, N, heads, nchunks, tiles_per_chunk, eps, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace msla
