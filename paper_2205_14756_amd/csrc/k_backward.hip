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
// writes the three gradients.  Both work on the vector ALUs with four lanes per token: lane
// (token slot l / 4, part p = l % 4) owns output columns 4p..4p+3; everything is fp32 in registers.
#include "msla_device.h"
#include "msla_kernels.h"

namespace msla {
namespace {

constexpr int kBwdThreads = 256;
// a state in LDS: rows padded from 17 to 20 floats, so that four columns are one 16-byte read
constexpr int kRowS = 20;
constexpr int kLdsState = 16 * kRowS;
__device__ __forceinline__ void stage_state(float* dst, const float* __restrict__ src, int tid, int nthreads) {
    for (int j = tid; j < kStateSize; j += nthreads) dst[(j / 17) * kRowS + j % 17] = src[j];
}

// What both kernels need of one token: its rectified query, and from S and dA the quantities g
// (this lane's four columns) and c.
template <class T>
struct TokenGrad {
    float rq[16];
    float g[4];
    float c;
};

template <class T>
__device__ __forceinline__ void load16(const T* p, float (&f)[16]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const f32x4 v = frag_to_f32<T>(load_frag<T>(p + i * 4));
#pragma unroll
        for (int r = 0; r < 4; ++r) f[i * 4 + r] = v[r];
    }
}

// S: this (image, head)'s forward state in LDS, [16][kRowS].  live: the token exists.
template <class T>
__device__ __forceinline__ TokenGrad<T> token_grad(const T* q_tok, const T* da_tok, const float* S, int p, float eps,
                                                   bool live) {
    TokenGrad<T> t;
    float q[16];
    f32x4 da = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int e = 0; e < 16; ++e) q[e] = 0.f;
    if (live) {
        load16<T>(q_tok, q);
        da = frag_to_f32<T>(load_frag<T>(da_tok + p * 4));
    }
    float den = eps;
    float num[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        t.rq[e] = fmaxf(q[e], 0.f);
        den = fmaf(t.rq[e], S[e * kRowS + 16], den);
        const f32x4 s4 = *(const f32x4*)(S + e * kRowS + p * 4);
#pragma unroll
        for (int j = 0; j < 4; ++j) num[j] = fmaf(t.rq[e], s4[j], num[j]);
    }
    const float inv = live ? 1.0f / den : 0.f;
    float dot = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        dot = fmaf(da[j], num[j] * inv, dot);
        t.g[j] = da[j] * inv;
    }
    dot += __shfl_xor(dot, 1);
    dot += __shfl_xor(dot, 2);
    t.c = -dot * inv;
    return t;
}

// partial dS of (image b, head h, chunk) -> partials[((b*heads + h)*nchunks + chunk)*272 ...]
template <class T>
__global__ __launch_bounds__(kBwdThreads) void backward_state_kernel(const T* __restrict__ qkv, const T* __restrict__ d_att,
                                                                     const float* __restrict__ kv32,
                                                                     float* __restrict__ partials, int N, int heads,
                                                                     int nchunks, int groups_per_chunk, float eps) {
    __shared__ __attribute__((aligned(16))) float S[kLdsState];
    __shared__ float red[4 * kStateSize];
    const int h = blockIdx.x % heads;
    const int chunk = (blockIdx.x / heads) % nchunks;
    const int b = blockIdx.x / (heads * nchunks);
    const int lane = lane_id(), wave = threadIdx.x >> 6, slot = lane >> 2, p = lane & 3;
    const long sid = (long)b * heads + h;
    stage_state(S, kv32 + sid * kStateSize, threadIdx.x, kBwdThreads);
    __syncthreads();
    const long ts = 3L * heads * 16;
    float acc[16][4], accs[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        accs[e] = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[e][j] = 0.f;
    }
    const long n_groups = ((long)N + 15) / 16;
    const long g_begin = (long)chunk * groups_per_chunk;
    const long g_end = g_begin + groups_per_chunk < n_groups ? g_begin + groups_per_chunk : n_groups;
    for (long g = g_begin + wave; g < g_end; g += 4) {
        const long n = g * 16 + slot;
        const bool live = n < N;
        const long tok = (long)b * N + (live ? n : 0);
        const TokenGrad<T> t = token_grad<T>(qkv + tok * ts + h * 48, d_att + tok * (heads * 16) + h * 16, S, p, eps, live);
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            accs[e] = fmaf(t.rq[e], t.c, accs[e]);
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[e][j] = fmaf(t.rq[e], t.g[j], acc[e][j]);
        }
    }
    // sum over the wave's 16 token slots, then over the four waves in a fixed order
#pragma unroll
    for (int e = 0; e < 16; ++e)
#pragma unroll
        for (int o = 4; o < 64; o <<= 1) {
            accs[e] += __shfl_xor(accs[e], o);
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[e][j] += __shfl_xor(acc[e][j], o);
        }
    float* mine = red + wave * kStateSize;
    if (slot == 0) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
#pragma unroll
            for (int j = 0; j < 4; ++j) mine[e * 17 + p * 4 + j] = acc[e][j];
            if (p == 0) mine[e * 17 + 16] = accs[e];
        }
    }
    __syncthreads();
    for (int j = threadIdx.x; j < kStateSize; j += kBwdThreads)
        partials[(sid * nchunks + chunk) * kStateSize + j] =
            (red[j] + red[kStateSize + j]) + (red[2 * kStateSize + j] + red[3 * kStateSize + j]);
}

template <class T>
__global__ __launch_bounds__(kBwdThreads) void backward_apply_kernel(const T* __restrict__ qkv, const T* __restrict__ d_att,
                                                                     const float* __restrict__ kv32,
                                                                     const float* __restrict__ ds32, T* __restrict__ d_qkv,
                                                                     int N, int heads, int blocks_per_image, float eps) {
    __shared__ __attribute__((aligned(16))) float S[kLdsState];
    __shared__ __attribute__((aligned(16))) float dS[kLdsState];
    const int h = blockIdx.x % heads;
    const int nb = (blockIdx.x / heads) % blocks_per_image;
    const int b = blockIdx.x / (heads * blocks_per_image);
    const int lane = lane_id(), wave = threadIdx.x >> 6, slot = lane >> 2, p = lane & 3;
    const long sid = (long)b * heads + h;
    stage_state(S, kv32 + sid * kStateSize, threadIdx.x, kBwdThreads);
    stage_state(dS, ds32 + sid * kStateSize, threadIdx.x, kBwdThreads);
    __syncthreads();
    const long ts = 3L * heads * 16;
    const long n = (long)nb * 64 + wave * 16 + slot;
    const bool live = n < N;
    const long tok = (long)b * N + (live ? n : 0);
    const T* row = qkv + tok * ts + h * 48;
    const TokenGrad<T> t = token_grad<T>(row, d_att + tok * (heads * 16) + h * 16, S, p, eps, live);
    // every lane needs all 16 columns of g for its rows of dQ: gather them from the token's four lanes
    float g_all[16];
#pragma unroll
    for (int pp = 0; pp < 4; ++pp)
#pragma unroll
        for (int j = 0; j < 4; ++j) g_all[pp * 4 + j] = __shfl(t.g[j], (lane & ~3) | pp);
    float q[16], k[16], v[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) q[e] = k[e] = v[e] = 0.f;
    if (live) {
        load16<T>(row, q);
        load16<T>(row + 16, k);
        load16<T>(row + 32, v);
    }
    f32x4 dq, dk, dv;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int e = p * 4 + i;
        float a = S[e * kRowS + 16] * t.c;
        float bk = dS[e * kRowS + 16];
#pragma unroll
        for (int f4 = 0; f4 < 16; f4 += 4) {
            const f32x4 s4 = *(const f32x4*)(S + e * kRowS + f4);
            const f32x4 d4 = *(const f32x4*)(dS + e * kRowS + f4);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                a = fmaf(s4[j], g_all[f4 + j], a);
                bk = fmaf(d4[j], v[f4 + j], bk);
            }
        }
        // (a lane's own Q and K entries, picked without a dynamic register index)
        float qe = 0.f, ke = 0.f;
#pragma unroll
        for (int pp = 0; pp < 4; ++pp) {
            qe = p == pp ? q[pp * 4 + i] : qe;
            ke = p == pp ? k[pp * 4 + i] : ke;
        }
        dq[i] = qe > 0.f ? a : 0.f;
        dk[i] = ke > 0.f ? bk : 0.f;
    }
    // dV: this lane's four columns of rk dS[:, :d], a 16-byte read per row
    {
        f32x4 c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int e2 = 0; e2 < 16; ++e2) {
            const f32x4 d4 = *(const f32x4*)(dS + e2 * kRowS + p * 4);
            const float rk = fmaxf(k[e2], 0.f);
#pragma unroll
            for (int i = 0; i < 4; ++i) c[i] = fmaf(rk, d4[i], c[i]);
        }
        dv = c;
    }
    if (live) {
        T* out = d_qkv + tok * ts + h * 48 + p * 4;
        store_frag<T>(out, frag_from_f32<T>(dq));
        store_frag<T>(out + 16, frag_from_f32<T>(dk));
        store_frag<T>(out + 32, frag_from_f32<T>(dv));
    }
}

template <class T>
hipError_t run_backward(const void* qkv, const void* d_att, const float* kv32, float* partials, float* ds32, void* frag_scratch,
                        float* scale_scratch, void* d_qkv, int B, int N, int heads, int nchunks, int tiles_per_chunk,
                        float eps, hipStream_t stream) {
    const long nb1 = (long)B * heads * nchunks;
    const int bpi = (N + 63) / 64;
    const long nb2 = (long)B * heads * bpi;
    if (nb1 <= 0 || nb1 > 0x7fffffffL || nb2 <= 0 || nb2 > 0x7fffffffL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((backward_state_kernel<T>), dim3((unsigned)nb1), dim3(kBwdThreads), 0, stream, (const T*)qkv,
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
