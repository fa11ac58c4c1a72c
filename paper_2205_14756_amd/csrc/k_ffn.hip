// The FFN+DWConv half of the EfficientViT building block (Section 3.1: a depthwise convolution is
// inserted into the FFN layer that follows the attention module; Fig. 2 left) and the residual
// additions of the block.  Declared reading (the paper prints no more than the sentence above):
//   h   = act(W1 y)                      1x1 expand, C -> E
//   g   = act(DW3x3(h))                  depthwise 3x3, stride 1, zero padding 1, cross-correlation
//   out = y + W2 g                       1x1 project, E -> C, no activation, residual
// with act = ReLU or hard-swish, no bias, no normalisation.
//
// Kernels here: the depthwise pass (vector ALUs, both activations fused: it reads the expand
// projection's result before its activation), the projection E -> C with the residual added to
// the fp32 sums before their one rounding, and a plain residual addition (y = x + MSLA(x)).
// The expand projection is the library's ordinary 1x1 projection.
#include "gemm_tile.h"
#include "msla_kernels.h"

namespace msla {
namespace {

template <int ACT>
__device__ __forceinline__ float activate(float a) {
    if constexpr (ACT == 0) return fmaxf(a, 0.f);
    else return a * fminf(fmaxf(a + 3.f, 0.f), 6.f) * (1.0f / 6.0f);
}

// 16 bytes of consecutive channels <-> fp32
template <class T>
struct Pack {
    static constexpr int N = 16 / (int)sizeof(T);
    static __device__ __forceinline__ void unpack(u32x4 v, float (&f)[N]) {
        if constexpr (sizeof(T) == 4) {
            const f32x4 x = __builtin_bit_cast(f32x4, v);
#pragma unroll
            for (int i = 0; i < 4; ++i) f[i] = x[i];
        } else {
            typedef typename Traits<T>::Vec Vec;
            const Vec x = __builtin_bit_cast(Vec, v);
#pragma unroll
            for (int i = 0; i < 8; ++i) f[i] = Traits<T>::to_f32(x[i]);
        }
    }
    static __device__ __forceinline__ u32x4 pack(const float (&f)[N]) {
        if constexpr (sizeof(T) == 4) {
            return __builtin_bit_cast(u32x4, f32x4{f[0], f[1], f[2], f[3]});
        } else {
            typename Traits<T>::Vec x;
#pragma unroll
            for (int i = 0; i < 8; ++i) x[i] = Traits<T>::from_f32(f[i]);
            return __builtin_bit_cast(u32x4, x);
        }
    }
};

constexpr int kDwRows = 8;       // output rows per thread (its window slides down them)

// g = act(DW3x3(act(h))).  A thread owns 16 bytes of channels at one column x and slides a 3x3
// window down kDwRows rows: three 16-byte loads per new row, the filter taps in registers.
// Consecutive threads take consecutive channel vectors, so every load and store is contiguous
// across the wave; the neighbouring columns' reads of the same rows hit the caches.
template <class T, int ACT>
__global__ __launch_bounds__(256) void ffn_dw_kernel(const T* __restrict__ h, const T* __restrict__ w_dw,
                                                     T* __restrict__ g, int B, int H, int W, int E, long n_items) {
    constexpr int V = Pack<T>::N;
    const long item = (long)blockIdx.x * 256 + threadIdx.x;
    if (item >= n_items) return;
    const int n_cv = E / V;
    const int cv = (int)(item % n_cv);
    long rest = item / n_cv;
    const int x = (int)(rest % W);
    rest /= W;
    const int strips = (H + kDwRows - 1) / kDwRows;
    const int y0 = (int)(rest % strips) * kDwRows;
    const int b = (int)(rest / strips);
    const int c0 = cv * V;

    float wt[9][V];
#pragma unroll
    for (int j = 0; j < V; ++j)
#pragma unroll
        for (int t = 0; t < 9; ++t) wt[t][j] = Traits<T>::to_f32(w_dw[(long)(c0 + j) * 9 + t]);

    const T* img = h + (long)b * H * W * E + c0;
    T* out = g + (long)b * H * W * E + c0;
    float win[3][3][V];        // [row slot][column x-1, x, x+1][channel]
    auto load_row = [&](int yy, float (&row)[3][V]) {
#pragma unroll
        for (int dx = 0; dx < 3; ++dx) {
            const int xx = x + dx - 1;
            u32x4 v = {0u, 0u, 0u, 0u};
            const bool ok = yy >= 0 && yy < H && xx >= 0 && xx < W;
            if (ok) v = *(const u32x4*)(img + ((long)yy * W + xx) * E);
            float f[V];
            Pack<T>::unpack(v, f);
#pragma unroll
            for (int j = 0; j < V; ++j) row[dx][j] = ok ? activate<ACT>(f[j]) : 0.f;     // padding is zero AFTER the activation
        }
    };
    load_row(y0 - 1, win[0]);
    load_row(y0, win[1]);
#pragma unroll
    for (int r = 0; r < kDwRows; ++r) {
        const int yy = y0 + r;
        load_row(yy + 1, win[(r + 2) % 3]);
        if (yy < H) {
            float acc[V];
#pragma unroll
            for (int j = 0; j < V; ++j) acc[j] = 0.f;
#pragma unroll
            for (int u = 0; u < 3; ++u)
#pragma unroll
                for (int dx = 0; dx < 3; ++dx)
#pragma unroll
                    for (int j = 0; j < V; ++j) acc[j] = fmaf(wt[u * 3 + dx][j], win[(r + u) % 3][dx][j], acc[j]);
#pragma unroll
            for (int j = 0; j < V; ++j) acc[j] = activate<ACT>(acc[j]);
            *(u32x4*)(out + ((long)yy * W + x) * E) = Pack<T>::pack(acc);
        }
    }
}

// y = a + b, 16 bytes a thread, fp32 addition, one rounding.
template <class T>
__global__ __launch_bounds__(256) void residual_add_kernel(const T* __restrict__ a, const T* __restrict__ b,
                                                           T* __restrict__ y, long n_vec) {
    constexpr int V = Pack<T>::N;
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= n_vec) return;
    float fa[V], fb[V];
    Pack<T>::unpack(((const u32x4*)a)[i], fa);
    Pack<T>::unpack(((const u32x4*)b)[i], fb);
#pragma unroll
    for (int j = 0; j < V; ++j) fa[j] += fb[j];
    ((u32x4*)y)[i] = Pack<T>::pack(fa);
}

// out[n, c] = res[n, c] + sum_e g[n, e] * w2[c, e]: tiled (256 channels x 128 tokens per workgroup,
// 64 x 64 per wave, any contraction length), next slab's loads in flight during the matrix
// instructions; the residual joins the fp32 sums in the epilogue.
template <class T, int WR, int WC>
__global__ __launch_bounds__(WR * WC * 64) void ffn_project_kernel(const T* __restrict__ g, const T* __restrict__ w2,
                                                                   const T* __restrict__ res, T* __restrict__ out,
                                                                   long n_tokens, int E, int c_out, int n_rb) {
    typedef GemmTile<T, WR, WC> G;
    extern __shared__ __attribute__((aligned(16))) char lds[];
    char* ldsR = lds;
    char* ldsC = lds + G::kLdsR;
    const unsigned L = xcd_remap(blockIdx.x, gridDim.x);
    const int rb = L % n_rb;
    const long tok0 = (long)(L / n_rb) * G::BC;
    const int oc0 = rb * G::BR;
    const int wave = threadIdx.x >> 6;
    const int wr = wave % WR, wc = wave / WR;

    f32x4 acc[4][4];
    G::zero(acc);
    u32x4 rw[G::kVecR], rc[G::kVecC];
    G::load_global(rw, w2, oc0, c_out, E, 0, E);
    G::load_global(rc, g, tok0, n_tokens, E, 0, E);
    for (int k0 = 0; k0 < E; k0 += G::BK) {
        G::store_lds_r(ldsR, rw);
        G::store_lds_c(ldsC, rc);
        __syncthreads();
        if (k0 + G::BK < E) {
            G::load_global(rw, w2, oc0, c_out, E, k0 + G::BK, E);
            G::load_global(rc, g, tok0, n_tokens, E, k0 + G::BK, E);
        }
        G::mma(acc, ldsR, ldsC, wr, wc);
        __syncthreads();
    }
    G::epilogue(acc, tok0, n_tokens, oc0, c_out, wr, wc, [res, out, c_out](long tok, int oc, f32x4 v) {
        const f32x4 r = frag_to_f32<T>(load_frag<T>(res + tok * c_out + oc));
        store_frag<T>(out + tok * c_out + oc, frag_from_f32<T>(f32x4{v[0] + r[0], v[1] + r[1], v[2] + r[2], v[3] + r[3]}));
    });
}

template <class T>
hipError_t run_dw(const void* h, const void* w_dw, void* g, int B, int H, int W, int E, int act, hipStream_t stream) {
    const long n_items = (long)B * ((H + kDwRows - 1) / kDwRows) * W * (E / Pack<T>::N);
    const long nblocks = (n_items + 255) / 256;
    if (nblocks <= 0 || nblocks > 0x7fffffffL) return hipErrorInvalidValue;
    if (act == 0)
        hipLaunchKernelGGL((ffn_dw_kernel<T, 0>), dim3((unsigned)nblocks), dim3(256), 0, stream, (const T*)h, (const T*)w_dw, (T*)g, B, H, W, E, n_items);
    else
        hipLaunchKernelGGL((ffn_dw_kernel<T, 1>), dim3((unsigned)nblocks), dim3(256), 0, stream, (const T*)h, (const T*)w_dw, (T*)g, B, H, W, E, n_items);
    return hipGetLastError();
}

template <class T>
hipError_t run_add(const void* a, const void* b, void* y, long n_elems, hipStream_t stream) {
    const long n_vec = n_elems / Pack<T>::N;
    const long nblocks = (n_vec + 255) / 256;
    if (nblocks <= 0 || nblocks > 0x7fffffffL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((residual_add_kernel<T>), dim3((unsigned)nblocks), dim3(256), 0, stream, (const T*)a, (const T*)b, (T*)y, n_vec);
    return hipGetLastError();
}

template <class T>
hipError_t run_ffn_project(const void* g, const void* w2, const void* res, void* out, long n_tokens, int E, int c_out,
                           hipStream_t stream) {
    typedef GemmTile<T, 4, 2> G;
    const int n_rb = (c_out + G::BR - 1) / G::BR;
    const long nblocks = ((n_tokens + G::BC - 1) / G::BC) * n_rb;
    if (nblocks <= 0 || nblocks > 0x7fffffffL) return hipErrorInvalidValue;
    constexpr int kLds = G::kLdsR + G::kLdsC;
    const hipError_t e = allow_dynamic_lds<ffn_project_kernel<T, 4, 2>>(kLds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((ffn_project_kernel<T, 4, 2>), dim3((unsigned)nblocks), dim3(G::kThreads), kLds, stream, (const T*)g,
                       (const T*)w2, (const T*)res, (T*)out, n_tokens, E, c_out, n_rb);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_ffn_dw(int dt, const void* h, const void* w_dw, void* g, int B, int H, int W, int E, int act,
                         hipStream_t stream) {
    switch (dt) {
        case 0: return run_dw<float>(h, w_dw, g, B, H, W, E, act, stream);
        case 1: return run_dw<_Float16>(h, w_dw, g, B, H, W, E, act, stream);
        case 2: return run_dw<__bf16>(h, w_dw, g, B, H, W, E, act, stream);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_residual_add(int dt, const void* a, const void* b, void* y, long n_elems, hipStream_t stream) {
    switch (dt) {
        case 0: return run_add<float>(a, b, y, n_elems, stream);
        case 1: return run_add<_Float16>(a, b, y, n_elems, stream);
        case 2: return run_add<__bf16>(a, b, y, n_elems, stream);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_ffn_project(int dt, const void* g, const void* w2, const void* res, void* out, long n_tokens, int E,
                              int c_out, hipStream_t stream) {
    switch (dt) {
        case 0: return run_ffn_project<float>(g, w2, res, out, n_tokens, E, c_out, stream);
        case 1: return run_ffn_project<_Float16>(g, w2, res, out, n_tokens, E, c_out, stream);
        case 2: return run_ffn_project<__bf16>(g, w2, res, out, n_tokens, E, c_out, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace msla
