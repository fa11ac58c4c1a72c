// The FFN+DWConv half of the EfficientViT building block (Section 3.1: a depthwise convolution is
// inserted into the FFN layer that follows the attention module; Fig. 2 left).  Declared reading (the paper prints no more than the sentence above):
//   h   = act(W1 y)                      1x1 expand, C -> E
//   g   = act(DW3x3(h))                  depthwise 3x3, stride 1, zero padding 1, cross-correlation
//   out = y + W2 g                       1x1 project, E -> C, no activation, residual
// with act = ReLU or hard-swish, no bias, no normalisation.
//
// Kernel here: the depthwise pass with its activation (vector ALUs).  Both projections are the
// library's 1x1 projection kernels: the first applies the activation to its fp32 sums, the second adds
// the residual to them, each before the one rounding; the block's y = x + MSLA(x) is formed the same
// way, in the epilogue of the attention module's output projection.
#include "msla_device.h"
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

constexpr int kDwRows = 16;      // output rows per thread (its window slides down them)

// g = act(DW3x3(h)), h being the expand projection's ACTIVATED result (its kernel applies the
// activation to its fp32 sums).  A thread owns 16 bytes of channels at one column x and slides a 3x3
// window down kDwRows rows: three 16-byte loads per new row -- requested one row ahead of their
// use, so a row's arithmetic covers the next row's latency -- and the filter taps in registers.
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
    struct Raw {
        u32x4 v[3];
        bool ok[3];
    };
    auto request = [&](int yy, Raw& r) {
#pragma unroll
        for (int dx = 0; dx < 3; ++dx) {
            const int xx = x + dx - 1;
            r.ok[dx] = yy >= 0 && yy < H && xx >= 0 && xx < W;
            r.v[dx] = u32x4{0u, 0u, 0u, 0u};
            if (r.ok[dx]) r.v[dx] = *(const u32x4*)(img + ((long)yy * W + xx) * E);
        }
    };
    auto unpack_row = [&](const Raw& r, float (&row)[3][V]) {
#pragma unroll
        for (int dx = 0; dx < 3; ++dx) {
            float f[V];
            Pack<T>::unpack(r.v[dx], f);
#pragma unroll
            for (int j = 0; j < V; ++j) row[dx][j] = f[j];        // (a masked load is zero: the padding)
        }
    };
    Raw ahead;
    request(y0 - 1, ahead);
    unpack_row(ahead, win[0]);
    request(y0, ahead);
    unpack_row(ahead, win[1]);
    request(y0 + 1, ahead);
#pragma unroll
    for (int r = 0; r < kDwRows; ++r) {
        const int yy = y0 + r;
        unpack_row(ahead, win[(r + 2) % 3]);           // row yy + 1
        if (r + 1 < kDwRows) request(yy + 2, ahead);   // in flight during this row's arithmetic
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

}  // namespace msla
