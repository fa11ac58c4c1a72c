// 1x1 projections  y[n, o] = sum_c x[n, c] * w[o, c]  (Section 3.1: Q = x W_Q,
// K = x W_K, V = x W_V; also the stand-alone form of the final projection).
// One workgroup computes 128 tokens x 256 output channels with 8 waves.
#include "gemm_tile.h"
#include "msla_kernels.h"

#ifndef MSLA_PROJ_WR
#define MSLA_PROJ_WR 4
#define MSLA_PROJ_WC 2
#endif

namespace msla {
namespace {

template <class T>
using ProjTile = GemmTile<T, MSLA_PROJ_WR, MSLA_PROJ_WC>;

template <class T>
struct PlainStore {
    T* y;
    long ld;
    __device__ __forceinline__ void operator()(long tok, int oc, f32x4 v) const {
        store_frag<T>(y + tok * ld + oc, frag_from_f32<T>(v));
    }
};

// Output channel o = (h*3 + t)*16 + e; a 4-channel group never straddles a (h, t) block.
template <class T>
struct QkvSplitStore {
    T* q_ms;
    long q_ms_stride;
    T* kv_raw;
    long kv_stride;
    __device__ __forceinline__ void operator()(long tok, int oc, f32x4 v) const {
        const int g = oc >> 4, e = oc & 15;
        const int h = g / 3, t = g - 3 * h;
        T* dst = (t == 0) ? q_ms + tok * q_ms_stride + h * 16 + e
                          : kv_raw + tok * kv_stride + h * 32 + (t - 1) * 16 + e;
        store_frag<T>(dst, frag_from_f32<T>(v));
    }
};

template <class T, class Epilogue>
__global__ __launch_bounds__(ProjTile<T>::kThreads) void project_kernel(const T* __restrict__ x, const T* __restrict__ w,
                                                      long n_tokens, int c_in, int c_out, int n_rb,
                                                      Epilogue ep) {
    typedef ProjTile<T> G;
    __shared__ __attribute__((aligned(16))) char lds[G::kLdsR + G::kLdsC];
    char* ldsR = lds;
    char* ldsC = lds + G::kLdsR;

    const unsigned L = xcd_remap(blockIdx.x, gridDim.x);
    const int rb = L % n_rb;                 // output-channel block: fastest, so the
    const long cb = L / n_rb;                // blocks that share a token tile are neighbours
    const int oc0 = rb * G::BR;
    const long tok0 = cb * G::BC;
    const int wave = threadIdx.x >> 6;
    const int wr = wave % MSLA_PROJ_WR, wc = wave / MSLA_PROJ_WR;

    f32x4 acc[4][4];
    G::zero(acc);
    u32x4 rw[G::kVecR], rx[G::kVecC];
    G::load_global(rw, w, oc0, c_out, c_in, 0, c_in);
    G::load_global(rx, x, tok0, n_tokens, c_in, 0, c_in);
    for (int k0 = 0; k0 < c_in; k0 += G::BK) {
        G::store_lds(ldsR, rw);
        G::store_lds(ldsC, rx);
        __syncthreads();
        if (k0 + G::BK < c_in) {
            G::load_global(rw, w, oc0, c_out, c_in, k0 + G::BK, c_in);
            G::load_global(rx, x, tok0, n_tokens, c_in, k0 + G::BK, c_in);
        }
        G::mma(acc, ldsR, ldsC, wr, wc);
        __syncthreads();
    }
    G::epilogue(acc, tok0, n_tokens, oc0, c_out, wr, wc, ep);
}

template <class T, class Epilogue>
hipError_t run_project(const void* x, const void* w, long n_tokens, int c_in, int c_out, Epilogue ep,
                       hipStream_t stream) {
    typedef ProjTile<T> G;
    const int n_rb = (c_out + G::BR - 1) / G::BR;
    const long n_cb = (n_tokens + G::BC - 1) / G::BC;
    const long nblocks = n_cb * n_rb;
    if (nblocks <= 0 || nblocks > 0x7fffffffL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((project_kernel<T, Epilogue>), dim3((unsigned)nblocks), dim3(G::kThreads), 0, stream,
                       (const T*)x, (const T*)w, n_tokens, c_in, c_out, n_rb, ep);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_linear(int dt, const void* x, const void* w, void* y, long n_tokens, int c_in, int c_out,
                         hipStream_t stream) {
    switch (dt) {
        case 0: return run_project<float>(x, w, n_tokens, c_in, c_out, PlainStore<float>{(float*)y, c_out}, stream);
        case 1: return run_project<_Float16>(x, w, n_tokens, c_in, c_out, PlainStore<_Float16>{(_Float16*)y, c_out}, stream);
        case 2: return run_project<__bf16>(x, w, n_tokens, c_in, c_out, PlainStore<__bf16>{(__bf16*)y, c_out}, stream);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_qkv_project(int dt, const void* x, const void* w_qkv, void* q_ms, long q_ms_stride,
                              void* kv_raw, long n_tokens, int c_in, int heads, hipStream_t stream) {
    const int c_out = 3 * heads * 16;
    const long kv_stride = 2L * heads * 16;
    switch (dt) {
        case 0: return run_project<float>(x, w_qkv, n_tokens, c_in, c_out,
                    QkvSplitStore<float>{(float*)q_ms, q_ms_stride, (float*)kv_raw, kv_stride}, stream);
        case 1: return run_project<_Float16>(x, w_qkv, n_tokens, c_in, c_out,
                    QkvSplitStore<_Float16>{(_Float16*)q_ms, q_ms_stride, (_Float16*)kv_raw, kv_stride}, stream);
        case 2: return run_project<__bf16>(x, w_qkv, n_tokens, c_in, c_out,
                    QkvSplitStore<__bf16>{(__bf16*)q_ms, q_ms_stride, (__bf16*)kv_raw, kv_stride}, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace msla
