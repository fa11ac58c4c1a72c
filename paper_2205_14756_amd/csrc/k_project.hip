// 1x1 projections  y[n, o] = sum_c x[n, c] * w[o, c]  (Section 3.1: Q = x W_Q,
// K = x W_K, V = x W_V; also the stand-alone form of the final projection).
// A tile is 128 tokens x 256 output channels, computed by 8 waves.
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

// Where the projection writes, and in which order it walks the weight rows.
template <class T>
struct PlainDest {
    T* y;
    long ld;
    __device__ __forceinline__ int row_of(int oc) const { return oc; }
    __device__ __forceinline__ T* operator()(long tok, int oc) const { return y + tok * ld + oc; }
};

// Q/K/V projection with split destinations.  The kernel walks the output channels in DESTINATION
// order -- first the Ct channels of Q (head-major), then the 2*Ct channels of K|V as they lie in
// kv_raw -- so a tile's channels of one token are one contiguous run in memory; row_of maps such a
// channel to its row (h*3 + t)*16 + e of w_qkv.
template <class T>
struct QkvSplitDest {
    T* q_ms;
    long q_ms_stride;
    T* kv_raw;
    long kv_stride;
    int Ct;
    __device__ __forceinline__ int row_of(int vc) const {
        if (vc < Ct) return (vc >> 4) * 48 + (vc & 15);
        const int v2 = vc - Ct;
        return (v2 >> 5) * 48 + 16 + (v2 & 31);
    }
    __device__ __forceinline__ T* operator()(long tok, int vc) const {
        return vc < Ct ? q_ms + tok * q_ms_stride + vc : kv_raw + tok * kv_stride + (vc - Ct);
    }
};

// Persistent workgroups: each takes a contiguous run of (token tile, channel block) tiles, channel
// block fastest, so the token tile it re-reads for the next channel block is still in its CU's
// cache, and consecutive workgroups (= one XCD, see xcd_remap) share the weights in one L2.
// The (tile, 128-byte contraction slab) pairs form one flat software pipeline over two LDS
// buffers: while the matrix cores work on slab g, the loads of slab g+1 -- the first slab of the
// next tile included -- are in flight into registers, and are parked in the other buffer before the
// single barrier of the step.  The epilogue's stores are not waited for, so they drain while the
// next tile is computed.
template <class T, class Epilogue>
__global__ __launch_bounds__(ProjTile<T>::kThreads) void project_kernel(const T* __restrict__ x, const T* __restrict__ w,
                                                      long n_tokens, int c_in, int c_out, int n_rb,
                                                      long n_tiles, long per, Epilogue ep) {
    typedef ProjTile<T> G;
    constexpr int kBuf = G::kLdsR + G::kLdsC;
    extern __shared__ __attribute__((aligned(16))) char lds[];

    const unsigned L = xcd_remap(blockIdx.x, gridDim.x);
    const long tile_begin = (long)L * per;
    const long tile_end = tile_begin + per < n_tiles ? tile_begin + per : n_tiles;
    if (tile_begin >= tile_end) return;
    const int wave = threadIdx.x >> 6;
    const int wr = wave % MSLA_PROJ_WR, wc = wave / MSLA_PROJ_WR;
    const int slabs = (c_in + G::BK - 1) / G::BK;

    f32x4 acc[4][4];
    G::zero(acc);
    u32x4 rw[G::kVecR], rx[G::kVecC];

    long tile = tile_begin;          // tile / slab being computed
    int slab = 0;
    long ntile = tile_begin;         // tile / slab being fetched
    int nslab = 0;
    auto fetch = [&]() {
        const int oc0 = (int)(ntile % n_rb) * G::BR;
        const long tok0 = (ntile / n_rb) * G::BC;
        G::load_global_rows(rw, w, oc0, c_out, c_in, nslab * G::BK, c_in,
                            [&ep](int r) { return ep.row_of(r); });
        G::load_global(rx, x, tok0, n_tokens, c_in, nslab * G::BK, c_in);
        if (++nslab == slabs) { nslab = 0; ++ntile; }
    };
    fetch();
    G::store_lds(lds, rw);
    G::store_lds(lds + G::kLdsR, rx);
    __syncthreads();
    int cur = 0;
    while (tile < tile_end) {
        const bool more = ntile < tile_end;
        if (more) fetch();
        G::mma(acc, lds + cur * kBuf, lds + cur * kBuf + G::kLdsR, wr, wc);
        if (more) {
            G::store_lds(lds + (cur ^ 1) * kBuf, rw);
            G::store_lds(lds + (cur ^ 1) * kBuf + G::kLdsR, rx);
        }
        __syncthreads();
        cur ^= 1;
        if (++slab == slabs) {
            // the buffer just consumed is free until the end of the next step: stage the results there
            G::epilogue_lds(acc, lds + (cur ^ 1) * kBuf, (tile / n_rb) * G::BC, n_tokens,
                            (int)(tile % n_rb) * G::BR, c_out, wr, wc, ep);
            G::zero(acc);
            slab = 0;
            ++tile;
            __syncthreads();     // nobody refills that buffer while a wave still stages in it
        }
    }
}

template <class T, class Epilogue>
hipError_t run_project(const void* x, const void* w, long n_tokens, int c_in, int c_out, Epilogue ep,
                       hipStream_t stream) {
    typedef ProjTile<T> G;
    const int n_rb = (c_out + G::BR - 1) / G::BR;
    const long n_cb = (n_tokens + G::BC - 1) / G::BC;
    const long n_tiles = n_cb * n_rb;
    if (n_tiles <= 0 || n_tiles > 0x7fffffffL) return hipErrorInvalidValue;
    // one resident workgroup per CU (two LDS buffers of 55 KB); whole channel-block groups per workgroup
    const long cus = compute_units();
    long per = (n_tiles + cus - 1) / cus;
    per = (per + n_rb - 1) / n_rb * n_rb;
    const long nblocks = (n_tiles + per - 1) / per;
    constexpr int kLds = 2 * (G::kLdsR + G::kLdsC);
    const hipError_t e = hipFuncSetAttribute((const void*)project_kernel<T, Epilogue>,
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((project_kernel<T, Epilogue>), dim3((unsigned)nblocks), dim3(G::kThreads), kLds, stream,
                       (const T*)x, (const T*)w, n_tokens, c_in, c_out, n_rb, n_tiles, per, ep);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_linear(int dt, const void* x, const void* w, void* y, long n_tokens, int c_in, int c_out,
                         hipStream_t stream) {
    switch (dt) {
        case 0: return run_project<float>(x, w, n_tokens, c_in, c_out, PlainDest<float>{(float*)y, c_out}, stream);
        case 1: return run_project<_Float16>(x, w, n_tokens, c_in, c_out, PlainDest<_Float16>{(_Float16*)y, c_out}, stream);
        case 2: return run_project<__bf16>(x, w, n_tokens, c_in, c_out, PlainDest<__bf16>{(__bf16*)y, c_out}, stream);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_qkv_project(int dt, const void* x, const void* w_qkv, void* q_ms, long q_ms_stride,
                              void* kv_raw, long n_tokens, int c_in, int heads, hipStream_t stream) {
    const int c_out = 3 * heads * 16;
    const long kv_stride = 2L * heads * 16;
    switch (dt) {
        case 0: return run_project<float>(x, w_qkv, n_tokens, c_in, c_out,
                    QkvSplitDest<float>{(float*)q_ms, q_ms_stride, (float*)kv_raw, kv_stride, heads * 16}, stream);
        case 1: return run_project<_Float16>(x, w_qkv, n_tokens, c_in, c_out,
                    QkvSplitDest<_Float16>{(_Float16*)q_ms, q_ms_stride, (_Float16*)kv_raw, kv_stride, heads * 16}, stream);
        case 2: return run_project<__bf16>(x, w_qkv, n_tokens, c_in, c_out,
                    QkvSplitDest<__bf16>{(__bf16*)q_ms, q_ms_stride, (__bf16*)kv_raw, kv_stride, heads * 16}, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace msla
