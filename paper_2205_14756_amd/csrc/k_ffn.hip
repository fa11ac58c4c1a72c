// The FFN+DWConv half of the EfficientViT building block (Section 3.1: a depthwise convolution is
// inserted into the FFN layer that follows the attention module; Fig. 2 left).  Declared reading (the paper prints no more than the sentence above):
//   h   = act(W1 y)                      1x1 expand, C -> E
//   g   = act(DW3x3(h))                  depthwise 3x3, stride 1, zero padding 1, cross-correlation
//   out = y + W2 g                       1x1 project, E -> C, no activation, residual
// with act = ReLU or hard-swish, no bias, no normalisation.
//
// Two launches: the expand projection is the library's 1x1 projection kernel with the activation
// applied to its fp32 sums; the kernel here does the rest -- depthwise 3x3, activation, the hidden -> C
// projection and the residual -- with the depthwise result produced on chip as the projection's token
// operand.  The block's y = x + MSLA(x) is formed in the epilogue of the attention module's output
// projection.
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

// out = res + act(DW3x3(h)) W2^T in ONE kernel: the depthwise result is made slab by slab where the
// projection needs it -- as the token operand of its matrix instructions -- and never reaches memory.
// A workgroup owns a 4 x 32-token block of one image and 256 output channels (8 waves of 64 x 64).  Per
// slab of BK hidden channels: the block's 6 x 34 halo of h and the weight slab go HBM -> registers -> LDS
// (requested during the previous slab's arithmetic); thread (column, 16-byte channel vector, upper or
// lower row pair) slides over its 4 halo rows x 3 columns and writes two tokens' activated sums into
// the token tile; then 32 MFMAs per wave.  The residual joins the fp32 sums in the LDS-staged epilogue.
template <class T, int ACT>
__global__ __launch_bounds__(512) void ffn_dw_project_kernel(const T* __restrict__ h, const T* __restrict__ w_dw,
                                                            const T* __restrict__ w2, const T* __restrict__ res,
                                                            T* __restrict__ out, int H, int W, int E, int c_out,
                                                            int tiles_x, int tiles_y, int n_rb) {
    typedef GemmTile<T, 4, 2> G;
    constexpr int V = Pack<T>::N;                 // channels per 16-byte vector
    constexpr int kVecSlab = G::BK / V;           // 8 vectors per token and slab
    constexpr int kHaloW = 34, kHaloH = 6, kHaloTok = kHaloW * kHaloH;
    constexpr int kHaloRow = 160;                 // bytes per halo token in LDS (128 + padding)
    constexpr int kHaloVec = (kHaloTok * kVecSlab + 511) / 512;
    extern __shared__ __attribute__((aligned(16))) char lds[];
    char* ldsR = lds;
    char* ldsC = lds + G::kLdsR;
    char* halo = ldsC + G::kLdsC;
    float* taps = (float*)(halo + kHaloTok * kHaloRow);      // [9][BK] fp32: the slab's filter taps

    const unsigned L = xcd_remap(blockIdx.x, gridDim.x);
    const int rb = L % n_rb;
    unsigned rest = L / n_rb;
    const int tx = rest % tiles_x;
    rest /= tiles_x;
    const int ty = rest % tiles_y;
    const int b = rest / tiles_y;
    const int y0 = ty * 4, x0 = tx * 32, oc0 = rb * G::BR;
    const T* img = h + (long)b * H * W * E;
    const int wave = threadIdx.x >> 6, wr = wave % 4, wc = wave / 4;

    // this thread's part of the depthwise pass: tile column, channel vector, row pair
    const int dvec = threadIdx.x & 7, dcol = (threadIdx.x >> 3) & 31, dhalf = threadIdx.x >> 8;

    f32x4 acc[4][4];
    G::zero(acc);
    u32x4 rw[G::kVecR], rh[kHaloVec], rt = {0u, 0u, 0u, 0u};
    // the slab's taps are BK*9 consecutive elements of w_dw: 16 bytes a thread for the first few threads
    constexpr int kTapVec = G::BK * 9 / V;
    auto fetch = [&](int k0) {
        G::load_global(rw, w2, oc0, c_out, E, k0, E);
        if (threadIdx.x < kTapVec && (long)k0 * 9 + (threadIdx.x + 1) * V <= (long)E * 9)
            rt = *(const u32x4*)(w_dw + (long)k0 * 9 + threadIdx.x * V);
#pragma unroll
        for (int i = 0; i < kHaloVec; ++i) {
            const int id = i * 512 + threadIdx.x;
            const int tok = id / kVecSlab, v = id - tok * kVecSlab;
            const int hy = tok / kHaloW, hx = tok - hy * kHaloW;
            const int yy = y0 - 1 + hy, xx = x0 - 1 + hx;
            u32x4 val = {0u, 0u, 0u, 0u};
            if (tok < kHaloTok && yy >= 0 && yy < H && xx >= 0 && xx < W && k0 + v * V < E)
                val = *(const u32x4*)(img + ((long)yy * W + xx) * E + k0 + v * V);
            rh[i] = val;
        }
    };
    auto park = [&]() {
        G::store_lds_r(ldsR, rw);
#pragma unroll
        for (int i = 0; i < kHaloVec; ++i) {
            const int id = i * 512 + threadIdx.x;
            const int tok = id / kVecSlab, v = id - tok * kVecSlab;
            if (tok < kHaloTok) *(u32x4*)(halo + tok * kHaloRow + v * 16) = rh[i];
        }
        if (threadIdx.x < kTapVec) {
            float f[V];
            Pack<T>::unpack(rt, f);
#pragma unroll
            for (int j = 0; j < V; ++j) {
                const int i = threadIdx.x * V + j;          // element (channel i / 9, tap i % 9) of the slab
                taps[(i % 9) * G::BK + i / 9] = f[j];
            }
        }
    };
    fetch(0);
    for (int k0 = 0; k0 < E; k0 += G::BK) {
        park();
        __syncthreads();
        if (k0 + G::BK < E) fetch(k0 + G::BK);
        float wt[9][V];
#pragma unroll
        for (int t = 0; t < 9; ++t)
#pragma unroll
            for (int j4 = 0; j4 < V; j4 += 4) {
                const f32x4 w4 = *(const f32x4*)(taps + t * G::BK + dvec * V + j4);
#pragma unroll
                for (int j = 0; j < 4; ++j) wt[t][j4 + j] = w4[j];
            }
        // ---- depthwise 3x3 + activation for tokens (2*dhalf, dcol) and (2*dhalf + 1, dcol)
        {
            float a0[V], a1[V];
#pragma unroll
            for (int j = 0; j < V; ++j) a0[j] = a1[j] = 0.f;
#pragma unroll
            for (int r = 0; r < 4; ++r) {            // halo rows 2*dhalf + r
#pragma unroll
                for (int dx = 0; dx < 3; ++dx) {
                    float f[V];
                    Pack<T>::unpack(*(const u32x4*)(halo + ((2 * dhalf + r) * kHaloW + dcol + dx) * kHaloRow + dvec * 16), f);
#pragma unroll
                    for (int j = 0; j < V; ++j) {
                        if (r < 3) a0[j] = fmaf(wt[r * 3 + dx][j], f[j], a0[j]);            // output row 2*dhalf: taps u = r
                        if (r > 0) a1[j] = fmaf(wt[(r - 1) * 3 + dx][j], f[j], a1[j]);      // output row 2*dhalf + 1: u = r - 1
                    }
                }
            }
#pragma unroll
            for (int j = 0; j < V; ++j) {
                a0[j] = activate<ACT>(a0[j]);
                a1[j] = activate<ACT>(a1[j]);
            }
            *(u32x4*)(ldsC + ((2 * dhalf) * 32 + dcol) * G::kRow + dvec * 16) = Pack<T>::pack(a0);
            *(u32x4*)(ldsC + ((2 * dhalf + 1) * 32 + dcol) * G::kRow + dvec * 16) = Pack<T>::pack(a1);
        }
        __syncthreads();
        G::mma(acc, ldsR, ldsC, wr, wc);
        __syncthreads();
    }
    // ---- results: tile token t = (row t / 32, column t % 32) of the block
    struct TileOut {
        T* out;
        long base;      // token index of (y0, x0)
        int W, rows, cols, c_out;
        __device__ __forceinline__ void store(int, int, int trow, int oc, u32x4 v) const {
            const int r = trow >> 5, c = trow & 31;
            if (r < rows && c < cols && oc < c_out) *(u32x4*)(out + (base + (long)r * W + c) * c_out + oc) = v;
        }
    };
    const long base = ((long)b * H + y0) * W + x0;
    const int rows = H - y0 < 4 ? H - y0 : 4, cols = W - x0 < 32 ? W - x0 : 32;
    const TileOut to{out, base, W, rows, cols, c_out};
    G::epilogue_lds_residual(acc, lds, oc0, wr, wc, to, [&](int trow, int oc) {
        const int r = trow >> 5, c = trow & 31;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (r < rows && c < cols && oc < c_out) v = *(const u32x4*)(res + (base + (long)r * W + c) * c_out + oc);
        return v;
    });
}

template <class T>
hipError_t run_dw_project(const void* h, const void* w_dw, const void* w2, const void* res, void* out, int B, int H, int W,
                          int E, int c_out, int act, hipStream_t stream) {
    typedef GemmTile<T, 4, 2> G;
    const int tiles_x = (W + 31) / 32, tiles_y = (H + 3) / 4;
    const int n_rb = (c_out + G::BR - 1) / G::BR;
    const long nblocks = (long)B * tiles_x * tiles_y * n_rb;
    if (nblocks <= 0 || nblocks > 0x7fffffffL) return hipErrorInvalidValue;
    constexpr int kLds = G::kLdsR + G::kLdsC + 204 * 160 + 9 * G::BK * 4;
    static_assert(G::kStageResBytes <= G::kLdsR + G::kLdsC, "the epilogue stages in the operand tiles");
    hipError_t e;
    if (act == 0) {
        e = allow_dynamic_lds<ffn_dw_project_kernel<T, 0>>(kLds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((ffn_dw_project_kernel<T, 0>), dim3((unsigned)nblocks), dim3(512), kLds, stream, (const T*)h,
                           (const T*)w_dw, (const T*)w2, (const T*)res, (T*)out, H, W, E, c_out, tiles_x, tiles_y, n_rb);
    } else {
        e = allow_dynamic_lds<ffn_dw_project_kernel<T, 1>>(kLds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((ffn_dw_project_kernel<T, 1>), dim3((unsigned)nblocks), dim3(512), kLds, stream, (const T*)h,
                           (const T*)w_dw, (const T*)w2, (const T*)res, (T*)out, H, W, E, c_out, tiles_x, tiles_y, n_rb);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_ffn_dw_project(int dt, const void* h, const void* w_dw, const void* w2, const void* res, void* out, int B,
                                 int H, int W, int E, int c_out, int act, hipStream_t stream) {
    switch (dt) {
        case 0: return run_dw_project<float>(h, w_dw, w2, res, out, B, H, W, E, c_out, act, stream);
        case 1: return run_dw_project<_Float16>(h, w_dw, w2, res, out, B, H, W, E, c_out, act, stream);
        case 2: return run_dw_project<__bf16>(h, w_dw, w2, res, out, B, H, W, E, c_out, act, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace msla
