// Per-token normalise-and-apply of Eq. (3), last line:
//   att[n, m*16 + f] = relu(Q_n) . KV[:, f] / (relu(Q_n) . KV[:, 16] + eps)
// for every head-branch m = s*heads + h of the multi-scale Q map, either
// written out (the module without projections) or fed straight into the final
// 1x1 projection of the concatenated heads (Section 3.1, last sentence) so the
// attention map never reaches HBM.
//
// A 16-token x one-head-branch unit is two MFMAs: the state is the row operand
// (prepared by the finalize kernel, hi and lo halves stacked along the
// contraction for the 16-bit types), relu(Q) the column operand.  The second
// MFMA uses a row operand whose 16 rows all equal Ksum, so every lane gets the
// denominator of its own token without a shuffle.  The result has 4
// consecutive channels of one token per lane.
#include "gemm_tile.h"
#include "msla_kernels.h"

#ifndef MSLA_APPLY_WR
#define MSLA_APPLY_WR 4
#define MSLA_APPLY_WC 2
#endif

namespace msla {
namespace {

template <class T>
using ApplyTile = GemmTile<T, MSLA_APPLY_WR, MSLA_APPLY_WC>;

// q: channels 4q..4q+3 of this lane's token (raw, not yet rectified).
// state: the 2048-byte operand block of (image, head-branch).  eps_s = eps * scale.
template <class T>
__device__ __forceinline__ f32x4 att_unit(typename Traits<T>::Frag qf, const char* state, float eps_s) {
    typedef Traits<T> Tr;
    const int lane = lane_id();
    const f32x4 z = {0.f, 0.f, 0.f, 0.f};
    qf = frag_relu<T>(qf);
    f32x4 num, den;
    if constexpr (Tr::kSplit) {
        typedef typename Tr::Vec Vec;
        const Vec a_kv = __builtin_bit_cast(Vec, *(const u32x4*)(state + lane * 16));
        const Vec a_ks = __builtin_bit_cast(Vec, *(const u32x4*)(state + 1024 + lane * 16));
        Vec b;
#pragma unroll
        for (int r = 0; r < 4; ++r) { b[r] = qf[r]; b[4 + r] = qf[r]; }   // pairs with {hi, lo}
        num = Tr::mma_vec(z, a_kv, b);
        den = Tr::mma_vec(z, a_ks, b);
    } else {
        const f32x4 a_kv = *(const f32x4*)(state + lane * 16);
        const f32x4 a_ks = *(const f32x4*)(state + 1024 + lane * 16);
        num = Tr::mma16(z, a_kv, qf);
        den = Tr::mma16(z, a_ks, qf);
    }
    const float inv = 1.0f / (den[0] + eps_s);
    return f32x4{num[0] * inv, num[1] * inv, num[2] * inv, num[3] * inv};
}

// ------------------------------------------------------------------ att only
// One wave per 16-token group of one image; it walks over the head-branches.
template <class T>
__global__ __launch_bounds__(256) void apply_kernel(const T* __restrict__ q_ms, const char* __restrict__ kvfrag,
                                                    const float* __restrict__ kvscale, T* __restrict__ att,
                                                    int N, int n_hb, int groups_per_image, long n_groups,
                                                    float eps) {
    const int wave = threadIdx.x >> 6;
    const int x16 = lane_id() & 15, q = lane_id() >> 4;
    const long g = (long)blockIdx.x * 4 + wave;
    if (g >= n_groups) return;
    const int b = (int)(g / groups_per_image);
    const int n = (int)(g % groups_per_image) * 16 + x16;
    const bool ok = n < N;
    const long ld = (long)n_hb * 16;
    const long row = ((long)b * N + n) * ld;
    for (int m = 0; m < n_hb; ++m) {
        typename Traits<T>::Frag qf = frag_zero<T>();
        if (ok) qf = load_frag<T>(q_ms + row + m * 16 + q * 4);
        const long sid = (long)b * n_hb + m;
        const f32x4 o = att_unit<T>(qf, kvfrag + sid * 2048, eps * kvscale[sid]);
        if (ok) store_frag<T>(att + row + m * 16 + q * 4, frag_from_f32<T>(o));
    }
}

// ------------------------------------------------- att fused into projection
// 128 tokens of one image x 256 output channels per workgroup, 8 waves.  Each
// iteration covers 128 contraction bytes = BK/16 head-branches; wave w makes
// the attention rows of token group w for them and writes them to the token
// tile in LDS while the weight tile arrives from the previous iteration's
// prefetch.  For bf16 the attention rows go to LDS as a hi and a lo tile (two
// MFMA passes), since 8 significant bits would cost half the error budget.
template <class T>
__global__ __launch_bounds__(ApplyTile<T>::kThreads) void apply_project_kernel(const T* __restrict__ q_ms,
                                                            const char* __restrict__ kvfrag,
                                                            const float* __restrict__ kvscale,
                                                            const T* __restrict__ w_proj, T* __restrict__ out,
                                                            int N, int n_hb, int c_out, int blocks_per_image,
                                                            int n_rb, float eps) {
    typedef ApplyTile<T> G;
    typedef typename Traits<T>::Frag Frag;
    constexpr int HB = G::BK / 16;   // head-branches per iteration
    constexpr int kWaves = G::kThreads / 64;
    constexpr int TG = (G::BC / 16) / kWaves;   // 16-token groups per wave for the attention rows
    static_assert(TG >= 1 && TG * kWaves * 16 == G::BC, "token groups must divide over the waves");
    constexpr bool kHiLo = Traits<T>::kHiLo;
    extern __shared__ __attribute__((aligned(16))) char lds[];
    char* ldsR = lds;
    char* ldsC = lds + G::kLdsR;
    char* ldsC_lo = ldsC + G::kLdsC;   // only with kHiLo

    const unsigned L = xcd_remap(blockIdx.x, gridDim.x);
    const int rb = L % n_rb;
    const unsigned tb = L / n_rb;
    const int b = tb / blocks_per_image;
    const int n0 = (tb % blocks_per_image) * G::BC;
    const int oc0 = rb * G::BR;
    const int wave = threadIdx.x >> 6;
    const int wr = wave % MSLA_APPLY_WR, wc = wave / MSLA_APPLY_WR;
    const int x16 = lane_id() & 15, q = lane_id() >> 4;
    const int K = n_hb * 16;

    // this lane's tokens for the attention rows: token groups wave, wave + kWaves, ...
    bool ok[TG];
    const T* q_row[TG];
#pragma unroll
    for (int g = 0; g < TG; ++g) {
        const int n_mine = n0 + (g * kWaves + wave) * 16 + x16;
        ok[g] = n_mine < N;
        q_row[g] = q_ms + ((long)b * N + n_mine) * K + q * 4;
    }
    const long sid0 = (long)b * n_hb;

    f32x4 acc[4][4];
    G::zero(acc);
    u32x4 rw[G::kVecR];
    Frag qreg[TG][HB];
    G::load_global(rw, w_proj, oc0, c_out, K, 0, K);
#pragma unroll
    for (int g = 0; g < TG; ++g)
#pragma unroll
        for (int j = 0; j < HB; ++j)
            qreg[g][j] = (ok[g] && j < n_hb) ? load_frag<T>(q_row[g] + j * 16) : frag_zero<T>();

    for (int k0 = 0; k0 < K; k0 += G::BK) {
        G::store_lds_r(ldsR, rw);
        const int m0 = k0 >> 4;
#pragma unroll
        for (int j = 0; j < HB; ++j) {
            const bool live = m0 + j < n_hb;
            const char* state = kvfrag + (sid0 + m0 + j) * 2048;
            const float eps_s = live ? eps * kvscale[sid0 + m0 + j] : 0.f;
#pragma unroll
            for (int g = 0; g < TG; ++g) {
                f32x4 o = {0.f, 0.f, 0.f, 0.f};
                if (live) o = att_unit<T>(qreg[g][j], state, eps_s);
                const int colb = (j * 16 + q * 4) * (int)sizeof(T);      // byte column inside the 128-byte slab
                const int off = ((g * kWaves + wave) * 16 + x16) * G::kRow + colb;
                if constexpr (kHiLo) {
                    Frag hi, lo;
                    frag_split<T>(o, hi, lo);
                    store_frag<T>(ldsC + off, hi);
                    store_frag<T>(ldsC_lo + off, lo);
                } else {
                    store_frag<T>(ldsC + off, frag_from_f32<T>(o));
                }
            }
        }
        __syncthreads();
        if (k0 + G::BK < K) {
            G::load_global(rw, w_proj, oc0, c_out, K, k0 + G::BK, K);
            const int m1 = m0 + HB;
#pragma unroll
            for (int g = 0; g < TG; ++g)
#pragma unroll
                for (int j = 0; j < HB; ++j)
                    qreg[g][j] = (ok[g] && m1 + j < n_hb) ? load_frag<T>(q_row[g] + (m1 + j) * 16) : frag_zero<T>();
        }
        G::mma(acc, ldsR, ldsC, wr, wc);
        if constexpr (kHiLo) G::mma(acc, ldsR, ldsC_lo, wr, wc);
        __syncthreads();
    }
    const long tok0 = (long)b * N + n0;
    G::epilogue(acc, tok0, (long)b * N + N, oc0, c_out, wr, wc,
                [out, c_out](long tok, int oc, f32x4 v) { store_frag<T>(out + tok * c_out + oc, frag_from_f32<T>(v)); });
}

template <class T>
hipError_t run_apply(const void* q_ms, const void* kvfrag, const float* kvscale, void* att, long n_tokens,
                     int N, int n_hb, float eps, hipStream_t stream) {
    const int gpi = (N + 15) / 16;
    const long n_groups = (n_tokens / N) * gpi;
    const long nblocks = (n_groups + 3) / 4;
    if (nblocks <= 0 || nblocks > 0x7fffffffL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((apply_kernel<T>), dim3((unsigned)nblocks), dim3(256), 0, stream, (const T*)q_ms,
                       (const char*)kvfrag, kvscale, (T*)att, N, n_hb, gpi, n_groups, eps);
    return hipGetLastError();
}

template <class T>
hipError_t run_apply_project(const void* q_ms, const void* kvfrag, const float* kvscale, const void* w_proj,
                             void* out, long n_tokens, int N, int n_hb, int c_out, float eps,
                             hipStream_t stream) {
    typedef ApplyTile<T> G;
    const int bpi = (N + G::BC - 1) / G::BC;
    const int n_rb = (c_out + G::BR - 1) / G::BR;
    const long nblocks = (n_tokens / N) * bpi * n_rb;
    if (nblocks <= 0 || nblocks > 0x7fffffffL) return hipErrorInvalidValue;
    constexpr int kLds = G::kLdsR + G::kLdsC * (Traits<T>::kHiLo ? 2 : 1);
    if (kLds > 48 * 1024) {   // above the default dynamic-LDS limit (the CU has 160 KB)
        const hipError_t e = hipFuncSetAttribute((const void*)apply_project_kernel<T>,
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((apply_project_kernel<T>), dim3((unsigned)nblocks), dim3(G::kThreads), kLds, stream,
                       (const T*)q_ms, (const char*)kvfrag, kvscale, (const T*)w_proj, (T*)out, N, n_hb, c_out,
                       bpi, n_rb, eps);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_apply(int dt, const void* q_ms, const void* kvfrag, const float* kvscale, void* att,
                        long n_tokens, int tokens_per_image, int n_hb, float eps, hipStream_t stream) {
    switch (dt) {
        case 0: return run_apply<float>(q_ms, kvfrag, kvscale, att, n_tokens, tokens_per_image, n_hb, eps, stream);
        case 1: return run_apply<_Float16>(q_ms, kvfrag, kvscale, att, n_tokens, tokens_per_image, n_hb, eps, stream);
        case 2: return run_apply<__bf16>(q_ms, kvfrag, kvscale, att, n_tokens, tokens_per_image, n_hb, eps, stream);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_apply_project(int dt, const void* q_ms, const void* kvfrag, const float* kvscale,
                                const void* w_proj, void* out, long n_tokens, int tokens_per_image, int n_hb,
                                int c_out, float eps, hipStream_t stream) {
    switch (dt) {
        case 0: return run_apply_project<float>(q_ms, kvfrag, kvscale, w_proj, out, n_tokens, tokens_per_image, n_hb, c_out, eps, stream);
        case 1: return run_apply_project<_Float16>(q_ms, kvfrag, kvscale, w_proj, out, n_tokens, tokens_per_image, n_hb, c_out, eps, stream);
        case 2: return run_apply_project<__bf16>(q_ms, kvfrag, kvscale, w_proj, out, n_tokens, tokens_per_image, n_hb, c_out, eps, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace msla
