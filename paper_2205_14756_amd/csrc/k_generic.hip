// The module for head sizes other than 16 (Section 3.1 fixes only "d channels per group"; 8 and 32 are
// the other sizes the architecture family uses).
//
// Head size 32.  fp32 storage: multi-scale aggregation and the Eq. (3) state as plain vector-ALU kernels
// templated on the head size D, following the definitions step by step with fp32 sums throughout (16-bit
// storage takes the tiled matrix-core kernel of k_aggregate32.hip instead); all types: the fixed-order sum of
// the partial states and the normalise-and-apply pass below.  The same storage points as the head-size-16
// path: projected Q/K/V and the Q tokens of every branch are stored in the storage type; aggregated K and V
// only feed the state.
//
//   generic_branch_state_kernel   one branch (raw, or depthwise k x k + grouped 1x1) of one (image, head,
//                                 chunk of 64-token groups): writes that branch's Q tokens, accumulates
//                                 KV = sum_n relu(K_n)^T [V_n, 1] into a per-workgroup partial state
//   generic_state_finalize_kernel fixed-order sum of the partial states
//   generic_apply_kernel          att_n = relu(Q_n) KV[:, :D] / (relu(Q_n) KV[:, D] + eps), on the matrix cores in fp32
//
// Head size 8 needs no kernels of its own: two heads side by side are one head of 16 whose grouped 1x1 is
// block-diagonal and whose state is used block by block (pair_head8_weights_kernel arranges the weights
// that way; the finalize step of the head-size-16 path masks the state operands).
#include <type_traits>

#include "msla_device.h"
#include "msla_kernels.h"

namespace msla {
namespace {

constexpr int kGenThreads = 256;
constexpr int kGenTokens = 64;       // tokens per step of a workgroup

template <class T, int D>
__global__ __launch_bounds__(kGenThreads) void generic_branch_state_kernel(
    const T* __restrict__ qkv, const T* __restrict__ w_dw, const T* __restrict__ w_gpw, T* __restrict__ q_ms,
    float* __restrict__ partials, int H, int W, int heads, int S, int branch, int ks, int nchunks, int groups_per_chunk) {
    constexpr int kState = D * (D + 1);
    constexpr int kAcc = (kState + kGenThreads - 1) / kGenThreads;
    __shared__ float dw[kGenTokens][3 * D];       // depthwise sums (or, raw branch, the tokens themselves)
    __shared__ float rk[kGenTokens][D];           // rectified K of the branch
    __shared__ float vv[kGenTokens][D];           // V of the branch
    const int h = blockIdx.x % heads;
    const int chunk = (blockIdx.x / heads) % nchunks;
    const int b = blockIdx.x / (heads * nchunks);
    const int N = H * W;
    const int Ct = heads * D;
    const long ts = 3L * Ct;                                   // elements from token to token of qkv
    const T* img = qkv + (long)b * N * ts + (long)h * 3 * D;   // this head's 3*D channels of token 0
    const int P = (ks - 1) / 2;
    const T* wd = w_dw + (long)h * 3 * D * ks * ks;            // [3*D][ks][ks] of this head
    const T* wg = w_gpw + (long)h * 3 * D * D;                 // [3*D][D] of this head

    float acc[kAcc];
#pragma unroll
    for (int i = 0; i < kAcc; ++i) acc[i] = 0.f;

    const int n_groups = (N + kGenTokens - 1) / kGenTokens;
    const int g_begin = chunk * groups_per_chunk;
    const int g_end = g_begin + groups_per_chunk < n_groups ? g_begin + groups_per_chunk : n_groups;
    for (int g = g_begin; g < g_end; ++g) {
        const int n0 = g * kGenTokens;
        // ---- A: depthwise k x k sums of the group's tokens (zero padding), or the raw tokens
        for (int it = threadIdx.x; it < kGenTokens * 3 * D; it += kGenThreads) {
            const int tk = it / (3 * D), c = it - tk * (3 * D);
            const int n = n0 + tk;
            float s = 0.f;
            if (n < N) {
                if (ks == 0) {
                    s = Traits<T>::to_f32(img[(long)n * ts + c]);
                } else {
                    const int y = n / W, x = n - y * W;
                    for (int u = 0; u < ks; ++u) {
                        const int yy = y + u - P;
                        if (yy < 0 || yy >= H) continue;
                        for (int v = 0; v < ks; ++v) {
                            const int xx = x + v - P;
                            if (xx < 0 || xx >= W) continue;
                            s = fmaf(Traits<T>::to_f32(wd[(c * ks + u) * ks + v]),
                                     Traits<T>::to_f32(img[((long)yy * W + xx) * ts + c]), s);
                        }
                    }
                }
            }
            dw[tk][c] = s;
        }
        __syncthreads();
        // ---- B: grouped 1x1 (D -> D inside each of Q, K, V); Q is stored, relu(K) and V go on to the state
        for (int it = threadIdx.x; it < kGenTokens * 3 * D; it += kGenThreads) {
            const int tk = it / (3 * D), c = it - tk * (3 * D);
            const int t = c / D, o = c - t * D;
            const int n = n0 + tk;
            float s;
            if (ks == 0) {
                s = dw[tk][c];
            } else {
                s = 0.f;
#pragma unroll 8
                for (int e = 0; e < D; ++e) s = fmaf(Traits<T>::to_f32(wg[(long)c * D + e]), dw[tk][t * D + e], s);
            }
            if (t == 0) {
                if (n < N) q_ms[((long)b * N + n) * ((long)S * Ct) + (long)(branch * heads + h) * D + o] = Traits<T>::from_f32(s);
            } else if (t == 1) {
                rk[tk][o] = n < N ? fmaxf(s, 0.f) : 0.f;       // Eq. (2); tokens past the image contribute nothing
            } else {
                vv[tk][o] = s;
            }
        }
        __syncthreads();
        // ---- C: KV[e][f] += sum_n relu(K_n[e]) * (f < D ? V_n[f] : 1)
#pragma unroll
        for (int i = 0; i < kAcc; ++i) {
            const int idx = threadIdx.x + i * kGenThreads;
            if (idx < kState) {
                const int e = idx / (D + 1), f = idx - e * (D + 1);
                float s = acc[i];
                if (f < D) {
                    for (int tk = 0; tk < kGenTokens; ++tk) s = fmaf(rk[tk][e], vv[tk][f], s);
                } else {
                    for (int tk = 0; tk < kGenTokens; ++tk) s += rk[tk][e];
                }
                acc[i] = s;
            }
        }
        __syncthreads();
    }
    float* out = partials + ((((long)b * S + branch) * heads + h) * nchunks + chunk) * kState;
#pragma unroll
    for (int i = 0; i < kAcc; ++i) {
        const int idx = threadIdx.x + i * kGenThreads;
        if (idx < kState) out[idx] = acc[i];
    }
}

template <int D>
__global__ __launch_bounds__(kGenThreads) void generic_state_finalize_kernel(const float* __restrict__ partials,
                                                                             float* __restrict__ kv32, int nchunks) {
    constexpr int kState = D * (D + 1);
    const long sid = blockIdx.x;
    for (int j = threadIdx.x; j < kState; j += kGenThreads) {
        const float* p = partials + sid * nchunks * kState + j;
        float v = 0.f;
        // chunk order (reproducible); eight loads in flight at a time, a launch is otherwise one load latency a chunk
        for (int c0 = 0; c0 < nchunks; c0 += 8) {
            float part[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) part[i] = c0 + i < nchunks ? p[(long)(c0 + i) * kState] : 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i) v += part[i];
        }
        kv32[sid * kState + j] = v;
    }
}

// Normalise-and-apply for heads of 32 channels on the matrix cores in fp32 (the operands -- rectified Q
// converted from the storage type, the fp32 state -- go in exactly).  A workgroup owns four neighbouring
// head-branches, one per wave (256 contiguous bytes of a token's row in the 16-bit types: whole lines), and
// kApplyGroups groups of 16 tokens; lane (token x16, q) holds channels 8q..8q+7 of its token (one 16-byte
// load in, one 16-byte store out in the 16-bit types).  The 32 x 32 product is a 2 x 2 arrangement of
// 16 x 16 x 16 contractions whose slots are numbered to fit that: contraction slot (q, r) of chunk jc is
// channel e = 8q + 4jc + r, output row 4q + r of chunk jo is channel f = 8q + 4jo + r.
constexpr int kApplyGroups = 8;

template <class T>
struct Row8 {                       // a lane's eight channels as loaded
    u32x4 v[sizeof(T) == 4 ? 2 : 1];
};
template <class T>
__device__ __forceinline__ Row8<T> load_row8(const T* p) {
    Row8<T> r;
    r.v[0] = *(const u32x4*)p;
    if constexpr (sizeof(T) == 4) r.v[1] = *(const u32x4*)(p + 4);
    return r;
}
template <class T>
__device__ __forceinline__ void widen_row8(const Row8<T>& r, float* out) {
    if constexpr (sizeof(T) == 4) {
        const f32x4 a = __builtin_bit_cast(f32x4, r.v[0]), b = __builtin_bit_cast(f32x4, r.v[1]);
#pragma unroll
        for (int i = 0; i < 4; ++i) out[i] = a[i], out[4 + i] = b[i];
    } else {
        const typename Traits<T>::Vec x = __builtin_bit_cast(typename Traits<T>::Vec, r.v[0]);
#pragma unroll
        for (int i = 0; i < 8; ++i) out[i] = Traits<T>::to_f32(x[i]);
    }
}
template <class T>
__device__ __forceinline__ void store_row8(T* p, const float* v) {
    if constexpr (sizeof(T) == 4) {
        *(f32x4*)p = f32x4{v[0], v[1], v[2], v[3]};
        *(f32x4*)(p + 4) = f32x4{v[4], v[5], v[6], v[7]};
    } else {
        typename Traits<T>::Vec x;
#pragma unroll
        for (int i = 0; i < 8; ++i) x[i] = Traits<T>::from_f32(v[i]);
        *(u32x4*)p = __builtin_bit_cast(u32x4, x);
    }
}

template <class T, int D>
__global__ __launch_bounds__(kGenThreads) void generic_apply_kernel(const T* __restrict__ q_ms, const float* __restrict__ kv32,
                                                                    T* __restrict__ att, int N, int n_hb, int blocks_per_image,
                                                                    float eps) {
    static_assert(D == 32, "2 x 2 blocks of 16");
    constexpr int kState = D * (D + 1);
    typedef Traits<float> F32;
    const int quads = (n_hb + 3) / 4;
    const int lane = lane_id(), wave = threadIdx.x >> 6, x16 = lane & 15, q = lane >> 4;
    const int m = (blockIdx.x % quads) * 4 + wave;
    const int nb = (blockIdx.x / quads) % blocks_per_image;
    const int b = blockIdx.x / (quads * blocks_per_image);
    if (m >= n_hb) return;      // no barrier below
    const float* st = kv32 + ((long)b * n_hb + m) * kState;
    // state operands: S[jc][jo] lane (x16, q) = KV[8q + 4jc + r][8(x16 >> 2) + 4jo + (x16 & 3)], r = 0..3
    f32x4 S[2][2];
    float ksum[8];
    const int fo = 8 * (x16 >> 2) + (x16 & 3);
#pragma unroll
    for (int jc = 0; jc < 2; ++jc)
#pragma unroll
        for (int jo = 0; jo < 2; ++jo)
#pragma unroll
            for (int r = 0; r < 4; ++r) S[jc][jo][r] = st[(8 * q + 4 * jc + r) * (D + 1) + fo + 4 * jo];
#pragma unroll
    for (int i = 0; i < 8; ++i) ksum[i] = st[(8 * q + i) * (D + 1) + D];

    const long pitch = (long)n_hb * D;
    const f32x4 z = {0.f, 0.f, 0.f, 0.f};
    auto fetch = [&](int u, bool& live, long& at) {
        const long n = ((long)nb * kApplyGroups + u) * 16 + x16;
        live = n < N;
        at = ((long)b * N + (live ? n : 0)) * pitch + (long)m * D + 8 * q;     // a token past the end reads token 0
        return load_row8<T>(q_ms + at);
    };
    bool live, live_next = false;
    long at, at_next = 0;
    Row8<T> cur = fetch(0, live, at), next = cur;
#pragma unroll
    for (int u = 0; u < kApplyGroups; ++u) {
        if (u + 1 < kApplyGroups) next = fetch(u + 1, live_next, at_next);
        float rq[8];
        widen_row8<T>(cur, rq);
        float den = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            rq[i] = live ? fmaxf(rq[i], 0.f) : 0.f;
            den = fmaf(rq[i], ksum[i], den);
        }
        den += __shfl_xor(den, 16);
        den += __shfl_xor(den, 32);
        const f32x4 lo = {rq[0], rq[1], rq[2], rq[3]}, hi = {rq[4], rq[5], rq[6], rq[7]};
        const f32x4 n0 = F32::mma16(F32::mma16(z, S[0][0], lo), S[1][0], hi);
        const f32x4 n1 = F32::mma16(F32::mma16(z, S[0][1], lo), S[1][1], hi);
        const float inv = 1.0f / (den + eps);
        if (live) {
            const float o[8] = {n0[0] * inv, n0[1] * inv, n0[2] * inv, n0[3] * inv,
                                n1[0] * inv, n1[1] * inv, n1[2] * inv, n1[3] * inv};
            store_row8<T>(att + at, o);
        }
        cur = next;
        live = live_next;
        at = at_next;
    }
}

// fixed-order sum of the partial states, then the normalise-and-apply pass
template <class T, int D>
hipError_t finish_generic(const GenericArgs& a, int N, hipStream_t stream) {
    const int S = 1 + a.n_scales;
    const int n_states = a.B * S * a.heads;
    hipLaunchKernelGGL((generic_state_finalize_kernel<D>), dim3((unsigned)n_states), dim3(kGenThreads), 0, stream, a.partials,
                       a.kv32, a.nchunks);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int bpi = (N + 16 * kApplyGroups - 1) / (16 * kApplyGroups);
    const long nb2 = (long)a.B * ((S * a.heads + 3) / 4) * bpi;
    if (nb2 > 0x7fffffffL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((generic_apply_kernel<T, D>), dim3((unsigned)nb2), dim3(kGenThreads), 0, stream, (const T*)a.q_ms, a.kv32,
                       (T*)a.att, N, S * a.heads, bpi, a.eps);
    return hipGetLastError();
}

template <class T, int D>
hipError_t run_generic(const GenericArgs& a, hipStream_t stream) {
    const int N = a.H * a.W;
    const int n_groups = (N + kGenTokens - 1) / kGenTokens;
    const int gpc = (n_groups + a.nchunks - 1) / a.nchunks;
    const long nb = (long)a.B * a.heads * a.nchunks;
    if (nb <= 0 || nb > 0x7fffffffL) return hipErrorInvalidValue;
    const int S = 1 + a.n_scales;
    size_t dw_off = 0;
    if constexpr (D == 32 && sizeof(T) == 2) {
        if (a.n_scales > 0) {
            // 16-bit storage: the tiled matrix-core form (k_aggregate32.hip); its first launch also does the
            // raw branch.  Same partial-state buffer, chunks counted in 8 x 32-token tiles.
            AggregateArgs g;
            g.q = a.qkv;
            g.k = (const T*)a.qkv + D;
            g.v = (const T*)a.qkv + 2 * D;
            g.q_ts = g.k_ts = g.v_ts = 3L * a.heads * D;
            g.q_hs = g.k_hs = g.v_hs = 3 * D;
            g.q_ms = a.q_ms;
            g.partials = a.partials;
            g.B = a.B; g.H = a.H; g.W = a.W; g.heads = a.heads; g.S = S;
            g.nchunks = a.nchunks;
            const long tiles = (long)((a.H + kAggTileH - 1) / kAggTileH) * ((a.W + kAggTileW - 1) / kAggTileW);
            g.tiles_per_chunk = (int)((tiles + a.nchunks - 1) / a.nchunks);
            for (int i = 0; i < a.n_scales; ++i) {
                const int ks = a.scales[i];
                g.w_dw = (const T*)a.w_dw + dw_off;
                g.w_gpw = (const T*)a.w_gpw + (size_t)i * 3 * a.heads * D * D;
                dw_off += (size_t)3 * a.heads * D * ks * ks;
                g.ks = ks;
                g.branch = i + 1;
                g.do_raw = (i == 0);
                g.copy_raw_q = (i == 0);
                const hipError_t e = launch_aggregate32(sizeof(T) == 2 && std::is_same<T, _Float16>::value ? 1 : 2, g, stream);
                if (e != hipSuccess) return e;
            }
            return finish_generic<T, D>(a, N, stream);
        }
    }
    for (int s = 0; s < S; ++s) {
        const int ks = s == 0 ? 0 : a.scales[s - 1];
        const T* wdw = s == 0 ? nullptr : (const T*)a.w_dw + dw_off;
        const T* wgp = s == 0 ? nullptr : (const T*)a.w_gpw + (size_t)(s - 1) * 3 * a.heads * D * D;
        if (s > 0) dw_off += (size_t)3 * a.heads * D * ks * ks;
        hipLaunchKernelGGL((generic_branch_state_kernel<T, D>), dim3((unsigned)nb), dim3(kGenThreads), 0, stream,
                           (const T*)a.qkv, wdw, wgp, (T*)a.q_ms, a.partials, a.H, a.W, a.heads, S, s, ks, a.nchunks, gpc);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return finish_generic<T, D>(a, N, stream);
}

template <class T>
hipError_t run_generic_d(const GenericArgs& a, hipStream_t stream) {
    if (a.head_dim == 32) return run_generic<T, 32>(a, stream);
    return hipErrorNotSupported;
}

// row of the paired arrangement -> row of the head-size-8 arrangement (channel order (h*3 + t)*d + e)
__device__ __forceinline__ int head8_row(int row16) {
    const int hp = row16 / 48, r = row16 - hp * 48, t = r >> 4, e16 = r & 15;
    return ((2 * hp + (e16 >> 3)) * 3 + t) * 8 + (e16 & 7);
}

template <class T>
__global__ __launch_bounds__(256) void pair_head8_weights_kernel(const T* __restrict__ w_qkv, const T* __restrict__ w_dw,
                                                                 const T* __restrict__ w_gpw, T* __restrict__ o_qkv,
                                                                 T* __restrict__ o_dw, T* __restrict__ o_gpw, int C, int rows,
                                                                 int n_scales, int k0, int k1, int k2, int k3, int k4, int k5,
                                                                 int k6, int k7) {
    const int ks[8] = {k0, k1, k2, k3, k4, k5, k6, k7};
    const long n_qkv = (long)rows * C;
    long n_dw = 0;
    for (int i = 0; i < n_scales; ++i) n_dw += (long)rows * ks[i] * ks[i];
    const long n_gpw = (long)n_scales * rows * 16;
    const long total = n_qkv + n_dw + n_gpw;
    for (long id = (long)blockIdx.x * blockDim.x + threadIdx.x; id < total; id += (long)gridDim.x * blockDim.x) {
        if (id < n_qkv) {
            const int row = (int)(id / C), c = (int)(id - (long)row * C);
            o_qkv[id] = w_qkv[(long)head8_row(row) * C + c];
        } else if (id < n_qkv + n_dw) {
            long r = id - n_qkv, base = 0;
            int i = 0;
            while (r >= (long)rows * ks[i] * ks[i]) {
                r -= (long)rows * ks[i] * ks[i];
                base += (long)rows * ks[i] * ks[i];
                ++i;
            }
            const int kk = ks[i] * ks[i];
            const int row = (int)(r / kk), tap = (int)(r - (long)row * kk);
            o_dw[base + r] = w_dw[base + (long)head8_row(row) * kk + tap];
        } else {
            const long r = id - n_qkv - n_dw;
            const int i = (int)(r / ((long)rows * 16));
            const int rem = (int)(r - (long)i * rows * 16);
            const int row = rem >> 4, col = rem & 15;
            const bool own = (col >> 3) == ((row & 15) >> 3);
            o_gpw[r] = own ? w_gpw[((long)i * rows + head8_row(row)) * 8 + (col & 7)] : Traits<T>::from_f32(0.f);
        }
    }
}

template <class T>
hipError_t run_pair_head8(const void* w_qkv, const void* w_dw, const void* w_gpw, void* o_qkv, void* o_dw, void* o_gpw, int C,
                          int heads8, const int* scales, int n_scales, hipStream_t stream) {
    int k[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int i = 0; i < n_scales; ++i) k[i] = scales[i];
    const int rows = 3 * heads8 * 8;
    hipLaunchKernelGGL((pair_head8_weights_kernel<T>), dim3(256), dim3(256), 0, stream, (const T*)w_qkv, (const T*)w_dw,
                       (const T*)w_gpw, (T*)o_qkv, (T*)o_dw, (T*)o_gpw, C, rows, n_scales, k[0], k[1], k[2], k[3], k[4], k[5],
                       k[6], k[7]);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_pair_head8_weights(int dt, const void* w_qkv, const void* w_dw, const void* w_gpw, void* w_qkv16,
                                     void* w_dw16, void* w_gpw16, int C, int heads8, const int* scales, int n_scales,
                                     hipStream_t stream) {
    if (heads8 <= 0 || heads8 % 2 != 0 || n_scales < 0 || n_scales > 8) return hipErrorInvalidValue;
    switch (dt) {
        case 0: return run_pair_head8<float>(w_qkv, w_dw, w_gpw, w_qkv16, w_dw16, w_gpw16, C, heads8, scales, n_scales, stream);
        case 1: return run_pair_head8<_Float16>(w_qkv, w_dw, w_gpw, w_qkv16, w_dw16, w_gpw16, C, heads8, scales, n_scales, stream);
        case 2: return run_pair_head8<__bf16>(w_qkv, w_dw, w_gpw, w_qkv16, w_dw16, w_gpw16, C, heads8, scales, n_scales, stream);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_generic_core(int dt, const GenericArgs& a, hipStream_t stream) {
    switch (dt) {
        case 0: return run_generic_d<float>(a, stream);
        case 1: return run_generic_d<_Float16>(a, stream);
        case 2: return run_generic_d<__bf16>(a, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace msla
