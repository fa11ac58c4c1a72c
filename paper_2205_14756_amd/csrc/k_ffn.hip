// The FFN+DWConv half of the EfficientViT building block (Section 3.1: a depthwise convolution is
// inserted into the FFN layer that follows the attention module; Fig. 2 left).  Declared reading (the
// paper prints no more than the sentence above):
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
    else return a * __builtin_amdgcn_fmed3f(fmaf(a, 1.0f / 6.0f, 0.5f), 0.f, 1.f);      // a * clip(a + 3, 0, 6) / 6
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

// The same operation for the 16-bit storage types with the waves specialised: the depthwise pass is
// vector-ALU work (144 mixed-precision FMAs a thread and slab), the projection matrix-core work, the
// staging LDS traffic -- three different units that a wave doing all three in turn keeps busy one at a
// time.  Sixteen waves: waves 0-7 (two per SIMD) only stage W2 slabs and issue matrix instructions, waves
// 8-15 (two per SIMD) only stage halo tiles and do the depthwise pass.  Everything in LDS is
// double-buffered and one barrier ends each step.  In step i
//   consumers   park W2 slab i+1, request slab i+2, multiply slab i  (token tile i%2 x weight tile i%2)
//   producers   park halo i+2, request halo i+3, depthwise pass of slab i+1 -> token tile (i+1)%2
// so every buffer written in a step was last read in the step before.  Rows are 128 bytes, unpadded, with
// the 16-byte chunk index XOR-ed with (row / 2) % 8 (full rate for operand reads and row-order writes).
// Requires one image's expanded map to stay below 2^31 bytes (32-bit offsets in a buffer resource).
template <class T, int ACT>
__global__ __launch_bounds__(1024) void ffn_dw_project_split_kernel(const T* __restrict__ h, const T* __restrict__ w_dw,
                                                                   const T* __restrict__ w2, const T* __restrict__ res,
                                                                   T* __restrict__ out, int H, int W, int E, int c_out,
                                                                   int tiles_x, int tiles_y, int n_rb) {
    static_assert(sizeof(T) == 2, "16-bit storage types");
    typedef GemmTile<T, 4, 2> G;
    typedef Traits<T> Tr;
    typedef typename Tr::Vec Vec;
    constexpr int BK = 64;                           // hidden channels per slab (128 bytes)
    constexpr int kHaloW = 34, kHaloH = 6, kHaloTok = kHaloW * kHaloH;
    constexpr int kWt = 256 * 128, kTok = 128 * 128, kHalo = kHaloTok * 128 + 128;
    constexpr int kHaloVec = (kHaloTok * 8 + 511) / 512;      // 16-byte vectors per producer thread and slab
    extern __shared__ __attribute__((aligned(16))) char lds[];
    char* const ldsW = lds;                          // 2 weight tiles
    char* const ldsC = ldsW + 2 * kWt;               // 2 token tiles (the activated depthwise sums)
    char* const ldsH = ldsC + 2 * kTok;              // 2 halo tiles

    const unsigned L = xcd_remap(blockIdx.x, gridDim.x);
    const int rb = L % n_rb;
    unsigned rest = L / n_rb;
    const int tx = rest % tiles_x;
    rest /= tiles_x;
    const int ty = rest % tiles_y;
    const int b = rest / tiles_y;
    const int y0 = ty * 4, x0 = tx * 32, oc0 = rb * G::BR;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n_slab = (E + BK - 1) / BK;
    const unsigned e_bytes = (unsigned)E * 2u;

    if (wave < 8) {
        // ------------------------------------------------------------ consumers
        const int wr = wave % 4, wc = wave / 4;
        const int lane = lane_id(), x16 = lane & 15, q = lane >> 4, g16 = (x16 >> 1) & 7;
        f32x4 acc[4][4];
        G::zero(acc);
        // weight slab: thread = (row v / 8, chunk v % 8) of vectors v = tid + i * 512
        const BufRsrc wres = make_rsrc(w2, (long)c_out * e_bytes);
        unsigned w_glb[4], w_lds[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int v = threadIdx.x + i * 512;
            const int row = v >> 3, chunk = v & 7;
            w_glb[i] = oc0 + row < c_out ? (unsigned)(oc0 + row) * e_bytes + chunk * 16 : kOobOffset;
            w_lds[i] = row * 128 + ((chunk ^ ((row >> 1) & 7)) * 16);
        }
        const int w_chunk = threadIdx.x & 7;
        u32x4 rw[4];
        // operand offsets of this lane for the two 32-slot halves of a slab
        const int a_off = (wr * 64 + x16) * 128, b_off = (wc * 64 + x16) * 128;
        const int c_lo = ((0 * 4 + q) ^ g16) * 16, c_hi = ((1 * 4 + q) ^ g16) * 16;
        for (int i = -3; i < n_slab; ++i) {
            if (i + 1 >= 0 && i + 1 < n_slab) {
                char* dst = ldsW + ((i + 1) & 1) * kWt;
#pragma unroll
                for (int j = 0; j < 4; ++j) *(u32x4*)(dst + w_lds[j]) = rw[j];
            }
            if (i + 2 >= 0 && i + 2 < n_slab) {
                const unsigned k_bytes = (unsigned)(i + 2) * 128u;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    rw[j] = buf_load16(wres, (w_glb[j] != kOobOffset && k_bytes + w_chunk * 16 < e_bytes) ? w_glb[j] + k_bytes
                                                                                                     : kOobOffset, 0);
            }
            if (i >= 0) {
                const char* wt = ldsW + (i & 1) * kWt + a_off;
                const char* ct = ldsC + (i & 1) * kTok + b_off;
#pragma unroll
                for (int kk = 0; kk < 2; ++kk) {
                    const int co = kk ? c_hi : c_lo;
                    Vec fa[4], fb[4];
#pragma unroll
                    for (int io = 0; io < 4; ++io) fa[io] = __builtin_bit_cast(Vec, *(const u32x4*)(wt + io * 16 * 128 + co));
#pragma unroll
                    for (int jt = 0; jt < 4; ++jt) fb[jt] = __builtin_bit_cast(Vec, *(const u32x4*)(ct + jt * 16 * 128 + co));
#pragma unroll
                    for (int io = 0; io < 4; ++io)
#pragma unroll
                        for (int jt = 0; jt < 4; ++jt) acc[io][jt] = Tr::mma_vec(acc[io][jt], fa[io], fb[jt]);
                }
            }
            __syncthreads();
        }
        // ---- results: tile token t = (row t / 32, column t % 32) of the block; staged in the weight tiles
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
        static_assert(G::kStageResBytes <= 2 * kWt, "the epilogue stages in the weight tiles");
        G::epilogue_lds_residual(acc, lds, oc0, wr, wc, to, [&](int trow, int oc) {
            const int r = trow >> 5, c = trow & 31;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (r < rows && c < cols && oc < c_out) v = *(const u32x4*)(res + (base + (long)r * W + c) * c_out + oc);
            return v;
        });
    } else {
        // ------------------------------------------------------------ producers
        // A wave is one 16-byte channel vector of the slab (8 channels), its lanes the tile's columns and
        // row pairs: the 72 filter taps a wave needs are then the same for all its lanes and live in scalar
        // registers, read straight from w_dw (8 channels x 9 taps are 144 consecutive bytes).  The halo is
        // kept as 8 planes [channel vector][halo token][16 bytes], so consecutive lanes read consecutive 16
        // bytes; a plane is padded by 16 bytes, which spreads the 8 planes a row-order copy writes to at once
        // over all banks.
        const int pt = threadIdx.x - 512;
        const int dvec = wave - 8, lane = lane_id(), dcol = lane & 31, dhalf = lane >> 5;
        constexpr int kPlane = kHaloTok * 16 + 16;
        static_assert(8 * kPlane <= kHalo + 128, "planes fit the halo buffer");
        const BufRsrc hres = make_rsrc(h + (long)b * H * W * E, (long)H * W * e_bytes);
        // halo copy: vector id = j * 512 + pt -> halo token id / 8, chunk id % 8
        unsigned h_glb[kHaloVec];
        int h_lds[kHaloVec];
#pragma unroll
        for (int j = 0; j < kHaloVec; ++j) {
            const int id = j * 512 + pt;
            const int tok = id >> 3, v = id & 7;
            const int hy = tok / kHaloW, hx = tok - hy * kHaloW;
            const int yy = y0 - 1 + hy, xx = x0 - 1 + hx;
            const bool ok = tok < kHaloTok && yy >= 0 && yy < H && xx >= 0 && xx < W;
            h_glb[j] = ok ? (unsigned)(yy * W + xx) * e_bytes + v * 16 : kOobOffset;
            h_lds[j] = tok < kHaloTok ? v * kPlane + tok * 16 : -1;
        }
        const int d_lds = dvec * kPlane + (2 * dhalf * kHaloW + dcol) * 16;
        const int t0 = (2 * dhalf) * 32 + dcol, t1 = t0 + 32;
        const int c_lds0 = t0 * 128 + ((dvec ^ ((t0 >> 1) & 7)) * 16), c_lds1 = t1 * 128 + ((dvec ^ ((t1 >> 1) & 7)) * 16);
        u32x4 rh[kHaloVec];
        for (int i = -3; i < n_slab; ++i) {
            if (i + 2 >= 0 && i + 2 < n_slab) {           // park halo i+2
                char* hd = ldsH + (i & 1) * (8 * kPlane);
#pragma unroll
                for (int j = 0; j < kHaloVec; ++j)
                    if (h_lds[j] >= 0) *(u32x4*)(hd + h_lds[j]) = rh[j];
            }
            if (i + 3 < n_slab) {                         // request halo i+3
                const unsigned k_bytes = (unsigned)(i + 3) * 128u;
#pragma unroll
                for (int j = 0; j < kHaloVec; ++j)
                    rh[j] = buf_load16(hres, (h_glb[j] != kOobOffset && k_bytes + (pt & 7) * 16 < e_bytes) ? h_glb[j] + k_bytes
                                                                                                     : kOobOffset, 0);
            }
            if (i + 1 >= 0 && i + 1 < n_slab) {           // depthwise 3x3 + activation of slab i+1
                const char* hs = ldsH + ((i + 1) & 1) * (8 * kPlane) + d_lds;
                char* cd = ldsC + ((i + 1) & 1) * kTok;
                // element (channel j, tap t) of this wave's 72 = vector (j * 9 + t) / 8, slot (j * 9 + t) % 8
                const int ch = (i + 1) * BK + dvec * 8;
                Vec wt[9];
#pragma unroll
                for (int t = 0; t < 9; ++t) {
                    u32x4 raw = {0u, 0u, 0u, 0u};
                    if (ch < E) raw = *(const u32x4*)(w_dw + (long)ch * 9 + t * 8);
                    wt[t] = __builtin_bit_cast(Vec, raw);
                }
                float a0[8], a1[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) a0[j] = a1[j] = 0.f;
#pragma unroll
                for (int r = 0; r < 4; ++r) {            // halo rows 2*dhalf + r
#pragma unroll
                    for (int dx = 0; dx < 3; ++dx) {
                        const Vec f = __builtin_bit_cast(Vec, *(const u32x4*)(hs + (r * kHaloW + dx) * 16));
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            const float fj = Tr::to_f32(f[j]);
                            if (r < 3) {            // output row 2*dhalf: tap row r
                                const int e = j * 9 + r * 3 + dx;
                                a0[j] = fmaf(Tr::to_f32(wt[e / 8][e % 8]), fj, a0[j]);
                            }
                            if (r > 0) {            // output row 2*dhalf + 1: tap row r - 1
                                const int e = j * 9 + (r - 1) * 3 + dx;
                                a1[j] = fmaf(Tr::to_f32(wt[e / 8][e % 8]), fj, a1[j]);
                            }
                        }
                    }
                }
                Vec o0, o1;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    o0[j] = Tr::from_f32(activate<ACT>(a0[j]));
                    o1[j] = Tr::from_f32(activate<ACT>(a1[j]));
                }
                *(u32x4*)(cd + c_lds0) = __builtin_bit_cast(u32x4, o0);
                *(u32x4*)(cd + c_lds1) = __builtin_bit_cast(u32x4, o1);
            }
            __syncthreads();
        }
    }
}

template <class T>
hipError_t run_dw_project(const void* h, const void* w_dw, const void* w2, const void* res, void* out, int B, int H, int W,
                          int E, int c_out, int act, hipStream_t stream) {
    typedef GemmTile<T, 4, 2> G;
    const int tiles_x = (W + 31) / 32, tiles_y = (H + 3) / 4;
    const int n_rb = (c_out + G::BR - 1) / G::BR;
    const long nblocks = (long)B * tiles_x * tiles_y * n_rb;
    if (nblocks <= 0 || nblocks > 0x7fffffffL) return hipErrorInvalidValue;
    hipError_t e;
    if constexpr (sizeof(T) == 2) {
        // waves specialised into depthwise producers and matrix-core consumers, where 32-bit offsets reach
        if ((long)H * W * E * 2 < 0x7fffffffL && (long)c_out * E * 2 < 0x7fffffffL && (long)E * 18 < 0x7fffffffL) {
            constexpr int kSplitLds = 2 * (256 * 128 + 128 * 128 + 204 * 128 + 128);
            if (act == 0) {
                e = allow_dynamic_lds<ffn_dw_project_split_kernel<T, 0>>(kSplitLds);
                if (e != hipSuccess) return e;
                hipLaunchKernelGGL((ffn_dw_project_split_kernel<T, 0>), dim3((unsigned)nblocks), dim3(1024), kSplitLds, stream,
                                   (const T*)h, (const T*)w_dw, (const T*)w2, (const T*)res, (T*)out, H, W, E, c_out, tiles_x,
                                   tiles_y, n_rb);
            } else {
                e = allow_dynamic_lds<ffn_dw_project_split_kernel<T, 1>>(kSplitLds);
                if (e != hipSuccess) return e;
                hipLaunchKernelGGL((ffn_dw_project_split_kernel<T, 1>), dim3((unsigned)nblocks), dim3(1024), kSplitLds, stream,
                                   (const T*)h, (const T*)w_dw, (const T*)w2, (const T*)res, (T*)out, H, W, E, c_out, tiles_x,
                                   tiles_y, n_rb);
            }
            return hipGetLastError();
        }
    }
    constexpr int kLds = G::kLdsR + G::kLdsC + 204 * 160 + 9 * G::BK * 4;
    static_assert(G::kStageResBytes <= G::kLdsR + G::kLdsC, "the epilogue stages in the operand tiles");
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
