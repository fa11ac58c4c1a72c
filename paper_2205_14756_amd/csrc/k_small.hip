// 1x1 projections with a long contraction (257 .. 1024 slots) for the 16-bit storage types:
// the Q/K/V projection of a wide module (Section 3.1: Q = x W_Q ...) and the fused
// normalise-and-apply + output projection (Eq. (3) + Section 3.1, last sentence) of a module with
// more than 32 head-branches.
//
// Such shapes have few tokens per channel (a late, low-resolution stage), so the weights are what
// a workgroup has to fetch.  A workgroup owns 128 output channels, 16 per wave, and keeps each
// wave's weight rows in registers (4 registers per 32 contraction slots: 128 at 1024); it walks
// over tiles of 32 tokens.  The tile's row operand -- the tokens themselves, or the attention rows
// of Eq. (3) made from the tile's Q tokens and the per-head states -- is put into LDS once, and
// every wave reads all of it against its own weights.  All weight requests are issued before the
// first tile is touched, so their latency is paid once, in parallel.
//
// LDS tile: [128-byte slab][32 rows][128 bytes], the 16-byte chunk index XOR-ed with (row/2)%8:
// operand reads (16 rows of one chunk), row-order copies and 8-byte attention stores all stay
// free of bank conflicts.  bf16 attention rows go in as a hi and a lo tile (8 significant bits
// alone would cost half the error budget).
#include "msla_device.h"
#include "msla_kernels.h"

namespace msla {
namespace {

constexpr int kSmallThreads = 512;
constexpr int kSmallTB = 32;             // tokens per tile
constexpr int kSmallChanBlock = 128;     // output channels per workgroup
constexpr int kSlabBytes = kSmallTB * 128;

__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }

// destination of output channel group g (16 channels) of token row `tok`
template <class T>
struct SmallPlain {
    T* y;
    int c_out;
    const T* res = nullptr;       // optional residual [n_tokens, c_out], added to the fp32 sums
    __device__ __forceinline__ T* at(long tok, int g) const { return y + tok * c_out + g * 16; }
    __device__ __forceinline__ f32x4 plus_residual(f32x4 v, long tok, int g, int c) const {
        if (res != nullptr) {
            const f32x4 r = frag_to_f32<T>(load_frag<T>(res + tok * c_out + g * 16 + c));
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] += r[e];
        }
        return v;
    }
};
// ... for the Q/K/V projection: group g = h*3 + t; Q goes to the branch-0 columns of the
// multi-scale Q map, K and V to the K|V map (token and head strides in elements)
template <class T>
struct SmallQkv {
    T* q_ms;
    long q_ms_stride;
    T* kv_raw;
    long kv_tok_stride, kv_head_stride;
    __device__ __forceinline__ f32x4 plus_residual(f32x4 v, long, int, int) const { return v; }
    __device__ __forceinline__ T* at(long tok, int g) const {
        const int h = g / 3, t = g - 3 * h;
        return t == 0 ? q_ms + tok * q_ms_stride + h * 16
                      : kv_raw + tok * kv_tok_stride + (long)h * kv_head_stride + (t - 1) * 16;
    }
};

struct SmallAttArgs {
    const char* kvfrag;       // per state: 64 lanes x 16 B of KV operands, then 64 x 16 B of Ksum operands
    const float* kvscale;
    int N;                    // tokens per image
    int n_hb;
    float eps;
};

// KC: contraction length in 32-slot chunks (weights: 4*KC registers).  kAtt: the row operand is
// the attention map of Eq. (3), made on the fly from src = the multi-scale Q map.
template <class T, int KC, bool kAtt, class Dest>
__global__ __launch_bounds__(kSmallThreads) void small_project_kernel(const T* __restrict__ src,
                                                                     const T* __restrict__ w, Dest dest,
                                                                     SmallAttArgs aa, long n_tokens, int K,
                                                                     int c_out, int n_cb, long n_tiles,
                                                                     int tiles_per_image) {
    typedef Traits<T> Tr;
    typedef typename Tr::Vec Vec;
    typedef typename Tr::Frag Frag;
    constexpr bool kHiLo = kAtt && Tr::kHiLo;
    constexpr int kTile = (KC / 2) * kSlabBytes;      // KC*32 slots * 2 bytes * 32 rows
    extern __shared__ __attribute__((aligned(16))) char lds[];
    char* tile_hi = lds;
    char* tile_lo = lds + kTile;                      // only with kHiLo

    const int cb = blockIdx.x % n_cb;
    const long first_tile = blockIdx.x / n_cb;
    const long tile_step = gridDim.x / n_cb;
    const int wave = threadIdx.x >> 6;
    const int lane = lane_id(), x16 = lane & 15, q = lane >> 4;
    const int g16 = (x16 >> 1) & 7;
    const int ch0 = cb * kSmallChanBlock + wave * 16;       // this wave's 16 output channels
    const unsigned row_bytes = (unsigned)K * 2u;

    // ---- weights: lane (channel x16, q) ends up with w[ch0 + x16][32 kk + 8 q .. + 8] for every chunk
    // kk.  They are fetched in row order -- a wave-level load covers two rows' 512 contiguous bytes;
    // read as fragments straight from memory it would cover sixteen 64-byte pieces a whole row
    // apart, which the memory path serves several times slower -- and dealt out through LDS, a round
    // of 256 contraction slots at a time, the next round's requests in flight meanwhile.
    Vec wf[KC];
    {
        constexpr int kRounds = KC / 8;
        const BufRsrc wres = make_rsrc(w, (long)c_out * row_bytes);
        u32x4 stage[2][8];
        auto request = [&](int r, u32x4 (&v)[8]) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int id = i * kSmallThreads + threadIdx.x;
                const int row = id >> 5, c = id & 31;
                const int ch = cb * kSmallChanBlock + row;
                const unsigned col = r * 512u + c * 16u;
                v[i] = buf_load16(wres, (ch < c_out && col < row_bytes) ? (unsigned)ch * row_bytes + col : kOobOffset, 0);
            }
        };
        request(0, stage[0]);
        static_for<0, kRounds>([&](auto r_c) {
            constexpr int r = decltype(r_c)::value;
            if constexpr (r + 1 < kRounds) request(r + 1, stage[(r + 1) & 1]);
            if constexpr (r > 0) __syncthreads();          // the previous round's fragments are out
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int id = i * kSmallThreads + threadIdx.x;
                const int row = id >> 5, c = id & 31;
                *(u32x4*)(lds + (c >> 3) * (kSmallChanBlock * 128) + row * 128 + swz(row, c & 7) * 16) = stage[r & 1][i];
            }
            __syncthreads();
#pragma unroll
            for (int j = 0; j < 8; ++j)
                wf[r * 8 + j] = __builtin_bit_cast(
                    Vec, *(const u32x4*)(lds + (j >> 1) * (kSmallChanBlock * 128) + (wave * 16 + x16) * 128 +
                                         ((((j & 1) * 4 + q) ^ g16) * 16)));
        });
        __syncthreads();
    }

    for (long tile = first_tile; tile < n_tiles; tile += tile_step) {
        // tile -> first token (in the whole map) and number of live rows
        long tok0;
        int rows;
        if constexpr (kAtt) {
            const long b = tile / tiles_per_image;
            const int n0 = (int)(tile - b * tiles_per_image) * kSmallTB;
            tok0 = b * aa.N + n0;
            rows = aa.N - n0 < kSmallTB ? aa.N - n0 : kSmallTB;
        } else {
            tok0 = tile * kSmallTB;
            rows = n_tokens - tok0 < kSmallTB ? (int)(n_tokens - tok0) : kSmallTB;
        }
        const BufRsrc sres = make_rsrc(src + tok0 * K, (long)rows * row_bytes);

        {
            // ---- copy the tile's rows (tokens, or Q tokens of every head-branch) in row order; rows
            // past the last token and slots past K read zero
            constexpr int kVecs = KC * 4 * kSmallTB / kSmallThreads;      // 16-byte vectors per thread
            static_assert(kVecs * kSmallThreads == KC * 4 * kSmallTB, "tile copy");
            u32x4 v[kVecs];
#pragma unroll
            for (int i = 0; i < kVecs; ++i) {
                const int id = i * kSmallThreads + threadIdx.x;
                const int row = id / (KC * 4), c = id - row * (KC * 4);
                v[i] = buf_load16(sres, c * 16u < row_bytes ? row * row_bytes + c * 16u : kOobOffset, 0);
            }
#pragma unroll
            for (int i = 0; i < kVecs; ++i) {
                const int id = i * kSmallThreads + threadIdx.x;
                const int row = id / (KC * 4), c = id - row * (KC * 4);
                *(u32x4*)(tile_hi + (c >> 3) * kSlabBytes + row * 128 + swz(row, c & 7) * 16) = v[i];
            }
        }
        if constexpr (kAtt) {
            // ---- attention rows (Eq. (3)), made in place: unit = (16 tokens jt, head-branch m); the
            // wave takes m = wave, wave + 8, ...  Lane (token x16, q) reads channels 4q..4q+3 of its
            // token's Q from the tile and writes the attention row's same channels where they were.
            __syncthreads();
            const long img = tok0 / aa.N;
            const f32x4 z = {0.f, 0.f, 0.f, 0.f};
            for (int m = wave; m < KC * 2; m += 8) {
                const bool live = m < aa.n_hb;
                const long sid = img * aa.n_hb + (live ? m : 0);
                const Vec a_kv = __builtin_bit_cast(Vec, *(const u32x4*)(aa.kvfrag + sid * 2048 + lane * 16));
                const Vec a_ks = __builtin_bit_cast(Vec, *(const u32x4*)(aa.kvfrag + sid * 2048 + 1024 + lane * 16));
                const float eps_s = aa.eps * aa.kvscale[sid];
#pragma unroll
                for (int jt = 0; jt < 2; ++jt) {
                    const int row = jt * 16 + x16;
                    const int off = (m >> 2) * kSlabBytes + row * 128 + (((m & 3) * 2 + (q >> 1)) ^ g16) * 16 + (q & 1) * 8;
                    const Frag qf = frag_relu_bits<T>(load_frag<T>(tile_hi + off));
                    Vec b;
#pragma unroll
                    for (int r = 0; r < 4; ++r) { b[r] = qf[r]; b[4 + r] = qf[r]; }     // pairs with {hi, lo} of the state
                    const f32x4 num = Tr::mma_vec(z, a_kv, b);
                    const f32x4 den = Tr::mma_vec(z, a_ks, b);
                    const float inv = live ? __builtin_amdgcn_rcpf(den[0] + eps_s) : 0.f;
                    const f32x4 o = {num[0] * inv, num[1] * inv, num[2] * inv, num[3] * inv};
                    if constexpr (kHiLo) {
                        Frag hi, lo;
                        frag_split<T>(o, hi, lo);
                        store_frag<T>(tile_hi + off, hi);
                        store_frag<T>(tile_lo + off, lo);
                    } else {
                        store_frag<T>(tile_hi + off, frag_from_f32<T>(o));
                    }
                }
            }
        }
        __syncthreads();

        // ---- 16 channels x 32 tokens per wave: D[channel 4q+r][token x16]
        f32x4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
        const int frag_off = x16 * 128 + (q ^ g16) * 16;
#pragma unroll
        for (int kk = 0; kk < KC; ++kk) {
#pragma unroll
            for (int jt = 0; jt < 2; ++jt) {
                const int off = (frag_off ^ ((kk & 1) * 64)) + (kk >> 1) * kSlabBytes + jt * 16 * 128;
                acc[jt] = Tr::mma_vec(acc[jt], wf[kk], __builtin_bit_cast(Vec, *(const u32x4*)(tile_hi + off)));
                if constexpr (kHiLo)
                    acc[jt] = Tr::mma_vec(acc[jt], wf[kk], __builtin_bit_cast(Vec, *(const u32x4*)(tile_lo + off)));
            }
        }
        // ---- lane (token x16, q): channels 4q..4q+3 of the wave's group, 8 bytes
        if (ch0 < c_out) {
#pragma unroll
            for (int jt = 0; jt < 2; ++jt) {
                const int row = jt * 16 + x16;
                if (row < rows)
                    store_frag<T>(dest.at(tok0 + row, ch0 >> 4) + q * 4,
                                  frag_from_f32<T>(dest.plus_residual(acc[jt], tok0 + row, ch0 >> 4, q * 4)));
            }
        }
        __syncthreads();       // the tile is rewritten by the next iteration
    }
}

template <class T, int KC, bool kAtt, class Dest>
hipError_t run_small(const void* src, const void* w, Dest dest, SmallAttArgs aa, long n_tokens, int K, int c_out,
                     long n_tiles, int tiles_per_image, hipStream_t stream) {
    const int n_cb = (c_out + kSmallChanBlock - 1) / kSmallChanBlock;
    if (n_tiles <= 0 || (long)c_out * K * 2 >= 0x7fffffffL) return hipErrorInvalidValue;
    // up to two workgroups' worth of tiles per CU at once; beyond that a workgroup walks several tiles
    long groups = (2L * compute_units() + n_cb - 1) / n_cb;
    if (groups > n_tiles) groups = n_tiles;
    if (groups < 1) groups = 1;
    constexpr int kTileBytes = (KC / 2) * kSlabBytes * ((kAtt && Traits<T>::kHiLo) ? 2 : 1);
    constexpr int kLds = kTileBytes > 4 * kSmallChanBlock * 128 ? kTileBytes : 4 * kSmallChanBlock * 128;   // tile(s), or a round of weights
    const hipError_t e = allow_dynamic_lds<small_project_kernel<T, KC, kAtt, Dest>>(kLds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((small_project_kernel<T, KC, kAtt, Dest>), dim3((unsigned)(groups * n_cb)),
                       dim3(kSmallThreads), kLds, stream, (const T*)src, (const T*)w, dest, aa, n_tokens, K, c_out,
                       n_cb, n_tiles, tiles_per_image);
    return hipGetLastError();
}

template <class T, bool kAtt, class Dest>
hipError_t run_small_k(const void* src, const void* w, Dest dest, SmallAttArgs aa, long n_tokens, int K, int c_out,
                       long n_tiles, int tiles_per_image, hipStream_t stream) {
    if (K <= 512) return run_small<T, 16, kAtt, Dest>(src, w, dest, aa, n_tokens, K, c_out, n_tiles, tiles_per_image, stream);
    if (K <= 768) return run_small<T, 24, kAtt, Dest>(src, w, dest, aa, n_tokens, K, c_out, n_tiles, tiles_per_image, stream);
    if (K <= 1024) return run_small<T, 32, kAtt, Dest>(src, w, dest, aa, n_tokens, K, c_out, n_tiles, tiles_per_image, stream);
    return hipErrorNotSupported;
}

}  // namespace

hipError_t launch_small_linear(int dt, const void* x, const void* w, void* y, long n_tokens, int c_in, int c_out,
                               hipStream_t stream) {
    const long n_tiles = (n_tokens + kSmallTB - 1) / kSmallTB;
    const SmallAttArgs none = {nullptr, nullptr, 0, 0, 0.f};
    switch (dt) {
        case 1: return run_small_k<_Float16, false>(x, w, SmallPlain<_Float16>{(_Float16*)y, c_out}, none, n_tokens, c_in, c_out, n_tiles, 0, stream);
        case 2: return run_small_k<__bf16, false>(x, w, SmallPlain<__bf16>{(__bf16*)y, c_out}, none, n_tokens, c_in, c_out, n_tiles, 0, stream);
    }
    return hipErrorNotSupported;
}

hipError_t launch_small_qkv_project(int dt, const void* x, const void* w_qkv, void* q_ms, long q_ms_stride,
                                    void* kv_raw, long kv_tok_stride, long kv_head_stride, long n_tokens, int c_in,
                                    int heads, hipStream_t stream) {
    const long n_tiles = (n_tokens + kSmallTB - 1) / kSmallTB;
    const SmallAttArgs none = {nullptr, nullptr, 0, 0, 0.f};
    const int c_out = 3 * heads * 16;
    switch (dt) {
        case 1: return run_small_k<_Float16, false>(x, w_qkv, SmallQkv<_Float16>{(_Float16*)q_ms, q_ms_stride, (_Float16*)kv_raw, kv_tok_stride, kv_head_stride}, none, n_tokens, c_in, c_out, n_tiles, 0, stream);
        case 2: return run_small_k<__bf16, false>(x, w_qkv, SmallQkv<__bf16>{(__bf16*)q_ms, q_ms_stride, (__bf16*)kv_raw, kv_tok_stride, kv_head_stride}, none, n_tokens, c_in, c_out, n_tiles, 0, stream);
    }
    return hipErrorNotSupported;
}

hipError_t launch_small_apply_project(int dt, const void* q_ms, const void* kvfrag, const float* kvscale,
                                      const void* w_proj, void* out, const void* res, long n_tokens, int tokens_per_image,
                                      int n_hb, int c_out, float eps, hipStream_t stream) {
    const int N = tokens_per_image;
    const int tpi = (N + kSmallTB - 1) / kSmallTB;
    const long n_tiles = (n_tokens / N) * tpi;
    const SmallAttArgs aa = {(const char*)kvfrag, kvscale, N, n_hb, eps};
    const int K = n_hb * 16;
    switch (dt) {
        case 1: return run_small_k<_Float16, true>(q_ms, w_proj, SmallPlain<_Float16>{(_Float16*)out, c_out, (const _Float16*)res}, aa, n_tokens, K, c_out, n_tiles, tpi, stream);
        case 2: return run_small_k<__bf16, true>(q_ms, w_proj, SmallPlain<__bf16>{(__bf16*)out, c_out, (const __bf16*)res}, aa, n_tokens, K, c_out, n_tiles, tpi, stream);
    }
    return hipErrorNotSupported;
}

}  // namespace msla
