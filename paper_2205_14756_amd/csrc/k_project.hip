// 1x1 projections  y[n, o] = sum_c x[n, c] * w[o, c]  (Section 3.1: Q = x W_Q,
// K = x W_K, V = x W_V; also the stand-alone form of the final projection).
// Two forms: a tiled one (256 output channels x 128 tokens per workgroup, any contraction length,
// every storage type) and, for 16-bit types with at most 256 contraction slots, a weight-stationary
// one that keeps the weights in registers and streams the tokens.
#include "gemm_tile.h"
#include "msla_kernels.h"

#ifndef MSLA_PROJ_WR
#define MSLA_PROJ_WR 4
#define MSLA_PROJ_WC 2
#endif

#ifndef MSLA_WS_IO
#define MSLA_WS_IO 3
#endif
#ifndef MSLA_WS_RESIDENT
#define MSLA_WS_RESIDENT 2
#endif
#ifndef MSLA_PROJ_BARRIER_AT
#define MSLA_PROJ_BARRIER_AT 0
#endif

namespace msla {
namespace {

template <class T>
using ProjTile = GemmTile<T, MSLA_PROJ_WR, MSLA_PROJ_WC>;

// Where the projection writes, and in which order it walks the weight rows.  tile(tok0) gives the
// writer for the token tile starting at tok0: buffer resources based at that token, so offsets fit
// 32 bits and rows past the last token are dropped by the range check.
template <class T>
struct PlainDest {
    T* y;
    long n_tokens;
    int c_out;
    // optional residual [n_tokens, c_out] that the tiled kernel adds to the fp32 sums before their one
    // rounding (y = res + x w^T); nullptr: none
    const T* res = nullptr;
    // optional activation applied to the fp32 sums before their one rounding: -1 none, 0 ReLU,
    // 1 hard-swish a * clip(a + 3, 0, 6) / 6, evaluated as a * clip(a / 6 + 1/2, 0, 1) (the FFN's expand projection)
    int act = -1;
    __host__ __device__ __forceinline__ bool has_residual() const { return res != nullptr; }
    // 16 bytes of the residual at (token, channel), zero past the ends
    __device__ __forceinline__ u32x4 residual16(long tok, int oc) const {
        u32x4 r = {0u, 0u, 0u, 0u};
        if (tok < n_tokens && oc < c_out) r = *(const u32x4*)(res + tok * c_out + oc);
        return r;
    }
    __device__ __forceinline__ f32x4 activate(f32x4 v) const {
        if (act == 0) {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = fmaxf(v[e], 0.f);
        } else if (act == 1) {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = v[e] * __builtin_amdgcn_fmed3f(fmaf(v[e], 1.0f / 6.0f, 0.5f), 0.f, 1.f);
        }
        return v;
    }
    struct Tile {
        BufRsrc y;
        unsigned row_bytes;
        int c_out;
        __device__ __forceinline__ void store(int, int, int row, int oc, u32x4 v) const {
            buf_store16(y, oc < c_out ? row * row_bytes + oc * (unsigned)sizeof(T) : kOobOffset, v);
        }
    };
    __device__ __forceinline__ int row_of(int oc) const { return oc; }
    __device__ __forceinline__ Tile tile(long tok0) const {
        const long rb = (long)c_out * (long)sizeof(T);
        return Tile{make_rsrc(y + tok0 * c_out, (n_tokens - tok0) * rb), (unsigned)rb, c_out};
    }
    // a writer that drops everything (what the pipelined epilogue holds before its first tile)
    __device__ __forceinline__ Tile none() const { return Tile{make_rsrc(y, 0), 0u, c_out}; }
    // A lane's part of a store that does not change from tile to tile: its byte offset inside a
    // group of 16 token rows (beyond every resource where the lane has nothing to write).
    struct Lane {
        unsigned off;
    };
    __device__ __forceinline__ Lane lane(int row, int oc, bool live) const {
        return Lane{live && oc < c_out ? (unsigned)row * (unsigned)(c_out * sizeof(T)) + oc * (unsigned)sizeof(T) : kOobOffset};
    }
    // (piece0 .. piece_end: the channels the storing wave covers; local0: the stored piece's first
    // channel counted from the wave's first -- both unused here)
    static __device__ __forceinline__ void store(const Tile& t, const Lane& l, int, int, int, int row0, u32x4 v) {
        buf_store16_at(t.y, l.off, (unsigned)row0 * t.row_bytes, v);
    }
};

// Q/K/V projection with split destinations.  The kernel walks the output channels in DESTINATION
// order -- first the Ct channels of Q (head-major), then the 2*Ct channels of K|V, head by head --
// so a tile's channels of one token are few contiguous runs in memory; row_of maps such a channel
// to its row (h*3 + t)*16 + e of w_qkv.
// The K|V map holds, for token n and head h, 32 contiguous channels (K then V) at
//   kv_raw + n * kv_tok_stride + h * kv_head_stride          (elements)
// -- token-major (2*Ct, 32) or head-major (32, padded token count * 32).  Head-major is what the
// aggregation pass reads best (a head's tokens are contiguous); its token count is padded to whole
// tiles, so the rows of a ragged last tile fall into the padding.  kv_span is the size of the map;
// a head-major map must stay below 2^31 bytes (32-bit offsets inside a tile's resource).
template <class T>
struct QkvSplitDest {
    __host__ __device__ __forceinline__ bool has_residual() const { return false; }
    __device__ __forceinline__ u32x4 residual16(long, int) const { return u32x4{0u, 0u, 0u, 0u}; }
    __device__ __forceinline__ f32x4 activate(f32x4 v) const { return v; }
    T* q_ms;
    long q_ms_stride;
    T* kv_raw;
    long kv_tok_stride, kv_head_stride, kv_span;
    long n_tokens;
    int Ct;
    struct Tile {
        BufRsrc q, kv;
        unsigned q_row_bytes, kv_row_bytes, kv_head_bytes;
        int Ct;
        int rows;       // tokens from this tile's first to the map's last
        __device__ __forceinline__ unsigned kv_off(int row, int vc) const {
            const int v2 = vc - Ct;
            return (unsigned)row * kv_row_bytes + (unsigned)(v2 >> 5) * kv_head_bytes + (unsigned)(v2 & 31) * (unsigned)sizeof(T);
        }
        __device__ __forceinline__ void store(int piece0, int piece_end, int row, int vc, u32x4 v) const {
            constexpr unsigned sz = (unsigned)sizeof(T);
            if (piece0 < Ct) buf_store16(q, vc < Ct ? row * q_row_bytes + vc * sz : kOobOffset, v);
            // (a row past the last token would not leave a head-major map's resource: it is masked here)
            if (piece_end > Ct) buf_store16(kv, (vc >= Ct && vc < 3 * Ct && row < rows) ? kv_off(row, vc) : kOobOffset, v);
        }
    };
    __device__ __forceinline__ int row_of(int vc) const {
        if (vc < Ct) return (vc >> 4) * 48 + (vc & 15);
        const int v2 = vc - Ct;
        return (v2 >> 5) * 48 + 16 + (v2 & 31);
    }
    __device__ __forceinline__ Tile tile(long tok0) const {
        const long qb = q_ms_stride * (long)sizeof(T), kb = kv_tok_stride * (long)sizeof(T);
        return Tile{make_rsrc(q_ms + tok0 * q_ms_stride, (n_tokens - tok0) * qb),
                    make_rsrc(kv_raw + tok0 * kv_tok_stride, (kv_span - tok0 * kv_tok_stride) * (long)sizeof(T)),
                    (unsigned)qb, (unsigned)kb, (unsigned)(kv_head_stride * sizeof(T)), Ct,
                    (int)(n_tokens - tok0 < 0x7fffffffL ? n_tokens - tok0 : 0x7fffffffL)};
    }
    __device__ __forceinline__ Tile none() const {
        return Tile{make_rsrc(q_ms, 0), make_rsrc(kv_raw, 0), 0u, 0u, 0u, Ct, 0};
    }
    struct Lane {
        unsigned q, kv;
    };
    __device__ __forceinline__ Lane lane(int row, int vc, bool live) const {
        constexpr unsigned sz = (unsigned)sizeof(T);
        const unsigned qb = (unsigned)(q_ms_stride * sizeof(T)), kb = (unsigned)(kv_tok_stride * sizeof(T));
        const unsigned hb = (unsigned)(kv_head_stride * sizeof(T));
        const int v2 = vc - Ct;
        return Lane{live && vc < Ct ? (unsigned)row * qb + vc * sz : kOobOffset,
                    live && vc >= Ct && vc < 3 * Ct ? (unsigned)row * kb + (unsigned)(v2 >> 5) * hb + (unsigned)(v2 & 31) * sz
                                                   : kOobOffset};
    }
    // piece0 .. piece_end: the wave's channel range, which tells (wave-uniformly) which maps it touches
    static __device__ __forceinline__ void store(const Tile& t, const Lane& l, int piece0, int piece_end, int, int row0, u32x4 v) {
        if (piece0 < t.Ct) buf_store16_at(t.q, l.q, (unsigned)row0 * t.q_row_bytes, v);
        if (piece_end > t.Ct) buf_store16_at(t.kv, l.kv, (unsigned)row0 * t.kv_row_bytes, v);
    }
};

// The same destinations for the weight-stationary kernel with 48 channels a wave: a wave is one
// head, and its three 16-channel blocks are that head's K, V and Q in this order.  K and V then
// pair up into one store of a token's 64-byte K|V run -- with a head-major map sixteen tokens' runs
// are one contiguous kilobyte -- the Q block pairs its two token groups, and which map a store
// goes to is known when the kernel is compiled: no branches, one offset a lane.
template <class T>
struct QkvHeadDest {
    __host__ __device__ __forceinline__ bool has_residual() const { return false; }
    __device__ __forceinline__ u32x4 residual16(long, int) const { return u32x4{0u, 0u, 0u, 0u}; }
    __device__ __forceinline__ f32x4 activate(f32x4 v) const { return v; }
    T* q_ms;
    long q_ms_stride;
    T* kv_raw;
    long kv_tok_stride, kv_head_stride, kv_span;
    long n_tokens;
    int Ct;
    struct Tile {
        BufRsrc q, kv;
        unsigned q_row_bytes, kv_row_bytes;
    };
    // channel vc of the walk = (head vc / 48, r = vc % 48): r < 32 is K|V channel r, else Q channel r - 32
    __device__ __forceinline__ int row_of(int vc) const {
        const int head = vc / 48, r = vc - head * 48;
        return head * 48 + (r < 32 ? 16 + r : r - 32);
    }
    __device__ __forceinline__ Tile tile(long tok0) const {
        const long qb = q_ms_stride * (long)sizeof(T), kb = kv_tok_stride * (long)sizeof(T);
        return Tile{make_rsrc(q_ms + tok0 * q_ms_stride, (n_tokens - tok0) * qb),
                    make_rsrc(kv_raw + tok0 * kv_tok_stride, (kv_span - tok0 * kv_tok_stride) * (long)sizeof(T)),
                    (unsigned)qb, (unsigned)kb};
    }
    __device__ __forceinline__ Tile none() const { return Tile{make_rsrc(q_ms, 0), make_rsrc(kv_raw, 0), 0u, 0u}; }
    struct Lane {
        unsigned off;
    };
    __device__ __forceinline__ Lane lane(int row, int vc, bool live) const {
        constexpr unsigned sz = (unsigned)sizeof(T);
        const int head = vc / 48, r = vc - head * 48;
        if (!live || vc >= 3 * Ct) return Lane{kOobOffset};
        if (r < 32)
            return Lane{(unsigned)row * (unsigned)(kv_tok_stride * sizeof(T)) +
                        (unsigned)head * (unsigned)(kv_head_stride * sizeof(T)) + (unsigned)r * sz};
        return Lane{(unsigned)row * (unsigned)(q_ms_stride * sizeof(T)) + (unsigned)(head * 16 + r - 32) * sz};
    }
    static __device__ __forceinline__ void store(const Tile& t, const Lane& l, int, int, int local0, int row0, u32x4 v) {
        if (local0 < 32) buf_store16_at(t.kv, l.off, (unsigned)row0 * t.kv_row_bytes, v);
        else buf_store16_at(t.q, l.off, (unsigned)row0 * t.q_row_bytes, v);
    }
};

// Persistent workgroups: each takes a contiguous run of (token tile, channel block) tiles, channel
// block fastest, so the token tile it re-reads for the next channel block is still in its CU's
// cache, and consecutive workgroups (= one XCD, see xcd_remap) share the weights in one L2.
// The (tile, 128-byte contraction slab) pairs form one flat software pipeline over two LDS
// buffers and two register sets: in the step that computes slab g, slab g+1 (requested one step
// earlier) is parked in the other LDS buffer and slab g+2 is requested.  All global accesses go
// through range-checked buffer resources with per-thread offsets that are fixed for a tile, so a
// step's instruction stream is little more than its loads, LDS traffic and matrix instructions.
// Requires c_out * c_in * sizeof(T) < 2^31 (the weights are one resource).
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
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wr = wave % MSLA_PROJ_WR, wc = wave / MSLA_PROJ_WR;
    const int slabs = (c_in + G::BK - 1) / G::BK;
    const unsigned row_bytes = (unsigned)c_in * (unsigned)sizeof(T);

    f32x4 acc[4][4];
    G::zero(acc);

    // (channel block, token block) of the tile being computed and of the tile being fetched; kept
    // as counters so that the loop contains no division
    int rb = (int)(tile_begin % n_rb), nrb = rb;
    long cb = tile_begin / n_rb, ncb = cb;
    long left = tile_end - tile_begin;      // tiles still to compute
    long nleft = left;                      // tiles still to fetch
    int slab = 0, nslab = 0;

    // Every thread fetches the same (row, 16-byte column) cells of each slab: kVecR weight vectors,
    // then kVecC token vectors.
    constexpr int kVecs = G::kVecR + G::kVecC;
    static_assert(kVecs <= 8, "the step interleaves at most 8 loads and 8 LDS stores with its MFMAs");
    struct Regs {
        u32x4 v[kVecs];
    };
    const unsigned col_bytes = (threadIdx.x & 7) * 16;
    const BufRsrc wres = make_rsrc(w, (long)c_out * row_bytes);
    BufRsrc xres = wres;
    unsigned off[kVecs];
#pragma unroll
    for (int i = 0; i < G::kVecC; ++i)
        off[G::kVecR + i] = ((threadIdx.x + i * G::kThreads) >> 3) * row_bytes + col_bytes;
    // offsets and resources of the tile (nrb, ncb) that is fetched next
    auto aim = [&]() {
#pragma unroll
        for (int i = 0; i < G::kVecR; ++i) {
            const int row = nrb * G::BR + ((threadIdx.x + i * G::kThreads) >> 3);
            off[i] = row < c_out ? (unsigned)ep.row_of(row) * row_bytes + col_bytes : kOobOffset;
        }
        const long tok0 = ncb * G::BC;
        xres = make_rsrc(x + tok0 * c_in, (n_tokens - tok0) * (long)row_bytes);
    };
    // The loads of one slab are issued one by one (so that they can be spread between matrix
    // instructions); a lane whose cell lies beyond the contraction length, or any lane once all
    // slabs have been requested, uses an out-of-range offset and gets zeros without a memory access.
    int kb = 0;
    bool kin = true;
    auto fetch_begin = [&]() {
        kb = nslab * 128;
        kin = nleft > 0 && kb + col_bytes < row_bytes;
    };
    auto fetch_one = [&](Regs& r, int i) {
        r.v[i] = buf_load16(i < G::kVecR ? wres : xres, kin ? off[i] : kOobOffset, kb);
    };
    auto fetch_end = [&]() {
        if (nleft > 0 && ++nslab == slabs) {
            nslab = 0;
            --nleft;
            if (++nrb == n_rb) { nrb = 0; ++ncb; }
            if (nleft > 0) aim();
        }
    };
    auto park_one = [&](char* buf, const Regs& r, int i) {
        if (i < G::kVecR) G::store_lds_one(buf, r.v[i], i);
        else G::store_lds_one(buf + G::kLdsR, r.v[i], i - G::kVecR);
    };

    int cur = 0;
    typename G::Frags f0, f1;
    // One pipeline step.  On entry slab g is in LDS buffer `cur` and its first-half operand
    // fragments are already in f0; slab g+1 sits in `held`; slab g+2 is requested now into `spare`.
    // A wave issues its instructions in order and an LDS or memory instruction waits for room in
    // that unit's queue, so a block of them ahead of the matrix instructions would keep the matrix
    // cores idle while the queues drain: they are dealt out one per MFMA instead.  Everything is
    // unconditional (past the last slab the stores park stale registers in the buffer nobody reads
    // and the fragment reads fetch unused data), so each half of the step is straight-line code;
    // there is one workgroup barrier per slab.
    auto step = [&](Regs& held, Regs& spare) {
        char* here = lds + cur * kBuf;
        char* next = lds + (cur ^ 1) * kBuf;
        fetch_begin();
#pragma unroll
        for (int m = 0; m < 16; ++m) {
            acc[m >> 2][m & 3] = Traits<T>::mma_vec(acc[m >> 2][m & 3], f0.a[m >> 2], f0.b[m & 3]);
            if (m < 4) f1.a[m] = G::load_frag_lds(here, wr * 64 + m * 16, 1);
            else if (m < 8) f1.b[m - 4] = G::load_frag_lds(here + G::kLdsR, wc * 64 + (m - 4) * 16, 1);
            if (m < kVecs) fetch_one(spare, m);
            if (m >= 8 && m - 8 < kVecs) park_one(next, held, m - 8);
            __builtin_amdgcn_sched_barrier(0);
        }
        fetch_end();
#pragma unroll
        for (int m = 0; m < 16; ++m) {
            if (m == MSLA_PROJ_BARRIER_AT) __syncthreads();
            acc[m >> 2][m & 3] = Traits<T>::mma_vec(acc[m >> 2][m & 3], f1.a[m >> 2], f1.b[m & 3]);
            constexpr int r0 = MSLA_PROJ_BARRIER_AT;
            if (m >= r0 && m < r0 + 4) f0.a[m - r0] = G::load_frag_lds(next, wr * 64 + (m - r0) * 16, 0);
            else if (m >= r0 + 4 && m < r0 + 8) f0.b[m - r0 - 4] = G::load_frag_lds(next + G::kLdsR, wc * 64 + (m - r0 - 4) * 16, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        cur ^= 1;
        if (++slab == slabs) {
            // every wave finished reading the buffer just consumed before the barrier above, and it is
            // not refilled before the next step: stage the results there
            {
#pragma unroll
                for (int io = 0; io < 4; ++io)
#pragma unroll
                    for (int jt = 0; jt < 4; ++jt) acc[io][jt] = ep.activate(acc[io][jt]);
            }
            if (ep.has_residual()) {
                const long tok0 = (long)cb * G::BC;
                G::epilogue_lds_residual(acc, here, rb * G::BR, wr, wc, ep.tile(tok0),
                                         [&](int row, int oc) { return ep.residual16(tok0 + row, oc); });
            } else {
                G::epilogue_lds(acc, here, rb * G::BR, wr, wc, ep.tile(cb * G::BC));
            }
            G::zero(acc);
            slab = 0;
            --left;
            if (++rb == n_rb) { rb = 0; ++cb; }
            __syncthreads();     // nobody refills that buffer while a wave still stages in it
        }
    };

    Regs ra, rb2;
    aim();
    fetch_begin();
#pragma unroll
    for (int i = 0; i < kVecs; ++i) fetch_one(ra, i);
    fetch_end();
#pragma unroll
    for (int i = 0; i < kVecs; ++i) park_one(lds, ra, i);
    fetch_begin();                           // slab 1 -> held by ra
#pragma unroll
    for (int i = 0; i < kVecs; ++i) fetch_one(ra, i);
    fetch_end();
    __syncthreads();
    G::load_frags(f0.a, f0.b, lds, lds + G::kLdsR, wr, wc, 0);
    while (left > 0) {
        step(ra, rb2);
        if (left <= 0) break;
        step(rb2, ra);
    }
}

// ---------------------------------------------------------------- weight-stationary form
// When a weight row is at most 512 bytes (the contraction is short, as in this module's 1x1
// projections), a wave keeps its 48 output channels' weights in registers for the whole kernel --
// KCH operand fragments per 16 channels -- and only the tokens stream: a workgroup of 4 waves owns
// 192 channels and walks over token tiles of 32.  A tile is copied HBM -> registers -> LDS once
// (double-buffered, one barrier per tile) and every wave reads all of it as MFMA operands.
// Against the tiled form above this moves a fraction of the bytes through LDS and L2 per
// multiply-add and needs no weight traffic in the loop at all.  Two such workgroups share a CU
// (one wave of each per SIMD); they drift apart, so one's barrier and result stores are covered
// by the other's matrix instructions.
template <class T, int KCH, int IO_ = MSLA_WS_IO>
struct WsShape {
    static_assert(sizeof(T) == 2 && KCH % 2 == 0, "16-bit elements, whole 128-byte slabs");
    static constexpr int kWaves = 4, kThreads = 256, kResident = MSLA_WS_RESIDENT;
    static constexpr int IO = IO_;                       // 16-channel groups per wave
    static constexpr int JT = 2;                         // 16-token groups per tile
    static constexpr int kChanWave = IO * 16, kChanBlock = kWaves * kChanWave;
    static constexpr int TB = JT * 16;                   // tokens per tile
    static constexpr int NS = KCH / 2;                   // 128-byte slabs per token row
    static constexpr int kRow = 160;                     // LDS row pitch of a slab (full-rate reads and writes)
    static constexpr int kSlab = TB * kRow;
    static constexpr int kBuf = NS * kSlab;
    static constexpr int kWeightStage = kChanBlock * kRow;        // one slab of the workgroup's weight rows
    static constexpr int kLds = 2 * kBuf > kWeightStage ? 2 * kBuf : kWeightStage;
    static_assert(TB * 8 == kThreads, "one 16-byte vector per thread and slab");
};

template <class T, int KCH, int IO, class Epilogue>
__global__ __launch_bounds__(256, MSLA_WS_RESIDENT) void project_ws_kernel(const T* __restrict__ x, const T* __restrict__ w,
                                                         long n_tokens, int c_in, int c_out, int n_cg,
                                                         long n_tt, long tiles_per_block, Epilogue ep) {
    typedef WsShape<T, KCH, IO> S;
    typedef typename Traits<T>::Vec Vec;
    extern __shared__ __attribute__((aligned(16))) char lds[];

    const unsigned L = xcd_remap(blockIdx.x, gridDim.x);
    const int cg = (int)(L % (unsigned)n_cg);
    const long t_begin = (long)(L / (unsigned)n_cg) * tiles_per_block;
    const long t_end = t_begin + tiles_per_block < n_tt ? t_begin + tiles_per_block : n_tt;
    if (t_begin >= t_end) return;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = lane_id(), x16 = lane & 15, q = lane >> 4;
    const unsigned row_bytes = (unsigned)c_in * 2u;
    const int ch0 = cg * S::kChanBlock + wave * S::kChanWave;     // this wave's first channel

    // token tile copy: thread = (row tid/8, 16-byte chunk tid%8) of each of the NS slabs
    const unsigned g_off = (threadIdx.x >> 3) * row_bytes + (threadIdx.x & 7) * 16;
    const unsigned l_off = (threadIdx.x >> 3) * S::kRow + (threadIdx.x & 7) * 16;
    u32x4 regs[S::NS];
    auto fetch = [&](long tile) {
        const long tok0 = tile * S::TB;
        const BufRsrc xres = make_rsrc(x + tok0 * c_in, tile < t_end ? (n_tokens - tok0) * (long)row_bytes : 0);
#pragma unroll
        for (int i = 0; i < S::NS; ++i)
            regs[i] = buf_load16(xres, (i * 128 + (threadIdx.x & 7) * 16 < row_bytes) ? g_off + i * 128 : kOobOffset, 0);
    };
    auto park = [&](char* buf) {
#pragma unroll
        for (int i = 0; i < S::NS; ++i) *(u32x4*)(buf + i * S::kSlab + l_off) = regs[i];
    };
    fetch(t_begin);     // requested ahead of the weights, so the first tile does not queue behind them

    // The weights: fragment (io, kk) = rows ch0 + io*16 + x16, contraction slots kk*32 + q*8 .. +7.
    // Read straight from memory in that shape every lane would touch its own cache line (64 address
    // cycles per instruction), so the workgroup's rows are copied slab by slab in row order -- 8 lanes
    // per 128-byte row segment -- through the token buffers, and picked up as fragments from there.
    Vec wf[S::IO][KCH];
    {
        const BufRsrc wres = make_rsrc(w, (long)c_out * row_bytes);
        constexpr int kWV = S::kChanBlock * 8 / S::kThreads;      // vectors per thread and slab: 6
        u32x4 wr[S::NS][kWV];
        unsigned base[kWV];
#pragma unroll
        for (int i = 0; i < kWV; ++i) {
            const int row = cg * S::kChanBlock + ((threadIdx.x + i * S::kThreads) >> 3);
            base[i] = row < c_out ? (unsigned)ep.row_of(row) * row_bytes + (threadIdx.x & 7) * 16 : kOobOffset;
        }
        // (the requests run two slabs ahead of the staging: the address path is busy with them for
        // longer than the data takes to arrive, so staging a slab overlaps with requesting later ones)
        auto request = [&](int sl) {
#pragma unroll
            for (int i = 0; i < kWV; ++i)
                wr[sl][i] = buf_load16(wres, (base[i] != kOobOffset && sl * 128 + (threadIdx.x & 7) * 16 < row_bytes)
                                                 ? base[i] + sl * 128 : kOobOffset, 0);
        };
        constexpr int kAheadW = S::NS < 2 ? S::NS : 2;
#pragma unroll
        for (int sl = 0; sl < kAheadW; ++sl) request(sl);
#pragma unroll
        for (int sl = 0; sl < S::NS; ++sl) {
            if (sl) __syncthreads();
#pragma unroll
            for (int i = 0; i < kWV; ++i)
                *(u32x4*)(lds + ((threadIdx.x + i * S::kThreads) >> 3) * S::kRow + (threadIdx.x & 7) * 16) = wr[sl][i];
            if (sl + kAheadW < S::NS) request(sl + kAheadW);
            __syncthreads();
#pragma unroll
            for (int io = 0; io < S::IO; ++io)
#pragma unroll
                for (int h = 0; h < 2; ++h)
                    wf[io][2 * sl + h] = __builtin_bit_cast(
                        Vec, *(const u32x4*)(lds + (wave * S::kChanWave + io * 16 + x16) * S::kRow + (h * 4 + q) * 16));
        }
        __syncthreads();
    }

    f32x4 acc[S::IO][S::JT];
    const char* frag_base = lds + x16 * S::kRow + q * 16;

    // Results leave one tile late: a tile's accumulators are rounded into `pend`, and during the
    // NEXT tile's matrix instructions they are stored, a pair of fragments at a time -- a few small
    // jobs dealt out over the contraction chunks, so the wave issues matrix instructions all the
    // while.  Before the first tile `dest` is an empty resource.
    typedef typename Traits<T>::Frag Frag;
    Frag pend[S::IO][S::JT];
#pragma unroll
    for (int io = 0; io < S::IO; ++io)
#pragma unroll
        for (int jt = 0; jt < S::JT; ++jt) pend[io][jt] = frag_zero<T>();
    auto dest = ep.none();
    // A fragment is 8 bytes a lane: channels 4q..4q+3 of one 16-channel block for token x16.  Two of
    // them leave in one 16-byte store: the odd 16-lane groups of one are swapped with the even
    // groups of the other, after which a lane holds 8 consecutive channels.  Blocks 2m and 2m+1 of
    // the same 16 tokens pair up (the lane then has channels 32m + 16*(q%2) + 8*(q/2) .. +7 of token
    // x16); an odd block count leaves the last block, which pairs its two token groups instead
    // (channels 8*(q/2) .. +7 of token 16*(q%2) + x16).  The lane's store offsets are fixed for the
    // kernel.
    constexpr int kPairs = S::IO / 2;                         // channel-block pairs per token group
    constexpr int kJobs = S::JT * kPairs + (S::IO % 2) * (S::JT / 2);
    static_assert(S::JT % 2 == 0 && kJobs <= KCH, "one flush job per contraction chunk at most");
    typename Epilogue::Lane where_pair[kPairs > 0 ? kPairs : 1], where_last;
#pragma unroll
    for (int m = 0; m < kPairs; ++m)
        where_pair[m] = ep.lane(x16, ch0 + 32 * m + (q & 1) * 16 + (q >> 1) * 8, true);
    where_last = ep.lane((q & 1) * 16 + x16, ch0 + (S::IO - 1) * 16 + (q >> 1) * 8, true);
    auto flush_job = [&](int job) {
        u32x2 even, odd;
        const bool last = job >= S::JT * kPairs;              // the unpaired block, two token groups
        const int jt = last ? 2 * (job - S::JT * kPairs) : job / (kPairs > 0 ? kPairs : 1);
        const int m = last ? 0 : job % (kPairs > 0 ? kPairs : 1);
        if (last) {
            even = __builtin_bit_cast(u32x2, pend[S::IO - 1][jt]);
            odd = __builtin_bit_cast(u32x2, pend[S::IO - 1][jt + 1]);
        } else {
            even = __builtin_bit_cast(u32x2, pend[2 * m][jt]);
            odd = __builtin_bit_cast(u32x2, pend[2 * m + (S::IO > 1 ? 1 : 0)][jt]);
        }
        const u32x2 s0 = __builtin_amdgcn_permlane16_swap(even[0], odd[0], false, false);
        const u32x2 s1 = __builtin_amdgcn_permlane16_swap(even[1], odd[1], false, false);
        const u32x4 v = {s0[0], s1[0], s0[1], s1[1]};
        if (last) Epilogue::store(dest, where_last, ch0 + (S::IO - 1) * 16, ch0 + S::IO * 16, (S::IO - 1) * 16, jt * 16, v);
        else Epilogue::store(dest, where_pair[m], ch0 + 32 * m, ch0 + 32 * m + 32, 32 * m, jt * 16, v);
    };

    park(lds);
    __syncthreads();
    int cur = 0;
    for (long tile = t_begin; tile < t_end; ++tile) {
        const char* here = frag_base + cur * S::kBuf;
        fetch(tile + 1);                       // past the end: a zero-length resource, no traffic
#pragma unroll
        for (int io = 0; io < S::IO; ++io)
#pragma unroll
            for (int jt = 0; jt < S::JT; ++jt) acc[io][jt] = f32x4{0.f, 0.f, 0.f, 0.f};
        // token operand fragments, requested two contraction chunks ahead of their use
        Vec bf[3][S::JT];
        auto read_b = [&](int kk) {
#pragma unroll
            for (int jt = 0; jt < S::JT; ++jt)
                bf[kk % 3][jt] = __builtin_bit_cast(
                    Vec, *(const u32x4*)(here + (kk >> 1) * S::kSlab + jt * 16 * S::kRow + (kk & 1) * 64));
        };
        read_b(0);
        read_b(1);
        static_for<0, KCH>([&](auto kk_c) {
            constexpr int kk = decltype(kk_c)::value;
            if constexpr (kk + 2 < KCH) read_b(kk + 2);
#pragma unroll
            for (int io = 0; io < S::IO; ++io)
#pragma unroll
                for (int jt = 0; jt < S::JT; ++jt)
                    acc[io][jt] = Traits<T>::mma_vec(acc[io][jt], wf[io][kk], bf[kk % 3][jt]);
            // the previous tile's results: job j rides in the middle of the j-th of kJobs runs of chunks
            static_for<0, kJobs>([&](auto job_c) {
                constexpr int job = decltype(job_c)::value;
                if constexpr ((2 * job + 1) * KCH / (2 * kJobs) == kk) flush_job(job);
            });
            __builtin_amdgcn_sched_barrier(0);
        });
        park(lds + (cur ^ 1) * S::kBuf);       // the other buffer was last read before the previous barrier
#pragma unroll
        for (int io = 0; io < S::IO; ++io)
#pragma unroll
            for (int jt = 0; jt < S::JT; ++jt) pend[io][jt] = frag_from_f32<T>(ep.activate(acc[io][jt]));
        dest = ep.tile(tile * S::TB);
        __syncthreads();
        cur ^= 1;
    }
#pragma unroll
    for (int job = 0; job < kJobs; ++job) flush_job(job);
}

template <class T, int KCH, int IO, class Epilogue>
hipError_t run_project_ws(const void* x, const void* w, long n_tokens, int c_in, int c_out, Epilogue ep,
                          hipStream_t stream) {
    typedef WsShape<T, KCH, IO> S;
    const int n_cg = (c_out + S::kChanBlock - 1) / S::kChanBlock;
    const long n_tt = (n_tokens + S::TB - 1) / S::TB;
    if (n_tt <= 0 || n_tt * n_cg > 0x7fffffffL) return hipErrorInvalidValue;
    if ((long)c_out * c_in * 2 >= 0x7fffffffL) return hipErrorInvalidValue;
    // kResident workgroups per CU; the channel groups of one token range sit next to each other
    const long slots = (long)compute_units() * S::kResident;
    const long groups = slots / n_cg > 0 ? slots / n_cg : 1;
    const long tiles_per_block = (n_tt + groups - 1) / groups;
    const long nblocks = (n_tt + tiles_per_block - 1) / tiles_per_block * n_cg;
    const hipError_t e = allow_dynamic_lds<project_ws_kernel<T, KCH, IO, Epilogue>>(S::kLds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((project_ws_kernel<T, KCH, IO, Epilogue>), dim3((unsigned)nblocks), dim3(S::kThreads), S::kLds,
                       stream, (const T*)x, (const T*)w, n_tokens, c_in, c_out, n_cg, n_tt, tiles_per_block, ep);
    return hipGetLastError();
}

#ifndef MSLA_PROJ_RESIDENT
#define MSLA_PROJ_RESIDENT 1
#endif

template <class T, class Epilogue>
hipError_t run_project(const void* x, const void* w, long n_tokens, int c_in, int c_out, Epilogue ep,
                       hipStream_t stream) {
    if constexpr (sizeof(T) == 2) {
        // short contraction: weights stay in registers
#ifndef MSLA_PROJ_NO_WS
        if (!ep.has_residual()) {      // (the weight-stationary form has no residual path)
            // 64 channels a wave where that divides the output and 48 does not (the FFN's expand projection:
            // 1024 channels are four such workgroups instead of five and a third of the 48-channel kind;
            // 42 against 57 us there, 24 against 31 at 512 channels, but 39.5 against 37 at 768), else 48
            if (c_out % 256 == 0 && c_out % 192 != 0) {
                if (c_in <= 128) return run_project_ws<T, 4, 4, Epilogue>(x, w, n_tokens, c_in, c_out, ep, stream);
                if (c_in <= 256) return run_project_ws<T, 8, 4, Epilogue>(x, w, n_tokens, c_in, c_out, ep, stream);
            }
            if (c_in <= 128) return run_project_ws<T, 4, MSLA_WS_IO, Epilogue>(x, w, n_tokens, c_in, c_out, ep, stream);
            if (c_in <= 256) return run_project_ws<T, 8, MSLA_WS_IO, Epilogue>(x, w, n_tokens, c_in, c_out, ep, stream);
        }
#endif
    }
    typedef ProjTile<T> G;
    const int n_rb = (c_out + G::BR - 1) / G::BR;
    const long n_cb = (n_tokens + G::BC - 1) / G::BC;
    const long n_tiles = n_cb * n_rb;
    if (n_tiles <= 0 || n_tiles > 0x7fffffffL) return hipErrorInvalidValue;
    // the weights are addressed with 32-bit byte offsets from their base, a token tile's rows too
    if ((long)c_out * c_in * (long)sizeof(T) >= 0x7fffffffL) return hipErrorInvalidValue;
    // one resident workgroup per CU (two LDS buffers of 60 KB); whole channel-block groups per workgroup
    const long cus = (long)compute_units() * MSLA_PROJ_RESIDENT;
    long per = (n_tiles + cus - 1) / cus;
    if (per > n_rb) per = (per + n_rb - 1) / n_rb * n_rb;     // small problems: spread the tiles instead
    const long nblocks = (n_tiles + per - 1) / per;
    constexpr int kLds = 2 * (G::kLdsR + G::kLdsC);
    const hipError_t e = allow_dynamic_lds<project_kernel<T, Epilogue>>(kLds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((project_kernel<T, Epilogue>), dim3((unsigned)nblocks), dim3(G::kThreads), kLds, stream,
                       (const T*)x, (const T*)w, n_tokens, c_in, c_out, n_rb, n_tiles, per, ep);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_linear(int dt, const void* x, const void* w, void* y, long n_tokens, int c_in, int c_out,
                         hipStream_t stream) {
    if (small_product(dt, n_tokens, c_in, c_out)) return launch_small_linear(dt, x, w, y, n_tokens, c_in, c_out, stream);
    switch (dt) {
        case 0: return run_project<float>(x, w, n_tokens, c_in, c_out, PlainDest<float>{(float*)y, n_tokens, c_out}, stream);
        case 1: return run_project<_Float16>(x, w, n_tokens, c_in, c_out, PlainDest<_Float16>{(_Float16*)y, n_tokens, c_out}, stream);
        case 2: return run_project<__bf16>(x, w, n_tokens, c_in, c_out, PlainDest<__bf16>{(__bf16*)y, n_tokens, c_out}, stream);
    }
    return hipErrorInvalidValue;
}

// y = act(x w^T) (the FFN's expand projection: act 0 ReLU, 1 hard-swish)
hipError_t launch_linear_act(int dt, const void* x, const void* w, void* y, long n_tokens, int c_in, int c_out, int act,
                             hipStream_t stream) {
    switch (dt) {
        case 0: return run_project<float>(x, w, n_tokens, c_in, c_out, PlainDest<float>{(float*)y, n_tokens, c_out, nullptr, act}, stream);
        case 1: return run_project<_Float16>(x, w, n_tokens, c_in, c_out, PlainDest<_Float16>{(_Float16*)y, n_tokens, c_out, nullptr, act}, stream);
        case 2: return run_project<__bf16>(x, w, n_tokens, c_in, c_out, PlainDest<__bf16>{(__bf16*)y, n_tokens, c_out, nullptr, act}, stream);
    }
    return hipErrorInvalidValue;
}

// y = res + x w^T (the FFN's hidden -> C projection with the block's residual: Section 3.1, Fig. 2 left)
hipError_t launch_linear_residual(int dt, const void* x, const void* w, const void* res, void* y, long n_tokens,
                                  int c_in, int c_out, hipStream_t stream) {
    switch (dt) {
        case 0: return run_project<float>(x, w, n_tokens, c_in, c_out, PlainDest<float>{(float*)y, n_tokens, c_out, (const float*)res}, stream);
        case 1: return run_project<_Float16>(x, w, n_tokens, c_in, c_out, PlainDest<_Float16>{(_Float16*)y, n_tokens, c_out, (const _Float16*)res}, stream);
        case 2: return run_project<__bf16>(x, w, n_tokens, c_in, c_out, PlainDest<__bf16>{(__bf16*)y, n_tokens, c_out, (const __bf16*)res}, stream);
    }
    return hipErrorInvalidValue;
}

template <class T>
hipError_t run_qkv_project(const void* x, const void* w_qkv, void* q_ms, long q_ms_stride, void* kv_raw,
                           long kv_tok_stride, long kv_head_stride, long kv_span, long n_tokens, int c_in, int heads,
                           hipStream_t stream) {
    const int c_out = 3 * heads * 16;
#ifndef MSLA_PROJ_NO_WS
    if constexpr (sizeof(T) == 2 && MSLA_WS_IO == 3) {
        // weight-stationary with one head a wave
        const QkvHeadDest<T> ep{(T*)q_ms, q_ms_stride, (T*)kv_raw, kv_tok_stride, kv_head_stride, kv_span, n_tokens, heads * 16};
        if (c_in <= 128) return run_project_ws<T, 4, 3, QkvHeadDest<T>>(x, w_qkv, n_tokens, c_in, c_out, ep, stream);
        if (c_in <= 256) return run_project_ws<T, 8, 3, QkvHeadDest<T>>(x, w_qkv, n_tokens, c_in, c_out, ep, stream);
    }
#endif
    return run_project<T>(x, w_qkv, n_tokens, c_in, c_out,
                          QkvSplitDest<T>{(T*)q_ms, q_ms_stride, (T*)kv_raw, kv_tok_stride, kv_head_stride, kv_span,
                                          n_tokens, heads * 16}, stream);
}

hipError_t launch_qkv_project(int dt, const void* x, const void* w_qkv, void* q_ms, long q_ms_stride,
                              void* kv_raw, long kv_tok_stride, long kv_head_stride, long kv_span,
                              long n_tokens, int c_in, int heads, hipStream_t stream) {
    if (small_product(dt, n_tokens, c_in, 3 * heads * 16))
        return launch_small_qkv_project(dt, x, w_qkv, q_ms, q_ms_stride, kv_raw, kv_tok_stride, kv_head_stride, n_tokens,
                                        c_in, heads, stream);
    switch (dt) {
        case 0: return run_qkv_project<float>(x, w_qkv, q_ms, q_ms_stride, kv_raw, kv_tok_stride, kv_head_stride, kv_span, n_tokens, c_in, heads, stream);
        case 1: return run_qkv_project<_Float16>(x, w_qkv, q_ms, q_ms_stride, kv_raw, kv_tok_stride, kv_head_stride, kv_span, n_tokens, c_in, heads, stream);
        case 2: return run_qkv_project<__bf16>(x, w_qkv, q_ms, q_ms_stride, kv_raw, kv_tok_stride, kv_head_stride, kv_span, n_tokens, c_in, heads, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace msla
