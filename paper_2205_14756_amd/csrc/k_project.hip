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

// Where the projection writes, and in which order it walks the weight rows.  tile(tok0) gives the
// writer for the token tile starting at tok0: buffer resources based at that token, so offsets fit
// 32 bits and rows past the last token are dropped by the range check.
template <class T>
struct PlainDest {
    T* y;
    long n_tokens;
    int c_out;
    struct Tile {
        BufRsrc y;
        unsigned row_bytes;
        int c_out;
        __device__ __forceinline__ void store(int, int row, int oc, u32x4 v) const {
            buf_store16(y, oc < c_out ? row * row_bytes + oc * (unsigned)sizeof(T) : kOobOffset, v);
        }
    };
    __device__ __forceinline__ int row_of(int oc) const { return oc; }
    __device__ __forceinline__ Tile tile(long tok0) const {
        const long rb = (long)c_out * (long)sizeof(T);
        return Tile{make_rsrc(y + tok0 * c_out, (n_tokens - tok0) * rb), (unsigned)rb, c_out};
    }
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
    long n_tokens;
    int Ct;
    struct Tile {
        BufRsrc q, kv;
        unsigned q_row_bytes, kv_row_bytes;
        int Ct;
        __device__ __forceinline__ void store(int piece0, int row, int vc, u32x4 v) const {
            constexpr unsigned sz = (unsigned)sizeof(T);
            if (piece0 < Ct) buf_store16(q, vc < Ct ? row * q_row_bytes + vc * sz : kOobOffset, v);
            if (piece0 + 64 > Ct)
                buf_store16(kv, (vc >= Ct && vc < 3 * Ct) ? row * kv_row_bytes + (vc - Ct) * sz : kOobOffset, v);
        }
    };
    __device__ __forceinline__ int row_of(int vc) const {
        if (vc < Ct) return (vc >> 4) * 48 + (vc & 15);
        const int v2 = vc - Ct;
        return (v2 >> 5) * 48 + 16 + (v2 & 31);
    }
    __device__ __forceinline__ Tile tile(long tok0) const {
        const long qb = q_ms_stride * (long)sizeof(T), kb = kv_stride * (long)sizeof(T);
        return Tile{make_rsrc(q_ms + tok0 * q_ms_stride, (n_tokens - tok0) * qb),
                    make_rsrc(kv_raw + tok0 * kv_stride, (n_tokens - tok0) * kb), (unsigned)qb, (unsigned)kb, Ct};
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
        __syncthreads();
#pragma unroll
        for (int m = 0; m < 16; ++m) {
            acc[m >> 2][m & 3] = Traits<T>::mma_vec(acc[m >> 2][m & 3], f1.a[m >> 2], f1.b[m & 3]);
            if (m < 4) f0.a[m] = G::load_frag_lds(next, wr * 64 + m * 16, 0);
            else if (m < 8) f0.b[m - 4] = G::load_frag_lds(next + G::kLdsR, wc * 64 + (m - 4) * 16, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        cur ^= 1;
        if (++slab == slabs) {
            // every wave finished reading the buffer just consumed before the barrier above, and it is
            // not refilled before the next step: stage the results there
            G::epilogue_lds(acc, here, rb * G::BR, wr, wc, ep.tile(cb * G::BC));
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

#ifndef MSLA_PROJ_RESIDENT
#define MSLA_PROJ_RESIDENT 1
#endif

template <class T, class Epilogue>
hipError_t run_project(const void* x, const void* w, long n_tokens, int c_in, int c_out, Epilogue ep,
                       hipStream_t stream) {
    typedef ProjTile<T> G;
    const int n_rb = (c_out + G::BR - 1) / G::BR;
    const long n_cb = (n_tokens + G::BC - 1) / G::BC;
    const long n_tiles = n_cb * n_rb;
    if (n_tiles <= 0 || n_tiles > 0x7fffffffL) return hipErrorInvalidValue;
    // the weights are addressed with 32-bit byte offsets from their base, a token tile's rows too
    if ((long)c_out * c_in * (long)sizeof(T) >= 0x7fffffffL) return hipErrorInvalidValue;
    // one resident workgroup per CU (two LDS buffers of 55 KB); whole channel-block groups per workgroup
    const long cus = (long)compute_units() * MSLA_PROJ_RESIDENT;
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
        case 0: return run_project<float>(x, w, n_tokens, c_in, c_out, PlainDest<float>{(float*)y, n_tokens, c_out}, stream);
        case 1: return run_project<_Float16>(x, w, n_tokens, c_in, c_out, PlainDest<_Float16>{(_Float16*)y, n_tokens, c_out}, stream);
        case 2: return run_project<__bf16>(x, w, n_tokens, c_in, c_out, PlainDest<__bf16>{(__bf16*)y, n_tokens, c_out}, stream);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_qkv_project(int dt, const void* x, const void* w_qkv, void* q_ms, long q_ms_stride,
                              void* kv_raw, long n_tokens, int c_in, int heads, hipStream_t stream) {
    const int c_out = 3 * heads * 16;
    const long kv_stride = 2L * heads * 16;
    switch (dt) {
        case 0: return run_project<float>(x, w_qkv, n_tokens, c_in, c_out,
                    QkvSplitDest<float>{(float*)q_ms, q_ms_stride, (float*)kv_raw, kv_stride, n_tokens, heads * 16}, stream);
        case 1: return run_project<_Float16>(x, w_qkv, n_tokens, c_in, c_out,
                    QkvSplitDest<_Float16>{(_Float16*)q_ms, q_ms_stride, (_Float16*)kv_raw, kv_stride, n_tokens, heads * 16}, stream);
        case 2: return run_project<__bf16>(x, w_qkv, n_tokens, c_in, c_out,
                    QkvSplitDest<__bf16>{(__bf16*)q_ms, q_ms_stride, (__bf16*)kv_raw, kv_stride, n_tokens, heads * 16}, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace msla
