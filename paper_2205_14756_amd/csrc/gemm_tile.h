// Workgroup-level tile of a 1x1 projection  y[n, o] = sum_c x[n, c] * w[o, c]
// (Section 3.1: Q = x W_Q etc., and the final projection of the concatenated
// heads), built on 16x16 MFMAs for wave64.
//
// Both operands are contiguous along the contraction index, which is what the
// matrix instruction wants: a lane fetches 16 contiguous bytes of one row.
// The weight rows are the MFMA "row operand" and the tokens its "column
// operand", so a lane ends up with 4 consecutive output channels of one token
// and stores them as one 8- or 16-byte word.
//
// LDS layout of a 128-byte contraction slab of R rows: row-major with a row pitch of 160 bytes.
// With that pitch both access patterns run at the full LDS rate: an MFMA operand read (16 lanes =
// 16 consecutive rows of one 16-byte column, four columns per instruction) and the copy of rows
// from HBM (8 lanes per row).  A pitch of 144 bytes, or column planes padded by 16 bytes, halve
// the 16-byte read rate on this chip.
#pragma once
#include "msla_device.h"

namespace msla {

template <class T, int WR, int WC>
struct GemmTile {
    typedef Traits<T> Tr;
    typedef typename Tr::Vec Vec;
    static constexpr int kThreads = WR * WC * 64;
    static constexpr int BR = WR * 64;                 // weight rows (output channels) per tile
    static constexpr int BC = WC * 64;                 // tokens per tile
    static constexpr int BK = 128 / (int)sizeof(T);    // contraction elements per iteration
    static constexpr int kRow = 160;                   // LDS row pitch in bytes
    static constexpr int kLdsR = BR * kRow;
    static constexpr int kLdsC = BC * kRow;
    static constexpr int kVecR = BR * 8 / kThreads;    // 16-byte vectors per thread, weight tile
    static constexpr int kVecC = BC * 8 / kThreads;    // ... token tile
    static_assert(BR * 8 % kThreads == 0 && BC * 8 % kThreads == 0, "tile/thread mismatch");

    // Rows [row0, row0+NR) x contraction [k0, k0+BK) of a row-major matrix with
    // leading dimension ld -> registers; out-of-range parts read as zero.
    template <int NV>
    static __device__ __forceinline__ void load_global(u32x4 (&regs)[NV], const T* __restrict__ base,
                                                       long row0, long row_limit, long ld,
                                                       int k0, int k_limit) {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int v = threadIdx.x + i * kThreads;
            const long row = row0 + (v >> 3);
            const int k = k0 + (v & 7) * Tr::kVec;
            u32x4 val = {0u, 0u, 0u, 0u};
            if (row < row_limit && k < k_limit) val = *(const u32x4*)(base + row * ld + k);
            regs[i] = val;
        }
    }

    // i-th 16-byte vector of this thread's share of a slab -> LDS
    static __device__ __forceinline__ void store_lds_one(char* lds, u32x4 reg, int i) {
        const int v = threadIdx.x + i * kThreads;
        *(u32x4*)(lds + (v >> 3) * kRow + (v & 7) * 16) = reg;
    }
    template <int NV>
    static __device__ __forceinline__ void store_lds(char* lds, const u32x4 (&regs)[NV]) {
#pragma unroll
        for (int i = 0; i < NV; ++i) store_lds_one(lds, regs[i], i);
    }
    static __device__ __forceinline__ void store_lds_r(char* lds, const u32x4 (&regs)[kVecR]) { store_lds(lds, regs); }
    static __device__ __forceinline__ void store_lds_c(char* lds, const u32x4 (&regs)[kVecC]) { store_lds(lds, regs); }

    // One MFMA operand: 16 rows starting at row0 of the tile, contraction half kk (0 or 1).
    static __device__ __forceinline__ Vec load_frag_lds(const char* lds, int row0, int kk) {
        const int x = lane_id() & 15, q = lane_id() >> 4;
        return __builtin_bit_cast(Vec, *(const u32x4*)(lds + (row0 + x) * kRow + (kk * 4 + q) * 16));
    }
    // acc[io][jt] += W-tile(rows wr*64 + io*16 ..) . X-tile(rows wc*64 + jt*16 ..)^T
    static __device__ __forceinline__ void load_frags(Vec (&a)[4], Vec (&b)[4], const char* ldsR, const char* ldsC,
                                                      int wr, int wc, int kk) {
#pragma unroll
        for (int io = 0; io < 4; ++io) a[io] = load_frag_lds(ldsR, wr * 64 + io * 16, kk);
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) b[jt] = load_frag_lds(ldsC, wc * 64 + jt * 16, kk);
    }

    struct Frags {
        Vec a[4], b[4];
    };
    static __device__ __forceinline__ void mma_half(f32x4 (&acc)[4][4], const Frags& f) {
#pragma unroll
        for (int io = 0; io < 4; ++io)
#pragma unroll
            for (int jt = 0; jt < 4; ++jt) acc[io][jt] = Tr::mma_vec(acc[io][jt], f.a[io], f.b[jt]);
    }

    static __device__ __forceinline__ void mma(f32x4 (&acc)[4][4], const char* ldsR, const char* ldsC,
                                               int wr, int wc) {
        Frags f0, f1;
        load_frags(f0.a, f0.b, ldsR, ldsC, wr, wc, 0);
        load_frags(f1.a, f1.b, ldsR, ldsC, wr, wc, 1);
        mma_half(acc, f0);
        mma_half(acc, f1);
    }

    static __device__ __forceinline__ void zero(f32x4 (&acc)[4][4]) {
#pragma unroll
        for (int io = 0; io < 4; ++io)
#pragma unroll
            for (int jt = 0; jt < 4; ++jt) acc[io][jt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // Hands every 4-channel group of the tile to ep(token, out_channel, values).
    template <class Epilogue>
    static __device__ __forceinline__ void epilogue(const f32x4 (&acc)[4][4], long tok0, long tok_limit,
                                                    int oc0, int oc_limit, int wr, int wc,
                                                    const Epilogue& ep) {
        const int x = lane_id() & 15, q = lane_id() >> 4;
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) {
            const long tok = tok0 + wc * 64 + jt * 16 + x;
            if (tok >= tok_limit) continue;
#pragma unroll
            for (int io = 0; io < 4; ++io) {
                const int oc = oc0 + wr * 64 + io * 16 + q * 4;
                if (oc < oc_limit) ep(tok, oc, acc[io][jt]);
            }
        }
    }

    // Epilogue through LDS: a wave parks one 16-token x 64-channel piece of its results at a time in
    // its own staging rows and writes it out as 16-byte words, so that consecutive lanes cover whole
    // 128-byte runs of a token's channels (an 8-byte-per-lane scatter costs the address path one
    // cycle per 32-byte segment).  dest(token, channel) returns where 16 bytes of channels starting
    // at a multiple of 16/sizeof(T) go; it is only called for valid tokens and channels.
    static constexpr int kStageRow = 64 * (int)sizeof(T) + 16;
    static constexpr int kStageWave = 16 * kStageRow;
    static constexpr int kStageBytes = WR * WC * kStageWave;

    // out.store(first and past-the-end channel of the wave's 64-channel piece (wave-uniform), token
    // row within the tile, channel, 16 bytes) writes -- or drops, beyond the ragged ends -- one word.
    template <class TileOut>
    static __device__ __forceinline__ void epilogue_lds(const f32x4 (&acc)[4][4], char* stage, int oc0, int wr,
                                                        int wc, const TileOut& out) {
        const int lane = lane_id();
        const int x = lane & 15, q = lane >> 4;
        char* mine = stage + (wr + WR * wc) * kStageWave;
        constexpr int kVecPerRow = 64 * (int)sizeof(T) / 16;        // 8 (16-bit) or 16 (fp32)
        constexpr int kPer = 16 * kVecPerRow / 64;                  // vectors per lane per piece
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int io = 0; io < 4; ++io)
                store_frag<T>(mine + x * kStageRow + (io * 16 + q * 4) * (int)sizeof(T), frag_from_f32<T>(acc[io][jt]));
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int i = 0; i < kPer; ++i) {
                const int v = lane + 64 * i;
                const int row = v / kVecPerRow, cv = v % kVecPerRow;
                const u32x4 val = *(const u32x4*)(mine + row * kStageRow + cv * 16);
                out.store(oc0 + wr * 64, oc0 + wr * 64 + 64, wc * 64 + jt * 16 + row, oc0 + wr * 64 + cv * Tr::kVec, val);
            }
        }
    }

    // The same with a residual: the wave parks its 16-token x 64-channel piece as fp32, each lane picks
    // up the 16 output bytes it will write (8 or 4 channels), adds the residual's same 16 bytes
    // (res(token row within the tile, channel) -> 16 bytes, zero past the ends) in fp32 and rounds
    // once.  Needs kStageResBytes of LDS.
    static constexpr int kStageResRow = 64 * 4 + 16;
    static constexpr int kStageResWave = 16 * kStageResRow;
    static constexpr int kStageResBytes = WR * WC * kStageResWave;
    template <class TileOut, class Res>
    static __device__ __forceinline__ void epilogue_lds_residual(const f32x4 (&acc)[4][4], char* stage, int oc0, int wr,
                                                                 int wc, const TileOut& out, const Res& res) {
        const int lane = lane_id();
        const int x = lane & 15, q = lane >> 4;
        char* mine = stage + (wr + WR * wc) * kStageResWave;
        constexpr int kVecPerRow = 64 * (int)sizeof(T) / 16;        // 8 (16-bit) or 16 (fp32)
        constexpr int kPer = 16 * kVecPerRow / 64;                  // output vectors per lane per piece
        constexpr int kCh = Tr::kVec;                               // channels per output vector
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int io = 0; io < 4; ++io) *(f32x4*)(mine + x * kStageResRow + (io * 16 + q * 4) * 4) = acc[io][jt];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int i = 0; i < kPer; ++i) {
                const int v = lane + 64 * i;
                const int row = v / kVecPerRow, cv = v % kVecPerRow;
                const int trow = wc * 64 + jt * 16 + row, oc = oc0 + wr * 64 + cv * kCh;
                const u32x4 r = res(trow, oc);
                u32x4 val;
                if constexpr (sizeof(T) == 4) {
                    const f32x4 a = *(const f32x4*)(mine + row * kStageResRow + cv * 16);
                    const f32x4 b = __builtin_bit_cast(f32x4, r);
                    val = __builtin_bit_cast(u32x4, f32x4{a[0] + b[0], a[1] + b[1], a[2] + b[2], a[3] + b[3]});
                } else {
                    const f32x4 a0 = *(const f32x4*)(mine + row * kStageResRow + cv * 32);
                    const f32x4 a1 = *(const f32x4*)(mine + row * kStageResRow + cv * 32 + 16);
                    const Vec b = __builtin_bit_cast(Vec, r);
                    Vec o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        o[e] = Tr::from_f32(a0[e] + Tr::to_f32(b[e]));
                        o[4 + e] = Tr::from_f32(a1[e] + Tr::to_f32(b[4 + e]));
                    }
                    val = __builtin_bit_cast(u32x4, o);
                }
                out.store(oc0 + wr * 64, oc0 + wr * 64 + 64, trow, oc, val);
            }
        }
    }
};

}  // namespace msla
