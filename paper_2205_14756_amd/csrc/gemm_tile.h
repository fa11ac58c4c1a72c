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
// LDS rows hold 128 contraction bytes and are padded to 144 so that 8 lanes
// reading the same 16-byte column of 8 consecutive rows touch all 32 banks.
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
    static constexpr int kRowStride = 144;             // bytes
    static constexpr int kLdsR = BR * kRowStride;
    static constexpr int kLdsC = BC * kRowStride;
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

    // Same, with the matrix rows given by a map (a permuted order of the weight rows).
    template <int NV, class RowMap>
    static __device__ __forceinline__ void load_global_rows(u32x4 (&regs)[NV], const T* __restrict__ base,
                                                            int row0, int row_limit, long ld, int k0,
                                                            int k_limit, const RowMap& row_of) {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int v = threadIdx.x + i * kThreads;
            const int row = row0 + (v >> 3);
            const int k = k0 + (v & 7) * Tr::kVec;
            u32x4 val = {0u, 0u, 0u, 0u};
            if (row < row_limit && k < k_limit) val = *(const u32x4*)(base + (long)row_of(row) * ld + k);
            regs[i] = val;
        }
    }

    template <int NV>
    static __device__ __forceinline__ void store_lds(char* lds, const u32x4 (&regs)[NV]) {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int v = threadIdx.x + i * kThreads;
            *(u32x4*)(lds + (v >> 3) * kRowStride + (v & 7) * 16) = regs[i];
        }
    }

    // acc[io][jt] += W-tile(rows wr*64 + io*16 ..) . X-tile(rows wc*64 + jt*16 ..)^T
    static __device__ __forceinline__ void mma(f32x4 (&acc)[4][4], const char* ldsR, const char* ldsC,
                                               int wr, int wc) {
        const int x = lane_id() & 15, q = lane_id() >> 4;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            Vec a[4], b[4];
#pragma unroll
            for (int io = 0; io < 4; ++io)
                a[io] = __builtin_bit_cast(Vec, *(const u32x4*)(ldsR + (wr * 64 + io * 16 + x) * kRowStride +
                                                                 (kk * 4 + q) * 16));
#pragma unroll
            for (int jt = 0; jt < 4; ++jt)
                b[jt] = __builtin_bit_cast(Vec, *(const u32x4*)(ldsC + (wc * 64 + jt * 16 + x) * kRowStride +
                                                                 (kk * 4 + q) * 16));
#pragma unroll
            for (int io = 0; io < 4; ++io)
#pragma unroll
                for (int jt = 0; jt < 4; ++jt) acc[io][jt] = Tr::mma_vec(acc[io][jt], a[io], b[jt]);
        }
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

    template <class Dest>
    static __device__ __forceinline__ void epilogue_lds(const f32x4 (&acc)[4][4], char* stage, long tok0,
                                                        long tok_limit, int oc0, int oc_limit, int wr, int wc,
                                                        const Dest& dest) {
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
                const long tok = tok0 + wc * 64 + jt * 16 + row;
                const int oc = oc0 + wr * 64 + cv * Tr::kVec;
                const u32x4 val = *(const u32x4*)(mine + row * kStageRow + cv * 16);
                if (tok < tok_limit && oc < oc_limit) *(u32x4*)dest(tok, oc) = val;
            }
        }
    }
};

}  // namespace msla
