// Multi-scale token aggregation fused with the state of Eq. (3) for heads of 32 channels, 16-bit storage
// (Section 3.1, last paragraph, with d = 32: depthwise k x k, grouped 1x1 with 3*heads groups of 32
// channels, then KV = sum_n relu(K_n)^T [V_n, 1] per image / branch / head).
//
// The form of the general head-size-16 kernel (k_aggregate.hip) with every 16 x 16 block doubled: one
// workgroup owns one (image, head) and a run of 8 x 32-token tiles; per tile it stages the halo tile of the
// head's raw K, V and Q channels in LDS, one map at a time (the next one on its way while the current one is
// swept), and each of its 4 waves takes 2 tile rows.  A lane (strip, q) owns 4
// consecutive tokens and channels 4q..4q+3 of one 16-channel block of Q, K or V and slides the k x k window
// along its strip in registers (fp32 sums), block after block.  The grouped 1x1 is a 2 x 2 arrangement of
// 16x16x16 matrix instructions, relu(K)^T V a 2 x 2 arrangement of accumulators contracted over the tokens;
// aggregated K and V never leave registers, aggregated Q is written with a lane storing 4 consecutive
// channels of its own token, and the raw branch rides along through an identity matrix, which is exact.
// Operand precision as in the head-size-16 kernel: depthwise sums and aggregated K/V as hi + lo pairs for
// bf16; for fp16 the Q sums as hi + lo, the K and V operands rounded once.
// Per-workgroup partial states [32][33] go to the buffer that the plain finalize kernel sums in a fixed order.
#include "msla_device.h"
#include "msla_kernels.h"

namespace msla {
namespace {

constexpr int TH = kAggTileH, TW = kAggTileW;
constexpr int kThreads32 = 256;
constexpr int D32 = 32, NB = 2;                      // head size; 16-channel blocks per Q, K or V
constexpr int kState32 = D32 * (D32 + 1);

template <class T, int KS>
struct Agg32Lds {
    static constexpr int P = (KS - 1) / 2;
    static constexpr int LH = TH + 2 * P, LW = TW + 2 * P;
    // One map (Q, K or V: 32 channels) of the halo tile at a time, two buffers: the next map is fetched while
    // the current one is swept, and two workgroups fit a CU.  32 channels + 8 bytes a pixel: a strip (4
    // pixels) is then 72 words on, 8 banks mod 32 (see lane_at in the kernel for the banks' low bits).
    static constexpr int kPixBytes = D32 * (int)sizeof(T) + 8;
    static constexpr int kMapBytes = LH * LW * kPixBytes;
    static constexpr int kTileBytes = 2 * kMapBytes;
    static constexpr int kWtsBytes = 3 * KS * KS * D32 * 4;          // fp32 [t][tap][32 ch]
    // per wave: [branch][K block][V block][lane] accumulator quads, then [branch][32] Ksum
    static constexpr int kWaveFloats = 2 * NB * NB * 256 + 2 * D32;
    static constexpr int kRedBytes = 4 * kWaveFloats * 4;
    static constexpr int kBytes = (kTileBytes > kRedBytes ? kTileBytes : kRedBytes) + kWtsBytes;
};

// (build knob, for experiments: waves a SIMD the register allocation is held to; 1 = no cap)
#ifndef MSLA_AGG32_WAVES
#define MSLA_AGG32_WAVES 1
#endif

template <class T, int KS>
__global__ __launch_bounds__(kThreads32, MSLA_AGG32_WAVES) void aggregate32_kernel(AggregateArgs a) {
    static_assert(sizeof(T) == 2, "16-bit storage types");
    typedef Traits<T> Tr;
    typedef typename Tr::Frag Frag;
    typedef Agg32Lds<T, KS> L;
    constexpr int P = L::P;
    constexpr int SZ = (int)sizeof(T);
    extern __shared__ __attribute__((aligned(16))) char lds[];
    char* tile = lds;
    float* wts = (float*)(lds + (L::kBytes - L::kWtsBytes));
    float* red = (float*)lds;   // reused after the last tile

    const unsigned Lid = xcd_remap(blockIdx.x, gridDim.x);
    const int h = Lid % a.heads;
    const int chunk = (Lid / a.heads) % a.nchunks;
    const int b = Lid / (a.heads * a.nchunks);
    const int Ct = a.heads * D32;
    const long N = (long)a.H * a.W;
    const long img_tok0 = (long)b * N;
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int x16 = lane & 15, q = lane >> 4;
    const f32x4 z = {0.f, 0.f, 0.f, 0.f};

    // depthwise filters of this head -> LDS as fp32 [t][tap][32]
    {
        const T* wdw = (const T*)a.w_dw + (long)h * 3 * D32 * KS * KS;
        for (int it = threadIdx.x; it < 3 * D32 * KS * KS; it += kThreads32) {
            const int ch = it / (KS * KS), tap = it - ch * (KS * KS);
            wts[((ch / D32) * KS * KS + tap) * D32 + (ch % D32)] = Tr::to_f32(wdw[it]);
        }
    }
    // grouped 1x1 weights of (h, t), block (out ob, in ib), as an MFMA operand: lane (o, q) holds
    // w[ob*16 + o][ib*16 + 4q .. 4q+3]
    Frag gpw[3][NB][NB];
#pragma unroll
    for (int t = 0; t < 3; ++t)
#pragma unroll
        for (int ob = 0; ob < NB; ++ob)
#pragma unroll
            for (int ib = 0; ib < NB; ++ib)
                gpw[t][ob][ib] = load_frag<T>((const T*)a.w_gpw + ((long)(h * 3 + t) * D32 + ob * 16 + x16) * D32 + ib * 16 + q * 4);
    Frag ident;
#pragma unroll
    for (int r = 0; r < 4; ++r) ident[r] = Tr::from_f32(x16 == q * 4 + r ? 1.0f : 0.0f);

    const T* maps[3] = {(const T*)a.q + (long)h * a.q_hs, (const T*)a.k + (long)h * a.k_hs, (const T*)a.v + (long)h * a.v_hs};
    const long map_ts[3] = {a.q_ts, a.k_ts, a.v_ts};
    T* q_ms = (T*)a.q_ms;
    const long q_ms_ts = (long)a.S * Ct;

    f32x4 kv_agg[NB][NB], kv_raw[NB][NB];
    float ks_agg[NB], ks_raw[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        ks_agg[i] = ks_raw[i] = 0.f;
#pragma unroll
        for (int j = 0; j < NB; ++j) kv_agg[i][j] = kv_raw[i][j] = z;
    }

    const int tiles_x = (a.W + TW - 1) / TW, tiles_y = (a.H + TH - 1) / TH;
    const int n_tiles = tiles_x * tiles_y;
    const int tile_begin = chunk * a.tiles_per_chunk;
    const int tile_end = min(n_tiles, tile_begin + a.tiles_per_chunk);
    // this lane's strip inside the tile
    const int srow = wave * 2 + (x16 >> 3);
    const int scol = (x16 & 7) * 4;
    // Byte offset of pixel scol + c inside a tile row, this lane's channel quad included.  The two 16-byte
    // halves of every 32 bytes of a pixel are swapped in pixels whose column has bit 4 set: the 32 lanes
    // that an 8-byte read serves together (q = 0, 1) would otherwise use half of the banks twice (a
    // strip's 800 bytes and a tile row are both 8 banks on, which leaves the banks' low bits to q).
    // (scol is a multiple of 4, so the bit is the same for the four pixels scol + 4j .. scol + 4j + 3: one
    // base per j, the pixels of a block at constant distances from it)
    int lane_at[(4 + KS - 1 + 3) / 4];
#pragma unroll
    for (int j = 0; j < (4 + KS - 1 + 3) / 4; ++j)
        lane_at[j] = scol * L::kPixBytes + ((q * 4 * SZ) ^ ((((scol + 4 * j) >> 4) & 1) * 16));

    // Stages: (tile, pass) with the passes in the order K, V, Q.  A stage's map goes global -> registers while
    // the stage before it is swept, registers -> LDS after that sweep, one barrier a stage.
    constexpr int VPT = D32 * SZ / 16;
    constexpr int kItems = L::LH * L::LW * VPT;                    // 16-byte vectors of one map's halo tile
    constexpr int kPer = (kItems + kThreads32 - 1) / kThreads32;
    u32x4 pre[kPer];
    auto map_of = [](int pass) { return pass == 0 ? 1 : pass == 1 ? 2 : 0; };
    auto fetch = [&](int tile_id, int pass) {
        const int ty0 = (tile_id / tiles_x) * TH, tx0 = (tile_id % tiles_x) * TW;
        const int t = map_of(pass);
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            const int it = threadIdx.x + j * kThreads32;
            const int vi = it % VPT, pix = it / VPT;
            const int ly = pix / L::LW, lx = pix - ly * L::LW;
            const int gy = ty0 - P + ly, gx = tx0 - P + lx;
            u32x4 val = {0u, 0u, 0u, 0u};
            if (it < kItems && gy >= 0 && gy < a.H && gx >= 0 && gx < a.W)
                val = *(const u32x4*)(maps[t] + (img_tok0 + (long)gy * a.W + gx) * map_ts[t] + vi * Tr::kVec);
            pre[j] = val;
        }
    };
    auto stash = [&](char* buf) {
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            const int it = threadIdx.x + j * kThreads32;
            if (it < kItems) {
                const int vi = it % VPT, pix = it / VPT;
                const int lx = pix % L::LW;
                char* dst = buf + pix * L::kPixBytes + ((vi * 16) ^ (((lx >> 4) & 1) * 16));
                ((u32x2*)dst)[0] = u32x2{pre[j][0], pre[j][1]};
                ((u32x2*)dst)[1] = u32x2{pre[j][2], pre[j][3]};
            }
        }
    };
    int cur = 0;
    if (tile_begin < tile_end) {
        fetch(tile_begin, 0);
        stash(tile);
    }
    __syncthreads();   // first map staged, wts written

    for (int tile_id = tile_begin; tile_id < tile_end; ++tile_id) {
        const int ty0 = (tile_id / tiles_x) * TH, tx0 = (tile_id % tiles_x) * TW;
        const int gy = ty0 + srow, gx0 = tx0 + scol;
        bool valid[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) valid[r] = (gy < a.H) && (gx0 + r < a.W);
        const long tok0 = img_tok0 + (long)gy * a.W + gx0;

        Frag aggK[NB][4], aggK_lo[NB][4], rawK[NB][4];
        // order K, V, Q: K's operands are kept for the V pass; Q only stores
#pragma unroll
        for (int pass = 0; pass < 3; ++pass) {
            const int t = (pass == 0) ? 1 : (pass == 1) ? 2 : 0;
            // Q's sums always as hi + lo: the sign of an aggregated Q component decides what passes the
            // rectifier of Eq. (2), so it keeps its fp32 accuracy up to its store
            const bool wide = Tr::kHiLo || t == 0;
            const bool more = pass < 2 || tile_id + 1 < tile_end;
            if (more) fetch(pass < 2 ? tile_id : tile_id + 1, pass < 2 ? pass + 1 : 0);
            const char* map = tile + cur * L::kMapBytes;
            Frag dwf[NB][4], dwl[NB][4], center[NB][4];
#pragma unroll
            for (int ib = 0; ib < NB; ++ib) {
                float acc[4][4];
#pragma unroll
                for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int c = 0; c < 4; ++c) acc[r][c] = 0.f;
                const char* src = map + ib * 16 * SZ;
                const float* wt = wts + t * KS * KS * D32 + ib * 16 + q * 4;
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    center[ib][r] = load_frag<T>(src + (srow + P) * L::LW * L::kPixBytes + lane_at[(r + P) >> 2] + (r + P) * L::kPixBytes);
                // one filter row at a time: 4+KS-1 pixels feed 4 tokens x KS taps x 4 channels.  A row's pixels
                // and taps are read from LDS while the row before it is worked on (two register sets in turn:
                // with one wave a SIMD nothing else hides those reads)
                struct Row {
                    Frag px[4 + KS - 1];
                    f32x4 w[KS];
                };
                auto read_row = [&](int u, Row& row) {
#pragma unroll
                    for (int c = 0; c < 4 + KS - 1; ++c)
                        row.px[c] = load_frag<T>(src + (srow + u) * L::LW * L::kPixBytes + lane_at[c >> 2] + c * L::kPixBytes);
#pragma unroll
                    for (int v = 0; v < KS; ++v) row.w[v] = *(const f32x4*)(wt + (u * KS + v) * D32);
                };
                auto sweep_row = [&](const Row& row) {
#pragma unroll
                    for (int v = 0; v < KS; ++v)
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const f32x4 d4 = frag_to_f32<T>(row.px[r + v]);
#pragma unroll
                            for (int c = 0; c < 4; ++c) acc[r][c] = fmaf(row.w[v][c], d4[c], acc[r][c]);
                        }
                };
                Row even, odd;
                read_row(0, even);
#pragma unroll 1
                for (int u = 0; u + 1 < KS; u += 2) {      // KS is odd: u + 2 <= KS - 1 here
                    read_row(u + 1, odd);
                    sweep_row(even);
                    read_row(u + 2, even);
                    sweep_row(odd);
                }
                sweep_row(even);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    f32x4 a4 = {acc[r][0], acc[r][1], acc[r][2], acc[r][3]};
                    if (!valid[r]) a4 = z;       // tokens outside the image contribute nothing
                    if (wide) frag_split<T>(a4, dwf[ib][r], dwl[ib][r]);
                    else dwf[ib][r] = frag_from_f32<T>(a4);
                    if (!valid[r]) center[ib][r] = frag_zero<T>();
                }
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if (t == 1) {
#pragma unroll
                    for (int ob = 0; ob < NB; ++ob) {
                        // lane (c, q) <- channel ob*16 + c of the r-th token of strips 4q..4q+3
                        f32x4 kf = z;
#pragma unroll
                        for (int ib = 0; ib < NB; ++ib) {
                            kf = Tr::mma16(kf, dwf[ib][r], gpw[1][ob][ib]);
                            if constexpr (Tr::kHiLo) kf = Tr::mma16(kf, dwl[ib][r], gpw[1][ob][ib]);
                        }
#pragma unroll
                        for (int c = 0; c < 4; ++c) kf[c] = fmaxf(kf[c], 0.f);      // Eq. (2): relu(K)
                        ks_agg[ob] += (kf[0] + kf[1]) + (kf[2] + kf[3]);
                        if constexpr (Tr::kHiLo) frag_split<T>(kf, aggK[ob][r], aggK_lo[ob][r]);
                        else aggK[ob][r] = frag_from_f32<T>(kf);
                        if (a.do_raw) {
                            const Frag rk = frag_relu<T>(frag_from_f32<T>(Tr::mma16(z, center[ob][r], ident)));
                            rawK[ob][r] = rk;
                            const f32x4 rf = frag_to_f32<T>(rk);
                            ks_raw[ob] += (rf[0] + rf[1]) + (rf[2] + rf[3]);
                        }
                    }
                } else if (t == 2) {
#pragma unroll
                    for (int ov = 0; ov < NB; ++ov) {
                        f32x4 vf = z;
#pragma unroll
                        for (int ib = 0; ib < NB; ++ib) {
                            vf = Tr::mma16(vf, dwf[ib][r], gpw[2][ov][ib]);
                            if constexpr (Tr::kHiLo) vf = Tr::mma16(vf, dwl[ib][r], gpw[2][ov][ib]);
                        }
                        // KV[e][f] += sum_n relu(K_n[e]) V_n[f], block (K block ok, V block ov)
                        Frag vh, vl;
                        if constexpr (Tr::kHiLo) frag_split<T>(vf, vh, vl);
                        else vh = frag_from_f32<T>(vf);
                        Frag rv;
                        if (a.do_raw) rv = frag_from_f32<T>(Tr::mma16(z, center[ov][r], ident));
#pragma unroll
                        for (int ok = 0; ok < NB; ++ok) {
                            kv_agg[ok][ov] = Tr::mma16(kv_agg[ok][ov], aggK[ok][r], vh);
                            if constexpr (Tr::kHiLo) {
                                kv_agg[ok][ov] = Tr::mma16(kv_agg[ok][ov], aggK[ok][r], vl);
                                kv_agg[ok][ov] = Tr::mma16(kv_agg[ok][ov], aggK_lo[ok][r], vh);
                            }
                            if (a.do_raw) kv_raw[ok][ov] = Tr::mma16(kv_raw[ok][ov], rawK[ok][r], rv);
                        }
                    }
                } else {
#pragma unroll
                    for (int ob = 0; ob < NB; ++ob) {
                        // transposed: lane (strip, q) <- output channels ob*16 + 4q..4q+3 of its own token r
                        f32x4 qq = z;
#pragma unroll
                        for (int ib = 0; ib < NB; ++ib) {
                            qq = Tr::mma16(qq, gpw[0][ob][ib], dwf[ib][r]);
                            qq = Tr::mma16(qq, gpw[0][ob][ib], dwl[ib][r]);
                        }
                        if (valid[r]) {
                            T* dst = q_ms + (tok0 + r) * q_ms_ts + h * D32 + ob * 16 + q * 4;
                            store_frag<T>(dst + (long)a.branch * Ct, frag_from_f32<T>(qq));
                            if (a.copy_raw_q) store_frag<T>(dst, center[ob][r]);
                        }
                    }
                }
            }
            // the next stage's map: registers -> the other buffer (free since the barrier of the stage before)
            if (more) stash(tile + (cur ^ 1) * L::kMapBytes);
            __syncthreads();
            cur ^= 1;
        }
    }

    // ---- workgroup partial state: combine the 4 q-groups of Ksum, then the 4 waves
#pragma unroll
    for (int ob = 0; ob < NB; ++ob) {
        ks_agg[ob] += __shfl_xor(ks_agg[ob], 16);
        ks_agg[ob] += __shfl_xor(ks_agg[ob], 32);
        ks_raw[ob] += __shfl_xor(ks_raw[ob], 16);
        ks_raw[ob] += __shfl_xor(ks_raw[ob], 32);
    }
    __syncthreads();   // tile memory is dead from here on
    {
        float* mine = red + wave * L::kWaveFloats;
#pragma unroll
        for (int ok = 0; ok < NB; ++ok)
#pragma unroll
            for (int ov = 0; ov < NB; ++ov) {
                *(f32x4*)(mine + ((0 * NB + ok) * NB + ov) * 256 + lane * 4) = kv_agg[ok][ov];
                *(f32x4*)(mine + ((1 * NB + ok) * NB + ov) * 256 + lane * 4) = kv_raw[ok][ov];
            }
        if (q == 0) {
#pragma unroll
            for (int ob = 0; ob < NB; ++ob) {
                mine[2 * NB * NB * 256 + ob * 16 + x16] = ks_agg[ob];
                mine[2 * NB * NB * 256 + D32 + ob * 16 + x16] = ks_raw[ob];
            }
        }
    }
    __syncthreads();
    for (int j = threadIdx.x; j < 2 * kState32; j += kThreads32) {
        const int which = j / kState32, idx = j - which * kState32;   // 0: aggregated, 1: raw
        if (which == 1 && !a.do_raw) continue;
        const int e = idx / (D32 + 1), f = idx - e * (D32 + 1);
        // KV[e][f] sits in block (e / 16, f / 16), lane (f % 16, (e % 16) / 4), element e % 4
        const int src = f < D32 ? ((which * NB + (e >> 4)) * NB + (f >> 4)) * 256 + ((((e & 15) >> 2) * 16) + (f & 15)) * 4 + (e & 3)
                                : 2 * NB * NB * 256 + which * D32 + e;
        const float s = (red[src] + red[L::kWaveFloats + src]) + (red[2 * L::kWaveFloats + src] + red[3 * L::kWaveFloats + src]);
        const int branch = which == 0 ? a.branch : 0;
        a.partials[((((long)b * a.S + branch) * a.heads + h) * a.nchunks + chunk) * kState32 + idx] = s;
    }
}

template <class T, int KS>
hipError_t run_ks32(const AggregateArgs& a, unsigned nblocks, hipStream_t stream) {
    constexpr int kLds = Agg32Lds<T, KS>::kBytes;
    static_assert(kLds <= 160 * 1024, "the halo tile of a head of 32 channels fits the LDS");
    const hipError_t e = allow_dynamic_lds<aggregate32_kernel<T, KS>>(kLds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((aggregate32_kernel<T, KS>), dim3(nblocks), dim3(kThreads32), kLds, stream, a);
    return hipGetLastError();
}

template <class T>
hipError_t run32(const AggregateArgs& a, hipStream_t stream) {
    const long nblocks = (long)a.B * a.heads * a.nchunks;
    if (nblocks <= 0 || nblocks > 0x7fffffffL) return hipErrorInvalidValue;
    if (a.ks == 3) return run_ks32<T, 3>(a, (unsigned)nblocks, stream);
    if (a.ks == 5) return run_ks32<T, 5>(a, (unsigned)nblocks, stream);
    if (a.ks == 7) return run_ks32<T, 7>(a, (unsigned)nblocks, stream);
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_aggregate32(int dt, const AggregateArgs& a, hipStream_t stream) {
    switch (dt) {
        case 1: return run32<_Float16>(a, stream);
        case 2: return run32<__bf16>(a, stream);
    }
    return hipErrorNotSupported;
}

}  // namespace msla
