// Multi-scale token aggregation fused with the state of Eq. (3), 16-bit storage
// types, with the depthwise convolution on the matrix cores.
//
// Section 3.1 (last paragraph): every Q, K and V map of every head is aggregated
// over nearby tokens by a small depthwise convolution followed by a grouped 1x1
// convolution (3*heads groups of d channels); Eq. (3) then needs, per image /
// branch / head, only  KV = sum_n relu(K_n)^T [V_n, 1].
//
// On the vector ALUs the depthwise taps (25 fp32 FMAs per output, packed fp32
// off) cost more time than the kernel's HBM traffic.  A depthwise convolution
// has no contraction over channels, but along one image row it is a banded
// (Toeplitz) matrix product: out[x0+i] = sum_k w[k-i] in[x0-p+k].  The
// 16-block 4x4x4 MFMA does 16 such independent 4x4 products at once, one block
// per channel of a (head, Q/K/V) group:
//     A_b[i][k] = w[b][u][4s + k - i]      (filter row u, k-step s; zero outside the band)
//     B_b[k][j] = in[b][row][x0(j) - p + 4s + k]   (4 x-blocks j of one image row)
//     D_b[i][j] += A_b B_b                 (4 outputs x0(j)+i of channel b)
// A wave sweeps a 16-token-wide strip downwards: each input row is read once
// from LDS and multiplied into the (up to) k rolling accumulators of the
// output rows it touches.  The Toeplitz operands of a head's 48 channels are
// built once per wave and stay in registers.  The workgroup is a two-stage pipeline: four waves
// stage the next tile (global loads, transposition, raw branch) while eight waves sweep the current
// one (a 16-column strip x 4 rows each), so HBM latency and matrix-core work overlap inside a CU and
// every SIMD hosts one staging and two sweeping waves.
//
// The halo tile is kept channel-planar in LDS ([channel][row][x], x contiguous),
// which is what B_b wants; the global maps are token-major, so staging goes
// through an MFMA with an identity (selection) matrix that hands each lane 4
// consecutive tokens of one channel -- exact, and as a by-product those are the
// operands of the raw branch's  KV += relu(K)^T V.
//
// After the depthwise pass a lane holds 4 tokens of one channel.  V is only
// permuted across lanes (ds_bpermute) into the KV operand layout; its grouped
// 1x1 is linear and is applied once to the accumulated 16x16 state at the end:
//     KV[e][f] = sum_c (sum_n relu(K_n[e]) dwV_n[c]) w_gpw[f][c].
// K and Q are transposed through a small per-wave LDS buffer into the operand
// layout of the grouped 1x1 (one 16x16x16 MFMA per 16 tokens), K's result being
// the row operand of KV, Q's (transposed product) going to HBM.
#include <algorithm>

#include "msla_device.h"
#include "msla_kernels.h"

namespace msla {
namespace {

constexpr int MTH = kAggMfmaTileH;   // 16 tile rows, split into groups of kSweepRows
constexpr int MTW = kAggMfmaTileW;   // 32 tile columns: two 16-token strips
constexpr int kSweepWaves = 8;       // 4 or 8: each sweeps a 16-column strip x 8 or 4 rows (8: two per SIMD)
constexpr int kThreads = (4 + kSweepWaves) * 64;     // 4 staging waves + the sweeping waves
constexpr int kSweepRows = MTH / (kSweepWaves / 2);

template <int KS>
struct MLds {
    static constexpr int P = (KS - 1) / 2;
    static constexpr int LH = MTH + 2 * P, LW = MTW + 2 * P;
    static constexpr int kRowBytes = 72;                       // 36 columns, 8-byte aligned
    static constexpr int kChanRaw = LH * kRowBytes;
    // The channel stride is an odd number of 8-byte slots (16 slots = all 32 banks).  A staging
    // write puts 16 channels of one x-block side by side: 16 different slots mod 16.  A sweeping
    // read covers, per 16 lanes, 4 x-blocks of the channels {g, g+4, g+8, g+12}: their strides are
    // 0, 4, 8, 12 slots mod 16 (times an odd number), the x-blocks fill the gaps.
    static constexpr int kChanBytes = kChanRaw + ((kChanRaw / 8) % 2 == 0 ? 8 : 0);
    static constexpr int kPlanarBytes = 48 * kChanBytes;
    static constexpr int kTokStride = 80;                      // transposition buffer: 16 tokens x 16 fp32 (+pad)
    static constexpr int kTransBytes = 16 * kTokStride;
    static constexpr int kBytes = 2 * kPlanarBytes + kSweepWaves * 2 * kTransBytes;   // two tiles in flight; two transposition buffers per sweeping wave
    static_assert(LW <= 36 && (kChanBytes / 8) % 2 == 1, "LDS layout");
};

template <class T> struct M4;
template <> struct M4<_Float16> {
    static __device__ __forceinline__ f32x4 mma(f16x4 a, f16x4 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_4x4x4f16(a, b, c, 0, 0, 0);
    }
};
template <> struct M4<__bf16> {
    static __device__ __forceinline__ f32x4 mma(bf16x4 a, bf16x4 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(__builtin_bit_cast(i16x4, a), __builtin_bit_cast(i16x4, b), c,
                                                      0, 0, 0);
    }
};

// Compiler-level ordering of LDS traffic inside one wave (the hardware already
// executes a wave's LDS instructions in order).
__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// The kernel's body for workgroup `bid` of `nblocks` (a launch may hold the workgroups of two scales, see
// aggregate_mfma_pair_kernel).
template <class T, int KS, bool kCopyRawQ>
__device__ __forceinline__ void aggregate_mfma_body(const AggregateArgs& a, unsigned bid, unsigned nblocks) {
    typedef Traits<T> Tr;
    typedef typename Tr::Frag Frag;
    typedef typename Tr::Vec Vec;
    typedef MLds<KS> L;
    constexpr int P = L::P;
    constexpr int NS = 2;                 // k-steps of 4 input columns: 4 + 2P <= 8
    extern __shared__ __attribute__((aligned(16))) char lds[];
    float* red = (float*)lds;             // reused after the last tile

    const unsigned Lid = xcd_remap(bid, nblocks);
    const int h = Lid % a.heads;
    const int chunk = (Lid / a.heads) % a.nchunks;
    const int b = Lid / (a.heads * a.nchunks);
    const int Ct = a.heads * 16;
    const long N = (long)a.H * a.W;
    const long img_tok0 = (long)b * N;

    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // scalar: row/strip math stays on the SALU
    const int role = wave >= 4;           // waves 0-3 stage tile i+1 while the others sweep tile i
    const int w4 = wave & 3;              // staging wave index
    const int sw = (wave - 4) & (kSweepWaves - 1);   // sweeping wave index
    const int x16 = lane & 15, q = lane >> 4;      // 16x16 MFMA view of the lane
    const int blk = lane >> 2, sub = lane & 3;     // 4x4x4 view: block, row/column inside it
    // block -> channel of the group: 16 consecutive lanes take channels 4 apart (LDS banks, see MLds)
    const int chn = 4 * (blk & 3) + (blk >> 2);
    char* trans = lds + 2 * L::kPlanarBytes + sw * 2 * L::kTransBytes;

    const T* wdw = (const T*)a.w_dw + (long)h * 48 * KS * KS;
    const T* wgp = (const T*)a.w_gpw + (long)h * 48 * 16;

    // selection matrices for staging: ident picks channel x16 out of 16; selk / selv pick it out of
    // the 32 contraction slots {K 0..15, V 0..15} of a 16-byte K|V load
    Frag ident;
    Vec selk, selv;
#pragma unroll
    for (int r = 0; r < 4; ++r) ident[r] = Tr::from_f32(x16 == q * 4 + r ? 1.0f : 0.0f);
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        selk[r] = Tr::from_f32(q * 8 + r == x16 ? 1.0f : 0.0f);
        selv[r] = Tr::from_f32(q * 8 + r == 16 + x16 ? 1.0f : 0.0f);
    }

    const T* qmap = (const T*)a.q + (long)h * a.q_hs;
    const T* kmap = (const T*)a.k + (long)h * a.k_hs;     // V follows K: 32 contiguous channels
    T* q_ms = (T*)a.q_ms;
    const long q_ms_ts = (long)a.S * Ct;

    f32x4 kv_agg = {0.f, 0.f, 0.f, 0.f}, kv_raw = {0.f, 0.f, 0.f, 0.f};
    // Ksum of the raw branch rides on the matrix cores as well: relu(K)^T . ones puts
    // sum_n relu(K_n[e]) into every column, i.e. lane (*, q) element r holds Ksum[4q + r]
    f32x4 ks_raw4 = {0.f, 0.f, 0.f, 0.f};
    float ks_agg = 0.f;
    Frag ones;
#pragma unroll
    for (int r = 0; r < 4; ++r) ones[r] = Tr::from_f32(1.0f);
    const f32x4 z = {0.f, 0.f, 0.f, 0.f};

    const int tiles_x = (a.W + MTW - 1) / MTW, tiles_y = (a.H + MTH - 1) / MTH;
    const int n_tiles = tiles_x * tiles_y;
    // a tile's first row and column, stepped along the row-major tile order without divisions
    struct TileAt {
        int ty0, tx0;
    };
    auto tile_at = [&](int tile_id) { return TileAt{(tile_id / tiles_x) * MTH, (tile_id % tiles_x) * MTW}; };
    auto tile_after = [&](TileAt t) {
        t.tx0 += MTW;
        if (t.tx0 >= tiles_x * MTW) { t.tx0 = 0; t.ty0 += MTH; }
        return t;
    };
    const int tile_begin = chunk * a.tiles_per_chunk;
    const int tile_end = min(n_tiles, tile_begin + a.tiles_per_chunk);

    const int strip = sw & 1, part = sw >> 1;     // 16-column strip, group of kSweepRows rows
    // The image's maps are addressed through buffer resources with 32-bit byte offsets (the host
    // checks that an image's map fits); a lane outside the image gets an offset beyond any resource,
    // so its load returns zero and its store is dropped -- no per-lane branches.
    const unsigned q_tb = (unsigned)(a.q_ts * sizeof(T)), k_tb = (unsigned)(a.k_ts * sizeof(T));
    const unsigned q_ms_tb = (unsigned)(q_ms_ts * sizeof(T));
    const BufRsrc rq = make_rsrc(qmap + img_tok0 * a.q_ts, ((N - 1) * a.q_ts + 16) * (long)sizeof(T));
    const BufRsrc rk = make_rsrc(kmap + img_tok0 * a.k_ts, ((N - 1) * a.k_ts + 32) * (long)sizeof(T));
    const BufRsrc rout = make_rsrc(q_ms + img_tok0 * q_ms_ts + (long)a.branch * Ct + h * 16,
                                   ((N - 1) * q_ms_ts + 16) * (long)sizeof(T));
    // lane part of the staging load offsets: token x16 of a 16-column group, channels of q
    const unsigned lane_q_off = x16 * q_tb + q * 4 * (unsigned)sizeof(T);
    const unsigned lane_k_off = x16 * k_tb + q * 8 * (unsigned)sizeof(T);

    // ---------------- staging: token-major global -> channel-planar LDS, raw branch on the way.
    // Halo rows are dealt to the waves round-robin (row w4 + 4j, j = 0..4) and handled two at a time
    // ("batch").  A row's first 32 columns are two groups of 16: lane (token x16, q) loads its
    // token's 4 Q channels and 8 of its 32 K|V channels, and after the selection MFMA lane
    // (channel x16, q) holds tokens lx0 + 4q .. + 3 of that channel.  The last 2P columns of the wave's
    // rows j = 0..3 share one more such load (token slot x16 = 4*(j) + column - 32), row 4 has a
    // mostly empty one of its own: a wave-level load costs the same however few of its lanes are live.
    // The loads of the next batch are issued before the current one is consumed, so they are in
    // flight during its MFMAs.
    struct Batch {
        Frag qf[2][2], qtail;
        u32x4 kvr[2][2], kvtail;
    };
    constexpr int kBatches = ((L::LH + 3) / 4 + 1) / 2;
    static_assert(kBatches == 3 && L::LW - 32 <= 4 && L::LH <= 20, "staging schedule below: 3 batches, 5 rows per wave, a 4-column tail");
    // tail slots of batch `it`: rows j = jbase + (x16 >> 2), column 32 + (x16 & 3)
    auto tail_jbase = [](int it) { return it == 2 ? 0 : 4; };

    auto issue = [&](TileAt at, int it, Batch& bt, bool live) {   // staging waves; !live: every lane masked
        const int ty0 = at.ty0, tx0 = at.tx0;
#pragma unroll
        for (int rr = 0; rr < 2; ++rr) {
            const int ly = w4 + 4 * (it + rr);
            const int gy = ty0 - P + ly;
            const bool row_ok = live && ly < L::LH && gy >= 0 && gy < a.H;
            // wave-uniform row offset (it may wrap below zero for lanes that are masked anyway)
            const unsigned tok_first = (unsigned)(gy * a.W + (tx0 - P));
            const unsigned qrow = tok_first * q_tb + lane_q_off, krow = tok_first * k_tb + lane_k_off;
#pragma unroll
            for (int cg = 0; cg < 2; ++cg) {
                const int gx = tx0 - P + cg * 16 + x16;
                const bool ok = row_ok && gx >= 0 && gx < a.W;
                bt.qf[rr][cg] = __builtin_bit_cast(Frag, buf_load8(rq, ok ? qrow + cg * 16 * q_tb : kOobOffset));
                bt.kvr[rr][cg] = buf_load16(rk, ok ? krow + cg * 16 * k_tb : kOobOffset, 0);
            }
        }
        if (it != 0) {
            const int j = tail_jbase(it) + (x16 >> 2), lx = 32 + (x16 & 3);
            const int ly = w4 + 4 * j;
            const int gy = ty0 - P + ly, gx = tx0 - P + lx;
            const bool ok = live && j <= 4 && ly < L::LH && lx < L::LW && gy >= 0 && gy < a.H && gx >= 0 && gx < a.W;
            const unsigned tok = (unsigned)(gy * a.W + gx);
            bt.qtail = __builtin_bit_cast(Frag, buf_load8(rq, ok ? tok * q_tb + q * 4 * (unsigned)sizeof(T) : kOobOffset));
            bt.kvtail = buf_load16(rk, ok ? tok * k_tb + q * 8 * (unsigned)sizeof(T) : kOobOffset, 0);
        }
    };

    auto consume = [&](TileAt at, int it, const Batch& bt, char* planar) {
        const int ty0 = at.ty0, tx0 = at.tx0;
#pragma unroll
        for (int rr = 0; rr < 2; ++rr) {
            const int ly = w4 + 4 * (it + rr);
            if (ly >= L::LH) break;
            const int gy = ty0 - P + ly;
            const bool row_interior = ly >= P && ly < P + MTH;
            const long tok_first = img_tok0 + (long)gy * a.W + (tx0 - P);
            char* dst_row = planar + x16 * L::kChanBytes + ly * L::kRowBytes + q * 8;
            // All six selection MFMAs of the row are issued before any result is touched, so their
            // latencies overlap (a conversion right behind its MFMA stalls the wave for the whole pass).
            f32x4 sq[2], sk[2], sv[2];
#pragma unroll
            for (int cg = 0; cg < 2; ++cg) {
                const Vec kvv = __builtin_bit_cast(Vec, bt.kvr[rr][cg]);
                sq[cg] = Tr::mma16(z, bt.qf[rr][cg], ident);
                sk[cg] = Tr::mma_vec(z, kvv, selk);
                sv[cg] = Tr::mma_vec(z, kvv, selv);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int cg = 0; cg < 2; ++cg) {
                const int lx0 = cg * 16;
                const Frag dq = frag_from_f32<T>(sq[cg]);
                const Frag dk = frag_from_f32<T>(sk[cg]);
                const Frag dv = frag_from_f32<T>(sv[cg]);
                store_frag<T>(dst_row + lx0 * 2, dq);
                store_frag<T>(dst_row + 16 * L::kChanBytes + lx0 * 2, dk);
                store_frag<T>(dst_row + 32 * L::kChanBytes + lx0 * 2, dv);
                if constexpr (kCopyRawQ) {
                    if (row_interior && lx0 + x16 >= P && gy < a.H && tx0 - P + lx0 + x16 < a.W)
                        store_frag<T>(q_ms + (tok_first + lx0 + x16) * q_ms_ts + h * 16 + q * 4, bt.qf[rr][cg]);
                }
                if (a.do_raw && row_interior) {
                    // raw branch: tokens of this tile's interior only (each token belongs to one tile)
                    Frag rk = frag_relu_bits<T>(dk);
                    if (cg == 0) {      // the first columns are halo
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            if (4 * q + r < P) rk[r] = Tr::from_f32(0.f);
                    }
                    ks_raw4 = Tr::mma16(ks_raw4, rk, ones);
                    kv_raw = Tr::mma16(kv_raw, rk, dv);
                }
            }
        }
        if (it != 0) {
            // the tail columns: lane (channel x16, q) ends up with columns 32..35 of row j = jbase + q
            const int j = tail_jbase(it) + q;
            const int ly = w4 + 4 * j;
            const bool row_ok = j <= 4 && ly < L::LH;
            const bool row_interior = row_ok && ly >= P && ly < P + MTH;
            const Vec kvv = __builtin_bit_cast(Vec, bt.kvtail);
            const f32x4 tq = Tr::mma16(z, bt.qtail, ident);
            const f32x4 tk = Tr::mma_vec(z, kvv, selk);
            const f32x4 tv = Tr::mma_vec(z, kvv, selv);
            __builtin_amdgcn_sched_barrier(0);
            const Frag dq = frag_from_f32<T>(tq);
            const Frag dk = frag_from_f32<T>(tk);
            const Frag dv = frag_from_f32<T>(tv);
            if (row_ok) {
                char* dst = planar + x16 * L::kChanBytes + ly * L::kRowBytes + 32 * 2;
                store_frag<T>(dst, dq);
                store_frag<T>(dst + 16 * L::kChanBytes, dk);
                store_frag<T>(dst + 32 * L::kChanBytes, dv);
            }
            if constexpr (kCopyRawQ) {
                // here the lane is still (token slot x16, q): row jbase + (x16 >> 2), column 32 + (x16 & 3)
                const int js = tail_jbase(it) + (x16 >> 2), lxs = 32 + (x16 & 3);
                const int lys = w4 + 4 * js;
                const int gys = ty0 - P + lys, gxs = tx0 - P + lxs;
                if (js <= 4 && lys >= P && lys < P + MTH && lxs < P + MTW && gys < a.H && gxs < a.W)
                    store_frag<T>(q_ms + (img_tok0 + (long)gys * a.W + gxs) * q_ms_ts + h * 16 + q * 4, bt.qtail);
            }
            if (a.do_raw) {
                Frag rk = frag_relu_bits<T>(dk);
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (!row_interior || 32 + r >= P + MTW) rk[r] = Tr::from_f32(0.f);
                ks_raw4 = Tr::mma16(ks_raw4, rk, ones);
                kv_raw = Tr::mma16(kv_raw, rk, dv);
            }
        }
    };

    // Software pipeline over the workgroup's tiles with two LDS tile buffers: in step i the staging
    // waves fill buffer (i+1)&1 with tile i+1 while the sweeping waves work through tile i in buffer
    // i&1; one barrier per step hands the buffers over.  A staging wave keeps a ring of three load
    // batches: as soon as a batch is consumed, the same rows of the NEXT tile are requested into its
    // registers, so two to three batches per wave are in flight all the time and the HBM latency is
    // covered by the rest of the step (the barrier gates the LDS writes, not the loads).
    // The two roles run separate loops with the same number of barriers (n_my_tiles + 1), so that
    // the register allocator does not have to keep one role's state alive for the other.
    const int n_my_tiles = tile_end - tile_begin;
    // The staging waves request the first tile before anything else, so those loads are in flight
    // while the filter taps travel to LDS.  In the loop no branch surrounds a load: past the last
    // tile the requests are still made, with every lane masked.  The counter of outstanding loads
    // then has the same history on every path, and a batch is waited for with the two younger
    // batches still in flight (the scheduler must not mix the three batches here either: entering
    // the loop with batch 0 requested last would make every wait in the loop cover the youngest
    // loads as well).
    if (role == 0) {
        Batch ring0, ring1, ring2;
        TileAt here = tile_at(tile_begin);
        issue(here, 0, ring0, n_my_tiles > 0);
        __builtin_amdgcn_sched_barrier(0);
        issue(here, 2, ring1, n_my_tiles > 0);
        __builtin_amdgcn_sched_barrier(0);
        issue(here, 4, ring2, n_my_tiles > 0);
        __builtin_amdgcn_sched_barrier(0);
        for (int i = 0; i < n_my_tiles; ++i) {
            const TileAt next = tile_after(here);
            const bool more = i + 1 < n_my_tiles;
            char* planar = lds + (i & 1) * L::kPlanarBytes;
            consume(here, 0, ring0, planar);
            issue(next, 0, ring0, more);
            consume(here, 2, ring1, planar);
            issue(next, 2, ring1, more);
            consume(here, 4, ring2, planar);
            issue(next, 4, ring2, more);
            here = next;
            __syncthreads();
        }
        __syncthreads();
    } else {
    // Toeplitz operands of the three 16-channel groups: lane (channel chn, output i = sub).  Each
    // sweeping wave copies the head's 48 x KS x KS filter taps, coalesced, into its own transposition
    // buffers (idle until its first sweep) and picks its band entries from there with branch-free
    // LDS reads (index clamped, value masked).  Nothing here involves another wave, so the staging
    // waves fill the first tile buffer meanwhile without a workgroup barrier.
    Frag toep[3][KS][NS];
    {
        constexpr int kTaps = 48 * KS * KS;
        static_assert((kTaps + 1) * sizeof(T) <= 2 * L::kTransBytes, "tap table");
        constexpr int kVecs = kTaps * (int)sizeof(T) / 16;      // 16-byte pieces: a head's taps are a multiple
        static_assert(kVecs * 16 == kTaps * (int)sizeof(T), "tap table in 16-byte pieces");
        T* wl = (T*)trans;
        u32x4 piece[(kVecs + 63) / 64];
#pragma unroll
        for (int j = 0; j < (kVecs + 63) / 64; ++j)
            if (j * 64 + lane < kVecs) piece[j] = ((const u32x4*)wdw)[j * 64 + lane];
#pragma unroll
        for (int j = 0; j < (kVecs + 63) / 64; ++j)
            if (j * 64 + lane < kVecs) ((u32x4*)wl)[j * 64 + lane] = piece[j];
        if (lane == 0) wl[kTaps] = Tr::from_f32(0.f);     // the entry read by masked-out slots
        wave_lds_fence();
#pragma unroll
        for (int t = 0; t < 3; ++t)
#pragma unroll
            for (int u = 0; u < KS; ++u)
#pragma unroll
                for (int s = 0; s < NS; ++s)
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const int v = 4 * s + k - sub;
                        const int idx = (v >= 0 && v < KS) ? ((t * 16 + chn) * KS + u) * KS + v : kTaps;
                        toep[t][u][s][k] = wl[idx];
                    }
        wave_lds_fence();
    }
    // grouped 1x1 weights of Q and K as 16x16 operands: lane (o, q) holds w[o][4q..4q+3]
    const Frag gpw_q = load_frag<T>(wgp + (0 * 16 + x16) * 16 + q * 4);
    const Frag gpw_k = load_frag<T>(wgp + (1 * 16 + x16) * 16 + q * 4);
    TileAt here = tile_at(tile_begin);
    for (int step = -1; step < n_my_tiles; ++step) {
        if (step >= 0) {
        const char* planar = lds + (step & 1) * L::kPlanarBytes;
        const int ty0 = here.ty0, tx0 = here.tx0;
        here = tile_after(here);
        // ---------------- depthwise sweep: this wave's strip (16 columns) x part (kSweepRows rows)
        constexpr int R = kSweepRows;
        const int col0 = 16 * strip + 4 * sub;            // interior column of this lane's x-block
        const int gy0 = ty0 + R * part;
        const int gx0 = tx0 + col0;
        const bool ragged = ty0 + MTH > a.H || tx0 + MTW > a.W;      // wave-uniform
        Frag aggK[R], aggK_lo[R];
        // The three passes (K, V, Q) form one flat, fully unrolled sequence of input rows.  A finished
        // output row goes through three stages in three consecutive iterations, so that no stage
        // waits for the one before it: (1) hand the row to LDS for transposition (K, Q) or to the
        // lane permutation (V); (2) pick it up in operand layout and issue the grouped-1x1 / state
        // MFMA; (3) rectify, pack, store.  Two transposition buffers alternate.
        constexpr int NR = R + 2 * P;
        f32x4 acc[KS];
        Frag s1v[2][2];                   // V (hi, lo) after the lane permutation
        f32x4 s2v[2];                     // MFMA results awaiting stage 3
        u32x2 q_held = {0u, 0u};          // an even Q row awaiting its partner
        auto pass_t = [](int pass) { return pass == 0 ? 1 : pass == 1 ? 2 : 0; };     // K, V, Q
        // A finished row sits as lane (channel chn, x-block sub) = 4 tokens of one channel.  It is
        // rounded to the operand type first (hi and lo halves for bf16), so everything that moves is
        // 8 bytes per lane.
        auto stage1 = [&](int it, f32x4 o) {
            const int t = pass_t(it / NR), y = it % NR - (KS - 1);
            const int gy = gy0 + y;
            if (t == 1 && ragged) {
                // tokens outside the image contribute nothing: their aggregated K is made 0, which
                // also removes their V from the state; Q rows of such tokens are simply not stored.
                // (Only a tile that sticks out of the image has such tokens.)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (gy >= a.H || gx0 + i >= a.W) o[i] = 0.f;
            }
            Frag hi, lo;
            if constexpr (Tr::kHiLo) frag_split<T>(o, hi, lo);
            else hi = frag_from_f32<T>(o);
            if (t == 2) {
                // V: lane (channel c, q) <- the lane that swept channel c, x-block q: tokens (x-block q, i),
                // the K operand's order
                const int from = 4 * (4 * (x16 & 3) + (x16 >> 2)) + q;
                const u32x2 h2 = __builtin_bit_cast(u32x2, hi);
                s1v[it & 1][0] = __builtin_bit_cast(Frag, u32x2{(unsigned)__shfl((int)h2[0], from),
                                                                (unsigned)__shfl((int)h2[1], from)});
                if constexpr (Tr::kHiLo) {
                    const u32x2 l2 = __builtin_bit_cast(u32x2, lo);
                    s1v[it & 1][1] = __builtin_bit_cast(Frag, u32x2{(unsigned)__shfl((int)l2[0], from),
                                                                    (unsigned)__shfl((int)l2[1], from)});
                }
            } else {
                // K, Q: the lane's 4 tokens of one channel go into a [token][channel] fp32 matrix; stage 2
                // picks up a token's 4 channels with one 16-byte read
                char* tb = trans + (it & 1) * L::kTransBytes;
                wave_lds_fence();
#pragma unroll
                for (int i = 0; i < 4; ++i) *(float*)(tb + (4 * sub + i) * L::kTokStride + chn * 4) = o[i];
                wave_lds_fence();
            }
        };
        // Stage 2 is split: the transposed row is requested from LDS at the top of an iteration and
        // used after the iteration's depthwise MFMAs, which cover the LDS latency.
        auto stage2_read = [&](int it) {
            const char* tb = trans + (it & 1) * L::kTransBytes;
            return *(const f32x4*)(tb + x16 * L::kTokStride + q * 16);
        };
        auto stage2 = [&](int it, f32x4 tq) {
            const int t = pass_t(it / NR), y = it % NR - (KS - 1);
            if (t == 2) {
                if constexpr (Tr::kHiLo) {
                    kv_agg = Tr::mma16(kv_agg, aggK[y], s1v[it & 1][0]);
                    kv_agg = Tr::mma16(kv_agg, aggK[y], s1v[it & 1][1]);
                    kv_agg = Tr::mma16(kv_agg, aggK_lo[y], s1v[it & 1][0]);
                } else {
                    kv_agg = Tr::mma16(kv_agg, aggK[y], s1v[it & 1][0]);
                }
                return;
            }
            // The depthwise sums of Q always go to the grouped 1x1 as hi + lo pairs, whatever the
            // storage type: which components of the aggregated Q pass the rectifier of Eq. (2) is a
            // discrete decision, so that Q must carry the accuracy of its fp32 sums up to the one
            // rounding of its store (a sum rounded to 11 bits first moves a component that is small
            // against its 16 terms across zero).  K only feeds the sums of Eq. (3), which are
            // continuous in it: fp16 takes its depthwise sums rounded once.
            Frag dwf, dwf_lo;
            if (Tr::kHiLo || t == 0) frag_split<T>(tq, dwf, dwf_lo);
            else dwf = frag_from_f32<T>(tq);
            if (t == 1) {
                f32x4 kf = Tr::mma16(z, dwf, gpw_k);
                if constexpr (Tr::kHiLo) kf = Tr::mma16(kf, dwf_lo, gpw_k);
                s2v[it & 1] = kf;
            } else {
                f32x4 qq = Tr::mma16(z, gpw_q, dwf);
                qq = Tr::mma16(qq, gpw_q, dwf_lo);
                s2v[it & 1] = qq;
            }
        };
        auto stage3 = [&](int it) {
            const int t = pass_t(it / NR), y = it % NR - (KS - 1);
            if (t == 1) {
                const f32x4 kf = relu_bits_f32(s2v[it & 1]);       // Eq. (2): relu(K), one integer max per value
                ks_agg += (kf[0] + kf[1]) + (kf[2] + kf[3]);
                if constexpr (Tr::kHiLo) frag_split<T>(kf, aggK[y], aggK_lo[y]);
                else aggK[y] = frag_from_f32<T>(kf);
            } else if (t == 0) {
                // lane (token x16 = 4*xblock + i, q): channels 4q..4q+3 of image row gy0 + y, 8 bytes.
                // Two rows share one store (a store instruction costs the same whatever its width): an
                // even row waits for the next one, then the odd 16-lane groups of the one are swapped
                // with the even groups of the other, which leaves lane (x16, q) with channels
                // 8*(q/2) .. +7 of its token in row y - 1 + q % 2.
                static_assert(R % 2 == 0, "Q rows are stored in pairs");
                const u32x2 v = __builtin_bit_cast(u32x2, frag_from_f32<T>(s2v[it & 1]));
                if (y % 2 == 0) {
                    q_held = v;
                } else {
                    const u32x2 s0 = __builtin_amdgcn_permlane16_swap(q_held[0], v[0], false, false);
                    const u32x2 s1 = __builtin_amdgcn_permlane16_swap(q_held[1], v[1], false, false);
                    const int gy = gy0 + y - 1 + (q & 1);
                    const int gx = tx0 + 16 * strip + x16;
                    const unsigned off = (unsigned)(gy * a.W + gx) * q_ms_tb + (q >> 1) * 8 * (unsigned)sizeof(T);
                    buf_store16(rout, gy < a.H && gx < a.W ? off : kOobOffset, u32x4{s0[0], s1[0], s0[1], s1[1]});
                }
            }
        };
        // input row i of the flat sequence: 8 columns (two k-steps) of this lane's channel and x-block
        Frag din[2][2];
        auto fetch_row = [&](int i, Frag (&d)[2]) {
            const int t = pass_t(i / NR), r = i % NR;
            const char* src = planar + (t * 16 + chn) * L::kChanBytes + (R * part + r) * L::kRowBytes + col0 * 2;
            d[0] = load_frag<T>(src);
            d[1] = load_frag<T>(src + 8);
        };
        fetch_row(0, din[0]);
        static_for<0, 3 * NR + 2>([&](auto it_c) {
            constexpr int it = decltype(it_c)::value;
            // iteration i finishes an output row iff it is the KS-th or a later input row of its pass
            constexpr auto has_row = [](int i) { return i >= 0 && i < 3 * NR && i % NR >= KS - 1; };
            constexpr bool kPickUp = has_row(it - 1) && ((it - 1) / NR != 1);     // K or Q row in the transposition buffer
            // LDS requests first: the next input row and the row handed over one iteration ago
            if constexpr (it + 1 < 3 * NR) fetch_row(it + 1, din[(it + 1) & 1]);
            f32x4 tq = z;
            if constexpr (kPickUp) tq = stage2_read(it - 1);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (it < 3 * NR) {
                const int pass = it / NR, r = it % NR;
                const int t = pass_t(pass);
                if (r == 0) {
#pragma unroll
                    for (int i = 0; i < KS; ++i) acc[i] = z;
                }
#pragma unroll
                for (int u = 0; u < KS; ++u) {
                    const int y = r - u;
                    if (y < 0 || y >= R) continue;
                    acc[y % KS] = M4<T>::mma(toep[t][u][0], din[it & 1][0], acc[y % KS]);
                    acc[y % KS] = M4<T>::mma(toep[t][u][1], din[it & 1][1], acc[y % KS]);
                }
            }
            if constexpr (has_row(it - 1)) stage2(it - 1, tq);
            if constexpr (has_row(it - 2)) stage3(it - 2);
            if constexpr (has_row(it)) {
                // output row y of 16 channels x 16 tokens is complete: lane (channel chn, x-block sub)
                // holds the 4 tokens gx0..gx0+3 of image row gy0 + y
                const int y = it % NR - (KS - 1);
                const f32x4 o = acc[y % KS];
                acc[y % KS] = z;
                stage1(it, o);
            }
        });
        }
        __syncthreads();
    }
    }

    // ---------------- workgroup partial state
    ks_agg += __shfl_xor(ks_agg, 16);
    ks_agg += __shfl_xor(ks_agg, 32);
    __syncthreads();   // tile memory is dead from here on
    // per wave: [which][lane] accumulator quads, then [which][16] Ksum; which 0 = aggregated (V before
    // its grouped 1x1), 1 = raw
    constexpr int kWaveFloats = 2 * 256 + 2 * 16;
    constexpr int kWaves = kThreads / 64;         // staging waves hold the raw state, sweeping waves the aggregated
    float* msum = red + kWaves * kWaveFloats;          // [16][16] summed pre-1x1 state of the aggregated branch
    {
        float* mine = red + wave * kWaveFloats;
        *(f32x4*)(mine + lane * 4) = kv_agg;
        *(f32x4*)(mine + 256 + lane * 4) = kv_raw;
        if (q == 0) mine[512 + x16] = ks_agg;
        if (x16 == 0) *(f32x4*)(mine + 512 + 16 + q * 4) = ks_raw4;
    }
    __syncthreads();
    auto wave_sum = [&](int src) {      // fixed order
        float t = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) t += red[w * kWaveFloats + src];
        return t;
    };
    if (threadIdx.x < 256) {
        // M[e][c] of the aggregated branch, summed over the waves: lane (c, e / 4), element e % 4
        const int j = threadIdx.x;
        const int e = j >> 4, c = j & 15;
        msum[j] = wave_sum(((e >> 2) * 16 + c) * 4 + (e & 3));
    }
    __syncthreads();
    for (int j = threadIdx.x; j < 2 * kStateSize; j += kThreads) {
        const int which = j / kStateSize, idx = j - which * kStateSize;   // 0: aggregated, 1: raw
        if (which == 1 && !a.do_raw) continue;
        const int e = idx / 17, f = idx - e * 17;
        float s;
        if (f == 16) {
            s = wave_sum(512 + which * 16 + e);
        } else if (which == 1) {
            s = wave_sum(256 + ((e >> 2) * 16 + f) * 4 + (e & 3));
        } else {
            // the grouped 1x1 of V, applied to the summed state: KV[e][f] = sum_c M[e][c] w_gpw[f][c]
            const T* wv = wgp + (2 * 16 + f) * 16;
            s = 0.f;
#pragma unroll
            for (int c = 0; c < 16; ++c) s = fmaf(msum[e * 16 + c], Tr::to_f32(wv[c]), s);
        }
        const int branch = which == 0 ? a.branch : 0;
        a.partials[((((long)b * a.S + branch) * a.heads + h) * a.nchunks + chunk) * kStateSize + idx] = s;
    }
}

template <class T, int KS, bool kCopyRawQ>
__global__ __launch_bounds__(kThreads) void aggregate_mfma_kernel(AggregateArgs a) {
    aggregate_mfma_body<T, KS, kCopyRawQ>(a, blockIdx.x, gridDim.x);
}

// Two aggregated scales in one launch: the first half of the grid works on scale A, the second on scale
// B (each half a multiple of 8 workgroups, so a workgroup's position among the XCDs is what it would be
// in a launch of its own).  Nothing is shared between the halves; what the single launch buys is that
// the compute units never drain between the two scales: a unit that finishes its scale-A workgroup goes
// straight on to a scale-B one.
template <class T, int KSA, int KSB>
__global__ __launch_bounds__(kThreads) void aggregate_mfma_pair_kernel(AggregateArgs a0, AggregateArgs a1) {
    const unsigned half = gridDim.x >> 1;
    if (blockIdx.x < half) aggregate_mfma_body<T, KSA, false>(a0, blockIdx.x, half);
    else aggregate_mfma_body<T, KSB, false>(a1, blockIdx.x - half, half);
}

template <class T, int KS>
hipError_t run_ks(const AggregateArgs& a, unsigned nblocks, hipStream_t stream) {
    constexpr int kLds = MLds<KS>::kBytes;
    // the copy of the raw Q tokens into the multi-scale map is compiled in only where it is wanted
    if (a.copy_raw_q) {
        const hipError_t e = allow_dynamic_lds<aggregate_mfma_kernel<T, KS, true>>(kLds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((aggregate_mfma_kernel<T, KS, true>), dim3(nblocks), dim3(kThreads), kLds, stream, a);
    } else {
        const hipError_t e = allow_dynamic_lds<aggregate_mfma_kernel<T, KS, false>>(kLds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((aggregate_mfma_kernel<T, KS, false>), dim3(nblocks), dim3(kThreads), kLds, stream, a);
    }
    return hipGetLastError();
}

template <class T>
hipError_t run(const AggregateArgs& a, hipStream_t stream) {
    const long nblocks = (long)a.B * a.heads * a.nchunks;
    if (nblocks <= 0 || nblocks > 0x7fffffffL) return hipErrorInvalidValue;
    // the kernel reads K and V of a token as one 32-channel run
    if ((const char*)a.v != (const char*)a.k + 16 * sizeof(T) || a.v_ts != a.k_ts || a.v_hs != a.k_hs)
        return hipErrorInvalidValue;
    // 32-bit byte offsets inside one image's maps
    const long widest = std::max(std::max(a.q_ts, a.k_ts), (long)a.S * a.heads * 16);
    if ((long)a.H * a.W * widest * (long)sizeof(T) > 0x7fffffffL) return hipErrorNotSupported;
    if (a.ks == 3) return run_ks<T, 3>(a, (unsigned)nblocks, stream);
    if (a.ks == 5) return run_ks<T, 5>(a, (unsigned)nblocks, stream);
    if (a.ks == 7) return hipErrorNotSupported;       // 7x7 takes the general kernel (the Toeplitz operands here span 8 input columns)
    return hipErrorInvalidValue;
}

template <class T, int KSA, int KSB>
hipError_t run_pair_ks(const AggregateArgs& a0, const AggregateArgs& a1, unsigned nblocks, hipStream_t stream) {
    constexpr int kLds = MLds<KSA>::kBytes > MLds<KSB>::kBytes ? MLds<KSA>::kBytes : MLds<KSB>::kBytes;
    const hipError_t e = allow_dynamic_lds<aggregate_mfma_pair_kernel<T, KSA, KSB>>(kLds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((aggregate_mfma_pair_kernel<T, KSA, KSB>), dim3(2 * nblocks), dim3(kThreads), kLds, stream, a0, a1);
    return hipGetLastError();
}

template <class T>
hipError_t run_pair(const AggregateArgs& a0, const AggregateArgs& a1, hipStream_t stream) {
    const long nblocks = (long)a0.B * a0.heads * a0.nchunks;
    if (nblocks <= 0 || 2 * nblocks > 0x7fffffffL) return hipErrorInvalidValue;
    if (nblocks % 8 != 0 || a0.copy_raw_q || a1.copy_raw_q) return hipErrorNotSupported;
    for (const AggregateArgs* a : {&a0, &a1}) {
        if ((const char*)a->v != (const char*)a->k + 16 * sizeof(T) || a->v_ts != a->k_ts || a->v_hs != a->k_hs)
            return hipErrorNotSupported;
        const long widest = std::max(std::max(a->q_ts, a->k_ts), (long)a->S * a->heads * 16);
        if ((long)a->H * a->W * widest * (long)sizeof(T) > 0x7fffffffL) return hipErrorNotSupported;
    }
    if (a0.ks == 3 && a1.ks == 5) return run_pair_ks<T, 3, 5>(a0, a1, (unsigned)nblocks, stream);
    if (a0.ks == 5 && a1.ks == 3) return run_pair_ks<T, 5, 3>(a0, a1, (unsigned)nblocks, stream);
    return hipErrorNotSupported;
}

}  // namespace

hipError_t launch_aggregate_mfma_pair(int dt, const AggregateArgs& a0, const AggregateArgs& a1, hipStream_t stream) {
#ifdef MSLA_AGG_NO_MFMA
    return hipErrorNotSupported;
#endif
    switch (dt) {
        case 1: return run_pair<_Float16>(a0, a1, stream);
        case 2: return run_pair<__bf16>(a0, a1, stream);
    }
    return hipErrorNotSupported;
}

hipError_t launch_aggregate_mfma(int dt, const AggregateArgs& a, hipStream_t stream) {
#ifdef MSLA_AGG_NO_MFMA
    return hipErrorNotSupported;      // build knob: every case takes the general kernel (as oversized images do)
#endif
    switch (dt) {
        case 1: return run<_Float16>(a, stream);
        case 2: return run<__bf16>(a, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace msla
