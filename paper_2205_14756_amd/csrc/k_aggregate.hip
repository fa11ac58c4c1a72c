// Multi-scale token aggregation fused with the state of Eq. (3).
//
// Section 3.1 (last paragraph): every Q, K and V map of every head is
// aggregated over nearby tokens by a small depthwise convolution followed by a
// grouped 1x1 convolution (3*heads groups of d channels).  Eq. (3) then needs,
// per image / branch / head, only  KV = sum_n relu(K_n)^T [V_n, 1].
//
// One workgroup owns one (image, head) and a run of 8 x 32-token tiles.  Per
// tile it stages the halo tile of the head's raw K, V and Q channels in LDS, one
// map at a time (the next one is fetched into registers while the current one is
// swept, and written to the other of two buffers after it), and each of its 4
// waves takes 2 tile rows (64 tokens):
//   - a lane (i, q) owns a strip of 4 consecutive tokens and channels 4q..4q+3
//     of one of Q/K/V; it slides the k x k window along the strip in registers
//     (fp32 sums), so the depthwise result is already an MFMA operand;
//   - the grouped 1x1 is one 16x16x16 MFMA per 16 tokens; for K and V its
//     result has one channel and 4 tokens per lane, which is the operand
//     layout of the next MFMA,  KV += relu(K)^T V, contracted over tokens, so
//     aggregated K and V never leave registers;
//   - aggregated Q is the only thing written to HBM (transposed MFMA, so a
//     lane stores 4 consecutive channels of one token);
//   - the raw branch runs through the same path with the centre tap and an
//     identity 1x1, which is exact.
// Per-workgroup partial states go to a buffer that a second kernel sums in a
// fixed order (deterministic), rescales and lays out as MFMA operands.
#include "msla_device.h"
#include "msla_kernels.h"

namespace msla {
namespace {

constexpr int TH = kAggTileH;   // tile rows
constexpr int TW = kAggTileW;   // tile columns; a strip is 4 tokens, 8 strips per row
constexpr int kAggThreads = 256;

template <class T, int KS>
struct AggLds {
    static constexpr int P = (KS - 1) / 2;
    static constexpr int LH = TH + 2 * P, LW = TW + 2 * P;
    // One map (Q, K or V: 16 channels) of the halo tile at a time, two buffers: the next map is fetched while
    // the current one is swept.  16 channels + 8 bytes a pixel: the strip stride (4 pixels) is then 8 banks
    // mod 32, which spreads the 64 lanes' 8-byte reads over the banks.
    static constexpr int kPixBytes = 16 * (int)sizeof(T) + 8;
    static constexpr int kMapBytes = LH * LW * kPixBytes;
    static constexpr int kTileBytes = 2 * kMapBytes;
    static constexpr int kWtsBytes = 3 * KS * KS * 16 * 4;     // fp32 [t][tap][16 ch]
    static constexpr int kRedBytes = 4 * (2 * 256 + 2 * 16) * 4;   // per wave: 2 x 64 lanes x 4 + 2 x 16 Ksum
    static constexpr int kBytes = (kTileBytes > kRedBytes ? kTileBytes : kRedBytes) + kWtsBytes;
};

// The three raw maps of one head (pointers already offset to the head).
template <class T>
struct HeadMaps {
    const T *q, *k, *v;
    long q_ts, k_ts, v_ts;   // elements per token
};

template <class T, int KS>
__global__ __launch_bounds__(kAggThreads) void aggregate_kernel(AggregateArgs a) {
    typedef Traits<T> Tr;
    typedef typename Tr::Frag Frag;
    typedef AggLds<T, KS> L;
    constexpr int P = L::P;
    extern __shared__ __attribute__((aligned(16))) char lds[];
    char* tile = lds;
    float* wts = (float*)(lds + (L::kBytes - L::kWtsBytes));
    float* red = (float*)lds;   // reused after the last tile

    const unsigned Lid = xcd_remap(blockIdx.x, gridDim.x);
    const int h = Lid % a.heads;
    const int chunk = (Lid / a.heads) % a.nchunks;
    const int b = Lid / (a.heads * a.nchunks);
    const int Ct = a.heads * 16;
    const long N = (long)a.H * a.W;
    const long img_tok0 = (long)b * N;

    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int x16 = lane & 15, q = lane >> 4;

    // depthwise filters of this head -> LDS as fp32 [t][tap][16]
    {
        const T* wdw = (const T*)a.w_dw + (long)h * 48 * KS * KS;
        for (int it = threadIdx.x; it < 48 * KS * KS; it += kAggThreads) {
            const int ch = it / (KS * KS), tap = it - ch * (KS * KS);
            wts[((ch >> 4) * KS * KS + tap) * 16 + (ch & 15)] = Tr::to_f32(wdw[it]);
        }
    }
    // grouped 1x1 weights of (h, t) as an MFMA operand: lane (o, q) holds w[o][4q..4q+3]
    Frag gpw[3];
#pragma unroll
    for (int t = 0; t < 3; ++t)
        gpw[t] = load_frag<T>((const T*)a.w_gpw + ((long)(h * 3 + t) * 16 + x16) * 16 + q * 4);
    Frag ident;
#pragma unroll
    for (int r = 0; r < 4; ++r) ident[r] = Tr::from_f32(x16 == q * 4 + r ? 1.0f : 0.0f);

    const HeadMaps<T> maps = {(const T*)a.q + (long)h * a.q_hs, (const T*)a.k + (long)h * a.k_hs,
                              (const T*)a.v + (long)h * a.v_hs, a.q_ts, a.k_ts, a.v_ts};
    T* q_ms = (T*)a.q_ms;
    const long q_ms_ts = (long)a.S * Ct;

    f32x4 kv_agg = {0.f, 0.f, 0.f, 0.f}, kv_raw = {0.f, 0.f, 0.f, 0.f};
    float ks_agg = 0.f, ks_raw = 0.f;

    const int tiles_x = (a.W + TW - 1) / TW, tiles_y = (a.H + TH - 1) / TH;
    const int n_tiles = tiles_x * tiles_y;
    const int tile_begin = chunk * a.tiles_per_chunk;
    const int tile_end = min(n_tiles, tile_begin + a.tiles_per_chunk);

    // this lane's strip inside the tile
    const int srow = wave * 2 + (x16 >> 3);
    const int scol = (x16 & 7) * 4;

    // Stages: (tile, pass) with the passes in the order K, V, Q.  A stage's map goes global -> registers while
    // the stage before it is swept, registers -> LDS after that sweep, one barrier a stage.
    constexpr int SZ = (int)sizeof(T);
    constexpr int VPT = 16 * SZ / 16;                              // 16-byte vectors per pixel of one map
    constexpr int kItems = L::LH * L::LW * VPT;
    constexpr int kPer = (kItems + kAggThreads - 1) / kAggThreads;
    u32x4 pre[kPer];
    auto fetch = [&](int tile_id, int pass) {
        const int ty0 = (tile_id / tiles_x) * TH, tx0 = (tile_id % tiles_x) * TW;
        const T* base = pass == 0 ? maps.k : pass == 1 ? maps.v : maps.q;
        const long ts = pass == 0 ? maps.k_ts : pass == 1 ? maps.v_ts : maps.q_ts;
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            const int it = threadIdx.x + j * kAggThreads;
            const int vi = it % VPT, pix = it / VPT;
            const int ly = pix / L::LW, lx = pix - ly * L::LW;
            const int gy = ty0 - P + ly, gx = tx0 - P + lx;
            u32x4 val = {0u, 0u, 0u, 0u};
            if (it < kItems && gy >= 0 && gy < a.H && gx >= 0 && gx < a.W)
                val = *(const u32x4*)(base + (img_tok0 + (long)gy * a.W + gx) * ts + vi * Tr::kVec);
            pre[j] = val;
        }
    };
    auto stash = [&](char* buf) {
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            const int it = threadIdx.x + j * kAggThreads;
            if (it < kItems) {
                const int vi = it % VPT, pix = it / VPT;
                char* dst = buf + pix * L::kPixBytes + vi * 16;
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

        Frag aggK[4], aggK_lo[4], rawK[4];
        // order K, V, Q: K's operands are kept for the V pass; Q only stores
#pragma unroll
        for (int pass = 0; pass < 3; ++pass) {
            const int t = (pass == 0) ? 1 : (pass == 1) ? 2 : 0;
            float acc[4][4];
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[r][c] = 0.f;
            const bool more = pass < 2 || tile_id + 1 < tile_end;
            if (more) fetch(pass < 2 ? tile_id : tile_id + 1, pass < 2 ? pass + 1 : 0);
            const char* src = tile + cur * L::kMapBytes + q * 4 * SZ;
            const float* wt = wts + t * KS * KS * 16 + q * 4;
            // raw tokens of the strip (the centre tap), for the raw branch / the raw-Q copy
            Frag center[4];
#pragma unroll
            for (int r = 0; r < 4; ++r)
                center[r] = load_frag<T>(src + ((srow + P) * L::LW + scol + r + P) * L::kPixBytes);
            // one filter row per iteration: 4+KS-1 pixels feed 4 tokens x KS taps x 4 channels
#pragma unroll 1
            for (int u = 0; u < KS; ++u) {
                Frag rowv[4 + KS - 1];
#pragma unroll
                for (int c = 0; c < 4 + KS - 1; ++c)
                    rowv[c] = load_frag<T>(src + ((srow + u) * L::LW + scol + c) * L::kPixBytes);
#pragma unroll
                for (int v = 0; v < KS; ++v) {
                    const f32x4 w4 = *(const f32x4*)(wt + (u * KS + v) * 16);
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const f32x4 d4 = frag_to_f32<T>(rowv[r + v]);
#pragma unroll
                        for (int c = 0; c < 4; ++c) acc[r][c] = fmaf(w4[c], d4[c], acc[r][c]);
                    }
                }
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const f32x4 z = {0.f, 0.f, 0.f, 0.f};
                f32x4 a4 = {acc[r][0], acc[r][1], acc[r][2], acc[r][3]};
                if (!valid[r]) a4 = z;       // tokens outside the image contribute nothing
                // depthwise sums as MFMA operand(s)
                // (Q's sums always as hi + lo: the sign of an aggregated Q component decides what
                // passes the rectifier of Eq. (2), so it keeps its fp32 accuracy up to its store)
                Frag dwf, dwf_lo;
                constexpr bool kWide = sizeof(T) == 2;     // fp32 operands are exact already
                if (Tr::kHiLo || (kWide && t == 0)) frag_split<T>(a4, dwf, dwf_lo);
                else dwf = frag_from_f32<T>(a4);
                const Frag rawf = valid[r] ? center[r] : frag_zero<T>();
                if (t == 1) {
                    // lane (c, q) <- channel c of the r-th token of strips 4q..4q+3
                    f32x4 kf = Tr::mma16(z, dwf, gpw[1]);
                    if constexpr (Tr::kHiLo) kf = Tr::mma16(kf, dwf_lo, gpw[1]);
#pragma unroll
                    for (int c = 0; c < 4; ++c) kf[c] = fmaxf(kf[c], 0.f);      // Eq. (2): relu(K)
                    ks_agg += (kf[0] + kf[1]) + (kf[2] + kf[3]);
                    if constexpr (Tr::kHiLo) frag_split<T>(kf, aggK[r], aggK_lo[r]);
                    else aggK[r] = frag_from_f32<T>(kf);
                    if (a.do_raw) {
                        const Frag rk = frag_relu<T>(frag_from_f32<T>(Tr::mma16(z, rawf, ident)));
                        rawK[r] = rk;
                        const f32x4 rf = frag_to_f32<T>(rk);
                        ks_raw += (rf[0] + rf[1]) + (rf[2] + rf[3]);
                    }
                } else if (t == 2) {
                    f32x4 vf = Tr::mma16(z, dwf, gpw[2]);
                    if constexpr (Tr::kHiLo) vf = Tr::mma16(vf, dwf_lo, gpw[2]);
                    // KV[e][f] += sum_n relu(K_n[e]) V_n[f]
                    if constexpr (Tr::kHiLo) {
                        Frag vh, vl;
                        frag_split<T>(vf, vh, vl);
                        kv_agg = Tr::mma16(kv_agg, aggK[r], vh);
                        kv_agg = Tr::mma16(kv_agg, aggK[r], vl);
                        kv_agg = Tr::mma16(kv_agg, aggK_lo[r], vh);
                    } else {
                        kv_agg = Tr::mma16(kv_agg, aggK[r], frag_from_f32<T>(vf));
                    }
                    if (a.do_raw) {
                        const Frag rv = frag_from_f32<T>(Tr::mma16(z, rawf, ident));
                        kv_raw = Tr::mma16(kv_raw, rawK[r], rv);
                    }
                } else {
                    // transposed: lane (strip i, q) <- output channels 4q..4q+3 of its own token r
                    f32x4 qq = Tr::mma16(z, gpw[0], dwf);
                    if constexpr (Tr::kHiLo || kWide) qq = Tr::mma16(qq, gpw[0], dwf_lo);
                    if (valid[r]) {
                        T* dst = q_ms + (tok0 + r) * q_ms_ts + h * 16 + q * 4;
                        store_frag<T>(dst + (long)a.branch * Ct, frag_from_f32<T>(qq));
                        if (a.copy_raw_q) store_frag<T>(dst, center[r]);
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
    ks_agg += __shfl_xor(ks_agg, 16);
    ks_agg += __shfl_xor(ks_agg, 32);
    ks_raw += __shfl_xor(ks_raw, 16);
    ks_raw += __shfl_xor(ks_raw, 32);
    __syncthreads();   // tile memory is dead from here on
    // per wave: [branch][lane] accumulator quads, then [branch][16] Ksum
    constexpr int kWaveFloats = 2 * 256 + 2 * 16;
    {
        float* mine = red + wave * kWaveFloats;
        *(f32x4*)(mine + lane * 4) = kv_agg;
        *(f32x4*)(mine + 256 + lane * 4) = kv_raw;
        if (q == 0) {
            mine[512 + x16] = ks_agg;
            mine[512 + 16 + x16] = ks_raw;
        }
    }
    __syncthreads();
    for (int j = threadIdx.x; j < 2 * kStateSize; j += kAggThreads) {
        const int which = j / kStateSize, idx = j - which * kStateSize;   // 0: aggregated, 1: raw
        if (which == 1 && !a.do_raw) continue;
        const int e = idx / 17, f = idx - e * 17;
        // KV[e][f] sits in lane (f, e / 4), element e % 4
        const int src = f < 16 ? which * 256 + ((e >> 2) * 16 + f) * 4 + (e & 3) : 512 + which * 16 + e;
        const float s = (red[src] + red[kWaveFloats + src]) + (red[2 * kWaveFloats + src] + red[3 * kWaveFloats + src]);
        const int branch = which == 0 ? a.branch : 0;
        a.partials[((((long)b * a.S + branch) * a.heads + h) * a.nchunks + chunk) * kStateSize + idx] = s;
    }
}

// Branch-0 state when the module has no aggregated scale: the raw K, V tokens
// of (image, head, chunk of 64-token groups), same operand path as above.
template <class T>
__global__ __launch_bounds__(kAggThreads) void raw_state_kernel(AggregateArgs a) {
    typedef Traits<T> Tr;
    typedef typename Tr::Frag Frag;
    __shared__ float red[4 * kStateSize];
    const unsigned Lid = xcd_remap(blockIdx.x, gridDim.x);
    const int h = Lid % a.heads;
    const int chunk = (Lid / a.heads) % a.nchunks;
    const int b = Lid / (a.heads * a.nchunks);
    const int Ct = a.heads * 16;
    const long N = (long)a.H * a.W;
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int x16 = lane & 15, q = lane >> 4;
    Frag ident;
#pragma unroll
    for (int r = 0; r < 4; ++r) ident[r] = Tr::from_f32(x16 == q * 4 + r ? 1.0f : 0.0f);
    const T* qp = (const T*)a.q + (long)h * a.q_hs;
    const T* kp = (const T*)a.k + (long)h * a.k_hs;
    const T* vp = (const T*)a.v + (long)h * a.v_hs;
    T* q_ms = (T*)a.q_ms;
    const long q_ms_ts = (long)a.S * Ct;
    f32x4 kv = {0.f, 0.f, 0.f, 0.f};
    float ks = 0.f;
    // a "tile" here is 64 consecutive tokens; each wave takes 16 of them per step
    const long n_groups = (N + 15) / 16;
    const long per_chunk = (long)a.tiles_per_chunk * 4;
    const long g_begin = (long)chunk * per_chunk;
    const long g_end = g_begin + per_chunk < n_groups ? g_begin + per_chunk : n_groups;
    const f32x4 z = {0.f, 0.f, 0.f, 0.f};
    for (long g = g_begin + wave; g < g_end; g += 4) {
        const long n = g * 16 + x16;
        const bool ok = n < N;
        const long tok = (long)b * N + n;
        Frag kf = frag_zero<T>(), vf = frag_zero<T>();
        if (ok) {
            kf = load_frag<T>(kp + tok * a.k_ts + q * 4);
            vf = load_frag<T>(vp + tok * a.v_ts + q * 4);
            if (a.copy_raw_q)
                store_frag<T>(q_ms + tok * q_ms_ts + h * 16 + q * 4, load_frag<T>(qp + tok * a.q_ts + q * 4));
        }
        const Frag rk = frag_relu<T>(frag_from_f32<T>(Tr::mma16(z, kf, ident)));
        const Frag rv = frag_from_f32<T>(Tr::mma16(z, vf, ident));
        const f32x4 rf = frag_to_f32<T>(rk);
        ks += (rf[0] + rf[1]) + (rf[2] + rf[3]);
        kv = Tr::mma16(kv, rk, rv);
    }
    ks += __shfl_xor(ks, 16);
    ks += __shfl_xor(ks, 32);
    float* mine = red + wave * kStateSize;
#pragma unroll
    for (int r = 0; r < 4; ++r) mine[(q * 4 + r) * 17 + x16] = kv[r];
    if (q == 0) mine[x16 * 17 + 16] = ks;
    __syncthreads();
    for (int j = threadIdx.x; j < kStateSize; j += kAggThreads) {
        const float s = (red[j] + red[kStateSize + j]) + (red[2 * kStateSize + j] + red[3 * kStateSize + j]);
        a.partials[((((long)b * a.S + 0) * a.heads + h) * a.nchunks + chunk) * kStateSize + j] = s;
    }
}

// The same state without the matrix cores: wavefront-level outer products on the vector ALUs and a
// shuffle reduction.  Four lanes share a token: lane (token slot l / 4, part p = l % 4) holds the
// token's 16 rectified K channels and its V channels 4p..4p+3, and accumulates KV[e][4p + j] for all
// e (64 fp32 sums) plus, in part 0's lanes, Ksum[e]; a wave takes 16 tokens per step.  At the end the
// 16 token slots are summed with xor-shuffles and the four waves through LDS.  It exists so that the
// choice of MFMA for this contraction can be measured (msla_forward_opts, MSLA_OPT_STATE_VALU).
template <class T>
__global__ __launch_bounds__(kAggThreads) void raw_state_valu_kernel(AggregateArgs a) {
    typedef Traits<T> Tr;
    typedef typename Tr::Frag Frag;
    __shared__ float red[4 * kStateSize];
    const unsigned Lid = xcd_remap(blockIdx.x, gridDim.x);
    const int h = Lid % a.heads;
    const int chunk = (Lid / a.heads) % a.nchunks;
    const int b = Lid / (a.heads * a.nchunks);
    const int Ct = a.heads * 16;
    const long N = (long)a.H * a.W;
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int slot = lane >> 2, p = lane & 3;
    const T* qp = (const T*)a.q + (long)h * a.q_hs;
    const T* kp = (const T*)a.k + (long)h * a.k_hs;
    const T* vp = (const T*)a.v + (long)h * a.v_hs;
    T* q_ms = (T*)a.q_ms;
    const long q_ms_ts = (long)a.S * Ct;
    float kv[16][4];
    float ks[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        ks[e] = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) kv[e][j] = 0.f;
    }
    const long n_groups = (N + 15) / 16;
    const long per_chunk = (long)a.tiles_per_chunk * 4;
    const long g_begin = (long)chunk * per_chunk;
    const long g_end = g_begin + per_chunk < n_groups ? g_begin + per_chunk : n_groups;
    for (long g = g_begin + wave; g < g_end; g += 4) {
        const long n = g * 16 + slot;
        const long tok = (long)b * N + n;
        Frag kf[4], vf = frag_zero<T>();
#pragma unroll
        for (int i = 0; i < 4; ++i) kf[i] = frag_zero<T>();
        if (n < N) {
#pragma unroll
            for (int i = 0; i < 4; ++i) kf[i] = load_frag<T>(kp + tok * a.k_ts + i * 4);
            vf = load_frag<T>(vp + tok * a.v_ts + p * 4);
            if (a.copy_raw_q)
                store_frag<T>(q_ms + tok * q_ms_ts + h * 16 + p * 4, load_frag<T>(qp + tok * a.q_ts + p * 4));
        }
        const f32x4 v4 = frag_to_f32<T>(vf);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const f32x4 k4 = frag_to_f32<T>(frag_relu<T>(kf[i]));       // Eq. (2): relu(K)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                ks[i * 4 + r] += k4[r];
#pragma unroll
                for (int j = 0; j < 4; ++j) kv[i * 4 + r][j] = fmaf(k4[r], v4[j], kv[i * 4 + r][j]);
            }
        }
    }
    // sum over the 16 token slots of the wave (lanes that differ in bits 2..5)
#pragma unroll
    for (int e = 0; e < 16; ++e) {
#pragma unroll
        for (int o = 4; o < 64; o <<= 1) {
            ks[e] += __shfl_xor(ks[e], o);
#pragma unroll
            for (int j = 0; j < 4; ++j) kv[e][j] += __shfl_xor(kv[e][j], o);
        }
    }
    float* mine = red + wave * kStateSize;
    if (slot == 0) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
#pragma unroll
            for (int j = 0; j < 4; ++j) mine[e * 17 + p * 4 + j] = kv[e][j];
            if (p == 0) mine[e * 17 + 16] = ks[e];
        }
    }
    __syncthreads();
    for (int j = threadIdx.x; j < kStateSize; j += kAggThreads) {
        const float s = (red[j] + red[kStateSize + j]) + (red[2 * kStateSize + j] + red[3 * kStateSize + j]);
        a.partials[((((long)b * a.S + 0) * a.heads + h) * a.nchunks + chunk) * kStateSize + j] = s;
    }
}

// One workgroup per (image, branch, head): fixed-order sum of the partial
// states, then the state as MFMA operands for the apply pass.  For the 16-bit
// storage types the state is multiplied by a power of two that puts its
// largest entry in [512, 1024) (numerator and denominator of Eq. (3) scale
// together) and split into a high and a low half, so the operands carry about
// twice the storage type's mantissa and cannot overflow fp16.
//   kvfrag[state][0][lane (f, q)] = { hi(KV[4q+r][f]) r<4, lo(...) r<4 }   (fp32: KV[4q+r][f])
//   kvfrag[state][1][lane (f, q)] = { hi(Ksum[4q+r]),      lo(...)      }   (fp32: Ksum[4q+r])
// split = 8: the 16 channels are two heads of 8 that were carried through the aggregation side by
// side.  Only the two diagonal 8 x 8 blocks of KV mean anything then; the operands keep those, and
// row f of the Ksum operand keeps the entries of f's own head, so that the apply pass -- unchanged --
// gives every output channel the numerator and the denominator of its own head (kv32 keeps all 272 sums).
template <class T>
__global__ __launch_bounds__(320) void state_finalize_kernel(const float* __restrict__ partials,
                                                             float* __restrict__ kv32, void* kvfrag,
                                                             float* __restrict__ kvscale, int nchunks, int split) {
    typedef Traits<T> Tr;
    __shared__ float st[kStateSize];
    __shared__ float wmax[5];
    const int s_id = blockIdx.x;
    const int j = threadIdx.x;
    float v = 0.f;
    if (j < kStateSize) {
        const float* p = partials + (long)s_id * nchunks * kStateSize + j;
        // the additions stay in chunk order; unrolling only lets several loads be in flight
#pragma unroll 8
        for (int c = 0; c < nchunks; ++c) v += p[(long)c * kStateSize];
        kv32[(long)s_id * kStateSize + j] = v;
        const int e = j / 17, f = j - e * 17;
        if (split > 0 && f < 16 && e / split != f / split) v = 0.f;
        st[j] = v;
    }
    float m = fabsf(v);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    if ((j & 63) == 0) wmax[j >> 6] = m;
    __syncthreads();
    float scale = 1.0f;
    if constexpr (Tr::kSplit) {
        const float mx = fmaxf(fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3])), wmax[4]);
        if (mx > 0.f && mx < INFINITY) {
            int ex;
            frexpf(mx, &ex);            // mx = m * 2^ex, m in [0.5, 1)
            scale = ldexpf(1.0f, 10 - ex);
        }
    }
    if (j == 0) kvscale[s_id] = scale;
    if (j < 64) {
        const int x16 = j & 15, q = j >> 4;
        char* out = (char*)kvfrag + (long)s_id * 2048;
        // Ksum[4q+r] as row x16 of the second operand sees it
        auto ksum = [&](int r) {
            const int e = q * 4 + r;
            return (split > 0 && e / split != x16 / split) ? 0.f : st[e * 17 + 16];
        };
        if constexpr (Tr::kSplit) {
            typename Tr::Vec fk, fs;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float a = st[(q * 4 + r) * 17 + x16] * scale;
                const typename Tr::elem ah = Tr::from_f32(a);
                fk[r] = ah;
                fk[4 + r] = Tr::from_f32(a - Tr::to_f32(ah));
                const float s = ksum(r) * scale;
                const typename Tr::elem sh = Tr::from_f32(s);
                fs[r] = sh;
                fs[4 + r] = Tr::from_f32(s - Tr::to_f32(sh));
            }
            *(u32x4*)(out + j * 16) = __builtin_bit_cast(u32x4, fk);
            *(u32x4*)(out + 1024 + j * 16) = __builtin_bit_cast(u32x4, fs);
        } else {
            f32x4 fk, fs;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                fk[r] = st[(q * 4 + r) * 17 + x16];
                fs[r] = ksum(r);
            }
            *(f32x4*)(out + j * 16) = fk;
            *(f32x4*)(out + 1024 + j * 16) = fs;
        }
    }
}

template <class T, int KS>
hipError_t run_aggregate_ks(const AggregateArgs& a, unsigned nblocks, hipStream_t stream) {
    constexpr int kLds = AggLds<T, KS>::kBytes;
    if (kLds > 48 * 1024) {   // above the default dynamic-LDS limit (the CU has 160 KB)
        const hipError_t e = allow_dynamic_lds<aggregate_kernel<T, KS>>(kLds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((aggregate_kernel<T, KS>), dim3(nblocks), dim3(kAggThreads), kLds, stream, a);
    return hipGetLastError();
}

template <class T>
hipError_t run_aggregate(const AggregateArgs& a, hipStream_t stream) {
    const long nblocks = (long)a.B * a.heads * a.nchunks;
    if (nblocks <= 0 || nblocks > 0x7fffffffL) return hipErrorInvalidValue;
    if (a.ks == 3) return run_aggregate_ks<T, 3>(a, (unsigned)nblocks, stream);
    if (a.ks == 5) return run_aggregate_ks<T, 5>(a, (unsigned)nblocks, stream);
    if (a.ks == 7) return run_aggregate_ks<T, 7>(a, (unsigned)nblocks, stream);
    return hipErrorInvalidValue;
}

template <class T>
hipError_t run_raw_state(const AggregateArgs& a, hipStream_t stream) {
    const long nblocks = (long)a.B * a.heads * a.nchunks;
    if (nblocks <= 0 || nblocks > 0x7fffffffL) return hipErrorInvalidValue;
    if (a.state_valu)
        hipLaunchKernelGGL((raw_state_valu_kernel<T>), dim3((unsigned)nblocks), dim3(kAggThreads), 0, stream, a);
    else
        hipLaunchKernelGGL((raw_state_kernel<T>), dim3((unsigned)nblocks), dim3(kAggThreads), 0, stream, a);
    return hipGetLastError();
}

template <class T>
hipError_t run_finalize(const float* partials, float* kv32, void* kvfrag, float* kvscale, int n_states,
                        int nchunks, int split, hipStream_t stream) {
    hipLaunchKernelGGL((state_finalize_kernel<T>), dim3((unsigned)n_states), dim3(320), 0, stream, partials,
                       kv32, kvfrag, kvscale, nchunks, split);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_aggregate(int dt, const AggregateArgs& a, hipStream_t stream) {
    switch (dt) {
        case 0: return run_aggregate<float>(a, stream);
        case 1: return run_aggregate<_Float16>(a, stream);
        case 2: return run_aggregate<__bf16>(a, stream);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_raw_state(int dt, const AggregateArgs& a, hipStream_t stream) {
    switch (dt) {
        case 0: return run_raw_state<float>(a, stream);
        case 1: return run_raw_state<_Float16>(a, stream);
        case 2: return run_raw_state<__bf16>(a, stream);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_state_finalize(int dt, const float* partials, float* kv32, void* kvfrag, float* kvscale,
                                 int n_states, int nchunks, hipStream_t stream, int split) {
    if (n_states <= 0 || (split != 0 && split != 8)) return hipErrorInvalidValue;
    switch (dt) {
        case 0: return run_finalize<float>(partials, kv32, kvfrag, kvscale, n_states, nchunks, split, stream);
        case 1: return run_finalize<_Float16>(partials, kv32, kvfrag, kvscale, n_states, nchunks, split, stream);
        case 2: return run_finalize<__bf16>(partials, kv32, kvfrag, kvscale, n_states, nchunks, split, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace msla
