// Per-token normalise-and-apply of Eq. (3), last line:
//   att[n, m*16 + f] = relu(Q_n) . KV[:, f] / (relu(Q_n) . KV[:, 16] + eps)
// for every head-branch m = s*heads + h of the multi-scale Q map, either
// written out (the module without projections) or fed straight into the final
// 1x1 projection of the concatenated heads (Section 3.1, last sentence) so the
// attention map never reaches HBM.
//
// A 16-token x one-head-branch unit is two MFMAs: the state is the row operand
// (prepared by the finalize kernel, hi and lo halves stacked along the
// contraction for the 16-bit types), relu(Q) the column operand.  The second
// MFMA uses a row operand whose 16 rows all equal Ksum, so every lane gets the
// denominator of its own token without a shuffle.  The result has 4
// consecutive channels of one token per lane.
#include "gemm_tile.h"
#include "msla_kernels.h"

#ifndef MSLA_APPLY_W_AHEAD
#define MSLA_APPLY_W_AHEAD 3
#endif
#ifndef MSLA_APPLY_WR
#define MSLA_APPLY_WR 4
#define MSLA_APPLY_WC 2
#endif

namespace msla {
namespace {

// q: channels 4q..4q+3 of this lane's token (raw, not yet rectified).
// state: the 2048-byte operand block of (image, head-branch).  eps_s = eps * scale.
template <class T>
struct StateOps {
    u32x4 kv, ks;       // row operands: the state, and Ksum in every row
    float eps_s;
};
template <class T>
__device__ __forceinline__ StateOps<T> load_state_ops(const char* kvfrag, const float* kvscale, long sid, float eps,
                                                      bool live) {
    StateOps<T> s;
    s.kv = *(const u32x4*)(kvfrag + sid * 2048 + lane_id() * 16);
    s.ks = *(const u32x4*)(kvfrag + sid * 2048 + 1024 + lane_id() * 16);
    s.eps_s = live ? eps * kvscale[sid] : 0.f;
    return s;
}
template <class T>
__device__ __forceinline__ f32x4 att_unit(typename Traits<T>::Frag qf, const StateOps<T>& st) {
    typedef Traits<T> Tr;
    const f32x4 z = {0.f, 0.f, 0.f, 0.f};
    qf = frag_relu<T>(qf);
    f32x4 num, den;
    if constexpr (Tr::kSplit) {
        typedef typename Tr::Vec Vec;
        Vec b;
#pragma unroll
        for (int r = 0; r < 4; ++r) { b[r] = qf[r]; b[4 + r] = qf[r]; }   // pairs with {hi, lo}
        num = Tr::mma_vec(z, __builtin_bit_cast(Vec, st.kv), b);
        den = Tr::mma_vec(z, __builtin_bit_cast(Vec, st.ks), b);
    } else {
        num = Tr::mma16(z, __builtin_bit_cast(f32x4, st.kv), qf);
        den = Tr::mma16(z, __builtin_bit_cast(f32x4, st.ks), qf);
    }
    const float inv = 1.0f / (den[0] + st.eps_s);
    return f32x4{num[0] * inv, num[1] * inv, num[2] * inv, num[3] * inv};
}
template <class T>
__device__ __forceinline__ f32x4 att_unit(typename Traits<T>::Frag qf, const char* state, float eps_s) {
    StateOps<T> st;
    st.kv = *(const u32x4*)(state + lane_id() * 16);
    st.ks = *(const u32x4*)(state + 1024 + lane_id() * 16);
    st.eps_s = eps_s;
    return att_unit<T>(qf, st);
}

// ------------------------------------------------------------------ att only
// One wave per 16-token group of one image; it walks over the head-branches.
template <class T>
__global__ __launch_bounds__(256) void apply_kernel(const T* __restrict__ q_ms, const char* __restrict__ kvfrag,
                                                    const float* __restrict__ kvscale, T* __restrict__ att,
                                                    int N, int n_hb, int groups_per_image, long n_groups,
                                                    float eps) {
    const int wave = threadIdx.x >> 6;
    const int x16 = lane_id() & 15, q = lane_id() >> 4;
    const long g = (long)blockIdx.x * 4 + wave;
    if (g >= n_groups) return;
    const int b = (int)(g / groups_per_image);
    const int n = (int)(g % groups_per_image) * 16 + x16;
    const bool ok = n < N;
    const long ld = (long)n_hb * 16;
    const long row = ((long)b * N + n) * ld;
    for (int m = 0; m < n_hb; ++m) {
        typename Traits<T>::Frag qf = frag_zero<T>();
        if (ok) qf = load_frag<T>(q_ms + row + m * 16 + q * 4);
        const long sid = (long)b * n_hb + m;
        const f32x4 o = att_unit<T>(qf, kvfrag + sid * 2048, eps * kvscale[sid]);
        if (ok) store_frag<T>(att + row + m * 16 + q * 4, frag_from_f32<T>(o));
    }
}

// ------------------------------------------------- att fused into projection
// WC*64 tokens of one image x WR*64 output channels per workgroup, one wave per 64 x 64
// (128 tokens x 256 channels, 8 waves, unless the map is small).  Each
// iteration covers 128 contraction bytes = BK/16 head-branches; wave w makes
// the attention rows of token group w for them and writes them to the token
// tile in LDS while the weight tile arrives from the previous iteration's
// prefetch.  For bf16 the attention rows go to LDS as a hi and a lo tile (two
// MFMA passes), since 8 significant bits would cost half the error budget.
template <class T, int WR, int WC>
__global__ __launch_bounds__(WR * WC * 64) void apply_project_kernel(const T* __restrict__ q_ms,
                                                            const char* __restrict__ kvfrag,
                                                            const float* __restrict__ kvscale,
                                                            const T* __restrict__ w_proj, T* __restrict__ out,
                                                            int N, int n_hb, int c_out, int blocks_per_image,
                                                            int n_rb, float eps, const T* __restrict__ res) {
    typedef GemmTile<T, WR, WC> G;
    typedef typename Traits<T>::Frag Frag;
    constexpr int HB = G::BK / 16;   // head-branches per iteration
    constexpr int kWaves = G::kThreads / 64;
    constexpr int TG = (G::BC / 16) / kWaves;   // 16-token groups per wave for the attention rows
    static_assert(TG >= 1 && TG * kWaves * 16 == G::BC, "token groups must divide over the waves");
    constexpr bool kHiLo = Traits<T>::kHiLo;
    extern __shared__ __attribute__((aligned(16))) char lds[];
    char* ldsR = lds;
    char* ldsC = lds + G::kLdsR;
    char* ldsC_lo = ldsC + G::kLdsC;   // only with kHiLo

    const unsigned L = xcd_remap(blockIdx.x, gridDim.x);
    const int rb = L % n_rb;
    const unsigned tb = L / n_rb;
    const int b = tb / blocks_per_image;
    const int n0 = (tb % blocks_per_image) * G::BC;
    const int oc0 = rb * G::BR;
    const int wave = threadIdx.x >> 6;
    const int wr = wave % WR, wc = wave / WR;
    const int x16 = lane_id() & 15, q = lane_id() >> 4;
    const int K = n_hb * 16;

    // this lane's tokens for the attention rows: token groups wave, wave + kWaves, ...
    bool ok[TG];
    const T* q_row[TG];
#pragma unroll
    for (int g = 0; g < TG; ++g) {
        const int n_mine = n0 + (g * kWaves + wave) * 16 + x16;
        ok[g] = n_mine < N;
        q_row[g] = q_ms + ((long)b * N + n_mine) * K + q * 4;
    }
    const long sid0 = (long)b * n_hb;

    f32x4 acc[4][4];
    G::zero(acc);
    u32x4 rw[G::kVecR];
    Frag qreg[TG][HB];
    // the state operands of a slab's head-branches are requested one slab ahead, like the weights
    StateOps<T> st[HB];
    auto fetch_states = [&](int m) {
#pragma unroll
        for (int j = 0; j < HB; ++j) {
            const bool live = m + j < n_hb;
            st[j] = load_state_ops<T>(kvfrag, kvscale, sid0 + (live ? m + j : 0), eps, live);
        }
    };
    G::load_global(rw, w_proj, oc0, c_out, K, 0, K);
    fetch_states(0);
#pragma unroll
    for (int g = 0; g < TG; ++g)
#pragma unroll
        for (int j = 0; j < HB; ++j)
            qreg[g][j] = (ok[g] && j < n_hb) ? load_frag<T>(q_row[g] + j * 16) : frag_zero<T>();

    for (int k0 = 0; k0 < K; k0 += G::BK) {
        G::store_lds_r(ldsR, rw);
        const int m0 = k0 >> 4;
#pragma unroll
        for (int j = 0; j < HB; ++j) {
            const bool live = m0 + j < n_hb;
#pragma unroll
            for (int g = 0; g < TG; ++g) {
                f32x4 o = {0.f, 0.f, 0.f, 0.f};
                if (live) o = att_unit<T>(qreg[g][j], st[j]);
                const int colb = (j * 16 + q * 4) * (int)sizeof(T);      // byte column inside the 128-byte slab
                const int off = ((g * kWaves + wave) * 16 + x16) * G::kRow + colb;
                if constexpr (kHiLo) {
                    Frag hi, lo;
                    frag_split<T>(o, hi, lo);
                    store_frag<T>(ldsC + off, hi);
                    store_frag<T>(ldsC_lo + off, lo);
                } else {
                    store_frag<T>(ldsC + off, frag_from_f32<T>(o));
                }
            }
        }
        __syncthreads();
        if (k0 + G::BK < K) {
            G::load_global(rw, w_proj, oc0, c_out, K, k0 + G::BK, K);
            const int m1 = m0 + HB;
            fetch_states(m1);
#pragma unroll
            for (int g = 0; g < TG; ++g)
#pragma unroll
                for (int j = 0; j < HB; ++j)
                    qreg[g][j] = (ok[g] && m1 + j < n_hb) ? load_frag<T>(q_row[g] + (m1 + j) * 16) : frag_zero<T>();
        }
        G::mma(acc, ldsR, ldsC, wr, wc);
        if constexpr (kHiLo) G::mma(acc, ldsR, ldsC_lo, wr, wc);
        __syncthreads();
    }
    const long tok0 = (long)b * N + n0;
    G::epilogue(acc, tok0, (long)b * N + N, oc0, c_out, wr, wc,
                [out, res, c_out](long tok, int oc, f32x4 v) {
                    if (res != nullptr) {
                        const f32x4 r = frag_to_f32<T>(load_frag<T>(res + tok * c_out + oc));
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] += r[e];
                    }
                    store_frag<T>(out + tok * c_out + oc, frag_from_f32<T>(v));
                });
}

// ------------------------------------------- att fused into projection, weight-stationary
// The same fusion for a contraction of at most 512 slots (n_hb <= 2*KCH head-branches): a wave
// keeps the projection weights of its IO*16 output channels in registers for the whole kernel, and
// the (scaled) state operands of its own KCH/4 head-branches for as long as the image lasts.  A
// workgroup of 8 waves owns 8*IO*16 output channels and walks over tiles of 32 tokens of one image:
// every wave makes the attention rows of its head-branches for the tile -- two MFMAs per 16 tokens
// and head-branch -- and writes them to the tile in LDS; after the barrier every wave reads the
// whole tile as MFMA operands against its weights.
//
// fp16 runs this as one software pipeline with a single barrier per tile: while the matrix cores
// work through tile t (16 chunks of IO*2 MFMAs), the same instruction stream carries, dealt out
// between the chunks, the attention rows of tile t+1 (three stages per unit), the copy of the Q
// tile t+2 from registers to LDS, the request for Q tile t+3, and the stores of tile t-1's results.
// Measured with the shader clock, a period that keeps those jobs in blocks of their own around the
// MFMAs spends 60 % of its cycles outside the matrix instructions, all waves idling together.
// bf16 needs the LDS for the hi and lo tiles and keeps the phases apart (two barriers per tile).
//
// LDS tiles are [128-byte slab][token][128 bytes] without padding; the 16-byte chunk index of a row
// is XOR-ed with (row / 2) % 8, which keeps the 16-byte operand reads (16 consecutive rows of one
// chunk), the row-order copies (8 lanes per row) and the 8-byte attention accesses conflict-free.
template <class T, int KCH, int IO>
struct WsApply {
    static_assert(sizeof(T) == 2 && KCH % 4 == 0, "16-bit elements; whole head-branch quadruples");
    static constexpr bool kHiLo = Traits<T>::kHiLo;
    static constexpr int kWaves = 8, kThreads = 512;
    static constexpr int JT = 2, TB = JT * 16;           // tokens per tile
    static constexpr int HBW = KCH / 4;                  // head-branches per wave
    static constexpr int kUnits = JT * HBW;              // attention units per wave and tile
    static constexpr int kChanWave = IO * 16, kChanBlock = kWaves * kChanWave;
    static constexpr int NS = KCH / 2;                   // 128-byte slabs per attention row
    static constexpr int kRow = 128;
    static constexpr int kSlab = TB * kRow;
    static constexpr int kBuf = NS * kSlab;              // one attention tile or Q tile
    static constexpr int kQV = NS / 2;                   // 16-byte vectors per thread of a Q tile
    static constexpr int kWeightStage = kChanBlock * kRow;
    // bf16 keeps hi and lo attention tiles.  Where six tiles fit the LDS (up to 24 head-branches) it runs
    // the same single-barrier pipeline as fp16 with two hi, two lo and two Q tiles; beyond that, hi,
    // lo and one Q tile with the phases kept apart.
    static constexpr bool kPipeHiLo = kHiLo && 6 * kBuf <= 160 * 1024;
    static constexpr int kTiles = (kPipeHiLo ? 6 : 4) * kBuf;
    static constexpr int kLds = kTiles;
    static_assert(kWeightStage <= kTiles, "the weights are staged through the tile area");
    static_assert(NS % 2 == 0 && TB * 16 == kThreads, "the Q tile copy takes two slabs per pass");
    static_assert(KCH == 2 * kUnits, "one attention unit per two chunks of matrix instructions");
};

__device__ __forceinline__ int lds_swizzle(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }

template <class T, int KCH, int IO, bool kRes>
__global__ __launch_bounds__(512) void apply_project_ws_kernel(const T* __restrict__ q_ms,
                                                               const char* __restrict__ kvfrag,
                                                               const float* __restrict__ kvscale,
                                                               const T* __restrict__ w_proj, T* __restrict__ out,
                                                               int N, int n_hb, int c_out, int n_cg,
                                                               int tiles_per_image, long n_tt,
                                                               long tiles_per_block, float eps,
                                                               const T* __restrict__ res) {
    typedef WsApply<T, KCH, IO> S;
    typedef Traits<T> Tr;
    typedef typename Tr::Vec Vec;
    typedef typename Tr::Frag Frag;
    constexpr bool kHiLo = S::kHiLo;
    constexpr int kUnits = S::kUnits;
    extern __shared__ __attribute__((aligned(16))) char lds[];

    const unsigned L = xcd_remap(blockIdx.x, gridDim.x);
    const int cg = (int)(L % (unsigned)n_cg);
    const long t_begin = (long)(L / (unsigned)n_cg) * tiles_per_block;
    const long t_end = t_begin + tiles_per_block < n_tt ? t_begin + tiles_per_block : n_tt;
    if (t_begin >= t_end) return;
    const int n_mine = (int)(t_end - t_begin);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = lane_id(), x16 = lane & 15, q = lane >> 4;
    const int K = n_hb * 16;
    const unsigned row_bytes = (unsigned)K * 2u;
    const int ch0 = cg * S::kChanBlock + wave * S::kChanWave;

    // tile number -> (image, first token in it, that token's index in the whole map), walked with
    // counters: no division and no wide multiplication in the loop (the scalar unit runs a wave's
    // instructions one after the other, some eight cycles each)
    struct Origin {
        int b, n0;
        unsigned tok;
    };
    auto advance = [&](Origin o) {
        const int left = N - o.n0;                  // tokens of the image from this tile on
        o.tok += left < S::TB ? left : S::TB;
        if (left <= S::TB) { o.n0 = 0; ++o.b; }
        else o.n0 += S::TB;
        return o;
    };
    const Origin first = {(int)(t_begin / tiles_per_image), (int)(t_begin % tiles_per_image) * S::TB,
                          (unsigned)((t_begin / tiles_per_image) * N + (t_begin % tiles_per_image) * S::TB)};

    // ---- Q tile: copied in row order (8 lanes per 128-byte row segment; read as fragments straight
    // from memory every lane would touch its own row) into LDS.  Rows past the image's last token
    // and tiles past this workgroup's last read as zero.
    const int q_slab = threadIdx.x >> 8, q_row = (threadIdx.x >> 3) & 31, q_chunk = threadIdx.x & 7;
    const int q_lds = q_slab * S::kSlab + q_row * S::kRow + lds_swizzle(q_row, q_chunk) * 16;
    const unsigned q_glb = q_row * row_bytes + q_slab * 128 + q_chunk * 16;
    u32x4 qv[S::kQV];
    BufRsrc qres;
    auto aim_q = [&](Origin o, bool live) {
        const int rows = live ? (N - o.n0 < S::TB ? N - o.n0 : S::TB) : 0;
        qres = make_rsrc_small(q_ms + (size_t)o.tok * (unsigned)K, (unsigned)rows * row_bytes);
    };
    auto fetch_q1 = [&](int i) {
        qv[i] = buf_load16(qres, q_slab * 128 + q_chunk * 16 + i * 256 < row_bytes ? q_glb + i * 256 : kOobOffset, 0);
    };
    // Eq. (3) only ever sees relu(Q): the rectifier is applied here, once per element, as integer
    // maxima on the bit patterns (negative values and -0 have the sign bit set)
    auto park_q1 = [&](int qb, int i) {       // qb: byte offset of the Q tile in LDS
        typedef short i16x8 __attribute__((ext_vector_type(8)));
        const i16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
        const i16x8 r = __builtin_elementwise_max(__builtin_bit_cast(i16x8, qv[i]), zero);
        *(u32x4*)(lds + qb + q_lds + 2 * i * S::kSlab) = __builtin_bit_cast(u32x4, r);
    };

    aim_q(first, true);      // requested ahead of the weights, so the first tile does not queue behind them
#pragma unroll
    for (int i = 0; i < S::kQV; ++i) fetch_q1(i);

    // ---- weights -> registers, copied in row order through LDS (fragment reads straight from
    // memory would touch one cache line per lane).  The registers the slabs wait in are the ones the
    // fragments move into.  The CU's address path needs longer for the 32 loads per thread than the
    // data takes to arrive, so the requests run kAheadW slabs ahead of the staging instead of all
    // being issued first: the staging of a slab then overlaps with the requests of the later ones.
    Vec wf[IO][KCH];
    const int g16 = (x16 >> 1) & 7;
    {
        const BufRsrc wres = make_rsrc(w_proj, (long)c_out * row_bytes);
        constexpr int kWV = S::kChanBlock * 8 / S::kThreads;      // vectors per thread and slab
        constexpr int kAheadW = S::NS < MSLA_APPLY_W_AHEAD ? S::NS : MSLA_APPLY_W_AHEAD;
        unsigned base[kWV];
        int wl[kWV];
#pragma unroll
        for (int i = 0; i < kWV; ++i) {
            const int r = (threadIdx.x + i * S::kThreads) >> 3;
            const int row = cg * S::kChanBlock + r;
            base[i] = row < c_out ? (unsigned)row * row_bytes + (threadIdx.x & 7) * 16 : kOobOffset;
            wl[i] = r * S::kRow + lds_swizzle(r, threadIdx.x & 7) * 16;
        }
        u32x4 wr[S::NS][kWV];
        auto request = [&](int sl) {
#pragma unroll
            for (int i = 0; i < kWV; ++i)
                wr[sl][i] = buf_load16(wres, (base[i] != kOobOffset && sl * 128 + (threadIdx.x & 7) * 16 < row_bytes)
                                                 ? base[i] + sl * 128 : kOobOffset, 0);
        };
#pragma unroll
        for (int sl = 0; sl < kAheadW; ++sl) request(sl);
#pragma unroll
        for (int sl = 0; sl < S::NS; ++sl) {
            if (sl) __syncthreads();
#pragma unroll
            for (int i = 0; i < kWV; ++i) *(u32x4*)(lds + wl[i]) = wr[sl][i];
            if (sl + kAheadW < S::NS) request(sl + kAheadW);
            __syncthreads();
#pragma unroll
            for (int io = 0; io < IO; ++io)
#pragma unroll
                for (int h = 0; h < 2; ++h)
                    wf[io][2 * sl + h] = __builtin_bit_cast(
                        Vec, *(const u32x4*)(lds + (wave * S::kChanWave + io * 16 + x16) * S::kRow + ((h * 4 + q) ^ g16) * 16));
        }
        __syncthreads();
    }

    // ---- this wave's head-branches: state operands and eps*scale, reloaded when the image changes
    Vec a_kv[S::HBW], a_ks[S::HBW];
    float eps_s[S::HBW];
    int img = -1;
    auto load_state = [&](int b) {
#pragma unroll
        for (int j = 0; j < S::HBW; ++j) {
            const int hb = wave * S::HBW + j;
            const long sid = (long)b * n_hb + (hb < n_hb ? hb : 0);
            a_kv[j] = __builtin_bit_cast(Vec, *(const u32x4*)(kvfrag + sid * 2048 + lane * 16));
            a_ks[j] = __builtin_bit_cast(Vec, *(const u32x4*)(kvfrag + sid * 2048 + 1024 + lane * 16));
            eps_s[j] = eps * kvscale[sid];
        }
        img = b;
    };

    // ---- attention rows of unit u = (jt, j) = 16 tokens x head-branch wave*HBW + j: Q tile ->
    // attention tile(s), a lane handling channels 4q..4q+3 of its token.  Three stages (request Q;
    // rectify and issue the two MFMAs; normalise and store) that the callers place in different
    // slots of their instruction stream, so no stage waits for the one before it.
    Frag att_q[2];
    f32x4 att_num, att_den;
    auto unit_off = [&](int u) {
        const int hb = wave * S::HBW + u % S::HBW;
        const int chunk = (hb & 3) * 2 + (q >> 1);
        return (hb >> 2) * S::kSlab + ((u / S::HBW) * 16 + x16) * S::kRow + (chunk ^ g16) * 16 + (q & 1) * 8;
    };
    auto att_a = [&](int qb, int u) { att_q[u & 1] = load_frag<T>((const T*)(lds + qb + unit_off(u))); };
    auto att_b = [&](int u) {
        const f32x4 z = {0.f, 0.f, 0.f, 0.f};
        const Frag qf = att_q[u & 1];         // rectified when the tile was parked
        Vec b;
#pragma unroll
        for (int r = 0; r < 4; ++r) { b[r] = qf[r]; b[4 + r] = qf[r]; }   // pairs with {hi, lo} of the state
        att_num = Tr::mma_vec(z, a_kv[u % S::HBW], b);
        att_den = Tr::mma_vec(z, a_ks[u % S::HBW], b);
    };
    auto att_c = [&](int u, int hi_tile, int lo_tile) {
        const int hb = wave * S::HBW + u % S::HBW;
        const f32x4 num = att_num;
        const float inv = hb < n_hb ? __builtin_amdgcn_rcpf(att_den[0] + eps_s[u % S::HBW]) : 0.f;
        const f32x4 o = {num[0] * inv, num[1] * inv, num[2] * inv, num[3] * inv};
        const int off = unit_off(u);
        if constexpr (kHiLo) {
            Frag hi, lo;
            frag_split<T>(o, hi, lo);
            store_frag<T>(lds + hi_tile + off, hi);
            store_frag<T>(lds + lo_tile + off, lo);
        } else {
            store_frag<T>(lds + hi_tile + off, frag_from_f32<T>(o));
        }
    };
    // all units of a tile, the stages of neighbouring units overlapped
    auto att_all = [&](int qb, int hi_tile, int lo_tile) {
        att_a(qb, 0);
#pragma unroll
        for (int u = 0; u < kUnits; ++u) {
            att_b(u);
            if (u + 1 < kUnits) att_a(qb, u + 1);
            att_c(u, hi_tile, lo_tile);
        }
    };

    // ---- projection: token-operand fragments are requested kAhead chunks ahead of their use (one
    // where the weights alone take half the register file)
    constexpr int kAhead = IO * KCH >= 32 ? 1 : 2;
    constexpr int kRing = kAhead + 1;
    f32x4 acc[IO][S::JT];
    const int frag_off = x16 * S::kRow + (q ^ g16) * 16;       // chunk (kk&1)*4 + q: the second half is ^ 64
    Vec bf[kRing][S::JT];
    Vec bl[S::kPipeHiLo ? kRing : 1][S::JT];          // the lo fragments of the pipelined hi/lo form
    auto read_b = [&](int tile, int kk) {
#pragma unroll
        for (int jt = 0; jt < S::JT; ++jt)
            bf[kk % kRing][jt] = __builtin_bit_cast(
                Vec, *(const u32x4*)(lds + tile + (frag_off ^ ((kk & 1) * 64)) + (kk >> 1) * S::kSlab + jt * 16 * S::kRow));
    };
    auto read_b_lo = [&](int tile, int kk) {
#pragma unroll
        for (int jt = 0; jt < S::JT; ++jt)
            bl[S::kPipeHiLo ? kk % kRing : 0][jt] = __builtin_bit_cast(
                Vec, *(const u32x4*)(lds + tile + (frag_off ^ ((kk & 1) * 64)) + (kk >> 1) * S::kSlab + jt * 16 * S::kRow));
    };
    auto mma_chunk = [&](int kk) {
#pragma unroll
        for (int io = 0; io < IO; ++io)
#pragma unroll
            for (int jt = 0; jt < S::JT; ++jt) acc[io][jt] = Tr::mma_vec(acc[io][jt], wf[io][kk], bf[kk % kRing][jt]);
    };
    auto mma_chunk_lo = [&](int kk) {
#pragma unroll
        for (int io = 0; io < IO; ++io)
#pragma unroll
            for (int jt = 0; jt < S::JT; ++jt)
                acc[io][jt] = Tr::mma_vec(acc[io][jt], wf[io][kk], bl[S::kPipeHiLo ? kk % kRing : 0][jt]);
    };
    auto zero_acc = [&]() {
#pragma unroll
        for (int io = 0; io < IO; ++io)
#pragma unroll
            for (int jt = 0; jt < S::JT; ++jt) acc[io][jt] = f32x4{0.f, 0.f, 0.f, 0.f};
    };

    // ---- results: finish() rounds a tile's accumulators into registers, a lane (token x16, q)
    // holding channels 4q..4q+3 of each 16-channel block: 8 bytes.  flush(p) writes piece p out with
    // one 16-byte store per lane: the odd 16-lane groups of one block are swapped with the even
    // groups of another, which leaves a lane with 8 consecutive channels -- of the two channel blocks
    // of 16 tokens (IO == 2: channels 16*(q%2) + 8*(q/2) .. +7 of token x16), or of one channel block
    // of both token groups (IO == 1: channels 8*(q/2) .. +7 of token 16*(q%2) + x16).
    static_assert(IO == 1 || IO == 2, "two 8-byte halves per store");
    constexpr int kPieces = IO == 2 ? S::JT : S::JT / 2;
    Frag pend[IO][S::JT];
    BufRsrc ores;
    const unsigned out_row = (unsigned)c_out * 2u;
    // (kRes: out = res + ..., the residual joining the fp32 sums before their one rounding --
    // the block's y = x + MSLA(x); o is the origin of the tile the accumulators belong to)
    auto finish = [&](Origin o) {
#pragma unroll
        for (int io = 0; io < IO; ++io)
#pragma unroll
            for (int jt = 0; jt < S::JT; ++jt) {
                f32x4 v = acc[io][jt];
                if constexpr (kRes) {
                    const int row = jt * 16 + x16, oc = ch0 + io * 16 + q * 4;
                    if (row < N - o.n0 && oc < c_out) {
                        const f32x4 r = frag_to_f32<T>(load_frag<T>(res + ((size_t)o.tok + row) * (unsigned)c_out + oc));
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] += r[e];
                    }
                }
                pend[io][jt] = frag_from_f32<T>(v);
            }
    };
    auto aim_out = [&](Origin o, bool live) {
        const int rows = live ? (N - o.n0 < S::TB ? N - o.n0 : S::TB) : 0;
        ores = make_rsrc_small(out + (size_t)o.tok * (unsigned)c_out, (unsigned)rows * out_row);
    };
    auto flush = [&](int p) {
        u32x2 even, odd;
        if constexpr (IO == 2) {
            even = __builtin_bit_cast(u32x2, pend[0][p]);
            odd = __builtin_bit_cast(u32x2, pend[IO - 1][p]);
        } else {
            even = __builtin_bit_cast(u32x2, pend[0][2 * p]);
            odd = __builtin_bit_cast(u32x2, pend[0][2 * p + 1]);
        }
        const u32x2 s0 = __builtin_amdgcn_permlane16_swap(even[0], odd[0], false, false);
        const u32x2 s1 = __builtin_amdgcn_permlane16_swap(even[1], odd[1], false, false);
        const int row = IO == 2 ? p * 16 + x16 : (2 * p + (q & 1)) * 16 + x16;
        const int oc = ch0 + (IO == 2 ? (q & 1) * 16 : 0) + (q >> 1) * 8;
        buf_store16_stream(ores, oc < c_out ? (unsigned)row * out_row + oc * 2u : kOobOffset,
                           u32x4{s0[0], s1[0], s0[1], s1[1]});
    };
    auto flush_all = [&](Origin o) {
        aim_out(o, true);
#pragma unroll
        for (int p = 0; p < kPieces; ++p) flush(p);
    };

    // the four tiles as byte offsets into LDS (plain numbers: a pointer chosen at run time would be
    // checked against null wherever something is added to it)
    constexpr int att0 = 0, att1 = S::kBuf, qb0 = 2 * S::kBuf, qb1 = 3 * S::kBuf;
    constexpr int lo0 = 4 * S::kBuf, lo1 = 5 * S::kBuf;      // (pipelined hi/lo form only)
    if constexpr (!kHiLo || S::kPipeHiLo) {
        // prologue: Q tiles 0 and 1 parked, Q tile 2 requested, attention rows of tile 0 made
        Origin o_att = first;                 // tile whose attention rows are made next
        Origin o_q = advance(first);          // tile whose Q is requested next
#pragma unroll
        for (int i = 0; i < S::kQV; ++i) park_q1(qb0, i);
        aim_q(o_q, 1 < n_mine);
#pragma unroll
        for (int i = 0; i < S::kQV; ++i) fetch_q1(i);
#pragma unroll
        for (int i = 0; i < S::kQV; ++i) park_q1(qb1, i);
        o_q = advance(o_q);
        aim_q(o_q, 2 < n_mine);
#pragma unroll
        for (int i = 0; i < S::kQV; ++i) fetch_q1(i);
        load_state(o_att.b);
        __syncthreads();
        att_all(qb0, att0, lo0);
        __syncthreads();
        Origin o_out = first;                 // tile whose results are written next
        o_att = advance(o_att);
        for (int t = 0; t < n_mine; ++t) {
            const bool odd = t & 1;
            const int here = odd ? att1 : att0;         // attention rows of tile t
            const int next = odd ? att0 : att1;         // ... of tile t+1, made now
            const int here_lo = odd ? lo1 : lo0, next_lo = odd ? lo0 : lo1;
            const int q_next = odd ? qb0 : qb1;         // Q of tile t+1
            const int q_park = odd ? qb1 : qb0;         // Q of tile t+2 goes where tile t's was
            if (t + 1 < n_mine && o_att.b != img) load_state(o_att.b);
            o_q = advance(o_q);
            aim_q(o_q, t + 3 < n_mine);                 // resource of Q tile t+3
            aim_out(o_out, t > 0);                      // ... and of the results of tile t-1 (none before the first)
            zero_acc();
            read_b(here, 0);
            if constexpr (S::kPipeHiLo) read_b_lo(here_lo, 0);
            if constexpr (kAhead > 1) {
                read_b(here, 1);
                if constexpr (S::kPipeHiLo) read_b_lo(here_lo, 1);
            }
            att_a(q_next, 0);
            // 16 slots of IO*2 matrix instructions; everything else rides between them.  Past the
            // last tile the extra jobs work on zeros that nobody reads.
            static_for<0, KCH>([&](auto kk_c) {
                constexpr int kk = decltype(kk_c)::value;
                if constexpr (kk + kAhead < KCH) {
                    read_b(here, kk + kAhead);
                    if constexpr (S::kPipeHiLo) read_b_lo(here_lo, kk + kAhead);
                }
                constexpr int u = kk / 2;
                if constexpr (kk % 2 == 0) {
                    att_b(u);
                    if constexpr (u + 1 < kUnits) att_a(q_next, u + 1);
                } else {
                    att_c(u, next, next_lo);
                }
                mma_chunk(kk);
                if constexpr (S::kPipeHiLo) mma_chunk_lo(kk);
                // Q tile t+2: registers -> LDS, then the same registers take the request for tile t+3
                constexpr int kParkAt = 1, kFetchAt = 3;
                if constexpr (kk >= kParkAt && kk < kParkAt + S::kQV) park_q1(q_park, kk - kParkAt);
                if constexpr (kk >= kFetchAt && kk < kFetchAt + S::kQV) fetch_q1(kk - kFetchAt);
                // results of tile t-1, a piece at a time
                static_assert(kFetchAt + S::kQV <= KCH && S::JT == 2, "slot plan");
                if constexpr (kk == KCH / 4) flush(0);
                if constexpr (kPieces > 1 && kk == 3 * KCH / 4) flush(1);
                __builtin_amdgcn_sched_barrier(0);
            });
            if (t > 0) o_out = advance(o_out);
            finish(o_out);
            o_att = advance(o_att);
            __syncthreads();
        }
        flush_all(o_out);
    } else {
        Origin o = first, o_q = first, o_out = first;
        for (int t = 0; t < n_mine; ++t) {
            if (o.b != img) load_state(o.b);
#pragma unroll
            for (int i = 0; i < S::kQV; ++i) park_q1(qb0, i);
            if (t > 0) {
                flush_all(o_out);
                o_out = advance(o_out);
            }
            o_q = advance(o_q);
            aim_q(o_q, t + 1 < n_mine);
#pragma unroll
            for (int i = 0; i < S::kQV; ++i) fetch_q1(i);
            __syncthreads();           // Q tile complete; every wave is done with the previous tiles
            att_all(qb0, att0, att1);
            __syncthreads();
            zero_acc();
            read_b(att0, 0);
#pragma unroll
            for (int kk = 0; kk < KCH; ++kk) {
                // the hi fragments come through the ring, one chunk ahead; the lo ones are read here
                Vec lo[S::JT];
#pragma unroll
                for (int jt = 0; jt < S::JT; ++jt)
                    lo[jt] = __builtin_bit_cast(
                        Vec, *(const u32x4*)(lds + att1 + (frag_off ^ ((kk & 1) * 64)) + (kk >> 1) * S::kSlab + jt * 16 * S::kRow));
                if (kk + 1 < KCH) read_b(att0, kk + 1);
                mma_chunk(kk);
#pragma unroll
                for (int io = 0; io < IO; ++io)
#pragma unroll
                    for (int jt = 0; jt < S::JT; ++jt) acc[io][jt] = Tr::mma_vec(acc[io][jt], wf[io][kk], lo[jt]);
            }
            finish(o);
            o = advance(o);
        }
        flush_all(o_out);
    }
}

template <class T, int KCH, int IO>
hipError_t run_apply_project_ws(const void* q_ms, const void* kvfrag, const float* kvscale, const void* w_proj,
                                void* out, const void* res, long n_tokens, int N, int n_hb, int c_out, float eps,
                                hipStream_t stream) {
    typedef WsApply<T, KCH, IO> S;
    const int n_cg = (c_out + S::kChanBlock - 1) / S::kChanBlock;
    const int tiles_per_image = (N + S::TB - 1) / S::TB;
    const long n_tt = (n_tokens / N) * tiles_per_image;
    if (n_tt <= 0 || n_tt * n_cg > 0x7fffffffL) return hipErrorInvalidValue;
    if ((long)c_out * n_hb * 32 >= 0x7fffffffL) return hipErrorInvalidValue;
    const long slots = compute_units();
    const long groups = slots / n_cg > 0 ? slots / n_cg : 1;
    const long tiles_per_block = (n_tt + groups - 1) / groups;
    const long nblocks = (n_tt + tiles_per_block - 1) / tiles_per_block * n_cg;
    // (the residual path is compiled apart: the headline variant has no register to spare for it)
    if (res != nullptr) {
        const hipError_t e = allow_dynamic_lds<apply_project_ws_kernel<T, KCH, IO, true>>(S::kLds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((apply_project_ws_kernel<T, KCH, IO, true>), dim3((unsigned)nblocks), dim3(S::kThreads), S::kLds,
                           stream, (const T*)q_ms, (const char*)kvfrag, kvscale, (const T*)w_proj, (T*)out, N, n_hb,
                           c_out, n_cg, tiles_per_image, n_tt, tiles_per_block, eps, (const T*)res);
    } else {
        const hipError_t e = allow_dynamic_lds<apply_project_ws_kernel<T, KCH, IO, false>>(S::kLds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((apply_project_ws_kernel<T, KCH, IO, false>), dim3((unsigned)nblocks), dim3(S::kThreads), S::kLds,
                           stream, (const T*)q_ms, (const char*)kvfrag, kvscale, (const T*)w_proj, (T*)out, N, n_hb,
                           c_out, n_cg, tiles_per_image, n_tt, tiles_per_block, eps, (const T*)res);
    }
    return hipGetLastError();
}

template <class T>
hipError_t run_apply(const void* q_ms, const void* kvfrag, const float* kvscale, void* att, long n_tokens,
                     int N, int n_hb, float eps, hipStream_t stream) {
    const int gpi = (N + 15) / 16;
    const long n_groups = (n_tokens / N) * gpi;
    const long nblocks = (n_groups + 3) / 4;
    if (nblocks <= 0 || nblocks > 0x7fffffffL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((apply_kernel<T>), dim3((unsigned)nblocks), dim3(256), 0, stream, (const T*)q_ms,
                       (const char*)kvfrag, kvscale, (T*)att, N, n_hb, gpi, n_groups, eps);
    return hipGetLastError();
}

template <class T, int WR, int WC>
hipError_t run_apply_project_tiled(const void* q_ms, const void* kvfrag, const float* kvscale, const void* w_proj,
                                   void* out, const void* res, long n_tokens, int N, int n_hb, int c_out, float eps,
                                   hipStream_t stream) {
    typedef GemmTile<T, WR, WC> G;
    const int bpi = (N + G::BC - 1) / G::BC;
    const int n_rb = (c_out + G::BR - 1) / G::BR;
    const long nblocks = (n_tokens / N) * bpi * n_rb;
    if (nblocks <= 0 || nblocks > 0x7fffffffL) return hipErrorInvalidValue;
    constexpr int kLds = G::kLdsR + G::kLdsC * (Traits<T>::kHiLo ? 2 : 1);
    if (kLds > 48 * 1024) {   // above the default dynamic-LDS limit (the CU has 160 KB)
        const hipError_t e = allow_dynamic_lds<apply_project_kernel<T, WR, WC>>(kLds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((apply_project_kernel<T, WR, WC>), dim3((unsigned)nblocks), dim3(G::kThreads), kLds, stream,
                       (const T*)q_ms, (const char*)kvfrag, kvscale, (const T*)w_proj, (T*)out, N, n_hb, c_out,
                       bpi, n_rb, eps, (const T*)res);
    return hipGetLastError();
}

template <class T>
hipError_t run_apply_project(const void* q_ms, const void* kvfrag, const float* kvscale, const void* w_proj,
                             void* out, const void* res, long n_tokens, int N, int n_hb, int c_out, float eps,
                             hipStream_t stream) {
#ifndef MSLA_APPLY_NO_WS
    if constexpr (sizeof(T) == 2) {
        // short contraction: weights and states stay in registers
        if (n_hb <= 32) {
            const bool narrow = c_out <= 128;
            if (n_hb <= 16)
                return narrow ? run_apply_project_ws<T, 8, 1>(q_ms, kvfrag, kvscale, w_proj, out, res, n_tokens, N, n_hb, c_out, eps, stream)
                              : run_apply_project_ws<T, 8, 2>(q_ms, kvfrag, kvscale, w_proj, out, res, n_tokens, N, n_hb, c_out, eps, stream);
            if (n_hb <= 24)
                return narrow ? run_apply_project_ws<T, 12, 1>(q_ms, kvfrag, kvscale, w_proj, out, res, n_tokens, N, n_hb, c_out, eps, stream)
                              : run_apply_project_ws<T, 12, 2>(q_ms, kvfrag, kvscale, w_proj, out, res, n_tokens, N, n_hb, c_out, eps, stream);
            return narrow ? run_apply_project_ws<T, 16, 1>(q_ms, kvfrag, kvscale, w_proj, out, res, n_tokens, N, n_hb, c_out, eps, stream)
                          : run_apply_project_ws<T, 16, 2>(q_ms, kvfrag, kvscale, w_proj, out, res, n_tokens, N, n_hb, c_out, eps, stream);
        }
    }
#endif
    // Tiled form: 64 x 64 per wave, 256 channels x 128 tokens per workgroup; a map too small to give
    // every CU such a tile takes 64-token tiles (measured on the 2048- and 1024-token workloads: 33
    // against 45 us and 17 against 25 us; still smaller workgroups were slower again)
    const long blocks = (n_tokens / N) * ((N + 64 * MSLA_APPLY_WC - 1) / (64 * MSLA_APPLY_WC)) *
                        ((c_out + 64 * MSLA_APPLY_WR - 1) / (64 * MSLA_APPLY_WR));
    if (MSLA_APPLY_WC == 2 && blocks < compute_units())
        return run_apply_project_tiled<T, MSLA_APPLY_WR, 1>(q_ms, kvfrag, kvscale, w_proj, out, res, n_tokens, N, n_hb, c_out, eps, stream);
    return run_apply_project_tiled<T, MSLA_APPLY_WR, MSLA_APPLY_WC>(q_ms, kvfrag, kvscale, w_proj, out, res, n_tokens, N, n_hb, c_out, eps, stream);
}

}  // namespace

hipError_t launch_apply(int dt, const void* q_ms, const void* kvfrag, const float* kvscale, void* att,
                        long n_tokens, int tokens_per_image, int n_hb, float eps, hipStream_t stream) {
    switch (dt) {
        case 0: return run_apply<float>(q_ms, kvfrag, kvscale, att, n_tokens, tokens_per_image, n_hb, eps, stream);
        case 1: return run_apply<_Float16>(q_ms, kvfrag, kvscale, att, n_tokens, tokens_per_image, n_hb, eps, stream);
        case 2: return run_apply<__bf16>(q_ms, kvfrag, kvscale, att, n_tokens, tokens_per_image, n_hb, eps, stream);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_apply_project(int dt, const void* q_ms, const void* kvfrag, const float* kvscale,
                                const void* w_proj, void* out, const void* res, long n_tokens, int tokens_per_image,
                                int n_hb, int c_out, float eps, hipStream_t stream) {
    // more head-branches than the register-resident form holds: the long-contraction kernel
    if (n_hb > 32 && small_product(dt, n_tokens, n_hb * 16, c_out))
        return launch_small_apply_project(dt, q_ms, kvfrag, kvscale, w_proj, out, res, n_tokens, tokens_per_image, n_hb, c_out,
                                          eps, stream);
    switch (dt) {
        case 0: return run_apply_project<float>(q_ms, kvfrag, kvscale, w_proj, out, res, n_tokens, tokens_per_image, n_hb, c_out, eps, stream);
        case 1: return run_apply_project<_Float16>(q_ms, kvfrag, kvscale, w_proj, out, res, n_tokens, tokens_per_image, n_hb, c_out, eps, stream);
        case 2: return run_apply_project<__bf16>(q_ms, kvfrag, kvscale, w_proj, out, res, n_tokens, tokens_per_image, n_hb, c_out, eps, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace msla
