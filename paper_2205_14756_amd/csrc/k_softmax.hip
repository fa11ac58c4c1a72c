// Softmax attention, the comparison point of ReLU linear attention (Section 3.1: Eq. (1) with
// Sim(Q, K) = exp(Q K^T / sqrt(d)); Fig. 3 compares the latency of the two forms):
//     O_i = sum_j exp(Q_i . K_j / sqrt(d)) V_j / sum_j exp(Q_i . K_j / sqrt(d))
// per image and head on a projected map qkv [B, N, 3*heads*16] (channel (h*3 + t)*16 + e).
//
// It is quadratic in N by definition; it is written the way such a kernel is written when it has to
// be fast (one pass over the keys with a running maximum and running sums, nothing of size N x N
// ever stored), so that the ratio to the linear form is a fair one.  A workgroup of 4 waves takes
// 64 queries of one (image, head), a wave 16 of them, and walks over the keys 64 at a time:
//     S^T[key][query] = K . Q^T      one 16x16x16 MFMA per 16 keys; lane (query x16, q) gets keys 4q..4q+3
//     running max per query (in-lane over 16 values, two shuffles over the four q groups), P = 2^(S - max)
//     O^T[f][query]  += V^T . P^T    one MFMA per 16 keys; P's fragment is S's, rounded to the storage type
// K (row-major) and V (transposed, so a lane's four keys are contiguous) go through LDS once per
// workgroup and key block, the next block's loads in flight during the arithmetic.
#include "msla_device.h"
#include "msla_kernels.h"

namespace msla {
namespace {

constexpr int kSmQ = 64;        // queries per workgroup
constexpr int kSmK = 64;        // keys per iteration

template <class T>
__global__ __launch_bounds__(256) void softmax_attention_kernel(const T* __restrict__ qkv, T* __restrict__ att, int N,
                                                                int heads, int q_blocks) {
    typedef Traits<T> Tr;
    typedef typename Tr::Frag Frag;
    constexpr int kFragBytes = 4 * (int)sizeof(T);
    constexpr int kKRow = 16 * (int)sizeof(T) + kFragBytes;          // K tile [key][16 d], padded
    constexpr int kVRow = kSmK * (int)sizeof(T) + kFragBytes;        // V^T tile [f][64 keys], padded
    __shared__ __attribute__((aligned(16))) char ldsK[2][kSmK * kKRow];
    __shared__ __attribute__((aligned(16))) char ldsV[2][16 * kVRow];

    const int qb = blockIdx.x % q_blocks;
    const int h = (blockIdx.x / q_blocks) % heads;
    const int b = blockIdx.x / (q_blocks * heads);
    const int wave = threadIdx.x >> 6, lane = lane_id(), x16 = lane & 15, q = lane >> 4;
    const long ts = 3L * heads * 16;                                  // elements from token to token
    const T* base = qkv + (long)b * N * ts + (long)h * 48;

    // this lane's query (column x16 of the wave's 16): its channels 4q..4q+3, scaled by log2(e)/sqrt(d)
    const int my_query = qb * kSmQ + wave * 16 + x16;
    Frag qf = frag_zero<T>();
    if (my_query < N) qf = load_frag<T>(base + (long)my_query * ts + q * 4);
    constexpr float kScale = 0.25f * 1.4426950408889634f;             // 1/sqrt(16) * log2(e)

    // cooperative loads of a key block: thread t < 128 brings 8 d-channels (or 4, fp32) of K, t >= 128 of V
    constexpr int kVec = 16 / (int)sizeof(T);                         // elements per 16-byte vector
    constexpr int kVecPerRow = 16 / kVec;                             // 2 (16-bit) or 4 (fp32)
    constexpr int kRowsPerPass = 128 / kVecPerRow;                    // keys covered by 128 threads
    constexpr int kPasses = kSmK / kRowsPerPass;                      // 1 (16-bit) or 2 (fp32)
    const int half = threadIdx.x >> 7, t7 = threadIdx.x & 127;
    u32x4 stage[kPasses];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int p = 0; p < kPasses; ++p) {
            const int key = k0 + p * kRowsPerPass + t7 / kVecPerRow;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (key < N) v = *(const u32x4*)(base + (long)key * ts + 16 + half * 16 + (t7 % kVecPerRow) * kVec);
            stage[p] = v;
        }
    };
    auto park = [&](int buf) {
#pragma unroll
        for (int p = 0; p < kPasses; ++p) {
            const int key = p * kRowsPerPass + t7 / kVecPerRow;
            const int c0 = (t7 % kVecPerRow) * kVec;
            if (half == 0) {
                // K: row-major, two (four) 8-byte pieces so that the padded rows stay 8-byte aligned
                const u32x4 v = stage[p];
                *(u32x2*)(ldsK[buf] + key * kKRow + c0 * (int)sizeof(T)) = u32x2{v[0], v[1]};
                *(u32x2*)(ldsK[buf] + key * kKRow + c0 * (int)sizeof(T) + 8) = u32x2{v[2], v[3]};
            } else {
                // V: transposed, element by element
                T e[kVec];
                __builtin_memcpy(e, &stage[p], 16);
#pragma unroll
                for (int j = 0; j < kVec; ++j) *(T*)(ldsV[buf] + (c0 + j) * kVRow + key * (int)sizeof(T)) = e[j];
            }
        }
    };

    float m_run = -INFINITY;            // running maximum of this lane's query (same in its four q lanes)
    float l_run = 0.f;                  // running sum over this lane's own keys
    f32x4 o = {0.f, 0.f, 0.f, 0.f};     // O^T[f = 4q + r][query x16]
    const f32x4 z = {0.f, 0.f, 0.f, 0.f};

    fetch(0);
    park(0);
    __syncthreads();
    const int n_blocks = (N + kSmK - 1) / kSmK;
    for (int blk = 0; blk < n_blocks; ++blk) {
        const int buf = blk & 1;
        if (blk + 1 < n_blocks) fetch((blk + 1) * kSmK);
        // scores of 64 keys x 16 queries: s[g][r] = key 16g + 4q + r
        f32x4 s[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const Frag kf = load_frag<T>(ldsK[buf] + (g * 16 + x16) * kKRow + q * kFragBytes);
            s[g] = Tr::mma16(z, kf, qf);
        }
        float mx = -INFINITY;
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int key = blk * kSmK + g * 16 + q * 4 + r;
                s[g][r] = key < N ? s[g][r] * kScale : -INFINITY;
                mx = fmaxf(mx, s[g][r]);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);             // finite from the first block on: it holds key 0
        const float keep = exp2f(m_run - m_new);
        m_run = m_new;
        l_run *= keep;
#pragma unroll
        for (int r = 0; r < 4; ++r) o[r] *= keep;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            f32x4 p;
#pragma unroll
            for (int r = 0; r < 4; ++r) p[r] = exp2f(s[g][r] - m_new);
            // the sum runs over what the matrix instruction sees, i.e. over the rounded weights
            const Frag pf = frag_from_f32<T>(p);
            const f32x4 pr = frag_to_f32<T>(pf);
            l_run += (pr[0] + pr[1]) + (pr[2] + pr[3]);
            const Frag vf = load_frag<T>(ldsV[buf] + x16 * kVRow + (g * 16 + q * 4) * (int)sizeof(T));
            o = Tr::mma16(o, vf, pf);
        }
        if (blk + 1 < n_blocks) park(buf ^ 1);
        __syncthreads();
    }
    // the denominators: sum over the four q lanes of a query
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
    const float inv = 1.0f / l_run;
    // lane (query x16, q) holds channels f = 4q..4q+3 of its query: 8 (16) contiguous bytes
    if (my_query < N)
        store_frag<T>(att + ((long)b * N + my_query) * (heads * 16) + h * 16 + q * 4,
                      frag_from_f32<T>(f32x4{o[0] * inv, o[1] * inv, o[2] * inv, o[3] * inv}));
}

template <class T>
hipError_t run_softmax(const void* qkv, void* att, int B, int N, int heads, hipStream_t stream) {
    const int q_blocks = (N + kSmQ - 1) / kSmQ;
    const long nblocks = (long)B * heads * q_blocks;
    if (nblocks <= 0 || nblocks > 0x7fffffffL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((softmax_attention_kernel<T>), dim3((unsigned)nblocks), dim3(256), 0, stream, (const T*)qkv, (T*)att,
                       N, heads, q_blocks);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_softmax_attention(int dt, const void* qkv, void* att, int B, int N, int heads, hipStream_t stream) {
    switch (dt) {
        case 0: return run_softmax<float>(qkv, att, B, N, heads, stream);
        case 1: return run_softmax<_Float16>(qkv, att, B, N, heads, stream);
        case 2: return run_softmax<__bf16>(qkv, att, B, N, heads, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace msla
