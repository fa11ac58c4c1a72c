// Device-side building blocks shared by the gfx950 kernels: storage-type traits,
// 8/16-byte vector moves, and the MFMA fragment conventions used everywhere.
//
// Fragment convention (all 16x16 MFMAs, wave64).  Lane l is (x, q) with
// x = l % 16 and q = l / 16.
//   "row operand"  A (16 x K):  lane (x, q) holds A[x][K-slots owned by q]
//   "col operand"  B (K x 16):  lane (x, q) holds B[K-slots owned by q][x]
//   result         D (16 x 16): lane (x, q) holds D[4q + r][x], r = 0..3
// A contraction index only has to be paired consistently between A and B, so
// for a 16-wide contraction the lane (x, q) always owns indices 4q..4q+3
// ("Frag"), whatever instruction the storage type maps to.
#pragma once
#include <hip/hip_runtime.h>
#include <type_traits>
#include <stdint.h>

namespace msla {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kHeadDim = 16;            // d of Section 3.1; the only head size built
constexpr int kStateSize = 16 * 17;     // d x (d+1) floats of the Eq. (3) state

// Compile-time loop: f(std::integral_constant<int, i>) for i in [B, E).  Unlike "#pragma unroll" it
// cannot be declined by the optimiser, so register arrays indexed by i never turn into scratch.
template <int B, int E, class F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (B < E) {
        f(std::integral_constant<int, B>{});
        static_for<B + 1, E>(f);
    }
}

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }

template <class T> struct Traits;

// ---------------------------------------------------------------- fp16
template <> struct Traits<_Float16> {
    typedef _Float16 elem;
    typedef f16x4 Frag;                 // 4 contraction slots
    typedef f16x8 Vec;                  // 16 bytes = 8 contraction slots
    static constexpr int kVec = 8;
    static constexpr bool kSplit = true;    // state fragments carry a hi and a lo half
    static constexpr bool kHiLo = false;    // 11 significant bits: in-register operands are rounded once
    static __device__ __forceinline__ float to_f32(elem v) { return (float)v; }
    static __device__ __forceinline__ elem from_f32(float v) { return (elem)v; }
    static __device__ __forceinline__ f32x4 mma16(f32x4 c, Frag a, Frag b) {
        return __builtin_amdgcn_mfma_f32_16x16x16f16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ f32x4 mma_vec(f32x4 c, Vec a, Vec b) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
    }
};

// ---------------------------------------------------------------- bf16
template <> struct Traits<__bf16> {
    typedef __bf16 elem;
    typedef bf16x4 Frag;
    typedef bf16x8 Vec;
    static constexpr int kVec = 8;
    static constexpr bool kSplit = true;
    // 8 significant bits are too few for operands that only live in registers or LDS (depthwise
    // sums, aggregated K/V, attention rows): those are fed to the matrix cores as hi + lo pairs.
    static constexpr bool kHiLo = true;
    static __device__ __forceinline__ float to_f32(elem v) { return (float)v; }
    static __device__ __forceinline__ elem from_f32(float v) { return (elem)v; }
    static __device__ __forceinline__ f32x4 mma16(f32x4 c, Frag a, Frag b) {
        return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(i16x4, a),
                                                         __builtin_bit_cast(i16x4, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ f32x4 mma_vec(f32x4 c, Vec a, Vec b) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
};

// ---------------------------------------------------------------- fp32
// True fp32 matrix instruction (16x16x4), four per 16-wide contraction.  The
// hardware contracts over q in each step; step r pairs a[r] with b[r], i.e.
// contraction index 4q + r, which is exactly the Frag convention.
template <> struct Traits<float> {
    typedef float elem;
    typedef f32x4 Frag;
    typedef f32x4 Vec;                  // 16 bytes = 4 contraction slots
    static constexpr int kVec = 4;
    static constexpr bool kSplit = false;
    static constexpr bool kHiLo = false;
    static __device__ __forceinline__ float to_f32(elem v) { return v; }
    static __device__ __forceinline__ elem from_f32(float v) { return v; }
    static __device__ __forceinline__ f32x4 mma16(f32x4 c, Frag a, Frag b) {
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[0], b[0], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[1], b[1], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[2], b[2], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[3], b[3], c, 0, 0, 0);
        return c;
    }
    static __device__ __forceinline__ f32x4 mma_vec(f32x4 c, Vec a, Vec b) { return mma16(c, a, b); }
};

template <class T>
__device__ __forceinline__ typename Traits<T>::Frag frag_from_f32(f32x4 v) {
    typename Traits<T>::Frag f;
    f[0] = Traits<T>::from_f32(v[0]);
    f[1] = Traits<T>::from_f32(v[1]);
    f[2] = Traits<T>::from_f32(v[2]);
    f[3] = Traits<T>::from_f32(v[3]);
    return f;
}

template <class T>
__device__ __forceinline__ f32x4 frag_to_f32(typename Traits<T>::Frag f) {
    f32x4 v;
    v[0] = Traits<T>::to_f32(f[0]);
    v[1] = Traits<T>::to_f32(f[1]);
    v[2] = Traits<T>::to_f32(f[2]);
    v[3] = Traits<T>::to_f32(f[3]);
    return v;
}

// v = hi + lo with hi = round(v) and lo = round(v - hi), both in the storage type.
template <class T>
__device__ __forceinline__ void frag_split(f32x4 v, typename Traits<T>::Frag& hi, typename Traits<T>::Frag& lo) {
    hi = frag_from_f32<T>(v);
    const f32x4 h = frag_to_f32<T>(hi);
    lo = frag_from_f32<T>(f32x4{v[0] - h[0], v[1] - h[1], v[2] - h[2], v[3] - h[3]});
}

template <class T>
__device__ __forceinline__ typename Traits<T>::Frag frag_zero() {
    typename Traits<T>::Frag f;
    f[0] = f[1] = f[2] = f[3] = Traits<T>::from_f32(0.0f);
    return f;
}

// Elementwise max(v, 0) on a fragment (Eq. (2): the rectifier on Q and K).
template <class T>
__device__ __forceinline__ typename Traits<T>::Frag frag_relu(typename Traits<T>::Frag f) {
    const typename Traits<T>::elem z = Traits<T>::from_f32(0.0f);
    f[0] = f[0] > z ? f[0] : z;
    f[1] = f[1] > z ? f[1] : z;
    f[2] = f[2] > z ? f[2] : z;
    f[3] = f[3] > z ? f[3] : z;
    return f;
}

// The same rectifier as integer maxima on the bit patterns (negative values and -0 have the sign
// bit set, so they compare below +0 as integers): one instruction per pair of 16-bit values,
// no canonicalisation of the input.  NaNs with a clear sign bit pass through.
// (Whole vectors are bit-cast here: __builtin_bit_cast applied to a single vector ELEMENT reads
// element 0 with this compiler.)
template <class T>
__device__ __forceinline__ typename Traits<T>::Frag frag_relu_bits(typename Traits<T>::Frag f) {
    if constexpr (sizeof(T) == 2) {
        typedef short i16x4v __attribute__((ext_vector_type(4)));
        const i16x4v zero = {0, 0, 0, 0};
        return __builtin_bit_cast(typename Traits<T>::Frag,
                                  __builtin_elementwise_max(__builtin_bit_cast(i16x4v, f), zero));
    } else {
        typedef int i32x4 __attribute__((ext_vector_type(4)));
        const i32x4 zero = {0, 0, 0, 0};
        return __builtin_bit_cast(typename Traits<T>::Frag,
                                  __builtin_elementwise_max(__builtin_bit_cast(i32x4, f), zero));
    }
}

__device__ __forceinline__ f32x4 relu_bits_f32(f32x4 v) {
    typedef int i32x4 __attribute__((ext_vector_type(4)));
    const i32x4 zero = {0, 0, 0, 0};
    return __builtin_bit_cast(f32x4, __builtin_elementwise_max(__builtin_bit_cast(i32x4, v), zero));
}

// 4 consecutive elements (one Frag) to / from memory.  8 bytes for the 16-bit
// types, 16 bytes for fp32; the address must be aligned to 8 bytes (LDS tiles
// are padded to 8-byte pixel strides), so fp32 moves as two 8-byte halves.
template <class T>
__device__ __forceinline__ typename Traits<T>::Frag load_frag(const void* p) {
    if constexpr (sizeof(T) == 2) {
        return __builtin_bit_cast(typename Traits<T>::Frag, *(const u32x2*)p);
    } else {
        const u32x2 lo = ((const u32x2*)p)[0], hi = ((const u32x2*)p)[1];
        u32x4 v = {lo[0], lo[1], hi[0], hi[1]};
        return __builtin_bit_cast(typename Traits<T>::Frag, v);
    }
}

template <class T>
__device__ __forceinline__ void store_frag(void* p, typename Traits<T>::Frag f) {
    if constexpr (sizeof(T) == 2) {
        *(u32x2*)p = __builtin_bit_cast(u32x2, f);
    } else {
        const u32x4 v = __builtin_bit_cast(u32x4, f);
        ((u32x2*)p)[0] = u32x2{v[0], v[1]};
        ((u32x2*)p)[1] = u32x2{v[2], v[3]};
    }
}

// Raw buffer resources: loads and stores through one are range-checked by the hardware against
// the byte count (a load out of range returns zero, a store out of range is dropped), which
// replaces per-lane branches at ragged ends.  Offsets are 32-bit, so a resource spans at most
// 2^31 - 1 bytes from its base; kOobOffset lies beyond any such span.
typedef __amdgpu_buffer_rsrc_t BufRsrc;
constexpr unsigned kOobOffset = 0x80000000u;
__device__ __forceinline__ BufRsrc make_rsrc(const void* base, long bytes) {
    const int n = bytes > 0x7fffffffL ? 0x7fffffff : (bytes < 0 ? 0 : (int)bytes);
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, n, 0x00020000);
}
// ... for a span known to be small (a tile): no clamping, so nothing but the descriptor words
__device__ __forceinline__ BufRsrc make_rsrc_small(const void* base, unsigned bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ u32x4 buf_load16(BufRsrc r, unsigned voffset, int soffset) {
    return __builtin_amdgcn_raw_buffer_load_b128(r, (int)voffset, soffset, 0);
}
__device__ __forceinline__ void buf_store16(BufRsrc r, unsigned voffset, u32x4 v) {
    __builtin_amdgcn_raw_buffer_store_b128(v, r, (int)voffset, 0, 0);
}
// ... with a wave-uniform byte offset (below 2^31) on top.  It is added to the lane's offset rather
// than handed to the instruction's scalar-offset field, for two reasons.  The range check covers the
// lane's offset only, so a row the scalar offset pushes past the end of the resource would still be
// written.  And the compiler leaves no wait state between a 16-byte store with a scalar offset and
// a vector instruction that overwrites the store's data registers, where this chip needs one: with
// the data registers reused right behind the store, the first word of some lanes came out wrong in
// about one launch in twenty.
__device__ __forceinline__ void buf_store16_at(BufRsrc r, unsigned voffset, unsigned soffset, u32x4 v) {
    __builtin_amdgcn_raw_buffer_store_b128(v, r, (int)(voffset + soffset), 0, 0);
}
// The same store written through to memory (the sc1 cache-policy bit): for output that no later
// kernel of the module reads.  Such lines are not left dirty in L2, where they would displace the
// maps the next call's kernels re-read and wait for the write-back at the end of the kernel; it
// measures slightly better than the non-temporal hint and clearly better than a plain store.
__device__ __forceinline__ void buf_store16_stream(BufRsrc r, unsigned voffset, u32x4 v) {
    __builtin_amdgcn_raw_buffer_store_b128(v, r, (int)voffset, 0, 16);
}
__device__ __forceinline__ u32x2 buf_load8(BufRsrc r, unsigned voffset) {
    return __builtin_amdgcn_raw_buffer_load_b64(r, (int)voffset, 0, 0);
}
__device__ __forceinline__ void buf_store8(BufRsrc r, unsigned voffset, u32x2 v) {
    __builtin_amdgcn_raw_buffer_store_b64(v, r, (int)voffset, 0, 0);
}


// Workgroup id -> logical id so that consecutive logical ids run on the same
// XCD.  The hardware deals workgroups round-robin over the 8 XCDs (each with
// its own L2); neighbours in the logical order share cache lines, so they
// should share an L2.  Identity when the grid is not a multiple of 8.
__device__ __forceinline__ unsigned xcd_remap(unsigned bid, unsigned nblocks) {
    constexpr unsigned kXcd = 8;
    if (nblocks % kXcd != 0) return bid;
    return (bid % kXcd) * (nblocks / kXcd) + bid / kXcd;
}

}  // namespace msla
