// Device-side helpers shared by libvelora's gfx950 kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace velora {

constexpr int kWave = 64;

// ---- bfloat16 <-> float32 (bf16 = upper half of an IEEE binary32) ----------
__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xFFFF0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(static_cast<uint32_t>(b) << 16); }

// float32 -> bfloat16, round-to-nearest-even, NaN stays a quiet NaN: gfx950's
// v_cvt_pk_bf16_f32 (one instruction per pair) through the compiler's native
// __bf16 conversion.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    return __builtin_bit_cast(uint16_t, static_cast<__bf16>(f));
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t));
}

// 16-byte load with the streaming (non-temporal) hint: the data is read once.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));   // one MFMA A or B operand (eight k-consecutive bf16)
typedef float f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream16(const uint4* p) {
    const u32x4 q = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    return make_uint4(q.x, q.y, q.z, q.w);
}

// ---- element traits for the two storage dtypes ------------------------------
struct F32Elem {
    using type = float;
    using vec = uint4;
    static constexpr int kPerVec = 4;  // elements in one 16-byte vector
    __device__ static __forceinline__ vec load_stream(const vec* p) { return load_stream16(p); }
    __device__ static __forceinline__ vec zero_vec() { return make_uint4(0u, 0u, 0u, 0u); }
    __device__ static __forceinline__ float load(const void* p, int64_t i) { return static_cast<const float*>(p)[i]; }
    __device__ static __forceinline__ void store(void* p, int64_t i, float x) { static_cast<float*>(p)[i] = x; }
    __device__ static __forceinline__ void unpack(const uint4& q, float* f) {
        f[0] = __uint_as_float(q.x); f[1] = __uint_as_float(q.y);
        f[2] = __uint_as_float(q.z); f[3] = __uint_as_float(q.w);
    }
};
struct Bf16Elem {
    using type = uint16_t;
    using vec = uint4;
    static constexpr int kPerVec = 8;
    __device__ static __forceinline__ vec load_stream(const vec* p) { return load_stream16(p); }
    __device__ static __forceinline__ vec zero_vec() { return make_uint4(0u, 0u, 0u, 0u); }
    __device__ static __forceinline__ float load(const void* p, int64_t i) { return bf16_to_f32(static_cast<const uint16_t*>(p)[i]); }
    __device__ static __forceinline__ void store(void* p, int64_t i, float x) { static_cast<uint16_t*>(p)[i] = f32_to_bf16(x); }
    __device__ static __forceinline__ void unpack(const uint4& q, float* f) {
        f[0] = bf16_lo(q.x); f[1] = bf16_hi(q.x); f[2] = bf16_lo(q.y); f[3] = bf16_hi(q.y);
        f[4] = bf16_lo(q.z); f[5] = bf16_hi(q.z); f[6] = bf16_lo(q.w); f[7] = bf16_hi(q.w);
    }
};

// bfloat16 in 8-byte vectors of four: for sub-token sizes that are a multiple of 4 but not of 8
struct Bf16Half {
    using type = uint16_t;
    using vec = uint2;
    static constexpr int kPerVec = 4;
    __device__ static __forceinline__ vec load_stream(const vec* p) {
        const u32x2 q = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p));
        return make_uint2(q.x, q.y);
    }
    __device__ static __forceinline__ vec zero_vec() { return make_uint2(0u, 0u); }
    __device__ static __forceinline__ void store(void* p, int64_t i, float x) { static_cast<uint16_t*>(p)[i] = f32_to_bf16(x); }
    __device__ static __forceinline__ void unpack(const uint2& q, float* f) {
        f[0] = bf16_lo(q.x); f[1] = bf16_hi(q.x); f[2] = bf16_lo(q.y); f[3] = bf16_hi(q.y);
    }
};

// ---- cross-lane sums over aligned groups of P lanes (P a power of two) -------
// Steps inside a row of 16 lanes use DPP (no LDS traffic); steps across rows
// use the LDS crossbar.  After the call every lane of a group holds the sum.
template <int kCtrl>
__device__ __forceinline__ float dpp_move(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), kCtrl, 0xF, 0xF, true));
}

template <int P>
__device__ __forceinline__ float group_sum(float x) {
    static_assert(P >= 1 && P <= 64 && (P & (P - 1)) == 0, "P must be a power of two <= 64");
    if constexpr (P >= 2) x += dpp_move<0xB1>(x);    // quad_perm [1,0,3,2]: lane ^ 1
    if constexpr (P >= 4) x += dpp_move<0x4E>(x);    // quad_perm [2,3,0,1]: lane ^ 2
    if constexpr (P >= 8) x += dpp_move<0x141>(x);   // row_half_mirror: pairs the two quads of 8 lanes
    if constexpr (P >= 16) x += dpp_move<0x140>(x);  // row_mirror: pairs the two halves of 16 lanes
    if constexpr (P >= 32) x += __shfl_xor(x, 16, 64);
    if constexpr (P >= 64) x += __shfl_xor(x, 32, 64);
    return x;
}

// Runtime-width variant for the generic kernels.
__device__ __forceinline__ float group_sum_rt(float x, int P) {
    for (int m = 1; m < P; m <<= 1) x += __shfl_xor(x, m, 64);
    return x;
}

__host__ __device__ constexpr int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Eight rows of an 8 x (2*NDW) block of 16-bit values, one row per register group, and its in-register
// transpose: the eight k-consecutive values of column c as one MFMA operand.
template <int NDW>
struct RawRow {
    uint32_t w[NDW];
};


// Column c of an 8-row block -> one MFMA fragment (rows 2i, 2i+1 share dword i).
template <int NDW>
__device__ __forceinline__ bf16x8 column_fragment(const RawRow<NDW> (&rows)[8], int c) {
    uint32_t f[4];
    const int dw = c >> 1;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t a = rows[2 * i].w[dw], b = rows[2 * i + 1].w[dw];
        // v_perm_b32: selector bytes 0-3 pick from the second operand, 4-7 from the first
        f[i] = (c & 1) ? __builtin_amdgcn_perm(b, a, 0x07060302u) : __builtin_amdgcn_perm(b, a, 0x05040100u);
    }
    uint4 q = make_uint4(f[0], f[1], f[2], f[3]);
    return __builtin_bit_cast(bf16x8, q);
}

}  // namespace velora
