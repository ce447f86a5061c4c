// Producer-side fusion for the attention projections of an LLaMA block (the
// paper compresses the value projection's input, Sec. 4): that input is
// X = RMSNorm(H) = H / sqrt(mean(H^2) + eps) * gamma, a row-wise kernel that has
// to stream H in and X out anyway.  This one also forms, from the values it
// stores, S = compress(group(X), v) of Sec. 3.1, so X is never re-read for
// compression.  S uses the lane layout and summation order of
// compress_vec_kernel and equals velora_compress(X, v) bit for bit.
#include "common.h"
#include "kernels.h"

#include <type_traits>

namespace velora {

typedef uint32_t u32x4_rn __attribute__((ext_vector_type(4)));

constexpr int kRmsMaxVecPerRow = 1024;   // 16 KB of LDS per wave: D <= 8192 (bf16) or 4096 (f32)

// One wave per token row; the row waits in LDS between the two passes.  P lanes
// share a sub-token (P = d / kPerVec, a power of two <= 64), as in compress.
template <typename E, int P>
__global__ __launch_bounds__(256) void rmsnorm_compress_row_kernel(const uint4* __restrict__ H,
                                                                  const float* __restrict__ gamma,
                                                                  const float* __restrict__ v,
                                                                  uint4* __restrict__ X,
                                                                  typename E::type* __restrict__ S, int64_t N,
                                                                  int vec_per_row, int M, float inv_D, float eps) {
    constexpr int kV = E::kPerVec;
    extern __shared__ uint4 row_lds[];               // [4 waves][vec_per_row]
    const int lane = threadIdx.x & (kWave - 1);
    const int w = threadIdx.x / kWave;
    uint4* my = row_lds + w * vec_per_row;
    const int p = lane % P;
    float vf[kV];
#pragma unroll
    for (int e = 0; e < kV; ++e) vf[e] = v[p * kV + e];

    const int64_t n_waves = static_cast<int64_t>(gridDim.x) * 4;
    for (int64_t row = static_cast<int64_t>(blockIdx.x) * 4 + w; row < N; row += n_waves) {
        const uint4* src = H + row * vec_per_row;
        float ss = 0.f;
        for (int i0 = 0; i0 < vec_per_row; i0 += 4 * kWave) {      // four loads in flight per lane
            uint4 q[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = i0 + u * kWave + lane;
                q[u] = i < vec_per_row ? load_stream16(&src[i]) : make_uint4(0u, 0u, 0u, 0u);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = i0 + u * kWave + lane;
                if (i < vec_per_row) my[i] = q[u];
                float f[kV];
                E::unpack(q[u], f);
#pragma unroll
                for (int e = 0; e < kV; ++e) ss = fmaf(f[e], f[e], ss);
            }
        }
        ss = group_sum<kWave>(ss);
        const float rinv = 1.f / sqrtf(ss * inv_D + eps);
        // the wave re-reads only what its own lanes wrote: no barrier needed
        for (int i = lane; i < vec_per_row; i += kWave) {
            float f[kV], x[kV];
            E::unpack(my[i], f);
            const float4 g0 = *reinterpret_cast<const float4*>(gamma + static_cast<int64_t>(i) * kV);
            x[0] = f[0] * rinv * g0.x; x[1] = f[1] * rinv * g0.y; x[2] = f[2] * rinv * g0.z; x[3] = f[3] * rinv * g0.w;
            if constexpr (kV == 8) {
                const float4 g1 = *reinterpret_cast<const float4*>(gamma + static_cast<int64_t>(i) * kV + 4);
                x[4] = f[4] * rinv * g1.x; x[5] = f[5] * rinv * g1.y; x[6] = f[6] * rinv * g1.z; x[7] = f[7] * rinv * g1.w;
            }
            uint4 q;
            if constexpr (kV == 4) {
                q = make_uint4(__float_as_uint(x[0]), __float_as_uint(x[1]), __float_as_uint(x[2]), __float_as_uint(x[3]));
            } else {
                q = make_uint4(pack_bf16x2(x[0], x[1]), pack_bf16x2(x[2], x[3]), pack_bf16x2(x[4], x[5]),
                               pack_bf16x2(x[6], x[7]));
            }
            const u32x4_rn out = {q.x, q.y, q.z, q.w};
            __builtin_nontemporal_store(out, reinterpret_cast<u32x4_rn*>(&X[row * vec_per_row + i]));
            float s[kV];
            E::unpack(q, s);                                       // the stored values
            float acc = 0.f;
#pragma unroll
            for (int e = 0; e < kV; ++e) acc = fmaf(s[e], vf[e], acc);
            acc = group_sum<P>(acc);
            if (p == 0) E::store(S, row * M + i / P, acc);
        }
    }
}

// The same with the row kept in registers between the two passes: NV 16-byte vectors per lane (a row is
// exactly 64 * NV vectors), lane l holding vectors l, l + 64, ...  The lane's slice of gamma stays in
// registers for the whole kernel (it would otherwise be re-read, at twice the row's bytes, for every row), and
// LDS is not used at all.  64 % P == 0, so every vector of a lane has the same position p in its sub-token.
template <typename E, int P, int NV>
__global__ __launch_bounds__(256) void rmsnorm_compress_reg_kernel(const uint4* __restrict__ H,
                                                                  const float* __restrict__ gamma,
                                                                  const float* __restrict__ v,
                                                                  uint4* __restrict__ X,
                                                                  typename E::type* __restrict__ S, int64_t N, int M,
                                                                  float inv_D, float eps) {
    constexpr int kV = E::kPerVec;
    constexpr int kVecPerRow = kWave * NV;
    const int lane = threadIdx.x & (kWave - 1);
    const int w = threadIdx.x / kWave;
    const int p = lane % P;
    float vf[kV], gf[NV][kV];
#pragma unroll
    for (int e = 0; e < kV; ++e) vf[e] = v[p * kV + e];
#pragma unroll
    for (int j = 0; j < NV; ++j)
#pragma unroll
        for (int e = 0; e < kV; ++e) gf[j][e] = gamma[(j * kWave + lane) * kV + e];

    const int64_t n_waves = static_cast<int64_t>(gridDim.x) * 4;
    for (int64_t row = static_cast<int64_t>(blockIdx.x) * 4 + w; row < N; row += n_waves) {
        const uint4* src = H + row * kVecPerRow;
        uint4 q[NV];
#pragma unroll
        for (int j = 0; j < NV; ++j) q[j] = load_stream16(&src[j * kWave + lane]);
        float ss = 0.f;
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            float f[kV];
            E::unpack(q[j], f);
#pragma unroll
            for (int e = 0; e < kV; ++e) ss = fmaf(f[e], f[e], ss);
        }
        ss = group_sum<kWave>(ss);
        const float rinv = 1.f / sqrtf(ss * inv_D + eps);
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            float f[kV], x[kV];
            E::unpack(q[j], f);
#pragma unroll
            for (int e = 0; e < kV; ++e) x[e] = f[e] * rinv * gf[j][e];
            uint4 o;
            if constexpr (kV == 4) {
                o = make_uint4(__float_as_uint(x[0]), __float_as_uint(x[1]), __float_as_uint(x[2]), __float_as_uint(x[3]));
            } else {
                o = make_uint4(pack_bf16x2(x[0], x[1]), pack_bf16x2(x[2], x[3]), pack_bf16x2(x[4], x[5]),
                               pack_bf16x2(x[6], x[7]));
            }
            const u32x4_rn out = {o.x, o.y, o.z, o.w};
            __builtin_nontemporal_store(out, reinterpret_cast<u32x4_rn*>(&X[row * kVecPerRow + j * kWave + lane]));
            float sv[kV];
            E::unpack(o, sv);                                      // the stored values
            float acc = 0.f;
#pragma unroll
            for (int e = 0; e < kV; ++e) acc = fmaf(sv[e], vf[e], acc);
            acc = group_sum<P>(acc);
            if (p == 0) E::store(S, row * M + (j * kWave + lane) / P, acc);
        }
    }
}

// Any shape: one block per row, X only; compress follows as its own launch.
template <typename E>
__global__ __launch_bounds__(256) void rmsnorm_generic_kernel(const typename E::type* __restrict__ H,
                                                             const float* __restrict__ gamma,
                                                             typename E::type* __restrict__ X, int64_t N, int64_t D,
                                                             float inv_D, float eps) {
    __shared__ float red[256];
    for (int64_t row = blockIdx.x; row < N; row += gridDim.x) {
        float ss = 0.f;
        for (int64_t j = threadIdx.x; j < D; j += 256) {
            const float f = E::load(H, row * D + j);
            ss = fmaf(f, f, ss);
        }
        red[threadIdx.x] = ss;
        __syncthreads();
        for (int s = 128; s > 0; s >>= 1) {
            if (threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
            __syncthreads();
        }
        const float rinv = 1.f / sqrtf(red[0] * inv_D + eps);
        __syncthreads();
        for (int64_t j = threadIdx.x; j < D; j += 256) E::store(X, row * D + j, E::load(H, row * D + j) * rinv * gamma[j]);
    }
}

namespace {

template <typename E, int P, int NV>
hipError_t launch_reg(const void* H, const float* gamma, const float* v, void* X, void* S, int64_t N, int64_t D,
                      int64_t M, float eps, const LaunchCfg& cfg, hipStream_t st) {
    int64_t grid = ceil_div(N, 4);
    if (grid > cfg.max_blocks) grid = cfg.max_blocks;
    hipLaunchKernelGGL((rmsnorm_compress_reg_kernel<E, P, NV>), dim3(static_cast<unsigned>(grid)), dim3(256), 0, st,
                       static_cast<const uint4*>(H), gamma, v, static_cast<uint4*>(X),
                       static_cast<typename E::type*>(S), N, static_cast<int>(M),
                       static_cast<float>(1.0 / static_cast<double>(D)), eps);
    return hipGetLastError();
}

template <typename E, int P>
hipError_t launch_row(const void* H, const float* gamma, const float* v, void* X, void* S, int64_t N, int64_t D,
                      int64_t M, float eps, const LaunchCfg& cfg, hipStream_t st) {
    const int vec_per_row = static_cast<int>(D / E::kPerVec);
    // rows of exactly 64, 128, 256, 512 (or 1024, bf16) vectors stay in registers
    switch (vec_per_row) {
        case 64:  return launch_reg<E, P, 1>(H, gamma, v, X, S, N, D, M, eps, cfg, st);
        case 128: return launch_reg<E, P, 2>(H, gamma, v, X, S, N, D, M, eps, cfg, st);
        case 256: return launch_reg<E, P, 4>(H, gamma, v, X, S, N, D, M, eps, cfg, st);
        case 512: return launch_reg<E, P, 8>(H, gamma, v, X, S, N, D, M, eps, cfg, st);
        default:  break;
    }
    const size_t lds = static_cast<size_t>(4) * vec_per_row * sizeof(uint4);
    int64_t grid = ceil_div(N, 4);
    if (grid > cfg.max_blocks) grid = cfg.max_blocks;
    hipLaunchKernelGGL((rmsnorm_compress_row_kernel<E, P>), dim3(static_cast<unsigned>(grid)), dim3(256), lds, st,
                       static_cast<const uint4*>(H), gamma, v, static_cast<uint4*>(X),
                       static_cast<typename E::type*>(S), N, vec_per_row, static_cast<int>(M),
                       static_cast<float>(1.0 / static_cast<double>(D)), eps);
    return hipGetLastError();
}

template <typename E>
hipError_t rmsnorm_any(const void* H, const float* gamma, const float* v, void* X, void* S, int64_t N, int64_t D,
                       int64_t M, float eps, bool vec_ok, const LaunchCfg& cfg, hipStream_t st) {
    const int64_t d = D / M;
    if (vec_ok && d % E::kPerVec == 0 && D / E::kPerVec <= kRmsMaxVecPerRow && M <= INT32_MAX) {
        switch (static_cast<int>(d / E::kPerVec)) {
            case 1:  return launch_row<E, 1>(H, gamma, v, X, S, N, D, M, eps, cfg, st);
            case 2:  return launch_row<E, 2>(H, gamma, v, X, S, N, D, M, eps, cfg, st);
            case 4:  return launch_row<E, 4>(H, gamma, v, X, S, N, D, M, eps, cfg, st);
            case 8:  return launch_row<E, 8>(H, gamma, v, X, S, N, D, M, eps, cfg, st);
            case 16: return launch_row<E, 16>(H, gamma, v, X, S, N, D, M, eps, cfg, st);
            case 32: return launch_row<E, 32>(H, gamma, v, X, S, N, D, M, eps, cfg, st);
            case 64: return launch_row<E, 64>(H, gamma, v, X, S, N, D, M, eps, cfg, st);
            default: break;
        }
    }
    int64_t grid = N < cfg.max_blocks ? N : cfg.max_blocks;
    hipLaunchKernelGGL((rmsnorm_generic_kernel<E>), dim3(static_cast<unsigned>(grid)), dim3(256), 0, st,
                       static_cast<const typename E::type*>(H), gamma, static_cast<typename E::type*>(X), N, D,
                       static_cast<float>(1.0 / static_cast<double>(D)), eps);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_compress(X, v, S, N * M, d, std::is_same<E, Bf16Elem>::value, vec_ok, cfg, st);
}

}  // namespace

hipError_t launch_rmsnorm_compress(const void* H, const float* gamma, const float* v, void* X, void* S, int64_t N,
                                   int64_t D, int64_t M, float eps, bool is_bf16, bool vec_ok, const LaunchCfg& cfg,
                                   hipStream_t st) {
    return is_bf16 ? rmsnorm_any<Bf16Elem>(H, gamma, v, X, S, N, D, M, eps, vec_ok, cfg, st)
                   : rmsnorm_any<F32Elem>(H, gamma, v, X, S, N, D, M, eps, vec_ok, cfg, st);
}

}  // namespace velora
