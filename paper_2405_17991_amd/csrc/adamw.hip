// AdamW step fed by the factored weight gradient.
//
// Sec. 3.1's reconstruction makes Listing 1's grad_weight a rank-structured
// array, dW[o, g*d + j] = T[o, g] * v[j], and the paper's training set-ups
// (Sec. 4.1, "Implementation details") hand it to AdamW.  This kernel forms each gradient element in
// registers from T and v and applies the optimiser update in the same pass, so
// the [O, D] gradient is never written to or read back from HBM: per element it
// moves the weight and the two moments in and out and nothing else.
//
// The kernel is a pure HBM stream (about 40 flops per 24 bytes); every weight
// and moment byte is touched once, hence the non-temporal loads and stores.
#include "common.h"
#include "kernels.h"

namespace velora {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ void adamw_element(float g, float& w, float& m, float& u, const AdamWScalars& a) {
    w *= a.decay;
    m = a.beta1 * m + a.one_minus_beta1 * g;
    u = a.beta2 * u + a.one_minus_beta2 * (g * g);
    const float denom = sqrtf(u) * a.inv_sqrt_bc2 + a.eps;
    w -= a.step_size * (m / denom);
}

// One thread per four consecutive elements of a row (d % 4 == 0, so the four
// share one T[o, g]).  IDX is uint32_t when O*D < 2^32, else uint64_t.
template <bool W_BF16, typename IDX>
__global__ __launch_bounds__(256) void adamw_factor_vec_kernel(const float* __restrict__ T, const float* __restrict__ v,
                                                               void* __restrict__ W, float* __restrict__ exp_avg,
                                                               float* __restrict__ exp_avg_sq, IDX n_vec, IDX D,
                                                               IDX M, IDX d, AdamWScalars a) {
    const IDX i = static_cast<IDX>(blockIdx.x) * 256u + threadIdx.x;
    if (i >= n_vec) return;
    const IDX e = i * 4u;
    const IDX o = e / D;
    const IDX c = e - o * D;
    const IDX gl = c / d;
    const IDX j = c - gl * d;
    const float tg = a.grad_scale * T[o * M + gl];
    const float4 vv = *reinterpret_cast<const float4*>(v + j);
    const float g[4] = {tg * vv.x, tg * vv.y, tg * vv.z, tg * vv.w};

    f32x4* mp = reinterpret_cast<f32x4*>(exp_avg + e);
    f32x4* up = reinterpret_cast<f32x4*>(exp_avg_sq + e);
    f32x4 m4 = __builtin_nontemporal_load(mp);
    f32x4 u4 = __builtin_nontemporal_load(up);
    float w[4];
    if constexpr (W_BF16) {
        const u32x2 q = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(static_cast<uint16_t*>(W) + e));
        w[0] = bf16_lo(q.x); w[1] = bf16_hi(q.x); w[2] = bf16_lo(q.y); w[3] = bf16_hi(q.y);
    } else {
        const f32x4 q = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(static_cast<float*>(W) + e));
        w[0] = q.x; w[1] = q.y; w[2] = q.z; w[3] = q.w;
    }
    float m[4] = {m4.x, m4.y, m4.z, m4.w};
    float u[4] = {u4.x, u4.y, u4.z, u4.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) adamw_element(g[k], w[k], m[k], u[k], a);
    m4 = {m[0], m[1], m[2], m[3]};
    u4 = {u[0], u[1], u[2], u[3]};
    __builtin_nontemporal_store(m4, mp);
    __builtin_nontemporal_store(u4, up);
    if constexpr (W_BF16) {
        const u32x2 q = {pack_bf16x2(w[0], w[1]), pack_bf16x2(w[2], w[3])};
        __builtin_nontemporal_store(q, reinterpret_cast<u32x2*>(static_cast<uint16_t*>(W) + e));
    } else {
        const f32x4 q = {w[0], w[1], w[2], w[3]};
        __builtin_nontemporal_store(q, reinterpret_cast<f32x4*>(static_cast<float*>(W) + e));
    }
}

// Any d, any alignment: one element per thread.
template <bool W_BF16>
__global__ __launch_bounds__(256) void adamw_factor_generic_kernel(const float* __restrict__ T,
                                                                   const float* __restrict__ v, void* __restrict__ W,
                                                                   float* __restrict__ exp_avg,
                                                                   float* __restrict__ exp_avg_sq, int64_t n, int64_t D,
                                                                   int64_t M, int64_t d, AdamWScalars a) {
    const int64_t e = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (e >= n) return;
    const int64_t o = e / D;
    const int64_t c = e - o * D;
    const int64_t gl = c / d;
    const int64_t j = c - gl * d;
    const float g = (a.grad_scale * T[o * M + gl]) * v[j];
    float w = W_BF16 ? bf16_to_f32(static_cast<uint16_t*>(W)[e]) : static_cast<float*>(W)[e];
    float m = exp_avg[e], u = exp_avg_sq[e];
    adamw_element(g, w, m, u, a);
    exp_avg[e] = m;
    exp_avg_sq[e] = u;
    if constexpr (W_BF16) static_cast<uint16_t*>(W)[e] = f32_to_bf16(w);
    else static_cast<float*>(W)[e] = w;
}

hipError_t launch_adamw_factor(const float* T, const float* v, void* W, bool w_bf16, float* exp_avg, float* exp_avg_sq,
                               int64_t O, int64_t D, int64_t M, bool vec_ok, const AdamWScalars& a, hipStream_t st) {
    const int64_t d = D / M;
    const int64_t n = O * D;
    if (vec_ok) {
        const int64_t n_vec = n / 4;
        const dim3 grid(static_cast<unsigned>(ceil_div(n_vec, 256))), block(256);
        if (n < (int64_t{1} << 32)) {
            const uint32_t nv = static_cast<uint32_t>(n_vec), D32 = static_cast<uint32_t>(D),
                           M32 = static_cast<uint32_t>(M), d32 = static_cast<uint32_t>(d);
            if (w_bf16)
                hipLaunchKernelGGL((adamw_factor_vec_kernel<true, uint32_t>), grid, block, 0, st, T, v, W, exp_avg,
                                   exp_avg_sq, nv, D32, M32, d32, a);
            else
                hipLaunchKernelGGL((adamw_factor_vec_kernel<false, uint32_t>), grid, block, 0, st, T, v, W, exp_avg,
                                   exp_avg_sq, nv, D32, M32, d32, a);
        } else {
            const uint64_t nv = static_cast<uint64_t>(n_vec), D64 = static_cast<uint64_t>(D),
                           M64 = static_cast<uint64_t>(M), d64 = static_cast<uint64_t>(d);
            if (w_bf16)
                hipLaunchKernelGGL((adamw_factor_vec_kernel<true, uint64_t>), grid, block, 0, st, T, v, W, exp_avg,
                                   exp_avg_sq, nv, D64, M64, d64, a);
            else
                hipLaunchKernelGGL((adamw_factor_vec_kernel<false, uint64_t>), grid, block, 0, st, T, v, W, exp_avg,
                                   exp_avg_sq, nv, D64, M64, d64, a);
        }
    } else {
        const dim3 grid(static_cast<unsigned>(ceil_div(n, 256))), block(256);
        if (w_bf16)
            hipLaunchKernelGGL((adamw_factor_generic_kernel<true>), grid, block, 0, st, T, v, W, exp_avg, exp_avg_sq, n,
                               D, M, d, a);
        else
            hipLaunchKernelGGL((adamw_factor_generic_kernel<false>), grid, block, 0, st, T, v, W, exp_avg, exp_avg_sq,
                               n, D, M, d, a);
    }
    return hipGetLastError();
}

}  // namespace velora
