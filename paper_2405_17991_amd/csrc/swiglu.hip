// Producer-side fusion for the layer the paper compresses first, the MLP down
// projection of an LLaMA block (Sec. 4): its input X = silu(gate) * up is an
// elementwise product that some kernel has to stream out anyway, so this one
// writes X and, from the very values it stores, the compressed activations
// S = compress(group(X), v) of Sec. 3.1 in the same pass.  X is then never
// re-read for compression: the extra pass of Listing 1's forward disappears.
//
// S is computed from the stored (rounded) X with the lane layout and summation
// order of compress_vec_kernel, so it equals velora_compress(X, v) bit for bit.
#include "common.h"
#include "kernels.h"

#include <type_traits>

namespace velora {

typedef uint32_t u32x4_nt __attribute__((ext_vector_type(4)));

// v_exp_f32 and v_rcp_f32 (about 1 ulp each): far inside what the stored dtype resolves, and the kernel
// stays bound by HBM rather than by a full-precision division per element
__device__ __forceinline__ float silu_mul(float g, float u) {
    return g * __builtin_amdgcn_rcpf(1.f + __expf(-g)) * u;
}

// Lane mapping as in compress_vec_kernel: P lanes per sub-token, L vectors per
// lane, U sub-tokens per lane group and trip.
template <typename E, int P, int L, int U>
__global__ __launch_bounds__(256) void swiglu_compress_vec_kernel(const uint4* __restrict__ gate,
                                                                 const uint4* __restrict__ up,
                                                                 const float* __restrict__ v,
                                                                 uint4* __restrict__ X,
                                                                 typename E::type* __restrict__ S, int64_t n_sub,
                                                                 int vps) {
    constexpr int kV = E::kPerVec;
    constexpr int SEG = kWave / P;
    const int lane = threadIdx.x & (kWave - 1);
    const int p = lane % P;
    const int seg = lane / P;
    const int64_t wave = (static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x) / kWave;
    const int64_t n_waves = static_cast<int64_t>(gridDim.x) * blockDim.x / kWave;
    const int64_t n_chunks = ceil_div(n_sub, static_cast<int64_t>(SEG) * U);

    float vf[L][kV];
#pragma unroll
    for (int l = 0; l < L; ++l)
#pragma unroll
        for (int e = 0; e < kV; ++e) vf[l][e] = (l * P + p) < vps ? v[(l * P + p) * kV + e] : 0.f;

    for (int64_t chunk = wave; chunk < n_chunks; chunk += n_waves) {
        const int64_t k0 = chunk * (SEG * U) + static_cast<int64_t>(seg) * U;
        uint4 qg[U][L], qu[U][L];
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int l = 0; l < L; ++l) {
                qg[u][l] = make_uint4(0u, 0u, 0u, 0u);
                qu[u][l] = make_uint4(0u, 0u, 0u, 0u);
                if (k0 + u < n_sub && l * P + p < vps) {
                    const int64_t i = (k0 + u) * vps + l * P + p;
                    qg[u][l] = load_stream16(&gate[i]);
                    qu[u][l] = load_stream16(&up[i]);
                }
            }
        float sum[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float acc = 0.f;
#pragma unroll
            for (int l = 0; l < L; ++l) {
                float fg[kV], fu[kV], x[kV];
                E::unpack(qg[u][l], fg);
                E::unpack(qu[u][l], fu);
#pragma unroll
                for (int e = 0; e < kV; ++e) x[e] = silu_mul(fg[e], fu[e]);
                // round to the storage dtype, store, and continue with the stored values
                uint4 q;
                if constexpr (kV == 4) {
                    q = make_uint4(__float_as_uint(x[0]), __float_as_uint(x[1]), __float_as_uint(x[2]),
                                   __float_as_uint(x[3]));
                } else {
                    q = make_uint4(pack_bf16x2(x[0], x[1]), pack_bf16x2(x[2], x[3]), pack_bf16x2(x[4], x[5]),
                                   pack_bf16x2(x[6], x[7]));
                }
                if (k0 + u < n_sub && l * P + p < vps) {
                    const u32x4_nt out = {q.x, q.y, q.z, q.w};
                    __builtin_nontemporal_store(
                        out, reinterpret_cast<u32x4_nt*>(&X[(k0 + u) * vps + l * P + p]));
                }
                float f[kV];
                E::unpack(q, f);
#pragma unroll
                for (int e = 0; e < kV; ++e) acc = fmaf(f[e], vf[l][e], acc);
            }
            sum[u] = group_sum<P>(acc);
        }
#pragma unroll
        for (int u0 = 0; u0 < U; u0 += P) {
            float val = sum[u0];
#pragma unroll
            for (int t = 1; t < P && u0 + t < U; ++t)
                if (p == t) val = sum[u0 + t];
            const int u = u0 + p;
            if (u < U && k0 + u < n_sub) E::store(S, k0 + u, val);
        }
    }
}

// Any size or alignment: X alone, one element per thread; compress follows as its own launch.
template <typename E>
__global__ __launch_bounds__(256) void swiglu_generic_kernel(const typename E::type* __restrict__ gate,
                                                            const typename E::type* __restrict__ up,
                                                            typename E::type* __restrict__ X, int64_t n) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += stride)
        E::store(X, i, silu_mul(E::load(gate, i), E::load(up, i)));
}

namespace {

template <typename E, int P, int L, int U>
hipError_t launch_vec(const void* gate, const void* up, const float* v, void* X, void* S, int64_t n_sub, int vps,
                      const LaunchCfg& cfg, hipStream_t st) {
    constexpr int SEG = kWave / P;
    const int64_t n_chunks = ceil_div(n_sub, static_cast<int64_t>(SEG) * U);
    int64_t grid = ceil_div(n_chunks, 4);
    if (grid < 1) grid = 1;
    if (grid > cfg.max_blocks) grid = cfg.max_blocks;
    hipLaunchKernelGGL((swiglu_compress_vec_kernel<E, P, L, U>), dim3(static_cast<unsigned>(grid)), dim3(256), 0, st,
                       static_cast<const uint4*>(gate), static_cast<const uint4*>(up), v, static_cast<uint4*>(X),
                       static_cast<typename E::type*>(S), n_sub, vps);
    return hipGetLastError();
}

template <typename E>
hipError_t swiglu_any(const void* gate, const void* up, const float* v, void* X, void* S, int64_t n_sub, int64_t d,
                      bool vec_ok, const LaunchCfg& cfg, hipStream_t st) {
    if (vec_ok && d % E::kPerVec == 0 && d / E::kPerVec <= 256) {
        // the same lanes-per-sub-token choice as dispatch_compress_vec, so S matches velora_compress bit for bit
        const int vps = static_cast<int>(d / E::kPerVec);
        if (vps <= 1) return launch_vec<E, 1, 1, 4>(gate, up, v, X, S, n_sub, vps, cfg, st);
        if (vps <= 2) return launch_vec<E, 2, 1, 4>(gate, up, v, X, S, n_sub, vps, cfg, st);
        if (vps <= 4) return launch_vec<E, 4, 1, 4>(gate, up, v, X, S, n_sub, vps, cfg, st);
        if (vps <= 8) return launch_vec<E, 8, 1, 4>(gate, up, v, X, S, n_sub, vps, cfg, st);
        if (vps <= 16) return launch_vec<E, 16, 1, 4>(gate, up, v, X, S, n_sub, vps, cfg, st);
        if (vps <= 32) return launch_vec<E, 32, 1, 4>(gate, up, v, X, S, n_sub, vps, cfg, st);
        if (vps <= 64) return launch_vec<E, 64, 1, 4>(gate, up, v, X, S, n_sub, vps, cfg, st);
        if (vps <= 128) return launch_vec<E, 64, 2, 2>(gate, up, v, X, S, n_sub, vps, cfg, st);
        return launch_vec<E, 64, 4, 1>(gate, up, v, X, S, n_sub, vps, cfg, st);
    }
    const int64_t n = n_sub * d;
    int64_t grid = ceil_div(n, 256 * 4);
    if (grid < 1) grid = 1;
    if (grid > cfg.max_blocks) grid = cfg.max_blocks;
    hipLaunchKernelGGL((swiglu_generic_kernel<E>), dim3(static_cast<unsigned>(grid)), dim3(256), 0, st,
                       static_cast<const typename E::type*>(gate), static_cast<const typename E::type*>(up),
                       static_cast<typename E::type*>(X), n);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_compress(X, v, S, n_sub, d, std::is_same<E, Bf16Elem>::value, vec_ok, cfg, st);
}

}  // namespace

hipError_t launch_swiglu_compress(const void* gate, const void* up, const float* v, void* X, void* S, int64_t n_sub,
                                  int64_t d, bool is_bf16, bool vec_ok, const LaunchCfg& cfg, hipStream_t st) {
    return is_bf16 ? swiglu_any<Bf16Elem>(gate, up, v, X, S, n_sub, d, vec_ok, cfg, st)
                   : swiglu_any<F32Elem>(gate, up, v, X, S, n_sub, d, vec_ok, cfg, st);
}

}  // namespace velora
