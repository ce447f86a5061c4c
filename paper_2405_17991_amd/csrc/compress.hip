// group + compress, and reconstruct + ungroup (paper Sec. 3.1).
//
// X[N, D] is row-major and d divides D, so "split every token into M = D/d
// sub-tokens" is nothing but reading the flat array in runs of d elements:
// sub-token k = n*M + g occupies elements [k*d, (k+1)*d).  compress is a flat
// batched dot product S[k] = <X[k*d : (k+1)*d], v>, reconstruct its transpose
// Xhat[k*d + j] = S[k] * v[j].  Both are pure HBM streams (about one flop per
// byte), so the kernels are built around 16-byte coalesced accesses with many
// loads in flight per wave; the arithmetic hides under the memory time.
#include "common.h"
#include "kernels.h"

namespace velora {

// ---------------------------------------------------------------------------
// Vectorised compress.
//   E   element traits (F32Elem: 4 per 16-byte vector, Bf16Elem: 8)
//   P   lanes that share one sub-token (d / E::kPerVec, capped at 64)
//   L   16-byte vectors each lane reads per sub-token (1 unless d > 64*kPerVec)
//   U   sub-tokens per lane group and iteration = independent loads in flight
// A wave iteration ("super-chunk") covers SEG*U consecutive sub-tokens, SEG =
// 64/P lane groups; group `seg` owns sub-tokens base + seg*U + [0, U), so after
// the cross-lane sums lane (seg, p) can store result u = p and the wave's
// stores form one contiguous run of S.
// ---------------------------------------------------------------------------
template <typename E, int P, int L, int U>
__global__ __launch_bounds__(256) void compress_vec_kernel(const typename E::vec* __restrict__ X,
                                                          const float* __restrict__ v,
                                                          typename E::type* __restrict__ S,
                                                          int64_t n_sub, int vps) {
    // vps = vectors (16 bytes; 8 for Bf16Half) per sub-token, P * (L - 1) < vps <= P * L: when d / kPerVec is not a power of
    // two the lanes (and vectors) past vps stay idle and contribute zeros
    constexpr int kV = E::kPerVec;
    constexpr int SEG = kWave / P;
    const int lane = threadIdx.x & (kWave - 1);
    const int p = lane % P;
    const int seg = lane / P;
    const int64_t wave = (static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x) / kWave;
    const int64_t n_waves = static_cast<int64_t>(gridDim.x) * blockDim.x / kWave;
    const int64_t n_chunks = ceil_div(n_sub, static_cast<int64_t>(SEG) * U);

    // this lane's slice of v never changes
    float vf[L][kV];
#pragma unroll
    for (int l = 0; l < L; ++l)
#pragma unroll
        for (int e = 0; e < kV; ++e) vf[l][e] = (l * P + p) < vps ? v[(l * P + p) * kV + e] : 0.f;

    for (int64_t chunk = wave; chunk < n_chunks; chunk += n_waves) {
        const int64_t k0 = chunk * (SEG * U) + static_cast<int64_t>(seg) * U;
        typename E::vec q[U][L];
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int l = 0; l < L; ++l) {
                q[u][l] = E::zero_vec();
                if (k0 + u < n_sub && l * P + p < vps) q[u][l] = E::load_stream(&X[(k0 + u) * vps + l * P + p]);
            }
        float sum[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float acc = 0.f;
#pragma unroll
            for (int l = 0; l < L; ++l) {
                float f[kV];
                E::unpack(q[u][l], f);
#pragma unroll
                for (int e = 0; e < kV; ++e) acc = fmaf(f[e], vf[l][e], acc);
            }
            sum[u] = group_sum<P>(acc);
        }
        // lane (seg, p) stores results u = p, p + P, ... of its group
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

// bf16 sub-tokens whose size is a multiple of 4 but not of 8 (d = 172: the 11008-wide layer at 64
// sub-tokens per token) start on a 16-byte boundary only every second time, but a PAIR of them is
// d / 4 whole 16-byte vectors.  One wave slot takes a pair: lane p loads vector p of the pair and keeps
// two slices of v, one for the elements that belong to the first sub-token and one for the second
// (the vector in the middle straddles both), so the loads are the 16-byte ones of the kernel above
// and only the arithmetic doubles.  With 8-byte loads (one sub-token of 43 vectors per wave slot) the
// layer ran at 0.68 of the HBM peak, as a pair of 43 16-byte vectors at the 0.74 of d = 344.
// Needs an even number of sub-tokens, X 16-byte aligned, 33 <= d / 4 <= 64.
template <int U>
__global__ __launch_bounds__(256) void compress_pair_kernel(const uint4* __restrict__ X, const float* __restrict__ v,
                                                           uint16_t* __restrict__ S, int64_t n_pairs, int vpp, int d) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t wave = (static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x) / kWave;
    const int64_t n_waves = static_cast<int64_t>(gridDim.x) * blockDim.x / kWave;
    const int64_t n_chunks = ceil_div(n_pairs, static_cast<int64_t>(U));
    float va[8], vb[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int idx = lane * 8 + e;
        va[e] = idx < d ? v[idx] : 0.f;
        vb[e] = (idx >= d && idx < 2 * d) ? v[idx - d] : 0.f;
    }
    for (int64_t chunk = wave; chunk < n_chunks; chunk += n_waves) {
        const int64_t k0 = chunk * U;
        uint4 q[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            q[u] = make_uint4(0u, 0u, 0u, 0u);
            if (k0 + u < n_pairs && lane < vpp) q[u] = load_stream16(&X[(k0 + u) * vpp + lane]);
        }
        float sa[U], sb[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float f[8];
            Bf16Elem::unpack(q[u], f);
            float a = 0.f, b = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                a = fmaf(f[e], va[e], a);
                b = fmaf(f[e], vb[e], b);
            }
            sa[u] = group_sum<kWave>(a);
            sb[u] = group_sum<kWave>(b);
        }
        // lane r < 2U stores result r of the wave's 2U consecutive sub-tokens
        float val = sa[0];
#pragma unroll
        for (int r = 1; r < 2 * U; ++r)
            if (lane == r) val = (r & 1) ? sb[r / 2] : sa[r / 2];
        if (lane < 2 * U && k0 + lane / 2 < n_pairs) Bf16Elem::store(S, 2 * k0 + lane, val);
    }
}

// Generic compress: any d, element-aligned pointers.  P lanes (power of two,
// chosen by the host) share a sub-token and stride over its elements.
template <typename E>
__global__ __launch_bounds__(256) void compress_generic_kernel(const typename E::type* __restrict__ X,
                                                              const float* __restrict__ v,
                                                              typename E::type* __restrict__ S,
                                                              int64_t n_sub, int d, int P) {
    const int lane = threadIdx.x & (kWave - 1);
    const int p = lane % P;
    const int seg = lane / P;
    const int SEG = kWave / P;
    const int64_t wave = (static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x) / kWave;
    const int64_t n_waves = static_cast<int64_t>(gridDim.x) * blockDim.x / kWave;
    const int64_t n_chunks = ceil_div(n_sub, SEG);
    for (int64_t chunk = wave; chunk < n_chunks; chunk += n_waves) {
        const int64_t k = chunk * SEG + seg;
        float acc = 0.f;
        if (k < n_sub)
            for (int j = p; j < d; j += P) acc = fmaf(E::load(X, k * d + j), v[j], acc);
        acc = group_sum_rt(acc, P);
        if (p == 0 && k < n_sub) E::store(S, k, acc);
    }
}

// ---------------------------------------------------------------------------
// Compress for sub-token sizes that no vector kernel takes (d not a multiple of 4 elements: d = 43 or 86 is
// what 256 or 128 sub-tokens per token make of an 11008-wide layer), when X itself is 16-byte aligned and
// holds a whole number of 16-byte vectors.  A tile of TS consecutive sub-tokens is TS * d consecutive
// elements and starts on a 16-byte boundary whatever d is (TS is a multiple of 8): the block copies it into
// LDS with streaming 16-byte loads, then thread k walks sub-token k in LDS element by element; the j-th
// element of v is the same for every lane (an LDS broadcast).  Four accumulators (j mod 4), combined
// (a0 + a1) + (a2 + a3): a fixed order.  Latency is hidden by the other blocks of the compute unit (a tile
// is at most 64 KB).  16384 x 11008 bf16 at d = 43: 490 us with the element-wise kernel below.
// ---------------------------------------------------------------------------
template <typename E, int TS>
__global__ __launch_bounds__(TS) void compress_tile_lds_kernel(const uint4* __restrict__ X, const float* __restrict__ v,
                                                               typename E::type* __restrict__ S, int64_t n_sub, int d,
                                                               int64_t n_vec_total) {
    extern __shared__ __attribute__((aligned(16))) unsigned char tile_raw[];
    using T = typename E::type;
    const int vpt = TS * d / E::kPerVec;                          // 16-byte vectors per tile (TS % kPerVec == 0)
    uint4* tile_v = reinterpret_cast<uint4*>(tile_raw);
    const T* tile_e = reinterpret_cast<const T*>(tile_raw);
    float* vs = reinterpret_cast<float*>(tile_raw + static_cast<size_t>(vpt) * 16);
    const int tid = threadIdx.x;
    for (int j = tid; j < d; j += TS) vs[j] = v[j];
    const int64_t n_tiles = ceil_div(n_sub, static_cast<int64_t>(TS));
    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int64_t v0 = tile * vpt;
        __syncthreads();                                          // the previous tile has been read (and vs written)
        for (int i0 = 0; i0 < vpt; i0 += 4 * TS) {                // four loads in flight per thread
            uint4 q[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = i0 + u * TS + tid;
                q[u] = (i < vpt && v0 + i < n_vec_total) ? load_stream16(&X[v0 + i]) : make_uint4(0u, 0u, 0u, 0u);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = i0 + u * TS + tid;
                if (i < vpt) tile_v[i] = q[u];
            }
        }
        __syncthreads();
        const int64_t k = tile * TS + tid;
        const T* row = tile_e + static_cast<size_t>(tid) * d;
        float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
        int j = 0;
        for (; j + 4 <= d; j += 4) {
            a0 = fmaf(E::load(row, j), vs[j], a0);
            a1 = fmaf(E::load(row, j + 1), vs[j + 1], a1);
            a2 = fmaf(E::load(row, j + 2), vs[j + 2], a2);
            a3 = fmaf(E::load(row, j + 3), vs[j + 3], a3);
        }
        if (j < d) a0 = fmaf(E::load(row, j), vs[j], a0);
        if (j + 1 < d) a1 = fmaf(E::load(row, j + 1), vs[j + 1], a1);
        if (j + 2 < d) a2 = fmaf(E::load(row, j + 2), vs[j + 2], a2);
        if (k < n_sub) E::store(S, k, (a0 + a1) + (a2 + a3));
    }
}

// ---------------------------------------------------------------------------
// reconstruct + ungroup (Sec. 3.1): Xhat[k*d + j] = S[k] * v[j].  Write-bound.
// The grid's thread count is a multiple of the 16-byte vectors per sub-token
// (vps, host-checked), so a thread keeps the same position j inside the
// sub-token for the whole grid-stride loop: its slice of v lives in registers
// and the loop body is one 2/4-byte load of S, kV multiplies and one streaming
// 16-byte store; consecutive threads write consecutive vectors.  One block per
// compute unit and kUnroll = 8 stores in flight per thread, each of them part of a
// grid-wide contiguous window: 59-62 us on 16384 x 11008 bf16 against 68 us with
// eight blocks per compute unit and four stores per thread in wave-private runs.
// ---------------------------------------------------------------------------
typedef uint32_t u32x4_store __attribute__((ext_vector_type(4)));

template <typename E, int kUnroll>
__global__ __launch_bounds__(256) void reconstruct_vec_kernel(const typename E::type* __restrict__ S,
                                                             const float* __restrict__ v,
                                                             uint4* __restrict__ Xhat,
                                                             int64_t n_sub, int vps) {
    constexpr int kV = E::kPerVec;
    const int64_t n_threads = static_cast<int64_t>(gridDim.x) * blockDim.x;     // a multiple of vps
    const int64_t t = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    const int64_t k_step = n_threads / vps;
    const int64_t k_base = t / vps;
    const int jv = static_cast<int>(t - k_base * vps);
    // One trip = kUnroll grid-wide windows: in window u every thread writes the vector next to its
    // neighbour's, so the whole chip writes one contiguous run of n_threads vectors at a time (the order
    // HBM takes fastest; one block per compute unit, eight stores in flight per thread).
    float vf[kV];
#pragma unroll
    for (int e = 0; e < kV; e += 4) {
        const float4 q = *reinterpret_cast<const float4*>(v + jv * kV + e);
        vf[e] = q.x; vf[e + 1] = q.y; vf[e + 2] = q.z; vf[e + 3] = q.w;
    }
    // Full trips (every window inside the array; the same test for all threads) run in a loop without
    // per-lane conditions: an index past the end is clamped to the last element and its value never
    // stored.  (Behind per-lane conditions the compiler's wait-count bookkeeping gives up and waits for
    // every load on its own and for all stores once per trip.)  The values of S are requested two trips
    // ahead of the stores that use them, into two alternating register sets, and stay raw until they
    // are used, so that nothing asks for them early: with one block per compute unit nothing else
    // hides their latency.
    using T = typename E::type;
    const int64_t trip = kUnroll * k_step;
    const int64_t n_full = n_sub / trip;
    auto fetch = [&](T (&r)[kUnroll], int64_t base) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int64_t kk = base + k_base + u * k_step;
            r[u] = S[kk < n_sub ? kk : n_sub - 1];
        }
    };
    auto value = [&](T r) -> float {
        if constexpr (sizeof(T) == 2) return bf16_to_f32(r);
        else return r;
    };
    auto store = [&](float s, int64_t kk) {
        float f[kV];
#pragma unroll
        for (int e = 0; e < kV; ++e) f[e] = s * vf[e];
        u32x4_store out;
        if constexpr (kV == 4) {
            out = u32x4_store{__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3])};
        } else {
            out = u32x4_store{pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]),
                              pack_bf16x2(f[6], f[7])};
        }
        __builtin_nontemporal_store(out, reinterpret_cast<u32x4_store*>(Xhat + kk * vps + jv));
    };
    auto full_trip = [&](T (&r)[kUnroll], int64_t base, bool refill) {
        float cur[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) cur[u] = value(r[u]);
        if (refill) fetch(r, base + 2 * trip);
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) store(cur[u], base + k_base + u * k_step);
    };
    T pa[kUnroll], pb[kUnroll];
    fetch(pa, 0);
    fetch(pb, trip);
    int64_t base = 0, i = 0;
    for (; i + 2 <= n_full; i += 2) {
        full_trip(pa, base, true);
        base += trip;
        full_trip(pb, base, true);
        base += trip;
    }
    if (i < n_full) {
        full_trip(pa, base, false);
        base += trip;
    }
    // the last, partial trip
    if (base < n_sub) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int64_t kk = base + k_base + u * k_step;
            if (kk < n_sub) store(E::load(S, kk), kk);
        }
    }
}

template <typename E>
__global__ __launch_bounds__(256) void reconstruct_generic_kernel(const typename E::type* __restrict__ S,
                                                                 const float* __restrict__ v,
                                                                 typename E::type* __restrict__ Xhat,
                                                                 int64_t n_elem, int d) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n_elem; i += stride) {
        const int64_t k = i / d;
        E::store(Xhat, i, E::load(S, k) * v[i - k * d]);
    }
}

// Reconstruct for sub-token sizes whose 16-byte vectors straddle sub-tokens (d not a multiple of the vector
// width), Xhat 16-byte aligned and a whole number of vectors: a thread still writes whole vectors; it finds
// the sub-token and the position of its vector's first element by one division and steps through the
// boundaries inside the vector.  v sits in LDS.  16384 x 11008 bf16 at d = 43: 186 us with the element-wise
// kernel above.
template <typename E>
__global__ __launch_bounds__(256) void reconstruct_straddle_kernel(const typename E::type* __restrict__ S,
                                                                  const float* __restrict__ v, uint4* __restrict__ Xhat,
                                                                  int64_t n_vec, int64_t n_sub, int d) {
    constexpr int kV = E::kPerVec;
    extern __shared__ float vs_lds[];
    for (int j = threadIdx.x; j < d; j += blockDim.x) vs_lds[j] = v[j];
    __syncthreads();
    const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n_vec; i += stride) {
        const int64_t e = i * kV;
        int64_t k = e / d;
        int j = static_cast<int>(e - k * d);
        float s = E::load(S, k);
        float r[kV];
#pragma unroll
        for (int u = 0; u < kV; ++u) {
            r[u] = s * vs_lds[j];
            if (++j == d) {
                j = 0;
                ++k;
                if (k < n_sub) s = E::load(S, k);
            }
        }
        u32x4_store out;
        if constexpr (kV == 8) {
            out = u32x4_store{pack_bf16x2(r[0], r[1]), pack_bf16x2(r[2], r[3]), pack_bf16x2(r[4], r[5]), pack_bf16x2(r[6], r[7])};
        } else {
            out = u32x4_store{__float_as_uint(r[0]), __float_as_uint(r[1]), __float_as_uint(r[2]), __float_as_uint(r[3])};
        }
        __builtin_nontemporal_store(out, reinterpret_cast<u32x4_store*>(&Xhat[i]));
    }
}

// ---------------------------------------------------------------------------
// host-side dispatch
// ---------------------------------------------------------------------------
namespace {

constexpr int kBlock = 256;

int grid_for(int64_t n_wave_items, int waves_per_block, int max_blocks) {
    int64_t b = ceil_div(n_wave_items, waves_per_block);
    if (b < 1) b = 1;
    if (b > max_blocks) b = max_blocks;
    return static_cast<int>(b);
}

template <typename E, int P, int L, int U>
hipError_t launch_compress_vec(const void* X, const float* v, void* S, int64_t n_sub, int vps, const LaunchCfg& cfg,
                               hipStream_t st) {
    constexpr int SEG = kWave / P;
    const int64_t n_chunks = ceil_div(n_sub, static_cast<int64_t>(SEG) * U);
    // Sub-tokens of more than 64 vectors (L > 1) keep 8 KB per wave in flight with fewer, longer sums per
    // wave; two blocks per compute unit then do better than eight (29.7 against 32.2 us on N = 16384,
    // D = 5120, d = 1024), as they do for a plain read stream on this chip.
    const int grid = grid_for(n_chunks, kBlock / kWave, L > 1 ? cfg.num_cus * 2 : cfg.max_blocks);
    hipLaunchKernelGGL((compress_vec_kernel<E, P, L, U>), dim3(grid), dim3(kBlock), 0, st,
                       static_cast<const typename E::vec*>(X), v, static_cast<typename E::type*>(S), n_sub, vps);
    return hipGetLastError();
}

template <typename E>
hipError_t dispatch_compress_vec(int vec_per_sub, const void* X, const float* v, void* S, int64_t n_sub,
                                 const LaunchCfg& cfg, hipStream_t st, bool* handled) {
    *handled = true;
    // lanes per sub-token: the next power of two (at most 64); vectors per lane: 1, 2 or 4
    const int vps = vec_per_sub;
    if (vps <= 1) return launch_compress_vec<E, 1, 1, 8>(X, v, S, n_sub, vps, cfg, st);
    if (vps <= 2) return launch_compress_vec<E, 2, 1, 8>(X, v, S, n_sub, vps, cfg, st);
    if (vps <= 4) return launch_compress_vec<E, 4, 1, 8>(X, v, S, n_sub, vps, cfg, st);
    if (vps <= 8) return launch_compress_vec<E, 8, 1, 8>(X, v, S, n_sub, vps, cfg, st);
    if (vps <= 16) return launch_compress_vec<E, 16, 1, 8>(X, v, S, n_sub, vps, cfg, st);
    if (vps <= 32) return launch_compress_vec<E, 32, 1, 8>(X, v, S, n_sub, vps, cfg, st);
    if (vps <= 64) return launch_compress_vec<E, 64, 1, 8>(X, v, S, n_sub, vps, cfg, st);
    if (vps <= 128) return launch_compress_vec<E, 64, 2, 4>(X, v, S, n_sub, vps, cfg, st);
    if (vps <= 256) return launch_compress_vec<E, 64, 4, 2>(X, v, S, n_sub, vps, cfg, st);
    *handled = false;
    return hipSuccess;
}

template <typename E>
hipError_t compress_any(const void* X, const float* v, void* S, int64_t n_sub, int64_t d, bool vec_ok,
                        const LaunchCfg& cfg, hipStream_t st) {
    if (vec_ok && d % E::kPerVec == 0) {
        bool handled = false;
        hipError_t e = dispatch_compress_vec<E>(static_cast<int>(d / E::kPerVec), X, v, S, n_sub, cfg, st, &handled);
        if (handled) return e;
    }
    if constexpr (std::is_same<E, Bf16Elem>::value) {
        // a multiple of 4 but not of 8 (the 11008-wide layer at 64 sub-tokens per token: d = 172): 8-byte vectors
        if (vec_ok && d % 8 == 4 && d / 4 >= 33 && d / 4 <= 64 && n_sub % 2 == 0) {
            constexpr int U = 8;
            const int64_t n_pairs = n_sub / 2;
            const int grid = grid_for(ceil_div(n_pairs, static_cast<int64_t>(U)), kBlock / kWave, cfg.max_blocks);
            hipLaunchKernelGGL((compress_pair_kernel<U>), dim3(grid), dim3(kBlock), 0, st, static_cast<const uint4*>(X), v,
                               static_cast<uint16_t*>(S), n_pairs, static_cast<int>(d / 4), static_cast<int>(d));
            return hipGetLastError();
        }
        if (d % 4 == 0 && (reinterpret_cast<uintptr_t>(X) & 7) == 0) {
            bool handled = false;
            hipError_t e = dispatch_compress_vec<Bf16Half>(static_cast<int>(d / 4), X, v, S, n_sub, cfg, st, &handled);
            if (handled) return e;
        }
    }
    // any other sub-token size, X 16-byte aligned and a whole number of vectors: tiles of 256 (or 64) sub-tokens
    // through LDS, as long as a tile and v fit 64 KB
    if (vec_ok && d <= 4096 && (static_cast<double>(n_sub) * static_cast<double>(d)) < 9.0e18) {
        const int64_t esize = sizeof(typename E::type);
        const int64_t n_elem = n_sub * d;
        if (n_elem % E::kPerVec == 0) {
            const int64_t n_vec_total = n_elem / E::kPerVec;
            auto go = [&](auto kernel, int ts) {
                const size_t lds = static_cast<size_t>(ts) * d * esize + static_cast<size_t>(d) * 4;
                const int64_t n_tiles = ceil_div(n_sub, static_cast<int64_t>(ts));
                int64_t grid = static_cast<int64_t>(cfg.num_cus) * (ts == 256 ? 8 : 32);
                if (grid > n_tiles) grid = n_tiles;
                hipLaunchKernelGGL(kernel, dim3(static_cast<unsigned>(grid)), dim3(ts), lds, st, static_cast<const uint4*>(X), v,
                                   static_cast<typename E::type*>(S), n_sub, static_cast<int>(d), n_vec_total);
                return hipGetLastError();
            };
            if (256 * d * esize + d * 4 <= 65536) return go(compress_tile_lds_kernel<E, 256>, 256);
            if (64 * d * esize + d * 4 <= 65536) return go(compress_tile_lds_kernel<E, 64>, 64);
        }
    }
    int P = 1;
    while (P < kWave && P < d) P <<= 1;
    const int64_t n_chunks = ceil_div(n_sub, kWave / P);
    const int grid = grid_for(n_chunks, kBlock / kWave, cfg.max_blocks);
    hipLaunchKernelGGL((compress_generic_kernel<E>), dim3(grid), dim3(kBlock), 0, st,
                       static_cast<const typename E::type*>(X), v, static_cast<typename E::type*>(S), n_sub,
                       static_cast<int>(d), P);
    return hipGetLastError();
}

template <typename E>
hipError_t reconstruct_any(const void* S, const float* v, void* Xhat, int64_t n_sub, int64_t d, bool vec_ok,
                           const LaunchCfg& cfg, hipStream_t st) {
    const int64_t n_elem = n_sub * d;
    // the streaming kernel wants (grid * 256) % vps == 0: grid a multiple of vps / gcd(vps, 256)
    int64_t vps = d / E::kPerVec, grid_quantum = 0;
    if (vec_ok && d % E::kPerVec == 0) {
        int64_t g = vps, h = kBlock;
        while (h) { const int64_t r = g % h; g = h; h = r; }
        grid_quantum = vps / g;
    }
    if (grid_quantum > 0 && grid_quantum <= 64) {
        const int64_t n_vec = n_elem / E::kPerVec;
        // one block per compute unit; rounded DOWN to the quantum (a few blocks more than compute units
        // would leave the last ones to run alone at one unit's share of the bandwidth)
        int64_t grid = grid_for(ceil_div(n_vec, kBlock * 8), 1, cfg.num_cus);
        grid = grid >= grid_quantum ? grid / grid_quantum * grid_quantum : grid_quantum;
        hipLaunchKernelGGL((reconstruct_vec_kernel<E, 8>), dim3(static_cast<unsigned>(grid)), dim3(kBlock), 0, st,
                           static_cast<const typename E::type*>(S), v, static_cast<uint4*>(Xhat), n_sub,
                           static_cast<int>(vps));
    } else if (vec_ok && n_elem % E::kPerVec == 0 && d <= 8192) {
        const int64_t n_vec = n_elem / E::kPerVec;
        const int grid = grid_for(ceil_div(n_vec, kBlock * 4), 1, cfg.num_cus * 8);
        hipLaunchKernelGGL((reconstruct_straddle_kernel<E>), dim3(grid), dim3(kBlock), static_cast<size_t>(d) * 4, st,
                           static_cast<const typename E::type*>(S), v, static_cast<uint4*>(Xhat), n_vec, n_sub,
                           static_cast<int>(d));
    } else {
        const int grid = grid_for(ceil_div(n_elem, kBlock), 1, cfg.max_blocks * 4);
        hipLaunchKernelGGL((reconstruct_generic_kernel<E>), dim3(grid), dim3(kBlock), 0, st,
                           static_cast<const typename E::type*>(S), v, static_cast<typename E::type*>(Xhat), n_elem,
                           static_cast<int>(d));
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_compress(const void* X, const float* v, void* S, int64_t n_sub, int64_t d, bool is_bf16,
                           bool vec_ok, const LaunchCfg& cfg, hipStream_t st) {
    return is_bf16 ? compress_any<Bf16Elem>(X, v, S, n_sub, d, vec_ok, cfg, st)
                   : compress_any<F32Elem>(X, v, S, n_sub, d, vec_ok, cfg, st);
}

hipError_t launch_reconstruct(const void* S, const float* v, void* Xhat, int64_t n_sub, int64_t d, bool is_bf16,
                              bool vec_ok, const LaunchCfg& cfg, hipStream_t st) {
    return is_bf16 ? reconstruct_any<Bf16Elem>(S, v, Xhat, n_sub, d, vec_ok, cfg, st)
                   : reconstruct_any<F32Elem>(S, v, Xhat, n_sub, d, vec_ok, cfg, st);
}

}  // namespace velora
