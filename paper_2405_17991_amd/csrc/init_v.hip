// Initialisation of the projection vector (paper Sec. 3.2, "Cheap
// initialisation strategies": the average of the first batch's sub-tokens;
// Sec. 3.1: v has unit length):
//     m[j] = 1/(N*M) * sum_k X[k*d + j],   v = m / ||m||_2
// i.e. the column mean of the flat [N*M, d] view of X.  One streaming pass over
// X (HBM-bound) produces per-block float32 partial column sums; they are
// combined in float64 in a fixed order, so the result is deterministic and the
// long sum never runs in a single float32 accumulator.
#include "common.h"
#include "kernels.h"

namespace velora {

// Same lane <-> element mapping as the vectorised compress kernel: lane
// (seg, p) always sees columns (l*P + p)*kPerVec + [0, kPerVec) of a sub-token.
template <typename E, int P, int L, int U>
__global__ __launch_bounds__(256) void colsum_vec_kernel(const uint4* __restrict__ X, float* __restrict__ partial,
                                                        int64_t n_sub, int d) {
    constexpr int kV = E::kPerVec;
    constexpr int SEG = kWave / P;
    constexpr int kWavesPerBlock = 256 / kWave;
    __shared__ float lds[kWavesPerBlock][L * kV][kWave + 1];
    const int vps = d / kV;        // vectors per sub-token, P * (L - 1) < vps <= P * L; lanes past it stay idle

    const int lane = threadIdx.x & (kWave - 1);
    const int wib = threadIdx.x / kWave;
    const int p = lane % P;
    const int seg = lane / P;
    const int64_t wave = (static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x) / kWave;
    const int64_t n_waves = static_cast<int64_t>(gridDim.x) * blockDim.x / kWave;
    const int64_t n_chunks = ceil_div(n_sub, static_cast<int64_t>(SEG) * U);

    float acc[L][kV];
#pragma unroll
    for (int l = 0; l < L; ++l)
#pragma unroll
        for (int e = 0; e < kV; ++e) acc[l][e] = 0.f;

    for (int64_t chunk = wave; chunk < n_chunks; chunk += n_waves) {
        const int64_t k0 = chunk * (SEG * U) + seg;
        uint4 q[U][L];
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int l = 0; l < L; ++l) {
                q[u][l] = make_uint4(0u, 0u, 0u, 0u);
                const int64_t k = k0 + static_cast<int64_t>(u) * SEG;
                if (k < n_sub && l * P + p < vps) q[u][l] = load_stream16(&X[k * vps + l * P + p]);
            }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int l = 0; l < L; ++l) {
                float f[kV];
                E::unpack(q[u][l], f);
#pragma unroll
                for (int e = 0; e < kV; ++e) acc[l][e] += f[e];
            }
    }
#pragma unroll
    for (int l = 0; l < L; ++l)
#pragma unroll
        for (int e = 0; e < kV; ++e) lds[wib][l * kV + e][lane] = acc[l][e];
    __syncthreads();
    // column j lives in lanes seg*P + p of every wave, slot l*kV + e
    for (int j = threadIdx.x; j < d; j += blockDim.x) {
        const int l = j / (P * kV);
        const int rem = j - l * (P * kV);
        const int pp = rem / kV;
        const int e = rem - pp * kV;
        float s = 0.f;
        for (int w = 0; w < kWavesPerBlock; ++w)
            for (int sg = 0; sg < SEG; ++sg) s += lds[w][l * kV + e][sg * P + pp];
        partial[static_cast<int64_t>(blockIdx.x) * d + j] = s;
    }
}

// Generic column sums: any d, element-aligned pointer.  C threads across
// columns (coalesced), R = 256/C sub-tokens in parallel.
template <typename E>
__global__ __launch_bounds__(256) void colsum_generic_kernel(const typename E::type* __restrict__ X,
                                                            float* __restrict__ partial, int64_t n_sub, int d,
                                                            int C, int64_t sub_per_block) {
    __shared__ float lds[256];
    const int R = 256 / C;
    const int c = threadIdx.x % C;
    const int r = threadIdx.x / C;
    const int64_t k_begin = static_cast<int64_t>(blockIdx.x) * sub_per_block;
    int64_t k_end = k_begin + sub_per_block;
    if (k_end > n_sub) k_end = n_sub;
    for (int j0 = 0; j0 < d; j0 += C) {
        const int j = j0 + c;
        float acc = 0.f;
        if (j < d)
            for (int64_t k = k_begin + r; k < k_end; k += R) acc += E::load(X, k * d + j);
        lds[threadIdx.x] = acc;
        __syncthreads();
        if (r == 0 && j < d) {
            float s = 0.f;
            for (int rr = 0; rr < R; ++rr) s += lds[rr * C + c];
            partial[static_cast<int64_t>(blockIdx.x) * d + j] = s;
        }
        __syncthreads();
    }
}

// Column sums for sub-token sizes the vector kernel cannot take (d not a multiple of 4 elements), X 16-byte
// aligned and a whole number of vectors, d <= 256: tiles of TS consecutive sub-tokens (TS a multiple of 8, so a
// tile starts on a 16-byte boundary whatever d is) are copied into LDS with streaming 16-byte loads and summed
// from there, C threads across the columns and 256 / C sub-tokens in parallel, as in the kernel above.
// Block b takes tiles b, b + grid, ...; one partial row per block.  16384 x 11008 bf16 at d = 43: 470 us with
// the element-wise loads of the kernel above.
template <typename E>
__global__ __launch_bounds__(256) void colsum_tile_lds_kernel(const uint4* __restrict__ X, float* __restrict__ partial,
                                                             int64_t n_sub, int d, int C, int TS, int64_t n_vec_total) {
    extern __shared__ __attribute__((aligned(16))) unsigned char tile_raw[];
    __shared__ float red[256];
    using T = typename E::type;
    const int vpt = TS * d / E::kPerVec;
    uint4* tile_v = reinterpret_cast<uint4*>(tile_raw);
    const T* tile_e = reinterpret_cast<const T*>(tile_raw);
    const int tid = threadIdx.x;
    const int R = 256 / C;
    const int c = tid % C;
    const int r = tid / C;
    const int64_t n_tiles = ceil_div(n_sub, static_cast<int64_t>(TS));
    float acc = 0.f;
    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int64_t v0 = tile * vpt;
        __syncthreads();                                          // the previous tile has been read
        for (int i0 = 0; i0 < vpt; i0 += 4 * 256) {
            uint4 q[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = i0 + u * 256 + tid;
                q[u] = (i < vpt && v0 + i < n_vec_total) ? load_stream16(&X[v0 + i]) : make_uint4(0u, 0u, 0u, 0u);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = i0 + u * 256 + tid;
                if (i < vpt) tile_v[i] = q[u];
            }
        }
        __syncthreads();
        const int64_t left = n_sub - tile * TS;
        const int rows = left < TS ? static_cast<int>(left) : TS;
        if (c < d)
            for (int k = r; k < rows; k += R) acc += E::load(tile_e, static_cast<int64_t>(k) * d + c);
    }
    red[tid] = acc;
    __syncthreads();
    if (r == 0 && c < d) {
        float s = 0.f;
        for (int rr = 0; rr < R; ++rr) s += red[rr * C + c];
        partial[static_cast<int64_t>(blockIdx.x) * d + c] = s;
    }
}

// Stage 1 of the combine: slice sl of the block axis, 32 columns per block;
// slices[sl][j] = sum over the slice's blocks of partial[b][j], in float64, in a
// fixed order (8 interleaved row lanes, then the lanes in order).
constexpr int kSlices = 8;

__global__ __launch_bounds__(256) void colsum_combine_kernel(const float* __restrict__ partial,
                                                            double* __restrict__ slices, int blocks, int d) {
    __shared__ double red[8][32];
    const int c = threadIdx.x & 31;
    const int r = threadIdx.x >> 5;
    const int j = blockIdx.x * 32 + c;
    const int per_slice = (blocks + kSlices - 1) / kSlices;
    const int b0 = blockIdx.y * per_slice;
    int b1 = b0 + per_slice;
    if (b1 > blocks) b1 = blocks;
    double s = 0.0;
    if (j < d) {
        // eight loads in flight per thread; the additions keep their order
        int b = b0 + r;
        for (; b + 56 < b1; b += 64) {
            float t[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) t[u] = partial[static_cast<int64_t>(b + 8 * u) * d + j];
#pragma unroll
            for (int u = 0; u < 8; ++u) s += static_cast<double>(t[u]);
        }
        for (; b < b1; b += 8) s += static_cast<double>(partial[static_cast<int64_t>(b) * d + j]);
    }
    red[r][c] = s;
    __syncthreads();
    if (r == 0 && j < d) {
        double t = 0.0;
        for (int rr = 0; rr < 8; ++rr) t += red[rr][c];
        slices[static_cast<int64_t>(blockIdx.y) * d + j] = t;
    }
}

// Stage 2 (one block): batch mean m_b = (sum of slices) / n_sub; with a running
// state, m = beta * state + (1 - beta) * m_b and state <- m (float32); v = m / ||m||.
// flag = 0, or 6 (and v = 1/sqrt(d)) when m is zero or not finite.
__global__ __launch_bounds__(256) void normalise_v_kernel(const double* __restrict__ slices, double* __restrict__ mean,
                                                         float* __restrict__ state, double beta,
                                                         float* __restrict__ v, int* __restrict__ flag, int d,
                                                         double inv_count) {
    __shared__ double red[256];
    __shared__ int bad[256];
    double ss = 0.0;
    int nonfinite = 0;
    for (int j = threadIdx.x; j < d; j += blockDim.x) {
        double m = 0.0;
        for (int sl = 0; sl < kSlices; ++sl) m += slices[static_cast<int64_t>(sl) * d + j];
        m *= inv_count;
        if (state != nullptr) {
            m = beta * static_cast<double>(state[j]) + (1.0 - beta) * m;
            state[j] = static_cast<float>(m);
        }
        mean[j] = m;
        ss += m * m;
        if (!isfinite(m)) nonfinite = 1;
    }
    red[threadIdx.x] = ss;
    bad[threadIdx.x] = nonfinite;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (threadIdx.x < s) {
            red[threadIdx.x] += red[threadIdx.x + s];
            bad[threadIdx.x] |= bad[threadIdx.x + s];
        }
        __syncthreads();
    }
    const double norm = sqrt(red[0]);
    const bool degenerate = bad[0] || !(norm > 0.0) || !isfinite(norm);
    for (int j = threadIdx.x; j < d; j += blockDim.x)
        v[j] = degenerate ? static_cast<float>(1.0 / sqrt(static_cast<double>(d))) : static_cast<float>(mean[j] / norm);
    if (threadIdx.x == 0) *flag = degenerate ? 6 : 0;
}

// ---------------------------------------------------------------------------
// compress and column sums in ONE pass over X (running-average v): the same
// loop as compress_vec_kernel with the projection vector of the previous
// batches, plus the per-lane column sums that will form the next one.
// ---------------------------------------------------------------------------
template <typename E, int P, int L, int U>
__global__ __launch_bounds__(256) void compress_colsum_vec_kernel(const uint4* __restrict__ X,
                                                                 const float* __restrict__ v,
                                                                 typename E::type* __restrict__ S,
                                                                 float* __restrict__ partial, int64_t n_sub, int d) {
    constexpr int kV = E::kPerVec;
    constexpr int SEG = kWave / P;
    constexpr int kWavesPerBlock = 256 / kWave;
    __shared__ float lds[kWavesPerBlock][L * kV][kWave + 1];
    const int vps = d / kV;        // as in compress_vec_kernel: lanes and vectors past vps stay idle

    const int lane = threadIdx.x & (kWave - 1);
    const int wib = threadIdx.x / kWave;
    const int p = lane % P;
    const int seg = lane / P;
    const int64_t wave = (static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x) / kWave;
    const int64_t n_waves = static_cast<int64_t>(gridDim.x) * blockDim.x / kWave;
    const int64_t n_chunks = ceil_div(n_sub, static_cast<int64_t>(SEG) * U);

    float vf[L][kV], acc[L][kV];
#pragma unroll
    for (int l = 0; l < L; ++l)
#pragma unroll
        for (int e = 0; e < kV; ++e) {
            vf[l][e] = (l * P + p) < vps ? v[(l * P + p) * kV + e] : 0.f;
            acc[l][e] = 0.f;
        }

    for (int64_t chunk = wave; chunk < n_chunks; chunk += n_waves) {
        const int64_t k0 = chunk * (SEG * U) + static_cast<int64_t>(seg) * U;
        uint4 q[U][L];
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int l = 0; l < L; ++l) {
                q[u][l] = make_uint4(0u, 0u, 0u, 0u);
                if (k0 + u < n_sub && l * P + p < vps) q[u][l] = load_stream16(&X[(k0 + u) * vps + l * P + p]);
            }
        float sum[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float dot = 0.f;
#pragma unroll
            for (int l = 0; l < L; ++l) {
                float f[kV];
                E::unpack(q[u][l], f);
#pragma unroll
                for (int e = 0; e < kV; ++e) {
                    dot = fmaf(f[e], vf[l][e], dot);
                    acc[l][e] += f[e];
                }
            }
            sum[u] = group_sum<P>(dot);
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
#pragma unroll
    for (int l = 0; l < L; ++l)
#pragma unroll
        for (int e = 0; e < kV; ++e) lds[wib][l * kV + e][lane] = acc[l][e];
    __syncthreads();
    for (int j = threadIdx.x; j < d; j += blockDim.x) {
        const int l = j / (P * kV);
        const int rem = j - l * (P * kV);
        const int pp = rem / kV;
        const int e = rem - pp * kV;
        float s = 0.f;
        for (int w = 0; w < kWavesPerBlock; ++w)
            for (int sg = 0; sg < SEG; ++sg) s += lds[w][l * kV + e][sg * P + pp];
        partial[static_cast<int64_t>(blockIdx.x) * d + j] = s;
    }
}

namespace {

constexpr size_t kFlagBytes = 256;

template <typename E, int P, int L, int U>
hipError_t launch_colsum_vec(const void* X, float* partial, int64_t n_sub, int d, int blocks, hipStream_t st) {
    hipLaunchKernelGGL((colsum_vec_kernel<E, P, L, U>), dim3(blocks), dim3(256), 0, st,
                       static_cast<const uint4*>(X), partial, n_sub, d);
    return hipGetLastError();
}

template <typename E>
hipError_t dispatch_colsum_vec(int vec_per_sub, const void* X, float* partial, int64_t n_sub, int d, int blocks,
                               hipStream_t st, bool* handled) {
    *handled = true;
    const int vps = vec_per_sub;   // lanes per sub-token: the next power of two, at most 64; 1, 2 or 4 vectors per lane
    if (vps <= 1) return launch_colsum_vec<E, 1, 1, 8>(X, partial, n_sub, d, blocks, st);
    if (vps <= 2) return launch_colsum_vec<E, 2, 1, 8>(X, partial, n_sub, d, blocks, st);
    if (vps <= 4) return launch_colsum_vec<E, 4, 1, 8>(X, partial, n_sub, d, blocks, st);
    if (vps <= 8) return launch_colsum_vec<E, 8, 1, 8>(X, partial, n_sub, d, blocks, st);
    if (vps <= 16) return launch_colsum_vec<E, 16, 1, 8>(X, partial, n_sub, d, blocks, st);
    if (vps <= 32) return launch_colsum_vec<E, 32, 1, 8>(X, partial, n_sub, d, blocks, st);
    if (vps <= 64) return launch_colsum_vec<E, 64, 1, 8>(X, partial, n_sub, d, blocks, st);
    if (vps <= 128) return launch_colsum_vec<E, 64, 2, 4>(X, partial, n_sub, d, blocks, st);
    if (vps <= 256) return launch_colsum_vec<E, 64, 4, 2>(X, partial, n_sub, d, blocks, st);
    *handled = false;
    return hipSuccess;
}

bool vec_shape_ok(int64_t d, int per_vec) {
    if (d % per_vec) return false;
    return d / per_vec <= 256;
}

template <typename E>
hipError_t colsum_any(const void* X, float* partial, int64_t n_sub, int64_t d, bool vec_ok, int blocks,
                      hipStream_t st) {
    if (vec_ok && vec_shape_ok(d, E::kPerVec)) {
        bool handled = false;
        hipError_t e = dispatch_colsum_vec<E>(static_cast<int>(d / E::kPerVec), X, partial, n_sub,
                                              static_cast<int>(d), blocks, st, &handled);
        if (handled) return e;
    }
    int C = 1;
    while (C < 256 && C < d) C <<= 1;
    const int64_t esize = sizeof(typename E::type);
    if (vec_ok && d <= 256 && (n_sub * d) % E::kPerVec == 0) {
        const int ts = 256 * d * esize <= 63 * 1024 ? 256 : 64 * d * esize <= 63 * 1024 ? 64 : 0;
        if (ts > 0) {
            hipLaunchKernelGGL((colsum_tile_lds_kernel<E>), dim3(blocks), dim3(256), static_cast<size_t>(ts) * d * esize, st,
                               static_cast<const uint4*>(X), partial, n_sub, static_cast<int>(d), C, ts,
                               n_sub * d / E::kPerVec);
            return hipGetLastError();
        }
    }
    const int64_t sub_per_block = ceil_div(n_sub, blocks);
    hipLaunchKernelGGL((colsum_generic_kernel<E>), dim3(blocks), dim3(256), 0, st,
                       static_cast<const typename E::type*>(X), partial, n_sub, static_cast<int>(d), C,
                       sub_per_block);
    return hipGetLastError();
}

template <typename E, int P, int L, int U>
hipError_t launch_compress_colsum_vec(const void* X, const float* v, void* S, float* partial, int64_t n_sub, int d,
                                      int blocks, hipStream_t st) {
    hipLaunchKernelGGL((compress_colsum_vec_kernel<E, P, L, U>), dim3(blocks), dim3(256), 0, st,
                       static_cast<const uint4*>(X), v, static_cast<typename E::type*>(S), partial, n_sub, d);
    return hipGetLastError();
}

template <typename E>
hipError_t dispatch_compress_colsum(int vec_per_sub, const void* X, const float* v, void* S, float* partial,
                                    int64_t n_sub, int d, int blocks, hipStream_t st) {
    const int vps = vec_per_sub;   // at most 256: fused_compress_update_ok
    if (vps <= 1) return launch_compress_colsum_vec<E, 1, 1, 8>(X, v, S, partial, n_sub, d, blocks, st);
    if (vps <= 2) return launch_compress_colsum_vec<E, 2, 1, 8>(X, v, S, partial, n_sub, d, blocks, st);
    if (vps <= 4) return launch_compress_colsum_vec<E, 4, 1, 8>(X, v, S, partial, n_sub, d, blocks, st);
    if (vps <= 8) return launch_compress_colsum_vec<E, 8, 1, 8>(X, v, S, partial, n_sub, d, blocks, st);
    if (vps <= 16) return launch_compress_colsum_vec<E, 16, 1, 8>(X, v, S, partial, n_sub, d, blocks, st);
    if (vps <= 32) return launch_compress_colsum_vec<E, 32, 1, 8>(X, v, S, partial, n_sub, d, blocks, st);
    if (vps <= 64) return launch_compress_colsum_vec<E, 64, 1, 8>(X, v, S, partial, n_sub, d, blocks, st);
    if (vps <= 128) return launch_compress_colsum_vec<E, 64, 2, 4>(X, v, S, partial, n_sub, d, blocks, st);
    return launch_compress_colsum_vec<E, 64, 4, 2>(X, v, S, partial, n_sub, d, blocks, st);
}

struct WsView {
    int* flag;
    double* mean;
    double* slices;
    float* partial;
};

WsView ws_view(void* ws, const InitVPlan& plan) {
    char* base = static_cast<char*>(ws);
    WsView w;
    w.flag = reinterpret_cast<int*>(base);
    w.mean = reinterpret_cast<double*>(base + kFlagBytes);
    w.slices = reinterpret_cast<double*>(base + plan.slices_off);
    w.partial = reinterpret_cast<float*>(base + plan.partial_off);
    return w;
}

hipError_t finish_v(const WsView& w, int blocks, int64_t n_sub, int64_t d, float* state, double beta, float* v,
                    hipStream_t st) {
    const int di = static_cast<int>(d);
    hipLaunchKernelGGL(colsum_combine_kernel, dim3(static_cast<unsigned>(ceil_div(d, 32)), kSlices), dim3(256), 0, st,
                       w.partial, w.slices, blocks, di);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(normalise_v_kernel, dim3(1), dim3(256), 0, st, w.slices, w.mean, state, beta, v, w.flag, di,
                       1.0 / static_cast<double>(n_sub));
    return hipGetLastError();
}

}  // namespace

InitVPlan plan_init_v(int64_t n_sub, int64_t d, bool is_bf16, const LaunchCfg& cfg) {
    InitVPlan p;
    // enough blocks to stream at full rate, few enough that the float64
    // combine pass over [blocks][d] stays negligible
    int64_t blocks = static_cast<int64_t>(cfg.num_cus) * 4;
    const int64_t per_vec = is_bf16 ? 8 : 4;
    const int64_t work_items = ceil_div(n_sub * d, 64 * per_vec * 8);   // wave iterations available
    if (blocks > ceil_div(work_items, 4)) blocks = ceil_div(work_items, 4);
    if (blocks < 1) blocks = 1;
    p.blocks = static_cast<int>(blocks);
    // the fused compress + column-sum kernel runs compress's grid
    int64_t fused = ceil_div(work_items, 4);
    if (fused > cfg.max_blocks) fused = cfg.max_blocks;
    if (fused < 1) fused = 1;
    p.fused_blocks = static_cast<int>(fused);
    const int64_t rows = blocks > fused ? blocks : fused;
    // flag | mean[d] f64 | slices[kSlices][d] f64 | partial[rows][d] f32
    p.slices_off = kFlagBytes + ceil_div(static_cast<int64_t>(d) * 8, 256) * 256;
    p.partial_off = p.slices_off + ceil_div(static_cast<int64_t>(d) * 8 * kSlices, 256) * 256;
    p.ws_bytes = p.partial_off + static_cast<size_t>(rows) * static_cast<size_t>(d) * sizeof(float);
    return p;
}

hipError_t launch_update_v(const void* X, float* state, double beta, float* v, int64_t n_sub, int64_t d,
                           bool is_bf16, bool vec_ok, void* ws, const InitVPlan& plan, hipStream_t st) {
    const WsView w = ws_view(ws, plan);
    hipError_t e = is_bf16 ? colsum_any<Bf16Elem>(X, w.partial, n_sub, d, vec_ok, plan.blocks, st)
                           : colsum_any<F32Elem>(X, w.partial, n_sub, d, vec_ok, plan.blocks, st);
    if (e != hipSuccess) return e;
    return finish_v(w, plan.blocks, n_sub, d, state, beta, v, st);
}

bool fused_compress_update_ok(int64_t d, bool is_bf16, bool vec_ok) {
    return vec_ok && vec_shape_ok(d, is_bf16 ? 8 : 4);
}

hipError_t launch_compress_update(const void* X, const float* v_in, void* S, float* state, double beta, float* v_out,
                                  int64_t n_sub, int64_t d, bool is_bf16, void* ws, const InitVPlan& plan,
                                  hipStream_t st) {
    const WsView w = ws_view(ws, plan);
    const int di = static_cast<int>(d);
    hipError_t e = is_bf16 ? dispatch_compress_colsum<Bf16Elem>(static_cast<int>(d / 8), X, v_in, S, w.partial, n_sub,
                                                                di, plan.fused_blocks, st)
                           : dispatch_compress_colsum<F32Elem>(static_cast<int>(d / 4), X, v_in, S, w.partial, n_sub,
                                                               di, plan.fused_blocks, st);
    if (e != hipSuccess) return e;
    return finish_v(w, plan.fused_blocks, n_sub, d, state, beta, v_out, st);
}

}  // namespace velora
