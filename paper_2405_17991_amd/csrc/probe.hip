// Streaming probes: what this chip's memory system delivers to the simplest kernels of this library's
// own making, so that a benchmark can state each hot-path kernel's rate against a ceiling measured in
// the same run on the same box as well as against the published peak.  Not part of the method.
//   read   every 16-byte vector of the buffer is loaded once (non-temporal), one block per compute
//          unit, eight loads in flight per thread; a folded word per block goes to `sink` so that
//          the loads cannot be dropped
//   write  every 16-byte vector is stored once (non-temporal), same launch shape
//   copy   read + write of equal size
// These shapes were the fastest of those measured for each direction (more than two blocks per compute
// unit is slower for both).
#include "common.h"
#include "kernels.h"

namespace velora {

namespace {
constexpr int kU = 8;

__global__ __launch_bounds__(256) void probe_read_kernel(const u32x4* __restrict__ p, int64_t n_vec,
                                                         uint32_t* __restrict__ sink) {
    u32x4 acc = {0u, 0u, 0u, 0u};
    const int64_t stride = static_cast<int64_t>(gridDim.x) * 256;
    int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    for (; i + (kU - 1) * stride < n_vec; i += kU * stride) {
        u32x4 x[kU];
#pragma unroll
        for (int u = 0; u < kU; ++u) x[u] = __builtin_nontemporal_load(p + i + u * stride);
#pragma unroll
        for (int u = 0; u < kU; ++u) acc ^= x[u];
    }
    for (; i < n_vec; i += stride) acc ^= __builtin_nontemporal_load(p + i);
    uint32_t f = acc.x ^ acc.y ^ acc.z ^ acc.w;
    for (int m = 1; m < kWave; m <<= 1) f ^= __shfl_xor(f, m, kWave);
    if ((threadIdx.x & (kWave - 1)) == 0) atomicXor(sink + (blockIdx.x & 63), f);
}

__global__ __launch_bounds__(256) void probe_write_kernel(u32x4* __restrict__ p, int64_t n_vec, uint32_t value) {
    const u32x4 v = {value, value, value, value};
    const int64_t stride = static_cast<int64_t>(gridDim.x) * 256;
    int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    for (; i + (kU - 1) * stride < n_vec; i += kU * stride) {
#pragma unroll
        for (int u = 0; u < kU; ++u) __builtin_nontemporal_store(v, p + i + u * stride);
    }
    for (; i < n_vec; i += stride) __builtin_nontemporal_store(v, p + i);
}

__global__ __launch_bounds__(256) void probe_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst,
                                                         int64_t n_vec) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * 256;
    int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    for (; i + (kU - 1) * stride < n_vec; i += kU * stride) {
        u32x4 x[kU];
#pragma unroll
        for (int u = 0; u < kU; ++u) x[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < kU; ++u) __builtin_nontemporal_store(x[u], dst + i + u * stride);
    }
    for (; i < n_vec; i += stride) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}
}  // namespace

hipError_t launch_probe(int kind, const void* src, void* dst, int64_t bytes, uint32_t* sink, const LaunchCfg& cfg,
                        hipStream_t st) {
    const int64_t n_vec = bytes / 16;
    int64_t blocks = cfg.num_cus;
    if (blocks > ceil_div(n_vec, 256)) blocks = ceil_div(n_vec, 256);
    const dim3 grid(static_cast<unsigned>(blocks)), block(256);
    if (kind == 0)
        hipLaunchKernelGGL(probe_read_kernel, grid, block, 0, st, static_cast<const u32x4*>(src), n_vec, sink);
    else if (kind == 1)
        hipLaunchKernelGGL(probe_write_kernel, grid, block, 0, st, static_cast<u32x4*>(dst), n_vec, 0u);
    else
        hipLaunchKernelGGL(probe_copy_kernel, grid, block, 0, st, static_cast<const u32x4*>(src),
                           static_cast<u32x4*>(dst), n_vec);
    return hipGetLastError();
}

}  // namespace velora
