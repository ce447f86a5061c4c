// Forward linear layer with the compression taken from the same tiles (paper
// Algorithm 1, forward: out = input @ weight^T next to compress(group(input), v)
// of Sec. 3.2).  Y[N, O] = X[N, D] * W[O, D]^T as a bf16 MFMA GEMM whose LDS
// tiles of X also feed the dot with v, so X is read from HBM once for both.
//
// GEMM.  Block tile 256 tokens x 256 outputs x 64 k, four waves in a 2 x 2 grid
// (wave tile 128 x 128 = 8 x 8 MFMA tiles of 16 x 16, 256 accumulator
// registers).  Both operands are k-contiguous, so a 16-byte piece of a row is
// already an MFMA fragment; LDS rows are 128 bytes, eight 16-byte chunks, chunk
// c of row r stored at position c ^ ((r >> 1) & 7), which makes both the linear
// writes and the fragment reads (16 rows x one chunk) bank-conflict free.
// Two LDS stages (2 x 64 KB).  What bounds the loop is the number of cache-line
// requests a CU can have outstanding (~70 x 128 B at ~500 cycles from L2), so
// the request queue must never drain at a wait point.  Two interleaved streams:
//   X tiles: global -> LDS directly (buffer_load ... lds), issued at the middle
//            of step t for step t+2, awaited at the middle of step t+1;
//   W tiles: global -> registers, issued at the end of step t for step t+3,
//            awaited at the end of step t+1 and written to LDS there.
// At each wait the other stream's batch is still in flight (s_waitcnt vmcnt(8),
// vector-memory operations complete in order).  Fragments are double-buffered in
// registers: the LDS reads for the next 32-k half run under the 64 MFMAs of the
// current one.  No other vector-memory load may sit inside the loop, or the
// counted waits would be off; v is therefore staged in LDS before the loop.
// Block order: consecutive block ids land on different XCDs (one L2 each), so
// XCD x takes a contiguous run of tiles, 32 blocks running together covering
// 4 token tiles x 8 output tiles where the tile counts allow it.
//
// Compression inside the GEMM.  Blocks of the first output tile also form
// S[n, g] = <X[n, g*d : (g+1)*d], v>.  v is split into two bf16 parts,
// v = hi + lo (|v - hi - lo| <= 2^-17 |v|), which become rows 0 and 1 of an
// otherwise zero 16-row A operand; one extra MFMA per token tile and 32-k half
// multiplies it with the X fragments that are in registers anyway, accumulating
// in float32, and rows 0 + 1 of the result are the dot.  d must be a multiple
// of 64 (a k-step then lies inside one sub-token) and at most 2048.
//
// Everything the MFMA kernel cannot take (float32, d or D not a multiple of 64,
// unaligned pointers) goes to a plain tiled FMA kernel plus the stand-alone
// compress kernel.
#include "common.h"
#include "kernels.h"

#include <type_traits>

namespace velora {

namespace {

constexpr int kBM = 256, kBN = 256, kBK = 64;
constexpr int kRowB = kBK * 2;                    // bytes per LDS row
constexpr int kStage = (kBM + kBN) * kRowB;       // 64 KB
constexpr int kMaxFusedD = 2048;                  // v table: 2 x 2048 bf16 = 8 KB behind the stages

typedef __attribute__((address_space(3))) void* lds_ptr;

__device__ __forceinline__ lds_ptr to_lds(char* p) { return (lds_ptr)p; }

}  // namespace

// One block's tile.  DO_S: this block also forms S for its 256 tokens.
template <bool DO_S>
__device__ __forceinline__ void linear_tile(char* lds, const uint16_t* __restrict__ X, const uint16_t* __restrict__ W,
                                            const float* __restrict__ v, uint16_t* __restrict__ Y,
                                            uint16_t* __restrict__ S, int N, int O, int D, int d, int64_t n0,
                                            int64_t o0) {
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int wm = w >> 1, wn = w & 1;
    const int q = lane >> 4, jj = lane & 15;
    // Range-checked descriptors over this block's rows: rows past N (or O) read as zeros.
    const int rows_x = N - n0 < kBM ? static_cast<int>(N - n0) : kBM;
    const int rows_w = O - o0 < kBN ? static_cast<int>(O - o0) : kBN;
    __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t*>(X + n0 * D), 0, static_cast<int>(static_cast<int64_t>(rows_x) * D * 2), 0x00020000);
    __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t*>(W + o0 * D), 0, static_cast<int>(static_cast<int64_t>(rows_w) * D * 2), 0x00020000);
    // One wave instruction moves 1 KB = 8 rows x 128 B; wave w owns rows 64w .. 64w+63 of both tiles.
    // lane -> row-in-8 = lane / 8, stored chunk = lane % 8, loaded chunk = stored ^ ((row >> 1) & 7).
    uint32_t gvoff[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int row = w * 64 + i * 8 + (lane >> 3);
        const int chunk = (lane & 7) ^ ((row >> 1) & 7);
        gvoff[i] = static_cast<uint32_t>(row) * static_cast<uint32_t>(D) * 2u + static_cast<uint32_t>(chunk) * 16u;
    }
    const int nk = D / kBK;
    // steps past the end re-fetch the last k block into the (free) stage: the counted waits stay uniform
    auto dma_x = [&](int t) {
        char* st = lds + (t & 1) * kStage;
        const int koff = (t < nk ? t : nk - 1) * kBK * 2;
#pragma unroll
        for (int i = 0; i < 8; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, to_lds(st + (w * 64 + i * 8) * kRowB), 16, gvoff[i], koff, 0, 0);
    };
    auto dma_w = [&](int t) {
        char* st = lds + (t & 1) * kStage;
        const int koff = (t < nk ? t : nk - 1) * kBK * 2;
#pragma unroll
        for (int i = 0; i < 8; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, to_lds(st + (kBM + w * 64 + i * 8) * kRowB), 16, gvoff[i], koff,
                                                     0, 0);
    };
    u32x4 wreg[8];
    auto regload_w = [&](int t) {
        const int koff = (t < nk ? t : nk - 1) * kBK * 2;
#pragma unroll
        for (int i = 0; i < 8; ++i) wreg[i] = __builtin_amdgcn_raw_buffer_load_b128(rw, gvoff[i], koff, 0);
    };
    auto store_w = [&](int t) {
        char* st = lds + (t & 1) * kStage;
#pragma unroll
        for (int i = 0; i < 8; ++i)
            *reinterpret_cast<u32x4*>(st + (kBM + w * 64 + i * 8) * kRowB + lane * 16) = wreg[i];
    };
    // fragment of rows base + 16b + jj, chunk 4*kk + q; (row >> 1) & 7 == (jj >> 1) & 7 because base is a multiple of 16
    uint32_t foff[2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
        foff[kk] = static_cast<uint32_t>(jj) * kRowB + static_cast<uint32_t>(((kk * 4 + q) ^ ((jj >> 1) & 7)) * 16);
    auto fread = [&](bf16x8 (&fx)[8], bf16x8 (&fw)[8], int t, int kk) {
        const char* st = lds + (t & 1) * kStage;
#pragma unroll
        for (int b = 0; b < 8; ++b)
            fx[b] = *reinterpret_cast<const bf16x8*>(st + (wm * 128 + b * 16) * kRowB + foff[kk]);
#pragma unroll
        for (int a = 0; a < 8; ++a)
            fw[a] = *reinterpret_cast<const bf16x8*>(st + (kBM + wn * 128 + a * 16) * kRowB + foff[kk]);
    };

    // v = hi + lo as bf16, staged behind the two stages: vtab[0][j] = hi, vtab[1][j] = lo
    uint16_t* vtab = reinterpret_cast<uint16_t*>(lds + 2 * kStage);
    if constexpr (DO_S) {
        for (int j = tid; j < d; j += 256) {
            const float x = v[j];
            const uint16_t hi = f32_to_bf16(x);
            vtab[j] = hi;
            vtab[d + j] = f32_to_bf16(x - bf16_to_f32(hi));
        }
    }
    __builtin_amdgcn_s_waitcnt(0);                // no load of v is outstanding when the counted streams start
    __builtin_amdgcn_sched_barrier(0);

    f32x4 acc[8][8];                              // [output tile][token tile]
#pragma unroll
    for (int a = 0; a < 8; ++a)
#pragma unroll
        for (int b = 0; b < 8; ++b) acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};
    f32x4 acc_s[4];                               // this wave's token tiles 4*wn .. 4*wn+3
#pragma unroll
    for (int b = 0; b < 4; ++b) acc_s[b] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto mma = [&](const bf16x8 (&fx)[8], const bf16x8 (&fw)[8]) {
#pragma unroll
        for (int a = 0; a < 8; ++a)
#pragma unroll
            for (int b = 0; b < 8; ++b)
                acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fw[a], fx[b], acc[a][b], 0, 0, 0);
    };
    // A operand with v: row 0 = hi, row 1 = lo, rows 2..15 zero; k = 8q .. 8q+7 of this 32-k half
    auto v_fragment = [&](int t, int kk) -> bf16x8 {
        const int vk = (t * kBK + kk * 32) % d + q * 8;
        const u32x4 raw = *reinterpret_cast<const u32x4*>(vtab + (jj & 1) * d + vk);
        const u32x4 zero = {0u, 0u, 0u, 0u};
        return __builtin_bit_cast(bf16x8, jj < 2 ? raw : zero);
    };
    auto mma_s = [&](const bf16x8 (&fx)[8], const bf16x8& vf) {
        if (wn == 0) {
#pragma unroll
            for (int b = 0; b < 4; ++b) acc_s[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, fx[b], acc_s[b], 0, 0, 0);
        } else {
#pragma unroll
            for (int b = 0; b < 4; ++b)
                acc_s[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, fx[b + 4], acc_s[b], 0, 0, 0);
        }
    };
    // lane (jj, q = 0) holds rows 0..3 of the result for token jj: S = row 0 + row 1
    auto flush_s = [&](int g) {
        const int M = D / d;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int64_t n = n0 + wm * 128 + (wn * 4 + b) * 16 + jj;
            if (q == 0 && n < N) S[n * M + g] = f32_to_bf16(acc_s[b][0] + acc_s[b][1]);
            acc_s[b] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
    };

    constexpr int kWaitVm8 = 0x0F78;              // s_waitcnt vmcnt(8), other counters unconstrained
    constexpr int kWaitVm8Lgkm0 = 0x0078;         // s_waitcnt vmcnt(8) lgkmcnt(0)
    bf16x8 fxA[8], fwA[8], fxB[8], fwB[8];
    bf16x8 vfA = {}, vfB = {};
    dma_x(0); dma_w(0);
    dma_x(1); dma_w(1);
    regload_w(2);
    __builtin_amdgcn_s_waitcnt(kWaitVm8);        // the four direct loads have landed; W(2) may still be in flight
    __syncthreads();                              // (also publishes vtab)
    fread(fxA, fwA, 0, 0);
    if constexpr (DO_S) vfA = v_fragment(0, 0);
    for (int t = 0; t < nk; ++t) {
        fread(fxB, fwB, t, 1);
        if constexpr (DO_S) vfB = v_fragment(t, 1);
        __builtin_amdgcn_sched_barrier(0);
        mma(fxA, fwA);
        if constexpr (DO_S) mma_s(fxA, vfA);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_waitcnt(kWaitVm8Lgkm0);   // X(t+1) landed; fragments B and this wave's W(t+1) stores done
        __syncthreads();                          // stage t&1 is free, stage (t+1)&1 is complete
        dma_x(t + 2);
        if (t + 1 < nk) {
            fread(fxA, fwA, t + 1, 0);
            if constexpr (DO_S) vfA = v_fragment(t + 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        mma(fxB, fwB);
        if constexpr (DO_S) {
            mma_s(fxB, vfB);
            if (((t + 1) * kBK) % d == 0) flush_s((t * kBK) / d);
        }
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_waitcnt(kWaitVm8);    // W(t+2) is in registers; X(t+2) may still be in flight
        store_w(t + 2);                           // stage t&1: free since this step's barrier
        regload_w(t + 3);
        __builtin_amdgcn_sched_barrier(0);
    }
    __builtin_amdgcn_s_waitcnt(0);                // nothing of this block is in flight when its LDS is released

    // D[i = output 4q + r][j = token jj] per tile: four consecutive outputs of one token per lane
#pragma unroll
    for (int a = 0; a < 8; ++a)
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const int64_t n = n0 + wm * 128 + b * 16 + jj, o = o0 + wn * 128 + a * 16 + q * 4;
            if (n < N && o < O) {   // O % 4 == 0: a lane's four outputs are all inside or all outside
                const u32x2 out = {pack_bf16x2(acc[a][b][0], acc[a][b][1]), pack_bf16x2(acc[a][b][2], acc[a][b][3])};
                *reinterpret_cast<u32x2*>(Y + n * O + o) = out;
            }
        }
}

template <bool FUSE>
__global__ __launch_bounds__(256) void linear_compress_mfma_kernel(const uint16_t* __restrict__ X,
                                                                  const uint16_t* __restrict__ W,
                                                                  const float* __restrict__ v,
                                                                  uint16_t* __restrict__ Y, uint16_t* __restrict__ S,
                                                                  int N, int O, int D, int d) {
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    const int To = (O + kBN - 1) / kBN, Tn = (N + kBM - 1) / kBM, T = To * Tn;
    const int per_xcd = (T + 7) / 8;
    const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3;
    const int vid = xcd * per_xcd + idx;
    if (idx >= per_xcd || vid >= T) return;       // whole block, before any barrier
    int tn = vid / To, to = vid % To;
    if (To % 8 == 0 && per_xcd % (4 * To) == 0) {
        const int band = idx / (4 * To), r = idx % (4 * To), panel = r / 32, within = r % 32;
        to = panel * 8 + within % 8;
        tn = xcd * (per_xcd / To) + band * 4 + within / 8;
    }
    const int64_t n0 = static_cast<int64_t>(tn) * kBM, o0 = static_cast<int64_t>(to) * kBN;
    if (FUSE && to == 0) linear_tile<true>(lds, X, W, v, Y, S, N, O, D, d, n0, o0);
    else linear_tile<false>(lds, X, W, v, Y, S, N, O, D, d, n0, o0);
}

// Any dtype, size and alignment: 64 x 64 output tile per block, 16-k slices through LDS, a 4 x 4 patch
// per thread, float32 FMA.  Not tuned; it exists so that every shape has a result.
template <typename E>
__global__ __launch_bounds__(256) void linear_generic_kernel(const typename E::type* __restrict__ X,
                                                            const typename E::type* __restrict__ W,
                                                            typename E::type* __restrict__ Y, int64_t N, int64_t O,
                                                            int64_t D) {
    __shared__ float xs[16][64 + 1], ws[16][64 + 1];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int64_t n0 = static_cast<int64_t>(blockIdx.x) * 64, o0 = static_cast<int64_t>(blockIdx.y) * 64;
    float acc[4][4] = {};
    for (int64_t k0 = 0; k0 < D; k0 += 16) {
        for (int i = threadIdx.x; i < 64 * 16; i += 256) {
            const int r = i >> 4, k = i & 15;
            const bool kin = k0 + k < D;
            xs[k][r] = (kin && n0 + r < N) ? E::load(X, (n0 + r) * D + k0 + k) : 0.f;
            ws[k][r] = (kin && o0 + r < O) ? E::load(W, (o0 + r) * D + k0 + k) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            float xv[4], wv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { xv[i] = xs[k][ty * 4 + i]; wv[i] = ws[k][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(xv[i], wv[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t n = n0 + ty * 4 + i, o = o0 + tx * 4 + j;
            if (n < N && o < O) E::store(Y, n * O + o, acc[i][j]);
        }
}

bool linear_mfma_ok(int64_t N, int64_t D, int64_t O, bool is_bf16, bool align16) {
    // 32-bit tile counts and byte offsets inside a 256-row tile; 8-byte Y stores
    return is_bf16 && align16 && D % kBK == 0 && O % 4 == 0 && D <= (1 << 21) && N < (int64_t{1} << 31) - kBM &&
           O < (int64_t{1} << 31) - kBN && ((N + kBM - 1) / kBM) * ((O + kBN - 1) / kBN) < (int64_t{1} << 28);
}

bool linear_fused_s_ok(int64_t d) { return d % kBK == 0 && d <= kMaxFusedD; }

hipError_t launch_linear_compress(const void* X, const void* W, const float* v, void* Y, void* S, int64_t N, int64_t D,
                                  int64_t O, int64_t M, bool is_bf16, bool align16, bool s_vec_ok, const LaunchCfg& cfg,
                                  hipStream_t st) {
    const int64_t d = D / M;
    if (linear_mfma_ok(N, D, O, is_bf16, align16)) {
        const bool fuse = linear_fused_s_ok(d);
        const int64_t tiles = ((N + kBM - 1) / kBM) * ((O + kBN - 1) / kBN);
        const unsigned grid = static_cast<unsigned>((tiles + 7) / 8 * 8);
        const size_t lds_bytes = 2 * static_cast<size_t>(kStage) + (fuse ? 2 * static_cast<size_t>(d) * 2 : 0);
        hipError_t e;
        if (fuse) {
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&linear_compress_mfma_kernel<true>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds_bytes));
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL(linear_compress_mfma_kernel<true>, dim3(grid), dim3(256), lds_bytes, st,
                               static_cast<const uint16_t*>(X), static_cast<const uint16_t*>(W), v,
                               static_cast<uint16_t*>(Y), static_cast<uint16_t*>(S), static_cast<int>(N),
                               static_cast<int>(O), static_cast<int>(D), static_cast<int>(d));
            return hipGetLastError();
        }
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&linear_compress_mfma_kernel<false>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds_bytes));
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(linear_compress_mfma_kernel<false>, dim3(grid), dim3(256), lds_bytes, st,
                           static_cast<const uint16_t*>(X), static_cast<const uint16_t*>(W), v,
                           static_cast<uint16_t*>(Y), static_cast<uint16_t*>(S), static_cast<int>(N),
                           static_cast<int>(O), static_cast<int>(D), static_cast<int>(d));
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        return launch_compress(X, v, S, N * M, d, true, s_vec_ok, cfg, st);
    }
    const dim3 grid(static_cast<unsigned>((N + 63) / 64), static_cast<unsigned>((O + 63) / 64));   // O <= 65535 * 64: caller
    if (is_bf16)
        hipLaunchKernelGGL(linear_generic_kernel<Bf16Elem>, grid, dim3(256), 0, st, static_cast<const uint16_t*>(X),
                           static_cast<const uint16_t*>(W), static_cast<uint16_t*>(Y), N, O, D);
    else
        hipLaunchKernelGGL(linear_generic_kernel<F32Elem>, grid, dim3(256), 0, st, static_cast<const float*>(X),
                           static_cast<const float*>(W), static_cast<float*>(Y), N, O, D);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_compress(X, v, S, N * M, d, is_bf16, s_vec_ok, cfg, st);
}

}  // namespace velora
