// Weight gradient from compressed activations (paper Listing 1, backward:
// grad_weight = grad_output^T @ ungroup(reconstruct(z, v))).
//
// Because the reconstructed input is Xhat[n, g*d + j] = S[n, g] * v[j]
// (Sec. 3.1), the gradient factors exactly:
//     T[o, g]        = sum_n G[n, o] * S[n, g]            (a skinny GEMM, K = N)
//     dW[o, g*d + j] = T[o, g] * v[j]                     (an expansion)
// which needs d times fewer flops than the dense product and never forms Xhat.
// The work is then bound by reading G once and writing dW once, so:
//   kernel 1 streams G exactly once, forms partial T over fixed token ranges
//            (split-K, because T alone is far too small to fill 256 CUs) with
//            bf16 MFMA, and writes the partials to the workspace;
//   kernel 2 sums the partials in a fixed order (deterministic, no float
//            atomics), multiplies by v and streams dW out with 16-byte stores.
//
// Kernels in this file, by the number of 16-group tiles ceil(M / 16) a block covers:
//   wgrad_partial_mfma_kernel      1 tile; 5-6 tiles when the blocks need several rounds; 8-byte G loads;
//                                  S that is not 16-byte aligned or has an odd element count
//   wgrad_partial_ws_kernel        2-3 tiles: loader waves + computing waves, 128-token chunks through LDS
//   wgrad_partial_ws256_kernel     1-3 tiles on more than 5376, 4-5 tiles on more than 8192 output features: the same
//                                  on 256-feature tiles
//   wgrad_partial_ws64_kernel      4 tiles, and 5-6 when every block is resident at once: 64-token chunks
//   wgrad_partial_shared_g_kernel  8, 12, 16 tiles (M up to 256; larger M in chunks of 256)
//   wgrad_partial_f32_mfma_kernel  float32 inputs (O a multiple of 4, 16-byte aligned G)
//   wgrad_partial_simple_kernel    whatever the MFMA kernels cannot take
//   wgrad_pack_s_kernel            S as ready-made MFMA fragments, for the kernels that read S that way
//   wgrad_expand_kernel            float32 dW rows below 32 KB, and what the sweep cannot take: one block per row
//   wgrad_expand_sweep_kernel      longer float32 rows and bf16 output: one sweep of the whole grid over dW
//   wgrad_reduce_kernel            dense T[O, M] for the factored hand-off
#include "common.h"
#include "kernels.h"

#include <atomic>
#ifdef VELORA_TUNING
#include <cstdlib>
#endif

namespace velora {


// ---------------------------------------------------------------------------
// Kernel 1, MFMA path (bf16 inputs).
//
// v_mfma_f32_16x16x32_bf16 computes D[16x16] += A[16x32] * B[32x16]; lane l
// supplies A[l%16][8*(l/16) + 0..7] and B[8*(l/16) + 0..7][l%16] (eight
// K-consecutive bf16 in four VGPRs) and receives D[4*(l/16) + 0..3][l%16].
// Here K runs over tokens n, A rows over sub-token groups g, B columns over
// output features o.  Both operands are stored with n as the SLOW axis
// (G[n][o], S[n][g]), so the eight K-consecutive values a lane needs sit in
// eight different rows.
//
// G (the big operand, read exactly once from HBM): a lane loads eight rows x
// CW columns (CW*2 bytes per row, coalesced across the 16 lanes that share a
// K-group) and transposes the 8 x CW block of 16-bit values inside its own
// registers with v_perm_b32, which yields CW ready B fragments for CW
// different columns.  The column a lane/fragment pair stands for is strided
// (o = o0 + jj*CW + c); MFMA columns need not be adjacent in memory and the
// epilogue undoes the mapping.  No LDS is involved, so loads can be issued
// ahead into a register ring (NST stages).  One stage is what is used: a CU
// sustains a bounded number of outstanding cache-line requests (about 80), which
// four waves with one 32-token step each already exceed, and deeper rings
// measured slower on every layer shape.
//
// S (small, re-read by every column tile).  Up to three group tiles (DIRECT):
// lane (jj, q) gathers its eight values S[8q + e][16*tile + jj] with 2-byte
// loads and pairs them up in registers.  More tiles: a tiny pre-pass re-lays S
// out as ready-made A fragments (pack kernel below), so the main loop fetches
// one 16-byte fragment per lane and 16-group tile with no transposition at all.
//
//   CW   G columns per lane (8 -> 16-byte loads, 4 -> 8-byte)
//   GT   16-group tiles per block (the block covers 16*GT groups g)
//   NST  ring depth: 32-token steps loaded ahead per wave
//   DIRECT  S operand is S[N, M] itself rather than the packed fragments
// Block = 4 waves; the waves take alternate 32-token steps of the block's token
// range and are summed through LDS at the end in a fixed order.
// grid = (o tiles of 16*CW, splits, g chunks of 16*GT)
// ---------------------------------------------------------------------------
#ifndef VELORA_SKIP
#define VELORA_SKIP 0            // measurement builds only: 1 no S loads, 2 no transposes / MFMAs, 4 no cross-wave sum
#endif
constexpr int kStep = 32;        // tokens per MFMA K-step
constexpr int kWavesPerBlock = 4;

// Packed S: for every 32-token step and 16-group tile, the 64 lanes' A
// fragments back to back (1 KiB): entry [(step*tiles + tile)*64 + lane] holds
// S[step*32 + 8*(lane/16) + 0..7][tile*16 + lane%16], zero outside S.
__global__ __launch_bounds__(256) void wgrad_pack_s_kernel(const uint16_t* __restrict__ S, uint4* __restrict__ packed,
                                                          int64_t N, int64_t M, int64_t tiles, int64_t total) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int lane = static_cast<int>(i & 63);
    const int64_t st = i >> 6;
    const int64_t step = st / tiles;
    const int64_t tile = st - step * tiles;
    const int64_t g = tile * 16 + (lane & 15);
    const int64_t n0 = step * kStep + (lane >> 4) * 8;
    uint32_t h[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int64_t n = n0 + e;
        h[e] = (g < M && n < N) ? static_cast<uint32_t>(S[n * M + g]) : 0u;
    }
    packed[i] = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
}

// cache-policy operand of the buffer loads that stream G: bit 1 = non-temporal
// (the data is read exactly once)
constexpr int kStreamAux = 2;

// CW consecutive bf16 through a buffer descriptor (wave-uniform base in SGPRs,
// 32-bit per-lane byte offset).  A raw buffer load whose offset is not below
// the descriptor's size returns zero without touching memory; the kernel uses
// that for every edge (rows past the token range, columns past O, steps past
// the end) instead of branching.
template <int CW, int AUX>
__device__ __forceinline__ RawRow<CW / 2> load_g(const __amdgpu_buffer_rsrc_t& rsrc, uint32_t voff) {
    RawRow<CW / 2> r;
    if constexpr (CW == 8) {
        const u32x4 q = __builtin_amdgcn_raw_buffer_load_b128(rsrc, voff, 0, AUX);
        r.w[0] = q.x; r.w[1] = q.y; r.w[2] = q.z; r.w[3] = q.w;
    } else {
        const u32x2 q = __builtin_amdgcn_raw_buffer_load_b64(rsrc, voff, 0, AUX);
        r.w[0] = q.x; r.w[1] = q.y;
    }
    return r;
}

// One 32-token step in flight.  S is either a ready fragment per tile (packed
// path) or eight 16-bit values per tile still to be paired up (direct path).
template <int CW, int GT, bool DIRECT>
struct WgradStage {
    RawRow<CW / 2> g[8];
    uint32_t s[GT][DIRECT ? 8 : 4];
};

// One MFMA result tile leaves the registers as it is: lane (jj, q) holds
// T[g0 + 4q + r][o0 + jj*CW + c], r < 4, and partial rows run along g, so the
// four values are one 16-byte store (Mp is a multiple of 4 and the workspace is
// 16-byte aligned; groups in [M, Mp) hold zeros).
template <int CW>
__device__ __forceinline__ void store_tile(float* __restrict__ out, const f32x4& t, int64_t o0, int jj, int q, int c,
                                           int64_t g0, int64_t O, int64_t Mp) {
    const int64_t o = o0 + jj * CW + c;
    const int64_t g = g0 + 4 * q;
    if (o < O && g < Mp) *reinterpret_cast<f32x4*>(out + o * Mp + g) = t;
}

// Which tokens a block sums over.  The token axis is cut into chunks of 128 (four waves x one 32-token
// step).  `chunk_stride` = 128: the block owns the contiguous range [split * rows_per_split, ...);
// `chunk_stride` = splits * 128: chunks are dealt to the splits round-robin, block `split` takes chunks
// split, split + splits, ...  Then all blocks of the grid walk through G together, window by window, and
// every row of G is fetched by its column tiles at about the same time, which DRAM serves faster than
// `splits` separate sweeps that are megabytes apart (measured on the 16384 x 4096 layer, loads only:
// 21.0 us against 22.4 us).  Either way the order of the summation depends on the sizes alone.
template <int CW, int GT, int NST, bool DIRECT>
__global__ __launch_bounds__(256) void wgrad_partial_mfma_kernel(const uint16_t* __restrict__ G,
                                                                const void* __restrict__ Sany,
                                                                float* __restrict__ partial, int64_t N, int64_t O,
                                                                int64_t M, int64_t Mp, int64_t rows_per_split,
                                                                int64_t tiles_packed, int cyclic) {
    constexpr int OT = 16 * CW;          // output features per block
    constexpr int NACC = GT * CW;        // accumulator tiles per wave
    constexpr int TP = NACC <= 24 ? NACC : (NACC % 24 == 0 ? 24 : 16);   // tiles reduced per pass: 2 regions x <= 24 KB of LDS
    constexpr int kChunk = kStep * kWavesPerBlock;
    __shared__ f32x4 red[2][TP][kWave];

    const int lane = threadIdx.x & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int q = lane >> 4;
    const int jj = lane & 15;
    const int64_t o0 = static_cast<int64_t>(blockIdx.x) * OT;
    const int split = blockIdx.y;
    const int splits = gridDim.y;
    const int64_t tile0 = static_cast<int64_t>(blockIdx.z) * GT;
    // first row, rows from there to the end of what this block may read, chunks it owns, rows between them
    int64_t row0, span_rows;
    int n_chunks;
    uint32_t chunk_stride;
    if (cyclic) {
        const int64_t total_chunks = ceil_div(N, kChunk);
        row0 = static_cast<int64_t>(split) * kChunk;
        span_rows = N - row0;
        n_chunks = static_cast<int>((total_chunks - split + splits - 1) / splits);
        chunk_stride = static_cast<uint32_t>(splits) * kChunk;
    } else {
        row0 = static_cast<int64_t>(split) * rows_per_split;
        span_rows = N - row0 < rows_per_split ? N - row0 : rows_per_split;
        n_chunks = static_cast<int>(ceil_div(span_rows, kChunk));
        chunk_stride = kChunk;
    }
    const bool col_ok = o0 + jj * CW < O;

    // One buffer descriptor per operand for the whole life of the block (rebuilding it for every step
    // measured 2.6 us slower on the 16384 x 4096 layer than adding the step's offset per lane).  A raw
    // buffer load whose offset is not below the descriptor's size returns zero without touching memory;
    // every edge uses that instead of a branch: rows past the end, columns past O (lane offset
    // 0x7FFFFFFF) and steps past the block's last chunk (step offset 0x80000000); sizes stay below 2^31
    // (checked on the host), so no sum of a lane and a step offset wraps around.
    constexpr uint32_t kLaneOut = 0x7FFFFFFFu, kStepOut = 0x80000000u;
    const uint32_t row_bytes = static_cast<uint32_t>(O) * 2u;
    uint32_t voff[8];
#pragma unroll
    for (int r = 0; r < 8; ++r)
        voff[r] = col_ok ? static_cast<uint32_t>(q * 8 + r) * row_bytes + static_cast<uint32_t>(jj * CW * 2) : kLaneOut;
    const __amdgpu_buffer_rsrc_t g_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<char*>(reinterpret_cast<const char*>(G) + (row0 * O + o0) * 2), 0,
        static_cast<int>(static_cast<uint32_t>(span_rows) * row_bytes - static_cast<uint32_t>(o0 * 2)), 0x00020000);
    // S of this block.  Direct path (few group tiles): S[N, M] itself, lane (jj, q) gathers
    // S[8q + e][16*tile + jj], e < 8, as eight 2-byte loads per tile.  Packed path: the fragment array,
    // entry (32-token step, tile), 1 KiB each.
    const uint32_t s_row_bytes = DIRECT ? static_cast<uint32_t>(M) * 2u : static_cast<uint32_t>(tiles_packed) * (1024u / kStep);
    const char* sbase = DIRECT ? reinterpret_cast<const char*>(Sany) + row0 * M * 2
                               : reinterpret_cast<const char*>(Sany) + ((row0 / kStep) * tiles_packed + tile0) * 1024;
    const int64_t span_steps = ceil_div(span_rows, kStep);
    const uint32_t s_bytes = DIRECT ? static_cast<uint32_t>(span_rows) * static_cast<uint32_t>(M) * 2u
                                    : static_cast<uint32_t>(span_steps * tiles_packed - tile0) * 1024u;
    const __amdgpu_buffer_rsrc_t s_rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(sbase), 0, static_cast<int>(s_bytes), 0x00020000);
    uint32_t s_voff[GT][DIRECT ? 8 : 1];
#pragma unroll
    for (int a = 0; a < GT; ++a) {
        if constexpr (DIRECT) {
            const int64_t g = (tile0 + a) * 16 + jj;
#pragma unroll
            for (int e = 0; e < 8; ++e)
                s_voff[a][e] = g < M ? (static_cast<uint32_t>(q * 8 + e) * static_cast<uint32_t>(M) + static_cast<uint32_t>(g)) * 2u
                                     : kLaneOut;
        } else {
            // tiles past the last real one are not in the array
            s_voff[a][0] = tile0 + a < tiles_packed ? static_cast<uint32_t>(lane) * 16u + a * 1024u : kLaneOut;
        }
    }

    f32x4 acc[GT][CW];
#pragma unroll
    for (int a = 0; a < GT; ++a)
#pragma unroll
        for (int c = 0; c < CW; ++c) acc[a][c] = f32x4{0.f, 0.f, 0.f, 0.f};

    WgradStage<CW, GT, DIRECT> st[NST];
    // first row of this wave's step in chunk i, relative to row0 (a multiple of 32)
    auto step_row = [&](int i) -> uint32_t { return static_cast<uint32_t>(i) * chunk_stride + static_cast<uint32_t>(w * kStep); };
    auto load_g_step = [&](WgradStage<CW, GT, DIRECT>& sg, int i) {
        const uint32_t off = i < n_chunks ? step_row(i) * row_bytes : kStepOut;
#pragma unroll
        for (int r = 0; r < 8; ++r) sg.g[r] = load_g<CW, kStreamAux>(g_rsrc, voff[r] + off);
    };
    auto load_s_step = [&](WgradStage<CW, GT, DIRECT>& sg, int i) {
        const uint32_t off = i < n_chunks ? step_row(i) * s_row_bytes : kStepOut;
        if constexpr (DIRECT) {
#pragma unroll
            for (int a = 0; a < GT; ++a)
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    sg.s[a][e] = static_cast<uint32_t>(__builtin_amdgcn_raw_buffer_load_b16(s_rsrc, s_voff[a][e] + off, 0, 0));
        } else {
#pragma unroll
            for (int a = 0; a < GT; ++a) {
                const u32x4 x = __builtin_amdgcn_raw_buffer_load_b128(s_rsrc, s_voff[a][0] + off, 0, 0);
                sg.s[a][0] = x.x; sg.s[a][1] = x.y; sg.s[a][2] = x.z; sg.s[a][3] = x.w;
            }
        }
    };
    auto s_fragment = [&](const WgradStage<CW, GT, DIRECT>& sg, int a) -> bf16x8 {
        uint4 f;
        if constexpr (DIRECT) {
            f = make_uint4(__builtin_amdgcn_perm(sg.s[a][1], sg.s[a][0], 0x05040100u),
                           __builtin_amdgcn_perm(sg.s[a][3], sg.s[a][2], 0x05040100u),
                           __builtin_amdgcn_perm(sg.s[a][5], sg.s[a][4], 0x05040100u),
                           __builtin_amdgcn_perm(sg.s[a][7], sg.s[a][6], 0x05040100u));
        } else {
            f = make_uint4(sg.s[a][0], sg.s[a][1], sg.s[a][2], sg.s[a][3]);
        }
        return __builtin_bit_cast(bf16x8, f);
    };

    // Register ring: NST steps of this wave are in flight.  Loads return in the order they were
    // issued, S first (it comes from L2), then G.  A trip waits for its step, turns the raw
    // registers into MFMA operands, re-issues both loads for the step NST chunks ahead into the
    // registers it has just freed, and only then runs the MFMAs, so that the wave always has at
    // least NST - 1 whole steps on their way while it computes.  Steps past the last chunk load
    // zeros, which keeps the loop free of branches.
#pragma unroll
    for (int s = 0; s < NST; ++s) {
        load_s_step(st[s], s);
        load_g_step(st[s], s);
    }
    for (int i = 0; i < n_chunks; i += NST) {
#pragma unroll
        for (int s = 0; s < NST; ++s) {
            bf16x8 gf[CW], sf[GT];
#if VELORA_SKIP & 2
            {
                uint32_t x = 0;
#pragma unroll
                for (int r = 0; r < 8; ++r)
#pragma unroll
                    for (int k = 0; k < CW / 2; ++k) x ^= st[s].g[r].w[k];
                acc[0][0][0] += __uint_as_float(x & 0x3fffffffu);
            }
#pragma unroll
            for (int c = 0; c < CW; ++c) gf[c] = bf16x8{};
#else
#pragma unroll
            for (int c = 0; c < CW; ++c) gf[c] = column_fragment(st[s].g, c);
#endif
#pragma unroll
            for (int a = 0; a < GT; ++a) sf[a] = s_fragment(st[s], a);
            __builtin_amdgcn_sched_barrier(0);
            if (!(VELORA_SKIP & 1)) load_s_step(st[s], i + s + NST);
            load_g_step(st[s], i + s + NST);
            __builtin_amdgcn_sched_barrier(0);
#if !(VELORA_SKIP & 2)
#pragma unroll
            for (int a = 0; a < GT; ++a)
#pragma unroll
                for (int c = 0; c < CW; ++c)
                    acc[a][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(sf[a], gf[c], acc[a][c], 0, 0, 0);
#endif
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#if VELORA_SKIP & 4
    // measurement only: no barrier is reached by anyone; wave 0 stores its own sums
    if (w == 0) {
        float* o_ = partial + static_cast<int64_t>(split) * O * Mp;
#pragma unroll
        for (int a = 0; a < GT; ++a)
#pragma unroll
            for (int c = 0; c < CW; ++c) store_tile<CW>(o_, acc[a][c], o0, jj, q, c, (tile0 + a) * 16, O, Mp);
    }
    return;
#endif

    // Sum the four waves in a fixed order, (w0 + w1) + (w2 + w3), through LDS in the accumulators' own
    // register layout (16-byte LDS accesses, no transpose): waves 1 and 3 publish, waves 0 and 2 add.
    // Then wave 2 publishes the first half of its sums and wave 0 the second half of its own, each adds
    // what the other published (the same two numbers either way round, so every tile is
    // (w0 + w1) + (w2 + w3) bit for bit) and stores its half of the block's partial tile straight from
    // its registers: the stores of the tile, which end the block, come from two waves at once.
    float* out = partial + static_cast<int64_t>(split) * O * Mp;
#pragma unroll
    for (int p0 = 0; p0 < NACC; p0 += TP) {
        constexpr int H = (TP + 1) / 2;                       // tiles of a pass finished by wave 0; wave 2 takes the rest
        if (w == 1 || w == 3) {
#pragma unroll
            for (int i = 0; i < TP; ++i)
                if (p0 + i < NACC) red[w >> 1][i][lane] = acc[(p0 + i) / CW][(p0 + i) % CW];
        }
        __syncthreads();
        if (w == 0 || w == 2) {
#pragma unroll
            for (int i = 0; i < TP; ++i)
                if (p0 + i < NACC) acc[(p0 + i) / CW][(p0 + i) % CW] += red[w >> 1][i][lane];
            // wave 2 hands over tiles [0, H), wave 0 tiles [H, TP), each in the region it has just read
#pragma unroll
            for (int i = 0; i < TP; ++i)
                if (p0 + i < NACC && (w == 2) == (i < H)) red[w >> 1][i][lane] = acc[(p0 + i) / CW][(p0 + i) % CW];
        }
        __syncthreads();
        if (w == 0 || w == 2) {
#pragma unroll
            for (int i = 0; i < TP; ++i)
                if (p0 + i < NACC && (w == 0) == (i < H)) {
                    const int a = (p0 + i) / CW, c = (p0 + i) % CW;
                    const f32x4 other = red[w == 0 ? 1 : 0][i][lane];
                    const f32x4 t = w == 0 ? acc[a][c] + other : other + acc[a][c];
                    store_tile<CW>(out, t, o0, jj, q, c, (tile0 + a) * 16, O, Mp);
                }
        }
        if (p0 + TP < NACC) __syncthreads();   // the next pass overwrites both regions
    }
}

// ---------------------------------------------------------------------------
// Kernel 1, MFMA path with loader waves (up to three group tiles, 16-byte aligned G and S).
//
// The per-wave kernel above makes every wave do everything in turn: wait for its loads, transpose,
// issue the next loads, run the MFMAs.  While a wave transposes and multiplies it requests nothing,
// and with the whole accumulator tile in its registers only one such wave fits on a SIMD, so the
// memory pipe drains at every step (the same kernel with the arithmetic taken out streams G 5 us
// faster on N = 16384, O = 4096, M = 43).  Here the two jobs belong to different waves of one block:
//   waves 0-3  only load: G tiles (32 tokens x 128 features each) and the S rows of the same tokens go
//              straight from memory into an LDS ring (buffer loads with the LDS bit: no registers, no
//              waiting for one's own arithmetic); a lane whose offset lies outside the descriptor
//              writes zeros, so edges need no branches here either;
//   waves 4-7  only compute: each takes one 32-token step of every 128-token chunk out of LDS (eight
//              16-byte reads per lane for G, eight 2-byte reads per group tile for S), transposes it
//              in registers exactly as above and runs the MFMAs; they issue no memory loads at all.
// One barrier per chunk hands a filled slot to the computing waves and an emptied one back to the
// loaders; the ring has three slots, so the loaders are always one to two chunks (43-88 KB per
// compute unit) ahead.  Every wave executes every barrier, whatever its role, and the trip count is the
// same for all waves of a block.  The cross-wave sum and the stores at the end are those of the
// per-wave kernel, done by waves 4-7 in the ring's memory.
// Dynamic LDS: 3 x (32 KB + GT x 4 KB) + 16 bytes.  grid = (o tiles of 128, splits, 1).
// ---------------------------------------------------------------------------
constexpr int kWsSlots = 3;
constexpr int kWsGroupRows = kStep * kWavesPerBlock;                  // 128 tokens per chunk
constexpr int kWsGBytes = kWsGroupRows * 256;                         // one chunk of a 128-feature stripe
constexpr size_t ws_kernel_lds_bytes(int gt) { return static_cast<size_t>(kWsSlots) * (kWsGBytes + gt * 4096) + 16; }

typedef __attribute__((address_space(3))) void* lds_void_ptr;

// Token (0..31 inside a 32-token step) of K slot (q, e) of the MFMA operands.  Any one-to-one choice is
// valid as long as G and S agree; it decides which LDS banks a 2-byte read of S hits.  Such a read is
// served half a wave at a time, i.e. lane groups q = 0, 1 together and q = 2, 3 together, 16 lanes x 2
// bytes = 8 banks each; the two groups' rows of S are dq tokens = dq * 2M bytes apart, and they collide
// when that is close to a multiple of 128 bytes (M = 32, 48, 80 with dq = 8).  The four maps put the
// pair dq = 8, 1, 2 or 4 tokens apart; the host picks the one whose distance is nearest to 64 bytes
// mod 128 (measured at M = 80, O = 5120: 37.5 us with dq = 8, 35.4 us with dq = 2).  A power-of-two
// M >= 64 collides under every map.
__host__ __device__ constexpr int token_of_slot(int mode, int q, int e) {
    switch (mode) {
        case 1: return q + 4 * e;
        case 2: return 2 * (q & 1) + (q >> 1) + 4 * e;
        case 3: return 4 * (q & 1) + (q >> 1) + 2 * (e & 1) + 8 * (e >> 1);
        default: return 8 * q + e;
    }
}
// Every map has the form token(q, 0) + (e & 1) * s1 + (e >> 1) * s2 with s1, s2 the same for all lanes, so a
// kernel short of registers can keep one per-lane base and eight wave-uniform offsets instead of eight
// per-lane addresses.
constexpr bool token_maps_are_affine() {
    for (int mode = 0; mode < 4; ++mode) {
        const int s1 = token_of_slot(mode, 0, 1) - token_of_slot(mode, 0, 0);
        const int s2 = token_of_slot(mode, 0, 2) - token_of_slot(mode, 0, 0);
        for (int q = 0; q < 4; ++q)
            for (int e = 0; e < 8; ++e)
                if (token_of_slot(mode, q, e) != token_of_slot(mode, q, 0) + (e & 1) * s1 + (e >> 1) * s2) return false;
    }
    return true;
}
static_assert(token_maps_are_affine(), "token_of_slot: base per lane + uniform offsets");

template <int GT>
__global__ __launch_bounds__(512) void wgrad_partial_ws_kernel(const uint16_t* __restrict__ G,
                                                              const uint16_t* __restrict__ S,
                                                              float* __restrict__ partial, int64_t N, int64_t O,
                                                              int64_t M, int64_t Mp, int64_t rows_per_split,
                                                              int cyclic, int tau_mode) {
    constexpr int CW = 8, OT = 128;
    constexpr int NACC = GT * CW;
    constexpr int TP = NACC;                              // <= 24 tiles: one pass of the cross-wave sum
    constexpr int kSBytes = GT * 4096;                    // S rows of one chunk: 128 tokens x M x 2 bytes <= this
    constexpr int kSlotBytes = kWsGBytes + kSBytes;
    constexpr int kLoadsPerChunk = 8 + GT;                // per loader wave: 8 of G, GT of S
    extern __shared__ __attribute__((aligned(1024))) char lds[];

    const int lane = threadIdx.x & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const bool loader = w < kWavesPerBlock;
    const int mw = w - kWavesPerBlock;                    // computing wave: which 32-token step of a chunk
    const int q = lane >> 4;
    const int jj = lane & 15;
    const int64_t o0 = static_cast<int64_t>(blockIdx.x) * OT;
    const int split = blockIdx.y;
    const int splits = gridDim.y;
    int64_t row0, span_rows;
    int n_chunks;
    uint32_t chunk_stride;
    if (cyclic) {
        const int64_t total_chunks = ceil_div(N, kWsGroupRows);
        row0 = static_cast<int64_t>(split) * kWsGroupRows;
        span_rows = N - row0;
        n_chunks = static_cast<int>((total_chunks - split + splits - 1) / splits);
        chunk_stride = static_cast<uint32_t>(splits) * kWsGroupRows;
    } else {
        row0 = static_cast<int64_t>(split) * rows_per_split;
        span_rows = N - row0 < rows_per_split ? N - row0 : rows_per_split;
        n_chunks = static_cast<int>(ceil_div(span_rows, kWsGroupRows));
        chunk_stride = kWsGroupRows;
    }
    constexpr uint32_t kLaneOut = 0x7FFFFFFFu, kStepOut = 0x80000000u;
    const uint32_t row_bytes = static_cast<uint32_t>(O) * 2u;
    const uint32_t s_row_bytes = static_cast<uint32_t>(M) * 2u;

    // ---- loader state: lane (lr = lane / 16, piece = lane % 16) fetches 16 bytes of row 32*w + 4*r + lr
    const bool col_ok = o0 + jj * CW < O;
    const uint32_t voff_g0 =
        col_ok ? static_cast<uint32_t>(32 * (w & 3) + q) * row_bytes + static_cast<uint32_t>(jj * 16) : kLaneOut;
    const uint32_t voff_gstep = col_ok ? 4u * row_bytes : 0u;     // from one of the eight loads to the next
    const __amdgpu_buffer_rsrc_t g_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<char*>(reinterpret_cast<const char*>(G) + (row0 * O + o0) * 2), 0,
        static_cast<int>(static_cast<uint32_t>(span_rows) * row_bytes - static_cast<uint32_t>(o0 * 2)), 0x00020000);
    const __amdgpu_buffer_rsrc_t s_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<char*>(reinterpret_cast<const char*>(S) + row0 * M * 2), 0,
        static_cast<int>(static_cast<uint32_t>(span_rows) * s_row_bytes), 0x00020000);
    auto issue_chunk = [&](int i) {
        char* slot = lds + (i % kWsSlots) * kSlotBytes;
        const bool real = i < n_chunks;
        const uint32_t g_off = real ? static_cast<uint32_t>(i) * chunk_stride * row_bytes : kStepOut;
        const uint32_t s_off = real ? static_cast<uint32_t>(i) * chunk_stride * s_row_bytes : kStepOut;
#pragma unroll
        for (int r = 0; r < 8; ++r)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(g_rsrc, (lds_void_ptr)(slot + (32 * (w & 3) + 4 * r) * 256), 16,
                                                     voff_g0 + r * voff_gstep + g_off, 0, 0, kStreamAux);
        // the chunk's S rows are one contiguous run of 128 * M * 2 bytes; KB j of it goes to loader wave j % 4
#pragma unroll
        for (int t = 0; t < GT; ++t) {
            const uint32_t kb = static_cast<uint32_t>((w & 3) + 4 * t);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(s_rsrc, (lds_void_ptr)(slot + kWsGBytes + kb * 1024), 16,
                                                     kb * 1024u + static_cast<uint32_t>(lane) * 16u + s_off, 0, 0, 0);
        }
    };

    // ---- computing state
    f32x4 acc[GT][CW];
#pragma unroll
    for (int a = 0; a < GT; ++a)
#pragma unroll
        for (int c = 0; c < CW; ++c) acc[a][c] = f32x4{0.f, 0.f, 0.f, 0.f};
    // byte offsets inside a slot: this lane's first G row (the other seven are 256 bytes apart) and its S
    // value of token 8q + e, group jj (tile a: + 32 a bytes).  A lane whose group lies past M in the last
    // tile reads some other token's value there and replaces it by zero afterwards.
    const int zero_off = kWsSlots * kSlotBytes;
    int g_lds[8], s_lds[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int tok = 32 * (mw & 3) + token_of_slot(tau_mode, q, e);
        g_lds[e] = tok * 256 + jj * 16;
        s_lds[e] = kWsGBytes + (tok * static_cast<int>(M) + jj) * 2;
    }
    const bool last_tile_ok = (GT - 1) * 16 + jj < M;
    (void)zero_off;

    // Two loops, one per role, with the same number of barriers.  Barrier i says: chunk i is in its slot
    // for everybody, and the slot of chunk i - 1 is free again.  It is a bare s_barrier: the loaders have
    // just waited for exactly the loads that matter, and the computing waves' LDS reads of chunk i - 1
    // ended with the MFMAs that consumed them; __syncthreads() would add a fence that makes every loader
    // wait for ALL its loads, the chunk in flight included.
    if (loader) {
        issue_chunk(0);
        issue_chunk(1);
        for (int i = 0; i < n_chunks; ++i) {
            // everything but the youngest chunk's loads of this wave has landed in LDS
            __builtin_amdgcn_s_waitcnt(0x0F70 | (kLoadsPerChunk & 15) | ((kLoadsPerChunk >> 4) << 14));
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            issue_chunk(i + 2);
        }
    } else {
        for (int i = 0; i < n_chunks; ++i) {
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            const int slot_off = (i % kWsSlots) * kSlotBytes;
            RawRow<4> rows[8];
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const uint4 x = *reinterpret_cast<const uint4*>(lds + slot_off + g_lds[r]);
                rows[r].w[0] = x.x; rows[r].w[1] = x.y; rows[r].w[2] = x.z; rows[r].w[3] = x.w;
            }
            uint32_t sv[GT][8];
#pragma unroll
            for (int a = 0; a < GT; ++a)
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    sv[a][e] = *reinterpret_cast<const uint16_t*>(lds + slot_off + s_lds[e] + a * 32);
            bf16x8 gf[CW];
#pragma unroll
            for (int c = 0; c < CW; ++c) gf[c] = column_fragment(rows, c);
#pragma unroll
            for (int a = 0; a < GT; ++a) {
                uint4 f = make_uint4(__builtin_amdgcn_perm(sv[a][1], sv[a][0], 0x05040100u),
                                     __builtin_amdgcn_perm(sv[a][3], sv[a][2], 0x05040100u),
                                     __builtin_amdgcn_perm(sv[a][5], sv[a][4], 0x05040100u),
                                     __builtin_amdgcn_perm(sv[a][7], sv[a][6], 0x05040100u));
                if (a == GT - 1 && !last_tile_ok) f = make_uint4(0u, 0u, 0u, 0u);
                const bf16x8 sf = __builtin_bit_cast(bf16x8, f);
#pragma unroll
                for (int c = 0; c < CW; ++c)
                    acc[a][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(sf, gf[c], acc[a][c], 0, 0, 0);
            }
        }
    }
    // the loaders' last two (empty) chunks must have landed before the ring is reused
    if (loader) __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();

    // (w4 + w5) + (w6 + w7), as in the per-wave kernel; the loaders only keep the barriers company
    f32x4 (*red)[TP][kWave] = reinterpret_cast<f32x4 (*)[TP][kWave]>(lds);
    float* out = partial + static_cast<int64_t>(split) * O * Mp;
    constexpr int H = (TP + 1) / 2;
#if VELORA_SKIP & 8
    // measurement builds only: the partial tile stored without the cross-wave sum (wrong values, same stores)
    if (mw == 0 || mw == 2) {
#pragma unroll
        for (int i = 0; i < TP; ++i)
            if ((mw == 0) == (i < H)) store_tile<CW>(out, acc[i / CW][i % CW], o0, jj, q, i % CW, (i / CW) * 16, O, Mp);
    }
    return;
#endif
    if (mw == 1 || mw == 3) {
#pragma unroll
        for (int i = 0; i < TP; ++i) red[mw >> 1][i][lane] = acc[i / CW][i % CW];
    }
    __syncthreads();
    if (mw == 0 || mw == 2) {
#pragma unroll
        for (int i = 0; i < TP; ++i) acc[i / CW][i % CW] += red[mw >> 1][i][lane];
#pragma unroll
        for (int i = 0; i < TP; ++i)
            if ((mw == 2) == (i < H)) red[mw >> 1][i][lane] = acc[i / CW][i % CW];
    }
    __syncthreads();
    if (mw == 0 || mw == 2) {
#pragma unroll
        for (int i = 0; i < TP; ++i)
            if ((mw == 0) == (i < H)) {
                const int a = i / CW, c = i % CW;
                const f32x4 other = red[mw == 0 ? 1 : 0][i][lane];
                const f32x4 t = mw == 0 ? acc[a][c] + other : other + acc[a][c];
                store_tile<CW>(out, t, o0, jj, q, c, a * 16, O, Mp);
            }
    }
}

// ---------------------------------------------------------------------------
// Kernel 1, loader waves, four to six group tiles (M up to 96).
//
// The same division of labour as above for tile counts whose accumulators no longer fit one wave per
// 128 features.  Chunks are 64 tokens (two 32-token steps), so that three ring slots of G (16 KB) and S
// rows (up to 12 KB) fit in LDS; the computing waves split a chunk four ways, by step (2) and by half of
// the 128 features (2): wave (step, half) reads 8 bytes per G row (its four strided columns), holds
// GT x 4 accumulator tiles, and takes its S values for one group tile at a time.  S comes straight from
// S[N, M]: no re-layout pre-pass (one launch and a round trip of S through memory less than the
// per-wave kernel needs at these tile counts).  At the end the two steps of each half are added
// (step 0 + step 1) and the step-0 waves store their halves of the tile.
// Dynamic LDS: 3 x (16 KB + NS x 4 KB), NS = 2 (four tiles) or 3.  grid = (o tiles of 128, splits, 1).
// ---------------------------------------------------------------------------
constexpr int kWs64Rows = 64;
constexpr int kWs64GBytes = kWs64Rows * 256;
constexpr int ws64_s_kb4(int gt) { return (2 * gt + 3) / 4; }          // 4 KB units of S area per slot
constexpr size_t ws64_kernel_lds_bytes(int gt) { return static_cast<size_t>(kWsSlots) * (kWs64GBytes + ws64_s_kb4(gt) * 4096); }

// column c (0..3) of an 8-row block whose rows hold four 16-bit values (two dwords)
__device__ __forceinline__ bf16x8 column_fragment4(const uint2 (&rows)[8], int c) {
    uint32_t f[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t a = (c >> 1) ? rows[2 * i].y : rows[2 * i].x;
        const uint32_t b = (c >> 1) ? rows[2 * i + 1].y : rows[2 * i + 1].x;
        f[i] = (c & 1) ? __builtin_amdgcn_perm(b, a, 0x07060302u) : __builtin_amdgcn_perm(b, a, 0x05040100u);
    }
    return __builtin_bit_cast(bf16x8, make_uint4(f[0], f[1], f[2], f[3]));
}

template <int GT>
__global__ __launch_bounds__(512) void wgrad_partial_ws64_kernel(const uint16_t* __restrict__ G,
                                                                const uint16_t* __restrict__ S,
                                                                float* __restrict__ partial, int64_t N, int64_t O,
                                                                int64_t M, int64_t Mp, int64_t rows_per_split,
                                                                int cyclic, int tau_mode) {
    constexpr int CW = 8, OT = 128, CH = 4;               // CH: column tiles per computing wave
    constexpr int NS = ws64_s_kb4(GT);                    // S loads per loader wave and chunk
    constexpr int kSlotBytes = kWs64GBytes + NS * 4096;
    constexpr int kLoadsPerChunk = 4 + NS;
    extern __shared__ __attribute__((aligned(1024))) char lds[];

    const int lane = threadIdx.x & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const bool loader = w < 4;
    const int mw = w - 4;
    const int step = mw & 1, half = (mw >> 1) & 1;
    const int q = lane >> 4;
    const int jj = lane & 15;
    const int64_t o0 = static_cast<int64_t>(blockIdx.x) * OT;
    const int split = blockIdx.y;
    const int splits = gridDim.y;
    // the planner's ranges are multiples of 128 tokens; here a chunk is 64, two per 128
    int64_t row0, span_rows;
    int n_chunks;
    uint32_t pair_stride;                                 // rows from one 128-token pair of chunks to the next
    if (cyclic) {
        const int64_t total_pairs = ceil_div(N, 128);
        row0 = static_cast<int64_t>(split) * 128;
        span_rows = N - row0;
        n_chunks = 2 * static_cast<int>((total_pairs - split + splits - 1) / splits);
        pair_stride = static_cast<uint32_t>(splits) * 128u;
    } else {
        row0 = static_cast<int64_t>(split) * rows_per_split;
        span_rows = N - row0 < rows_per_split ? N - row0 : rows_per_split;
        n_chunks = 2 * static_cast<int>(ceil_div(span_rows, 128));
        pair_stride = 128u;
    }
    auto chunk_row = [&](int i) -> uint32_t { return static_cast<uint32_t>(i >> 1) * pair_stride + static_cast<uint32_t>(i & 1) * 64u; };
    constexpr uint32_t kLaneOut = 0x7FFFFFFFu, kStepOut = 0x80000000u;
    const uint32_t row_bytes = static_cast<uint32_t>(O) * 2u;
    const uint32_t s_row_bytes = static_cast<uint32_t>(M) * 2u;

    const bool col_ok = o0 + jj * CW < O;
    const uint32_t voff_g0 =
        col_ok ? static_cast<uint32_t>(16 * (w & 3) + q) * row_bytes + static_cast<uint32_t>(jj * 16) : kLaneOut;
    const uint32_t voff_gstep = col_ok ? 4u * row_bytes : 0u;
    const __amdgpu_buffer_rsrc_t g_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<char*>(reinterpret_cast<const char*>(G) + (row0 * O + o0) * 2), 0,
        static_cast<int>(static_cast<uint32_t>(span_rows) * row_bytes - static_cast<uint32_t>(o0 * 2)), 0x00020000);
    const __amdgpu_buffer_rsrc_t s_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<char*>(reinterpret_cast<const char*>(S) + row0 * M * 2), 0,
        static_cast<int>(static_cast<uint32_t>(span_rows) * s_row_bytes), 0x00020000);
    auto issue_chunk = [&](int i) {
        char* slot = lds + (i % kWsSlots) * kSlotBytes;
        const bool real = i < n_chunks;
        const uint32_t g_off = real ? chunk_row(i) * row_bytes : kStepOut;
        const uint32_t s_off = real ? chunk_row(i) * s_row_bytes : kStepOut;
#pragma unroll
        for (int r = 0; r < 4; ++r)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(g_rsrc, (lds_void_ptr)(slot + (16 * (w & 3) + 4 * r) * 256), 16,
                                                     voff_g0 + r * voff_gstep + g_off, 0, 0, kStreamAux);
#pragma unroll
        for (int t = 0; t < NS; ++t) {
            const uint32_t kb = static_cast<uint32_t>((w & 3) + 4 * t);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(s_rsrc, (lds_void_ptr)(slot + kWs64GBytes + kb * 1024), 16,
                                                     kb * 1024u + static_cast<uint32_t>(lane) * 16u + s_off, 0, 0, 0);
        }
    };

    f32x4 acc[GT][CH];
#pragma unroll
    for (int a = 0; a < GT; ++a)
#pragma unroll
        for (int c = 0; c < CH; ++c) acc[a][c] = f32x4{0.f, 0.f, 0.f, 0.f};
    int g_lds[8], s_lds[8];                               // token_of_slot: which token sits in K slot (q, e)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int tok = 32 * step + token_of_slot(tau_mode, q, e);
        g_lds[e] = tok * 256 + jj * 16 + half * 8;
        s_lds[e] = kWs64GBytes + (tok * static_cast<int>(M) + jj) * 2;
    }
    const bool last_tile_ok = (GT - 1) * 16 + jj < M;

    if (loader) {
        issue_chunk(0);
        issue_chunk(1);
        for (int i = 0; i < n_chunks; ++i) {
            __builtin_amdgcn_s_waitcnt(0x0F70 | (kLoadsPerChunk & 15) | ((kLoadsPerChunk >> 4) << 14));
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            issue_chunk(i + 2);
        }
    } else {
        for (int i = 0; i < n_chunks; ++i) {
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            const int slot_off = (i % kWsSlots) * kSlotBytes;
            uint2 rows[8];
#pragma unroll
            for (int r = 0; r < 8; ++r) rows[r] = *reinterpret_cast<const uint2*>(lds + slot_off + g_lds[r]);
            bf16x8 gf[CH];
#pragma unroll
            for (int c = 0; c < CH; ++c) gf[c] = column_fragment4(rows, c);
#pragma unroll
            for (int a = 0; a < GT; ++a) {
                uint32_t sv[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) sv[e] = *reinterpret_cast<const uint16_t*>(lds + slot_off + s_lds[e] + a * 32);
                uint4 f = make_uint4(__builtin_amdgcn_perm(sv[1], sv[0], 0x05040100u),
                                     __builtin_amdgcn_perm(sv[3], sv[2], 0x05040100u),
                                     __builtin_amdgcn_perm(sv[5], sv[4], 0x05040100u),
                                     __builtin_amdgcn_perm(sv[7], sv[6], 0x05040100u));
                if (a == GT - 1 && !last_tile_ok) f = make_uint4(0u, 0u, 0u, 0u);
                const bf16x8 sf = __builtin_bit_cast(bf16x8, f);
#pragma unroll
                for (int c = 0; c < CH; ++c)
                    acc[a][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(sf, gf[c], acc[a][c], 0, 0, 0);
            }
        }
    }
    if (loader) __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();

    // step 0 + step 1 for each half of the features; the step-0 waves store
    constexpr int NT = GT * CH;                            // tiles per computing wave (<= 24)
    f32x4 (*red)[NT][kWave] = reinterpret_cast<f32x4 (*)[NT][kWave]>(lds);
    float* out = partial + static_cast<int64_t>(split) * O * Mp;
    if (!loader && step == 1) {
#pragma unroll
        for (int i = 0; i < NT; ++i) red[half][i][lane] = acc[i / CH][i % CH];
    }
    __syncthreads();
    if (!loader && step == 0) {
#pragma unroll
        for (int i = 0; i < NT; ++i) {
            const int a = i / CH, c = i % CH;
            const f32x4 t = acc[a][c] + red[half][i][lane];
            store_tile<CW>(out, t, o0, jj, q, half * CH + c, a * 16, O, Mp);
        }
    }
}

// ---------------------------------------------------------------------------
// Kernel 1, loader waves on a 256-feature tile (one to five group tiles).
//
// The same division of labour as wgrad_partial_ws64_kernel, with twice the features per block: a chunk
// is 64 tokens x 256 features of G (32 KB) plus those tokens' rows of S, and each of the four computing
// waves takes one 32-token step of it and one 128-feature half (eight column tiles, as in the 128-wide
// kernel).  S is fetched once per 256 output features instead of once per 128: with 43 sub-tokens per
// token that takes the S share of a block's cache-line requests from 27 % to 16 %, and the partial
// kernels are bound by the number of requests a compute unit can keep in flight.  The price is twice the
// token ranges for the same number of blocks (twice the partial sums written here and read back by the
// expansion), which is why this pays only on wide outputs, where the 128-feature layout has few ranges.
// grid = (o tiles of 256, splits); 512 threads; 3 slots x (32 KB + 4, 8 or 12 KB) of dynamic LDS.
// ---------------------------------------------------------------------------
constexpr int kWs256GBytes = kWs64Rows * 512;
constexpr size_t ws256_kernel_lds_bytes(int gt) { return static_cast<size_t>(kWsSlots) * (kWs256GBytes + ws64_s_kb4(gt) * 4096); }

template <int GT>
__global__ __launch_bounds__(512) void wgrad_partial_ws256_kernel(const uint16_t* __restrict__ G,
                                                                 const uint16_t* __restrict__ S,
                                                                 float* __restrict__ partial, int64_t N, int64_t O,
                                                                 int64_t M, int64_t Mp, int64_t rows_per_split,
                                                                 int cyclic, int tau_mode) {
    constexpr int OT = 256, CH = 8;                       // CH: column tiles per computing wave
    constexpr bool kTwoBatches = GT >= 5;
    constexpr int NS = ws64_s_kb4(GT);                    // S loads per loader wave and chunk
    constexpr int kSlotBytes = kWs256GBytes + NS * 4096;
    constexpr int kLoadsPerChunk = 8 + NS;
    static_assert(static_cast<size_t>(2) * GT * CH * kWave * sizeof(f32x4) <= ws256_kernel_lds_bytes(GT),
                  "the cross-wave sum reuses the ring");
    extern __shared__ __attribute__((aligned(1024))) char lds[];

    const int lane = threadIdx.x & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const bool loader = w < 4;
    const int mw = w - 4;
    const int step = mw & 1, half = (mw >> 1) & 1;
    const int q = lane >> 4;
    const int jj = lane & 15;
    const int64_t o0 = static_cast<int64_t>(blockIdx.x) * OT;
    const int split = blockIdx.y;
    const int splits = gridDim.y;
    // the planner's ranges are multiples of 128 tokens; here a chunk is 64, two per 128
    int64_t row0, span_rows;
    int n_chunks;
    uint32_t pair_stride;                                 // rows from one 128-token pair of chunks to the next
    if (cyclic) {
        const int64_t total_pairs = ceil_div(N, 128);
        row0 = static_cast<int64_t>(split) * 128;
        span_rows = N - row0;
        n_chunks = 2 * static_cast<int>((total_pairs - split + splits - 1) / splits);
        pair_stride = static_cast<uint32_t>(splits) * 128u;
    } else {
        row0 = static_cast<int64_t>(split) * rows_per_split;
        span_rows = N - row0 < rows_per_split ? N - row0 : rows_per_split;
        n_chunks = 2 * static_cast<int>(ceil_div(span_rows, 128));
        pair_stride = 128u;
    }
    if (span_rows <= 0) { n_chunks = 0; span_rows = 0; }
    auto chunk_row = [&](int i) -> uint32_t { return static_cast<uint32_t>(i >> 1) * pair_stride + static_cast<uint32_t>(i & 1) * 64u; };
    constexpr uint32_t kLaneOut = 0x7FFFFFFFu, kStepOut = 0x80000000u;
    const uint32_t row_bytes = static_cast<uint32_t>(O) * 2u;
    const uint32_t s_row_bytes = static_cast<uint32_t>(M) * 2u;

    // loader wave w, instruction r: rows 16 w + 2 r + (lane / 32) of the chunk, 16 bytes at (lane % 32) * 16 of
    // the 512-byte row piece; LDS-direct loads land lane after lane, i.e. as [row][512 bytes]
    const int lrow = lane >> 5, lcol = lane & 31;
    const bool col_ok = o0 + lcol * 8 < O;
    const uint32_t voff_g0 =
        col_ok ? static_cast<uint32_t>(16 * (w & 3) + lrow) * row_bytes + static_cast<uint32_t>(lcol * 16) : kLaneOut;
    const uint32_t voff_gstep = col_ok ? 2u * row_bytes : 0u;
    const __amdgpu_buffer_rsrc_t g_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<char*>(reinterpret_cast<const char*>(G) + (row0 * O + o0) * 2), 0,
        static_cast<int>(static_cast<uint32_t>(span_rows) * row_bytes - (span_rows > 0 ? static_cast<uint32_t>(o0 * 2) : 0u)),
        0x00020000);
    const __amdgpu_buffer_rsrc_t s_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<char*>(reinterpret_cast<const char*>(S) + row0 * M * 2), 0,
        static_cast<int>(static_cast<uint32_t>(span_rows) * s_row_bytes), 0x00020000);
    auto issue_chunk = [&](int i) {
        char* slot = lds + (i % kWsSlots) * kSlotBytes;
        const bool real = i < n_chunks;
        const uint32_t g_off = real ? chunk_row(i) * row_bytes : kStepOut;
        const uint32_t s_off = real ? chunk_row(i) * s_row_bytes : kStepOut;
#pragma unroll
        for (int r = 0; r < 8; ++r)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(g_rsrc, (lds_void_ptr)(slot + (16 * (w & 3) + 2 * r) * 512), 16,
                                                     voff_g0 + r * voff_gstep + g_off, 0, 0, kStreamAux);
#pragma unroll
        for (int t = 0; t < NS; ++t) {
            const uint32_t kb = static_cast<uint32_t>((w & 3) + 4 * t);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(s_rsrc, (lds_void_ptr)(slot + kWs256GBytes + kb * 1024), 16,
                                                     kb * 1024u + static_cast<uint32_t>(lane) * 16u + s_off, 0, 0, 0);
        }
    };

    f32x4 acc[GT][CH];
#pragma unroll
    for (int a = 0; a < GT; ++a)
#pragma unroll
        for (int c = 0; c < CH; ++c) acc[a][c] = f32x4{0.f, 0.f, 0.f, 0.f};
    // token_of_slot: which token sits in K slot (q, e).  One per-lane base each for G and S plus eight
    // wave-uniform offsets (scalar registers): eight per-lane addresses each would not fit beside the
    // accumulators of five tiles.
    const int tok_s1 = token_of_slot(tau_mode, 0, 1) - token_of_slot(tau_mode, 0, 0);
    const int tok_s2 = token_of_slot(tau_mode, 0, 2) - token_of_slot(tau_mode, 0, 0);
    const int tok0 = 32 * step + token_of_slot(tau_mode, q, 0);
    const int g_lds0 = tok0 * 512 + jj * 32 + half * 16;
    const int s_lds0 = kWs256GBytes + (tok0 * static_cast<int>(M) + jj) * 2;
    int g_lds[8], s_lds[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int dt = __builtin_amdgcn_readfirstlane((e & 1) * tok_s1 + (e >> 1) * tok_s2);
        g_lds[e] = dt * 512;
        s_lds[e] = dt * static_cast<int>(M) * 2;
    }
    const bool last_tile_ok = (GT - 1) * 16 + jj < M;

    // the two role loops and their barriers: as in wgrad_partial_ws_kernel
    if (loader) {
        issue_chunk(0);
        issue_chunk(1);
        for (int i = 0; i < n_chunks; ++i) {
            __builtin_amdgcn_s_waitcnt(0x0F70 | (kLoadsPerChunk & 15) | ((kLoadsPerChunk >> 4) << 14));
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            issue_chunk(i + 2);
        }
    } else {
        for (int i = 0; i < n_chunks; ++i) {
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            const int slot_off = (i % kWsSlots) * kSlotBytes;
            const char* g_base = lds + (slot_off + g_lds0);
            const char* s_base = lds + (slot_off + s_lds0);
            auto s_fragment = [&](int a) -> bf16x8 {
                uint32_t sv[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) sv[e] = *reinterpret_cast<const uint16_t*>(s_base + s_lds[e] + a * 32);
                uint4 f = make_uint4(__builtin_amdgcn_perm(sv[1], sv[0], 0x05040100u),
                                     __builtin_amdgcn_perm(sv[3], sv[2], 0x05040100u),
                                     __builtin_amdgcn_perm(sv[5], sv[4], 0x05040100u),
                                     __builtin_amdgcn_perm(sv[7], sv[6], 0x05040100u));
                if (a == GT - 1 && !last_tile_ok) f = make_uint4(0u, 0u, 0u, 0u);
                return __builtin_bit_cast(bf16x8, f);
            };
            if constexpr (!kTwoBatches) {
                RawRow<4> rows[8];
#pragma unroll
                for (int r = 0; r < 8; ++r) {
                    const uint4 x = *reinterpret_cast<const uint4*>(g_base + g_lds[r]);
                    rows[r].w[0] = x.x; rows[r].w[1] = x.y; rows[r].w[2] = x.z; rows[r].w[3] = x.w;
                }
                bf16x8 gf[CH];
#pragma unroll
                for (int c = 0; c < CH; ++c) gf[c] = column_fragment(rows, c);
#pragma unroll
                for (int a = 0; a < GT; ++a) {
                    const bf16x8 sf = s_fragment(a);
#pragma unroll
                    for (int c = 0; c < CH; ++c)
                        acc[a][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(sf, gf[c], acc[a][c], 0, 0, 0);
                }
            } else {
                // five tiles: 160 accumulator registers leave no room for eight G fragments and their rows at
                // once (two waves per SIMD, 256 registers each), so the S fragments are formed first and the
                // wave's eight column tiles go through in two batches of four
#pragma unroll
                for (int cb = 0; cb < 2; ++cb) {
                    uint2 rows[8];
#pragma unroll
                    for (int r = 0; r < 8; ++r) rows[r] = *reinterpret_cast<const uint2*>(g_base + g_lds[r] + cb * 8);
                    bf16x8 gf[4];
#pragma unroll
                    for (int c = 0; c < 4; ++c) gf[c] = column_fragment4(rows, c);
#pragma unroll
                    for (int a = 0; a < GT; ++a) {
                        const bf16x8 sf = s_fragment(a);
#pragma unroll
                        for (int c = 0; c < 4; ++c)
                            acc[a][cb * 4 + c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(sf, gf[c], acc[a][cb * 4 + c], 0, 0, 0);
                    }
                }
            }
        }
    }
    if (loader) __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();

    // step 0 + step 1 for each half of the features; the step-0 waves store.  Lane jj's column tile c of
    // half h is feature o0 + 16 jj + 8 h + c (the 32-byte piece a lane reads holds sixteen features).
    constexpr int NT = GT * CH;
    f32x4 (*red)[NT][kWave] = reinterpret_cast<f32x4 (*)[NT][kWave]>(lds);
    float* out = partial + static_cast<int64_t>(split) * O * Mp;
    // The lane's index once more, from the hardware and behind the loop: carried across the loop, it and
    // what is derived from it are the registers that five tiles' accumulators leave no room for.
    int lane_e;
    asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(lane_e));
    const int q_e = lane_e >> 4, jj_e = lane_e & 15;
    if (!loader && step == 1) {
#pragma unroll
        for (int i = 0; i < NT; ++i) red[half][i][lane_e] = acc[i / CH][i % CH];
    }
    __syncthreads();
    if (!loader && step == 0) {
#pragma unroll
        for (int i = 0; i < NT; ++i) {
            const int a = i / CH, c = i % CH;
            const f32x4 t = acc[a][c] + red[half][i][lane_e];
            store_tile<16>(out, t, o0, jj_e, q_e, half * CH + c, a * 16, O, Mp);
        }
    }
}

// ---------------------------------------------------------------------------
// Kernel 1, MFMA path for many group tiles (8, 12 or 16 per block).
//
// With that many tiles a wave cannot hold accumulators for all of them, so the
// block's NW waves (4 or 8) split the tiles (GTW each) and all walk every
// 32-token step of the block's range.  They then need the same G tile
// (32 tokens x 128 features, 8 KB): each wave fetches its share of it from HBM
// (8 / NW rows of every 8-row group) into a register ring NG steps deep,
// publishes it in a double-buffered LDS tile, and after one barrier every wave
// reads the whole tile back in the lane layout of the in-register transpose.
// G is thus read once per block, S (packed fragments) once per 128 output
// features.  A wave only carries 1-2 KB of G per step, so the G ring is deep
// (NG = 8); S comes from L2 and needs a shorter ring (NS).
// A wave that waits to issue loads (a CU sustains a bounded number of
// outstanding cache-line requests; per step a block asks for 64 lines of G and
// 8 lines of S per tile) issues no MFMAs meanwhile, so with one wave per SIMD
// the two times add up.  At 16 tiles the block therefore has eight waves of two
// tiles each, two per SIMD (under 256 registers), and one wave's MFMAs fill the
// other's stalls: measured 57 us against 64 us for four waves of four tiles at
// N = 16384, O = 5120, M = 216.  At 8 and 12 tiles eight waves measured no
// faster than four.  Covering 256 features per block (half the S re-reads)
// measured no faster either.
// grid = (o tiles of 128, splits, g chunks of NW*GTW tiles)
// ---------------------------------------------------------------------------
template <int GTW, int NW, int NG, int NS>
__global__ __launch_bounds__(NW * 64) void wgrad_partial_shared_g_kernel(const uint16_t* __restrict__ G,
                                                                    const void* __restrict__ Spk,
                                                                    float* __restrict__ partial, int64_t N,
                                                                    int64_t O, int64_t M, int64_t Mp,
                                                                    int64_t rows_per_split, int64_t tiles_packed) {
    static_assert(NG % 2 == 0, "the LDS buffer index must be a compile-time function of the ring slot");
    static_assert(NG % NS == 0, "the S ring slot must be a compile-time function of the G ring slot");
    static_assert(NW == 4 || NW == 8, "a wave fetches 8 / NW rows of every 8-row group");
    constexpr int CW = 8;
    constexpr int OT = 16 * CW;
    constexpr int RPW = 8 / NW;                        // rows of every 8-row group this wave fetches
    __shared__ uint4 gtile[2][kStep][16];              // [buffer][token][16-byte chunk of 8 features]

    const int lane = threadIdx.x & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int q = lane >> 4;
    const int jj = lane & 15;
    const int64_t o0 = static_cast<int64_t>(blockIdx.x) * OT;
    const int split = blockIdx.y;
    const int64_t tile0 = static_cast<int64_t>(blockIdx.z) * (GTW * NW) + w * GTW;
    const int64_t kb = static_cast<int64_t>(split) * rows_per_split;
    int64_t ke = kb + rows_per_split;
    if (ke > N) ke = N;
    const int rows = static_cast<int>(ke - kb);
    const int n_steps = (rows + kStep - 1) / kStep;

    const uint32_t row_bytes = static_cast<uint32_t>(O) * 2u;
    const bool col_ok = o0 + jj * CW < O;
    uint32_t voff[RPW];                                // this wave's rows of every 8-row group
#pragma unroll
    for (int i = 0; i < RPW; ++i)
        voff[i] = col_ok ? static_cast<uint32_t>(q * 8 + RPW * w + i) * row_bytes + static_cast<uint32_t>(jj * CW * 2)
                         : 0xFFFFFFFFu;
    const char* gblock = reinterpret_cast<const char*>(G) + (kb * O + o0) * 2;
    const uint32_t gblock_bytes = static_cast<uint32_t>(rows) * row_bytes - static_cast<uint32_t>(o0 * 2);
    const uint32_t step_bytes = static_cast<uint32_t>(kStep) * row_bytes;
    // S fragments of this wave's tiles; tiles past the last real one are never fetched (they read as zeros)
    const uint32_t s_step_bytes = static_cast<uint32_t>(tiles_packed) * 1024u;
    const bool any_tile = tile0 < tiles_packed;
    const char* sblock = reinterpret_cast<const char*>(Spk) +
                         ((kb / kStep) * tiles_packed + (any_tile ? tile0 : 0)) * 1024;
    const uint32_t sblock_bytes =
        any_tile ? static_cast<uint32_t>(n_steps) * s_step_bytes - static_cast<uint32_t>(tile0) * 1024u : 0u;
    uint32_t s_voff[GTW];
#pragma unroll
    for (int a = 0; a < GTW; ++a)
        s_voff[a] = tile0 + a < tiles_packed ? static_cast<uint32_t>(lane) * 16u + a * 1024u : 0xFFFFFFFFu;

    f32x4 acc[GTW][CW];
#pragma unroll
    for (int a = 0; a < GTW; ++a)
#pragma unroll
        for (int c = 0; c < CW; ++c) acc[a][c] = f32x4{0.f, 0.f, 0.f, 0.f};

    u32x4 gr[NG][RPW];
    u32x4 sr[NS][GTW];
    auto load_g_step = [&](u32x4 (&dst)[RPW], int t) {
        const uint32_t off = static_cast<uint32_t>(t) * step_bytes;
        const uint32_t left = t < n_steps ? gblock_bytes - off : 0u;
        __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<char*>(gblock + (t < n_steps ? off : 0u)), 0, static_cast<int>(left), 0x00020000);
#pragma unroll
        for (int i = 0; i < RPW; ++i) dst[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, voff[i], 0, kStreamAux);
    };
    auto load_s_step = [&](u32x4 (&dst)[GTW], int t) {
        const uint32_t off = static_cast<uint32_t>(t) * s_step_bytes;
        const uint32_t left = (t < n_steps && off < sblock_bytes) ? sblock_bytes - off : 0u;
        __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<char*>(sblock + (left ? off : 0u)), 0, static_cast<int>(left), 0x00020000);
#pragma unroll
        for (int a = 0; a < GTW; ++a) dst[a] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, s_voff[a], 0, 0);
    };

#pragma unroll
    for (int s = 0; s < NG; ++s) load_g_step(gr[s], s);
#pragma unroll
    for (int s = 0; s < NS; ++s) load_s_step(sr[s], s);
    // Software pipeline: while the matrix pipe works on step t, the wave
    // publishes its share of step t+1, reads the whole tile t+1 back and
    // transposes it, so LDS latency and the v_perm work hide under the MFMAs.
    // One barrier per step is enough with two LDS buffers: a wave writes
    // buffer (t+1)&1 only after the barrier of step t-1, which every wave
    // passes with its reads of tile t-1 already in registers.
    auto publish = [&](const u32x4 (&src)[RPW], int buf) {
#pragma unroll
        for (int i = 0; i < RPW; ++i)
            gtile[buf][q * 8 + RPW * w + i][jj] = make_uint4(src[i].x, src[i].y, src[i].z, src[i].w);
    };
    auto read_tile = [&](RawRow<4> (&rowsv)[8], int buf) {
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const uint4 x = gtile[buf][q * 8 + r][jj];
            rowsv[r].w[0] = x.x; rowsv[r].w[1] = x.y; rowsv[r].w[2] = x.z; rowsv[r].w[3] = x.w;
        }
    };
    bf16x8 gf[CW];
    {
        publish(gr[0], 0);
        load_g_step(gr[0], NG);
        __syncthreads();
        RawRow<4> rowsv[8];
        read_tile(rowsv, 0);
#pragma unroll
        for (int c = 0; c < CW; ++c) gf[c] = column_fragment(rowsv, c);
    }
    for (int base = 0; base < n_steps; base += NG) {
#pragma unroll
        for (int s = 0; s < NG; ++s) {
            const int t = base + s;
            const int sn = (s + 1) % NG;           // ring slot of step t+1
            const int bufn = (s + 1) & 1;          // == (t+1) & 1 because NG is even
            const int ss = s % NS;                 // == t % NS because NS divides NG
            publish(gr[sn], bufn);
            load_g_step(gr[sn], t + 1 + NG);
            __syncthreads();
            RawRow<4> rowsv[8];
            read_tile(rowsv, bufn);
#pragma unroll
            for (int a = 0; a < GTW; ++a) {
                const bf16x8 sf = __builtin_bit_cast(bf16x8, sr[ss][a]);
#pragma unroll
                for (int c = 0; c < CW; ++c)
                    acc[a][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(sf, gf[c], acc[a][c], 0, 0, 0);
            }
#pragma unroll
            for (int c = 0; c < CW; ++c) gf[c] = column_fragment(rowsv, c);
            __builtin_amdgcn_sched_barrier(0);
            load_s_step(sr[ss], t + NS);
        }
    }

    // every wave owns its tiles and stores them straight from its registers
    float* out = partial + static_cast<int64_t>(split) * O * Mp;
#pragma unroll
    for (int a = 0; a < GTW; ++a)
#pragma unroll
        for (int c = 0; c < CW; ++c) store_tile<CW>(out, acc[a][c], o0, jj, q, c, (tile0 + a) * 16, O, Mp);
}

// ---------------------------------------------------------------------------
// Kernel 1, float32 inputs on the float32 matrix instruction.
//
// v_mfma_f32_16x16x4_f32: D[16x16] += A[16x4] * B[4x16]; lane l supplies A[l%16][l/16] and B[l/16][l%16], ONE
// value each, so with the reduction index (the token) as the slow axis of both operands nothing has to be
// transposed: lane (q, jj) of k step ks takes token 4 ks + q, the value S[token][16 a + jj] for group tile a
// and eight consecutive features G[token][o0 + 8 jj .. + 7] (two 16-byte loads, 512 contiguous bytes per
// token and wave), of which feature c feeds column tile c (the same strided column map as the bf16 kernels,
// so the epilogue is theirs).  A block owns 128 features x one token range x GT group tiles; its four waves
// take alternate 16-token steps with the next step's loads in flight, and are summed (w0 + w2) + (w1 + w3)
// through LDS at the end.  The instruction runs at 1/16 of the bf16 rate: with 43 groups per token the
// matrix pipes need about as long as HBM needs for G, which is still an order of magnitude less than the
// plain-FMA kernel below needs (N = 16384, O = 4096, M = 43: 514 us).
// Edges as in the bf16 kernels: range-checked descriptors return zeros past the token range, past O and
// past M.  Needs O % 4 == 0, 16-byte aligned G, and byte offsets inside a token range below 2^31.
// grid = (o tiles of 128, splits, chunks of GT group tiles)
// ---------------------------------------------------------------------------
constexpr int kF32Step = 16;                           // tokens per step and wave: four k steps of the instruction

template <int GT>
__global__ __launch_bounds__(256) void wgrad_partial_f32_mfma_kernel(const float* __restrict__ G,
                                                                    const float* __restrict__ S,
                                                                    float* __restrict__ partial, int64_t N, int64_t O,
                                                                    int64_t M, int64_t Mp, int64_t rows_per_split) {
    constexpr int CW = 8, NT = GT * CW;
    __shared__ f32x4 red[2][NT][kWave];
    const int lane = threadIdx.x & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int q = lane >> 4;
    const int jj = lane & 15;
    const int64_t o0 = static_cast<int64_t>(blockIdx.x) * (16 * CW);
    const int split = blockIdx.y;
    const int64_t g0 = static_cast<int64_t>(blockIdx.z) * (16 * GT);
    const int64_t kb = static_cast<int64_t>(split) * rows_per_split;
    int64_t ke = kb + rows_per_split;
    if (ke > N) ke = N;
    const int rows = ke > kb ? static_cast<int>(ke - kb) : 0;
    const int n_steps = (rows + kF32Step - 1) / kF32Step;

    constexpr uint32_t kOut = 0x80000000u;             // an offset no descriptor here covers
    const uint32_t row_bytes = static_cast<uint32_t>(O) * 4u;
    const uint32_t s_row_bytes = static_cast<uint32_t>(M) * 4u;
    const bool lo_ok = o0 + jj * CW < O, hi_ok = o0 + jj * CW + 4 < O;
    const uint32_t g_lane = static_cast<uint32_t>(q) * row_bytes + static_cast<uint32_t>(jj * CW * 4);
    const __amdgpu_buffer_rsrc_t g_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<char*>(reinterpret_cast<const char*>(G) + (kb * O + o0) * 4), 0,
        rows > 0 ? static_cast<int>(static_cast<uint32_t>(rows) * row_bytes - static_cast<uint32_t>(o0 * 4)) : 0, 0x00020000);
    const __amdgpu_buffer_rsrc_t s_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<char*>(reinterpret_cast<const char*>(S) + kb * M * 4), 0,
        static_cast<int>(static_cast<uint32_t>(rows) * s_row_bytes), 0x00020000);
    uint32_t s_lane[GT];
#pragma unroll
    for (int a = 0; a < GT; ++a)
        s_lane[a] = g0 + 16 * a + jj < M ? static_cast<uint32_t>(q) * s_row_bytes + static_cast<uint32_t>((g0 + 16 * a + jj) * 4)
                                         : kOut;

    struct Stage {
        f32x4 glo[4], ghi[4];                          // [k step]: features 8 jj .. + 3 and + 4 .. + 7 of token 4 ks + q
        float sv[4][GT];
    };
    auto load_step = [&](Stage& st, int t) {
        // step t covers tokens 16 t .. 16 t + 15 of the range; past the last step: offsets nothing covers
        const bool real = t < n_steps;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const uint32_t r = static_cast<uint32_t>(t * kF32Step + ks * 4);
            const uint32_t goff = r * row_bytes + g_lane;
            st.glo[ks] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(g_rsrc, real && lo_ok ? goff : kOut, 0, kStreamAux));
            st.ghi[ks] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(g_rsrc, real && hi_ok ? goff + 16u : kOut, 0, kStreamAux));
#pragma unroll
            for (int a = 0; a < GT; ++a)
                st.sv[ks][a] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                                                             s_rsrc, real && s_lane[a] != kOut ? r * s_row_bytes + s_lane[a] : kOut, 0, 0));
        }
    };

    f32x4 acc[GT][CW];
#pragma unroll
    for (int a = 0; a < GT; ++a)
#pragma unroll
        for (int c = 0; c < CW; ++c) acc[a][c] = f32x4{0.f, 0.f, 0.f, 0.f};
    auto compute = [&](const Stage& st) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int a = 0; a < GT; ++a)
#pragma unroll
                for (int c = 0; c < CW; ++c) {
                    const float b = c < 4 ? st.glo[ks][c] : st.ghi[ks][c - 4];
                    acc[a][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(st.sv[ks][a], b, acc[a][c], 0, 0, 0);
                }
    };

    // two register stages: the loads of this wave's next step are in flight while it works on the current one
    Stage sa, sb;
    load_step(sa, w);
    for (int t = w; t < n_steps; t += 8) {
        load_step(sb, t + 4);
        compute(sa);
        if (t + 4 >= n_steps) break;
        load_step(sa, t + 8);
        compute(sb);
    }

    // (w0 + w2) + (w1 + w3), a fixed order
    if (w >= 2) {
#pragma unroll
        for (int i = 0; i < NT; ++i) red[w - 2][i][lane] = acc[i / CW][i % CW];
    }
    __syncthreads();
    if (w < 2) {
#pragma unroll
        for (int i = 0; i < NT; ++i) acc[i / CW][i % CW] += red[w][i][lane];
    }
    __syncthreads();
    if (w == 1) {
#pragma unroll
        for (int i = 0; i < NT; ++i) red[0][i][lane] = acc[i / CW][i % CW];
    }
    __syncthreads();
    if (w == 0) {
        float* out = partial + static_cast<int64_t>(split) * O * Mp;
#pragma unroll
        for (int i = 0; i < NT; ++i) {
            const f32x4 t = acc[i / CW][i % CW] + red[0][i][lane];
            store_tile<CW>(out, t, o0, jj, q, i % CW, g0 + (i / CW) * 16, O, Mp);
        }
    }
}

// ---------------------------------------------------------------------------
// Kernel 1, generic path: float32 inputs, or shapes/pointers the MFMA path
// cannot take.  Plain FMA; thread (ol, gq) owns output feature o0+ol and the
// groups g0 + gq + 4*i, i < 4.
// grid = (o tiles of 64, splits, g tiles of 16)
// ---------------------------------------------------------------------------
template <typename E>
__global__ __launch_bounds__(256) void wgrad_partial_simple_kernel(const typename E::type* __restrict__ G,
                                                                  const typename E::type* __restrict__ S,
                                                                  float* __restrict__ partial, int64_t N, int64_t O,
                                                                  int64_t M, int64_t Mp, int64_t rows_per_split) {
    const int ol = threadIdx.x & 63;
    const int gq = threadIdx.x >> 6;
    const int64_t o = static_cast<int64_t>(blockIdx.x) * 64 + ol;
    const int split = blockIdx.y;
    const int64_t g0 = static_cast<int64_t>(blockIdx.z) * 16 + gq;
    const int64_t kb = static_cast<int64_t>(split) * rows_per_split;
    int64_t ke = kb + rows_per_split;
    if (ke > N) ke = N;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    if (o < O) {
        // eight tokens per trip so that the loads of a trip are independent
        for (int64_t n0 = kb; n0 < ke; n0 += 8) {
            float gv[8], sv[8][4];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int64_t n = n0 + u;
                const bool ok = n < ke;
                gv[u] = ok ? E::load(G, n * O + o) : 0.f;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int64_t g = g0 + 4 * i;
                    sv[u][i] = (ok && g < M) ? E::load(S, n * M + g) : 0.f;
                }
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[i] = fmaf(gv[u], sv[u][i], acc[i]);
        }
        float* out = partial + (static_cast<int64_t>(split) * O + o) * Mp;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t g = g0 + 4 * i;
            if (g < M) out[g] = acc[i];
        }
    }
}

// ---------------------------------------------------------------------------
// Kernel 2: T[o, :] = sum over splits (fixed order), dW[o, g*d + j] (+)= T[o,g]*v[j].
// A block owns one output row (or a few short ones).  The row's partials are
// loaded by all of its threads at once (one memory latency, not one per split),
// summed in split order through LDS, then the row is streamed out.
// VEC: four consecutive columns per lane (needs d % 4 == 0 and an aligned dW).
// ---------------------------------------------------------------------------
// The block shape is chosen by the host so that a thread issues about four
// 16-byte stores: long rows get up to 1024 threads (few rows being written at
// any moment helps HBM write efficiency), short rows are grouped.
constexpr int kTChunk = 2048;
constexpr int kExpandThreads = 1024;

template <bool OUT_BF16, bool VEC>
__global__ __launch_bounds__(kExpandThreads) void wgrad_expand_kernel(const float* __restrict__ partial,
                                                                     const float* __restrict__ v,
                                                                     void* __restrict__ dW, int splits, int64_t O,
                                                                     int64_t D, int64_t M, int64_t Mp, int d,
                                                                     int d_shift, int accumulate, int rows_per_block,
                                                                     int vec8) {
    __shared__ float P[kTChunk];     // partials of the block's rows: [row][split][group]
    __shared__ float T[kTChunk / 2];  // their sums: [row][group]
    const int64_t split_stride = O * Mp;
    // thread -> (row slot r, position p inside the row's share of threads)
    const int tpr = static_cast<int>(blockDim.x) / rows_per_block;   // threads per row
    const int r = threadIdx.x / tpr;
    const int p = threadIdx.x - r * tpr;
    const int64_t o = static_cast<int64_t>(blockIdx.x) * rows_per_block + r;
    const bool row_ok = r < rows_per_block && o < O;
    // groups are staged in LDS in chunks of mchunk per row, sized so that all
    // splits of a chunk fit; the loads of a chunk are spread over the row's
    // threads (one latency, not one per split) and then summed in split order
    int mchunk = kTChunk / (rows_per_block * splits);
    if (mchunk > kTChunk / 2 / rows_per_block) mchunk = kTChunk / 2 / rows_per_block;
    if (mchunk >= 4) mchunk &= ~3;   // a chunk of groups then starts on a multiple of four columns whatever d is
    for (int64_t gc0 = 0; gc0 < M; gc0 += mchunk) {
        const int gcn = static_cast<int>((M - gc0) < mchunk ? (M - gc0) : mchunk);
        float* Pr = P + r * splits * mchunk;
        if (row_ok) {
            const float* prow = partial + o * Mp + gc0;
            for (int idx = p; idx < gcn * splits; idx += tpr) {
                const int sp = idx / gcn, gl = idx - sp * gcn;
                Pr[sp * mchunk + gl] = prow[sp * split_stride + gl];
            }
        }
        __syncthreads();
        if (row_ok) {
            for (int gl = p; gl < gcn; gl += tpr) {
                // split order, eight LDS reads in flight at a time (one read latency per eight splits instead of
                // one per split: with 40 ranges on a small layer the chain was a microsecond of a 6 us kernel)
                float s = 0.f;
                int sp = 0;
                for (; sp + 8 <= splits; sp += 8) {
                    float t[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) t[u] = Pr[(sp + u) * mchunk + gl];
#pragma unroll
                    for (int u = 0; u < 8; ++u) s += t[u];
                }
                for (; sp < splits; ++sp) s += Pr[sp * mchunk + gl];
                T[r * mchunk + gl] = s;
            }
        }
        __syncthreads();
        if (row_ok) {
            const float* Tr = T + r * mchunk;
            const int64_t c_begin = gc0 * d;
            const int64_t c_count = static_cast<int64_t>(gcn) * d;
            if constexpr (VEC && OUT_BF16) {
                // eight bf16 = one 16-byte store per thread and trip when the sub-token size allows it
                if (vec8) {
                    for (int64_t i = p; i < c_count / 8; i += tpr) {
                        const int64_t cl = i * 8;
                        const int gl = d_shift >= 0 ? static_cast<int>(cl >> d_shift) : static_cast<int>(cl / d);
                        const int j = static_cast<int>(cl - static_cast<int64_t>(gl) * d);
                        const float tg = Tr[gl];
                        const float4 va = *reinterpret_cast<const float4*>(v + j);
                        const float4 vb = *reinterpret_cast<const float4*>(v + j + 4);
                        float r[8] = {tg * va.x, tg * va.y, tg * va.z, tg * va.w, tg * vb.x, tg * vb.y, tg * vb.z, tg * vb.w};
                        const int64_t e = o * D + c_begin + cl;
                        uint4* q = reinterpret_cast<uint4*>(static_cast<uint16_t*>(dW) + e);
                        if (accumulate) {
                            const uint4 old = *q;
                            r[0] += bf16_lo(old.x); r[1] += bf16_hi(old.x); r[2] += bf16_lo(old.y); r[3] += bf16_hi(old.y);
                            r[4] += bf16_lo(old.z); r[5] += bf16_hi(old.z); r[6] += bf16_lo(old.w); r[7] += bf16_hi(old.w);
                        }
                        const u32x4 packed_out = {pack_bf16x2(r[0], r[1]), pack_bf16x2(r[2], r[3]),
                                                  pack_bf16x2(r[4], r[5]), pack_bf16x2(r[6], r[7])};
                        __builtin_nontemporal_store(packed_out, reinterpret_cast<u32x4*>(q));
                    }
                } else {
                    for (int64_t i = p; i < c_count / 4; i += tpr) {
                        const int64_t cl = i * 4;
                        const int gl = d_shift >= 0 ? static_cast<int>(cl >> d_shift) : static_cast<int>(cl / d);
                        const int j = static_cast<int>(cl - static_cast<int64_t>(gl) * d);
                        const float tg = Tr[gl];
                        const float4 vv = *reinterpret_cast<const float4*>(v + j);
                        float r0 = tg * vv.x, r1 = tg * vv.y, r2 = tg * vv.z, r3 = tg * vv.w;
                        const int64_t e = o * D + c_begin + cl;
                        uint2* q = reinterpret_cast<uint2*>(static_cast<uint16_t*>(dW) + e);
                        if (accumulate) {
                            const uint2 old = *q;
                            r0 += bf16_lo(old.x); r1 += bf16_hi(old.x); r2 += bf16_lo(old.y); r3 += bf16_hi(old.y);
                        }
                        const u32x2 packed_out = {pack_bf16x2(r0, r1), pack_bf16x2(r2, r3)};
                        __builtin_nontemporal_store(packed_out, reinterpret_cast<u32x2*>(q));
                    }
                }
            } else if constexpr (VEC) {
                for (int64_t i = p; i < c_count / 4; i += tpr) {
                    const int64_t cl = i * 4;
                    const int gl = d_shift >= 0 ? static_cast<int>(cl >> d_shift) : static_cast<int>(cl / d);
                    const int j = static_cast<int>(cl - static_cast<int64_t>(gl) * d);
                    const float tg = Tr[gl];
                    const float4 vv = *reinterpret_cast<const float4*>(v + j);
                    float r0 = tg * vv.x, r1 = tg * vv.y, r2 = tg * vv.z, r3 = tg * vv.w;
                    const int64_t e = o * D + c_begin + cl;
                    float4* q = reinterpret_cast<float4*>(static_cast<float*>(dW) + e);
                    if (accumulate) {
                        const float4 old = *q;
                        r0 += old.x; r1 += old.y; r2 += old.z; r3 += old.w;
                    }
                    const f32x4 out4 = {r0, r1, r2, r3};
                    __builtin_nontemporal_store(out4, reinterpret_cast<f32x4*>(q));
                }
            } else if (!OUT_BF16 && vec8 && (mchunk >= M || (mchunk & 3) == 0)) {
                // float32 rows whose sub-token size is not a multiple of four (d = 43: 256 sub-tokens per token on
                // an 11008-wide layer): still four columns per 16-byte store; a group boundary may fall inside
                // the four (at most one, d >= 4), so every column looks up its own group and element of v
                for (int64_t i = p; i < c_count / 4; i += tpr) {
                    const int64_t cl = i * 4;
                    int gl = static_cast<int>(cl / d);
                    int j = static_cast<int>(cl - static_cast<int64_t>(gl) * d);
                    float r[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        r[u] = Tr[gl] * v[j];
                        if (++j == d) { j = 0; ++gl; }
                    }
                    const int64_t e = o * D + c_begin + cl;
                    float4* q = reinterpret_cast<float4*>(static_cast<float*>(dW) + e);
                    if (accumulate) {
                        const float4 old = *q;
                        r[0] += old.x; r[1] += old.y; r[2] += old.z; r[3] += old.w;
                    }
                    const f32x4 out4 = {r[0], r[1], r[2], r[3]};
                    __builtin_nontemporal_store(out4, reinterpret_cast<f32x4*>(q));
                }
            } else {
                for (int64_t cl = p; cl < c_count; cl += tpr) {
                    const int gl = static_cast<int>(cl / d);
                    const int j = static_cast<int>(cl - static_cast<int64_t>(gl) * d);
                    float x = Tr[gl] * v[j];
                    const int64_t e = o * D + c_begin + cl;
                    if constexpr (OUT_BF16) {
                        uint16_t* q = static_cast<uint16_t*>(dW) + e;
                        if (accumulate) x += bf16_to_f32(*q);
                        *q = f32_to_bf16(x);
                    } else {
                        float* q = static_cast<float*>(dW) + e;
                        if (accumulate) x += *q;
                        *q = x;
                    }
                }
            }
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------
// Kernel 2, window sweep: dW as ONE sweep of the whole grid, straight from the split partials.
// 16-byte vector i of dW belongs to thread i mod (grid * 256), so that at any moment all compute
// units write one contiguous window of grid * 4 KB.  HBM takes that order at 6.2-6.3 TB/s on this
// chip; the same bytes written as one private row (or 32 KB piece) per block reach 5.5-5.7 TB/s and
// more than two blocks per compute unit 4.9 TB/s (plain fill kernels on the 4096 x 11008 float32
// array).  Hence one block per compute unit and eight stores in flight per thread.
// A group's 16-byte vectors are consecutive (D = M * d), so vector i needs T at flat index i / dv,
// and the 256 vectors of a block in one window touch at most 256 / dv + 2 consecutive entries of
// it.  For the U windows of the NEXT trip the block's first U * NL threads each load one entry's
// partials (all splits, summed in split order) ahead of the stores, and put the sums into the
// other half of a small LDS table afterwards; the stores read T and v from LDS, so the only
// vector-memory instructions between them are those few loads.  One bare barrier per trip (a fence
// would wait for the stores).  Needs dv >= 16, d <= 2048, at most 8 * NS8 splits, partials
// below 2 GiB and fewer than 2^31 - 2^24 vectors.
// ---------------------------------------------------------------------------
constexpr int kSweepU = 8;
constexpr int kSweepNL = 18;

template <bool OUT_BF16, int VW, int NS8, bool ACC>
__global__ __launch_bounds__(256) void wgrad_expand_sweep_kernel(const float* __restrict__ partial,
                                                                uint32_t split_stride_b, uint32_t part_bytes,
                                                                const float* __restrict__ v, void* __restrict__ dW,
                                                                uint32_t n_vec, uint32_t dv, uint32_t dv_inv,
                                                                uint32_t M, uint32_t Mp, uint32_t n_groups) {
    constexpr int U = kSweepU, NL = kSweepNL, NS = 8 * NS8;
    constexpr uint32_t VB = OUT_BF16 ? 2u * VW : 16u;       // bytes of one vector of dW
    __shared__ float Tt[2][U * NL + 1];                     // [half][window * nl + entry]; the last slot is a dump
    __shared__ __attribute__((aligned(16))) float vs[2048];
    const uint32_t stride = gridDim.x * 256u;
    const uint32_t t = threadIdx.x;
    for (uint32_t k = t; k < dv * VW; k += 256u) vs[k] = v[k];

    // Everything below is straight-line code inside one loop whose only branches are uniform: with
    // divergent branches around the loads and stores the compiler's wait-count bookkeeping falls back
    // to "wait for everything", which drains the store stream once per trip (35 against 29 us).
    // Threads without a table entry load from past the end of the descriptor (zeros, no memory
    // request) and write their sum to the dump slot; stores past the end of dW are dropped by the
    // range check of a descriptor that is rebuilt for every trip.
    const uint32_t nl = 255u / dv + 2u;                     // table entries one window of a block can touch
    const bool fetcher = t < static_cast<uint32_t>(U) * nl;
    const uint32_t fu = t / nl, fk = t - fu * nl;
    const uint32_t slot = fetcher ? t : static_cast<uint32_t>(U * NL);
    const __amdgpu_buffer_rsrc_t pr =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(partial), 0, part_bytes, 0x00020000);
    auto fetch = [&](float (&px)[NS], uint32_t trip_base) {   // trip_base: the block's first vector in window 0 of that trip
        const uint32_t b = trip_base + fu * stride;             // the block's first vector in window fu
        const uint32_t L = b / dv + fk;
        const bool ok = fetcher && b < n_vec && L < n_groups;
        const uint32_t o = L / M, g = L - o * M;
        const uint32_t off = ok ? (o * Mp + g) * 4u : 0x80000000u;
#pragma unroll
        for (int s = 0; s < NS; ++s)
            px[s] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(pr, off + s * split_stride_b, 0, 0));
    };
    auto publish = [&](const float (&px)[NS], int half) {
        float sum = 0.f;
#pragma unroll
        for (int s = 0; s < NS; ++s) sum += px[s];
        Tt[half][slot] = sum;
    };
    auto lds_barrier = [&]() {
        __builtin_amdgcn_s_waitcnt(0xC07F);      // lgkmcnt(0): LDS writes done; vector memory is not waited for
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };

    // Which 256-vector piece of a window the block takes.  Blocks are dealt to the eight XCDs round-robin,
    // and each XCD has its own L2: with piece = block id every XCD would fetch every line of the partials
    // (8 x 5.8 MB on the 4096 x 11008 layer with 8 splits); with the pieces of one XCD next to each other
    // it fetches an eighth of them.  The order in which the chip as a whole writes dW does not change.
    const uint32_t piece = (gridDim.x & 7u) == 0u ? (blockIdx.x & 7u) * (gridDim.x >> 3) + (blockIdx.x >> 3) : blockIdx.x;
    uint32_t jb = (piece * 256u) % dv;          // position of the block's first vector of the window inside its group
    const uint32_t sr = stride % dv;
    auto store_trip = [&](uint32_t base, int half) {
        // the trip's U windows seen from the block's first vector of window 0: at most U * stride vectors
        const uint32_t left = n_vec - base;                       // base < n_vec here
        const uint32_t span = left < U * stride ? left : U * stride;
        const __amdgpu_buffer_rsrc_t wr = __builtin_amdgcn_make_buffer_rsrc(
            static_cast<unsigned char*>(dW) + static_cast<size_t>(base) * VB, 0, span * VB, 0x00020000);
        // accumulate: this trip's old values first, all U loads in flight at once.  Loaded one by one in front
        // of their stores they would each wait for the store before them (same descriptor, so the compiler
        // keeps the order): eight memory round trips per trip, 123 against 69 us for the 4096 x 11008 float32
        // array.  (Loading them a whole trip ahead into a second register set: 73 us.)
        u32x4 oldv[ACC ? U : 1];
        if constexpr (ACC) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t off = (u * stride + t) * VB;
                if constexpr (!OUT_BF16 || VW == 8) {
                    oldv[u] = __builtin_amdgcn_raw_buffer_load_b128(wr, off, 0, 0);
                } else {
                    const u32x2 o2 = __builtin_amdgcn_raw_buffer_load_b64(wr, off, 0, 0);
                    oldv[u] = u32x4{o2.x, o2.y, 0u, 0u};
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t off = (u * stride + t) * VB;           // past `span` vectors: dropped (loads: zero)
            const uint32_t x = jb + t;
            const uint32_t k = __umulhi(x, dv_inv);               // x / dv (x < dv + 256)
            const uint32_t j = x - k * dv;
            jb += sr;
            if (jb >= dv) jb -= dv;
            const float tg = Tt[half][u * nl + k];
            const f32x4 va = *reinterpret_cast<const f32x4*>(vs + j * VW);
            if constexpr (!OUT_BF16) {
                f32x4 r = {tg * va.x, tg * va.y, tg * va.z, tg * va.w};
                if constexpr (ACC) r += __builtin_bit_cast(f32x4, oldv[u]);
                __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, r), wr, off, 0, kStreamAux);
            } else if constexpr (VW == 8) {
                const f32x4 vb = *reinterpret_cast<const f32x4*>(vs + j * VW + 4);
                float r[8] = {tg * va.x, tg * va.y, tg * va.z, tg * va.w, tg * vb.x, tg * vb.y, tg * vb.z, tg * vb.w};
                if constexpr (ACC) {
                    const u32x4 old = oldv[u];
                    r[0] += bf16_lo(old.x); r[1] += bf16_hi(old.x); r[2] += bf16_lo(old.y); r[3] += bf16_hi(old.y);
                    r[4] += bf16_lo(old.z); r[5] += bf16_hi(old.z); r[6] += bf16_lo(old.w); r[7] += bf16_hi(old.w);
                }
                __builtin_amdgcn_raw_buffer_store_b128(u32x4{pack_bf16x2(r[0], r[1]), pack_bf16x2(r[2], r[3]),
                                                             pack_bf16x2(r[4], r[5]), pack_bf16x2(r[6], r[7])},
                                                       wr, off, 0, kStreamAux);
            } else {
                float r[4] = {tg * va.x, tg * va.y, tg * va.z, tg * va.w};
                if constexpr (ACC) {
                    const u32x4 old = oldv[u];
                    r[0] += bf16_lo(old.x); r[1] += bf16_hi(old.x); r[2] += bf16_lo(old.y); r[3] += bf16_hi(old.y);
                }
                __builtin_amdgcn_raw_buffer_store_b64(u32x2{pack_bf16x2(r[0], r[1]), pack_bf16x2(r[2], r[3])}, wr, off, 0,
                                                      kStreamAux);
            }
        }
    };

    // Loads run two trips ahead of the stores that use them, into two alternating register sets, so
    // that the wait in front of publish() is for loads that have had a whole trip of stores to come
    // back.  Everything is compiler-visible straight-line code, so its wait counts come out as counts
    // (vmcnt(7..13) behind this trip's stores and the other set's loads), not as "wait for everything".
    const uint32_t tstep = U * stride;
    uint32_t base = piece * 256u;               // the block's first vector in window 0 of the current trip
    float pa[NS], pb[NS];
    fetch(pa, base);
    publish(pa, 0);
    lds_barrier();
    fetch(pa, base + tstep);
    while (base < n_vec) {
        fetch(pb, base + 2 * tstep);
        store_trip(base, 0);
        publish(pa, 1);
        lds_barrier();
        base += tstep;
        if (base >= n_vec) break;
        fetch(pa, base + 2 * tstep);
        store_trip(base, 1);
        publish(pb, 0);
        lds_barrier();
        base += tstep;
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
namespace {

// Measurement knobs.  They exist only in builds made with -DVELORA_TUNING (never the shipped
// library, whose calls depend on their arguments and the device alone): there they are read from the
// process environment, here they are their defaults at compile time.
#ifdef VELORA_TUNING
int env_int(const char* name, int fallback) {
    const char* s = std::getenv(name);
    if (!s || !*s) return fallback;
    return std::atoi(s);
}
#else
constexpr int env_int(const char*, int fallback) { return fallback; }
#endif

struct MfmaChoice {
    int cw, gt, nw, chunks;   // cw == 0: the MFMA path cannot take this call
    bool shared;
    bool s_align16;           // S is 16-byte aligned (the loader-wave kernel moves it in 16-byte pieces)
};

// How a block covers the group axis.  Depends on M only, so the workspace query
// can use it.
//   gt      16-group tiles per block: the smallest supported count that covers M,
//           else chunks of 16 tiles
//   shared  the block's nw waves split the tiles (gt / nw each) and share every G
//           tile through LDS; otherwise each of four waves holds all gt tiles and
//           the waves alternate token steps
struct Tiling {
    int gt, nw;
    bool shared;
    int64_t chunks;
};

Tiling tiling_for(int64_t M) {
    static const int kSupported[] = {1, 2, 3, 4, 5, 6, 8, 12, 16};
    const int64_t need = ceil_div(M, 16);
    Tiling t{16, 8, true, ceil_div(need, 16)};
    if (need <= 16) {
        for (int g : kSupported)
            if (g >= need) { t.gt = g; t.chunks = 1; break; }
        t.shared = t.gt >= 8;
        t.nw = t.gt == 16 ? 8 : 4;
    }
    // tuning aid: gt * 10 + waves per block (0 = the per-wave kernel)
    const int forced = env_int("VELORA_WGRAD_TILING", 0);
    if (forced > 0 && need <= forced / 10) {
        t.gt = forced / 10; t.nw = forced % 10; t.shared = t.nw != 0; t.chunks = 1;
    }
    return t;
}

// S operand: the [N, M] array itself (direct gather, at most three group tiles:
// beyond that the 8 two-byte loads per tile and step cost more registers and
// issue slots than the packing pre-pass does time) or the packed fragment array.
bool direct_s(const Tiling& t) { return !t.shared && t.gt <= 3; }

// Up to five group tiles on many output features: blocks of 256 features (wgrad_partial_ws256_kernel).
// Halving the S fetches costs twice the token ranges, i.e. twice the partial sums written and read back
// (the more groups per token, the more bytes that is).  Measured on whole calls, N = 16384, narrow -> wide:
//   one to three tiles:  O = 11008: M = 16 93.5 -> 89.6 us, M = 32 99.8 -> 92.6; O = 13824, M = 20: 128.5 ->
//     119.8; O = 8192: M = 16 71.8 -> 69.6, M = 32 74.3 -> 71.2, M = 43 110.7 -> 106.6; O = 7168: M = 16 64.0 ->
//     61.8, M = 32 66.5 -> 62.8; O = 6144: M = 16 54.4 -> 53.5, M = 32 57.3 -> 55.6, M = 43 83.9 -> 83.1;
//     O = 5632: M = 16 52.5 -> 50.3, M = 32 54.4 -> 52.4, M = 43 79.4 -> 76.9; but O = 5120: M = 5 +1.5 us,
//     M = 20 +1.4 us; O = 4096: M = 43 58.1 -> 58.9 (the partial kernel gains 1.3 us, the expansion of 16
//     ranges instead of 8 loses 1.6); O = 2048, M = 6, N = 65536: 49.4 -> 55.9
//   four and five tiles: O = 11008, M = 64: 101.5 -> 94.1; O = 13824, M = 80: 133.4 -> 124.8; but O = 8192:
//     M = 64 75.2 -> 76.0, M = 80 81.7 -> 86.2; O = 6144: M = 64 59.5 -> 62.1, M = 80 66.7 -> 69.6; O = 5120:
//     M = 54 79.1 -> 81.5, M = 80 57.9 -> 65.0
// Hence: up to three tiles when 128-feature tiles alone outnumber a sixth of the compute units (the narrow
// layout then has at most five ranges), four and five tiles when they outnumber a quarter (at most three
// ranges and several rounds of blocks).  The planner counts blocks accordingly; a call that cannot take
// the wide kernel (alignment) runs the 128-feature kernels on the same ranges.
// (measurement builds: VELORA_WGRAD_WIDE=0 never, 2 for every call with up to five tiles)
bool wide_tiles(const Tiling& t, int64_t O, int num_cus) {
    const int mode = env_int("VELORA_WGRAD_WIDE", 1);
    if (t.shared || t.gt > 5 || t.chunks != 1 || mode == 0) return false;
    return mode == 2 || ceil_div(O, 128) * (t.gt <= 3 ? 6 : 4) > num_cus;
}

MfmaChoice choose_mfma(int64_t O, int64_t M, int g_align, int s_align, const WgradPlan& plan) {
    MfmaChoice ch{0, 0, 4, 0, false, s_align >= 16};
    const Tiling tl = tiling_for(M);
    // byte offsets inside a block's token range are 32-bit
    if (static_cast<double>(plan.rows_per_split) * static_cast<double>(O) * 2.0 >= 2147483648.0) return ch;
    if (static_cast<double>(plan.rows_per_split / kStep + 1) * static_cast<double>(plan.tiles_packed) * 1024.0 >=
        2147483648.0)
        return ch;
    if (tl.chunks > 65535) return ch;
    if (static_cast<double>(plan.rows_per_split) * static_cast<double>(M) * 2.0 >= 2147483648.0) return ch;
    int cw = env_int("VELORA_WGRAD_CW", 8);
    while (cw >= 4 && (O % cw != 0 || g_align < 2 * cw)) cw >>= 1;
    if (cw < 4) return ch;
    ch.cw = cw; ch.gt = tl.gt; ch.nw = tl.nw; ch.chunks = static_cast<int>(tl.chunks);
    ch.shared = tl.shared && cw == 8;     // 8-byte G loads: the per-wave kernel with the same tiles
    return ch;
}

template <int CW, int GT, int NST, bool DIRECT>
hipError_t launch_mfma(const void* G, const void* s_operand, float* partial, int64_t N, int64_t O, int64_t M,
                       const WgradPlan& plan, int chunks, hipStream_t st) {
    dim3 grid(static_cast<unsigned>(ceil_div(O, 16 * CW)), static_cast<unsigned>(plan.splits),
              static_cast<unsigned>(chunks));
    hipLaunchKernelGGL((wgrad_partial_mfma_kernel<CW, GT, NST, DIRECT>), grid, dim3(256), 0, st,
                       static_cast<const uint16_t*>(G), s_operand, partial, N, O, M, plan.Mp, plan.rows_per_split,
                       plan.tiles_packed, plan.cyclic ? 1 : 0);
    return hipGetLastError();
}

// The token_of_slot map for S rows of M values: the pair distance (in bytes, mod 128) nearest to 64.
int pick_tau_mode(int64_t M) {
    const int forced = env_int("VELORA_WGRAD_TAU", -1);
    if (forced >= 0) return forced;
    static const int kDq[4] = {8, 1, 2, 4};
    int best = 0, best_dist = 1 << 30;
    for (int m = 0; m < 4; ++m) {
        const int off = static_cast<int>((kDq[m] * M * 2) % 128);
        const int dist = off > 64 ? off - 64 : 64 - off;
        if (dist < best_dist) { best_dist = dist; best = m; }
    }
    return best;
}

template <int GT>
hipError_t launch_ws(const void* G, const void* S, float* partial, int64_t N, int64_t O, int64_t M, const WgradPlan& plan,
                     hipStream_t st) {
    // more than 64 KB of dynamic LDS has to be allowed once per device and kernel
    static std::atomic<bool> allowed[64];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const size_t lds_bytes = ws_kernel_lds_bytes(GT);
    if (dev < 0 || dev >= 64 || !allowed[dev].load(std::memory_order_acquire)) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&wgrad_partial_ws_kernel<GT>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds_bytes));
        if (e != hipSuccess) return e;
        if (dev >= 0 && dev < 64) allowed[dev].store(true, std::memory_order_release);
    }
    dim3 grid(static_cast<unsigned>(ceil_div(O, 128)), static_cast<unsigned>(plan.splits), 1);
    hipLaunchKernelGGL((wgrad_partial_ws_kernel<GT>), grid, dim3(512), lds_bytes, st, static_cast<const uint16_t*>(G),
                       static_cast<const uint16_t*>(S), partial, N, O, M, plan.Mp, plan.rows_per_split,
                       plan.cyclic ? 1 : 0, pick_tau_mode(M));
    return hipGetLastError();
}

template <int GT>
hipError_t launch_ws64(const void* G, const void* S, float* partial, int64_t N, int64_t O, int64_t M,
                       const WgradPlan& plan, hipStream_t st) {
    static std::atomic<bool> allowed[64];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const size_t lds_bytes = ws64_kernel_lds_bytes(GT);
    if (dev < 0 || dev >= 64 || !allowed[dev].load(std::memory_order_acquire)) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&wgrad_partial_ws64_kernel<GT>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds_bytes));
        if (e != hipSuccess) return e;
        if (dev >= 0 && dev < 64) allowed[dev].store(true, std::memory_order_release);
    }
    dim3 grid(static_cast<unsigned>(ceil_div(O, 128)), static_cast<unsigned>(plan.splits), 1);
    hipLaunchKernelGGL((wgrad_partial_ws64_kernel<GT>), grid, dim3(512), lds_bytes, st, static_cast<const uint16_t*>(G),
                       static_cast<const uint16_t*>(S), partial, N, O, M, plan.Mp, plan.rows_per_split,
                       plan.cyclic ? 1 : 0, pick_tau_mode(M));
    return hipGetLastError();
}

template <int GT>
hipError_t launch_ws256(const void* G, const void* S, float* partial, int64_t N, int64_t O, int64_t M,
                        const WgradPlan& plan, hipStream_t st) {
    static std::atomic<bool> allowed[64];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const size_t lds_bytes = ws256_kernel_lds_bytes(GT);
    if (dev < 0 || dev >= 64 || !allowed[dev].load(std::memory_order_acquire)) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&wgrad_partial_ws256_kernel<GT>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds_bytes));
        if (e != hipSuccess) return e;
        if (dev >= 0 && dev < 64) allowed[dev].store(true, std::memory_order_release);
    }
    dim3 grid(static_cast<unsigned>(ceil_div(O, 256)), static_cast<unsigned>(plan.splits), 1);
    hipLaunchKernelGGL((wgrad_partial_ws256_kernel<GT>), grid, dim3(512), lds_bytes, st, static_cast<const uint16_t*>(G),
                       static_cast<const uint16_t*>(S), partial, N, O, M, plan.Mp, plan.rows_per_split,
                       plan.cyclic ? 1 : 0, pick_tau_mode(M));
    return hipGetLastError();
}

#define VELORA_MFMA_CASE(CW, GT, NST, DIRECT) \
    if (ch.cw == CW && ch.gt == GT)           \
        return launch_mfma<CW, GT, NST, DIRECT>(G, s_operand, partial, N, O, M, plan, ch.chunks, st);

template <int GTW, int NW, int NG, int NS>
hipError_t launch_shared_g(const void* G, const void* s_operand, float* partial, int64_t N, int64_t O, int64_t M,
                           const WgradPlan& plan, int chunks, hipStream_t st) {
    dim3 grid(static_cast<unsigned>(ceil_div(O, 128)), static_cast<unsigned>(plan.splits),
              static_cast<unsigned>(chunks));
    hipLaunchKernelGGL((wgrad_partial_shared_g_kernel<GTW, NW, NG, NS>), grid, dim3(NW * 64), 0, st,
                       static_cast<const uint16_t*>(G), s_operand, partial, N, O, M, plan.Mp, plan.rows_per_split,
                       plan.tiles_packed);
    return hipGetLastError();
}

#define VELORA_SHARED_G_CASE(TILES, NW, NG, NS)                  \
    if (ch.shared && ch.gt == TILES && ch.nw == NW)              \
        return launch_shared_g<TILES / NW, NW, NG, NS>(G, s_operand, partial, N, O, M, plan, ch.chunks, st);

hipError_t dispatch_mfma(const MfmaChoice& ch, const void* G, const void* s_operand, float* partial, int64_t N,
                         int64_t O, int64_t M, const WgradPlan& plan, hipStream_t st, bool* handled) {
    *handled = true;
    VELORA_SHARED_G_CASE(8, 4, 8, 4) VELORA_SHARED_G_CASE(12, 4, 8, 4) VELORA_SHARED_G_CASE(16, 4, 8, 4)
    VELORA_SHARED_G_CASE(8, 8, 8, 4) VELORA_SHARED_G_CASE(16, 8, 8, 4)
    if (ch.shared) { *handled = false; return hipSuccess; }
    // loader waves + computing waves: up to three group tiles straight from S[N, M], 16-byte loads of both
    // (N * M even: a buffer load checks its range per 4 bytes, and the last 2-byte value of an odd-sized S
    // would sit in a word that straddles the end of the array)
    // With a single group tile the per-wave kernel is as fast (62.4 against 63.2 us on N = 16384, O = 11008,
    // M = 16) and stays; with two or three the split is worth 2-6 us (29.0 against 30.8 us on O = 4096,
    // M = 43; 78.5 against 84.4 us on O = 13824, M = 20).
    const int ws_mode = env_int("VELORA_WGRAD_WS", 1);   // measurement builds: 0 never, 2 also for one tile
    const bool wide = wide_tiles(tiling_for(M), O, plan.num_cus);
    if (ch.cw == 8 && ch.gt <= 3 && (ch.gt >= 2 || ws_mode == 2 || wide) && ch.s_align16 && plan.tiles_packed == 0 &&
        (N * M) % 2 == 0 && ws_mode != 0) {
        if (wide) {
            if (ch.gt == 1) return launch_ws256<1>(G, s_operand, partial, N, O, M, plan, st);
            if (ch.gt == 2) return launch_ws256<2>(G, s_operand, partial, N, O, M, plan, st);
            return launch_ws256<3>(G, s_operand, partial, N, O, M, plan, st);
        }
        if (ch.gt == 1) return launch_ws<1>(G, s_operand, partial, N, O, M, plan, st);
        if (ch.gt == 2) return launch_ws<2>(G, s_operand, partial, N, O, M, plan, st);
        return launch_ws<3>(G, s_operand, partial, N, O, M, plan, st);
    }
    // Ring depth 1 everywhere it was measured (2-4 were 1-5 us slower on every layer
    // shape): a CU sustains a fixed number of outstanding cache-line requests, which
    // four waves with one 32-token step each already exceed, and deeper rings only
    // cost registers.
    // Steps in flight per wave.  Two for two to four group tiles, where a step's S loads, transposes and
    // MFMAs take long enough that a wave with a single step in flight leaves the memory pipe short
    // (measured: 31 against 38 us on N = 16384, O = 4096, M = 43; 82 against 88 us on O = 13824, M = 20);
    // one for a single tile, where the second step only costs registers (25.0 against 25.6 us on
    // O = 4096, M = 16), and for five and more tiles, where it does not fit the register file.
    const int ring = env_int("VELORA_WGRAD_RING", 0);   // measurement builds: 1 or 2 for every tile count
    if (ring != 1) {
        if (ring == 2) { VELORA_MFMA_CASE(8, 1, 2, true) VELORA_MFMA_CASE(4, 1, 2, true) }
        VELORA_MFMA_CASE(8, 2, 2, true) VELORA_MFMA_CASE(8, 3, 2, true) VELORA_MFMA_CASE(8, 4, 2, false)
        VELORA_MFMA_CASE(4, 2, 2, true) VELORA_MFMA_CASE(4, 3, 2, true) VELORA_MFMA_CASE(4, 4, 2, false)
    }
    VELORA_MFMA_CASE(8, 1, 1, true) VELORA_MFMA_CASE(8, 2, 1, true) VELORA_MFMA_CASE(8, 3, 1, true)
    VELORA_MFMA_CASE(8, 4, 1, false) VELORA_MFMA_CASE(8, 5, 1, false) VELORA_MFMA_CASE(8, 6, 1, false)
    VELORA_MFMA_CASE(4, 1, 1, true) VELORA_MFMA_CASE(4, 2, 1, true) VELORA_MFMA_CASE(4, 3, 1, true)
    VELORA_MFMA_CASE(4, 4, 1, false) VELORA_MFMA_CASE(4, 5, 1, false) VELORA_MFMA_CASE(4, 6, 1, false)
    VELORA_MFMA_CASE(4, 8, 1, false) VELORA_MFMA_CASE(4, 12, 1, false) VELORA_MFMA_CASE(4, 16, 1, false)
    *handled = false;
    return hipSuccess;
}
#undef VELORA_MFMA_CASE
#undef VELORA_SHARED_G_CASE

template <typename E>
hipError_t launch_simple(const void* G, const void* S, float* partial, int64_t N, int64_t O, int64_t M,
                         const WgradPlan& plan, hipStream_t st) {
    dim3 grid(static_cast<unsigned>(ceil_div(O, 64)), static_cast<unsigned>(plan.splits),
              static_cast<unsigned>(ceil_div(M, 16)));
    hipLaunchKernelGGL((wgrad_partial_simple_kernel<E>), grid, dim3(256), 0, st,
                       static_cast<const typename E::type*>(G), static_cast<const typename E::type*>(S), partial, N,
                       O, M, plan.Mp, plan.rows_per_split);
    return hipGetLastError();
}

// float32 inputs on the float32 matrix instruction: up to three group tiles per block, more groups in
// further blocks (which read G again)
bool f32_mfma_ok(int64_t O, int64_t M, int g_align, const WgradPlan& plan) {
    return O % 4 == 0 && g_align >= 16 &&
           static_cast<double>(plan.rows_per_split + 32) * static_cast<double>(O) * 4.0 < 2147483648.0 &&
           static_cast<double>(plan.rows_per_split + 32) * static_cast<double>(M) * 4.0 < 2147483648.0 &&
           ceil_div(M, 48) <= 65535;
}

hipError_t launch_f32_mfma(const void* G, const void* S, float* partial, int64_t N, int64_t O, int64_t M,
                           const WgradPlan& plan, hipStream_t st) {
    const int gt = M <= 16 ? 1 : M <= 32 ? 2 : 3;
    dim3 grid(static_cast<unsigned>(ceil_div(O, 128)), static_cast<unsigned>(plan.splits),
              static_cast<unsigned>(ceil_div(M, 16 * gt)));
    auto go = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, grid, dim3(256), 0, st, static_cast<const float*>(G), static_cast<const float*>(S),
                           partial, N, O, M, plan.Mp, plan.rows_per_split);
        return hipGetLastError();
    };
    if (gt == 1) return go(wgrad_partial_f32_mfma_kernel<1>);
    if (gt == 2) return go(wgrad_partial_f32_mfma_kernel<2>);
    return go(wgrad_partial_f32_mfma_kernel<3>);
}

template <bool OUT_BF16, bool VEC>
hipError_t launch_expand(const float* partial, int splits, int64_t Mp, const float* v, void* dW, int64_t O, int64_t D,
                         int64_t M, bool accumulate, bool dw_align16, hipStream_t st) {
    const int d = static_cast<int>(D / M);
    int d_shift = -1;
    if ((d & (d - 1)) == 0) {
        d_shift = 0;
        while ((1 << d_shift) < d) ++d_shift;
    }
    // Block shape: about `spt` 16-byte stores (or 4x as many scalars) per thread,
    // 256..1024 threads; short rows are grouped (power of two, <= 16 rows).
    // (measured: 4 stores per thread is at or near the best block shape for
    // every layer shape of the five configurations)
    const bool any4 = !OUT_BF16 && !VEC && d >= 4 && D % 4 == 0 && dw_align16;   // see the kernel's third branch
    const bool vec8 = (OUT_BF16 && VEC && d % 8 == 0 && dw_align16) || any4;
    const int64_t per_row = ceil_div(D, OUT_BF16 && vec8 ? 8 : 4);
    const int spt = 4;
    int64_t threads = ceil_div(ceil_div(per_row, spt), 64) * 64;
    if (threads > kExpandThreads) threads = kExpandThreads;
    int rows_per_block = 1;
    if (threads < 256) {
        while (rows_per_block < 16 && threads * rows_per_block * 2 <= 256 && rows_per_block * 2 * splits <= kTChunk)
            rows_per_block *= 2;
        threads = threads * rows_per_block;
        threads = ceil_div(threads, 64) * 64;
        // a row's share of the block must be the same for every row
        while (threads % rows_per_block) threads += 64;
    }
    hipLaunchKernelGGL((wgrad_expand_kernel<OUT_BF16, VEC>), dim3(static_cast<unsigned>(ceil_div(O, rows_per_block))),
                       dim3(static_cast<unsigned>(threads)), 0, st, partial, v, dW, splits, O, D, M, Mp, d, d_shift,
                       accumulate ? 1 : 0, rows_per_block, vec8 ? 1 : 0);
    return hipGetLastError();
}


}  // namespace

namespace {
WgradPlan plan_wgrad_uncached(int64_t N, int64_t O, int64_t D, int64_t M, bool is_bf16, const LaunchCfg& cfg);
}

// The plan is a pure function of (N, O, D, M, dtype, CU count); a training loop asks for the same few
// again and again, so each thread remembers the last ones it computed (no locks, nothing shared).
WgradPlan plan_wgrad(int64_t N, int64_t O, int64_t D, int64_t M, bool is_bf16, const LaunchCfg& cfg) {
#ifdef VELORA_TUNING
    return plan_wgrad_uncached(N, O, D, M, is_bf16, cfg);   // the knobs may change between calls
#else
    struct Entry {
        int64_t N, O, D, M;
        int bf16, cus;
        WgradPlan plan;
    };
    constexpr int kEntries = 16;
    thread_local Entry memo[kEntries];
    thread_local int used = 0, next = 0;
    for (int i = 0; i < used; ++i) {
        const Entry& e = memo[i];
        if (e.N == N && e.O == O && e.D == D && e.M == M && e.bf16 == (is_bf16 ? 1 : 0) && e.cus == cfg.num_cus)
            return e.plan;
    }
    Entry& e = memo[next];
    e.N = N; e.O = O; e.D = D; e.M = M; e.bf16 = is_bf16 ? 1 : 0; e.cus = cfg.num_cus;
    e.plan = plan_wgrad_uncached(N, O, D, M, is_bf16, cfg);
    next = (next + 1) % kEntries;
    if (used < kEntries) ++used;
    return e.plan;
#endif
}

namespace {
WgradPlan plan_wgrad_uncached(int64_t N, int64_t O, int64_t D, int64_t M, bool is_bf16, const LaunchCfg& cfg) {
    WgradPlan p;
    p.Mp = ceil_div(M, 4) * 4;
    const int64_t in_b = is_bf16 ? 2 : 4;
    Tiling tl{1, 4, false, 1};
    if (is_bf16) tl = tiling_for(M);
    const int gt = tl.gt;
    const int64_t o_tiles = (is_bf16 && wide_tiles(tl, O, cfg.num_cus) ? ceil_div(O, 256) : ceil_div(O, 128)) * tl.chunks;
    // Each split writes a partial tile that the second kernel reads back.
    const double per_split = static_cast<double>(O) * p.Mp * 8.0;
    const int64_t min_rows = is_bf16 ? 256 : 32;   // the plain-FMA kernel is latency-bound per token
    int64_t max_splits = ceil_div(N, min_rows);
    if (max_splits > 1024) max_splits = 1024;
    if (max_splits < 1) max_splits = 1;
    int64_t splits = 1;
    if (is_bf16) {
        // Cost model, in ns.  The G stream is bound per CU (outstanding cache-line
        // requests, ~20 B/ns), so the kernel takes as long as the busiest CU:
        // (blocks per CU, rounded up) x (tokens per block + a block's start-up and
        // epilogue, worth ~384 tokens) x 256 B per token; blocks beyond what a CU
        // holds at once run as further rounds that each pay a drain; every split
        // adds a partial tile that is written here and read back by the expansion.
        // Measured over the layer shapes of the five configurations, the split that
        // minimises this is the fastest or within 2 % of it; in particular exactly
        // one block per CU beats two of half the length.
        const int64_t resident = gt == 1 ? 3 : gt <= 3 ? 2 : 1;   // blocks a CU holds at once (registers)
        const double ns_per_row = 256.0 / 20.0;
        const double partial_ns = per_split / (5000.0 * cfg.num_cus / 256.0);
        double best = 0.0;
        for (int64_t s = 1; s <= max_splits; ++s) {
            const int64_t rows = ceil_div(ceil_div(N, s), 128) * 128;
            const int64_t sp = ceil_div(N, rows);
            const int64_t per_cu = ceil_div(o_tiles * sp, cfg.num_cus);
            const int64_t rounds = ceil_div(per_cu, resident);
            const double cost = static_cast<double>(per_cu) * static_cast<double>(rows + 384) * ns_per_row +
                                static_cast<double>(rounds - 1) * 3000.0 + static_cast<double>(sp) * partial_ns;
            if (s == 1 || cost < best) { best = cost; splits = sp; }
        }
    } else {
        // plain-FMA kernel: two blocks per CU, partial traffic under ~15 % of what the call must move
        const double must_move = static_cast<double>(N) * O * in_b + static_cast<double>(O) * D * 4.0;
        const int64_t traffic_cap = static_cast<int64_t>(0.15 * must_move / per_split);
        splits = (static_cast<int64_t>(cfg.num_cus) * 2) / o_tiles;
        if (splits > traffic_cap) splits = traffic_cap;
        if (splits > max_splits) splits = max_splits;
    }
    const int forced = env_int("VELORA_WGRAD_SPLITS", 0);   // tuning aid; 0 = automatic
    if (forced > 0) splits = forced;
    if (splits < 1) splits = 1;
    if (splits > 1024) splits = 1024;   // also bounds the expand kernel's LDS staging (kTChunk / splits >= 2)
    const int64_t row_quantum = is_bf16 ? 128 : 32;
    int64_t rows = ceil_div(ceil_div(N, splits), row_quantum) * row_quantum;
    p.rows_per_split = rows;
    p.splits = static_cast<int>(ceil_div(N, rows));
    p.partial_bytes = static_cast<size_t>(p.splits) * static_cast<size_t>(O) * static_cast<size_t>(p.Mp) * sizeof(float);
    p.partial_bytes = (p.partial_bytes + 255) / 256 * 256;
    p.num_cus = cfg.num_cus;
    p.tiles_packed = 0;
    p.packed_bytes = 0;
    if (is_bf16 && !direct_s(tl)) {
        p.tiles_packed = ceil_div(M, 16);          // real tiles only: blocks never fetch the padding
        p.packed_bytes = static_cast<size_t>(ceil_div(N, kStep)) * static_cast<size_t>(p.tiles_packed) * 1024;
    }
    p.ws_bytes = p.partial_bytes + p.packed_bytes;
    // Chunks of 128 tokens dealt to the splits round-robin (see wgrad_partial_mfma_kernel) when a block's
    // 32-bit offsets can span the whole arrays; otherwise every split keeps a contiguous range.
    const double lim = 2147483648.0 - 16777216.0;
    p.cyclic = is_bf16 && env_int("VELORA_WGRAD_CYCLIC", 1) != 0 &&
               static_cast<double>(N) * static_cast<double>(O) * 2.0 < lim &&
               static_cast<double>(N) * static_cast<double>(M) * 2.0 < lim && static_cast<double>(p.packed_bytes) < lim;
    return p;
}
}  // namespace

namespace {

// pack (if needed) + partial kernel: leaves partial[splits][O][Mp] in the workspace
hipError_t launch_partials(const void* G, const void* S, int64_t N, int64_t O, int64_t M, bool is_bf16, int g_align,
                           int s_align, void* ws, const WgradPlan& plan, int phases, hipStream_t st) {
    float* partial = static_cast<float*>(ws);
    hipError_t e = hipSuccess;
    bool done = false;
    if (is_bf16 && env_int("VELORA_WGRAD_FORCE_SIMPLE", 0) == 0) {
        const MfmaChoice ch = choose_mfma(O, M, g_align, s_align, plan);
        // Four group tiles: loader waves, S straight from S[N, M], no re-layout pre-pass (N * M even for the
        // same reason as in dispatch_mfma): 28.6 against 36.2 us on N = 16384, O = 4096, M = 64 and 35.6
        // against 42.6 us on O = 5120, M = 54, pre-pass included.  Five and six tiles: the same kernel when
        // every block is resident at once (at most one per compute unit), where the per-wave kernel's four
        // waves are all a compute unit has to hide latency with (O = 5120: 59.7 against 65.0 us at M = 74,
        // 65.9 against 67.2 us at M = 80); with several rounds of blocks it is level or behind
        // (O = 13824, M = 80: 147 against 144 us), so those stay with the per-wave kernel.
        // (measurement builds: VELORA_WGRAD_WS=0 never, 2 for every launch with four to six tiles)
        const int ws_mode = env_int("VELORA_WGRAD_WS", 1);
        if (ch.cw == 8 && !ch.shared && (ch.gt == 4 || ch.gt == 5) && ch.chunks == 1 && ch.s_align16 && (N * M) % 2 == 0 &&
            ws_mode != 0 && wide_tiles(tiling_for(M), O, plan.num_cus)) {
            if (!(phases & 2)) return hipSuccess;
            if (ch.gt == 4) return launch_ws256<4>(G, S, partial, N, O, M, plan, st);
            return launch_ws256<5>(G, S, partial, N, O, M, plan, st);
        }
        const bool one_round = ceil_div(O, 128) * plan.splits <= plan.num_cus;
        const int ws64_max_gt = ws_mode == 2 || one_round ? 6 : 4;
        if (ch.cw == 8 && !ch.shared && ch.gt >= 4 && ch.gt <= ws64_max_gt && ch.chunks == 1 && ch.s_align16 &&
            (N * M) % 2 == 0 && ws_mode != 0) {
            if (!(phases & 2)) return hipSuccess;
            if (ch.gt == 4) return launch_ws64<4>(G, S, partial, N, O, M, plan, st);
            if (ch.gt == 5) return launch_ws64<5>(G, S, partial, N, O, M, plan, st);
            return launch_ws64<6>(G, S, partial, N, O, M, plan, st);
        }
        if (ch.cw != 0) {
            const void* s_operand = S;
            if (plan.tiles_packed > 0) {
                uint4* packed = reinterpret_cast<uint4*>(static_cast<char*>(ws) + plan.partial_bytes);
                const int64_t total = ceil_div(N, kStep) * plan.tiles_packed * 64;
                if (phases & 1)
                    hipLaunchKernelGGL(wgrad_pack_s_kernel, dim3(static_cast<unsigned>(ceil_div(total, 256))), dim3(256),
                                       0, st, static_cast<const uint16_t*>(S), packed, N, M, plan.tiles_packed, total);
                e = hipGetLastError();
                if (e != hipSuccess) return e;
                s_operand = packed;
            }
            if (phases & 2) e = dispatch_mfma(ch, G, s_operand, partial, N, O, M, plan, st, &done);
            else done = true;
            if (e != hipSuccess) return e;
        }
    }
    if (!done && !is_bf16 && env_int("VELORA_WGRAD_FORCE_SIMPLE", 0) == 0 && f32_mfma_ok(O, M, g_align, plan)) {
        if (!(phases & 2)) return hipSuccess;
        return launch_f32_mfma(G, S, partial, N, O, M, plan, st);
    }
    if (!done) {
        e = is_bf16 ? launch_simple<Bf16Elem>(G, S, partial, N, O, M, plan, st)
                    : launch_simple<F32Elem>(G, S, partial, N, O, M, plan, st);
    }
    return e;
}

hipError_t expand_any(const float* partial, int splits, int64_t Mp, const float* v, int v_align, void* dW,
                      bool dw_bf16, int dw_align, bool accumulate, int64_t O, int64_t D, int64_t M, hipStream_t st) {
    const int64_t d = D / M;
    const bool vec = (d % 4 == 0) && v_align >= 16 && dw_align >= (dw_bf16 ? 8 : 16);
    if (dw_bf16) {
        return vec ? launch_expand<true, true>(partial, splits, Mp, v, dW, O, D, M, accumulate, dw_align >= 16, st)
                   : launch_expand<true, false>(partial, splits, Mp, v, dW, O, D, M, accumulate, false, st);
    }
    return vec ? launch_expand<false, true>(partial, splits, Mp, v, dW, O, D, M, accumulate, true, st)
               : launch_expand<false, false>(partial, splits, Mp, v, dW, O, D, M, accumulate, dw_align >= 16, st);
}

}  // namespace

// T[o, g] = sum over splits of partial[split][o][g], fixed order; T is dense [O, M].
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const float* __restrict__ partial, float* __restrict__ T,
                                                          int splits, int64_t O, int64_t M, int64_t Mp) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i >= O * M) return;
    const int64_t o = i / M, g = i - o * M;
    const float* p = partial + o * Mp + g;
    const int64_t stride = O * Mp;
    float s = 0.f;
    int sp = 0;
    for (; sp + 8 <= splits; sp += 8) {           // eight loads in flight; the additions keep their order
        float t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) t[u] = p[(sp + u) * stride];
#pragma unroll
        for (int u = 0; u < 8; ++u) s += t[u];
    }
    for (; sp < splits; ++sp) s += p[sp * stride];
    T[i] = s;
}

namespace {

template <bool OUT_BF16, int VW>
hipError_t launch_expand_sweep(const float* partial, int splits, int64_t split_stride, size_t part_bytes, int64_t t_stride,
                               const float* v, void* dW, int64_t O, int64_t D, int64_t M, bool accumulate,
                               const LaunchCfg& cfg, hipStream_t st) {
    const int64_t n_vec = O * D / VW;
    const uint32_t dv = static_cast<uint32_t>(D / M / VW);
    int64_t blocks = cfg.num_cus;                                // one block per compute unit
    if (blocks > ceil_div(n_vec, 256)) blocks = ceil_div(n_vec, 256);
    const uint32_t dv_inv = static_cast<uint32_t>(4294967296ull / dv) + 1u;   // exact x / dv for x * dv < 2^32
    auto go = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, st, partial,
                           static_cast<uint32_t>(split_stride * 4), static_cast<uint32_t>(part_bytes), v, dW,
                           static_cast<uint32_t>(n_vec), dv, dv_inv, static_cast<uint32_t>(M),
                           static_cast<uint32_t>(t_stride), static_cast<uint32_t>(O * M));
        return hipGetLastError();
    };
    if (splits <= 8)
        return accumulate ? go(wgrad_expand_sweep_kernel<OUT_BF16, VW, 1, true>)
                          : go(wgrad_expand_sweep_kernel<OUT_BF16, VW, 1, false>);
    return accumulate ? go(wgrad_expand_sweep_kernel<OUT_BF16, VW, 2, true>)
                      : go(wgrad_expand_sweep_kernel<OUT_BF16, VW, 2, false>);
}

// dW (+)= (sum over splits of partial[split]) (x) v, rows of partial `t_stride` floats apart: the window
// sweep when its vectors fit the shape and the pointers, else the row-by-row kernel.
hipError_t expand_best(const float* partial, int splits, int64_t t_stride, const float* v, int v_align, void* dW,
                       bool dw_bf16, int dw_align, bool accumulate, int64_t O, int64_t D, int64_t M,
                       const LaunchCfg& cfg, hipStream_t st) {
    const int64_t d = D / M;
    const double lim = 2147483648.0 - 16777216.0;
    const size_t part_bytes = static_cast<size_t>(splits) * static_cast<size_t>(O) * static_cast<size_t>(t_stride) * 4;
    // sixteen split strides stay below 2^30 bytes: the offsets of the splits a kernel asks for beyond
    // the last real one then land past the end of the descriptor (zeros) without wrapping around
    // Rows of 32 KB and more: measured against the row-by-row kernel on whole calls, alternating in one
    // process, the sweep is ahead on every such layer shape (-2.4 us on 4096 x 11008 with M = 43,
    // -3.6 us with M = 64, -4.4 us on 5120 x 13824 with M = 54, -7.4 us with M = 216); with shorter rows
    // the many small blocks of the row kernel interleave as well (-1.8 .. +0.9 us for the sweep on the
    // 4096- and 5120-wide layers, no trend).
    const int sweep_mode = env_int("VELORA_WGRAD_SWEEP", 1);   // measurement builds: 0 never, 2 whenever it fits
    // bf16 output: the sweep is ahead at every row length it was measured on (whole calls, N = 16384:
    // 4096 x 11008: 49.5 -> 45.0 us; 5120 x 13824: 61.7 -> 58.2 us at M = 54, 96.8 -> 93.3 us at M = 216;
    // 4096 x 4096, M = 32: 37.1 -> 35.5; 5120 x 5120: 45.0 -> 43.0 at M = 20, 53.5 -> 50.1 at M = 80;
    // 11008 x 4096, M = 32: 76.9 -> 75.0; 2048 x 768, N = 65536: 48.4 -> 47.3; level on 3072 x 768), so it
    // runs whenever the shape fits it.  float32 rows of 22-28 KB: no trend.
    const bool long_rows = dw_bf16 || D * 4 >= 32768;
    const bool fits = static_cast<double>(O) * static_cast<double>(D) / 4.0 < lim &&
                      static_cast<double>(O) * static_cast<double>(t_stride) <= 16777216.0 && splits <= 16 && d <= 2048 &&
                      (sweep_mode == 2 || (sweep_mode == 1 && long_rows));
    if (fits) {
        const int64_t ss = O * t_stride;
        if (!dw_bf16 && d % 4 == 0 && d / 4 >= 16 && dw_align >= 16)
            return launch_expand_sweep<false, 4>(partial, splits, ss, part_bytes, t_stride, v, dW, O, D, M, accumulate, cfg, st);
        if (dw_bf16 && d % 8 == 0 && d / 8 >= 16 && dw_align >= 16)
            return launch_expand_sweep<true, 8>(partial, splits, ss, part_bytes, t_stride, v, dW, O, D, M, accumulate, cfg, st);
        if (dw_bf16 && d % 4 == 0 && d / 4 >= 16 && dw_align >= 8)
            return launch_expand_sweep<true, 4>(partial, splits, ss, part_bytes, t_stride, v, dW, O, D, M, accumulate, cfg, st);
    }
    return expand_any(partial, splits, t_stride, v, v_align, dW, dw_bf16, dw_align, accumulate, O, D, M, st);
}

}  // namespace

hipError_t launch_wgrad(const void* G, const void* S, const float* v, int64_t N, int64_t O, int64_t D, int64_t M,
                        bool is_bf16, int g_align, int s_align, int v_align, void* dW, bool dw_bf16, int dw_align,
                        bool accumulate, void* ws, const WgradPlan& plan, const LaunchCfg& cfg, hipStream_t st) {
    const int phases = env_int("VELORA_WGRAD_PHASES", 7);   // tuning aid: 1 pack, 2 partial, 4 expand
    hipError_t e = launch_partials(G, S, N, O, M, is_bf16, g_align, s_align, ws, plan, phases, st);
    if (e != hipSuccess) return e;
    if (!(phases & 4)) return hipSuccess;
    return expand_best(static_cast<const float*>(ws), plan.splits, plan.Mp, v, v_align, dW, dw_bf16, dw_align, accumulate,
                       O, D, M, cfg, st);
}

hipError_t launch_wgrad_factor(const void* G, const void* S, int64_t N, int64_t O, int64_t M, bool is_bf16,
                               int g_align, int s_align, float* T, void* ws, const WgradPlan& plan, hipStream_t st) {
    hipError_t e = launch_partials(G, S, N, O, M, is_bf16, g_align, s_align, ws, plan, 7, st);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(wgrad_reduce_kernel, dim3(static_cast<unsigned>(ceil_div(O * M, 256))), dim3(256), 0, st,
                       static_cast<const float*>(ws), T, plan.splits, O, M, plan.Mp);
    return hipGetLastError();
}

hipError_t launch_expand_factor(const float* T, const float* v, int v_align, void* dW, bool dw_bf16, int dw_align,
                                bool accumulate, int64_t O, int64_t D, int64_t M, const LaunchCfg& cfg, hipStream_t st) {
    return expand_best(T, 1, M, v, v_align, dW, dw_bf16, dw_align, accumulate, O, D, M, cfg, st);
}

}  // namespace velora
