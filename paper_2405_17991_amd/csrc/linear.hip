// Forward linear layer with the compression taken from the same tiles (paper
// Listing 1, forward: out = input @ weight^T next to compress(group(input), v)
// of Sec. 3.1).  Y[N, O] = X[N, D] * W[O, D]^T as a bf16 MFMA GEMM whose LDS
// tiles of X also feed the dot with v, so X is read from HBM once for both.
//
// GEMM.  Block tile 256 tokens x 256 outputs x 64 k, four waves in a 2 x 2 grid
// (wave tile 128 x 128 = 8 x 8 MFMA tiles of 16 x 16, 256 accumulator
// registers).  Both operands are k-contiguous, so a 16-byte piece of a row is
// already an MFMA fragment; LDS rows are 128 bytes, eight 16-byte chunks, chunk
// c of row r stored at position c ^ ((r >> 1) & 7), which makes both the linear
// writes and the fragment reads (16 rows x one chunk) bank-conflict free.
// Two LDS stages (2 x 64 KB).  A step needs 512 cache lines per block and a CU
// keeps about 70 requests of 128 B outstanding (300-500 cycles from L2), so the
// request queue must never drain at a wait point and loads must not arrive in
// bursts (a wave that cannot issue a load issues no MFMA either).  A step is two
// halves of 64 MFMAs (eight rows of eight); after every row come two LDS reads
// of the next half's fragments (fragments are double-buffered in registers) and
// one instruction of each load stream:
//   W tiles: pass through registers.  First half of step t: piece i of W(t+1)
//            goes from registers to its LDS stage, then a load refills the
//            register with W(t+2) (a full step in flight);
//   A tiles: global -> LDS directly (buffer_load ... lds) during the second half
//            of step t (for step t+2), awaited at the middle of step t+1.
// One barrier per step, between the halves: before it every wave has finished
// reading stage t&1 (its fragments for the second half are in registers) and
// has A(t+1) and W(t+1) in stage (t+1)&1 (s_waitcnt vmcnt(8): the eight younger
// loads are W(t+2); vector-memory operations complete in order).
// The MFMAs are inline assembly with the accumulators tied to AGPRs.  With the
// builtin, the register allocator starts to move accumulators between the two
// register files as soon as other instructions sit between the MFMAs (hundreds
// of copies per step, or spills); tied to AGPRs the 256 accumulators stay put
// and the loop is exactly the sequence written here.  The counted wait stays
// correct if the compiler adds vector-memory operations (a spill) inside the
// loop, since it only needs eight younger loads behind the batch it waits for,
// but each such operation costs overlap: v is therefore staged in LDS before
// the loop, and the build rejects register spills in this kernel.
// Block order: consecutive block ids land on different XCDs (one L2 each), so
// XCD x takes a contiguous run of tile ids, and ids are laid out in groups of
// four token tiles (output tiles outer): the 32 blocks an XCD runs together
// cover about 4 token tiles x 8 output tiles.
//
// Compression inside the GEMM.  The blocks of a token tile share out
// S[n, g] = <X[n, g*d : (g+1)*d], v>: the block of output tile `to` takes the
// sub-tokens g with g % To == to (To output tiles), so the extra work is spread
// evenly.  v is split into two bf16 parts, v = hi + lo (|v - hi - lo| <=
// 2^-17 |v|), which become rows 0 and 1 of an otherwise zero 16-row A operand;
// one extra MFMA per token tile and 32-k half multiplies it with the X
// fragments that are in registers anyway, accumulating in float32, and rows
// 0 + 1 of the result are the dot.  d must be a multiple of 64 (a k-step then
// lies inside one sub-token) and at most 2048.
//
// Everything the MFMA kernel cannot take (float32, d or D not a multiple of 64,
// unaligned pointers) goes to a plain tiled FMA kernel plus the stand-alone
// compress kernel.
#include "common.h"
#include "kernels.h"

#include <atomic>
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

// One block's tile of  Out[R, C] = A[R, K] * B,  A k-contiguous (X, or grad_output).
//   NN = false: B = W[C, K], k-contiguous (the forward: Out = X W^T)
//   NN = true:  B = W[K, C], c-contiguous (the backward: grad_input = grad_output W).  The W stream passes
//               through registers anyway, so a thread fetches an 8 k x 8 column block (eight 16-byte row
//               pieces), transposes it in registers (v_perm_b32) and writes eight ready operands into
//               the k-contiguous LDS layout of the forward; everything after that is the same code.
//   DO_S: this block also forms its share of S for its 256 rows (forward only).
template <bool DO_S, bool NN>
__device__ __forceinline__ void linear_tile(char* lds, const uint16_t* __restrict__ A, const uint16_t* __restrict__ W,
                                            const float* __restrict__ v, uint16_t* __restrict__ Out,
                                            uint16_t* __restrict__ S, int R, int C, int K, int d, int64_t n0,
                                            int64_t o0) {
    static_assert(!(DO_S && NN), "S belongs to the forward");
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int wm = w >> 1, wn = w & 1;
    const int q = lane >> 4, jj = lane & 15;
    // Range-checked descriptors over this block's rows: rows past R (or C) read as zeros.
    const int rows_x = R - n0 < kBM ? static_cast<int>(R - n0) : kBM;
    const int rows_w = C - o0 < kBN ? static_cast<int>(C - o0) : kBN;
    __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t*>(A + n0 * K), 0, static_cast<int>(static_cast<int64_t>(rows_x) * K * 2), 0x00020000);
    // One wave instruction moves 1 KB; wave w owns a quarter of each tile.
    // k-contiguous tiles: 8 rows x 128 B per instruction; lane -> row-in-8 = lane / 8, stored chunk = lane % 8,
    // loaded chunk = stored ^ ((row >> 1) & 7).
    uint32_t gvoff[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int row = w * 64 + i * 8 + (lane >> 3);
        const int chunk = (lane & 7) ^ ((row >> 1) & 7);
        gvoff[i] = static_cast<uint32_t>(row) * static_cast<uint32_t>(K) * 2u + static_cast<uint32_t>(chunk) * 16u;
    }
    // c-contiguous W tile (NN): thread -> k group tid % 8 (rows 8kg .. 8kg+7), column chunk tid / 8 (8 columns);
    // a chunk past the last column gets an offset no descriptor covers
    const int kg = tid & 7, chunk_w = tid >> 3;
    const uint32_t wvoff_nn = o0 + chunk_w * 8 < C ? static_cast<uint32_t>(kg * 8) * static_cast<uint32_t>(C) * 2u +
                                                         static_cast<uint32_t>(chunk_w) * 16u
                                                   : 0xFFFFFFFFu;
    const int nk = K / kBK;
    // steps past the end re-fetch the last k block into the (free) stage: the counted waits stay uniform
    auto w_rsrc = [&](int tc) -> __amdgpu_buffer_rsrc_t {
        if constexpr (NN) {   // the 64 k rows of step tc, from column o0 to the end of the last row
            return __builtin_amdgcn_make_buffer_rsrc(
                const_cast<uint16_t*>(W + static_cast<int64_t>(tc) * kBK * C + o0), 0,
                static_cast<int>((static_cast<int64_t>(kBK) * C - o0) * 2), 0x00020000);
        } else {
            return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(W + o0 * K), 0,
                                                     static_cast<int>(static_cast<int64_t>(rows_w) * K * 2), 0x00020000);
        }
    };
    auto dma_x = [&](int t) {
        char* st = lds + (t & 1) * kStage;
        const int koff = (t < nk ? t : nk - 1) * kBK * 2;
#pragma unroll
        for (int i = 0; i < 8; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, to_lds(st + (w * 64 + i * 8) * kRowB), 16, gvoff[i], koff, 0, 0);
    };
    auto dma_w = [&](int t) {                     // NT only
        char* st = lds + (t & 1) * kStage + kBM * kRowB + w * (kBN * kRowB / 4);
        const int tc = t < nk ? t : nk - 1;
        const __amdgpu_buffer_rsrc_t rw = w_rsrc(tc);
#pragma unroll
        for (int i = 0; i < 8; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, to_lds(st + i * 1024), 16, gvoff[i], tc * kBK * 2, 0, 0);
    };
    // The W stream passes through registers.
    u32x4 wregP[8], wregQ[8];
    auto load_w_piece = [&](u32x4& r, int i, const __amdgpu_buffer_rsrc_t& rw, int tc) {
        r = NN ? __builtin_amdgcn_raw_buffer_load_b128(rw, wvoff_nn, i * C * 2, 0)        // row 8kg + i
               : __builtin_amdgcn_raw_buffer_load_b128(rw, gvoff[i], tc * kBK * 2, 0);
    };
    // NN: dword j of column i's fragment (rows 2j, 2j+1 of the 8 x 8 block share it); v_perm_b32 selector bytes
    // 0-3 pick from the second operand, 4-7 from the first
    auto w_column_dword = [&](const u32x4 (&wr)[8], int i, int j) -> uint32_t {
        const uint32_t lo = wr[2 * j][i >> 1], hi = wr[2 * j + 1][i >> 1];
        return (i & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u) : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
    };
    // piece i of the W tile of step t, from registers to its LDS stage.  NT: the 16 bytes as loaded.  NN: `col`
    // holds column 8*chunk + i of the 8 x 8 block, which is k chunk kg of LDS row 8*chunk + i (swizzled as above).
    auto store_w_piece = [&](const u32x4 (&wr)[8], const u32x4& col, int i, int t) {
        if constexpr (NN) {
            char* st = lds + (t & 1) * kStage + kBM * kRowB;
            const int n = chunk_w * 8 + i;
            *reinterpret_cast<u32x4*>(st + n * kRowB + ((kg ^ ((n >> 1) & 7)) * 16)) = col;
        } else {
            char* st = lds + (t & 1) * kStage + kBM * kRowB + w * (kBN * kRowB / 4);
            *reinterpret_cast<u32x4*>(st + i * 1024 + lane * 16) = wr[i];
        }
    };
    // fragment of rows base + 16b + jj, chunk 4*kk + q; (row >> 1) & 7 == (jj >> 1) & 7 because base is a multiple of 16
    uint32_t foff[2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
        foff[kk] = static_cast<uint32_t>(jj) * kRowB + static_cast<uint32_t>(((kk * 4 + q) ^ ((jj >> 1) & 7)) * 16);
    auto fread_x = [&](int b, int t, int kk) -> bf16x8 {
        return *reinterpret_cast<const bf16x8*>(lds + (t & 1) * kStage + (wm * 128 + b * 16) * kRowB + foff[kk]);
    };
    auto fread_w = [&](int a, int t, int kk) -> bf16x8 {
        return *reinterpret_cast<const bf16x8*>(lds + (t & 1) * kStage + (kBM + wn * 128 + a * 16) * kRowB + foff[kk]);
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

    // A operand with v: row 0 = hi, row 1 = lo, rows 2..15 zero; k = 8q .. 8q+7 of this 32-k half
    auto v_fragment = [&](int kpos, int kk) -> bf16x8 {      // kpos: the step's first k inside its sub-token
        const int vk = kpos + kk * 32 + q * 8;
        const u32x4 raw = *reinterpret_cast<const u32x4*>(vtab + (jj & 1) * d + vk);
        const u32x4 zero = {0u, 0u, 0u, 0u};
        return __builtin_bit_cast(bf16x8, jj < 2 ? raw : zero);
    };
    // Four more MFMAs per half with accumulators in ordinary VGPRs (the AGPRs are full), written like the main
    // ones (see below).  The compiler does not know that this statement holds MFMAs, and it may put register
    // copies or the select of v_fragment right next to it, so the statement brings its own wait states: a few
    // before the first MFMA (operands just written by vector instructions) and 20 after the last (its result
    // may be read by a vector instruction; 19 is the most this chip asks for).  The matrix pipe works through
    // the four MFMAs meanwhile.
#define VELORA_S_MFMAS(X0, X1, X2, X3)                                                                          \
    asm volatile("s_nop 3\n\t"                                                                                \
                 "v_mfma_f32_16x16x32_bf16 %0, %4, %5, %0\n\t"                                                \
                 "v_mfma_f32_16x16x32_bf16 %1, %4, %6, %1\n\t"                                                \
                 "v_mfma_f32_16x16x32_bf16 %2, %4, %7, %2\n\t"                                                \
                 "v_mfma_f32_16x16x32_bf16 %3, %4, %8, %3\n\t"                                                \
                 "s_nop 15\n\ts_nop 3"                                                                        \
                 : "+v"(acc_s[0]), "+v"(acc_s[1]), "+v"(acc_s[2]), "+v"(acc_s[3])                               \
                 : "v"(vf), "v"(X0), "v"(X1), "v"(X2), "v"(X3))
    auto mma_s = [&](const bf16x8 (&fx)[8], const bf16x8& vf) {
        if (wn == 0) {
            VELORA_S_MFMAS(fx[0], fx[1], fx[2], fx[3]);
        } else {
            VELORA_S_MFMAS(fx[4], fx[5], fx[6], fx[7]);
        }
    };
#undef VELORA_S_MFMAS
    // lane (jj, q = 0) holds rows 0..3 of the result for token jj: S = row 0 + row 1
    auto flush_s = [&](int g) {
        const int M = K / d;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int64_t n = n0 + wm * 128 + (wn * 4 + b) * 16 + jj;
            if (q == 0 && n < R) S[n * M + g] = f32_to_bf16(acc_s[b][0] + acc_s[b][1]);
            acc_s[b] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        asm volatile("s_nop 7" ::: "memory");
    };

    // Half a step: 64 MFMAs in eight rows (one W fragment against the eight token fragments).  Behind the first
    // MFMAs of every row, one each (an instruction that follows an MFMA issues while the matrix pipe works on
    // it; a group of several costs about five cycles apiece), come two LDS reads of the next half's fragments
    // (token fragments first: row 0 of the next half needs all eight; then the W fragments in row order) and
    // this half's share of the two load streams:
    //   first half  (SECOND = false): one piece of the W tile held in registers (step tl - 1) goes to its LDS
    //                                 stage, and one load of step tl refills that register (NN: the other set)
    //   second half (SECOND = true):  one direct-to-LDS load of the A tile of step tl
    // The MFMAs are written as inline assembly with the accumulators tied to AGPRs: with the builtin, the
    // register allocator moves accumulators between the two register files as soon as loads are placed
    // between the MFMAs.  The compiler does not know these statements are MFMAs, so it places no wait states
    // for them; none are needed here: an accumulator is touched again 64 MFMAs later at the earliest, the
    // operands come from LDS reads (s_waitcnt, which the compiler does place), and the epilogue waits below.
    auto half = [&](auto second, const bf16x8 (&fx)[8], const bf16x8 (&fw)[8], bf16x8 (&nx)[8], bf16x8 (&nw)[8],
                    int tf, int kf, int tl, u32x4 (&wst)[8], u32x4 (&wld)[8]) {
        constexpr bool SECOND = decltype(second)::value;
        const int tc = tl < nk ? tl : nk - 1;     // steps past the end re-fetch the last k block (never used)
        const __amdgpu_buffer_rsrc_t rw = w_rsrc(tc);
        char* sx = lds + (tl & 1) * kStage;
#pragma unroll
        for (int a = 0; a < 8; ++a) {
            u32x4 col = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int b = 0; b < 8; ++b) {
                asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[a][b]) : "v"(fw[a]), "v"(fx[b]));
                // one other instruction behind an MFMA issues in its shadow; several in a row do not
                if (b < 2) {
                    const int i = a * 2 + b;
                    if (i < 8) nx[i] = fread_x(i, tf, kf);
                    else nw[i - 8] = fread_w(i - 8, tf, kf);
                } else if constexpr (SECOND) {
                    if (b == 2)
                        __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, to_lds(sx + (w * 64 + a * 8) * kRowB), 16, gvoff[a],
                                                                 tc * kBK * 2, 0, 0);
                    if constexpr (NN) {
                        // the refilled register moves over to the set the next step stores from; written as
                        // assembly so that the two moves stay in these slots instead of sinking to the loop's end
                        if (b == 3 || b == 4) {
                            const int h = (b - 3) * 2;
                            const u32x2 src = {wld[a][h], wld[a][h + 1]};
                            u32x2 dst;
                            asm volatile("v_mov_b64 %0, %1" : "=v"(dst) : "v"(src));
                            wst[a][h] = dst[0];
                            wst[a][h + 1] = dst[1];
                        }
                    }
                } else if constexpr (NN) {        // four permutes build the column, then the store and the refill
                    if (b < 6) col[b - 2] = w_column_dword(wst, a, b - 2);
                    else if (b == 6) store_w_piece(wst, col, a, tl - 1);
                    else load_w_piece(wld[a], a, rw, tc);
                } else {
                    if (b == 2) store_w_piece(wst, col, a, tl - 1);
                    else if (b == 3) load_w_piece(wld[a], a, rw, tc);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    constexpr int kWaitVm8Lgkm0 = 0x0078;         // s_waitcnt vmcnt(8) lgkmcnt(0)
    bf16x8 fxA[8], fwA[8], fxB[8], fwB[8];
    // S is shared out over the blocks of a token tile: block `to` takes the sub-tokens g with g % To == to, so
    // every block carries the same small extra (one in To of the steps has the eight extra MFMAs).
    const int To = (C + kBN - 1) / kBN, to = static_cast<int>(o0 / kBN);
    int s_g = 0, s_gmod = 0, s_kpos = 0;          // sub-token of the current step, g % To, first k inside it
    // One step.  On entry: stage t&1 complete, fragments (t, kk0) in set A, W(t+1) in wst (or on its way).
    auto step = [&](int t, u32x4 (&wst)[8], u32x4 (&wld)[8]) {
        const bool s_mine = DO_S && s_gmod == to;   // uniform
        if constexpr (DO_S) {
            if (__builtin_expect(s_mine, false)) mma_s(fxA, v_fragment(s_kpos, 0));
        }
        __builtin_amdgcn_sched_barrier(0);
        // MFMAs (t, kk0); reads (t, kk1); W(t+1) -> stage (t+1)&1 (free since the previous barrier); W(t+2) -> registers
        half(std::false_type{}, fxA, fwA, fxB, fwB, t, 1, t + 2, wst, wld);
        __builtin_amdgcn_s_waitcnt(kWaitVm8Lgkm0);   // A(t+1) landed (the eight younger loads are W(t+2)); this wave's
                                                     // LDS reads and its W(t+1) writes are done
        __syncthreads();                          // stage t&1 is free, stage (t+1)&1 is complete
        if constexpr (DO_S) {
            if (__builtin_expect(s_mine, false)) mma_s(fxB, v_fragment(s_kpos, 1));
        }
        __builtin_amdgcn_sched_barrier(0);
        // MFMAs (t, kk1); reads (t+1, kk0) (past the end: a stage nobody uses); A(t+2) -> stage t&1
        half(std::true_type{}, fxB, fwB, fxA, fwA, t + 1, 0, t + 2, wst, wld);
        if constexpr (DO_S) {
            s_kpos += kBK;
            if (__builtin_expect(s_kpos == d, false)) {   // the sub-token ends with this step
                if (s_mine) flush_s(s_g);
                s_kpos = 0;
                ++s_g;
                s_gmod = s_gmod + 1 == To ? 0 : s_gmod + 1;
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    dma_x(0);
    if constexpr (NN) {
        const __amdgpu_buffer_rsrc_t rw0 = w_rsrc(0);
#pragma unroll
        for (int i = 0; i < 8; ++i) load_w_piece(wregQ[i], i, rw0, 0);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const u32x4 col = {w_column_dword(wregQ, i, 0), w_column_dword(wregQ, i, 1), w_column_dword(wregQ, i, 2),
                               w_column_dword(wregQ, i, 3)};
            store_w_piece(wregQ, col, i, 0);
        }
    } else {
        dma_w(0);
    }
    dma_x(1);
    {
        const int tc = nk > 1 ? 1 : 0;
        const __amdgpu_buffer_rsrc_t rw1 = w_rsrc(tc);
#pragma unroll
        for (int i = 0; i < 8; ++i) load_w_piece(wregP[i], i, rw1, tc);
    }
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(0);                // the first tiles have landed, W(1) is in registers
    __syncthreads();                              // (also publishes vtab)
#pragma unroll
    for (int b = 0; b < 8; ++b) fxA[b] = fread_x(b, 0, 0);
#pragma unroll
    for (int a = 0; a < 8; ++a) fwA[a] = fread_w(a, 0, 0);
    // Nothing is pending when the loop starts: the compiler merges the counters' state at this entry with the
    // state at the back edge, and reads still outstanding here would make it wait for more at the top of
    // every step.
    __builtin_amdgcn_s_waitcnt(0);
    __builtin_amdgcn_sched_barrier(0);
    for (int t = 0; t < nk; ++t) {
        // NN: the column of piece i is built from all eight registers of the tile, so the refill goes to a second
        // set, which moves over during the second half (it was requested in the first).  NT: piece i is stored,
        // then refilled in place.
        if constexpr (NN) step(t, wregP, wregQ);
        else step(t, wregP, wregP);
    }
    __builtin_amdgcn_s_waitcnt(0);                // nothing of this block is in flight when its LDS is released
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");   // the last MFMAs have written the accumulators read below

    // D[i = output 4q + r][j = token jj] per tile: four consecutive outputs of one token per lane.
    if (C % 8 == 0) {
        // Through LDS, so that the tile leaves in 16-byte stores that fill whole 128-byte pieces of a row
        // (8-byte stores in 32-byte runs cost 1.3-1.7 times the bytes at the memory): in two passes of 64
        // outputs the wave writes its 128 tokens x 64 outputs into its own region (rows 144 bytes apart,
        // which spreads the 16 tokens of a tile over the banks), reads 16-byte pieces back, eight lanes per
        // row, and stores them.  LDS serves a wave's operations in order, so the region needs no barrier
        // of its own; the one below is for the stages it overlays.
        __syncthreads();                          // every wave has read its last fragments
        char* ep = lds + w * (128 * 144);
        // stores through a descriptor over this tile's valid rows: rows past R fall outside it and are
        // dropped; a lane whose eight outputs lie past C gets an offset outside every descriptor
        const __amdgpu_buffer_rsrc_t ro = __builtin_amdgcn_make_buffer_rsrc(
            Out + n0 * C, 0, static_cast<int>(static_cast<int64_t>(rows_x) * C * 2), 0x00020000);
        const uint32_t row_off = static_cast<uint32_t>(wm * 128 + (lane >> 3)) * static_cast<uint32_t>(C) * 2u;
#pragma unroll
        for (int p = 0; p < 2; ++p) {
#pragma unroll
            for (int a4 = 0; a4 < 4; ++a4)
#pragma unroll
                for (int b = 0; b < 8; ++b) {
                    const f32x4& c = acc[p * 4 + a4][b];
                    const u32x2 out = {pack_bf16x2(c[0], c[1]), pack_bf16x2(c[2], c[3])};
                    *reinterpret_cast<u32x2*>(ep + (b * 16 + jj) * 144 + a4 * 32 + q * 8) = out;
                }
            __builtin_amdgcn_sched_barrier(0);
            const int64_t o = o0 + wn * 128 + p * 64 + (lane & 7) * 8;
            const uint32_t col_off = o < C ? row_off + static_cast<uint32_t>(o) * 2u : 0xFFFFFFFFu;
            u32x4 piece[16];
#pragma unroll
            for (int i = 0; i < 16; ++i)
                piece[i] = *reinterpret_cast<const u32x4*>(ep + (i * 8 + (lane >> 3)) * 144 + (lane & 7) * 16);
#pragma unroll
            for (int i = 0; i < 16; ++i)
                __builtin_amdgcn_raw_buffer_store_b128(
                    piece[i], ro, o < C ? col_off + static_cast<uint32_t>(i * 8) * static_cast<uint32_t>(C) * 2u : 0xFFFFFFFFu,
                    0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    } else {
#pragma unroll
        for (int a = 0; a < 8; ++a)
#pragma unroll
            for (int b = 0; b < 8; ++b) {
                const int64_t n = n0 + wm * 128 + b * 16 + jj, o = o0 + wn * 128 + a * 16 + q * 4;
                if (n < R && o < C) {   // C % 4 == 0: a lane's four outputs are all inside or all outside
                    const u32x2 out = {pack_bf16x2(acc[a][b][0], acc[a][b][1]), pack_bf16x2(acc[a][b][2], acc[a][b][3])};
                    *reinterpret_cast<u32x2*>(Out + n * C + o) = out;
                }
            }
    }
}

// Out[R, C] = A[R, K] * W^T (NN = false, W[C, K]) or A * W (NN = true, W[K, C]); FUSE: S = compress(A, v) as well.
template <bool FUSE, bool NN>
__global__ __launch_bounds__(256) void linear_mfma_kernel(const uint16_t* __restrict__ A, const uint16_t* __restrict__ W,
                                                         const float* __restrict__ v, uint16_t* __restrict__ Out,
                                                         uint16_t* __restrict__ S, int R, int C, int K, int d) {
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    const int To = (C + kBN - 1) / kBN, Tn = (R + kBM - 1) / kBM, T = To * Tn;
    const int per_xcd = (T + 7) / 8;
    const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3;
    const int vid = xcd * per_xcd + idx;
    if (idx >= per_xcd || vid >= T) return;       // whole block, before any barrier
    // grouped order: four token tiles at a time, output tiles outer, so 32 consecutive ids (what one XCD runs
    // together) touch about 4 + 8 distinct operand tiles per k step instead of 1 + 32
    constexpr int kGroup = 4;
    const int in_group = kGroup * To;
    const int first_tn = (vid / in_group) * kGroup;
    const int group_rows = Tn - first_tn < kGroup ? Tn - first_tn : kGroup;
    const int tn = first_tn + (vid % in_group) % group_rows, to = (vid % in_group) / group_rows;
    const int64_t n0 = static_cast<int64_t>(tn) * kBM, o0 = static_cast<int64_t>(to) * kBN;
    linear_tile<FUSE, NN>(lds, A, W, v, Out, S, R, C, K, d, n0, o0);
}

// Any dtype, size and alignment: 64 x 64 output tile per block, 16-k slices through LDS, a 4 x 4 patch
// per thread, float32 FMA.  Not tuned; it exists so that every shape has a result.
// Out[R, C] = A[R, K] * W^T (W[C, K]) or, NN, A * W (W[K, C]).
template <typename E, bool NN>
__global__ __launch_bounds__(256) void linear_generic_kernel(const typename E::type* __restrict__ A,
                                                            const typename E::type* __restrict__ W,
                                                            typename E::type* __restrict__ Out, int64_t R, int64_t C,
                                                            int64_t K) {
    __shared__ float xs[16][64 + 1], ws[16][64 + 1];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int64_t n0 = static_cast<int64_t>(blockIdx.x) * 64, o0 = static_cast<int64_t>(blockIdx.y) * 64;
    float acc[4][4] = {};
    for (int64_t k0 = 0; k0 < K; k0 += 16) {
        for (int i = threadIdx.x; i < 64 * 16; i += 256) {
            const int r = i >> 4, k = i & 15;
            xs[k][r] = (k0 + k < K && n0 + r < R) ? E::load(A, (n0 + r) * K + k0 + k) : 0.f;
            if constexpr (NN) {
                const int kw = i >> 6, c = i & 63;          // consecutive threads along the contiguous axis
                ws[kw][c] = (k0 + kw < K && o0 + c < C) ? E::load(W, (k0 + kw) * C + o0 + c) : 0.f;
            } else {
                ws[k][r] = (k0 + k < K && o0 + r < C) ? E::load(W, (o0 + r) * K + k0 + k) : 0.f;
            }
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
            if (n < R && o < C) E::store(Out, n * C + o, acc[i][j]);
        }
}

namespace {

// R rows, C output columns, K reduction length.  32-bit tile counts and byte offsets inside a tile.
bool mfma_shape_ok(int64_t R, int64_t C, int64_t K, int c_multiple) {
    return K % kBK == 0 && C % c_multiple == 0 && K <= (1 << 21) && C <= (1 << 21) && R < (int64_t{1} << 31) - kBM &&
           ((R + kBM - 1) / kBM) * ((C + kBN - 1) / kBN) < (int64_t{1} << 28);
}

template <bool FUSE, bool NN>
hipError_t launch_mfma(const void* A, const void* W, const float* v, void* Out, void* S, int64_t R, int64_t C,
                       int64_t K, int64_t d, hipStream_t st) {
    const int64_t tiles = ((R + kBM - 1) / kBM) * ((C + kBN - 1) / kBN);
    const unsigned grid = static_cast<unsigned>((tiles + 7) / 8 * 8);
    const size_t lds_bytes = 2 * static_cast<size_t>(kStage) + (FUSE ? 2 * static_cast<size_t>(d) * 2 : 0);
    // more than 64 KB of dynamic LDS has to be allowed once per kernel and device (the call is not free)
    static std::atomic<bool> allowed[64];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64 || !allowed[dev].load(std::memory_order_acquire)) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&linear_mfma_kernel<FUSE, NN>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 2 * kStage + 4 * kMaxFusedD);
        if (e != hipSuccess) return e;
        if (dev >= 0 && dev < 64) allowed[dev].store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL((linear_mfma_kernel<FUSE, NN>), dim3(grid), dim3(256), lds_bytes, st,
                       static_cast<const uint16_t*>(A), static_cast<const uint16_t*>(W), v, static_cast<uint16_t*>(Out),
                       static_cast<uint16_t*>(S), static_cast<int>(R), static_cast<int>(C), static_cast<int>(K),
                       static_cast<int>(d));
    return hipGetLastError();
}

template <bool NN>
hipError_t launch_generic(const void* A, const void* W, void* Out, int64_t R, int64_t C, int64_t K, bool is_bf16,
                          hipStream_t st) {
    const dim3 grid(static_cast<unsigned>((R + 63) / 64), static_cast<unsigned>((C + 63) / 64));   // C <= 65535 * 64: caller
    if (is_bf16)
        hipLaunchKernelGGL((linear_generic_kernel<Bf16Elem, NN>), grid, dim3(256), 0, st, static_cast<const uint16_t*>(A),
                           static_cast<const uint16_t*>(W), static_cast<uint16_t*>(Out), R, C, K);
    else
        hipLaunchKernelGGL((linear_generic_kernel<F32Elem, NN>), grid, dim3(256), 0, st, static_cast<const float*>(A),
                           static_cast<const float*>(W), static_cast<float*>(Out), R, C, K);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_linear_compress(const void* X, const void* W, const float* v, void* Y, void* S, int64_t N, int64_t D,
                                  int64_t O, int64_t M, bool is_bf16, bool align16, bool s_vec_ok, const LaunchCfg& cfg,
                                  hipStream_t st) {
    const int64_t d = D / M;
    hipError_t e;
    if (is_bf16 && align16 && mfma_shape_ok(N, O, D, 4)) {
        if (d % kBK == 0 && d <= kMaxFusedD) return launch_mfma<true, false>(X, W, v, Y, S, N, O, D, d, st);
        e = launch_mfma<false, false>(X, W, v, Y, S, N, O, D, d, st);
    } else {
        e = launch_generic<false>(X, W, Y, N, O, D, is_bf16, st);
    }
    if (e != hipSuccess) return e;
    return launch_compress(X, v, S, N * M, d, is_bf16, s_vec_ok, cfg, st);
}

hipError_t launch_grad_input(const void* G, const void* W, void* dX, int64_t N, int64_t O, int64_t D, bool is_bf16,
                             bool align16, hipStream_t st) {
    if (is_bf16 && align16 && mfma_shape_ok(N, D, O, 8))
        return launch_mfma<false, true>(G, W, nullptr, dX, nullptr, N, D, O, 0, st);
    return launch_generic<true>(G, W, dX, N, D, O, is_bf16, st);
}

}  // namespace velora
