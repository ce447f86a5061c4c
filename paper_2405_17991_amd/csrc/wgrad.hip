// Weight gradient from compressed activations (paper Algorithm 1, backward:
// grad_weight = grad_output^T @ ungroup(reconstruct(z, v))).
//
// Because the reconstructed input is Xhat[n, g*d + j] = S[n, g] * v[j]
// (Sec. 3.2), the gradient factors exactly:
//     T[o, g]        = sum_n G[n, o] * S[n, g]            (a skinny GEMM, K = N)
//     dW[o, g*d + j] = T[o, g] * v[j]                     (an expansion)
// which needs d times fewer flops than the dense product and never forms Xhat.
// The work is then bound by reading G once and writing dW once, so:
//   kernel 1 streams G exactly once, forms partial T over fixed token ranges
//            (split-K, because T alone is far too small to fill 256 CUs) with
//            bf16 MFMA, and writes the partials to the workspace;
//   kernel 2 sums the partials in a fixed order (deterministic, no float
//            atomics), multiplies by v and streams dW out with 16-byte stores.
#include "common.h"
#include "kernels.h"

#include <cstdlib>

namespace velora {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------
// Kernel 1, MFMA path (bf16 inputs).
//
// v_mfma_f32_16x16x32_bf16 computes D[16x16] += A[16x32] * B[32x16]; lane l
// supplies A[l%16][8*(l/16) + 0..7] and B[8*(l/16) + 0..7][l%16] (eight
// K-consecutive bf16 in four VGPRs) and receives D[4*(l/16) + 0..3][l%16].
// Here K runs over tokens n, A rows over sub-token groups g, B columns over
// output features o.  Both operands are stored with n as the SLOW axis
// (G[n][o], S[n][g]), so the eight K-consecutive values a lane needs are eight
// different rows.  Instead of staging through LDS, a lane loads eight rows x
// C columns (C*2 bytes per row, coalesced across the 16 lanes that share a
// K-group) and transposes the 8 x C block of 16-bit values inside its own
// registers with v_perm_b32; that yields C ready fragments for C different
// columns.  The column a lane/fragment pair stands for is strided
// (o = o0 + jj*CW + c), which is harmless: MFMA rows/columns need not be
// adjacent in memory, the epilogue undoes the mapping.
//
//   CW   G columns per lane (8 -> 16-byte loads, 4 -> 8-byte)
//   CWS  S columns per lane (8, 4, 2 or 1)
//   NS   S load sets; the block covers 16*CWS*NS groups g
// Block = 4 waves; the waves take alternate 32-token steps of the block's token
// range and are summed through LDS at the end in a fixed order.
// grid = (o tiles of 16*CW, splits, g chunks of 16*CWS*NS)
// ---------------------------------------------------------------------------
template <int NDW>
struct RawRow {
    uint32_t w[NDW];
};

// Load C consecutive bf16 (C*2 bytes) from a wave-uniform base plus a 32-bit
// per-lane byte offset, so the address can be formed as SGPR pair + VGPR.
template <int C>
__device__ __forceinline__ RawRow<(C >= 2 ? C / 2 : 1)> load_cols(const char* base, uint32_t voff, bool ok) {
    RawRow<(C >= 2 ? C / 2 : 1)> r;
    const char* p = base + voff;
    if constexpr (C == 8) {
        uint4 q = make_uint4(0u, 0u, 0u, 0u);
        if (ok) q = *reinterpret_cast<const uint4*>(p);
        r.w[0] = q.x; r.w[1] = q.y; r.w[2] = q.z; r.w[3] = q.w;
    } else if constexpr (C == 4) {
        uint2 q = make_uint2(0u, 0u);
        if (ok) q = *reinterpret_cast<const uint2*>(p);
        r.w[0] = q.x; r.w[1] = q.y;
    } else if constexpr (C == 2) {
        r.w[0] = ok ? *reinterpret_cast<const uint32_t*>(p) : 0u;
    } else {
        r.w[0] = ok ? static_cast<uint32_t>(*reinterpret_cast<const uint16_t*>(p)) : 0u;
    }
    return r;
}

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

template <int CW, int CWS, int NS>
struct WgradRaw {
    RawRow<CW / 2> g[8];
    RawRow<(CWS >= 2 ? CWS / 2 : 1)> s[NS][8];
};

template <int CW, int CWS, int NS>
struct WgradFrags {
    bf16x8 g[CW];
    bf16x8 s[NS * CWS];
};

// One 32-token step of this wave.  gptr/sptr are wave-uniform and point at the
// step's first token (row) and the block's first column; gvoff/svoff hold the
// lane's (8*q rows, column) byte offset.  EDGE adds the bounds predicates
// needed for a ragged last step or a partial column tile; out-of-range
// elements read as zero and are never dereferenced.
template <int CW, int CWS, int NS, bool EDGE>
__device__ __forceinline__ void wgrad_load(WgradRaw<CW, CWS, NS>& t, const char* gptr, const char* sptr,
                                           uint32_t gvoff, uint32_t svoff, uint32_t g_row_bytes,
                                           uint32_t s_row_bytes, int rows_left, int q, bool col_ok,
                                           const bool (&g_ok)[NS]) {
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        const bool ok = !EDGE || (col_ok && (q * 8 + r) < rows_left);
        t.g[r] = load_cols<CW>(gptr + static_cast<uint64_t>(r) * g_row_bytes, gvoff, ok);
    }
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const bool ok = g_ok[s] && (!EDGE || (q * 8 + r) < rows_left);
            t.s[s][r] = load_cols<CWS>(sptr + static_cast<uint64_t>(r) * s_row_bytes, svoff + s * 16 * CWS * 2, ok);
        }
}

template <int CW, int CWS, int NS>
__device__ __forceinline__ void wgrad_transpose(const WgradRaw<CW, CWS, NS>& t, WgradFrags<CW, CWS, NS>& f) {
#pragma unroll
    for (int c = 0; c < CW; ++c) f.g[c] = column_fragment(t.g, c);
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
        for (int cs = 0; cs < CWS; ++cs) f.s[s * CWS + cs] = column_fragment(t.s[s], cs);
}

template <int CW, int CWS, int NS>
__device__ __forceinline__ void wgrad_mma(const WgradFrags<CW, CWS, NS>& f, f32x4 (&acc)[NS * CWS][CW]) {
#pragma unroll
    for (int a = 0; a < NS * CWS; ++a)
#pragma unroll
        for (int c = 0; c < CW; ++c)
            acc[a][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.s[a], f.g[c], acc[a][c], 0, 0, 0);
}

template <int CW, int CWS, int NS>
__global__ __launch_bounds__(256) void wgrad_partial_mfma_kernel(const uint16_t* __restrict__ G,
                                                                const uint16_t* __restrict__ S,
                                                                float* __restrict__ partial, int64_t N, int64_t O,
                                                                int64_t M, int64_t Mp, int64_t rows_per_split) {
    constexpr int OT = 16 * CW;          // output features per block
    constexpr int CAPS = 16 * CWS;       // groups per S set
    constexpr int kWaves = 4;
    constexpr int kStep = 32;            // tokens per MFMA K-step
    __shared__ float lds[OT][CAPS + 1];

    const int lane = threadIdx.x & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int q = lane >> 4;
    const int jj = lane & 15;
    const int64_t o0 = static_cast<int64_t>(blockIdx.x) * OT;
    const int split = blockIdx.y;
    const int64_t gbase = static_cast<int64_t>(blockIdx.z) * CAPS * NS;
    const int64_t kb = static_cast<int64_t>(split) * rows_per_split;
    int64_t ke = kb + rows_per_split;
    if (ke > N) ke = N;
    const int n_steps = static_cast<int>(ceil_div(ke - kb, kStep));
    const int n_full = static_cast<int>((ke - kb) / kStep);    // steps with all 32 tokens in range
    const bool col_edge = o0 + OT > O;                         // block-uniform

    const uint32_t g_row_bytes = static_cast<uint32_t>(O) * 2u;
    const uint32_t s_row_bytes = static_cast<uint32_t>(M) * 2u;
    const uint32_t gvoff = static_cast<uint32_t>(q * 8) * g_row_bytes + static_cast<uint32_t>(jj * CW * 2);
    const uint32_t svoff = static_cast<uint32_t>(q * 8) * s_row_bytes + static_cast<uint32_t>(jj * CWS * 2);
    const bool col_ok = o0 + jj * CW < O;
    bool g_ok[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) g_ok[s] = gbase + s * CAPS + jj * CWS < M;

    const char* gblock = reinterpret_cast<const char*>(G) + (kb * O + o0) * 2;
    const char* sblock = reinterpret_cast<const char*>(S) + (kb * M + gbase) * 2;
    const uint64_t g_step_bytes = static_cast<uint64_t>(kStep) * g_row_bytes;
    const uint64_t s_step_bytes = static_cast<uint64_t>(kStep) * s_row_bytes;

    f32x4 acc[NS * CWS][CW];
#pragma unroll
    for (int a = 0; a < NS * CWS; ++a)
#pragma unroll
        for (int c = 0; c < CW; ++c) acc[a][c] = f32x4{0.f, 0.f, 0.f, 0.f};

    WgradRaw<CW, CWS, NS> raw;
    WgradFrags<CW, CWS, NS> fr;
    auto load_step = [&](int t) {
        const char* gp = gblock + t * g_step_bytes;
        const char* sp = sblock + t * s_step_bytes;
        if (col_edge || t >= n_full) {
            const int rows_left = static_cast<int>(ke - kb) - t * kStep;
            wgrad_load<CW, CWS, NS, true>(raw, gp, sp, gvoff, svoff, g_row_bytes, s_row_bytes, rows_left, q, col_ok, g_ok);
        } else {
            wgrad_load<CW, CWS, NS, false>(raw, gp, sp, gvoff, svoff, g_row_bytes, s_row_bytes, kStep, q, col_ok, g_ok);
        }
    };
    // The raw registers are free again as soon as the fragments are built, so
    // the next step's loads are in flight while this step's MFMAs run.
    int t = w;
    if (t < n_steps) load_step(t);
    while (t < n_steps) {
        wgrad_transpose(raw, fr);
        const int tn = t + kWaves;
        if (tn < n_steps) load_step(tn);
        wgrad_mma(fr, acc);
        t = tn;
    }

    // Sum the four waves in a fixed order through LDS, one S set at a time, and
    // write the block's partial tile with lanes running along g.
    float* out = partial + static_cast<int64_t>(split) * O * Mp;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        for (int wv = 0; wv < kWaves; ++wv) {
            if (w == wv) {
#pragma unroll
                for (int cs = 0; cs < CWS; ++cs)
#pragma unroll
                    for (int c = 0; c < CW; ++c)
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            float* cell = &lds[jj * CW + c][(q * 4 + r) * CWS + cs];
                            const float val = acc[s * CWS + cs][c][r];
                            *cell = (wv == 0) ? val : (*cell + val);
                        }
            }
            __syncthreads();
        }
        for (int idx = threadIdx.x; idx < OT * CAPS; idx += blockDim.x) {
            const int ol = idx / CAPS, gl = idx % CAPS;
            const int64_t o = o0 + ol, g = gbase + s * CAPS + gl;
            if (o < O && g < M) out[o * Mp + g] = lds[ol][gl];
        }
        __syncthreads();
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
        for (int64_t n = kb; n < ke; ++n) {
            const float gv = E::load(G, n * O + o);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int64_t g = g0 + 4 * i;
                if (g < M) acc[i] = fmaf(gv, E::load(S, n * M + g), acc[i]);
            }
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
// One block per output row; T is staged in LDS in chunks of kTChunk groups.
// VEC: four consecutive columns per lane (needs d % 4 == 0 and an aligned dW).
// ---------------------------------------------------------------------------
constexpr int kTChunk = 2048;

template <bool OUT_BF16, bool VEC>
__global__ __launch_bounds__(256) void wgrad_expand_kernel(const float* __restrict__ partial,
                                                          const float* __restrict__ v, void* __restrict__ dW,
                                                          int splits, int64_t O, int64_t D, int64_t M, int64_t Mp,
                                                          int d, int d_shift, int accumulate) {
    __shared__ float T[kTChunk];
    const int64_t o = blockIdx.x;
    const float* prow = partial + o * Mp;
    const int64_t split_stride = O * Mp;
    for (int64_t gc0 = 0; gc0 < M; gc0 += kTChunk) {
        const int gcn = static_cast<int>((M - gc0) < kTChunk ? (M - gc0) : kTChunk);
        for (int gl = threadIdx.x; gl < gcn; gl += blockDim.x) {
            float s = 0.f;
            for (int sp = 0; sp < splits; ++sp) s += prow[sp * split_stride + gc0 + gl];
            T[gl] = s;
        }
        __syncthreads();
        const int64_t c_begin = gc0 * d;
        const int64_t c_count = static_cast<int64_t>(gcn) * d;
        if constexpr (VEC) {
            for (int64_t i = threadIdx.x; i < c_count / 4; i += blockDim.x) {
                const int64_t cl = i * 4;
                const int gl = d_shift >= 0 ? static_cast<int>(cl >> d_shift) : static_cast<int>(cl / d);
                const int j = static_cast<int>(cl - static_cast<int64_t>(gl) * d);
                const float tg = T[gl];
                const float4 vv = *reinterpret_cast<const float4*>(v + j);
                float r0 = tg * vv.x, r1 = tg * vv.y, r2 = tg * vv.z, r3 = tg * vv.w;
                const int64_t e = o * D + c_begin + cl;
                if constexpr (OUT_BF16) {
                    uint2* p = reinterpret_cast<uint2*>(static_cast<uint16_t*>(dW) + e);
                    if (accumulate) {
                        const uint2 old = *p;
                        r0 += bf16_lo(old.x); r1 += bf16_hi(old.x); r2 += bf16_lo(old.y); r3 += bf16_hi(old.y);
                    }
                    *p = make_uint2(pack_bf16x2(r0, r1), pack_bf16x2(r2, r3));
                } else {
                    float4* p = reinterpret_cast<float4*>(static_cast<float*>(dW) + e);
                    if (accumulate) {
                        const float4 old = *p;
                        r0 += old.x; r1 += old.y; r2 += old.z; r3 += old.w;
                    }
                    *p = make_float4(r0, r1, r2, r3);
                }
            }
        } else {
            for (int64_t cl = threadIdx.x; cl < c_count; cl += blockDim.x) {
                const int gl = static_cast<int>(cl / d);
                const int j = static_cast<int>(cl - static_cast<int64_t>(gl) * d);
                float r = T[gl] * v[j];
                const int64_t e = o * D + c_begin + cl;
                if constexpr (OUT_BF16) {
                    uint16_t* p = static_cast<uint16_t*>(dW) + e;
                    if (accumulate) r += bf16_to_f32(*p);
                    *p = f32_to_bf16(r);
                } else {
                    float* p = static_cast<float*>(dW) + e;
                    if (accumulate) r += *p;
                    *p = r;
                }
            }
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
namespace {

struct MfmaChoice {
    int cw, cws, ns;   // cw == 0: no MFMA configuration fits
};

int max_sets(int cws) { return cws == 8 ? 2 : 4; }

MfmaChoice choose_mfma(int64_t O, int64_t M, int g_align, int s_align) {
    MfmaChoice best{0, 0, 0};
    // per-lane byte offsets inside a 32-token step are 32-bit
    if (O > (INT64_C(1) << 24) || M > (INT64_C(1) << 24)) return best;
    int64_t best_chunks = 0, best_gt = 0;
    for (int cws = 8; cws >= 1; cws >>= 1) {
        if (M % cws != 0 || s_align < 2 * cws) continue;
        const int64_t cap_set = 16 * cws;
        int64_t ns = ceil_div(M, cap_set);
        if (ns > max_sets(cws)) ns = max_sets(cws);
        const int64_t chunks = ceil_div(M, cap_set * ns);
        const int64_t gt = ns * cws;
        if (best.cws == 0 || chunks < best_chunks || (chunks == best_chunks && gt < best_gt)) {
            best.cws = cws; best.ns = static_cast<int>(ns);
            best_chunks = chunks; best_gt = gt;
        }
    }
    if (best.cws == 0) return best;
    const int64_t gt = static_cast<int64_t>(best.ns) * best.cws;
    int cw = gt <= 4 ? 8 : 4;
    while (cw >= 4 && (O % cw != 0 || g_align < 2 * cw)) cw >>= 1;
    if (cw < 4) return MfmaChoice{0, 0, 0};
    best.cw = cw;
    return best;
}

template <int CW, int CWS, int NS>
hipError_t launch_mfma(const void* G, const void* S, float* partial, int64_t N, int64_t O, int64_t M,
                       const WgradPlan& plan, hipStream_t st) {
    dim3 grid(static_cast<unsigned>(ceil_div(O, 16 * CW)), static_cast<unsigned>(plan.splits),
              static_cast<unsigned>(ceil_div(M, 16 * CWS * NS)));
    hipLaunchKernelGGL((wgrad_partial_mfma_kernel<CW, CWS, NS>), grid, dim3(256), 0, st,
                       static_cast<const uint16_t*>(G), static_cast<const uint16_t*>(S), partial, N, O, M, plan.Mp,
                       plan.rows_per_split);
    return hipGetLastError();
}

#define VELORA_MFMA_CASE(CW, CWS, NS) \
    if (ch.cw == CW && ch.cws == CWS && ch.ns == NS) return launch_mfma<CW, CWS, NS>(G, S, partial, N, O, M, plan, st);

hipError_t dispatch_mfma(const MfmaChoice& ch, const void* G, const void* S, float* partial, int64_t N, int64_t O,
                         int64_t M, const WgradPlan& plan, hipStream_t st, bool* handled) {
    *handled = true;
    VELORA_MFMA_CASE(8, 1, 1) VELORA_MFMA_CASE(8, 1, 2) VELORA_MFMA_CASE(8, 1, 3) VELORA_MFMA_CASE(8, 1, 4)
    VELORA_MFMA_CASE(8, 2, 1) VELORA_MFMA_CASE(8, 2, 2) VELORA_MFMA_CASE(8, 4, 1)
    VELORA_MFMA_CASE(4, 1, 1) VELORA_MFMA_CASE(4, 1, 2) VELORA_MFMA_CASE(4, 1, 3) VELORA_MFMA_CASE(4, 1, 4)
    VELORA_MFMA_CASE(4, 2, 1) VELORA_MFMA_CASE(4, 2, 2) VELORA_MFMA_CASE(4, 2, 3) VELORA_MFMA_CASE(4, 2, 4)
    VELORA_MFMA_CASE(4, 4, 1) VELORA_MFMA_CASE(4, 4, 2) VELORA_MFMA_CASE(4, 4, 3) VELORA_MFMA_CASE(4, 4, 4)
    VELORA_MFMA_CASE(4, 8, 1) VELORA_MFMA_CASE(4, 8, 2)
    *handled = false;
    return hipSuccess;
}
#undef VELORA_MFMA_CASE

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

template <bool OUT_BF16, bool VEC>
hipError_t launch_expand(const float* partial, const float* v, void* dW, int64_t O, int64_t D, int64_t M,
                         const WgradPlan& plan, bool accumulate, hipStream_t st) {
    const int d = static_cast<int>(D / M);
    int d_shift = -1;
    if ((d & (d - 1)) == 0) {
        d_shift = 0;
        while ((1 << d_shift) < d) ++d_shift;
    }
    hipLaunchKernelGGL((wgrad_expand_kernel<OUT_BF16, VEC>), dim3(static_cast<unsigned>(O)), dim3(256), 0, st, partial,
                       v, dW, plan.splits, O, D, M, plan.Mp, d, d_shift, accumulate ? 1 : 0);
    return hipGetLastError();
}

int env_int(const char* name, int fallback) {
    const char* s = std::getenv(name);
    if (!s || !*s) return fallback;
    return std::atoi(s);
}

}  // namespace

WgradPlan plan_wgrad(int64_t N, int64_t O, int64_t D, int64_t M, bool is_bf16, const LaunchCfg& cfg) {
    WgradPlan p;
    p.Mp = ceil_div(M, 4) * 4;
    const int64_t in_b = is_bf16 ? 2 : 4;
    // Enough blocks to occupy every CU twice ...
    const int64_t o_tiles = ceil_div(O, 128);
    int64_t splits = ceil_div(static_cast<int64_t>(cfg.num_cus) * 2, o_tiles);
    // ... but keep the partial write + re-read under ~10 % of the bytes the
    // two kernels must move anyway, and give each block at least 256 tokens.
    const double must_move = static_cast<double>(N) * O * in_b + static_cast<double>(O) * D * 4.0;
    const double per_split = static_cast<double>(O) * p.Mp * 8.0;
    const int64_t traffic_cap = static_cast<int64_t>(0.10 * must_move / per_split);
    if (splits > traffic_cap) splits = traffic_cap;
    if (splits > ceil_div(N, 256)) splits = ceil_div(N, 256);
    const int forced = env_int("VELORA_WGRAD_SPLITS", 0);   // tuning aid; 0 = automatic
    if (forced > 0) splits = forced;
    if (splits < 1) splits = 1;
    if (splits > 65535) splits = 65535;
    int64_t rows = ceil_div(ceil_div(N, splits), 128) * 128;
    p.rows_per_split = rows;
    p.splits = static_cast<int>(ceil_div(N, rows));
    p.ws_bytes = static_cast<size_t>(p.splits) * static_cast<size_t>(O) * static_cast<size_t>(p.Mp) * sizeof(float);
    return p;
}

hipError_t launch_wgrad(const void* G, const void* S, const float* v, int64_t N, int64_t O, int64_t D, int64_t M,
                        bool is_bf16, int g_align, int s_align, int v_align, void* dW, bool dw_bf16, int dw_align,
                        bool accumulate, void* ws, const WgradPlan& plan, const LaunchCfg& cfg, hipStream_t st) {
    (void)cfg;
    float* partial = static_cast<float*>(ws);
    hipError_t e = hipSuccess;
    bool done = false;
    if (is_bf16 && env_int("VELORA_WGRAD_FORCE_SIMPLE", 0) == 0) {
        const MfmaChoice ch = choose_mfma(O, M, g_align, s_align);
        if (ch.cw != 0) {
            e = dispatch_mfma(ch, G, S, partial, N, O, M, plan, st, &done);
            if (e != hipSuccess) return e;
        }
    }
    if (!done) {
        e = is_bf16 ? launch_simple<Bf16Elem>(G, S, partial, N, O, M, plan, st)
                    : launch_simple<F32Elem>(G, S, partial, N, O, M, plan, st);
        if (e != hipSuccess) return e;
    }
    const int64_t d = D / M;
    const bool vec = (d % 4 == 0) && v_align >= 16 && dw_align >= (dw_bf16 ? 8 : 16);
    if (dw_bf16) {
        return vec ? launch_expand<true, true>(partial, v, dW, O, D, M, plan, accumulate, st)
                   : launch_expand<true, false>(partial, v, dW, O, D, M, plan, accumulate, st);
    }
    return vec ? launch_expand<false, true>(partial, v, dW, O, D, M, plan, accumulate, st)
               : launch_expand<false, false>(partial, v, dW, O, D, M, plan, accumulate, st);
}

}  // namespace velora
