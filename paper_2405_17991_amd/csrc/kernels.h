// Internal launch interface between the C-ABI layer (api.hip) and the kernels.
// Every function only enqueues work on `st` and returns hipGetLastError().
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace velora {

struct LaunchCfg {
    int num_cus;     // compute units of the current device
    int max_blocks;  // cap for grid-stride streaming kernels (256-thread blocks)
};

// ---- compress.hip ----
hipError_t launch_compress(const void* X, const float* v, void* S, int64_t n_sub, int64_t d, bool is_bf16,
                           bool vec_ok, const LaunchCfg& cfg, hipStream_t st);
hipError_t launch_reconstruct(const void* S, const float* v, void* Xhat, int64_t n_sub, int64_t d, bool is_bf16,
                              bool vec_ok, const LaunchCfg& cfg, hipStream_t st);

// ---- swiglu.hip ----
// X = silu(gate) * up stored in the inputs' dtype, and S = compress(X, v) from the stored values, one pass.
// vec_ok: gate, up, X 16-byte aligned (then d % 8 == 0 (bf16) / d % 4 == 0 (f32) takes the fused kernel).
hipError_t launch_swiglu_compress(const void* gate, const void* up, const float* v, void* X, void* S, int64_t n_sub,
                                  int64_t d, bool is_bf16, bool vec_ok, const LaunchCfg& cfg, hipStream_t st);

// ---- rmsnorm.hip ----
// X = H / sqrt(mean(H^2) + eps) * gamma stored in H's dtype, and S = compress(X, v) from the stored values.
// vec_ok: H, X, gamma and v 16-byte aligned (then a power-of-two d / kPerVec <= 64 and a row of at most
// 1024 vectors take the fused kernel).
hipError_t launch_rmsnorm_compress(const void* H, const float* gamma, const float* v, void* X, void* S, int64_t N,
                                   int64_t D, int64_t M, float eps, bool is_bf16, bool vec_ok, const LaunchCfg& cfg,
                                   hipStream_t st);

// ---- linear.hip ----
// Y[N, O] = X[N, D] * W[O, D]^T stored in the inputs' dtype and S = compress(X, v).  bf16 inputs with 16-byte
// aligned X, W and Y, D % 64 == 0 and O % 4 == 0 take the MFMA kernel (S inside it when d % 64 == 0 and
// d <= 2048, else by the compress kernel); everything else a plain FMA kernel plus the compress kernel.
// s_vec_ok: X is 16-byte aligned (for the compress kernel).  Requires O <= 65535 * 64.
hipError_t launch_linear_compress(const void* X, const void* W, const float* v, void* Y, void* S, int64_t N, int64_t D,
                                  int64_t O, int64_t M, bool is_bf16, bool align16, bool s_vec_ok, const LaunchCfg& cfg,
                                  hipStream_t st);

// dX[N, D] = G[N, O] * W[O, D] stored in the inputs' dtype.  bf16 with 16-byte aligned G, W and dX, O % 64 == 0 and
// D % 8 == 0 takes the MFMA kernel, everything else the plain FMA kernel.  Requires D <= 65535 * 64.
hipError_t launch_grad_input(const void* G, const void* W, void* dX, int64_t N, int64_t O, int64_t D, bool is_bf16,
                             bool align16, hipStream_t st);

// ---- init_v.hip ----
// Workspace layout: [int32 flag | pad to 256 B | mean[d] f64 | slices[8][d] f64 | float partial[rows][d]].
struct InitVPlan {
    int blocks;         // partial-sum blocks of the stand-alone column-sum kernel
    int fused_blocks;   // blocks of the fused compress + column-sum kernel
    size_t ws_bytes;    // total workspace
    size_t slices_off;
    size_t partial_off;
};
InitVPlan plan_init_v(int64_t n_sub, int64_t d, bool is_bf16, const LaunchCfg& cfg);
// v = normalise(m), m = batch mean, or beta*state + (1-beta)*batch mean when state != nullptr (state <- m).
// Leaves the status word (0 | 6) at the start of the workspace; does not synchronise.
hipError_t launch_update_v(const void* X, float* state, double beta, float* v, int64_t n_sub, int64_t d,
                           bool is_bf16, bool vec_ok, void* ws, const InitVPlan& plan, hipStream_t st);
// One pass: S = compress(X, v_in) and the same update of (state, v_out) from this batch.
bool fused_compress_update_ok(int64_t d, bool is_bf16, bool vec_ok);
hipError_t launch_compress_update(const void* X, const float* v_in, void* S, float* state, double beta, float* v_out,
                                  int64_t n_sub, int64_t d, bool is_bf16, void* ws, const InitVPlan& plan,
                                  hipStream_t st);

// ---- wgrad.hip ----
// Workspace layout: float partial[splits][O][Mp] (Mp = M rounded up to 4),
// then, for bf16 inputs with more than three 16-group tiles (M > 48), room for S
// re-laid out as MFMA fragments (ceil(N/32) steps x tiles_packed tiles x 1 KiB);
// the kernels for four to six tiles use it only when they cannot read S in place.
struct WgradPlan {
    int splits;        // number of token ranges (split-K)
    int64_t rows_per_split;
    int64_t Mp;
    int64_t tiles_packed;
    bool cyclic;       // token chunks are dealt to the splits round-robin instead of as contiguous ranges
    int num_cus;       // compute units the plan was made for
    size_t partial_bytes;
    size_t packed_bytes;
    size_t ws_bytes;
};
WgradPlan plan_wgrad(int64_t N, int64_t O, int64_t D, int64_t M, bool is_bf16, const LaunchCfg& cfg);
// g_align / s_align / dw_align / v_align: largest power of two (<= 16) dividing the pointer.
hipError_t launch_wgrad(const void* G, const void* S, const float* v, int64_t N, int64_t O, int64_t D, int64_t M,
                        bool is_bf16, int g_align, int s_align, int v_align, void* dW, bool dw_bf16, int dw_align,
                        bool accumulate, void* ws, const WgradPlan& plan, const LaunchCfg& cfg, hipStream_t st);

// T[O, M] = G^T S only (the factor of the gradient), and its expansion dW (+)= T (x) v.
hipError_t launch_wgrad_factor(const void* G, const void* S, int64_t N, int64_t O, int64_t M, bool is_bf16,
                               int g_align, int s_align, float* T, void* ws, const WgradPlan& plan, hipStream_t st);
hipError_t launch_expand_factor(const float* T, const float* v, int v_align, void* dW, bool dw_bf16, int dw_align,
                                bool accumulate, int64_t O, int64_t D, int64_t M, const LaunchCfg& cfg, hipStream_t st);

// ---- probe.hip ----
// kind 0: read `bytes` of src (a folded word per block is xor-ed into sink[0..63]); 1: write `bytes` of
// zeros to dst; 2: copy.  bytes a multiple of 16, pointers 16-byte aligned.
hipError_t launch_probe(int kind, const void* src, void* dst, int64_t bytes, uint32_t* sink, const LaunchCfg& cfg,
                        hipStream_t st);

// ---- adamw.hip ----
// Scalars of one AdamW step, precomputed on the host in double precision.
struct AdamWScalars {
    float decay;            // 1 - lr * weight_decay
    float beta1, one_minus_beta1;
    float beta2, one_minus_beta2;
    float step_size;        // lr / (1 - beta1^step)
    float inv_sqrt_bc2;     // 1 / sqrt(1 - beta2^step)
    float eps;
    float grad_scale;
};
// W, exp_avg, exp_avg_sq [O, D] updated in place from the gradient grad_scale * T (x) v.
// vec_ok: d % 4 == 0 and all five pointers 16-byte aligned (8 for a bf16 W).
hipError_t launch_adamw_factor(const float* T, const float* v, void* W, bool w_bf16, float* exp_avg, float* exp_avg_sq,
                               int64_t O, int64_t D, int64_t M, bool vec_ok, const AdamWScalars& a, hipStream_t st);

}  // namespace velora
