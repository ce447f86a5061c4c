/*
 * libvelora -- C ABI of the MI355X (gfx950) implementation of the VeLoRA hot
 * path: rank-1 sub-token compression of a linear layer's input activations and
 * the weight gradient built on it (paper Sec. 3.1 "VeLoRA", Sec. 3.2 "Cheap
 * initialisation strategies", Listing 1).
 *
 * Symbols
 *   N  tokens (batch x sequence, flattened)      D  input features
 *   O  output features                           M  sub-tokens per token
 *   d = D / M  sub-token size (the paper writes "M" for this size; this
 *              library follows the convention S[N, M], d = D/M)
 *   X[N, D] activations, S[N, M] compressed activations, v[d] projection
 *   vector, G[N, O] gradient of the loss w.r.t. the layer output,
 *   dW[O, D] gradient w.r.t. the weight (layout of grad_output^T @ input).
 *
 * Conventions common to every call
 *   - Every data pointer is a DEVICE pointer owned by the caller, to a
 *     row-major contiguous array.  The library neither allocates nor frees
 *     device memory; calls that need scratch take a caller-provided workspace
 *     of at least velora_workspace_bytes(...) bytes.
 *   - v is always float32.  X, S and G share one storage dtype (float32 or
 *     bfloat16); arithmetic is float32 accumulate, and values are rounded to
 *     the storage dtype with round-to-nearest-even when stored.
 *   - Calls are asynchronous: work is enqueued on `stream` (a hipStream_t, 0 =
 *     the null stream) and the call returns.  velora_init_v is the exception:
 *     it waits for its own work so that it can report a degenerate mean.
 *   - Arguments are validated on the host before anything is launched; on any
 *     error other than VELORA_ERR_HIP / VELORA_ERR_DEGENERATE nothing was
 *     launched and the outputs are untouched.  No C++ exception crosses the
 *     boundary.  The library keeps no state between calls; concurrent calls on
 *     different streams with disjoint outputs/workspaces are safe.
 *   - Apart from velora_init_v, no call allocates, synchronises or clears
 *     memory, so a sequence of calls can be recorded into a HIP graph.  Some
 *     kernels use more than 64 KB of LDS and raise their limit
 *     (hipFuncSetAttribute) at their first launch on a device: run the
 *     sequence once eagerly before capturing it.  What the library remembers
 *     between calls (those per-device flags, the last launch plans per
 *     thread) never changes a result.
 *   - Pointers must be aligned to their element size (VELORA_ERR_ALIGN
 *     otherwise).  16-byte aligned pointers with d a multiple of 8 (bf16) or 4
 *     (f32) take the vectorised kernels; anything else takes slower generic
 *     kernels with identical results up to summation order.
 */
#ifndef VELORA_H_
#define VELORA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    VELORA_OK = 0,
    VELORA_ERR_NULL = 1,        /* a required pointer is NULL                           */
    VELORA_ERR_SHAPE = 2,       /* N, D, O or M <= 0, or M does not divide D            */
    VELORA_ERR_DTYPE = 3,       /* dtype value not in velora_dtype                      */
    VELORA_ERR_ALIGN = 4,       /* pointer not aligned to its element size              */
    VELORA_ERR_WORKSPACE = 5,   /* workspace NULL or smaller than velora_workspace_bytes */
    VELORA_ERR_DEGENERATE = 6,  /* init_v: mean of the sub-tokens is zero or not finite */
    VELORA_ERR_HIP = 7          /* a HIP runtime call failed                            */
} velora_status;

typedef enum { VELORA_F32 = 0, VELORA_BF16 = 1 } velora_dtype;

typedef enum {
    VELORA_OP_INIT_V = 0,
    VELORA_OP_COMPRESS = 1,
    VELORA_OP_RECONSTRUCT = 2,
    VELORA_OP_WEIGHT_GRAD = 3,
    VELORA_OP_WEIGHT_GRAD_FACTOR = 4
} velora_op;

typedef void* velora_stream; /* hipStream_t */

/* Human-readable name of a status code (static storage, never NULL). */
const char* velora_status_string(velora_status st);

/* Library version, major*10000 + minor*100 + patch. */
int velora_version(void);

/*
 * Bytes of device workspace the given call needs for these sizes (0 if none).
 * Pass the same N, D, O, M and input dtype as to the call itself; arguments an
 * op does not use (e.g. O for VELORA_OP_INIT_V) are ignored.  Returns 0 for
 * invalid shapes (the call itself will report the error).
 */
size_t velora_workspace_bytes(velora_op op, int64_t N, int64_t D, int64_t O, int64_t M,
                              velora_dtype in_dt);

/*
 * Initialise the projection vector (Sec. 3.2: the average of the first batch's
 * sub-tokens; Sec. 3.1: unit length):
 *     m[j] = 1/(N*M) * sum_{n<N, g<M} X[n, g*d + j],      v = m / ||m||_2
 * The average runs over all tokens AND all groups: one v per layer.
 *   X   [N, D] device, dtype xdt (read only)
 *   v   [d]    device, float32 (written)
 *   ws  device workspace, >= velora_workspace_bytes(VELORA_OP_INIT_V, N, D, 0, M, xdt)
 * Synchronises `stream` before returning.  If ||m|| is zero or any m[j] is not
 * finite, writes v[j] = 1/sqrt(d) and returns VELORA_ERR_DEGENERATE.
 */
velora_status velora_init_v(const void* X, int64_t N, int64_t D, int64_t M, velora_dtype xdt,
                            float* v, void* ws, size_t ws_bytes, velora_stream stream);

/*
 * Per-batch projection vector (the "running average" and instance-wise rows of
 * the initialisation ablation, Sec. 5.3 / Table 5c; the paper gives no formula,
 * this is the reading taken):
 *     m_b = mean of this batch's N*M sub-tokens
 *     m   = mean_state ? beta * mean_state + (1 - beta) * m_b : m_b
 *     mean_state <- m (if given),   v = m / ||m||_2
 * beta = 0 with a state (or no state at all) is the instance-wise variant: v
 * follows every batch.  0 <= beta <= 1 (VELORA_ERR_SHAPE otherwise).
 *   X [N, D] device (read only); mean_state [d] device float32 (read and
 *   written) or NULL; v [d] device float32 (written); ws as for velora_init_v.
 * Asynchronous.  A zero or non-finite m gives v[j] = 1/sqrt(d); the status word
 * (0 or VELORA_ERR_DEGENERATE) is left in the first 4 bytes of ws.
 */
velora_status velora_update_v(const void* X, int64_t N, int64_t D, int64_t M, velora_dtype xdt,
                              float* mean_state, float beta, float* v, void* ws, size_t ws_bytes,
                              velora_stream stream);

/*
 * compress with the current vector and update the vector for the next batch in
 * ONE pass over X (running average: batch t is compressed with the v formed
 * from the batches before it):
 *     S = compress(X, v_in);   (mean_state, v_out) updated from X as in velora_update_v.
 * v_out may be the same buffer as v_in (it is written after S is complete).
 * S is bit-identical to velora_compress(X, v_in).  Same workspace and status
 * word as velora_update_v.
 */
velora_status velora_compress_update(const void* X, const float* v_in, int64_t N, int64_t D, int64_t M,
                                     velora_dtype xdt, void* S, float* mean_state, float beta,
                                     float* v_out, void* ws, size_t ws_bytes, velora_stream stream);

/*
 * group + compress (Sec. 3.1, Eq. 1):  S[n, g] = sum_{j<d} X[n, g*d + j] * v[j].
 *   X [N, D] device, dtype xdt (read only);  v [d] device float32 (read only)
 *   S [N, M] device, dtype xdt (written; float32 accumulate, RNE on store)
 */
velora_status velora_compress(const void* X, const float* v, int64_t N, int64_t D, int64_t M,
                              velora_dtype xdt, void* S, velora_stream stream);

/*
 * The same compress, taken where X is produced.  The layer the paper compresses
 * first is the MLP down projection of an LLaMA block (Sec. 4, opening paragraph;
 * Sec. 5.4 "Choice of layers"), whose input is the elementwise product
 * X = silu(gate) * up, silu(x) = x / (1 + exp(-x)).  This
 * call writes X and, in the same pass and from the very values it stores,
 * S = compress(group(X), v) (Sec. 3.1, Eq. 1): X is never re-read for
 * compression.  float32 arithmetic, one RNE rounding when X is stored; S is what
 * velora_compress returns on the stored X (bit for bit when gate, up and X are
 * 16-byte aligned and d is a multiple of 8 (bf16) or 4 (f32); otherwise X is
 * written first and compressed by a second launch).
 *   gate, up [N, D] device, dtype dt (read only);  v [d] device float32 (read only)
 *   X [N, D] and S [N, M] device, dtype dt (written).  X may alias gate or up.
 */
velora_status velora_swiglu_compress(const void* gate, const void* up, const float* v, int64_t N, int64_t D,
                                     int64_t M, velora_dtype dt, void* X, void* S, velora_stream stream);

/*
 * The forward of the layer with the compression taken from the same pass (Sec. 3.1
 * and Listing 1, forward: the output is the dense product, next to it
 * compress(group(input), v) is what is kept for backward):
 *     Y[n, o] = sum_c X[n, c] * W[o, c]         (W in the nn.Linear layout [O, D])
 *     S[n, g] = sum_{j<d} X[n, g*d + j] * v[j]
 * Products of the stored inputs accumulated in float32, one RNE rounding when Y
 * and S are stored in dtype dt.  For bf16 inputs with 16-byte aligned X, W, Y,
 * D a multiple of 64 and O a multiple of 4 this is one MFMA kernel; when d is
 * also a multiple of 64 (and at most 2048) S comes out of that kernel, from
 * the tiles of X it has loaded, so X is read once for both results; there v
 * enters as the sum of two bf16 numbers (relative error 2^-17, far below the
 * rounding of S).  Every other case runs a plain FMA kernel for Y and the
 * compress kernel for S.
 *   X [N, D], W [O, D] device, dtype dt (read only);  v [d] device float32 (read only)
 *   Y [N, O], S [N, M] device, dtype dt (written).  O <= 65535 * 64.
 */
velora_status velora_linear_compress(const void* X, const void* W, const float* v, int64_t N, int64_t D, int64_t O,
                                     int64_t M, velora_dtype dt, void* Y, void* S, velora_stream stream);

/*
 * The other half of the layer's backward (Listing 1, backward:
 * grad_input = grad_output @ weight; it needs neither the input nor S):
 *     dX[n, c] = sum_o G[n, o] * W[o, c]
 * Products of the stored inputs accumulated in float32, one RNE rounding when dX
 * is stored in dtype dt.  bf16 with 16-byte aligned pointers, O a multiple of 64
 * and D a multiple of 8 runs the MFMA kernel of velora_linear_compress with W
 * read in its own [O, D] layout (transposed in registers); every other case a
 * plain FMA kernel.
 *   G [N, O], W [O, D] device, dtype dt (read only);  dX [N, D] device, dtype dt (written).  D <= 65535 * 64.
 */
velora_status velora_grad_input(const void* G, const void* W, int64_t N, int64_t O, int64_t D, velora_dtype dt,
                                void* dX, velora_stream stream);

/*
 * The other producer: the attention projections of an LLaMA block (the paper
 * compresses the value projection's input, Sec. 4 and Sec. 5.4) read X = RMSNorm(H),
 *     X[n, j] = H[n, j] / sqrt(mean_j H[n, j]^2 + eps) * gamma[j].
 * This call writes X and, from the values it stores, S = compress(group(X), v)
 * (Sec. 3.1, Eq. 1) in one pass over H.  float32 arithmetic, one RNE rounding
 * when X is stored; S is what velora_compress returns on the stored X (bit for
 * bit in the fused kernel: H, X, gamma 16-byte aligned, d / 8 (bf16) or d / 4
 * (f32) a power of two <= 64, D <= 8192 (bf16) or 4096 (f32); otherwise X is
 * written first and compressed by a second launch).
 *   H [N, D] device, dtype dt (read only); gamma [D], v [d] device float32 (read only)
 *   X [N, D] and S [N, M] device, dtype dt (written).  X may alias H.
 * eps < 0 is VELORA_ERR_SHAPE.
 */
velora_status velora_rmsnorm_compress(const void* H, const float* gamma, float eps, const float* v, int64_t N,
                                      int64_t D, int64_t M, velora_dtype dt, void* X, void* S,
                                      velora_stream stream);

/*
 * reconstruct + ungroup (Sec. 3.1, Eq. 2):  Xhat[n, g*d + j] = S[n, g] * v[j].
 * The materialising form; velora_weight_grad never needs it.
 *   S [N, M] device, dtype dt (read only);  v [d] device float32 (read only)
 *   Xhat [N, D] device, dtype dt (written)
 */
velora_status velora_reconstruct(const void* S, const float* v, int64_t N, int64_t D, int64_t M,
                                 velora_dtype dt, void* Xhat, velora_stream stream);

/*
 * Weight gradient from the compressed activations (Listing 1, backward:
 * input_hat = ungroup(reconstruct(z, v)); grad_weight = grad_output^T @ input_hat):
 *     dW[o, g*d + j] (+)= sum_{n<N} G[n, o] * S[n, g] * v[j]
 * evaluated as T = G^T S followed by the expansion with v, which is the same
 * sum re-associated; Xhat is never formed.
 *   G  [N, O] device, dtype in_dt (read only)
 *   S  [N, M] device, dtype in_dt (read only)
 *   v  [d]    device float32 (read only)
 *   dW [O, D] device, dtype dw_dt (float32 or bfloat16).  accumulate == 0:
 *      overwritten; accumulate != 0: the result is added to the existing
 *      contents (in float32, rounded once on store).
 *   ws device workspace, >= velora_workspace_bytes(VELORA_OP_WEIGHT_GRAD, N, D, O, M, in_dt)
 * Deterministic: the reduction over tokens is split in a fixed way that
 * depends only on the sizes; no floating-point atomics.
 */
velora_status velora_weight_grad(const void* G, const void* S, const float* v,
                                 int64_t N, int64_t O, int64_t D, int64_t M, velora_dtype in_dt,
                                 void* dW, velora_dtype dw_dt, int accumulate,
                                 void* ws, size_t ws_bytes, velora_stream stream);

/*
 * velora_weight_grad for callers that cannot allocate or own a workspace: code under
 * HIP graph capture that may not call hipMalloc, tight serving or training loops,
 * harnesses that forbid allocation.  Same arguments, kernels, split and result
 * (bit for bit) as velora_weight_grad, without `ws`: the partial sums (and, for
 * M > 48, the re-laid-out S) live in a static device array of
 * VELORA_STATIC_SCRATCH_BYTES that is part of the library's code object, so every
 * GPU the library is used on holds that much memory until the process ends.
 * The call allocates and frees nothing (no hipMalloc / hipFree / allocating library
 * routine).  The first call on a device looks the array's address up once
 * (hipGetSymbolAddress, with that device current) and keeps it per device; make that
 * first call outside a stream capture.
 * A shape whose workspace requirement (velora_workspace_bytes(VELORA_OP_WEIGHT_GRAD, ...))
 * exceeds VELORA_STATIC_SCRATCH_BYTES is refused with VELORA_ERR_WORKSPACE before any
 * launch; the other argument errors are those of velora_weight_grad.
 * Every call on a GPU uses that GPU's one array, whatever the stream: calls that may
 * run concurrently on one GPU (different streams, different threads) race on it and
 * must be serialised by the caller; calls on one stream are safe back to back.  The
 * array keeps the previous call's contents; the kernels overwrite every word they
 * later read, nothing has to be cleared.
 */
#define VELORA_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
velora_status velora_weight_grad_static(const void* G, const void* S, const float* v,
                                        int64_t N, int64_t O, int64_t D, int64_t M, velora_dtype in_dt,
                                        void* dW, velora_dtype dw_dt, int accumulate, velora_stream stream);

/*
 * The factored hand-off of the same gradient.  Since the reconstruction of
 * Sec. 3.1 is Xhat[n, g*d+j] = S[n,g]*v[j], Listing 1's grad_weight equals
 * T (x) v with T[o, g] = sum_n G[n, o] * S[n, g]: d times smaller than dW.  A
 * caller that reduces gradients across devices or applies the update itself
 * can take T and expand later (or never materialise dW).
 *
 * velora_weight_grad_factor:  T[O, M] (float32, dense, overwritten) = G^T S.
 *   G [N, O], S [N, M] device, dtype in_dt (read only); v is not needed.
 *   ws >= velora_workspace_bytes(VELORA_OP_WEIGHT_GRAD_FACTOR, N, M, O, M, in_dt)
 *   (pass D = M in the query; the factor does not depend on the sub-token size).
 * velora_expand_factor:  dW[o, g*d + j] (+)= T[o, g] * v[j].
 *   T [O, M] device float32, v [d] device float32 (read only); dW [O, D] device,
 *   dtype dw_dt; accumulate as in velora_weight_grad.  No workspace.
 * velora_weight_grad(...) is factor followed by expand (its token split may
 * differ, so the two agree to rounding, not bit for bit).
 */
velora_status velora_weight_grad_factor(const void* G, const void* S, int64_t N, int64_t O, int64_t M,
                                        velora_dtype in_dt, float* T, void* ws, size_t ws_bytes,
                                        velora_stream stream);
velora_status velora_expand_factor(const float* T, const float* v, int64_t O, int64_t D, int64_t M, void* dW,
                                   velora_dtype dw_dt, int accumulate, velora_stream stream);

/*
 * AdamW step taken straight from the factored gradient (the paper's training
 * set-ups, Sec. 4.1 "Implementation details", use AdamW; the gradient is
 * Listing 1's grad_weight in the factored form above).  With g[o, g*d + j] = grad_scale * T[o, g] * v[j], in
 * place and in float32:
 *     W <- W * (1 - lr * weight_decay)
 *     exp_avg    <- beta1 * exp_avg    + (1 - beta1) * g
 *     exp_avg_sq <- beta2 * exp_avg_sq + (1 - beta2) * g^2
 *     W <- W - lr / (1 - beta1^step) * exp_avg / (sqrt(exp_avg_sq) / sqrt(1 - beta2^step) + eps)
 * (decoupled weight decay, bias-corrected moments; step counts from 1).  dW is
 * never materialised: the call moves W and the two moments through HBM once.
 *   T [O, M], v [d] device float32 (read only)
 *   W [O, D] device, dtype w_dt (float32, or bfloat16 rounded RNE on store)
 *   exp_avg, exp_avg_sq [O, D] device float32 (read and written)
 * VELORA_ERR_SHAPE also for step < 1, a beta outside [0, 1), eps < 0 or a
 * non-finite lr / weight_decay / grad_scale.  No workspace.
 */
velora_status velora_adamw_step_factor(const float* T, const float* v, int64_t O, int64_t D, int64_t M, void* W,
                                       velora_dtype w_dt, float* exp_avg, float* exp_avg_sq, float lr, float beta1,
                                       float beta2, float eps, float weight_decay, int64_t step, float grad_scale,
                                       velora_stream stream);

/*
 * Measurement aid, not part of the method: the plainest streaming kernels this
 * library can write, for a benchmark that wants to state a kernel's rate against
 * a ceiling measured on the same box in the same run (the hot path is bound by
 * HBM; see velora_compress and velora_weight_grad).
 *   kind 0  read:  every 16-byte vector of src[0, bytes) is loaded once; sink
 *                  (device, 64 uint32, zeroed by the caller or not) receives
 *                  folded words so that the loads are real.  dst is ignored.
 *   kind 1  write: zeros to dst[0, bytes).  src and sink are ignored.
 *   kind 2  copy:  dst[0, bytes) = src[0, bytes).  sink is ignored.
 * bytes > 0 and a multiple of 16, the pointers used 16-byte aligned
 * (VELORA_ERR_SHAPE / VELORA_ERR_ALIGN / VELORA_ERR_NULL otherwise); one block
 * per compute unit, eight 16-byte accesses in flight per thread, non-temporal.
 */
velora_status velora_bandwidth_probe(int kind, const void* src, void* dst, int64_t bytes, uint32_t* sink,
                                     velora_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* VELORA_H_ */
