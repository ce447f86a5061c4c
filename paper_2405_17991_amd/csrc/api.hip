// C-ABI entry points of libvelora: argument validation, launch planning and
// error mapping.  Nothing here touches device memory contents; the arithmetic
// lives in compress.hip, swiglu.hip, rmsnorm.hip, init_v.hip, wgrad.hip and adamw.hip.
#include "../../include/velora.h"

#include <atomic>

#include "common.h"
#include "kernels.h"

#include <cmath>

// Scratch of velora_weight_grad_static: part of the code object, one copy per GPU at its own address.
// Host code never passes this name to a kernel; it passes the address hipGetSymbolAddress returned.
static __device__ __align__(256) unsigned char velora_static_scratch[VELORA_STATIC_SCRATCH_BYTES];

namespace {

using velora::LaunchCfg;

constexpr int kMaxDevices = 64;
std::atomic<void*> g_static_scratch_ptr[kMaxDevices];   // zero-initialised: not looked up yet
constexpr int kDefaultCus = 256;   // MI355X; used when no device can be queried

LaunchCfg current_cfg() {
    static std::atomic<int> cached[kMaxDevices];   // zero-initialised: 0 = not queried
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < kMaxDevices) {
        cus = cached[dev].load(std::memory_order_relaxed);
        if (cus == 0) {
            int n = 0;
            if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) {
                cus = n;
                cached[dev].store(n, std::memory_order_relaxed);
            }
        }
    } else {
        (void)hipGetLastError();   // clear the sticky "no device" error
    }
    if (cus <= 0) cus = kDefaultCus;
    LaunchCfg c;
    c.num_cus = cus;
    c.max_blocks = cus * 8;        // 8 blocks x 4 waves = full wave occupancy per CU
    return c;
}

int ptr_align(const void* p) {
    const uintptr_t a = reinterpret_cast<uintptr_t>(p);
    int al = 16;
    while (al > 1 && (a % static_cast<uintptr_t>(al)) != 0) al >>= 1;
    return al;
}

bool dtype_ok(velora_dtype dt) { return dt == VELORA_F32 || dt == VELORA_BF16; }
int elem_bytes(velora_dtype dt) { return dt == VELORA_BF16 ? 2 : 4; }

bool shape_ok(int64_t N, int64_t D, int64_t M) { return N > 0 && D > 0 && M > 0 && M <= D && D % M == 0; }

// Sizes that would overflow 64-bit element counts or 32-bit sub-token sizes are
// rejected as shapes.
bool size_ok(int64_t rows, int64_t cols) {
    return rows > 0 && cols > 0 && cols <= (INT64_C(1) << 40) / rows;
}

velora_status hip_status(hipError_t e) { return e == hipSuccess ? VELORA_OK : VELORA_ERR_HIP; }

}  // namespace

extern "C" {

const char* velora_status_string(velora_status st) {
    switch (st) {
        case VELORA_OK: return "VELORA_OK";
        case VELORA_ERR_NULL: return "VELORA_ERR_NULL: a required pointer is NULL";
        case VELORA_ERR_SHAPE: return "VELORA_ERR_SHAPE: sizes must be positive and M must divide D";
        case VELORA_ERR_DTYPE: return "VELORA_ERR_DTYPE: unknown dtype";
        case VELORA_ERR_ALIGN: return "VELORA_ERR_ALIGN: pointer not aligned to its element size";
        case VELORA_ERR_WORKSPACE: return "VELORA_ERR_WORKSPACE: workspace missing or too small";
        case VELORA_ERR_DEGENERATE: return "VELORA_ERR_DEGENERATE: sub-token mean is zero or not finite";
        case VELORA_ERR_HIP: return "VELORA_ERR_HIP: a HIP runtime call failed";
    }
    return "VELORA: unknown status";
}

int velora_version(void) { return 100; }

size_t velora_workspace_bytes(velora_op op, int64_t N, int64_t D, int64_t O, int64_t M, velora_dtype in_dt) {
    if (!dtype_ok(in_dt) || !shape_ok(N, D, M) || !size_ok(N, D)) return 0;
    const LaunchCfg cfg = current_cfg();
    switch (op) {
        case VELORA_OP_INIT_V:
            return velora::plan_init_v(N * M, D / M, in_dt == VELORA_BF16, cfg).ws_bytes;
        case VELORA_OP_WEIGHT_GRAD:
            if (O <= 0 || !size_ok(N, O) || !size_ok(O, D)) return 0;
            return velora::plan_wgrad(N, O, D, M, in_dt == VELORA_BF16, cfg).ws_bytes;
        case VELORA_OP_WEIGHT_GRAD_FACTOR:
            if (O <= 0 || !size_ok(N, O) || !size_ok(O, M)) return 0;
            return velora::plan_wgrad(N, O, M, M, in_dt == VELORA_BF16, cfg).ws_bytes;
        case VELORA_OP_COMPRESS:
        case VELORA_OP_RECONSTRUCT:
            return 0;
    }
    return 0;
}

velora_status velora_init_v(const void* X, int64_t N, int64_t D, int64_t M, velora_dtype xdt, float* v, void* ws,
                            size_t ws_bytes, velora_stream stream) {
    if (!X || !v) return VELORA_ERR_NULL;
    if (!dtype_ok(xdt)) return VELORA_ERR_DTYPE;
    if (!shape_ok(N, D, M) || !size_ok(N, D) || D / M > INT32_MAX / 8) return VELORA_ERR_SHAPE;
    if (ptr_align(X) < elem_bytes(xdt) || ptr_align(v) < 4) return VELORA_ERR_ALIGN;
    const LaunchCfg cfg = current_cfg();
    const bool bf = xdt == VELORA_BF16;
    const velora::InitVPlan plan = velora::plan_init_v(N * M, D / M, bf, cfg);
    if (!ws || ws_bytes < plan.ws_bytes) return VELORA_ERR_WORKSPACE;
    if (ptr_align(ws) < 16) return VELORA_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e = velora::launch_update_v(X, nullptr, 0.0, v, N * M, D / M, bf, ptr_align(X) >= 16, ws, plan, st);
    if (e != hipSuccess) return VELORA_ERR_HIP;
    int flag = -1;
    e = hipMemcpyAsync(&flag, ws, sizeof(int), hipMemcpyDeviceToHost, st);
    if (e != hipSuccess) return VELORA_ERR_HIP;
    e = hipStreamSynchronize(st);
    if (e != hipSuccess) return VELORA_ERR_HIP;
    if (flag == 0) return VELORA_OK;
    return flag == VELORA_ERR_DEGENERATE ? VELORA_ERR_DEGENERATE : VELORA_ERR_HIP;
}

velora_status velora_update_v(const void* X, int64_t N, int64_t D, int64_t M, velora_dtype xdt, float* mean_state,
                              float beta, float* v, void* ws, size_t ws_bytes, velora_stream stream) {
    if (!X || !v) return VELORA_ERR_NULL;
    if (!dtype_ok(xdt)) return VELORA_ERR_DTYPE;
    if (!shape_ok(N, D, M) || !size_ok(N, D) || D / M > INT32_MAX / 8 || !(beta >= 0.f && beta <= 1.f))
        return VELORA_ERR_SHAPE;
    if (ptr_align(X) < elem_bytes(xdt) || ptr_align(v) < 4 || (mean_state && ptr_align(mean_state) < 4))
        return VELORA_ERR_ALIGN;
    const LaunchCfg cfg = current_cfg();
    const bool bf = xdt == VELORA_BF16;
    const velora::InitVPlan plan = velora::plan_init_v(N * M, D / M, bf, cfg);
    if (!ws || ws_bytes < plan.ws_bytes) return VELORA_ERR_WORKSPACE;
    if (ptr_align(ws) < 16) return VELORA_ERR_ALIGN;
    return hip_status(velora::launch_update_v(X, mean_state, static_cast<double>(beta), v, N * M, D / M, bf,
                                              ptr_align(X) >= 16, ws, plan, static_cast<hipStream_t>(stream)));
}

velora_status velora_compress_update(const void* X, const float* v_in, int64_t N, int64_t D, int64_t M,
                                     velora_dtype xdt, void* S, float* mean_state, float beta, float* v_out,
                                     void* ws, size_t ws_bytes, velora_stream stream) {
    if (!X || !v_in || !S || !v_out) return VELORA_ERR_NULL;
    if (!dtype_ok(xdt)) return VELORA_ERR_DTYPE;
    if (!shape_ok(N, D, M) || !size_ok(N, D) || D / M > INT32_MAX / 8 || !(beta >= 0.f && beta <= 1.f))
        return VELORA_ERR_SHAPE;
    const int eb = elem_bytes(xdt);
    if (ptr_align(X) < eb || ptr_align(S) < eb || ptr_align(v_in) < 4 || ptr_align(v_out) < 4 ||
        (mean_state && ptr_align(mean_state) < 4))
        return VELORA_ERR_ALIGN;
    const LaunchCfg cfg = current_cfg();
    const bool bf = xdt == VELORA_BF16;
    const velora::InitVPlan plan = velora::plan_init_v(N * M, D / M, bf, cfg);
    if (!ws || ws_bytes < plan.ws_bytes) return VELORA_ERR_WORKSPACE;
    if (ptr_align(ws) < 16) return VELORA_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool vec_ok = ptr_align(X) >= 16;
    if (velora::fused_compress_update_ok(D / M, bf, vec_ok))
        return hip_status(velora::launch_compress_update(X, v_in, S, mean_state, static_cast<double>(beta), v_out,
                                                         N * M, D / M, bf, ws, plan, st));
    // shapes the one-pass kernel does not take: compress, then the update as a second pass
    hipError_t e = velora::launch_compress(X, v_in, S, N * M, D / M, bf, vec_ok, cfg, st);
    if (e != hipSuccess) return VELORA_ERR_HIP;
    return hip_status(velora::launch_update_v(X, mean_state, static_cast<double>(beta), v_out, N * M, D / M, bf, vec_ok,
                                              ws, plan, st));
}

velora_status velora_compress(const void* X, const float* v, int64_t N, int64_t D, int64_t M, velora_dtype xdt,
                              void* S, velora_stream stream) {
    if (!X || !v || !S) return VELORA_ERR_NULL;
    if (!dtype_ok(xdt)) return VELORA_ERR_DTYPE;
    if (!shape_ok(N, D, M) || !size_ok(N, D) || D / M > INT32_MAX / 8) return VELORA_ERR_SHAPE;
    const int eb = elem_bytes(xdt);
    if (ptr_align(X) < eb || ptr_align(S) < eb || ptr_align(v) < 4) return VELORA_ERR_ALIGN;
    const LaunchCfg cfg = current_cfg();
    const bool vec_ok = ptr_align(X) >= 16;
    return hip_status(velora::launch_compress(X, v, S, N * M, D / M, xdt == VELORA_BF16, vec_ok, cfg,
                                              static_cast<hipStream_t>(stream)));
}

velora_status velora_swiglu_compress(const void* gate, const void* up, const float* v, int64_t N, int64_t D,
                                     int64_t M, velora_dtype dt, void* X, void* S, velora_stream stream) {
    if (!gate || !up || !v || !X || !S) return VELORA_ERR_NULL;
    if (!dtype_ok(dt)) return VELORA_ERR_DTYPE;
    if (!shape_ok(N, D, M) || !size_ok(N, D) || D / M > INT32_MAX / 8) return VELORA_ERR_SHAPE;
    const int eb = elem_bytes(dt);
    if (ptr_align(gate) < eb || ptr_align(up) < eb || ptr_align(X) < eb || ptr_align(S) < eb || ptr_align(v) < 4)
        return VELORA_ERR_ALIGN;
    const LaunchCfg cfg = current_cfg();
    const bool vec_ok = ptr_align(gate) >= 16 && ptr_align(up) >= 16 && ptr_align(X) >= 16;
    return hip_status(velora::launch_swiglu_compress(gate, up, v, X, S, N * M, D / M, dt == VELORA_BF16, vec_ok, cfg,
                                                     static_cast<hipStream_t>(stream)));
}

velora_status velora_linear_compress(const void* X, const void* W, const float* v, int64_t N, int64_t D, int64_t O,
                                     int64_t M, velora_dtype dt, void* Y, void* S, velora_stream stream) {
    if (!X || !W || !v || !Y || !S) return VELORA_ERR_NULL;
    if (!dtype_ok(dt)) return VELORA_ERR_DTYPE;
    if (!shape_ok(N, D, M) || !size_ok(N, D) || D / M > INT32_MAX / 8 || O <= 0 || O > INT64_C(65535) * 64 ||
        !size_ok(N, O) || !size_ok(O, D))
        return VELORA_ERR_SHAPE;
    const int eb = elem_bytes(dt);
    if (ptr_align(X) < eb || ptr_align(W) < eb || ptr_align(Y) < eb || ptr_align(S) < eb || ptr_align(v) < 4)
        return VELORA_ERR_ALIGN;
    const LaunchCfg cfg = current_cfg();
    const bool align16 = ptr_align(X) >= 16 && ptr_align(W) >= 16 && ptr_align(Y) >= 16;
    return hip_status(velora::launch_linear_compress(X, W, v, Y, S, N, D, O, M, dt == VELORA_BF16, align16,
                                                     ptr_align(X) >= 16, cfg, static_cast<hipStream_t>(stream)));
}

velora_status velora_grad_input(const void* G, const void* W, int64_t N, int64_t O, int64_t D, velora_dtype dt,
                                void* dX, velora_stream stream) {
    if (!G || !W || !dX) return VELORA_ERR_NULL;
    if (!dtype_ok(dt)) return VELORA_ERR_DTYPE;
    if (N <= 0 || O <= 0 || D <= 0 || D > INT64_C(65535) * 64 || !size_ok(N, O) || !size_ok(N, D) || !size_ok(O, D))
        return VELORA_ERR_SHAPE;
    const int eb = elem_bytes(dt);
    if (ptr_align(G) < eb || ptr_align(W) < eb || ptr_align(dX) < eb) return VELORA_ERR_ALIGN;
    const bool align16 = ptr_align(G) >= 16 && ptr_align(W) >= 16 && ptr_align(dX) >= 16;
    return hip_status(velora::launch_grad_input(G, W, dX, N, O, D, dt == VELORA_BF16, align16,
                                                static_cast<hipStream_t>(stream)));
}

velora_status velora_rmsnorm_compress(const void* H, const float* gamma, float eps, const float* v, int64_t N,
                                      int64_t D, int64_t M, velora_dtype dt, void* X, void* S,
                                      velora_stream stream) {
    if (!H || !gamma || !v || !X || !S) return VELORA_ERR_NULL;
    if (!dtype_ok(dt)) return VELORA_ERR_DTYPE;
    if (!shape_ok(N, D, M) || !size_ok(N, D) || D / M > INT32_MAX / 8 || !(eps >= 0.f)) return VELORA_ERR_SHAPE;
    const int eb = elem_bytes(dt);
    if (ptr_align(H) < eb || ptr_align(X) < eb || ptr_align(S) < eb || ptr_align(v) < 4 || ptr_align(gamma) < 4)
        return VELORA_ERR_ALIGN;
    const LaunchCfg cfg = current_cfg();
    const bool vec_ok = ptr_align(H) >= 16 && ptr_align(X) >= 16 && ptr_align(gamma) >= 16;
    return hip_status(velora::launch_rmsnorm_compress(H, gamma, v, X, S, N, D, M, eps, dt == VELORA_BF16, vec_ok, cfg,
                                                      static_cast<hipStream_t>(stream)));
}

velora_status velora_reconstruct(const void* S, const float* v, int64_t N, int64_t D, int64_t M, velora_dtype dt,
                                 void* Xhat, velora_stream stream) {
    if (!S || !v || !Xhat) return VELORA_ERR_NULL;
    if (!dtype_ok(dt)) return VELORA_ERR_DTYPE;
    if (!shape_ok(N, D, M) || !size_ok(N, D) || D / M > INT32_MAX / 8) return VELORA_ERR_SHAPE;
    const int eb = elem_bytes(dt);
    if (ptr_align(S) < eb || ptr_align(Xhat) < eb || ptr_align(v) < 4) return VELORA_ERR_ALIGN;
    const LaunchCfg cfg = current_cfg();
    const bool vec_ok = ptr_align(Xhat) >= 16 && ptr_align(v) >= 16;
    return hip_status(velora::launch_reconstruct(S, v, Xhat, N * M, D / M, dt == VELORA_BF16, vec_ok, cfg,
                                                 static_cast<hipStream_t>(stream)));
}

namespace {

// host-side checks shared by velora_weight_grad and velora_weight_grad_static
velora_status check_weight_grad(const void* G, const void* S, const float* v, int64_t N, int64_t O, int64_t D,
                                int64_t M, velora_dtype in_dt, const void* dW, velora_dtype dw_dt) {
    if (!G || !S || !v || !dW) return VELORA_ERR_NULL;
    if (!dtype_ok(in_dt) || !dtype_ok(dw_dt)) return VELORA_ERR_DTYPE;
    if (!shape_ok(N, D, M) || O <= 0 || !size_ok(N, D) || !size_ok(N, O) || !size_ok(O, D) ||
        D / M > INT32_MAX / 8 || O > INT32_MAX)
        return VELORA_ERR_SHAPE;
    const int eb = elem_bytes(in_dt);
    if (ptr_align(G) < eb || ptr_align(S) < eb || ptr_align(v) < 4 || ptr_align(dW) < elem_bytes(dw_dt))
        return VELORA_ERR_ALIGN;
    return VELORA_OK;
}

}  // namespace

velora_status velora_weight_grad(const void* G, const void* S, const float* v, int64_t N, int64_t O, int64_t D,
                                 int64_t M, velora_dtype in_dt, void* dW, velora_dtype dw_dt, int accumulate,
                                 void* ws, size_t ws_bytes, velora_stream stream) {
    const velora_status chk = check_weight_grad(G, S, v, N, O, D, M, in_dt, dW, dw_dt);
    if (chk != VELORA_OK) return chk;
    const LaunchCfg cfg = current_cfg();
    const bool bf = in_dt == VELORA_BF16;
    const velora::WgradPlan plan = velora::plan_wgrad(N, O, D, M, bf, cfg);
    if (!ws || ws_bytes < plan.ws_bytes) return VELORA_ERR_WORKSPACE;
    if (ptr_align(ws) < 16) return VELORA_ERR_ALIGN;
    return hip_status(velora::launch_wgrad(G, S, v, N, O, D, M, bf, ptr_align(G), ptr_align(S), ptr_align(v), dW,
                                           dw_dt == VELORA_BF16, ptr_align(dW), accumulate != 0, ws, plan, cfg,
                                           static_cast<hipStream_t>(stream)));
}

velora_status velora_weight_grad_static(const void* G, const void* S, const float* v, int64_t N, int64_t O, int64_t D,
                                        int64_t M, velora_dtype in_dt, void* dW, velora_dtype dw_dt, int accumulate,
                                        velora_stream stream) {
    const velora_status chk = check_weight_grad(G, S, v, N, O, D, M, in_dt, dW, dw_dt);
    if (chk != VELORA_OK) return chk;
    const LaunchCfg cfg = current_cfg();
    const bool bf = in_dt == VELORA_BF16;
    const velora::WgradPlan plan = velora::plan_wgrad(N, O, D, M, bf, cfg);
    if (plan.ws_bytes > VELORA_STATIC_SCRATCH_BYTES) return VELORA_ERR_WORKSPACE;   // refused before the device is touched
    // The array's name is only a host-side handle: its device address differs per GPU and is looked up
    // once per device, with that device current; from then on only the looked-up pointer is used.
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return VELORA_ERR_HIP;
    }
    void* scratch = g_static_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!scratch) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(velora_static_scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return VELORA_ERR_HIP;
        }
        g_static_scratch_ptr[dev].store(p, std::memory_order_release);
        scratch = p;
    }
    return hip_status(velora::launch_wgrad(G, S, v, N, O, D, M, bf, ptr_align(G), ptr_align(S), ptr_align(v), dW,
                                           dw_dt == VELORA_BF16, ptr_align(dW), accumulate != 0, scratch, plan, cfg,
                                           static_cast<hipStream_t>(stream)));
}

velora_status velora_weight_grad_factor(const void* G, const void* S, int64_t N, int64_t O, int64_t M,
                                        velora_dtype in_dt, float* T, void* ws, size_t ws_bytes,
                                        velora_stream stream) {
    if (!G || !S || !T) return VELORA_ERR_NULL;
    if (!dtype_ok(in_dt)) return VELORA_ERR_DTYPE;
    if (N <= 0 || O <= 0 || M <= 0 || !size_ok(N, O) || !size_ok(N, M) || !size_ok(O, M) || O > INT32_MAX)
        return VELORA_ERR_SHAPE;
    const int eb = elem_bytes(in_dt);
    if (ptr_align(G) < eb || ptr_align(S) < eb || ptr_align(T) < 4) return VELORA_ERR_ALIGN;
    const LaunchCfg cfg = current_cfg();
    const bool bf = in_dt == VELORA_BF16;
    // the split plan of the factor does not depend on d; D = M stands for "no expansion"
    const velora::WgradPlan plan = velora::plan_wgrad(N, O, M, M, bf, cfg);
    if (!ws || ws_bytes < plan.ws_bytes) return VELORA_ERR_WORKSPACE;
    if (ptr_align(ws) < 16) return VELORA_ERR_ALIGN;
    return hip_status(velora::launch_wgrad_factor(G, S, N, O, M, bf, ptr_align(G), ptr_align(S), T, ws, plan,
                                                  static_cast<hipStream_t>(stream)));
}

velora_status velora_expand_factor(const float* T, const float* v, int64_t O, int64_t D, int64_t M, void* dW,
                                   velora_dtype dw_dt, int accumulate, velora_stream stream) {
    if (!T || !v || !dW) return VELORA_ERR_NULL;
    if (!dtype_ok(dw_dt)) return VELORA_ERR_DTYPE;
    if (!shape_ok(O, D, M) || !size_ok(O, D) || D / M > INT32_MAX / 8 || O > INT32_MAX) return VELORA_ERR_SHAPE;
    if (ptr_align(T) < 4 || ptr_align(v) < 4 || ptr_align(dW) < elem_bytes(dw_dt)) return VELORA_ERR_ALIGN;
    return hip_status(velora::launch_expand_factor(T, v, ptr_align(v), dW, dw_dt == VELORA_BF16, ptr_align(dW),
                                                   accumulate != 0, O, D, M, current_cfg(),
                                                   static_cast<hipStream_t>(stream)));
}

velora_status velora_adamw_step_factor(const float* T, const float* v, int64_t O, int64_t D, int64_t M, void* W,
                                       velora_dtype w_dt, float* exp_avg, float* exp_avg_sq, float lr, float beta1,
                                       float beta2, float eps, float weight_decay, int64_t step, float grad_scale,
                                       velora_stream stream) {
    if (!T || !v || !W || !exp_avg || !exp_avg_sq) return VELORA_ERR_NULL;
    if (!dtype_ok(w_dt)) return VELORA_ERR_DTYPE;
    if (!shape_ok(O, D, M) || !size_ok(O, D)) return VELORA_ERR_SHAPE;
    if (step < 1 || !(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f) || !(eps >= 0.f) ||
        !std::isfinite(lr) || !std::isfinite(weight_decay) || !std::isfinite(grad_scale))
        return VELORA_ERR_SHAPE;
    if (ptr_align(T) < 4 || ptr_align(v) < 4 || ptr_align(exp_avg) < 4 || ptr_align(exp_avg_sq) < 4 ||
        ptr_align(W) < elem_bytes(w_dt))
        return VELORA_ERR_ALIGN;
    const int64_t d = D / M;
    const bool vec_ok = d % 4 == 0 && ptr_align(v) >= 16 && ptr_align(exp_avg) >= 16 && ptr_align(exp_avg_sq) >= 16 &&
                        ptr_align(W) >= (w_dt == VELORA_BF16 ? 8 : 16);
    velora::AdamWScalars a;
    const double bc1 = 1.0 - std::pow(static_cast<double>(beta1), static_cast<double>(step));
    const double bc2 = 1.0 - std::pow(static_cast<double>(beta2), static_cast<double>(step));
    a.decay = static_cast<float>(1.0 - static_cast<double>(lr) * static_cast<double>(weight_decay));
    a.beta1 = beta1;
    a.one_minus_beta1 = static_cast<float>(1.0 - static_cast<double>(beta1));
    a.beta2 = beta2;
    a.one_minus_beta2 = static_cast<float>(1.0 - static_cast<double>(beta2));
    a.step_size = static_cast<float>(static_cast<double>(lr) / bc1);
    a.inv_sqrt_bc2 = static_cast<float>(1.0 / std::sqrt(bc2));
    a.eps = eps;
    a.grad_scale = grad_scale;
    return hip_status(velora::launch_adamw_factor(T, v, W, w_dt == VELORA_BF16, exp_avg, exp_avg_sq, O, D, M, vec_ok, a,
                                                  static_cast<hipStream_t>(stream)));
}

velora_status velora_bandwidth_probe(int kind, const void* src, void* dst, int64_t bytes, uint32_t* sink,
                                     velora_stream stream) {
    if (kind < 0 || kind > 2 || bytes <= 0 || bytes % 16 != 0) return VELORA_ERR_SHAPE;
    if ((kind != 1 && !src) || (kind != 0 && !dst) || (kind == 0 && !sink)) return VELORA_ERR_NULL;
    if ((kind != 1 && ptr_align(src) < 16) || (kind != 0 && ptr_align(dst) < 16) || (kind == 0 && ptr_align(sink) < 4))
        return VELORA_ERR_ALIGN;
    return hip_status(velora::launch_probe(kind, src, dst, bytes, sink, current_cfg(), static_cast<hipStream_t>(stream)));
}

}  // extern "C"
