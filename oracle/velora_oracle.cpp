// CPU oracle for the VeLoRA hot path.  TEST INFRASTRUCTURE ONLY.
//
// This file is the plain, slow, obviously-correct statement of what the
// library's kernels must compute.  It is used by the tests, by the smoke
// check and by the benchmark's cpu_baseline leg, and by nothing else: the
// product path never calls it and shares no code, header, table or helper
// with it.  It is written from the paper's definitions:
//
//   group / ungroup   : Sec. 3.1 ("VeLoRA"), Eq. 1 and Eq. 2 (a reshape that
//                       splits every token of depth D into D/d contiguous,
//                       non-overlapping sub-tokens of size d);
//   compress(z; v)    : Sec. 3.1, z_p = z . v  (one scalar per sub-token);
//   reconstruct(z_p;v): Sec. 3.1, z_hat = z_p . v^T;
//   proj_v            : Sec. 3.1, (z . v) . v^T with v a fixed unit vector;
//   init of v         : Sec. 3.2 "Cheap initialisation strategies" (average
//                       of the first batch's sub-tokens) + unit length (Sec. 3.1);
//   per-batch v       : Sec. 5.3 "Initialisation strategy" / Table 5c (running
//                       average, instance-wise); no formula is printed, the
//                       reading is stated at the function;
//   grad_weight       : Listing 1 (backward): grad_output^T @ input_hat.
//
// Naming: the paper writes M for the sub-token size.  Here d is the sub-token
// size and M = D/d the number of sub-tokens per token.
//
// All arithmetic is double precision; inputs are widened exactly from their
// storage dtype (float32, or bfloat16 given as uint16 bit patterns).  Threads
// only partition independent outputs; no blocking, fusion or reordering of the
// sums: every sum runs over its index in ascending order.
//
// Parity status: every function below is pinned by tests/test_oracle_pins.py
// (closed forms, invariants, special cases, brute force).  Nothing here is
// "parity unpinned".

#include <cmath>
#include <cstdint>
#include <cstring>
#include <functional>
#include <thread>
#include <vector>

namespace {

enum { DT_F32 = 0, DT_BF16 = 1 };

// ---- storage formats, from their definitions ------------------------------
// bfloat16 = the upper 16 bits of an IEEE-754 binary32 (1 sign, 8 exponent,
// 7 fraction bits).
inline double widen_bf16(uint16_t b) {
    uint32_t u = static_cast<uint32_t>(b) << 16;
    float f;
    std::memcpy(&f, &u, 4);
    return static_cast<double>(f);
}

// Round a double to the nearest bfloat16, ties to even, in ONE rounding.
uint16_t round_to_bf16(double x) {
    uint16_t sign = std::signbit(x) ? 0x8000u : 0u;
    if (std::isnan(x)) return 0x7FC0u;
    double a = std::fabs(x);
    if (a == 0.0) return sign;
    if (std::isinf(a)) return sign | 0x7F80u;
    int e;
    std::frexp(a, &e);               // a = f * 2^e, f in [0.5, 1)
    int E = e - 1;                   // floor(log2 a)
    if (E < -126) E = -126;          // subnormal range shares the exponent -126
    // significand in units of 2^(E-7); nearbyint honours the default
    // round-to-nearest-even mode.
    double q = std::nearbyint(std::ldexp(a, 7 - E));
    if (q >= 256.0) { q = 128.0; E += 1; }
    if (E > 127) return sign | 0x7F80u;
    uint16_t bits;
    if (q < 128.0) bits = static_cast<uint16_t>(q);                      // subnormal
    else bits = static_cast<uint16_t>(((E + 127) << 7) | (static_cast<int>(q) - 128));
    return sign | bits;
}

inline double load(const void* p, int dt, int64_t i) {
    if (dt == DT_F32) return static_cast<double>(static_cast<const float*>(p)[i]);
    return widen_bf16(static_cast<const uint16_t*>(p)[i]);
}

inline void store(void* p, int dt, int64_t i, double x) {
    if (dt == DT_F32) static_cast<float*>(p)[i] = static_cast<float>(x);   // RNE cast
    else static_cast<uint16_t*>(p)[i] = round_to_bf16(x);
}

// Run fn(begin, end) over [0, n) split into contiguous ranges, one per thread.
void parallel_ranges(int64_t n, int nthreads, const std::function<void(int64_t, int64_t)>& fn) {
    if (nthreads < 1) nthreads = 1;
    if (nthreads > n) nthreads = static_cast<int>(n > 0 ? n : 1);
    if (nthreads == 1) { fn(0, n); return; }
    std::vector<std::thread> th;
    int64_t per = (n + nthreads - 1) / nthreads;
    for (int t = 0; t < nthreads; ++t) {
        int64_t b = t * per, e = b + per;
        if (e > n) e = n;
        if (b >= e) break;
        th.emplace_back(fn, b, e);
    }
    for (auto& t : th) t.join();
}

}  // namespace

extern "C" {

uint16_t velora_oracle_round_bf16(double x) { return round_to_bf16(x); }
double velora_oracle_widen_bf16(uint16_t b) { return widen_bf16(b); }

// out[i] = x[i] stored as dt (float32 by the cast, bfloat16 by round_to_bf16): one rounding from float64.
void velora_oracle_store_array(const double* x, int dt, int64_t n, void* out) {
    for (int64_t i = 0; i < n; ++i) store(out, dt, i, x[i]);
}

// Sec. 3.2: v = average of all N*M sub-tokens of the first batch; Sec. 3.1:
// unit length.  mean_out (may be null) receives the un-normalised average.
// Returns 0, or 6 when the average is zero or not finite, in which case
// v[j] = 1/sqrt(d) (the paper is silent on this case).
int velora_oracle_init_v(const void* X, int dt, int64_t N, int64_t D, int64_t M,
                         double* mean_out, float* v_out, int nthreads) {
    const int64_t d = D / M;
    std::vector<double> m(static_cast<size_t>(d), 0.0);
    // each j is an independent sum over (n, g) in ascending order
    parallel_ranges(d, nthreads, [&](int64_t j0, int64_t j1) {
        for (int64_t j = j0; j < j1; ++j) {
            double acc = 0.0;
            for (int64_t n = 0; n < N; ++n)
                for (int64_t g = 0; g < M; ++g)
                    acc += load(X, dt, n * D + g * d + j);
            m[static_cast<size_t>(j)] = acc / static_cast<double>(N * M);
        }
    });
    double ss = 0.0;
    bool finite = true;
    for (int64_t j = 0; j < d; ++j) {
        ss += m[j] * m[j];
        if (!std::isfinite(m[j])) finite = false;
    }
    if (mean_out) for (int64_t j = 0; j < d; ++j) mean_out[j] = m[j];
    double norm = std::sqrt(ss);
    if (!finite || !(norm > 0.0) || !std::isfinite(norm)) {
        for (int64_t j = 0; j < d; ++j) v_out[j] = static_cast<float>(1.0 / std::sqrt(static_cast<double>(d)));
        return 6;
    }
    for (int64_t j = 0; j < d; ++j) v_out[j] = static_cast<float>(m[j] / norm);
    return 0;
}

// Per-batch vector (the "running average" / instance-wise rows of the
// initialisation ablation, Sec. 5.3, Table 5c).  The paper prints no formula;
// the reading taken: m_b = this batch's sub-token average (as in init_v),
// m = beta * state_in + (1 - beta) * m_b when a state is given, else m = m_b;
// state_out = m rounded to float32; v = m / ||m|| (from the unrounded m).
// Same degenerate rule and return value as velora_oracle_init_v.
int velora_oracle_update_v(const void* X, int dt, int64_t N, int64_t D, int64_t M, const float* state_in,
                           double beta, float* state_out, float* v_out, int nthreads) {
    const int64_t d = D / M;
    std::vector<double> mb(static_cast<size_t>(d));
    std::vector<float> tmp(static_cast<size_t>(d));
    velora_oracle_init_v(X, dt, N, D, M, mb.data(), tmp.data(), nthreads);
    double ss = 0.0;
    bool finite = true;
    std::vector<double> m(static_cast<size_t>(d));
    for (int64_t j = 0; j < d; ++j) {
        m[j] = state_in ? beta * static_cast<double>(state_in[j]) + (1.0 - beta) * mb[j] : mb[j];
        ss += m[j] * m[j];
        if (!std::isfinite(m[j])) finite = false;
    }
    if (state_out) for (int64_t j = 0; j < d; ++j) state_out[j] = static_cast<float>(m[j]);
    const double norm = std::sqrt(ss);
    if (!finite || !(norm > 0.0) || !std::isfinite(norm)) {
        for (int64_t j = 0; j < d; ++j) v_out[j] = static_cast<float>(1.0 / std::sqrt(static_cast<double>(d)));
        return 6;
    }
    for (int64_t j = 0; j < d; ++j) v_out[j] = static_cast<float>(m[j] / norm);
    return 0;
}

// Sec. 3.1: S[n, g] = sum_j X[n, g*d + j] * v[j].
// S_exact (double, may be null) and S_store (storage dtype, may be null).
void velora_oracle_compress(const void* X, int dt, const float* v, int64_t N, int64_t D, int64_t M,
                            double* S_exact, void* S_store, int nthreads) {
    const int64_t d = D / M;
    parallel_ranges(N, nthreads, [&](int64_t n0, int64_t n1) {
        for (int64_t n = n0; n < n1; ++n)
            for (int64_t g = 0; g < M; ++g) {
                double acc = 0.0;
                for (int64_t j = 0; j < d; ++j)
                    acc += load(X, dt, n * D + g * d + j) * static_cast<double>(v[j]);
                if (S_exact) S_exact[n * M + g] = acc;
                if (S_store) store(S_store, dt, n * M + g, acc);
            }
    });
}

// Sec. 3.1: Xhat[n, g*d + j] = S[n, g] * v[j]  (reconstruct, then ungroup).
void velora_oracle_reconstruct(const void* S, int dt, const float* v, int64_t N, int64_t D, int64_t M,
                               double* Xhat, int nthreads) {
    const int64_t d = D / M;
    parallel_ranges(N, nthreads, [&](int64_t n0, int64_t n1) {
        for (int64_t n = n0; n < n1; ++n)
            for (int64_t g = 0; g < M; ++g) {
                double s = load(S, dt, n * M + g);
                for (int64_t j = 0; j < d; ++j)
                    Xhat[n * D + g * d + j] = s * static_cast<double>(v[j]);
            }
    });
}

// Listing 1, backward: materialise Xhat, then dW[o, c] = sum_n G[n, o] * Xhat[n, c].
void velora_oracle_weight_grad_bruteforce(const void* G, const void* S, const float* v,
                                          int64_t N, int64_t O, int64_t D, int64_t M, int dt,
                                          double* dW, int nthreads) {
    std::vector<double> Xhat(static_cast<size_t>(N * D));
    velora_oracle_reconstruct(S, dt, v, N, D, M, Xhat.data(), nthreads);
    parallel_ranges(O, nthreads, [&](int64_t o0, int64_t o1) {
        for (int64_t o = o0; o < o1; ++o) {
            double* row = dW + o * D;
            for (int64_t c = 0; c < D; ++c) row[c] = 0.0;
            for (int64_t n = 0; n < N; ++n) {
                double g = load(G, dt, n * O + o);
                const double* xh = Xhat.data() + n * D;
                for (int64_t c = 0; c < D; ++c) row[c] += g * xh[c];
            }
        }
    });
}

// The same definition evaluated for a chosen set of output rows only (used at
// sizes where all O rows would take hours).  Xhat is formed one token at a
// time; out[r, c] = dW[rows[r], c].
void velora_oracle_weight_grad_bruteforce_rows(const void* G, const void* S, const float* v,
                                               int64_t N, int64_t O, int64_t D, int64_t M, int dt,
                                               const int64_t* rows, int64_t nrows,
                                               double* out, int nthreads) {
    const int64_t d = D / M;
    parallel_ranges(nrows, nthreads, [&](int64_t r0, int64_t r1) {
        std::vector<double> xh(static_cast<size_t>(D));
        for (int64_t r = r0; r < r1; ++r)
            for (int64_t c = 0; c < D; ++c) out[r * D + c] = 0.0;
        for (int64_t n = 0; n < N; ++n) {
            for (int64_t g = 0; g < M; ++g) {
                double s = load(S, dt, n * M + g);
                for (int64_t j = 0; j < d; ++j) xh[g * d + j] = s * static_cast<double>(v[j]);
            }
            for (int64_t r = r0; r < r1; ++r) {
                double gg = load(G, dt, n * O + rows[r]);
                double* row = out + r * D;
                for (int64_t c = 0; c < D; ++c) row[c] += gg * xh[c];
            }
        }
    });
}

// The algebraically identical association: because Xhat[n, g*d+j] = S[n,g]*v[j],
// T[o, g] = sum_n G[n, o] * S[n, g] and dW[o, g*d + j] = T[o, g] * v[j].
// T_out (may be null) receives T[O, M].
void velora_oracle_weight_grad_factored(const void* G, const void* S, const float* v,
                                        int64_t N, int64_t O, int64_t D, int64_t M, int dt,
                                        double* T_out, double* dW, int nthreads) {
    const int64_t d = D / M;
    parallel_ranges(O, nthreads, [&](int64_t o0, int64_t o1) {
        std::vector<double> T(static_cast<size_t>(M));
        for (int64_t o = o0; o < o1; ++o) {
            for (int64_t g = 0; g < M; ++g) T[g] = 0.0;
            for (int64_t n = 0; n < N; ++n) {
                double gg = load(G, dt, n * O + o);
                for (int64_t g = 0; g < M; ++g) T[g] += gg * load(S, dt, n * M + g);
            }
            for (int64_t g = 0; g < M; ++g) {
                if (T_out) T_out[o * M + g] = T[g];
                if (dW)
                    for (int64_t j = 0; j < d; ++j) dW[o * D + g * d + j] = T[g] * static_cast<double>(v[j]);
            }
        }
    });
}

// Listing 1, forward (the dense product is left as it is): Y[n, o] = sum_c X[n, c] * W[o, c],
// with the weight stored [O, D] as the shape of grad_weight implies.
void velora_oracle_linear(const void* X, const void* W, int dt, int64_t N, int64_t D, int64_t O,
                          double* Y, int nthreads) {
    parallel_ranges(N, nthreads, [&](int64_t n0, int64_t n1) {
        for (int64_t n = n0; n < n1; ++n)
            for (int64_t o = 0; o < O; ++o) {
                double acc = 0.0;
                for (int64_t c = 0; c < D; ++c) acc += load(X, dt, n * D + c) * load(W, dt, o * D + c);
                Y[n * O + o] = acc;
            }
    });
}

}  // extern "C"
