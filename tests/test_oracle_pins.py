"""Pins for the CPU oracle: everything here runs without a GPU.

The oracle (oracle/velora_oracle.cpp) is checked against things other than
itself: a hand-worked example (tests/golden/worked_example_sec3_1.txt), closed
forms, projector invariants that follow from |v| = 1 (paper Sec. 3.1), the
gradient-similarity identity of the appendix ("Gradient Similarity"), the
no-sub-token special case of Sec. 3.2 ("Connection to parameter efficient
fine-tuning"), special cases that reduce to a gather or to a textbook matrix
product, and pure-Python brute force on tiny inputs.
"""
import math
import os

import numpy as np
import pytest

import oracle
import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "worked_example_sec3_1.txt")


def _read_golden():
    out, name = {}, None
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            try:
                row = [float(t) for t in line.split()]
                out[name].append(row)
            except ValueError:
                name = line
                out[name] = []
    return {k: np.array(v, dtype=np.float64) for k, v in out.items()}


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _rand(shape, seed, dtype=wl.F32, sigma=1.0):
    return wl.random_tensor(shape[0], shape[1], dtype, seed, sigma=sigma)


# ------------------------------------------------------------------ bf16 format
class TestBf16Format:
    def test_roundtrip_all_bit_patterns(self):
        for b in range(0, 1 << 16, 1):
            exp = (b >> 7) & 0xFF
            if exp == 0xFF and (b & 0x7F):      # NaN payloads are not preserved
                continue
            assert oracle.round_bf16(oracle.widen_bf16(b)) == b

    def test_ties_to_even_and_single_rounding(self):
        one = 0x3F80
        assert oracle.round_bf16(1.0 + 2.0 ** -8) == one             # tie -> even (down)
        assert oracle.round_bf16(1.0 + 3 * 2.0 ** -8) == one + 2      # tie -> even (up)
        assert oracle.round_bf16(1.0 + 2.0 ** -8 + 2.0 ** -30) == one + 1
        # would be a tie after a first rounding to float32; one rounding from
        # double must see that it lies above the tie
        assert oracle.round_bf16(1.0 + 2.0 ** -8 + 2.0 ** -40) == one + 1
        assert oracle.round_bf16(-(1.0 + 2.0 ** -8)) == 0x8000 | one

    def test_range_ends(self):
        assert oracle.round_bf16(0.0) == 0
        assert oracle.round_bf16(-0.0) == 0x8000
        assert oracle.round_bf16(1e40) == 0x7F80
        assert oracle.round_bf16(-1e40) == 0xFF80
        big = oracle.widen_bf16(0x7F7F)                               # largest finite
        assert oracle.round_bf16(big) == 0x7F7F
        assert oracle.round_bf16(big * (1 + 2.0 ** -8)) == 0x7F80     # more than half an ulp above it
        assert oracle.round_bf16(big * (1 + 2.0 ** -10)) == 0x7F7F    # less than half an ulp above it
        assert oracle.round_bf16(2.0 ** -133) == 1                    # smallest subnormal
        assert oracle.round_bf16(2.0 ** -134) == 0                    # tie -> even (0)
        assert oracle.round_bf16(2.0 ** -126) == 0x0080               # smallest normal

    def test_agrees_with_independent_bit_trick(self):
        a = np.random.default_rng(3).standard_normal(20000).astype(np.float32) * 37.0
        want = wl.f32_to_bf16_bits(a)
        got = np.array([oracle.round_bf16(float(x)) for x in a], dtype=np.uint16)
        assert (got == want).all()

    def test_array_store_rounds_once(self):
        """The store of Y and dX in the training dtype is one rounding from float64: a value just above a
        bfloat16 tie, by less than float32 resolves, must go up (through float32 first it would land on the
        tie and go to even), and the array routine agrees with the scalar one element by element."""
        one = 0x3F80
        x = np.array([1.0 + 2.0 ** -8 + 2.0 ** -30, 1.0 + 2.0 ** -8, -(1.0 + 3 * 2.0 ** -8 - 2.0 ** -40), 0.0, 1e40,
                      2.0 ** -134, 3.0e-39], dtype=np.float64)
        got = oracle._store(x, oracle.DT_BF16)
        assert got.dtype == np.uint16
        assert got[0] == one + 1 and got[1] == one and got[2] == (0x8000 | (one + 1)) and got[4] == 0x7F80
        assert (got == np.array([oracle.round_bf16(float(t)) for t in x], dtype=np.uint16)).all()
        r = np.random.default_rng(9).standard_normal((37, 53)) * 1e-3
        got2 = oracle._store(r, oracle.DT_BF16)
        assert got2.shape == r.shape
        assert (got2.ravel() == np.array([oracle.round_bf16(float(t)) for t in r.ravel()], dtype=np.uint16)).all()
        f = oracle._store(r, oracle.DT_F32)
        assert f.dtype == np.float32 and (f == r.astype(np.float32)).all()


# ------------------------------------------------------------------ worked example
class TestWorkedExample:
    def test_compress_reconstruct_weight_grad_init(self):
        g = _read_golden()
        v = _f32(g["v"][0])
        X = _f32(g["X"])
        G = _f32(g["G"])
        S_exact, S_store = oracle.compress(X, v, M=2)
        np.testing.assert_allclose(S_exact, g["S"], rtol=0, atol=2e-7)
        np.testing.assert_allclose(S_store, g["S"], rtol=0, atol=5e-7)
        Xhat = oracle.reconstruct(S_store, v, D=4)
        np.testing.assert_allclose(Xhat, g["Xhat"], rtol=0, atol=1e-6)
        dW = oracle.weight_grad_bruteforce(G, S_store, v, D=4)
        np.testing.assert_allclose(dW, g["dW"], rtol=0, atol=3e-6)
        T, dWf = oracle.weight_grad_factored(G, S_store, v, D=4)
        np.testing.assert_allclose(dWf, g["dW"], rtol=0, atol=3e-6)
        vi, mean, rc = oracle.init_v(X, M=2)
        assert rc == 0
        np.testing.assert_allclose(mean, g["mean"][0], rtol=0, atol=1e-15)
        np.testing.assert_allclose(vi, g["v_init"][0], rtol=0, atol=6e-8)


# ------------------------------------------------------------------ compress / reconstruct
class TestCompressReconstruct:
    @pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
    def test_gather_is_bit_exact(self, dtype):
        # v = e_j turns compress into a gather: pins group()'s indexing with no arithmetic.
        N, D, d = 7, 48, 8
        M = D // d
        X = _rand((N, D), 11, dtype)
        for j in (0, 3, 7):
            v = np.zeros(d, dtype=np.float32)
            v[j] = 1.0
            S_exact, S_store = oracle.compress(X, v, M)
            want = X.reshape(N, M, d)[:, :, j]
            assert (S_store == want).all()
            assert (S_exact == wl.to_f64(want, dtype)).all()

    def test_exact_on_multiples_of_v(self):
        # sub-token k = c_k * v with v = (1/4,...,1/4) in R^16 (unit length) and
        # integer c_k: every quantity is exactly representable.
        N, M, d = 5, 3, 16
        v = np.full(d, 0.25, dtype=np.float32)
        c = np.arange(-7, 8, dtype=np.float64).reshape(N, M)
        X = _f32((c[:, :, None] * v[None, None, :].astype(np.float64)).reshape(N, M * d))
        S_exact, S_store = oracle.compress(X, v, M)
        assert (S_exact == c).all()
        assert (S_store == c).all()
        Xhat = oracle.reconstruct(S_store, v, D=M * d)
        assert (Xhat == X.astype(np.float64)).all()

    def test_sign_and_d_equals_one(self):
        X = _rand((9, 10), 5)
        for sgn in (1.0, -1.0):
            S_exact, S_store = oracle.compress(X, np.array([sgn], dtype=np.float32), M=10)
            assert (S_store == sgn * X).all()
            Xhat = oracle.reconstruct(S_store, np.array([sgn], dtype=np.float32), D=10)
            assert (Xhat == X.astype(np.float64)).all()

    def test_against_python_loops(self):
        N, D, d = 3, 6, 2
        M = D // d
        X = _rand((N, D), 21)
        v = wl.random_unit_v(d, 4)
        S_exact, _ = oracle.compress(X, v, M)
        for n in range(N):
            for g in range(M):
                acc = 0.0
                for j in range(d):
                    acc += float(X[n, g * d + j]) * float(v[j])
                assert S_exact[n, g] == pytest.approx(acc, rel=1e-15, abs=1e-300)

    @pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
    def test_matches_reshape_matvec(self, dtype):
        N, D, d = 33, 96, 32
        M = D // d
        X = _rand((N, D), 8, dtype)
        v = wl.random_unit_v(d, 2)
        S_exact, S_store = oracle.compress(X, v, M)
        want = (wl.to_f64(X, dtype).reshape(N * M, d) @ v.astype(np.float64)).reshape(N, M)
        np.testing.assert_allclose(S_exact, want, rtol=1e-13, atol=1e-14)
        # the stored value is the exact value rounded once to the storage dtype
        if dtype == wl.F32:
            assert (S_store == S_exact.astype(np.float32)).all()
        else:
            ulp = np.abs(want) * 2.0 ** -8 + 1e-30
            assert (np.abs(wl.to_f64(S_store, dtype) - want) <= ulp).all()

    def test_projector_invariants(self):
        N, D, d = 17, 64, 16
        M = D // d
        X = _rand((N, D), 13)
        v = wl.random_unit_v(d, 9)
        vd = v.astype(np.float64)
        vn2 = float(vd @ vd)                      # 1 up to float32 rounding of v
        S, _ = oracle.compress(X, v, M)
        z = X.astype(np.float64).reshape(N * M, d)
        s = S.reshape(-1)
        # contraction (Cauchy-Schwarz with |v| = 1)
        assert (np.abs(s) <= np.linalg.norm(z, axis=1) * math.sqrt(vn2) * (1 + 1e-12)).all()
        # reconstruct from exact S (float64 S given as f32 would round): use numpy outer
        S32 = _f32(S)
        Xhat = oracle.reconstruct(S32, v, D).reshape(N * M, d)
        s32 = S32.astype(np.float64).reshape(-1)
        # residual orthogonal to v, Pythagoras, |Xhat| <= |X|
        res = z - Xhat
        np.testing.assert_allclose(res @ vd, s - s32 * vn2, atol=1e-12)
        assert np.linalg.norm(Xhat) <= np.linalg.norm(z) * (1 + 1e-6)
        np.testing.assert_allclose((z * z).sum(1), s * s + ((z - s[:, None] * vd) ** 2).sum(1), rtol=1e-6)
        # idempotence: compress(reconstruct(S)) = S * |v|^2
        S2, _ = oracle.compress(_f32(Xhat.reshape(N, D)), v, M)
        np.testing.assert_allclose(S2.reshape(-1), s32 * vn2, rtol=0, atol=3e-7)
        # appendix "Gradient Similarity": sim(proj z_i, proj z_j) = (v.z_i)(v.z_j)
        gram = Xhat @ Xhat.T
        np.testing.assert_allclose(gram, np.outer(s32, s32) * vn2, rtol=1e-12, atol=1e-12)

    def test_linearity(self):
        N, D, d = 6, 32, 8
        A = _rand((N, D), 1)
        B = _rand((N, D), 2)
        v = wl.random_unit_v(d, 3)
        # integer combinations of float32 stay exactly representable only if we
        # form the combination in float64 and compare against float64 sums
        SA, _ = oracle.compress(A, v, D // d)
        SB, _ = oracle.compress(B, v, D // d)
        C = _f32(2.0 * A.astype(np.float64) - 0.5 * B.astype(np.float64))
        SC, _ = oracle.compress(C, v, D // d)
        np.testing.assert_allclose(SC, 2.0 * SA - 0.5 * SB, rtol=0, atol=2e-6)

    def test_reconstruct_python_loops(self):
        N, M, d = 2, 3, 4
        S = _rand((N, M), 17)
        v = wl.random_unit_v(d, 6)
        Xhat = oracle.reconstruct(S, v, M * d)
        for n in range(N):
            for g in range(M):
                for j in range(d):
                    assert Xhat[n, g * d + j] == float(S[n, g]) * float(v[j])


# ------------------------------------------------------------------ init_v
class TestInitV:
    def test_constant_subtokens(self):
        d, M, N = 8, 4, 5
        u = np.array([1, -2, 3, 0.5, 0, 4, -1, 2], dtype=np.float64)
        X = _f32(np.tile(u, (N, M)))
        v, mean, rc = oracle.init_v(X, M)
        assert rc == 0
        np.testing.assert_allclose(mean, u, rtol=0, atol=1e-15)
        np.testing.assert_allclose(v, u / np.linalg.norm(u), rtol=0, atol=6e-8)
        # natural sign is kept
        v2, _, _ = oracle.init_v(-X, M)
        np.testing.assert_allclose(v2, -u / np.linalg.norm(u), rtol=0, atol=6e-8)

    def test_mean_runs_over_tokens_and_groups(self):
        # sub-token (n, g) = (n + 1) * (g + 1) * u  ->  mean = mean_n(n+1) * mean_g(g+1) * u
        d, M, N = 4, 3, 5
        u = np.array([1.0, 2.0, -1.0, 0.5])
        X = np.zeros((N, M * d))
        for n in range(N):
            for g in range(M):
                X[n, g * d:(g + 1) * d] = (n + 1) * (g + 1) * u
        v, mean, rc = oracle.init_v(_f32(X), M)
        np.testing.assert_allclose(mean, 3.0 * 2.0 * u, rtol=1e-15)
        np.testing.assert_allclose(np.linalg.norm(v.astype(np.float64)), 1.0, atol=1e-7)

    @pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
    def test_matches_column_mean_and_permutation_invariance(self, dtype):
        N, D, d = 40, 96, 16
        M = D // d
        X = _rand((N, D), 31, dtype)
        X64 = wl.to_f64(X, dtype)
        v, mean, rc = oracle.init_v(X, M)
        want = X64.reshape(N * M, d).mean(axis=0)
        np.testing.assert_allclose(mean, want, rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(v, want / np.linalg.norm(want), atol=6e-8)
        assert abs(np.linalg.norm(v.astype(np.float64)) - 1.0) < 2e-7
        perm = np.random.default_rng(0).permutation(N)
        v2, mean2, _ = oracle.init_v(np.ascontiguousarray(X[perm]), M)
        np.testing.assert_allclose(mean2, mean, rtol=1e-12, atol=1e-16)
        gperm = np.random.default_rng(1).permutation(M)
        Xg = np.ascontiguousarray(X.reshape(N, M, d)[:, gperm, :].reshape(N, D))
        _, mean3, _ = oracle.init_v(Xg, M)
        np.testing.assert_allclose(mean3, mean, rtol=1e-12, atol=1e-16)

    def test_degenerate(self):
        d, M = 4, 2
        v, mean, rc = oracle.init_v(np.zeros((3, M * d), dtype=np.float32), M)
        assert rc == oracle.ERR_DEGENERATE
        assert (v == np.float32(0.5)).all()
        u = np.array([1.0, 2.0, 3.0, 4.0])
        X = _f32(np.concatenate([u, -u])[None, :])        # the two sub-tokens cancel
        v, mean, rc = oracle.init_v(X, M)
        assert rc == oracle.ERR_DEGENERATE and (v == np.float32(0.5)).all()
        Xn = np.ones((2, M * d), dtype=np.float32)
        Xn[1, 3] = np.inf
        v, _, rc = oracle.init_v(Xn, M)
        assert rc == oracle.ERR_DEGENERATE and (v == np.float32(0.5)).all()


# ------------------------------------------------------------------ per-batch v
class TestUpdateV:
    def test_reduces_to_init_v_without_state_or_with_beta_zero(self):
        X = _rand((50, 96), 3) + np.float32(0.25)
        v0, _, rc0 = oracle.init_v(X, 6)
        v1, st1, rc1 = oracle.update_v(X, 6)
        assert rc0 == rc1 == 0 and st1 is None and (v0 == v1).all()
        state = _f32(np.linspace(-1, 1, 16))
        v2, st2, _ = oracle.update_v(X, 6, state=state, beta=0.0)
        assert (v2 == v0).all()
        _, mean, _ = oracle.init_v(X, 6)
        assert (st2 == mean.astype(np.float32)).all()

    def test_beta_one_keeps_the_state(self):
        X = _rand((20, 32), 4)
        state = _f32([3.0, 0.0, -4.0, 0.0, 0.0, 0.0, 0.0, 0.0])
        v, st, rc = oracle.update_v(X, 4, state=state, beta=1.0)
        assert rc == 0 and (st == state).all()
        np.testing.assert_allclose(v, state / 5.0, rtol=0, atol=1e-7)

    def test_closed_form_on_constant_subtokens(self):
        # every sub-token equals u, state w: m = beta*w + (1-beta)*u exactly (dyadic values)
        u = np.array([1.0, -2.0, 0.5, 4.0])
        w = np.array([-3.0, 2.0, 1.5, 0.0])
        X = _f32(np.tile(u, (7, 3)))
        for beta in (0.25, 0.5, 0.75):
            v, st, rc = oracle.update_v(X, 3, state=_f32(w), beta=beta)
            m = beta * w + (1 - beta) * u
            assert (st == m.astype(np.float32)).all()
            np.testing.assert_allclose(v, m / np.linalg.norm(m), rtol=0, atol=6e-8)

    def test_chain_equals_exponential_average_of_batch_means(self):
        d, M = 8, 4
        batches = [_rand((30, d * M), 10 + i) + np.float32(i) for i in range(4)]
        beta = 0.5
        state = np.zeros(d, dtype=np.float32)
        expect = np.zeros(d)
        for X in batches:
            v, state, _ = oracle.update_v(X, M, state=state, beta=beta)
            mb = X.astype(np.float64).reshape(-1, d).mean(0)
            expect = beta * expect + (1 - beta) * mb
        np.testing.assert_allclose(state, expect, rtol=1e-6, atol=1e-7)
        np.testing.assert_allclose(v, expect / np.linalg.norm(expect), rtol=0, atol=2e-6)

    def test_degenerate(self):
        v, st, rc = oracle.update_v(np.zeros((4, 8), dtype=np.float32), 2, state=np.zeros(4, dtype=np.float32), beta=0.5)
        assert rc == oracle.ERR_DEGENERATE and (v == np.float32(0.5)).all() and (st == 0).all()


# ------------------------------------------------------------------ weight gradient
class TestWeightGrad:
    @pytest.mark.parametrize("N,O,D,d,dtype", [
        (5, 3, 8, 2, wl.F32), (9, 7, 12, 4, wl.F32), (16, 5, 6, 6, wl.BF16),
        (11, 4, 10, 1, wl.BF16), (33, 6, 24, 8, wl.F32),
    ])
    def test_factored_equals_bruteforce(self, N, O, D, d, dtype):
        M = D // d
        G = _rand((N, O), 40 + N, dtype, sigma=0.02)
        S = _rand((N, M), 50 + N, dtype)
        v = wl.random_unit_v(d, N)
        dWb = oracle.weight_grad_bruteforce(G, S, v, D)
        T, dWf = oracle.weight_grad_factored(G, S, v, D)
        np.testing.assert_allclose(dWf, dWb, rtol=1e-12, atol=1e-16)
        rows = [O - 1, 0, O // 2]
        dWr = oracle.weight_grad_bruteforce_rows(G, S, v, D, rows)
        np.testing.assert_allclose(dWr, dWb[rows], rtol=1e-14, atol=1e-18)

    def test_against_python_loops_nonsquare(self):
        # N, O, D all different: a transposed operand or swapped index cannot pass
        N, O, D, d = 4, 3, 6, 3
        M = D // d
        G = _rand((N, O), 3)
        S = _rand((N, M), 4)
        v = wl.random_unit_v(d, 5)
        dW = oracle.weight_grad_bruteforce(G, S, v, D)
        assert dW.shape == (O, D)
        for o in range(O):
            for c in range(D):
                acc = 0.0
                for n in range(N):
                    xhat = float(S[n, c // d]) * float(v[c % d])
                    acc += float(G[n, o]) * xhat
                assert dW[o, c] == pytest.approx(acc, rel=1e-14, abs=1e-300)

    def test_single_one_in_G_copies_a_reconstructed_token(self):
        N, O, D, d = 6, 5, 8, 4
        S = _rand((N, D // d), 9)
        v = wl.random_unit_v(d, 1)
        Xhat = oracle.reconstruct(S, v, D)
        for (n, o) in [(0, 0), (5, 4), (2, 3)]:
            G = np.zeros((N, O), dtype=np.float32)
            G[n, o] = 1.0
            for fn in (oracle.weight_grad_bruteforce,
                       lambda *a: oracle.weight_grad_factored(*a)[1]):
                dW = fn(G, S, v, D)
                assert (dW[o] == Xhat[n]).all()
                mask = np.ones(O, dtype=bool)
                mask[o] = False
                assert (dW[mask] == 0).all()

    def test_no_subtoken_case_is_rank_one(self):
        # Sec. 3.2 "Connection to parameter efficient fine-tuning": with d = D the
        # gradient is (G^T X v) v^T.
        N, O, D = 12, 5, 16
        X = _rand((N, D), 77)
        G = _rand((N, O), 78, sigma=0.02)
        v = wl.random_unit_v(D, 7)
        S_exact, S_store = oracle.compress(X, v, M=1)
        dW = oracle.weight_grad_bruteforce(G, S_store, v, D)
        want = np.outer(G.astype(np.float64).T @ S_store.astype(np.float64)[:, 0], v.astype(np.float64))
        np.testing.assert_allclose(dW, want, rtol=1e-12, atol=1e-18)
        assert np.linalg.matrix_rank(dW) == 1
        # and S itself is X v
        np.testing.assert_allclose(S_exact[:, 0], X.astype(np.float64) @ v.astype(np.float64), rtol=1e-13)

    def test_d_equals_one_is_dense_product(self):
        N, O, D = 10, 4, 7
        X = _rand((N, D), 5)
        G = _rand((N, O), 6)
        one = np.ones(1, dtype=np.float32)
        _, S = oracle.compress(X, one, M=D)
        for dW in (oracle.weight_grad_bruteforce(G, S, one, D), oracle.weight_grad_factored(G, S, one, D)[1]):
            np.testing.assert_allclose(dW, G.astype(np.float64).T @ X.astype(np.float64), rtol=1e-13, atol=1e-16)

    def test_block_structure_and_linearity(self):
        N, O, D, d = 14, 6, 24, 8
        M = D // d
        G1 = _rand((N, O), 1, sigma=0.1)
        G2 = _rand((N, O), 2, sigma=0.1)
        S = _rand((N, M), 3)
        v = wl.random_unit_v(d, 8)
        vd = v.astype(np.float64)
        T, dW = oracle.weight_grad_factored(G1, S, v, D)
        blocks = dW.reshape(O, M, d)
        # every d-wide block of a row is T[o, g] * v, so rank(dW) <= M and
        # projecting the rows back onto v returns T (times |v|^2)
        np.testing.assert_allclose(blocks, T[:, :, None] * vd[None, None, :], rtol=1e-15)
        np.testing.assert_allclose(blocks @ vd, T * float(vd @ vd), rtol=1e-12, atol=1e-18)
        assert np.linalg.matrix_rank(dW) <= M
        np.testing.assert_allclose(T, G1.astype(np.float64).T @ S.astype(np.float64), rtol=1e-12, atol=1e-18)
        G3 = _f32(G1.astype(np.float64) + 2.0 * G2.astype(np.float64))
        dW1 = oracle.weight_grad_bruteforce(G1, S, v, D)
        dW2 = oracle.weight_grad_bruteforce(G2, S, v, D)
        dW3 = oracle.weight_grad_bruteforce(G3, S, v, D)
        np.testing.assert_allclose(dW3, dW1 + 2.0 * dW2, rtol=0, atol=1e-6)

    def test_config1_tiny_bruteforce_vs_factored(self):
        # BASELINE configuration 1: X[256,64] ~ N(0,1) seed 0, M = 4 (d = 16),
        # G ~ N(0, 0.02), v = normalised mean of X's sub-tokens.
        sh = wl.shape_by_name("cfg1_tiny")
        X, G = wl.make_X(sh), wl.make_G(sh)
        v, _, rc = oracle.init_v(X, sh.M)
        assert rc == 0
        _, S = oracle.compress(X, v, sh.M)
        dWb = oracle.weight_grad_bruteforce(G, S, v, sh.D)
        _, dWf = oracle.weight_grad_factored(G, S, v, sh.D)
        np.testing.assert_allclose(dWf, dWb, rtol=1e-11, atol=1e-16)
        # |Xhat| <= |X|
        Xhat = oracle.reconstruct(S, v, sh.D)
        assert np.linalg.norm(Xhat) <= np.linalg.norm(X.astype(np.float64))


class TestLinear:
    @pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
    def test_matches_matmul(self, dtype):
        X = _rand((9, 20), 1, dtype)
        W = _rand((7, 20), 2, dtype)
        Y = oracle.linear(X, W)
        np.testing.assert_allclose(Y, wl.to_f64(X, dtype) @ wl.to_f64(W, dtype).T, rtol=1e-13, atol=1e-15)


class TestLinearCompress:
    """Listing 1's forward as one call: pinned to the library matmul, to a triple loop on a tiny case,
    and to the already pinned compress."""

    def test_triple_loop_and_library(self):
        X = _rand((5, 12), 3, wl.BF16); W = _rand((4, 12), 4, wl.BF16)
        v = wl.random_unit_v(6, 1)
        Y, Ys, S, Ss = oracle.linear_compress(X, W, v, 2)
        Xf, Wf = wl.to_f64(X, wl.BF16), wl.to_f64(W, wl.BF16)
        want = np.zeros((5, 4))
        for n in range(5):
            for o in range(4):
                for c in range(12):
                    want[n, o] += Xf[n, c] * Wf[o, c]
        np.testing.assert_allclose(Y, want, rtol=1e-14, atol=1e-300)
        np.testing.assert_allclose(Y, Xf @ Wf.T, rtol=1e-13, atol=1e-15)
        assert Ys.dtype == np.uint16 and (Ys == wl.f32_to_bf16_bits(Y.astype(np.float32))).all()
        S2, Ss2 = oracle.compress(X, v, 2)
        assert (S == S2).all() and (Ss == Ss2).all()
        # S[n, g] from the definition, by hand
        np.testing.assert_allclose(S[2, 1], float(Xf[2, 6:12] @ v.astype(np.float64)), rtol=1e-14)

    def test_identity_and_transposition(self):
        # W = I gives Y = X; a single 1 at W[o, c] copies column c of X into column o of Y (pins the [O, D] layout)
        X = _rand((7, 8), 5)
        v = wl.random_unit_v(4, 2)
        Y, Ys, _, _ = oracle.linear_compress(X, np.eye(8, dtype=np.float32), v, 2)
        assert (Y == X.astype(np.float64)).all() and (Ys == X).all()
        W = np.zeros((3, 8), dtype=np.float32); W[2, 5] = 1.0
        Y, _, _, _ = oracle.linear_compress(X, W, v, 2)
        assert (Y[:, 2] == X[:, 5]).all() and (Y[:, :2] == 0).all()


class TestGradInput:
    def test_triple_loop_layout_and_adjointness(self):
        G = _rand((5, 4), 6, wl.BF16); W = _rand((4, 12), 7, wl.BF16)
        dX, dXs = oracle.grad_input(G, W)
        Gf, Wf = wl.to_f64(G, wl.BF16), wl.to_f64(W, wl.BF16)
        want = np.zeros((5, 12))
        for n in range(5):
            for c in range(12):
                for o in range(4):
                    want[n, c] += Gf[n, o] * Wf[o, c]
        np.testing.assert_allclose(dX, want, rtol=1e-14, atol=1e-300)
        assert dXs.dtype == np.uint16 and (dXs == wl.f32_to_bf16_bits(dX.astype(np.float32))).all()
        # adjoint of the forward: <G, X W^T> = <G W, X> for any X (the defining property of grad_input)
        X = _rand((5, 12), 8, wl.BF16)
        Y = oracle.linear(X, W)
        np.testing.assert_allclose((Gf * Y).sum(), (dX * wl.to_f64(X, wl.BF16)).sum(), rtol=1e-12)
        # a one-hot grad_output row selects a row of W
        G1 = np.zeros((2, 4), dtype=np.float32); G1[0, 2] = 1.0; G1[1, 0] = 1.0
        W32 = _rand((4, 12), 9)
        d1, _ = oracle.grad_input(G1, W32)
        assert (d1[0] == W32[2]).all() and (d1[1] == W32[0]).all()


# ------------------------------------------------------------------ AdamW on the factored gradient
class TestAdamWFactor:
    """The fused optimiser step of the factored gradient, pinned to the library
    optimiser (torch.optim.AdamW on the CPU, float64, fed the expanded gradient)
    and to closed forms."""

    HYP = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=1e-2)

    def _case(self, O=7, M=3, d=4, seed=0):
        rng = np.random.default_rng(seed)
        T = rng.standard_normal((O, M))
        v = rng.standard_normal(d)
        v /= np.linalg.norm(v)
        W = rng.standard_normal((O, M * d)) * 0.1
        return T, v, W

    def test_matches_library_adamw_over_several_steps(self):
        import torch
        T0, v, W0 = self._case()
        h = self.HYP
        p = torch.nn.Parameter(torch.tensor(W0, dtype=torch.float64))
        opt = torch.optim.AdamW([p], lr=h["lr"], betas=(h["beta1"], h["beta2"]), eps=h["eps"],
                                weight_decay=h["weight_decay"])
        W, m, u = W0, np.zeros_like(W0), np.zeros_like(W0)
        for step in range(1, 6):
            T = T0 * (1.0 + 0.3 * step) * (-1.0) ** step
            # the library is fed the gradient in its plain definition (Listing 1 backward)
            G = np.zeros_like(W0)
            for o in range(T.shape[0]):
                for g in range(T.shape[1]):
                    for j in range(v.size):
                        G[o, g * v.size + j] = 0.5 * T[o, g] * v[j]
            p.grad = torch.tensor(G, dtype=torch.float64)
            opt.step()
            W, m, u = oracle.adamw_step_factor(T, v, W, m, u, step=step, grad_scale=0.5, **h)
            np.testing.assert_allclose(W, p.detach().numpy(), rtol=1e-12, atol=1e-14)
            st = opt.state[p]
            np.testing.assert_allclose(m, st["exp_avg"].numpy(), rtol=1e-12, atol=1e-16)
            np.testing.assert_allclose(u, st["exp_avg_sq"].numpy(), rtol=1e-12, atol=1e-18)

    def test_first_step_moves_by_lr_times_sign(self):
        # m = (1-b1) g, u = (1-b2) g^2 and both bias corrections cancel: step = lr * g / (|g| + eps)
        T, v, W = self._case(seed=1)
        z = np.zeros_like(W)
        W1, m1, u1 = oracle.adamw_step_factor(T, v, W, z, z, lr=1e-2, beta1=0.9, beta2=0.99, eps=0.0,
                                              weight_decay=0.0, step=1)
        g = np.kron(T, v.reshape(1, -1))
        np.testing.assert_allclose(W1, W - 1e-2 * np.sign(g), rtol=0, atol=1e-15)
        np.testing.assert_allclose(m1, 0.1 * g, rtol=1e-13)
        np.testing.assert_allclose(u1, 0.01 * g * g, rtol=1e-12)

    def test_zero_gradient_leaves_only_decoupled_decay(self):
        T, v, W = self._case(seed=2)
        z = np.zeros_like(W)
        W1, m1, u1 = oracle.adamw_step_factor(np.zeros_like(T), v, W, z, z, lr=0.1, beta1=0.9, beta2=0.999,
                                              eps=1e-8, weight_decay=0.5, step=3)
        np.testing.assert_allclose(W1, W * (1 - 0.05), rtol=1e-15)
        assert not m1.any() and not u1.any()

    def test_gradient_layout_is_group_major(self):
        # a single non-zero T[o, g] with v = e_j touches exactly column g*d + j of row o
        O, M, d = 3, 4, 5
        T = np.zeros((O, M)); T[1, 2] = 2.0
        v = np.zeros(d); v[3] = 1.0
        z = np.zeros((O, M * d))
        _, m1, _ = oracle.adamw_step_factor(T, v, z, z, z, lr=1e-3, beta1=0.5, beta2=0.5, eps=1e-8,
                                            weight_decay=0.0, step=1)
        expect = np.zeros((O, M * d)); expect[1, 2 * d + 3] = 1.0
        assert (m1 == expect).all()

    def test_agrees_with_weight_grad_of_the_same_inputs(self):
        # the factor this step consumes is the one weight_grad_factored hands over
        X = _rand((40, 24), 5); Gm = _rand((40, 6), 6, sigma=0.02)
        v, _, _ = oracle.init_v(X, 3)
        S, _ = oracle.compress(X, v, 3)
        T, dW = oracle.weight_grad_factored(Gm, S.astype(np.float32), v, 24)
        z = np.zeros((6, 24))
        _, m1, _ = oracle.adamw_step_factor(T, v, z, z, z, lr=1e-3, beta1=0.0, beta2=0.5, eps=1e-8,
                                            weight_decay=0.0, step=1)
        np.testing.assert_allclose(m1, dW, rtol=1e-12, atol=1e-18)


# ------------------------------------------------------------------ producer-side fusion: silu(gate) * up, then compress
class TestSwigluCompress:
    def test_matches_library_silu_times_up(self):
        import torch
        g = _rand((9, 32), 21, sigma=3.0); u = _rand((9, 32), 22)
        v = oracle.init_v(_rand((9, 32), 23) + np.float32(0.5), 4)[0]
        X, Xs, S, Ss = oracle.swiglu_compress(g, u, v, 4)
        ref = (torch.nn.functional.silu(torch.tensor(g, dtype=torch.float64)) * torch.tensor(u, dtype=torch.float64)).numpy()
        np.testing.assert_allclose(X, ref, rtol=1e-14, atol=1e-300)
        assert Xs.dtype == np.float32 and (Xs == ref.astype(np.float32)).all()

    def test_silu_closed_forms(self):
        x = np.array([[0.0, 1.0, -1.0, 20.0, -20.0, 0.5, -0.5, 3.0]], dtype=np.float32)
        one = np.ones_like(x)
        v = np.zeros(8, dtype=np.float32); v[0] = 1.0
        X, _, _, _ = oracle.swiglu_compress(x, one, v, 1)
        assert X[0, 0] == 0.0
        np.testing.assert_allclose(X[0, 1] - X[0, 2], 1.0, rtol=1e-15)          # silu(x) - silu(-x) = x
        np.testing.assert_allclose(X[0, 5] - X[0, 6], 0.5, rtol=1e-15)
        np.testing.assert_allclose(X[0, 3], 20.0 / (1.0 + np.exp(-20.0)), rtol=1e-15)
        np.testing.assert_allclose(X[0, 1], 1.0 / (1.0 + np.exp(-1.0)), rtol=1e-15)
        assert abs(X[0, 4]) < 1e-7                                              # silu(-20) ~ -4e-8

    def test_compress_is_taken_from_the_stored_activation(self):
        g = wl.to_storage(_rand((6, 16), 31, sigma=2.0), wl.BF16); u = wl.to_storage(_rand((6, 16), 32), wl.BF16)
        v = wl.random_unit_v(8, 5)
        X, Xs, S, Ss = oracle.swiglu_compress(g, u, v, 2)
        assert Xs.dtype == np.uint16
        # the stored activation is the bfloat16 nearest to the exact value ...
        near = wl.f32_to_bf16_bits(X.astype(np.float32))
        assert (Xs == near).all()
        assert np.abs(wl.bf16_bits_to_f32(Xs).astype(np.float64) - X).max() <= np.abs(X).max() * 2.0 ** -8
        # ... and S is what compress gives on exactly those stored bits
        S2, Ss2 = oracle.compress(Xs, v, 2)
        assert (S == S2).all() and (Ss == Ss2).all()


class TestRmsnormCompress:
    def test_matches_library_rms_norm(self):
        import torch
        H = _rand((11, 48), 41, sigma=1.5); gamma = _f32(np.linspace(0.5, 1.5, 48))
        v = wl.random_unit_v(8, 2)
        X, Xs, S, Ss = oracle.rmsnorm_compress(H, gamma, 1e-5, v, 6)
        ref = torch.nn.functional.rms_norm(torch.tensor(H, dtype=torch.float64), (48,),
                                           torch.tensor(gamma, dtype=torch.float64), 1e-5).numpy()
        np.testing.assert_allclose(X, ref, rtol=1e-13, atol=1e-300)
        S2, Ss2 = oracle.compress(Xs, v, 6)
        assert (S == S2).all() and (Ss == Ss2).all()

    def test_closed_forms(self):
        # a constant row c normalises to sign(c) (eps = 0); gamma scales columns; rows are independent
        H = _f32([[3.0] * 8, [-2.0] * 8, [1.0, -1.0] * 4])
        gamma = _f32([1, 2, 3, 4, 5, 6, 7, 8])
        v = _f32([1, 0, 0, 0])
        X, _, S, _ = oracle.rmsnorm_compress(H, gamma, 0.0, v, 2)
        np.testing.assert_allclose(X[0], gamma, rtol=1e-15)
        np.testing.assert_allclose(X[1], -gamma.astype(np.float64), rtol=1e-15)
        np.testing.assert_allclose(X[2], gamma * np.array([1, -1] * 4), rtol=1e-15)
        np.testing.assert_allclose(S[0], [1.0, 5.0], rtol=1e-7)      # v = e_0 picks columns 0 and 4
        # unit RMS before gamma: mean square of X / gamma is 1
        Hr = _rand((5, 64), 43, sigma=4.0)
        Xr, _, _, _ = oracle.rmsnorm_compress(Hr, np.ones(64, dtype=np.float32), 0.0, wl.random_unit_v(16, 1), 4)
        np.testing.assert_allclose((Xr ** 2).mean(axis=1), 1.0, rtol=1e-13)

    def test_eps_matters_only_for_tiny_rows(self):
        H = _f32([[1e-4] * 16])
        v = wl.random_unit_v(16, 1)
        X0, _, _, _ = oracle.rmsnorm_compress(H, np.ones(16, dtype=np.float32), 0.0, v, 1)
        X1, _, _, _ = oracle.rmsnorm_compress(H, np.ones(16, dtype=np.float32), 1e-6, v, 1)
        np.testing.assert_allclose(X0[0], 1.0, rtol=1e-6)
        h = np.float64(np.float32(1e-4))
        np.testing.assert_allclose(X1[0], h / np.sqrt(h * h + 1e-6), rtol=1e-12)
