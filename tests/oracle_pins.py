"""The pins that tie the CPU oracle to something other than itself.

Each pin is a function that raises AssertionError when the oracle disagrees with what the
paper's definitions (eq. (1)-(3)), the worked example of Fig. 1, or plain mathematics fix.
`test_oracle_pins.py` runs them against the real oracle; `test_oracle_mutants.py` runs them
against deliberately broken builds of the oracle's C source and demands that every planted
mistake is caught.

The dense brute force here is numpy FP64 on the scattered M x K matrix: the same sums with the
zero terms left in, so agreement is expected to ~1e-13 relative to sum|terms|.
"""
import numpy as np

import helpers
import oracle
from paper_2311_00368_amd import inputs

TIGHT = 1e-12     # FP64 oracle vs FP64 brute force, relative to sum|terms|


def _rand_problem(seed, M=37, K=29, D=13, N=11, p=0.3):
    rng = np.random.default_rng(seed)
    dense = (rng.random((M, K)) < p) * rng.uniform(-1, 1, (M, K))
    dense[3, :] = 0.0                       # an empty row
    rowptr, colidx, vals = inputs.csr_from_dense(dense)
    A = rng.normal(size=(M, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    Bn = rng.uniform(-1, 1, (K, N)).astype(np.float32)
    C = rng.normal(size=(K, N)).astype(np.float32)
    return M, K, D, N, rowptr, colidx, vals, A, B, Bn, C


def _close(got, want, scale, tol=TIGHT):
    assert got.shape == want.shape
    assert np.all(np.abs(got - want) <= tol * scale + 1e-300), float(np.max(np.abs(got - want)))


# ------------------------------------------------------------------ worked example
def pin_fig1_hand_results():
    g = helpers.load_golden("fig1_example.txt")
    rp, ci, v = g["ia"].astype(np.int32), g["ja"].astype(np.int32), g["avalue"].astype(np.float32)
    O, _ = oracle.spmm(5, 4, 2, rp, ci, v, g["spmm_B"])
    np.testing.assert_array_equal(O, g["spmm_O"])
    P, _ = oracle.sddmm(5, 4, 2, rp, ci, None, g["sddmm_A"], g["spmm_B"])
    np.testing.assert_array_equal(P, g["sddmm_P_ones"])
    P, _ = oracle.sddmm(5, 4, 2, rp, ci, v, g["sddmm_A"], g["spmm_B"])
    np.testing.assert_array_equal(P, g["sddmm_P_scaled"])
    O, _ = oracle.fusedmm(5, 4, 2, 2, rp, ci, None, g["sddmm_A"], g["spmm_B"], g["fused_C"])
    np.testing.assert_array_equal(O, g["fused_O_ones"])
    O, _ = oracle.fusedmm(5, 4, 2, 2, rp, ci, v, g["sddmm_A"], g["spmm_B"], g["fused_C"])
    np.testing.assert_array_equal(O, g["fused_O_scaled"])


# ------------------------------------------------------------------ dense brute force
def pin_spmm_dense_bruteforce():
    for seed in range(3):
        M, K, D, N, rp, ci, v, A, B, Bn, C = _rand_problem(seed)
        S = inputs.csr_to_dense(M, K, rp, ci, v)
        O, a = oracle.spmm(M, K, N, rp, ci, v, Bn)
        _close(O, S @ Bn.astype(np.float64), np.abs(S) @ np.abs(Bn.astype(np.float64)))
        _close(a, np.abs(S) @ np.abs(Bn.astype(np.float64)), a)


def pin_sddmm_dense_bruteforce():
    for seed in range(3):
        M, K, D, N, rp, ci, v, A, B, Bn, C = _rand_problem(seed)
        A64, B64 = A.astype(np.float64), B.astype(np.float64)
        full = A64 @ B64.T
        fabs = np.abs(A64) @ np.abs(B64).T
        rows = np.repeat(np.arange(M), np.diff(rp))
        P, a = oracle.sddmm(M, K, D, rp, ci, v, A, B)
        _close(P, v.astype(np.float64) * full[rows, ci], np.abs(v) * fabs[rows, ci])
        _close(a, np.abs(v) * fabs[rows, ci], a)
        P1, a1 = oracle.sddmm(M, K, D, rp, ci, None, A, B)      # the paper's all-ones mask
        _close(P1, full[rows, ci], fabs[rows, ci])
        _close(a1, fabs[rows, ci], a1)


def pin_fusedmm_dense_bruteforce():
    for seed in range(3):
        M, K, D, N, rp, ci, v, A, B, Bn, C = _rand_problem(seed)
        A64, B64, C64 = A.astype(np.float64), B.astype(np.float64), C.astype(np.float64)
        S = inputs.csr_to_dense(M, K, rp, ci, v)
        mask = inputs.csr_to_dense(M, K, rp, ci, None)
        scale = (np.abs(S) * (np.abs(A64) @ np.abs(B64).T)) @ np.abs(C64)
        O, a = oracle.fusedmm(M, K, D, N, rp, ci, v, A, B, C)
        _close(O, (S * (A64 @ B64.T)) @ C64, scale)
        _close(a, scale, a)
        O1, a1 = oracle.fusedmm(M, K, D, N, rp, ci, None, A, B, C)
        _close(O1, (mask * (A64 @ B64.T)) @ C64, (mask * (np.abs(A64) @ np.abs(B64).T)) @ np.abs(C64))
        # D != N and D == N both follow the same definition
        O2, _ = oracle.fusedmm(M, K, D, D, rp, ci, v, A, B, B)
        _close(O2, (S * (A64 @ B64.T)) @ B64, (np.abs(S) * (np.abs(A64) @ np.abs(B64).T)) @ np.abs(B64))


# ------------------------------------------------------------------ special cases
def pin_spmm_identity_and_permutation_are_bit_exact():
    rng = np.random.default_rng(5)
    K, N = 23, 9
    B = rng.uniform(-1, 1, (K, N)).astype(np.float32)
    eye_rp = np.arange(K + 1, dtype=np.int32)
    O, a = oracle.spmm(K, K, N, eye_rp, np.arange(K, dtype=np.int32), np.ones(K, np.float32), B)
    np.testing.assert_array_equal(O, B.astype(np.float64))
    np.testing.assert_array_equal(a, np.abs(B).astype(np.float64))
    perm = rng.permutation(K).astype(np.int32)
    O, _ = oracle.spmm(K, K, N, eye_rp, perm, np.ones(K, np.float32), B)
    np.testing.assert_array_equal(O, B[perm].astype(np.float64))
    s = rng.uniform(-2, 2, K).astype(np.float32)               # one entry per row: scaled rows
    O, _ = oracle.spmm(K, K, N, eye_rp, perm, s, B)
    np.testing.assert_array_equal(O, s[:, None].astype(np.float64) * B[perm].astype(np.float64))


def pin_spmm_matches_scipy_sparse():
    import scipy.sparse as sp
    M, K, D, N, rp, ci, v, A, B, Bn, C = _rand_problem(11, M=64, K=80, N=17)
    S = sp.csr_matrix((v.astype(np.float64), ci, rp), shape=(M, K))
    O, a = oracle.spmm(M, K, N, rp, ci, v, Bn)
    _close(O, S @ Bn.astype(np.float64), a)


def pin_sddmm_full_pattern_is_gemm_and_rank_one():
    rng = np.random.default_rng(7)
    M, K, D = 9, 14, 21
    A = rng.normal(size=(M, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    rp = (np.arange(M + 1) * K).astype(np.int32)
    ci = np.tile(np.arange(K, dtype=np.int32), M)
    P, a = oracle.sddmm(M, K, D, rp, ci, None, A, B)
    A64, B64 = A.astype(np.float64), B.astype(np.float64)
    _close(P.reshape(M, K), A64 @ B64.T, np.abs(A64) @ np.abs(B64).T)
    # D = 1: outer product entries, exact
    P, _ = oracle.sddmm(M, K, 1, rp, ci, None, A[:, :1].copy(), B[:, :1].copy())
    np.testing.assert_array_equal(P.reshape(M, K), A64[:, :1] * B64[:, 0][None, :])


def pin_fusedmm_equals_spmm_of_sddmm():
    M, K, D, N, rp, ci, v, A, B, Bn, C = _rand_problem(13)
    O, a = oracle.fusedmm(M, K, D, N, rp, ci, v, A, B, C)
    # all-FP64 composition through the dense form
    P, aP = oracle.sddmm(M, K, D, rp, ci, v, A, B)
    Pd = inputs.csr_to_dense(M, K, rp, ci, P)
    _close(O, Pd @ C.astype(np.float64), a)
    _close(a, inputs.csr_to_dense(M, K, rp, ci, aP) @ np.abs(C.astype(np.float64)), a)
    # FP32-rounded intermediate: differs by at most one FP32 rounding of each score
    O32, _ = oracle.fusedmm_unfused_fp32(M, K, D, N, rp, ci, v, A, B, C)
    assert np.all(np.abs(O32 - O) <= 2.0 ** -23 * a)
    assert np.any(O32 != O)


def pin_full_pattern_fusedmm_is_two_gemms():
    rng = np.random.default_rng(17)
    M, K, D, N = 6, 10, 7, 5
    A = rng.normal(size=(M, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    C = rng.normal(size=(K, N)).astype(np.float32)
    rp = (np.arange(M + 1) * K).astype(np.int32)
    ci = np.tile(np.arange(K, dtype=np.int32), M)
    O, a = oracle.fusedmm(M, K, D, N, rp, ci, None, A, B, C)
    A64, B64, C64 = A.astype(np.float64), B.astype(np.float64), C.astype(np.float64)
    _close(O, (A64 @ B64.T) @ C64, (np.abs(A64) @ np.abs(B64).T) @ np.abs(C64))


# ------------------------------------------------------------------ invariants
def pin_linearity_and_column_split():
    M, K, D, N, rp, ci, v, A, B, Bn, C = _rand_problem(19)
    O, a = oracle.spmm(M, K, N, rp, ci, v, Bn)
    O2, _ = oracle.spmm(M, K, N, rp, ci, (2 * v).astype(np.float32), Bn)
    np.testing.assert_array_equal(O2, 2 * O)                          # power-of-two scale: exact
    Ol, _ = oracle.spmm(M, K, 4, rp, ci, v, np.ascontiguousarray(Bn[:, :4]))
    Or, _ = oracle.spmm(M, K, N - 4, rp, ci, v, np.ascontiguousarray(Bn[:, 4:]))
    np.testing.assert_array_equal(np.hstack([Ol, Or]), O)
    F, fa = oracle.fusedmm(M, K, D, N, rp, ci, v, A, B, C)
    F2, _ = oracle.fusedmm(M, K, D, N, rp, ci, v, (4 * A).astype(np.float32), B, C)
    np.testing.assert_array_equal(F2, 4 * F)
    F3, _ = oracle.fusedmm(M, K, D, N, rp, ci, v, A, B, (-0.5 * C).astype(np.float32))
    np.testing.assert_array_equal(F3, -0.5 * F)
    assert np.all(a >= np.abs(O)) and np.all(fa >= np.abs(F) * (1 - 1e-15))


def pin_stored_order_and_duplicates():
    rng = np.random.default_rng(23)
    M, K, D, N, rp, ci, v, A, B, Bn, C = _rand_problem(23)
    ci2, v2 = ci.copy(), v.copy()
    for i in range(M):                                              # shuffle inside every row
        lo, hi = rp[i], rp[i + 1]
        perm = rng.permutation(hi - lo)
        ci2[lo:hi], v2[lo:hi] = ci[lo:hi][perm], v[lo:hi][perm]
    O, a = oracle.spmm(M, K, N, rp, ci, v, Bn)
    O2, _ = oracle.spmm(M, K, N, rp, ci2, v2, Bn)
    _close(O2, O, a)
    F, fa = oracle.fusedmm(M, K, D, N, rp, ci, v, A, B, C)
    F2, _ = oracle.fusedmm(M, K, D, N, rp, ci2, v2, A, B, C)
    _close(F2, F, fa)
    P, _ = oracle.sddmm(M, K, D, rp, ci, v, A, B)
    P2, _ = oracle.sddmm(M, K, D, rp, ci2, v2, A, B)
    for i in range(M):                                              # one value per stored entry
        lo, hi = rp[i], rp[i + 1]
        np.testing.assert_array_equal(np.sort(P2[lo:hi]), np.sort(P[lo:hi]))
    # duplicated entries: SPMM sums them, SDDMM keeps one result per stored entry
    rp_d, ci_d = helpers.csr_from_rows([[2, 2, 5], [], [0, 0, 0]], 8)
    v_d = np.array([1, 2, 3, 4, 5, 6], np.float32)
    Bd = rng.uniform(-1, 1, (8, 3)).astype(np.float32)
    Od, _ = oracle.spmm(3, 8, 3, rp_d, ci_d, v_d, Bd)
    B64 = Bd.astype(np.float64)
    want = np.stack([3.0 * B64[2] + 3.0 * B64[5], np.zeros(3), 15.0 * B64[0]])
    _close(Od, want, np.abs(want) + 1)
    Ad = rng.normal(size=(3, 4)).astype(np.float32)
    Bd4 = rng.normal(size=(8, 4)).astype(np.float32)
    Pd, _ = oracle.sddmm(3, 8, 4, rp_d, ci_d, v_d, Ad, Bd4)
    assert Pd.shape == (6,) and abs(Pd[1] - 2 * Pd[0]) < 1e-12 and abs(Pd[5] * 4 - Pd[3] * 6) < 1e-12


def pin_empty_rows_and_row_subsets():
    rng = np.random.default_rng(29)
    for name, M, K, rp, ci in helpers.edge_patterns(rng):
        v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
        A = rng.normal(size=(M, 5)).astype(np.float32)
        B = rng.normal(size=(K, 5)).astype(np.float32)
        C = rng.normal(size=(K, 6)).astype(np.float32)
        S = inputs.csr_to_dense(M, K, rp, ci, v)
        O, a = oracle.spmm(M, K, 6, rp, ci, v, C)
        _close(O, S @ C.astype(np.float64), np.abs(S) @ np.abs(C.astype(np.float64)) + 1e-30)
        empty = np.diff(rp) == 0
        assert np.all(O[empty] == 0) and np.all(a[empty] == 0), name
        F, fa = oracle.fusedmm(M, K, 5, 6, rp, ci, v, A, B, C)
        assert np.all(F[empty] == 0), name
        P, pa = oracle.sddmm(M, K, 5, rp, ci, v, A, B)
        Pd = np.zeros((M, K))
        np.add.at(Pd, (np.repeat(np.arange(M), np.diff(rp)), ci), P)
        _close(F, Pd @ C.astype(np.float64), fa + 1e-30)
        rows = np.array(sorted(set(rng.integers(0, M, size=5).tolist())), dtype=np.int32)
        Os, as_ = oracle.spmm(M, K, 6, rp, ci, v, C, rows=rows)
        np.testing.assert_array_equal(Os, O[rows])
        np.testing.assert_array_equal(as_, a[rows])
        Fs, _ = oracle.fusedmm(M, K, 5, 6, rp, ci, v, A, B, C, rows=rows)
        np.testing.assert_array_equal(Fs, F[rows])
        Ps, _ = oracle.sddmm(M, K, 5, rp, ci, v, A, B, rows=rows)
        for i in range(M):
            seg = slice(rp[i], rp[i + 1])
            if i in rows:
                np.testing.assert_array_equal(Ps[seg], P[seg])
            else:
                assert np.all(np.isnan(Ps[seg]))


def pin_fp64_accumulation():
    # 1 + 2^-30 * 2^10 terms: FP32 accumulation would lose every small term, FP64 keeps them
    n = 1024
    rp, ci = helpers.csr_from_rows([list(range(n + 1))], n + 1)
    v = np.ones(n + 1, np.float32)
    B = np.full((n + 1, 1), 2.0 ** -30, np.float32)
    B[0, 0] = 1.0
    O, _ = oracle.spmm(1, n + 1, 1, rp, ci, v, B)
    assert O[0, 0] == 1.0 + n * 2.0 ** -30
    A = np.ones((1, n + 1), np.float32)
    Bt = B.reshape(1, n + 1).copy()
    rp1, ci1 = helpers.csr_from_rows([[0]], 1)
    P, _ = oracle.sddmm(1, 1, n + 1, rp1, ci1, None, A, Bt)
    assert P[0] == 1.0 + n * 2.0 ** -30


def pin_tolerance_rule():
    want = np.array([1.0, -2.0, 0.0])
    a = np.array([4.0, 2.0, 0.0])
    assert oracle.within_tolerance(want + np.array([3.9e-5, -1.9e-5, 0.0]), want, a)[0]
    assert not oracle.within_tolerance(want + np.array([4.1e-5, 0.0, 0.0]), want, a)[0]
    assert not oracle.within_tolerance(want + np.array([0.0, 0.0, 1e-30]), want, a)[0]
    assert not oracle.within_tolerance(np.array([1.0, np.nan, 0.0]), want, a)[0]


PINS = [v for k, v in sorted(globals().items()) if k.startswith("pin_")]
