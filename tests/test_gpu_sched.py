"""Planned calls on UNEVEN rows: the schedule that csrk_plan_create makes for patterns whose columns are ordered but
whose rows differ widely in length (rows sorted by length into blocks, every block's K cut into as many ranges as its
share of the work asks for, the LDS-tiled kernels run over that table, partial rows of cut blocks added up in range
order).  Every row of every output is compared with the CPU oracle, for every kernel family the schedule can launch
(narrow and wide SPMM / FusedMM), with rows of every length from empty to K,
on the library's own scratch, on a plan's reserved workspace, and twice in a row (same bits)."""

import numpy as np
import pytest

import helpers
import oracle
from paper_2311_00368_amd import inputs
from test_gpu_parity import check, csrk, dev  # noqa: F401  (csrk is a fixture)
from test_gpu_plan import Planned, env  # noqa: F401  (env is a fixture)

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def skewed_pattern(seed, M, K, mean, sigma=1.0, full_rows=0, empty_rows=0):
    """Log-normal row lengths, some rows replaced by full rows (every column) and by empty rows."""
    rp, ci = inputs.lognormal_csr(seed, M, K, mean, sigma)
    rows = [ci[rp[i]:rp[i + 1]] for i in range(M)]
    rng = np.random.default_rng(seed)
    pick = rng.permutation(M)
    for i in pick[:full_rows]:
        rows[i] = np.arange(K, dtype=np.int32)
    for i in pick[full_rows:full_rows + empty_rows]:
        rows[i] = np.zeros(0, dtype=np.int32)
    lens = np.array([len(r) for r in rows], dtype=np.int64)
    rp2 = np.zeros(M + 1, dtype=np.int32)
    rp2[1:] = np.cumsum(lens)
    return rp2, np.concatenate(rows).astype(np.int32)


@pytest.mark.parametrize("N,D", [(32, 32), (64, 64), (128, 64), (256, 32), (512, 64), (96, 20), (384, 64)])
def test_scheduled_calls_match_the_oracle_on_every_row(csrk, env, N, D):
    if N <= 128:
        env(CSRK_KTILE="2")     # outputs this narrow take the schedule only where the tiled kernels are forced
    M, K = 2048 + 37, 4096
    rp, ci = skewed_pattern(11 + N, M, K, 0.08 * K, full_rows=40, empty_rows=25)
    lens = np.diff(rp)
    assert lens.max() == K and lens.min() == 0 and lens.max() > 2 * lens.mean() + 64
    p = Planned(csrk, M, K, rp, ci)
    nnz, sorted_, even = csrk.csrk_plan_info(p.plan)
    assert sorted_ and not even
    rng = np.random.default_rng(N * 7 + D)
    v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
    A = rng.normal(size=(M, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    C = rng.normal(size=(K, N)).astype(np.float32)
    p.spmm(N, v, C)
    p.fused(D, N, v, A, B, C)
    # the schedule is what ran: with it switched off the same plan takes other kernels, whose sums round differently
    with_schedule = csrk.spmm_csr_plan(p.plan, N, dev(v), dev(C)).cpu().numpy()
    env(CSRK_SCHED="2")
    without = csrk.spmm_csr_plan(p.plan, N, dev(v), dev(C)).cpu().numpy()
    assert not np.array_equal(with_schedule, without)
    np.testing.assert_allclose(with_schedule, without, rtol=0, atol=1e-3 * float(np.abs(without).max()))
    p.close()


@pytest.mark.parametrize("N", [64, 320])
def test_scheduled_calls_without_values_and_on_a_tail_of_k(csrk, env, N):
    # vals = NULL (all ones) and a K that is no multiple of any tile height; few rows: the tiled kernels are forced
    env(CSRK_KTILE="2")
    M, K, D = 1500, 3001, 64
    rp, ci = skewed_pattern(5, M, K, 0.1 * K, full_rows=20, empty_rows=10)
    p = Planned(csrk, M, K, rp, ci)
    rng = np.random.default_rng(3)
    A = rng.normal(size=(M, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    C = rng.normal(size=(K, N)).astype(np.float32)
    O = csrk.spmm_csr_plan(p.plan, N, None, dev(C))
    want, a = oracle.spmm(M, K, N, rp, ci, np.ones(len(ci), dtype=np.float32), C)
    check(O.cpu().numpy(), want, a, "scheduled spmm, vals = NULL")
    O = csrk.fusedmm_csr_plan(p.plan, D, N, None, dev(A), dev(B), dev(C))
    want, a = oracle.fusedmm(M, K, D, N, rp, ci, None, A, B, C)
    check(O.cpu().numpy(), want, a, "scheduled fusedmm, vals = NULL")
    p.close()


def test_scheduled_calls_on_a_reserved_workspace_repeat_bit_for_bit(csrk):
    w = inputs.workload("fused8k_skew", scale=0.5)
    M, K = w.M, w.K
    f = dict(w.ops["fusedmm"])
    f["N"] = 256                        # wide enough for the schedule under automatic choice
    f["C"] = np.random.default_rng(8).normal(size=(K, 256)).astype(np.float32)
    p = Planned(csrk, M, K, w.rowptr, w.colidx)
    d_v, d_A, d_B, d_C = dev(w.vals), dev(f["A"]), dev(f["B"]), dev(f["C"])
    first = csrk.fusedmm_csr_plan(p.plan, f["D"], f["N"], d_v, d_A, d_B, d_C).cpu().numpy()
    want, a = oracle.fusedmm(M, K, f["D"], f["N"], w.rowptr, w.colidx, w.vals, f["A"], f["B"], f["C"])
    check(first, want, a, "scheduled fusedmm, library scratch")
    csrk.csrk_plan_reserve(p.plan, 256)
    for _ in range(2):
        again = csrk.fusedmm_csr_plan(p.plan, f["D"], f["N"], d_v, d_A, d_B, d_C).cpu().numpy()
        np.testing.assert_array_equal(again, first)
    p.close()


def test_skewed_8192_square_with_512_columns_planned(csrk):
    w = inputs.workload("fused8k_skew")
    f = dict(w.ops["fusedmm"])
    f["N"] = 512
    f["C"] = np.random.default_rng(9).normal(size=(w.K, 512)).astype(np.float32)
    p = Planned(csrk, w.M, w.K, w.rowptr, w.colidx)
    O = csrk.fusedmm_csr_plan(p.plan, f["D"], f["N"], dev(w.vals), dev(f["A"]), dev(f["B"]), dev(f["C"]))
    rows = np.arange(0, w.M, 7)
    want, a = oracle.fusedmm(w.M, w.K, f["D"], f["N"], w.rowptr, w.colidx, w.vals, f["A"], f["B"], f["C"], rows=rows)
    check(O.cpu().numpy()[rows], want, a, "skewed 8192^2, N = 512, planned, every 7th row")
    p.close()


@pytest.mark.parametrize("N", [256, 512])
def test_unplanned_calls_on_uneven_rows_with_wide_outputs(csrk, N):
    # Without a plan, outputs of more than 128 columns take the tiled kernels on moderately uneven rows as well
    # (longest row up to 16 mean rows); beyond that the equal-share kernels.  Both against the oracle, every row.
    M, K, D = 4096 + 11, 4096, 64
    rng = np.random.default_rng(N)
    A = rng.normal(size=(M, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    C = rng.normal(size=(K, N)).astype(np.float32)
    for name, (rp, ci) in {
        "longest row about 10 mean rows": inputs.lognormal_csr(21, M, K, 0.1 * K, 1.0),
        "a few full rows among short ones": skewed_pattern(22, M, K, 0.03 * K, sigma=0.5, full_rows=12, empty_rows=5),
    }.items():
        lens = np.diff(rp)
        assert lens.max() > 2 * lens.mean() + 64
        v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
        d_rp, d_ci, d_v = dev(rp), dev(ci), dev(v)
        O = csrk.spmm_csr(M, K, N, d_rp, d_ci, d_v, dev(C))
        want, a = oracle.spmm(M, K, N, rp, ci, v, C)
        check(O.cpu().numpy(), want, a, f"unplanned spmm N={N}, {name}")
        O = csrk.fusedmm_csr(M, K, D, N, d_rp, d_ci, d_v, dev(A), dev(B), dev(C))
        want, a = oracle.fusedmm(M, K, D, N, rp, ci, v, A, B, C)
        check(O.cpu().numpy(), want, a, f"unplanned fusedmm N={N}, {name}")


@pytest.mark.parametrize("N", [64, 256])
def test_scheduled_calls_on_adversarial_patterns(csrk, env, N):
    # The degenerate cases of the row loop (empty rows in front, at the end and in runs; rows of length one; one row
    # that holds every column among empty ones; lengths around the 64-entry chunks), each padded with empty rows to
    # the 256 rows a schedule is made from, and one pattern in which a single row holds most of the entries.
    env(CSRK_KTILE="2")
    rng = np.random.default_rng(17)
    K, D = 1024, 32
    A0 = rng.normal(size=(4096, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    C = rng.normal(size=(K, N)).astype(np.float32)
    full = list(range(K))
    lens = [0, 1, 63, 64, 65, 127, 128, 129, 255, 256, 257, 1000]
    cases = {
        "one full row among empty ones": [[]] * 100 + [full] + [[]] * 199,
        "empty first and last, rows of length one and two long rows between":
            [[]] * 3 + [[int(rng.integers(K))] for _ in range(150)] + [full[:500], full[300:]] + [[int(rng.integers(K))] for _ in range(150)] + [[]] * 3,
        "ragged lengths": [sorted(rng.permutation(K)[:n].tolist()) for n in lens] * 22,
        "one row with most of the entries": [sorted(rng.permutation(K)[:int(rng.integers(0, 6))].tolist()) for _ in range(299)] + [full],
    }
    for name, rows in cases.items():
        M = len(rows)
        rp, ci = helpers.csr_from_rows(rows, K)
        lens_ = np.diff(rp)
        assert M >= 256 and lens_.max() > 2 * lens_.mean() + 64, name
        p = Planned(csrk, M, K, rp, ci)
        _, sorted_, even = csrk.csrk_plan_info(p.plan)
        assert sorted_ and not even, name
        v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
        p.spmm(N, v, C)
        p.fused(D, N, v, A0[:M], B, C)
        p.close()
