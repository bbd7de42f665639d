"""Planned calls (`csrk_plan_create` + `*_csr_plan`) against the CPU oracle, to the same bar as the
unplanned ones: the pattern is analysed once on the host side of the plan, and a planned call
launches only the kernel that does the work.  Covered: every kernel family a plan can choose
(whole rows, LDS-tiled wide / narrow / SDDMM, K-split for small M, general equal shares), patterns
the tiled kernels must not be given (unsorted, duplicated columns, skewed rows), edge patterns,
one plan used for several widths and operations, and what plan creation reports and refuses."""

import numpy as np
import pytest

import helpers
import oracle
from paper_2311_00368_amd import inputs
from test_gpu_parity import check, csrk, dev  # noqa: F401  (csrk is a fixture)
from test_gpu_random import CASES_PER_SEED, random_case

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


class Planned:
    """One pattern on the device with its plan; runs the three operations and checks them."""

    def __init__(self, csrk, M, K, rp, ci):
        self.csrk, self.M, self.K, self.rp, self.ci = csrk, M, K, rp, ci
        self.d_rp, self.d_ci = dev(rp), dev(ci)
        self.plan = csrk.csrk_plan_create(M, K, self.d_rp, self.d_ci)

    def close(self):
        self.csrk.csrk_plan_destroy(self.plan)
        np.testing.assert_array_equal(self.d_rp.cpu().numpy(), self.rp)
        np.testing.assert_array_equal(self.d_ci.cpu().numpy(), self.ci)

    def spmm(self, N, v, B):
        O = self.csrk.spmm_csr_plan(self.plan, N, dev(v), dev(B))
        torch.cuda.synchronize()
        want, a = oracle.spmm(self.M, self.K, N, self.rp, self.ci, v, B)
        check(O.cpu().numpy(), want, a, f"planned spmm M={self.M} K={self.K} N={N}")

    def sddmm(self, D, v, A, B):
        P = self.csrk.sddmm_csr_plan(self.plan, D, dev(v), dev(A), dev(B))
        torch.cuda.synchronize()
        want, a = oracle.sddmm(self.M, self.K, D, self.rp, self.ci, v, A, B)
        check(P.cpu().numpy(), want, a, f"planned sddmm M={self.M} K={self.K} D={D}")

    def fused(self, D, N, v, A, B, C):
        O = self.csrk.fusedmm_csr_plan(self.plan, D, N, dev(v), dev(A), dev(B), dev(C))
        torch.cuda.synchronize()
        want, a = oracle.fusedmm(self.M, self.K, D, N, self.rp, self.ci, v, A, B, C)
        check(O.cpu().numpy(), want, a, f"planned fusedmm M={self.M} K={self.K} D={D} N={N}")

    def sampled(self, rows, D, N, v, A, B, C, B_spmm):
        """All three operations, the oracle on the output rows in `rows` only (rows are independent)."""
        d_v = dev(v)
        O = self.csrk.spmm_csr_plan(self.plan, N, d_v, dev(B_spmm))
        want, a = oracle.spmm(self.M, self.K, N, self.rp, self.ci, v, B_spmm, rows=rows)
        check(O.cpu().numpy()[rows], want, a, f"planned spmm M={self.M} N={N}, {len(rows)} rows")
        O = self.csrk.fusedmm_csr_plan(self.plan, D, N, d_v, dev(A), dev(B), dev(C))
        want, a = oracle.fusedmm(self.M, self.K, D, N, self.rp, self.ci, v, A, B, C, rows=rows)
        check(O.cpu().numpy()[rows], want, a, f"planned fusedmm M={self.M} D={D} N={N}, {len(rows)} rows")
        P = self.csrk.sddmm_csr_plan(self.plan, D, d_v, dev(A), dev(B))
        want, a = oracle.sddmm(self.M, self.K, D, self.rp, self.ci, v, A, B, rows=rows)
        sel = ~np.isnan(want)
        check(P.cpu().numpy()[sel], want[sel], a[sel], f"planned sddmm M={self.M} D={D}, {len(rows)} rows")

    def all_ops(self, rng, D, N, ones=False):
        nnz = len(self.ci)
        v = None if ones else rng.uniform(-1, 1, nnz).astype(np.float32)
        A = rng.normal(size=(self.M, D)).astype(np.float32)
        B = rng.normal(size=(self.K, D)).astype(np.float32)
        C = rng.normal(size=(self.K, N)).astype(np.float32)
        self.spmm(N, np.ones(nnz, dtype=np.float32) if ones else v, C)
        self.sddmm(D, v, A, B)
        self.fused(D, N, v, A, B, C)


@pytest.fixture
def env(monkeypatch):
    def setter(**kv):
        for k, val in kv.items():
            if val is None:
                monkeypatch.delenv(k, raising=False)
            else:
                monkeypatch.setenv(k, str(val))
    return setter


# (M, K, density, D, N): small S (whole rows), mid sizes that take the tiled kernels on their own, ragged widths
AUTO_SHAPES = [(512, 512, 0.1, 64, 64), (1024, 1024, 0.3, 32, 128), (4096, 4096, 0.3, 128, 128),
               (4096, 4096, 0.1, 64, 256), (8192, 2048, 0.2, 32, 32), (3000, 5000, 0.25, 60, 500),
               (2048, 8192, 0.2, 64, 512), (700, 900, 0.2, 7, 13),
               # small dense S with 12+ rows per CU: planned calls take the narrow tiled kernels here
               (3072, 1024, 0.3, 128, 128), (4096, 1024, 0.2, 32, 32), (4100, 1000, 0.3, 64, 100)]


@pytest.mark.parametrize("shape", AUTO_SHAPES)
def test_planned_calls_with_automatic_kernel_choice(csrk, shape):
    M, K, p, D, N = shape
    rng = np.random.default_rng(M + K + N)
    rp, ci = inputs.bernoulli_csr(M % 97, M, K, p)
    pl = Planned(csrk, M, K, rp, ci)
    nnz, srt, even = csrk.csrk_plan_info(pl.plan)
    assert (nnz, srt, even) == (len(ci), True, True)
    pl.all_ops(rng, D, N)
    pl.close()


@pytest.mark.parametrize("shape", [(64, 64, 1.0, 64, 256), (333, 417, 0.3, 4, 4), (1000, 1300, 0.05, 32, 260),
                                   (65, 3000, 0.3, 100, 128), (2048, 2048, 0.3, 64, 512), (130, 70, 1.0, 60, 500),
                                   (100, 4000, 0.3, 128, 32), (48, 6000, 0.5, 64, 512)])
def test_planned_calls_with_tiled_kernels_forced(csrk, env, shape):
    # CSRK_KTILE=2: tiled kernels wherever they can run, so small, ragged and small-M (K-split) cases reach them
    M, K, p, D, N = shape
    env(CSRK_KTILE=2, CSRK_ROWS=3)
    rng = np.random.default_rng(M * 3 + K + N)
    rp, ci = inputs.bernoulli_csr(M % 89, M, K, p)
    pl = Planned(csrk, M, K, rp, ci)
    pl.all_ops(rng, D, N)
    pl.all_ops(rng, D, N, ones=True)
    pl.close()


def test_planned_calls_with_very_many_short_rows(csrk):
    M, K = 300_000, 64
    rng = np.random.default_rng(5)
    rp, ci = inputs.bernoulli_csr(1, M, K, 0.1)
    pl = Planned(csrk, M, K, rp, ci)
    pl.all_ops(rng, 16, 32)
    pl.all_ops(rng, 64, 128)
    pl.close()


def test_planned_calls_at_the_benchmark_size_every_row(csrk):
    # the 16384 x 16384 workload the benchmark times, planned: every output row and every stored entry
    w = inputs.workload("large16k")
    pl = Planned(csrk, w.M, w.K, w.rowptr, w.colidx)
    assert csrk.csrk_plan_info(pl.plan) == (len(w.colidx), True, True)
    f = w.ops["fusedmm"]
    pl.spmm(512, w.vals, w.ops["spmm"]["B"])
    pl.fused(64, 512, w.vals, f["A"], f["B"], f["C"])
    pl.sddmm(64, w.vals, f["A"], f["B"])
    pl.close()


def test_one_plan_serves_many_widths_and_repeated_calls(csrk):
    M, K = 4096, 4096
    rng = np.random.default_rng(11)
    rp, ci = inputs.bernoulli_csr(5, M, K, 0.2)
    pl = Planned(csrk, M, K, rp, ci)
    for D, N in [(64, 512), (32, 32), (128, 128), (16, 260), (64, 512)]:
        pl.all_ops(rng, D, N)
    pl.close()


def test_plans_keep_unsuitable_patterns_away_from_the_tiled_kernels(csrk, env):
    rng = np.random.default_rng(3)
    M, K = 2048, 2048
    rp, ci = inputs.bernoulli_csr(9, M, K, 0.3)
    # unsorted: one row written backwards; duplicates: one column repeated; skewed: log-normal row lengths
    ci_uns = ci.copy()
    ci_uns[rp[700]:rp[701]] = ci_uns[rp[700]:rp[701]][::-1]
    ci_dup = ci.copy()
    ci_dup[rp[5] + 1] = ci_dup[rp[5]]
    cases = [("unsorted", rp, ci_uns, False, True), ("duplicates", rp, ci_dup, False, True)]
    rp_s, ci_s = inputs.lognormal_csr(4, M, K, 200.0, 1.2)
    cases.append(("skewed", rp_s, ci_s, True, False))
    for force in (None, 2):
        env(CSRK_KTILE=force)
        for name, r, c, srt, even in cases:
            pl = Planned(csrk, M, K, r, c)
            assert csrk.csrk_plan_info(pl.plan)[1:] == (srt, even), name
            pl.all_ops(rng, 64, 256)
            pl.all_ops(rng, 32, 64)
            pl.close()


def test_planned_calls_on_edge_patterns(csrk, env):
    rng = np.random.default_rng(17)
    for force in (None, 2):
        env(CSRK_KTILE=force)
        for name, M, K, rp, ci in helpers.edge_patterns(rng):
            pl = Planned(csrk, M, K, rp, ci)
            pl.all_ops(rng, 8, 12)
            pl.all_ops(rng, 64, 256)
            pl.close()


def test_planned_results_equal_unplanned_bit_for_bit_where_the_same_kernel_runs(csrk):
    # dense even pattern, no K-split: both ways run the same tiled kernel on the same data
    M, K, N, D = 4096, 2048, 512, 64
    rng = np.random.default_rng(23)
    rp, ci = inputs.bernoulli_csr(2, M, K, 0.25)
    v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
    A, B = (rng.normal(size=(n, D)).astype(np.float32) for n in (M, K))
    C = rng.normal(size=(K, N)).astype(np.float32)
    d_rp, d_ci, d_v, d_A, d_B, d_C = (dev(x) for x in (rp, ci, v, A, B, C))
    plan = csrk.csrk_plan_create(M, K, d_rp, d_ci)
    for _ in range(2):
        assert torch.equal(csrk.spmm_csr_plan(plan, N, d_v, d_C), csrk.spmm_csr(M, K, N, d_rp, d_ci, d_v, d_C))
        assert torch.equal(csrk.sddmm_csr_plan(plan, D, d_v, d_A, d_B), csrk.sddmm_csr(M, K, D, d_rp, d_ci, d_v, d_A, d_B))
        assert torch.equal(csrk.fusedmm_csr_plan(plan, D, N, d_v, d_A, d_B, d_C),
                           csrk.fusedmm_csr(M, K, D, N, d_rp, d_ci, d_v, d_A, d_B, d_C))
    csrk.csrk_plan_destroy(plan)


def test_plan_creation_refuses_broken_patterns_and_empty_ones_work(csrk):
    rp = np.array([0, 2, 1, 3], dtype=np.int32)
    ci = np.array([0, 1, 2], dtype=np.int32)
    with pytest.raises(csrk.CsrkError):
        csrk.csrk_plan_create(3, 4, dev(rp), dev(ci))
    rp = np.array([0, 1, 2, 3], dtype=np.int32)
    with pytest.raises(csrk.CsrkError):
        csrk.csrk_plan_create(3, 2, dev(rp), dev(ci))      # column 2 outside [0, 2)
    # no stored entries at all
    M, K, N = 5, 7, 8
    d_rp = dev(np.zeros(M + 1, dtype=np.int32))
    d_ci = torch.empty(0, dtype=torch.int32, device="cuda")
    plan = csrk.csrk_plan_create(M, K, d_rp, d_ci)
    assert csrk.csrk_plan_info(plan) == (0, True, True)
    O = csrk.spmm_csr_plan(plan, N, None, torch.ones(K, N, device="cuda"))
    assert torch.count_nonzero(O).item() == 0
    csrk.csrk_plan_destroy(plan)
    csrk.csrk_plan_destroy(plan)        # a second destroy of the wrapper is a no-op


@pytest.mark.parametrize("seed", [201, 202])
def test_planned_calls_on_random_shapes(csrk, monkeypatch, seed):
    # the randomised run of test_gpu_random.py (shapes, widths, densities, row-length mixes, kernel-family
    # settings) through plans
    for c in range(CASES_PER_SEED):
        what, env_vars, (M, K, D, N), (rp, ci, v), (A, B, C) = random_case(seed, c)
        for name, value in env_vars.items():
            monkeypatch.setenv(name, value)
        pl = Planned(csrk, M, K, rp, ci)
        try:
            pl.spmm(N, v, C)
            pl.fused(D, N, v, A, B, C)
            if len(ci):
                pl.sddmm(D, v, A, B)
        except AssertionError as e:
            raise AssertionError(f"{what}: {e}") from e
        pl.close()
