"""Parity over the paper's own benchmark grid (section "Sparse Matrix Collection": 12 (M, K) pairs x sparsity
70 / 80 / 90 % x N in {32, 128}, D = N) in the mode that produces the throughput figures of the sweep: automatic
kernel choice, unplanned and planned calls.  The paper's matrices are randomized and not available; each point is
the seeded Bernoulli stand-in the sweep uses (`inputs.custom_workload`).

Per point the oracle computes at least 257 output rows - every 61st row (a stride coprime to the 16 / 32 / 48 / 64
rows a workgroup of the tiled kernels owns and to the 4 rows of a wavefront, so every wavefront and row slot of
those layouts is met) plus the first and last four rows - for all three operations; the unplanned and the planned
result are both held to |gpu - oracle| <= 1e-5 * sum|terms| on those rows."""
import numpy as np
import pytest

import oracle
from paper_2311_00368_amd import inputs
from paper_2311_00368_amd.sweep import MK, SPARSITY, WIDTHS

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

REL_TOL = 1e-5
STRIDE = 61
POINTS = [(mk, kk, sp, n) for (mk, kk) in MK for sp in SPARSITY for n in WIDTHS]


@pytest.fixture(scope="module")
def csrk():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2311_00368_amd import binding
    binding.load(build_if_missing=False)
    return binding


def sample_rows(M):
    stride = STRIDE if M >= 257 * STRIDE else max(1, (M // 257) | 1)      # odd: coprime to every power of two
    rows = np.unique(np.concatenate([np.arange(0, M, stride), np.arange(4), np.arange(M - 4, M)])).astype(np.int32)
    assert len(rows) >= 257
    return rows


def check(got, want, abs_sum, what):
    ok, worst = oracle.within_tolerance(got, want, abs_sum, REL_TOL)
    assert ok, f"{what}: worst |err|/sum|terms| = {worst:.3e} (limit {REL_TOL})"


def test_the_grid_has_72_points():
    assert len(POINTS) == 72 and len(set(POINTS)) == 72


@pytest.mark.parametrize("mk,kk,sp,n", POINTS, ids=[f"{m}k-{k}k-{n}-{sp}" for (m, k, sp, n) in POINTS])
def test_grid_point_unplanned_and_planned(csrk, monkeypatch, mk, kk, sp, n):
    for name in ("CSRK_KTILE", "CSRK_ROWS", "CSRK_KSPLIT", "CSRK_KSPLIT_S", "CSRK_WORKERS"):
        monkeypatch.delenv(name, raising=False)       # automatic choice: what the sweep times
    M, K, D, N = mk * 1024, kk * 1024, n, n
    w = inputs.custom_workload(M, K, 1.0 - sp / 100.0, N, D)
    f = w.ops["fusedmm"]
    rows = sample_rows(M)
    dev = lambda a: torch.from_numpy(a).cuda()
    rp, ci, v = dev(w.rowptr), dev(w.colidx), dev(w.vals)
    A, B, C = dev(f["A"]), dev(f["B"]), dev(f["C"])
    plan = csrk.csrk_plan_create(M, K, rp, ci)
    try:
        tag = f"{mk}k/{kk}k/{n}/{sp}%"
        want, a = oracle.spmm(M, K, N, w.rowptr, w.colidx, w.vals, f["C"], rows=rows)
        check(csrk.spmm_csr(M, K, N, rp, ci, v, C).cpu().numpy()[rows], want, a, f"spmm {tag}")
        check(csrk.spmm_csr_plan(plan, N, v, C).cpu().numpy()[rows], want, a, f"planned spmm {tag}")
        want, a = oracle.fusedmm(M, K, D, N, w.rowptr, w.colidx, w.vals, f["A"], f["B"], f["C"], rows=rows)
        check(csrk.fusedmm_csr(M, K, D, N, rp, ci, v, A, B, C).cpu().numpy()[rows], want, a, f"fusedmm {tag}")
        check(csrk.fusedmm_csr_plan(plan, D, N, v, A, B, C).cpu().numpy()[rows], want, a, f"planned fusedmm {tag}")
        want, a = oracle.sddmm(M, K, D, w.rowptr, w.colidx, w.vals, f["A"], f["B"], rows=rows)
        sel = ~np.isnan(want)
        check(csrk.sddmm_csr(M, K, D, rp, ci, v, A, B).cpu().numpy()[sel], want[sel], a[sel], f"sddmm {tag}")
        check(csrk.sddmm_csr_plan(plan, D, v, A, B).cpu().numpy()[sel], want[sel], a[sel], f"planned sddmm {tag}")
        # the library must not touch the index arrays
        assert torch.equal(rp.cpu(), torch.from_numpy(w.rowptr)) and torch.equal(ci.cpu(), torch.from_numpy(w.colidx))
    finally:
        csrk.csrk_plan_destroy(plan)
