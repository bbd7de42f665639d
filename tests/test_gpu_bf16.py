"""The bfloat16-operand entry points against the CPU oracle.

The dense operands are rounded to bfloat16 by the input generator; the kernels widen them exactly and compute
in FP32, so the expected result is the oracle's (FP64) on the widened operands and the bar is the FP32 one:
|gpu - oracle| <= 1e-5 * sum|terms| per output entry."""
import numpy as np
import pytest

import helpers
import oracle
from paper_2311_00368_amd import inputs
from test_gpu_parity import check, csrk, dev  # noqa: F401  (csrk is a fixture)

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def dev_bf16(a):
    bits, widened = inputs.to_bf16(a)
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16), widened


def run_all(csrk, M, K, D, N, rp, ci, v, A, B, C, rows=None):
    dA, wA = dev_bf16(A)
    dB, wB = dev_bf16(B)
    dC, wC = dev_bf16(C)
    d_rp, d_ci, d_v = dev(rp), dev(ci), dev(v)
    O = csrk.spmm_csr_bf16(M, K, N, d_rp, d_ci, d_v, dC)
    torch.cuda.synchronize()
    want, a = oracle.spmm(M, K, N, rp, ci, v, wC, rows=rows)
    got = O.cpu().numpy()
    check(got if rows is None else got[rows], want, a, f"spmm_bf16 M={M} K={K} N={N}")
    if len(ci):
        P = csrk.sddmm_csr_bf16(M, K, D, d_rp, d_ci, d_v, dA, dB)
        torch.cuda.synchronize()
        want, a = oracle.sddmm(M, K, D, rp, ci, v, wA, wB, rows=rows)
        got = P.cpu().numpy()
        if rows is not None:
            sel = ~np.isnan(want)
            got, want, a = got[sel], want[sel], a[sel]
        check(got, want, a, f"sddmm_bf16 M={M} K={K} D={D}")
    O = csrk.fusedmm_csr_bf16(M, K, D, N, d_rp, d_ci, d_v, dA, dB, dC)
    torch.cuda.synchronize()
    want, a = oracle.fusedmm(M, K, D, N, rp, ci, v, wA, wB, wC, rows=rows)
    got = O.cpu().numpy()
    check(got if rows is None else got[rows], want, a, f"fusedmm_bf16 M={M} K={K} D={D} N={N}")
    np.testing.assert_array_equal(d_rp.cpu().numpy(), rp)
    np.testing.assert_array_equal(d_ci.cpu().numpy(), ci)


@pytest.mark.parametrize("M,K,D,N", [(1, 1, 8, 8), (70, 300, 16, 64), (333, 417, 64, 128), (1000, 129, 128, 256),
                                     (257, 700, 64, 512), (130, 70, 60, 500), (100, 257, 3, 5), (64, 640, 72, 104),
                                     (500, 500, 256, 1024), (90, 2000, 136, 40)])
@pytest.mark.parametrize("p", [0.05, 0.3])
def test_bf16_widths_ragged(csrk, M, K, D, N, p):
    rng = np.random.default_rng(M + K + D + N)
    rp, ci = inputs.bernoulli_csr(D + N, M, K, p)
    v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
    A = rng.normal(size=(M, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    C = rng.normal(size=(K, N)).astype(np.float32)
    run_all(csrk, M, K, D, N, rp, ci, v, A, B, C)


def test_bf16_edge_patterns(csrk):
    rng = np.random.default_rng(5)
    for name, M, K, rp, ci in helpers.edge_patterns(rng):
        v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
        for D, N in [(64, 64), (8, 256), (20, 36)]:
            A = rng.normal(size=(M, D)).astype(np.float32)
            B = rng.normal(size=(K, D)).astype(np.float32)
            C = rng.normal(size=(K, N)).astype(np.float32)
            run_all(csrk, M, K, D, N, rp, ci, v, A, B, C)


def test_bf16_skewed_and_even_mid_size(csrk):
    # skewed rows: equal shares with heads; even rows with enough cells of S: whole rows by the row analysis
    w = inputs.workload("fused8k_skew", scale=0.25)
    f = w.ops["fusedmm"]
    rows = np.arange(0, w.M, 17).astype(np.int32)
    run_all(csrk, w.M, w.K, 64, 64, w.rowptr, w.colidx, w.vals, f["A"], f["B"], f["C"], rows=rows)
    w = inputs.custom_workload(9000, 2048, 0.05, 128, 64, seed=2)
    f = w.ops["fusedmm"]
    rows = np.arange(0, w.M, 31).astype(np.int32)
    run_all(csrk, w.M, w.K, 64, 128, w.rowptr, w.colidx, w.vals, f["A"], f["B"], f["C"], rows=rows)


def test_bf16_nan_in_unreferenced_rows_does_not_leak(csrk):
    rng = np.random.default_rng(9)
    M, K, D, N = 200, 300, 64, 128
    poisoned = [0, 7, 150, 299]
    rows = [sorted(c for c in rng.permutation(K)[: int(rng.integers(0, 90))] if c not in poisoned) for _ in range(M)]
    rp, ci = helpers.csr_from_rows(rows, K)
    v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
    A = rng.normal(size=(M, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    C = rng.normal(size=(K, N)).astype(np.float32)
    B[poisoned] = np.nan
    C[poisoned] = np.inf
    run_all(csrk, M, K, D, N, rp, ci, v, A, B, C)


def test_bf16_at_the_benchmark_size_on_sampled_rows(csrk):
    # 16384 x 16384 at 20 %, widths 64 / 512 (what `bench.py --bf16` times): every 31st output row (a stride coprime to the kernels' row layouts) and the ends
    w = inputs.workload("large16k")
    rows = np.unique(np.concatenate([np.arange(3, w.M, 31), [0, 1, 2, w.M - 3, w.M - 2, w.M - 1]])).astype(np.int32)
    f = w.ops["fusedmm"]
    run_all(csrk, w.M, w.K, 64, 512, w.rowptr, w.colidx, w.vals, f["A"], f["B"], f["C"], rows=rows)
