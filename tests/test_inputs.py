"""Seeded input generator: determinism, CSR validity, the paper's Fig. 1 conventions and the
statistics the workload recipes promise.  CPU only."""
import numpy as np
import pytest

import helpers
from paper_2311_00368_amd import inputs


def test_fig1_dense_to_csr_matches_printed_arrays():
    # paper Fig. 1: 0-based indices, rowptr[M] = nnz, values in row-major order
    g = helpers.load_golden("fig1_example.txt")
    rowptr, colidx, vals = inputs.csr_from_dense(g["dense"])
    assert rowptr.dtype == np.int32 and colidx.dtype == np.int32 and vals.dtype == np.float32
    np.testing.assert_array_equal(rowptr, g["ia"].astype(np.int32))
    np.testing.assert_array_equal(colidx, g["ja"].astype(np.int32))
    np.testing.assert_array_equal(vals, g["avalue"].astype(np.float32))
    back = inputs.csr_to_dense(5, 4, rowptr, colidx, vals)
    np.testing.assert_array_equal(back, g["dense"])


def test_raw_stream_is_counter_based_and_streams_differ():
    a = inputs.raw_u64(0, 0, 0, 1000)
    b = inputs.raw_u64(0, 0, 500, 500)
    np.testing.assert_array_equal(a[500:], b)              # value depends on the index only
    assert not np.array_equal(a, inputs.raw_u64(1, 0, 0, 1000))   # seed matters
    assert not np.array_equal(a, inputs.raw_u64(0, 1, 0, 1000))   # stream matters
    assert len(np.unique(a)) == 1000
    bits = np.unpackbits(a.view(np.uint8))
    assert abs(bits.mean() - 0.5) < 0.01


def test_dense_generators_distribution_and_determinism():
    u = inputs.uniform(0, inputs.STREAM_B, (512, 64))
    np.testing.assert_array_equal(u, inputs.uniform(0, inputs.STREAM_B, (512, 64)))
    assert u.dtype == np.float32 and u.min() >= -1.0 and u.max() <= 1.0
    assert abs(u.mean()) < 0.01 and abs(u.var() - 1.0 / 3.0) < 0.01
    u01 = inputs.uniform(0, inputs.STREAM_VALS, 100000, 0.0, 1.0)
    assert u01.min() >= 0.0 and u01.max() <= 1.0 and abs(u01.mean() - 0.5) < 0.01
    z = inputs.normal(0, inputs.STREAM_A, 200000)
    assert abs(z.mean()) < 0.01 and abs(z.std() - 1.0) < 0.01
    assert abs(np.mean(z ** 3)) < 0.05 and abs(np.mean(z ** 4) - 3.0) < 0.1


def _check_csr(M, K, rowptr, colidx):
    assert rowptr.shape == (M + 1,) and rowptr[0] == 0 and np.all(np.diff(rowptr) >= 0)
    assert colidx.shape == (rowptr[M],)
    assert colidx.min() >= 0 and colidx.max() < K
    # ascending and unique within every row
    d = np.diff(colidx.astype(np.int64))
    row_start = np.zeros(len(colidx), dtype=bool)
    row_start[rowptr[:-1][rowptr[:-1] < len(colidx)]] = True
    assert np.all(d[~row_start[1:]] > 0)


@pytest.mark.parametrize("p", [0.1, 0.2, 0.3])
def test_bernoulli_pattern(p):
    M = K = 1024
    rowptr, colidx = inputs.bernoulli_csr(0, M, K, p)
    _check_csr(M, K, rowptr, colidx)
    # nnz ~ Binomial(M*K, p): mean M*K*(1-sparsity) as in the paper's notation table
    nnz, mean, sd = int(rowptr[M]), M * K * p, np.sqrt(M * K * p * (1 - p))
    assert abs(nnz - mean) < 4 * sd
    # column marginals are uniform
    counts = np.bincount(colidx, minlength=K)
    assert abs(counts.mean() - M * p) < 4 * np.sqrt(M * p * (1 - p) / K)
    rp2, ci2 = inputs.bernoulli_csr(0, M, K, p)
    np.testing.assert_array_equal(rowptr, rp2)
    np.testing.assert_array_equal(colidx, ci2)
    assert not np.array_equal(colidx[:100], inputs.bernoulli_csr(1, M, K, p)[1][:100])


def test_lognormal_pattern_statistics():
    M = K = 2048
    rowptr, colidx = inputs.lognormal_csr(0, M, K, 819.0 / 4, 1.0)
    _check_csr(M, K, rowptr, colidx)
    lens = np.diff(rowptr)
    assert lens.min() >= 1 and lens.max() <= K
    # arithmetic mean `mean` before clipping; the median of a log-normal is mean*exp(-sigma^2/2)
    assert abs(lens.mean() - 819.0 / 4) / (819.0 / 4) < 0.1
    assert abs(np.median(lens) - 819.0 / 4 * np.exp(-0.5)) / (819.0 / 4) < 0.1
    assert lens.max() > 8 * np.median(lens)        # skewed
    counts = np.bincount(colidx, minlength=K)      # columns uniform
    assert counts.std() / counts.mean() < 0.2


def test_workload_shapes_scaled():
    w = inputs.workload("tiny")
    assert (w.M, w.K) == (512, 512) and set(w.ops) == {"spmm", "sddmm", "fusedmm"}
    assert abs(w.nnz - 26214) < 4 * np.sqrt(26214 * 0.9)
    assert w.vals.min() >= -1 and w.vals.max() <= 1
    w = inputs.workload("sddmm4k", scale=0.125)
    assert (w.M, w.K) == (512, 512) and w.ops["sddmm"]["A"].shape == (512, 128)
    assert w.vals.min() >= 0.0
    w = inputs.workload("fused8k_skew", scale=0.125)
    assert w.M == 1024 and w.ops["fusedmm"]["C"].shape == (1024, 64)
    assert abs(w.nnz / (w.M * w.K) - 0.1) < 0.02
    w = inputs.workload("large16k", scale=1 / 32)
    assert w.M == 512 and w.ops["spmm"]["B"].shape == (512, 512)
    assert w.ops["fusedmm"]["A"].shape == (512, 64) and w.ops["fusedmm"]["B"].shape == (512, 64)
    assert abs(w.nnz / (w.M * w.K) - 0.2) < 0.01


def test_rounding_helper_matches_the_definition():
    # bfloat16 = the upper 16 bits of a single, round to nearest even: spot values with known patterns
    a = np.array([1.0, -2.0, 0.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, 1.0 + 3 * 2.0 ** -8, 3.0e38, np.inf],
                 dtype=np.float32)
    bits, w = inputs.to_bf16(a)
    assert bits.tolist() == [0x3F80, 0xC000, 0x0000, 0x3F80, 0x3F81, 0x3F82, 0x7F62, 0x7F80]
    assert w[3] == 1.0 and w[4] == np.float32(1.0 + 2.0 ** -7)
