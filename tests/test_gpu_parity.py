"""Parity of the HIP path (through the C-ABI binding) with the CPU oracle, element by element,
on the same seeded inputs.  Bar: |gpu - oracle| <= 1e-5 * sum|terms| for every output entry
(`oracle.within_tolerance`); index arrays must come back bit-identical."""
import numpy as np
import pytest

import helpers
import oracle
from paper_2311_00368_amd import inputs

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

REL_TOL = 1e-5


@pytest.fixture(scope="module")
def csrk():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2311_00368_amd import binding
    binding.load(build_if_missing=False)
    return binding


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


def check(got, want, abs_sum, what):
    ok, worst = oracle.within_tolerance(got, want, abs_sum, REL_TOL)
    assert ok, f"{what}: worst |err|/sum|terms| = {worst:.3e} (limit {REL_TOL})"
    return worst


def run_spmm(csrk, M, K, N, rp, ci, v, B, rows=None):
    d_rp, d_ci = dev(rp), dev(ci)
    O = csrk.spmm_csr(M, K, N, d_rp, d_ci, dev(v), dev(B))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(d_rp.cpu().numpy(), rp)
    np.testing.assert_array_equal(d_ci.cpu().numpy(), ci)
    got = O.cpu().numpy()
    want, a = oracle.spmm(M, K, N, rp, ci, v, B, rows=rows)
    return check(got if rows is None else got[rows], want, a, f"spmm M={M} K={K} N={N}")


def run_sddmm(csrk, M, K, D, rp, ci, v, A, B, rows=None, inplace=False):
    d_v = dev(v)
    P = csrk.sddmm_csr(M, K, D, dev(rp), dev(ci), d_v, dev(A), dev(B), P=d_v if inplace else None)
    torch.cuda.synchronize()
    got = P.cpu().numpy()
    want, a = oracle.sddmm(M, K, D, rp, ci, v, A, B, rows=rows)
    if rows is not None:
        sel = ~np.isnan(want)
        got, want, a = got[sel], want[sel], a[sel]
    return check(got, want, a, f"sddmm M={M} K={K} D={D}")


def run_fused(csrk, M, K, D, N, rp, ci, v, A, B, C, rows=None):
    O = csrk.fusedmm_csr(M, K, D, N, dev(rp), dev(ci), dev(v), dev(A), dev(B), dev(C))
    torch.cuda.synchronize()
    got = O.cpu().numpy()
    want, a = oracle.fusedmm(M, K, D, N, rp, ci, v, A, B, C, rows=rows)
    return check(got if rows is None else got[rows], want, a, f"fusedmm M={M} K={K} D={D} N={N}")


# ------------------------------------------------------------------ small workloads
def test_tiny_all_three(csrk):
    w = inputs.workload("tiny")
    o = w.ops
    run_spmm(csrk, w.M, w.K, 64, w.rowptr, w.colidx, w.vals, o["spmm"]["B"])
    run_sddmm(csrk, w.M, w.K, 64, w.rowptr, w.colidx, w.vals, o["sddmm"]["A"], o["sddmm"]["B"])
    f = o["fusedmm"]
    run_fused(csrk, w.M, w.K, 64, 64, w.rowptr, w.colidx, w.vals, f["A"], f["B"], f["C"])


def test_fig1_example_exact(csrk):
    g = helpers.load_golden("fig1_example.txt")
    rp, ci, v = g["ia"].astype(np.int32), g["ja"].astype(np.int32), g["avalue"].astype(np.float32)
    f32 = lambda k: g[k].astype(np.float32)
    O = csrk.spmm_csr(5, 4, 2, dev(rp), dev(ci), dev(v), dev(f32("spmm_B"))).cpu().numpy()
    np.testing.assert_array_equal(O, g["spmm_O"])
    P = csrk.sddmm_csr(5, 4, 2, dev(rp), dev(ci), None, dev(f32("sddmm_A")), dev(f32("spmm_B"))).cpu().numpy()
    np.testing.assert_array_equal(P, g["sddmm_P_ones"])
    P = csrk.sddmm_csr(5, 4, 2, dev(rp), dev(ci), dev(v), dev(f32("sddmm_A")), dev(f32("spmm_B"))).cpu().numpy()
    np.testing.assert_array_equal(P, g["sddmm_P_scaled"])
    O = csrk.fusedmm_csr(5, 4, 2, 2, dev(rp), dev(ci), dev(v), dev(f32("sddmm_A")), dev(f32("spmm_B")),
                         dev(f32("fused_C"))).cpu().numpy()
    np.testing.assert_array_equal(O, g["fused_O_scaled"])
    O = csrk.fusedmm_csr(5, 4, 2, 2, dev(rp), dev(ci), None, dev(f32("sddmm_A")), dev(f32("spmm_B")),
                         dev(f32("fused_C"))).cpu().numpy()
    np.testing.assert_array_equal(O, g["fused_O_ones"])


WIDTHS = [1, 3, 4, 32, 64, 100, 128, 132, 256, 260, 512, 516, 1028]


@pytest.mark.parametrize("N", WIDTHS)
def test_spmm_widths_ragged(csrk, N):
    rng = np.random.default_rng(N)
    M, K = 333, 417
    rp, ci = inputs.bernoulli_csr(N, M, K, 0.15)
    v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
    B = rng.uniform(-1, 1, (K, N)).astype(np.float32)
    run_spmm(csrk, M, K, N, rp, ci, v, B)


@pytest.mark.parametrize("D", WIDTHS)
def test_sddmm_widths_ragged(csrk, D):
    rng = np.random.default_rng(D)
    M, K = 333, 417
    rp, ci = inputs.bernoulli_csr(D, M, K, 0.15)
    v = rng.uniform(0, 1, len(ci)).astype(np.float32)
    A = rng.normal(size=(M, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    run_sddmm(csrk, M, K, D, rp, ci, v, A, B)
    run_sddmm(csrk, M, K, D, rp, ci, None, A, B)


@pytest.mark.parametrize("D,N", [(1, 1), (3, 5), (4, 4), (64, 64), (64, 512), (128, 128), (100, 36), (32, 260),
                                 (256, 64), (260, 100), (512, 1028), (16, 16), (520, 8)])
def test_fusedmm_widths_ragged(csrk, D, N):
    rng = np.random.default_rng(D * 1000 + N)
    M, K = 210, 301
    rp, ci = inputs.bernoulli_csr(D + N, M, K, 0.2)
    v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
    A = rng.normal(size=(M, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    C = rng.normal(size=(K, N)).astype(np.float32)
    run_fused(csrk, M, K, D, N, rp, ci, v, A, B, C)
    run_fused(csrk, M, K, D, N, rp, ci, None, A, B, C)


# ------------------------------------------------------------------ degenerate patterns
def test_edge_patterns_all_ops(csrk):
    rng = np.random.default_rng(99)
    for name, M, K, rp, ci in helpers.edge_patterns(rng):
        v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
        for D, N in [(64, 64), (5, 7), (128, 256)]:
            A = rng.normal(size=(M, D)).astype(np.float32)
            B = rng.normal(size=(K, D)).astype(np.float32)
            C = rng.normal(size=(K, N)).astype(np.float32)
            run_spmm(csrk, M, K, N, rp, ci, v, C)
            run_fused(csrk, M, K, D, N, rp, ci, v, A, B, C)
            if len(ci):
                run_sddmm(csrk, M, K, D, rp, ci, v, A, B)


def test_one_dense_row_spans_many_workers(csrk):
    # a single row holding every entry: cut into as many segments as there are workers,
    # all partial sums must be combined in order
    rng = np.random.default_rng(3)
    K, N, D = 300000, 64, 64
    rp, ci = helpers.csr_from_rows([[], list(rng.permutation(K)), []], K)
    v = rng.uniform(-1, 1, K).astype(np.float32)
    A = rng.normal(size=(3, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    C = rng.normal(size=(K, N)).astype(np.float32)
    run_spmm(csrk, 3, K, N, rp, ci, v, C)
    run_fused(csrk, 3, K, D, N, rp, ci, v, A, B, C)
    run_sddmm(csrk, 3, K, D, rp, ci, v, A, B)


@pytest.mark.parametrize("N,D", [(32, 16), (128, 64)])
def test_very_many_short_rows(csrk, N, D):
    # more rows than the wave-wide row search covers in three rounds (64^3) and than the row analysis is asked for
    M, K = 300_000, 64
    rng = np.random.default_rng(N)
    rp, ci = inputs.bernoulli_csr(1, M, K, 0.1)
    v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
    A = rng.normal(size=(M, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    C = rng.normal(size=(K, N)).astype(np.float32)
    run_spmm(csrk, M, K, N, rp, ci, v, C)
    run_sddmm(csrk, M, K, D, rp, ci, v, A, B)
    run_fused(csrk, M, K, D, N, rp, ci, v, A, B, C)


def test_nan_in_unreferenced_row_does_not_leak(csrk):
    rng = np.random.default_rng(4)
    M, K, N = 64, 64, 64
    rows = [[c for c in rng.permutation(K)[:20] if c != 0] for _ in range(M)]   # column 0 never referenced
    rp, ci = helpers.csr_from_rows(rows, K)
    v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
    B = rng.uniform(-1, 1, (K, N)).astype(np.float32)
    B[0, :] = np.nan
    O = csrk.spmm_csr(M, K, N, dev(rp), dev(ci), dev(v), dev(B)).cpu().numpy()
    assert np.all(np.isfinite(O))
    A = rng.normal(size=(M, N)).astype(np.float32)
    O = csrk.fusedmm_csr(M, K, N, N, dev(rp), dev(ci), dev(v), dev(A), dev(B), dev(B)).cpu().numpy()
    assert np.all(np.isfinite(O))


def test_sddmm_in_place_and_determinism(csrk):
    w = inputs.workload("fused8k_skew", scale=0.125)
    f = w.ops["fusedmm"]
    run_sddmm(csrk, w.M, w.K, 64, w.rowptr, w.colidx, w.vals, f["A"], f["B"], inplace=True)
    args = (w.M, w.K, 64, 64, dev(w.rowptr), dev(w.colidx), dev(w.vals), dev(f["A"]), dev(f["B"]), dev(f["C"]))
    O1 = csrk.fusedmm_csr(*args).cpu().numpy()
    O2 = csrk.fusedmm_csr(*args).cpu().numpy()
    np.testing.assert_array_equal(O1, O2)       # partial rows are combined in a fixed order


def test_empty_dimensions_and_errors(csrk):
    z = torch.zeros(1, dtype=torch.int32, device="cuda")
    e_i = torch.empty(0, dtype=torch.int32, device="cuda")
    e_f = torch.empty(0, dtype=torch.float32, device="cuda")
    O = csrk.spmm_csr(0, 5, 4, z, e_i, e_f, torch.zeros(5, 4, device="cuda"))
    assert O.shape == (0, 4)
    rp = torch.zeros(4, dtype=torch.int32, device="cuda")
    O = csrk.spmm_csr(3, 5, 4, rp, e_i, e_f, torch.ones(5, 4, device="cuda"), O=torch.full((3, 4), 7.0, device="cuda"))
    assert torch.all(O == 0)
    O = csrk.fusedmm_csr(3, 5, 2, 4, rp, e_i, None, torch.ones(3, 2, device="cuda"), torch.ones(5, 2, device="cuda"),
                         torch.ones(5, 4, device="cuda"), O=torch.full((3, 4), 7.0, device="cuda"))
    assert torch.all(O == 0)
    lib = csrk.load()
    assert lib.spmm_csr(-1, 5, 4, None, None, None, None, None, None) == 1
    assert b"negative" in lib.csrk_last_error()
    assert lib.spmm_csr(3, 5, 4, None, None, None, None, None, None) == 1
    assert b"NULL" in lib.csrk_last_error()
    assert lib.sddmm_csr(3, 5, 1 << 25, None, None, None, None, None, None, None) == 2


def test_validate_csr(csrk):
    rp, ci = inputs.bernoulli_csr(0, 200, 300, 0.1)
    assert csrk.csrk_validate_csr(200, 300, dev(rp), dev(ci)) == (0, True)
    bad = ci.copy()
    bad[17] = 300
    assert csrk.csrk_validate_csr(200, 300, dev(rp), dev(bad))[0] & 4
    sw = ci.copy()
    lo = rp[5]
    sw[lo], sw[lo + 1] = ci[lo + 1], ci[lo]
    assert csrk.csrk_validate_csr(200, 300, dev(rp), dev(sw)) == (0, False)
    brp = rp.copy()
    brp[10] = brp[9] - 1
    assert csrk.csrk_validate_csr(200, 300, dev(brp), dev(ci))[0] & 2


# ------------------------------------------------------------------ the five workloads
def test_workload_spmm4k_full(csrk):
    w = inputs.workload("spmm4k")
    run_spmm(csrk, w.M, w.K, 256, w.rowptr, w.colidx, w.vals, w.ops["spmm"]["B"])


def test_workload_sddmm4k_full(csrk):
    w = inputs.workload("sddmm4k")
    o = w.ops["sddmm"]
    run_sddmm(csrk, w.M, w.K, 128, w.rowptr, w.colidx, w.vals, o["A"], o["B"])


def test_workload_fused8k_skew_full(csrk):
    w = inputs.workload("fused8k_skew")
    f = w.ops["fusedmm"]
    run_fused(csrk, w.M, w.K, 64, 64, w.rowptr, w.colidx, w.vals, f["A"], f["B"], f["C"])


def test_workload_large16k_every_row(csrk):
    # full size, in the launch configuration the benchmark times, every output row and every stored entry
    # against the oracle: this is the only size at which the un-split 4-rows-per-wavefront tiled kernels run,
    # and every wavefront and row slot of their layout must be looked at
    w = inputs.workload("large16k")
    run_spmm(csrk, w.M, w.K, 512, w.rowptr, w.colidx, w.vals, w.ops["spmm"]["B"])
    f = w.ops["fusedmm"]
    run_fused(csrk, w.M, w.K, 64, 512, w.rowptr, w.colidx, w.vals, f["A"], f["B"], f["C"])
    s = w.ops["sddmm"]
    run_sddmm(csrk, w.M, w.K, 64, w.rowptr, w.colidx, w.vals, s["A"], s["B"])


def test_sddmm_with_128_float_rows_at_the_benchmark_size(csrk):
    # SDDMM alone at 16384 x 16384 / 20 % with the longer of the two dot lengths of the workloads (D = 128),
    # every stored entry compared
    w = inputs.workload("large16k")
    A = inputs.normal(0, inputs.STREAM_A, (w.M, 128))
    B = inputs.normal(0, inputs.STREAM_B, (w.K, 128))
    run_sddmm(csrk, w.M, w.K, 128, w.rowptr, w.colidx, w.vals, A, B)
    run_sddmm(csrk, w.M, w.K, 128, w.rowptr, w.colidx, None, A, B)


# ------------------------------------------------------------------ call-site variations
def test_misaligned_operands_take_the_scalar_path(csrk):
    # dense operands that start 4 bytes off a 16-byte boundary cannot use 128-bit accesses;
    # the library must notice and still be right
    rng = np.random.default_rng(8)
    M, K, N, D = 200, 300, 64, 64
    rp, ci = inputs.bernoulli_csr(8, M, K, 0.2)
    v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
    A = rng.normal(size=(M, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    C = rng.normal(size=(K, N)).astype(np.float32)

    def off(a):                 # same values, storage shifted by one float
        buf = torch.empty(a.size + 1, dtype=torch.float32, device="cuda")
        view = buf[1:].view(a.shape)
        view.copy_(torch.from_numpy(a))
        assert view.data_ptr() % 16 == 4
        return view

    d_rp, d_ci, d_v = dev(rp), dev(ci), dev(v)
    O = csrk.spmm_csr(M, K, N, d_rp, d_ci, d_v, off(C)).cpu().numpy()
    want, a = oracle.spmm(M, K, N, rp, ci, v, C)
    check(O, want, a, "spmm misaligned B")
    O_buf = torch.empty(M * N + 1, dtype=torch.float32, device="cuda")[1:].view(M, N)
    csrk.spmm_csr(M, K, N, d_rp, d_ci, d_v, dev(C), O=O_buf)
    check(O_buf.cpu().numpy(), want, a, "spmm misaligned O")
    P = csrk.sddmm_csr(M, K, D, d_rp, d_ci, d_v, off(A), off(B)).cpu().numpy()
    wantp, ap = oracle.sddmm(M, K, D, rp, ci, v, A, B)
    check(P, wantp, ap, "sddmm misaligned A, B")
    F = csrk.fusedmm_csr(M, K, D, N, d_rp, d_ci, d_v, off(A), dev(B), off(C)).cpu().numpy()
    wantf, af = oracle.fusedmm(M, K, D, N, rp, ci, v, A, B, C)
    check(F, wantf, af, "fusedmm misaligned A, C")


def test_side_stream_and_growing_scratch(csrk):
    # calls enqueued on a non-default stream, with output widths that make the library's
    # partial-row scratch grow between calls
    rng = np.random.default_rng(9)
    M, K = 300, 400
    rp, ci = inputs.bernoulli_csr(9, M, K, 0.25)
    v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
    d_rp, d_ci, d_v = dev(rp), dev(ci), dev(v)
    csrk.csrk_release_workspace()
    side = torch.cuda.Stream()
    for N in (8, 64, 640, 72):
        C = rng.normal(size=(K, N)).astype(np.float32)
        d_C = dev(C)
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            O = csrk.spmm_csr(M, K, N, d_rp, d_ci, d_v, d_C)
        side.synchronize()
        want, a = oracle.spmm(M, K, N, rp, ci, v, C)
        check(O.cpu().numpy(), want, a, f"spmm on a side stream, N={N}")


def test_back_to_back_calls_do_not_disturb_each_other(csrk):
    # three different calls queued without synchronising in between share the library's
    # flags and scratch; stream order must keep them apart
    w = inputs.workload("tiny")
    f = w.ops["fusedmm"]
    d = dict(rp=dev(w.rowptr), ci=dev(w.colidx), v=dev(w.vals), A=dev(f["A"]), B=dev(f["B"]), C=dev(f["C"]))
    outs = []
    for _ in range(3):
        outs.append((csrk.spmm_csr(w.M, w.K, 64, d["rp"], d["ci"], d["v"], d["C"]),
                     csrk.sddmm_csr(w.M, w.K, 64, d["rp"], d["ci"], d["v"], d["A"], d["B"]),
                     csrk.fusedmm_csr(w.M, w.K, 64, 64, d["rp"], d["ci"], d["v"], d["A"], d["B"], d["C"])))
    torch.cuda.synchronize()
    so, sa = oracle.spmm(w.M, w.K, 64, w.rowptr, w.colidx, w.vals, f["C"])
    po, pa = oracle.sddmm(w.M, w.K, 64, w.rowptr, w.colidx, w.vals, f["A"], f["B"])
    fo, fa = oracle.fusedmm(w.M, w.K, 64, 64, w.rowptr, w.colidx, w.vals, f["A"], f["B"], f["C"])
    for O, P, F in outs:
        check(O.cpu().numpy(), so, sa, "spmm back to back")
        check(P.cpu().numpy(), po, pa, "sddmm back to back")
        check(F.cpu().numpy(), fo, fa, "fusedmm back to back")
    for O, P, F in outs[1:]:
        assert torch.equal(O, outs[0][0]) and torch.equal(P, outs[0][1]) and torch.equal(F, outs[0][2])


@pytest.mark.parametrize("shape", [(4096, 4096, 0.3, 128, 128), (8192, 2048, 0.2, 32, 32), (4100, 1000, 0.25, 100, 60),
                                   (9000, 3000, 0.07, 128, 64), (5000, 5000, 0.2, 256, 64)])
def test_automatic_kernel_choice_mid_sizes(csrk, shape):
    # shapes around the dispatch thresholds (narrow tiled / wide tiled / general), default mode,
    # a sample of rows checked (rows are independent)
    M, K, p, N, D = shape
    w = inputs.custom_workload(M, K, p, N, D, seed=3)
    rows = np.unique(np.concatenate([np.arange(0, M, 37), [0, 1, 2, 3, M - 4, M - 3, M - 2, M - 1]])).astype(np.int32)
    f = w.ops["fusedmm"]
    run_spmm(csrk, M, K, N, w.rowptr, w.colidx, w.vals, f["C"], rows=rows)
    run_sddmm(csrk, M, K, D, w.rowptr, w.colidx, w.vals, f["A"], f["B"], rows=rows)
    run_fused(csrk, M, K, D, N, w.rowptr, w.colidx, w.vals, f["A"], f["B"], f["C"], rows=rows)


@pytest.mark.parametrize("shape", [(8192, 2048, 0.05, 32, 32), (4096, 2048, 0.01, 512, 64), (9000, 4096, 0.04, 128, 128),
                                   (2000, 1000, 0.1, 128, 128), (700, 2048, 0.3, 64, 64), (3500, 900, 0.2, 36, 32),
                                   (1024, 8192, 0.1, 256, 64), (3000, 4096, 0.03, 256, 32), (5000, 2048, 0.02, 512, 64)])
def test_whole_rows_paths_for_even_matrices(csrk, shape):
    """Matrices whose rows are about equally long are dealt out row by row instead of in equal shares of the
    stored entries: by the host's choice where S is small (one, two or four wavefronts per row), by the row
    analysis' verdict where a tiled kernel was tried and turned down (too sparse here) or S is large.  Same
    arithmetic per row (Algorithms 2 and 3), so the same bar."""
    M, K, p, N, D = shape
    w = inputs.custom_workload(M, K, p, N, D, seed=11)
    rows = np.unique(np.concatenate([np.arange(0, M, 29), [0, 1, 2, 3, M - 4, M - 3, M - 2, M - 1]])).astype(np.int32)
    f = w.ops["fusedmm"]
    run_spmm(csrk, M, K, N, w.rowptr, w.colidx, w.vals, f["C"], rows=rows)
    run_sddmm(csrk, M, K, D, w.rowptr, w.colidx, w.vals, f["A"], f["B"], rows=rows)
    run_fused(csrk, M, K, D, N, w.rowptr, w.colidx, w.vals, f["A"], f["B"], f["C"], rows=rows)


def test_whole_rows_forced_on_uneven_and_ragged_inputs(csrk, monkeypatch):
    """CSRK_ROWS=2 sends every call the row kernels can run through them: empty rows, one dense row, widths that
    need the tail handling, M below one workgroup."""
    monkeypatch.setenv("CSRK_ROWS", "2")
    rng = np.random.default_rng(21)
    for name, M, K, rp, ci in helpers.edge_patterns(rng):
        v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
        for D, N in [(64, 64), (32, 128), (8, 256), (128, 4)]:
            A = rng.normal(size=(M, D)).astype(np.float32)
            B = rng.normal(size=(K, D)).astype(np.float32)
            C = rng.normal(size=(K, N)).astype(np.float32)
            run_spmm(csrk, M, K, N, rp, ci, v, C)
            run_fused(csrk, M, K, D, N, rp, ci, v, A, B, C)
            if len(ci):
                run_sddmm(csrk, M, K, D, rp, ci, v, A, B)
                run_sddmm(csrk, M, K, D, rp, ci, v, A, B, inplace=True)
