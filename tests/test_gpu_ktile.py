"""The LDS-tiled SPMM / FusedMM kernels against the CPU oracle.

By default the library picks these kernels only for large shapes; CSRK_KTILE=2 makes it take
them wherever the kernel can run at all (output width a multiple of 4 up to 2048 - beyond 512 in
column slabs, one launch each - dot length a multiple of 4 up to 64), so small and ragged cases reach them too.  Patterns the kernels cannot
take (columns not ascending, or too sparse) must fall back to the general kernels on the device
and still give the right answer."""
import os

import numpy as np
import pytest

import helpers
from paper_2311_00368_amd import inputs
import oracle
from test_gpu_parity import check, csrk, dev, run_fused, run_sddmm, run_spmm  # noqa: F401  (csrk is a fixture)

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def force_ktile():
    old = os.environ.get("CSRK_KTILE")
    os.environ["CSRK_KTILE"] = "2"
    yield
    if old is None:
        os.environ.pop("CSRK_KTILE", None)
    else:
        os.environ["CSRK_KTILE"] = old


@pytest.mark.parametrize("M,K,N", [(64, 64, 256), (100, 257, 512), (333, 417, 4), (1000, 129, 260), (65, 1000, 128),
                                   (2048, 2048, 512), (130, 70, 500)])
@pytest.mark.parametrize("p", [0.05, 0.3, 1.0])
def test_spmm_ktile(csrk, M, K, N, p):
    rng = np.random.default_rng(M + K + N)
    rp, ci = inputs.bernoulli_csr(N, M, K, p)
    v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
    B = rng.uniform(-1, 1, (K, N)).astype(np.float32)
    run_spmm(csrk, M, K, N, rp, ci, v, B)


@pytest.mark.parametrize("M,K,D,N", [(64, 64, 64, 256), (100, 257, 64, 512), (333, 417, 4, 4), (1000, 129, 32, 260),
                                     (2048, 2048, 64, 512), (130, 70, 60, 500), (70, 300, 16, 64),
                                     (300, 700, 128, 128), (257, 129, 100, 32), (1100, 900, 96, 64), (90, 2000, 128, 4),
                                     (500, 500, 32, 32), (64, 640, 68, 100)])
@pytest.mark.parametrize("p", [0.05, 0.3, 0.7, 1.0])   # 0.7: rows overflow the wide kernel's 32-entry slots, not the chunk
def test_fusedmm_ktile(csrk, M, K, D, N, p):
    rng = np.random.default_rng(M + K + N + D)
    rp, ci = inputs.bernoulli_csr(N + D, M, K, p)
    v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
    A = rng.normal(size=(M, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    C = rng.normal(size=(K, N)).astype(np.float32)
    run_fused(csrk, M, K, D, N, rp, ci, v, A, B, C)
    run_fused(csrk, M, K, D, N, rp, ci, None, A, B, C)


@pytest.mark.parametrize("N,D", [(32, 32), (64, 64), (128, 16), (256, 8), (512, 64), (64, 128), (128, 100)])
def test_three_rows_per_wavefront(csrk, N, D):
    # between 8193 and 12288 rows (and between 16385 and 24576) the SPMM and SDDMM tiled kernels run with 3 rows per
    # wavefront, 48 per workgroup: here with a ragged last workgroup and a last partial tile
    M, K = 9001, 300
    rng = np.random.default_rng(N + D)
    rp, ci = inputs.bernoulli_csr(N, M, K, 0.3)
    v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
    A = rng.normal(size=(M, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    C = rng.normal(size=(K, N)).astype(np.float32)
    run_spmm(csrk, M, K, N, rp, ci, v, C)
    run_sddmm(csrk, M, K, D, rp, ci, v, A, B)
    run_fused(csrk, M, K, D, N, rp, ci, v, A, B, C)


@pytest.mark.parametrize("N,D", [(128, 32), (256, 64), (100, 128)])
def test_three_rows_per_wavefront_fused(csrk, N, D):
    # FusedMM takes its 3-row version (the 4-row layout, fourth row empty) only above 16384 rows and 64 columns
    M, K = 16500, 150
    rng = np.random.default_rng(N * 7 + D)
    rp, ci = inputs.bernoulli_csr(D, M, K, 0.3)
    v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
    A = rng.normal(size=(M, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    C = rng.normal(size=(K, N)).astype(np.float32)
    run_fused(csrk, M, K, D, N, rp, ci, v, A, B, C)
    run_fused(csrk, M, K, D, N, rp, ci, None, A, B, C)


@pytest.mark.parametrize("M,K,D", [(64, 64, 64), (100, 257, 128), (333, 417, 4), (1000, 1300, 32), (65, 3000, 100),
                                   (2048, 2048, 64), (130, 70, 60), (4096, 600, 128)])
@pytest.mark.parametrize("p", [0.05, 0.3, 1.0])
def test_sddmm_ktile(csrk, M, K, D, p):
    rng = np.random.default_rng(M + K + D)
    rp, ci = inputs.bernoulli_csr(D, M, K, p)
    v = rng.uniform(0, 1, len(ci)).astype(np.float32)
    A = rng.normal(size=(M, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    run_sddmm(csrk, M, K, D, rp, ci, v, A, B)
    run_sddmm(csrk, M, K, D, rp, ci, None, A, B)
    run_sddmm(csrk, M, K, D, rp, ci, v, A, B, inplace=True)


def test_edge_patterns_ktile(csrk):
    # includes unsorted and duplicated columns, empty rows, one full row: the device-side
    # analysis must route each to a kernel that handles it
    rng = np.random.default_rng(77)
    for name, M, K, rp, ci in helpers.edge_patterns(rng):
        v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
        for D, N in [(64, 64), (64, 512), (8, 256)]:
            A = rng.normal(size=(M, D)).astype(np.float32)
            B = rng.normal(size=(K, D)).astype(np.float32)
            C = rng.normal(size=(K, N)).astype(np.float32)
            run_spmm(csrk, M, K, N, rp, ci, v, C)
            run_fused(csrk, M, K, D, N, rp, ci, v, A, B, C)
            if len(ci):
                run_sddmm(csrk, M, K, D, rp, ci, v, A, B)


def test_sorted_with_duplicates_and_dense_rows_ktile(csrk):
    rng = np.random.default_rng(5)
    K, N, D = 700, 512, 64
    rows = []
    for i in range(150):
        n = int(rng.integers(0, 3 * K))
        rows.append(sorted(rng.integers(0, K, size=n).tolist()))      # ascending, many repeats, rows > 64 per tile
    rp, ci = helpers.csr_from_rows(rows, K)
    v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
    A = rng.normal(size=(150, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    C = rng.normal(size=(K, N)).astype(np.float32)
    run_spmm(csrk, 150, K, N, rp, ci, v, C)
    run_fused(csrk, 150, K, D, N, rp, ci, v, A, B, C)
    run_sddmm(csrk, 150, K, D, rp, ci, v, A, B)


def test_skewed_rows_ktile(csrk):
    w = inputs.workload("fused8k_skew", scale=0.25)
    f = w.ops["fusedmm"]
    rng = np.random.default_rng(1)
    C = rng.normal(size=(w.K, 256)).astype(np.float32)
    run_spmm(csrk, w.M, w.K, 256, w.rowptr, w.colidx, w.vals, C)
    run_fused(csrk, w.M, w.K, 64, 256, w.rowptr, w.colidx, w.vals, f["A"], f["B"], C)
    run_sddmm(csrk, w.M, w.K, 64, w.rowptr, w.colidx, w.vals, f["A"], f["B"])


@pytest.mark.parametrize("swap_at", [0, 1, 62, 63, 64, 65, 126, 127, 128, 191, 500, -2])
def test_one_descending_pair_anywhere_is_noticed(csrk, swap_at):
    # The tiled kernels check column order themselves while streaming; a single swapped pair of
    # neighbours, wherever it sits relative to the 64-entry chunks, must send the call to the
    # general kernels (the result must still match the oracle).
    rng = np.random.default_rng(1000 + swap_at)
    M, K, D, N = 70, 1500, 64, 512
    rows = []
    for i in range(M):
        L = int(rng.integers(5, 1400))
        rows.append(sorted(rng.permutation(K)[:L].tolist()))
    victim = int(rng.integers(0, M))
    rows[victim] = sorted(rng.permutation(K)[:1300].tolist())      # long row: many chunks, > 64 entries in a tile
    p = swap_at if swap_at >= 0 else len(rows[victim]) + swap_at
    rows[victim][p], rows[victim][p + 1] = rows[victim][p + 1], rows[victim][p]
    rp, ci = helpers.csr_from_rows(rows, K)
    assert csrk.csrk_validate_csr(M, K, dev(rp), dev(ci)) == (0, False)
    v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
    A = rng.normal(size=(M, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    C = rng.normal(size=(K, N)).astype(np.float32)
    run_spmm(csrk, M, K, N, rp, ci, v, C)
    run_fused(csrk, M, K, D, N, rp, ci, v, A, B, C)
    run_sddmm(csrk, M, K, D, rp, ci, v, A, B)
    # and the same pattern put back in order goes through the tiled kernels
    rows[victim] = sorted(rows[victim])
    rp, ci = helpers.csr_from_rows(rows, K)
    run_spmm(csrk, M, K, N, rp, ci, v, C)
    run_fused(csrk, M, K, D, N, rp, ci, v, A, B, C)
    run_sddmm(csrk, M, K, D, rp, ci, v, A, B)


@pytest.mark.parametrize("N,D", [(512, 64), (256, 64), (128, 128), (32, 32)])
def test_nonfinite_values_in_unreferenced_rows_do_not_leak_ktile(csrk, N, D):
    """Rows of the dense right-hand operands that no stored entry references may hold NaN / Inf: the
    tiled kernels stage them in LDS with the rest of the tile (and idle lanes of the score stages walk
    tile rows they have no entry for), but nothing of them may reach an output (only stored entries
    contribute: eq. (1)-(3))."""
    rng = np.random.default_rng(N + D)
    M, K = 200, 300
    poisoned = [0, 1, 63, 64, 150, 299]            # first row of a tile, tile edges, last row
    rows = [sorted(c for c in rng.permutation(K)[: int(rng.integers(0, 120))] if c not in poisoned) for _ in range(M)]
    rp, ci = helpers.csr_from_rows(rows, K)
    v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
    A = rng.normal(size=(M, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    C = rng.normal(size=(K, N)).astype(np.float32)
    B[poisoned, :] = np.nan
    C[poisoned, :] = np.inf
    O = csrk.spmm_csr(M, K, N, dev(rp), dev(ci), dev(v), dev(C)).cpu().numpy()
    assert np.all(np.isfinite(O))
    P = csrk.sddmm_csr(M, K, D, dev(rp), dev(ci), dev(v), dev(A), dev(B)).cpu().numpy()
    assert np.all(np.isfinite(P))
    O = csrk.fusedmm_csr(M, K, D, N, dev(rp), dev(ci), dev(v), dev(A), dev(B), dev(C)).cpu().numpy()
    assert np.all(np.isfinite(O))
    # and with clean operands the same calls agree with the oracle
    B[poisoned, :] = 0.5
    C[poisoned, :] = -0.25
    run_spmm(csrk, M, K, N, rp, ci, v, C)
    run_sddmm(csrk, M, K, D, rp, ci, v, A, B)
    run_fused(csrk, M, K, D, N, rp, ci, v, A, B, C)


def _env(name, value):
    old = os.environ.get(name)
    if value is None:
        os.environ.pop(name, None)
    else:
        os.environ[name] = value
    return old


@pytest.mark.parametrize("M,K,D,N", [(300, 4096, 64, 512), (1000, 2500, 32, 256), (130, 3000, 128, 128), (257, 2048, 64, 64)])
def test_ksplit_agrees_with_unsplit_and_repeats_bit_for_bit(csrk, M, K, D, N):
    """Small M: the tiled SPMM / FusedMM kernels cut K into ranges, one workgroup per (row block, range), and a
    second kernel adds the partial outputs in a fixed order.  Same answer (to the oracle's tolerance) as with the
    split switched off, and the same bits on every run."""
    rng = np.random.default_rng(M + K)
    rp, ci = inputs.bernoulli_csr(7, M, K, 0.2)
    v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
    A = rng.normal(size=(M, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    C = rng.normal(size=(K, N)).astype(np.float32)
    args = (dev(rp), dev(ci), dev(v))
    dA, dB, dC = dev(A), dev(B), dev(C)
    outs = {}
    for split in ("1", "2"):                       # 1 = automatic split, 2 = off
        old = _env("CSRK_KSPLIT", split)
        try:
            run_spmm(csrk, M, K, N, rp, ci, v, C)
            run_fused(csrk, M, K, D, N, rp, ci, v, A, B, C)
            outs[split] = (csrk.spmm_csr(M, K, N, *args, dC).cpu().numpy(),
                           csrk.fusedmm_csr(M, K, D, N, *args, dA, dB, dC).cpu().numpy())
            again = (csrk.spmm_csr(M, K, N, *args, dC).cpu().numpy(),
                     csrk.fusedmm_csr(M, K, D, N, *args, dA, dB, dC).cpu().numpy())
            assert np.array_equal(outs[split][0], again[0]) and np.array_equal(outs[split][1], again[1])
        finally:
            _env("CSRK_KSPLIT", old)
    # the two ways differ only by where partial sums are rounded
    for a, b in zip(outs["1"], outs["2"]):
        assert np.allclose(a, b, rtol=0, atol=1e-5 * (np.abs(a).max() + 1) * 50)


@pytest.mark.parametrize("kind", ["shuffled", "rotated", "big_first", "one_swap_far_from_range_starts"])
def test_ksplit_never_trusts_a_binary_search_in_unsorted_rows(csrk, kind):
    """With K cut into ranges a workgroup finds its starting entry in each row by binary search, which means
    nothing if the row is not sorted; such inputs must be noticed by the full order check that the workgroups
    of a K-split launch make of their row blocks, and handed to the general kernels."""
    rng = np.random.default_rng(len(kind))
    M, K, D, N = 200, 4096, 64, 512
    rows = []
    for i in range(M):
        cols = sorted(rng.permutation(K)[: int(rng.integers(300, 1200))].tolist())
        if kind == "shuffled":
            cols = rng.permutation(cols).tolist()
        elif kind == "rotated" and i % 3 == 0:
            h = len(cols) // 2
            cols = cols[h:] + cols[:h]                       # two sorted halves, the larger columns first
        elif kind == "big_first" and i % 5 == 0:
            cols = [cols[-1]] + cols[:-1]
        rows.append(cols)
    if kind == "one_swap_far_from_range_starts":
        r = rows[77]
        p = next(i for i, c in enumerate(r) if c > 700)      # well inside the first range
        r[p], r[p + 1] = r[p + 1], r[p]
    rp, ci = helpers.csr_from_rows(rows, K)
    v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
    A = rng.normal(size=(M, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    C = rng.normal(size=(K, N)).astype(np.float32)
    run_spmm(csrk, M, K, N, rp, ci, v, C)
    run_fused(csrk, M, K, D, N, rp, ci, v, A, B, C)
    run_spmm(csrk, M, K, 128, rp, ci, v, C[:, :128].copy())
    run_fused(csrk, M, K, D, 128, rp, ci, v, A, B, C[:, :128].copy())


def test_unsorted_and_sorted_patterns_in_turn(csrk):
    # The ordering flag lives in two sets of flag words that take turns from one tiled attempt to the next; a report
    # of descending columns in one call must neither be lost nor leak into the calls after it, whatever the operation.
    rng = np.random.default_rng(77)
    M, K, N, D = 700, 900, 128, 32
    rp, ci = inputs.bernoulli_csr(3, M, K, 0.2)
    ci_bad = ci.copy()
    ci_bad[rp[300]:rp[301]] = ci_bad[rp[300]:rp[301]][::-1]
    v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
    A = rng.normal(size=(M, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    C = rng.normal(size=(K, N)).astype(np.float32)
    for cols in (ci_bad, ci, ci, ci_bad, ci_bad, ci, ci_bad, ci):
        run_spmm(csrk, M, K, N, rp, cols, v, C)
        run_fused(csrk, M, K, D, N, rp, cols, v, A, B, C)
        run_sddmm(csrk, M, K, D, rp, cols, v, A, B)


def test_released_workspace_is_rebuilt_with_clear_flags(csrk):
    # the flag words live in the workspace: after a release the next tiled attempt must find them cleared again,
    # also when the call before the release had reported descending columns
    rng = np.random.default_rng(5)
    M, K, N = 300, 400, 256
    rp, ci = inputs.bernoulli_csr(8, M, K, 0.25)
    ci_bad = ci.copy()
    ci_bad[rp[10]:rp[11]] = ci_bad[rp[10]:rp[11]][::-1]
    v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
    C = rng.normal(size=(K, N)).astype(np.float32)
    for cols in (ci_bad, ci, ci_bad, ci):
        run_spmm(csrk, M, K, N, rp, cols, v, C)
        torch.cuda.synchronize()
        csrk.csrk_release_workspace()
        run_spmm(csrk, M, K, N, rp, ci, v, C)


@pytest.mark.parametrize("S", [2, 3, 5, 7, 8])
def test_every_number_of_k_ranges(csrk, monkeypatch, S):
    # CSRK_KSPLIT_S fixes the number of ranges K is cut into (otherwise chosen from M and the CU count)
    monkeypatch.setenv("CSRK_KSPLIT_S", str(S))
    rng = np.random.default_rng(S)
    M, K, D = 301, 4100, 64
    rp, ci = inputs.bernoulli_csr(S, M, K, 0.1)
    v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
    A = rng.normal(size=(M, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    for N in (512, 128, 64):
        C = rng.normal(size=(K, N)).astype(np.float32)
        run_spmm(csrk, M, K, N, rp, ci, v, C)
        run_fused(csrk, M, K, D, N, rp, ci, v, A, B, C)


# outputs wider than one kernel's 512 columns: slabs of 512 columns and a remainder, one launch each (516 -> 512 + 4;
# 768 -> 512 + 256, the remainder in the 256-wide kernel; 1500 -> 512 + 512 + 476; 2048 -> 4 x 512); M = 130 and 300
# with long rows take the K-split and its shared combine step
@pytest.mark.parametrize("M,K,N", [(64, 64, 516), (333, 417, 768), (1000, 129, 1024), (130, 3000, 1500), (2100, 700, 2048),
                                   (300, 4096, 1024)])
@pytest.mark.parametrize("p", [0.05, 0.4])
def test_outputs_wider_than_one_kernel_go_in_column_slabs(csrk, M, K, N, p):
    rng = np.random.default_rng(M + K + N)
    rp, ci = inputs.bernoulli_csr(N, M, K, p)
    v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
    A = rng.normal(size=(M, 64)).astype(np.float32)
    B = rng.normal(size=(K, 64)).astype(np.float32)
    C = rng.uniform(-1, 1, (K, N)).astype(np.float32)
    run_spmm(csrk, M, K, N, rp, ci, v, C)
    run_fused(csrk, M, K, 64, N, rp, ci, v, A, B, C)
    run_fused(csrk, M, K, 40, N, rp, ci, None, A[:, :40].copy(), B[:, :40].copy(), C)
    # dot products of 65 to 128 floats: the narrow kernel, 128 columns of the output per launch
    A2 = rng.normal(size=(M, 128)).astype(np.float32)
    B2 = rng.normal(size=(K, 128)).astype(np.float32)
    run_fused(csrk, M, K, 128, N, rp, ci, v, A2, B2, C)
    run_fused(csrk, M, K, 100, N, rp, ci, None, A2[:, :100].copy(), B2[:, :100].copy(), C)
    # a plan on the same pattern, and the same pattern with one row written backwards (general kernels redo it)
    plan = csrk.csrk_plan_create(M, K, dev(rp), dev(ci))
    got = csrk.spmm_csr_plan(plan, N, dev(v), dev(C))
    assert torch.equal(got, csrk.spmm_csr(M, K, N, dev(rp), dev(ci), dev(v), dev(C)))
    csrk.csrk_plan_destroy(plan)
    r = M // 2
    ci2, v2 = ci.copy(), v.copy()
    ci2[rp[r]:rp[r + 1]] = ci2[rp[r]:rp[r + 1]][::-1]
    v2[rp[r]:rp[r + 1]] = v2[rp[r]:rp[r + 1]][::-1]
    run_spmm(csrk, M, K, N, rp, ci2, v2, C)
    run_fused(csrk, M, K, 64, N, rp, ci2, v2, A, B, C)
    run_fused(csrk, M, K, 128, N, rp, ci2, v2, A2, B2, C)


@pytest.mark.parametrize("M,K,D,N", [(333, 417, 128, 256), (1000, 700, 72, 512), (130, 3000, 128, 260), (2100, 300, 96, 200)])
@pytest.mark.parametrize("p", [0.05, 0.3, 1.0])
def test_fusedmm_long_dot_products_with_wide_outputs(csrk, M, K, D, N, p):
    rng = np.random.default_rng(M + K + N + D)
    rp, ci = inputs.bernoulli_csr(N + D, M, K, p)
    v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
    A = rng.normal(size=(M, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    C = rng.normal(size=(K, N)).astype(np.float32)
    run_fused(csrk, M, K, D, N, rp, ci, v, A, B, C)
    run_fused(csrk, M, K, D, N, rp, ci, None, A, B, C)
    plan = csrk.csrk_plan_create(M, K, dev(rp), dev(ci))
    got = csrk.fusedmm_csr_plan(plan, D, N, dev(v), dev(A), dev(B), dev(C))
    assert torch.equal(got, csrk.fusedmm_csr(M, K, D, N, dev(rp), dev(ci), dev(v), dev(A), dev(B), dev(C)))
    csrk.csrk_plan_destroy(plan)


def test_wide_outputs_with_automatic_kernel_choice(csrk, monkeypatch):
    monkeypatch.setenv("CSRK_KTILE", "1")
    M, K, N = 4096, 4096, 1024
    rng = np.random.default_rng(8)
    rp, ci = inputs.bernoulli_csr(3, M, K, 0.1)
    v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
    A = rng.normal(size=(M, 64)).astype(np.float32)
    B = rng.normal(size=(K, 64)).astype(np.float32)
    C = rng.uniform(-1, 1, (K, N)).astype(np.float32)
    rows = np.unique(np.concatenate([np.arange(0, M, 7), [M - 4, M - 3, M - 2, M - 1]])).astype(np.int32)   # a stride coprime to the 64 rows of a workgroup
    run_spmm(csrk, M, K, N, rp, ci, v, C, rows=rows)
    run_fused(csrk, M, K, 64, N, rp, ci, v, A, B, C, rows=rows)
    A2 = rng.normal(size=(M, 128)).astype(np.float32)
    B2 = rng.normal(size=(K, 128)).astype(np.float32)
    run_fused(csrk, M, K, 128, 512, rp, ci, v, A2, B2, np.ascontiguousarray(C[:, :512]), rows=rows)


# dot products longer than the 128 floats one launch of the tiled SDDMM kernel takes: pieces of 128, the later ones
# added to P (132 -> 128 + 4; 300 -> 128 + 128 + 44); in place the general kernels run (every piece needs vals)
@pytest.mark.parametrize("M,K,D", [(64, 64, 132), (333, 417, 256), (1000, 1300, 300), (65, 3000, 512), (2100, 300, 1024)])
@pytest.mark.parametrize("p", [0.05, 0.4])
def test_sddmm_long_dot_products_go_in_pieces(csrk, M, K, D, p):
    rng = np.random.default_rng(M + K + D)
    rp, ci = inputs.bernoulli_csr(D, M, K, p)
    v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
    A = rng.normal(size=(M, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    run_sddmm(csrk, M, K, D, rp, ci, v, A, B)
    run_sddmm(csrk, M, K, D, rp, ci, None, A, B)
    run_sddmm(csrk, M, K, D, rp, ci, v, A, B, inplace=True)
    plan = csrk.csrk_plan_create(M, K, dev(rp), dev(ci))
    got = csrk.sddmm_csr_plan(plan, D, dev(v), dev(A), dev(B))
    assert torch.equal(got, csrk.sddmm_csr(M, K, D, dev(rp), dev(ci), dev(v), dev(A), dev(B)))
    csrk.csrk_plan_destroy(plan)
    r = M // 2
    ci2, v2 = ci.copy(), v.copy()
    ci2[rp[r]:rp[r + 1]] = ci2[rp[r]:rp[r + 1]][::-1]
    v2[rp[r]:rp[r + 1]] = v2[rp[r]:rp[r + 1]][::-1]
    run_sddmm(csrk, M, K, D, rp, ci2, v2, A, B)


def test_sddmm_long_dot_products_with_automatic_kernel_choice(csrk, monkeypatch):
    monkeypatch.setenv("CSRK_KTILE", "1")
    M, K, D = 8192, 4096, 256
    rng = np.random.default_rng(9)
    rp, ci = inputs.bernoulli_csr(4, M, K, 0.2)
    v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
    A = rng.normal(size=(M, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    run_sddmm(csrk, M, K, D, rp, ci, v, A, B, rows=np.unique(np.concatenate([np.arange(0, M, 13), [M - 4, M - 3, M - 2, M - 1]])).astype(np.int32))


def test_sddmm_in_place_on_unsorted_columns_where_the_tiled_kernel_would_be_tried(csrk):
    # 9 M cells: beyond the whole-row kernels' range, so an attempt with the tiled kernel is in reach.  In place it
    # would overwrite values that the general kernel needs when the columns turn out unsorted.
    M, K, D = 3000, 3000, 64
    rng = np.random.default_rng(1)
    rp, ci = inputs.bernoulli_csr(3, M, K, 0.3)
    v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
    for r in (5, 500, M - 1):
        ci[rp[r]:rp[r + 1]] = ci[rp[r]:rp[r + 1]][::-1]
    A = rng.normal(size=(M, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    run_sddmm(csrk, M, K, D, rp, ci, v, A, B)
    run_sddmm(csrk, M, K, D, rp, ci, v, A, B, inplace=True)
    # sorted again: in place through a plan (tiled kernel), and without one (general kernel)
    rp, ci = inputs.bernoulli_csr(3, M, K, 0.3)
    run_sddmm(csrk, M, K, D, rp, ci, v, A, B, inplace=True)
    plan = csrk.csrk_plan_create(M, K, dev(rp), dev(ci))
    d_v = dev(v)
    got = csrk.sddmm_csr_plan(plan, D, d_v, dev(A), dev(B), P=d_v)
    assert got.data_ptr() == d_v.data_ptr()
    assert torch.equal(got, csrk.sddmm_csr(M, K, D, dev(rp), dev(ci), dev(v), dev(A), dev(B)))
    csrk.csrk_plan_destroy(plan)


def test_row_rotation_of_the_rotated_multiply_add(csrk):
    # The tiled SDDMM kernel and FusedMM's score stage walk a row of B in rotated order and take the matching piece
    # of A through the row rotation of the multiply-add's cross-lane operand: rotation by S must hand lane l the
    # operand of lane (l - S) mod 16 of its row of 16 lanes, for every S the kernels use.
    got = csrk.csrk_debug_row_rotation().cpu().numpy()
    lanes = np.arange(64)
    for S in range(16):
        want = (lanes & ~15) | ((lanes - S) & 15)
        np.testing.assert_array_equal(got[S], want.astype(np.float32), err_msg=f"rotation by {S}")


def test_phase_clock_build_computes_the_same_results(csrk):
    # the measuring builds of the 512-column kernels (csrk_tile_phases) are the production code plus cycle counters
    M, K, N, D = 1024, 2048, 512, 64
    rng = np.random.default_rng(77)
    rp, ci = inputs.bernoulli_csr(6, M, K, 0.2)
    v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
    A = rng.normal(size=(M, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    C = rng.normal(size=(K, N)).astype(np.float32)
    d_rp, d_ci, d_v = dev(rp), dev(ci), dev(v)
    cyc, tiles, O = csrk.csrk_tile_phases(csrk.CSRK_OP_SPMM, M, K, D, N, d_rp, d_ci, d_v, None, None, dev(C))
    assert tiles == K // 64 and cyc[4] > 0 and cyc[6] == 0 and all(c >= 0 for c in cyc)
    want, a = oracle.spmm(M, K, N, rp, ci, v, C)
    check(O.cpu().numpy(), want, a, "spmm, measuring build")
    cyc, tiles, O = csrk.csrk_tile_phases(csrk.CSRK_OP_FUSEDMM, M, K, D, N, d_rp, d_ci, d_v, dev(A), dev(B), dev(C))
    assert cyc[4] > 0 and cyc[6] > 0
    want, a = oracle.fusedmm(M, K, D, N, rp, ci, v, A, B, C)
    check(O.cpu().numpy(), want, a, "fusedmm, measuring build")
