"""The calls that bring their own scratch: *_csr_ws on a caller's workspace and planned calls on a plan's reserved
workspace.  Same arithmetic as the plain calls, so the same bar against the oracle; on top of that these calls must
share nothing (two streams, two workspaces, both right) and must be capturable in a HIP graph (they allocate
nothing and never synchronise), replayed several times with other work in between."""
import numpy as np
import pytest

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


def workspace(csrk, M, K, N, D, poison=True):
    nbytes = max(csrk.csrk_workspace_bytes(op, M, K, N, D)
                 for op in (csrk.CSRK_OP_SPMM, csrk.CSRK_OP_SDDMM, csrk.CSRK_OP_FUSEDMM))
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    if poison:
        ws.fill_(0xFF)      # the contents on entry must not matter: all-ones words are NaNs and raised flags
    assert ws.data_ptr() % 256 == 0
    return ws


def operands(rng, M, K, D, N, nnz):
    v = rng.uniform(-1, 1, nnz).astype(np.float32)
    A = rng.normal(size=(M, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    C = rng.normal(size=(K, N)).astype(np.float32)
    return v, A, B, C


# (M, K, density, D, N): whole rows, general kernels, narrow and wide tiled kernels, small M with K cut into ranges
SHAPES = [(512, 512, 0.1, 64, 64), (700, 900, 0.2, 7, 13), (4096, 4096, 0.1, 64, 256), (2048, 8192, 0.2, 64, 512),
          (3072, 4096, 0.3, 128, 128), (9000, 3000, 0.07, 128, 64), (16384, 4096, 0.2, 64, 512)]


@pytest.mark.parametrize("shape", SHAPES)
def test_workspace_calls_match_the_oracle(csrk, shape):
    M, K, p, D, N = shape
    rng = np.random.default_rng(M + 3 * K + N)
    rp, ci = inputs.bernoulli_csr(M % 91, M, K, p)
    v, A, B, C = operands(rng, M, K, D, N, len(ci))
    ws = workspace(csrk, M, K, N, D)
    d_rp, d_ci, d_v = dev(rp), dev(ci), dev(v)
    rows = np.unique(np.concatenate([np.arange(0, M, 13), np.arange(M - 4, M)])).astype(np.int32)
    for rep in range(2):        # a second call finds the workspace as the first one left it
        O = csrk.spmm_csr_ws(M, K, N, d_rp, d_ci, d_v, dev(C), ws)
        want, a = oracle.spmm(M, K, N, rp, ci, v, C, rows=rows)
        check(O.cpu().numpy()[rows], want, a, f"spmm_csr_ws {shape} call {rep}")
        F = csrk.fusedmm_csr_ws(M, K, D, N, d_rp, d_ci, d_v, dev(A), dev(B), dev(C), ws)
        want, a = oracle.fusedmm(M, K, D, N, rp, ci, v, A, B, C, rows=rows)
        check(F.cpu().numpy()[rows], want, a, f"fusedmm_csr_ws {shape} call {rep}")
        P = csrk.sddmm_csr_ws(M, K, D, d_rp, d_ci, d_v, dev(A), dev(B), ws)
        want, a = oracle.sddmm(M, K, D, rp, ci, v, A, B, rows=rows)
        sel = ~np.isnan(want)
        check(P.cpu().numpy()[sel], want[sel], a[sel], f"sddmm_csr_ws {shape} call {rep}")
    # same kernels as the plain calls where both analyse by a launch: identical bits
    if M > 8192:
        assert torch.equal(O, csrk.spmm_csr(M, K, N, d_rp, d_ci, d_v, dev(C)))


def test_workspace_calls_on_skewed_unsorted_and_edge_patterns(csrk):
    import helpers
    rng = np.random.default_rng(17)
    w = inputs.workload("fused8k_skew", scale=0.25)
    f = w.ops["fusedmm"]
    ws = workspace(csrk, w.M, w.K, 64, 64)
    F = csrk.fusedmm_csr_ws(w.M, w.K, 64, 64, dev(w.rowptr), dev(w.colidx), dev(w.vals), dev(f["A"]), dev(f["B"]), dev(f["C"]), ws)
    want, a = oracle.fusedmm(w.M, w.K, 64, 64, w.rowptr, w.colidx, w.vals, f["A"], f["B"], f["C"])
    check(F.cpu().numpy(), want, a, "fusedmm_csr_ws skewed")
    # unsorted columns in a shape that tries the tiled kernel: the general kernel behind it must take over
    M, K, D, N = 3000, 3000, 64, 128
    rp, ci = inputs.bernoulli_csr(3, M, K, 0.3)
    for r in (5, 500, M - 1):
        ci[rp[r]:rp[r + 1]] = ci[rp[r]:rp[r + 1]][::-1]
    v, A, B, C = operands(rng, M, K, D, N, len(ci))
    ws = workspace(csrk, M, K, N, D)
    for rep in range(2):
        O = csrk.spmm_csr_ws(M, K, N, dev(rp), dev(ci), dev(v), dev(C), ws)
        want, a = oracle.spmm(M, K, N, rp, ci, v, C)
        check(O.cpu().numpy(), want, a, "spmm_csr_ws unsorted")
        P = csrk.sddmm_csr_ws(M, K, D, dev(rp), dev(ci), dev(v), dev(A), dev(B), ws)
        want, a = oracle.sddmm(M, K, D, rp, ci, v, A, B)
        check(P.cpu().numpy(), want, a, "sddmm_csr_ws unsorted")
    # ... and right after it a sorted pattern on the same workspace: the raised flag must not linger
    rp, ci = inputs.bernoulli_csr(3, M, K, 0.3)
    O = csrk.spmm_csr_ws(M, K, N, dev(rp), dev(ci), dev(v), dev(C), ws)
    want, a = oracle.spmm(M, K, N, rp, ci, v, C)
    check(O.cpu().numpy(), want, a, "spmm_csr_ws sorted after unsorted")
    for name, M, K, rp, ci in helpers.edge_patterns(rng):
        v, A, B, C = operands(rng, M, K, 32, 128, len(ci))
        ws = workspace(csrk, M, K, 128, 32)
        O = csrk.spmm_csr_ws(M, K, 128, dev(rp), dev(ci), dev(v), dev(C), ws)
        want, a = oracle.spmm(M, K, 128, rp, ci, v, C)
        check(O.cpu().numpy(), want, a, f"spmm_csr_ws {name}")
        F = csrk.fusedmm_csr_ws(M, K, 32, 128, dev(rp), dev(ci), dev(v), dev(A), dev(B), dev(C), ws)
        want, a = oracle.fusedmm(M, K, 32, 128, rp, ci, v, A, B, C)
        check(F.cpu().numpy(), want, a, f"fusedmm_csr_ws {name}")


def test_workspace_too_small_or_misaligned_is_refused(csrk):
    M, K, N = 1024, 1024, 256
    rng = np.random.default_rng(2)
    rp, ci = inputs.bernoulli_csr(1, M, K, 0.1)
    v, A, B, C = operands(rng, M, K, 64, N, len(ci))
    need = csrk.csrk_workspace_bytes(csrk.CSRK_OP_SPMM, M, K, N)
    assert need >= 8192 * N * 4
    small = torch.empty(need // 2, dtype=torch.uint8, device="cuda")
    with pytest.raises(csrk.CsrkError) as e:
        csrk.spmm_csr_ws(M, K, N, dev(rp), dev(ci), dev(v), dev(C), small)
    assert e.value.code == 4 and "workspace" in str(e.value)
    tiny = torch.empty(64, dtype=torch.uint8, device="cuda")
    with pytest.raises(csrk.CsrkError) as e:
        csrk.sddmm_csr_ws(M, K, 64, dev(rp), dev(ci), dev(v), dev(A), dev(B), tiny)
    assert e.value.code == 4
    big = torch.empty(need + 256, dtype=torch.uint8, device="cuda")
    with pytest.raises(csrk.CsrkError) as e:
        csrk.spmm_csr_ws(M, K, N, dev(rp), dev(ci), dev(v), dev(C), big[16:])
    assert e.value.code == 1
    with pytest.raises(csrk.CsrkError):
        csrk.csrk_workspace_bytes(9, M, K, N)


def test_two_streams_with_two_workspaces_run_side_by_side(csrk):
    # Calls on different streams with different workspaces share nothing.  Two long-running calls (different
    # operations, different patterns) are enqueued alternately on two streams many times with no synchronisation
    # in between; every result is compared with the oracle afterwards.
    rng = np.random.default_rng(23)
    jobs = []
    for seed, (M, K, p, D, N) in enumerate([(6144, 8192, 0.2, 64, 512), (8192, 4096, 0.1, 64, 256)]):
        rp, ci = inputs.bernoulli_csr(40 + seed, M, K, p)
        v, A, B, C = operands(rng, M, K, D, N, len(ci))
        jobs.append(dict(M=M, K=K, D=D, N=N, rp=rp, ci=ci, v=v, A=A, B=B, C=C, d={k: dev(x) for k, x in
                         dict(rp=rp, ci=ci, v=v, A=A, B=B, C=C).items()}, ws=workspace(csrk, M, K, N, D),
                         stream=torch.cuda.Stream(), outs=[]))
    torch.cuda.synchronize()
    reps = 6
    for rep in range(reps):
        for j in jobs:
            d = j["d"]
            with torch.cuda.stream(j["stream"]):
                O = csrk.spmm_csr_ws(j["M"], j["K"], j["N"], d["rp"], d["ci"], d["v"], d["C"], j["ws"])
                F = csrk.fusedmm_csr_ws(j["M"], j["K"], j["D"], j["N"], d["rp"], d["ci"], d["v"], d["A"], d["B"], d["C"], j["ws"])
                j["outs"].append((O, F))
    torch.cuda.synchronize()
    for j in jobs:
        rows = np.unique(np.concatenate([np.arange(0, j["M"], 61), np.arange(j["M"] - 4, j["M"])])).astype(np.int32)
        so, sa = oracle.spmm(j["M"], j["K"], j["N"], j["rp"], j["ci"], j["v"], j["C"], rows=rows)
        fo, fa = oracle.fusedmm(j["M"], j["K"], j["D"], j["N"], j["rp"], j["ci"], j["v"], j["A"], j["B"], j["C"], rows=rows)
        for rep, (O, F) in enumerate(j["outs"]):
            check(O.cpu().numpy()[rows], so, sa, f"spmm on its own stream, call {rep}")
            check(F.cpu().numpy()[rows], fo, fa, f"fusedmm on its own stream, call {rep}")
            assert torch.equal(O, j["outs"][0][0]) and torch.equal(F, j["outs"][0][1])


@pytest.mark.parametrize("shape", [(16384, 4096, 0.2, 64, 512), (2048, 8192, 0.2, 64, 512), (8192, 8192, 0.05, 64, 64),
                                   (4096, 4096, 0.08, 64, 256)])
def test_planned_and_workspace_calls_replay_from_a_hip_graph(csrk, shape):
    # wide tiled kernel alone; K cut into ranges (tiled kernel + adding step); general kernel + combine step; uneven rows
    # with a wide output (the plan's schedule with its adding step; unplanned: the tiled kernel on its regular grid)
    M, K, p, D, N = shape
    rng = np.random.default_rng(M + K)
    if p < 0.1:
        rp, ci = inputs.lognormal_csr(7, M, K, p * K, 1.0)      # skewed rows: equal shares and partial rows
    else:
        rp, ci = inputs.bernoulli_csr(7, M, K, p)
    v, A, B, C = operands(rng, M, K, D, N, len(ci))
    d_rp, d_ci, d_v, d_A, d_B, d_C = dev(rp), dev(ci), dev(v), dev(A), dev(B), dev(C)
    plan = csrk.csrk_plan_create(M, K, d_rp, d_ci)
    csrk.csrk_plan_reserve(plan, N)
    ws = workspace(csrk, M, K, N, D)
    # eager results first (this also sets the kernels' launch attributes outside the capture)
    want_O = csrk.spmm_csr_plan(plan, N, d_v, d_C)
    want_F = csrk.fusedmm_csr_plan(plan, D, N, d_v, d_A, d_B, d_C)
    want_P = csrk.sddmm_csr_plan(plan, D, d_v, d_A, d_B)
    want_O2 = csrk.spmm_csr_ws(M, K, N, d_rp, d_ci, d_v, d_C, ws)
    torch.cuda.synchronize()
    so, sa = oracle.spmm(M, K, N, rp, ci, v, C)
    check(want_O.cpu().numpy(), so, sa, f"planned spmm on the plan's workspace {shape}")
    check(want_O2.cpu().numpy(), so, sa, f"spmm_csr_ws {shape}")
    fo, fa = oracle.fusedmm(M, K, D, N, rp, ci, v, A, B, C)
    check(want_F.cpu().numpy(), fo, fa, f"planned fusedmm on the plan's workspace {shape}")
    O = torch.zeros_like(want_O)
    F = torch.zeros_like(want_F)
    P = torch.zeros_like(want_P)
    O2 = torch.zeros_like(want_O)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        csrk.spmm_csr_plan(plan, N, d_v, d_C, O=O)
        csrk.sddmm_csr_plan(plan, D, d_v, d_A, d_B, P=P)
        csrk.fusedmm_csr_plan(plan, D, N, d_v, d_A, d_B, d_C, O=F)
        csrk.spmm_csr_ws(M, K, N, d_rp, d_ci, d_v, d_C, ws, O=O2)
    for replay in range(4):
        for t in (O, F, P, O2):
            t.fill_(float("nan"))
        ws.fill_(0xFF if replay % 2 else 0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(O, want_O), f"replay {replay}: planned spmm"
        assert torch.equal(P, want_P), f"replay {replay}: planned sddmm"
        assert torch.equal(F, want_F), f"replay {replay}: planned fusedmm"
        assert torch.equal(O2, want_O2), f"replay {replay}: spmm_csr_ws"
        # the program's own eager work between replays (same bits where planned and unplanned calls run the same
        # kernel; over a schedule the ranges of K are cut differently)
        eager = csrk.spmm_csr(M, K, N, d_rp, d_ci, d_v, d_C)
        if p < 0.1 and N > 128:
            check(eager.cpu().numpy(), so, sa, f"eager spmm between replays {shape}")
        else:
            assert torch.equal(eager, want_O)
    del g
    csrk.csrk_plan_destroy(plan)
