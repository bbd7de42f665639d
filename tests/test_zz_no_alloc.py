"""fusedmm_csr_static, the entry point for callers that cannot allocate: same results as fusedmm_csr (both held to
|gpu - oracle| <= 1e-5 * sum|terms|, and to each other), on calls in a row that share the one static scratch area -
the second with a smaller input, then shapes that take other kernels - and a clear refusal of what does not fit."""
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
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run_both(csrk, M, K, D, N, rp, ci, seed, what):
    rng = np.random.default_rng(seed)
    v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
    A = rng.normal(size=(M, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    C = rng.normal(size=(K, N)).astype(np.float32)
    d = [dev(x) for x in (rp, ci, v, A, B, C)]
    O = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    csrk.fusedmm_csr_static(M, K, D, N, *d, O)
    torch.cuda.synchronize()
    plain = csrk.fusedmm_csr(M, K, D, N, *d)
    torch.cuda.synchronize()
    want, a = oracle.fusedmm(M, K, D, N, rp, ci, v, A, B, C)
    for name, got in (("fusedmm_csr_static", O), ("fusedmm_csr", plain)):
        ok, worst = oracle.within_tolerance(got.cpu().numpy(), want, a, REL_TOL)
        assert ok, f"{what}: {name}: worst |err|/sum|terms| = {worst:.3e}"
    diff = np.abs(O.cpu().numpy().astype(np.float64) - plain.cpu().numpy().astype(np.float64))
    assert np.all(diff <= 2 * REL_TOL * a), f"{what}: the two entry points differ by more than the bar allows"
    assert np.array_equal(d[0].cpu().numpy(), rp) and np.array_equal(d[1].cpu().numpy(), ci)


def test_static_scratch_calls_in_a_row(csrk):
    # 1: skewed rows - the general kernel in equal shares, partial rows through the scratch area and the combine step
    M, K = 4096, 4096
    rp, ci = inputs.lognormal_csr(3, M, K, 400.0, 1.0)
    run_both(csrk, M, K, 64, 64, rp, ci, 1, "first call (skewed 4096^2)")
    # 2: a smaller input right behind it on the same area
    M, K = 1500, 2000
    rp, ci = inputs.bernoulli_csr(4, M, K, 0.1)
    run_both(csrk, M, K, 32, 128, rp, ci, 2, "second call (smaller)")
    # 3: a short matrix whose reduction dimension is cut into ranges: partial outputs in the area, added up afterwards
    M, K = 1024, 8192
    rp, ci = inputs.bernoulli_csr(5, M, K, 0.2)
    run_both(csrk, M, K, 64, 256, rp, ci, 3, "third call (K cut into ranges)")
    # 4: the wide tiled kernel, then unsorted columns in a shape that tries it (the general kernel must take over)
    M, K = 16384, 2048
    rp, ci = inputs.bernoulli_csr(6, M, K, 0.2)
    run_both(csrk, M, K, 64, 512, rp, ci, 4, "fourth call (wide tiled kernel)")
    ci2 = ci.copy()
    ci2[rp[70]:rp[71]] = ci2[rp[70]:rp[71]][::-1]
    run_both(csrk, M, K, 64, 512, rp, ci2, 5, "fifth call (unsorted row)")
    run_both(csrk, M, K, 64, 512, rp, ci, 6, "sixth call (sorted again)")
    # empty matrix and empty rows
    rp0 = np.zeros(33, dtype=np.int32)
    run_both(csrk, 32, 100, 16, 64, rp0, np.zeros(0, dtype=np.int32), 7, "no entries")


def test_static_scratch_refuses_what_does_not_fit(csrk):
    M, K, D, N = 256, 256, 16, 1024
    rp, ci = inputs.bernoulli_csr(1, M, K, 0.1)
    rng = np.random.default_rng(0)
    v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
    O = torch.zeros((M, N), dtype=torch.float32, device="cuda")
    with pytest.raises(csrk.CsrkError) as e:
        csrk.fusedmm_csr_static(M, K, D, N, dev(rp), dev(ci), dev(v), dev(rng.normal(size=(M, D)).astype(np.float32)),
                                dev(rng.normal(size=(K, D)).astype(np.float32)),
                                dev(rng.normal(size=(K, N)).astype(np.float32)), O)
    assert e.value.code == 4 and "fusedmm_csr_static" in str(e.value) and "bytes" in str(e.value)
    assert torch.count_nonzero(O).item() == 0       # nothing was enqueued
