"""Randomised parity run: seeded random shapes, widths, densities and row-length mixes through every kernel
family (automatic choice, tiled kernels forced, general path only; K-split on and off; whole-row kernels
automatic, forced and off), each case checked element by element against the CPU oracle to the usual bar.
The shapes are small enough for the oracle but cross the 64-entry chunk, the tile heights, the 16 / 64-row
workgroup blocks and the width classes (4 .. 512, multiples of 4 and not)."""
import numpy as np
import pytest

import helpers
from paper_2311_00368_amd import inputs
from test_gpu_parity import csrk, run_fused, run_sddmm, run_spmm  # noqa: F401  (csrk is a fixture)

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

WIDTHS = [4, 8, 16, 32, 36, 64, 100, 128, 132, 256, 260, 384, 512]
CASES_PER_SEED = 40


def random_case(seed, c):
    """Case number c of a seed: environment settings, sizes, pattern and operands."""
    rng = np.random.default_rng(seed * 100000 + c)
    mode = ["1", "2", "2", "3"][c % 4]
    ksplit = ["1", "1", "2"][c % 3]
    rows_mode = ["1", "2", "1", "3", "2"][c % 5]
    M = int(rng.choice([1, 17, 64, 65, 200, 500, 1024, 1500, 2048, 3000, 4096, 5000]))
    K = int(rng.choice([1, 63, 64, 65, 130, 500, 1024, 2048, 3000, 4096, 6000]))
    N = int(rng.choice(WIDTHS))
    D = int(rng.choice([4, 16, 32, 60, 64, 68, 128]))
    p = float(rng.choice([0.0, 0.01, 0.05, 0.1, 0.2, 0.3, 0.6, 1.0]))
    if M * K * p > 4e6:
        p = 4e6 / (M * K)
    kind = c % 5
    what = f"seed {seed} case {c}: KTILE={mode} KSPLIT={ksplit} ROWS={rows_mode} M={M} K={K} N={N} D={D} p={p:.3f} kind={kind}"
    if kind < 3:
        rp, ci = inputs.bernoulli_csr(c + 7, M, K, p)
    else:
        # mixed row lengths: empty, single, short, about K*p, one chunk and a bit, full; sorted; repeats when kind == 4
        rows = []
        for _ in range(M):
            length = int(rng.choice([0, 1, 3, int(K * p) + 1, min(K, 70), K]))
            if M * K > 2e6:
                length = min(length, int(K * p) + 5)
            cols = rng.integers(0, K, size=length) if kind == 4 else rng.permutation(K)[:length]
            rows.append(sorted(int(x) for x in cols))
        rp, ci = helpers.csr_from_rows(rows, K)
    v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
    A = rng.normal(size=(M, D)).astype(np.float32)
    B = rng.normal(size=(K, D)).astype(np.float32)
    C = rng.normal(size=(K, N)).astype(np.float32)
    env = {"CSRK_KTILE": mode, "CSRK_KSPLIT": ksplit, "CSRK_ROWS": rows_mode}
    return what, env, (M, K, D, N), (rp, ci, v), (A, B, C)


@pytest.mark.parametrize("seed", [101, 102, 103, 104])
def test_random_shapes_all_kernel_families(csrk, monkeypatch, seed):
    for c in range(CASES_PER_SEED):
        what, env, (M, K, D, N), (rp, ci, v), (A, B, C) = random_case(seed, c)
        for name, value in env.items():
            monkeypatch.setenv(name, value)
        try:
            run_spmm(csrk, M, K, N, rp, ci, v, C)
            run_fused(csrk, M, K, D, N, rp, ci, v, A, B, C)
            if len(ci):
                run_sddmm(csrk, M, K, D, rp, ci, v, A, B)
        except AssertionError as e:
            raise AssertionError(f"{what}: {e}") from e


@pytest.mark.parametrize("seed", [301, 302])
def test_random_wide_outputs_and_long_dot_products(csrk, monkeypatch, seed):
    # widths beyond one launch of the tiled kernels (outputs over 512 columns, dot products over 128 floats and
    # over 64 with a wide output), every kernel-family setting, SDDMM also in place
    for c in range(12):
        rng = np.random.default_rng(seed * 1000 + c)
        env = {"CSRK_KTILE": ["2", "1", "2", "3"][c % 4], "CSRK_KSPLIT": ["1", "1", "2"][c % 3], "CSRK_ROWS": ["3", "1"][c % 2]}
        M = int(rng.choice([65, 300, 1024, 2100]))
        K = int(rng.choice([64, 700, 2048, 4100]))
        N = int(rng.choice([260, 516, 640, 768, 1024, 1500, 2048]))
        D = int(rng.choice([64, 72, 100, 128, 132, 256, 300]))
        p = float(rng.choice([0.02, 0.1, 0.3, 1.0]))
        if M * K * p > 1e6:
            p = 1e6 / (M * K)
        what = f"seed {seed} case {c}: {env} M={M} K={K} N={N} D={D} p={p:.3f}"
        for name, value in env.items():
            monkeypatch.setenv(name, value)
        rp, ci = inputs.bernoulli_csr(c + 11, M, K, p)
        v = rng.uniform(-1, 1, len(ci)).astype(np.float32)
        A = rng.normal(size=(M, D)).astype(np.float32)
        B = rng.normal(size=(K, D)).astype(np.float32)
        C = rng.normal(size=(K, N)).astype(np.float32)
        try:
            run_spmm(csrk, M, K, N, rp, ci, v, C)
            run_fused(csrk, M, K, D, N, rp, ci, v, A, B, C)
            if len(ci):
                run_sddmm(csrk, M, K, D, rp, ci, v, A, B)
                run_sddmm(csrk, M, K, D, rp, ci, v, A, B, inplace=True)
        except AssertionError as e:
            raise AssertionError(f"{what}: {e}") from e
