"""The library's choice of kernel family replayed on the CPU against a recorded sweep (profiles/sweep72_threeway.md:
the paper's 72 grid points, every operation timed with the family forced three ways, with automatic choice, and
planned).  `csrk_explain_choice` is the choice function of the compute calls themselves, callable without a device.

Guards: (1) the families it names today are the ones recorded - a change to a threshold that moves a grid point to
another family fails here until the sweep is run again; (2) the family named is within 10 % of the best forced
one at every point; (3) the automatic calls as measured were within 10 % of the best forced one, plus 6 us for an
unplanned call (what a turned-down tiled attempt costs: the row analysis and a launch that stands down) and 3 us for
a planned one (calls of 13-30 us, timer resolution)."""

import os

import pytest

from paper_2311_00368_amd import binding

TABLE = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "profiles", "sweep72_threeway.md")
OPS = {"spmm": binding.CSRK_OP_SPMM, "sddmm": binding.CSRK_OP_SDDMM, "fusedmm": binding.CSRK_OP_FUSEDMM}
TILED = ("tiled narrow", "tiled wide", "tiled SDDMM")


def recorded():
    rows, cus = [], None
    with open(TABLE) as f:
        for line in f:
            cells = [c.strip() for c in line.strip().strip("|").split("|")]
            if len(cells) == 14 and cells[0] == "shape":
                cus = int(cells[12].split("(")[1].split()[0])
            if len(cells) == 14 and cells[1].isdigit():
                rows.append(dict(shape=cells[0], M=int(cells[1]), K=int(cells[2]), N=int(cells[3]), nnz=int(cells[4]),
                                 longest=int(cells[5]), op=cells[6], auto=float(cells[7]), tiled=float(cells[8]),
                                 rows=float(cells[9]), shares=float(cells[10]), planned=float(cells[11]),
                                 family=cells[12], family_planned=cells[13]))
    return rows, cus


def test_the_table_is_complete():
    rows, cus = recorded()
    assert cus == 256
    assert len(rows) == 72 * 3
    assert {r["op"] for r in rows} == set(OPS)


def test_choice_function_names_the_recorded_families():
    rows, cus = recorded()
    for r in rows:
        for planned, key in ((False, "family"), (True, "family_planned")):
            fam = binding.csrk_explain_choice(OPS[r["op"]], cus, r["M"], r["K"], r["N"], r["N"], r["nnz"], r["longest"], planned)
            assert binding.FAMILY_NAMES[fam] == r[key], (r["shape"], r["op"], planned)


def forced_time_of(family, r):
    # the general kernels' whole-row branch has no forced run of its own: it lies between the whole-row kernels and
    # equal shares, the better of which stands in for it
    return r["tiled"] if family in TILED else min(r["rows"], r["shares"])


def test_chosen_family_is_within_ten_percent_of_the_best_forced_one():
    rows, _ = recorded()
    for r in rows:
        best = min(r["tiled"], r["rows"], r["shares"])
        assert forced_time_of(r["family"], r) <= 1.10 * best + 6.0, (r["shape"], r["op"], r)
        assert forced_time_of(r["family_planned"], r) <= 1.10 * best + 3.0, (r["shape"], r["op"], r)


def test_automatic_calls_were_within_ten_percent_of_the_best_forced_one():
    rows, _ = recorded()
    for r in rows:
        best = min(r["tiled"], r["rows"], r["shares"])
        assert r["auto"] <= 1.10 * best + 6.0, (r["shape"], r["op"], r)
        assert r["planned"] <= 1.10 * best + 3.0, (r["shape"], r["op"], r)


@pytest.mark.parametrize("planned", [False, True])
def test_choice_at_the_benchmark_shapes(planned):
    # 16384^2 / 20 %: the wide tiled kernels and tiled SDDMM; the skewed 8192^2 pattern: equal shares at 64 columns,
    # the wide tiled kernels (unplanned) or the plan's schedule at 512
    cus, M, nnz = 256, 16384, 53696561
    assert binding.FAMILY_NAMES[binding.csrk_explain_choice(OPS["spmm"], cus, M, M, 512, 0, nnz, 3500, planned)] == "tiled wide"
    assert binding.FAMILY_NAMES[binding.csrk_explain_choice(OPS["fusedmm"], cus, M, M, 512, 64, nnz, 3500, planned)] == "tiled wide"
    assert binding.FAMILY_NAMES[binding.csrk_explain_choice(OPS["sddmm"], cus, M, M, 0, 64, nnz, 3500, planned)] == "tiled SDDMM"
    M, nnz, longest = 8192, 6618785, 8192
    assert binding.FAMILY_NAMES[binding.csrk_explain_choice(OPS["fusedmm"], cus, M, M, 64, 64, nnz, longest, planned)] == "general, equal shares"
    wide = binding.FAMILY_NAMES[binding.csrk_explain_choice(OPS["fusedmm"], cus, M, M, 512, 64, nnz, longest, planned)]
    assert wide == ("schedule" if planned else "tiled wide")


def test_choice_function_refuses_nonsense():
    with pytest.raises(Exception):
        binding.csrk_explain_choice(99, 256, 1024, 1024, 64, 64, 1000, 10)
    with pytest.raises(Exception):
        binding.csrk_explain_choice(OPS["spmm"], 0, 1024, 1024, 64, 64, 1000, 10)
    with pytest.raises(Exception):
        binding.csrk_explain_choice(OPS["spmm"], 256, 0, 1024, 64, 64, 1000, 10)
