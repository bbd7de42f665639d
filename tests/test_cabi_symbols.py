"""The C-ABI library loads on a machine without a GPU and exports every function that
include/csrk.h declares.  No compute call is made here."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "csrk.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(?:csrk_status|const\s+char\s*\*)\s*(\w+)\s*\(", text)
    assert names
    return names


def test_header_lists_the_three_operations():
    names = declared_functions()
    for fn in ("spmm_csr", "sddmm_csr", "fusedmm_csr"):
        assert fn in names


def test_library_exports_every_declared_symbol():
    from paper_2311_00368_amd import binding
    lib = binding.load()
    for fn in declared_functions():
        assert hasattr(lib, fn), f"libcsrk.so does not export {fn}"
    assert binding.csrk_version().startswith("csrk ")
    assert binding.csrk_last_error() == ""


def test_binding_has_same_names():
    from paper_2311_00368_amd import binding
    for fn in declared_functions():
        assert callable(getattr(binding, fn)), f"binding lacks {fn}"


def test_product_path_does_not_touch_the_oracle():
    pkg = os.path.join(ROOT, "paper_2311_00368_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h", ".c")):
                src = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in src and "from oracle" not in src and "csr_oracle" not in src, f


def test_argument_errors_are_reported_before_any_device_work():
    # calls that must fail on their arguments alone: they return a status and a message without touching a GPU
    from paper_2311_00368_amd import binding
    lib = binding.load()
    null = ctypes.c_void_p(None)
    invalid = 1     # CSRK_INVALID_ARG
    assert lib.spmm_csr(-1, 4, 4, null, null, null, null, null, null) == invalid
    assert "spmm_csr" in binding.csrk_last_error()
    assert lib.sddmm_csr(4, -2, 4, null, null, null, null, null, null, null) == invalid
    assert lib.fusedmm_csr(4, 4, 4, -1, null, null, null, null, null, null, null, null) == invalid
    assert lib.spmm_csr(4, 4, 4, null, null, null, null, null, null) == invalid          # rowptr and O are NULL
    assert lib.spmm_csr(0, 4, 4, null, null, null, null, null, null) == 0                # no rows: nothing to do
    assert lib.csrk_plan_create(4, 4, null, null, null, None) == invalid                 # nowhere to put the plan
    assert lib.csrk_plan_destroy(null) == 0
    assert lib.csrk_plan_info(null, None, None, None) == invalid
    assert lib.spmm_csr_plan(null, 4, null, null, null, null) == invalid
    assert lib.sddmm_csr_plan(null, 4, null, null, null, null, null) == invalid
    assert lib.fusedmm_csr_plan(null, 4, 4, null, null, null, null, null, null) == invalid
    assert "plan" in binding.csrk_last_error()
