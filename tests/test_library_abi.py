"""The C-ABI library loads and exports every function the public header declares (no GPU needed)."""
import ctypes as C
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "muxmatch.h")
LIB = os.path.join(ROOT, "paper_2303_13803_amd", "libmuxmatch.so")


def _declared_functions():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(mf_[a-z_]+)\s*\(", text)))


def test_header_declares_the_three_named_calls():
    names = _declared_functions()
    for must in ("mf_score_pairs", "mf_solve_assignment", "mf_schedule_round", "mf_check_certificate",
                 "mf_create", "mf_destroy"):
        assert must in names


def test_library_exports_every_declared_function():
    assert os.path.exists(LIB), "build the library first: python paper_2303_13803_amd/build.py"
    lib = C.CDLL(LIB)
    for name in _declared_functions():
        assert hasattr(lib, name), f"{name} is declared in muxmatch.h but not exported"


def test_binding_lists_the_same_functions():
    from paper_2303_13803_amd import binding
    assert sorted(binding.EXPORTS) == _declared_functions()


def test_error_strings_and_argument_checks_without_a_device():
    from paper_2303_13803_amd import binding
    lib = binding.raw_library()
    for code in (0, -1, -2, -3, -4, -5, -6):
        assert binding.strerror(code) not in ("", "unknown error")
    assert binding.strerror(-99) == "unknown error"
    handle = C.c_void_p()
    assert lib.mf_create(None, 0, None, 4, 4) == binding.ERR_ARG              # no place for the handle
    assert lib.mf_create(C.byref(handle), 0, None, 4, 1 << 20) == binding.ERR_ARG   # beyond the id field of a packed word
    assert lib.mf_create(C.byref(handle), 0, None, 0, 4) == binding.ERR_ARG
    assert lib.mf_destroy(None) == binding.ERR_ARG
    assert lib.mf_set_option(None, b"theta", 8) == binding.ERR_ARG


def test_result_struct_matches_the_header():
    from paper_2303_13803_amd import binding
    text = open(HEADER).read()
    body = text[text.index("/* Filled on the host by the solving calls. */"):]
    body = body[:body.index("} mf_result;")]
    fields = re.findall(r"^\s*(?:int64_t|int32_t|float)\s+(\w+);", body, flags=re.M)
    assert fields == [name for name, _ in binding.Result._fields_]
