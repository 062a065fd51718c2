"""The C-ABI library loads and exports every symbol include/*.h declares (liec.h: the method's calls,
liec_testing.h: testing and measurement aids); argument checks that need no GPU return the documented
status codes."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", n) for n in ("liec.h", "liec_testing.h")]
AIDS = ("liec_force_search_mode", "liec_get_search_state", "liec_set_search_wait", "liec_set_group_bitmap", "liec_set_gather_batching", "liec_profile_begin",
        "liec_profile_end", "liec_device_copy")


def _declared_in(header):
    text = open(header).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(liec_[a-z0-9_]+)\s*\(", text)))


def _declared_functions():
    return sorted(set(n for h in HEADERS for n in _declared_in(h)))


@pytest.fixture(scope="module")
def lib():
    import paper_2402_11857_amd as pkg

    if not os.path.exists(pkg.library_path()):
        from paper_2402_11857_amd import _build

        _build.build_library()
    return pkg.lib()


def test_header_declares_the_north_star_calls():
    names = _declared_functions()
    for required in ("liec_create", "liec_step", "liec_destroy"):
        assert required in names


def test_every_declared_symbol_is_exported(lib):
    for name in _declared_functions():
        assert hasattr(lib, name), f"{name} is declared in include/ but not exported"


def test_the_method_header_holds_no_testing_aids():
    """liec.h declares the method's calls; the aids the tests and the measurement script use live in
    liec_testing.h."""
    method, aids = _declared_in(HEADERS[0]), _declared_in(HEADERS[1])
    for name in AIDS:
        assert name in aids and name not in method


def test_status_strings(lib):
    assert lib.liec_status_string(0) == b"ok"
    assert b"invalid" in lib.liec_status_string(1)


@pytest.mark.parametrize("args", [
    (0, 16, 1, 0, 0.1),          # N < 1
    (2, 0, 1, 0, 0.1),           # d < 1
    (2, 1 << 31, 1, 0, 0.1),     # d too large
    (2, 16, 7, 0, 0.1),          # unknown operator
    (2, 16, 2, 0, 0.1),          # top-k with k = 0
    (2, 16, 2, 17, 0.1),         # top-k with k > d
    (2, 16, 1, 0, float("nan")), # lr not finite
    (65536, 16, 1, 0, 0.1),      # more rows than a launch grid's y dimension holds
    (2, 16, 4, 0, 0.1),          # random-k with k = 0
    (2, 16, 4, 17, 0.1),         # random-k with k > d
])
def test_create_rejects_bad_arguments_before_touching_the_device(lib, args):
    h = ctypes.c_void_p()
    N, d, comp, k, lr = args
    assert lib.liec_create(ctypes.byref(h), N, d, comp, k, lr) == 1
    assert not h.value


def test_null_handles_are_rejected_or_ignored(lib):
    assert lib.liec_step(None, None, None, None) == 1
    assert lib.liec_set_lr(None, 0.1) == 1
    assert lib.liec_set_random(None, 1, 2) == 1
    assert lib.liec_force_search_mode(None, 0) == 1
    assert lib.liec_set_search_wait(None, 0) == 1
    assert lib.liec_get_search_state(None, 0, None) == 1
    assert lib.liec_set_group_bitmap(None, 0) == 1
    assert lib.liec_set_gather_batching(None, 0) == 1
    assert lib.liec_l2_norm(None, None, 1, None) == 1
    assert lib.liec_iteration(None, 0, 4, None, None, None) == 1
    assert lib.liec_iteration(None, 0, 1, None, None, None) == 1      # a period of 1 would never compress
    assert lib.liec_scratch_bytes(None) == 0
    lib.liec_destroy(None)
    assert lib.liec_create(None, 1, 1, 0, 0, 0.1) == 1


def test_binding_refuses_to_run_without_a_gpu():
    import torch

    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    from paper_2402_11857_amd import LiecContext

    with pytest.raises(RuntimeError):
        LiecContext(2, 16, "sign")


def test_product_never_imports_the_oracle():
    pkg_dir = os.path.join(ROOT, "paper_2402_11857_amd")
    for base, _, files in os.walk(pkg_dir):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                src = open(os.path.join(base, f)).read()
                assert "oracle" not in src.lower(), f"{f} mentions the oracle"


def test_header_is_plain_c(tmp_path):
    """include/liec.h must be usable from C: no C++ types, every declaration a plain C prototype."""
    import subprocess

    src = tmp_path / "use_header.c"
    src.write_text('#include "liec.h"\n#include "liec_testing.h"\n'
                   "int main(void) {\n"
                   "    liec_ctx *c = 0;\n"
                   "    liec_info info;\n"
                   "    liec_status (*step)(liec_ctx *, const float *, float *, float *) = liec_step;\n"
                   "    (void)c; (void)info; (void)step;\n"
                   "    return (int)LIEC_COMP_RANDK - 4;\n"
                   "}\n")
    inc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
    run = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only", "-I", inc, str(src)],
                         capture_output=True, text=True)
    assert run.returncode == 0, run.stderr
