"""CPU-side checks of the C-ABI library: it loads, exports what the header declares, and rejects bad
arguments before touching the GPU."""
import ctypes
import os
import re

import pytest

import paper_2412_00061_amd as pkg
from paper_2412_00061_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "ctcspec.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    # every function declaration of the header: a return type at the start of a line, a name, "("
    return sorted(set(re.findall(r"^(?:int|void|size_t|const char\*)\s+(\w+)\s*\(", text, flags=re.M)))


def test_library_exports_every_declared_symbol():
    lib = pkg.load_library()
    names = _declared_functions()
    assert {"ctc_draft_topk", "ctc_collapse_tree", "tree_verify_attn", "accept_longest", "verify_head_argmax",
            "kv_commit"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert set(binding.EXPORTS) == set(names)


def test_create_rejects_bad_limits_without_gpu():
    lib = pkg.load_library()
    handle = ctypes.c_void_p()
    assert lib.ctcspec_create(ctypes.byref(handle), None, None) == -1
    bad = binding._Limits(1, 9, 4, 100, 128, 4, 16)  # T = 9 > compiled maximum
    assert lib.ctcspec_create(ctypes.byref(handle), None, ctypes.byref(bad)) == -2
    assert handle.value is None
    assert b"limits" in lib.ctcspec_last_error(None)
    zero = binding._Limits(0, 4, 4, 100, 128, 4, 16)
    assert lib.ctcspec_create(ctypes.byref(handle), None, ctypes.byref(zero)) == -1


def test_stage_calls_reject_null_context():
    lib = pkg.load_library()
    assert lib.ctc_draft_topk(None, 0, None, None, None, 1, 1, 1, 1, 1, None, None, None, None) == -1
    assert lib.accept_longest(None, None, None, None, None, None, 1, 1, 1, None, None, None, None) == -1
    lib.ctcspec_destroy(None)  # must be a no-op


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_LIB", None)
    monkeypatch.setattr(binding, "_HERE", str(tmp_path))
    with pytest.raises(binding.CtcspecError, match="no CPU fallback"):
        binding.load_library()
