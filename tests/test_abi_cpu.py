"""CPU-side checks of the C ABI: the library loads, exports every symbol the header declares,
and validates arguments before touching a device."""
import ctypes as C
import os
import re

import pytest

from paper_1502_00512_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_1502_00512_amd.build import build
        build()
    return binding.load()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "rnnlm.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(rnnlm_[a-z_]+)\s*\(", header))
    assert declared == set(binding.SYMBOLS)
    for name in declared:
        assert hasattr(lib, name), name


def test_workspace_bytes_validates_config(lib):
    assert binding.rnnlm_workspace_bytes(1000, 64, 4, 8, binding.RNNLM_FP32) > 0
    assert binding.rnnlm_workspace_bytes(0, 64, 4, 8, binding.RNNLM_FP32) == 0
    assert binding.rnnlm_workspace_bytes(1000, 64, 4, 8, 7) == 0
    assert binding.rnnlm_workspace_bytes(1000, -1, 4, 8, binding.RNNLM_BF16_FP32MASTER) == 0
    small = binding.rnnlm_workspace_bytes(1000, 64, 4, 8, binding.RNNLM_BF16_FP32MASTER)
    big = binding.rnnlm_workspace_bytes(64000, 1024, 128, 20, binding.RNNLM_BF16_FP32MASTER)
    assert 0 < small < big < 4 << 30


def test_init_rejects_bad_arguments_without_a_device(lib):
    cfg = binding.rnnlm_config(100, 16, 2, 4, 0, 0)
    out = C.c_void_p()
    assert lib.rnnlm_init(None, None, C.byref(out)) == -1
    buf = binding.rnnlm_buffers(0, 0, 0, 0, 0, 0, 0)
    assert lib.rnnlm_init(C.byref(cfg), C.byref(buf), C.byref(out)) == -1 and not out.value
    assert lib.rnnlm_init(C.byref(cfg), C.byref(buf), None) == -1
    # null handle on every call that takes one
    assert lib.rnnlm_forward_logprob(None, None, None, 1, None, None) == -1
    assert lib.rnnlm_train_chunk(None, None, None, 1, 0.1, None, None, None) == -1
    assert lib.rnnlm_reset_state(None, None) == -1
    assert lib.rnnlm_check(None, None) == -1
    lib.rnnlm_free(None)


def test_status_strings(lib):
    assert binding.status_string(0) == "ok"
    assert "token" in binding.status_string(-2)
    assert binding.status_string(-99) == "unknown status"
