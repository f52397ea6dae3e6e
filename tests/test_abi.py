"""The C-ABI library loads and exports what include/remoe.h declares; argument errors are reported.

No GPU work is launched here: every call below fails validation on the host before any kernel.
"""
import ctypes
import os
import re

import pytest

import paper_2605_27081_amd as remoe
from paper_2605_27081_amd import build as hip_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not hip_build.is_built():
        hip_build.build()
    return remoe.load_library()


def _declared_functions():
    names = []
    inc = os.path.join(ROOT, "include")
    for header in sorted(os.listdir(inc)):
        if not header.endswith(".h"):
            continue
        text = open(os.path.join(inc, header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names += re.findall(r"\b([a-z_0-9]+)\s*\([^;{}]*\)\s*;", text)
    return sorted(set(names))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert {"moe_route", "moe_forward", "trace_reuse", "lru_simulate", "remoe_workspace_bytes",
            "remoe_last_error", "remoe_version", "moe_decode", "moe_decode_static", "remoe_profile_enable",
            "remoe_copy_probe"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in remoe.h but not exported"


def test_version_and_workspace_size(lib):
    assert remoe.remoe_version() >= 100
    d = remoe.LayerDesc(2048, 128, 768, 8, 1, 0, 0, 1)
    small, big = remoe.remoe_workspace_bytes(d, 128), remoe.remoe_workspace_bytes(d, 65536)
    assert 0 < small < big
    # at least the activations and the per-(token, expert) rows must fit
    assert big >= 65536 * 8 * (768 + 2048) * 2
    assert big % 256 == 0


@pytest.mark.parametrize("fields,fragment", [
    ((2048, 0, 768, 8, 1, 0, 0, 1), "n_experts"),
    ((2048, 129, 768, 8, 1, 0, 0, 1), "n_experts"),
    ((2048, 128, 768, 9, 1, 0, 0, 1), "top_k"),
    ((2048, 4, 768, 5, 1, 0, 0, 1), "top_k"),
    ((2050, 128, 768, 8, 1, 0, 0, 1), "hidden"),
    ((2048, 128, 768, 8, 1, 0, 0, 7), "dtype"),
    ((2048, 128, 700, 8, 1, 0, 0, 1), "inter"),
    ((2048, 128, 768, 8, 1, 0, 1, 1), "shared_gate"),
    ((2048, 128, 768, 8, 2, 0, 0, 1), "renorm"),
])
def test_bad_descriptors_are_rejected(lib, fields, fragment):
    d = remoe.LayerDesc(*fields)
    assert lib.remoe_workspace_bytes(ctypes.byref(d), 16) == 0
    assert fragment in remoe.remoe_last_error()
    st = lib.moe_forward(ctypes.byref(d), None, 16, *([None] * 12), 0, None)
    assert st < 0


def test_null_and_range_arguments_are_rejected(lib):
    d = remoe.LayerDesc(256, 16, 128, 2, 0, 0, 0, 0)
    assert lib.moe_route(ctypes.byref(d), None, 8, None, None, None, None, None, None) == -1
    assert "NULL" in remoe.remoe_last_error()
    assert lib.moe_route(None, None, 8, None, None, None, None, None, None) == -1
    assert lib.moe_route(ctypes.byref(d), None, -1, None, None, None, None, None, None) == -1
    assert lib.moe_forward(ctypes.byref(d), None, 8, *([None] * 12), 0, None) == -1
    assert lib.trace_reuse(None, 2, 5, 4, 16, None, None, None) == -1
    assert lib.trace_reuse(None, 2, 5, 0, 16, None, None, None) == -1
    assert lib.trace_reuse(None, 2, 5, 4, 129, None, None, None) == -1
    assert lib.lru_simulate(None, 1, 1, 4, 16, 0, 0, 0, None, None, None, None, None) == -1
    assert "capacity" in remoe.remoe_last_error()
    assert lib.lru_simulate(None, 1, 1, 4, 16, 4, 0, -1, None, None, None, None, None) == -1
    assert lib.lru_simulate(None, 1, 1 << 24, 4, 16, 4, 0, 0, None, None, None, None, None) == -1
    # empty problems are fine and launch nothing
    assert lib.moe_route(ctypes.byref(d), None, 0, None, None, None, None, None, None) == 0
    assert lib.trace_reuse(None, 0, 5, 4, 16, None, None, None) == 0
    assert lib.lru_simulate(None, 0, 5, 4, 16, 4, 0, 0, None, None, None, None, None) == 0


def test_binding_refuses_host_tensors(lib):
    import torch
    d = remoe.LayerDesc(256, 16, 128, 2, 0, 0, 0, 0)
    x = torch.zeros(4, 256)
    with pytest.raises(remoe.RemoeError):
        remoe.moe_route(d, x, x, x, x)
