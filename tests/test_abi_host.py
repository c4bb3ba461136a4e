"""CPU-side checks of the C-ABI library: it loads, exports every declared entry point,
and rejects malformed problems before touching a device."""
import ctypes as C
import os
import re
from dataclasses import replace

import numpy as np
import pytest

from paper_2504_17096_amd import binding, workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2504_17096_amd import build
    if build.is_stale():
        build.build()
    return binding.load_library()


def test_exports_every_declared_entry_point(lib):
    header = open(os.path.join(ROOT, "include", "sailor.h")).read()
    declared = set(re.findall(r"sailor_status\s+(sailor_\w+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_result_struct_layout_matches_header():
    assert C.sizeof(binding.sailor_result) == 96
    assert binding.sailor_result.mask.offset == 32
    assert binding.sailor_result.pool.offset == 84
    assert C.sizeof(binding.sailor_constraint) == 16


def _create(lib, prob):
    s, keep = binding.marshal_problem(prob)
    h = C.c_void_p()
    return lib.sailor_plan_create(C.byref(s), C.byref(h)), h


@pytest.mark.parametrize("mutate", [
    lambda p: replace(p, mb_values=np.array([2, 1], np.int32)),               # not ascending
    lambda p: replace(p, tp_values=np.array([0, 1, 2], np.int32)),            # non-positive
    lambda p: replace(p, partition_layers=p.partition_layers + 1),            # rows do not sum to L
    lambda p: replace(p, bandwidth=p.bandwidth * 0.0),                        # non-positive link
    lambda p: replace(p, t_fwd=-p.t_fwd),                                     # negative time
    lambda p: replace(p, avail=-np.ones_like(p.avail)),
    lambda p: replace(p, max_segments=4),
    lambda p: replace(p, global_batch=0),
    lambda p: replace(p, dp_values=np.arange(1, 40, dtype=np.int32)),          # too many degrees
    lambda p: replace(p, mem_capacity=np.full_like(p.mem_capacity, 2 ** 63)),  # would overflow
    lambda p: replace(p, price_per_hour=p.price_per_hour * np.nan),
])
def test_malformed_problems_are_rejected(lib, mutate):
    rc, h = _create(lib, mutate(W.config1()))
    assert rc == binding.SAILOR_EINVAL and not h.value


def test_null_arguments(lib):
    assert lib.sailor_plan_create(None, None) == binding.SAILOR_EINVAL
    assert lib.sailor_plan_destroy(None) == binding.SAILOR_OK
    assert lib.sailor_plan_num_candidates(None, None) == binding.SAILOR_EINVAL
    assert lib.sailor_plan_set_avail(None, None) == binding.SAILOR_EINVAL
    assert lib.sailor_best_plan(None, 0, None, None, None) == binding.SAILOR_EINVAL


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/libsailor.so")
    with pytest.raises(ImportError):
        binding.load_library()
