"""CPU-side checks of the C-ABI library: it loads, exports every declared entry point,
and rejects malformed problems before touching a device."""
import ctypes as C
import os
import subprocess
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


def test_microbenchmark_library_exports_what_its_header_declares(lib):
    from paper_2504_17096_amd import microbench
    header = open(os.path.join(ROOT, "include", "sailor_microbench.h")).read()
    declared = set(re.findall(r"int\s+(sailor_microbench_\w+)\s*\(", header))
    assert declared == set(microbench.EXPORTS) and len(declared) == 3
    mlib = microbench.load_library()
    for name in declared:
        assert getattr(mlib, name) is not None


def test_struct_layouts_match_the_header(tmp_path):
    """sizeof / offsetof as a C compiler sees the header against the ctypes mirrors."""
    fields = {"sailor_problem": ["n_layers", "per_segment_tp", "n_bw_coef", "mixed_types", "global_batch", "mb_values",
                                 "embed_params", "grad_bytes_per_param", "t_fwd", "egress_per_byte",
                                 "bw_poly"],
              "sailor_result": ["index", "iter_time_s", "mask", "pp", "mb_index", "cut", "pool",
                                "seg_tp", "seg_tp_index", "zone", "type_a", "type_b"],
              "sailor_constraint": ["bound", "has_bound"],
              "sailor_search_options": ["beam_width", "max_runs", "use_incumbent", "incumbent", "allow_split",
                                        "stage_tp"],
              "sailor_stage_plan": ["found", "exact", "pp", "partition", "mask", "peak_mem_bytes",
                                    "iter_time_s", "eval_cost", "expanded", "incumbent_used",
                                    "incumbent", "pool", "pool_b", "stage_tp_index"]}
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "sailor.h"', 'int main(void) {']
    for st, fl in fields.items():
        lines.append(f'printf("{st} %zu\\n", sizeof({st}));')
        for f in fl:
            lines.append(f'printf("{st}.{f} %zu\\n", offsetof({st}, {f}));')
    lines += ['return 0; }']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    out = dict(l.split() for l in subprocess.run([str(exe)], check=True, capture_output=True,
                                                 text=True).stdout.splitlines())
    for st, fl in fields.items():
        cls = getattr(binding, st)
        assert C.sizeof(cls) == int(out[st])
        for f in fl:
            assert getattr(cls, f).offset == int(out[f"{st}.{f}"]), (st, f)
    assert C.sizeof(binding.sailor_result) == 160 and binding.sailor_result.mask.offset == 32


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
    lambda p: replace(p, bw_poly=np.full((p.n_zones, p.n_zones, 2), np.inf)),  # not finite
    lambda p: replace(p, bw_poly=np.ones((p.n_zones, p.n_zones, 9))),          # too many coefficients
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


def test_product_sources_do_not_reach_into_the_oracle():
    # the checker and the product share nothing but the seeded input generators
    import pathlib
    import re
    root = pathlib.Path(__file__).resolve().parent.parent
    pkg = root / "paper_2504_17096_amd"
    sources = list(pkg.glob("*.py")) + [f for f in (pkg / "csrc").iterdir() if f.is_file()]
    sources.append(root / "include" / "sailor.h")
    assert len(sources) >= 7
    for f in sources:
        text = f.read_text()
        assert not re.search(r"^\s*(from|import)\s+oracle\b", text, re.M), f
        assert "sailor_oracle" not in text and "oracle/" not in text, f
    for f in (root / "oracle").iterdir():
        if f.suffix in (".py", ".c", ".h"):
            text = f.read_text()
            assert "paper_2504_17096_amd" not in text and "sailor.h" not in text, f
