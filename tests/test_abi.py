"""The C-ABI library: it loads without a GPU, exports every function the public header
declares, and its host-only helpers agree with the oracle's reading of the paper."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import workflow as owf

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def ob():
    from paper_2604_19004_amd import binding, build
    if not os.path.exists(build.lib_path()):
        build.build()
    binding.load()
    return binding


def declared_functions():
    text = open(os.path.join(ROOT, "include", "ocean_spgemm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(ocean_[a-z0-9_]+)\s*\(", text))
    names -= {"ocean_allocator", "ocean_csr", "ocean_options", "ocean_stats"}
    return sorted(names)


def test_every_declared_symbol_is_exported(ob):
    lib = ctypes.CDLL(ob._build.lib_path())
    names = declared_functions()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in include/ocean_spgemm.h but not exported"


def test_struct_layouts_match_the_header(ob, tmp_path):
    src = tmp_path / "sz.c"
    src.write_text('#include "ocean_spgemm.h"\n#include <stdio.h>\n#include <stddef.h>\n'
                   'int main(){printf("%zu %zu %zu %zu %zu\\n", sizeof(ocean_csr), sizeof(ocean_options), '
                   'sizeof(ocean_stats), offsetof(ocean_stats, bin_ms), offsetof(ocean_options, allocator));}')
    exe = tmp_path / "sz"
    import subprocess
    subprocess.run(["gcc", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    got = [int(x) for x in subprocess.run([str(exe)], capture_output=True, text=True, check=True).stdout.split()]
    assert got[0] == ctypes.sizeof(ob.ocean_csr)
    assert got[1] == ctypes.sizeof(ob.ocean_options)
    assert got[2] == ctypes.sizeof(ob.ocean_stats)
    assert got[3] == ob.ocean_stats.bin_ms.offset
    assert got[4] == ob.ocean_options.allocator.offset


def test_defaults_are_the_papers_parameters(ob):
    o = ob.default_options()
    assert (o.upper_bound_avg_products, o.er_threshold, o.cr_threshold) == (64.0, 8.0, 8.0)      # Table 1
    assert (o.sample_ratio, o.sample_min, o.sample_max) == (0.03, 600, 10000)                      # Section 4.3
    assert o.workflow == ob.WF_AUTO and o.hll_registers == 0 and o.estimate_scale == 1.0
    assert o.bitmap_query_cr == 2.0 and o.assist_sigmas == 1.0                                      # Section 4.3 / 4.1
    assert o.selector == ob.SEL_MI355X     # Table 1 with its CR threshold re-derived for this GPU; SEL_TABLE1 = as printed


def test_host_helpers_agree_with_the_oracle(ob):
    for rows in (1, 7, 600, 601, 19999, 20001, 333334, 10 ** 7):
        assert ob.sample_size(rows) == owf.sample_size(rows)
    for rows, seed in ((100, 1), (4096, 2), (1 << 20, 3)):
        assert np.array_equal(ob.sample_rows(rows, ob.default_options(sample_seed=seed)), owf.sample_rows(rows, seed))
    grid = [0.0, 1.0, 7.999, 8.0, 8.001, 63.999, 64.0, 64.001, 1e9]
    for avg in grid:
        for er in grid:
            for cr in grid:
                assert ob.select_workflow(avg, er, cr) == owf.select_workflow(avg, er, cr)
    for er in (0.0, 47.999, 48.0, 1e6):
        assert ob.hll_register_count(er) == owf.hll_registers(er)
    # the re-tuned rule: hand-checked corners, then the grid against the oracle's reading
    U, H, S = owf.UPPER_BOUND, owf.HLL, owf.SYMBOLIC
    assert ob.select_workflow_tuned(10.0, 100.0, 100.0, 1e9, 0.0) == U
    assert ob.select_workflow_tuned(100.0, 30.0, 3.2, 4e8, 0.0) == H           # light rows only: threshold 3.0
    assert ob.select_workflow_tuned(100.0, 30.0, 3.2, 4e8, 4e8) == S           # heavy rows only: threshold 4.5
    assert ob.select_workflow_tuned(100.0, 30.0, 3.75, 4e8, 2e8) == H          # half and half: threshold 3.75
    assert ob.select_workflow_tuned(100.0, 30.0, 3.74, 4e8, 2e8) == S
    assert ob.select_workflow_tuned(100.0, 7.9, 100.0, 4e8, 0.0) == S          # ER below 8
    assert ob.select_workflow_tuned(100.0, 30.0, 3.2, 1e6, 0.0) == S           # small problem: two passes, unsampled
    assert ob.select_workflow_tuned(100.0, 30.0, 100.0, 1e6, 0.0) == S
    assert ob.select_workflow_tuned(100.0, 30.0, 2.99, 4e8, 0.0) == S          # below the light threshold: two passes
    assert ob.select_workflow_tuned(100.0, 30.0, 3.0, 4e8, 0.0) == H
    assert ob.select_workflow_tuned(100.0, 30.0, 1.2, 4e8, 4e8) == S           # heavy rows: two passes, whatever the CR
    assert ob.select_workflow_tuned(100.0, 30.0, 0.99, 4e8, 0.0) == S          # below the light threshold
    low = ob.default_options(tuned_cr_light=1.0)                                  # estimation from CR 1.0 on: below 1.5 the bound
    assert ob.select_workflow_tuned(100.0, 30.0, 1.2, 4e8, 0.0, low) == U
    assert ob.select_workflow_tuned(100.0, 30.0, 1.5, 4e8, 0.0, low) == H
    assert owf.select_workflow_tuned(100.0, 30.0, 1.2, 4e8, 0.0, cr_light=1.0) == U
    for avg in grid:
        for er in grid:
            for cr in (0.5, 1.0, 1.499, 1.5, 2.0, 2.75, 2.999, 3.0, 3.75, 4.5, 8.0):
                for p_, h_ in ((1e3, 0.0), (1e8, 0.0), (1e8, 5e7), (1e8, 1e8)):
                    assert ob.select_workflow_tuned(avg, er, cr, p_, h_) == owf.select_workflow_tuned(avg, er, cr, p_, h_)
    num, sym = ob.bin_layout()
    assert num == sorted(num) and sym == sorted(sym) and num[-1] == sym[-1] == 2 ** 31 - 1


def test_product_path_fails_loudly_without_a_gpu(ob):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    from paper_2604_19004_amd import workloads as W
    A = W.erdos_renyi(64, 4, seed=1)
    with pytest.raises(RuntimeError):
        ob.to_device(A)
