"""The measurement tools around the library: the instrumented build with time stamps in the kernels
(paper_2510_26577_amd/timeline.py), the few-rows comparison against a vector-ALU kernel
(paper_2510_26577_amd/small_rows.py) and the profile writers.  CPU part: shapes, names, the plain build's refusal
of the stamp read.  GPU part: the alternative kernel agrees with the library and with the oracle; the stamps of
the instrumented build are ordered and its outputs are the plain build's."""
import ctypes
import os
import subprocess
import sys

import numpy as np
import pytest

from paper_2510_26577_amd import binding, profile_kernels, small_rows, timeline

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_cases_of_the_few_rows_comparison_have_the_rows_they_claim():
    rows = {}
    for name in small_rows.CASES:
        w, nq = small_rows.make_case(name)
        G = w.Hq // w.Hkv
        rows[name] = (nq if nq is not None else int(w.max_T)) * G
        assert w.max_T <= 128 and (nq is None or nq <= int(w.T.min()))
    assert rows == {"cfg1": 8, "decode_B64": 4, "draft_q12": 24}
    a = small_rows.AttnArgs()
    assert ctypes.sizeof(a) == 10 * 8 + 6 * 4 + 4 + 4 + 2 * 8      # ten pointers, six ints, the scale (+ padding), two pointers


def test_workload_names_and_profile_commands():
    for name in ("cfg1", "cfg2", "cfg2_B32", "cfg3_B16", "cfg4"):
        assert timeline.get_workload(name).B >= 1
    with pytest.raises(SystemExit):
        timeline.get_workload("nope")
    assert profile_kernels.bench_args("cfg3_B64+fp8") == ["--workload", "cfg3_B64", "--kv-fp8"]
    assert profile_kernels.bench_args("cfg2") == ["--workload", "cfg2"]
    for cs in profile_kernels.COUNTER_SETS:                      # what one rocprofv3 --pmc run can hold
        assert sum(c.startswith("SQ_") for c in cs) <= 8 and sum(c.startswith("GRBM_") for c in cs) <= 2


def test_plain_build_has_no_time_stamps():
    lib = binding.load_library()
    buf = (ctypes.c_uint64 * 8)()
    assert lib.tva_timeline_read(buf, 1) == -2                   # TVA_UNSUPPORTED: no GPU is touched


@pytest.mark.gpu
@pytest.mark.parametrize("name", small_rows.CASES)
def test_vector_alu_alternative_agrees_with_the_library(name):
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    s = small_rows.Prepared(name, 0)
    st = torch.cuda.current_stream()
    s.run_mfma(st)
    s.run_valu(st)
    torch.cuda.synchronize()
    fin = torch.isfinite(s.lse_m)
    assert bool((torch.isfinite(s.lse_v) == fin).all())
    assert float((s.out_m - s.out_v).abs().max()) <= small_rows.TOL_O
    assert float((s.lse_m[fin] - s.lse_v[fin]).abs().max()) <= small_rows.TOL_LSE
    if name == "cfg1":                                           # the alternative against the oracle itself
        from oracle import tva_oracle
        ro, rl = tva_oracle.tree_verify_attn(s.w)
        assert np.abs(s.out_v.cpu().numpy().astype(np.float64) - ro).max() <= small_rows.TOL_O
        assert np.abs(s.lse_v.cpu().numpy().astype(np.float64) - rl).max() <= small_rows.TOL_LSE


@pytest.mark.gpu
def test_instrumented_build_stamps_are_ordered():
    """One process loads one build, so the instrumented one runs in a child: its summary must show every stage
    after the one before, for every workgroup (the minima of the stage differences are not negative)."""
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    if not os.path.exists(binding.TIMELINE_LIB_PATH):
        pytest.skip("libtva_timeline.so not built")
    r = subprocess.run([sys.executable, "-m", "paper_2510_26577_amd.timeline", "--workload", "cfg3_B4", "--copies", "4",
                        "--replays", "2"], cwd=ROOT, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr[-2000:]
    stage_lines = [l for l in r.stdout.splitlines() if l.startswith("  + ")]
    assert len(stage_lines) == 6                                 # five attention stages + the merge block
    for l in stage_lines:
        assert float(l.split("min")[1].split()[0]) >= 0.0, l
    assert "merge kernel" in r.stdout and "gap between" in r.stdout
