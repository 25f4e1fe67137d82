"""The host-side graph packer under AddressSanitizer and UBSan (host code only: g++,
no GPU).  It writes into one growing byte vector through raw pointers, which is exactly
what a sanitizer is good at checking."""
import os
import shutil
import subprocess

import numpy as np
import pytest

from workloads import build_csr, make_workload, random_layered_dag
from workloads.dags import _finish

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_1711_01912_amd", "csrc")


@pytest.fixture(scope="module")
def harness(tmp_path_factory):
    if shutil.which("g++") is None:
        pytest.skip("no host compiler")
    out = tmp_path_factory.mktemp("packer") / "harness"
    cmd = ["g++", "-std=c++17", "-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fno-omit-frame-pointer", os.path.join(ROOT, "tests", "packer_harness.cpp"),
           os.path.join(CSRC, "graph.cpp"), os.path.join(CSRC, "cost.cpp"), "-o", str(out)]
    subprocess.run(cmd, check=True)
    return str(out)


def _dump(w, d):
    np.array([w.n, w.m, w.L], dtype=np.int64).tofile(os.path.join(d, "hdr.bin"))
    for name, dt in (("succ_ptr", np.int32), ("succ_idx", np.int32), ("succ_t", np.int64), ("pred_ptr", np.int32),
                     ("pred_idx", np.int32), ("pred_eid", np.int32), ("c", np.int64), ("level_ptr", np.int32),
                     ("level_vtx", np.int32)):
        np.ascontiguousarray(getattr(w, name), dtype=dt).tofile(os.path.join(d, name + ".bin"))


def _deep(seed):
    rng = np.random.default_rng(9500 + seed)
    depth = int(rng.integers(250, 600))
    widths = rng.integers(20, 110, size=depth)
    n, level, src, dst = random_layered_dag(rng, widths, 1, 3, depth - 1)
    csr = build_csr(n, src, dst, rng.integers(0, 3000, size=len(src)), level)
    return _finish(f"deep-{seed}", csr, rng.integers(1, 400, size=n), 2, [1, 2], [[1, 3], [3, 1]],
                   np.zeros((1, n), dtype=np.uint8))


@pytest.mark.parametrize("case", ["tiny", "mlp", "inception", "hubs", "sparse", "deep0", "deep1", "wide-weights"])
def test_packer_is_clean_under_sanitizers(harness, tmp_path, case):
    if case == "hubs":
        w = make_workload("comm_heavy", P=1, levels=5, width=600, hub_degree=300)
    elif case == "sparse":
        w = make_workload("large_sparse", P=1, levels=150, width=200)
    elif case.startswith("deep"):
        w = _deep(int(case[4:]))
    elif case == "wide-weights":
        w = make_workload("tiny", P=1)
        w.c = w.c * 2**36
    else:
        w = make_workload(case, P=1)
    _dump(w, str(tmp_path))
    run = subprocess.run([harness, str(tmp_path)], capture_output=True, text=True)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "rc=0" in run.stdout
    if case.startswith("deep") or case == "inception":
        assert "far_b=0" not in run.stdout
