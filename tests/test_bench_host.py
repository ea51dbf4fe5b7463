"""Host-side checks of the benchmark: the figures it quotes from profiles are current, the probe library it drives
exports what its binding names, and it refuses more than one GPU."""
import ctypes as C
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _git(*args):
    return subprocess.run(["git", "-C", ROOT, *args], capture_output=True, text=True)


def test_profiled_traffic_belongs_to_the_current_score_kernels():
    """bench.py prints HBM bytes per launch taken from a rocprofv3 profile: they are only worth printing while the
    score kernels are the ones that were profiled."""
    import bench
    commit = bench.TRAFFIC_SOURCE["commit"]
    assert os.path.exists(os.path.join(ROOT, bench.TRAFFIC_SOURCE["file"]))
    if _git("rev-parse", "--git-dir").returncode != 0 or _git("cat-file", "-e", commit + "^{commit}").returncode != 0:
        pytest.skip("no git history here to compare against")
    changed = _git("diff", "--quiet", commit, "--", "paper_2603_11564_amd/csrc/score.hip")
    assert changed.returncode == 0, (f"csrc/score.hip differs from commit {commit}, where {bench.TRAFFIC_SOURCE['file']} "
                                     "was measured: profile the kernels again and update both")
    assert commit in open(os.path.join(ROOT, bench.TRAFFIC_SOURCE["file"])).read()


def test_probe_library_exports_what_its_binding_names():
    from paper_2603_11564_amd import ceiling
    lib = ceiling.load_library()
    for name in ceiling.EXPORTS:
        assert hasattr(lib, name), name
    n = lib.dapq_ceiling_num_mixes()
    assert n >= 10
    mixes = ceiling.slice_mixes()
    assert len(mixes) == n and mixes[0]["mfma"] == 1 and mixes[0]["exp"] == 0
    assert any(m["mfma"] == 1 and m["exp"] == 2 and m["fma"] == 2 and m["add"] == 2 and m["scalar"] == 0 for m in mixes)
    assert lib.dapq_ceiling_slice_mix(n, None) is None
    out = (C.c_double * 5)()
    assert lib.dapq_ceiling_slice(-1, 1, 10, 0, 1, out) != 0      # rejected before anything touches a GPU


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "one GPU" in r.stderr
