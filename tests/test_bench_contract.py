"""Host-side checks of bench.py: what it refuses, what its byte accounting says, and that every profile
summary it quotes exists.  No GPU is touched."""
import importlib
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, cwd=ROOT)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_algorithmic_bytes_per_kernel():
    bench = importlib.import_module("bench")
    M, N, K, voted = 4, 1_200_000_000, 1_200_000, 4_792_815
    kb = lambda name, **kw: bench.kernel_bytes(name, M, N, K, kw.pop("rows", M), voted, kw.pop("dense", False),
                                               kw.pop("tally", False), kw.pop("votes", False), **kw)
    assert kb("filter") == 4.0 * M * N                       # one read of the gradients
    assert kb("filter", rows=3) == 4.0 * 3 * N               # rows that skipped the pass are not counted
    assert kb("filter_mem") == 12.0 * M * N                  # g~ and e read, e written
    assert kb("filter_mem", mem_pass_bytes=8.0) == 8.0 * M * N
    assert kb("vote_sparse") == 4.0 * M * K + 8.0 * voted    # the words, a read and a write per voted parameter
    assert kb("vote_dense", votes=True) == 4.0 * M * K + 1.0 * N
    assert kb("vote_dense", tally=True, votes=True) == 4.0 * M * K + 5.0 * N
    assert kb("apply_update") == 1.0 * N + 8.0 * voted
    assert kb("vote_momentum", dense=True) == 4.0 * M * K + 16.0 * N


def test_quoted_profiles_exist_and_hold_their_command():
    bench = importlib.import_module("bench")
    for (workload, variant, kernel), (nbytes, path) in bench.PROFILED_TRAFFIC.items():
        full = os.path.join(ROOT, path)
        assert os.path.isfile(full), path
        text = open(full).read()
        assert "rocprofv3 --pmc FETCH_SIZE" in text and "rocprofv3 --pmc WRITE_SIZE" in text and "-- python3 bench.py" in text, path
        assert f"--workload {workload}" in text, (path, workload)
        assert nbytes > 0
