"""Host-side behaviour of bench.py and of the entry module (no GPU needed)."""
import json
import os
import subprocess
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    for extra_env, args in (({}, ["--gpus", "2"]), ({"WORLD_SIZE": "2"}, [])):
        env = dict(os.environ, **extra_env)
        r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], env=env,
                           capture_output=True, text=True, timeout=120)
        assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_byte_model_matches_its_definition():
    import bench
    M, K, N, nnz = 1000, 900, 64, 12345
    assert bench.model_bytes(M, N, nnz) == 4 * (M + 1) + 8 * nnz + 4 * nnz * N + 4 * M * N
    assert bench.model_bytes(M, N, nnz, has_vals=False) == 4 * (M + 1) + 4 * nnz + 4 * nnz * N + 4 * M * N
    assert bench.compulsory_bytes(M, K, N, nnz) == 4 * (M + 1) + 8 * nnz + 4 * K * N + 4 * M * N
    # the figure quoted for the large workload: about 30.3 GB algorithmic, 1.04 GB compulsory
    assert abs(bench.model_bytes(232_965, 64, 114_693_532) - 30.34e9) < 0.01e9
    assert abs(bench.compulsory_bytes(232_965, 232_965, 64, 114_693_532) - 1.038e9) < 0.001e9
    assert bench.geomean([2.0, 8.0]) == 4.0 and bench.geomean([]) is None


def test_every_profile_names_its_command_and_measured_traffic_agrees():
    import bench
    import re
    prof = os.path.join(ROOT, "profiles")
    for table in (bench.MEASURED_TRAFFIC_BYTES, bench.MEASURED_TRAFFIC_BYTES_BF16):
        for key, entries in table.items():
            for value, shape, fname in entries:
                text = open(os.path.join(prof, fname)).read()
                assert "rocprofv3 --kernel-trace --stats" in text and "rocprofv3 --pmc FETCH_SIZE" in text
                assert shape in text, (key, shape)                      # the summary was made with this launch shape
                total = float(re.search(r"total ([0-9.]+) GB", text).group(1)) * 1e9
                assert abs(total - value) <= 0.002 * value, (key, total, value)
    for f in os.listdir(prof):
        assert f.endswith((".md", ".txt")) and os.path.getsize(os.path.join(prof, f)) < 20_000


def test_traffic_is_null_for_a_launch_shape_without_a_profile():
    import bench
    plan = dict(vec=4, lanes_per_row=16, tiles_per_lane=1, chunk_nnz=1024, col_blocks=1, k_parts=8)
    assert bench.measured_traffic(bench.MEASURED_TRAFFIC_BYTES, "large_dense_degree/N64/sum", plan) == bench.MEASURED_TRAFFIC_BYTES["large_dense_degree/N64/sum"][0][0]
    plan["k_parts"] = 9
    assert bench.measured_traffic(bench.MEASURED_TRAFFIC_BYTES, "large_dense_degree/N64/sum", plan) is None
    assert bench.measured_traffic(bench.MEASURED_TRAFFIC_BYTES, "no_such_workload/N1/sum", plan) is None
