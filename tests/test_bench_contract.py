"""The benchmark's command-line contract, as far as it can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and not r.stdout.strip()


def test_world_size_above_one_is_refused():
    env = dict(os.environ, WORLD_SIZE="2", RANK="0")
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True,
                       timeout=120, env=env)
    assert r.returncode != 0 and "ONE GPU" in r.stderr


def test_workload_table_is_consistent():
    sys.path.insert(0, ROOT)
    import bench
    assert "large_topk" in bench.WORKLOADS           # the headline workload
    for name, w in bench.WORKLOADS.items():
        assert w["comp"] in ("topk", "randk", "sign", "qsgd"), name
        assert w["n"] >= 1 and w["d"] >= 1 and w["gamma"] > 0 and w["lr"] > 0, name
        if w["comp"] in ("topk", "randk"):
            assert 1 <= w["k"] <= w["d"], name
        layers = bench.layer_table_of(w)
        if layers is not None:
            assert int(layers[0][-1] + layers[1][-1]) == w["d"], name
    for kernel, bytes_per_entry in bench.KERNEL_BYTES_PER_ELEM.items():
        assert kernel.startswith("k_") and bytes_per_entry % 4 == 0
