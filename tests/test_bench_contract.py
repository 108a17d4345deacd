"""bench.py argument contract that can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    for extra_env, args in (({}, ["--gpus", "2"]), ({"WORLD_SIZE": "2"}, [])):
        env = dict(os.environ, **extra_env)
        res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")] + args, capture_output=True, text=True,
                             env=env, timeout=120)
        assert res.returncode != 0
        assert "ONE GPU" in res.stderr and res.stdout.strip() == ""


def test_profiles_name_the_workload_the_bench_times():
    import json
    from paper_2509_26541_amd import workloads as wl
    with open(os.path.join(ROOT, "paper_2509_26541_amd", "hbm_traffic.json")) as f:
        traffic = json.load(f)
    name = wl.CONFIGS[1].name                      # the default workload of bench.py
    assert name in traffic and traffic[name]["attn_bytes_per_launch"] > 0
    path = os.path.join(ROOT, traffic[name]["profile"])
    assert os.path.exists(path)
    text = open(path).read()
    assert "rocprofv3 --kernel-trace --stats" in text and "--pmc FETCH_SIZE" in text and "bench.py --config 2" in text
    # the traffic figure belongs to one version of the kernel source; bench.py reports it only for that one
    assert len(traffic[name]["attn_bf16_hip_sha16"]) == 16
