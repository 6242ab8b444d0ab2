"""Host-side checks of bench.py's command line (no GPU needed): more than one GPU is refused with a message,
and the traffic figure is read from the committed rocprofv3 summary of the same workload and kernel variant."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args, env=None):
    e = dict(os.environ)
    e.update(env or {})
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          env=e, timeout=120)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _run("--gpus", "2")
    assert r.returncode == 2 and "single-GPU" in r.stderr and r.stdout.strip() == ""
    r = _run(env={"WORLD_SIZE": "4"})
    assert r.returncode == 2 and "single-GPU" in r.stderr


def test_traffic_is_taken_from_the_profile_of_the_same_kernel_variant():
    sys.path.insert(0, ROOT)
    import bench
    path = os.path.join(ROOT, "profiles", "gate_up_traffic_qwen3_layer_layered.txt")
    text = open(path).read()
    variant = [l for l in text.splitlines() if l.startswith("variant: ")][0][len("variant: "):]
    t, source = bench.traffic_from_profiles("qwen3_layer", "layered", variant)
    assert t is not None and 8.0e8 < t < 1.0e9            # ~900 MB per gate_up launch, above the 840 MB algorithmic
    assert source == os.path.join("profiles", "gate_up_traffic_qwen3_layer_layered.txt")   # the line says where it is from
    assert bench.traffic_from_profiles("qwen3_layer", "layered", variant + "x") == (None, None)   # another kernel: no figure
    assert bench.traffic_from_profiles("no_such_workload", "layered", variant) == (None, None)


def test_default_run_covers_every_baseline_configuration():
    sys.path.insert(0, ROOT)
    import bench
    from paper_2510_08055_amd import inputs
    runs = [bench.HEADLINE] + bench.ALSO
    assert bench.HEADLINE == ("qwen3_group8", "layered")          # the largest single-GPU configuration
    for wl in ("tiny_f32", "qwen3_layer", "qwen3_group8", "mixtral_zipf", "decode_large"):
        assert any(r[0] == wl for r in runs), wl
    assert ("qwen3_group8", "chunked") in runs and ("tiny_f32", "chunked") in runs
    assert all(r[0] in inputs.WORKLOADS and r[0] in bench.BOUND for r in runs)
