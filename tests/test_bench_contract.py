"""Host-side checks of bench.py's command line: one GPU only, a clear message without a GPU, the workload table names the
configurations the headline is quoted on.  (The figures themselves need a GPU and are checked by bench.py's own parity gate.)"""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args):
    env = dict(os.environ, HIP_VISIBLE_DEVICES="", CUDA_VISIBLE_DEVICES="")
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True, env=env, timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = run("--gpus", "2")
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_without_a_gpu_the_bench_says_so_and_prints_no_line():
    r = run("--steps", "2", "--warmup", "1")
    assert r.returncode == 3 and "no GPU" in r.stderr and r.stdout.strip() == ""


def test_default_workload_is_the_largest_single_gpu_configuration():
    sys.path.insert(0, ROOT)
    import bench
    ap_default = [a for a in ("llama65b_mlp_pair_3bit",) if a in bench.WORKLOADS]
    assert ap_default, "the 65B MLP pair must be a workload"
    shapes, bits, frac, skew, B = bench.WORKLOADS["llama65b_mlp_pair_3bit"]
    assert shapes == [(22016, 8192), (8192, 22016)] and bits == 3 and abs(frac - 0.0045) < 1e-12 and skew == (0.01, 0.30) and B == 1
    old = sys.argv
    try:
        sys.argv = ["bench.py"]
        assert bench.parse().workload == "llama65b_mlp_pair_3bit"
    finally:
        sys.argv = old
    # every configuration the survey lists has a workload: 7B pair (3 and 4 bit), 13B shapes, 65B shapes, the decode step, batches
    for name in ("single_4096_4bit", "llama7b_mlp_pair_3bit", "llama7b_mlp_pair_4bit", "llama13b_attn_3bit", "llama13b_mlp_pair_3bit",
                 "llama13b_up_3bit_sparse0.05", "llama13b_up_3bit_sparse1.0", "llama65b_attn_3bit", "llama65b_attn_3bit_batch4"):
        assert name in bench.WORKLOADS, name
    for name in ("llama7b_decode_step_3bit", "llama7b_decode_step_3bit_multi_step"):
        assert name in bench.DECODE_STEP, name
