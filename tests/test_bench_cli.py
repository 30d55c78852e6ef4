"""bench.py's command line on a machine without a GPU: what it refuses, before anything touches the device."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True, timeout=120)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = run("--gpus", "2", "--steps", "4", "--warmup", "1")
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_unknown_workload_is_refused():
    r = run("--workload", "cfg9_nothing")
    assert r.returncode == 2 and "unknown workload" in r.stderr and r.stdout.strip() == ""


def test_the_tiny_parity_workload_is_not_a_bench_line():
    r = run("--workload", "cfg1_tiny_pair")
    assert r.returncode == 2 and "parity-test workload" in r.stderr


def test_step_counts_beyond_the_workload_are_refused():
    r = run("--workload", "cfg2_s15_decode", "--steps", "600")
    assert r.returncode == 2 and "warmup + steps" in r.stderr
    r = run("--seqs", "129")
    assert r.returncode == 2 and "--seqs" in r.stderr
