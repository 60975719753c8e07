"""Host-side behaviour of bench.py that needs no GPU: more than one GPU is refused with a message, the kernel name in
the roofline record follows the library's plan, and the HBM-traffic figure taken from profiles/ is reported only for
the kernel source it was counted on."""
import hashlib
import importlib.util
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def load_bench():
    spec = importlib.util.spec_from_file_location("bench_under_test", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=300)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr) or "1 GPU" in (r.stdout + r.stderr) or "single" in (r.stdout + r.stderr).lower()


def test_kernel_name_follows_the_plan():
    b = load_bench()
    assert b.attention_kernel_name(1024, 64, False) == "tree_attn_bf16_kernel<2, false>"
    assert b.attention_kernel_name(1024, 64, True) == "tree_attn_bf16_kernel<2, true>"
    assert b.attention_kernel_name(32, 64, False) == "tree_attn_split_kernel<false>"       # one layer of one context
    assert b.attention_kernel_name(1024, 128, False) == "tree_attn_bf16_kernel<4, false>"
    assert b.attention_kernel_name(1024, 256, False) == "tree_attn_bf16_kernel<8, false>"
    assert b.attention_kernel_name(32, 256, False) == "tree_attn_bf16_kernel<8, false>"    # wide units never take the split plan


def test_traffic_from_profiles_is_tied_to_the_kernel_source():
    b = load_bench()
    rec = json.load(open(os.path.join(ROOT, "profiles", "tree_attn_bf16_llama7b_traffic.json")))
    src = os.path.join(ROOT, "paper_2311_08252_amd", "csrc", "attention.hip")
    current = hashlib.sha256(open(src, "rb").read()).hexdigest()
    value, where = b.profiled_traffic("llama7b")
    if rec["attention_hip_sha256"] == current:
        assert value == rec["hbm_bytes_per_launch"] and "profiles/" in where
        # the counted bytes are the algorithmic ones to a tenth of a per cent: nothing is read twice
        assert abs(value / rec["algorithmic_bytes_per_launch"] - 1.0) < 1e-3
    else:
        assert value is None and "older kernel source" in where
    assert b.profiled_traffic("no-such-workload") == (None, None)
