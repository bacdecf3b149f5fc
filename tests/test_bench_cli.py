"""bench.py's command line (no GPU needed): one GPU by design, and the workload-name grammar it relies on."""
import os
import subprocess
import sys

import pytest

from paper_2604_17834_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    for extra_env, args in (({}, ["--gpus", "2"]), ({"WORLD_SIZE": "2"}, [])):
        env = dict(os.environ)
        env.update(extra_env)
        out = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")] + args, env=env, capture_output=True,
                             text=True, timeout=120)
        assert out.returncode == 2
        assert "single-GPU" in out.stderr and out.stdout.strip() == ""


def test_workload_name_suffixes():
    a, fmt, br, bc, N, dt, _ = synth.workload("bcsr_gate_proj_b64_f32", scale=0.02)
    assert (fmt, br, bc, dt, a.dtype, (a.m, a.k)) == ("bcsr", 64, 64, "f32", "f32", (18944, 3584))
    a, fmt, br, bc, N, dt, _ = synth.workload("wcsr_zipf_bf16", scale=0.002)
    assert (fmt, br, bc, dt, a.dtype) == ("wcsr", 16, 8, "bf16", "bf16")
    a, fmt, br, bc, N, dt, _ = synth.workload("wcsr_scrambled_band", scale=0.001)
    assert fmt == "wcsr" and a.m == a.k == 4096 and a.nnz > 26 * 4096
    with pytest.raises(KeyError):
        synth.workload("no_such_workload")
