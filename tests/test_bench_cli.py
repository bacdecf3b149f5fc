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


def test_committed_traffic_figures_name_kernels_that_exist():
    # bench.py reports roofline.traffic from profiles/hbm_traffic.json, counted once with rocprofv3; the entry names
    # the kernel it was counted on, and that kernel must still exist with that many template arguments
    import glob
    import json
    import re
    src = "\n".join(open(f).read() for f in glob.glob(os.path.join(ROOT, "paper_2604_17834_amd", "csrc", "*.hip")))
    table = json.load(open(os.path.join(ROOT, "profiles", "hbm_traffic.json")))
    checked = 0
    for workload, entry in table.items():
        if workload.startswith("_"):
            continue
        m = re.match(r"^asp::(\w+)(?:<(.*)>)?$", entry["kernel"])
        assert m, entry["kernel"]
        name, args = m.group(1), m.group(2)
        d = re.search(r"template\s*<([^>]*)>\s*__global__[^;{]*?\bvoid\s+" + name + r"\s*\(", src)
        if args is None:
            assert re.search(r"__global__[^;{]*?\bvoid\s+" + name + r"\s*\(", src), name
        else:
            assert d, "no kernel template named " + name
            assert len(d.group(1).split(",")) == len(args.split(",")), (entry["kernel"], d.group(1))
        assert entry["bytes_per_launch"] == pytest.approx(entry["fetch_bytes"] + entry["write_bytes"], rel=2e-3)
        checked += 1
    assert checked >= 5
    # the summaries under profiles/ name the headline kernel with its current template arguments
    for f in glob.glob(os.path.join(ROOT, "profiles", "*.txt")):
        for args in re.findall(r"bcsr_spmm_wide_kernel<([^>]*)>", open(f).read()):
            assert len(args.split(",")) == 2, (f, args)
