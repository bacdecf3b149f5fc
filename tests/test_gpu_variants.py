"""Every benchmarking switch of the library (the rungs of `bench.py --ablation` and of the tile-width study, after
the paper's feature-by-feature study, Section IV-B, and its tile-width study, Section IV-C) selects a kernel
variant that must compute the same product: one child process per switch setting (the library reads a switch once
per process), each on the projection workload's matrix at a reduced dense width, checked against the oracle at the
usual tolerance (bf16: 1e-2 * S + 1e-5, fp32: 1e-5 * S) on sampled columns, every output checked for having been written.
"""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CHILD = os.path.join(ROOT, "tests", "variant_child.py")

# (switches, workload, dense width, entry, expected tile width or None)
VARIANTS = [
    ({}, "bcsr_gate_proj", 2048, "", 512),                                                  # the default, for reference
    ({"ASP_BCSR_KERNEL": "regstage", "ASP_BCSR_BN": "256"}, "bcsr_gate_proj", 2048, "", 256),  # synchronous register-staged loads
    ({"ASP_BCSR_KERNEL": "regstage", "ASP_BCSR_BN": "128"}, "bcsr_gate_proj", 1024, "", 128),
    ({"ASP_BCSR_KERNEL": "regstage", "ASP_BCSR_BN": "64"}, "bcsr_gate_proj", 1024, "", 64),
    ({"ASP_BCSR_BN": "256"}, "bcsr_gate_proj", 2048, "", 256),                               # direct-to-LDS ring, 2 workgroups per CU
    ({"ASP_BCSR_BN": "128"}, "bcsr_gate_proj", 2048, "", 128),
    ({"ASP_BCSR_BN": "64"}, "bcsr_gate_proj", 2048, "", 64),
    ({"ASP_BCSR_BN": "256", "ASP_BCSR_SCHEDULE": "atomic"}, "bcsr_gate_proj", 2048, "", 256),  # tiles pulled from atomic counters
    ({"ASP_BCSR_BN": "256", "ASP_BCSR_SCHEDULE": "atomic"}, "bcsr_gate_proj", 16384 + 64, "", 256),  # ... with a masked tail tile
    ({"ASP_BCSR_BN": "256", "ASP_BCSR_SCHEDULE": "atomic"}, "bcsr_down_proj", 4096, "", 256),     # ... 28 long block-rows
    ({"ASP_BCSR_BN": "256", "ASP_BCSR_SCHEDULE": "atomic"}, "bcsr_sweep_b128_s95", 2048, "", 256),  # ... empty block-rows, geometric lengths
    ({"ASP_BCSR_BN": "256", "ASP_BCSR_GROUP_N": "1"}, "bcsr_gate_proj", 2048, "", 256),
    ({"ASP_BCSR_BN": "256", "ASP_BCSR_WGS_PER_CU": "1"}, "bcsr_gate_proj", 2048, "", 256),
    ({"ASP_BCSR_WORKGROUPS": "128"}, "bcsr_gate_proj", 2048, "", 512),                       # half of the compute units idle
    ({"ASP_BCSR_WORKGROUPS": "64"}, "bcsr_gate_proj_b64", 2048 + 72, "", 512),               # ... composite form, masked tail
    ({"ASP_BCSR_XCD_AWARE": "0"}, "bcsr_gate_proj", 2048, "", 512),                          # tiles dealt without regard to XCDs
    ({"ASP_BCSR_GROUP_N": "1"}, "bcsr_gate_proj", 2048, "", 512),
    ({"ASP_BCSR_GROUP_N": "4"}, "bcsr_gate_proj", 2048, "", 512),
    ({"ASP_BCSR_GROUP_N": "3"}, "bcsr_gate_proj", 2560, "", 512),                            # a narrower last group
    ({"ASP_BCSR_COMPOSITE": "0"}, "bcsr_gate_proj_b64", 2048, "", 256),                      # small blocks on their own kernel
    ({"ASP_BCSR_COMPOSITE": "1"}, "bcsr_gate_proj_b32", 2048, "", 512),                      # ... and forced onto 128-row stacks
    ({"ASP_BCSR_XT": "generic"}, "bcsr_small", 256, "xt", None),                             # no matrix cores
    ({"ASP_WCSR_MAX_BN": "64"}, "wcsr_zipf", 256, "", 64),
    ({"ASP_WCSR_MAX_BN": "128"}, "wcsr_zipf", 256, "", 128),
]


@pytest.mark.parametrize("switches,workload,N,entry,bn", VARIANTS,
                         ids=["+".join("%s=%s" % kv for kv in v[0].items()) or "default" for v in VARIANTS])
def test_switched_variant_matches_oracle(switches, workload, N, entry, bn):
    env = {k: v for k, v in os.environ.items() if not k.startswith("ASP_")}
    env.update(switches)
    scale = "0.125" if workload.startswith("wcsr") else "1"   # 131072 rows keep the irregular workload's long rows
    cmd = [sys.executable, CHILD, workload, str(N), entry or "-", scale]
    out = subprocess.run(cmd, env=env, capture_output=True, text=True, timeout=300)
    assert out.returncode == 0, "child failed:\n%s\n%s" % (out.stdout[-2000:], out.stderr[-2000:])
    res = json.loads(out.stdout.strip().splitlines()[-1])
    assert res["ok"] and not res["unwritten"]
    if bn is not None:
        assert res["bn"] == bn, res
