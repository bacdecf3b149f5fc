"""Child process of tests/test_gpu_variants.py: one product through the C ABI under whatever benchmarking switches
(ASP_* environment variables) the parent set, checked against the oracle; prints one JSON line.

The switches are read once per process inside the library, hence a process per variant.

    python tests/variant_child.py <workload> <N> [xt|-] [scale]
"""
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402
import torch  # noqa: E402

import oracle  # noqa: E402
from paper_2604_17834_amd import binding as asp  # noqa: E402
from paper_2604_17834_amd import synth  # noqa: E402


def main():
    name, N = sys.argv[1], int(sys.argv[2])
    xt = len(sys.argv) > 3 and sys.argv[3] == "xt"
    scale = float(sys.argv[4]) if len(sys.argv) > 4 else 1.0
    a, fmt, b_row, b_col, _, dt, seedB = synth.workload(name, scale)
    print("variant", {k: v for k, v in os.environ.items() if k.startswith("ASP_")}, name, "N", N, "xt", xt,
          file=sys.stderr, flush=True)
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream().cuda_stream
    B = synth.dense_normal(a.k, N, dt, seedB)            # k x N; the K-contiguous entry gets its transpose
    tdt = torch.int16 if dt == "bf16" else torch.float32
    src = np.ascontiguousarray(B.T) if xt else B
    Bd = torch.from_numpy(src.view(np.int16) if dt == "bf16" else src).cuda()
    Cd = torch.empty((N, a.m) if xt else (a.m, N), dtype=tdt, device="cuda")
    Cd.fill_(0x7FC1 if dt == "bf16" else float("nan"))   # every element must be overwritten
    h = asp.asp_create_from_csr(fmt, dt, b_row, b_col, a.m, a.k, a.row_ptr, a.col_idx, a.values)
    try:
        plan = asp.asp_plan_spmm(h, N)
        asp.asp_reserve(h, N)
        (asp.asp_spmm_xt if xt else asp.asp_spmm)(h, Bd.data_ptr(), Cd.data_ptr(), N, stream)
        torch.cuda.synchronize()
    finally:
        asp.asp_destroy(h)
    rng = np.random.default_rng(3)
    cols = np.unique(np.r_[0:32, N - 32:N, rng.choice(N, 64, replace=False)])
    got = Cd.cpu().numpy()
    got = np.ascontiguousarray(got[cols].T if xt else got[:, cols])
    unwritten = bool((Cd == 0x7FC1).any()) if dt == "bf16" else bool(torch.isnan(Cd).any())
    got = synth.to_f64(got.view(np.uint16), "bf16") if dt == "bf16" else got.astype(np.float64)
    ref, S = oracle.spmm(a.m, a.k, a.row_ptr, a.col_idx, a.values, dt, np.ascontiguousarray(B[:, cols]))
    bound = 1e-2 * S + 1e-5 if dt == "bf16" else 1e-5 * S
    ok = bool(np.isfinite(got).all() and (np.abs(got - ref) <= bound).all()) and not unwritten
    print(json.dumps({"ok": ok, "bn": int(plan.bn), "n_tiles": int(plan.n_tiles), "workgroups": int(plan.workgroups),
                      "unwritten": unwritten, "checked_columns": int(len(cols))}))
    return 0 if ok else 1


if __name__ == "__main__":
    sys.exit(main())
