"""Offline half of the method (Sec. 4.3, Algorithm 2): profile the model's best plans on the device for a
set of shapes and write the winners to a plan table that ``binding.ffuse_load_shipped_plans`` (or
``ffuse_plan_table_load``) reads back at run time.

    python -m paper_2512_12949_amd.tune_plans [--out FILE] [--top-k 8] [--reps 10] [workload ...]

Needs an MI355X.  Without workload names: the benchmark configurations and the paper's m = 128 tables.
Operands are random (only the shapes matter for the timing)."""
import argparse
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SHIPPED = os.path.join(HERE, "plans_mi355x.txt")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", default=SHIPPED)
    ap.add_argument("--top-k", type=int, default=8)
    ap.add_argument("--reps", type=int, default=10)
    ap.add_argument("workloads", nargs="*")
    args = ap.parse_args()

    import torch
    from . import binding as ff
    from . import inputs

    names = args.workloads or (["gpt", "llama", "large", "decode16", "decode64"] + [f"G{i}" for i in range(1, 11)] + [f"S{i}" for i in range(1, 9)])
    tdt = {"bf16": torch.bfloat16, "f16": torch.float16}
    ff.ffuse_plan_table_clear()
    for name in names:
        w = inputs.WORKLOADS[name]
        if w.dtype not in tdt:
            continue
        dt = ff.DTYPE_CODE[w.dtype]
        mk = lambda r, c, s: (torch.randn(r, c, device="cuda") * s).to(tdt[w.dtype])
        X, W1, W2 = mk(w.M, w.K, 1.0), mk(w.K, w.N1, w.K ** -0.5), mk(w.N1, w.N2, w.N1 ** -0.5)
        W3 = mk(w.K, w.N1, w.K ** -0.5) if w.gated else None
        Y = torch.empty(w.M, w.N2, device="cuda", dtype=tdt[w.dtype])
        nws = max(ff.ffuse_workspace_bytes(dt, w.gated, w.M, w.K, w.N1, w.N2, False), 256)
        ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
        ff.ffuse_set_workspace(ws)
        plan, ms = ff.ffuse_tune(dt, X, W1, W3, W2, w.act, Y, top_k=args.top_k, reps=args.reps)
        ff.ffuse_set_workspace(None)
        d = plan.as_dict()
        print(f"{name:9s} {w.shape}: {ms * 1e3:8.1f} us  family {d['family']} bm {d['bm']} bh {d['bh']} bk {d['bk']} splits {d['splits']} raster {d['raster']}", flush=True)
        del X, W1, W2, W3, Y, ws
        torch.cuda.empty_cache()
    n = ff.ffuse_plan_table_save(args.out)
    print(f"{n} entries written to {args.out}")


if __name__ == "__main__":
    sys.exit(main())
