"""Benchmark of the structured-OBS pruning hot path on one MI355X.

One "step" is one pass of the whole path over one synthetic layer that is already resident in
HBM: Hessian accumulation (H = 2 X X^T), dampened Cholesky inverse, and the greedy loop that
removes every structure of the layer (Algorithm 1).  Default workload: configuration 3, the
BERT-base feed-forward down-projection (W 768 x 3072, 16384 calibration tokens, post-GELU).

Prints ONE JSON line.  `value` is seconds per layer for the whole path (lower is better).
`roofline` describes the greedy-loop kernel against HBM bandwidth with the algorithmic byte
count  sum over steps of (8 r^2 + 8 d_row r + 4 r), r = live columns;  `roofline_hessian` the
Hessian kernel against the fp32 matrix-core peak with d (d + 1) n_tok useful flops.
`cpu_baseline` is the fp64 CPU oracle timed on this host on the same layer.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# HBM bytes per launch of the greedy-loop kernel from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs summarised
# in profiles/greedy_loop_and_hessian_config3_hbm_counters.md (KiB, already scaled by the copy-kernel factors);
# --traffic-kib overrides them after a new counter run.
MEASURED_TRAFFIC_KIB = {3: (3333971.0, 3124632.0)}
HBM_PEAK_GBS = 8000.0
MFMA_F32_PEAK_TFLOPS = 157.3


def loop_algorithmic_bytes(d_row, d_col, group_size, n_remove):
    """Live-square model of the greedy loop: per step read+write the live r x r block of the
    fp32 inverse Hessian (8 r^2), read+write the live d_row x r block of W (8 d_row r) and read
    the pivot rows (4 g r)."""
    total = 0
    r = d_col
    for _ in range(n_remove):
        total += 8 * r * r + 8 * d_row * r + 4 * group_size * r
        r -= group_size
    return total


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=3, help="workload configuration 1..4")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="also run one plain device-to-device copy of this many MiB before the timed steps, so a "
                         "rocprofv3 --pmc run of this command holds a kernel of known HBM traffic to scale counters by")
    ap.add_argument("--traffic-kib", type=float, nargs=2, default=None, metavar=("FETCH", "WRITE"),
                    help="per-launch HBM KiB of the loop kernel from rocprofv3 --pmc runs (for the record)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (layers are independent and would be sharded one "
              "per GPU without communication); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2302_04089_amd import workloads, ziplm

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    ziplm.lib()
    spec = workloads.config(args.config)
    d, m, g, G = spec.d_col, spec.d_row, spec.group_size, spec.n_groups
    t0 = time.time()
    X_host = workloads.make_X(spec)
    W_host = workloads.make_W(spec)
    gen_s = time.time() - t0

    X = torch.from_numpy(X_host).cuda()
    W0 = torch.from_numpy(W_host).cuda()
    W = torch.empty_like(W0)
    H = torch.empty((d, d), dtype=torch.float32, device="cuda")
    Hi = torch.empty_like(H)
    ws_h = torch.empty(max(ziplm.ziplm_hessian_workspace_bytes(d, spec.n_tok), 256), dtype=torch.uint8, device="cuda")
    ws_i = torch.empty(ziplm.ziplm_hinv_workspace_bytes(d), dtype=torch.uint8, device="cuda")
    ws_p = torch.empty(ziplm.ziplm_prune_workspace_bytes(m, d, g, 0), dtype=torch.uint8, device="cuda")

    def ev():
        return torch.cuda.Event(enable_timing=True)

    stage_ms = {"hessian": [], "hinv": [], "loop": []}
    result = {}

    def one_step(record):
        e = [ev() for _ in range(4)]
        W.copy_(W0)
        H.zero_()
        e[0].record()
        ziplm.ziplm_hessian_accumulate(H, X, 2.0, workspace=ws_h)
        e[1].record()
        ziplm.ziplm_hinv(H, spec.damp_rel, out=Hi, workspace=ws_i, check=False)
        e[2].record()
        order, err, _ = ziplm.ziplm_structured_obs_prune(W, Hi, g, G, workspace=ws_p, check=False)
        e[3].record()
        if record:
            result["events"].append(e)
        return order, err

    if args.calibration_copy_mib > 0:
        n = args.calibration_copy_mib * (1 << 20) // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)          # reads n*4 bytes, writes n*4 bytes
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        one_step(False)
    torch.cuda.synchronize()
    result["events"] = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        order, err = one_step(True)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    for e in result["events"]:
        stage_ms["hessian"].append(e[0].elapsed_time(e[1]))
        stage_ms["hinv"].append(e[1].elapsed_time(e[2]))
        stage_ms["loop"].append(e[2].elapsed_time(e[3]))
    ms_per_step = wall * 1e3 / args.steps
    mean = {k: float(np.mean(v)) for k, v in stage_ms.items()}

    order_h = order.cpu().numpy()
    assert sorted(order_h.tolist()) == list(range(G)), "loop did not remove every structure exactly once"
    assert float(W.abs().max()) == 0.0

    loop_bytes = loop_algorithmic_bytes(m, d, g, G)
    loop_gbs = loop_bytes / (mean["loop"] * 1e-3) / 1e9
    syrk_flops = float(d) * (d + 1) * spec.n_tok
    hess_tflops = syrk_flops / (mean["hessian"] * 1e-3) / 1e12

    traffic = None
    kib = args.traffic_kib if args.traffic_kib is not None else MEASURED_TRAFFIC_KIB.get(args.config)
    if kib is not None:
        traffic = (kib[0] + kib[1]) * 1024.0

    out = {
        "metric": "structured-OBS prune time per layer (Hessian + inverse + greedy loop)",
        "value": ms_per_step / 1e3,
        "unit": "s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "config %d: %s, W %dx%d, group %d, %d tokens %s, damp %.2g, remove all %d"
                   % (args.config, spec.name, m, d, g, spec.n_tok, spec.x_kind, spec.damp_rel, G)},
        "stage_ms": mean,
        "hessian_tflops": hess_tflops,
        "loop_hbm_gbs": loop_gbs,
        "us_per_loop_step": mean["loop"] * 1e3 / G,
        "roofline": {"kernel": "greedy loop", "bound": "hbm", "achieved": loop_gbs, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": loop_gbs / HBM_PEAK_GBS, "traffic": traffic,
                     "algorithmic_bytes": loop_bytes},
        "roofline_hessian": {"kernel": "hessian syrk", "bound": "mfma", "achieved": hess_tflops,
                             "peak": MFMA_F32_PEAK_TFLOPS, "unit": "TFLOP/s",
                             "frac": hess_tflops / MFMA_F32_PEAK_TFLOPS, "useful_flops": syrk_flops},
    }

    if not args.no_cpu_baseline:
        from oracle import ziplm_oracle as oracle
        oracle.build()
        t0 = time.perf_counter()
        H_or = oracle.hessian(X_host, 2.0)
        t1 = time.perf_counter()
        Hi_or, _ = oracle.hinv(H_or, spec.damp_rel)
        t2 = time.perf_counter()
        oracle.prune(W_host, Hi_or.astype(np.float32), g, G)
        t3 = time.perf_counter()
        out["cpu_baseline"] = {
            "value": t3 - t0, "unit": "s", "cores": oracle.threads(), "kind": "oracle",
            "sample": "the whole layer of the same workload, once (Hessian %.2f s, inverse %.2f s, loop %.2f s)"
                      % (t1 - t0, t2 - t1, t3 - t2)}
    out["input_generation_s"] = gen_s
    print(json.dumps(out))


if __name__ == "__main__":
    main()
