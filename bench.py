"""Benchmark of the structured-OBS pruning hot path on one MI355X.

One "step" is one pass of the whole path over one synthetic layer that is already resident in
HBM: Hessian accumulation (H = 2 X X^T), dampened Cholesky inverse, and the greedy loop that
removes every structure of the layer (Algorithm 1).  Default workload: configuration 3, the
BERT-base feed-forward down-projection (W 768 x 3072, 16384 calibration tokens, post-GELU).

Prints ONE JSON line.  `value` is seconds per layer for the whole path (lower is better); with
--config 5 it is seconds for the 24 problems of the 12-layer sweep (Hessians and inverses of
the layers on a few streams, then the loops of each kind in one batched call).
`roofline` describes the greedy-loop kernel against HBM bandwidth with the algorithmic byte
count  sum over steps of (8 r^2 + 8 d_row r + 4 r), r = live columns (`achieved`, `frac`: the
model rate the target is stated in).  The kernel defers the eliminations and does not move those
bytes, so the same object also carries what bounds it in fact: `traffic` (HBM bytes per launch from
the rocprofv3 counter runs recorded under profiles/), `physical_gbs` / `physical_frac` (those bytes
over the measured time: the rate at the memory pins) and `handoff_us` / `latency_floor_frac`
(the one-way hand-off time between two workgroups measured on this device just before the timed
steps, times the number of removals, over the loop time: the serial chain of Algorithm 1 cannot run
faster than one hand-off per removal).  `roofline_hessian` prices the Hessian kernel against the
fp32 matrix-core peak with d (d + 1) n_tok useful flops.  `hbm_triad_gbs` is what a plain triad over
1 GiB arrays reaches on the same device (the achievable HBM rate; `frac_of_triad` prices the loop
against it).  `cpu_baseline` is the fp64 CPU oracle timed on this host on the same layer.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_F32_PEAK_TFLOPS = 157.3


def recorded_traffic_bytes(config):
    """HBM bytes per launch of the greedy-loop kernel as the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs measured
    them (scaled by the same counters' reading for a kernel of known traffic): the line
    `traffic_bytes_per_launch: N` of profiles/greedy_loop_config<N>_hbm_counters.md, or None without that record."""
    import re
    path = os.path.join(ROOT, "profiles", "greedy_loop_config%d_hbm_counters.md" % config)
    try:
        m = re.search(r"traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read())
    except OSError:
        return None
    return float(m.group(1)) if m else None


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
    ap.add_argument("--sweep-streams", type=int, default=3,
                    help="configuration 5 only: streams the Hessians and inverses of the layers are spread over")
    ap.add_argument("--config", type=int, default=3, help="workload configuration 1..5 (5: the 24-problem sweep)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--x-layout", choices=("feature", "token"), default="feature",
                    help="layout of the calibration inputs handed to the Hessian call: feature-major X[d_col][n_tok] "
                         "(the configurations' layout) or token-major X[n_tok][d_col] (how activations are captured)")
    ap.add_argument("--loop-kernel", choices=("deferred", "eager"), default="deferred",
                    help="single-column loops through ziplm_structured_obs_prune (deferred eliminations) or through "
                         "ziplm_structured_obs_prune_eager (the whole state read and written every step)")
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
    if args.config == 5:
        # the sweep: 12 layers, each an attention output projection (heads) and a feed-forward down-projection (columns)
        specs = [workloads.config(5, layer=l, kind=k) for l in range(12) for k in ("attn", "ffn")]
    else:
        specs = [workloads.config(args.config)]

    class Problem:
        pass

    t0 = time.time()
    problems = []
    for spec in specs:
        q = Problem()
        q.spec = spec
        q.X = torch.from_numpy(workloads.make_X(spec)).cuda()
        if args.x_layout == "token":
            q.X = q.X.t().contiguous()
        q.W0 = torch.from_numpy(workloads.make_W(spec)).cuda()
        d, m, g = spec.d_col, spec.d_row, spec.group_size
        q.W = torch.empty_like(q.W0)
        q.H = torch.empty((d, d), dtype=torch.float32, device="cuda")
        q.Hi = torch.empty_like(q.H)
        q.ws_h = torch.empty(max(ziplm.ziplm_hessian_workspace_bytes(d, spec.n_tok), 256), dtype=torch.uint8, device="cuda")
        q.ws_i = torch.empty(ziplm.ziplm_hinv_workspace_bytes(d), dtype=torch.uint8, device="cuda")
        eager = args.loop_kernel == "eager" and g == 1
        q.ws_p = torch.empty(ziplm.ziplm_prune_eager_workspace_bytes(m, d, 0) if eager else
                             ziplm.ziplm_prune_workspace_bytes(m, d, g, 0), dtype=torch.uint8, device="cuda")
        problems.append(q)
    gen_s = time.time() - t0
    # one exchange area (uncached device memory, kept for the life of the process) for every single-column loop
    xbytes = max([ziplm.ziplm_prune_exchange_bytes(12 if args.config == 5 else 1, q.spec.d_row, q.spec.d_col, q.spec.group_size)
                  for q in problems])
    exchange = ziplm.ziplm_exchange_alloc(xbytes) if xbytes > 0 else None
    x_layout = ziplm.X_TOKEN_MAJOR if args.x_layout == "token" else ziplm.X_FEATURE_MAJOR
    if args.loop_kernel == "eager" and args.config == 5:
        print("bench.py: --loop-kernel eager times one layer; use it with --config 1, 3 or 4", file=sys.stderr)
        sys.exit(2)

    def ev():
        return torch.cuda.Event(enable_timing=True)

    stage_ms = {"hessian": [], "hinv": [], "loop": []}
    loop_ms_columns = []          # loop time of the single-column problems of one step (the roofline kernel)
    hess_ms_all = []
    result = {}

    # configuration 5: the twelve problems of either kind share one shape and go through the batched call (the
    # loops are latency bound; layers do not interact, so several of them run side by side)
    class Stack:
        pass

    stacks = []
    if args.config == 5:
        for g in sorted({q.spec.group_size for q in problems}):
            sk = Stack()
            sk.members = [q for q in problems if q.spec.group_size == g]
            sk.spec = hs = sk.members[0].spec
            n = len(sk.members)
            sk.W = torch.empty((n, hs.d_row, hs.d_col), dtype=torch.float32, device="cuda")
            sk.Hi = torch.empty((n, hs.d_col, hs.d_col), dtype=torch.float32, device="cuda")
            sk.ws = torch.empty(ziplm.ziplm_prune_batch_workspace_bytes(n, hs.d_row, hs.d_col, hs.group_size, 0),
                                dtype=torch.uint8, device="cuda")
            for i, q in enumerate(sk.members):
                q.W, q.Hi = sk.W[i], sk.Hi[i]            # views into the stacks
                q.ws_p = None
            stacks.append(sk)
    stacked = {id(q) for sk in stacks for q in sk.members}

    # configuration 5: Hessians and inverses of different layers go to a few streams in turn (default priority;
    # the calls are independent on disjoint buffers), so that the latency-bound inverse of one layer runs under the
    # matrix-core-bound Hessian of another; the batched loops follow on the main stream
    main = torch.cuda.current_stream()
    side = [torch.cuda.Stream() for _ in range(args.sweep_streams)] if (stacks and args.sweep_streams > 1) else []

    def one_step(record):
        marks = []
        for s_ in side:
            s_.wait_stream(main)                 # the previous step's loops still use W and Hinv
        for i, q in enumerate(problems):
            spec = q.spec
            e = [ev() for _ in range(4)]
            with torch.cuda.stream(side[(i // 2) % len(side)] if side else main):      # both problems of a layer on one stream
                q.W.copy_(q.W0)
                q.H.zero_()
                e[0].record()
                ziplm.ziplm_hessian_accumulate(q.H, q.X, 2.0, layout=x_layout, workspace=q.ws_h)
                e[1].record()
                ziplm.ziplm_hinv(q.H, spec.damp_rel, out=q.Hi, workspace=q.ws_i, check=False)
                e[2].record()
            if id(q) in stacked:
                e[3] = e[2]                      # pruned below, all problems of one shape together
            elif args.loop_kernel == "eager" and spec.group_size == 1:
                q.order, q.err, _ = ziplm.ziplm_structured_obs_prune_eager(q.W, q.Hi, spec.n_groups, workspace=q.ws_p,
                                                                           check=False)
                e[3].record()
            else:
                q.order, q.err, _ = ziplm.ziplm_structured_obs_prune(q.W, q.Hi, spec.group_size, spec.n_groups,
                                                                     workspace=q.ws_p, check=False,
                                                                     exchange=exchange if spec.group_size == 1 else None)
                e[3].record()
            marks.append(e)
        for s_ in side:
            main.wait_stream(s_)
        for sk in stacks:
            eb = [ev(), ev()]
            eb[0].record()
            order_b, err_b, _ = ziplm.ziplm_structured_obs_prune_batch(sk.W, sk.Hi, sk.spec.group_size, sk.spec.n_groups,
                                                                       workspace=sk.ws, check=False,
                                                                       exchange=exchange if sk.spec.group_size == 1 else None)
            eb[1].record()
            for i, q in enumerate(sk.members):
                q.order, q.err = order_b[i], err_b[i]
            marks.append(eb)
        if record:
            result["events"].append(marks)

    # one-way hand-off between two workgroups on different XCDs through the memory the loop exchanges its
    # candidates in, measured on this device before anything else is running
    handoff_us = None
    if exchange is not None:
        handoff_us = min(ziplm.ziplm_selftest_handoff_latency(2000, 1, exchange=exchange) for _ in range(3))
    for _ in range(args.warmup):
        one_step(False)
    torch.cuda.synchronize()
    result["events"] = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step(True)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    for marks in result["events"]:
        tot = [0.0, 0.0, 0.0]
        cols = 0.0
        for sk, eb in zip(stacks, marks[len(problems):]):
            dt = eb[0].elapsed_time(eb[1])
            tot[2] += dt
            if sk.spec.group_size == 1:
                cols += dt
        for q, e in zip(problems, marks):
            dt = [e[i].elapsed_time(e[i + 1]) for i in range(2)] + [0.0 if id(q) in stacked else e[2].elapsed_time(e[3])]
            tot = [a + b for a, b in zip(tot, dt)]
            if q.spec.group_size == 1:
                cols += dt[2]
        stage_ms["hessian"].append(tot[0])
        stage_ms["hinv"].append(tot[1])
        stage_ms["loop"].append(tot[2])
        loop_ms_columns.append(cols)
    ms_per_step = wall * 1e3 / args.steps
    mean = {k: float(np.mean(v)) for k, v in stage_ms.items()}
    median = {k: float(np.median(v)) for k, v in stage_ms.items()}

    for q in problems:
        G = q.spec.n_groups
        assert sorted(q.order.cpu().numpy().tolist()) == list(range(G)), "loop did not remove every structure exactly once"
        assert float(q.W.abs().max()) == 0.0

    # achievable HBM rate on this device: a plain triad a = b + s * c over 1 GiB arrays (3 x 4 bytes per element)
    n_tri = 1 << 28
    ta = torch.empty(n_tri, dtype=torch.float32, device="cuda")
    tb = torch.ones(n_tri, dtype=torch.float32, device="cuda")
    tc = torch.ones(n_tri, dtype=torch.float32, device="cuda")
    for _ in range(2):
        torch.add(tb, tc, alpha=0.5, out=ta)
    e0, e1 = ev(), ev()
    e0.record()
    for _ in range(10):
        torch.add(tb, tc, alpha=0.5, out=ta)
    e1.record()
    torch.cuda.synchronize()
    triad_gbs = 10 * 3 * 4 * n_tri / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del ta, tb, tc

    column_specs = [q.spec for q in problems if q.spec.group_size == 1]
    loop_bytes = sum(loop_algorithmic_bytes(sp.d_row, sp.d_col, 1, sp.n_groups) for sp in column_specs)
    loop_ms = float(np.mean(loop_ms_columns)) if column_specs else None
    loop_gbs = loop_bytes / (loop_ms * 1e-3) / 1e9 if column_specs else None     # head-only workloads: time only
    syrk_flops = sum(float(q.spec.d_col) * (q.spec.d_col + 1) * q.spec.n_tok for q in problems)
    hess_tflops = syrk_flops / (mean["hessian"] * 1e-3) / 1e12

    traffic = recorded_traffic_bytes(args.config) if (column_specs and args.loop_kernel == "deferred") else None
    physical_gbs = traffic / (loop_ms * 1e-3) / 1e9 if (traffic and column_specs) else None

    if args.config == 5:
        workload = ("config 5: GPT-2-small-shaped sweep, 12 layers x (attention out-proj W 768x768 in 12 heads of 64 "
                    "columns, N(0,1) inputs + FFN down-proj W 768x3072 single columns, GELU inputs), 32768 tokens each, "
                    "damp 0.01, remove everything; value = all 24 problems, the twelve loops of either kind in one batched call; "
                    "Hessians and inverses of the layers on %d streams in turn (their stage times and the Hessian "
                    "rate are then measured under overlap; --sweep-streams 1 gives them undisturbed)" % max(1, len(side)))
        n_steps_loop = sum(sp.n_groups for sp in column_specs)      # the 12 x 3072 single-column removals
        chain_steps = (len(column_specs) + 3) // 4 * column_specs[0].n_groups     # four loops side by side per launch
    else:
        spec = specs[0]
        workload = ("config %d: %s, W %dx%d, group %d, %d tokens %s, damp %.2g, remove all %d"
                    % (args.config, spec.name, spec.d_row, spec.d_col, spec.group_size, spec.n_tok, spec.x_kind,
                       spec.damp_rel, spec.n_groups))
        if args.x_layout == "token":
            workload += "; X token-major"
        if args.loop_kernel == "eager":
            workload += "; loop on the eager kernel"
        n_steps_loop = chain_steps = spec.n_groups
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
        "config": {"workload": workload},
        "stage_ms": mean,
        "stage_ms_median": median,
        "hessian_tflops": hess_tflops,
        "loop_hbm_gbs": loop_gbs,
        "us_per_loop_step": (loop_ms if column_specs else mean["loop"]) * 1e3 / n_steps_loop,
        "hbm_triad_gbs": triad_gbs,
        "head_loops_ms": (mean["loop"] - loop_ms) if (column_specs and len(column_specs) < len(problems)) else None,
        "roofline": {"kernel": "greedy loop", "bound": "hbm", "achieved": loop_gbs, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": loop_gbs / HBM_PEAK_GBS if column_specs else None,
                     "frac_of_triad": loop_gbs / triad_gbs if column_specs else None,
                     "traffic": traffic, "algorithmic_bytes": loop_bytes,
                     "physical_gbs": physical_gbs,
                     "physical_frac": physical_gbs / HBM_PEAK_GBS if physical_gbs else None,
                     "handoff_us": handoff_us,
                     "latency_floor_frac": (chain_steps * handoff_us * 1e-3 / loop_ms) if (handoff_us and column_specs) else None},
        "roofline_hessian": {"kernel": "hessian syrk", "bound": "mfma", "achieved": hess_tflops,
                             "peak": MFMA_F32_PEAK_TFLOPS, "unit": "TFLOP/s",
                             "frac": hess_tflops / MFMA_F32_PEAK_TFLOPS, "useful_flops": syrk_flops},
    }

    if not args.no_cpu_baseline:
        from oracle import ziplm_oracle as oracle
        oracle.build()
        # config 5: one layer (its two problems) is timed and multiplied by 12
        sample_specs = specs[:2] if args.config == 5 else specs
        parts = [0.0, 0.0, 0.0]
        for sp in sample_specs:
            X_host = workloads.make_X(sp)
            W_host = workloads.make_W(sp)
            t0 = time.perf_counter()
            H_or = oracle.hessian(X_host, 2.0)
            t1 = time.perf_counter()
            Hi_or, _ = oracle.hinv(H_or, sp.damp_rel)
            t2 = time.perf_counter()
            oracle.prune(W_host, Hi_or.astype(np.float32), sp.group_size, sp.n_groups)
            t3 = time.perf_counter()
            parts = [parts[0] + t1 - t0, parts[1] + t2 - t1, parts[2] + t3 - t2]
            del X_host
        mult = 12 if args.config == 5 else 1
        out["cpu_baseline"] = {
            "value": mult * sum(parts), "unit": "s", "cores": oracle.threads(), "kind": "oracle",
            "sample": ("layer 0 of the sweep (both problems), once, times 12" if args.config == 5 else
                       "the whole layer of the same workload, once")
                      + " (Hessian %.2f s, inverse %.2f s, loop %.2f s)" % tuple(mult * x for x in parts)}
    out["input_generation_s"] = gen_s
    print(json.dumps(out), flush=True)
    # Device memory, streams and events are released here, while everything that watches the HIP runtime (a profiler's
    # interposed library, for one) is still alive: left to interpreter shutdown they were destroyed after such a
    # tool's own teardown, and the process then ended in a segmentation fault after its output had been written.
    result.clear()
    del problems, stacks, side
    torch.cuda.synchronize()
    torch.cuda.empty_cache()


if __name__ == "__main__":
    main()
