#!/usr/bin/env python3
"""Layer-wise QODA against a global-quantization extra-gradient scheme on the same kernels (one GPU, K simulated nodes).

Sec. 4 argues two things about the two-call extra-gradient family with one global level sequence: it exchanges
twice per round, and (Remark after eq. (MQV)) one sequence for the whole vector cannot beat one per layer type.  This
script measures both on synthetic layer-shaped gradients:

  qoda        per-layer norms, one fitted sequence per layer, one quantize + exchange + fused step per round;
  eg_global   one norm per node, one fitted sequence, two quantize + exchange + plain-step legs per round.

Printed: one JSON line with milliseconds and message bytes per round for both, and the aggregated quantization error
||mean_k Vhat_k - mean_k V_k||^2 / ||mean_k V_k||^2 of both configurations (the error norm itself is taken with
torch: it is a measurement, not part of the path).
"""
from __future__ import annotations

import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="txl", choices=["dcgan", "txl", "gpt1p3b"])
    ap.add_argument("--rounds", type=int, default=5)
    args = ap.parse_args()

    import torch

    from paper_2505_14371_amd import qoda, workloads

    if not torch.cuda.is_available():
        print("compare_global.py: no GPU visible", file=sys.stderr)
        return 1
    dev = torch.device("cuda:0")
    w = workloads.get(args.workload)
    L, K, S, d = len(w.sizes), w.num_nodes, w.points, w.total
    off, flat_len = workloads.padded_offsets(w.sizes)

    def ptrs(t):
        return [t.data_ptr() + 4 * int(o) for o in off]

    grad = [workloads.node_torch(w, k, 1, dev)[0] for k in range(K)]
    gptrs = [p for k in range(K) for p in ptrs(grad[k])]
    true_mean = torch.zeros(flat_len, dtype=torch.float32, device=dev)
    for k in range(K):
        true_mean += grad[k] / K
    tm2 = float(torch.sum(true_mean.double() ** 2))
    x = torch.randn(flat_len, dtype=torch.float32, device=dev)
    y = torch.zeros_like(x)
    xh = torch.zeros_like(x)
    mean = torch.zeros_like(x)
    acc = torch.zeros(1, dtype=torch.float64, device=dev)
    eta = torch.ones(2, dtype=torch.float32, device=dev)
    gamma = torch.full((1,), 0.01, dtype=torch.float32, device=dev)
    out = {"workload": args.workload, "num_nodes": K, "coordinates": d, "level_points": S, "rounds": args.rounds}

    def timed(fn):
        fn()                                              # warm-up
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for t in range(args.rounds):
            fn(t + 2)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / args.rounds

    def rel_error(ctx, msgs):
        ctx.dequant_aggregate(msgs, ptrs(mean))
        torch.cuda.synchronize()
        return float(torch.sum((mean.double() - true_mean.double()) ** 2)) / tm2

    # ---- QODA: layer-wise
    ctx = qoda.Context(w.sizes, list(range(L)), [S] * L, K, w.seed)
    mb = ctx.message_bytes()
    msg = [[torch.zeros(mb, dtype=torch.uint8, device=dev) for _ in range(K)] for _ in range(2)]
    state = {"cur": 0}

    def qoda_round(t=1):
        cur = state["cur"]
        ctx.fit_levels_keep_norms(gptrs, t)
        ctx.quantize_all(gptrs, t, msg[cur], msg[1 - cur] if t > 1 else None)
        ctx.step(msg[cur], ptrs(x), ptrs(y), ptrs(xh), acc, None, eta)
        state["cur"] = 1 - cur

    out["qoda"] = {"ms_per_round": timed(qoda_round), "exchanges_per_round": 1, "message_bytes_per_node_per_round": mb,
                   "relative_error_of_the_mean": rel_error(ctx, msg[1 - state["cur"]])}
    ctx.close()
    del msg

    # ---- extra-gradient with one norm per node and one sequence
    ctx = qoda.Context(w.sizes, [0] * L, [S], K, w.seed, norm_scope=qoda.SCOPE_VECTOR)
    mb = ctx.message_bytes()
    msg1 = [torch.zeros(mb, dtype=torch.uint8, device=dev) for _ in range(K)]

    def eg_round(t=1):
        ctx.fit_levels_keep_norms(gptrs, 2 * t)
        for leg in (0, 1):                                # the same synthetic vectors stand in for both operator calls
            ctx.quantize_all(gptrs, 2 * t + leg, msg1, None)
            ctx.extrapolate(msg1, ptrs(x), ptrs(xh if leg == 0 else x), gamma)

    out["eg_global"] = {"ms_per_round": timed(eg_round), "exchanges_per_round": 2,
                        "message_bytes_per_node_per_round": 2 * mb,
                        "relative_error_of_the_mean": rel_error(ctx, msg1)}
    ctx.close()
    out["bytes_ratio_eg_over_qoda"] = out["eg_global"]["message_bytes_per_node_per_round"] / \
        out["qoda"]["message_bytes_per_node_per_round"]
    out["time_ratio_eg_over_qoda"] = out["eg_global"]["ms_per_round"] / out["qoda"]["ms_per_round"]
    out["error_ratio_global_over_layerwise"] = out["eg_global"]["relative_error_of_the_mean"] / \
        out["qoda"]["relative_error_of_the_mean"]
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
