#!/usr/bin/env python3
"""Throughput of the QODA hot path on one MI355X.

One step = one round of Alg. 1's device work over all K simulated nodes: (level fit when the workload is adaptive)
-> quantize + pack all nodes -> fused decode + K-way mean + dual-averaging update.  Inputs (two sets of the K nodes'
synthetic gradients, used in alternation, plus state and message buffers) are resident in HBM before the timed region.

Prints ONE JSON line: whole-job GB/s of fp32 gradient pushed through the path on the headline workload (timed over
exactly --steps rounds, also reported as the median over 5 groups of them), the roofline of the dominant kernel from HIP
-event timings taken inside the timed region, bandwidth ceilings measured on this device with the kernels' own access
type, the same measurement for the second large workload (`secondary`), and the CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X published HBM3E bandwidth
VALU_LANE_OPS = 39.3e12    # 256 CU x 4 SIMD x 16 lanes x 2.4 GHz: vector instructions x 64 lanes per second
GROUPS = 5                 # the timed rounds are split into this many groups; the median over groups is reported


def _library():
    from paper_2505_14371_amd import qoda

    if not os.path.exists(qoda.LIB_PATH):
        from paper_2505_14371_amd import build

        build.build()
    return qoda


def _cpu_baseline(w, model, K, scope=0, kind=2, sample_target=6e7):
    """The oracle, as it stands, single-threaded, on a bounded sample of the same data: a run of consecutive
    tensors (skipping a leading embedding-sized one) for up to 4 nodes, one full round."""
    import oracle

    L = len(w.sizes)
    Ks = min(K, 4)
    start = 1 if (L > 2 and w.sizes[0] > sample_target) else 0
    layers, tot = [], 0
    for l in range(start, L):
        layers.append(l)
        tot += w.sizes[l]
        if tot >= sample_target:
            break
    sizes = [w.sizes[l] for l in layers]
    S = w.points
    grads = []
    for k in range(Ks):
        flat = model["grad"][k]
        grads.append([flat[int(model["off"][l]): int(model["off"][l]) + w.sizes[l]].cpu().numpy() for l in layers])
    lev = [(np.arange(S, dtype=np.float64) / (S - 1)).astype(np.float32) for _ in sizes]
    x1 = [np.zeros(s, np.float32) for s in sizes]
    y = [np.zeros(s, np.float32) for s in sizes]
    t0 = time.perf_counter()
    if w.adaptive:
        flat = [grads[k][i] for k in range(Ks) for i in range(len(sizes))]
        lev, _, _, _ = oracle.fit_levels(sizes, list(range(len(sizes))), [S] * len(sizes), Ks, flat, lev, scope=scope, norm_kind=kind)
    msgs, deltas = [], []
    for k in range(Ks):
        m, _, dl, _ = oracle.quantize(sizes, [S] * len(sizes), lev, grads[k], w.seed, 1, k, scope=scope, norm_kind=kind)
        msgs.append(m)
        deltas.append(dl)
    mean = oracle.dequant_aggregate(sizes, [S] * len(sizes), msgs, scope=scope)
    _, eta = oracle.step_size(deltas, 0.0)
    for i in range(len(sizes)):
        oracle.oda_update(mean[i], x1[i], y[i], eta, eta, want_next=False)
    dt = time.perf_counter() - t0
    gbytes = 4.0 * Ks * tot / 1e9
    return {"value": gbytes / dt, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"one round, nodes 0..{Ks - 1}, tensors {layers[0]}..{layers[-1]} "
                      f"({tot} coordinates per node, {Ks * tot} node-coordinates) in {dt:.1f} s",
            "ns_per_node_coordinate": dt / (Ks * tot) * 1e9}


def _ceilings(qoda, ctx, a, b, nbytes):
    """Bandwidth this device sustains for the kernels' own access type (nontemporal 128-bit loads and stores over
    64 KiB tiles) at several read/write mixes, and for a plain copy kernel: GB/s of total traffic.  Where a tile's
    stores fall relative to its loads matters by several per cent, so every mix is measured with the destination
    shifted by a few distances against the source: the figure is the best of them, the others are kept beside it."""
    if nbytes < (1 << 28):   # a streaming ceiling needs a buffer well beyond the caches: only the large workloads give one
        return None
    shifts = (0, 1024, 4352, 69888)
    nb = (nbytes - (1 << 20)) // 65536 * 65536
    src, dst = a.data_ptr(), b.data_ptr()
    out = {}
    for name, stores in (("read_nt_GBps", 0), ("mix_1_store_per_8_loads_nt_GBps", 2), ("mix_1_store_per_2_loads_nt_GBps", 8),
                         ("copy_nt_GBps", 16)):
        rates = []
        for sh in (shifts if stores else shifts[:1]):
            ctx.profile_enable(["k_stream"])
            for _ in range(5):
                ctx.stream_calibration(src, dst + sh, nb, stores)
            ms, n = ctx.profile_read()["k_stream"]
            rates.append(nb * (1.0 + stores / 16.0) / (ms / n * 1e-3) / 1e9)
        out[name] = max(rates)
        if stores:
            out[name.replace("_GBps", "_by_shift_GBps")] = dict(zip((str(x) for x in shifts), rates))
    ctx.profile_enable(["k_copy_f4"])
    for _ in range(5):
        ctx.copy_calibration(a, b, nb)
    ms, n = ctx.profile_read()["k_copy_f4"]
    out["copy_kernel_GBps"] = 2.0 * nb / (ms / n * 1e-3) / 1e9
    ctx.profile_enable(False)
    return out


def run_workload(args, name, steps, warmup, with_ceilings):
    """Build the workload on the device, run warm-up and timed rounds, return the measurements as a dict."""
    import torch

    qoda = _library()
    from paper_2505_14371_amd import workloads

    dev = torch.device("cuda:0")
    w = workloads.get(name)
    L, K, S, d = len(w.sizes), w.num_nodes, w.points, w.total
    scope = {"layer": qoda.SCOPE_LAYER, "vector": qoda.SCOPE_VECTOR, "bucket": qoda.SCOPE_BUCKET}[args.norm_scope]
    bucket = scope == qoda.SCOPE_BUCKET
    kind = {"l2": qoda.NORM_L2, "l1": qoda.NORM_L1, "linf": qoda.NORM_LINF}[args.norm_kind]
    ctx = qoda.Context(w.sizes, list(range(L)), [S] * L, K, w.seed, norm_scope=scope, norm_kind=kind)
    off, flat_len = workloads.padded_offsets(w.sizes)

    def ptrs(t):
        base = t.data_ptr()
        return [base + 4 * int(o) for o in off]

    # two sets of gradients (rounds 1 and 2 of the generator), used in alternation: no round re-quantizes the buffers
    # the previous one read
    nsets = 2 if 2 * 4.0 * K * flat_len < 0.7 * torch.cuda.get_device_properties(0).total_memory else 1
    grad = [[workloads.node_torch(w, k, r + 1, dev)[0] for k in range(K)] for r in range(nsets)]
    mbytes = ctx.message_bytes()
    msg = [[torch.zeros(mbytes, dtype=torch.uint8, device=dev) for _ in range(K)] for _ in range(2)]
    x1 = torch.randn(flat_len, dtype=torch.float32, device=dev)
    y = torch.zeros(flat_len, dtype=torch.float32, device=dev)
    xh = torch.zeros(flat_len, dtype=torch.float32, device=dev)
    xn = torch.zeros(flat_len, dtype=torch.float32, device=dev) if args.x_next else None
    acc = torch.zeros(1, dtype=torch.float64, device=dev)
    eta = torch.ones(2, dtype=torch.float32, device=dev)
    alt = args.q_hat > 0.0
    alt_sums = torch.zeros(2, dtype=torch.float64, device=dev)
    # the pointer sets never change: marshalled once, outside the timed region
    gptrs = [qoda.pointer_array([p for k in range(K) for p in ptrs(g[k])]) for g in grad]
    x1p, yp, xhp = (qoda.pointer_array(ptrs(t)) for t in (x1, y, xh))
    xnp = qoda.pointer_array(ptrs(xn)) if xn is not None else None
    msg_arr = [qoda.pointer_array(m) for m in msg]
    state = {"cur": 0, "t": 0}

    def one_round():
        state["t"] += 1
        t, cur = state["t"], state["cur"]
        g = gptrs[t % nsets]
        every = max(args.fit_every, 1)
        if bucket and every > 1:
            ctx.gather_statistics(t % every == 0)        # only the round before an update step gathers
        if w.adaptive and (every == 1 or t % every == 1):
            if bucket and t > 1:
                # bucket scope: the fit uses the statistics gathered by the previous quantize pass (the order of
                # Alg. 1: the levels are updated before the round's vectors exist) and reads no gradient
                ctx.fit_levels(None, t)
            else:
                # layer / vector scope: the fit runs on the round's own vectors (they exist by now on this device) and
                # keeps their norms for the quantize call below
                ctx.fit_levels_keep_norms(g, t)
        ctx.quantize_all(g, t, msg_arr[cur], msg_arr[1 - cur] if (t > 1 and not alt) else None)
        if alt:
            ctx.step_alt(msg_arr[cur], x1p, yp, xhp, alt_sums, eta, args.q_hat, xnp)
        else:
            ctx.step(msg_arr[cur], x1p, yp, xhp, acc, xnp, eta)
        state["cur"] = 1 - cur

    # warm-up rounds, all kernel classes timed: gives the per-kernel breakdown and names the dominant kernel
    ctx.profile_enable(True)
    for _ in range(max(warmup, 2)):
        one_round()
    torch.cuda.synchronize()
    warm = ctx.profile_read()
    dec = "k_decode<alt>" if alt else "k_decode<true>"
    timed_classes = ("k_sumsq<false>", "k_sumsq<true>", "k_quantize", dec, "k_bucket_max", "k_bucket_hist")
    dom = max((n for n in warm if n in timed_classes), key=lambda n: warm[n][0])
    # timed region: only the dominant kernel is bracketed by events (every timed launch costs a few microseconds
    # of idle time around it, which matters for the millisecond-scale workloads).  The rounds are split into GROUPS
    # groups with an event between them; nothing else separates the groups.
    ctx.profile_enable([dom])
    groups = [steps // GROUPS + (1 if i < steps % GROUPS else 0) for i in range(GROUPS)]
    groups = [g for g in groups if g > 0]
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(len(groups) + 1)]
    torch.cuda.synchronize()
    t_host0 = time.perf_counter()
    ev[0].record()
    for i, g in enumerate(groups):
        for _ in range(g):
            one_round()
        ev[i + 1].record()
    torch.cuda.synchronize()
    t_host = time.perf_counter() - t_host0
    total_ms = ev[0].elapsed_time(ev[-1])
    per_group = [ev[i].elapsed_time(ev[i + 1]) / g for i, g in enumerate(groups)]
    prof = ctx.profile_read()
    ctx.profile_enable(False)
    if ctx.status() != qoda.OK:
        raise RuntimeError("non-finite input flagged")

    c1_bits = 1 + max(1, int(np.ceil(np.log2(S))))
    # packed bytes per node (sign + index, plus one fp32 norm per 128 entries under bucket scope), no padding
    body_bytes = (c1_bits / 8.0 + (4.0 / 128.0 if bucket else 0.0)) * d
    alg = {"k_sumsq<false>": 4.0 * K * d, "k_sumsq<true>": 4.0 * K * d,
           "k_bucket_max": 4.0 * K * d, "k_bucket_hist": 4.0 * K * d,
           "k_quantize": 4.0 * K * d + (1.0 if alt else 2.0) * K * body_bytes,   # eq. (Alt) reads no previous message
           dec: float(K * body_bytes) + (20.0 if xn is not None else 16.0) * d}
    kernels = {n: {"avg_ms": ms / cnt, "launches": cnt, "from": "warm-up rounds"} for n, (ms, cnt) in warm.items()}
    dom_ms = prof[dom][0] / prof[dom][1]                 # from the timed region
    kernels[dom] = {"avg_ms": dom_ms, "launches": prof[dom][1], "from": "timed region"}
    achieved = alg[dom] / (dom_ms * 1e-3) / 1e9
    # model time of each big kernel: max(algorithmic bytes / HBM peak, vector instructions x 64 lanes / lane-op rate),
    # the instruction counts per node-coordinate measured with rocprofv3 (profiles/sq_counters.json)
    valu = {}
    spath = os.path.join(ROOT, "profiles", "sq_counters.json")
    if os.path.exists(spath):
        try:
            valu = json.load(open(spath)).get("valu_instructions_per_node_coordinate", {}).get(name, {})
        except Exception:
            valu = {}
    for n in kernels:
        if n in alg:
            kernels[n]["algorithmic_GBps"] = alg[n] / (kernels[n]["avg_ms"] * 1e-3) / 1e9
            t_hbm = alg[n] / (HBM_PEAK_GBS * 1e9) * 1e3
            kernels[n]["model_ms_hbm"] = t_hbm
            if n in valu:
                t_alu = valu[n] * K * d / VALU_LANE_OPS * 1e3
                kernels[n]["model_ms_valu"] = t_alu
                kernels[n]["model_ms"] = max(t_hbm, t_alu)
                kernels[n]["model_bound"] = "hbm" if t_hbm >= t_alu else "valu"
    traffic, tsrc = None, None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            # counters were collected under the main rule; eq. (Alt) reads no previous message in the quantizer
            key = name + ("+alt" if alt else "") + ("" if scope == qoda.SCOPE_LAYER else "+" + args.norm_scope)
            key += "" if kind == qoda.NORM_L2 else "+" + args.norm_kind   # (no counter runs for the other kinds)
            traffic = json.load(open(tpath)).get(key, {}).get(dom)
            tsrc = f"profiles/traffic.json[{key}] (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE on the torch-free probe; " \
                   "counters cannot be read inside this run)" if traffic is not None else None
        except Exception:
            traffic = None

    ms_per_step = total_ms / steps
    grad_bytes = 4.0 * K * d
    if bucket:   # norms and fit statistics are computed inside the quantize pass
        alg_round = alg["k_quantize"] + alg[dec]
    else:
        alg_round = sum(alg[n] for n in (("k_sumsq<true>" if (w.adaptive and args.fit_every <= 1) else "k_sumsq<false>"),
                                         "k_quantize", dec))
    med = statistics.median(per_group)
    out = {
        "value": grad_bytes / (ms_per_step * 1e-3) / 1e9,
        "unit": "GB/s",
        "steps": steps, "warmup": max(warmup, 2), "ms_per_step": ms_per_step,
        "repetitions": len(groups), "rounds_per_repetition": groups,
        "ms_per_step_median": med, "ms_per_step_min": min(per_group), "ms_per_step_max": max(per_group),
        "value_at_median": grad_bytes / (med * 1e-3) / 1e9,
        "config": {"workload": name, "num_nodes": K, "coordinates": d, "tensors": L, "level_points": S,
                   "adaptive_levels": w.adaptive, "message_bytes_per_node": mbytes, "x_next": xn is not None,
                   "step_sizes": f"eq. (Alt), q_hat={args.q_hat}" if alt else "eq. (general_stepsize)",
                   "norm_scope": args.norm_scope, "norm_kind": args.norm_kind, "gradient_sets_alternated": nsets,
                   "levels_fitted_every": max(args.fit_every, 1) if w.adaptive else None},
        "hbm_peak_fraction_algorithmic": alg_round / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "algorithmic_bytes_per_step": alg_round,
        "host_wall_ms_per_step": t_host / steps * 1e3,
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": tsrc, "avg_ms": dom_ms,
                     "algorithmic_bytes_per_launch": alg[dom]},
        "kernels": kernels,
    }
    if with_ceilings:
        out["measured_ceilings"] = _ceilings(qoda, ctx, y, xh, min(flat_len * 4, 4 << 30))
    keep = {"grad": grad[0], "off": off, "w": w, "K": K, "scope": scope, "kind": kind}
    return out, keep


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="gpt1p3b", choices=["bilinear", "microbench", "dcgan", "txl", "gpt1p3b"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-secondary", action="store_true", help="skip the second large workload")
    ap.add_argument("--x-next", action="store_true", help="also materialise X_{t+1}")
    ap.add_argument("--norm-scope", default="layer", choices=["layer", "vector", "bucket"],
                    help="what one norm covers: a layer (default), the node's whole vector, or buckets of 128 entries")
    ap.add_argument("--norm-kind", default="l2", choices=["l2", "l1", "linf"],
                    help="the q of the L^q normalisation (Sec. 2.2); the workloads' default is L2")
    ap.add_argument("--fit-every", type=int, default=1,
                    help="update the levels every N rounds (the workloads say every round, the default; the paper's "
                         "experiments every few thousand steps)")
    ap.add_argument("--q-hat", type=float, default=0.0,
                    help="> 0: the step sizes of eq. (Alt) with this exponent instead of eq. (general_stepsize)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the K nodes are K message buffers on one device); "
              "--gpus must be 1", file=sys.stderr)
        return 2

    import torch

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    try:
        head, keep = run_workload(args, args.workload, args.steps, args.warmup, with_ceilings=True)
    except RuntimeError as e:
        print(f"bench.py: {e}", file=sys.stderr)
        return 1
    out = {"metric": "GB/s fp32 gradient through quantize+aggregate+QODA step; % of HBM peak",
           "value": head.pop("value"), "unit": head.pop("unit"), "n_gpus": 1, "steps": head.pop("steps"),
           "warmup": head.pop("warmup"), "ms_per_step": head.pop("ms_per_step"), "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic"}
    out.update(head)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = _cpu_baseline(keep["w"], keep, keep["K"], keep["scope"], keep["kind"])
    del keep
    # the other workload of at least 150 M coordinates, in the same process, after the headline's buffers are gone
    other = {"gpt1p3b": "txl", "txl": "gpt1p3b"}.get(args.workload)
    if other and not args.no_secondary:
        import gc

        gc.collect()
        torch.cuda.empty_cache()
        try:
            sec, _ = run_workload(args, other, max(args.steps, 25) if other == "txl" else args.steps, args.warmup,
                                  with_ceilings=False)
            out["secondary"] = {other: sec}
        except RuntimeError as e:
            out["secondary"] = {other: {"error": str(e)}}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
