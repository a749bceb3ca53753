#!/usr/bin/env python3
"""Benchmark of the forest-verification hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input: dsbd_forest_attention (one
transformer layer's attention over the draft forest), dsbd_verify_forest and dsbd_select_beams, on the
largest configuration (c5: W=8 beams, 31-node trees, prefix 8192, GQA 32/8, head_dim 128, vocabulary
128256).  Inputs are resident in HBM before the timed region; steps rotate over several copies of the
inputs so that the 256 MB Infinity Cache cannot serve the K/V and logit streams.

Prints one JSON line: nodes verified per second, plus the roofline of the dominant kernel (algorithmic
bytes / its HIP-event duration) and the CPU oracle's rate on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBS = 8000.0   # MI355X datasheet
# HBM bytes per launch on c5 measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (each scaled by what the same
# counter reads for a 256 MiB copy): see profiles/bench_c5_hbm_traffic.md.  Only valid for the default workload.
MEASURED_TRAFFIC_C5 = {"attention": 286.0e6 + 33.0e6, "vocab_stats": 254.6e6 + 0.9e6, "verify_layers": 44.8e6 + 0.3e6}


def cpu_baseline(sample_trees=8):
    """The oracle, as it stands, on the first `sample_trees` beams of the c5 workload (all 8: the benchmark's
    batch itself, about 15 s of CPU work; fewer: a prompt of the same tree shape, prefix length, heads and
    vocabulary with that many beams)."""
    import numpy as np
    from dsbd_synth import make_workload
    import gpu_util as gu
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = 1
    w = make_workload("c5", W=sample_trees)
    t0 = time.perf_counter()
    gu.oracle_attention(w)
    t1 = time.perf_counter()
    gu.oracle_verify(w, t=-1.0)
    t2 = time.perf_counter()
    return {"value": w.n_nodes / (t2 - t0), "unit": "nodes/s", "cores": int(cores), "kind": "oracle",
            "sample": "%s of c5 (%d nodes), once: attention %.2f s + verify %.2f s on %d host threads"
                      % ("the whole batch" if sample_trees == 8 else "first %d of the 8 beams" % sample_trees,
                         w.n_nodes, t1 - t0, t2 - t1, cores)}


def commit_measurement(dsbd, torch, w, d, o, reps=10):
    """Cache commit along the plan of the last step (not part of `value`: it is a row beyond the verification path).
    Policy measured: the first next beam of every source tree continues in its source buffer (tree rows appended),
    every other next beam gets a fresh buffer (whole prefix copied)."""
    grow = w.max_depth + 1
    L = [int(x) for x in w.own_len]
    cap = max(L) + grow
    mk = lambda: torch.empty((cap, w.Hkv, w.D), dtype=torch.bfloat16, device="cuda")
    k_src, v_src = d.kv.keep[0], d.kv.keep[1]
    src_k, src_v = [mk() for _ in L], [mk() for _ in L]
    for b in range(len(L)):
        src_k[b][:L[b]] = k_src[b]; src_v[b][:L[b]] = v_src[b]
    kv = dsbd.PrefixKV([src_k[b][:L[b]] for b in range(len(L))], [src_v[b][:L[b]] for b in range(len(L))])
    nx = o["nx"]
    torch.cuda.synchronize()
    n_next, src_tree, path_len = nx.n_next.cpu().numpy(), nx.src_tree.cpu().numpy(), nx.path_len.cpu().numpy()
    dst_k, dst_v, taken, moved = [], [], set(), 0
    row = w.Hkv * w.D * 2
    for p in range(w.n_prompts):
        for s_ in range(w.W_cap):
            b = int(src_tree[p, s_]) if s_ < int(n_next[p]) else -1
            if b >= 0 and b not in taken:
                taken.add(b); dst_k.append(src_k[b]); dst_v.append(src_v[b])
                moved += int(path_len[p, s_]) * row * 2 * 2
            elif b >= 0:
                dst_k.append(mk()); dst_v.append(mk())
                moved += (L[b] + int(path_len[p, s_])) * row * 2 * 2
            else:
                dst_k.append(None); dst_v.append(None)
    dst = dsbd.KVDst(dst_k, dst_v, kv)
    fault = torch.zeros(1, dtype=torch.int32, device="cuda")
    dsbd.dsbd_commit_kv(d.forest, kv, d.k_tree, d.v_tree, nx, w.W_cap, dst, fault=fault)
    dsbd.dsbd_timing_enable(dsbd.DSBD_KERNEL_KV_COMMIT, reps)
    for _ in range(reps):
        dsbd.dsbd_commit_kv(d.forest, kv, d.k_tree, d.v_tree, nx, w.W_cap, dst, fault=fault)
    torch.cuda.synchronize()
    ms = sorted(dsbd.dsbd_timing_collect(reps))
    dsbd.dsbd_timing_enable(0, 0)
    assert int(fault.item()) == 0
    med = ms[len(ms) // 2]
    return {"ms": med, "next_beams": int(n_next.sum()), "continued_in_place": len(taken),
            "bytes_read_plus_written": moved, "achieved": moved / (med * 1e-3) / 1e9 if med > 0 else 0.0,
            "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": (moved / (med * 1e-3) / 1e9 / HBM_PEAK_GBS) if med > 0 else 0.0,
            "note": "copies count read + write; not included in value / ms_per_step"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=60)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="c5")
    ap.add_argument("--copies", type=int, default=3, help="input copies rotated through (cold caches)")
    ap.add_argument("--t", type=float, default=-1.0, help="threshold of the dynamic width; < 0 = fixed width")
    ap.add_argument("--kernel", default="attention", choices=["attention", "vocab_stats", "verify_layers"],
                    help="kernel whose duration is measured with HIP events for the roofline")
    ap.add_argument("--shared-len", type=int, default=None,
                    help="control run: leading prefix tokens shared by the beams of a prompt (the caches then serve most K/V)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-commit", action="store_true", help="skip the (separately reported) cache-commit measurement")
    ap.add_argument("--no-warp", action="store_true", help="skip the (separately reported) warped verification")
    ap.add_argument("--no-draft", action="store_true", help="skip the (separately reported) draft-side sampling step")
    ap.add_argument("--warp-top-k", type=int, default=10, help="warping of the separately reported runs (the paper's setting)")
    ap.add_argument("--warp-top-p", type=float, default=0.8)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path has no multi-GPU part); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2409_16560_amd as dsbd
    from dsbd_synth import make_workload
    from dsbd_synth.workloads import algorithmic_bytes
    import gpu_util as gu

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    w = make_workload(args.config) if args.shared_len is None else make_workload(args.config, shared_len=args.shared_len)
    attn_bytes, verify_bytes = algorithmic_bytes(w, share_prefix=True)
    sets = [gu.DeviceWorkload(w)]
    for _ in range(args.copies - 1):
        sets.append(gu.DeviceWorkload(w))
    # caller-owned outputs and workspaces, allocated once
    outs = []
    for d in sets:
        N, Hq, D = d.q.shape
        Hkv = d.k_tree.shape[1]
        o = {
            "out": torch.empty_like(d.q), "lse": torch.empty((N, Hq), dtype=torch.float32, device="cuda"),
            "aws": torch.empty(dsbd.dsbd_forest_attention_workspace_bytes(d.forest, d.kv, Hq, Hkv, D), dtype=torch.uint8, device="cuda"),
            "afault": torch.zeros(1, dtype=torch.int32, device="cuda"),
            "vres": dsbd.VerifyResult.allocate(d.forest, w.W_cap),
            "vws": torch.empty(dsbd.dsbd_verify_forest_workspace_bytes(d.forest, w.V, 0, 1, w.W_cap, args.t), dtype=torch.uint8, device="cuda"),
            "nx": dsbd.NextBeams.allocate(d.forest, w.W_cap),
        }
        outs.append(o)

    def step(i):
        d, o = sets[i % len(sets)], outs[i % len(sets)]
        d.attention(out=o["out"], lse=o["lse"], workspace=o["aws"], fault=o["afault"])
        d.verify(t=args.t, result=o["vres"], workspace=o["vws"])
        dsbd.dsbd_select_beams(d.forest, o["vres"], result=o["nx"])

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    kid = {"attention": dsbd.DSBD_KERNEL_ATTENTION, "vocab_stats": dsbd.DSBD_KERNEL_VOCAB_STATS,
           "verify_layers": dsbd.DSBD_KERNEL_VERIFY_LAYERS}[args.kernel]
    dsbd.dsbd_timing_enable(kid, args.steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    kms = dsbd.dsbd_timing_collect(args.steps)
    dsbd.dsbd_timing_enable(0, 0)
    for o in outs:
        assert int(o["afault"].item()) == 0 and int(o["vres"].fault.item()) == 0

    # per-call breakdown (separate, untimed for the headline): events around each library call
    def timed_calls(fn, reps=20):
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for i, (a, b) in enumerate(ev):
            a.record(); fn(i); b.record()
        torch.cuda.synchronize()
        ts = sorted(a.elapsed_time(b) for a, b in ev)
        return ts[len(ts) // 2]
    br = {
        "attention_ms": timed_calls(lambda i: sets[i % len(sets)].attention(out=outs[i % len(sets)]["out"], lse=outs[i % len(sets)]["lse"], workspace=outs[i % len(sets)]["aws"], fault=outs[i % len(sets)]["afault"])),
        "verify_ms": timed_calls(lambda i: sets[i % len(sets)].verify(t=args.t, result=outs[i % len(sets)]["vres"], workspace=outs[i % len(sets)]["vws"])),
        "select_ms": timed_calls(lambda i: dsbd.dsbd_select_beams(sets[i % len(sets)].forest, outs[i % len(sets)]["vres"], result=outs[i % len(sets)]["nx"])),
    }

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    kavg_ms = sum(kms) / max(1, len(kms))
    kbytes = {"attention": attn_bytes, "vocab_stats": verify_bytes, "verify_layers": 0}[args.kernel]
    achieved = kbytes / (kavg_ms * 1e-3) / 1e9 if kavg_ms > 0 else 0.0
    res = {
        "metric": "forest nodes verified/sec; achieved HBM GB/s vs peak (1 MI355X)",
        "value": w.n_nodes / (ms_per_step * 1e-3), "unit": "nodes/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 attention (fp32 accumulate), fp32 vocab statistics, fp64 accept/resample decisions",
        "data": "synthetic",
        "config": {"workload": "%s: %d beams, %d forest nodes, prefix %d, Hq/Hkv %d/%d, D %d, V %d, %s width"
                               % (args.config, w.n_trees, w.n_nodes, int(w.own_len.max() + w.shared_len.max()),
                                  w.Hq, w.Hkv, w.D, w.V, "fixed" if args.t < 0 else "dynamic t=%g" % args.t),
                   "input_copies_rotated": len(sets),
                   **({} if args.shared_len is None else {"control_shared_prefix_tokens": args.shared_len})},
        "roofline": {"bound": "hbm", "kernel": args.kernel, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": MEASURED_TRAFFIC_C5.get(args.kernel) if args.config == "c5" else None,
                     "algorithmic_bytes_per_launch": kbytes, "avg_launch_ms": kavg_ms, "launches_timed": len(kms)},
        "step_algorithmic_bytes": attn_bytes + verify_bytes,
        "step_hbm_frac": (attn_bytes + verify_bytes) / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "breakdown_ms": br,
    }
    if not args.no_commit:
        res["next_rows"] = {"kv_commit": commit_measurement(dsbd, torch, w, sets[0], outs[0])}
    if not args.no_warp:
        # the same verification with the warping operation on the joints (reported apart from the headline)
        k, p_ = args.warp_top_k, args.warp_top_p
        wws = torch.empty(dsbd.dsbd_verify_forest_workspace_bytes(sets[0].forest, w.V, 0, 1, w.W_cap, args.t, k, p_),
                          dtype=torch.uint8, device="cuda")
        call = lambda i: sets[i % len(sets)].verify(t=args.t, result=outs[i % len(sets)]["vres"], workspace=wws,
                                                    top_k=k, top_p=p_)
        for i in range(5):
            call(i)
        torch.cuda.synchronize()
        reps = 20
        dsbd.dsbd_timing_enable(dsbd.DSBD_KERNEL_VERIFY_LAYERS, reps)
        call_ms = timed_calls(call, reps)
        lk = dsbd.dsbd_timing_collect(reps)
        dsbd.dsbd_timing_enable(0, 0)
        assert int(outs[0]["vres"].fault.item()) == 0
        res.setdefault("next_rows", {})["warped_verify"] = {
            "top_k": k, "top_p": p_, "verify_ms": call_ms, "verify_layers_kernel_ms": sum(lk) / max(1, len(lk)),
            "plain_verify_ms": br["verify_ms"], "note": "dsbd_verify_forest with top_k / top_p set; not part of value"}
    if not args.no_draft:
        # one beam-sampling step of the small model at the benchmark's shape: 16 beams in, 16 draws out (per prompt)
        W_S = 16
        d0 = sets[0]
        zq = d0.logits_q[:W_S].contiguous()
        cum = torch.linspace(-3.0, 0.0, W_S, dtype=torch.float64, device="cuda")
        off = torch.tensor([0, W_S], dtype=torch.int32, device="cuda")
        uu = d0.u_fill.reshape(-1)[:W_S].contiguous()
        dr = {}
        for name, (k, p_) in (("plain", (0, 1.0)), ("warped", (args.warp_top_k, args.warp_top_p))):
            call = lambda i: dsbd.dsbd_draft_layer(off, zq, cum, uu, W_S, max_prompt_beams=W_S, top_k=k, top_p=p_)
            for i in range(3):
                call(i)
            torch.cuda.synchronize()
            dr[name + "_ms"] = timed_calls(call, 20)
        dr.update({"beams_in": W_S, "draws": W_S, "V": w.V, "top_k": args.warp_top_k, "top_p": args.warp_top_p,
                   "note": "dsbd_draft_layer (statistics + sampling kernels, workspace allocated per call); not part of value"})
        res.setdefault("next_rows", {})["draft_layer"] = dr
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline()
    print(json.dumps(res))


if __name__ == "__main__":
    main()
