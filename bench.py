#!/usr/bin/env python3
"""Benchmark of the forest-verification hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input: dsbd_forest_attention (one transformer
layer's attention over the draft forest) and dsbd_verify_forest_select (dsbd_verify_forest and dsbd_select_beams in
one call: the layer kernel writes the next-beam plan along with the output beams), on the largest configuration
(c5: W=8 beams, 31-node trees, prefix 8192, GQA 32/8, head_dim 128, vocabulary 128256).  Inputs are resident in HBM
before the timed region; steps rotate over several copies of the inputs so that the 256 MB Infinity Cache cannot
serve the K/V and logit streams.

Prints one JSON line.  `value` = forest nodes verified per second over the timed steps.  `roofline` is the WHOLE step
against the HBM peak (algorithmic bytes of the step / step time), because no single kernel stands for the step: the
attention kernel and the vocabulary statistics stream from HBM, the layer kernel is bound by the latency of its
dependent reductions and moves next to nothing.  `roofline_kernels` lists every kernel of the step with its own
HIP-event duration (the library's timing hook on the stream the kernel is launched on) and, where it streams, its own
fraction.  `other_configs` holds the step on c5 with the dynamic width (t = 0.9, 0.7) and with an independent draft
model, on c4 (fixed and dynamic width), c3 and c2; `stream_read_ceiling` a plain
streaming read on the same box; `cpu_baseline` the CPU oracle on the same workload.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X datasheet


def measured_traffic(version):
    """HBM bytes per launch on c5 from the committed rocprofv3 counter summary (profiles/bench_c5_hbm_traffic.md:
    FETCH_SIZE / WRITE_SIZE, each scaled by what the same counter reads for a plain copy).  The summary names the
    library version it was taken with; a library that has moved on gets null instead of stale numbers."""
    path = os.path.join(ROOT, "profiles", "bench_c5_hbm_traffic.md")
    try:
        text = open(path).read()
    except OSError:
        return None
    m = re.search(r"library version: `([^`]*)`", text)
    if not m or m.group(1) != version:
        return None
    out = {}
    for line in text.splitlines():
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if "probe" in cells[0]:
            continue                    # the streaming-read probe is no part of the step
        if len(cells) >= 5 and re.fullmatch(r"[0-9.]+", cells[2] or "x") and re.fullmatch(r"[0-9.]+", cells[4] or "x"):
            out[cells[0]] = (float(cells[2]) + float(cells[4])) * 1e6
    return out or None


class Case:
    """One configuration resident on the device: `copies` uploads of the same workload with caller-owned outputs and
    workspaces, and the step that runs on them."""

    def __init__(self, dsbd, torch, config, copies, t, **overrides):
        from dsbd_synth import make_workload
        from dsbd_synth.device import DeviceWorkload
        from dsbd_synth.workloads import algorithmic_bytes
        self.dsbd, self.torch, self.t, self.config = dsbd, torch, t, config
        self.w = w = make_workload(config, **overrides)
        self.attn_bytes, self.verify_bytes = algorithmic_bytes(w, share_prefix=True)
        self.sets = [DeviceWorkload(w) for _ in range(copies)]
        self.outs = []
        for d in self.sets:
            N, Hq, D = d.q.shape
            Hkv = d.k_tree.shape[1]
            self.outs.append({
                "out": torch.empty_like(d.q), "lse": torch.empty((N, Hq), dtype=torch.float32, device="cuda"),
                "aws": torch.empty(dsbd.dsbd_forest_attention_workspace_bytes(d.forest, d.kv, Hq, Hkv, D), dtype=torch.uint8, device="cuda"),
                "afault": torch.zeros(1, dtype=torch.int32, device="cuda"),
                "vres": dsbd.VerifyResult.allocate(d.forest, w.W_cap),
                "vws": torch.empty(dsbd.dsbd_verify_forest_workspace_bytes(d.forest, w.V, 0, 1, w.W_cap, 0.9), dtype=torch.uint8, device="cuda"),
                "nx": dsbd.NextBeams.allocate(d.forest, w.W_cap),
            })

    def attention(self, i):
        d, o = self.sets[i % len(self.sets)], self.outs[i % len(self.sets)]
        d.attention(out=o["out"], lse=o["lse"], workspace=o["aws"], fault=o["afault"])

    def verify(self, i, t=None, **kw):
        d, o = self.sets[i % len(self.sets)], self.outs[i % len(self.sets)]
        d.verify(t=self.t if t is None else t, result=o["vres"], workspace=kw.pop("workspace", o["vws"]), **kw)

    def select(self, i):
        d, o = self.sets[i % len(self.sets)], self.outs[i % len(self.sets)]
        self.dsbd.dsbd_select_beams(d.forest, o["vres"], result=o["nx"])

    def verify_select(self, i, t=None):
        d, o = self.sets[i % len(self.sets)], self.outs[i % len(self.sets)]
        d.verify_select(t=self.t if t is None else t, result=o["vres"], next_beams=o["nx"], workspace=o["vws"])

    def step(self, i, t=None):
        # verification and selection through the one-call form (the layer kernel writes the next-beam plan itself)
        self.attention(i); self.verify_select(i, t)

    def check_faults(self):
        for o in self.outs:
            assert int(o["afault"].item()) == 0 and int(o["vres"].fault.item()) == 0

    def event_times(self, fn, reps, warmup=3):
        """Milliseconds of `reps` calls of fn(i), each between a pair of events on the launch stream."""
        torch = self.torch
        for i in range(warmup):
            fn(i)
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for i, (a, b) in enumerate(ev):
            a.record(); fn(warmup + i); b.record()
        torch.cuda.synchronize()
        return sorted(a.elapsed_time(b) for a, b in ev)

    def describe(self):
        w = self.w
        return "%s: %d prompts, %d beams, %d forest nodes, prefix %s, Hq/Hkv %d/%d, D %d, V %d, %s width" % (
            self.config, w.n_prompts, w.n_trees, w.n_nodes,
            ("%d" % int(w.own_len.max() + w.shared_len.max())) if w.n_prompts == 1 else
            ("%d..%d" % (int((w.own_len + w.shared_len).min()), int((w.own_len + w.shared_len).max()))),
            w.Hq, w.Hkv, w.D, w.V, "fixed" if self.t < 0 else "dynamic t=%g" % self.t)

    def step_summary(self, reps, t=None):
        ts = self.event_times(lambda i: self.step(i, t), reps)
        med = ts[len(ts) // 2]
        nbytes = self.attn_bytes + self.verify_bytes
        return {"workload": self.describe() if t is None else self.describe().rsplit(",", 1)[0] + ", " + ("fixed width" if t < 0 else "dynamic t=%g width" % t),
                "step_ms_median": med, "step_ms_min": ts[0], "steps_timed": len(ts),
                "nodes_per_s": self.w.n_nodes / (med * 1e-3), "step_algorithmic_bytes": nbytes,
                "step_hbm_frac": nbytes / (med * 1e-3) / 1e9 / HBM_PEAK_GBS, "input_copies_rotated": len(self.sets)}


def cpu_baseline():
    """The oracle, as it stands, on the benchmark's own batch (c5, all 8 beams) with the host's threads as numpy finds
    them, and once more on the first two beams with the numerical libraries held to one thread."""
    import numpy as np
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from dsbd_synth import make_workload
    import gpu_util as gu           # the oracle's wrappers (only this leg of the benchmark loads the oracle)
    cores = len(os.sched_getaffinity(0))

    def run(w):
        t0 = time.perf_counter()
        gu.oracle_attention(w)
        t1 = time.perf_counter()
        gu.oracle_verify(w, t=-1.0)
        t2 = time.perf_counter()
        return t1 - t0, t2 - t1

    w = make_workload("c5")
    ta, tv = run(w)
    res = {"value": w.n_nodes / (ta + tv), "unit": "nodes/s", "cores": int(cores), "kind": "oracle",
           "sample": "the whole c5 batch (%d nodes), once: attention %.2f s + verify %.2f s; %d host cores available to the "
                     "process (numpy's libraries decide how many they use)" % (w.n_nodes, ta, tv, cores)}
    try:
        from threadpoolctl import threadpool_limits
        w2 = make_workload("c5", W=2)
        with threadpool_limits(limits=1):
            ta1, tv1 = run(w2)
        res["one_thread"] = {"value": w2.n_nodes / (ta1 + tv1), "unit": "nodes/s", "cores": 1,
                             "sample": "first 2 of the 8 beams (%d nodes), numerical libraries limited to one thread: "
                                       "attention %.2f s + verify %.2f s" % (w2.n_nodes, ta1, tv1)}
    except Exception as e:      # threadpoolctl missing: say so instead of guessing
        res["one_thread"] = {"value": None, "note": "not measured: %s" % e}
    return res


def commit_measurement(dsbd, torch, case, reps=10):
    """Cache commit along the plan of the last step (not part of `value`: it is a row beyond the verification path).
    Policy measured: the first next beam of every source tree continues in its source buffer (tree rows appended),
    every other next beam gets a fresh buffer (whole prefix copied)."""
    w, d, o = case.w, case.sets[0], case.outs[0]
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
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="c5")
    ap.add_argument("--copies", type=int, default=3, help="input copies rotated through (cold caches)")
    ap.add_argument("--t", type=float, default=-1.0, help="threshold of the dynamic width; < 0 = fixed width")
    ap.add_argument("--shared-len", type=int, default=None,
                    help="control run: leading prefix tokens shared by the beams of a prompt (the caches then serve most K/V)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true", help="skip the steps on c4 / c3 / c2 (reported apart from the headline)")
    ap.add_argument("--no-commit", action="store_true", help="skip the (separately reported) cache-commit measurement")
    ap.add_argument("--no-warp", action="store_true", help="skip the (separately reported) warped verification")
    ap.add_argument("--no-draft", action="store_true", help="skip the (separately reported) draft-side sampling step")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="first copy 256 MiB device to device (a kernel of known traffic, for scaling a profiler's byte counters)")
    ap.add_argument("--warp-top-k", type=int, default=10, help="warping of the separately reported runs (the paper's setting)")
    ap.add_argument("--warp-top-p", type=float, default=0.8)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path has no multi-GPU part); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2409_16560_amd as dsbd

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.calibration_copy:
        x = torch.ones(1 << 28, dtype=torch.uint8, device="cuda")
        y = torch.empty_like(x)
        y.copy_(x)
        torch.cuda.synchronize()
        del x, y
    kw = {} if args.shared_len is None else {"shared_len": args.shared_len}
    case = Case(dsbd, torch, args.config, args.copies, args.t, **kw)
    w = case.w

    # ---- the timed region: W untimed steps, then exactly K steps between two synchronisations
    for i in range(args.warmup):
        case.step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        case.step(args.warmup + i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    case.check_faults()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # ---- the same step between HIP events on the launch stream, step by step: median and minimum
    ev_steps = max(100, args.steps)
    ts = case.event_times(case.step, ev_steps)
    # ---- per call (events around each library call)
    br = {name + "_ms": (lambda v: v[len(v) // 2])(case.event_times(fn, 30))
          for name, fn in (("attention", case.attention), ("verify", case.verify), ("verify_select", case.verify_select),
                           ("select", case.select))}
    # ---- per kernel: the library's timing hook stamps the kernel's own start and end (one kernel at a time)
    kernels = []
    step_bytes = case.attn_bytes + case.verify_bytes
    traffic = measured_traffic(dsbd.dsbd_version()) if args.config == "c5" and args.shared_len is None else None
    for name, kid, nbytes, names in (
            ("forest_attention (main kernel)", dsbd.DSBD_KERNEL_ATTENTION, case.attn_bytes, ("forest_attention",)),
            ("vocab_stats_kernel", dsbd.DSBD_KERNEL_VOCAB_STATS, case.verify_bytes, ("vocab_stats_kernel",)),
            ("verify_layers_kernel", dsbd.DSBD_KERNEL_VERIFY_LAYERS, 0, ("verify_layers_kernel",))):
        reps = 30
        dsbd.dsbd_timing_enable(kid, 4 * reps)
        for i in range(reps):
            case.step(i)
        torch.cuda.synchronize()
        kms = dsbd.dsbd_timing_collect(4 * reps)
        dsbd.dsbd_timing_enable(0, 0)
        avg = sum(kms) / max(1, len(kms))
        tr = None
        if traffic:
            hit = [v for k, v in traffic.items() if any(k.startswith(n) for n in names) and "combine" not in k]
            tr = hit[0] if hit else None
        entry = {"kernel": name, "avg_launch_ms": avg, "launches_timed": len(kms), "algorithmic_bytes_per_launch": nbytes,
                 "traffic": tr, "measured": "inside the step (the statistics pass and the layer kernel run side by side on two streams)"}
        if nbytes:
            entry.update({"bound": "hbm", "achieved": nbytes / (avg * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                          "frac": nbytes / (avg * 1e-3) / 1e9 / HBM_PEAK_GBS})
        else:
            entry.update({"bound": "latency", "note": "dependent reductions among its workgroups; it re-reads the logit rows of each layer's input beams from the caches and has no algorithmic bytes of its own"})
        kernels.append(entry)
    kernels.sort(key=lambda e: -e["avg_launch_ms"])

    achieved = step_bytes / (ms_per_step * 1e-3) / 1e9
    res = {
        "metric": "forest nodes verified/sec; achieved HBM GB/s vs peak (1 MI355X)",
        "value": w.n_nodes / (ms_per_step * 1e-3), "unit": "nodes/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 attention (fp32 accumulate), fp32 vocab statistics, fp64 accept/resample decisions",
        "data": "synthetic",
        "config": {"workload": case.describe(), "input_copies_rotated": len(case.sets),
                   **({} if args.shared_len is None else {"control_shared_prefix_tokens": args.shared_len})},
        "roofline": {"bound": "hbm", "kernel": "whole step: forest attention + merge, vocabulary statistics beside the layer kernel (which also writes the next-beam plan)",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": (sum(traffic.values()) if traffic else None),
                     "algorithmic_bytes_per_step": step_bytes, "target_frac": 0.60,
                     "note": "the step is not bound by one kernel; the per-kernel figures are in roofline_kernels (longest first)"},
        "roofline_kernels": kernels,
        "step_algorithmic_bytes": step_bytes,
        "step_hbm_frac": achieved / HBM_PEAK_GBS,
        "step_ms_median": ts[len(ts) // 2], "step_ms_min": ts[0], "step_event_samples": len(ts),
        "breakdown_ms": br,
    }
    # ---- a plain streaming read on the same box: what "HBM-bound" can mean here
    try:
        buf = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        buf.zero_()
        gbs = dsbd.dsbd_stream_read_probe(buf, reps=10)
        res["stream_read_ceiling"] = {"achieved": gbs, "unit": "GB/s", "frac_of_peak": gbs / HBM_PEAK_GBS,
                                      "note": "plain non-temporal 16-byte loads over 1 GiB, best of 10; the step's bytes at this rate: %.1f us"
                                              % (step_bytes / gbs / 1e3)}
        del buf
    except Exception as e:
        res["stream_read_ceiling"] = {"achieved": None, "note": str(e)}

    if not args.no_commit:
        res["next_rows"] = {"kv_commit": commit_measurement(dsbd, torch, case)}
    if not args.no_warp:
        # the same verification with the warping operation on the joints (reported apart from the headline)
        k, p_ = args.warp_top_k, args.warp_top_p
        wws = torch.empty(dsbd.dsbd_verify_forest_workspace_bytes(case.sets[0].forest, w.V, 0, 1, w.W_cap, 0.9, k, p_),
                          dtype=torch.uint8, device="cuda")
        call = lambda i: case.verify(i, workspace=wws, top_k=k, top_p=p_)
        reps = 20
        cts = case.event_times(call, reps)
        dsbd.dsbd_timing_enable(dsbd.DSBD_KERNEL_VERIFY_LAYERS, reps)
        for i in range(reps):
            call(i)
        torch.cuda.synchronize()
        lk = dsbd.dsbd_timing_collect(reps)
        dsbd.dsbd_timing_enable(0, 0)
        case.check_faults()
        # ... and with the dynamic width on top (t = 0.9): the setting of the paper's experiments (warped joints, Section 3.2's width)
        dts = case.event_times(lambda i: case.verify(i, 0.9, workspace=wws, top_k=k, top_p=p_), reps)
        case.check_faults()
        res.setdefault("next_rows", {})["warped_verify"] = {
            "top_k": k, "top_p": p_, "verify_ms": cts[len(cts) // 2], "verify_layers_kernel_ms": sum(lk) / max(1, len(lk)),
            "plain_verify_ms": br["verify_ms"], "warped_dynamic_t0.9_verify_ms": dts[len(dts) // 2],
            "note": "dsbd_verify_forest with top_k / top_p set; not part of value"}
    if not args.no_draft:
        # one beam-sampling step of the small model at the benchmark's shape: 16 beams in, 16 draws out (per prompt)
        W_S = 16
        d0 = case.sets[0]
        zq = d0.logits_q[:W_S].contiguous()
        cum = torch.linspace(-3.0, 0.0, W_S, dtype=torch.float64, device="cuda")
        off = torch.tensor([0, W_S], dtype=torch.int32, device="cuda")
        uu = d0.u_fill.reshape(-1)[:W_S].contiguous()
        dr = {}
        for name, (k, p_) in (("plain", (0, 1.0)), ("warped", (args.warp_top_k, args.warp_top_p))):
            call = lambda i: dsbd.dsbd_draft_layer(off, zq, cum, uu, W_S, max_prompt_beams=W_S, top_k=k, top_p=p_)
            v = case.event_times(call, 20)
            dr[name + "_ms"] = v[len(v) // 2]
        dr.update({"beams_in": W_S, "draws": W_S, "V": w.V, "top_k": args.warp_top_k, "top_p": args.warp_top_p,
                   "note": "dsbd_draft_layer (statistics + sampling kernels, workspace allocated per call); not part of value"})
        res.setdefault("next_rows", {})["draft_layer"] = dr
    if not args.no_other_configs and args.config == "c5" and args.shared_len is None:
        # the other configurations (parity-test cases; here only their step times, apart from the headline)
        # first the benchmark's own configuration with the dynamic width (Section 3.2; t = 0.9 and 0.7) ...
        other = [case.step_summary(60, t=t_) for t_ in (0.9, 0.7)]
        case.check_faults()
        del case
        torch.cuda.empty_cache()
        # ... and with a draft model independent of the target (near-total rejection: the residual path), fixed width
        for cfg, copies, ts_, kw_ in (("c5", 3, (-1.0,), {"draft": "indep"}), ("c4", 2, (-1.0, 0.9), {}),
                                      ("c3", 3, (-1.0,), {}), ("c2", 3, (-1.0,), {})):
            c = Case(dsbd, torch, cfg, copies, ts_[0], **kw_)
            for t_ in ts_:
                e = c.step_summary(60, t=t_)
                if kw_:
                    e["workload"] += ", draft logits independent of the target"
                other.append(e)
            c.check_faults()
            del c
            torch.cuda.empty_cache()
        res["other_configs"] = other
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline()
    print(json.dumps(res))


if __name__ == "__main__":
    main()
