#!/usr/bin/env python3
"""Benchmark of the DSSD verification step on one MI355X.

A "step" is one pass of the whole hot path -- dssd_verify_batch, dssd_residual_sample,
dssd_bonus_sample back to back on one stream -- over one synthetic batch that is already
resident in HBM.  Prints ONE JSON line:  verified draft positions per second for the whole
step, the HBM roofline figure of the dominant kernel (the row softmax statistics, timed with
HIP events on the launch stream inside the timed region), and the CPU oracle timed on a
bounded sample of the same batch (a reported baseline, not a target).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published peak
EVENT_POOL = 2048       # timing brackets the library keeps per kernel between two resets
MAX_ROUNDS = 8          # early exit: most rounds a step can have

# HBM bytes per launch of row_chunk_stats from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by
# what the same counters read for a plain copy of known size; profiles/step_cfg4_hbm_bytes_pmc.txt).
# Taken in profiler runs of their own, not in the run that prints them, and valid only for the
# sources they were taken with: reported as null once any file the kernel and its launch are made
# of has changed.
PMC_TRAFFIC = {
    "cfg4_B1024_ragged_g1-16_V256000_bf16": {
        "sources_sha256": "356bceb6c3e77400b74ab95efee821a421e29f1cce235e7f0586a8b29a7dd6e9",
        "bytes_per_launch": int((2426287.5 * 2.0 + 4776.9 * 1.0) * 1024),
        "source": "profiles/step_cfg4_hbm_bytes_pmc.txt (separate rocprofv3 --pmc runs, not this run)",
    },
}
KERNEL_SOURCES = ("dssd_device.hpp", "dssd_kernels.hpp", "dssd.hip")   # what row_chunk_stats and its launch are made of


def kernel_sources_digest():
    import hashlib
    d = os.path.join(ROOT, "paper_2507_12000_amd", "csrc")
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        h.update(name.encode())
        with open(os.path.join(d, name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def algorithmic_bytes(inputs, n_rej, C_bonus_fraction):
    """Bytes the method must move in one step: every logits row once; for each rejected
    session its P row again plus its Q row; for each accepted session one chunk of the bonus
    row; the per-position gathers; the result records.  n_rej: rejected sessions per step (a
    mean over the steps measured, so it need not be whole)."""
    V, B, R_L, R_Q = inputs["V"], inputs["B"], inputs["R_L"], inputs["R_Q"]
    s_L = inputs["logits"].element_size()
    stats = R_L * V * s_L
    resid = n_rej * V * (s_L + 4)
    bonus = (B - n_rej) * V * s_L * C_bonus_fraction
    gathers = R_Q * (4 + 4 + s_L)
    return dict(row_stats=stats, residual=resid, bonus=bonus, gathers=gathers, records=12 * B,
                total=stats + resid + bonus + gathers + 12 * B)


def cpu_baseline(inputs, seed, budget_s=12.0):
    """Time the oracle, as it stands, single-threaded, on the first sessions of the batch."""
    import numpy as np
    import torch
    import parity
    from oracle import oracle as O
    B = inputs["B"]
    off = inputs["draft_offsets"]
    off = (np.arange(B + 1) * inputs["gamma"]) if off is None else off.cpu().numpy().astype(np.int64)

    def host_slice(b0, b1):
        q0, q1 = int(off[b0]), int(off[b1])
        sub = dict(inputs)
        sub.update(B=b1 - b0, R_Q=q1 - q0, R_L=q1 - q0 + b1 - b0,
                   logits=inputs["logits"][q0 + b0:q1 + b1], draft_probs=inputs["draft_probs"][q0:q1],
                   draft_tokens=inputs["draft_tokens"][q0:q1],
                   draft_offsets=None if inputs["draft_offsets"] is None
                   else (inputs["draft_offsets"][b0:b1 + 1] - int(off[b0])),
                   inv_temperature=None if inputs["inv_temperature"] is None
                   else inputs["inv_temperature"][b0:b1])
        return parity.to_numpy_inputs(sub), q1 - q0

    def run(h):
        t0 = time.perf_counter()
        O.verify_batch(h["logits"], h["dtype"], h["draft_probs"], h["draft_tokens"], h["V"],
                       gamma=h["gamma"], draft_offsets=h["draft_offsets"],
                       inv_temperature=h["inv_temperature"], seed=seed, step=0)
        return time.perf_counter() - t0

    h1, pos1 = host_slice(0, 1)
    run(h1)                                   # page in, warm the caches
    t1 = max(run(h1), 1e-6)
    per_pos = t1 / max(pos1, 1)
    n = 1
    while n < B and per_pos * int(off[n]) < budget_s:
        n += 1
    h, pos = host_slice(0, n)
    t = run(h)
    out = {"value": pos / t, "unit": "positions/s", "cores": 1, "kind": "oracle",
           "sample": f"first {n} of {B} sessions ({pos} draft positions), one thread, {t:.2f} s",
           "rows_per_s": (pos + n) / t}
    # The same oracle with the sessions (independent units) spread over the host's threads:
    # a second reported figure, sized to about the same wall time.
    cores = min(len(os.sched_getaffinity(0)), int(os.environ.get("OMP_NUM_THREADS", "16")), 16)
    m = n
    while m < B and per_pos * int(off[m]) < budget_s * cores * 0.6:
        m += 1
    if cores > 1 and m >= 2 * cores:
        hm, posm = host_slice(0, m)
        t0 = time.perf_counter()
        parity.run_oracle(hm, seed, 0, workers=cores)
        tm = time.perf_counter() - t0
        out["all_cores"] = {"value": posm / tm, "unit": "positions/s", "cores": cores,
                            "sample": f"first {m} of {B} sessions ({posm} draft positions), "
                                      f"one session per task on {cores} threads, {tm:.2f} s"}
    return out


def time_graph_replays(ctx, D, torch, run, batch, out, inputs, w, args):
    """One step recorded into a HIP graph together with the increment of the step counter the
    kernels read at run time, then replayed: what a serving loop that cannot afford per-launch
    host work would do.  The increment is a launch of its own and is inside the timed region."""
    dev = inputs["logits"].device
    counter = torch.zeros(1, dtype=torch.int64, device=dev)
    batch.step = 0
    batch.step_counter = counter.data_ptr()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        run(batch, out)
        counter.add_(1)
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            run(batch, out)
            counter.add_(1)
    torch.cuda.synchronize()
    for _ in range(args.warmup):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        graph.replay()
    torch.cuda.synchronize()
    el = time.perf_counter() - t0
    assert int(counter.item()) == 1 + args.warmup + args.steps
    return {"metric": "verified_draft_positions_per_sec", "value": inputs["R_Q"] * args.steps / el,
            "unit": "positions/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": 1e3 * el / args.steps, "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "f32", "data": "synthetic",
            "config": {"workload": w.name, "entry": "dssd_step_fused" if args.fused else
                       "dssd_verify_batch+dssd_residual_sample+dssd_bonus_sample",
                       "mode": "hip graph replay, step counter in device memory"},
            "roofline": None, "cpu_baseline": None}


def time_topk_lists(ctx, D, torch, inputs, outs, out, args):
    """The same truncated batch handed over as top-k lists (dssd_step_topk): k (id, value) pairs
    per row instead of V values, so nothing of size V is streamed.  What the step costs when the
    sampler upstream already holds the lists.  Beside the headline, never `value`."""
    def pack(x, used, k):
        chunks_i, chunks_v = [], []
        for r0 in range(0, x.shape[0], 512):                 # by slabs: a temporary of the row size each
            xs, us = x[r0:r0 + 512].float(), used[r0:r0 + 512]
            vals, idx = torch.topk(torch.where(us, xs, torch.full_like(xs, -float("inf"))), k, dim=1)
            keep = torch.isfinite(vals)
            chunks_i.append(torch.where(keep, idx, torch.full_like(idx, -1)).to(torch.int32))
            chunks_v.append(torch.where(keep, vals, torch.zeros_like(vals)))
        return torch.cat(chunks_i).contiguous(), torch.cat(chunks_v).contiguous()

    lg, q = inputs["logits"], inputs["draft_probs"]
    k, cut = 1, 0
    for x, used in ((lg, torch.isfinite), (q, lambda t: t > 0)):
        for r0 in range(0, x.shape[0], 512):
            n = used(x[r0:r0 + 512]).sum(1)
            cut += int((n > 64).sum().item())
            k = max(k, int(n.clamp(max=64).max().item()))
    # rows with more than 64 entries (the sessions whose draft is uniform over V) keep their 64
    # largest: a timing stand-in, counted below
    p_idx, p_logit = pack(lg, torch.isfinite(lg), k)
    q_idx, q_prob = pack(q, q > 0, k)
    off, it = inputs.get("draft_offsets"), inputs.get("inv_temperature")
    dp = lambda t: None if t is None else t.data_ptr()       # noqa: E731
    tb = D.dssd_topk_batch(B=inputs["B"], k=k, gamma=inputs["gamma"], V=inputs["V"], total_drafts=inputs["R_Q"],
                           draft_offsets=dp(off), p_idx=dp(p_idx), p_logit=dp(p_logit), q_idx=dp(q_idx),
                           q_prob=dp(q_prob), draft_tokens=dp(inputs["draft_tokens"]), inv_temperature=dp(it),
                           seed=args.seed, step=0, session_base=0, reserved=0, step_counter=None)
    s = ctx.stream()
    for n in range(args.warmup):
        tb.step = n
        D.dssd_step_topk(ctx.handle, tb, out, s)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for n in range(args.steps):
        tb.step = args.warmup + n
        D.dssd_step_topk(ctx.handle, tb, out, s)
    torch.cuda.synchronize()
    el = time.perf_counter() - t0
    return {"entry": "dssd_step_topk", "k": k, "ms_per_step": 1e3 * el / args.steps,
            "value": inputs["R_Q"] * args.steps / el, "unit": "positions/s",
            "list_bytes_per_step": int((inputs["R_L"] + inputs["R_Q"]) * k * 8), "rows_cut_to_64_entries": cut}


def time_split_path(ctx, D, torch, inputs, outs, args):
    """The same batch through the paper's split: the edge verifies from the uploaded scalars
    q_i(x_i) and draws bonus tokens, exports P_n of every rejected session as fp16 (the downlink
    payload), and the device redraws from the received rows and its own Q rows.  Reported beside
    the headline figure, never as `value`."""
    dev = outs["rejected"].device
    rows = torch.arange(inputs["R_Q"], device=dev)
    qs = inputs["draft_probs"][rows, inputs["draft_tokens"].long()].contiguous()
    batch = D.make_batch(inputs, seed=args.seed, step=0, q_scalars=qs)
    out = D.dssd_out(accepted_len=outs["accepted_len"].data_ptr(), rejected=outs["rejected"].data_ptr(),
                     out_token=outs["out_token"].data_ptr())
    p_rows = torch.empty((inputs["B"], inputs["V"]), device=dev, dtype=torch.float16)
    dbatch = D.make_device_batch(inputs, p_rows, outs["accepted_len"], outs["rejected"], outs["out_token"],
                                 seed=args.seed, step=0)
    s = ctx.stream()

    def one(step):
        batch.step = step
        dbatch.step = step
        D.dssd_verify_batch(ctx.handle, batch, out, s)
        D.dssd_bonus_sample(ctx.handle, batch, out, s)
        D.dssd_export_p_rows(ctx.handle, batch, p_rows.data_ptr(), D.DSSD_F16, s)
        D.dssd_residual_sample_from_p(ctx.handle, dbatch, s)

    for k in range(args.warmup):
        one(k)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        one(args.warmup + k)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    D.dssd_profile_reset(ctx.handle)          # kernel breakdown from a separate region
    D.dssd_profile_enable(ctx.handle, True)
    for k in range(min(args.steps, 50)):
        one(args.warmup + args.steps + k)
    torch.cuda.synchronize()
    D.dssd_profile_enable(ctx.handle, False)
    ks = {}
    for k in range(D.K_COUNT):
        ms, n = D.dssd_profile_read(ctx.handle, k)
        if n:
            ks[D.kernel_name(k)] = 1e3 * ms / n
    n_rej = int(outs["rejected"].sum().item())
    V, s_L = inputs["V"], inputs["logits"].element_size()
    export_bytes = n_rej * V * (s_L + 2)          # read the logits row, write the fp16 row
    device_bytes = n_rej * V * (2 + 4)            # read the fp16 row and the Q row
    return {"ms_per_step": 1e3 * elapsed / args.steps,
            "positions_per_sec": inputs["R_Q"] * args.steps / elapsed,
            "downlink": "fp16", "rejected_sessions": n_rej, "kernels_avg_us": ks,
            "export_p_rows_GBps": export_bytes / (ks["export_p_rows"] * 1e-6) / 1e9 if "export_p_rows" in ks else None,
            "device_resid_mass_GBps": device_bytes / (ks["device_resid_mass"] * 1e-6) / 1e9
            if "device_resid_mass" in ks else None,
            "downlink_bytes_per_rejected_session": V * 2, "uplink_bytes_per_position": 8}


def step_event_stats(torch, run_step, n, first_step):
    """n steps, each bracketed by a pair of HIP events on the launch stream (torch's current
    stream, which the library launches on): median / min / max of one step.  A region of its own:
    the brackets cost queue time, so `value` never comes from here."""
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
    for k, (a, b) in enumerate(pairs):
        a.record()
        run_step(first_step + k)
        b.record()
    torch.cuda.synchronize()
    ms = sorted(a.elapsed_time(b) for a, b in pairs)
    return {"median_ms": ms[len(ms) // 2], "min_ms": ms[0], "max_ms": ms[-1], "steps": n}


PROBE_LOADS = (1, 2, 4, 8)
PROBE_CAPS = (0, 8, 12, 16, 24)


def read_ceiling(ctx, D, torch, buf, nbytes, launches=12):
    """Best rate of the pure-read probe over loads per lane and waves resident per compute unit:
    the read ceiling of this chip for the statistics kernel's kind of access."""
    best, table = None, {}
    for loads in PROBE_LOADS:
        for cap in PROBE_CAPS:
            for _ in range(2):
                D.dssd_probe_read(ctx.handle, buf, nbytes, loads, cap, ctx.stream())
            torch.cuda.synchronize()
            D.dssd_profile_reset(ctx.handle)
            D.dssd_profile_enable(ctx.handle, 1 << D.K_READ_PROBE)
            for _ in range(launches):
                D.dssd_probe_read(ctx.handle, buf, nbytes, loads, cap, ctx.stream())
            torch.cuda.synchronize()
            D.dssd_profile_enable(ctx.handle, False)
            ms, n = D.dssd_profile_read(ctx.handle, D.K_READ_PROBE)
            unit = 1024 * loads
            rate = (nbytes // unit) * unit / (ms / n * 1e-3) / 1e9
            table[f"loads{loads}_cap{cap}"] = round(rate, 1)
            if best is None or rate > best[0]:
                best = (rate, loads, cap)
    return {"GBps": best[0], "loads_per_lane": best[1], "waves_per_cu": best[2], "all_GBps": table}


def config_summary(D, torch, synth, idx, seed, steps, warmup):
    """One benchmark workload, briefly: the three calls and the whole-step call (wall-clock mean,
    and per-step events for the spread), the statistics kernel's rate, the whole step's rate."""
    dev = "cuda:0"
    w = synth.WORKLOADS[idx]
    inputs = synth.generate(w, seed=seed, device=dev)
    torch.cuda.synchronize()
    ctx = D.Context(dev, max_rows=inputs["R_L"], max_V=w.V)
    batch = D.make_batch(inputs, seed=seed, step=0)
    outs, out = D.alloc_out(inputs, dev, debug=False)
    res = {"workload": w.name, "logits_rows": inputs["R_L"], "draft_positions": inputs["R_Q"]}

    def timed(run):
        def one(step):
            batch.step = step
            run(batch, out)
        for k in range(warmup):
            one(k)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(steps):
            one(warmup + k)
        torch.cuda.synchronize()
        mean_ms = 1e3 * (time.perf_counter() - t0) / steps
        return mean_ms, step_event_stats(torch, one, min(steps, 100), warmup + steps)

    D.dssd_profile_reset(ctx.handle)
    D.dssd_profile_enable(ctx.handle, 1 << D.K_ROW_STATS)
    mean3, ev3 = timed(ctx.step)
    D.dssd_profile_enable(ctx.handle, False)
    k1_ms, k1_n = D.dssd_profile_read(ctx.handle, D.K_ROW_STATS)
    meanf, evf = timed(ctx.step_fused)
    rejected = outs["rejected"].cpu().numpy()
    s_L = inputs["logits"].element_size()
    C = -(-w.V // (4096 if s_L == 2 else 2048))
    ab = algorithmic_bytes(inputs, int(rejected.sum()), 1.0 / C)   # the last step's count stands for all
    k1_us = 1e3 * k1_ms / max(k1_n, 1)
    res.update({
        "three_calls": {"ms_per_step": mean3, "positions_per_sec": inputs["R_Q"] / (mean3 * 1e-3), "events": ev3},
        "whole_step_call": {"ms_per_step": meanf, "positions_per_sec": inputs["R_Q"] / (meanf * 1e-3), "events": evf},
        "row_chunk_stats": {"avg_launch_us": k1_us, "GBps": ab["row_stats"] / (k1_us * 1e-6) / 1e9,
                            "frac_of_hbm_peak": ab["row_stats"] / (k1_us * 1e-6) / 1e9 / HBM_PEAK_GBS},
        "step_algorithmic_bytes": ab["total"],
        "step_frac_of_hbm_peak": ab["total"] / (mean3 * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "rejected_sessions": int(rejected.sum()),
        "note": ("launch-latency-bound" if idx == 0 else "inputs fit the last-level cache" if idx == 1 else None),
    })
    ctx.close()
    del inputs, batch, outs, out
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--fused", action="store_true",
                    help="run the step through dssd_step_fused (one launch where the batch allows it)")
    ap.add_argument("--fused-limit", type=int, default=None,
                    help="largest grid (workgroups) dssd_step_fused runs as one launch (library default 512)")
    ap.add_argument("--early-exit", action="store_true",
                    help="DSSD_FLAG_EARLY_EXIT: read each session's rows only up to its first rejection "
                         "(a mode beside the headline, which reads every row)")
    ap.add_argument("--graph", action="store_true",
                    help="record one step (plus the bump of a device-resident step counter) into a HIP "
                         "graph and time its replays; prints a reduced line (no per-kernel events)")
    ap.add_argument("--fused-pair-limit", type=int, default=None,
                    help="largest grid dssd_step_fused runs as two launches (library default 512)")
    ap.add_argument("--top-k", type=int, default=0,
                    help="truncate both models to their top-k tokens (the paper's experiments use k = 10) and "
                         "run the step in sparse-support mode; 0 = the benchmark workload as defined")
    ap.add_argument("--top-k-dense", action="store_true",
                    help="with --top-k: keep the dense samplers (no DSSD_FLAG_SPARSE_SUPPORT)")
    ap.add_argument("--rotate", type=int, default=1,
                    help="cycle through this many copies of the inputs (defeats cache residency of small batches)")
    ap.add_argument("--split", action="store_true",
                    help="also time the edge/device split path (q scalars up, fp16 P rows down)")
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="timed steps (default 200; 1000 for --config 0, whose step is a few microseconds)")
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=4, help="index into the five benchmark workloads")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-all-configs", action="store_true",
                    help="skip the brief runs of the other benchmark workloads after the headline")
    ap.add_argument("--headline-only", action="store_true",
                    help="skip the figures beside the headline (whole-step call, early exit, two batches in "
                         "flight): what a profiler run of the headline kernels wants")
    ap.add_argument("--copy-probe", action="store_true",
                    help="run a plain device copy of known size instead (calibrates the HBM byte counters)")
    args = ap.parse_args()
    if args.steps is None:
        args.steps = 1000 if args.config == 0 else 200
    if args.gpus != 1:
        print("bench.py measures one GPU: the verification step shards by session with no "
              "collective, and no multi-GPU run is part of this benchmark (use --gpus 1).", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2507_12000_amd import binding as D, synth
    if not torch.cuda.is_available():
        print("bench.py needs a GPU (there is no CPU fallback)", file=sys.stderr)
        sys.exit(1)
    dev = "cuda:0"
    if args.copy_probe:
        # 2 GiB read + 2 GiB written per launch by torch's elementwise copy kernel
        n = 1 << 30
        src = torch.arange(n, device=dev, dtype=torch.int16)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / 10
        print(json.dumps({"copy_probe": True, "bytes_read_per_launch": 2 * n, "bytes_written_per_launch": 2 * n,
                          "launches": 10, "GBps_read_plus_write": 4 * n / dt / 1e9}))
        return
    w = synth.WORKLOADS[args.config]
    flags = 0
    if args.top_k > 0:
        w = synth.scaled(w, top_k=args.top_k, name=f"{w.name}_top{args.top_k}")
        flags = 0 if args.top_k_dense else D.FLAG_SPARSE_SUPPORT
    if args.early_exit:
        flags |= D.FLAG_EARLY_EXIT
    inputs = synth.generate(w, seed=args.seed, device=dev)
    torch.cuda.synchronize()
    ctx = D.Context(dev, max_rows=inputs["R_L"], max_V=w.V)
    batch = D.make_batch(inputs, seed=args.seed, step=0, flags=flags)
    outs, out = D.alloc_out(inputs, dev, debug=False)
    # --rotate N: N copies of the inputs at different addresses, used in turn, so that a batch
    # smaller than the chip's 256 MB last-level cache is really read from HBM every step
    copies = [inputs] + [dict(inputs, logits=inputs["logits"].clone(), draft_probs=inputs["draft_probs"].clone())
                         for _ in range(max(args.rotate, 1) - 1)]
    batches = [batch] + [D.make_batch(c, seed=args.seed, step=0, flags=flags) for c in copies[1:]]

    run = ctx.step_fused if args.fused else ctx.step

    def step_fn(_batch, out_):
        bt = batches[step_fn.count % len(batches)]
        bt.step = _batch.step
        step_fn.count += 1
        run(bt, out_)
    step_fn.count = 0
    if args.fused_limit is not None:
        D.dssd_set_fused_limit(ctx.handle, args.fused_limit)
    if args.fused_pair_limit is not None:
        D.dssd_set_fused_pair_limit(ctx.handle, args.fused_pair_limit)
    if args.graph:
        print(json.dumps(time_graph_replays(ctx, D, torch, run, batch, out, inputs, w, args)))
        ctx.close()
        return
    for k in range(args.warmup):
        batch.step = k
        step_fn(batch, out)
    torch.cuda.synchronize()

    def read_kernels():
        ks = {}
        for k in range(D.K_COUNT):
            ms, n = D.dssd_profile_read(ctx.handle, k)
            ks[D.kernel_name(k)] = {"avg_us": 1e3 * ms / max(n, 1), "launches": n}
        return ks

    # Timed region.  Only the dominant kernel is bracketed by HIP events here (every bracket
    # costs queue time; with all kernels bracketed a 15 us step reads as 47 us).
    dom_id = D.K_ROW_STATS_BLOCK if args.early_exit else D.K_ROW_STATS
    if args.fused and not args.early_exit:   # which kernel does this batch run as?  one untimed probe step tells
        D.dssd_profile_reset(ctx.handle)
        D.dssd_profile_enable(ctx.handle, 1 << D.K_FUSED_STEP)
        step_fn(batch, out)
        torch.cuda.synchronize()
        if D.dssd_profile_read(ctx.handle, D.K_FUSED_STEP)[1]:
            dom_id = D.K_FUSED_STEP
    # (with early exit the library may decide that the batch is too small for it and run the
    # default kernels: whichever statistics kernel was launched is the one that is reported)
    cands = [D.K_ROW_STATS_BLOCK, D.K_ROW_STATS, D.K_FUSED_STEP] if args.early_exit else [dom_id]
    # The library holds a fixed pool of event pairs per kernel (EVENT_POOL brackets between two
    # resets): a longer run brackets its first steps only.  Early exit launches the statistics
    # kernel once per round, at most MAX_ROUNDS times a step.
    bracketed = min(args.steps, EVENT_POOL // (MAX_ROUNDS if args.early_exit else 1))
    D.dssd_profile_reset(ctx.handle)
    D.dssd_profile_enable(ctx.handle, sum(1 << k for k in cands))
    t0 = time.perf_counter()
    for k in range(args.steps):
        if k == bracketed:
            D.dssd_profile_enable(ctx.handle, False)   # a host-side switch: nothing is synchronised
        batch.step = args.warmup + k
        step_fn(batch, out)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    D.dssd_profile_enable(ctx.handle, False)
    dom_id = next(k for k in cands if D.dssd_profile_read(ctx.handle, k)[1] > 0)
    dom_ms, dom_n = D.dssd_profile_read(ctx.handle, dom_id)
    assert dom_n == bracketed or (args.early_exit and dom_n % bracketed == 0)
    dom_per_step = dom_n // bracketed      # early exit: the statistics kernel runs once per round

    # How many sessions a step rejects depends on the step's random numbers: the timed steps are
    # run once more, untimed, to count them (the byte figures below use the mean).
    rej_total = torch.zeros((), dtype=torch.int64, device=dev)
    for k in range(args.steps):
        batch.step = args.warmup + k
        step_fn(batch, out)
        rej_total += outs["rejected"].sum()
    mean_rejected = float(rej_total.item()) / max(args.steps, 1)

    # Per-kernel breakdown from a second, separate region with every kernel bracketed.
    D.dssd_profile_reset(ctx.handle)
    D.dssd_profile_enable(ctx.handle, True)
    rej_total.zero_()
    n_breakdown = min(args.steps, 50)
    for k in range(n_breakdown):
        batch.step = args.warmup + args.steps + k
        step_fn(batch, out)
        rej_total += outs["rejected"].sum()
    torch.cuda.synchronize()
    D.dssd_profile_enable(ctx.handle, False)
    kernels = {k: v for k, v in read_kernels().items() if v["launches"]}
    mean_rejected_breakdown = float(rej_total.item()) / max(n_breakdown, 1)
    rejected = outs["rejected"].cpu().numpy()   # the last step's flags, for the paper's link model
    s_L = inputs["logits"].element_size()
    chunk_elems = 4096 if s_L == 2 else 2048
    C = -(-w.V // chunk_elems)
    ab = algorithmic_bytes(inputs, mean_rejected, 1.0 / C)
    if flags & D.FLAG_SPARSE_SUPPORT:   # the samplers touch a few dozen entries per session, not rows
        ab["total"] -= ab["residual"] + ab["bonus"]
        ab["residual"] = ab["bonus"] = 0
    if args.early_exit:   # the rows of the blocks that were visited: their statistics are not NaN
        dbg_t, dbg_out = D.alloc_out(inputs, dev, debug=True)
        batch.step = 0
        step_fn(batch, dbg_out)
        torch.cuda.synchronize()
        visited = int((~torch.isnan(dbg_t["row_stats"][:, 1])).sum().item())
        del dbg_t, dbg_out
        ab["total"] += visited * w.V * s_L - ab["row_stats"]
        ab["row_stats"] = visited * w.V * s_L
        ab["rows_visited"] = visited
    ms_per_step = 1e3 * elapsed / args.steps
    # dominant kernel: the row statistics, or the single fused launch when the step ran as one
    dom = D.kernel_name(dom_id)
    dom_bytes = ab["total"] if dom_id == D.K_FUSED_STEP else ab["row_stats"]
    k1_us = 1e3 * dom_ms / dom_n * dom_per_step   # per step (all rounds together)
    achieved = dom_bytes / (k1_us * 1e-6) / 1e9
    pmc = PMC_TRAFFIC.get(w.name)
    traffic = (pmc["bytes_per_launch"] if pmc and dom == "row_chunk_stats"
               and pmc["sources_sha256"] == kernel_sources_digest() else None)
    result = {
        "metric": "verified_draft_positions_per_sec",
        "value": inputs["R_Q"] * args.steps / elapsed,
        "unit": "positions/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "accum_dtype": "f32", "logits_dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "entry": "dssd_step_fused" if args.fused else
                   "dssd_verify_batch+dssd_residual_sample+dssd_bonus_sample", "B": w.B, "V": w.V, "logits_dtype": w.dtype,
                   "input_copies_rotated": max(args.rotate, 1), "top_k": args.top_k, "sparse_support": bool(flags & D.FLAG_SPARSE_SUPPORT),
                   "early_exit": bool(flags & D.FLAG_EARLY_EXIT),
                   "logits_rows": inputs["R_L"], "draft_positions": inputs["R_Q"],
                   "rejected_sessions": mean_rejected},
        "vocab_rows_per_sec": inputs["R_L"] * args.steps / elapsed,
        "step_algorithmic_GBps": ab["total"] / (ms_per_step * 1e-3) / 1e9,
        "step_frac_of_hbm_peak": ab["total"] / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "kernels_separate_region": kernels,
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic, "traffic_source": pmc["source"] if traffic else None,
                     "algorithmic_bytes_per_launch": dom_bytes, "avg_launch_us": k1_us},
    }
    # The paper's communication model (Sec. 2.2, 3.1) fed with what this step measured: the share
    # of sessions with a rejection is its indicator a.  Link as in Table 1: T_NTT = 20 ms and 8 ms
    # to move one vocabulary distribution (so the rate scales with this workload's V at 16 bit).
    from paper_2507_12000_amd import latency_model as LM
    rate = LM.distribution_bits(w.V, 16) / 8e-3
    link = LM.Link(t_ntt=20e-3, rate_up=rate, rate_down=rate)
    mean_gamma = inputs["R_Q"] / max(w.B, 1)
    result["paper_comm_model"] = {
        "link": "T_NTT 20 ms, 8 ms per vocabulary distribution at 16 bit (Table 1's setting)",
        "mean_gamma": mean_gamma, "rejected_share": float(rejected.mean()),
        "dsd_comm_ms": 1e3 * (mean_gamma * LM.distribution_bits(w.V, 16) / link.rate_up + link.t_ntt),
        "dssd_comm_ms": 1e3 * LM.dssd_comm_time_from_flags(rejected.tolist(), w.V, 16, link)}
    # read ceiling of this chip for the statistics kernel's kind of access, over the same buffer:
    # the best of a sweep of the pure-read probe
    lg = inputs["logits"]
    nbytes = lg.numel() * lg.element_size()
    if nbytes >= (256 << 20):
        ceil = read_ceiling(ctx, D, torch, lg.data_ptr(), nbytes)
        result["roofline"]["measured_read_ceiling_GBps"] = ceil["GBps"]
        result["roofline"]["measured_read_ceiling_probe"] = {k: ceil[k] for k in ("loads_per_lane", "waves_per_cu")}
        result["roofline"]["frac_of_measured_read_ceiling"] = achieved / ceil["GBps"]
        result["roofline"]["probe_sweep_GBps"] = ceil["all_GBps"]
        # the second streaming kernel against the same peak, and against what the probe reaches
        # over as many bytes as one of its launches moves (a launch that short pays its ramp and
        # tail: the ceiling of a 1 GB launch is below that of a 5 GB one)
        rm = kernels.get("resid_mass")
        rm_bytes = mean_rejected_breakdown * w.V * (s_L + 4)   # over the launches that were bracketed
        if rm and rm_bytes >= (64 << 20) and not args.early_exit:
            rate = rm_bytes / (rm["avg_us"] * 1e-6) / 1e9
            short = read_ceiling(ctx, D, torch, lg.data_ptr(), min(nbytes, int(rm_bytes)))
            result["resid_mass_roofline"] = {
                "bound": "hbm", "achieved": rate, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": rate / HBM_PEAK_GBS, "algorithmic_bytes_per_launch": rm_bytes,
                "rejected_sessions_per_launch": mean_rejected_breakdown,
                "avg_launch_us": rm["avg_us"],
                "measured_read_ceiling_same_bytes_GBps": short["GBps"],
                "measured_read_ceiling_probe": {k: short[k] for k in ("loads_per_lane", "waves_per_cu")},
                "frac_of_measured_read_ceiling": rate / short["GBps"]}
    # spread of one step: per-step HIP events in a region of their own
    def one_step(step):
        batch.step = step
        step_fn(batch, out)
    result["step_events"] = step_event_stats(torch, one_step, min(args.steps, 100), args.warmup + 2 * args.steps)
    if not args.fused and not args.early_exit and not args.headline_only:
        # the same step through the single whole-step call (bit-identical outputs; it folds the
        # bonus draw into the accept launch, or runs one launch for small batches): a second
        # figure beside the headline, which stays the three calls
        for k in range(args.warmup):
            batch.step = k
            ctx.step_fused(batch, out)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(args.steps):
            batch.step = args.warmup + k
            ctx.step_fused(batch, out)
        torch.cuda.synchronize()
        el = time.perf_counter() - t0
        result["whole_step_call"] = {"entry": "dssd_step_fused", "ms_per_step": 1e3 * el / args.steps,
                                     "value": inputs["R_Q"] * args.steps / el, "unit": "positions/s"}
    if not args.fused and not args.early_exit and not args.headline_only:
        # the same step when the caller allows rows after a session's first rejection to stay
        # unread (DSSD_FLAG_EARLY_EXIT): same records and tokens, fewer bytes.  A figure beside
        # the headline, which reads every row.
        ee = D.make_batch(inputs, seed=args.seed, step=0, flags=flags | D.FLAG_EARLY_EXIT)
        for k in range(args.warmup):
            ee.step = k
            ctx.step_fused(ee, out)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(args.steps):
            ee.step = args.warmup + k
            ctx.step_fused(ee, out)
        torch.cuda.synchronize()
        el = time.perf_counter() - t0
        result["early_exit_mode"] = {"entry": "dssd_step_fused + DSSD_FLAG_EARLY_EXIT",
                                     "ms_per_step": 1e3 * el / args.steps,
                                     "value": inputs["R_Q"] * args.steps / el, "unit": "positions/s"}
    if not args.fused and not args.early_exit and not args.headline_only:
        # two independent batches in flight, one context and one stream each (here: the same
        # inputs, separate outputs and workspaces): the launches of one fill the ramps and tails
        # of the other.  Throughput of a server with more than one batch queued; not the headline.
        ctx2 = D.Context(dev, max_rows=inputs["R_L"], max_V=w.V)
        outs2, out2 = D.alloc_out(inputs, dev, debug=False)
        pairs = [(ctx, batch, out, torch.cuda.Stream()), (ctx2, D.make_batch(inputs, seed=args.seed, step=0, flags=flags),
                                                          out2, torch.cuda.Stream())]
        for _, _, _, st in pairs:
            st.wait_stream(torch.cuda.current_stream())

        def both(n, first_step):
            for k in range(n):
                cx, bt, ot, st = pairs[k % 2]
                with torch.cuda.stream(st):
                    bt.step = first_step + k
                    cx.step_fused(bt, ot)
        result["two_batches_in_flight"] = {"entry": "dssd_step_fused, two contexts on two streams"}
        for name, fl in (("default", flags), ("early_exit", flags | D.FLAG_EARLY_EXIT)):
            for _, bt, _, _ in pairs:
                bt.flags = fl
            both(args.warmup, 0)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            both(args.steps, args.warmup)
            torch.cuda.synchronize()
            el = time.perf_counter() - t0
            result["two_batches_in_flight"][name] = {"ms_per_step": 1e3 * el / args.steps,
                                                      "value": inputs["R_Q"] * args.steps / el,
                                                      "unit": "positions/s"}
        batch.flags = flags
        ctx2.close()
    if args.top_k > 0 and not args.headline_only:
        result["topk_lists"] = time_topk_lists(ctx, D, torch, inputs, outs, out, args)
    if args.split:
        result["split_path"] = time_split_path(ctx, D, torch, inputs, outs, args)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(inputs, args.seed, budget_s=15.0)
    ctx.close()
    plain = (not args.fused and not args.early_exit and not args.headline_only and not args.no_all_configs
             and args.top_k == 0 and args.rotate <= 1)
    if plain:
        # the other benchmark workloads, briefly (the headline's inputs are released first)
        head = {"workload": w.name, "three_calls": {"ms_per_step": ms_per_step, "events": result["step_events"]},
                "whole_step_call": result.get("whole_step_call"),
                "row_chunk_stats": {"avg_launch_us": k1_us, "GBps": achieved, "frac_of_hbm_peak": achieved / HBM_PEAK_GBS},
                "step_frac_of_hbm_peak": result["step_frac_of_hbm_peak"]}
        del inputs, batch, batches, copies, outs, out, lg
        torch.cuda.empty_cache()
        result["all_configs"] = {}
        for idx in range(len(synth.WORKLOADS)):
            if idx == args.config:
                result["all_configs"][f"cfg{idx}"] = head
            else:
                result["all_configs"][f"cfg{idx}"] = config_summary(D, torch, synth, idx, args.seed,
                                                                    steps=200 if idx < 2 else 60, warmup=10)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
