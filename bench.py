#!/usr/bin/env python3
"""Benchmark of the DropMatch verify step on one MI355X.

A step is one `dropmatch_verify` call (mask rows -> LM-head contraction + argmax ->
vote/accept) on one batch of seeded synthetic input already resident in HBM.  Prints ONE
JSON line: whole-step throughput in positions/s (a position is one row of h), the roofline
figure of the dominant kernel (its own duration from HIP events recorded by the library on
the launch stream), the same for the compute-bound `batched` workload (object `secondary`,
timed in the same process after the headline workload) and the CPU oracle timed on a
bounded sample of the headline workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload head8b]

Order per workload: an untimed clock-ramp phase (the step repeated for a fixed wall-clock
time: a GPU that has been idle runs its first launches at low clocks; reported as `ramp`,
not part of `warmup`), W untimed warm-up steps, then exactly K timed steps between two
synchronisations.
"""
import argparse
import json
import os
import statistics
import sys
import time

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16, published
FP32_VALU_PEAK_TFLOPS = 157.3
RAMP_SECONDS = 0.4            # untimed clock-ramp phase before the warm-up steps
ROOT = os.path.dirname(os.path.abspath(__file__))


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=100, help="untimed steps after the clock-ramp phase")
    ap.add_argument("--workload", default="head8b", help="head8b (the benchmark line), tiny, bigvocab, tree, batched")
    ap.add_argument("--rule", default="any", choices=["any", "majority", "js", "alg1"],
                    help="acceptance rule: any (Eq. 4, the benchmark line), majority (Eq. 7), js (Eq. 6), "
                         "alg1 (Algorithm 1 = Eq. 6 else Eq. 7); js/alg1 go through dropmatch_verify_js")
    ap.add_argument("--paths", type=int, default=0, help="override K, the dropout paths per row (rows sweep)")
    ap.add_argument("--batch", type=int, default=0, help="override B, the number of sequences (rows sweep)")
    ap.add_argument("--p-drop", type=float, default=-1.0, help="override the dropout probability p (bigvocab sweep)")
    ap.add_argument("--temperature", type=float, default=0.0,
                    help="> 0: path tokens sampled from Softmax(l / temperature) instead of the arg max")
    ap.add_argument("--top-p", type=float, default=0.0,
                    help="with --temperature: 0 < top-p < 1 samples from the nucleus of that distribution only")
    ap.add_argument("--graph", action="store_true",
                    help="time replays of a HIP graph that holds one captured step instead of eager calls")
    ap.add_argument("--static", action="store_true",
                    help="call dropmatch_verify_static (the library's fixed workspace, no context) instead of dropmatch_verify")
    ap.add_argument("--sparse-correction", action="store_true",
                    help="path logits as clean row minus corrections over the dropped dimensions (DM_FLAG_SPARSE_CORRECTION)")
    ap.add_argument("--separate-vote", action="store_true",
                    help="run the acceptance step as its own kernel (DM_FLAG_SEPARATE_VOTE) instead of as the tail of another launch")
    ap.add_argument("--ramp-seconds", type=float, default=RAMP_SECONDS, help="length of the untimed clock-ramp phase")
    ap.add_argument("--secondary", default="auto",
                    help="workload of the `secondary` object: auto = batched when the headline workload is head8b "
                         "with default options, none = leave it out, or a workload name")
    ap.add_argument("--secondary-steps", type=int, default=0, help="timed steps of the secondary workload (0: min(steps, 40))")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing (for profiler runs)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain device copy of 1 GiB (reference for HBM counters under rocprofv3 --pmc)")
    return ap.parse_args()


def read_traffic(workload):
    """HBM bytes per launch of the contraction kernel from the committed counter summary, if any."""
    path = os.path.join(ROOT, "profiles", f"lmhead_{workload}_pmc.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1]), os.path.relpath(path, ROOT)
    except OSError:
        pass
    return None, None


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(wl, W, h, draft, seeds, parent, probs=None, rule=0, temperature=None, top_p=None):
    """The oracle, as it stands, on the first rows of sequence 0 of the same inputs."""
    from oracle import dropmatch_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    n_pos = min(wl.T, 8)
    reps, total = 0, 0.0
    while reps < 20 and total < 10.0:          # about 10 s of CPU work
        t0 = time.perf_counter()
        if probs is not None:
            out = orc.verify_js(h[:1, :n_pos], W, draft[:1, :n_pos], probs[:1, :n_pos], seeds[:1], wl.K, wl.p,
                                rule=rule)
        else:
            out = orc.verify(h[:1, :n_pos], W, draft[:1, :n_pos], seeds[:1], wl.K, wl.p, rule=rule,
                             parent=None if parent is None else parent[:1, :n_pos], temperature=temperature, top_p=top_p)
        total += time.perf_counter() - t0
        reps += 1
        assert out["path_ids"].shape == (1, n_pos, wl.K)
    return {"value": n_pos * reps / total, "unit": "positions/s", "cores": int(threads), "cpu": cpu_model(),
            "kind": "oracle",
            "sample": f"first {n_pos} positions of sequence 0 (K={wl.K} paths each, full V={wl.V}, d={wl.d}), "
                      f"{reps} repetitions, {total:.1f} s in total incl. widening W to float64 each time"}


def describe(wl):
    return (f"{wl.name}: d={wl.d} V={wl.V} {wl.dtype} B={wl.B} T={wl.T} K={wl.K} p={wl.p}"
            + (" tree" if wl.tree else " chain") + (" +bonus row" if wl.bonus else ""))


def run_workload(wl, args, steps, warmup, rule_name="any", temperature=0.0, top_p=0.0, graph=False, static=False,
                 other_kernels=True, keep_host=False, sparse=False):
    """Generate the workload, make it resident, time `steps` steps.  Returns a dict of measurements
    (and, with keep_host, the host arrays the CPU baseline needs)."""
    import numpy as np
    import torch
    from paper_2603_03333_amd import binding as dmb
    from paper_2603_03333_amd import workloads as wk

    bf16 = wl.dtype == "bf16"
    tdt = torch.bfloat16 if bf16 else torch.float32
    # ---- seeded synthetic inputs (host), then resident in HBM
    W = wk.make_weight(wl)
    h = wk.make_hidden(wl)
    seeds = wk.make_seeds(wl)
    W_dev = torch.from_numpy(W).to(tdt).cuda()
    h_dev = torch.from_numpy(h).to(tdt).cuda()
    if not keep_host:
        W = None
    # greedy tokens for planting draft tokens: a plain library matmul, input preparation only
    hf = h_dev.float().reshape(-1, wl.d)
    best_val = torch.full((hf.shape[0],), -float("inf"), device="cuda")
    best_idx = torch.zeros((hf.shape[0],), dtype=torch.int64, device="cuda")
    chunk = 16384
    js = rule_name in ("js", "alg1")
    rule = {"any": dmb.DM_RULE_ANY, "majority": dmb.DM_RULE_MAJORITY, "js": dmb.DM_RULE_JS,
            "alg1": dmb.DM_RULE_JS_OR_MAJORITY}[rule_name]
    clean = np.empty((hf.shape[0], wl.V), dtype=np.float32) if js else None   # undropped logits for the draft stand-in
    for c0 in range(0, wl.V, chunk):
        blk = hf @ W_dev[c0:c0 + chunk].float().T
        if js:
            clean[:, c0:c0 + chunk] = blk.cpu().numpy()
        val, idx = blk.max(dim=1)
        upd = val > best_val
        best_val = torch.where(upd, val, best_val)
        best_idx = torch.where(upd, idx + c0, best_idx)
    del blk, hf
    greedy_np = best_idx.reshape(wl.B, wl.T).cpu().numpy().astype(np.int32)
    parent = None
    if wl.tree:
        parent = wk.make_tree_parents(wl)
        draft = wk.make_tree_draft_ids(wl, parent, greedy_np)
    else:
        draft = wk.make_draft_ids(wl, greedy_np)
    draft_dev = torch.from_numpy(draft).cuda()
    parent_dev = None if parent is None else torch.from_numpy(parent).cuda()

    probs = probs_dev = None
    if js:
        probs = wk.make_draft_probs(wl, clean.reshape(wl.B, wl.T, wl.V))
        probs_dev = torch.from_numpy(probs).cuda()
        del clean

    ctx = dmb.dm_create(0, wl.rows, wl.d, wl.V)
    nucleus = temperature > 0 and 0.0 < top_p < 1.0
    if js or nucleus:
        dmb.dm_reserve_js(ctx, wl.B * wl.T, wl.K)
    prm, keep = dmb.make_params(wl.B, wl.T, wl.K, wl.d, wl.V, dmb.DM_BF16 if bf16 else dmb.DM_F32, wl.p,
                                [int(s) for s in seeds], parent=parent_dev, rule=rule,
                                flags=(dmb.DM_FLAG_SAMPLE_PATHS if temperature > 0 else 0) |
                                      (dmb.DM_FLAG_SPARSE_CORRECTION if sparse else 0) |
                                      (dmb.DM_FLAG_SEPARATE_VOTE if getattr(args, "separate_vote", False) else 0),
                                temperature=temperature, top_p=top_p)
    kernel = dmb.dm_kernel_choice(prm)
    out = dict(accept_len=torch.zeros(wl.B, dtype=torch.int32, device="cuda"),
               best_node=torch.zeros(wl.B, dtype=torch.int32, device="cuda"),
               accept_mask=torch.zeros((wl.B, wl.T), dtype=torch.uint8, device="cuda"),
               hit=torch.zeros((wl.B, wl.T), dtype=torch.uint8, device="cuda"),
               path_ids=torch.zeros((wl.B, wl.T, wl.K), dtype=torch.int32, device="cuda"),
               vote_ids=torch.zeros((wl.B, wl.T), dtype=torch.int32, device="cuda"),
               vote_cnt=torch.zeros((wl.B, wl.T), dtype=torch.int32, device="cuda"))
    if js:
        out["js_draft"] = torch.zeros((wl.B, wl.T), dtype=torch.float32, device="cuda")
        out["js_heads"] = torch.zeros((wl.B, wl.T, wl.K), dtype=torch.float32, device="cuda")
    state = {"stream": torch.cuda.current_stream()}

    def step():
        if js:
            dmb.dropmatch_verify_js(ctx, prm, h_dev, W_dev, draft_dev, probs_dev, stream=state["stream"], **out)
        elif static:
            dmb.dropmatch_verify_static(0, prm, h_dev, W_dev, draft_dev, stream=state["stream"], **out)
        else:
            dmb.dropmatch_verify(ctx, prm, h_dev, W_dev, draft_dev, stream=state["stream"], **out)

    timed = step
    if graph:
        side = torch.cuda.Stream()
        side.wait_stream(state["stream"])
        with torch.cuda.stream(side):
            state["stream"] = side
            step()                                   # warm-up on the capture stream
        side.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            state["stream"] = torch.cuda.current_stream()
            step()
        state["stream"] = torch.cuda.current_stream()
        timed = g.replay

    # ---- clock ramp (untimed, not warm-up): the step itself for a fixed wall-clock time
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ramp_steps = 0
    while time.perf_counter() - t0 < args.ramp_seconds:
        for _ in range(8):
            timed()
        ramp_steps += 8
        torch.cuda.synchronize()
    ramp_s = time.perf_counter() - t0
    for _ in range(warmup):
        timed()
    torch.cuda.synchronize()
    # ---- the timed region.  The library brackets the contraction kernel of a sample of these very
    # calls with two HIP events that take the launch's own timestamps; a captured graph and the
    # context-free entry point hold no events, so there the kernel is timed in the pass after the region.
    live = not graph and not static and not sparse
    stride = max(1, min(8, steps // 10))          # an event pair costs ~4 us of stream time: sample, but get >= 10 samples
    if live:
        dmb.dm_set_profiling_stride(ctx, stride)
        dmb.dm_set_profiling(ctx, 2)
    t0 = time.perf_counter()
    for _ in range(steps):
        timed()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    lm_samples = []
    if live:
        lm_samples = dmb.dm_get_profile_samples(ctx, 1)
        dmb.dm_set_profiling(ctx, False)
        dmb.dm_set_profiling_stride(ctx, 1)

    # ---- per-step durations (median, min): a pass of its own with stream events around every step
    nper = min(steps, 200)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(nper)]
    for a, b in evs:
        a.record()
        timed()
        b.record()
    torch.cuda.synchronize()
    step_ms = [a.elapsed_time(b) for a, b in evs]

    # ---- the other kernels: a pass with events around every kernel
    stages = [0.0] * 5
    pass2 = []
    if sparse:
        pass2 = list(step_ms)      # no per-kernel events on this path: the whole step stands in
    elif other_kernels or not live:
        dmb.dm_set_profiling(ctx, True)
        for _ in range(min(steps, 512)):
            if static:
                dmb.dropmatch_verify(ctx, prm, h_dev, W_dev, draft_dev, **out)   # same kernels, on a context that records
            else:
                step()
        _, stages = dmb.dm_get_profile_stages(ctx)
        pass2 = dmb.dm_get_profile_samples(ctx, 1)
        dmb.dm_set_profiling(ctx, False)
    if not live:
        lm_samples = pass2
    ms_lm = statistics.fmean(lm_samples)

    # ---- what this machine delivers to a bare streaming read of the same W (the achievable ceiling beside the
    # published peak): the library's plain read kernel, stream events around each call, median
    ceiling = None
    if kernel == 1 and wl.rows * 2.0 / (2 if bf16 else 4) <= MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9):
        nbytes = W_dev.numel() * W_dev.element_size() // 16 * 16
        for _ in range(5):
            dmb.dm_debug_stream_read(ctx, W_dev, nbytes)
        sevs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(30)]
        for a, b in sevs:
            a.record()
            dmb.dm_debug_stream_read(ctx, W_dev, nbytes)
            b.record()
        torch.cuda.synchronize()
        t_med = statistics.median(a.elapsed_time(b) for a, b in sevs)
        ceiling = {"achieved": nbytes / (t_med * 1e-3) / 1e9, "unit": "GB/s", "ms": t_med,
                   "what": "plain read kernel (16-byte loads, 2 workgroups per CU) over the same W, median of 30 calls, "
                           "stream events around each call"}

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    esize = 2 if bf16 else 4
    M = wl.rows
    if kernel == 1:          # rows of the masked-row workspace the MFMA kernels read (zero rows past M)
        m_pad = (M + 31) // 32 * 32 if M <= 128 else (M + 255) // 256 * 256
    else:
        m_pad = (M + 127) // 128 * 128
    alg_bytes = wl.V * wl.d * esize + m_pad * wl.d * esize + M * 8
    if js or nucleus:                        # the contraction also writes every logit once (Eq. (5)/(6), nucleus)
        alg_bytes += M * wl.V * 4
    alg_flops = 2.0 * M * wl.d * wl.V
    sec = ms_lm * 1e-3
    if kernel == 1 and M * 2.0 / esize <= MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9):
        roof = {"bound": "hbm", "achieved": alg_bytes / sec / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "algorithmic_bytes_per_launch": alg_bytes}
    elif kernel == 1:
        roof = {"bound": "mfma", "achieved": alg_flops / sec / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "algorithmic_flops_per_launch": alg_flops}
    else:
        roof = {"bound": "alu", "achieved": alg_flops / sec / 1e12, "peak": FP32_VALU_PEAK_TFLOPS, "unit": "TFLOP/s",
                "algorithmic_flops_per_launch": alg_flops}
    roof["frac"] = roof["achieved"] / roof["peak"]
    if ceiling is not None:
        roof["stream_ceiling"] = ceiling
        roof["frac_of_stream_ceiling"] = roof["achieved"] / ceiling["achieved"]
    traffic, tfile = read_traffic(wl.name) if rule_name in ("any", "majority") and temperature == 0 else (None, None)
    roof["traffic"] = traffic
    roof["traffic_source"] = (f"{tfile}: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of this command, "
                              "scaled by the same counters of a 1 GiB copy; a constant read from that file, "
                              "not measured in this run") if traffic else None
    roof["kernel"] = ("lmhead_mfma_kernel" if M <= 128 else "lmhead_mfma_big_kernel") if kernel == 1 \
        else "lmhead_generic_kernel"
    if sparse:
        roof["kernel"] = "whole step: clean rows (contraction kernel, K = 1) + drop_lists_kernel + sparse_correct_kernel + vote"
    roof["kernel_ms"] = ms_lm
    roof["kernel_ms_median"] = statistics.median(lm_samples)
    roof["kernel_ms_min"] = min(lm_samples)
    roof["events_over_calls"] = len(lm_samples)
    roof["kernel_ms_source"] = (f"HIP events on the launch, every {stride}th timed step" if live
                                else "HIP events on the stream, pass after the timed region")
    if other_kernels:
        ms_mask, _, ms_js1, ms_js2, ms_vote = stages
        roof["other_kernels_ms"] = {"mask_rows": ms_mask, "vote_accept": ms_vote}
        roof["kernel_ms_second_pass"] = statistics.fmean(pass2) if pass2 else None
        if js:
            k4 = (wl.K + 3) // 4 * 4
            pass_bytes = wl.B * wl.T * wl.V * 4 * k4          # stored logits read once per JS pass
            roof["other_kernels_ms"].update({"js_stats": ms_js1, "js_terms": ms_js2})
            roof["js_passes"] = {"bound": "hbm", "unit": "GB/s", "peak": HBM_PEAK_GBS,
                                 "js_stats_achieved": pass_bytes / (ms_js1 * 1e-3) / 1e9 if ms_js1 else None,
                                 "js_terms_achieved": (pass_bytes + wl.B * wl.T * wl.V * 4) / (ms_js2 * 1e-3) / 1e9}
        if nucleus:
            k4 = (wl.K + 3) // 4 * 4
            pass_bytes = wl.B * wl.T * wl.V * 4 * k4          # stored logits read once per pass
            roof["other_kernels_ms"]["nucleus_passes"] = ms_js1
            roof["nucleus"] = {"bound": "hbm", "unit": "GB/s", "peak": HBM_PEAK_GBS, "passes": 4,
                               "achieved": 4 * pass_bytes / (ms_js1 * 1e-3) / 1e9}
    dmb.dm_destroy(ctx)
    positions = wl.B * wl.T
    res = {"value": positions / (dt / steps), "ms_per_step": dt / steps * 1e3, "steps": steps, "warmup": warmup,
           "step_ms_median": statistics.median(step_ms), "step_ms_min": min(step_ms),
           "step_ms_source": f"stream events around each of {nper} steps, in a pass after the timed region "
                             "(an event pair adds a few microseconds)",
           "ramp": {"steps": ramp_steps, "seconds": round(ramp_s, 3),
                    "note": "untimed clock-ramp phase before the warm-up steps; not counted as warmup"},
           "roofline": roof, "rows": M, "positions_per_step": positions, "nucleus": nucleus}
    if keep_host:
        res["host"] = (W, h, draft, seeds, parent, probs, rule)
    del W_dev, h_dev
    torch.cuda.empty_cache()
    return res


def main():
    args = parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (got --gpus {args.gpus}); "
              "across GPUs the step would shard by vocabulary rows (one small max-reduce of the argmax keys) "
              "or by sequences (no exchange)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2603_03333_amd import workloads as wk

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    wl = wk.CONFIGS[args.workload]
    default_line = (args.workload == "head8b" and not args.paths and not args.batch and args.p_drop < 0 and
                    args.rule == "any" and args.temperature == 0 and not args.graph and not args.static and
                    not args.sparse_correction)
    if args.paths:
        wl = wl.with_(K=args.paths)
    if args.batch:
        wl = wl.with_(B=args.batch)
    if args.p_drop >= 0.0:
        wl = wl.with_(p=args.p_drop)
    js = args.rule in ("js", "alg1")
    nucleus = args.temperature > 0 and 0.0 < args.top_p < 1.0
    if js and wl.tree:
        print("bench.py: the distribution-level rules are defined for chains only", file=sys.stderr)
        sys.exit(2)
    if nucleus and js:
        print("bench.py: sampled path tokens go with the token-level rules", file=sys.stderr)
        sys.exit(2)
    if args.static and (js or nucleus):
        print("bench.py: --static goes with the token-level rules and without a nucleus", file=sys.stderr)
        sys.exit(2)

    m = run_workload(wl, args, args.steps, args.warmup, args.rule, args.temperature, args.top_p, args.graph,
                     args.static, other_kernels=not args.sparse_correction, keep_host=not args.no_cpu_baseline,
                     sparse=args.sparse_correction)
    result = {
        "metric": "MC-dropout LM-head verify: positions/s; HBM GB/s or MFMA % of peak",
        "value": m["value"],
        "unit": "positions/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": m["ms_per_step"],
        "step_ms_median": m["step_ms_median"], "step_ms_min": m["step_ms_min"], "step_ms_source": m["step_ms_source"],
        "ramp": m["ramp"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if wl.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": describe(wl),
                   "rows": m["rows"], "positions_per_step": m["positions_per_step"], "rule": args.rule,
                   "launch": "hip graph replay" if args.graph else "eager",
                   "entry_point": "dropmatch_verify_static" if args.static else
                                  ("dropmatch_verify_js" if js else "dropmatch_verify"),
                   "path_tokens": (f"sampled, temperature {args.temperature}"
                                   + (f", nucleus top-p {args.top_p}" if nucleus else "")) if args.temperature > 0 else "arg max"},
        "roofline": m["roofline"],
    }
    host = m.pop("host", None)
    if not args.no_cpu_baseline:
        W, h, draft, seeds, parent, probs, rule = host
        result["cpu_baseline"] = cpu_baseline(wl, W, h, draft, seeds, parent, probs, rule,
                                              args.temperature if args.temperature > 0 else None,
                                              args.top_p if nucleus else None)
    del host, m

    # ---- the compute-bound target, in the same process: the batched workload, plain arg max, Eq. (4)
    sec_name = args.secondary
    if sec_name == "auto":
        sec_name = "batched" if default_line else "none"
    if sec_name != "none":
        import gc
        gc.collect()
        swl = wk.CONFIGS[sec_name]
        ssteps = args.secondary_steps or max(1, min(args.steps, 40))
        s = run_workload(swl, args, ssteps, min(args.warmup, 10), other_kernels=False)
        result["secondary"] = {"workload": describe(swl), "rows": s["rows"], "positions_per_step": s["positions_per_step"],
                               "rule": "any", "path_tokens": "arg max", "value": s["value"], "unit": "positions/s",
                               "steps": s["steps"], "warmup": s["warmup"], "ms_per_step": s["ms_per_step"],
                               "step_ms_median": s["step_ms_median"], "step_ms_min": s["step_ms_min"],
                               "ramp": s["ramp"], "roofline": s["roofline"]}
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
