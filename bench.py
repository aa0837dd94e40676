#!/usr/bin/env python3
"""Benchmark of the DropMatch verify step on one MI355X.

A step is one `dropmatch_verify` call (mask rows -> LM-head contraction + argmax ->
vote/accept) on one batch of seeded synthetic input already resident in HBM.  Prints ONE
JSON line: whole-step throughput in positions/s (a position is one row of h), the roofline
figure of the dominant kernel (its own duration from HIP events recorded by the library on
the launch stream) and the CPU oracle timed on a bounded sample of the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload head8b]
"""
import argparse
import json
import os
import sys
import time

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
EVENT_STRIDE = 8              # the dominant kernel is bracketed by HIP events on every 8th timed step
MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16, published
FP32_VALU_PEAK_TFLOPS = 157.3
ROOT = os.path.dirname(os.path.abspath(__file__))


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=100,
                    help="untimed steps; the first ~50 steps after idle run at ramping clocks")
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
                return float(line.split(":", 1)[1])
    except OSError:
        pass
    return None


def cpu_baseline(wl, W, h, draft, seeds, parent, probs=None, rule=0, temperature=None, top_p=None):
    """The oracle, as it stands, on the first rows of sequence 0 of the same inputs."""
    import numpy as np
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
    return {"value": n_pos * reps / total, "unit": "positions/s", "cores": int(threads), "kind": "oracle",
            "sample": f"first {n_pos} positions of sequence 0 (K={wl.K} paths each, full V={wl.V}, d={wl.d}), "
                      f"{reps} repetitions, {total:.1f} s in total incl. widening W to float64 each time"}


def main():
    args = parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (got --gpus {args.gpus}); "
              "across GPUs the step would shard by vocabulary rows (one small max-reduce of the argmax keys) "
              "or by sequences (no exchange)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2603_03333_amd import binding as dmb
    from paper_2603_03333_amd import workloads as wk

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    wl = wk.CONFIGS[args.workload]
    if args.paths:
        wl = wl.with_(K=args.paths)
    if args.batch:
        wl = wl.with_(B=args.batch)
    if args.p_drop >= 0.0:
        wl = wl.with_(p=args.p_drop)
    bf16 = wl.dtype == "bf16"
    tdt = torch.bfloat16 if bf16 else torch.float32

    # ---- seeded synthetic inputs (host), then resident in HBM
    W = wk.make_weight(wl)
    h = wk.make_hidden(wl)
    seeds = wk.make_seeds(wl)
    W_dev = torch.from_numpy(W).to(tdt).cuda()
    h_dev = torch.from_numpy(h).to(tdt).cuda()
    # greedy tokens for planting draft tokens: a plain library matmul, input preparation only
    hf = h_dev.float().reshape(-1, wl.d)
    best_val = torch.full((hf.shape[0],), -float("inf"), device="cuda")
    best_idx = torch.zeros((hf.shape[0],), dtype=torch.int64, device="cuda")
    chunk = 16384
    js = args.rule in ("js", "alg1")
    rule = {"any": dmb.DM_RULE_ANY, "majority": dmb.DM_RULE_MAJORITY, "js": dmb.DM_RULE_JS,
            "alg1": dmb.DM_RULE_JS_OR_MAJORITY}[args.rule]
    if js and wl.tree:
        print("bench.py: the distribution-level rules are defined for chains only", file=sys.stderr)
        sys.exit(2)
    clean = np.empty((hf.shape[0], wl.V), dtype=np.float32) if js else None   # undropped logits for the draft stand-in
    for c0 in range(0, wl.V, chunk):
        blk = hf @ W_dev[c0:c0 + chunk].float().T
        if js:
            clean[:, c0:c0 + chunk] = blk.cpu().numpy()
        val, idx = blk.max(dim=1)
        upd = val > best_val
        best_val = torch.where(upd, val, best_val)
        best_idx = torch.where(upd, idx + c0, best_idx)
    greedy = best_idx.reshape(wl.B, wl.T)
    greedy_np = greedy.cpu().numpy().astype(np.int32)
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
    nucleus = args.temperature > 0 and 0.0 < args.top_p < 1.0
    if nucleus and js:
        print("bench.py: sampled path tokens go with the token-level rules", file=sys.stderr)
        sys.exit(2)
    if js or nucleus:
        dmb.dm_reserve_js(ctx, wl.B * wl.T, wl.K)
    prm, keep = dmb.make_params(wl.B, wl.T, wl.K, wl.d, wl.V, dmb.DM_BF16 if bf16 else dmb.DM_F32, wl.p,
                                [int(s) for s in seeds], parent=parent_dev, rule=rule,
                                flags=dmb.DM_FLAG_SAMPLE_PATHS if args.temperature > 0 else 0,
                                temperature=args.temperature, top_p=args.top_p)
    kernel = dmb.dm_kernel_choice(prm)
    out = dict(accept_len=torch.zeros(wl.B, dtype=torch.int32, device="cuda"),
               best_node=torch.zeros(wl.B, dtype=torch.int32, device="cuda"),
               accept_mask=torch.zeros((wl.B, wl.T), dtype=torch.uint8, device="cuda"),
               hit=torch.zeros((wl.B, wl.T), dtype=torch.uint8, device="cuda"),
               path_ids=torch.zeros((wl.B, wl.T, wl.K), dtype=torch.int32, device="cuda"),
               vote_ids=torch.zeros((wl.B, wl.T), dtype=torch.int32, device="cuda"),
               vote_cnt=torch.zeros((wl.B, wl.T), dtype=torch.int32, device="cuda"))
    stream = torch.cuda.current_stream()

    if js:
        out["js_draft"] = torch.zeros((wl.B, wl.T), dtype=torch.float32, device="cuda")
        out["js_heads"] = torch.zeros((wl.B, wl.T, wl.K), dtype=torch.float32, device="cuda")

    def step():
        if js:
            dmb.dropmatch_verify_js(ctx, prm, h_dev, W_dev, draft_dev, probs_dev, stream=stream, **out)
        else:
            dmb.dropmatch_verify(ctx, prm, h_dev, W_dev, draft_dev, stream=stream, **out)

    timed = step
    if args.graph:
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        with torch.cuda.stream(side):
            stream = side
            step()                                   # warm-up on the capture stream
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            stream = torch.cuda.current_stream()
            step()
        stream = torch.cuda.current_stream()
        timed = graph.replay
    for _ in range(args.warmup):
        timed()
    torch.cuda.synchronize()
    # ---- the timed region.  The library brackets the contraction kernel of (up to 512 of) these very
    # calls with two HIP events on the launch stream; a captured graph holds no events, so with
    # --graph the kernel is timed in the pass after the region instead.
    live = not args.graph
    if live:
        # an event pair costs ~4 us of stream time (2 % of a head8b step): sample every 8th step
        dmb.dm_set_profiling_stride(ctx, EVENT_STRIDE)
        dmb.dm_set_profiling(ctx, 2)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        timed()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    positions = wl.B * wl.T
    n_live, ms_lm_live = 0, 0.0
    if live:
        n_live, stages = dmb.dm_get_profile_stages(ctx)
        ms_lm_live = stages[1]
        dmb.dm_set_profiling(ctx, False)
        dmb.dm_set_profiling_stride(ctx, 1)

    # ---- the other kernels: a second pass with events around every kernel
    nprof = min(args.steps, 512)
    dmb.dm_set_profiling(ctx, True)
    for _ in range(nprof):
        step()
    n_calls, (ms_mask, ms_lm, ms_js1, ms_js2, ms_vote) = dmb.dm_get_profile_stages(ctx)
    dmb.dm_set_profiling(ctx, False)
    ms_lm_pass2 = ms_lm
    if live:
        ms_lm, n_calls = ms_lm_live, n_live

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
        roof = {"bound": "hbm", "achieved": alg_bytes / sec / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s"}
    elif kernel == 1:
        roof = {"bound": "mfma", "achieved": alg_flops / sec / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s"}
    else:
        roof = {"bound": "alu", "achieved": alg_flops / sec / 1e12, "peak": FP32_VALU_PEAK_TFLOPS, "unit": "TFLOP/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["traffic"] = read_traffic(wl.name) if args.rule in ("any", "majority") else None
    roof["kernel"] = ("lmhead_mfma_kernel" if M <= 128 else "lmhead_mfma_big_kernel") if kernel == 1 \
        else "lmhead_generic_kernel"
    roof["kernel_ms"] = ms_lm
    roof["other_kernels_ms"] = {"mask_rows": ms_mask, "vote_accept": ms_vote}
    if js:
        k4 = (wl.K + 3) // 4 * 4
        pass_bytes = wl.B * wl.T * wl.V * 4 * k4          # stored logits read once per JS pass
        roof["other_kernels_ms"].update({"js_stats": ms_js1, "js_terms": ms_js2})
        roof["js_passes"] = {"bound": "hbm", "unit": "GB/s", "peak": HBM_PEAK_GBS,
                             "js_stats_achieved": pass_bytes / (ms_js1 * 1e-3) / 1e9,
                             "js_terms_achieved": (pass_bytes + wl.B * wl.T * wl.V * 4) / (ms_js2 * 1e-3) / 1e9}
    if nucleus:
        k4 = (wl.K + 3) // 4 * 4
        pass_bytes = wl.B * wl.T * wl.V * 4 * k4          # stored logits read once per pass, four passes
        roof["other_kernels_ms"]["nucleus_passes"] = ms_js1
        roof["nucleus"] = {"bound": "hbm", "unit": "GB/s", "peak": HBM_PEAK_GBS, "passes": 4,
                           "achieved": 4 * pass_bytes / (ms_js1 * 1e-3) / 1e9}
    roof["events_over_calls"] = n_calls
    roof["kernel_ms_source"] = (f"HIP events on the launch, every {EVENT_STRIDE}th timed step" if live
                                else "HIP events on the stream, pass after the timed region")
    roof["kernel_ms_second_pass"] = ms_lm_pass2

    result = {
        "metric": "MC-dropout LM-head verify: positions/s; HBM GB/s or MFMA % of peak",
        "value": positions / (dt / args.steps),
        "unit": "positions/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": f"{wl.name}: d={wl.d} V={wl.V} {wl.dtype} B={wl.B} T={wl.T} K={wl.K} p={wl.p}"
                               + (" tree" if wl.tree else " chain") + (" +bonus row" if wl.bonus else ""),
                   "rows": M, "positions_per_step": positions, "rule": args.rule,
                   "launch": "hip graph replay" if args.graph else "eager",
                   "path_tokens": (f"sampled, temperature {args.temperature}"
                                   + (f", nucleus top-p {args.top_p}" if nucleus else "")) if args.temperature > 0 else "arg max"},
        "roofline": roof,
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, W, h, draft, seeds, parent, probs, rule,
                                              args.temperature if args.temperature > 0 else None,
                                              args.top_p if nucleus else None)
    dmb.dm_destroy(ctx)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
