#!/usr/bin/env python3
"""Benchmark of the fused decode stream on one MI355X.

A "step" is one pass of the whole hot path over the live requests: flover_step (admission, one launch per operation
over all live rows, greedy tokens back on the host) followed by flover_reorder_evict (eviction, Algorithm 3, shuffle
copy).  Default workload: the LLaMA-7B-shaped stream (bf16, 128 requests, Poisson arrivals, prompts 32-1024,
log-uniform generation lengths 16-1024), all weights and caches resident in HBM before the timed region.
Pre-processing of arriving requests (flover_add_request) happens between steps and is timed separately.

Prints ONE JSON line (metric = generated tokens/s of the fused stream) with a `roofline` object for the dominant
kernel (ragged decode attention, HBM-bound) and a `cpu_baseline` object (the CPU oracle on a bounded sample).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
STEP_TARGET = 0.60        # stated target: the decode step sustains this fraction of peak HBM bandwidth on the 7B stream


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed steps (0 = the whole stream)")
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="c4", choices=["c4", "c3", "c1", "c2", "c5", "poisson32", "const32", "shuffle32"])
    ap.add_argument("--lambda-ms", type=float, default=500.0,
                    help="poisson32: mean inter-arrival gap in the paper's milliseconds (Section VI-C); converted to "
                         "decode steps with the paper's 5800 ms per 512 iterations")
    ap.add_argument("--interval-ms", type=float, default=500.0,
                    help="const32 / shuffle32: constant gap between two requests in the paper's milliseconds (Section VI-B)")
    ap.add_argument("--gen-max", type=int, default=512,
                    help="shuffle32: generation lengths are uniform on [128, gen-max] (Section VI-D)")
    ap.add_argument("--async-preprocess", action="store_true",
                    help="pre-processing on the library's second stream, beside the fused iterations (Section V-B); "
                         "flover_add_request then only enqueues, and tokens_per_s_incl_preprocess is the figure to read")
    ap.add_argument("--no-overlap-contexts", dest="overlap_contexts", action="store_false",
                    help="pre-processing inside flover_add_request on the iterations' stream (async_preprocess = 0).  The "
                         "default is async_preprocess = 2: the library's two pre-processing streams, waited for by the "
                         "next iteration, so that the context passes of requests that arrive together run side by side; "
                         "same schedule and results, the iterations are not overlapped")
    ap.add_argument("--pipeline", type=int, default=2, metavar="D",
                    help="pipelined token return: keep up to D (1..3) iterations submitted before collecting the oldest "
                         "(flover_step_submit / flover_step_collect); 0 = the synchronous flover_step, which also gives the "
                         "per-live-row-count breakdown")
    ap.add_argument("--by-length", action="store_true",
                    help="Algorithm 3 on entries weighted by cached length (fewest bytes moved) instead of 0/1 occupancy")
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (debug only; reported)")
    ap.add_argument("--requests", type=int, default=0, help="override the number of requests (debug only; reported)")
    ap.add_argument("--profile-level", type=int, default=1)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--seed", type=int, default=4)
    ap.add_argument("--cached-context", action="store_true",
                    help="profiler runs: requests join with their context cache taken as present (no pre-processing "
                         "kernels), so every launch in the trace is a fused-iteration launch")
    ap.add_argument("--shuffle-off", action="store_true",
                    help="the variant without memory shuffle (Section VI-D): finished slots stay inside the window as holes")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="MiB",
                    help="only run the plain copy kernel on MiB mebibytes, 10 times (reference for profiler byte counters)")
    return ap.parse_args()


def step_bytes(cfg, lens):
    """Algorithmic bytes one fused step has to move: weights once, each row's own KV rows, the new KV rows, embedding
    rows, fp32 logits."""
    import flover_synth as synth
    e = synth.DTYPE_BYTES[cfg.dtype]
    kvb = cfg.kv_bytes_per_token()
    M = len(lens)
    return cfg.weight_bytes_per_step() + sum(l + 1 for l in lens) * kvb + M * kvb + M * cfg.H * e + M * cfg.V * 4


def run_stream(srv, cfg, reqs, max_steps, cached=False, async_pre=False):
    """Drives the stream; returns totals.  Steps are bracketed by host clocks; flover_step and flover_reorder_evict
    both return only after their GPU work has completed.  Per-step bookkeeping is kept to array operations so the
    Python driver adds as little as possible between two steps."""
    import numpy as np
    import torch
    pending = sorted(reqs, key=lambda r: (r.arrival_step, r.req_id))
    idx_of = {r.req_id: k for k, r in enumerate(reqs)}
    lens = np.zeros(len(reqs), np.int64)          # cached rows per request (by index in reqs)
    i = done = s = 0
    tokens = 0
    t_steps = t_pre = 0.0
    moves = 0
    bytes_moved = 0
    rec_n, rec_t, rec_len = [], [], []
    clock = time.perf_counter
    torch.cuda.synchronize()
    while done < len(reqs) and (max_steps <= 0 or s < max_steps):
        if i < len(pending) and pending[i].arrival_step <= s:
            t0 = clock()
            while i < len(pending) and pending[i].arrival_step <= s:
                r = pending[i]
                if cached:
                    srv.add_request_cached(r.req_id, len(r.prompt) - 1, int(r.prompt[-1]), r.gen_len)
                else:
                    srv.add_request(r.req_id, r.prompt, r.gen_len)
                lens[idx_of[r.req_id]] = len(r.prompt) - 1
                i += 1
            if not async_pre:
                torch.cuda.synchronize()
            t_pre += clock() - t0
        t1 = clock()
        out = srv.step()
        rr = srv.reorder_evict()
        dt = clock() - t1
        t_steps += dt
        n = out.n_live
        if n:
            ids = np.fromiter((idx_of[int(r)] for r in out.req_id), np.int64, n)
            rec_len.append(int(lens[ids].sum()))
            lens[ids] += 1
            done += int(out.finished.sum())
        else:
            rec_len.append(0)
        rec_n.append(n)
        rec_t.append(dt)
        tokens += n
        moves += len(rr.moves)
        bytes_moved += rr.bytes_moved
        s += 1
    e = __import__("flover_synth").DTYPE_BYTES[cfg.dtype]
    kvb = cfg.kv_bytes_per_token()
    per_step = [(n, t, (cfg.weight_bytes_per_step() + (sl + n) * kvb + n * kvb + n * cfg.H * e + n * cfg.V * 4) if n else 0)
                for n, t, sl in zip(rec_n, rec_t, rec_len)]
    return {"steps": s, "tokens": tokens, "t_steps": t_steps, "t_pre": t_pre, "moves": moves,
            "bytes_moved": bytes_moved, "per_step": per_step, "all_done": done == len(reqs)}


def run_stream_pipelined(srv, cfg, reqs, max_steps, depth, async_pre=False):
    """Same stream with pipelined token return.  Iterations overlap, so only totals are timed: the clock runs from
    the first submission to the last collection, minus the time spent in flover_add_request (pre-processing; the
    pipeline is drained before each arrival burst so that no iteration time is booked there)."""
    import collections
    import numpy as np
    import torch
    pending = sorted(reqs, key=lambda r: (r.arrival_step, r.req_id))
    lens = {}
    q = collections.deque()
    i = done = s = tokens = moves = bytes_moved = 0
    t_pre = 0.0
    tot_bytes = 0
    clock = time.perf_counter
    e = __import__("flover_synth").DTYPE_BYTES[cfg.dtype]
    kvb = cfg.kv_bytes_per_token()

    per_iter = []           # (rows, seconds from the previous collection -- or its own submission -- to its collection, bytes)
    t_prev = 0.0

    def collect():
        nonlocal done, tokens, t_prev
        out = srv.step_collect()
        now = clock()
        n_k, b_k, t_sub = q.popleft()
        per_iter.append((n_k, now - max(t_prev, t_sub), b_k))
        t_prev = now
        tokens += out.n_live
        for rid, fin in zip(out.req_id, out.finished):
            if fin:
                done += 1

    torch.cuda.synchronize()
    t_begin = clock()
    live_lens = {}
    while done < len(reqs) and (max_steps <= 0 or s < max_steps):
        if i < len(pending) and pending[i].arrival_step <= s:
            if not async_pre:
                while q:
                    collect()
            t0 = clock()
            while i < len(pending) and pending[i].arrival_step <= s:
                r = pending[i]
                srv.add_request(r.req_id, r.prompt, r.gen_len)
                live_lens[r.req_id] = [len(r.prompt) - 1, r.gen_len]
                i += 1
            if not async_pre:
                torch.cuda.synchronize()
            t_pre += clock() - t0
        t_sub = clock()
        n = srv.step_submit()
        rr = srv.reorder_evict()
        moves += len(rr.moves)
        bytes_moved += rr.bytes_moved
        s += 1
        if n:
            it_bytes = 0
            if not async_pre:      # lengths of the rows are known on the host: every admitted request that still has budget
                sl = 0
                for rid in list(live_lens):
                    ln = live_lens[rid]
                    sl += ln[0]
                    ln[0] += 1
                    ln[1] -= 1
                    if ln[1] == 0:
                        del live_lens[rid]
                it_bytes = cfg.weight_bytes_per_step() + (sl + n) * kvb + n * kvb + n * cfg.H * e + n * cfg.V * 4
                tot_bytes += it_bytes
            q.append((n, it_bytes, t_sub))
        while q and (len(q) >= depth or n == 0):
            collect()
    while q:
        collect()
    total = clock() - t_begin - t_pre
    return {"steps": s, "tokens": tokens, "t_steps": total, "t_pre": t_pre, "moves": moves, "bytes_moved": bytes_moved,
            "per_step": [(1, total, tot_bytes)], "per_iter": per_iter if not async_pre else [],
            "all_done": done == len(reqs)}


def cpu_baseline(cfg_full, weights_dev, reqs):
    """The oracle as it stands, timed on this machine's host cores on a bounded sample of the same workload: the first three
    requests of the stream live together, their prompts cut to the last 4 tokens, 5 fused steps at full depth and width.
    With 3 to 8 cached rows per request the sample's time is all weight arithmetic: a weights-dominated baseline."""
    import dataclasses
    import numpy as np
    from oracle import oracle as orc
    n_req, n_steps, keep = 3, 5, 4
    cfg = dataclasses.replace(cfg_full, C=n_req, S=64)
    w = {k: v.cpu() for k, v in weights_dev.items()}
    srv = orc.OracleServer(cfg, w)
    for r in reqs[:n_req]:
        srv.add_request(r.req_id, np.asarray(r.prompt[-keep:]), n_steps)
    t0 = time.perf_counter()
    toks = 0
    live = set()
    for _ in range(n_steps):
        out = srv.step(False)
        srv.reorder_evict()
        toks += out.n_live
        live.add(out.n_live)
    dt = time.perf_counter() - t0
    srv.close()
    return {"value": toks / dt, "unit": "tokens/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": "%d requests of the stream live together (%s rows per step), prompts cut to their last %d tokens, "
                      "%d fused steps = %d tokens at full depth (%d layers) and width, cached rows per request %d..%d, "
                      "i.e. weights-dominated; the context passes of the cut prompts are not timed; %.1f s"
                      % (n_req, "/".join(str(x) for x in sorted(live)), keep, n_steps, toks, cfg.L, keep - 1,
                         keep - 1 + n_steps - 1, dt)}


def run_c2(a):
    """Config 2, the decode-attention + reorder micro-benchmark: 256 live requests, 32 heads, head_dim 128, bf16, per-request
    KV length U{1..4096}; every step 10% of the live requests finish at seeded indices, are compacted away by
    flover_reorder_evict, and are replaced by fresh requests (length U{1..4096}, cache content taken as present) so
    that 256 stay live.  Driven through the library's own scheduler on a one-layer model whose other operations are
    negligible (hidden 4096, FFN 64, vocabulary 64); the attention and shuffle-copy kernels are timed with HIP events."""
    import numpy as np
    import torch
    import flover_synth as synth
    import paper_2305_13484_amd as fl
    torch.cuda.set_device(0)
    S, C = 4096, 256
    cfg = synth.ModelConfig("c2_attention_reorder_bf16", synth.ARCH_LLAMA, synth.DT_BF16, 1, 4096, 32, 128, 64, 64, S, C,
                            ln_eps=1e-6)
    weights = synth.make_weights(cfg, a.seed, device="cuda")
    srv = fl.Flover(cfg, weights)
    srv.kv_cache().normal_()          # K, V ~ N(0,1); filling is outside the timed region
    rng = np.random.default_rng(a.seed)
    next_id = 0
    lens = {}

    def refill(k):
        nonlocal next_id
        for _ in range(k):
            n = int(rng.integers(1, S - 1))                # cached rows; the step appends one more
            srv.add_request_cached(next_id, n, int(rng.integers(0, cfg.V)), S - 1 - n)
            lens[next_id] = n
            next_id += 1

    refill(C)
    steps = a.steps or 1000
    for phase, nsteps in (("warm", a.warmup), ("timed", steps)):
        srv.set_profile(1)
        tok = moves = 0
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(nsteps):
            out = srv.step()
            tok += out.n_live
            live = [int(r) for r, f in zip(out.req_id, out.finished) if not f]
            for r in out.req_id:
                lens[int(r)] += 1
            kill = rng.choice(len(live), size=min(26, len(live)), replace=False)
            for j in kill:
                srv.mark_finished(live[j])
            rr = srv.reorder_evict()
            moves += len(rr.moves)
            for r in rr.evicted:
                lens.pop(int(r), None)
            refill(C - (out.n_live - len(rr.evicted)))
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
    prof = srv.get_profile()
    srv.close()
    att, cp = prof["attention"], prof["compact"]
    ach = att["bytes"] / (att["ms"] * 1e-3) / 1e9
    line = {
        "metric": "generated tokens/s per fused decode stream", "value": round(tok / dt, 2), "unit": "tokens/s",
        "n_gpus": 1, "steps": steps, "warmup": a.warmup, "ms_per_step": round(1e3 * dt / steps, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "c2: decode-attention + reorder micro-benchmark, 256 live, 32 heads, head_dim 128, KV length "
                               "U{1..4096}, 10% finish per step at seeded indices, refilled to 256", "seed": a.seed},
        "roofline": {"bound": "hbm", "kernel": "attn_partial_kernel", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": None, "launches": att["launches"],
                     "avg_launch_us": round(1e3 * att["ms"] / att["launches"], 2),
                     "avg_bytes_per_launch": att["bytes"] // att["launches"]},
        "compaction": {"GB/s": round(cp["bytes"] / (cp["ms"] * 1e-3) / 1e9, 1) if cp["launches"] else None,
                       "frac": round(cp["bytes"] / (cp["ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4) if cp["launches"] else None,
                       "launches": cp["launches"], "moves": moves,
                       "avg_launch_us": round(1e3 * cp["ms"] / cp["launches"], 2) if cp["launches"] else None,
                       "avg_bytes_per_launch": cp["bytes"] // cp["launches"] if cp["launches"] else None},
        "cpu_baseline": None,
    }
    print(json.dumps(line))


def committed_traffic(kernel: str):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary of this workload (FETCH_SIZE and
    WRITE_SIZE runs, scaled by the copy probe); None if the summary is absent."""
    path = os.path.join(ROOT, "profiles", "c4_llama7b_first200steps_hbm_counters.txt")
    if not os.path.exists(path):
        return None
    import re
    for line in open(path):
        m = re.match(r"#\s*%s: traffic_bytes_per_launch=(\d+) algorithmic_bytes_per_launch=(\d+)" % kernel, line)
        if m:
            return {"bytes_per_launch": int(m.group(1)), "algorithmic_bytes_per_launch_same_run": int(m.group(2)),
                    "ratio": round(int(m.group(1)) / int(m.group(2)), 4),
                    "window": "first 200 fused steps of this workload, context caches taken as present "
                              "(bench.py --cached-context --steps 200 --warmup 0)",
                    "source": "profiles/c4_llama7b_first200steps_hbm_counters.txt"}
    return None


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one process, one MI355X); --gpus %d is not supported" % a.gpus,
              file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    import flover_synth as synth
    import paper_2305_13484_amd as fl
    fl.load_library()
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)

    if a.copy_probe:
        n = a.copy_probe << 20
        src = torch.zeros(n, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(10):
            fl.k_copy_probe(dst, src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes": n, "launches": 10}))
        return

    if a.workload == "c4":
        cfg = synth.llama_7b(L=a.layers or 32)
        reqs = synth.stream_c4(a.seed, cfg.V, n=a.requests or 128)
        wl = "c4: LLaMA-7B shape bf16, 128 requests, Poisson(2/step) arrivals, prompts U{32..1024}, generation log-uniform 16..1024, max_concurrency 128, max_seq 2048"
    elif a.workload == "c3":
        cfg = synth.gpt_1p3b(L=a.layers or 24)
        reqs = synth.stream_c3(a.seed, cfg.V, n=a.requests or 64)
        wl = "c3: GPT-1.3B shape fp16, 64 requests, Poisson(0.25/step) arrivals, prompts U{64..512}, generation U{32..1024}"
    elif a.workload == "poisson32":
        # Section VI-C: 32 requests of 512 output tokens, exponential inter-arrival gaps; LLaMA-7B shape, 32 slots
        cfg = synth.llama_7b(L=a.layers or 32, C=32, S=1024)
        gap_steps = a.lambda_ms / (5800.0 / 512.0)
        arr = synth.exponential_gap_arrivals(int(a.lambda_ms), 32, gap_steps)
        rng = np.random.default_rng(a.seed)
        reqs = [synth.Request(i, int(t), rng.integers(0, cfg.V, size=128).astype(np.int32), 512) for i, t in enumerate(arr)]
        wl = "poisson32: LLaMA-7B shape bf16, 32 requests x 512 tokens, exponential gaps, mean %.0f ms = %.1f steps" % (
            a.lambda_ms, gap_steps)
    elif a.workload in ("const32", "shuffle32"):
        # Sections VI-B / VI-D: 32 requests a constant interval apart; 512 output tokens each (const32) or
        # generation lengths uniform on [128, gen-max] (shuffle32); LLaMA-7B shape, 32 slots
        gmax = 512 if a.workload == "const32" else a.gen_max
        cfg = synth.llama_7b(L=a.layers or 32, C=32, S=128 + max(512, gmax) + 1)
        gap_steps = max(1, int(round(a.interval_ms / (5800.0 / 512.0))))
        rng = np.random.default_rng(a.seed)
        gens = np.full(32, 512) if a.workload == "const32" else rng.integers(128, gmax + 1, size=32)
        reqs = [synth.Request(i, i * gap_steps, rng.integers(0, cfg.V, size=128).astype(np.int32), int(g))
                for i, g in enumerate(gens)]
        wl = "%s: LLaMA-7B shape bf16, 32 requests %.0f ms = %d steps apart, generation %s" % (
            a.workload, a.interval_ms, gap_steps, "512" if a.workload == "const32" else "U{128..%d}" % gmax)
    elif a.workload == "c5":
        # LLaMA-30B shape: 512 requests contend for as many 2048-token slots (3.05 GiB each) as fit beside the 65 GB of
        # weights; the weights are generated and handed over layer by layer
        import dataclasses
        free = torch.cuda.mem_get_info()[0]
        cfg = None
        for slots in range(64, 7, -4):
            cand = synth.llama_30b(L=a.layers or 60, C=slots)
            if fl.arena_bytes(cand, 1 if a.async_preprocess else (2 if a.overlap_contexts else 0)) + (6 << 30) <= free:
                cfg = cand
                break
        assert cfg is not None, "not enough free device memory for the 30B shape"
        reqs = synth.stream_c5(a.seed, cfg.V, n=a.requests or 512)
        if not a.steps:
            a.steps = 1200
        wl = ("c5: LLaMA-30B shape bf16, 512 requests, bursty Poisson arrivals (1 / 8 per step alternating every 200 "
              "steps), prompts U{16..512}, generation U{8..2048}, max_concurrency %d (what fits in device memory), "
              "first %d steps" % (cfg.C, a.steps))
    elif a.workload == "c1":
        cfg = synth.tiny_gpt()
        reqs = synth.stream_c1(a.seed, cfg.V)
        wl = "c1: tiny GPT fp32, 8 requests"
    else:
        run_c2(a)
        return

    # pre-processing mode of the library: 1 = beside the iterations, 2 = two overlapped streams joined by the next iteration
    a.pre_mode = 1 if a.async_preprocess else (2 if a.overlap_contexts else 0)
    t0 = time.perf_counter()
    cpu = None
    if a.workload == "c5":
        glob, layers = synth.make_weights_layerwise(cfg, a.seed, device="cuda")
        srv = fl.Flover(cfg, glob, shuffle_off=a.shuffle_off, by_length=a.by_length, async_preprocess=a.pre_mode)
        for l, wl_ in enumerate(layers):
            srv.set_layer_weights(l, wl_)
        del glob, layers, wl_
        t_w = time.perf_counter() - t0
        a.pipeline = 0          # requests wait for slots here: the synchronous driver keeps the per-row byte accounting
    else:
        weights = synth.make_weights(cfg, a.seed, device="cuda")
        torch.cuda.synchronize()
        t_w = time.perf_counter() - t0
        srv = fl.Flover(cfg, weights, shuffle_off=a.shuffle_off, by_length=a.by_length, async_preprocess=a.pre_mode)
        if not a.no_cpu_baseline:
            cpu = cpu_baseline(cfg, weights, reqs)
        del weights
    torch.cuda.empty_cache()

    # warm-up: a throwaway stream of a few short requests through the same context
    if a.warmup > 0:
        rng = np.random.default_rng(1)
        wp = min(200, cfg.S // 2)
        warm = [synth.Request(10 ** 6 + i, 0, rng.integers(0, cfg.V, size=wp).astype(np.int32),
                              max(1, min(a.warmup, cfg.S - wp - 1))) for i in range(min(8, cfg.C))]
        run_stream(srv, cfg, warm, 0, cached=a.cached_context, async_pre=a.async_preprocess)

    srv.set_profile(a.profile_level)
    piped = a.pipeline if (not a.cached_context and cfg.eos_id < 0) else 0
    if piped:
        res = run_stream_pipelined(srv, cfg, reqs, a.steps, piped, async_pre=a.async_preprocess)
    else:
        res = run_stream(srv, cfg, reqs, a.steps, cached=a.cached_context, async_pre=a.async_preprocess)
    prof = srv.get_profile()
    srv.close()

    K = res["steps"]
    total = res["t_steps"]
    att = prof["attention"]
    roof = None
    # the committed byte counters were taken on this workload (first 200 steps, see profiles/); not on the others
    traffic = committed_traffic("attn_partial_kernel") if (a.workload == "c4" and not a.layers and not a.requests) else None
    # the counters' bytes per launch belong beside `achieved` only when this run covers the window they were taken on
    same_window = bool(traffic) and a.cached_context and a.steps == 200 and a.warmup == 0
    if att["launches"]:
        ach = att["bytes"] / (att["ms"] * 1e-3) / 1e9
        roof = {"bound": "hbm", "kernel": "attn_partial_kernel (ragged decode attention, one launch per layer)",
                "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4),
                "traffic": traffic["bytes_per_launch"] if same_window else None,
                "traffic_ratio": (traffic or {}).get("ratio"), "traffic_window": (traffic or {}).get("window"),
                "traffic_detail": traffic,
                "timed_launches": att["launches"], "timing": "HIP events that take the dispatch's own start and end time stamps; one layer in eight at "
                                                               "profile level 1",
                "avg_launch_us": round(1e3 * att["ms"] / att["launches"], 2),
                "avg_bytes_per_launch": att["bytes"] // att["launches"]}
    per = res["per_step"]
    tot_bytes = sum(b for _, _, b in per)
    step_gbs = tot_bytes / total / 1e9 if total > 0 else 0.0
    buckets = {}
    # synchronous step: each step is bracketed by host clocks; pipelined: the time from one collection to the next
    # (iterations run back to back on the GPU, so that is the iteration's own time whenever the host keeps up)
    rec = res.get("per_iter", []) if piped else per
    for lo, hi in ((1, 16), (17, 32), (33, 64), (65, 10 ** 9)):
        sel = [(n, t, b) for n, t, b in rec if lo <= n <= hi]
        if sel:
            tt = sum(t for _, t, _ in sel)
            buckets["live_%d_%s" % (lo, hi if hi < 10 ** 9 else "up")] = {
                "steps": len(sel), "ms_per_step": round(1e3 * tt / len(sel), 3),
                "hbm_GBs": round(sum(b for _, _, b in sel) / tt / 1e9, 1)}
    # per-step achieved bandwidth as a distribution
    dist = None
    if rec:
        g = sorted((b / t / 1e9, n) for n, t, b in rec if n and t > 0 and b)
        if g:
            pick = lambda q: round(g[min(len(g) - 1, int(q * len(g)))][0], 1)
            dist = {"p10": pick(0.10), "p50": pick(0.50), "p90": pick(0.90),
                    "token_weighted_mean": round(sum(v * n for v, n in g) / sum(n for _, n in g), 1)}
    gemms = {}
    for k in ("gemm_qkv", "gemm_out", "gemm_ff1", "gemm_ff2", "gemm_lm", "compact"):
        p = prof[k]
        if p["launches"]:
            gemms[k] = {"GB/s": round(p["bytes"] / (p["ms"] * 1e-3) / 1e9, 1), "launches": p["launches"],
                        "avg_us": round(1e3 * p["ms"] / p["launches"], 2)}
    gk = [prof[k] for k in ("gemm_qkv", "gemm_out", "gemm_ff1", "gemm_ff2", "gemm_lm") if prof[k]["launches"]]
    if gk:
        gms, gby = sum(p["ms"] for p in gk), sum(p["bytes"] for p in gk)
        gemms["weight_gemms_all"] = {"GB/s": round(gby / (gms * 1e-3) / 1e9, 1), "frac": round(gby / (gms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                                     "launches": sum(p["launches"] for p in gk),
                                     "timing": "HIP events that take the dispatch's own start and end time stamps; at profile "
                                               "level 1 the middle layer's four GEMMs and the output projection, every fourth "
                                               "iteration"}
    line = {
        "metric": "generated tokens/s per fused decode stream", "value": round(res["tokens"] / total, 2),
        "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": a.warmup, "ms_per_step": round(1e3 * total / K, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": synth.DTYPE_NAME[cfg.dtype],
        "data": "synthetic",
        "config": {"workload": wl, "layers": cfg.L, "requests": len(reqs), "whole_stream": res["all_done"],
                   "seed": a.seed, "cached_context": a.cached_context, "shuffle_off": a.shuffle_off, "by_length": a.by_length,
                   "async_preprocess": a.async_preprocess, "overlap_contexts": a.pre_mode == 2, "pipeline": piped},
        "tokens": res["tokens"], "mean_live": round(res["tokens"] / K, 2),
        "step_hbm_GBs": round(step_gbs, 1), "step_hbm_frac": round(step_gbs / HBM_PEAK_GBS, 4),
        "target": {"step_hbm_frac": STEP_TARGET, "met": bool(step_gbs / HBM_PEAK_GBS >= STEP_TARGET)}, "by_live_rows": buckets,
        "step_hbm_GBs_distribution": dist,
        "per_step_timing": ("time between consecutive collections of pipelined iterations" if piped
                            else "host clock around flover_step + flover_reorder_evict"),
        "preprocess_s": round(res["t_pre"], 3), "tokens_per_s_incl_preprocess": round(res["tokens"] / (total + res["t_pre"]), 2),
        "shuffle_moves": res["moves"], "shuffle_bytes": res["bytes_moved"],
        "total_iterations_from_first_token": K - min(r.arrival_step for r in reqs),
        "overlap": round(res["tokens"] / max(1, K - min(r.arrival_step for r in reqs)) / len(reqs), 4),
        "roofline": roof, "other_kernels": gemms, "cpu_baseline": cpu, "weights_gen_s": round(t_w, 2),
        "context": "paper (A100 80GB, FasterTransformer base): 11x (GPT-J 6B) and 16x (LLaMA 65B, TP-4) speedup over "
                   "FasterTransformer at 32 parallel requests; no absolute tokens/s published",
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
