"""Pins for the oracle's decoder and scheduler: things the paper and the mathematics fix.

  fused == alone            Section V-C: fused iterations perform identical operations per request
  shuffle on == off         Section VI-D compares both variants of the same computation
  shuffle = permutation     Section V-D: valid buffers are moved together, nothing else changes
  cache == recomputation    textbook identity of cached decoding
  closed forms              softmax / norm / rotary special cases
  PyTorch CPU ops           third opinion assembled from library routines
  iteration counters        Section VI-C table definitions
"""
import dataclasses
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import oracle as orc
import flover_synth as synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def run_stream(srv, reqs, want_logits=True, reorder=True, max_steps=100000):
    """Drive a server through a stream counted in decode steps; returns per-request tokens/logits and counters."""
    toks, logits = {}, {}
    pending = sorted(reqs, key=lambda r: (r.arrival_step, r.req_id))
    i, s, live_hist, moves_total = 0, 0, [], 0
    done = 0
    while done < len(reqs) and s < max_steps:
        while i < len(pending) and pending[i].arrival_step <= s:
            r = pending[i]
            srv.add_request(r.req_id, r.prompt, r.gen_len)
            i += 1
        out = srv.step(want_logits)
        live_hist.append(out.n_live)
        for j in range(out.n_live):
            rid = int(out.req_id[j])
            toks.setdefault(rid, []).append(int(out.token[j]))
            if want_logits:
                logits.setdefault(rid, []).append(out.logits[j])
            done += int(out.finished[j])
        if reorder:
            rr = srv.reorder_evict()
            moves_total += len(rr.moves)
        s += 1
    return toks, logits, live_hist, moves_total


@pytest.fixture(scope="module")
def tiny_gpt():
    cfg = synth.tiny_gpt()
    return cfg, synth.make_weights(cfg, 11)


def test_fused_equals_alone_and_shuffle_on_equals_off(tiny_gpt):
    cfg, w = tiny_gpt
    reqs = synth.stream_small(5, cfg.V, n=6, arrive_hi=6, p_lo=3, p_hi=9, g_lo=3, g_hi=12)
    srv = orc.OracleServer(cfg, w)
    toks, logits, live, moves = run_stream(srv, reqs)
    assert max(live) >= 3          # requests really overlap
    for r in reqs:
        t_alone, l_alone = orc.solo_decode(cfg, w, r.prompt, r.gen_len)
        assert len(toks[r.req_id]) == r.gen_len
        assert np.array_equal(np.asarray(toks[r.req_id]), t_alone)
        assert np.array_equal(np.stack(logits[r.req_id]), l_alone)      # bit-identical
    srv_off = orc.OracleServer(cfg, w, shuffle_off=True)
    toks_off, logits_off, _, _ = run_stream(srv_off, reqs)
    for r in reqs:
        assert toks_off[r.req_id] == toks[r.req_id]
        assert np.array_equal(np.stack(logits_off[r.req_id]), np.stack(logits[r.req_id]))


def test_length_weighted_shuffle_is_the_same_rescheduling_and_minimises_rows_moved(tiny_gpt):
    # Algorithm 3 with entries weighted by cached length: results per request unchanged, and at every eviction the
    # rows left outside the chosen window are the fewest any window allows.
    cfg, w = tiny_gpt
    cfg = dataclasses.replace(cfg, C=6)
    reqs = synth.stream_small(21, cfg.V, n=14, arrive_hi=10, p_lo=2, p_hi=30, g_lo=2, g_hi=14)
    ref, _, _, _ = run_stream(orc.OracleServer(cfg, w), reqs, want_logits=False)
    srv = orc.OracleServer(cfg, w, by_length=True)
    pending = sorted(reqs, key=lambda r: (r.arrival_step, r.req_id))
    toks = {r.req_id: [] for r in reqs}
    i = done = s = checked = 0
    while done < len(reqs):
        while i < len(pending) and pending[i].arrival_step <= s:
            srv.add_request(pending[i].req_id, pending[i].prompt, pending[i].gen_len)
            i += 1
        out = srv.step(False)
        for k in range(out.n_live):
            toks[int(out.req_id[k])].append(int(out.token[k]))
        done += int(out.finished.sum())
        st = srv.state()
        lo, hi = st["lo"], st["hi"]
        weights = [0 if st["state"][j] in (0, 3) else int(st["len"][j]) + 1 for j in range(lo, hi)]
        rr = srv.reorder_evict()
        n1 = sum(1 for x in weights if x)
        if n1:
            best = min(sum(weights) - sum(weights[o:o + n1]) for o in range(len(weights) - n1 + 1))
            assert rr.min_cost == best
            outside = sum(weights) - sum(weights[rr.mem_offset:rr.mem_offset + n1])
            assert outside == best
            checked += len(rr.moves) > 0
        s += 1
    assert checked > 0
    for r in reqs:
        assert toks[r.req_id] == ref[r.req_id]


def test_capacity_wait_and_slot_reuse(tiny_gpt):
    cfg, w = tiny_gpt
    cfg = dataclasses.replace(cfg, C=3)
    reqs = synth.stream_small(9, cfg.V, n=7, arrive_hi=2, p_lo=2, p_hi=5, g_lo=2, g_hi=7)
    srv = orc.OracleServer(cfg, w)
    toks, _, live, _ = run_stream(srv, reqs, want_logits=False)
    assert max(live) == 3          # never more than max_concurrency; the rest waited
    for r in reqs:
        t_alone, _ = orc.solo_decode(cfg, w, r.prompt, r.gen_len, want_logits=False)
        assert np.array_equal(np.asarray(toks[r.req_id]), t_alone)


def test_reorder_is_a_pure_permutation(tiny_gpt):
    cfg, w = tiny_gpt
    srv = orc.OracleServer(cfg, w)
    rng = np.random.default_rng(2)
    for rid in range(8):
        srv.add_request(rid, rng.integers(0, cfg.V, size=int(rng.integers(2, 7))), 20)
    for _ in range(3):
        srv.step(False)
        srv.reorder_evict()
    for rid in (1, 2, 5):
        srv.mark_finished(rid)
    st = srv.state()

    def snapshot():
        st = srv.state()
        snap = {}
        for s in range(cfg.C):
            if st["state"][s] in (1, 2):
                kv = [srv.read_kv(l, which, s, h, int(st["len"][s])) for l in range(cfg.L) for which in (0, 1)
                      for h in range(cfg.nh)]
                snap[int(st["req_id"][s])] = (int(st["len"][s]), int(st["next_token"][s]), int(st["generated"][s]),
                                              np.stack(kv).tobytes())
        return snap

    srv_state_before = {k: v for k, v in snapshot().items() if k not in (1, 2, 5)}
    rr = srv.reorder_evict()
    assert sorted(rr.evicted.tolist()) == [1, 2, 5]
    after = snapshot()
    assert after.keys() == srv_state_before.keys()
    for k in after:
        assert after[k] == srv_state_before[k]
    st = srv.state()
    occ = [1 if s in (1, 2) else 0 for s in st["state"]]
    assert occ == [0] * st["lo"] + [1] * 5 + [0] * (cfg.C - st["lo"] - 5)
    assert st["hi"] - st["lo"] == 5 == rr.new_size
    # occupancy was 1 0 0 1 1 0 1 1 -> best window holds 4 of the 5, one move
    assert len(rr.moves) == rr.min_cost == 1
    kvb = cfg.kv_bytes_per_token()
    assert rr.bytes_moved == 2 * sum(srv_state_before[int(st["req_id"][d])][0] for _, d in rr.moves) * kvb


def test_eos_finishes_request(tiny_gpt):
    cfg, w = tiny_gpt
    prompt = [5, 9, 200]
    t_alone, _ = orc.solo_decode(cfg, w, prompt, 12, want_logits=False)
    eos = int(t_alone[4])
    first = int(np.argmax(t_alone == eos))
    cfg_eos = dataclasses.replace(cfg, eos_id=eos)
    t_eos, _ = orc.solo_decode(cfg_eos, w, prompt, 12, want_logits=False)
    assert t_eos.tolist() == t_alone[:first + 1].tolist()      # EOS itself is returned, then the request ends


@pytest.mark.parametrize("make", [synth.tiny_gpt, synth.tiny_llama])
def test_cache_equals_recomputation(make):
    cfg = make()
    w = synth.make_weights(cfg, 21)
    prompt = np.random.default_rng(4).integers(0, cfg.V, size=5)
    toks, logits = orc.solo_decode(cfg, w, prompt, 6)
    seq = list(prompt) + toks.tolist()[:-1]
    full = orc.full_forward(cfg, w, seq)
    # positions P-1 .. P+G-2 of the full pass produced the G generated tokens
    np.testing.assert_allclose(full[len(prompt) - 1:], logits, rtol=0, atol=1e-6 * np.abs(logits).max())
    assert np.array_equal(np.argmax(full[len(prompt) - 1:], axis=1), toks)


# ---- third opinion from PyTorch CPU library ops (fp32 configs)

def torch_forward(cfg, w, tokens):
    T = len(tokens)
    tok = torch.as_tensor(np.asarray(tokens), dtype=torch.long)
    W = {k: v.double() for k, v in w.items()}
    x = W["wte"][tok]
    if cfg.arch == synth.ARCH_GPT:
        x = x + W["wpe"][:T]

    def nrm(x, g, b):
        if cfg.arch == synth.ARCH_GPT:
            return F.layer_norm(x, (cfg.H,), g, b, cfg.ln_eps)
        return x * torch.rsqrt(x.pow(2).mean(-1, keepdim=True) + cfg.ln_eps) * g

    def rot(t):   # [T, nh, d]
        half = cfg.d // 2
        inv = cfg.rope_theta ** (-torch.arange(0, half, dtype=torch.float64) * 2 / cfg.d)
        ang = torch.arange(T, dtype=torch.float64)[:, None] * inv[None, :]
        cs, sn = ang.cos()[:, None, :], ang.sin()[:, None, :]
        a, b = t[..., :half], t[..., half:]
        return torch.cat([a * cs - b * sn, b * cs + a * sn], -1)

    for l in range(cfg.L):
        h = nrm(x, W["ln1_g"][l], W["ln1_b"][l] if "ln1_b" in W else None)
        qkv = F.linear(h, W["wqkv"][l], W["bqkv"][l] if "bqkv" in W else None)
        q, k, v = [t.reshape(T, cfg.nh, cfg.d) for t in qkv.split(cfg.H, dim=-1)]
        if cfg.arch == synth.ARCH_LLAMA:
            q, k = rot(q), rot(k)
        a = F.scaled_dot_product_attention(q.transpose(0, 1), k.transpose(0, 1), v.transpose(0, 1), is_causal=True)
        a = a.transpose(0, 1).reshape(T, cfg.H)
        x = x + F.linear(a, W["wo"][l], W["bo"][l] if "bo" in W else None)
        h = nrm(x, W["ln2_g"][l], W["ln2_b"][l] if "ln2_b" in W else None)
        if cfg.arch == synth.ARCH_GPT:
            m = F.linear(F.gelu(F.linear(h, W["w1"][l], W["b1"][l]), approximate="tanh"), W["w2"][l], W["b2"][l])
        else:
            m = F.linear(F.silu(F.linear(h, W["w1"][l])) * F.linear(h, W["wu"][l]), W["w2"][l])
        x = x + m
    h = nrm(x, W["lnf_g"], W["lnf_b"] if "lnf_b" in W else None)
    return F.linear(h, W["wte"] if cfg.arch == synth.ARCH_GPT else W["wlm"]).numpy()


@pytest.mark.parametrize("make", [synth.tiny_gpt, synth.tiny_llama])
def test_against_pytorch_cpu_ops(make):
    cfg = make()
    w = synth.make_weights(cfg, 33)
    seq = np.random.default_rng(8).integers(0, cfg.V, size=9)
    ref = torch_forward(cfg, w, seq)
    got = orc.full_forward(cfg, w, seq)
    assert np.abs(got - ref).max() <= 1e-5 * np.abs(ref).max()
    # and through the cached path
    toks, logits = orc.solo_decode(cfg, w, seq[:4], 3)
    ref2 = torch_forward(cfg, w, list(seq[:4]) + toks.tolist()[:-1])[3:]
    assert np.abs(logits - ref2).max() <= 1e-5 * np.abs(ref2).max()
    assert np.array_equal(np.argmax(ref2, axis=1), toks)


@pytest.mark.parametrize("dtype", [synth.DT_BF16, synth.DT_F16])
def test_sixteen_bit_config_stays_close_to_fp32_library_result(dtype):
    # rounding points only perturb: the 16-bit oracle stays within the format's precision of the unrounded math
    cfg = synth.tiny_llama(dtype)
    w = synth.make_weights(cfg, 35)
    seq = np.random.default_rng(9).integers(0, cfg.V, size=7)
    ref = torch_forward(cfg, w, seq)
    got = orc.full_forward(cfg, w, seq)
    tol = 2e-2 if dtype == synth.DT_BF16 else 4e-3
    err = np.abs(got - ref).max() / np.abs(ref).max()
    assert 0 < err <= tol


# ---- storage formats against the library's conversions

@pytest.mark.parametrize("dtype,tdt", [(synth.DT_BF16, torch.bfloat16), (synth.DT_F16, torch.float16),
                                       (synth.DT_F32, torch.float32)])
def test_rounding_matches_library_conversion(dtype, tdt):
    rng = np.random.default_rng(1)
    vals = np.concatenate([rng.standard_normal(2000) * 10.0 ** rng.integers(-6, 4, size=2000),
                           [0.0, 1.0, -1.0, 1.00390625, 1.001953125, 65504.0, 65520.0, 6e-8, 3e-8, 1e-40]])
    vals = vals.astype(np.float32).astype(np.float64)     # the product rounds from fp32 values
    ref = torch.from_numpy(vals).float().to(tdt).double().numpy()
    got = np.asarray([orc.round_to(v, dtype) for v in vals])
    assert np.array_equal(got, ref)


@pytest.mark.parametrize("dtype,tdt", [(synth.DT_BF16, torch.bfloat16), (synth.DT_F16, torch.float16),
                                       (synth.DT_F32, torch.float32)])
def test_gemm_reads_storage_formats_like_the_library(dtype, tdt):
    g = torch.Generator().manual_seed(5)
    x = torch.randn((5, 96), generator=g).to(tdt)
    W = torch.randn((17, 96), generator=g).to(tdt)
    ref = (x.double() @ W.double().T).numpy()
    got = orc.gemm(dtype, x, W)
    np.testing.assert_allclose(got, ref, rtol=1e-13, atol=1e-13)
    cols = [16, 3, 3, 0]
    np.testing.assert_allclose(orc.gemm(dtype, x, W, cols), ref[:, cols], rtol=1e-13, atol=1e-13)


# ---- closed forms of the attention step

def test_attention_closed_forms():
    dtype = synth.DT_BF16
    q, k, v, slots, lens = synth.attention_case(3, M=6, C=9, nh=2, d=64, S=40, dtype=dtype, len_lo=1, len_hi=40)
    lens[0] = 1                       # a single cached row: the output is that V row exactly
    pairs = [(m, h) for m in range(6) for h in range(2)]
    out = orc.attention(dtype, q, k, v, slots, lens, pairs).reshape(6, 2, 64)
    assert np.array_equal(out[0], v[slots[0], :, 0].double().numpy())
    # all K rows equal: uniform weights, output = mean of the V rows
    k2 = k.clone()
    k2[slots[1], :, :lens[1]] = k2[slots[1], :, :1]
    out2 = orc.attention(dtype, q, k2, v, slots, lens, pairs).reshape(6, 2, 64)
    np.testing.assert_allclose(out2[1], v[slots[1], :, :lens[1]].double().mean(1).numpy(), rtol=1e-12, atol=1e-12)
    # library routine on every pair
    for (m, h), o in zip(pairs, out.reshape(-1, 64)):
        n = int(lens[m])
        kk = k[slots[m], h, :n].double()
        vv = v[slots[m], h, :n].double()
        ref = F.scaled_dot_product_attention(q[m, h].double()[None, None], kk[None], vv[None])[0, 0]
        np.testing.assert_allclose(o, ref.numpy(), rtol=1e-10, atol=1e-12)
    # rows of the cache at or beyond len must not matter
    k3, v3 = k.clone(), v.clone()
    for m in range(6):
        k3[slots[m], :, lens[m]:] = 7.0
        v3[slots[m], :, lens[m]:] = -3.0
    assert np.array_equal(orc.attention(dtype, q, k3, v3, slots, lens, pairs).reshape(6, 2, 64), out)


def test_rotary_closed_forms():
    d, theta = 64, 10000.0
    half = d // 2
    rng = np.random.default_rng(12)
    q, k = rng.standard_normal(d), rng.standard_normal(d)
    assert np.array_equal(orc.rope(q, 0), q)                                   # position 0 is the identity
    np.testing.assert_allclose(np.linalg.norm(orc.rope(q, 37)), np.linalg.norm(q), rtol=1e-13)   # a rotation
    base = orc.rope(q, 5) @ orc.rope(k, 2)
    for shift in (1, 100, 1777):                                               # only the relative position matters
        np.testing.assert_allclose(orc.rope(q, 5 + shift) @ orc.rope(k, 2 + shift), base, rtol=1e-9, atol=1e-9)
    assert abs(orc.rope(q, 5) @ orc.rope(k, 3) - base) > 1e-3                  # and it does matter
    # pair i is (i, i + d/2) and turns by pos * theta^(-2i/d): unit vectors at position 1
    for i in (0, 1, half - 1):
        e = np.zeros(d)
        e[i] = 1.0
        r = orc.rope(e, 1)
        ang = theta ** (-2.0 * i / d)
        expect = np.zeros(d)
        expect[i], expect[i + half] = math.cos(ang), math.sin(ang)
        np.testing.assert_allclose(r, expect, atol=1e-15)
        e = np.zeros(d)
        e[i + half] = 1.0
        expect = np.zeros(d)
        expect[i], expect[i + half] = -math.sin(ang), math.cos(ang)
        np.testing.assert_allclose(orc.rope(e, 1), expect, atol=1e-15)
    assert abs(orc.rope(np.eye(d)[0], 1)[0] - 0.5403023058681398) < 1e-15     # cos(1 rad), pair 0 has frequency 1


def test_norm_closed_forms():
    cfg = synth.tiny_llama()
    w = synth.make_weights(cfg, 2)
    w = {k: v.clone() for k, v in w.items()}
    w["lnf_g"].fill_(1.0)
    w["wlm"].zero_()
    for j in range(cfg.H):
        w["wlm"][j, j] = 1.0          # logits[0:H] = final-normed hidden state
    lg = orc.full_forward(cfg, w, [3, 7, 11])
    rms = np.sqrt((lg[:, :cfg.H] ** 2).mean(1))
    np.testing.assert_allclose(rms, 1.0, atol=1e-4)      # RMSNorm with unit gain gives unit rms (up to eps)
    cfg_g = synth.tiny_gpt()
    wg = {k: v.clone() for k, v in synth.make_weights(cfg_g, 2).items()}
    wg["lnf_g"].fill_(1.0)
    wg["lnf_b"].zero_()
    # GPT ties the output matrix to wte: make the first H embeddings the identity to read the hidden state
    wg["wte"][:cfg_g.H].zero_()
    for j in range(cfg_g.H):
        wg["wte"][j, j] = 1.0
    lg = orc.full_forward(cfg_g, wg, [300, 700, 900])[:, :cfg_g.H]
    np.testing.assert_allclose(lg.mean(1), 0.0, atol=1e-6)
    np.testing.assert_allclose(lg.var(1), 1.0, atol=1e-3)     # up to eps / var


# ---- scheduler counters against the Poisson table's definitions

def test_iteration_counters_follow_section_vi_c():
    """32 requests of 512 tokens with exponential gaps: total iterations = (last arrival) + 512 counted from the
    first request's first token, overlap = mean live / 32 = 512 / total iterations; the printed table obeys the
    same relation to within a few points and our totals fall in the statistical band around the printed ones."""
    rows = [tuple(float(x) for x in l.split()) for l in open(os.path.join(GOLD, "poisson_table.txt"))
            if not l.startswith("#") and l.strip()]
    for lam, iters, overlap, _ in rows:
        assert abs(100.0 * 512 / iters - overlap) < 5.0
    cfg = synth.ModelConfig("sched_only", synth.ARCH_GPT, synth.DT_F32, 1, 8, 1, 8, 8, 16, 520, 32)
    w = synth.make_weights(cfg, 1)
    ms_per_iter = 5800.0 / 512.0
    for lam, iters, overlap, _ in (rows[0], rows[7]):
        arr = synth.exponential_gap_arrivals(int(lam), 32, lam / ms_per_iter)
        reqs = [synth.Request(i, int(a), np.asarray([1, 2], np.int32), 512) for i, a in enumerate(arr)]
        srv = orc.OracleServer(cfg, w)
        _, _, live, moves = run_stream(srv, reqs, want_logits=False)
        first = int(arr[0])
        total = len(live) - first
        assert total == int(arr[-1]) - first + 512
        assert moves == 0                                   # equal lengths finish in arrival order (FIFO case)
        my_overlap = 100.0 * (sum(live) / total) / 32
        assert abs(my_overlap - 100.0 * 512 / total) < 1e-9
        mean_total = 31 * lam / ms_per_iter + 512
        sd = math.sqrt(31) * lam / ms_per_iter
        assert abs(total - mean_total) < 4 * sd + 2
        assert abs(iters - mean_total) < 4 * sd + 2        # the printed totals sit in the same band


@pytest.mark.parametrize("mode", ["slots", "by_length"])
def test_scheduler_invariants_under_random_operations(tiny_gpt, mode):
    """Properties the paper's text fixes for the scheduler, checked on the oracle after every call of a long random
    sequence of arrivals, iterations, forced finishes and reorders (capacity 5, so the window fills up, wraps below and
    requests queue):
      * a new request's slot is adjacent to the live region -- the slot behind its end, or the one before its start --
        and an empty region restarts at slot 0 (Section V-C: new request memory is placed adjacent to the current space);
      * a request waits only when neither neighbour is free, and waiting requests are served first come first served
        (Section V-A: more requests wait until a running one finishes);
      * after a reorder the occupied slots are exactly the window [lo, hi): no hole is left (Section V-D);
      * a reorder never changes which requests are live, nor their lengths or budgets; evicted are exactly the finished;
      * every iteration advances every live request by exactly one token."""
    cfg, w = tiny_gpt
    cfg = dataclasses.replace(cfg, C=5, S=48)
    srv = orc.OracleServer(cfg, w, by_length=mode == "by_length")
    rng = np.random.default_rng(17 if mode == "slots" else 18)
    next_id, arrival_order, admitted_order = 0, [], []
    events = {"wait": 0, "wrap": 0, "moves": 0, "restart": 0}
    for op in range(400):
        st = srv.state()
        kind = rng.choice(["add", "add", "step", "step", "step", "finish"])
        if kind == "add":
            P, G = int(rng.integers(1, 9)), int(rng.integers(1, 12))
            lo, hi, waiting = st["lo"], st["hi"], st["waiting"]
            slot = srv.add_request(next_id, rng.integers(0, cfg.V, size=P), G)
            arrival_order.append(next_id)
            if slot >= 0:
                admitted_order.append(next_id)
                assert waiting == 0                                   # nobody overtakes the queue
                assert st["state"][slot] == 0                         # the slot was free
                if lo == hi:
                    assert slot == 0
                    events["restart"] += 1
                else:
                    assert slot in (hi, lo - 1)
                    events["wrap"] += slot == lo - 1
            else:
                events["wait"] += 1
                assert waiting > 0 or (lo == 0 and hi == cfg.C)       # waits only when no neighbour is free
            next_id += 1
        elif kind == "step":
            before = srv.state()
            out = srv.step(False)
            after = srv.state()
            # requests that were waiting and got a slot in this call, in queue order
            newly = [int(after["req_id"][s]) for s in range(cfg.C)
                     if after["state"][s] != 0 and int(after["req_id"][s]) not in
                     [int(before["req_id"][t]) for t in range(cfg.C) if before["state"][t] != 0]]
            admitted_order += sorted(newly, key=arrival_order.index)
            assert list(out.slot) == sorted(out.slot)                  # rows in slot order
            for j in range(out.n_live):
                s = int(out.slot[j])
                was = before["generated"][s] if before["state"][s] in (1, 2) and before["req_id"][s] == out.req_id[j] else 0
                assert after["generated"][s] == was + 1
                if before["state"][s] in (1, 2) and before["req_id"][s] == out.req_id[j]:
                    assert after["len"][s] == before["len"][s] + 1     # one more cached position
            live_before = {int(before["req_id"][s]) for s in range(cfg.C) if before["state"][s] in (1, 2)}
            assert live_before <= {int(r) for r in out.req_id}         # every live request advanced
            rr = srv.reorder_evict()
            st2 = srv.state()
            fin = {int(out.req_id[j]) for j in range(out.n_live) if out.finished[j]}
            assert fin <= {int(r) for r in rr.evicted}
            occ = [int(x != 0) for x in st2["state"]]
            assert occ == [0] * st2["lo"] + [1] * (st2["hi"] - st2["lo"]) + [0] * (cfg.C - st2["hi"])
            survivors = {int(after["req_id"][s]): (int(after["len"][s]), int(after["generated"][s]))
                         for s in range(cfg.C) if after["state"][s] in (1, 2)}
            kept = {int(st2["req_id"][s]): (int(st2["len"][s]), int(st2["generated"][s]))
                    for s in range(cfg.C) if st2["state"][s] != 0}
            assert kept == survivors
            events["moves"] += len(rr.moves)
        else:
            live = [int(st["req_id"][s]) for s in range(cfg.C) if st["state"][s] in (1, 2)]
            if live:
                srv.mark_finished(live[int(rng.integers(len(live)))])
    # first come, first served: slots were handed out in arrival order
    assert admitted_order == arrival_order[:len(admitted_order)]
    assert all(v > 0 for v in events.values()), events
    srv.close()
