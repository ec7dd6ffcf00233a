"""Shared drivers for the parity tests: run the HIP path and the CPU oracle in lockstep on one request stream."""
import numpy as np
import torch

import flover_synth as synth
from oracle import oracle as orc

TOL = {synth.DT_F32: 1e-5, synth.DT_F16: 2e-2, synth.DT_BF16: 2e-2}   # max |gpu - ref| / max |ref| per logits row


def to_device(weights):
    return {k: v.cuda() for k, v in weights.items()}


class Lockstep:
    """Feeds the same stream to both sides, compares every step, re-synchronises after a near tie."""

    def __init__(self, cfg, weights, shuffle_off=False, by_length=False, overlapped_contexts=False):
        """overlapped_contexts: the library pre-processes on its own two streams (async_preprocess = 2), so the context
        passes of requests that arrive together run side by side and the next iteration waits for them on its stream:
        every request joins at the iteration the oracle admits it in."""
        import paper_2305_13484_amd as fl
        self.cfg = cfg
        self.overlapped = overlapped_contexts
        self.gpu = fl.Flover(cfg, to_device(weights), shuffle_off=shuffle_off, by_length=by_length,
                             async_preprocess=2 if overlapped_contexts else 0)
        self.cpu = orc.OracleServer(cfg, weights, shuffle_off=shuffle_off, by_length=by_length)
        self.tol = TOL[cfg.dtype]
        self.max_err = 0.0
        self.ties = 0
        self.tokens = {}
        self.gpu_logits = {}
        self.steps = 0
        self.moves = 0
        self.compared_rows = 0

    def add(self, req):
        a = self.gpu.add_request(req.req_id, req.prompt, req.gen_len)
        b = self.cpu.add_request(req.req_id, req.prompt, req.gen_len)
        assert a == b, "slot assignment differs"

    def step(self, keep_logits=False):
        g = self.gpu.step(want_logits=True)
        c = self.cpu.step(True)
        assert g.n_live == c.n_live
        assert np.array_equal(g.req_id, c.req_id) and np.array_equal(g.slot, c.slot)
        if g.n_live:
            gl = g.logits.cpu().double().numpy()
            scale = np.abs(c.logits).max(axis=1)
            err = np.abs(gl - c.logits).max(axis=1) / scale
            self.max_err = max(self.max_err, float(err.max()))
            assert err.max() <= self.tol, "logits error %g > %g at step %d" % (err.max(), self.tol, self.steps)
            self.compared_rows += g.n_live
            for j in range(g.n_live):
                rid = int(g.req_id[j])
                if keep_logits:
                    self.gpu_logits.setdefault(rid, []).append(g.logits[j].cpu().clone())
                if g.token[j] != c.token[j]:
                    srt = np.sort(c.logits[j])
                    margin = srt[-1] - srt[-2]
                    assert margin <= 2 * self.tol * scale[j], "token differs beyond a near tie"
                    self.ties += 1
                    if not c.finished[j]:
                        self.gpu.set_next_token(rid, int(c.token[j]))      # teacher forcing
                self.tokens.setdefault(rid, []).append(int(c.token[j]))
            assert np.array_equal(g.finished, c.finished)
        self.steps += 1
        return g, c

    def reorder(self):
        g = self.gpu.reorder_evict()
        c = self.cpu.reorder_evict()
        assert np.array_equal(g.evicted, c.evicted)
        assert (g.mem_offset, g.new_lo, g.new_size, g.min_cost) == (c.mem_offset, c.new_lo, c.new_size, c.min_cost)
        assert g.moves == c.moves
        assert g.bytes_moved == c.bytes_moved
        self.moves += len(g.moves)
        gs, cs = self.gpu.state(), self.cpu.state()
        for k in ("lo", "hi", "waiting"):
            assert gs[k] == cs[k]
        for k in ("state", "len", "generated"):
            assert np.array_equal(gs[k], cs[k]), k
        live = gs["state"] != 0
        assert np.array_equal(gs["req_id"][live], cs["req_id"][live])
        return g, c

    def run(self, reqs, keep_logits=False, max_steps=100000):
        pending = sorted(reqs, key=lambda r: (r.arrival_step, r.req_id))
        i, done, s = 0, 0, 0
        live_hist = []
        while done < len(reqs) and s < max_steps:
            while i < len(pending) and pending[i].arrival_step <= s:
                self.add(pending[i])
                i += 1
            g, _ = self.step(keep_logits)
            live_hist.append(g.n_live)
            done += int(g.finished.sum())
            self.reorder()
            s += 1
        return live_hist

    def close(self):
        self.gpu.close()
        self.cpu.close()


def gpu_run_stream(cfg, weights_dev, reqs, shuffle_off=False, want_logits=True, async_preprocess=False,
                   finish_at=None, stats=None):
    """The HIP path alone over a stream; returns per-request token lists and logits (device tensors).
    finish_at: {req_id: n} forces the request to finish after its n-th token (so that the shuffle has work)."""
    import paper_2305_13484_amd as fl
    srv = fl.Flover(cfg, weights_dev, shuffle_off=shuffle_off, async_preprocess=async_preprocess)
    finish_at = finish_at or {}
    pending = sorted(reqs, key=lambda r: (r.arrival_step, r.req_id))
    toks, logits = {}, {}
    i, done, s = 0, 0, 0
    while done < len(reqs):
        while i < len(pending) and pending[i].arrival_step <= s:
            srv.add_request(pending[i].req_id, pending[i].prompt, pending[i].gen_len)
            i += 1
        out = srv.step(want_logits)
        for j in range(out.n_live):
            rid = int(out.req_id[j])
            toks.setdefault(rid, []).append(int(out.token[j]))
            if want_logits:
                logits.setdefault(rid, []).append(out.logits[j].clone())
            if not out.finished[j] and finish_at.get(rid) == len(toks[rid]):
                srv.mark_finished(rid)
                done += 1
        done += int(out.finished.sum())
        rr = srv.reorder_evict()
        if stats is not None:
            stats["moves"] = stats.get("moves", 0) + len(rr.moves)
            stats["steps"] = stats.get("steps", 0) + 1
        s += 1
    srv.close()
    return toks, logits


def gpu_run_stream_pipelined(cfg, weights_dev, reqs, depth=2, shuffle_off=False, async_preprocess=False, want_logits=True,
                             stats=None):
    """The HIP path with pipelined token return: up to `depth` iterations submitted before the oldest is collected."""
    import collections
    import time
    import torch
    import paper_2305_13484_amd as fl
    srv = fl.Flover(cfg, weights_dev, shuffle_off=shuffle_off, async_preprocess=async_preprocess)
    bufs = [torch.empty((cfg.C, cfg.V), dtype=torch.float32, device="cuda") for _ in range(depth + 1)]
    pending = sorted(reqs, key=lambda r: (r.arrival_step, r.req_id))
    toks, logits = {}, {}
    q = collections.deque()
    i = done = s = k = 0
    deadline = time.time() + 120
    while done < len(reqs):
        assert time.time() < deadline
        while i < len(pending) and pending[i].arrival_step <= s:
            srv.add_request(pending[i].req_id, pending[i].prompt, pending[i].gen_len)
            i += 1
        n = srv.step_submit(bufs[k] if want_logits else None)
        rr = srv.reorder_evict()
        if stats is not None:
            stats["moves"] = stats.get("moves", 0) + len(rr.moves)
            stats["max_outstanding"] = max(stats.get("max_outstanding", 0), len(q) + (1 if n else 0))
        s += 1
        if n:
            q.append(k)
            k = (k + 1) % len(bufs)
        while q and (len(q) >= depth or n == 0):
            b = q.popleft()
            out = srv.step_collect()
            for j in range(out.n_live):
                rid = int(out.req_id[j])
                toks.setdefault(rid, []).append(int(out.token[j]))
                if want_logits:
                    logits.setdefault(rid, []).append(bufs[b][j].clone())
            done += int(out.finished.sum())
    srv.close()
    return toks, logits


class LockstepPipelined(Lockstep):
    """The oracle beside the pipelined form of the iteration (flover_step_submit / flover_step_collect): the scheduler
    state advances at submission, so slot assignment, window, evictions and move lists are compared right after every
    submission + reorder; tokens, finished flags and logits of an iteration arrive `depth` submissions later and are
    compared then with what the oracle's step of the same number produced.  There is no teacher forcing here (the next
    iteration already runs on the device-resident token), so a near tie fails the run: use it where tokens are exact."""

    def __init__(self, cfg, weights, depth=2, shuffle_off=False, by_length=False, overlapped_contexts=False):
        super().__init__(cfg, weights, shuffle_off=shuffle_off, by_length=by_length,
                         overlapped_contexts=overlapped_contexts)
        import collections
        self.depth = depth
        self.queue = collections.deque()          # (oracle step result, logits buffer) of submitted iterations
        self.bufs = [torch.empty((cfg.C, cfg.V), dtype=torch.float32, device="cuda") for _ in range(depth + 1)]
        self.k = 0
        self.max_outstanding = 0

    def submit(self):
        n = self.gpu.step_submit(self.bufs[self.k])
        c = self.cpu.step(True)
        assert n == c.n_live, "rows of the submitted iteration differ"
        if n:
            self.queue.append((c, self.bufs[self.k]))
            self.k = (self.k + 1) % len(self.bufs)
        self.max_outstanding = max(self.max_outstanding, len(self.queue))
        return n, c

    def collect(self):
        c, buf = self.queue.popleft()
        g = self.gpu.step_collect()
        assert g.n_live == c.n_live
        assert np.array_equal(g.req_id, c.req_id) and np.array_equal(g.slot, c.slot)
        gl = buf[:g.n_live].cpu().double().numpy()
        scale = np.abs(c.logits).max(axis=1)
        err = np.abs(gl - c.logits).max(axis=1) / scale
        self.max_err = max(self.max_err, float(err.max()))
        assert err.max() <= self.tol, "logits error %g > %g" % (err.max(), self.tol)
        assert np.array_equal(g.token, c.token), "token differs (pipelined runs cannot be re-synchronised)"
        assert np.array_equal(g.finished, c.finished)
        self.compared_rows += g.n_live
        for j in range(g.n_live):
            self.tokens.setdefault(int(g.req_id[j]), []).append(int(g.token[j]))
        self.steps += 1

    def run(self, reqs, max_steps=100000):
        pending = sorted(reqs, key=lambda r: (r.arrival_step, r.req_id))
        i = s = 0
        finished = 0
        while finished < len(reqs) and s < max_steps:
            while i < len(pending) and pending[i].arrival_step <= s:
                self.add(pending[i])
                i += 1
            n, c = self.submit()
            finished += int(c.finished.sum())
            self.reorder()                         # state comparison: next_token is not part of it (device-resident)
            s += 1
            while self.queue and (len(self.queue) >= self.depth or n == 0):
                self.collect()
        while self.queue:
            self.collect()
        return s


def oracle_per_request(cfg, weights, reqs, shuffle_off=False):
    """Every request's tokens and fp32-valued logits from the oracle's fused run of the stream (by the oracle's own
    pinned invariant these do not depend on the schedule)."""
    srv = orc.OracleServer(cfg, weights, shuffle_off=shuffle_off)
    pending = sorted(reqs, key=lambda r: (r.arrival_step, r.req_id))
    toks, logits = {}, {}
    i = done = s = 0
    while done < len(reqs):
        while i < len(pending) and pending[i].arrival_step <= s:
            srv.add_request(pending[i].req_id, pending[i].prompt, pending[i].gen_len)
            i += 1
        out = srv.step(True)
        for j in range(out.n_live):
            toks.setdefault(int(out.req_id[j]), []).append(int(out.token[j]))
            logits.setdefault(int(out.req_id[j]), []).append(out.logits[j])
        done += int(out.finished.sum())
        srv.reorder_evict()
        s += 1
    srv.close()
    return toks, logits


def assert_matches_oracle_per_request(cfg, got, want, reqs, max_ties=2):
    """got: (tokens, device logits) per request from the HIP path under any schedule; want: oracle_per_request.
    Token by token: logits within the tolerance of the dtype, token ids equal.  Where the ids differ the oracle's two
    best logits must be a near tie (closer than twice the allowed error); nothing can re-synchronise a finished run, so
    the rest of that request is left out.  Returns the worst logits error."""
    tol = TOL[cfg.dtype]
    worst, ties, compared, total = 0.0, 0, 0, 0
    for r in reqs:
        gt, gl = got[0][r.req_id], torch.stack(got[1][r.req_id]).cpu().double().numpy()
        wt, wl = want[0][r.req_id], np.stack(want[1][r.req_id])
        assert len(gt) == len(wt) == r.gen_len
        total += r.gen_len
        for t in range(r.gen_len):
            scale = np.abs(wl[t]).max()
            err = float(np.abs(gl[t] - wl[t]).max() / scale)
            worst = max(worst, err)
            assert err <= tol, (r.req_id, t, err)
            compared += 1
            if gt[t] != wt[t]:
                srt = np.sort(wl[t])
                assert srt[-1] - srt[-2] <= 2 * tol * scale, "tokens of request %d differ beyond a near tie" % r.req_id
                ties += 1
                break
    assert ties <= max_ties and (ties == 0 or cfg.dtype != synth.DT_F32), "near ties: %d" % ties
    assert compared >= 0.8 * total
    return worst
