"""ctypes binding of the CPU oracle (test infrastructure; see flover_oracle.cpp).

Only tests, the smoke entry and the benchmark's cpu_baseline leg import this.
Inputs are host arrays (numpy, or CPU torch tensors for the 16-bit dtypes); nothing here
touches a GPU or the product library.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Dict, List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "flover_oracle.cpp")
_LIB = os.path.join(_HERE, "liboracle.so")

WEIGHT_FIELDS = ["wte", "wpe", "ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo", "ln2_g", "ln2_b", "w1", "b1", "wu", "w2",
                 "b2", "lnf_g", "lnf_b", "wlm"]


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC])
    return _LIB


class OrcConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ["arch", "dtype", "L", "H", "nh", "d", "F", "V", "S", "C", "eos_id", "shuffle_mode"]] + \
               [("ln_eps", C.c_double), ("rope_theta", C.c_double)]


class OrcWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in WEIGHT_FIELDS]


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        L.orc_create.restype = C.c_void_p
        L.orc_create.argtypes = [C.POINTER(OrcConfig), C.POINTER(OrcWeights)]
        L.orc_destroy.argtypes = [C.c_void_p]
        L.orc_add_request.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_int32)]
        L.orc_step.argtypes = [C.c_void_p, C.POINTER(C.c_int32)] + [C.c_void_p] * 5
        L.orc_mark_finished.argtypes = [C.c_void_p, C.c_uint64]
        L.orc_set_next_token.argtypes = [C.c_void_p, C.c_uint64, C.c_int32]
        L.orc_reorder_evict.argtypes = [C.c_void_p] + [C.c_void_p] * 5
        L.orc_get_state.argtypes = [C.c_void_p] + [C.c_void_p] * 6
        L.orc_read_kv.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p]
        L.orc_full_forward.argtypes = [C.POINTER(OrcConfig), C.POINTER(OrcWeights), C.c_void_p, C.c_int, C.c_void_p]
        L.orc_find_window.argtypes = [C.c_void_p, C.c_int] + [C.POINTER(C.c_int32)] * 3
        L.orc_plan_moves.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        L.orc_attention.argtypes = [C.c_int] + [C.c_void_p] * 5 + [C.c_int] * 3 + [C.c_void_p, C.c_int, C.c_void_p]
        L.orc_gemm.argtypes = [C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_int,
                               C.c_void_p]
        L.orc_compact.argtypes = [C.c_void_p] + [C.c_int] * 6 + [C.c_void_p] * 3 + [C.c_int]
        L.orc_round.restype = C.c_double
        L.orc_round.argtypes = [C.c_double, C.c_int]
        L.orc_num_threads.restype = C.c_int
        L.orc_rope.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_double]
        _lib = L
    return _lib


def num_threads() -> int:
    return int(lib().orc_num_threads())


def _ptr(t) -> int:
    """Address of a host buffer: numpy array or CPU torch tensor (contiguous)."""
    if isinstance(t, np.ndarray):
        assert t.flags["C_CONTIGUOUS"]
        return t.ctypes.data
    assert t.device.type == "cpu" and t.is_contiguous()
    return t.data_ptr()


def make_config(cfg, shuffle_off: bool = False, by_length: bool = False) -> OrcConfig:
    return OrcConfig(cfg.arch, cfg.dtype, cfg.L, cfg.H, cfg.nh, cfg.d, cfg.F, cfg.V, cfg.S, cfg.C, cfg.eos_id,
                     1 if shuffle_off else 2 if by_length else 0, cfg.ln_eps, cfg.rope_theta)


def make_weights(weights: Dict[str, object]) -> OrcWeights:
    w = OrcWeights()
    for n in WEIGHT_FIELDS:
        setattr(w, n, _ptr(weights[n]) if n in weights else None)
    return w


class StepResult:
    def __init__(self, req_id, slot, token, finished, logits):
        self.req_id, self.slot, self.token, self.finished, self.logits = req_id, slot, token, finished, logits

    @property
    def n_live(self):
        return len(self.req_id)


class ReorderResult:
    def __init__(self, evicted, mem_offset, new_size, moves, new_lo, min_cost, bytes_moved):
        self.evicted, self.mem_offset, self.new_size = evicted, mem_offset, new_size
        self.moves, self.new_lo, self.min_cost, self.bytes_moved = moves, new_lo, min_cost, bytes_moved


class OracleServer:
    """The fused run: scheduler + slots + decoder + Algorithm 3 + shuffle, on the CPU."""

    def __init__(self, cfg, weights: Dict[str, object], shuffle_off: bool = False, by_length: bool = False):
        self.cfg = cfg
        self._weights = weights         # keep the host buffers alive
        self._c = make_config(cfg, shuffle_off, by_length)
        self._w = make_weights(weights)
        self._h = lib().orc_create(C.byref(self._c), C.byref(self._w))

    def close(self):
        if self._h:
            lib().orc_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()

    def add_request(self, req_id: int, prompt: Sequence[int], max_new: int) -> int:
        p = np.ascontiguousarray(np.asarray(prompt, dtype=np.int32))
        slot = C.c_int32(-2)
        rc = lib().orc_add_request(self._h, req_id, p.ctypes.data, len(p), max_new, C.byref(slot))
        if rc != 0:
            raise ValueError("oracle rejected the request")
        return slot.value

    def step(self, want_logits: bool = True) -> StepResult:
        Cn, V = self.cfg.C, self.cfg.V
        n = C.c_int32(0)
        rid = np.zeros(Cn, np.uint64)
        slot = np.zeros(Cn, np.int32)
        tok = np.zeros(Cn, np.int32)
        fin = np.zeros(Cn, np.int32)
        logits = np.zeros((Cn, V), np.float64) if want_logits else None
        lib().orc_step(self._h, C.byref(n), rid.ctypes.data, slot.ctypes.data, tok.ctypes.data, fin.ctypes.data,
                       logits.ctypes.data if want_logits else None)
        k = n.value
        return StepResult(rid[:k].copy(), slot[:k].copy(), tok[:k].copy(), fin[:k].copy(),
                          logits[:k].copy() if want_logits else None)

    def mark_finished(self, req_id: int):
        if lib().orc_mark_finished(self._h, req_id) != 0:
            raise ValueError("no such live request")

    def set_next_token(self, req_id: int, tok: int):
        if lib().orc_set_next_token(self._h, req_id, tok) != 0:
            raise ValueError("no such live request")

    def reorder_evict(self) -> ReorderResult:
        Cn = self.cfg.C
        out6 = np.zeros(6, np.int32)
        ev = np.zeros(Cn, np.uint64)
        src = np.zeros(Cn, np.int32)
        dst = np.zeros(Cn, np.int32)
        b = np.zeros(1, np.int64)
        lib().orc_reorder_evict(self._h, out6.ctypes.data, ev.ctypes.data, src.ctypes.data, dst.ctypes.data,
                                b.ctypes.data)
        nm = int(out6[3])
        return ReorderResult(ev[:out6[0]].copy(), int(out6[1]), int(out6[2]),
                             list(zip(src[:nm].tolist(), dst[:nm].tolist())), int(out6[4]), int(out6[5]), int(b[0]))

    def state(self):
        Cn = self.cfg.C
        lhw = np.zeros(3, np.int32)
        st = np.zeros(Cn, np.int32)
        rid = np.zeros(Cn, np.uint64)
        ln = np.zeros(Cn, np.int32)
        nt = np.zeros(Cn, np.int32)
        gen = np.zeros(Cn, np.int32)
        lib().orc_get_state(self._h, lhw.ctypes.data, st.ctypes.data, rid.ctypes.data, ln.ctypes.data, nt.ctypes.data,
                            gen.ctypes.data)
        return {"lo": int(lhw[0]), "hi": int(lhw[1]), "waiting": int(lhw[2]), "state": st, "req_id": rid, "len": ln,
                "next_token": nt, "generated": gen}

    def read_kv(self, layer: int, which: int, slot: int, head: int, n: int) -> np.ndarray:
        out = np.zeros((n, self.cfg.d), np.float64)
        lib().orc_read_kv(self._h, layer, which, slot, head, n, out.ctypes.data)
        return out


def solo_decode(cfg, weights, prompt, gen_len, want_logits=True):
    """Decode one request ALONE from an empty cache: the definition of the result that a fused run must reproduce."""
    import dataclasses
    solo_cfg = dataclasses.replace(cfg, C=1)
    srv = OracleServer(solo_cfg, weights)
    srv.add_request(0, prompt, gen_len)
    toks, logits = [], []
    while True:
        r = srv.step(want_logits)
        if r.n_live == 0:
            break
        toks.append(int(r.token[0]))
        if want_logits:
            logits.append(r.logits[0])
        srv.reorder_evict()
    srv.close()
    return np.asarray(toks, np.int32), (np.stack(logits) if want_logits else None)


def full_forward(cfg, weights, tokens) -> np.ndarray:
    c, w = make_config(cfg), make_weights(weights)
    t = np.ascontiguousarray(np.asarray(tokens, np.int32))
    out = np.zeros((len(t), cfg.V), np.float64)
    lib().orc_full_forward(C.byref(c), C.byref(w), t.ctypes.data, len(t), out.ctypes.data)
    return out


def find_window(arr):
    a = np.ascontiguousarray(np.asarray(arr, np.int32))
    off, cost, nz = C.c_int32(), C.c_int32(), C.c_int32()
    lib().orc_find_window(a.ctypes.data, len(a), C.byref(off), C.byref(cost), C.byref(nz))
    return off.value, cost.value, nz.value


def plan_moves(arr, off, non_zero):
    a = np.ascontiguousarray(np.asarray(arr, np.int32))
    src = np.zeros(max(len(a), 1), np.int32)
    dst = np.zeros(max(len(a), 1), np.int32)
    n = lib().orc_plan_moves(a.ctypes.data, len(a), off, non_zero, src.ctypes.data, dst.ctypes.data)
    return list(zip(src[:n].tolist(), dst[:n].tolist()))


def attention(dtype, q, kcache, vcache, slot, length, pairs) -> np.ndarray:
    """q [M][nh][d], caches [C][nh][S][d] (host, model dtype); pairs = list of (row, head). Returns [n_pairs][d] float64."""
    nh, d = q.shape[1], q.shape[2]
    S = kcache.shape[2]
    slot = np.ascontiguousarray(np.asarray(slot, np.int32))
    length = np.ascontiguousarray(np.asarray(length, np.int32))
    pr = np.ascontiguousarray(np.asarray(pairs, np.int32).reshape(-1, 2))
    out = np.zeros((len(pr), d), np.float64)
    lib().orc_attention(dtype, _ptr(q), _ptr(kcache), _ptr(vcache), slot.ctypes.data, length.ctypes.data, nh, d, S,
                        pr.ctypes.data, len(pr), out.ctypes.data)
    return out


def gemm(dtype, x, W, cols=None) -> np.ndarray:
    M, K = x.shape
    N = W.shape[0]
    if cols is None:
        out = np.zeros((M, N), np.float64)
        lib().orc_gemm(dtype, _ptr(x), _ptr(W), M, N, K, None, 0, out.ctypes.data)
    else:
        cc = np.ascontiguousarray(np.asarray(cols, np.int32))
        out = np.zeros((M, len(cc)), np.float64)
        lib().orc_gemm(dtype, _ptr(x), _ptr(W), M, N, K, cc.ctypes.data, len(cc), out.ctypes.data)
    return out


def compact(cache, L, Cn, nh, S, d, ebytes, moves_src, moves_dst, moves_len):
    """In-place slot-to-slot byte copy on a host cache buffer [L][2][C][nh][S][d]."""
    src = np.ascontiguousarray(np.asarray(moves_src, np.int32))
    dst = np.ascontiguousarray(np.asarray(moves_dst, np.int32))
    ln = np.ascontiguousarray(np.asarray(moves_len, np.int32))
    lib().orc_compact(_ptr(cache), L, Cn, nh, S, d, ebytes, src.ctypes.data, dst.ctypes.data, ln.ctypes.data, len(src))


def round_to(x: float, dtype: int) -> float:
    return float(lib().orc_round(float(x), dtype))


def rope(vec, pos: int, theta: float = 10000.0) -> np.ndarray:
    v = np.ascontiguousarray(np.asarray(vec, np.float64)).copy()
    lib().orc_rope(v.ctypes.data, len(v), pos, theta)
    return v
