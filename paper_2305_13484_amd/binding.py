"""Thin ctypes binding of libflover.so (include/flover.h): same names, argument marshalling only.

PyTorch is used for device memory (the arena, weights, outputs) and the stream handle.  If the HIP library has not
been built this module raises on first use -- there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libflover.so")

EXPORTED_SYMBOLS = [
    "flover_query_arena_bytes", "flover_init", "flover_destroy", "flover_last_error", "flover_add_request",
    "flover_step", "flover_reorder_evict", "flover_mark_finished", "flover_set_next_token", "flover_get_state",
    "flover_get_kv_cache", "flover_last_step_launches", "flover_step_submit", "flover_step_collect", "flover_set_layer_weights", "flover_k_gemm_plan", "flover_set_profile", "flover_get_profile", "flover_k_find_window", "flover_k_attention_workspace_bytes",
    "flover_k_decode_attention", "flover_k_compact_workspace_bytes", "flover_k_compact", "flover_k_gemm_tiled_bytes",
    "flover_k_gemm_workspace_bytes", "flover_k_gemm_retile", "flover_k_gemm", "flover_add_request_cached",
    "flover_k_copy_probe", "flover_k_decode_attention_noalloc", "flover_k_gated_retile", "flover_k_gated_workspace_bytes", "flover_k_gated_mlp",
]

WEIGHT_FIELDS = ["wte", "wpe", "ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo", "ln2_g", "ln2_b", "w1", "b1", "wu", "w2",
                 "b2", "lnf_g", "lnf_b", "wlm"]
_TORCH_DT = {0: torch.float32, 1: torch.float16, 2: torch.bfloat16}
_DT_OF = {torch.float32: 0, torch.float16: 1, torch.bfloat16: 2}


class FloverError(RuntimeError):
    pass


class _Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ["arch", "dtype", "n_layer", "hidden", "n_head", "head_dim", "ffn", "vocab", "max_seq",
                 "max_concurrency", "eos_id", "shuffle_mode", "async_preprocess"]] + \
               [("norm_eps", C.c_float), ("rope_theta", C.c_float), ("stream", C.c_void_p), ("arena", C.c_void_p),
                ("arena_bytes", C.c_uint64)]


class _Weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in WEIGHT_FIELDS]


class _StepOut(C.Structure):
    _fields_ = [("capacity", C.c_int32), ("n_live", C.c_int32), ("req_id", C.c_void_p), ("slot", C.c_void_p),
                ("token", C.c_void_p), ("finished", C.c_void_p), ("logits", C.c_void_p)]


class _ReorderOut(C.Structure):
    _fields_ = [("capacity", C.c_int32), ("n_evicted", C.c_int32), ("evicted_req_id", C.c_void_p),
                ("mem_offset", C.c_int32), ("new_lo", C.c_int32), ("new_size", C.c_int32), ("min_cost", C.c_int32),
                ("n_moves", C.c_int32), ("move_src", C.c_void_p), ("move_dst", C.c_void_p), ("bytes_moved", C.c_int64)]


_lib = None


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FloverError("libflover.so is not built: run `python -m paper_2305_13484_amd.build` "
                          "(or __graft_entry__.build()); there is no fallback path")
    L = C.CDLL(_LIB_PATH)
    L.flover_last_error.restype = C.c_char_p
    L.flover_last_error.argtypes = [C.c_void_p]
    L.flover_query_arena_bytes.argtypes = [C.POINTER(_Config), C.POINTER(C.c_uint64)]
    L.flover_init.argtypes = [C.POINTER(_Config), C.POINTER(_Weights), C.POINTER(C.c_void_p)]
    L.flover_destroy.argtypes = [C.c_void_p]
    L.flover_add_request.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_int32)]
    L.flover_add_request_cached.argtypes = [C.c_void_p, C.c_uint64, C.c_int32, C.c_int32, C.c_int32,
                                            C.POINTER(C.c_int32)]
    L.flover_k_copy_probe.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p]
    L.flover_step.argtypes = [C.c_void_p, C.POINTER(_StepOut)]
    L.flover_set_layer_weights.argtypes = [C.c_void_p, C.c_int32, C.POINTER(_Weights)]
    L.flover_step_submit.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_int32)]
    L.flover_step_collect.argtypes = [C.c_void_p, C.POINTER(_StepOut)]
    L.flover_reorder_evict.argtypes = [C.c_void_p, C.POINTER(_ReorderOut)]
    L.flover_mark_finished.argtypes = [C.c_void_p, C.c_uint64]
    L.flover_set_next_token.argtypes = [C.c_void_p, C.c_uint64, C.c_int32]
    L.flover_get_state.argtypes = [C.c_void_p] + [C.c_void_p] * 6
    L.flover_get_kv_cache.argtypes = [C.c_void_p, C.POINTER(C.c_void_p), C.POINTER(C.c_uint64)]
    L.flover_last_step_launches.argtypes = [C.c_void_p, C.POINTER(C.c_int32)]
    L.flover_set_profile.argtypes = [C.c_void_p, C.c_int32]
    L.flover_get_profile.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_double), C.POINTER(C.c_int64),
                                     C.POINTER(C.c_int64)]
    L.flover_k_find_window.argtypes = [C.c_void_p, C.c_int32] + [C.POINTER(C.c_int32)] * 3
    L.flover_k_attention_workspace_bytes.argtypes = [C.c_int32] * 4 + [C.POINTER(C.c_uint64)]
    L.flover_k_decode_attention.argtypes = [C.c_int32] + [C.c_void_p] * 5 + [C.c_int32] * 5 + \
                                           [C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p]
    L.flover_k_decode_attention_noalloc.argtypes = [C.c_int32] + [C.c_void_p] * 5 + [C.c_int32] * 5 + \
                                                   [C.c_void_p, C.c_void_p]
    L.flover_k_compact_workspace_bytes.argtypes = [C.c_int32, C.POINTER(C.c_uint64)]
    L.flover_k_compact.argtypes = [C.c_void_p] + [C.c_int32] * 6 + [C.c_void_p] * 3 + [C.c_int32, C.c_void_p,
                                                                                     C.c_uint64, C.c_void_p]
    L.flover_k_gemm_tiled_bytes.argtypes = [C.c_int32] * 3 + [C.POINTER(C.c_uint64)]
    L.flover_k_gemm_workspace_bytes.argtypes = [C.c_int32] * 4 + [C.POINTER(C.c_uint64)]
    L.flover_k_gemm_retile.argtypes = [C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    L.flover_k_gemm.argtypes = [C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                C.c_void_p, C.c_uint64, C.c_void_p]
    L.flover_k_gated_retile.argtypes = [C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    L.flover_k_gated_workspace_bytes.argtypes = [C.c_int32] * 4 + [C.POINTER(C.c_uint64)]
    L.flover_k_gated_mlp.argtypes = [C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                     C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p]
    _lib = L
    return L


def _check(rc: int, ctx=None):
    if rc != 0:
        msg = load_library().flover_last_error(ctx)
        raise FloverError("flover error %d: %s" % (rc, (msg or b"").decode()))


def _stream_ptr() -> int:
    return torch.cuda.current_stream().cuda_stream


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


class StepOut:
    def __init__(self, req_id, slot, token, finished, logits):
        self.req_id, self.slot, self.token, self.finished, self.logits = req_id, slot, token, finished, logits

    @property
    def n_live(self):
        return len(self.req_id)


class ReorderOut:
    def __init__(self, evicted, mem_offset, new_lo, new_size, min_cost, moves, bytes_moved):
        self.evicted, self.mem_offset, self.new_lo, self.new_size = evicted, mem_offset, new_lo, new_size
        self.min_cost, self.moves, self.bytes_moved = min_cost, moves, bytes_moved


class Flover:
    """One context = one fused decode stream on the current device and the current torch stream.

    cfg: any object with fields arch, dtype, L, H, nh, d, F, V, S, C, eos_id, ln_eps, rope_theta.
    weights: dict of device tensors (names of flover_weights), each [out][in] / stacked over layers."""

    def __init__(self, cfg, weights: Dict[str, torch.Tensor], shuffle_off: bool = False, by_length: bool = False,
                 async_preprocess: int = 0):   # 0 | 1 | 2 as in flover_config (True counts as 1)
        L = load_library()
        self.cfg = cfg
        self._ctx = None
        c = _Config(cfg.arch, cfg.dtype, cfg.L, cfg.H, cfg.nh, cfg.d, cfg.F, cfg.V, cfg.S, cfg.C, cfg.eos_id,
                    1 if shuffle_off else 2 if by_length else 0, int(async_preprocess), cfg.ln_eps, cfg.rope_theta, None, None, 0)
        need = C.c_uint64(0)
        _check(L.flover_query_arena_bytes(C.byref(c), C.byref(need)))
        self.arena = torch.empty(int(need.value) + 256, dtype=torch.uint8, device="cuda")
        base = (self.arena.data_ptr() + 255) // 256 * 256
        self._arena_off = base - self.arena.data_ptr()
        c.arena, c.arena_bytes, c.stream = base, need.value, _stream_ptr()
        w = _Weights()
        for n in WEIGHT_FIELDS:
            t = weights.get(n)
            if t is not None:
                assert t.is_cuda and t.is_contiguous() and t.dtype == _TORCH_DT[cfg.dtype], n
            setattr(w, n, t.data_ptr() if t is not None else None)
        ctx = C.c_void_p()
        _check(L.flover_init(C.byref(c), C.byref(w), C.byref(ctx)))
        self._ctx = ctx
        Cn = cfg.C
        self._rid = np.zeros(Cn, np.uint64)
        self._slot = np.zeros(Cn, np.int32)
        self._tok = np.zeros(Cn, np.int32)
        self._fin = np.zeros(Cn, np.int32)
        self._src = np.zeros(Cn, np.int32)
        self._dst = np.zeros(Cn, np.int32)
        self._logits = None

    def set_layer_weights(self, layer: int, weights: Dict[str, torch.Tensor]):
        """Hand over ONE layer's tensors (names of flover_weights, without the leading layer dimension or with a
        leading dimension of 1) to a context created with no per-layer tensors."""
        w = _Weights()
        for n in WEIGHT_FIELDS:
            t = weights.get(n)
            if t is not None:
                assert t.is_cuda and t.is_contiguous() and t.dtype == _TORCH_DT[self.cfg.dtype], n
            setattr(w, n, t.data_ptr() if t is not None else None)
        _check(load_library().flover_set_layer_weights(self._ctx, layer, C.byref(w)), self._ctx)

    def close(self):
        if self._ctx is not None:
            load_library().flover_destroy(self._ctx)
            self._ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def add_request(self, req_id: int, prompt: Sequence[int], max_new_tokens: int) -> int:
        p = _i32(prompt)
        slot = C.c_int32(-2)
        _check(load_library().flover_add_request(self._ctx, req_id, p.ctypes.data, len(p), max_new_tokens,
                                                 C.byref(slot)), self._ctx)
        return slot.value

    def add_request_cached(self, req_id: int, context_len: int, next_token: int, max_new_tokens: int) -> int:
        slot = C.c_int32(-2)
        _check(load_library().flover_add_request_cached(self._ctx, req_id, context_len, next_token, max_new_tokens,
                                                        C.byref(slot)), self._ctx)
        return slot.value

    def step(self, want_logits: bool = False) -> StepOut:
        Cn = self.cfg.C
        if want_logits and self._logits is None:
            self._logits = torch.empty((Cn, self.cfg.V), dtype=torch.float32, device="cuda")
        so = _StepOut(Cn, 0, self._rid.ctypes.data, self._slot.ctypes.data, self._tok.ctypes.data,
                      self._fin.ctypes.data, self._logits.data_ptr() if want_logits else None)
        _check(load_library().flover_step(self._ctx, C.byref(so)), self._ctx)
        n = so.n_live
        return StepOut(self._rid[:n].copy(), self._slot[:n].copy(), self._tok[:n].copy(), self._fin[:n].copy(),
                       self._logits[:n] if want_logits else None)

    def step_submit(self, logits: Optional[torch.Tensor] = None) -> int:
        """Enqueue one iteration (pipelined token return); returns its row count (0: nothing enqueued)."""
        n = C.c_int32(0)
        _check(load_library().flover_step_submit(self._ctx, logits.data_ptr() if logits is not None else None,
                                                 C.byref(n)), self._ctx)
        return n.value

    def step_collect(self) -> StepOut:
        """Tokens of the oldest submitted iteration."""
        Cn = self.cfg.C
        so = _StepOut(Cn, 0, self._rid.ctypes.data, self._slot.ctypes.data, self._tok.ctypes.data,
                      self._fin.ctypes.data, None)
        _check(load_library().flover_step_collect(self._ctx, C.byref(so)), self._ctx)
        n = so.n_live
        return StepOut(self._rid[:n].copy(), self._slot[:n].copy(), self._tok[:n].copy(), self._fin[:n].copy(), None)

    def reorder_evict(self) -> ReorderOut:
        Cn = self.cfg.C
        ro = _ReorderOut(Cn, 0, self._rid.ctypes.data, 0, 0, 0, 0, 0, self._src.ctypes.data, self._dst.ctypes.data, 0)
        _check(load_library().flover_reorder_evict(self._ctx, C.byref(ro)), self._ctx)
        nm = ro.n_moves
        return ReorderOut(self._rid[:ro.n_evicted].copy(), ro.mem_offset, ro.new_lo, ro.new_size, ro.min_cost,
                          list(zip(self._src[:nm].tolist(), self._dst[:nm].tolist())), int(ro.bytes_moved))

    def mark_finished(self, req_id: int):
        _check(load_library().flover_mark_finished(self._ctx, req_id), self._ctx)

    def set_next_token(self, req_id: int, token: int):
        _check(load_library().flover_set_next_token(self._ctx, req_id, token), self._ctx)

    def last_step_launches(self) -> int:
        n = C.c_int32(0)
        _check(load_library().flover_last_step_launches(self._ctx, C.byref(n)), self._ctx)
        return n.value

    PROF_KINDS = ["attention", "gemm_qkv", "gemm_out", "gemm_ff1", "gemm_ff2", "gemm_lm", "compact"]

    def set_profile(self, level: int):
        _check(load_library().flover_set_profile(self._ctx, level), self._ctx)

    def get_profile(self):
        out = {}
        for k, name in enumerate(self.PROF_KINDS):
            ms, n, b = C.c_double(), C.c_int64(), C.c_int64()
            _check(load_library().flover_get_profile(self._ctx, k, C.byref(ms), C.byref(n), C.byref(b)), self._ctx)
            out[name] = {"ms": ms.value, "launches": n.value, "bytes": b.value}
        return out

    def state(self):
        Cn = self.cfg.C
        lhw = np.zeros(3, np.int32)
        st, rid, ln, nt, gen = (np.zeros(Cn, np.int32), np.zeros(Cn, np.uint64), np.zeros(Cn, np.int32),
                                np.zeros(Cn, np.int32), np.zeros(Cn, np.int32))
        _check(load_library().flover_get_state(self._ctx, lhw.ctypes.data, st.ctypes.data, rid.ctypes.data,
                                               ln.ctypes.data, nt.ctypes.data, gen.ctypes.data), self._ctx)
        return {"lo": int(lhw[0]), "hi": int(lhw[1]), "waiting": int(lhw[2]), "state": st, "req_id": rid, "len": ln,
                "next_token": nt, "generated": gen}

    def kv_cache(self) -> torch.Tensor:
        """View of the KV cache inside the arena: [L][2][C][nh][S][d] in the model dtype."""
        base, nbytes = C.c_void_p(), C.c_uint64()
        _check(load_library().flover_get_kv_cache(self._ctx, C.byref(base), C.byref(nbytes)), self._ctx)
        off = base.value - self.arena.data_ptr()
        c = self.cfg
        return self.arena[off:off + nbytes.value].view(_TORCH_DT[c.dtype]).view(c.L, 2, c.C, c.nh, c.S, c.d)


# ------------------------------------------------------------------ operation-level entry points

def k_gemm_plan(dtype: int, N: int, K: int, context_rows: int = 0) -> Tuple[int, int]:
    """(slices, k-blocks per slice) of the weight GEMM; host only."""
    s, kbs = C.c_int32(), C.c_int32()
    _check(load_library().flover_k_gemm_plan(dtype, N, K, context_rows, C.byref(s), C.byref(kbs)))
    return s.value, kbs.value


def arena_bytes(cfg, async_preprocess: int = 0) -> int:
    """flover_query_arena_bytes for a config object (fields as for Flover)."""
    c = _Config(cfg.arch, cfg.dtype, cfg.L, cfg.H, cfg.nh, cfg.d, cfg.F, cfg.V, cfg.S, cfg.C, cfg.eos_id, 0,
                int(async_preprocess), cfg.ln_eps, cfg.rope_theta, None, None, 0)
    need = C.c_uint64(0)
    _check(load_library().flover_query_arena_bytes(C.byref(c), C.byref(need)))
    return int(need.value)


def k_find_window(arr) -> Tuple[int, int, int]:
    a = _i32(arr)
    off, cost, nz = C.c_int32(), C.c_int32(), C.c_int32()
    _check(load_library().flover_k_find_window(a.ctypes.data, len(a), C.byref(off), C.byref(cost), C.byref(nz)))
    return off.value, cost.value, nz.value


class AttentionWorkspace:
    def __init__(self, M, nh, d, max_len):
        n = C.c_uint64()
        _check(load_library().flover_k_attention_workspace_bytes(M, nh, d, max_len, C.byref(n)))
        self.buf = torch.empty(int(n.value), dtype=torch.uint8, device="cuda")


def k_decode_attention(q: torch.Tensor, kcache: torch.Tensor, vcache: torch.Tensor, slot, length,
                       out: Optional[torch.Tensor] = None, workspace: Optional[AttentionWorkspace] = None):
    """q [M][nh][d], caches [C][nh][S][d] (device, same dtype); slot, length: host int arrays [M]."""
    M, nh, d = q.shape
    Cn, _, S, _ = kcache.shape
    slot, length = _i32(slot), _i32(length)
    if out is None:
        out = torch.empty_like(q)
    if workspace is None:
        workspace = AttentionWorkspace(M, nh, d, int(length.max()) if M else 1)
    assert q.is_contiguous() and kcache.is_contiguous() and vcache.is_contiguous() and out.is_contiguous()
    _check(load_library().flover_k_decode_attention(_DT_OF[q.dtype], q.data_ptr(), kcache.data_ptr(),
                                                    vcache.data_ptr(), slot.ctypes.data, length.ctypes.data, M, Cn, nh,
                                                    d, S, out.data_ptr(), workspace.buf.data_ptr(),
                                                    workspace.buf.numel(), _stream_ptr()))
    return out


def k_decode_attention_noalloc(q: torch.Tensor, kcache: torch.Tensor, vcache: torch.Tensor, slot, length,
                               out: torch.Tensor):
    """flover_k_decode_attention_noalloc: as k_decode_attention, workspace inside the library; `out` is the caller's."""
    M, nh, d = q.shape
    Cn, _, S, _ = kcache.shape
    slot, length = _i32(slot), _i32(length)
    assert q.is_contiguous() and kcache.is_contiguous() and vcache.is_contiguous() and out.is_contiguous()
    _check(load_library().flover_k_decode_attention_noalloc(_DT_OF[q.dtype], q.data_ptr(), kcache.data_ptr(),
                                                            vcache.data_ptr(), slot.ctypes.data, length.ctypes.data, M,
                                                            Cn, nh, d, S, out.data_ptr(), _stream_ptr()))
    return out


def k_compact(cache: torch.Tensor, src, dst, length):
    """cache [L][2][C][nh][S][d] (device), moved in place."""
    Ln, two, Cn, nh, S, d = cache.shape
    assert two == 2 and cache.is_contiguous()
    src, dst, length = _i32(src), _i32(dst), _i32(length)
    n = C.c_uint64()
    _check(load_library().flover_k_compact_workspace_bytes(len(src), C.byref(n)))
    ws = torch.empty(int(n.value), dtype=torch.uint8, device="cuda")
    _check(load_library().flover_k_compact(cache.data_ptr(), Ln, Cn, nh, S, d, cache.element_size(), src.ctypes.data,
                                           dst.ctypes.data, length.ctypes.data, len(src), ws.data_ptr(), ws.numel(),
                                           _stream_ptr()))
    torch.cuda.current_stream().synchronize()     # ws is released on return
    return cache


class TiledWeight:
    def __init__(self, W: torch.Tensor):
        self.N, self.K = W.shape
        self.dtype = _DT_OF[W.dtype]
        n = C.c_uint64()
        _check(load_library().flover_k_gemm_tiled_bytes(self.dtype, self.N, self.K, C.byref(n)))
        self.buf = torch.empty(int(n.value), dtype=torch.uint8, device="cuda")
        _check(load_library().flover_k_gemm_retile(self.dtype, W.data_ptr(), self.N, self.K, self.buf.data_ptr(),
                                                   _stream_ptr()))


def k_gemm(x: torch.Tensor, W, out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None):
    """y[M][N] fp32 = x[M][K] . W[N][K]^T; W a device tensor or a TiledWeight."""
    tw = W if isinstance(W, TiledWeight) else TiledWeight(W)
    M, K = x.shape
    assert K == tw.K and _DT_OF[x.dtype] == tw.dtype
    rows = (M + 127) // 128 * 128 if M <= 128 else (M + 255) // 256 * 256
    xp = x
    if M != rows:
        xp = torch.zeros((rows, K), dtype=x.dtype, device=x.device)
        xp[:M] = x
    if out is None:
        out = torch.empty((M, tw.N), dtype=torch.float32, device=x.device)
    if workspace is None:
        n = C.c_uint64()
        _check(load_library().flover_k_gemm_workspace_bytes(tw.dtype, M, tw.N, K, C.byref(n)))
        workspace = torch.empty(int(n.value), dtype=torch.uint8, device="cuda")
    _check(load_library().flover_k_gemm(tw.dtype, xp.data_ptr(), tw.buf.data_ptr(), M, tw.N, K, out.data_ptr(),
                                        workspace.data_ptr(), workspace.numel(), _stream_ptr()))
    torch.cuda.current_stream().synchronize()
    return out


class GatedWeight:
    """Gate and up projections [F][K] of a gated MLP, re-tiled together for k_gated_mlp."""

    def __init__(self, Wgate: torch.Tensor, Wup: torch.Tensor):
        assert Wgate.shape == Wup.shape and Wgate.dtype == Wup.dtype and Wgate.is_contiguous() and Wup.is_contiguous()
        self.F, self.K = Wgate.shape
        self.dtype = _DT_OF[Wgate.dtype]
        n = C.c_uint64()
        _check(load_library().flover_k_gemm_tiled_bytes(self.dtype, 2 * self.F, self.K, C.byref(n)))
        self.buf = torch.empty(int(n.value), dtype=torch.uint8, device="cuda")
        _check(load_library().flover_k_gated_retile(self.dtype, Wgate.data_ptr(), Wup.data_ptr(), self.F, self.K,
                                                    self.buf.data_ptr(), _stream_ptr()))


def k_gated_mlp(x: torch.Tensor, gw: GatedWeight, out: Optional[torch.Tensor] = None, sync: bool = True,
                context_pass: bool = False):
    """act[M][F] = silu(x . Wgate^T) * (x . Wup^T) in the model dtype; rows of a fused iteration, or of one request's
    context pass."""
    M, K = x.shape
    assert K == gw.K and _DT_OF[x.dtype] == gw.dtype
    rows = (M + 127) // 128 * 128 if M <= 128 else (M + 255) // 256 * 256
    xp = x
    if M != rows:
        xp = torch.zeros((rows, K), dtype=x.dtype, device=x.device)
        xp[:M] = x
    if out is None:
        out = torch.empty((M, gw.F), dtype=x.dtype, device=x.device)
    n = C.c_uint64()
    _check(load_library().flover_k_gated_workspace_bytes(gw.dtype, M, gw.F, K, C.byref(n)))
    ws = torch.empty(max(int(n.value), 16), dtype=torch.uint8, device="cuda")
    _check(load_library().flover_k_gated_mlp(gw.dtype, xp.data_ptr(), gw.buf.data_ptr(), M, gw.F, K,
                                             1 if context_pass else 0, out.data_ptr(), ws.data_ptr(), int(n.value),
                                             _stream_ptr()))
    if sync:
        torch.cuda.current_stream().synchronize()
    return out


def k_copy_probe(dst: torch.Tensor, src: torch.Tensor):
    assert dst.is_contiguous() and src.is_contiguous() and dst.numel() * dst.element_size() == src.numel() * src.element_size()
    _check(load_library().flover_k_copy_probe(dst.data_ptr(), src.data_ptr(), src.numel() * src.element_size(),
                                              _stream_ptr()))
