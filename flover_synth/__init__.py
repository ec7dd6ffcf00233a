"""Seeded synthetic inputs for the fused decode step (weights, request streams,
attention/compaction micro-benchmark tensors).

This module holds NO arithmetic of the method: it only draws random numbers
and lays them out in the shapes the workloads name.  Both the CPU oracle's
tests and the HIP path's tests/bench take their inputs from here, so the two
sides always see the same bits.

Workload recipe (stands in for the paper's pretrained GPT-J / LLaMA checkpoints
and unnamed prompts, Section VI-A, which are not available offline):
  * matrices, embeddings and biases ~ N(0, 0.02); norm gains = 1 + N(0, 0.02)
  * prompt token ids uniform over the vocabulary
  * arrivals: uniform step, constant interval, or Poisson counts per decode
    step (Section IV models arrivals as a Poisson process)
  * generation lengths: uniform (Section VI-D uses U(a, b)) or log-uniform
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional

import numpy as np
import torch

ARCH_GPT = 0
ARCH_LLAMA = 1
DT_F32 = 0
DT_F16 = 1
DT_BF16 = 2

TORCH_DTYPE = {DT_F32: torch.float32, DT_F16: torch.float16, DT_BF16: torch.bfloat16}
DTYPE_NAME = {DT_F32: "f32", DT_F16: "f16", DT_BF16: "bf16"}
DTYPE_BYTES = {DT_F32: 4, DT_F16: 2, DT_BF16: 2}


@dataclasses.dataclass(frozen=True)
class ModelConfig:
    name: str
    arch: int
    dtype: int
    L: int      # layers
    H: int      # hidden
    nh: int     # heads
    d: int      # head_dim (H == nh * d)
    F: int      # FFN width
    V: int      # vocab
    S: int      # max_seq: slot capacity in tokens
    C: int      # max_concurrency: slots
    eos_id: int = -1
    ln_eps: float = 1e-5
    rope_theta: float = 10000.0

    def kv_bytes_per_token(self) -> int:
        return 2 * self.L * self.H * DTYPE_BYTES[self.dtype]

    def matmul_params_per_layer(self) -> int:
        H, F = self.H, self.F
        if self.arch == ARCH_GPT:
            return 3 * H * H + 3 * H + H * H + H + H * F + F + F * H + H
        return 3 * H * H + H * H + 3 * H * F

    def weight_bytes_per_step(self) -> int:
        e = DTYPE_BYTES[self.dtype]
        return (self.L * self.matmul_params_per_layer() + self.V * self.H) * e


def tiny_gpt(C: int = 8, S: int = 128, eos_id: int = -1) -> ModelConfig:
    return ModelConfig("c1_tiny_gpt_f32", ARCH_GPT, DT_F32, 2, 256, 4, 64, 1024, 1024, S, C,
                       eos_id=eos_id, ln_eps=1e-5)


def tiny_llama(dtype: int = DT_F32, C: int = 8, S: int = 128) -> ModelConfig:
    return ModelConfig("tiny_llama_" + DTYPE_NAME[dtype], ARCH_LLAMA, dtype, 2, 256, 4, 64, 704, 1024, S, C,
                       ln_eps=1e-6)


def small_gpt16(dtype: int = DT_F16, C: int = 8, S: int = 128) -> ModelConfig:
    """A small GPT in a 16-bit dtype with head_dim 128 (the shape class of the 1.3B config)."""
    return ModelConfig("small_gpt_" + DTYPE_NAME[dtype], ARCH_GPT, dtype, 2, 512, 4, 128, 2048, 1000, S, C,
                       ln_eps=1e-5)


def small_llama16(dtype: int = DT_BF16, C: int = 16, S: int = 160, L: int = 2) -> ModelConfig:
    """A small LLaMA in a 16-bit dtype with head_dim 128 (the shape class of the 7B config)."""
    return ModelConfig("small_llama_" + DTYPE_NAME[dtype], ARCH_LLAMA, dtype, L, 512, 4, 128, 1376, 2000, S, C,
                       ln_eps=1e-6)


def gpt_1p3b(L: int = 24, C: int = 64) -> ModelConfig:
    return ModelConfig("c3_gpt1p3b_f16", ARCH_GPT, DT_F16, L, 2048, 16, 128, 8192, 50257, 2048, C, ln_eps=1e-5)


def llama_7b(L: int = 32, C: int = 128, S: int = 2048) -> ModelConfig:
    return ModelConfig("c4_llama7b_bf16", ARCH_LLAMA, DT_BF16, L, 4096, 32, 128, 11008, 32000, S, C, ln_eps=1e-6)


def llama_30b(L: int = 60, C: int = 64) -> ModelConfig:
    return ModelConfig("c5_llama30b_bf16", ARCH_LLAMA, DT_BF16, L, 6656, 52, 128, 17920, 32000, 2048, C, ln_eps=1e-6)


# --------------------------------------------------------------------------- weights

WEIGHT_SHAPES_GPT = {
    "wte": lambda c: (c.V, c.H), "wpe": lambda c: (c.S, c.H),
    "ln1_g": lambda c: (c.L, c.H), "ln1_b": lambda c: (c.L, c.H),
    "wqkv": lambda c: (c.L, 3 * c.H, c.H), "bqkv": lambda c: (c.L, 3 * c.H),
    "wo": lambda c: (c.L, c.H, c.H), "bo": lambda c: (c.L, c.H),
    "ln2_g": lambda c: (c.L, c.H), "ln2_b": lambda c: (c.L, c.H),
    "w1": lambda c: (c.L, c.F, c.H), "b1": lambda c: (c.L, c.F),
    "w2": lambda c: (c.L, c.H, c.F), "b2": lambda c: (c.L, c.H),
    "lnf_g": lambda c: (c.H,), "lnf_b": lambda c: (c.H,),
}
WEIGHT_SHAPES_LLAMA = {
    "wte": lambda c: (c.V, c.H),
    "ln1_g": lambda c: (c.L, c.H),
    "wqkv": lambda c: (c.L, 3 * c.H, c.H),
    "wo": lambda c: (c.L, c.H, c.H),
    "ln2_g": lambda c: (c.L, c.H),
    "w1": lambda c: (c.L, c.F, c.H),    # gate
    "wu": lambda c: (c.L, c.F, c.H),    # up
    "w2": lambda c: (c.L, c.H, c.F),    # down
    "lnf_g": lambda c: (c.H,),
    "wlm": lambda c: (c.V, c.H),
}


def weight_shapes(cfg: ModelConfig) -> Dict[str, tuple]:
    table = WEIGHT_SHAPES_GPT if cfg.arch == ARCH_GPT else WEIGHT_SHAPES_LLAMA
    return {k: f(cfg) for k, f in table.items()}


def make_weights(cfg: ModelConfig, seed: int, device: str = "cpu") -> Dict[str, torch.Tensor]:
    """All weights in the config dtype, every linear weight stored [out, in] (input index
    contiguous), stacked over layers in the leading dimension.  Drawn in fp32 and rounded
    to the dtype.  `device` only chooses where the draw happens (values differ between
    devices; a test always hands the same tensors to both sides)."""
    dt = TORCH_DTYPE[cfg.dtype]
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    out: Dict[str, torch.Tensor] = {}
    for name, shape in weight_shapes(cfg).items():
        t = torch.empty(shape, dtype=dt, device=device)
        lead = shape[0] if len(shape) == 3 else 1
        view = t if len(shape) == 3 else t.unsqueeze(0)
        for i in range(lead):       # per-layer draws bound the fp32 temporary
            r = torch.randn(view[i].shape, generator=gen, device=device, dtype=torch.float32) * 0.02
            if name.endswith("_g"):
                r += 1.0
            view[i].copy_(r)
        out[name] = t
    return out


PER_LAYER_NAMES = ("ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo", "ln2_g", "ln2_b", "w1", "b1", "wu", "w2", "b2")


def make_weights_layerwise(cfg: ModelConfig, seed: int, device: str = "cpu"):
    """For models too large to hold as one stacked copy: (global tensors, iterator over per-layer dicts).  Layer l is
    drawn from its own seed, so layers can be produced (and dropped) one at a time; same distributions as make_weights."""
    one = dataclasses.replace(cfg, L=1)
    glob = {k: v for k, v in make_weights(one, seed, device).items() if k not in PER_LAYER_NAMES}

    def layers():
        for l in range(cfg.L):
            w = make_weights(one, seed * 1009 + 17 + l, device)
            yield {k: w[k][0].contiguous() for k in PER_LAYER_NAMES if k in w}

    return glob, layers()


# --------------------------------------------------------------------------- request streams

@dataclasses.dataclass
class Request:
    req_id: int
    arrival_step: int
    prompt: np.ndarray      # int32 [P]
    gen_len: int            # G: number of tokens to generate


def _finish(rng, arrivals, P, G, V) -> List[Request]:
    order = np.argsort(arrivals, kind="stable")
    reqs = []
    for rid, i in enumerate(order):
        prompt = rng.integers(0, V, size=int(P[i]), dtype=np.int64).astype(np.int32)
        reqs.append(Request(rid, int(arrivals[i]), prompt, int(G[i])))
    return reqs


def poisson_arrivals(rng, n: int, rate_of_step) -> np.ndarray:
    """Arrival step of each of n requests when the number arriving in step s is Poisson(rate_of_step(s))."""
    arr = []
    s = 0
    while len(arr) < n:
        k = int(rng.poisson(rate_of_step(s)))
        arr.extend([s] * k)
        s += 1
    return np.asarray(arr[:n], dtype=np.int64)


def stream_c1(seed: int, V: int = 1024, n: int = 8) -> List[Request]:
    """8 requests, arrival step U{0..20}, prompt length U{8..32}, generation length U{16..64}."""
    rng = np.random.default_rng(seed)
    arr = rng.integers(0, 21, size=n)
    P = rng.integers(8, 33, size=n)
    G = rng.integers(16, 65, size=n)
    return _finish(rng, arr, P, G, V)


def stream_c3(seed: int, V: int = 50257, n: int = 64) -> List[Request]:
    """64 requests, Poisson arrivals (mean 1 per 4 steps), prompt U{64..512}, generation U{32..1024}."""
    rng = np.random.default_rng(seed)
    arr = poisson_arrivals(rng, n, lambda s: 0.25)
    P = rng.integers(64, 513, size=n)
    G = rng.integers(32, 1025, size=n)
    return _finish(rng, arr, P, G, V)


def stream_c4(seed: int, V: int = 32000, n: int = 128, p_lo: int = 32, p_hi: int = 1024,
              g_lo: int = 16, g_hi: int = 1024, rate: float = 2.0) -> List[Request]:
    """128 requests, Poisson arrivals (mean 2 per step), prompt U{32..1024}, generation log-uniform 16..1024."""
    rng = np.random.default_rng(seed)
    arr = poisson_arrivals(rng, n, lambda s: rate)
    P = rng.integers(p_lo, p_hi + 1, size=n)
    u = rng.random(size=n)
    G = np.minimum(np.floor(g_lo * (g_hi / g_lo) ** u).astype(np.int64), g_hi)
    return _finish(rng, arr, P, G, V)


def stream_c5(seed: int, V: int = 32000, n: int = 512, S: int = 2048) -> List[Request]:
    """512 requests, bursty Poisson (rate alternating 1 and 8 per step every 200 steps), prompt U{16..512},
    generation U{8..2048} clamped so that prompt + generation fits the slot."""
    rng = np.random.default_rng(seed)
    arr = poisson_arrivals(rng, n, lambda s: 1.0 if (s // 200) % 2 == 0 else 8.0)
    P = rng.integers(16, 513, size=n)
    G = np.minimum(rng.integers(8, 2049, size=n), S - P)
    return _finish(rng, arr, P, G, V)


def stream_bursty(seed: int, V: int, n: int, period: int, rate_lo: float, rate_hi: float, p_lo: int, p_hi: int, g_lo: int,
                  g_hi: int) -> List[Request]:
    """The arrival pattern of the 30B configuration at any scale: Poisson counts per step whose rate alternates between
    rate_lo and rate_hi every `period` steps; prompt and generation lengths uniform."""
    rng = np.random.default_rng(seed)
    arr = poisson_arrivals(rng, n, lambda s: rate_lo if (s // period) % 2 == 0 else rate_hi)
    P = rng.integers(p_lo, p_hi + 1, size=n)
    G = rng.integers(g_lo, g_hi + 1, size=n)
    return _finish(rng, arr, P, G, V)


def stream_small(seed: int, V: int, n: int, arrive_hi: int, p_lo: int, p_hi: int, g_lo: int, g_hi: int) -> List[Request]:
    rng = np.random.default_rng(seed)
    arr = rng.integers(0, arrive_hi + 1, size=n)
    P = rng.integers(p_lo, p_hi + 1, size=n)
    G = rng.integers(g_lo, g_hi + 1, size=n)
    return _finish(rng, arr, P, G, V)


def stream_constant_interval(seed: int, V: int, n: int, gap_steps: int, P: int, G: int) -> List[Request]:
    """Section VI-B: requests separated by a constant interval, here counted in decode steps."""
    rng = np.random.default_rng(seed)
    arr = np.arange(n, dtype=np.int64) * gap_steps
    return _finish(rng, arr, np.full(n, P), np.full(n, G), V)


def exponential_gap_arrivals(seed: int, n: int, mean_gap_steps: float) -> np.ndarray:
    """Section IV / VI-C: inter-arrival gaps drawn from an exponential distribution, quantised to steps."""
    rng = np.random.default_rng(seed)
    gaps = rng.exponential(mean_gap_steps, size=n)
    gaps[0] = 0.0
    return np.floor(np.cumsum(gaps)).astype(np.int64)


# --------------------------------------------------------------------------- micro-benchmark tensors (config 2)

def attention_case(seed: int, M: int, C: int, nh: int, d: int, S: int, dtype: int, len_lo: int, len_hi: int,
                   device: str = "cpu", fill: str = "valid"):
    """One layer's K/V cache [C][nh][S][d], q [M][nh][d] ~ N(0,1), distinct seeded slots and lengths
    (len = number of cached rows the query attends to, U{len_lo..len_hi}).
    fill="valid" draws only the rows < len of the used slots (the rest stay zero); "all" draws everything."""
    dt = TORCH_DTYPE[dtype]
    rng = np.random.default_rng(seed)
    slots = rng.permutation(C)[:M].astype(np.int32)
    lens = rng.integers(len_lo, len_hi + 1, size=M).astype(np.int32)
    gen = torch.Generator(device=device)
    gen.manual_seed(seed + 1)
    q = torch.randn((M, nh, d), generator=gen, device=device, dtype=torch.float32).to(dt)
    if fill == "all":
        k = torch.empty((C, nh, S, d), dtype=dt, device=device)
        v = torch.empty((C, nh, S, d), dtype=dt, device=device)
        for c in range(C):
            k[c].copy_(torch.randn((nh, S, d), generator=gen, device=device, dtype=torch.float32))
            v[c].copy_(torch.randn((nh, S, d), generator=gen, device=device, dtype=torch.float32))
    else:
        k = torch.zeros((C, nh, S, d), dtype=dt, device=device)
        v = torch.zeros((C, nh, S, d), dtype=dt, device=device)
        for s, n in zip(slots.tolist(), lens.tolist()):
            k[s, :, :n].copy_(torch.randn((nh, n, d), generator=gen, device=device, dtype=torch.float32))
            v[s, :, :n].copy_(torch.randn((nh, n, d), generator=gen, device=device, dtype=torch.float32))
    return q, k, v, slots, lens


def occupancy_arrays(seed: int, n_arrays: int, max_len: int) -> List[np.ndarray]:
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n_arrays):
        n = int(rng.integers(1, max_len + 1))
        p = rng.random()
        out.append((rng.random(n) < p).astype(np.int32))
    return out
