"""Seeded synthetic inputs for the KV-cache quantization path.

This module serves the CPU oracle's tests, the GPU parity tests and the
benchmark alike.  It holds none of the method's arithmetic: it only produces
fp16 tensors (queries, keys, values) whose shapes and value structure follow
the workloads the paper measures on -- Llama-3.1-8B and Qwen2.5-7B caches
(experimental-settings appendix), keys with a few strong outlier channels
(Section 4.2) -- because the model weights and prompts themselves are not
available here.

Values come from a counter-based generator: a 64-bit integer hash of
(seed, tensor id, flat element index) feeds an Irwin-Hall sum of twelve 16-bit
uniforms, so an element depends only on its index.  Everything up to the final
fp16 rounding is integer arithmetic or single IEEE fp32 operations in torch,
which makes the CPU and the GPU produce the same bits and lets a test draw any
slice of a large tensor without materialising the rest.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

import torch

_M64 = (1 << 64) - 1


def _i64(x: int) -> int:
    """Python int -> two's complement int64 value."""
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


_C1 = _i64(0x9E3779B97F4A7C15)
_C2 = _i64(0xBF58476D1CE4E5B9)
_C3 = _i64(0x94D049BB133111EB)


def _lsr(x: torch.Tensor, k: int) -> torch.Tensor:
    """Logical shift right on int64 (torch's >> is arithmetic)."""
    return (x >> k) & ((1 << (64 - k)) - 1)


def _mix(x: torch.Tensor) -> torch.Tensor:
    """splitmix64 finaliser on int64 tensors (wrapping arithmetic)."""
    x = (x ^ _lsr(x, 30)) * _C2
    x = (x ^ _lsr(x, 27)) * _C3
    return x ^ _lsr(x, 31)


def _key(seed: int, tensor_id: int) -> int:
    k = (seed * 0x9E3779B97F4A7C15 + tensor_id * 0xD1B54A32D192ED03 + 0x2545F4914F6CDD1D) & _M64
    k ^= k >> 29
    k = (k * 0xBF58476D1CE4E5B9) & _M64
    k ^= k >> 32
    return k


def standard_normal(seed: int, tensor_id: int, index: torch.Tensor) -> torch.Tensor:
    """Approximately N(0,1) fp32 values, one per int64 flat index, bit-reproducible on any device."""
    base = index * 3 + _i64(_key(seed, tensor_id))
    total = torch.zeros_like(index)
    for w in range(3):
        h = _mix((base + w) * _C1)
        for f in range(4):
            total = total + ((h >> (16 * f)) & 0xFFFF)
    # twelve uniforms on [0, 65535]: mean 393210, standard deviation ~65536
    return (total - 393210).to(torch.float32) * (1.0 / 65536.0)


def uniform_u32(seed: int, tensor_id: int, n: int) -> List[int]:
    """n seeded 32-bit integers (host side; used for choosing outlier channels)."""
    idx = torch.arange(n, dtype=torch.int64)
    h = _mix((idx + _i64(_key(seed, tensor_id))) * _C1)
    return [int(v) for v in (_lsr(h, 32)).tolist()]


# --------------------------------------------------------------------------- workloads


@dataclass
class Workload:
    """One synthetic cache configuration (shapes, per-layer bits, value structure)."""

    name: str
    n_layers: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    context: int                      # tokens in the cache before the decode step
    kbits: List[int]
    vbits: List[int]
    seed: int
    group: int = 32
    residual: int = 32
    outlier_channels: int = 0         # key channels per (layer, kv head) scaled by outlier_scale
    outlier_scale: float = 10.0
    key_bias_std: float = 0.0         # std of a per-channel offset added to the keys
    note: str = ""
    extra: dict = field(default_factory=dict)

    @property
    def g_q(self) -> int:
        return self.n_q_heads // self.n_kv_heads


def schedule_from_spec(n_layers: int, spec: Sequence[Tuple[int, int, Sequence[int]]]) -> Tuple[List[int], List[int]]:
    """[(kbits, vbits, layers), ...] -> per-layer lists.  Every layer must be covered exactly once."""
    kb, vb = [0] * n_layers, [0] * n_layers
    for k, v, layers in spec:
        for l in layers:
            if kb[l]:
                raise ValueError("layer %d listed twice" % l)
            kb[l], vb[l] = k, v
    if not all(kb):
        raise ValueError("schedule leaves layers unset")
    return kb, vb


def _rng(a: int, b: int) -> List[int]:
    return list(range(a, b + 1))


def llama_mix_325() -> Tuple[List[int], List[int]]:
    """The benchmark's 3.25-bit schedule: layers 0-3 and 28-31 K4V4, layers 4-27 K4V2."""
    return schedule_from_spec(32, [(4, 4, _rng(0, 3) + _rng(28, 31)), (4, 2, _rng(4, 27))])


def llama_kivi_c325() -> Tuple[List[int], List[int]]:
    """Llama-3.1-8B KIVI 3.25-bit schedule as listed in the paper's table of searched configurations."""
    return schedule_from_spec(32, [
        (8, 4, [13, 17]),
        (4, 4, [1, 2, 3, 7, 29, 31]),
        (4, 2, [5, 6] + _rng(8, 12) + _rng(14, 16) + _rng(18, 24) + [26, 28, 30]),
        (2, 2, [0, 4, 25, 27]),
    ])


def llama_kivi_c490() -> Tuple[List[int], List[int]]:
    """Llama-3.1-8B KIVI 4.90-bit schedule from the same table."""
    return schedule_from_spec(32, [
        (8, 4, [4, 6] + _rng(8, 12) + _rng(14, 16) + _rng(18, 20) + [22] + _rng(25, 28) + [30]),
        (4, 4, [1, 2, 3, 7, 29, 31]),
        (4, 2, [5, 21, 23, 24]),
        (2, 4, [0]),
        (2, 2, [13, 17]),
    ])


def qwen_kivi_c392() -> Tuple[List[int], List[int]]:
    """Qwen2.5-7B KIVI 3.92-bit schedule from the same table (28 layers; uniform pairs KV8 / KV4 / KV2)."""
    return schedule_from_spec(28, [
        (8, 8, [0, 2, 6, 11, 15, 17]),
        (4, 4, [4, 5, 8, 12] + _rng(22, 26)),
        (2, 2, [1, 3, 7, 9, 10, 13, 14, 16] + _rng(18, 21) + [27]),
    ])


def qwen_mix_40() -> Tuple[List[int], List[int]]:
    """The benchmark's 4.0-bit schedule for the 28-layer Qwen shape: even layers K8V2, odd K4V2."""
    return [8 if l % 2 == 0 else 4 for l in range(28)], [2] * 28


def config1() -> Workload:
    return Workload("cfg1-gqa8x2-T512-K8V4", 1, 1, 8, 2, 128, 512, [8], [4], seed=1, outlier_channels=4,
                    note="single layer correctness case")


def config2(batch: int = 16, context: int = 4096) -> Workload:
    return Workload("llama8b-B%d-T%d-K8V8" % (batch, context), 32, batch, 32, 8, 128, context,
                    [8] * 32, [8] * 32, seed=2, outlier_channels=3, note="uniform KV8 baseline")


def config3(batch: int = 16, context: int = 8192) -> Workload:
    kb, vb = llama_mix_325()
    return Workload("llama8b-B%d-T%d-mix3.25" % (batch, context), 32, batch, 32, 8, 128, context, kb, vb,
                    seed=3, outlier_channels=3, note="3.25-bit mixed schedule")


def config4(batch: int = 8, context: int = 32768) -> Workload:
    kb, vb = qwen_mix_40()
    return Workload("qwen7b-B%d-T%d-mix4.0" % (batch, context), 28, batch, 28, 4, 128, context, kb, vb,
                    seed=4, key_bias_std=20.0, note="g_q = 7, biased keys")


SCHEDULES = {
    # family -> schedule name -> (function, layers, q heads, kv heads, extra Workload arguments)
    "llama8b": {"mix3.25": llama_mix_325, "kivi-c3.25": llama_kivi_c325, "kivi-c4.90": llama_kivi_c490},
    "qwen7b": {"mix4.0": qwen_mix_40, "kivi-c3.92": qwen_kivi_c392},
}


def named(family: str, schedule: str, batch: int, context: int) -> Workload:
    """Workload of a model shape (llama8b: 32 layers, 32/8 heads; qwen7b: 28 layers, 28/4 heads, biased keys) with one
    of its layer-wise schedules, or "K<k>V<v>" for a uniform pair."""
    shape = {"llama8b": (32, 32, 8, dict(seed=3, outlier_channels=3)), "qwen7b": (28, 28, 4, dict(seed=4, key_bias_std=20.0))}[family]
    L, hq, hkv, extra = shape
    if schedule in SCHEDULES[family]:
        kb, vb = SCHEDULES[family][schedule]()
    else:
        import re

        m = re.fullmatch(r"K(\d+)V(\d+)", schedule)
        if not m:
            raise ValueError("unknown schedule %r for %s (have %s or K<k>V<v>)" % (schedule, family, ", ".join(SCHEDULES[family])))
        kb, vb = [int(m.group(1))] * L, [int(m.group(2))] * L
    return Workload("%s-B%d-T%d-%s" % (family, batch, context, schedule), L, batch, hq, hkv, 128, context, kb, vb, **extra)


def llama_uniform(kbit: int, vbit: int, batch: int, context: int, seed: int = 5) -> Workload:
    return Workload("llama8b-B%d-T%d-K%dV%d" % (batch, context, kbit, vbit), 32, batch, 32, 8, 128, context,
                    [kbit] * 32, [vbit] * 32, seed=seed, outlier_channels=3)


def llama_mix(batch: int, context: int, seed: int = 5) -> Workload:
    w = config3(batch, context)
    w.seed = seed
    return w


# --------------------------------------------------------------------------- tensors

_K, _V, _Q, _CH, _BIAS, _QP = 0, 1, 2, 3, 4, 5


def _tid(layer: int, kind: int, stream: int = 0) -> int:
    return (stream * 4096 + layer) * 8 + kind


def key_channel_profile(w: Workload, layer: int) -> Tuple[torch.Tensor, torch.Tensor]:
    """Per (kv head, channel) multiplier and offset of the keys, fp32 [Hkv, D] each (host tensors)."""
    scale = torch.ones(w.n_kv_heads, w.head_dim, dtype=torch.float32)
    if w.outlier_channels:
        for h in range(w.n_kv_heads):
            draws = uniform_u32(w.seed, _tid(layer, _CH) * 1024 + h, w.head_dim)
            order = sorted(range(w.head_dim), key=lambda d: (draws[d], d))
            for d in order[: w.outlier_channels]:
                scale[h, d] = w.outlier_scale
    bias = torch.zeros(w.n_kv_heads, w.head_dim, dtype=torch.float32)
    if w.key_bias_std:
        idx = torch.arange(w.n_kv_heads * w.head_dim, dtype=torch.int64)
        bias = (standard_normal(w.seed, _tid(layer, _BIAS), idx) * float(w.key_bias_std)).reshape(
            w.n_kv_heads, w.head_dim)
    return scale, bias


def _flat_index(w: Workload, n_tokens: int, t0: int, t1: int, bh: torch.Tensor | None, device) -> torch.Tensor:
    """Flat indices of tokens [t0, t1) of a [B*Hkv, n_tokens, D] tensor, for all or selected (b, h) rows."""
    BH = w.batch * w.n_kv_heads
    rows = torch.arange(BH, dtype=torch.int64, device=device) if bh is None else bh.to(device=device, dtype=torch.int64)
    tok = torch.arange(t0, t1, dtype=torch.int64, device=device)
    ch = torch.arange(w.head_dim, dtype=torch.int64, device=device)
    return (rows[:, None, None] * n_tokens + tok[None, :, None]) * w.head_dim + ch[None, None, :]


def kv_tokens(w: Workload, layer: int, t0: int, t1: int, device="cpu", stream: int = 0,
              bh: torch.Tensor | None = None, total: int | None = None):
    """fp16 keys and values for tokens [t0, t1) of a stream that is `total` tokens long.

    Returns (K, V) shaped [B, Hkv, t1-t0, D]; with `bh` (a 1-D tensor of b*Hkv+h row numbers)
    shaped [len(bh), t1-t0, D] for just those rows.  `stream` separates the prefill context (0)
    from tokens appended during decode (1).
    """
    total = w.context if total is None else total
    idx = _flat_index(w, total, t0, t1, bh, device)
    k = standard_normal(w.seed, _tid(layer, _K, stream), idx)
    v = standard_normal(w.seed, _tid(layer, _V, stream), idx)
    scale, bias = key_channel_profile(w, layer)
    rows = torch.arange(w.batch * w.n_kv_heads, dtype=torch.int64) if bh is None else bh.to("cpu", torch.int64)
    head = (rows % w.n_kv_heads).to(torch.int64)
    sc = scale[head].to(device)[:, None, :]
    bi = bias[head].to(device)[:, None, :]
    k = k * sc
    k = k + bi
    k16, v16 = k.to(torch.float16), v.to(torch.float16)
    if bh is None:
        shape = (w.batch, w.n_kv_heads, t1 - t0, w.head_dim)
        return k16.reshape(shape), v16.reshape(shape)
    return k16, v16


def query(w: Workload, layer: int, step: int = 0, device="cpu") -> torch.Tensor:
    """fp16 decode query [B, Hq, D] for one layer and decode step."""
    n = w.batch * w.n_q_heads * w.head_dim
    idx = torch.arange(n, dtype=torch.int64, device=device) + step * n
    return standard_normal(w.seed, _tid(layer, _Q), idx).to(torch.float16).reshape(w.batch, w.n_q_heads, w.head_dim)


def prefill_queries(w: Workload, layer: int, n_q: int, device="cpu", heads=None) -> torch.Tensor:
    """fp16 queries [B, Hq, n_q, D] of the last n_q prompt positions of one layer (standard normal, like the decode
    queries).  heads: optional (first, count) range of query heads to draw, for sampling a large tensor."""
    h0, hc = (0, w.n_q_heads) if heads is None else heads
    b = torch.arange(w.batch, dtype=torch.int64, device=device).view(-1, 1, 1)
    h = torch.arange(h0, h0 + hc, dtype=torch.int64, device=device).view(1, -1, 1)
    e = torch.arange(n_q * w.head_dim, dtype=torch.int64, device=device).view(1, 1, -1)
    idx = (b * w.n_q_heads + h) * (n_q * w.head_dim) + e
    return standard_normal(w.seed, _tid(layer, _QP), idx.reshape(-1)).to(torch.float16).reshape(w.batch, hc, n_q, w.head_dim)
