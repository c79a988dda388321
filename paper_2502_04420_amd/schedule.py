"""Host-side helpers for layer-wise precision tables (no GPU work)."""
from __future__ import annotations

import re
from typing import List, Sequence, Tuple


def equivalent_precision(kbits: Sequence[int], vbits: Sequence[int]) -> float:
    """Average nominal bits per cached element, f_m(P) = sum(P) / (2 L) (Section 5.1 of the paper).

    Scales and zero-points are not counted, exactly as in the paper's definition.
    """
    if len(kbits) != len(vbits) or not kbits:
        raise ValueError("need one (key bits, value bits) pair per layer")
    return (sum(kbits) + sum(vbits)) / (2.0 * len(kbits))


def bytes_per_token(kbits: int, vbits: int, head_dim: int = 128, group: int = 32, scale_bytes: int = 4,
                    zero_bytes: int = 2) -> int:
    """Bytes one cached token of one kv head occupies once quantized, metadata included.

    Codes: head_dim * bits / 8 per tensor.  Metadata: keys carry (s, z) per channel per group of
    `group` tokens, values (s, z) per token per `group` channels -- head_dim / group pairs per token
    for each tensor.  The library stores s as fp32 and z as fp16 (z is a minimum of fp16 inputs, so
    the narrow store is exact); pass zero_bytes=4 for the all-fp32 figure.  16 bits means fp16 with
    no metadata.
    """
    total = 0
    for bits in (kbits, vbits):
        total += head_dim * bits // 8
        if bits < 16:
            total += (head_dim // group) * (scale_bytes + zero_bytes)
    return total


def parse_pairs(spec: str) -> Tuple[List[int], List[int]]:
    """'K8V4,KV4,K4V2' -> ([8, 4, 4], [4, 4, 2]); 'KV8' means K8V8 (the paper's shorthand)."""
    kb, vb = [], []
    for item in spec.replace(" ", "").split(","):
        m = re.fullmatch(r"K(\d+)V(\d+)", item) or re.fullmatch(r"KV(\d+)", item)
        if not m:
            raise ValueError("bad precision pair %r" % item)
        g = [int(x) for x in m.groups()]
        k, v = (g[0], g[0]) if len(g) == 1 else g
        if k not in (2, 4, 8, 16) or v not in (2, 4, 8, 16):
            raise ValueError("unsupported bits in %r" % item)
        kb.append(k)
        vb.append(v)
    return kb, vb
