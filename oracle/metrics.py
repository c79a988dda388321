"""Error figures of Section 3.2 of the paper, computed with the oracle (a reporting tool, test infrastructure).

    e_k = mean(|K - K^| / |K|),  e_v = mean(|V - V^| / |V|)      relative cache errors
    e_a = mean(|a - a^|)                                          absolute attention-score error
    e_o = mean(|o - o^| / |o|)                                    relative attention-output error

with a, o from exact attention on the fp16 cache and a^, o^ from attention over the dequantized cache
(Eq. 1 with K^, V^ of Eq. 2).  Elements whose reference value is zero are left out of the relative means.
"""
from __future__ import annotations

import numpy as np

from . import OracleCache, attention_exact


def error_metrics(q, K, V, kbits: int, vbits: int, group: int = 32, residual: int = 32, key_per_token: bool = False,
                  scale_fp16: bool = False) -> dict:
    """q fp16 [B, Hq, D]; K, V fp16 [B, Hkv, T, D] (one layer, the whole context appended at once)."""
    q, K, V = (np.ascontiguousarray(x, dtype=np.float16) for x in (q, K, V))
    B, Hq, D = q.shape
    Hkv = K.shape[1]
    oc = OracleCache(1, B, Hq, Hkv, D, [kbits], [vbits], group=group, residual=residual, scale_fp16=scale_fp16,
                     key_per_token=key_per_token)
    try:
        oc.quantize_append(0, K, V)
        Kh, Vh = oc.reconstruct(0)
        _, o_hat, a_hat = oc.decode_attention(0, q, want_p=True)
    finally:
        oc.close()
    _, o_ref, a_ref = attention_exact(q, K, V, want_p=True)
    K64, V64 = K.astype(np.float64), V.astype(np.float64)

    def rel(ref, hat):
        m = ref != 0
        return float(np.mean(np.abs(ref[m] - hat[m]) / np.abs(ref[m])))

    return {"e_k": rel(K64, Kh), "e_v": rel(V64, Vh), "e_a": float(np.mean(np.abs(a_ref - a_hat))), "e_o": rel(o_ref, o_hat)}
