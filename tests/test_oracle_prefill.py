"""Pins for the oracle's prefill-stage attention (the prompt's own causal attention reading the dequantized
cache, Section 5.3's calibration design): textbook causal attention on fp16 tensors, the pinned decode oracle
on the last row, a library-routine recomputation on the pinned reconstruction, and the one-token closed form."""
import numpy as np
import pytest
from scipy.special import softmax

from test_oracle_attention import _rand16


def _numpy_causal(q, K, V, T):
    """Eq. 1 under a causal mask with library routines in float64.  q [B,Hq,n_q,D] are the last n_q of T positions;
    K, V [B,Hkv,T,D]."""
    q, K, V = q.astype(np.float64), K.astype(np.float64), V.astype(np.float64)
    B, Hq, n_q, D = q.shape
    gq = Hq // K.shape[1]
    pos = np.arange(T - n_q, T)
    mask = np.arange(T)[None, :] <= pos[:, None]                     # [n_q, T]
    out = np.zeros((B, Hq, n_q, D))
    for b in range(B):
        for h in range(Hq):
            s = q[b, h] @ K[b, h // gq].T / np.sqrt(D)
            out[b, h] = softmax(np.where(mask, s, -np.inf), axis=-1) @ V[b, h // gq]
    return out


def test_fp16_layer_is_textbook_causal_attention(oracle_mod):
    rng = np.random.default_rng(11)
    for (B, Hq, Hkv, T, D, n_q) in [(2, 4, 2, 75, 128, 75), (1, 7, 1, 33, 64, 10), (1, 2, 2, 1, 128, 1)]:
        K, V = _rand16(rng, B, Hkv, T, D, scale=2.0), _rand16(rng, B, Hkv, T, D)
        q = _rand16(rng, B, Hq, n_q, D)
        oc = oracle_mod.OracleCache(1, B, Hq, Hkv, D, [16], [16])
        oc.quantize_append(0, K, V)
        o16, o64 = oc.prefill_attention(0, q)
        ref = _numpy_causal(q, K, V, T)
        assert np.allclose(o64, ref, rtol=1e-11, atol=1e-13)
        assert np.array_equal(o16, o64.astype(np.float16))


@pytest.mark.parametrize("per_token", [False, True])
@pytest.mark.parametrize("kb,vb", [(8, 8), (4, 2), (2, 4), (16, 2), (4, 16)])
def test_quantized_layer_against_reconstruction_and_decode(oracle_mod, kb, vb, per_token):
    rng = np.random.default_rng(100 + 10 * kb + vb + per_token)
    B, Hq, Hkv, D, T = 2, 6, 2, 128, 32 * 4 + 13
    K, V = _rand16(rng, B, Hkv, T, D, scale=1.5), _rand16(rng, B, Hkv, T, D)
    K[:, :, :, 5] *= 9
    q = _rand16(rng, B, Hq, T, D)
    oc = oracle_mod.OracleCache(1, B, Hq, Hkv, D, [kb], [vb], key_per_token=per_token)
    oc.quantize_append(0, K, V)
    npk, nr = oc.tokens(0)
    assert (npk, nr) == (96, 45)
    o16, o64 = oc.prefill_attention(0, q)
    # (a) library-routine recomputation on the reconstruction (itself pinned against the exported codes)
    Kh, Vh = oc.reconstruct(0)
    assert np.allclose(o64, _numpy_causal(q, Kh, Vh, T), rtol=1e-11, atol=1e-13)
    # (b) the last query sees every token: it is the decode oracle's answer for that query
    d16, d64 = oc.decode_attention(0, q[:, :, -1, :])
    assert np.array_equal(o64[:, :, -1, :], d64) and np.array_equal(o16[:, :, -1, :], d16)
    # (c) position 0 attends to itself only: the output is that token's value as the cache holds it
    gq = Hq // Hkv
    for h in range(Hq):
        assert np.array_equal(o64[:, h, 0, :], Vh[:, h // gq, 0, :])
    # (d) fewer queries are the tail of the full call
    p16, p64 = oc.prefill_attention(0, q[:, :, -17:, :])
    assert np.array_equal(p64, o64[:, :, -17:, :])
    # (d') queries at picked positions are the rows of the full call at those positions
    pos = [0, 1, 31, 32, 95, 96, 97, 140]
    a16, a64 = oc.prefill_attention_at(0, np.ascontiguousarray(q[:, :, pos, :]), pos)
    assert np.array_equal(a64, o64[:, :, pos, :]) and np.array_equal(a16, o16[:, :, pos, :])
    with pytest.raises(ValueError):
        oc.prefill_attention_at(0, np.ascontiguousarray(q[:, :, :1, :]), [T])
    # (e) quantization is visible where it should be: rows that see quantized tokens differ from the fp16 result
    if kb <= 4 or vb <= 4:
        exact = _numpy_causal(q, K, V, T)
        assert np.abs(o64 - exact).max() > 1e-3


def test_bad_arguments(oracle_mod):
    oc = oracle_mod.OracleCache(1, 1, 2, 1, 128, [4], [4])
    q = np.zeros((1, 2, 4, 128), dtype=np.float16)
    with pytest.raises(ValueError):
        oc.prefill_attention(0, q)                                   # empty cache
    oc.quantize_append(0, np.zeros((1, 1, 3, 128), dtype=np.float16), np.zeros((1, 1, 3, 128), dtype=np.float16))
    with pytest.raises(ValueError):
        oc.prefill_attention(0, q)                                   # more queries than tokens
