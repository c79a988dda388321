"""Pins for the oracle's attention (Section 3.1, Eq. 1) and for the way quantized and
full-precision tokens enter it: library routines, closed forms, invariants, and an
independent numpy reconstruction of X^ from the canonical dump."""
import numpy as np
import pytest
from scipy.special import softmax

import kvq_workloads as W


def _rand16(rng, *shape, scale=1.0):
    return (rng.standard_normal(shape) * scale).astype(np.float16)


def _numpy_attention(q, K, V):
    """Eq. 1 with library routines in float64; q [B,Hq,D], K,V [B,Hkv,T,D] (any float dtype)."""
    q, K, V = q.astype(np.float64), K.astype(np.float64), V.astype(np.float64)
    B, Hq, D = q.shape
    gq = Hq // K.shape[1]
    out = np.zeros((B, Hq, D))
    p = np.zeros((B, Hq, K.shape[2]))
    for b in range(B):
        for h in range(Hq):
            p[b, h] = softmax(K[b, h // gq] @ q[b, h] / np.sqrt(D))
            out[b, h] = p[b, h] @ V[b, h // gq]
    return out, p


def test_exact_attention_matches_scipy(oracle_mod):
    rng = np.random.default_rng(1)
    for (B, Hq, Hkv, T, D) in [(2, 8, 2, 37, 128), (1, 7, 1, 5, 64), (3, 4, 4, 1, 32), (1, 6, 3, 130, 128)]:
        q, K, V = _rand16(rng, B, Hq, D), _rand16(rng, B, Hkv, T, D, scale=2.0), _rand16(rng, B, Hkv, T, D)
        o16, o64, p = oracle_mod.attention_exact(q, K, V, want_p=True)
        ro, rp = _numpy_attention(q, K, V)
        assert np.allclose(o64, ro, rtol=1e-12, atol=1e-13)
        assert np.allclose(p, rp, rtol=1e-12, atol=1e-15)
        assert np.all(np.abs(p.sum(-1) - 1) < 1e-12)
        assert np.array_equal(o16.view(np.uint16), o64.astype(np.float16).view(np.uint16))


def test_tiny_hand_computable_cases(oracle_mod):
    # one token: the output is that token's value row
    q = np.array([[[1.0, -2.0]]], dtype=np.float16)
    K = np.array([[[[0.5, 0.25]]]], dtype=np.float16)
    V = np.array([[[[3.0, -4.0]]]], dtype=np.float16)
    o16, o64 = oracle_mod.attention_exact(q, K, V)
    assert o64.tolist() == [[[3.0, -4.0]]]
    # two tokens, D = 4: p = sigmoid of the logit gap; q.k0 = 2, q.k1 = 0 -> gap = 2 / sqrt(4) = 1
    q = np.array([[[1.0, 1.0, 0.0, 0.0]]], dtype=np.float16)
    K = np.array([[[[1.0, 1.0, 5.0, 5.0], [1.0, -1.0, 7.0, -7.0]]]], dtype=np.float16)
    V = np.array([[[[1.0, 0.0, 2.0, 0.0], [0.0, 1.0, 0.0, 4.0]]]], dtype=np.float16)
    _, o64, p = oracle_mod.attention_exact(q, K, V, want_p=True)
    p0 = 1.0 / (1.0 + np.exp(-1.0))
    assert np.allclose(p[0, 0], [p0, 1 - p0], rtol=1e-14)
    assert np.allclose(o64[0, 0], [p0, 1 - p0, 2 * p0, 4 * (1 - p0)], rtol=1e-14)
    # all keys equal -> uniform weights -> mean of the values
    rng = np.random.default_rng(2)
    V = _rand16(rng, 1, 1, 9, 8)
    K = np.tile(_rand16(rng, 1, 1, 1, 8), (1, 1, 9, 1))
    q = _rand16(rng, 1, 3, 8)
    _, o64, p = oracle_mod.attention_exact(q, K, V, want_p=True)
    assert np.allclose(p, 1.0 / 9, rtol=1e-13)
    assert np.allclose(o64, np.broadcast_to(V.astype(np.float64).mean(2), (1, 3, 8)), rtol=1e-13)


def test_softmax_is_invariant_to_a_common_key_shift(oracle_mod):
    """Adding the same vector to every key adds the same constant to every logit."""
    rng = np.random.default_rng(3)
    q = _rand16(rng, 1, 4, 16)
    Kint = rng.integers(-8, 8, (1, 2, 20, 16)).astype(np.float16)
    shift = rng.integers(-8, 8, (1, 2, 1, 16)).astype(np.float16)
    V = _rand16(rng, 1, 2, 20, 16)
    _, o1, p1 = oracle_mod.attention_exact(q, Kint, V, want_p=True)
    _, o2, p2 = oracle_mod.attention_exact(q, (Kint + shift).astype(np.float16), V, want_p=True)
    assert np.allclose(p1, p2, rtol=1e-11)
    assert np.allclose(o1, o2, rtol=1e-11, atol=1e-13)


def test_gqa_head_mapping(oracle_mod):
    """q head h reads kv head h // g_q: equal queries inside a group give equal rows; Hq == Hkv is per-head MHA."""
    rng = np.random.default_rng(4)
    K, V = _rand16(rng, 1, 2, 11, 32), _rand16(rng, 1, 2, 11, 32)
    q1 = _rand16(rng, 1, 1, 32)
    q = np.tile(q1, (1, 6, 1))
    _, o64 = oracle_mod.attention_exact(q, K, V)
    assert np.array_equal(o64[0, 0], o64[0, 1]) and np.array_equal(o64[0, 1], o64[0, 2])
    assert np.array_equal(o64[0, 3], o64[0, 5]) and not np.allclose(o64[0, 0], o64[0, 3])
    # per-head: kv head 1 with one q head equals the (b, h) = (0, 1) slice run alone
    _, o_mha = oracle_mod.attention_exact(np.tile(q1, (1, 2, 1)), K, V)
    _, o_one = oracle_mod.attention_exact(q1, K[:, 1:2], V[:, 1:2])
    assert np.array_equal(o_mha[0, 1], o_one[0, 0])
    assert np.array_equal(o_mha[0, 1], o64[0, 3])


def _unpack_le(packed, bits, n):
    """Independent little-endian unpack with numpy: element i sits at bits [i*bits, (i+1)*bits)."""
    b = np.unpackbits(packed.astype(np.uint8), axis=-1, bitorder="little")
    b = b[..., : n * bits].reshape(packed.shape[:-1] + (n, bits))
    return (b * (1 << np.arange(bits))).sum(-1)


def _reconstruct(ex, kb, vb, D, G):
    """X^ = Q(X) s + z rebuilt in numpy from the canonical dump, then the fp16 tail appended."""
    B, H = ex["k_res"].shape[:2]
    Np = ex["n_packed"]
    if kb < 16:
        codes = _unpack_le(ex["k_codes"], kb, G)                          # [B,H,Np/G,D,G]
        kh = codes * ex["k_scale"][..., None].astype(np.float64) + ex["k_zero"][..., None].astype(np.float64)
        kh = kh.transpose(0, 1, 2, 4, 3).reshape(B, H, Np, D)
    else:
        kh = ex["k_codes"].view(np.float16).astype(np.float64)
    if vb < 16:
        codes = _unpack_le(ex["v_codes"], vb, D).reshape(B, H, Np, D // G, G)
        vh = codes * ex["v_scale"][..., None].astype(np.float64) + ex["v_zero"][..., None].astype(np.float64)
        vh = vh.reshape(B, H, Np, D)
    else:
        vh = ex["v_codes"].view(np.float16).astype(np.float64)
    kh = np.concatenate([kh, ex["k_res"].view(np.float16).astype(np.float64)], axis=2)
    vh = np.concatenate([vh, ex["v_res"].view(np.float16).astype(np.float64)], axis=2)
    return kh, vh


@pytest.mark.parametrize("kb,vb", [(8, 4), (4, 2), (2, 8), (8, 8), (16, 4), (4, 16), (2, 2)])
def test_decode_equals_exact_attention_over_reconstructed_cache(oracle_mod, kb, vb):
    """The decode output is Eq. 1 applied to [X^ of the quantized tokens, fp16 tail], rebuilt independently."""
    rng = np.random.default_rng(10 * kb + vb)
    B, Hq, Hkv, D, T = 2, 6, 2, 64, 32 * 4 + 19
    K = _rand16(rng, B, Hkv, T, D, scale=1.5)
    K[:, :, :, 5] *= 10
    V = _rand16(rng, B, Hkv, T, D)
    q = _rand16(rng, B, Hq, D)
    oc = oracle_mod.OracleCache(1, B, Hq, Hkv, D, [kb], [vb])
    oc.quantize_append(0, K, V)
    o16, o64, p = oc.decode_attention(0, q, want_p=True)
    ex = oc.export(0)
    assert (ex["n_packed"], ex["n_residual"]) == (96, 51)
    kh, vh = _reconstruct(ex, kb, vb, D, 32)
    ro, rp = _numpy_attention(q, kh, vh)
    assert np.allclose(o64, ro, rtol=1e-11, atol=1e-13)
    assert np.allclose(p, rp, rtol=1e-11, atol=1e-15)
    assert np.all(np.abs(p.sum(-1) - 1) < 1e-12)
    assert np.array_equal(o16.view(np.uint16), o64.astype(np.float16).view(np.uint16))
    # the fp16 tail is the newest tokens, untouched
    assert np.array_equal(ex["k_res"], K[:, :, 96:].view(np.uint16))
    assert np.array_equal(ex["v_res"], V[:, :, 96:].view(np.uint16))
    # each reconstructed element is within half a step of the original (Eq. 2 with round-to-nearest)
    if kb < 16:
        step = np.repeat(ex["k_scale"].astype(np.float64), 32, axis=2)
        assert np.all(np.abs(kh[:, :, :96] - K[:, :, :96].astype(np.float64)) <= step / 2 * (1 + 1e-6) + 1e-6)
    if vb < 16:
        step = np.repeat(ex["v_scale"].astype(np.float64), 32, axis=3)
        assert np.all(np.abs(vh[:, :, :96] - V[:, :, :96].astype(np.float64)) <= step / 2 * (1 + 1e-6) + 1e-6)


def test_key_groups_run_over_tokens_and_value_groups_over_channels(oracle_mod):
    """Keys whose channels live on very different offsets, values whose tokens do: with the KIVI axes every
    step is exactly 1 and the codes are the small integers themselves; any other grouping would not be."""
    rng = np.random.default_rng(11)
    B, H, D, T = 1, 1, 64, 64 + 32
    small_k = rng.integers(0, 4, (B, H, T, D))
    small_k[:, :, 0::32, :] = 0
    small_k[:, :, 1::32, :] = 3
    K = (small_k + 16.0 * np.arange(D)[None, None, None, :]).astype(np.float16)        # per-channel offset
    small_v = rng.integers(0, 16, (B, H, T, D))
    small_v[..., 0::32] = 0
    small_v[..., 1::32] = 15
    V = (small_v + 32.0 * (np.arange(T) % 50)[None, None, :, None]).astype(np.float16)  # per-token offset
    oc = oracle_mod.OracleCache(1, B, 1, H, D, [2], [4])
    oc.quantize_append(0, K, V)
    ex = oc.export(0)
    assert ex["n_packed"] == 64
    assert np.all(ex["k_scale"] == 1.0) and np.all(ex["v_scale"] == 1.0)
    assert np.array_equal(ex["k_zero"][0, 0, 0], 16.0 * np.arange(D))
    assert np.array_equal(ex["v_zero"][0, 0, :, 0], 32.0 * (np.arange(64) % 50))
    kc = _unpack_le(ex["k_codes"], 2, 32)          # [B,H,2,D,32]
    assert np.array_equal(kc.transpose(0, 1, 2, 4, 3).reshape(B, H, 64, D), small_k[:, :, :64])
    vc = _unpack_le(ex["v_codes"], 4, D)
    assert np.array_equal(vc, small_v[:, :, :64])


def test_sixteen_bit_mode_is_exact_attention(oracle_mod):
    rng = np.random.default_rng(12)
    B, Hq, Hkv, D, T = 2, 8, 2, 128, 200
    q, K, V = _rand16(rng, B, Hq, D), _rand16(rng, B, Hkv, T, D), _rand16(rng, B, Hkv, T, D)
    oc = oracle_mod.OracleCache(1, B, Hq, Hkv, D, [16], [16])
    oc.quantize_append(0, K, V)
    o16, o64 = oc.decode_attention(0, q)
    e16, e64 = oracle_mod.attention_exact(q, K, V)
    assert np.array_equal(o64, e64) and np.array_equal(o16.view(np.uint16), e16.view(np.uint16))


def test_logit_error_is_bounded_by_half_steps(oracle_mod):
    """|score - score^| <= sum_d |q_d| s_d / (2 sqrt(D)) follows from |k - k^| <= s / 2."""
    rng = np.random.default_rng(13)
    B, Hq, Hkv, D, T = 1, 4, 1, 128, 64 + 32
    q, K, V = _rand16(rng, B, Hq, D), _rand16(rng, B, Hkv, T, D), _rand16(rng, B, Hkv, T, D)
    for kb in (2, 4, 8):
        oc = oracle_mod.OracleCache(1, B, Hq, Hkv, D, [kb], [16])
        oc.quantize_append(0, K, V)
        ex = oc.export(0)
        kh, _ = _reconstruct(ex, kb, 16, D, 32)
        s_hat = np.einsum("bhd,btd->bht", q.astype(np.float64), kh[:, 0]) / np.sqrt(D)
        s_ref = np.einsum("bhd,btd->bht", q.astype(np.float64), K[:, 0].astype(np.float64)) / np.sqrt(D)
        step = np.repeat(ex["k_scale"][0, 0].astype(np.float64), 32, axis=0)          # [64, D]
        bound = np.abs(q.astype(np.float64))[0] @ step.T / (2 * np.sqrt(D))              # [Hq, 64]
        assert np.all(np.abs(s_hat - s_ref)[0, :, :64] <= bound * (1 + 1e-6) + 1e-9)
        assert np.all(np.abs(s_hat - s_ref)[0, :, 64:] == 0)


def test_dominating_key_makes_output_insensitive_to_key_bits(oracle_mod):
    """One key with a far larger logit than the rest: the output is that token's value row whatever the key bits
    (the concentrated-attention case of the paper's lemma on robustness of sparse heads)."""
    rng = np.random.default_rng(14)
    B, Hq, Hkv, D, T = 1, 2, 1, 128, 96
    q = np.full((B, Hq, D), 1.0, dtype=np.float16)
    K = _rand16(rng, B, Hkv, T, D, scale=0.1)
    K[0, 0, 17] = 6.0
    V = _rand16(rng, B, Hkv, T, D)
    for kb in (2, 4, 8):
        oc = oracle_mod.OracleCache(1, B, Hq, Hkv, D, [kb], [16])
        oc.quantize_append(0, K, V)
        _, o64, p = oc.decode_attention(0, q, want_p=True)
        assert np.all(p[:, :, 17] > 1 - 1e-9)
        assert np.allclose(o64[0, 0], V[0, 0, 17].astype(np.float64), atol=1e-7)


def test_outlier_channels_get_proportionally_larger_steps(oracle_mod):
    """Per-channel key grouping isolates outlier channels: their step grows ~10x, the others are untouched."""
    w = W.config1()
    K, V = W.kv_tokens(w, 0, 0, w.context)
    scale, _ = W.key_channel_profile(w, 0)
    assert int((scale == 10.0).sum()) == 4 * w.n_kv_heads
    oc = oracle_mod.OracleCache(1, 1, 8, 2, 128, [8], [4])
    oc.quantize_append(0, K.numpy(), V.numpy())
    ks = oc.export(0)["k_scale"].astype(np.float64).mean(axis=2)[0]      # [Hkv, D]
    out = scale.numpy() == 10.0
    ratio = ks[out].mean() / ks[~out].mean()
    assert 8.0 < ratio < 12.0
