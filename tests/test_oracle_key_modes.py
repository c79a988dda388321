"""Pins for the oracle's second key grouping (keys per token over 32 channels, the paper's per-token-asym mode),
its reconstruct() view of the cache, and the error figures of Section 3.2 computed with it."""
import numpy as np
import pytest

import kvq_workloads as W
from test_oracle_attention import _numpy_attention, _rand16, _unpack_le


def _reconstruct_per_token_keys(ex, kb, D, G):
    B, H = ex["k_res"].shape[:2]
    Np = ex["n_packed"]
    codes = _unpack_le(ex["k_codes"], kb, D).reshape(B, H, Np, D // G, G)
    kh = codes * ex["k_scale"][..., None].astype(np.float64) + ex["k_zero"][..., None].astype(np.float64)
    return np.concatenate([kh.reshape(B, H, Np, D), ex["k_res"].view(np.float16).astype(np.float64)], axis=2)


@pytest.mark.parametrize("bits", [8, 4, 2])
def test_per_token_keys_are_coded_like_values(oracle_mod, bits):
    """The value path (per token over 32 channels) is pinned elsewhere; fed the same tensor, per-token keys must
    produce the very same codes, scales and zero-points."""
    rng = np.random.default_rng(40 + bits)
    X = _rand16(rng, 2, 3, 32 * 3 + 7, 128, scale=2.0)
    oc = oracle_mod.OracleCache(1, 2, 3, 3, 128, [bits], [bits], key_per_token=True)
    oc.quantize_append(0, X, X)
    ex = oc.export(0)
    assert ex["n_packed"] == 64
    for a, b in (("k_codes", "v_codes"), ("k_scale", "v_scale"), ("k_zero", "v_zero"), ("k_res", "v_res")):
        assert ex[a].shape == ex[b].shape and np.array_equal(ex[a], ex[b]), a
    # and the default grouping is a different encoding of the same tensor
    od = oracle_mod.OracleCache(1, 2, 3, 3, 128, [bits], [bits])
    od.quantize_append(0, X, X)
    assert od.export(0)["k_scale"].shape == (2, 3, 2, 128)


@pytest.mark.parametrize("per_token", [False, True])
@pytest.mark.parametrize("kb,vb", [(8, 4), (4, 2), (2, 2), (16, 8)])
def test_reconstruct_and_decode_agree_with_independent_numpy(oracle_mod, kb, vb, per_token):
    from test_oracle_attention import _reconstruct

    rng = np.random.default_rng(7 * kb + vb + per_token)
    B, Hq, Hkv, D, T = 1, 4, 2, 64, 32 * 3 + 9
    K, V, q = _rand16(rng, B, Hkv, T, D, scale=1.5), _rand16(rng, B, Hkv, T, D), _rand16(rng, B, Hq, D)
    K[:, :, :, 3] *= 8
    oc = oracle_mod.OracleCache(1, B, Hq, Hkv, D, [kb], [vb], key_per_token=per_token)
    oc.quantize_append(0, K, V)
    ex = oc.export(0)
    if per_token and kb < 16:
        # values through the shared helper (its key branch is given a dummy fp16 tensor), keys with the per-token rule
        dummy = {**ex, "k_codes": np.zeros((B, Hkv, ex["n_packed"], D), dtype=np.uint16)}
        _, vh = _reconstruct(dummy, 16, vb, D, 32)
        kh = _reconstruct_per_token_keys(ex, kb, D, 32)
    else:
        kh, vh = _reconstruct(ex, kb, vb, D, 32)
    Kh, Vh = oc.reconstruct(0)
    assert np.array_equal(Kh, kh) and np.array_equal(Vh, vh)
    o16, o64, p = oc.decode_attention(0, q, want_p=True)
    ro, rp = _numpy_attention(q, kh, vh)
    assert np.allclose(o64, ro, rtol=1e-11, atol=1e-13) and np.allclose(p, rp, rtol=1e-11, atol=1e-15)
    if per_token and kb < 16:
        step = np.repeat(ex["k_scale"].astype(np.float64), 32, axis=3)
        assert np.all(np.abs(kh[:, :, :64] - K[:, :, :64].astype(np.float64)) <= step / 2 * (1 + 1e-6) + 1e-6)


def test_error_figures_follow_their_definitions_and_the_papers_direction(oracle_mod):
    """e_k, e_v, e_a, e_o: zero for a 16-bit cache; equal to a direct numpy evaluation; and, on keys with
    outlier channels, grouping keys per channel gives a smaller key error and score error than per token at
    every precision while the value error does not depend on the key grouping (direction of the paper's
    table of per-channel vs per-token errors)."""
    from oracle.metrics import error_metrics

    w = W.Workload("metrics", 1, 1, 8, 2, 128, 512, [8], [8], seed=5, outlier_channels=3)
    K, V = (x.numpy() for x in W.kv_tokens(w, 0, 0, 512))
    q = W.query(w, 0).numpy()
    z = error_metrics(q, K, V, 16, 16)
    assert z == {"e_k": 0.0, "e_v": 0.0, "e_a": 0.0, "e_o": 0.0}
    prev = None
    for bits in (8, 4, 2):
        pc = error_metrics(q, K, V, bits, bits, residual=0)
        pt = error_metrics(q, K, V, bits, bits, residual=0, key_per_token=True)
        assert pc["e_k"] < 0.75 * pt["e_k"] and pc["e_a"] < pt["e_a"]
        assert pc["e_v"] == pt["e_v"]
        if prev is not None:
            assert pc["e_k"] > 4 * prev["e_k"] and pc["e_v"] > 4 * prev["e_v"] and pc["e_a"] > 2 * prev["e_a"]
        prev = pc
    # direct evaluation of the definitions for one setting
    oc = oracle_mod.OracleCache(1, 1, 8, 2, 128, [4], [2], residual=0)
    oc.quantize_append(0, K, V)
    Kh, Vh = oc.reconstruct(0)
    _, o_hat, a_hat = oc.decode_attention(0, q, want_p=True)
    o_ref, a_ref = _numpy_attention(q, K.astype(np.float64), V.astype(np.float64))
    m = error_metrics(q, K, V, 4, 2, residual=0)
    K64, V64 = K.astype(np.float64), V.astype(np.float64)
    assert m["e_k"] == pytest.approx(np.mean(np.abs(K64 - Kh)[K64 != 0] / np.abs(K64[K64 != 0])), rel=1e-12)
    assert m["e_v"] == pytest.approx(np.mean(np.abs(V64 - Vh)[V64 != 0] / np.abs(V64[V64 != 0])), rel=1e-12)
    assert m["e_a"] == pytest.approx(np.mean(np.abs(a_ref - a_hat)), rel=1e-9)
    assert m["e_o"] == pytest.approx(np.mean(np.abs(o_ref - o_hat) / np.abs(o_ref)), rel=1e-9)
