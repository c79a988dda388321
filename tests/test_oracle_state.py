"""Pins for the full-precision window: the closed form N_p(T) and independence from how appends are chunked."""
import numpy as np
import pytest


def _np_closed_form(T, G=32, R=32):
    return G * (max(T - R, 0) // G)


def _dumps_equal(a, b):
    assert a.keys() == b.keys()
    for k in a:
        if isinstance(a[k], np.ndarray):
            assert a[k].dtype == b[k].dtype and a[k].shape == b[k].shape, k
            assert np.array_equal(a[k].view(np.uint8), b[k].view(np.uint8)), k
        else:
            assert a[k] == b[k], k


@pytest.mark.parametrize("R", [0, 32, 64])
def test_packed_count_follows_closed_form(oracle_mod, R):
    rng = np.random.default_rng(1)
    B, H, D = 1, 1, 32
    oc = oracle_mod.OracleCache(1, B, 1, H, D, [4], [4], residual=R)
    T = 0
    for n in [1, 1, 30, 1, 31, 1, 1, 64, 5, 27, 100, 1]:
        K = rng.standard_normal((B, H, n, D)).astype(np.float16)
        oc.quantize_append(0, K, K)
        T += n
        npk, nr = oc.tokens(0)
        assert npk == _np_closed_form(T, 32, R) and npk + nr == T
        assert nr < R + 32 and (T < R or nr >= R)


def test_last_32_tokens_stay_fp16_at_512(oracle_mod):
    """The small correctness configuration: 512 tokens -> 480 quantized + 32 in fp16."""
    K = np.zeros((1, 2, 512, 128), dtype=np.float16)
    oc = oracle_mod.OracleCache(1, 1, 8, 2, 128, [8], [4])
    oc.quantize_append(0, K, K)
    assert oc.tokens(0) == (480, 32)


@pytest.mark.parametrize("kb,vb", [(8, 4), (2, 16), (16, 2)])
def test_chunked_appends_equal_bulk_append(oracle_mod, kb, vb):
    rng = np.random.default_rng(2)
    B, Hq, H, D, T = 2, 4, 2, 64, 32 * 5 + 7
    K = rng.standard_normal((B, H, T, D)).astype(np.float16)
    V = rng.standard_normal((B, H, T, D)).astype(np.float16)
    q = rng.standard_normal((B, Hq, D)).astype(np.float16)

    def run(chunks):
        oc = oracle_mod.OracleCache(1, B, Hq, H, D, [kb], [vb])
        t = 0
        for n in chunks:
            oc.quantize_append(0, K[:, :, t:t + n], V[:, :, t:t + n])
            t += n
        assert t == T
        return oc.export(0), oc.decode_attention(0, q)[1]

    bulk, o_bulk = run([T])
    for chunks in ([1] * T, [31, 33, 1, 64, 38], [100, 67], [63, 1, 1, 102]):
        d, o = run(chunks)
        _dumps_equal(bulk, d)
        assert np.array_equal(o, o_bulk)


def test_layers_are_independent_and_reset_clears(oracle_mod):
    rng = np.random.default_rng(3)
    K = rng.standard_normal((1, 1, 70, 32)).astype(np.float16)
    oc = oracle_mod.OracleCache(2, 1, 1, 1, 32, [8, 2], [2, 8])
    oc.quantize_append(1, K, K)
    assert oc.tokens(0) == (0, 0) and oc.tokens(1) == (32, 38)
    with pytest.raises(ValueError):
        oc.decode_attention(0, np.zeros((1, 1, 32), dtype=np.float16))
    oc.reset(1)
    assert oc.tokens(1) == (0, 0)
