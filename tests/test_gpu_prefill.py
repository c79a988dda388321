"""GPU parity of the prefill-stage attention (causal attention of the prompt over the dequantized cache) against the
CPU oracle, every element.

Bars: per tensor ||gpu - oracle||_2 / ||oracle||_2 <= 1e-3, and per element |gpu - oracle| <= 2e-3 + 2^-10 |oracle|.
The second term is one fp16 spacing of the value: early prompt positions average over few tokens, so their
outputs reach the magnitude of single values (2..8 here), where a result that is right to well under the absolute
budget can still round to the neighbouring fp16 number.
"""
import numpy as np
import pytest
import torch

import kvq_workloads as W
from test_gpu_parity import _pair, kvq_mod  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu

MAX_ABS = 2e-3
REL_L2 = 1e-3


def assert_prefill_close(gpu_out, ora64, where=""):
    g = gpu_out.float().cpu().numpy().astype(np.float64)
    assert g.shape == ora64.shape, (where, g.shape, ora64.shape)
    assert np.all(np.isfinite(g)), where
    err = np.abs(g - ora64)
    bound = MAX_ABS + 2.0 ** -10 * np.abs(ora64)
    worst = (err - bound).max()
    assert worst <= 0, (where, "elementwise", float(err.max()), np.unravel_index(np.argmax(err - bound), err.shape))
    rel = np.linalg.norm(g - ora64) / max(np.linalg.norm(ora64), 1e-30)
    assert rel <= REL_L2, (where, "rel l2", rel)
    return rel


def _run(kvq_mod, oracle_mod, w, n_q, meta=None, keys=None, max_tokens=None, low_parts=None):
    kw = {}
    if meta is not None:
        kw["meta_dtype"] = meta
    if keys is not None:
        kw["key_mode"] = keys
    g = kvq_mod.KVQ(1, w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, max_tokens or (w.context + 64), w.kbits, w.vbits, **kw)
    o = oracle_mod.OracleCache(1, w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.kbits, w.vbits,
                               scale_fp16=meta == kvq_mod.META_FP16 if meta is not None else False,
                               key_per_token=keys == kvq_mod.KEYS_PER_TOKEN if keys is not None else False)
    K, V = W.kv_tokens(w, 0, 0, w.context)
    g.quantize_append(0, K.cuda(), V.cuda())
    o.quantize_append(0, K.numpy(), V.numpy())
    if low_parts is not None:
        g.set_prefill_options(low_parts)
    q = W.prefill_queries(w, 0, n_q)
    out = g.prefill_attention(0, q.cuda())
    o16, o64 = o.prefill_attention(0, q.numpy())
    return out, o64, g, o, q


PAIRS = [(8, 8), (8, 4), (4, 4), (4, 2), (2, 2), (2, 8), (16, 16), (16, 4), (2, 16)]


@pytest.mark.parametrize("kb,vb", PAIRS)
def test_all_precision_pairs_full_prompt(kvq_mod, oracle_mod, kb, vb):
    """10 blocks plus a ragged window (51 tokens): three query tiles of 128, the last one partial; g_q = 4."""
    w = W.Workload("prefill", 1, 2, 8, 2, 128, 32 * 11 + 19, [kb], [vb], seed=300 + kb * 17 + vb, outlier_channels=3)
    out, o64, g, o, q = _run(kvq_mod, oracle_mod, w, w.context)
    assert g.layer_tokens(0) == (320, 51)
    assert_prefill_close(out, o64, "K%dV%d" % (kb, vb))
    g.close()


# keys: (channels multiplied, by how much, standard deviation of a per-channel offset)
KEY_SHAPES = {"three large channels": (3, 12.0, 0.0), "no large channel": (0, 1.0, 0.0), "all channels 1.4x": (128, 1.4, 0.0),
              "all channels 12x": (128, 12.0, 0.0), "offset on every channel": (0, 1.0, 20.0),
              "large channels and offsets": (4, 12.0, 6.0)}


@pytest.mark.parametrize("shape", list(KEY_SHAPES))
@pytest.mark.parametrize("kb", [8, 4, 2])
def test_low_parts_kept_for_all_channels_or_for_the_selected(kvq_mod, oracle_mod, shape, kb):
    """The dequantized keys enter as two fp16 numbers; per cache the kernel keeps the second one for all channels or
    for the 32 where it matters most (decided on the GPU from the stored metadata and the queries).  Whatever it decides
    for keys of these kinds, the result meets the same bars as with the choice switched off (low_parts = 1)."""
    n, mult, offs = KEY_SHAPES[shape]
    w = W.Workload("lowparts", 1, 2, 8, 2, 128, 32 * 9 + 21, [kb], [4], seed=900 + kb, outlier_channels=n, outlier_scale=mult,
                   key_bias_std=offs)
    for low_parts in (0, 1):
        out, o64, g, o, q = _run(kvq_mod, oracle_mod, w, w.context, low_parts=low_parts)
        assert_prefill_close(out, o64, "%s K%d low_parts %d" % (shape, kb, low_parts))
        g.close()


def test_prefill_options_reject_unknown_values(kvq_mod):
    g = kvq_mod.KVQ(1, 1, 4, 1, 128, 128, [4], [2])
    for bad in (-1, 2):
        with pytest.raises(kvq_mod.KVQError):
            g.set_prefill_options(bad)
    g.set_prefill_options(1)
    g.set_prefill_options(0)
    g.close()


@pytest.mark.parametrize("T,n_q", [(1, 1), (5, 5), (31, 31), (32, 32), (33, 7), (63, 63), (64, 64), (65, 65), (96, 1), (127, 100),
                                   (200, 129), (257, 256), (300, 17)])
def test_ragged_lengths_and_query_counts(kvq_mod, oracle_mod, T, n_q):
    """Lengths around the window and block boundaries, with fewer queries than tokens (the last n_q positions)."""
    w = W.Workload("ragged", 1, 1, 4, 1, 128, T, [4], [2], seed=400 + T, outlier_channels=2)
    out, o64, g, o, q = _run(kvq_mod, oracle_mod, w, n_q)
    assert_prefill_close(out, o64, "T%d nq%d" % (T, n_q))
    g.close()


@pytest.mark.parametrize("hq,hkv", [(1, 1), (7, 1), (8, 1), (6, 3), (28, 4)])
def test_head_ratios(kvq_mod, oracle_mod, hq, hkv):
    w = W.Workload("heads", 1, 2, hq, hkv, 128, 32 * 5 + 9, [4], [4], seed=500 + hq, outlier_channels=2)
    out, o64, g, o, q = _run(kvq_mod, oracle_mod, w, w.context)
    assert_prefill_close(out, o64, "Hq%d Hkv%d" % (hq, hkv))
    g.close()


@pytest.mark.parametrize("kb,vb", [(8, 4), (4, 2), (2, 2)])
def test_fp16_scales_and_per_token_keys(kvq_mod, oracle_mod, kb, vb):
    w = W.Workload("modes", 1, 1, 8, 2, 128, 32 * 7 + 40, [kb], [vb], seed=600 + kb + vb, outlier_channels=3)
    for meta, keys in ((kvq_mod.META_FP16, kvq_mod.KEYS_PER_CHANNEL), (kvq_mod.META_FP32, kvq_mod.KEYS_PER_TOKEN),
                       (kvq_mod.META_FP16, kvq_mod.KEYS_PER_TOKEN)):
        out, o64, g, o, q = _run(kvq_mod, oracle_mod, w, w.context, meta=meta, keys=keys)
        assert_prefill_close(out, o64, "K%dV%d meta %d keys %d" % (kb, vb, meta, keys))
        g.close()


def test_last_row_is_the_decode_step_and_cache_is_untouched(kvq_mod, oracle_mod):
    """With every token visible the last query is a decode query: both kernels agree with the oracle; the call
    leaves the cache as it was (export before == export after); chunked appends give the same answer."""
    from test_gpu_parity import assert_export_equal, assert_outputs_close

    w = W.Workload("last", 1, 2, 8, 2, 128, 32 * 6 + 33, [4], [2], seed=77, outlier_channels=3)
    g, o = _pair(kvq_mod, oracle_mod, w, 512)
    K, V = W.kv_tokens(w, 0, 0, w.context)
    for t0, t1 in ((0, 100), (100, 101), (101, w.context)):
        g.quantize_append(0, K[:, :, t0:t1].contiguous().cuda(), V[:, :, t0:t1].contiguous().cuda())
    o.quantize_append(0, K.numpy(), V.numpy())
    q = W.prefill_queries(w, 0, 40)
    before = o.export(0)
    out = g.prefill_attention(0, q.cuda())
    assert_export_equal(g.debug_export(0), before, "after prefill attention")
    o16, o64 = o.prefill_attention(0, q.numpy())
    assert_prefill_close(out, o64, "chunked")
    dec = g.decode_attention(0, q[:, :, -1, :].contiguous().cuda())
    d16, d64 = o.decode_attention(0, q[:, :, -1, :].contiguous().numpy())
    assert_outputs_close(dec, d16, d64, "decode on the last query")
    assert np.array_equal(d64, o64[:, :, -1, :])
    g.close()


def test_argument_errors(kvq_mod):
    g = kvq_mod.KVQ(1, 1, 4, 1, 128, 256, [4], [4])
    q = torch.zeros(1, 4, 8, 128, dtype=torch.float16, device="cuda:0")
    with pytest.raises(kvq_mod.KVQError):
        g.prefill_attention(0, q)                                   # empty layer
    z = torch.zeros(1, 1, 5, 128, dtype=torch.float16, device="cuda:0")
    g.quantize_append(0, z, z)
    with pytest.raises(kvq_mod.KVQError):
        g.prefill_attention(0, q)                                   # 8 queries, 5 tokens
    with pytest.raises(kvq_mod.KVQError):
        g.prefill_attention(1, q[:, :, :5].contiguous())            # bad layer
    out = g.prefill_attention(0, q[:, :, :5].contiguous())
    assert torch.all(out == 0)
    g.close()


def test_llama_shape_full_prompt_sampled_rows(kvq_mod, oracle_mod):
    """The benchmark's prefill-attention shape (Llama-3.1-8B heads, batch 16, 8192-token prompt, every position a
    query, K4V2 layer of the 3.25-bit mix), in the launch configuration bench.py times.  The oracle recomputes sampled
    (batch, kv head) pairs at sampled positions one by one: the first tokens, block and query-tile boundaries, the
    middle of the prompt, the window and the last token."""
    w = W.config3(16, 8192)
    layer = 16
    kb, vb = w.kbits[layer], w.vbits[layer]
    assert (kb, vb) == (4, 2)
    T, gq = w.context, w.n_q_heads // w.n_kv_heads
    g = kvq_mod.KVQ(1, w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, T + 64, [kb], [vb])
    for t0 in range(0, T, 2048):
        K, V = W.kv_tokens(w, layer, t0, t0 + 2048, device="cuda:0")
        g.quantize_append(0, K, V)
    del K, V
    q = torch.empty(w.batch, w.n_q_heads, T, w.head_dim, dtype=torch.float16, device="cuda:0")
    for h0 in range(0, w.n_q_heads, gq):
        q[:, h0:h0 + gq] = W.prefill_queries(w, layer, T, device="cuda:0", heads=(h0, gq))
    out = g.prefill_attention(0, q)
    torch.cuda.synchronize()
    pos = [0, 1, 2, 15, 16, 31, 32, 33, 127, 128, 129, 255, 256, 1000, 2047, 2048, 4095, 4096, 5555, 8100, 8159, 8160, 8190, 8191]
    worst = 0.0
    for bh in (0, 45, 127):                         # (b, h) = (0, 0), (5, 5), (15, 7)
        b, h = divmod(bh, w.n_kv_heads)
        rows = torch.tensor([bh])
        Kc, Vc = W.kv_tokens(w, layer, 0, T, bh=rows)
        o = oracle_mod.OracleCache(1, 1, gq, 1, w.head_dim, [kb], [vb])
        o.quantize_append(0, Kc.numpy()[None], Vc.numpy()[None])
        assert o.tokens(0) == g.layer_tokens(0)
        qs = q[b, h * gq:(h + 1) * gq][:, pos].cpu().numpy()[None]                 # [1, gq, n, D]
        o16, o64 = o.prefill_attention_at(0, np.ascontiguousarray(qs), pos)
        got = out[b, h * gq:(h + 1) * gq][:, pos][None]
        worst = max(worst, assert_prefill_close(got, o64, "bh %d" % bh))
        o.close()
    g.close()
    assert worst > 0


def test_qwen_shape_prompt_with_key_offsets_sampled_rows(kvq_mod, oracle_mod):
    """The Qwen2.5-7B shape (28 query / 4 kv heads, keys with a large offset on every channel), batch 4, a prompt of
    8192 + 19 tokens (a 51-token fp16 window behind 255 packed units), K4V2.  The kernel takes the offsets off the
    packed keys and lowers the window's scores by the matching amount; sampled (batch, kv head) pairs at sampled
    positions, the window's among them, against the oracle, with the choice of low-part channels on and off."""
    w = W.named("qwen7b", "K4V2", 4, 8192 + 19)
    layer, (kb, vb) = 1, (4, 2)
    T, gq = w.context, w.n_q_heads // w.n_kv_heads
    g = kvq_mod.KVQ(1, w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, T + 64, [kb], [vb])
    for t0 in range(0, T, 2048):
        K, V = W.kv_tokens(w, layer, t0, min(T, t0 + 2048), device="cuda:0")
        g.quantize_append(0, K, V)
    del K, V
    assert g.layer_tokens(0) == (8160, 51)
    q = torch.empty(w.batch, w.n_q_heads, T, w.head_dim, dtype=torch.float16, device="cuda:0")
    for h0 in range(0, w.n_q_heads, gq):
        q[:, h0:h0 + gq] = W.prefill_queries(w, layer, T, device="cuda:0", heads=(h0, gq))
    pos = [0, 1, 31, 32, 33, 255, 256, 1000, 4095, 4096, 8159, 8160, 8161, 8191, 8192, 8200, T - 2, T - 1]
    for low_parts in (0, 1):
        g.set_prefill_options(low_parts)
        out = g.prefill_attention(0, q)
        torch.cuda.synchronize()
        for bh in (0, 6, 15):                       # (b, h) = (0, 0), (1, 2), (3, 3)
            b, h = divmod(bh, w.n_kv_heads)
            Kc, Vc = W.kv_tokens(w, layer, 0, T, bh=torch.tensor([bh]))
            o = oracle_mod.OracleCache(1, 1, gq, 1, w.head_dim, [kb], [vb])
            o.quantize_append(0, Kc.numpy()[None], Vc.numpy()[None])
            assert o.tokens(0) == g.layer_tokens(0)
            qs = q[b, h * gq:(h + 1) * gq][:, pos].cpu().numpy()[None]
            o16, o64 = o.prefill_attention_at(0, np.ascontiguousarray(qs), pos)
            assert_prefill_close(out[b, h * gq:(h + 1) * gq][:, pos][None], o64, "bh %d low_parts %d" % (bh, low_parts))
            o.close()
    g.close()


def test_llama_heads_32k_prompt_sampled_rows(kvq_mod, oracle_mod):
    """A 32768-token prompt (Llama-3.1-8B heads, batch 3 = 24 caches, i.e. two passes; K8V4 layer): 1023 packed units per
    cache and 128 query tiles per head.  Sampled (batch, kv head) pairs at sampled positions against the oracle."""
    w = W.Workload("prefill32k", 1, 3, 32, 8, 128, 32768, [8], [4], seed=911, outlier_channels=3)
    T, gq = w.context, w.n_q_heads // w.n_kv_heads
    g = kvq_mod.KVQ(1, w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, T + 64, w.kbits, w.vbits)
    for t0 in range(0, T, 8192):
        K, V = W.kv_tokens(w, 0, t0, t0 + 8192, device="cuda:0")
        g.quantize_append(0, K, V)
    del K, V
    q = torch.empty(w.batch, w.n_q_heads, T, w.head_dim, dtype=torch.float16, device="cuda:0")
    for h0 in range(0, w.n_q_heads, gq):
        q[:, h0:h0 + gq] = W.prefill_queries(w, 0, T, device="cuda:0", heads=(h0, gq))
    out = g.prefill_attention(0, q)
    torch.cuda.synchronize()
    pos = [0, 31, 32, 255, 256, 8191, 8192, 16383, 16384, 20000, 32511, 32512, 32735, 32736, 32766, 32767]
    for bh in (0, 13, 23):                          # first pass, first pass, second pass
        b, h = divmod(bh, w.n_kv_heads)
        Kc, Vc = W.kv_tokens(w, 0, 0, T, bh=torch.tensor([bh]))
        o = oracle_mod.OracleCache(1, 1, gq, 1, w.head_dim, w.kbits, w.vbits)
        o.quantize_append(0, Kc.numpy()[None], Vc.numpy()[None])
        assert o.tokens(0) == g.layer_tokens(0)
        qs = q[b, h * gq:(h + 1) * gq][:, pos].cpu().numpy()[None]
        o16, o64 = o.prefill_attention_at(0, np.ascontiguousarray(qs), pos)
        assert_prefill_close(out[b, h * gq:(h + 1) * gq][:, pos][None], o64, "bh %d" % bh)
        o.close()
    g.close()


@pytest.mark.parametrize("batch,hkv,room", [(5, 4, 1), (3, 8, 1), (17, 1, 1), (7, 8, 3), (5, 8, 4)])
def test_more_caches_than_one_pass_holds(kvq_mod, oracle_mod, batch, hkv, room):
    """The scratch area holds 16 caches of max_tokens each; a pass takes as many caches as fit (a multiple of 8 when
    not all).  Prompt of 293 tokens (8 packed units): with max_tokens = 293 (9 units of room per cache) 18 caches fit:
    20 = 16 + 4 and 24 = 16 + 8 caches take two passes, 17 take one whose count is no multiple of the 8 XCDs; with
    three times the room 54 fit: 56 = 48 + 8; with four times 72 fit: 40 in one pass.  Queries are a proper tail."""
    w = W.Workload("chunks", 1, batch, 2 * hkv, hkv, 128, 32 * 9 + 5, [4], [2], seed=700 + batch, outlier_channels=2)
    out, o64, g, o, q = _run(kvq_mod, oracle_mod, w, 270, max_tokens=room * w.context)
    assert_prefill_close(out, o64, "B%d Hkv%d" % (batch, hkv))
    g.close()
