"""kvq_decode_attention_noalloc: the decode call whose split partials live in the library's built-in device array
instead of the caller's workspace.  Through the C ABI, against kvq_decode_attention on the same cache: same kernels
and the same split plan, so the outputs must agree bit for bit (which implies the bars of the parity tests, that the
existing call is held to against the oracle).  Two calls in a row, the second on a smaller input, so that records the
first call left in the shared array cannot leak into the second; then the limit and the error it returns."""
import ctypes
from ctypes import c_void_p

import numpy as np
import pytest
import torch

import kvq_workloads as W

pytestmark = pytest.mark.gpu

MAX_ABS = 2e-3
REL_L2 = 1e-3


@pytest.fixture(scope="module")
def kvq_mod():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2502_04420_amd as pkg

    pkg.load_library()
    return pkg


def _filled(kvq_mod, w, max_tokens):
    g = kvq_mod.KVQ(1, w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, max_tokens, w.kbits, w.vbits)
    K, V = W.kv_tokens(w, 0, 0, w.context, device="cuda:0")
    g.quantize_append(0, K, V)
    return g


def _both(g, q):
    """(existing entry point's output, new entry point's output), both through the raw C ABI."""
    lib, h = g._lib, g._h
    ref = torch.empty_like(q)
    out = torch.full_like(q, float("nan"))
    assert lib.kvq_decode_attention(h, 0, c_void_p(q.data_ptr()), c_void_p(ref.data_ptr())) == 0
    assert lib.kvq_decode_attention_noalloc(h, 0, c_void_p(q.data_ptr()), c_void_p(out.data_ptr())) == 0
    torch.cuda.synchronize()
    return ref, out


def _assert_same(ref, out, where):
    r, o = ref.float().cpu().numpy().astype(np.float64), out.float().cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(o)), where
    assert np.abs(o - r).max() <= MAX_ABS and np.linalg.norm(o - r) / np.linalg.norm(r) <= REL_L2, where
    assert torch.equal(ref, out), where + ": same kernels and split plan, yet the bits differ"


def test_noalloc_matches_decode_attention_twice_second_call_smaller(kvq_mod, oracle_mod):
    # first call: 8 sequences x 4 kv heads, g_q = 7, 8200 tokens: 64 splits per cache, 14336 of the 16384 records
    w1 = W.Workload("na-large", 1, 8, 28, 4, 128, 8200, [4], [2], seed=2100, outlier_channels=3, key_bias_std=20.0)
    g1 = _filled(kvq_mod, w1, 8264)
    q1 = W.query(w1, 0, device="cuda:0")
    ref1, out1 = _both(g1, q1)
    _assert_same(ref1, out1, "large call")
    # second call, smaller in every respect (batch, heads, context, splits): it shares the array with the first
    w2 = W.Workload("na-small", 1, 2, 8, 2, 128, 32 * 9 + 17, [8], [4], seed=2101, outlier_channels=3)
    g2 = _filled(kvq_mod, w2, 512)
    q2 = W.query(w2, 0, device="cuda:0")
    ref2, out2 = _both(g2, q2)
    _assert_same(ref2, out2, "small call after the large one")
    # and against the oracle itself, to the bars of the parity tests
    o = oracle_mod.OracleCache(1, w2.batch, w2.n_q_heads, w2.n_kv_heads, w2.head_dim, w2.kbits, w2.vbits)
    K, V = W.kv_tokens(w2, 0, 0, w2.context)
    o.quantize_append(0, K.numpy(), V.numpy())
    _, o64 = o.decode_attention(0, q2.cpu().numpy())
    got = out2.float().cpu().numpy().astype(np.float64)
    assert np.abs(got - o64).max() <= MAX_ABS and np.linalg.norm(got - o64) / np.linalg.norm(o64) <= REL_L2
    # the first context again after the small call: still the same bits
    ref1b, out1b = _both(g1, q1)
    assert torch.equal(out1b, out1) and torch.equal(ref1b, ref1)
    g1.close()
    g2.close()


def test_noalloc_rejects_what_the_array_cannot_hold(kvq_mod):
    # 160 query rows, 124 packed blocks + window, splits forced to the maximum: the plan arrives at 125 token ranges
    # (one block each, the window on the last), 160 x 125 = 20000 records > 16384
    w = W.Workload("na-limit", 1, 20, 8, 1, 128, 32 * 125 + 5, [4], [4], seed=2102)
    g = _filled(kvq_mod, w, 32 * 132)
    q = W.query(w, 0, device="cuda:0")
    out = torch.zeros_like(q)
    lib, h = g._lib, g._h
    g.set_decode_options(0, 128)
    rc = lib.kvq_decode_attention_noalloc(h, 0, c_void_p(q.data_ptr()), c_void_p(out.data_ptr()))
    assert rc == -6                                                      # KVQ_ESCRATCH
    assert b"16384" in lib.kvq_last_error() and b"20000" in lib.kvq_last_error(), lib.kvq_last_error()
    torch.cuda.synchronize()
    assert not out.any()                                                 # nothing was enqueued
    with pytest.raises(kvq_mod.KVQError):
        g.decode_attention_noalloc(0, q, out)
    g.set_decode_options(0, 64)                                          # 63 token ranges, 10080 records: accepted
    ref, got = _both(g, q)
    _assert_same(ref, got, "after a rejected call")
    g.close()


def test_noalloc_recorded_into_a_graph_and_replayed(kvq_mod):
    """The callers the entry point is for: a decode call recorded into a HIP graph (stream capture forbids
    allocation) and replayed with new queries.  The address of the built-in array is looked up by an eager call
    before the capture.  Every replay is checked against an eager kvq_decode_attention on the same inputs, with eager
    work and synchronisations between the replays."""
    side = torch.cuda.Stream()
    w = W.Workload("na-graph", 1, 4, 16, 4, 128, 32 * 40 + 50, [4], [2], seed=2300, outlier_channels=3)
    with torch.cuda.stream(side):
        g = kvq_mod.KVQ(1, w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, 2048, w.kbits, w.vbits, stream=side)
        K, V = W.kv_tokens(w, 0, 0, w.context, device="cuda:0")
        g.quantize_append(0, K, V)
        lib, h = g._lib, g._h
        q = W.query(w, 0, 0, device="cuda:0").clone()
        out = torch.empty_like(q)
        ref = torch.empty_like(q)
        assert lib.kvq_decode_attention_noalloc(h, 0, c_void_p(q.data_ptr()), c_void_p(out.data_ptr())) == 0     # address lookup, eager
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        rc = lib.kvq_decode_attention_noalloc(h, 0, c_void_p(q.data_ptr()), c_void_p(out.data_ptr()))
    assert rc == 0, lib.kvq_last_error()
    for step in range(1, 4):
        with torch.cuda.stream(side):
            q.copy_(W.query(w, 0, step, device="cuda:0"))
            out.fill_(float("nan"))
            graph.replay()
            assert lib.kvq_decode_attention(h, 0, c_void_p(q.data_ptr()), c_void_p(ref.data_ptr())) == 0
        side.synchronize()
        assert torch.equal(out, ref), "replay %d differs from the eager call" % step
    g.close()
