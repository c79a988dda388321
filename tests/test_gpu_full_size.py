"""GPU parity at the benchmark's full shapes, in the launch configuration bench.py times (automatic splits,
default kernel): the oracle recomputes sampled (batch, kv head) caches one by one -- every code, scale and
zero-point of those caches bit for bit, and the attention output of all their query heads within the bars.
Inputs are generated on the GPU by the seeded workload generator; the oracle gets the same rows on the CPU."""
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


def _check_layer(kvq_mod, oracle_mod, w, layer, extra_tokens, samples, meta16=False, fused=False):
    """fused: the extra tokens arrive through kvq_append_decode_attention, the one-call decode step bench.py times (its
    last call's output is the one compared); else through kvq_quantize_append, followed by one kvq_decode_attention."""
    kb, vb = w.kbits[layer], w.vbits[layer]
    g = kvq_mod.KVQ(1, w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.context + 64, [kb], [vb],
                    meta_dtype=kvq_mod.META_FP16 if meta16 else kvq_mod.META_FP32)
    K, V = W.kv_tokens(w, layer, 0, w.context, device="cuda:0")
    g.quantize_append(0, K, V)
    del K, V
    # a few single-token appends as in the decode loop (they land in the fp16 window, possibly after a flush)
    Kn, Vn = W.kv_tokens(w, layer, 0, extra_tokens, device="cuda:0", stream=1, total=extra_tokens)
    q = W.query(w, layer, 0, device="cuda:0")
    if fused:
        assert extra_tokens >= 1
        scratch_q = W.query(w, layer, 1, device="cuda:0")
        for t in range(extra_tokens):
            out_t = g.append_decode_attention(0, Kn[:, :, t:t + 1].contiguous(), Vn[:, :, t:t + 1].contiguous(),
                                              q if t == extra_tokens - 1 else scratch_q)
        out = out_t.float().cpu().numpy().astype(np.float64)
    else:
        for t in range(extra_tokens):
            g.quantize_append(0, Kn[:, :, t:t + 1].contiguous(), Vn[:, :, t:t + 1].contiguous())
        out = g.decode_attention(0, q).float().cpu().numpy().astype(np.float64)
    dump = g.debug_export(0)
    gq = w.n_q_heads // w.n_kv_heads
    worst = 0.0
    for bh in samples:
        b, h = divmod(bh, w.n_kv_heads)
        rows = torch.tensor([bh])
        Kc, Vc = W.kv_tokens(w, layer, 0, w.context, bh=rows)
        Kd, Vd = W.kv_tokens(w, layer, 0, extra_tokens, stream=1, bh=rows, total=extra_tokens)
        o = oracle_mod.OracleCache(1, 1, gq, 1, w.head_dim, [kb], [vb], scale_fp16=meta16)
        o.quantize_append(0, Kc.numpy()[None], Vc.numpy()[None])
        for t in range(extra_tokens):
            o.quantize_append(0, np.ascontiguousarray(Kd.numpy()[None, :, t:t + 1]), np.ascontiguousarray(Vd.numpy()[None, :, t:t + 1]))
        od = o.export(0)
        assert od["n_packed"] == dump["n_packed"] and od["n_residual"] == dump["n_residual"]
        for key in ("k_codes", "k_scale", "k_zero", "v_codes", "v_scale", "v_zero", "k_res", "v_res"):
            if key not in od:
                continue
            gt = dump[key][b, h].cpu()
            gt = gt.view(torch.uint16).numpy() if gt.dtype == torch.float16 else gt.numpy()
            assert np.array_equal(gt.view(np.uint8), od[key][0, 0].view(np.uint8)), (w.name, layer, bh, key)
        qs = q[b, h * gq:(h + 1) * gq].cpu().numpy()[None]
        o16, o64 = o.decode_attention(0, qs)
        got = out[b, h * gq:(h + 1) * gq]
        err = np.abs(got - o64[0]).max()
        rel = np.linalg.norm(got - o64[0]) / np.linalg.norm(o64[0])
        assert err <= MAX_ABS and rel <= REL_L2, (w.name, layer, bh, err, rel)
        worst = max(worst, rel)
        o.close()
    g.close()
    return worst


def test_llama_shape_batch16_context8192_mix_and_kv8(kvq_mod, oracle_mod):
    """The benchmark's Llama-3.1-8B shape (3.25-bit mix: K4V4 and K4V2 layers) and uniform K8V8 at the same shape."""
    w = W.config3(16, 8192)
    samples = [0, 37, 77, 127]                      # (b, h) = (0,0), (4,5), (9,5), (15,7)
    _check_layer(kvq_mod, oracle_mod, w, 0, 3, samples[:2])            # K4V4 layer
    _check_layer(kvq_mod, oracle_mod, w, 16, 40, samples)              # K4V2 layer; 40 appends force a window flush
    w8 = W.named("llama8b", "K8V8", 16, 8192)
    _check_layer(kvq_mod, oracle_mod, w8, 5, 1, samples[1:3])
    _check_layer(kvq_mod, oracle_mod, w, 16, 2, samples[2:], meta16=True)   # the narrow-metadata variant at full size


def test_llama_shape_fused_decode_steps_across_a_flush(kvq_mod, oracle_mod):
    """The call bench.py times, in its launch configuration: kvq_append_decode_attention at batch 16, context 8192
    (automatic splits: the new token is read from the caller's tensor by the last split of every cache), 40 steps, so
    that a window flush of 32 tokens falls inside; cache state bit for bit and the last step's output within the bars."""
    w = W.config3(16, 8192)
    _check_layer(kvq_mod, oracle_mod, w, 16, 40, [0, 61, 127], fused=True)     # K4V2 layer
    _check_layer(kvq_mod, oracle_mod, w, 30, 33, [5, 100], fused=True)         # K4V4 layer
    w8 = W.named("llama8b", "K8V8", 16, 8192)
    _check_layer(kvq_mod, oracle_mod, w8, 7, 34, [64], fused=True)
    wq = W.config4(8, 32768)
    _check_layer(kvq_mod, oracle_mod, wq, 1, 35, [9], fused=True)              # Qwen shape (g_q = 7), K4V2 layer


def test_qwen_shape_batch8_context32768_biased_keys(kvq_mod, oracle_mod):
    """The Qwen2.5-7B shape: g_q = 7, keys with a large per-channel offset, 32K context (K8V2 and K4V2 layers)."""
    w = W.config4(8, 32768)
    _check_layer(kvq_mod, oracle_mod, w, 0, 1, [3, 30])                # K8V2 layer
    _check_layer(kvq_mod, oracle_mod, w, 1, 33, [17])                  # K4V2 layer


def test_llama_shape_batch16_context4096_uniform_kv8(kvq_mod, oracle_mod):
    """Uniform K8V8 at batch 16, context 4096 (the benchmark's second configuration), one decode step."""
    w = W.named("llama8b", "K8V8", 16, 4096)
    _check_layer(kvq_mod, oracle_mod, w, 0, 1, [5, 90])
    _check_layer(kvq_mod, oracle_mod, w, 31, 1, [127])


def test_llama_shape_batch32_context32768(kvq_mod, oracle_mod):
    """The 32K point that bench.py also times (batch 32): a K8V8 layer, which the planner serves with half as many
    groups as the narrow pairs, and a K4V2 layer."""
    w8 = W.named("llama8b", "K8V8", 32, 32768)
    _check_layer(kvq_mod, oracle_mod, w8, 3, 1, [200])
    w = W.config3(32, 32768)
    _check_layer(kvq_mod, oracle_mod, w, 16, 2, [11])


def test_llama_shape_batch64_context32768_one_bulk_append(kvq_mod, oracle_mod):
    """The largest point of the sweep, the whole prompt in one append: 2^31 elements per input tensor, so every index
    that is not computed in 64 bits would show."""
    w = W.config3(64, 32768)
    _check_layer(kvq_mod, oracle_mod, w, 16, 2, [511, 256])            # K4V2 layer: last and a middle (batch, kv head)
    w8 = W.named("llama8b", "K8V8", 64, 32768)
    _check_layer(kvq_mod, oracle_mod, w8, 3, 1, [300])
    _check_layer(kvq_mod, oracle_mod, w, 1, 2, [129], fused=True)      # K4V4 layer of the mix at the largest sweep point
