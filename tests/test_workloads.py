"""The synthetic-input module: reproducible, sliceable, and shaped as documented."""
import numpy as np
import torch

import kvq_workloads as W


def test_standard_normal_moments_and_determinism():
    idx = torch.arange(1 << 18, dtype=torch.int64)
    x = W.standard_normal(9, 3, idx)
    assert x.dtype == torch.float32
    assert abs(x.mean().item()) < 0.01 and abs(x.std().item() - 1) < 0.01
    assert 2.8 < (x ** 4).mean().item() < 3.1
    assert torch.equal(x, W.standard_normal(9, 3, idx))
    assert not torch.equal(x, W.standard_normal(9, 4, idx))
    assert not torch.equal(x, W.standard_normal(10, 3, idx))
    # an element depends only on its index
    sub = idx[1000:2000:7]
    assert torch.equal(W.standard_normal(9, 3, sub), x[1000:2000:7])


def test_slices_equal_the_full_tensor():
    w = W.config4(batch=2, context=96)
    K, V = W.kv_tokens(w, 5, 0, 96)
    assert K.shape == (2, 4, 96, 128) and K.dtype == torch.float16
    K2, V2 = W.kv_tokens(w, 5, 32, 64)
    assert torch.equal(K2, K[:, :, 32:64]) and torch.equal(V2, V[:, :, 32:64])
    rows = torch.tensor([1, 6])
    K3, V3 = W.kv_tokens(w, 5, 0, 96, bh=rows)
    assert torch.equal(K3, K.reshape(8, 96, 128)[rows]) and torch.equal(V3, V.reshape(8, 96, 128)[rows])
    Kd, _ = W.kv_tokens(w, 5, 0, 4, stream=1, total=64)
    assert not torch.equal(Kd, K[:, :, :4])


def test_value_structure():
    w = W.config2(batch=1, context=256)
    K, V = W.kv_tokens(w, 7, 0, 256)
    scale, bias = W.key_channel_profile(w, 7)
    assert int((scale == 10).sum()) == 3 * w.n_kv_heads and not bias.any()
    std = K.float().std(dim=2)[0]
    assert torch.all((std > 7)[scale == 10]) and torch.all((std < 1.5)[scale == 1])
    assert abs(V.float().std().item() - 1) < 0.02
    w4 = W.config4(batch=1, context=256)
    K4, _ = W.kv_tokens(w4, 0, 0, 256)
    _, bias4 = W.key_channel_profile(w4, 0)
    assert 14 < bias4.std().item() < 26
    assert torch.allclose(K4.float().mean(dim=2)[0], bias4, atol=0.5)
    q = W.query(w4, 3, step=2)
    assert q.shape == (1, 28, 128) and q.dtype == torch.float16
    assert not torch.equal(q, W.query(w4, 3, step=3))


def test_schedules_cover_every_layer():
    for fn, n in ((W.llama_mix_325, 32), (W.llama_kivi_c325, 32), (W.llama_kivi_c490, 32), (W.qwen_mix_40, 28)):
        kb, vb = fn()
        assert len(kb) == n and len(vb) == n and set(kb) | set(vb) <= {2, 4, 8}
