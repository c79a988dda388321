"""CPU-only checks of the product's host side: the C ABI loads and exports what include/kvq.h declares,
argument validation returns the documented codes without touching a GPU, and the schedule helpers."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2502_04420_amd import binding

    if not os.path.exists(binding.library_path()):
        from paper_2502_04420_amd.build import build

        build(verbose=False)
    return binding.load_library()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "kvq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kvq_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(lib):
    names = _declared_functions()
    assert {"kvq_configure", "kvq_quantize_append", "kvq_decode_attention", "kvq_workspace_bytes"} <= set(names)
    for name in names:
        assert getattr(lib, name) is not None, name
    from paper_2502_04420_amd import binding

    assert sorted(binding.EXPORTED) == names


def _cfg(**over):
    from paper_2502_04420_amd import binding

    kw = dict(n_layers=2, batch=2, n_q_heads=8, n_kv_heads=2, head_dim=128, max_tokens=256, kbits=[8, 4], vbits=[4, 2])
    kw.update(over)
    return binding.make_config(**kw)


def test_workspace_bytes_and_config_validation(lib):
    cfg, keep = _cfg()
    need = lib.kvq_workspace_bytes(ctypes.byref(cfg))
    assert need > 0 and need % 256 == 0
    # codes + metadata of 8 blocks per (b, h) for both layers must fit
    assert need >= 4 * 8 * ((4096 + 2048 + 2 * 768) + (2048 + 1024 + 2 * 768))
    c16, k16 = _cfg(meta_dtype=1)          # fp16 scales: 256 bytes less per block and tensor
    need16 = lib.kvq_workspace_bytes(ctypes.byref(c16))
    assert 0 < need16 < need and need - need16 >= 4 * 8 * 4 * 256
    for bad in (dict(head_dim=64), dict(group=16), dict(n_q_heads=7), dict(kbits=[8, 3]), dict(vbits=[1, 2]),
                dict(max_tokens=0), dict(batch=0), dict(residual=-1), dict(meta_dtype=2), dict(key_mode=2), dict(batch=32768)):
        c, k = _cfg(**bad)
        assert lib.kvq_workspace_bytes(ctypes.byref(c)) == 0, bad
        h = ctypes.c_void_p()
        assert lib.kvq_configure(ctypes.byref(h), ctypes.byref(c), ctypes.c_void_p(256), 1 << 40, None) == -1, bad
    assert lib.kvq_workspace_bytes(None) == 0


def test_configure_and_call_errors_without_gpu(lib):
    cfg, keep = _cfg()
    need = lib.kvq_workspace_bytes(ctypes.byref(cfg))
    h = ctypes.c_void_p()
    assert lib.kvq_configure(ctypes.byref(h), ctypes.byref(cfg), None, need, None) == -4          # no workspace
    assert lib.kvq_configure(ctypes.byref(h), ctypes.byref(cfg), ctypes.c_void_p(256 + 8), need, None) == -4   # misaligned
    assert lib.kvq_configure(ctypes.byref(h), ctypes.byref(cfg), ctypes.c_void_p(256), need - 1, None) == -4   # too small
    assert lib.kvq_configure(None, ctypes.byref(cfg), ctypes.c_void_p(256), need, None) == -1
    # a fake (never dereferenced) workspace pointer is enough for the host-side checks below
    assert lib.kvq_configure(ctypes.byref(h), ctypes.byref(cfg), ctypes.c_void_p(256), need, None) == 0
    try:
        fake = ctypes.c_void_p(4096)
        assert lib.kvq_decode_attention(h, 0, fake, fake) == -3          # no token yet
        assert lib.kvq_decode_attention(h, 2, fake, fake) == -1          # bad layer
        assert lib.kvq_decode_attention(h, 0, None, fake) == -1
        assert lib.kvq_quantize_append(h, -1, fake, fake, 1) == -1
        assert lib.kvq_quantize_append(h, 0, fake, fake, 0) == -1
        assert lib.kvq_quantize_append(h, 0, fake, None, 1) == -1
        assert lib.kvq_quantize_append(h, 0, fake, fake, 257) == -2      # beyond max_tokens
        assert lib.kvq_append_decode_attention(h, 0, fake, fake, None, fake) == -1
        assert lib.kvq_append_decode_attention(h, 7, fake, fake, fake, fake) == -1
        a, b = ctypes.c_int32(-1), ctypes.c_int32(-1)
        assert lib.kvq_layer_tokens(h, 1, ctypes.byref(a), ctypes.byref(b)) == 0 and (a.value, b.value) == (0, 0)
        assert lib.kvq_layer_tokens(h, 5, ctypes.byref(a), ctypes.byref(b)) == -1
        assert lib.kvq_reset(h, -1) == 0 and lib.kvq_reset(h, 2) == -1
        assert lib.kvq_set_decode_options(h, 3, 0) == -1 and lib.kvq_set_decode_options(h, 1, 129) == -1
        assert lib.kvq_set_kernel_events(h, ctypes.c_void_p(8), None) == -1     # exactly one event
        assert lib.kvq_set_kernel_events(h, None, None) == 0
        assert lib.kvq_set_decode_options(h, 2, 8) == 0
        assert lib.kvq_debug_export(h, 0, *([None] * 8)) == 0              # empty layer: nothing to do
    finally:
        lib.kvq_destroy(h)
    for code in (0, -1, -2, -3, -4, -5, -99):
        assert len(lib.kvq_strerror(code)) > 0
    assert lib.kvq_last_error() is not None


def test_library_load_brings_torch_first():
    """The library must bind to the HIP runtime that torch ships (the one that owns torch's streams and allocations):
    loading it in a fresh interpreter, before anything imported torch, has to import torch on the way."""
    import subprocess
    import sys

    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = ("import sys; sys.path.insert(0, %r); import paper_2502_04420_amd as p; "
            "assert 'torch' not in sys.modules; p.load_library(); assert 'torch' in sys.modules" % root)
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr[-2000:]


def test_binding_refuses_cpu_device(lib):
    import paper_2502_04420_amd as pkg

    with pytest.raises(ValueError):
        pkg.KVQ(1, 1, 4, 1, 128, 64, [8], [8], device="cpu")


def test_equivalent_precision_matches_the_papers_printed_values():
    import kvq_workloads as W
    from paper_2502_04420_amd import bytes_per_token, equivalent_precision, parse_pairs

    gold = {}
    with open(os.path.join(ROOT, "tests", "golden", "equivalent_precision.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                name, val = [p.strip() for p in line.split("|")]
                gold[name] = float(val)
    for name, printed in gold.items():
        kb, vb = getattr(W, name)()
        assert round(equivalent_precision(kb, vb), 2) in (printed, round(printed + 0.01, 2)), name   # 4.906 prints as 4.90 / 4.91
    assert equivalent_precision(*W.llama_mix_325()) == 3.25
    assert equivalent_precision(*W.qwen_mix_40()) == 4.0
    assert equivalent_precision([4], [4]) == 4.0 and 16 / equivalent_precision([4], [2]) == pytest.approx(5.33, abs=0.01)
    # bytes per token per kv head (head_dim 128, group 32): as stored (fp32 scales, fp16 zero-points), all fp32
    pairs = ((8, 8), (8, 4), (8, 2), (4, 4), (4, 2), (2, 2), (16, 16))
    assert [bytes_per_token(k, v) for k, v in pairs] == [304, 240, 208, 176, 144, 112, 512]
    assert [bytes_per_token(k, v, zero_bytes=4) for k, v in pairs] == [320, 256, 224, 192, 160, 128, 512]
    assert parse_pairs("K8V4, KV4,K4V2") == ([8, 4, 4], [4, 4, 2])
    with pytest.raises(ValueError):
        parse_pairs("K3V4")


def _split_ranges(n_blocks, n_res, splits, units, rem):
    """The units [u0, u1) of every split as the kernels read the plan: blocks first, the window's chunks on the last."""
    out = []
    for s in range(splits):
        big = splits - rem                                   # the last `rem` splits take one unit more
        u0 = min(s * units + max(0, s - big), n_blocks)
        u1 = min(u0 + units + (1 if s >= big else 0), n_blocks)
        if s == splits - 1:
            u1 = n_blocks + (n_res + 31) // 32
        out.append((u0, u1))
    return out


def test_split_plan_covers_every_unit_once_and_leaves_no_split_empty(lib):
    """kvq_debug_split_plan over many shapes, lengths, widths, kernel variants and forced split counts: the splits'
    ranges tile the blocks in order, the window sits on the last split, no split is empty (an empty split would hand
    the merge a record without a maximum), blocks per split differ by at most one in front of the window's units, and
    a forced split count is never exceeded."""
    i32 = ctypes.c_int32
    seen_uneven = False
    for batch, hq, hkv in ((1, 1, 1), (2, 8, 2), (16, 32, 8), (8, 28, 4), (64, 32, 8)):
        for kb, vb in ((2, 2), (4, 2), (8, 8), (16, 4), (16, 16)):
            max_tokens = 40000
            cfg, keep = _cfg(n_layers=1, batch=batch, n_q_heads=hq, n_kv_heads=hkv, max_tokens=max_tokens, kbits=[kb], vbits=[vb])
            for T in (1, 31, 32, 33, 63, 64, 65, 95, 96, 97, 127, 128, 160, 200, 1000, 4005, 8192, 8200, 8223, 32768, 32800, 39999):
                over = T - 32
                n_p = 32 * (over // 32) if over > 0 else 0
                n_blocks, n_res = n_p // 32, T - n_p
                for variant in (1, 2):
                    for forced in (0, 1, 2, 3, 7, 16, 100, 128):
                        s, u, r = i32(), i32(), i32()
                        assert lib.kvq_debug_split_plan(ctypes.byref(cfg), 0, T, variant, forced, ctypes.byref(s), ctypes.byref(u), ctypes.byref(r)) == 0
                        splits, units, rem = s.value, u.value, r.value
                        where = (batch, hkv, kb, vb, T, variant, forced, splits, units, rem)
                        assert 1 <= splits <= 128 and (forced == 0 or splits <= forced), where
                        assert units >= 0 and 0 <= rem < splits, where
                        ranges = _split_ranges(n_blocks, n_res, splits, units, rem)
                        assert ranges[0][0] == 0 and ranges[-1][1] == n_blocks + (n_res + 31) // 32, where
                        for (a0, a1), (b0, b1) in zip(ranges, ranges[1:]):
                            assert a1 == b0, where                       # in order, no gap, no overlap
                        assert all(u1 > u0 for u0, u1 in ranges), where  # nobody is empty
                        # the splits that lie in front of the window's virtual units
                        blocks = [u1 - u0 for k, (u0, u1) in enumerate(ranges[:-1]) if k * units + max(0, k - (splits - rem)) + units + (k >= splits - rem) <= n_blocks]
                        if blocks:
                            assert max(blocks) - min(blocks) <= 1, where
                            seen_uneven |= max(blocks) != min(blocks)
    assert seen_uneven
    s, u, r = i32(), i32(), i32()
    cfg, keep = _cfg()
    for bad in ((5, 10, 2, 0), (0, 0, 2, 0), (0, 257, 2, 0), (0, 10, 3, 0), (0, 10, 2, 129), (-1, 10, 2, 0)):
        assert lib.kvq_debug_split_plan(ctypes.byref(cfg), bad[0], bad[1], bad[2], bad[3], ctypes.byref(s), ctypes.byref(u), ctypes.byref(r)) == -1, bad
    assert lib.kvq_debug_split_plan(ctypes.byref(cfg), 0, 10, 2, 0, None, ctypes.byref(u), ctypes.byref(r)) == -1
