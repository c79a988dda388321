"""ctypes binding of the C ABI in ``include/kvq.h``: argument marshalling only.

PyTorch appears here for device memory (the workspace and the caller's tensors) and for
the current HIP stream; every step of the path runs in the library's kernels.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, c_char_p, c_int32, c_size_t, c_uint8, c_void_p
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libkvq.so")
_lib = None

EXPORTED = [
    "kvq_workspace_bytes", "kvq_configure", "kvq_quantize_append", "kvq_decode_attention", "kvq_decode_attention_noalloc", "kvq_debug_split_plan", "kvq_append_decode_attention", "kvq_prefill_attention",
    "kvq_layer_tokens", "kvq_reset", "kvq_debug_export", "kvq_set_decode_options", "kvq_set_prefill_options", "kvq_set_kernel_events", "kvq_destroy", "kvq_strerror",
    "kvq_last_error",
]


class KVQError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("kvq status %d: %s" % (status, message))
        self.status = status


class _Config(ctypes.Structure):
    _fields_ = [("n_layers", c_int32), ("batch", c_int32), ("n_q_heads", c_int32), ("n_kv_heads", c_int32),
                ("head_dim", c_int32), ("max_tokens", c_int32), ("group", c_int32), ("residual", c_int32),
                ("kbits", POINTER(c_uint8)), ("vbits", POINTER(c_uint8)), ("meta_dtype", c_int32), ("key_mode", c_int32)]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libkvq.so.  There is no fallback: a missing library is an error."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError("%s is not built; run `python -m paper_2502_04420_amd.build` "
                          "(or __graft_entry__.build())" % _LIB_PATH)
    # torch first: it brings the HIP runtime it was built with, and the library must bind to that same copy (the one
    # that owns torch's streams and allocations), not pull in a second runtime of its own
    import torch  # noqa: F401

    lib = ctypes.CDLL(_LIB_PATH)
    lib.kvq_workspace_bytes.restype = c_size_t
    lib.kvq_workspace_bytes.argtypes = [POINTER(_Config)]
    lib.kvq_configure.restype = c_int32
    lib.kvq_configure.argtypes = [POINTER(c_void_p), POINTER(_Config), c_void_p, c_size_t, c_void_p]
    lib.kvq_quantize_append.restype = c_int32
    lib.kvq_quantize_append.argtypes = [c_void_p, c_int32, c_void_p, c_void_p, c_int32]
    lib.kvq_decode_attention.restype = c_int32
    lib.kvq_decode_attention.argtypes = [c_void_p, c_int32, c_void_p, c_void_p]
    lib.kvq_decode_attention_noalloc.restype = c_int32
    lib.kvq_decode_attention_noalloc.argtypes = [c_void_p, c_int32, c_void_p, c_void_p]
    lib.kvq_append_decode_attention.restype = c_int32
    lib.kvq_append_decode_attention.argtypes = [c_void_p, c_int32, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.kvq_prefill_attention.restype = c_int32
    lib.kvq_prefill_attention.argtypes = [c_void_p, c_int32, c_void_p, c_int32, c_void_p]
    lib.kvq_layer_tokens.restype = c_int32
    lib.kvq_layer_tokens.argtypes = [c_void_p, c_int32, POINTER(c_int32), POINTER(c_int32)]
    lib.kvq_reset.restype = c_int32
    lib.kvq_reset.argtypes = [c_void_p, c_int32]
    lib.kvq_debug_export.restype = c_int32
    lib.kvq_debug_export.argtypes = [c_void_p, c_int32] + [c_void_p] * 8
    lib.kvq_set_decode_options.restype = c_int32
    lib.kvq_set_decode_options.argtypes = [c_void_p, c_int32, c_int32]
    lib.kvq_set_prefill_options.restype = c_int32
    lib.kvq_set_prefill_options.argtypes = [c_void_p, c_int32]
    lib.kvq_set_kernel_events.restype = c_int32
    lib.kvq_set_kernel_events.argtypes = [c_void_p, c_void_p, c_void_p]
    lib.kvq_destroy.restype = None
    lib.kvq_destroy.argtypes = [c_void_p]
    lib.kvq_strerror.restype = c_char_p
    lib.kvq_strerror.argtypes = [c_int32]
    lib.kvq_last_error.restype = c_char_p
    lib.kvq_last_error.argtypes = []
    _lib = lib
    return lib


def _check(status: int):
    if status != 0:
        lib = load_library()
        msg = lib.kvq_strerror(status).decode()
        detail = lib.kvq_last_error().decode()
        raise KVQError(status, msg + (" (%s)" % detail if status in (-5, -6) and detail else ""))


META_FP32, META_FP16 = 0, 1
KEYS_PER_CHANNEL, KEYS_PER_TOKEN = 0, 1


def make_config(n_layers, batch, n_q_heads, n_kv_heads, head_dim, max_tokens, kbits, vbits, group=32, residual=32,
                meta_dtype=META_FP32, key_mode=KEYS_PER_CHANNEL):
    """Returns (_Config, keepalive) -- the byte arrays must outlive the struct."""
    kb = (c_uint8 * len(kbits))(*kbits)
    vb = (c_uint8 * len(vbits))(*vbits)
    cfg = _Config(n_layers, batch, n_q_heads, n_kv_heads, head_dim, max_tokens, group, residual,
                  ctypes.cast(kb, POINTER(c_uint8)), ctypes.cast(vb, POINTER(c_uint8)), meta_dtype, key_mode)
    return cfg, (kb, vb)


def workspace_bytes(**kw) -> int:
    cfg, _keep = make_config(**kw)
    return int(load_library().kvq_workspace_bytes(ctypes.byref(cfg)))


class KVQ:
    """kvq_configure / kvq_quantize_append / kvq_decode_attention on torch device tensors."""

    def __init__(self, n_layers: int, batch: int, n_q_heads: int, n_kv_heads: int, head_dim: int, max_tokens: int,
                 kbits: Sequence[int], vbits: Sequence[int], group: int = 32, residual: int = 32,
                 device="cuda:0", stream=None, meta_dtype: int = META_FP32, key_mode: int = KEYS_PER_CHANNEL):
        import torch

        self._torch = torch
        self._lib = load_library()
        if len(kbits) != n_layers or len(vbits) != n_layers:
            raise ValueError("need one (key bits, value bits) pair per layer")
        self.n_layers, self.batch, self.n_q_heads, self.n_kv_heads = n_layers, batch, n_q_heads, n_kv_heads
        self.head_dim, self.max_tokens, self.group, self.residual = head_dim, max_tokens, group, residual
        self.kbits, self.vbits = list(kbits), list(vbits)
        self.device = torch.device(device)
        cfg, self._keep = make_config(n_layers, batch, n_q_heads, n_kv_heads, head_dim, max_tokens, self.kbits,
                                      self.vbits, group, residual, meta_dtype, key_mode)
        self.meta_dtype, self.key_mode = meta_dtype, key_mode
        need = int(self._lib.kvq_workspace_bytes(ctypes.byref(cfg)))
        if need == 0:
            raise KVQError(-1, "configuration rejected by kvq_workspace_bytes")
        if self.device.type != "cuda":
            raise ValueError("the cache lives in GPU memory; device must be a cuda device")
        with torch.cuda.device(self.device):
            self.workspace = torch.empty(need, dtype=torch.uint8, device=self.device)
            s = torch.cuda.current_stream(self.device) if stream is None else stream
        self.stream = s
        self._h = c_void_p()
        _check(self._lib.kvq_configure(ctypes.byref(self._h), ctypes.byref(cfg), c_void_p(self.workspace.data_ptr()),
                                       need, c_void_p(s.cuda_stream)))

    # -- helpers
    def _dev_ptr(self, t, shape, dtype, name):
        torch = self._torch
        if not isinstance(t, torch.Tensor) or t.device != self.device:
            raise ValueError("%s must be a tensor on %s" % (name, self.device))
        if t.dtype != dtype or tuple(t.shape) != tuple(shape) or not t.is_contiguous():
            raise ValueError("%s must be contiguous %s of shape %s, got %s %s" % (name, dtype, tuple(shape), t.dtype,
                                                                                  tuple(t.shape)))
        return c_void_p(t.data_ptr())

    def close(self):
        if getattr(self, "_h", None):
            self._lib.kvq_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the three calls of the path
    def quantize_append(self, layer: int, K, V):
        """K, V: fp16 [batch, n_kv_heads, n_tokens, head_dim] on the device."""
        torch = self._torch
        n = int(K.shape[2]) if K.dim() == 4 else -1
        shape = (self.batch, self.n_kv_heads, n, self.head_dim)
        kp = self._dev_ptr(K, shape, torch.float16, "K")
        vp = self._dev_ptr(V, shape, torch.float16, "V")
        _check(self._lib.kvq_quantize_append(self._h, layer, kp, vp, n))

    def decode_attention(self, layer: int, q, out=None):
        """q: fp16 [batch, n_q_heads, head_dim]; returns out of the same shape (allocated if not given)."""
        torch = self._torch
        shape = (self.batch, self.n_q_heads, self.head_dim)
        qp = self._dev_ptr(q, shape, torch.float16, "q")
        if out is None:
            out = torch.empty(shape, dtype=torch.float16, device=self.device)
        op = self._dev_ptr(out, shape, torch.float16, "out")
        _check(self._lib.kvq_decode_attention(self._h, layer, qp, op))
        return out

    def decode_attention_noalloc(self, layer: int, q, out):
        """kvq_decode_attention_noalloc: the splits' partial results live in the library's built-in device array.  The
        output tensor is the caller's (nothing is allocated on the way)."""
        torch = self._torch
        shape = (self.batch, self.n_q_heads, self.head_dim)
        qp = self._dev_ptr(q, shape, torch.float16, "q")
        op = self._dev_ptr(out, shape, torch.float16, "out")
        _check(self._lib.kvq_decode_attention_noalloc(self._h, layer, qp, op))
        return out

    def append_decode_attention(self, layer: int, K, V, q, out=None):
        """One decode step: append one token per sequence (K, V: fp16 [batch, n_kv_heads, 1, head_dim]) and attend."""
        torch = self._torch
        kshape = (self.batch, self.n_kv_heads, 1, self.head_dim)
        kp = self._dev_ptr(K, kshape, torch.float16, "K")
        vp = self._dev_ptr(V, kshape, torch.float16, "V")
        shape = (self.batch, self.n_q_heads, self.head_dim)
        qp = self._dev_ptr(q, shape, torch.float16, "q")
        if out is None:
            out = torch.empty(shape, dtype=torch.float16, device=self.device)
        op = self._dev_ptr(out, shape, torch.float16, "out")
        _check(self._lib.kvq_append_decode_attention(self._h, layer, kp, vp, qp, op))
        return out

    def prefill_attention(self, layer: int, q, out=None):
        """Causal attention of the last n_q tokens over the layer's cache as it stands.
        q: fp16 [batch, n_q_heads, n_q, head_dim]; returns out of the same shape (allocated if not given)."""
        torch = self._torch
        if q.dim() != 4:
            raise ValueError("q must be [batch, n_q_heads, n_q, head_dim]")
        shape = (self.batch, self.n_q_heads, int(q.shape[2]), self.head_dim)
        qp = self._dev_ptr(q, shape, torch.float16, "q")
        if out is None:
            out = torch.empty(shape, dtype=torch.float16, device=self.device)
        op = self._dev_ptr(out, shape, torch.float16, "out")
        _check(self._lib.kvq_prefill_attention(self._h, layer, qp, shape[2], op))
        return out

    # -- bookkeeping and debugging
    def layer_tokens(self, layer: int):
        a, b = c_int32(), c_int32()
        _check(self._lib.kvq_layer_tokens(self._h, layer, ctypes.byref(a), ctypes.byref(b)))
        return a.value, b.value

    def reset(self, layer: int = -1):
        _check(self._lib.kvq_reset(self._h, layer))

    def set_decode_options(self, variant: int = 0, splits: int = 0):
        _check(self._lib.kvq_set_decode_options(self._h, variant, splits))

    def set_prefill_options(self, low_parts: int = 0):
        _check(self._lib.kvq_set_prefill_options(self._h, low_parts))

    def set_kernel_events(self, begin_event=None, end_event=None):
        """Raw hipEvent_t handles (integers or c_void_p) recorded around the main decode kernel; None switches off."""
        _check(self._lib.kvq_set_kernel_events(self._h, begin_event, end_event))

    def debug_export(self, layer: int) -> dict:
        """Canonical dump as device tensors (same keys and shapes as the documented export format)."""
        torch = self._torch
        npk, nr = self.layer_tokens(layer)
        kb, vb = self.kbits[layer], self.vbits[layer]
        B, H, D, G = self.batch, self.n_kv_heads, self.head_dim, self.group
        dev = self.device
        r = {"n_packed": npk, "n_residual": nr}

        def z(shape, dtype):
            return torch.zeros(shape, dtype=dtype, device=dev)

        if kb < 16 and self.key_mode == KEYS_PER_TOKEN:
            r["k_codes"] = z((B, H, npk, D * kb // 8), torch.uint8)
            r["k_scale"] = z((B, H, npk, D // G), torch.float32)
            r["k_zero"] = z((B, H, npk, D // G), torch.float32)
        elif kb < 16:
            r["k_codes"] = z((B, H, npk // G, D, G * kb // 8), torch.uint8)
            r["k_scale"] = z((B, H, npk // G, D), torch.float32)
            r["k_zero"] = z((B, H, npk // G, D), torch.float32)
        else:
            r["k_codes"] = z((B, H, npk, D), torch.float16)
        if vb < 16:
            r["v_codes"] = z((B, H, npk, D * vb // 8), torch.uint8)
            r["v_scale"] = z((B, H, npk, D // G), torch.float32)
            r["v_zero"] = z((B, H, npk, D // G), torch.float32)
        else:
            r["v_codes"] = z((B, H, npk, D), torch.float16)
        r["k_res"] = z((B, H, nr, D), torch.float16)
        r["v_res"] = z((B, H, nr, D), torch.float16)

        def p(name):
            t = r.get(name)
            return c_void_p(t.data_ptr()) if t is not None and t.numel() else None

        _check(self._lib.kvq_debug_export(self._h, layer, p("k_codes"), p("k_scale"), p("k_zero"), p("v_codes"),
                                          p("v_scale"), p("v_zero"), p("k_res"), p("v_res")))
        return r
