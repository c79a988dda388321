"""CPU oracle for the mixed-precision KV-cache path (KVTuner, arXiv 2502.04420).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import this package; the product path never does.
The arithmetic lives in ``kvq_oracle.c`` (plain C, written from Section 3.1
Eq. 1, Section 3.2 Eq. 2 and the KIVI settings of the experimental-settings
appendix); this module only compiles it with gcc and marshals numpy arrays.

Every function of the oracle is pinned by ``tests/test_oracle_*.py`` against
hand-worked groups, exact rational arithmetic, closed forms and library
routines, so none of it is "parity unpinned" with respect to the equations.
The paper prints no worked numeric example of codes or attention outputs, so
no pin compares against a number printed in the paper other than the
equivalent-precision figures of its searched schedules.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from ctypes import POINTER, c_double, c_float, c_int, c_uint8, c_uint16, c_void_p

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kvq_oracle.c")
_LIB = os.path.join(_HERE, "libkvq_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-std=c11", "-O2", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
             "-fno-fast-math", "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    lib = ctypes.CDLL(build())
    u8p, u16p, f32p, f64p = POINTER(c_uint8), POINTER(c_uint16), POINTER(c_float), POINTER(c_double)
    lib.kvo_half_to_float.restype = c_float
    lib.kvo_half_to_float.argtypes = [c_uint16]
    lib.kvo_double_to_half.restype = c_uint16
    lib.kvo_double_to_half.argtypes = [c_double]
    lib.kvo_quantize_group.restype = None
    lib.kvo_quantize_group.argtypes = [f32p, c_int, c_int, f32p, f32p, u8p]
    lib.kvo_quantize_group_ex.restype = None
    lib.kvo_quantize_group_ex.argtypes = [f32p, c_int, c_int, c_int, f32p, f32p, u8p]
    lib.kvo_set_scale_fp16.restype = c_int
    lib.kvo_set_scale_fp16.argtypes = [c_void_p, c_int]
    lib.kvo_set_key_per_token.restype = c_int
    lib.kvo_set_key_per_token.argtypes = [c_void_p, c_int]
    lib.kvo_reconstruct.restype = c_int
    lib.kvo_reconstruct.argtypes = [c_void_p, c_int, f64p, f64p]
    lib.kvo_create.restype = c_void_p
    lib.kvo_create.argtypes = [c_int] * 7 + [u8p, u8p]
    lib.kvo_destroy.restype = None
    lib.kvo_destroy.argtypes = [c_void_p]
    lib.kvo_reset.restype = c_int
    lib.kvo_reset.argtypes = [c_void_p, c_int]
    lib.kvo_quantize_append.restype = c_int
    lib.kvo_quantize_append.argtypes = [c_void_p, c_int, u16p, u16p, c_int]
    lib.kvo_tokens.restype = c_int
    lib.kvo_tokens.argtypes = [c_void_p, c_int, POINTER(c_int), POINTER(c_int)]
    lib.kvo_decode_attention.restype = c_int
    lib.kvo_decode_attention.argtypes = [c_void_p, c_int, u16p, u16p, f64p, f64p]
    lib.kvo_prefill_attention_at.restype = c_int
    lib.kvo_prefill_attention_at.argtypes = [c_void_p, c_int, u16p, POINTER(c_int), c_int, u16p, f64p]
    lib.kvo_prefill_attention.restype = c_int
    lib.kvo_prefill_attention.argtypes = [c_void_p, c_int, u16p, c_int, u16p, f64p]
    lib.kvo_attention_exact.restype = None
    lib.kvo_attention_exact.argtypes = [u16p, u16p, u16p] + [c_int] * 5 + [u16p, f64p, f64p]
    lib.kvo_export.restype = c_int
    lib.kvo_export.argtypes = [c_void_p, c_int, u8p, f32p, f32p, u8p, f32p, f32p, u16p, u16p]
    lib.kvo_num_threads.restype = c_int
    lib.kvo_num_threads.argtypes = []
    _lib = lib
    return lib


def _ptr(a: np.ndarray, ctype):
    return a.ctypes.data_as(POINTER(ctype))


def _as_u16(a) -> np.ndarray:
    """fp16 array (numpy float16, or anything with the same bits) -> contiguous uint16 view."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        return a.view(np.uint16)
    if a.dtype == np.uint16:
        return a
    raise TypeError("expected float16 data, got %s" % a.dtype)


def num_threads() -> int:
    return int(_load().kvo_num_threads())


def half_to_float(bits: int) -> float:
    return float(_load().kvo_half_to_float(int(bits)))


def double_to_half_bits(x: float) -> int:
    return int(_load().kvo_double_to_half(float(x)))


def quantize_group(x, bits: int, scale_fp16: bool = False):
    """Eq. 2 on one group.  x: 1-D float32.  Returns (scale, zero, codes[uint8]).

    scale_fp16: the narrow-metadata variant (scale rounded once to fp16 and used that way)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    s, z = c_float(), c_float()
    codes = np.zeros(x.size, dtype=np.uint8)
    if scale_fp16:
        _load().kvo_quantize_group_ex(_ptr(x, c_float), x.size, bits, 1, ctypes.byref(s), ctypes.byref(z),
                                      _ptr(codes, c_uint8))
    else:
        _load().kvo_quantize_group(_ptr(x, c_float), x.size, bits, ctypes.byref(s), ctypes.byref(z),
                                   _ptr(codes, c_uint8))
    return np.float32(s.value), np.float32(z.value), codes


def attention_exact(q, K, V, want_p: bool = False):
    """Eq. 1 on raw fp16 q [B,Hq,D], K,V [B,Hkv,T,D].  Returns (out fp16, out fp64[, p])."""
    qu, Ku, Vu = _as_u16(q), _as_u16(K), _as_u16(V)
    B, Hq, D = qu.shape
    _, Hkv, T, _ = Ku.shape
    out = np.zeros((B, Hq, D), dtype=np.uint16)
    o64 = np.zeros((B, Hq, D), dtype=np.float64)
    p = np.zeros((B, Hq, T), dtype=np.float64) if want_p else None
    _load().kvo_attention_exact(_ptr(qu, c_uint16), _ptr(Ku, c_uint16), _ptr(Vu, c_uint16), B, Hq, Hkv,
                                T, D, _ptr(out, c_uint16), _ptr(o64, c_double),
                                _ptr(p, c_double) if want_p else None)
    res = (out.view(np.float16), o64)
    return res + (p,) if want_p else res


class OracleCache:
    """The oracle's mirror of configure / quantize_append / decode_attention."""

    def __init__(self, n_layers, batch, n_q_heads, n_kv_heads, head_dim, kbits, vbits, group=32,
                 residual=32, scale_fp16=False, key_per_token=False):
        self.L, self.B, self.Hq, self.Hkv, self.D = n_layers, batch, n_q_heads, n_kv_heads, head_dim
        self.G, self.R = group, residual
        self.kbits = np.ascontiguousarray(kbits, dtype=np.uint8)
        self.vbits = np.ascontiguousarray(vbits, dtype=np.uint8)
        assert self.kbits.size == n_layers and self.vbits.size == n_layers
        self._h = _load().kvo_create(n_layers, batch, n_q_heads, n_kv_heads, head_dim, group, residual,
                                     _ptr(self.kbits, c_uint8), _ptr(self.vbits, c_uint8))
        if not self._h:
            raise ValueError("invalid oracle configuration")
        if scale_fp16 and _load().kvo_set_scale_fp16(self._h, 1):
            raise ValueError("could not select the fp16-scale variant")
        self.key_per_token = bool(key_per_token)
        if key_per_token and _load().kvo_set_key_per_token(self._h, 1):
            raise ValueError("could not select per-token key grouping")

    def close(self):
        if self._h:
            _load().kvo_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def reset(self, layer: int = -1):
        if _load().kvo_reset(self._h, layer):
            raise ValueError("bad layer")

    def quantize_append(self, layer: int, K, V):
        Ku, Vu = _as_u16(K), _as_u16(V)
        assert Ku.shape == Vu.shape and Ku.ndim == 4
        assert Ku.shape[0] == self.B and Ku.shape[1] == self.Hkv and Ku.shape[3] == self.D
        rc = _load().kvo_quantize_append(self._h, layer, _ptr(Ku, c_uint16), _ptr(Vu, c_uint16), Ku.shape[2])
        if rc:
            raise ValueError("oracle quantize_append failed (%d)" % rc)

    def tokens(self, layer: int):
        a, b = c_int(), c_int()
        if _load().kvo_tokens(self._h, layer, ctypes.byref(a), ctypes.byref(b)):
            raise ValueError("bad layer")
        return a.value, b.value

    def decode_attention(self, layer: int, q, want_p: bool = False):
        """Returns (out fp16 [B,Hq,D], out fp64[, p [B,Hq,T]])."""
        qu = _as_u16(q)
        assert qu.shape == (self.B, self.Hq, self.D)
        npk, nr = self.tokens(layer)
        T = npk + nr
        out = np.zeros((self.B, self.Hq, self.D), dtype=np.uint16)
        o64 = np.zeros((self.B, self.Hq, self.D), dtype=np.float64)
        p = np.zeros((self.B, self.Hq, T), dtype=np.float64) if want_p else None
        rc = _load().kvo_decode_attention(self._h, layer, _ptr(qu, c_uint16), _ptr(out, c_uint16),
                                          _ptr(o64, c_double), _ptr(p, c_double) if want_p else None)
        if rc:
            raise ValueError("oracle decode_attention failed (%d)" % rc)
        res = (out.view(np.float16), o64)
        return res + (p,) if want_p else res

    def prefill_attention(self, layer: int, q):
        """Causal attention of the last n_q tokens over the cache as it stands (Section 5.3's calibration
        design: the prompt's attention reads the dequantized cache).  q fp16 [B, Hq, n_q, D].
        Returns (out fp16 [B, Hq, n_q, D], out fp64)."""
        qu = _as_u16(q)
        assert qu.ndim == 4 and qu.shape[0] == self.B and qu.shape[1] == self.Hq and qu.shape[3] == self.D
        n_q = qu.shape[2]
        out = np.zeros(qu.shape, dtype=np.uint16)
        o64 = np.zeros(qu.shape, dtype=np.float64)
        rc = _load().kvo_prefill_attention(self._h, layer, _ptr(qu, c_uint16), n_q, _ptr(out, c_uint16), _ptr(o64, c_double))
        if rc:
            raise ValueError("oracle prefill_attention failed (%d)" % rc)
        return out.view(np.float16), o64

    def prefill_attention_at(self, layer: int, q, positions):
        """The same for queries at given absolute positions (shared by all heads): q fp16 [B, Hq, n, D], row i is
        the query at positions[i].  Returns (out fp16, out fp64), both [B, Hq, n, D]."""
        qu = _as_u16(q)
        pos = np.ascontiguousarray(np.asarray(positions, dtype=np.int32))
        assert qu.ndim == 4 and qu.shape[0] == self.B and qu.shape[1] == self.Hq and qu.shape[3] == self.D
        assert pos.ndim == 1 and pos.shape[0] == qu.shape[2]
        out = np.zeros(qu.shape, dtype=np.uint16)
        o64 = np.zeros(qu.shape, dtype=np.float64)
        rc = _load().kvo_prefill_attention_at(self._h, layer, _ptr(qu, c_uint16), _ptr(pos, c_int), pos.shape[0],
                                              _ptr(out, c_uint16), _ptr(o64, c_double))
        if rc:
            raise ValueError("oracle prefill_attention_at failed (%d)" % rc)
        return out.view(np.float16), o64

    def reconstruct(self, layer: int):
        """The layer's cache as attention sees it, in double: (K^, V^) [B, Hkv, T, D]; quantized tokens as
        code * s + z (Eq. 2), window tokens as their fp16 values."""
        npk, nr = self.tokens(layer)
        shape = (self.B, self.Hkv, npk + nr, self.D)
        Kh, Vh = np.zeros(shape, dtype=np.float64), np.zeros(shape, dtype=np.float64)
        if _load().kvo_reconstruct(self._h, layer, _ptr(Kh, c_double), _ptr(Vh, c_double)):
            raise ValueError("bad layer")
        return Kh, Vh

    def export(self, layer: int) -> dict:
        """Canonical dump: packed codes, scales, zero-points, full-precision tail."""
        npk, nr = self.tokens(layer)
        kb, vb = int(self.kbits[layer]), int(self.vbits[layer])
        B, H, D, G = self.B, self.Hkv, self.D, self.G
        r = {"n_packed": npk, "n_residual": nr}
        if kb < 16 and self.key_per_token:
            r["k_codes"] = np.zeros((B, H, npk, D * kb // 8), dtype=np.uint8)
            r["k_scale"] = np.zeros((B, H, npk, D // G), dtype=np.float32)
            r["k_zero"] = np.zeros((B, H, npk, D // G), dtype=np.float32)
        elif kb < 16:
            r["k_codes"] = np.zeros((B, H, npk // G, D, G * kb // 8), dtype=np.uint8)
            r["k_scale"] = np.zeros((B, H, npk // G, D), dtype=np.float32)
            r["k_zero"] = np.zeros((B, H, npk // G, D), dtype=np.float32)
        else:
            r["k_codes"] = np.zeros((B, H, npk, D), dtype=np.uint16)
        if vb < 16:
            r["v_codes"] = np.zeros((B, H, npk, D * vb // 8), dtype=np.uint8)
            r["v_scale"] = np.zeros((B, H, npk, D // G), dtype=np.float32)
            r["v_zero"] = np.zeros((B, H, npk, D // G), dtype=np.float32)
        else:
            r["v_codes"] = np.zeros((B, H, npk, D), dtype=np.uint16)
        r["k_res"] = np.zeros((B, H, nr, D), dtype=np.uint16)
        r["v_res"] = np.zeros((B, H, nr, D), dtype=np.uint16)

        def p8(name):
            a = r.get(name)
            return None if a is None else a.ctypes.data_as(POINTER(c_uint8))

        def pf(name):
            a = r.get(name)
            return None if a is None else _ptr(a, c_float)

        rc = _load().kvo_export(self._h, layer, p8("k_codes"), pf("k_scale"), pf("k_zero"), p8("v_codes"),
                                pf("v_scale"), pf("v_zero"), _ptr(r["k_res"], c_uint16),
                                _ptr(r["v_res"], c_uint16))
        if rc:
            raise ValueError("oracle export failed (%d)" % rc)
        return r
