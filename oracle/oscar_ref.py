"""ctypes loader and numpy front-end of the C oracle (test infrastructure only).

The arithmetic lives in ``oscar_oracle.c``; this file only allocates numpy
arrays, fills the C struct and forwards calls.  Nothing here is used by the
product path.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

F32, BF16, F16 = 0, 1, 2
ZP_INT, ZP_MIN = 0, 1
SCALE_NONE, SCALE_L2, SCALE_MAX, SCALE_MEAN_ABS = 0, 1, 2, 3
NORM_PER_HEAD, NORM_ALL_KV_HEADS = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oscar_oracle.c")
_SO = os.path.join(_HERE, "liboscar_oracle.so")
_lib = None


def build_oracle(force: bool = False) -> str:
    """Compile the oracle with gcc.  Contraction off: the encoder is defined in
    one fixed fp32 operation order."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-shared", "-fPIC", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


class _CCache(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "d", "bits", "k_group", "v_group", "R", "meta_dtype", "zp_mode", "rotate",
        "scale_mode", "norm_scope", "batch", "n_kv_heads", "cap_tokens")] + [
        ("n_packed", C.c_void_p), ("n_res", C.c_void_p),
        ("k_codes", C.c_void_p), ("k_delta", C.c_void_p), ("k_zero", C.c_void_p),
        ("k_norm", C.c_void_p), ("v_codes", C.c_void_p), ("v_delta", C.c_void_p),
        ("v_zero", C.c_void_p), ("res_k", C.c_void_p), ("res_v", C.c_void_p),
        ("res_norm", C.c_void_p)]


def lib():
    global _lib
    if _lib is None:
        build_oracle()
        L = C.CDLL(_SO)
        fp = C.POINTER(C.c_float)
        L.oref_round_dtype.restype = C.c_float
        L.oref_round_dtype.argtypes = [C.c_float, C.c_int]
        L.oref_round_meta.restype = C.c_float
        L.oref_round_meta.argtypes = [C.c_float, C.c_int]
        L.oref_sumabs_tree.restype = C.c_float
        L.oref_sumabs_tree.argtypes = [fp, C.c_int]
        L.oref_fwht.argtypes = [fp, C.c_int]
        L.oref_sumsq_tree.restype = C.c_float
        L.oref_sumsq_tree.argtypes = [fp, C.c_int]
        L.oref_key_transform.argtypes = [fp, C.c_int, C.c_int, C.c_int, C.c_int, fp, fp]
        L.oref_query_transform.argtypes = [fp, C.c_int, C.c_int, fp]
        L.oref_token_norm_all_heads.restype = C.c_float
        L.oref_token_norm_all_heads.argtypes = [fp, C.c_int, C.c_size_t, C.c_int, C.c_int, C.c_int]
        L.oref_key_transform_given_norm.argtypes = [fp, C.c_int, C.c_int, C.c_float, fp]
        L.oref_quant_params.argtypes = [C.c_float, C.c_float, C.c_int, C.c_int, C.c_int, fp, fp]
        L.oref_quant_code.restype = C.c_uint8
        L.oref_quant_code.argtypes = [C.c_float, C.c_float, C.c_float, C.c_int, C.c_int]
        L.oref_dequant.restype = C.c_double
        L.oref_dequant.argtypes = [C.c_uint8, C.c_float, C.c_float, C.c_int]
        L.oref_quant_group.argtypes = [fp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, fp, fp,
                                       C.POINTER(C.c_uint8), C.c_int]
        L.oref_append.restype = C.c_int
        L.oref_append.argtypes = [C.POINTER(_CCache), fp, fp, C.c_int, C.c_void_p, C.c_int,
                                  C.c_int]
        L.oref_decode_attn.argtypes = [C.POINTER(_CCache), fp, C.c_int, C.c_float, fp, C.c_int]
        L.oref_dequantize_stream.argtypes = [C.POINTER(_CCache), C.c_int, C.c_int,
                                             C.POINTER(C.c_double), C.POINTER(C.c_double)]
        L.oref_plain_attn.argtypes = [fp, fp, fp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                      C.c_void_p, C.c_float, fp, C.c_int]
        L.oref_max_threads.restype = C.c_int
        _lib = L
    return _lib


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _fp(a):
    return a.ctypes.data_as(C.POINTER(C.c_float))


# ---- thin wrappers of the primitives (for the pin tests) -------------------

def round_dtype(x: float, dtype: int) -> float:
    return float(lib().oref_round_dtype(C.c_float(x), dtype))


def round_meta(x: float, dtype: int) -> float:
    """Storage rounding of a metadata value: nearest even, saturating at the largest finite value."""
    return float(lib().oref_round_meta(C.c_float(x), dtype))


def fwht(x) -> np.ndarray:
    """Normalized Sylvester Hadamard transform of the last axis."""
    y = _f32(x).copy()
    rows = y.reshape(-1, y.shape[-1])
    for r in rows:
        lib().oref_fwht(_fp(r), r.shape[0])
    return y


def sumsq_tree(x) -> float:
    y = _f32(x)
    return float(lib().oref_sumsq_tree(_fp(y), y.shape[0]))


def sumabs_tree(x) -> float:
    y = _f32(x)
    return float(lib().oref_sumabs_tree(_fp(y), y.shape[0]))


def key_transform(k, rotate=1, scale_mode=SCALE_L2, meta_dtype=F32):
    k = _f32(k)
    u = np.empty_like(k)
    n = np.zeros(1, np.float32)
    lib().oref_key_transform(_fp(k), k.shape[0], rotate, scale_mode, meta_dtype, _fp(u), _fp(n))
    return u, float(n[0])


def token_norm_all_heads(k_heads, rotate=1, meta_dtype=F32) -> float:
    """k_heads: [n_kv_heads, d] of one token; the one norm over all its kv heads."""
    k = _f32(k_heads)
    return float(lib().oref_token_norm_all_heads(_fp(k), k.shape[0], k.shape[1], k.shape[1],
                                                 rotate, meta_dtype))


def key_transform_given_norm(k, nf, rotate=1):
    k = _f32(k)
    u = np.empty_like(k)
    lib().oref_key_transform_given_norm(_fp(k), k.shape[0], rotate, C.c_float(nf), _fp(u))
    return u


def query_transform(q, rotate=1):
    q = _f32(q)
    out = np.empty_like(q)
    lib().oref_query_transform(_fp(q), q.shape[0], rotate, _fp(out))
    return out


def quant_params(mn, mx, bits, meta_dtype=F32, zp_mode=ZP_INT):
    d = np.zeros(1, np.float32)
    z = np.zeros(1, np.float32)
    lib().oref_quant_params(C.c_float(mn), C.c_float(mx), bits, meta_dtype, zp_mode, _fp(d),
                            _fp(z))
    return float(d[0]), float(z[0])


def quant_code(x, delta, zero, bits, zp_mode=ZP_INT) -> int:
    return int(lib().oref_quant_code(C.c_float(x), C.c_float(delta), C.c_float(zero), bits,
                                     zp_mode))


def dequant(c, delta, zero, zp_mode=ZP_INT) -> float:
    return float(lib().oref_dequant(C.c_uint8(c), C.c_float(delta), C.c_float(zero), zp_mode))


def quant_group(x, bits, meta_dtype=F32, zp_mode=ZP_INT):
    x = _f32(x)
    d = np.zeros(1, np.float32)
    z = np.zeros(1, np.float32)
    codes = np.zeros(x.shape[0], np.uint8)
    lib().oref_quant_group(_fp(x), x.shape[0], 1, bits, meta_dtype, zp_mode, _fp(d), _fp(z),
                           codes.ctypes.data_as(C.POINTER(C.c_uint8)), 1)
    return codes, float(d[0]), float(z[0])


def max_threads() -> int:
    return int(lib().oref_max_threads())


def plain_attn(q, k, v, seq_lens=None, scale=0.0, nthreads=1) -> np.ndarray:
    """Plain attention on un-rotated K, V ([B,S,Hkv,d]); q [B,Hq,d]."""
    q, k, v = _f32(q), _f32(k), _f32(v)
    B, S, Hkv, d = k.shape
    Hq = q.shape[1]
    out = np.empty_like(q)
    sl = None
    if seq_lens is not None:
        sl = np.ascontiguousarray(seq_lens, dtype=np.int32)
    lib().oref_plain_attn(_fp(q), _fp(k), _fp(v), B, S, Hq, Hkv, d,
                          sl.ctypes.data if sl is not None else None, C.c_float(scale),
                          _fp(out), nthreads)
    return out


# ---- the cache --------------------------------------------------------------

@dataclass
class OracleConfig:
    head_dim: int = 128
    bits: int = 2
    k_group: int = 128
    v_group: int = 32
    page_size: int = 128
    meta_dtype: int = F16
    zp_mode: int = ZP_INT
    rotate: int = 1
    scale_mode: int = SCALE_L2
    norm_scope: int = NORM_PER_HEAD


class OracleCache:
    """Canonical unpacked cache for [batch] sequences x [n_kv_heads] heads."""

    def __init__(self, cfg: OracleConfig, batch: int, n_kv_heads: int, cap_tokens: int):
        R, d = cfg.page_size, cfg.head_dim
        assert cap_tokens % R == 0 and R % cfg.k_group == 0 and d % cfg.v_group == 0
        self.cfg, self.batch, self.n_kv_heads, self.cap = cfg, batch, n_kv_heads, cap_tokens
        B, H = batch, n_kv_heads
        self.n_packed = np.zeros(B, np.int32)
        self.n_res = np.zeros(B, np.int32)
        self.k_codes = np.zeros((B, H, cap_tokens, d), np.uint8)
        self.k_delta = np.zeros((B, H, cap_tokens // cfg.k_group, d), np.float32)
        self.k_zero = np.zeros_like(self.k_delta)
        self.k_norm = np.zeros((B, H, cap_tokens), np.float32)
        self.v_codes = np.zeros((B, H, cap_tokens, d), np.uint8)
        self.v_delta = np.zeros((B, H, cap_tokens, d // cfg.v_group), np.float32)
        self.v_zero = np.zeros_like(self.v_delta)
        self.res_k = np.zeros((B, H, R, d), np.float32)
        self.res_v = np.zeros((B, H, R, d), np.float32)
        self.res_norm = np.zeros((B, H, R), np.float32)
        c = _CCache()
        c.d, c.bits, c.k_group, c.v_group, c.R = d, cfg.bits, cfg.k_group, cfg.v_group, R
        c.meta_dtype, c.zp_mode, c.rotate, c.scale_mode = (cfg.meta_dtype, cfg.zp_mode,
                                                          cfg.rotate, cfg.scale_mode)
        c.norm_scope = cfg.norm_scope
        c.batch, c.n_kv_heads, c.cap_tokens = B, H, cap_tokens
        for name in ("n_packed", "n_res", "k_codes", "k_delta", "k_zero", "k_norm", "v_codes",
                     "v_delta", "v_zero", "res_k", "res_v", "res_norm"):
            setattr(c, name, getattr(self, name).ctypes.data)
        self._c = c

    def append(self, k, v, new_lens=None, eager=False, nthreads=1):
        """k, v: [batch, T, n_kv_heads, d] (values already rounded to the input dtype)."""
        k, v = _f32(k), _f32(v)
        assert k.shape == v.shape and k.shape[0] == self.batch and k.shape[2] == self.n_kv_heads
        nl = None if new_lens is None else np.ascontiguousarray(new_lens, dtype=np.int32)
        rc = lib().oref_append(C.byref(self._c), _fp(k), _fp(v), k.shape[1],
                               nl.ctypes.data if nl is not None else None, int(eager), nthreads)
        if rc != 0:
            raise ValueError("oracle append: capacity or length error")

    def decode_attn(self, q, scale=0.0, nthreads=1) -> np.ndarray:
        """q: [batch, n_q_heads, d] un-rotated; returns fp32 [batch, n_q_heads, d]."""
        q = _f32(q)
        out = np.empty_like(q)
        lib().oref_decode_attn(C.byref(self._c), _fp(q), q.shape[1], C.c_float(scale), _fp(out),
                               nthreads)
        return out

    def dequantize(self, b: int, h: int):
        """(k_hat, v_hat) float64 [total, d]; k_hat is in the rotated basis."""
        total = int(self.n_packed[b] + self.n_res[b])
        d = self.cfg.head_dim
        kh = np.zeros((total, d), np.float64)
        vh = np.zeros((total, d), np.float64)
        lib().oref_dequantize_stream(C.byref(self._c), b, h,
                                     kh.ctypes.data_as(C.POINTER(C.c_double)),
                                     vh.ctypes.data_as(C.POINTER(C.c_double)))
        return kh, vh
