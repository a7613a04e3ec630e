"""ctypes binding of the C-ABI HIP library (argument marshalling only).

Every step of the hot path runs inside ``liboscar_hip.so``; PyTorch is used for
device memory and streams.  There is no CPU fallback: if the library is missing
the import of any entry point raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import numpy as np

F32, BF16, F16 = 0, 1, 2
ZP_INT, ZP_MIN = 0, 1
NORM_PER_HEAD, NORM_ALL_KV_HEADS = 0, 1
ROTATION_ON, ROTATION_OFF = 0, 1
SCALE_L2, SCALE_NONE, SCALE_MAX, SCALE_MEAN_ABS = 0, 1, 2, 3
OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_CAPACITY, ERR_WORKSPACE, ERR_HIP = 0, -1, -2, -3, -4, -5
APPEND_EAGER = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
# OSCAR_HIP_LIB points at an alternative build of the same library (profiling variants)
LIB_PATH = os.environ.get("OSCAR_HIP_LIB") or os.path.join(_HERE, "liboscar_hip.so")

EXPORTS = ("oscar_version", "oscar_status_string", "oscar_cache_sizes",
           "oscar_decode_auto_splits", "oscar_decode_workspace_bytes", "oscar_quantize_append",
           "oscar_decode_attn", "oscar_decode_attn_partial", "oscar_decode_attn_reduce",
           "oscar_bf16_decode_attn", "oscar_debug_dump", "oscar_timer_create",
           "oscar_timer_destroy", "oscar_timer_elapsed_us", "oscar_decode_attn_partial_timed",
           "oscar_probe_stream_read", "oscar_rotate", "oscar_rotate_columns",
           "oscar_debug_force_generic_decode", "oscar_decode_attn_noalloc",
           "oscar_decode_step", "oscar_cache_layer")


class OscarError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


class CConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "head_dim", "n_q_heads", "n_kv_heads", "bits", "k_group", "v_group", "page_size",
        "io_dtype", "meta_dtype", "zp_mode", "norm_scope", "rotation", "scale_mode")]


class CCache(C.Structure):
    _fields_ = [("cfg", CConfig), ("batch", C.c_int32), ("max_pages_per_seq", C.c_int32),
                ("num_pages", C.c_int32), ("reserved_", C.c_int32)] + [
        (n, C.c_void_p) for n in ("k_codes", "k_meta", "k_norms", "v_codes", "v_meta", "res_k",
                                  "res_v", "res_norm", "block_table", "seq_lens", "res_lens",
                                  "dev_status", "tickets")]


class CPoolSizes(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in (
        "k_codes", "k_meta", "k_norms", "v_codes", "v_meta", "res_k", "res_v", "res_norm",
        "block_table", "seq_lens", "res_lens", "tickets", "page_bytes_per_kv_head",
        "bytes_per_token_kv_head")]


_lib = None


def lib():
    """Load liboscar_hip.so (after torch, so both share one HIP runtime)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with "
                          "`python -m paper_2605_19660_amd.build` (there is no fallback path)")
    import torch  # noqa: F401  (loads the HIP runtime the library links against)
    L = C.CDLL(LIB_PATH)
    vp, i32, u32, sz, f32 = C.c_void_p, C.c_int32, C.c_uint32, C.c_size_t, C.c_float
    L.oscar_version.restype = C.c_int
    L.oscar_status_string.restype = C.c_char_p
    L.oscar_status_string.argtypes = [C.c_int]
    L.oscar_cache_sizes.restype = C.c_int
    L.oscar_cache_sizes.argtypes = [C.POINTER(CConfig), i32, i32, i32, C.POINTER(CPoolSizes)]
    L.oscar_cache_layer.restype = C.c_int
    L.oscar_cache_layer.argtypes = [C.POINTER(CCache), i32, i32, C.POINTER(CCache)]
    L.oscar_decode_auto_splits.restype = i32
    L.oscar_decode_auto_splits.argtypes = [C.POINTER(CConfig), i32, i32]
    L.oscar_decode_workspace_bytes.restype = sz
    L.oscar_decode_workspace_bytes.argtypes = [C.POINTER(CConfig), i32, i32]
    L.oscar_quantize_append.restype = C.c_int
    L.oscar_quantize_append.argtypes = [vp, vp, i32, vp, C.POINTER(CCache), i32, u32, vp]
    L.oscar_decode_attn.restype = C.c_int
    L.oscar_decode_attn.argtypes = [vp, C.POINTER(CCache), vp, i32, f32, i32, i32, vp, sz, vp]
    L.oscar_decode_attn_noalloc.restype = C.c_int
    L.oscar_decode_attn_noalloc.argtypes = [vp, C.POINTER(CCache), vp, i32, f32, i32, i32, vp]
    L.oscar_decode_step.restype = C.c_int
    L.oscar_decode_step.argtypes = [vp, vp, vp, C.POINTER(CCache), vp, i32, f32, i32, i32, vp, sz, vp, vp]
    L.oscar_decode_attn_partial.restype = C.c_int
    L.oscar_decode_attn_partial.argtypes = [vp, C.POINTER(CCache), f32, i32, vp, sz, vp]
    L.oscar_decode_attn_partial_timed.restype = C.c_int
    L.oscar_decode_attn_partial_timed.argtypes = [vp, C.POINTER(CCache), f32, i32, vp, sz, vp, vp]
    L.oscar_timer_create.restype = C.c_int
    L.oscar_timer_create.argtypes = [C.POINTER(vp)]
    L.oscar_timer_destroy.restype = C.c_int
    L.oscar_timer_destroy.argtypes = [vp]
    L.oscar_timer_elapsed_us.restype = C.c_int
    L.oscar_timer_elapsed_us.argtypes = [vp, C.POINTER(C.c_float)]
    L.oscar_rotate.restype = C.c_int
    L.oscar_rotate.argtypes = [vp, vp, vp, C.c_int64, i32, i32, C.c_uint32, vp]
    L.oscar_rotate_columns.restype = C.c_int
    L.oscar_rotate_columns.argtypes = [vp, vp, C.c_int64, C.c_int64, i32, vp]
    L.oscar_probe_stream_read.restype = C.c_int
    L.oscar_probe_stream_read.argtypes = [vp, sz, i32, vp, vp, vp]
    L.oscar_decode_attn_reduce.restype = C.c_int
    L.oscar_decode_attn_reduce.argtypes = [C.POINTER(CCache), vp, i32, i32, vp, sz, vp]
    L.oscar_bf16_decode_attn.restype = C.c_int
    L.oscar_bf16_decode_attn.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, i32,
                                         f32, i32, i32, vp, sz, vp]
    L.oscar_debug_force_generic_decode.restype = C.c_int
    L.oscar_debug_force_generic_decode.argtypes = [i32]
    L.oscar_debug_dump.restype = C.c_int
    L.oscar_debug_dump.argtypes = [C.POINTER(CCache), i32, i32, i32] + [vp] * 11 + [vp]
    _lib = L
    return L


def status_string(status: int) -> str:
    return lib().oscar_status_string(status).decode()


def _check(rc: int, where: str):
    if rc != OK:
        raise OscarError(rc, where)


@dataclass
class Config:
    n_q_heads: int
    n_kv_heads: int
    head_dim: int = 128
    bits: int = 2
    k_group: int = 128
    v_group: int = 32
    page_size: int = 128
    io_dtype: int = BF16
    meta_dtype: int = F16
    zp_mode: int = ZP_INT
    norm_scope: int = NORM_PER_HEAD
    rotation: int = ROTATION_ON
    scale_mode: int = SCALE_L2

    def c(self) -> CConfig:
        return CConfig(self.head_dim, self.n_q_heads, self.n_kv_heads, self.bits, self.k_group,
                       self.v_group, self.page_size, self.io_dtype, self.meta_dtype, self.zp_mode,
                       self.norm_scope, self.rotation, self.scale_mode)


def torch_dtype(code: int):
    import torch
    return {F32: torch.float32, BF16: torch.bfloat16, F16: torch.float16}[code]


def dtype_code(dt) -> int:
    import torch
    return {torch.float32: F32, torch.bfloat16: BF16, torch.float16: F16}[dt]


def cache_sizes(cfg: Config, batch: int, num_pages: int, max_pages_per_seq: int) -> CPoolSizes:
    out = CPoolSizes()
    cc = cfg.c()
    _check(lib().oscar_cache_sizes(C.byref(cc), batch, num_pages, max_pages_per_seq,
                                   C.byref(out)), "oscar_cache_sizes")
    return out


def _stream_ptr(stream):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


class Cache:
    """Device pools of one paged OScaR cache, allocated through torch.

    block_table defaults to sequence-major identity; pass `page_perm` (a permutation of
    range(num_pages)) to scatter logical pages over physical ones."""

    def __init__(self, cfg: Config, batch: int, max_pages_per_seq: int, device="cuda",
                 num_pages: int | None = None, page_perm=None, fused: bool = True):
        import torch
        self.cfg, self.batch, self.max_pages_per_seq = cfg, batch, max_pages_per_seq
        self.num_pages = num_pages if num_pages is not None else batch * max_pages_per_seq
        self.device = torch.device(device)
        sz = cache_sizes(cfg, batch, self.num_pages, max_pages_per_seq)
        self.sizes = sz

        def pool(nbytes):
            return torch.zeros(int(nbytes), dtype=torch.uint8, device=self.device)

        self.k_codes, self.k_meta, self.k_norms = pool(sz.k_codes), pool(sz.k_meta), pool(sz.k_norms)
        self.v_codes, self.v_meta = pool(sz.v_codes), pool(sz.v_meta)
        self.res_k, self.res_v, self.res_norm = pool(sz.res_k), pool(sz.res_v), pool(sz.res_norm)
        table = np.arange(batch * max_pages_per_seq, dtype=np.int64)
        if page_perm is not None:
            table = np.asarray(page_perm, dtype=np.int64)[:batch * max_pages_per_seq]
        assert table.max() < self.num_pages
        self.block_table = torch.from_numpy(table.astype(np.int32).reshape(batch, max_pages_per_seq)).to(self.device)
        self.seq_lens = torch.zeros(batch, dtype=torch.int32, device=self.device)
        self.res_lens = torch.zeros(batch, dtype=torch.int32, device=self.device)
        self.dev_status = torch.zeros(1, dtype=torch.int32, device=self.device)
        self.tickets = torch.zeros(int(sz.tickets) // 4, dtype=torch.int32, device=self.device)
        self.fused = fused
        self._c = CCache()
        self._c.cfg = cfg.c()
        self._c.batch, self._c.max_pages_per_seq, self._c.num_pages = batch, max_pages_per_seq, self.num_pages
        for n in ("k_codes", "k_meta", "k_norms", "v_codes", "v_meta", "res_k", "res_v", "res_norm",
                  "block_table", "seq_lens", "res_lens", "dev_status"):
            setattr(self._c, n, getattr(self, n).data_ptr())
        self._c.tickets = self.tickets.data_ptr() if fused else None

    @property
    def c(self) -> CCache:
        return self._c

    def packed_bytes(self) -> int:
        s = self.sizes
        return int(s.k_codes + s.k_meta + s.k_norms + s.v_codes + s.v_meta)


class _LayerView:
    """One layer of a MultiLayerCache: an object with the attributes the call wrappers use."""

    def __init__(self, parent: "MultiLayerCache", layer: int):
        self.parent, self.layer = parent, layer
        self.cfg, self.batch, self.max_pages_per_seq = parent.cfg, parent.batch, parent.max_pages_per_seq
        self._c = CCache()
        _check(lib().oscar_cache_layer(C.byref(parent._c), parent.n_layers, layer, C.byref(self._c)),
               "oscar_cache_layer")
        self.seq_lens, self.res_lens = parent.seq_lens[layer], parent.res_lens[layer]
        self.dev_status = parent.dev_status

    @property
    def c(self) -> CCache:
        return self._c


class MultiLayerCache:
    """n_layers caches that share one block table: every pool is allocated n_layers times as large
    and sliced per layer by oscar_cache_layer; seq_lens / res_lens are [n_layers, batch]."""

    def __init__(self, cfg: Config, batch: int, max_pages_per_seq: int, n_layers: int, device="cuda",
                 page_perm=None):
        import torch
        self.cfg, self.batch, self.max_pages_per_seq, self.n_layers = cfg, batch, max_pages_per_seq, n_layers
        self.num_pages = batch * max_pages_per_seq
        self.device = torch.device(device)
        sz = cache_sizes(cfg, batch, self.num_pages, max_pages_per_seq)
        self.sizes = sz

        def pool(nbytes):
            return torch.zeros(int(nbytes) * n_layers, dtype=torch.uint8, device=self.device)

        self.k_codes, self.k_meta, self.k_norms = pool(sz.k_codes), pool(sz.k_meta), pool(sz.k_norms)
        self.v_codes, self.v_meta = pool(sz.v_codes), pool(sz.v_meta)
        self.res_k, self.res_v, self.res_norm = pool(sz.res_k), pool(sz.res_v), pool(sz.res_norm)
        table = np.arange(batch * max_pages_per_seq, dtype=np.int64)
        if page_perm is not None:
            table = np.asarray(page_perm, dtype=np.int64)[:batch * max_pages_per_seq]
        self.block_table = torch.from_numpy(table.astype(np.int32).reshape(batch, max_pages_per_seq)).to(self.device)
        self.seq_lens = torch.zeros(n_layers, batch, dtype=torch.int32, device=self.device)
        self.res_lens = torch.zeros(n_layers, batch, dtype=torch.int32, device=self.device)
        self.dev_status = torch.zeros(1, dtype=torch.int32, device=self.device)
        self.tickets = torch.zeros(n_layers, dtype=torch.int32, device=self.device)
        self._c = CCache()
        self._c.cfg = cfg.c()
        self._c.batch, self._c.max_pages_per_seq, self._c.num_pages = batch, max_pages_per_seq, self.num_pages
        for n in ("k_codes", "k_meta", "k_norms", "v_codes", "v_meta", "res_k", "res_v", "res_norm",
                  "block_table", "seq_lens", "res_lens", "dev_status", "tickets"):
            setattr(self._c, n, getattr(self, n).data_ptr())
        self.layers = [_LayerView(self, l) for l in range(n_layers)]

    def layer(self, l: int) -> _LayerView:
        return self.layers[l]


def quantize_append(cache: Cache, k, v, new_lens=None, eager: bool = False,
                    max_seq_len_hint: int = -1, stream=None):
    """oscar_quantize_append: k, v device tensors [batch, T, n_kv_heads, d] of the io dtype."""
    assert k.is_cuda and v.is_cuda and k.is_contiguous() and v.is_contiguous()
    assert k.shape == v.shape and k.dtype == v.dtype == torch_dtype(cache.cfg.io_dtype)
    assert k.shape[0] == cache.batch and k.shape[2] == cache.cfg.n_kv_heads and k.shape[3] == cache.cfg.head_dim
    nl = None if new_lens is None else new_lens.data_ptr()
    rc = lib().oscar_quantize_append(k.data_ptr(), v.data_ptr(), k.shape[1], nl, C.byref(cache.c),
                                     max_seq_len_hint, APPEND_EAGER if eager else 0,
                                     _stream_ptr(stream))
    _check(rc, "oscar_quantize_append")


def decode_auto_splits(cfg: Config, batch: int, max_seq_len: int) -> int:
    cc = cfg.c()
    return int(lib().oscar_decode_auto_splits(C.byref(cc), batch, max_seq_len))


def decode_workspace_bytes(cfg: Config, batch: int, num_splits: int) -> int:
    cc = cfg.c()
    return int(lib().oscar_decode_workspace_bytes(C.byref(cc), batch, num_splits))


def decode_attn(cache: Cache, q, out=None, scale: float = 0.0, max_seq_len_hint: int = 0,
                num_splits: int = 0, workspace=None, stream=None):
    """oscar_decode_attn: q [batch, n_q_heads, d] (un-rotated); returns `out` (fp32 by default)."""
    import torch
    assert q.is_cuda and q.is_contiguous() and q.dtype == torch_dtype(cache.cfg.io_dtype)
    assert tuple(q.shape) == (cache.batch, cache.cfg.n_q_heads, cache.cfg.head_dim)
    if out is None:
        out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
    if num_splits == 0:
        num_splits = decode_auto_splits(cache.cfg, cache.batch, max_seq_len_hint)
    if workspace is None:
        workspace = torch.empty(decode_workspace_bytes(cache.cfg, cache.batch, num_splits),
                                dtype=torch.uint8, device=q.device)
    rc = lib().oscar_decode_attn(q.data_ptr(), C.byref(cache.c), out.data_ptr(),
                                 dtype_code(out.dtype), scale, max_seq_len_hint, num_splits,
                                 workspace.data_ptr(), workspace.numel(), _stream_ptr(stream))
    _check(rc, "oscar_decode_attn")
    return out


def decode_step(cache: Cache, k_new, v_new, q, out, workspace, num_splits: int,
                max_seq_len_hint: int, scale: float = 0.0, stream=None, timer: "Timer | None" = None):
    """oscar_decode_step: append one token per sequence (k_new, v_new: [batch, 1, n_kv_heads, d]),
    then decode attention into `out`; the caller brings workspace and output."""
    rc = lib().oscar_decode_step(k_new.data_ptr(), v_new.data_ptr(), q.data_ptr(), C.byref(cache.c),
                                 out.data_ptr(), dtype_code(out.dtype), scale, max_seq_len_hint,
                                 num_splits, workspace.data_ptr(), workspace.numel(),
                                 _stream_ptr(stream), timer.handle if timer is not None else None)
    _check(rc, "oscar_decode_step")
    return out


NOALLOC_SCRATCH_BYTES = 4 << 20


def decode_attn_noalloc(cache: Cache, q, out, scale: float = 0.0, max_seq_len_hint: int = 0,
                        num_splits: int = 0, stream=None):
    """oscar_decode_attn_noalloc: the caller brings `out`; nothing is allocated on either side."""
    rc = lib().oscar_decode_attn_noalloc(q.data_ptr(), C.byref(cache.c), out.data_ptr(),
                                         dtype_code(out.dtype), scale, max_seq_len_hint, num_splits,
                                         _stream_ptr(stream))
    _check(rc, "oscar_decode_attn_noalloc")
    return out


def debug_force_generic_decode(on: bool) -> bool:
    """oscar_debug_force_generic_decode: route every decode launch to the plain-ALU kernel."""
    return bool(lib().oscar_debug_force_generic_decode(1 if on else 0))


class Timer:
    """oscar_timer: device time of one kernel launched by decode_attn_partial(timer=...)."""

    def __init__(self):
        self.handle = C.c_void_p()
        _check(lib().oscar_timer_create(C.byref(self.handle)), "oscar_timer_create")

    def elapsed_us(self) -> float:
        us = C.c_float()
        _check(lib().oscar_timer_elapsed_us(self.handle, C.byref(us)), "oscar_timer_elapsed_us")
        return us.value

    def close(self):
        if self.handle:
            lib().oscar_timer_destroy(self.handle)
            self.handle = C.c_void_p()


ROTATE_NORMALIZE, ROTATE_FAST_RSQRT, ROTATE_MATRIX_CORE = 1, 2, 4


def rotate(x, normalize: bool = False, fast_rsqrt: bool = False, meta_dtype: int = F16, stream=None,
           matrix_core: bool = False):
    """oscar_rotate on a [..., 128] tensor: H(x)/sqrt(128) as fp32, or (normalize) the fp16
    unit-norm rotated vectors and their norms."""
    import torch
    assert x.is_cuda and x.is_contiguous() and x.shape[-1] == 128
    n_vec = x.numel() // 128
    if normalize:
        out = torch.empty(x.shape, dtype=torch.float16, device=x.device)
        norms = torch.empty(x.shape[:-1], dtype=torch_dtype(meta_dtype), device=x.device)
    else:
        out = torch.empty(x.shape, dtype=torch.float32, device=x.device)
        norms = None
    flags = ((ROTATE_NORMALIZE if normalize else 0) | (ROTATE_FAST_RSQRT if fast_rsqrt else 0) |
             (ROTATE_MATRIX_CORE if matrix_core else 0))
    rc = lib().oscar_rotate(x.data_ptr(), out.data_ptr(), None if norms is None else norms.data_ptr(),
                            n_vec, dtype_code(x.dtype), meta_dtype, flags, _stream_ptr(stream))
    _check(rc, "oscar_rotate")
    return (out, norms) if normalize else out


def rotate_columns(w, stream=None):
    """oscar_rotate_columns on a [n_heads*128, n_cols] matrix: H applied along the rows of every
    128-row block, fp32 result (OScaR-Preprocess: H W_O)."""
    import torch
    assert w.is_cuda and w.is_contiguous() and w.dim() == 2 and w.shape[0] % 128 == 0
    out = torch.empty(w.shape, dtype=torch.float32, device=w.device)
    rc = lib().oscar_rotate_columns(w.data_ptr(), out.data_ptr(), w.shape[0], w.shape[1],
                                    dtype_code(w.dtype), _stream_ptr(stream))
    _check(rc, "oscar_rotate_columns")
    return out


def probe_stream_read(src, nbytes: int, workgroups: int, timer: "Timer | None" = None, stream=None):
    """oscar_probe_stream_read: plain streaming read of the first `nbytes` bytes of tensor `src`."""
    assert src.is_cuda and src.is_contiguous() and nbytes <= src.numel() * src.element_size()
    rc = lib().oscar_probe_stream_read(src.data_ptr(), nbytes, workgroups, None,
                                       _stream_ptr(stream), timer.handle if timer else None)
    _check(rc, "oscar_probe_stream_read")


def decode_attn_partial(cache: Cache, q, workspace, num_splits: int, scale: float = 0.0,
                        stream=None, timer: "Timer | None" = None):
    """oscar_decode_attn_partial(_timed): first pass only (writes split partials to `workspace`)."""
    if timer is not None:
        rc = lib().oscar_decode_attn_partial_timed(q.data_ptr(), C.byref(cache.c), scale,
                                                   num_splits, workspace.data_ptr(),
                                                   workspace.numel(), _stream_ptr(stream),
                                                   timer.handle)
        _check(rc, "oscar_decode_attn_partial_timed")
        return
    rc = lib().oscar_decode_attn_partial(q.data_ptr(), C.byref(cache.c), scale, num_splits,
                                         workspace.data_ptr(), workspace.numel(),
                                         _stream_ptr(stream))
    _check(rc, "oscar_decode_attn_partial")


def decode_attn_reduce(cache: Cache, out, workspace, num_splits: int, stream=None):
    """oscar_decode_attn_reduce: merge the split partials in `workspace` into `out`."""
    rc = lib().oscar_decode_attn_reduce(C.byref(cache.c), out.data_ptr(), dtype_code(out.dtype),
                                        num_splits, workspace.data_ptr(), workspace.numel(),
                                        _stream_ptr(stream))
    _check(rc, "oscar_decode_attn_reduce")
    return out


def bf16_decode_attn(q, k, v, seq_lens, out=None, scale: float = 0.0, max_seq_len_hint: int = 0,
                     num_splits: int = 0, workspace=None, stream=None, head_major: bool = False):
    """oscar_bf16_decode_attn: comparator on an uncompressed cache, [batch, S, n_kv_heads, d]
    or (head_major) [batch, n_kv_heads, S, d]."""
    import torch
    assert q.is_cuda and k.is_contiguous() and v.is_contiguous() and q.is_contiguous()
    if head_major:
        B, Hkv, S, d = k.shape
    else:
        B, S, Hkv, d = k.shape
    Hq = q.shape[1]
    cfg = Config(Hq, Hkv, d)
    if out is None:
        out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
    if num_splits == 0:
        num_splits = decode_auto_splits(cfg, B, max_seq_len_hint or S)
    if workspace is None:
        workspace = torch.empty(decode_workspace_bytes(cfg, B, num_splits), dtype=torch.uint8,
                                device=q.device)
    rc = lib().oscar_bf16_decode_attn(q.data_ptr(), k.data_ptr(), v.data_ptr(),
                                      None if seq_lens is None else seq_lens.data_ptr(),
                                      out.data_ptr(), dtype_code(k.dtype), dtype_code(out.dtype), B,
                                      S, 1 if head_major else 0, Hq, Hkv, d, scale, max_seq_len_hint, num_splits,
                                      workspace.data_ptr(), workspace.numel(), _stream_ptr(stream))
    _check(rc, "oscar_bf16_decode_attn")
    return out


def debug_dump(cache: Cache, b: int, h: int, cap_tokens: int | None = None, stream=None) -> dict:
    """oscar_debug_dump: layout-free host copy of one (sequence, kv head)."""
    cfg = cache.cfg
    cap = cap_tokens if cap_tokens is not None else cache.max_pages_per_seq * cfg.page_size
    d, R = cfg.head_dim, cfg.page_size
    out = {
        "k_codes": np.zeros((cap, d), np.uint8),
        "k_delta": np.zeros((cap // cfg.k_group, d), np.float32),
        "k_zero": np.zeros((cap // cfg.k_group, d), np.float32),
        "k_norm": np.zeros(cap, np.float32),
        "v_codes": np.zeros((cap, d), np.uint8),
        "v_delta": np.zeros((cap, d // cfg.v_group), np.float32),
        "v_zero": np.zeros((cap, d // cfg.v_group), np.float32),
        "res_k": np.zeros((R, d), np.float32),
        "res_v": np.zeros((R, d), np.float32),
        "res_norm": np.zeros(R, np.float32),
        "lens": np.zeros(2, np.int32),
    }
    order = ("k_codes", "k_delta", "k_zero", "k_norm", "v_codes", "v_delta", "v_zero", "res_k",
             "res_v", "res_norm", "lens")
    rc = lib().oscar_debug_dump(C.byref(cache.c), b, h, cap,
                                *[out[n].ctypes.data for n in order], _stream_ptr(stream))
    _check(rc, "oscar_debug_dump")
    return out
