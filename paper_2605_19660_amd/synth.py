"""Seeded synthetic KV-cache workloads.

Inputs only: this module holds none of OScaR's arithmetic (no rotation, scaling,
quantization or attention) and imports neither the HIP binding nor the oracle.
Both are fed the arrays it returns.

The workloads stand in for the long-context Qwen3-8B / Llama-3-8B decoding runs
and the multi-modal token-norm-imbalance patterns the paper measures on (its
efficiency section and its TNI observations: channel-wise key outliers,
low/high-norm outlier tokens, inter-modality norm gaps); real activations are
not available.  Recipe:

* base K, V ~ N(0,1) of shape [batch, tokens, n_kv_heads, head_dim];
* a few outlier channels per KV head multiply K and V by a constant;
* a per-(sequence, token) norm multiplier m_t, shared by heads and by K and V:
  LogNormal(0, sigma), optionally times a per-segment modality scale;
* queries ~ N(0,1);
* everything rounded once to the workload's input dtype and returned as fp32
  arrays holding exactly representable values.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

SEED_BASE = 0x05CA2000


@dataclass(frozen=True)
class Workload:
    name: str
    config_id: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    context: int
    io_dtype: str            # "f32" | "bf16" | "f16"
    bits: int = 2
    k_group: int = 128
    v_group: int = 32
    page_size: int = 128
    meta_dtype: str = "f16"  # "f16" | "f32"
    outlier_channels: tuple = ()      # fixed channels (same for every head); empty = seeded per head
    n_outliers: int = 4
    outlier_gain: float = 8.0
    norm_sigma: float = 0.7
    segments: bool = False            # modality segments with scales {1, 5, 0.3}
    segment_scales: tuple = (1.0, 5.0, 0.3)
    segment_len: tuple = (1024, 8192)

    @property
    def seed(self) -> int:
        return SEED_BASE + self.config_id

    def replace(self, **kw) -> "Workload":
        import dataclasses
        return dataclasses.replace(self, **kw)


# The five configurations the benchmark description names.
TINY = Workload("tiny", 0, 1, 1, 1, 128, 512, "f32", meta_dtype="f32",
                outlier_channels=(3, 17, 64, 100), outlier_gain=10.0, norm_sigma=0.5)
LLAMA8B_32K = Workload("llama3-8b-like-b8-s32k", 1, 8, 32, 8, 128, 32768, "bf16")
LONG_128K = Workload("long-b1-s128k", 2, 1, 32, 8, 128, 131072, "bf16")
HIGH_BATCH_8K = Workload("highbatch-b64-s8k", 3, 64, 32, 8, 128, 8192, "bf16")
OMNI_64K = Workload("omni-b4-g7-s64k", 4, 4, 28, 4, 128, 65536, "bf16", segments=True)
CONFIGS = (TINY, LLAMA8B_32K, LONG_128K, HIGH_BATCH_8K, OMNI_64K)


def round_to_dtype(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp32 values to `dtype` (nearest even) and widen back to fp32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f32":
        return x
    if dtype == "f16":
        return x.astype(np.float16).astype(np.float32)
    if dtype == "bf16":
        u = x.view(np.uint32).astype(np.uint64)
        u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
        return u.astype(np.uint32).view(np.float32).reshape(x.shape)
    raise ValueError(dtype)


def outlier_channel_table(w: Workload) -> np.ndarray:
    """[n_kv_heads, n_outliers] channel indices."""
    if w.outlier_channels:
        return np.tile(np.asarray(w.outlier_channels, np.int64), (w.n_kv_heads, 1))
    rng = np.random.default_rng([w.seed, 0xC4A])
    return np.stack([rng.choice(w.head_dim, size=w.n_outliers, replace=False)
                     for _ in range(w.n_kv_heads)])


def token_multipliers(w: Workload, b: int, start: int, count: int) -> np.ndarray:
    """Norm multiplier m_t of tokens [start, start+count) of sequence b (fp32)."""
    total = w.context + 8192
    assert start + count <= total, "window beyond the generated horizon"
    rng = np.random.default_rng([w.seed, 0x70C, b])
    m = np.exp(rng.normal(0.0, w.norm_sigma, size=total)).astype(np.float32)
    if w.segments:
        srng = np.random.default_rng([w.seed, 0x5E6, b])
        seg = np.empty(total, np.float32)
        pos, kind = 0, 0
        while pos < total:
            ln = int(srng.integers(w.segment_len[0], w.segment_len[1] + 1))
            seg[pos:pos + ln] = w.segment_scales[kind % len(w.segment_scales)]
            pos += ln
            kind += 1
        m = m * seg
    return m[start:start + count]


def make_kv(w: Workload, b: int, start: int = 0, count: int | None = None,
            heads: slice | None = None):
    """K, V of tokens [start, start+count) of sequence b: fp32 [count, n_kv_heads, d]
    holding values exactly representable in w.io_dtype.  Deterministic in
    (workload seed, b, start-chunk); chunks are generated per 4096-token tile so any
    window can be produced without materialising the whole sequence."""
    count = w.context - start if count is None else count
    tile = 4096
    ch = outlier_channel_table(w)
    ks, vs = [], []
    t0 = (start // tile) * tile
    m_all = token_multipliers(w, b, t0, start + count - t0)
    for ts in range(t0, start + count, tile):
        rng = np.random.default_rng([w.seed, 0xDA7A, b, ts // tile])
        k = rng.standard_normal((tile, w.n_kv_heads, w.head_dim), dtype=np.float32)
        v = rng.standard_normal((tile, w.n_kv_heads, w.head_dim), dtype=np.float32)
        for h in range(w.n_kv_heads):
            k[:, h, ch[h]] *= np.float32(w.outlier_gain)
            v[:, h, ch[h]] *= np.float32(w.outlier_gain)
        m = m_all[ts - t0: ts - t0 + tile]
        if m.shape[0] < tile:
            k, v = k[:m.shape[0]], v[:m.shape[0]]
        k *= m[:, None, None]
        v *= m[:, None, None]
        lo, hi = max(start, ts) - ts, min(start + count, ts + tile) - ts
        ks.append(k[lo:hi])
        vs.append(v[lo:hi])
    k = np.concatenate(ks, axis=0)
    v = np.concatenate(vs, axis=0)
    if heads is not None:
        k, v = k[:, heads], v[:, heads]
    return round_to_dtype(k, w.io_dtype), round_to_dtype(v, w.io_dtype)


def make_kv_batch(w: Workload, start: int = 0, count: int | None = None):
    """[batch, count, n_kv_heads, d] K and V (small workloads only)."""
    ks, vs = zip(*(make_kv(w, b, start, count) for b in range(w.batch)))
    return np.stack(ks), np.stack(vs)


def make_q(w: Workload, step: int = 0) -> np.ndarray:
    """Queries [batch, n_q_heads, d] for decode step `step`."""
    rng = np.random.default_rng([w.seed, 0x9E7, step])
    q = rng.standard_normal((w.batch, w.n_q_heads, w.head_dim), dtype=np.float32)
    return round_to_dtype(q, w.io_dtype)


def cache_bytes_per_token_kvh(w: Workload) -> int:
    """Resident packed-cache bytes of one token of one KV head."""
    meta = 2 if w.meta_dtype == "f16" else 4
    d = w.head_dim
    codes = d * w.bits // 8
    k_meta = 2 * meta * d // w.k_group
    v_meta = 2 * meta * d // w.v_group
    return codes + k_meta + meta + codes + v_meta


def make_kv_device(w: Workload, device="cuda", b_range=None):
    """Full-size K, V on the GPU: torch tensors [batch, context, n_kv_heads, d] of the
    workload's io dtype.  Same recipe as make_kv (base N(0,1), outlier channels, per-token
    multipliers) but drawn with torch's seeded device generator so that hundreds of
    megabytes need not cross PCIe; a slice copied back to the host feeds the oracle."""
    import torch
    dt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[w.io_dtype]
    bs = range(w.batch) if b_range is None else b_range
    ch = torch.from_numpy(outlier_channel_table(w)).to(device)
    gain = torch.ones(w.n_kv_heads, w.head_dim, device=device)
    gain.scatter_(1, ch, float(w.outlier_gain))
    ks, vs = [], []
    for b in bs:
        gen = torch.Generator(device=device)
        gen.manual_seed(w.seed * 1000 + b)
        m = torch.from_numpy(token_multipliers(w, b, 0, w.context)).to(device)
        scale = m[:, None, None] * gain[None]
        k = torch.randn(w.context, w.n_kv_heads, w.head_dim, device=device, generator=gen)
        ks.append((k * scale).to(dt))
        v = torch.randn(w.context, w.n_kv_heads, w.head_dim, device=device, generator=gen)
        vs.append((v * scale).to(dt))
        del k, v
    return torch.stack(ks), torch.stack(vs)
