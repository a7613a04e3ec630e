"""GPU parity: the HIP library (through its C ABI) against the CPU oracle on the same
seeded inputs.  Encoder outputs (codes, Delta, zero-points, norms, residual) must be
bit-exact; decode outputs within rel-L2 <= 1e-3 and max-abs <= 5e-3 of the oracle on
the same cache."""
import numpy as np
import pytest

import oracle
from oracle import OracleCache, OracleConfig
from paper_2605_19660_amd import synth

pytestmark = pytest.mark.gpu

REL_L2 = 1e-3
MAX_ABS = 5e-3

DT = {"f32": 0, "bf16": 1, "f16": 2}


def _torch():
    import torch
    return torch


def _ob():
    from paper_2605_19660_amd import binding
    return binding


def to_dev(x, io):
    torch = _torch()
    dt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[io]
    return torch.from_numpy(np.ascontiguousarray(x)).to("cuda").to(dt).contiguous()


def make_pair(w: synth.Workload, cap_pages, page_perm=None, fused=True, zp_mode=0, norm_scope=0,
              rotation_off=False, scale="l2"):
    ob = _ob()
    import oracle as orc
    g_scale = {"l2": ob.SCALE_L2, "none": ob.SCALE_NONE, "max": ob.SCALE_MAX, "mean_abs": ob.SCALE_MEAN_ABS}[scale]
    o_scale = {"l2": orc.SCALE_L2, "none": orc.SCALE_NONE, "max": orc.SCALE_MAX, "mean_abs": orc.SCALE_MEAN_ABS}[scale]
    cfg = ob.Config(w.n_q_heads, w.n_kv_heads, w.head_dim, w.bits, w.k_group, w.v_group,
                    w.page_size, DT[w.io_dtype], DT[w.meta_dtype], zp_mode=zp_mode,
                    norm_scope=norm_scope, rotation=ob.ROTATION_OFF if rotation_off else ob.ROTATION_ON,
                    scale_mode=g_scale)
    g = ob.Cache(cfg, w.batch, cap_pages, page_perm=page_perm, fused=fused)
    o = OracleCache(OracleConfig(w.head_dim, w.bits, w.k_group, w.v_group, w.page_size,
                                 DT[w.meta_dtype], zp_mode=zp_mode, norm_scope=norm_scope,
                                 rotate=0 if rotation_off else 1, scale_mode=o_scale),
                    w.batch, w.n_kv_heads, (cap_pages + 1) * w.page_size)
    return g, o


def assert_cache_equal(g, o, w):
    ob = _ob()
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            d = ob.debug_dump(g, b, h)
            npk, nr = int(o.n_packed[b]), int(o.n_res[b])
            assert (int(d["lens"][0]), int(d["lens"][1])) == (npk + nr, nr), (b, h, d["lens"], npk, nr)
            ngk = npk // w.k_group
            for name, got, want in (
                    ("k_codes", d["k_codes"][:npk], o.k_codes[b, h, :npk]),
                    ("v_codes", d["v_codes"][:npk], o.v_codes[b, h, :npk]),
                    ("k_delta", d["k_delta"][:ngk], o.k_delta[b, h, :ngk]),
                    ("k_zero", d["k_zero"][:ngk], o.k_zero[b, h, :ngk]),
                    ("k_norm", d["k_norm"][:npk], o.k_norm[b, h, :npk]),
                    ("v_delta", d["v_delta"][:npk], o.v_delta[b, h, :npk]),
                    ("v_zero", d["v_zero"][:npk], o.v_zero[b, h, :npk]),
                    ("res_k", d["res_k"][:nr], o.res_k[b, h, :nr]),
                    ("res_v", d["res_v"][:nr], o.res_v[b, h, :nr]),
                    ("res_norm", d["res_norm"][:nr], o.res_norm[b, h, :nr])):
                if not np.array_equal(got, want):
                    bad = np.argwhere(got != want)
                    raise AssertionError(f"{name} differs at (b={b},h={h}): {len(bad)} of {got.size}; "
                                         f"first {bad[0]} got {got[tuple(bad[0])]} want {want[tuple(bad[0])]}")


def assert_decode_close(got, want):
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    rel = np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-30)
    mx = np.abs(got - want).max()
    assert rel <= REL_L2 and mx <= MAX_ABS, (rel, mx)


# ------------------------------------------------------------------ encoder --

def test_tiny_config_bitexact_encoder_and_decode():
    w = synth.TINY
    k, v = synth.make_kv_batch(w)
    q = synth.make_q(w)
    g, o = make_pair(w, 8)
    ob = _ob()
    ob.quantize_append(g, to_dev(k, w.io_dtype), to_dev(v, w.io_dtype), eager=True, max_seq_len_hint=0)
    o.append(k, v, eager=True)
    assert_cache_equal(g, o, w)
    out = ob.decode_attn(g, to_dev(q, w.io_dtype), max_seq_len_hint=w.context)
    assert_decode_close(out.cpu().numpy(), o.decode_attn(q))


@pytest.mark.parametrize("io,meta,bits,kg,vg", [
    ("bf16", "f16", 2, 128, 32),
    ("bf16", "f16", 4, 128, 32),
    ("bf16", "f16", 2, 32, 32),
    ("f16", "f16", 2, 64, 64),
    ("bf16", "f32", 4, 32, 128),
    ("f32", "f16", 2, 128, 128),
])
def test_prefill_bitexact_ragged(io, meta, bits, kg, vg):
    w = synth.LLAMA8B_32K.replace(batch=2, n_q_heads=8, n_kv_heads=2, context=128 * 5 + 37,
                                  io_dtype=io, meta_dtype=meta, bits=bits, k_group=kg, v_group=vg)
    k, v = synth.make_kv_batch(w)
    q = synth.make_q(w)
    g, o = make_pair(w, 8)
    ob = _ob()
    ob.quantize_append(g, to_dev(k, io), to_dev(v, io), eager=True, max_seq_len_hint=0)
    o.append(k, v, eager=True)
    assert_cache_equal(g, o, w)
    out = ob.decode_attn(g, to_dev(q, io), max_seq_len_hint=w.context)
    assert_decode_close(out.cpu().numpy(), o.decode_attn(q))


def test_prefill_on_a_grid_past_the_ticket_limit_then_single_tokens():
    """A prefill of more than 1024 workgroups updates the lengths with the second, small kernel
    (the library drops the ticket for such grids); the one-token appends behind it draw tickets
    again.  Lengths, every code and the residual must match the oracle after each of them."""
    ob = _ob()
    w = synth.LLAMA8B_32K.replace(batch=4, n_q_heads=32, n_kv_heads=8, context=128 * 40 + 37)
    assert w.n_kv_heads * ((128 + w.context) // 128) * w.batch > 1024
    k, v = synth.make_kv_batch(w)
    g, o = make_pair(w, 44)
    n0 = w.context - 2
    ob.quantize_append(g, to_dev(k[:, :n0], w.io_dtype), to_dev(v[:, :n0], w.io_dtype), eager=True,
                       max_seq_len_hint=0)
    o.append(k[:, :n0], v[:, :n0], eager=True)
    assert_cache_equal(g, o, w)
    assert int(g.tickets.item()) == 0
    for t in (n0, n0 + 1):
        ob.quantize_append(g, to_dev(k[:, t:t + 1], w.io_dtype), to_dev(v[:, t:t + 1], w.io_dtype))
        o.append(k[:, t:t + 1], v[:, t:t + 1])
        assert_cache_equal(g, o, w)
        assert int(g.tickets.item()) == 0
    q = synth.make_q(w)
    out = ob.decode_attn(g, to_dev(q, w.io_dtype), max_seq_len_hint=w.context)
    assert_decode_close(out.cpu().numpy(), o.decode_attn(q))
    assert int(g.dev_status.item()) == 0


def test_incremental_appends_deferred_flush_and_ragged_new_lens():
    """Mixed chunk sizes, per-sequence new_lens, flush of a full residual deferred to the
    next append (the block stays 16-bit through the attention in between)."""
    torch = _torch()
    ob = _ob()
    w = synth.LLAMA8B_32K.replace(batch=3, n_q_heads=12, n_kv_heads=3, context=700)
    k, v = synth.make_kv_batch(w)
    g, o = make_pair(w, 8)
    pos = np.zeros(w.batch, np.int64)
    steps = [(100, [100, 60, 0]), (28, [28, 28, 28]), (1, [1, 1, 1]), (130, [130, 40, 129]),
             (1, [0, 1, 1]), (256, [256, 200, 1]), (1, [1, 1, 1])]
    step_id = 0
    for T, lens in steps:
        kk = np.zeros((w.batch, T, w.n_kv_heads, w.head_dim), np.float32)
        vv = np.zeros_like(kk)
        for b in range(w.batch):
            kk[b, :lens[b]] = k[b, pos[b]:pos[b] + lens[b]]
            vv[b, :lens[b]] = v[b, pos[b]:pos[b] + lens[b]]
        nl = np.asarray(lens, np.int32)
        ob.quantize_append(g, to_dev(kk, w.io_dtype), to_dev(vv, w.io_dtype),
                           new_lens=torch.from_numpy(nl).cuda())
        o.append(kk, vv, new_lens=nl)
        pos += nl
        assert_cache_equal(g, o, w)
        q = synth.make_q(w, step_id)
        out = ob.decode_attn(g, to_dev(q, w.io_dtype), max_seq_len_hint=int(pos.max()))
        assert_decode_close(out.cpu().numpy(), o.decode_attn(q))
        step_id += 1
    assert int(g.dev_status.item()) == 0


@pytest.mark.parametrize("seed,bits,kg,vg,norm_all", [(0, 2, 128, 32, False), (1, 4, 32, 64, False),
                                                       (2, 2, 64, 128, True)])
def test_random_append_schedules(seed, bits, kg, vg, norm_all):
    """Seeded random schedules: chunk sizes from 1 to a few blocks, per-sequence lengths
    (zeros included), prefill and decode rules mixed.  After every call the whole cache state is
    bit-exact against the oracle; the decode is checked every few calls."""
    torch = _torch()
    ob = _ob()
    rng = np.random.default_rng(1000 + seed)
    w = synth.LLAMA8B_32K.replace(batch=3, n_q_heads=6, n_kv_heads=3, context=1500, bits=bits,
                                  k_group=kg, v_group=vg)
    k, v = synth.make_kv_batch(w)
    g, o = make_pair(w, 14, norm_scope=1 if norm_all else 0)
    pos = np.zeros(w.batch, np.int64)
    for call in range(24):
        T = int(rng.choice([1, 1, 2, 17, 127, 128, 129, 200, 300]))
        lens = [int(rng.integers(0, T + 1)) if rng.random() < 0.5 else T for _ in range(w.batch)]
        lens = [min(n, w.context - int(pos[b])) for b, n in enumerate(lens)]
        eager = bool(rng.random() < 0.4)
        kk = np.zeros((w.batch, T, w.n_kv_heads, w.head_dim), np.float32)
        vv = np.zeros_like(kk)
        for b in range(w.batch):
            kk[b, :lens[b]] = k[b, pos[b]:pos[b] + lens[b]]
            vv[b, :lens[b]] = v[b, pos[b]:pos[b] + lens[b]]
        nl = np.asarray(lens, np.int32)
        ob.quantize_append(g, to_dev(kk, w.io_dtype), to_dev(vv, w.io_dtype),
                           new_lens=torch.from_numpy(nl).cuda(), eager=eager)
        o.append(kk, vv, new_lens=nl, eager=eager)
        pos += nl
        assert_cache_equal(g, o, w)
        if call % 4 == 3:
            q = synth.make_q(w, call)
            out = ob.decode_attn(g, to_dev(q, w.io_dtype), max_seq_len_hint=max(1, int(pos.max())))
            assert_decode_close(out.cpu().numpy(), o.decode_attn(q))
    assert int(g.dev_status.item()) == 0


def test_empty_appends_change_nothing_even_on_a_full_residual():
    """A call that brings a sequence no token leaves it untouched under either rule: a full
    16-bit residual (completed by a decode-rule append) keeps waiting through prefill-rule calls
    with new_lens = 0 and through T = 0 calls, and is flushed by the next token."""
    torch = _torch()
    ob = _ob()
    w = synth.LLAMA8B_32K.replace(batch=2, n_q_heads=4, n_kv_heads=2, context=400)
    k, v = synth.make_kv_batch(w)
    g, o = make_pair(w, 5)
    kd, vd = to_dev(k, w.io_dtype), to_dev(v, w.io_dtype)
    ob.quantize_append(g, kd[:, :128].contiguous(), vd[:, :128].contiguous())     # residual full, not flushed
    o.append(k[:, :128], v[:, :128])
    assert_cache_equal(g, o, w)
    assert int(g.res_lens[0].item()) == 128
    nl = np.asarray([0, 5], np.int32)                                              # sequence 0 gets nothing
    ob.quantize_append(g, kd[:, 128:133].contiguous(), vd[:, 128:133].contiguous(), eager=True,
                       new_lens=torch.from_numpy(nl).cuda())
    o.append(k[:, 128:133], v[:, 128:133], new_lens=nl, eager=True)
    assert_cache_equal(g, o, w)
    assert g.res_lens.tolist() == [128, 5] and g.seq_lens.tolist() == [128, 133]
    ob.quantize_append(g, kd[:, :0].contiguous(), vd[:, :0].contiguous(), eager=True)   # T = 0
    o.append(k[:, :0], v[:, :0], eager=True)
    assert_cache_equal(g, o, w)
    nl = np.asarray([1, 0], np.int32)
    ob.quantize_append(g, kd[:, 128:129].contiguous(), vd[:, 128:129].contiguous(),
                       new_lens=torch.from_numpy(nl).cuda())
    o.append(k[:, 128:129], v[:, 128:129], new_lens=nl)
    assert_cache_equal(g, o, w)
    assert g.res_lens.tolist() == [1, 5] and g.seq_lens.tolist() == [129, 133]
    q = synth.make_q(w)
    out = ob.decode_attn(g, to_dev(q, w.io_dtype), max_seq_len_hint=133)
    assert_decode_close(out.cpu().numpy(), o.decode_attn(q))


def test_token_by_token_equals_bulk_on_gpu():
    ob = _ob()
    w = synth.LLAMA8B_32K.replace(batch=1, n_q_heads=4, n_kv_heads=1, context=300)
    k, v = synth.make_kv_batch(w)
    ga, o = make_pair(w, 4)
    gb, _ = make_pair(w, 4)
    kd, vd = to_dev(k, w.io_dtype), to_dev(v, w.io_dtype)
    ob.quantize_append(ga, kd, vd)                       # one deferred bulk call
    for t in range(w.context):
        ob.quantize_append(gb, kd[:, t:t + 1].contiguous(), vd[:, t:t + 1].contiguous())
    o.append(k, v)
    assert_cache_equal(ga, o, w)
    assert_cache_equal(gb, o, w)


# ------------------------------------------------------------------- decode --

@pytest.mark.parametrize("hq,hkv,bits", [(1, 1, 2), (8, 2, 2), (28, 4, 2), (16, 2, 4), (6, 2, 4)])
def test_decode_gqa_variants_split_and_page_permutation_invariance(hq, hkv, bits):
    ob = _ob()
    w = synth.OMNI_64K.replace(batch=2, n_q_heads=hq, n_kv_heads=hkv, context=128 * 9 + 77,
                               bits=bits, segment_len=(100, 400))
    k, v = synth.make_kv_batch(w)
    q = synth.make_q(w)
    rng = np.random.default_rng(3)
    perm = rng.permutation(2 * 12)
    g, o = make_pair(w, 12)
    gp, _ = make_pair(w, 12, page_perm=perm)
    kd, vd, qd = to_dev(k, w.io_dtype), to_dev(v, w.io_dtype), to_dev(q, w.io_dtype)
    ob.quantize_append(g, kd, vd, eager=True)
    ob.quantize_append(gp, kd, vd, eager=True)
    o.append(k, v, eager=True)
    want = o.decode_attn(q)
    outs = []
    for splits in (1, 2, 3, 5, 16):
        out = ob.decode_attn(g, qd, max_seq_len_hint=w.context, num_splits=splits).cpu().numpy()
        assert_decode_close(out, want)
        outs.append(out)
    for a in outs[1:]:
        assert np.abs(a - outs[0]).max() <= 2e-5 * max(1.0, np.abs(outs[0]).max())
    outp = ob.decode_attn(gp, qd, max_seq_len_hint=w.context, num_splits=3).cpu().numpy()
    assert np.array_equal(outp, outs[2])
    # a bf16 output buffer is the rounded fp32 result
    import torch
    ob16 = ob.decode_attn(g, qd, out=torch.empty_like(qd), max_seq_len_hint=w.context, num_splits=3)
    assert torch.equal(ob16.float().cpu(), torch.from_numpy(outs[2]).to(torch.bfloat16).float())


@pytest.mark.parametrize("seed", range(16))
def test_random_decode_configurations(seed):
    """Seeded random draws over the decode's whole argument space: GQA group, bits, group sizes
    (both kernels), element types, zero-point form, ablation switches, batch, ragged lengths
    (empty, residual-only and exact-page sequences included), a permuted block table and the
    split count.  Encoder bit-exact, decode within tolerance, every time."""
    torch = _torch()
    ob = _ob()
    rng = np.random.default_rng(7000 + seed)
    hkv = int(rng.choice([1, 2, 3]))
    gq = int(rng.choice([1, 2, 4, 5, 7, 8]))
    bits = int(rng.choice([2, 4]))
    kg, vg = [(128, 32), (32, 32), (128, 128), (64, 64), (32, 128)][int(rng.integers(5))]
    io, meta = [("bf16", "f16"), ("f16", "f16"), ("bf16", "f32"), ("f32", "f16")][int(rng.integers(4))]
    zp = int(rng.integers(2))
    rotation_off = bool(rng.random() < 0.25)
    scale = str(rng.choice(["l2", "l2", "l2", "max", "mean_abs", "none"]))
    norm_all = bool(scale == "l2" and rng.random() < 0.3)
    batch = int(rng.integers(1, 5))
    eager = bool(rng.random() < 0.7)
    splits = int(rng.choice([0, 1, 2, 3, 7, 16]))
    cap = 10
    w = synth.LLAMA8B_32K.replace(batch=batch, n_q_heads=hkv * gq, n_kv_heads=hkv, context=cap * 128 - 1,
                                  io_dtype=io, meta_dtype=meta, bits=bits, k_group=kg, v_group=vg)
    k, v = synth.make_kv_batch(w)
    q = synth.make_q(w, seed)
    perm = rng.permutation(batch * cap)
    g, o = make_pair(w, cap, page_perm=perm, zp_mode=zp, norm_scope=1 if norm_all else 0,
                     rotation_off=rotation_off, scale=scale)
    special = [0, 57, 128, 256, 1, 127, 129]
    lens = np.array([int(rng.choice(special)) if rng.random() < 0.4 else int(rng.integers(0, w.context + 1))
                     for _ in range(batch)], np.int32)
    T = max(1, int(lens.max()))
    ob.quantize_append(g, to_dev(k[:, :T], io), to_dev(v[:, :T], io), eager=eager,
                       new_lens=torch.from_numpy(lens).cuda(), max_seq_len_hint=0)
    o.append(k[:, :T], v[:, :T], new_lens=lens, eager=eager)
    assert_cache_equal(g, o, w)
    out = ob.decode_attn(g, to_dev(q, io), max_seq_len_hint=T, num_splits=splits).cpu().numpy()
    assert np.isfinite(out).all()
    assert_decode_close(out, o.decode_attn(q))
    assert int(g.dev_status.item()) == 0


@pytest.mark.parametrize("path", ["mfma", "generic"])
@pytest.mark.parametrize("scale", [0.03, 0.25])
def test_decode_custom_softmax_scale(path, scale, monkeypatch):
    """softmax_scale > 0 replaces 1/sqrt(d) in both decode kernels and in the comparator."""
    torch = _torch()
    ob = _ob()
    if path == "generic":
        _ob().debug_force_generic_decode(True)
    w = synth.LLAMA8B_32K.replace(batch=2, n_q_heads=8, n_kv_heads=2, context=128 * 4 + 33)
    k, v = synth.make_kv_batch(w)
    q = synth.make_q(w)
    g, o = make_pair(w, 6)
    ob.quantize_append(g, to_dev(k, w.io_dtype), to_dev(v, w.io_dtype), eager=True, max_seq_len_hint=0)
    o.append(k, v, eager=True)
    out = ob.decode_attn(g, to_dev(q, w.io_dtype), scale=scale, max_seq_len_hint=w.context).cpu().numpy()
    want = o.decode_attn(q, scale=scale)
    assert_decode_close(out, want)
    assert np.abs(want - o.decode_attn(q)).max() > 1e-2      # the scale matters on these inputs
    if path == "mfma":
        lens = torch.full((w.batch,), w.context, dtype=torch.int32, device="cuda")
        outp = ob.bf16_decode_attn(to_dev(q, w.io_dtype), to_dev(k, w.io_dtype), to_dev(v, w.io_dtype),
                                   lens, scale=scale).cpu().numpy()
        assert_decode_close(outp, oracle.plain_attn(q, k, v, scale=scale))


@pytest.mark.parametrize("gq", [4, 7])
@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("kg,vg", [(128, 32), (128, 64), (128, 128), (64, 32), (64, 64), (64, 128),
                                   (32, 32), (32, 64), (32, 128)])
def test_decode_every_group_size_combination(kg, vg, bits, gq):
    """All nine (G_k, G_v) pairs x INT2/INT4 x one and two head slots per lane group run on the
    matrix-core kernel: encoder bit-exact, decode within tolerance, with a non-empty residual
    and two splits."""
    ob = _ob()
    w = synth.LLAMA8B_32K.replace(batch=2, n_q_heads=2 * gq, n_kv_heads=2, context=128 * 5 + 70,
                                  bits=bits, k_group=kg, v_group=vg)
    k, v = synth.make_kv_batch(w)
    q = synth.make_q(w)
    g, o = make_pair(w, 8)
    ob.quantize_append(g, to_dev(k, w.io_dtype), to_dev(v, w.io_dtype), eager=True, max_seq_len_hint=0)
    o.append(k, v, eager=True)
    assert_cache_equal(g, o, w)
    out = ob.decode_attn(g, to_dev(q, w.io_dtype), max_seq_len_hint=w.context, num_splits=2)
    assert_decode_close(out.cpu().numpy(), o.decode_attn(q))


@pytest.mark.parametrize("bits", [2, 4])
def test_decode_long_stream_one_split_crosses_block_table_chunks(bits):
    """One split over 300 pages: every wave walks 75 pages, more than the 64 block-table entries
    it keeps in a register, with a shuffled block table; a full (deferred) residual on top."""
    ob = _ob()
    n_pages = 300
    w = synth.LLAMA8B_32K.replace(batch=1, n_q_heads=4, n_kv_heads=1, context=128 * n_pages + 128,
                                  bits=bits)
    k, v = synth.make_kv_batch(w)
    q = synth.make_q(w)
    rng = np.random.default_rng(11)
    g, o = make_pair(w, n_pages + 2, page_perm=rng.permutation(n_pages + 2))
    kd, vd = to_dev(k, w.io_dtype), to_dev(v, w.io_dtype)
    ob.quantize_append(g, kd, vd)          # deferred rule: the last 128 tokens stay 16-bit
    o.append(k, v)
    assert int(o.n_res[0]) == 128 and int(o.n_packed[0]) == 128 * n_pages
    want = o.decode_attn(q)
    for splits in (1, 2):
        out = ob.decode_attn(g, to_dev(q, w.io_dtype), max_seq_len_hint=w.context, num_splits=splits)
        assert_decode_close(out.cpu().numpy(), want)


@pytest.mark.parametrize("hq,hkv,bits,out_dt", [(8, 2, 2, "f32"), (28, 4, 2, "bf16"), (16, 2, 4, "f32")])
def test_single_split_writes_the_output_itself_with_the_bits_of_the_two_pass_route(hq, hkv, bits, out_dt):
    """One split: oscar_decode_attn lets the matrix-core kernel write `out` and launches no reduce
    pass.  The separate partial + reduce calls always go through the workspace; both routes must
    give the same bits, ragged lengths, an empty and a residual-only sequence included."""
    torch = _torch()
    ob = _ob()
    w = synth.LLAMA8B_32K.replace(batch=4, n_q_heads=hq, n_kv_heads=hkv, context=128 * 5 + 61, bits=bits)
    k, v = synth.make_kv_batch(w)
    g, o = make_pair(w, 8)
    nl = np.asarray([w.context, 128 * 2 + 3, 0, 77], np.int32)
    ob.quantize_append(g, to_dev(k, w.io_dtype), to_dev(v, w.io_dtype), eager=True,
                       new_lens=torch.from_numpy(nl).cuda(), max_seq_len_hint=0)
    o.append(k, v, new_lens=nl, eager=True)
    q = to_dev(synth.make_q(w), w.io_dtype)
    dt = {"f32": torch.float32, "bf16": torch.bfloat16}[out_dt]
    ws = torch.zeros(ob.decode_workspace_bytes(g.cfg, w.batch, 1), dtype=torch.uint8, device="cuda")
    direct = torch.full((w.batch, hq, w.head_dim), 7.0, dtype=dt, device="cuda")
    ob.decode_attn(g, q, out=direct, max_seq_len_hint=w.context, num_splits=1, workspace=ws)
    assert not ws.any().item(), "the single-split route left records in the workspace"
    two_pass = torch.full_like(direct, 9.0)
    ob.decode_attn_partial(g, q, ws, 1)
    ob.decode_attn_reduce(g, two_pass, ws, 1)
    assert torch.equal(direct.view(torch.uint8), two_pass.view(torch.uint8))
    assert not direct[2].any().item()                          # the empty sequence: zeros
    if out_dt == "f32":
        assert_decode_close(direct.cpu().numpy(), o.decode_attn(synth.make_q(w)))


@pytest.mark.parametrize("scale", [2.0 ** -12, 2.0 ** 6])
def test_decode_extreme_value_magnitudes(scale):
    """Values (and so their step sizes) far from 1: the per-page power-of-two operand scaling of
    the matrix-core path has to follow; tolerance relative to the output scale."""
    ob = _ob()
    w = synth.LLAMA8B_32K.replace(batch=2, n_q_heads=8, n_kv_heads=2, context=128 * 6 + 40, io_dtype="f16")
    k, v = synth.make_kv_batch(w)
    v = (v * scale).astype(np.float32)
    v = np.asarray(to_dev(v, "f16").float().cpu().numpy())     # what fp16 holds
    assert np.isfinite(v).all()
    q = synth.make_q(w)
    g, o = make_pair(w, 8)
    ob.quantize_append(g, to_dev(k, "f16"), to_dev(v, "f16"), eager=True)
    o.append(k, v, eager=True)
    assert_cache_equal(g, o, w)
    got = ob.decode_attn(g, to_dev(q, "f16"), max_seq_len_hint=w.context).cpu().numpy()
    want = o.decode_attn(q)
    assert_decode_close(got / scale, want / scale)


def test_decode_edge_cases_empty_residual_only_and_exact_pages():
    torch = _torch()
    ob = _ob()
    w = synth.LLAMA8B_32K.replace(batch=4, n_q_heads=8, n_kv_heads=2, context=256)
    k, v = synth.make_kv_batch(w)
    q = synth.make_q(w)
    g, o = make_pair(w, 4)
    lens = np.asarray([0, 5, 256, 128], np.int32)    # empty, residual only, two full pages, one page
    ob.quantize_append(g, to_dev(k, w.io_dtype), to_dev(v, w.io_dtype),
                       new_lens=torch.from_numpy(lens).cuda(), eager=True)
    o.append(k, v, new_lens=lens, eager=True)
    assert_cache_equal(g, o, w)
    want = o.decode_attn(q)
    assert not want[0].any()
    for splits in (1, 4):
        out = ob.decode_attn(g, to_dev(q, w.io_dtype), max_seq_len_hint=256, num_splits=splits).cpu().numpy()
        assert_decode_close(out, want)
        assert not out[0].any()


def test_capacity_and_argument_errors():
    torch = _torch()
    ob = _ob()
    w = synth.LLAMA8B_32K.replace(batch=1, n_q_heads=4, n_kv_heads=1, context=400)
    k, v = synth.make_kv_batch(w)
    g, o = make_pair(w, 2)                            # room for 2 pages + residual
    kd, vd = to_dev(k, w.io_dtype), to_dev(v, w.io_dtype)
    with pytest.raises(ob.OscarError) as e:           # host-side check through the hint
        ob.quantize_append(g, kd, vd, eager=True, max_seq_len_hint=0)
    assert e.value.status == ob.ERR_CAPACITY
    ob.quantize_append(g, kd, vd, eager=True)         # no hint: the device guard drops it
    torch.cuda.synchronize()
    assert int(g.dev_status.item()) == ob.ERR_CAPACITY and int(g.seq_lens.item()) == 0
    ob.quantize_append(g, kd[:, :300].contiguous(), vd[:, :300].contiguous(), eager=True)
    o.append(k[:, :300], v[:, :300], eager=True)
    assert_cache_equal(g, o, w)
    q = to_dev(synth.make_q(w), w.io_dtype)
    with pytest.raises(ob.OscarError) as e:
        ob.decode_attn(g, q, max_seq_len_hint=300, num_splits=4,
                       workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert e.value.status == ob.ERR_WORKSPACE


@pytest.mark.parametrize("path", ["mfma", "generic"])
@pytest.mark.parametrize("fused", [True, False])
@pytest.mark.parametrize("hq,hkv,bits,kg,vg", [(8, 2, 2, 128, 32), (14, 2, 2, 32, 32),
                                              (16, 2, 4, 128, 128), (3, 1, 4, 128, 32)])
def test_decode_paths_and_fusion_agree_with_oracle(monkeypatch, path, fused, hq, hkv, bits, kg, vg):
    """Matrix-core and plain-ALU partial passes, with the length update of the appends folded
    into the append launch (ticket) or as a separate launch."""
    import torch
    ob = _ob()
    _ob().debug_force_generic_decode(path == "generic")
    w = synth.LLAMA8B_32K.replace(batch=2, n_q_heads=hq, n_kv_heads=hkv, context=128 * 6 + 100,
                                  bits=bits, k_group=kg, v_group=vg)
    k, v = synth.make_kv_batch(w)
    g, o = make_pair(w, 10, fused=fused)
    kd, vd = to_dev(k, w.io_dtype), to_dev(v, w.io_dtype)
    ob.quantize_append(g, kd[:, :700].contiguous(), vd[:, :700].contiguous(), eager=True)
    o.append(k[:, :700], v[:, :700], eager=True)
    for step in range(3):
        lo, hi = 700 + 56 * step, 700 + 56 * (step + 1)
        ob.quantize_append(g, kd[:, lo:hi].contiguous(), vd[:, lo:hi].contiguous())
        o.append(k[:, lo:hi], v[:, lo:hi])
        assert_cache_equal(g, o, w)
        q = synth.make_q(w, step)
        for splits in (1, 3):
            out = ob.decode_attn(g, to_dev(q, w.io_dtype), max_seq_len_hint=hi, num_splits=splits)
            assert_decode_close(out.cpu().numpy(), o.decode_attn(q))
    torch.cuda.synchronize()
    assert int(g.tickets.abs().sum().item()) == 0       # every ticket handed back


# ------------------------------------------------ float zero-point variant --

@pytest.mark.parametrize("io,meta,bits,kg,vg,path", [
    ("bf16", "f16", 2, 128, 32, "mfma"),
    ("bf16", "f16", 4, 32, 32, "mfma"),
    ("f16", "f16", 2, 128, 128, "generic"),
    ("f32", "f32", 4, 64, 64, "mfma"),      # fp32 metadata: the generic kernel either way
])
def test_float_zero_point_mode_bitexact_and_decode(io, meta, bits, kg, vg, path, monkeypatch):
    """zp_mode = ZP_MIN (zero-point = the group minimum, x = Delta*c + zero): encoder bit-exact,
    token-by-token appends included, and both decode kernels within tolerance."""
    ob = _ob()
    if path == "generic":
        _ob().debug_force_generic_decode(True)
    w = synth.LLAMA8B_32K.replace(batch=2, n_q_heads=8, n_kv_heads=2, context=128 * 3 + 61,
                                  io_dtype=io, meta_dtype=meta, bits=bits, k_group=kg, v_group=vg)
    k, v = synth.make_kv_batch(w)
    q = synth.make_q(w)
    g, o = make_pair(w, 8, zp_mode=ob.ZP_MIN)
    n0 = 128 * 2 + 17
    ob.quantize_append(g, to_dev(k[:, :n0], io), to_dev(v[:, :n0], io), eager=True, max_seq_len_hint=0)
    o.append(k[:, :n0], v[:, :n0], eager=True)
    for t in range(n0, w.context):      # crosses a page boundary: one deferred flush
        ob.quantize_append(g, to_dev(k[:, t:t + 1], io), to_dev(v[:, t:t + 1], io))
        o.append(k[:, t:t + 1], v[:, t:t + 1])
    assert_cache_equal(g, o, w)
    out = ob.decode_attn(g, to_dev(q, io), max_seq_len_hint=w.context)
    assert_decode_close(out.cpu().numpy(), o.decode_attn(q))


@pytest.mark.parametrize("io,meta,bits,kg,n_kv,zp", [
    ("bf16", "f16", 2, 128, 8, 0),
    ("f16", "f16", 4, 32, 3, 0),       # a head count that is no multiple of the fetch width
    ("f32", "f32", 2, 64, 1, 0),       # one head: the scope makes no difference
    ("bf16", "f16", 2, 128, 5, 1),
])
def test_norm_over_all_kv_heads_bitexact_and_decode(io, meta, bits, kg, n_kv, zp):
    """norm_scope = NORM_ALL_KV_HEADS (App. "Fused Hadamard-Norm Kernel"): one norm per token
    from the squared sums of all kv heads.  Prefill (whole blocks), a mixed block (old residual
    tokens + new ones), token-by-token appends with a deferred flush: cache bit-exact against
    the oracle, every head of a token holding the same norm; decode within tolerance."""
    ob = _ob()
    w = synth.LLAMA8B_32K.replace(batch=2, n_q_heads=2 * n_kv, n_kv_heads=n_kv, context=128 * 3 + 61,
                                  io_dtype=io, meta_dtype=meta, bits=bits, k_group=kg)
    k, v = synth.make_kv_batch(w)
    q = synth.make_q(w)
    g, o = make_pair(w, 8, zp_mode=zp, norm_scope=ob.NORM_ALL_KV_HEADS)
    n0, n1 = 128 + 17, 128 * 2 + 99
    ob.quantize_append(g, to_dev(k[:, :n0], io), to_dev(v[:, :n0], io), eager=True, max_seq_len_hint=0)
    o.append(k[:, :n0], v[:, :n0], eager=True)
    ob.quantize_append(g, to_dev(k[:, n0:n1], io), to_dev(v[:, n0:n1], io), eager=True)   # mixed block
    o.append(k[:, n0:n1], v[:, n0:n1], eager=True)
    for t in range(n1, w.context):      # crosses a page boundary: one deferred flush
        ob.quantize_append(g, to_dev(k[:, t:t + 1], io), to_dev(v[:, t:t + 1], io))
        o.append(k[:, t:t + 1], v[:, t:t + 1])
    assert_cache_equal(g, o, w)
    if n_kv > 1:
        d0, d1 = ob.debug_dump(g, 1, 0), ob.debug_dump(g, 1, n_kv - 1)
        assert np.array_equal(d0["k_norm"], d1["k_norm"]) and np.array_equal(d0["res_norm"], d1["res_norm"])
    out = ob.decode_attn(g, to_dev(q, io), max_seq_len_hint=w.context)
    assert_decode_close(out.cpu().numpy(), o.decode_attn(q))


@pytest.mark.parametrize("rotation_off,scale,io,meta,bits,path", [
    (True, "none", "bf16", "f16", 2, "auto"),        # plain per-channel keys / per-token values
    (True, "l2", "bf16", "f16", 2, "auto"),          # scaling alone (matrix-core kernel)
    (True, "l2", "bf16", "f16", 2, "generic"),
    (False, "none", "f16", "f16", 2, "auto"),        # rotation alone
    (False, "max", "bf16", "f16", 4, "auto"),        # (matrix-core kernel)
    (False, "mean_abs", "bf16", "f16", 2, "auto"),
    (True, "mean_abs", "f32", "f32", 2, "auto"),
])
def test_ablation_switches_bitexact_and_decode(rotation_off, scale, io, meta, bits, path, monkeypatch):
    """App. "Ablation Study": rotation off (K and Q un-rotated), scaling off, and the maximum /
    mean-absolute-value coefficients.  Encoder bit-exact against the oracle with the same
    switches (prefill + token-by-token appends over a flush), decode in tolerance (the
    matrix-core kernel takes the cases whose keys are scaled into [-1, 1], the generic one the
    others)."""
    ob = _ob()
    if path == "generic":
        _ob().debug_force_generic_decode(True)
    w = synth.LLAMA8B_32K.replace(batch=2, n_q_heads=8, n_kv_heads=2, context=128 * 2 + 77,
                                  io_dtype=io, meta_dtype=meta, bits=bits)
    k, v = synth.make_kv_batch(w)
    q = synth.make_q(w)
    g, o = make_pair(w, 8, rotation_off=rotation_off, scale=scale)
    n0 = 128 + 101
    ob.quantize_append(g, to_dev(k[:, :n0], io), to_dev(v[:, :n0], io), eager=True, max_seq_len_hint=0)
    o.append(k[:, :n0], v[:, :n0], eager=True)
    for t in range(n0, w.context):
        ob.quantize_append(g, to_dev(k[:, t:t + 1], io), to_dev(v[:, t:t + 1], io))
        o.append(k[:, t:t + 1], v[:, t:t + 1])
    assert_cache_equal(g, o, w)
    out = ob.decode_attn(g, to_dev(q, io), max_seq_len_hint=w.context)
    assert_decode_close(out.cpu().numpy(), o.decode_attn(q))


# ----------------------------------------------------------------- graphs --

@pytest.mark.parametrize("path", ["mfma", "generic"])
def test_decode_step_replays_from_a_captured_graph(path, monkeypatch):
    """Sequence lengths live on the device and every entry point only enqueues, so a whole decode
    step (append one token, partial pass, reduce) can be captured once and replayed: 40 replays
    with fresh tokens and queries, eager work and synchronizations in between, each compared
    bit for bit with the same step run eagerly on a twin cache; the replays cross a residual
    flush.  At the end the replayed cache is bit-exact against the oracle."""
    torch = _torch()
    ob = _ob()
    if path == "generic":
        _ob().debug_force_generic_decode(True)
    n0, steps, splits = 128 * 2 + 100, 40, 3
    w = synth.LLAMA8B_32K.replace(batch=2, n_q_heads=8, n_kv_heads=2, context=n0 + steps)
    k, v = synth.make_kv_batch(w)
    kd, vd = to_dev(k, w.io_dtype), to_dev(v, w.io_dtype)
    gc, o = make_pair(w, 5)
    ec, _ = make_pair(w, 5)
    warm, _ = make_pair(w, 5)
    for c in (gc, ec, warm):
        ob.quantize_append(c, kd[:, :n0].contiguous(), vd[:, :n0].contiguous(), eager=True, max_seq_len_hint=0)
    o.append(k[:, :n0], v[:, :n0], eager=True)
    sk, sv = torch.zeros_like(kd[:, :1]).contiguous(), torch.zeros_like(vd[:, :1]).contiguous()
    sq = torch.zeros(w.batch, w.n_q_heads, 128, dtype=kd.dtype, device="cuda")
    ws = torch.empty(ob.decode_workspace_bytes(gc.cfg, w.batch, splits), dtype=torch.uint8, device="cuda")
    ws_e = torch.empty_like(ws)
    out_g = torch.zeros(w.batch, w.n_q_heads, 128, dtype=torch.float32, device="cuda")
    out_e = torch.zeros_like(out_g)

    def step(c, kk, vv, qq, wsp, out):
        ob.quantize_append(c, kk, vv)
        ob.decode_attn_partial(c, qq, wsp, splits)
        ob.decode_attn_reduce(c, out, wsp, splits)

    step(warm, sk, sv, sq, ws, out_g)          # every kernel loaded before the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(gc, sk, sv, sq, ws, out_g)
    # (the capture itself enqueued nothing: the cache is still at n0 tokens)
    torch.cuda.synchronize()
    assert int(gc.seq_lens[0].item()) == n0
    for t in range(steps):
        q = to_dev(synth.make_q(w, t), w.io_dtype)
        sk.copy_(kd[:, n0 + t:n0 + t + 1])
        sv.copy_(vd[:, n0 + t:n0 + t + 1])
        sq.copy_(q)
        graph.replay()
        step(ec, kd[:, n0 + t:n0 + t + 1].contiguous(), vd[:, n0 + t:n0 + t + 1].contiguous(), q, ws_e, out_e)
        torch.cuda.synchronize()
        assert torch.equal(out_g, out_e), t
        o.append(k[:, n0 + t:n0 + t + 1], v[:, n0 + t:n0 + t + 1])
    assert_cache_equal(gc, o, w)
    assert_decode_close(out_g.cpu().numpy(), o.decode_attn(synth.make_q(w, steps - 1)))


# -------------------------------------------------------------- comparator --

@pytest.mark.parametrize("io", ["bf16", "f16"])
def test_bf16_comparator_matches_plain_attention_oracle(io):
    torch = _torch()
    ob = _ob()
    w = synth.LLAMA8B_32K.replace(batch=3, n_q_heads=8, n_kv_heads=2, context=1000, io_dtype=io)
    k, v = synth.make_kv_batch(w)
    q = synth.make_q(w)
    lens = np.asarray([1000, 1, 517], np.int32)
    want = oracle.plain_attn(q, k, v, seq_lens=lens)
    for splits in (1, 7):
        out = ob.bf16_decode_attn(to_dev(q, io), to_dev(k, io), to_dev(v, io),
                                  torch.from_numpy(lens).cuda(), num_splits=splits).cpu().numpy()
        assert_decode_close(out, want)
        # same cache with each kv head's tokens contiguous
        kh = to_dev(k, io).permute(0, 2, 1, 3).contiguous()
        vh = to_dev(v, io).permute(0, 2, 1, 3).contiguous()
        out = ob.bf16_decode_attn(to_dev(q, io), kh, vh, torch.from_numpy(lens).cuda(),
                                  num_splits=splits, head_major=True).cpu().numpy()
        assert_decode_close(out, want)


@pytest.mark.parametrize("seed", range(6))
def test_bf16_comparator_random_shapes(seed):
    """Seeded random GQA groups, lengths (zero and one included), capacities that are no multiple
    of the kernel's token step, split counts and both layouts."""
    torch = _torch()
    ob = _ob()
    rng = np.random.default_rng(8100 + seed)
    hkv = int(rng.choice([1, 2, 4]))
    gq = int(rng.choice([1, 2, 4, 7, 8]))
    io = str(rng.choice(["bf16", "f16"]))
    batch = int(rng.integers(1, 5))
    S = int(rng.choice([1, 3, 64, 257, 1000, 1531]))
    w = synth.LLAMA8B_32K.replace(batch=batch, n_q_heads=hkv * gq, n_kv_heads=hkv, context=S, io_dtype=io)
    k, v = synth.make_kv_batch(w)
    q = synth.make_q(w, seed)
    lens = np.array([int(rng.choice([0, 1, S])) if rng.random() < 0.4 else int(rng.integers(0, S + 1))
                     for _ in range(batch)], np.int32)
    want = oracle.plain_attn(q, k, v, seq_lens=lens)
    splits = int(rng.choice([1, 2, 5, 16]))
    kd, vd = to_dev(k, io), to_dev(v, io)
    if rng.random() < 0.5:
        out = ob.bf16_decode_attn(to_dev(q, io), kd, vd, torch.from_numpy(lens).cuda(), num_splits=splits)
    else:
        out = ob.bf16_decode_attn(to_dev(q, io), kd.permute(0, 2, 1, 3).contiguous(),
                                  vd.permute(0, 2, 1, 3).contiguous(), torch.from_numpy(lens).cuda(),
                                  num_splits=splits, head_major=True)
    out = out.cpu().numpy()
    assert np.isfinite(out).all()
    assert_decode_close(out, want)


# ------------------------------------------------- full size, sampled check --

@pytest.mark.parametrize("wi,bits,samples", [
    (1, 2, ((0, 0), (3, 5), (7, 7))),        # Llama-3-8B-like, batch 8, 32K: the benchmark's workload
    (2, 2, ((0, 2), (0, 7))),                # batch 1, 128K
    (3, 4, ((0, 1), (41, 6), (63, 3))),      # batch 64, 8K, INT4
    (4, 2, ((1, 0), (3, 3))),                # omni-like, GQA 7, 64K
])
def test_full_size_configs_sampled_against_oracle(wi, bits, samples):
    """The benchmark's configurations at their full sizes, in the launch configuration the
    benchmark times (prefill of the whole context, then a few one-token decode appends, automatic
    split count): every encoder output of sampled (sequence, kv head) streams bit-exact, decode
    outputs of their query heads within tolerance."""
    torch = _torch()
    ob = _ob()
    w = synth.CONFIGS[wi].replace(bits=bits)
    kd, vd = synth.make_kv_device(w)
    qh = synth.make_q(w)
    n_extra = 37
    pages = (w.context + n_extra) // w.page_size + 2
    g, _ = make_pair(w, pages)
    ob.quantize_append(g, kd, vd, eager=True, max_seq_len_hint=0)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1234 + wi)
    dt = ob.torch_dtype(DT[w.io_dtype])
    ek = torch.randn(w.batch, n_extra, w.n_kv_heads, w.head_dim, device="cuda", generator=gen).to(dt)
    ev = torch.randn(w.batch, n_extra, w.n_kv_heads, w.head_dim, device="cuda", generator=gen).to(dt)
    for t in range(n_extra):
        ob.quantize_append(g, ek[:, t:t + 1].contiguous(), ev[:, t:t + 1].contiguous())
    out = ob.decode_attn(g, to_dev(qh, w.io_dtype), max_seq_len_hint=w.context + n_extra).cpu().numpy()
    gq = w.n_q_heads // w.n_kv_heads
    for (b, h) in samples:
        ks = torch.cat([kd[b, :, h], ek[b, :, h]]).float().cpu().numpy()[None, :, None, :]
        vs = torch.cat([vd[b, :, h], ev[b, :, h]]).float().cpu().numpy()[None, :, None, :]
        o = OracleCache(OracleConfig(w.head_dim, w.bits, w.k_group, w.v_group, w.page_size,
                                     DT[w.meta_dtype]), 1, 1, pages * w.page_size)
        o.append(ks[:, :w.context], vs[:, :w.context], eager=True)
        for t in range(w.context, w.context + n_extra):
            o.append(ks[:, t:t + 1], vs[:, t:t + 1])
        d = ob.debug_dump(g, b, h)
        npk, nr = int(o.n_packed[0]), int(o.n_res[0])
        assert (int(d["lens"][0]), int(d["lens"][1])) == (npk + nr, nr)
        assert np.array_equal(d["k_codes"][:npk], o.k_codes[0, 0, :npk])
        assert np.array_equal(d["v_codes"][:npk], o.v_codes[0, 0, :npk])
        assert np.array_equal(d["k_delta"][:npk // w.k_group], o.k_delta[0, 0, :npk // w.k_group])
        assert np.array_equal(d["k_zero"][:npk // w.k_group], o.k_zero[0, 0, :npk // w.k_group])
        assert np.array_equal(d["k_norm"][:npk], o.k_norm[0, 0, :npk])
        assert np.array_equal(d["v_delta"][:npk], o.v_delta[0, 0, :npk])
        assert np.array_equal(d["v_zero"][:npk], o.v_zero[0, 0, :npk])
        assert np.array_equal(d["res_k"][:nr], o.res_k[0, 0, :nr])
        assert np.array_equal(d["res_norm"][:nr], o.res_norm[0, 0, :nr])
        want = o.decode_attn(qh[b:b + 1, h * gq:(h + 1) * gq], nthreads=4)
        assert_decode_close(out[b, h * gq:(h + 1) * gq], want[0])
    del g, kd, vd
    torch.cuda.empty_cache()


# ------------------------------------------------------------- one-call step --

def test_decode_step_equals_append_then_decode_and_the_oracle():
    """oscar_decode_step = oscar_quantize_append of one token per sequence (decode rule) followed by
    oscar_decode_attn: identical outputs to the two calls on a twin cache over 140 steps (a
    deferred flush included), the cache bit-exact against the oracle, errors before any launch."""
    torch = _torch()
    ob = _ob()
    n0, steps, splits = 128 + 120, 140, 3
    w = synth.LLAMA8B_32K.replace(batch=2, n_q_heads=8, n_kv_heads=2, context=n0 + steps)
    k, v = synth.make_kv_batch(w)
    kd, vd = to_dev(k, w.io_dtype), to_dev(v, w.io_dtype)
    a, o = make_pair(w, 5)
    b, _ = make_pair(w, 5)
    for c in (a, b):
        ob.quantize_append(c, kd[:, :n0].contiguous(), vd[:, :n0].contiguous(), eager=True, max_seq_len_hint=0)
    o.append(k[:, :n0], v[:, :n0], eager=True)
    ws = torch.empty(ob.decode_workspace_bytes(a.cfg, w.batch, splits), dtype=torch.uint8, device="cuda")
    out_a = torch.zeros(w.batch, w.n_q_heads, 128, dtype=torch.float32, device="cuda")
    for t in range(steps):
        q = to_dev(synth.make_q(w, t), w.io_dtype)
        kt, vt = kd[:, n0 + t:n0 + t + 1].contiguous(), vd[:, n0 + t:n0 + t + 1].contiguous()
        ob.decode_step(a, kt, vt, q, out_a, ws, splits, n0 + t + 1)
        ob.quantize_append(b, kt, vt)
        out_b = ob.decode_attn(b, q, max_seq_len_hint=n0 + t + 1, num_splits=splits)
        assert torch.equal(out_a, out_b), t
        o.append(k[:, n0 + t:n0 + t + 1], v[:, n0 + t:n0 + t + 1])
        if t % 35 == 0 or t == steps - 1:
            assert_decode_close(out_a.cpu().numpy(), o.decode_attn(synth.make_q(w, t)))
    assert_cache_equal(a, o, w)
    # argument errors: nothing is enqueued, the cache does not move
    before = a.seq_lens.clone()
    with pytest.raises(ob.OscarError) as e:
        ob.decode_step(a, kt, vt, q, out_a, torch.empty(8, dtype=torch.uint8, device="cuda"), splits, n0 + steps + 1)
    assert e.value.status == ob.ERR_WORKSPACE
    with pytest.raises(ob.OscarError) as e:
        ob.decode_step(a, kt, vt, q, out_a, ws, splits, 0)
    assert e.value.status == ob.ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert torch.equal(a.seq_lens, before)


# --------------------------------------------------------------- multi-layer --

def test_three_layers_share_one_block_table():
    """A three-layer cache (pools [layer][page][kv head], per-layer lengths, ONE shuffled block
    table): every layer takes its own K, V (prefill, then decode steps in layer order: append and
    attend in layer 0 before layer 1 sees the token, with a flush on the way), and is compared
    with its own oracle cache: encoder outputs bit for bit, attention in tolerance.  Layers must
    not see each other's data although they share page numbers."""
    torch = _torch()
    ob = _ob()
    L, n0, steps = 3, 128 * 2 + 100, 40
    w = synth.LLAMA8B_32K.replace(batch=2, n_q_heads=8, n_kv_heads=2, context=n0 + steps)
    rng = np.random.default_rng(17)
    cfg = ob.Config(w.n_q_heads, w.n_kv_heads)
    ml = ob.MultiLayerCache(cfg, w.batch, 5, L, page_perm=rng.permutation(w.batch * 5))
    ks, vs, oracles = [], [], []
    for l in range(L):
        wl = w.replace(config_id=40 + l)               # different seed per layer
        k, v = synth.make_kv_batch(wl)
        ks.append(k)
        vs.append(v)
        oracles.append(OracleCache(OracleConfig(), w.batch, w.n_kv_heads, 6 * 128))
    for l in range(L):
        ob.quantize_append(ml.layer(l), to_dev(ks[l][:, :n0], w.io_dtype), to_dev(vs[l][:, :n0], w.io_dtype),
                           eager=True, max_seq_len_hint=0)
        oracles[l].append(ks[l][:, :n0], vs[l][:, :n0], eager=True)
    splits = 2
    ws = torch.empty(ob.decode_workspace_bytes(cfg, w.batch, splits), dtype=torch.uint8, device="cuda")
    out = torch.zeros(w.batch, w.n_q_heads, 128, dtype=torch.float32, device="cuda")
    for t in range(steps):
        for l in range(L):
            q = synth.make_q(w, 100 * l + t)
            ob.decode_step(ml.layer(l), to_dev(ks[l][:, n0 + t:n0 + t + 1], w.io_dtype),
                           to_dev(vs[l][:, n0 + t:n0 + t + 1], w.io_dtype), to_dev(q, w.io_dtype),
                           out, ws, splits, n0 + t + 1)
            oracles[l].append(ks[l][:, n0 + t:n0 + t + 1], vs[l][:, n0 + t:n0 + t + 1])
            if t % 13 == 0 or t == steps - 1:
                assert_decode_close(out.cpu().numpy(), oracles[l].decode_attn(q))
        # between layers of a step the lengths differ by one token
        assert ml.seq_lens[:, 0].tolist() == [n0 + t + 1] * L
    for l in range(L):
        assert_cache_equal(ml.layer(l), oracles[l], w)
    assert int(ml.dev_status.item()) == 0 and int(ml.tickets.abs().sum().item()) == 0
    # the helper rejects what it cannot slice
    import ctypes as C
    view = ob.CCache()
    assert ob.lib().oscar_cache_layer(C.byref(ml._c), L, L, C.byref(view)) == ob.ERR_INVALID_ARG
    assert ob.lib().oscar_cache_layer(C.byref(ml._c), 0, 0, C.byref(view)) == ob.ERR_INVALID_ARG


def test_cache_state_is_its_buffers_copy_and_resume():
    """Checkpoint and resume: the whole state of a cache is the bytes of its buffers (pools,
    residual window, lengths, block table).  Copied through host memory into a second cache's
    freshly allocated buffers, it decodes to the same bits, and both caches stay identical bit for
    bit through further decode steps, a page flush included; the resumed one still matches the
    oracle."""
    torch = _torch()
    ob = _ob()
    n0, steps = 128 * 3 + 120, 20            # the flush comes 8 steps in
    w = synth.LLAMA8B_32K.replace(batch=3, n_q_heads=8, n_kv_heads=2, context=n0 + steps)
    k, v = synth.make_kv_batch(w)
    cfg = ob.Config(w.n_q_heads, w.n_kv_heads)
    perm = np.random.default_rng(5).permutation(w.batch * 6)
    a = ob.Cache(cfg, w.batch, 6, page_perm=perm)
    ref = OracleCache(OracleConfig(), w.batch, w.n_kv_heads, 6 * 128)
    ob.quantize_append(a, to_dev(k[:, :n0], w.io_dtype), to_dev(v[:, :n0], w.io_dtype), max_seq_len_hint=0)
    ref.append(k[:, :n0], v[:, :n0])
    names = ("k_codes", "k_meta", "k_norms", "v_codes", "v_meta", "res_k", "res_v", "res_norm",
             "block_table", "seq_lens", "res_lens")
    saved = {n: getattr(a, n).cpu().numpy().copy() for n in names}      # the checkpoint
    b = ob.Cache(cfg, w.batch, 6)
    for n in names:
        getattr(b, n).copy_(torch.from_numpy(saved[n]).to(getattr(b, n).device))
    splits = 2
    ws = torch.empty(ob.decode_workspace_bytes(cfg, w.batch, splits), dtype=torch.uint8, device="cuda")
    oa = torch.zeros(w.batch, w.n_q_heads, 128, dtype=torch.float32, device="cuda")
    obuf = torch.zeros_like(oa)
    for t in range(steps):
        q = to_dev(synth.make_q(w, 300 + t), w.io_dtype)
        kn, vn = to_dev(k[:, n0 + t:n0 + t + 1], w.io_dtype), to_dev(v[:, n0 + t:n0 + t + 1], w.io_dtype)
        ob.decode_step(a, kn, vn, q, oa, ws, splits, n0 + t + 1)
        ob.decode_step(b, kn, vn, q, obuf, ws, splits, n0 + t + 1)
        ref.append(k[:, n0 + t:n0 + t + 1], v[:, n0 + t:n0 + t + 1])
        assert np.array_equal(oa.cpu().numpy(), obuf.cpu().numpy()), t
    assert_decode_close(obuf.cpu().numpy(), ref.decode_attn(synth.make_q(w, 300 + steps - 1)))
    for n in names:
        assert np.array_equal(getattr(a, n).cpu().numpy(), getattr(b, n).cpu().numpy()), n
    assert_cache_equal(b, ref, w)
    assert int(b.dev_status.item()) == 0


@pytest.mark.parametrize("bits,context", [(2, 32768), (4, 16384)])
def test_decode_is_reproducible_launch_after_launch(bits, context):
    """The decode output of one cache and one query is the same bits on every launch, at a size
    that fills the chip (two workgroups per CU), with residual tokens, warm and cold.  (A build
    in which the output of an asm block had been placed on a register that a matrix instruction
    still in flight was going to write differed from launch to launch; the kernels keep such
    registers allocated now, and tests/test_asm_hazards.py scans the compiler's output for it.)"""
    torch = _torch()
    ob = _ob()
    w = synth.LLAMA8B_32K.replace(context=context, bits=bits)
    cfg = ob.Config(w.n_q_heads, w.n_kv_heads, bits=bits)
    kd, vd = synth.make_kv_device(w)
    c = ob.Cache(cfg, w.batch, context // 128 + 2)
    ob.quantize_append(c, kd, vd, eager=True, max_seq_len_hint=0)
    g = torch.Generator(device="cuda")
    g.manual_seed(5)
    for _ in range(37):
        kn = torch.randn(w.batch, 1, w.n_kv_heads, 128, device="cuda", generator=g).to(torch.bfloat16)
        vn = torch.randn(w.batch, 1, w.n_kv_heads, 128, device="cuda", generator=g).to(torch.bfloat16)
        ob.quantize_append(c, kn, vn, max_seq_len_hint=context + 64)
    del kd, vd
    q = to_dev(synth.make_q(w), w.io_dtype)
    splits = ob.decode_auto_splits(cfg, w.batch, context + 64)
    ws = torch.empty(ob.decode_workspace_bytes(cfg, w.batch, splits), dtype=torch.uint8, device="cuda")
    out = torch.empty(w.batch, w.n_q_heads, 128, dtype=torch.float32, device="cuda")
    junk = torch.empty(384 << 20, dtype=torch.uint8, device="cuda")
    first, differing = None, 0
    for i in range(60):
        if i % 4 == 0:
            junk.fill_(i & 255)            # push the cache out of the last-level cache now and then
        ob.decode_attn_partial(c, q, ws, splits)
        ob.decode_attn_reduce(c, out, ws, splits)
        o = out.clone()
        if first is None:
            first = o
        elif not torch.equal(o, first):
            differing += 1
    assert differing == 0
    assert int(c.dev_status.item()) == 0
