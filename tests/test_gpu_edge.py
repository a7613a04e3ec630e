"""GPU parity on the encoder's degenerate inputs, and a check of the published page layout that
does not go through oscar_debug_dump.

Degenerate inputs (Eq. 3-4 and App. "Quantization Format and Cache Organization" leave them to
the implementation; the readings are the oracle's): constant key channels and value groups
(Delta = 0 guard), an all-zero key token, inputs on exact rounding ties, a token norm beyond the
fp16 range, and nearly constant groups far from zero (integer zero-points in the thousands).
Every encoder output must be bit-exact against the oracle, then the decode within tolerance."""
import numpy as np
import pytest

from oracle import OracleCache, OracleConfig
from paper_2605_19660_amd import synth

from test_gpu_parity import (DT, REL_L2, MAX_ABS, _ob, _torch, assert_cache_equal,
                             assert_decode_close, make_pair, to_dev)

pytestmark = pytest.mark.gpu


def _degenerate_kv(w, rng):
    """K, V [batch, 3*128 + 40, n_kv, 128] with the special structures planted; values exactly
    representable in fp16 and bf16 alike unless noted."""
    T = 3 * 128 + 40
    k = rng.standard_normal((w.batch, T, w.n_kv_heads, 128)).astype(np.float32)
    v = rng.standard_normal((w.batch, T, w.n_kv_heads, 128)).astype(np.float32)
    k, v = synth.round_to_dtype(k, w.io_dtype), synth.round_to_dtype(v, w.io_dtype)
    # page 0 of sequence 0: one token repeated 128 times -> every key channel constant over the
    # group (and every value group repeated, but not constant inside a token)
    k[0, :128] = k[0, 0]
    v[0, :128] = v[0, 0]
    # page 1: an all-zero key token, a constant value group, an all-zero value group, a whole
    # all-zero value token
    k[0, 128 + 7] = 0.0
    v[0, 128 + 9, :, 32:64] = 0.75
    v[0, 128 + 10, :, 64:96] = 0.0
    v[0, 128 + 11] = 0.0
    # exact ties in a value group: multiples of 0.125 in [0, 0.75] -> Delta = 0.25, x/Delta on .5
    steps = np.array([0, 1, 2, 3, 4, 5, 6, 3, 1, 5, 0, 6, 2, 4, 3, 5] * 2, np.float32) * np.float32(0.125)
    v[0, 128 + 20, :, 0:32] = steps
    v[0, 128 + 21, :, 96:128] = -steps
    # residual part (tokens 384..): a zero key token and a constant value group there too
    k[0, 384 + 3] = 0.0
    v[0, 384 + 4, :, 0:32] = -2.5
    if w.batch > 1:
        # sequence 1: whole pages of zeros (keys and values)
        k[1, 128:256] = 0.0
        v[1, 128:256] = 0.0
    return k, v


@pytest.mark.parametrize("io,bits,kg,vg", [("bf16", 2, 128, 32), ("f16", 4, 32, 64), ("f16", 2, 64, 128)])
def test_degenerate_groups_zero_tokens_and_ties(io, bits, kg, vg):
    ob = _ob()
    rng = np.random.default_rng(4200 + bits + kg)
    w = synth.LLAMA8B_32K.replace(batch=2, n_q_heads=8, n_kv_heads=2, context=3 * 128 + 40,
                                  io_dtype=io, bits=bits, k_group=kg, v_group=vg)
    k, v = _degenerate_kv(w, rng)
    q = synth.make_q(w)
    for zp in (0, 1):
        g, o = make_pair(w, 5, zp_mode=zp)
        ob.quantize_append(g, to_dev(k, io), to_dev(v, io), eager=True, max_seq_len_hint=0)
        o.append(k, v, eager=True)
        assert_cache_equal(g, o, w)
        # what the readings promise, seen on the GPU's own cache
        d = ob.debug_dump(g, 0, 0)
        assert d["k_norm"][128 + 7] == 0.0 and d["res_norm"][3] == 0.0 and not d["res_k"][3].any()
        assert not d["k_codes"][:128].any()                      # constant channels: code 0 ...
        if zp == 0:
            kd0 = d["k_delta"][0]
            assert np.all(kd0 > 0)                               # ... and Delta = |value| (or 1)
        out = ob.decode_attn(g, to_dev(q, io), max_seq_len_hint=w.context).cpu().numpy()
        assert np.isfinite(out).all()
        assert_decode_close(out, o.decode_attn(q))


@pytest.mark.parametrize("bits", [2, 4])
def test_exact_ties_and_constant_channels_without_rotation(bits):
    """Rotation and scaling off, so that the planted key values reach the quantizer unchanged:
    channels on exact half-steps of Delta (round half to even decides every code), channels that
    are constant over a whole group (exact round trip), and nearly constant channels far from
    zero, whose integer zero-point is in the thousands (the packed words must still hold the
    codes of Eq. 3 bit for bit)."""
    ob = _ob()
    rng = np.random.default_rng(4300 + bits)
    qmax = 2 ** bits - 1
    w = synth.LLAMA8B_32K.replace(batch=1, n_q_heads=4, n_kv_heads=2, context=2 * 128 + 17,
                                  io_dtype="f16", bits=bits, k_group=128, v_group=32)
    T = w.context
    k = synth.round_to_dtype(rng.standard_normal((1, T, 2, 128)).astype(np.float32), "f16")
    v = synth.round_to_dtype(rng.standard_normal((1, T, 2, 128)).astype(np.float32), "f16")
    half = rng.integers(0, 2 * qmax + 1, size=(T, 2)).astype(np.float32) * np.float32(0.125)
    half[0], half[1] = 0.0, qmax * 0.25                          # range qmax/4 -> Delta = 0.25
    half[128], half[129] = 0.0, qmax * 0.25
    k[0, :, :, 5] = half                                         # ties: x/Delta in {0, .5, 1, ...}
    k[0, :, :, 6] = -half
    k[0, :, :, 40] = 0.3125                                      # constant channels
    k[0, :, :, 41] = 0.0
    k[0, :, :, 42] = -7.0
    tog = rng.integers(0, 2, size=(T, 2)).astype(np.float32)
    tog[0], tog[1], tog[128], tog[129] = 0, 1, 0, 1
    k[0, :, :, 70] = np.float32(0.5) + tog * np.float32(2.0 ** -11)      # z = -3072 (2-bit), -15360 (4-bit)
    k[0, :, :, 71] = np.float32(-3.0) - tog * np.float32(2.0 ** -9)
    k[0, :, :, 72] = np.float32(0.5) + tog * np.float32(2.0 ** -11)      # neighbours in one packed word
    # values: nearly constant groups far from zero (fp16 spacing at 100 is 1/16)
    v[0, :, :, 0:32] = np.float32(100.0) + rng.integers(0, 2, size=(T, 2, 32)).astype(np.float32) * np.float32(0.0625)
    v[0, :, 0, 0], v[0, :, 0, 1], v[0, :, 1, 0], v[0, :, 1, 1] = 100.0, 100.0625, 100.0, 100.0625
    v[0, :, :, 64:96] = np.float32(-512.0) - rng.integers(0, 3, size=(T, 2, 32)).astype(np.float32) * np.float32(0.5)
    q = synth.make_q(w) * np.float32(0.05)
    for meta in ("f16", "f32"):
        wm = w.replace(meta_dtype=meta)
        g, o = make_pair(wm, 4, rotation_off=True, scale="none")
        ob.quantize_append(g, to_dev(k, "f16"), to_dev(v, "f16"), eager=True, max_seq_len_hint=0)
        o.append(k, v, eager=True)
        assert_cache_equal(g, o, wm)
        d = ob.debug_dump(g, 0, 1)
        # the planted structure is really there: large zero-points, exact constants
        assert abs(d["k_zero"][0, 70]) >= 2048 and abs(d["v_zero"][0, 0]) >= 4096
        assert not d["k_codes"][:256, 40:43].any()
        kd, kz = d["k_delta"][0], d["k_zero"][0]
        for ch, val in ((40, 0.3125), (41, 0.0), (42, -7.0)):
            assert kd[ch] * (0 - kz[ch]) == val
        out = ob.decode_attn(g, to_dev(q, "f16"), max_seq_len_hint=T).cpu().numpy()
        want = o.decode_attn(q)
        scale = max(1.0, np.abs(want).max())
        assert_decode_close(out / scale, want / scale)


@pytest.mark.parametrize("io", ["bf16", "f16"])
def test_token_norm_beyond_fp16_range(io):
    """Keys whose norm exceeds 65504 with fp16 metadata: the stored norm saturates, K_u is the
    rotated key over the stored norm; encoder bit-exact (pages and residual), decode finite and
    within tolerance."""
    ob = _ob()
    w = synth.LLAMA8B_32K.replace(batch=2, n_q_heads=8, n_kv_heads=2, context=128 * 2 + 30, io_dtype=io)
    k, v = synth.make_kv_batch(w)
    k = k.copy()
    for (b, t, target) in ((0, 17, 7.0e4), (0, 200, 9.0e4), (1, 128 + 129, 6.6e4), (1, 5, 65510.0)):
        for h in range(w.n_kv_heads):
            k[b, t, h] *= np.float32(target / np.linalg.norm(k[b, t, h].astype(np.float64)))
    k = synth.round_to_dtype(k, io)
    assert np.isfinite(k).all()
    q = synth.make_q(w) * np.float32(2e-3)        # moderate logits in spite of the huge keys
    q = synth.round_to_dtype(q, io)
    g, o = make_pair(w, 4)
    ob.quantize_append(g, to_dev(k, io), to_dev(v, io), eager=True, max_seq_len_hint=0)
    o.append(k, v, eager=True)
    assert_cache_equal(g, o, w)
    d = ob.debug_dump(g, 0, 0)
    assert d["k_norm"][17] == 65504.0 and d["k_norm"][200] == 65504.0
    out = ob.decode_attn(g, to_dev(q, io), max_seq_len_hint=w.context).cpu().numpy()
    assert np.isfinite(out).all()
    assert_decode_close(out, o.decode_attn(q))


# --------------------------------------------------------------- page layout --

def _slot(bits, kk, e):
    """Code number inside a 32-code chunk of MFMA k-step kk, vector element e (formula printed in
    the header's description of v_codes / k_meta)."""
    if bits == 2:
        return 16 * (kk // 2) + 4 * (kk % 2) + e // 2 + 8 * (e % 2)
    return 8 * kk + e // 2 + 4 * (e % 2)


def _chunk_start(bits, tile, n, q4):
    return ((tile // 2) * 64 + n * 4 + q4) * 8 * bits + (tile % 2) * 4 * bits


def _code_at(raw, start, u, bits):
    bit = u * bits
    return (int(raw[start + bit // 8]) >> (bit % 8)) & ((1 << bits) - 1)


def _unpermute_page(raw, bits, kg, vg, meta_np):
    """One page of one kv head from raw pool bytes, following only the layout the header prints."""
    R = D = 128
    ngk, ngv = R // kg, D // vg
    kc = np.zeros((R, D), np.uint8)
    vc = np.zeros((R, D), np.uint8)
    for t in range(R):
        for j in range(D):
            kc[t, j] = _code_at(raw["k_codes"], _chunk_start(bits, t // 16, t % 16, j // 32), j % 32, bits)
    for c in range(D):
        for q4 in range(4):
            start = _chunk_start(bits, c // 16, c % 16, q4)
            for kk in range(4):
                for e in range(8):
                    vc[16 * e + 4 * kk + q4, c] = _code_at(raw["v_codes"], start, _slot(bits, kk, e), bits)
    km = raw["k_meta"].view(meta_np).astype(np.float32).reshape(2, ngk, D)
    kd = np.zeros((ngk, D), np.float32)
    kz = np.zeros((ngk, D), np.float32)
    for q4 in range(4):
        for kk in range(4):
            for e in range(8):
                pos, ch = 32 * q4 + 8 * kk + e, 32 * q4 + _slot(bits, kk, e)
                kd[:, ch] = km[0, :, pos]
                kz[:, ch] = km[1, :, pos]
    tpos = np.array([(t % 16) * 8 + t // 16 for t in range(R)])
    kn = raw["k_norms"].view(meta_np).astype(np.float32)[tpos]
    vm = raw["v_meta"].view(meta_np).astype(np.float32).reshape(2, ngv, R)
    vd = vm[0][:, tpos].T.copy()
    vz = vm[1][:, tpos].T.copy()
    return kc, kd, kz, kn, vc, vd, vz


@pytest.mark.parametrize("bits,kg,vg,meta", [(2, 128, 32, "f16"), (4, 32, 64, "f16"), (2, 64, 128, "f32"),
                                             (4, 128, 32, "f32")])
def test_published_page_layout_read_back_without_the_library(bits, kg, vg, meta):
    """The raw bytes of the five pools are copied to the host with torch and un-permuted in Python
    from the formulas printed in include/oscar.h alone (pool indexing [physical page][kv head],
    chunk offsets, code slots, metadata positions), with a shuffled block table; the result must
    equal the oracle's canonical cache."""
    ob = _ob()
    w = synth.LLAMA8B_32K.replace(batch=2, n_q_heads=6, n_kv_heads=3, context=128 * 3 + 11, bits=bits,
                                  k_group=kg, v_group=vg, meta_dtype=meta)
    k, v = synth.make_kv_batch(w)
    rng = np.random.default_rng(5)
    cap = 4
    perm = rng.permutation(w.batch * cap)
    g, o = make_pair(w, cap, page_perm=perm)
    ob.quantize_append(g, to_dev(k, w.io_dtype), to_dev(v, w.io_dtype), eager=True, max_seq_len_hint=0)
    o.append(k, v, eager=True)
    _torch().cuda.synchronize()
    meta_np = np.float16 if meta == "f16" else np.float32
    mb = 2 if meta == "f16" else 4
    per_page = {"k_codes": 128 * 128 * bits // 8, "k_meta": 2 * (128 // kg) * 128 * mb,
                "k_norms": 128 * mb, "v_codes": 128 * 128 * bits // 8, "v_meta": 2 * (128 // vg) * 128 * mb}
    assert sum(per_page.values()) == g.sizes.page_bytes_per_kv_head
    pools = {n: getattr(g, n).cpu().numpy() for n in per_page}
    table = g.block_table.cpu().numpy()
    assert np.array_equal(table.reshape(-1), perm[:w.batch * cap])
    n_pages = w.context // 128
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            for p in range(n_pages):
                unit = int(table[b, p]) * w.n_kv_heads + h
                raw = {n: pools[n][unit * per_page[n]:(unit + 1) * per_page[n]] for n in per_page}
                kc, kd, kz, kn, vc, vd, vz = _unpermute_page(raw, bits, kg, vg, meta_np)
                sl = slice(128 * p, 128 * (p + 1))
                gsl = slice((128 // kg) * p, (128 // kg) * (p + 1))
                assert np.array_equal(kc, o.k_codes[b, h, sl]), (b, h, p, "k_codes")
                assert np.array_equal(vc, o.v_codes[b, h, sl]), (b, h, p, "v_codes")
                assert np.array_equal(kd, o.k_delta[b, h, gsl]), (b, h, p, "k_delta")
                assert np.array_equal(kz, o.k_zero[b, h, gsl]), (b, h, p, "k_zero")
                assert np.array_equal(kn, o.k_norm[b, h, sl]), (b, h, p, "k_norms")
                assert np.array_equal(vd, o.v_delta[b, h, sl]), (b, h, p, "v_delta")
                assert np.array_equal(vz, o.v_zero[b, h, sl]), (b, h, p, "v_zero")
    # the residual, as documented: [sequence][kv head][R][d] fp16 K_u, io-dtype V, metadata norms
    nr = w.context % 128
    rk = g.res_k.view(_torch().float16).reshape(w.batch, w.n_kv_heads, 128, 128).float().cpu().numpy()
    rn = g.res_norm.view(_torch().float16 if meta == "f16" else _torch().float32) \
        .reshape(w.batch, w.n_kv_heads, 128).float().cpu().numpy()
    assert np.array_equal(rk[:, :, :nr], o.res_k[:, :, :nr])
    assert np.array_equal(rn[:, :, :nr], o.res_norm[:, :, :nr])
    assert g.seq_lens.tolist() == [w.context] * w.batch and g.res_lens.tolist() == [nr] * w.batch
