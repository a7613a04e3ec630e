"""Measurement aids of the C ABI (timer, timed partial pass, stream-read probe): they must
not change results and must reject what they cannot run."""
import numpy as np
import pytest

import oracle
from paper_2605_19660_amd import synth

pytestmark = pytest.mark.gpu


def _ob():
    from paper_2605_19660_amd import binding as ob
    return ob


def test_timed_partial_pass_matches_untimed_and_reports_a_duration():
    import torch
    ob = _ob()
    w = synth.LLAMA8B_32K.replace(batch=2, n_q_heads=8, n_kv_heads=2, context=128 * 9 + 50)
    io = {"bf16": ob.BF16, "f16": ob.F16, "f32": ob.F32}[w.io_dtype]
    cfg = ob.Config(w.n_q_heads, w.n_kv_heads, w.head_dim, w.bits, w.k_group, w.v_group,
                    w.page_size, io, ob.F16)
    k, v = synth.make_kv_batch(w)
    dt = ob.torch_dtype(io)
    c = ob.Cache(cfg, w.batch, 12)
    ob.quantize_append(c, torch.from_numpy(k).cuda().to(dt), torch.from_numpy(v).cuda().to(dt),
                       eager=True, max_seq_len_hint=0)
    q = torch.from_numpy(synth.make_q(w)).cuda().to(dt)
    splits = 3
    ws = torch.empty(ob.decode_workspace_bytes(cfg, w.batch, splits), dtype=torch.uint8, device="cuda")
    out_a = torch.empty(w.batch, w.n_q_heads, w.head_dim, dtype=torch.float32, device="cuda")
    out_b = torch.empty_like(out_a)
    ob.decode_attn_partial(c, q, ws, splits)
    ob.decode_attn_reduce(c, out_a, ws, splits)
    t = ob.Timer()
    with pytest.raises(ob.OscarError):      # nothing launched with it yet
        t.elapsed_us()
    ob.decode_attn_partial(c, q, ws, splits, timer=t)
    ob.decode_attn_reduce(c, out_b, ws, splits)
    us = t.elapsed_us()
    t.close()
    assert 0.0 < us < 1e5
    torch.cuda.synchronize()
    assert np.array_equal(out_a.cpu().numpy(), out_b.cpu().numpy())


def test_stream_read_probe_runs_and_rejects_ragged_sizes():
    import torch
    ob = _ob()
    buf = torch.ones(64 << 20, dtype=torch.uint8, device="cuda")
    t = ob.Timer()
    ob.probe_stream_read(buf, 32768 * 64 * 16, 64, timer=t)
    assert 0.0 < t.elapsed_us() < 1e5
    t.close()
    with pytest.raises(ob.OscarError) as e:
        ob.probe_stream_read(buf, 32768 * 64 + 1024, 64)
    assert e.value.status == ob.ERR_INVALID_ARG
    with pytest.raises(ob.OscarError):
        ob.probe_stream_read(buf, 32768 * 64, 0)


@pytest.mark.parametrize("io", ["bf16", "f16", "f32"])
def test_stand_alone_rotation_matches_oracle_transforms(io):
    """oscar_rotate: H(x)/sqrt(128) bit-exact against the oracle's query transform; with
    normalization, fp16 K_u and the stored norm bit-exact against its key transform (fp16 and
    fp32 norms); the reciprocal-square-root variant within one fp16 ulp / the norm's rounding."""
    import torch
    import oracle
    ob = _ob()
    rng = np.random.default_rng(1234)
    n_vec = 16 * 5 + 7                      # ragged: last workgroup partly empty
    x = rng.standard_normal((n_vec, 128)).astype(np.float32)
    x[:, [3, 77]] *= 9.0
    x *= np.exp(rng.normal(0.0, 0.7, (n_vec, 1))).astype(np.float32)
    x[5] = 0.0                              # zero vector: norm 0, K_u = 0
    dt = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}[io]
    xd = torch.from_numpy(x).cuda().to(dt).contiguous()
    xr = xd.float().cpu().numpy()           # the values the kernel sees
    got = ob.rotate(xd).cpu().numpy()
    want = np.stack([oracle.query_transform(v) for v in xr])
    assert np.array_equal(got, want)
    for meta, ometa in ((ob.F16, oracle.F16), (ob.F32, oracle.F32)):
        u, n = ob.rotate(xd, normalize=True, meta_dtype=meta)
        u, n = u.float().cpu().numpy(), n.float().cpu().numpy()
        ref = [oracle.key_transform(v, meta_dtype=ometa) for v in xr]
        assert np.array_equal(u, np.stack([r[0] for r in ref]))
        assert np.array_equal(n, np.asarray([r[1] for r in ref], np.float32))
    u2, n2 = ob.rotate(xd, normalize=True, fast_rsqrt=True)
    u2, n2 = u2.float().cpu().numpy(), n2.float().cpu().numpy()
    ref = [oracle.key_transform(v, meta_dtype=oracle.F16) for v in xr]
    u_ref = np.stack([r[0] for r in ref])
    n_ref = np.asarray([r[1] for r in ref], np.float32)
    # the exact mode divides by the stored (fp16-rounded) norm, the fast one by the unrounded one
    assert np.all(np.abs(u2 - u_ref) <= 2.0 ** -10 * np.abs(u_ref) + 2.0 ** -24)
    assert np.all(np.abs(n2 - n_ref) <= 2.0 ** -10 * n_ref)
    with pytest.raises(ob.OscarError):
        ob.rotate(xd, normalize=False, fast_rsqrt=True)


@pytest.mark.parametrize("io", ["bf16", "f16"])
def test_matrix_core_rotation_variant_within_tolerance(io):
    """OSCAR_ROTATE_MATRIX_CORE (App. "Fused Hadamard-Norm Kernel": H_128 = H_8 (x) H_16, the H_16
    factor on matrix tiles): the same rotation in another summation order, so parity is by
    tolerance, like the reciprocal-square-root mode: the plain rotation within fp32 rounding of
    the oracle's (and of the closed-form Hadamard product in double), normalized keys within one
    fp16 ulp, norms within one ulp of the storage type; fp32 input is refused."""
    import torch
    import oracle
    ob = _ob()
    rng = np.random.default_rng(4321)
    n_vec = 64 * 3 + 37                     # ragged: odd count, last workgroup partly empty
    x = rng.standard_normal((n_vec, 128)).astype(np.float32)
    x[:, [3, 77]] *= 9.0
    x *= np.exp(rng.normal(0.0, 0.7, (n_vec, 1))).astype(np.float32)
    x[5] = 0.0
    x[n_vec - 1] *= 100.0
    dt = {"bf16": torch.bfloat16, "f16": torch.float16}[io]
    xd = torch.from_numpy(x).cuda().to(dt).contiguous()
    xr = xd.float().cpu().numpy()
    got = ob.rotate(xd, matrix_core=True).cpu().numpy()
    want = np.stack([oracle.query_transform(v) for v in xr])
    i = np.arange(128)
    H = ((-1.0) ** np.array([[bin(a & b).count("1") for b in i] for a in i])) / np.sqrt(128.0)
    exact = xr.astype(np.float64) @ H.T
    scale = np.linalg.norm(xr.astype(np.float64), axis=1, keepdims=True) + 1e-30
    assert np.abs(got - exact).max() <= 1e-5 * np.abs(exact).max()
    assert (np.abs(got - exact) / scale).max() <= 4e-7          # fp32 accumulation of 128 exact terms
    assert (np.abs(got - want) / scale).max() <= 6e-7
    assert not got[5].any()
    for meta, ometa, ulp in ((ob.F16, oracle.F16, 2.0 ** -10), (ob.F32, oracle.F32, 2.0 ** -22)):
        for fast in (False, True):
            u, n = ob.rotate(xd, normalize=True, meta_dtype=meta, matrix_core=True, fast_rsqrt=fast)
            u, n = u.float().cpu().numpy(), n.float().cpu().numpy()
            ref = [oracle.key_transform(v, meta_dtype=ometa) for v in xr]
            u_ref = np.stack([r[0] for r in ref])
            n_ref = np.asarray([r[1] for r in ref], np.float32)
            assert np.all(np.abs(n - n_ref) <= ulp * n_ref), (meta, fast)
            # one fp16 ulp of the element, plus what the norm's own ulp moves it
            assert np.all(np.abs(u - u_ref) <= (2.0 ** -10 + 2 * ulp) * np.abs(u_ref) + 2.0 ** -24), (meta, fast)
            assert n[5] == 0.0 and not u[5].any()
    with pytest.raises(ob.OscarError) as e:
        ob.rotate(xd.float(), matrix_core=True)
    assert e.value.status == ob.ERR_UNSUPPORTED


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_weight_preprocessing_rotations(dt):
    """OScaR-Preprocess (Algorithm "The OScaR algorithm"): W_V <- W_V H and W_O <- H W_O, one H per
    head.  W_V H is oscar_rotate on the head segments of W_V's rows, H W_O is
    oscar_rotate_columns; both bit-exact against the oracle's butterfly, equal to the closed-form
    Hadamard product, and (X W_V H)(H W_O) = X W_V W_O (H is orthogonal and symmetric)."""
    import torch
    ob = _ob()
    rng = np.random.default_rng(3)
    d_model, n_kv, n_q = 192, 2, 4          # n_cols not a multiple of the 256-thread block
    tdt = {"f32": torch.float32, "bf16": torch.bfloat16}[dt]
    w_v = torch.from_numpy(rng.standard_normal((d_model, n_kv * 128)).astype(np.float32)).to(tdt)
    w_o = torch.from_numpy(rng.standard_normal((n_q * 128, d_model + 77)).astype(np.float32)).to(tdt)
    wv32, wo32 = w_v.float().numpy(), w_o.float().numpy()
    got_v = ob.rotate(w_v.cuda().reshape(d_model, n_kv, 128)).cpu().numpy().reshape(d_model, n_kv * 128)
    got_o = ob.rotate_columns(w_o.cuda()).cpu().numpy()
    want_v = oracle.fwht(wv32.reshape(d_model, n_kv, 128)).reshape(d_model, n_kv * 128)
    want_o = oracle.fwht(np.ascontiguousarray(wo32.T).reshape(-1, n_q, 128)).reshape(-1, n_q * 128).T
    assert np.array_equal(got_v, want_v)
    assert np.array_equal(got_o, want_o)
    i = np.arange(128)
    H = ((-1.0) ** np.array([[bin(a & b).count("1") for b in i] for a in i])) / np.sqrt(128)
    for h in range(n_q):
        blk = slice(128 * h, 128 * (h + 1))
        assert np.allclose(got_o[blk], H @ wo32[blk].astype(np.float64), rtol=1e-5, atol=1e-5)
    # the rotation cancels between the value projection and the output projection
    x = rng.standard_normal((5, d_model))
    g = n_q // n_kv
    v_plain = (x @ wv32.astype(np.float64)).reshape(5, n_kv, 128)
    v_rot = (x @ got_v.astype(np.float64)).reshape(5, n_kv, 128)
    mix = rng.random((n_q, 5, 5))
    mix /= mix.sum(-1, keepdims=True)        # stand-in for attention probabilities
    a_plain = np.concatenate([mix[h] @ v_plain[:, h // g] for h in range(n_q)], axis=1)
    a_rot = np.concatenate([mix[h] @ v_rot[:, h // g] for h in range(n_q)], axis=1)
    o_plain = a_plain @ wo32.astype(np.float64)
    o_rot = a_rot @ got_o.astype(np.float64)
    assert np.abs(o_rot - o_plain).max() <= 1e-4 * np.abs(o_plain).max()


def test_everything_runs_on_the_callers_stream():
    """Append, decode (both passes, timed and untimed) and rotation enqueued on a side stream
    (default priority) give the results of the default stream, and nothing runs before the side
    stream is released: the library only enqueues on the stream it is given."""
    import torch
    ob = _ob()
    w = synth.LLAMA8B_32K.replace(batch=2, n_q_heads=8, n_kv_heads=2, context=128 * 3 + 40)
    cfg = ob.Config(w.n_q_heads, w.n_kv_heads)
    k, v = synth.make_kv_batch(w)
    kd, vd = torch.from_numpy(k).cuda().bfloat16(), torch.from_numpy(v).cuda().bfloat16()
    q = torch.from_numpy(synth.make_q(w)).cuda().bfloat16()
    ref = ob.Cache(cfg, w.batch, 6)
    ob.quantize_append(ref, kd, vd, eager=True, max_seq_len_hint=0)
    want = ob.decode_attn(ref, q, max_seq_len_hint=w.context, num_splits=3)
    want_rot = ob.rotate(q)
    torch.cuda.synchronize()

    side = torch.cuda.Stream()
    c = ob.Cache(cfg, w.batch, 6)
    ws = torch.empty(ob.decode_workspace_bytes(cfg, w.batch, 3), dtype=torch.uint8, device="cuda")
    out = torch.zeros(w.batch, w.n_q_heads, 128, dtype=torch.float32, device="cuda")
    gate = torch.cuda.Event()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        # a long-running fill keeps the side stream busy while the calls below are enqueued
        big = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        for _ in range(8):
            big.fill_(1)
        ob.quantize_append(c, kd, vd, eager=True, max_seq_len_hint=0, stream=side)
        tm = ob.Timer()
        ob.decode_attn_partial(c, q, ws, 3, stream=side, timer=tm)
        ob.decode_attn_reduce(c, out, ws, 3, stream=side)
        rot = ob.rotate(q, stream=side)
        gate.record(side)
    gate.synchronize()
    assert tm.elapsed_us() > 0
    tm.close()
    assert torch.equal(out, want)
    assert torch.equal(rot, want_rot)
    assert torch.equal(c.seq_lens, ref.seq_lens) and torch.equal(c.res_lens, ref.res_lens)
    da, db = ob.debug_dump(c, 1, 1), ob.debug_dump(ref, 1, 1)
    npk = 128 * 3
    for name in ("k_codes", "v_codes", "k_norm", "v_delta"):
        assert np.array_equal(da[name][:npk], db[name][:npk]), name
