"""Measurement aids of the C ABI (timer, timed partial pass, stream-read probe): they must
not change results and must reject what they cannot run."""
import numpy as np
import pytest

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
