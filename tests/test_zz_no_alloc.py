"""oscar_decode_attn_noalloc (split-K partials in the library's own fixed device buffer) against
oscar_decode_attn (caller workspace): same kernels, so the outputs must be identical, on two
calls in a row, the second on a smaller input; oversized requests are refused."""
import numpy as np
import pytest

from paper_2605_19660_amd import synth

pytestmark = pytest.mark.gpu


def _setup(batch, hq, hkv, context, bits, pages):
    import torch
    from paper_2605_19660_amd import binding as ob
    w = synth.LLAMA8B_32K.replace(batch=batch, n_q_heads=hq, n_kv_heads=hkv, context=context, bits=bits)
    k, v = synth.make_kv_batch(w)
    q = synth.make_q(w)
    cfg = ob.Config(hq, hkv, bits=bits)
    c = ob.Cache(cfg, batch, pages)
    dev = lambda x: torch.from_numpy(np.ascontiguousarray(x)).cuda().to(torch.bfloat16).contiguous()
    ob.quantize_append(c, dev(k), dev(v), eager=True, max_seq_len_hint=0)
    return ob, torch, w, c, dev(q)


def test_noalloc_decode_equals_workspace_decode_twice_second_smaller():
    ob, torch, w1, c1, q1 = _setup(3, 16, 4, 128 * 20 + 77, 2, 22)
    _, _, w2, c2, q2 = _setup(1, 8, 2, 128 * 3 + 5, 4, 5)
    for (w, c, q, splits) in ((w1, c1, q1, 6), (w2, c2, q2, 2), (w1, c1, q1, 0)):
        want = ob.decode_attn(c, q, max_seq_len_hint=w.context, num_splits=splits)
        got = torch.full_like(want, float("nan"))
        free_before = torch.cuda.memory_allocated()
        ob.decode_attn_noalloc(c, q, got, max_seq_len_hint=w.context, num_splits=splits)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == free_before
        assert torch.equal(got, want), (w.name, splits, (got - want).abs().max().item())
    # a bf16 output buffer works as in the workspace call
    want16 = ob.decode_attn(c2, q2, out=torch.empty_like(q2), max_seq_len_hint=w2.context, num_splits=2)
    got16 = ob.decode_attn_noalloc(c2, q2, torch.empty_like(q2), max_seq_len_hint=w2.context, num_splits=2)
    assert torch.equal(got16, want16)


def test_noalloc_decode_rejects_partials_beyond_its_buffer():
    ob, torch, w, c, q = _setup(3, 16, 4, 128 * 2, 2, 3)
    out = torch.zeros(w.batch, w.n_q_heads, 128, dtype=torch.float32, device="cuda")
    too_many = 512                       # 3 * 16 * 512 * 520 B = 12.8 MB > 4 MiB
    assert ob.decode_workspace_bytes(c.cfg, w.batch, too_many) > ob.NOALLOC_SCRATCH_BYTES
    with pytest.raises(ob.OscarError) as e:
        ob.decode_attn_noalloc(c, q, out, max_seq_len_hint=w.context, num_splits=too_many)
    assert e.value.status == ob.ERR_WORKSPACE
    torch.cuda.synchronize()
    assert not out.any()                 # nothing was enqueued
