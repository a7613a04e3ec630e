"""The C-ABI library loads, exports every symbol the header declares, and its
host-only entry points behave (no GPU needed)."""
import ctypes as C
import os
import re

import pytest

from paper_2605_19660_amd import binding as ob

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "oscar.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(oscar_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    L = ob.lib()
    names = declared_symbols()
    assert set(names) == set(ob.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_version_and_status_strings():
    assert ob.lib().oscar_version() == 100
    assert ob.status_string(0) == "ok"
    for code in (-1, -2, -3, -4, -5):
        assert ob.status_string(code) not in ("ok", "unknown status")


def test_cache_sizes_match_the_format():
    cfg = ob.Config(32, 8)                     # INT2, G_k=128, G_v=32, fp16 metadata
    sz = ob.cache_sizes(cfg, 8, 16, 4)
    assert sz.page_bytes_per_kv_head == 11008 and sz.bytes_per_token_kv_head == 86
    assert sz.k_codes == 16 * 8 * 4096 and sz.v_meta == 16 * 8 * 2048
    assert sz.res_k == 8 * 8 * 128 * 128 * 2
    assert ob.cache_sizes(ob.Config(32, 8, bits=4), 1, 1, 1).bytes_per_token_kv_head == 150
    assert ob.cache_sizes(ob.Config(32, 8, k_group=32), 1, 1, 1).bytes_per_token_kv_head == 98
    assert ob.cache_sizes(ob.Config(1, 1, io_dtype=ob.F32, meta_dtype=ob.F32), 1, 1, 1).bytes_per_token_kv_head == 108


@pytest.mark.parametrize("kw,code", [
    (dict(head_dim=64), ob.ERR_UNSUPPORTED),
    (dict(bits=3), ob.ERR_UNSUPPORTED),
    (dict(zp_mode=7), ob.ERR_INVALID_ARG),
    (dict(bits=0), ob.ERR_INVALID_ARG),
    (dict(k_group=48), ob.ERR_INVALID_ARG),
    (dict(k_group=16), ob.ERR_UNSUPPORTED),
    (dict(norm_scope=5), ob.ERR_INVALID_ARG),
    (dict(rotation=2), ob.ERR_INVALID_ARG),
    (dict(scale_mode=4), ob.ERR_INVALID_ARG),
    (dict(norm_scope=ob.NORM_ALL_KV_HEADS, scale_mode=ob.SCALE_MAX), ob.ERR_UNSUPPORTED),
    (dict(n_q_heads=30), ob.ERR_INVALID_ARG),
    (dict(n_q_heads=128), ob.ERR_UNSUPPORTED),
    (dict(io_dtype=7), ob.ERR_INVALID_ARG),
])
def test_config_validation(kw, code):
    base = dict(n_q_heads=32, n_kv_heads=8)
    base.update(kw)
    with pytest.raises(ob.OscarError) as e:
        ob.cache_sizes(ob.Config(**base), 1, 1, 1)
    assert e.value.status == code


def test_null_arguments_are_rejected_before_any_launch():
    L = ob.lib()
    assert L.oscar_quantize_append(None, None, 1, None, None, -1, 0, None) == ob.ERR_INVALID_ARG
    assert L.oscar_decode_attn(None, None, None, 0, 0.0, 1, 1, None, 0, None) == ob.ERR_INVALID_ARG
    cc = ob.Config(32, 8).c()
    assert L.oscar_cache_sizes(C.byref(cc), 1, 1, 1, None) == ob.ERR_INVALID_ARG
    assert ob.decode_workspace_bytes(ob.Config(32, 8), 8, 16) == 8 * 32 * 16 * 130 * 4


def test_split_heuristic_and_host_side_argument_checks_of_the_aids():
    """Host logic that needs no GPU: the split count aims at one round of resident workgroups
    (two per CU, one for the register-hungry two-slot variants; 256 CUs assumed without a device)
    and never gives a wave fewer than two pages; the aids reject bad arguments before any launch."""
    L = ob.lib()
    assert ob.decode_auto_splits(ob.Config(32, 8), 8, 32768) == 8            # 512 / 64 units
    assert ob.decode_auto_splits(ob.Config(28, 4), 4, 65536) == 32           # 512 / 16 units (g = 7)
    assert ob.decode_auto_splits(ob.Config(28, 4, bits=4), 4, 65536) == 16   # that variant: one per CU
    assert ob.decode_auto_splits(ob.Config(32, 8), 1, 4096) == 4             # 32 pages / 8
    assert ob.decode_auto_splits(ob.Config(32, 8), 64, 8192) == 1
    assert ob.decode_auto_splits(ob.Config(32, 8), 1, 0) == 1
    assert L.oscar_rotate(None, None, None, 4, ob.BF16, ob.F16, 0, None) == ob.ERR_INVALID_ARG
    assert L.oscar_probe_stream_read(None, 1 << 20, 4, None, None, None) == ob.ERR_INVALID_ARG
    assert L.oscar_rotate_columns(None, None, 128, 4, ob.F32, None) == ob.ERR_INVALID_ARG
    assert L.oscar_timer_elapsed_us(None, None) == ob.ERR_INVALID_ARG
    assert L.oscar_timer_destroy(None) == ob.OK
    assert L.oscar_bf16_decode_attn(None, None, None, None, None, ob.BF16, ob.F32, 1, 128, 0, 8, 2, 128,
                                    0.0, 0, 1, None, 0, None) == ob.ERR_INVALID_ARG


def test_bench_refuses_more_than_one_gpu():
    """One GPU only: bench.py --gpus N with N above 1 exits with a message that says so."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_missing_library_fails_loudly(monkeypatch):
    """No CPU fallback: with no HIP library at the configured path the binding raises."""
    import importlib
    monkeypatch.setenv("OSCAR_HIP_LIB", "/nonexistent/liboscar_hip.so")
    mod = importlib.reload(importlib.import_module("paper_2605_19660_amd.binding"))
    try:
        with pytest.raises(ImportError):
            mod.lib()
    finally:
        monkeypatch.delenv("OSCAR_HIP_LIB")
        importlib.reload(mod)


def test_cache_layer_views_are_plain_pointer_arithmetic():
    """oscar_cache_layer (host only): layer l of a multi-layer allocation starts l whole per-layer
    pools into every pool and l * batch entries into the length arrays; block table and status
    word are shared; bad layer numbers are refused."""
    cfg = ob.Config(32, 8, bits=4, k_group=32)
    batch, pages, max_pages, L = 3, 24, 8, 5
    sz = ob.cache_sizes(cfg, batch, pages, max_pages)
    allc = ob.CCache()
    allc.cfg = cfg.c()
    allc.batch, allc.max_pages_per_seq, allc.num_pages = batch, max_pages, pages
    names = ("k_codes", "k_meta", "k_norms", "v_codes", "v_meta", "res_k", "res_v", "res_norm",
             "block_table", "seq_lens", "res_lens", "dev_status", "tickets")
    base = {n: 0x10000000 * (i + 1) for i, n in enumerate(names)}
    for n in names:
        setattr(allc, n, base[n])
    for layer in range(L):
        view = ob.CCache()
        assert ob.lib().oscar_cache_layer(C.byref(allc), L, layer, C.byref(view)) == ob.OK
        for n in ("k_codes", "k_meta", "k_norms", "v_codes", "v_meta", "res_k", "res_v", "res_norm",
                  "seq_lens", "res_lens", "tickets"):
            assert getattr(view, n) == base[n] + layer * getattr(sz, n), (n, layer)
        assert view.block_table == base["block_table"] and view.dev_status == base["dev_status"]
        assert (view.batch, view.max_pages_per_seq, view.num_pages) == (batch, max_pages, pages)
    assert sz.seq_lens == 4 * batch and sz.tickets == 4
    view = ob.CCache()
    for bad in (-1, L):
        assert ob.lib().oscar_cache_layer(C.byref(allc), L, bad, C.byref(view)) == ob.ERR_INVALID_ARG
    assert ob.lib().oscar_cache_layer(None, L, 0, C.byref(view)) == ob.ERR_INVALID_ARG
    allc.tickets = None                      # optional pointers stay NULL in the view
    assert ob.lib().oscar_cache_layer(C.byref(allc), L, 2, C.byref(view)) == ob.OK and not view.tickets


def test_time_stamped_variant_exports_the_same_entry_points_and_its_reader():
    """The library phase_profile.py runs (built by `build.py --stamps`) is the product library plus
    one reader for the stamps; no compute call here."""
    path = os.path.join(os.path.dirname(ob.LIB_PATH), "liboscar_hip_stamps.so")
    if not os.path.exists(path):
        pytest.skip("liboscar_hip_stamps.so not built (python -m paper_2605_19660_amd.build --stamps)")
    lib = C.CDLL(path)
    for name in ob.EXPORTS:
        assert hasattr(lib, name), name
    lib.oscar_debug_read_stamps.argtypes = [C.c_void_p, C.c_size_t]
    lib.oscar_debug_read_stamps.restype = C.c_int
    assert lib.oscar_debug_read_stamps(None, 0) == ob.ERR_INVALID_ARG
    assert not hasattr(ob.lib(), "oscar_debug_read_stamps")
