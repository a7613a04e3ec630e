#!/usr/bin/env python3
"""Benchmark of the OScaR hot path on one MI355X.

One "step" = one decode step of the whole hot path over the workload's batch:
  oscar_quantize_append of 1 new token per sequence (rotation, token scaling, residual
  append, block flush when due)  +  oscar_decode_attn over the packed + residual cache
  (query rotation, split-K partial pass, reduce pass).
The compressed cache was built beforehand by a timed oscar_quantize_append prefill of the
whole context, which is reported separately.  Everything is resident in HBM before the
timed region.  To keep the numbers HBM numbers and not Infinity-Cache numbers the steps
rotate over several independent cache copies (think: layers) whose total footprint exceeds
twice the 256 MB last-level cache.

Prints ONE JSON line: metric / value / unit / step counts / config, plus
  parity             a sampled (sequence, kv head) stream of the workload checked against the CPU
                     oracle before anything is timed (codes bit for bit, decode output in tolerance),
  roofline           the split-K partial kernel: algorithmic bytes per launch over its mean device
                     time (HIP events attached to every 5th dispatch of the timed region), against
                     8 TB/s; `traffic` = HBM bytes per launch from FETCH_SIZE / WRITE_SIZE counter runs,
  stream_read_probe  the same timing method on a loads-only kernel of the same launch shape,
  quantize_append_prefill, bf16_decode (the 16-bit comparator), cpu_baseline (the CPU oracle),
  other_workloads    compact records of the other configurations the benchmark description names
                     (batch 1 x 128K with its 131072-token prefill, batch 64 x 8K at INT2 and INT4
                     with tokens/s and resident bytes, the GQA-7 omni-like one), each from its own
                     short run (fixed 20 + 200 steps, whatever --steps says).
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X published HBM3E bandwidth
# HBM bytes per launch of the decode kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs,
# each scaled by the same counter's reading for a plain 256 MiB copy kernel (summary under
# profiles/); counters cannot be read from inside this process, so the figure is keyed by
# the workload it was measured on and reported as null for any other.
MEASURED_TRAFFIC = {("llama3-8b-like-b8-s32k", 2, 8): 182_300_126,
                    ("long-b1-s128k", 2, 64): 91_611_048,
                    ("omni-b4-g7-s64k", 2, 32): 92_713_848}
# The same kernel's mean duration over the decode steps in the committed `rocprofv3
# --kernel-trace` summaries (the dispatch's own begin/end timestamps), for comparison with the
# figure measured here: an event pair around a launch also holds the queue's hand-over from the
# event marker to the dispatch and reads 2-3 us more.  Keyed like MEASURED_TRAFFIC.
PROFILED_KERNEL_US = {("llama3-8b-like-b8-s32k", 2, 8): 33.13,
                      ("long-b1-s128k", 2, 64): 20.54,
                      ("omni-b4-g7-s64k", 2, 32): 25.54,
                      ("highbatch-b64-s8k", 2, 1): 67.12,
                      ("highbatch-b64-s8k", 4, 1): 117.32}


def profiled(w, splits, cache_bytes):
    us = PROFILED_KERNEL_US.get((w.name, w.bits, splits))
    if us is None:
        return None
    return {"avg_kernel_us": us, "frac": cache_bytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS,
            "summary": "profiles/decode_mfma_%s%s.txt" % (w.name, "-int4" if w.bits == 4 else ""),
            "what": "mean over the decode steps of a rocprofv3 kernel trace of this bench (dispatch timestamps)"}
# The encoder kernel alone on the whole-context prefill, median over the prefill launches in the
# same kernel trace (the call timed here also holds the length-update kernel behind it).
PROFILED_PREFILL_US = {("llama3-8b-like-b8-s32k", 2): 239.9}


def profiled_prefill(w, pre_bytes):
    us = PROFILED_PREFILL_US.get((w.name, w.bits))
    if us is None:
        return None
    return {"kernel_us": us, "frac": pre_bytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS,
            "summary": "profiles/quantize_append_%s.txt" % w.name}
EV_EVERY = 5                # every 5th launch of the decode kernel carries a HIP event pair (5 is
                            # coprime to the usual copy counts, so every cache copy gets sampled)
LLC_BYTES = 256 << 20       # Infinity Cache


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2048)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--workload", type=int, default=1, help="index into the five configurations")
    ap.add_argument("--bits", type=int, default=0, help="override bits (2|4)")
    ap.add_argument("--k-group", type=int, default=0, help="override G for keys (32|64|128 tokens)")
    ap.add_argument("--v-group", type=int, default=0, help="override G for values (32|64|128 channels)")
    ap.add_argument("--splits", type=int, default=0, help="override the split-K factor")
    ap.add_argument("--context", type=int, default=0, help="override the context length (multiple of 128)")
    ap.add_argument("--batch", type=int, default=0, help="override the batch size")
    ap.add_argument("--copies", type=int, default=0, help="override the number of cache copies")
    ap.add_argument("--norm-all-heads", action="store_true",
                    help="token norm over all kv heads instead of per (token, kv head)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-bf16", action="store_true")
    ap.add_argument("--no-extra-workloads", action="store_true",
                    help="skip the compact records of the other configurations")
    ap.add_argument("--no-parity", action="store_true", help="skip the in-run check against the oracle")
    ap.add_argument("--bf16-splits", type=int, default=0, help="override the comparator's split-K factor")
    ap.add_argument("--sweep", choices=["context", "batch"], default=None,
                    help="run the context sweep (batch 1) or the batch sweep (4K context) instead "
                         "of one workload; prints one JSON object with a list of points")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch a plain elementwise copy of 256 MiB five times, so that a "
                         "rocprofv3 --pmc run can scale FETCH_SIZE / WRITE_SIZE by a known size")
    return ap.parse_args()


def cpu_baseline(w, kd, vd, q_host, ob_cfg, budget_s=12.0):
    """The oracle, as it stands, on a bounded sample of the same workload: prefill-encode
    the sampled sequences, then time decode steps (append one token + attention) for about
    `budget_s` seconds."""
    import oracle
    nb = min(w.batch, 4)
    threads = max(1, min(oracle.max_threads(), os.cpu_count() or 1, 16))
    k = kd[:nb].float().cpu().numpy()
    v = vd[:nb].float().cpu().numpy()
    meta = {"f16": oracle.F16, "f32": oracle.F32}[w.meta_dtype]
    cache = oracle.OracleCache(oracle.OracleConfig(w.head_dim, w.bits, w.k_group, w.v_group,
                                                   w.page_size, meta, norm_scope=ob_cfg.norm_scope),
                               nb, w.n_kv_heads,
                               (w.context // w.page_size + 2) * w.page_size)
    t0 = time.perf_counter()
    cache.append(k, v, eager=True, nthreads=threads)
    t_enc = time.perf_counter() - t0
    n_steps, t_steps = 0, 0.0
    while n_steps < 64 and (n_steps == 0 or t_steps + t_steps / n_steps < budget_s):
        knew, vnew = k[:, n_steps:n_steps + 1].copy(), v[:, n_steps:n_steps + 1].copy()
        t0 = time.perf_counter()
        cache.append(knew, vnew, nthreads=threads)
        cache.decode_attn(q_host[:nb], nthreads=threads)
        t_steps += time.perf_counter() - t0
        n_steps += 1
    t_step = t_steps / n_steps
    scale = w.batch / nb
    return {
        "value": t_step * scale * 1e6, "unit": "us/step", "cores": threads, "kind": "oracle",
        "sample": f"{nb} of {w.batch} sequences x all {w.n_kv_heads} kv heads x full {w.context} "
                  f"context; {n_steps} decode steps timed ({t_step:.3f} s each) and scaled x{scale:g}; "
                  f"prefill encode of the sample took {t_enc:.2f} s "
                  f"({nb * w.context * w.n_kv_heads / t_enc / 1e6:.2f} M token-heads/s)",
    }


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2605_19660_amd import binding as ob, synth

    torch.cuda.set_device(0)
    w = synth.CONFIGS[args.workload]
    if args.bits:
        w = w.replace(bits=args.bits)
    if args.k_group or args.v_group:
        w = w.replace(k_group=args.k_group or w.k_group, v_group=args.v_group or w.v_group,
                      name="%s-gk%d-gv%d" % (w.name, args.k_group or w.k_group, args.v_group or w.v_group))
    if args.context or args.batch:
        w = w.replace(context=args.context or w.context, batch=args.batch or w.batch,
                      name="%s-b%d-s%d" % (w.name, args.batch or w.batch, args.context or w.context))
    if args.sweep:
        # the shape of the paper's efficiency figures: context sweep at batch 1, batch sweep at
        # 4K context, on the chosen workload's heads; one compact record per point
        base = w
        points = ([(1, s) for s in (1024, 4096, 16384, 32768, 65536, 131072)] if args.sweep == "context"
                  else [(b, 4096) for b in (1, 4, 16, 64, 128)])
        rows = []
        for (bb, ss) in points:
            wp = base.replace(batch=bb, context=ss, name="%s-b%d-s%d" % (base.name, bb, ss))
            r = compact_record(args, wp, np, torch, ob, synth, bf16=True)
            r.update({"batch": bb, "context": ss})
            rows.append(r)
            torch.cuda.empty_cache()
        print(json.dumps({"sweep": args.sweep, "workload": base.name, "bits": base.bits, "points": rows}))
        return
    res = measure(args, w, np, torch, ob, synth)
    if not args.no_extra_workloads and args.workload == 1 and not (args.bits or args.k_group or args.v_group
                                                                    or args.context or args.batch):
        torch.cuda.empty_cache()
        extra = []
        for (wi, bits) in ((2, 2), (3, 2), (3, 4), (4, 2)):
            extra.append(compact_record(args, synth.CONFIGS[wi].replace(bits=bits), np, torch, ob, synth))
            torch.cuda.empty_cache()
        # a scaling point beyond the named configurations: the headline workload's shape and batch
        # at the longest context of the paper's sweep (721 MB of cache per launch), where the
        # fixed cost of a launch is 5 % of the kernel instead of 15 %
        long_w = synth.CONFIGS[1].replace(name="llama3-8b-like-b8-s128k", context=131072)
        rec = compact_record(args, long_w, np, torch, ob, synth)
        rec["note"] = "scaling point, not one of the named configurations"
        extra.append(rec)
        torch.cuda.empty_cache()
        res["other_workloads"] = extra
    print(json.dumps(res))


def make_config(args, w, ob):
    io = {"f32": ob.F32, "bf16": ob.BF16, "f16": ob.F16}[w.io_dtype]
    meta = {"f32": ob.F32, "f16": ob.F16}[w.meta_dtype]
    return ob.Config(w.n_q_heads, w.n_kv_heads, w.head_dim, w.bits, w.k_group, w.v_group,
                     w.page_size, io, meta,
                     norm_scope=ob.NORM_ALL_KV_HEADS if args.norm_all_heads else ob.NORM_PER_HEAD), io


def build_caches(args, w, cfg, kd, vd, pages, n_copies, np, torch, ob, stream):
    """oscar_quantize_append prefill of the whole context into n_copies caches, then the same
    prefill timed: the copies are emptied (lengths to zero) and filled again, round after round
    for about 0.1 s, every launch between two events; the median of the second half is reported.
    (Timed once per freshly allocated cache, each launch followed allocations and a
    synchronization and ran on a GPU whose clocks had dropped; the refill writes the same bytes.)"""
    caches = []
    for ci in range(n_copies):
        c = ob.Cache(cfg, w.batch, pages)
        ob.quantize_append(c, kd, vd, eager=True, max_seq_len_hint=0, stream=stream)
        caches.append(c)
    torch.cuda.synchronize()
    t_pre = []
    t0 = time.perf_counter()
    while len(t_pre) < 4 * n_copies or (time.perf_counter() - t0 < 0.1 and len(t_pre) < 2000):
        evs = []
        for c in caches:
            c.seq_lens.zero_()
            c.res_lens.zero_()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            ob.quantize_append(c, kd, vd, eager=True, max_seq_len_hint=0, stream=stream)
            e1.record(stream)
            evs.append((e0, e1))
        torch.cuda.synchronize()
        t_pre += [a.elapsed_time(b) * 1e3 for a, b in evs]
    assert all(int(c.dev_status.item()) == 0 for c in caches)
    return caches, float(np.median(t_pre[len(t_pre) // 2:]))


def parity_check(w, cfg, cache, kd, vd, q, q_host, splits, np, torch, ob):
    """One sampled (sequence, kv head) stream of the workload against the CPU oracle, before any
    timing: every encoder output of the stream bit for bit, the decode output of its query heads
    within the stated tolerance (rel-L2 <= 1e-3, max-abs <= 5e-3)."""
    import oracle
    b, h = w.batch // 2, (w.n_kv_heads * 5) // 8
    meta = {"f16": oracle.F16, "f32": oracle.F32}[w.meta_dtype]
    o = oracle.OracleCache(oracle.OracleConfig(w.head_dim, w.bits, w.k_group, w.v_group, w.page_size, meta),
                           1, 1, (w.context // w.page_size + 1) * w.page_size)
    ks = kd[b, :, h].float().cpu().numpy()[None, :, None, :]
    vs = vd[b, :, h].float().cpu().numpy()[None, :, None, :]
    o.append(ks, vs, eager=True, nthreads=4)
    d = ob.debug_dump(cache, b, h)
    npk, nr = int(o.n_packed[0]), int(o.n_res[0])
    exact = (int(d["lens"][0]), int(d["lens"][1])) == (npk + nr, nr)
    for name, got, want in (("k_codes", d["k_codes"][:npk], o.k_codes[0, 0, :npk]),
                            ("v_codes", d["v_codes"][:npk], o.v_codes[0, 0, :npk]),
                            ("k_delta", d["k_delta"][:npk // w.k_group], o.k_delta[0, 0, :npk // w.k_group]),
                            ("k_zero", d["k_zero"][:npk // w.k_group], o.k_zero[0, 0, :npk // w.k_group]),
                            ("k_norm", d["k_norm"][:npk], o.k_norm[0, 0, :npk]),
                            ("v_delta", d["v_delta"][:npk], o.v_delta[0, 0, :npk]),
                            ("v_zero", d["v_zero"][:npk], o.v_zero[0, 0, :npk]),
                            ("res_k", d["res_k"][:nr], o.res_k[0, 0, :nr])):
        exact = exact and bool(np.array_equal(got, want))
    out = ob.decode_attn(cache, q, max_seq_len_hint=w.context, num_splits=splits).cpu().numpy()
    gq = w.n_q_heads // w.n_kv_heads
    want = o.decode_attn(q_host[b:b + 1, h * gq:(h + 1) * gq], nthreads=4)[0].astype(np.float64)
    got = out[b, h * gq:(h + 1) * gq].astype(np.float64)
    rel = float(np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-30))
    mx = float(np.abs(got - want).max())
    ok = bool(exact and rel <= 1e-3 and mx <= 5e-3)
    rec = {"checked": True, "passed": ok, "stream": {"sequence": b, "kv_head": h, "tokens": w.context},
           "encoder_bit_exact": bool(exact), "decode_rel_l2": rel, "decode_max_abs": mx,
           "tolerance": {"rel_l2": 1e-3, "max_abs": 5e-3}}
    if not ok:
        print(json.dumps({"error": "parity check against the oracle failed", "parity": rec}), file=sys.stderr)
        sys.exit(3)
    return rec


PREHEAT_S = 0.15


def preheat(caches, q, out, ws, splits, torch, ob, stream, seconds=PREHEAT_S):
    """Keeps the GPU busy with decode-attention launches (no appends: these are not steps) for
    `seconds` right before the warm-up steps.  After the host-side work that precedes the timed
    region (building inputs, the oracle check) the GPU has been idle for seconds and its clocks
    take tens of milliseconds of continuous work to come back up: measured here, the same kernel
    ran 15-30 % slower during the first ~30 ms after such a pause.  A decode loop in service never
    pauses like that, so the W warm-up steps and K timed steps start from a busy GPU."""
    n_copies = len(caches)
    t0 = time.perf_counter()
    i = 0
    while time.perf_counter() - t0 < seconds:
        for _ in range(32):
            ob.decode_attn_partial(caches[i % n_copies], q, ws, splits, stream=stream)
            ob.decode_attn_reduce(caches[i % n_copies], out, ws, splits, stream=stream)
            i += 1
        torch.cuda.synchronize()
    return i


def run_steps(args_steps, warmup, w, cfg, caches, q, new_k, new_v, out, ws, splits, np, torch, ob, stream):
    """warmup untimed steps, then exactly args_steps timed ones between synchronizations.  A step
    is one oscar_decode_step call (append one token per sequence + attention).  Every EV_EVERY-th
    step's partial kernel carries an event pair, whatever the step count."""
    n_copies = len(caches)
    hint = w.context + warmup + args_steps + 1

    def step(i, ev=None):
        ob.decode_step(caches[i % n_copies], new_k[i], new_v[i], q, out, ws, splits, hint,
                       stream=stream, timer=ev)

    # Everything the timed region needs on the host exists before the warm-up steps, so that
    # nothing but the synchronization separates the last warm-up step from the first timed one
    # (a GPU left idle for a few milliseconds runs the next kernels several per cent slower).
    # The first event-carrying launch of a process pays a one-time host cost (tens of ms when
    # the previous process's memory is still being reclaimed): it is taken in the warm-up.
    warm_ev = ob.Timer()
    evs = [ob.Timer() if i % EV_EVERY == 0 else None for i in range(args_steps)]
    g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    g0.record(stream)       # events are created at their first record: keep that, and whatever
    g1.record(stream)       # else a first use costs on the host, outside the timed region
    heat_launches = preheat(caches, q, out, ws, splits, torch, ob, stream)
    if warmup == 0:
        ob.decode_attn_partial(caches[0], q, ws, splits, stream=stream, timer=warm_ev)
    for i in range(warmup):
        step(i, warm_ev if i == 0 else None)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    g0.record(stream)
    for i in range(args_steps):
        step(warmup + i, evs[i])
    g1.record(stream)
    t_enq = time.perf_counter() - t0
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    k_samples = [e.elapsed_us() for e in evs if e is not None]
    for e in evs + [warm_ev]:
        if e is not None:
            e.close()
    assert all(int(c.dev_status.item()) == 0 for c in caches)
    return {"us_step": wall / args_steps * 1e6, "span_us": g0.elapsed_time(g1) * 1e3 / args_steps,
            "enqueue_us": t_enq / args_steps * 1e6, "k_us": float(np.mean(k_samples)),
            "k_samples": len(k_samples), "k_list": [round(x, 2) for x in k_samples[:64]],
            "preheat_launches": heat_launches}


def step_inputs(w, io, total_steps, torch, ob):
    gen = torch.Generator(device="cuda")
    gen.manual_seed(w.seed + 77)
    dt = ob.torch_dtype(io)
    new_k = torch.randn(total_steps, w.batch, 1, w.n_kv_heads, w.head_dim, device="cuda", generator=gen).to(dt)
    new_v = torch.randn(total_steps, w.batch, 1, w.n_kv_heads, w.head_dim, device="cuda", generator=gen).to(dt)
    return new_k, new_v


def compact_record(args, w, np, torch, ob, synth, bf16=False, steps=200, warmup=20):
    """One configuration in brief: timed whole-context prefill, then `steps` decode steps."""
    cfg, io = make_config(args, w, ob)
    R = w.page_size
    total = steps + warmup
    pages = (w.context + total) // R + 2
    stream = torch.cuda.current_stream()
    kd, vd = synth.make_kv_device(w)
    bytes_tok = synth.cache_bytes_per_token_kvh(w)
    units = w.batch * w.n_kv_heads * (w.context // R) * R
    cache_bytes = units * bytes_tok
    n_copies = min(32, max(2, math.ceil(2 * LLC_BYTES / cache_bytes) + 1))
    caches, pre_us = build_caches(args, w, cfg, kd, vd, pages, n_copies, np, torch, ob, stream)
    el = 2 if w.io_dtype != "f32" else 4
    pre_bytes = w.batch * w.n_kv_heads * w.context * (2 * w.head_dim * el) + units * bytes_tok
    new_k, new_v = step_inputs(w, io, total, torch, ob)
    q = torch.from_numpy(synth.make_q(w)).cuda().to(ob.torch_dtype(io)).contiguous()
    out = torch.empty(w.batch, w.n_q_heads, w.head_dim, dtype=torch.float32, device="cuda")
    splits = args.splits or ob.decode_auto_splits(cfg, w.batch, w.context + total)
    ws = torch.empty(ob.decode_workspace_bytes(cfg, w.batch, splits), dtype=torch.uint8, device="cuda")
    r = run_steps(steps, warmup, w, cfg, caches, q, new_k, new_v, out, ws, splits, np, torch, ob, stream)
    gbs = cache_bytes / (r["k_us"] * 1e-6) / 1e9
    rec = {"workload": w.name, "bits": w.bits, "batch": w.batch, "context": w.context,
           "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads, "splits": splits,
           "cache_copies_rotated": n_copies, "steps": steps, "warmup": warmup,
           "us_per_step": r["us_step"], "device_span_us_per_step": r["span_us"],
           "partial_us": r["k_us"], "hbm_gbs": gbs, "frac": gbs / HBM_PEAK_GBS,
           "algorithmic_bytes_per_launch": cache_bytes,
           "traffic": MEASURED_TRAFFIC.get((w.name, w.bits, splits)),
           "profiled": profiled(w, splits, cache_bytes),
           "decode_tokens_per_s": w.batch / (r["us_step"] * 1e-6),
           "resident_cache_bytes": cache_bytes, "cache_bytes_per_token_kv_head": bytes_tok,
           "prefill_tokens": w.batch * w.context, "prefill_us": pre_us,
           "prefill_hbm_gbs": pre_bytes / (pre_us * 1e-6) / 1e9,
           "prefill_frac": pre_bytes / (pre_us * 1e-6) / 1e9 / HBM_PEAK_GBS}
    if bf16 and w.io_dtype in ("bf16", "f16"):
        lens = torch.full((w.batch,), w.context, dtype=torch.int32, device="cuda")
        kh = kd.permute(0, 2, 1, 3).contiguous()
        vh = vd.permute(0, 2, 1, 3).contiguous()
        for _ in range(3):
            ob.bf16_decode_attn(q, kh, vh, lens, out=out, num_splits=splits, workspace=ws, stream=stream, head_major=True)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record(stream)
        for _ in range(20):
            ob.bf16_decode_attn(q, kh, vh, lens, out=out, num_splits=splits, workspace=ws, stream=stream, head_major=True)
        e1.record(stream)
        torch.cuda.synchronize()
        rec["bf16_us"] = e0.elapsed_time(e1) * 1e3 / 20
        del kh, vh
    del caches, kd, vd, new_k, new_v
    return rec


def measure(args, w, np, torch, ob, synth):
    cfg, io = make_config(args, w, ob)
    R = w.page_size
    total_steps = args.steps + args.warmup
    pages = (w.context + total_steps) // R + 2
    stream = torch.cuda.current_stream()

    kd, vd = synth.make_kv_device(w)
    bytes_tok = synth.cache_bytes_per_token_kvh(w)
    units = w.batch * w.n_kv_heads * (w.context // R) * R      # packed token-heads read per step
    cache_bytes = units * bytes_tok
    # (small caches: at most 32 copies, i.e. those points run warm in the last-level cache)
    n_copies = args.copies or min(32, max(2, math.ceil(2 * LLC_BYTES / cache_bytes) + 1))

    # ---- prefill: quantize_append of the whole context, timed per copy ----
    caches, pre_us = build_caches(args, w, cfg, kd, vd, pages, n_copies, np, torch, ob, stream)
    el = 2 if w.io_dtype != "f32" else 4
    pre_units = w.batch * w.n_kv_heads * w.context
    pre_bytes = pre_units * (2 * w.head_dim * el) + units * bytes_tok

    # ---- per-step inputs ----
    dt = ob.torch_dtype(io)
    new_k, new_v = step_inputs(w, io, total_steps, torch, ob)
    q_host = synth.make_q(w)
    q = torch.from_numpy(q_host).cuda().to(dt).contiguous()
    out = torch.empty(w.batch, w.n_q_heads, w.head_dim, dtype=torch.float32, device="cuda")
    splits = args.splits or ob.decode_auto_splits(cfg, w.batch, w.context + total_steps)
    ws = torch.empty(ob.decode_workspace_bytes(cfg, w.batch, splits), dtype=torch.uint8, device="cuda")

    # ---- parity first, then timing ----
    parity = None
    if not args.no_parity and not args.norm_all_heads:
        parity = parity_check(w, cfg, caches[0], kd, vd, q, q_host, splits, np, torch, ob)

    r = run_steps(args.steps, args.warmup, w, cfg, caches, q, new_k, new_v, out, ws, splits, np, torch, ob, stream)
    us_step, gpu_span_us, enqueue_us, k_us = r["us_step"], r["span_us"], r["enqueue_us"], r["k_us"]
    achieved = cache_bytes / (k_us * 1e-6) / 1e9

    # the same kernel timed on every launch of a separate, untimed-for-`value` region of decode
    # steps (cold: the copies keep rotating), for a steadier average than the few samples a short
    # timed region holds
    sep = []
    hint = w.context + total_steps + 1
    for i in range(48):
        t = ob.Timer()
        ob.decode_attn_partial(caches[i % n_copies], q, ws, splits, stream=stream, timer=t)
        ob.decode_attn_reduce(caches[i % n_copies], out, ws, splits, stream=stream)
        sep.append(t)
    torch.cuda.synchronize()
    sep_us = [t.elapsed_us() for t in sep]
    for t in sep:
        t.close()
    sep_us = float(np.mean(sep_us[8:]))

    # the same kernel on ONE cache copy, launched back to back: what it shows when whatever
    # fits of the cache stays in the 256 MB last-level cache (reported beside the cold figure)
    warm = []
    for i in range(24):
        t = ob.Timer()
        ob.decode_attn_partial(caches[0], q, ws, splits, stream=stream, timer=t)
        torch.cuda.synchronize()
        if i >= 8:
            warm.append(t.elapsed_us())
        t.close()
    warm_us = float(np.mean(warm))
    prop = torch.cuda.get_device_properties(0)
    if args.calibrate_copy:
        src = torch.zeros(64 << 20, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.add(src, 1, out=dst)          # reads 256 MiB, writes 256 MiB per launch
        torch.cuda.synchronize()
        del src, dst

    # ---- BF16 comparator on the same logical K, V (its 1 GB+ stream is already cold), in the
    # layout that suits it best: each kv head's tokens contiguous, as a paged 16-bit cache
    # stores them; the token-major figure (the layout K and V are produced in) is kept too ----
    bf16 = None
    if not args.no_bf16 and w.io_dtype in ("bf16", "f16"):
        lens = torch.full((w.batch,), w.context, dtype=torch.int32, device="cuda")
        bsplits = args.bf16_splits or ob.decode_auto_splits(cfg, w.batch, w.context)
        bws = torch.empty(ob.decode_workspace_bytes(cfg, w.batch, bsplits), dtype=torch.uint8, device="cuda")
        n_rep = max(5, min(50, args.steps // 4))
        b_bytes = w.batch * w.n_kv_heads * w.context * 2 * w.head_dim * 2

        def time_bf16(kk, vv, head_major):
            for _ in range(3):
                ob.bf16_decode_attn(q, kk, vv, lens, out=out, num_splits=bsplits, workspace=bws,
                                    stream=stream, head_major=head_major)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record(stream)
            for _ in range(n_rep):
                ob.bf16_decode_attn(q, kk, vv, lens, out=out, num_splits=bsplits, workspace=bws,
                                    stream=stream, head_major=head_major)
            e1.record(stream)
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e3 / n_rep

        tm_us = time_bf16(kd, vd, False)
        kh = kd.permute(0, 2, 1, 3).contiguous()
        vh = vd.permute(0, 2, 1, 3).contiguous()
        hm_us = time_bf16(kh, vh, True)
        del kh, vh
        b_us = min(tm_us, hm_us)
        bf16 = {"us_per_step": b_us, "hbm_gbs": b_bytes / (b_us * 1e-6) / 1e9, "splits": bsplits,
                "layout": "head-major" if hm_us <= tm_us else "token-major",
                "us_token_major": tm_us, "us_head_major": hm_us}

    # ---- what the same timing method shows for a pure streaming read of as many bytes ----
    # (the uncompressed K tensor serves as the source; windows rotate so the stream is cold)
    stream_read = None
    src_bytes = kd.numel() * kd.element_size()
    unit = 32768 * 512
    probe_bytes = min(cache_bytes, src_bytes // 3) // unit * unit
    if probe_bytes > 0:
        n_win = max(1, min(4, src_bytes // probe_bytes))
        kd_u8 = kd.view(torch.uint8).reshape(-1)
        ts = []
        for i in range(12):
            t = ob.Timer()
            win = kd_u8[(i % n_win) * probe_bytes:]
            ob.probe_stream_read(win, probe_bytes, 512, timer=t, stream=stream)
            us = t.elapsed_us()
            t.close()
            if i >= 4:
                ts.append(us)
        p_us = float(np.mean(ts))
        stream_read = {"bytes": probe_bytes, "us": p_us, "hbm_gbs": probe_bytes / (p_us * 1e-6) / 1e9,
                       "frac": probe_bytes / (p_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                       "what": "oscar_probe_stream_read: 512 workgroups x 256 threads, 1 KB wave loads, loads only"}

    # ---- stand-alone rotation + token scaling of all keys (kernel (i) on its own) ----
    rot = None
    if w.meta_dtype == "f16":
        def time_rotate(matrix_core):
            ts = []
            for i in range(4):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                ku, kn = ob.rotate(kd, normalize=True, stream=stream, matrix_core=matrix_core)
                e1.record(stream)
                torch.cuda.synchronize()
                if i:
                    ts.append(e0.elapsed_time(e1) * 1e3)
                del ku, kn
            return float(np.median(ts))
        r_us = time_rotate(False)
        r_bytes = pre_units * (w.head_dim * el + w.head_dim * 2 + 2)
        rot = {"vectors": pre_units, "us": r_us, "hbm_gbs": r_bytes / (r_us * 1e-6) / 1e9,
               "frac": r_bytes / (r_us * 1e-6) / 1e9 / HBM_PEAK_GBS, "algorithmic_bytes": r_bytes,
               "what": "oscar_rotate(NORMALIZE) on every key vector: read input, write fp16 K_u + norm "
                       "(includes the output allocation of the binding)"}
        if w.io_dtype in ("bf16", "f16"):
            m_us = time_rotate(True)
            rot["matrix_core_us"] = m_us
            rot["matrix_core_frac"] = r_bytes / (m_us * 1e-6) / 1e9 / HBM_PEAK_GBS

    res = {
        "metric": "int%d_decode_attn_us_per_step" % w.bits,
        "value": us_step, "unit": "us/step", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": us_step / 1e3, "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": "u%d codes, f32 accumulate" % w.bits,
        "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "n_q_heads": w.n_q_heads,
                   "n_kv_heads": w.n_kv_heads, "head_dim": w.head_dim, "context": w.context,
                   "bits": w.bits, "k_group": w.k_group, "v_group": w.v_group,
                   "io_dtype": w.io_dtype,
                   "norm_scope": "all kv heads" if args.norm_all_heads else "per kv head",
        "step": "oscar_decode_step: append 1 token/seq (1 launch) + decode attention (partial + reduce launches)",
                   "splits": splits, "cache_copies_rotated": n_copies},
        "roofline": {"bound": "hbm",
                     "kernel": ("oscar_decode_mfma_kernel" if w.meta_dtype == "f16"
                                else "oscar_decode_partial_kernel") + " (split-K partial pass)",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": MEASURED_TRAFFIC.get((w.name, w.bits, splits)),
                     "algorithmic_bytes_per_launch": cache_bytes,
                     "avg_kernel_us": k_us,
                     "profiled": profiled(w, splits, cache_bytes)},
        "paper_context": "the paper reports, end to end on Qwen3-8B with one NVIDIA H20 141 GB (INT2, G=32, "
                         "FP16 residual): up to 3.0x decode speedup at 128K context, 5.3x smaller memory "
                         "footprint and 4.1x throughput against BF16 FlashDecoding-v2; other hardware and an "
                         "end-to-end metric: context, not the target",
        "decode_tokens_per_s": w.batch / (us_step * 1e-6),
        "device_span_us_per_step": gpu_span_us,
        "host_enqueue_us_per_step": enqueue_us,
        "cache_bytes_per_token_kv_head": bytes_tok,
        "cache_bytes_per_token_all_heads": bytes_tok * w.n_kv_heads,
        "resident_cache_bytes": cache_bytes,
        "warm_single_copy_kernel_us": warm_us,
        "device": {"name": prop.name, "compute_units": prop.multi_processor_count,
                   "memory_gib": round(prop.total_memory / 2**30, 1),
                   "l2_cache_mib": round(getattr(prop, "L2_cache_size", 0) / 2**20, 1)},
        "compression_vs_16bit": 2 * w.head_dim * 2 / bytes_tok,
        "separate_region_kernel_us": sep_us,
        "preheat": {"seconds": PREHEAT_S, "attention_launches": r["preheat_launches"],
                    "what": "decode-attention launches without appends, right before the warm-up steps (GPU clocks ramp)"},
        "kernel_event_samples_in_timed_region": r["k_samples"],
        "kernel_event_samples_us": r["k_list"],
        "quantize_append_prefill": {"tokens": w.batch * w.context, "us": pre_us,
                                    "hbm_gbs": pre_bytes / (pre_us * 1e-6) / 1e9,
                                    "frac": pre_bytes / (pre_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                                    "algorithmic_bytes": pre_bytes,
                                    "what": "one oscar_quantize_append call (encoder kernel, then the small "
                                            "length-update kernel) between two events; median over refills",
                                    "profiled": profiled_prefill(w, pre_bytes)},
    }
    if parity:
        res["parity"] = parity
    if rot:
        res["rotate_keys"] = rot
    if stream_read:
        res["stream_read_probe"] = stream_read
    if bf16:
        res["bf16_decode"] = bf16
        res["speedup_vs_bf16_decode"] = bf16["us_per_step"] / us_step
        res["kernel_speedup_vs_bf16_decode"] = bf16["us_per_step"] / k_us
        if stream_read:
            # the comparator is not a tuned kernel: also relate the compressed path to a 16-bit
            # decode that would stream its bytes at the rate of the loads-only probe
            ideal_us = b_bytes / (stream_read["hbm_gbs"] * 1e9) * 1e6
            res["bf16_decode"]["us_at_stream_probe_rate"] = ideal_us
            res["kernel_speedup_vs_bf16_at_stream_probe_rate"] = ideal_us / k_us
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(w, kd, vd, q_host, cfg)
    return res


if __name__ == "__main__":
    main()
