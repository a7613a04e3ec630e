"""Where one launch of the matrix-core decode kernel spends its time, from inside the kernel.

    python -m paper_2605_19660_amd.phase_profile [--workload N] [--reps K]

Runs the library built with phase time stamps (`python -m paper_2605_19660_amd.build --stamps`,
built here if missing): lane 0 of every wave of the first four and the last four workgroups of the
grid writes the constant-rate counter (100 MHz, common to all CUs) at the boundaries of the
kernel's phases.  The script keeps the GPU busy for a while (clocks), launches the kernel once
between two events on a cache copy that is not in the last-level cache, reads the stamps back
and prints them in microseconds after the earliest entry among the sampled workgroups.  The
stamps themselves cost a scalar memory instruction and a wait each (about 1 % of the kernel).
"""
from __future__ import annotations

import argparse
import ctypes as C
import os
import sys
import time

HERE = os.path.dirname(os.path.abspath(__file__))
STAMP_NAMES = {0: "entry", 1: "arguments", 2: "first page (key side) asked for", 3: "queries rotated", 4: "prologue done",
               5: "first logits", 24: "loop done", 25: "results in LDS", 26: "barrier passed",
               27: "record written"}


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", type=int, default=1)
    ap.add_argument("--reps", type=int, default=3)
    ap.add_argument("--residual", type=int, default=0,
                    help="tokens appended one call behind the prefill (0..128): they stay in the 16-bit window")
    args = ap.parse_args()

    lib_path = os.path.join(HERE, "liboscar_hip_stamps.so")
    if not os.path.exists(lib_path):
        from . import build
        build.build_stamps()
    os.environ["OSCAR_HIP_LIB"] = lib_path       # read by the binding when it loads the library
    import numpy as np
    import torch
    from . import binding as ob, synth

    w = synth.CONFIGS[args.workload]
    io = {"f32": ob.F32, "bf16": ob.BF16, "f16": ob.F16}[w.io_dtype]
    meta = {"f32": ob.F32, "f16": ob.F16}[w.meta_dtype]
    cfg = ob.Config(w.n_q_heads, w.n_kv_heads, w.head_dim, w.bits, w.k_group, w.v_group, w.page_size,
                    io, meta)
    kd, vd = synth.make_kv_device(w)
    pages = w.context // w.page_size + 3
    if not 0 <= args.residual <= w.page_size:
        sys.exit("--residual must be 0..%d" % w.page_size)
    cache_mb = w.batch * w.n_kv_heads * w.context * synth.cache_bytes_per_token_kvh(w) / 1e6
    n_copies = max(2, int(512 / cache_mb) + 2)
    caches = []
    for _ in range(n_copies):
        c = ob.Cache(cfg, w.batch, pages)
        ob.quantize_append(c, kd, vd, eager=True, max_seq_len_hint=0)
        if args.residual:
            ob.quantize_append(c, kd[:, :args.residual].contiguous(), vd[:, :args.residual].contiguous())
        caches.append(c)
    del kd, vd
    q = torch.from_numpy(synth.make_q(w)).cuda().to(ob.torch_dtype(io)).contiguous()
    out = torch.empty(w.batch, w.n_q_heads, w.head_dim, dtype=torch.float32, device="cuda")
    splits = ob.decode_auto_splits(cfg, w.batch, w.context + args.residual)
    ws = torch.empty(ob.decode_workspace_bytes(cfg, w.batch, splits), dtype=torch.uint8, device="cuda")
    lib = ob.lib()
    lib.oscar_debug_read_stamps.argtypes = [C.c_void_p, C.c_size_t]
    lib.oscar_debug_read_stamps.restype = C.c_int

    pages_per_wave = -(-(w.context // w.page_size) // (4 * splits))
    print("# workload %s: batch %d, %d kv heads, context %d, %d-bit; %d splits -> %d workgroups, %d pages per wave"
          % (w.name, w.batch, w.n_kv_heads, w.context, w.bits, splits, splits * w.n_kv_heads * w.batch,
             pages_per_wave) + ("; %d tokens in the 16-bit residual window" % args.residual if args.residual else ""))
    print("# us after the earliest entry among the sampled workgroups; slots 0-3: splits 0-3 of (sequence 0, kv head 0),")
    print("# the first workgroups of the grid; slots 4-7: splits 0-3 of the last sequence's last kv head")
    for rep in range(args.reps):
        t0 = time.perf_counter()
        i = 0
        while time.perf_counter() - t0 < 0.15:       # a busy GPU: see bench.py's preheat
            for _ in range(32):
                ob.decode_attn_partial(caches[i % n_copies], q, ws, splits)
                ob.decode_attn_reduce(caches[i % n_copies], out, ws, splits)
                i += 1
            torch.cuda.synchronize()
        tm = ob.Timer()
        ob.decode_attn_partial(caches[i % n_copies], q, ws, splits, timer=tm)
        torch.cuda.synchronize()
        ev_us = tm.elapsed_us()
        tm.close()
        buf = (C.c_ulonglong * (8 * 4 * 32))()
        rc = lib.oscar_debug_read_stamps(buf, C.sizeof(buf))
        if rc != 0:
            sys.exit("oscar_debug_read_stamps failed: %d" % rc)
        a = np.frombuffer(buf, dtype=np.uint64).reshape(8, 4, 32).astype(np.int64)
        t_first = a[:, :, 0].min()
        print("\n# launch %d: %.2f us between its two events; last stamp %.2f us after the first"
              % (rep, ev_us, (a[:, :, 27].max() - t_first) / 100.0))
        hdr = ["slot", "wave"] + [STAMP_NAMES[k] for k in (0, 1, 2, 3, 4)] + ["page iteration tops"] + \
              [STAMP_NAMES[k] for k in (5, 24, 25, 26, 27)]
        print(" | ".join(hdr))
        for slot in (0, 3, 4, 7):
            for wave in (0, 3):
                t = (a[slot, wave] - t_first) / 100.0
                tops = " ".join("%.2f" % t[8 + k] for k in range(min(16, pages_per_wave)))
                print(" | ".join(["%d" % slot, "%d" % wave] + ["%.2f" % t[k] for k in (0, 1, 2, 3, 4)] + [tops] +
                                 ["%.2f" % t[k] for k in (5, 24, 25, 26, 27)]))


if __name__ == "__main__":
    main()
