#!/usr/bin/env python3
"""Benchmark of the MLA decode hot path on one MI355X.

A "step" is one whole call of the path (split-KV main kernel + LSE combine kernel) over one batch
of seeded synthetic input that is already resident in HBM.  The workload is the configuration the
headline metric is quoted on: batch 16, 16 heads, KV length 65536 per sequence, bf16.

Prints ONE JSON line.  `value` is algorithmic bytes per call / wall time per call (TB/s);
`roofline` is the main kernel alone, timed with events on the launch stream; `cpu_baseline` is
the fp64 oracle timed on this machine's host cores over a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "MLA decode us/call + achieved HBM TB/s (b=16, 16 heads, KV=64K, bf16)"
HBM_PEAK_GBPS = 8000.0          # MI355X published peak
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "mla_decode_split_b16_kv64k_traffic.json")
CPU_SAMPLE_SEQS = 16            # sequences of the batch the oracle is timed on, best of 3 (the whole headline batch: about 1 s per call on 16 host threads)
PROBE_WORKGROUPS = (176, 208, 256)


def load_probe():
    """The streaming-read probe (measurement only, its own library): built if missing, loaded with ctypes."""
    import ctypes
    from paper_2506_01969_amd import build as hip_build
    if not os.path.exists(hip_build.PROBE_LIB_PATH):
        hip_build.build_probe()
    lib = ctypes.CDLL(hip_build.PROBE_LIB_PATH)
    lib.hbm_probe_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p,
                                   ctypes.POINTER(ctypes.c_size_t), ctypes.c_void_p]
    lib.hbm_probe_read.restype = ctypes.c_int
    return lib


def probe_ceiling(torch, buffers, launches=30, workgroups=PROBE_WORKGROUPS):
    """What a plain streaming read of the same buffers reaches (no arithmetic, the main kernel's request pattern),
    for each number of workgroups: average of `launches` launches timed with events on the launch stream,
    buffers rotated.  -> list of {"workgroups", "us", "gb_per_s"}."""
    import ctypes
    lib = load_probe()
    sink = torch.zeros((16,), dtype=torch.int32, device=buffers[0].device)
    stream = ctypes.c_void_p(torch.cuda.current_stream(buffers[0].device).cuda_stream)
    nbytes = buffers[0].numel() * buffers[0].element_size()
    got = ctypes.c_size_t(0)
    res = []
    for wg in workgroups:
        if nbytes < wg * 4 * 36 * 1024:          # less than one round of 36 KB per wavefront: nothing to stream
            continue

        def launch(i):
            rc = lib.hbm_probe_read(ctypes.c_void_p(buffers[i % len(buffers)].data_ptr()), nbytes, wg,
                                    ctypes.c_void_p(sink.data_ptr()), ctypes.byref(got), stream)
            if rc != 0:
                raise RuntimeError("hbm_probe_read failed")
        for i in range(5):
            launch(i)
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(launches)]
        for i in range(launches):
            ev[i][0].record()
            launch(i)
            ev[i][1].record()
        torch.cuda.synchronize()
        us = sum(a.elapsed_time(b) for a, b in ev) / launches * 1e3
        res.append({"workgroups": wg, "us": us, "gb_per_s": got.value / us / 1e3, "bytes": got.value})
    return res


def unit_flag(mla, args):
    return {"auto": 0, "fine": mla.UNIT_FINE, "coarse": mla.UNIT_COARSE}[args.unit]


def lds_patterns():
    """(name, op, 64 byte offsets) of the main kernel's three LDS access patterns (op 0 ds_read_b128: the K operand,
    2 ds_read_b64_tr_b16: the V^T operand, 1 ds_write_b128: the tile write) for candidate row strides and token orders.
    Lane l = 16 g + r16.  Rows are 1152 bytes of data, `stride` bytes apart."""
    lanes = range(64)
    pats = [("ds_read_b128, 64 lanes x 16 B contiguous (reference)", 0, [16 * l for l in lanes]),
            ("ds_write_b128, 64 lanes x 16 B contiguous (reference)", 1, [16 * l for l in lanes]),
            ("ds_read_b64_tr_b16, 64 lanes x 8 B contiguous (reference)", 2, [8 * l for l in lanes])]
    even_odd = lambda r: ((2 * r) & 15) + (r >> 3)
    for stride in (1152, 1168, 1184, 1200, 1216, 1248):
        pats.append(("K operand: lane -> row r16, chunk g; row stride %d" % stride, 0, [(l & 15) * stride + 16 * (l >> 4) for l in lanes]))
    pats.append(("K operand: lane -> row 2 r16 mod 16 + (r16 >= 8) (even rows first), chunk g; row stride 1168", 0,
                 [even_odd(l & 15) * 1168 + 16 * (l >> 4) for l in lanes]))
    for d in (0, 16, 32, 64, 256):
        pats.append(("K operand, row stride 1168, groups %d bytes apart instead of 16" % d, 0, [(l & 15) * 1168 + d * (l >> 4) for l in lanes]))
    for stride in (1168, 1184):
        for ct in (0, 1, 5):
            pats.append(("V^T operand: quad q of k-group g -> row 4 g + q, value tile %d; row stride %d" % (ct, stride), 2,
                         [(4 * (l >> 4) + ((l & 15) >> 2)) * stride + (l & 3) * 8 + 32 * ct for l in lanes]))
    pats.append(("V^T operand: rows 8 (g & 1) + (g >> 1) + 2 q (even rows first), value tile 0; row stride 1168", 2,
                 [(8 * ((l >> 4) & 1) + (l >> 5) + 2 * ((l & 15) >> 2)) * 1168 + (l & 3) * 8 for l in lanes]))
    pats.append(("V^T operand: rows 8 (g & 1) + (g >> 1) + 2 q (even rows first), value tile 0; row stride 1184", 2,
                 [(8 * ((l >> 4) & 1) + (l >> 5) + 2 * ((l & 15) >> 2)) * 1184 + (l & 3) * 8 for l in lanes]))
    for stride in (1168, 1184):
        for i in (0, 1, 4, 8):
            pats.append(("tile write: load %d of 36 (lane l holds 16-byte chunk 64 i + l of the tile); row stride %d" % (i, stride), 1,
                         [((64 * i + l) // 72) * stride + 16 * ((64 * i + l) % 72) for l in lanes]))
    # the direct orientation (comparison kernel) reads K and V as above; its P crosses lanes through LDS, heads `ps` floats apart
    for ps in (32, 36, 40):
        pats.append(("direct orientation, P to LDS: ds_write_b32 at float (4 g + i) %d + r16" % ps, 3, [((4 * (l >> 4)) * ps + (l & 15)) * 4 for l in lanes]))
        pats.append(("direct orientation, P from LDS: ds_read_b128 at float %d r16 + 4 g" % ps, 0, [((l & 15) * ps + 4 * (l >> 4)) * 4 for l in lanes]))
    return pats


def lds_probe(torch, dev):
    """One launch of the LDS probe kernel per pattern of lds_patterns(), in order; prints the patterns' names as one
    JSON line, so that a rocprofv3 --pmc run of this mode can be read dispatch by dispatch."""
    import ctypes
    from paper_2506_01969_amd import build as hip_build
    if not os.path.exists(hip_build.LDS_PROBE_LIB_PATH):
        hip_build.build_lds_probe()
    lib = ctypes.CDLL(hip_build.LDS_PROBE_LIB_PATH)
    lib.lds_probe_run.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    lib.lds_probe_run.restype = ctypes.c_int
    sink = torch.zeros((16,), dtype=torch.int32, device=dev)
    names = []
    for name, op, offs in lds_patterns():
        assert len(offs) == 64 and all(o % 4 == 0 and 0 <= o <= 40 * 1024 - 16 for o in offs), name
        table = torch.tensor(offs, dtype=torch.int32, device=dev)
        rc = lib.lds_probe_run(ctypes.c_void_p(table.data_ptr()), op, ctypes.c_void_p(sink.data_ptr()),
                               ctypes.c_void_p(torch.cuda.current_stream(dev).cuda_stream))
        if rc != 0:
            raise RuntimeError("lds_probe_run failed")
        torch.cuda.synchronize()
        names.append(name)
    print(json.dumps({"lds_probe_patterns_in_dispatch_order": names, "iterations_per_launch": 4096}))


def timeline(torch, inputs, dev, args):
    """Where the time of one call goes, from the measurement build of the library (the product source compiled
    with -DMLA_TIMELINE: every wavefront of the main kernel and every block of the merge kernel record the
    100 MHz real-time counter at their phase boundaries).  Prints one JSON line: for each phase the minimum,
    median and maximum over the wavefronts (blocks), in microseconds after the first wavefront's start, as
    medians over `--steps` calls (each preceded by warm calls on rotated KV buffers)."""
    import ctypes
    import statistics
    from paper_2506_01969_amd import build as hip_build
    if not os.path.exists(hip_build.TIMELINE_LIB_PATH):
        hip_build.build_timeline()
    L = ctypes.CDLL(hip_build.TIMELINE_LIB_PATH)
    vp, ci = ctypes.c_void_p, ctypes.c_int
    L.mla_decode.argtypes = [vp, vp, ctypes.c_int64, vp, ci, ci, ci, ctypes.c_float, vp, vp, vp, ctypes.c_size_t, vp]
    L.mla_decode.restype = ci
    L.mla_decode_workspace_size.argtypes = [ci, ci, ci, ci, ctypes.POINTER(ctypes.c_size_t), ctypes.POINTER(ci)]
    L.mla_timeline_buffer.argtypes = [vp]
    cfg = inputs.CONFIGS[args.config]
    q, kv, lens = inputs.make_config(args.config)
    batch, max_seqlen = cfg["batch"], cfg["seqlen"]
    qd, ld = q.to(dev), lens.to(dev)
    n_buf = max(2, min(16, -(-(512 << 20) // (kv.numel() * 2))))
    kvs = [kv.to(dev)]
    for _ in range(n_buf - 1):
        kvs.append(kvs[0].clone())
    need, nwg = ctypes.c_size_t(0), ci(0)
    assert L.mla_decode_workspace_size(batch, 16, max_seqlen, 0, ctypes.byref(need), ctypes.byref(nwg)) == 0
    ws = torch.empty((need.value,), dtype=torch.uint8, device=dev)
    out = torch.empty((batch, 1, 16, 512), dtype=torch.float32, device=dev)
    lse = torch.empty((batch, 16), dtype=torch.float32, device=dev)
    blocks = batch * 16 * 16                                    # the widest merge launch
    stamps = torch.zeros(((1 << 20) + blocks * 4,), dtype=torch.int64, device=dev)
    stream = vp(torch.cuda.current_stream(dev).cuda_stream)

    def call(i):
        st = L.mla_decode(vp(qd.data_ptr()), vp(kvs[i % n_buf].data_ptr()), kvs[0].stride(0), vp(ld.data_ptr()), batch, 16,
                          max_seqlen, inputs.SCALE, vp(out.data_ptr()), vp(lse.data_ptr()), vp(ws.data_ptr()), need.value, stream)
        assert st == 0, st
    names = ["start", "lengths_summed", "first_piece_known", "first_loads_issued", "first_tile_in_lds", "last_tile_done",
             "accumulators_in_lds", "results_stored"]
    cnames = ["start", "lengths_summed", "merged", "stored"]
    rows = {("split", n): [] for n in names}
    rows.update({("combine", n): [] for n in cnames})
    gaps = []
    for rep_ in range(args.steps):
        L.mla_timeline_buffer(None)
        for i in range(max(args.warmup, 3)):
            call(rep_ + i)
        stamps.zero_()
        torch.cuda.synchronize()
        L.mla_timeline_buffer(vp(stamps.data_ptr()))
        call(rep_)
        torch.cuda.synchronize()
        host = stamps.cpu()
        sp = host[:nwg.value * 4 * 8].view(-1, 8)
        sp = sp[sp[:, 0] != 0].double() / 100.0                   # 100 MHz -> microseconds
        cb = host[(1 << 20):].view(-1, 4)
        cb = cb[cb[:, 0] != 0].double() / 100.0
        t0 = float(sp[:, 0].min())
        for i, n in enumerate(names):
            col = sp[:, i][sp[:, i] != 0] - t0
            if col.numel():
                rows[("split", n)].append((float(col.min()), float(col.median()), float(col.max())))
        for i, n in enumerate(cnames):
            if cb.shape[0]:
                col = cb[:, i] - t0
                rows[("combine", n)].append((float(col.min()), float(col.median()), float(col.max())))
        if cb.shape[0]:
            gaps.append(float(cb[:, 0].min()) - float(sp[:, 7].max()))
    L.mla_timeline_buffer(None)
    med = lambda v: [round(statistics.median(x[j] for x in v), 2) for j in range(3)] if v else None
    print(json.dumps({"timeline_us_after_first_wavefront_start": "min / median / max over wavefronts (blocks), medians of %d calls" % args.steps,
                      "config": args.config, "batch": batch, "max_seqlen": max_seqlen, "workgroups": nwg.value,
                      "main_kernel": {n: med(rows[("split", n)]) for n in names},
                      "merge_kernel": {n: med(rows[("combine", n)]) for n in cnames},
                      "gap_main_end_to_merge_start_us": round(statistics.median(gaps), 2) if gaps else None}))


def sweep(torch, inputs, mla, dev, args):
    """Whole-call time over the grid of the paper's Figure 1 (Section 4.1: batch 16 and 32, KV length
    512 ... 64K, one query token, 16 heads).  Values are drawn on the device (timing only; parity over
    these shapes is the job of the tests).  KV buffers are rotated so that consecutive calls cannot be
    served from the 256 MB last-level cache."""
    g = torch.Generator(device=dev).manual_seed(inputs.BASE_SEED)
    for batch in [int(x) for x in args.batches.split(",")]:
        for n in [int(x) for x in args.kv_lens.split(",")]:
            kv_bytes = batch * n * inputs.D_QK * 2
            n_buf = max(2, min(64, -(-(512 << 20) // kv_bytes)))
            dt = torch.float16 if args.dtype == "fp16" else torch.bfloat16
            q = torch.randn((batch, 1, 16, inputs.D_QK), device=dev, generator=g).to(dt)
            kvs = [torch.randn((batch, n, inputs.D_QK), device=dev, generator=g).to(dt)
                   for _ in range(n_buf)]
            lens = torch.full((batch,), n, dtype=torch.int32, device=dev)
            need, nwg = mla.mla_decode_workspace_size(batch, 16, n, args.workgroups)
            ws = torch.empty((need,), dtype=torch.uint8, device=dev)
            out = torch.empty((batch, 1, 16, 512), dtype=torch.float32, device=dev)
            lse = torch.empty((batch, 16), dtype=torch.float32, device=dev)

            phases = None if args.unit == "auto" else (mla.PHASE_SPLIT | mla.PHASE_COMBINE | unit_flag(mla, args))

            def step(i):
                mla.mla_decode(q, kvs[i % n_buf], lens, inputs.SCALE, out=out, lse=lse, workspace=ws,
                               num_workgroups=args.workgroups or None, phases=phases)
            for i in range(args.warmup):
                step(i)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(args.steps):
                step(i)
            torch.cuda.synchronize()
            us = (time.perf_counter() - t0) / args.steps * 1e6
            alg = inputs.algorithmic_bytes([n] * batch)
            print(json.dumps({"dtype": args.dtype, "batch": batch, "kv_len": n, "us_per_call": round(us, 2),
                              "tb_per_s": round(alg / us / 1e6, 3),
                              "tflops_paper_style": round(inputs.algorithmic_flops([n] * batch) / us / 1e6, 1),
                              "workgroups": nwg, "kv_buffers_rotated": n_buf}), flush=True)
            del kvs


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=4, help="benchmark configuration id (4 = headline)")
    ap.add_argument("--workgroups", type=int, default=0, help="force the number of workgroups (0 = automatic)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--orientation", choices=("transposed", "direct"), default="transposed",
                    help="transposed = equations (1)-(4), the library's own choice; direct = Section 3.1 as written "
                         "(comparison variant, bf16 and one query token only)")
    ap.add_argument("--q-len", type=int, default=1,
                    help="query tokens per sequence (1 = the headline metric; the paper names 1 or 2)")
    ap.add_argument("--dtype", choices=("bf16", "fp16"), default="bf16",
                    help="element type of q and the KV cache (bf16 = the headline metric; fp16 = the paper's own)")
    ap.add_argument("--unit", choices=("auto", "fine", "coarse"), default="auto",
                    help="rows per unit of the KV stream: auto = the library's rule (128, or 32 for a short stream), "
                         "fine = 32, coarse = 128 (comparison)")
    ap.add_argument("--sweep", action="store_true",
                    help="time the whole call over batch 16 and 32 x KV length 512 ... 64K (the grid of the "
                         "paper's Figure 1) and print one JSON line per point instead of the benchmark line")
    ap.add_argument("--batches", default="16,32", help="batch sizes of --sweep")
    ap.add_argument("--kv-lens", default="512,1024,2048,4096,8192,16384,32768,65536", help="KV lengths of --sweep")
    ap.add_argument("--timeline", action="store_true",
                    help="per-phase time stamps of one call of --config from the measurement build of the library "
                         "(medians over --steps calls), as one JSON line; then exit")
    ap.add_argument("--lds-probe", action="store_true",
                    help="only launch the LDS access-pattern probe once per pattern (the main kernel's K, V^T and tile-write "
                         "patterns for candidate row strides; for rocprofv3 --pmc SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE) and exit")
    ap.add_argument("--ceiling-probe", action="store_true",
                    help="only run the plain streaming-read probe (no arithmetic, the main kernel's request pattern) over "
                         "the KV buffers of --config for several numbers of workgroups, print one JSON line each and exit")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain device-to-device copy of 1 GiB five times (counter calibration "
                         "for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE) and exit")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is a single-GPU kernel library; run with --gpus 1 "
              "(no sharding, collectives or multi-rank path exists)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2506_01969_amd import inputs, mla

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    mla.lib()                                   # fail loudly if the HIP library is missing
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.copy_calibration:
        src = torch.full((1 << 28,), 1.0, dtype=torch.float32, device=dev)     # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": src.numel() * 4, "copy_calibration_bytes_written": src.numel() * 4,
                          "copies": 5}))
        return

    if args.lds_probe:
        lds_probe(torch, dev)
        return

    if args.sweep:
        sweep(torch, inputs, mla, dev, args)
        return

    if args.timeline:
        timeline(torch, inputs, dev, args)
        return

    cfg = inputs.CONFIGS[args.config]
    dt = torch.float16 if args.dtype == "fp16" else torch.bfloat16
    q, kv, lens = inputs.make_config(args.config, dtype=dt, q_len=args.q_len)
    batch, max_seqlen = cfg["batch"], cfg["seqlen"]
    alg_bytes = inputs.algorithmic_bytes(lens.tolist())
    alg_flops = inputs.algorithmic_flops(lens.tolist())

    qd, ld = q.to(dev), lens.to(dev)
    kv_bytes = kv.numel() * 2
    # rotate over enough KV copies that no call can be served from the 256 MB last-level cache
    n_buf = max(2, -(-(512 << 20) // kv_bytes))
    kvs = [kv.to(dev)]
    for _ in range(n_buf - 1):
        kvs.append(kvs[0].clone())
    nwg = args.workgroups or None
    need, _ = mla.mla_decode_workspace_size(batch * args.q_len, 16, max_seqlen, args.workgroups)
    nwg_used = args.workgroups or mla.mla_decode_planned_workgroups(batch, args.q_len, max_seqlen)
    ws = torch.empty((need,), dtype=torch.uint8, device=dev)
    out = torch.empty((batch, args.q_len, 16, 512), dtype=torch.float32, device=dev)
    lse = torch.empty((batch, args.q_len, 16), dtype=torch.float32, device=dev)
    # q, out and lse of the extra query tokens are algorithmic bytes too; the KV rows are still read once
    alg_bytes += (args.q_len - 1) * batch * (16 * 576 * 2 + 16 * 512 * 4 + 16 * 4)
    alg_flops *= args.q_len

    orient = (mla.ORIENT_DIRECT if args.orientation == "direct" else 0) | unit_flag(mla, args)

    if args.ceiling_probe:
        for r in probe_ceiling(torch, kvs, launches=max(args.steps, 10), workgroups=(64, 128, 160, 176, 192, 208, 224, 256)):
            print(json.dumps({"probe": "streaming read, 36 x 1 KB in flight per wavefront, 4 wavefronts per workgroup",
                              "config": args.config, **r}), flush=True)
        return

    def step(i, phases=mla.PHASE_SPLIT | mla.PHASE_COMBINE):
        mla.mla_decode(qd, kvs[i % n_buf], ld, inputs.SCALE, out=out, lse=lse, workspace=ws,
                       num_workgroups=nwg, phases=phases | orient)

    # ---- the practical ceiling: a plain streaming read of the same buffers ------------------------
    probed = probe_ceiling(torch, kvs, launches=100)
    ceiling = max(probed, key=lambda r: r["gb_per_s"]) if probed else None     # None: buffers too small to stream (config 1)

    # ---- main kernel alone, events on the launch stream (torch's current stream) ---------------
    # The roofline figure is the kernel's average launch duration: at least 200 launches after at least 50
    # untimed ones, whatever --steps and --warmup say (the first few hundred launches of this kernel in a
    # process run 2-3 % slower; the kernel trace this figure is compared with averages 160 launches).
    kernel_launches, kernel_warm = max(args.steps, 200), max(args.warmup, 50)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(kernel_launches)]
    for i in range(kernel_warm):
        step(i, mla.PHASE_SPLIT)
    torch.cuda.synchronize()
    for i in range(kernel_launches):
        ev[i][0].record()
        step(i, mla.PHASE_SPLIT)
        ev[i][1].record()
    torch.cuda.synchronize()
    durs = sorted(a.elapsed_time(b) for a, b in ev)
    split_ms_avg = sum(durs) / len(durs)
    split_ms_med = durs[len(durs) // 2]
    achieved_gbps = alg_bytes / (split_ms_avg * 1e-3) / 1e9

    # ---- whole call ----------------------------------------------------------------------------
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall / args.steps * 1e3
    tbps = alg_bytes / (ms_per_step * 1e-3) / 1e12

    # ---- whole call again, each call bracketed by events on the launch stream: the spread ----------
    evw = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for i in range(args.steps):
        evw[i][0].record()
        step(i)
        evw[i][1].record()
    torch.cuda.synchronize()
    call_us = sorted(a.elapsed_time(b) * 1e3 for a, b in evw)
    call_stats = {"median_us": call_us[len(call_us) // 2], "min_us": call_us[0],
                  "p90_us": call_us[min(len(call_us) - 1, (len(call_us) * 9) // 10)]}

    traffic, traffic_source = None, None
    if (args.config == 4 and args.dtype == "bf16" and args.q_len == 1 and args.orientation != "direct"
            and not args.workgroups and os.path.exists(TRAFFIC_FILE)):   # the counters were read for this launch only
        try:
            traffic = json.load(open(TRAFFIC_FILE)).get("hbm_bytes_per_launch")
            traffic_source = "profiles/%s (static: rocprofv3 FETCH_SIZE + WRITE_SIZE of this launch, read in separate runs, not by this run)" % os.path.basename(TRAFFIC_FILE)
        except (OSError, ValueError):
            traffic = None

    # ---- CPU baseline: the oracle as it stands, on a bounded sample ----------------------------
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import mla_oracle
        ns = min(CPU_SAMPLE_SEQS, batch)
        qs, kvsamp, ls = q[:ns], kv[:ns], lens[:ns]
        qb, kvb = inputs.bits16(qs), inputs.bits16(kvsamp)
        cpu_s = None
        for _ in range(3):                                   # best of three
            t0 = time.perf_counter()
            ref_o, ref_l = mla_oracle.decode_general(qb, kvb, ls.numpy(), inputs.SCALE, inputs.D_V,
                                                     dtype=mla_oracle.F16 if args.dtype == "fp16" else mla_oracle.BF16)
            dt_s = time.perf_counter() - t0
            cpu_s = dt_s if cpu_s is None else min(cpu_s, dt_s)
        ref_o = ref_o.reshape(ns, args.q_len * 16, 512)
        sample_bytes = inputs.algorithmic_bytes(ls.tolist())
        # the same sample doubles as a sanity check of the benchmarked output: one whole call (both kernels) first
        out.fill_(float("nan"))
        step(0)
        torch.cuda.synchronize()
        got = out.cpu().numpy().reshape(batch, args.q_len * 16, 512)[:ns]
        max_abs = float(abs(got - ref_o).max())
        cpu = {"value": sample_bytes / cpu_s / 1e12, "unit": "TB/s", "cores": mla_oracle.threads(), "kind": "oracle",
               "sample": "first %d of %d sequences, all 16 heads, full KV (%d tokens), best of 3 oracle calls" % (
                   ns, batch, int(ls.sum())),
               "seconds": cpu_s, "us_per_call_equiv": cpu_s * 1e6 * (alg_bytes / sample_bytes),
               "gpu_vs_oracle_max_abs_on_sample": max_abs}

    line = {
        "metric": METRIC, "value": tbps, "unit": "TB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "us_per_call": ms_per_step * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": "config %d: MLA decode batch %d, q_len %d, 16 heads, shared 576-d %s latent KV, "
                               "KV length %s, scale 1/sqrt(192), d_v 512" % (
                                   args.config, batch, args.q_len, args.dtype, "%d per sequence" % max_seqlen if cfg["ragged"] is None
                                   else "ragged uniform[%d,%d]" % cfg["ragged"]),
                   "total_kv_tokens": int(lens.sum()), "algorithmic_bytes_per_call": alg_bytes,
                   "algorithmic_flops_per_call": alg_flops, "workgroups": nwg_used,
                   "kv_buffers_rotated": n_buf, "orientation": args.orientation,
                   "call_event_timing": call_stats, "hbm_peak_frac_whole_call": tbps * 1e3 / HBM_PEAK_GBPS,
                   "tflops_whole_call": alg_flops / (ms_per_step * 1e-3) / 1e12},
        "roofline": {"bound": "hbm", "kernel": "mla_decode_split_kernel", "achieved": achieved_gbps,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved_gbps / HBM_PEAK_GBPS, "traffic": traffic,
                     "traffic_source": traffic_source,
                     "achievable": ceiling["gb_per_s"] if ceiling else None,
                     "frac_of_achievable": achieved_gbps / ceiling["gb_per_s"] if ceiling else None,
                     "achievable_source": "plain streaming read of the same KV buffers measured by this run (%d workgroups, "
                                          "%.1f us per launch, no arithmetic): csrc/hbm_probe.hip" % (ceiling["workgroups"], ceiling["us"])
                                          if ceiling else None,
                     "avg_us": split_ms_avg * 1e3, "median_us": split_ms_med * 1e3,
                     "launches_timed": kernel_launches, "launches_untimed_before": kernel_warm},
        "cpu_baseline": cpu,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
