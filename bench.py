#!/usr/bin/env python3
"""Benchmark of the LogQuant decode hot path on one MI355X.

One "step" is one pass of the whole hot path over one batch: append the new token's
K/V rows, run the filtering + 2-bit quantization + compaction when the
original-precision window is full, then decode attention over both regions.
Consecutive steps rotate over several independent copies of the cache (as the layers
of a model would), so every step reads its cache from HBM rather than from the
256 MB last-level cache.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed steps (default: one window W)")
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", type=int, default=3, help="1..5, see BASELINE.json configs")
    ap.add_argument("--copies", type=int, default=0, help="cache copies to rotate over (0 = auto)")
    ap.add_argument("--bits", type=int, default=2, choices=(2, 4),
                    help="code width; 2 is BASELINE.json's setting, 4 the paper's higher-precision variant")
    ap.add_argument("--fp-budget", type=int, default=0,
                    help="override the workload's fp budget F = 2W (e.g. 84 or 170: the paper's W = floor(R/3), "
                         "R = 128 / 256, which the group size does not divide)")
    ap.add_argument("--per-sequence", action="store_true",
                    help="rows of different lengths (seeded, between L/2 and L) through the per-sequence entry "
                         "points; reports the same line for that batch")
    ap.add_argument("--unfused", action="store_true",
                    help="time the step as separate append and attention launches instead of logquant_decode_step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true",
                    help="skip the attention / compress legs of the other four BASELINE.json configs")
    ap.add_argument("--plain-valu", action="store_true",
                    help="time the plain vector-unit attention kernel of liblogquant_plain.so instead of the product's "
                         "(matrix unit or vector unit: the measurement behind that choice)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a plain 256 MiB device copy a few times (reference for HBM counters)")
    return ap.parse_args()


def slots_per_event(wl):
    """Quantized slots one filtering event takes: W rounded up to whole key groups."""
    W, G = wl["F"] // 2, wl["G"]
    return -(-W // G) * G


def q_capacity(wl):
    Wq = slots_per_event(wl)
    qcap = (wl["L"] // (wl["F"] // 2) + 4) * Wq
    while qcap % 64:
        qcap += Wq
    return qcap


def build_states(wl, cfg_id, copies):
    """Cache copy 0 is 5 tokens short of a full window (it fires one compress during
    the timed region), the others have just been compressed: L tokens.  The states are
    built with logquant_prefill (bit-identical to streaming the tokens through
    logquant_append / logquant_compress; tests/test_gpu_prefill.py), which is timed on
    the way.  Returns (cfg, caches, prefill record)."""
    import torch
    from paper_2503_19950_amd import binding, inputs
    from paper_2503_19950_amd.binding import to_dev
    W, L, dt = wl["F"] // 2, wl["L"], wl["dtype"]
    qcap = q_capacity(wl)
    cfg = binding.make_config(wl["B"], wl["Hq"], wl["Hkv"], wl["d"], wl["F"], wl["G"], dt, qcap,
                              wl.get("bits", 2))
    tdt = torch.bfloat16 if dt == "bf16" else torch.float16
    Kd = torch.empty((wl["B"], wl["Hkv"], L, wl["d"]), dtype=tdt, device="cuda:0")
    Vd = torch.empty_like(Kd)
    step = 1 << 14
    for t0 in range(0, L, step):
        t1 = min(L, t0 + step)
        K, V = inputs.batch_kv(cfg_id, t0, t1, wl)
        Kd[:, :, t0:t1] = to_dev(K, dt)
        Vd[:, :, t0:t1] = to_dev(V, dt)
    near = L - 5
    first = binding.DeviceCache(cfg)
    first.prefill(Kd[:, :, :near].contiguous(), Vd[:, :, :near].contiguous())
    dc = binding.DeviceCache(cfg)
    stream = torch.cuda.current_stream()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(8)]
    for i in range(4):                                   # same buffers, counts rewound: 1 warm-up + 3 timed
        dc.set_counts((0, 0, 0))
        ev[2 * i].record(stream)
        dc.prefill(Kd, Vd)
        ev[2 * i + 1].record(stream)
    torch.cuda.synchronize()
    ms = sorted(ev[2 * i].elapsed_time(ev[2 * i + 1]) for i in range(1, 4))[1]
    n_q = dc.c.n_q                                # slots; of every Wq slots W hold tokens
    n_tok = n_q // slots_per_event(wl) * W
    sizes = binding.logquant_sizes(cfg)
    bh = wl["B"] * wl["Hkv"]
    written = bh * (n_tok * (wl["d"] * wl.get("bits", 2) // 4 + 4 * -(-wl["d"] // wl["G"])) + n_q // wl["G"] * 4 * wl["d"]
                    + dc.c.n_fp * 4 * wl["d"])
    read = 2 * Kd.numel() * 2
    prefill = {"ms_per_call": ms, "tokens_per_s": wl["B"] * L / (ms * 1e-3),
               "algorithmic_bytes": read + written, "GBps": (read + written) / (ms * 1e-3) / 1e9}
    del Kd, Vd, sizes
    caches = [first, dc] + [dc.clone() for _ in range(copies - 2)]
    torch.cuda.synchronize()
    return cfg, caches, prefill


def filler_kv_device(wl, cfg_id, L):
    """[B][Hkv][L][d] K and V on the device in which eight seeded slices repeat (drawing
    every slice of the big batches on the host would take minutes; what is timed does not
    depend on the values)."""
    import torch
    from paper_2503_19950_amd import inputs
    from paper_2503_19950_amd.binding import to_dev
    B, H, d, dt = wl["B"], wl["Hkv"], wl["d"], wl["dtype"]
    n = min(8, B * H)
    Ks, Vs = [], []
    for i in range(n):
        k, v = inputs.slice_kv(cfg_id, i // H, i % H, 0, L, wl)
        Ks.append(to_dev(k, dt))
        Vs.append(to_dev(v, dt))
    idx = torch.arange(B * H, device="cuda:0") % n
    K = torch.stack(Ks)[idx].reshape(B, H, L, d).contiguous()
    V = torch.stack(Vs)[idx].reshape(B, H, L, d).contiguous()
    return K, V


def time_launches(fn, n, stream, warm=20):
    """fn(i) enqueues launch i; returns microseconds per launch over n back-to-back launches
    between one HIP event before and one after, on `stream`."""
    import torch
    for i in range(warm):
        fn(i)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for i in range(n):
        fn(i)
    e1.record(stream)
    e1.synchronize()
    return e0.elapsed_time(e1) * 1e3 / n


def compress_leg(binding, cfg, wl, dc, stream, calls=24):
    """logquant_compress on a full window, timed on its own: the counts are put back to
    n_fp = 3W before every call (the call only depends on the counts; the rows beyond the
    live ones hold whatever the buffers held).  Returns (us per call, bytes moved per call)."""
    import torch
    W = wl["F"] // 2
    Wq = slots_per_event(wl)
    saved = dc.counts()
    cur, n_fp, n_q = saved
    sh = stream.cuda_stream
    ts = []
    for i in range(calls + 4):
        dc.set_counts((cur, 3 * W, n_q))
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        st = binding.logquant_compress(cfg, dc.c, dc.workspace, sh)
        e1.record(stream)
        assert st == 0, binding.logquant_status_string(st)
        if i >= 4:
            ts.append((e0, e1))
    torch.cuda.synchronize()
    dc.set_counts(saved)
    us = float(sorted(e0.elapsed_time(e1) * 1e3 for e0, e1 in ts)[len(ts) // 2])
    d, G, bits = wl["d"], wl["G"], wl.get("bits", 2)
    per_slice = 3 * W * 4 * d + W * (d * bits // 4 + 4 * -(-d // G)) + Wq // G * 4 * d + 2 * W * 4 * d
    return us, wl["B"] * wl["Hkv"] * per_slice


def read_ceiling(binding, nbytes, copies, stream, launches=200):
    """Pure reading of as many bytes as one attention launch reads, rotating over `copies`
    buffers: the measured HBM ceiling at this size (GB/s)."""
    import torch
    n = max(2, copies)
    bufs = [torch.ones(max(16, int(nbytes)) // 16 * 16, dtype=torch.uint8, device="cuda:0") for _ in range(n)]
    sink = torch.zeros(8192, dtype=torch.int32, device="cuda:0")
    sh = stream.cuda_stream
    torch.cuda.synchronize()

    def fn(i):
        st = binding.logquant_read_probe(bufs[i % n], bufs[0].numel(), sink, sh)
        assert st == 0
    us = time_launches(fn, launches, stream)
    return {"us_per_launch": us, "bytes": int(bufs[0].numel()), "GBps": bufs[0].numel() / (us * 1e-6) / 1e9}


def attention_config_leg(binding, wl, cfg_id, stream, launches=200):
    """One of the other benchmark configs at its full size, in the launch shape the
    library picks: decode attention back to back over a rotation of cache copies, and the
    compress call on a full window.  States come from logquant_prefill on filler slices."""
    import torch
    W, L, dt = wl["F"] // 2, wl["L"], wl["dtype"]
    qcap = q_capacity(wl)
    cfg = binding.make_config(wl["B"], wl["Hq"], wl["Hkv"], wl["d"], wl["F"], wl["G"], dt, qcap, wl.get("bits", 2))
    K, V = filler_kv_device(wl, cfg_id, L)
    first = binding.DeviceCache(cfg)
    first.prefill(K, V)
    del K, V
    plan = binding.logquant_decode_plan(cfg, first.c.n_fp, first.c.n_q)
    copies = max(2, min(16, -(-(1 << 30) // max(1, plan.bytes_read))))
    caches = [first] + [first.clone() for _ in range(copies - 1)]
    from paper_2503_19950_amd import inputs
    from paper_2503_19950_amd.binding import to_dev
    q = to_dev(inputs.queries(cfg_id, 0, wl), dt)
    out = torch.empty_like(q)
    sh = stream.cuda_stream
    torch.cuda.synchronize()

    def fn(i):
        dc = caches[i % copies]
        st = binding.logquant_decode_attn(cfg, dc.c, q, 0.0, out, dc.workspace, sh)
        assert st == 0
    us = time_launches(fn, launches, stream)
    comp_us, comp_bytes = compress_leg(binding, cfg, wl, caches[0], stream)
    gbps = plan.bytes_read / (us * 1e-6) / 1e9
    rec = {"workload": wl["name"], "B": wl["B"], "Hq": wl["Hq"], "Hkv": wl["Hkv"], "d": wl["d"], "L": L, "dtype": dt,
           "group": wl["G"], "fp_budget": wl["F"], "n_fp": first.c.n_fp, "n_q": first.c.n_q,
           "attn_blocks": plan.blocks, "attn_splits": plan.splits, "waves_per_block": plan.waves_per_block,
           "cache_copies_rotated": copies, "launches_timed": launches,
           "us_per_launch": us, "algorithmic_bytes": int(plan.bytes_read), "GBps": gbps, "frac": gbps / HBM_PEAK_GBS,
           "kv_tokens_per_s": wl["B"] * L / (us * 1e-6),
           "compress_us": comp_us, "compress_bytes": int(comp_bytes), "compress_GBps": comp_bytes / (comp_us * 1e-6) / 1e9}
    if plan.bytes_read < (8 << 20):
        rec["note"] = "latency-bound: %.1f MB per launch; a fraction of HBM peak says nothing here" % (plan.bytes_read / 1e6)
    elif wl["B"] * wl["Hkv"] < 64:
        rec["compress_note"] = "compress moves %.1f MB: launch-latency-bound" % (comp_bytes / 1e6)
    del caches, first
    torch.cuda.empty_cache()
    return rec


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not supported (the path shards by "
              "kv head / batch row, each GPU running the same kernels on its slices)" % a.gpus, file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2503_19950_amd import binding, inputs
    from paper_2503_19950_amd.binding import to_dev

    wl = dict(inputs.WORKLOADS[a.workload])
    wl["bits"] = a.bits
    if a.bits != 2:
        wl["name"] += "_bits%d" % a.bits
    if a.fp_budget:
        wl["F"] = a.fp_budget
        wl["name"] += "_F%d" % a.fp_budget
    W, L, dt = wl["F"] // 2, wl["L"], wl["dtype"]
    steps = a.steps or W
    if a.per_sequence:
        return main_per_sequence(a, wl, steps)
    # everything is enqueued on one non-default stream (default priority); the events that time
    # the kernels are recorded on that same stream
    stream = torch.cuda.Stream()
    torch.cuda.set_stream(stream)
    # enough copies that the rotation's footprint is >= 1 GiB (4x the 256 MB last-level cache)
    cfg_probe = binding.make_config(wl["B"], wl["Hq"], wl["Hkv"], wl["d"], wl["F"], wl["G"], dt,
                                    q_capacity(wl), a.bits)
    plan0 = binding.logquant_decode_plan(cfg_probe, 2 * W, (L - 2 * W) // W * slots_per_event(wl))
    copies = a.copies or max(2, min(16, -(-(1 << 30) // max(1, plan0.bytes_read))))
    t_build = time.time()
    cfg, caches, prefill = build_states(wl, a.workload, copies)
    t_build = time.time() - t_build

    # per-step inputs: one new token per sequence and one query, seeded
    n_in = steps + a.warmup
    newK, newV = inputs.batch_kv(a.workload, L, L + n_in, wl)          # [B][Hkv][n_in][d]
    # [n_in][B][Hkv][1][d]: step j's rows are one contiguous block
    newK = to_dev(newK, dt).permute(2, 0, 1, 3).unsqueeze(3).contiguous()
    newV = to_dev(newV, dt).permute(2, 0, 1, 3).unsqueeze(3).contiguous()
    qs = to_dev(np.stack([inputs.queries(a.workload, s, wl) for s in range(n_in)]), dt)
    out = torch.empty_like(qs[0])
    sh = stream.cuda_stream
    torch.cuda.synchronize()

    fused = not a.unfused
    attend = binding.logquant_decode_attn
    if a.plain_valu:
        from paper_2503_19950_amd import plain_reference
        attend = plain_reference.logquant_plain_decode_attn
        fused = False

    def run(n, record):
        """n steps of the hot path; with record, HIP events around every attention launch."""
        ev = []
        n_compress = 0
        visits = [0] * len(caches)
        for s in range(n):
            i = s % len(caches)
            dc = caches[i]
            j = visits[i]
            visits[i] += 1
            if fused and not record and dc.c.n_fp + 1 < 3 * W:
                # append and attention in one launch (logquant_decode_step)
                st = binding.logquant_decode_step(cfg, dc.c, newK[j], newV[j], qs[s], 0.0, out, dc.workspace, sh)
                assert st == 0, binding.logquant_status_string(st)
                continue
            st = binding.logquant_append(cfg, dc.c, newK[j], newV[j], 1, sh)
            assert st == 0, binding.logquant_status_string(st)
            if dc.c.n_fp == 3 * W:
                st = binding.logquant_compress(cfg, dc.c, dc.workspace, sh)
                assert st == 0, binding.logquant_status_string(st)
                n_compress += 1
            if record:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
            st = attend(cfg, dc.c, qs[s], 0.0, out, dc.workspace, sh)
            assert st == 0, binding.logquant_status_string(st)
            if record:
                e1.record(stream)
                ev.append((e0, e1))
        return ev, n_compress

    saved = [dc.counts() for dc in caches]
    run(a.warmup, False)
    torch.cuda.synchronize()
    for dc, c in zip(caches, saved):
        dc.set_counts(c)

    # timed region 1: the whole hot path, K steps, wall clock between two synchronisations
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    _, n_compress = run(steps, False)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps
    for dc, c in zip(caches, saved):
        dc.set_counts(c)

    # timed region 2: single attention launches bracketed by an event pair each (the pair costs
    # a few microseconds itself): spread of single launches
    ev, _ = run(min(steps, 64), True)
    torch.cuda.synchronize()
    attn_event_pct = [float(x) for x in np.percentile([e0.elapsed_time(e1) * 1e3 for e0, e1 in ev], [10, 50, 90])]
    for dc, c in zip(caches, saved):
        dc.set_counts(c)

    # timed region 3: the attention launches alone, back to back on the launch stream, rotating
    # over the cache copies, one HIP event before and one after.  Kernel durations measured
    # this way agree with rocprofv3's kernel trace; the roofline figures are taken from here.
    nb2b = max(200, steps)

    def attn_fn(i):
        dc = caches[i % len(caches)]
        st = attend(cfg, dc.c, qs[0], 0.0, out, dc.workspace, sh)
        assert st == 0
    attn_us = time_launches(attn_fn, nb2b, stream)
    attn_bytes = float(np.mean([binding.logquant_decode_plan(cfg, caches[s % len(caches)].c.n_fp,
                                                             caches[s % len(caches)].c.n_q).bytes_read
                                for s in range(nb2b)]))
    achieved = attn_bytes / (attn_us * 1e-6) / 1e9

    # timed region 4: logquant_compress on a full window, on its own
    comp_us, comp_bytes = compress_leg(binding, cfg, wl, caches[1], stream)

    # the machine's pure-read ceiling at this size, live
    ceiling = read_ceiling(binding, attn_bytes, len(caches), stream)

    plan = binding.logquant_decode_plan(cfg, caches[1].c.n_fp, caches[1].c.n_q)
    counters = stored_counters(wl["name"])
    result = {
        "metric": "decode-attn effective KV tokens/sec",
        "value": wl["B"] * L / (ms_per_step * 1e-3),
        "unit": "KV tokens/s",
        "n_gpus": 1, "steps": steps, "warmup": a.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dt, "data": "synthetic",
        "config": {"workload": wl["name"], "B": wl["B"], "Hq": wl["Hq"], "Hkv": wl["Hkv"],
                   "d": wl["d"], "L": L, "group": wl["G"], "fp_budget": wl["F"], "bits": wl["bits"],
                   "cache_copies_rotated": len(caches), "compress_events_in_timed_region": n_compress,
                   "fused_append": fused, "attn_blocks": plan.blocks, "attn_splits": plan.splits,
                   "stream": "non-default", "attention_kernel": "plain vector-unit" if a.plain_valu else "matrix-instruction"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": read_traffic(wl["name"]),
                     "traffic_source": "stored: profiles/decode_attn_%s_hbm_traffic.txt (rocprofv3 --pmc runs)" % wl["name"],
                     "kernel": "decode attention", "us_per_launch": attn_us,
                     "algorithmic_bytes_per_launch": attn_bytes, "launches_timed": nb2b,
                     "single_launch_event_pair_us_p10_p50_p90": attn_event_pct,
                     "measured_read_ceiling": ceiling,
                     "frac_of_measured_read_ceiling": achieved / ceiling["GBps"],
                     "other_roofs": counters},
        "compress_us_per_call": comp_us,
        "compress": {"us_per_call": comp_us, "bytes_moved": int(comp_bytes), "GBps": comp_bytes / (comp_us * 1e-6) / 1e9,
                     "calls_timed": 24,
                     "note": "latency-bound at this batch (%.1f MB per call)" % (comp_bytes / 1e6) if comp_bytes < (32 << 20) else None},
        "kv_tokens_per_s_attention_only": wl["B"] * L / (attn_us * 1e-6),
        "token_heads_per_s": wl["B"] * wl["Hkv"] * L / (ms_per_step * 1e-3),
        "prefill": prefill,
        "state_build_s": t_build,
    }
    if a.calibration_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        result["calibration_copy_bytes"] = 256 << 20
    del caches
    torch.cuda.empty_cache()
    if not a.no_per_config and not a.plain_valu and a.bits == 2 and not a.fp_budget:
        per = []
        for w in (1, 2, 4, 5):
            if w == a.workload:
                continue
            per.append(attention_config_leg(binding, dict(inputs.WORKLOADS[w], bits=2), w, stream))
        result["per_config"] = per
    if not a.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, a.workload)
    print(json.dumps(result), flush=True)


def main_per_sequence(a, wl, steps):
    """The same measurement for a batch whose rows have different lengths: states built by
    logquant_prefill_seq, a step is logquant_decode_step_seq for every row (append_seq +
    compress_seq + decode_attn_seq at the steps where some row's window fills)."""
    import numpy as np
    import torch
    from paper_2503_19950_amd import binding, inputs
    from paper_2503_19950_amd.binding import to_dev
    B, L, dt, W = wl["B"], wl["L"], wl["dtype"], wl["F"] // 2
    wl["name"] += "_per_sequence"
    lengths = [int(x) for x in np.random.default_rng(inputs.SEED).integers(L // 2, L + 1, size=B)]
    cfg = binding.make_config(B, wl["Hq"], wl["Hkv"], wl["d"], wl["F"], wl["G"], dt, q_capacity(wl), a.bits)
    tdt = torch.bfloat16 if dt == "bf16" else torch.float16
    n_in = steps + a.warmup
    Kd = torch.empty((B, wl["Hkv"], L + n_in, wl["d"]), dtype=tdt, device="cuda:0")
    Vd = torch.empty_like(Kd)
    for t0 in range(0, L + n_in, 1 << 14):
        t1 = min(L + n_in, t0 + (1 << 14))
        K, V = inputs.batch_kv(a.workload, t0, t1, wl)
        Kd[:, :, t0:t1] = to_dev(K, dt)
        Vd[:, :, t0:t1] = to_dev(V, dt)
    one = binding.logquant_decode_plan_seq(cfg, [2 * W] * B, [(l - 2 * W) // W * slots_per_event(wl) for l in lengths])
    copies = a.copies or max(2, min(16, -(-(1 << 30) // max(1, one.bytes_read))))
    Kp, Vp = Kd[:, :, :L].contiguous(), Vd[:, :, :L].contiguous()
    caches = []
    for _ in range(copies):
        dc = binding.DeviceCacheSeq(cfg)
        dc.prefill_seq(Kp, Vp, lengths)
        caches.append(dc)
    del Kp, Vp
    # step j of a cache: row b's token at its own position lengths[b] + j
    idx = torch.tensor(lengths, device="cuda:0")
    n_new = -(-a.warmup // copies) + -(-steps // copies)      # visits per cache copy, warm-up included
    newK = torch.stack([Kd[torch.arange(B), :, idx + j] for j in range(n_new)]).unsqueeze(3).contiguous()
    newV = torch.stack([Vd[torch.arange(B), :, idx + j] for j in range(n_new)]).unsqueeze(3).contiguous()
    qs = to_dev(np.stack([inputs.queries(a.workload, s, wl) for s in range(n_in)]), dt)
    out = torch.empty_like(qs[0])
    stream = torch.cuda.current_stream()

    def run(n, visits):
        n_sep = 0
        for s in range(n):
            dc = caches[s % copies]
            j = visits[s % copies]
            visits[s % copies] += 1
            if all(dc.n_fp[b] + 1 < 3 * W for b in range(B)):
                dc.decode_step_seq(newK[j], newV[j], qs[s], out)
            else:
                dc.append_seq(newK[j], newV[j])
                dc.compress_seq()
                dc.decode_attn_seq(qs[s], out)
                n_sep += 1
        return n_sep

    visits = [0] * copies
    run(a.warmup, visits)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    n_sep = run(steps, visits)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
    nb2b = max(200, steps)
    for s in range(20):
        caches[s % copies].decode_attn_seq(qs[0], out)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for s in range(nb2b):
        caches[s % copies].decode_attn_seq(qs[0], out)
    e1.record(stream)
    torch.cuda.synchronize()
    attn_us = e0.elapsed_time(e1) * 1e3 / nb2b     # includes the small launch that hands over the counts
    dc = caches[0]
    plan = binding.logquant_decode_plan_seq(cfg, list(dc.n_fp), list(dc.n_q))
    achieved = plan.bytes_read / (attn_us * 1e-6) / 1e9
    tokens = sum(lengths)
    print(json.dumps({
        "metric": "decode-attn effective KV tokens/sec", "value": tokens / (ms_per_step * 1e-3), "unit": "KV tokens/s",
        "n_gpus": 1, "steps": steps, "warmup": a.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": dt, "data": "synthetic",
        "config": {"workload": wl["name"], "B": B, "Hq": wl["Hq"], "Hkv": wl["Hkv"], "d": wl["d"],
                   "L_min": min(lengths), "L_max": max(lengths), "L_mean": tokens / B, "group": wl["G"],
                   "fp_budget": wl["F"], "bits": wl["bits"], "cache_copies_rotated": copies,
                   "steps_with_a_compress": n_sep, "attn_blocks": plan.blocks, "attn_splits": plan.splits},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                     "kernel": "decode attention (per-sequence counts; with the launch that hands them over)",
                     "us_per_launch": attn_us, "algorithmic_bytes_per_launch": float(plan.bytes_read),
                     "launches_timed": nb2b}}), flush=True)


def stored_counters(workload_name):
    """Instruction-issue roofs of the attention kernel from the stored rocprofv3 --pmc summary
    (profiles/decode_attn_<workload>_instruction_counters.txt): the time the vector and the
    matrix instructions of one launch take if nothing else limits them (256 compute units x
    4 SIMDs, 2.4 GHz, 4 cycles per vector instruction; SQ_INSTS_VALU counts the matrix
    instructions too, so they are taken off), beside the HBM roofs above."""
    path = os.path.join(ROOT, "profiles", "decode_attn_%s_instruction_counters.txt" % workload_name)
    vals = {}
    try:
        for line in open(path):
            parts = line.split()
            if len(parts) == 2 and parts[0].startswith("SQ_"):
                vals[parts[0]] = float(parts[1])
    except OSError:
        return None
    if "SQ_INSTS_VALU" not in vals:
        return None
    simds, hz = 1024.0, 2.4e9
    out = {"source": "stored: profiles/decode_attn_%s_instruction_counters.txt" % workload_name,
           "valu_issue_us": (vals["SQ_INSTS_VALU"] - vals.get("SQ_INSTS_MFMA", 0.0)) * 4.0 / simds / hz * 1e6}
    if "SQ_VALU_MFMA_BUSY_CYCLES" in vals:
        out["mfma_busy_us"] = vals["SQ_VALU_MFMA_BUSY_CYCLES"] / simds / hz * 1e6
    return out


def read_traffic(workload_name):
    """HBM bytes per attention launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    (two runs, scaled by a plain copy of known size); the figures are kept with the
    commands that produced them in profiles/decode_attn_<workload>_hbm_traffic.txt."""
    path = os.path.join(ROOT, "profiles", "decode_attn_%s_hbm_traffic.txt" % workload_name)
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def cpu_baseline(wl, cfg_id):
    """The oracle's decode attention, as it stands, on a bounded sample of the same
    workload: a few (batch row, kv head) slices at the full context length."""
    import numpy as np
    from oracle import attention
    from tests.gpu_util import build_oracle
    from paper_2503_19950_amd import inputs
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count()
    gh = wl["Hq"] // wl["Hkv"]
    q = inputs.queries(cfg_id, 0, wl)
    t_total, n_slices = 0.0, 0
    budget_s = 12.0
    t_begin = time.perf_counter()
    for h in range(wl["Hkv"]):
        oc = build_oracle(wl, cfg_id, wl["L"], 0, h)          # state building is not timed
        best = None
        for _ in range(2):
            t0 = time.perf_counter()
            attention.decode_attention(oc, q[0, h * gh:(h + 1) * gh])
            dt_ = time.perf_counter() - t0
            best = dt_ if best is None else min(best, dt_)
        t_total += best
        n_slices += 1
        if time.perf_counter() - t_begin > budget_s:
            break
    per_slice = t_total / n_slices
    whole = per_slice * wl["B"] * wl["Hkv"]
    return {"value": wl["B"] * wl["L"] / whole, "unit": "KV tokens/s", "cores": int(cores),
            "kind": "oracle",
            "sample": "%d of %d (batch row, kv head) slices at L=%d, decode attention only, best of 2 "
                      "each, extrapolated to the whole batch" % (n_slices, wl["B"] * wl["Hkv"], wl["L"])}


if __name__ == "__main__":
    main()
