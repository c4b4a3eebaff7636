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
    plan0 = None
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
    stream = torch.cuda.current_stream()
    sh = stream.cuda_stream

    fused = not a.unfused

    def run(n, record):
        """n steps; returns per-kernel event pairs when record is True (then with the
        separate append / compress / attention calls, so that each can be bracketed)."""
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
                if record:
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(stream)
                st = binding.logquant_compress(cfg, dc.c, dc.workspace, sh)
                assert st == 0, binding.logquant_status_string(st)
                n_compress += 1
                if record:
                    e1.record(stream)
                    ev.append(("compress", e0, e1, 0))
            if record:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                nbytes = binding.logquant_decode_plan(cfg, dc.c.n_fp, dc.c.n_q).bytes_read
                e0.record(stream)
            st = binding.logquant_decode_attn(cfg, dc.c, qs[s], 0.0, out, dc.workspace, sh)
            assert st == 0, binding.logquant_status_string(st)
            if record:
                e1.record(stream)
                ev.append(("attn", e0, e1, nbytes))
        return ev, n_compress

    saved = [dc.counts() for dc in caches]
    run(a.warmup, False)
    torch.cuda.synchronize()
    for dc, c in zip(caches, saved):
        dc.set_counts(c)

    # timed region 1: the whole hot path, K steps, wall clock
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    _, n_compress = run(steps, False)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps
    for dc, c in zip(caches, saved):
        dc.set_counts(c)

    # timed region 2: the same K steps with HIP events around every attention / compress
    # launch (same stream), for the per-kernel durations the roofline is computed from
    ev, _ = run(steps, True)
    torch.cuda.synchronize()
    attn = [(e0.elapsed_time(e1) * 1e3, nb) for k, e0, e1, nb in ev if k == "attn"]
    comp = [e0.elapsed_time(e1) * 1e3 for k, e0, e1, nb in ev if k == "compress"]
    attn_event_us = float(np.mean([t for t, _ in attn]))   # includes the event markers' own cost
    attn_event_pct = [float(x) for x in np.percentile([t for t, _ in attn], [10, 50, 90])]

    # timed region 3: the attention launches alone, back to back on the launch stream,
    # rotating over the cache copies, one HIP event before and one after.  Kernel
    # durations measured this way agree with rocprofv3's kernel trace (an event pair
    # around every single launch adds several microseconds of marker cost), so the
    # roofline figures are taken from here.
    for dc, c in zip(caches, saved):
        dc.set_counts(c)
    nb2b = max(200, steps)
    for s in range(20):
        binding.logquant_decode_attn(cfg, caches[s % len(caches)].c, qs[0], 0.0, out,
                                     caches[s % len(caches)].workspace, sh)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for s in range(nb2b):
        dc = caches[s % len(caches)]
        binding.logquant_decode_attn(cfg, dc.c, qs[0], 0.0, out, dc.workspace, sh)
    e1.record(stream)
    torch.cuda.synchronize()
    b2b_us = e0.elapsed_time(e1) * 1e3 / nb2b
    b2b_bytes = float(np.mean([binding.logquant_decode_plan(cfg, caches[s % len(caches)].c.n_fp,
                                                            caches[s % len(caches)].c.n_q).bytes_read
                               for s in range(nb2b)]))
    attn_us, attn_bytes = b2b_us, b2b_bytes
    achieved = attn_bytes / (attn_us * 1e-6) / 1e9

    plan = binding.logquant_decode_plan(cfg, caches[1].c.n_fp, caches[1].c.n_q)
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
                   "fused_append": not a.unfused, "attn_blocks": plan.blocks, "attn_splits": plan.splits},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                     "kernel": "decode attention", "us_per_launch": attn_us,
                     "algorithmic_bytes_per_launch": attn_bytes, "launches_timed": nb2b,
                     "in_step_loop_event_pair_us": attn_event_us,
                     "single_launch_event_pair_us_p10_p50_p90": attn_event_pct,
                     "plain_copy_reference_GBps": plain_copy_reference()},
        "compress_us_per_call": float(np.mean(comp)) if comp else None,
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
    result["roofline"]["traffic"] = read_traffic(wl["name"])
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


def plain_copy_reference():
    """What plain streaming reaches on this machine, for scale: a device-to-device copy of 1 GiB
    (four times the last-level cache), bytes read plus bytes written over time, best of 5."""
    import torch
    src = torch.ones(1 << 30, dtype=torch.uint8, device="cuda:0")
    dst = torch.empty_like(src)
    best = None
    for i in range(7):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        dst.copy_(src)
        e1.record()
        torch.cuda.synchronize()
        if i >= 2:
            t = e0.elapsed_time(e1)
            best = t if best is None else min(best, t)
    return 2.0 * src.numel() / (best * 1e-3) / 1e9


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
