"""Helpers of the GPU parity tests: build the same cache state through the C ABI
(on the GPU) and through the oracle (on the CPU) and compare them."""
import numpy as np

from oracle import attention, layout
from oracle.cache import SliceCache
from paper_2503_19950_amd import inputs
from paper_2503_19950_amd.binding import to_dev, torch_dtype  # noqa: F401  (used by the tests through this module)

TOL = {"f16": 2e-3, "bf16": 1e-2}      # max-abs tolerance on attention outputs
MANT_BITS = {"f16": 11, "bf16": 8}     # significand bits of the output type (half an ulp of x: 2^(floor(log2 |x|) - bits))


def make_wl(**kw):
    wl = dict(B=1, Hq=4, Hkv=1, d=128, dtype="f16", G=32, F=64, dist="normal", v_outliers=False,
              sinks=0, L=0)
    wl.update(kw)
    return wl


def build_gpu(wl, seed_id, L, q_capacity=None, poison=False, b_list=None):
    """Stream L tokens of workload `wl` through logquant_append / logquant_compress."""
    from paper_2503_19950_amd import binding
    W = wl["F"] // 2
    if q_capacity is None:
        q_capacity = q_capacity_for(wl, L)
    cfg = binding.make_config(wl["B"], wl["Hq"], wl["Hkv"], wl["d"], wl["F"], wl["G"], wl["dtype"],
                              q_capacity, wl.get("bits", 2))
    dc = binding.DeviceCache(cfg, poison=poison)
    step = 3 * W * 8
    for t0 in range(0, L, step):
        t1 = min(L, t0 + step)
        K, V = inputs.batch_kv(seed_id, t0, t1, wl)
        dc.stream_in(to_dev(K, wl["dtype"]), to_dev(V, wl["dtype"]))
    return dc


def build_oracle(wl, seed_id, L, b, h):
    c = SliceCache(wl["F"] // 2, wl["G"], wl["d"], wl["dtype"], wl.get("bits", 2))
    step = 1 << 15
    for t0 in range(0, L, step):
        K, V = inputs.slice_kv(seed_id, b, h, t0, min(L, t0 + step), wl)
        c.append_block(K, V)
    return c


def _np(t, np_dtype):
    return t.cpu().numpy().view(np_dtype)


def check_state(dc, oc, wl, b, h, counts=None):
    """Bit-exact comparison of one (b, h) slice of the GPU cache with the oracle.
    counts: (cur, n_fp, n_q) of batch row b when the cache keeps them per sequence."""
    d, G, dt = wl["d"], wl["G"], wl["dtype"]
    W = wl["F"] // 2
    cap, qcap = fp_rows_allocated(W), dc.cfg.q_capacity
    nkc, ngc = d // 32, -(-d // G)
    bh = b * wl["Hkv"] + h
    cur, have_fp, have_q = counts if counts is not None else (dc.c.cur, dc.c.n_fp, dc.c.n_q)
    # the library counts quantized slots (padding behind short key groups included)
    n_fp, n_q = oc.n_fp, oc.n_q // W * layout.slots_per_event(W, G)
    assert (have_fp, have_q) == (n_fp, n_q)
    pos_fp = _np(dc.pos_fp[cur], np.int32)[b * cap:b * cap + n_fp]
    assert pos_fp.tolist() == oc.pos_fp, "fp positions"
    pos_q = _np(dc.pos_q, np.int32)[b * qcap:b * qcap + n_q]
    assert pos_q.tolist() == layout.to_slots(np.array(oc.pos_q, np.int64), W, G, fill=-1).tolist(), "quantized positions"
    for which, buf, rows in (("k", dc.k_fp[cur], oc.K_fp), ("v", dc.v_fp[cur], oc.V_fp)):
        flat = _np(buf, np.uint16)[bh * cap * d:(bh + 1) * cap * d]
        got = layout.gather_fp(flat, which, n_fp, d)
        assert np.array_equal(got, inputs.to_bits16(rows, dt)), "fp rows " + which
    if n_q == 0:
        return
    bits = wl.get("bits", 2)
    nw = n_q // 32 * 64 * nkc * (bits // 2)
    for which, buf, codes in (("k", dc.k_codes, oc.K_codes), ("v", dc.v_codes, oc.V_codes)):
        words = _np(buf, np.uint32)[bh * (qcap // 32) * 64 * nkc * (bits // 2):][:nw]
        want = layout.pack_codes(layout.to_slots(codes, W, G), which, bits=bits)   # padding slots: zero codes
        assert np.array_equal(words, want), "packed codes " + which
    # scales and zero-points are values of T, stored as fp16 whatever T is
    for buf, meta, name in ((dc.k_scale, oc.K_scale, "k_scale"), (dc.k_zero, oc.K_zero, "k_zero")):
        got = _np(buf, np.uint16)[bh * (qcap // G) * d:][:n_q // G * d]
        assert np.array_equal(got, inputs.to_bits16(meta, "f16").ravel()), name
    for buf, meta, name in ((dc.v_scale, oc.V_scale, "v_scale"), (dc.v_zero, oc.V_zero, "v_zero")):
        got = _np(buf, np.uint16)[bh * (qcap // 32) * ngc * 32:][:n_q // 32 * ngc * 32]
        want = layout.scatter_v_meta(layout.to_slots(inputs.to_bits16(meta, "f16"), W, G), d, G)   # padding: zeros
        assert np.array_equal(got, want), name


def check_attention(dc, oc_by_slice, wl, q_np, scale=0.0):
    """Run logquant_decode_attn for the whole batch; compare the heads of the given
    (b, h) slices with the oracle (bound: assert_outputs_close).  Returns the largest
    abs error seen."""
    dt = wl["dtype"]
    gh = wl["Hq"] // wl["Hkv"]
    out = dc.decode_attn(to_dev(q_np, dt), softmax_scale=scale)
    import torch
    torch.cuda.synchronize()
    out = out.float().cpu().numpy()
    assert np.isfinite(out).all()
    worst = 0.0
    for (b, h), oc in oc_by_slice.items():
        want = attention.decode_attention(oc, q_np[b, h * gh:(h + 1) * gh], scale if scale > 0 else None)
        worst = max(worst, assert_outputs_close(out[b, h * gh:(h + 1) * gh], want, dt,
                                                "attention (b=%d,h=%d)" % (b, h)))
    return worst


# running totals over a test session: elements compared, and of those the ones that fell
# into the band where the bound is relaxed (printed by conftest at the end of the run)
BAND_STATS = {"compared": 0, "relaxed": 0, "worst_plain": 0.0, "worst_relaxed_vs_rounded_ulps": 0.0}


def half_ulp_in_T(x, dt):
    """Half a unit in the last place of |x| as a value of T (normal range)."""
    e = np.floor(np.log2(np.maximum(np.abs(x), 2.0 ** -14)))
    return 2.0 ** (e - MANT_BITS[dt])


# Relative size of what the kernel's own arithmetic contributes before the output is rounded to
# T (fp32 logits of tens of nats carry ~1e-5 nats of rounding noise, which moves an output by
# about that fraction of the spread of the value rows; bf16 caches also round the products
# p * vs once to fp16).  Only used to find the one band where the stated tolerance leaves less
# room than that beside the rounding to T itself: fp16 outputs with 4 <= |o| < 8, where half an
# ulp is 1.953e-3 of the 2e-3.
COMPUTE_NOISE = {"f16": 2.0 ** -15, "bf16": 2.0 ** -12}


def output_bound(want, dt):
    """Elementwise bound on |output - oracle| (see assert_outputs_close), the mask of the
    elements where it is relaxed by half an ulp, and that half ulp."""
    want = np.asarray(want, np.float64)
    hu = half_ulp_in_T(want, dt)
    relaxed = hu > TOL[dt]
    noise = COMPUTE_NOISE[dt] * np.abs(want)
    no_room = ~relaxed & (TOL[dt] - hu < noise)
    return TOL[dt] + np.where(relaxed, hu, 0.0) + np.where(no_room, noise, 0.0), relaxed, hu


def assert_outputs_close(got, want, dt, where):
    """Attention outputs against the oracle's fp64 result: max-abs error <= TOL (2e-3 for
    fp16, 1e-2 for bf16) for every element whose half ulp in T is at most TOL, i.e.
    wherever a correctly rounded result of type T meets the tolerance (bf16 |o| < 4,
    fp16 |o| < 8).  Only above that, where no value of T can be held to TOL, the bound
    adds that half ulp, and the result must also lie within one ulp of the oracle's value
    rounded to T.  One band is left with less room than fp32 arithmetic needs beside the
    rounding to T (fp16, 4 <= |o| < 8: 4.7e-5); there the bound is TOL + 2^-15 |o|
    (at most 2.25e-3).  Returns the largest abs error."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    diff = np.abs(got - want)
    bound, relaxed, hu = output_bound(want, dt)
    BAND_STATS["compared"] += diff.size
    BAND_STATS["relaxed"] += int(relaxed.sum())
    if (~relaxed).any():
        BAND_STATS["worst_plain"] = max(BAND_STATS["worst_plain"], float(diff[~relaxed].max()))
    bad = diff > bound
    assert not bad.any(), "%s: abs err %.3e at |o| = %.3f, tolerance %.1e" % (
        where, diff[bad].max(), np.abs(want)[bad].max(), TOL[dt])
    if relaxed.any():
        want_T = inputs.to_T(want.astype(np.float32), dt).astype(np.float64)
        ulps = np.abs(got - want_T)[relaxed] / (2.0 * hu[relaxed])
        BAND_STATS["worst_relaxed_vs_rounded_ulps"] = max(BAND_STATS["worst_relaxed_vs_rounded_ulps"],
                                                          float(ulps.max()))
        assert ulps.max() <= 1.0, "%s: %.2f ulp from the oracle rounded to %s at |o| = %.3f" % (
            where, ulps.max(), dt, np.abs(want)[relaxed][ulps.argmax()])
        BAND_STATS["calls_with_relaxed"] = BAND_STATS.get("calls_with_relaxed", 0) + 1
        if BAND_STATS["calls_with_relaxed"] <= 12 or relaxed.sum() > diff.size // 4:
            print("  %s: %d of %d outputs have half an ulp above the tolerance (|o| up to %.1f); there: max err %.3e "
                  "against fp64, %.2f ulp against the oracle rounded to %s" % (
                      where, int(relaxed.sum()), diff.size, np.abs(want).max(), diff[relaxed].max(), ulps.max(), dt),
                  flush=True)
    return float(diff.max())


def same_up_to_order_noise(x, y, dt, where):
    """Two outputs of the HIP path for the same mathematical input that differ only in the
    order in which the rows are visited (row order in memory, number of context splits).
    What depends on that order: the order of the fp32 sums, and the moments at which the
    running maximum of the online softmax moves, which decide how the probabilities (and,
    for bf16 caches, the products p * vs) are rounded to fp16 - all of it part of the
    kernel's arithmetic noise COMPUTE_NOISE, relative to the magnitude of the head's values.
    Bound per element: ulp_T(|o|) + 4 * COMPUTE_NOISE * max(1, max |o| of the head), i.e.
    1.2e-4 (fp16) / 9.8e-4 (bf16) for outputs of order one: a sixteenth / a tenth of the
    output tolerance.  Returns (largest excess over one ulp as a fraction of that
    allowance, number of elements that differ)."""
    x = np.asarray(x, np.float64)
    y = np.asarray(y, np.float64)
    ulp = 2.0 * half_ulp_in_T(np.maximum(np.abs(x), np.abs(y)), dt)
    allow = 4.0 * COMPUTE_NOISE[dt] * np.maximum(1.0, np.abs(x).max(axis=-1, keepdims=True)) * np.ones_like(x)
    excess = (np.abs(x - y) - ulp) / allow
    i = excess.argmax()
    assert excess.ravel()[i] <= 1.0, "%s: |diff| %.3e at |o| = %.3e (one ulp there: %.3e, noise allowance %.1e)" % (
        where, np.abs(x - y).ravel()[i], np.abs(x).ravel()[i], ulp.ravel()[i], allow.ravel()[i])
    return float(excess.max()), int((x != y).sum())


def batch_kv_sampled(seed_id, t0, t1, wl, distinct):
    """[B][Hkv][n][d] K and V in which only the slices listed in `distinct` (and the
    eight filler slices (0, 0..7)) carry their own seeded data; every other slice
    repeats one of the fillers.  Used at sizes where drawing every slice would take
    minutes; the launch shape is that of the full workload."""
    B, H, d = wl["B"], wl["Hkv"], wl["d"]
    n = t1 - t0
    K = np.empty((B, H, n, d), np.float32)
    V = np.empty((B, H, n, d), np.float32)
    fill = [inputs.slice_kv(seed_id, 0, h % H, t0, t1, wl) for h in range(min(8, H))]
    own = {bh: inputs.slice_kv(seed_id, bh[0], bh[1], t0, t1, wl) for bh in distinct}
    for b in range(B):
        for h in range(H):
            k, v = own.get((b, h)) or fill[(b * H + h) % len(fill)]
            K[b, h], V[b, h] = k, v
    return K, V


def build_gpu_sampled(wl, seed_id, L, distinct, q_capacity=None):
    from paper_2503_19950_amd import binding
    W = wl["F"] // 2
    if q_capacity is None:
        q_capacity = (L // W + 2) * W
        while q_capacity % 64:
            q_capacity += W
    cfg = binding.make_config(wl["B"], wl["Hq"], wl["Hkv"], wl["d"], wl["F"], wl["G"], wl["dtype"],
                              q_capacity, wl.get("bits", 2))
    dc = binding.DeviceCache(cfg)
    step = 3 * W * 8
    for t0 in range(0, L, step):
        t1 = min(L, t0 + step)
        K, V = batch_kv_sampled(seed_id, t0, t1, wl, distinct)
        dc.stream_in(to_dev(K, wl["dtype"]), to_dev(V, wl["dtype"]))
        print("  streamed", t1, "of", L, flush=True)
    return dc


def q_capacity_for(wl, L):
    """A valid q_capacity (multiple of the slots of one event and of 64) with room for L tokens."""
    W = wl["F"] // 2
    Wq = layout.slots_per_event(W, wl["G"])
    q_capacity = max(64, -(-L // (2 * W)) * 2 * Wq)
    while q_capacity % 64 or q_capacity % Wq:
        q_capacity += Wq
    return q_capacity


def fp_rows_allocated(W):
    """Rows per slice of the fp buffers: 3W rounded up to whole 32-row tiles."""
    return -(-3 * W // 32) * 32


def new_cache(wl, L, q_capacity=None, poison=False):
    from paper_2503_19950_amd import binding
    if q_capacity is None:
        q_capacity = q_capacity_for(wl, L)
    cfg = binding.make_config(wl["B"], wl["Hq"], wl["Hkv"], wl["d"], wl["F"], wl["G"], wl["dtype"],
                              q_capacity, wl.get("bits", 2))
    return binding.DeviceCache(cfg, poison=poison)


def build_gpu_prefill(wl, seed_id, L, q_capacity=None, poison=False, kv=None):
    """The same state as build_gpu, through one logquant_prefill call."""
    dc = new_cache(wl, L, q_capacity, poison)
    K, V = kv if kv is not None else inputs.batch_kv(seed_id, 0, L, wl)
    dc.prefill(to_dev(K, wl["dtype"]), to_dev(V, wl["dtype"]))
    return dc


def live_buffers(dc, wl):
    """Every buffer of the cache restricted to what the counts make meaningful, as numpy."""
    d, G = wl["d"], wl["G"]
    W = wl["F"] // 2
    cap, qcap, BH = fp_rows_allocated(W), dc.cfg.q_capacity, wl["B"] * wl["Hkv"]
    nkc, ngc = d // 32, -(-d // G)
    cur, n_fp, n_q = dc.c.cur, dc.c.n_fp, dc.c.n_q
    out = {"counts": np.array([n_fp, n_q])}
    out["pos_fp"] = _np(dc.pos_fp[cur], np.int32).reshape(wl["B"], cap)[:, :n_fp]
    out["pos_q"] = _np(dc.pos_q, np.int32).reshape(wl["B"], qcap)[:, :n_q]
    for which, buf in (("k", dc.k_fp[cur]), ("v", dc.v_fp[cur])):
        flat = _np(buf, np.uint16).reshape(BH, cap * d)
        out["fp_" + which] = np.stack([layout.gather_fp(flat[i], which, n_fp, d) for i in range(BH)])
    wpl = nkc * (wl.get("bits", 2) // 2)
    out["k_codes"] = _np(dc.k_codes, np.uint32).reshape(BH, -1)[:, :n_q // 32 * 64 * wpl]
    out["v_codes"] = _np(dc.v_codes, np.uint32).reshape(BH, -1)[:, :n_q // 32 * 64 * wpl]
    out["k_scale"] = _np(dc.k_scale, np.uint16).reshape(BH, -1)[:, :n_q // G * d]
    out["k_zero"] = _np(dc.k_zero, np.uint16).reshape(BH, -1)[:, :n_q // G * d]
    out["v_scale"] = _np(dc.v_scale, np.uint16).reshape(BH, -1)[:, :n_q // 32 * ngc * 32]
    out["v_zero"] = _np(dc.v_zero, np.uint16).reshape(BH, -1)[:, :n_q // 32 * ngc * 32]
    return out
