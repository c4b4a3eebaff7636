"""Seeded synthetic inputs for the five benchmark workloads.

This module holds no arithmetic of the method: it only draws random tensors
with the shapes and value structure of the workloads (normal or Laplace
entries, a few key channels scaled up as outlier channels, a few leading rows
scaled up as attention sinks) and rounds them once to the cache type.  Both the
HIP path and the CPU oracle are fed from here.  The tensors stand in for the
real-model KV states the paper measures on (Sec. 3.1: Llama-3-class grouped
query models, Qwen1.5/Phi-3-class multi-head models), which need weights and
datasets that are not available offline.

Values are returned as float32 arrays that hold numbers exactly representable
in the cache type ("f16" or "bf16").
"""
import numpy as np

SEED = 2503_19950
CHUNK = 4096          # tokens per independently seeded chunk of a slice
T_K, T_V, T_Q, T_OUTLIER_K, T_OUTLIER_V = 0, 1, 2, 3, 4

# B, Hq, Hkv, d, L (tokens in the cache when the decode step is measured),
# dtype, G (group size), F (fp budget = 2W), dist, and the structure knobs:
#   four key channels per kv head are always scaled x10 (outlier channels);
#   v_outliers: also scale four (independently drawn) value channels x10;
#   sinks: number of leading positions whose KEY rows are scaled x5 (tokens that
#          attract attention); sink_v: scale their value rows as well.
# Workload 3 carries the structure on both tensors, as its text states ("K,V ~ N(0,1) plus
# outlier channels x10 and a few per-token attention-sink rows scaled x5").
WORKLOADS = {
    1: dict(name="cfg1_small_L512", B=1, Hq=32, Hkv=8, d=128, L=512, dtype="f16", G=32, F=128,
            dist="normal", v_outliers=False, sinks=0),
    2: dict(name="cfg2_llama3_8b_B8_L8192", B=8, Hq=32, Hkv=8, d=128, L=8192, dtype="f16", G=32,
            F=256, dist="normal", v_outliers=False, sinks=0),
    3: dict(name="cfg3_long_context_L131072", B=1, Hq=32, Hkv=8, d=128, L=131072, dtype="bf16",
            G=64, F=512, dist="normal", v_outliers=True, sinks=4, sink_v=True),
    4: dict(name="cfg4_batch64_L4096_128steps", B=64, Hq=32, Hkv=8, d=128, L=4096, dtype="f16",
            G=32, F=256, dist="normal", v_outliers=False, sinks=0, steps=128),
    5: dict(name="cfg5_mha_d96_L32768", B=16, Hq=32, Hkv=32, d=96, L=32768, dtype="bf16", G=64,
            F=384, dist="laplace", v_outliers=False, sinks=0),
}


def to_T(x, dtype):
    """Round float32 to the cache type (nearest, ties to even), keep as float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f16":
        return x.astype(np.float16).astype(np.float32)
    if dtype == "bf16":
        u = x.view(np.uint32)
        r = ((u.astype(np.uint64) + 0x7FFF + ((u >> 16) & 1)) >> 16 << 16).astype(np.uint32)
        return r.view(np.float32)
    raise ValueError(dtype)


def to_bits16(x, dtype):
    """float32 array of exact T values -> uint16 bit patterns of T."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f16":
        return x.astype(np.float16).view(np.uint16)
    return (x.view(np.uint32) >> 16).astype(np.uint16)


def from_bits16(u, dtype):
    u = np.ascontiguousarray(u, dtype=np.uint16)
    if dtype == "f16":
        return u.view(np.float16).astype(np.float32)
    return (u.astype(np.uint32) << 16).view(np.float32)


def _rng(*key):
    return np.random.Generator(np.random.PCG64([SEED, *key]))


def outlier_channels(cfg_id, h, d, tensor):
    """Four fixed channels per kv head (a property of the 'model', not of the
    batch row)."""
    return np.sort(_rng(cfg_id, h, tensor).choice(d, size=4, replace=False))


def _draw(rng, shape, dist):
    if dist == "laplace":
        return rng.laplace(0.0, 1.0, size=shape).astype(np.float32)
    return rng.standard_normal(size=shape, dtype=np.float32)


def slice_kv(cfg_id, b, h, t0, t1, wl=None):
    """K and V rows t0..t1-1 of batch row b, kv head h: two [t1-t0][d] arrays."""
    wl = wl or WORKLOADS[cfg_id]
    d = wl["d"]
    out = []
    for tensor, outl in ((T_K, True), (T_V, wl["v_outliers"])):
        parts = []
        for ch in range(t0 // CHUNK, (max(t1, t0 + 1) - 1) // CHUNK + 1):
            x = _draw(_rng(cfg_id, b, h, tensor, ch), (CHUNK, d), wl["dist"])
            lo, hi = max(t0, ch * CHUNK), min(t1, (ch + 1) * CHUNK)
            parts.append(x[lo - ch * CHUNK:hi - ch * CHUNK])
        x = np.concatenate(parts, 0) if parts else np.zeros((0, d), np.float32)
        if outl:
            x[:, outlier_channels(cfg_id, h, d, T_OUTLIER_K if tensor == T_K else T_OUTLIER_V)] *= 10.0
        if wl["sinks"] and t0 < wl["sinks"] and (tensor == T_K or wl.get("sink_v", False)):
            x[:max(0, min(wl["sinks"], t1) - t0)] *= 5.0
        if wl.get("gain", 1.0) != 1.0:      # whole tensor scaled (test cases at the edge of the value range)
            x *= np.float32(wl["gain"])
        out.append(to_T(x, wl["dtype"]))
    return out[0], out[1]


def batch_kv(cfg_id, t0, t1, wl=None):
    """[B][Hkv][t1-t0][d] K and V for all slices (float32 holding T values)."""
    wl = wl or WORKLOADS[cfg_id]
    B, H, d = wl["B"], wl["Hkv"], wl["d"]
    K = np.empty((B, H, t1 - t0, d), np.float32)
    V = np.empty((B, H, t1 - t0, d), np.float32)
    for b in range(B):
        for h in range(H):
            K[b, h], V[b, h] = slice_kv(cfg_id, b, h, t0, t1, wl)
    return K, V


def queries(cfg_id, step=0, wl=None):
    """[B][Hq][d] query of decode step `step` (float32 holding T values)."""
    wl = wl or WORKLOADS[cfg_id]
    x = _draw(_rng(cfg_id, T_Q, step), (wl["B"], wl["Hq"], wl["d"]), "normal")
    return to_T(x, wl["dtype"])


# ---------------------------------------------------------------------------
# Spiky variant of a slice, for the attention-error diagnostic (the paper's Sec. 2.2
# observes that the positions which attract attention thin out with their distance
# from the newest token roughly like 1/distance; Table 2 measures what that means for
# quantizing or evicting the other tokens).  A fixed unit direction per kv head is
# added to the key rows of `n_spikes` positions whose distance from the newest token
# is log-uniform, and to every query, so those positions carry most of the attention
# mass.  Pure data generation: nothing of the method is computed here.
T_TOPIC, T_SPIKES = 5, 6


def topic_direction(cfg_id, h, d):
    u = _rng(cfg_id, h, T_TOPIC).standard_normal(d)
    return (u / np.linalg.norm(u)).astype(np.float32)


def spike_positions(cfg_id, b, h, L, n_spikes):
    """Distinct positions in [0, L): distance to position L-1 is floor(L**U), U uniform."""
    u = _rng(cfg_id, b, h, T_SPIKES).random(4 * n_spikes)
    dist = np.floor(np.exp(u * np.log(L))).astype(np.int64)
    pos = np.unique(np.clip(L - 1 - dist, 0, L - 1))
    return pos[-n_spikes:] if pos.size > n_spikes else pos


def slice_kv_spiky(cfg_id, b, h, L, wl=None, n_spikes=48, gain=12.0):
    """slice_kv(…, 0, L) with the topic direction added to the spike rows of K."""
    wl = wl or WORKLOADS[cfg_id]
    K, V = slice_kv(cfg_id, b, h, 0, L, wl)
    pos = spike_positions(cfg_id, b, h, L, n_spikes)
    K = K.copy()
    K[pos] += gain * topic_direction(cfg_id, h, wl["d"])
    return to_T(K, wl["dtype"]), V, pos


def queries_spiky(cfg_id, step=0, wl=None, gain=12.0):
    """queries(…) with each head's query shifted along its kv head's topic direction."""
    wl = wl or WORKLOADS[cfg_id]
    q = queries(cfg_id, step, wl).copy()
    gh = wl["Hq"] // wl["Hkv"]
    for h in range(wl["Hkv"]):
        q[:, h * gh:(h + 1) * gh] += gain * topic_direction(cfg_id, h, wl["d"])
    return to_T(q, wl["dtype"])
