"""Streaming cache state of one (batch row, kv head) slice.  Test infrastructure only.

Rows of K and V follow Algorithm 1 (Sec. 2.5): tokens are appended to the
original-precision list; when it holds 3W rows the even logical rows below 2W
and the newest W rows stay, the odd logical rows below 2W leave.  Fig. 6's
caption and Sec. 2.3 say the leaving rows are quantized rather than dropped;
they are quantized once, at the event that evicts them, and appended to the
quantized region in eviction order (Sec. 2.4: storage order is free).
"""
import numpy as np

from . import selection
from . import quantizer


class SliceCache:
    def __init__(self, W, G, d, dtype, bits=2):
        self.W, self.G, self.d, self.dtype, self.bits = W, G, d, dtype, bits
        self.pos_fp = []                                   # absolute positions, logical order
        self.K_fp = np.zeros((0, d), dtype=np.float32)     # exact values of T
        self.V_fp = np.zeros((0, d), dtype=np.float32)
        ngc = -(-d // G)
        self.pos_q = []
        # quantized region, one chunk per compress event (joined on demand):
        # K_codes/V_codes [n_q][d] uint8, K_scale/K_zero [events * ceil(W/G)][d],
        # V_scale/V_zero [n_q][ceil(d/G)]
        self._chunks = {"K_codes": [np.zeros((0, d), np.uint8)],
                        "V_codes": [np.zeros((0, d), np.uint8)],
                        "K_scale": [np.zeros((0, d), np.float32)],
                        "K_zero": [np.zeros((0, d), np.float32)],
                        "V_scale": [np.zeros((0, ngc), np.float32)],
                        "V_zero": [np.zeros((0, ngc), np.float32)]}
        self.n_total = 0
        self.events = 0

    @property
    def n_fp(self):
        return len(self.pos_fp)

    @property
    def n_q(self):
        return len(self.pos_q)

    def append(self, k_row, v_row):
        """Append one token; run the filtering step when the list reaches 3W
        (eager trigger, see selection.stream_eager)."""
        self.pos_fp = self.pos_fp + [self.n_total]
        self.n_total += 1
        self.K_fp = np.concatenate([self.K_fp, np.asarray(k_row, np.float32)[None]], 0)
        self.V_fp = np.concatenate([self.V_fp, np.asarray(v_row, np.float32)[None]], 0)
        if len(self.pos_fp) == 3 * self.W:
            self.compress()

    def append_block(self, K, V):
        """Append rows one event at a time (same result as row-by-row append)."""
        K = np.asarray(K, np.float32)
        V = np.asarray(V, np.float32)
        i = 0
        while i < K.shape[0]:
            room = 3 * self.W - len(self.pos_fp)
            n = min(room, K.shape[0] - i)
            self.pos_fp = self.pos_fp + list(range(self.n_total, self.n_total + n))
            self.n_total += n
            self.K_fp = np.concatenate([self.K_fp, K[i:i + n]], 0)
            self.V_fp = np.concatenate([self.V_fp, V[i:i + n]], 0)
            i += n
            if len(self.pos_fp) == 3 * self.W:
                self.compress()

    def compress(self):
        W = self.W
        kept, evicted = selection.compress_event(self.pos_fp, W)
        # the same slices, applied to the rows
        K_ev, V_ev = self.K_fp[1:2 * W:2], self.V_fp[1:2 * W:2]
        self.K_fp = np.concatenate([self.K_fp[0:2 * W:2], self.K_fp[2 * W:3 * W]], 0)
        self.V_fp = np.concatenate([self.V_fp[0:2 * W:2], self.V_fp[2 * W:3 * W]], 0)
        self.pos_fp = kept
        kc, ks, kz = quantizer.quantize_keys(K_ev, self.G, self.dtype, self.bits)
        vc, vs, vz = quantizer.quantize_values(V_ev, self.G, self.dtype, self.bits)
        self.pos_q = self.pos_q + evicted
        for name, arr in (("K_codes", kc), ("V_codes", vc), ("K_scale", ks),
                          ("K_zero", kz), ("V_scale", vs), ("V_zero", vz)):
            self._chunks[name].append(arr)
        self.events += 1

    def _joined(self, name):
        ch = self._chunks[name]
        if len(ch) > 1:
            self._chunks[name] = ch = [np.concatenate(ch, 0)]
        return ch[0]

    K_codes = property(lambda self: self._joined("K_codes"))
    V_codes = property(lambda self: self._joined("V_codes"))
    K_scale = property(lambda self: self._joined("K_scale"))
    K_zero = property(lambda self: self._joined("K_zero"))
    V_scale = property(lambda self: self._joined("V_scale"))
    V_zero = property(lambda self: self._joined("V_zero"))

    def rows_fp64(self):
        """All rows the decode step attends over: fp rows, then dequantized rows."""
        Kq = quantizer.dequantize_keys(self.K_codes, self.K_scale, self.K_zero, self.G, self.W)
        Vq = quantizer.dequantize_values(self.V_codes, self.V_scale, self.V_zero, self.G)
        K = np.concatenate([self.K_fp.astype(np.float64), Kq], 0)
        V = np.concatenate([self.V_fp.astype(np.float64), Vq], 0)
        return K, V
