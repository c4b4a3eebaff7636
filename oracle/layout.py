"""Physical index functions of the cache buffers.  Test infrastructure only.

Sec. 2.4 / Eq. 3 of the paper make the storage order of rows free; the library
documents (in its public header) where element (slot t, channel c) of one
(batch row, kv head) slice lives in each buffer.  This module restates those
index functions from that documentation, vectorised with numpy, so that the
oracle's logical arrays can be turned into the exact words the library must
produce.  All functions work on ONE (b, h) slice and return offsets relative
to the start of that slice.
"""
import numpy as np


def kperm(x):
    x = np.asarray(x)
    return 8 * ((x % 16) // 4) + 4 * (x // 16) + (x % 4)


def k_fp_index(t, c, d):
    """Element index (in units of T) of fp key (slot t, channel c)."""
    nkc = d // 32
    return (((t // 16) * nkc + c // 32) * 64 + 16 * ((c % 32) // 8) + t % 16) * 8 + c % 8


def v_fp_index(t, c, d):
    nnt = d // 16
    k = kperm(t % 32)
    return (((t // 32) * nnt + c // 16) * 64 + 16 * (k // 8) + c % 16) * 8 + k % 8


def k_code_word_bit(t, c, d, bits=2):
    """(word index, first bit) of the key code of (slot t, channel c)."""
    nkc = d // 32
    o = ((t % 32) // 16) * nkc + c // 32
    lane = 16 * ((c % 32) // 8) + t % 16
    if bits == 2:
        word = ((t // 32) * 64 + lane) * nkc + o // 2
        bit = 8 * (o % 2) + 2 * ((c % 8) // 2) + 16 * (c % 2)
    else:
        word = ((t // 32) * 64 + lane) * 2 * nkc + o
        bit = 4 * ((c % 8) // 2) + 16 * (c % 2)
    return word, bit


def v_code_word_bit(t, c, d, bits=2):
    nkc = d // 32
    k = kperm(t % 32)
    lane = 16 * (k // 8) + c % 16
    if bits == 2:
        word = ((t // 32) * 64 + lane) * nkc + (c // 16) // 2
        bit = 8 * ((c // 16) % 2) + 2 * ((k % 8) // 2) + 16 * (k % 2)
    else:
        word = ((t // 32) * 64 + lane) * 2 * nkc + c // 16
        bit = 4 * ((k % 8) // 2) + 16 * (k % 2)
    return word, bit


def k_meta_index(t, c, d, G):
    return (t // G) * d + c


def v_meta_index(t, c, d, G):
    ngc = -(-d // G)
    return ((t // 32) * ngc + c // G) * 32 + kperm(t % 32)


def _grid(n, d):
    t = np.arange(n)[:, None]
    c = np.arange(d)[None, :]
    return t, c


def pack_codes(codes, which, n_slots_alloc=None, bits=2):
    """codes uint8 [n][d] (values below 2^bits) -> uint32 words of one slice.

    `which` is 'k' or 'v'.  The result covers ceil(n/32) blocks of 32 slots
    (or n_slots_alloc/32 blocks when given); untouched bits are zero."""
    n, d = codes.shape
    n_alloc = n_slots_alloc if n_slots_alloc is not None else -(-n // 32) * 32
    words = np.zeros(n_alloc // 32 * 64 * (d // 32) * (bits // 2), dtype=np.uint32)
    t, c = _grid(n, d)
    fn = k_code_word_bit if which == "k" else v_code_word_bit
    w, b = fn(t, c, d, bits)
    w = np.broadcast_to(w, (n, d)).ravel()
    b = np.broadcast_to(b, (n, d)).ravel().astype(np.uint32)
    np.bitwise_or.at(words, w, codes.ravel().astype(np.uint32) << b)
    return words


def unpack_codes(words, which, n, d, bits=2):
    t, c = _grid(n, d)
    fn = k_code_word_bit if which == "k" else v_code_word_bit
    w, b = fn(t, c, d, bits)
    return ((words[w] >> b.astype(np.uint32)) & np.uint32((1 << bits) - 1)).astype(np.uint8)


def scatter_fp(rows, which, cap):
    """rows [n][d] -> flat array of cap*d elements in the fp buffer's order
    (slots >= n left at zero)."""
    n, d = rows.shape
    out = np.zeros(cap * d, dtype=rows.dtype)
    t, c = _grid(n, d)
    idx = (k_fp_index if which == "k" else v_fp_index)(t, c, d)
    out[np.broadcast_to(idx, (n, d)).ravel()] = rows.ravel()
    return out


def gather_fp(flat, which, n, d):
    t, c = _grid(n, d)
    idx = (k_fp_index if which == "k" else v_fp_index)(t, c, d)
    return flat[np.broadcast_to(idx, (n, d))]


# Scales and zero-points are stored as fp16 bit patterns whatever the cache type (the
# library's header says so); the scatter functions below only place 16-bit patterns.
def scatter_k_meta(meta, d, G):
    """meta [n_q/G][d] -> flat (identity order: group-major, channel-minor)."""
    return np.ascontiguousarray(meta).ravel()


def scatter_v_meta(meta, d, G, n_slots_alloc=None):
    """meta [n][ceil(d/G)] -> flat array in the v_scale / v_zero order."""
    n, ngc = meta.shape
    n_alloc = n_slots_alloc if n_slots_alloc is not None else -(-n // 32) * 32
    out = np.zeros(n_alloc // 32 * ngc * 32, dtype=meta.dtype)
    t = np.arange(n)[:, None]
    g = np.arange(ngc)[None, :]
    idx = ((t // 32) * ngc + g) * 32 + kperm(t % 32)
    out[idx.ravel()] = meta.ravel()
    return out


def gather_v_meta(flat, n, d, G):
    ngc = -(-d // G)
    t = np.arange(n)[:, None]
    g = np.arange(ngc)[None, :]
    return flat[((t // 32) * ngc + g) * 32 + kperm(t % 32)]


def slots_per_event(W, G):
    """Quantized slots one filtering event occupies: ceil(W/G) * G."""
    return -(-W // G) * G


def token_slots(n_tok, W, G):
    """Slot of the i-th quantized token (eviction order): events of W tokens each start
    at a multiple of slots_per_event; the slots behind a short last group are padding."""
    i = np.arange(n_tok)
    return (i // W) * slots_per_event(W, G) + i % W


def to_slots(rows, W, G, fill=0):
    """[n_tok][...] in eviction order -> [n_slots][...] with `fill` in the padding slots."""
    rows = np.asarray(rows)
    n_tok = rows.shape[0]
    out = np.full((n_tok // W * slots_per_event(W, G),) + rows.shape[1:], fill, dtype=rows.dtype)
    out[token_slots(n_tok, W, G)] = rows
    return out
