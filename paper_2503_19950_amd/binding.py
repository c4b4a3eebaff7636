"""ctypes binding of liblogquant.so: argument marshalling only.

The functions carry the names of the C entry points declared in
include/logquant.h.  PyTorch appears only as the owner of device memory and of
the HIP stream; every step of the path runs in the library's kernels.  There is
no fallback: if the shared library is missing, importing this module fails.
"""
import ctypes as C
import os

# PyTorch ships its own HIP runtime.  It has to be in the process before the library
# is loaded so that the library binds to that same runtime (matched by soname); two
# HIP runtimes in one process cannot both open the GPU.
import torch  # noqa: F401  (device memory and streams come from here as well)

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "liblogquant.so")

LQ_OK, LQ_ERR_NULL, LQ_ERR_SHAPE, LQ_ERR_UNSUPPORTED, LQ_ERR_CAPACITY, LQ_ERR_STATE, LQ_ERR_HIP = range(7)
LQ_F16, LQ_BF16 = 0, 1


class lq_config(C.Structure):
    _fields_ = [("B", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("d", C.c_int32),
                ("fp_budget", C.c_int32), ("group", C.c_int32), ("bits", C.c_int32),
                ("dtype", C.c_int32), ("q_capacity", C.c_int32)]


class lq_cache(C.Structure):
    _fields_ = [("k_fp", C.c_void_p * 2), ("v_fp", C.c_void_p * 2), ("pos_fp", C.c_void_p * 2),
                ("k_codes", C.c_void_p), ("v_codes", C.c_void_p),
                ("k_scale", C.c_void_p), ("k_zero", C.c_void_p),
                ("v_scale", C.c_void_p), ("v_zero", C.c_void_p),
                ("pos_q", C.c_void_p),
                ("cur", C.c_int32), ("n_fp", C.c_int32), ("n_q", C.c_int32)]


class lq_cache_seq(C.Structure):
    _fields_ = [("k_fp", C.c_void_p * 2), ("v_fp", C.c_void_p * 2), ("pos_fp", C.c_void_p * 2),
                ("k_codes", C.c_void_p), ("v_codes", C.c_void_p),
                ("k_scale", C.c_void_p), ("k_zero", C.c_void_p),
                ("v_scale", C.c_void_p), ("v_zero", C.c_void_p),
                ("pos_q", C.c_void_p),
                ("cur", C.POINTER(C.c_int32)), ("n_fp", C.POINTER(C.c_int32)), ("n_q", C.POINTER(C.c_int32)),
                ("seq_state", C.c_void_p)]


class lq_sizes(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in ("k_fp", "v_fp", "pos_fp", "k_codes", "v_codes", "k_meta",
                                          "v_meta", "pos_q", "workspace")]


class lq_plan(C.Structure):
    _fields_ = [("blocks", C.c_int32), ("waves_per_block", C.c_int32), ("splits", C.c_int32),
                ("fp_waves", C.c_int32), ("bytes_read", C.c_int64)]


EXPORTS = ("logquant_sizes", "logquant_workspace_bytes", "logquant_workspace_init", "logquant_append", "logquant_compress",
           "logquant_prefill", "logquant_prefill_positions", "logquant_decode_attn", "logquant_decode_attn_static",
           "logquant_decode_step", "logquant_decode_plan",
           "logquant_seq_state_bytes", "logquant_prefill_seq", "logquant_append_seq", "logquant_compress_seq",
           "logquant_decode_attn_seq", "logquant_decode_step_seq", "logquant_decode_plan_seq",
           "logquant_read_probe", "logquant_status_string")

if not os.path.exists(LIB_PATH):
    raise ImportError("liblogquant.so is not built: run `python -m paper_2503_19950_amd.build` "
                      "(there is no fallback path)")
_lib = C.CDLL(LIB_PATH)

_lib.logquant_sizes.argtypes = [C.POINTER(lq_config), C.POINTER(lq_sizes)]
_lib.logquant_sizes.restype = C.c_int
_lib.logquant_workspace_bytes.argtypes = [C.POINTER(lq_config)]
_lib.logquant_workspace_bytes.restype = C.c_size_t
_lib.logquant_workspace_init.argtypes = [C.POINTER(lq_config), C.c_void_p, C.c_void_p]
_lib.logquant_workspace_init.restype = C.c_int
_lib.logquant_append.argtypes = [C.POINTER(lq_config), C.POINTER(lq_cache), C.c_void_p, C.c_void_p,
                                 C.c_int32, C.c_void_p]
_lib.logquant_append.restype = C.c_int
_lib.logquant_compress.argtypes = [C.POINTER(lq_config), C.POINTER(lq_cache), C.c_void_p, C.c_void_p]
_lib.logquant_compress.restype = C.c_int
_lib.logquant_prefill.argtypes = [C.POINTER(lq_config), C.POINTER(lq_cache), C.c_void_p, C.c_void_p, C.c_int32,
                                  C.c_void_p]
_lib.logquant_prefill.restype = C.c_int
_lib.logquant_prefill_positions.argtypes = [C.c_int32, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                                            C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
_lib.logquant_prefill_positions.restype = C.c_int
_lib.logquant_decode_attn.argtypes = [C.POINTER(lq_config), C.POINTER(lq_cache), C.c_void_p, C.c_float,
                                      C.c_void_p, C.c_void_p, C.c_void_p]
_lib.logquant_decode_attn.restype = C.c_int
_lib.logquant_decode_attn_static.argtypes = [C.POINTER(lq_config), C.POINTER(lq_cache), C.c_void_p, C.c_float,
                                             C.c_void_p, C.c_void_p]
_lib.logquant_decode_attn_static.restype = C.c_int
_lib.logquant_decode_step.argtypes = [C.POINTER(lq_config), C.POINTER(lq_cache), C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_float, C.c_void_p, C.c_void_p, C.c_void_p]
_lib.logquant_decode_step.restype = C.c_int
_lib.logquant_decode_plan.argtypes = [C.POINTER(lq_config), C.c_int32, C.c_int32, C.POINTER(lq_plan)]
_lib.logquant_decode_plan.restype = C.c_int
_I32P = C.POINTER(C.c_int32)
_lib.logquant_seq_state_bytes.argtypes = [C.POINTER(lq_config)]
_lib.logquant_seq_state_bytes.restype = C.c_size_t
_lib.logquant_prefill_seq.argtypes = [C.POINTER(lq_config), C.POINTER(lq_cache_seq), C.c_void_p, C.c_void_p, _I32P,
                                      C.c_int32, C.c_void_p]
_lib.logquant_prefill_seq.restype = C.c_int
_lib.logquant_append_seq.argtypes = [C.POINTER(lq_config), C.POINTER(lq_cache_seq), C.c_void_p, C.c_void_p, _I32P,
                                     C.c_void_p]
_lib.logquant_append_seq.restype = C.c_int
_lib.logquant_compress_seq.argtypes = [C.POINTER(lq_config), C.POINTER(lq_cache_seq), C.c_void_p]
_lib.logquant_compress_seq.restype = C.c_int
_lib.logquant_decode_attn_seq.argtypes = [C.POINTER(lq_config), C.POINTER(lq_cache_seq), C.c_void_p, C.c_float,
                                          C.c_void_p, C.c_void_p, C.c_void_p]
_lib.logquant_decode_attn_seq.restype = C.c_int
_lib.logquant_decode_step_seq.argtypes = [C.POINTER(lq_config), C.POINTER(lq_cache_seq), C.c_void_p, C.c_void_p,
                                          C.c_void_p, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p]
_lib.logquant_decode_step_seq.restype = C.c_int
_lib.logquant_decode_plan_seq.argtypes = [C.POINTER(lq_config), _I32P, _I32P, C.POINTER(lq_plan)]
_lib.logquant_decode_plan_seq.restype = C.c_int
_lib.logquant_read_probe.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
_lib.logquant_read_probe.restype = C.c_int
_lib.logquant_status_string.argtypes = [C.c_int]
_lib.logquant_status_string.restype = C.c_char_p


class LogQuantError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s: %s" % (where, logquant_status_string(status)))


def _ptr(x):
    """Device (or null) pointer of a torch tensor / int / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _p(struct):
    return C.byref(struct) if struct is not None else None


def logquant_status_string(status):
    return _lib.logquant_status_string(int(status)).decode()


def logquant_sizes(cfg):
    out = lq_sizes()
    st = _lib.logquant_sizes(_p(cfg), C.byref(out))
    if st != LQ_OK:
        raise LogQuantError(st, "logquant_sizes")
    return out


def logquant_workspace_bytes(cfg):
    return int(_lib.logquant_workspace_bytes(_p(cfg)))


def logquant_workspace_init(cfg, workspace, stream=0):
    return _lib.logquant_workspace_init(_p(cfg), _ptr(workspace), stream)


def logquant_append(cfg, cache, k_new, v_new, n_new, stream=0):
    return _lib.logquant_append(_p(cfg), _p(cache), _ptr(k_new), _ptr(v_new), int(n_new), stream)


def logquant_compress(cfg, cache, workspace=None, stream=0):
    return _lib.logquant_compress(_p(cfg), _p(cache), _ptr(workspace), stream)


def logquant_prefill(cfg, cache, k, v, L, stream=0):
    return _lib.logquant_prefill(_p(cfg), _p(cache), _ptr(k), _ptr(v), int(L), stream)


def logquant_prefill_positions(W, L):
    """-> (status, pos_fp list, pos_q list); host arithmetic only."""
    n_fp, n_q = C.c_int32(0), C.c_int32(0)
    st = _lib.logquant_prefill_positions(int(W), int(L), None, C.byref(n_fp), None, C.byref(n_q))
    if st != LQ_OK:
        return st, None, None
    a = (C.c_int32 * max(1, n_fp.value))()
    q = (C.c_int32 * max(1, n_q.value))()
    st = _lib.logquant_prefill_positions(int(W), int(L), a, C.byref(n_fp), q, C.byref(n_q))
    return st, list(a[:n_fp.value]), list(q[:n_q.value])


def logquant_decode_attn(cfg, cache, q, softmax_scale, out, workspace, stream=0):
    return _lib.logquant_decode_attn(_p(cfg), _p(cache), _ptr(q), float(softmax_scale), _ptr(out),
                                     _ptr(workspace), stream)


def logquant_decode_attn_static(cfg, cache, q, softmax_scale, out, stream=0):
    return _lib.logquant_decode_attn_static(_p(cfg), _p(cache), _ptr(q), float(softmax_scale), _ptr(out), stream)


def logquant_decode_step(cfg, cache, k_new, v_new, q, softmax_scale, out, workspace, stream=0):
    return _lib.logquant_decode_step(_p(cfg), _p(cache), _ptr(k_new), _ptr(v_new), _ptr(q), float(softmax_scale),
                                     _ptr(out), _ptr(workspace), stream)


def logquant_decode_plan(cfg, n_fp, n_q):
    out = lq_plan()
    st = _lib.logquant_decode_plan(_p(cfg), int(n_fp), int(n_q), C.byref(out))
    if st != LQ_OK:
        raise LogQuantError(st, "logquant_decode_plan")
    return out


def _i32(values):
    """Host int32 array (or null) from a Python sequence."""
    if values is None:
        return None
    return (C.c_int32 * len(values))(*[int(x) for x in values])


def logquant_seq_state_bytes(cfg):
    return int(_lib.logquant_seq_state_bytes(_p(cfg)))


def logquant_prefill_seq(cfg, cache, k, v, L, L_stride, stream=0):
    return _lib.logquant_prefill_seq(_p(cfg), _p(cache), _ptr(k), _ptr(v), _i32(L), int(L_stride), stream)


def logquant_append_seq(cfg, cache, k_new, v_new, active=None, stream=0):
    return _lib.logquant_append_seq(_p(cfg), _p(cache), _ptr(k_new), _ptr(v_new), _i32(active), stream)


def logquant_compress_seq(cfg, cache, stream=0):
    return _lib.logquant_compress_seq(_p(cfg), _p(cache), stream)


def logquant_decode_attn_seq(cfg, cache, q, softmax_scale, out, workspace, stream=0):
    return _lib.logquant_decode_attn_seq(_p(cfg), _p(cache), _ptr(q), float(softmax_scale), _ptr(out),
                                         _ptr(workspace), stream)


def logquant_decode_step_seq(cfg, cache, k_new, v_new, q, softmax_scale, out, workspace, stream=0):
    return _lib.logquant_decode_step_seq(_p(cfg), _p(cache), _ptr(k_new), _ptr(v_new), _ptr(q),
                                         float(softmax_scale), _ptr(out), _ptr(workspace), stream)


def logquant_decode_plan_seq(cfg, n_fp, n_q):
    out = lq_plan()
    st = _lib.logquant_decode_plan_seq(_p(cfg), _i32(n_fp), _i32(n_q), C.byref(out))
    if st != LQ_OK:
        raise LogQuantError(st, "logquant_decode_plan_seq")
    return out


def logquant_read_probe(buf, nbytes, sink, stream=0):
    return _lib.logquant_read_probe(_ptr(buf), int(nbytes), _ptr(sink), stream)


def torch_dtype(dtype):
    import torch
    return torch.bfloat16 if dtype == "bf16" else torch.float16


def to_dev(x, dtype, device="cuda:0"):
    """float32 numpy array of exact T values -> device tensor of type T."""
    import numpy as np
    import torch
    return torch.from_numpy(np.ascontiguousarray(x)).to(device).to(torch_dtype(dtype))


def make_config(B, Hq, Hkv, d, fp_budget, group, dtype, q_capacity, bits=2):
    return lq_config(B, Hq, Hkv, d, fp_budget, group, bits, LQ_BF16 if dtype == "bf16" else LQ_F16,
                     q_capacity)


class DeviceCache:
    """Owner of the device buffers of one lq_cache (torch tensors) plus the
    workspace.  Only allocation and pointer bookkeeping happen here."""

    def __init__(self, cfg, device="cuda:0", poison=False):
        import torch
        self.torch = torch
        self.cfg = cfg
        self.device = torch.device(device)
        sz = logquant_sizes(cfg)
        self.sizes = sz

        def buf(nbytes):
            t = torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device=self.device)
            t.fill_(0xFF if poison else 0)   # 0xFF..: NaN patterns in fp16/bf16
            return t

        self.k_fp = [buf(sz.k_fp), buf(sz.k_fp)]
        self.v_fp = [buf(sz.v_fp), buf(sz.v_fp)]
        self.pos_fp = [buf(sz.pos_fp), buf(sz.pos_fp)]
        self.k_codes, self.v_codes = buf(sz.k_codes), buf(sz.v_codes)
        self.k_scale, self.k_zero = buf(sz.k_meta), buf(sz.k_meta)
        self.v_scale, self.v_zero = buf(sz.v_meta), buf(sz.v_meta)
        self.pos_q = buf(sz.pos_q)
        self.workspace = buf(sz.workspace)
        c = lq_cache()
        for i in range(2):
            c.k_fp[i] = self.k_fp[i].data_ptr()
            c.v_fp[i] = self.v_fp[i].data_ptr()
            c.pos_fp[i] = self.pos_fp[i].data_ptr()
        c.k_codes, c.v_codes = self.k_codes.data_ptr(), self.v_codes.data_ptr()
        c.k_scale, c.k_zero = self.k_scale.data_ptr(), self.k_zero.data_ptr()
        c.v_scale, c.v_zero = self.v_scale.data_ptr(), self.v_zero.data_ptr()
        c.pos_q = self.pos_q.data_ptr()
        c.cur = c.n_fp = c.n_q = 0
        self.c = c
        self._check(logquant_workspace_init(cfg, self.workspace, self._stream()), "logquant_workspace_init")

    BUFFERS = ("k_codes", "v_codes", "k_scale", "k_zero", "v_scale", "v_zero", "pos_q")

    def clone(self):
        """A second cache with its own device buffers and the same contents/counts."""
        other = DeviceCache(self.cfg, device=self.device)
        for i in range(2):
            other.k_fp[i].copy_(self.k_fp[i])
            other.v_fp[i].copy_(self.v_fp[i])
            other.pos_fp[i].copy_(self.pos_fp[i])
        for name in self.BUFFERS:
            getattr(other, name).copy_(getattr(self, name))
        other.c.cur, other.c.n_fp, other.c.n_q = self.c.cur, self.c.n_fp, self.c.n_q
        return other

    def counts(self):
        return (self.c.cur, self.c.n_fp, self.c.n_q)

    def set_counts(self, counts):
        """Rewind the host-side counts (the device buffers are left as they are)."""
        self.c.cur, self.c.n_fp, self.c.n_q = counts

    @property
    def W(self):
        return self.cfg.fp_budget // 2

    def _stream(self):
        return self.torch.cuda.current_stream(self.device).cuda_stream

    def _check(self, st, where):
        if st != LQ_OK:
            raise LogQuantError(st, where)

    def append(self, k_new, v_new):
        """k_new, v_new: [B][Hkv][n][d] tensors of the cache dtype, contiguous."""
        n = k_new.shape[2]
        assert k_new.is_contiguous() and v_new.is_contiguous()
        self._check(logquant_append(self.cfg, self.c, k_new, v_new, n, self._stream()), "logquant_append")

    def compress(self):
        self._check(logquant_compress(self.cfg, self.c, self.workspace, self._stream()), "logquant_compress")

    def prefill(self, K, V):
        """K, V: [B][Hkv][L][d] tensors of the cache dtype, contiguous; the cache must be empty."""
        assert K.is_contiguous() and V.is_contiguous()
        self._check(logquant_prefill(self.cfg, self.c, K, V, K.shape[2], self._stream()), "logquant_prefill")

    def stream_in(self, K, V):
        """Append [B][Hkv][n][d] rows with the eager trigger: compress whenever the
        fp region reaches 3W rows.  Returns the number of compress events."""
        n, i, ev, cap = K.shape[2], 0, 0, 3 * self.W
        while i < n:
            m = min(cap - self.c.n_fp, n - i)
            self.append(K[:, :, i:i + m].contiguous(), V[:, :, i:i + m].contiguous())
            i += m
            if self.c.n_fp == cap:
                self.compress()
                ev += 1
        return ev

    def decode_step(self, k_new, v_new, q, out=None, softmax_scale=0.0):
        """Append one token ([B][Hkv][1][d]) and attend, in one launch."""
        if out is None:
            out = self.torch.empty_like(q)
        assert k_new.is_contiguous() and v_new.is_contiguous()
        self._check(logquant_decode_step(self.cfg, self.c, k_new, v_new, q, softmax_scale, out, self.workspace,
                                         self._stream()), "logquant_decode_step")
        return out

    def decode_attn(self, q, out=None, softmax_scale=0.0):
        if out is None:
            out = self.torch.empty_like(q)
        self._check(logquant_decode_attn(self.cfg, self.c, q, softmax_scale, out, self.workspace,
                                         self._stream()), "logquant_decode_attn")
        return out


class DeviceCacheSeq(DeviceCache):
    """The same device buffers with per-sequence counts (lq_cache_seq): host arrays of B
    entries for cur / n_fp / n_q and the device scratch the calls pass them through."""

    def __init__(self, cfg, device="cuda:0", poison=False):
        super().__init__(cfg, device, poison)
        B = cfg.B
        self.cur, self.n_fp, self.n_q = ((C.c_int32 * B)() for _ in range(3))
        self.seq_state = self.torch.zeros(max(logquant_seq_state_bytes(cfg), 16), dtype=self.torch.uint8,
                                          device=self.device)
        cs = lq_cache_seq()
        for name, _ in lq_cache._fields_[:10]:
            setattr(cs, name, getattr(self.c, name))
        cs.cur = C.cast(self.cur, _I32P)
        cs.n_fp = C.cast(self.n_fp, _I32P)
        cs.n_q = C.cast(self.n_q, _I32P)
        cs.seq_state = self.seq_state.data_ptr()
        self.cs = cs

    def prefill_seq(self, K, V, L):
        assert K.is_contiguous() and V.is_contiguous()
        self._check(logquant_prefill_seq(self.cfg, self.cs, K, V, L, K.shape[2], self._stream()), "logquant_prefill_seq")

    def append_seq(self, k_new, v_new, active=None):
        assert k_new.is_contiguous() and v_new.is_contiguous()
        self._check(logquant_append_seq(self.cfg, self.cs, k_new, v_new, active, self._stream()), "logquant_append_seq")

    def compress_seq(self):
        self._check(logquant_compress_seq(self.cfg, self.cs, self._stream()), "logquant_compress_seq")

    def decode_attn_seq(self, q, out=None, softmax_scale=0.0):
        if out is None:
            out = self.torch.empty_like(q)
        self._check(logquant_decode_attn_seq(self.cfg, self.cs, q, softmax_scale, out, self.workspace,
                                             self._stream()), "logquant_decode_attn_seq")
        return out

    def decode_step_seq(self, k_new, v_new, q, out=None, softmax_scale=0.0):
        if out is None:
            out = self.torch.empty_like(q)
        assert k_new.is_contiguous() and v_new.is_contiguous()
        self._check(logquant_decode_step_seq(self.cfg, self.cs, k_new, v_new, q, softmax_scale, out, self.workspace,
                                             self._stream()), "logquant_decode_step_seq")
        return out

    def view(self, b):
        """Counts of sequence b as a (cur, n_fp, n_q) triple."""
        return (self.cur[b], self.n_fp[b], self.n_q[b])
