"""ctypes binding of liblogquant_plain.so: decode attention by a plain vector-unit kernel
(one token at a time, every element read through the layout index functions).  A test and
measurement aid: the tests cross-check the matrix-instruction kernel against it, the
benchmark times it for the matrix-unit-or-vector-unit comparison.  The product path
(binding.py, liblogquant.so) never loads it."""
import ctypes as C
import os

from . import binding as B

LIB_PATH = os.path.join(B.HERE, "liblogquant_plain.so")
if not os.path.exists(LIB_PATH):
    raise ImportError("liblogquant_plain.so is not built: run `python -m paper_2503_19950_amd.build`")
_lib = C.CDLL(LIB_PATH)
_lib.logquant_plain_decode_attn.argtypes = [C.POINTER(B.lq_config), C.POINTER(B.lq_cache), C.c_void_p, C.c_float,
                                            C.c_void_p, C.c_void_p, C.c_void_p]
_lib.logquant_plain_decode_attn.restype = C.c_int


def logquant_plain_decode_attn(cfg, cache, q, softmax_scale, out, workspace, stream=0):
    return _lib.logquant_plain_decode_attn(C.byref(cfg), C.byref(cache), B._ptr(q), float(softmax_scale),
                                           B._ptr(out), B._ptr(workspace), stream)


def decode_attn(dc, q, out=None, softmax_scale=0.0):
    """DeviceCache.decode_attn through the plain kernel."""
    if out is None:
        out = dc.torch.empty_like(q)
    st = logquant_plain_decode_attn(dc.cfg, dc.c, q, softmax_scale, out, dc.workspace, dc._stream())
    if st != B.LQ_OK:
        raise B.LogQuantError(st, "logquant_plain_decode_attn")
    return out
