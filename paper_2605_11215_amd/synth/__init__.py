"""Seeded synthetic inputs (gradient streams, initial parameters).

`reference_np` is the NumPy statement of the streams; `fill_device` runs the device twin
(`synth.hip`, built as libsynth.so), which returns the same bits.  Inputs only: nothing of
the gradient path's arithmetic lives here.
"""
import ctypes as C
import os

from . import reference_np  # noqa: F401
from .reference_np import TAG_GRAD, TAG_PARAM, TAG_SCHEDULE, KIND_NORMAL, KIND_STUDENT_T3  # noqa: F401

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libsynth.so")
_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libsynth.so is not built; run `python -m paper_2605_11215_amd.build`")
        # PyTorch ships its own HIP runtime; it has to be in the process first so that this library
        # binds to the same runtime instead of loading a second one (device pointers and streams
        # are shared between the two).
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        L.synth_fill.argtypes = [C.c_void_p, C.c_int, C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32,
                                 C.c_uint32, C.c_double, C.c_int, C.c_void_p]
        L.synth_fill.restype = C.c_int
        _lib = L
    return _lib


def fill_device(out, seed, tag, mb_id, it, scale, kind=KIND_NORMAL, start=0, n=None):
    """Fill the first n elements of the torch device tensor `out` (float32 or bfloat16) with stream
    elements start .. start+n-1, on torch's current stream."""
    import torch
    n = out.numel() if n is None else n
    assert out.is_contiguous() and out.dtype in (torch.float32, torch.bfloat16) and n <= out.numel()
    rc = lib().synth_fill(out.data_ptr(), int(out.dtype == torch.bfloat16), start, n, seed, tag, mb_id, it,
                          float(scale), kind, torch.cuda.current_stream().cuda_stream or None)
    if rc != 0:
        raise RuntimeError("synth_fill failed with %d" % rc)
    return out
