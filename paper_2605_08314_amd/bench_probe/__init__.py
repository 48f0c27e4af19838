"""ctypes loader of libbenchprobe.so: the benchmark's two measurement kernels (a pure streaming read, a plain copy).
Not part of the library's interface; only bench.py imports this."""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbenchprobe.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2605_08314_amd.build`")
_lib = ctypes.CDLL(LIB_PATH)
_vp, _sz = ctypes.c_void_p, ctypes.c_size_t
_lib.benchprobe_read.argtypes = [_vp, _sz, _vp, _vp]
_lib.benchprobe_copy.argtypes = [_vp, _vp, _sz, _vp]


def _stream():
    return torch.cuda.current_stream().cuda_stream or None


def read(src: torch.Tensor, sink: torch.Tensor) -> None:
    assert _lib.benchprobe_read(src.data_ptr(), src.numel() * src.element_size(), sink.data_ptr(), _stream()) == 0


def copy(dst: torch.Tensor, src: torch.Tensor) -> None:
    assert _lib.benchprobe_copy(dst.data_ptr(), src.data_ptr(), src.numel() * src.element_size(), _stream()) == 0
