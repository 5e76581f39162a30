"""ctypes binding of the HIP generator (gen.hip): same bytes as gen.gen_vectors, made on the GPU."""
from __future__ import annotations

import ctypes
import os

import numpy as np
import torch  # noqa: F401  -- loaded before the HIP library so both share PyTorch's HIP runtime

from . import gen

_LIB = None


def _lib():
    global _LIB
    if _LIB is None:
        path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libsynthgen.so")
        if not os.path.exists(path):
            raise RuntimeError("libsynthgen.so is not built: run `python -m paper_1102_3828_amd.build`")
        _LIB = ctypes.CDLL(path)
        _LIB.synth_generate.restype = ctypes.c_int
        _LIB.synth_generate.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int,
                                        ctypes.c_int, ctypes.c_uint64, ctypes.c_int64, ctypes.c_int64,
                                        ctypes.c_void_p, ctypes.c_void_p]
    return _LIB


class DeviceMixture:
    """The mixture's tables resident on the GPU (torch tensors)."""

    def __init__(self, mix: gen.Mixture, device="cuda:0"):
        import torch
        self.mix = mix
        self.device = torch.device(device)
        self.centres = torch.from_numpy(np.ascontiguousarray(mix.centres)).to(self.device)
        self.cum = torch.from_numpy(mix.cum_thresh.view(np.int32).copy()).to(self.device)
        self.gauss = torch.from_numpy(mix.gauss.copy()).to(self.device)

    def generate(self, stream_id: int, start: int, n: int, out=None):
        """uint8 [n, d] device tensor with vectors start..start+n-1 of the stream."""
        import torch
        d = self.mix.d
        if out is None:
            out = torch.empty((n, d), dtype=torch.uint8, device=self.device)
        assert out.is_contiguous() and out.shape == (n, d) and out.dtype == torch.uint8
        key = int(gen.stream_key(self.mix.seed, stream_id))
        st = torch.cuda.current_stream(self.device).cuda_stream
        rc = _lib().synth_generate(self.centres.data_ptr(), self.cum.data_ptr(), self.gauss.data_ptr(),
                                   self.mix.G, d, ctypes.c_uint64(key), start, n, out.data_ptr(),
                                   ctypes.c_void_p(st))
        if rc != 0:
            raise RuntimeError(f"synth_generate failed with code {rc}")
        return out
