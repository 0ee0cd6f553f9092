"""Device side of the seeded input generator: fills torch bf16 tensors in place on the GPU with the
same bits msa_synth.normal_bf16_bits produces on the host (needed for banks of tens of GiB)."""
import ctypes
import os

import numpy as np
import torch

import msa_synth as S

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmsa_synth.so")
_lib = None
_table_dev = {}


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built; run python -c 'import __graft_entry__ as g; g.build()'")
        _lib = ctypes.CDLL(LIB_PATH)
        _lib.msa_synth_fill_bf16.restype = ctypes.c_int
        _lib.msa_synth_fill_bf16.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64,
                                             ctypes.c_uint64, ctypes.c_uint64, ctypes.c_void_p]
    return _lib


def bits_to_torch(bits, device="cuda"):
    """uint16 bf16 bit patterns (numpy) -> torch.bfloat16 tensor of the same shape."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16)
    return t.to(device)


def torch_to_bits(t):
    """torch.bfloat16 tensor -> uint16 bit patterns (numpy, host)."""
    return t.detach().contiguous().cpu().view(torch.int16).numpy().view(np.uint16)


def fill_normal_(tensor, seed, start=0):
    """Fill a contiguous bf16 CUDA tensor with elements [start, start + numel) of the seeded stream."""
    assert tensor.is_cuda and tensor.dtype == torch.bfloat16 and tensor.is_contiguous()
    lib = _load()
    dev = tensor.device.index or 0
    if dev not in _table_dev:
        _table_dev[dev] = torch.from_numpy(S.quantile_table().view(np.int16)).to(tensor.device)
    stream = torch.cuda.current_stream(tensor.device).cuda_stream
    rc = lib.msa_synth_fill_bf16(_table_dev[dev].data_ptr(), tensor.data_ptr(), seed, start,
                                 tensor.numel(), ctypes.c_void_p(stream))
    if rc != 0:
        raise RuntimeError(f"msa_synth_fill_bf16 failed: {rc}")
    return tensor
