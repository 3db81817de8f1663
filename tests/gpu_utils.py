"""Helpers for GPU tests: numpy bit arrays <-> device tensors (torch is plumbing only)."""
import numpy as np
import torch

_SIGNED = {np.dtype(np.uint8): np.uint8, np.dtype(np.uint16): np.int16, np.dtype(np.uint32): np.int32,
           np.dtype(np.uint64): np.int64}


def to_dev(a):
    a = np.ascontiguousarray(a)
    return torch.from_numpy(a.view(_SIGNED[a.dtype])).cuda()


def dev_empty(nbytes_or_shape, np_dtype=np.uint8):
    t = {np.uint8: torch.uint8, np.uint16: torch.int16, np.uint32: torch.int32, np.uint64: torch.int64}[np_dtype]
    return torch.empty(nbytes_or_shape, dtype=t, device="cuda")


def to_host(t, np_dtype):
    torch.cuda.synchronize()
    return t.cpu().numpy().view(np_dtype)
