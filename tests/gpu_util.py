"""Helpers for the GPU parity tests: device buffers via torch, calls via the C ABI."""
from __future__ import annotations

import numpy as np
import torch

from paper_2001_05585_amd import binding as B

NAN_BITS = 0x7E00
GUARD = 64            # halves of NaN poison on each side of the data (128 bytes: keeps 16-byte phase)


def stream_handle() -> int:
    return torch.cuda.current_stream().cuda_stream


class DeviceInput:
    """fp16 data on the GPU, surrounded by NaN poison, optionally shifted off 16-byte alignment."""

    def __init__(self, x: np.ndarray, shift: int = 0, poison: bool = True):
        bits = np.ascontiguousarray(x).view(np.uint16)
        n = bits.size
        fill = NAN_BITS if poison else 0
        buf = np.full(n + 2 * GUARD + 8, fill, dtype=np.uint16)
        start = GUARD + shift
        buf[start:start + n] = bits
        self.host = buf
        self.tensor = torch.from_numpy(buf.view(np.int16)).cuda()
        assert self.tensor.data_ptr() % 16 == 0
        self.start = start
        self.n = n
        self.ptr = self.tensor.data_ptr() + 2 * start

    def set(self, index: int, value_bits: int) -> None:
        v = int(np.array([value_bits], dtype=np.uint16).view(np.int16)[0])
        self.tensor[self.start + index] = v


class Outputs:
    """A device array of floats, pre-filled with a sentinel; slot i is an `out` pointer."""

    SENTINEL = -12345.0

    def __init__(self, count: int = 1):
        self.tensor = torch.full((count,), self.SENTINEL, dtype=torch.float32, device="cuda")

    def ptr(self, i: int = 0) -> int:
        return self.tensor.data_ptr() + 4 * i

    def get(self) -> np.ndarray:
        torch.cuda.synchronize()
        return self.tensor.cpu().numpy()


def gpu_sum(x: np.ndarray, tuning=None, shift: int = 0, n: int | None = None) -> np.float32:
    """One call of mfr_sum_f16_ex on a poisoned, possibly misaligned copy of x."""
    d = DeviceInput(x, shift)
    o = Outputs(1)
    B.mfr_sum_f16_ex(d.ptr, d.n if n is None else n, o.ptr(0), tuning, stream_handle())
    return np.float32(o.get()[0])


def f32(v: float) -> np.float32:
    return np.float32(v)
