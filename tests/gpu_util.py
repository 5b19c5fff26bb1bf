"""Helpers shared by the GPU tests: device buffers with guard bands, bit-exact comparison."""
import numpy as np
import torch

from paper_1705_01598_amd import binding as B

GUARD = 1024  # elements of sentinel on each side of the output buffer
SENT64 = 0x7FF8DEADBEEF0123
SENT32 = 0x7FC0BEEF


def np_uint(a):
    a = np.ascontiguousarray(a)
    return a.view({4: np.uint32, 8: np.uint64}[a.dtype.itemsize])


def torch_int_dtype(elem):
    return torch.int64 if elem == 8 else torch.int32


def to_device(a_np):
    """numpy array -> cuda tensor of same-size signed ints (bits preserved)."""
    bits = np_uint(a_np).view(np.int64 if a_np.dtype.itemsize == 8 else np.int32)
    return torch.from_numpy(bits).cuda()


class GuardedOut:
    """Output buffer pre-filled with a sentinel and fenced by sentinel guard bands."""

    def __init__(self, volume, elem, offset_elems=0):
        self.elem = elem
        self.volume = volume
        self.sent = SENT64 if elem == 8 else SENT32
        self.off = GUARD + offset_elems
        self.buf = torch.full((volume + 2 * GUARD + offset_elems,), self.sent,
                              dtype=torch_int_dtype(elem), device="cuda")

    @property
    def ptr(self):
        return self.buf.data_ptr() + self.off * self.elem

    def view(self):
        return self.buf[self.off:self.off + self.volume]

    def guards_intact(self):
        lo = self.buf[:self.off]
        hi = self.buf[self.off + self.volume:]
        return bool((lo == self.sent).all().item()) and bool((hi == self.sent).all().item())


def run_plan(plan, a_dev, volume, elem, offset_elems=0):
    """Execute on the current torch stream; returns (output as numpy uint, guards ok)."""
    out = GuardedOut(volume, elem, offset_elems)
    stream = torch.cuda.current_stream().cuda_stream
    B.tperm_execute(plan, a_dev.data_ptr(), out.ptr, stream)
    torch.cuda.synchronize()
    res = out.view().cpu().numpy()
    return np_uint(res), out.guards_intact()
