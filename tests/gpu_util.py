"""Helpers of the GPU parity tests: device buffers with canaries, host copies."""
import numpy as np
import torch

CANARY = 0xA5


def dev(a):
    """numpy array -> device tensor with the same bytes (uint64 offsets travel as int64)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint64:
        a = a.view(np.int64)
    return torch.from_numpy(a).cuda()


def host(t):
    return t.detach().cpu().numpy()


class Guarded:
    """A uint8/float32 device buffer of `n` items followed by canary bytes, to catch writes past the end."""

    def __init__(self, n, dtype=torch.uint8, pad=64):
        self.n, self.pad, self.dtype = n, pad, dtype
        item = torch.empty(0, dtype=dtype).element_size()
        self.raw = torch.full((n * item + pad,), CANARY, dtype=torch.uint8, device="cuda")
        self.t = self.raw[: n * item].view(dtype)

    def check(self):
        tail = host(self.raw[self.raw.numel() - self.pad:])
        assert np.all(tail == CANARY), "kernel wrote past the end of its output"
        return host(self.t)
