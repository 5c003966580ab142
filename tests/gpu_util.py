"""Helpers of the GPU parity tests: device buffers with canary guard bands."""

import numpy as np
import torch

GUARD = 256
CANARY = 0xA5


class DevBuf:
    """``n`` device bytes with GUARD canary bytes on either side.

    ``shift`` moves the payload start by that many bytes (to build buffers whose
    addresses disagree modulo 16)."""

    def __init__(self, n, fill=None, shift=0):
        self.n = int(n)
        self.shift = shift
        self.raw = torch.full((self.n + 2 * GUARD + 16,), CANARY, dtype=torch.uint8, device="cuda")
        assert self.raw.data_ptr() % 256 == 0
        self.lo = GUARD + shift
        if fill is not None:
            self.view().copy_(torch.from_numpy(np.ascontiguousarray(fill)))

    def view(self):
        return self.raw[self.lo:self.lo + self.n]

    def ptr(self, off=0):
        return self.raw.data_ptr() + self.lo + off

    def host(self):
        return self.view().cpu().numpy()

    def guards_intact(self):
        lo = self.raw[:self.lo].cpu().numpy()              # only the two bands cross to the host
        hi = self.raw[self.lo + self.n:].cpu().numpy()
        return bool((lo == CANARY).all() and (hi == CANARY).all())


def stream():
    return torch.cuda.current_stream()


def sync():
    torch.cuda.current_stream().synchronize()
