"""Helpers for the GPU parity tests: host <-> device movement of bit patterns
and guarded device arenas.  No arithmetic of the method lives here."""
import numpy as np
import torch

SENTINEL = 0xC3


def to_dev(a: np.ndarray) -> torch.Tensor:
    """numpy array -> uint8 device tensor holding the same bytes."""
    b = np.ascontiguousarray(a).view(np.uint8).reshape(-1)
    t = torch.from_numpy(b.copy())
    return t.cuda()


def to_host(t: torch.Tensor, dtype, count=None) -> np.ndarray:
    a = t.detach().cpu().numpy().view(dtype)
    return a if count is None else a[:count]


class Arena:
    """One device byte buffer, sentinel-filled, that hands out 16-byte aligned
    sub-buffers separated by guard bytes; check_guards() verifies that nothing
    outside the handed-out ranges was written."""

    def __init__(self, sizes_bytes, guard=64, offset=0):
        self.ranges = []
        pos = guard
        for nb in sizes_bytes:
            pos = (pos + 15) // 16 * 16 + offset
            self.ranges.append((pos, nb))
            pos += nb + guard
        self.total = (pos + 15) // 16 * 16 + 16
        self.buf = torch.full((self.total,), SENTINEL, dtype=torch.uint8, device="cuda")
        self.base = self.buf.data_ptr()
        assert self.base % 16 == 0
        # the fill ran on torch's stream; the library's calls run on streams of the
        # caller's choice, which do not wait for it
        torch.cuda.synchronize()

    def ptr(self, i):
        return self.base + self.ranges[i][0]

    def ptrs(self):
        return [self.ptr(i) for i in range(len(self.ranges))]

    def fill(self, i, a: np.ndarray):
        o, nb = self.ranges[i]
        b = np.ascontiguousarray(a).view(np.uint8).reshape(-1)
        assert b.size == nb
        if nb:
            self.buf[o:o + nb] = torch.from_numpy(b.copy()).cuda()
            torch.cuda.synchronize()

    def get(self, i, dtype) -> np.ndarray:
        o, nb = self.ranges[i]
        return self.buf[o:o + nb].cpu().numpy().view(dtype)

    def check_guards(self):
        h = self.buf.cpu().numpy()
        mask = np.ones(self.total, dtype=bool)
        for o, nb in self.ranges:
            mask[o:o + nb] = False
        bad = np.nonzero(h[mask] != SENTINEL)[0]
        assert bad.size == 0, "bytes outside the output ranges were written"
