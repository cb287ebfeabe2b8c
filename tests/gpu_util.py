"""Device-buffer helpers for the GPU tests: guarded allocations and uploads."""
import numpy as np
import torch

GUARD = 64          # guard elements on each side of a buffer
DEV = "cuda:0"

_NP_TO_TORCH = {np.dtype(np.uint16): torch.int16, np.dtype(np.uint32): torch.int32,
                np.dtype(np.float32): torch.float32, np.dtype(np.int16): torch.int16,
                np.dtype(np.int32): torch.int32}
_SIGNED_VIEW = {np.dtype(np.uint16): np.int16, np.dtype(np.uint32): np.int32}


class Guarded:
    """A device buffer of n elements with canary regions before and after it.
    ``skew`` shifts the start by that many elements off 16-byte alignment."""

    def __init__(self, n, np_dtype, skew=0, fill=None):
        self.np_dtype = np.dtype(np_dtype)
        tdt = _NP_TO_TORCH[self.np_dtype]
        self.n = n
        self.lead = GUARD + skew
        self.whole = torch.empty(n + 2 * GUARD + skew + 16, dtype=tdt, device=DEV)
        assert self.whole.data_ptr() % 256 == 0
        self.pattern = 0x5A5A if self.np_dtype.itemsize == 2 else 0x5A5A5A5A
        if tdt == torch.float32:
            self.whole.view(torch.int32).fill_(self.pattern)
        else:
            self.whole.fill_(self.pattern)
        self.t = self.whole[self.lead:self.lead + n]
        if fill is not None:
            self.t.copy_(to_torch(fill))

    def numpy(self):
        return from_torch(self.t, self.np_dtype)

    def guards_intact(self):
        w = self.whole.view(torch.int32) if self.whole.dtype == torch.float32 else self.whole
        w = w.cpu().numpy()
        head, tail = w[:self.lead], w[self.lead + self.n:]
        pat = np.array(self.pattern).astype(w.dtype) if self.np_dtype.itemsize == 2 else \
            np.array(self.pattern, dtype=np.int64).astype(np.int32)
        return bool(np.all(head == pat) and np.all(tail == pat))


def to_torch(a):
    a = np.ascontiguousarray(a)
    if a.dtype in _SIGNED_VIEW:
        a = a.view(_SIGNED_VIEW[a.dtype])
    return torch.from_numpy(a)


def upload(a):
    return to_torch(a).to(DEV)


def from_torch(t, np_dtype):
    a = t.detach().cpu().numpy()
    np_dtype = np.dtype(np_dtype)
    return a.view(np_dtype) if a.dtype != np_dtype else a
