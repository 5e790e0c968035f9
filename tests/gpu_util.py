"""Helpers shared by the GPU parity tests (not a test module)."""
import ctypes

import numpy as np
import torch

from paper_1902_04610_amd import salus


class DevicePool:
    """A torch-owned byte buffer plus the library pool that manages it."""

    def __init__(self, capacity, **kw):
        self.buf = torch.empty(capacity, dtype=torch.uint8, device="cuda")
        assert self.buf.data_ptr() % 256 == 0
        self.stream = torch.cuda.current_stream().cuda_stream
        self.pool = salus.Pool(self.buf.data_ptr(), capacity, stream=self.stream, **kw)
        self.capacity = capacity

    def write(self, off, arr):
        a = np.ascontiguousarray(arr).view(np.uint8).reshape(-1)
        self.buf[off:off + a.size].copy_(torch.from_numpy(a))

    def read(self, off, nbytes, dtype=np.uint8):
        return self.buf[off:off + nbytes].cpu().numpy().view(dtype)

    def sync(self):
        torch.cuda.synchronize()

    def close(self):
        self.sync()
        self.pool.close()


def norm_rel_err(got, ref):
    """max |got - ref| / max |ref| over one output matrix."""
    ref = np.asarray(ref, np.float64)
    return float(np.abs(np.asarray(got, np.float64) - ref).max() / max(np.abs(ref).max(), 1e-30))


def np_ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def mlp_layout(dims, esz, M):
    """Offsets of a dense stack inside a job: weights back to back in the
    persistent block; x, h (ping-pong) and y in the lane, 256-byte aligned."""
    up = lambda v: (v + 255) // 256 * 256
    w_offs, off = [], 0
    for K, N in zip(dims[:-1], dims[1:]):
        w_offs.append(off)
        off += up(K * N * esz)
    P = off
    x_off = 0
    y_off = up(M * dims[0] * esz)
    h_off = y_off + up(M * dims[-1] * 4)
    layers = [(K, N, 0, 0) for K, N in zip(dims[:-1], dims[1:])]
    E = h_off + salus.forward_work_bytes(M, layers, salus.BF16 if esz == 2 else salus.F32)
    return w_offs, P, x_off, y_off, h_off, max(E, 256)
