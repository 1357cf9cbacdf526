"""Helpers for the GPU parity tests: move a synthetic workload to the device and call the C-ABI binding."""
import numpy as np
import torch

from paper_2508_08256_amd import binding as B


def tdtype(dtype):
    return torch.float16 if dtype == B.F16 else torch.bfloat16


def to_dev(words, dtype):
    """uint16 words (numpy) -> 16-bit float tensor on the GPU, bit for bit."""
    return torch.from_numpy(np.ascontiguousarray(words).view(np.int16)).cuda().view(tdtype(dtype))


def words_of(t):
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


class DeviceWorkload:
    def __init__(self, wl, group_size=32):
        self.wl = wl
        self.cfg = B.make_config(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.max_ctx, wl.dtype, group_size=group_size)
        self.K = to_dev(wl.K, wl.dtype)
        self.V = to_dev(wl.V, wl.dtype)
        self.q = to_dev(wl.q, wl.dtype)
        self.k_new = to_dev(wl.k_new, wl.dtype)
        self.v_new = to_dev(wl.v_new, wl.dtype)
        self.seq_lens = i32(wl.seq_lens)
        self.budgets = i32(wl.budgets)
        self.cache = B.DeviceCache(self.cfg, self.K, self.V, self.seq_lens)

    def workspace(self, max_budget):
        return B.make_workspace(self.cfg, max_budget)
