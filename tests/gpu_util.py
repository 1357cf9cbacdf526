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


class PagedWorkload(DeviceWorkload):
    """The same workload with its K / V rows in a block pool: pool [n_pool][n_kv_heads][block_tokens][128], the
    sequences' blocks scattered over it by a seeded permutation, the unused pool blocks filled with a poison
    pattern (so that a stray read shows up in the results and a stray write in `poison_intact`)."""

    POISON = 0x7BFF  # the largest finite fp16; a large finite bf16

    def __init__(self, wl, block_tokens, group_size=32, seed=0, spare_blocks=5):
        self.wl = wl
        self.cfg = B.make_config(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.max_ctx, wl.dtype, group_size=group_size)
        self.block_tokens = bt = block_tokens
        per_seq = wl.max_ctx // bt
        n_pool = wl.batch * per_seq + spare_blocks
        perm = np.random.default_rng(seed).permutation(n_pool).astype(np.int32)
        self.table_np = perm[: wl.batch * per_seq].reshape(wl.batch, per_seq)
        self.spare = perm[wl.batch * per_seq:]
        pools = []
        for rows in (wl.K, wl.V):
            pool = np.full((n_pool, wl.n_kv_heads, bt, 128), self.POISON, np.uint16)
            r = rows.reshape(wl.batch, wl.n_kv_heads, per_seq, bt, 128)
            for b in range(wl.batch):
                pool[self.table_np[b]] = r[b].transpose(1, 0, 2, 3)
            pools.append(pool)
        self.K = to_dev(pools[0], wl.dtype)
        self.V = to_dev(pools[1], wl.dtype)
        self.q = to_dev(wl.q, wl.dtype)
        self.k_new = to_dev(wl.k_new, wl.dtype)
        self.v_new = to_dev(wl.v_new, wl.dtype)
        self.seq_lens = i32(wl.seq_lens)
        self.budgets = i32(wl.budgets)
        self.block_table = i32(self.table_np)
        self.cache = B.DeviceCache(self.cfg, self.K, self.V, self.seq_lens, self.block_table)

    def logical(self, pool):
        """[units][max_ctx][128] uint16 words gathered from a pool tensor through the block table."""
        wl = self.wl
        p = words_of(pool)
        out = np.empty((wl.batch, wl.n_kv_heads, wl.max_ctx // self.block_tokens, self.block_tokens, 128), np.uint16)
        for b in range(wl.batch):
            out[b] = p[self.table_np[b]].transpose(1, 0, 2, 3)
        return out.reshape(wl.batch * wl.n_kv_heads, wl.max_ctx, 128)

    def poison_intact(self):
        return all(bool((words_of(pool)[self.spare] == self.POISON).all()) for pool in (self.K, self.V))
