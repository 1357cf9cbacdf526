"""Seeded synthetic decode-step inputs shaped like long-context LLM attention layers.

This module only draws random tensors; it holds none of the method's
arithmetic (no quantizer, no scores, no selection, no softmax) and is the one
piece of code that both the HIP path's tests and the CPU oracle's tests use.

Recipe per unit (one batch element, one kv head), head_dim D:
  * K_noise, V ~ N(0, 1), q ~ N(0, 1) for each of the n_rep query heads of the unit;
  * a per-head channel scale vector: ones (``chan="ones"``) or exp(0.5 N(0,1))
    (``chan="lognormal"``), with ``n_outlier`` channels (chosen by the seed) multiplied by 8;
    K = K_noise * scale (V has no outlier channels);
  * ``n_planted`` positions drawn uniformly without replacement from [0, L) get
    K[t] = 0.8 * qhat * sqrt(D) + 0.2 * K[t], qhat = qsum / |qsum|, qsum = sum of the unit's queries;
  * everything is rounded to the 16-bit storage dtype.
Values are returned as raw uint16 words (layout [units][Lcap][D]) so they can go to either side
unchanged.  Rows at positions >= L are zero.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

F16, BF16 = 0, 1


def f32_to_words(x: np.ndarray, dtype: int) -> np.ndarray:
    """Round binary32 values to the 16-bit storage dtype (nearest even); return the raw words."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == F16:
        return x.astype(np.float16).view(np.uint16)
    u = x.view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def words_to_f32(w: np.ndarray, dtype: int) -> np.ndarray:
    w = np.ascontiguousarray(w, dtype=np.uint16)
    if dtype == F16:
        return w.view(np.float16).astype(np.float32)
    return (w.astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class Workload:
    """One layer's decode-step inputs.  Units are ordered batch-major: u = b * n_kv_heads + h."""
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    max_ctx: int
    dtype: int
    seq_lens: np.ndarray        # [batch] int32
    budgets: np.ndarray         # [batch] int32
    K: np.ndarray               # [units][max_ctx][D] uint16
    V: np.ndarray               # [units][max_ctx][D] uint16
    q: np.ndarray               # [units][n_rep][D] uint16  (== [batch][n_q_heads][D])
    k_new: np.ndarray           # [units][D] uint16: the key appended by this step
    v_new: np.ndarray           # [units][D] uint16
    planted: list               # per unit: sorted int array of planted positions

    @property
    def n_rep(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def units(self) -> int:
        return self.batch * self.n_kv_heads

    @property
    def unit_lens(self) -> np.ndarray:
        return np.repeat(self.seq_lens, self.n_kv_heads).astype(np.int32)

    @property
    def unit_budgets(self) -> np.ndarray:
        return np.repeat(self.budgets, self.n_kv_heads).astype(np.int32)


def budget_from_fraction(L, frac: float = 0.11):
    """Token budget as a share of the context, rounded to nearest, at least 1."""
    return np.maximum(1, np.floor(np.asarray(L, dtype=np.float64) * frac + 0.5)).astype(np.int32)


def make_workload(name: str, seed: int, batch: int, n_q_heads: int, n_kv_heads: int, seq_lens,
                  budgets, dtype: int = F16, head_dim: int = 128, max_ctx: int | None = None,
                  chan: str = "ones", n_outlier: int = 4, n_planted: int = 16,
                  plant: bool = True) -> Workload:
    rng = np.random.default_rng(seed)
    seq_lens = np.asarray(seq_lens, dtype=np.int32).reshape(batch)
    budgets = np.asarray(budgets, dtype=np.int32).reshape(batch)
    D = head_dim
    n_rep = n_q_heads // n_kv_heads
    assert n_rep * n_kv_heads == n_q_heads
    if max_ctx is None:
        max_ctx = int(-(-(int(seq_lens.max()) + 1) // 64) * 64)
    U = batch * n_kv_heads
    K = np.zeros((U, max_ctx, D), np.uint16)
    V = np.zeros((U, max_ctx, D), np.uint16)
    q = np.zeros((U, n_rep, D), np.uint16)
    k_new = np.zeros((U, D), np.uint16)
    v_new = np.zeros((U, D), np.uint16)
    planted = []
    # the channel scale is a property of the kv head, shared by every batch element
    head_scale = []
    for h in range(n_kv_heads):
        sc = np.ones(D, np.float32) if chan == "ones" else np.exp(0.5 * rng.standard_normal(D)).astype(np.float32)
        out_ch = rng.choice(D, size=n_outlier, replace=False)
        sc[out_ch] *= 8.0
        head_scale.append(sc)
    for b in range(batch):
        L = int(seq_lens[b])
        for h in range(n_kv_heads):
            u = b * n_kv_heads + h
            sc = head_scale[h]
            Kf = rng.standard_normal((L, D), dtype=np.float32) * sc
            Vf = rng.standard_normal((L, D), dtype=np.float32)
            qf = rng.standard_normal((n_rep, D), dtype=np.float32)
            qsum = qf.sum(axis=0)
            qhat = qsum / np.linalg.norm(qsum)
            npl = min(n_planted, L) if plant else 0
            pos = np.sort(rng.choice(L, size=npl, replace=False)) if npl > 0 else np.zeros(0, np.int64)
            if npl > 0:
                Kf[pos] = 0.8 * qhat * np.sqrt(np.float32(D)) + 0.2 * Kf[pos]
            K[u, :L] = f32_to_words(Kf, dtype)
            V[u, :L] = f32_to_words(Vf, dtype)
            q[u] = f32_to_words(qf, dtype)
            k_new[u] = f32_to_words(rng.standard_normal(D, dtype=np.float32) * sc, dtype)
            v_new[u] = f32_to_words(rng.standard_normal(D, dtype=np.float32), dtype)
            planted.append(pos.astype(np.int64))
    return Workload(name, batch, n_q_heads, n_kv_heads, D, max_ctx, dtype, seq_lens, budgets, K, V, q,
                    k_new, v_new, planted)


# ---------------------------------------------------------------------------------------------
# Named configurations (the benchmark configurations of this build; shapes follow LLaMA-2-7B and
# Llama-3-8B attention layers at 4k..128k tokens, the setting of the paper's Sec. 4).

def config1(seed: int = 1000) -> Workload:
    """Small correctness case: batch 1, 8 MHA heads, 4096 tokens, budget 512, fp16, 16 planted."""
    return make_workload("config1", seed, 1, 8, 8, [4096], [512], F16, n_planted=16, max_ctx=4096 + 64)


def small_ragged(seed: int = 7, dtype: int = F16, n_rep: int = 1) -> Workload:
    """Tiny ragged batch crossing several tiles with partial tail groups."""
    lens = [1000, 333, 64, 1]
    return make_workload("small_ragged", seed, 4, 2 * n_rep, 2, lens, [100, 50, 64, 4], dtype,
                         n_planted=4, max_ctx=1024,
                         chan="lognormal" if dtype == BF16 else "ones")


def config2_shape():
    return dict(batch=1, n_q_heads=32, n_kv_heads=32, L=32768, budget=3604, dtype=F16, n_planted=64,
                chan="ones")


def config3_shape():
    return dict(batch=4, n_q_heads=32, n_kv_heads=8, L=131072, budget=4096, dtype=BF16, n_planted=64,
                chan="lognormal")


# ---------------------------------------------------------------------------------------------
# Device-side generator for the large configurations (same recipe, torch's generator on the GPU;
# the tensors are copied back to the host when the oracle needs them).

def make_workload_device(name: str, seed: int, batch: int, n_q_heads: int, n_kv_heads: int, seq_lens,
                         budgets, dtype: int = F16, head_dim: int = 128, max_ctx: int | None = None,
                         chan: str = "ones", n_outlier: int = 4, n_planted: int = 64, device="cuda"):
    """Returns a dict of torch tensors on ``device`` (K, V, q, k_new, v_new in the 16-bit dtype,
    seq_lens / budgets int32) plus ``planted`` (list of host int64 arrays per unit)."""
    import torch

    tdt = torch.float16 if dtype == F16 else torch.bfloat16
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    host_rng = np.random.default_rng(seed)
    seq_lens = np.asarray(seq_lens, dtype=np.int32).reshape(batch)
    budgets = np.asarray(budgets, dtype=np.int32).reshape(batch)
    D = head_dim
    n_rep = n_q_heads // n_kv_heads
    if max_ctx is None:
        max_ctx = int(-(-(int(seq_lens.max()) + 1) // 64) * 64)
    U = batch * n_kv_heads
    K = torch.zeros((U, max_ctx, D), dtype=tdt, device=device)
    V = torch.zeros((U, max_ctx, D), dtype=tdt, device=device)
    qf = torch.randn((U, n_rep, D), generator=gen, device=device, dtype=torch.float32)
    head_scale = torch.ones((n_kv_heads, D), device=device)
    if chan != "ones":
        head_scale = torch.exp(0.5 * torch.randn((n_kv_heads, D), generator=gen, device=device))
    for h in range(n_kv_heads):
        out_ch = host_rng.choice(D, size=n_outlier, replace=False)
        head_scale[h, torch.as_tensor(out_ch, device=device)] *= 8.0
    planted = []
    for b in range(batch):
        L = int(seq_lens[b])
        for h in range(n_kv_heads):
            u = b * n_kv_heads + h
            Kf = torch.randn((L, D), generator=gen, device=device, dtype=torch.float32) * head_scale[h]
            qsum = qf[u].sum(dim=0)
            qhat = qsum / qsum.norm()
            npl = min(n_planted, L)
            pos = np.sort(host_rng.choice(L, size=npl, replace=False)).astype(np.int64)
            pt = torch.as_tensor(pos, device=device)
            Kf[pt] = 0.8 * qhat * float(np.sqrt(D)) + 0.2 * Kf[pt]
            K[u, :L] = Kf.to(tdt)
            V[u, :L] = torch.randn((L, D), generator=gen, device=device, dtype=torch.float32).to(tdt)
            planted.append(pos)
            del Kf
    k_new = (torch.randn((U, D), generator=gen, device=device) *
             head_scale.repeat(batch, 1)).to(tdt)
    v_new = torch.randn((U, D), generator=gen, device=device).to(tdt)
    return dict(name=name, batch=batch, n_q_heads=n_q_heads, n_kv_heads=n_kv_heads, head_dim=D,
                max_ctx=max_ctx, dtype=dtype, K=K, V=V, q=qf.to(tdt), k_new=k_new, v_new=v_new,
                seq_lens=torch.as_tensor(seq_lens, device=device),
                budgets=torch.as_tensor(budgets, device=device), planted=planted)


def words_of(t) -> np.ndarray:
    """Raw uint16 words of a 16-bit torch tensor, on the host."""
    import torch

    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
