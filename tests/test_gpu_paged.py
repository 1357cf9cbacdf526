"""K / V rows held in a block pool behind a block table (the layout of paged serving caches): every entry point
gives the results of the contiguous layout bit for bit, and those of the oracle on the logical rows."""
import numpy as np
import pytest
import torch

from paper_2508_08256_amd import binding as B
from paper_2508_08256_amd import synth
from helpers import check_index_sets, oracle_step

pytestmark = pytest.mark.gpu
F16, BF16 = B.F16, B.BF16


@pytest.fixture(scope="module")
def gu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_util

    return gpu_util


def _step(dw, append, mb):
    wl = dw.wl
    out = torch.full((1, wl.units, wl.n_rep, 128), float("nan"), dtype=torch.float32, device="cuda")
    idx = torch.full((1, wl.units, mb), -1, dtype=torch.int32, device="cuda")
    cnt = torch.full((1, wl.units), -1, dtype=torch.int32, device="cuda")
    kn = dw.k_new[None].contiguous() if append else None
    vn = dw.v_new[None].contiguous() if append else None
    B.decode_step(dw.cfg, [dw.cache], dw.q[None].contiguous(), kn, vn, dw.budgets, mb, out, idx, cnt,
                  dw.workspace(mb))
    torch.cuda.synchronize()
    return out.cpu().numpy()[0], idx.cpu().numpy()[0], cnt.cpu().numpy()[0]


def _same_packed(a, b):
    for x, y in zip(a.unpack(), b.unpack()):
        assert np.array_equal(x, y)
    assert torch.equal(a.kabsmax, b.kabsmax)


@pytest.mark.parametrize("dtype,n_rep", [(F16, 1), (BF16, 4)])
@pytest.mark.parametrize("block_tokens", [64, 256])
def test_paged_rows_give_the_contiguous_results(gu, oracle, dtype, n_rep, block_tokens):
    # lengths: in the middle of a block, one short of a block end, exactly at a block end (the appended row opens
    # a new block), a single row
    lens = [1500, 1023, 1024, 1]
    wl = synth.make_workload("paged", 70 + block_tokens + dtype, 4, 2 * n_rep, 2, lens, [120, 64, 200, 2], dtype,
                             max_ctx=1536, n_planted=4, chan="lognormal" if dtype == BF16 else "ones")
    flat = gu.DeviceWorkload(wl)
    paged = gu.PagedWorkload(wl, block_tokens, seed=block_tokens)
    assert np.array_equal(paged.logical(paged.K), wl.K)
    for dw in (flat, paged):
        B.quantize_keys(dw.cfg, dw.cache)
    torch.cuda.synchronize()
    _same_packed(flat.cache, paged.cache)
    # dense attention over all rows
    outs = []
    for dw in (flat, paged):
        o = torch.zeros((wl.units, wl.n_rep, 128), dtype=torch.float32, device="cuda")
        B.dense_attn(dw.cfg, dw.cache, dw.q, 0, o, B.make_workspace(dw.cfg, dw.cfg.max_ctx))
        outs.append(o.cpu().numpy())
    assert np.array_equal(outs[0], outs[1])
    # the fused step without and with an append
    mb = int(wl.budgets.max())
    for append in (False, True):
        a = _step(flat, append, mb)
        b = _step(paged, append, mb)
        for x, y in zip(a, b):
            assert np.array_equal(x, y), append
    r = oracle_step(oracle, wl, append=True)
    out_p, idx_p, cnt_p = b
    check_index_sets(idx_p, cnt_p, r["idx"], r["count"], r["scores"], r["L"])
    want = oracle.attention(r["K"], r["V"], wl.q, r["L"], r["sm_scale"], wl.dtype,
                            np.ascontiguousarray(np.where(idx_p < 0, 0, idx_p)), cnt_p, 2)
    assert np.abs(out_p - want).max() <= 2e-3
    # the appended rows landed where the block table says, nothing else moved
    Kl, Vl = paged.logical(paged.K), paged.logical(paged.V)
    for u in range(wl.units):
        n = int(r["L"][u])
        assert np.array_equal(Kl[u, :n], r["K"][u, :n]) and np.array_equal(Vl[u, :n], r["V"][u, :n]), u
        assert (Kl[u, n:] == wl.K[u, n:]).all()
    assert paged.poison_intact()
    _same_packed(flat.cache, paged.cache)
    # sparse attention on a given selection
    outs = []
    idx_d, cnt_d = gu.i32(np.where(idx_p < 0, 0, idx_p)), gu.i32(cnt_p)
    for dw in (flat, paged):
        o = torch.zeros((wl.units, wl.n_rep, 128), dtype=torch.float32, device="cuda")
        B.sparse_attn(dw.cfg, dw.cache, dw.q, idx_d, cnt_d, mb, o, dw.workspace(mb))
        outs.append(o.cpu().numpy())
    assert np.array_equal(outs[0], outs[1])


@pytest.mark.parametrize("g", [128, 256])
def test_paged_rows_with_long_groups_and_appends(gu, oracle, g):
    """Blocks of exactly one group (g = 256) or two (g = 128): bulk quantization and 300 appends that cross group
    and block boundaries, against the oracle's append on the logical rows."""
    dtype = BF16
    wl = synth.make_workload(f"pagedg{g}", 90 + g, 2, 4, 2, [700, 255], [64, 32], dtype, max_ctx=1280, n_planted=2,
                             chan="lognormal")
    paged = gu.PagedWorkload(wl, 256, group_size=g, seed=g)
    B.quantize_keys(paged.cfg, paged.cache)
    K, V, L = wl.K.copy(), wl.V.copy(), wl.unit_lens.copy()
    bits, s, z = oracle.quantize(K, L, g, dtype, 2)
    rng = np.random.default_rng(g)
    steps = 300
    kn_all = synth.f32_to_words(rng.standard_normal((steps, wl.units, 128)).astype(np.float32) * 1.5, dtype)
    vn_all = synth.f32_to_words(rng.standard_normal((steps, wl.units, 128)).astype(np.float32), dtype)
    kn_d, vn_d = gu.to_dev(kn_all, dtype), gu.to_dev(vn_all, dtype)
    for t in range(steps):
        B.append_key(paged.cfg, paged.cache, kn_d[t], vn_d[t])
        paged.seq_lens.add_(1)
        oracle.append(K, V, L, kn_all[t], vn_all[t], bits, s, z, g, dtype)
        L = (L + 1).astype(np.int32)
    torch.cuda.synchronize()
    got = paged.cache.unpack()
    for u in range(wl.units):
        n = int(L[u])
        ng = (n + g - 1) // g
        assert np.array_equal(got[0][u, :n], bits[u, :n]), u
        assert np.array_equal(got[1][u, :ng], s[u, :ng]) and np.array_equal(got[2][u, :ng], z[u, :ng]), u
        assert np.array_equal(paged.logical(paged.K)[u, :n], K[u, :n])
        assert np.array_equal(paged.logical(paged.V)[u, :n], V[u, :n])
    assert paged.poison_intact()


def test_paged_page_minmax(gu):
    wl = synth.make_workload("pagedmm", 5, 2, 4, 2, [900, 130], [64, 32], F16, max_ctx=1024, n_planted=2)
    flat = gu.DeviceWorkload(wl)
    paged = gu.PagedWorkload(wl, 128, seed=3)
    metas = []
    for dw in (flat, paged):
        m = torch.zeros(B.page_meta_bytes(dw.cfg, 16) // 4, dtype=torch.int32, device="cuda")
        B.page_minmax(dw.cfg, dw.cache, 16, m)
        metas.append(m.cpu().numpy())
    assert np.array_equal(metas[0], metas[1])
