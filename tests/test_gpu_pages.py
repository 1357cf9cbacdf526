"""GPU parity of the page-level importance workload (the page-retrieval baseline of Sec. 3.2 and the averaged
quantized score of Sec. 4.4) against the oracle: page min/max vectors bit-exact (bulk and appended), page scores
exact (Eq. 3 as printed, one query head) or within fp32 summation tolerance, page expansion exact, and the whole
pipeline page score -> top pages -> tokens -> attention."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from helpers import check_index_sets  # noqa: E402
from paper_2508_08256_amd import binding as B  # noqa: E402
from paper_2508_08256_amd import synth  # noqa: E402

pytestmark = pytest.mark.gpu
F16, BF16 = 0, 1


@pytest.fixture(scope="module")
def gu():
    import gpu_util

    assert torch.cuda.is_available()
    return gpu_util


def _meta_of(t):
    m = t.cpu().numpy().view(np.uint32)
    return (m & 0xffff).astype(np.uint16), (m >> 16).astype(np.uint16)


@pytest.mark.parametrize("dtype,n_rep,page", [(F16, 1, 16), (BF16, 4, 16), (F16, 2, 32), (BF16, 1, 8)])
def test_page_pipeline_matches_oracle(gu, oracle, dtype, n_rep, page):
    lens = [2000, 333, 64, 1]
    budgets = [320, 64, 64, 32]
    wl = synth.make_workload("pages", 60 + page + dtype, 4, 2 * n_rep, 2, lens, budgets, dtype, max_ctx=2048,
                             n_planted=4, chan="lognormal" if dtype == BF16 else "ones")
    dw = gu.DeviceWorkload(wl)
    cfg = dw.cfg
    U, NP = wl.units, wl.max_ctx // page
    L = wl.unit_lens.copy()
    # ---- page min / max vectors: bulk, then 40 appended rows ------------------------------------------------
    meta = torch.zeros(B.page_meta_bytes(cfg, page) // 4, dtype=torch.int32, device="cuda")
    B.page_minmax(cfg, dw.cache, page, meta)
    torch.cuda.synchronize()
    K = wl.K.copy()
    kmin_o, kmax_o = oracle.page_minmax(K, L, page, dtype)
    kmin_g, kmax_g = _meta_of(meta)
    assert np.array_equal(kmin_g.reshape(U, NP, 128), kmin_o) and np.array_equal(kmax_g.reshape(U, NP, 128), kmax_o)
    rng = np.random.default_rng(page)
    steps = 40
    kn_all = synth.f32_to_words(rng.standard_normal((steps, U, 128)).astype(np.float32) * 2.0, dtype)
    kn_d = gu.to_dev(kn_all, dtype)
    for t in range(steps):
        B.page_append(cfg, dw.seq_lens, page, kn_d[t], meta)
        dw.K[torch.arange(U), torch.as_tensor(L.astype(np.int64)).cuda()] = kn_d[t]   # the row itself
        dw.seq_lens.add_(1)
        for u in range(U):
            K[u, L[u]] = kn_all[t, u]
        L = (L + 1).astype(np.int32)
    torch.cuda.synchronize()
    kmin_o, kmax_o = oracle.page_minmax(K, L, page, dtype)
    kmin_g, kmax_g = _meta_of(meta)
    assert np.array_equal(kmin_g.reshape(U, NP, 128), kmin_o) and np.array_equal(kmax_g.reshape(U, NP, 128), kmax_o)
    # ---- page scores -------------------------------------------------------------------------------------------
    ps = torch.zeros((U, NP), dtype=torch.float32, device="cuda")
    npg = -(-L // page)
    for mode in (0, 1):
        B.page_score(cfg, meta, page, dw.seq_lens, 0, dw.q, mode, ps)
        torch.cuda.synchronize()
        want = oracle.page_score(kmin_o, kmax_o, wl.q, L, page, dtype, mode)
        got = ps.cpu().numpy().astype(np.float64)
        for u in range(U):
            n = int(npg[u])
            assert np.all(np.isneginf(got[u, n:]))
            if mode == 0 and n_rep == 1:
                assert np.array_equal(got[u, :n], want[u, :n])          # products of 16-bit floats are exact in fp32
            else:
                scale = np.abs(want[u, :n]).max() + 1e-30
                assert np.all(np.abs(got[u, :n] - want[u, :n]) <= 1e-4 * scale), (mode, u)
    # ---- the retrieval pipeline on the page scores of Eq. 3 (mode 0 leaves many exact ties: mode 1 here) ----------
    max_pages = max(b // page for b in budgets)
    pcfg = B.make_config(wl.batch, wl.n_q_heads, wl.n_kv_heads, NP, dtype)
    page_budgets = gu.i32(np.array([max(1, b // page) for b in budgets]))
    page_lens = gu.i32(np.array([-(-int(l) // page) for l in (np.array(lens) + steps)]))
    pidx = torch.full((U, max_pages), -1, dtype=torch.int32, device="cuda")
    pcnt = torch.zeros(U, dtype=torch.int32, device="cuda")
    B.topk(pcfg, ps, page_lens, 0, page_budgets, max_pages, pidx, pcnt)
    mb = max(budgets)
    idx = torch.full((U, mb), -1, dtype=torch.int32, device="cuda")
    cnt = torch.zeros(U, dtype=torch.int32, device="cuda")
    B.expand_pages(cfg, pidx, pcnt, max_pages, dw.seq_lens, 0, page, idx, cnt, mb)
    out = torch.zeros((U, wl.n_rep, 128), dtype=torch.float32, device="cuda")
    B.sparse_attn(cfg, dw.cache, dw.q, idx, cnt, mb, out, dw.workspace(mb))
    torch.cuda.synchronize()
    ub_pages = np.repeat(np.array([max(1, b // page) for b in budgets], np.int32), wl.n_kv_heads)
    pidx_o, pcnt_o = oracle.topk(want, npg.astype(np.int32), ub_pages, max_pages)
    check_index_sets(pidx.cpu().numpy(), pcnt.cpu().numpy(), pidx_o, pcnt_o, want, npg)
    idx_o, cnt_o = oracle.expand_pages(np.ascontiguousarray(pidx.cpu().numpy()), pcnt.cpu().numpy(), L, page, mb)
    assert np.array_equal(cnt.cpu().numpy(), cnt_o)
    ig = idx.cpu().numpy()
    for u in range(U):
        assert np.array_equal(ig[u, :cnt_o[u]], idx_o[u, :cnt_o[u]])
    ref = oracle.attention(K, wl.V, wl.q, L, 1.0 / np.sqrt(128.0), dtype, np.ascontiguousarray(np.where(ig < 0, 0, ig)),
                           cnt_o, 4)
    assert np.abs(out.cpu().numpy() - ref).max() <= 2e-3


def test_page_mean_of_quantized_scores(gu, oracle):
    wl = synth.small_ragged(9, F16, 1)
    dw = gu.DeviceWorkload(wl)
    B.quantize_keys(dw.cfg, dw.cache)
    sc = torch.zeros((wl.units, wl.max_ctx), dtype=torch.float32, device="cuda")
    B.score(dw.cfg, dw.cache, dw.q, 0, sc)
    pm = torch.zeros((wl.units, wl.max_ctx // 16), dtype=torch.float32, device="cuda")
    B.page_mean_score(dw.cfg, sc, dw.seq_lens, 0, 16, pm)
    torch.cuda.synchronize()
    L = wl.unit_lens
    sc_h = sc.cpu().numpy().astype(np.float64)
    for u in range(wl.units):
        sc_h[u, L[u]:] = 0.0
    want = oracle.page_mean(np.ascontiguousarray(sc_h), L, 16)       # of the GPU's own token scores
    got = pm.cpu().numpy().astype(np.float64)
    for u in range(wl.units):
        n = -(-int(L[u]) // 16)
        assert np.all(np.isneginf(got[u, n:]))
        assert np.all(np.abs(got[u, :n] - want[u, :n]) <= 1e-5 * (np.abs(sc_h[u]).max() + 1e-30))
