"""The second kernel of the fused step (threshold + attention in one launch) on the paths an ordinary run rarely takes,
and a direct check of WHICH rows it attended over.

* The kernel's checksums (count and sum of the token indices of the rows every workgroup gathered, test flag 2) must
  equal those of the index list the step reports: the attention output alone cannot show a handful of wrong rows
  among thousands inside its 2e-3 tolerance, the checksums can.
* With test flag 1 no workgroup picks up the published threshold: all threshold-bin rows are then attended over by the
  merging workgroup's fallback.  Same selection, same checksums, output equal to the ordinary path up to summation order.
* R = 0 (a zero query, or an all-zero key cache): every score is zero, the budget goes to the lowest indices.
* The three-kernel form (threshold kernel, then selection + attention) on shapes whose step takes the two-kernel one.
* The hand-off between workgroups (candidates, threshold word, partials) repeated over a few hundred launches with many
  small workgroups per unit: every launch must reproduce the first one bit for bit.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from helpers import check_index_sets, oracle_step  # noqa: E402
from paper_2508_08256_amd import binding as B  # noqa: E402
from paper_2508_08256_amd import synth  # noqa: E402

pytestmark = pytest.mark.gpu
F16, BF16 = 0, 1
FORCE_LATE, CHECKSUMS = 1, 2
THREE_KERNELS = 4     # phases 2 + 64, 3 + 64


@pytest.fixture(scope="module")
def gu():
    import gpu_util

    assert torch.cuda.is_available()
    return gpu_util


def _ctl_checksums(ws, units):
    """(count, index sum) the kernel accumulated in the unit control blocks at the head of the workspace."""
    ctl = ws[: units * 64].cpu().numpy().view(np.uint32).reshape(units, 16)
    return ctl[:, 14].copy(), ctl[:, 15].copy()


def _clear_checksums(ws, units):
    ctl = ws[: units * 64].view(torch.int32).view(units, 16)
    ctl[:, 14:16] = 0


def _step(gu, wl, flags, append=True):
    """One fused step issued kernel by kernel with test flags on the second one."""
    dw = gu.DeviceWorkload(wl)
    B.quantize_keys(dw.cfg, dw.cache)
    mb = int(wl.budgets.max())
    out = torch.full((1, wl.units, wl.n_rep, 128), float("nan"), dtype=torch.float32, device="cuda")
    idx = torch.full((1, wl.units, mb), -1, dtype=torch.int32, device="cuda")
    cnt = torch.full((1, wl.units), -1, dtype=torch.int32, device="cuda")
    kn = dw.k_new[None].contiguous() if append else None
    vn = dw.v_new[None].contiguous() if append else None
    ws = dw.workspace(mb)
    args = (dw.cfg, [dw.cache], dw.q[None].contiguous(), kn, vn, dw.budgets, mb, out, idx, cnt, ws)
    _clear_checksums(ws, wl.units)
    # + 16 f, f = 1..3: the two-kernel form whatever the shape; + 64: the three-kernel form whatever the shape
    for p in (1, 2 + 16 * flags, 3 + 16 * flags):
        B.decode_step_phase(*args, p)
    torch.cuda.synchronize()
    return out.cpu().numpy()[0], idx.cpu().numpy()[0], cnt.cpu().numpy()[0], _ctl_checksums(ws, wl.units)


def _check_sums(idx, cnt, sums):
    for u in range(len(cnt)):
        sel = idx[u, :cnt[u]].astype(np.uint64)
        assert sums[0][u] == cnt[u], (u, sums[0][u], cnt[u])
        assert sums[1][u] == np.uint32(int(sel.sum()) & 0xFFFFFFFF), (u, sums[1][u], int(sel.sum()))


WORKLOADS = [
    ("ragged_f16", lambda: synth.small_ragged(7, F16, 1)),
    ("ragged_bf16_gqa4", lambda: synth.small_ragged(8, BF16, 4)),
    ("config1", lambda: synth.config1()),
    ("gqa2_long", lambda: synth.make_workload("g2", 31, 2, 8, 4, [9000, 4133], [700, 333], BF16, chan="lognormal",
                                              n_planted=8)),
    ("gqa8", lambda: synth.make_workload("g8", 32, 1, 16, 2, [5000], [64], F16, n_planted=4)),
    ("edge_lens", lambda: synth.make_workload("edge", 11, 8, 16, 8, [0, 1, 31, 32, 33, 64, 65, 191],
                                              [1, 1, 5, 32, 40, 7, 65, 20], F16, max_ctx=192, n_planted=1, plant=False)),
]


@pytest.mark.parametrize("name,make", WORKLOADS, ids=[w[0] for w in WORKLOADS])
def test_attended_rows_are_the_reported_selection(gu, oracle, name, make):
    wl = make()
    print(f"[step paths] {name}", flush=True)
    r = oracle_step(oracle, wl, append=True)
    out, idx, cnt, sums = _step(gu, wl, CHECKSUMS)
    check_index_sets(idx, cnt, r["idx"], r["count"], r["scores"], r["L"])
    _check_sums(idx, cnt, sums)
    want = oracle.attention(r["K"], r["V"], wl.q, r["L"], r["sm_scale"], wl.dtype,
                            np.ascontiguousarray(np.where(idx < 0, 0, idx)), cnt, 4)
    assert np.abs(out - want).max() <= 2e-3
    # the fallback: nobody picks up the threshold, the merging workgroup attends over every threshold-bin row
    out2, idx2, cnt2, sums2 = _step(gu, wl, CHECKSUMS | FORCE_LATE)
    assert np.array_equal(idx2, idx) and np.array_equal(cnt2, cnt)
    _check_sums(idx2, cnt2, sums2)
    assert np.abs(out2 - want).max() <= 2e-3
    assert np.abs(out2 - out).max() <= 1e-5 * max(1.0, float(np.abs(out).max()))


@pytest.mark.parametrize("name,make", WORKLOADS, ids=[w[0] for w in WORKLOADS])
def test_three_kernel_form_on_any_shape(gu, oracle, name, make):
    """The form long grouped-query grids take, forced on small shapes: same selection, same output bar."""
    wl = make()
    print(f"[step paths, three kernels] {name}", flush=True)
    r = oracle_step(oracle, wl, append=True)
    out, idx, cnt, _ = _step(gu, wl, THREE_KERNELS)
    check_index_sets(idx, cnt, r["idx"], r["count"], r["scores"], r["L"])
    want = oracle.attention(r["K"], r["V"], wl.q, r["L"], r["sm_scale"], wl.dtype,
                            np.ascontiguousarray(np.where(idx < 0, 0, idx)), cnt, 4)
    assert np.abs(out - want).max() <= 2e-3


@pytest.mark.parametrize("kind", ["zero_query", "zero_keys", "zero_keys_then_append"])
@pytest.mark.parametrize("flags", [CHECKSUMS, CHECKSUMS | FORCE_LATE])
def test_zero_score_range(gu, oracle, kind, flags):
    """R = sum_c |q_c| absmax_c = 0: the histogram has no width, every score is exactly zero and the ties go to the
    lowest token indices (a unit with a live query sits next to the degenerate one)."""
    wl = synth.make_workload("r0", 77, 2, 4, 2, [1500, 300], [100, 37], F16, n_planted=2)
    if kind == "zero_query":
        wl.q[0:2] = 0                      # both query heads of unit 0
    else:
        wl.K[1, :] = 0                     # unit 1's cached keys
        if kind == "zero_keys":
            wl.k_new[1] = 0
    append = True
    r = oracle_step(oracle, wl, append=append)
    out, idx, cnt, sums = _step(gu, wl, flags, append=append)
    check_index_sets(idx, cnt, r["idx"], r["count"], r["scores"], r["L"])
    _check_sums(idx, cnt, sums)
    u = 0 if kind == "zero_query" else 1
    if kind != "zero_keys_then_append":
        assert np.array_equal(idx[u, :cnt[u]], np.arange(cnt[u]))      # all scores tie: the lowest indices
    want = oracle.attention(r["K"], r["V"], wl.q, r["L"], r["sm_scale"], wl.dtype,
                            np.ascontiguousarray(np.where(idx < 0, 0, idx)), cnt, 4)
    assert np.abs(out - want).max() <= 2e-3
    # the stand-alone calls on the same inputs
    dw = gu.DeviceWorkload(wl)
    B.quantize_keys(dw.cfg, dw.cache)
    B.append_key(dw.cfg, dw.cache, dw.k_new, dw.v_new)
    scores = torch.zeros((wl.units, wl.max_ctx), dtype=torch.float32, device="cuda")
    B.score(dw.cfg, dw.cache, dw.q, 1, scores)
    mb = int(wl.budgets.max())
    for call in ("topk", "topk_ws"):
        i2 = torch.full((wl.units, mb), -1, dtype=torch.int32, device="cuda")
        c2 = torch.full((wl.units,), -1, dtype=torch.int32, device="cuda")
        if call == "topk":
            B.topk(dw.cfg, scores, dw.seq_lens, 1, dw.budgets, mb, i2, c2)
        else:
            B.topk_ws(dw.cfg, scores, dw.seq_lens, 1, dw.budgets, mb, i2, c2, dw.workspace(mb))
        torch.cuda.synchronize()
        check_index_sets(i2.cpu().numpy(), c2.cpu().numpy(), r["idx"], r["count"], r["scores"], r["L"])


def test_hand_off_between_workgroups_is_stable_over_many_launches(gu, oracle):
    """Many units, many small workgroups per unit (a budget near the context makes every 1024-token range a workgroup
    of its own), a few hundred launches on one workspace: the candidates, the threshold word, the flags and the
    partials all cross workgroups through memory, so a stale read would show as a launch that differs from the
    first.  The first launch is checked against the oracle."""
    lens = [6100 + 517 * (i % 5) for i in range(16)]
    buds = [int(0.45 * l) for l in lens]
    wl = synth.make_workload("handoff", 55, 16, 4, 4, lens, buds, F16, n_planted=8)
    r = oracle_step(oracle, wl, append=True)
    dw = gu.DeviceWorkload(wl)
    B.quantize_keys(dw.cfg, dw.cache)
    mb = int(wl.budgets.max())
    kn, vn = dw.k_new[None].contiguous(), dw.v_new[None].contiguous()
    out = torch.zeros((1, wl.units, wl.n_rep, 128), dtype=torch.float32, device="cuda")
    idx = torch.full((1, wl.units, mb), -1, dtype=torch.int32, device="cuda")
    cnt = torch.full((1, wl.units), -1, dtype=torch.int32, device="cuda")
    ws = dw.workspace(mb)
    q = dw.q[None].contiguous()
    first = None
    # a priming launch: the first append raises the unit's per-channel bound, and with it the histogram's range and the
    # split of a workgroup's rows into sure ones and candidates (hence the order they are summed in) for later launches
    B.decode_step(dw.cfg, [dw.cache], q, kn, vn, dw.budgets, mb, out, idx, cnt, ws)
    for it in range(300):
        out.fill_(float("nan"))
        # every launch appends the same row at the same place (seq_lens is the caller's and stays as it is)
        B.decode_step(dw.cfg, [dw.cache], q, kn, vn, dw.budgets, mb, out, idx, cnt, ws)
        torch.cuda.synchronize()
        got = (out.clone(), idx.clone(), cnt.clone())
        if first is None:
            first = got
            idx_g, cnt_g = idx.cpu().numpy()[0], cnt.cpu().numpy()[0]
            check_index_sets(idx_g, cnt_g, r["idx"], r["count"], r["scores"], r["L"])
            want = oracle.attention(r["K"], r["V"], wl.q, r["L"], r["sm_scale"], wl.dtype,
                                    np.ascontiguousarray(np.where(idx_g < 0, 0, idx_g)), cnt_g, 4)
            assert np.abs(out.cpu().numpy()[0] - want).max() <= 2e-3
        else:
            assert torch.equal(got[1], first[1]) and torch.equal(got[2], first[2]), f"selection differs at launch {it}"
            assert torch.equal(got[0], first[0]), f"output differs at launch {it}"

