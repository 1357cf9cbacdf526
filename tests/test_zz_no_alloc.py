"""fier_decode_step_static (the step on the library's own scratch array, for callers that cannot allocate) against
fier_decode_step on a caller-provided workspace: same kernels, so outputs and selections must be bit-identical.
Two calls in a row on the shared array, the second with a smaller input (another workspace layout inside the same
array), then the first shape again."""
import numpy as np
import pytest
import torch

from gpu_util import DeviceWorkload
from paper_2508_08256_amd import binding as B
from paper_2508_08256_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gu():
    assert torch.cuda.is_available(), "GPU tests need the MI355X"
    B.lib()
    return True


def _both(wl, append=True):
    """(out, idx, count) of the workspace call and of the static-scratch call on the same inputs."""
    res = []
    for static in (False, True):
        dw = DeviceWorkload(wl)            # a fresh cache each time: the step appends a row
        B.quantize_keys(dw.cfg, dw.cache)
        mb = int(wl.budgets.max())
        out = torch.full((1, wl.units, wl.n_rep, 128), 7.0, dtype=torch.float32, device="cuda")
        idx = torch.full((1, wl.units, mb), -1, dtype=torch.int32, device="cuda")
        cnt = torch.full((1, wl.units), -1, dtype=torch.int32, device="cuda")
        kn = dw.k_new[None].contiguous() if append else None
        vn = dw.v_new[None].contiguous() if append else None
        q = dw.q[None].contiguous()
        if static:
            B.decode_step_static(dw.cfg, [dw.cache], q, kn, vn, dw.budgets, mb, out, idx, cnt)
        else:
            B.decode_step(dw.cfg, [dw.cache], q, kn, vn, dw.budgets, mb, out, idx, cnt, dw.workspace(mb))
        torch.cuda.synchronize()
        res.append((out.cpu().numpy(), idx.cpu().numpy(), cnt.cpu().numpy(), dw.cache.kbits.cpu().numpy()))
    return res


def test_static_scratch_step_equals_workspace_step(gu):
    big = synth.make_workload("noalloc_big", 901, 2, 8, 4, [5000, 3077], [550, 300], synth.BF16, chan="lognormal",
                              n_planted=8)
    small = synth.make_workload("noalloc_small", 902, 1, 4, 4, [700], [96], synth.F16, n_planted=4)
    for wl in (big, small, big):       # the second call is smaller, the third finds the array laid out for it
        (o_ws, i_ws, c_ws, b_ws), (o_st, i_st, c_st, b_st) = _both(wl)
        assert np.array_equal(c_ws, c_st)
        assert np.array_equal(i_ws, i_st)
        assert np.array_equal(o_ws, o_st), float(np.abs(o_ws - o_st).max())
        assert np.array_equal(b_ws, b_st)
        assert (c_st[0] == np.minimum(wl.unit_budgets, wl.unit_lens + 1)).all()


def test_static_scratch_rejects_what_does_not_fit(gu):
    """Beyond the array's 48 MiB the call returns FIER_EWORKSPACE and enqueues nothing (dummy pointers would fault)."""
    import ctypes as C

    cfg = B.make_config(16, 32, 8, 65536, B.BF16)
    assert B.workspace_bytes(cfg, 7209) > (48 << 20)
    good = B.Cache(0x1000, 0x2000, 0x3000, 0x4000, 0x4800, 0x5000)
    arr = (B.Cache * 1)(good)
    st = B.lib().fier_decode_step_static(C.byref(cfg), arr, 1, 0x6000, None, None, 0x5100, 7209, 0x9000, None, None, None)
    assert st == B.EWORKSPACE
