"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol, validates arguments on the
host before launching anything, and its packed layout has the size Eq. 8 says (no GPU needed)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2508_08256_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "fier.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(fier_[a-z_]+)\s*\(", hdr))
    assert declared == set(B.SYMBOLS), declared ^ set(B.SYMBOLS)
    lib = B.lib()
    for name in declared:
        assert getattr(lib, name) is not None


def test_status_strings():
    assert B.status_string(0) == "ok"
    for st in (-1, -2, -3, -4, -5, -6):
        assert B.status_string(st) not in ("ok", "unknown status")
    assert B.status_string(-99) == "unknown status"


def test_config_validation():
    ok = B.make_config(2, 32, 8, 4096, B.BF16)
    assert B.check_config(ok) == B.OK
    assert B.check_config(B.make_config(2, 32, 8, 4096, head_dim=64)) == B.EUNSUPPORTED
    assert B.check_config(B.make_config(2, 32, 8, 4096, group_size=128)) == B.OK
    assert B.check_config(B.make_config(2, 32, 8, 4096, group_size=48)) == B.EUNSUPPORTED
    assert B.check_config(B.make_config(2, 32, 8, 4160, group_size=256)) == B.ESHAPE   # 256 does not divide it
    assert B.packed_meta_bytes(B.make_config(2, 32, 8, 4096, group_size=256)) == 2 * 8 * 16 * 512
    assert B.check_config(B.make_config(2, 30, 8, 4096)) == B.ESHAPE
    assert B.check_config(B.make_config(2, 72, 8, 4096)) == B.EUNSUPPORTED      # n_rep = 9
    assert B.check_config(B.make_config(2, 32, 8, 4100)) == B.ESHAPE            # not a multiple of 64
    assert B.check_config(B.make_config(0, 32, 8, 4096)) == B.EINVAL
    assert B.check_config(B.make_config(2, 32, 8, 4096, kv_dtype=7)) == B.EINVAL
    assert B.packed_bits_bytes(B.make_config(2, 30, 8, 4096)) == 0
    assert B.workspace_bytes(ok, 0) == 0 and B.workspace_bytes(ok, 512) > 0


def test_packed_size_is_one_eighth_of_the_key_cache():
    """Eq. 8 at g = 32: (1 + 32/g)/16 = 0.125 of a 16-bit key cache; Tab. 4 prints 0.125 for Fier-g32."""
    cfg = B.make_config(4, 32, 8, 131072, B.BF16)
    key_bytes = cfg.units * cfg.max_ctx * cfg.head_dim * 2
    packed = B.packed_bits_bytes(cfg) + B.packed_meta_bytes(cfg)
    assert packed / key_bytes == 0.125
    assert B.packed_bits_bytes(cfg) == key_bytes // 16 and B.packed_meta_bytes(cfg) == key_bytes // 16
    assert packed == 32 * cfg.units * cfg.max_ctx


def test_calls_reject_bad_arguments_before_any_launch():
    lib = B.lib()
    cfg = B.make_config(1, 8, 8, 256)
    cache = B.Cache(0, 0, 0, 0, 0, 0)
    assert lib.fier_quantize_keys(C.byref(cfg), C.byref(cache), None) == B.EINVAL
    assert lib.fier_quantize_keys(None, C.byref(cache), None) == B.EINVAL
    cache = B.Cache(0x1000, 0x2008, 0x3000, 0x4000, 0x4800, 0x5000)
    assert lib.fier_quantize_keys(C.byref(cfg), C.byref(cache), None) == B.EALIGN
    good = B.Cache(0x1000, 0x2000, 0x3000, 0x4000, 0x4800, 0x5000)
    assert lib.fier_append_key(C.byref(cfg), C.byref(good), None, None, None) == B.EINVAL
    assert lib.fier_score(C.byref(cfg), C.byref(good), 0x6000, 2, 0x7000, None) == B.EINVAL
    assert lib.fier_score(C.byref(cfg), C.byref(good), 0x6004, 0, 0x7000, None) == B.EALIGN
    assert lib.fier_topk(C.byref(cfg), 0x6000, 0x5000, 0, 0x5100, 0, 0x7000, 0x8000, None) == B.EINVAL
    big = 1 << 30
    assert lib.fier_sparse_attn(C.byref(cfg), C.byref(good), 0x6000, 0x7000, 0x8000, 16, 0x9000, None, big,
                                None) == B.EWORKSPACE
    assert lib.fier_sparse_attn(C.byref(cfg), C.byref(good), 0x6000, 0x7000, 0x8000, 512, 0x9000, 0xA000, big,
                                None) == B.EINVAL                                 # budget above capacity
    assert lib.fier_dense_attn(C.byref(cfg), C.byref(good), 0x6000, 0, 0x9000, None, big, None) == B.EWORKSPACE
    arr = (B.Cache * 1)(good)
    assert lib.fier_decode_step(C.byref(cfg), arr, 1, 0x6000, 0x7000, None, 0x5100, 16, 0x9000, None, None,
                                0xA000, big, None) == B.EINVAL                    # k_new without v_new
    assert lib.fier_decode_step(C.byref(cfg), arr, 0, 0x6000, None, None, 0x5100, 16, 0x9000, None, None,
                                0xA000, big, None) == B.EINVAL
    bad = B.make_config(1, 8, 8, 256, head_dim=96)
    assert lib.fier_quantize_keys(C.byref(bad), C.byref(good), None) == B.EUNSUPPORTED


def test_block_table_fields_are_validated():
    lib = B.lib()
    cfg = B.make_config(1, 8, 8, 1024, group_size=128)
    ptrs = (0x1000, 0x2000, 0x3000, 0x4000, 0x4800, 0x5000)

    def status(table, block_tokens):
        return lib.fier_quantize_keys(C.byref(cfg), C.byref(B.Cache(*ptrs, table, block_tokens)), None)

    assert status(None, 64) == B.EINVAL          # a block size without a table
    assert status(0x6000, 0) == B.ESHAPE
    assert status(0x6000, 64) == B.ESHAPE        # smaller than a quantization group
    assert status(0x6000, 192) == B.ESHAPE       # not a power of two
    assert status(0x6000, 2048) == B.ESHAPE      # does not divide the row capacity
    assert status(0x6002, 128) == B.EALIGN
    cfg32 = B.make_config(1, 8, 8, 1024)
    assert lib.fier_quantize_keys(C.byref(cfg32), C.byref(B.Cache(*ptrs, 0x6000, 32)), None) == B.ESHAPE
    arr = (B.Cache * 1)(B.Cache(*ptrs, 0x6000, 96))
    assert lib.fier_decode_step(C.byref(cfg32), arr, 1, 0x6000, None, None, 0x5100, 16, 0x9000, None, None,
                                0xA000, 1 << 30, None) == B.ESHAPE
    assert lib.fier_page_minmax(C.byref(cfg32), C.byref(B.Cache(*ptrs, 0x6000, 96)), 16, 0x7000, None) == B.ESHAPE


def test_unpack_helpers_follow_the_documented_layout():
    """bit i of word d of a token <-> channel 64 (d & 1) + 2 i + (d >> 1);  meta word = s | z << 16."""
    cfg = B.make_config(1, 2, 2, 128)
    lib = B.lib()
    rng = np.random.default_rng(0)
    bits = rng.integers(0, 2, (cfg.units, cfg.max_ctx, 128)).astype(np.uint8)
    packed = np.zeros((cfg.units, cfg.max_ctx, 4), np.uint32)
    for c in range(128):
        d = (c // 64) + 2 * (c % 2)
        i = (c % 64) // 2
        packed[:, :, d] |= bits[:, :, c].astype(np.uint32) << np.uint32(i)
    got = np.zeros_like(bits)
    lib.fier_unpack_bits(C.byref(cfg), packed.ctypes.data_as(C.c_void_p), got.ctypes.data_as(C.c_void_p))
    assert np.array_equal(got, bits)
    s = rng.integers(0, 65536, (cfg.units, cfg.max_ctx // 32, 128)).astype(np.uint16)
    z = rng.integers(0, 65536, s.shape).astype(np.uint16)
    meta = s.astype(np.uint32) | (z.astype(np.uint32) << np.uint32(16))
    s2, z2 = np.zeros_like(s), np.zeros_like(z)
    lib.fier_unpack_meta(C.byref(cfg), meta.ctypes.data_as(C.c_void_p), s2.ctypes.data_as(C.c_void_p),
                         z2.ctypes.data_as(C.c_void_p))
    assert np.array_equal(s2, s) and np.array_equal(z2, z)


def test_no_cpu_fallback_when_library_missing(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "libfier.so"))
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        B.lib()


def test_every_call_checks_the_workspace_size_before_any_launch():
    """Every entry point that carves a workspace takes its size and returns FIER_EWORKSPACE, on the host and before
    any launch, when it is smaller than fier_workspace_bytes for the selection size the call works with: the
    budget for the sparse calls, the row capacity for whole-cache attention (also inside the mixed step).  Dummy
    pointers: nothing may be launched (a launch on them would fault; on this machine there is not even a GPU)."""
    lib = B.lib()
    cfg = B.make_config(1, 8, 8, 4096)
    good = B.Cache(0x1000, 0x2000, 0x3000, 0x4000, 0x4800, 0x5000)
    arr = (B.Cache * 1)(good)
    ws = 0x100000
    need64, need_all = B.workspace_bytes(cfg, 64), B.workspace_bytes(cfg, 4096)
    assert 0 < need64 < need_all
    cfgp, cachep = C.byref(cfg), C.byref(good)
    assert lib.fier_sparse_attn(cfgp, cachep, 0x6000, 0x7000, 0x8000, 64, 0x9000, ws, need64 - 1, None) == B.EWORKSPACE
    assert lib.fier_sparse_attn(cfgp, cachep, 0x6000, 0x7000, 0x8000, 65, 0x9000, ws, need64, None) == B.EWORKSPACE
    assert lib.fier_dense_attn(cfgp, cachep, 0x6000, 0, 0x9000, ws, need64, None) == B.EWORKSPACE
    assert lib.fier_dense_attn(cfgp, cachep, 0x6000, 0, 0x9000, ws, need_all - 1, None) == B.EWORKSPACE
    assert lib.fier_topk_ws(cfgp, 0x6000, 0x5000, 0, 0x5100, 64, 0x7000, 0x8000, ws, need64 - 1, None) == B.EWORKSPACE
    step = (cfgp, arr, 1, 0x6000, None, None, 0x5100, 64, 0x9000, None, None)
    assert lib.fier_decode_step(*step, ws, need64 - 1, None) == B.EWORKSPACE
    assert lib.fier_decode_step(*step, ws, 0, None) == B.EWORKSPACE
    assert lib.fier_decode_step(*step, None, need64, None) == B.EWORKSPACE
    assert lib.fier_decode_step_phase(*step, ws, need64 - 1, 1, None) == B.EWORKSPACE
    dense = (C.c_uint8 * 1)(1)
    mixed = (cfgp, arr, 1, dense, 0x6000, None, None, 0x5100, 64, 0x9000, None, None)
    assert lib.fier_decode_step_mixed(*mixed, ws, need64, None) == B.EWORKSPACE      # a dense layer needs max_ctx
    assert lib.fier_decode_step_mixed(*mixed, ws, need_all - 1, None) == B.EWORKSPACE
    none_dense = (C.c_uint8 * 1)(0)
    mixed0 = (cfgp, arr, 1, none_dense, 0x6000, None, None, 0x5100, 64, 0x9000, None, None)
    assert lib.fier_decode_step_mixed(*mixed0, ws, need64 - 1, None) == B.EWORKSPACE
    # the workspace must be 256-byte aligned, as the header says
    assert lib.fier_decode_step(*step, ws + 16, need64, None) == B.EALIGN
    assert lib.fier_sparse_attn(cfgp, cachep, 0x6000, 0x7000, 0x8000, 64, 0x9000, ws + 128, need64, None) == B.EALIGN


def test_binding_passes_the_workspace_size(monkeypatch):
    """The binding hands the tensor's size to the C entry point, which refuses a short one."""
    import types

    import torch

    monkeypatch.setattr(B, "_stream", lambda: None)   # no GPU here; the check comes before any launch

    cfg = B.make_config(1, 8, 8, 4096)
    small = torch.zeros(B.workspace_bytes(cfg, 64), dtype=torch.uint8)
    cache = types.SimpleNamespace(c=B.Cache(0x1000, 0x2000, 0x3000, 0x4000, 0x4800, 0x5000))
    t = types.SimpleNamespace(data_ptr=lambda: 0x6000)
    for call in (lambda: B.dense_attn(cfg, cache, t, 0, t, small),
                 lambda: B.sparse_attn(cfg, cache, t, t, t, 65, t, small),
                 lambda: B.decode_step_mixed(cfg, [cache], [True], t, None, None, t, 64, t, None, None, small)):
        with pytest.raises(B.FierError) as e:
            call()
        assert e.value.status == B.EWORKSPACE


def test_form_of_the_step_follows_from_the_shape():
    """fier_decode_step_kernels: two kernels with one or two query heads per kv head; with more of them where the
    second kernel's grid is at most twice the resident one and the index list is not asked for; three otherwise;
    0 for an invalid configuration."""
    k = B.decode_step_kernels
    for with_list in (False, True):
        assert k(B.make_config(1, 8, 8, 4160), 512, with_list) == 2                 # 8 units x 4k tokens
        assert k(B.make_config(1, 32, 32, 32832), 3604, with_list) == 2             # 32 units x 32k
        assert k(B.make_config(1, 32, 32, 65600), 256, with_list) == 2
        assert k(B.make_config(1, 32, 32, 65600), 16384, with_list) == 2
        assert k(B.make_config(2, 32, 16, 32832, B.BF16), 3604, with_list) == 2     # two query heads per kv head
        assert k(B.make_config(4, 32, 32, 131136), 4096, with_list) == 2            # 128 MHA units x 128k
        assert k(B.make_config(32, 32, 8, 131136, B.BF16), 4096, with_list) == 3    # GQA far beyond the resident grid
    assert k(B.make_config(8, 32, 8, 32832, B.BF16), 3604) == 2      # four query heads per kv head, resident grid
    assert k(B.make_config(4, 32, 8, 131136, B.BF16), 4096) == 2
    assert k(B.make_config(8, 32, 8, 131136, B.BF16), 4096) == 2     # up to twice the resident grid
    assert k(B.make_config(8, 32, 8, 32832, B.BF16), 3604, True) == 3    # the same with the index list as an output
    assert k(B.make_config(4, 32, 8, 131136, B.BF16), 4096, True) == 3
    assert k(B.make_config(2, 30, 8, 4096), 64) == 0
    assert k(B.make_config(1, 8, 8, 4160), 0) == 0
