"""ctypes binding of include/fier.h.  Argument marshalling only: every step runs in the HIP kernels.

Tensors are torch tensors on the GPU (PyTorch is used for device memory and streams only); each function
has the name and the argument order of the C entry point and enqueues on torch's current stream.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfier.so")

F16, BF16 = 0, 1
OK = 0
EINVAL, ESHAPE, EALIGN, EWORKSPACE, EUNSUPPORTED, EHIP = -1, -2, -3, -4, -5, -6

SYMBOLS = ["fier_packed_bits_bytes", "fier_packed_meta_bytes", "fier_workspace_bytes", "fier_workspace_scores_offset",
           "fier_status_string",
           "fier_check_config", "fier_quantize_keys", "fier_append_key", "fier_score", "fier_topk", "fier_topk_ws",
           "fier_sparse_attn", "fier_dense_attn", "fier_decode_step", "fier_decode_step_static", "fier_decode_step_mixed", "fier_decode_step_phase",
           "fier_decode_step_kernels", "fier_page_meta_bytes",
           "fier_page_minmax", "fier_page_append", "fier_page_score", "fier_page_mean_score", "fier_expand_pages", "fier_unpack_bits",
           "fier_unpack_meta"]


class FierError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {status_string(status)} ({status})")


class Config(C.Structure):
    _fields_ = [("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("group_size", C.c_int32), ("max_ctx", C.c_int32), ("batch", C.c_int32),
                ("kv_dtype", C.c_int32), ("sm_scale", C.c_float)]

    @property
    def units(self):
        return self.batch * self.n_kv_heads

    @property
    def n_rep(self):
        return self.n_q_heads // self.n_kv_heads


class Cache(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("kbits", C.c_void_p), ("kmeta", C.c_void_p),
                ("kabsmax", C.c_void_p), ("seq_lens", C.c_void_p), ("block_table", C.c_void_p),
                ("block_tokens", C.c_int32)]


def make_config(batch, n_q_heads, n_kv_heads, max_ctx, kv_dtype=F16, head_dim=128, group_size=32, sm_scale=None):
    if sm_scale is None:
        sm_scale = 1.0 / float(np.sqrt(head_dim))
    return Config(n_q_heads, n_kv_heads, head_dim, group_size, max_ctx, batch, kv_dtype, sm_scale)


_lib = None


def lib():
    """Load libfier.so.  Raises if it has not been built: the product has no other path."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2508_08256_amd.build` "
                               "(there is no CPU fallback)")
        L = C.CDLL(LIB_PATH)
        vp, i32, cfgp = C.c_void_p, C.c_int32, C.POINTER(Config)
        cachep = C.POINTER(Cache)
        L.fier_packed_bits_bytes.restype = C.c_size_t
        L.fier_packed_bits_bytes.argtypes = [cfgp]
        L.fier_packed_meta_bytes.restype = C.c_size_t
        L.fier_packed_meta_bytes.argtypes = [cfgp]
        L.fier_workspace_bytes.restype = C.c_size_t
        L.fier_workspace_bytes.argtypes = [cfgp, i32]
        L.fier_workspace_scores_offset.restype = C.c_size_t
        L.fier_workspace_scores_offset.argtypes = [cfgp, i32]
        L.fier_decode_step_kernels.restype = C.c_int
        L.fier_decode_step_kernels.argtypes = [cfgp, i32, i32]
        L.fier_status_string.restype = C.c_char_p
        L.fier_status_string.argtypes = [C.c_int]
        L.fier_check_config.restype = C.c_int
        L.fier_check_config.argtypes = [cfgp]
        L.fier_quantize_keys.restype = C.c_int
        L.fier_quantize_keys.argtypes = [cfgp, cachep, vp]
        L.fier_append_key.restype = C.c_int
        L.fier_append_key.argtypes = [cfgp, cachep, vp, vp, vp]
        L.fier_score.restype = C.c_int
        L.fier_score.argtypes = [cfgp, cachep, vp, i32, vp, vp]
        L.fier_topk.restype = C.c_int
        L.fier_topk.argtypes = [cfgp, vp, vp, i32, vp, i32, vp, vp, vp]
        L.fier_topk_ws.restype = C.c_int
        L.fier_topk_ws.argtypes = [cfgp, vp, vp, i32, vp, i32, vp, vp, vp, C.c_size_t, vp]
        L.fier_sparse_attn.restype = C.c_int
        L.fier_sparse_attn.argtypes = [cfgp, cachep, vp, vp, vp, i32, vp, vp, C.c_size_t, vp]
        L.fier_dense_attn.restype = C.c_int
        L.fier_dense_attn.argtypes = [cfgp, cachep, vp, i32, vp, vp, C.c_size_t, vp]
        L.fier_decode_step.restype = C.c_int
        L.fier_decode_step.argtypes = [cfgp, cachep, i32, vp, vp, vp, vp, i32, vp, vp, vp, vp, C.c_size_t, vp]
        L.fier_decode_step_static.restype = C.c_int
        L.fier_decode_step_static.argtypes = [cfgp, cachep, i32, vp, vp, vp, vp, i32, vp, vp, vp, vp]
        L.fier_page_meta_bytes.restype = C.c_size_t
        L.fier_page_meta_bytes.argtypes = [cfgp, i32]
        L.fier_page_minmax.restype = C.c_int
        L.fier_page_minmax.argtypes = [cfgp, cachep, i32, vp, vp]
        L.fier_page_append.restype = C.c_int
        L.fier_page_append.argtypes = [cfgp, vp, i32, vp, vp, vp]
        L.fier_page_score.restype = C.c_int
        L.fier_page_score.argtypes = [cfgp, vp, i32, vp, i32, vp, i32, vp, vp]
        L.fier_page_mean_score.restype = C.c_int
        L.fier_page_mean_score.argtypes = [cfgp, vp, vp, i32, i32, vp, vp]
        L.fier_expand_pages.restype = C.c_int
        L.fier_expand_pages.argtypes = [cfgp, vp, vp, i32, vp, i32, i32, vp, vp, i32, vp]
        L.fier_decode_step_mixed.restype = C.c_int
        L.fier_decode_step_mixed.argtypes = [cfgp, cachep, i32, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp, C.c_size_t, vp]
        L.fier_decode_step_phase.restype = C.c_int
        L.fier_decode_step_phase.argtypes = [cfgp, cachep, i32, vp, vp, vp, vp, i32, vp, vp, vp, vp, C.c_size_t, i32, vp]
        L.fier_unpack_bits.restype = None
        L.fier_unpack_bits.argtypes = [cfgp, vp, vp]
        L.fier_unpack_meta.restype = None
        L.fier_unpack_meta.argtypes = [cfgp, vp, vp, vp]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().fier_status_string(int(status)).decode()


def _check(status: int, what: str):
    if status != OK:
        raise FierError(status, what)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    import torch

    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def packed_bits_bytes(cfg: Config) -> int:
    return int(lib().fier_packed_bits_bytes(C.byref(cfg)))


def packed_meta_bytes(cfg: Config) -> int:
    return int(lib().fier_packed_meta_bytes(C.byref(cfg)))


def workspace_bytes(cfg: Config, max_budget: int) -> int:
    return int(lib().fier_workspace_bytes(C.byref(cfg), int(max_budget)))


def workspace_scores(cfg: Config, max_budget: int, workspace):
    """View of the step's score array [units][max_ctx] float32 inside a workspace tensor (for inspection)."""
    import torch

    off = int(lib().fier_workspace_scores_offset(C.byref(cfg), int(max_budget)))
    assert off > 0 and off % 4 == 0
    n = cfg.units * cfg.max_ctx
    return workspace[off:off + 4 * n].view(torch.float32).view(cfg.units, cfg.max_ctx)


def decode_step_kernels(cfg: Config, max_budget: int, with_index_list: bool = False) -> int:
    """2 or 3: the number of kernels fier_decode_step launches per layer for this shape, without or with idx_out
    (the optional index-list kernel of the two-kernel form not counted)."""
    return int(lib().fier_decode_step_kernels(C.byref(cfg), int(max_budget), 1 if with_index_list else 0))


def make_workspace(cfg: Config, max_budget: int):
    """A zero-filled workspace on the GPU (the library keeps its counters zero from then on)."""
    import torch

    n = workspace_bytes(cfg, max_budget)
    assert n > 0
    return torch.zeros(n, dtype=torch.uint8, device="cuda")


def _ws(workspace):
    """(pointer, size in bytes) of a workspace tensor, as the C entry points take it; they check the size."""
    if workspace is None:
        return None, 0
    return C.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size()


def check_config(cfg: Config) -> int:
    return int(lib().fier_check_config(C.byref(cfg)))


class DeviceCache:
    """One layer's buffers on the GPU.  k, v: [units][max_ctx][128] 16-bit tensors; seq_lens [batch] int32.
    With block_table ([batch][max_ctx / block_tokens] int32), k and v are block pools
    [pool blocks][n_kv_heads][block_tokens][128] instead."""

    def __init__(self, cfg: Config, k, v, seq_lens, block_table=None):
        import torch

        self.cfg = cfg
        self.k, self.v, self.seq_lens, self.block_table = k, v, seq_lens, block_table
        assert k.is_cuda and k.is_contiguous() and v.is_contiguous() and k.shape == v.shape
        assert k.element_size() == 2
        block_tokens = 0
        if block_table is None:
            assert tuple(k.shape) == (cfg.units, cfg.max_ctx, cfg.head_dim), k.shape
        else:
            assert k.dim() == 4 and k.shape[1] == cfg.n_kv_heads and k.shape[3] == cfg.head_dim, k.shape
            block_tokens = int(k.shape[2])
            assert block_table.is_cuda and block_table.dtype == torch.int32 and block_table.is_contiguous()
            assert tuple(block_table.shape) == (cfg.batch, cfg.max_ctx // block_tokens), block_table.shape
        assert seq_lens.dtype == torch.int32 and seq_lens.numel() == cfg.batch
        self.kbits = torch.zeros(packed_bits_bytes(cfg) // 4, dtype=torch.int32, device=k.device)
        self.kmeta = torch.zeros(packed_meta_bytes(cfg) // 4, dtype=torch.int32, device=k.device)
        self.kabsmax = torch.zeros(cfg.units * cfg.head_dim, dtype=torch.float32, device=k.device)
        self.c = Cache(k.data_ptr(), v.data_ptr(), self.kbits.data_ptr(), self.kmeta.data_ptr(),
                       self.kabsmax.data_ptr(), seq_lens.data_ptr(),
                       block_table.data_ptr() if block_table is not None else None, block_tokens)

    def unpack(self):
        """Logical view of the packed state on the host: bits [units][max_ctx][D] u8, s, z [units][groups][D] u16."""
        cfg = self.cfg
        kb = self.kbits.cpu().numpy().view(np.uint32)
        km = self.kmeta.cpu().numpy().view(np.uint32)
        bits = np.zeros((cfg.units, cfg.max_ctx, cfg.head_dim), np.uint8)
        s = np.zeros((cfg.units, cfg.max_ctx // cfg.group_size, cfg.head_dim), np.uint16)
        z = np.zeros_like(s)
        L = lib()
        L.fier_unpack_bits(C.byref(cfg), kb.ctypes.data_as(C.c_void_p), bits.ctypes.data_as(C.c_void_p))
        L.fier_unpack_meta(C.byref(cfg), km.ctypes.data_as(C.c_void_p), s.ctypes.data_as(C.c_void_p),
                           z.ctypes.data_as(C.c_void_p))
        return bits, s, z


def quantize_keys(cfg: Config, cache: DeviceCache):
    _check(lib().fier_quantize_keys(C.byref(cfg), C.byref(cache.c), _stream()), "fier_quantize_keys")


def append_key(cfg: Config, cache: DeviceCache, k_new, v_new):
    _check(lib().fier_append_key(C.byref(cfg), C.byref(cache.c), _ptr(k_new), _ptr(v_new), _stream()),
           "fier_append_key")


def score(cfg: Config, cache: DeviceCache, q, extra_tokens: int, scores):
    _check(lib().fier_score(C.byref(cfg), C.byref(cache.c), _ptr(q), int(extra_tokens), _ptr(scores), _stream()),
           "fier_score")


def topk(cfg: Config, scores, seq_lens, extra_tokens: int, budgets, max_budget: int, idx, count):
    _check(lib().fier_topk(C.byref(cfg), _ptr(scores), _ptr(seq_lens), int(extra_tokens), _ptr(budgets),
                           int(max_budget), _ptr(idx), _ptr(count), _stream()), "fier_topk")


def topk_ws(cfg: Config, scores, seq_lens, extra_tokens: int, budgets, max_budget: int, idx, count, workspace):
    _check(lib().fier_topk_ws(C.byref(cfg), _ptr(scores), _ptr(seq_lens), int(extra_tokens), _ptr(budgets),
                              int(max_budget), _ptr(idx), _ptr(count), *_ws(workspace), _stream()), "fier_topk_ws")


def sparse_attn(cfg: Config, cache: DeviceCache, q, idx, count, max_budget: int, out, workspace):
    _check(lib().fier_sparse_attn(C.byref(cfg), C.byref(cache.c), _ptr(q), _ptr(idx), _ptr(count), int(max_budget),
                                  _ptr(out), *_ws(workspace), _stream()),
           "fier_sparse_attn")


def dense_attn(cfg: Config, cache: DeviceCache, q, extra_tokens: int, out, workspace):
    _check(lib().fier_dense_attn(C.byref(cfg), C.byref(cache.c), _ptr(q), int(extra_tokens), _ptr(out),
                                 *_ws(workspace), _stream()), "fier_dense_attn")


def decode_step(cfg: Config, caches, q, k_new, v_new, budgets, max_budget: int, out, idx_out, count_out, workspace):
    """caches: list of DeviceCache (one per layer); q/k_new/v_new/out carry a leading layer dimension."""
    arr = (Cache * len(caches))(*[c.c for c in caches])
    _check(lib().fier_decode_step(C.byref(cfg), arr, len(caches), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(budgets),
                                  int(max_budget), _ptr(out), _ptr(idx_out), _ptr(count_out),
                                  *_ws(workspace), _stream()), "fier_decode_step")


def decode_step_static(cfg: Config, caches, q, k_new, v_new, budgets, max_budget: int, out, idx_out, count_out):
    """fier_decode_step on the library's own scratch array: no workspace argument, nothing is allocated."""
    arr = (Cache * len(caches))(*[c.c for c in caches])
    _check(lib().fier_decode_step_static(C.byref(cfg), arr, len(caches), _ptr(q), _ptr(k_new), _ptr(v_new),
                                         _ptr(budgets), int(max_budget), _ptr(out), _ptr(idx_out), _ptr(count_out),
                                         _stream()), "fier_decode_step_static")


def page_meta_bytes(cfg: Config, page_tokens: int) -> int:
    return int(lib().fier_page_meta_bytes(C.byref(cfg), int(page_tokens)))


def page_minmax(cfg: Config, cache: DeviceCache, page_tokens: int, page_meta):
    _check(lib().fier_page_minmax(C.byref(cfg), C.byref(cache.c), int(page_tokens), _ptr(page_meta), _stream()),
           "fier_page_minmax")


def page_append(cfg: Config, seq_lens, page_tokens: int, k_new, page_meta):
    _check(lib().fier_page_append(C.byref(cfg), _ptr(seq_lens), int(page_tokens), _ptr(k_new), _ptr(page_meta),
                                  _stream()), "fier_page_append")


def page_score(cfg: Config, page_meta, page_tokens: int, seq_lens, extra_tokens: int, q, mode: int, page_scores):
    _check(lib().fier_page_score(C.byref(cfg), _ptr(page_meta), int(page_tokens), _ptr(seq_lens), int(extra_tokens),
                                 _ptr(q), int(mode), _ptr(page_scores), _stream()), "fier_page_score")


def page_mean_score(cfg: Config, scores, seq_lens, extra_tokens: int, page_tokens: int, page_scores):
    _check(lib().fier_page_mean_score(C.byref(cfg), _ptr(scores), _ptr(seq_lens), int(extra_tokens), int(page_tokens),
                                      _ptr(page_scores), _stream()), "fier_page_mean_score")


def expand_pages(cfg: Config, page_idx, page_count, max_pages: int, seq_lens, extra_tokens: int, page_tokens: int,
                 idx, count, max_budget: int):
    _check(lib().fier_expand_pages(C.byref(cfg), _ptr(page_idx), _ptr(page_count), int(max_pages), _ptr(seq_lens),
                                   int(extra_tokens), int(page_tokens), _ptr(idx), _ptr(count), int(max_budget),
                                   _stream()), "fier_expand_pages")


def decode_step_mixed(cfg: Config, caches, dense_layers, q, k_new, v_new, budgets, max_budget: int, out, idx_out,
                      count_out, workspace):
    """fier_decode_step with full attention on the layers flagged in dense_layers (a sequence of bools)."""
    arr = (Cache * len(caches))(*[c.c for c in caches])
    flags = (C.c_uint8 * len(caches))(*[1 if d else 0 for d in dense_layers])
    _check(lib().fier_decode_step_mixed(C.byref(cfg), arr, len(caches), flags, _ptr(q), _ptr(k_new), _ptr(v_new),
                                        _ptr(budgets), int(max_budget), _ptr(out), _ptr(idx_out), _ptr(count_out),
                                        *_ws(workspace), _stream()), "fier_decode_step_mixed")


def decode_step_phase(cfg: Config, caches, q, k_new, v_new, budgets, max_budget: int, out, idx_out, count_out,
                      workspace, phase: int):
    """One kernel of the fused step alone (see fier_decode_step_phase in fier.h); for measurement and tests."""
    arr = (Cache * len(caches))(*[c.c for c in caches])
    _check(lib().fier_decode_step_phase(C.byref(cfg), arr, len(caches), _ptr(q), _ptr(k_new), _ptr(v_new),
                                        _ptr(budgets), int(max_budget), _ptr(out), _ptr(idx_out), _ptr(count_out),
                                        *_ws(workspace), int(phase), _stream()), "fier_decode_step_phase")
