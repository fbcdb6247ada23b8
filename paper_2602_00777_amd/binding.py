"""Thin ctypes binding over ``libhylra.so`` (declared in ``include/hylra.h``).

Argument marshalling only: PyTorch supplies device memory and the current HIP
stream; every step of the path runs in the library's kernels.  There is no
fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhylra.so")

FULL, REUSE = 0, 1
FLAG_DETERMINISTIC, FLAG_TOPK_EVERY_FULL_LAYER = 1, 2
PROFILE_CLASSES = ("full_attn", "full_finalize", "reuse_attn", "reuse_combine", "probe")

EXPORTS = (
    "hylra_create", "hylra_create_ex", "hylra_destroy", "hylra_reset", "hylra_status_str", "hylra_last_error",
    "hylra_full_attn_topk", "hylra_reuse_sparse_attn", "hylra_decode_step",
    "hylra_reuse_sparse_attn_static",
    "hylra_full_attn_topk_blocks", "hylra_reuse_block_attn", "hylra_decode_step_blocks",
    "hylra_full_attn_topk_paged", "hylra_reuse_sparse_attn_paged", "hylra_decode_step_paged",
    "hylra_full_attn_topk_blocks_paged", "hylra_reuse_block_attn_paged", "hylra_decode_step_blocks_paged",
    "hylra_overlap_counts", "hylra_similarity_matrix", "hylra_policy_search",
    "hylra_offload_slot_bytes", "hylra_gather_rows", "hylra_decode_step_offloaded",
    "hylra_gather_blocks", "hylra_decode_step_offloaded_blocks",
    "hylra_append_full_attn_topk", "hylra_append_reuse_sparse_attn", "hylra_decode_step_append",
    "hylra_set_option", "hylra_get_info", "hylra_profile_enable", "hylra_profile_reset", "hylra_profile_read",
    "hylra_probe_copy", "hylra_probe_read", "hylra_probe_gather",
)


class HylraError(RuntimeError):
    def __init__(self, status: int, what: str, detail: str):
        super().__init__("%s: status %d (%s)" % (what, status, detail))
        self.status = status


class Shape(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("ctx_len", ctypes.c_int32),
        ("kv_stride_b", ctypes.c_int64), ("kv_stride_h", ctypes.c_int64),
        ("kv_stride_n", ctypes.c_int64), ("scale", ctypes.c_float),
    ]


class Paged(ctypes.Structure):
    _fields_ = [
        ("page_size", ctypes.c_int32), ("max_pages", ctypes.c_int32),
        ("stride_page", ctypes.c_int64), ("stride_head", ctypes.c_int64), ("stride_row", ctypes.c_int64),
        ("block_table", ctypes.c_void_p), ("seq_lens", ctypes.c_void_p),
    ]


_lib = None


def load_library() -> ctypes.CDLL:
    """Loads the built library; raises if it has not been built (no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            "%s is missing: build it with `python -m paper_2602_00777_amd.build`" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32 = ctypes.c_void_p, ctypes.c_int32
    sp = ctypes.POINTER(Shape)
    lib.hylra_create.argtypes = [ctypes.POINTER(vp), sp, i32, ctypes.c_int]
    lib.hylra_create_ex.argtypes = [ctypes.POINTER(vp), sp, i32, ctypes.c_int, ctypes.c_uint32]
    lib.hylra_destroy.argtypes = [vp]
    lib.hylra_reset.argtypes = [vp]
    lib.hylra_status_str.argtypes = [ctypes.c_int]
    lib.hylra_status_str.restype = ctypes.c_char_p
    lib.hylra_last_error.argtypes = [vp]
    lib.hylra_last_error.restype = ctypes.c_char_p
    lib.hylra_full_attn_topk.argtypes = [vp, sp, vp, vp, vp, i32, vp, vp, vp]
    lib.hylra_reuse_sparse_attn.argtypes = [vp, sp, vp, vp, vp, vp, i32, vp, vp]
    lib.hylra_decode_step.argtypes = [vp, sp, i32, vp, vp, vp, vp, i32, vp, vp, vp]
    lib.hylra_reuse_sparse_attn_static.argtypes = [sp, vp, vp, vp, vp, i32, vp, vp]
    lib.hylra_full_attn_topk_blocks.argtypes = [vp, sp, vp, vp, vp, i32, i32, vp, vp, vp]
    lib.hylra_reuse_block_attn.argtypes = [vp, sp, vp, vp, vp, vp, i32, i32, vp, vp]
    lib.hylra_decode_step_blocks.argtypes = [vp, sp, i32, vp, vp, vp, vp, i32, i32, vp, vp, vp]
    pp = ctypes.POINTER(Paged)
    lib.hylra_full_attn_topk_paged.argtypes = [vp, sp, pp, vp, vp, vp, i32, vp, vp, vp]
    lib.hylra_reuse_sparse_attn_paged.argtypes = [vp, sp, pp, vp, vp, vp, vp, i32, vp, vp]
    lib.hylra_decode_step_paged.argtypes = [vp, sp, pp, i32, vp, vp, vp, vp, i32, vp, vp, vp]
    lib.hylra_full_attn_topk_blocks_paged.argtypes = [vp, sp, pp, vp, vp, vp, i32, i32, vp, vp, vp]
    lib.hylra_reuse_block_attn_paged.argtypes = [vp, sp, pp, vp, vp, vp, vp, i32, i32, vp, vp]
    lib.hylra_decode_step_blocks_paged.argtypes = [vp, sp, pp, i32, vp, vp, vp, vp, i32, i32, vp, vp, vp]
    lib.hylra_offload_slot_bytes.argtypes = [sp, i32]
    lib.hylra_gather_rows.argtypes = [vp, sp, vp, vp, vp, i32, vp, vp, vp, vp]
    lib.hylra_decode_step_offloaded.argtypes = [vp, sp, i32, vp, vp, vp, vp, i32, vp, vp, vp, ctypes.c_size_t, vp, vp]
    lib.hylra_gather_blocks.argtypes = [vp, sp, pp, vp, vp, vp, i32, i32, vp, vp, vp, vp]
    lib.hylra_decode_step_offloaded_blocks.argtypes = [vp, sp, pp, i32, vp, vp, vp, vp, i32, i32, vp, vp, vp,
                                                       ctypes.c_size_t, vp, vp]
    lib.hylra_append_full_attn_topk.argtypes = [vp, sp, pp, vp, vp, vp, vp, vp, i32, vp, vp, vp]
    lib.hylra_append_reuse_sparse_attn.argtypes = [vp, sp, pp, vp, vp, vp, vp, vp, vp, i32, vp, vp]
    lib.hylra_decode_step_append.argtypes = [vp, sp, pp, i32, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp]
    lib.hylra_overlap_counts.argtypes = [vp, i32, vp, i32, i32, i32, i32, vp, vp]
    lib.hylra_similarity_matrix.argtypes = [i32, vp, vp]
    lib.hylra_policy_search.argtypes = [vp, i32, vp, ctypes.c_double, vp, ctypes.POINTER(i32),
                                        ctypes.POINTER(ctypes.c_double)]
    lib.hylra_set_option.argtypes = [vp, ctypes.c_char_p, i32]
    lib.hylra_get_info.argtypes = [vp, ctypes.c_char_p, ctypes.POINTER(i32)]
    lib.hylra_profile_enable.argtypes = [vp, i32]
    lib.hylra_profile_reset.argtypes = [vp]
    lib.hylra_profile_read.argtypes = [vp, i32, ctypes.POINTER(i32), ctypes.POINTER(ctypes.c_double)]
    lib.hylra_probe_copy.argtypes = [vp, vp, vp, ctypes.c_size_t, vp]
    lib.hylra_probe_read.argtypes = [vp, vp, ctypes.c_size_t, vp, vp]
    lib.hylra_probe_gather.argtypes = [vp, sp, vp, vp, vp, i32, vp, vp]
    for name in EXPORTS:
        if name not in ("hylra_status_str", "hylra_last_error", "hylra_offload_slot_bytes"):
            getattr(lib, name).restype = ctypes.c_int
    lib.hylra_offload_slot_bytes.restype = ctypes.c_size_t
    _lib = lib
    return lib


def _stream_ptr(device) -> int:
    return torch.cuda.current_stream(device).cuda_stream


def make_shape(q: torch.Tensor, K: torch.Tensor, scale: float = 0.0) -> Shape:
    """Shape descriptor for q [B,Hq,d] and K [B,Hkv,N,d] (strides taken from K)."""
    B, Hq, d = q.shape
    Bk, Hkv, N, dk = K.shape
    if (Bk, dk) != (B, d):
        raise ValueError("q %s and K %s disagree" % (tuple(q.shape), tuple(K.shape)))
    if K.stride(3) != 1:
        raise ValueError("the innermost dimension of K and V must be contiguous")
    return Shape(B, Hq, Hkv, d, N, K.stride(0), K.stride(1), K.stride(2), float(scale))


class PagedCache:
    """Describes a paged KV cache for the ``*_paged`` calls: ``block_table`` int32 [B, max_pages]
    (device), optional ``seq_lens`` int32 [B] (device), ``ctx_len`` = the largest sequence
    length of the call.  Pools are bf16 tensors [pages, Hkv, page_size, d] (any strides with a
    contiguous innermost dimension); K and V pools of a layer share shape and strides."""

    def __init__(self, block_table: Optional[torch.Tensor], page_size: int, ctx_len: int,
                 seq_lens: Optional[torch.Tensor] = None):
        for name, t in (("block_table", block_table), ("seq_lens", seq_lens)):
            if t is not None and (t.dtype != torch.int32 or not t.is_cuda or not t.is_contiguous()):
                raise TypeError("%s must be a contiguous int32 CUDA tensor" % name)
        if block_table is not None and (block_table.dim() != 2 or (seq_lens is not None and tuple(seq_lens.shape) != (block_table.shape[0],))):
            raise ValueError("block_table must be [B, max_pages] and seq_lens [B]")
        if block_table is None and seq_lens is None:
            raise ValueError("a contiguous cache without seq_lens needs no PagedCache")
        self.block_table, self.seq_lens = block_table, seq_lens
        self.page_size, self.ctx_len = int(page_size), int(ctx_len)

    def describe(self, q: torch.Tensor, pool: torch.Tensor, scale: float = 0.0) -> Tuple[Shape, Paged]:
        if self.block_table is None:
            # contiguous cache [B, Hkv, N, d] with per-sequence lengths only
            shp = make_shape(q, pool, scale)
            if shp.ctx_len != self.ctx_len or tuple(self.seq_lens.shape) != (shp.batch,):
                raise ValueError("cache %s disagrees with ctx_len = %d or seq_lens" % (tuple(pool.shape), self.ctx_len))
            return shp, Paged(0, 0, 0, 0, 0, None, self.seq_lens.data_ptr())
        B, Hq, d = q.shape
        P, Hkv, ps, dk = pool.shape
        if dk != d or ps != self.page_size or self.block_table.shape[0] != B:
            raise ValueError("q %s, pool %s and the block table disagree" % (tuple(q.shape), tuple(pool.shape)))
        if pool.stride(3) != 1:
            raise ValueError("the innermost dimension of the pools must be contiguous")
        shp = Shape(B, Hq, Hkv, d, self.ctx_len, 0, 0, 0, float(scale))
        pg = Paged(self.page_size, self.block_table.shape[1], pool.stride(0), pool.stride(1), pool.stride(2),
                   self.block_table.data_ptr(), self.seq_lens.data_ptr() if self.seq_lens is not None else None)
        return shp, pg


def similarity_matrix(counts) -> "numpy.ndarray":
    """hylra_similarity_matrix on a host int64 [L, L] array of overlap counts."""
    import numpy as np

    counts = np.ascontiguousarray(np.asarray(counts, dtype=np.int64))
    L = counts.shape[0]
    M = np.empty((L, L), np.float64)
    rc = load_library().hylra_similarity_matrix(L, counts.ctypes.data, M.ctypes.data)
    if rc != 0:
        raise HylraError(rc, "hylra_similarity_matrix", "bad argument")
    return M


def policy_search(M, theta: float):
    """hylra_policy_search (host only): returns (policy uint8 [L], n_full, sum_sim)."""
    import numpy as np

    M = np.ascontiguousarray(np.asarray(M, dtype=np.float64))
    L = M.shape[0]
    if M.shape != (L, L):
        raise ValueError("M must be square")
    policy = np.empty(L, np.uint8)
    n_full, s = ctypes.c_int32(), ctypes.c_double()
    rc = load_library().hylra_policy_search(None, L, M.ctypes.data, float(theta), policy.ctypes.data,
                                            ctypes.byref(n_full), ctypes.byref(s))
    if rc != 0:
        raise HylraError(rc, "hylra_policy_search", "bad argument")
    return policy, n_full.value, s.value


def reuse_sparse_attn_static(q, K, V, idx, out, scale: float = 0.0):
    """hylra_reuse_sparse_attn_static: the Reuse layer without a context and without any
    allocation (the caller passes ``out``); runs on the current device."""
    Context._check_inputs(q, K, V)
    if idx.dtype != torch.int32 or not idx.is_cuda or not idx.is_contiguous():
        raise TypeError("idx must be a contiguous int32 CUDA tensor")
    if out.dtype != torch.float32 or not out.is_cuda or not out.is_contiguous() or out.shape != q.shape:
        raise TypeError("out must be a contiguous float32 CUDA tensor shaped like q")
    shp = make_shape(q, K, scale)
    if tuple(idx.shape[:2]) != (shp.batch, shp.n_kv_heads):
        raise ValueError("idx must be [B, Hkv, k]")
    lib = load_library()
    with torch.cuda.device(q.device):
        rc = lib.hylra_reuse_sparse_attn_static(ctypes.byref(shp), q.data_ptr(), K.data_ptr(), V.data_ptr(),
                                                idx.data_ptr(), idx.shape[2], out.data_ptr(), _stream_ptr(q.device))
    if rc != 0:
        raise HylraError(rc, "hylra_reuse_sparse_attn_static", lib.hylra_last_error(None).decode())
    return out


class Context:
    """Owns one ``hylra_ctx`` (a fixed device workspace) on one GPU."""

    def __init__(self, batch: int, n_q_heads: int, n_kv_heads: int, head_dim: int, ctx_len: int,
                 max_k: int, device: int = 0, deterministic: bool = False, topk_every_full_layer: bool = False):
        self._lib = load_library()
        self._h = ctypes.c_void_p()
        self.device = torch.device("cuda", device)
        shp = Shape(batch, n_q_heads, n_kv_heads, head_dim, ctx_len, 0, 0, 0, 0.0)
        flags = (FLAG_DETERMINISTIC if deterministic else 0) | (FLAG_TOPK_EVERY_FULL_LAYER if topk_every_full_layer else 0)
        rc = self._lib.hylra_create_ex(ctypes.byref(self._h), ctypes.byref(shp), max_k, device, flags)
        if rc != 0:
            raise HylraError(rc, "hylra_create_ex", self._lib.hylra_last_error(None).decode())

    def close(self):
        if getattr(self, "_h", None) and self._h.value:
            torch.cuda.synchronize(self.device)
            self._lib.hylra_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def _check(self, rc: int, what: str):
        if rc != 0:
            raise HylraError(rc, what, self._lib.hylra_last_error(self._h).decode())

    @staticmethod
    def _check_inputs(q, K, V):
        for name, t in (("q", q), ("K", K), ("V", V)):
            if t.dtype != torch.bfloat16 or not t.is_cuda:
                raise TypeError("%s must be a bfloat16 CUDA tensor" % name)
        if not q.is_contiguous():
            raise ValueError("q must be contiguous")
        if V.shape != K.shape or V.stride() != K.stride():
            raise ValueError("K and V must share shape and strides")

    # -- the three calls of the hot path -------------------------------------------------
    def full_attn_topk(self, q, K, V, k: int, out=None, idx=None, scale: float = 0.0):
        """hylra_full_attn_topk: returns (out fp32 [B,Hq,d], idx int32 [B,Hkv,k])."""
        self._check_inputs(q, K, V)
        shp = make_shape(q, K, scale)
        if out is None:
            out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
        if idx is None:
            idx = torch.empty((shp.batch, shp.n_kv_heads, k), dtype=torch.int32, device=q.device)
        rc = self._lib.hylra_full_attn_topk(self._h, ctypes.byref(shp), q.data_ptr(), K.data_ptr(),
                                            V.data_ptr(), k, out.data_ptr(), idx.data_ptr(),
                                            _stream_ptr(q.device))
        self._check(rc, "hylra_full_attn_topk")
        return out, idx

    def reuse_sparse_attn(self, q, K, V, idx, out=None, scale: float = 0.0):
        """hylra_reuse_sparse_attn: returns out fp32 [B,Hq,d]."""
        self._check_inputs(q, K, V)
        if idx.dtype != torch.int32 or not idx.is_cuda or not idx.is_contiguous():
            raise TypeError("idx must be a contiguous int32 CUDA tensor")
        shp = make_shape(q, K, scale)
        if tuple(idx.shape[:2]) != (shp.batch, shp.n_kv_heads):
            raise ValueError("idx must be [B, Hkv, k]")
        if out is None:
            out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
        rc = self._lib.hylra_reuse_sparse_attn(self._h, ctypes.byref(shp), q.data_ptr(),
                                               K.data_ptr(), V.data_ptr(), idx.data_ptr(),
                                               idx.shape[2], out.data_ptr(), _stream_ptr(q.device))
        self._check(rc, "hylra_reuse_sparse_attn")
        return out

    # -- paged cache, per-sequence lengths -------------------------------------------------
    def full_attn_topk_paged(self, q, K_pool, V_pool, cache: PagedCache, k: int, out=None, idx=None,
                             scale: float = 0.0):
        """hylra_full_attn_topk_paged: returns (out fp32 [B,Hq,d], idx int32 [B,Hkv,k])."""
        self._check_inputs(q, K_pool, V_pool)
        shp, pg = cache.describe(q, K_pool, scale)
        if out is None:
            out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
        if idx is None:
            idx = torch.empty((shp.batch, shp.n_kv_heads, k), dtype=torch.int32, device=q.device)
        rc = self._lib.hylra_full_attn_topk_paged(self._h, ctypes.byref(shp), ctypes.byref(pg), q.data_ptr(),
                                                  K_pool.data_ptr(), V_pool.data_ptr(), k, out.data_ptr(),
                                                  idx.data_ptr(), _stream_ptr(q.device))
        self._check(rc, "hylra_full_attn_topk_paged")
        return out, idx

    def reuse_sparse_attn_paged(self, q, K_pool, V_pool, cache: PagedCache, idx, out=None, scale: float = 0.0):
        """hylra_reuse_sparse_attn_paged: returns out fp32 [B,Hq,d]."""
        self._check_inputs(q, K_pool, V_pool)
        if idx.dtype != torch.int32 or not idx.is_cuda or not idx.is_contiguous():
            raise TypeError("idx must be a contiguous int32 CUDA tensor")
        shp, pg = cache.describe(q, K_pool, scale)
        if tuple(idx.shape[:2]) != (shp.batch, shp.n_kv_heads):
            raise ValueError("idx must be [B, Hkv, k]")
        if out is None:
            out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
        rc = self._lib.hylra_reuse_sparse_attn_paged(self._h, ctypes.byref(shp), ctypes.byref(pg), q.data_ptr(),
                                                     K_pool.data_ptr(), V_pool.data_ptr(), idx.data_ptr(),
                                                     idx.shape[2], out.data_ptr(), _stream_ptr(q.device))
        self._check(rc, "hylra_reuse_sparse_attn_paged")
        return out

    def full_attn_topk_blocks_paged(self, q, K_pool, V_pool, cache: PagedCache, block: int, kb: int,
                                    out=None, bidx=None, scale: float = 0.0):
        """hylra_full_attn_topk_blocks_paged: returns (out fp32 [B,Hq,d], bidx int32 [B,Hkv,kb])."""
        self._check_inputs(q, K_pool, V_pool)
        shp, pg = cache.describe(q, K_pool, scale)
        if out is None:
            out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
        if bidx is None:
            bidx = torch.empty((shp.batch, shp.n_kv_heads, kb), dtype=torch.int32, device=q.device)
        rc = self._lib.hylra_full_attn_topk_blocks_paged(self._h, ctypes.byref(shp), ctypes.byref(pg),
                                                         q.data_ptr(), K_pool.data_ptr(), V_pool.data_ptr(),
                                                         block, kb, out.data_ptr(), bidx.data_ptr(),
                                                         _stream_ptr(q.device))
        self._check(rc, "hylra_full_attn_topk_blocks_paged")
        return out, bidx

    def reuse_block_attn_paged(self, q, K_pool, V_pool, cache: PagedCache, bidx, block: int, out=None,
                               scale: float = 0.0):
        """hylra_reuse_block_attn_paged: returns out fp32 [B,Hq,d]."""
        self._check_inputs(q, K_pool, V_pool)
        if bidx.dtype != torch.int32 or not bidx.is_cuda or not bidx.is_contiguous():
            raise TypeError("bidx must be a contiguous int32 CUDA tensor")
        shp, pg = cache.describe(q, K_pool, scale)
        if tuple(bidx.shape[:2]) != (shp.batch, shp.n_kv_heads):
            raise ValueError("bidx must be [B, Hkv, kb]")
        if out is None:
            out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
        rc = self._lib.hylra_reuse_block_attn_paged(self._h, ctypes.byref(shp), ctypes.byref(pg), q.data_ptr(),
                                                    K_pool.data_ptr(), V_pool.data_ptr(), bidx.data_ptr(),
                                                    block, bidx.shape[2], out.data_ptr(), _stream_ptr(q.device))
        self._check(rc, "hylra_reuse_block_attn_paged")
        return out

    # -- index-guided prefetch (offloaded caches) -------------------------------------------
    def gather_rows(self, K_src, V_src, idx, device=None):
        """hylra_gather_rows: K_src / V_src bf16 [B,Hkv,N,d] in device or pinned host memory;
        returns (K_dst, V_dst bf16 [B,Hkv,k,d], idx_dst int32 [B,Hkv,k]) on the GPU."""
        dev = idx.device if device is None else device
        B, Hkv, N, d = K_src.shape
        if K_src.dtype != torch.bfloat16 or V_src.shape != K_src.shape or V_src.stride() != K_src.stride():
            raise TypeError("K_src and V_src must be bfloat16 tensors of one shape and stride set")
        if not (K_src.is_cuda or K_src.is_pinned()) or not (V_src.is_cuda or V_src.is_pinned()):
            raise TypeError("the source caches must be in device or pinned host memory")
        k = idx.shape[2]
        shp = Shape(B, Hkv, Hkv, d, N, K_src.stride(0), K_src.stride(1), K_src.stride(2), 0.0)
        Kd = torch.empty((B, Hkv, k, d), dtype=torch.bfloat16, device=dev)
        Vd = torch.empty_like(Kd)
        idd = torch.empty((B, Hkv, k), dtype=torch.int32, device=dev)
        rc = self._lib.hylra_gather_rows(self._h, ctypes.byref(shp), K_src.data_ptr(), V_src.data_ptr(),
                                         idx.data_ptr(), k, Kd.data_ptr(), Vd.data_ptr(), idd.data_ptr(),
                                         _stream_ptr(dev))
        self._check(rc, "hylra_gather_rows")
        return Kd, Vd, idd

    def gather_blocks(self, K_src, V_src, bidx, block: int, paged: Optional[PagedCache] = None, n_q_heads=None):
        """hylra_gather_blocks: K_src / V_src a contiguous cache [B,Hkv,N,d] or (with a paged
        ``paged``) pools, in device or pinned host memory; returns (K_dst, V_dst bf16
        [B,Hkv,kb*block,d], idx_dst int32 [B,Hkv,kb*block]) on the GPU."""
        dev = bidx.device
        if not (K_src.is_cuda or K_src.is_pinned()) or not (V_src.is_cuda or V_src.is_pinned()):
            raise TypeError("the source caches must be in device or pinned host memory")
        B, Hkv, kb = bidx.shape
        d = K_src.shape[3]
        qlike = torch.empty((B, Hkv, d), dtype=torch.bfloat16, device="meta")
        if paged is not None:
            shp, pg = paged.describe(qlike, K_src)
            pgp = ctypes.byref(pg)
        else:
            shp, pgp = make_shape(qlike, K_src), None
        rows = kb * block
        Kd = torch.empty((B, Hkv, rows, d), dtype=torch.bfloat16, device=dev)
        Vd = torch.empty_like(Kd)
        idd = torch.empty((B, Hkv, rows), dtype=torch.int32, device=dev)
        rc = self._lib.hylra_gather_blocks(self._h, ctypes.byref(shp), pgp, K_src.data_ptr(), V_src.data_ptr(),
                                           bidx.data_ptr(), block, kb, Kd.data_ptr(), Vd.data_ptr(), idd.data_ptr(),
                                           _stream_ptr(dev))
        self._check(rc, "hylra_gather_blocks")
        return Kd, Vd, idd

    # -- append the current token, then attend -------------------------------------------------
    def append_full_attn_topk(self, q, k_new, v_new, K, V, k: int, paged: Optional[PagedCache] = None,
                              out=None, idx=None, scale: float = 0.0):
        """hylra_append_full_attn_topk: K / V (pools if paged) receive the new rows; returns (out, idx)."""
        self._check_inputs(q, K, V)
        shp, pgp, keep = self._describe(q, K, paged, scale)
        if out is None:
            out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
        if idx is None:
            idx = torch.empty((shp.batch, shp.n_kv_heads, k), dtype=torch.int32, device=q.device)
        rc = self._lib.hylra_append_full_attn_topk(self._h, ctypes.byref(shp), pgp, q.data_ptr(), k_new.data_ptr(),
                                                   v_new.data_ptr(), K.data_ptr(), V.data_ptr(), k, out.data_ptr(),
                                                   idx.data_ptr(), _stream_ptr(q.device))
        self._check(rc, "hylra_append_full_attn_topk")
        return out, idx

    def append_reuse_sparse_attn(self, q, k_new, v_new, K, V, idx, paged: Optional[PagedCache] = None,
                                 out=None, scale: float = 0.0):
        """hylra_append_reuse_sparse_attn: returns out."""
        self._check_inputs(q, K, V)
        shp, pgp, keep = self._describe(q, K, paged, scale)
        if out is None:
            out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
        rc = self._lib.hylra_append_reuse_sparse_attn(self._h, ctypes.byref(shp), pgp, q.data_ptr(), k_new.data_ptr(),
                                                      v_new.data_ptr(), K.data_ptr(), V.data_ptr(), idx.data_ptr(),
                                                      idx.shape[2], out.data_ptr(), _stream_ptr(q.device))
        self._check(rc, "hylra_append_reuse_sparse_attn")
        return out

    @staticmethod
    def _describe(q, K, paged, scale):
        if paged is None:
            return make_shape(q, K, scale), None, None
        shp, pg = paged.describe(q, K, scale)
        return shp, ctypes.byref(pg), pg

    def decode_step_append(self, policy: Sequence[int], q_l, k_new_l, v_new_l, K_l, V_l, k: int,
                           paged: Optional[PagedCache] = None, scale: float = 0.0):
        """hylra_decode_step_append: returns (outs, idx_buf)."""
        run, outs, idx_buf = self.prepare_step_append(policy, q_l, k_new_l, v_new_l, K_l, V_l, k, paged, scale)
        run()
        return outs, idx_buf

    def prepare_step_append(self, policy: Sequence[int], q_l, k_new_l, v_new_l, K_l, V_l, k: int,
                            paged: Optional[PagedCache] = None, scale: float = 0.0):
        """Marshals hylra_decode_step_append once; returns (run, outs, idx_buf)."""
        L = len(policy)
        dev = q_l[0].device
        for l in range(L):
            self._check_inputs(q_l[l], K_l[l], V_l[l])
        shp, pgp, keep = self._describe(q_l[0], K_l[0], paged, scale)
        outs = [torch.empty(q_l[l].shape, dtype=torch.float32, device=dev) for l in range(L)]
        idx_buf = torch.empty((shp.batch, shp.n_kv_heads, k), dtype=torch.int32, device=dev)
        arr = ctypes.c_void_p * L
        pol = (ctypes.c_uint8 * L)(*[int(p) for p in policy])
        ptrs = [arr(*[t.data_ptr() for t in ts]) for ts in (q_l, k_new_l, v_new_l, K_l, V_l, outs)]
        held = (q_l, k_new_l, v_new_l, K_l, V_l, paged, keep)

        def run():
            rc = self._lib.hylra_decode_step_append(self._h, ctypes.byref(shp), pgp, L, pol, ptrs[0], ptrs[1], ptrs[2],
                                                    ptrs[3], ptrs[4], k, ptrs[5], idx_buf.data_ptr(), _stream_ptr(dev))
            self._check(rc, "hylra_decode_step_append")
            return held is not None

        return run, outs, idx_buf

    def prepare_step_offloaded(self, policy: Sequence[int], q_l, K_l, V_l, k: int, n_slots: int = 2,
                               copy_stream: Optional[torch.cuda.Stream] = None, scale: float = 0.0,
                               block: int = 0, paged: Optional[PagedCache] = None):
        """hylra_decode_step_offloaded (hylra_decode_step_offloaded_blocks with block > 0 or a
        paged cache; k then counts blocks): K_l[l] / V_l[l] of Reuse layers may be pinned host
        tensors.  Returns (run, outs, idx_buf, copy_stream); run() enqueues one step on the
        current stream (attention) and the copy stream (gathers)."""
        L = len(policy)
        dev = q_l[0].device
        general = block > 0 or paged is not None
        blk = block if block > 0 else 1
        shp, pgp, keep_pg = self._describe(q_l[0], K_l[0], paged, scale)
        for l in range(L):
            o, _, og = self._describe(q_l[l], K_l[l], paged, scale)
            if bytes(o) != bytes(shp) or V_l[l].stride() != K_l[l].stride() or (og is not None and bytes(og) != bytes(keep_pg)):
                raise ValueError("all layers must share one shape and stride set")
            if policy[l] == FULL and not K_l[l].is_cuda:
                raise TypeError("the caches of Full layers must be in device memory")
            if not (K_l[l].is_cuda or K_l[l].is_pinned()):
                raise TypeError("offloaded caches must be in pinned host memory")
        outs = [torch.empty(q_l[l].shape, dtype=torch.float32, device=dev) for l in range(L)]
        idx_buf = torch.empty((shp.batch, shp.n_kv_heads, k), dtype=torch.int32, device=dev)
        slot = self._lib.hylra_offload_slot_bytes(ctypes.byref(shp), k * blk)
        staging = torch.empty(slot * n_slots + 256, dtype=torch.uint8, device=dev)
        base = (staging.data_ptr() + 255) // 256 * 256
        if copy_stream is None:
            copy_stream = torch.cuda.Stream(device=dev)
        arr = ctypes.c_void_p * L
        pol = (ctypes.c_uint8 * L)(*[int(p) for p in policy])
        qa, Ka, Va = (arr(*[t.data_ptr() for t in ts]) for ts in (q_l, K_l, V_l))
        oa = arr(*[t.data_ptr() for t in outs])
        keep = (q_l, K_l, V_l, staging, paged, keep_pg)

        def run():
            if general:
                rc = self._lib.hylra_decode_step_offloaded_blocks(self._h, ctypes.byref(shp), pgp, L, pol, qa, Ka, Va,
                                                                  blk, k, oa, idx_buf.data_ptr(), base, slot * n_slots,
                                                                  _stream_ptr(dev), copy_stream.cuda_stream)
                self._check(rc, "hylra_decode_step_offloaded_blocks")
            else:
                rc = self._lib.hylra_decode_step_offloaded(self._h, ctypes.byref(shp), L, pol, qa, Ka, Va, k, oa,
                                                           idx_buf.data_ptr(), base, slot * n_slots,
                                                           _stream_ptr(dev), copy_stream.cuda_stream)
                self._check(rc, "hylra_decode_step_offloaded")
            return keep is not None

        return run, outs, idx_buf, copy_stream

    # -- offline profiling ------------------------------------------------------------------
    def overlap_counts(self, idx_l: Sequence[torch.Tensor], ctx_len: int) -> torch.Tensor:
        """hylra_overlap_counts: int64 [L, L] device tensor of pooled |S_i ∩ S_j| (i <= j)."""
        L = len(idx_l)
        B, H, k = idx_l[0].shape
        for t in idx_l:
            if t.dtype != torch.int32 or not t.is_cuda or not t.is_contiguous() or tuple(t.shape) != (B, H, k):
                raise TypeError("every idx must be a contiguous int32 CUDA tensor of one shape [B, Hkv, k]")
        counts = torch.empty((L, L), dtype=torch.int64, device=idx_l[0].device)
        ptrs = (ctypes.c_void_p * L)(*[t.data_ptr() for t in idx_l])
        rc = self._lib.hylra_overlap_counts(self._h, L, ptrs, B, H, k, int(ctx_len), counts.data_ptr(),
                                            _stream_ptr(idx_l[0].device))
        self._check(rc, "hylra_overlap_counts")
        return counts

    # -- block-level variant ---------------------------------------------------------------
    def full_attn_topk_blocks(self, q, K, V, block: int, kb: int, out=None, bidx=None, scale: float = 0.0):
        """hylra_full_attn_topk_blocks: returns (out fp32 [B,Hq,d], bidx int32 [B,Hkv,kb])."""
        self._check_inputs(q, K, V)
        shp = make_shape(q, K, scale)
        if out is None:
            out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
        if bidx is None:
            bidx = torch.empty((shp.batch, shp.n_kv_heads, kb), dtype=torch.int32, device=q.device)
        rc = self._lib.hylra_full_attn_topk_blocks(self._h, ctypes.byref(shp), q.data_ptr(),
                                                   K.data_ptr(), V.data_ptr(), block, kb,
                                                   out.data_ptr(), bidx.data_ptr(),
                                                   _stream_ptr(q.device))
        self._check(rc, "hylra_full_attn_topk_blocks")
        return out, bidx

    def reuse_block_attn(self, q, K, V, bidx, block: int, out=None, scale: float = 0.0):
        """hylra_reuse_block_attn: returns out fp32 [B,Hq,d]."""
        self._check_inputs(q, K, V)
        if bidx.dtype != torch.int32 or not bidx.is_cuda or not bidx.is_contiguous():
            raise TypeError("bidx must be a contiguous int32 CUDA tensor")
        shp = make_shape(q, K, scale)
        if tuple(bidx.shape[:2]) != (shp.batch, shp.n_kv_heads):
            raise ValueError("bidx must be [B, Hkv, kb]")
        if out is None:
            out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
        rc = self._lib.hylra_reuse_block_attn(self._h, ctypes.byref(shp), q.data_ptr(),
                                              K.data_ptr(), V.data_ptr(), bidx.data_ptr(), block,
                                              bidx.shape[2], out.data_ptr(), _stream_ptr(q.device))
        self._check(rc, "hylra_reuse_block_attn")
        return out

    def prepare_step(self, policy: Sequence[int], q_l, K_l, V_l, k: int, scale: float = 0.0,
                     block: int = 0, paged: Optional[PagedCache] = None):
        """Marshals the per-layer pointer arrays of hylra_decode_step once, so that a timed
        loop contains nothing but the C call.  Returns a zero-argument callable plus the
        output tensors (outs, idx_buf).  block > 0 selects hylra_decode_step_blocks, with k
        counting blocks; paged selects hylra_decode_step_paged (hylra_decode_step_blocks_paged
        with block > 0), with K_l / V_l the pools."""
        L = len(policy)
        for l in range(L):
            self._check_inputs(q_l[l], K_l[l], V_l[l])
        pg = None
        if paged is not None:
            shp, pg = paged.describe(q_l[0], K_l[0], scale)
            for l in range(1, L):
                o, og = paged.describe(q_l[l], K_l[l], scale)
                if bytes(o) != bytes(shp) or bytes(og) != bytes(pg):
                    raise ValueError("all layers must share one shape and stride set")
        else:
            shp = make_shape(q_l[0], K_l[0], scale)
        for l in range(1, L if paged is None else 0):
            o = make_shape(q_l[l], K_l[l], scale)
            if bytes(o) != bytes(shp):
                raise ValueError("all layers must share one shape and stride set")
        dev = q_l[0].device
        outs = [torch.empty(q_l[l].shape, dtype=torch.float32, device=dev) for l in range(L)]
        idx_buf = torch.empty((shp.batch, shp.n_kv_heads, k), dtype=torch.int32, device=dev)
        arr = ctypes.c_void_p * L
        pol = (ctypes.c_uint8 * L)(*[int(p) for p in policy])
        qa = arr(*[t.data_ptr() for t in q_l])
        Ka = arr(*[t.data_ptr() for t in K_l])
        Va = arr(*[t.data_ptr() for t in V_l])
        oa = arr(*[t.data_ptr() for t in outs])
        keep = (q_l, K_l, V_l, paged)

        def run():
            if pg is not None and block > 0:
                rc = self._lib.hylra_decode_step_blocks_paged(self._h, ctypes.byref(shp), ctypes.byref(pg), L, pol,
                                                              qa, Ka, Va, block, k, oa, idx_buf.data_ptr(),
                                                              _stream_ptr(dev))
                self._check(rc, "hylra_decode_step_blocks_paged")
            elif pg is not None:
                rc = self._lib.hylra_decode_step_paged(self._h, ctypes.byref(shp), ctypes.byref(pg), L, pol,
                                                       qa, Ka, Va, k, oa, idx_buf.data_ptr(), _stream_ptr(dev))
                self._check(rc, "hylra_decode_step_paged")
            elif block > 0:
                rc = self._lib.hylra_decode_step_blocks(self._h, ctypes.byref(shp), L, pol, qa, Ka, Va,
                                                        block, k, oa, idx_buf.data_ptr(),
                                                        _stream_ptr(dev))
                self._check(rc, "hylra_decode_step_blocks")
            else:
                rc = self._lib.hylra_decode_step(self._h, ctypes.byref(shp), L, pol, qa, Ka, Va, k, oa,
                                                 idx_buf.data_ptr(), _stream_ptr(dev))
                self._check(rc, "hylra_decode_step")
            return keep is not None

        return run, outs, idx_buf

    def decode_step(self, policy: Sequence[int], q_l, K_l, V_l, k: int, scale: float = 0.0,
                    block: int = 0, paged: Optional[PagedCache] = None):
        """hylra_decode_step (or _blocks when block > 0): returns (list of out per layer, idx of
        the last Full layer)."""
        run, outs, idx_buf = self.prepare_step(policy, q_l, K_l, V_l, k, scale, block, paged)
        run()
        return outs, idx_buf

    # -- knobs and measurement aids ----------------------------------------------------------
    def reset(self):
        self._check(self._lib.hylra_reset(self._h), "hylra_reset")

    def set_option(self, name: str, value: int):
        self._check(self._lib.hylra_set_option(self._h, name.encode(), int(value)), "hylra_set_option")

    def get_info(self, name: str) -> int:
        v = ctypes.c_int32()
        self._check(self._lib.hylra_get_info(self._h, name.encode(), ctypes.byref(v)), "hylra_get_info")
        return v.value

    def profile_enable(self, on: bool = True):
        self._check(self._lib.hylra_profile_enable(self._h, 1 if on else 0), "hylra_profile_enable")

    def profile_reset(self):
        self._check(self._lib.hylra_profile_reset(self._h), "hylra_profile_reset")

    def profile_read(self) -> dict:
        res = {}
        for c, name in enumerate(PROFILE_CLASSES):
            n, ms = ctypes.c_int32(), ctypes.c_double()
            self._check(self._lib.hylra_profile_read(self._h, c, ctypes.byref(n), ctypes.byref(ms)),
                        "hylra_profile_read")
            res[name] = (n.value, ms.value)
        return res

    def probe_copy(self, dst: torch.Tensor, src: torch.Tensor):
        nbytes = src.numel() * src.element_size()
        self._check(self._lib.hylra_probe_copy(self._h, dst.data_ptr(), src.data_ptr(), nbytes,
                                               _stream_ptr(src.device)), "hylra_probe_copy")

    def probe_read(self, src: torch.Tensor, sink: torch.Tensor):
        nbytes = src.numel() * src.element_size()
        self._check(self._lib.hylra_probe_read(self._h, src.data_ptr(), nbytes, sink.data_ptr(),
                                               _stream_ptr(src.device)), "hylra_probe_read")

    def probe_gather(self, K: torch.Tensor, V: torch.Tensor, idx: torch.Tensor, sink: torch.Tensor):
        B, Hkv, N, d = K.shape
        shp = Shape(B, Hkv, Hkv, d, N, K.stride(0), K.stride(1), K.stride(2), 0.0)
        self._check(self._lib.hylra_probe_gather(self._h, ctypes.byref(shp), K.data_ptr(), V.data_ptr(),
                                                 idx.data_ptr(), idx.shape[2], sink.data_ptr(),
                                                 _stream_ptr(K.device)), "hylra_probe_gather")
