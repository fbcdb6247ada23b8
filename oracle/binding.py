"""ctypes loader for ``hylra_oracle.c`` (test infrastructure only).

Inputs are numpy arrays, either float64 or uint16 (bf16 bit patterns); a torch
CPU tensor of dtype bfloat16/float64 is accepted and viewed without copying
its values.  Outputs are numpy float64 / int32.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hylra_oracle.c")
_LIB = os.path.join(_HERE, "libhylra_oracle.so")
_lock = threading.Lock()
_lib = None

F64, BF16 = 0, 1


def build(force: bool = True) -> str:
    """Compile the oracle with gcc (-O2, OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.run(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", tmp, _SRC, "-lm"],
            check=True,
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            # HYLRA_ORACLE_LIB: a library built elsewhere from the same source (the sanitizer
            # test builds one with -fsanitize=address,undefined)
            path = os.environ.get("HYLRA_ORACLE_LIB")
            if not path:
                build(force=False)
                path = _LIB
            lib = ctypes.CDLL(path)
            vp, i32, i64, f64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_long, ctypes.c_double
            lib.hylra_oracle_full_attn_topk.argtypes = [i32, i32, i32, i32, i32, i64, i32, f64,
                                                        vp, vp, vp, vp, vp, vp]
            lib.hylra_oracle_full_attn_topk.restype = i32
            lib.hylra_oracle_reuse_sparse_attn.argtypes = [i32, i32, i32, i32, i32, i64, i32, f64,
                                                           vp, vp, vp, vp, vp]
            lib.hylra_oracle_reuse_sparse_attn.restype = i32
            lib.hylra_oracle_decode_step.argtypes = [i32, i32, vp, i32, i32, i32, i32, i64, i32,
                                                     f64, vp, vp, vp, vp, vp, vp]
            lib.hylra_oracle_decode_step.restype = i32
            lib.hylra_oracle_full_attn_topk_blocks.argtypes = [i32, i32, i32, i32, i32, i64, i32, i32, f64,
                                                               vp, vp, vp, vp, vp, vp]
            lib.hylra_oracle_full_attn_topk_blocks.restype = i32
            lib.hylra_oracle_reuse_block_attn.argtypes = [i32, i32, i32, i32, i32, i64, i32, i32, f64,
                                                          vp, vp, vp, vp, vp]
            lib.hylra_oracle_reuse_block_attn.restype = i32
            lib.hylra_oracle_overlap.argtypes = [vp, vp, i32]
            lib.hylra_oracle_overlap.restype = f64
            lib.hylra_oracle_overlap_counts.argtypes = [i32, i32, i32, i32, vp, vp]
            lib.hylra_oracle_overlap_counts.restype = None
            lib.hylra_oracle_policy_search.argtypes = [i32, vp, f64, vp, vp]
            lib.hylra_oracle_policy_search.restype = i32
            lib.hylra_oracle_threads.restype = i32
            _lib = lib
    return _lib


def _as_np(x):
    """numpy view of a float64 / bf16-bit-pattern tensor, C-contiguous."""
    if not isinstance(x, np.ndarray):  # torch tensor
        import torch

        x = x.detach().cpu().contiguous()
        if x.dtype == torch.bfloat16:
            x = x.view(torch.int16).numpy().view(np.uint16)
        elif x.dtype == torch.float64:
            x = x.numpy()
        else:
            raise TypeError("oracle takes float64 or bfloat16 tensors, got %s" % x.dtype)
    if x.dtype == np.float64:
        kind = F64
    elif x.dtype == np.uint16:
        kind = BF16
    else:
        raise TypeError("oracle takes float64 or uint16 (bf16 bits) arrays, got %s" % x.dtype)
    return np.ascontiguousarray(x), kind


def _triple(q, K, V):
    q, kq = _as_np(q)
    K, kk = _as_np(K)
    V, kv = _as_np(V)
    if not (kq == kk == kv):
        raise TypeError("q, K, V must share one element type")
    B, Hq, d = q.shape
    Bk, Hkv, N, dk = K.shape
    if (Bk, dk) != (B, d) or V.shape != K.shape:
        raise ValueError("shape mismatch: q %s K %s V %s" % (q.shape, K.shape, V.shape))
    return q, K, V, kq, B, Hq, Hkv, d, N


def _ptr(a):
    return ctypes.c_void_p(a.ctypes.data) if a is not None else None


def _check(rc, what):
    if rc != 0:
        raise RuntimeError("%s failed with oracle status %d" % (what, rc))


def full_attn_topk(q, K, V, k, scale=0.0, want_out=True, want_idx=True, want_shat=False):
    """Full layer of Algorithm 2: returns (out [B,Hq,d], idx [B,Hkv,k], shat or None)."""
    q, K, V, kind, B, Hq, Hkv, d, N = _triple(q, K, V)
    out = np.empty((B, Hq, d), np.float64) if want_out else None
    idx = np.empty((B, Hkv, k), np.int32) if want_idx else None
    shat = np.empty((B, Hkv, N), np.float64) if want_shat else None
    rc = _load().hylra_oracle_full_attn_topk(kind, B, Hq, Hkv, d, N, int(k), float(scale),
                                             _ptr(q), _ptr(K), _ptr(V), _ptr(out), _ptr(idx),
                                             _ptr(shat))
    _check(rc, "full_attn_topk")
    return out, idx, shat


def reuse_sparse_attn(q, K, V, idx, scale=0.0):
    """Reuse layer of Algorithm 2: out [B,Hq,d] over the rows named by idx [B,Hkv,k]."""
    q, K, V, kind, B, Hq, Hkv, d, N = _triple(q, K, V)
    idx = np.ascontiguousarray(np.asarray(idx, dtype=np.int32))
    if idx.shape[:2] != (B, Hkv):
        raise ValueError("idx shape %s does not match [B=%d, Hkv=%d, k]" % (idx.shape, B, Hkv))
    k = idx.shape[2]
    out = np.empty((B, Hq, d), np.float64)
    rc = _load().hylra_oracle_reuse_sparse_attn(kind, B, Hq, Hkv, d, N, k, float(scale),
                                                _ptr(q), _ptr(K), _ptr(V), _ptr(idx), _ptr(out))
    _check(rc, "reuse_sparse_attn")
    return out


def full_attn_topk_blocks(q, K, V, block, kb, scale=0.0, want_bscore=False):
    """Full layer, block-level TopK: returns (out [B,Hq,d], bidx [B,Hkv,kb], bscore or None)."""
    q, K, V, kind, B, Hq, Hkv, d, N = _triple(q, K, V)
    nblk = -(-N // int(block))
    out = np.empty((B, Hq, d), np.float64)
    bidx = np.empty((B, Hkv, int(kb)), np.int32)
    bscore = np.empty((B, Hkv, nblk), np.float64) if want_bscore else None
    rc = _load().hylra_oracle_full_attn_topk_blocks(kind, B, Hq, Hkv, d, N, int(block), int(kb),
                                                    float(scale), _ptr(q), _ptr(K), _ptr(V),
                                                    _ptr(out), _ptr(bidx), _ptr(bscore))
    _check(rc, "full_attn_topk_blocks")
    return out, bidx, bscore


def reuse_block_attn(q, K, V, bidx, block, scale=0.0):
    """Reuse layer on inherited block numbers bidx [B,Hkv,kb]: out [B,Hq,d]."""
    q, K, V, kind, B, Hq, Hkv, d, N = _triple(q, K, V)
    bidx = np.ascontiguousarray(np.asarray(bidx, dtype=np.int32))
    if bidx.shape[:2] != (B, Hkv):
        raise ValueError("bidx shape %s does not match [B=%d, Hkv=%d, kb]" % (bidx.shape, B, Hkv))
    out = np.empty((B, Hq, d), np.float64)
    rc = _load().hylra_oracle_reuse_block_attn(kind, B, Hq, Hkv, d, N, int(block), bidx.shape[2],
                                               float(scale), _ptr(q), _ptr(K), _ptr(V), _ptr(bidx),
                                               _ptr(out))
    _check(rc, "reuse_block_attn")
    return out


def decode_step(policy, q_l, K_l, V_l, k, scale=0.0):
    """Algorithm 2 over all layers.  Returns (outs list, idx_final, idx_trace [L,B,Hkv,k])."""
    L = len(policy)
    trip = [_triple(q_l[l], K_l[l], V_l[l]) for l in range(L)]
    kind, B, Hq, Hkv, d, N = trip[0][3:]
    for t in trip:
        if t[3:] != (kind, B, Hq, Hkv, d, N):
            raise ValueError("all layers must share one shape and element type")
    pol = np.ascontiguousarray(np.asarray(policy, dtype=np.uint8))
    outs = [np.empty((B, Hq, d), np.float64) for _ in range(L)]
    idx = np.full((B, Hkv, k), -1, np.int32)
    trace = np.empty((L, B, Hkv, k), np.int32)
    arr = ctypes.c_void_p * L
    rc = _load().hylra_oracle_decode_step(
        kind, L, _ptr(pol), B, Hq, Hkv, d, N, int(k), float(scale),
        arr(*[t[0].ctypes.data for t in trip]), arr(*[t[1].ctypes.data for t in trip]),
        arr(*[t[2].ctypes.data for t in trip]), arr(*[o.ctypes.data for o in outs]),
        _ptr(idx), _ptr(trace))
    _check(rc, "decode_step")
    return outs, idx, trace


def overlap(a, b):
    """Overlap ratio |a ∩ b| / k of two index sets of equal size (Eq. 2)."""
    a = np.ascontiguousarray(np.asarray(a, dtype=np.int32).ravel())
    b = np.ascontiguousarray(np.asarray(b, dtype=np.int32).ravel())
    if a.size != b.size:
        raise ValueError("sets must have equal size")
    return _load().hylra_oracle_overlap(_ptr(a), _ptr(b), a.size)


def overlap_counts(idx_l):
    """Pooled overlap counts of the layers' index sets: int64 [L, L], entries i <= j filled
    (sum over all (batch, KV head) sets of |S_i ∩ S_j|), the rest zero."""
    arrs = [np.ascontiguousarray(np.asarray(a, dtype=np.int32)) for a in idx_l]
    L = len(arrs)
    B, H, k = arrs[0].shape
    for a in arrs:
        if a.shape != (B, H, k):
            raise ValueError("all layers must share one idx shape")
    counts = np.zeros((L, L), np.int64)
    ptrs = (ctypes.c_void_p * L)(*[a.ctypes.data for a in arrs])
    _load().hylra_oracle_overlap_counts(L, B, H, k, ptrs, _ptr(counts))
    return counts


def similarity_matrix(counts):
    """M[i][j] = counts[i][j] / counts[j][j] for i <= j (diagonal 1), zero below the diagonal."""
    counts = np.asarray(counts, dtype=np.float64)
    L = counts.shape[0]
    M = np.zeros((L, L))
    for j in range(L):
        for i in range(j + 1):
            M[i, j] = counts[i, j] / counts[j, j] if counts[j, j] > 0 else (1.0 if i == j else 0.0)
    return M


def policy_search(M, theta):
    """Algorithm 1: returns (policy uint8 [L] with 0 = Full, 1 = Reuse; C* Full layers; S*)."""
    M = np.ascontiguousarray(np.asarray(M, dtype=np.float64))
    L = M.shape[0]
    policy = np.empty(L, np.uint8)
    s = ctypes.c_double()
    c = _load().hylra_oracle_policy_search(L, _ptr(M), float(theta), _ptr(policy), ctypes.byref(s))
    return policy, int(c), float(s.value)


def gather_rows(K, V, idx):
    """Index-guided prefetch, plain definition (paper: "index-guided offloading"; Algorithm 2,
    K^sparse = K^cache[I], V^sparse = V^cache[I]): returns (K_sparse, V_sparse, idx_compact)
    with K_sparse[b,g,t] = K[b,g,idx[b,g,t]] (zero rows for padding entries, i.e. < 0 or >= N)
    and idx_compact[b,g,t] = t, or -1 for padding.  Element type is kept."""
    K, _ = _as_np(K)
    V, _ = _as_np(V)
    idx = np.asarray(idx, dtype=np.int64)
    B, H, N, d = K.shape
    k = idx.shape[2]
    Ks, Vs = np.zeros((B, H, k, d), K.dtype), np.zeros((B, H, k, d), V.dtype)
    ic = np.full((B, H, k), -1, np.int32)
    for b in range(B):
        for g in range(H):
            for t in range(k):
                j = idx[b, g, t]
                if 0 <= j < N:
                    Ks[b, g, t] = K[b, g, j]
                    Vs[b, g, t] = V[b, g, j]
                    ic[b, g, t] = t
    return Ks, Vs, ic


def gather_blocks(K, V, bidx, block, lens=None):
    """Index-guided prefetch at block granularity (paper: "selective prefetching of only the
    critical KV blocks"; blocks as in the block-level variant: `block` consecutive rows, the last
    block of a sequence possibly short).  Slot t * block + r of the compact cache holds row
    bidx[b,g,t] * block + r of sequence b when that row exists (block number in range and row
    below the sequence's length), else zeros.  Returns (K_sparse, V_sparse [B,H,kb*block,d],
    idx_compact [B,H,kb*block] = the slot's own number, or -1 where the slot holds no row)."""
    K, _ = _as_np(K)
    V, _ = _as_np(V)
    bidx = np.asarray(bidx, dtype=np.int64)
    B, H, N, d = K.shape
    kb = bidx.shape[2]
    block = int(block)
    Ks, Vs = np.zeros((B, H, kb * block, d), K.dtype), np.zeros((B, H, kb * block, d), V.dtype)
    ic = np.full((B, H, kb * block), -1, np.int32)
    for b in range(B):
        n = N if lens is None else int(lens[b])
        for g in range(H):
            for t in range(kb):
                c = bidx[b, g, t]
                if c < 0:
                    continue
                for r in range(block):
                    j = c * block + r
                    if j < n:
                        Ks[b, g, t * block + r] = K[b, g, j]
                        Vs[b, g, t * block + r] = V[b, g, j]
                        ic[b, g, t * block + r] = t * block + r
    return Ks, Vs, ic


def append_rows(K, V, k_new, v_new, lens):
    """Decode-time cache update that precedes Algorithm 2 (its K^cache, V^cache hold the
    current token): the token's key and value of every (batch, KV head), k_new / v_new
    [B,Hkv,d], become row lens[b] of sequence b.  Returns copies (K', V', lens + 1)."""
    K, _ = _as_np(K)
    V, _ = _as_np(V)
    k_new, _ = _as_np(k_new)
    v_new, _ = _as_np(v_new)
    lens = np.asarray(lens, dtype=np.int64)
    B, H, N, d = K.shape
    if k_new.shape != (B, H, d) or v_new.shape != (B, H, d) or lens.shape != (B,):
        raise ValueError("k_new / v_new must be [B,Hkv,d] and lens [B]")
    if lens.min() < 0 or lens.max() >= N:
        raise ValueError("a sequence has no free row left")
    K2, V2 = K.copy(), V.copy()
    for b in range(B):
        for g in range(H):
            K2[b, g, lens[b]] = k_new[b, g]
            V2[b, g, lens[b]] = v_new[b, g]
    return K2, V2, (lens + 1).astype(np.int32)


def threads():
    return _load().hylra_oracle_threads()
