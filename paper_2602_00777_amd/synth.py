"""Seeded synthetic decode-attention workloads.

This module only DRAWS inputs (queries, KV caches, planted positions, policy
vectors).  It holds none of the method's arithmetic: no scores, no softmax, no
selection.  Both the HIP path and the CPU oracle are fed from here so that they
see identical tensors.

The paper evaluates on long prompts (8K-60K tokens, top-k budget 2048) through
real models; neither the prompts nor the weights are available, so the inputs
here imitate only the shapes and the sparsity structure: i.i.d. N(0,1) caches
in which a small planted set of positions per KV head is pushed towards the
group's mean query direction, and that set drifts from layer to layer with a
fixed carry-over fraction (the inter-layer similarity the method relies on).
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch

FULL, REUSE = 0, 1


@dataclass(frozen=True)
class Workload:
    name: str
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    batch: int
    ctx_len: int
    top_k: int
    full_layers: Tuple[int, ...]
    plant_frac: float          # fraction of positions planted per (batch, KV head)
    beta: float                # planted rows get beta * q_hat added to K
    carry: float               # fraction of the planted set kept from layer l to l+1
    sink_prefix: int = 0       # positions 0..sink_prefix-1 are planted in every layer
    seed: int = 0
    description: str = field(default="", compare=False)

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def n_planted(self) -> int:
        return int(round(self.plant_frac * self.ctx_len))

    def policy(self) -> np.ndarray:
        p = np.full(self.n_layers, REUSE, dtype=np.uint8)
        p[list(self.full_layers)] = FULL
        return p

    def kv_bytes_per_layer(self) -> int:
        return 2 * self.batch * self.n_kv_heads * self.ctx_len * self.head_dim * 2


def _every(step: int, n: int) -> Tuple[int, ...]:
    return tuple(range(0, n, step))


WORKLOADS = {
    "toy": Workload("toy", 2, 8, 2, 64, 1, 2048, 128, (0,), 0.02, 3.0, 1.0, seed=0,
                    description="2-layer toy, policy [full, reuse]"),
    "llama3_8b_32k": Workload("llama3_8b_32k", 32, 32, 8, 128, 8, 32768, 2048,
                              (0, 1, 2, 15, 31), 0.01, 2.5, 0.8, seed=0,
                              description="Llama-3-8B-shaped, batch 8, 32K context"),
    "long_131k": Workload("long_131k", 32, 32, 8, 128, 1, 131072, 4096, _every(4, 32),
                          0.01, 2.5, 0.8, seed=0,
                          description="single sequence, 128K context, full every 4th layer"),
    "serve_b32_16k": Workload("serve_b32_16k", 32, 32, 8, 128, 32, 16384, 1024, (0, 1, 31),
                              0.005, 2.5, 0.8, seed=0,
                              description="high-batch serving shape"),
    "qwen25_7b_64k": Workload("qwen25_7b_64k", 28, 28, 4, 128, 4, 65536, 2048, (0, 1, 27),
                              0.01, 2.5, 0.7, sink_prefix=4, seed=0,
                              description="Qwen2.5-7B-shaped, GQA group 7, 64K context"),
}


def scaled(w: Workload, **changes) -> Workload:
    """Copy of a workload with some fields replaced (for reduced-size test cases)."""
    return replace(w, **changes)


def planted_positions(w: Workload) -> List[np.ndarray]:
    """Planted position sets, one int64 array [B, Hkv, P(+sink)] per layer.

    Layer 0 draws P positions uniformly without replacement.  Each later layer
    keeps a random ``carry`` fraction of the previous layer's set and redraws
    the rest from positions outside it, so the set size stays constant.
    """
    rng = np.random.RandomState(w.seed + 7919)
    P = w.n_planted
    lo = w.sink_prefix
    B, H, N = w.batch, w.n_kv_heads, w.ctx_len
    if P + lo > N:
        raise ValueError("planted set larger than the context")
    keep_n = int(round(w.carry * P))
    sink = np.arange(lo, dtype=np.int64)
    layers: List[np.ndarray] = []
    cur = np.empty((B, H, P), dtype=np.int64)
    for b in range(B):
        for h in range(H):
            cur[b, h] = lo + rng.permutation(N - lo)[:P]
    for l in range(w.n_layers):
        if l > 0:
            nxt = np.empty_like(cur)
            for b in range(B):
                for h in range(H):
                    old = cur[b, h]
                    kept = old[rng.permutation(P)[:keep_n]]
                    free = np.ones(N, dtype=bool)
                    free[old] = False
                    free[:lo] = False
                    pool = np.flatnonzero(free)
                    fresh = pool[rng.permutation(pool.size)[:P - keep_n]]
                    nxt[b, h] = np.concatenate([kept, fresh])
            cur = nxt
        full = np.concatenate([np.broadcast_to(sink, (B, H, lo)), cur], axis=2) if lo else cur
        layers.append(np.sort(full, axis=2))
    return layers


def make_layer(w: Workload, layer: int, planted: Optional[np.ndarray], device="cpu"):
    """Draw one layer's (q, K, V) as bf16 tensors on ``device``.

    q [B,Hq,d], K and V [B,Hkv,N,d] are N(0,1) in fp32; rows of K at the planted
    positions get ``beta * q_hat`` added, q_hat being the unit vector along the
    mean of the group's queries; then everything is rounded to bf16.
    """
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed((w.seed * 1000003 + layer * 7 + 1) & 0x7FFFFFFF)
    B, Hq, Hkv, d, N = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ctx_len
    q = torch.randn((B, Hq, d), generator=gen, device=dev, dtype=torch.float32)
    K = torch.randn((B, Hkv, N, d), generator=gen, device=dev, dtype=torch.float32)
    if planted is not None and planted.shape[-1] > 0 and w.beta != 0.0:
        qm = q.view(B, Hkv, w.group, d).mean(dim=2)
        q_hat = qm / qm.norm(dim=-1, keepdim=True)
        pos = torch.as_tensor(planted, device=dev)                    # [B,Hkv,P]
        boost = (w.beta * q_hat).unsqueeze(2).expand(-1, -1, pos.shape[2], -1)
        K.scatter_add_(2, pos.unsqueeze(-1).expand(-1, -1, -1, d), boost.contiguous())
    Kb = K.to(torch.bfloat16)
    del K
    V = torch.randn((B, Hkv, N, d), generator=gen, device=dev, dtype=torch.float32)
    Vb = V.to(torch.bfloat16)
    del V
    return q.to(torch.bfloat16), Kb, Vb


def make_workload(w: Workload, device="cpu", layers: Optional[Sequence[int]] = None):
    """All (or the listed) layers of a workload: (policy, planted, [(q,K,V) per layer])."""
    planted = planted_positions(w)
    which = range(w.n_layers) if layers is None else layers
    data = [make_layer(w, l, planted[l], device) for l in which]
    return w.policy(), planted, data


# ---- paged caches and ragged batches (layout only) ------------------------------------------

def page_table(batch: int, ctx_len: int, page_size: int, seed: int = 0, spare_pages: int = 3) -> np.ndarray:
    """A block table int32 [B, ceil(N / page_size)] that scatters the pages of every sequence
    over a pool of B * pages + spare_pages pages (a random permutation, as a serving engine's
    allocator would leave them after many requests)."""
    per_seq = -(-ctx_len // page_size)
    rng = np.random.RandomState(seed + 104729)
    perm = rng.permutation(batch * per_seq + spare_pages)[:batch * per_seq]
    return perm.reshape(batch, per_seq).astype(np.int32)


def to_pool(x: torch.Tensor, table: np.ndarray, page_size: int, n_pages: Optional[int] = None) -> torch.Tensor:
    """Copies a contiguous cache tensor x [B,Hkv,N,d] into a pool [pages, Hkv, page_size, d]
    laid out by ``table`` (rows past N in a sequence's last page are zero)."""
    B, H, N, d = x.shape
    per_seq = table.shape[1]
    if n_pages is None:
        n_pages = int(table.max()) + 1
    pad = per_seq * page_size - N
    if pad:
        x = torch.cat([x, torch.zeros((B, H, pad, d), dtype=x.dtype, device=x.device)], dim=2)
    pages = x.view(B, H, per_seq, page_size, d).permute(0, 2, 1, 3, 4).reshape(B * per_seq, H, page_size, d)
    pool = torch.zeros((n_pages, H, page_size, d), dtype=x.dtype, device=x.device)
    pool[torch.as_tensor(table.reshape(-1).astype(np.int64), device=x.device)] = pages
    return pool


def ragged_lengths(batch: int, ctx_len: int, seed: int = 0, shortest: float = 0.25) -> np.ndarray:
    """Sequence lengths int32 [B]: uniform in [shortest * N, N], the first one exactly N."""
    rng = np.random.RandomState(seed + 15485863)
    lens = rng.randint(max(1, int(shortest * ctx_len)), ctx_len + 1, size=batch)
    lens[0] = ctx_len
    return lens.astype(np.int32)
