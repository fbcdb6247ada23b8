"""GPU parity over seeded random shapes, with the library choosing its kernels by itself: the
planner's branches (kernel per group size, head_dim and batch; split counts; self-scheduling
or even splits; single- or three-launch selection) are reached by the shapes, not by options.
Every case is drawn from its seed alone and is compared with the CPU oracle like the fixed
cases of the other parity tests."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_00777_amd import binding, synth
from tests.parity import assert_idx_valid, assert_out_close

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def say(msg):
    print("[case] " + msg, flush=True)


def draw(seed, big_batch=False):
    """A shape whose oracle run stays around a second: batch * n_kv_heads * ctx_len <= 600K rows
    (1.5M for the large batches of short sequences)."""
    rng = np.random.RandomState(1000003 * seed + 17)
    d = int(rng.choice([64, 128]))
    G = int(rng.choice([1, 2, 3, 4, 5, 7, 8]))
    Hkv = int(rng.choice([1, 2, 4, 8]))
    B = int(rng.choice([64, 100, 128, 256, 300] if big_batch else [1, 2, 3, 5, 8, 16, 40]))
    cap = max(300, (1500000 if big_batch else 600000) // (B * Hkv))
    N = int(rng.randint(200, min(cap, 50000) + 1))
    k = int(rng.randint(1, min(N, 3000) + 1))
    modes = (["ragged", "paged+ragged", "blocks+paged+ragged", "plain"] if big_batch else
             ["plain", "plain", "paged", "ragged", "paged+ragged", "blocks", "blocks+paged+ragged"])
    mode = str(rng.choice(modes))
    page = int(rng.choice([1, 8, 16, 64, 256]))
    block = int(rng.choice([2, 16, 33, 128]))
    return rng, B, Hkv, G, d, N, k, mode, page, block


@pytest.mark.parametrize("seed", range(1000, 1016))
def test_random_large_batch(seed):
    """Batches of 64 to 300 short sequences, mostly of unequal lengths."""
    check_shape(seed, True)


@pytest.mark.parametrize("seed", range(96))
def test_random_shape(seed):
    check_shape(seed, False)


def check_shape(seed, big_batch):
    rng, B, Hkv, G, d, N, k, mode, page, block = draw(seed, big_batch)
    say("seed %d: B=%d Hkv=%d G=%d d=%d N=%d k=%d mode=%s page=%d block=%d" % (seed, B, Hkv, G, d, N, k, mode, page, block))
    w = synth.Workload("case", 1, Hkv * G, Hkv, d, B, N, 1, (0,), 0.02, 3.0, 1.0, seed=5000 + seed)
    q, K, V = synth.make_layer(w, 0, synth.planted_positions(w)[0], DEV)
    q2 = torch.roll(q, 1, dims=0).contiguous() if B > 1 else torch.roll(q, 1, dims=1).contiguous()
    lens = np.full(B, N, np.int32)
    if "ragged" in mode:
        lens = rng.randint(0, N + 1, size=B).astype(np.int32)
        lens[rng.randint(B)] = N
    use_cache = mode not in ("plain", "blocks")
    Kc, Vc, cache = K, V, None
    if "paged" in mode:
        table = synth.page_table(B, N, page, seed)
        n_pages = int(table.max()) + 1
        Kc, Vc = synth.to_pool(K, table, page, n_pages), synth.to_pool(V, table, page, n_pages)
        cache = binding.PagedCache(torch.from_numpy(table).to(DEV), page, N,
                                   torch.from_numpy(lens).to(DEV) if "ragged" in mode else None)
    elif "ragged" in mode:
        cache = binding.PagedCache(None, 0, N, torch.from_numpy(lens).to(DEV))
    blocks = "blocks" in mode
    if blocks:
        k = max(1, min(k // block, -(-N // block)))           # k counts blocks
    with binding.Context(B, Hkv * G, Hkv, d, N, min(N, k * block) if blocks else k) as ctx:
        for rep in range(2):                                  # twice: counters, maps and scratch are reused
            if blocks and use_cache:
                out, idx = ctx.full_attn_topk_blocks_paged(q, Kc, Vc, cache, block, k)
                sp = ctx.reuse_block_attn_paged(q2, Kc, Vc, cache, idx, block)
            elif blocks:
                out, idx = ctx.full_attn_topk_blocks(q, K, V, block, k)
                sp = ctx.reuse_block_attn(q2, K, V, idx, block)
            elif use_cache:
                out, idx = ctx.full_attn_topk_paged(q, Kc, Vc, cache, k)
                sp = ctx.reuse_sparse_attn_paged(q2, Kc, Vc, cache, idx)
            else:
                out, idx = ctx.full_attn_topk(q, K, V, k)
                sp = ctx.reuse_sparse_attn(q2, K, V, idx)
            torch.cuda.synchronize()
        out, idx, sp = out.cpu().numpy(), idx.cpu().numpy(), sp.cpu().numpy()
    for b in range(B):
        n = int(lens[b])
        if n == 0:
            assert np.all(out[b] == 0) and np.all(sp[b] == 0) and np.all(idx[b] == -1), "empty sequence b=%d" % b
            continue
        qb, Kb, Vb = q[b:b + 1], K[b:b + 1, :, :n], V[b:b + 1, :, :n]
        if blocks:
            kk = min(k, -(-n // block))
            ref_out, ref_idx, score = oracle.full_attn_topk_blocks(qb, Kb, Vb, block, kk, want_bscore=True)
        else:
            kk = min(k, n)
            ref_out, ref_idx, score = oracle.full_attn_topk(qb, Kb, Vb, kk, want_shat=True)
        assert_out_close(out[b:b + 1], ref_out, "full out b=%d" % b)
        assert np.all(idx[b, :, kk:] == -1), "entries past the sequence's own count must be -1 (b=%d)" % b
        assert_idx_valid(idx[b:b + 1, :, :kk], score, kk, "idx b=%d" % b, exact_ref=ref_idx)
        sel = idx[b:b + 1, :, :kk]
        ref_sp = (oracle.reuse_block_attn(q2[b:b + 1], Kb, Vb, sel, block) if blocks
                  else oracle.reuse_sparse_attn(q2[b:b + 1], Kb, Vb, sel))
        assert_out_close(sp[b:b + 1], ref_sp, "reuse out b=%d" % b)
