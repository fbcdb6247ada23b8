"""GPU parity of the paged-cache / per-sequence-length entry points against the CPU oracle.
The oracle has no notion of pages or of a batch of unequal lengths: it is called per sequence
on that sequence's own first n_b rows of the contiguous tensors the pools were filled from."""
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


def make_case(seed, B, Hkv, G, d, N, page_size, ragged):
    w = synth.Workload("case", 1, Hkv * G, Hkv, d, B, N, 1, (0,), 0.02, 3.0, 1.0, seed=seed)
    q, K, V = synth.make_layer(w, 0, synth.planted_positions(w)[0], DEV)
    table = synth.page_table(B, N, page_size, seed)
    n_pages = int(table.max()) + 1
    Kp, Vp = synth.to_pool(K, table, page_size, n_pages), synth.to_pool(V, table, page_size, n_pages)
    lens = synth.ragged_lengths(B, N, seed) if ragged else None
    if ragged and B > 2:
        lens[1] = 1                      # a one-row sequence
        lens[2] = min(N, 37)             # shorter than k in most cases
    cache = binding.PagedCache(torch.from_numpy(table).to(DEV), page_size, N,
                               torch.from_numpy(lens).to(DEV) if ragged else None)
    return q, K, V, Kp, Vp, cache, (lens if ragged else np.full(B, N, np.int32))


def oracle_full(q, K, V, lens, k):
    """Per sequence: the oracle on its first n_b rows with min(k, n_b)."""
    B = q.shape[0]
    outs, idxs, shats = [], [], []
    for b in range(B):
        n, kb = int(lens[b]), min(k, int(lens[b]))
        o, i, s = oracle.full_attn_topk(q[b:b + 1], K[b:b + 1, :, :n], V[b:b + 1, :, :n], kb, want_shat=True)
        outs.append(o[0]), idxs.append(i[0]), shats.append(s[0])
    return outs, idxs, shats


def check_full(out, idx, refs, lens, k, what):
    outs, idxs, shats = refs
    for b in range(len(lens)):
        kb = min(k, int(lens[b]))
        assert_out_close(out[b:b + 1], outs[b][None], "%s out b=%d" % (what, b))
        assert np.all(idx[b, :, kb:] == -1), "%s: entries past min(k, n_b) must be -1 (b=%d)" % (what, b)
        assert_idx_valid(idx[b:b + 1, :, :kb], shats[b][None], kb, "%s idx b=%d" % (what, b), exact_ref=idxs[b][None])


CASES = [
    # B, Hkv, G, d,   N,    k,  page, ragged
    (2, 2, 4, 128, 3000, 200, 16, False),
    (4, 2, 4, 128, 5003, 300, 16, True),
    (3, 1, 2, 64, 2048, 128, 64, True),
    (4, 2, 7, 128, 3001, 256, 32, True),        # matrix-core Full kernel
    (1, 1, 4, 128, 40000, 1000, 128, False),    # three-launch selection
    (3, 1, 4, 128, 36000, 900, 16, True),
    (16, 8, 4, 128, 1500, 64, 16, True),        # self-scheduling Full kernel (batch * n_kv_heads >= 64)
    (2, 1, 1, 128, 700, 700, 1, True),          # one row per page; k = longest sequence
]


@pytest.mark.parametrize("B,Hkv,G,d,N,k,page,ragged", CASES)
def test_paged_full_and_reuse_match_oracle(B, Hkv, G, d, N, k, page, ragged):
    say("paged B=%d Hkv=%d G=%d d=%d N=%d k=%d page=%d ragged=%s" % (B, Hkv, G, d, N, k, page, ragged))
    q, K, V, Kp, Vp, cache, lens = make_case(500 + N + G, B, Hkv, G, d, N, page, ragged)
    refs = oracle_full(q, K, V, lens, k)
    with binding.Context(B, Hkv * G, Hkv, d, N, k) as ctx:
        for rep in range(2):
            out, idx = ctx.full_attn_topk_paged(q, Kp, Vp, cache, k)
            torch.cuda.synchronize()
            out, idx = out.cpu().numpy(), idx.cpu().numpy()
            check_full(out, idx, refs, lens, k, "paged full (launch %d)" % rep)
        # Reuse on the GPU's own sets (padding included), against the oracle on the same sets
        sparse = ctx.reuse_sparse_attn_paged(q, Kp, Vp, cache, torch.from_numpy(idx).to(DEV))
        torch.cuda.synchronize()
        sparse = sparse.cpu().numpy()
    for b in range(B):
        n = int(lens[b])
        ref = oracle.reuse_sparse_attn(q[b:b + 1], K[b:b + 1, :, :n], V[b:b + 1, :, :n], idx[b:b + 1])
        assert_out_close(sparse[b:b + 1], ref, "paged reuse b=%d" % b)


@pytest.mark.parametrize("variant", [23, 43, 52, 72, 74])
def test_paged_full_kernel_variants(variant):
    say("paged full variant=%d" % variant)
    B, Hkv, G, d, N, k, page = 3, 2, 4, 128, 6000, 300, 16
    q, K, V, Kp, Vp, cache, lens = make_case(77, B, Hkv, G, d, N, page, True)
    refs = oracle_full(q, K, V, lens, k)
    with binding.Context(B, Hkv * G, Hkv, d, N, k) as ctx:
        ctx.set_option("full_variant", variant)
        for split_rows in (0, 768):
            ctx.set_option("full_split_rows", split_rows)
            out, idx = ctx.full_attn_topk_paged(q, Kp, Vp, cache, k)
            torch.cuda.synchronize()
            check_full(out.cpu().numpy(), idx.cpu().numpy(), refs, lens, k, "variant %d split %d" % (variant, split_rows))


@pytest.mark.parametrize("variant,waves", [(1, 4), (4, 4), (4, 8), (5, 8), (6, 4), (5, 0)])    # (5, 0): merge by packets
def test_paged_reuse_kernel_variants(variant, waves):
    say("paged reuse variant=%d waves=%d" % (variant, waves))
    B, Hkv, G, d, N, k, page = 3, 2, 4, 128, 4000, 1024, 16
    q, K, V, Kp, Vp, cache, lens = make_case(78, B, Hkv, G, d, N, page, True)
    rng = np.random.RandomState(variant)
    idx = np.stack([[np.sort(rng.permutation(N)[:k]) for _ in range(Hkv)] for _ in range(B)]).astype(np.int32)
    idx[:, :, ::9] = -1
    with binding.Context(B, Hkv * G, Hkv, d, N, k) as ctx:
        ctx.set_option("reuse_variant", variant)
        ctx.set_option("reuse_waves", waves)
        out = ctx.reuse_sparse_attn_paged(q, Kp, Vp, cache, torch.from_numpy(idx).to(DEV))
        torch.cuda.synchronize()
        out = out.cpu().numpy()
        assert ctx.get_info("last_reuse_merge") == (2 if waves == 0 else 1)
    for b in range(B):
        n = int(lens[b])
        ref = oracle.reuse_sparse_attn(q[b:b + 1], K[b:b + 1, :, :n], V[b:b + 1, :, :n],
                                       np.where(idx[b:b + 1] >= n, -1, idx[b:b + 1]))
        assert_out_close(out[b:b + 1], ref, "paged reuse b=%d" % b)


def test_paged_decode_step_chain():
    """Algorithm 2 over a paged, ragged batch: Full layers hand their sets to the Reuse layers."""
    say("paged decode step")
    B, Hkv, G, d, N, k, page, L = 4, 2, 4, 128, 3000, 256, 16, 5
    w = synth.Workload("chain", L, Hkv * G, Hkv, d, B, N, k, (0, 3), 0.02, 3.0, 0.8, seed=5)
    policy, _, data = synth.make_workload(w, DEV)
    table = synth.page_table(B, N, page, 5)
    lens = synth.ragged_lengths(B, N, 5)
    pools = [(synth.to_pool(K, table, page), synth.to_pool(V, table, page)) for _, K, V in data]
    cache = binding.PagedCache(torch.from_numpy(table).to(DEV), page, N, torch.from_numpy(lens).to(DEV))
    qs = [x[0] for x in data]
    with binding.Context(B, Hkv * G, Hkv, d, N, k) as ctx:
        outs, idx_buf = ctx.decode_step(policy, qs, [p[0] for p in pools], [p[1] for p in pools], k, paged=cache)
        torch.cuda.synchronize()
        cur = None
        for l in range(L):
            q, K, V = data[l]
            if policy[l] == synth.FULL:
                refs = oracle_full(q, K, V, lens, k)
                _, gidx = ctx.full_attn_topk_paged(q, pools[l][0], pools[l][1], cache, k)
                torch.cuda.synchronize()
                cur = gidx.cpu().numpy()
                check_full(outs[l].cpu().numpy(), cur, refs, lens, k, "step layer %d" % l)
            else:
                o = outs[l].cpu().numpy()
                for b in range(B):
                    n = int(lens[b])
                    ref = oracle.reuse_sparse_attn(q[b:b + 1], K[b:b + 1, :, :n], V[b:b + 1, :, :n], cur[b:b + 1])
                    assert_out_close(o[b:b + 1], ref, "step layer %d b=%d" % (l, b))
        assert np.array_equal(idx_buf.cpu().numpy(), cur)


def test_paged_block_decode_step_chain():
    """The layer chain with block indices on a paged, ragged batch: equal to the single calls."""
    say("paged block decode step")
    B, Hkv, G, d, N, block, kb, page, L = 4, 2, 4, 128, 3000, 32, 8, 16, 5
    w = synth.Workload("chain", L, Hkv * G, Hkv, d, B, N, kb * block, (0, 3), 0.02, 3.0, 0.8, seed=6)
    policy, _, data = synth.make_workload(w, DEV)
    table = synth.page_table(B, N, page, 6)
    lens = synth.ragged_lengths(B, N, 6)
    pools = [(synth.to_pool(K, table, page), synth.to_pool(V, table, page)) for _, K, V in data]
    cache = binding.PagedCache(torch.from_numpy(table).to(DEV), page, N, torch.from_numpy(lens).to(DEV))
    qs = [x[0] for x in data]
    with binding.Context(B, Hkv * G, Hkv, d, N, kb * block) as ctx:
        outs, idx_buf = ctx.decode_step(policy, qs, [p[0] for p in pools], [p[1] for p in pools], kb,
                                        block=block, paged=cache)
        torch.cuda.synchronize()
        cur = None
        for l in range(L):
            if policy[l] == synth.FULL:
                o, cur = ctx.full_attn_topk_blocks_paged(qs[l], pools[l][0], pools[l][1], cache, block, kb)
            else:
                o = ctx.reuse_block_attn_paged(qs[l], pools[l][0], pools[l][1], cache, cur, block)
            torch.cuda.synchronize()
            assert torch.allclose(o, outs[l], rtol=1e-5, atol=1e-6), "layer %d" % l
        assert torch.equal(idx_buf, cur)
        # and the first Full layer against the oracle, per sequence
        q, K, V = data[0]
        first = ctx.full_attn_topk_blocks_paged(q, pools[0][0], pools[0][1], cache, block, kb)[1].cpu().numpy()
        for b in range(B):
            n = int(lens[b])
            kk = min(kb, -(-n // block))
            _, ref_bidx, bs = oracle.full_attn_topk_blocks(q[b:b + 1], K[b:b + 1, :, :n], V[b:b + 1, :, :n], block, kk,
                                                           want_bscore=True)
            assert_idx_valid(first[b:b + 1, :, :kk], bs, kk, "b=%d" % b, exact_ref=ref_bidx)


@pytest.mark.parametrize("B,Hkv,G,d,N,k", [(4, 2, 4, 128, 5003, 300), (16, 8, 4, 128, 1500, 64), (3, 2, 7, 128, 3001, 256),
                                          (2, 2, 2, 64, 2048, 128)])
def test_sequence_lengths_on_a_contiguous_cache(B, Hkv, G, d, N, k):
    """block_table == NULL: per-sequence lengths over the ordinary [B,Hkv,N,d] cache."""
    say("ragged contiguous B=%d Hkv=%d G=%d d=%d N=%d k=%d" % (B, Hkv, G, d, N, k))
    w = synth.Workload("case", 1, Hkv * G, Hkv, d, B, N, 1, (0,), 0.02, 3.0, 1.0, seed=N)
    q, K, V = synth.make_layer(w, 0, synth.planted_positions(w)[0], DEV)
    lens = synth.ragged_lengths(B, N, N)
    lens[-1] = min(N, 29)
    cache = binding.PagedCache(None, 0, N, torch.from_numpy(lens).to(DEV))
    refs = oracle_full(q, K, V, lens, k)
    with binding.Context(B, Hkv * G, Hkv, d, N, k) as ctx:
        out, idx = ctx.full_attn_topk_paged(q, K, V, cache, k)
        sparse = ctx.reuse_sparse_attn_paged(q, K, V, cache, idx)
        torch.cuda.synchronize()
        out, idx, sparse = out.cpu().numpy(), idx.cpu().numpy(), sparse.cpu().numpy()
    check_full(out, idx, refs, lens, k, "ragged contiguous")
    for b in range(B):
        n = int(lens[b])
        ref = oracle.reuse_sparse_attn(q[b:b + 1], K[b:b + 1, :, :n], V[b:b + 1, :, :n], idx[b:b + 1])
        assert_out_close(sparse[b:b + 1], ref, "ragged contiguous reuse b=%d" % b)


BLOCK_CASES = [
    # B, Hkv, G, d,   N,  block, kb, page (0: contiguous with lengths)
    (4, 2, 4, 128, 4099, 128, 7, 16),       # blocks of 8 pages
    (3, 2, 4, 128, 3000, 48, 20, 32),       # blocks that straddle pages
    (3, 1, 7, 128, 3001, 100, 11, 0),
    (4, 2, 2, 64, 2048, 16, 40, 64),        # several blocks per page
    (16, 8, 4, 128, 1500, 32, 8, 16),       # self-scheduling Full kernel
    (2, 1, 4, 128, 36000, 8, 300, 16),      # three-launch selection over 4500 blocks
]


@pytest.mark.parametrize("B,Hkv,G,d,N,block,kb,page", BLOCK_CASES)
def test_paged_block_level_variant(B, Hkv, G, d, N, block, kb, page):
    """Block TopK and block reuse per sequence: sequence b has ceil(n_b / block) blocks."""
    say("paged blocks B=%d Hkv=%d G=%d d=%d N=%d block=%d kb=%d page=%d" % (B, Hkv, G, d, N, block, kb, page))
    q, K, V, Kp, Vp, cache, lens = make_case(900 + N + block, B, Hkv, G, d, N, page or 16, True)
    lens[0] = N                                     # one sequence of full length ...
    lens[-1] = max(1, N - block // 2 - 1)           # ... and one whose last block is short
    dlens = torch.from_numpy(lens).to(DEV)
    if page:
        cache = binding.PagedCache(cache.block_table, page, N, dlens)
    else:
        cache, Kp, Vp = binding.PagedCache(None, 0, N, dlens), K, V
    q2 = torch.roll(q, 1, dims=1).contiguous()      # another query for the Reuse layer
    with binding.Context(B, Hkv * G, Hkv, d, N, min(N, kb * block)) as ctx:
        out, bidx = ctx.full_attn_topk_blocks_paged(q, Kp, Vp, cache, block, kb)
        sparse = {}
        for variant in (1, 4):
            ctx.set_option("reuse_variant", variant)
            sparse[variant] = ctx.reuse_block_attn_paged(q2, Kp, Vp, cache, bidx, block)
        torch.cuda.synchronize()
        out, bidx = out.cpu().numpy(), bidx.cpu().numpy()
        sparse = {v: o.cpu().numpy() for v, o in sparse.items()}
    for b in range(B):
        n = int(lens[b])
        nb = -(-n // block)
        kk = min(kb, nb)
        Kb, Vb = K[b:b + 1, :, :n], V[b:b + 1, :, :n]
        ref_out, ref_bidx, bs = oracle.full_attn_topk_blocks(q[b:b + 1], Kb, Vb, block, kk, want_bscore=True)
        assert_out_close(out[b:b + 1], ref_out, "full out b=%d" % b)
        assert np.all(bidx[b, :, kk:] == -1), "entries past min(kb, blocks of the sequence) must be -1 (b=%d)" % b
        assert_idx_valid(bidx[b:b + 1, :, :kk], bs, kk, "block idx b=%d" % b, exact_ref=ref_bidx)
        ref = oracle.reuse_block_attn(q2[b:b + 1], Kb, Vb, bidx[b:b + 1, :, :kk], block)
        for v, o in sparse.items():
            assert_out_close(o[b:b + 1], ref, "reuse v%d b=%d" % (v, b))


SKEWED = [
    # B, Hkv, G, d,   N,   k, page, lengths of the first sequences (the rest: 1 + 13 b rows)
    (16, 4, 4, 128, 6000, 128, 16, (6000, 0, 1, 750, 40)),      # one long sequence gets most workgroups
    (16, 4, 4, 128, 6000, 128, 0, (33, 6000, 5999, 0, 0)),      # contiguous cache
    (32, 2, 2, 64, 4000, 64, 32, (4000, 7, 0, 2100)),           # head_dim 64: the vector self-scheduling kernel
    (64, 1, 4, 128, 3000, 32, 16, (3000, 3000, 1)),
    (300, 1, 4, 128, 700, 32, 16, (700, 0, 1, 699)),            # more sequences than threads in the deal's workgroup
]


@pytest.mark.parametrize("B,Hkv,G,d,N,k,page,head", SKEWED)
def test_skewed_lengths_deal_workgroups_by_rows(B, Hkv, G, d, N, k, page, head):
    """Very unequal lengths: the self-scheduling Full kernels give every (batch, KV head) a share
    of the workgroups in proportion to its rows (several segments for a long sequence, one
    workgroup for an empty one); with the even deal switched on the result is the same."""
    say("skewed B=%d Hkv=%d G=%d d=%d N=%d k=%d page=%d" % (B, Hkv, G, d, N, k, page))
    q, K, V, Kp, Vp, cache, _ = make_case(1300 + B + N, B, Hkv, G, d, N, page or 16, False)
    lens = np.array([(1 + 13 * b) % (N + 1) for b in range(B)], np.int32)
    lens[:len(head)] = head
    dlens = torch.from_numpy(lens).to(DEV)
    if page:
        cache = binding.PagedCache(cache.block_table, page, N, dlens)
    else:
        cache, Kp, Vp = binding.PagedCache(None, 0, N, dlens), K, V
    outs, idxs, shats = oracle_full(q, K, V, np.maximum(lens, 1), k)       # (the oracle wants a row; see below)
    with binding.Context(B, Hkv * G, Hkv, d, N, k) as ctx:
        res = {}
        for even in (0, 1):
            ctx.set_option("ragged_even", even)
            for rep in range(2):                                           # twice: counters and maps are reused
                out, idx = ctx.full_attn_topk_paged(q, Kp, Vp, cache, k)
                torch.cuda.synchronize()
            res[even] = (out.cpu().numpy(), idx.cpu().numpy())
    for even, (out, idx) in res.items():
        for b in range(B):
            n = int(lens[b])
            if n == 0:
                assert np.all(out[b] == 0) and np.all(idx[b] == -1), "empty sequence b=%d (even=%d)" % (b, even)
                continue
            kk = min(k, n)
            assert_out_close(out[b:b + 1], outs[b][None], "out b=%d even=%d" % (b, even))
            assert np.all(idx[b, :, kk:] == -1)
            assert_idx_valid(idx[b:b + 1, :, :kk], shats[b][None], kk, "idx b=%d even=%d" % (b, even), exact_ref=idxs[b][None])
    assert np.array_equal(res[0][1], res[1][1])


def test_paged_zero_length_sequence_and_errors():
    say("paged zero length, errors")
    B, Hkv, G, d, N, k, page = 3, 2, 4, 128, 1000, 100, 16
    q, K, V, Kp, Vp, cache, lens = make_case(79, B, Hkv, G, d, N, page, True)
    lens = lens.copy()
    lens[1] = 0
    cache = binding.PagedCache(cache.block_table, page, N, torch.from_numpy(lens).to(DEV))
    with binding.Context(B, Hkv * G, Hkv, d, N, k) as ctx:
        out, idx = ctx.full_attn_topk_paged(q, Kp, Vp, cache, k)
        sparse = ctx.reuse_sparse_attn_paged(q, Kp, Vp, cache, idx)
        torch.cuda.synchronize()
        out, idx, sparse = out.cpu().numpy(), idx.cpu().numpy(), sparse.cpu().numpy()
        assert np.all(out[1] == 0.0) and np.all(idx[1] == -1) and np.all(sparse[1] == 0.0)
        keep = [0, 2]
        refs = oracle_full(q[keep], K[keep], V[keep], lens[keep], k)
        check_full(out[keep], idx[keep], refs, lens[keep], k, "paged with an empty sequence")
        # argument checks
        bad = binding.PagedCache(cache.block_table, 24, N)
        with pytest.raises(binding.HylraError) as e:
            ctx.full_attn_topk_paged(q, Kp.view(-1, Hkv, 24, d)[:Kp.shape[0]], Vp.view(-1, Hkv, 24, d)[:Kp.shape[0]], bad, k)
        assert e.value.status == 1
        short = binding.PagedCache(cache.block_table[:, :10].contiguous(), page, N)
        with pytest.raises(binding.HylraError) as e:
            ctx.full_attn_topk_paged(q, Kp, Vp, short, k)
        assert e.value.status == 1
