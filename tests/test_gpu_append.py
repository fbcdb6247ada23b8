"""GPU parity of the append-then-attend entry points: the current token's key / value rows are
written into the cache (contiguous or paged, equal or per-sequence lengths) and the attention
of the same call covers them.  Reference: oracle.append_rows on the contiguous tensors, then the
oracle per sequence on its first n_b + 1 rows; the cache itself is compared bit for bit."""
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


def bits(t):
    return t.cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def make(seed, B, Hkv, G, d, N, layer=0):
    w = synth.Workload("case", layer + 1, Hkv * G, Hkv, d, B, N, 1, (0,), 0.02, 3.0, 1.0, seed=seed)
    q, K, V = synth.make_layer(w, layer, synth.planted_positions(w)[layer], DEV)
    gen = torch.Generator().manual_seed(seed * 31 + layer)
    k_new = torch.randn((B, Hkv, d), generator=gen).to(torch.bfloat16).to(DEV)
    v_new = torch.randn((B, Hkv, d), generator=gen).to(torch.bfloat16).to(DEV)
    # make the new key matter: push it along the group's mean query so that it is selected
    k_new = (k_new.float() + 3.0 * q.view(B, Hkv, G, d).float().mean(2)).to(torch.bfloat16)
    return q, K, V, k_new, v_new


def oracle_after_append(q, K, V, k_new, v_new, lens, k):
    K2, V2, n2 = oracle.append_rows(K.cpu(), V.cpu(), k_new.cpu(), v_new.cpu(), lens)
    outs, idxs, shats = [], [], []
    for b in range(q.shape[0]):
        n, kb = int(n2[b]), min(k, int(n2[b]))
        o, i, s = oracle.full_attn_topk(q[b:b + 1].cpu(), K2[b:b + 1, :, :n], V2[b:b + 1, :, :n], kb, want_shat=True)
        outs.append(o[0]), idxs.append(i[0]), shats.append(s[0])
    return K2, V2, n2, outs, idxs, shats


def check_full(out, idx, refs, k, what):
    K2, V2, n2, outs, idxs, shats = refs
    for b in range(len(n2)):
        kb = min(k, int(n2[b]))
        assert_out_close(out[b:b + 1], outs[b][None], "%s out b=%d" % (what, b))
        assert np.all(idx[b, :, kb:] == -1)
        assert_idx_valid(idx[b:b + 1, :, :kb], shats[b][None], kb, "%s idx b=%d" % (what, b), exact_ref=idxs[b][None])


@pytest.mark.parametrize("B,Hkv,G,d,N,k", [(2, 2, 4, 128, 3000, 200), (1, 2, 4, 64, 1500, 64), (3, 1, 7, 128, 2049, 300),
                                          (1, 2, 4, 128, 5000, 1024)])       # (the last: Reuse merge by packets)
def test_append_contiguous_equal_lengths(B, Hkv, G, d, N, k):
    """cache == NULL: the token becomes row N - 1 of every sequence."""
    say("append contiguous B=%d Hkv=%d G=%d d=%d N=%d k=%d" % (B, Hkv, G, d, N, k))
    q, K, V, k_new, v_new = make(900 + N, B, Hkv, G, d, N)
    lens = np.full(B, N - 1)
    refs = oracle_after_append(q, K, V, k_new, v_new, lens, k)
    Kc, Vc = K.clone(), V.clone()
    with binding.Context(B, Hkv * G, Hkv, d, N, k) as ctx:
        out, idx = ctx.append_full_attn_topk(q, k_new, v_new, Kc, Vc, k)
        torch.cuda.synchronize()
        assert np.array_equal(bits(Kc), refs[0]) and np.array_equal(bits(Vc), refs[1])
        out, idx = out.cpu().numpy(), idx.cpu().numpy()
        check_full(out, idx, refs, k, "append full")
        # the new row is among the selected ones (its key was pushed along the query)
        assert np.all((idx == N - 1).any(axis=2))
        # Reuse on a restored cache: same append, attention over the set just selected (which
        # names the new row: it must be read from k_new / v_new, the restored cache holds another
        # row there).  Once with the row written by the Reuse kernel itself, once by a launch of
        # its own before it.
        ref = oracle.reuse_sparse_attn(q.cpu(), refs[0], refs[1], idx)
        for unfused in (0, 1):
            ctx.set_option("append_unfused", unfused)
            Kc2, Vc2 = K.clone(), V.clone()
            sparse = ctx.append_reuse_sparse_attn(q, k_new, v_new, Kc2, Vc2, torch.from_numpy(idx).to(DEV))
            torch.cuda.synchronize()
            assert np.array_equal(bits(Kc2), refs[0]) and np.array_equal(bits(Vc2), refs[1])
            assert_out_close(sparse.cpu().numpy(), ref, "append reuse, append_unfused=%d" % unfused)
            if k == 1024:
                assert ctx.get_info("last_reuse_merge") == 2


@pytest.mark.parametrize("page", [0, 16, 1])
def test_append_with_sequence_lengths(page):
    """Per-sequence lengths (contiguous cache, 16-row pages, one-row pages): the token lands at
    each sequence's own length, one sequence is empty before the call, one is one row short of
    the capacity."""
    say("append with lengths, page=%d" % page)
    B, Hkv, G, d, N, k = 4, 2, 4, 128, 2500, 128
    q, K, V, k_new, v_new = make(77 + page, B, Hkv, G, d, N)
    lens = np.array([N - 1, 0, 37, 1200], np.int32)
    refs = oracle_after_append(q, K, V, k_new, v_new, lens, k)
    lens_d = torch.from_numpy(lens).to(DEV)
    if page:
        table = synth.page_table(B, N, page, 3)
        Kp, Vp = synth.to_pool(K, table, page), synth.to_pool(V, table, page)
        cache = binding.PagedCache(torch.from_numpy(table).to(DEV), page, N, lens_d)
    else:
        Kp, Vp = K.clone(), V.clone()
        cache = binding.PagedCache(None, 0, N, lens_d)
    with binding.Context(B, Hkv * G, Hkv, d, N, k) as ctx:
        out, idx = ctx.append_full_attn_topk(q, k_new, v_new, Kp, Vp, k, paged=cache)
        torch.cuda.synchronize()
        assert np.array_equal(lens_d.cpu().numpy(), lens), "the caller's lengths must not be written"
        check_full(out.cpu().numpy(), idx.cpu().numpy(), refs, k, "append full page=%d" % page)
        # the cache: exactly the appended rows changed
        if page:
            want_K = synth.to_pool(torch.from_numpy(refs[0].view(np.int16)).view(torch.bfloat16).to(DEV), table, page)
            want_V = synth.to_pool(torch.from_numpy(refs[1].view(np.int16)).view(torch.bfloat16).to(DEV), table, page)
            assert torch.equal(Kp.view(torch.int16), want_K.view(torch.int16))
            assert torch.equal(Vp.view(torch.int16), want_V.view(torch.int16))
        else:
            assert np.array_equal(bits(Kp), refs[0]) and np.array_equal(bits(Vp), refs[1])
        # Reuse with the same append on restored caches, over the set just selected (sequence 1 was
        # empty: its only row is the new one; the set of every sequence names its new row)
        idx_d = idx
        idx_h = idx.cpu().numpy()
        for b in range(B):
            assert np.all((idx_h[b] == lens[b]).any(axis=1)), "the new row of sequence %d is not selected" % b
        for unfused in (0, 1):
            ctx.set_option("append_unfused", unfused)
            if page:
                Kq, Vq = synth.to_pool(K, table, page), synth.to_pool(V, table, page)
            else:
                Kq, Vq = K.clone(), V.clone()
            sparse = ctx.append_reuse_sparse_attn(q, k_new, v_new, Kq, Vq, idx_d, paged=cache)
            torch.cuda.synchronize()
            assert np.array_equal(lens_d.cpu().numpy(), lens), "the caller's lengths must not be written"
            assert torch.equal(Kq.view(torch.int16), Kp.view(torch.int16)), "cache after append (K), append_unfused=%d" % unfused
            assert torch.equal(Vq.view(torch.int16), Vp.view(torch.int16)), "cache after append (V), append_unfused=%d" % unfused
            for b in range(B):
                n = int(lens[b]) + 1
                ref = oracle.reuse_sparse_attn(q[b:b + 1].cpu(), refs[0][b:b + 1, :, :n], refs[1][b:b + 1, :, :n], idx_h[b:b + 1])
                assert_out_close(sparse[b:b + 1].cpu().numpy(), ref, "append reuse page=%d b=%d unfused=%d" % (page, b, unfused))


@pytest.mark.parametrize("unfused", [0, 1])
def test_decode_step_append_chain(unfused):
    """Algorithm 2 with every layer's cache receiving its own new row first (paged, ragged); the
    Reuse layers write their row themselves (0) or a launch before them does (1)."""
    say("decode step with append, append_unfused=%d" % unfused)
    B, Hkv, G, d, N, k, page, L = 3, 2, 4, 128, 3000, 256, 16, 5
    policy = np.array([0, 1, 1, 0, 1], np.uint8)
    lens = np.array([N - 1, 700, 2011], np.int32)
    table = synth.page_table(B, N, page, 9)
    layers = [make(300, B, Hkv, G, d, N, layer=l) for l in range(L)]
    qs = [x[0] for x in layers]
    pools = [(synth.to_pool(x[1], table, page), synth.to_pool(x[2], table, page)) for x in layers]
    cache = binding.PagedCache(torch.from_numpy(table).to(DEV), page, N, torch.from_numpy(lens).to(DEV))
    with binding.Context(B, Hkv * G, Hkv, d, N, k) as ctx:
        ctx.set_option("append_unfused", unfused)
        outs, idx_buf = ctx.decode_step_append(policy, qs, [x[3] for x in layers], [x[4] for x in layers],
                                               [p[0] for p in pools], [p[1] for p in pools], k, paged=cache)
        torch.cuda.synchronize()
        cur = None
        for l in range(L):
            q, K, V, k_new, v_new = layers[l]
            refs = oracle_after_append(q, K, V, k_new, v_new, lens, k)
            for which in (0, 1):         # the layer's pools: exactly the appended rows changed
                want = synth.to_pool(torch.from_numpy(refs[which].view(np.int16)).view(torch.bfloat16).to(DEV), table, page)
                assert torch.equal(pools[l][which].view(torch.int16), want.view(torch.int16)), "layer %d pool %d" % (l, which)
            if policy[l] == 0:
                # the set in force: read by running the layer alone on the (already appended) pools
                _, gidx = ctx.full_attn_topk_paged(q, pools[l][0], pools[l][1],
                                                   binding.PagedCache(cache.block_table, page, N, torch.from_numpy(lens + 1).to(DEV)), k)
                torch.cuda.synchronize()
                cur = gidx.cpu().numpy()
                check_full(outs[l].cpu().numpy(), cur, refs, k, "step layer %d" % l)
            else:
                for b in range(B):
                    n = int(lens[b]) + 1
                    ref = oracle.reuse_sparse_attn(q[b:b + 1].cpu(), refs[0][b:b + 1, :, :n], refs[1][b:b + 1, :, :n], cur[b:b + 1])
                    assert_out_close(outs[l][b:b + 1].cpu().numpy(), ref, "step layer %d b=%d" % (l, b))
        assert np.array_equal(idx_buf.cpu().numpy(), cur)


def test_append_errors():
    say("append errors")
    B, Hkv, G, d, N, k = 1, 2, 4, 128, 512, 32
    q, K, V, k_new, v_new = make(5, B, Hkv, G, d, N)
    with binding.Context(B, Hkv * G, Hkv, d, N, k) as ctx:
        flat = torch.zeros(k_new.numel() + 8, dtype=torch.bfloat16, device=DEV)
        mis = flat[1:1 + k_new.numel()].view(k_new.shape)
        with pytest.raises(binding.HylraError) as e:
            ctx.append_full_attn_topk(q, mis, v_new, K, V, k)
        assert e.value.status == 1
        with pytest.raises(binding.HylraError) as e:
            ctx.append_full_attn_topk(q, k_new, v_new, K, V, N + 1)
        assert e.value.status == 1
