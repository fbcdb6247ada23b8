"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.

test_full_size_decode_step_all_pairs: the benchmarked call itself, hylra_decode_step with the
workload's own policy at full shape, every layer and every (batch, KV head) pair against the
oracle (tests/step_check.py); the same for the append, paged and per-sequence-length forms of
the step.  The per-call tests below them run the first Full and the first Reuse layer through
the single-layer entry points, token-level and block-level, again on every pair."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_00777_amd import binding, synth
from tests.parity import assert_idx_valid, assert_out_close

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.timeout(600)
@pytest.mark.parametrize("name", ["llama3_8b_32k", "long_131k", "serve_b32_16k", "qwen25_7b_64k"])
def test_full_size_decode_step_all_pairs(name):
    from tests.step_check import check_step

    print("[case] full size decode step, all layers, all pairs: %s" % name, flush=True)
    w = synth.WORKLOADS[name]
    policy = w.policy()
    planted = synth.planted_positions(w)
    data = [synth.make_layer(w, l, planted[l], DEV) for l in range(w.n_layers)]
    qs, Ks, Vs = [x[0] for x in data], [x[1] for x in data], [x[2] for x in data]
    del data
    with binding.Context(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ctx_len, w.top_k) as ctx:
        run, outs, idx_buf = ctx.prepare_step(policy, qs, Ks, Vs, w.top_k)
        run()
        run()                    # the benchmark times repeated steps on one context
        torch.cuda.synchronize()
        res = check_step(ctx, policy, qs, Ks, Vs, w.top_k, outs, idx_buf,
                         say=lambda m: print("  " + m, flush=True))
    print("  %s" % res, flush=True)
    assert res["layers"] == w.n_layers and res["pairs"] == w.n_layers * w.batch * w.n_kv_heads


@pytest.mark.timeout(600)
@pytest.mark.parametrize("name", ["llama3_8b_32k", "long_131k", "qwen25_7b_64k"])
def test_full_size_decode_step_append_all_pairs(name):
    """hylra_decode_step_append at full shape: the caches start with another row at position
    N - 1, the step receives the true rows as k_new / v_new (every layer its own), and must leave
    the caches exactly as they were drawn and give the outputs of a step over them -- every
    layer and every pair against the oracle.  The Reuse layers write their row inside their own
    launch (merging by packets at the small-batch shapes), the Full layers with a launch before."""
    from tests.step_check import check_step

    print("[case] full size decode step with append, all layers, all pairs: %s" % name, flush=True)
    w = synth.WORKLOADS[name]
    policy = w.policy()
    planted = synth.planted_positions(w)
    N = w.ctx_len
    qs, Ks, Vs, k_new, v_new = [], [], [], [], []
    for l in range(w.n_layers):
        q, K, V = synth.make_layer(w, l, planted[l], DEV)
        # the token's key is pushed along the group's mean query, so that every set names row N - 1
        qm = q.view(w.batch, w.n_kv_heads, w.group, w.head_dim).float().mean(2)
        K[:, :, N - 1, :] = (K[:, :, N - 1, :].float() + 3.0 * qm).to(torch.bfloat16)
        k_new.append(K[:, :, N - 1, :].clone()), v_new.append(V[:, :, N - 1, :].clone())
        K[:, :, N - 1, :] = 7.0                    # what the append must replace
        V[:, :, N - 1, :] = -3.0
        qs.append(q), Ks.append(K), Vs.append(V)
    with binding.Context(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, N, w.top_k) as ctx:
        run, outs, idx_buf = ctx.prepare_step_append(policy, qs, k_new, v_new, Ks, Vs, w.top_k)
        run()
        run()
        torch.cuda.synchronize()
        for l in range(w.n_layers):
            assert torch.equal(Ks[l][:, :, N - 1, :].view(torch.int16), k_new[l].view(torch.int16)), "layer %d: K row" % l
            assert torch.equal(Vs[l][:, :, N - 1, :].view(torch.int16), v_new[l].view(torch.int16)), "layer %d: V row" % l
        if w.batch * w.n_kv_heads <= 16:
            assert ctx.get_info("last_reuse_merge") == 2
        assert bool((idx_buf == N - 1).any(dim=2).all()), "the new row is not in every index set"
        res = check_step(ctx, policy, qs, Ks, Vs, w.top_k, outs, idx_buf,
                         say=lambda m: print("  " + m, flush=True))
    print("  %s" % res, flush=True)
    assert res["layers"] == w.n_layers and res["pairs"] == w.n_layers * w.batch * w.n_kv_heads


@pytest.mark.timeout(600)
@pytest.mark.parametrize("name,page,ragged", [("llama3_8b_32k", 16, False), ("llama3_8b_32k", 16, True), ("long_131k", 64, False)])
def test_full_size_paged_step_against_contiguous_step(name, page, ragged):
    """hylra_decode_step_paged at full shape on pools scattered by a random block table (and with
    per-sequence lengths): with equal lengths it must select the sets of the contiguous step
    (which the test above checks against the oracle on every pair) and give its Reuse outputs
    bit for bit and its Full outputs to the last bits; with lengths, the step over the
    contiguous cache with the same lengths is the reference, and is itself checked against the
    oracle on every layer and pair, each sequence on the rows it has."""
    print("[case] full size paged step %s page=%d ragged=%s" % (name, page, ragged), flush=True)
    w = synth.WORKLOADS[name]
    policy = w.policy()
    planted = synth.planted_positions(w)
    N = w.ctx_len
    table = synth.page_table(w.batch, N, page, w.seed)
    lens = synth.ragged_lengths(w.batch, N, w.seed) if ragged else None
    lens_d = torch.from_numpy(lens).to(DEV) if ragged else None
    qs, Ks, Vs, Kp, Vp = [], [], [], [], []
    for l in range(w.n_layers):
        q, K, V = synth.make_layer(w, l, planted[l], DEV)
        qs.append(q), Ks.append(K), Vs.append(V)
        Kp.append(synth.to_pool(K, table, page)), Vp.append(synth.to_pool(V, table, page))
    flat = binding.PagedCache(None, 0, N, lens_d) if ragged else None
    paged = binding.PagedCache(torch.from_numpy(table).to(DEV), page, N, lens_d)
    with binding.Context(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, N, w.top_k) as ctx:
        run, outs, idx_buf = ctx.prepare_step(policy, qs, Ks, Vs, w.top_k, paged=flat)
        run()
        torch.cuda.synchronize()
        if ragged:               # the reference step itself, every layer and pair against the oracle
            from tests.step_check import check_step
            res = check_step(ctx, policy, qs, Ks, Vs, w.top_k, outs, idx_buf, lens=lens)
            print("  %s" % res, flush=True)
            assert res["layers"] == w.n_layers
        want = [o.clone() for o in outs]
        want_idx = idx_buf.clone()
        run, outs, idx_buf = ctx.prepare_step(policy, qs, Kp, Vp, w.top_k, paged=paged)
        run()
        run()
        torch.cuda.synchronize()
    assert torch.equal(idx_buf, want_idx), "index sets differ"
    for l in range(w.n_layers):
        if policy[l] == synth.REUSE:
            assert torch.equal(outs[l], want[l]), "Reuse layer %d differs" % l
        else:
            err = (outs[l] - want[l]).abs().max().item() / want[l].abs().max().item()
            assert err < 1e-5, "Full layer %d differs by %.2e" % (l, err)


@pytest.mark.parametrize("name", ["llama3_8b_32k", "long_131k", "serve_b32_16k", "qwen25_7b_64k"])
def test_full_size_full_then_reuse(name):
    print("[case] full size %s" % name, flush=True)
    w = synth.WORKLOADS[name]
    full_l = int(np.flatnonzero(w.policy() == synth.FULL)[0])
    reuse_l = int(np.flatnonzero(w.policy() == synth.REUSE)[0])
    planted = synth.planted_positions(synth.scaled(w, n_layers=reuse_l + 1))
    G, d, N, k = w.group, w.head_dim, w.ctx_len, w.top_k
    with binding.Context(w.batch, w.n_q_heads, w.n_kv_heads, d, N, k) as ctx:
        q, K, V = synth.make_layer(w, full_l, planted[full_l], DEV)
        out, idx = ctx.full_attn_topk(q, K, V, k)
        torch.cuda.synchronize()
        out_h, idx_h = out.cpu().numpy(), idx.cpu().numpy()
        # any-size properties, all pairs
        assert np.all(np.isfinite(out_h))
        assert idx_h.min() >= 0 and idx_h.max() < N
        assert np.all(np.diff(idx_h.astype(np.int64), axis=-1) > 0)
        ref_out, ref_idx, shat = oracle.full_attn_topk(q.cpu(), K.cpu(), V.cpu(), k, want_shat=True)
        assert_out_close(out_h, ref_out, "%s full out" % name)
        assert_idx_valid(idx_h, shat, k, "%s idx" % name, exact_ref=ref_idx)
        del q, K, V, shat
        # the Reuse layer on the set the Full layer just produced
        q, K, V = synth.make_layer(w, reuse_l, planted[reuse_l], DEV)
        out2 = ctx.reuse_sparse_attn(q, K, V, idx)
        torch.cuda.synchronize()
        out2_h = out2.cpu().numpy()
        assert np.all(np.isfinite(out2_h))
        ref = oracle.reuse_sparse_attn(q.cpu(), K.cpu(), V.cpu(), idx_h)
        assert_out_close(out2_h, ref, "%s reuse out" % name)
    # the planted positions are what the selection finds (statistical sanity of the workload)
    hit = np.mean([np.isin(planted[full_l][b, g], idx_h[b, g]).mean() for b in range(w.batch) for g in range(w.n_kv_heads)])
    assert hit > 0.6, hit


@pytest.mark.parametrize("name,block", [("llama3_8b_32k", 128), ("long_131k", 16), ("long_131k", 2)])
def test_full_size_block_variant(name, block):
    """The block-level variant at full shape: block TopK then block reuse, every pair."""
    print("[case] full size blocks %s block=%d" % (name, block), flush=True)
    w = synth.WORKLOADS[name]
    full_l = int(np.flatnonzero(w.policy() == synth.FULL)[0])
    reuse_l = int(np.flatnonzero(w.policy() == synth.REUSE)[0])
    planted = synth.planted_positions(synth.scaled(w, n_layers=reuse_l + 1))
    G, d, N, kb = w.group, w.head_dim, w.ctx_len, w.top_k // block
    nblk = -(-N // block)
    with binding.Context(w.batch, w.n_q_heads, w.n_kv_heads, d, N, w.top_k) as ctx:
        q, K, V = synth.make_layer(w, full_l, planted[full_l], DEV)
        out, bidx = ctx.full_attn_topk_blocks(q, K, V, block, kb)
        torch.cuda.synchronize()
        out_h, bidx_h = out.cpu().numpy(), bidx.cpu().numpy()
        assert np.all(np.isfinite(out_h))
        assert bidx_h.min() >= 0 and bidx_h.max() < nblk
        assert np.all(np.diff(bidx_h.astype(np.int64), axis=-1) > 0)
        ref_out, ref_bidx, bs = oracle.full_attn_topk_blocks(q.cpu(), K.cpu(), V.cpu(), block, kb, want_bscore=True)
        assert_out_close(out_h, ref_out, "%s full out" % name)
        assert_idx_valid(bidx_h, bs, kb, "%s bidx" % name, exact_ref=ref_bidx)
        del q, K, V
        q, K, V = synth.make_layer(w, reuse_l, planted[reuse_l], DEV)
        out2 = ctx.reuse_block_attn(q, K, V, bidx, block)
        torch.cuda.synchronize()
        out2_h = out2.cpu().numpy()
        assert np.all(np.isfinite(out2_h))
        ref = oracle.reuse_block_attn(q.cpu(), K.cpu(), V.cpu(), bidx_h, block)
        assert_out_close(out2_h, ref, "%s reuse out" % name)
