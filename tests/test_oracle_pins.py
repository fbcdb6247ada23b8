"""Pins for the CPU oracle: everything here checks ``oracle/`` against something that is
not the oracle itself -- hand-worked values (tests/golden), an independent pure-Python brute
force on tiny inputs, closed forms, invariants of softmax attention, and library routines
(torch SDPA / topk in fp64) as a referee.  No GPU needed.
"""
import itertools
import math
import os

import numpy as np
import pytest
import torch

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")
LN = {"LN2": math.log(2.0), "LN4": math.log(4.0), "HALF_LN2": 0.5 * math.log(2.0)}


def read_golden(name):
    out = {}
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, val = line.split(":", 1)
            rows = [[LN[t] if t in LN else float(t) for t in r.split()] for r in val.split("|")]
            out[key.strip()] = np.array(rows if len(rows) > 1 else rows[0], dtype=np.float64)
    return out


# --------------------------------------------------------------------------------------
# 1. hand-worked examples
# --------------------------------------------------------------------------------------
def test_golden_single_head():
    g = read_golden("single_head_4tok.txt")
    q = g["q"].reshape(1, 1, 4)
    K = g["K"].reshape(1, 1, 4, 4)
    V = g["V"].reshape(1, 1, 4, 4)
    out, idx, shat = oracle.full_attn_topk(q, K, V, 2, want_shat=True)
    np.testing.assert_allclose(shat[0, 0], g["scores"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(out[0, 0], g["full_out"], rtol=0, atol=1e-15)
    for k in (1, 2, 3, 4):
        _, idx, _ = oracle.full_attn_topk(q, K, V, k)
        assert idx[0, 0].tolist() == g["top%d" % k].astype(int).reshape(-1).tolist()
    for rows, key in (((1, 2), "sparse_on_1_2"), ((3,), "sparse_on_3"), ((0, 2), "sparse_on_0_2")):
        o = oracle.reuse_sparse_attn(q, K, V, np.array(rows, np.int32).reshape(1, 1, -1))
        np.testing.assert_allclose(o[0, 0], g[key], rtol=0, atol=1e-15)
    # probabilities: recover them with one-hot V
    eye = np.eye(4).reshape(1, 1, 4, 4)
    p, _, _ = oracle.full_attn_topk(q, K, eye, 1)
    np.testing.assert_allclose(p[0, 0], g["probs"], rtol=0, atol=1e-15)


def test_golden_gqa():
    g = read_golden("gqa_4tok.txt")
    q = np.stack([g["q0"], g["q1"]]).reshape(1, 2, 4)
    K = g["K"].reshape(1, 1, 4, 4)
    V = g["V"].reshape(1, 1, 4, 4)
    out, _, shat = oracle.full_attn_topk(q, K, V, 1, want_shat=True)
    np.testing.assert_allclose(shat[0, 0], g["mean_scores"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(out[0, 0], g["full_out0"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(out[0, 1], g["full_out1"], rtol=0, atol=1e-15)
    for k in (1, 2, 3):
        _, idx, _ = oracle.full_attn_topk(q, K, V, k)
        assert idx[0, 0].tolist() == g["top%d" % k].astype(int).reshape(-1).tolist()
    o = oracle.reuse_sparse_attn(q, K, V, np.array([0, 2], np.int32).reshape(1, 1, 2))
    np.testing.assert_allclose(o[0, 0], g["sparse_on_0_2_out0"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(o[0, 1], g["sparse_on_0_2_out1"], rtol=0, atol=1e-15)


def test_golden_through_bf16_entry():
    """The bf16 entry point converts bit patterns exactly: an example whose inputs are
    bf16-exact gives the same hand-worked numbers.  Scores (0,1,2,0) -> weights (1,e,e^2,1)."""
    q = torch.tensor([[[2.0, 0, 0, 0]]], dtype=torch.bfloat16)
    K = torch.tensor([[[[0.0, 0, 0, 0], [1, 0, 0, 0], [2, 0, 0, 0], [0, 0, 0, 0]]]], dtype=torch.bfloat16)
    V = torch.tensor([[[[1.0, 0, 0, 0], [0, 1, 0, 0], [1, 1, 0, 0], [0, 0, 0, 0]]]], dtype=torch.bfloat16)
    out, idx, _ = oracle.full_attn_topk(q, K, V, 3)
    e = math.e
    z = 2 + e + e * e
    np.testing.assert_allclose(out[0, 0], [(1 + e * e) / z, (e + e * e) / z, 0, 0], rtol=1e-15)
    assert idx[0, 0].tolist() == [0, 1, 2]


# --------------------------------------------------------------------------------------
# 2. independent brute force (pure Python, exact-ish sums) on tiny inputs
# --------------------------------------------------------------------------------------
def brute_full(q, K, V, k):
    B, Hq, d = q.shape
    _, Hkv, N, _ = K.shape
    G = Hq // Hkv
    out = np.zeros((B, Hq, d))
    idx = np.zeros((B, Hkv, k), np.int64)
    for b in range(B):
        for kv in range(Hkv):
            heads = [h for h in range(Hq) if h // G == kv]
            per_head = []
            for h in heads:
                s = [math.fsum(float(q[b, h, c]) * float(K[b, kv, j, c]) for c in range(d)) / math.sqrt(d)
                     for j in range(N)]
                per_head.append(s)
                top = max(s)
                e = [math.exp(x - top) for x in s]
                z = math.fsum(e)
                for c in range(d):
                    out[b, h, c] = math.fsum(e[j] * float(V[b, kv, j, c]) for j in range(N)) / z
            mean = [math.fsum(s[j] for s in per_head) / G for j in range(N)]
            order = sorted(range(N), key=lambda j: (-mean[j], j))
            idx[b, kv] = sorted(order[:k])
    return out, idx


def brute_sparse(q, K, V, idx):
    B, Hq, d = q.shape
    _, Hkv, N, _ = K.shape
    G = Hq // Hkv
    out = np.zeros((B, Hq, d))
    for b in range(B):
        for h in range(Hq):
            kv = h // G
            rows = [int(t) for t in idx[b, kv] if t >= 0]
            s = [math.fsum(float(q[b, h, c]) * float(K[b, kv, j, c]) for c in range(d)) / math.sqrt(d)
                 for j in rows]
            top = max(s)
            e = [math.exp(x - top) for x in s]
            z = math.fsum(e)
            for c in range(d):
                out[b, h, c] = math.fsum(e[i] * float(V[b, kv, j, c]) for i, j in enumerate(rows)) / z
    return out


@pytest.mark.parametrize("seed", range(6))
def test_brute_force_tiny(seed):
    rng = np.random.RandomState(seed)
    B = rng.randint(1, 3)
    Hkv = rng.randint(1, 4)
    G = rng.randint(1, 4)
    d = int(rng.choice([2, 3, 8]))
    N = rng.randint(3, 17)
    q = rng.randn(B, Hkv * G, d)
    K = rng.randn(B, Hkv, N, d)
    V = rng.randn(B, Hkv, N, d)
    for k in sorted({1, 2, N // 2 + 1, N}):
        out, idx, _ = oracle.full_attn_topk(q, K, V, k)
        bo, bi = brute_full(q, K, V, k)
        np.testing.assert_allclose(out, bo, rtol=1e-12, atol=1e-14)
        assert np.array_equal(idx, bi)
        pick = np.stack([[np.sort(rng.permutation(N)[:k]) for _ in range(Hkv)] for _ in range(B)])
        np.testing.assert_allclose(oracle.reuse_sparse_attn(q, K, V, pick),
                                   brute_sparse(q, K, V, pick), rtol=1e-12, atol=1e-14)


def test_brute_force_with_ties():
    """Integer-valued keys make many exactly tied scores; lower position must win."""
    rng = np.random.RandomState(11)
    q = rng.randint(-1, 2, size=(1, 4, 4)).astype(np.float64)
    K = rng.randint(-1, 2, size=(1, 2, 24, 4)).astype(np.float64)
    V = rng.randn(1, 2, 24, 4)
    for k in range(1, 25):
        _, idx, _ = oracle.full_attn_topk(q, K, V, k)
        _, bi = brute_full(q, K, V, k)
        assert np.array_equal(idx, bi), k


# --------------------------------------------------------------------------------------
# 3. library referee: single-query SDPA and topk in fp64
# --------------------------------------------------------------------------------------
@pytest.mark.parametrize("G,d", [(1, 16), (4, 64), (7, 32)])
def test_against_torch_sdpa_and_topk(G, d):
    torch.manual_seed(G * 100 + d)
    B, Hkv, N, k = 2, 3, 200, 17
    q = torch.randn(B, Hkv * G, d, dtype=torch.float64)
    K = torch.randn(B, Hkv, N, d, dtype=torch.float64)
    V = torch.randn(B, Hkv, N, d, dtype=torch.float64)
    out, idx, shat = oracle.full_attn_topk(q, K, V, k, want_shat=True)
    # the library's grouped-query convention: consecutive query heads share one KV head
    ref = torch.nn.functional.scaled_dot_product_attention(
        q.unsqueeze(2), K.repeat_interleave(G, dim=1), V.repeat_interleave(G, dim=1)).squeeze(2)
    np.testing.assert_allclose(out, ref.numpy(), rtol=1e-11, atol=1e-13)
    logits = torch.einsum("bhgd,bhnd->bhgn", q.view(B, Hkv, G, d), K) / math.sqrt(d)
    mean = logits.mean(dim=2)
    np.testing.assert_allclose(shat, mean.numpy(), rtol=1e-11, atol=1e-13)
    tk = torch.topk(mean, k, dim=-1).indices.sort(dim=-1).values
    assert np.array_equal(idx, tk.numpy())
    # reuse branch == SDPA over the gathered rows
    gi = tk.unsqueeze(-1).expand(-1, -1, -1, d)
    Ks, Vs = K.gather(2, gi), V.gather(2, gi)
    ref_s = torch.nn.functional.scaled_dot_product_attention(
        q.unsqueeze(2), Ks.repeat_interleave(G, dim=1), Vs.repeat_interleave(G, dim=1)).squeeze(2)
    np.testing.assert_allclose(oracle.reuse_sparse_attn(q, K, V, idx), ref_s.numpy(),
                               rtol=1e-11, atol=1e-13)


def test_explicit_scale_argument():
    rng = np.random.RandomState(5)
    q, K, V = rng.randn(1, 2, 8), rng.randn(1, 1, 30, 8), rng.randn(1, 1, 30, 8)
    a, _, sa = oracle.full_attn_topk(q, K, V, 4, scale=0.0, want_shat=True)
    b, _, sb = oracle.full_attn_topk(q, K, V, 4, scale=1.0 / math.sqrt(8), want_shat=True)
    np.testing.assert_allclose(a, b, rtol=1e-14)
    c, _, sc = oracle.full_attn_topk(q * 2.0, K, V, 4, scale=0.5 / math.sqrt(8), want_shat=True)
    np.testing.assert_allclose(a, c, rtol=1e-13)
    np.testing.assert_allclose(sa, sc, rtol=1e-13)


# --------------------------------------------------------------------------------------
# 4. invariants and closed forms
# --------------------------------------------------------------------------------------
def _rand(seed, B=2, Hkv=2, G=2, N=40, d=8):
    rng = np.random.RandomState(seed)
    return rng.randn(B, Hkv * G, d), rng.randn(B, Hkv, N, d), rng.randn(B, Hkv, N, d)


def test_weights_sum_to_one_and_constant_values():
    q, K, V = _rand(1)
    ones = np.ones_like(V)
    out, _, _ = oracle.full_attn_topk(q, K, ones * 3.25, 3)
    np.testing.assert_allclose(out, 3.25, rtol=1e-14)
    idx = np.tile(np.array([1, 5, 9], np.int32), (2, 2, 1))
    np.testing.assert_allclose(oracle.reuse_sparse_attn(q, K, ones * -2.5, idx), -2.5, rtol=1e-14)


def test_output_in_convex_hull():
    q, K, V = _rand(2)
    out, idx, _ = oracle.full_attn_topk(q, K, V, 6)
    G = 2
    for b in range(2):
        for h in range(4):
            lo, hi = V[b, h // G].min(axis=0), V[b, h // G].max(axis=0)
            assert np.all(out[b, h] >= lo - 1e-12) and np.all(out[b, h] <= hi + 1e-12)
    o = oracle.reuse_sparse_attn(q, K, V, idx)
    for b in range(2):
        for h in range(4):
            rows = V[b, h // G][idx[b, h // G]]
            assert np.all(o[b, h] >= rows.min(axis=0) - 1e-12)
            assert np.all(o[b, h] <= rows.max(axis=0) + 1e-12)


def test_full_equals_sparse_when_k_is_context_length():
    q, K, V = _rand(3)
    N = K.shape[2]
    out, idx, _ = oracle.full_attn_topk(q, K, V, N)
    assert np.array_equal(idx, np.broadcast_to(np.arange(N), idx.shape))
    np.testing.assert_allclose(oracle.reuse_sparse_attn(q, K, V, idx), out, rtol=1e-13, atol=1e-15)


def test_reuse_invariant_under_index_permutation_and_padding():
    q, K, V = _rand(4)
    rng = np.random.RandomState(0)
    idx = np.stack([[np.sort(rng.permutation(40)[:9]) for _ in range(2)] for _ in range(2)]).astype(np.int32)
    base = oracle.reuse_sparse_attn(q, K, V, idx)
    perm = idx[:, :, rng.permutation(9)]
    np.testing.assert_allclose(oracle.reuse_sparse_attn(q, K, V, perm), base, rtol=1e-13)
    padded = np.concatenate([np.full((2, 2, 3), -1, np.int32), idx, np.full((2, 2, 2), -1, np.int32)], axis=2)
    np.testing.assert_allclose(oracle.reuse_sparse_attn(q, K, V, padded), base, rtol=1e-13)


def test_cache_row_permutation_equivariance():
    q, K, V = _rand(5)
    N = K.shape[2]
    perm = np.random.RandomState(1).permutation(N)
    out, idx, _ = oracle.full_attn_topk(q, K, V, 7)
    out_p, idx_p, _ = oracle.full_attn_topk(q, K[:, :, perm], V[:, :, perm], 7)
    np.testing.assert_allclose(out_p, out, rtol=1e-12)
    # scores are distinct with probability one, so the selected SET maps through the permutation
    for b in range(2):
        for g in range(2):
            assert set(perm[idx_p[b, g]].tolist()) == set(idx[b, g].tolist())


def test_key_shift_invariance():
    """Adding one vector u to every key adds q.u/sqrt(d) to every score of a head: softmax
    and the ranking of the group mean are unchanged."""
    q, K, V = _rand(6)
    u = np.random.RandomState(2).randn(8)
    out, idx, _ = oracle.full_attn_topk(q, K, V, 5)
    out_s, idx_s, _ = oracle.full_attn_topk(q, K + u, V, 5)
    np.testing.assert_allclose(out_s, out, rtol=1e-10)
    assert np.array_equal(idx, idx_s)


def test_dominant_key_limit():
    """One key far along q: softmax collapses onto that row and it is the first pick."""
    rng = np.random.RandomState(7)
    d, N = 8, 30
    q = rng.randn(1, 1, d)
    K, V = rng.randn(1, 1, N, d), rng.randn(1, 1, N, d)
    K[0, 0, 17] = 200.0 * q[0, 0] / np.linalg.norm(q[0, 0])
    out, idx, _ = oracle.full_attn_topk(q, K, V, 1)
    np.testing.assert_allclose(out[0, 0], V[0, 0, 17], rtol=1e-9, atol=1e-12)
    assert idx[0, 0, 0] == 17


def test_two_token_closed_form():
    """Two keys: p0 = sigmoid(s0 - s1)."""
    d = 4
    q = np.array([[[1.0, -2.0, 0.5, 3.0]]])
    K = np.array([[[[0.3, 0.1, -1.0, 0.2], [-0.4, 0.6, 0.9, 0.1]]]])
    V = np.array([[[[1.0, 10.0, 100.0, 1000.0], [2.0, 20.0, 200.0, 2000.0]]]])
    s = (K[0, 0] @ q[0, 0]) / math.sqrt(d)
    p0 = 1.0 / (1.0 + math.exp(s[1] - s[0]))
    out, idx, _ = oracle.full_attn_topk(q, K, V, 1)
    np.testing.assert_allclose(out[0, 0], p0 * V[0, 0, 0] + (1 - p0) * V[0, 0, 1], rtol=1e-14)
    assert idx[0, 0, 0] == (0 if s[0] >= s[1] else 1)


def test_group_of_one_equals_per_head_algorithm():
    """G = 1: each head ranks by its own scores (the paper's single-head statement)."""
    q, K, V = _rand(8, Hkv=3, G=1)
    out, idx, shat = oracle.full_attn_topk(q, K, V, 5, want_shat=True)
    for h in range(3):
        o1, i1, s1 = oracle.full_attn_topk(q[:, h:h + 1], K[:, h:h + 1], V[:, h:h + 1], 5, want_shat=True)
        np.testing.assert_array_equal(o1[:, 0], out[:, h])
        np.testing.assert_array_equal(i1[:, 0], idx[:, h])


def test_grouping_is_consecutive_heads():
    """Heads 0..G-1 read KV head 0, the next G read KV head 1: swapping the two KV heads
    must swap the two halves of the output."""
    q, K, V = _rand(9, B=1, Hkv=2, G=3)
    out, idx, _ = oracle.full_attn_topk(q, K, V, 4)
    qs = np.concatenate([q[:, 3:], q[:, :3]], axis=1)
    out_s, idx_s, _ = oracle.full_attn_topk(qs, K[:, ::-1], V[:, ::-1], 4)
    np.testing.assert_array_equal(out_s[:, :3], out[:, 3:])
    np.testing.assert_array_equal(out_s[:, 3:], out[:, :3])
    np.testing.assert_array_equal(idx_s[:, 0], idx[:, 1])


def test_full_output_is_dense_not_topk_restricted():
    """The Full branch attends over ALL rows; only the Reuse branch is restricted."""
    q, K, V = _rand(10)
    out, idx, _ = oracle.full_attn_topk(q, K, V, 5)
    sparse = oracle.reuse_sparse_attn(q, K, V, idx)
    assert np.max(np.abs(out - sparse)) > 1e-3


# --------------------------------------------------------------------------------------
# 5. the layer chain (Alg. 2 outer loop)
# --------------------------------------------------------------------------------------
def _layers(L, seed, **kw):
    data = [_rand(seed + l, **kw) for l in range(L)]
    return [x[0] for x in data], [x[1] for x in data], [x[2] for x in data]


def test_chain_all_full_equals_independent_calls():
    qs, Ks, Vs = _layers(3, 20)
    outs, idx, trace = oracle.decode_step([0, 0, 0], qs, Ks, Vs, 6)
    for l in range(3):
        o, i, _ = oracle.full_attn_topk(qs[l], Ks[l], Vs[l], 6)
        np.testing.assert_array_equal(outs[l], o)
        np.testing.assert_array_equal(trace[l], i)
    np.testing.assert_array_equal(idx, trace[2])


def test_chain_reuse_inherits_from_last_full_layer():
    qs, Ks, Vs = _layers(5, 30)
    policy = [0, 1, 1, 0, 1]
    outs, idx, trace = oracle.decode_step(policy, qs, Ks, Vs, 6)
    _, i0, _ = oracle.full_attn_topk(qs[0], Ks[0], Vs[0], 6)
    _, i3, _ = oracle.full_attn_topk(qs[3], Ks[3], Vs[3], 6)
    for l, src in ((0, i0), (1, i0), (2, i0), (3, i3), (4, i3)):
        np.testing.assert_array_equal(trace[l], src)
    for l, src in ((1, i0), (2, i0), (4, i3)):
        np.testing.assert_array_equal(outs[l], oracle.reuse_sparse_attn(qs[l], Ks[l], Vs[l], src))
    np.testing.assert_array_equal(idx, i3)
    assert not np.array_equal(i0, i3)


def test_chain_rejects_reuse_at_layer_zero():
    qs, Ks, Vs = _layers(2, 40)
    with pytest.raises(RuntimeError):
        oracle.decode_step([1, 0], qs, Ks, Vs, 4)


def test_jump3_and_full_baseline_policies_are_plain_policy_vectors():
    """The paper's two baselines: all-Full, and a fixed stride of 3 between Full layers."""
    qs, Ks, Vs = _layers(7, 50)
    jump3 = [0 if l % 3 == 0 else 1 for l in range(7)]
    _, _, trace = oracle.decode_step(jump3, qs, Ks, Vs, 5)
    for l in range(7):
        src = 3 * (l // 3)
        np.testing.assert_array_equal(trace[l], trace[src])


# --------------------------------------------------------------------------------------
# 6. overlap ratio (Eq. 2) and the planted-set statistics of the synthetic inputs
# --------------------------------------------------------------------------------------
def test_overlap_ratio():
    assert oracle.overlap([1, 2, 3, 4], [3, 4, 5, 6]) == 0.5
    assert oracle.overlap([1, 2, 3, 4], [4, 3, 2, 1]) == 1.0
    assert oracle.overlap([1, 2], [3, 4]) == 0.0


def test_argument_errors():
    q, K, V = _rand(60)
    with pytest.raises(RuntimeError):
        oracle.full_attn_topk(q, K, V, 0)
    with pytest.raises(RuntimeError):
        oracle.full_attn_topk(q, K, V, K.shape[2] + 1)
    bad = np.full((2, 2, 3), K.shape[2], np.int32)
    with pytest.raises(RuntimeError):
        oracle.reuse_sparse_attn(q, K, V, bad)


# --------------------------------------------------------------------------------------
# 7. block-level variant (block TopK, block reuse)
# --------------------------------------------------------------------------------------
def test_block_variant_hand_worked():
    """The single-head golden example with blocks of 2: token scores (0, ln2, ln4, 0) give block
    scores (ln2, ln4): top-1 block is block 1 = tokens {2,3}, weights (4,1)/5."""
    g = read_golden("single_head_4tok.txt")
    q = g["q"].reshape(1, 1, 4)
    K = g["K"].reshape(1, 1, 4, 4)
    V = g["V"].reshape(1, 1, 4, 4)
    out, bidx, bs = oracle.full_attn_topk_blocks(q, K, V, 2, 1, want_bscore=True)
    np.testing.assert_allclose(out[0, 0], g["full_out"], rtol=0, atol=1e-15)     # dense output unchanged
    np.testing.assert_allclose(bs[0, 0], [math.log(2.0), math.log(4.0)], rtol=0, atol=1e-15)
    assert bidx[0, 0].tolist() == [1]
    o = oracle.reuse_block_attn(q, K, V, bidx, 2)
    np.testing.assert_allclose(o[0, 0], [0.8, 0.8, 0, 0], rtol=0, atol=1e-15)   # (4*V2 + 1*V3)/5
    _, both, _ = oracle.full_attn_topk_blocks(q, K, V, 2, 2)
    assert both[0, 0].tolist() == [0, 1]
    np.testing.assert_allclose(oracle.reuse_block_attn(q, K, V, both, 2)[0, 0], g["full_out"], atol=1e-15)


def test_block_variant_against_brute_force_and_token_level():
    rng = np.random.RandomState(70)
    B, Hkv, G, d, N = 2, 2, 3, 8, 29          # 29 is not a multiple of the block sizes below
    q, K, V = rng.randn(B, Hkv * G, d), rng.randn(B, Hkv, N, d), rng.randn(B, Hkv, N, d)
    dense, _, shat = oracle.full_attn_topk(q, K, V, 1, want_shat=True)
    for block in (1, 4, 5, 29, 40):
        nblk = -(-N // block)
        for kb in sorted({1, nblk // 2 + 1, nblk}):
            out, bidx, bs = oracle.full_attn_topk_blocks(q, K, V, block, kb, want_bscore=True)
            np.testing.assert_array_equal(out, dense)
            for b in range(B):
                for g in range(Hkv):
                    ref = [max(shat[b, g, c * block:min(N, (c + 1) * block)]) for c in range(nblk)]
                    np.testing.assert_allclose(bs[b, g], ref, rtol=0, atol=0)
                    order = sorted(range(nblk), key=lambda c: (-ref[c], c))
                    assert bidx[b, g].tolist() == sorted(order[:kb])
            # block reuse == token reuse over the tokens of the blocks
            tok = np.full((B, Hkv, kb * block), -1, np.int32)
            for b in range(B):
                for g in range(Hkv):
                    t = [c * block + j for c in bidx[b, g] for j in range(block) if c * block + j < N]
                    tok[b, g, :len(t)] = t
            np.testing.assert_allclose(oracle.reuse_block_attn(q, K, V, bidx, block),
                                       oracle.reuse_sparse_attn(q, K, V, tok), rtol=1e-13, atol=1e-15)
            if block == 1:   # blocks of one token are the token-level algorithm
                _, idx, _ = oracle.full_attn_topk(q, K, V, kb)
                np.testing.assert_array_equal(bidx, idx)
    # padding blocks are skipped; all blocks selected = dense attention
    _, allb, _ = oracle.full_attn_topk_blocks(q, K, V, 4, 8)
    padded = np.concatenate([np.full((B, Hkv, 2), -1, np.int32), allb], axis=2)
    np.testing.assert_allclose(oracle.reuse_block_attn(q, K, V, padded, 4), dense, rtol=1e-13, atol=1e-15)
    with pytest.raises(RuntimeError):
        oracle.full_attn_topk_blocks(q, K, V, 4, 9)
    with pytest.raises(RuntimeError):
        oracle.reuse_block_attn(q, K, V, np.full((B, Hkv, 1), 8, np.int32), 4)


def test_block_variant_ties_go_to_lower_block():
    q = np.zeros((1, 1, 4)); q[0, 0, 0] = 2.0
    K = np.zeros((1, 1, 8, 4)); K[0, 0, :, 0] = [1, 0, 0, 1, 0, 0, 1, 0]     # blocks of 2: scores 1,1,0,1
    V = np.random.RandomState(1).randn(1, 1, 8, 4)
    _, bidx, bs = oracle.full_attn_topk_blocks(q, K, V, 2, 2, want_bscore=True)
    assert bs[0, 0].tolist() == [1.0, 1.0, 0.0, 1.0]
    assert bidx[0, 0].tolist() == [0, 1]


# ---- offline profiling step: overlap counts (Eq. 2) and policy search (Algorithm 1) ----------

def test_overlap_counts_against_python_sets():
    """Pooled |S_i ∩ S_j| against Python set intersections; padding (-1) is no member."""
    rng = np.random.RandomState(3)
    L, B, H, k, N = 5, 2, 3, 20, 60
    idx = [np.stack([[np.sort(rng.permutation(N)[:k]) for _ in range(H)] for _ in range(B)]).astype(np.int32)
           for _ in range(L)]
    idx[2][:, :, -4:] = -1
    counts = oracle.overlap_counts(idx)
    for i in range(L):
        for j in range(L):
            if i > j:
                assert counts[i, j] == 0
                continue
            want = sum(len((set(idx[i][b, h].tolist()) - {-1}) & set(idx[j][b, h].tolist()))
                       for b in range(B) for h in range(H))
            assert counts[i, j] == want
    M = oracle.similarity_matrix(counts)
    assert np.allclose(np.diag(M), 1.0)
    assert counts[2, 2] == B * H * (k - 4)
    # one set per layer: the pooled ratio is the pairwise overlap ratio of Eq. 2
    one = [a[:1, :1] for a in idx[:2]]
    assert oracle.similarity_matrix(oracle.overlap_counts(one))[0, 1] == oracle.overlap(one[0], one[1])


def _policy_value(M, policy, theta):
    """(C, S) of a policy vector under the path rules of Algorithm 1, or None if a reused layer
    falls below the threshold."""
    src, C, S = 0, 0, 0.0
    for j, a in enumerate(policy):
        if a == 0:
            src, C = j, C + 1
        elif M[src, j] < theta:
            return None
        S += M[src, j]
    return C, S


def _brute_force_policy(M, theta):
    L = M.shape[0]
    best = None
    for bits in itertools.product((0, 1), repeat=L - 1):
        pol = (0,) + bits
        v = _policy_value(M, pol, theta)
        if v is None:
            continue
        if best is None or v[0] < best[0][0] or (v[0] == best[0][0] and v[1] > best[0][1]):
            best = (v, pol)
    return best


@pytest.mark.parametrize("seed", range(8))
def test_policy_search_against_exhaustive_search(seed):
    """Algorithm 1 against all 2^(L-1) policies on random similarity matrices (generic values:
    no ties, so the optimal policy is unique)."""
    rng = np.random.RandomState(seed)
    L = 4 + seed
    M = np.triu(rng.uniform(0.2, 1.0, size=(L, L)))
    np.fill_diagonal(M, 1.0)
    for theta in (0.0, 0.4, 0.7, 0.95):
        pol, C, S = oracle.policy_search(M, theta)
        (bc, bs), bpol = _brute_force_policy(M, theta)
        assert C == bc and S == pytest.approx(bs, abs=1e-12)
        assert tuple(pol.tolist()) == bpol
        assert _policy_value(M, pol, theta) == (C, pytest.approx(S, abs=1e-12))


def test_policy_search_closed_forms():
    L = 10
    ones = np.triu(np.ones((L, L)))
    # threshold above every off-diagonal entry: every layer is Full
    M = np.triu(np.full((L, L), 0.5)); np.fill_diagonal(M, 1.0)
    pol, C, S = oracle.policy_search(M, 0.6)
    assert pol.tolist() == [0] * L and C == L and S == L
    # threshold below everything: only layer 0 is Full
    pol, C, S = oracle.policy_search(M, 0.1)
    assert pol.tolist() == [0] + [1] * (L - 1) and C == 1 and S == pytest.approx(1 + 0.5 * (L - 1))
    # similarity above the threshold only up to two layers back: a Full layer every third
    # layer (the "Jump3" baseline of the paper's evaluation), and no cheaper policy exists
    band = np.zeros((L, L))
    for i in range(L):
        for j in range(i, L):
            band[i, j] = 1.0 if i == j else (0.9 - 0.1 * (j - i) if j - i <= 2 else 0.1)
    pol, C, S = oracle.policy_search(band, 0.5)
    assert C == math.ceil(L / 3)
    assert _policy_value(band, pol, 0.5) == (C, pytest.approx(S))
    assert all(sum(1 for _ in grp) <= 2 for key, grp in itertools.groupby(pol.tolist()) if key == 1)
    # all similarities equal to 1: every policy with one Full layer ties; the value is what is fixed
    pol, C, S = oracle.policy_search(ones, 1.0)
    assert C == 1 and S == L and pol[0] == 0


# --------------------------------------------------------------------------------------
# 8. index-guided prefetch (compacted caches) and the decode-time cache update
# --------------------------------------------------------------------------------------
def test_gather_rows_hand_written():
    """Three rows of two columns, one head: entries (2, padding, 0, one past the cache)."""
    K = np.array([[[[1., 2.], [3., 4.], [5., 6.]]]])
    V = -K
    idx = np.array([[[2, -1, 0, 3]]], np.int32)
    Ks, Vs, ic = oracle.gather_rows(K, V, idx)
    assert Ks.tolist() == [[[[5., 6.], [0., 0.], [1., 2.], [0., 0.]]]]
    assert Vs.tolist() == [[[[-5., -6.], [0., 0.], [-1., -2.], [0., 0.]]]]
    assert ic.tolist() == [[[0, -1, 2, -1]]]


def test_gather_rows_against_fancy_indexing_and_reuse_identity():
    q, K, V = _rand(21, B=2, Hkv=3, G=2, N=50, d=8)
    rng = np.random.RandomState(5)
    idx = np.stack([[rng.permutation(50)[:12] for _ in range(3)] for _ in range(2)]).astype(np.int32)
    Ks, Vs, ic = oracle.gather_rows(K, V, idx)
    assert np.array_equal(Ks, np.take_along_axis(K, idx[..., None].astype(np.int64), axis=2))
    assert np.array_equal(Vs, np.take_along_axis(V, idx[..., None].astype(np.int64), axis=2))
    assert np.array_equal(ic, np.broadcast_to(np.arange(12), ic.shape))
    # with padding and out-of-range entries: attention over the compacted cache with the compact
    # set is attention over the source cache with the original set
    idx[:, :, ::4] = -1
    idx[:, :, 5] = 50
    Ks, Vs, ic = oracle.gather_rows(K, V, idx)
    assert np.all(ic[:, :, ::4] == -1) and np.all(ic[:, :, 5] == -1) and np.all(Ks[:, :, 5] == 0)
    want = oracle.reuse_sparse_attn(q, K, V, np.where(idx >= 50, -1, idx))
    np.testing.assert_allclose(oracle.reuse_sparse_attn(q, Ks, Vs, ic), want, rtol=1e-13, atol=1e-15)
    # bf16 bit patterns keep their element type and their bits
    Kb = (rng.randint(0, 1 << 16, size=K.shape)).astype(np.uint16)
    Ksb, _, _ = oracle.gather_rows(Kb, Kb, idx)
    assert Ksb.dtype == np.uint16 and np.array_equal(Ksb[0, 1, 1], Kb[0, 1, idx[0, 1, 1]])


def test_gather_blocks_hand_written_and_identity():
    """Five rows in blocks of two (the last block has one row): blocks (2, 0, padding)."""
    K = np.arange(10, dtype=np.float64).reshape(1, 1, 5, 2) + 1.0
    V = 10.0 * K
    bidx = np.array([[[2, 0, -1]]], np.int32)
    Ks, Vs, ic = oracle.gather_blocks(K, V, bidx, 2)
    assert Ks[0, 0].tolist() == [[9., 10.], [0., 0.], [1., 2.], [3., 4.], [0., 0.], [0., 0.]]
    assert np.array_equal(Vs, 10.0 * Ks)
    assert ic.tolist() == [[[0, -1, 2, 3, -1, -1]]]
    # a shorter sequence: rows at or past its length are no rows
    _, _, ic4 = oracle.gather_blocks(K, V, np.array([[[1, 0]]], np.int32), 2, lens=[3])
    assert ic4.tolist() == [[[0, -1, 2, 3]]]
    # block of one row is the row-level gather
    idx = np.array([[[4, -1, 1]]], np.int32)
    for a, b in zip(oracle.gather_blocks(K, V, idx, 1), oracle.gather_rows(K, V, idx)):
        assert np.array_equal(a, b)
    # attention over the compacted cache equals block attention over the source cache
    q, K, V = _rand(22, B=2, Hkv=2, G=3, N=43, d=8)
    rng = np.random.RandomState(6)
    for block in (4, 5, 16):
        nblk = -(-43 // block)
        kb = min(3, nblk)
        bidx = np.stack([[rng.permutation(nblk)[:kb] for _ in range(2)] for _ in range(2)]).astype(np.int32)
        bidx[0, 0, 0] = -1
        Ks, Vs, ic = oracle.gather_blocks(K, V, bidx, block)
        want = oracle.reuse_block_attn(q, K, V, bidx, block)
        np.testing.assert_allclose(oracle.reuse_sparse_attn(q, Ks, Vs, ic), want, rtol=1e-13, atol=1e-15)


def test_append_rows_then_attend_equals_attention_on_the_longer_cache():
    # hand-written: the new rows land at each sequence's own length, nothing else moves
    K = np.zeros((2, 1, 4, 2)); V = np.zeros((2, 1, 4, 2))
    K2, V2, n2 = oracle.append_rows(K, V, np.array([[[1., 2.]], [[3., 4.]]]), np.array([[[5., 6.]], [[7., 8.]]]), [3, 0])
    assert n2.tolist() == [4, 1]
    assert K2[0, 0].tolist() == [[0., 0.], [0., 0.], [0., 0.], [1., 2.]] and K2[1, 0].tolist() == [[3., 4.], [0., 0.], [0., 0.], [0., 0.]]
    assert V2[0, 0, 3].tolist() == [5., 6.] and V2[1, 0, 0].tolist() == [7., 8.] and not K.any()
    with pytest.raises(ValueError):
        oracle.append_rows(K, V, np.zeros((2, 1, 2)), np.zeros((2, 1, 2)), [4, 0])
    # a cache of N + 1 rows, its last row handed over as the new token
    q, K, V = _rand(23, B=2, Hkv=2, G=2, N=31, d=8)
    Kc, Vc = K.copy(), V.copy()
    Kc[:, :, 30] = 99.0          # stale contents of the free row must not matter
    Vc[:, :, 30] = -99.0
    K2, V2, n2 = oracle.append_rows(Kc, Vc, K[:, :, 30], V[:, :, 30], [30, 30])
    assert np.array_equal(K2, K) and np.array_equal(V2, V) and n2.tolist() == [31, 31]
    a, ia, _ = oracle.full_attn_topk(q, K2, V2, 9)
    b, ib, _ = oracle.full_attn_topk(q, K, V, 9)
    assert np.array_equal(a, b) and np.array_equal(ia, ib)
