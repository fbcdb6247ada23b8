"""The synthetic workload generator: shapes, determinism, and the planted-set structure that
stands in for the paper's inter-layer similarity (overlap ratio, Eq. 2).  CPU only."""
import numpy as np
import torch

import oracle
from paper_2602_00777_amd import synth


def test_workload_table_matches_the_benchmark_configs():
    w = synth.WORKLOADS
    assert w["toy"].policy().tolist() == [0, 1]
    l = w["llama3_8b_32k"]
    assert (l.n_layers, l.n_q_heads, l.n_kv_heads, l.head_dim, l.batch, l.ctx_len, l.top_k) == (32, 32, 8, 128, 8, 32768, 2048)
    assert np.flatnonzero(l.policy() == 0).tolist() == [0, 1, 2, 15, 31]
    assert l.kv_bytes_per_layer() == 1 << 30
    assert np.flatnonzero(w["long_131k"].policy() == 0).tolist() == list(range(0, 32, 4))
    assert np.flatnonzero(w["serve_b32_16k"].policy() == 0).tolist() == [0, 1, 31]
    qw = w["qwen25_7b_64k"]
    assert qw.group == 7 and np.flatnonzero(qw.policy() == 0).tolist() == [0, 1, 27]
    assert [w[n].n_planted for n in ("toy", "llama3_8b_32k", "long_131k", "serve_b32_16k", "qwen25_7b_64k")] == [41, 328, 1311, 82, 655]


def test_planted_sets_carry_over():
    w = synth.scaled(synth.WORKLOADS["llama3_8b_32k"], n_layers=5, batch=1, n_kv_heads=2, n_q_heads=8, ctx_len=4000)
    p = synth.planted_positions(w)
    P = w.n_planted
    for l in range(1, 5):
        for g in range(2):
            a, b = p[l - 1][0, g], p[l][0, g]
            assert len(set(b.tolist())) == P and b.min() >= 0 and b.max() < 4000
            assert len(np.intersect1d(a, b)) == round(0.8 * P)
    q = synth.scaled(synth.WORKLOADS["qwen25_7b_64k"], n_layers=3, batch=1, ctx_len=3000)
    for layer in synth.planted_positions(q):
        assert layer[0, 0, :4].tolist() == [0, 1, 2, 3]
        assert layer.shape[-1] == q.n_planted + 4


def test_generator_is_deterministic_and_bf16():
    w = synth.scaled(synth.WORKLOADS["toy"], ctx_len=256, top_k=16)
    _, planted, a = synth.make_workload(w)
    _, _, b = synth.make_workload(w)
    for (qa, Ka, Va), (qb, Kb, Vb) in zip(a, b):
        assert qa.dtype == Ka.dtype == Va.dtype == torch.bfloat16
        assert torch.equal(qa, qb) and torch.equal(Ka, Kb) and torch.equal(Va, Vb)
    assert a[0][1].shape == (1, 2, 256, 64)


def test_planted_positions_are_what_full_attention_selects():
    """Planted rows sit about beta standard deviations above the background in group-mean score,
    so most of them (about 0.9 in expectation; small-sample noise allowed for) are among the oracle's top-k, and consecutive Full layers overlap roughly
    by the carry-over fraction of the planted set."""
    w = synth.scaled(synth.WORKLOADS["toy"], n_layers=2, ctx_len=2048, top_k=128, carry=0.5)
    _, planted, data = synth.make_workload(w)
    sets = []
    for l in range(2):
        q, K, V = data[l]
        _, idx, _ = oracle.full_attn_topk(q, K, V, w.top_k)
        sets.append(idx)
        for g in range(w.n_kv_heads):
            assert np.isin(planted[l][0, g], idx[0, g]).mean() > 0.7
    ov = np.mean([oracle.overlap(sets[0][0, g], sets[1][0, g]) for g in range(w.n_kv_heads)])
    assert 0.1 < ov < 0.6
