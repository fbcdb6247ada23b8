"""The entry point that allocates nothing (hylra_reuse_sparse_attn_static) against the
context-owning entry point it is a variant of, through the C ABI: two calls in a row on one
GPU, the second with a smaller input, each checked against hylra_reuse_sparse_attn and the
oracle under the output rule of tests/parity.py."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_00777_amd import binding
from tests.parity import assert_out_close

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def case(seed, B, Hkv, G, d, N, k):
    gen = torch.Generator().manual_seed(seed)
    q = torch.randn((B, Hkv * G, d), generator=gen).to(torch.bfloat16)
    K = torch.randn((B, Hkv, N, d), generator=gen).to(torch.bfloat16)
    V = torch.randn((B, Hkv, N, d), generator=gen).to(torch.bfloat16)
    rng = np.random.RandomState(seed)
    idx = np.stack([[np.sort(rng.permutation(N)[:k]) for _ in range(Hkv)] for _ in range(B)]).astype(np.int32)
    idx[:, :, ::7] = -1                 # padding entries
    return q, K, V, idx


def test_static_entry_matches_context_entry_twice_in_a_row():
    shapes = [(11, 4, 4, 4, 128, 5000, 2048), (12, 2, 2, 4, 128, 900, 100)]     # the second is smaller
    for n, (seed, B, Hkv, G, d, N, k) in enumerate(shapes):
        print("[case] static reuse call %d: B=%d Hkv=%d G=%d d=%d N=%d k=%d" % (n, B, Hkv, G, d, N, k), flush=True)
        q, K, V, idx = case(seed, B, Hkv, G, d, N, k)
        qd, Kd, Vd, idd = q.to(DEV), K.to(DEV), V.to(DEV), torch.from_numpy(idx).to(DEV)
        out = torch.full(q.shape, float("nan"), dtype=torch.float32, device=DEV)
        binding.reuse_sparse_attn_static(qd, Kd, Vd, idd, out)
        torch.cuda.synchronize()
        with binding.Context(B, Hkv * G, Hkv, d, N, k) as ctx:
            want = ctx.reuse_sparse_attn(qd, Kd, Vd, idd)
            torch.cuda.synchronize()
        got, want = out.cpu().numpy(), want.cpu().numpy()
        assert_out_close(got, want, "static vs context entry, call %d" % n)
        assert_out_close(got, oracle.reuse_sparse_attn(q, K, V, idx), "static vs oracle, call %d" % n)
        print("  bit-equal to the context entry: %s" % np.array_equal(got, want), flush=True)


def test_static_entry_head_dim_64_and_limits():
    print("[case] static reuse d=64, then a shape beyond the static workspace", flush=True)
    q, K, V, idx = case(13, 2, 2, 2, 64, 1500, 300)
    qd, Kd, Vd, idd = q.to(DEV), K.to(DEV), V.to(DEV), torch.from_numpy(idx).to(DEV)
    out = torch.empty(q.shape, dtype=torch.float32, device=DEV)
    binding.reuse_sparse_attn_static(qd, Kd, Vd, idd, out)
    torch.cuda.synchronize()
    assert_out_close(out.cpu().numpy(), oracle.reuse_sparse_attn(q, K, V, idx), "static d=64 vs oracle")
    # more (batch, KV head) pairs than the array has counters for: refused before any launch
    B, Hkv = 300, 8
    qb = torch.zeros((B, Hkv, 64), dtype=torch.bfloat16, device=DEV)
    Kb = torch.zeros((B, Hkv, 16, 64), dtype=torch.bfloat16, device=DEV)
    ib = torch.zeros((B, Hkv, 4), dtype=torch.int32, device=DEV)
    ob = torch.full(qb.shape, 7.0, dtype=torch.float32, device=DEV)
    with pytest.raises(binding.HylraError) as e:
        binding.reuse_sparse_attn_static(qb, Kb, Kb, ib, ob)
    assert e.value.status == 3 and "static workspace" in str(e.value)
    torch.cuda.synchronize()
    assert torch.all(ob == 7.0)
