"""GPU parity of the index-guided prefetch: the gather of the selected rows (byte work:
bit-exact against the oracle's plain definition), from device memory and from pinned host
memory, and the offloaded decode step against the resident one and the oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_00777_amd import binding, synth
from tests.parity import assert_out_close
from tests.step_check import check_step

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def say(msg):
    print("[case] " + msg, flush=True)


def bits(t):
    return t.cpu().view(torch.int16).numpy().view(np.uint16)


@pytest.mark.parametrize("B,Hkv,d,N,k,pinned", [(2, 2, 128, 3000, 700, False), (2, 3, 128, 3000, 513, True),
                                                 (1, 2, 64, 1000, 64, True), (1, 1, 128, 50, 1, True)])
def test_gather_rows_is_exact(B, Hkv, d, N, k, pinned):
    say("gather rows B=%d Hkv=%d d=%d N=%d k=%d pinned=%s" % (B, Hkv, d, N, k, pinned))
    gen = torch.Generator().manual_seed(N + k)
    K = torch.randn((B, Hkv, N, d), generator=gen).to(torch.bfloat16)
    V = torch.randn((B, Hkv, N, d), generator=gen).to(torch.bfloat16)
    rng = np.random.RandomState(k)
    idx = np.stack([[rng.permutation(N)[:k] for _ in range(Hkv)] for _ in range(B)]).astype(np.int32)
    if k > 8:
        idx[:, :, ::5] = -1
        idx[:, :, 3] = N
    Ks, Vs = (K.pin_memory(), V.pin_memory()) if pinned else (K.to(DEV), V.to(DEV))
    rK, rV, ri = oracle.gather_rows(K, V, np.where(idx >= N, -1, idx))
    with binding.Context(B, Hkv, Hkv, d, N, k) as ctx:
        Kd, Vd, idd = ctx.gather_rows(Ks, Vs, torch.from_numpy(idx).to(DEV))
        torch.cuda.synchronize()
    assert np.array_equal(bits(Kd), rK) and np.array_equal(bits(Vd), rV)
    assert np.array_equal(idd.cpu().numpy(), ri)


@pytest.mark.parametrize("n_slots", [1, 2, 5])
def test_offloaded_step_equals_resident_step(n_slots):
    """Reuse layers' caches in pinned host memory, gathers on a second stream: outputs and the
    final index set must equal the resident step's bit for bit (same kernels over the same
    rows), and match the oracle."""
    say("offloaded step n_slots=%d" % n_slots)
    w = synth.scaled(synth.WORKLOADS["toy"], n_layers=9, full_layers=(0, 1, 5), ctx_len=2500, top_k=300,
                     n_q_heads=16, n_kv_heads=4, head_dim=128, batch=2)
    policy, _, data = synth.make_workload(w, DEV)
    qs, Ks, Vs = [x[0] for x in data], [x[1] for x in data], [x[2] for x in data]
    Ko = [K if policy[l] == synth.FULL else K.cpu().pin_memory() for l, K in enumerate(Ks)]
    Vo = [V if policy[l] == synth.FULL else V.cpu().pin_memory() for l, V in enumerate(Vs)]
    with binding.Context(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ctx_len, w.top_k) as ctx:
        ctx.set_option("full_variant", 23)          # statically split: bit-reproducible Full outputs
        want, want_idx = ctx.decode_step(policy, qs, Ks, Vs, w.top_k)
        torch.cuda.synchronize()
        run, outs, idx_buf, copy_stream = ctx.prepare_step_offloaded(policy, qs, Ko, Vo, w.top_k, n_slots=n_slots)
        for rep in range(3):
            for o in outs:
                o.fill_(float("nan"))
            run()
            torch.cuda.synchronize()
            for l in range(w.n_layers):
                assert torch.equal(outs[l], want[l]), "layer %d differs from the resident step (run %d)" % (l, rep)
            assert torch.equal(idx_buf, want_idx)
        # ... and the oracle, every layer: Full layers against its dense attention, Reuse layers
        # against its sparse attention over the source cache (on the GPU's own set where that
        # differs from the oracle's inside the tie band)
        res = check_step(ctx, policy, qs, Ks, Vs, w.top_k, outs, idx_buf)
    assert res["layers"] == w.n_layers
    ref_outs, ref_idx, _ = oracle.decode_step(policy, qs, Ks, Vs, w.top_k)
    if np.array_equal(ref_idx, want_idx.cpu().numpy()):
        for l in range(w.n_layers):
            assert_out_close(outs[l].cpu().numpy(), ref_outs[l], "offloaded step layer %d vs oracle.decode_step" % l)


def test_offloaded_step_errors():
    say("offloaded step errors")
    w = synth.scaled(synth.WORKLOADS["toy"], n_layers=2, ctx_len=600, top_k=64)
    policy, _, data = synth.make_workload(w, DEV)
    qs, Ks, Vs = [x[0] for x in data], [x[1] for x in data], [x[2] for x in data]
    with binding.Context(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ctx_len, w.top_k) as ctx:
        with pytest.raises(binding.HylraError) as e:
            run, *_ = ctx.prepare_step_offloaded(policy, qs, Ks, Vs, w.top_k, n_slots=0)
            run()
        assert e.value.status == 3
        with pytest.raises(binding.HylraError) as e:
            run, *_ = ctx.prepare_step_offloaded([1, 0], qs, Ks, Vs, w.top_k)
            run()
        assert e.value.status == 4
