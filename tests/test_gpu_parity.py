"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs, element by element.  Sizes are chosen so the oracle finishes in seconds while
the kernels still run several tiles, several splits and a ragged tail."""
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


def rand_case(seed, B, Hkv, G, d, N, plant=0.02, beta=3.0):
    w = synth.Workload("case", 1, Hkv * G, Hkv, d, B, N, 1, (0,), plant, beta, 1.0, seed=seed)
    planted = synth.planted_positions(w)
    return synth.make_layer(w, 0, planted[0], DEV)


def run_full(ctx, q, K, V, k):
    out, idx = ctx.full_attn_topk(q, K, V, k)
    torch.cuda.synchronize()
    return out.cpu().numpy(), idx.cpu().numpy()


FULL_CASES = [
    # B, Hkv, G, d,   N,    k
    (1, 1, 1, 64, 5, 2),
    (1, 1, 4, 128, 1, 1),
    (2, 2, 4, 128, 1000, 64),
    (1, 2, 4, 64, 2048, 128),
    (1, 3, 1, 128, 1027, 100),
    (2, 1, 2, 64, 4099, 333),
    (1, 2, 3, 128, 777, 50),
    (1, 1, 5, 64, 1500, 77),
    (1, 2, 6, 128, 900, 60),
    (1, 2, 7, 128, 3001, 256),
    (1, 1, 8, 64, 2500, 200),
    (1, 1, 8, 128, 1300, 1299),
    (3, 2, 4, 128, 8192, 512),
]


@pytest.mark.parametrize("B,Hkv,G,d,N,k", FULL_CASES)
def test_full_attn_topk_matches_oracle(B, Hkv, G, d, N, k):
    say("full B=%d Hkv=%d G=%d d=%d N=%d k=%d" % (B, Hkv, G, d, N, k))
    q, K, V = rand_case(100 + N + G, B, Hkv, G, d, N)
    with binding.Context(B, Hkv * G, Hkv, d, N, k) as ctx:
        out, idx = run_full(ctx, q, K, V, k)
    ref_out, ref_idx, shat = oracle.full_attn_topk(q, K, V, k, want_shat=True)
    assert_out_close(out, ref_out, "full out")
    assert_idx_valid(idx, shat, k, "full idx", exact_ref=ref_idx)


@pytest.mark.parametrize("variant", [23, 43, 52, 72, 74])
def test_full_kernel_variants(variant):
    say("full variant=%d" % variant)
    B, Hkv, G, d, N, k = 2, 2, 4, 128, 5003, 300
    q, K, V = rand_case(17, B, Hkv, G, d, N)
    ref_out, ref_idx, shat = oracle.full_attn_topk(q, K, V, k, want_shat=True)
    with binding.Context(B, Hkv * G, Hkv, d, N, k) as ctx:
        ctx.set_option("full_variant", variant)
        ctx.set_option("full_split_rows", 768)
        for rep in range(2):
            out, idx = run_full(ctx, q, K, V, k)
            assert_out_close(out, ref_out, "full out")
            assert_idx_valid(idx, shat, k, "full idx", exact_ref=ref_idx)


@pytest.mark.parametrize("B,Hkv,G,d,N,k", [(1, 1, 4, 128, 5003, 300), (2, 2, 2, 128, 20000, 1000), (1, 2, 4, 64, 3000, 100),
                                          (1, 1, 3, 128, 50, 7), (1, 2, 1, 128, 1, 1), (1, 1, 4, 128, 70001, 2048),
                                          (16, 8, 4, 128, 1500, 64)])
@pytest.mark.parametrize("variant", [43, 74])
def test_full_self_scheduling_kernel(B, Hkv, G, d, N, k, variant):
    """The Full kernel that hands out rows at run time, with its own planning: one or several
    segments per (batch, KV head), more workgroups than chunks, a single tile, and launch after
    launch (its chunk counters return to zero by themselves)."""
    say("full self-scheduling variant=%d B=%d Hkv=%d G=%d d=%d N=%d k=%d" % (variant, B, Hkv, G, d, N, k))
    if variant == 74 and d != 128:
        pytest.skip("the second matrix-core kernel is built for head_dim 128")
    q, K, V = rand_case(23 + N, B, Hkv, G, d, N)
    ref_out, ref_idx, shat = oracle.full_attn_topk(q, K, V, k, want_shat=True)
    with binding.Context(B, Hkv * G, Hkv, d, N, k) as ctx:
        ctx.set_option("full_variant", variant)
        for rep in range(3):
            out, idx = run_full(ctx, q, K, V, k)
            assert_out_close(out, ref_out, "full out (launch %d)" % rep)
            assert_idx_valid(idx, shat, k, "full idx (launch %d)" % rep, exact_ref=ref_idx)


@pytest.mark.parametrize("N,k", [(5003, 300), (20000, 1500), (40000, 3000)])
def test_finalize_paths(N, k):
    """The selection, in one launch and in two, with the first histogram made inside the streaming
    kernel or by a launch of its own, including the many-ties fallbacks (a chunk's list overflowing; more
    tied candidates than can be ranked), at sizes that span one to several chunks."""
    say("finalize paths N=%d k=%d" % (N, k))
    B, Hkv, G, d = 1, 2, 4, 64
    q, K, V = rand_case(19 + N, B, Hkv, G, d, N)
    gen = torch.Generator().manual_seed(N)
    Kt = torch.randint(-1, 2, K.shape, generator=gen).to(torch.bfloat16).to(DEV)     # heavy exact ties
    qt = torch.randint(-1, 2, q.shape, generator=gen).to(torch.bfloat16).to(DEV)
    Kz = torch.zeros_like(K)                                                          # one giant tie
    ref = [oracle.full_attn_topk(q, K, V, k, want_shat=True),
           oracle.full_attn_topk(qt, Kt, V, k, want_shat=True),
           oracle.full_attn_topk(q, Kz, V, k, want_shat=True)]
    with binding.Context(B, Hkv * G, Hkv, d, N, k) as ctx:
        for unfused, two in ((0, 0), (1, 0), (0, 1), (1, 1)):
            ctx.set_option("hist_unfused", unfused)
            ctx.set_option("topk_two_launches", two)     # the selection in one launch, or as scan + emit
            for rep in range(2):                         # (launch after launch: the headers are left empty)
                for (qq, KK), (ro, ri, rs), exact in (((q, K), ref[0], False), ((qt, Kt), ref[1], True), ((q, Kz), ref[2], True)):
                    out, idx = run_full(ctx, qq, KK, V, k)
                    assert ctx.get_info("last_topk_launches") == 1 + two
                    assert_out_close(out, ro, "out")
                    assert_idx_valid(idx, rs, k, "idx", exact_ref=ri)
                    if exact:      # d = 64 and integer inputs: scores are exact, sets must be equal
                        assert np.array_equal(idx, ri)


@pytest.mark.parametrize("unroll", [1, 2, 4, 8])
def test_reuse_kernel_unrolls(unroll):
    say("reuse unroll=%d" % unroll)
    B, Hkv, G, d, N, k = 2, 2, 4, 128, 5003, 700
    q, K, V = rand_case(18, B, Hkv, G, d, N)
    rng = np.random.RandomState(unroll)
    idx = np.stack([[np.sort(rng.permutation(N)[:k]) for _ in range(Hkv)] for _ in range(B)]).astype(np.int32)
    ref = oracle.reuse_sparse_attn(q, K, V, idx)
    with binding.Context(B, Hkv * G, Hkv, d, N, k) as ctx:
        ctx.set_option("reuse_unroll", unroll)
        for variant in (1, 2, 3, 4):        # vector kernel (streaming / plain loads), matrix-core kernel
            if variant >= 3 and unroll == 1:
                continue
            ctx.set_option("reuse_variant", variant)
            out = ctx.reuse_sparse_attn(q, K, V, torch.from_numpy(idx).to(DEV))
            torch.cuda.synchronize()
            assert_out_close(out.cpu().numpy(), ref, "reuse out")


@pytest.mark.parametrize("variant,waves", [(3, 4), (4, 8), (5, 4), (5, 8), (6, 4), (6, 8)])
def test_reuse_matrix_core_kernels(variant, waves):
    """Both matrix-core Reuse kernels, with workgroups of 4 and of 8 waves, for every group size,
    with padding entries, several sweeps per workgroup and a ragged tail."""
    say("reuse matrix-core variant=%d waves=%d" % (variant, waves))
    for G, (B, Hkv, N, k) in zip(range(1, 9), [(1, 2, 3000, 700), (2, 1, 2000, 513), (1, 1, 1500, 64), (2, 2, 5003, 1100),
                                                (1, 1, 900, 31), (1, 2, 4000, 1024), (2, 1, 2500, 900), (1, 1, 1300, 1300)]):
        q, K, V = rand_case(40 + G, B, Hkv, G, 128, N)
        rng = np.random.RandomState(10 * variant + G)
        idx = np.stack([[np.sort(rng.permutation(N)[:k]) for _ in range(Hkv)] for _ in range(B)]).astype(np.int32)
        idx[:, :, ::7] = -1                      # padding entries
        idx[:, :, 5::41] = N + 3
        ref = oracle.reuse_sparse_attn(q, K, V, np.where(idx >= N, -1, idx))
        with binding.Context(B, Hkv * G, Hkv, 128, N, k) as ctx:
            ctx.set_option("reuse_variant", variant)
            ctx.set_option("reuse_waves", waves)
            for split_rows in (0, 2048):
                ctx.set_option("reuse_split_rows", split_rows)
                out = ctx.reuse_sparse_attn(q, K, V, torch.from_numpy(idx).to(DEV))
                torch.cuda.synchronize()
                assert_out_close(out.cpu().numpy(), ref, "reuse out G=%d split_rows=%d" % (G, split_rows))


@pytest.mark.parametrize("split_rows", [128, 256, 4096])
def test_full_result_does_not_depend_on_split(split_rows):
    say("full split_rows=%d" % split_rows)
    B, Hkv, G, d, N, k = 1, 2, 4, 128, 5000, 300
    q, K, V = rand_case(7, B, Hkv, G, d, N)
    ref_out, ref_idx, shat = oracle.full_attn_topk(q, K, V, k, want_shat=True)
    with binding.Context(B, Hkv * G, Hkv, d, N, k) as ctx:
        ctx.set_option("full_split_rows", split_rows)
        out, idx = run_full(ctx, q, K, V, k)
    assert_out_close(out, ref_out, "full out")
    assert_idx_valid(idx, shat, k, "full idx", exact_ref=ref_idx)


def test_full_k_equals_context_and_k_one():
    say("full k=N and k=1")
    B, Hkv, G, d, N = 1, 2, 4, 128, 700
    q, K, V = rand_case(8, B, Hkv, G, d, N)
    with binding.Context(B, Hkv * G, Hkv, d, N, N) as ctx:
        out, idx = run_full(ctx, q, K, V, N)
        assert np.array_equal(idx, np.broadcast_to(np.arange(N), idx.shape))
        sparse = ctx.reuse_sparse_attn(q, K, V, torch.from_numpy(idx).to(DEV))
        torch.cuda.synchronize()
        # full attention equals sparse attention over every row
        assert_out_close(sparse.cpu().numpy(), out, "sparse(k=N) vs full")
        out1, idx1 = run_full(ctx, q, K, V, 1)
    _, ref1, shat = oracle.full_attn_topk(q, K, V, 1, want_shat=True)
    assert_idx_valid(idx1, shat, 1, "k=1", exact_ref=ref1)
    assert np.array_equal(idx1, ref1)


@pytest.mark.parametrize("G", [1, 2, 4])
def test_full_exact_ties_go_to_lower_position(G):
    """Small-integer keys and queries with d = 64 (scale 1/8): every score is exact in fp32
    and fp64 alike and heavily tied, so the GPU set must equal the oracle's exactly, which
    checks the lower-position tie rule and the many-ties selection path."""
    say("full ties G=%d" % G)
    B, Hkv, d, N, k = 1, 2, 64, 6000, 500
    gen = torch.Generator().manual_seed(5 + G)
    q = torch.randint(-1, 2, (B, Hkv * G, d), generator=gen).to(torch.bfloat16).to(DEV)
    K = torch.randint(-1, 2, (B, Hkv, N, d), generator=gen).to(torch.bfloat16).to(DEV)
    V = torch.randn((B, Hkv, N, d), generator=gen).to(torch.bfloat16).to(DEV)
    with binding.Context(B, Hkv * G, Hkv, d, N, k) as ctx:
        out, idx = run_full(ctx, q, K, V, k)
        # all keys identical: every score ties, the first k positions win
        K0 = torch.zeros_like(K)
        out0, idx0 = run_full(ctx, q, K0, V, k)
    ref_out, ref_idx, _ = oracle.full_attn_topk(q, K, V, k)
    assert np.array_equal(idx, ref_idx)
    assert_out_close(out, ref_out, "ties out")
    assert np.array_equal(idx0, np.broadcast_to(np.arange(k), idx0.shape))
    ref0, _, _ = oracle.full_attn_topk(q, K0, V, k)
    assert_out_close(out0, ref0, "uniform attention out")


REUSE_CASES = [
    # B, Hkv, G, d,  N,    k
    (1, 1, 1, 64, 50, 1),
    (2, 2, 4, 128, 3000, 128),
    (1, 2, 4, 64, 2048, 128),
    (1, 1, 7, 128, 5000, 777),
    (2, 3, 2, 128, 999, 33),
    (1, 2, 8, 64, 4000, 2048),
    (4, 8, 4, 128, 4096, 512),
    (1, 1, 3, 128, 100, 100),
    (1, 1, 5, 128, 300, 17),
    (1, 1, 6, 64, 300, 130),
]


@pytest.mark.parametrize("B,Hkv,G,d,N,k", REUSE_CASES)
def test_reuse_sparse_attn_matches_oracle(B, Hkv, G, d, N, k):
    say("reuse B=%d Hkv=%d G=%d d=%d N=%d k=%d" % (B, Hkv, G, d, N, k))
    q, K, V = rand_case(200 + N + G, B, Hkv, G, d, N)
    rng = np.random.RandomState(k)
    idx = np.stack([[np.sort(rng.permutation(N)[:k]) for _ in range(Hkv)] for _ in range(B)]).astype(np.int32)
    with binding.Context(B, Hkv * G, Hkv, d, N, k) as ctx:
        out = ctx.reuse_sparse_attn(q, K, V, torch.from_numpy(idx).to(DEV))
        torch.cuda.synchronize()
    assert_out_close(out.cpu().numpy(), oracle.reuse_sparse_attn(q, K, V, idx), "reuse out")


@pytest.mark.parametrize("B,Hkv,G,d,N,k", [(4, 8, 4, 128, 8192, 2048), (2, 4, 7, 128, 6000, 1000), (8, 2, 4, 64, 4096, 1024),
                                          (2, 2, 4, 128, 3000, 200), (1, 3, 5, 64, 2000, 100), (32, 8, 4, 128, 2048, 1024)])
def test_reuse_fused_merge_equals_two_kernel_merge(B, Hkv, G, d, N, k):
    """The in-kernel merge (last-arriving workgroup; with one workgroup per (batch, KV head) the
    output straight from that workgroup) must give bit-identical results to the separate merge
    kernel, launch after launch (the arrival counters reset themselves)."""
    say("reuse fused merge B=%d Hkv=%d G=%d d=%d N=%d k=%d" % (B, Hkv, G, d, N, k))
    q, K, V = rand_case(300 + G, B, Hkv, G, d, N)
    rng = np.random.RandomState(k)
    idx = np.stack([[np.sort(rng.permutation(N)[:k]) for _ in range(Hkv)] for _ in range(B)]).astype(np.int32)
    gidx = torch.from_numpy(idx).to(DEV)
    with binding.Context(B, Hkv * G, Hkv, d, N, k) as ctx:
        ctx.set_option("reuse_unfused", 1)
        two = ctx.reuse_sparse_attn(q, K, V, gidx).clone()
        ctx.set_option("reuse_unfused", 0)
        outs = []
        for it in range(40):
            o = torch.full(q.shape, float("nan"), dtype=torch.float32, device=DEV)
            ctx.reuse_sparse_attn(q, K, V, gidx, out=o)
            outs.append(o)
        torch.cuda.synchronize()
        # the shapes with k <= 256 or many pairs are covered by one workgroup per pair
        assert ctx.get_info("last_reuse_merge") in ((3,) if ctx.get_info("last_reuse_splits") == 1 else (1, 2))
        assert (ctx.get_info("last_reuse_splits") == 1) == ((B, k) in ((2, 200), (1, 100), (32, 1024)))
    for it, o in enumerate(outs):
        assert torch.equal(o, two), "fused merge differs at launch %d" % it
    assert_out_close(two.cpu().numpy(), oracle.reuse_sparse_attn(q, K, V, idx), "reuse out")


@pytest.mark.parametrize("B,Hkv,G,k,unroll", [(1, 8, 4, 4096, 0), (2, 8, 7, 2048, 0), (4, 8, 4, 2048, 8), (1, 4, 1, 1024, 4),
                                              (1, 2, 8, 4096, 0), (3, 5, 3, 512, 4)])
def test_reuse_packet_merge_equals_two_kernel_merge(B, Hkv, G, k, unroll):
    """The merge by packets (every workgroup of a (batch, KV head) merges a slice of the columns
    from 64-bit {value, tag} units it polls) must give bit-identical results to the separate
    merge kernel over the same partials, launch after launch (the units are cleared by their
    readers), also when launches of another shape run in between."""
    say("reuse packet merge B=%d Hkv=%d G=%d k=%d unroll=%d" % (B, Hkv, G, k, unroll))
    d, N = 128, 8192
    q, K, V = rand_case(310 + G, B, Hkv, G, d, N)
    rng = np.random.RandomState(k)
    idx = np.stack([[np.sort(rng.permutation(N)[:k]) for _ in range(Hkv)] for _ in range(B)]).astype(np.int32)
    idx[:, :, k // 3] = -1                       # a padding entry
    gidx = torch.from_numpy(idx).to(DEV)
    other = gidx[:, :, :256].contiguous()
    with binding.Context(B, Hkv * G, Hkv, d, N, k) as ctx:
        # same split both times: wave tiles of 32 rows (unroll 4: 128 entries per workgroup) or of 64
        ctx.set_option("reuse_unroll", unroll if unroll else 4)
        if unroll == 8:
            ctx.set_option("reuse_waves", 8)
        ctx.set_option("reuse_unfused", 1)
        two = ctx.reuse_sparse_attn(q, K, V, gidx).clone()
        ctx.set_option("reuse_unfused", 0)
        ctx.set_option("reuse_merge", 2)         # packets whenever the launch allows them
        if unroll == 0:                          # the automatic choice must be this very split
            ctx.set_option("reuse_unroll", 0)
            ctx.set_option("reuse_merge", 0)
        ctx.profile_enable(True)
        outs = []
        for it in range(30):
            o = torch.full(q.shape, float("nan"), dtype=torch.float32, device=DEV)
            ctx.reuse_sparse_attn(q, K, V, gidx, out=o)
            outs.append(o)
            if it % 7 == 3:
                ctx.reuse_sparse_attn(q, K, V, other)
        torch.cuda.synchronize()
        prof = ctx.profile_read()
        assert prof["reuse_combine"][0] == 0
        ctx.reuse_sparse_attn(q, K, V, gidx)
        assert ctx.get_info("last_reuse_merge") == 2, "the launch did not merge by packets"
        assert ctx.get_info("last_reuse_splits") == k // (512 if unroll == 8 else 128)
        assert ctx.get_info("last_reuse_wave_rows") == (64 if unroll == 8 else 32)
    for it, o in enumerate(outs):
        assert torch.equal(o, two), "packet merge differs at launch %d" % it
    assert_out_close(two.cpu().numpy(), oracle.reuse_sparse_attn(q, K, V, idx), "reuse out")


def test_two_contexts_on_two_streams_share_the_device():
    """Two contexts, each on a stream of its own, run launches whose workgroups wait for one
    another (Reuse merge by packets, one-launch selection) at the same time: each launch holds
    at most one workgroup per compute unit, so both fit, and the results are those of running
    them one after the other."""
    say("two contexts on two streams")
    B, Hkv, G, d, N, k = 1, 8, 4, 128, 8192, 2048
    cases = [rand_case(330 + i, B, Hkv, G, d, N) for i in range(2)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    with binding.Context(B, Hkv * G, Hkv, d, N, k) as c0, binding.Context(B, Hkv * G, Hkv, d, N, k) as c1:
        ctxs = [c0, c1]
        want = []
        for ctx, (q, K, V) in zip(ctxs, cases):
            out, idx = ctx.full_attn_topk(q, K, V, k)
            sparse = ctx.reuse_sparse_attn(q, K, V, idx)
            torch.cuda.synchronize()
            assert ctx.get_info("last_reuse_merge") == 2 and ctx.get_info("last_topk_launches") == 1
            want.append((out.clone(), idx.clone(), sparse.clone()))
        got = [[], []]
        torch.cuda.synchronize()
        for rep in range(10):
            for i, (ctx, (q, K, V)) in enumerate(zip(ctxs, cases)):
                with torch.cuda.stream(streams[i]):
                    out, idx = ctx.full_attn_topk(q, K, V, k)
                    sparse = ctx.reuse_sparse_attn(q, K, V, idx)
                    got[i].append((out, idx, sparse))
        torch.cuda.synchronize()
    for i in range(2):
        for rep, (out, idx, sparse) in enumerate(got[i]):
            assert torch.equal(idx, want[i][1]), "context %d launch %d: index set" % (i, rep)
            assert torch.equal(sparse, want[i][2]), "context %d launch %d: Reuse output" % (i, rep)
            err = (out - want[i][0]).abs().max().item() / want[i][0].abs().max().item()
            assert err < 1e-5, "context %d launch %d: Full output differs by %.2e" % (i, rep, err)


def test_reuse_padding_order_and_out_of_range_entries():
    say("reuse padding")
    B, Hkv, G, d, N, k = 1, 2, 4, 128, 1000, 200
    q, K, V = rand_case(9, B, Hkv, G, d, N)
    rng = np.random.RandomState(3)
    base = np.stack([[rng.permutation(N)[:150] for _ in range(Hkv)] for _ in range(B)]).astype(np.int32)
    idx = np.full((B, Hkv, k), -1, np.int32)
    idx[:, :, 10:160] = base                     # unsorted, padded on both sides
    ref = oracle.reuse_sparse_attn(q, K, V, idx)
    gidx = idx.copy()
    gidx[:, :, 0] = N                            # >= N is skipped by the library as padding
    gidx[:, :, 199] = 2 ** 31 - 1
    with binding.Context(B, Hkv * G, Hkv, d, N, k) as ctx:
        out = ctx.reuse_sparse_attn(q, K, V, torch.from_numpy(gidx).to(DEV))
        empty = ctx.reuse_sparse_attn(q, K, V, torch.full((B, Hkv, k), -1, dtype=torch.int32, device=DEV))
        torch.cuda.synchronize()
    assert_out_close(out.cpu().numpy(), ref, "reuse padded")
    assert np.all(empty.cpu().numpy() == 0.0)


def test_strided_cache_views():
    """K and V as views of a larger allocation (a cache with room for more tokens)."""
    say("strided views")
    B, Hkv, G, d, N, k = 2, 2, 4, 128, 1500, 100
    q, K, V = rand_case(10, B, Hkv, G, d, N)
    bigK = torch.zeros((B, Hkv, N + 500, d + 64), dtype=torch.bfloat16, device=DEV)
    bigV = torch.zeros_like(bigK)
    bigK[:, :, :N, :d] = K
    bigV[:, :, :N, :d] = V
    Kv, Vv = bigK[:, :, :N, :d], bigV[:, :, :N, :d]
    ref_out, ref_idx, shat = oracle.full_attn_topk(q, K, V, k, want_shat=True)
    with binding.Context(B, Hkv * G, Hkv, d, N, k) as ctx:
        out, idx = run_full(ctx, q, Kv, Vv, k)
        sp = ctx.reuse_sparse_attn(q, Kv, Vv, torch.from_numpy(ref_idx).to(DEV))
        torch.cuda.synchronize()
    assert_out_close(out, ref_out, "strided full")
    assert_idx_valid(idx, shat, k, "strided idx", exact_ref=ref_idx)
    assert_out_close(sp.cpu().numpy(), oracle.reuse_sparse_attn(q, K, V, ref_idx), "strided reuse")


def check_chain(w, ctx=None):
    policy, planted, data = synth.make_workload(w, DEV)
    qs, Ks, Vs = [x[0] for x in data], [x[1] for x in data], [x[2] for x in data]
    own = ctx is None
    if own:
        ctx = binding.Context(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ctx_len, w.top_k)
    try:
        outs, idx_buf = ctx.decode_step(policy, qs, Ks, Vs, w.top_k)
        torch.cuda.synchronize()
    finally:
        if own:
            ctx.close()
    outs = [o.cpu().numpy() for o in outs]
    # oracle, layer by layer; a Reuse layer is evaluated on the GPU's own set when that set
    # differs from the oracle's only inside the tie band (checked by assert_idx_valid)
    # -- the GPU set in force is only observable after the last Full layer, so re-run each
    # Full layer alone to read its set.
    with binding.Context(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ctx_len, w.top_k) as c2:
        cur = None
        for l in range(w.n_layers):
            if policy[l] == synth.FULL:
                ref_out, ref_idx, shat = oracle.full_attn_topk(qs[l], Ks[l], Vs[l], w.top_k, want_shat=True)
                _, gidx = run_full(c2, qs[l], Ks[l], Vs[l], w.top_k)
                assert_idx_valid(gidx, shat, w.top_k, "layer %d idx" % l, exact_ref=ref_idx)
                cur = gidx
            else:
                ref_out = oracle.reuse_sparse_attn(qs[l], Ks[l], Vs[l], cur)
            assert_out_close(outs[l], ref_out, "layer %d out" % l)
    assert np.array_equal(idx_buf.cpu().numpy(), cur)
    return planted, cur


def test_decode_step_toy_config():
    """The smallest benchmark configuration: 2-layer toy, policy [full, reuse]."""
    say("decode_step toy")
    w = synth.WORKLOADS["toy"]
    planted, idx = check_chain(w)
    # the planted positions are what the selection is meant to find
    hit = np.mean([np.isin(planted[0][0, g], idx[0, g]).mean() for g in range(w.n_kv_heads)])
    assert hit > 0.7


def test_decode_step_longer_chain_and_baseline_policies():
    say("decode_step 7 layers")
    base = synth.scaled(synth.WORKLOADS["llama3_8b_32k"], n_layers=7, batch=2, n_q_heads=8,
                        n_kv_heads=2, ctx_len=3000, top_k=200, full_layers=(0, 1, 4))
    check_chain(base)
    check_chain(synth.scaled(base, full_layers=tuple(range(7))))          # all-Full baseline
    check_chain(synth.scaled(base, full_layers=(0, 3, 6)))                # fixed stride of 3
    check_chain(synth.scaled(synth.WORKLOADS["qwen25_7b_64k"], n_layers=4, batch=1, ctx_len=2500,
                             top_k=150, full_layers=(0, 1)))              # group of 7, sink prefix


@pytest.mark.parametrize("batch,ctx_len,top_k", [(16, 3000, 512), (1, 6000, 2048)])
def test_decode_step_replayed_from_a_hip_graph(batch, ctx_len, top_k):
    """hylra_decode_step only launches kernels on the caller's stream, so a caller may capture
    it in a HIP graph.  Replays (with eager launches and synchronisations in between) must give
    the eager result: this covers the counters the kernels reset themselves.  Index sets and the
    Reuse layers' outputs must be bit-identical; a Full layer's output may differ in the last
    bits, because the self-scheduling kernel groups the rows into partial sums differently from
    run to run (the row scores, and hence the index sets, do not depend on the grouping).
    Batch 16: the self-scheduling Full kernel (batch * n_kv_heads >= 64) and the Reuse merge by
    arrival counter; batch 1 with k = 2048: the Reuse merge by packets, whose units the
    consumers clear themselves and which takes no launch number from the host."""
    say("decode step under graph capture, batch %d" % batch)
    w = synth.scaled(synth.WORKLOADS["toy"], n_layers=6, full_layers=(0, 3), batch=batch, n_q_heads=32, n_kv_heads=8,
                     head_dim=128, ctx_len=ctx_len, top_k=top_k)
    policy, _, data = synth.make_workload(w, DEV)
    qs, Ks, Vs = [x[0] for x in data], [x[1] for x in data], [x[2] for x in data]
    with binding.Context(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ctx_len, w.top_k) as ctx:
        run, outs, idx_buf = ctx.prepare_step(policy, qs, Ks, Vs, w.top_k)
        run()
        torch.cuda.synchronize()
        want = [o.clone() for o in outs] + [idx_buf.clone()]
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            run()
        for rep in range(4):
            for o in outs:
                o.fill_(float("nan"))
            idx_buf.fill_(-7)
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(idx_buf, want[-1]), "replay %d: index sets differ from the eager step" % rep
            for l, (got, ref) in enumerate(zip(outs, want)):
                if policy[l] == synth.REUSE:
                    assert torch.equal(got, ref), "replay %d: Reuse layer %d differs from the eager step" % (rep, l)
                else:
                    err = (got - ref).abs().max().item() / ref.abs().max().item()
                    assert err < 1e-5, "replay %d: Full layer %d differs from the eager step by %.2e" % (rep, l, err)
            run()                                   # eager work between replays
            torch.cuda.synchronize()


@pytest.mark.parametrize("variant", [23, 43])
def test_results_are_deterministic(variant):
    """Run to run, index sets and Reuse outputs are bit-identical with every kernel; the Full
    output is too with the statically split kernels.  (The self-scheduling Full kernel hands
    rows to workgroups at run time, so its partial sums group differently from run to run and
    the output can move in the last bits; the row scores and the index sets cannot.)"""
    say("determinism variant=%d" % variant)
    B, Hkv, G, d, N, k = 2, 2, 4, 128, 6000, 400
    q, K, V = rand_case(12, B, Hkv, G, d, N)
    with binding.Context(B, Hkv * G, Hkv, d, N, k) as ctx:
        ctx.set_option("full_variant", variant)
        a_out, a_idx = run_full(ctx, q, K, V, k)
        b_out, b_idx = run_full(ctx, q, K, V, k)
        ra = ctx.reuse_sparse_attn(q, K, V, torch.from_numpy(a_idx).to(DEV)).cpu().numpy()
        rb = ctx.reuse_sparse_attn(q, K, V, torch.from_numpy(a_idx).to(DEV)).cpu().numpy()
    assert np.array_equal(a_idx, b_idx)
    if variant == 23:
        assert np.array_equal(a_out, b_out)
    else:
        assert np.max(np.abs(a_out - b_out)) <= 1e-5 * np.max(np.abs(a_out))
    assert np.array_equal(ra, rb)


def test_creation_flags():
    """HYLRA_FLAG_DETERMINISTIC: the Full output is bit-identical from run to run at a shape whose
    default kernel hands rows out at run time.  HYLRA_FLAG_TOPK_EVERY_FULL_LAYER: same outputs
    and final set as the step that skips the TopK nobody reads."""
    say("creation flags")
    B, Hkv, G, d, N, k = 16, 4, 4, 128, 8192, 300        # batch * n_kv_heads = 64: self-scheduling by default
    q, K, V = rand_case(31, B, Hkv, G, d, N)
    with binding.Context(B, Hkv * G, Hkv, d, N, k, deterministic=True) as ctx:
        a_out, a_idx = run_full(ctx, q, K, V, k)
        for _ in range(3):
            b_out, b_idx = run_full(ctx, q, K, V, k)
            assert np.array_equal(a_out, b_out) and np.array_equal(a_idx, b_idx)
    ref_out, ref_idx, shat = oracle.full_attn_topk(q, K, V, k, want_shat=True)
    assert_out_close(a_out, ref_out, "deterministic flag")
    assert_idx_valid(a_idx, shat, k, "deterministic flag", exact_ref=ref_idx)
    w = synth.scaled(synth.WORKLOADS["llama3_8b_32k"], n_layers=5, batch=2, n_q_heads=8, n_kv_heads=2, ctx_len=3000,
                     top_k=200, full_layers=(0, 1, 2, 4))
    policy, _, data = synth.make_workload(w, DEV)
    qs, Ks, Vs = [x[0] for x in data], [x[1] for x in data], [x[2] for x in data]
    res = []
    for every in (False, True):
        with binding.Context(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ctx_len, w.top_k, deterministic=True,
                             topk_every_full_layer=every) as ctx:
            ctx.profile_enable(True)
            ctx.profile_reset()
            outs, idx_buf = ctx.decode_step(policy, qs, Ks, Vs, w.top_k)
            torch.cuda.synchronize()
            res.append(([o.cpu().numpy() for o in outs], idx_buf.cpu().numpy()))
    for l in range(w.n_layers):
        assert np.array_equal(res[0][0][l], res[1][0][l]), "layer %d" % l
    assert np.array_equal(res[0][1], res[1][1])
    with pytest.raises(binding.HylraError):
        binding.load_library()      # (loaded) -- an unknown flag bit is refused
        import ctypes
        h = ctypes.c_void_p()
        shp = binding.Shape(1, 8, 2, 128, 128, 0, 0, 0, 0.0)
        rc = binding.load_library().hylra_create_ex(ctypes.byref(h), ctypes.byref(shp), 8, 0, 0x80)
        if rc != 0:
            raise binding.HylraError(rc, "hylra_create_ex", binding.load_library().hylra_last_error(None).decode())


def test_error_codes():
    say("error codes")
    B, Hkv, G, d, N, k = 1, 2, 4, 128, 512, 32
    q, K, V = rand_case(13, B, Hkv, G, d, N)
    with binding.Context(B, Hkv * G, Hkv, d, N, k) as ctx:
        for bad_k in (0, N + 1):
            with pytest.raises(binding.HylraError) as e:
                ctx.full_attn_topk(q, K, V, bad_k)
            assert e.value.status == 1
        with pytest.raises(binding.HylraError) as e:
            ctx.full_attn_topk(q, K, V, k + 1)          # above the context's max_k
        assert e.value.status == 3
        with pytest.raises(binding.HylraError) as e:
            ctx.decode_step([1, 0], [q, q], [K, K], [V, V], k)
        assert e.value.status == 4
        with pytest.raises(binding.HylraError) as e:
            ctx.decode_step([0, 2], [q, q], [K, K], [V, V], k)
        assert e.value.status == 4
        # misaligned K (offset by one element)
        flat = torch.zeros(K.numel() + 8, dtype=torch.bfloat16, device=DEV)
        Kmis = flat[1:1 + K.numel()].view(K.shape)
        with pytest.raises(binding.HylraError) as e:
            ctx.full_attn_topk(q, Kmis, Kmis, k)
        assert e.value.status == 1
        # a larger context than the workspace was sized for
        q2, K2, V2 = rand_case(14, B, Hkv, G, d, 4 * N)
        with pytest.raises(binding.HylraError) as e:
            ctx.full_attn_topk(q2, K2, V2, k)
        assert e.value.status == 3
        # a launch that gave up a bounded wait (simulated from the host): every call fails until reset
        ctx.set_option("simulate_give_up", 1)
        for call in (lambda: ctx.full_attn_topk(q, K, V, k), lambda: ctx.reuse_sparse_attn(q, K, V, torch.zeros((B, Hkv, k), dtype=torch.int32, device=DEV))):
            with pytest.raises(binding.HylraError) as e:
                call()
            assert e.value.status == 5 and "hylra_reset" in str(e.value)
        ctx.reset()
        # the context still works after failed calls
        out, idx = run_full(ctx, q, K, V, k)
    ref_out, ref_idx, shat = oracle.full_attn_topk(q, K, V, k, want_shat=True)
    assert_out_close(out, ref_out, "after errors")
    assert_idx_valid(idx, shat, k, "after errors")
    with pytest.raises(binding.HylraError) as e:
        binding.Context(1, 8, 2, 96, 128, 8)              # head_dim 96 is not built
    assert e.value.status == 2
    with pytest.raises(binding.HylraError) as e:
        binding.Context(1, 18, 2, 128, 128, 8)            # group of 9
    assert e.value.status == 2


def test_profile_and_probe_aids():
    """Event-based kernel timing and the two measurement kernels of the C ABI."""
    say("profile / probe")
    B, Hkv, G, d, N, k = 1, 2, 4, 128, 4096, 256
    q, K, V = rand_case(21, B, Hkv, G, d, N)
    with binding.Context(B, Hkv * G, Hkv, d, N, k) as ctx:
        ctx.profile_enable(True)
        ctx.profile_reset()
        out, idx = ctx.full_attn_topk(q, K, V, k)
        for _ in range(3):
            ctx.reuse_sparse_attn(q, K, V, idx)
        torch.cuda.synchronize()
        prof = ctx.profile_read()
        assert prof["full_attn"][0] == 1 and prof["full_finalize"][0] == 1      # streaming pass; the selection in one launch
        assert ctx.get_info("last_topk_launches") == 1
        ctx.set_option("topk_two_launches", 1)
        ctx.profile_reset()
        out2, idx2 = ctx.full_attn_topk(q, K, V, k)
        torch.cuda.synchronize()
        assert ctx.profile_read()["full_finalize"][0] == 2 and ctx.get_info("last_topk_launches") == 2   # scan + emit
        assert torch.equal(idx2, idx)
        ctx.set_option("topk_two_launches", 0)
        ctx.profile_reset()
        ctx.full_attn_topk(q, K, V, k)
        for _ in range(3):
            ctx.reuse_sparse_attn(q, K, V, idx)
        torch.cuda.synchronize()
        prof = ctx.profile_read()
        assert prof["reuse_attn"][0] == 3 and prof["reuse_combine"][0] == 0
        for name in ("full_attn", "full_finalize", "reuse_attn"):
            assert 0.0 < prof[name][1] < 50.0          # milliseconds
        ctx.profile_reset()
        assert ctx.profile_read()["full_attn"] == (0, 0.0)
        src = torch.randint(0, 255, (1 << 20,), dtype=torch.uint8, device=DEV)
        dst = torch.zeros_like(src)
        sink = torch.zeros(16384, dtype=torch.uint8, device=DEV)
        ctx.probe_copy(dst, src)
        ctx.probe_read(src, sink)
        torch.cuda.synchronize()
        assert torch.equal(dst, src)
        assert ctx.profile_read()["probe"][0] == 2
        # the bare gather reads the rows a Reuse layer would read and writes nothing
        pad = idx.clone()
        pad[:, :, ::3] = -1
        pad[:, :, 1] = N
        sink.fill_(3)
        ctx.probe_gather(K, V, pad, sink)
        torch.cuda.synchronize()
        assert ctx.profile_read()["probe"][0] == 3 and torch.all(sink == 3)
        ctx.profile_enable(False)
        with pytest.raises(binding.HylraError):
            ctx.set_option("no_such_option", 1)
