"""Whole-step parity against the CPU oracle at any size, every (batch, KV head) pair.

Used by the full-size GPU tests and by bench.py's untimed post-run check.  One layer's cache
at a time crosses to the host (through a pinned staging buffer), so the host never holds more
than one layer.  Full layers: output against the oracle's dense attention, and -- where the
layer's set is handed to a Reuse layer or returned -- the index set under the tie-band rule of
tests/parity.py.  Reuse layers: output against the oracle evaluated on the GPU's own set of
the layer they inherit from (that set has just been validated against the oracle's ranking;
inside the band the two sets may legitimately differ).  The set a Full layer produced inside
the step is not observable afterwards (the next Full layer overwrites the buffer), so it is
read by running that layer alone: index sets are bit-reproducible from launch to launch, and
a step that handed the wrong set on would fail the Reuse comparison.
"""
import time

import numpy as np
import torch

import oracle
from tests.parity import assert_idx_valid, assert_out_close

FULL, REUSE = 0, 1


class _Stage:
    """Pinned host staging for one tensor shape (reused for every layer)."""

    def __init__(self):
        self.buf = {}

    def fetch(self, t, slot):
        key = (slot, tuple(t.shape), t.dtype)
        if key not in self.buf:
            self.buf[key] = torch.empty(t.shape, dtype=t.dtype, pin_memory=True)
        self.buf[key].copy_(t, non_blocking=False)
        return self.buf[key]


def check_step(ctx, policy, qs, Ks, Vs, k, outs, idx_buf, layers=None, say=None, lens=None):
    """Compares the outputs of one hylra_decode_step (outs, idx_buf; contiguous token-level
    layout) with the oracle on every pair of the layers in `layers` (None: all).  lens: the
    per-sequence lengths the step ran with (hylra_decode_step_paged without a block table);
    sequence b is then checked on its first lens[b] rows, its set holds min(k, lens[b]) entries
    and -1 behind them.  Raises AssertionError on the first violation; returns a summary dict."""
    L = len(policy)
    want = set(range(L)) if layers is None else set(int(l) for l in layers)
    src_of = {}
    last_full = -1
    for l in range(L):
        if policy[l] == FULL:
            last_full = l
        src_of[l] = last_full
    need_idx = {src_of[l] for l in want if policy[l] == REUSE}
    need_idx |= {l for l in want if policy[l] == FULL and (l + 1 == L or policy[l + 1] == REUSE)}
    if layers is None:
        need_idx.add(last_full)
    stage = _Stage()
    gpu_idx = {}
    summary = {"layers": 0, "pairs": 0, "max_err_full": 0.0, "max_err_reuse": 0.0, "sets_differing_in_band": 0,
               "oracle_s": 0.0}
    B, Hkv = Ks[0].shape[0], Ks[0].shape[1]
    if lens is not None:
        return _check_step_lens(ctx, policy, qs, Ks, Vs, k, outs, idx_buf, lens, want, need_idx, src_of, last_full,
                                layers is None, stage, summary, say)
    for l in sorted(want | need_idx):
        if policy[l] == REUSE and l not in want:
            continue
        q, K, V = qs[l].cpu(), stage.fetch(Ks[l], "K"), stage.fetch(Vs[l], "V")
        t0 = time.perf_counter()
        if policy[l] == FULL:
            sel = l in need_idx
            ref_out, ref_idx, shat = oracle.full_attn_topk(q, K, V, k, want_out=l in want, want_idx=sel, want_shat=sel)
            summary["oracle_s"] += time.perf_counter() - t0
            if sel:
                _, g = ctx.full_attn_topk(qs[l], Ks[l], Vs[l], k)
                torch.cuda.synchronize()
                gpu_idx[l] = g.cpu().numpy()
                summary["sets_differing_in_band"] += assert_idx_valid(gpu_idx[l], shat, k, "layer %d idx" % l, exact_ref=ref_idx)
            if l in want:
                err = assert_out_close(outs[l].cpu().numpy(), ref_out, "layer %d (Full) out" % l)
                summary["max_err_full"] = max(summary["max_err_full"], err)
        else:
            ref_out = oracle.reuse_sparse_attn(q, K, V, gpu_idx[src_of[l]])
            summary["oracle_s"] += time.perf_counter() - t0
            err = assert_out_close(outs[l].cpu().numpy(), ref_out, "layer %d (Reuse of %d) out" % (l, src_of[l]))
            summary["max_err_reuse"] = max(summary["max_err_reuse"], err)
        if l in want:
            summary["layers"] += 1
            summary["pairs"] += B * Hkv
        if say:
            say("layer %d %s checked on %d pairs" % (l, "Full" if policy[l] == FULL else "Reuse", B * Hkv))
    if layers is None:
        assert np.array_equal(idx_buf.cpu().numpy(), gpu_idx[last_full]), "idx_buf is not the last Full layer's set"
    return summary


def _check_step_lens(ctx, policy, qs, Ks, Vs, k, outs, idx_buf, lens, want, need_idx, src_of, last_full, whole,
                     stage, summary, say):
    """check_step for a step that ran with per-sequence lengths: the oracle is called per
    sequence on the rows that sequence has."""
    from paper_2602_00777_amd import binding

    B, Hkv, N = Ks[0].shape[0], Ks[0].shape[1], Ks[0].shape[2]
    cache = binding.PagedCache(None, 0, N, torch.from_numpy(np.asarray(lens, np.int32)).to(qs[0].device))
    gpu_idx = {}
    for l in sorted(want | need_idx):
        if policy[l] == REUSE and l not in want:
            continue
        q, K, V = qs[l].cpu(), stage.fetch(Ks[l], "K"), stage.fetch(Vs[l], "V")
        got = outs[l].cpu().numpy()
        if policy[l] == FULL and l in need_idx:
            _, g = ctx.full_attn_topk_paged(qs[l], Ks[l], Vs[l], cache, k)
            torch.cuda.synchronize()
            gpu_idx[l] = g.cpu().numpy()
        t0 = time.perf_counter()
        for b in range(B):
            n = int(lens[b])
            kb = min(k, n)
            if n == 0:
                assert np.all(got[b] == 0.0), "layer %d: a sequence without rows must give zeros" % l
                continue
            qb, Kb, Vb = q[b:b + 1], K[b:b + 1, :, :n], V[b:b + 1, :, :n]
            if policy[l] == FULL:
                sel = l in need_idx
                ref_out, ref_idx, shat = oracle.full_attn_topk(qb, Kb, Vb, kb, want_out=l in want, want_idx=sel, want_shat=sel)
                if sel:
                    assert np.all(gpu_idx[l][b, :, kb:] == -1), "layer %d b=%d: entries behind the set" % (l, b)
                    summary["sets_differing_in_band"] += assert_idx_valid(gpu_idx[l][b:b + 1, :, :kb], shat, kb,
                                                                          "layer %d b=%d idx" % (l, b), exact_ref=ref_idx)
                if l in want:
                    err = assert_out_close(got[b:b + 1], ref_out, "layer %d (Full) b=%d out" % (l, b))
                    summary["max_err_full"] = max(summary["max_err_full"], err)
            else:
                ref_out = oracle.reuse_sparse_attn(qb, Kb, Vb, gpu_idx[src_of[l]][b:b + 1])
                err = assert_out_close(got[b:b + 1], ref_out, "layer %d (Reuse of %d) b=%d out" % (l, src_of[l], b))
                summary["max_err_reuse"] = max(summary["max_err_reuse"], err)
        summary["oracle_s"] += time.perf_counter() - t0
        if l in want:
            summary["layers"] += 1
            summary["pairs"] += B * Hkv
        if say:
            say("layer %d %s checked on %d pairs" % (l, "Full" if policy[l] == FULL else "Reuse", B * Hkv))
    if whole:
        assert np.array_equal(idx_buf.cpu().numpy(), gpu_idx[last_full]), "idx_buf is not the last Full layer's set"
    return summary
