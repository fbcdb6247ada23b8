"""Comparison rules shared by the GPU parity tests.

Outputs: max over elements of |gpu - ref| / max(|ref|, 1e-2 * max_c |ref[b,h,c]|) must be
<= 2e-3 (fp32 accumulation over bf16 inputs against the fp64 oracle; the floor keeps the
relative error meaningful for components that happen to be near zero).

Index sets: with tau the oracle's k-th largest group-mean score, the GPU set must hold exactly
k distinct in-range positions in ascending order, contain every position whose oracle score
exceeds tau + 1e-4 and none whose score is below tau - 1e-4.  Inside that band the fp32 and
fp64 rankings may legitimately differ.
"""
import numpy as np

OUT_TOL = 2e-3
BAND = 1e-4


def out_error(gpu, ref):
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    floor = 1e-2 * np.max(np.abs(ref), axis=-1, keepdims=True)
    denom = np.maximum(np.abs(ref), np.maximum(floor, 1e-300))
    return float(np.max(np.abs(gpu - ref) / denom))


def assert_out_close(gpu, ref, what=""):
    assert np.all(np.isfinite(np.asarray(gpu))), "non-finite output %s" % what
    err = out_error(gpu, ref)
    assert err <= OUT_TOL, "%s: max relative error %.3e > %.1e" % (what, err, OUT_TOL)
    return err


def assert_idx_valid(gpu_idx, shat, k, what="", exact_ref=None):
    """gpu_idx [B,Hkv,k] int; shat [B,Hkv,N] oracle group-mean scores.  Returns the number of
    (b, g) pairs whose set differs from the oracle's inside the tie band."""
    gpu_idx = np.asarray(gpu_idx)
    B, H, N = shat.shape
    assert gpu_idx.shape == (B, H, k), "%s: idx shape %s" % (what, gpu_idx.shape)
    differing = 0
    for b in range(B):
        for g in range(H):
            ids = gpu_idx[b, g].astype(np.int64)
            assert ids.min() >= 0 and ids.max() < N, "%s: position out of range at (%d,%d)" % (what, b, g)
            assert np.all(np.diff(ids) > 0), "%s: positions not strictly ascending at (%d,%d)" % (what, b, g)
            s = shat[b, g]
            tau = np.partition(s, N - k)[N - k]
            chosen = np.zeros(N, dtype=bool)
            chosen[ids] = True
            must = s > tau + BAND
            never = s < tau - BAND
            assert not np.any(must & ~chosen), "%s: a position above the band is missing at (%d,%d)" % (what, b, g)
            assert not np.any(never & chosen), "%s: a position below the band was chosen at (%d,%d)" % (what, b, g)
            if exact_ref is not None and not np.array_equal(ids, exact_ref[b, g]):
                differing += 1
    return differing
