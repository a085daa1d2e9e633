"""Pins for the oracle's threshold rule of the autoregressive mode (Sec. 2.4, Eq. 8): calibration of
the threshold on a sample, selection as index lists, and the streaming append to the nugget cache."""
import numpy as np
import pytest
import torch

import oracle
import workloads as W


def _cu(lens):
    return np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)


def test_calibration_closed_forms_and_library_cross_check():
    # a permutation of 0..n-1: the k highest are n-k..n-1, so the threshold is n-k-1 and exactly k exceed it
    rng = np.random.default_rng(7)
    for n, (num, den) in [(10, (1, 5)), (1000, (1, 10)), (4096, (1, 20)), (37, (1, 10))]:
        k = oracle.nugget_count(n, num, den)
        s = rng.permutation(n).astype(np.float32)
        lam = oracle.threshold_from_sample(s, num, den)
        assert lam == n - k - 1
        assert int((s > lam).sum()) == k
    # Gaussian sample: equals the (k+1)-th element of a library sort, and keeps exactly k = ceil(n/r) (r ~ t/k)
    s = W.normal(31, 0, (5000,), 1.0, torch.float32).numpy()
    lam = oracle.threshold_from_sample(s, 1, 10)
    assert lam == np.sort(s)[::-1][500]
    assert int((s > lam).sum()) == 500


def test_calibration_ties_specials_and_keep_everything():
    # ties at the threshold: fewer than k exceed it, at least k+1 reach it
    s = np.array([3, 3, 3, 2, 2, 2, 2, 1, 1, 1], dtype=np.float32)
    lam = oracle.threshold_from_sample(s, 1, 2)  # k = 5 -> 6th highest = 2
    assert lam == 2.0 and (s > lam).sum() == 3 and (s >= lam).sum() >= 6
    # k >= n keeps everything: -inf
    assert oracle.threshold_from_sample(s, 1, 1) == -np.inf
    # NaN ranks lowest; -0 and +0 are one value, reported as +0
    t = np.array([np.nan, 5, np.nan, 1, -0.0, 7], dtype=np.float32)
    assert oracle.threshold_from_sample(t, 1, 3) == 1.0          # k = 2 -> 3rd highest of (7, 5, 1, 0, nan, nan)
    z = oracle.threshold_from_sample(t, 1, 2)                    # k = 3 -> 4th highest = -0 -> +0
    assert z == 0.0 and not np.signbit(np.float32(z))
    assert oracle.threshold_from_sample(t, 4, 6) == -np.inf      # k = 4 -> 5th highest is NaN: keep all


def test_index_lists_match_indicator_and_are_strict():
    s = W.normal(32, 0, (900,), 1.0, torch.float32).numpy()
    s[[5, 17, 400]] = np.nan
    s[[6, 401]] = 0.25
    lens = [200, 0, 300, 400]
    cu = _cu(lens)
    counts, cu_k, idx = oracle.select_threshold_indices(s, cu, 0.25)
    alpha, counts2 = oracle.select_threshold(s, cu, 0.25)
    assert np.array_equal(counts, counts2) and np.array_equal(cu_k, _cu(counts))
    for b in range(len(lens)):
        seg = s[cu[b]:cu[b + 1]]
        want = np.nonzero(seg > np.float32(0.25))[0]          # strict: 0.25 itself and NaN are dropped
        assert np.array_equal(idx[cu_k[b]:cu_k[b + 1]], want)
        assert np.array_equal(np.nonzero(alpha[cu[b]:cu[b + 1]])[0], want)
    # -inf keeps everything but NaN (and -inf itself)
    c3, _, i3 = oracle.select_threshold_indices(s, cu, -np.inf)
    assert int(c3.sum()) == 900 - 3


def test_rule_is_causal_and_agrees_with_topk_at_the_calibrated_threshold():
    s = W.normal(33, 0, (700,), 1.0, torch.float32).numpy()
    lam = oracle.threshold_from_sample(s, 1, 10)
    _, _, full = oracle.select_threshold_indices(s, _cu([700]), lam)
    # Eq. 8 does not look at later tokens: the kept set of a prefix is a prefix of the kept set
    for t in (1, 50, 333, 699):
        _, _, part = oracle.select_threshold_indices(s[:t], _cu([t]), lam)
        assert np.array_equal(part, full[full < t])
    # calibrated on the sequence itself (no ties) the rule keeps exactly the TopK set of Eq. 14
    k = oracle.nugget_count(700, 1, 10)
    topk = oracle.select_topk(s, _cu([700]), _cu([k]), 0)
    assert np.array_equal(full, topk)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_streaming_append_equals_batch_selection_and_gather(dtype):
    B, n, H_kv, d_h, cap = 3, 60, 2, 8, 64
    s = W.normal(34, 0, (B * n,), 1.0, torch.float32).numpy()
    K = W.to_numpy(W.normal(34, 1, (B * n, H_kv, d_h), 1.0, dtype, "cpu"))
    V = W.to_numpy(W.normal(34, 2, (B * n, H_kv, d_h), 1.0, dtype, "cpu"))
    lam = 0.3
    Kn = np.zeros((B, cap, H_kv, d_h), dtype=K.dtype)
    Vn = np.zeros_like(Kn)
    counts = np.zeros(B, dtype=np.int32)
    for t in range(n):  # token t of every sequence leaves the window at step t
        rows = [b * n + t for b in range(B)]
        assert oracle.stream_append(s[rows], lam, K[rows], V[rows], counts, Kn, Vn) == 0
    cu = _cu([n] * B)
    c_ref, cu_k, idx = oracle.select_threshold_indices(s, cu, lam)
    Kg, Vg = oracle.gather(K, V, idx, cu, cu_k)
    assert np.array_equal(counts, c_ref)
    for b in range(B):
        assert np.array_equal(Kn[b, :counts[b]], Kg[cu_k[b]:cu_k[b + 1]])
        assert np.array_equal(Vn[b, :counts[b]], Vg[cu_k[b]:cu_k[b + 1]])
        assert not Kn[b, counts[b]:].any()
    assert not np.array_equal(Kn, Vn)


def test_streaming_append_full_cache_drops_and_reports():
    B, H_kv, d_h, cap = 2, 1, 4, 2
    Kn = np.zeros((B, cap, H_kv, d_h), dtype=np.float32)
    Vn = np.zeros_like(Kn)
    counts = np.array([2, 1], dtype=np.int32)
    rows = np.arange(B * H_kv * d_h, dtype=np.float32).reshape(B, H_kv, d_h) + 1
    dropped = oracle.stream_append(np.array([1.0, 1.0], dtype=np.float32), 0.0, rows, -rows, counts, Kn, Vn)
    assert dropped == 1 and list(counts) == [2, 2]
    assert not Kn[0].any() and np.array_equal(Kn[1, 1], rows[1]) and np.array_equal(Vn[1, 1], -rows[1])
