"""Pins for the oracle TopK selection (Eq. 14, tie-break lowest index, optional force-last)."""
import numpy as np
import pytest
import torch

import oracle
import workloads as W


def _cu(lengths):
    return oracle.cu_from_lengths(lengths)


def _ordkey(f: np.float32) -> int:
    """Order-preserving integer image of an fp32 score: NaN lowest, -0 == +0."""
    if np.isnan(f):
        return 0
    if f == 0:
        f = np.float32(0.0)
    u = int(np.array(f, dtype=np.float32).view(np.uint32))
    return (u ^ 0xFFFFFFFF) if (u >> 31) else (u | 0x80000000)


def brute_force(scores, n_lens, k_lens, force_last=False):
    """Top-k of distinct 64-bit composites (key << 32 | ~index): exactly one right answer."""
    out, off = [], 0
    for n, k in zip(n_lens, k_lens):
        s = scores[off:off + n]
        comp = [(_ordkey(s[i]) << 32) | (0xFFFFFFFF - i) for i in range(n)]
        if force_last and n > 0:
            comp[n - 1] = (1 << 64) | (0xFFFFFFFF - (n - 1))
        top = sorted(range(n), key=lambda i: comp[i], reverse=True)[:k]
        out.extend(sorted(top))
        off += n
    return np.array(out, dtype=np.int32)


def _run(scores, n_lens, k_lens, flags=0):
    return oracle.select_topk(np.asarray(scores, dtype=np.float32), _cu(n_lens), _cu(k_lens), flags)


def test_closed_forms():
    n, k = 100, 13
    assert list(_run(np.full(n, 2.5), [n], [k])) == list(range(k))  # all tied: first k
    assert list(_run(-np.arange(n), [n], [k])) == list(range(k))  # strictly decreasing: first k
    assert list(_run(np.arange(n), [n], [k])) == list(range(n - k, n))  # strictly increasing: last k
    perm = W.integers(3, 0, (n,), 0, 10**9).argsort().numpy().astype(np.float32)
    got = _run(perm, [n], [k])
    assert list(got) == sorted(np.nonzero(perm >= n - k)[0])
    # two levels: all highs, then the lowest-index lows
    s = np.zeros(n, dtype=np.float32)
    highs = [90, 4, 57, 33]
    s[highs] = 1.0
    lows = [i for i in range(n) if i not in highs][: k - len(highs)]
    assert list(_run(s, [n], [k])) == sorted(highs + lows)


def test_ratio_one_selects_everything_and_k_zero_is_empty():
    s = W.normal(4, 0, (77,), 1.0, torch.float32).numpy()
    assert list(_run(s, [77], [77])) == list(range(77))
    assert len(_run(s, [77], [0])) == 0
    assert list(_run(s, [40, 0, 37], [4, 0, 37])[4:]) == list(range(37))


@pytest.mark.parametrize("seed", range(6))
def test_brute_force_random_ragged_with_ties(seed):
    n_lens = [int(v) for v in W.integers(seed, 1, (5,), 1, 300)]
    k_lens = [oracle.nugget_count(n, 1, 7) for n in n_lens]
    s = W.normal(seed, 2, (sum(n_lens),), 1.0, torch.float32)
    if seed % 2:
        s = W.quantise16(s)  # heavy ties
    s = s.numpy()
    for fl in (0, oracle.FORCE_LAST):
        got = _run(s, n_lens, k_lens, fl)
        assert np.array_equal(got, brute_force(s, n_lens, k_lens, bool(fl)))


def test_specials_nan_inf_signed_zero():
    s = np.array([np.nan, -np.inf, 0.0, -0.0, np.inf, 1.0, -1.0, np.nan, 0.0, np.inf], dtype=np.float32)
    n = len(s)
    for k in range(n + 1):
        assert np.array_equal(_run(s, [n], [k]), brute_force(s, [n], [k]))
    # ordering spelled out: +inf (4, 9), 1.0 (5), zeros by index (2, 3, 8), -1, -inf, NaNs by index
    order = [4, 9, 5, 2, 3, 8, 6, 1, 0, 7]
    for k in range(n + 1):
        assert list(_run(s, [n], [k])) == sorted(order[:k])


def test_invariants_and_monotone_maps():
    n_lens = [257, 64, 1, 1000]
    k_lens = [oracle.nugget_count(n, 1, 10) for n in n_lens]
    s = W.quantise16(W.normal(9, 0, (sum(n_lens),), 1.0, torch.float32)).numpy()
    idx = _run(s, n_lens, k_lens)
    off = ko = 0
    for n, k in zip(n_lens, k_lens):
        sel = idx[ko:ko + k]
        seg = s[off:off + n]
        assert len(sel) == k and np.all(np.diff(sel) > 0) and sel.min() >= 0 and sel.max() < n
        mask = np.zeros(n, bool)
        mask[sel] = True
        if k < n:
            assert seg[mask].min() >= seg[~mask].max()
            tied_out = np.nonzero(~mask & (seg == seg[mask].min()))[0]
            tied_in = np.nonzero(mask & (seg == seg[mask].min()))[0]
            if len(tied_out):
                assert tied_out.min() > tied_in.max()
        off, ko = off + n, ko + k
    # exact strictly monotone maps leave the selection unchanged (cf. the sigmoid of Eq. 6)
    assert np.array_equal(_run(2 * s, n_lens, k_lens), idx)
    assert np.array_equal(_run(s + 16, n_lens, k_lens), idx)
    sig = 1.0 / (1.0 + np.exp(-s.astype(np.float64)))  # 16 distinct levels stay distinct in fp32
    assert np.array_equal(_run(sig.astype(np.float32), n_lens, k_lens), idx)


def test_force_last_always_contains_last_token():
    n_lens = [50, 3, 1]
    k_lens = [5, 1, 1]
    s = np.concatenate([np.linspace(5, 0, 50), [9, 8, 7], [1]]).astype(np.float32)
    got = _run(s, n_lens, k_lens, oracle.FORCE_LAST)
    assert list(got[:5]) == [0, 1, 2, 3, 49]
    assert list(got[5:]) == [2, 0]
    # even against a +inf elsewhere and k = 1
    s2 = np.array([np.inf, 0, 0, -5], dtype=np.float32)
    assert list(_run(s2, [4], [1], oracle.FORCE_LAST)) == [3]
    assert list(_run(s2, [4], [2], oracle.FORCE_LAST)) == [0, 3]


def test_library_cross_check_tie_free():
    n, k = 4096, 410
    s = W.normal(21, 0, (n,), 1.0, torch.float32)
    assert len(torch.unique(s)) == n
    want = torch.topk(s, k).indices.sort().values.numpy()
    assert np.array_equal(_run(s.numpy(), [n], [k]), want)
    st = torch.sort(W.quantise16(s), descending=True, stable=True).indices[:k].sort().values.numpy()
    assert np.array_equal(_run(W.quantise16(s).numpy(), [n], [k]), st)


def test_k_above_n_is_rejected():
    with pytest.raises(ValueError):
        _run(np.zeros(4), [4], [5])


def test_threshold_rule_matches_indicator():
    s = W.normal(30, 0, (500,), 1.0, torch.float32).numpy()
    alpha, counts = oracle.select_threshold(s, _cu([200, 300]), 0.5)
    assert np.array_equal(alpha, (s > 0.5).astype(np.uint8))
    assert list(counts) == [int((s[:200] > 0.5).sum()), int((s[200:] > 0.5).sum())]
    # strict inequality: a score equal to the threshold is dropped
    a2, _ = oracle.select_threshold(np.array([0.5, 0.6], dtype=np.float32), _cu([2]), 0.5)
    assert list(a2) == [0, 1]
