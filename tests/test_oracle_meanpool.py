"""Pins for the oracle's mean-pool compaction (the pooling baseline of Sec. 5.1: even chunks, one mean per chunk)."""
import numpy as np
import pytest
import torch

import oracle
import workloads as W


def _cu(lens):
    return np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)


def test_chunk_boundaries_read_out_by_one_hot_rows():
    # token t carries e_t: the pooled row j then holds 1/len on exactly the positions of chunk j
    n, k, d = 10, 3, 16
    K = np.zeros((n, 1, d), dtype=np.float32)
    K[np.arange(n), 0, np.arange(n)] = 1.0
    Kn, Vn = oracle.meanpool(K, 2 * K, _cu([n]), _cu([k]))
    want = [(0, 3), (3, 6), (6, 10)]  # floor(j n / k)
    for j, (a, b) in enumerate(want):
        row = np.zeros(d, dtype=np.float32)
        row[a:b] = np.float32(1.0 / (b - a))
        assert np.array_equal(Kn[j, 0], row) and np.array_equal(Vn[j, 0], np.float32(2.0) * row)
    # every token lands in exactly one chunk
    assert np.allclose((Kn[:, 0] > 0).sum(axis=0)[:n], 1)


def test_ratio_one_is_identity_and_constant_rows_stay():
    K = W.to_numpy(W.normal(40, 0, (12, 2, 8), 1.0, torch.bfloat16))
    V = W.to_numpy(W.normal(40, 1, (12, 2, 8), 1.0, torch.bfloat16))
    Kn, Vn = oracle.meanpool(K, V, _cu([5, 7]), _cu([5, 7]))
    assert np.array_equal(Kn, K) and np.array_equal(Vn, V)
    C = np.broadcast_to(K[:1], K.shape).copy()
    Kc, _ = oracle.meanpool(C, C, _cu([12]), _cu([4]))
    assert all(np.array_equal(Kc[j], K[0]) for j in range(4))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_matches_float64_library_mean_with_one_rounding(dtype):
    lens, ks = [37, 100, 8], [4, 10, 8]
    N = sum(lens)
    Kt = W.normal(41, 0, (N, 2, 8), 1.0, dtype)
    Vt = W.normal(41, 1, (N, 2, 8), 1.0, dtype)
    Kn, Vn = oracle.meanpool(W.to_numpy(Kt), W.to_numpy(Vt), _cu(lens), _cu(ks))
    cu, cuk = _cu(lens), _cu(ks)
    for src, got in ((Kt, Kn), (Vt, Vn)):
        x = src.double().numpy()
        for b, (n, k) in enumerate(zip(lens, ks)):
            for j in range(k):
                a, e = cu[b] + j * n // k, cu[b] + (j + 1) * n // k
                want = torch.from_numpy(x[a:e].mean(axis=0)).to(dtype)  # torch rounds float64 -> dtype once, RNE
                assert np.array_equal(got[cuk[b] + j], W.to_numpy(want)), (b, j)


def test_head_major_layout_and_k_v_not_swapped():
    K = W.to_numpy(W.normal(42, 0, (20, 3, 4), 1.0, torch.float32))
    V = W.to_numpy(W.normal(42, 1, (20, 3, 4), 1.0, torch.float32))
    a, b = oracle.meanpool(K, V, _cu([20]), _cu([5]))
    ah, bh = oracle.meanpool(K, V, _cu([20]), _cu([5]), oracle.HEAD_MAJOR)
    assert np.array_equal(ah, a.transpose(1, 0, 2)) and np.array_equal(bh, b.transpose(1, 0, 2))
    assert not np.array_equal(a, b)


def _bf16_value(bits: int):
    from fractions import Fraction
    sign = -1 if bits & 0x8000 else 1
    e, m = (bits >> 7) & 0xFF, bits & 0x7F
    assert 0 < e < 255
    return sign * (Fraction(128 + m, 128) * Fraction(2) ** (e - 127))


def _nearest_bf16_bits(x):
    """Round-to-nearest-even of an exact rational to bf16, by comparing exact distances (normal range only)."""
    start = int(np.array([float(x)], dtype=np.float32).view(np.uint32)[0]) >> 16
    best = None
    for bits in range(start - 2, start + 3):
        dist = abs(_bf16_value(bits) - x)
        if best is None or dist < best[0] or (dist == best[0] and bits % 2 == 0):
            best = (dist, bits)
    return best[1]


@pytest.mark.parametrize("x_bits,y_bits,t_exp,t_sign,trap", [
    (0x3F80, 0x3F81, -40, +1, True),    # mean = midpoint + 2^-42: up, to the odd neighbour (two roundings: even)
    (0x3F80, 0x3F81, -40, -1, False),   # midpoint - 2^-42: down, which is also where a tie would go
    (0x3F81, 0x3F82, -40, +1, False),   # midpoint whose even neighbour is above: up either way
    (0x3F81, 0x3F82, -40, -1, True),    # down, to the odd neighbour
    (0xBF80, 0xBF81, -40, -1, True),    # negative mirror of the first case
    (0x3F80, 0x3F80, -40, -1, False),   # just below a representable value: the fp32 rounding goes up past it
])
def test_one_rounding_in_the_double_rounding_trap(x_bits, y_bits, t_exp, t_sign, trap):
    # A chunk of four bf16 rows {x, y, t, 0} whose exact mean lies 2^-42 away from the midpoint of two bf16
    # values.  Rounding it to fp32 first lands exactly on the midpoint and a second rounding then ties to even;
    # the pooled row is defined with ONE rounding of the exact mean.  Expected bits from exact rationals.
    from fractions import Fraction
    t = t_sign * Fraction(2) ** t_exp
    t_bits = ((127 + t_exp) << 7) | (0x8000 if t_sign < 0 else 0)
    assert _bf16_value(t_bits) == t
    mean = (_bf16_value(x_bits) + _bf16_value(y_bits) + t) / 4
    want = _nearest_bf16_bits(mean)
    two_roundings = int(torch.tensor([float(mean)], dtype=torch.float64).float().bfloat16().view(torch.int16)[0]) & 0xFFFF
    K = np.array([x_bits, y_bits, t_bits, 0], dtype=np.uint16).reshape(4, 1, 1).repeat(8, axis=2)
    Kn, Vn = oracle.meanpool(K, K, _cu([4]), _cu([1]))
    assert int(Kn[0, 0, 0]) == want and int(Vn[0, 0, 3]) == want
    assert (two_roundings != want) == trap  # rounding through fp32 gets the trap cases wrong
