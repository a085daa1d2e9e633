"""Pins for the oracle's 2-layer scorer (Sec. 2.1 / App. B: a feedforward network d -> d_hid -> 1)."""
import math

import numpy as np
import pytest
import torch

import oracle
import workloads as W


def test_hand_values_of_the_three_activations():
    x = np.zeros((1, 2), dtype=np.float32)            # zero input: s = w2 . act(b1) + b2
    W1 = np.ones((2, 2), dtype=np.float32)
    b1 = np.array([1.0, -1.0], dtype=np.float32)
    w2 = np.array([2.0, 3.0], dtype=np.float32)
    phi1 = 0.5 * (1 + math.erf(1 / math.sqrt(2)))     # Phi(1) = 0.8413...
    assert oracle.score_mlp(x, W1, b1, w2, 0.5, oracle.RELU)[0] == np.float32(2.5)
    assert oracle.score_mlp(x, W1, b1, w2, 0.0, oracle.GELU)[0] == np.float32(2 * phi1 - 3 * (1 - phi1))
    assert oracle.score_mlp(x, W1, b1, w2, 0.0, oracle.TANH)[0] == np.float32(-math.tanh(1.0))


def test_relu_on_positive_preactivations_is_the_linear_scorer_through_a_permutation():
    # W1 = permutation matrix, b1 large: h = P x + c > 0, so s = (P^T w2) . x + c sum(w2) + b2 -- a
    # transposed W1 would apply P^T instead of P
    d, N = 16, 9
    rng = np.random.default_rng(3)
    perm = rng.permutation(d)
    P = np.zeros((d, d), dtype=np.float32)
    P[np.arange(d), perm] = 1.0                       # (P x)[j] = x[perm[j]]
    x = rng.integers(-4, 5, size=(N, d)).astype(np.float32)
    w2 = (rng.integers(-2, 3, size=d) / 4).astype(np.float32)
    c = np.float32(8.0)
    got = oracle.score_mlp(x, P, np.full(d, c, dtype=np.float32), w2, 0.25, oracle.RELU)
    w_eff = np.zeros(d, dtype=np.float32)
    w_eff[perm] = w2                                  # P^T w2
    want = oracle.score(x, w_eff, float(c * w2.sum() + 0.25))
    assert np.array_equal(got, want)                  # small integers and quarters: exact
    w_wrong = w2[perm]                                # what P^T in place of P would give
    assert not np.array_equal(got, oracle.score(x, w_wrong, float(c * w2.sum() + 0.25)))


@pytest.mark.parametrize("act,fn", [(0, torch.relu), (1, lambda h: torch.nn.functional.gelu(h)), (2, torch.tanh)])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_matches_float64_library_composition(act, fn, dtype):
    N, d, dh = 33, 48, 40
    x = W.normal(50, 0, (N, d), 1.0, dtype)
    W1 = W.normal(50, 1, (dh, d), d ** -0.5, dtype)
    b1 = W.normal(50, 2, (dh,), 0.5, torch.float32)
    w2 = W.normal(50, 3, (dh,), dh ** -0.5, dtype)
    got = oracle.score_mlp(W.to_numpy(x), W.to_numpy(W1), b1.numpy(), W.to_numpy(w2), 0.125, act)
    want = (fn(x.double() @ W1.double().T + b1.double()) @ w2.double() + 0.125).float().numpy()
    assert np.allclose(got, want, rtol=0, atol=2e-7 * (1 + np.abs(want).max()))


def test_negative_zero_is_canonicalised_and_bias_shifts():
    x = np.zeros((2, 4), dtype=np.float32)
    W1 = np.zeros((3, 4), dtype=np.float32)
    z = oracle.score_mlp(x, W1, np.zeros(3, dtype=np.float32), -np.ones(3, dtype=np.float32), 0.0, oracle.TANH)
    assert not np.signbit(z).any()
    s = oracle.score_mlp(x, W1, np.ones(3, dtype=np.float32), np.ones(3, dtype=np.float32), 1.5, oracle.RELU)
    assert np.array_equal(s, np.full(2, 4.5, dtype=np.float32))
