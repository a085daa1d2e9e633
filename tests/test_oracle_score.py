"""Pins for the oracle Scorer (Eq. 6 / Eq. 15 as a linear head d -> 1)."""
import numpy as np
import torch

import oracle
import workloads as W


def _bf16(t):
    return W.to_numpy(t.to(torch.bfloat16))


def test_unit_weight_reads_out_a_channel():
    x = W.normal(11, 0, (37, 24), 1.0, torch.float32)
    for c in (0, 5, 23):
        w = torch.zeros(24)
        w[c] = 1.0
        s = oracle.score(x.numpy(), w.numpy())
        assert np.array_equal(s, x[:, c].numpy())
    xb = x.to(torch.bfloat16)
    w = torch.zeros(24, dtype=torch.bfloat16)
    w[7] = 1.0
    assert np.array_equal(oracle.score(W.to_numpy(xb), W.to_numpy(w)), xb[:, 7].float().numpy())


def test_integer_inputs_give_exact_sums():
    x, w = W.exact_arithmetic_inputs(5, 64, 256, torch.float32)
    s = oracle.score(x.numpy(), w.numpy())
    exact = (x.to(torch.int64) * torch.round(w * 64).to(torch.int64)).sum(1).double() / 64.0
    assert np.array_equal(s.astype(np.float64), exact.numpy())
    xb, wb = W.exact_arithmetic_inputs(5, 64, 256, torch.bfloat16)
    assert np.array_equal(oracle.score(W.to_numpy(xb), W.to_numpy(wb)), s)


def test_matches_float64_library_matvec():
    for dtype in (torch.float32, torch.bfloat16):
        x = W.normal(12, 0, (129, 200), 1.0, dtype)
        w = W.normal(12, 1, (200,), 200 ** -0.5, dtype)
        s = oracle.score(W.to_numpy(x), W.to_numpy(w), bias=0.25)
        ref = torch.mv(x.double(), w.double()) + 0.25
        # one fp32 rounding of a double sum; the library may sum in another order
        assert np.allclose(s, ref.numpy(), rtol=0, atol=1e-6)
        assert np.max(np.abs(s.astype(np.float64) - ref.numpy())) <= 2.5e-7 * (1 + np.max(np.abs(ref.numpy())))


def test_linearity_in_the_weight_and_bias_shift():
    x = W.normal(13, 0, (50, 64), 1.0, torch.float32)
    w1 = W.integers(13, 1, (64,), -3, 3).float()
    w2 = W.integers(13, 2, (64,), -3, 3).float()
    xi = W.integers(13, 3, (50, 64), -5, 5).float()
    s1, s2 = oracle.score(xi.numpy(), w1.numpy()), oracle.score(xi.numpy(), w2.numpy())
    s12 = oracle.score(xi.numpy(), (w1 + w2).numpy())
    assert np.array_equal(s12, s1 + s2)  # all exact in fp32
    assert np.array_equal(oracle.score(xi.numpy(), w1.numpy(), bias=3.0), s1 + 3.0)
    del x


def test_transposed_operand_or_dropped_term_would_fail():
    # a non-symmetric case whose answer is known in closed form: x[t, c] = t + 1 if c == t % d else 0
    N, d = 12, 5
    x = np.zeros((N, d), dtype=np.float32)
    for t in range(N):
        x[t, t % d] = t + 1
    w = np.arange(1, d + 1, dtype=np.float32)
    s = oracle.score(x, w)
    assert np.array_equal(s, np.array([(t + 1) * (t % d + 1) for t in range(N)], dtype=np.float32))


def test_negative_zero_is_canonicalised():
    x = np.array([[-1.0, 0.0]], dtype=np.float32)
    w = np.array([0.0, 1.0], dtype=np.float32)
    s = oracle.score(x, w)
    assert s[0] == 0 and not np.signbit(s[0])


def test_score_layers_is_the_scorer_layer_by_layer():
    L, N, d = 3, 17, 24
    x = W.normal(31, 0, (L, N, d), 1.0, torch.float32)
    w = W.normal(31, 1, (L, d), 0.3, torch.float32)
    b = np.array([0.5, -1.25, 0.0], dtype=np.float32)
    got = oracle.score_layers(x.numpy(), w.numpy(), b)
    want = (torch.einsum("lnd,ld->ln", x.double(), w.double()) + torch.from_numpy(b).double()[:, None]).float().numpy()
    assert np.array_equal(got, want)  # float64 sums of 24 products, rounded once
    assert np.array_equal(oracle.score_layers(x.numpy(), w.numpy())[1], oracle.score(x[1].numpy(), w[1].numpy()))
