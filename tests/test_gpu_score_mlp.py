"""GPU parity of dodo_score_mlp (2-layer scorer of App. B) against the oracle.

Tolerance: |s - s_ref| <= 1e-4 (1 + |s_ref|).  bf16 products are exact in fp32; the d-term sums inside the
MFMA and the d_hid-term sum of w2 * act(h) are fp32 in an order that differs from the oracle's: with
d = d_hid = 4096, O(1) pre-activations and scores, the accumulated rounding is a few 1e-6 (observed),
erff / tanhf add about 1e-7 relative per term."""
import numpy as np
import pytest
import torch

import oracle
import workloads as W
from gpu_util import dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def D():
    import paper_2310_02409_amd as D
    return D


def _case(seed, N, d, dh, dtype):
    x = W.normal(seed, 0, (N, d), 1.0, dtype)
    W1 = W.normal(seed, 1, (dh, d), d ** -0.5, dtype)
    b1 = W.normal(seed, 2, (dh,), 0.5, torch.float32)
    w2 = W.normal(seed, 3, (dh,), dh ** -0.5, dtype)
    return x, W1, b1, w2


def _check(got, want):
    err = np.abs(got - want)
    assert np.all(err <= 1e-4 * (1 + np.abs(want))), f"max err {err.max():.3e}"
    return float(err.max())


@pytest.mark.parametrize("N,d,dh", [(300, 64, 256), (257, 128, 512), (1000, 256, 768), (5, 64, 256), (700, 192, 256),
                                    (300, 64, 1280)])  # 5 hidden tiles over 4 splits: one split has none
@pytest.mark.parametrize("act", [0, 1, 2])
def test_mfma_path_small_shapes(D, N, d, dh, act):
    x, W1, b1, w2 = _case(900 + N, N, d, dh, torch.bfloat16)
    want = oracle.score_mlp(W.to_numpy(x), W.to_numpy(W1), b1.numpy(), W.to_numpy(w2), 0.25, act)
    got = D.dodo_score_mlp(x.to(dev()), W1.to(dev()), b1.to(dev()), w2.to(dev()), 0.25, act).cpu().numpy()
    _check(got, want)


@pytest.mark.parametrize("dtype,N,d,dh", [(torch.float32, 512, 256, 256), (torch.bfloat16, 37, 40, 100),
                                          (torch.float32, 9, 24, 7)])
def test_plain_path_any_shape(D, dtype, N, d, dh):
    x, W1, b1, w2 = _case(950 + N, N, d, dh, dtype)
    for act in (0, 1, 2):
        want = oracle.score_mlp(W.to_numpy(x), W.to_numpy(W1), b1.numpy(), W.to_numpy(w2), -0.5, act)
        got = D.dodo_score_mlp(x.to(dev()), W1.to(dev()), b1.to(dev()), w2.to(dev()), -0.5, act).cpu().numpy()
        _check(got, want)


def test_row_stride_and_determinism(D):
    N, d, dh = 600, 64, 256
    x, W1, b1, w2 = _case(960, N, d, dh, torch.bfloat16)
    wide = torch.zeros((N, d + 24), dtype=torch.bfloat16)
    wide[:, :d] = x
    want = oracle.score_mlp(W.to_numpy(x), W.to_numpy(W1), b1.numpy(), W.to_numpy(w2), 0.0, 1)
    a = D.dodo_score_mlp(wide.to(dev())[:, :d], W1.to(dev()), b1.to(dev()), w2.to(dev()), 0.0, 1)
    b = D.dodo_score_mlp(wide.to(dev())[:, :d], W1.to(dev()), b1.to(dev()), w2.to(dev()), 0.0, 1)
    _check(a.cpu().numpy(), want)
    assert torch.equal(a, b)


def test_llama7b_shape_sampled_tokens(D):
    # the paper's scorer size: d = d_hid = 4096 (16.8 M parameters) on the prefill workload's 32768 tokens
    wl = W.config(2)
    N, d = wl.N, wl.d_model
    x = W.make_inputs(wl, dev(), which=["hidden"])["hidden"]
    W1 = W.normal(wl.seed, 40, (d, d), d ** -0.5, torch.bfloat16, dev())
    b1 = W.normal(wl.seed, 41, (d,), 0.5, torch.float32, dev())
    w2 = W.normal(wl.seed, 42, (d,), d ** -0.5, torch.bfloat16, dev())
    got = D.dodo_score_mlp(x, W1, b1, w2, 0.125, 1)
    rows = [0, 1, 255, 256, 4095, 4096, 17000, 32767] + [int(v) for v in np.random.default_rng(1).integers(0, N, 8)]
    want = oracle.score_mlp(W.to_numpy(x[rows].cpu()), W.to_numpy(W1.cpu()), b1.cpu().numpy(), W.to_numpy(w2.cpu()), 0.125, 1)
    _check(got[rows].cpu().numpy(), want)
