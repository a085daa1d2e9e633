"""GPU parity: dodo_ste_score_grad (fed with O and lse of the HIP forward call) against the oracle."""
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


def _case(seed, q_lens, k_lens, m_lens, H, H_kv, d_h, dtype):
    mk = lambda tid, n, h: W.normal(seed, tid, (n, h, d_h), 1.0, dtype)
    t = dict(Q=mk(0, sum(q_lens), H), Kn=mk(1, sum(k_lens), H_kv), Vn=mk(2, sum(k_lens), H_kv),
             Kl=mk(3, sum(m_lens), H_kv), Vl=mk(4, sum(m_lens), H_kv), dO=mk(5, sum(q_lens), H))
    cu = [oracle.cu_from_lengths(x) for x in (q_lens, k_lens, m_lens)]
    return t, cu


def _gpu(D, t, cu, q_lens, k_lens, m_lens, scale, grad_scale, layout=0, grad=None, accumulate=False):
    d = {k: v.to(dev()) for k, v in t.items()}
    cu_q, cu_k, cu_l = (torch.from_numpy(c).to(dev()) for c in cu)
    O, lse = D.dodo_nugget_attention(d["Q"], d["Kn"], d["Vn"], d["Kl"], d["Vl"], cu_q, cu_k, cu_l, max(q_lens),
                                     max(k_lens), max(m_lens), scale, want_lse=True)
    Kn, Vn = d["Kn"], d["Vn"]
    if layout == 1:
        Kn, Vn = Kn.permute(1, 0, 2).contiguous(), Vn.permute(1, 0, 2).contiguous()
    return D.dodo_ste_score_grad(d["Q"], Kn, Vn, d["dO"], O, lse, cu_q, cu_k, max(q_lens), max(k_lens), scale, grad_scale,
                                 layout, grad=grad, accumulate=accumulate)


def _check(got, want, dtype):
    """fp32: |err| <= 1e-5 of the largest gradient.  bf16: 2e-2 of it -- O comes back rounded to bf16 (relative
    2^-9), which moves D[j] = dO[j].O[j] by a few 1e-3 per row, and the rows' errors add up like a random walk."""
    got = got.cpu().double().numpy()
    ref = max(np.abs(want).max(), 1e-30)
    tol = 1e-5 if dtype == torch.float32 else 2e-2
    assert np.all(np.isfinite(got))
    assert np.abs(got - want).max() <= tol * ref, f"max err {np.abs(got - want).max():.3e} vs scale {ref:.3e}"


@pytest.mark.parametrize("dtype,H,H_kv,d_h", [(torch.float32, 4, 2, 64), (torch.float32, 2, 2, 128),
                                              (torch.bfloat16, 4, 4, 64)])
def test_plain_kernel(D, dtype, H, H_kv, d_h):
    q_lens, k_lens, m_lens = [7, 3, 40, 4, 0], [6, 0, 19, 2, 5], [9, 3, 0, 2, 4]
    t, cu = _case(700, q_lens, k_lens, m_lens, H, H_kv, d_h, dtype)
    scale = d_h ** -0.5
    want = oracle.ste_score_grad(*(W.to_numpy(t[k]) for k in ("Q", "Kn", "Vn", "Kl", "Vl", "dO")), *cu, scale, scale)
    _check(_gpu(D, t, cu, q_lens, k_lens, m_lens, scale, scale), want, dtype)


@pytest.mark.parametrize("q_lens,k_lens,m_lens,H,H_kv", [
    ([128], [64], [128], 2, 2),
    ([100, 37, 256, 16, 0], [13, 200, 0, 77, 9], [150, 37, 300, 16, 3], 4, 2),   # ragged, GQA, partial tiles, no queries
    ([300], [103], [300], 3, 1),
    ([33, 200], [130, 65], [0, 100], 2, 2),
    ([1100, 70], [600, 257], [1200, 70], 2, 1),   # three nugget tiles per workgroup row, 35 query tiles
])
def test_mfma_kernel_bf16(D, q_lens, k_lens, m_lens, H, H_kv):
    t, cu = _case(701, q_lens, k_lens, m_lens, H, H_kv, 128, torch.bfloat16)
    scale = 128 ** -0.5
    want = oracle.ste_score_grad(*(W.to_numpy(t[k]) for k in ("Q", "Kn", "Vn", "Kl", "Vl", "dO")), *cu, scale, 1.0)
    got = _gpu(D, t, cu, q_lens, k_lens, m_lens, scale, 1.0)
    _check(got, want, torch.bfloat16)
    # head-major cache: the same sums
    got_hm = _gpu(D, t, cu, q_lens, k_lens, m_lens, scale, 1.0, layout=1)
    assert torch.equal(got, got_hm)


def test_accumulates_over_layers_and_is_deterministic(D):
    q_lens, k_lens, m_lens, H = [90, 64], [70, 20], [100, 64], 4
    scale = 128 ** -0.5
    total = np.zeros(sum(k_lens))
    grad = torch.full((sum(k_lens),), 123.0, device=dev())  # overwritten by the first layer
    for layer in range(3):
        t, cu = _case(710 + layer, q_lens, k_lens, m_lens, H, H, 128, torch.bfloat16)
        total += oracle.ste_score_grad(*(W.to_numpy(t[k]) for k in ("Q", "Kn", "Vn", "Kl", "Vl", "dO")), *cu, scale, scale)
        _gpu(D, t, cu, q_lens, k_lens, m_lens, scale, scale, grad=grad, accumulate=layer > 0)
    _check(grad, total, torch.bfloat16)
    first = _gpu(D, t, cu, q_lens, k_lens, m_lens, scale, scale).clone()
    for _ in range(5):
        assert torch.equal(_gpu(D, t, cu, q_lens, k_lens, m_lens, scale, scale), first)


def test_prefill_shape_two_sequences(D):
    # workload-2 shape per sequence (512 query rows, 410 nuggets, 640 local rows), 8 heads
    q_lens, k_lens, m_lens, H = [512, 512], [410, 410], [640, 640], 8
    t, cu = _case(720, q_lens, k_lens, m_lens, H, H, 128, torch.bfloat16)
    scale = 128 ** -0.5
    want = oracle.ste_score_grad(*(W.to_numpy(t[k]) for k in ("Q", "Kn", "Vn", "Kl", "Vl", "dO")), *cu, scale, scale)
    _check(_gpu(D, t, cu, q_lens, k_lens, m_lens, scale, scale), want, torch.bfloat16)
