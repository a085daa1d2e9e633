"""Helpers of the GPU parity tests: run the HIP path through the C-ABI binding and the oracle on the same bits."""
import math

import numpy as np
import torch

import oracle
import workloads as W


def dev():
    return torch.device("cuda:0")


def oracle_counts(seq_lens, num, den):
    ks = [oracle.nugget_count(n, num, den) for n in seq_lens]
    return ks, oracle.cu_from_lengths(ks)


def check_attention(O_gpu: torch.Tensor, O_ref: np.ndarray, dtype: torch.dtype):
    """The bar: fp32 -> max error relative to the largest reference magnitude <= 1e-5 and an
    element-wise |err| <= 1e-5 |ref| + 1e-6;  bf16 -> max absolute error <= 2e-2."""
    got = O_gpu.detach().float().cpu().double().numpy()
    assert np.all(np.isfinite(got))
    err = np.abs(got - O_ref)
    if dtype == torch.float32:
        denom = max(1e-30, np.max(np.abs(O_ref)))
        assert err.max() / denom <= 1e-5, f"fp32 max normalised error {err.max() / denom:.3e}"
        assert np.all(err <= 1e-5 * np.abs(O_ref) + 1e-6), f"fp32 element-wise bound broken, max err {err.max():.3e}"
    else:
        assert err.max() <= 2e-2, f"bf16 max abs error {err.max():.3e}"
    return float(err.max())


def check_lse(lse_gpu: torch.Tensor, lse_ref: np.ndarray, dtype: torch.dtype):
    got = lse_gpu.detach().cpu().double().numpy()
    inf_ref = np.isneginf(lse_ref)
    assert np.array_equal(np.isneginf(got), inf_ref)
    tol = 1e-5 if dtype == torch.float32 else 2e-2
    fin = ~inf_ref
    if fin.any():
        assert np.max(np.abs(got[fin] - lse_ref[fin]) / (1 + np.abs(lse_ref[fin]))) <= tol


def make_attention_case(seed, q_lens, k_lens, m_lens, H, H_kv, d_h, dtype, device):
    Sq, Kt, Sm = sum(q_lens), sum(k_lens), sum(m_lens)
    mk = lambda tid, n, h: W.normal(seed, tid, (n, h, d_h), 1.0, dtype, "cpu")
    t = dict(Q=mk(0, Sq, H), Kn=mk(1, Kt, H_kv), Vn=mk(2, Kt, H_kv), Kl=mk(3, Sm, H_kv), Vl=mk(4, Sm, H_kv))
    cu = dict(cu_q=W.cumulative(q_lens), cu_nuggets=W.cumulative(k_lens), cu_local=W.cumulative(m_lens))
    host = {k: W.to_numpy(v) for k, v in {**t, **cu}.items()}
    devt = {k: v.to(device) for k, v in {**t, **cu}.items()}
    return host, devt


def default_scale(d_h):
    return 1.0 / math.sqrt(d_h)
