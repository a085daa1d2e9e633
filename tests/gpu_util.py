"""Helpers of the GPU parity tests: run the HIP path through the C-ABI binding and the oracle on the same bits."""
import concurrent.futures
import math
import os

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


def oracle_workers() -> int:
    """Independent single-threaded oracle instances run side by side (the oracle itself has no threads)."""
    return max(1, min(16, os.cpu_count() or 1))


def oracle_attention_rows_parallel(host, Kn, Vn, cu_nuggets, scale, rows):
    """oracle.attention_rows over `rows` ((sequence, head, query row) triples), the list cut into pieces
    that separate single-threaded oracle calls work through side by side (rows are independent).
    host: Q, Kl, Vl, cu_q, cu_local as numpy arrays.  Returns (O float64 [R, d_h], lse float64 [R])."""
    rows = np.asarray(rows, dtype=np.int32).reshape(-1, 3)
    n_workers = oracle_workers()
    pieces = [p for p in np.array_split(np.arange(len(rows)), 8 * n_workers) if len(p)]

    def one(piece):
        return oracle.attention_rows(host["Q"], Kn, Vn, host["Kl"], host["Vl"], host["cu_q"], cu_nuggets,
                                     host["cu_local"], scale, rows[piece])
    with concurrent.futures.ThreadPoolExecutor(max_workers=n_workers) as ex:
        outs = list(ex.map(one, pieces))
    return np.concatenate([o for o, _ in outs]), np.concatenate([l for _, l in outs])


def slab_rows(pairs, q_lens):
    """All query rows of the given (sequence, head) pairs as (b, h, i) triples."""
    return [(b, h, i) for b, h in pairs for i in range(q_lens[b])]


def nan_outputs(Q: torch.Tensor, H: int):
    """Output buffers filled with NaN, so that a row the kernel never wrote cannot pass a comparison."""
    O = torch.full_like(Q, float("nan"))
    lse = torch.full((Q.shape[0], H), float("nan"), dtype=torch.float32, device=Q.device)
    return O, lse


def check_rows(O: torch.Tensor, lse: torch.Tensor, cu_q, rows, O_ref, lse_ref, dtype):
    """Compares the (b, h, i) rows of O [Sq, H, d_h] / lse [Sq, H] with the oracle's, to the bar of check_attention."""
    rows = np.asarray(rows, dtype=np.int64).reshape(-1, 3)
    tok = torch.from_numpy(np.asarray(cu_q, dtype=np.int64)[rows[:, 0]] + rows[:, 2]).to(O.device)
    hh = torch.from_numpy(rows[:, 1]).to(O.device)
    err = check_attention(O[tok, hh], O_ref, dtype)
    check_lse(lse[tok, hh], lse_ref, dtype)
    return err
