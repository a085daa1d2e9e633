"""GPU parity: dodo_nugget_attention_indexed (nuggets read in place through the index list) against the
oracle, and bit for bit against the HIP gather followed by the HIP attention."""
import numpy as np
import pytest
import torch

import oracle
import workloads as W
from gpu_util import check_attention, check_lse, default_scale, dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def D():
    import paper_2310_02409_amd as D
    return D


def _case(seed, n_lens, k_lens, q_lens, m_lens, H, H_kv, d_h, dtype, pad_heads=0):
    N, Sq, Sm = sum(n_lens), sum(q_lens), sum(m_lens)
    mk = lambda tid, n, h: W.normal(seed, tid, (n, h, d_h), 1.0, dtype, "cpu")
    K, V = mk(0, N, H_kv + pad_heads), mk(1, N, H_kv + pad_heads)
    t = dict(Q=mk(2, Sq, H), Kl=mk(3, Sm, H_kv), Vl=mk(4, Sm, H_kv))
    s = W.normal(seed, 5, (N,), 1.0, torch.float32).numpy()
    cu_s, cu_k = oracle.cu_from_lengths(n_lens), oracle.cu_from_lengths(k_lens)
    idx = oracle.select_topk(s, cu_s, cu_k)
    cu = dict(cu_s=cu_s, cu_k=cu_k, cu_q=oracle.cu_from_lengths(q_lens), cu_l=oracle.cu_from_lengths(m_lens), idx=idx)
    host = {k: W.to_numpy(v) for k, v in t.items()}
    host.update(K=W.to_numpy(K[:, :H_kv].contiguous()), V=W.to_numpy(V[:, :H_kv].contiguous()), **cu)
    devt = {k: v.to(dev()) for k, v in t.items()}
    devt.update({k: torch.from_numpy(v).to(dev()) for k, v in cu.items()})
    devt.update(K=K.to(dev())[:, :H_kv], V=V.to(dev())[:, :H_kv])  # views: token stride (H_kv + pad_heads) d_h
    return host, devt


def _check(D, seed, n_lens, k_lens, q_lens, m_lens, H, H_kv, d_h, dtype, pad_heads=0):
    host, d = _case(seed, n_lens, k_lens, q_lens, m_lens, H, H_kv, d_h, dtype, pad_heads)
    scale = default_scale(d_h)
    O_ref, lse_ref = oracle.attention_indexed(host["Q"], host["K"], host["V"], host["idx"], host["cu_s"], host["Kl"],
                                              host["Vl"], host["cu_q"], host["cu_k"], host["cu_l"], scale)
    O, lse = D.dodo_nugget_attention_indexed(d["Q"], d["K"], d["V"], d["idx"], d["cu_s"], d["Kl"], d["Vl"], d["cu_q"],
                                             d["cu_k"], d["cu_l"], max(q_lens), max(k_lens), max(m_lens), max(n_lens),
                                             scale, want_lse=True)
    check_attention(O, O_ref, dtype)
    check_lse(lse, lse_ref, dtype)
    # the same arithmetic in the same order as the packed form: identical bits
    Kn, Vn = D.dodo_gather_nuggets(d["K"].contiguous(), d["V"].contiguous(), d["idx"], d["cu_s"], d["cu_k"],
                                   int(host["cu_k"][-1]))
    O2, lse2 = D.dodo_nugget_attention(d["Q"], Kn, Vn, d["Kl"], d["Vl"], d["cu_q"], d["cu_k"], d["cu_l"], max(q_lens),
                                       max(k_lens), max(m_lens), scale, want_lse=True)
    assert torch.equal(O, O2) and torch.equal(lse, lse2)


@pytest.mark.parametrize("dtype,H,H_kv,d_h", [(torch.float32, 4, 4, 64), (torch.bfloat16, 8, 2, 128),
                                              (torch.bfloat16, 4, 4, 64), (torch.float32, 4, 2, 128)])
def test_decode_ragged(D, dtype, H, H_kv, d_h):
    n_lens = [2050, 4100, 999, 1, 7]
    k_lens = [205, 410, 333, 1, 0]
    _check(D, 500, n_lens, k_lens, [1] * 5, [257, 257, 40, 3, 5], H, H_kv, d_h, dtype)


def test_decode_split_k_and_padded_token_stride(D):
    _check(D, 501, [9000, 4000], [3277, 1500], [1, 1], [1089, 1025], 2, 2, 128, torch.bfloat16, pad_heads=1)


@pytest.mark.parametrize("n_lens,k_lens,q_lens,m_lens,H,H_kv", [
    ([700], [64], [128], [128], 2, 2),                                       # 4-wavefront kernel
    ([4096, 4096], [410, 410], [512, 512], [640, 640], 4, 4),                # workload-2 shape, fewer heads
    ([130, 2000, 5, 800], [13, 200, 0, 77], [100, 37, 256, 16], [150, 37, 300, 16], 4, 2),  # ragged, GQA, partial tiles
    ([1030], [103], [300], [300], 3, 1),                                     # compressor mode
    ([5000, 90], [500, 9], [64, 200], [0, 100], 2, 2),                       # nuggets only; short local buffer
])
def test_block_kernel_bf16(D, n_lens, k_lens, q_lens, m_lens, H, H_kv):
    _check(D, 502, n_lens, k_lens, q_lens, m_lens, H, H_kv, 128, torch.bfloat16)
    _check(D, 505, n_lens, k_lens, q_lens, m_lens, H, H_kv, 64, torch.bfloat16)


def test_block_kernel_padded_token_stride_and_long_index_list(D):
    _check(D, 503, [20000], [4000], [256], [256], 2, 1, 128, torch.bfloat16, pad_heads=1)


def test_limits_are_reported(D):
    # more nuggets in a sequence than the query-block kernel keeps in LDS: refused, not wrong
    host, d = _case(504, [9000], [7681], [256], [256], 1, 1, 128, torch.bfloat16)
    with pytest.raises(D.DodoError) as e:
        D.dodo_nugget_attention_indexed(d["Q"], d["K"], d["V"], d["idx"], d["cu_s"], d["Kl"], d["Vl"], d["cu_q"],
                                        d["cu_k"], d["cu_l"], 256, 7681, 256, 9000)
    assert e.value.status == -2
