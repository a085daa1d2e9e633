"""GPU parity of the query-block kernel's paired launch form, over whole tensors.

When a launch has at least one workgroup per compute unit with two query blocks each, a workgroup takes a
heavy and a light query block one after the other, and neighbouring workgroups of an XCD swap blocks across two
(sequence, head) pairs.  That form needs >= 256 (sequence, head) pairs with more than 256 query rows; the
cases here have 264 (an odd number of groups of 8, so the last group has no partner), ragged query counts,
few nuggets and short local buffers, so that the oracle still covers every output row.  Outputs are filled
with NaN before each call.
"""
import concurrent.futures

import numpy as np
import pytest
import torch

import oracle
import workloads as W
from gpu_util import (check_attention, check_lse, check_rows, default_scale, dev, nan_outputs,
                      oracle_attention_rows_parallel, oracle_workers, slab_rows)

pytestmark = pytest.mark.gpu

Q_LENS = [512, 300, 257, 256, 100, 511, 384, 17, 512, 450, 333]
K_LENS = [70, 0, 13, 64, 100, 1, 65, 30, 129, 7, 90]
TAUS = [0, 5, 64, 0, 100, 3, 0, 16, 1, 63, 20]
H, H_KV, D_H = 24, 8, 128


@pytest.fixture(scope="module")
def D():
    import paper_2310_02409_amd as D
    return D


def _context_case(seed):
    """A context with K, V [N, H_kv, d_h] and index lists of K_LENS nuggets per sequence, plus Q and local rows."""
    n_lens = [max(1, 3 * k + 5) for k in K_LENS]
    m_lens = [q + t for q, t in zip(Q_LENS, TAUS)]
    mk = lambda tid, n, h: W.normal(seed, tid, (n, h, D_H), 1.0, torch.bfloat16, "cpu")
    t = dict(K=mk(0, sum(n_lens), H_KV), V=mk(1, sum(n_lens), H_KV), Q=mk(2, sum(Q_LENS), H),
             Kl=mk(3, sum(m_lens), H_KV), Vl=mk(4, sum(m_lens), H_KV))
    s = W.normal(seed, 5, (sum(n_lens),), 1.0, torch.float32).numpy()
    cu = dict(cu_s=oracle.cu_from_lengths(n_lens), cu_k=oracle.cu_from_lengths(K_LENS),
              cu_q=oracle.cu_from_lengths(Q_LENS), cu_l=oracle.cu_from_lengths(m_lens))
    cu["idx"] = oracle.select_topk(s, cu["cu_s"], cu["cu_k"])
    host = {k: W.to_numpy(v) for k, v in t.items()}
    host.update(cu)
    devt = {k: v.to(dev()) for k, v in t.items()}
    devt.update({k: torch.from_numpy(v).to(dev()) for k, v in cu.items()})
    return host, devt, n_lens, m_lens


def test_paired_query_blocks_whole_tensor_plain_and_indexed(D):
    host, d, n_lens, m_lens = _context_case(700)
    scale = default_scale(D_H)
    Kn_ref, Vn_ref = oracle.gather(host["K"], host["V"], host["idx"], host["cu_s"], host["cu_k"])
    Kn, Vn = D.dodo_gather_nuggets(d["K"], d["V"], d["idx"], d["cu_s"], d["cu_k"], sum(K_LENS))
    assert np.array_equal(W.to_numpy(Kn), Kn_ref) and np.array_equal(W.to_numpy(Vn), Vn_ref)
    O, lse = nan_outputs(d["Q"], H)
    D.dodo_nugget_attention(d["Q"], Kn, Vn, d["Kl"], d["Vl"], d["cu_q"], d["cu_k"], d["cu_l"], max(Q_LENS), max(K_LENS),
                            max(m_lens), scale, O=O, lse=lse)
    rows = slab_rows([(b, h) for b in range(len(Q_LENS)) for h in range(H)], Q_LENS)
    hh = dict(Q=host["Q"], Kl=host["Kl"], Vl=host["Vl"], cu_q=host["cu_q"], cu_local=host["cu_l"])
    O_ref, lse_ref = oracle_attention_rows_parallel(hh, Kn_ref, Vn_ref, host["cu_k"], scale, rows)
    check_rows(O, lse, host["cu_q"], rows, O_ref, lse_ref, torch.bfloat16)
    # the gather-free form of the same launch shape: identical bits
    O2, lse2 = nan_outputs(d["Q"], H)
    D.dodo_nugget_attention_indexed(d["Q"], d["K"], d["V"], d["idx"], d["cu_s"], d["Kl"], d["Vl"], d["cu_q"], d["cu_k"],
                                    d["cu_l"], max(Q_LENS), max(K_LENS), max(m_lens), max(n_lens), scale, O=O2, lse=lse2)
    assert torch.equal(O, O2) and torch.equal(lse, lse2)
    # head-major cache: identical bits as well
    O3, lse3 = nan_outputs(d["Q"], H)
    D.dodo_nugget_attention(d["Q"], Kn.permute(1, 0, 2).contiguous(), Vn.permute(1, 0, 2).contiguous(), d["Kl"], d["Vl"],
                            d["cu_q"], d["cu_k"], d["cu_l"], max(Q_LENS), max(K_LENS), max(m_lens), scale,
                            D.HEAD_MAJOR, O=O3, lse=lse3)
    assert torch.equal(O, O3) and torch.equal(lse, lse3)


def test_paired_query_blocks_whole_tensor_segment_form(D):
    # 11 texts cut into segments of 300 tokens (two query blocks each), 33 entries x 8 heads = 264 pairs, walked
    # from the back of the batch; every row of every entry against the attention oracle on the plan's ranges
    n_lens = [700, 890, 601, 900, 650, 777, 820, 610, 899, 745, 888]
    seg_len, tau, Hs = 300, 40, 8
    N = sum(n_lens)
    mk = lambda tid, h: W.normal(701, tid, (N, h, D_H), 1.0, torch.bfloat16)
    Qt, Kt_, Vt, Ke, Ve = mk(0, Hs), mk(1, Hs), mk(2, Hs), mk(3, Hs), mk(4, Hs)
    s = W.normal(701, 5, (N,), 1.0, torch.float32).numpy()
    k_lens = [oracle.nugget_count(n, 1, 10) for n in n_lens]
    cu_s, cu_k = oracle.cu_from_lengths(n_lens), oracle.cu_from_lengths(k_lens)
    idx = oracle.select_topk(s, cu_s, cu_k)
    Kn_h, Vn_h = oracle.gather(W.to_numpy(Ke), W.to_numpy(Ve), idx, cu_s, cu_k)
    Qh, Kh, Vh = W.to_numpy(Qt), W.to_numpy(Kt_), W.to_numpy(Vt)
    plan_ref = oracle.segment_plan(idx, cu_s, cu_k, seg_len, tau)
    E = len(plan_ref[1])
    assert E == 33
    to = lambda a: torch.from_numpy(a).to(dev())
    plan = D.dodo_segment_plan(to(idx), to(cu_s), to(cu_k), seg_len, tau, E)
    for g, w in zip(plan[:5], plan_ref):
        assert np.array_equal(g.cpu().numpy(), w)
    scale = default_scale(D_H)
    Qd = Qt.to(dev())
    O, lse = nan_outputs(Qd, Hs)
    D.dodo_nugget_attention_segments(Qd, to(Kn_h.view(np.int16)).view(torch.bfloat16), to(Vn_h.view(np.int16)).view(torch.bfloat16),
                                     Kt_.to(dev()), Vt.to(dev()), plan[0], plan[1], plan[2], plan[3], plan[4], seg_len,
                                     max(k_lens), seg_len + tau, scale, O=O, lse=lse)
    cu_q, ns, nl, ls, ll = plan_ref
    one = lambda m: np.array([0, m], np.int32)

    def entry(e):
        return oracle.attention(Qh[cu_q[e]:cu_q[e + 1]], Kn_h[ns[e]:ns[e] + nl[e]], Vn_h[ns[e]:ns[e] + nl[e]],
                                Kh[ls[e]:ls[e] + ll[e]], Vh[ls[e]:ls[e] + ll[e]], one(cu_q[e + 1] - cu_q[e]), one(nl[e]),
                                one(ll[e]), scale)
    with concurrent.futures.ThreadPoolExecutor(max_workers=oracle_workers()) as ex:
        refs = list(ex.map(entry, range(E)))
    O_ref = np.concatenate([r[0] for r in refs])
    lse_ref = np.concatenate([r[1] for r in refs])
    check_attention(O, O_ref, torch.bfloat16)
    check_lse(lse, lse_ref, torch.bfloat16)
