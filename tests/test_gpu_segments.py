"""GPU parity: dodo_segment_plan (bit-exact) and dodo_nugget_attention_segments against the oracle's
segment form of the autoregressive objective."""
import numpy as np
import pytest
import torch

import oracle
import workloads as W
from gpu_util import check_attention, check_lse, dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def D():
    import paper_2310_02409_amd as D
    return D


def _case(seed, n_lens, H, H_kv, d_h, dtype, keep=(1, 4)):
    N = sum(n_lens)
    mk = lambda tid, h: W.normal(seed, tid, (N, h, d_h), 1.0, dtype)
    Q, K, V, Ke, Ve = mk(0, H), mk(1, H_kv), mk(2, H_kv), mk(3, H_kv), mk(4, H_kv)
    s = W.normal(seed, 5, (N,), 1.0, torch.float32).numpy()
    k_lens = [oracle.nugget_count(n, *keep) for n in n_lens]
    cu_s, cu_k = oracle.cu_from_lengths(n_lens), oracle.cu_from_lengths(k_lens)
    idx = oracle.select_topk(s, cu_s, cu_k)
    Kn, Vn = oracle.gather(W.to_numpy(Ke), W.to_numpy(Ve), idx, cu_s, cu_k)
    host = dict(Q=W.to_numpy(Q), K=W.to_numpy(K), V=W.to_numpy(V), Kn=Kn, Vn=Vn, idx=idx, cu_s=cu_s, cu_k=cu_k)
    glob = torch.from_numpy(np.concatenate([idx[cu_k[b]:cu_k[b + 1]] + cu_s[b] for b in range(len(n_lens))])).long()
    devt = dict(Q=Q.to(dev()), K=K.to(dev()), V=V.to(dev()), Kn=Ke[glob].to(dev()), Vn=Ve[glob].to(dev()),
                idx=torch.from_numpy(idx).to(dev()), cu_s=torch.from_numpy(cu_s).to(dev()),
                cu_k=torch.from_numpy(cu_k).to(dev()))
    return host, devt, k_lens


@pytest.mark.parametrize("n_lens,seg_len,tau,extra", [([10, 3], 4, 2, 0), ([700, 1, 0, 333], 64, 17, 5),
                                                      ([1000], 1, 8, 0), ([50, 60], 128, 0, 2)])
def test_plan_bit_exact(D, n_lens, seg_len, tau, extra):
    host, d, _ = _case(600, n_lens, 1, 1, 64, torch.float32)
    want = oracle.segment_plan(host["idx"], host["cu_s"], host["cu_k"], seg_len, tau)
    E = len(want[1])
    got = D.dodo_segment_plan(d["idx"], d["cu_s"], d["cu_k"], seg_len, tau, E + extra)
    assert int(got[5].item()) == E
    assert np.array_equal(got[0].cpu().numpy()[:E], want[0][:E]) and bool((got[0][E:] == sum(n_lens)).all())
    for g, w in zip(got[1:5], want[1:5]):
        g = g.cpu().numpy()
        assert np.array_equal(g[:E], w)
        assert not g[E:].any()  # entries beyond the last segment are empty
    # a capacity that is too small is visible in the count
    if E > 1:
        short = D.dodo_segment_plan(d["idx"], d["cu_s"], d["cu_k"], seg_len, tau, E - 1)
        assert int(short[5].item()) == E and np.array_equal(short[1].cpu().numpy(), want[1][:E - 1])


def _attend(D, d, plan, seg_len, tau, max_k, scale):
    return D.dodo_nugget_attention_segments(d["Q"], d["Kn"], d["Vn"], d["K"], d["V"], plan[0], plan[1], plan[2], plan[3],
                                            plan[4], seg_len, max_k, seg_len + tau, scale, want_lse=True)


@pytest.mark.parametrize("dtype,n_lens,seg_len,tau,H,H_kv,d_h", [
    (torch.float32, [90, 31], 8, 5, 4, 2, 64),        # split-K kernel, fp32
    (torch.bfloat16, [150, 40], 12, 30, 2, 2, 128),   # split-K kernel (segments shorter than 16 rows)
    (torch.bfloat16, [300, 77, 129], 64, 20, 4, 2, 128),   # 4-wavefront query-block kernel
    (torch.bfloat16, [700, 180], 256, 100, 2, 1, 128),     # 8-wavefront query-block kernel, ragged last segments
])
def test_segment_attention_matches_the_rule(D, dtype, n_lens, seg_len, tau, H, H_kv, d_h):
    host, d, k_lens = _case(601, n_lens, H, H_kv, d_h, dtype, keep=(1, 3))
    scale = d_h ** -0.5
    O_ref, lse_ref = oracle.attention_segment_mask(host["Q"], host["Kn"], host["Vn"], host["K"], host["V"], host["idx"],
                                                   host["cu_s"], host["cu_k"], seg_len, tau, scale)
    E = sum(-(-n // seg_len) for n in n_lens)
    plan = D.dodo_segment_plan(d["idx"], d["cu_s"], d["cu_k"], seg_len, tau, E)
    O, lse = _attend(D, d, plan, seg_len, tau, max(k_lens), scale)
    check_attention(O, O_ref, dtype)
    check_lse(lse, lse_ref, dtype)


def test_training_shape_sampled_rows(D):
    # 4 texts of 4096 tokens, 10x compression, segments of 512 with 128 uncompressed earlier tokens, 8 heads:
    # 32 entries through the 8-wavefront kernel; sampled rows against the attention oracle on the plan's ranges
    n_lens, seg_len, tau, H, d_h = [4096] * 4, 512, 128, 8, 128
    host, d, k_lens = _case(602, n_lens, H, H, d_h, torch.bfloat16, keep=(1, 10))
    scale = d_h ** -0.5
    plan_ref = oracle.segment_plan(host["idx"], host["cu_s"], host["cu_k"], seg_len, tau)
    E = len(plan_ref[1])
    plan = D.dodo_segment_plan(d["idx"], d["cu_s"], d["cu_k"], seg_len, tau, E)
    for g, w in zip(plan[:5], plan_ref):
        assert np.array_equal(g.cpu().numpy(), w)
    O, lse = _attend(D, d, plan, seg_len, tau, max(k_lens), scale)
    cu_q, ns, nl, ls, ll = plan_ref
    rng = np.random.default_rng(602)
    for e in rng.choice(E, 6, replace=False):
        rows = [(0, int(h), int(i)) for h, i in zip(rng.integers(0, H, 4), rng.integers(0, cu_q[e + 1] - cu_q[e], 4))]
        one = lambda m: np.array([0, m], np.int32)
        Or, lr = oracle.attention_rows(host["Q"][cu_q[e]:cu_q[e + 1]], host["Kn"][ns[e]:ns[e] + nl[e]],
                                       host["Vn"][ns[e]:ns[e] + nl[e]], host["K"][ls[e]:ls[e] + ll[e]],
                                       host["V"][ls[e]:ls[e] + ll[e]], one(cu_q[e + 1] - cu_q[e]), one(nl[e]), one(ll[e]),
                                       scale, rows)
        got = torch.stack([O[cu_q[e] + i, h] for _, h, i in rows])
        check_attention(got, Or, torch.bfloat16)
        check_lse(torch.stack([lse[cu_q[e] + i, h] for _, h, i in rows]), lr, torch.bfloat16)
