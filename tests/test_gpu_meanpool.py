"""GPU parity of dodo_meanpool_nuggets (pooling baseline's compaction, Sec. 5.1) against the oracle: bit-exact."""
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


def _cu(lens):
    return np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)


@pytest.mark.parametrize("dtype,H_kv,d_h,layout", [
    (torch.bfloat16, 32, 128, 0), (torch.bfloat16, 2, 64, 1), (torch.float32, 4, 64, 0), (torch.float32, 3, 128, 1),
])
def test_meanpool_bit_exact_ragged(D, dtype, H_kv, d_h, layout):
    lens = [517, 64, 1, 300, 7]
    ks = [52, 64, 1, 15, 2]  # ratios 10, 1 (identity), single token, 20, uneven chunks
    N, Kt = sum(lens), sum(ks)
    K = W.normal(800, 0, (N, H_kv, d_h), 1.0, dtype)
    V = W.normal(800, 1, (N, H_kv, d_h), 1.0, dtype)
    # a few values far below their neighbours: sums that are not exact in single precision
    K.view(-1)[::1013] *= 2.0 ** -20
    Kn_ref, Vn_ref = oracle.meanpool(W.to_numpy(K), W.to_numpy(V), _cu(lens), _cu(ks), layout)
    Kn, Vn = D.dodo_meanpool_nuggets(K.to(dev()), V.to(dev()), torch.from_numpy(_cu(lens)).to(dev()),
                                     torch.from_numpy(_cu(ks)).to(dev()), Kt, layout)
    assert np.array_equal(W.to_numpy(Kn.cpu()), Kn_ref)
    assert np.array_equal(W.to_numpy(Vn.cpu()), Vn_ref)


def test_meanpool_workload_shape_sampled_rows(D):
    # the prefill workload's shape: 8 x 4096 tokens, 410 chunks each; the oracle checks one sequence
    wl = W.config(2)
    g = W.make_inputs(wl, dev(), which=["K", "V"])
    cu_k, ks = D.cu_nuggets_from_lengths(wl.seq_lens, wl.keep_num, wl.keep_den, dev())
    Kn, Vn = D.dodo_meanpool_nuggets(g["K"], g["V"], g["cu_seqlens"], cu_k, sum(ks))
    n, k = wl.seq_lens[3], ks[3]
    a = sum(wl.seq_lens[:3])
    Kr, Vr = oracle.meanpool(W.to_numpy(g["K"][a:a + n].cpu()), W.to_numpy(g["V"][a:a + n].cpu()), _cu([n]), _cu([k]))
    o = sum(ks[:3])
    assert np.array_equal(W.to_numpy(Kn[o:o + k].cpu()), Kr) and np.array_equal(W.to_numpy(Vn[o:o + k].cpu()), Vr)


def test_meanpool_one_rounding_where_two_would_differ(D):
    # chunks {x, y, t, 0} whose exact mean is 2^-42 away from the midpoint of two bf16 values: rounding through
    # single precision would tie to even; the kernel, like the oracle, rounds the double once
    quads = [(0x3F80, 0x3F81, 0x2B80), (0x3F80, 0x3F81, 0xAB80), (0x3F81, 0x3F82, 0x2B80), (0x3F81, 0x3F82, 0xAB80),
             (0xBF80, 0xBF81, 0xAB80), (0x3F80, 0x3F80, 0xAB80)]
    H_kv, d_h = 2, 64
    rows = np.array([[x, y, t, 0] for x, y, t in quads], dtype=np.uint16).reshape(-1)  # 6 chunks of 4 tokens
    K = np.repeat(rows[:, None, None], H_kv, axis=1).repeat(d_h, axis=2)
    cu_s, cu_k = _cu([len(rows)]), _cu([len(quads)])
    Kn_ref, Vn_ref = oracle.meanpool(K, K, cu_s, cu_k)
    Kt_ = torch.from_numpy(K.view(np.int16)).view(torch.bfloat16).to(dev())
    through_fp32 = W.to_numpy(Kt_.double().view(len(quads), 4, H_kv, d_h).mean(dim=1).float().bfloat16())
    assert not np.array_equal(through_fp32, Kn_ref)  # the inputs do sit in the trap
    Kn, Vn = D.dodo_meanpool_nuggets(Kt_, Kt_, torch.from_numpy(cu_s).to(dev()), torch.from_numpy(cu_k).to(dev()),
                                     len(quads))
    assert np.array_equal(W.to_numpy(Kn), Kn_ref) and np.array_equal(W.to_numpy(Vn), Vn_ref)
