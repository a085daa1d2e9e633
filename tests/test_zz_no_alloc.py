"""GPU test of dodo_nugget_attention_noalloc (the entry point that allocates nothing): same output, bit for
bit, as dodo_nugget_attention with a caller-owned workspace, and parity with the oracle, on two calls in a
row of which the second is smaller."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import check_attention, check_lse, default_scale, dev, make_attention_case, nan_outputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def D():
    import paper_2310_02409_amd as D
    return D


def _both(D, seed, q_lens, k_lens, m_lens, H, H_kv, d_h, dtype):
    host, t = make_attention_case(seed, q_lens, k_lens, m_lens, H, H_kv, d_h, dtype, dev())
    scale = default_scale(d_h)
    mq, mk, mm = max(q_lens), max(k_lens), max(m_lens)
    O_ws, lse_ws = nan_outputs(t["Q"], H)
    D.dodo_nugget_attention(t["Q"], t["Kn"], t["Vn"], t["Kl"], t["Vl"], t["cu_q"], t["cu_nuggets"], t["cu_local"], mq, mk,
                            mm, scale, D.TOKEN_MAJOR, O=O_ws, lse=lse_ws)
    O, lse = nan_outputs(t["Q"], H)
    D.dodo_nugget_attention_noalloc(t["Q"], t["Kn"], t["Vn"], t["Kl"], t["Vl"], t["cu_q"], t["cu_nuggets"], t["cu_local"],
                                    mq, mk, mm, scale, D.TOKEN_MAJOR, O, lse)
    assert torch.equal(O, O_ws) and torch.equal(lse, lse_ws)
    O_ref, lse_ref = oracle.attention(host["Q"], host["Kn"], host["Vn"], host["Kl"], host["Vl"], host["cu_q"],
                                      host["cu_nuggets"], host["cu_local"], scale)
    check_attention(O, O_ref, dtype)
    check_lse(lse, lse_ref, dtype)


def test_two_calls_in_a_row_second_smaller(D):
    code = D.BF16
    # few (sequence, head) pairs over many rows: the split-K kernel splits, so the scratch buffer is in use
    assert D.dodo_nugget_attention_workspace_bytes(2, 2, 128, 1, 3277, 1089, code) > 0
    _both(D, 900, [1, 1], [3277, 1500], [1089, 1025], 2, 2, 128, torch.bfloat16)
    assert D.dodo_nugget_attention_workspace_bytes(1, 2, 128, 1, 1200, 300, code) > 0
    _both(D, 901, [1], [1200], [300], 2, 1, 128, torch.bfloat16)
    # and back to a larger one, in single precision with the smaller head size
    _both(D, 902, [1, 1, 1], [2000, 700, 0], [300, 5, 900], 2, 1, 64, torch.float32)


def test_calls_that_need_no_scratch_and_the_limit(D):
    # a query block goes to the matrix-core kernel, a large batch of decode rows does not split: no scratch needed
    _both(D, 903, [130, 64], [90, 31], [200, 64], 4, 2, 128, torch.bfloat16)
    _both(D, 904, [1] * 5, [205, 410, 333, 1, 0], [257, 257, 40, 3, 5], 32, 32, 128, torch.bfloat16)
