"""GPU parity: dodo_nugget_attention (split-K and MFMA query-block kernels) against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import workloads as W
from gpu_util import check_attention, check_lse, default_scale, dev, make_attention_case

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def D():
    import paper_2310_02409_amd as D
    return D


def _run(D, devt, q_lens, k_lens, m_lens, scale, layout=0, want_lse=True):
    return D.dodo_nugget_attention(devt["Q"], devt["Kn"], devt["Vn"], devt["Kl"], devt["Vl"], devt["cu_q"],
                                   devt["cu_nuggets"], devt["cu_local"], max(q_lens), max(k_lens), max(m_lens),
                                   scale, layout, want_lse=want_lse)


def _full_check(D, seed, q_lens, k_lens, m_lens, H, H_kv, d_h, dtype, scale=None):
    host, devt = make_attention_case(seed, q_lens, k_lens, m_lens, H, H_kv, d_h, dtype, dev())
    scale = default_scale(d_h) if scale is None else scale
    O_ref, lse_ref = oracle.attention(host["Q"], host["Kn"], host["Vn"], host["Kl"], host["Vl"], host["cu_q"],
                                      host["cu_nuggets"], host["cu_local"], scale)
    O, lse = _run(D, devt, q_lens, k_lens, m_lens, scale)
    err = check_attention(O, O_ref, dtype)
    check_lse(lse, lse_ref, dtype)
    return err


# ---------------------------------------------------------------- split-K kernel (decode, fp32, small q)
@pytest.mark.parametrize("dtype,H,H_kv,d_h", [
    (torch.float32, 4, 4, 64), (torch.bfloat16, 32, 32, 128), (torch.bfloat16, 8, 2, 128),
    (torch.bfloat16, 4, 4, 64), (torch.float32, 4, 2, 128),
    (torch.bfloat16, 32, 8, 128), (torch.bfloat16, 64, 8, 128), (torch.float32, 32, 16, 64), (torch.bfloat16, 12, 3, 128),
])
def test_decode_ragged(D, dtype, H, H_kv, d_h):
    k_lens = [205, 410, 333, 1, 0]
    m_lens = [257, 257, 40, 3, 5]
    _full_check(D, 400, [1] * 5, k_lens, m_lens, H, H_kv, d_h, dtype)


def test_small_query_blocks_grouped_heads(D):
    # 2 <= q < 16 rows per sequence go through the bandwidth-bound kernel too; grouped heads in both placements
    _full_check(D, 407, [3, 15, 1, 7], [100, 31, 200, 0], [20, 15, 64, 9], 32, 8, 128, torch.bfloat16)
    _full_check(D, 408, [5, 2], [77, 300], [5, 40], 8, 4, 64, torch.float32)


def test_grouped_heads_served_by_one_workgroup(D):
    # enough (sequence, row, KV head) triples that a workgroup serves the 8 (or 4) query heads of a KV head together
    _full_check(D, 420, [15] * 6 + [3, 1], [100, 31, 200, 0, 64, 65, 17, 300], [20, 15, 64, 9, 15, 40, 3, 1], 64, 8, 128,
                torch.bfloat16)
    _full_check(D, 421, [4] * 19 + [2], [50] * 10 + [7] * 10, [4, 9] * 10, 32, 4, 64, torch.float32)
    _full_check(D, 422, [1] * 70, [33 + 3 * b for b in range(70)], [17] * 70, 64, 8, 128, torch.bfloat16)
    _full_check(D, 423, [1] * 80, [40] * 80, [9] * 80, 16, 4, 64, torch.bfloat16)


def test_neighbouring_heads_served_by_one_workgroup(D):
    # multi-head attention (every query head its own KV head) with thousands of (sequence, head) pairs: two
    # neighbouring heads share a workgroup for the sake of contiguous reads; each keeps its own rows and state
    rng = np.random.default_rng(6)
    B = 72
    k_lens = [int(v) for v in rng.integers(0, 90, B)]
    m_lens = [int(v) for v in rng.integers(1, 40, B)]
    _full_check(D, 431, [1] * B, k_lens, m_lens, 32, 32, 64, torch.bfloat16)
    _full_check(D, 432, [1] * (B - 1) + [0], k_lens, m_lens, 32, 32, 128, torch.float32)
    # ... and with two query rows as well (2 heads x 2 rows per workgroup)
    _full_check(D, 433, [2] * B, k_lens, m_lens, 32, 32, 64, torch.bfloat16)


def test_query_rows_served_by_one_workgroup(D):
    # small query blocks with enough (sequence, row group, head) triples that a workgroup serves 8 (or 4 x 2 heads)
    # query rows together: every row stops at its own causal limit, row groups reach past ragged ends
    rng = np.random.default_rng(5)
    q_lens = [int(v) for v in rng.integers(1, 16, 40)]
    k_lens = [int(v) for v in rng.integers(0, 120, 40)]
    m_lens = [int(v) for v in rng.integers(0, 40, 40)]
    _full_check(D, 426, q_lens, k_lens, m_lens, 32, 32, 128, torch.bfloat16)
    _full_check(D, 427, q_lens, k_lens, m_lens, 16, 8, 64, torch.bfloat16)
    # fp32 query blocks of any length take this kernel: 33 rows = 4 full row groups and one row
    _full_check(D, 428, [33, 32, 7, 1] * 6, [52, 0, 9, 100] * 6, [48, 32, 3, 5] * 6, 8, 8, 64, torch.float32)
    _full_check(D, 429, [33, 32, 7, 1] * 8, [52, 0, 9, 100] * 8, [40, 40, 3, 5] * 8, 8, 2, 128, torch.float32)


def test_decode_split_k_paths(D):
    # few (sequence, head) pairs and many rows: the split count goes above 1 and the last split combines
    assert D.dodo_nugget_attention_workspace_bytes(2, 2, 128, 1, 3277, 1089, D.BF16) > 0
    _full_check(D, 401, [1, 1], [3277, 1500], [1089, 1025], 2, 2, 128, torch.bfloat16)
    _full_check(D, 402, [1], [2000], [300], 2, 1, 64, torch.float32)


def test_split_k_workspace_is_reusable_and_needs_no_initialisation(D):
    # the last split of a row waits for the flags of the others and clears them: the same workspace
    # serves call after call, and bytes that are not the "ready" value are as good as zeros
    q_lens, k_lens, m_lens, H, d_h = [1, 1], [3000, 1234], [700, 1025], 2, 128
    need = D.dodo_nugget_attention_workspace_bytes(2, H, d_h, 1, max(k_lens), max(m_lens), D.BF16)
    assert need > 0
    ws = torch.full((need,), 0xFF, dtype=torch.uint8, device=dev())
    scale = default_scale(d_h)
    for seed in (410, 411, 412):
        host, devt = make_attention_case(seed, q_lens, k_lens, m_lens, H, H, d_h, torch.bfloat16, dev())
        O_ref, lse_ref = oracle.attention(host["Q"], host["Kn"], host["Vn"], host["Kl"], host["Vl"], host["cu_q"],
                                          host["cu_nuggets"], host["cu_local"], scale)
        O, lse = D.dodo_nugget_attention(devt["Q"], devt["Kn"], devt["Vn"], devt["Kl"], devt["Vl"], devt["cu_q"],
                                         devt["cu_nuggets"], devt["cu_local"], 1, max(k_lens), max(m_lens), scale, 0,
                                         want_lse=True, ws=ws)
        check_attention(O, O_ref, torch.bfloat16)
        check_lse(lse, lse_ref, torch.bfloat16)


def test_split_k_grid_limit_is_reported(D):
    # more (sequence, query-row group) pairs than the second grid dimension takes: refused before any launch
    B = 66000
    host, d = make_attention_case(440, [1] * B, [1] * B, [1] * B, 1, 1, 64, torch.float32, dev())
    with pytest.raises(D.DodoError) as e:
        D.dodo_nugget_attention(d["Q"], d["Kn"], d["Vn"], d["Kl"], d["Vl"], d["cu_q"], d["cu_nuggets"], d["cu_local"],
                                1, 1, 1, 0.125)
    assert e.value.status == -2
    # ... and one below the limit runs and is right
    B = 65535
    _full_check(D, 441, [1] * B, [1] * B, [1] * B, 1, 1, 64, torch.float32)


def test_tiny_fp32_config_block_through_split_k_kernel(D):
    # workload 1: 32 causal query rows, 16 earlier local rows, 52 nuggets, 4 heads x 64, fp32
    _full_check(D, 403, [32], [52], [48], 4, 4, 64, torch.float32)
    _full_check(D, 404, [7, 3], [10, 0], [7, 9], 2, 2, 128, torch.float32)


def test_rows_that_see_nothing(D):
    # no nuggets and a local buffer shorter than the query block: the first rows have an empty visible set
    _full_check(D, 405, [4], [0], [2], 2, 2, 64, torch.float32)
    _full_check(D, 406, [40], [0], [20], 2, 2, 128, torch.bfloat16)


# ---------------------------------------------------------------- MFMA query-block kernel
@pytest.mark.parametrize("q_lens,k_lens,m_lens,H,H_kv", [
    ([128], [64], [128], 2, 2),
    ([512, 512], [410, 410], [640, 640], 4, 4),       # workload-2 shape, fewer heads
    ([100, 37, 256, 16], [13, 200, 0, 77], [150, 37, 300, 16], 4, 2),  # ragged, GQA, partial tiles
    ([300], [103], [300], 3, 1),                      # tau = 0 (compressor mode), q not a tile multiple
    ([64, 200], [500, 9], [0, 100], 2, 2),            # nuggets only; local shorter than the block
])
def test_block_attention_bf16(D, q_lens, k_lens, m_lens, H, H_kv):
    _full_check(D, 410, q_lens, k_lens, m_lens, H, H_kv, 128, torch.bfloat16)
    _full_check(D, 417, q_lens, k_lens, m_lens, H, H_kv, 64, torch.bfloat16)  # the same kernels with 64-wide heads


def test_block_attention_scale_argument_and_head_major_cache(D):
    q_lens, k_lens, m_lens = [130, 64], [90, 31], [200, 64]
    host, devt = make_attention_case(411, q_lens, k_lens, m_lens, 4, 2, 128, torch.bfloat16, dev())
    for scale in (0.05, 0.2):
        O_ref, lse_ref = oracle.attention(host["Q"], host["Kn"], host["Vn"], host["Kl"], host["Vl"], host["cu_q"],
                                          host["cu_nuggets"], host["cu_local"], scale)
        O, lse = _run(D, devt, q_lens, k_lens, m_lens, scale)
        check_attention(O, O_ref, torch.bfloat16)
        check_lse(lse, lse_ref, torch.bfloat16)
        hm = dict(devt)
        hm["Kn"] = devt["Kn"].permute(1, 0, 2).contiguous()
        hm["Vn"] = devt["Vn"].permute(1, 0, 2).contiguous()
        O2, _ = _run(D, hm, q_lens, k_lens, m_lens, scale, layout=1)
        assert torch.equal(O, O2)


def test_block_kernel_row_equals_decode_kernel_row(D):
    # the same query row through both kernels (block: q rows at once; split-K: one row, truncated local buffer)
    q, k, tau = 48, 100, 20
    host, devt = make_attention_case(412, [q], [k], [tau + q], 4, 4, 128, torch.bfloat16, dev())
    scale = default_scale(128)
    O_blk, _ = _run(D, devt, [q], [k], [tau + q], scale)
    for i in (0, 17, 47):
        m_i = tau + i + 1
        d1 = dict(devt)
        d1["Q"] = devt["Q"][i:i + 1].contiguous()
        d1["Kl"], d1["Vl"] = devt["Kl"][:m_i].contiguous(), devt["Vl"][:m_i].contiguous()
        d1["cu_q"] = W.cumulative([1], dev())
        d1["cu_local"] = W.cumulative([m_i], dev())
        O_dec, _ = _run(D, d1, [1], [k], [m_i], scale)
        assert torch.max(torch.abs(O_dec[0].float() - O_blk[i].float())) <= 2e-2


def test_block_attention_64_wide_heads_head_major_and_paired_launch(D):
    # head-major cache with 64-wide heads, and a launch with two query blocks per workgroup (>= 256 (sequence, head)
    # pairs of more than 256 rows), whole tensor against the oracle
    q_lens, k_lens, m_lens = [130, 64], [90, 31], [200, 64]
    host, devt = make_attention_case(424, q_lens, k_lens, m_lens, 4, 2, 64, torch.bfloat16, dev())
    O_ref, lse_ref = oracle.attention(host["Q"], host["Kn"], host["Vn"], host["Kl"], host["Vl"], host["cu_q"],
                                      host["cu_nuggets"], host["cu_local"], 0.11)
    O, lse = _run(D, devt, q_lens, k_lens, m_lens, 0.11)
    check_attention(O, O_ref, torch.bfloat16)
    check_lse(lse, lse_ref, torch.bfloat16)
    hm = dict(devt)
    hm["Kn"], hm["Vn"] = devt["Kn"].permute(1, 0, 2).contiguous(), devt["Vn"].permute(1, 0, 2).contiguous()
    O2, _ = _run(D, hm, q_lens, k_lens, m_lens, 0.11, layout=1)
    assert torch.equal(O, O2)
    q_lens = [512, 300, 257, 400, 511, 384, 290, 512, 450, 333, 260]
    _full_check(D, 425, q_lens, [40, 0, 13, 64, 1, 65, 30, 70, 7, 50, 33], [q + t for q, t in zip(q_lens, [0, 5, 64, 0, 3, 0, 16, 1, 63, 20, 9])],
                24, 8, 64, torch.bfloat16)


def test_attention_is_deterministic(D):
    q_lens, k_lens, m_lens = [256], [410], [384]
    _, devt = make_attention_case(413, q_lens, k_lens, m_lens, 8, 8, 128, torch.bfloat16, dev())
    first, _ = _run(D, devt, q_lens, k_lens, m_lens, 0.088)
    first = first.clone()
    for _ in range(20):
        O, _ = _run(D, devt, q_lens, k_lens, m_lens, 0.088)
        assert torch.equal(O, first)
    _, devd = make_attention_case(414, [1] * 4, [3000] * 4, [500] * 4, 2, 2, 128, torch.bfloat16, dev())
    first, _ = _run(D, devd, [1] * 4, [3000] * 4, [500] * 4, 0.088)
    first = first.clone()
    for _ in range(20):
        O, _ = _run(D, devd, [1] * 4, [3000] * 4, [500] * 4, 0.088)
        assert torch.equal(O, first)


@pytest.mark.parametrize("scale", [8.0, -0.09, 0.0])
def test_block_attention_exact_fallback_paths(D, scale):
    # 8-wavefront kernel: a huge scale spreads the logits far beyond the fixed per-row exponent offset
    # (rows fall back to the running-maximum loop); non-positive scales take that loop from the start
    _full_check(D, 415, [300, 130], [200, 64], [364, 130], 2, 2, 128, torch.bfloat16, scale=scale)
    # 4-wavefront kernel (short query block) with the same scales
    _full_check(D, 416, [100], [70], [120], 2, 1, 128, torch.bfloat16, scale=scale)
    # 64-wide heads, both kernels
    _full_check(D, 418, [300, 130], [200, 64], [364, 130], 2, 2, 64, torch.bfloat16, scale=scale)
    _full_check(D, 419, [100], [70], [120], 2, 1, 64, torch.bfloat16, scale=scale)
