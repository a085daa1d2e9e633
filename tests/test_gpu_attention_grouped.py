"""GPU parity: the matrix-core kernel for a few query vectors per K/V row (grouped-query heads and small query
blocks, bf16, d_h = 128 or 64) against the oracle, through dodo_nugget_attention and its variants."""
import numpy as np
import pytest
import torch

import oracle
import workloads as W
from gpu_util import check_attention, check_lse, default_scale, dev, make_attention_case, nan_outputs

pytestmark = pytest.mark.gpu
BF = torch.bfloat16


@pytest.fixture(scope="module")
def D():
    import paper_2310_02409_amd as D
    return D


def _check(D, seed, q_lens, k_lens, m_lens, H, H_kv, layout=0, ws="wanted", scale=None, d_h=128):
    host, t = make_attention_case(seed, q_lens, k_lens, m_lens, H, H_kv, d_h, BF, dev())
    scale = default_scale(d_h) if scale is None else scale
    B, mq, mk, mm = len(q_lens), max(q_lens), max(k_lens), max(m_lens)
    O_ref, lse_ref = oracle.attention(host["Q"], host["Kn"], host["Vn"], host["Kl"], host["Vl"], host["cu_q"],
                                      host["cu_nuggets"], host["cu_local"], scale)
    Kn, Vn = t["Kn"], t["Vn"]
    if layout == D.HEAD_MAJOR:
        Kn, Vn = Kn.transpose(0, 1).contiguous(), Vn.transpose(0, 1).contiguous()
    O, lse = nan_outputs(t["Q"], H)
    if ws == "wanted":  # as much as the kernel would like to have
        need = D.dodo_nugget_attention_workspace_bytes_grouped(B, H, H_kv, d_h, mq, mk, mm, D.BF16)
    elif ws == "plain":  # what the query without H_kv asks for: fewer splits, same result to the tolerance
        need = D.dodo_nugget_attention_workspace_bytes(B, H, d_h, mq, mk, mm, D.BF16)
    else:
        need = int(ws)
    buf = torch.zeros(max(need, 16), dtype=torch.uint8, device=dev()) if need else None
    for _ in range(2):  # the second call finds the workspace as the first left it
        D.dodo_nugget_attention(t["Q"], Kn, Vn, t["Kl"], t["Vl"], t["cu_q"], t["cu_nuggets"], t["cu_local"], mq, mk, mm,
                                scale, layout, O=O, lse=lse, ws=buf)
        check_attention(O, O_ref, BF)
        check_lse(lse, lse_ref, BF)
    return O, lse, need


@pytest.mark.parametrize("H,H_kv", [(32, 8), (64, 8), (40, 8), (32, 4), (32, 1)])
def test_grouped_heads_decode_large_batch(D, H, H_kv):
    # one workgroup of two wavefronts per (sequence, KV head): group sizes 4, 8, 5 (not a power of two), 32
    rng = np.random.default_rng(H * 100 + H_kv)
    B = 70
    k_lens = [int(v) for v in rng.integers(0, 150, B)]
    m_lens = [int(v) for v in rng.integers(1, 70, B)]
    k_lens[3], m_lens[3] = 0, 1
    k_lens[4], m_lens[4] = 31, 33   # one ragged tile each
    k_lens[5], m_lens[5] = 64, 32   # whole tiles only
    _check(D, 700 + H_kv, [1] * B, k_lens, m_lens, H, H_kv)


def test_grouped_heads_decode_splits_over_workgroups(D):
    # few (sequence, KV head) pairs and long caches: the keys of a pair are split over workgroups, whose partial
    # records the last one merges; with the larger workspace more splits than with the plain one
    q, k, m = [1, 1], [3277, 1500], [1089, 1025]
    _, _, wanted = _check(D, 710, q, k, m, 64, 8)
    _, _, plain = _check(D, 710, q, k, m, 64, 8, ws="plain")
    assert wanted > plain
    _check(D, 711, q, k, m, 32, 8, layout=1)
    # four wavefronts per workgroup (fewer than two workgroups per compute unit in all), ragged split ends
    _check(D, 712, [1] * 5, [205, 410, 333, 1, 0], [257, 257, 40, 3, 5], 64, 8)
    _check(D, 713, [1] * 3, [2000, 37, 900], [300, 700, 31], 40, 8)


def test_small_query_blocks_share_their_keys(D):
    # 2 <= q <= 8 rows: vector (row, head); every row stops at its own causal limit (also m_b < q_b: early rows see
    # no local row at all), ragged q_b, sequences without queries
    rng = np.random.default_rng(9)
    B = 48
    q_lens = [int(v) for v in rng.integers(0, 5, B)]
    q_lens[0], q_lens[1] = 4, 0
    k_lens = [int(v) for v in rng.integers(0, 120, B)]
    m_lens = [int(v) for v in rng.integers(0, 40, B)]
    m_lens[0] = 2
    _check(D, 720, q_lens, k_lens, m_lens, 32, 4)    # 8 heads x up to 4 rows = 32 vectors
    _check(D, 721, q_lens, k_lens, m_lens, 40, 8)    # 5 heads x 4 rows
    q8 = [int(v) for v in rng.integers(1, 9, B)]
    _check(D, 722, q8, k_lens, m_lens, 32, 32)       # multi-head attention: 8 rows of one head
    _check(D, 723, q8, k_lens, [0] * B, 16, 4)       # nuggets only
    _check(D, 724, q8, [0] * B, [max(m, 1) for m in m_lens], 16, 4)  # local rows only


def test_more_than_32_vectors_take_several_passes(D):
    # rows x heads beyond one tile: the rows are dealt out to up to four launches, each with its own causal limits
    rng = np.random.default_rng(13)
    B = 40
    q_lens = [int(v) for v in rng.integers(0, 16, B)]
    q_lens[0], q_lens[1], q_lens[2] = 15, 0, 4        # all passes, none, exactly the first
    k_lens = [int(v) for v in rng.integers(0, 120, B)]
    m_lens = [int(v) for v in rng.integers(0, 40, B)]
    m_lens[0] = 7                                       # fewer local rows than query rows: early rows see none
    _check(D, 780, q_lens, k_lens, m_lens, 64, 8)      # 8 heads x 15 rows: four passes of 4 rows
    _check(D, 781, q_lens, k_lens, m_lens, 16, 4)      # 4 heads x 15 rows: two passes of 8 rows
    _check(D, 782, [min(q, 8) for q in q_lens], k_lens, m_lens, 32, 2, d_h=64)   # 16 heads x 8 rows: four passes of 2
    _check(D, 783, [min(q, 6) for q in q_lens], k_lens, m_lens, 20, 4)           # 5 heads x 6 rows: one pass of 6
    # few sequences and long caches: every pass splits the keys over workgroups, all on one workspace
    _check(D, 784, [15, 9], [3277, 1500], [1089, 1025], 64, 8)
    _check(D, 785, [7, 7, 2], [2000, 37, 900], [300, 700, 31], 40, 8, layout=1)


def test_heads_of_64_channels(D):
    # the same kernel with half the channels: other tile sizes, LDS swizzles and fragment counts
    rng = np.random.default_rng(12)
    B = 70
    k_lens = [int(v) for v in rng.integers(0, 150, B)]
    m_lens = [int(v) for v in rng.integers(1, 70, B)]
    k_lens[3], m_lens[3] = 0, 1
    k_lens[4], m_lens[4] = 31, 33
    _check(D, 770, [1] * B, k_lens, m_lens, 32, 8, d_h=64)
    _check(D, 771, [1] * B, k_lens, m_lens, 40, 8, d_h=64, layout=1)
    q_lens = [int(v) for v in rng.integers(0, 5, B)]
    _check(D, 772, q_lens, k_lens, m_lens, 32, 4, d_h=64)
    _check(D, 773, [int(v) for v in rng.integers(1, 9, B)], k_lens, m_lens, 16, 16, d_h=64)
    # split over workgroups (two and four wavefronts each)
    _check(D, 774, [1, 1], [3277, 1500], [1089, 1025], 64, 8, d_h=64)
    _check(D, 775, [1] * 5, [205, 410, 333, 1, 0], [257, 257, 40, 3, 5], 64, 8, d_h=64)
    _check(D, 776, [2] * 3, [2000, 37, 900], [300, 700, 31], 40, 8, d_h=64)


def test_softmax_scale_and_large_logits(D):
    # a scale that makes single keys dominate: the running maximum moves from tile to tile
    _check(D, 730, [1] * 40, [100] * 40, [64] * 40, 32, 8, scale=1.5)


def test_run_to_run_deterministic(D):
    host, t = make_attention_case(740, [1, 1], [3277, 1500], [1089, 1025], 64, 8, 128, BF, dev())
    need = D.dodo_nugget_attention_workspace_bytes_grouped(2, 64, 8, 128, 1, 3277, 1089, D.BF16)
    ws = torch.zeros(need, dtype=torch.uint8, device=dev())
    outs = []
    for _ in range(4):
        O, lse = D.dodo_nugget_attention(t["Q"], t["Kn"], t["Vn"], t["Kl"], t["Vl"], t["cu_q"], t["cu_nuggets"],
                                         t["cu_local"], 1, 3277, 1089, default_scale(128), 0, want_lse=True, ws=ws)
        outs.append((O.clone(), lse.clone()))
    for O, lse in outs[1:]:
        assert torch.equal(O, outs[0][0]) and torch.equal(lse, outs[0][1])
    n_slots = need // ((128 + 3) * 4)
    assert not bool(ws.view(torch.int32)[-n_slots:].any())  # the flags of the largest layout are left cleared


def test_workspace_needs_no_zero_fill_and_is_reusable(D):
    # bytes that are not the "ready" value are as good as zeros, and a workspace serves call after call
    q, k, m, H, H_kv = [1, 1], [3000, 1234], [700, 1025], 64, 8
    need = D.dodo_nugget_attention_workspace_bytes_grouped(2, H, H_kv, 128, 1, max(k), max(m), D.BF16)
    assert need > D.dodo_nugget_attention_workspace_bytes(2, H, 128, 1, max(k), max(m), D.BF16)
    ws = torch.full((need,), 0xFF, dtype=torch.uint8, device=dev())
    for seed in (790, 791, 792):
        host, t = make_attention_case(seed, q, k, m, H, H_kv, 128, BF, dev())
        O_ref, lse_ref = oracle.attention(host["Q"], host["Kn"], host["Vn"], host["Kl"], host["Vl"], host["cu_q"],
                                          host["cu_nuggets"], host["cu_local"], default_scale(128))
        O, lse = D.dodo_nugget_attention(t["Q"], t["Kn"], t["Vn"], t["Kl"], t["Vl"], t["cu_q"], t["cu_nuggets"],
                                         t["cu_local"], 1, max(k), max(m), default_scale(128), 0, want_lse=True, ws=ws)
        check_attention(O, O_ref, BF)
        check_lse(lse, lse_ref, BF)


def test_caches_with_room_to_grow_and_segment_ranges(D):
    # start + length ranges for the nuggets (cached form) and for both kinds of rows (segment form)
    rng = np.random.default_rng(11)
    B, H, H_kv, cap = 40, 32, 8, 96
    lens = [int(v) for v in rng.integers(0, cap, B)]
    m_lens = [int(v) for v in rng.integers(1, 50, B)]
    mk = lambda tid, n, h: W.normal(750, tid, (n, h, 128), 1.0, BF, "cpu")
    Q, Kc, Vc = mk(0, B, H), mk(1, B * cap, H_kv), mk(2, B * cap, H_kv)
    Kl, Vl = mk(3, sum(m_lens), H_kv), mk(4, sum(m_lens), H_kv)
    start = np.arange(B, dtype=np.int32) * cap
    cu_q, cu_l = W.cumulative([1] * B), W.cumulative(m_lens)
    scale = default_scale(128)
    # oracle on the packed equivalent
    rows = np.concatenate([np.arange(s, s + n) for s, n in zip(start, lens)]).astype(np.int64)
    Kn_p, Vn_p = Kc[torch.from_numpy(rows)], Vc[torch.from_numpy(rows)]
    O_ref, lse_ref = oracle.attention(W.to_numpy(Q), W.to_numpy(Kn_p), W.to_numpy(Vn_p), W.to_numpy(Kl), W.to_numpy(Vl),
                                      W.to_numpy(cu_q), oracle.cu_from_lengths(lens), W.to_numpy(cu_l), scale)
    d = dev()
    O, lse = D.dodo_nugget_attention_cached(Q.to(d), Kc.to(d), Vc.to(d), Kl.to(d), Vl.to(d), cu_q.to(d),
                                            torch.from_numpy(start).to(d), torch.tensor(lens, dtype=torch.int32, device=d),
                                            cu_l.to(d), 1, cap, max(m_lens), scale, want_lse=True)
    check_attention(O, O_ref, BF)
    check_lse(lse, lse_ref, BF)
    loc_start = W.to_numpy(cu_l)[:-1].astype(np.int32)
    O2, lse2 = D.dodo_nugget_attention_segments(Q.to(d), Kc.to(d), Vc.to(d), Kl.to(d), Vl.to(d), cu_q.to(d),
                                                torch.from_numpy(start).to(d),
                                                torch.tensor(lens, dtype=torch.int32, device=d),
                                                torch.from_numpy(loc_start).to(d),
                                                torch.tensor(m_lens, dtype=torch.int32, device=d), 1, cap, max(m_lens),
                                                scale, want_lse=True)
    check_attention(O2, O_ref, BF)
    check_lse(lse2, lse_ref, BF)


def test_entry_point_that_allocates_nothing(D):
    # the library's own buffer bounds the number of splits; same results to the tolerance, twice in a row, the
    # second call smaller
    for seed, q, k, m, H, H_kv in ((760, [1, 1], [3277, 1500], [1089, 1025], 64, 8), (761, [1], [1200], [300], 32, 8),
                                   (762, [1] * 70, [90] * 70, [33] * 70, 32, 8)):
        host, t = make_attention_case(seed, q, k, m, H, H_kv, 128, BF, dev())
        scale = default_scale(128)
        O_ref, lse_ref = oracle.attention(host["Q"], host["Kn"], host["Vn"], host["Kl"], host["Vl"], host["cu_q"],
                                          host["cu_nuggets"], host["cu_local"], scale)
        O, lse = nan_outputs(t["Q"], H)
        D.dodo_nugget_attention_noalloc(t["Q"], t["Kn"], t["Vn"], t["Kl"], t["Vl"], t["cu_q"], t["cu_nuggets"],
                                        t["cu_local"], max(q), max(k), max(m), scale, D.TOKEN_MAJOR, O, lse)
        check_attention(O, O_ref, BF)
        check_lse(lse, lse_ref, BF)
