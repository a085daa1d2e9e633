"""Pins for the oracle nugget attention (Eq. 13 compressor mode, Eq. 9 mixed resolution, Eq. 3)."""
import math

import numpy as np
import pytest
import torch

import oracle
import workloads as W


def _inputs(seed, q_lens, k_lens, m_lens, H=4, H_kv=2, d_h=8, dtype=torch.float32):
    Sq, Kt, Sm = sum(q_lens), sum(k_lens), sum(m_lens)
    mk = lambda tid, n, h: W.normal(seed, tid, (n, h, d_h), 1.0, dtype)
    Q, Kn, Vn, Kl, Vl = mk(0, Sq, H), mk(1, Kt, H_kv), mk(2, Kt, H_kv), mk(3, Sm, H_kv), mk(4, Sm, H_kv)
    cu = [oracle.cu_from_lengths(x) for x in (q_lens, k_lens, m_lens)]
    return Q, Kn, Vn, Kl, Vl, cu


def _np(*ts):
    return [W.to_numpy(t) for t in ts]


def dense_masked_softmax(Q, Kn, Vn, Kl, Vl, cu, scale):
    """Brute force: explicit boolean mask over the concatenated keys, row softmax in float64."""
    cu_q, cu_k, cu_m = cu
    H, H_kv = Q.shape[1], Kl.shape[1]
    O = torch.zeros(Q.shape, dtype=torch.float64)
    for b in range(len(cu_q) - 1):
        q = Q[cu_q[b]:cu_q[b + 1]].double()
        keys = torch.cat([Kn[cu_k[b]:cu_k[b + 1]], Kl[cu_m[b]:cu_m[b + 1]]]).double()
        vals = torch.cat([Vn[cu_k[b]:cu_k[b + 1]], Vl[cu_m[b]:cu_m[b + 1]]]).double()
        qn, kn, mn = q.shape[0], int(cu_k[b + 1] - cu_k[b]), int(cu_m[b + 1] - cu_m[b])
        mask = torch.zeros(qn, kn + mn, dtype=torch.bool)
        for i in range(qn):
            mask[i, :kn] = True
            for j in range(mn):
                mask[i, kn + j] = bool(j <= mn - qn + i)
        for h in range(H):
            kvh = h // (H // H_kv)
            logits = scale * q[:, h] @ keys[:, kvh].T
            logits = logits.masked_fill(~mask, float("-inf"))
            p = torch.softmax(logits, dim=-1)
            p = torch.nan_to_num(p, nan=0.0)
            O[cu_q[b]:cu_q[b + 1], h] = p @ vals[:, kvh]
    return O.numpy()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_brute_force_dense_mask(dtype):
    Q, Kn, Vn, Kl, Vl, cu = _inputs(50, [5, 1, 7, 3], [4, 9, 0, 2], [8, 6, 7, 0], dtype=dtype)
    scale = 1 / math.sqrt(8)
    O, lse = oracle.attention(*_np(Q, Kn, Vn, Kl, Vl), *cu, scale)
    want = dense_masked_softmax(Q, Kn, Vn, Kl, Vl, cu, scale)
    assert np.allclose(O, want, rtol=1e-12, atol=1e-13)


def test_ratio_one_reduces_to_causal_attention_library():
    # all n context tokens kept as nuggets, then q = m query tokens: plain causal attention over n + q tokens
    n, q, H, d_h = 11, 6, 2, 16
    Q, Kn, Vn, Kl, Vl, cu = _inputs(51, [q], [n], [q], H=H, H_kv=H, d_h=d_h)
    scale = 1 / math.sqrt(d_h)
    O, _ = oracle.attention(*_np(Q, Kn, Vn, Kl, Vl), *cu, scale)
    keys = torch.cat([Kn, Kl]).double().permute(1, 0, 2)[None]
    vals = torch.cat([Vn, Vl]).double().permute(1, 0, 2)[None]
    qq = Q.double().permute(1, 0, 2)[None]
    full_mask = torch.ones(n + q, n + q, dtype=torch.bool).tril()[n:]  # last q rows of the causal mask
    ref = torch.nn.functional.scaled_dot_product_attention(qq, keys, vals, attn_mask=full_mask, scale=scale)
    assert np.allclose(O, ref[0].permute(1, 0, 2).numpy(), rtol=1e-12, atol=1e-13)


def test_zero_query_reads_out_the_mask():
    # Q = 0 -> uniform weights; one-hot V rows -> output = indicator of visible keys / count
    q, k, m, d_h = 4, 3, 6, 16
    Q = np.zeros((q, 1, d_h), np.float32)
    Kn = W.normal(52, 0, (k, 1, d_h), 1.0, torch.float32).numpy()
    Kl = W.normal(52, 1, (m, 1, d_h), 1.0, torch.float32).numpy()
    Vn = np.zeros((k, 1, d_h), np.float32)
    Vl = np.zeros((m, 1, d_h), np.float32)
    for j in range(k):
        Vn[j, 0, j] = 1
    for j in range(m):
        Vl[j, 0, k + j] = 1
    cu = [oracle.cu_from_lengths(x) for x in ([q], [k], [m])]
    O, lse = oracle.attention(Q, Kn, Vn, Kl, Vl, *cu, 0.3)
    for i in range(q):
        vis = k + (m - q + i + 1)
        want = np.zeros(d_h)
        want[:vis] = 1.0 / vis
        assert np.allclose(O[i, 0], want, atol=1e-15)
        assert np.isclose(lse[i, 0], math.log(vis))


def test_single_key_and_equal_values_and_logit_shift():
    Q, Kn, Vn, Kl, Vl, cu = _inputs(53, [3], [5], [3], H=2, H_kv=2, d_h=8)
    Vn2, Vl2 = Vn.clone(), Vl.clone()
    Vn2[:] = Vl[0]
    Vl2[:] = Vl[0]
    O, _ = oracle.attention(*_np(Q, Kn, Vn2, Kl, Vl2), *cu, 0.5)
    assert np.allclose(O, np.broadcast_to(Vl[0].double().numpy(), O.shape), atol=1e-15)
    # one visible key: output is exactly its V row, lse its logit
    Q1, Kn1, Vn1, Kl1, Vl1, cu1 = _inputs(54, [1], [0], [1], H=1, H_kv=1, d_h=4)
    O1, lse1 = oracle.attention(*_np(Q1, Kn1, Vn1, Kl1, Vl1), *cu1, 2.0)
    assert np.array_equal(O1[0, 0], Vl1[0, 0].double().numpy())
    assert np.isclose(lse1[0, 0], 2.0 * float((Q1[0, 0].double() * Kl1[0, 0].double()).sum()))


def test_nugget_permutation_invariance_and_gqa_head_mapping():
    Q, Kn, Vn, Kl, Vl, cu = _inputs(55, [4], [7], [4], H=4, H_kv=2)
    O, lse = oracle.attention(*_np(Q, Kn, Vn, Kl, Vl), *cu, 0.4)
    perm = torch.tensor([3, 0, 6, 2, 5, 1, 4])
    O2, lse2 = oracle.attention(*_np(Q, Kn[perm], Vn[perm], Kl, Vl), *cu, 0.4)
    assert np.allclose(O, O2, rtol=1e-13, atol=1e-14) and np.allclose(lse, lse2, rtol=1e-13)
    # heads 0,1 share kv head 0 and heads 2,3 share kv head 1: expand to MHA and compare
    rep = lambda t: t.repeat_interleave(2, dim=1)
    O3, _ = oracle.attention(*_np(Q, rep(Kn), rep(Vn), rep(Kl), rep(Vl)), *cu, 0.4)
    assert np.array_equal(O, O3)


def test_split_identity_lse_merge():
    # Attn over [A ; B] == LSE-weighted merge of Attn(A) and Attn(B): pins lse and the nugget/local split
    Q, Kn, Vn, Kl, Vl, cu = _inputs(56, [1], [9], [5], H=2, H_kv=2)
    full, lse = oracle.attention(*_np(Q, Kn, Vn, Kl, Vl), *cu, 0.7)
    e = lambda t: t[:0]
    cu0 = oracle.cu_from_lengths([0])
    oa, la = oracle.attention(*_np(Q, Kn, Vn, e(Kl), e(Vl)), cu[0], cu[1], cu0, 0.7)
    ob, lb = oracle.attention(*_np(Q, e(Kn), e(Vn), Kl, Vl), cu[0], cu0, cu[2], 0.7)
    wa, wb = np.exp(la - lse)[..., None], np.exp(lb - lse)[..., None]
    assert np.allclose(full, wa * oa + wb * ob, rtol=1e-12, atol=1e-13)
    assert np.allclose(np.logaddexp(la, lb), lse, rtol=1e-13)


def test_block_rows_equal_one_row_decode_calls():
    # row i of a q-row block == a one-token call whose local buffer stops at that row
    q, k, tau = 5, 6, 3
    Q, Kn, Vn, Kl, Vl, cu = _inputs(57, [q], [k], [tau + q])
    O, lse = oracle.attention(*_np(Q, Kn, Vn, Kl, Vl), *cu, 0.35)
    for i in range(q):
        m_i = tau + i + 1
        Oi, li = oracle.attention(*_np(Q[i:i + 1], Kn, Vn, Kl[:m_i], Vl[:m_i]), oracle.cu_from_lengths([1]), cu[1],
                                  oracle.cu_from_lengths([m_i]), 0.35)
        assert np.array_equal(Oi[0], O[i]) and np.array_equal(li[0], lse[i])


def test_empty_visible_set_and_short_local_buffer():
    # m < q: the first rows see no local row; with no nuggets either they output 0 / -inf
    Q, Kn, Vn, Kl, Vl, cu = _inputs(58, [4], [0], [2], H=1, H_kv=1)
    O, lse = oracle.attention(*_np(Q, Kn, Vn, Kl, Vl), *cu, 1.0)
    assert np.all(O[:2] == 0) and np.all(np.isneginf(lse[:2]))
    assert np.array_equal(O[2, 0], Vl[0, 0].double().numpy())


def test_sampled_rows_equal_full_result_and_head_major_cache():
    Q, Kn, Vn, Kl, Vl, cu = _inputs(59, [3, 4], [5, 2], [6, 4], dtype=torch.bfloat16)
    O, lse = oracle.attention(*_np(Q, Kn, Vn, Kl, Vl), *cu, 0.3)
    rows = [(0, 0, 0), (1, 3, 3), (0, 2, 1), (1, 1, 0)]
    Or, lr = oracle.attention_rows(*_np(Q, Kn, Vn, Kl, Vl), *cu, 0.3, rows)
    for r, (b, h, i) in enumerate(rows):
        assert np.array_equal(Or[r], O[cu[0][b] + i, h]) and lr[r] == lse[cu[0][b] + i, h]
    Oh, _ = oracle.attention(*_np(Q, Kn.permute(1, 0, 2).contiguous(), Vn.permute(1, 0, 2).contiguous(), Kl, Vl),
                             *cu, 0.3, layout=oracle.HEAD_MAJOR)
    assert np.array_equal(O, Oh)


def test_whole_path_at_ratio_one_is_causal_attention_on_uncompressed_kv():
    # score -> select(k = n) -> gather -> attention == causal attention over the raw K/V
    wl = W.Workload("t", torch.float32, [13, 7], 16, 2, 2, 8, 1, 1, [3, 2], [0, 0], seed=77)
    t = W.make_inputs(wl)
    n = {k: W.to_numpy(v) for k, v in t.items()}
    s = oracle.score(n["hidden"], n["w"])
    k_lens = [oracle.nugget_count(x, wl.keep_num, wl.keep_den) for x in wl.seq_lens]
    cu_k = oracle.cu_from_lengths(k_lens)
    idx = oracle.select_topk(s, n["cu_seqlens"], cu_k, oracle.FORCE_LAST)
    Kn, Vn = oracle.gather(n["K"], n["V"], idx, n["cu_seqlens"], cu_k)
    assert np.array_equal(Kn, n["K"])
    O, _ = oracle.attention(n["Q"], Kn, Vn, n["Kl"], n["Vl"], n["cu_q"], cu_k, n["cu_local"], 0.25)
    want = dense_masked_softmax(t["Q"], t["K"], t["V"], t["Kl"], t["Vl"],
                                (n["cu_q"], n["cu_seqlens"], n["cu_local"]), 0.25)
    assert np.allclose(O, want, rtol=1e-12, atol=1e-13)


def test_indexed_form_is_masked_attention_over_the_uncompressed_context():
    # Attention over [all context tokens ; local rows] in float64 with every context token that is not a nugget
    # masked out never forms a packed cache, yet must give the same rows (softmax ignores the order of keys).
    n_lens, q_lens, H, H_kv, d_h = [50, 23], [6, 3], 4, 2, 8
    m_lens = [9, 3]
    N = sum(n_lens)
    K = W.normal(77, 0, (N, H_kv, d_h), 1.0, torch.float32)
    V = W.normal(77, 1, (N, H_kv, d_h), 1.0, torch.float32)
    Q = W.normal(77, 2, (sum(q_lens), H, d_h), 1.0, torch.float32)
    Kl = W.normal(77, 3, (sum(m_lens), H_kv, d_h), 1.0, torch.float32)
    Vl = W.normal(77, 4, (sum(m_lens), H_kv, d_h), 1.0, torch.float32)
    s = W.normal(77, 5, (N,), 1.0, torch.float32).numpy()
    k_lens = [oracle.nugget_count(n, 1, 5) for n in n_lens]
    cu_s, cu_k = oracle.cu_from_lengths(n_lens), oracle.cu_from_lengths(k_lens)
    cu_q, cu_l = oracle.cu_from_lengths(q_lens), oracle.cu_from_lengths(m_lens)
    idx = oracle.select_topk(s, cu_s, cu_k)
    scale = 0.3
    O, lse = oracle.attention_indexed(Q.numpy(), K.numpy(), V.numpy(), idx, cu_s, Kl.numpy(), Vl.numpy(), cu_q, cu_k,
                                      cu_l, scale)
    for b in range(2):
        chosen = torch.zeros(n_lens[b], dtype=torch.bool)
        chosen[torch.from_numpy(idx[cu_k[b]:cu_k[b + 1]]).long()] = True
        for h in range(H):
            kvh = h // (H // H_kv)
            keys = torch.cat([K[cu_s[b]:cu_s[b + 1], kvh], Kl[cu_l[b]:cu_l[b + 1], kvh]]).double()
            vals = torch.cat([V[cu_s[b]:cu_s[b + 1], kvh], Vl[cu_l[b]:cu_l[b + 1], kvh]]).double()
            for i in range(q_lens[b]):
                vis_local = torch.arange(m_lens[b]) <= m_lens[b] - q_lens[b] + i
                mask = torch.cat([chosen, vis_local])
                logits = (keys @ Q[cu_q[b] + i, h].double()) * scale
                logits[~mask] = -float("inf")
                p = torch.softmax(logits, 0)
                assert np.allclose(O[cu_q[b] + i, h], (p @ vals).numpy(), rtol=1e-12, atol=1e-13)
                assert np.isclose(lse[cu_q[b] + i, h], torch.logsumexp(logits, 0).item(), rtol=1e-12)
