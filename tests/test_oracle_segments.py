"""Pins for the oracle's segment form of the autoregressive objective (Sec. 2.4, "Learning")."""
import numpy as np
import pytest
import torch

import oracle
import workloads as W


def _case(seed, n_lens, H, H_kv, d_h, dtype=torch.float32, keep=(1, 4)):
    N = sum(n_lens)
    mk = lambda tid, h: W.normal(seed, tid, (N, h, d_h), 1.0, dtype)
    Q, K, V, Ke, Ve = mk(0, H), mk(1, H_kv), mk(2, H_kv), mk(3, H_kv), mk(4, H_kv)  # Ke, Ve: the encoder's states
    s = W.normal(seed, 5, (N,), 1.0, torch.float32).numpy()
    k_lens = [oracle.nugget_count(n, *keep) for n in n_lens]
    cu_s, cu_k = oracle.cu_from_lengths(n_lens), oracle.cu_from_lengths(k_lens)
    idx = oracle.select_topk(s, cu_s, cu_k)
    Kn, Vn = oracle.gather(W.to_numpy(Ke), W.to_numpy(Ve), idx, cu_s, cu_k)
    return dict(Q=Q, K=K, V=V, Kn=Kn, Vn=Vn, idx=idx, cu_s=cu_s, cu_k=cu_k)


def test_plan_hand_example():
    # one text of 10 tokens, nuggets at 1, 4, 5, 9; segments of 4, tau = 2:
    #   c=0: t=0, tokens 0..3, no nugget, local rows 0..3      c=1: t=2, tokens 4..7, nuggets {1}, rows 2..7
    #   c=2: t=6, tokens 8..9, nuggets {1,4,5}, rows 6..9
    # a second text of 3 tokens with its single nugget at 2 starts at token 10 and nugget 4
    idx = np.array([1, 4, 5, 9, 2], np.int32)
    cu_q, ns, nl, ls, ll = oracle.segment_plan(idx, np.array([0, 10, 13], np.int32), np.array([0, 4, 5], np.int32), 4, 2)
    assert list(cu_q) == [0, 4, 8, 10, 13]
    assert list(ns) == [0, 0, 0, 4] and list(nl) == [0, 1, 3, 0]
    assert list(ls) == [0, 2, 6, 10] and list(ll) == [4, 6, 4, 3]


def test_one_segment_without_nuggets_is_causal_attention():
    # seg_len >= n: t = 0 for every token, no nugget is visible: plain causal self-attention
    c = _case(60, [19], 2, 2, 8)
    O, lse = oracle.attention_segment_mask(W.to_numpy(c["Q"]), c["Kn"], c["Vn"], W.to_numpy(c["K"]), W.to_numpy(c["V"]),
                                           c["idx"], c["cu_s"], c["cu_k"], 32, 5, 0.35)
    q, k, v = (t.double().transpose(0, 1) for t in (c["Q"], c["K"], c["V"]))
    want = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True, scale=0.35).transpose(0, 1)
    assert np.allclose(O, want.numpy(), rtol=1e-12, atol=1e-13)


def test_segments_of_one_token_are_decode_steps_of_the_mixed_resolution_rule():
    # seg_len = 1: token i has its own splitting index max(0, i - tau): Eq. 9 one token at a time, through the
    # decode form of the attention oracle (nuggets of the first i - tau tokens, tau earlier rows and the token itself)
    tau = 3
    c = _case(61, [14, 6], 4, 2, 8)
    Qn, Kx, Vx = W.to_numpy(c["Q"]), W.to_numpy(c["K"]), W.to_numpy(c["V"])
    O, lse = oracle.attention_segment_mask(Qn, c["Kn"], c["Vn"], Kx, Vx, c["idx"], c["cu_s"], c["cu_k"], 1, tau, 0.4)
    for b, n in enumerate([14, 6]):
        s0, k0, k1 = int(c["cu_s"][b]), int(c["cu_k"][b]), int(c["cu_k"][b + 1])
        for i in range(n):
            t = max(0, i - tau)
            kvis = int(np.sum(c["idx"][k0:k1] < t))
            one = lambda m: np.array([0, m], np.int32)
            Oi, li = oracle.attention(Qn[s0 + i:s0 + i + 1], c["Kn"][k0:k0 + kvis], c["Vn"][k0:k0 + kvis],
                                      Kx[s0 + t:s0 + i + 1], Vx[s0 + t:s0 + i + 1], one(1), one(kvis), one(i + 1 - t), 0.4)
            assert np.allclose(O[s0 + i], Oi[0], rtol=1e-12, atol=1e-13) and np.allclose(lse[s0 + i], li[0], rtol=1e-12)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_matches_dense_masked_softmax_built_from_the_rule(dtype):
    # keys = [every nugget of the text ; every token of the text]; the mask is written as boolean matrices
    seg_len, tau, scale = 5, 3, 0.3
    n_lens = [23, 9]
    c = _case(62, n_lens, 2, 1, 4, dtype, keep=(1, 3))
    O, lse = oracle.attention_segment_mask(W.to_numpy(c["Q"]), c["Kn"], c["Vn"], W.to_numpy(c["K"]), W.to_numpy(c["V"]),
                                           c["idx"], c["cu_s"], c["cu_k"], seg_len, tau, scale)
    f64 = lambda a: torch.from_numpy(oracle._to_f64(a)) if isinstance(a, np.ndarray) else a.double()
    for b, n in enumerate(n_lens):
        s0, k0, k1 = int(c["cu_s"][b]), int(c["cu_k"][b]), int(c["cu_k"][b + 1])
        i = torch.arange(n)[:, None]
        t = torch.clamp((i // seg_len) * seg_len - tau, min=0)
        nug_mask = torch.from_numpy(c["idx"][k0:k1].astype(np.int64))[None, :] < t
        tok = torch.arange(n)[None, :]
        mask = torch.cat([nug_mask, (tok >= t) & (tok <= i)], 1)
        for h in range(2):
            keys = torch.cat([f64(c["Kn"][k0:k1, 0]), f64(c["K"][s0:s0 + n, 0])])
            vals = torch.cat([f64(c["Vn"][k0:k1, 0]), f64(c["V"][s0:s0 + n, 0])])
            logits = scale * f64(c["Q"][s0:s0 + n, h]) @ keys.T
            logits = logits.masked_fill(~mask, -float("inf"))
            assert np.allclose(O[s0:s0 + n, h], (torch.softmax(logits, 1) @ vals).numpy(), rtol=1e-12, atol=1e-13)
            assert np.allclose(lse[s0:s0 + n, h], torch.logsumexp(logits, 1).numpy(), rtol=1e-12)


def test_plan_entries_reproduce_the_rule_through_the_batched_attention_oracle():
    # the plan's entries, fed to the attention oracle as a batch (ranges copied out), give the same rows
    seg_len, tau, scale = 6, 4, 0.25
    n_lens = [20, 7, 1]
    c = _case(63, n_lens, 2, 2, 8)
    Qn, Kx, Vx = W.to_numpy(c["Q"]), W.to_numpy(c["K"]), W.to_numpy(c["V"])
    O, lse = oracle.attention_segment_mask(Qn, c["Kn"], c["Vn"], Kx, Vx, c["idx"], c["cu_s"], c["cu_k"], seg_len, tau, scale)
    cu_q, ns, nl, ls, ll = oracle.segment_plan(c["idx"], c["cu_s"], c["cu_k"], seg_len, tau)
    assert len(ns) == sum(-(-n // seg_len) for n in n_lens)
    Kn = np.concatenate([c["Kn"][a:a + m] for a, m in zip(ns, nl)])
    Vn = np.concatenate([c["Vn"][a:a + m] for a, m in zip(ns, nl)])
    Kl = np.concatenate([Kx[a:a + m] for a, m in zip(ls, ll)])
    Vl = np.concatenate([Vx[a:a + m] for a, m in zip(ls, ll)])
    O2, lse2 = oracle.attention(Qn, Kn, Vn, Kl, Vl, cu_q, oracle.cu_from_lengths(list(nl)), oracle.cu_from_lengths(list(ll)), scale)
    assert np.allclose(O, O2, rtol=1e-12, atol=1e-13) and np.allclose(lse, lse2, rtol=1e-12)


def test_plain_loops_equal_the_library_restatement():
    # the C++ loops against the same definition written with numpy's routines (matrix products, exp, sums):
    # plan bit for bit, attention to double-precision rounding; bf16 and fp32 inputs, grouped heads, ragged texts
    import numpy_pins
    for dtype, n_lens, seg_len, tau, H, H_kv in ((torch.float32, [37, 1, 0, 20], 8, 3, 4, 2),
                                                 (torch.bfloat16, [50, 13], 16, 40, 2, 1)):
        N = sum(n_lens)
        mk = lambda tid, h: W.to_numpy(W.normal(77, tid, (N, h, 16), 1.0, dtype))
        Q, K, V, Ke, Ve = mk(0, H), mk(1, H_kv), mk(2, H_kv), mk(3, H_kv), mk(4, H_kv)
        k_lens = [oracle.nugget_count(n, 1, 4) for n in n_lens]
        cu_s, cu_k = oracle.cu_from_lengths(n_lens), oracle.cu_from_lengths(k_lens)
        idx = oracle.select_topk(W.normal(77, 5, (N,), 1.0, torch.float32).numpy(), cu_s, cu_k)
        Kn, Vn = oracle.gather(Ke, Ve, idx, cu_s, cu_k)
        for a, b in zip(oracle.segment_plan(idx, cu_s, cu_k, seg_len, tau), numpy_pins.segment_plan(idx, cu_s, cu_k, seg_len, tau)):
            assert np.array_equal(a, b)
        O, lse = oracle.attention_segment_mask(Q, Kn, Vn, K, V, idx, cu_s, cu_k, seg_len, tau, 0.3)
        O2, lse2 = numpy_pins.attention_segment_mask(Q, Kn, Vn, K, V, idx, cu_s, cu_k, seg_len, tau, 0.3)
        assert np.allclose(O, O2, rtol=1e-12, atol=1e-13) and np.allclose(lse, lse2, rtol=1e-12, atol=1e-13)
