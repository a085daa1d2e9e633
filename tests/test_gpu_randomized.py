"""GPU parity on seeded random ragged shapes: both attention kernels, the TopK select (one workgroup per sequence
and chunked), the score gradient and the 2-layer scorer against the oracle.  Complements the hand-picked cases."""
import numpy as np
import pytest
import torch

import oracle
import workloads as W
from gpu_util import check_attention, check_lse, dev, make_attention_case

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def D():
    import paper_2310_02409_amd as D
    return D


def test_attention_random_shapes(D):
    rng = np.random.default_rng(11)
    for it in range(40):
        B = int(rng.integers(1, 5))
        block = rng.random() < 0.6  # query-block kernel (bf16, >= 16 rows) or split-K kernel
        dtype = torch.bfloat16 if block or rng.random() < 0.5 else torch.float32
        d_h = int(rng.choice([64, 128]))
        H_kv = int(rng.choice([1, 2, 4]))
        H = H_kv * int(rng.choice([1, 2]))
        qmax = int(rng.choice([16, 64, 130, 300, 520])) if block else int(rng.choice([1, 3, 9]))
        q_lens = [int(rng.integers(0 if B > 1 else 1, qmax + 1)) for _ in range(B)]
        q_lens[0] = max(q_lens[0], 16 if block else 1)
        k_lens = [int(rng.integers(0, 600)) for _ in range(B)]
        m_lens = [int(rng.integers(0, 700)) for _ in range(B)]
        host, d = make_attention_case(1000 + it, q_lens, k_lens, m_lens, H, H_kv, d_h, dtype, dev())
        scale = d_h ** -0.5
        O_ref, lse_ref = oracle.attention(host["Q"], host["Kn"], host["Vn"], host["Kl"], host["Vl"], host["cu_q"],
                                          host["cu_nuggets"], host["cu_local"], scale)
        O, lse = D.dodo_nugget_attention(d["Q"], d["Kn"], d["Vn"], d["Kl"], d["Vl"], d["cu_q"], d["cu_nuggets"],
                                         d["cu_local"], max(q_lens), max(k_lens), max(m_lens), scale, want_lse=True)
        case = f"case {it}: {dtype} d_h={d_h} H={H}/{H_kv} q={q_lens} k={k_lens} m={m_lens}"
        try:
            check_attention(O, O_ref, dtype)
            check_lse(lse, lse_ref, dtype)
        except AssertionError as e:
            raise AssertionError(f"{case}: {e}") from e


def test_attention_random_shapes_shared_kv_rows(D):
    # many (sequence, head, row) triples, several query heads per KV head and / or a few query rows: the split-K
    # kernel serves up to 8 query vectors that read the same K/V rows from one workgroup (heads x rows in all
    # combinations the launch rule picks), each row with its own causal limit
    rng = np.random.default_rng(15)
    for it in range(14):
        B = int(rng.integers(6, 40))
        dtype = torch.bfloat16 if rng.random() < 0.6 else torch.float32
        d_h = int(rng.choice([64, 128]))
        H_kv = int(rng.choice([1, 2, 4]))
        H = H_kv * int(rng.choice([1, 2, 4, 8]))
        qmax = int(rng.choice([1, 2, 3, 5, 8, 13]))
        q_lens = [int(rng.integers(0, qmax + 1)) for _ in range(B)]
        q_lens[0] = qmax
        k_lens = [int(rng.integers(0, 300)) for _ in range(B)]
        m_lens = [int(rng.integers(0, 200)) for _ in range(B)]
        if it % 5 == 4:  # long rows as well: several splits per row group, merged by the last one
            k_lens[1], m_lens[1] = 2500, 900
        host, d = make_attention_case(5000 + it, q_lens, k_lens, m_lens, H, H_kv, d_h, dtype, dev())
        scale = d_h ** -0.5
        O_ref, lse_ref = oracle.attention(host["Q"], host["Kn"], host["Vn"], host["Kl"], host["Vl"], host["cu_q"],
                                          host["cu_nuggets"], host["cu_local"], scale)
        O, lse = D.dodo_nugget_attention(d["Q"], d["Kn"], d["Vn"], d["Kl"], d["Vl"], d["cu_q"], d["cu_nuggets"],
                                         d["cu_local"], max(q_lens), max(k_lens), max(m_lens), scale, want_lse=True)
        case = f"case {it}: {dtype} d_h={d_h} H={H}/{H_kv} q={q_lens} k={k_lens} m={m_lens}"
        try:
            check_attention(O, O_ref, dtype)
            check_lse(lse, lse_ref, dtype)
        except AssertionError as e:
            raise AssertionError(f"{case}: {e}") from e


def test_select_random_shapes(D):
    rng = np.random.default_rng(12)
    for it in range(16):
        B = int(rng.integers(1, 6))
        long_seqs = it % 2 == 0  # long sequences take the chunked form (the binding passes the workspace)
        n_lens = [int(rng.integers(0, 40000 if long_seqs else 5000)) for _ in range(B)]
        n_lens[0] = max(n_lens[0], 5)
        k_lens = [int(rng.integers(0, n + 1)) for n in n_lens]
        k_lens[0] = max(k_lens[0], 1)
        flags = int(rng.integers(0, 2))
        s = W.normal(2000 + it, 0, (sum(n_lens),), 1.0, torch.float32)
        if rng.random() < 0.5:
            s = W.quantise16(s)
        cu_s, cu_k = oracle.cu_from_lengths(n_lens), oracle.cu_from_lengths(k_lens)
        ref = oracle.select_topk(s.numpy(), cu_s, cu_k, flags)
        got = D.dodo_select_topk(s.to(dev()), torch.from_numpy(cu_s).to(dev()), torch.from_numpy(cu_k).to(dev()),
                                 max(n_lens), max(k_lens), int(cu_k[-1]), flags)
        assert np.array_equal(got.cpu().numpy(), ref), f"case {it}: n={n_lens} k={k_lens} flags={flags}"


def test_score_gradient_random_shapes(D):
    rng = np.random.default_rng(13)
    for it in range(8):
        B = int(rng.integers(1, 4))
        H_kv = int(rng.choice([1, 2]))
        H = H_kv * int(rng.choice([1, 2]))
        q_lens = [int(rng.integers(0, 400)) for _ in range(B)]
        q_lens[0] = max(q_lens[0], 16)
        k_lens = [int(rng.integers(0, 700)) for _ in range(B)]
        k_lens[0] = max(k_lens[0], 1)
        m_lens = [int(rng.integers(0, 300)) for _ in range(B)]
        mk = lambda tid, n, h: W.normal(3000 + it, tid, (n, h, 128), 1.0, torch.bfloat16)
        t = dict(Q=mk(0, sum(q_lens), H), Kn=mk(1, sum(k_lens), H_kv), Vn=mk(2, sum(k_lens), H_kv),
                 Kl=mk(3, sum(m_lens), H_kv), Vl=mk(4, sum(m_lens), H_kv), dO=mk(5, sum(q_lens), H))
        cu = [oracle.cu_from_lengths(x) for x in (q_lens, k_lens, m_lens)]
        scale = 128 ** -0.5
        want = oracle.ste_score_grad(*(W.to_numpy(t[k]) for k in ("Q", "Kn", "Vn", "Kl", "Vl", "dO")), *cu, scale, 1.0)
        d = {k: v.to(dev()) for k, v in t.items()}
        cq, ck, cl = (torch.from_numpy(c).to(dev()) for c in cu)
        O, lse = D.dodo_nugget_attention(d["Q"], d["Kn"], d["Vn"], d["Kl"], d["Vl"], cq, ck, cl, max(q_lens), max(k_lens),
                                         max(m_lens), scale, want_lse=True)
        got = D.dodo_ste_score_grad(d["Q"], d["Kn"], d["Vn"], d["dO"], O, lse, cq, ck, max(q_lens), max(k_lens), scale,
                                    1.0).cpu().double().numpy()
        ref = max(np.abs(want).max(), 1e-30)
        assert np.abs(got - want).max() <= 2e-2 * ref, f"case {it}: q={q_lens} k={k_lens} m={m_lens}"


def test_score_mlp_random_shapes(D):
    rng = np.random.default_rng(14)
    for it in range(8):
        N, d = int(rng.integers(1, 1500)), 64 * int(rng.integers(1, 6))
        dh, act = 256 * int(rng.integers(1, 7)), int(rng.integers(0, 3))
        x = W.normal(4000 + it, 0, (N, d), 1.0, torch.bfloat16)
        W1 = W.normal(4000 + it, 1, (dh, d), d ** -0.5, torch.bfloat16)
        b1 = W.normal(4000 + it, 2, (dh,), 0.5, torch.float32)
        w2 = W.normal(4000 + it, 3, (dh,), dh ** -0.5, torch.bfloat16)
        want = oracle.score_mlp(W.to_numpy(x), W.to_numpy(W1), b1.numpy(), W.to_numpy(w2), 0.1, act)
        got = D.dodo_score_mlp(x.to(dev()), W1.to(dev()), b1.to(dev()), w2.to(dev()), 0.1, act).cpu().numpy()
        assert np.all(np.abs(got - want) <= 1e-4 * (1 + np.abs(want))), f"case {it}: N={N} d={d} d_hid={dh} act={act}"
