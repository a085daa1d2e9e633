"""Pins for the oracle's score gradient of the straight-through estimator (Sec. 2.5, Eq. 17-18)."""
import numpy as np
import torch

import oracle
import workloads as W


def _case(seed, q_lens, k_lens, m_lens, H, H_kv, d_h):
    mk = lambda tid, n, h: W.normal(seed, tid, (n, h, d_h), 1.0, torch.float32)
    t = dict(Q=mk(0, sum(q_lens), H), Kn=mk(1, sum(k_lens), H_kv), Vn=mk(2, sum(k_lens), H_kv),
             Kl=mk(3, sum(m_lens), H_kv), Vl=mk(4, sum(m_lens), H_kv), dO=mk(5, sum(q_lens), H))
    cu = [oracle.cu_from_lengths(x) for x in (q_lens, k_lens, m_lens)]
    return t, cu


def _autograd(t, cu, scale, H, H_kv):
    """The paper's construction, literally: xi_bar = xi + s - stopgrad(s) on the nugget logits, loss = <O, dO>."""
    cu_q, cu_k, cu_l = cu
    s = torch.zeros(t["Kn"].shape[0], dtype=torch.float64, requires_grad=True)
    loss = torch.zeros((), dtype=torch.float64)
    for b in range(len(cu_q) - 1):
        q_b, k_b, m_b = (int(c[b + 1] - c[b]) for c in (cu_q, cu_k, cu_l))
        for h in range(H):
            kvh = h // (H // H_kv)
            q = t["Q"][cu_q[b]:cu_q[b + 1], h].double()
            kn, vn = t["Kn"][cu_k[b]:cu_k[b + 1], kvh].double(), t["Vn"][cu_k[b]:cu_k[b + 1], kvh].double()
            kl, vl = t["Kl"][cu_l[b]:cu_l[b + 1], kvh].double(), t["Vl"][cu_l[b]:cu_l[b + 1], kvh].double()
            sb = s[cu_k[b]:cu_k[b + 1]]
            xi_n = q @ kn.T + sb[None, :] - sb.detach()[None, :]
            xi_l = q @ kl.T
            i = torch.arange(q_b)[:, None]
            mask_l = torch.arange(m_b)[None, :] <= m_b - q_b + i
            xi = torch.cat([xi_n, xi_l.masked_fill(~mask_l, -float("inf"))], 1) * scale
            rows = torch.isfinite(xi).any(1)
            o = torch.softmax(xi[rows], 1) @ torch.cat([vn, vl])
            loss = loss + (o * t["dO"][cu_q[b]:cu_q[b + 1], h].double()[rows]).sum()
    loss.backward()
    return s.grad.numpy()


def test_matches_autograd_through_the_stop_gradient_construction():
    # ragged batch with GQA, a sequence without nuggets, one without local rows, rows that see nothing
    q_lens, k_lens, m_lens, H, H_kv, d_h = [7, 3, 5, 4], [6, 0, 9, 2], [9, 3, 0, 2], 4, 2, 8
    t, cu = _case(90, q_lens, k_lens, m_lens, H, H_kv, d_h)
    scale = 0.3
    got = oracle.ste_score_grad(*(t[k].numpy() for k in ("Q", "Kn", "Vn", "Kl", "Vl", "dO")), *cu, scale, scale)
    want = _autograd(t, cu, scale, H, H_kv)
    assert np.allclose(got, want, rtol=1e-10, atol=1e-12)
    assert np.abs(want).max() > 1e-3  # the case is not degenerate


def test_gradients_of_a_sequence_sum_to_minus_the_local_share():
    # a row's softmax-input gradients sum to zero over ALL its keys, so without local rows the nugget gradients of
    # every sequence cancel; with local rows they do not
    t, cu = _case(91, [5, 6], [4, 7], [0, 0], 2, 2, 8)
    g = oracle.ste_score_grad(*(t[k].numpy() for k in ("Q", "Kn", "Vn", "Kl", "Vl", "dO")), *cu, 0.5, 1.0)
    assert abs(g[:4].sum()) < 1e-12 and abs(g[4:].sum()) < 1e-12 and np.abs(g).max() > 1e-3
    t, cu = _case(91, [5, 6], [4, 7], [5, 8], 2, 2, 8)
    g = oracle.ste_score_grad(*(t[k].numpy() for k in ("Q", "Kn", "Vn", "Kl", "Vl", "dO")), *cu, 0.5, 1.0)
    assert abs(g[:4].sum()) > 1e-3


def test_single_nugget_single_local_row_closed_form():
    # one query, keys {nugget z, local x}: p = sigmoid(scale (q.z - q.x)), dl/dxi_z = p (1 - p) dO.(v_z - v_x)
    q = np.array([[[1.0, 2.0]]], np.float32); kz = np.array([[[0.5, -1.0]]], np.float32); vz = np.array([[[3.0, 1.0]]], np.float32)
    kx = np.array([[[2.0, 0.25]]], np.float32); vx = np.array([[[-1.0, 4.0]]], np.float32); dO = np.array([[[0.5, -2.0]]], np.float32)
    one = np.array([0, 1], np.int32)
    scale = 0.7
    p = 1.0 / (1.0 + np.exp(-scale * ((1 * 0.5 + 2 * -1.0) - (1 * 2.0 + 2 * 0.25))))
    want = 3.0 * p * (1 - p) * (0.5 * (3.0 - -1.0) + -2.0 * (1.0 - 4.0))
    got = oracle.ste_score_grad(q, kz, vz, kx, vx, dO, one, one, one, scale, 3.0)
    assert np.allclose(got, [want], rtol=1e-12)


def test_finite_difference_of_the_loss_in_the_nugget_logits():
    # central differences of <O, dO> in a bias added to one nugget's logits (all heads, all rows)
    q_lens, k_lens, m_lens, H, d_h = [4], [5], [6], 2, 8
    t, cu = _case(92, q_lens, k_lens, m_lens, H, H, d_h)
    scale = 0.4
    g = oracle.ste_score_grad(*(t[k].numpy() for k in ("Q", "Kn", "Vn", "Kl", "Vl", "dO")), *cu, scale, 1.0)

    def loss(bias):  # bias [k] added to the softmax input of the nugget columns
        total = 0.0
        for h in range(H):
            xi_n = scale * (t["Q"][:, h].double() @ t["Kn"][:, h].double().T) + torch.from_numpy(bias)[None, :]
            xi_l = scale * (t["Q"][:, h].double() @ t["Kl"][:, h].double().T)
            i = torch.arange(4)[:, None]
            xi_l = xi_l.masked_fill(~(torch.arange(6)[None, :] <= 6 - 4 + i), -float("inf"))
            o = torch.softmax(torch.cat([xi_n, xi_l], 1), 1) @ torch.cat([t["Vn"][:, h], t["Vl"][:, h]]).double()
            total += float((o * t["dO"][:, h].double()).sum())
        return total
    for i in range(5):
        e = np.zeros(5); e[i] = 1e-5
        fd = (loss(e) - loss(-e)) / 2e-5
        assert abs(fd - g[i]) < 1e-7 * max(1.0, abs(g[i]))


def test_plain_loops_equal_the_library_restatement():
    # the C++ loops against the same definition written with numpy's routines, bf16 and fp32, grouped heads,
    # sequences without nuggets, without local rows and with a local buffer shorter than the query block
    import numpy_pins
    import workloads as W
    for dtype in (torch.float32, torch.bfloat16):
        q_lens, k_lens, m_lens, H, H_kv, d_h = [5, 3, 0, 4], [7, 0, 3, 2], [9, 3, 2, 1], 4, 2, 16
        mk = lambda tid, n, h: W.to_numpy(W.normal(88, tid, (n, h, d_h), 1.0, dtype))
        Q, dO = mk(0, sum(q_lens), H), mk(1, sum(q_lens), H)
        Kn, Vn = mk(2, sum(k_lens), H_kv), mk(3, sum(k_lens), H_kv)
        Kl, Vl = mk(4, sum(m_lens), H_kv), mk(5, sum(m_lens), H_kv)
        cu = [oracle.cu_from_lengths(x) for x in (q_lens, k_lens, m_lens)]
        got = oracle.ste_score_grad(Q, Kn, Vn, Kl, Vl, dO, *cu, 0.25, 0.7)
        want = numpy_pins.ste_score_grad(Q, Kn, Vn, Kl, Vl, dO, *cu, 0.25, 0.7)
        assert np.allclose(got, want, rtol=1e-11, atol=1e-13)
