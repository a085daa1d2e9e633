"""The same three definitions written a second time, with numpy's library routines (matrix products, exp, sums),
as pins of the C++ oracle's plain loops: the segment plan and segment-mask attention of the autoregressive
objective (Sec. 2.4) and the score gradient of the straight-through estimator (Sec. 2.5, Eq. 17-18)."""
import numpy as np


def _to_f64(a: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    assert a.dtype == np.float32
    return a.astype(np.float64)


def segment_plan(nugget_idx, cu_seqlens, cu_nuggets, seg_len: int, tau: int):
    """Entries of the segment form of the autoregressive objective (Sec. 2.4, "Learning"): the tokens of segment c
    of a text share the splitting index t = max(0, c seg_len - tau).  Returns int32 arrays
    (seg_cu_q [E+1], nug_start, nug_len, loc_start, loc_len [E]), texts in order, segments in order."""
    cu_q, ns, nl, ls, ll = [], [], [], [], []
    B = len(cu_seqlens) - 1
    for b in range(B):
        s0, n = int(cu_seqlens[b]), int(cu_seqlens[b + 1] - cu_seqlens[b])
        idx = [int(i) for i in nugget_idx[cu_nuggets[b]:cu_nuggets[b + 1]]]
        c = 0
        while c * seg_len < n:
            t = max(0, c * seg_len - tau)
            cu_q.append(s0 + c * seg_len)
            ns.append(int(cu_nuggets[b]))
            nl.append(sum(1 for i in idx if i < t))
            ls.append(s0 + t)
            ll.append(min((c + 1) * seg_len, n) - t)
            c += 1
    cu_q.append(int(cu_seqlens[B]))
    return tuple(np.asarray(a, dtype=np.int32) for a in (cu_q, ns, nl, ls, ll))


def attention_segment_mask(Q, Kn, Vn, K, V, nugget_idx, cu_seqlens, cu_nuggets, seg_len: int, tau: int, scale: float):
    """Attention under the segment form of the autoregressive objective (Sec. 2.4, Eq. 9 with a splitting index
    shared by the tokens of a segment), one query token at a time: token i of a text, in segment c = i // seg_len
    with t = max(0, c seg_len - tau), attends over the text's nuggets whose index is below t (rows of the packed,
    token-major Kn / Vn) and the text's own tokens t .. i (rows of K / V).  Returns (O, lse) in float64."""
    Q, Kn, Vn, K, V = (_to_f64(a) for a in (Q, Kn, Vn, K, V))
    N, H, d_h = Q.shape
    H_kv = K.shape[1]
    O = np.zeros((N, H, d_h))
    lse = np.zeros((N, H))
    for b in range(len(cu_seqlens) - 1):
        s0, n = int(cu_seqlens[b]), int(cu_seqlens[b + 1] - cu_seqlens[b])
        k0, k1 = int(cu_nuggets[b]), int(cu_nuggets[b + 1])
        for i in range(n):
            t = max(0, (i // seg_len) * seg_len - tau)
            nug_rows = [k0 + j for j in range(k1 - k0) if nugget_idx[k0 + j] < t]
            for h in range(H):
                kvh = h // (H // H_kv)
                keys = np.concatenate([Kn[nug_rows, kvh], K[s0 + t:s0 + i + 1, kvh]])
                vals = np.concatenate([Vn[nug_rows, kvh], V[s0 + t:s0 + i + 1, kvh]])
                logits = scale * (keys @ Q[s0 + i, h])
                m = logits.max()
                p = np.exp(logits - m)
                O[s0 + i, h] = (p @ vals) / p.sum()
                lse[s0 + i, h] = m + np.log(p.sum())
    return O, lse


def ste_score_grad(Q, Kn, Vn, Kl, Vl, dO, cu_q, cu_nuggets, cu_local, scale: float, grad_scale: float):
    """Gradient that the straight-through estimator hands to the scores (Sec. 2.5, Eq. 17-18) for one layer:
    grad[i] = grad_scale * sum over heads h and query rows j of dl/dxi[j, i], where xi[j, i] is the input of the
    softmax for query row j and nugget i, and dl/dxi = P (dP - D) with P the attention weights of Eq. 13 / Eq. 9
    (over nuggets and the causally visible local rows), dP[j, i] = dO[j] . v_i and D[j] = dO[j] . O[j].
    Token-major nugget cache; returns float64 [Kt]."""
    Q, Kn, Vn, Kl, Vl, dO = (_to_f64(a) for a in (Q, Kn, Vn, Kl, Vl, dO))
    H, H_kv = Q.shape[1], Kl.shape[1]
    grad = np.zeros(Kn.shape[0])
    for b in range(len(cu_q) - 1):
        q0, q1 = int(cu_q[b]), int(cu_q[b + 1])
        k0, k1 = int(cu_nuggets[b]), int(cu_nuggets[b + 1])
        l0, l1 = int(cu_local[b]), int(cu_local[b + 1])
        q_b, k_b, m_b = q1 - q0, k1 - k0, l1 - l0
        for h in range(H):
            kvh = h // (H // H_kv)
            keys = np.concatenate([Kn[k0:k1, kvh], Kl[l0:l1, kvh]])
            vals = np.concatenate([Vn[k0:k1, kvh], Vl[l0:l1, kvh]])
            for j in range(q_b):
                n_loc = max(0, min(m_b, m_b - q_b + j + 1))
                vis = k_b + n_loc
                if vis == 0 or k_b == 0:
                    continue
                xi = scale * (keys[:vis] @ Q[q0 + j, h])
                p = np.exp(xi - xi.max())
                p /= p.sum()
                o = p @ vals[:vis]
                d_p = vals[:k_b] @ dO[q0 + j, h]
                big_d = dO[q0 + j, h] @ o
                grad[k0:k1] += grad_scale * p[:k_b] * (d_p - big_d)
    return grad


