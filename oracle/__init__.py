"""Dodo hot-path oracle: TEST INFRASTRUCTURE, not product code.

Thin numpy/ctypes front end of ``dodo_oracle.cpp`` (every function's arithmetic is there) -- the plain,
single-threaded, double-precision CPU statement of the Dodo compression path
(arXiv 2310.02409: Eq. 5, 6, 8, 9, 13, 14, 15 and the count rule of Sec. 2.3).
Only the tests, the smoke check and the benchmark's ``cpu_baseline`` leg may
import this package; the HIP library never does, and nothing here imports it.

Arrays are numpy: ``float32`` for fp32 data, ``uint16`` for bfloat16 bit
patterns.  All index arrays are ``int32``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dodo_oracle.cpp")
_LIB = os.path.join(_HERE, "libdodo_oracle.so")

F32, BF16 = 0, 1
FORCE_LAST = 1
TOKEN_MAJOR, HEAD_MAJOR = 0, 1

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (host only).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-std=c++17", "-O2", "-fPIC", "-shared", "-Wall", "-Wextra", "-ffp-contract=off",
               _SRC, "-o", _LIB]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.oracle_nugget_count.restype = ctypes.c_int64
        lib.oracle_nugget_count.argtypes = [ctypes.c_int64] * 3
        lib.oracle_select_topk.restype = ctypes.c_int
        lib.oracle_threshold_from_sample.restype = ctypes.c_float
        lib.oracle_stream_append.restype = ctypes.c_int32
        lib.oracle_select_threshold_indices.restype = None
        lib.oracle_segment_plan.restype = ctypes.c_int64
        lib.oracle_attention_segment_mask.restype = None
        lib.oracle_ste_score_grad.restype = None
        for name in ("oracle_score", "oracle_score_mlp", "oracle_select_threshold", "oracle_gather", "oracle_meanpool", "oracle_attention",
                     "oracle_attention_rows"):
            getattr(lib, name).restype = None
        _lib = lib
    return _lib


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError(f"oracle takes float32 or uint16 (bf16 bits) arrays, got {a.dtype}")


def _p(a):
    return ctypes.c_void_p(a.ctypes.data) if a is not None else ctypes.c_void_p(0)


def _c(a, dtype=None):
    a = np.ascontiguousarray(a) if dtype is None else np.ascontiguousarray(a, dtype=dtype)
    return a


def _to_f64(a: np.ndarray) -> np.ndarray:
    """float32 values, or bf16 values given as their uint16 bits, as float64 (exact)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    assert a.dtype == np.float32
    return a.astype(np.float64)


def nugget_count(n: int, num: int, den: int) -> int:
    """k = clamp(ceil(n * num / den), 1, n); 0 for an empty context (Sec. 2.3, Eq. 7)."""
    return int(_load().oracle_nugget_count(int(n), int(num), int(den)))


def cu_from_lengths(lengths) -> np.ndarray:
    cu = np.zeros(len(lengths) + 1, dtype=np.int64)
    np.cumsum(np.asarray(lengths, dtype=np.int64), out=cu[1:])
    assert cu[-1] < 2**31
    return cu.astype(np.int32)


def score(hidden: np.ndarray, w: np.ndarray, bias: float = 0.0) -> np.ndarray:
    """Linear-head Scorer (Eq. 6 / Eq. 15) over a packed [N, d] array -> fp32 [N]."""
    hidden, w = _c(hidden), _c(w)
    assert hidden.ndim == 2 and w.shape == (hidden.shape[1],) and w.dtype == hidden.dtype
    N, d = hidden.shape
    out = np.empty(N, dtype=np.float32)
    _load().oracle_score(_p(hidden), _p(w), ctypes.c_float(bias), _dtype_code(hidden), ctypes.c_int64(N),
                         ctypes.c_int64(d), ctypes.c_int64(d), _p(out))
    return out


def score_layers(hidden: np.ndarray, w: np.ndarray, biases=None) -> np.ndarray:
    """The Scorer of Eq. 6 / Eq. 15 layer by layer: hidden [L, N, d], w [L, d], biases [L] or None -> fp32 [L, N]."""
    assert hidden.ndim == 3 and w.shape == (hidden.shape[0], hidden.shape[2])
    return np.stack([score(hidden[l], w[l], 0.0 if biases is None else float(biases[l])) for l in range(hidden.shape[0])])


RELU, GELU, TANH = 0, 1, 2


def score_mlp(hidden: np.ndarray, W1: np.ndarray, b1: np.ndarray, w2: np.ndarray, b2: float = 0.0,
              act: int = RELU) -> np.ndarray:
    """2-layer scorer (App. B): s = w2 . act(W1 x + b1) + b2, W1 [d_hid, d]; fp32 [N]."""
    hidden, W1, w2 = _c(hidden), _c(W1), _c(w2)
    b1 = _c(b1, np.float32)
    assert hidden.ndim == 2 and W1.ndim == 2 and W1.shape[1] == hidden.shape[1] and W1.shape[0] == len(w2) == len(b1)
    assert hidden.dtype == W1.dtype == w2.dtype
    N, d = hidden.shape
    out = np.empty(N, dtype=np.float32)
    _load().oracle_score_mlp(_p(hidden), _p(W1), _p(b1), _p(w2), ctypes.c_float(b2), ctypes.c_int(act),
                             _dtype_code(hidden), ctypes.c_int64(N), ctypes.c_int64(d), ctypes.c_int64(W1.shape[0]),
                             ctypes.c_int64(d), _p(out))
    return out


def select_topk(scores: np.ndarray, cu_seqlens: np.ndarray, cu_nuggets: np.ndarray, flags: int = 0) -> np.ndarray:
    """TopK selection (Eq. 14): sequence-local, ascending indices, packed by cu_nuggets."""
    scores = _c(scores, np.float32)
    cu_seqlens, cu_nuggets = _c(cu_seqlens, np.int32), _c(cu_nuggets, np.int32)
    B = len(cu_seqlens) - 1
    out = np.empty(int(cu_nuggets[-1]), dtype=np.int32)
    rc = _load().oracle_select_topk(_p(scores), _p(cu_seqlens), _p(cu_nuggets), ctypes.c_int32(B),
                                    ctypes.c_uint32(flags), _p(out))
    if rc != 0:
        raise ValueError("nugget count exceeds sequence length")
    return out


def select_threshold(scores: np.ndarray, cu_seqlens: np.ndarray, lam: float):
    """Threshold selection (Eq. 8): (alpha flags uint8 [N], kept count per sequence int32 [B])."""
    scores, cu_seqlens = _c(scores, np.float32), _c(cu_seqlens, np.int32)
    B = len(cu_seqlens) - 1
    alpha = np.zeros(len(scores), dtype=np.uint8)
    counts = np.zeros(B, dtype=np.int32)
    _load().oracle_select_threshold(_p(scores), _p(cu_seqlens), ctypes.c_int32(B), ctypes.c_float(lam), _p(alpha),
                                    _p(counts))
    return alpha, counts


def meanpool(K: np.ndarray, V: np.ndarray, cu_seqlens: np.ndarray, cu_nuggets: np.ndarray, layout: int = TOKEN_MAJOR):
    """Pooling baseline's compaction (Sec. 5.1): k_b even chunks per sequence, each mean-pooled into one row."""
    K, V = _c(K), _c(V)
    assert K.ndim == 3 and K.shape == V.shape and K.dtype == V.dtype
    cu_seqlens, cu_nuggets = _c(cu_seqlens, np.int32), _c(cu_nuggets, np.int32)
    _, H_kv, d_h = K.shape
    B = len(cu_seqlens) - 1
    Kt = int(cu_nuggets[-1])
    shape = (Kt, H_kv, d_h) if layout == TOKEN_MAJOR else (H_kv, Kt, d_h)
    Kn, Vn = np.zeros(shape, dtype=K.dtype), np.zeros(shape, dtype=K.dtype)
    _load().oracle_meanpool(_p(K), _p(V), _dtype_code(K), _p(cu_seqlens), _p(cu_nuggets), ctypes.c_int32(B),
                            ctypes.c_int64(Kt), ctypes.c_int32(H_kv), ctypes.c_int32(d_h),
                            ctypes.c_int64(H_kv * d_h), _p(Kn), _p(Vn), ctypes.c_int(layout))
    return Kn, Vn


def threshold_from_sample(sample: np.ndarray, num: int, den: int) -> float:
    """Threshold calibration (Sec. 2.4): the (k+1)-th highest of the sampled scores, k = nugget_count(n)."""
    sample = _c(sample, np.float32)
    return float(_load().oracle_threshold_from_sample(_p(sample), ctypes.c_int64(len(sample)), ctypes.c_int64(num),
                                                      ctypes.c_int64(den)))


def select_threshold_indices(scores: np.ndarray, cu_seqlens: np.ndarray, lam: float):
    """Threshold selection (Eq. 8) as packed index lists: (counts [B], cu_nuggets [B+1], nugget_idx [sum counts])."""
    scores, cu_seqlens = _c(scores, np.float32), _c(cu_seqlens, np.int32)
    B = len(cu_seqlens) - 1
    counts = np.zeros(B, dtype=np.int32)
    cu_nuggets = np.zeros(B + 1, dtype=np.int32)
    idx = np.zeros(len(scores), dtype=np.int32)
    _load().oracle_select_threshold_indices(_p(scores), _p(cu_seqlens), ctypes.c_int32(B), ctypes.c_float(lam),
                                            _p(counts), _p(cu_nuggets), _p(idx))
    return counts, cu_nuggets, idx[: int(cu_nuggets[-1])].copy()


def stream_append(scores: np.ndarray, lam: float, K_rows: np.ndarray, V_rows: np.ndarray, counts: np.ndarray,
                  Kn: np.ndarray, Vn: np.ndarray) -> int:
    """One step of the autoregressive mode: append the rows [B, H_kv, d_h] whose score exceeds lam to the caches
    [B, cap, H_kv, d_h] in place, update counts in place; returns how many tokens a full cache dropped."""
    scores = _c(scores, np.float32)
    K_rows, V_rows = _c(K_rows), _c(V_rows)
    assert Kn.flags.c_contiguous and Vn.flags.c_contiguous and counts.dtype == np.int32 and counts.flags.c_contiguous
    B, H_kv, d_h = K_rows.shape
    cap = Kn.shape[1]
    return int(_load().oracle_stream_append(_p(scores), ctypes.c_float(lam), _p(K_rows), _p(V_rows), _dtype_code(K_rows),
                                            ctypes.c_int32(B), ctypes.c_int32(H_kv), ctypes.c_int32(d_h),
                                            ctypes.c_int64(H_kv * d_h), ctypes.c_int32(cap), _p(counts), _p(Kn),
                                            _p(Vn)))


def gather(K: np.ndarray, V: np.ndarray, nugget_idx: np.ndarray, cu_seqlens: np.ndarray, cu_nuggets: np.ndarray,
           layout: int = TOKEN_MAJOR):
    """Sub-selection (Eq. 5) of K/V rows [N, H_kv, d_h] into the nugget cache."""
    K, V = _c(K), _c(V)
    assert K.ndim == 3 and K.shape == V.shape and K.dtype == V.dtype
    nugget_idx, cu_seqlens, cu_nuggets = _c(nugget_idx, np.int32), _c(cu_seqlens, np.int32), _c(cu_nuggets, np.int32)
    _, H_kv, d_h = K.shape
    B = len(cu_seqlens) - 1
    Kt = int(cu_nuggets[-1])
    shape = (Kt, H_kv, d_h) if layout == TOKEN_MAJOR else (H_kv, Kt, d_h)
    Kn, Vn = np.zeros(shape, dtype=K.dtype), np.zeros(shape, dtype=K.dtype)
    _load().oracle_gather(_p(K), _p(V), _dtype_code(K), _p(nugget_idx), _p(cu_seqlens), _p(cu_nuggets),
                          ctypes.c_int32(B), ctypes.c_int64(Kt), ctypes.c_int32(H_kv), ctypes.c_int32(d_h),
                          ctypes.c_int64(H_kv * d_h), _p(Kn), _p(Vn), ctypes.c_int(layout))
    return Kn, Vn


def gather_layers(K: np.ndarray, V: np.ndarray, nugget_idx: np.ndarray, cu_seqlens: np.ndarray, cu_nuggets: np.ndarray,
                  layout: int = TOKEN_MAJOR):
    """Sub-selection (Eq. 5) of K/V [L, N, H_kv, d_h]: every layer is packed with the one index list (Sec. 2.1)."""
    assert K.ndim == 4 and K.shape == V.shape
    per_layer = [gather(K[l], V[l], nugget_idx, cu_seqlens, cu_nuggets, layout) for l in range(K.shape[0])]
    return np.stack([kv[0] for kv in per_layer]), np.stack([kv[1] for kv in per_layer])


def _attn_common(Q, Kn, Vn, Kl, Vl, cu_q, cu_nuggets, cu_local, layout):
    Q, Kn, Vn, Kl, Vl = _c(Q), _c(Kn), _c(Vn), _c(Kl), _c(Vl)
    assert Q.ndim == 3 and Kn.ndim == 3 and Kl.ndim == 3
    assert Q.dtype == Kn.dtype == Vn.dtype == Kl.dtype == Vl.dtype
    cu_q, cu_nuggets, cu_local = _c(cu_q, np.int32), _c(cu_nuggets, np.int32), _c(cu_local, np.int32)
    _, H, d_h = Q.shape
    H_kv = Kl.shape[1]
    Kt = int(cu_nuggets[-1])
    want = (Kt, H_kv, d_h) if layout == TOKEN_MAJOR else (H_kv, Kt, d_h)
    assert Kn.shape == want and Vn.shape == want, (Kn.shape, want)
    assert Kl.shape == Vl.shape == (int(cu_local[-1]), H_kv, d_h)
    assert Q.shape[0] == int(cu_q[-1]) and H % H_kv == 0
    return Q, Kn, Vn, Kl, Vl, cu_q, cu_nuggets, cu_local, H, H_kv, d_h, Kt


def attention(Q, Kn, Vn, Kl, Vl, cu_q, cu_nuggets, cu_local, scale: float, layout: int = TOKEN_MAJOR):
    """Nugget attention (Eq. 13 / Eq. 9) for all rows -> (O float64 [Sq,H,d_h], lse float64 [Sq,H])."""
    Q, Kn, Vn, Kl, Vl, cu_q, cu_nuggets, cu_local, H, H_kv, d_h, Kt = _attn_common(
        Q, Kn, Vn, Kl, Vl, cu_q, cu_nuggets, cu_local, layout)
    B = len(cu_q) - 1
    O = np.zeros(Q.shape, dtype=np.float64)
    lse = np.zeros(Q.shape[:2], dtype=np.float64)
    _load().oracle_attention(_p(Q), _p(Kn), _p(Vn), _p(Kl), _p(Vl), _p(cu_q), _p(cu_nuggets), _p(cu_local),
                             ctypes.c_int32(B), ctypes.c_int32(H), ctypes.c_int32(H_kv), ctypes.c_int32(d_h),
                             ctypes.c_double(scale), _dtype_code(Q), ctypes.c_int(layout), ctypes.c_int64(Kt),
                             _p(O), _p(lse))
    return O, lse


def attention_indexed(Q, K, V, nugget_idx, cu_seqlens, Kl, Vl, cu_q, cu_nuggets, cu_local, scale: float):
    """Nugget attention with the nuggets named by an index list into the context's K, V [N, H_kv, d_h]: the
    sub-selection of Eq. 5 followed by the attention of Eq. 13 / Eq. 9, as two steps."""
    Kn, Vn = gather(K, V, nugget_idx, cu_seqlens, cu_nuggets, TOKEN_MAJOR)
    return attention(Q, Kn, Vn, Kl, Vl, cu_q, cu_nuggets, cu_local, scale, TOKEN_MAJOR)


def segment_plan(nugget_idx, cu_seqlens, cu_nuggets, seg_len: int, tau: int):
    """Entries of the segment form of the autoregressive objective (Sec. 2.4, "Learning"): the tokens of segment c
    of a text share the splitting index t = max(0, c seg_len - tau).  Returns int32 arrays
    (seg_cu_q [E+1], nug_start, nug_len, loc_start, loc_len [E]), texts in order, segments in order."""
    nugget_idx, cu_seqlens, cu_nuggets = _c(nugget_idx, np.int32), _c(cu_seqlens, np.int32), _c(cu_nuggets, np.int32)
    B = len(cu_seqlens) - 1
    E = sum(-(-int(cu_seqlens[b + 1] - cu_seqlens[b]) // seg_len) for b in range(B))
    cu_q = np.zeros(E + 1, dtype=np.int32)
    ns, nl, ls, ll = (np.zeros(E, dtype=np.int32) for _ in range(4))
    got = _load().oracle_segment_plan(_p(nugget_idx), _p(cu_seqlens), _p(cu_nuggets), ctypes.c_int32(B),
                                      ctypes.c_int32(seg_len), ctypes.c_int32(tau), ctypes.c_int64(E), _p(cu_q), _p(ns),
                                      _p(nl), _p(ls), _p(ll))
    assert got == E
    return cu_q, ns, nl, ls, ll


def attention_segment_mask(Q, Kn, Vn, K, V, nugget_idx, cu_seqlens, cu_nuggets, seg_len: int, tau: int, scale: float):
    """Attention under the segment form of the autoregressive objective (Sec. 2.4, Eq. 9 with a splitting index
    shared by the tokens of a segment), one query token at a time: token i of a text, in segment c = i // seg_len
    with t = max(0, c seg_len - tau), attends over the text's nuggets whose index is below t (rows of the packed,
    token-major Kn / Vn) and the text's own tokens t .. i (rows of K / V).  Returns (O, lse) in float64."""
    Q, Kn, Vn, K, V = _c(Q), _c(Kn), _c(Vn), _c(K), _c(V)
    assert Q.dtype == Kn.dtype == Vn.dtype == K.dtype == V.dtype and K.shape == V.shape and Kn.shape == Vn.shape
    nugget_idx, cu_seqlens, cu_nuggets = _c(nugget_idx, np.int32), _c(cu_seqlens, np.int32), _c(cu_nuggets, np.int32)
    N, H, d_h = Q.shape
    H_kv = K.shape[1]
    assert K.shape == (N, H_kv, d_h) and Kn.shape[1:] == (H_kv, d_h) and H % H_kv == 0
    O = np.zeros((N, H, d_h), dtype=np.float64)
    lse = np.zeros((N, H), dtype=np.float64)
    _load().oracle_attention_segment_mask(_p(Q), _p(Kn), _p(Vn), _p(K), _p(V), _p(nugget_idx), _p(cu_seqlens),
                                          _p(cu_nuggets), ctypes.c_int32(len(cu_seqlens) - 1), ctypes.c_int32(H),
                                          ctypes.c_int32(H_kv), ctypes.c_int32(d_h), ctypes.c_int32(seg_len),
                                          ctypes.c_int32(tau), ctypes.c_double(scale), _dtype_code(Q), _p(O), _p(lse))
    return O, lse


def ste_score_grad(Q, Kn, Vn, Kl, Vl, dO, cu_q, cu_nuggets, cu_local, scale: float, grad_scale: float):
    """Gradient that the straight-through estimator hands to the scores (Sec. 2.5, Eq. 17-18) for one layer:
    grad[i] = grad_scale * sum over heads h and query rows j of dl/dxi[j, i], where xi[j, i] is the input of the
    softmax for query row j and nugget i, and dl/dxi = P (dP - D) with P the attention weights of Eq. 13 / Eq. 9
    (over nuggets and the causally visible local rows), dP[j, i] = dO[j] . v_i and D[j] = dO[j] . O[j].
    Token-major nugget cache; returns float64 [Kt]."""
    Q, Kn, Vn, Kl, Vl, dO = _c(Q), _c(Kn), _c(Vn), _c(Kl), _c(Vl), _c(dO)
    assert Q.dtype == Kn.dtype == Vn.dtype == Kl.dtype == Vl.dtype == dO.dtype and dO.shape == Q.shape
    cu_q, cu_nuggets, cu_local = _c(cu_q, np.int32), _c(cu_nuggets, np.int32), _c(cu_local, np.int32)
    _, H, d_h = Q.shape
    H_kv = Kl.shape[1]
    Kt = Kn.shape[0]
    assert Kn.shape == Vn.shape == (Kt, H_kv, d_h) and Kt == int(cu_nuggets[-1])
    grad = np.zeros(Kt, dtype=np.float64)
    _load().oracle_ste_score_grad(_p(Q), _p(Kn), _p(Vn), _p(Kl), _p(Vl), _p(dO), _p(cu_q), _p(cu_nuggets), _p(cu_local),
                                  ctypes.c_int32(len(cu_q) - 1), ctypes.c_int32(H), ctypes.c_int32(H_kv),
                                  ctypes.c_int32(d_h), ctypes.c_double(scale), ctypes.c_double(grad_scale),
                                  _dtype_code(Q), ctypes.c_int64(Kt), _p(grad))
    return grad


def attention_rows(Q, Kn, Vn, Kl, Vl, cu_q, cu_nuggets, cu_local, scale: float, rows, layout: int = TOKEN_MAJOR):
    """Nugget attention for sampled (b, h, i) triples -> (O float64 [R,d_h], lse float64 [R])."""
    Q, Kn, Vn, Kl, Vl, cu_q, cu_nuggets, cu_local, H, H_kv, d_h, Kt = _attn_common(
        Q, Kn, Vn, Kl, Vl, cu_q, cu_nuggets, cu_local, layout)
    rows = np.asarray(rows, dtype=np.int32).reshape(-1, 3)
    rb, rh, ri = (np.ascontiguousarray(rows[:, j]) for j in range(3))
    R = len(rows)
    O = np.zeros((R, d_h), dtype=np.float64)
    lse = np.zeros(R, dtype=np.float64)
    _load().oracle_attention_rows(_p(Q), _p(Kn), _p(Vn), _p(Kl), _p(Vl), _p(cu_q), _p(cu_nuggets), _p(cu_local),
                                  ctypes.c_int32(H), ctypes.c_int32(H_kv), ctypes.c_int32(d_h),
                                  ctypes.c_double(scale), _dtype_code(Q), ctypes.c_int(layout), ctypes.c_int64(Kt),
                                  ctypes.c_int64(R), _p(rb), _p(rh), _p(ri), _p(O), _p(lse))
    return O, lse
