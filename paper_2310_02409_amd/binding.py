"""ctypes binding of libdodo.so: argument marshalling only."""
from __future__ import annotations

import ctypes
import math
import os
from typing import Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdodo.so")

F32, BF16 = 0, 1
RELU, GELU, TANH = 0, 1, 2
FORCE_LAST = 1
TOKEN_MAJOR, HEAD_MAJOR = 0, 1


class DodoError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where} failed: {status} ({dodo_status_string(status)})")


def _load(path: str = LIB_PATH) -> ctypes.CDLL:
    if not os.path.exists(path):
        raise ImportError(
            f"{path} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()'). "
            "There is no fallback path.")
    L = ctypes.CDLL(path)
    i32, i64, u32, vp, sz, f32 = (ctypes.c_int32, ctypes.c_int64, ctypes.c_uint32, ctypes.c_void_p, ctypes.c_size_t,
                                  ctypes.c_float)
    L.dodo_version.restype = ctypes.c_int
    L.dodo_version.argtypes = []
    L.dodo_status_string.restype = ctypes.c_char_p
    L.dodo_status_string.argtypes = [ctypes.c_int]
    L.dodo_nugget_count.restype = i64
    L.dodo_nugget_count.argtypes = [i64, i64, i64]
    L.dodo_score.restype = ctypes.c_int
    L.dodo_score.argtypes = [vp, vp, f32, ctypes.c_int, i64, i32, i64, vp, vp]
    L.dodo_score_layers.restype = ctypes.c_int
    L.dodo_score_layers.argtypes = [vp, vp, vp, ctypes.c_int, i32, i64, i32, i64, i64, i64, i64, vp, vp]
    L.dodo_select_topk_workspace_bytes.restype = sz
    L.dodo_select_topk_workspace_bytes.argtypes = [i32, i32]
    L.dodo_select_topk.restype = ctypes.c_int
    L.dodo_select_topk.argtypes = [vp, vp, vp, i32, i32, i32, u32, vp, vp, sz, vp]
    L.dodo_ste_score_grad_workspace_bytes.restype = sz
    L.dodo_ste_score_grad_workspace_bytes.argtypes = [i64, i32, i64]
    L.dodo_ste_score_grad.restype = ctypes.c_int
    L.dodo_ste_score_grad.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i64, i64, f32, f32,
                                      ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, vp, sz, vp]
    L.dodo_segment_plan.restype = ctypes.c_int
    L.dodo_segment_plan.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp]
    L.dodo_nugget_attention_segments.restype = ctypes.c_int
    L.dodo_nugget_attention_segments.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32,
                                                 i64, f32, ctypes.c_int, ctypes.c_int, vp, vp, vp, sz, vp]
    L.dodo_nugget_attention_indexed.restype = ctypes.c_int
    L.dodo_nugget_attention_indexed.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32,
                                                i32, i64, f32, ctypes.c_int, vp, vp, vp, sz, vp]
    L.dodo_gather_nuggets_layers.restype = ctypes.c_int
    L.dodo_gather_nuggets_layers.argtypes = [vp, vp, ctypes.c_int, vp, vp, vp, i32, i64, i32, i32, i32, i64, i64, i64, vp,
                                             vp, ctypes.c_int, vp]
    L.dodo_gather_nuggets.restype = ctypes.c_int
    L.dodo_gather_nuggets.argtypes = [vp, vp, ctypes.c_int, vp, vp, vp, i32, i64, i32, i32, i64, vp, vp, ctypes.c_int,
                                      vp]
    L.dodo_nugget_attention_workspace_bytes.restype = sz
    L.dodo_nugget_attention_workspace_bytes.argtypes = [i32, i32, i32, i32, i32, i32, ctypes.c_int]
    L.dodo_nugget_attention_workspace_bytes_grouped.restype = sz
    L.dodo_nugget_attention_workspace_bytes_grouped.argtypes = [i32, i32, i32, i32, i32, i32, i32, ctypes.c_int]
    L.dodo_nugget_attention.restype = ctypes.c_int
    L.dodo_nugget_attention.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, i64, f32,
                                        ctypes.c_int, ctypes.c_int, vp, vp, vp, sz, vp]
    L.dodo_nugget_attention_noalloc.restype = ctypes.c_int
    L.dodo_nugget_attention_noalloc.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, i64, f32,
                                                ctypes.c_int, ctypes.c_int, vp, vp, vp]
    L.dodo_probe_read.restype = ctypes.c_int
    L.dodo_probe_read.argtypes = [vp, sz, vp, vp]
    L.dodo_probe_copy.restype = ctypes.c_int
    L.dodo_probe_copy.argtypes = [vp, vp, sz, vp]
    L.dodo_score_mlp_workspace_bytes.restype = sz
    L.dodo_score_mlp_workspace_bytes.argtypes = [ctypes.c_int, i64, i32, i32]
    L.dodo_score_mlp.restype = ctypes.c_int
    L.dodo_score_mlp.argtypes = [vp, vp, vp, vp, f32, ctypes.c_int, ctypes.c_int, i64, i32, i32, i64, vp, vp, sz, vp]
    L.dodo_meanpool_nuggets.restype = ctypes.c_int
    L.dodo_meanpool_nuggets.argtypes = [vp, vp, ctypes.c_int, vp, vp, i32, i64, i32, i32, i64, vp, vp, ctypes.c_int, vp]
    L.dodo_nugget_attention_cached.restype = ctypes.c_int
    L.dodo_nugget_attention_cached.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32,
                                               i64, f32, ctypes.c_int, ctypes.c_int, vp, vp, vp, sz, vp]
    L.dodo_threshold_from_sample.restype = ctypes.c_int
    L.dodo_threshold_from_sample.argtypes = [vp, i64, i64, i64, vp, vp, sz, vp]
    L.dodo_threshold_from_sample_workspace_bytes.restype = sz
    L.dodo_threshold_from_sample_workspace_bytes.argtypes = [i64]
    L.dodo_select_threshold.restype = ctypes.c_int
    L.dodo_select_threshold.argtypes = [vp, vp, i32, vp, vp, vp, vp, vp]
    L.dodo_stream_append.restype = ctypes.c_int
    L.dodo_stream_append.argtypes = [vp, vp, vp, vp, ctypes.c_int, i32, i32, i32, i64, i32, vp, vp, vp, vp, vp]
    return L


lib = _load()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"dodo takes float32 or bfloat16 tensors, got {t.dtype}")


def _ptr(t: Optional[torch.Tensor]) -> int:
    return 0 if t is None else t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _check(rc: int, where: str) -> None:
    if rc != 0:
        raise DodoError(rc, where)


def _dev(*ts: Optional[torch.Tensor]) -> None:
    for t in ts:
        if t is not None and (not t.is_cuda or not t.is_contiguous()):
            raise ValueError("dodo tensors must be contiguous device tensors")


def _dev_rows(*ts: torch.Tensor) -> None:
    """Device tensors whose rows (all dimensions but the first) are contiguous; the first dimension may be strided."""
    for t in ts:
        inner = 1
        for size, stride in zip(reversed(t.shape[1:]), reversed(t.stride()[1:])):
            if size != 1 and stride != inner:
                raise ValueError("dodo tensors must have contiguous rows")
            inner *= size
        if not t.is_cuda or (t.shape[0] > 1 and t.stride(0) < inner):
            raise ValueError("dodo tensors must be device tensors with a row stride of at least a row")


def dodo_version() -> int:
    return int(lib.dodo_version())


def dodo_status_string(status: int) -> str:
    return lib.dodo_status_string(int(status)).decode()


def dodo_nugget_count(n: int, num: int, den: int) -> int:
    return int(lib.dodo_nugget_count(int(n), int(num), int(den)))


def cu_nuggets_from_lengths(seq_lens: Sequence[int], num: int, den: int, device) -> Tuple[torch.Tensor, list]:
    """Host-side prefix sums of dodo_nugget_count over the batch, uploaded as int32."""
    ks = [dodo_nugget_count(n, num, den) for n in seq_lens]
    cu = [0]
    for k in ks:
        cu.append(cu[-1] + k)
    return torch.tensor(cu, dtype=torch.int32, device=device), ks


def dodo_score(hidden: torch.Tensor, w: torch.Tensor, bias: float = 0.0,
               scores: Optional[torch.Tensor] = None) -> torch.Tensor:
    """scores[t] = hidden[t] . w + bias (fp32 [N]) for packed hidden [N, d]."""
    _dev(w, scores)
    _dev_rows(hidden)
    N, d = hidden.shape
    assert w.shape == (d,) and w.dtype == hidden.dtype
    if scores is None:
        scores = torch.empty(N, dtype=torch.float32, device=hidden.device)
    assert scores.dtype == torch.float32 and scores.numel() == N
    _check(lib.dodo_score(_ptr(hidden), _ptr(w), float(bias), _dtype_code(hidden), N, d, hidden.stride(0),
                          _ptr(scores), _stream()), "dodo_score")
    return scores


def dodo_score_layers(hidden: torch.Tensor, w: torch.Tensor, biases: Optional[torch.Tensor] = None,
                      scores: Optional[torch.Tensor] = None) -> torch.Tensor:
    """scores[l, t] = hidden[l, t] . w[l] + biases[l] (fp32 [L, N]) for hidden [L, N, d], w [L, d], in one launch."""
    _dev(w, biases)
    if not hidden.is_cuda or hidden.stride(2) != 1 or (scores is not None and not scores.is_cuda):
        raise ValueError("hidden must be a device tensor [L, N, d] with unit stride along d")
    L, N, d = hidden.shape
    assert w.shape == (L, d) and w.dtype == hidden.dtype
    if scores is None:
        scores = torch.empty((L, N), dtype=torch.float32, device=hidden.device)
    assert scores.dtype == torch.float32 and scores.shape == (L, N) and scores.stride(1) == 1
    assert biases is None or (biases.dtype == torch.float32 and biases.numel() == L)
    _check(lib.dodo_score_layers(_ptr(hidden), _ptr(w), _ptr(biases), _dtype_code(hidden), L, N, d, hidden.stride(1),
                                 hidden.stride(0), w.stride(0), scores.stride(0), _ptr(scores), _stream()),
           "dodo_score_layers")
    return scores


def dodo_select_topk_workspace_bytes(B: int, max_n: int) -> int:
    return int(lib.dodo_select_topk_workspace_bytes(B, max_n))


def dodo_select_topk(scores: torch.Tensor, cu_seqlens: torch.Tensor, cu_nuggets: torch.Tensor, max_n: int, max_k: int,
                     total_nuggets: int, flags: int = 0, nugget_idx: Optional[torch.Tensor] = None,
                     ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Sequence-local, ascending indices of each sequence's top-k scores, packed by cu_nuggets (int32 [Kt])."""
    _dev(scores, cu_seqlens, cu_nuggets, nugget_idx, ws)
    assert scores.dtype == torch.float32 and cu_seqlens.dtype == torch.int32 and cu_nuggets.dtype == torch.int32
    B = cu_seqlens.numel() - 1
    assert cu_nuggets.numel() == B + 1
    if nugget_idx is None:
        nugget_idx = torch.empty(total_nuggets, dtype=torch.int32, device=scores.device)
    assert nugget_idx.dtype == torch.int32 and nugget_idx.numel() >= total_nuggets
    need = dodo_select_topk_workspace_bytes(B, max_n)
    if need and ws is None:
        # zero-filled, as the library requires before the first use (a call leaves it zero-filled)
        ws = torch.zeros(need, dtype=torch.uint8, device=scores.device)
    _check(lib.dodo_select_topk(_ptr(scores), _ptr(cu_seqlens), _ptr(cu_nuggets), B, max_n, max_k, flags,
                                _ptr(nugget_idx), _ptr(ws), 0 if ws is None else ws.numel(), _stream()),
           "dodo_select_topk")
    return nugget_idx


def dodo_gather_nuggets(K: torch.Tensor, V: torch.Tensor, nugget_idx: torch.Tensor, cu_seqlens: torch.Tensor,
                        cu_nuggets: torch.Tensor, total_nuggets: int, layout: int = TOKEN_MAJOR,
                        Kn: Optional[torch.Tensor] = None, Vn: Optional[torch.Tensor] = None):
    """Packs the chosen rows of K, V [N, H_kv, d_h] into the nugget cache."""
    _dev(nugget_idx, cu_seqlens, cu_nuggets, Kn, Vn)
    _dev_rows(K, V)
    _, H_kv, d_h = K.shape
    assert V.shape == K.shape and V.dtype == K.dtype and V.stride() == K.stride()
    B = cu_seqlens.numel() - 1
    shape = (total_nuggets, H_kv, d_h) if layout == TOKEN_MAJOR else (H_kv, total_nuggets, d_h)
    if Kn is None:
        Kn = torch.empty(shape, dtype=K.dtype, device=K.device)
    if Vn is None:
        Vn = torch.empty(shape, dtype=K.dtype, device=K.device)
    assert tuple(Kn.shape) == shape and tuple(Vn.shape) == shape
    _check(lib.dodo_gather_nuggets(_ptr(K), _ptr(V), _dtype_code(K), _ptr(nugget_idx), _ptr(cu_seqlens),
                                   _ptr(cu_nuggets), B, total_nuggets, H_kv, d_h, K.stride(0), _ptr(Kn), _ptr(Vn),
                                   layout, _stream()), "dodo_gather_nuggets")
    return Kn, Vn


def dodo_gather_nuggets_layers(K: torch.Tensor, V: torch.Tensor, nugget_idx: torch.Tensor, cu_seqlens: torch.Tensor,
                               cu_nuggets: torch.Tensor, total_nuggets: int, layout: int = TOKEN_MAJOR,
                               Kn: Optional[torch.Tensor] = None, Vn: Optional[torch.Tensor] = None):
    """Packs the chosen rows of K, V [L, N, H_kv, d_h] of all L layers (one shared index list) in one launch."""
    _dev(nugget_idx, cu_seqlens, cu_nuggets)
    if not (K.is_cuda and V.is_cuda):
        raise ValueError("dodo tensors must be device tensors")
    L, _, H_kv, d_h = K.shape
    assert V.shape == K.shape and V.dtype == K.dtype and K.stride() == V.stride()
    assert K.stride(3) == 1 and K.stride(2) == d_h
    B = cu_seqlens.numel() - 1
    shape = (L, total_nuggets, H_kv, d_h) if layout == TOKEN_MAJOR else (L, H_kv, total_nuggets, d_h)
    if Kn is None:
        Kn = torch.empty(shape, dtype=K.dtype, device=K.device)
    if Vn is None:
        Vn = torch.empty(shape, dtype=K.dtype, device=K.device)
    assert tuple(Kn.shape) == shape and tuple(Vn.shape) == shape and Kn.stride() == Vn.stride()
    assert Kn[0].is_contiguous() and Vn[0].is_contiguous()
    _check(lib.dodo_gather_nuggets_layers(_ptr(K), _ptr(V), _dtype_code(K), _ptr(nugget_idx), _ptr(cu_seqlens),
                                          _ptr(cu_nuggets), B, total_nuggets, L, H_kv, d_h, K.stride(1), K.stride(0),
                                          Kn.stride(0), _ptr(Kn), _ptr(Vn), layout, _stream()),
           "dodo_gather_nuggets_layers")
    return Kn, Vn


def dodo_nugget_attention_workspace_bytes(B: int, H: int, d_h: int, max_q: int, max_k: int, max_local: int,
                                          dtype: int) -> int:
    return int(lib.dodo_nugget_attention_workspace_bytes(B, H, d_h, max_q, max_k, max_local, dtype))


def dodo_nugget_attention_workspace_bytes_grouped(B: int, H: int, H_kv: int, d_h: int, max_q: int, max_k: int,
                                                  max_local: int, dtype: int) -> int:
    return int(lib.dodo_nugget_attention_workspace_bytes_grouped(B, H, H_kv, d_h, max_q, max_k, max_local, dtype))


def dodo_nugget_attention(Q: torch.Tensor, Kn: torch.Tensor, Vn: torch.Tensor, Kl: torch.Tensor, Vl: torch.Tensor,
                          cu_q: torch.Tensor, cu_nuggets: torch.Tensor, cu_local: torch.Tensor, max_q: int,
                          max_k: int, max_local: int, softmax_scale: Optional[float] = None,
                          layout: int = TOKEN_MAJOR, O: Optional[torch.Tensor] = None,
                          lse: Optional[torch.Tensor] = None, want_lse: bool = False,
                          ws: Optional[torch.Tensor] = None):
    """Attention of Q [Sq, H, d_h] over [nuggets ; causally visible local rows]; returns (O, lse or None)."""
    _dev(Q, Kn, Vn, Kl, Vl, cu_q, cu_nuggets, cu_local, O, lse, ws)
    Sq, H, d_h = Q.shape
    H_kv = Kl.shape[1]
    Kt = Kn.shape[0] if layout == TOKEN_MAJOR else Kn.shape[1]
    B = cu_q.numel() - 1
    if softmax_scale is None:
        softmax_scale = 1.0 / math.sqrt(d_h)
    if O is None:
        O = torch.empty_like(Q)
    if lse is None and want_lse:
        lse = torch.empty((Sq, H), dtype=torch.float32, device=Q.device)
    code = _dtype_code(Q)
    need = dodo_nugget_attention_workspace_bytes_grouped(B, H, H_kv, d_h, max_q, max_k, max_local, code)
    if need and ws is None:
        # zero-filled: the split-K flags must not hold the library's "ready" value on entry
        ws = torch.zeros(need, dtype=torch.uint8, device=Q.device)
    _check(lib.dodo_nugget_attention(_ptr(Q), _ptr(Kn), _ptr(Vn), _ptr(Kl), _ptr(Vl), _ptr(cu_q), _ptr(cu_nuggets),
                                     _ptr(cu_local), B, H, H_kv, d_h, max_q, max_k, max_local, Kt,
                                     float(softmax_scale), code, layout, _ptr(O), _ptr(lse), _ptr(ws),
                                     0 if ws is None else ws.numel(), _stream()), "dodo_nugget_attention")
    return O, lse


def dodo_nugget_attention_noalloc(Q: torch.Tensor, Kn: torch.Tensor, Vn: torch.Tensor, Kl: torch.Tensor,
                                  Vl: torch.Tensor, cu_q: torch.Tensor, cu_nuggets: torch.Tensor,
                                  cu_local: torch.Tensor, max_q: int, max_k: int, max_local: int, softmax_scale: float,
                                  layout: int, O: torch.Tensor, lse: Optional[torch.Tensor] = None) -> None:
    """dodo_nugget_attention into the caller's O (and lse) with the library's own static scratch buffer:
    neither this wrapper nor the call allocates anything."""
    _dev(Q, Kn, Vn, Kl, Vl, cu_q, cu_nuggets, cu_local, O, lse)
    Sq, H, d_h = Q.shape
    _check(lib.dodo_nugget_attention_noalloc(_ptr(Q), _ptr(Kn), _ptr(Vn), _ptr(Kl), _ptr(Vl), _ptr(cu_q),
                                             _ptr(cu_nuggets), _ptr(cu_local), cu_q.numel() - 1, H, Kl.shape[1], d_h,
                                             max_q, max_k, max_local,
                                             Kn.shape[0] if layout == TOKEN_MAJOR else Kn.shape[1],
                                             float(softmax_scale), _dtype_code(Q), layout, _ptr(O), _ptr(lse),
                                             _stream()), "dodo_nugget_attention_noalloc")


def dodo_nugget_attention_indexed(Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, nugget_idx: torch.Tensor,
                                  cu_seqlens: torch.Tensor, Kl: torch.Tensor, Vl: torch.Tensor, cu_q: torch.Tensor,
                                  cu_nuggets: torch.Tensor, cu_local: torch.Tensor, max_q: int, max_k: int,
                                  max_local: int, max_n: int, softmax_scale: Optional[float] = None,
                                  O: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None,
                                  want_lse: bool = False, ws: Optional[torch.Tensor] = None):
    """dodo_nugget_attention with the nuggets read in place from the context's K, V [N, H_kv, d_h] through
    the index list (no packed cache); returns (O, lse or None)."""
    _dev(Q, nugget_idx, cu_seqlens, Kl, Vl, cu_q, cu_nuggets, cu_local, O, lse, ws)
    if not (K.is_cuda and V.is_cuda) or K.stride() != V.stride() or K.stride(2) != 1 or K.stride(1) != K.shape[2]:
        raise ValueError("K, V must be device tensors [N, H_kv, d_h] with contiguous rows and equal strides")
    Sq, H, d_h = Q.shape
    H_kv = K.shape[1]
    B = cu_q.numel() - 1
    if softmax_scale is None:
        softmax_scale = 1.0 / math.sqrt(d_h)
    if O is None:
        O = torch.empty_like(Q)
    if lse is None and want_lse:
        lse = torch.empty((Sq, H), dtype=torch.float32, device=Q.device)
    code = _dtype_code(Q)
    need = dodo_nugget_attention_workspace_bytes(B, H, d_h, max_q, max_k, max_local, code)
    if need and ws is None:
        ws = torch.zeros(need, dtype=torch.uint8, device=Q.device)
    _check(lib.dodo_nugget_attention_indexed(_ptr(Q), _ptr(K), _ptr(V), _ptr(nugget_idx), _ptr(cu_seqlens), _ptr(Kl),
                                             _ptr(Vl), _ptr(cu_q), _ptr(cu_nuggets), _ptr(cu_local), B, H, H_kv, d_h,
                                             max_q, max_k, max_local, max_n, K.stride(0), float(softmax_scale), code,
                                             _ptr(O), _ptr(lse), _ptr(ws), 0 if ws is None else ws.numel(), _stream()),
           "dodo_nugget_attention_indexed")
    return O, lse


def dodo_ste_score_grad_workspace_bytes(Sq: int, H: int, Kt: int) -> int:
    return int(lib.dodo_ste_score_grad_workspace_bytes(Sq, H, Kt))


def dodo_ste_score_grad(Q: torch.Tensor, Kn: torch.Tensor, Vn: torch.Tensor, dO: torch.Tensor, O: torch.Tensor,
                        lse: torch.Tensor, cu_q: torch.Tensor, cu_nuggets: torch.Tensor, max_q: int, max_k: int,
                        softmax_scale: Optional[float] = None, grad_scale: Optional[float] = None,
                        layout: int = TOKEN_MAJOR, grad: Optional[torch.Tensor] = None, accumulate: bool = False,
                        ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Score gradient of the straight-through estimator (Eq. 17-18) for one layer; returns fp32 [Kt]."""
    _dev(Q, Kn, Vn, dO, O, lse, cu_q, cu_nuggets, grad, ws)
    Sq, H, d_h = Q.shape
    H_kv = Kn.shape[1] if layout == TOKEN_MAJOR else Kn.shape[0]
    Kt = Kn.shape[0] if layout == TOKEN_MAJOR else Kn.shape[1]
    B = cu_q.numel() - 1
    assert dO.shape == Q.shape and O.shape == Q.shape and lse.shape == (Sq, H) and lse.dtype == torch.float32
    assert dO.dtype == Q.dtype == O.dtype == Kn.dtype == Vn.dtype
    if softmax_scale is None:
        softmax_scale = 1.0 / math.sqrt(d_h)
    if grad_scale is None:
        grad_scale = softmax_scale
    if grad is None:
        assert not accumulate
        grad = torch.empty(Kt, dtype=torch.float32, device=Q.device)
    need = dodo_ste_score_grad_workspace_bytes(Sq, H, Kt)
    if need and ws is None:
        ws = torch.empty(need, dtype=torch.uint8, device=Q.device)
    _check(lib.dodo_ste_score_grad(_ptr(Q), _ptr(Kn), _ptr(Vn), _ptr(dO), _ptr(O), _ptr(lse), _ptr(cu_q),
                                   _ptr(cu_nuggets), B, H, H_kv, d_h, max_q, max_k, Sq, Kt, float(softmax_scale),
                                   float(grad_scale), int(bool(accumulate)), _dtype_code(Q), layout, _ptr(grad), _ptr(ws),
                                   0 if ws is None else ws.numel(), _stream()), "dodo_ste_score_grad")
    return grad


def dodo_segment_plan(nugget_idx: torch.Tensor, cu_seqlens: torch.Tensor, cu_nuggets: torch.Tensor, seg_len: int,
                      tau: int, capacity: int):
    """Entries of the segment form of the autoregressive objective (Sec. 2.4): returns the device int32 arrays
    (seg_cu_q [capacity+1], seg_nug_start, seg_nug_len, seg_loc_start, seg_loc_len [capacity], n_segments [1])."""
    _dev(nugget_idx, cu_seqlens, cu_nuggets)
    B = cu_seqlens.numel() - 1
    mk = lambda n: torch.empty(n, dtype=torch.int32, device=cu_seqlens.device)
    seg_cu_q, ns, nl, ls, ll, cnt = mk(capacity + 1), mk(capacity), mk(capacity), mk(capacity), mk(capacity), mk(1)
    _check(lib.dodo_segment_plan(_ptr(nugget_idx), _ptr(cu_seqlens), _ptr(cu_nuggets), B, seg_len, tau, capacity,
                                 _ptr(seg_cu_q), _ptr(ns), _ptr(nl), _ptr(ls), _ptr(ll), _ptr(cnt), _stream()),
           "dodo_segment_plan")
    return seg_cu_q, ns, nl, ls, ll, cnt


def dodo_nugget_attention_segments(Q: torch.Tensor, Kn: torch.Tensor, Vn: torch.Tensor, K: torch.Tensor,
                                   V: torch.Tensor, seg_cu_q: torch.Tensor, seg_nug_start: torch.Tensor,
                                   seg_nug_len: torch.Tensor, seg_loc_start: torch.Tensor, seg_loc_len: torch.Tensor,
                                   max_q: int, max_k: int, max_local: int, softmax_scale: Optional[float] = None,
                                   layout: int = TOKEN_MAJOR, O: Optional[torch.Tensor] = None,
                                   lse: Optional[torch.Tensor] = None, want_lse: bool = False,
                                   ws: Optional[torch.Tensor] = None):
    """dodo_nugget_attention over (start, length) ranges of the nugget cache and of the texts' own K, V
    [N, H_kv, d_h], one entry per segment; returns (O, lse or None)."""
    _dev(Q, Kn, Vn, K, V, seg_cu_q, seg_nug_start, seg_nug_len, seg_loc_start, seg_loc_len, O, lse, ws)
    Sq, H, d_h = Q.shape
    H_kv = K.shape[1]
    Kt = Kn.shape[0] if layout == TOKEN_MAJOR else Kn.shape[1]
    n_seg = seg_cu_q.numel() - 1
    if softmax_scale is None:
        softmax_scale = 1.0 / math.sqrt(d_h)
    if O is None:
        O = torch.empty_like(Q)
    if lse is None and want_lse:
        lse = torch.empty((Sq, H), dtype=torch.float32, device=Q.device)
    code = _dtype_code(Q)
    need = dodo_nugget_attention_workspace_bytes_grouped(n_seg, H, H_kv, d_h, max_q, max_k, max_local, code)
    if need and ws is None:
        ws = torch.zeros(need, dtype=torch.uint8, device=Q.device)
    _check(lib.dodo_nugget_attention_segments(_ptr(Q), _ptr(Kn), _ptr(Vn), _ptr(K), _ptr(V), _ptr(seg_cu_q),
                                              _ptr(seg_nug_start), _ptr(seg_nug_len), _ptr(seg_loc_start),
                                              _ptr(seg_loc_len), n_seg, H, H_kv, d_h, max_q, max_k, max_local, Kt,
                                              float(softmax_scale), code, layout, _ptr(O), _ptr(lse), _ptr(ws),
                                              0 if ws is None else ws.numel(), _stream()),
           "dodo_nugget_attention_segments")
    return O, lse


def dodo_nugget_attention_cached(Q: torch.Tensor, Kn: torch.Tensor, Vn: torch.Tensor, Kl: torch.Tensor,
                                 Vl: torch.Tensor, cu_q: torch.Tensor, nugget_start: torch.Tensor,
                                 nugget_len: torch.Tensor, cu_local: torch.Tensor, max_q: int, max_k: int,
                                 max_local: int, softmax_scale: Optional[float] = None, layout: int = TOKEN_MAJOR,
                                 O: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None,
                                 want_lse: bool = False, ws: Optional[torch.Tensor] = None):
    """dodo_nugget_attention over caches with room to grow: nuggets of sequence b are the rows
    nugget_start[b] .. + nugget_len[b] of Kn / Vn [rows, H_kv, d_h]; returns (O, lse or None)."""
    _dev(Q, Kn, Vn, Kl, Vl, cu_q, nugget_start, nugget_len, cu_local, O, lse, ws)
    Sq, H, d_h = Q.shape
    H_kv = Kl.shape[1]
    Kt = Kn.shape[0] if layout == TOKEN_MAJOR else Kn.shape[1]
    B = cu_q.numel() - 1
    if softmax_scale is None:
        softmax_scale = 1.0 / math.sqrt(d_h)
    if O is None:
        O = torch.empty_like(Q)
    if lse is None and want_lse:
        lse = torch.empty((Sq, H), dtype=torch.float32, device=Q.device)
    code = _dtype_code(Q)
    need = dodo_nugget_attention_workspace_bytes_grouped(B, H, H_kv, d_h, max_q, max_k, max_local, code)
    if need and ws is None:
        ws = torch.zeros(need, dtype=torch.uint8, device=Q.device)
    _check(lib.dodo_nugget_attention_cached(_ptr(Q), _ptr(Kn), _ptr(Vn), _ptr(Kl), _ptr(Vl), _ptr(cu_q),
                                            _ptr(nugget_start), _ptr(nugget_len), _ptr(cu_local), B, H, H_kv, d_h,
                                            max_q, max_k, max_local, Kt, float(softmax_scale), code, layout, _ptr(O),
                                            _ptr(lse), _ptr(ws), 0 if ws is None else ws.numel(), _stream()),
           "dodo_nugget_attention_cached")
    return O, lse


def dodo_threshold_from_sample_workspace_bytes(n: int) -> int:
    return int(lib.dodo_threshold_from_sample_workspace_bytes(n))


def dodo_threshold_from_sample(sample: torch.Tensor, num: int, den: int, out: Optional[torch.Tensor] = None,
                               ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Threshold Lambda (device tensor with one fp32) from sampled scores: the (k+1)-th highest, k = nugget count."""
    _dev(sample, out, ws)
    assert sample.dtype == torch.float32 and sample.is_contiguous()
    if out is None:
        out = torch.empty(1, dtype=torch.float32, device=sample.device)
    need = dodo_threshold_from_sample_workspace_bytes(sample.numel())
    if need and ws is None:
        ws = torch.empty(need, dtype=torch.uint8, device=sample.device)
    _check(lib.dodo_threshold_from_sample(_ptr(sample), sample.numel(), num, den, _ptr(out), _ptr(ws),
                                          0 if ws is None else ws.numel(), _stream()), "dodo_threshold_from_sample")
    return out


def dodo_select_threshold(scores: torch.Tensor, cu_seqlens: torch.Tensor, lam: torch.Tensor):
    """Threshold selection (Eq. 8): returns (counts [B], cu_nuggets [B+1], nugget_idx with room for all tokens),
    all on the device; the first cu_nuggets[B] entries of nugget_idx are the packed index lists."""
    _dev(scores, cu_seqlens, lam)
    assert scores.dtype == torch.float32 and lam.dtype == torch.float32
    B = cu_seqlens.numel() - 1
    counts = torch.empty(B, dtype=torch.int32, device=scores.device)
    cu_nuggets = torch.empty(B + 1, dtype=torch.int32, device=scores.device)
    idx = torch.empty(max(1, scores.numel()), dtype=torch.int32, device=scores.device)
    _check(lib.dodo_select_threshold(_ptr(scores), _ptr(cu_seqlens), B, _ptr(lam), _ptr(counts), _ptr(cu_nuggets),
                                     _ptr(idx), _stream()), "dodo_select_threshold")
    return counts, cu_nuggets, idx


def dodo_stream_append(scores: torch.Tensor, lam: torch.Tensor, K_rows: torch.Tensor, V_rows: torch.Tensor,
                       counts: torch.Tensor, Kn: torch.Tensor, Vn: torch.Tensor,
                       dropped: Optional[torch.Tensor] = None) -> None:
    """One decode step: rows [B, H_kv, d_h] whose score exceeds Lambda are appended to the caches
    [B, cap, H_kv, d_h] (in place), counts [B] int32 is updated in place."""
    _dev(scores, lam, K_rows, V_rows, counts, Kn, Vn, dropped)
    B, H_kv, d_h = K_rows.shape
    cap = Kn.shape[1]
    assert Kn.shape == (B, cap, H_kv, d_h) and Kn.is_contiguous() and Vn.is_contiguous()
    assert K_rows.stride(2) == 1 and K_rows.stride(1) == d_h and V_rows.stride() == K_rows.stride()
    _check(lib.dodo_stream_append(_ptr(scores), _ptr(lam), _ptr(K_rows), _ptr(V_rows), _dtype_code(K_rows), B, H_kv,
                                  d_h, K_rows.stride(0), cap, _ptr(counts), _ptr(dropped), _ptr(Kn), _ptr(Vn),
                                  _stream()), "dodo_stream_append")


def dodo_meanpool_nuggets(K: torch.Tensor, V: torch.Tensor, cu_seqlens: torch.Tensor, cu_nuggets: torch.Tensor,
                          Kt: int, layout: int = TOKEN_MAJOR, Kn: Optional[torch.Tensor] = None,
                          Vn: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Pooling baseline's compaction: K, V [N, H_kv, d_h] -> mean-pooled caches of Kt rows."""
    _dev(K, V, cu_seqlens, cu_nuggets, Kn, Vn)
    N, H_kv, d_h = K.shape
    shape = (Kt, H_kv, d_h) if layout == TOKEN_MAJOR else (H_kv, Kt, d_h)
    if Kn is None:
        Kn = torch.empty(shape, dtype=K.dtype, device=K.device)
    if Vn is None:
        Vn = torch.empty(shape, dtype=K.dtype, device=K.device)
    B = cu_seqlens.numel() - 1
    _check(lib.dodo_meanpool_nuggets(_ptr(K), _ptr(V), _dtype_code(K), _ptr(cu_seqlens), _ptr(cu_nuggets), B, Kt, H_kv,
                                     d_h, H_kv * d_h, _ptr(Kn), _ptr(Vn), layout, _stream()), "dodo_meanpool_nuggets")
    return Kn, Vn


def dodo_score_mlp_workspace_bytes(dtype: int, N: int, d: int, d_hid: int) -> int:
    return int(lib.dodo_score_mlp_workspace_bytes(dtype, N, d, d_hid))


def dodo_score_mlp(hidden: torch.Tensor, W1: torch.Tensor, b1: torch.Tensor, w2: torch.Tensor, b2: float = 0.0,
                   act: int = RELU, out: Optional[torch.Tensor] = None,
                   ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """2-layer scorer (App. B): s = w2 . act(W1 x + b1) + b2 with W1 [d_hid, d]; returns fp32 scores [N]."""
    _dev(W1, b1, w2, out, ws)
    if not hidden.is_cuda or hidden.stride(1) != 1:
        raise ValueError("hidden must be a device tensor with unit stride along d")
    N, d = hidden.shape
    d_hid = W1.shape[0]
    assert W1.shape == (d_hid, d) and b1.shape == (d_hid,) and w2.shape == (d_hid,) and b1.dtype == torch.float32
    assert W1.dtype == hidden.dtype == w2.dtype
    if out is None:
        out = torch.empty(N, dtype=torch.float32, device=hidden.device)
    code = _dtype_code(hidden)
    need = dodo_score_mlp_workspace_bytes(code, N, d, d_hid)
    if need and ws is None:
        ws = torch.empty(need, dtype=torch.uint8, device=hidden.device)
    _check(lib.dodo_score_mlp(_ptr(hidden), _ptr(W1), _ptr(b1), _ptr(w2), float(b2), act, code, N, d, d_hid,
                              hidden.stride(0), _ptr(out), _ptr(ws), 0 if ws is None else ws.numel(), _stream()),
           "dodo_score_mlp")
    return out


def dodo_probe_read(src: torch.Tensor, sink: torch.Tensor) -> None:
    """Measurement aid: a read-only pass over src (sink: one int32 device word)."""
    _dev(src, sink)
    _check(lib.dodo_probe_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink), _stream()), "dodo_probe_read")


def dodo_probe_copy(src: torch.Tensor, dst: torch.Tensor) -> None:
    """Measurement aid: a plain copy of src into dst."""
    _dev(src, dst)
    assert src.numel() * src.element_size() == dst.numel() * dst.element_size()
    _check(lib.dodo_probe_copy(_ptr(src), _ptr(dst), src.numel() * src.element_size(), _stream()), "dodo_probe_copy")
