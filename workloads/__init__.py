"""Seeded synthetic inputs for the Dodo hot path (shared by tests, smoke and bench).

This module only draws numbers and lays them out; it holds none of the
method's arithmetic (no scorer, no selection, no counts, no attention) and
imports neither the HIP binding nor the oracle.  Both sides consume the bits
produced here.

Every tensor is a pure function of (seed, tensor_id, element index): a
SplitMix64-style counter hash gives two uniforms per element, Box-Muller in
float64 turns them into a standard normal, which is scaled and rounded to the
storage type.  The generator runs on whatever torch device is asked for; a test
generates once and copies the same bits to the other side.

The five named workloads mirror the shapes the paper runs the method on
(LLaMA-7B/13B attention shapes, 10x / 20x compression, a few hundred to a few
thousand context tokens, Sec. 3-6) with Gaussian stand-ins for hidden states
and projected Q/K/V; no dataset text or trained weight is involved.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional

import torch

_MASK64 = (1 << 64) - 1


def _s64(v: int) -> int:
    """Python int (mod 2^64) -> the signed value torch.int64 stores."""
    v &= _MASK64
    return v - (1 << 64) if v >= (1 << 63) else v


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift on int64 tensors."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix(x: torch.Tensor) -> torch.Tensor:
    x = (x ^ _lsr(x, 30)) * _s64(0xBF58476D1CE4E5B9)
    x = (x ^ _lsr(x, 27)) * _s64(0x94D049BB133111EB)
    return x ^ _lsr(x, 31)


def _mix_int(v: int) -> int:
    v &= _MASK64
    v = ((v ^ (v >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    v = ((v ^ (v >> 27)) * 0x94D049BB133111EB) & _MASK64
    return v ^ (v >> 31)


def _stream_key(seed: int, tensor_id: int) -> int:
    return _mix_int(_mix_int(seed) ^ (0x9E3779B97F4A7C15 * (tensor_id + 1)))


def uniform_bits(seed: int, tensor_id: int, start: int, count: int, device) -> torch.Tensor:
    """int64 tensor of `count` hashed 64-bit words for element indices start..start+count."""
    key = _stream_key(seed, tensor_id)
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    return _mix(idx * _s64(0x9E3779B97F4A7C15) + _s64(key))


def normal(seed: int, tensor_id: int, shape, std: float, dtype: torch.dtype, device="cpu",
           chunk: int = 1 << 23) -> torch.Tensor:
    """N(0, std^2) tensor of `shape`, reproducible element by element."""
    numel = int(math.prod(shape))
    out = torch.empty(numel, dtype=dtype, device=device)
    for start in range(0, numel, chunk):
        cnt = min(chunk, numel - start)
        h1 = uniform_bits(seed, 2 * tensor_id, start, cnt, device)
        h2 = uniform_bits(seed, 2 * tensor_id + 1, start, cnt, device)
        u1 = (_lsr(h1, 11).to(torch.float64) + 1.0) * (2.0 ** -53)  # (0, 1]
        u2 = _lsr(h2, 11).to(torch.float64) * (2.0 ** -53)  # [0, 1)
        z = torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)
        out[start:start + cnt] = (z * std).to(dtype)
    return out.reshape(shape)


def integers(seed: int, tensor_id: int, shape, lo: int, hi: int, device="cpu") -> torch.Tensor:
    """Uniform integers in [lo, hi] as int64."""
    numel = int(math.prod(shape))
    h = uniform_bits(seed, tensor_id, 0, numel, device)
    return (_lsr(h, 16) % (hi - lo + 1) + lo).reshape(shape)


@dataclasses.dataclass
class Workload:
    name: str
    dtype: torch.dtype
    seq_lens: List[int]  # context tokens n_b per sequence
    d_model: int
    H: int
    H_kv: int
    d_h: int
    keep_num: int  # keep-fraction num/den (10x compression -> 1/10)
    keep_den: int
    q_lens: List[int]  # query rows per sequence
    tau: List[int]  # uncompressed local tokens preceding the query block
    layers: int = 1
    seed: int = 0xD0D00000
    quantise_scores: bool = False  # the 16-level tie stress of the long-context case

    @property
    def B(self) -> int:
        return len(self.seq_lens)

    @property
    def local_lens(self) -> List[int]:
        """Rows of the local K/V buffer: tau earlier tokens, then the query block itself."""
        return [t + q for t, q in zip(self.tau, self.q_lens)]

    @property
    def N(self) -> int:
        return sum(self.seq_lens)


def ragged_lengths(seed: int, tensor_id: int, B: int, lo: int, hi: int) -> List[int]:
    return [int(v) for v in integers(seed, tensor_id, (B,), lo, hi)]


def config(i: int, scale_down: int = 1) -> Workload:
    """The five benchmark workloads.  `scale_down` divides batch and context
    length (never head shapes) to give oracle-sized variants of the same recipe."""
    s = scale_down
    bf = torch.bfloat16
    if i == 1:
        return Workload("c1_tiny_fp32", torch.float32, [512], 256, 4, 4, 64, 1, 10, [32], [16], seed=0xD0D00001)
    if i == 2:
        B, n, q, tau = max(1, 8 // s), 4096 // s, max(16, 512 // s), max(8, 128 // s)
        return Workload("c2_llama7b_prefill", bf, [n] * B, 4096, 32, 32, 128, 1, 10, [q] * B, [tau] * B,
                        seed=0xD0D00002)
    if i == 3:
        B = max(2, 64 // s)
        lens = ragged_lengths(0xD0D00003, 900, B, 4096 // s, 8192 // s)
        return Workload("c3_llama7b_decode", bf, lens, 4096, 32, 32, 128, 1, 20, [1] * B, [max(4, 256 // s)] * B,
                        layers=32, seed=0xD0D00003)
    if i == 4:
        B, n = max(1, 16 // s), 2048 // s
        return Workload("c4_llama13b_autoencode", bf, [n] * B, 5120, 40, 40, 128, 1, 20, [n] * B, [0] * B,
                        layers=40, seed=0xD0D00004)
    if i == 5:
        n, q = 32768 // s, max(16, 1024 // s)
        return Workload("c5_long_context", bf, [n] * 2, 4096, 32, 32, 128, 1, 10, [q] * 2, [0] * 2,
                        seed=0xD0D00005, quantise_scores=True)
    raise ValueError(f"no workload {i}")


# tensor ids inside one layer's stream
_T_HIDDEN, _T_W, _T_K, _T_V, _T_Q, _T_KL, _T_VL = range(7)
_T_PER_LAYER = 16


def make_inputs(wl: Workload, device="cpu", layer: int = 0, which: Optional[List[str]] = None
                ) -> Dict[str, torch.Tensor]:
    """Packed tensors of one layer: hidden [N,d], w [d], K,V [N,H_kv,d_h],
    Q [sum q,H,d_h], Kl,Vl [sum m,H_kv,d_h], plus int32 cu_seqlens / cu_q / cu_local."""
    base = layer * _T_PER_LAYER
    N, Sq, Sm = wl.N, sum(wl.q_lens), sum(wl.local_lens)
    specs = {
        "hidden": (_T_HIDDEN, (N, wl.d_model), 1.0),
        "w": (_T_W, (wl.d_model,), wl.d_model ** -0.5),
        "K": (_T_K, (N, wl.H_kv, wl.d_h), 1.0),
        "V": (_T_V, (N, wl.H_kv, wl.d_h), 1.0),
        "Q": (_T_Q, (Sq, wl.H, wl.d_h), 1.0),
        "Kl": (_T_KL, (Sm, wl.H_kv, wl.d_h), 1.0),
        "Vl": (_T_VL, (Sm, wl.H_kv, wl.d_h), 1.0),
    }
    out: Dict[str, torch.Tensor] = {}
    for name, (tid, shape, std) in specs.items():
        if which is None or name in which:
            out[name] = normal(wl.seed, base + tid, shape, std, wl.dtype, device)
    out["cu_seqlens"] = cumulative(wl.seq_lens, device)
    out["cu_q"] = cumulative(wl.q_lens, device)
    out["cu_local"] = cumulative(wl.local_lens, device)
    return out


def cumulative(lengths, device="cpu") -> torch.Tensor:
    cu = [0]
    for v in lengths:
        cu.append(cu[-1] + int(v))
    assert cu[-1] < 2 ** 31
    return torch.tensor(cu, dtype=torch.int32, device=device)


def quantise16(scores: torch.Tensor) -> torch.Tensor:
    """Input preparation of the tie-stress workload: snap fp32 scores to the 16
    levels -8..7 (half-unit steps of the raw score), still stored as fp32."""
    return torch.clamp(torch.round(2.0 * scores.float()), -8.0, 7.0)


def exact_arithmetic_inputs(seed: int, N: int, d: int, dtype: torch.dtype, device="cpu"):
    """Hidden states in {-4..4} and weights in {-2..2}/64: every partial sum of
    the scorer is exactly representable in fp32 in any summation order, and
    scores collide massively."""
    x = integers(seed, 50, (N, d), -4, 4, device).to(dtype)
    w = (integers(seed, 51, (d,), -2, 2, device).to(torch.float64) / 64.0).to(dtype)
    return x, w


def to_numpy(t: torch.Tensor):
    """CPU numpy view for the oracle: float32 stays float32, bfloat16 becomes its uint16 bits."""
    import numpy as np
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()
