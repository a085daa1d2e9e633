"""The whole step (score, select, gather, block attention, decode token with the split-K workspace, a small query
block through the entry point that allocates nothing) is captured into a HIP graph and replayed: every replay, with eager work and synchronisations in between, must reproduce the eager
results bit for bit (the library records kernel launches only: no memset nodes, no allocation, no host read-back)."""
import pytest
import torch

import workloads as W
from gpu_util import dev

pytestmark = pytest.mark.gpu


def test_step_replays_from_a_graph():
    import paper_2310_02409_amd as D
    wl = W.config(2, scale_down=4)
    g = W.make_inputs(wl, dev())
    B = wl.B
    cu_k, ks = D.cu_nuggets_from_lengths(wl.seq_lens, wl.keep_num, wl.keep_den, dev())
    Kt, max_n, max_k = sum(ks), max(wl.seq_lens), max(ks)
    scores = torch.empty(wl.N, dtype=torch.float32, device=dev())
    idx = torch.empty(Kt, dtype=torch.int32, device=dev())
    Kn = torch.empty((Kt, wl.H_kv, wl.d_h), dtype=wl.dtype, device=dev())
    Vn = torch.empty_like(Kn)
    O = torch.empty_like(g["Q"])
    scale = wl.d_h ** -0.5
    # a decode token per sequence over long local buffers, so that the split-K kernel really splits
    m_dec = 3000
    Qd = W.normal(wl.seed, 50, (B, wl.H, wl.d_h), 1.0, wl.dtype, dev())
    Kld = W.normal(wl.seed, 51, (B * m_dec, wl.H_kv, wl.d_h), 1.0, wl.dtype, dev())
    Vld = W.normal(wl.seed, 52, (B * m_dec, wl.H_kv, wl.d_h), 1.0, wl.dtype, dev())
    cu_qd, cu_ld = W.cumulative([1] * B, dev()), W.cumulative([m_dec] * B, dev())
    Od = torch.empty_like(Qd)
    need = D.dodo_nugget_attention_workspace_bytes(B, wl.H, wl.d_h, 1, max_k, m_dec, D.BF16)
    assert need > 0
    ws = torch.zeros(need, dtype=torch.uint8, device=dev())
    # four query rows per sequence over the same rows: the matrix-core kernel for several vectors per K/V row, split
    # over workgroups, with its partial records and flags in the library's own buffer
    Q4 = W.normal(wl.seed, 53, (B * 4, wl.H, wl.d_h), 1.0, wl.dtype, dev())
    cu_q4 = W.cumulative([4] * B, dev())
    O4 = torch.empty_like(Q4)

    def step():
        D.dodo_score(g["hidden"], g["w"], 0.0, scores)
        D.dodo_select_topk(scores, g["cu_seqlens"], cu_k, max_n, max_k, Kt, D.FORCE_LAST, idx)
        D.dodo_gather_nuggets(g["K"], g["V"], idx, g["cu_seqlens"], cu_k, Kt, D.TOKEN_MAJOR, Kn, Vn)
        D.dodo_nugget_attention(g["Q"], Kn, Vn, g["Kl"], g["Vl"], g["cu_q"], cu_k, g["cu_local"], max(wl.q_lens), max_k,
                                max(wl.local_lens), scale, D.TOKEN_MAJOR, O)
        D.dodo_nugget_attention(Qd, Kn, Vn, Kld, Vld, cu_qd, cu_k, cu_ld, 1, max_k, m_dec, scale, D.TOKEN_MAJOR, Od, ws=ws)
        D.dodo_nugget_attention_noalloc(Q4, Kn, Vn, Kld, Vld, cu_q4, cu_k, cu_ld, 4, max_k, m_dec, scale, D.TOKEN_MAJOR, O4)

    step()
    torch.cuda.synchronize()
    want = [t.clone() for t in (scores, idx, Kn, Vn, O, Od, O4)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(4):
        for t in (scores, idx, Kn, Vn, O, Od, O4):
            t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip((scores, idx, Kn, Vn, O, Od, O4), want):
            assert torch.equal(got, ref), f"replay {rep} differs from the eager result"
        step()  # eager work between the replays
        torch.cuda.synchronize()
        assert not bool(ws.view(torch.int32)[-(need // 4 // (wl.d_h + 3)):].any())  # the flags are left cleared
