"""GPU parity: dodo_score, dodo_select_topk, dodo_gather_nuggets against the oracle (through the C ABI)."""
import numpy as np
import pytest
import torch

import oracle
import workloads as W
from gpu_util import dev, oracle_counts

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def D():
    import paper_2310_02409_amd as D
    return D


# ---------------------------------------------------------------- scorer
@pytest.mark.parametrize("dtype,N,d", [
    (torch.float32, 512, 256), (torch.bfloat16, 1000, 4096), (torch.bfloat16, 77, 5120),
    (torch.float32, 33, 4096), (torch.bfloat16, 5, 8), (torch.bfloat16, 4097, 520), (torch.float32, 130, 8200),
])
def test_score_matches_oracle(D, dtype, N, d):
    x = W.normal(100, 0, (N, d), 1.0, dtype)
    w = W.normal(100, 1, (d,), d ** -0.5, dtype)
    ref = oracle.score(W.to_numpy(x), W.to_numpy(w), 0.125)
    got = D.dodo_score(x.to(dev()), w.to(dev()), 0.125).cpu().numpy()
    # fp32 accumulation of d products of magnitude ~ |x||w|: error << 1e-5 (1 + |s|)
    assert np.all(np.abs(got - ref) <= 1e-5 * (1 + np.abs(ref))), np.max(np.abs(got - ref))


def test_score_exact_arithmetic_inputs_are_bit_exact(D):
    for dtype in (torch.float32, torch.bfloat16):
        x, w = W.exact_arithmetic_inputs(7, 2048, 4096, dtype)
        ref = oracle.score(W.to_numpy(x), W.to_numpy(w))
        got = D.dodo_score(x.to(dev()), w.to(dev())).cpu().numpy()
        assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))


def test_score_is_deterministic_and_respects_row_stride(D):
    x = W.normal(101, 0, (300, 1024), 1.0, torch.bfloat16).to(dev())
    w = W.normal(101, 1, (512,), 0.05, torch.bfloat16).to(dev())
    view = x[:, :512]  # row stride 1024, d = 512
    scores = torch.empty(300, dtype=torch.float32, device=dev())
    rc = D.lib.dodo_score(view.data_ptr(), w.data_ptr(), 0.0, D.BF16, 300, 512, 1024, scores.data_ptr(),
                          torch.cuda.current_stream().cuda_stream)
    assert rc == 0
    ref = oracle.score(W.to_numpy(view.contiguous()), W.to_numpy(w))
    assert np.all(np.abs(scores.cpu().numpy() - ref) <= 1e-5 * (1 + np.abs(ref)))
    first = scores.clone()
    for _ in range(20):
        D.lib.dodo_score(view.data_ptr(), w.data_ptr(), 0.0, D.BF16, 300, 512, 1024, scores.data_ptr(),
                         torch.cuda.current_stream().cuda_stream)
        assert torch.equal(scores, first)


@pytest.mark.parametrize("dtype,d,pad,unaligned", [
    (torch.bfloat16, 4096, 64, False), (torch.bfloat16, 5120, 0, True), (torch.float32, 1536, 8, True),
    (torch.bfloat16, 520, 8, True), (torch.float32, 4096, 0, False),
])
def test_score_strided_rows_and_unaligned_weights_through_the_binding(D, dtype, d, pad, unaligned):
    # rows further apart than d elements; a weight vector that does not start on a 16-byte boundary is staged
    # element by element instead of with 16-byte loads
    N = 257
    hid = W.normal(102, 0, (N, d + pad), 1.0, dtype)
    wfull = W.normal(102, 1, (d + 8,), d ** -0.5, dtype)
    lo = 1 if unaligned else 0
    ref = oracle.score(W.to_numpy(hid[:, :d].contiguous()), W.to_numpy(wfull[lo:lo + d].contiguous()), 0.25)
    got = D.dodo_score(hid.to(dev())[:, :d], wfull.to(dev())[lo:lo + d], 0.25).cpu().numpy()
    assert np.all(np.abs(got - ref) <= 1e-5 * (1 + np.abs(ref))), np.max(np.abs(got - ref))


@pytest.mark.parametrize("dtype,L,N,d", [(torch.bfloat16, 5, 700, 4096), (torch.float32, 3, 129, 256), (torch.bfloat16, 2, 64, 1000)])
def test_score_layers_matches_oracle_and_the_single_layer_call(D, dtype, L, N, d):
    x = W.normal(130, 0, (L, N, d), 1.0, dtype)
    w = W.normal(130, 1, (L, d), d ** -0.5, dtype)
    b = W.normal(130, 2, (L,), 1.0, torch.float32)
    ref = oracle.score_layers(W.to_numpy(x), W.to_numpy(w), b.numpy())
    xd, wd, bd = x.to(dev()), w.to(dev()), b.to(dev())
    got = D.dodo_score_layers(xd, wd, bd, scores=torch.full((L, N), float("nan"), device=dev()))
    assert np.all(np.abs(got.cpu().numpy() - ref) <= 1e-5 * (1 + np.abs(ref)))
    for l in range(L):
        assert torch.equal(got[l], D.dodo_score(xd[l], wd[l], float(b[l])))
    # no biases; padded rows and room between the layers of the output
    xp = torch.zeros((L, N + 3, d + 8), dtype=dtype, device=dev())
    xp[:, :N, :d] = xd
    out = torch.full((L, 2 * N), 7.0, device=dev())
    D.dodo_score_layers(xp[:, :N, :d], wd, None, scores=out[:, :N])
    ref0 = oracle.score_layers(W.to_numpy(x), W.to_numpy(w))
    assert np.all(np.abs(out[:, :N].cpu().numpy() - ref0) <= 1e-5 * (1 + np.abs(ref0))) and bool((out[:, N:] == 7.0).all())


# ---------------------------------------------------------------- select
def _select_both(D, scores_np, n_lens, k_lens, flags=0):
    cu_s, cu_k = oracle.cu_from_lengths(n_lens), oracle.cu_from_lengths(k_lens)
    ref = oracle.select_topk(scores_np, cu_s, cu_k, flags)
    got = D.dodo_select_topk(torch.from_numpy(scores_np).to(dev()), torch.from_numpy(cu_s).to(dev()),
                             torch.from_numpy(cu_k).to(dev()), max(n_lens), max(max(k_lens), 1), int(cu_k[-1]),
                             flags).cpu().numpy()
    assert np.array_equal(got, ref)
    return got


@pytest.mark.parametrize("flags", [0, 1])
@pytest.mark.parametrize("n_lens,den", [
    ([512], 10), ([4096] * 8, 10), ([2048] * 16, 20), ([1, 2, 3, 64, 65, 127, 128, 129, 4095, 4097, 5000], 10),
    ([32768, 32768], 10), ([40000, 37000], 10), ([100, 0, 300], 3), ([8192, 4096, 6000], 20),
])
def test_select_bit_exact_gaussian_and_quantised(D, n_lens, den, flags):
    k_lens = [oracle.nugget_count(n, 1, den) for n in n_lens]
    s = W.normal(200 + den, len(n_lens), (sum(n_lens),), 1.0, torch.float32)
    _select_both(D, s.numpy(), n_lens, k_lens, flags)
    _select_both(D, W.quantise16(s).numpy(), n_lens, k_lens, flags)  # heavy ties: winners decided by index


def test_select_specials_and_degenerate_counts(D):
    s = W.normal(210, 0, (3000,), 1.0, torch.float32).numpy().copy()
    s[::7] = np.nan
    s[3::11] = np.inf
    s[5::13] = -np.inf
    s[1::17] = 0.0
    s[2::19] = -0.0
    for k in (1, 2, 150, 1500, 2999, 3000):
        for flags in (0, 1):
            _select_both(D, s, [3000], [k], flags)
    const = np.full(5000, -3.25, np.float32)
    assert list(_select_both(D, const, [5000], [500])) == list(range(500))
    # k_b = 0 for some sequences, k_b = n_b for others
    _select_both(D, s, [1000, 1000, 1000], [0, 1000, 17])


def test_select_on_gpu_scores_matches_oracle_select_on_the_same_array(D):
    # shared-array rule: the oracle selects on the scores the GPU scorer produced, and vice versa
    wl = W.config(2, scale_down=4)
    t = W.make_inputs(wl, which=["hidden", "w"])
    s_gpu = D.dodo_score(t["hidden"].to(dev()), t["w"].to(dev())).cpu().numpy()
    k_lens, _ = oracle_counts(wl.seq_lens, wl.keep_num, wl.keep_den)
    _select_both(D, s_gpu, wl.seq_lens, k_lens, 1)
    s_or = oracle.score(W.to_numpy(t["hidden"]), W.to_numpy(t["w"]))
    _select_both(D, s_or, wl.seq_lens, k_lens, 1)


def test_exact_arithmetic_raw_inputs_to_indices_bit_exact(D):
    # scores are exact in any summation order, so scorer + select must agree end to end, ties and all
    n_lens = [3000, 1234]
    x, w = W.exact_arithmetic_inputs(9, sum(n_lens), 1024, torch.bfloat16)
    k_lens, cu_k = oracle_counts(n_lens, 1, 10)
    cu_s = oracle.cu_from_lengths(n_lens)
    ref = oracle.select_topk(oracle.score(W.to_numpy(x), W.to_numpy(w)), cu_s, cu_k)
    s_gpu = D.dodo_score(x.to(dev()), w.to(dev()))
    got = D.dodo_select_topk(s_gpu, torch.from_numpy(cu_s).to(dev()), torch.from_numpy(cu_k).to(dev()), max(n_lens),
                             max(k_lens), int(cu_k[-1]))
    assert np.array_equal(got.cpu().numpy(), ref)


def test_select_is_deterministic(D):
    n_lens = [32768, 20000]
    k_lens, cu_k = oracle_counts(n_lens, 1, 10)
    s = W.quantise16(W.normal(220, 0, (sum(n_lens),), 1.0, torch.float32)).to(dev())
    cu_s = torch.from_numpy(oracle.cu_from_lengths(n_lens)).to(dev())
    cu_kd = torch.from_numpy(cu_k).to(dev())
    first = D.dodo_select_topk(s, cu_s, cu_kd, max(n_lens), max(k_lens), int(cu_k[-1])).clone()
    for _ in range(100):
        assert torch.equal(D.dodo_select_topk(s, cu_s, cu_kd, max(n_lens), max(k_lens), int(cu_k[-1])), first)


def test_select_long_sequences_over_several_workgroups(D):
    # with the workspace, sequences beyond 8192 tokens are cut into chunks that exchange histograms and counts
    n_lens = [20000, 9000, 33000, 70, 0]
    B = len(n_lens)
    need = D.dodo_select_topk_workspace_bytes(B, max(n_lens))
    assert need > 0 and D.dodo_select_topk_workspace_bytes(B, 8192) == 0
    ws = torch.zeros(need, dtype=torch.uint8, device=dev())  # zero-filled once, reused by every call below
    cu_s = oracle.cu_from_lengths(n_lens)
    base = W.normal(230, 0, (sum(n_lens),), 1.0, torch.float32)
    spec = base.numpy().copy()
    spec[::7] = np.nan
    spec[3::11] = np.inf
    spec[5::13] = -np.inf
    spec[1::17] = 0.0
    spec[2::19] = -0.0
    cases = [(base.numpy(), [oracle.nugget_count(n, 1, 10) for n in n_lens]),
             (W.quantise16(base).numpy(), [oracle.nugget_count(n, 1, 20) for n in n_lens]),
             (spec, [1, 9000, 1, 35, 0]), (spec, [20000, 4500, 16000, 70, 0]),
             (np.full(sum(n_lens), 2.5, np.float32), [2000, 1, 3300, 7, 0])]
    for scores, k_lens in cases:
        cu_k = oracle.cu_from_lengths(k_lens)
        sd, csd, ckd = torch.from_numpy(scores).to(dev()), torch.from_numpy(cu_s).to(dev()), torch.from_numpy(cu_k).to(dev())
        for flags in (0, 1):
            ref = oracle.select_topk(scores, cu_s, cu_k, flags)
            got = D.dodo_select_topk(sd, csd, ckd, max(n_lens), max(k_lens), int(cu_k[-1]), flags, ws=ws)
            assert np.array_equal(got.cpu().numpy(), ref)
            assert not bool(ws.any())  # left as it was found
            # without a (large enough) workspace: one workgroup per sequence, same result
            one = D.dodo_select_topk(sd, csd, ckd, max(n_lens), max(k_lens), int(cu_k[-1]), flags,
                                     ws=torch.zeros(16, dtype=torch.uint8, device=dev()))
            assert torch.equal(got, one)


def test_select_reports_a_wait_that_ran_out_and_heals_its_workspace(D):
    # The chunks of a long sequence wait for each other through arrival counters in the (zero-filled) workspace.
    # A counter that is not zero when the call begins can never reach the chunk count: the bounded waits of that
    # sequence give up, every workgroup still ends normally, the status word (first word of the workspace) says
    # so, the sequence's list holds a safe index, other sequences are untouched, and the workspace comes back
    # zero-filled, so that the next call is right again.
    n_lens = [20000, 20000]
    k_lens = [2000, 2000]
    need = D.dodo_select_topk_workspace_bytes(2, 20000)
    assert need > 0
    ws = torch.zeros(need // 4, dtype=torch.int32, device=dev())
    first_arrival_counter = 16 + 4 * 256  # header words, then the four histograms of sequence 0
    ws[first_arrival_counter] = 1000
    scores = W.normal(240, 0, (sum(n_lens),), 1.0, torch.float32)
    cu_s, cu_k = oracle.cu_from_lengths(n_lens), oracle.cu_from_lengths(k_lens)
    ref = oracle.select_topk(scores.numpy(), cu_s, cu_k, 1)
    args = (scores.to(dev()), torch.from_numpy(cu_s).to(dev()), torch.from_numpy(cu_k).to(dev()), 20000, 2000, 4000, 1)
    got = D.dodo_select_topk(*args, ws=ws.view(torch.uint8)).cpu().numpy()
    assert int(ws[0]) == 1                                  # DODO_SELECT_WAIT_FAILED
    assert np.all(got[:2000] == 19999)                      # the failed sequence: a safe index everywhere
    assert np.array_equal(got[2000:], ref[2000:])           # the other sequence is right
    assert not bool(ws[1:].any())                           # healed: zero-filled again apart from the status word
    ws[0] = 0
    got = D.dodo_select_topk(*args, ws=ws.view(torch.uint8)).cpu().numpy()
    assert np.array_equal(got, ref) and not bool(ws.any())


# ---------------------------------------------------------------- gather
@pytest.mark.parametrize("dtype,H_kv,d_h", [(torch.bfloat16, 32, 128), (torch.float32, 4, 64), (torch.bfloat16, 3, 64),
                                            (torch.bfloat16, 40, 128)])
@pytest.mark.parametrize("layout", [0, 1])
def test_gather_bit_exact(D, dtype, H_kv, d_h, layout):
    n_lens = [700, 1, 0, 333]
    N = sum(n_lens)
    K = W.normal(300, 0, (N, H_kv, d_h), 1.0, dtype)
    V = W.normal(300, 1, (N, H_kv, d_h), 1.0, dtype)
    k_lens, cu_k = oracle_counts(n_lens, 1, 5)
    cu_s = oracle.cu_from_lengths(n_lens)
    s = W.normal(300, 2, (N,), 1.0, torch.float32).numpy()
    idx = oracle.select_topk(s, cu_s, cu_k)
    Kn_ref, Vn_ref = oracle.gather(W.to_numpy(K), W.to_numpy(V), idx, cu_s, cu_k, layout)
    Kn, Vn = D.dodo_gather_nuggets(K.to(dev()), V.to(dev()), torch.from_numpy(idx).to(dev()),
                                   torch.from_numpy(cu_s).to(dev()), torch.from_numpy(cu_k).to(dev()),
                                   int(cu_k[-1]), layout)
    assert np.array_equal(W.to_numpy(Kn), Kn_ref) and np.array_equal(W.to_numpy(Vn), Vn_ref)


@pytest.mark.parametrize("dtype,H_kv,d_h,layout", [
    (torch.bfloat16, 40, 128, 0), (torch.bfloat16, 1, 64, 1), (torch.float32, 5, 64, 0), (torch.float32, 40, 128, 1),
    (torch.bfloat16, 3, 128, 0),
])
def test_gather_row_widths_and_token_stride(D, dtype, H_kv, d_h, layout):
    # rows from 128 bytes to 20 KiB (the workgroup size follows the row width), tokens one head further apart than
    # the heads that are gathered
    n_lens = [90, 0, 41, 300, 7]
    N = sum(n_lens)
    K = W.normal(301, 0, (N, H_kv + 1, d_h), 1.0, dtype)
    V = W.normal(301, 1, (N, H_kv + 1, d_h), 1.0, dtype)
    k_lens, cu_k = oracle_counts(n_lens, 1, 3)
    cu_s = oracle.cu_from_lengths(n_lens)
    idx = oracle.select_topk(W.normal(301, 2, (N,), 1.0, torch.float32).numpy(), cu_s, cu_k)
    Kn_ref, Vn_ref = oracle.gather(W.to_numpy(K[:, :H_kv].contiguous()), W.to_numpy(V[:, :H_kv].contiguous()), idx, cu_s,
                                   cu_k, layout)
    Kn, Vn = D.dodo_gather_nuggets(K.to(dev())[:, :H_kv], V.to(dev())[:, :H_kv], torch.from_numpy(idx).to(dev()),
                                   torch.from_numpy(cu_s).to(dev()), torch.from_numpy(cu_k).to(dev()), int(cu_k[-1]),
                                   layout)
    assert np.array_equal(W.to_numpy(Kn), Kn_ref) and np.array_equal(W.to_numpy(Vn), Vn_ref)


def test_gather_ratio_one_is_identity(D):
    n_lens = [129, 64]
    K = W.normal(301, 0, (sum(n_lens), 8, 128), 1.0, torch.bfloat16).to(dev())
    V = W.normal(301, 1, (sum(n_lens), 8, 128), 1.0, torch.bfloat16).to(dev())
    cu = torch.from_numpy(oracle.cu_from_lengths(n_lens)).to(dev())
    idx = torch.cat([torch.arange(n, dtype=torch.int32) for n in n_lens]).to(dev())
    Kn, Vn = D.dodo_gather_nuggets(K, V, idx, cu, cu, sum(n_lens))
    assert torch.equal(Kn, K) and torch.equal(Vn, V)


@pytest.mark.parametrize("dtype,L,H_kv,d_h", [(torch.bfloat16, 5, 32, 128), (torch.float32, 2, 4, 64), (torch.bfloat16, 1, 3, 64)])
@pytest.mark.parametrize("layout", [0, 1])
def test_gather_layers_bit_exact(D, dtype, L, H_kv, d_h, layout):
    n_lens = [300, 1, 0, 211]
    N = sum(n_lens)
    K = W.normal(310, 0, (L, N, H_kv, d_h), 1.0, dtype)
    V = W.normal(310, 1, (L, N, H_kv, d_h), 1.0, dtype)
    k_lens, cu_k = oracle_counts(n_lens, 1, 5)
    cu_s = oracle.cu_from_lengths(n_lens)
    s = W.normal(310, 2, (N,), 1.0, torch.float32).numpy()
    idx = oracle.select_topk(s, cu_s, cu_k)
    Kn_ref, Vn_ref = oracle.gather_layers(W.to_numpy(K), W.to_numpy(V), idx, cu_s, cu_k, layout)
    args = (torch.from_numpy(idx).to(dev()), torch.from_numpy(cu_s).to(dev()), torch.from_numpy(cu_k).to(dev()),
            int(cu_k[-1]), layout)
    Kn, Vn = D.dodo_gather_nuggets_layers(K.to(dev()), V.to(dev()), *args)
    assert np.array_equal(W.to_numpy(Kn), Kn_ref) and np.array_equal(W.to_numpy(Vn), Vn_ref)
    # strided views: a padded token stride in the source and room between the layers of the destination
    Kp = torch.zeros((L, N, H_kv + 1, d_h), dtype=dtype, device=dev())
    Vp = torch.zeros_like(Kp)
    Kp[:, :, :H_kv] = K.to(dev())
    Vp[:, :, :H_kv] = V.to(dev())
    Kt = int(cu_k[-1])
    shape = (Kt, H_kv, d_h) if layout == 0 else (H_kv, Kt, d_h)
    Kbig = torch.full((L, 2) + shape, 7.0, dtype=dtype, device=dev())
    Vbig = torch.full((L, 2) + shape, 7.0, dtype=dtype, device=dev())
    D.dodo_gather_nuggets_layers(Kp[:, :, :H_kv], Vp[:, :, :H_kv], *args, Kn=Kbig[:, 0], Vn=Vbig[:, 0])
    assert np.array_equal(W.to_numpy(Kbig[:, 0]), Kn_ref) and np.array_equal(W.to_numpy(Vbig[:, 0]), Vn_ref)
    assert bool((Kbig[:, 1] == 7.0).all()) and bool((Vbig[:, 1] == 7.0).all())


@pytest.mark.parametrize("B", [65, 130, 200])
@pytest.mark.parametrize("layout", [0, 1])
def test_gather_many_sequences(D, B, layout):
    # more than 64 sequences: the destination row's sequence is found by the binary search, not the ballot;
    # empty sequences, sequences without nuggets, and (token-major) a nugget total given as an upper bound
    n_lens = [int(v) for v in W.integers(320, 7, (B,), 0, 90)]
    n_lens[3], n_lens[B - 1] = 0, 57
    k_lens = [min(n, int(v)) for n, v in zip(n_lens, W.integers(320, 8, (B,), 0, 12))]
    k_lens[5], k_lens[B - 1] = 0, 9
    N, Kt = sum(n_lens), sum(k_lens)
    H_kv, d_h, dtype = 6, 128, torch.bfloat16
    K, V = W.normal(320, 0, (N, H_kv, d_h), 1.0, dtype), W.normal(320, 1, (N, H_kv, d_h), 1.0, dtype)
    cu_s, cu_k = oracle.cu_from_lengths(n_lens), oracle.cu_from_lengths(k_lens)
    idx = oracle.select_topk(W.normal(320, 2, (N,), 1.0, torch.float32).numpy(), cu_s, cu_k)
    Kn_ref, Vn_ref = oracle.gather(W.to_numpy(K), W.to_numpy(V), idx, cu_s, cu_k, layout)
    to = lambda a: torch.from_numpy(a).to(dev())
    Kd, Vd = K.to(dev()), V.to(dev())
    Kn, Vn = D.dodo_gather_nuggets(Kd, Vd, to(idx), to(cu_s), to(cu_k), Kt, layout)
    assert np.array_equal(W.to_numpy(Kn), Kn_ref) and np.array_equal(W.to_numpy(Vn), Vn_ref)
    # the same through the all-layers entry point (two layers reading the same rows)
    K2, V2 = torch.stack([Kd, Kd]), torch.stack([Vd, Vd])
    Kn2, Vn2 = D.dodo_gather_nuggets_layers(K2, V2, to(idx), to(cu_s), to(cu_k), Kt, layout)
    for l in range(2):
        assert torch.equal(Kn2[l], Kn) and torch.equal(Vn2[l], Vn)
    if layout == 0:
        extra = 37
        Kb = torch.full((Kt + extra, H_kv, d_h), 7.0, dtype=dtype, device=dev())
        Vb = torch.full_like(Kb, 7.0)
        D.dodo_gather_nuggets(Kd, Vd, to(idx), to(cu_s), to(cu_k), Kt + extra, layout, Kn=Kb, Vn=Vb)
        assert torch.equal(Kb[:Kt], Kn) and torch.equal(Vb[:Kt], Vn)
        assert bool((Kb[Kt:] == 7.0).all()) and bool((Vb[Kt:] == 7.0).all())
