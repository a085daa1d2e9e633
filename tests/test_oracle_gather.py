"""Pins for the oracle sub-selection of K/V rows (Eq. 5)."""
import numpy as np
import torch

import oracle
import workloads as W


def _case(dtype, n_lens, H_kv=3, d_h=8, seed=40):
    N = sum(n_lens)
    K = W.normal(seed, 0, (N, H_kv, d_h), 1.0, dtype)
    V = W.normal(seed, 1, (N, H_kv, d_h), 1.0, dtype)
    k_lens = [oracle.nugget_count(n, 1, 4) for n in n_lens]
    s = W.normal(seed, 2, (N,), 1.0, torch.float32).numpy()
    cu_s, cu_k = oracle.cu_from_lengths(n_lens), oracle.cu_from_lengths(k_lens)
    idx = oracle.select_topk(s, cu_s, cu_k)
    return K, V, idx, cu_s, cu_k


def test_matches_library_index_select_bit_for_bit():
    for dtype in (torch.float32, torch.bfloat16):
        K, V, idx, cu_s, cu_k = _case(dtype, [33, 1, 90])
        Kn, Vn = oracle.gather(W.to_numpy(K), W.to_numpy(V), idx, cu_s, cu_k)
        glob = np.concatenate([idx[cu_k[b]:cu_k[b + 1]] + cu_s[b] for b in range(3)])
        wantK = torch.index_select(K, 0, torch.from_numpy(glob).long())
        wantV = torch.index_select(V, 0, torch.from_numpy(glob).long())
        assert np.array_equal(Kn, W.to_numpy(wantK)) and np.array_equal(Vn, W.to_numpy(wantV))


def test_head_major_is_the_transpose_of_token_major():
    K, V, idx, cu_s, cu_k = _case(torch.bfloat16, [64, 20])
    Kt, Vt = oracle.gather(W.to_numpy(K), W.to_numpy(V), idx, cu_s, cu_k, oracle.TOKEN_MAJOR)
    Kh, Vh = oracle.gather(W.to_numpy(K), W.to_numpy(V), idx, cu_s, cu_k, oracle.HEAD_MAJOR)
    assert np.array_equal(Kh, Kt.transpose(1, 0, 2)) and np.array_equal(Vh, Vt.transpose(1, 0, 2))


def test_ratio_one_is_identity_and_k_and_v_are_not_swapped():
    n_lens = [17, 5]
    N = sum(n_lens)
    K = W.normal(41, 0, (N, 2, 4), 1.0, torch.float32).numpy()
    V = -K - 100.0
    cu = oracle.cu_from_lengths(n_lens)
    idx = np.concatenate([np.arange(n) for n in n_lens]).astype(np.int32)
    Kn, Vn = oracle.gather(K, V, idx, cu, cu)
    assert np.array_equal(Kn, K) and np.array_equal(Vn, V)


def test_indices_are_sequence_local():
    # row value encodes its global token id; sequence 1 picks local rows 0 and 2
    K = np.arange(7, dtype=np.float32).reshape(7, 1, 1).repeat(2, axis=2)
    Kn, _ = oracle.gather(K, K, np.array([1, 0, 2], np.int32), oracle.cu_from_lengths([4, 3]),
                          oracle.cu_from_lengths([1, 2]))
    assert list(Kn[:, 0, 0]) == [1.0, 4.0, 6.0]


def test_layers_share_the_index_list_and_match_library_indexing():
    # [L, N, H_kv, d_h]: every layer is indexed with the same rows (Sec. 2.1); layer l's values are offset by 1000 l
    n_lens = [21, 40]
    K0, V0, idx, cu_s, cu_k = _case(torch.float32, n_lens)
    L = 3
    K = torch.stack([K0 + 1000.0 * l for l in range(L)])
    V = torch.stack([V0 - 1000.0 * l for l in range(L)])
    glob = torch.from_numpy(np.concatenate([idx[cu_k[b]:cu_k[b + 1]] + cu_s[b] for b in range(2)])).long()
    Kn, Vn = oracle.gather_layers(K.numpy(), V.numpy(), idx, cu_s, cu_k)
    assert np.array_equal(Kn, K[:, glob].numpy()) and np.array_equal(Vn, V[:, glob].numpy())
    Kh, Vh = oracle.gather_layers(K.numpy(), V.numpy(), idx, cu_s, cu_k, oracle.HEAD_MAJOR)
    assert np.array_equal(Kh, Kn.transpose(0, 2, 1, 3)) and np.array_equal(Vh, Vn.transpose(0, 2, 1, 3))
