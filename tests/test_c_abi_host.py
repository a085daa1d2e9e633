"""Host-only checks of the C-ABI library: it loads, exports every symbol include/dodo.h declares, and
rejects bad arguments before touching a device (no compute calls here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "dodo.h")


@pytest.fixture(scope="module")
def lib():
    import paper_2310_02409_amd as D
    return D.lib


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dodo_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    names = _declared_functions()
    assert {"dodo_score", "dodo_select_topk", "dodo_gather_nuggets", "dodo_nugget_attention", "dodo_nugget_count",
            "dodo_version", "dodo_status_string", "dodo_select_topk_workspace_bytes",
            "dodo_nugget_attention_workspace_bytes", "dodo_nugget_attention_cached", "dodo_threshold_from_sample",
            "dodo_select_threshold", "dodo_stream_append", "dodo_meanpool_nuggets", "dodo_score_mlp",
            "dodo_score_mlp_workspace_bytes", "dodo_gather_nuggets_layers",
            "dodo_nugget_attention_indexed", "dodo_segment_plan", "dodo_nugget_attention_segments",
            "dodo_ste_score_grad", "dodo_ste_score_grad_workspace_bytes"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in dodo.h but not exported"


def test_version_and_status_strings():
    import paper_2310_02409_amd as D
    assert D.dodo_version() == 100
    assert D.dodo_status_string(0) == "ok"
    assert "invalid" in D.dodo_status_string(-1)
    assert "unsupported" in D.dodo_status_string(-2)
    assert "workspace" in D.dodo_status_string(-3)
    assert D.dodo_status_string(-99) == "unknown status"


def test_nugget_count_matches_the_papers_worked_sizes():
    import paper_2310_02409_amd as D
    rows = [l.split() for l in open(os.path.join(ROOT, "tests", "golden", "nugget_counts.txt"))
            if l.strip() and not l.startswith("#")]
    for n, r, k in rows:
        assert D.dodo_nugget_count(int(n), 1, int(r)) == int(k)
    assert [D.dodo_nugget_count(n, 1, 10) for n in (512, 4096, 32768)] == [52, 410, 3277]
    assert D.dodo_nugget_count(8192, 1, 20) == 410 and D.dodo_nugget_count(2048, 1, 20) == 103
    assert D.dodo_nugget_count(0, 1, 10) == 0 and D.dodo_nugget_count(5, 1, 100) == 1
    assert D.dodo_nugget_count(7, 1, 1) == 7 and D.dodo_nugget_count(7, 3, 1) == 7
    assert D.dodo_nugget_count(10, 0, 5) == -1 and D.dodo_nugget_count(10, 1, 0) == -1
    assert D.dodo_nugget_count(2 ** 62, 1, 10) == (2 ** 62 + 9) // 10


def test_nugget_count_agrees_with_the_oracle_everywhere():
    import oracle
    import paper_2310_02409_amd as D
    for n in list(range(0, 300)) + [4095, 4096, 4097, 8191, 32768, 10 ** 7]:
        for num, den in [(1, 10), (1, 20), (1, 5), (1, 1), (3, 7), (7, 100)]:
            assert D.dodo_nugget_count(n, num, den) == oracle.nugget_count(n, num, den)


P = 0x1000  # any non-null, 16-byte aligned fake pointer: validation must fail before it is used


def test_score_argument_validation(lib):
    assert lib.dodo_score(0, P, 0.0, 1, 8, 64, 64, P, 0) == -1          # null hidden
    assert lib.dodo_score(P, P, 0.0, 1, -1, 64, 64, P, 0) == -1         # negative N
    assert lib.dodo_score(P, P, 0.0, 1, 8, 64, 32, P, 0) == -1          # stride < d
    assert lib.dodo_score(P, P, 0.0, 7, 8, 64, 64, P, 0) == -2          # dtype
    assert lib.dodo_score(P, P, 0.0, 1, 8, 60, 64, P, 0) == -2          # d not a multiple of 8
    i32, i64, vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p
    lib.dodo_score_layers.argtypes = [vp, vp, vp, ctypes.c_int, i32, i64, i32, i64, i64, i64, i64, vp, vp]
    assert lib.dodo_score_layers(P, P, None, 1, 3, 8, 64, 64, 8 * 64, 64, 4, P, None) == -1   # layers of scores overlap
    assert lib.dodo_score_layers(P, P, None, 1, 3, 8, 64, 64, -1, 64, 8, P, None) == -1       # negative stride
    assert lib.dodo_score_layers(P, P, None, 1, 0, 8, 64, 64, 8 * 64, 64, 8, P, None) == 0    # no layers: no-op
    assert lib.dodo_score_layers(P, P, None, 1, 70000, 8, 64, 64, 8 * 64, 64, 8, P, None) == -2
    assert lib.dodo_score(P + 2, P, 0.0, 1, 8, 64, 64, P, 0) == -2      # misaligned
    assert lib.dodo_score(0, 0, 0.0, 1, 0, 64, 64, 0, 0) == 0           # N == 0 is a no-op


def test_select_argument_validation(lib):
    assert lib.dodo_select_topk(0, P, P, 2, 10, 5, 0, P, 0, 0, 0) == -1
    assert lib.dodo_select_topk(P, P, P, 2, 10, 11, 0, P, 0, 0, 0) == -1  # max_k > max_n
    assert lib.dodo_select_topk(P, P, P, 2, 10, 0, 0, P, 0, 0, 0) == -1   # max_k == 0
    assert lib.dodo_select_topk(P, P, P, 2, 10, 5, 6, P, 0, 0, 0) == -1   # unknown flag bits
    assert lib.dodo_select_topk(P, P, P, -1, 10, 5, 0, P, 0, 0, 0) == -1
    assert lib.dodo_select_topk(0, 0, 0, 0, 10, 5, 0, 0, 0, 0, 0) == 0    # B == 0 is a no-op
    assert lib.dodo_select_topk_workspace_bytes(8, 4096) == 0
    # the workspace form: a 64-byte header that starts with the status word, then a block per sequence
    one, two = lib.dodo_select_topk_workspace_bytes(1, 32768), lib.dodo_select_topk_workspace_bytes(2, 32768)
    assert one > 64 and one % 4 == 0 and (two - one) == (one - 64)


def test_gather_argument_validation(lib):
    assert lib.dodo_gather_nuggets(0, P, 1, P, P, P, 2, 10, 4, 64, 256, P, P, 0, 0) == -1
    assert lib.dodo_gather_nuggets(P, P, 1, P, P, P, 2, 10, 4, 64, 100, P, P, 0, 0) == -1   # stride < H_kv*d_h
    assert lib.dodo_gather_nuggets(P, P, 1, P, P, P, 2, 10, 4, 64, 256, P, P, 2, 0) == -1   # layout
    assert lib.dodo_gather_nuggets(P, P, 5, P, P, P, 2, 10, 4, 64, 256, P, P, 0, 0) == -2   # dtype
    G = lib.dodo_gather_nuggets_layers
    assert G(P, P, 1, P, P, P, 2, 10, 0, 4, 64, 256, 0, 0, P, P, 0, 0) == 0            # no layers: no-op
    assert G(P, P, 1, P, P, P, 2, 10, -1, 4, 64, 256, 0, 0, P, P, 0, 0) == -1
    assert G(P, P, 1, P, P, P, 2, 10, 3, 4, 64, 256, 4096, 100, P, P, 0, 0) == -1      # layers of the output overlap
    assert G(P, P, 1, P, P, P, 2, 10, 3, 4, 64, 256, 4100, 2560, P, P, 0, 0) == -2     # layer stride not 16-byte
    assert G(P, P, 1, P, P, P, 2, 10, 70000, 4, 64, 256, 4096, 2560, P, P, 0, 0) == -2  # too many layers
    assert lib.dodo_gather_nuggets(P, P, 1, P, P, P, 2, 10, 4, 60, 240, P, P, 0, 0) == -2   # row not 16-byte multiple
    assert lib.dodo_gather_nuggets(P, P, 1, P, P, P, 2, 0, 4, 64, 256, P, P, 0, 0) == 0     # no nuggets: no-op


def test_attention_argument_validation(lib):
    def call(Q=P, Kn=P, Vn=P, Kl=P, Vl=P, B=2, H=8, H_kv=8, d_h=128, max_q=64, max_k=10, max_local=64, Kt=20,
             scale=0.1, dtype=1, layout=0, O=P, ws=0, ws_bytes=0):
        return lib.dodo_nugget_attention(Q, Kn, Vn, Kl, Vl, P, P, P, B, H, H_kv, d_h, max_q, max_k, max_local, Kt, scale,
                                         dtype, layout, O, 0, ws, ws_bytes, 0)
    assert call(Q=0) == -1
    assert call(H=8, H_kv=3) == -1
    assert call(layout=3) == -1
    assert call(scale=float("nan")) == -1
    assert call(Kn=0) == -1                       # nuggets expected but no cache
    assert call(dtype=4) == -2
    assert call(d_h=96) == -2
    assert call(Q=P + 4) == -2
    assert call(B=0) == 0 and call(max_q=0) == 0  # nothing to do
    # decode shape with few (sequence, head) pairs needs a split-K workspace
    need = lib.dodo_nugget_attention_workspace_bytes(2, 2, 128, 1, 3277, 1089, 1)
    assert need > 0
    assert call(B=2, H=2, H_kv=2, max_q=1, max_k=3277, max_local=1089, ws=0, ws_bytes=0) == -3
    assert call(B=2, H=2, H_kv=2, max_q=1, max_k=3277, max_local=1089, ws=P, ws_bytes=need - 1) == -3
    assert lib.dodo_nugget_attention_workspace_bytes(8, 32, 128, 512, 410, 640, 1) == 0
    # with the number of KV heads known: never less; more for a small batch of grouped heads (bf16, at least 4
    # query vectors per K/V row); the same where that kernel does not apply
    lib.dodo_nugget_attention_workspace_bytes_grouped.restype = ctypes.c_size_t
    G = lib.dodo_nugget_attention_workspace_bytes_grouped
    plain = lib.dodo_nugget_attention_workspace_bytes(2, 64, 128, 1, 3277, 1089, 1)
    assert G(2, 64, 8, 128, 1, 3277, 1089, 1) > plain
    assert G(2, 64, 8, 128, 1, 3277, 1089, 1) % ((128 + 3) * 4 * 2 * 64) == 0   # whole splits of 2 x 64 records
    assert G(2, 64, 64, 128, 1, 3277, 1089, 1) == plain    # one vector per row
    assert G(2, 64, 8, 64, 1, 3277, 1089, 1) > lib.dodo_nugget_attention_workspace_bytes(2, 64, 64, 1, 3277, 1089, 1)
    assert G(2, 64, 8, 64, 1, 3277, 1089, 1) % ((64 + 3) * 4 * 2 * 64) == 0     # heads of 64 channels: smaller records
    assert G(2, 64, 8, 128, 1, 3277, 1089, 0) == lib.dodo_nugget_attention_workspace_bytes(2, 64, 128, 1, 3277, 1089, 0)
    assert G(64, 64, 8, 128, 1, 410, 257, 1) == 0          # enough (sequence, KV head) pairs: no split wanted
    assert G(2, 64, 8, 128, 512, 3277, 1089, 1) == 0       # query blocks go to the other matrix-core kernel
    assert G(2, 64, 8, 128, 15, 3277, 1089, 1) > lib.dodo_nugget_attention_workspace_bytes(2, 64, 128, 15, 3277, 1089, 1)  # four passes
    assert G(2, 128, 2, 128, 1, 3277, 1089, 1) == lib.dodo_nugget_attention_workspace_bytes(2, 128, 128, 1, 3277, 1089, 1)  # 64 heads per KV head
    assert G(2, 64, 5, 128, 1, 3277, 1089, 1) == plain     # H_kv does not divide H: the plain size (the call refuses)


def test_threshold_path_argument_validation(lib):
    P = ctypes.c_void_p(16)  # never dereferenced: validation fails first
    i64 = ctypes.c_int64
    assert lib.dodo_threshold_from_sample(P, i64(0), i64(1), i64(10), P, None, ctypes.c_size_t(0), None) == -1
    assert lib.dodo_threshold_from_sample(P, i64(10), i64(0), i64(10), P, None, ctypes.c_size_t(0), None) == -1
    assert lib.dodo_threshold_from_sample(None, i64(10), i64(1), i64(10), P, None, ctypes.c_size_t(0), None) == -1
    lib.dodo_threshold_from_sample_workspace_bytes.restype = ctypes.c_size_t
    assert lib.dodo_threshold_from_sample_workspace_bytes(i64(1000)) == 0
    assert lib.dodo_threshold_from_sample_workspace_bytes(i64(400000)) == 4096
    assert lib.dodo_select_threshold(P, P, -1, P, P, P, P, None) == -1
    assert lib.dodo_select_threshold(P, P, 0, P, P, P, P, None) == 0
    assert lib.dodo_select_threshold(P, P, 2, None, P, P, P, None) == -1
    # stream append: shapes, stride, dtype, 16-byte rows
    ok = dict(B=2, H_kv=2, d_h=64, stride=128, cap=8, dtype=1)
    def call(**kw):
        a = {**ok, **kw}
        return lib.dodo_stream_append(P, P, P, P, a["dtype"], a["B"], a["H_kv"], a["d_h"], i64(a["stride"]), a["cap"], P,
                                      None, P, P, None)
    assert call(B=-1) == -1 and call(stride=100) == -1 and call(cap=-1) == -1
    assert call(dtype=7) == -2 and call(d_h=3, H_kv=1, stride=3) == -2
    assert call(B=0) == 0


def test_indexed_attention_argument_validation(lib):
    A = lib.dodo_nugget_attention_indexed
    #  Q  K  V idx cu_s Kl Vl cu_q cu_k cu_l  B  H H_kv d_h  mq  mk  ml  max_n stride scale dtype O lse ws ws_bytes stream
    assert A(P, P, P, 0, P, P, P, P, P, P, 2, 4, 4, 128, 1, 10, 5, 100, 512, 0.1, 1, P, 0, 0, 0, 0) == -1  # no index list
    assert A(P, P, P, P, P, P, P, P, P, P, 2, 4, 4, 128, 1, 10, 5, 9, 512, 0.1, 1, P, 0, 0, 0, 0) == -1   # max_k > max_n
    assert A(P, P, P, P, P, P, P, P, P, P, 2, 4, 4, 128, 1, 10, 5, 100, 500, 0.1, 1, P, 0, 0, 0, 0) == -1  # stride < H_kv d_h
    assert A(P, P, P, P, P, P, P, P, P, P, 2, 4, 4, 128, 1, 10, 5, 100, 516, 0.1, 1, P, 0, 0, 0, 0) == -2  # stride not 16-byte
    assert A(0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 4, 4, 128, 1, 10, 5, 100, 512, 0.1, 1, 0, 0, 0, 0, 0) == 0   # B == 0
    # query-block kernel: index list longer than its LDS buffer, and byte offsets beyond 31 bits
    assert A(P, P, P, P, P, P, P, P, P, P, 2, 4, 4, 128, 256, 7681, 5, 9000, 512, 0.1, 1, P, 0, 0, 0, 0) == -2
    assert A(P, P, P, P, P, P, P, P, P, P, 2, 4, 4, 128, 64, 4097, 5, 9000, 512, 0.1, 1, P, 0, 0, 0, 0) == -2
    assert A(P, P, P, P, P, P, P, P, P, P, 2, 4, 4, 128, 256, 10, 5, 3000000, 512, 0.1, 1, P, 0, 0, 0, 0) == -2


def test_segment_plan_argument_validation(lib):
    S = lib.dodo_segment_plan
    assert S(P, P, P, 2, 0, 4, 8, P, P, P, P, P, 0, 0) == -1    # seg_len == 0
    assert S(P, P, P, 2, 16, -1, 8, P, P, P, P, P, 0, 0) == -1  # tau < 0
    assert S(P, P, P, 2, 16, 4, 8, 0, P, P, P, P, 0, 0) == -1   # no output
    assert S(P, P, P, 2, 16, 4, 8, P, P, 0, P, P, 0, 0) == -1
    assert S(0, P, P, 2, 16, 4, 8, P, P, P, P, P, 0, 0) == -1   # no index list


def test_ste_score_grad_argument_validation(lib):
    G = lib.dodo_ste_score_grad
    lib.dodo_ste_score_grad_workspace_bytes.restype = ctypes.c_size_t
    assert lib.dodo_ste_score_grad_workspace_bytes(ctypes.c_int64(100), 4, ctypes.c_int64(10)) == (2 * 100 * 4 + 4 * 10) * 4
    #  Q  Kn Vn dO O lse cu_q cu_k B  H H_kv d_h mq mk  Sq  Kt  scale gscale acc dtype layout grad ws ws_bytes stream
    i64 = ctypes.c_int64
    assert G(P, P, P, P, P, P, P, P, 2, 4, 3, 128, 8, 8, i64(16), i64(10), 0.1, 0.1, 0, 1, 0, P, P, 1 << 20, 0) == -1  # H % H_kv
    assert G(P, P, P, P, P, P, P, P, 2, 4, 4, 128, 8, 8, i64(16), i64(10), 0.1, 0.1, 0, 1, 5, P, P, 1 << 20, 0) == -1  # layout
    assert G(P, P, P, P, P, P, P, P, 2, 4, 4, 100, 8, 8, i64(16), i64(10), 0.1, 0.1, 0, 1, 0, P, P, 1 << 20, 0) == -2  # d_h % 8
    assert G(P, P, P, P, P, P, P, P, 2, 4, 4, 128, 8, 8, i64(16), i64(10), 0.1, 0.1, 0, 1, 0, P, P, 16, 0) == -3       # workspace
    assert G(P, P, P, P, P, 0, P, P, 2, 4, 4, 128, 8, 8, i64(16), i64(10), 0.1, 0.1, 0, 1, 0, P, P, 1 << 20, 0) == -1  # lse missing
    assert G(0, 0, 0, 0, 0, 0, 0, 0, 0, 4, 4, 128, 8, 8, i64(16), i64(10), 0.1, 0.1, 0, 1, 0, 0, 0, 0, 0) == 0         # B == 0
