"""The C-ABI library on a host without a GPU: it loads, exports what include/pqtopk.h declares, sizes its
workspace by pure host arithmetic and rejects bad arguments before any HIP call (so dummy pointers are safe)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "pqtopk.h")
HEADERS = sorted(os.path.join(ROOT, "include", f) for f in os.listdir(os.path.join(ROOT, "include")) if f.endswith(".h"))

OK, NULL, SHAPE, UNSUPPORTED, WORKSPACE, ALIGN, HIP = 0, -1, -2, -3, -4, -5, -6


@pytest.fixture(scope="module")
def lib(pqlib_path):
    L = ctypes.CDLL(pqlib_path)
    P, I, LL, SZ = ctypes.c_void_p, ctypes.c_int, ctypes.c_longlong, ctypes.c_size_t
    L.pq_subitem_scores.argtypes = [P, P, P, I, I, I, I, P]
    L.pq_score_topk_workspace_bytes.argtypes = [LL, I, I, I, I]
    L.pq_score_topk_workspace_bytes.restype = SZ
    L.pq_score_topk.argtypes = [P, P, LL, I, I, I, I, P, P, P, SZ, P]
    L.pq_score_topk_profile.argtypes = [P, P, LL, I, I, I, I, P, P, P, SZ, P, I, P]
    L.pq_score_topk_u16_workspace_bytes.argtypes = [LL, I, I, I, I]
    L.pq_score_topk_u16_workspace_bytes.restype = SZ
    L.pq_score_topk_u16.argtypes = [P, P, LL, I, I, I, I, P, P, P, SZ, P]
    L.pq_score_topk_u16_profile.argtypes = [P, P, LL, I, I, I, I, P, P, P, SZ, P, I, P]
    L.pq_score_topk_subset_workspace_bytes.argtypes = [LL, I, I, I, I]
    L.pq_score_topk_subset_workspace_bytes.restype = SZ
    L.pq_score_topk_subset.argtypes = [P, P, P, LL, LL, I, I, I, I, P, P, P, SZ, P]
    L.pq_topk_scores_workspace_bytes.argtypes = [LL, I, I]
    L.pq_topk_scores_workspace_bytes.restype = SZ
    L.pq_topk_scores.argtypes = [P, LL, LL, I, I, P, P, P, SZ, P]
    L.pq_recjpq_scores.argtypes = [P, P, LL, I, I, I, P, LL, P]
    L.pq_reconstruct_items.argtypes = [P, P, LL, I, I, I, P, P]
    L.pq_default_scores.argtypes = [P, P, LL, I, I, P, LL, P]
    L.pq_read_bandwidth_profile.argtypes = [P, SZ, P, I, P]
    L.pq_strerror.argtypes = [I]
    L.pq_strerror.restype = ctypes.c_char_p
    return L


def declared_functions():
    """Every function any header under include/ declares (comments stripped)."""
    names = set()
    for header in HEADERS:
        text = re.sub(r"/\*.*?\*/", "", open(header).read(), flags=re.S)
        names |= set(re.findall(r"\b(pq_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_header_symbols_are_exported(lib):
    names = declared_functions()
    assert {"pq_subitem_scores", "pq_score_topk", "pq_score_topk_workspace_bytes", "pq_strerror"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_header_error_codes_match():
    text = open(HEADER).read()
    codes = dict(re.findall(r"#define\s+(PQ_[A-Z_]+)\s+(-?\d+)", text))
    assert int(codes["PQ_OK"]) == OK and int(codes["PQ_ERR_NULL"]) == NULL and int(codes["PQ_ERR_SHAPE"]) == SHAPE
    assert int(codes["PQ_ERR_UNSUPPORTED"]) == UNSUPPORTED and int(codes["PQ_ERR_WORKSPACE"]) == WORKSPACE
    assert int(codes["PQ_ERR_ALIGN"]) == ALIGN and int(codes["PQ_ERR_HIP"]) == HIP


def test_strerror(lib):
    seen = set()
    for c in (OK, NULL, SHAPE, UNSUPPORTED, WORKSPACE, ALIGN, HIP, -99):
        msg = lib.pq_strerror(c)
        assert msg and len(msg) > 1
        seen.add(msg)
    assert len(seen) == 8


def test_workspace_bytes(lib):
    ws = lib.pq_score_topk_workspace_bytes
    big = ws(1_280_000, 1, 8, 256, 10)
    assert big > 0 and big % 16 == 0
    assert ws(1_280_000, 64, 8, 256, 10) >= 64 * 10 * 8
    assert ws(50_000_000, 32, 8, 256, 10) > 0
    assert ws(10, 1, 8, 256, 10) >= 80
    for bad in ((0, 1, 8, 256, 10), (10, 0, 8, 256, 1), (10, 1, 0, 256, 1), (10, 1, 8, 0, 1), (10, 1, 8, 257, 1),
                (10, 1, 8, 256, 0), (10, 1, 8, 256, 11), (2 ** 31, 1, 8, 256, 10), (10 ** 6, 1, 8, 256, 513),
                (10 ** 6, 1, 129, 256, 10), (10 ** 6, 65536, 8, 256, 10)):
        assert ws(*bad) == 0, bad


def test_subitem_scores_argument_errors(lib):
    f = lib.pq_subitem_scores
    p = 0x10000
    assert f(None, p, p, 1, 64, 4, 256, None) == NULL
    assert f(p, None, p, 1, 64, 4, 256, None) == NULL
    assert f(p, p, None, 1, 64, 4, 256, None) == NULL
    assert f(p, p, p, 0, 64, 4, 256, None) == SHAPE
    assert f(p, p, p, 1, 0, 4, 256, None) == SHAPE
    assert f(p, p, p, 1, 64, 0, 256, None) == SHAPE
    assert f(p, p, p, 1, 64, 4, 0, None) == SHAPE
    assert f(p, p, p, 1, 64, 4, 65537, None) == SHAPE        # (Eq. 4 itself serves alphabets of up to 65536 sub-ids)
    assert f(p, p, p, 1, 66, 4, 256, None) == SHAPE          # d % m != 0
    assert f(p, p, p, 65536, 64, 4, 256, None) == UNSUPPORTED
    assert f(p + 2, p, p, 1, 64, 4, 256, None) == ALIGN


def test_score_topk_argument_errors(lib):
    f = lib.pq_score_topk
    p = 0x10000
    big = 1 << 30
    good = dict(codes=p, S=p, N=1000, B=1, m=8, b=256, K=10, ids=p, sc=p, ws=p, wsb=big, st=None)

    def call(**kw):
        a = dict(good, **kw)
        return f(a["codes"], a["S"], a["N"], a["B"], a["m"], a["b"], a["K"], a["ids"], a["sc"], a["ws"], a["wsb"],
                 a["st"])

    for name in ("codes", "S", "ids", "sc", "ws"):
        assert call(**{name: None}) == NULL, name
    assert call(N=0) == SHAPE and call(B=0) == SHAPE and call(m=0) == SHAPE and call(b=0) == SHAPE
    assert call(K=0) == SHAPE and call(b=257) == SHAPE and call(K=1001) == SHAPE and call(N=2 ** 31) == SHAPE
    assert call(N=10 ** 6, K=513) == UNSUPPORTED and call(m=129) == UNSUPPORTED and call(B=65536) == UNSUPPORTED
    assert call(N=10 ** 6, m=128, K=512) == UNSUPPORTED                # tables + candidate lists exceed LDS
    assert call(codes=p + 8) == ALIGN and call(ws=p + 4) == ALIGN and call(S=p + 1) == ALIGN
    assert call(ids=p + 2) == ALIGN and call(sc=p + 3) == ALIGN
    need = lib.pq_score_topk_workspace_bytes(1000, 1, 8, 256, 10)
    assert call(wsb=need - 1) == WORKSPACE
    # the profiling variant validates the same way, plus its own arguments
    g = lib.pq_score_topk_profile
    assert g(p, p, 1000, 1, 8, 256, 10, p, p, p, big, None, 3, None) == NULL
    out = ctypes.c_float(0)
    assert g(p, p, 1000, 1, 8, 256, 10, p, p, p, big, None, 0, ctypes.addressof(out)) == SHAPE
    assert g(None, p, 1000, 1, 8, 256, 10, p, p, p, big, None, 3, ctypes.addressof(out)) == NULL


def test_score_topk_u16_argument_errors(lib):
    f = lib.pq_score_topk_u16
    ws = lib.pq_score_topk_u16_workspace_bytes
    p = 0x10000
    big = 1 << 30
    good = dict(codes=p, S=p, N=100000, B=1, m=8, b=1024, K=10, ids=p, sc=p, ws=p, wsb=big, st=None)

    def call(**kw):
        a = dict(good, **kw)
        return f(a["codes"], a["S"], a["N"], a["B"], a["m"], a["b"], a["K"], a["ids"], a["sc"], a["ws"], a["wsb"],
                 a["st"])

    for name in ("codes", "S", "ids", "sc", "ws"):
        assert call(**{name: None}) == NULL, name
    assert call(N=0) == SHAPE and call(B=0) == SHAPE and call(m=0) == SHAPE and call(b=0) == SHAPE and call(K=0) == SHAPE
    assert call(b=65537) == SHAPE and call(K=100001) == SHAPE and call(N=2 ** 31) == SHAPE
    assert call(K=513) == UNSUPPORTED and call(m=129) == UNSUPPORTED and call(B=65536) == UNSUPPORTED
    # a table too large for LDS is read from memory: every alphabet up to 65536 is served
    assert ws(100000, 1, 8, 8192, 10) > 0 and ws(100000, 1, 2, 65536, 10) > 0 and ws(100000, 1, 64, 1024, 10) > 0
    assert ws(100000, 1, 128, 65536, 512) > 0 and ws(100000, 1, 8, 65537, 10) == 0
    assert ws(100000, 1, 8, 4096, 10) > 0 and ws(100000, 1, 1, 32768, 10) > 0 and ws(100000, 3, 5, 300, 100) > 0
    assert call(codes=p + 8) == ALIGN and call(ws=p + 4) == ALIGN and call(S=p + 1) == ALIGN
    assert call(wsb=ws(100000, 1, 8, 1024, 10) - 1) == WORKSPACE
    g = lib.pq_score_topk_u16_profile
    out = ctypes.c_float(0)
    assert g(p, p, 1000, 1, 8, 1024, 10, p, p, p, big, None, 3, None) == NULL
    assert g(p, p, 1000, 1, 8, 1024, 10, p, p, p, big, None, 0, ctypes.addressof(out)) == SHAPE
    assert g(p, p, 1000, 1, 8, 65537, 10, p, p, p, big, None, 3, ctypes.addressof(out)) == SHAPE


def test_score_topk_subset_argument_errors(lib):
    f = lib.pq_score_topk_subset
    ws = lib.pq_score_topk_subset_workspace_bytes
    p = 0x10000
    big = 1 << 30
    good = dict(codes=p, S=p, sub=p, n=500, N=1000, B=1, m=8, b=256, K=10, ids=p, sc=p, ws=p, wsb=big, st=None)

    def call(**kw):
        a = dict(good, **kw)
        return f(a["codes"], a["S"], a["sub"], a["n"], a["N"], a["B"], a["m"], a["b"], a["K"], a["ids"], a["sc"],
                 a["ws"], a["wsb"], a["st"])

    for name in ("codes", "S", "sub", "ids", "sc", "ws"):
        assert call(**{name: None}) == NULL, name
    assert call(n=0) == SHAPE and call(N=0) == SHAPE and call(B=0) == SHAPE and call(m=0) == SHAPE
    assert call(b=0) == SHAPE and call(b=257) == SHAPE and call(K=0) == SHAPE
    assert call(K=501) == SHAPE                                       # K exceeds the list, not the catalogue
    assert call(n=1001) == SHAPE                                      # a list of distinct ids cannot exceed N
    assert call(N=2 ** 31) == SHAPE
    assert call(n=10 ** 5, N=10 ** 6, K=513) == UNSUPPORTED and call(m=129) == UNSUPPORTED
    assert call(B=65536) == UNSUPPORTED
    assert call(codes=p + 8) == ALIGN and call(sub=p + 2) == ALIGN and call(ws=p + 4) == ALIGN
    assert call(ids=p + 1) == ALIGN and call(sc=p + 3) == ALIGN and call(S=p + 2) == ALIGN
    need = ws(500, 1, 8, 256, 10)
    assert need > 0 and need % 16 == 0
    assert call(wsb=need - 1) == WORKSPACE
    assert ws(100_000, 3, 8, 256, 100) >= 3 * 100 * 8
    for bad in ((0, 1, 8, 256, 1), (10, 1, 8, 256, 11), (10, 0, 8, 256, 1), (10, 1, 0, 256, 1), (10, 1, 8, 257, 1),
                (2 ** 31, 1, 8, 256, 10), (10 ** 6, 1, 8, 256, 513), (10 ** 6, 1, 129, 256, 10)):
        assert ws(*bad) == 0, bad


def test_comparison_scorers_argument_errors(lib):
    p, big = 0x10000, 1 << 30
    f = lib.pq_topk_scores
    assert f(None, 1000, 1000, 1, 10, p, p, p, big, None) == NULL
    assert f(p, 1000, 1000, 1, 10, None, p, p, big, None) == NULL
    assert f(p, 1000, 1000, 1, 10, p, p, None, big, None) == NULL
    assert f(p, 1000, 0, 1, 10, p, p, p, big, None) == SHAPE
    assert f(p, 1000, 1000, 0, 10, p, p, p, big, None) == SHAPE
    assert f(p, 1000, 1000, 1, 0, p, p, p, big, None) == SHAPE
    assert f(p, 1000, 1000, 1, 1001, p, p, p, big, None) == SHAPE
    assert f(p, 999, 1000, 1, 10, p, p, p, big, None) == SHAPE               # row shorter than N
    assert f(p, 10 ** 6, 10 ** 6, 1, 513, p, p, p, big, None) == UNSUPPORTED
    assert f(p + 4, 1000, 1000, 1, 10, p, p, p, big, None) == ALIGN
    assert f(p, 1001, 1000, 2, 10, p, p, p, big, None) == ALIGN              # rows of a batch must stay 16-byte aligned
    need = lib.pq_topk_scores_workspace_bytes(1000, 1, 10)
    assert need > 0 and need % 16 == 0
    assert f(p, 1000, 1000, 1, 10, p, p, p, need - 1, None) == WORKSPACE
    for bad in ((0, 1, 1), (10, 0, 1), (10, 1, 0), (10, 1, 11), (2 ** 31, 1, 1), (10 ** 6, 1, 513)):
        assert lib.pq_topk_scores_workspace_bytes(*bad) == 0, bad

    g = lib.pq_recjpq_scores
    assert g(None, p, 1000, 1, 8, 256, p, 1000, None) == NULL and g(p, p, 1000, 1, 8, 256, None, 1000, None) == NULL
    assert g(p, p, 0, 1, 8, 256, p, 1000, None) == SHAPE and g(p, p, 1000, 1, 8, 257, p, 1000, None) == SHAPE
    assert g(p, p, 1000, 1, 8, 256, p, 999, None) == SHAPE
    assert g(p, p, 1000, 1, 129, 256, p, 1000, None) == UNSUPPORTED and g(p, p + 2, 1000, 1, 8, 256, p, 1000, None) == ALIGN

    h = lib.pq_reconstruct_items
    assert h(None, p, 1000, 64, 4, 256, p, None) == NULL and h(p, p, 1000, 64, 4, 256, None, None) == NULL
    assert h(p, p, 1000, 66, 4, 256, p, None) == SHAPE and h(p, p, 0, 64, 4, 256, p, None) == SHAPE
    assert h(p, p, 1000, 258, 129, 256, p, None) == UNSUPPORTED and h(p, p, 1000, 64, 4, 256, p + 1, None) == ALIGN

    r = lib.pq_read_bandwidth_profile
    out = ctypes.c_float(0)
    assert r(None, 1 << 20, None, 3, ctypes.addressof(out)) == NULL and r(p, 1 << 20, None, 3, None) == NULL
    assert r(p, 8, None, 3, ctypes.addressof(out)) == SHAPE and r(p, 1 << 20, None, 0, ctypes.addressof(out)) == SHAPE
    assert r(p + 8, 1 << 20, None, 3, ctypes.addressof(out)) == ALIGN

    e = lib.pq_default_scores
    assert e(None, p, 1000, 1, 64, p, 1000, None) == NULL and e(p, None, 1000, 1, 64, p, 1000, None) == NULL
    assert e(p, p, 1000, 0, 64, p, 1000, None) == SHAPE and e(p, p, 1000, 1, 64, p, 999, None) == SHAPE
    assert e(p, p, 1000, 1, 66, p, 1000, None) == UNSUPPORTED and e(p + 4, p, 1000, 1, 64, p, 1000, None) == ALIGN


def test_binding_fails_loudly_without_library(tmp_path, monkeypatch):
    from paper_2408_09992_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError, match="missing"):
        binding.lib()


def test_product_does_not_reach_the_oracle():
    """Nothing in the package imports, loads or includes anything from oracle/."""
    pkg = os.path.join(ROOT, "paper_2408_09992_amd")
    pat = re.compile(r"^\s*(from|import)\s+oracle\b|pq_oracle|libpq_oracle|#include\s+\".*oracle", re.M)
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h", ".cpp")):
                assert not pat.search(open(os.path.join(dirpath, fn)).read()), fn


def test_workspace_bytes_over_a_grid_of_shapes(lib):
    """The launch planner behind the workspace size (pure host arithmetic) over a grid of shapes: every supported
    problem gets a workspace that holds at least one list of K keys per query and stays small next to the codes."""
    ws, ws16, wsub = lib.pq_score_topk_workspace_bytes, lib.pq_score_topk_u16_workspace_bytes, lib.pq_score_topk_subset_workspace_bytes
    n_checked = 0
    for N in (1, 7, 1000, 123_457, 1_280_000, 50_000_000, 2 ** 31 - 1):
        for B in (1, 2, 3, 5, 17, 48, 64, 100, 384, 1024, 65535):
            for m in (1, 3, 4, 8, 12, 16, 32, 64, 128):
                for K in (1, 10, 12, 13, 28, 29, 64, 100, 192, 193, 448, 512):
                    if K > N:
                        continue
                    need = ws(N, B, m, 256, K)
                    if m == 128 and K > 64:
                        continue                              # (may exceed LDS: allowed to be unsupported)
                    assert need >= B * K * 8 and need % 16 == 0, (N, B, m, K, need)
                    assert need <= 64 * B * K * 8 * 64 + (1 << 20), (N, B, m, K, need)   # at most a few thousand lists per query
                    sub = wsub(N, B, m, 256, K)
                    assert sub >= B * K * 8, (N, B, m, K, sub)
                    if m <= 16:
                        need16 = ws16(N, B, m, 1024, K)
                        assert need16 >= B * K * 8 and need16 % 16 == 0, (N, B, m, K, need16)
                    n_checked += 1
    assert n_checked > 5000
