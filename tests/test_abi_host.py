"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the header
declares, and every argument check returns its status before anything is enqueued."""
import ctypes as C
import os
import re

import pytest

import paper_2502_00299_amd as pkg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(pkg.LIB_PATH):
        from paper_2502_00299_amd import build
        build.build(verbose=False)
    return pkg.load_library()


def header_functions():
    text = open(os.path.join(ROOT, "include", "chunkkv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(chunkkv_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = header_functions()
    assert set(names) == set(pkg.SYMBOLS)
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings(lib):
    seen = {lib.chunkkv_status_string(i).decode() for i in range(6)}
    assert len(seen) == 6 and "ok" in seen
    assert lib.chunkkv_status_string(99).decode() == "unknown status"


def good(**kw):
    d = dict(n_q_heads=32, n_kv_heads=8, head_dim=128, window=32, chunk=10, dtype=pkg.BF16, seqlen=[8192],
             n_keep=[816], kv_base=[0], kv_stride_head=8192 * 128, kv_stride_tok=128)
    d.update(kw)
    return pkg.Problem(**d)


FAKE = C.c_void_p(0x1000)  # never dereferenced: every call below fails its argument check first


def score_rc(lib, prob, q=FAKE, k=FAKE, out=FAKE, ws=FAKE, ws_bytes=1 << 40):
    return lib.chunkkv_score(C.byref(prob.as_c()), q, k, out, None, ws, ws_bytes, None)


def test_workspace_size_is_positive_and_grows_with_layers(lib):
    p = good()
    a = pkg.chunkkv_workspace_bytes(p, 1, 1)
    b = pkg.chunkkv_workspace_bytes(p, 32, 1)
    c = pkg.chunkkv_workspace_bytes(p, 32, 2)
    assert 0 < a < c < b


def test_every_storage_type_is_accepted(lib):
    """fp32, bf16 and fp16 caches pass validation; the 16-bit types need the same workspace."""
    sizes = {dt: pkg.chunkkv_workspace_bytes(good(dtype=dt), 4, 2) for dt in (pkg.F32, pkg.BF16, pkg.F16)}
    assert all(v > 0 for v in sizes.values()) and sizes[pkg.BF16] == sizes[pkg.F16]
    assert (pkg.F32, pkg.BF16, pkg.F16) == (0, 1, 2)          # the enum of the header
    assert score_rc(lib, good(dtype=pkg.F16), ws=None) == 4   # argument checks reach the workspace check


@pytest.mark.parametrize("kw,status", [
    (dict(n_q_heads=30), 2),                       # Hq % Hkv != 0
    (dict(window=0), 2),
    (dict(chunk=0), 2),
    (dict(seqlen=[16]), 2),                        # w > L
    (dict(n_keep=[8161]), 2),                      # n_keep > P
    (dict(n_keep=[-1]), 2),
    (dict(sel_cap=5), 2),                          # needs ceil(816/10)+1 = 83
    (dict(score_cap=10), 2),                       # needs 816
    (dict(kv_stride_tok=100), 2),                  # < head_dim
    (dict(kv_stride_tok=132), 2),                  # rows not 16-byte aligned
    (dict(kv_base=[3]), 2),
    (dict(softmax_scale=-1.0), 2),
    (dict(head_dim=96), 3),
    (dict(dtype=7), 3),
    (dict(flags=4), 3),                            # unknown flag bit
    (dict(flags=0x80000000), 3),
    (dict(window=64, n_q_heads=128, n_keep=[100]), 3),   # g*w = 1024 rows > 512
    # K rows of one (sequence, kv-head) must span < 2 GiB: 1.1 M tokens of a packed 8-head bf16 cache do not
    (dict(seqlen=[1_100_000], n_keep=[1000], kv_stride_head=128, kv_stride_tok=8 * 128), 3),
])
def test_problem_validation(lib, kw, status):
    p = good(**kw)
    assert score_rc(lib, p) == status
    assert pkg.chunkkv_workspace_bytes(p) == 0


def test_flags_travel_per_call(lib):
    """Selection mode and scoring path are bits of chunkkv_problem.flags: every combination of the known bits
    passes validation, the flags change no workspace requirement's validity, and the library exports no
    process-wide switch for them."""
    assert (pkg.FLAG_WHOLE_CHUNKS, pkg.FLAG_TWO_PASS) == (1, 2)       # the values of the header
    for flags in (0, pkg.FLAG_WHOLE_CHUNKS, pkg.FLAG_TWO_PASS, pkg.FLAG_WHOLE_CHUNKS | pkg.FLAG_TWO_PASS):
        p = good(flags=flags)
        assert pkg.chunkkv_workspace_bytes(p, 4, 2) > 0
        assert score_rc(lib, p, ws=None) == 4                           # reaches the workspace check
    header = open(os.path.join(ROOT, "include", "chunkkv.h")).read()
    assert "CHUNKKV_FLAG_WHOLE_CHUNKS 1u" in header and "CHUNKKV_FLAG_TWO_PASS 2u" in header
    assert not [n for n in header_functions() if "_set_" in n]
    for name in ("chunkkv_set_whole_chunks", "chunkkv_set_single_pass", "chunkkv_set_overlap"):
        assert not hasattr(lib, name) or pytest.fail(f"{name} is still exported")


def test_null_pointers_and_workspace(lib):
    p = good()
    assert lib.chunkkv_score(None, FAKE, FAKE, FAKE, None, FAKE, 1 << 40, None) == 1
    assert score_rc(lib, p, q=None) == 1
    assert score_rc(lib, p, k=None) == 1
    assert score_rc(lib, p, out=None) == 1
    assert score_rc(lib, p, q=C.c_void_p(0x1004)) == 2             # misaligned device pointer
    assert score_rc(lib, p, ws=None) == 4
    assert score_rc(lib, p, ws_bytes=pkg.chunkkv_workspace_bytes(p) - 1) == 4
    cp = p.as_c()
    assert lib.chunkkv_chunk_topk(C.byref(cp), None, FAKE, FAKE, FAKE, None, 0, None) == 1
    assert lib.chunkkv_compact(C.byref(cp), FAKE, None, FAKE, FAKE, FAKE, FAKE, FAKE, None) == 1
    bad_out = good(out_base=[0], out_stride_head=848 * 128, out_stride_tok=100)
    assert lib.chunkkv_compact(C.byref(bad_out.as_c()), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None) == 2


def test_stack_argument_checks(lib):
    p = good()
    cp = p.as_c()
    n = 4
    tab = (C.c_void_p * n)(*[0x1000] * n)
    hole = (C.c_void_p * n)(0x1000, None, 0x1000, None)
    ws = pkg.chunkkv_workspace_bytes(p, n, 2)
    call = lambda q, k, reuse, nl=n, wsb=ws: lib.chunkkv_compress_stack(
        C.byref(cp), nl, reuse, q, k, tab, tab, tab, FAKE, FAKE, FAKE, FAKE, wsb, None)
    assert call(tab, tab, 0) == 2                  # R < 1
    assert call(tab, tab, 2, nl=0) == 2
    assert call(hole, hole, 2) == 1                # K of layer 1 missing
    assert call(hole, tab, 1) == 1                 # every layer needs Q when R = 1
    assert call(tab, tab, 2, wsb=ws - 1) == 4
    assert call(None, tab, 2) == 1


def test_lse_argument_checks(lib):
    # the log-sum-exp variants check what the plain calls check, plus the lse pointers (error paths only:
    # every call returns before a launch)
    p = good()
    cp = p.as_c()
    ws = pkg.chunkkv_workspace_bytes(p)
    assert lib.chunkkv_score_lse(C.byref(cp), FAKE, FAKE, None, FAKE, None, FAKE, ws, None) == 1
    assert lib.chunkkv_score_lse(C.byref(cp), FAKE, None, FAKE, FAKE, None, FAKE, ws, None) == 1
    assert lib.chunkkv_score_lse(C.byref(cp), FAKE, FAKE, FAKE, FAKE, None, FAKE, ws - 1, None) == 4
    n = 4
    tab = (C.c_void_p * n)(*[0x1000] * n)
    hole = (C.c_void_p * n)(0x1000, None, 0x1000, None)
    nol = (C.c_void_p * n)(None, None, 0x1000, None)
    ws4 = pkg.chunkkv_workspace_bytes(p, n, 2)
    call = lambda lse, reuse, wsb=ws4: lib.chunkkv_compress_stack_lse(
        C.byref(cp), n, reuse, tab, tab, tab, lse, tab, tab, FAKE, FAKE, FAKE, FAKE, wsb, None)
    assert call(None, 2) == 1
    assert call(nol, 2) == 1                       # leader layer 0 has no lse
    assert call(hole, 1) == 1                      # every layer is a leader when R = 1
    assert call(hole, 2, wsb=ws4 - 1) == 4         # lse of the non-leader layers may be missing


def test_layer_and_jaccard_argument_checks(lib):
    p = good()
    cp = p.as_c()
    ws = pkg.chunkkv_workspace_bytes(p)
    layer = lambda l, R, q, k=FAKE, wsb=ws: lib.chunkkv_compress_layer(
        C.byref(cp), l, R, q, None, k, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, wsb, None)
    assert layer(-1, 2, FAKE) == 2
    assert layer(0, 0, FAKE) == 2
    assert layer(0, 2, None) == 1                  # a leader layer needs its window queries
    assert layer(2, 2, None) == 1
    assert layer(1, 2, None, k=None) == 1
    assert layer(1, 2, None, wsb=ws - 1) == 4      # a follower layer passes the checks up to the workspace
    assert lib.chunkkv_jaccard(C.byref(cp), 1, FAKE, FAKE, FAKE, FAKE, None) == 2
    assert lib.chunkkv_jaccard(C.byref(cp), 3, FAKE, None, FAKE, FAKE, None) == 1
    assert lib.chunkkv_jaccard(C.byref(cp), 3, FAKE, FAKE, FAKE, None, None) == 1


def test_hybrid_stack_argument_checks(lib):
    # chunk size per reuse group: the table is validated entry by entry, capacities against the smallest entry
    n, R = 5, 2
    tab = (C.c_void_p * n)(*[0x1000] * n)
    chunks = lambda *c: (C.c_int32 * len(c))(*c)
    p1 = good(chunk=1)                               # capacities sized for chunk 1 hold for every chunk size
    cp1 = p1.as_c()
    ws = lib.chunkkv_workspace_bytes_hybrid(C.byref(cp1), n, R, chunks(10, 1, 5))
    assert ws >= max(pkg.chunkkv_workspace_bytes(good(chunk=c, sel_cap=p1.sel_cap, score_cap=p1.score_cap), n, R)
                     for c in (10, 1, 5))
    call = lambda cp, table, wsb=ws, q=tab: lib.chunkkv_compress_stack_hybrid(
        C.byref(cp), n, R, table, q, tab, tab, None, tab, tab, FAKE, FAKE, FAKE, FAKE, wsb, None)
    assert call(cp1, None) == 1
    assert call(cp1, chunks(10, 0, 5)) == 2
    assert call(cp1, chunks(10, -3, 5)) == 2
    assert call(cp1, chunks(10, 1, 5), wsb=ws - 1) == 4
    assert call(cp1, chunks(10, 1, 5), q=None) == 1
    assert lib.chunkkv_workspace_bytes_hybrid(C.byref(cp1), n, R, chunks(10, 0, 5)) == 0
    assert lib.chunkkv_workspace_bytes_hybrid(C.byref(cp1), n, R, None) == 0
    # capacities sized for chunk 10 are too small for a group of chunk 1
    cp10 = good().as_c()
    assert call(cp10, chunks(10, 1, 5)) == 2
    assert call(cp10, chunks(10, 20, 10), wsb=1 << 40, q=None) == 1    # ... but fine for chunk sizes >= 10


def test_quality_metrics_argument_checks(lib):
    p = good()
    cp = p.as_c()
    ws = pkg.chunkkv_quality_workspace_bytes(p)
    assert ws >= max(pkg.chunkkv_decode_workspace_bytes(p, True), pkg.chunkkv_decode_workspace_bytes(p, False))
    call = lambda q=FAKE, k=FAKE, ko=FAKE, l1=FAKE, cos=FAKE, wsb=ws: lib.chunkkv_quality_metrics(
        C.byref(cp), None, q, k, FAKE, ko, FAKE, l1, cos, FAKE, wsb, None)
    assert call(q=None) == 1 and call(k=None) == 1 and call(ko=None) == 1 and call(l1=None) == 1 and call(cos=None) == 1
    assert call(k=C.c_void_p(0x1004)) == 2
    assert call(wsb=ws - 1) == 4
    bad = good(out_base=[0], out_stride_head=848 * 128, out_stride_tok=100)
    assert pkg.chunkkv_quality_workspace_bytes(bad) == 0


def test_missing_library_fails_loudly(tmp_path):
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        pkg.load_library(str(tmp_path / "nope.so"))


def test_decode_argument_checks(lib):
    p = good(out_base=[0], out_stride_head=848 * 128, out_stride_tok=128)
    cp = p.as_c()
    full, comp = pkg.chunkkv_decode_workspace_bytes(p, False), pkg.chunkkv_decode_workspace_bytes(p, True)
    assert 0 < comp < full                       # fewer key ranges over the 10 % cache
    f = lib.chunkkv_decode_attention
    assert f(None, 0, None, FAKE, FAKE, FAKE, FAKE, None, FAKE, full, None) == 1
    assert f(C.byref(cp), 0, None, None, FAKE, FAKE, FAKE, None, FAKE, full, None) == 1
    assert f(C.byref(cp), 0, None, FAKE, None, FAKE, FAKE, None, FAKE, full, None) == 1
    assert f(C.byref(cp), 0, None, FAKE, FAKE, None, FAKE, None, FAKE, full, None) == 1
    assert f(C.byref(cp), 0, None, FAKE, FAKE, FAKE, None, None, FAKE, full, None) == 1
    assert f(C.byref(cp), 0, None, C.c_void_p(0x1008), FAKE, FAKE, FAKE, None, FAKE, full, None) == 2
    assert f(C.byref(cp), 0, None, FAKE, FAKE, FAKE, FAKE, None, None, full, None) == 4
    assert f(C.byref(cp), 0, None, FAKE, FAKE, FAKE, FAKE, None, FAKE, full - 1, None) == 4
    assert f(C.byref(cp), 1, None, FAKE, FAKE, FAKE, FAKE, None, FAKE, comp - 1, None) == 4
    # the compressed layout needs the output geometry of the problem
    bad_out = good(out_base=[0], out_stride_head=848 * 128, out_stride_tok=100)
    assert pkg.chunkkv_decode_workspace_bytes(bad_out, True) == 0
    assert pkg.chunkkv_decode_workspace_bytes(bad_out, False) == full
    assert f(C.byref(bad_out.as_c()), 1, None, FAKE, FAKE, FAKE, FAKE, None, FAKE, full, None) == 2
    assert pkg.chunkkv_decode_workspace_bytes(good(head_dim=96), False) == 0
