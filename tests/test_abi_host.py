"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, answers the size queries, and rejects bad arguments before launching anything."""
import ctypes
import re
from pathlib import Path

import pytest

import oracle
import paper_2604_16957_amd as tq
from paper_2604_16957_amd import binding as B

ROOT = Path(__file__).resolve().parent.parent


def _declared_functions():
    text = (ROOT / "include" / "tq.h").read_text()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tq_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert {"tq_quantize_kv", "tq_sdpa_int4_decode", "tq_dequant_then_attend", "tq_sdpa_int4_partial",
            "tq_sdpa_int4_reduce", "tq_workspace_bytes", "tq_status_string"} <= set(names)
    lib = ctypes.CDLL(str(tq.library_path()))
    for n in names:
        assert hasattr(lib, n), n


def test_size_queries_follow_the_papers_format():
    # 5 bits/element (Sec. 2.1): one 128K layer of the 70B shape is 160 MiB; 80 layers are 12.5 GiB
    assert tq.tq_kv_bytes(1, 8, 131072, 128) == 167772160
    assert tq.tq_kv_bytes(1, 8, 131072, 128) * 80 == oracle.kv_bytes_int4(80, 8, 131072, 128)
    assert tq.tq_kv_bytes(1, 16, 32768, 256) == 167772160
    # 4 + 32/g bits per element (Sec. 2.1): 5.0, 4.5, 4.25
    for g, bits in ((32, 5.0), (64, 4.5), (128, 4.25)):
        assert tq.tq_kv_bytes_grouped(1, 8, 131072, 128, g) * 8 == 2 * 8 * 131072 * 128 * bits
        assert tq.tq_kv_bytes_grouped(1, 8, 131072, 128, g) * 80 == oracle.kv_bytes_int4(80, 8, 131072, 128, group=g)
    assert tq.tq_kv_bytes_grouped(1, 8, 1024, 128, 48) == 0 and tq.tq_kv_bytes_grouped(1, 8, 1024, 128, 256) == 0
    assert tq.tq_dense_scratch_bytes(1, 8, 131072, 128) == 2 * 8 * 131072 * 128 * 2
    assert tq.tq_workspace_bytes(1, 64, 128) % 256 == 0 and tq.tq_workspace_bytes(1, 64, 128) > 0
    assert tq.tq_workspace_bytes(0, 64, 128) == 0 and tq.tq_kv_bytes(1, 8, 0, 128) == 0
    for args in [(1, 8, 131072), (1, 1, 1024), (4, 8, 131072), (1, 16, 32768), (1, 1, 1), (1, 1, 33)]:
        n = tq.tq_plan_splits(*args)
        assert 1 <= n <= 128
        assert n <= (args[2] + 31) // 32


def test_status_strings():
    seen = {tq.tq_status_string(s) for s in range(0, -9, -1)}
    assert len(seen) == 9 and "unknown status" not in seen
    assert tq.tq_status_string(-99) == "unknown status"


FAKE = 0x10000  # 16- and 256-byte aligned, never dereferenced: validation fails first


def _cache(**kw):
    f = dict(k_codes=FAKE, v_codes=FAKE, k_scale=FAKE, k_zero=FAKE, v_scale=FAKE, v_zero=FAKE,
             batch=1, n_kv_heads=8, head_dim=128, group_size=32, capacity=1024, layout=0)
    f.update(kw)
    return B.TqKvCacheStruct(*[f[n] for n, _ in B.TqKvCacheStruct._fields_])


def _decode(cache, q=FAKE, hq=64, S=1024, out=FAKE, ws=FAKE, wsb=None, opts=None):
    wsb = tq.tq_workspace_bytes(1, 64, 128) if wsb is None else wsb
    return B.raw().tq_sdpa_int4_decode(ctypes.byref(cache) if cache is not None else None, q, hq, S, 0.1, out,
                                       ws, wsb, opts, None)


def test_decode_rejects_bad_arguments_without_a_gpu():
    E = B
    assert _decode(None) == E.TQ_ERR_NULL
    assert _decode(_cache(k_scale=None)) == E.TQ_ERR_NULL
    assert _decode(_cache(), q=None) == E.TQ_ERR_NULL
    assert _decode(_cache(), out=None) == E.TQ_ERR_NULL
    assert _decode(_cache(), ws=None) == E.TQ_ERR_NULL
    assert _decode(_cache(head_dim=64)) == E.TQ_ERR_SHAPE
    assert _decode(_cache(head_dim=192)) == E.TQ_ERR_SHAPE
    assert _decode(_cache(head_dim=512), wsb=tq.tq_workspace_bytes(1, 64, 512), opts=ctypes.byref(B.TqDecodeOptsStruct(0, 1, 0, 2))) \
        == E.TQ_ERR_UNSUPPORTED                                          # several query tokens: matrix-core kernels only
    assert _decode(_cache(head_dim=1024)) == E.TQ_ERR_SHAPE
    assert _decode(_cache(group_size=48)) == E.TQ_ERR_SHAPE and _decode(_cache(group_size=16)) == E.TQ_ERR_SHAPE
    assert _decode(_cache(group_size=256)) == E.TQ_ERR_SHAPE
    # groups of 64 / 128: the matrix-core kernel covers them at head_dim 128 (groups of 128: an even capacity);
    # elsewhere the generic kernel only (no matrix-core variant, one query token)
    wsb256 = tq.tq_workspace_bytes(2, 64, 256)
    for kw in (dict(group_size=64, head_dim=256), dict(group_size=128, head_dim=256), dict(group_size=128, capacity=1025)):
        assert _decode(_cache(**kw), wsb=wsb256, opts=ctypes.byref(B.TqDecodeOptsStruct(0, 2, 0, 0))) == E.TQ_ERR_UNSUPPORTED
        assert _decode(_cache(**kw), wsb=wsb256, opts=ctypes.byref(B.TqDecodeOptsStruct(0, 0, 0, 2))) == E.TQ_ERR_UNSUPPORTED
    f = B.raw().tq_decode_launches
    for g, hd, want in ((64, 128, 1), (128, 128, 1), (64, 256, 2), (128, 256, 2)):
        c = _cache(group_size=g, head_dim=hd)
        assert f(ctypes.byref(c), 64, 1024, 0.1, None) == want        # one launch = the matrix-core kernel merges in place
    assert _decode(_cache(batch=0)) == E.TQ_ERR_SHAPE
    assert _decode(_cache(layout=7)) == E.TQ_ERR_SHAPE
    assert _decode(_cache(), hq=63) == E.TQ_ERR_SHAPE
    assert _decode(_cache(), hq=0) == E.TQ_ERR_SHAPE
    assert _decode(_cache(), S=0) == E.TQ_ERR_EMPTY
    assert _decode(_cache(), S=-5) == E.TQ_ERR_EMPTY
    assert _decode(_cache(), S=1025) == E.TQ_ERR_CAPACITY
    assert _decode(_cache(v_codes=FAKE + 4)) == E.TQ_ERR_ALIGN
    assert _decode(_cache(), q=FAKE + 2) == E.TQ_ERR_ALIGN
    assert _decode(_cache(), ws=FAKE + 16) == E.TQ_ERR_ALIGN
    assert _decode(_cache(), wsb=1000) == E.TQ_ERR_WORKSPACE
    bad = B.TqDecodeOptsStruct(0, 9)
    assert _decode(_cache(), opts=ctypes.byref(bad)) == E.TQ_ERR_UNSUPPORTED
    neg = B.TqDecodeOptsStruct(-1, 0)
    assert _decode(_cache(), opts=ctypes.byref(neg)) == E.TQ_ERR_UNSUPPORTED
    negw = B.TqDecodeOptsStruct(0, 0, -3)
    assert _decode(_cache(), opts=ctypes.byref(negw)) == E.TQ_ERR_UNSUPPORTED
    # several query tokens per sequence: 0 and 1 mean one; more than 8, a negative count and the generic kernel
    # are refused; the workspace holds batch * n_queries rows; a sequence holds all its queries
    ws3 = tq.tq_workspace_bytes(3, 64, 128)
    for nq, kw, want in ((9, {}, E.TQ_ERR_UNSUPPORTED), (-1, {}, E.TQ_ERR_UNSUPPORTED),
                         (3, dict(wsb=ws3 - 1), E.TQ_ERR_WORKSPACE), (3, dict(wsb=ws3, S=2), E.TQ_ERR_EMPTY)):
        o = B.TqDecodeOptsStruct(0, 0, 0, nq)
        assert _decode(_cache(), opts=ctypes.byref(o), **kw) == want
    assert _decode(_cache(), opts=ctypes.byref(B.TqDecodeOptsStruct(0, 1, 0, 3)), wsb=ws3) == E.TQ_ERR_UNSUPPORTED
    f = B.raw().tq_decode_launches
    c = _cache()
    # 4 query tokens x 8 heads per KV head: two 16-row tiles per KV head, whose chunks the merge kernel merges;
    # one query token (8 rows) at this length is merged by the decode kernel itself
    assert f(ctypes.byref(c), 64, 1024, 0.1, ctypes.byref(B.TqDecodeOptsStruct(0, 0, 0, 4))) == 2
    assert f(ctypes.byref(c), 64, 1024, 0.1, ctypes.byref(B.TqDecodeOptsStruct(0, 0, 0, 1))) == 1
    assert f(ctypes.byref(c), 64, 1024, -0.1, ctypes.byref(B.TqDecodeOptsStruct(0, 0, 0, 4))) == 0
    assert f(ctypes.byref(c), 64, 3, 0.1, ctypes.byref(B.TqDecodeOptsStruct(0, 0, 0, 4))) == 0


def test_quantize_rejects_bad_arguments_without_a_gpu():
    E = B
    q = B.raw().tq_quantize_kv
    c = _cache()
    assert q(None, FAKE, FAKE, 0, 1, None) == E.TQ_ERR_NULL
    assert q(ctypes.byref(c), None, FAKE, 0, 1, None) == E.TQ_ERR_NULL
    assert q(ctypes.byref(c), FAKE, None, 0, 1, None) == E.TQ_ERR_NULL
    assert q(ctypes.byref(c), FAKE, FAKE, 0, 0, None) == E.TQ_ERR_EMPTY
    assert q(ctypes.byref(c), FAKE, FAKE, -1, 1, None) == E.TQ_ERR_CAPACITY
    assert q(ctypes.byref(c), FAKE, FAKE, 1024, 1, None) == E.TQ_ERR_CAPACITY
    assert q(ctypes.byref(c), FAKE, FAKE, 1000, 25, None) == E.TQ_ERR_CAPACITY
    assert q(ctypes.byref(c), FAKE + 8, FAKE, 0, 1, None) == E.TQ_ERR_ALIGN
    c2 = _cache(head_dim=96)
    assert q(ctypes.byref(c2), FAKE, FAKE, 0, 1, None) == E.TQ_ERR_SHAPE


def test_reduce_and_baseline_reject_bad_arguments_without_a_gpu():
    E = B
    r = B.raw().tq_sdpa_int4_reduce
    wsb = tq.tq_workspace_bytes(1, 64, 128)
    assert r(1, 64, 128, 4, None, wsb, FAKE, None) == E.TQ_ERR_NULL
    assert r(1, 64, 100, 4, FAKE, wsb, FAKE, None) == E.TQ_ERR_SHAPE
    assert r(1, 64, 128, 0, FAKE, wsb, FAKE, None) == E.TQ_ERR_EMPTY
    assert r(1, 64, 128, 100000, FAKE, wsb, FAKE, None) == E.TQ_ERR_UNSUPPORTED
    assert r(1, 64, 128, 4, FAKE, 10, FAKE, None) == E.TQ_ERR_WORKSPACE
    d = B.raw().tq_dequant_then_attend
    c = _cache()
    need = tq.tq_dense_scratch_bytes(1, 8, 1024, 128)
    assert d(ctypes.byref(c), FAKE, 64, 1024, 0.1, FAKE, FAKE, wsb, None, need, None, None) == E.TQ_ERR_NULL
    assert d(ctypes.byref(c), FAKE, 64, 1024, 0.1, FAKE, FAKE, wsb, FAKE, need - 1, None, None) == E.TQ_ERR_WORKSPACE
    assert d(ctypes.byref(c), FAKE, 64, 2000, 0.1, FAKE, FAKE, wsb, FAKE, need, None, None) == E.TQ_ERR_CAPACITY
    win = B.TqDecodeOptsStruct(0, 0, 128)         # the comparator has no sliding window
    assert d(ctypes.byref(c), FAKE, 64, 1024, 0.1, FAKE, FAKE, wsb, FAKE, need, ctypes.byref(win), None) == E.TQ_ERR_UNSUPPORTED


def test_varlen_entry_points_reject_bad_arguments_without_a_gpu():
    E = B
    c = _cache()
    wsb = tq.tq_workspace_bytes(1, 64, 128)
    d = B.raw().tq_sdpa_int4_decode_varlen
    assert d(ctypes.byref(c), FAKE, 64, None, 1024, 0.1, FAKE, FAKE, wsb, None, None) == E.TQ_ERR_NULL
    assert d(ctypes.byref(c), FAKE, 64, FAKE + 2, 1024, 0.1, FAKE, FAKE, wsb, None, None) == E.TQ_ERR_ALIGN
    assert d(ctypes.byref(c), FAKE, 64, FAKE, 0, 0.1, FAKE, FAKE, wsb, None, None) == E.TQ_ERR_EMPTY
    assert d(ctypes.byref(c), FAKE, 64, FAKE, 1025, 0.1, FAKE, FAKE, wsb, None, None) == E.TQ_ERR_CAPACITY
    assert d(ctypes.byref(c), FAKE, 63, FAKE, 1024, 0.1, FAKE, FAKE, wsb, None, None) == E.TQ_ERR_SHAPE
    assert d(ctypes.byref(c), FAKE, 64, FAKE, 1024, 0.1, FAKE, FAKE, 8, None, None) == E.TQ_ERR_WORKSPACE
    q = B.raw().tq_quantize_kv_varlen
    assert q(ctypes.byref(c), FAKE, FAKE, None, 1, None) == E.TQ_ERR_NULL
    assert q(ctypes.byref(c), None, FAKE, FAKE, 1, None) == E.TQ_ERR_NULL
    assert q(ctypes.byref(c), FAKE, FAKE, FAKE, 0, None) == E.TQ_ERR_EMPTY
    assert q(ctypes.byref(c), FAKE, FAKE, FAKE, 1025, None) == E.TQ_ERR_CAPACITY
    assert q(ctypes.byref(c), FAKE, FAKE, FAKE + 1, 1, None) == E.TQ_ERR_ALIGN


def test_append_decode_rejects_bad_arguments_without_a_gpu():
    E = B
    c = _cache()
    wsb = tq.tq_workspace_bytes(1, 64, 128)
    f = B.raw().tq_sdpa_int4_append_decode
    assert f(ctypes.byref(c), None, FAKE, FAKE, 64, 1024, 0.1, FAKE, FAKE, wsb, None, None) == E.TQ_ERR_NULL
    assert f(ctypes.byref(c), FAKE, None, FAKE, 64, 1024, 0.1, FAKE, FAKE, wsb, None, None) == E.TQ_ERR_NULL
    assert f(ctypes.byref(c), FAKE, FAKE, None, 64, 1024, 0.1, FAKE, FAKE, wsb, None, None) == E.TQ_ERR_NULL
    assert f(ctypes.byref(c), FAKE + 8, FAKE, FAKE, 64, 1024, 0.1, FAKE, FAKE, wsb, None, None) == E.TQ_ERR_ALIGN
    assert f(ctypes.byref(c), FAKE, FAKE, FAKE, 64, 0, 0.1, FAKE, FAKE, wsb, None, None) == E.TQ_ERR_EMPTY
    assert f(ctypes.byref(c), FAKE, FAKE, FAKE, 64, 1025, 0.1, FAKE, FAKE, wsb, None, None) == E.TQ_ERR_CAPACITY


def test_paged_entry_points_reject_bad_arguments_without_a_gpu():
    E = B
    pool = _cache(batch=64, capacity=256)         # 64 pages of 256 tokens
    wsb = tq.tq_workspace_bytes(4, 64, 128)
    d = B.raw().tq_sdpa_int4_decode_paged
    ok_args = lambda **kw: dict(dict(pool=pool, tbl=FAKE, mb=8, batch=4, q=FAKE, hq=64, lens=FAKE, S=2048, out=FAKE,
                                     ws=FAKE, wsb=wsb, opts=None), **kw)

    def call(**kw):
        a = ok_args(**kw)
        return d(ctypes.byref(a["pool"]), a["tbl"], a["mb"], a["batch"], a["q"], a["hq"], a["lens"], a["S"], 0.1,
                 a["out"], a["ws"], a["wsb"], a["opts"], None)

    assert call(tbl=None) == E.TQ_ERR_NULL
    assert call(lens=None) == E.TQ_ERR_NULL
    assert call(q=None) == E.TQ_ERR_NULL
    assert call(pool=_cache(batch=64, capacity=200)) == E.TQ_ERR_SHAPE      # page length not a power of two
    assert call(pool=_cache(batch=64, capacity=16)) == E.TQ_ERR_SHAPE       # shorter than a tile
    assert call(batch=0) == E.TQ_ERR_SHAPE
    assert call(mb=0) == E.TQ_ERR_SHAPE
    assert call(S=2049) == E.TQ_ERR_CAPACITY                                # more than max_blocks pages hold
    assert call(S=0) == E.TQ_ERR_EMPTY
    assert call(tbl=FAKE + 2) == E.TQ_ERR_ALIGN
    assert call(wsb=wsb - 1) == E.TQ_ERR_WORKSPACE
    qz = B.raw().tq_quantize_kv_paged
    assert qz(ctypes.byref(pool), None, 8, 4, FAKE, FAKE, FAKE, 1, None) == E.TQ_ERR_NULL
    assert qz(ctypes.byref(pool), FAKE, 8, 4, FAKE, FAKE, None, 1, None) == E.TQ_ERR_NULL
    assert qz(ctypes.byref(pool), FAKE, 8, 4, FAKE, FAKE, FAKE, 0, None) == E.TQ_ERR_EMPTY
    assert qz(ctypes.byref(pool), FAKE, 8, 4, FAKE, FAKE, FAKE, 2049, None) == E.TQ_ERR_CAPACITY


def test_decode_launch_count_query():
    f = B.raw().tq_decode_launches
    short = _cache()                                                  # 1024 tokens: launch-bound
    assert f(ctypes.byref(short), 64, 1024, 0.1, None) == 1           # matrix-core kernel merges in place
    generic = B.TqDecodeOptsStruct(0, 1)
    assert f(ctypes.byref(short), 64, 1024, 0.1, ctypes.byref(generic)) == 2
    assert f(ctypes.byref(short), 64, 1024, -0.1, None) == 2          # non-positive scale: generic kernel
    assert f(ctypes.byref(short), 8 * 16, 1024, 0.1, None) == 2       # GQA ratio 16: a 16-row tile, merge kernel
    assert f(ctypes.byref(short), 8 * 4, 1024, 0.1, None) == 1        # GQA ratio 4: merged in place
    forced = B.TqDecodeOptsStruct(0, 2)
    assert f(ctypes.byref(short), 8 * 16, 1024, 0.1, ctypes.byref(forced)) == 2
    assert f(ctypes.byref(short), 8 * 8, 1024, 0.1, ctypes.byref(forced)) == 1
    assert f(ctypes.byref(short), 64, 1024, -0.1, ctypes.byref(forced)) == 0
    assert f(ctypes.byref(short), 63, 1024, 0.1, None) == 0
    assert f(ctypes.byref(short), 64, 0, 0.1, None) == 0 and f(ctypes.byref(short), 64, 1025, 0.1, None) == 0
    assert f(None, 64, 1024, 0.1, None) == 0
    long = _cache(capacity=131072)                                    # stream-bound: separate merge kernel
    assert f(ctypes.byref(long), 64, 131072, 0.1, None) == 2
    assert f(ctypes.byref(long), 64, 8192, 0.1, None) == 1
    big = _cache(batch=512)                                           # 4096 rows of one chunk each: no merge at all
    assert f(ctypes.byref(big), 64, 16, 0.1, None) == 1


def test_append_decode_with_lengths_rejects_bad_arguments_without_a_gpu():
    E = B
    c = _cache()
    wsb = tq.tq_workspace_bytes(1, 64, 128)
    f = B.raw().tq_sdpa_int4_append_decode_varlen
    ok = dict(k=FAKE, v=FAKE, q=FAKE, lens=FAKE, S=1024, out=FAKE, ws=FAKE, wsb=wsb)
    def call(**kw):
        a = dict(ok, **kw)
        return f(ctypes.byref(c), a["k"], a["v"], a["q"], 64, a["lens"], a["S"], 0.1, a["out"], a["ws"], a["wsb"], None, None)
    assert call(k=None) == E.TQ_ERR_NULL and call(v=None) == E.TQ_ERR_NULL and call(lens=None) == E.TQ_ERR_NULL
    assert call(q=None) == E.TQ_ERR_NULL and call(out=None) == E.TQ_ERR_NULL
    assert call(S=0) == E.TQ_ERR_EMPTY and call(S=1025) == E.TQ_ERR_CAPACITY
    assert call(k=FAKE + 8) == E.TQ_ERR_ALIGN and call(lens=FAKE + 2) == E.TQ_ERR_ALIGN
    assert call(wsb=wsb - 1) == E.TQ_ERR_WORKSPACE
    g = B.raw().tq_sdpa_int4_append_decode_paged
    pool = _cache(batch=64, capacity=256)
    wsb4 = tq.tq_workspace_bytes(4, 64, 128)
    def callp(**kw):
        a = dict(dict(tbl=FAKE, mb=8, k=FAKE, v=FAKE, lens=FAKE, S=2048, wsb=wsb4), **kw)
        return g(ctypes.byref(pool), a["tbl"], a["mb"], 4, a["k"], a["v"], FAKE, 64, a["lens"], a["S"], 0.1, FAKE, FAKE,
                 a["wsb"], None, None)
    assert callp(tbl=None) == E.TQ_ERR_NULL and callp(k=None) == E.TQ_ERR_NULL and callp(lens=None) == E.TQ_ERR_NULL
    assert callp(S=2049) == E.TQ_ERR_CAPACITY and callp(mb=0) == E.TQ_ERR_SHAPE
    assert callp(wsb=wsb4 - 1) == E.TQ_ERR_WORKSPACE and callp(v=FAKE + 4) == E.TQ_ERR_ALIGN


def test_measurement_probe_is_not_part_of_the_product_abi():
    """The read-bandwidth probe the benchmark times belongs to the bench (bench_probe.hip), not to the library."""
    lib = ctypes.CDLL(str(tq.library_path()))
    assert not hasattr(lib, "tq_probe_read_stream") and not hasattr(lib, "bench_probe_read_stream")
    assert "probe" not in (ROOT / "include" / "tq.h").read_text()


def test_binding_fails_loudly_when_library_is_missing(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "_LIB_PATH", tmp_path / "nope.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        B.raw()
