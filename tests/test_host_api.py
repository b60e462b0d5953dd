"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, sizes agree with the format description, and every argument error is caught
before the first HIP call."""
import ctypes as C
import os
import re

import pytest

import fmt

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def bpc():
    import paper_2105_07829_amd as bpc
    if not os.path.exists(bpc.LIB_PATH):
        bpc.build()
    bpc.lib()
    return bpc


def test_library_exports_every_declared_symbol(bpc):
    header = open(os.path.join(ROOT, "include", "bpc.h")).read()
    declared = set(re.findall(r"\b(bpc_[a-z_0-9]+)\s*\(", header))
    declared -= {n for n in declared if n.endswith("_t")}
    assert declared == set(bpc.EXPORTS)
    raw = C.CDLL(bpc.LIB_PATH)
    for name in declared:
        assert hasattr(raw, name), name


def test_sizes_follow_the_record_format(bpc):
    pe = 1 << 20
    assert bpc.partition_stride(bpc.make_params(bpc.SIGN, pe)) == fmt.stride("sign", pe)
    assert bpc.partition_stride(bpc.make_params(bpc.DITHER, pe)) == fmt.stride("dither", pe)
    assert bpc.partition_stride(bpc.make_params(bpc.NATDITHER, pe)) == fmt.stride("natdither", pe)
    for s in (7, 8, 15, 16, 31, 32, 63):     # 4, 5, 6 and 7 bits per element
        assert bpc.partition_stride(bpc.make_params(bpc.DITHER, pe, levels=s)) == fmt.stride("dither", pe, levels=s)
    assert bpc.partition_stride(bpc.make_params(bpc.IDENTITY, pe)) == fmt.stride("identity", pe)
    assert bpc.partition_stride(bpc.make_params(bpc.TOPK, pe, k_ratio=0.01)) == fmt.stride("topk", pe, 0.01)
    assert bpc.partition_stride(bpc.make_params(bpc.RANDK, pe, k_ratio=0.01)) == fmt.stride("randk", pe, 0.01)
    p = bpc.make_params(bpc.TOPK, pe, k_ratio=0.01)
    assert bpc.partition_k(p, pe) == 10485 and bpc.partition_k(p, 391_208) == 3912 and bpc.partition_k(p, 3) == 1
    assert bpc.payload_bytes(p, 25_557_032) == 25 * fmt.stride("topk", pe, 0.01)
    assert bpc.payload_bytes(p, 0) == 0
    assert bpc.workspace_bytes(p, 25_557_032, 8) >= 4 * 25_557_032


def test_sizes_agree_with_the_oracle(bpc, orc):
    for kind_b, kind_o, kw in [(bpc.SIGN, orc.SIGN, {}), (bpc.DITHER, orc.DITHER, {}),
                               (bpc.TOPK, orc.TOPK, dict(k_ratio=0.013)), (bpc.RANDK, orc.RANDK, dict(k_ratio=0.2)),
                               (bpc.IDENTITY, orc.IDENTITY, {})]:
        for pe in (1024, 5120, 1 << 20):
            pb, po = bpc.make_params(kind_b, pe, **kw), orc.make_params(kind_o, pe, **kw)
            assert bpc.partition_stride(pb) == orc.partition_stride(po)
            for D in (1, pe - 1, pe, 3 * pe + 17):
                assert bpc.payload_bytes(pb, D) == orc.payload_bytes(po, D)
                d_last = D - (D - 1) // pe * pe
                assert bpc.partition_k(pb, d_last) == orc.partition_k(po, d_last)


def test_invalid_params_are_rejected(bpc):
    bad = [bpc.make_params(bpc.SIGN, 0), bpc.make_params(bpc.SIGN, 1000), bpc.make_params(9, 1024),
           bpc.make_params(bpc.SIGN, (1 << 28) + 1024),
           bpc.make_params(bpc.TOPK, 1024, k_ratio=0.0), bpc.make_params(bpc.TOPK, 1024, k_ratio=1.5),
           bpc.make_params(bpc.RANDK, 1024, k_ratio=-1.0), bpc.make_params(bpc.DITHER, 1024, levels=0),
           bpc.make_params(bpc.DITHER, 1024, levels=64), bpc.make_params(bpc.NATDITHER, 1024, levels=8),
           bpc.make_params(bpc.DITHER, 1024, norm=5)]
    for p in bad:
        assert bpc.partition_stride(p) == 0
        assert bpc.payload_bytes(p, 4096) == 0
        assert bpc.workspace_bytes(p, 4096, 1) == 0
        st = bpc.lib().bpc_compress(C.byref(p), 0x1000, bpc.F32, None, 4096, 0x2000, 0x3000, 1 << 30, None)
        assert st == bpc.ERR_INVALID_ARG


def test_argument_errors_come_before_any_device_work(bpc):
    """Pointers below are fake addresses: every call must return before touching them."""
    L = bpc.lib()
    p = bpc.make_params(bpc.SIGN, 1024)
    D = 5000
    ws = bpc.workspace_bytes(p, D, 1)
    G, R, PL, WS = 0x10000, 0x20000, 0x30000, 0x40000
    assert L.bpc_compress(None, G, bpc.F32, R, D, PL, WS, ws, None) == bpc.ERR_INVALID_ARG
    assert L.bpc_compress(C.byref(p), None, bpc.F32, R, D, PL, WS, ws, None) == bpc.ERR_INVALID_ARG
    assert L.bpc_compress(C.byref(p), G, 7, R, D, PL, WS, ws, None) == bpc.ERR_INVALID_ARG
    assert L.bpc_compress(C.byref(p), G, bpc.F32, R, D, None, WS, ws, None) == bpc.ERR_INVALID_ARG
    assert L.bpc_compress(C.byref(p), G + 4, bpc.F32, R, D, PL, WS, ws, None) == bpc.ERR_ALIGNMENT
    assert L.bpc_compress(C.byref(p), G, bpc.F32, R + 8, D, PL, WS, ws, None) == bpc.ERR_ALIGNMENT
    assert L.bpc_compress(C.byref(p), G, bpc.F32, R, D, PL + 2, WS, ws, None) == bpc.ERR_ALIGNMENT
    assert L.bpc_compress(C.byref(p), G, bpc.F32, R, D, PL, WS, ws - 1, None) == bpc.ERR_WORKSPACE
    assert L.bpc_compress(C.byref(p), G, bpc.F32, R, D, PL, None, ws, None) == bpc.ERR_WORKSPACE
    assert L.bpc_compress(C.byref(p), G, bpc.F32, R, 0, PL, WS, ws, None) == bpc.OK   # empty gradient
    assert L.bpc_decompress(C.byref(p), None, D, R, None) == bpc.ERR_INVALID_ARG
    assert L.bpc_decompress(C.byref(p), PL, D, R + 4, None) == bpc.ERR_ALIGNMENT
    assert L.bpc_decompress(C.byref(p), PL, 0, R, None) == bpc.OK
    # aggregate
    n = 3
    arr = (bpc.Params * n)(*[p] * n)
    ptrs = (C.c_void_p * n)(PL, PL + 0x1000, PL + 0x2000)
    assert L.bpc_server_aggregate(arr, ptrs, 0, C.byref(p), R, D, PL, WS, ws, None) == bpc.ERR_INVALID_ARG
    assert L.bpc_server_aggregate(arr, ptrs, 65, C.byref(p), R, D, PL, WS, ws, None) == bpc.ERR_UNSUPPORTED
    assert L.bpc_server_aggregate(arr, None, n, C.byref(p), R, D, PL, WS, ws, None) == bpc.ERR_INVALID_ARG
    other = bpc.make_params(bpc.DITHER, 1024)
    assert L.bpc_server_aggregate(arr, ptrs, n, C.byref(other), R, D, PL, WS, 1 << 30, None) == bpc.ERR_INVALID_ARG
    ptrs_bad = (C.c_void_p * n)(PL, None, PL)
    assert L.bpc_server_aggregate(arr, ptrs_bad, n, C.byref(p), R, D, PL, WS, ws, None) == bpc.ERR_INVALID_ARG
    ptrs_mis = (C.c_void_p * n)(PL, PL + 4, PL)
    assert L.bpc_server_aggregate(arr, ptrs_mis, n, C.byref(p), R, D, PL, WS, ws, None) == bpc.ERR_ALIGNMENT
    assert L.bpc_server_aggregate(arr, ptrs, n, C.byref(p), R, D, PL, WS, 16, None) == bpc.ERR_WORKSPACE
    assert L.bpc_server_aggregate(arr, ptrs, n, C.byref(p), R, 0, PL, WS, ws, None) == bpc.OK
    # update
    o = bpc.make_opt(bpc.OPT_ADAM, 1e-3, 0.9, 0.999, 1e-8, 0.01, 1)
    X, M, V = 0x50000, 0x60000, 0x70000
    assert L.bpc_adaptive_update(C.byref(p), PL, D, X, M, V, None, WS, ws, None) == bpc.ERR_INVALID_ARG
    assert L.bpc_adaptive_update(C.byref(p), PL, D, None, M, V, C.byref(o), WS, ws, None) == bpc.ERR_INVALID_ARG
    assert L.bpc_adaptive_update(C.byref(p), PL, D, X, M + 4, V, C.byref(o), WS, ws, None) == bpc.ERR_ALIGNMENT
    assert L.bpc_adaptive_update(C.byref(p), PL, D, X, M, V, C.byref(o), WS, 8, None) == bpc.ERR_WORKSPACE
    bad = bpc.make_opt(bpc.OPT_ADAM, 1e-3, 1.0, 0.999, 1e-8, 0.0, 1)
    assert L.bpc_adaptive_update(C.byref(p), PL, D, X, M, V, C.byref(bad), WS, ws, None) == bpc.ERR_INVALID_ARG
    bad = bpc.make_opt(5, 1e-3, 0.9, 0.999, 1e-8, 0.0, 1)
    assert L.bpc_adaptive_update(C.byref(p), PL, D, X, M, V, C.byref(bad), WS, ws, None) == bpc.ERR_INVALID_ARG
    assert L.bpc_adaptive_update(C.byref(p), PL, 0, X, M, V, C.byref(o), WS, ws, None) == bpc.OK


def test_update_workspace_covers_more_blocks_than_partitions(bpc):
    """LANS blocks are layers: a gradient has far more of them than partitions.  The sizing call
    must then ask for more than the common workspace, and the update must refuse anything less."""
    L = bpc.lib()
    p = bpc.make_params(bpc.SIGN, 1 << 20)
    D = 3 * (1 << 20) + 5
    common = bpc.workspace_bytes(p, D, 1)
    assert bpc.update_workspace_bytes(p, D, 0) == common
    few = bpc.update_workspace_bytes(p, D, 2)
    many = 400
    need = bpc.update_workspace_bytes(p, D, many)
    # per block: its totals and a counter; per tile of 8192 elements: two slots of three sums
    assert common <= few < need and need >= common + 20 * many + 48 * (D // 8192)
    assert need % 256 == 0
    o = bpc.make_opt(bpc.OPT_LANS, 1e-3, 0.9, 0.999, 1e-8, 0.01, 1)
    o.block_offsets, o.n_blocks = 0x80000, many          # fake device address: never dereferenced here
    PL, WS, X, M, V = 0x30000, 0x40000, 0x50000, 0x60000, 0x70000
    assert L.bpc_adaptive_update(C.byref(p), PL, D, X, M, V, C.byref(o), WS, common, None) == bpc.ERR_WORKSPACE
    assert L.bpc_adaptive_update(C.byref(p), PL, D, X, M, V, C.byref(o), WS, need - 1, None) == bpc.ERR_WORKSPACE
    assert bpc.update_workspace_bytes(bpc.make_params(bpc.SIGN, 1000), D, 3) == 0


def test_sparse_kinds_refuse_more_partitions_than_a_grid_dimension_holds(bpc):
    """Some top-k / random-k launches carry the partition number in the second grid dimension
    (at most 65535): such a shape is refused before anything is enqueued."""
    L = bpc.lib()
    G, R, PL, WS = 0x10000, 0x20000, 0x30000, 0x40000
    D = 65536 * 1024
    for kind in (bpc.TOPK, bpc.TOPK16, bpc.RANDK):
        p = bpc.make_params(kind, 1024, k_ratio=0.01)
        assert L.bpc_compress(C.byref(p), G, bpc.F32, R, D, PL, WS, 1 << 40, None) == bpc.ERR_UNSUPPORTED
        assert L.bpc_decompress(C.byref(p), PL, D, R, None) == bpc.ERR_UNSUPPORTED
        arr = (bpc.Params * 1)(p)
        ptrs = (C.c_void_p * 1)(PL)
        assert L.bpc_server_aggregate(arr, ptrs, 1, C.byref(p), R, D, PL, WS, 1 << 40, None) == bpc.ERR_UNSUPPORTED
        o = bpc.make_opt(bpc.OPT_ADAM, 1e-3, 0.9, 0.999, 1e-8, 0.01, 1)
        assert L.bpc_adaptive_update(C.byref(p), PL, D, R, R, R, C.byref(o), WS, 1 << 40, None) == bpc.ERR_UNSUPPORTED


def test_workspace_check_validates_its_arguments(bpc):
    L = bpc.lib()
    assert L.bpc_workspace_check(None, 100, 0x1000, None) == bpc.ERR_INVALID_ARG
    # no workspace pointer = the library's static one, which is too small for this shape
    p = bpc.make_params(bpc.TOPK, 1 << 20, k_ratio=0.01)
    assert L.bpc_workspace_check(C.byref(p), 1 << 24, None, None) == bpc.ERR_WORKSPACE


def test_static_workspace_entry_point_validates_before_any_device_work(bpc):
    """bpc_compress_static_ws: the argument checks of bpc_compress, then the size limit, all on
    the host (fake pointers below)."""
    L = bpc.lib()
    G, R, PL = 0x10000, 0x20000, 0x30000
    p = bpc.make_params(bpc.SIGN, 1 << 20)
    f = L.bpc_compress_static_ws
    assert f(None, G, bpc.F32, R, 4096, PL, None) == bpc.ERR_INVALID_ARG
    assert f(C.byref(p), None, bpc.F32, R, 4096, PL, None) == bpc.ERR_INVALID_ARG
    assert f(C.byref(p), G, 5, R, 4096, PL, None) == bpc.ERR_INVALID_ARG
    assert f(C.byref(p), G, bpc.F32, R, 4096, None, None) == bpc.ERR_INVALID_ARG
    assert f(C.byref(p), G + 8, bpc.F32, R, 4096, PL, None) == bpc.ERR_ALIGNMENT
    assert f(C.byref(p), G, bpc.F32, R, 0, PL, None) == bpc.OK
    # beyond the static array: refused, and the limit is where the sizing call says it is
    big = 1 << 31
    assert bpc.workspace_bytes(p, big, 1) > bpc.STATIC_WS_BYTES
    assert f(C.byref(p), G, bpc.F32, R, big, PL, None) == bpc.ERR_WORKSPACE
    t = bpc.make_params(bpc.TOPK, 1 << 20, k_ratio=0.01)
    assert bpc.workspace_bytes(t, 1 << 21, 1) > bpc.STATIC_WS_BYTES
    assert f(C.byref(t), G, bpc.F32, R, 1 << 21, PL, None) == bpc.ERR_WORKSPACE
    header = open(os.path.join(ROOT, "include", "bpc.h")).read()
    assert re.search(r"#define\s+BPC_STATIC_WS_BYTES\s+\(4u << 20\)", header) and bpc.STATIC_WS_BYTES == 4 << 20
    # the shapes the header names as covered do fit
    for kind, D in ((bpc.SIGN, 800_000_000), (bpc.DITHER, 800_000_000), (bpc.TOPK, 500_000)):
        q = bpc.make_params(kind, 1 << 21 if kind != bpc.TOPK else 1 << 20, k_ratio=0.01)
        assert bpc.workspace_bytes(q, D, 1) <= bpc.STATIC_WS_BYTES, (kind, D)


def test_bypass_mask_sizes_and_limits(bpc, orc):
    """Partitions under the size threshold travel as identity records: record offsets and the
    payload size follow from the mask (and agree with the oracle's record sizes); more than 64
    runs of one class are refused; the masks of one server call must mark the same partitions."""
    import numpy as np
    L = bpc.lib()
    pe = 1024
    D = 6 * pe + 100
    mask = np.array([0, 1, 1, 0, 1, 0, 1], dtype=np.uint8)
    for kind_b, kind_o, kw in [(bpc.SIGN, orc.SIGN, {}), (bpc.TOPK, orc.TOPK, dict(k_ratio=0.05)),
                               (bpc.DITHER, orc.DITHER, dict(levels=15))]:
        plain = bpc.make_params(kind_b, pe, **kw)
        p = bpc.make_params(kind_b, pe, bypass=mask, **kw)
        sizes = orc.record_sizes_bypass(orc.make_params(kind_o, pe, **kw), mask, D)
        ident = bpc.partition_stride(bpc.make_params(bpc.IDENTITY, pe))
        assert sizes == [ident if b else bpc.partition_stride(plain) for b in mask]
        offs = np.concatenate([[0], np.cumsum(sizes)])
        assert bpc.payload_bytes(p, D) == offs[-1]
        for k in range(7):
            assert bpc.partition_offset(p, D, k) == offs[k]
            assert bpc.partition_offset(plain, D, k) == k * bpc.partition_stride(plain)
        assert bpc.partition_offset(p, D, 7) == 2 ** 64 - 1            # no such partition
        # a mask of zeros is no mask
        zeros = bpc.make_params(kind_b, pe, bypass=np.zeros(7, np.uint8), **kw)
        assert bpc.payload_bytes(zeros, D) == bpc.payload_bytes(plain, D)
    # 65 runs: refused by every entry point before any device work
    many = np.arange(65, dtype=np.uint8) & 1
    p = bpc.make_params(bpc.SIGN, pe, bypass=many)
    D2 = 65 * pe
    assert bpc.payload_bytes(p, D2) == 0 and bpc.partition_offset(p, D2, 0) == 2 ** 64 - 1
    G, R, PL, WS = 0x10000, 0x20000, 0x30000, 0x40000
    assert L.bpc_compress(C.byref(p), G, bpc.F32, R, D2, PL, WS, 1 << 30, None) == bpc.ERR_UNSUPPORTED
    assert L.bpc_decompress(C.byref(p), PL, D2, R, None) == bpc.ERR_UNSUPPORTED
    o = bpc.make_opt(bpc.OPT_ADAM, 1e-3, 0.9, 0.999, 1e-8, 0.01, 1)
    assert L.bpc_adaptive_update(C.byref(p), PL, D2, R, R, R, C.byref(o), WS, 1 << 30, None) == bpc.ERR_UNSUPPORTED
    ok64 = bpc.make_params(bpc.SIGN, pe, bypass=np.arange(64, dtype=np.uint8) & 1)
    assert bpc.payload_bytes(ok64, 64 * pe) > 0
    # server: every worker's mask must mark the partitions the outgoing one marks
    a = bpc.make_params(bpc.SIGN, pe, bypass=mask)
    b = bpc.make_params(bpc.SIGN, pe, bypass=np.array([0, 1, 1, 0, 0, 0, 1], dtype=np.uint8))
    c = bpc.make_params(bpc.SIGN, pe)
    ptrs = (C.c_void_p * 2)(PL, PL + 0x100000)
    for pair in ((a, b), (a, c)):
        arr = (bpc.Params * 2)(*pair)
        assert L.bpc_server_aggregate(arr, ptrs, 2, C.byref(a), R, D, PL, WS, 1 << 30, None) == bpc.ERR_INVALID_ARG
    # LANS with caller-defined blocks takes no mask with more than one run
    lo = bpc.make_opt(bpc.OPT_LANS, 1e-3, 0.9, 0.999, 1e-8, 0.01, 1)
    lo.block_offsets, lo.n_blocks = 0x80000, 3
    assert L.bpc_adaptive_update(C.byref(a), PL, D, R, R, R, C.byref(lo), WS, 1 << 30, None) == bpc.ERR_UNSUPPORTED


def test_status_strings(bpc):
    L = bpc.lib()
    seen = {L.bpc_status_string(i).decode() for i in range(7)}
    assert len(seen) == 7 and "ok" in seen
    assert L.bpc_status_string(99).decode() == "unknown status"
    assert L.bpc_last_hip_error() == 0


def test_missing_library_fails_loudly(monkeypatch):
    import paper_2105_07829_amd as bpc
    monkeypatch.setattr(bpc, "_lib", None)
    monkeypatch.setattr(bpc, "LIB_PATH", "/nonexistent/libbpc.so")
    with pytest.raises(ImportError):
        bpc.lib()
