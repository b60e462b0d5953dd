"""bpc_compress_static_ws (the entry point for callers that cannot allocate device memory)
against bpc_compress on a caller-owned workspace: same kernels, so every byte of the message
and of the residual must be equal.  Two calls in a row share the library's static device array,
the second on a smaller input, so whatever the first call left there must not leak into the
second."""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2105_07829_amd as bpc
    bpc.lib()
    return bpc


def _inputs(D, dtype, seed):
    rng = np.random.default_rng(seed)
    g = (rng.standard_t(3.0, D) * 1e-3).astype(np.float16 if dtype == "f16" else np.float32)
    e = (rng.standard_normal(D) * 1e-4).astype(np.float32)
    return g, e


def _both_ways(bpc, prm, g_np, e_np, use_ef):
    """(payload, residual) from bpc_compress and from bpc_compress_static_ws, as numpy arrays."""
    L = bpc.lib()
    D = g_np.size
    code = bpc.F16 if g_np.dtype == np.float16 else bpc.F32
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    nbytes = bpc.payload_bytes(prm, D)
    out = []
    for static in (False, True):
        g = torch.from_numpy(g_np).cuda()
        e = torch.from_numpy(e_np.copy()).cuda() if use_ef else None
        pay = torch.full((nbytes,), 0xA5, dtype=torch.uint8, device="cuda")
        e_ptr = C.c_void_p(e.data_ptr()) if use_ef else None
        if static:
            st = L.bpc_compress_static_ws(C.byref(prm), C.c_void_p(g.data_ptr()), code, e_ptr, D,
                                          C.c_void_p(pay.data_ptr()), stream)
            assert st == bpc.OK, L.bpc_status_string(st)
            assert L.bpc_workspace_check(C.byref(prm), D, None, stream) == bpc.OK
        else:
            ws = torch.empty(bpc.workspace_bytes(prm, D, 1), dtype=torch.uint8, device="cuda")
            st = L.bpc_compress(C.byref(prm), C.c_void_p(g.data_ptr()), code, e_ptr, D, C.c_void_p(pay.data_ptr()),
                                C.c_void_p(ws.data_ptr()), ws.numel(), stream)
            assert st == bpc.OK, L.bpc_status_string(st)
            assert L.bpc_workspace_check(C.byref(prm), D, C.c_void_p(ws.data_ptr()), stream) == bpc.OK
        torch.cuda.synchronize()
        out.append((pay.cpu().numpy(), e.cpu().numpy() if use_ef else None))
    return out


CASES = [
    # kind, keyword arguments, partition elements, dtype, first D, second (smaller) D
    ("sign", {}, 16384 * 4, "f16", 16384 * 4 * 5 + 16384 + 1234, 16384 * 4 + 16384 * 2),
    ("sign", {}, 16384, "f32", 16384 * 9 + 77, 4097),
    ("dither", dict(levels=4, seed=11, stream_id=(3 << 32) | 5), 16384 * 2, "f16", 16384 * 2 * 6 + 4100, 16384 * 3),
    ("natdither", dict(levels=3, seed=5, stream_id=9), 16384, "f32", 16384 * 3 + 1, 1000),
    ("dither", dict(levels=15, seed=2, stream_id=1), 16384, "f32", 16384 * 4 + 999, 16384 + 5),
    ("topk", dict(k_ratio=0.01), 65536, "f32", 65536 * 5 + 4321, 65536 + 100),
    ("randk", dict(k_ratio=0.02, seed=8, stream_id=77, value_scale=-1.0), 32768, "f32", 32768 * 7 + 3, 9000),
    ("fp16", {}, 8192, "f32", 8192 * 3 + 17, 100),
    ("identity", {}, 8192, "f16", 8192 * 2 + 18, 8192),
]


@pytest.mark.parametrize("kind,kw,pe,dtype,d_first,d_second", CASES,
                         ids=[f"{c[0]}-{c[3]}-{i}" for i, c in enumerate(CASES)])
def test_static_workspace_matches_caller_workspace_twice_in_a_row(kind, kw, pe, dtype, d_first, d_second):
    bpc = _gpu()
    code = {"sign": bpc.SIGN, "dither": bpc.DITHER, "natdither": bpc.NATDITHER, "topk": bpc.TOPK,
            "randk": bpc.RANDK, "fp16": bpc.FP16, "identity": bpc.IDENTITY}[kind]
    prm = bpc.make_params(code, pe, **kw)
    assert d_second < d_first
    for call, D in enumerate((d_first, d_second)):
        assert bpc.workspace_bytes(prm, D, 1) <= bpc.STATIC_WS_BYTES
        g, e = _inputs(D, dtype, seed=100 * call + len(kind))
        (pay_ws, res_ws), (pay_st, res_st) = _both_ways(bpc, prm, g, e, use_ef=True)
        assert np.array_equal(pay_ws, pay_st), f"{kind}: message differs on call {call} (D = {D})"
        assert np.array_equal(res_ws.view(np.uint32), res_st.view(np.uint32)), f"{kind}: residual differs on call {call}"
    # and without error feedback (residual pointer NULL), on the smaller input again
    g, e = _inputs(d_second, dtype, seed=7)
    (pay_ws, _), (pay_st, _) = _both_ways(bpc, prm, g, e, use_ef=False)
    assert np.array_equal(pay_ws, pay_st)


def test_static_workspace_refuses_what_does_not_fit():
    bpc = _gpu()
    L = bpc.lib()
    prm = bpc.make_params(bpc.TOPK, 1 << 20, k_ratio=0.01)
    D = 1 << 22
    assert bpc.workspace_bytes(prm, D, 1) > bpc.STATIC_WS_BYTES
    g = torch.zeros(D, dtype=torch.float32, device="cuda")
    e = torch.ones(D, dtype=torch.float32, device="cuda")
    pay = torch.full((bpc.payload_bytes(prm, D),), 0xA5, dtype=torch.uint8, device="cuda")
    st = L.bpc_compress_static_ws(C.byref(prm), C.c_void_p(g.data_ptr()), bpc.F32, C.c_void_p(e.data_ptr()), D,
                                  C.c_void_p(pay.data_ptr()), None)
    assert st == bpc.ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((e == 1).all()) and bool((pay == 0xA5).all())      # nothing was touched


def test_static_workspace_at_a_bert_base_sized_sign_call():
    """The full BERT-base shape (110 M half-precision elements, scaled sign) fits the static array."""
    bpc = _gpu()
    D, pe = 110_000_000, 1 << 21
    prm = bpc.make_params(bpc.SIGN, pe)
    assert bpc.workspace_bytes(prm, D, 1) <= bpc.STATIC_WS_BYTES
    gen = torch.Generator(device="cuda").manual_seed(5)
    g = (torch.randn(D, device="cuda", generator=gen) * 1e-3).to(torch.float16)
    e0 = torch.randn(D, device="cuda", generator=gen) * 1e-4
    outs = []
    for static in (False, True):
        e = e0.clone()
        pay = torch.zeros(bpc.payload_bytes(prm, D), dtype=torch.uint8, device="cuda")
        if static:
            bpc.bpc_compress_static_ws(prm, g, e, pay)
            bpc.workspace_check(prm, D, None)
        else:
            ws = torch.empty(bpc.workspace_bytes(prm, D, 1), dtype=torch.uint8, device="cuda")
            bpc.bpc_compress(prm, g, e, pay, ws)
            bpc.workspace_check(prm, D, ws)
        outs.append((pay, e))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1].view(torch.int32), outs[1][1].view(torch.int32))
