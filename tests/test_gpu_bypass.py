"""GPU parity of calls whose partitions partly bypass compression (the size threshold of
Section 4.2): a masked partition is carried as an identity record with a zero residual, the
others go through the compressor, records follow each other at the offsets the mask fixes.
Every stage against the oracle's partition-by-partition form on the same inputs."""
import numpy as np
import pytest

import fmt

pytestmark = pytest.mark.gpu

REL = 1e-6

KW = {
    "sign": {},
    "topk": dict(k_ratio=0.01),
    "topk16": dict(k_ratio=0.013),
    "randk": dict(k_ratio=0.02, value_scale=1.0, seed=0x1234567890ABCDEF, stream_id=(2 << 32) | 5),
    "dither": dict(levels=4, seed=0xFEEDFACECAFEBEEF, stream_id=(7 << 32) | 1),
    "dither_5bit": dict(levels=15, seed=0xC0FFEE, stream_id=(5 << 32) | 3),
    "natdither": dict(levels=5, seed=0xABCDEF, stream_id=(3 << 32) | 2),
    "fp16": {},
}
# (partition size, elements, mask): partitions of two tiles with a ragged last one that is
# compressed; partitions of several register-resident tiles with a ragged bypassed tail; one run
# of each class only; everything bypassed
CASES = [
    (8192, 5 * 8192 + 321, [0, 1, 1, 0, 1, 0]),
    (131072, 3 * 131072 + 70000, [1, 0, 0, 1]),
    (8192, 3 * 8192, [0, 0, 1]),
    (8192, 2 * 8192 + 5, [1, 1, 1]),
]


@pytest.fixture(scope="module")
def gu():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import gpu_util
    gpu_util.bpc.lib()
    return gpu_util


def rng(seed):
    return np.random.default_rng(seed)


def base_kind(name):
    return name.split("_")[0]


def both(gu, orc, name, pe, mask, **over):
    kw = dict(KW[name])
    kw.update(over)
    return gu.both_params(orc, base_kind(name), pe, bypass=np.asarray(mask, np.uint8), **kw)


def headers(pay, offs, mask):
    """Header word 0 of every record as f32 (the scale of a sign / dithering record)."""
    return np.array([fmt.header_f32(pay[offs[k]:offs[k] + 16]) for k in range(len(mask))], dtype=np.float32)


def compare_records(name, pe, D, mask, offs, pay_gpu, pay_ref):
    kind = base_kind(name)
    assert pay_gpu.size == pay_ref.size == offs[-1]
    k_cap = fmt.k_of(KW[name].get("k_ratio", 0.0), pe) if kind in ("topk", "topk16", "randk") else 0
    for k, d in enumerate(fmt.part_sizes(D, pe)):
        rg, rr = pay_gpu[offs[k]:offs[k + 1]], pay_ref[offs[k]:offs[k + 1]]
        if mask[k]:
            ranges = fmt.defined_bytes("identity", d)
        else:
            kk = fmt.k_of(KW[name]["k_ratio"], d) if k_cap else 0
            ranges = fmt.defined_bytes(kind, d, kk, k_cap, part_elems=pe, levels=KW[name].get("levels", 4))
        for lo, hi in ranges:
            assert np.array_equal(rg[lo:hi], rr[lo:hi]), (name, "partition", k, "bytes", lo, hi)


def with_gpu_scales(name, mask, offs, pay_gpu, pay_ref, redo):
    """Scales within tolerance; if one differs in its last bit the oracle is re-run with the
    card's, so that every packed bit is decided on equal terms."""
    if base_kind(name) not in ("sign", "dither", "natdither"):
        return pay_ref
    hg, hr = headers(pay_gpu, offs, mask), headers(pay_ref, offs, mask)
    live = np.array(mask) == 0
    assert np.all(np.abs(hg[live].astype(np.float64) - hr[live]) <= REL * np.abs(hr[live]))
    if not np.array_equal(hg[live], hr[live]):
        return redo(np.where(live, hg, 0).astype(np.float32))
    return pay_ref


@pytest.mark.parametrize("name", sorted(KW))
@pytest.mark.parametrize("case", range(len(CASES)))
def test_masked_pipeline(gu, orc, name, case):
    """Workers (f16 and f32 gradients, error feedback), server, decompress, Adam-style and LANS
    update with the same mask on every call."""
    import torch
    bpc = gu.bpc
    pe, D, mask = CASES[case]
    n = 3
    kind = base_kind(name)
    sizes = None
    pays_ref, pays_gpu, ins = [], [], []
    for i in range(n):
        over = {"stream_id": (1 << 32) | i} if "stream_id" in KW[name] else {}
        po, pb = both(gu, orc, name, pe, mask, **over)
        ins.append((po, pb))
        if sizes is None:
            sizes = orc.record_sizes_bypass(po, mask, D)
            offs = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
            assert bpc.payload_bytes(pb, D) == offs[-1]
        dt = np.float16 if i % 2 else np.float32
        g = (rng(40 + i).standard_t(3.0, D) * 1e-3).astype(dt)
        e = (rng(50 + i).standard_normal(D) * 3e-4).astype(np.float32)
        res_ref = e.copy()
        pay_ref = orc.compress_bypass(po, mask, g, res_ref)
        # the library's call
        gd, rd = gu.to_dev(g), gu.to_dev(e)
        pay = gu.new_payload(pb, D)
        ws = gu.new_ws(pb, D)
        bpc.bpc_compress(pb, gd, rd, pay, ws)
        bpc.workspace_check(pb, D, ws)
        pay_gpu, res_gpu = gu.to_host(pay)[:offs[-1]], gu.to_host(rd)

        def redo(norms, po=po, g=g, e=e, res_ref=res_ref):
            po2, _ = both(gu, orc, name, pe, mask, norm_override=norms, **over)
            r2 = e.copy()
            out = orc.compress_bypass(po2, mask, g, r2)
            res_ref[:] = r2
            return out

        pay_ref = with_gpu_scales(name, mask, offs, pay_gpu, pay_ref, redo)
        compare_records(name, pe, D, mask, offs, pay_gpu, pay_ref)
        for k, d in enumerate(fmt.part_sizes(D, pe)):
            lo = k * pe
            if mask[k]:
                assert not res_gpu[lo:lo + d].any(), (name, "residual of a bypassed partition", k)
            elif kind in ("topk", "topk16", "fp16"):
                assert np.array_equal(res_gpu[lo:lo + d].view(np.uint32), res_ref[lo:lo + d].view(np.uint32))
        assert gu.close(res_gpu, res_ref, REL), name
        pays_ref.append(pay_ref)
        pays_gpu.append(pay_gpu)

    # server: the oracle's messages in, so that both sides start from identical bytes
    over = {"stream_id": (1 << 32) | (1 << 16)} if "stream_id" in KW[name] else {}
    out_o, out_b = both(gu, orc, name, pe, mask, **over)
    et = (rng(77).standard_normal(D) * 2e-4).astype(np.float32)
    res_ref = et.copy()
    p_ref = orc.server_aggregate_bypass([p[0] for p in ins], pays_ref, out_o, mask, res_ref, D)
    pls = [gu.to_dev(p) for p in pays_ref]
    rd = gu.to_dev(et)
    out_pl = gu.new_payload(out_b, D)
    ws = gu.new_ws(out_b, D, n)
    bpc.bpc_server_aggregate([p[1] for p in ins], pls, out_b, rd, D, out_pl, ws)
    bpc.workspace_check(out_b, D, ws)
    p_gpu, res_gpu = gu.to_host(out_pl)[:offs[-1]], gu.to_host(rd)

    def redo_server(norms):
        o2, _ = both(gu, orc, name, pe, mask, norm_override=norms, **over)
        r2 = et.copy()
        out = orc.server_aggregate_bypass([p[0] for p in ins], pays_ref, o2, mask, r2, D)
        res_ref[:] = r2
        return out

    p_ref = with_gpu_scales(name, mask, offs, p_gpu, p_ref, redo_server)
    if kind == "randk":
        # Delta passes through float atomics whose order is free: values at the tolerance
        for k, d in enumerate(fmt.part_sizes(D, pe)):
            rg, rr = p_gpu[offs[k]:offs[k + 1]], p_ref[offs[k]:offs[k + 1]]
            if mask[k]:
                assert np.array_equal(rg[:16 + 4 * d], rr[:16 + 4 * d])
            else:
                kg, vg = fmt.randk_values(rg)
                kr, vr = fmt.randk_values(rr)
                assert kg == kr and gu.close(vg, vr, REL)
    else:
        compare_records(name, pe, D, mask, offs, p_gpu, p_ref)
    for k, d in enumerate(fmt.part_sizes(D, pe)):
        if mask[k]:
            assert not res_gpu[k * pe:k * pe + d].any()
    assert gu.close(res_gpu, res_ref, REL), name

    # decompress and update read the oracle's outgoing message
    dec_ref = orc.decompress_bypass(out_o, mask, p_ref, D)
    out = torch.full((D,), 7.0, dtype=torch.float32, device=gu.DEV)
    bpc.bpc_decompress(out_b, gu.to_dev(p_ref), out)
    assert np.array_equal(gu.to_host(out).view(np.uint32), dec_ref.view(np.uint32)), name

    x0 = (rng(1).standard_normal(D) * 0.02).astype(np.float32)
    m0 = (rng(2).standard_normal(D) * 1e-3).astype(np.float32)
    v0 = (rng(3).random(D) * 1e-5).astype(np.float32)
    for opt_kind in ("adam", "lans"):
        ko = orc.OPT_ADAM if opt_kind == "adam" else orc.OPT_LANS
        kb = bpc.OPT_ADAM if opt_kind == "adam" else bpc.OPT_LANS
        lr = 1e-3 if opt_kind == "adam" else 0.5
        oo = orc.make_opt(ko, lr, 0.9, 0.999, 1e-8, 0.01, 3)
        ob = bpc.make_opt(kb, lr, 0.9, 0.999, 1e-8, 0.01, 3)
        x, m, v = x0.copy(), m0.copy(), v0.copy()
        orc.adaptive_update_bypass(out_o, mask, p_ref, D, x, m, v, oo)
        xg, mg, vg = gu.gpu_update(out_b, p_ref, x0, m0, v0, ob)
        assert np.array_equal(mg.view(np.uint32), m.view(np.uint32)), (name, opt_kind)
        assert np.array_equal(vg.view(np.uint32), v.view(np.uint32)), (name, opt_kind)
        if opt_kind == "adam":
            assert np.array_equal(xg.view(np.uint32), x.view(np.uint32)), name
        else:
            blocks = np.array(sorted(set(range(0, D, pe)) | {D}))
            assert gu.lans_step_close(xg, x, x0, blocks), name
