"""GPU parity at the full sizes and in the launch configuration that bench.py times.

For each workload of the benchmark spec the whole pipeline runs on the GPU (n workers with non-zero
residuals, server aggregate, update) on seeded synthetic gradients generated on the card.
Partitions are independent units of the method, so the oracle recomputes a sample of them
(first, a middle one, the ragged last one) from exactly the bytes the GPU consumed: the
gradient / residual slices for the worker stage, the GPU's own n worker records for the
server stage, the GPU's own pulled record for the update.  Same bars as the small tests.
"""
import numpy as np
import pytest

import fmt

pytestmark = pytest.mark.gpu

REL = 1e-6


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available()
    import gpu_util
    import synth
    gpu_util.bpc.lib()
    return gpu_util, synth, torch


def sample_partitions(P):
    return sorted({0, P // 2, P - 1})


def record_equal(kind, rec_g, rec_o, d, k, k_cap, pe=0, levels=4):
    for lo, hi in fmt.defined_bytes(kind, d, k, k_cap, part_elems=pe, levels=levels):
        if not np.array_equal(rec_g[lo:hi], rec_o[lo:hi]):
            return False
    return True


@pytest.mark.parametrize("name", ["sign_1m", "resnet50", "vgg16", "bert_base", "bert_large", "bert_large_natural",
                                  "bert_large_5bit", "bert_large_fp16", "bert_base_topk16"])
def test_full_size_pipeline(env, orc, name):
    gu, synth, torch = env
    bpc = gu.bpc
    w = synth.WORKLOADS[name]
    D, n, kind = w["D"], w["n_workers"], w["kind"]
    pe = synth.part_elems(w["dtype"])
    P = (D + pe - 1) // pe
    kw = dict(k_ratio=w.get("k_ratio", 0.01), levels=w.get("levels", 4), value_scale=w.get("value_scale", 1.0),
              seed=synth.BASE_SEED)
    kind_o = {"sign": orc.SIGN, "topk": orc.TOPK, "randk": orc.RANDK, "dither": orc.DITHER,
              "natdither": orc.NATDITHER, "fp16": orc.FP16, "topk16": orc.TOPK16}[kind]
    kind_b = gu.KIND_B[kind]
    k_cap = fmt.k_of(kw["k_ratio"], pe) if kind in ("topk", "topk16", "randk") else 0
    dev = gu.DEV

    def prm_b(stream):
        return bpc.make_params(kind_b, pe, stream_id=stream, **kw)

    def prm_o(stream, part, norm=None):
        return orc.make_params(kind_o, pe, stream_id=stream, first_partition=part,
                               norm_override=None if norm is None else np.array([norm], np.float32), **kw)

    p0 = prm_b(0)
    strd = bpc.partition_stride(p0)
    ws = torch.zeros(bpc.workspace_bytes(p0, D, n), dtype=torch.uint8, device=dev)
    parts = sample_partitions(P)

    def sl(p):
        return slice(p * pe, min(D, (p + 1) * pe))

    # ---------------- worker stage, every worker on the GPU, worker 0 checked
    pays = []
    for i in range(n):
        g = synth.device_gradient(w["dist"], D, w["dtype"], worker=i, device=dev)
        e = synth.device_gradient("normal", D, "f32", worker=100 + i, device=dev) * 0.3
        if i == 0:
            g_host = {p: g[sl(p)].cpu().numpy() for p in parts}
            e_host = {p: e[sl(p)].cpu().numpy() for p in parts}
        pay = torch.zeros(bpc.payload_bytes(p0, D), dtype=torch.uint8, device=dev)
        bpc.bpc_compress(prm_b((1 << 32) | i), g, e, pay, ws)
        pays.append(pay)
        if i == 0:
            e_after = {p: e[sl(p)].cpu().numpy() for p in parts}
        del g, e
    torch.cuda.synchronize()
    assert bpc.workspace_status(p0, D, ws) == 0
    for p in parts:
        d = sl(p).stop - sl(p).start
        k = fmt.k_of(kw["k_ratio"], d) if k_cap else 0
        rec_g = pays[0][p * strd:(p + 1) * strd].cpu().numpy()
        res_o = e_host[p].copy()
        rec_o = orc.compress(prm_o((1 << 32) | 0, p), g_host[p], res_o)
        if kind in ("sign", "dither", "natdither"):
            hg, ho = fmt.header_f32(rec_g), fmt.header_f32(rec_o)
            assert abs(float(hg) - float(ho)) <= REL * abs(float(ho))
            if hg != ho:       # packed bits on equal terms: oracle with the GPU's scale
                res_o = e_host[p].copy()
                rec_o = orc.compress(prm_o((1 << 32) | 0, p, norm=hg), g_host[p], res_o)
        assert record_equal(kind, rec_g, rec_o, d, k, k_cap, pe, kw["levels"]), (name, "worker", p)
        if kind in ("topk", "topk16", "fp16"):
            assert np.array_equal(e_after[p].view(np.uint32), res_o.view(np.uint32))
        else:
            assert gu.close(e_after[p], res_o, REL), (name, "worker residual", p)

    # ---------------- server stage on the GPU's own worker messages
    sres = synth.device_gradient("normal", D, "f32", worker=999, device=dev) * 0.2
    s_host = {p: sres[sl(p)].cpu().numpy() for p in parts}
    out_pay = torch.zeros(bpc.payload_bytes(p0, D), dtype=torch.uint8, device=dev)
    ins_b = [prm_b((1 << 32) | i) for i in range(n)]
    out_stream = (1 << 32) | (1 << 16)
    bpc.bpc_server_aggregate(ins_b, pays, prm_b(out_stream), sres, D, out_pay, ws)
    torch.cuda.synchronize()
    assert bpc.workspace_status(p0, D, ws) == 0
    for p in parts:
        d = sl(p).stop - sl(p).start
        k = fmt.k_of(kw["k_ratio"], d) if k_cap else 0
        recs = [pays[i][p * strd:(p + 1) * strd].cpu().numpy() for i in range(n)]
        ins_o = [prm_o((1 << 32) | i, p) for i in range(n)]
        rec_g = out_pay[p * strd:(p + 1) * strd].cpu().numpy()
        res_o = s_host[p].copy()
        rec_o = orc.server_aggregate(ins_o, recs, prm_o(out_stream, p), res_o, d)
        if kind in ("sign", "dither", "natdither"):
            hg, ho = fmt.header_f32(rec_g), fmt.header_f32(rec_o)
            assert abs(float(hg) - float(ho)) <= REL * abs(float(ho))
            if hg != ho:
                res_o = s_host[p].copy()
                rec_o = orc.server_aggregate(ins_o, recs, prm_o(out_stream, p, norm=hg), res_o, d)
        if kind == "randk":      # values of Delta come through float atomics: tolerance
            kg, vg = fmt.randk_values(rec_g)
            ko, vo = fmt.randk_values(rec_o)
            assert kg == ko and gu.close(vg, vo, REL)
        else:
            assert record_equal(kind, rec_g, rec_o, d, k, k_cap, pe, kw["levels"]), (name, "server", p)
        got = sres[sl(p)].cpu().numpy()
        if kind in ("topk", "topk16", "fp16"):
            assert np.array_equal(got.view(np.uint32), res_o.view(np.uint32))
        else:
            assert gu.close(got, res_o, REL), (name, "server residual", p)

    # ---------------- update stage on the GPU's own pulled message
    x = synth.device_params(D, device=dev)
    m = synth.device_gradient("normal", D, "f32", worker=777, device=dev)
    v = synth.device_gradient("normal", D, "f32", worker=778, device=dev).abs() * 1e-3
    before = {p: tuple(t[sl(p)].cpu().numpy() for t in (x, m, v)) for p in parts}
    step = 3
    bpc.bpc_adaptive_update(prm_b(out_stream), out_pay, x, m, v,
                            bpc.make_opt(bpc.OPT_ADAM, 1e-3, 0.9, 0.999, 1e-8, 0.01, step), ws)
    torch.cuda.synchronize()
    for p in parts:
        d = sl(p).stop - sl(p).start
        xo, mo, vo = (a.copy() for a in before[p])
        rec = out_pay[p * strd:(p + 1) * strd].cpu().numpy()
        orc.adaptive_update(prm_o(out_stream, p), rec, d, xo, mo, vo,
                            orc.make_opt(orc.OPT_ADAM, 1e-3, 0.9, 0.999, 1e-8, 0.01, step))
        for got, ref in ((x, xo), (m, mo), (v, vo)):
            assert np.array_equal(got[sl(p)].cpu().numpy().view(np.uint32), ref.view(np.uint32)), (name, "update", p)
    # ---------------- and a LANS step (the partitions are the blocks) on the state that step left
    before = {p: tuple(t[sl(p)].cpu().numpy() for t in (x, m, v)) for p in parts}
    step = 4
    bpc.bpc_adaptive_update(prm_b(out_stream), out_pay, x, m, v,
                            bpc.make_opt(bpc.OPT_LANS, 1e-3, 0.9, 0.999, 1e-8, 0.01, step), ws)
    torch.cuda.synchronize()
    for p in parts:
        d = sl(p).stop - sl(p).start
        xo, mo, vo = (a.copy() for a in before[p])
        rec = out_pay[p * strd:(p + 1) * strd].cpu().numpy()
        orc.adaptive_update(prm_o(out_stream, p), rec, d, xo, mo, vo,
                            orc.make_opt(orc.OPT_LANS, 1e-3, 0.9, 0.999, 1e-8, 0.01, step))
        for got, ref in ((m, mo), (v, vo)):
            assert np.array_equal(got[sl(p)].cpu().numpy().view(np.uint32), ref.view(np.uint32)), (name, "lans", p)
        assert gu.close(x[sl(p)].cpu().numpy(), xo, REL), (name, "lans x", p)
    del pays, sres, out_pay, x, m, v, ws
    torch.cuda.empty_cache()
