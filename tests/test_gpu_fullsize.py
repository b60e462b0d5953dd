"""GPU parity at the full sizes and in the launch configuration that bench.py times.

For each workload of the benchmark spec the whole pipeline runs on the GPU (n workers with non-zero
residuals, server aggregate, update) on seeded synthetic gradients generated on the card.
Partitions are independent units of the method, so the oracle recomputes them one by one
from exactly the bytes the GPU consumed: the gradient / residual slices for the worker stage,
the GPU's own n worker records for the server stage, the GPU's own pulled record for the
update.  On the two shapes that carry the throughput target (bert_base, bert_large) EVERY
partition of worker 0, of the server and of the update is compared, and a second worker (the
last one: another Philox stream id, another set of input buffers) on a sample; on the other
shapes a sample of partitions (first, a middle one, the ragged last one).  A LANS step over
layer-shaped caller-defined blocks, which cross partitions, is compared over the whole
gradient.  The same pipeline also runs on f32 arrays of more than 4 GiB (sign, dithering, top-k,
random-k, FP16; the partitions around the 4 GiB offset and the last ones are compared).  Same bars
as the small tests.
"""
from concurrent.futures import ThreadPoolExecutor

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


EVERY_PARTITION = ("bert_base", "bert_large")


def sample_partitions(P):
    return sorted({0, P // 2, P - 1})


def for_each(parts, check):
    """check(p) for every partition, spread over host threads (the oracle is plain C called
    through ctypes, which releases the interpreter lock).  Assertion errors surface here."""
    with ThreadPoolExecutor(16) as pool:
        list(pool.map(check, parts))


def record_equal(kind, rec_g, rec_o, d, k, k_cap, pe=0, levels=4):
    for lo, hi in fmt.defined_bytes(kind, d, k, k_cap, part_elems=pe, levels=levels):
        if not np.array_equal(rec_g[lo:hi], rec_o[lo:hi]):
            return False
    return True


@pytest.mark.parametrize("name", ["sign_1m", "resnet50", "vgg16", "bert_base", "bert_large", "bert_large_natural",
                                  "bert_large_5bit", "bert_large_fp16", "bert_base_topk16"])
def test_full_size_pipeline(env, orc, name):
    run_pipeline(env, orc, name, env[1].WORKLOADS[name])


# Shapes whose f32 arrays (gradient, residuals, parameters, moments) are larger than 4 GiB: every
# offset beyond 2^32 bytes has to come out of 64-bit arithmetic.  Partition 1024 starts exactly at
# 4 GiB; the sample takes it, its neighbour below and the last two (the last one ragged).
BEYOND_4GIB_D = (1 << 30) + 3 * (1 << 20) + 4321
BEYOND_4GIB = {
    "sign": dict(kind="sign"), "dither": dict(kind="dither", levels=4), "topk": dict(kind="topk", k_ratio=0.001),
    "randk": dict(kind="randk", k_ratio=0.001, value_scale=-1.0), "fp16": dict(kind="fp16"),
}


@pytest.mark.parametrize("name", sorted(BEYOND_4GIB))
def test_arrays_beyond_4_gib(env, orc, name):
    w = dict(D=BEYOND_4GIB_D, dtype="f32", dist="normal", n_workers=2, ef=True, opt="adam", **BEYOND_4GIB[name])
    P = (w["D"] + env[1].part_elems("f32") - 1) // env[1].part_elems("f32")
    run_pipeline(env, orc, name + "_beyond_4gib", w, sample=[0, 1023, 1024, P - 2, P - 1])


def run_pipeline(env, orc, name, w, sample=None):
    gu, synth, torch = env
    bpc = gu.bpc
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
    sampled = sample_partitions(P) if sample is None else sorted(set(sample))
    parts = list(range(P)) if name in EVERY_PARTITION else sampled

    def sl(p):
        return slice(p * pe, min(D, (p + 1) * pe))

    # ---------------- worker stage, every worker on the GPU; worker 0 checked on `parts`, the
    # last worker on the sample
    checked = {0: parts, n - 1: sampled} if n > 1 else {0: parts}
    pays, g_host, e_host, e_after = [], {}, {}, {}
    for i in range(n):
        g = synth.device_gradient(w["dist"], D, w["dtype"], worker=i, device=dev)
        e = synth.device_gradient("normal", D, "f32", worker=100 + i, device=dev) * 0.3
        if i in checked:
            g_host[i] = {p: g[sl(p)].cpu().numpy() for p in checked[i]}
            e_host[i] = {p: e[sl(p)].cpu().numpy() for p in checked[i]}
        pay = torch.zeros(bpc.payload_bytes(p0, D), dtype=torch.uint8, device=dev)
        bpc.bpc_compress(prm_b((1 << 32) | i), g, e, pay, ws)
        bpc.workspace_check(p0, D, ws)
        pays.append(pay)
        if i in checked:
            e_after[i] = {p: e[sl(p)].cpu().numpy() for p in checked[i]}
        del g, e
    for i in checked:
        pay_host = pays[i].cpu().numpy()

        def check_worker(p, i=i, pay_host=pay_host):
            d = sl(p).stop - sl(p).start
            k = fmt.k_of(kw["k_ratio"], d) if k_cap else 0
            rec_g = pay_host[p * strd:(p + 1) * strd]
            res_o = e_host[i][p].copy()
            rec_o = orc.compress(prm_o((1 << 32) | i, p), g_host[i][p], res_o)
            if kind in ("sign", "dither", "natdither"):
                hg, ho = fmt.header_f32(rec_g), fmt.header_f32(rec_o)
                assert abs(float(hg) - float(ho)) <= REL * abs(float(ho)), (name, "worker", i, "scale", p)
                if hg != ho:       # packed bits on equal terms: oracle with the GPU's scale
                    res_o = e_host[i][p].copy()
                    rec_o = orc.compress(prm_o((1 << 32) | i, p, norm=hg), g_host[i][p], res_o)
            assert record_equal(kind, rec_g, rec_o, d, k, k_cap, pe, kw["levels"]), (name, "worker", i, p)
            if kind in ("topk", "topk16", "fp16"):
                assert np.array_equal(e_after[i][p].view(np.uint32), res_o.view(np.uint32)), (name, "worker", i, p)
            else:
                assert gu.close(e_after[i][p], res_o, REL), (name, "worker residual", i, p)

        for_each(checked[i], check_worker)
    del g_host, e_host, e_after

    # ---------------- server stage on the GPU's own worker messages
    sres = synth.device_gradient("normal", D, "f32", worker=999, device=dev) * 0.2
    s_host = {p: sres[sl(p)].cpu().numpy() for p in parts}
    out_pay = torch.zeros(bpc.payload_bytes(p0, D), dtype=torch.uint8, device=dev)
    ins_b = [prm_b((1 << 32) | i) for i in range(n)]
    out_stream = (1 << 32) | (1 << 16)
    bpc.bpc_server_aggregate(ins_b, pays, prm_b(out_stream), sres, D, out_pay, ws)
    bpc.workspace_check(p0, D, ws)
    pays_host = [pay.cpu().numpy() for pay in pays]
    out_host = out_pay.cpu().numpy()
    sres_host = sres.cpu().numpy()

    def check_server(p):
        d = sl(p).stop - sl(p).start
        k = fmt.k_of(kw["k_ratio"], d) if k_cap else 0
        recs = [pays_host[i][p * strd:(p + 1) * strd] for i in range(n)]
        ins_o = [prm_o((1 << 32) | i, p) for i in range(n)]
        rec_g = out_host[p * strd:(p + 1) * strd]
        res_o = s_host[p].copy()
        rec_o = orc.server_aggregate(ins_o, recs, prm_o(out_stream, p), res_o, d)
        if kind in ("sign", "dither", "natdither"):
            hg, ho = fmt.header_f32(rec_g), fmt.header_f32(rec_o)
            assert abs(float(hg) - float(ho)) <= REL * abs(float(ho)), (name, "server scale", p)
            if hg != ho:
                res_o = s_host[p].copy()
                rec_o = orc.server_aggregate(ins_o, recs, prm_o(out_stream, p, norm=hg), res_o, d)
        if kind == "randk":      # values of Delta come through float atomics: tolerance
            kg, vg = fmt.randk_values(rec_g)
            ko, vo = fmt.randk_values(rec_o)
            assert kg == ko and gu.close(vg, vo, REL), (name, "server values", p)
        else:
            assert record_equal(kind, rec_g, rec_o, d, k, k_cap, pe, kw["levels"]), (name, "server", p)
        got = sres_host[sl(p)]
        if kind in ("topk", "topk16", "fp16"):
            assert np.array_equal(got.view(np.uint32), res_o.view(np.uint32)), (name, "server residual", p)
        else:
            assert gu.close(got, res_o, REL), (name, "server residual", p)

    for_each(parts, check_server)
    del pays, pays_host, sres, sres_host, s_host

    # ---------------- update stage on the GPU's own pulled message
    x = synth.device_params(D, device=dev)
    m = synth.device_gradient("normal", D, "f32", worker=777, device=dev)
    v = synth.device_gradient("normal", D, "f32", worker=778, device=dev).abs() * 1e-3
    before = [t.cpu().numpy() for t in (x, m, v)]
    step = 3
    bpc.bpc_adaptive_update(prm_b(out_stream), out_pay, x, m, v,
                            bpc.make_opt(bpc.OPT_ADAM, 1e-3, 0.9, 0.999, 1e-8, 0.01, step), ws)
    bpc.workspace_check(p0, D, ws)
    after = [t.cpu().numpy() for t in (x, m, v)]

    def check_adam(p):
        d = sl(p).stop - sl(p).start
        xo, mo, vo = (a[sl(p)].copy() for a in before)
        rec = out_host[p * strd:(p + 1) * strd]
        orc.adaptive_update(prm_o(out_stream, p), rec, d, xo, mo, vo,
                            orc.make_opt(orc.OPT_ADAM, 1e-3, 0.9, 0.999, 1e-8, 0.01, step))
        for got, ref in zip(after, (xo, mo, vo)):
            assert np.array_equal(got[sl(p)].view(np.uint32), ref.view(np.uint32)), (name, "update", p)

    for_each(parts, check_adam)
    # ---------------- and a LANS step (the partitions are the blocks) on the state that step left
    before = after
    step = 4
    bpc.bpc_adaptive_update(prm_b(out_stream), out_pay, x, m, v,
                            bpc.make_opt(bpc.OPT_LANS, 1e-3, 0.9, 0.999, 1e-8, 0.01, step), ws)
    bpc.workspace_check(p0, D, ws)
    after = [t.cpu().numpy() for t in (x, m, v)]

    def check_lans(p):
        d = sl(p).stop - sl(p).start
        xo, mo, vo = (a[sl(p)].copy() for a in before)
        rec = out_host[p * strd:(p + 1) * strd]
        orc.adaptive_update(prm_o(out_stream, p), rec, d, xo, mo, vo,
                            orc.make_opt(orc.OPT_LANS, 1e-3, 0.9, 0.999, 1e-8, 0.01, step))
        for got, ref in zip(after[1:], (mo, vo)):
            assert np.array_equal(got[sl(p)].view(np.uint32), ref.view(np.uint32)), (name, "lans", p)
        assert gu.lans_step_close(after[0][sl(p)], xo, before[0][sl(p)]), (name, "lans x", p)

    for_each(parts, check_lans)
    del out_pay, x, m, v, ws
    torch.cuda.empty_cache()


@pytest.mark.parametrize("name,hidden", [("bert_base", 768), ("bert_large", 1024)])
@pytest.mark.parametrize("lr", [1e-3, 0.5])
def test_full_size_lans_step_over_layer_blocks(env, orc, name, hidden, lr):
    """Algorithm 5 normalises over layers, not partitions: one LANS step with caller-defined
    blocks sized like the tensors of a BERT encoder stack (synth.layer_blocks: a few hundred
    blocks from `hidden` to tens of millions of elements, most boundaries inside a partition),
    on the whole gradient, against the oracle over the whole gradient.  The learning rate of 0.5
    makes a step as large as x, so that its error is not hidden behind the rounding of x."""
    gu, synth, torch = env
    bpc = gu.bpc
    w = synth.WORKLOADS[name]
    D, kind = w["D"], w["kind"]
    pe = synth.part_elems(w["dtype"])
    kw = dict(levels=w.get("levels", 4), seed=synth.BASE_SEED, stream_id=(1 << 32) | (1 << 16))
    kind_o = {"sign": orc.SIGN, "dither": orc.DITHER}[kind]
    pb, po = bpc.make_params(gu.KIND_B[kind], pe, **kw), orc.make_params(kind_o, pe, **kw)
    dev = gu.DEV
    blocks = synth.layer_blocks(D, hidden)
    # a pulled message: the worker-side call on a synthetic Delta
    delta = synth.device_gradient(w["dist"], D, "f32", worker=5, device=dev)
    pay = torch.zeros(bpc.payload_bytes(pb, D), dtype=torch.uint8, device=dev)
    ws = torch.zeros(bpc.update_workspace_bytes(pb, D, len(blocks) - 1), dtype=torch.uint8, device=dev)
    bpc.bpc_compress(pb, delta, None, pay, ws)
    bpc.workspace_check(pb, D, ws)
    del delta
    x = synth.device_params(D, device=dev)
    m = synth.device_gradient("normal", D, "f32", worker=777, device=dev)
    v = synth.device_gradient("normal", D, "f32", worker=778, device=dev).abs() * 1e-3
    xo, mo, vo = (t.cpu().numpy() for t in (x, m, v))
    x_before = xo.copy()
    step = 2
    blocks_dev = torch.from_numpy(blocks.astype(np.int64)).to(dev)
    bpc.bpc_adaptive_update(pb, pay, x, m, v,
                            bpc.make_opt(bpc.OPT_LANS, lr, 0.9, 0.999, 1e-8, 0.01, step, block_offsets=blocks_dev), ws)
    bpc.workspace_check(pb, D, ws)
    orc.adaptive_update(po, pay.cpu().numpy(), D, xo, mo, vo,
                        orc.make_opt(orc.OPT_LANS, lr, 0.9, 0.999, 1e-8, 0.01, step, block_offsets=blocks))
    assert np.array_equal(m.cpu().numpy().view(np.uint32), mo.view(np.uint32))
    assert np.array_equal(v.cpu().numpy().view(np.uint32), vo.view(np.uint32))
    assert gu.lans_step_close(x.cpu().numpy(), xo, x_before, blocks)
    del x, m, v, pay, ws
    torch.cuda.empty_cache()


def test_full_size_masked_pipeline_with_a_shared_scale(env, orc):
    """The bert_base shape (scaled sign, f16 gradients, 16 workers) with what a deployment adds
    to it (Section 4.2 size threshold; Section 3.2 scaled sign with one scale for all workers):
    a few partitions bypass compression and the workers all quantise with one short scale per
    partition, so the server takes the counting form of the sum between runs of bypassed
    partitions.  Worker 0 and the last worker, the server and an Adam step are compared on
    every partition with the oracle, partition by partition."""
    gu, synth, torch = env
    bpc = gu.bpc
    w = synth.WORKLOADS["bert_base"]
    D, n = w["D"], w["n_workers"]
    assert w["kind"] == "sign" and n == 16
    pe = synth.part_elems(w["dtype"])
    P = (D + pe - 1) // pe
    dev = gu.DEV
    mask = np.zeros(P, np.uint8)
    mask[[3, 4, P // 2, P - 1]] = 1
    # one scale per partition, all short (low six significand bits clear) and different
    scales = (np.uint32(0x3A83F1C0) + np.arange(P, dtype=np.uint32) * 64).view(np.float32)
    shared = gu.to_dev(scales)

    def prm_b(stream, shared_scale):
        return bpc.make_params(bpc.SIGN, pe, stream_id=stream, seed=synth.BASE_SEED, bypass=mask,
                               norm_override=shared if shared_scale else None)

    def prm_o(stream, part, norm=None):
        return orc.make_params(orc.IDENTITY if mask[part] else orc.SIGN, pe, stream_id=stream, seed=synth.BASE_SEED,
                               first_partition=part,
                               norm_override=None if norm is None else np.array([norm], np.float32))

    p_in = [prm_b((1 << 32) | i, True) for i in range(n)]
    out_stream = (1 << 32) | (1 << 16)
    p_out = prm_b(out_stream, False)
    offs = [bpc.partition_offset(p_out, D, p) for p in range(P)] + [bpc.payload_bytes(p_out, D)]
    assert offs == sorted(offs) and offs[P] - offs[P - 1] == 16 + 4 * pe      # the last one is bypassed
    ws = torch.zeros(bpc.workspace_bytes(p_out, D, n), dtype=torch.uint8, device=dev)
    parts = list(range(P))

    def sl(p):
        return slice(p * pe, min(D, (p + 1) * pe))

    def defined(p):
        d = sl(p).stop - sl(p).start
        return fmt.defined_bytes("identity" if mask[p] else "sign", d)

    def same_record(a, b, p):
        return all(np.array_equal(a[lo:hi], b[lo:hi]) for lo, hi in defined(p))

    checked = (0, n - 1)
    pays, g_host, e_host, e_after = [], {}, {}, {}
    for i in range(n):
        g = synth.device_gradient(w["dist"], D, w["dtype"], worker=i, device=dev)
        e = synth.device_gradient("normal", D, "f32", worker=100 + i, device=dev) * 0.3
        if i in checked:
            g_host[i], e_host[i] = g.cpu().numpy(), e.cpu().numpy()
        pay = torch.zeros(offs[P], dtype=torch.uint8, device=dev)
        bpc.bpc_compress(p_in[i], g, e, pay, ws)
        bpc.workspace_check(p_out, D, ws)
        pays.append(pay)
        if i in checked:
            e_after[i] = e.cpu().numpy()
        del g, e
    pays_host = [pay.cpu().numpy() for pay in pays]
    for i in checked:
        def check_worker(p, i=i):
            res_o = e_host[i][sl(p)].copy()
            rec_o = orc.compress(prm_o((1 << 32) | i, p, norm=scales[p]), g_host[i][sl(p)], res_o)
            assert same_record(pays_host[i][offs[p]:offs[p + 1]], rec_o, p), ("worker", i, p)
            assert np.array_equal(e_after[i][sl(p)].view(np.uint32), res_o.view(np.uint32)), ("worker residual", i, p)

        for_each(parts, check_worker)
    del g_host, e_host, e_after

    sres = synth.device_gradient("normal", D, "f32", worker=999, device=dev) * 0.2
    s_host = sres.cpu().numpy()
    out_pay = torch.zeros(offs[P], dtype=torch.uint8, device=dev)
    bpc.bpc_server_aggregate(p_in, pays, p_out, sres, D, out_pay, ws)
    bpc.workspace_check(p_out, D, ws)
    out_host, sres_host = out_pay.cpu().numpy(), sres.cpu().numpy()

    def check_server(p):
        d = sl(p).stop - sl(p).start
        recs = [np.ascontiguousarray(pays_host[i][offs[p]:offs[p + 1]]) for i in range(n)]
        ins_o = [prm_o((1 << 32) | i, p, norm=scales[p]) for i in range(n)]
        rec_g = out_host[offs[p]:offs[p + 1]]
        res_o = s_host[sl(p)].copy()
        rec_o = orc.server_aggregate(ins_o, recs, prm_o(out_stream, p), res_o, d)
        if not mask[p]:
            hg, ho = fmt.header_f32(rec_g), fmt.header_f32(rec_o)
            assert abs(float(hg) - float(ho)) <= REL * abs(float(ho)), ("server scale", p)
            if hg != ho:
                res_o = s_host[sl(p)].copy()
                rec_o = orc.server_aggregate(ins_o, recs, prm_o(out_stream, p, norm=hg), res_o, d)
        assert same_record(rec_g, rec_o, p), ("server", p)
        assert gu.close(sres_host[sl(p)], res_o, REL), ("server residual", p)

    for_each(parts, check_server)
    del pays, pays_host, sres

    x = synth.device_params(D, device=dev)
    m = synth.device_gradient("normal", D, "f32", worker=777, device=dev)
    v = synth.device_gradient("normal", D, "f32", worker=778, device=dev).abs() * 1e-3
    before = [t.cpu().numpy() for t in (x, m, v)]
    bpc.bpc_adaptive_update(p_out, out_pay, x, m, v, bpc.make_opt(bpc.OPT_ADAM, 1e-3, 0.9, 0.999, 1e-8, 0.01, 3), ws)
    bpc.workspace_check(p_out, D, ws)
    after = [t.cpu().numpy() for t in (x, m, v)]

    def check_adam(p):
        d = sl(p).stop - sl(p).start
        xo, mo, vo = (a[sl(p)].copy() for a in before)
        orc.adaptive_update(prm_o(out_stream, p), np.ascontiguousarray(out_host[offs[p]:offs[p + 1]]), d, xo, mo, vo,
                            orc.make_opt(orc.OPT_ADAM, 1e-3, 0.9, 0.999, 1e-8, 0.01, 3))
        for got, ref in zip(after, (xo, mo, vo)):
            assert np.array_equal(got[sl(p)].view(np.uint32), ref.view(np.uint32)), ("update", p)

    for_each(parts, check_adam)
    del out_pay, x, m, v, ws
    torch.cuda.empty_cache()
