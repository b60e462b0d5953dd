"""GPU parity: the HIP path through the C ABI against the CPU oracle, stage by stage on identical
inputs.  Bit-exact on packed sign bits, dithering nibbles, top-k indices and values, random-k
values and Philox draws; 1e-6 relative (f32 arithmetic; the f16 cases widen exactly and are held
to the same bar) on scales, norms, residuals and optimizer state."""
import numpy as np
import pytest

import fmt

pytestmark = pytest.mark.gpu

PE = 8192          # two kernel tiles per partition
REL = 1e-6
SHAPES = [2 * PE + 4137, PE, 37, 1]        # ragged tail over two tiles; exact; tiny; single element


@pytest.fixture(scope="module")
def gu():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import gpu_util
    gpu_util.bpc.lib()
    return gpu_util


def rng(seed):
    return np.random.default_rng(seed)


def grads(D, dtype, seed, scale=1e-3):
    g = rng(seed).standard_t(3.0, size=D) * scale
    return g.astype(dtype)


KW = {
    "identity": {},
    "fp16": {},
    "sign": {},
    "topk": dict(k_ratio=0.01),
    "topk16": dict(k_ratio=0.013),
    "randk": dict(k_ratio=0.02, value_scale=1.0, seed=0x1234567890ABCDEF, stream_id=(2 << 32) | 5),
    "randk_scaled": dict(k_ratio=0.02, value_scale=-1.0, seed=99, stream_id=3),
    # every worker draws from the same stream: the server sums the value vectors before it scatters
    "randk_shared": dict(k_ratio=0.02, value_scale=-1.0, seed=1234, stream_id=77, _shared=True),
    "dither": dict(levels=4, seed=0xFEEDFACECAFEBEEF, stream_id=(7 << 32) | 1),
    "dither_linf": dict(levels=7, norm=1, seed=5, stream_id=9),
    "dither_5bit": dict(levels=15, seed=0xC0FFEE, stream_id=(5 << 32) | 3),
    "dither_7bit": dict(levels=63, norm=1, seed=77, stream_id=(6 << 32) | 4),
    "natdither": dict(levels=5, seed=0xABCDEF, stream_id=(3 << 32) | 2),
    "natdither_linf": dict(levels=3, norm=1, seed=6, stream_id=10),
}


def base_kind(name):
    return name.split("_")[0]


def compare_payload(gu, orc, name, po, pay_gpu, pay_ref, D, pe, ref_fn):
    """ref_fn(norms) -> oracle payload computed with the given per-partition norm override."""
    kind = base_kind(name)
    strd = orc.partition_stride(po)
    sizes = fmt.part_sizes(D, pe)
    assert pay_gpu.size == pay_ref.size == strd * len(sizes)
    if kind in ("sign", "dither", "natdither"):
        # scale / norm within tolerance, then every packed bit on equal terms
        hg = np.array([fmt.header_f32(fmt.record(pay_gpu, p, strd)) for p in range(len(sizes))], dtype=np.float32)
        hr = np.array([fmt.header_f32(fmt.record(pay_ref, p, strd)) for p in range(len(sizes))], dtype=np.float32)
        assert np.all(np.abs(hg.astype(np.float64) - hr) <= REL * np.abs(hr))
        if not np.array_equal(hg, hr):
            pay_ref = ref_fn(hg)
    k_cap = fmt.k_of(KW[name].get("k_ratio", 0.0), pe) if kind in ("topk", "topk16", "randk") else 0
    for p, d in enumerate(sizes):
        rg, rr = fmt.record(pay_gpu, p, strd), fmt.record(pay_ref, p, strd)
        k = fmt.k_of(KW[name]["k_ratio"], d) if k_cap else 0
        for lo, hi in fmt.defined_bytes(kind, d, k, k_cap, part_elems=pe, levels=KW[name].get("levels", 4)):
            assert np.array_equal(rg[lo:hi], rr[lo:hi]), (name, "partition", p, "bytes", lo, hi)
    return pay_ref


@pytest.mark.parametrize("name", sorted(KW))
@pytest.mark.parametrize("dtype", [np.float32, np.float16])
@pytest.mark.parametrize("ef", [True, False])
def test_worker_stage(gu, orc, name, dtype, ef):
    for D in SHAPES:
        po, pb = gu.both_params(orc, base_kind(name), PE, **KW[name])
        g = grads(D, dtype, 11 + D)
        e = (rng(5 + D).standard_normal(D) * 3e-4).astype(np.float32) if ef else None
        res_ref = None if e is None else e.copy()
        pay_ref = orc.compress(po, g, res_ref)
        pay_gpu, res_gpu = gu.gpu_compress(pb, g, e)

        def redo(norms):
            po2, _ = gu.both_params(orc, base_kind(name), PE, norm_override=norms, **KW[name])
            r2 = None if e is None else e.copy()
            out = orc.compress(po2, g, r2)
            if r2 is not None:
                res_ref[:] = r2
            return out

        compare_payload(gu, orc, name, po, pay_gpu, pay_ref, D, PE, redo)
        if ef:
            if base_kind(name) in ("identity", "topk", "topk16", "fp16"):
                assert np.array_equal(res_gpu.view(np.uint32), res_ref.view(np.uint32))
            else:
                assert gu.close(res_gpu, res_ref, REL), name


BIG_PE = 131072                          # several register-resident tiles per partition (4 worker-side, 16 server-side)
BIG_D = 2 * BIG_PE + 70000               # tail partition: full tiles and a ragged one


@pytest.mark.parametrize("name", sorted(KW))
@pytest.mark.parametrize("dtype", [np.float32, np.float16])
@pytest.mark.parametrize("ef", [True, False])
def test_worker_stage_large_partitions(gu, orc, name, dtype, ef):
    """Same comparison on partitions that span several register-resident tiles."""
    for D in (BIG_D, BIG_PE, 65536 + 3):
        po, pb = gu.both_params(orc, base_kind(name), BIG_PE, **KW[name])
        g = grads(D, dtype, 17 + D)
        e = (rng(3 + D).standard_normal(D) * 3e-4).astype(np.float32) if ef else None
        res_ref = None if e is None else e.copy()
        pay_ref = orc.compress(po, g, res_ref)
        pay_gpu, res_gpu = gu.gpu_compress(pb, g, e)

        def redo(norms):
            po2, _ = gu.both_params(orc, base_kind(name), BIG_PE, norm_override=norms, **KW[name])
            r2 = None if e is None else e.copy()
            out = orc.compress(po2, g, r2)
            if r2 is not None:
                res_ref[:] = r2
            return out

        compare_payload(gu, orc, name, po, pay_gpu, pay_ref, D, BIG_PE, redo)
        if ef:
            if base_kind(name) in ("identity", "topk", "topk16", "fp16"):
                assert np.array_equal(res_gpu.view(np.uint32), res_ref.view(np.uint32))
            else:
                assert gu.close(res_gpu, res_ref, REL), name


@pytest.mark.parametrize("name", sorted(KW))
@pytest.mark.parametrize("ef", [True, False])
@pytest.mark.parametrize("n", [1, 3, 4, 16])     # (3: a mean that rounds)
def test_server_stage(gu, orc, name, ef, n):
    for D in SHAPES[:3]:
        kw = dict(KW[name])
        ins = []
        for i in range(n):
            if "stream_id" in kw and not kw.get("_shared"):
                kw["stream_id"] = (1 << 32) | i
            ins.append(gu.both_params(orc, base_kind(name), PE, **kw))
        if "stream_id" in kw:
            kw["stream_id"] = (1 << 32) | (1 << 16)
        out_o, out_b = gu.both_params(orc, base_kind(name), PE, **kw)
        payloads = [orc.compress(ins[i][0], grads(D, np.float32, 100 * i + D), None) for i in range(n)]
        et = (rng(77 + D).standard_normal(D) * 2e-4).astype(np.float32) if ef else None
        res_ref = None if et is None else et.copy()
        pay_ref = orc.server_aggregate([p[0] for p in ins], payloads, out_o, res_ref, D)
        pay_gpu, res_gpu = gu.gpu_server([p[1] for p in ins], payloads, out_b, et, D)

        def redo(norms):
            o2, _ = gu.both_params(orc, base_kind(name), PE, norm_override=norms, **kw)
            r2 = None if et is None else et.copy()
            out = orc.server_aggregate([p[0] for p in ins], payloads, o2, r2, D)
            if r2 is not None:
                res_ref[:] = r2
            return out

        if base_kind(name) == "randk":
            # values of Delta pass through float atomics whose order is free: tolerance, not bits
            strd = orc.partition_stride(out_o)
            for p, d in enumerate(fmt.part_sizes(D, PE)):
                kg, vg = fmt.randk_values(fmt.record(pay_gpu, p, strd))
                kr, vr = fmt.randk_values(fmt.record(pay_ref, p, strd))
                assert kg == kr and gu.close(vg, vr, REL)
        else:
            compare_payload(gu, orc, name, out_o, pay_gpu, pay_ref, D, PE, redo)
        if ef:
            if base_kind(name) in ("identity", "topk", "topk16", "fp16"):
                assert np.array_equal(res_gpu.view(np.uint32), res_ref.view(np.uint32))
            else:
                assert gu.close(res_gpu, res_ref, REL), name


@pytest.mark.parametrize("name", [k for k in sorted(KW) if base_kind(k) in ("sign", "dither", "natdither")])
@pytest.mark.parametrize("ef", [True, False])
@pytest.mark.parametrize("n", [3, 8, 16])
def test_server_stage_large_partitions(gu, orc, name, ef, n):
    """Server stage on partitions that span several tiles of the single-pass kernel, with and
    without a ragged last partition."""
    for D in (BIG_D, 2 * BIG_PE, 65536 + 3):
        kw = dict(KW[name])
        ins = []
        for i in range(n):
            if "stream_id" in kw and not kw.get("_shared"):
                kw["stream_id"] = (1 << 32) | i
            ins.append(gu.both_params(orc, base_kind(name), BIG_PE, **kw))
        if "stream_id" in kw:
            kw["stream_id"] = (1 << 32) | (1 << 16)
        out_o, out_b = gu.both_params(orc, base_kind(name), BIG_PE, **kw)
        payloads = [orc.compress(ins[i][0], grads(D, np.float32, 100 * i + D), None) for i in range(n)]
        et = (rng(78 + D).standard_normal(D) * 2e-4).astype(np.float32) if ef else None
        res_ref = None if et is None else et.copy()
        pay_ref = orc.server_aggregate([p[0] for p in ins], payloads, out_o, res_ref, D)
        pay_gpu, res_gpu = gu.gpu_server([p[1] for p in ins], payloads, out_b, et, D)

        def redo(norms):
            o2, _ = gu.both_params(orc, base_kind(name), BIG_PE, norm_override=norms, **kw)
            r2 = None if et is None else et.copy()
            out = orc.server_aggregate([p[0] for p in ins], payloads, o2, r2, D)
            if r2 is not None:
                res_ref[:] = r2
            return out

        compare_payload(gu, orc, name, out_o, pay_gpu, pay_ref, D, BIG_PE, redo)
        if ef:
            assert gu.close(res_gpu, res_ref, REL), name


@pytest.mark.parametrize("name", sorted(KW))
def test_decompress(gu, orc, name):
    for pe, D in [(PE, D) for D in SHAPES] + [(BIG_PE, BIG_D)]:
        po, pb = gu.both_params(orc, base_kind(name), pe, **KW[name])
        payload = orc.compress(po, grads(D, np.float32, 3 + D), None)
        ref = orc.decompress(po, payload, D)
        got = gu.gpu_decompress(pb, payload, D)
        assert np.array_equal(got.view(np.uint32), ref.view(np.uint32)), name


@pytest.mark.parametrize("name", sorted(KW))
@pytest.mark.parametrize("opt_kind", ["adam", "lans", "lans_blocks", "lans_phi", "lans_long_step"])
def test_update_stage(gu, orc, name, opt_kind):
    """m, v to the bit; the Adam-style x to the bit; the LANS step within the error the kernel's
    reciprocals and f32 partial sums can cause (gpu_util.lans_step_close).  With the usual
    learning rate a step is smaller than the rounding of x, so "lans_long_step" repeats the
    comparison with a learning rate of 0.5, where a step is as large as x itself and an error
    of the step of 1e-5 relative would show."""
    import torch
    bpc = gu.bpc
    D = 2 * PE + 4137
    lr = 0.5 if opt_kind == "lans_long_step" else 1e-3
    po, pb = gu.both_params(orc, base_kind(name), PE, **KW[name])
    payload = orc.compress(po, grads(D, np.float32, 21, scale=1e-2), None)
    x0 = (rng(1).standard_normal(D) * 0.02).astype(np.float32)
    m0 = (rng(2).standard_normal(D) * 1e-3).astype(np.float32)
    v0 = (rng(3).random(D) * 1e-5).astype(np.float32)
    blocks = np.array([0, 10, 700, PE + 3, 2 * PE, D], dtype=np.uint64) if opt_kind == "lans_blocks" else None
    phi = (0.05, 0.4) if opt_kind == "lans_phi" else (0.0, float("inf"))
    ko = orc.OPT_ADAM if opt_kind == "adam" else orc.OPT_LANS
    kb = bpc.OPT_ADAM if opt_kind == "adam" else bpc.OPT_LANS
    step = 3
    oo = orc.make_opt(ko, lr, 0.9, 0.999, 1e-8, 0.01, step, phi_lo=phi[0], phi_hi=phi[1], block_offsets=blocks)
    blocks_dev = None if blocks is None else torch.from_numpy(blocks.astype(np.int64)).to(gu.DEV)
    ob = bpc.make_opt(kb, lr, 0.9, 0.999, 1e-8, 0.01, step, phi_lo=phi[0], phi_hi=phi[1], block_offsets=blocks_dev)
    x, m, v = x0.copy(), m0.copy(), v0.copy()
    orc.adaptive_update(po, payload, D, x, m, v, oo)
    xg, mg, vg = gu.gpu_update(pb, payload, x0, m0, v0, ob)
    assert np.array_equal(mg.view(np.uint32), m.view(np.uint32))     # element-wise f32, same order
    assert np.array_equal(vg.view(np.uint32), v.view(np.uint32))
    if opt_kind == "adam":
        assert np.array_equal(xg.view(np.uint32), x.view(np.uint32))
    else:
        lans_blocks = blocks if blocks is not None else np.array([0, PE, 2 * PE, D])
        assert gu.lans_step_close(xg, x, x0, lans_blocks)


@pytest.mark.parametrize("name", sorted(KW))
@pytest.mark.parametrize("pe", [1024, 3072, 12288])
def test_partitions_that_are_no_multiple_of_a_tile(gu, orc, name, pe):
    """Partition sizes the single-pass kernels do not take (their tiles are 8192 elements): the
    smallest one, one below a tile of the streaming kernels, one and a half tiles.  Every stage
    against the oracle: worker (both gradient types), server with three workers, decode, an
    Adam-style and a LANS step."""
    bpc = gu.bpc
    kw = dict(KW[name])
    kind = base_kind(name)
    D = 3 * pe + 517
    ins = []
    for i in range(3):
        if "stream_id" in kw and not kw.get("_shared"):
            kw["stream_id"] = (1 << 32) | i
        ins.append(gu.both_params(orc, kind, pe, **kw))
    if "stream_id" in kw:
        kw["stream_id"] = (1 << 32) | (1 << 16)
    po, pb = gu.both_params(orc, kind, pe, **kw)

    def with_norms(call):
        def redo(norms):
            return call(gu.both_params(orc, kind, pe, norm_override=norms, **kw)[0])
        return redo

    for dtype in (np.float32, np.float16):
        g = grads(D, dtype, 31 + pe)
        e = (rng(7 + pe).standard_normal(D) * 3e-4).astype(np.float32)
        res_ref = e.copy()
        pay_ref = orc.compress(po, g, res_ref)
        pay_gpu, res_gpu = gu.gpu_compress(pb, g, e.copy())

        def again(p2, g=g, e=e, res_ref=res_ref):
            r2 = e.copy()
            out = orc.compress(p2, g, r2)
            res_ref[:] = r2
            return out

        compare_payload(gu, orc, name, po, pay_gpu, pay_ref, D, pe, with_norms(again))
        if kind in ("identity", "topk", "topk16", "fp16"):
            assert np.array_equal(res_gpu.view(np.uint32), res_ref.view(np.uint32))
        else:
            assert gu.close(res_gpu, res_ref, REL), (name, dtype)
    payloads = [orc.compress(ins[i][0], grads(D, np.float32, 100 * i + pe), None) for i in range(3)]
    et = (rng(78 + pe).standard_normal(D) * 2e-4).astype(np.float32)
    res_ref = et.copy()
    pay_ref = orc.server_aggregate([p[0] for p in ins], payloads, po, res_ref, D)
    pay_gpu, res_gpu = gu.gpu_server([p[1] for p in ins], payloads, pb, et.copy(), D)

    def again_s(p2):
        r2 = et.copy()
        out = orc.server_aggregate([p[0] for p in ins], payloads, p2, r2, D)
        res_ref[:] = r2
        return out

    if kind == "randk":
        strd = orc.partition_stride(po)
        for p, d in enumerate(fmt.part_sizes(D, pe)):
            kg, vg = fmt.randk_values(fmt.record(pay_gpu, p, strd))
            kr, vr = fmt.randk_values(fmt.record(pay_ref, p, strd))
            assert kg == kr and gu.close(vg, vr, REL)
    else:
        pay_ref = compare_payload(gu, orc, name, po, pay_gpu, pay_ref, D, pe, with_norms(again_s))
    if kind in ("identity", "topk", "topk16", "fp16"):
        assert np.array_equal(res_gpu.view(np.uint32), res_ref.view(np.uint32))
    else:
        assert gu.close(res_gpu, res_ref, REL), name
    assert np.array_equal(gu.gpu_decompress(pb, pay_ref, D).view(np.uint32), orc.decompress(po, pay_ref, D).view(np.uint32))
    x0 = (rng(1).standard_normal(D) * 0.02).astype(np.float32)
    m0 = (rng(2).standard_normal(D) * 1e-3).astype(np.float32)
    v0 = (rng(3).random(D) * 1e-5).astype(np.float32)
    for ko, kb in ((orc.OPT_ADAM, bpc.OPT_ADAM), (orc.OPT_LANS, bpc.OPT_LANS)):
        x, m, v = x0.copy(), m0.copy(), v0.copy()
        orc.adaptive_update(po, pay_ref, D, x, m, v, orc.make_opt(ko, 1e-3, 0.9, 0.999, 1e-8, 0.01, 3))
        xg, mg, vg = gu.gpu_update(pb, pay_ref, x0, m0, v0, bpc.make_opt(kb, 1e-3, 0.9, 0.999, 1e-8, 0.01, 3))
        assert np.array_equal(mg.view(np.uint32), m.view(np.uint32))
        assert np.array_equal(vg.view(np.uint32), v.view(np.uint32))
        if ko == orc.OPT_ADAM:
            assert np.array_equal(xg.view(np.uint32), x.view(np.uint32))
        else:
            assert gu.lans_step_close(xg, x, x0, np.array([0, pe, 2 * pe, 3 * pe, D]))


@pytest.mark.parametrize("name", sorted(KW))
@pytest.mark.parametrize("opt_kind", ["adam", "lans", "lans_blocks", "lans_long_step", "lans_blocks_long_step"])
def test_update_stage_large_partitions(gu, orc, name, opt_kind):
    """Partitions of several tiles of the update kernels (16 tiles of the single-pass LANS kernel,
    whose workgroups exchange their parts of the three block norms), a last partition of full
    tiles and a ragged one, and a gradient of less than a tile."""
    import torch
    bpc = gu.bpc
    for D in (BIG_D, 4137):
        po, pb = gu.both_params(orc, base_kind(name), BIG_PE, **KW[name])
        payload = orc.compress(po, grads(D, np.float32, 23, scale=1e-2), None)
        x0 = (rng(4).standard_normal(D) * 0.02).astype(np.float32)
        m0 = (rng(5).standard_normal(D) * 1e-3).astype(np.float32)
        v0 = (rng(6).random(D) * 1e-5).astype(np.float32)
        ko = orc.OPT_ADAM if opt_kind == "adam" else orc.OPT_LANS
        kb = bpc.OPT_ADAM if opt_kind == "adam" else bpc.OPT_LANS
        # caller-defined blocks: inside a tile, across tiles and across a partition boundary
        blocks = np.array(sorted({0, min(1000, D), min(BIG_PE + 3, D), min(2 * BIG_PE, D), D}), dtype=np.uint64) \
            if opt_kind.startswith("lans_blocks") else None
        blocks_dev = None if blocks is None else torch.from_numpy(blocks.astype(np.int64)).to(gu.DEV)
        lr = 0.5 if opt_kind.endswith("long_step") else 1e-3    # (a step as large as x: see test_update_stage)
        oo = orc.make_opt(ko, lr, 0.9, 0.999, 1e-8, 0.01, 5, block_offsets=blocks)
        ob = bpc.make_opt(kb, lr, 0.9, 0.999, 1e-8, 0.01, 5, block_offsets=blocks_dev)
        x, m, v = x0.copy(), m0.copy(), v0.copy()
        orc.adaptive_update(po, payload, D, x, m, v, oo)
        xg, mg, vg = gu.gpu_update(pb, payload, x0, m0, v0, ob)
        assert np.array_equal(mg.view(np.uint32), m.view(np.uint32)), (name, D)
        assert np.array_equal(vg.view(np.uint32), v.view(np.uint32)), (name, D)
        if opt_kind == "adam":
            assert np.array_equal(xg.view(np.uint32), x.view(np.uint32)), (name, D)
        else:
            lans_blocks = blocks if blocks is not None else np.array(sorted(set(range(0, D, BIG_PE)) | {D}))
            assert gu.lans_step_close(xg, x, x0, lans_blocks), (name, D)


def test_deterministic_bytes(gu, orc):
    """Same call twice gives identical bytes for the kinds whose arithmetic has a fixed order."""
    D = 2 * PE + 4137
    for name in ("sign", "topk", "topk16", "dither", "dither_7bit", "natdither", "identity", "fp16"):
        po, pb = gu.both_params(orc, base_kind(name), PE, **KW[name])
        g = grads(D, np.float16, 8)
        e = (rng(9).standard_normal(D) * 3e-4).astype(np.float32)
        a = gu.gpu_compress(pb, g, e)
        b = gu.gpu_compress(pb, g, e)
        assert np.array_equal(a[1], b[1])
        strd = orc.partition_stride(po)
        for p, d in enumerate(fmt.part_sizes(D, PE)):
            k = fmt.k_of(KW[name].get("k_ratio", 1.0), d)
            for lo, hi in fmt.defined_bytes(base_kind(name), d, k, fmt.k_of(KW[name].get("k_ratio", 1.0), PE),
                                            part_elems=PE, levels=KW[name].get("levels", 4)):
                assert np.array_equal(fmt.record(a[0], p, strd)[lo:hi], fmt.record(b[0], p, strd)[lo:hi])


@pytest.mark.parametrize("name", ["sign", "topk", "dither", "dither_5bit", "natdither", "randk", "identity", "fp16", "topk16"])
def test_chained_pipeline_three_steps(gu, orc, name):
    """Algorithm 4 + the Adam-style update chained on the GPU only (each stage consumes the GPU's
    own previous outputs) against the chained oracle."""
    bpc = gu.bpc
    D, n, steps = 2 * PE + 4137, 4, 3
    x_o = (rng(1).standard_normal(D) * 0.02).astype(np.float32)
    m_o, v_o = np.zeros(D, np.float32), np.zeros(D, np.float32)
    x_g, m_g, v_g = x_o.copy(), m_o.copy(), v_o.copy()
    e_o = [np.zeros(D, np.float32) for _ in range(n)]
    e_g = [np.zeros(D, np.float32) for _ in range(n)]
    et_o, et_g = np.zeros(D, np.float32), np.zeros(D, np.float32)
    diff_bytes = 0
    for t in range(1, steps + 1):
        ins, pay_o, pay_g = [], [], []
        for i in range(n):
            kw = dict(KW[name])
            if "stream_id" in kw and not kw.get("_shared"):
                kw["stream_id"] = (t << 32) | i
            po, pb = gu.both_params(orc, base_kind(name), PE, **kw)
            ins.append((po, pb))
            g = grads(D, np.float16, 1000 * t + i)
            pay_o.append(orc.compress(po, g, e_o[i]))
            pg, e_g[i] = gu.gpu_compress(pb, g, e_g[i])
            pay_g.append(pg)
        kw = dict(KW[name])
        if "stream_id" in kw:
            kw["stream_id"] = (t << 32) | (1 << 16)
        out_o, out_b = gu.both_params(orc, base_kind(name), PE, **kw)
        p_o = orc.server_aggregate([p[0] for p in ins], pay_o, out_o, et_o, D)
        p_g, et_g = gu.gpu_server([p[1] for p in ins], pay_g, out_b, et_g, D)
        if base_kind(name) in ("sign", "dither", "natdither"):
            strd = orc.partition_stride(out_o)
            for p, d in enumerate(fmt.part_sizes(D, PE)):
                for lo, hi in fmt.defined_bytes(base_kind(name), d, part_elems=PE, levels=KW[name].get("levels", 4)):
                    diff_bytes += int((fmt.record(p_o, p, strd)[lo:hi] != fmt.record(p_g, p, strd)[lo:hi]).sum())
        oo = orc.make_opt(orc.OPT_ADAM, 1e-3, 0.9, 0.999, 1e-8, 0.01, t)
        ob = bpc.make_opt(bpc.OPT_ADAM, 1e-3, 0.9, 0.999, 1e-8, 0.01, t)
        orc.adaptive_update(out_o, p_o, D, x_o, m_o, v_o, oo)
        x_g, m_g, v_g = gu.gpu_update(out_b, p_g, x_g, m_g, v_g, ob)
    print(f"chained {name}: differing message bytes over {steps} steps = {diff_bytes}")
    # norms are f64 sums rounded once: a different bit needs a sum within ~1e-13 of a rounding
    # boundary, so the chains are expected to agree to the last bit; allow the documented bar
    for a, b in ((x_g, x_o), (m_g, m_o), (v_g, v_o), (et_g, et_o)):
        assert gu.close(a, b, REL)
    for i in range(n):
        assert gu.close(e_g[i], e_o[i], REL)
    if base_kind(name) in ("sign", "dither", "natdither"):
        assert diff_bytes == 0
