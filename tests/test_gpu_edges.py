"""GPU parity on the degenerate inputs of the method: empty gradients, all-zero and constant
vectors (zero scale / norm, top-k ties inside and across tiles), values so small that s/nu
overflows, the largest number of workers the server accepts.  Same bars as test_gpu_parity:
bits, indices and draws exact; floating-point values to 1e-6 relative."""
import numpy as np
import pytest

import fmt

pytestmark = pytest.mark.gpu

REL = 1e-6
PE = 8192          # one tile of the single-pass server kernels per partition
BIG_PE = 131072    # several tiles per partition


@pytest.fixture(scope="module")
def gu():
    import torch
    assert torch.cuda.is_available()
    import gpu_util
    gpu_util.bpc.lib()
    return gpu_util


KW = {
    "sign": {},
    "topk": dict(k_ratio=0.01),
    "topk16": dict(k_ratio=0.01),
    "randk": dict(k_ratio=0.02, value_scale=1.0, seed=11, stream_id=(2 << 32) | 5),
    "dither": dict(levels=4, seed=0xFEED, stream_id=(7 << 32) | 1),
    "natdither": dict(levels=6, seed=0xBEEF, stream_id=(7 << 32) | 2),
    "identity": {},
    "fp16": {},
}


def defined_equal(kind, pay_a, pay_b, po, orc, D, pe, kw):
    strd = orc.partition_stride(po)
    k_cap = fmt.k_of(kw.get("k_ratio", 0.01), pe) if kind in ("topk", "topk16", "randk") else 0
    for p, d in enumerate(fmt.part_sizes(D, pe)):
        k = fmt.k_of(kw.get("k_ratio", 0.01), d) if k_cap else 0
        ra, rb = fmt.record(pay_a, p, strd), fmt.record(pay_b, p, strd)
        for lo, hi in fmt.defined_bytes(kind, d, k, k_cap):
            if not np.array_equal(ra[lo:hi], rb[lo:hi]):
                return False
    return True


@pytest.mark.parametrize("kind", sorted(KW))
def test_empty_gradient_is_a_no_op(gu, orc, kind):
    import torch
    bpc = gu.bpc
    _, pb = gu.both_params(orc, kind, PE, **KW[kind])
    g = torch.empty(0, dtype=torch.float32, device=gu.DEV)
    guard = torch.full((64,), 0x5A, dtype=torch.uint8, device=gu.DEV)
    ws = torch.zeros(256, dtype=torch.uint8, device=gu.DEV)
    bpc.bpc_compress(pb, g, None, guard, ws)
    bpc.bpc_decompress(pb, guard, g)
    bpc.bpc_server_aggregate([pb], [guard], pb, None, 0, guard, ws)
    bpc.bpc_adaptive_update(pb, guard, g, g, g, bpc.make_opt(bpc.OPT_ADAM, 1e-3, 0.9, 0.999, 1e-8, 0.0, 1), ws)
    torch.cuda.synchronize()
    assert bool((guard == 0x5A).all())


@pytest.mark.parametrize("kind", sorted(KW))
@pytest.mark.parametrize("pe", [PE, BIG_PE])
def test_all_zero_vectors(gu, orc, kind, pe):
    """sigma = 0 / nu = 0 / every key ties at 0: zero scale, level 0 everywhere, the k lowest
    indices for top-k; residuals stay zero."""
    D = 2 * pe + 4099
    po, pb = gu.both_params(orc, kind, pe, **KW[kind])
    g = np.zeros(D, np.float32)
    g[5] = -0.0                       # a negative zero is not "less than zero"
    res_ref = np.zeros(D, np.float32)
    pay_ref = orc.compress(po, g, res_ref)
    pay_gpu, res_gpu = gu.gpu_compress(pb, g, np.zeros(D, np.float32))
    assert defined_equal(kind, pay_gpu, pay_ref, po, orc, D, pe, KW[kind])
    assert np.array_equal(res_gpu.view(np.uint32) & 0x7fffffff, res_ref.view(np.uint32) & 0x7fffffff)
    out = gu.gpu_decompress(pb, pay_gpu, D)
    assert np.array_equal(out, orc.decompress(po, pay_ref, D))


@pytest.mark.parametrize("pe", [PE, BIG_PE])
@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_topk_ties_take_the_lowest_indices(gu, orc, pe, dtype):
    """Every magnitude equal (signs mixed): the kept set is decided by index alone, inside a
    tile, across the tiles of a partition and in a ragged last partition."""
    D = 2 * pe + 4099
    po, pb = gu.both_params(orc, "topk", pe, k_ratio=0.013)
    rs = np.random.default_rng(5)
    g = (np.where(rs.random(D) < 0.5, -1.0, 1.0) * 0.25).astype(dtype)
    # a handful of larger entries late in each partition, so the ties fill the rest of k
    g[pe - 7] = 3.0
    g[2 * pe - 1] = -2.0
    g[D - 1] = 5.0
    e = np.zeros(D, np.float32)
    res_ref = e.copy()
    pay_ref = orc.compress(po, g, res_ref)
    pay_gpu, res_gpu = gu.gpu_compress(pb, g, e.copy())
    assert defined_equal("topk", pay_gpu, pay_ref, po, orc, D, pe, dict(k_ratio=0.013))
    assert np.array_equal(res_gpu.view(np.uint32), res_ref.view(np.uint32))


@pytest.mark.parametrize("kind", ["topk", "topk16", "randk"])
@pytest.mark.parametrize("pe", [PE, BIG_PE])
def test_sparse_kinds_that_keep_everything(gu, orc, kind, pe):
    """k_ratio = 1, the largest k there is: top-k then keeps every element (its residual is all
    zeros, or the half-rounding error), random-k makes d draws with replacement.  Worker, server
    with two workers, decode and an Adam-style step against the oracle."""
    kw = dict(k_ratio=1.0)
    if kind == "randk":
        kw.update(value_scale=1.0, seed=21, stream_id=(4 << 32) | 9)
    D = pe + 1234
    rs = np.random.default_rng(5 + pe)
    po, pb = gu.both_params(orc, kind, pe, **kw)
    pays = []
    for i in range(2):
        g = (rs.standard_normal(D) * 1e-2).astype(np.float32)
        e = (rs.standard_normal(D) * 1e-3).astype(np.float32)
        res_ref = e.copy()
        pay_ref = orc.compress(po, g, res_ref)
        pay_gpu, res_gpu = gu.gpu_compress(pb, g, e.copy())
        assert defined_equal(kind, pay_gpu, pay_ref, po, orc, D, pe, kw), ("worker", i)
        if kind == "randk":   # (an element drawn three times: q - 3q against ((q - q) - q) - q)
            assert gu.close(res_gpu, res_ref, 1e-6)
        else:
            assert np.array_equal(res_gpu.view(np.uint32), res_ref.view(np.uint32))
        pays.append(pay_ref)
    et = (rs.standard_normal(D) * 1e-3).astype(np.float32)
    res_ref = et.copy()
    out_ref = orc.server_aggregate([po, po], pays, po, res_ref, D)
    out_gpu, res_gpu = gu.gpu_server([pb, pb], pays, pb, et, D)
    if kind == "randk":       # (values of Delta pass through float atomics whose order is free)
        strd = orc.partition_stride(po)
        for p, d in enumerate(fmt.part_sizes(D, pe)):
            kg, vg = fmt.randk_values(fmt.record(out_gpu, p, strd))
            kr, vr = fmt.randk_values(fmt.record(out_ref, p, strd))
            assert kg == kr and gu.close(vg, vr, 1e-6)
        assert gu.close(res_gpu, res_ref, 1e-6)
    else:
        assert defined_equal(kind, out_gpu, out_ref, po, orc, D, pe, kw), "server"
        assert np.array_equal(res_gpu.view(np.uint32), res_ref.view(np.uint32))
    assert np.array_equal(gu.gpu_decompress(pb, out_ref, D).view(np.uint32), orc.decompress(po, out_ref, D).view(np.uint32))
    x0 = (rs.standard_normal(D) * 0.02).astype(np.float32)
    m0 = (rs.standard_normal(D) * 1e-3).astype(np.float32)
    v0 = (rs.random(D) * 1e-5).astype(np.float32)
    x, m, v = x0.copy(), m0.copy(), v0.copy()
    orc.adaptive_update(po, out_ref, D, x, m, v, orc.make_opt(orc.OPT_ADAM, 1e-3, 0.9, 0.999, 1e-8, 0.01, 2))
    xg, mg, vg = gu.gpu_update(pb, out_ref, x0, m0, v0, gu.bpc.make_opt(gu.bpc.OPT_ADAM, 1e-3, 0.9, 0.999, 1e-8, 0.01, 2))
    for a, b in ((xg, x), (mg, m), (vg, v)):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


@pytest.mark.parametrize("kind", ["topk", "topk16"])
@pytest.mark.parametrize("case", ["short_list", "mixed", "many_duplicates", "sparse", "large_k"])
def test_topk_selection_forms(gu, orc, kind, case):
    """The selection runs on a short list of a partition's largest elements where that list
    comes out between k and its capacity, and over the whole partition otherwise, partition by
    partition: both give the oracle's record and residual.  short_list: continuous values; mixed: one partition of
    equal magnitudes between two ordinary ones; many_duplicates: 16 distinct magnitudes;
    sparse: fewer non-zeros than k; large_k: k beyond what a short list holds."""
    pe = BIG_PE
    D = 2 * pe + 70001
    ratio = 0.3 if case == "large_k" else 0.011
    po, pb = gu.both_params(orc, kind, pe, k_ratio=ratio)
    rs = np.random.default_rng(17)
    g = rs.standard_normal(D).astype(np.float32)
    e = (0.3 * rs.standard_normal(D)).astype(np.float32)
    if case == "mixed":
        g[pe:2 * pe] = np.where(rs.random(pe) < 0.5, -0.5, 0.5)
        e[pe:2 * pe] = 0.0
        g[pe + 77] = 4.0
    elif case == "many_duplicates":
        g = (rs.integers(-8, 9, D) * 0.125).astype(np.float32)
        e[:] = 0.0
    elif case == "sparse":
        keep = rs.random(D) < 0.004
        g = np.where(keep, g, 0.0).astype(np.float32)
        e[:] = 0.0
    res_ref = e.copy()
    pay_ref = orc.compress(po, g, res_ref)
    pay_gpu, res_gpu = gu.gpu_compress(pb, g, e.copy())
    assert defined_equal(kind, pay_gpu, pay_ref, po, orc, D, pe, dict(k_ratio=ratio))
    assert np.array_equal(res_gpu.view(np.uint32), res_ref.view(np.uint32))


def test_randk_server_partition_of_many_slices(gu, orc):
    """Random-k server on a partition of more than 1024 x 8192 elements: the sum of the decoded
    messages is formed in LDS slices of 16384 elements instead of 8192 (values to 1e-6: the
    order of the float adds inside a slice is free)."""
    pe = 9 * 1024 * 1024
    D = pe + 12345
    n = 2
    kw = dict(k_ratio=0.0005, value_scale=-1.0, seed=11)
    ins = [gu.both_params(orc, "randk", pe, stream_id=(3 << 32) | i, **kw) for i in range(n)]
    out_o, out_b = gu.both_params(orc, "randk", pe, stream_id=(3 << 32) | 99, **kw)
    rs = np.random.default_rng(31)
    payloads = [orc.compress(ins[i][0], (rs.standard_normal(D) * 1e-3).astype(np.float32), None) for i in range(n)]
    et = (rs.standard_normal(D) * 2e-4).astype(np.float32)
    res_ref = et.copy()
    pay_ref = orc.server_aggregate([p[0] for p in ins], payloads, out_o, res_ref, D)
    pay_gpu, res_gpu = gu.gpu_server([p[1] for p in ins], payloads, out_b, et, D)
    strd = orc.partition_stride(out_o)
    for p, d in enumerate(fmt.part_sizes(D, pe)):
        kg, vg = fmt.randk_values(fmt.record(pay_gpu, p, strd))
        kr, vr = fmt.randk_values(fmt.record(pay_ref, p, strd))
        assert kg == kr and gu.close(vg, vr, REL)
    assert gu.close(res_gpu, res_ref, REL)


@pytest.mark.parametrize("kind", ["topk", "topk16"])
@pytest.mark.parametrize("ratio", [0.011, 0.3])
def test_topk_server_both_forms(gu, orc, kind, ratio):
    """Top-k server on partitions of several groups of 8192 elements, with a k the short list
    takes and with one it does not (then the five passes run on Delta as a whole); several
    workers keep the same coordinates, so sums of three terms occur and their order shows."""
    pe = BIG_PE
    D = 2 * pe + 70001
    n = 3
    ins = [gu.both_params(orc, kind, pe, k_ratio=ratio) for _ in range(n)]
    out_o, out_b = gu.both_params(orc, kind, pe, k_ratio=ratio)
    rs = np.random.default_rng(41)
    common = rs.standard_normal(D).astype(np.float32)          # shared large coordinates
    payloads = [orc.compress(ins[i][0], (common + 0.3 * rs.standard_normal(D)).astype(np.float32), None) for i in range(n)]
    et = (0.05 * rs.standard_normal(D)).astype(np.float32)
    res_ref = et.copy()
    pay_ref = orc.server_aggregate([p[0] for p in ins], payloads, out_o, res_ref, D)
    pay_gpu, res_gpu = gu.gpu_server([p[1] for p in ins], payloads, out_b, et, D)
    assert defined_equal(kind, pay_gpu, pay_ref, out_o, orc, D, pe, dict(k_ratio=ratio))
    assert np.array_equal(res_gpu.view(np.uint32), res_ref.view(np.uint32))


@pytest.mark.parametrize("kind", ["topk", "topk16"])
def test_topk_heavy_tail(gu, orc, kind):
    """A few hundred coordinates four orders of magnitude above the rest (far more than the 64
    eighth-octave bins above the guess that the load pass counts in LDS): worker and server
    still give the oracle's record and residual."""
    pe = BIG_PE
    D = 2 * pe + 70001
    ratio = 0.011
    n = 3
    ins = [gu.both_params(orc, kind, pe, k_ratio=ratio) for _ in range(n)]
    out_o, out_b = gu.both_params(orc, kind, pe, k_ratio=ratio)
    rs = np.random.default_rng(43)
    common = rs.standard_normal(D).astype(np.float32)
    tail = rs.choice(D, 300, replace=False)
    common[tail] *= np.float32(3e4) if kind == "topk" else np.float32(2e3)   # (half-precision values: below 65504)
    grads = [(common + 0.3 * rs.standard_normal(D)).astype(np.float32) for _ in range(n)]
    e = (0.3 * rs.standard_normal(D)).astype(np.float32)
    res_ref = e.copy()
    pay_ref = orc.compress(ins[0][0], grads[0], res_ref)
    pay_gpu, res_gpu = gu.gpu_compress(ins[0][1], grads[0], e.copy())
    assert defined_equal(kind, pay_gpu, pay_ref, ins[0][0], orc, D, pe, dict(k_ratio=ratio))
    assert np.array_equal(res_gpu.view(np.uint32), res_ref.view(np.uint32))
    payloads = [orc.compress(ins[i][0], grads[i], None) for i in range(n)]
    et = (0.05 * rs.standard_normal(D)).astype(np.float32)
    res_ref = et.copy()
    pay_ref = orc.server_aggregate([p[0] for p in ins], payloads, out_o, res_ref, D)
    pay_gpu, res_gpu = gu.gpu_server([p[1] for p in ins], payloads, out_b, et, D)
    assert defined_equal(kind, pay_gpu, pay_ref, out_o, orc, D, pe, dict(k_ratio=ratio))
    assert np.array_equal(res_gpu.view(np.uint32), res_ref.view(np.uint32))


def test_topk_sample_that_misleads(gu, orc):
    """The short list is built from a guess taken from a sample of the partition (512 chunks of
    eight elements; chunk c is chunk c*stride + (c*37) % stride of the partition, stride =
    (d/8)/512).  Large values planted on 100 sampled elements only put the guess above all but
    those 100, so the list comes out shorter than k and the selection has to fall back on the
    whole partition; the record must be the oracle's all the same.  (Mirrors the sampling rule
    of the kernel: if that changes, this test still passes but no longer takes that branch.)"""
    pe = BIG_PE
    D = 2 * pe
    ratio = 0.011
    po, pb = gu.both_params(orc, "topk", pe, k_ratio=ratio)
    rs = np.random.default_rng(23)
    g = (0.5 * rs.random(D) - 0.25).astype(np.float32)
    e = np.zeros(D, np.float32)
    stride = (pe // 8) // 512
    c = np.arange(512)
    chunk = c * stride + (c * 37) % stride
    sampled = (8 * chunk[:, None] + np.arange(8)[None, :]).ravel()
    planted = rs.choice(sampled, 100, replace=False)
    g[planted] = (10.0 + rs.random(100)).astype(np.float32)          # partition 0 only
    res_ref = e.copy()
    pay_ref = orc.compress(po, g, res_ref)
    pay_gpu, res_gpu = gu.gpu_compress(pb, g, e.copy())
    assert defined_equal("topk", pay_gpu, pay_ref, po, orc, D, pe, dict(k_ratio=ratio))
    assert np.array_equal(res_gpu.view(np.uint32), res_ref.view(np.uint32))


@pytest.mark.parametrize("kind", ["dither", "natdither"])
@pytest.mark.parametrize("norm", [0, 1])
def test_dither_tiny_values_divide_per_element(gu, orc, norm, kind):
    """nu so small that s/nu is not finite: the quantiser divides per element instead."""
    D = BIG_PE + 777
    kw = dict(levels=7, norm=norm, seed=3, stream_id=4)
    po, pb = gu.both_params(orc, kind, BIG_PE, **kw)
    rs = np.random.default_rng(8)
    g = (rs.standard_normal(D) * 1e-42).astype(np.float32)      # subnormal magnitudes
    e = (rs.standard_normal(D) * 1e-43).astype(np.float32)
    res_ref = e.copy()
    pay_ref = orc.compress(po, g, res_ref)
    pay_gpu, res_gpu = gu.gpu_compress(pb, g, e.copy())
    strd = orc.partition_stride(po)
    for p in range(len(fmt.part_sizes(D, BIG_PE))):
        assert fmt.header_f32(fmt.record(pay_gpu, p, strd)) == fmt.header_f32(fmt.record(pay_ref, p, strd))
    assert defined_equal(kind, pay_gpu, pay_ref, po, orc, D, BIG_PE, kw)
    assert np.array_equal(res_gpu.view(np.uint32), res_ref.view(np.uint32))


@pytest.mark.parametrize("kind", ["sign", "dither", "natdither", "topk", "topk16", "randk", "identity", "fp16"])
def test_server_with_the_most_workers(gu, orc, kind):
    n = gu.bpc.MAX_WORKERS
    D = PE + 1234
    kw = dict(KW[kind])
    ins = []
    for i in range(n):
        if "stream_id" in kw:
            kw["stream_id"] = (1 << 32) | i
        ins.append(gu.both_params(orc, kind, PE, **kw))
    if "stream_id" in kw:
        kw["stream_id"] = (1 << 32) | (1 << 16)
    out_o, out_b = gu.both_params(orc, kind, PE, **kw)
    rs = np.random.default_rng(21)
    payloads = [orc.compress(ins[i][0], (rs.standard_normal(D) * 1e-3).astype(np.float32), None) for i in range(n)]
    et = (rs.standard_normal(D) * 2e-4).astype(np.float32)
    res_ref = et.copy()
    pay_ref = orc.server_aggregate([p[0] for p in ins], payloads, out_o, res_ref, D)
    pay_gpu, res_gpu = gu.gpu_server([p[1] for p in ins], payloads, out_b, et.copy(), D)
    strd = orc.partition_stride(out_o)
    if kind in ("sign", "dither", "natdither"):
        # scale within tolerance; then every packed bit on equal terms: where a scale differs in
        # its last bit the oracle runs again with the scales the card found
        n_parts = len(fmt.part_sizes(D, PE))
        hg = np.array([fmt.header_f32(fmt.record(pay_gpu, p, strd)) for p in range(n_parts)], dtype=np.float32)
        ho = np.array([fmt.header_f32(fmt.record(pay_ref, p, strd)) for p in range(n_parts)], dtype=np.float32)
        assert np.all(np.abs(hg.astype(np.float64) - ho) <= REL * np.abs(ho))
        if not np.array_equal(hg, ho):
            o2, _ = gu.both_params(orc, kind, PE, norm_override=hg, **kw)
            res_ref = et.copy()
            pay_ref = orc.server_aggregate([p[0] for p in ins], payloads, o2, res_ref, D)
        assert defined_equal(kind, pay_gpu, pay_ref, out_o, orc, D, PE, kw)
    elif kind == "randk":
        for p in range(len(fmt.part_sizes(D, PE))):
            kg, vg = fmt.randk_values(fmt.record(pay_gpu, p, strd))
            kr, vr = fmt.randk_values(fmt.record(pay_ref, p, strd))
            assert kg == kr and gu.close(vg, vr, REL)
    else:
        assert defined_equal(kind, pay_gpu, pay_ref, out_o, orc, D, PE, kw)
    if kind in ("identity", "topk", "topk16", "fp16"):
        assert np.array_equal(res_gpu.view(np.uint32), res_ref.view(np.uint32))
    else:
        assert gu.close(res_gpu, res_ref, REL)


@pytest.mark.parametrize("n", [4, 8, 16, 3])
@pytest.mark.parametrize("scale_bits", [0x3A83F1C0, 0x3A83126F, 0x3A83F1C0 | (1 << 31)])
def test_sign_server_with_a_shared_scale(gu, orc, n, scale_bits):
    """Scaled-sign messages that all carry one scale: with a short, positive scale (low six bits
    of the significand clear) the server may form the n-term sum from bit counts, which is then
    exact and so the plain sum; a scale with a full significand or a negative one must take the
    additions in worker order (as do fewer than 16 workers, where counting does not pay).  Either
    way every bit of the outgoing message and the residual are the oracle's.
    Partitions of several tiles with a ragged last one, with and without a server residual."""
    sigma = np.uint32(scale_bits).view(np.float32)
    for pe, D in ((PE, 2 * PE + 4137), (BIG_PE, 2 * BIG_PE + 70000)):
        scales = np.full(len(fmt.part_sizes(D, pe)), sigma, np.float32)
        ins = [gu.both_params(orc, "sign", pe, norm_override=scales) for _ in range(n)]
        rs = np.random.default_rng(33 + n)
        payloads = [orc.compress(ins[i][0], (rs.standard_normal(D) * 1e-3).astype(np.float32), None) for i in range(n)]
        out_o, out_b = gu.both_params(orc, "sign", pe)
        # the library is told that the workers shared their scales by params that all name one array
        shared = gu.to_dev(scales)
        plain = [gu.bpc.make_params(gu.bpc.SIGN, pe, norm_override=shared) for _ in range(n)]
        for ef in (True, False):
            et = (rs.standard_normal(D) * 2e-4).astype(np.float32) if ef else None
            res_ref = None if et is None else et.copy()
            pay_ref = orc.server_aggregate([p[0] for p in ins], payloads, out_o, res_ref, D)
            pay_gpu, res_gpu = gu.gpu_server(plain, payloads, out_b, None if et is None else et.copy(), D)
            strd = orc.partition_stride(out_o)
            n_parts = len(fmt.part_sizes(D, pe))
            hg = np.array([fmt.header_f32(fmt.record(pay_gpu, p, strd)) for p in range(n_parts)], dtype=np.float32)
            ho = np.array([fmt.header_f32(fmt.record(pay_ref, p, strd)) for p in range(n_parts)], dtype=np.float32)
            assert np.all(np.abs(hg.astype(np.float64) - ho) <= REL * np.abs(ho))
            if not np.array_equal(hg, ho):
                o2, _ = gu.both_params(orc, "sign", pe, norm_override=hg)
                res_ref = None if et is None else et.copy()
                pay_ref = orc.server_aggregate([p[0] for p in ins], payloads, o2, res_ref, D)
            assert defined_equal("sign", pay_gpu, pay_ref, out_o, orc, D, pe, {})
            if ef:
                assert gu.close(res_gpu, res_ref, REL)


@pytest.mark.parametrize("n", [16, 8, 3])
@pytest.mark.parametrize("case", ["subnormal", "mixed", "huge", "zero_and_negative"])
def test_sign_server_scales_at_the_ends_of_the_float_range(gu, orc, n, case):
    """The n-term sum of +-sigma_i with scales that are subnormal, zero, negative, or so large that
    the sum comes near the end of the range: the card's sum (a fused multiply-add by +-1 per worker
    for 4, 8 and 16 workers; a rolled loop of additions for other n) must give what the oracle's
    additions in worker order give, subnormal results and signed zeros included.  The outgoing
    scale is handed to both sides, so the message and the residual are compared bit for bit."""
    D = 2 * PE + 4137
    n_parts = len(fmt.part_sizes(D, PE))
    rs = np.random.default_rng(5 + n)
    pick = {"subnormal": [1e-40, 3e-39, 7e-45, 1.1e-38],
            "mixed": [1e-40, 2.5e-3, 1e-38, 3.0, 1e-20],
            "huge": [1e37, 2e37, 5e36],
            "zero_and_negative": [0.0, -0.0, -1e-3, 2e-3, -3e-40]}[case]
    ins, payloads = [], []
    for i in range(n):
        scales = np.full(n_parts, pick[i % len(pick)], np.float32)
        po, pb = gu.both_params(orc, "sign", PE, norm_override=scales)
        ins.append((po, pb))
        payloads.append(orc.compress(po, (rs.standard_normal(D) * 1e-3).astype(np.float32), None))
    mag = {"subnormal": 1e-40, "mixed": 1e-3, "huge": 1e36, "zero_and_negative": 1e-4}[case]
    out_scale = np.full(n_parts, mag, np.float32)
    out_o, out_b = gu.both_params(orc, "sign", PE, norm_override=out_scale)
    plain = [gu.bpc.make_params(gu.bpc.SIGN, PE) for _ in range(n)]
    for ef in (True, False):
        et = (rs.standard_normal(D) * mag).astype(np.float32) if ef else None
        res_ref = None if et is None else et.copy()
        pay_ref = orc.server_aggregate([p[0] for p in ins], payloads, out_o, res_ref, D)
        pay_gpu, res_gpu = gu.gpu_server(plain, payloads, out_b, None if et is None else et.copy(), D)
        assert defined_equal("sign", pay_gpu, pay_ref, out_o, orc, D, PE, {})
        if ef:
            assert np.array_equal(res_gpu.view(np.uint32), res_ref.view(np.uint32))


def test_fp16_conversion_at_the_ends_of_the_half_range(gu, orc):
    """Round to nearest even on the card as in the oracle: ties, the subnormal halves, what
    rounds up to infinity (its residual is then -inf / +inf on both sides)."""
    D = PE + 517
    rs = np.random.default_rng(12)
    g = (rs.standard_normal(D) * 1e-3).astype(np.float32)
    special = np.array([65504.0, 65519.9, 65520.0, -65520.0, 70000.0, -1e6, 2.0 ** -24, 2.0 ** -25,
                        np.nextafter(np.float32(2.0 ** -25), np.float32(1)), -2.0 ** -26, 2.0 ** -14,
                        np.nextafter(np.float32(2.0 ** -14), np.float32(0)), 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11,
                        1e-45, -1e-45, 0.0, -0.0], dtype=np.float32)
    g[100:100 + special.size] = special
    g[PE - 3:PE + 3] = special[:6]                      # across the partition boundary
    po, pb = gu.both_params(orc, "fp16", PE)
    e = np.zeros(D, np.float32)
    res_ref = e.copy()
    pay_ref = orc.compress(po, g, res_ref)
    pay_gpu, res_gpu = gu.gpu_compress(pb, g, e.copy())
    assert defined_equal("fp16", pay_gpu, pay_ref, po, orc, D, PE, {})
    assert np.array_equal(res_gpu.view(np.uint32), res_ref.view(np.uint32))
    assert np.array_equal(gu.gpu_decompress(pb, pay_gpu, D).view(np.uint32), orc.decompress(po, pay_ref, D).view(np.uint32))


@pytest.mark.parametrize("n", [2, 3, 4, 5, 8, 16])
@pytest.mark.parametrize("ef", [True, False])
def test_fp16_server_forms_and_ragged_ends(gu, orc, n, ef):
    """The FP16 server with its unrolled (4, 8, 16 workers) and its rolled form, on a gradient
    whose last partition ends inside a row of a tile and on an odd element, with signed zeros
    among the messages (the sum starts from +0 and runs in worker order, so -0 survives only
    where it must); then the worker on f16 gradients of the same odd length."""
    for D in (2 * PE + 4101, PE + 1, 3):
        po, pb = gu.both_params(orc, "fp16", PE)
        rs = np.random.default_rng(1000 * n + D)
        payloads = []
        for i in range(n):
            g = (rs.standard_t(3.0, D) * 1e-3).astype(np.float32)
            g[::7] = -0.0 if i % 2 else 0.0
            payloads.append(orc.compress(po, g, None))
        et = (rs.standard_normal(D) * 2e-4).astype(np.float32) if ef else None
        res_ref = None if et is None else et.copy()
        pay_ref = orc.server_aggregate([po] * n, payloads, po, res_ref, D)
        pay_gpu, res_gpu = gu.gpu_server([pb] * n, payloads, pb, et, D)
        assert defined_equal("fp16", pay_gpu, pay_ref, po, orc, D, PE, {}), (n, D)
        if ef:
            assert np.array_equal(res_gpu.view(np.uint32), res_ref.view(np.uint32))
        g16 = (rs.standard_t(3.0, D) * 1e-3).astype(np.float16)
        e = (rs.standard_normal(D) * 3e-4).astype(np.float32) if ef else None
        res_ref = None if e is None else e.copy()
        pay_ref = orc.compress(po, g16, res_ref)
        pay_gpu, res_gpu = gu.gpu_compress(pb, g16, e)
        assert defined_equal("fp16", pay_gpu, pay_ref, po, orc, D, PE, {}), ("worker", D)
        if ef:
            assert np.array_equal(res_gpu.view(np.uint32), res_ref.view(np.uint32))


@pytest.mark.parametrize("kind", ["sign", "dither", "topk", "identity"])
@pytest.mark.parametrize("lr", [1e-3, 0.5])
def test_lans_blocks_of_every_shape_in_one_call(gu, orc, kind, lr):
    """Caller-defined LANS blocks (Algorithm 5's layers) that stress every path of the one-pass
    kernel: ninety small blocks inside one tile of 8192 elements (more than it keeps weights
    for), blocks of one element, empty blocks, a block that starts exactly on a tile, blocks that
    start and end inside tiles and span several of them, across partition boundaries, and a
    block that runs to the ragged end."""
    import torch
    bpc = gu.bpc
    pe = 65536
    D = 5 * pe + 12345
    offs = [0] + list(range(100, 9001, 100)) + [9001, 9001, 9002, 8192 * 2, 8192 * 2 + 1, 8192 * 4 + 77,
                                                pe + 8192 * 3, pe + 8192 * 3, 3 * pe - 5, 3 * pe + 8192, 5 * pe + 7, D]
    blocks = np.array(offs, dtype=np.uint64)
    assert np.all(np.diff(blocks.astype(np.int64)) >= 0)
    po, pb = gu.both_params(orc, kind, pe, **KW[kind])
    rs = np.random.default_rng(77)
    payload = orc.compress(po, (rs.standard_t(3.0, D) * 1e-2).astype(np.float32), None)
    x0 = (rs.standard_normal(D) * 0.02).astype(np.float32)
    m0 = (rs.standard_normal(D) * 1e-3).astype(np.float32)
    v0 = (rs.random(D) * 1e-5).astype(np.float32)
    oo = orc.make_opt(orc.OPT_LANS, lr, 0.9, 0.999, 1e-8, 0.01, 4, block_offsets=blocks)
    ob = bpc.make_opt(bpc.OPT_LANS, lr, 0.9, 0.999, 1e-8, 0.01, 4,
                      block_offsets=torch.from_numpy(blocks.astype(np.int64)).to(gu.DEV))
    x, m, v = x0.copy(), m0.copy(), v0.copy()
    orc.adaptive_update(po, payload, D, x, m, v, oo)
    xg, mg, vg = gu.gpu_update(pb, payload, x0, m0, v0, ob)
    assert np.array_equal(mg.view(np.uint32), m.view(np.uint32))
    assert np.array_equal(vg.view(np.uint32), v.view(np.uint32))
    assert gu.lans_step_close(xg, x, x0, blocks)
