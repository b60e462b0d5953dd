"""Worker calls that overlap on two streams (the GPU analogue of the paper's inter-task
parallelism, Section 4.2): a top-k or random-k worker call is a chain of launches of which only
the streaming pass fills the device, so consecutive workers take turns on two streams, each with
its own workspace, and the server call joins them.  Every message and residual must be what the
calls give one after the other on one stream, and what the oracle gives."""
import numpy as np
import pytest

import fmt

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available()
    import gpu_util
    import synth
    gpu_util.bpc.lib()
    return gpu_util, synth, torch


def run_workers(bpc, torch, prms, grads, residuals, D, overlapped):
    """n worker calls, serial on the current stream or alternating over two streams; returns the
    payload tensors (residuals are updated in place)."""
    n = len(grads)
    pays = [torch.full((bpc.payload_bytes(prms[0], D),), 0xA5, dtype=torch.uint8, device="cuda") for _ in range(n)]
    main = torch.cuda.current_stream()
    if not overlapped:
        ws = torch.empty(bpc.workspace_bytes(prms[0], D, 1), dtype=torch.uint8, device="cuda")
        for i in range(n):
            bpc.bpc_compress(prms[i], grads[i], residuals[i], pays[i], ws)
        bpc.workspace_check(prms[0], D, ws)
        return pays
    side = [torch.cuda.Stream(), torch.cuda.Stream()]
    wss = [torch.empty(bpc.workspace_bytes(prms[0], D, 1), dtype=torch.uint8, device="cuda") for _ in side]
    for s in side:
        s.wait_stream(main)
    for i in range(n):
        with torch.cuda.stream(side[i % 2]):
            bpc.bpc_compress(prms[i], grads[i], residuals[i], pays[i], wss[i % 2])
    for s in side:
        main.wait_stream(s)
    for ws in wss:
        bpc.workspace_check(prms[0], D, ws)
    return pays


@pytest.mark.parametrize("kind,kw", [("topk", dict(k_ratio=0.01)), ("topk16", dict(k_ratio=0.004)),
                                     ("randk", dict(k_ratio=0.01, value_scale=-1.0, seed=3))])
def test_overlapped_workers_equal_serial_workers_and_the_oracle(env, orc, kind, kw):
    gu, synth, torch = env
    bpc = gu.bpc
    pe, n = 1 << 18, 8
    D = 9 * pe + 70001                      # ten partitions, the last one ragged
    rs = np.random.default_rng(5)
    scales = np.exp(rs.uniform(np.log(1e-4), np.log(1e-1), size=10)).astype(np.float32)
    g_np = [(rs.standard_normal(D).astype(np.float32) * 1e-3 * np.repeat(scales, pe)[:D]) for _ in range(n)]
    e_np = [(rs.standard_normal(D) * 3e-4).astype(np.float32) for _ in range(n)]
    prms = [bpc.make_params(gu.KIND_B[kind], pe, stream_id=(2 << 32) | i, **kw) for i in range(n)]
    outs = {}
    for overlapped in (False, True):
        grads = [torch.from_numpy(a).cuda() for a in g_np]
        res = [torch.from_numpy(a.copy()).cuda() for a in e_np]
        pays = run_workers(bpc, torch, prms, grads, res, D, overlapped)
        torch.cuda.synchronize()
        outs[overlapped] = ([p.cpu().numpy() for p in pays], [r.cpu().numpy() for r in res])
    strd = bpc.partition_stride(prms[0])
    k_cap = fmt.k_of(kw["k_ratio"], pe)
    for i in range(n):
        for p, d in enumerate(fmt.part_sizes(D, pe)):
            k = fmt.k_of(kw["k_ratio"], d)
            a, b = fmt.record(outs[False][0][i], p, strd), fmt.record(outs[True][0][i], p, strd)
            for lo, hi in fmt.defined_bytes(kind, d, k, k_cap):
                assert np.array_equal(a[lo:hi], b[lo:hi]), (kind, "worker", i, "partition", p)
        assert np.array_equal(outs[False][1][i].view(np.uint32), outs[True][1][i].view(np.uint32)), (kind, "residual", i)
    # and the oracle, on two of the workers (one from each stream)
    kind_o = {"topk": orc.TOPK, "topk16": orc.TOPK16, "randk": orc.RANDK}[kind]
    for i in (2, 5):
        po = orc.make_params(kind_o, pe, stream_id=(2 << 32) | i, **kw)
        res_o = e_np[i].copy()
        pay_o = orc.compress(po, g_np[i], res_o)
        for p, d in enumerate(fmt.part_sizes(D, pe)):
            k = fmt.k_of(kw["k_ratio"], d)
            a, b = fmt.record(outs[True][0][i], p, strd), fmt.record(pay_o, p, strd)
            for lo, hi in fmt.defined_bytes(kind, d, k, k_cap):
                assert np.array_equal(a[lo:hi], b[lo:hi]), (kind, "oracle, worker", i, "partition", p)
        if kind == "randk":
            assert gu.close(outs[True][1][i], res_o, 1e-6)
        else:
            assert np.array_equal(outs[True][1][i].view(np.uint32), res_o.view(np.uint32))


def test_overlapped_workers_at_the_resnet50_shape(env):
    """The launch configuration bench.py times for the ResNet-50-shaped workload: eight top-k
    workers alternating over two streams, against the same calls on one stream."""
    gu, synth, torch = env
    bpc = gu.bpc
    w = synth.WORKLOADS["resnet50"]
    D, n, pe = w["D"], w["n_workers"], synth.part_elems(w["dtype"])
    prms = [bpc.make_params(bpc.TOPK, pe, k_ratio=w["k_ratio"], stream_id=(1 << 32) | i) for i in range(n)]
    outs = {}
    for overlapped in (False, True):
        grads = [synth.device_gradient(w["dist"], D, w["dtype"], worker=i, device="cuda") for i in range(n)]
        res = [synth.device_gradient("normal", D, "f32", worker=100 + i, device="cuda") * 0.3 for i in range(n)]
        pays = run_workers(bpc, torch, prms, grads, res, D, overlapped)
        torch.cuda.synchronize()
        outs[overlapped] = (pays, res)
    strd = bpc.partition_stride(prms[0])
    k_cap = fmt.k_of(w["k_ratio"], pe)
    for i in range(n):
        a, b = outs[False][0][i].cpu().numpy(), outs[True][0][i].cpu().numpy()
        for p, d in enumerate(fmt.part_sizes(D, pe)):
            for lo, hi in fmt.defined_bytes("topk", d, fmt.k_of(w["k_ratio"], d), k_cap):
                assert np.array_equal(fmt.record(a, p, strd)[lo:hi], fmt.record(b, p, strd)[lo:hi]), (i, p)
        assert torch.equal(outs[False][1][i].view(torch.int32), outs[True][1][i].view(torch.int32)), i
