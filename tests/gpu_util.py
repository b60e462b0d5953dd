"""Helpers of the GPU parity tests: move numpy inputs to the card, call the C-ABI library
through its Python binding, bring results back."""
import numpy as np
import torch

import paper_2105_07829_amd as bpc

DEV = "cuda"

KIND_B = {"identity": bpc.IDENTITY, "sign": bpc.SIGN, "topk": bpc.TOPK, "randk": bpc.RANDK, "dither": bpc.DITHER,
          "natdither": bpc.NATDITHER, "fp16": bpc.FP16, "topk16": bpc.TOPK16}


def both_params(orc, kind, pe, **kw):
    """The same compressor description for the oracle and for the library."""
    kind_o = {"identity": orc.IDENTITY, "sign": orc.SIGN, "topk": orc.TOPK, "randk": orc.RANDK,
              "dither": orc.DITHER, "natdither": orc.NATDITHER, "fp16": orc.FP16, "topk16": orc.TOPK16}[kind]
    kw = {k: v for k, v in kw.items() if not k.startswith("_")}     # "_..." keys are notes for the tests
    kw_o, kw_b = dict(kw), dict(kw)
    kw_o.pop("bypass", None)                      # the oracle takes the mask per call, not in its params
    if isinstance(kw.get("norm_override"), np.ndarray):
        kw_b["norm_override"] = to_dev(kw["norm_override"])     # the library reads the scales on the card
    return orc.make_params(kind_o, pe, **kw_o), bpc.make_params(KIND_B[kind], pe, **kw_b)


def to_dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def to_host(t):
    return None if t is None else t.cpu().numpy()


def new_ws(pb, D, n=1):
    return torch.zeros(max(bpc.workspace_bytes(pb, D, n), 256), dtype=torch.uint8, device=DEV)


def new_payload(pb, D, fill=0xA5):
    # filled with a pattern so that bytes the library must write cannot pass by accident
    return torch.full((max(bpc.payload_bytes(pb, D), 16),), fill, dtype=torch.uint8, device=DEV)


def gpu_compress(pb, grad_np, res_np):
    D = grad_np.size
    g = to_dev(grad_np)
    r = to_dev(res_np)
    payload = new_payload(pb, D)
    ws = new_ws(pb, D)
    bpc.bpc_compress(pb, g, r, payload, ws)
    torch.cuda.synchronize()
    assert D == 0 or bpc.workspace_status(pb, D, ws) == 0, "a device-side wait timed out"
    return to_host(payload)[:bpc.payload_bytes(pb, D)], to_host(r)


def gpu_decompress(pb, payload_np, D):
    out = torch.full((max(D, 1),), 7.0, dtype=torch.float32, device=DEV)[:D]
    pl = to_dev(payload_np) if payload_np.size else torch.empty(16, dtype=torch.uint8, device=DEV)
    bpc.bpc_decompress(pb, pl, out)
    torch.cuda.synchronize()
    return to_host(out)


def gpu_server(in_pbs, payloads_np, out_pb, res_np, D):
    pls = [to_dev(p) for p in payloads_np]
    r = to_dev(res_np)
    out_payload = new_payload(out_pb, D)
    ws = new_ws(out_pb, D, len(pls))
    ws[:].zero_()
    bpc.bpc_server_aggregate(in_pbs, pls, out_pb, r, D, out_payload, ws)
    torch.cuda.synchronize()
    assert bpc.workspace_status(out_pb, D, ws) == 0, "a device-side wait timed out"
    return to_host(out_payload)[:bpc.payload_bytes(out_pb, D)], to_host(r)


def gpu_update(pb, payload_np, x_np, m_np, v_np, opt_b):
    x, m, v = to_dev(x_np), to_dev(m_np), to_dev(v_np)
    D = x_np.size
    ws = torch.empty(max(bpc.update_workspace_bytes(pb, D, int(opt_b.n_blocks)), 256), dtype=torch.uint8, device=DEV)
    bpc.bpc_adaptive_update(pb, to_dev(payload_np), x, m, v, opt_b, ws)
    if D:
        bpc.workspace_check(pb, D, ws)      # waits for the stream; raises if a device-side wait gave up
    torch.cuda.synchronize()
    return to_host(x), to_host(m), to_host(v)


def close(a, b, rel):
    """|a - b| <= rel * (|b| + mean|b|): relative tolerance for arrays that cross zero."""
    a64, b64 = a.astype(np.float64), b.astype(np.float64)
    scale = np.abs(b64) + (np.abs(b64).mean() if b64.size else 0.0)
    return bool(np.all(np.abs(a64 - b64) <= rel * scale + 1e-45))


def lans_step_close(x_gpu, x_ref, x_before, blocks=None, rel=2e-6):
    """The LANS step x_before - x_after of the library against the oracle's.

    The single-pass LANS kernel forms the ratios r and c with the hardware's reciprocal and
    square root (each within 1 ulp, four of them in a row: 4 * 2^-24 = 2.4e-7 relative) and its
    block norms from f32 partial sums of 512 squares (a few 1e-7 relative), so an element of the
    step lr * phi * (beta1 * u_r / |u_r| + (1 - beta1) * u_c / |u_c|) is off by at most about
    2.4e-7 + 2 * 4e-7 + a few roundings < 2e-6 of its terms; where the two terms cancel the
    bound is relative to their size, taken here as the mean |step| of the element's block.
    On top comes the one rounding of x - step to f32 on either side (2^-24 |x| each).
    `blocks`: ascending offsets of the LANS blocks (None: one block)."""
    xb = x_before.astype(np.float64)
    sg, sr = xb - x_gpu.astype(np.float64), xb - x_ref.astype(np.float64)
    if blocks is None:
        blocks = np.array([0, x_ref.size])
    blocks = np.asarray(blocks, dtype=np.int64)
    sizes = np.diff(blocks)
    sums = np.add.reduceat(np.abs(sr), blocks[:-1][sizes > 0]) if x_ref.size else np.zeros(0)
    mean = np.repeat(sums / sizes[sizes > 0], sizes[sizes > 0])
    tol = rel * (np.abs(sr) + mean) + 2.0 ** -23 * np.abs(x_ref.astype(np.float64)) + 1e-45
    return bool(np.all(np.abs(sg - sr) <= tol))
