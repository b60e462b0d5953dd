"""ctypes binding of the CPU oracle (``bpc_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, ``__graft_entry__.smoke()``
and the ``cpu_baseline`` leg of ``bench.py``.  Works on numpy arrays in host
memory; imports nothing from the GPU package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libbpc_oracle.so")

IDENTITY, SIGN, TOPK, RANDK, DITHER, NATDITHER, FP16, TOPK16 = 0, 1, 2, 3, 4, 5, 6, 7
F32, F16 = 0, 1
NORM_L2, NORM_LINF = 0, 1
OPT_LANS, OPT_ADAM = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (scalar, no FMA contraction)."""
    src = os.path.join(_HERE, "bpc_oracle.c")
    hdr = os.path.join(_HERE, "bpc_oracle.h")
    if (not force and os.path.exists(_SO)
            and os.path.getmtime(_SO) >= max(os.path.getmtime(src), os.path.getmtime(hdr))):
        return _SO
    cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
           "-Wall", "-Wextra", "-o", _SO, src, "-lm"]
    subprocess.run(cmd, check=True)
    return _SO


class Params(C.Structure):
    _fields_ = [("kind", C.c_int), ("norm", C.c_int), ("part_elems", C.c_uint64),
                ("k_ratio", C.c_double), ("levels", C.c_uint), ("value_scale", C.c_float),
                ("seed", C.c_uint64), ("stream_id", C.c_uint64), ("first_partition", C.c_uint64),
                ("norm_override", C.c_void_p)]


class Opt(C.Structure):
    _fields_ = [("kind", C.c_int), ("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float),
                ("eps", C.c_float), ("weight_decay", C.c_float), ("bias_corr1", C.c_float),
                ("bias_corr2", C.c_float), ("phi_lo", C.c_float), ("phi_hi", C.c_float),
                ("block_offsets", C.c_void_p), ("n_blocks", C.c_uint64)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_SO)
        L.orc_philox4x32_10.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        L.orc_philox4x32_10.restype = None
        L.orc_half_to_float.argtypes = [C.c_uint16]
        L.orc_half_to_float.restype = C.c_float
        L.orc_float_to_half.argtypes = [C.c_float]
        L.orc_float_to_half.restype = C.c_uint16
        L.orc_partition_k.argtypes = [C.POINTER(Params), C.c_uint64]
        L.orc_partition_k.restype = C.c_uint64
        L.orc_partition_stride.argtypes = [C.POINTER(Params)]
        L.orc_partition_stride.restype = C.c_size_t
        L.orc_payload_bytes.argtypes = [C.POINTER(Params), C.c_uint64]
        L.orc_payload_bytes.restype = C.c_size_t
        L.orc_encode_partition.argtypes = [C.POINTER(Params), C.c_uint64, C.c_void_p, C.c_void_p,
                                           C.c_uint64, C.c_void_p]
        L.orc_encode_partition.restype = None
        L.orc_decode_partition.argtypes = [C.POINTER(Params), C.c_uint64, C.c_void_p, C.c_uint64,
                                           C.c_void_p]
        L.orc_decode_partition.restype = None
        L.orc_compress.argtypes = [C.POINTER(Params), C.c_void_p, C.c_int, C.c_void_p, C.c_uint64,
                                   C.c_void_p]
        L.orc_compress.restype = C.c_int
        L.orc_decompress.argtypes = [C.POINTER(Params), C.c_void_p, C.c_uint64, C.c_void_p]
        L.orc_decompress.restype = C.c_int
        L.orc_server_aggregate.argtypes = [C.POINTER(Params), C.c_void_p, C.c_int, C.POINTER(Params),
                                           C.c_void_p, C.c_uint64, C.c_void_p]
        L.orc_server_aggregate.restype = C.c_int
        L.orc_adaptive_update.argtypes = [C.POINTER(Params), C.c_void_p, C.c_uint64, C.c_void_p,
                                          C.c_void_p, C.c_void_p, C.POINTER(Opt)]
        L.orc_adaptive_update.restype = C.c_int
        _lib = L
    return _lib


def make_params(kind, part_elems, k_ratio=0.01, levels=4, norm=NORM_L2, value_scale=1.0, seed=0,
                stream_id=0, first_partition=0, norm_override=None) -> Params:
    """``norm_override``: float32 numpy array (one per partition) kept alive by the caller."""
    p = Params()
    p.kind, p.norm, p.part_elems, p.k_ratio = int(kind), int(norm), int(part_elems), float(k_ratio)
    p.levels, p.value_scale, p.seed, p.stream_id = int(levels), float(value_scale), int(seed), int(stream_id)
    p.first_partition = int(first_partition)
    if norm_override is not None:
        assert norm_override.dtype == np.float32 and norm_override.flags.c_contiguous
        p._keep = norm_override
        p.norm_override = norm_override.ctypes.data
    else:
        p.norm_override = None
    return p


def make_opt(kind, lr, beta1, beta2, eps, weight_decay, step, phi_lo=0.0, phi_hi=float("inf"),
             block_offsets=None) -> Opt:
    o = Opt()
    o.kind, o.lr, o.beta1, o.beta2, o.eps, o.weight_decay = int(kind), lr, beta1, beta2, eps, weight_decay
    # bias corrections from the float32 values of beta that the update itself uses
    b1, b2 = float(np.float32(beta1)), float(np.float32(beta2))
    o.bias_corr1 = 1.0 - b1 ** step
    o.bias_corr2 = 1.0 - b2 ** step
    o.phi_lo, o.phi_hi = phi_lo, phi_hi
    if block_offsets is not None:
        bo = np.ascontiguousarray(block_offsets, dtype=np.uint64)
        o._keep = bo
        o.block_offsets = bo.ctypes.data
        o.n_blocks = len(bo) - 1
    else:
        o.block_offsets = None
        o.n_blocks = 0
    return o


def _ptr(a):
    return None if a is None else a.ctypes.data


def philox4x32_10(ctr, key) -> np.ndarray:
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    out = np.zeros(4, dtype=np.uint32)
    lib().orc_philox4x32_10(c.ctypes.data, k.ctypes.data, out.ctypes.data)
    return out


def half_to_float(h: int) -> float:
    return float(lib().orc_half_to_float(int(h)))


def float_to_half(x: float) -> int:
    return int(lib().orc_float_to_half(float(x)))


def partition_k(p: Params, d: int) -> int:
    return int(lib().orc_partition_k(C.byref(p), d))


def partition_stride(p: Params) -> int:
    return int(lib().orc_partition_stride(C.byref(p)))


def payload_bytes(p: Params, D: int) -> int:
    return int(lib().orc_payload_bytes(C.byref(p), D))


def _check_grad(grad):
    assert grad.flags.c_contiguous
    if grad.dtype == np.float32:
        return F32
    if grad.dtype == np.float16:
        return F16
    raise TypeError(grad.dtype)


def compress(p: Params, grad: np.ndarray, residual: np.ndarray | None) -> np.ndarray:
    """Worker side.  ``residual`` (float32) is updated in place.  Returns the payload bytes."""
    dt = _check_grad(grad)
    D = grad.size
    if residual is not None:
        assert residual.dtype == np.float32 and residual.size == D and residual.flags.c_contiguous
    payload = np.zeros(payload_bytes(p, D), dtype=np.uint8)
    rc = lib().orc_compress(C.byref(p), _ptr(grad), dt, _ptr(residual), D, _ptr(payload))
    if rc:
        raise ValueError("orc_compress: invalid arguments")
    return payload


def decompress(p: Params, payload: np.ndarray, D: int) -> np.ndarray:
    out = np.zeros(D, dtype=np.float32)
    rc = lib().orc_decompress(C.byref(p), _ptr(payload), D, _ptr(out))
    if rc:
        raise ValueError("orc_decompress: invalid arguments")
    return out


def server_aggregate(in_params, payloads, out_params: Params, server_residual, D: int) -> np.ndarray:
    n = len(payloads)
    arr = (Params * n)(*in_params)
    ptrs = (C.c_void_p * n)(*[pl.ctypes.data for pl in payloads])
    out_payload = np.zeros(payload_bytes(out_params, D), dtype=np.uint8)
    if server_residual is not None:
        assert server_residual.dtype == np.float32 and server_residual.size == D
    rc = lib().orc_server_aggregate(arr, ptrs, n, C.byref(out_params), _ptr(server_residual), D,
                                    _ptr(out_payload))
    if rc:
        raise ValueError("orc_server_aggregate: invalid arguments")
    return out_payload


def adaptive_update(p: Params, payload: np.ndarray, D: int, param, m, v, opt: Opt) -> None:
    for a in (param, m, v):
        assert a.dtype == np.float32 and a.size == D and a.flags.c_contiguous
    rc = lib().orc_adaptive_update(C.byref(p), _ptr(payload), D, _ptr(param), _ptr(m), _ptr(v),
                                   C.byref(opt))
    if rc:
        raise ValueError("orc_adaptive_update: invalid arguments")


def encode_partition(p: Params, part_no: int, q: np.ndarray, norm=None) -> np.ndarray:
    assert q.dtype == np.float32 and q.flags.c_contiguous
    rec = np.zeros(partition_stride(p), dtype=np.uint8)
    nrm = None if norm is None else np.array([norm], dtype=np.float32)
    lib().orc_encode_partition(C.byref(p), part_no, _ptr(nrm), _ptr(q), q.size, _ptr(rec))
    return rec


def decode_partition(p: Params, part_no: int, rec: np.ndarray, d: int) -> np.ndarray:
    out = np.zeros(d, dtype=np.float32)
    lib().orc_decode_partition(C.byref(p), part_no, _ptr(rec), d, _ptr(out))
    return out


# ---------------------------------------------------------------------------------------------
# The size threshold of Section 4.2: tensors under a threshold are not compressed.  Here the
# unit is the partition: `mask[p]` non-zero means partition p is carried as it is (an IDENTITY
# record, residual 0), the others go through the compressor.  Written partition by partition,
# each through the plain functions above, so the records simply follow each other.
def _part_params(p: Params, part: int, bypassed: bool) -> Params:
    q = Params()
    C.memmove(C.byref(q), C.byref(p), C.sizeof(Params))
    q.first_partition = p.first_partition + part
    if bypassed:
        q.kind = IDENTITY
    if p.norm_override:
        q.norm_override = p.norm_override + 4 * part
        q._keep = getattr(p, "_keep", None)
    return q


def _parts(p: Params, D: int):
    pe = int(p.part_elems)
    return [(k, k * pe, min(D, (k + 1) * pe)) for k in range((D + pe - 1) // pe)]


def record_sizes_bypass(p: Params, mask, D: int):
    """Bytes of every partition's record: the kind's stride, or that of an IDENTITY record of
    part_elems elements for a bypassed partition (records follow each other directly)."""
    ident = _part_params(p, 0, True)
    return [partition_stride(ident) if mask[k] else partition_stride(p) for k, _, _ in _parts(p, D)]


def compress_bypass(p: Params, mask, grad: np.ndarray, residual) -> np.ndarray:
    recs = []
    for k, lo, hi in _parts(p, grad.size):
        res = None if residual is None else residual[lo:hi]
        recs.append(compress(_part_params(p, k, bool(mask[k])), grad[lo:hi], res))
    return np.concatenate(recs) if recs else np.zeros(0, np.uint8)


def decompress_bypass(p: Params, mask, payload: np.ndarray, D: int) -> np.ndarray:
    out = np.zeros(D, dtype=np.float32)
    offs = np.concatenate([[0], np.cumsum(record_sizes_bypass(p, mask, D))]).astype(np.int64)
    for k, lo, hi in _parts(p, D):
        out[lo:hi] = decompress(_part_params(p, k, bool(mask[k])), payload[offs[k]:offs[k + 1]], hi - lo)
    return out


def server_aggregate_bypass(in_params, payloads, out_params: Params, mask, server_residual, D: int) -> np.ndarray:
    offs = np.concatenate([[0], np.cumsum(record_sizes_bypass(out_params, mask, D))]).astype(np.int64)
    recs = []
    for k, lo, hi in _parts(out_params, D):
        ins = [_part_params(q, k, bool(mask[k])) for q in in_params]
        res = None if server_residual is None else server_residual[lo:hi]
        recs.append(server_aggregate(ins, [np.ascontiguousarray(pl[offs[k]:offs[k + 1]]) for pl in payloads],
                                     _part_params(out_params, k, bool(mask[k])), res, hi - lo))
    return np.concatenate(recs) if recs else np.zeros(0, np.uint8)


def adaptive_update_bypass(p: Params, mask, payload: np.ndarray, D: int, param, m, v, opt: Opt) -> None:
    """Blocks of the update are the partitions (no caller-defined blocks here)."""
    assert not opt.block_offsets
    offs = np.concatenate([[0], np.cumsum(record_sizes_bypass(p, mask, D))]).astype(np.int64)
    for k, lo, hi in _parts(p, D):
        adaptive_update(_part_params(p, k, bool(mask[k])), np.ascontiguousarray(payload[offs[k]:offs[k + 1]]), hi - lo,
                        param[lo:hi], m[lo:hi], v[lo:hi], opt)
