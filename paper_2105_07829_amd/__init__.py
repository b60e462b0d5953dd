"""Python binding of libbpc (include/bpc.h): two-way error-feedback gradient compression
on one MI355X.

Argument marshalling only: every function takes torch tensors that live on the GPU, passes
their ``data_ptr()`` and the current HIP stream through the C ABI, and raises ``BpcError``
on a non-zero status.  All arithmetic happens in the HIP kernels of ``csrc/``; there is no
CPU fallback -- if the shared library is missing, loading fails.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(_HERE, "libbpc.so")

# enums of include/bpc.h
IDENTITY, SIGN, TOPK, RANDK, DITHER, NATDITHER, FP16, TOPK16 = 0, 1, 2, 3, 4, 5, 6, 7
F32, F16 = 0, 1
NORM_L2, NORM_LINF = 0, 1
OPT_LANS, OPT_ADAM = 0, 1
OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_ALIGNMENT, ERR_HIP, ERR_WAIT = range(7)
MAX_WORKERS = 64

HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-ffp-contract=off",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-fPIC"]

EXPORTS = ["bpc_partition_k", "bpc_partition_stride", "bpc_payload_bytes", "bpc_partition_offset", "bpc_workspace_bytes",
           "bpc_update_workspace_bytes", "bpc_workspace_status_offset", "bpc_workspace_check", "bpc_compress", "bpc_compress_static_ws", "bpc_decompress", "bpc_server_aggregate", "bpc_adaptive_update",
           "bpc_stream_probe", "bpc_status_string", "bpc_last_hip_error"]


def _hipcc(cmd, verbose):
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)


def build(verbose: bool = False, jobs: int = 8) -> str:
    """Compile csrc/*.hip for gfx950 into libbpc.so (in-tree): one object per source file, the
    files compiled side by side (no kernel calls across files, so no relocatable device code),
    then one link.  Every call compiles every file."""
    from concurrent.futures import ThreadPoolExecutor

    srcs = sorted(f for f in os.listdir(_CSRC) if f.endswith(".hip"))
    obj_dir = os.path.join(_HERE, "_build")
    os.makedirs(obj_dir, exist_ok=True)
    objs = [os.path.join(obj_dir, f[:-4] + ".o") for f in srcs]
    with ThreadPoolExecutor(max_workers=max(1, jobs)) as pool:
        list(pool.map(lambda so: _hipcc(["hipcc", *HIPCC_FLAGS, "-c", os.path.join(_CSRC, so[0]), "-o", so[1]], verbose),
                      zip(srcs, objs)))
    _hipcc(["hipcc", "--offload-arch=gfx950", "-fPIC", "-shared", "-o", LIB_PATH, *objs], verbose)
    return LIB_PATH


class BpcError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().bpc_status_string(status).decode()
        if status == ERR_HIP:
            msg += f" (hipError_t {lib().bpc_last_hip_error()})"
        super().__init__(f"{where}: {msg}")


class Params(C.Structure):
    _fields_ = [("kind", C.c_int32), ("norm", C.c_int32), ("part_elems", C.c_uint64),
                ("k_ratio", C.c_double), ("levels", C.c_uint32), ("value_scale", C.c_float),
                ("seed", C.c_uint64), ("stream_id", C.c_uint64), ("norm_override", C.c_void_p),
                ("bypass", C.c_void_p)]


class Opt(C.Structure):
    _fields_ = [("kind", C.c_int32), ("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float),
                ("eps", C.c_float), ("weight_decay", C.c_float), ("bias_corr1", C.c_float),
                ("bias_corr2", C.c_float), ("phi_lo", C.c_float), ("phi_hi", C.c_float),
                ("reserved", C.c_uint32), ("block_offsets", C.c_void_p), ("n_blocks", C.c_uint64)]


_lib = None


def lib():
    """The loaded shared library.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} not found: run __graft_entry__.build() (hipcc) first; "
                              "there is no fallback path")
        L = C.CDLL(LIB_PATH)
        PP = C.POINTER(Params)
        L.bpc_partition_k.argtypes = [PP, C.c_uint64]
        L.bpc_partition_k.restype = C.c_uint64
        L.bpc_partition_stride.argtypes = [PP]
        L.bpc_partition_stride.restype = C.c_size_t
        L.bpc_payload_bytes.argtypes = [PP, C.c_uint64]
        L.bpc_payload_bytes.restype = C.c_size_t
        L.bpc_partition_offset.argtypes = [PP, C.c_uint64, C.c_uint64]
        L.bpc_partition_offset.restype = C.c_size_t
        L.bpc_workspace_bytes.argtypes = [PP, C.c_uint64, C.c_int]
        L.bpc_workspace_bytes.restype = C.c_size_t
        L.bpc_workspace_status_offset.argtypes = [PP, C.c_uint64]
        L.bpc_workspace_status_offset.restype = C.c_size_t
        L.bpc_update_workspace_bytes.argtypes = [PP, C.c_uint64, C.c_uint64]
        L.bpc_update_workspace_bytes.restype = C.c_size_t
        L.bpc_workspace_check.argtypes = [PP, C.c_uint64, C.c_void_p, C.c_void_p]
        L.bpc_workspace_check.restype = C.c_int
        L.bpc_compress.argtypes = [PP, C.c_void_p, C.c_int, C.c_void_p, C.c_uint64, C.c_void_p,
                                   C.c_void_p, C.c_size_t, C.c_void_p]
        L.bpc_compress.restype = C.c_int
        L.bpc_compress_static_ws.argtypes = [PP, C.c_void_p, C.c_int, C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p]
        L.bpc_compress_static_ws.restype = C.c_int
        L.bpc_decompress.argtypes = [PP, C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p]
        L.bpc_decompress.restype = C.c_int
        L.bpc_server_aggregate.argtypes = [PP, C.POINTER(C.c_void_p), C.c_int, PP, C.c_void_p,
                                           C.c_uint64, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.bpc_server_aggregate.restype = C.c_int
        L.bpc_adaptive_update.argtypes = [PP, C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.POINTER(Opt), C.c_void_p, C.c_size_t, C.c_void_p]
        L.bpc_adaptive_update.restype = C.c_int
        L.bpc_stream_probe.argtypes = [C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p]
        L.bpc_stream_probe.restype = C.c_int
        L.bpc_status_string.argtypes = [C.c_int]
        L.bpc_status_string.restype = C.c_char_p
        L.bpc_last_hip_error.argtypes = []
        L.bpc_last_hip_error.restype = C.c_int
        _lib = L
    return _lib


def make_params(kind, part_elems, k_ratio=0.01, levels=4, norm=NORM_L2, value_scale=1.0, seed=0,
                stream_id=0, norm_override=None, bypass=None) -> Params:
    """``norm_override``: float32 GPU tensor with one value per partition, or None.
    ``bypass``: numpy uint8 array (host) with one byte per partition, or None: partitions whose
    byte is non-zero are carried uncompressed."""
    p = Params()
    p.kind, p.norm, p.part_elems, p.k_ratio = int(kind), int(norm), int(part_elems), float(k_ratio)
    p.levels, p.value_scale, p.seed, p.stream_id = int(levels), float(value_scale), int(seed), int(stream_id)
    if norm_override is not None:
        p._keep = norm_override
        p.norm_override = norm_override.data_ptr()
    else:
        p.norm_override = None
    if bypass is not None:
        import numpy as np

        mask = np.ascontiguousarray(bypass, dtype=np.uint8)
        p._keep_mask = mask
        p.bypass = mask.ctypes.data
    else:
        p.bypass = None
    return p


def make_opt(kind, lr, beta1, beta2, eps, weight_decay, step, phi_lo=0.0, phi_hi=float("inf"),
             block_offsets=None) -> Opt:
    """``step`` is t >= 1; bias corrections 1 - beta^t are formed here in double precision from
    the float32 values of beta.  ``block_offsets``: int64/uint64 GPU tensor of n_blocks+1 offsets."""
    import numpy as np

    o = Opt()
    o.kind, o.lr, o.beta1, o.beta2, o.eps, o.weight_decay = int(kind), lr, beta1, beta2, eps, weight_decay
    b1, b2 = float(np.float32(beta1)), float(np.float32(beta2))
    o.bias_corr1 = 1.0 - b1 ** step
    o.bias_corr2 = 1.0 - b2 ** step
    o.phi_lo, o.phi_hi = phi_lo, phi_hi
    o.reserved = 0
    if block_offsets is not None:
        o._keep = block_offsets
        o.block_offsets = block_offsets.data_ptr()
        o.n_blocks = block_offsets.numel() - 1
    else:
        o.block_offsets = None
        o.n_blocks = 0
    return o


def _stream(stream):
    if stream is not None:
        return C.c_void_p(stream)
    import torch

    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _check(status, where):
    if status != OK:
        raise BpcError(status, where)


def partition_k(p: Params, d: int) -> int:
    return int(lib().bpc_partition_k(C.byref(p), d))


def partition_stride(p: Params) -> int:
    return int(lib().bpc_partition_stride(C.byref(p)))


def partition_offset(p: Params, D: int, part: int) -> int:
    return int(lib().bpc_partition_offset(C.byref(p), D, part))


def payload_bytes(p: Params, D: int) -> int:
    return int(lib().bpc_payload_bytes(C.byref(p), D))


def workspace_bytes(p: Params, D: int, n: int = 1) -> int:
    return int(lib().bpc_workspace_bytes(C.byref(p), D, n))


def update_workspace_bytes(p: Params, D: int, n_blocks: int = 0) -> int:
    return int(lib().bpc_update_workspace_bytes(C.byref(p), D, n_blocks))


def workspace_status(p: Params, D: int, ws) -> int:
    """Value of the workspace status word (synchronises the device); 0 means no wait timed out."""
    off = int(lib().bpc_workspace_status_offset(C.byref(p), D))
    return int(ws[off:off + 4].view(dtype=__import__("torch").int32).item())


def workspace_check(p: Params, D: int, ws, stream=None) -> None:
    """Waits for the stream and raises BpcError(ERR_WAIT) if a device-side wait of the last call
    on ``ws`` gave up (its outputs are then undefined)."""
    _check(lib().bpc_workspace_check(C.byref(p), D, _ptr(ws), _stream(stream)), "bpc_workspace_check")


def _dtype_code(grad):
    import torch

    if grad.dtype == torch.float32:
        return F32
    if grad.dtype == torch.float16:
        return F16
    raise TypeError(f"gradient dtype {grad.dtype} not supported")


def bpc_compress(p: Params, grad, residual, payload, ws, stream=None) -> None:
    """q = grad + residual; payload = C(q); residual = q - decode(payload) (in place)."""
    st = lib().bpc_compress(C.byref(p), _ptr(grad), _dtype_code(grad), _ptr(residual), grad.numel(),
                            _ptr(payload), _ptr(ws), ws.numel() * ws.element_size(), _stream(stream))
    _check(st, "bpc_compress")


PROBE_COPY, PROBE_WORKER_MIX, PROBE_UPDATE_MIX = 0, 1, 2
PROBE_BYTES_PER_ELEMENT = {PROBE_COPY: 8, PROBE_WORKER_MIX: 10, PROBE_UPDATE_MIX: 24}


def bpc_stream_probe(mix: int, a, b, c, stream=None) -> None:
    """One streaming kernel with a stage's memory traffic and none of its arithmetic (see bpc.h)."""
    _check(lib().bpc_stream_probe(mix, _ptr(a), _ptr(b), _ptr(c), c.numel(), _stream(stream)), "bpc_stream_probe")


STATIC_WS_BYTES = 4 << 20


def bpc_compress_static_ws(p: Params, grad, residual, payload, stream=None) -> None:
    """bpc_compress on the library's static device workspace (no workspace argument)."""
    st = lib().bpc_compress_static_ws(C.byref(p), _ptr(grad), _dtype_code(grad), _ptr(residual), grad.numel(),
                                      _ptr(payload), _stream(stream))
    _check(st, "bpc_compress_static_ws")


def bpc_decompress(p: Params, payload, out, stream=None) -> None:
    st = lib().bpc_decompress(C.byref(p), _ptr(payload), out.numel(), _ptr(out), _stream(stream))
    _check(st, "bpc_decompress")


def bpc_server_aggregate(in_params, payloads, out_params: Params, server_residual, D: int, out_payload, ws,
                         stream=None) -> None:
    n = len(payloads)
    arr = (Params * n)(*in_params)
    ptrs = (C.c_void_p * n)(*[pl.data_ptr() for pl in payloads])
    st = lib().bpc_server_aggregate(arr, ptrs, n, C.byref(out_params), _ptr(server_residual), D,
                                    _ptr(out_payload), _ptr(ws), ws.numel() * ws.element_size(),
                                    _stream(stream))
    _check(st, "bpc_server_aggregate")


def bpc_adaptive_update(p: Params, payload, param, m, v, opt: Opt, ws, stream=None) -> None:
    st = lib().bpc_adaptive_update(C.byref(p), _ptr(payload), param.numel(), _ptr(param), _ptr(m), _ptr(v),
                                   C.byref(opt), _ptr(ws), ws.numel() * ws.element_size(), _stream(stream))
    _check(st, "bpc_adaptive_update")
