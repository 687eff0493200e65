"""ctypes binding of libssmm.so -- same names as include/ssmm.h, argument marshalling only.

PyTorch is used for device memory and the current HIP stream; every step of the
path runs in the library's kernels.  There is no CPU fallback: a missing library
or a non-zero status raises.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, c_char_p, c_int, c_int32, c_int64, c_size_t, c_void_p

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("SSMM_LIB_PATH", os.path.join(_PKG, "libssmm.so"))   # override: tuning builds

SSMM_OK, SSMM_EINVAL, SSMM_ESHAPE, SSMM_EWORKSPACE, SSMM_EHIP, SSMM_ELIMIT = 0, -1, -2, -3, -4, -5


class Format(ctypes.Structure):
    """ssmm_format: (N, M, V); (1, 1, 0) is plain 2:4."""
    _fields_ = [("N", c_int32), ("M", c_int32), ("V", c_int32)]

    def __iter__(self):
        return iter((self.N, self.M, self.V))


class SsmmError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} (status {status})")


EXPORTS = {
    "ssmm_strerror": (c_char_p, [c_int]),
    "ssmm_compressed_sizes": (c_int, [c_int64, c_int64, Format, POINTER(c_size_t), POINTER(c_size_t),
                                      POINTER(c_size_t), POINTER(c_size_t)]),
    "ssmm_compress_weights": (c_int, [c_void_p, c_int, c_int64, c_int64, Format, c_void_p, c_void_p, c_void_p,
                                      c_void_p, c_void_p]),
    "ssmm_decompress_weights": (c_int, [c_void_p, c_void_p, c_void_p, c_int, c_int64, c_int64, Format, c_void_p,
                                        c_void_p]),
    "ssmm_untile_weights": (c_int, [c_void_p, c_int, c_int64, c_int64, Format, c_void_p, c_void_p, c_void_p,
                                    c_void_p]),
    "ssmm_expand_tiled_weights": (c_int, [c_void_p, c_int, c_int64, c_int64, Format, c_void_p, c_void_p]),
    "ssmm_route_workspace_bytes": (c_size_t, [c_int, c_int, c_int, c_int]),
    "ssmm_route_bucket": (c_int, [c_void_p, c_int, c_int, c_int, c_int, c_int, c_void_p, c_void_p, c_void_p,
                                  c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]),
    "ssmm_route_bucket_noalloc": (c_int, [c_void_p, c_int, c_int, c_int, c_int, c_int, c_void_p, c_void_p, c_void_p,
                                          c_void_p, c_void_p, c_void_p, c_void_p]),
    "ssmm_router_logits": (c_int, [c_void_p, c_int, c_int, c_void_p, c_int, c_void_p, c_void_p]),
    "ssmm_ffn_workspace_bytes": (c_size_t, [c_int, c_int, c_int, c_int, c_int, Format]),
    "ssmm_expert_ffn": (c_int, [c_void_p, c_int, c_int, c_int, c_int, Format, c_void_p, c_void_p, c_void_p,
                                c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_void_p, c_void_p, c_size_t,
                                c_void_p]),
    "ssmm_expert_ffn_timed": (c_int, [c_void_p, c_int, c_int, c_int, c_int, Format, c_void_p, c_void_p, c_void_p,
                                      c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_void_p, c_void_p, c_size_t,
                                      c_void_p, POINTER(c_void_p)]),
    "ssmm_expert_ffn_variant": (c_int, [c_void_p, c_int, c_int, c_int, c_int, Format, c_int, c_int, c_void_p, c_void_p,
                                        c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_void_p, c_void_p,
                                        c_size_t, c_void_p, POINTER(c_void_p)]),
    "ssmm_matmul_workspace_bytes": (c_size_t, [c_int64, c_int64, c_int, Format]),
    "ssmm_matmul": (c_int, [c_void_p, c_int64, c_int64, Format, c_void_p, c_int64, c_void_p, c_int, c_void_p, c_void_p,
                            c_size_t, c_void_p]),
}

_lib = None


def lib():
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2503_10725_amd.build` "
                               "(or __graft_entry__.build()) first; there is no fallback path")
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in EXPORTS.items():
            fn = getattr(handle, name)
            fn.restype, fn.argtypes = res, args
        _lib = handle
    return _lib


TUNE_LIB_PATH = os.path.join(_PKG, "libssmm_tune.so")


class tuning_library:
    """Context manager: calls inside go to libssmm_tune.so, the build of the same sources whose tile and
    split rules read override knobs (SSMM_DOWN_SPLITS, SSMM_PIPE, ...) from the environment.  For tests
    that force a code path and for sweeps; the library itself has no such knobs."""

    def __enter__(self):
        global _lib
        if not os.path.exists(TUNE_LIB_PATH):
            raise RuntimeError(f"{TUNE_LIB_PATH} is missing: run `python -m paper_2503_10725_amd.build` first")
        self.saved = lib()
        handle = ctypes.CDLL(TUNE_LIB_PATH)
        for name, (res, args) in EXPORTS.items():
            fn = getattr(handle, name)
            fn.restype, fn.argtypes = res, args
        _lib = handle
        return handle

    def __exit__(self, *exc):
        global _lib
        _lib = self.saved
        return False


def strerror(status):
    return lib().ssmm_strerror(int(status)).decode()


def _check(status, where):
    if status != SSMM_OK:
        raise SsmmError(status, where)


def _fmt(f):
    return f if isinstance(f, Format) else Format(*f)


def _ptr(t, dtype=None):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected dtype {dtype}, got {t.dtype}")
    return c_void_p(t.data_ptr())


def _stream():
    return c_void_p(torch.cuda.current_stream().cuda_stream)


def compressed_sizes(rows, K, fmt):
    """(values_bytes, meta_bytes, index_bytes, tiled_bytes) of one matrix."""
    out = [c_size_t(0) for _ in range(4)]
    _check(lib().ssmm_compressed_sizes(rows, K, _fmt(fmt), *[ctypes.byref(o) for o in out]), "ssmm_compressed_sizes")
    return tuple(int(o.value) for o in out)


def compress_weights(w_dense, fmt, canonical=True, tiled=True):
    """w_dense bf16 [E][rows][K] -> dict(values, meta, index, tiled); absent parts are None."""
    E, rows, K = w_dense.shape
    fmt = _fmt(fmt)
    vb, mb, ib, tb = compressed_sizes(rows, K, fmt)
    dev = w_dense.device
    values = meta = index = til = None
    if canonical or ib:          # a vector-wise format keeps its Sub-Row choice in the canonical index array
        values = torch.empty((E, vb // (K // 2) // 2, K // 2), dtype=torch.bfloat16, device=dev)
        meta = torch.empty((E, values.shape[1], mb // values.shape[1] // 4), dtype=torch.int32, device=dev)
        index = torch.empty((E, values.shape[1], ib // values.shape[1]), dtype=torch.uint8, device=dev) if ib else None
    if tiled:
        til = torch.empty((E * tb,), dtype=torch.uint8, device=dev)
    _check(lib().ssmm_compress_weights(_ptr(w_dense, torch.bfloat16), E, rows, K, fmt, _ptr(values), _ptr(meta),
                                       _ptr(index), _ptr(til), _stream()), "ssmm_compress_weights")
    return {"values": values, "meta": meta, "index": index, "tiled": til}


def decompress_weights(values, meta, index, rows, K, fmt):
    E = values.shape[0]
    out = torch.empty((E, rows, K), dtype=torch.bfloat16, device=values.device)
    _check(lib().ssmm_decompress_weights(_ptr(values, torch.bfloat16), _ptr(meta, torch.int32), _ptr(index), E, rows,
                                         K, _fmt(fmt), _ptr(out), _stream()), "ssmm_decompress_weights")
    return out


def untile_weights(tiled, E, rows, K, fmt):
    fmt = _fmt(fmt)
    vb, mb, ib, tb = compressed_sizes(rows, K, fmt)
    rc = vb // (K // 2) // 2
    values = torch.empty((E, rc, K // 2), dtype=torch.bfloat16, device=tiled.device)
    meta = torch.empty((E, rc, mb // rc // 4), dtype=torch.int32, device=tiled.device)
    index = torch.empty((E, rc, ib // rc), dtype=torch.uint8, device=tiled.device) if ib else None
    _check(lib().ssmm_untile_weights(_ptr(tiled), E, rows, K, fmt, _ptr(values), _ptr(meta), _ptr(index), _stream()),
           "ssmm_untile_weights")
    return values, meta, index


def expand_tiled_weights(tiled, E, rows, K, fmt):
    """Kernel-ready gathered format -> kernel-ready plain 2:4 of the same pruned matrices."""
    tb = compressed_sizes(rows, K, (1, 1, 0))[3]
    out = torch.empty((E * tb,), dtype=torch.uint8, device=tiled.device)
    _check(lib().ssmm_expand_tiled_weights(_ptr(tiled), E, rows, K, _fmt(fmt), _ptr(out), _stream()),
           "ssmm_expand_tiled_weights")
    return out


def route_workspace_bytes(T, E, topk, n_shared):
    return int(lib().ssmm_route_workspace_bytes(T, E, topk, n_shared))


class RouteBuffers:
    """Caller-owned outputs and workspace of route_bucket for a fixed (T, E, topk, n_shared)."""

    def __init__(self, T, E, topk, n_shared, device):
        slots, P = topk + n_shared, T * (topk + n_shared)
        i32, f32 = torch.int32, torch.float32
        self.T, self.E, self.topk, self.n_shared = T, E, topk, n_shared
        self.topk_ids = torch.empty((T, topk), dtype=i32, device=device)
        self.topk_w = torch.empty((T, topk), dtype=f32, device=device)
        self.expert_offsets = torch.empty((E + n_shared + 1,), dtype=i32, device=device)
        self.sel = torch.empty((P,), dtype=i32, device=device)
        self.sel_w = torch.empty((P,), dtype=f32, device=device)
        self.inv = torch.empty((T, slots), dtype=i32, device=device)
        self.workspace = torch.empty((max(route_workspace_bytes(T, E, topk, n_shared), 256),), dtype=torch.uint8,
                                     device=device)


def route_bucket(logits, topk, n_shared, renormalize, buf: RouteBuffers = None):
    """logits f32 [T][E] -> RouteBuffers (allocated here unless given)."""
    T, E = logits.shape
    if buf is None:
        buf = RouteBuffers(T, E, topk, n_shared, logits.device)
    _check(lib().ssmm_route_bucket(_ptr(logits, torch.float32), T, E, topk, n_shared, int(bool(renormalize)),
                                   _ptr(buf.topk_ids), _ptr(buf.topk_w), _ptr(buf.expert_offsets), _ptr(buf.sel),
                                   _ptr(buf.sel_w), _ptr(buf.inv), _ptr(buf.workspace), buf.workspace.numel(),
                                   _stream()), "ssmm_route_bucket")
    return buf


def route_bucket_noalloc(logits, topk, n_shared, renormalize, buf: RouteBuffers):
    """route_bucket through the entry point that takes no workspace and allocates nothing:
    every output tensor of `buf` must exist already (its workspace is not used)."""
    T, E = logits.shape
    _check(lib().ssmm_route_bucket_noalloc(_ptr(logits, torch.float32), T, E, topk, n_shared, int(bool(renormalize)),
                                           _ptr(buf.topk_ids), _ptr(buf.topk_w), _ptr(buf.expert_offsets),
                                           _ptr(buf.sel), _ptr(buf.sel_w), _ptr(buf.inv), _stream()),
           "ssmm_route_bucket_noalloc")
    return buf


def ffn_workspace_bytes(T, H, F, E_total, slots, fmt):
    return int(lib().ssmm_ffn_workspace_bytes(T, H, F, E_total, slots, _fmt(fmt)))


def router_logits(x, wr, logits=None):
    """x bf16 [T][H], wr bf16 [E][H] -> logits f32 [T][E] (the input of route_bucket)."""
    T, H = x.shape
    E = wr.shape[0]
    if logits is None:
        logits = torch.empty((T, E), dtype=torch.float32, device=x.device)
    _check(lib().ssmm_router_logits(_ptr(x, torch.bfloat16), T, H, _ptr(wr, torch.bfloat16), E, _ptr(logits, torch.float32),
                                    _stream()), "ssmm_router_logits")
    return logits


ACTIVATIONS = {"silu": 1, "gelu_tanh": 2, "relu": 3}   # ssmm_activation


def expert_ffn(x, F, fmt, wg_tiled, wu_tiled, wd_tiled, route: RouteBuffers, y=None, workspace=None, events=None,
               activation="silu", gated=True):
    """x bf16 [T][H] -> y bf16 [T][H] through the E_total experts' encoded weights.
    `events`: None, or a ctypes array of four hipEvent_t (see ssmm_expert_ffn_timed).
    Another `activation` or `gated=False` (wu_tiled may then be None) goes through
    ssmm_expert_ffn_variant."""
    T, H = x.shape
    fmt = _fmt(fmt)
    E_total = route.E + route.n_shared
    slots = route.topk + route.n_shared
    if y is None:
        y = torch.empty((T, H), dtype=torch.bfloat16, device=x.device)
    if workspace is None:
        workspace = torch.empty((max(ffn_workspace_bytes(T, H, F, E_total, slots, fmt), 256),), dtype=torch.uint8,
                                device=x.device)
    tail = (_ptr(wg_tiled), _ptr(wu_tiled) if wu_tiled is not None else None, _ptr(wd_tiled),
            _ptr(route.expert_offsets), _ptr(route.sel), _ptr(route.sel_w), _ptr(route.inv), slots,
            _ptr(y, torch.bfloat16), _ptr(workspace), workspace.numel(), _stream())
    head = (_ptr(x, torch.bfloat16), T, H, F, E_total, fmt)
    if activation != "silu" or not gated:
        _check(lib().ssmm_expert_ffn_variant(*head, ACTIVATIONS[activation], 1 if gated else 0, *tail, events),
               "ssmm_expert_ffn_variant")
    elif events is None:
        _check(lib().ssmm_expert_ffn(*head, *tail), "ssmm_expert_ffn")
    else:
        _check(lib().ssmm_expert_ffn_timed(*head, *tail, events), "ssmm_expert_ffn_timed")
    return y


def matmul(a_tiled, rows, K, fmt, b, sel=None, n=None, c=None, workspace=None):
    """C = A x B[:, SEL]: a_tiled = kernel-ready form of one rows x K matrix, b bf16 [n_b][K],
    sel i32 [n] or None (columns 0..n-1) -> c bf16 [n][rows]."""
    n_b = b.shape[0]
    if sel is not None:
        n = sel.numel()
    elif n is None:
        n = n_b
    if c is None:
        c = torch.empty((n, rows), dtype=torch.bfloat16, device=b.device)
    if workspace is None:
        workspace = torch.empty((int(lib().ssmm_matmul_workspace_bytes(rows, K, n, _fmt(fmt))),), dtype=torch.uint8,
                                device=b.device)
    _check(lib().ssmm_matmul(_ptr(a_tiled), rows, K, _fmt(fmt), _ptr(b, torch.bfloat16), n_b,
                             _ptr(sel, torch.int32) if sel is not None else None, n, _ptr(c, torch.bfloat16),
                             _ptr(workspace), workspace.numel(), _stream()), "ssmm_matmul")
    return c


class HipEvents:
    """Four hipEvent_t per step for ssmm_expert_ffn_timed, created straight from the HIP
    runtime (torch's events only see torch's own record calls)."""

    def __init__(self, steps):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [POINTER(c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [POINTER(ctypes.c_float), c_void_p, c_void_p]
        self.hip.hipEventDestroy.argtypes = [c_void_p]
        self.steps = []
        for _ in range(steps):
            arr = (c_void_p * 4)()
            for i in range(4):
                ev = c_void_p()
                if self.hip.hipEventCreate(ctypes.byref(ev)) != 0:
                    raise RuntimeError("hipEventCreate failed")
                arr[i] = ev
            self.steps.append(arr)

    def elapsed_ms(self):
        """Mean milliseconds of (gate/up, down, combine) over the recorded steps; call after a sync."""
        tot = [0.0, 0.0, 0.0]
        for arr in self.steps:
            for i in range(3):
                ms = ctypes.c_float(0)
                if self.hip.hipEventElapsedTime(ctypes.byref(ms), arr[i], arr[i + 1]) != 0:
                    raise RuntimeError("hipEventElapsedTime failed")
                tot[i] += ms.value
        return [t / len(self.steps) for t in tot]

    def close(self):
        for arr in self.steps:
            for i in range(4):
                self.hip.hipEventDestroy(arr[i])
        self.steps = []
