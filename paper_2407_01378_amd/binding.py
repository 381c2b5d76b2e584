"""ctypes binding of libthc.so: argument marshalling only.

Every function has the name and argument order of its C entry point in
include/thc.h and does no arithmetic of its own; PyTorch supplies device memory
and the stream.  The library must have been built (python -m
paper_2407_01378_amd.build): there is no fallback, a missing library raises.
"""
import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libthc.so")

THC_F32, THC_BF16 = 0, 1
THC_OK = 0

_lib = None

_u8pp = ctypes.POINTER(ctypes.c_void_p)


class ThcBucket(ctypes.Structure):
    """thc_bucket of include/thc.h."""
    _fields_ = [("grads", _u8pp), ("payloads", _u8pp), ("scale", ctypes.c_void_p),
                ("out", ctypes.c_void_p), ("n", ctypes.c_uint64), ("seed", ctypes.c_uint64)]


_bucketp = ctypes.POINTER(ThcBucket)
_SIGNATURES = {
    "thc_batch_workspace_bytes": (ctypes.c_uint64, [_bucketp, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint32]),
    "thc_encode_all_batch": (ctypes.c_int, [_bucketp, ctypes.c_uint32, ctypes.c_int, ctypes.c_uint32,
                                            ctypes.c_uint32, ctypes.c_uint32, ctypes.c_void_p, ctypes.c_uint64,
                                            ctypes.c_void_p]),
    "thc_aggregate_decode_batch": (ctypes.c_int, [_bucketp, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint32,
                                                  ctypes.c_uint32, ctypes.c_void_p, ctypes.c_uint64,
                                                  ctypes.c_void_p]),
    "thc_status_string": (ctypes.c_char_p, [ctypes.c_int]),
    "thc_version": (ctypes.c_int, []),
    "thc_rounding_bits": (ctypes.c_uint32, []),
    "thc_num_chunks": (ctypes.c_uint64, [ctypes.c_uint64, ctypes.c_uint32]),
    "thc_payload_bytes": (ctypes.c_uint64, [ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint32]),
    "thc_sum_bytes": (ctypes.c_uint32, [ctypes.c_uint32, ctypes.c_uint32]),
    "rht_forward": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64, ctypes.c_uint32,
                                   ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p]),
    "rht_inverse": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32,
                                   ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p]),
    "thc_chunk_absmax": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64,
                                        ctypes.c_uint32, ctypes.c_uint64, ctypes.c_void_p,
                                        ctypes.c_void_p]),
    "thc_scale_reduce": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64,
                                        ctypes.c_void_p, ctypes.c_void_p]),
    "thc_encode": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64, ctypes.c_uint32,
                                  ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint32,
                                  ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                  ctypes.c_void_p]),
    "thc_aggregate": (ctypes.c_int, [_u8pp, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_uint32,
                                     ctypes.c_uint32, ctypes.c_void_p, ctypes.c_void_p]),
    "thc_decode": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint32,
                                  ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint64,
                                  ctypes.c_uint32, ctypes.c_void_p, ctypes.c_void_p]),
    "thc_encode_all_workspace_bytes": (ctypes.c_uint64, [ctypes.c_uint32, ctypes.c_uint64,
                                                         ctypes.c_uint32]),
    "thc_encode_all": (ctypes.c_int, [_u8pp, ctypes.c_int, ctypes.c_uint32, ctypes.c_uint64,
                                      ctypes.c_uint32, ctypes.c_uint64, ctypes.c_uint32, _u8pp,
                                      ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64,
                                      ctypes.c_void_p]),
    "thc_encode_all_static": (ctypes.c_int, [_u8pp, ctypes.c_int, ctypes.c_uint32, ctypes.c_uint64,
                                             ctypes.c_uint32, ctypes.c_uint64, ctypes.c_uint32, _u8pp,
                                             ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]),
    "thc_workspace_clear": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p]),
    "thc_encode_all_cleared": (ctypes.c_int, [_u8pp, ctypes.c_int, ctypes.c_uint32, ctypes.c_uint64,
                                      ctypes.c_uint32, ctypes.c_uint64, ctypes.c_uint32, _u8pp,
                                      ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64,
                                      ctypes.c_void_p]),
    "thc_sat_encode_all_cleared": (ctypes.c_int, [_u8pp, ctypes.c_int, ctypes.c_uint32, ctypes.c_uint64,
                                      ctypes.c_uint32, ctypes.c_uint64, ctypes.c_uint32, _u8pp,
                                      ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64,
                                      ctypes.c_void_p]),
    "thc_set_spin_limit": (None, [ctypes.c_uint32]),
    "thc_aggregate_decode_is_fused": (ctypes.c_int, [ctypes.c_uint32, ctypes.c_uint32,
                                                     ctypes.c_uint32]),
    "thc_aggregate_decode": (ctypes.c_int, [_u8pp, ctypes.c_uint32, ctypes.c_void_p,
                                            ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint64,
                                            ctypes.c_uint32, ctypes.c_void_p, ctypes.c_void_p,
                                            ctypes.c_void_p]),
    "topkc_num_chunks": (ctypes.c_uint64, [ctypes.c_uint64, ctypes.c_uint32]),
    "topkc_chunk_norms": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64, ctypes.c_uint32,
                                         ctypes.c_void_p, ctypes.c_void_p]),
    "topkc_sum_norms": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_void_p,
                                       ctypes.c_void_p]),
    "topkc_select_workspace_bytes": (ctypes.c_uint64, [ctypes.c_uint64]),
    "topkc_select": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_void_p,
                                    ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p]),
    "topkc_gather_sum": (ctypes.c_int, [_u8pp, ctypes.c_int, ctypes.c_uint32, ctypes.c_uint64,
                                        ctypes.c_uint32, ctypes.c_void_p, ctypes.c_uint32, ctypes.c_void_p,
                                        ctypes.c_void_p]),
    "topkc_scatter_mean": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint32,
                                          ctypes.c_uint32, ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p]),
    "thc_chunk_minmax": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64, ctypes.c_uint32,
                                        ctypes.c_uint64, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]),
    "thc_range_reduce": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64,
                                        ctypes.c_void_p, ctypes.c_void_p]),
    "thc_encode_minmax": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64, ctypes.c_uint32,
                                         ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_int,
                                         ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]),
    "thc_decode_minmax": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint32,
                                         ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint64,
                                         ctypes.c_uint32, ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                         ctypes.c_void_p]),
    "thc_encode_all_minmax_workspace_bytes": (ctypes.c_uint64, [ctypes.c_uint32, ctypes.c_uint64,
                                                                ctypes.c_uint32]),
    "thc_encode_all_minmax": (ctypes.c_int, [_u8pp, ctypes.c_int, ctypes.c_uint32, ctypes.c_uint64,
                                             ctypes.c_uint32, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int,
                                             _u8pp, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64,
                                             ctypes.c_void_p]),
    "thc_aggregate_decode_minmax": (ctypes.c_int, [_u8pp, ctypes.c_uint32, ctypes.c_void_p, ctypes.c_uint64,
                                                   ctypes.c_uint32, ctypes.c_uint64, ctypes.c_uint32,
                                                   ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]),
    "thc_full_log2": (ctypes.c_uint32, [ctypes.c_uint64]),
    "rht_forward_full": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64, ctypes.c_uint32,
                                        ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p]),
    "rht_forward_full_absmax": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64, ctypes.c_uint32,
                                               ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]),
    "rht_forward_full_deferred": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64, ctypes.c_uint32,
                                                 ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]),
    "thc_full_encode_deferred": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint64,
                                                ctypes.c_uint32, ctypes.c_uint32, ctypes.c_void_p,
                                                ctypes.c_void_p, ctypes.c_void_p]),
    "rht_inverse_full": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32,
                                        ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p]),
    "thc_full_absmax": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_uint32, ctypes.c_void_p,
                                       ctypes.c_void_p]),
    "thc_full_encode": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64,
                                       ctypes.c_uint32, ctypes.c_uint32, ctypes.c_void_p,
                                       ctypes.c_void_p, ctypes.c_void_p]),
    "thc_full_decode": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint32,
                                       ctypes.c_uint32, ctypes.c_uint32, ctypes.c_void_p,
                                       ctypes.c_void_p]),
    "thc_full_decode_inverse": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint32,
                                               ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint64,
                                               ctypes.c_uint32, ctypes.c_void_p, ctypes.c_void_p,
                                               ctypes.c_void_p]),
    "thc_sat_max": (ctypes.c_uint32, [ctypes.c_uint32]),
    "thc_sat_encode": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64, ctypes.c_uint32,
                                      ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint32,
                                      ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                      ctypes.c_void_p]),
    "thc_sat_encode_all": (ctypes.c_int, [_u8pp, ctypes.c_int, ctypes.c_uint32, ctypes.c_uint64,
                                          ctypes.c_uint32, ctypes.c_uint64, ctypes.c_uint32, _u8pp,
                                          ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64,
                                          ctypes.c_void_p]),
    "thc_sat_aggregate": (ctypes.c_int, [_u8pp, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_uint32,
                                         ctypes.c_uint32, ctypes.c_void_p, ctypes.c_void_p,
                                         ctypes.c_void_p]),
    "thc_sat_decode": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint32,
                                      ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint64,
                                      ctypes.c_uint32, ctypes.c_void_p, ctypes.c_void_p]),
    "thc_sat_aggregate_decode_is_fused": (ctypes.c_int, [ctypes.c_uint32, ctypes.c_uint32,
                                                         ctypes.c_uint32]),
    "thc_sat_aggregate_decode": (ctypes.c_int, [_u8pp, ctypes.c_uint32, ctypes.c_void_p,
                                                ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint64,
                                                ctypes.c_uint32, ctypes.c_void_p, ctypes.c_void_p,
                                                ctypes.c_void_p, ctypes.c_void_p]),
}


class ThcError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


def lib():
    """The loaded shared library (loads it on first use; raises if it is not built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2407_01378_amd.build`; "
                "there is no fallback path")
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype = res
            fn.argtypes = args
        _lib = handle
    return _lib


def exported_names():
    return sorted(_SIGNATURES)


def status_string(status):
    return lib().thc_status_string(int(status)).decode()


def _check(status, where):
    if status != THC_OK:
        raise ThcError(status, where)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _dtype_code(t):
    if t.dtype == torch.float32:
        return THC_F32
    if t.dtype == torch.bfloat16:
        return THC_BF16
    raise TypeError(f"gradient dtype {t.dtype} is not fp32 or bf16")


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _flat(t, dtype=None):
    if not t.is_contiguous() or t.dim() != 1:
        raise ValueError("expected a contiguous 1-D tensor")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {t.dtype}")
    return t


# ------------------------------------------------------------------ size helpers
def thc_version():
    return lib().thc_version()


def thc_rounding_bits():
    return lib().thc_rounding_bits()


def thc_num_chunks(n, chunk_log2):
    return lib().thc_num_chunks(n, chunk_log2)


def thc_payload_bytes(n, chunk_log2, bits):
    return lib().thc_payload_bytes(n, chunk_log2, bits)


def thc_sum_bytes(W, bits):
    return lib().thc_sum_bytes(W, bits)


# ------------------------------------------------------------------- entry points
def rht_forward(x, chunk_log2, seed, y, stream=None):
    _flat(x), _flat(y, torch.float32)
    _check(lib().rht_forward(_ptr(x), _dtype_code(x), x.numel(), chunk_log2, seed, _ptr(y),
                             _stream(stream)), "rht_forward")
    return y


def rht_inverse(y, n, chunk_log2, seed, x, stream=None):
    _flat(y, torch.float32), _flat(x, torch.float32)
    _check(lib().rht_inverse(_ptr(y), n, chunk_log2, seed, _ptr(x), _stream(stream)),
           "rht_inverse")
    return x


def thc_chunk_absmax(grad, chunk_log2, seed, absmax, stream=None):
    _flat(grad), _flat(absmax, torch.float32)
    _check(lib().thc_chunk_absmax(_ptr(grad), _dtype_code(grad), grad.numel(), chunk_log2, seed,
                                  _ptr(absmax), _stream(stream)), "thc_chunk_absmax")
    return absmax


def thc_scale_reduce(absmax_all, W, chunks, scale, stream=None):
    _check(lib().thc_scale_reduce(_ptr(absmax_all), W, chunks, _ptr(scale), _stream(stream)),
           "thc_scale_reduce")
    return scale


def thc_encode(grad, chunk_log2, seed, worker, bits, shared_scale, payload, scale_out=None,
               stream=None):
    _flat(grad), _flat(payload, torch.uint8)
    _check(lib().thc_encode(_ptr(grad), _dtype_code(grad), grad.numel(), chunk_log2, seed, worker,
                            bits, _ptr(shared_scale), _ptr(payload), _ptr(scale_out),
                            _stream(stream)), "thc_encode")
    return payload


def thc_aggregate(payloads, n, chunk_log2, bits, sums, stream=None):
    W = len(payloads)
    arr = (ctypes.c_void_p * max(W, 1))(*[p.data_ptr() for p in payloads])
    _check(lib().thc_aggregate(ctypes.cast(arr, _u8pp), W, n, chunk_log2, bits, _ptr(sums),
                               _stream(stream)), "thc_aggregate")
    return sums


def thc_decode(sums, scale, W, n, chunk_log2, seed, bits, out, stream=None):
    _flat(out, torch.float32)
    _check(lib().thc_decode(_ptr(sums), _ptr(scale), W, n, chunk_log2, seed, bits, _ptr(out),
                            _stream(stream)), "thc_decode")
    return out


# ------------------------------------------------------------- batched / fused forms
def _ptr_array(tensors):
    arr = (ctypes.c_void_p * max(len(tensors), 1))(*[t.data_ptr() for t in tensors])
    return arr, ctypes.cast(arr, _u8pp)


def thc_encode_all_workspace_bytes(W, n, chunk_log2):
    return lib().thc_encode_all_workspace_bytes(W, n, chunk_log2)


def _encode_all(name, grads, chunk_log2, seed, bits, payloads, scale, workspace, stream, check=False):
    """check=True synchronises the device after the call and raises ThcError(-7) if a bounded
    wait between workgroups expired (the workspace's first word); marshalling otherwise."""
    W = len(grads)
    n = grads[0].numel()
    for g in grads:
        _flat(g)
        if g.numel() != n or g.dtype != grads[0].dtype:
            raise ValueError("all workers must have gradients of one size and dtype")
    keep_g, pg = _ptr_array(grads)
    keep_p, pp = _ptr_array(payloads)
    _check(getattr(lib(), name)(pg, _dtype_code(grads[0]), W, n, chunk_log2, seed, bits, pp,
                                _ptr(scale), _ptr(workspace),
                                workspace.numel() * workspace.element_size(), _stream(stream)),
           name)
    if check:
        torch.cuda.synchronize(workspace.device)
        if thc_encode_all_timed_out(workspace):
            raise ThcError(-7, name + " (a bounded wait between workgroups expired)")
    return payloads


def thc_encode_all(grads, chunk_log2, seed, bits, payloads, scale, workspace, stream=None, check=False):
    return _encode_all("thc_encode_all", grads, chunk_log2, seed, bits, payloads, scale, workspace, stream, check)


def thc_encode_all_cleared(grads, chunk_log2, seed, bits, payloads, scale, workspace, stream=None, check=False):
    return _encode_all("thc_encode_all_cleared", grads, chunk_log2, seed, bits, payloads, scale,
                       workspace, stream, check)


# ------------------------------------------------------------ several buckets per launch
def _bucket_array(buckets):
    """buckets: list of dicts with keys n, seed and any of grads (list of W tensors), payloads
    (list of W tensors), scale, out.  Returns (keep-alive objects, ctypes array)."""
    arr = (ThcBucket * max(len(buckets), 1))()
    keep = []
    for i, b in enumerate(buckets):
        if b.get("grads") is not None:
            kg, pg = _ptr_array(b["grads"])
            keep.append(kg)
            arr[i].grads = pg
        if b.get("payloads") is not None:
            kp, pp = _ptr_array(b["payloads"])
            keep.append(kp)
            arr[i].payloads = pp
        arr[i].scale = None if b.get("scale") is None else b["scale"].data_ptr()
        arr[i].out = None if b.get("out") is None else b["out"].data_ptr()
        arr[i].n = int(b["n"])
        arr[i].seed = int(b.get("seed", 0))
    return keep, arr


def thc_batch_workspace_bytes(ns, W, chunk_log2):
    keep, arr = _bucket_array([dict(n=n) for n in ns])
    return lib().thc_batch_workspace_bytes(arr, len(ns), W, chunk_log2)


def thc_encode_all_batch(buckets, chunk_log2, bits, workspace, stream=None):
    W = len(buckets[0]["grads"]) if buckets else 1
    keep, arr = _bucket_array(buckets)
    dt = _dtype_code(buckets[0]["grads"][0]) if buckets else THC_F32
    _check(lib().thc_encode_all_batch(arr, len(buckets), dt, W, chunk_log2, bits, _ptr(workspace),
                                      workspace.numel() * workspace.element_size(), _stream(stream)),
           "thc_encode_all_batch")


def thc_aggregate_decode_batch(buckets, chunk_log2, bits, workspace, stream=None):
    W = len(buckets[0]["payloads"]) if buckets else 1
    keep, arr = _bucket_array(buckets)
    _check(lib().thc_aggregate_decode_batch(arr, len(buckets), W, chunk_log2, bits, _ptr(workspace),
                                            workspace.numel() * workspace.element_size(), _stream(stream)),
           "thc_aggregate_decode_batch")


THC_STATIC_SCRATCH_BYTES = 2 << 20


def thc_encode_all_static(grads, chunk_log2, seed, bits, payloads, scale, timed_out=None, stream=None):
    W = len(grads)
    n = grads[0].numel()
    for g in grads:
        _flat(g)
        if g.numel() != n or g.dtype != grads[0].dtype:
            raise ValueError("all workers must have gradients of one size and dtype")
    keep_g, pg = _ptr_array(grads)
    keep_p, pp = _ptr_array(payloads)
    _check(lib().thc_encode_all_static(pg, _dtype_code(grads[0]), W, n, chunk_log2, seed, bits, pp,
                                       _ptr(scale), _ptr(timed_out), _stream(stream)),
           "thc_encode_all_static")
    return payloads


def thc_workspace_clear(workspace, stream=None):
    _flat(workspace)
    _check(lib().thc_workspace_clear(_ptr(workspace), workspace.numel() * workspace.element_size(),
                                     _stream(stream)), "thc_workspace_clear")
    return workspace


def thc_encode_all_timed_out(workspace):
    """Reads the workspace's error word (synchronises): True if a bounded wait expired."""
    return bool(workspace.view(torch.uint8)[:4].cpu().numpy().view("<u4")[0])


def thc_set_spin_limit(polls):
    lib().thc_set_spin_limit(polls)


def thc_aggregate_decode_is_fused(W, chunk_log2, bits):
    return bool(lib().thc_aggregate_decode_is_fused(W, chunk_log2, bits))


def thc_aggregate_decode(payloads, scale, n, chunk_log2, seed, bits, sums, out, stream=None):
    W = len(payloads)
    keep_p, pp = _ptr_array(payloads)
    _flat(out, torch.float32)
    _check(lib().thc_aggregate_decode(pp, W, _ptr(scale), n, chunk_log2, seed, bits, _ptr(sums),
                                      _ptr(out), _stream(stream)), "thc_aggregate_decode")
    return out


# ------------------------------------------------------ saturation-based aggregation
def thc_sat_max(bits):
    return lib().thc_sat_max(bits)


def thc_sat_encode(grad, chunk_log2, seed, worker, bits, shared_scale, payload, scale_out=None,
                   stream=None):
    _flat(grad), _flat(payload, torch.uint8)
    _check(lib().thc_sat_encode(_ptr(grad), _dtype_code(grad), grad.numel(), chunk_log2, seed,
                                worker, bits, _ptr(shared_scale), _ptr(payload), _ptr(scale_out),
                                _stream(stream)), "thc_sat_encode")
    return payload


def thc_sat_encode_all(grads, chunk_log2, seed, bits, payloads, scale, workspace, stream=None, check=False):
    return _encode_all("thc_sat_encode_all", grads, chunk_log2, seed, bits, payloads, scale, workspace,
                       stream, check)


def thc_sat_encode_all_cleared(grads, chunk_log2, seed, bits, payloads, scale, workspace, stream=None, check=False):
    return _encode_all("thc_sat_encode_all_cleared", grads, chunk_log2, seed, bits, payloads, scale,
                       workspace, stream, check)


def thc_sat_aggregate(payloads, n, chunk_log2, bits, aggregate, overflow_count=None, stream=None):
    keep_p, pp = _ptr_array(payloads)
    _check(lib().thc_sat_aggregate(pp, len(payloads), n, chunk_log2, bits, _ptr(aggregate),
                                   _ptr(overflow_count), _stream(stream)), "thc_sat_aggregate")
    return aggregate


def thc_sat_decode(aggregate, scale, W, n, chunk_log2, seed, bits, out, stream=None):
    _flat(out, torch.float32)
    _check(lib().thc_sat_decode(_ptr(aggregate), _ptr(scale), W, n, chunk_log2, seed, bits,
                                _ptr(out), _stream(stream)), "thc_sat_decode")
    return out


def thc_sat_aggregate_decode_is_fused(W, chunk_log2, bits):
    return bool(lib().thc_sat_aggregate_decode_is_fused(W, chunk_log2, bits))


def thc_sat_aggregate_decode(payloads, scale, n, chunk_log2, seed, bits, aggregate, overflow_count,
                             out, stream=None):
    keep_p, pp = _ptr_array(payloads)
    _flat(out, torch.float32)
    _check(lib().thc_sat_aggregate_decode(pp, len(payloads), _ptr(scale), n, chunk_log2, seed, bits,
                                          _ptr(aggregate), _ptr(overflow_count), _ptr(out),
                                          _stream(stream)), "thc_sat_aggregate_decode")
    return out


# -------------------------------------------------------------------- full rotation
def thc_full_log2(n):
    return lib().thc_full_log2(n)


def rht_forward_full_absmax(x, log2_size, seed, y, absmax, stream=None):
    _flat(x), _flat(y, torch.float32), _flat(absmax, torch.float32)
    _check(lib().rht_forward_full_absmax(_ptr(x), _dtype_code(x), x.numel(), log2_size, seed, _ptr(y),
                                         _ptr(absmax), _stream(stream)), "rht_forward_full_absmax")
    return y


def rht_forward_full_deferred(x, log2_size, seed, y, absmax, stream=None):
    """Every pass but the last in y, the last one evaluated for absmax only."""
    _flat(x), _flat(y, torch.float32), _flat(absmax, torch.float32)
    _check(lib().rht_forward_full_deferred(_ptr(x), _dtype_code(x), x.numel(), log2_size, seed, _ptr(y),
                                           _ptr(absmax), _stream(stream)), "rht_forward_full_deferred")
    return y


def thc_full_encode_deferred(y, n, log2_size, seed, worker, bits, scale, payload, stream=None):
    """The last pass on the y of rht_forward_full_deferred, quantized into payload."""
    _check(lib().thc_full_encode_deferred(_ptr(y), n, log2_size, seed, worker, bits, _ptr(scale), _ptr(payload),
                                          _stream(stream)), "thc_full_encode_deferred")
    return payload


def rht_forward_full(x, log2_size, seed, y, stream=None):
    _flat(x), _flat(y, torch.float32)
    _check(lib().rht_forward_full(_ptr(x), _dtype_code(x), x.numel(), log2_size, seed, _ptr(y),
                                  _stream(stream)), "rht_forward_full")
    return y


def rht_inverse_full(y, n, log2_size, seed, x, stream=None):
    _flat(y, torch.float32), _flat(x, torch.float32)
    _check(lib().rht_inverse_full(_ptr(y), n, log2_size, seed, _ptr(x), _stream(stream)),
           "rht_inverse_full")
    return x


def thc_full_absmax(y, log2_size, absmax, stream=None):
    _check(lib().thc_full_absmax(_ptr(y), log2_size, _ptr(absmax), _stream(stream)), "thc_full_absmax")
    return absmax


def thc_full_encode(y, log2_size, seed, worker, bits, scale, payload, stream=None):
    _check(lib().thc_full_encode(_ptr(y), log2_size, seed, worker, bits, _ptr(scale), _ptr(payload),
                                 _stream(stream)), "thc_full_encode")
    return payload


def thc_full_decode(sums, scale, W, log2_size, bits, yhat, stream=None):
    _check(lib().thc_full_decode(_ptr(sums), _ptr(scale), W, log2_size, bits, _ptr(yhat),
                                 _stream(stream)), "thc_full_decode")
    return yhat


def thc_full_decode_inverse(sums, scale, W, n, log2_size, seed, bits, work, x, stream=None):
    """thc_full_decode + rht_inverse_full in one call; `work` is 2^log2_size fp32 of scratch."""
    _check(lib().thc_full_decode_inverse(_ptr(sums), _ptr(scale), W, n, log2_size, seed, bits, _ptr(work),
                                         _ptr(x), _stream(stream)), "thc_full_decode_inverse")
    return x


# -------------------------------------------------------------------- min/max range
def thc_chunk_minmax(grad, chunk_log2, seed, rotate, range_out, stream=None):
    _flat(grad), _flat(range_out, torch.float32)
    _check(lib().thc_chunk_minmax(_ptr(grad), _dtype_code(grad), grad.numel(), chunk_log2, seed,
                                  int(bool(rotate)), _ptr(range_out), _stream(stream)), "thc_chunk_minmax")
    return range_out


def thc_range_reduce(range_all, W, chunks, range_out, stream=None):
    _check(lib().thc_range_reduce(_ptr(range_all), W, chunks, _ptr(range_out), _stream(stream)),
           "thc_range_reduce")
    return range_out


def thc_encode_minmax(grad, chunk_log2, seed, worker, bits, rotate, range_, payload, stream=None):
    _flat(grad), _flat(payload, torch.uint8)
    _check(lib().thc_encode_minmax(_ptr(grad), _dtype_code(grad), grad.numel(), chunk_log2, seed, worker,
                                   bits, int(bool(rotate)), _ptr(range_), _ptr(payload), _stream(stream)),
           "thc_encode_minmax")
    return payload


def thc_decode_minmax(sums, range_, W, n, chunk_log2, seed, bits, rotate, out, stream=None):
    _flat(out)
    _check(lib().thc_decode_minmax(_ptr(sums), _ptr(range_), W, n, chunk_log2, seed, bits,
                                   int(bool(rotate)), _dtype_code(out), _ptr(out), _stream(stream)),
           "thc_decode_minmax")
    return out


def thc_encode_all_minmax_workspace_bytes(W, n, chunk_log2):
    return lib().thc_encode_all_minmax_workspace_bytes(W, n, chunk_log2)


def thc_encode_all_minmax(grads, chunk_log2, seed, bits, rotate, payloads, range_, workspace, stream=None):
    W = len(grads)
    n = grads[0].numel()
    for g in grads:
        _flat(g)
        if g.numel() != n or g.dtype != grads[0].dtype:
            raise ValueError("all workers must have gradients of one size and dtype")
    keep_g, pg = _ptr_array(grads)
    keep_p, pp = _ptr_array(payloads)
    _check(lib().thc_encode_all_minmax(pg, _dtype_code(grads[0]), W, n, chunk_log2, seed, bits,
                                       int(bool(rotate)), pp, _ptr(range_), _ptr(workspace),
                                       workspace.numel() * workspace.element_size(), _stream(stream)),
           "thc_encode_all_minmax")


def thc_aggregate_decode_minmax(payloads, range_, n, chunk_log2, seed, bits, rotate, out, stream=None):
    W = len(payloads)
    keep_p, pp = _ptr_array(payloads)
    _flat(out, torch.float32)
    _check(lib().thc_aggregate_decode_minmax(pp, W, _ptr(range_), n, chunk_log2, seed, bits,
                                             int(bool(rotate)), _ptr(out), _stream(stream)),
           "thc_aggregate_decode_minmax")
    return out


# ---------------------------------------------------------------------------- TopKC
def topkc_num_chunks(n, C):
    return lib().topkc_num_chunks(n, C)


def topkc_chunk_norms(grad, C, norms, stream=None):
    _flat(grad), _flat(norms, torch.float16)
    _check(lib().topkc_chunk_norms(_ptr(grad), _dtype_code(grad), grad.numel(), C, _ptr(norms),
                                   _stream(stream)), "topkc_chunk_norms")
    return norms


def topkc_sum_norms(norms_all, W, P, s, stream=None):
    _check(lib().topkc_sum_norms(_ptr(norms_all), W, P, _ptr(s), _stream(stream)), "topkc_sum_norms")
    return s


def topkc_select_workspace_bytes(P):
    return lib().topkc_select_workspace_bytes(P)


def topkc_select(s, J, indices, workspace, stream=None):
    _flat(s, torch.float16), _flat(indices, torch.int32)
    _check(lib().topkc_select(_ptr(s), s.numel(), J, _ptr(indices), _ptr(workspace),
                              workspace.numel() * workspace.element_size(), _stream(stream)), "topkc_select")
    return indices


def topkc_gather_sum(grads, C, indices, J, values, stream=None):
    keep, pg = _ptr_array(grads)
    _flat(values, torch.float16)
    _check(lib().topkc_gather_sum(pg, _dtype_code(grads[0]), len(grads), grads[0].numel(), C, _ptr(indices), J,
                                  _ptr(values), _stream(stream)), "topkc_gather_sum")
    return values


def topkc_scatter_mean(values, indices, J, C, W, out, stream=None):
    _flat(out, torch.float32)
    _check(lib().topkc_scatter_mean(_ptr(values), _ptr(indices), J, C, W, out.numel(), _ptr(out),
                                    _stream(stream)), "topkc_scatter_mean")
    return out
