"""CPU-only checks of the C ABI: the library loads, exports every function the
header declares, and rejects bad arguments on the host before any HIP call (so no
GPU is needed: none of these calls may reach a launch)."""
import ctypes
import os
import re

import pytest

import paper_2407_01378_amd as thc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "thc.h")


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(thc.binding.LIB_PATH):
        from paper_2407_01378_amd.build import build_library
        build_library(verbose=False)
    return thc.lib()


def _declared():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    names = re.findall(r"\b([a-z_0-9]+)\s*\(", src)
    return sorted({n for n in names if n.startswith(("thc_", "rht_", "topkc_"))})


def test_every_declared_function_is_exported_and_bound(L):
    declared = _declared()
    assert {"rht_forward", "rht_inverse", "thc_chunk_absmax", "thc_scale_reduce", "thc_encode",
            "thc_aggregate", "thc_decode", "thc_status_string", "thc_version", "thc_num_chunks",
            "thc_payload_bytes", "thc_sum_bytes"} <= set(declared)
    for name in declared:
        assert hasattr(L, name), name
    assert sorted(thc.exported_names()) == declared


def test_size_helpers(L):
    assert thc.thc_version() >= 100
    assert thc.thc_rounding_bits() == 8
    assert thc.thc_num_chunks(0, 14) == 0
    assert thc.thc_num_chunks(1, 14) == 1
    assert thc.thc_num_chunks(1 << 14, 14) == 1
    assert thc.thc_num_chunks((1 << 14) + 1, 14) == 2
    assert thc.thc_num_chunks(25_557_032, 14) == 1560
    assert thc.thc_num_chunks(1_300_000_000, 14) == 79346
    assert thc.thc_num_chunks(10, 0) == 0 and thc.thc_num_chunks(10, 15) == 0
    assert thc.thc_payload_bytes(25_557_032, 14, 4) == 1560 * 8192
    assert thc.thc_payload_bytes(1 << 20, 10, 2) == (1 << 20) // 4
    assert thc.thc_payload_bytes(3, 1, 2) == 1          # 4 coordinates of 2 bits
    assert thc.thc_payload_bytes(1, 1, 2) == 1          # half a byte is counted whole
    assert thc.thc_payload_bytes(10, 14, 3) == 0
    assert thc.thc_sum_bytes(4, 4) == 1 and thc.thc_sum_bytes(8, 4) == 1
    assert thc.thc_sum_bytes(17, 4) == 1 and thc.thc_sum_bytes(18, 4) == 2
    assert thc.thc_sum_bytes(8, 8) == 2 and thc.thc_sum_bytes(257, 8) == 2
    assert thc.thc_sum_bytes(258, 8) == 0 and thc.thc_sum_bytes(0, 4) == 0
    assert thc.thc_sum_bytes(8, 5) == 0


def test_status_strings(L):
    seen = set()
    for code in range(0, -9, -1):
        s = thc.status_string(code)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 9
    assert thc.status_string(-99) == "unknown status"


def test_bad_arguments_are_rejected_on_the_host(L):
    """Dummy non-null addresses are never dereferenced: every call below must fail
    validation (or be a no-op) before anything is enqueued."""
    p = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1001)
    nul = ctypes.c_void_p(0)
    F32, BF16 = thc.THC_F32, thc.THC_BF16
    # chunk_log2
    assert L.rht_forward(p, F32, 100, 0, 0, p, nul) == -3
    assert L.rht_forward(p, F32, 100, 15, 0, p, nul) == -3
    assert L.rht_inverse(p, 100, 15, 0, p, nul) == -3
    assert L.thc_chunk_absmax(p, F32, 100, 20, 0, p, nul) == -3
    # dtype
    assert L.rht_forward(p, 7, 100, 10, 0, p, nul) == -5
    assert L.thc_encode(p, 2, 100, 10, 0, 0, 4, nul, p, nul, nul) == -5
    # bits
    for bad in (0, 1, 3, 5, 16):
        assert L.thc_encode(p, F32, 100, 10, 0, 0, bad, nul, p, nul, nul) == -2
        assert L.thc_decode(p, p, 4, 100, 10, 0, bad, p, nul) == -2
    # workers
    arr = (ctypes.c_void_p * 1)(0x1000)
    pp = ctypes.cast(arr, ctypes.POINTER(ctypes.c_void_p))
    assert L.thc_aggregate(pp, 0, 100, 10, 4, p, nul) == -4
    assert L.thc_aggregate(pp, 4370, 100, 10, 4, p, nul) == -4      # 4370 * 15 = 65550
    assert L.thc_decode(p, p, 0, 100, 10, 0, 4, p, nul) == -4
    assert L.thc_decode(p, p, 258, 100, 10, 0, 8, p, nul) == -4
    assert L.thc_scale_reduce(p, 0, 10, p, nul) == -4
    # size
    assert L.rht_forward(p, F32, 1 << 50, 10, 0, p, nul) == -6
    # n == 0: success, nothing touched, even with null buffers
    assert L.rht_forward(nul, F32, 0, 10, 0, nul, nul) == 0
    assert L.rht_inverse(nul, 0, 10, 0, nul, nul) == 0
    assert L.thc_chunk_absmax(nul, BF16, 0, 14, 0, nul, nul) == 0
    assert L.thc_encode(nul, F32, 0, 10, 0, 0, 4, nul, nul, nul, nul) == 0
    assert L.thc_aggregate(pp, 1, 0, 10, 4, nul, nul) == 0
    assert L.thc_decode(nul, nul, 4, 0, 10, 0, 4, nul, nul) == 0
    assert L.thc_scale_reduce(nul, 4, 0, nul, nul) == 0
    # null pointers
    assert L.rht_forward(nul, F32, 100, 10, 0, p, nul) == -1
    assert L.rht_forward(p, F32, 100, 10, 0, nul, nul) == -1
    assert L.rht_inverse(p, 100, 10, 0, nul, nul) == -1
    assert L.thc_chunk_absmax(p, F32, 100, 10, 0, nul, nul) == -1
    assert L.thc_scale_reduce(nul, 4, 10, p, nul) == -1
    assert L.thc_encode(p, F32, 100, 10, 0, 0, 4, nul, nul, nul, nul) == -1
    assert L.thc_aggregate(ctypes.cast(nul, ctypes.POINTER(ctypes.c_void_p)), 1, 100, 10, 4, p, nul) == -1
    arr0 = (ctypes.c_void_p * 2)(0x1000, 0)
    assert L.thc_aggregate(ctypes.cast(arr0, ctypes.POINTER(ctypes.c_void_p)), 2, 100, 10, 4, p, nul) == -1
    assert L.thc_decode(p, nul, 4, 100, 10, 0, 4, p, nul) == -1
    # alignment
    assert L.rht_forward(odd, F32, 100, 10, 0, p, nul) == -8
    assert L.rht_forward(ctypes.c_void_p(0x1002), F32, 100, 10, 0, p, nul) == -8
    assert L.rht_forward(odd, BF16, 100, 10, 0, p, nul) == -8
    assert L.thc_encode(p, F32, 100, 10, 0, 0, 4, nul, ctypes.c_void_p(0x1008), nul, nul) == -8
    assert L.thc_decode(ctypes.c_void_p(0x1004), p, 4, 100, 10, 0, 4, p, nul) == -8
    arr1 = (ctypes.c_void_p * 1)(0x1004)
    assert L.thc_aggregate(ctypes.cast(arr1, ctypes.POINTER(ctypes.c_void_p)), 1, 100, 10, 4, p, nul) == -8


def test_cleared_workspace_entry_points_validate_on_the_host(L):
    p, nul = ctypes.c_void_p(0x1000), ctypes.c_void_p(0)
    assert L.thc_workspace_clear(nul, 0, nul) == 0                 # nothing to clear
    assert L.thc_workspace_clear(nul, 64, nul) == -1
    assert L.thc_workspace_clear(ctypes.c_void_p(0x1004), 64, nul) == -8
    assert L.thc_workspace_clear(p, 62, nul) == -8                  # not whole words
    arr = (ctypes.c_void_p * 2)(0x1000, 0x2000)
    pp = ctypes.cast(arr, ctypes.POINTER(ctypes.c_void_p))
    for fn in (L.thc_encode_all_cleared, L.thc_sat_encode_all_cleared):
        assert fn(pp, thc.THC_BF16, 2, 100, 14, 0, 3, pp, p, p, 1 << 20, nul) == -2      # bits
        assert fn(pp, thc.THC_BF16, 2, 100, 15, 0, 4, pp, p, p, 1 << 20, nul) == -3      # chunk
        assert fn(pp, 9, 2, 100, 14, 0, 4, pp, p, p, 1 << 20, nul) == -5                 # dtype
        assert fn(pp, thc.THC_BF16, 2, 0, 14, 0, 4, pp, p, p, 0, nul) == 0               # n = 0
        assert fn(pp, thc.THC_BF16, 2, 100, 14, 0, 4, pp, p, nul, 1 << 20, nul) == -1    # workspace
        assert fn(pp, thc.THC_BF16, 2, 100, 14, 0, 4, pp, p, p, 8, nul) == -6            # too small
    # one arrival counter per chunk on top of the range words
    assert L.thc_encode_all_workspace_bytes(8, 1 << 14, 14) == 16 + 4 * (8 * 8 + 1)


def test_binding_refuses_to_run_without_the_library(monkeypatch, tmp_path):
    import paper_2407_01378_amd.binding as B
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        B.lib()


def test_sat_entry_points_validate_on_the_host(L):
    p = ctypes.c_void_p(0x1000)
    nul = ctypes.c_void_p(0)
    F32 = thc.THC_F32
    assert [L.thc_sat_max(b) for b in (2, 4, 8, 3)] == [1, 7, 127, 0]
    arr = (ctypes.c_void_p * 65)(*([0x1000] * 65))
    pp = ctypes.cast(arr, ctypes.POINTER(ctypes.c_void_p))
    # workers: 1..64
    assert L.thc_sat_aggregate(pp, 0, 100, 10, 4, p, nul, nul) == -4
    assert L.thc_sat_aggregate(pp, 65, 100, 10, 4, p, nul, nul) == -4
    assert L.thc_sat_aggregate_decode(pp, 65, p, 100, 14, 0, 4, p, nul, p, nul) == -4
    assert L.thc_sat_decode(p, p, 0, 100, 10, 0, 4, p, nul) == -4
    # bits, chunk, dtype
    assert L.thc_sat_aggregate(pp, 4, 100, 10, 3, p, nul, nul) == -2
    assert L.thc_sat_decode(p, p, 4, 100, 15, 0, 4, p, nul) == -3
    assert L.thc_sat_encode(p, 9, 100, 10, 0, 0, 4, nul, p, nul, nul) == -5
    # null / alignment
    assert L.thc_sat_aggregate(pp, 4, 100, 10, 4, nul, nul, nul) == -1
    assert L.thc_sat_aggregate(pp, 4, 100, 10, 4, ctypes.c_void_p(0x1008), nul, nul) == -8
    assert L.thc_sat_aggregate(pp, 4, 100, 10, 4, p, ctypes.c_void_p(0x1004), nul) == -8
    assert L.thc_sat_decode(nul, p, 4, 100, 10, 0, 4, p, nul) == -1
    assert L.thc_sat_aggregate_decode(pp, 4, p, 100, 10, 0, 4, nul, nul, p, nul) == -1   # unfused shape needs it
    assert L.thc_sat_aggregate_decode(pp, 4, nul, 100, 14, 0, 4, nul, nul, p, nul) == -1
    # n == 0
    assert L.thc_sat_aggregate(pp, 4, 0, 10, 4, nul, nul, nul) == 0
    assert L.thc_sat_decode(nul, nul, 4, 0, 10, 0, 4, nul, nul) == 0
    assert L.thc_sat_aggregate_decode(pp, 4, nul, 0, 14, 0, 4, nul, nul, nul, nul) == 0
    assert L.thc_sat_encode(nul, F32, 0, 10, 0, 0, 4, nul, nul, nul, nul) == 0
    assert L.thc_sat_aggregate_decode_is_fused(8, 14, 4) == 1
    assert L.thc_sat_aggregate_decode_is_fused(8, 10, 4) == 0
    assert L.thc_sat_aggregate_decode_is_fused(65, 14, 4) == 0


def test_batched_and_static_entry_points_validate_on_the_host(L):
    """Every call below fails validation, or has nothing to do, before any HIP call."""
    p = ctypes.c_void_p(0x1000)
    nul = ctypes.c_void_p(0)
    F32, BF16 = thc.THC_F32, thc.THC_BF16

    def buckets(*ns, ptr=0x1000, W=4):
        arr = (thc.binding.ThcBucket * max(len(ns), 1))()
        keep = []
        for i, n in enumerate(ns):
            g = (ctypes.c_void_p * W)(*([ptr] * W))
            q = (ctypes.c_void_p * W)(*([ptr] * W))
            keep += [g, q]
            arr[i].grads = ctypes.cast(g, type(arr[i].grads))
            arr[i].payloads = ctypes.cast(q, type(arr[i].payloads))
            arr[i].scale = 0x1000
            arr[i].out = 0x1000
            arr[i].n = n
            arr[i].seed = i
        return keep, arr

    keep, one = buckets(100)
    # sizes: 16-byte header, one record of 40 + 16 W bytes rounded up to 16, (8 W + 1) words per chunk
    assert L.thc_batch_workspace_bytes(one, 1, 4, 14) == 16 + 112 + 4 * (8 * 4 + 1)
    assert L.thc_batch_workspace_bytes(one, 1, 4, 10) == 0
    assert L.thc_batch_workspace_bytes(one, 0, 4, 14) == 16
    for fn, extra in ((L.thc_encode_all_batch, (F32,)), (L.thc_aggregate_decode_batch, ())):
        def call(arr, count, W, l, bits, ws, ws_bytes):
            return fn(arr, count, *extra, W, l, bits, ws, ws_bytes, nul)
        assert call(one, 1, 4, 10, 4, p, 1 << 20) == -3          # chunk size
        assert call(one, 1, 4, 14, 3, p, 1 << 20) == -2          # bits
        assert call(one, 1, 0, 14, 4, p, 1 << 20) == -4          # workers
        assert call(one, 1, 65, 14, 2, p, 1 << 20) == -4
        assert call(one, 4097, 4, 14, 4, p, 1 << 20) == -6       # too many buckets
        assert call(ctypes.cast(nul, ctypes.POINTER(thc.binding.ThcBucket)), 1, 4, 14, 4, p, 1 << 20) == -1
        assert call(one, 1, 4, 14, 4, nul, 1 << 20) == -1        # workspace
        assert call(one, 1, 4, 14, 4, ctypes.c_void_p(0x1004), 1 << 20) == -8
        assert call(one, 1, 4, 14, 4, p, 16) == -6               # workspace too small
        assert call(one, 0, 4, 14, 4, nul, 0) == 0               # nothing to do
        keep0, empty = buckets(0, 0)
        assert call(empty, 2, 4, 14, 4, nul, 0) == 0
        keep1, odd = buckets(100, ptr=0x1008)
        assert call(odd, 1, 4, 14, 4, p, 1 << 20) == -8          # unaligned bucket pointers
    assert L.thc_encode_all_batch(one, 1, 9, 4, 14, 4, p, 1 << 20, nul) == -5
    assert L.thc_aggregate_decode_batch(one, 1, 1, 14, 8, p, 1 << 20, nul) == -4    # one worker of 8-bit payloads: not fused

    # static-scratch form
    g = (ctypes.c_void_p * 4)(*([0x1000] * 4))
    pg = ctypes.cast(g, ctypes.POINTER(ctypes.c_void_p))
    assert thc.THC_STATIC_SCRATCH_BYTES == 2 << 20
    assert L.thc_encode_all_static(pg, F32, 4, 100, 15, 0, 4, pg, p, nul, nul) == -3
    assert L.thc_encode_all_static(pg, 5, 4, 100, 14, 0, 4, pg, p, nul, nul) == -5
    assert L.thc_encode_all_static(pg, F32, 4, 100, 14, 0, 7, pg, p, nul, nul) == -2
    assert L.thc_encode_all_static(pg, F32, 0, 100, 14, 0, 4, pg, p, nul, nul) == -4
    assert L.thc_encode_all_static(pg, BF16, 4, 0, 14, 0, 4, pg, p, nul, nul) == 0
    assert L.thc_encode_all_static(pg, F32, 4, 100, 14, 0, 4, pg, p, ctypes.c_void_p(0x1002), nul) == -8
    big = ((2 << 20) // (4 * (8 * 4 + 1)) + 1) * (1 << 14)       # one chunk more than the array has words for
    assert L.thc_encode_all_static(pg, F32, 4, big, 14, 0, 4, pg, p, nul, nul) == -6


def test_one_pass_minmax_entry_points_validate_on_the_host(L):
    p = ctypes.c_void_p(0x1000)
    nul = ctypes.c_void_p(0)
    F32 = thc.THC_F32
    g = (ctypes.c_void_p * 4)(*([0x1000] * 4))
    pg = ctypes.cast(g, ctypes.POINTER(ctypes.c_void_p))
    odd = (ctypes.c_void_p * 4)(0x1000, 0x1008, 0x1000, 0x1000)
    podd = ctypes.cast(odd, ctypes.POINTER(ctypes.c_void_p))
    # two words per wave and worker, one counter per chunk, 16-byte header
    assert L.thc_encode_all_minmax_workspace_bytes(4, 100, 14) == 16 + 4 * (2 * 8 * 4 + 1)
    assert L.thc_encode_all_minmax_workspace_bytes(4, 100, 10) == 0
    assert L.thc_encode_all_minmax_workspace_bytes(65, 100, 14) == 0
    enc = L.thc_encode_all_minmax
    assert enc(pg, F32, 4, 100, 10, 0, 4, 1, pg, p, p, 1 << 20, nul) == -3
    assert enc(pg, 3, 4, 100, 14, 0, 4, 1, pg, p, p, 1 << 20, nul) == -5
    assert enc(pg, F32, 4, 100, 14, 0, 6, 1, pg, p, p, 1 << 20, nul) == -2
    assert enc(pg, F32, 0, 100, 14, 0, 4, 1, pg, p, p, 1 << 20, nul) == -4
    assert enc(pg, F32, 65, 100, 14, 0, 2, 1, pg, p, p, 1 << 20, nul) == -4
    assert enc(pg, F32, 4, 0, 14, 0, 4, 0, pg, nul, nul, 0, nul) == 0
    assert enc(pg, F32, 4, 100, 14, 0, 4, 0, pg, nul, p, 1 << 20, nul) == -1
    assert enc(podd, F32, 4, 100, 14, 0, 4, 0, pg, p, p, 1 << 20, nul) == -8
    assert enc(pg, F32, 4, 100, 14, 0, 4, 0, pg, ctypes.c_void_p(0x1004), p, 1 << 20, nul) == -8
    assert enc(pg, F32, 4, 100, 14, 0, 4, 0, pg, p, p, 100, nul) == -6
    dec = L.thc_aggregate_decode_minmax
    assert dec(pg, 4, p, 100, 10, 0, 4, 1, p, nul) == -3
    assert dec(pg, 4, p, 100, 14, 0, 5, 1, p, nul) == -2
    assert dec(pg, 65, p, 100, 14, 0, 4, 1, p, nul) == -4        # more workers than the one-launch forms take
    assert dec(pg, 65, p, 100, 14, 0, 2, 0, p, nul) == -4
    assert dec(pg, 4, p, 0, 14, 0, 4, 1, nul, nul) == 0
    assert dec(pg, 4, nul, 100, 14, 0, 4, 1, p, nul) == -1
    assert dec(podd, 4, p, 100, 14, 0, 4, 0, p, nul) == -8
    assert dec(pg, 4, p, 100, 14, 0, 4, 0, ctypes.c_void_p(0x1004), nul) == -8


def test_full_rotation_entry_points_validate_on_the_host(L):
    """Every call fails validation before anything is enqueued (dummy addresses)."""
    p = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1004)      # 4-byte aligned only
    nul = ctypes.c_void_p(0)
    F32 = thc.THC_F32
    assert thc.thc_full_log2(1) == 15 and thc.thc_full_log2((1 << 15) + 1) == 16
    assert thc.thc_full_log2(1 << 33) == 33 and thc.thc_full_log2((1 << 33) + 1) == 0
    for l in (0, 14, 34):               # log2_size out of range
        assert L.rht_forward_full(p, F32, 10, l, 0, p, nul) == -3
        assert L.rht_forward_full_absmax(p, F32, 10, l, 0, p, p, nul) == -3
        assert L.rht_forward_full_deferred(p, F32, 10, l, 0, p, p, nul) == -3
        assert L.rht_inverse_full(p, 10, l, 0, p, nul) == -3
        assert L.thc_full_absmax(p, l, p, nul) == -3
        assert L.thc_full_encode(p, l, 0, 0, 4, p, p, nul) == -3
        assert L.thc_full_encode_deferred(p, 10, l, 0, 0, 4, p, p, nul) == -3
        assert L.thc_full_decode(p, p, 4, l, 4, p, nul) == -3
        assert L.thc_full_decode_inverse(p, p, 4, 10, l, 0, 4, p, p, nul) == -3
    too_many = (1 << 15) + 1            # n > 2^log2_size
    assert L.rht_forward_full(p, F32, too_many, 15, 0, p, nul) == -6
    assert L.rht_forward_full_deferred(p, F32, too_many, 15, 0, p, p, nul) == -6
    assert L.rht_inverse_full(p, too_many, 15, 0, p, nul) == -6
    assert L.thc_full_encode_deferred(p, too_many, 15, 0, 0, 4, p, p, nul) == -6
    assert L.thc_full_decode_inverse(p, p, 4, too_many, 15, 0, 4, p, p, nul) == -6
    assert L.rht_forward_full(p, 9, 10, 15, 0, p, nul) == -5                     # dtype
    for bad in (0, 3, 16):                                                       # bits
        assert L.thc_full_encode(p, 15, 0, 0, bad, p, p, nul) == -2
        assert L.thc_full_encode_deferred(p, 10, 15, 0, 0, bad, p, p, nul) == -2
        assert L.thc_full_decode(p, p, 4, 15, bad, p, nul) == -2
        assert L.thc_full_decode_inverse(p, p, 4, 10, 15, 0, bad, p, p, nul) == -2
    assert L.thc_full_decode(p, p, 0, 15, 4, p, nul) == -4                       # workers
    assert L.thc_full_decode_inverse(p, p, 300, 10, 15, 0, 8, p, p, nul) == -4
    # null pointers
    assert L.rht_forward_full(p, F32, 10, 15, 0, nul, nul) == -1
    assert L.rht_forward_full(nul, F32, 10, 15, 0, p, nul) == -1
    assert L.rht_forward_full_absmax(p, F32, 10, 15, 0, p, nul, nul) == -1
    assert L.rht_forward_full_deferred(p, F32, 10, 15, 0, p, nul, nul) == -1
    assert L.rht_inverse_full(nul, 10, 15, 0, p, nul) == -1
    assert L.thc_full_encode(p, 15, 0, 0, 4, nul, p, nul) == -1
    assert L.thc_full_encode_deferred(p, 10, 15, 0, 0, 4, p, nul, nul) == -1
    assert L.thc_full_decode_inverse(p, p, 4, 10, 15, 0, 4, nul, p, nul) == -1
    # alignment: the arrays need 16 bytes
    assert L.rht_forward_full(p, F32, 10, 15, 0, odd, nul) == -8
    assert L.rht_forward_full_deferred(odd, F32, 10, 15, 0, p, p, nul) == -8
    assert L.rht_inverse_full(p, 10, 15, 0, odd, nul) == -8
    assert L.thc_full_encode(odd, 15, 0, 0, 4, p, p, nul) == -8
    assert L.thc_full_encode_deferred(p, 10, 15, 0, 0, 4, p, odd, nul) == -8
    assert L.thc_full_decode_inverse(p, p, 4, 10, 15, 0, 4, odd, p, nul) == -8
    assert L.thc_full_decode_inverse(p, p, 4, 10, 15, 0, 4, p, odd, nul) == -8
    # nothing to do
    assert L.rht_inverse_full(nul, 0, 15, 0, nul, nul) == 0
    assert L.thc_full_decode_inverse(nul, nul, 4, 0, 15, 0, 4, nul, nul, nul) == 0


def test_header_is_plain_c(tmp_path):
    """include/thc.h is a C header: it compiles as C99 with pedantic warnings as errors, and
    as C++ (the library's own translation units include it that way)."""
    import shutil
    import subprocess
    src = tmp_path / "use_thc.c"
    src.write_text('#include "thc.h"\nint main(void) { thc_dtype d = THC_BF16; thc_bucket b; (void)b; '
                   "return d == 1 && THC_ERR_ALIGN == -8 ? 0 : 1; }\n")
    inc = os.path.join(ROOT, "include")
    for cc, flags in (("gcc", ["-std=c99", "-pedantic-errors"]), ("g++", ["-std=c++17", "-x", "c++"])):
        if shutil.which(cc) is None:
            pytest.skip(f"{cc} is not installed")
        res = subprocess.run([cc, *flags, "-Wall", "-Wextra", "-Werror", f"-I{inc}", "-fsyntax-only", str(src)],
                             stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        assert res.returncode == 0, res.stdout
