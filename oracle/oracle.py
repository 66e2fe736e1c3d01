"""ctypes front end of the CPU oracle (``sparseloco_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's ``cpu_baseline`` leg.  The product package never imports it, and
this module imports nothing from the product package.  It only marshals numpy
arrays into the C functions; all arithmetic of the method is in the C file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsparseloco_oracle.so")

LAYOUT_FLAT = 0
LAYOUT_TILE = 1


class SloTensor(C.Structure):
    _fields_ = [
        ("rows", C.c_int64),
        ("cols", C.c_int64),
        ("offset", C.c_int64),
        ("layout", C.c_int32),
        ("reserved", C.c_int32),
    ]


def build() -> str:
    """Compile the oracle's C source (always recompiles)."""
    subprocess.check_call(["sh", os.path.join(_HERE, "build.sh")])
    return _LIB_PATH


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            build()
        L = C.CDLL(_LIB_PATH)
        i64, i32, vp = C.c_int64, C.c_int, C.c_void_p
        tp = C.POINTER(SloTensor)
        L.slo_tensor_chunks.restype = i64
        L.slo_tensor_chunks.argtypes = [tp, i32]
        L.slo_num_chunks.restype = i64
        L.slo_num_chunks.argtypes = [tp, i32, i32]
        L.slo_element_of.restype = i64
        L.slo_element_of.argtypes = [tp, i32, i64, i32]
        L.slo_record_bytes.restype = i64
        L.slo_record_bytes.argtypes = [i32]
        L.slo_payload_bytes.restype = i64
        L.slo_payload_bytes.argtypes = [tp, i32, i32, i32]
        L.slo_tensor_block_bytes.restype = i64
        L.slo_tensor_block_bytes.argtypes = [tp, i32, i32]
        L.slo_pack_record.restype = None
        L.slo_pack_record.argtypes = [vp, vp, i32, vp]
        L.slo_unpack_record.restype = None
        L.slo_unpack_record.argtypes = [vp, i32, vp, vp]
        L.slo_pack_indices.restype = i32
        L.slo_pack_indices.argtypes = [vp, vp, i64, i32, vp]
        L.slo_tree_sum.restype = C.c_double
        L.slo_tree_sum.argtypes = [vp, i64]
        L.slo_accumulate.restype = None
        L.slo_accumulate.argtypes = [vp, vp, C.c_float, i64]
        L.slo_topk_chunk.restype = i32
        L.slo_topk_chunk.argtypes = [tp, i32, i64, vp, i32, vp, vp]
        L.slo_quantize_tensor.restype = i32
        L.slo_quantize_tensor.argtypes = [vp, i64, i32, vp, vp, vp]
        L.slo_compress.restype = i32
        L.slo_compress.argtypes = [tp, i32, i32, i32, vp, vp, C.c_float, i32, vp, vp, vp, vp, vp]
        L.slo_decompress_avg_apply.restype = i32
        L.slo_decompress_avg_apply.argtypes = [tp, i32, i32, i32, vp, vp, i32, C.c_float]
        L.slo_decompress_dense.restype = i32
        L.slo_decompress_dense.argtypes = [tp, i32, i32, i32, vp, vp]
        L.slo_header_bytes_b.restype = i64
        L.slo_header_bytes_b.argtypes = [i32]
        L.slo_record_bytes_b.restype = i64
        L.slo_record_bytes_b.argtypes = [i32, i32]
        L.slo_tensor_block_bytes_b.restype = i64
        L.slo_tensor_block_bytes_b.argtypes = [tp, i32, i32, i32]
        L.slo_payload_bytes_b.restype = i64
        L.slo_payload_bytes_b.argtypes = [tp, i32, i32, i32, i32]
        L.slo_pack_record_b.restype = None
        L.slo_pack_record_b.argtypes = [vp, vp, vp, i32, i32, vp]
        L.slo_unpack_record_b.restype = None
        L.slo_unpack_record_b.argtypes = [vp, i32, i32, vp, vp, vp]
        L.slo_quantize_tensor_b.restype = i32
        L.slo_quantize_tensor_b.argtypes = [vp, i64, i32, i32, vp, vp, vp]
        L.slo_compress_b.restype = i32
        L.slo_compress_b.argtypes = [tp, i32, i32, i32, i32, vp, vp, C.c_float, i32, vp, vp, vp, vp, vp]
        L.slo_decompress_avg_apply_b.restype = i32
        L.slo_decompress_avg_apply_b.argtypes = [tp, i32, i32, i32, i32, vp, vp, i32, C.c_float]
        L.slo_decompress_dense_b.restype = i32
        L.slo_decompress_dense_b.argtypes = [tp, i32, i32, i32, i32, vp, vp]
        L.slo_lom_direction.restype = None
        L.slo_lom_direction.argtypes = [tp, i32, vp, vp, C.c_float, vp]
        L.slo_dense_avg_apply.restype = i32
        L.slo_dense_avg_apply.argtypes = [tp, i32, vp, vp, vp, i32, C.c_float, C.c_float]
        L.slo_decompress_avg_apply_nesterov_b.restype = i32
        L.slo_decompress_avg_apply_nesterov_b.argtypes = [tp, i32, i32, i32, i32, vp, vp, vp, i32, C.c_float,
                                                          C.c_float]
        L.slo_sub_topk.restype = i32
        L.slo_sub_topk.argtypes = [tp, i32, i32, i32, vp, vp]
        L.slo_fmix32.restype = C.c_uint32
        L.slo_fmix32.argtypes = [C.c_uint32]
        L.slo_random_key.restype = C.c_uint32
        L.slo_random_key.argtypes = [C.c_uint32, C.c_uint32, C.c_uint32]
        L.slo_compress_random_b.restype = i32
        L.slo_compress_random_b.argtypes = [tp, i32, i32, i32, i32, vp, vp, C.c_float, C.c_uint32, vp, vp]
        L.slo_validate_payload.restype = i32
        L.slo_validate_payload.argtypes = [tp, i32, i32, i32, vp]
        L.slo_rice_param.restype = i32
        L.slo_rice_param.argtypes = [i32]
        L.slo_rice_max_bytes.restype = i64
        L.slo_rice_max_bytes.argtypes = [tp, i32, i32, i32]
        L.slo_rice_encode.restype = i64
        L.slo_rice_encode.argtypes = [tp, i32, i32, i32, vp, vp, i64]
        L.slo_rice_decode.restype = i32
        L.slo_rice_decode.argtypes = [tp, i32, i32, i32, vp, i64, vp]
        L.slo_rice_qfield_bytes.restype = i32
        L.slo_rice_qfield_bytes.argtypes = [i32]
        L.slo_rice_dir_entry_bytes.restype = i64
        L.slo_rice_dir_entry_bytes.argtypes = [i32]
        L.slo_rice_rem_bytes.restype = i64
        L.slo_rice_rem_bytes.argtypes = [i32]
        L.slo_rice_fixed_bytes.restype = i64
        L.slo_rice_fixed_bytes.argtypes = [i32, i32]
        L.slo_rice_max_bytes_b.restype = i64
        L.slo_rice_max_bytes_b.argtypes = [tp, i32, i32, i32, i32]
        L.slo_rice_encode_b.restype = i64
        L.slo_rice_encode_b.argtypes = [tp, i32, i32, i32, i32, vp, vp, i64]
        L.slo_rice_decode_b.restype = i32
        L.slo_rice_decode_b.argtypes = [tp, i32, i32, i32, i32, vp, i64, vp]
        L.slo_max_threads.restype = i32
        L.slo_max_threads.argtypes = []
        _lib = L
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _check(a, dtype):
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.flags["C_CONTIGUOUS"], (
        f"need C-contiguous {dtype} array"
    )
    return a


def make_tensors(descs):
    """descs: iterable of (rows, cols, offset, layout) -> ctypes array."""
    descs = list(descs)
    arr = (SloTensor * max(1, len(descs)))()
    for i, (r, c, off, lay) in enumerate(descs):
        arr[i] = SloTensor(int(r), int(c), int(off), int(lay), 0)
    return arr, len(descs)


def num_chunks(descs, tile=64):
    arr, n = make_tensors(descs)
    return int(lib().slo_num_chunks(arr, n, tile))


def tensor_chunks(desc, tile=64):
    arr, _ = make_tensors([desc])
    return int(lib().slo_tensor_chunks(arr, tile))


def element_of(desc, c, j, tile=64):
    arr, _ = make_tensors([desc])
    return int(lib().slo_element_of(arr, tile, int(c), int(j)))


def record_bytes(k):
    return int(lib().slo_record_bytes(k))


def payload_bytes(descs, k, tile=64):
    arr, n = make_tensors(descs)
    return int(lib().slo_payload_bytes(arr, n, tile, k))


def tensor_block_bytes(desc, k, tile=64):
    arr, _ = make_tensors([desc])
    return int(lib().slo_tensor_block_bytes(arr, tile, k))


def pack_record(idx, code):
    idx = _check(np.ascontiguousarray(idx, dtype=np.uint16), np.uint16)
    code = _check(np.ascontiguousarray(code, dtype=np.uint8), np.uint8)
    k = idx.size
    out = np.zeros(record_bytes(k), dtype=np.uint8)
    lib().slo_pack_record(_ptr(idx), _ptr(code), k, _ptr(out))
    return out


def unpack_record(rec, k):
    rec = _check(np.ascontiguousarray(rec, dtype=np.uint8), np.uint8)
    idx = np.zeros(k, dtype=np.uint16)
    code = np.zeros(k, dtype=np.uint8)
    lib().slo_unpack_record(_ptr(rec), k, _ptr(idx), _ptr(code))
    return idx, code


def pack_indices(idx, code, n_chunks, k):
    idx = _check(np.ascontiguousarray(idx, dtype=np.uint16), np.uint16)
    code = _check(np.ascontiguousarray(code, dtype=np.uint8), np.uint8)
    out = np.zeros(n_chunks * record_bytes(k), dtype=np.uint8)
    st = lib().slo_pack_indices(_ptr(idx), _ptr(code), n_chunks, k, _ptr(out))
    if st:
        raise ValueError(f"slo_pack_indices: status {st}")
    return out


def tree_sum(values):
    v = np.ascontiguousarray(values, dtype=np.float64)
    return float(lib().slo_tree_sum(_ptr(v), v.size))


def accumulate(e, delta, beta):
    """In place: e <- fma(beta, e, delta)."""
    _check(e, np.float32), _check(delta, np.float32)
    assert e.size == delta.size
    lib().slo_accumulate(_ptr(e), _ptr(delta), float(beta), e.size)


def topk_chunk(desc, c, a, k, tile=64):
    arr, _ = make_tensors([desc])
    _check(a, np.float32)
    idx = np.zeros(k, dtype=np.uint16)
    val = np.zeros(k, dtype=np.float32)
    n = lib().slo_topk_chunk(arr, tile, int(c), _ptr(a), k, _ptr(idx), _ptr(val))
    if n < 0:
        raise ValueError("chunk has fewer than k valid elements")
    return idx, val


def quantize_tensor(x, n_chunks, k):
    """x: the tensor's selected values in canonical order. -> codes, lut, stats"""
    x = _check(np.ascontiguousarray(x, dtype=np.float32), np.float32)
    assert x.size == n_chunks * k
    code = np.zeros(x.size, dtype=np.uint8)
    lut = np.zeros(4, dtype=np.float32)
    stats = np.zeros(8, dtype=np.float64)
    st = lib().slo_quantize_tensor(_ptr(x), n_chunks, k, _ptr(code), _ptr(lut), _ptr(stats))
    if st:
        raise RuntimeError(f"slo_quantize_tensor: status {st}")
    return code, lut, stats


def compress(descs, k, e, delta, beta, tile=64, ef_frozen=False, want_detail=False):
    """Updates e in place; returns payload bytes (and the selection when asked)."""
    arr, n = make_tensors(descs)
    _check(e, np.float32), _check(delta, np.float32)
    nbytes = int(lib().slo_payload_bytes(arr, n, tile, k))
    payload = np.zeros(nbytes, dtype=np.uint8)
    det = None
    args = [None, None, None, None]
    if want_detail:
        nc = int(lib().slo_num_chunks(arr, n, tile))
        det = dict(
            idx=np.zeros(nc * k, dtype=np.uint16),
            val=np.zeros(nc * k, dtype=np.float32),
            code=np.zeros(nc * k, dtype=np.uint8),
            lut=np.zeros(4 * n, dtype=np.float32),
        )
        args = [_ptr(det["idx"]), _ptr(det["val"]), _ptr(det["code"]), _ptr(det["lut"])]
    st = lib().slo_compress(arr, n, tile, k, _ptr(e), _ptr(delta), float(beta),
                            int(bool(ef_frozen)), _ptr(payload), *args)
    if st:
        raise ValueError(f"slo_compress: status {st}")
    return (payload, det) if want_detail else payload


def decompress_avg_apply(descs, k, theta, payloads, lr, tile=64):
    """In place: theta <- theta - lr * mean_r(dequantised payload_r)."""
    arr, n = make_tensors(descs)
    _check(theta, np.float32)
    R = len(payloads)
    for p in payloads:
        _check(p, np.uint8)
    ptrs = (C.c_void_p * max(1, R))(*[p.ctypes.data for p in payloads])
    st = lib().slo_decompress_avg_apply(arr, n, tile, k, _ptr(theta), ptrs, R, float(lr))
    if st:
        raise ValueError(f"slo_decompress_avg_apply: status {st}")


def decompress_dense(descs, k, payload, n_elems, tile=64):
    arr, n = make_tensors(descs)
    out = np.zeros(n_elems, dtype=np.float32)
    st = lib().slo_decompress_dense(arr, n, tile, k, _ptr(payload), _ptr(out))
    if st:
        raise ValueError(f"slo_decompress_dense: status {st}")
    return out


# ---- other value widths: bits in {1, 2, 3, 4} or 32 (unquantized fp32 values) ----
def header_bytes_b(bits):
    return int(lib().slo_header_bytes_b(bits))


def record_bytes_b(k, bits):
    return int(lib().slo_record_bytes_b(k, bits))


def tensor_block_bytes_b(desc, k, bits, tile=64):
    arr, _ = make_tensors([desc])
    return int(lib().slo_tensor_block_bytes_b(arr, tile, k, bits))


def payload_bytes_b(descs, k, bits, tile=64):
    arr, n = make_tensors(descs)
    return int(lib().slo_payload_bytes_b(arr, n, tile, k, bits))


def pack_record_b(idx, sent, bits):
    """sent: the k codes (bits <= 4) or the k fp32 values (bits = 32)."""
    idx = _check(np.ascontiguousarray(idx, dtype=np.uint16), np.uint16)
    k = idx.size
    out = np.zeros(record_bytes_b(k, bits), dtype=np.uint8)
    if bits == 32:
        val = _check(np.ascontiguousarray(sent, dtype=np.float32), np.float32)
        lib().slo_pack_record_b(_ptr(idx), None, _ptr(val), k, bits, _ptr(out))
    else:
        code = _check(np.ascontiguousarray(sent, dtype=np.uint8), np.uint8)
        lib().slo_pack_record_b(_ptr(idx), _ptr(code), None, k, bits, _ptr(out))
    return out


def unpack_record_b(rec, k, bits):
    rec = _check(np.ascontiguousarray(rec, dtype=np.uint8), np.uint8)
    idx = np.zeros(k, dtype=np.uint16)
    code = np.zeros(k, dtype=np.uint8)
    val = np.zeros(k, dtype=np.float32)
    lib().slo_unpack_record_b(_ptr(rec), k, bits, _ptr(idx), _ptr(code), _ptr(val))
    return idx, (val if bits == 32 else code)


def quantize_tensor_b(x, n_chunks, k, bits):
    x = _check(np.ascontiguousarray(x, dtype=np.float32), np.float32)
    assert x.size == n_chunks * k
    code = np.zeros(x.size, dtype=np.uint8)
    lut = np.zeros(1 << bits, dtype=np.float32)
    stats = np.zeros(4 + (1 << bits), dtype=np.float64)
    st = lib().slo_quantize_tensor_b(_ptr(x), n_chunks, k, bits, _ptr(code), _ptr(lut), _ptr(stats))
    if st:
        raise RuntimeError(f"slo_quantize_tensor_b: status {st}")
    return code, lut, stats


def compress_b(descs, k, bits, e, delta, beta, tile=64, ef_frozen=False, want_detail=False):
    arr, n = make_tensors(descs)
    _check(e, np.float32), _check(delta, np.float32)
    nbytes = int(lib().slo_payload_bytes_b(arr, n, tile, k, bits))
    payload = np.zeros(nbytes, dtype=np.uint8)
    det = None
    args = [None, None, None, None]
    if want_detail:
        nc = int(lib().slo_num_chunks(arr, n, tile))
        nb = 0 if bits == 32 else 1 << bits
        det = dict(
            idx=np.zeros(nc * k, dtype=np.uint16),
            val=np.zeros(nc * k, dtype=np.float32),
            code=np.zeros(nc * k, dtype=np.uint8),
            lut=np.zeros(max(1, nb * n), dtype=np.float32),
        )
        args = [_ptr(det["idx"]), _ptr(det["val"]), _ptr(det["code"]), _ptr(det["lut"])]
    st = lib().slo_compress_b(arr, n, tile, k, bits, _ptr(e), _ptr(delta), float(beta),
                              int(bool(ef_frozen)), _ptr(payload), *args)
    if st:
        raise ValueError(f"slo_compress_b: status {st}")
    return (payload, det) if want_detail else payload


def decompress_avg_apply_b(descs, k, bits, theta, payloads, lr, tile=64):
    arr, n = make_tensors(descs)
    _check(theta, np.float32)
    R = len(payloads)
    for p in payloads:
        _check(p, np.uint8)
    ptrs = (C.c_void_p * max(1, R))(*[p.ctypes.data for p in payloads])
    st = lib().slo_decompress_avg_apply_b(arr, n, tile, k, bits, _ptr(theta), ptrs, R, float(lr))
    if st:
        raise ValueError(f"slo_decompress_avg_apply_b: status {st}")


def decompress_dense_b(descs, k, bits, payload, n_elems, tile=64, out=None):
    """Writes the sent values into `out` (zeros by default) at the positions the payload names."""
    arr, n = make_tensors(descs)
    if out is None:
        out = np.zeros(n_elems, dtype=np.float32)
    _check(out, np.float32)
    st = lib().slo_decompress_dense_b(arr, n, tile, k, bits, _ptr(payload), _ptr(out))
    if st:
        raise ValueError(f"slo_decompress_dense_b: status {st}")
    return out


# ---- outer steps of the DiLoCo family (dense momentum variants) ----
def lom_direction(descs, m, delta, mu, out=None):
    """m <- mu*m + delta in place; returns dir = delta + mu*m (tensor elements only)."""
    arr, n = make_tensors(descs)
    _check(m, np.float32), _check(delta, np.float32)
    if out is None:
        out = np.zeros_like(delta)
    _check(out, np.float32)
    lib().slo_lom_direction(arr, n, _ptr(m), _ptr(delta), float(mu), _ptr(out))
    return out


def dense_avg_apply(descs, theta, dirs, lr, m=None, mu=0.0):
    arr, n = make_tensors(descs)
    _check(theta, np.float32)
    R = len(dirs)
    for d in dirs:
        _check(d, np.float32)
    if m is not None:
        _check(m, np.float32)
    ptrs = (C.c_void_p * max(1, R))(*[d.ctypes.data for d in dirs])
    st = lib().slo_dense_avg_apply(arr, n, _ptr(theta), None if m is None else _ptr(m), ptrs, R,
                                   float(lr), float(mu))
    if st:
        raise ValueError(f"slo_dense_avg_apply: status {st}")


def decompress_avg_apply_nesterov_b(descs, k, bits, theta, m, payloads, lr, mu, tile=64):
    arr, n = make_tensors(descs)
    _check(theta, np.float32), _check(m, np.float32)
    R = len(payloads)
    for p in payloads:
        _check(p, np.uint8)
    ptrs = (C.c_void_p * max(1, R))(*[p.ctypes.data for p in payloads])
    st = lib().slo_decompress_avg_apply_nesterov_b(arr, n, tile, k, bits, _ptr(theta), _ptr(m), ptrs, R,
                                                   float(lr), float(mu))
    if st:
        raise ValueError(f"slo_decompress_avg_apply_nesterov_b: status {st}")


def sub_topk(descs, k, m, tile=64, want_idx=False):
    """m <- m - Top-k(m) chunk-wise, in place."""
    arr, n = make_tensors(descs)
    _check(m, np.float32)
    idx = np.zeros(num_chunks(descs, tile) * k, dtype=np.uint16) if want_idx else None
    st = lib().slo_sub_topk(arr, n, tile, k, _ptr(m), None if idx is None else _ptr(idx))
    if st:
        raise ValueError(f"slo_sub_topk: status {st}")
    return idx


def validate_payload(descs, k, payload, tile=64):
    """True when every record is strictly ascending and inside its tensor."""
    arr, n = make_tensors(descs)
    _check(payload, np.uint8)
    return int(lib().slo_validate_payload(arr, n, tile, k, _ptr(payload))) == 0


def max_threads():
    return int(lib().slo_max_threads())


def rice_param(k):
    return int(lib().slo_rice_param(k))


RICE_GROUP = 16      # chunks per directory entry of the coded format


def rice_qfield_bytes(k):
    return int(lib().slo_rice_qfield_bytes(k))


def rice_dir_entry_bytes(k):
    return int(lib().slo_rice_dir_entry_bytes(k))


def rice_rem_bytes(k):
    return int(lib().slo_rice_rem_bytes(k))


def rice_fixed_bytes(k, bits=2):
    return int(lib().slo_rice_fixed_bytes(k, bits))


def rice_max_bytes(descs, k, tile=64):
    arr, n = make_tensors(descs)
    return int(lib().slo_rice_max_bytes(arr, n, tile, k))


def rice_encode(descs, k, payload, tile=64):
    """Plain-format payload -> coded buffer (trimmed to its size)."""
    arr, n = make_tensors(descs)
    _check(payload, np.uint8)
    cap = int(lib().slo_rice_max_bytes(arr, n, tile, k))
    out = np.zeros(cap, dtype=np.uint8)
    size = int(lib().slo_rice_encode(arr, n, tile, k, _ptr(payload), _ptr(out), cap))
    if size < 0:
        raise ValueError(f"slo_rice_encode: status {size}")
    return out[:size].copy()


def rice_decode(descs, k, coded, tile=64):
    arr, n = make_tensors(descs)
    _check(coded, np.uint8)
    out = np.full(int(lib().slo_payload_bytes(arr, n, tile, k)), 0xEE, dtype=np.uint8)
    st = lib().slo_rice_decode(arr, n, tile, k, _ptr(coded), coded.size, _ptr(out))
    if st:
        raise ValueError(f"slo_rice_decode: status {st}")
    return out


def rice_max_bytes_b(descs, k, bits, tile=64):
    arr, n = make_tensors(descs)
    return int(lib().slo_rice_max_bytes_b(arr, n, tile, k, bits))


def rice_encode_b(descs, k, bits, payload, tile=64):
    arr, n = make_tensors(descs)
    _check(payload, np.uint8)
    cap = rice_max_bytes_b(descs, k, bits, tile)
    out = np.zeros(cap, dtype=np.uint8)
    size = int(lib().slo_rice_encode_b(arr, n, tile, k, bits, _ptr(payload), _ptr(out), cap))
    if size < 0:
        raise ValueError(f"slo_rice_encode_b: status {size}")
    return out[:size].copy()


def rice_decode_b(descs, k, bits, coded, tile=64):
    arr, n = make_tensors(descs)
    _check(coded, np.uint8)
    out = np.zeros(payload_bytes_b(descs, k, bits, tile), dtype=np.uint8)
    st = lib().slo_rice_decode_b(arr, n, tile, k, bits, _ptr(coded), coded.size, _ptr(out))
    if st:
        raise ValueError(f"slo_rice_decode_b: status {st}")
    return out


# ---- Random-k ablation ----
def fmix32(h):
    return int(lib().slo_fmix32(int(h) & 0xFFFFFFFF))


def random_key(seed, chunk, j):
    return int(lib().slo_random_key(int(seed) & 0xFFFFFFFF, int(chunk) & 0xFFFFFFFF, int(j)))


def compress_random_b(descs, k, bits, e, delta, beta, seed, tile=64, want_idx=False):
    arr, n = make_tensors(descs)
    _check(e, np.float32), _check(delta, np.float32)
    payload = np.zeros(int(lib().slo_payload_bytes_b(arr, n, tile, k, bits)), dtype=np.uint8)
    idx = np.zeros(int(lib().slo_num_chunks(arr, n, tile)) * k, dtype=np.uint16) if want_idx else None
    st = lib().slo_compress_random_b(arr, n, tile, k, bits, _ptr(e), _ptr(delta), float(beta),
                                     int(seed) & 0xFFFFFFFF, _ptr(payload), None if idx is None else _ptr(idx))
    if st:
        raise ValueError(f"slo_compress_random_b: status {st}")
    return (payload, idx) if want_idx else payload
