"""Thin ctypes binding of libsparseloco.so - argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI declared in
include/sparseloco.h; the functions here carry the same names and only turn
torch tensors (device memory owned by the caller) into pointers.  There is no
CPU fallback: if the library has not been built, importing symbols raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libsparseloco.so")

SL_LAYOUT_FLAT = 0
SL_LAYOUT_TILE64 = 1
SL_COMPRESS_DEFAULT = 0
SL_COMPRESS_EF_FROZEN = 1
SL_COMPRESS_DEFER_RESIDUAL = 2
SL_MAX_WORKERS = 64
SL_NOALLOC_SCRATCH_BYTES = 64 * 1024 * 1024
SL_ERR_TOO_LARGE = -6

EXPORTS = [
    "sl_plan_create", "sl_plan_destroy", "sl_plan_num_chunks", "sl_plan_num_elements",
    "sl_payload_bytes", "sl_payload_tensor_offset", "sl_workspace_bytes", "sl_compress",
    "sl_decompress_avg_apply", "sl_pack_indices", "sl_strerror", "sl_last_hip_error",
    "sl_profile_begin", "sl_profile_end", "sl_residual_apply",
    "sl_rice_max_bytes", "sl_rice_encode", "sl_rice_decode", "sl_compress_params",
    "sl_payload_validate", "sl_plan_create_bits", "sl_plan_value_bits", "sl_pack_indices_bits",
    "sl_lom_direction", "sl_dense_avg_apply", "sl_decompress_avg_apply_nesterov", "sl_sub_topk",
    "sl_compress_random_k", "sl_compress_noalloc", "sl_plan_set_codes_wave_below", "sl_coded_fixed_bytes",
    "sl_compress_coded", "sl_decompress_avg_apply_coded", "sl_decompress_avg_apply_nesterov_coded",
]
PROF_PHASES = ["select", "stats", "codes", "lut", "residual", "apply", "index"]


class SlTensor(C.Structure):
    _fields_ = [("rows", C.c_int64), ("cols", C.c_int64), ("offset", C.c_int64),
                ("layout", C.c_int32), ("reserved", C.c_int32)]


class SparseLoCoError(RuntimeError):
    def __init__(self, fn: str, status: int):
        msg = lib().sl_strerror(status).decode()
        hip = lib().sl_last_hip_error().decode()
        super().__init__(f"{fn}: {msg} ({status})" + (f": {hip}" if status == -3 and hip else ""))
        self.status = status


_lib = None


def lib():
    """Loads the built library; raises if it is missing (there is no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is not built - run `python -m paper_2508_15706_amd.build` "
                "(or __graft_entry__.build()) first; this package has no CPU fallback")
        L = C.CDLL(LIB_PATH)
        vp, i64, i32, sz = C.c_void_p, C.c_int64, C.c_int, C.c_size_t
        L.sl_plan_create.restype = i32
        L.sl_plan_create.argtypes = [C.POINTER(SlTensor), i32, i32, C.POINTER(vp)]
        L.sl_plan_create_bits.restype = i32
        L.sl_plan_create_bits.argtypes = [C.POINTER(SlTensor), i32, i32, i32, C.POINTER(vp)]
        L.sl_plan_value_bits.restype = i32
        L.sl_plan_value_bits.argtypes = [vp]
        L.sl_pack_indices_bits.restype = i32
        L.sl_pack_indices_bits.argtypes = [vp, vp, vp, i64, i32, i32, vp, vp]
        L.sl_lom_direction.restype = i32
        L.sl_lom_direction.argtypes = [vp, vp, vp, C.c_float, vp, vp]
        L.sl_dense_avg_apply.restype = i32
        L.sl_dense_avg_apply.argtypes = [vp, vp, vp, C.POINTER(vp), i32, C.c_float, C.c_float, vp]
        L.sl_decompress_avg_apply_nesterov.restype = i32
        L.sl_decompress_avg_apply_nesterov.argtypes = [vp, vp, vp, C.POINTER(vp), i32, C.c_float, C.c_float, vp]
        L.sl_sub_topk.restype = i32
        L.sl_sub_topk.argtypes = [vp, vp, vp]
        L.sl_plan_destroy.restype = i32
        L.sl_plan_destroy.argtypes = [vp]
        L.sl_plan_num_chunks.restype = i64
        L.sl_plan_num_chunks.argtypes = [vp]
        L.sl_plan_num_elements.restype = i64
        L.sl_plan_num_elements.argtypes = [vp]
        L.sl_payload_bytes.restype = sz
        L.sl_payload_bytes.argtypes = [vp]
        L.sl_payload_tensor_offset.restype = sz
        L.sl_payload_tensor_offset.argtypes = [vp, i32]
        L.sl_workspace_bytes.restype = sz
        L.sl_workspace_bytes.argtypes = [vp]
        L.sl_compress.restype = i32
        L.sl_compress.argtypes = [vp, vp, vp, C.c_float, i32, vp, vp, vp, vp]
        L.sl_compress_noalloc.restype = i32
        L.sl_compress_noalloc.argtypes = [vp, vp, vp, C.c_float, i32, vp, vp, vp]
        L.sl_compress_random_k.restype = i32
        L.sl_compress_random_k.argtypes = [vp, vp, vp, C.c_float, i32, vp, vp, vp, C.c_uint32, vp]
        L.sl_compress_params.restype = i32
        L.sl_compress_params.argtypes = [vp, vp, vp, vp, C.c_float, i32, vp, vp, vp, vp]
        L.sl_payload_validate.restype = i32
        L.sl_payload_validate.argtypes = [vp, vp, vp, vp]
        L.sl_residual_apply.restype = i32
        L.sl_residual_apply.argtypes = [vp, vp, vp, vp]
        L.sl_decompress_avg_apply.restype = i32
        L.sl_decompress_avg_apply.argtypes = [vp, vp, C.POINTER(vp), i32, C.c_float, vp]
        L.sl_pack_indices.restype = i32
        L.sl_pack_indices.argtypes = [vp, vp, i64, i32, vp, vp]
        L.sl_plan_set_codes_wave_below.restype = i32
        L.sl_plan_set_codes_wave_below.argtypes = [vp, i64]
        L.sl_coded_fixed_bytes.restype = sz
        L.sl_coded_fixed_bytes.argtypes = [vp]
        L.sl_compress_coded.restype = i32
        L.sl_compress_coded.argtypes = [vp, vp, vp, C.c_float, i32, vp, vp, vp, sz, vp, vp]
        L.sl_decompress_avg_apply_coded.restype = i32
        L.sl_decompress_avg_apply_coded.argtypes = [vp, vp, C.POINTER(vp), C.POINTER(sz), i32, C.c_float, vp]
        L.sl_decompress_avg_apply_nesterov_coded.restype = i32
        L.sl_decompress_avg_apply_nesterov_coded.argtypes = [vp, vp, vp, C.POINTER(vp), C.POINTER(sz), i32,
                                                             C.c_float, C.c_float, vp]
        L.sl_rice_max_bytes.restype = sz
        L.sl_rice_max_bytes.argtypes = [vp]
        L.sl_rice_encode.restype = i32
        L.sl_rice_encode.argtypes = [vp, vp, vp, sz, vp, vp]
        L.sl_rice_decode.restype = i32
        L.sl_rice_decode.argtypes = [vp, vp, sz, vp, vp]
        L.sl_profile_begin.restype = i32
        L.sl_profile_begin.argtypes = [vp, i32]
        L.sl_profile_end.restype = i32
        L.sl_profile_end.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(i32)]
        L.sl_strerror.restype = C.c_char_p
        L.sl_strerror.argtypes = [i32]
        L.sl_last_hip_error.restype = C.c_char_p
        L.sl_last_hip_error.argtypes = []
        _lib = L
    return _lib


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream or None
    return int(stream) or None


def _dev_ptr(t: Optional[torch.Tensor], dtype=None) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected dtype {dtype}, got {t.dtype}")
    return t.data_ptr()


class Plan:
    """Owner of an sl_plan handle."""

    def __init__(self, handle: int, k: int, n_tensors: int):
        self.handle, self.k, self.n_tensors = handle, k, n_tensors

    @property
    def value_bits(self) -> int:
        return int(lib().sl_plan_value_bits(self.handle))

    @property
    def num_chunks(self) -> int:
        return int(lib().sl_plan_num_chunks(self.handle))

    @property
    def num_elements(self) -> int:
        return int(lib().sl_plan_num_elements(self.handle))

    @property
    def payload_bytes(self) -> int:
        return int(lib().sl_payload_bytes(self.handle))

    @property
    def workspace_bytes(self) -> int:
        return int(lib().sl_workspace_bytes(self.handle))

    def tensor_offset(self, t: int) -> int:
        return int(lib().sl_payload_tensor_offset(self.handle, t))

    def close(self):
        if self.handle:
            lib().sl_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def sl_plan_create(descs: Sequence[Sequence[int]], k: int) -> Plan:
    """descs: (rows, cols, offset, layout) per tensor."""
    descs = list(descs)
    arr = (SlTensor * max(1, len(descs)))()
    for i, (r, c, off, lay) in enumerate(descs):
        arr[i] = SlTensor(int(r), int(c), int(off), int(lay), 0)
    h = C.c_void_p()
    st = lib().sl_plan_create(arr, len(descs), int(k), C.byref(h))
    if st:
        raise SparseLoCoError("sl_plan_create", st)
    return Plan(h.value, int(k), len(descs))


def sl_plan_create_bits(descs: Sequence[Sequence[int]], k: int, value_bits: int) -> Plan:
    """sl_plan_create for payload values of 1, 2, 3, 4 bits or unquantized fp32 (32)."""
    descs = list(descs)
    arr = (SlTensor * max(1, len(descs)))()
    for i, (r, c, off, lay) in enumerate(descs):
        arr[i] = SlTensor(int(r), int(c), int(off), int(lay), 0)
    h = C.c_void_p()
    st = lib().sl_plan_create_bits(arr, len(descs), int(k), int(value_bits), C.byref(h))
    if st:
        raise SparseLoCoError("sl_plan_create_bits", st)
    return Plan(h.value, int(k), len(descs))


def sl_plan_value_bits(plan: Plan) -> int:
    return plan.value_bits


def sl_compress(plan: Plan, e: Optional[torch.Tensor], delta: torch.Tensor, beta: float,
                payload: torch.Tensor, workspace: torch.Tensor, flags: int = SL_COMPRESS_DEFAULT,
                pending: Optional[torch.Tensor] = None, stream=None) -> None:
    st = lib().sl_compress(plan.handle, _dev_ptr(e, torch.float32), _dev_ptr(delta, torch.float32),
                           float(beta), int(flags), _dev_ptr(pending, torch.uint8),
                           _dev_ptr(payload, torch.uint8), _dev_ptr(workspace, torch.uint8),
                           _stream_ptr(stream))
    if st:
        raise SparseLoCoError("sl_compress", st)


def sl_compress_noalloc(plan: Plan, e: Optional[torch.Tensor], delta: torch.Tensor, beta: float,
                        payload: torch.Tensor, flags: int = SL_COMPRESS_DEFAULT,
                        pending: Optional[torch.Tensor] = None, stream=None) -> None:
    """sl_compress with the library's own fixed scratch array in place of a workspace."""
    st = lib().sl_compress_noalloc(plan.handle, _dev_ptr(e, torch.float32), _dev_ptr(delta, torch.float32),
                                   float(beta), int(flags), _dev_ptr(pending, torch.uint8),
                                   _dev_ptr(payload, torch.uint8), _stream_ptr(stream))
    if st:
        raise SparseLoCoError("sl_compress_noalloc", st)


def sl_compress_random_k(plan: Plan, e: Optional[torch.Tensor], delta: torch.Tensor, beta: float,
                         payload: torch.Tensor, workspace: torch.Tensor, seed: int,
                         flags: int = SL_COMPRESS_DEFAULT, pending: Optional[torch.Tensor] = None,
                         stream=None) -> None:
    st = lib().sl_compress_random_k(plan.handle, _dev_ptr(e, torch.float32), _dev_ptr(delta, torch.float32),
                                    float(beta), int(flags), _dev_ptr(pending, torch.uint8),
                                    _dev_ptr(payload, torch.uint8), _dev_ptr(workspace, torch.uint8),
                                    int(seed) & 0xFFFFFFFF, _stream_ptr(stream))
    if st:
        raise SparseLoCoError("sl_compress_random_k", st)


def sl_residual_apply(plan: Plan, e: torch.Tensor, payload: torch.Tensor, stream=None) -> None:
    st = lib().sl_residual_apply(plan.handle, _dev_ptr(e, torch.float32),
                                 _dev_ptr(payload, torch.uint8), _stream_ptr(stream))
    if st:
        raise SparseLoCoError("sl_residual_apply", st)


def sl_decompress_avg_apply(plan: Plan, theta: torch.Tensor, payloads: Sequence[torch.Tensor],
                            lr: float, stream=None) -> None:
    R = len(payloads)
    ptrs = (C.c_void_p * max(1, R))(*[_dev_ptr(p, torch.uint8) for p in payloads])
    st = lib().sl_decompress_avg_apply(plan.handle, _dev_ptr(theta, torch.float32), ptrs, R,
                                       float(lr), _stream_ptr(stream))
    if st:
        raise SparseLoCoError("sl_decompress_avg_apply", st)


def sl_decompress_avg_apply_nesterov(plan: Plan, theta: torch.Tensor, momentum: torch.Tensor,
                                     payloads: Sequence[torch.Tensor], lr: float, mu: float, stream=None) -> None:
    R = len(payloads)
    ptrs = (C.c_void_p * max(1, R))(*[_dev_ptr(p, torch.uint8) for p in payloads])
    st = lib().sl_decompress_avg_apply_nesterov(plan.handle, _dev_ptr(theta, torch.float32),
                                                _dev_ptr(momentum, torch.float32), ptrs, R, float(lr),
                                                float(mu), _stream_ptr(stream))
    if st:
        raise SparseLoCoError("sl_decompress_avg_apply_nesterov", st)


def sl_lom_direction(plan: Plan, m: torch.Tensor, delta: torch.Tensor, mu: float, out: torch.Tensor,
                     stream=None) -> None:
    st = lib().sl_lom_direction(plan.handle, _dev_ptr(m, torch.float32), _dev_ptr(delta, torch.float32),
                                float(mu), _dev_ptr(out, torch.float32), _stream_ptr(stream))
    if st:
        raise SparseLoCoError("sl_lom_direction", st)


def sl_dense_avg_apply(plan: Plan, theta: torch.Tensor, momentum: Optional[torch.Tensor],
                       dirs: Sequence[torch.Tensor], lr: float, mu: float = 0.0, stream=None) -> None:
    R = len(dirs)
    ptrs = (C.c_void_p * max(1, R))(*[_dev_ptr(d, torch.float32) for d in dirs])
    st = lib().sl_dense_avg_apply(plan.handle, _dev_ptr(theta, torch.float32),
                                  _dev_ptr(momentum, torch.float32), ptrs, R, float(lr), float(mu),
                                  _stream_ptr(stream))
    if st:
        raise SparseLoCoError("sl_dense_avg_apply", st)


def sl_sub_topk(plan: Plan, m: torch.Tensor, stream=None) -> None:
    st = lib().sl_sub_topk(plan.handle, _dev_ptr(m, torch.float32), _stream_ptr(stream))
    if st:
        raise SparseLoCoError("sl_sub_topk", st)


def sl_pack_indices(idx: torch.Tensor, codes: torch.Tensor, n_chunks: int, k: int,
                    out: torch.Tensor, stream=None) -> None:
    st = lib().sl_pack_indices(_dev_ptr(idx, torch.uint16), _dev_ptr(codes, torch.uint8),
                               int(n_chunks), int(k), _dev_ptr(out, torch.uint8), _stream_ptr(stream))
    if st:
        raise SparseLoCoError("sl_pack_indices", st)


def sl_pack_indices_bits(idx: torch.Tensor, codes: Optional[torch.Tensor], values: Optional[torch.Tensor],
                         n_chunks: int, k: int, value_bits: int, out: torch.Tensor, stream=None) -> None:
    st = lib().sl_pack_indices_bits(_dev_ptr(idx, torch.uint16), _dev_ptr(codes, torch.uint8),
                                    _dev_ptr(values, torch.float32), int(n_chunks), int(k),
                                    int(value_bits), _dev_ptr(out, torch.uint8), _stream_ptr(stream))
    if st:
        raise SparseLoCoError("sl_pack_indices_bits", st)


def alloc_payload(plan: Plan, device="cuda") -> torch.Tensor:
    return torch.zeros(max(16, plan.payload_bytes), dtype=torch.uint8, device=device)


def alloc_workspace(plan: Plan, device="cuda") -> torch.Tensor:
    return torch.empty(plan.workspace_bytes, dtype=torch.uint8, device=device)


def sl_profile_begin(plan: Plan, max_calls: int) -> None:
    st = lib().sl_profile_begin(plan.handle, int(max_calls))
    if st:
        raise SparseLoCoError("sl_profile_begin", st)


def sl_profile_end(plan: Plan) -> dict:
    """-> {phase: (mean ms per call, calls)}"""
    ms = (C.c_double * len(PROF_PHASES))()
    calls = (C.c_int * len(PROF_PHASES))()
    st = lib().sl_profile_end(plan.handle, ms, calls)
    if st:
        raise SparseLoCoError("sl_profile_end", st)
    return {name: (ms[i], calls[i]) for i, name in enumerate(PROF_PHASES)}


def sl_plan_set_codes_wave_below(plan: Plan, n_chunks: int) -> None:
    st = lib().sl_plan_set_codes_wave_below(plan.handle, int(n_chunks))
    if st:
        raise SparseLoCoError("sl_plan_set_codes_wave_below", st)


def sl_coded_fixed_bytes(plan: Plan) -> int:
    return int(lib().sl_coded_fixed_bytes(plan.handle))


def alloc_coded(plan: Plan, device="cuda") -> torch.Tensor:
    return torch.zeros(max(16, sl_rice_max_bytes(plan)), dtype=torch.uint8, device=device)


def coded_size(coded: torch.Tensor) -> int:
    """Bytes of a coded buffer that travel (its header's size field; waits for the device)."""
    return int(coded[8:16].cpu().numpy().view("<u8")[0])


def sl_compress_coded(plan: Plan, e: Optional[torch.Tensor], delta: torch.Tensor, beta: float,
                      record: torch.Tensor, coded: torch.Tensor, workspace: torch.Tensor,
                      flags: int = SL_COMPRESS_DEFAULT, pending: Optional[torch.Tensor] = None,
                      stream=None) -> None:
    st = lib().sl_compress_coded(plan.handle, _dev_ptr(e, torch.float32), _dev_ptr(delta, torch.float32),
                                 float(beta), int(flags), _dev_ptr(pending, torch.uint8),
                                 _dev_ptr(record, torch.uint8), _dev_ptr(coded, torch.uint8), coded.numel(),
                                 _dev_ptr(workspace, torch.uint8), _stream_ptr(stream))
    if st:
        raise SparseLoCoError("sl_compress_coded", st)


def sl_decompress_avg_apply_coded(plan: Plan, theta: torch.Tensor, coded: Sequence[torch.Tensor],
                                  coded_bytes: Sequence[int], lr: float, stream=None) -> None:
    R = len(coded)
    ptrs = (C.c_void_p * max(1, R))(*[_dev_ptr(p, torch.uint8) for p in coded])
    sizes = (C.c_size_t * max(1, R))(*[int(b) for b in coded_bytes])
    st = lib().sl_decompress_avg_apply_coded(plan.handle, _dev_ptr(theta, torch.float32), ptrs, sizes, R,
                                             float(lr), _stream_ptr(stream))
    if st:
        raise SparseLoCoError("sl_decompress_avg_apply_coded", st)


def sl_decompress_avg_apply_nesterov_coded(plan: Plan, theta: torch.Tensor, momentum: torch.Tensor,
                                           coded: Sequence[torch.Tensor], coded_bytes: Sequence[int], lr: float,
                                           mu: float, stream=None) -> None:
    R = len(coded)
    ptrs = (C.c_void_p * max(1, R))(*[_dev_ptr(p, torch.uint8) for p in coded])
    sizes = (C.c_size_t * max(1, R))(*[int(b) for b in coded_bytes])
    st = lib().sl_decompress_avg_apply_nesterov_coded(plan.handle, _dev_ptr(theta, torch.float32),
                                                      _dev_ptr(momentum, torch.float32), ptrs, sizes, R,
                                                      float(lr), float(mu), _stream_ptr(stream))
    if st:
        raise SparseLoCoError("sl_decompress_avg_apply_nesterov_coded", st)


def sl_rice_max_bytes(plan: Plan) -> int:
    return int(lib().sl_rice_max_bytes(plan.handle))


def sl_rice_encode(plan: Plan, payload: torch.Tensor, out: torch.Tensor, workspace: torch.Tensor,
                   stream=None) -> None:
    """The coded size is in out[8:16] (little-endian uint64) once the stream work is done."""
    st = lib().sl_rice_encode(plan.handle, _dev_ptr(payload, torch.uint8), _dev_ptr(out, torch.uint8),
                              out.numel(), _dev_ptr(workspace, torch.uint8), _stream_ptr(stream))
    if st:
        raise SparseLoCoError("sl_rice_encode", st)


def sl_rice_decode(plan: Plan, coded: torch.Tensor, in_bytes: int, payload: torch.Tensor,
                   stream=None) -> None:
    st = lib().sl_rice_decode(plan.handle, _dev_ptr(coded, torch.uint8), int(in_bytes),
                              _dev_ptr(payload, torch.uint8), _stream_ptr(stream))
    if st:
        raise SparseLoCoError("sl_rice_decode", st)


def sl_compress_params(plan: Plan, e: Optional[torch.Tensor], theta_outer: torch.Tensor,
                       theta_local: torch.Tensor, beta: float, payload: torch.Tensor,
                       workspace: torch.Tensor, flags: int = SL_COMPRESS_DEFAULT,
                       pending: Optional[torch.Tensor] = None, stream=None) -> None:
    st = lib().sl_compress_params(plan.handle, _dev_ptr(e, torch.float32),
                                  _dev_ptr(theta_outer, torch.float32), _dev_ptr(theta_local, torch.float32),
                                  float(beta), int(flags), _dev_ptr(pending, torch.uint8),
                                  _dev_ptr(payload, torch.uint8), _dev_ptr(workspace, torch.uint8),
                                  _stream_ptr(stream))
    if st:
        raise SparseLoCoError("sl_compress_params", st)


def sl_payload_validate(plan: Plan, payload: torch.Tensor, workspace: torch.Tensor, stream=None) -> bool:
    """True when every record is well formed (waits for the stream)."""
    st = lib().sl_payload_validate(plan.handle, _dev_ptr(payload, torch.uint8),
                                   _dev_ptr(workspace, torch.uint8), _stream_ptr(stream))
    if st == -2:
        return False
    if st:
        raise SparseLoCoError("sl_payload_validate", st)
    return True
