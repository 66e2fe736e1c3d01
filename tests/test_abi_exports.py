"""The C-ABI library loads and exports every function include/sparseloco.h declares
(no compute calls: this runs without a GPU)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "sparseloco.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sl_[a-z_0-9]+)\s*\(", text)))


def test_header_functions_are_exported_and_bound():
    from paper_2508_15706_amd import binding
    names = declared_functions()
    assert {"sl_compress", "sl_decompress_avg_apply", "sl_pack_indices"} <= set(names)
    lib = ctypes.CDLL(binding.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in sparseloco.h but not exported"
    assert sorted(binding.EXPORTS) == names
    for n in ("sl_compress", "sl_decompress_avg_apply", "sl_pack_indices", "sl_plan_create"):
        assert callable(getattr(binding, n))


def test_host_side_argument_validation_needs_no_gpu():
    """Bad shapes are rejected before any device work."""
    from paper_2508_15706_amd import binding
    L = binding.lib()
    assert L.sl_strerror(0) == b"ok" and L.sl_strerror(-1) == b"invalid argument"
    h = ctypes.c_void_p()
    bad = (binding.SlTensor * 1)(binding.SlTensor(64, 64, 0, 1, 0))
    assert L.sl_plan_create(bad, 1, 6, ctypes.byref(h)) == -1          # k % 4 != 0
    assert L.sl_plan_create(bad, 1, 8192, ctypes.byref(h)) == -1       # k > 4096
    small = (binding.SlTensor * 1)(binding.SlTensor(1, 100, 0, 0, 0))
    assert L.sl_plan_create(small, 1, 128, ctypes.byref(h)) == -1      # chunk smaller than k
    odd = (binding.SlTensor * 1)(binding.SlTensor(64, 64, 2, 1, 0))
    assert L.sl_plan_create(odd, 1, 32, ctypes.byref(h)) == -1         # misaligned offset
    # limits: products that would overflow 64 bits, or work lists too long to build, are refused up front
    for rows, cols, lay in ((1 << 40, 1 << 40, 0), (1 << 62, 4, 0), (1 << 23, 1 << 24, 1), (1 << 20, 1 << 25, 0),
                            (1 << 22, 1 << 22, 1)):
        huge = (binding.SlTensor * 1)(binding.SlTensor(rows, cols, 0, lay, 0))
        assert L.sl_plan_create(huge, 1, 64, ctypes.byref(h)) == -1, (rows, cols, lay)
    two = (binding.SlTensor * 2)(binding.SlTensor(64, 64, 0, 1, 0), binding.SlTensor(64, 64, 4092, 1, 0))
    assert L.sl_plan_create(two, 2, 64, ctypes.byref(h)) == -1         # overlapping tensors
    assert L.sl_plan_create_bits(bad, 1, 64, 5, ctypes.byref(h)) == -1   # no such value width
    assert L.sl_plan_create_bits(bad, 1, 4, 3, ctypes.byref(h)) == -1    # records must end on a byte
    assert h.value is None
    assert L.sl_pack_indices(None, None, 1, 6, None, None) == -1
    assert L.sl_payload_bytes(None) == 0
