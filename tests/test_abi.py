"""Host-side checks that need no GPU: the C-ABI library loads, exports every
symbol the header declares, and validates arguments before touching a device."""
import ctypes
import os
import re

from paper_2508_06753_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "w2mm.h")).read()
    return sorted(set(re.findall(r"W2_API\s+(?:const\s+char\*|int)\s+(w2_\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert len(names) >= 13
    lib = ctypes.CDLL(binding.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in w2mm.h but not exported"
    assert sorted(binding.EXPORTED) == names


def test_tuning_structure_matches_the_header():
    # the binding's ctypes mirror of w2_tuning_t: the header's fields, all int, in the header's order
    text = open(os.path.join(ROOT, "include", "w2mm.h")).read()
    body = re.search(r"typedef struct \{(.*?)\} w2_tuning_t;", text, re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"\bint\s+(\w+)\s*;", body)
    assert len(fields) >= 20 and len(re.findall(r";", body)) == len(fields), "a field that is not a plain int"
    assert [n for n, _ in binding.Tuning._fields_] == fields
    assert all(t is ctypes.c_int for _, t in binding.Tuning._fields_)
    assert ctypes.sizeof(binding.Tuning) == 4 * len(fields)


def test_sizes_and_shape_rules_on_host():
    lib = binding.raw()
    assert binding.packed_size(4096, 4096, 128) == 4096 * 4096 // 4 + (4096 // 128) * 4096 * 2
    assert binding.packed_size(4096, 28672, 64) == 4096 * 28672 // 4 + (4096 // 64) * 28672 * 2
    # N padded to a multiple of 16 inside the blob
    assert binding.packed_size(256, 8, 128) == 16 * 256 // 4 + 256
    assert binding.workspace_size(1, 4096, 4096, 128) == 0
    out = ctypes.c_size_t(0)
    for K, N, G, rc in [(100, 64, 128, binding.ERR_UNSUPPORTED_SHAPE),
                        (256, 60, 128, binding.ERR_UNSUPPORTED_SHAPE),
                        (256, 64, 96, binding.ERR_UNSUPPORTED_SHAPE),
                        (0, 64, 128, binding.ERR_INVALID_ARG),
                        (256, -8, 128, binding.ERR_INVALID_ARG)]:
        assert lib.w2_packed_size(K, N, G, ctypes.byref(out)) == rc
        assert lib.w2_last_error() != b""
    assert lib.w2_packed_size(256, 64, 128, None) == binding.ERR_INVALID_ARG
    assert lib.w2_status_string(0) == b"ok"
    assert lib.w2_status_string(binding.ERR_MISALIGNED) == b"misaligned pointer or stride"


def test_null_and_misaligned_arguments_rejected_before_launch():
    lib = binding.raw()
    # all of these fail validation, so no device is touched
    assert lib.w2_prepack(None, None, 256, 64, 128, 0, None, 0, None, None) == binding.ERR_INVALID_ARG
    assert lib.w2_prepack(ctypes.c_void_p(16), ctypes.c_void_p(16), 256, 64, 128, 7,
                          ctypes.c_void_p(16), 1 << 20, None, None) == binding.ERR_INVALID_ARG
    assert lib.w2_prepack(ctypes.c_void_p(16), ctypes.c_void_p(16), 256, 64, 128, 0,
                          ctypes.c_void_p(24), 1 << 20, None, None) == binding.ERR_MISALIGNED
    assert lib.w2_prepack(ctypes.c_void_p(16), ctypes.c_void_p(16), 256, 64, 128, 0,
                          ctypes.c_void_p(32), 100, None, None) == binding.ERR_BUFFER_TOO_SMALL
    assert lib.w2_quantize_rows(None, 0, 1, 256, 256, 128, None, None, None, None) == binding.ERR_INVALID_ARG
    assert lib.w2_quantize_rows(ctypes.c_void_p(16), 0, 1, 256, 100, 128, ctypes.c_void_p(16),
                                ctypes.c_void_p(16), None, None) == binding.ERR_MISALIGNED
    assert lib.w2_quantize_rows(None, 0, 0, 256, 256, 128, None, None, None, None) == 0   # M == 0
    assert lib.w2_matmul_a8(None, 256, 64, 128, None, None, 1, None, 64, None, 0, None) == binding.ERR_INVALID_ARG
    assert lib.w2_matmul_a16(None, 256, 64, 128, None, 256, 1, None, 64, None, 0, None) == binding.ERR_INVALID_ARG
    assert lib.w2_matmul_a16(None, 256, 64, 128, None, 256, 0, None, 64, None, 0, None) == 0
