"""CPU-side checks of the boundary: the shared library loads and exports every symbol
the header declares; shape arithmetic needs no GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = sorted(os.path.join(ROOT, "include", f) for f in os.listdir(os.path.join(ROOT, "include"))
                 if f.endswith(".h"))
LIB = os.path.join(ROOT, "paper_2602_20191_amd", "libmbq.so")


def declared_symbols():
    names = set()
    for header in HEADERS:
        text = open(header).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names.update(re.findall(r"\b(mbq_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        import paper_2602_20191_amd.build as b

        b.build()
    return ctypes.CDLL(LIB)


def test_header_declares_the_entry_points():
    names = declared_symbols()
    for must in ("mbq_encode", "mbq_route", "mbq_linear", "mbq_unpack", "mbq_dequant", "mbq_blob_bytes"):
        assert must in names


def test_library_exports_every_declared_symbol(lib):
    for name in declared_symbols():
        assert hasattr(lib, name), name


def test_binding_lists_the_same_symbols():
    import paper_2602_20191_amd as pkg

    assert sorted(pkg.EXPORTS) == declared_symbols()


def test_shape_arithmetic_matches_the_documented_blob_format(lib):
    import oracle as O

    lib.mbq_blob_bytes.restype = ctypes.c_size_t
    lib.mbq_blob_bytes.argtypes = [ctypes.c_int64, ctypes.c_int64]
    lib.mbq_last_error.restype = ctypes.c_char_p
    for N, K in [(16, 256), (21, 384), (3, 128), (4096, 4096), (11008, 4096), (8192, 28672)]:
        assert lib.mbq_blob_bytes(N, K) == O.blob_bytes(N, K)
    assert lib.mbq_blob_bytes(16, 100) == 0          # K not a multiple of the group size
    assert b"multiple" in lib.mbq_last_error()
    assert lib.mbq_blob_bytes(0, 128) == 0
    assert lib.mbq_blob_bytes(-1, 128) == 0


def test_argument_errors_are_reported_without_a_gpu(lib):
    lib.mbq_linear.restype = ctypes.c_int
    lib.mbq_linear.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                               ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                               ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p]
    lib.mbq_route.restype = ctypes.c_int
    lib.mbq_route.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
                              ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                              ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    # bad shape, bad algo, null pointers, unsupported precision count: all refused before any launch
    assert lib.mbq_linear(None, 4, None, 16, 100, None, None, None, None, None, 0, 0, None) == 2
    assert lib.mbq_linear(None, 4, None, 16, 128, None, None, None, None, None, 0, 9, None) == 1
    assert lib.mbq_linear(None, 4, None, 16, 128, None, None, None, None, None, 0, 0, None) == 1
    assert lib.mbq_linear(None, 0, None, 16, 128, None, None, None, None, None, 0, 0, None) == 0   # T = 0: no-op
    assert lib.mbq_route(None, 4, 128, None, None, 3, None, None, None, None, None, 0, None) == 2
    assert lib.mbq_route(None, 4, 128, None, None, 4, None, None, None, None, None, 0, None) == 1


def test_route_workspace_contract(lib):
    """The workspace needs the documented 256-byte alignment (refused before any launch) and the headers no longer
    ask the caller to clear it."""
    lib.mbq_route.restype = ctypes.c_int
    lib.mbq_route.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
                              ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                              ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.mbq_last_error.restype = ctypes.c_char_p
    fake = 0x10000                                            # never dereferenced: the call is refused first
    for ws in (fake + 8, fake + 64, fake + 128):
        assert lib.mbq_route(fake, 4, 128, fake, fake, 4, fake, fake, fake, None, ws, 256, None) == 3
        assert b"misaligned" in lib.mbq_last_error()
    assert lib.mbq_route(fake, 4, 128, fake, fake, 4, fake, fake, fake, None, fake, 255, None) == 3
    for header in HEADERS:
        text = open(header).read()
        assert "ZERO before" not in text and "zero before first use" not in text


def test_hooks_and_static_scratch(lib):
    lib.mbq_set_knob.restype = ctypes.c_int
    lib.mbq_set_knob.argtypes = [ctypes.c_int, ctypes.c_int]
    assert lib.mbq_set_knob(6, 1) != 0                        # the old "skip the preparation" hook is gone
    assert lib.mbq_set_knob(8, 1) != 0 and lib.mbq_set_knob(-1, 0) != 0
    assert lib.mbq_set_knob(4, 0) == 0
    lib.mbq_static_scratch_bytes.restype = ctypes.c_size_t
    assert lib.mbq_static_scratch_bytes() == 8 << 20


def test_configuration_checks_need_no_gpu(lib):
    """Which slice configurations the library runs is decided from the numbers alone."""
    class Cfg(ctypes.Structure):
        _fields_ = [("n_slices", ctypes.c_int), ("slice_bits", ctypes.c_int * 4), ("group", ctypes.c_int)]

    def cfg(bits, group=128):
        c = Cfg()
        c.n_slices = len(bits)
        for e, b in enumerate(bits[:4]):
            c.slice_bits[e] = b
        c.group = group
        return c

    lib.mbq_config_check.restype = ctypes.c_int
    lib.mbq_config_bits.restype = ctypes.c_int
    lib.mbq_config_precision_value.restype = ctypes.c_int
    lib.mbq_config_counts_bits.restype = ctypes.c_int
    for bits in [(2, 2, 2, 2), (4, 2, 2), (2, 4, 2), (4, 4), (6, 2), (8,), (2, 2, 2), (2,)]:
        c = cfg(bits)
        assert lib.mbq_config_check(ctypes.byref(c)) == 0, bits
        acc = 0
        for p, b in enumerate(bits):
            acc += b
            assert lib.mbq_config_bits(ctypes.byref(c), p) == acc
            assert lib.mbq_config_precision_value(ctypes.byref(c), p) == acc // 2 - 1
        assert lib.mbq_config_counts_bits(ctypes.byref(c)) == 0
        assert lib.mbq_config_bits(ctypes.byref(c), len(bits)) == -1
    for bits in [(3, 1, 2, 2), (3, 2, 1), (1, 1), (4, 1, 1, 2), (5,), (1, 2, 2, 2)]:     # an odd cumulative width
        c = cfg(bits)
        assert lib.mbq_config_check(ctypes.byref(c)) == 0, bits
        assert lib.mbq_config_counts_bits(ctypes.byref(c)) == 1
        acc = 0
        for p, b in enumerate(bits):
            acc += b
            assert lib.mbq_config_bits(ctypes.byref(c), p) == acc
            assert lib.mbq_config_precision_value(ctypes.byref(c), p) == acc - 1
    for bits, group in [((2, 2, 2, 2), 16), ((2, 2, 2, 2), 96), ((2, 2, 2, 2), 256), ((4, 4, 2), 128), ((3, 3, 3), 128),
                        ((), 128), ((0, 2), 128), ((2, 2, 2, 2, 2), 128)]:
        c = cfg(bits, group)
        assert lib.mbq_config_check(ctypes.byref(c)) == 2, (bits, group)
    assert lib.mbq_config_check(None) == 2
    # groups of 64 and 32 columns: same code section, 256 / group {s0, z0} pairs per row and 256-column tile
    lib.mbq_blob_bytes_cfg.restype = ctypes.c_size_t
    lib.mbq_blob_bytes_cfg.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64]
    lib.mbq_blob_bytes.restype = ctypes.c_size_t
    lib.mbq_blob_bytes.argtypes = [ctypes.c_int64, ctypes.c_int64]
    N, K = 37, 640                                                   # 3 row tiles x 3 column tiles
    code_bytes = 4 * 3 * 3 * 1024
    for group, per_tile in ((128, 2), (64, 4), (32, 8)):
        c = cfg((3, 2, 1), group)
        assert lib.mbq_config_check(ctypes.byref(c)) == 0
        assert lib.mbq_blob_bytes_cfg(ctypes.byref(c), N, K) == code_bytes + 3 * 3 * per_tile * 16 * 8
    assert lib.mbq_blob_bytes_cfg(ctypes.byref(cfg((2, 2, 2, 2))), N, K) == lib.mbq_blob_bytes(N, K)
    assert lib.mbq_blob_bytes_cfg(ctypes.byref(cfg((2, 2, 2, 2), 48)), N, K) == 0
    assert lib.mbq_blob_bytes_cfg(ctypes.byref(cfg((2, 2, 2, 2), 64)), N, 192) == 0      # K stays a multiple of 128


def test_activation_quantiser_arguments_are_checked_without_a_gpu(lib):
    lib.mbq_act_quant.restype = ctypes.c_int
    lib.mbq_act_quant.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int] + [ctypes.c_void_p] * 6
    lib.mbq_scale_rows.restype = ctypes.c_int
    lib.mbq_scale_rows.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64] + [ctypes.c_void_p] * 3
    fake = 0x10000                                            # never dereferenced: the calls are refused first
    assert lib.mbq_act_quant(fake, 4, 100, 4, None, None, fake, fake, None, None) == 2      # K not a multiple of 128
    assert lib.mbq_act_quant(fake, 4, 128, 1, None, None, fake, fake, None, None) == 1      # abits
    assert lib.mbq_act_quant(fake, 4, 128, 9, None, None, fake, fake, None, None) == 1
    assert lib.mbq_act_quant(fake, 4, 128, 4, fake, None, fake, fake, None, None) == 1      # shift without scale
    assert lib.mbq_act_quant(fake + 2, 4, 128, 4, None, None, fake, fake, None, None) == 1  # misaligned X
    assert lib.mbq_act_quant(None, 4, 128, 4, None, None, fake, fake, None, None) == 1
    assert lib.mbq_act_quant(None, 0, 128, 4, None, None, None, None, None, None) == 0      # no tokens: nothing to do
    assert lib.mbq_scale_rows(None, 4, 16, fake, None, None) == 1
    assert lib.mbq_scale_rows(fake, 4, 0, fake, None, None) == 2
    assert lib.mbq_scale_rows(None, 0, 16, None, None, None) == 0
