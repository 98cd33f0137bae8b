"""Host-only checks of the C ABI library: it loads, exports every symbol the
header declares, validates descriptions without touching a device, and plans
layouts that respect the LDS budget.  No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2506_17255_amd as skl
from paper_2506_17255_amd import build as skl_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def built():
    if not os.path.exists(skl_build.lib_path()):
        skl_build.build_library()
    skl.load_library()


def header_symbols():
    names = set()
    for fn in os.listdir(os.path.join(ROOT, "include")):
        if fn.endswith(".h"):
            txt = open(os.path.join(ROOT, "include", fn)).read()
            txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
            names |= set(re.findall(r"\b(sketch_linear_\w+)\s*\(", txt))
    return names


def test_library_exports_every_declared_symbol():
    L = skl.load_library()
    decl = header_symbols()
    assert decl == set(skl.EXPORTS)
    for n in decl:
        assert hasattr(L, n), n


def test_struct_sizes_match_header_layout():
    assert ctypes.sizeof(skl.skl_desc_t) == 96
    assert skl.skl_desc_t.state_bits.offset == skl.SKL_DESC_SIZE_V1 == 72
    assert ctypes.sizeof(skl.skl_info_t) == 64
    assert skl.skl_info_t.decode_segments.offset == skl.SKL_INFO_SIZE_V1 == 40


def good(**over):
    kw = dict(in_features=8, out_features=16, tile_in=4, tile_out=8, d=2,
              hash_a=np.uint32([3, 5]), hash_c=np.uint32([7, 11]),
              group_width=np.uint32([3, 4, 5, 6]), states=np.zeros(2 * 18, dtype=np.uint16))
    kw.update(over)
    return skl.make_desc(**kw)


def status_of(desc):
    try:
        skl.sketch_linear_device_bytes(desc)
        return skl.SKL_OK
    except skl.SketchLinearError as e:
        assert e.message, "every failure carries a message"
        return e.status


def test_valid_description_is_accepted():
    assert status_of(good()) == skl.SKL_OK
    assert skl.sketch_linear_device_bytes(good()) >= 4096 + 2 * 36


@pytest.mark.parametrize("over,status", [
    (dict(struct_size=8), skl.SKL_ERR_INVALID_ARG),
    (dict(in_features=0), skl.SKL_ERR_INVALID_ARG),
    (dict(tile_in=3), skl.SKL_ERR_INVALID_ARG),
    (dict(tile_out=5), skl.SKL_ERR_INVALID_ARG),
    (dict(d=0), skl.SKL_ERR_INVALID_ARG),
    (dict(d=9), skl.SKL_ERR_INVALID_ARG),
    (dict(query_mode=2), skl.SKL_ERR_INVALID_ARG),
    (dict(flags=8), skl.SKL_ERR_INVALID_ARG),
    (dict(flags=6), skl.SKL_ERR_INVALID_ARG),
    (dict(hash_a=None), skl.SKL_ERR_INVALID_ARG),
    (dict(states=None, n_states=36), skl.SKL_ERR_INVALID_ARG),
    (dict(hash_a=np.uint32([1 << 24, 5])), skl.SKL_ERR_INVALID_ARG),
    (dict(hash_c=np.uint32([7, 1 << 24])), skl.SKL_ERR_INVALID_ARG),
    (dict(group_width=np.uint32([3, 0, 5, 6]), states=np.zeros(28, dtype=np.uint16)), skl.SKL_ERR_INVALID_ARG),
    (dict(group_width=np.uint32([3, 65536, 5, 6])), skl.SKL_ERR_INVALID_ARG),
    (dict(n_states=35), skl.SKL_ERR_INVALID_ARG),
    (dict(states=np.uint16([0] * 35 + [0x7C00])), skl.SKL_ERR_NONFINITE),
    (dict(states=np.uint16([0xFE00] + [0] * 35)), skl.SKL_ERR_NONFINITE),
])
def test_bad_descriptions_are_rejected(over, status):
    assert status_of(good(**over)) == status


def test_group_address_space_limit():
    d = good(in_features=1 << 13, out_features=1 << 12, tile_in=1 << 13, tile_out=1 << 12,
             group_width=np.uint32([1]), states=np.zeros(2, dtype=np.uint16))
    assert status_of(d) == skl.SKL_ERR_INVALID_ARG          # 2^25 addresses in one group


def test_table_too_large_for_lds_is_unsupported():
    K = 65535
    d = good(in_features=4, out_features=4, tile_in=4, tile_out=4, d=8,
             hash_a=np.arange(1, 9, dtype=np.uint32), hash_c=np.arange(8, dtype=np.uint32),
             group_width=np.uint32([K]), states=np.zeros(8 * K, dtype=np.uint16))
    assert status_of(d) == skl.SKL_ERR_UNSUPPORTED


def test_null_arguments():
    L = skl.load_library()
    n = ctypes.c_uint64(0)
    assert L.sketch_linear_device_bytes(None, ctypes.byref(n)) == skl.SKL_ERR_INVALID_ARG
    assert L.sketch_linear_device_bytes(ctypes.byref(good()), None) == skl.SKL_ERR_INVALID_ARG
    h = ctypes.c_void_p(None)
    assert L.sketch_linear_create(ctypes.byref(good()), None, 1 << 20, None, ctypes.byref(h)) == skl.SKL_ERR_INVALID_ARG
    assert "dev_buf" in skl.sketch_linear_last_error()
    assert L.sketch_linear_create(ctypes.byref(good()), 4096, 16, None, ctypes.byref(h)) == skl.SKL_ERR_BUFFER_TOO_SMALL
    assert L.sketch_linear_create(ctypes.byref(good()), 4097, 1 << 20, None, ctypes.byref(h)) == skl.SKL_ERR_INVALID_ARG
    assert L.sketch_linear_create(ctypes.byref(good()), 4096, 1 << 20, None, None) == skl.SKL_ERR_INVALID_ARG
    assert L.sketch_linear_gemv(None, 16, 0, 8, 32, 2, 16, 1, 64, 0, None) == skl.SKL_ERR_INVALID_ARG
    assert L.sketch_linear_gemm(None, 16, 0, 8, 32, 2, 16, 1, 64, 0, None) == skl.SKL_ERR_INVALID_ARG
    assert L.sketch_linear_reconstruct(None, 16, None, 0, None) == skl.SKL_ERR_INVALID_ARG
    assert L.sketch_linear_workspace_bytes(None, 0, 1, ctypes.byref(n)) == skl.SKL_ERR_INVALID_ARG
    assert L.sketch_linear_info(None, None) == skl.SKL_ERR_INVALID_ARG
    assert L.sketch_linear_gemv_partials(None, None, 0, 0, 1, None, 0, None) == skl.SKL_ERR_INVALID_ARG
    L.sketch_linear_destroy(None)


def test_device_bytes_scale_with_the_sketch_not_with_the_layer():
    # 0.5 bit/weight row sketches of a 4096 x 11008 layer: the library keeps
    # two copies of the tables (one with a padding word per state row, one
    # without) of about 1/16 byte per weight each, far below the 2 bytes of fp16
    in_f, out_f, d, K = 4096, 11008, 4, 86
    desc = skl.make_desc(in_f, out_f, 1, out_f, d, np.uint32([3, 5, 7, 9]), np.uint32([1, 2, 3, 4]),
                         np.full(in_f, K, dtype=np.uint32), np.zeros(in_f * d * K, dtype=np.uint16))
    nbytes = skl.sketch_linear_device_bytes(desc)
    assert 2 * in_f * d * K * 2 <= nbytes <= 2.3 * in_f * d * K * 2
    assert nbytes < 0.15 * in_f * out_f


# ------------------------------------------------------------ low-bit states
def good_lowbit(bits=4, **over):
    n = 2 * 18
    codes = np.zeros(n if bits == 8 else (n + 1) // 2, dtype=np.uint8)
    kw = dict(states=None, n_states=n, state_bits=bits, codes=codes, scales=np.zeros(4 * 2, dtype=np.uint16))
    kw.update(over)
    return good(**kw)


def test_first_version_of_the_descriptor_is_still_accepted():
    assert status_of(good(struct_size=skl.SKL_DESC_SIZE_V1)) == skl.SKL_OK
    # in the first layout the trailing fields do not exist: whatever follows the struct is not read
    d = good(struct_size=skl.SKL_DESC_SIZE_V1, state_bits=4)
    assert status_of(d) == skl.SKL_OK


@pytest.mark.parametrize("bits", [8, 4])
def test_low_bit_description_is_accepted_and_smaller(bits):
    assert status_of(good_lowbit(bits)) == skl.SKL_OK
    in_f, out_f, d, K = 4096, 11008, 4, 86
    n = in_f * d * K
    args = (in_f, out_f, 1, out_f, d, np.uint32([3, 5, 7, 9]), np.uint32([1, 2, 3, 4]), np.full(in_f, K, dtype=np.uint32))
    full = skl.sketch_linear_device_bytes(skl.make_desc(*args, np.zeros(n, dtype=np.uint16)))
    low = skl.sketch_linear_device_bytes(skl.make_desc(*args, None, n_states=n, state_bits=bits,
                                                       codes=np.zeros(n * bits // 8, dtype=np.uint8),
                                                       scales=np.zeros(in_f * d, dtype=np.uint16)))
    # resident: codes, scales and metadata only (the 16-bit tables are expanded per call in the workspace)
    assert n * bits // 8 <= low <= n * bits // 8 + 400 * 1024
    assert low < full * (bits / 32 + 0.05)


@pytest.mark.parametrize("over,status", [
    (dict(state_bits=5), skl.SKL_ERR_INVALID_ARG),
    (dict(reserved_=1), skl.SKL_ERR_INVALID_ARG),
    (dict(codes=None), skl.SKL_ERR_INVALID_ARG),
    (dict(scales=None), skl.SKL_ERR_INVALID_ARG),
    (dict(states=np.zeros(36, dtype=np.uint16)), skl.SKL_ERR_INVALID_ARG),       # both forms at once
    (dict(scales=np.uint16([0, 0, 0x7C00, 0, 0, 0, 0, 0])), skl.SKL_ERR_NONFINITE),
    (dict(scales=np.uint16([0, 0, 0xBC00, 0, 0, 0, 0, 0])), skl.SKL_ERR_INVALID_ARG),
    (dict(codes=np.uint8([0] * 17 + [0x80])), skl.SKL_ERR_INVALID_ARG),          # the nibble -8
    (dict(codes=np.uint8([0x08] + [0] * 17)), skl.SKL_ERR_INVALID_ARG),
    (dict(n_states=35), skl.SKL_ERR_INVALID_ARG),
])
def test_bad_low_bit_descriptions_are_rejected(over, status):
    reserved = over.pop("reserved_", 0)
    d = good_lowbit(4, **over)
    d.reserved = reserved
    assert status_of(d) == status


def test_eight_bit_code_minus_128_is_rejected():
    codes = np.zeros(36, dtype=np.uint8)
    codes[7] = 0x80
    assert status_of(good_lowbit(8, codes=codes)) == skl.SKL_ERR_INVALID_ARG
    codes[7] = 0x81                                          # -127 is the end code
    assert status_of(good_lowbit(8, codes=codes)) == skl.SKL_OK


# ------------------------------------------------------ sketch construction
def test_build_workspace_and_argument_checks():
    geom = good(states=None, n_states=36)                    # a description without states: enough for construction
    need = skl.sketch_linear_build_workspace_bytes(geom)
    assert need >= 36 * 8 + 5 * 8 + 4 * 4
    L = skl.load_library()
    n = ctypes.c_uint64(0)
    assert L.sketch_linear_build_workspace_bytes(None, ctypes.byref(n)) == skl.SKL_ERR_INVALID_ARG
    assert L.sketch_linear_build_workspace_bytes(ctypes.byref(geom), None) == skl.SKL_ERR_INVALID_ARG
    assert L.sketch_linear_build_states(ctypes.byref(geom), None, None, None, 0, None) == skl.SKL_ERR_INVALID_ARG
    assert L.sketch_linear_build_states(ctypes.byref(geom), 4096, 8192, 256 * 64, 8, None) == skl.SKL_ERR_BUFFER_TOO_SMALL
    assert L.sketch_linear_build_states(ctypes.byref(geom), 4096 + 2, 8192, 256 * 64, need, None) == skl.SKL_ERR_INVALID_ARG
    bad = good(states=None, n_states=35)
    assert L.sketch_linear_build_workspace_bytes(ctypes.byref(bad), ctypes.byref(n)) == skl.SKL_ERR_INVALID_ARG


def test_grouped_decode_null_arguments():
    L = skl.load_library()
    n = ctypes.c_uint64(0)
    assert L.sketch_linear_gemv_group_workspace_bytes(None, 1, 1, ctypes.byref(n)) == skl.SKL_ERR_INVALID_ARG
    one = (ctypes.c_void_p * 1)(None)
    assert L.sketch_linear_gemv_group_workspace_bytes(one, 1, 1, ctypes.byref(n)) == skl.SKL_ERR_INVALID_ARG
    assert L.sketch_linear_gemv_group_workspace_bytes(one, 0, 1, ctypes.byref(n)) == skl.SKL_ERR_INVALID_ARG
    assert L.sketch_linear_gemv_group(one, 1, None, 0, 0, one, 0, 0, 1, None, 0, None) == skl.SKL_ERR_INVALID_ARG
    assert L.sketch_linear_gemv_gate_up(None, None, None, 0, 0, None, 0, 0, 1, None, 0, None) == skl.SKL_ERR_INVALID_ARG


def test_microbench_argument_checks():
    """The ceiling kernels (kinds 0..4) check their arguments before anything is launched."""
    L = skl.load_library()
    work = ctypes.c_uint64(0)
    fake = ctypes.c_void_p(256)                 # aligned, never dereferenced by the checks
    assert L.sketch_linear_microbench(5, 10, fake, 1 << 23, None, ctypes.byref(work)) == skl.SKL_ERR_INVALID_ARG
    assert b"kind" in L.sketch_linear_last_error()
    assert L.sketch_linear_microbench(4, 10, None, 1 << 23, None, ctypes.byref(work)) == skl.SKL_ERR_INVALID_ARG
    assert L.sketch_linear_microbench(4, 10, ctypes.c_void_p(264), 1 << 23, None, ctypes.byref(work)) == skl.SKL_ERR_INVALID_ARG
    assert L.sketch_linear_microbench(4, 0, fake, 1 << 23, None, ctypes.byref(work)) == skl.SKL_ERR_INVALID_ARG
    assert L.sketch_linear_microbench(2, (1 << 20) + 1, fake, 1 << 23, None, ctypes.byref(work)) == skl.SKL_ERR_INVALID_ARG
    assert L.sketch_linear_microbench(4, 10, fake, 1 << 23, None, None) == skl.SKL_ERR_INVALID_ARG
