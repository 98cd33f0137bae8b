"""Host-only checks of the flat layer file: a description written to an image (or a file) and opened again gives
the same geometry, parameters, widths and states; anything that is not an intact layer file is refused."""
import ctypes
import struct

import numpy as np
import pytest

import oracle
import paper_2506_17255_amd as skl
import workloads as wk
from skl_harness import desc_of as harness_desc_of


def small_sketch(bits=0, d=3, tile_in=1):
    rng = np.random.default_rng(77 + bits)
    in_f, out_f = 24, 40
    tile_out = out_f if tile_in == 1 else 20
    n_groups = (in_f // tile_in) * (out_f // tile_out)
    widths = rng.integers(3, 17, size=n_groups).astype(np.uint32)
    A = (2 * rng.integers(0, 1 << 23, size=d) + 1).astype(np.uint32)
    C = rng.integers(0, 1 << 24, size=d).astype(np.uint32)
    states = (rng.standard_normal(int(widths.sum()) * d).astype(np.float32) * np.float32(0.05)).astype(np.float16).view(np.uint16)
    sk = oracle.Sketch(in_f, out_f, tile_in, tile_out, d, A, C, widths, states)
    return oracle.quantize(sk, bits) if bits else sk


def desc_of(sk, query_mode=0, flags=0, struct_size=None):
    desc = harness_desc_of(sk, flags, query_mode)
    if struct_size is not None:
        desc.struct_size = struct_size
    return desc


def array_at(ptr, n, dtype):
    if not n:
        return np.zeros(0, dtype=dtype)
    return np.frombuffer((ctypes.c_char * (n * np.dtype(dtype).itemsize)).from_address(ptr), dtype=dtype).copy()


def same_description(a, b, n_groups):
    for f in ("in_features", "out_features", "tile_in", "tile_out", "d", "query_mode", "flags", "n_states"):
        assert getattr(a, f) == getattr(b, f), f
    assert (a.state_bits or 0) % 16 == (b.state_bits or 0) % 16
    assert np.array_equal(array_at(a.hash_a, a.d, np.uint32), array_at(b.hash_a, b.d, np.uint32))
    assert np.array_equal(array_at(a.hash_c, a.d, np.uint32), array_at(b.hash_c, b.d, np.uint32))
    assert np.array_equal(array_at(a.group_width, n_groups, np.uint32), array_at(b.group_width, n_groups, np.uint32))
    if a.state_bits in (8, 4):
        nbytes = a.n_states if a.state_bits == 8 else (a.n_states + 1) // 2
        assert np.array_equal(array_at(a.codes, nbytes, np.uint8), array_at(b.codes, nbytes, np.uint8))
        assert np.array_equal(array_at(a.scales, n_groups * a.d, np.uint16), array_at(b.scales, n_groups * b.d, np.uint16))
    else:
        assert np.array_equal(array_at(a.states, a.n_states, np.uint16), array_at(b.states, b.n_states, np.uint16))


@pytest.mark.parametrize("bits,tile_in,mode", [(0, 1, 0), (0, 4, 1), (8, 1, 0), (4, 1, 1), (4, 4, 0)])
def test_a_layer_file_gives_the_description_back(bits, tile_in, mode, tmp_path):
    sk = small_sketch(bits, tile_in=tile_in)
    desc = desc_of(sk, query_mode=mode, flags=2 if tile_in == 1 else 0)
    n_groups = len(sk.group_width)
    n = skl.sketch_linear_file_bytes(desc)
    assert n % 64 == 0 and n >= 128
    image = np.zeros(n, dtype=np.uint8)
    skl.sketch_linear_file_write(desc, image)
    assert bytes(image[:8]) == b"SKLAYER1"
    back = skl.sketch_linear_file_open(image)
    assert back.state_bits == bits
    same_description(desc, back, n_groups)
    # through a file on disk: the same bytes, and a read-write memory map of it opens in place
    path = tmp_path / "layer.skl"
    skl.sketch_linear_file_save(desc, str(path))
    assert path.read_bytes() == image.tobytes()
    mapped = np.memmap(path, dtype=np.uint8, mode="r+")
    same_description(desc, skl.sketch_linear_file_open(mapped), n_groups)
    # the plan of the reopened layer is the plan of the original
    assert skl.sketch_linear_plan(back)[0] == skl.sketch_linear_plan(desc)[0]


def test_the_first_version_of_the_description_struct_can_be_saved():
    sk = small_sketch()
    desc = desc_of(sk, struct_size=skl.SKL_DESC_SIZE_V1)
    image = np.zeros(skl.sketch_linear_file_bytes(desc), dtype=np.uint8)
    skl.sketch_linear_file_write(desc, image)
    same_description(desc_of(sk), skl.sketch_linear_file_open(image), len(sk.group_width))


def test_what_is_not_an_intact_layer_file_is_refused():
    sk = small_sketch()
    desc = desc_of(sk)
    n = skl.sketch_linear_file_bytes(desc)
    good = np.zeros(n, dtype=np.uint8)
    skl.sketch_linear_file_write(desc, good)

    def refused(image, status=skl.SKL_ERR_INVALID_ARG, why=""):
        with pytest.raises(skl.SketchLinearError) as err:
            skl.sketch_linear_file_open(image)
        assert err.value.status == status, err.value
        assert why in err.value.message, err.value

    refused(np.zeros(64, dtype=np.uint8), why="header")         # shorter than a header
    bad = good.copy(); bad[0] ^= 1; refused(bad, why="magic")
    bad = good.copy(); bad[8:12] = np.frombuffer(struct.pack("<I", 2), dtype=np.uint8)
    refused(bad, skl.SKL_ERR_UNSUPPORTED)                       # another version
    refused(good[:n - 64].copy(), why="truncated")
    for pos in (20, 130, n - 1):                                # a flipped bit in the header, the parameters, the states
        bad = good.copy(); bad[pos] ^= 4; refused(bad, why="checksum")
    # a consistent checksum does not make impossible offsets acceptable
    bad = good.copy()
    bad[64:72] = np.frombuffer(struct.pack("<Q", 64), dtype=np.uint8)          # off_hash_a inside the header
    bad[112:120] = 0
    # recompute the checksum the way the format defines it (FNV-1a over the header with a zero checksum, then the payload)
    h = 0xCBF29CE484222325
    for byte in bad.tobytes():
        h = ((h ^ byte) * 0x100000001B3) & 0xFFFFFFFFFFFFFFFF
    bad[112:120] = np.frombuffer(struct.pack("<Q", h), dtype=np.uint8)
    refused(bad, why="offsets")
    # non-finite states are refused like in create()
    states = sk.states.copy(); states[5] = 0x7C00
    sk_inf = oracle.Sketch(sk.in_features, sk.out_features, sk.tile_in, sk.tile_out, sk.d, sk.hash_a, sk.hash_c, sk.group_width, states)
    with pytest.raises(skl.SketchLinearError) as err:
        skl.sketch_linear_file_bytes(desc_of(sk_inf))
    assert err.value.status == skl.SKL_ERR_NONFINITE
    # too small an image for writing
    with pytest.raises(skl.SketchLinearError) as err:
        skl.sketch_linear_file_write(desc, np.zeros(n - 64, dtype=np.uint8))
    assert err.value.status == skl.SKL_ERR_BUFFER_TOO_SMALL
