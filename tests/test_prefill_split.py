"""Host-side checks of the prefill work split (no GPU call is made).

The main prefill kernel multiplies 256 x 256 output tiles, one input-channel
block at a time.  The split hands every workgroup whole tiles plus an equal
share of the blocks of the tiles left over; shares that cover part of a tile
leave float32 partials in numbered slots.  These tests enumerate the split
through the C ABI and check the properties the kernels rely on.
"""
import itertools

import pytest

import paper_2506_17255_amd as skl


KERNELS = [skl.SKL_PREFILL_FUSED, skl.SKL_PREFILL_STAGED]


def split(out_features, n_blocks, tokens, kernel=skl.SKL_PREFILL_FUSED):
    segs, shape = skl.sketch_linear_prefill_split(out_features, n_blocks, tokens, kernel)
    return segs, shape


def m_tiles_of(tokens, mt=256):
    return (tokens + mt - 1) // mt


def tiles_of_xcd(mu, xcd, n_tiles, m_tiles):
    """Tiles dealt to an XCD: units of mu token tiles of one output-tile column go round the XCDs
    (mu = 1: single tiles, the fused kernel; the staged kernel takes the largest mu that stays balanced)."""
    n_units = (n_tiles // m_tiles) * (m_tiles // mu)
    return mu * ((n_units - xcd + 7) // 8) if n_units > xcd else 0


def unit_of_tile(mu, tm, tn, m_tiles):
    return tn * (m_tiles // mu) + tm // mu


def xcd_of_tile(mu, tm, tn, m_tiles):
    return unit_of_tile(mu, tm, tn, m_tiles) % 8


def index_on_xcd(mu, tm, tn, m_tiles):
    """Position of a tile in its XCD's list."""
    return (unit_of_tile(mu, tm, tn, m_tiles) // 8) * mu + tm % mu


SHAPES = [
    (11008, 64, 2048),    # the benchmark layer: 344 tiles on 256 workgroups
    (4096, 64, 2048),     # fewer tiles than workgroups (staged kernel: one half-height tile per workgroup)
    (4096, 64, 1900),     # the same with a ragged last token tile
    (3840, 64, 2048),     # 240 half-height tiles
    (3584, 64, 2048),     # 224 half-height tiles: full-height tiles again
    (4096, 172, 2048),    # the down projection's block count
    (28672, 128, 2048),   # 896 tiles: three whole rounds and a leftover
    (256, 1, 1),          # a single tile of a single block
    (300, 3, 257),        # ragged in both directions, tiny
    (11008, 64, 1),       # decode-sized call through the prefill path
    (5000, 7, 1000),
    (65536, 5, 4096),
    (256 * 33, 64, 2048), # one tile more than a whole round on one XCD
]


@pytest.mark.parametrize("kernel", KERNELS)
@pytest.mark.parametrize("out_features,n_blocks,tokens", SHAPES)
def test_every_block_of_every_tile_is_multiplied_once(out_features, n_blocks, tokens, kernel):
    segs, (gx, l_max, p_cap, n_tiles, mu, mt) = split(out_features, n_blocks, tokens, kernel)
    assert mt in (128, 256) and (mt == 256 or kernel == skl.SKL_PREFILL_STAGED)
    m_tiles = m_tiles_of(tokens, mt)
    n_col = (out_features + 255) // 256
    assert n_tiles == m_tiles * n_col
    seen = {}
    for xcd, wg, tm, tn, k0, k1, whole, slot in segs:
        assert xcd < 8 and wg < gx
        assert tm < m_tiles and tn < n_col
        assert 0 <= k0 < k1 <= n_blocks
        # tiles dealt out in whole rounds are stored by the main kernel; every share of a leftover tile
        # leaves a partial for the fix-up pass, also a share that happens to cover the tile
        tiles_of = tiles_of_xcd(mu, xcd, n_tiles, m_tiles)
        in_round = index_on_xcd(mu, tm, tn, m_tiles) < (tiles_of // gx) * gx
        if mt == 128:                   # half-height tiles: one whole tile per workgroup, nothing left over
            assert tiles_of <= gx == 32 and l_max == 0
            in_round = True
        assert whole == int(in_round)
        if in_round:
            assert k0 == 0 and k1 == n_blocks
        assert xcd_of_tile(mu, tm, tn, m_tiles) == xcd          # a tile stays on one XCD
        for b in range(k0, k1):
            assert (tm, tn, b) not in seen
            seen[(tm, tn, b)] = (xcd, wg)
    assert len(seen) == n_tiles * n_blocks


@pytest.mark.parametrize("kernel", KERNELS)
@pytest.mark.parametrize("out_features,n_blocks,tokens", SHAPES)
def test_partial_slots_are_distinct_dense_and_in_workgroup_order(out_features, n_blocks, tokens, kernel):
    segs, (gx, l_max, p_cap, n_tiles, mu, mt) = split(out_features, n_blocks, tokens, kernel)
    by_tile = {}
    slots = set()
    for xcd, wg, tm, tn, k0, k1, whole, slot in segs:
        if whole:
            continue
        assert slot < 8 * l_max * p_cap                 # inside the workspace the library asks for
        assert slot not in slots
        slots.add(slot)
        by_tile.setdefault((tm, tn), []).append((slot, wg, k0, k1))
    for parts in by_tile.values():
        parts.sort()
        base = parts[0][0]
        assert base % p_cap == 0                        # a tile's slots start at its own row of the slot table
        assert [s for s, *_ in parts] == list(range(base, base + len(parts)))
        assert len(parts) <= p_cap
        wgs = [w for _, w, *_ in parts]
        assert wgs == sorted(wgs) and len(set(wgs)) == len(wgs)
        # consecutive block ranges covering the whole tile
        assert parts[0][2] == 0 and parts[-1][3] == n_blocks
        for (_, _, _, e), (_, _, b, _) in zip(parts, parts[1:]):
            assert e == b


@pytest.mark.parametrize("kernel", KERNELS)
@pytest.mark.parametrize("out_features,n_blocks,tokens", SHAPES)
def test_workgroups_get_equal_work(out_features, n_blocks, tokens, kernel):
    segs, (gx, l_max, p_cap, n_tiles, mu, mt) = split(out_features, n_blocks, tokens, kernel)
    load = {}
    for xcd, wg, tm, tn, k0, k1, whole, slot in segs:
        load[(xcd, wg)] = load.get((xcd, wg), 0) + k1 - k0
    for xcd in range(8):
        mine = [v for (x, _), v in load.items() if x == xcd]
        if mine:
            # within an XCD: whole rounds are equal, leftover shares differ by at most one block;
            # workgroups without a share (fewer leftover blocks than workgroups) do one block less at most
            assert max(mine) - min(mine) <= 1 or len(mine) < gx
    total = sum(load.values())
    assert total == n_tiles * n_blocks
    if kernel == skl.SKL_PREFILL_FUSED:
        assert mu == 1
    assert m_tiles_of(tokens, mt) % mu == 0
    # the busiest workgroup is close to the ideal share when there is enough work to go round (the staged
    # kernel's dealing units are chosen so that the busiest XCD stays within 3 % of dealing single tiles)
    if mt == 128:
        assert max(load.values()) == n_blocks               # one whole tile each
    elif total >= 8 * gx * 8:
        assert max(load.values()) <= total / (8 * gx) + n_blocks / 8 + 1


@pytest.mark.parametrize("kernel", KERNELS)
def test_small_exhaustive_sweep(kernel):
    for n_tiles_out, n_blocks, tokens in itertools.product(range(1, 41), (1, 2, 5, 31, 64), (1, 256, 257, 2048)):
        out_features = 256 * n_tiles_out - 3
        segs, (gx, l_max, p_cap, n_tiles, mu, mt) = split(out_features, n_blocks, tokens, kernel)
        covered = sum(k1 - k0 for *_, k0, k1, _, _ in segs)
        assert covered == n_tiles * n_blocks
        keys = set()
        for xcd, wg, tm, tn, k0, k1, whole, slot in segs:
            for b in range(k0, k1):
                keys.add((tm, tn, b))
        assert len(keys) == covered


def leftover_tiles(shape, tokens, kernel):
    """(xcd, l, token tile, output tile) of every tile the fix-up pass finishes."""
    gx, l_max, p_cap, n_tiles, mu, mt = shape
    if mt == 128:                       # one whole half-height tile per workgroup: nothing for the fix-up pass
        assert l_max == 0
        return
    m_tiles = (tokens + 255) // 256
    n_mg = m_tiles // mu
    for xcd in range(8):
        tiles_of = tiles_of_xcd(mu, xcd, n_tiles, m_tiles)
        rounds = tiles_of // gx
        for l in range(tiles_of - rounds * gx):
            k = rounds * gx + l
            u = xcd + 8 * (k // mu)
            yield xcd, l, (u % n_mg) * mu + k % mu, u // n_mg


def check_fixup_reads_only_written_slots(out_features, n_blocks, tokens, kernel=skl.SKL_PREFILL_FUSED):
    """The fix-up pass adds slots [base, base + parts) of every leftover tile: each must have been written
    by a partial segment of that tile, and whole-tile segments never belong to a leftover tile."""
    segs, shape = split(out_features, n_blocks, tokens, kernel)
    gx, l_max, p_cap, n_tiles, mu, mt = shape
    written = {}
    for xcd, wg, tm, tn, k0, k1, whole, slot in segs:
        if not whole:
            written.setdefault((tm, tn), []).append(slot)
    left = list(leftover_tiles(shape, tokens, kernel))
    assert len(left) == len(written)
    for xcd, l, tm, tn in left:
        assert l < l_max
        slots = sorted(written[(tm, tn)])
        base = (xcd * l_max + l) * p_cap
        assert slots == list(range(base, base + len(slots))), (out_features, n_blocks, tokens, xcd, l)
    for xcd, wg, tm, tn, k0, k1, whole, slot in segs:
        if whole:
            assert (tm, tn) not in written


@pytest.mark.parametrize("kernel", KERNELS)
@pytest.mark.parametrize("out_features,n_blocks,tokens", SHAPES + [(7936, 16, 2048), (256 * 57, 1, 256), (4864, 1, 768)])
def test_fixup_reads_only_written_slots(out_features, n_blocks, tokens, kernel):
    check_fixup_reads_only_written_slots(out_features, n_blocks, tokens, kernel)


@pytest.mark.parametrize("kernel", KERNELS)
def test_fixup_slots_with_few_blocks(kernel):
    """Layers with fewer channel blocks than workgroups per XCD: a leftover share can cover exactly one tile."""
    for n_blocks in range(1, 33):
        for n_tiles_out in (1, 2, 7, 19, 31, 57, 64):
            for tokens in (256, 768, 2048):
                check_fixup_reads_only_written_slots(256 * n_tiles_out, n_blocks, tokens, kernel)


def test_half_height_tiles_are_used_where_they_fill_the_chip_once():
    S = skl.SKL_PREFILL_STAGED
    for out_features, tokens, want in [(4096, 2048, 128), (4096, 1900, 128), (3840, 2048, 128), (3584, 2048, 256),
                                        (4352, 2048, 256), (11008, 2048, 256), (8192, 1024, 128), (8192, 1000, 128),
                                        (16384, 512, 128), (4096, 4096, 256), (4096, 1024, 256)]:
        segs, (gx, l_max, p_cap, n_tiles, mu, mt) = split(out_features, 64, tokens, S)
        assert mt == want, (out_features, tokens)
        if mt == 128:
            assert gx == 32 and l_max == 0 and p_cap == 0
            assert len(segs) == n_tiles and all(s[6] == 1 for s in segs)
            assert len({(s[0], s[1]) for s in segs}) == n_tiles     # one tile per workgroup
    segs, shape = split(4096, 64, 2048, skl.SKL_PREFILL_FUSED)
    assert shape[5] == 256


def test_argument_errors():
    L = skl.load_library()
    import ctypes
    n = ctypes.c_uint64(0)
    F = skl.SKL_PREFILL_FUSED
    assert L.sketch_linear_prefill_split(F, 4096, 64, 2048, None, 0, None, None) == skl.SKL_ERR_INVALID_ARG
    assert L.sketch_linear_prefill_split(F, 4096, 64, 2048, None, 5, ctypes.byref(n), None) == skl.SKL_ERR_INVALID_ARG
    assert L.sketch_linear_prefill_split(F, 0, 64, 2048, None, 0, ctypes.byref(n), None) == skl.SKL_ERR_INVALID_ARG
    assert L.sketch_linear_prefill_split(F, 4096, 64, 0, None, 0, ctypes.byref(n), None) == skl.SKL_ERR_INVALID_ARG
    assert L.sketch_linear_prefill_split(1, 4096, 64, 2048, None, 0, ctypes.byref(n), None) == skl.SKL_ERR_INVALID_ARG
    assert L.sketch_linear_prefill_split(F, 4096, 64, 2048, None, 0, ctypes.byref(n), None) == skl.SKL_OK
    assert n.value >= 8
