"""Host-only checks of the decode planner (no GPU call): for the benchmark's layer shapes the split the library
picks is the cheapest one under its own cost model among its candidates (up to the model's 3 % resolution, where
occupied CUs and fewer segments decide), and the plans the measurements in the design notes were taken with are
still the ones picked."""
import dataclasses

import numpy as np
import pytest

import oracle
import paper_2506_17255_amd as skl
import workloads as wk


def description(wl):
    widths = oracle.allocate_widths(wk.gen_importance(wl), wl.budget_states, wl.d).astype(np.uint32)
    A, C = wk.gen_hash_params(wl)
    n = int(widths.sum()) * wl.d
    return skl.make_desc(wl.in_features, wl.out_features, wl.tile_in, wl.tile_out, wl.d, A, C, widths,
                         np.zeros(n, dtype=np.uint16))


SHAPES = {"cfg2_q_proj": wk.cfg2(), "cfg3_up": wk.cfg3("up"), "cfg3_down": wk.cfg3("down"), "cfg4_4096": wk.cfg4(4096, 0.5),
          "cfg4_11008_0.75": wk.cfg4(11008, 0.75), "cfg5_70b": wk.cfg5_70b(),
          # four times the states of cfg3_up (the state count of the paper's 4-bit recipe): wide sketches, narrow blocks
          "cfg3_up_4x_states": dataclasses.replace(wk.cfg3("up"), bpw=2.0)}


def units_per_segment_limit(info):
    """One 64-output unit per wavefront and 16 wavefronts at most; two units per wavefront for layers made of
    one- and two-word blocks only."""
    return 32 if info["block_classes"] & ~3 == 0 else 16


@pytest.mark.parametrize("name", sorted(SHAPES))
def test_the_picked_decode_split_is_the_cheapest_the_kernels_can_run(name):
    wl = SHAPES[name]
    desc = description(wl)
    info, cost = skl.sketch_linear_plan(desc)
    assert info["path"] == 1 and cost > 0
    units = (wl.out_features + 63) // 64
    S0, G0 = info["decode_segments"], info["decode_groups"]
    limit = units_per_segment_limit(info)
    assert (units + S0 - 1) // S0 <= limit
    again, cost_again = skl.sketch_linear_plan(desc, S0, G0)
    assert again == info and cost_again == cost
    # the planner's candidates: for layers of 16 blocks or more the groups come in multiples of 8 (one share per XCD)
    step = 8 if info["n_blocks"] >= 16 else 1
    assert G0 % step == 0
    found = {}
    groups = sorted(set(list(range(step, 65, step)) + [G0, 96, 128, 256]))
    for G in (g for g in groups if g <= info["n_blocks"]):
        for S in range((units + 31) // 32, min(units, 64) + 1):
            try:
                other, c = skl.sketch_linear_plan(desc, S, G)
            except skl.SketchLinearError as e:
                assert e.status == skl.SKL_ERR_UNSUPPORTED
                continue
            assert (units + S - 1) // S <= limit
            assert other["decode_segments"] == S and other["decode_groups"] == G
            found[(S, G)] = c
    assert len(found) > 50
    best = min(found.values())
    # splits priced within 3 % of the cheapest are equals for the model: the pick is the one among them that
    # occupies the most CUs, then the one with the fewest segments
    equals = {k: c for k, c in found.items() if c <= best * 1.03}
    assert (S0, G0) in equals, (S0, G0, cost, best)
    cus = lambda k: min(k[0] * k[1], 256)
    for k in equals:
        assert cus(k) < cus((S0, G0)) or (cus(k) == cus((S0, G0)) and k[0] >= S0), (k, equals[k], (S0, G0), cost)


def test_splits_the_kernels_cannot_run_are_refused():
    desc = description(wk.cfg3("up"))
    # more than 32 units per segment; more than 16 on a layer with eight-word blocks; > 64 blocks per group; > blocks
    for S, G in ((1, 16), (10, 16), (16, 1), (16, 71), (16, 10000)):
        with pytest.raises(skl.SketchLinearError) as err:
            skl.sketch_linear_plan(desc, S, G)
        assert err.value.status == skl.SKL_ERR_UNSUPPORTED
    with pytest.raises(skl.SketchLinearError) as err:
        skl.sketch_linear_plan(desc, 16, 0)
    assert err.value.status == skl.SKL_ERR_INVALID_ARG


def test_benchmark_layers_keep_their_measured_plans():
    """The splits the design notes' timings were taken with."""
    for name, want in (("cfg3_up", (16, 16)), ("cfg3_down", (8, 32)), ("cfg2_q_proj", (8, 32)), ("cfg5_70b", (16, 16)),
                       ("cfg3_up_4x_states", (8, 32))):
        info, _ = skl.sketch_linear_plan(description(SHAPES[name]))
        assert (info["decode_segments"], info["decode_groups"]) == want, name


def test_layers_of_narrow_blocks_take_two_units_per_wavefront():
    desc = description(SHAPES["cfg3_up_4x_states"])
    info, _ = skl.sketch_linear_plan(desc)
    assert info["block_classes"] & ~3 == 0
    units = (11008 + 63) // 64
    assert 16 < (units + info["decode_segments"] - 1) // info["decode_segments"] <= 32
    other, _ = skl.sketch_linear_plan(desc, 6, 38)          # 29 units per segment: 15 wavefronts of two units
    assert (other["decode_segments"], other["decode_groups"]) == (6, 38)
