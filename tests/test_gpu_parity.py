"""GPU parity: every entry point of the C ABI against the CPU oracle.

Bars (also stated per test):
  * reconstructed weights: bit-exact (integer compare of binary16 patterns);
  * gemv / gemm outputs: relative Frobenius error <= 1e-3 against the fp64
    oracle (float32 and binary16 outputs), and against the oracle rounded to
    bfloat16 for bfloat16 outputs (the rounding alone is ~1.7e-3);
  * one-hot activations: the float32 output must equal the reconstructed
    weight exactly -- this checks the fused kernels' own query stage.
"""
import functools

import numpy as np
import pytest

import oracle
import paper_2506_17255_amd as skl
import workloads as wk
from skl_harness import GpuLayer, build_sketch, rel_fro, round_to_bf16

pytestmark = pytest.mark.gpu

TOL = 1e-3


# ------------------------------------------------------------------ layers
def custom_layer(name, in_f, out_f, tj, to, d, widths, seed):
    rng = np.random.default_rng(seed)
    W = (rng.standard_normal((in_f, out_f)) * 0.02).astype(np.float16)
    A = (2 * rng.integers(0, 1 << 23, size=d) + 1).astype(np.uint32)
    C = rng.integers(0, 1 << 24, size=d).astype(np.uint32)
    return W, oracle.update(W, tj, to, d, A, C, np.asarray(widths, dtype=np.uint32))


@functools.lru_cache(maxsize=None)
def small_case(name):
    rng = np.random.default_rng(abs(hash(name)) % (1 << 31))
    if name == "cfg1":                       # one 256x256 group, d=2, K=1024: per-weight hashing
        return build_sketch(wk.cfg1())
    if name == "row_ragged":                 # row sketches; in % 8 != 0, out % 32 != 0
        return custom_layer(name, 100, 300, 1, 300, 4, [11] * 100, 1)
    if name == "row_classes":                # four width classes -> all four table layouts in one layer
        widths = np.array([11] * 150 + [120] * 20 + [220] * 13 + [350] * 9)
        np.random.default_rng(2).shuffle(widths)
        return custom_layer(name, 192, 520, 1, 520, 4, widths, 2)
    if name == "row_d1":
        return custom_layer(name, 64, 256, 1, 256, 1, [16] * 64, 3)
    if name == "row_d2_importance":
        widths = np.where(np.arange(72) % 9 == 0, 48, 12)
        return custom_layer(name, 72, 1000, 1, 1000, 2, widths, 4)
    if name == "row_d5":
        return custom_layer(name, 40, 384, 1, 384, 5, [20] * 40, 5)
    if name == "row_d8":
        return custom_layer(name, 24, 130, 1, 130, 8, [9] * 24, 6)
    if name == "row_big_table":              # one-word rows, table above 64 KiB of LDS
        return custom_layer(name, 16, 2048, 1, 2048, 4, [1100] * 16, 7)
    if name == "row_single":                 # degenerate: one input channel, one output
        return custom_layer(name, 1, 1, 1, 1, 3, [1], 8)
    if name == "row_four_words":             # mostly blocks of four words per state row, three widths among them,
        widths = np.array([11] * 40 + [120] * 70 + [129] * 50 + [150] * 40)   # ragged last block of each width
        np.random.default_rng(13).shuffle(widths)
        return custom_layer(name, 200, 300, 1, 300, 4, widths, 13)
    if name == "row_four_words_d6":          # the same with six sketch rows (four words from width 76 on)
        widths = np.array([20] * 30 + [80] * 45 + [100] * 60 + [150] * 9)
        np.random.default_rng(14).shuffle(widths)
        return custom_layer(name, 144, 520, 1, 520, 6, widths, 14)
    if name == "tile_ragged":                # 2-D groups, per-group widths, tile_out < workgroup
        return custom_layer(name, 96, 160, 32, 80, 3, rng.integers(5, 60, size=6), 9)
    if name == "tile_wide":                  # tile_out above one workgroup of lanes, tile_in % 16 != 0
        return custom_layer(name, 12, 600, 6, 300, 2, [37, 41, 43, 47], 10)
    if name == "tile_d8_K1":                 # width 1: every weight of a group shares one state per row
        return custom_layer(name, 16, 64, 8, 32, 8, [1, 2, 1, 3], 11)
    if name == "tile_forced_1d":             # row geometry pushed through the per-weight path
        return custom_layer(name, 40, 200, 1, 200, 3, [13] * 40, 12)
    raise KeyError(name)


SMALL = ["cfg1", "row_ragged", "row_classes", "row_d1", "row_d2_importance", "row_d5", "row_d8",
         "row_big_table", "row_single", "tile_ragged", "tile_wide", "tile_d8_K1", "tile_forced_1d"]


def flags_of(name):
    return 1 if name == "tile_forced_1d" else 0


def prefill_cases(names):
    """(name, flags) pairs: every layer with the kernel its plan picks, row-sketch layers also with the
    staged prefill asked for (weights rebuilt once per call into the workspace)."""
    out = []
    for n in names:
        out.append((n, flags_of(n)))
        if n.startswith("row"):
            out.append((n, skl.FLAG_STAGED_PREFILL))
            out.append((n, skl.FLAG_FUSED_PREFILL))
    return out


def expect_prefill_kernel(g, name, flags):
    if not name.startswith("row"):
        want = skl.SKL_PREFILL_PER_WEIGHT
    elif flags & skl.FLAG_STAGED_PREFILL or name == "row_big_table":     # a table above the fused kernel's LDS plan
        want = skl.SKL_PREFILL_STAGED
    else:
        want = skl.SKL_PREFILL_FUSED
    assert g.info["prefill_kernel"] == want
    if name.startswith("row"):
        from_tokens = 0 if want == skl.SKL_PREFILL_STAGED else 0xFFFFFFFF if flags & skl.FLAG_FUSED_PREFILL else 513
        assert g.info["prefill_staged_from"] == from_tokens


@functools.lru_cache(maxsize=None)
def expected_W_hat(name):
    return oracle.query(small_case(name)[1])


# ----------------------------------------------------------- reconstruct
@pytest.mark.parametrize("name", SMALL)
def test_reconstruct_bit_exact(name):
    W, sk = small_case(name)
    with GpuLayer(sk, flags_of(name)) as g:
        assert g.info["path"] == (1 if name.startswith("row") else 0)
        got = g.reconstruct()
    assert np.array_equal(got, expected_W_hat(name))


@pytest.mark.parametrize("name", SMALL)
def test_hash_operator_comparator_bit_exact(name):
    """The per-weight hash operator (states fetched from device memory, nothing staged) gives the same W_hat."""
    W, sk = small_case(name)
    with GpuLayer(sk, flags_of(name)) as g:
        got = g.reconstruct(hash_op=True)
    assert np.array_equal(got, expected_W_hat(name))


# ------------------------------------------------------------------ gemv
@pytest.mark.parametrize("batch", [1, 2, 5, 8, 16])
@pytest.mark.parametrize("name", SMALL)
def test_gemv_matches_oracle(name, batch):
    W, sk = small_case(name)
    W_hat = expected_W_hat(name)
    rng = np.random.default_rng(100 + batch)
    x = rng.standard_normal((batch, sk.in_features)).astype(np.float16)
    ref = oracle.linear(W_hat, x)
    with GpuLayer(sk, flags_of(name)) as g:
        y32 = g.gemv(x, "f32", ldx=sk.in_features + 8, ldy=sk.out_features + 24)
        y16 = g.gemv(x, "f16")
        again = g.gemv(x, "f32")
    assert rel_fro(y32, ref) <= TOL, rel_fro(y32, ref)
    assert rel_fro(y16, ref) <= TOL, rel_fro(y16, ref)
    assert rel_fro(y32, ref) <= 1e-5          # float32 accumulation: far inside the bar
    assert np.array_equal(y32, again), "summation order must not change from run to run"


@pytest.mark.parametrize("batch", [1, 5])
@pytest.mark.parametrize("name", SMALL)
def test_gemv_partials_sum_to_the_output(name, batch):
    """The diagnostic first stage alone: its per-unit partial sums add up to y."""
    W, sk = small_case(name)
    W_hat = expected_W_hat(name)
    rng = np.random.default_rng(300 + batch)
    x = rng.standard_normal((batch, sk.in_features)).astype(np.float16)
    ref = oracle.linear(W_hat, x)
    with GpuLayer(sk, flags_of(name)) as g:
        parts = g.gemv_partials(x)
    y = parts.astype(np.float64).sum(axis=0)
    assert rel_fro(y, ref) <= 1e-5, rel_fro(y, ref)


@pytest.mark.parametrize("batch", [1, 16])
@pytest.mark.parametrize("name", SMALL)
def test_gemv_one_hot_probe_is_exact(name, batch):
    """x = e_j  =>  y = W_hat[j][:] exactly: one exact product, all other terms zero."""
    W, sk = small_case(name)
    W_hat = expected_W_hat(name).view(np.float16).astype(np.float32)
    rng = np.random.default_rng(7)
    js = rng.choice(sk.in_features, size=min(batch, sk.in_features), replace=False)
    x = np.zeros((batch, sk.in_features), dtype=np.float16)
    for b, j in enumerate(js):
        x[b, j] = 1.0
    with GpuLayer(sk, flags_of(name)) as g:
        y = g.gemv(x, "f32")
    for b, j in enumerate(js):
        assert np.array_equal(y[b], W_hat[j]), (name, b, j)
    assert np.all(y[len(js):] == 0)


# ------------------------------------------------------------------ gemm
@pytest.mark.parametrize("tokens", [1, 70, 200])
@pytest.mark.parametrize("name,flags", prefill_cases(SMALL))
def test_gemm_matches_oracle(name, flags, tokens):
    W, sk = small_case(name)
    W_hat = expected_W_hat(name)
    rng = np.random.default_rng(200 + tokens)
    Xf = rng.standard_normal((tokens, sk.in_features)).astype(np.float32)
    Xb = wk.f32_to_bf16_bits(Xf)
    ref = oracle.linear(W_hat, Xb, x_kind="bf16")
    with GpuLayer(sk, flags) as g:
        expect_prefill_kernel(g, name, flags)
        y32 = g.gemm(Xb, "bf16", "f32", ldx=sk.in_features + 8, ldy=sk.out_features + 8)
        ybf = g.gemm(Xb, "bf16", "bf16")
        y16 = g.gemm(Xb, "bf16", "f16")
        Xh = Xf.astype(np.float16)
        yh = g.gemm(Xh.view(np.uint16), "f16", "f32")
    assert rel_fro(y32, ref) <= 1e-5, rel_fro(y32, ref)
    assert rel_fro(y16, ref) <= TOL
    assert rel_fro(ybf, round_to_bf16(ref)) <= TOL, rel_fro(ybf, round_to_bf16(ref))
    assert rel_fro(yh, oracle.linear(W_hat, Xh)) <= 1e-5


@pytest.mark.parametrize("name,flags", prefill_cases(["row_ragged", "row_classes", "row_d5", "row_big_table", "row_single"]))
def test_gemm_strides_and_several_token_tiles(name, flags):
    """Three token tiles with a ragged last one (the work split then shares tiles between workgroups),
    rows of X that are not 16-byte aligned, rows of Y that are and that are not."""
    W, sk = small_case(name)
    W_hat = expected_W_hat(name)
    tokens = 600
    rng = np.random.default_rng(77)
    Xf = rng.standard_normal((tokens, sk.in_features)).astype(np.float32)
    Xb = wk.f32_to_bf16_bits(Xf)
    ref = oracle.linear(W_hat, Xb, x_kind="bf16")
    pad = (-sk.out_features) % 8
    with GpuLayer(sk, flags) as g:
        expect_prefill_kernel(g, name, flags)
        y_odd = g.gemm(Xb, "bf16", "bf16", ldx=sk.in_features + 3, ldy=sk.out_features + pad + 5)
        y_al = g.gemm(Xb, "bf16", "bf16", ldx=sk.in_features + 8, ldy=sk.out_features + pad + 16)
        y16 = g.gemm(Xb, "bf16", "f16", ldy=sk.out_features + pad + 8)
        y32 = g.gemm(Xb, "bf16", "f32", ldx=sk.in_features + 1, ldy=sk.out_features + pad + 4)
        y32_odd = g.gemm(Xb, "bf16", "f32", ldy=sk.out_features + pad + 3)
    assert rel_fro(y32, ref) <= 1e-5
    assert np.array_equal(y32, y32_odd)                 # the two store paths round the same sums
    assert np.array_equal(y_odd, y_al)
    assert rel_fro(y_al, round_to_bf16(ref)) <= TOL
    assert rel_fro(y16, ref) <= TOL


@pytest.mark.parametrize("tokens", [1, 300, 700])
@pytest.mark.parametrize("name,flags", prefill_cases(["row_four_words", "row_four_words_d6"]))
def test_gemm_blocks_of_four_words(name, flags, tokens):
    """Layers whose blocks hold 32 channels (four words per state row): the prefill kernel rebuilds their
    operand words between the MFMAs of the block before, with its own lane layout."""
    W, sk = small_case(name)
    W_hat = oracle.query(sk)
    rng = np.random.default_rng(900 + tokens)
    Xb = wk.f32_to_bf16_bits(rng.standard_normal((tokens, sk.in_features)).astype(np.float32))
    ref = oracle.linear(W_hat, Xb, x_kind="bf16")
    with GpuLayer(sk, flags) as g:
        expect_prefill_kernel(g, name, flags)
        assert np.array_equal(g.reconstruct(), W_hat)
        y32 = g.gemm(Xb, "bf16", "f32")
        ybf = g.gemm(Xb, "bf16", "bf16", ldx=sk.in_features + 8, ldy=sk.out_features + 8)
        x1 = rng.standard_normal((1, sk.in_features)).astype(np.float16)
        y1 = g.gemv(x1, "f32")
    assert rel_fro(y32, ref) <= 1e-5, rel_fro(y32, ref)
    assert rel_fro(ybf, round_to_bf16(ref)) <= TOL
    assert rel_fro(y1, oracle.linear(W_hat, x1)) <= 1e-5


@pytest.mark.parametrize("flags", [0, skl.FLAG_STAGED_PREFILL, skl.FLAG_FUSED_PREFILL])
def test_gemm_is_bit_identical_from_run_to_run(flags):
    W, sk = small_case("row_classes")
    rng = np.random.default_rng(78)
    Xb = wk.f32_to_bf16_bits(rng.standard_normal((700, sk.in_features)).astype(np.float32))
    with GpuLayer(sk, flags) as g:
        runs = [g.gemm(Xb, "bf16", "f32") for _ in range(3)]
    assert np.array_equal(runs[0], runs[1]) and np.array_equal(runs[0], runs[2])


@pytest.mark.parametrize("name,flags", prefill_cases(["row_ragged", "row_classes", "tile_ragged", "cfg1"]))
def test_gemm_identity_probe_is_exact(name, flags):
    """X = I  =>  Y = W_hat exactly (float32 output)."""
    W, sk = small_case(name)
    W_hat = expected_W_hat(name).view(np.float16).astype(np.float32)
    X = np.eye(sk.in_features, dtype=np.float32)
    with GpuLayer(sk, flags) as g:
        y = g.gemm(wk.f32_to_bf16_bits(X), "bf16", "f32")
    assert np.array_equal(y, W_hat)


@pytest.mark.parametrize("flags", [skl.FLAG_FUSED_PREFILL, skl.FLAG_STAGED_PREFILL])
def test_gemm_with_fewer_blocks_than_workgroups_and_a_dirty_workspace(flags):
    """64 input channels (one channel block), 4864 outputs, 768 tokens: 57 tiles, so some XCDs finish a
    leftover tile with a single share that covers it whole.  The workspace starts full of NaN patterns:
    whatever the fix-up pass adds must have been written by this call."""
    W, sk = custom_layer("few_blocks", 64, 4864, 1, 4864, 4, [40] * 64, 21)
    W_hat = oracle.query(sk)
    rng = np.random.default_rng(79)
    Xb = wk.f32_to_bf16_bits(rng.standard_normal((768, 64)).astype(np.float32))
    ref = oracle.linear(W_hat, Xb, x_kind="bf16")
    with GpuLayer(sk, flags) as g:
        ws, need = g.workspace(1, 768)
        ws.fill_(0xFF)
        y32 = g.gemm(Xb, "bf16", "f32")
        ws.fill_(0xFF)
        ybf = g.gemm(Xb, "bf16", "bf16")
    assert rel_fro(y32, ref) <= 1e-5
    assert rel_fro(ybf, round_to_bf16(ref)) <= TOL


def test_gemm_with_one_half_height_tile_per_workgroup():
    """Calls whose 128-token tiles number between 225 and 256 (here 58 token tiles x 4 output-tile columns,
    both ragged; 160 channels are three channel blocks, the last one partly filled) take the staged
    kernel's single-round mode: one whole tile per workgroup, no partials, no fix-up pass.  The workspace
    starts full of NaN patterns."""
    widths = np.array([30] * 120 + [140] * 40)
    np.random.default_rng(5).shuffle(widths)
    W, sk = custom_layer("half_tiles", 160, 1000, 1, 1000, 4, widths, 23)
    W_hat = oracle.query(sk)
    tokens = 128 * 58 - 37
    segs, shape = skl.sketch_linear_prefill_split(1000, 3, tokens, skl.SKL_PREFILL_STAGED)
    assert shape[5] == 128 and shape[3] == 232
    rng = np.random.default_rng(81)
    Xb = wk.f32_to_bf16_bits(rng.standard_normal((tokens, 160)).astype(np.float32))
    ref = oracle.linear(W_hat, Xb, x_kind="bf16")
    with GpuLayer(sk, skl.FLAG_STAGED_PREFILL) as g:
        ws, need = g.workspace(1, tokens)
        ws.fill_(0xFF)
        y32 = g.gemm(Xb, "bf16", "f32")
        ws.fill_(0xFF)
        y32_odd = g.gemm(Xb, "bf16", "f32", ldx=163, ldy=1003)
        ybf = g.gemm(Xb, "bf16", "bf16")
        ybf_odd = g.gemm(Xb, "bf16", "bf16", ldy=1005)
        y16 = g.gemm(Xb, "bf16", "f16", ldy=1008)
        again = g.gemm(Xb, "bf16", "f32")
    with GpuLayer(sk, skl.FLAG_FUSED_PREFILL) as g:
        y_fused = g.gemm(Xb, "bf16", "f32")
    assert rel_fro(y32, ref) <= 1e-5, rel_fro(y32, ref)
    assert np.array_equal(y32, y32_odd) and np.array_equal(y32, again)
    assert np.array_equal(ybf, ybf_odd)
    assert rel_fro(ybf, round_to_bf16(ref)) <= TOL
    assert rel_fro(y16, ref) <= TOL
    assert rel_fro(y_fused, ref) <= 1e-5


def test_gemm_row_equals_gemv():
    W, sk = small_case("row_classes")
    rng = np.random.default_rng(5)
    X = rng.standard_normal((3, sk.in_features)).astype(np.float16)
    with GpuLayer(sk) as g:
        Y = g.gemm(X.view(np.uint16), "f16", "f32")
        y = g.gemv(X, "f32")
    assert rel_fro(Y, y) <= 1e-5


# ------------------------------------------- query mode 1: Eq. (5) as printed
SIGNED = ["cfg1", "row_ragged", "row_classes", "row_d1", "row_d5", "row_d8", "row_big_table", "row_four_words",
          "tile_ragged", "tile_d8_K1", "tile_forced_1d"]


@pytest.mark.parametrize("name", SIGNED)
def test_signed_max_query_mode(name):
    """Max of the signed values instead of Max by magnitude: another order-key encoding and decode, the same
    kernels.  Reconstruction (staged kernel and hash-operator comparator) bit-exact, one-hot probes of the fused decode
    exact, decode at batch 1 and 8 and both prefill kernels against the oracle in the same mode."""
    W, sk = small_case(name)
    W_hat = oracle.query(sk, oracle.QUERY_SIGNED_MAX)
    assert not np.array_equal(W_hat, oracle.query(sk)) or sk.d == 1          # the two readings differ on this layer
    rng = np.random.default_rng(400)
    x = rng.standard_normal((8, sk.in_features)).astype(np.float16)
    Xb = wk.f32_to_bf16_bits(rng.standard_normal((300, sk.in_features)).astype(np.float32))
    ref = oracle.linear(W_hat, x)
    ref_X = oracle.linear(W_hat, Xb, x_kind="bf16")
    j = rng.choice(sk.in_features, size=min(16, sk.in_features), replace=False)
    probe = np.zeros((j.size, sk.in_features), dtype=np.float16)
    probe[np.arange(j.size), j] = 1.0
    for flags in ([flags_of(name)] if not name.startswith("row") else [skl.FLAG_FUSED_PREFILL, skl.FLAG_STAGED_PREFILL]):
        with GpuLayer(sk, flags, query_mode=1) as g:
            assert np.array_equal(g.reconstruct(), W_hat)
            assert np.array_equal(g.reconstruct(hash_op=True), W_hat)
            assert rel_fro(g.gemv(x[:1], "f32"), ref[:1]) <= 1e-5
            assert rel_fro(g.gemv(x, "f32"), ref) <= 1e-5
            assert np.array_equal(g.gemv(probe, "f32"), W_hat.view(np.float16).astype(np.float32)[j])
            assert np.array_equal(g.gemv(probe[:1], "f32"), W_hat.view(np.float16).astype(np.float32)[j[:1]])
            assert rel_fro(g.gemm(Xb, "bf16", "f32"), ref_X) <= 1e-5


@pytest.mark.parametrize("bits", [8, 4])
def test_signed_max_query_mode_with_low_bit_states(bits):
    W, sk = small_case("row_classes")
    q = oracle.quantize(sk, bits)
    W_hat = oracle.query(q, oracle.QUERY_SIGNED_MAX)
    x = np.random.default_rng(401).standard_normal((3, sk.in_features)).astype(np.float16)
    with GpuLayer(q, query_mode=1) as g:
        assert np.array_equal(g.reconstruct(), W_hat)
        assert rel_fro(g.gemv(x, "f32"), oracle.linear(W_hat, x)) <= 1e-5


# ------------------------------------------------------- low-bit states
LOWBIT = ["cfg1", "row_ragged", "row_classes", "row_d1", "row_d5", "row_d8", "row_big_table", "row_single",
          "tile_ragged", "tile_d8_K1", "tile_forced_1d"]


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("name", LOWBIT)
def test_low_bit_states_match_oracle(name, bits):
    """States kept as 8-/4-bit codes with one scale per sketch row (Sec. 3.3, last paragraph): the
    library expands them on the device per call; reconstructed weights are bit-exact against the
    oracle's query over the states the codes stand for, outputs within the floating-point bar."""
    W, sk = small_case(name)
    q = oracle.quantize(sk, bits)
    W_hat = oracle.query(q)
    rng = np.random.default_rng(300 + bits)
    x = rng.standard_normal((5, sk.in_features)).astype(np.float16)
    Xf = rng.standard_normal((300, sk.in_features)).astype(np.float32)
    Xb = wk.f32_to_bf16_bits(Xf)
    with GpuLayer(q, flags_of(name)) as g:
        got = g.reconstruct()
        assert np.array_equal(got, W_hat), (name, bits, int(np.sum(got != W_hat)))
        y1 = g.gemv(x[:1], "f32")
        y5 = g.gemv(x, "f32", ldx=sk.in_features + 8, ldy=sk.out_features + 24)
        y16 = g.gemv(x, "f16")
        Y = g.gemm(Xb, "bf16", "f32")
        Ybf = g.gemm(Xb[:70], "bf16", "bf16")
        full = GpuLayer(oracle.Sketch(q.in_features, q.out_features, q.tile_in, q.tile_out, q.d, q.hash_a, q.hash_c,
                                      q.group_width, q.states), flags_of(name))
        with full as f:
            # the same states given as binary16: the kernels see identical tables, so identical results
            assert np.array_equal(f.gemv(x, "f32"), g.gemv(x, "f32"))
            assert np.array_equal(f.gemm(Xb, "bf16", "f32"), Y)
            assert g.info["table_bytes"] < f.info["table_bytes"] or sk.states.size < 64
    ref = oracle.linear(W_hat, x)
    assert rel_fro(y1, ref[:1]) <= 1e-5
    assert rel_fro(y5, ref) <= 1e-5
    assert rel_fro(y16, ref) <= TOL
    refX = oracle.linear(W_hat, Xb, x_kind="bf16")
    assert rel_fro(Y, refX) <= 1e-5
    assert rel_fro(Ybf, round_to_bf16(refX[:70])) <= TOL


@pytest.mark.parametrize("bits", [8, 4])
def test_low_bit_dequantisation_over_every_scale_and_code(bits):
    """Every finite positive binary16 scale (31744 of them, one input channel each) with every code in its
    sketch row: the states the library expands on the device are those of the oracle, bit for bit.  (The
    device multiplies by the reciprocal of qmax instead of dividing; this is the exhaustive check of that.)"""
    qmax = 127 if bits == 8 else 7
    K = 2 * qmax + 1
    in_f, out_f, d = 31744, 2048, 1
    scales = np.arange(in_f, dtype=np.uint16)                       # patterns 0x0000 .. 0x7BFF
    codes = np.tile(np.arange(-qmax, qmax + 1, dtype=np.int8), in_f)
    widths = np.full(in_f, K, dtype=np.uint32)
    states = oracle.dequantize_states(in_f, out_f, 1, out_f, d, widths, bits, codes, scales)
    q = oracle.QuantSketch(in_f, out_f, 1, out_f, d, np.uint32([0x9E3779]), np.uint32([0x12345]), widths, states,
                           bits=bits, codes=codes, scales=scales)
    W_hat = oracle.query(q)
    assert len(np.unique(W_hat[-1])) == K                           # every state of a row is reached by some output
    with GpuLayer(q) as g:
        assert np.array_equal(g.reconstruct(), W_hat)


def test_low_bit_workspace_holds_the_expanded_tables():
    import paper_2506_17255_amd as skl
    W, sk = small_case("row_classes")
    q = oracle.quantize(sk, 4)
    with GpuLayer(q) as g, GpuLayer(sk) as f:
        for op, n in ((0, 1), (0, 16), (1, 300), (2, 0)):
            need_q = skl.sketch_linear_workspace_bytes(g.handle, op, n)
            need_f = skl.sketch_linear_workspace_bytes(f.handle, op, n)
            assert need_q >= need_f + 2 * sk.states.size        # room for the 16-bit tables
        assert skl.sketch_linear_workspace_bytes(f.handle, 2, 0) == 0
        t = g.torch
        out = t.zeros(sk.in_features * sk.out_features, dtype=t.int16, device=g.dev)
        lib = skl.load_library()
        assert lib.sketch_linear_reconstruct(g.handle, out.data_ptr(), None, 0, None) == skl.SKL_ERR_INVALID_ARG
        small = t.zeros(16, dtype=t.uint8, device=g.dev)
        assert lib.sketch_linear_reconstruct(g.handle, out.data_ptr(), small.data_ptr(), 16, None) == skl.SKL_ERR_BUFFER_TOO_SMALL


# ------------------------------------------------------- grouped decode
@pytest.mark.parametrize("n_layers", [1, 2, 3, 4])
def test_grouped_decode_equals_separate_calls(n_layers):
    """q/k/v-style groups: layers of one shape with their own sketches (different widths, so different plans)
    on the same activations, one launch; bit-identical to one sketch_linear_gemv per layer and within the
    floating-point bar of the oracle."""
    import paper_2506_17255_amd as skl
    in_f, out_f, d = 192, 520, 4
    rng = np.random.default_rng(40 + n_layers)
    x = rng.standard_normal((1, in_f)).astype(np.float16)
    cases = []
    for i in range(n_layers):
        widths = rng.choice([11, 40, 100, 300], size=in_f, p=[0.7, 0.15, 0.1, 0.05])
        cases.append(custom_layer(f"group{i}", in_f, out_f, 1, out_f, d, widths, 500 + 10 * n_layers + i))
    layers = [GpuLayer(sk) for _, sk in cases]
    try:
        g0 = layers[0]
        t = g0.torch
        xd = t.from_numpy(x.view(np.int16)).to(g0.dev)
        for ydt, tdt in ((skl.SKL_F32, t.float32), (skl.SKL_F16, t.float16)):
            ys = [t.full((out_f,), float("nan"), dtype=tdt, device=g0.dev) for _ in layers]
            need = skl.sketch_linear_gemv_group_workspace_bytes([g.handle for g in layers])
            ws = t.empty(max(need, 16), dtype=t.uint8, device=g0.dev)
            skl.sketch_linear_gemv_group([g.handle for g in layers], xd.data_ptr(), skl.SKL_F16, in_f, [y.data_ptr() for y in ys],
                                         ydt, out_f, 1, ws.data_ptr(), ws.numel(), g0.stream())
            t.cuda.synchronize()
            for g, y, (W, sk) in zip(layers, ys, cases):
                alone = g.gemv(x, "f32" if ydt == skl.SKL_F32 else "f16")
                assert np.array_equal(y.cpu().numpy(), alone[0])
                ref = oracle.linear(oracle.query(sk), x)
                assert rel_fro(y.float().cpu().numpy()[None, :], ref) <= (1e-5 if ydt == skl.SKL_F32 else TOL)
    finally:
        for g in layers:
            g.close()


@pytest.mark.parametrize("h_dtype", ["f32", "f16"])
def test_gate_up_epilogue_matches_oracle(h_dtype):
    """Eq. (2), first half: h = SiLU(x W_gate) * (x W_up) from one grouped launch."""
    import paper_2506_17255_amd as skl
    in_f, out_f, d = 160, 777, 4
    rng = np.random.default_rng(61)
    x = (rng.standard_normal((1, in_f)) * 4).astype(np.float16)
    (Wg, skg), (Wu, sku) = (custom_layer("gate", in_f, out_f, 1, out_f, d, rng.choice([11, 60, 200], size=in_f), 70),
                            custom_layer("up", in_f, out_f, 1, out_f, d, [25] * in_f, 71))
    ref = oracle.gate_up(oracle.linear(oracle.query(skg), x), oracle.linear(oracle.query(sku), x))
    with GpuLayer(skg) as gg, GpuLayer(sku) as gu:
        t = gg.torch
        xd = t.from_numpy(x.view(np.int16)).to(gg.dev)
        tdt, sdt = (t.float32, skl.SKL_F32) if h_dtype == "f32" else (t.float16, skl.SKL_F16)
        h = t.full((out_f + 3,), float("nan"), dtype=tdt, device=gg.dev)
        need = skl.sketch_linear_gemv_group_workspace_bytes([gg.handle, gu.handle])
        ws = t.empty(need, dtype=t.uint8, device=gg.dev)
        skl.sketch_linear_gemv_gate_up(gg.handle, gu.handle, xd.data_ptr(), skl.SKL_F16, in_f, h.data_ptr(), sdt, out_f, 1,
                                       ws.data_ptr(), ws.numel(), gg.stream())
        t.cuda.synchronize()
        got = h.float().cpu().numpy()
        assert np.all(np.isnan(got[out_f:]))                   # nothing written past the layer's outputs
        # composition of the separate calls in float32 (same sums, same activation formula)
        yg, yu = gg.gemv(x, "f32")[0].astype(np.float32), gu.gemv(x, "f32")[0].astype(np.float32)
    assert rel_fro(got[None, :out_f], ref) <= (1e-5 if h_dtype == "f32" else TOL)
    sep = yg / (1 + np.exp(-yg.astype(np.float64))) * yu
    assert rel_fro(got[None, :out_f], sep[None, :]) <= (1e-6 if h_dtype == "f32" else TOL)


@pytest.mark.parametrize("shape", [(16, 2048, 4, 1100), (64, 4096, 3, 16), (8, 64, 8, 5), (3, 1, 2, 1)])
def test_grouped_decode_other_shapes(shape):
    """Wide outputs (more than twelve wavefronts per workgroup), tables above 64 KiB, d = 8, a 1-output layer."""
    import paper_2506_17255_amd as skl
    in_f, out_f, d, K = shape
    rng = np.random.default_rng(in_f + out_f)
    x = rng.standard_normal((1, in_f)).astype(np.float16)
    cases = [custom_layer(f"gs{i}", in_f, out_f, 1, out_f, d, [K] * in_f, 900 + i) for i in range(2)]
    layers = [GpuLayer(sk) for _, sk in cases]
    try:
        t = layers[0].torch
        xd = t.from_numpy(x.view(np.int16)).to(layers[0].dev)
        ys = [t.full((out_f,), float("nan"), dtype=t.float32, device=layers[0].dev) for _ in layers]
        need = skl.sketch_linear_gemv_group_workspace_bytes([g.handle for g in layers])
        ws = t.empty(max(need, 16), dtype=t.uint8, device=layers[0].dev)
        skl.sketch_linear_gemv_group([g.handle for g in layers], xd.data_ptr(), skl.SKL_F16, in_f, [y.data_ptr() for y in ys],
                                     skl.SKL_F32, out_f, 1, ws.data_ptr(), ws.numel(), layers[0].stream())
        t.cuda.synchronize()
        for g, y in zip(layers, ys):
            assert np.array_equal(y.cpu().numpy(), g.gemv(x, "f32")[0])
    finally:
        for g in layers:
            g.close()


@pytest.mark.parametrize("batch", [2, 5, 16])
def test_grouped_decode_batched(batch):
    """The batched (MFMA) decode kernel for a group of layers, with row strides, and the gate/up epilogue."""
    import paper_2506_17255_amd as skl
    in_f, out_f, d = 192, 520, 4
    rng = np.random.default_rng(70 + batch)
    x = rng.standard_normal((batch, in_f)).astype(np.float16)
    cases = [custom_layer(f"gb{i}", in_f, out_f, 1, out_f, d, rng.choice([11, 40, 100, 300], size=in_f, p=[0.7, 0.15, 0.1, 0.05]),
                          600 + i) for i in range(3)]
    layers = [GpuLayer(sk) for _, sk in cases]
    try:
        g0 = layers[0]
        t = g0.torch
        ldx, ldy = in_f + 8, out_f + 24
        xb = np.zeros((batch, ldx), dtype=np.float16)
        xb[:, :in_f] = x
        xd = t.from_numpy(xb.view(np.int16)).to(g0.dev)
        ys = [t.full((batch, ldy), float("nan"), dtype=t.float32, device=g0.dev) for _ in layers]
        need = skl.sketch_linear_gemv_group_workspace_bytes([g.handle for g in layers], batch)
        ws = t.empty(need, dtype=t.uint8, device=g0.dev)
        skl.sketch_linear_gemv_group([g.handle for g in layers], xd.data_ptr(), skl.SKL_F16, ldx, [y.data_ptr() for y in ys],
                                     skl.SKL_F32, ldy, batch, ws.data_ptr(), ws.numel(), g0.stream())
        t.cuda.synchronize()
        alone = []
        for g, y, (W, sk) in zip(layers, ys, cases):
            got = y.cpu().numpy()
            assert np.all(np.isnan(got[:, out_f:]))
            a = g.gemv(x, "f32")
            alone.append(a)
            assert np.array_equal(got[:, :out_f], a)
            assert rel_fro(got[:, :out_f], oracle.linear(oracle.query(sk), x)) <= 1e-5
        h = t.full((batch, ldy), float("nan"), dtype=t.float32, device=g0.dev)
        need2 = skl.sketch_linear_gemv_group_workspace_bytes([layers[0].handle, layers[1].handle], batch)
        skl.sketch_linear_gemv_gate_up(layers[0].handle, layers[1].handle, xd.data_ptr(), skl.SKL_F16, ldx, h.data_ptr(),
                                       skl.SKL_F32, ldy, batch, ws.data_ptr(), max(need2, 16), g0.stream())
        t.cuda.synchronize()
        hh = h.cpu().numpy()
        assert np.all(np.isnan(hh[:, out_f:]))
        ref = oracle.gate_up(oracle.linear(oracle.query(cases[0][1]), x), oracle.linear(oracle.query(cases[1][1]), x))
        assert rel_fro(hh[:, :out_f], ref) <= 1e-5
    finally:
        for g in layers:
            g.close()


def test_grouped_decode_with_low_bit_layers():
    import paper_2506_17255_amd as skl
    W, sk = small_case("row_classes")
    q4, q8 = oracle.quantize(sk, 4), oracle.quantize(sk, 8)
    rng = np.random.default_rng(95)
    x = rng.standard_normal((1, sk.in_features)).astype(np.float16)
    with GpuLayer(sk) as g, GpuLayer(q4) as g4, GpuLayer(q8) as g8:
        t = g.torch
        xd = t.from_numpy(x.view(np.int16)).to(g.dev)
        layers = [g4, g, g8]
        ys = [t.full((sk.out_features,), float("nan"), dtype=t.float32, device=g.dev) for _ in layers]
        need = skl.sketch_linear_gemv_group_workspace_bytes([l.handle for l in layers])
        assert need >= 2 * 2 * sk.states.size
        ws = t.empty(need, dtype=t.uint8, device=g.dev)
        skl.sketch_linear_gemv_group([l.handle for l in layers], xd.data_ptr(), skl.SKL_F16, sk.in_features,
                                     [y.data_ptr() for y in ys], skl.SKL_F32, sk.out_features, 1, ws.data_ptr(), ws.numel(),
                                     g.stream())
        t.cuda.synchronize()
        for l, y in zip(layers, ys):
            assert np.array_equal(y.cpu().numpy(), l.gemv(x, "f32")[0])
        for l, y, s_ in zip(layers, ys, (q4, sk, q8)):
            assert rel_fro(y.cpu().numpy()[None, :], oracle.linear(oracle.query(s_), x)) <= 1e-5


def test_grouped_decode_rejects_mixed_shapes_and_bad_arguments():
    import ctypes
    import paper_2506_17255_amd as skl
    _, a = custom_layer("ga", 64, 256, 1, 256, 4, [16] * 64, 1)
    _, b = custom_layer("gb", 64, 128, 1, 128, 4, [16] * 64, 2)
    _, c = small_case("tile_ragged")
    with GpuLayer(a) as ga, GpuLayer(b) as gb, GpuLayer(c) as gc, GpuLayer(oracle.quantize(a, 8)) as gq:
        t = ga.torch
        x = t.zeros(96, dtype=t.float16, device=ga.dev)
        y = [t.zeros(256, dtype=t.float32, device=ga.dev) for _ in range(2)]
        ws = t.zeros(1 << 20, dtype=t.uint8, device=ga.dev)

        def status(layers, ys=None, x_dt=skl.SKL_F16, y_dt=skl.SKL_F32, nbytes=1 << 20, batch=1):
            ys = ys or [v.data_ptr() for v in y[:len(layers)]]
            try:
                skl.sketch_linear_gemv_group([g.handle for g in layers], x.data_ptr(), x_dt, 96, ys, y_dt, 256, batch,
                                             ws.data_ptr(), nbytes, ga.stream())
                return skl.SKL_OK
            except skl.SketchLinearError as e:
                return e.status

        assert status([ga, ga]) == skl.SKL_OK
        assert status([ga, gb]) == skl.SKL_ERR_UNSUPPORTED            # different out_features
        assert status([gc]) == skl.SKL_ERR_UNSUPPORTED                # not a row-sketch layer
        assert status([ga, gq]) == skl.SKL_OK                         # low-bit states may join a group
        assert status([ga, ga], ys=[y[0].data_ptr(), y[0].data_ptr()]) == skl.SKL_ERR_INVALID_ARG   # outputs overlap
        assert status([ga], x_dt=skl.SKL_BF16) == skl.SKL_ERR_UNSUPPORTED
        assert status([ga], y_dt=skl.SKL_BF16) == skl.SKL_ERR_UNSUPPORTED
        assert status([ga, ga], nbytes=64) == skl.SKL_ERR_BUFFER_TOO_SMALL
        assert status([ga], batch=17) == skl.SKL_ERR_INVALID_ARG
        assert status([ga], batch=0) == skl.SKL_ERR_INVALID_ARG
        L = skl.load_library()
        assert L.sketch_linear_gemv_group(None, 1, None, 0, 0, None, 0, 0, 1, None, 0, None) == skl.SKL_ERR_INVALID_ARG
        five = (ctypes.c_void_p * 5)(*[ga.handle] * 5)
        assert L.sketch_linear_gemv_group(five, 5, x.data_ptr(), 0, 96, five, 2, 256, 1, ws.data_ptr(), 1 << 20, None) == skl.SKL_ERR_INVALID_ARG
        t.cuda.synchronize()


# ------------------------------------------------- sketch construction
@pytest.mark.parametrize("name", SMALL)
def test_states_built_on_the_gpu_equal_the_oracle_update(name):
    """Eq. 4 on the device: bit-identical states to the oracle's sequential update stream."""
    from skl_harness import build_states_on_gpu
    W, sk = small_case(name)
    got = build_states_on_gpu(W, sk.tile_in, sk.tile_out, sk.d, sk.hash_a, sk.hash_c, sk.group_width)
    assert np.array_equal(got, sk.states), (name, int(np.sum(got != sk.states)))


@pytest.mark.parametrize("geom", [(48, 96, 1, 96, 3, 7), (32, 64, 8, 32, 4, 5), (40, 40, 40, 40, 2, 300)])
def test_states_built_on_the_gpu_with_many_magnitude_ties(geom):
    """Weights from a handful of values of both signs: almost every bucket sees equal magnitudes, so the
    first-arrival rule of Eq. 4 (and the sign the state keeps) decides most states."""
    from skl_harness import build_states_on_gpu
    in_f, out_f, tj, to, d, K = geom
    rng = np.random.default_rng(in_f * 1000 + out_f)
    W = rng.choice(np.array([-2.0, -1.0, -0.5, 0.0, 0.5, 1.0, 2.0], dtype=np.float16), size=(in_f, out_f))
    W[rng.random((in_f, out_f)) < 0.05] = np.float16(-0.0)
    A = rng.integers(1, 1 << 24, d) | 1
    C = rng.integers(0, 1 << 24, d)
    widths = np.full((in_f // tj) * (out_f // to), K, dtype=np.uint32)
    sk = oracle.update(W, tj, to, d, A, C, widths)
    got = build_states_on_gpu(W, tj, to, d, A, C, widths)
    assert np.array_equal(got, sk.states)
    twice = build_states_on_gpu(W, tj, to, d, A, C, widths)
    assert np.array_equal(got, twice)                  # independent of the order in which threads arrive


# ------------------------------------------------------------ HIP graphs
def test_calls_replay_correctly_from_a_hip_graph():
    """Every entry point only enqueues kernels (no memset or copy nodes), so a caller may capture it: decode,
    grouped decode, prefill and a low-bit layer captured once, replayed three times with eager work and
    synchronisation in between, each replay compared with the eager results."""
    import paper_2506_17255_amd as skl
    W, sk = small_case("row_classes")
    q = oracle.quantize(sk, 4)
    rng = np.random.default_rng(90)
    with GpuLayer(sk) as g, GpuLayer(q) as gq:
        t = g.torch
        dev = g.dev
        x = t.from_numpy(rng.standard_normal((1, sk.in_features)).astype(np.float16).view(np.int16)).to(dev)
        X = t.from_numpy(wk.f32_to_bf16_bits(rng.standard_normal((300, sk.in_features)).astype(np.float32)).view(np.int16)).to(dev)
        y = {k: t.zeros(sk.out_features, dtype=t.float32, device=dev) for k in ("gemv", "grp0", "grp1", "lowbit")}
        Y = t.zeros(300, sk.out_features, dtype=t.float32, device=dev)
        sizes = [skl.sketch_linear_workspace_bytes(g.handle, 0, 1), skl.sketch_linear_workspace_bytes(g.handle, 1, 300),
                 skl.sketch_linear_workspace_bytes(gq.handle, 0, 1), skl.sketch_linear_gemv_group_workspace_bytes([g.handle] * 2)]
        ws = [t.empty(n, dtype=t.uint8, device=dev) for n in sizes]

        def enqueue(stream):
            skl.sketch_linear_gemv(g.handle, x.data_ptr(), skl.SKL_F16, sk.in_features, y["gemv"].data_ptr(), skl.SKL_F32,
                                   sk.out_features, 1, ws[0].data_ptr(), sizes[0], stream)
            skl.sketch_linear_gemm(g.handle, X.data_ptr(), skl.SKL_BF16, sk.in_features, Y.data_ptr(), skl.SKL_F32,
                                   sk.out_features, 300, ws[1].data_ptr(), sizes[1], stream)
            skl.sketch_linear_gemv(gq.handle, x.data_ptr(), skl.SKL_F16, sk.in_features, y["lowbit"].data_ptr(), skl.SKL_F32,
                                   sk.out_features, 1, ws[2].data_ptr(), sizes[2], stream)
            skl.sketch_linear_gemv_group([g.handle, g.handle], x.data_ptr(), skl.SKL_F16, sk.in_features,
                                         [y["grp0"].data_ptr(), y["grp1"].data_ptr()], skl.SKL_F32, sk.out_features, 1,
                                         ws[3].data_ptr(), sizes[3], stream)

        enqueue(g.stream())                                   # eager (also the one-time kernel attribute calls)
        t.cuda.synchronize()
        want = {k: v.clone() for k, v in y.items()}
        want_Y = Y.clone()
        graph = t.cuda.CUDAGraph()
        with t.cuda.graph(graph):
            enqueue(t.cuda.current_stream().cuda_stream)
        for rep in range(3):
            for v in y.values():
                v.fill_(float(rep))                           # eager work between the replays
            Y.zero_()
            t.cuda.synchronize()
            graph.replay()
            t.cuda.synchronize()
            for k in y:
                assert t.equal(y[k], want[k]), (rep, k)
            assert t.equal(Y, want_Y), rep
        assert t.equal(want["grp0"], want["gemv"]) and t.equal(want["grp1"], want["gemv"])
        del graph


# ----------------------------------------------------------- error paths
def test_call_time_validation():
    import paper_2506_17255_amd as skl
    W, sk = small_case("row_ragged")
    with GpuLayer(sk) as g:
        t = g.torch
        x = t.zeros(16, sk.in_features, dtype=t.float16, device=g.dev)
        y = t.zeros(16, sk.out_features, dtype=t.float32, device=g.dev)
        ws, need = g.workspace(0, 16)
        args = dict(layer=g.handle, x=x.data_ptr(), x_dtype=skl.SKL_F16, ldx=sk.in_features, y=y.data_ptr(),
                    y_dtype=skl.SKL_F32, ldy=sk.out_features, batch=16, workspace=ws.data_ptr(),
                    workspace_bytes=need, hip_stream=g.stream())

        def status(**over):
            try:
                skl.sketch_linear_gemv(**{**args, **over})
                return 0
            except skl.SketchLinearError as e:
                return e.status
        assert status() == 0
        assert status(batch=0) == skl.SKL_ERR_INVALID_ARG
        assert status(batch=17) == skl.SKL_ERR_INVALID_ARG
        assert status(x_dtype=skl.SKL_BF16) == skl.SKL_ERR_UNSUPPORTED
        assert status(y_dtype=skl.SKL_BF16) == skl.SKL_ERR_UNSUPPORTED
        assert status(ldx=sk.in_features - 1) == skl.SKL_ERR_INVALID_ARG
        assert status(ldy=sk.out_features - 1) == skl.SKL_ERR_INVALID_ARG
        assert status(workspace_bytes=need - 1) == skl.SKL_ERR_BUFFER_TOO_SMALL
        assert status(workspace=0) == skl.SKL_ERR_INVALID_ARG
        assert status(x=x.data_ptr() + 2) == skl.SKL_ERR_INVALID_ARG
        assert status(y=x.data_ptr()) == skl.SKL_ERR_INVALID_ARG          # aliasing
        assert status(x=0) == skl.SKL_ERR_INVALID_ARG
        t.cuda.synchronize()


@pytest.mark.gpu
@pytest.mark.parametrize("name,bits,mode", [("row_classes", 0, 0), ("row_classes", 4, 1), ("cfg1", 0, 0), ("tile_ragged", 8, 0)])
def test_a_layer_created_from_its_file_image_is_the_same_layer(name, bits, mode):
    """Sec. 3.1: the states, select parameters and widths are the whole layer; written to the flat file format
    and opened in place they give the oracle's reconstruction (Eq. 5) bit for bit and the same decode output."""
    W, sk = small_case(name)
    if bits:
        sk = oracle.quantize(sk, bits)
    want = oracle.query(sk, mode)
    x = np.random.default_rng(31).standard_normal((2, sk.in_features)).astype(np.float16)
    with GpuLayer(sk, flags_of(name), mode, through_file=True) as g, GpuLayer(sk, flags_of(name), mode) as direct:
        assert g.info == direct.info
        assert np.array_equal(g.reconstruct(), want)
        assert np.array_equal(g.gemv(x, "f32"), direct.gemv(x, "f32"))


def test_ceiling_kernels_run_and_report_their_work():
    """The five small kernels behind the measured ceilings of the benchmark: each launches, finishes and
    reports a positive amount of work; the matrix-core rate with operands of random bits is a real rate
    (positive, not above the constant-operand one by more than measurement noise)."""
    import torch
    dev = torch.device("cuda:0")
    ws = torch.empty((4 << 20) + (64 << 20), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    rate = {}
    for kind in range(5):
        iters = 200 if kind < 2 else 4000
        ts = []
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            work = skl.sketch_linear_microbench(kind, iters, ws.data_ptr(), ws.numel(), stream)
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1) * 1e-3)
        assert work > 0
        rate[kind] = work / min(ts)
    assert rate[2] > 1e14 and rate[4] > 1e14
    assert rate[4] <= 1.1 * rate[2]
