"""GPU parity at the benchmark's full sizes, in the launch configuration the
benchmark times.  Reconstructed weights are compared bit for bit over the
whole layer; decode outputs are compared on all outputs; prefill outputs on
a grid of rows and columns the oracle computes one by one that puts samples
into every 256 x 256 output tile (the unit the prefill kernels divide the
work by, including every tile that several workgroups share), and over the
whole output against numpy's binary64 product of the oracle's weights, tile
by tile."""
import functools

import numpy as np
import pytest

import oracle
import workloads as wk
import paper_2506_17255_amd as skl
from skl_harness import (GpuLayer, build_sketch, matmul_f64, rel_fro, round_to_bf16, stratified_sample,
                         worst_tile_rel_fro)

pytestmark = pytest.mark.gpu
TOL = 1e-3


@functools.lru_cache(maxsize=2)
def layer(key):
    wl = {"cfg2": wk.cfg2(), "cfg2_2d": wk.cfg2(True), "cfg3_up": wk.cfg3("up"), "cfg3_down": wk.cfg3("down"),
          "cfg4_4096_0.5": wk.cfg4(4096, 0.5), "cfg4_11008_0.75": wk.cfg4(11008, 0.75),
          "cfg4_11008_0.5": wk.cfg4(11008, 0.5), "cfg4_4096_0.75": wk.cfg4(4096, 0.75)}[key]
    W, sk = build_sketch(wl)
    return wl, sk, oracle.query(sk)


@pytest.mark.parametrize("key", ["cfg2", "cfg2_2d", "cfg3_up", "cfg3_down"])
def test_decode_layers(key):
    wl, sk, W_hat = layer(key)
    print(f"[full-size] {wl.name}: {sk.bits_per_weight:.4f} bit/weight", flush=True)
    with GpuLayer(sk) as g:
        assert np.array_equal(g.reconstruct(), W_hat)
        assert np.array_equal(g.reconstruct(hash_op=True), W_hat)
        for batch in wl.batches:
            x = wk.gen_x(wl, batch)
            ref = oracle.linear(W_hat, x)              # every output of every batch row
            y = g.gemv(x, "f32")
            assert rel_fro(y, ref) <= 1e-5
            for b in range(batch):
                assert rel_fro(y[b], ref[b]) <= 1e-5
            y16 = g.gemv(x, "f16")
            assert rel_fro(y16, ref) <= TOL
        # whole-output check at batch 1 against the fp64 oracle
        x = wk.gen_x(wl, 1)
        assert rel_fro(g.gemv(x, "f32"), oracle.linear(W_hat, x)) <= 1e-5


def check_prefill(g, W_hat, X, seed, expect_kernel=None):
    """Prefill outputs of layer g against the oracle: samples in every output tile, then every output."""
    tokens, out = X.shape[0], W_hat.shape[1]
    if expect_kernel is not None:
        assert g.info["prefill_kernel"] == expect_kernel
    rows, cols = stratified_sample(tokens, out, seed)
    ref = oracle.linear(W_hat, X[rows], x_kind="bf16", cols=cols)
    full = matmul_f64(W_hat, X)
    assert rel_fro(full[np.ix_(rows, cols)], ref) <= 1e-12          # the library routine agrees with the oracle's loops
    y32 = g.gemm(X, "bf16", "f32")
    assert rel_fro(y32[np.ix_(rows, cols)], ref) <= 1e-5
    assert worst_tile_rel_fro(y32, full) <= 1e-5
    ybf = g.gemm(X, "bf16", "bf16")
    assert rel_fro(ybf[np.ix_(rows, cols)], round_to_bf16(ref)) <= TOL
    assert worst_tile_rel_fro(ybf, round_to_bf16(full)) <= TOL
    return y32


@pytest.mark.parametrize("kernel", ["by_call", "fused"])
@pytest.mark.parametrize("key", ["cfg4_4096_0.5", "cfg4_4096_0.75", "cfg4_11008_0.5", "cfg4_11008_0.75"])
def test_prefill_layers(key, kernel):
    """Configuration 4: 2048 tokens through 4096 x 4096 and 4096 x 11008 at 0.5 and 0.75 bit/weight, with the
    kernel the library picks for a call of this length (the staged one) and with the fused kernel asked for."""
    wl, sk, W_hat = layer(key)
    X = wk.gen_X_bf16(wl, wl.tokens)
    with GpuLayer(sk, skl.FLAG_FUSED_PREFILL if kernel == "fused" else 0) as g:
        print(f"[full-size] {wl.name}: prefill kernel {g.info['prefill_kernel']}, staged from {g.info['prefill_staged_from']} tokens, "
              f"block classes {g.info['block_classes']:#x}", flush=True)
        assert g.info["prefill_staged_from"] == (0xFFFFFFFF if kernel == "fused" else 513)
        assert np.array_equal(g.reconstruct(), W_hat)
        y32 = check_prefill(g, W_hat, X, 4, expect_kernel=skl.SKL_PREFILL_FUSED)
        # property that holds at any size: every row of the prefill equals the decode of that row
        for t in (0, 1037, wl.tokens - 1):
            xh = wk.bf16_bits_to_f32(X[t:t + 1]).astype(np.float16)
            assert rel_fro(y32[t:t + 1], g.gemv(xh, "f32")) <= 1e-5


def test_signed_max_query_mode_on_the_up_projection():
    """Query mode 1 (Eq. 5 as printed) at full size: 4096 x 11008, importance widths, decode and prefill."""
    wl, sk, _ = layer("cfg3_up")
    W_hat = oracle.query(sk, oracle.QUERY_SIGNED_MAX)
    x = wk.gen_x(wl, 8)
    X = wk.gen_X_bf16(wl, 2048)
    with GpuLayer(sk, query_mode=1) as g:
        assert np.array_equal(g.reconstruct(), W_hat)
        assert rel_fro(g.gemv(x[:1], "f32"), oracle.linear(W_hat, x[:1])) <= 1e-5
        assert rel_fro(g.gemv(x, "f32"), oracle.linear(W_hat, x)) <= 1e-5
        check_prefill(g, W_hat, X, 11)


@pytest.mark.parametrize("index", range(7))
def test_stack_block_layers(index):
    """The seven linear layers of the first decoder block of the Llama-2-7B-shaped stack (q, k, v, o, gate,
    up, down; own seed each): bit-exact weights and batch-1 decode against the oracle."""
    wl = wk.cfg5_stack(1)[index]
    W, sk = build_sketch(wl)
    W_hat = oracle.query(sk)
    print(f"[full-size] {wl.name}: {sk.bits_per_weight:.4f} bit/weight", flush=True)
    x = wk.gen_x(wl, 1)
    with GpuLayer(sk) as g:
        assert np.array_equal(g.reconstruct(), W_hat)
        y = g.gemv(x, "f32")
        y16 = g.gemv(x, "f16")
    ref = oracle.linear(W_hat, x)
    assert rel_fro(y, ref) <= 1e-5
    assert rel_fro(y16, ref) <= TOL


def test_every_layer_of_the_stack():
    """All 224 layers of the Llama-2-7B-shaped stack (own seed, own outlier channels each): the weights
    the library reconstructs have the digest of the oracle's, and the batch-1 decode matches the oracle's
    output.  The oracle's share (update, query, linear: ~7 s per layer) runs in a pool of host processes."""
    import hashlib
    import multiprocessing as mp
    import os
    from skl_harness import oracle_stack_layer
    n_layers = 224
    workers = max(1, min(16, os.cpu_count() or 1))
    done = 0
    with mp.get_context("spawn").Pool(workers) as pool:
        for index, sk, digest, y_ref in pool.imap_unordered(oracle_stack_layer, range(n_layers)):
            wl = wk.cfg5_stack(32)[index]
            with GpuLayer(sk) as g:
                got = g.reconstruct()
                assert hashlib.sha1(np.ascontiguousarray(got).tobytes()).hexdigest() == digest, wl.name
                assert rel_fro(g.gemv(wk.gen_x(wl, 1), "f32"), y_ref) <= 1e-5, wl.name
            done += 1
            if done % 16 == 0:
                print(f"[full-size] stack: {done} of {n_layers} layers checked", flush=True)
    assert done == n_layers


def test_70b_shaped_layer():
    """8192 x 28672, d = 4, 0.5 bit/weight with importance widths: decode at batch 1 over all outputs and the
    2048-token prefill on sampled rows and columns; narrow blocks (two words per state row) at full size."""
    wl = wk.cfg5_70b()
    W, sk = build_sketch(wl)
    W_hat = oracle.query(sk)
    print(f"[full-size] {wl.name}: {sk.bits_per_weight:.4f} bit/weight", flush=True)
    x = wk.gen_x(wl, 1)
    X = wk.gen_X_bf16(wl, wl.tokens)
    with GpuLayer(sk) as g:
        print(f"[full-size] prefill kernel {g.info['prefill_kernel']}, block classes {g.info['block_classes']:#x}", flush=True)
        assert np.array_equal(g.reconstruct(), W_hat)
        y = g.gemv(x, "f32")
        assert rel_fro(y, oracle.linear(W_hat, x)) <= 1e-5
        check_prefill(g, W_hat, X, 5)


@pytest.mark.parametrize("bits,mult", [(4, 4.0), (8, 2.0)])
def test_low_bit_layer(bits, mult):
    """The up projection with low-bit states at 0.5 bit/weight: 4-bit codes with four times the states
    (one state per eight weights, the paper's recipe, Sec. 4) and 8-bit codes with twice the states."""
    import dataclasses
    wl = dataclasses.replace(wk.cfg3("up"), bpw=0.5 * mult)
    W, sk = build_sketch(wl)
    q = oracle.quantize(sk, bits)
    print(f"[full-size] {wl.name} {bits}-bit states: {q.bits_per_weight:.4f} bit/weight", flush=True)
    assert 0.49 < q.bits_per_weight < 0.52
    W_hat = oracle.query(q)
    x = wk.gen_x(wl, 16)
    X = wk.gen_X_bf16(wl, 2048)
    with GpuLayer(q) as g:
        print(f"[full-size] prefill kernel {g.info['prefill_kernel']}, block classes {g.info['block_classes']:#x}", flush=True)
        assert np.array_equal(g.reconstruct(), W_hat)
        assert rel_fro(g.gemv(x[:1], "f32"), oracle.linear(W_hat, x[:1])) <= 1e-5
        assert rel_fro(g.gemv(x, "f32"), oracle.linear(W_hat, x)) <= 1e-5
        check_prefill(g, W_hat, X, bits)
        assert g.info["table_bytes"] * 8 <= 0.52 * wl.in_features * wl.out_features


def test_sketch_construction_of_the_up_projection():
    """All 45 M weights of the benchmark layer through the device-side update (Eq. 4)."""
    from skl_harness import build_states_on_gpu
    wl = wk.cfg3("up")
    W, sk = build_sketch(wl)
    got = build_states_on_gpu(W, sk.tile_in, sk.tile_out, sk.d, sk.hash_a, sk.hash_c, sk.group_width)
    assert np.array_equal(got, sk.states)


def mixed_stack_budgets(n_blocks=32):
    """Sketch space of every layer of the Llama-2-7B-shaped stack under layer-wise importance (Sec. 3.2):
    synthetic layer scales times the row-wise values, 0.5 bit/weight on average."""
    shapes = wk.cfg5_stack(n_blocks)
    scales = wk.gen_layer_scales(len(shapes))
    imp = [oracle.layer_importance(s * wk.gen_importance(wl)) for s, wl in zip(scales, shapes)]
    sizes = [wl.n_weights for wl in shapes]
    return shapes, oracle.allocate_layer_budgets(imp, sum(sizes) // 32, sizes=sizes)


@pytest.mark.parametrize("which", ["least", "most"])
def test_layer_with_a_layer_wise_budget(which):
    """The up projection that the layer-wise allocation gives the least / the most space: other width
    classes and table sizes than the uniform 0.5 bit/weight layers, same kernels, same bar."""
    shapes, budgets = mixed_stack_budgets()
    ups = [i for i, wl in enumerate(shapes) if wl.name.endswith("_up")]
    bpw = [16.0 * budgets[i] / shapes[i].n_weights for i in ups]
    i = ups[int(np.argmin(bpw) if which == "least" else np.argmax(bpw))]
    wl = shapes[i]
    widths = oracle.allocate_widths(wk.gen_importance(wl), int(budgets[i]), wl.d)
    W, sk = build_sketch(wl, widths=widths)
    print(f"[full-size] {wl.name}: {sk.bits_per_weight:.4f} bit/weight, widths {sorted(set(widths.tolist()))}", flush=True)
    assert (sk.bits_per_weight < 0.35) if which == "least" else (sk.bits_per_weight > 0.7)
    W_hat = oracle.query(sk)
    x = wk.gen_x(wl, 1)
    X = wk.gen_X_bf16(wl, 300)
    cols = np.sort(np.random.default_rng(6).choice(wl.out_features, size=192, replace=False))
    with GpuLayer(sk) as g:
        assert np.array_equal(g.reconstruct(), W_hat)
        assert rel_fro(g.gemv(x, "f32"), oracle.linear(W_hat, x)) <= 1e-5
        x8 = wk.gen_x(wl, 8)
        assert rel_fro(g.gemv(x8, "f32")[:, cols], oracle.linear(W_hat, x8, cols=cols)) <= 1e-5
        y = g.gemm(X, "bf16", "f32")
        assert rel_fro(y[:, cols], oracle.linear(W_hat, X, x_kind="bf16", cols=cols)) <= 1e-5
