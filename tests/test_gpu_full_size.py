"""GPU parity at the benchmark's full sizes, in the launch configuration the
benchmark times.  Reconstructed weights are compared bit for bit over the
whole layer; outputs are compared on all outputs (gemv) or on sampled rows
and columns the oracle computes one by one (gemm)."""
import functools

import numpy as np
import pytest

import oracle
import workloads as wk
from skl_harness import GpuLayer, build_sketch, rel_fro, round_to_bf16

pytestmark = pytest.mark.gpu
TOL = 1e-3


@functools.lru_cache(maxsize=2)
def layer(key):
    wl = {"cfg2": wk.cfg2(), "cfg2_2d": wk.cfg2(True), "cfg3_up": wk.cfg3("up"), "cfg3_down": wk.cfg3("down"),
          "cfg4_4096_0.5": wk.cfg4(4096, 0.5), "cfg4_11008_0.75": wk.cfg4(11008, 0.75)}[key]
    W, sk = build_sketch(wl)
    return wl, sk, oracle.query(sk)


@pytest.mark.parametrize("key", ["cfg2", "cfg2_2d", "cfg3_up", "cfg3_down"])
def test_decode_layers(key):
    wl, sk, W_hat = layer(key)
    print(f"[full-size] {wl.name}: {sk.bits_per_weight:.4f} bit/weight", flush=True)
    with GpuLayer(sk) as g:
        assert np.array_equal(g.reconstruct(), W_hat)
        for batch in wl.batches:
            x = wk.gen_x(wl, batch)
            cols = np.random.default_rng(batch).choice(wl.out_features, size=256, replace=False)
            ref = oracle.linear(W_hat, x, cols=cols)
            y = g.gemv(x, "f32")
            assert rel_fro(y[:, cols], ref) <= TOL
            assert rel_fro(y[:, cols], ref) <= 1e-5
            y16 = g.gemv(x, "f16")
            assert rel_fro(y16[:, cols], ref) <= TOL
        # whole-output check at batch 1 against the fp64 oracle
        x = wk.gen_x(wl, 1)
        assert rel_fro(g.gemv(x, "f32"), oracle.linear(W_hat, x)) <= 1e-5


@pytest.mark.parametrize("key", ["cfg4_4096_0.5", "cfg4_11008_0.75"])
def test_prefill_layers(key):
    wl, sk, W_hat = layer(key)
    X = wk.gen_X_bf16(wl, wl.tokens)
    rng = np.random.default_rng(4)
    rows = np.sort(rng.choice(wl.tokens, size=24, replace=False))
    cols = np.sort(rng.choice(wl.out_features, size=192, replace=False))
    ref = oracle.linear(W_hat, X[rows], x_kind="bf16", cols=cols)
    with GpuLayer(sk) as g:
        assert np.array_equal(g.reconstruct(), W_hat)
        y32 = g.gemm(X, "bf16", "f32")
        assert rel_fro(y32[np.ix_(rows, cols)], ref) <= 1e-5
        ybf = g.gemm(X, "bf16", "bf16")
        assert rel_fro(ybf[np.ix_(rows, cols)], round_to_bf16(ref)) <= TOL
        # property that holds at any size: every row of the prefill equals the decode of that row
        t = int(rows[0])
        xh = wk.bf16_bits_to_f32(X[t:t + 1]).astype(np.float16)
        assert rel_fro(y32[t:t + 1], g.gemv(xh, "f32")) <= 1e-5
