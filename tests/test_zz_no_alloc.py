"""The decode entry point that allocates nothing (scratch in a device array inside the library) against
the entry point that takes a workspace: same kernels, same summation order, so the outputs must be
bit-identical; both are also held to the oracle.  Two calls in a row on the same GPU, the second with a
smaller layer and batch, so that what the first call left in the shared array cannot leak into the second."""
import numpy as np
import pytest

import oracle
import paper_2506_17255_amd as skl
import workloads as wk
from skl_harness import DT, GpuLayer, build_sketch, rel_fro

pytestmark = pytest.mark.gpu


def gemv_static(g: GpuLayer, x_f16: np.ndarray, y_dtype: str) -> np.ndarray:
    t = g.torch
    batch, in_f = x_f16.shape
    xd = t.from_numpy(np.ascontiguousarray(x_f16).view(np.int16)).to(g.dev)
    ydt = {"f32": t.float32, "f16": t.float16}[y_dtype]
    yd = t.full((batch, g.sk.out_features), float("nan"), dtype=ydt, device=g.dev)
    skl.sketch_linear_gemv_static(g.handle, xd.data_ptr(), skl.SKL_F16, in_f, yd.data_ptr(), DT[y_dtype],
                                  g.sk.out_features, batch, g.stream())
    t.cuda.synchronize()
    return yd.cpu().numpy()


def test_static_scratch_decode_matches_the_workspace_decode():
    first = wk.small("noalloc_first", 1024, 2048 + 192, 1, 2048 + 192, 4, 0.5, 301, outlier_frac=0.02, width_mult=4.0)
    second = wk.small("noalloc_second", 256, 300, 1, 300, 3, 0.5, 302)
    for wl, batch in ((first, 8), (second, 1)):
        W, sk = build_sketch(wl)
        W_hat = oracle.query(sk)
        x = wk.gen_x(wl, batch)
        ref = oracle.linear(W_hat, x)
        with GpuLayer(sk) as g:
            for y_dtype in ("f32", "f16"):
                print(f"[no-alloc] {wl.name} batch {batch} {y_dtype}", flush=True)
                want = g.gemv(x, y_dtype)
                got = gemv_static(g, x, y_dtype)
                assert np.array_equal(got.view(np.uint8), np.ascontiguousarray(want).view(np.uint8))
                assert rel_fro(got, ref) <= (1e-5 if y_dtype == "f32" else 1e-3)


def test_static_scratch_limit_is_an_error_not_a_launch():
    """A call whose scratch would not fit the static array is refused before anything is enqueued.  The layer
    is 8192 x 65536 with random finite states (no oracle needed: the two entry points are compared with each
    other); its batch-16 partial sums exceed the array, its batch-1 partial sums fit."""
    in_f, out_f, d, K = 8192, 65536, 2, 64
    rng = np.random.default_rng(303)
    states = (rng.standard_normal(in_f * d * K, dtype=np.float32) * np.float32(0.02)).astype(np.float16).view(np.uint16)
    sk = oracle.Sketch(in_features=in_f, out_features=out_f, tile_in=1, tile_out=out_f, d=d,
                       hash_a=np.uint32([0x9E3779, 0x5BD1E9]), hash_c=np.uint32([0, 0x7F4A7C]),
                       group_width=np.full(in_f, K, dtype=np.uint32), states=states)
    x16 = rng.standard_normal((16, in_f), dtype=np.float32).astype(np.float16)
    with GpuLayer(sk) as g:
        assert skl.sketch_linear_workspace_bytes(g.handle, 0, 16) > skl.SKL_STATIC_SCRATCH_MAX
        with pytest.raises(skl.SketchLinearError) as err:
            gemv_static(g, x16, "f32")
        assert err.value.status == skl.SKL_ERR_UNSUPPORTED
        assert skl.sketch_linear_workspace_bytes(g.handle, 0, 1) <= skl.SKL_STATIC_SCRATCH_MAX
        assert np.array_equal(gemv_static(g, x16[:1], "f32"), g.gemv(x16[:1], "f32"))
