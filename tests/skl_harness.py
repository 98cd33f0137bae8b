"""Test-side plumbing: torch owns device memory and streams, the library is
called through its C ABI binding, the oracle provides sketches and expected
values.  Nothing here computes any step of the method."""
from __future__ import annotations

import numpy as np

import oracle
import paper_2506_17255_amd as skl
import workloads as wk

DT = {"f16": skl.SKL_F16, "bf16": skl.SKL_BF16, "f32": skl.SKL_F32}


def torch_mod():
    import torch
    return torch


def build_sketch(wl: wk.Workload, W=None, widths=None):
    """(W, oracle.Sketch) for a workload: seeded weights, seeded hash
    parameters, importance-aware widths, states from the oracle's update."""
    W = wk.gen_weight(wl) if W is None else W
    A, C = wk.gen_hash_params(wl)
    if widths is None:
        widths = oracle.allocate_widths(wk.gen_importance(wl), wl.budget_states, wl.d)
    return W, oracle.update(W, wl.tile_in, wl.tile_out, wl.d, A, C, widths)


def desc_of(sk: oracle.Sketch, flags: int = 0, query_mode: int = 0):
    if isinstance(sk, oracle.QuantSketch):
        codes = np.ascontiguousarray(sk.codes, dtype=np.int8)
        packed = codes.view(np.uint8) if sk.bits == 8 else wk.pack_nibbles(codes)
        return skl.make_desc(sk.in_features, sk.out_features, sk.tile_in, sk.tile_out, sk.d,
                             np.ascontiguousarray(sk.hash_a, dtype=np.uint32),
                             np.ascontiguousarray(sk.hash_c, dtype=np.uint32),
                             np.ascontiguousarray(sk.group_width, dtype=np.uint32), None, n_states=codes.size,
                             flags=flags, query_mode=query_mode, state_bits=sk.bits, codes=packed,
                             scales=np.ascontiguousarray(sk.scales, dtype=np.uint16))
    return skl.make_desc(sk.in_features, sk.out_features, sk.tile_in, sk.tile_out, sk.d,
                         np.ascontiguousarray(sk.hash_a, dtype=np.uint32),
                         np.ascontiguousarray(sk.hash_c, dtype=np.uint32),
                         np.ascontiguousarray(sk.group_width, dtype=np.uint32),
                         np.ascontiguousarray(sk.states, dtype=np.uint16), flags=flags, query_mode=query_mode)


class GpuLayer:
    """A layer resident on cuda:0 plus the buffers its calls need."""

    def __init__(self, sk: oracle.Sketch, flags: int = 0, query_mode: int = 0, through_file: bool = False):
        torch = torch_mod()
        if not torch.cuda.is_available():
            raise RuntimeError("GPU tests need a GPU")
        self.torch = torch
        self.sk = sk
        self.dev = torch.device("cuda:0")
        desc = desc_of(sk, flags, query_mode)
        if through_file:                    # the description as a flat layer file image, opened in place
            image = np.zeros(skl.sketch_linear_file_bytes(desc), dtype=np.uint8)
            skl.sketch_linear_file_write(desc, image)
            desc = skl.sketch_linear_file_open(image)
        nbytes = skl.sketch_linear_device_bytes(desc)
        self.dev_buf = torch.zeros(nbytes, dtype=torch.uint8, device=self.dev)
        self.handle = skl.sketch_linear_create(desc, self.dev_buf.data_ptr(), nbytes, self.stream())
        self.info = skl.sketch_linear_info(self.handle)
        self._ws = None

    def stream(self) -> int:
        return self.torch.cuda.current_stream().cuda_stream

    def close(self):
        if self.handle:
            self.torch.cuda.synchronize()
            skl.sketch_linear_destroy(self.handle)
            self.handle = None

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    def workspace(self, op: int, n: int):
        need = skl.sketch_linear_workspace_bytes(self.handle, op, n)
        if self._ws is None or self._ws.numel() < max(need, 16):
            self._ws = self.torch.empty(max(need, 16), dtype=self.torch.uint8, device=self.dev)
        return self._ws, need

    def reconstruct(self, hash_op: bool = False) -> np.ndarray:
        """W_hat through the LDS-staged reconstruction, or (hash_op) through the per-weight comparator."""
        t = self.torch
        out = t.full((self.sk.in_features, self.sk.out_features), 0x7E00, dtype=t.int16, device=self.dev)
        ws, need = self.workspace(2, 0)
        call = skl.sketch_linear_reconstruct_hash_op if hash_op else skl.sketch_linear_reconstruct
        call(self.handle, out.data_ptr(), ws.data_ptr(), ws.numel(), self.stream())
        t.cuda.synchronize()
        return out.cpu().numpy().view(np.uint16)

    def gemv_partials(self, x_f16: np.ndarray) -> np.ndarray:
        """The partial sums the first gemv kernel leaves in the workspace, as float32 [n_units][batch][out]."""
        t = self.torch
        batch, in_f = x_f16.shape
        xd = t.from_numpy(np.ascontiguousarray(x_f16).view(np.int16)).to(self.dev)
        ws, need = self.workspace(0, batch)
        ws.zero_()
        skl.sketch_linear_gemv_partials(self.handle, xd.data_ptr(), skl.SKL_F16, in_f, batch, ws.data_ptr(),
                                        ws.numel(), self.stream())
        t.cuda.synchronize()
        n = self.info["n_units"] * batch * self.sk.out_features
        return ws[:4 * n].view(t.float32).cpu().numpy().reshape(self.info["n_units"], batch, self.sk.out_features)

    def gemv(self, x_f16: np.ndarray, y_dtype: str = "f32", ldx=None, ldy=None) -> np.ndarray:
        t = self.torch
        batch, in_f = x_f16.shape
        ldx = ldx or in_f
        ldy = ldy or self.sk.out_features
        xb = np.zeros((batch, ldx), dtype=np.float16)
        xb[:, :in_f] = x_f16
        xd = t.from_numpy(xb.view(np.int16)).to(self.dev)
        ydt = {"f32": t.float32, "f16": t.float16}[y_dtype]
        yd = t.full((batch, ldy), float("nan"), dtype=ydt, device=self.dev)
        ws, need = self.workspace(0, batch)
        skl.sketch_linear_gemv(self.handle, xd.data_ptr(), skl.SKL_F16, ldx, yd.data_ptr(), DT[y_dtype], ldy,
                               batch, ws.data_ptr(), ws.numel(), self.stream())
        t.cuda.synchronize()
        y = yd.cpu().numpy()
        if ldy > self.sk.out_features:
            assert np.all(np.isnan(y[:, self.sk.out_features:].astype(np.float32))), "wrote past out_features"
        return y[:, :self.sk.out_features]

    def gemm(self, X_bits: np.ndarray, x_dtype: str = "bf16", y_dtype: str = "f32", ldx=None, ldy=None) -> np.ndarray:
        t = self.torch
        tokens, in_f = X_bits.shape
        ldx = ldx or in_f
        ldy = ldy or self.sk.out_features
        xb = np.zeros((tokens, ldx), dtype=np.uint16)
        xb[:, :in_f] = X_bits
        xd = t.from_numpy(xb.view(np.int16)).to(self.dev)
        ydt = {"f32": t.float32, "f16": t.float16, "bf16": t.bfloat16}[y_dtype]
        yd = t.full((tokens, ldy), float("nan"), dtype=ydt, device=self.dev)
        ws, need = self.workspace(1, tokens)
        skl.sketch_linear_gemm(self.handle, xd.data_ptr(), DT[x_dtype], ldx, yd.data_ptr(), DT[y_dtype], ldy,
                               tokens, ws.data_ptr(), ws.numel(), self.stream())
        t.cuda.synchronize()
        y = yd.float().cpu().numpy() if y_dtype == "bf16" else yd.cpu().numpy()
        if ldy > self.sk.out_features:
            assert np.all(np.isnan(y[:, self.sk.out_features:].astype(np.float32))), "wrote past out_features"
        return y[:, :self.sk.out_features]


def rel_fro(got, ref) -> float:
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300))


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """fp64 -> float32 -> bfloat16 (nearest even) -> float64, to compare bf16
    outputs with the oracle rounded the same way."""
    return wk.bf16_bits_to_f32(wk.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))).astype(np.float64)


def build_states_on_gpu(W: np.ndarray, tile_in, tile_out, d, hash_a, hash_c, widths) -> np.ndarray:
    """Sketch states of W ([in][out] binary16) built by the library on cuda:0 (uint16 bit patterns)."""
    t = torch_mod()
    dev = t.device("cuda:0")
    in_f, out_f = W.shape
    wd = np.ascontiguousarray(widths, dtype=np.uint32).ravel()
    n_states = int(wd.sum()) * d
    desc = skl.make_desc(in_f, out_f, tile_in, tile_out, d, np.ascontiguousarray(hash_a, dtype=np.uint32),
                         np.ascontiguousarray(hash_c, dtype=np.uint32), wd, None, n_states=n_states)
    Wd = t.from_numpy(np.ascontiguousarray(W).view(np.int16)).to(dev)
    states = t.full((n_states,), 0x7E00, dtype=t.int16, device=dev)
    need = skl.sketch_linear_build_workspace_bytes(desc)
    ws = t.empty(need + 256, dtype=t.uint8, device=dev)
    off = (-ws.data_ptr()) % 256
    skl.sketch_linear_build_states(desc, Wd.data_ptr(), states.data_ptr(), ws.data_ptr() + off, need,
                                   t.cuda.current_stream().cuda_stream)
    return states.cpu().numpy().view(np.uint16)


def stratified_sample(tokens: int, out_features: int, seed: int, per_tile_rows: int = 3, per_tile_cols: int = 4, tile: int = 256):
    """Sorted rows and columns such that every tile x tile output tile holds per_tile_rows x per_tile_cols
    elements of the grid rows x cols (fewer in a ragged last tile that is narrower than that)."""
    rng = np.random.default_rng(seed)
    rows, cols = [], []
    for t0 in range(0, tokens, tile):
        n = min(tile, tokens - t0)
        rows += (t0 + rng.choice(n, size=min(per_tile_rows, n), replace=False)).tolist()
    for o0 in range(0, out_features, tile):
        n = min(tile, out_features - o0)
        cols += (o0 + rng.choice(n, size=min(per_tile_cols, n), replace=False)).tolist()
    return np.sort(np.array(rows)), np.sort(np.array(cols))


def matmul_f64(W_hat_bits: np.ndarray, X: np.ndarray, x_kind: str = "bf16") -> np.ndarray:
    """All outputs at once: numpy's binary64 matrix product of the oracle's reconstructed weights (a library
    routine on the oracle's W_hat; the oracle's own linear() is pinned against the same routine)."""
    Xf = wk.bf16_bits_to_f32(X).astype(np.float64) if x_kind == "bf16" else np.asarray(X, dtype=np.float16).astype(np.float64)
    return Xf @ W_hat_bits.view(np.float16).astype(np.float64)


def worst_tile_rel_fro(got, ref, tile: int = 256) -> float:
    """Largest relative Frobenius error over the tile x tile output tiles: one wrong tile cannot hide in the
    norm of the whole output."""
    got = np.asarray(got, dtype=np.float64)
    worst = 0.0
    for t0 in range(0, ref.shape[0], tile):
        for o0 in range(0, ref.shape[1], tile):
            r = ref[t0:t0 + tile, o0:o0 + tile]
            g = got[t0:t0 + tile, o0:o0 + tile]
            worst = max(worst, float(np.linalg.norm(g - r) / max(np.linalg.norm(r), 1e-300)))
    return worst


def oracle_stack_layer(index: int):
    """Worker for process pools (no GPU, no torch): the sketch of layer `index` of the Llama-2-7B-shaped
    stack from the oracle's update, a digest of the oracle's reconstructed weights and its batch-1 output."""
    import hashlib
    wl = wk.cfg5_stack(32)[index]
    W, sk = build_sketch(wl)
    W_hat = oracle.query(sk)
    y = oracle.linear(W_hat, wk.gen_x(wl, 1))
    return index, sk, hashlib.sha1(np.ascontiguousarray(W_hat).tobytes()).hexdigest(), y
