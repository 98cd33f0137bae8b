"""ctypes binding of libsketch_linear.so: argument marshalling only.

Every function has the name of the C entry point it calls (see
include/sketch_linear.h).  Device pointers and the HIP stream are plain
integers (``tensor.data_ptr()``, ``torch.cuda.current_stream().cuda_stream``);
this module imports neither torch nor numpy and holds no arithmetic of the
method.  If the library has not been built the import of the symbols fails
loudly: there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os

from .build import lib_path

SKL_OK = 0
SKL_ERR_INVALID_ARG = 1
SKL_ERR_UNSUPPORTED = 2
SKL_ERR_BUFFER_TOO_SMALL = 3
SKL_ERR_NONFINITE = 4
SKL_ERR_HIP = 5
SKL_ERR_NO_MEMORY = 6

SKL_F16, SKL_BF16, SKL_F32 = 0, 1, 2
FLAG_HASH_PER_WEIGHT = 1
FLAG_STAGED_PREFILL = 2
FLAG_FUSED_PREFILL = 4

STATUS_NAMES = {0: "SKL_OK", 1: "SKL_ERR_INVALID_ARG", 2: "SKL_ERR_UNSUPPORTED",
                3: "SKL_ERR_BUFFER_TOO_SMALL", 4: "SKL_ERR_NONFINITE", 5: "SKL_ERR_HIP",
                6: "SKL_ERR_NO_MEMORY"}

# skl_info_t.prefill_kernel
SKL_PREFILL_PER_WEIGHT, SKL_PREFILL_FUSED, SKL_PREFILL_STAGED = 0, 3, 4

EXPORTS = ("sketch_linear_device_bytes", "sketch_linear_create", "sketch_linear_info",
           "sketch_linear_workspace_bytes", "sketch_linear_gemv", "sketch_linear_gemm",
           "sketch_linear_reconstruct", "sketch_linear_gemv_partials", "sketch_linear_prefill_split",
           "sketch_linear_build_workspace_bytes", "sketch_linear_build_states",
           "sketch_linear_gemv_group_workspace_bytes", "sketch_linear_gemv_group", "sketch_linear_gemv_gate_up",
           "sketch_linear_plan", "sketch_linear_gemv_static", "sketch_linear_reconstruct_hash_op", "sketch_linear_microbench",
           "sketch_linear_file_bytes", "sketch_linear_file_write", "sketch_linear_file_save", "sketch_linear_file_open",
           "sketch_linear_debug_violations", "sketch_linear_debug_selftest",
           "sketch_linear_destroy", "sketch_linear_last_error")


class SketchLinearError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {message}")
        self.status = status
        self.message = message


class skl_desc_t(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_uint32), ("in_features", ctypes.c_uint32),
                ("out_features", ctypes.c_uint32), ("tile_in", ctypes.c_uint32),
                ("tile_out", ctypes.c_uint32), ("d", ctypes.c_uint32),
                ("query_mode", ctypes.c_uint32), ("flags", ctypes.c_uint32),
                ("hash_a", ctypes.c_void_p), ("hash_c", ctypes.c_void_p),
                ("group_width", ctypes.c_void_p), ("states", ctypes.c_void_p),
                ("n_states", ctypes.c_uint64),
                # end of the first version of the struct (SKL_DESC_SIZE_V1 bytes)
                ("state_bits", ctypes.c_uint32), ("reserved", ctypes.c_uint32),
                ("codes", ctypes.c_void_p), ("scales", ctypes.c_void_p)]


SKL_DESC_SIZE_V1 = 72
SKL_STATIC_SCRATCH_MAX = 16 << 20     # bytes of the device array behind sketch_linear_gemv_static


class skl_info_t(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_uint32), ("path", ctypes.c_uint32),
                ("n_units", ctypes.c_uint32), ("max_table_bytes", ctypes.c_uint32),
                ("table_bytes", ctypes.c_uint64), ("n_weights", ctypes.c_uint64),
                ("n_states", ctypes.c_uint64),
                # end of the first version of the struct (SKL_INFO_SIZE_V1 bytes)
                ("decode_segments", ctypes.c_uint32), ("decode_groups", ctypes.c_uint32),
                ("block_classes", ctypes.c_uint32), ("prefill_kernel", ctypes.c_uint32),
                ("n_blocks", ctypes.c_uint32), ("prefill_staged_from", ctypes.c_uint32)]


SKL_INFO_SIZE_V1 = 40

_lib = None


def load_library(path: str | None = None):
    """Load the built library; raises if it is missing (build it first with
    ``python -m paper_2506_17255_amd.build`` or ``__graft_entry__.build()``)."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is not built; run __graft_entry__.build() first "
                          "(there is no CPU fallback for the sketch-linear kernels)")
    L = ctypes.CDLL(path)
    vp, u32, u64 = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64
    L.sketch_linear_device_bytes.argtypes = [ctypes.POINTER(skl_desc_t), ctypes.POINTER(u64)]
    L.sketch_linear_create.argtypes = [ctypes.POINTER(skl_desc_t), vp, u64, vp, ctypes.POINTER(vp)]
    L.sketch_linear_info.argtypes = [vp, ctypes.POINTER(skl_info_t)]
    L.sketch_linear_plan.argtypes = [ctypes.POINTER(skl_desc_t), u32, u32, ctypes.POINTER(skl_info_t), ctypes.POINTER(ctypes.c_double)]
    L.sketch_linear_workspace_bytes.argtypes = [vp, u32, u32, ctypes.POINTER(u64)]
    L.sketch_linear_gemv.argtypes = [vp, vp, ctypes.c_int, u32, vp, ctypes.c_int, u32, u32, vp, u64, vp]
    L.sketch_linear_gemm.argtypes = [vp, vp, ctypes.c_int, u32, vp, ctypes.c_int, u32, u32, vp, u64, vp]
    L.sketch_linear_reconstruct.argtypes = [vp, vp, vp, u64, vp]
    L.sketch_linear_reconstruct_hash_op.argtypes = [vp, vp, vp, u64, vp]
    L.sketch_linear_microbench.argtypes = [u32, u32, vp, u64, vp, ctypes.POINTER(u64)]
    L.sketch_linear_gemv_partials.argtypes = [vp, vp, ctypes.c_int, u32, u32, vp, u64, vp]
    L.sketch_linear_prefill_split.argtypes = [u32, u32, u32, u32, ctypes.POINTER(u32), u64, ctypes.POINTER(u64),
                                              ctypes.POINTER(u32)]
    L.sketch_linear_build_workspace_bytes.argtypes = [ctypes.POINTER(skl_desc_t), ctypes.POINTER(u64)]
    L.sketch_linear_build_states.argtypes = [ctypes.POINTER(skl_desc_t), vp, vp, vp, u64, vp]
    L.sketch_linear_gemv_group_workspace_bytes.argtypes = [ctypes.POINTER(vp), u32, u32, ctypes.POINTER(u64)]
    L.sketch_linear_gemv_group.argtypes = [ctypes.POINTER(vp), u32, vp, ctypes.c_int, u32, ctypes.POINTER(vp), ctypes.c_int, u32,
                                           u32, vp, u64, vp]
    L.sketch_linear_gemv_gate_up.argtypes = [vp, vp, vp, ctypes.c_int, u32, vp, ctypes.c_int, u32, u32, vp, u64, vp]
    L.sketch_linear_destroy.argtypes = [vp]
    L.sketch_linear_destroy.restype = None
    L.sketch_linear_last_error.argtypes = []
    L.sketch_linear_last_error.restype = ctypes.c_char_p
    L.sketch_linear_gemv_static.argtypes = [vp, vp, ctypes.c_int, u32, vp, ctypes.c_int, u32, u32, vp]
    for n in EXPORTS[:-2]:
        getattr(L, n).restype = ctypes.c_int
    _lib = L
    return L


def sketch_linear_last_error() -> str:
    return load_library().sketch_linear_last_error().decode()


def _check(status: int):
    if status != SKL_OK:
        raise SketchLinearError(status, sketch_linear_last_error())


def make_desc(in_features, out_features, tile_in, tile_out, d, hash_a, hash_c, group_width, states,
              n_states=None, query_mode=0, flags=0, struct_size=None, state_bits=0, codes=None, scales=None):
    """Build a skl_desc_t from host arrays.  ``hash_a``, ``hash_c``,
    ``group_width`` (uint32) and ``states`` (uint16) are objects exposing the
    buffer protocol with those element types, or None; the returned
    descriptor keeps them alive.  Low-bit states: ``state_bits`` 8 or 4,
    ``codes`` (bytes: int8 per state, or packed nibbles) and ``scales``
    (uint16), ``states`` None and ``n_states`` given."""
    desc = skl_desc_t()
    desc.struct_size = ctypes.sizeof(skl_desc_t) if struct_size is None else struct_size
    desc.in_features, desc.out_features = in_features, out_features
    desc.tile_in, desc.tile_out, desc.d = tile_in, tile_out, d
    desc.query_mode, desc.flags = query_mode, flags
    keep = []

    def ptr(buf, itemsize):
        if buf is None:
            return None
        mv = memoryview(buf)
        if not mv.c_contiguous or mv.itemsize != itemsize:
            raise TypeError("descriptor arrays must be contiguous with the documented element size")
        keep.append(buf)
        if mv.nbytes == 0:
            return None
        arr = (ctypes.c_char * mv.nbytes).from_buffer_copy(mv) if mv.readonly else (ctypes.c_char * mv.nbytes).from_buffer(mv)
        keep.append(arr)
        return ctypes.cast(arr, ctypes.c_void_p).value

    desc.hash_a = ptr(hash_a, 4)
    desc.hash_c = ptr(hash_c, 4)
    desc.group_width = ptr(group_width, 4)
    desc.states = ptr(states, 2)
    desc.state_bits = state_bits
    desc.codes = ptr(codes, 1)
    desc.scales = ptr(scales, 2)
    if n_states is None:
        n_states = 0 if states is None else memoryview(states).nbytes // 2
    desc.n_states = n_states
    desc._keep = keep
    return desc


def sketch_linear_device_bytes(desc: skl_desc_t) -> int:
    n = ctypes.c_uint64(0)
    _check(load_library().sketch_linear_device_bytes(ctypes.byref(desc) if desc is not None else None, ctypes.byref(n)))
    return n.value


def sketch_linear_create(desc: skl_desc_t, dev_buf: int, dev_bytes: int, hip_stream: int = 0) -> int:
    """Returns the opaque layer handle (an integer address)."""
    h = ctypes.c_void_p(None)
    _check(load_library().sketch_linear_create(ctypes.byref(desc) if desc is not None else None, dev_buf, dev_bytes,
                                               hip_stream, ctypes.byref(h)))
    return h.value


def sketch_linear_info(layer: int) -> dict:
    info = skl_info_t()
    info.struct_size = ctypes.sizeof(skl_info_t)
    _check(load_library().sketch_linear_info(layer, ctypes.byref(info)))
    return {n: getattr(info, n) for n, _ in skl_info_t._fields_ if n != "struct_size"}


def sketch_linear_plan(desc: skl_desc_t, segments: int = 0, groups: int = 0):
    """Host only.  (info dict, decode cost in microseconds by the planner's model) for the library's plan, or
    for the decode split (segments, groups) if given."""
    info = skl_info_t()
    info.struct_size = ctypes.sizeof(skl_info_t)
    cost = ctypes.c_double(0.0)
    _check(load_library().sketch_linear_plan(ctypes.byref(desc), segments, groups, ctypes.byref(info), ctypes.byref(cost)))
    return {n: getattr(info, n) for n, _ in skl_info_t._fields_ if n != "struct_size"}, cost.value


def sketch_linear_workspace_bytes(layer: int, op: int, n: int) -> int:
    b = ctypes.c_uint64(0)
    _check(load_library().sketch_linear_workspace_bytes(layer, op, n, ctypes.byref(b)))
    return b.value


def sketch_linear_gemv(layer: int, x: int, x_dtype: int, ldx: int, y: int, y_dtype: int, ldy: int, batch: int,
                       workspace: int, workspace_bytes: int, hip_stream: int = 0) -> None:
    _check(load_library().sketch_linear_gemv(layer, x, x_dtype, ldx, y, y_dtype, ldy, batch, workspace,
                                             workspace_bytes, hip_stream))


def sketch_linear_gemv_static(layer: int, x: int, x_dtype: int, ldx: int, y: int, y_dtype: int, ldy: int, batch: int,
                              hip_stream: int = 0) -> None:
    _check(load_library().sketch_linear_gemv_static(layer, x, x_dtype, ldx, y, y_dtype, ldy, batch, hip_stream))


def sketch_linear_gemm(layer: int, X: int, x_dtype: int, ldx: int, Y: int, y_dtype: int, ldy: int, tokens: int,
                       workspace: int, workspace_bytes: int, hip_stream: int = 0) -> None:
    _check(load_library().sketch_linear_gemm(layer, X, x_dtype, ldx, Y, y_dtype, ldy, tokens, workspace,
                                             workspace_bytes, hip_stream))


def sketch_linear_gemv_partials(layer: int, x: int, x_dtype: int, ldx: int, batch: int, workspace: int,
                                workspace_bytes: int, hip_stream: int = 0) -> None:
    _check(load_library().sketch_linear_gemv_partials(layer, x, x_dtype, ldx, batch, workspace, workspace_bytes,
                                                      hip_stream))


def sketch_linear_prefill_split(out_features: int, n_blocks: int, tokens: int, kernel: int = SKL_PREFILL_FUSED):
    """Host only.  Returns (segments, shape): segments is a list of 8-tuples (xcd, workgroup, token tile,
    output tile, first block, end block, whole, slot), shape is (workgroups per XCD, partial tiles per XCD,
    slots per partial tile, tiles, token tiles per dealing unit, tokens per tile)."""
    L = load_library()
    n = ctypes.c_uint64(0)
    shape = (ctypes.c_uint32 * 6)()
    _check(L.sketch_linear_prefill_split(kernel, out_features, n_blocks, tokens, None, 0, ctypes.byref(n), shape))
    buf = (ctypes.c_uint32 * (8 * max(n.value, 1)))()
    _check(L.sketch_linear_prefill_split(kernel, out_features, n_blocks, tokens, buf, n.value, ctypes.byref(n), shape))
    segs = [tuple(buf[8 * i:8 * i + 8]) for i in range(n.value)]
    return segs, tuple(shape)


def _ptr_array(values):
    return (ctypes.c_void_p * len(values))(*values)


def sketch_linear_gemv_group_workspace_bytes(layers, batch: int = 1) -> int:
    n = ctypes.c_uint64(0)
    _check(load_library().sketch_linear_gemv_group_workspace_bytes(_ptr_array(layers), len(layers), batch, ctypes.byref(n)))
    return n.value


def sketch_linear_gemv_group(layers, x: int, x_dtype: int, ldx: int, ys, y_dtype: int, ldy: int, batch: int, workspace: int,
                             workspace_bytes: int, hip_stream: int = 0) -> None:
    """``layers``: handles; ``ys``: device addresses of the outputs ([batch][ldy] each), one per layer."""
    _check(load_library().sketch_linear_gemv_group(_ptr_array(layers), len(layers), x, x_dtype, ldx, _ptr_array(ys), y_dtype,
                                                   ldy, batch, workspace, workspace_bytes, hip_stream))


def sketch_linear_gemv_gate_up(gate: int, up: int, x: int, x_dtype: int, ldx: int, h: int, h_dtype: int, ldh: int, batch: int,
                               workspace: int, workspace_bytes: int, hip_stream: int = 0) -> None:
    _check(load_library().sketch_linear_gemv_gate_up(gate, up, x, x_dtype, ldx, h, h_dtype, ldh, batch, workspace,
                                                     workspace_bytes, hip_stream))


def sketch_linear_build_workspace_bytes(desc: skl_desc_t) -> int:
    n = ctypes.c_uint64(0)
    _check(load_library().sketch_linear_build_workspace_bytes(ctypes.byref(desc), ctypes.byref(n)))
    return n.value


def sketch_linear_build_states(desc: skl_desc_t, W_dev: int, states_dev: int, workspace: int, workspace_bytes: int,
                               hip_stream: int = 0) -> None:
    _check(load_library().sketch_linear_build_states(ctypes.byref(desc), W_dev, states_dev, workspace, workspace_bytes,
                                                     hip_stream))


def sketch_linear_reconstruct(layer: int, W_hat_dev: int, workspace: int = 0, workspace_bytes: int = 0,
                              hip_stream: int = 0) -> None:
    _check(load_library().sketch_linear_reconstruct(layer, W_hat_dev, workspace, workspace_bytes, hip_stream))


def sketch_linear_reconstruct_hash_op(layer: int, W_hat_dev: int, workspace: int = 0, workspace_bytes: int = 0,
                                      hip_stream: int = 0) -> None:
    _check(load_library().sketch_linear_reconstruct_hash_op(layer, W_hat_dev, workspace, workspace_bytes, hip_stream))


def sketch_linear_microbench(kind: int, iters: int, workspace: int, workspace_bytes: int, hip_stream: int = 0) -> int:
    """Enqueues one ceiling kernel; returns the work it does (lane-instructions, bytes or flops)."""
    work = ctypes.c_uint64(0)
    _check(load_library().sketch_linear_microbench(kind, iters, workspace, workspace_bytes, hip_stream, ctypes.byref(work)))
    return work.value


def sketch_linear_file_bytes(desc: skl_desc_t) -> int:
    n = ctypes.c_uint64(0)
    _check(load_library().sketch_linear_file_bytes(ctypes.byref(desc), ctypes.byref(n)))
    return n.value


def sketch_linear_file_write(desc: skl_desc_t, image) -> None:
    """Writes the layer file of ``desc`` into ``image`` (a writable object with the buffer protocol)."""
    mv = memoryview(image)
    buf = (ctypes.c_char * mv.nbytes).from_buffer(mv)
    _check(load_library().sketch_linear_file_write(ctypes.byref(desc), buf, mv.nbytes))


def sketch_linear_file_save(desc: skl_desc_t, path: str) -> None:
    _check(load_library().sketch_linear_file_save(ctypes.byref(desc), os.fsencode(path)))


def sketch_linear_file_open(image) -> skl_desc_t:
    """The description held by a layer file image (a writable, 8-byte aligned object with the buffer
    protocol: a bytearray, a numpy array, a writable memory map).  The description points into the image
    and keeps it alive."""
    mv = memoryview(image)
    buf = (ctypes.c_char * mv.nbytes).from_buffer(mv)
    desc = skl_desc_t()
    _check(load_library().sketch_linear_file_open(buf, mv.nbytes, ctypes.byref(desc)))
    desc._keep = [image, buf]
    return desc


def sketch_linear_debug_selftest(value: int, limit: int, hip_stream: int = 0) -> None:
    _check(load_library().sketch_linear_debug_selftest(value, limit, hip_stream))


def sketch_linear_debug_violations():
    """(count, first) of the range asserts of the debug build; raises SKL_ERR_UNSUPPORTED in the normal build."""
    count = ctypes.c_uint64(0)
    first = (ctypes.c_uint32 * 5)()
    _check(load_library().sketch_linear_debug_violations(ctypes.byref(count), first))
    return count.value, dict(zip(("code", "value", "limit", "workgroup", "thread"), first))


def sketch_linear_destroy(layer: int) -> None:
    load_library().sketch_linear_destroy(layer)
