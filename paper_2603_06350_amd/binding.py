"""ctypes binding of libmoe_gfx950.so: the same calls as include/moe.h.

Argument marshalling only: tensors are passed as device pointers, every step of
the layer runs in the library's HIP kernels.  There is no CPU fallback; loading
fails loudly if the library has not been built (python -m paper_2603_06350_amd.build).
"""
from __future__ import annotations

import ctypes
import os

MOE_F32 = 0
MOE_BF16 = 1

# MOE_GFX950_LIB points the binding at another build of the same library (same C ABI).
_LIB_PATH = os.environ.get("MOE_GFX950_LIB") or os.path.join(
    os.path.dirname(os.path.abspath(__file__)), "libmoe_gfx950.so")
_lib = None

EXPORTS = ("moe_workspace_bytes", "moe_route", "moe_route_ws", "moe_count_and_permute",
           "moe_count_and_permute_static", "moe_grouped_ffn",
           "moe_grouped_ffn_part", "moe_grouped_ffn_gather",
           "moe_grouped_ffn_gather_part", "moe_grouped_ffn_combine_k1", "moe_ffn_workspace_bytes", "moe_grouped_ffn_ws", "moe_combine", "moe_scale_replicas", "moe_replica_segments",
           "moe_place_replicas",
           "moe_strerror")
MOE_MAX_EXTRA_REPLICAS = 65536
MOE_STATIC_SCRATCH_BYTES = 1 << 20


class MoeShape(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int32), ("d", ctypes.c_int32), ("E", ctypes.c_int32),
                ("k", ctypes.c_int32), ("F", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("renorm", ctypes.c_int32)]


class MoeError(RuntimeError):
    def __init__(self, call, code):
        self.code = code
        super().__init__(f"{call} failed: {code} ({strerror(code)})")


def lib_path() -> str:
    return _LIB_PATH


def load():
    """Loads the shared library (once).  Raises if it is missing: no fallback path exists."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} not built; run `python -m paper_2603_06350_amd.build`")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32p, f32p = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p
    shp = ctypes.POINTER(MoeShape)
    lib.moe_workspace_bytes.argtypes = [shp, ctypes.POINTER(ctypes.c_size_t)]
    lib.moe_route.argtypes = [shp, vp, vp, f32p, i32p, f32p, f32p, vp]
    lib.moe_route_ws.argtypes = [shp, vp, vp, f32p, i32p, f32p, f32p, vp, ctypes.c_size_t, vp]
    lib.moe_count_and_permute.argtypes = [shp, vp, i32p, i32p, i32p, i32p, i32p, vp, vp,
                                          ctypes.c_size_t, vp]
    lib.moe_count_and_permute_static.argtypes = [shp, vp, i32p, i32p, i32p, i32p, i32p, vp, vp]
    lib.moe_grouped_ffn.argtypes = [shp, vp, i32p, vp, vp, vp, vp, vp, vp]
    lib.moe_grouped_ffn_part.argtypes = [shp, vp, i32p, vp, vp, vp, vp, vp, ctypes.c_int, vp]
    lib.moe_grouped_ffn_gather.argtypes = [shp, vp, i32p, i32p, vp, vp, vp, vp, vp, vp]
    lib.moe_grouped_ffn_gather_part.argtypes = [shp, vp, i32p, i32p, vp, vp, vp, vp, vp,
                                                ctypes.c_int, vp]
    lib.moe_grouped_ffn_combine_k1.argtypes = [shp, vp, i32p, i32p, vp, vp, vp, f32p, vp, vp, vp]
    lib.moe_ffn_workspace_bytes.argtypes = [shp, ctypes.POINTER(ctypes.c_size_t)]
    lib.moe_grouped_ffn_ws.argtypes = [shp, vp, i32p, i32p, vp, vp, vp, vp, vp, ctypes.c_int, vp,
                                       ctypes.c_size_t, vp]
    lib.moe_combine.argtypes = [shp, vp, i32p, f32p, vp, vp]
    lib.moe_scale_replicas.argtypes = [ctypes.c_int32, i32p, ctypes.c_int64, ctypes.c_int64,
                                       ctypes.c_double, i32p, vp, vp]
    lib.moe_replica_segments.argtypes = [ctypes.c_int32, i32p, i32p, ctypes.c_int32, i32p, i32p,
                                         i32p, vp]
    lib.moe_place_replicas.argtypes = [ctypes.c_int32, i32p, i32p, ctypes.c_int32, i32p, i32p, i32p,
                                       ctypes.c_int32, i32p, vp, i32p, i32p, vp]
    lib.moe_strerror.argtypes = [ctypes.c_int]
    lib.moe_strerror.restype = ctypes.c_char_p
    for name in EXPORTS[:-1]:
        getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def _ptr(t):
    """Device pointer of a tensor-like (anything with data_ptr()), an int, or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        return None
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def make_shape(T, d, E, k, F, dtype, renorm) -> MoeShape:
    return MoeShape(int(T), int(d), int(E), int(k), int(F), int(dtype), int(renorm))


def strerror(code: int) -> str:
    return load().moe_strerror(int(code)).decode()


def _check(call, rc):
    if rc != 0:
        raise MoeError(call, rc)


def moe_workspace_bytes(shape: MoeShape) -> int:
    out = ctypes.c_size_t(0)
    _check("moe_workspace_bytes", load().moe_workspace_bytes(ctypes.byref(shape), ctypes.byref(out)))
    return int(out.value)


def moe_route(shape, x, w_gate, gate_bias, topk_idx, topk_w, scores_out=None, stream=None):
    _check("moe_route", load().moe_route(ctypes.byref(shape), _ptr(x), _ptr(w_gate), _ptr(gate_bias),
                                         _ptr(topk_idx), _ptr(topk_w), _ptr(scores_out),
                                         _stream(stream)))


def moe_route_ws(shape, x, w_gate, gate_bias, topk_idx, topk_w, scores_out, workspace,
                 workspace_bytes, stream=None):
    _check("moe_route_ws",
           load().moe_route_ws(ctypes.byref(shape), _ptr(x), _ptr(w_gate), _ptr(gate_bias),
                               _ptr(topk_idx), _ptr(topk_w), _ptr(scores_out), _ptr(workspace),
                               ctypes.c_size_t(int(workspace_bytes)), _stream(stream)))


def moe_count_and_permute(shape, x, topk_idx, counts, offsets, dst_row, src_assign, x_perm,
                          workspace, workspace_bytes, stream=None):
    _check("moe_count_and_permute",
           load().moe_count_and_permute(ctypes.byref(shape), _ptr(x), _ptr(topk_idx), _ptr(counts),
                                        _ptr(offsets), _ptr(dst_row), _ptr(src_assign),
                                        _ptr(x_perm), _ptr(workspace),
                                        ctypes.c_size_t(int(workspace_bytes)), _stream(stream)))


def moe_count_and_permute_static(shape, x, topk_idx, counts, offsets, dst_row, src_assign, x_perm,
                                 stream=None):
    _check("moe_count_and_permute_static",
           load().moe_count_and_permute_static(ctypes.byref(shape), _ptr(x), _ptr(topk_idx),
                                               _ptr(counts), _ptr(offsets), _ptr(dst_row),
                                               _ptr(src_assign), _ptr(x_perm), _stream(stream)))


def moe_grouped_ffn(shape, x_perm, offsets, w1, w3, w2, h, y_perm, stream=None):
    _check("moe_grouped_ffn",
           load().moe_grouped_ffn(ctypes.byref(shape), _ptr(x_perm), _ptr(offsets), _ptr(w1),
                                  _ptr(w3), _ptr(w2), _ptr(h), _ptr(y_perm), _stream(stream)))


def moe_grouped_ffn_part(shape, x_perm, offsets, w1, w3, w2, h, y_perm, part, stream=None):
    _check("moe_grouped_ffn_part",
           load().moe_grouped_ffn_part(ctypes.byref(shape), _ptr(x_perm), _ptr(offsets), _ptr(w1),
                                       _ptr(w3), _ptr(w2), _ptr(h), _ptr(y_perm), int(part),
                                       _stream(stream)))


def moe_grouped_ffn_gather(shape, x, src_assign, offsets, w1, w3, w2, h, y_perm, stream=None):
    _check("moe_grouped_ffn_gather",
           load().moe_grouped_ffn_gather(ctypes.byref(shape), _ptr(x), _ptr(src_assign),
                                         _ptr(offsets), _ptr(w1), _ptr(w3), _ptr(w2), _ptr(h),
                                         _ptr(y_perm), _stream(stream)))


def moe_grouped_ffn_gather_part(shape, x, src_assign, offsets, w1, w3, w2, h, y_perm, part,
                                stream=None):
    _check("moe_grouped_ffn_gather_part",
           load().moe_grouped_ffn_gather_part(ctypes.byref(shape), _ptr(x), _ptr(src_assign),
                                              _ptr(offsets), _ptr(w1), _ptr(w3), _ptr(w2), _ptr(h),
                                              _ptr(y_perm), int(part), _stream(stream)))


def moe_grouped_ffn_combine_k1(shape, x, src_assign, offsets, w1, w3, w2, topk_w, h, y, stream=None):
    _check("moe_grouped_ffn_combine_k1",
           load().moe_grouped_ffn_combine_k1(ctypes.byref(shape), _ptr(x), _ptr(src_assign),
                                             _ptr(offsets), _ptr(w1), _ptr(w3), _ptr(w2), _ptr(topk_w),
                                             _ptr(h), _ptr(y), _stream(stream)))


def moe_ffn_workspace_bytes(shape: MoeShape) -> int:
    out = ctypes.c_size_t(0)
    _check("moe_ffn_workspace_bytes",
           load().moe_ffn_workspace_bytes(ctypes.byref(shape), ctypes.byref(out)))
    return int(out.value)


def moe_grouped_ffn_ws(shape, x, src_assign, offsets, w1, w3, w2, h, y_perm, parts, workspace,
                       workspace_bytes, stream=None):
    _check("moe_grouped_ffn_ws",
           load().moe_grouped_ffn_ws(ctypes.byref(shape), _ptr(x), _ptr(src_assign), _ptr(offsets),
                                     _ptr(w1), _ptr(w3), _ptr(w2), _ptr(h), _ptr(y_perm), int(parts),
                                     _ptr(workspace), int(workspace_bytes), _stream(stream)))


def moe_combine(shape, y_perm, dst_row, topk_w, y, stream=None):
    _check("moe_combine", load().moe_combine(ctypes.byref(shape), _ptr(y_perm), _ptr(dst_row),
                                             _ptr(topk_w), _ptr(y), _stream(stream)))


def moe_scale_replicas(E, loads, expert_mem, mem_cap, cv_threshold, replicas, cv_out=None, stream=None):
    _check("moe_scale_replicas",
           load().moe_scale_replicas(int(E), _ptr(loads), int(expert_mem), int(mem_cap),
                                     float(cv_threshold), _ptr(replicas), _ptr(cv_out),
                                     _stream(stream)))


def moe_replica_segments(E, offsets, replicas, max_segments, seg_offsets, seg_expert, n_segments,
                         stream=None):
    _check("moe_replica_segments",
           load().moe_replica_segments(int(E), _ptr(offsets), _ptr(replicas), int(max_segments),
                                       _ptr(seg_offsets), _ptr(seg_expert), _ptr(n_segments),
                                       _stream(stream)))


def moe_place_replicas(E, loads, replicas, n_gpus, prev_replicas, prev_gpu, gpu_slots, max_segments,
                       gpu_of, gpu_load, gpu_count, n_warm, stream=None):
    _check("moe_place_replicas",
           load().moe_place_replicas(int(E), _ptr(loads), _ptr(replicas), int(n_gpus),
                                     _ptr(prev_replicas), _ptr(prev_gpu), _ptr(gpu_slots),
                                     int(max_segments), _ptr(gpu_of), _ptr(gpu_load),
                                     _ptr(gpu_count), _ptr(n_warm), _stream(stream)))
