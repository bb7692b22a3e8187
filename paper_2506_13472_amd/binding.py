"""ctypes binding of librosaq.so: argument marshalling only.

Names mirror the C ABI in include/rosaq.h.  Device buffers are plain integer
addresses (e.g. torch.Tensor.data_ptr()); host arrays are numpy arrays.  Nothing
here computes: if the shared library is missing the import of this module's
`lib()` fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

Q_NONE, Q_FULL, Q_HEADWISE = 0, 1, 2
SELECT_TOP, SELECT_TOP_PER_HEAD, SELECT_BOTTOM, SELECT_CONSECUTIVE, SELECT_TOP_AND_BOTTOM = range(5)

ERR_NAMES = {0: "OK", -1: "NULL", -2: "SHAPE", -3: "ARG", -4: "MODE", -5: "ALIGN",
             -6: "WORKSPACE", -7: "NONFINITE", -8: "HIP", -9: "NOMEM", -10: "HOSTONLY",
             -11: "NOCONVERGE"}

LIB_PATH = os.environ.get("ROSAQ_LIB") or os.path.join(os.path.dirname(os.path.abspath(__file__)), "librosaq.so")

EXPORTED = ["rosaq_pack_weights", "rosaq_workspace_bytes", "rosaq_workspace_bytes_batch", "rosaq_workspace_bytes_min", "rosaq_linear", "rosaq_linear_headwise",
            "rosaq_linear_headwise_static", "rosaq_linear_batch", "rosaq_linear_swiglu", "rosaq_mlp_swiglu", "rosaq_workspace_bytes_mlp", "rosaq_stream_probe", "rosaq_packed_clone", "rosaq_pca_headwise", "rosaq_pca_full",
            "rosaq_packed_info", "rosaq_packed_export", "rosaq_tune", "rosaq_launch_shape", "rosaq_block_map", "rosaq_packed_image", "rosaq_free",
            "rosaq_last_error"]


class PackDesc(C.Structure):
    _fields_ = [("out_features", C.c_int32), ("in_features", C.c_int32),
                ("W", C.c_void_p), ("ldw", C.c_int64),
                ("q_mode", C.c_int32), ("head_dim", C.c_int32),
                ("Q", C.c_void_p), ("eigenvalues", C.c_void_p),
                ("K", C.c_int32), ("bits", C.c_int32), ("group", C.c_int32),
                ("select_rule", C.c_int32), ("host_only", C.c_int32), ("select_arg", C.c_int32),
                ("rotation_absorbed", C.c_int32)]


class RosaqError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"rosaq error {ERR_NAMES.get(code, code)} ({code}): {text}")
        self.code = code


_lib = None


def lib() -> C.CDLL:
    """The loaded shared library (built in-tree by paper_2506_13472_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built: run `python -m paper_2506_13472_amd.build`")
        try:
            # PyTorch ships its own HIP runtime (same soname); load it first so the
            # process holds one runtime and streams / pointers are interchangeable.
            import torch  # noqa: F401
        except ImportError:
            pass
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
        L.rosaq_pack_weights.argtypes = [C.POINTER(PackDesc), vp, C.POINTER(vp)]
        L.rosaq_pack_weights.restype = C.c_int
        L.rosaq_packed_clone.argtypes = [vp, vp, C.POINTER(vp)]
        L.rosaq_packed_clone.restype = C.c_int
        L.rosaq_workspace_bytes.argtypes = [vp, i32]
        L.rosaq_workspace_bytes.restype = sz
        L.rosaq_workspace_bytes_min.argtypes = [vp, i32]
        L.rosaq_workspace_bytes_min.restype = sz
        L.rosaq_workspace_bytes_batch.argtypes = [C.POINTER(vp), i32, i32]
        L.rosaq_workspace_bytes_batch.restype = sz
        for f in (L.rosaq_linear, L.rosaq_linear_headwise):
            f.argtypes = [vp, vp, i32, i64, vp, i64, vp, sz, vp]
            f.restype = C.c_int
        L.rosaq_linear_headwise_static.argtypes = [vp, vp, i32, i64, vp, i64, vp]
        L.rosaq_linear_headwise_static.restype = C.c_int
        L.rosaq_linear_batch.argtypes = [C.POINTER(vp), i32, vp, i32, i64, C.POINTER(vp),
                                         C.POINTER(i64), vp, sz, vp]
        L.rosaq_linear_batch.restype = C.c_int
        L.rosaq_linear_swiglu.argtypes = [vp, vp, vp, i32, i64, vp, i64, vp, sz, vp]
        L.rosaq_linear_swiglu.restype = C.c_int
        L.rosaq_mlp_swiglu.argtypes = [vp, vp, vp, vp, i32, i64, vp, i64, vp, sz, vp]
        L.rosaq_mlp_swiglu.restype = C.c_int
        L.rosaq_workspace_bytes_mlp.argtypes = [vp, vp, vp, i32]
        L.rosaq_workspace_bytes_mlp.restype = sz
        L.rosaq_pca_headwise.argtypes = [vp, i32, i32, i64, vp, vp, vp]
        L.rosaq_pca_headwise.restype = C.c_int
        L.rosaq_pca_full.argtypes = [vp, i32, i32, i64, vp, vp, vp]
        L.rosaq_pca_full.restype = C.c_int
        L.rosaq_stream_probe.argtypes = [vp, sz, vp, sz, sz, i32, i32, vp, sz, vp]
        L.rosaq_stream_probe.restype = C.c_int
        L.rosaq_packed_info.argtypes = [vp] + [C.POINTER(i32)] * 6 + [C.POINTER(sz)]
        L.rosaq_packed_info.restype = C.c_int
        L.rosaq_packed_export.argtypes = [vp, vp, vp, vp, vp, vp]
        L.rosaq_packed_export.restype = C.c_int
        L.rosaq_tune.argtypes = [C.c_char_p, i32]
        L.rosaq_tune.restype = C.c_int
        L.rosaq_launch_shape.argtypes = [i32, i32, i32, i32, C.POINTER(i32)]
        L.rosaq_launch_shape.restype = C.c_int
        L.rosaq_packed_image.argtypes = [vp, i32, vp, C.POINTER(sz)]
        L.rosaq_packed_image.restype = C.c_int
        L.rosaq_block_map.argtypes = [i32, i32, i32, C.POINTER(i32), C.POINTER(i32)]
        L.rosaq_block_map.restype = C.c_int
        L.rosaq_free.argtypes = [vp]
        L.rosaq_free.restype = None
        L.rosaq_last_error.argtypes = []
        L.rosaq_last_error.restype = C.c_char_p
        _lib = L
    return _lib


def rosaq_last_error() -> str:
    return lib().rosaq_last_error().decode()


def _check(rc: int):
    if rc != 0:
        raise RosaqError(rc, rosaq_last_error())


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


class Packed:
    """Owner of one rosaq_packed_t handle."""

    def __init__(self, handle: int):
        self.handle = C.c_void_p(handle)
        n, d, k, b, g, m = (C.c_int32() for _ in range(6))
        dev = C.c_size_t()
        _check(lib().rosaq_packed_info(self.handle, n, d, k, b, g, m, dev))
        self.N, self.D, self.K, self.bits, self.group, self.q_mode = (v.value for v in (n, d, k, b, g, m))
        self.device_bytes = dev.value

    def free(self):
        if self.handle:
            lib().rosaq_free(self.handle)
            self.handle = C.c_void_p(None)

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def rosaq_pack_weights(W: np.ndarray, Q, eigenvalues: np.ndarray, K: int, bits: int, q_mode: int,
                       group: int = 128, head_dim: int = 128, select_rule: int = 0, select_arg: int = 0, rotation_absorbed: bool = False,
                       host_only: bool = False, stream: int = 0, ldw: int | None = None,
                       out_features: int | None = None, in_features: int | None = None) -> Packed:
    """W fp16 [N, D]; Q fp32 ([D, D] or [H, 128, 128]) or None; eigenvalues fp64 [D]."""
    W = None if W is None else np.ascontiguousarray(W, dtype=np.float16)
    Qc = None if Q is None else np.ascontiguousarray(Q, dtype=np.float32)
    lam = None if eigenvalues is None else np.ascontiguousarray(eigenvalues, dtype=np.float64)
    d = PackDesc()
    d.out_features = out_features if out_features is not None else (W.shape[0] if W is not None else 0)
    d.in_features = in_features if in_features is not None else (W.shape[1] if W is not None else 0)
    d.W = _ptr(W)
    d.ldw = ldw if ldw is not None else d.in_features
    d.q_mode, d.head_dim = q_mode, head_dim
    d.Q, d.eigenvalues = _ptr(Qc), _ptr(lam)
    d.K, d.bits, d.group, d.select_rule, d.host_only = K, bits, group, select_rule, int(host_only)
    d.select_arg = select_arg
    d.rotation_absorbed = int(rotation_absorbed)
    out = C.c_void_p()
    _check(lib().rosaq_pack_weights(C.byref(d), C.c_void_p(stream), C.byref(out)))
    return Packed(out.value)


def rosaq_packed_clone(p: Packed, stream: int = 0) -> Packed:
    out = C.c_void_p()
    _check(lib().rosaq_packed_clone(p.handle, C.c_void_p(stream), C.byref(out)))
    return Packed(out.value)


def rosaq_packed_export(p: Packed) -> dict:
    G = (p.D - p.K) // p.group
    sal = np.empty(p.K, np.int32)
    W_S = np.empty((p.N, p.K), np.float16)
    codes = np.empty((p.N, p.D - p.K), np.uint8)
    scales = np.empty((p.N, G), np.float16)
    zeros = np.empty((p.N, G), np.float16)
    _check(lib().rosaq_packed_export(p.handle, _ptr(sal), _ptr(W_S), _ptr(codes), _ptr(scales), _ptr(zeros)))
    return dict(salient_idx=sal, W_S=W_S, codes=codes, scales=scales, zeros=zeros)


def rosaq_workspace_bytes(p: Packed, M: int) -> int:
    return lib().rosaq_workspace_bytes(p.handle, M)


def rosaq_workspace_bytes_min(p: Packed, M: int) -> int:
    return lib().rosaq_workspace_bytes_min(p.handle, M)


def rosaq_workspace_bytes_batch(layers, M: int) -> int:
    arr = (C.c_void_p * len(layers))(*[p.handle.value for p in layers])
    return lib().rosaq_workspace_bytes_batch(arr, len(layers), M)


def rosaq_linear(p: Packed, x_ptr: int, M: int, ldx: int, y_ptr: int, ldy: int, ws_ptr: int,
                 ws_bytes: int, stream: int = 0):
    _check(lib().rosaq_linear(p.handle, x_ptr, M, ldx, y_ptr, ldy, ws_ptr, ws_bytes, stream))


def rosaq_linear_headwise(p: Packed, x_ptr: int, M: int, ldx: int, y_ptr: int, ldy: int, ws_ptr: int,
                          ws_bytes: int, stream: int = 0):
    _check(lib().rosaq_linear_headwise(p.handle, x_ptr, M, ldx, y_ptr, ldy, ws_ptr, ws_bytes, stream))


def rosaq_linear_headwise_static(p: Packed, x_ptr: int, M: int, ldx: int, y_ptr: int, ldy: int, stream: int = 0):
    _check(lib().rosaq_linear_headwise_static(p.handle, x_ptr, M, ldx, y_ptr, ldy, stream))


class BatchArgs:
    """Marshalled argument arrays of one rosaq_linear_batch call (reusable)."""

    def __init__(self, layers, y_ptrs, ldys):
        n = len(layers)
        self.count = n
        self.layers = (C.c_void_p * n)(*[p.handle.value for p in layers])
        self.ys = (C.c_void_p * n)(*y_ptrs)
        self.ldys = (C.c_int64 * n)(*ldys)
        self._keep = list(layers)


def rosaq_linear_batch(args: BatchArgs, x_ptr: int, M: int, ldx: int, ws_ptr: int, ws_bytes: int,
                       stream: int = 0):
    _check(lib().rosaq_linear_batch(args.layers, args.count, x_ptr, M, ldx, args.ys, args.ldys,
                                    ws_ptr, ws_bytes, stream))


def rosaq_linear_swiglu(gate: Packed, up: Packed, x_ptr: int, M: int, ldx: int, y_ptr: int, ldy: int,
                        ws_ptr: int, ws_bytes: int, stream: int = 0):
    _check(lib().rosaq_linear_swiglu(gate.handle, up.handle, x_ptr, M, ldx, y_ptr, ldy, ws_ptr, ws_bytes, stream))


def rosaq_workspace_bytes_mlp(gate: Packed, up: Packed, down: Packed, M: int) -> int:
    return lib().rosaq_workspace_bytes_mlp(gate.handle, up.handle, down.handle, M)


def rosaq_mlp_swiglu(gate: Packed, up: Packed, down: Packed, x_ptr: int, M: int, ldx: int, y_ptr: int, ldy: int,
                     ws_ptr: int, ws_bytes: int, stream: int = 0):
    _check(lib().rosaq_mlp_swiglu(gate.handle, up.handle, down.handle, x_ptr, M, ldx, y_ptr, ldy, ws_ptr,
                                  ws_bytes, stream))


def rosaq_pca_headwise(x_ptr: int, n_cal: int, D: int, ldx: int, stream: int = 0):
    """Returns (Q fp32 [D/128, 128, 128], eigenvalues fp64 [D]) for device activations at x_ptr."""
    Q = np.empty((max(D // 128, 0), 128, 128), np.float32)
    lam = np.empty(max(D, 0), np.float64)
    _check(lib().rosaq_pca_headwise(x_ptr, n_cal, D, ldx, _ptr(Q), _ptr(lam), stream))
    return Q, lam


def rosaq_pca_full(x_ptr: int, n_cal: int, D: int, ldx: int, stream: int = 0):
    """Returns (Q fp32 [D, D], eigenvalues fp64 [D]) for device activations at x_ptr."""
    Q = np.empty((max(D, 0), max(D, 0)), np.float32)
    lam = np.empty(max(D, 0), np.float64)
    _check(lib().rosaq_pca_full(x_ptr, n_cal, D, ldx, _ptr(Q), _ptr(lam), stream))
    return Q, lam


def rosaq_stream_probe(src_ptr: int, src_bytes: int, shared_ptr: int, shared_bytes: int,
                       shared_bytes_per_workgroup: int, workgroups: int, threads: int,
                       sink_ptr: int, sink_bytes: int, stream: int = 0):
    _check(lib().rosaq_stream_probe(src_ptr, src_bytes, shared_ptr, shared_bytes,
                                    shared_bytes_per_workgroup, workgroups, threads, sink_ptr,
                                    sink_bytes, stream))


def rosaq_launch_shape(M: int, channels: int, in_features: int, bits: int):
    """(mt, nt, waves per workgroup, units in flight, splits) of the main GEMM such a launch would get."""
    out = (C.c_int32 * 5)()
    _check(lib().rosaq_launch_shape(M, channels, in_features, bits, out))
    return tuple(out)


def rosaq_packed_image(p: "Packed", which: int) -> np.ndarray:
    """The weight image the kernels read (0: fp16 fragments, 1: low-bit records) as uint32 words."""
    n = C.c_size_t(0)
    _check(lib().rosaq_packed_image(p.handle, which, None, C.byref(n)))
    out = np.empty(n.value // 4, np.uint32)
    _check(lib().rosaq_packed_image(p.handle, which, out.ctypes.data_as(C.c_void_p), C.byref(n)))
    return out


def rosaq_block_map(workgroup: int, chunks: int, row_groups: int):
    """Grid size for workgroup < 0; else (chunk, row_group), or None for a padding workgroup."""
    c, m = C.c_int32(-1), C.c_int32(-1)
    r = lib().rosaq_block_map(workgroup, chunks, row_groups, C.byref(c), C.byref(m))
    if r < 0:
        _check(r)
    if workgroup < 0:
        return r
    return (c.value, m.value) if r else None


def rosaq_tune(key: str, value: int):
    _check(lib().rosaq_tune(key.encode(), value))
