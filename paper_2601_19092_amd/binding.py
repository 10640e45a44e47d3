"""ctypes binding of libaxe_hip.so -- argument marshalling only.

Every operation runs in the HIP kernels behind the C ABI declared in include/axe.h; nothing is
computed here and there is no CPU fallback: if the shared library has not been built, loading
fails with an error.  PyTorch tensors are used only as owners of device memory (data_ptr) and
for the current HIP stream.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libaxe_hip.so")

AXE_OK, AXE_EINVAL, AXE_ESHAPE, AXE_EALIAS, AXE_ERANGE, AXE_EUNSUPPORTED, AXE_EHIP, AXE_ENOFORM, AXE_ETIMEOUT = 0, -1, -2, -3, -4, -5, -6, -7, -8
AXE_BF16, AXE_FP8_E4M3, AXE_F32, AXE_F16 = 1, 2, 3, 4
AXE_TILE_AUTO, AXE_TILE_64x64x32, AXE_TILE_256x256x64, AXE_TILE_256x224x64 = 0, 1, 2, 3
(AXE_DESC_A_G2L_THREADS, AXE_DESC_B_G2L_THREADS, AXE_DESC_A_LDS, AXE_DESC_B_LDS, AXE_DESC_A_OPERAND,
 AXE_DESC_B_OPERAND, AXE_DESC_ACC, AXE_DESC_C_STORE) = range(8)
AXE_MAX_RANK = 8
AXE_SCALE_F32, AXE_SCALE_E8M0 = 0, 1
AXE_EPI_NONE, AXE_EPI_SWIGLU = 0, 1
AXE_GROUPED_AUTO, AXE_GROUPED_TILES, AXE_GROUPED_STREAM, AXE_GROUPED_TILES_256, AXE_GROUPED_TILES_128 = 0, 1, 2, 3, 4

EXPORTS = ["axe_layout_eval", "axe_relayout", "axe_gemm", "axe_gemm_grouped", "axe_gemm_grouped_check", "axe_gemm_grouped_pair", "axe_gemm_grouped_pair_fused",
           "axe_gemm_grouped_pair_status", "axe_gemm_grouped_pair_static", "axe_gemm_grouped_kernel", "axe_gemm_grouped_describe", "axe_gemm_tile", "axe_gemm_describe", "axe_strerror",
           "axe_last_error", "axe_version", "axe_layout_span", "axe_layout_canonicalize", "axe_layout_gap_condition",
           "axe_layout_equal", "axe_layout_group", "axe_layout_tile", "axe_layout_direct_sum", "axe_layout_flatten", "axe_layout_tile_of",
           "axe_layout_slice"]


class axe_iter_t(C.Structure):
    _fields_ = [("extent", C.c_int64), ("stride", C.c_int64), ("axis", C.c_int32)]


class axe_layout_t(C.Structure):
    _fields_ = [("n_axes", C.c_int32), ("axis_names", C.POINTER(C.c_char_p)),
                ("n_d", C.c_int32), ("d", C.POINTER(axe_iter_t)),
                ("n_r", C.c_int32), ("r", C.POINTER(axe_iter_t)),
                ("offset", C.POINTER(C.c_int64)),
                ("swz_axis", C.c_int32), ("swz_bits", C.c_int32), ("swz_base", C.c_int32), ("swz_shift", C.c_int32)]


class axe_gemm_desc_t(C.Structure):
    _fields_ = [("M", C.c_int64), ("N", C.c_int64), ("K", C.c_int64),
                ("in_dtype", C.c_int32), ("out_dtype", C.c_int32),
                ("A", axe_layout_t), ("B", axe_layout_t), ("C", axe_layout_t),
                ("mem_axis", C.c_int32),
                ("a_elems", C.c_int64), ("b_elems", C.c_int64), ("c_elems", C.c_int64),
                ("d_scale_a", C.c_void_p), ("d_scale_b", C.c_void_p),
                ("scale_block", C.c_int32), ("tile_hint", C.c_int32), ("scale_dtype", C.c_int32),
                ("scale_a_rows", C.c_int32)]


class axe_gemm_grouped_desc_t(C.Structure):
    _fields_ = [("M", C.c_int64), ("N", C.c_int64), ("K", C.c_int64), ("G", C.c_int32),
                ("in_dtype", C.c_int32), ("out_dtype", C.c_int32),
                ("A", axe_layout_t), ("B", axe_layout_t), ("C", axe_layout_t),
                ("mem_axis", C.c_int32),
                ("a_elems", C.c_int64), ("b_elems", C.c_int64), ("c_elems", C.c_int64), ("epilogue", C.c_int32),
                ("kernel_hint", C.c_int32), ("d_scale_a", C.c_void_p), ("d_scale_b", C.c_void_p), ("scale_dtype", C.c_int32)]


class AxeError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"axe error {code}: {message}")
        self.code = code
        self.message = message


_lib = None


def load(path: str) -> C.CDLL:
    """Loads a build of the library and declares its entry points (raises if it has not been built: there is no fallback)."""
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it with `python -m paper_2601_19092_amd.build` "
                           "(or __graft_entry__.build()); this package has no CPU fallback")
    L = C.CDLL(path)
    vp, i64, i32 = C.c_void_p, C.c_int64, C.c_int32
    LP = C.POINTER(axe_layout_t)
    L.axe_layout_eval.restype = C.c_int
    L.axe_layout_eval.argtypes = [LP, i32, C.POINTER(i64), i64, vp, vp, vp]
    L.axe_relayout.restype = C.c_int
    L.axe_relayout.argtypes = [LP, LP, i32, C.POINTER(i64), i32, i32, vp, i64, vp, i64, vp]
    L.axe_gemm.restype = C.c_int
    L.axe_gemm.argtypes = [C.POINTER(axe_gemm_desc_t), vp, vp, vp, vp]
    L.axe_gemm_grouped.restype = C.c_int
    L.axe_gemm_grouped.argtypes = [C.POINTER(axe_gemm_grouped_desc_t), vp, vp, vp, vp, vp]
    L.axe_gemm_grouped_check.restype = C.c_int
    L.axe_gemm_grouped_check.argtypes = [C.POINTER(axe_gemm_grouped_desc_t)]
    GP = C.POINTER(axe_gemm_grouped_desc_t)
    L.axe_gemm_grouped_pair.restype = C.c_int
    L.axe_gemm_grouped_pair.argtypes = [GP, GP, vp, vp, vp, vp, vp, vp, vp, i64, vp]
    L.axe_gemm_grouped_pair_static.restype = C.c_int
    L.axe_gemm_grouped_pair_static.argtypes = [GP, GP, vp, vp, vp, vp, vp, vp, vp]
    L.axe_gemm_grouped_pair_fused.restype = C.c_int
    L.axe_gemm_grouped_pair_fused.argtypes = [GP, GP]
    L.axe_gemm_grouped_pair_status.restype = C.c_int
    L.axe_gemm_grouped_pair_status.argtypes = [vp, i64, vp]
    L.axe_gemm_tile.restype = C.c_int
    L.axe_gemm_tile.argtypes = [C.POINTER(axe_gemm_desc_t)]
    L.axe_gemm_grouped_kernel.restype = C.c_int
    L.axe_gemm_grouped_kernel.argtypes = [C.POINTER(axe_gemm_grouped_desc_t)]
    L.axe_gemm_grouped_describe.restype = C.c_int
    L.axe_gemm_grouped_describe.argtypes = [C.POINTER(axe_gemm_grouped_desc_t), i32, LP, C.POINTER(i64), C.POINTER(i32), vp, C.c_size_t]
    L.axe_gemm_describe.restype = C.c_int
    L.axe_gemm_describe.argtypes = [C.POINTER(axe_gemm_desc_t), i32, LP, C.POINTER(i64), C.POINTER(i32), vp,
                                    C.c_size_t]
    P64, P32, sz = C.POINTER(i64), C.POINTER(i32), C.c_size_t
    for name, args in (("axe_layout_span", [LP, P64]), ("axe_layout_canonicalize", [LP, LP, vp, sz]),
                       ("axe_layout_gap_condition", [LP]), ("axe_layout_equal", [LP, LP]),
                       ("axe_layout_group", [LP, i32, P64, LP, P32, vp, sz]),
                       ("axe_layout_tile", [LP, i32, P64, LP, P64, LP, P64, vp, sz]),
                       ("axe_layout_direct_sum", [LP, i32, P64, LP, P64, LP, P64, vp, sz]),
                       ("axe_layout_flatten", [LP, P64, i32, LP, vp, sz]),
                       ("axe_layout_tile_of", [LP, i32, P64, LP, P64, LP, P64, vp, sz]),
                       ("axe_layout_slice", [LP, i32, P64, P64, P64, LP, vp, sz])):
        getattr(L, name).restype = C.c_int
        getattr(L, name).argtypes = args
    L.axe_strerror.restype = C.c_char_p
    L.axe_strerror.argtypes = [C.c_int]
    L.axe_last_error.restype = C.c_char_p
    L.axe_version.restype = i32
    return L


def lib() -> C.CDLL:
    """The HIP library, loaded on first use."""
    global _lib
    if _lib is None:
        _lib = load(LIB_PATH)
    return _lib


def _check(rc: int) -> None:
    if rc != 0:
        L = lib()
        msg = L.axe_last_error().decode() or L.axe_strerror(rc).decode()
        raise AxeError(rc, msg)


class Layout:
    """Host-side holder of an axe_layout_t and of the ctypes arrays it points to.

    spec = {"D": [(extent, stride, axis_name), ...], "R": [...], "O": {axis_name: value},
            "swizzle": None | (axis_name, bits, base, shift)}; `axes` fixes the axis order
    (default: order of first appearance in D, R, O, swizzle)."""

    def __init__(self, spec: dict, axes: Optional[Sequence[str]] = None):
        names: List[str] = list(axes) if axes is not None else []
        def idx(a: str) -> int:
            if a not in names:
                if axes is not None:
                    raise ValueError(f"axis {a!r} not in {axes}")
                names.append(a)
            return names.index(a)
        D = [(int(e), int(s), idx(a)) for e, s, a in spec["D"]]
        R = [(int(e), int(s), idx(a)) for e, s, a in spec.get("R", ())]
        O = {idx(a): int(v) for a, v in (spec.get("O") or {}).items()}
        z = spec.get("swizzle")
        zi = (idx(z[0]), int(z[1]), int(z[2]), int(z[3])) if z else (-1, 0, 0, 0)
        self.axes = names
        self._d = (axe_iter_t * max(1, len(D)))(*[axe_iter_t(*t) for t in D])
        self._r = (axe_iter_t * max(1, len(R)))(*[axe_iter_t(*t) for t in R])
        self._o = (C.c_int64 * max(1, len(names)))(*[O.get(i, 0) for i in range(len(names))])
        self._names = (C.c_char_p * max(1, len(names)))(*[n.encode() for n in names])
        self.c = axe_layout_t(len(names), self._names, len(D), self._d, len(R), self._r, self._o, *zi)
        self.E_R = 1
        for e, _, _ in R:
            self.E_R *= e

    def axis(self, name: str) -> int:
        return self.axes.index(name)


_raw_stream = None


def _stream_ptr(stream=None) -> int:
    """The hipStream_t to launch on: the given torch stream (or raw handle), else torch's current stream of the current
    device.  (torch.cuda.current_stream() builds a Python object per call, 2.5 us -- as much as a small launch; the raw
    getter it is built on is used when the installed torch has it.)"""
    global _raw_stream
    if stream is not None:
        return stream if isinstance(stream, int) else int(stream.cuda_stream)
    import torch
    if _raw_stream is None:
        _raw_stream = getattr(torch._C, "_cuda_getCurrentRawStream", False)
    if _raw_stream:
        return int(_raw_stream(torch.cuda.current_device()))
    return int(torch.cuda.current_stream().cuda_stream)


def _shape_arr(shape: Sequence[int]):
    return (C.c_int64 * len(shape))(*[int(s) for s in shape])


def axe_layout_eval(layout: Layout, shape: Sequence[int], n: int, flat_idx=None, out=None, stream=None):
    """Device evaluation of the induced map; returns an int64 CUDA tensor [n, E_R, n_axes]."""
    import torch
    if out is None:
        out = torch.empty((n, layout.E_R, len(layout.axes)), dtype=torch.int64, device="cuda")
    idx_ptr = None
    if flat_idx is not None:
        assert flat_idx.dtype == torch.int64 and flat_idx.is_cuda and flat_idx.is_contiguous() and flat_idx.numel() == n
        idx_ptr = flat_idx.data_ptr()
    assert out.dtype == torch.int64 and out.is_cuda and out.is_contiguous()
    assert out.numel() == n * layout.E_R * len(layout.axes)
    _check(lib().axe_layout_eval(C.byref(layout.c), len(shape), _shape_arr(shape), n, idx_ptr, out.data_ptr(),
                                 _stream_ptr(stream)))
    return out


def axe_relayout(src: Layout, dst: Layout, shape: Sequence[int], src_buf, dst_buf, mem_axis: str = "m",
                 elem_bytes: Optional[int] = None, stream=None):
    """dst_buf[f_dst(x)] = src_buf[f_src(x)]; buffers are 1-D CUDA tensors of one element size."""
    eb = elem_bytes if elem_bytes is not None else src_buf.element_size()
    assert src_buf.is_cuda and dst_buf.is_cuda and src_buf.is_contiguous() and dst_buf.is_contiguous()
    assert src.axes.index(mem_axis) == dst.axes.index(mem_axis), "memory axis must have the same index in both layouts"
    s_elems = src_buf.numel() * src_buf.element_size() // eb
    d_elems = dst_buf.numel() * dst_buf.element_size() // eb
    _check(lib().axe_relayout(C.byref(src.c), C.byref(dst.c), len(shape), _shape_arr(shape), eb, src.axis(mem_axis),
                              src_buf.data_ptr(), s_elems, dst_buf.data_ptr(), d_elems, _stream_ptr(stream)))
    return dst_buf


class GemmDesc:
    """Holder of an axe_gemm_desc_t (keeps the three layouts alive)."""

    def __init__(self, M: int, N: int, K: int, in_dtype: int, out_dtype: int, A: Layout, B: Layout, Cl: Layout,
                 a_elems: int, b_elems: int, c_elems: int, scale_a=None, scale_b=None, scale_block: int = 128,
                 tile_hint: int = AXE_TILE_AUTO, mem_axis: str = "m", scale_dtype: int = AXE_SCALE_F32,
                 scale_a_rows: int = 0):
        ma = A.axis(mem_axis)
        assert B.axis(mem_axis) == ma and Cl.axis(mem_axis) == ma, "memory axis must have the same index in A, B, C"
        self.layouts = (A, B, Cl)
        self.scales = (scale_a, scale_b)
        self.c = axe_gemm_desc_t(M, N, K, in_dtype, out_dtype, A.c, B.c, Cl.c, ma, a_elems, b_elems, c_elems,
                                 scale_a.data_ptr() if scale_a is not None else None,
                                 scale_b.data_ptr() if scale_b is not None else None, scale_block, tile_hint, scale_dtype,
                                 scale_a_rows)


def axe_gemm(desc: GemmDesc, A_buf, B_buf, C_buf, stream=None):
    assert A_buf.is_cuda and B_buf.is_cuda and C_buf.is_cuda
    _check(lib().axe_gemm(C.byref(desc.c), A_buf.data_ptr(), B_buf.data_ptr(), C_buf.data_ptr(), _stream_ptr(stream)))
    return C_buf


class GroupedGemmDesc:
    """Holder of an axe_gemm_grouped_desc_t (keeps the three layouts alive).  A: (M, K), B: (G, K, N), Cl: (M, N)."""

    def __init__(self, M: int, N: int, K: int, G: int, A: Layout, B: Layout, Cl: Layout, a_elems: int, b_elems: int,
                 c_elems: int, in_dtype: int = AXE_BF16, out_dtype: int = AXE_BF16, mem_axis: str = "m",
                 epilogue: int = 0, kernel_hint: int = 0, scale_a=None, scale_b=None, scale_dtype: int = AXE_SCALE_F32):
        ma = A.axis(mem_axis)
        assert B.axis(mem_axis) == ma and Cl.axis(mem_axis) == ma, "memory axis must have the same index in A, B, C"
        self.layouts = (A, B, Cl)
        self.c = axe_gemm_grouped_desc_t(M, N, K, G, in_dtype, out_dtype, A.c, B.c, Cl.c, ma, a_elems, b_elems, c_elems, epilogue,
                                         kernel_hint, scale_a.data_ptr() if scale_a is not None else None,
                                         scale_b.data_ptr() if scale_b is not None else None, scale_dtype)
        self.scales = (scale_a, scale_b)


def axe_gemm_grouped(desc: GroupedGemmDesc, A_buf, B_buf, C_buf, group_rows, stream=None):
    """group_rows: int32 device tensor of G + 1 row offsets."""
    assert A_buf.is_cuda and B_buf.is_cuda and C_buf.is_cuda and group_rows.is_cuda
    assert str(group_rows.dtype) == "torch.int32" and group_rows.numel() == desc.c.G + 1 and group_rows.is_contiguous()
    _check(lib().axe_gemm_grouped(C.byref(desc.c), A_buf.data_ptr(), B_buf.data_ptr(), C_buf.data_ptr(),
                                  group_rows.data_ptr(), _stream_ptr(stream)))
    return C_buf


def axe_gemm_grouped_pair(desc1: GroupedGemmDesc, desc2: GroupedGemmDesc, A_buf, B1_buf, H_buf, B2_buf, C_buf, group_rows,
                          sync=None, stream=None):
    """Both grouped GEMMs of an MoE layer's expert computation; with `sync` (int32 device tensor, M + 1 words) as one launch."""
    assert all(t.is_cuda for t in (A_buf, B1_buf, H_buf, B2_buf, C_buf, group_rows))
    assert str(group_rows.dtype) == "torch.int32" and group_rows.numel() == desc1.c.G + 1 and group_rows.is_contiguous()
    if sync is not None:
        assert sync.is_cuda and str(sync.dtype) == "torch.int32" and sync.is_contiguous()
    _check(lib().axe_gemm_grouped_pair(C.byref(desc1.c), C.byref(desc2.c), A_buf.data_ptr(), B1_buf.data_ptr(), H_buf.data_ptr(),
                                       B2_buf.data_ptr(), C_buf.data_ptr(), group_rows.data_ptr(),
                                       sync.data_ptr() if sync is not None else None, sync.numel() if sync is not None else 0,
                                       _stream_ptr(stream)))
    return C_buf


def axe_gemm_grouped_pair_static(desc1: GroupedGemmDesc, desc2: GroupedGemmDesc, A_buf, B1_buf, H_buf, B2_buf, C_buf, group_rows,
                                 stream=None):
    """axe_gemm_grouped_pair on the library's own workspace (nothing is allocated; calls on one device must not overlap)."""
    assert all(t.is_cuda for t in (A_buf, B1_buf, H_buf, B2_buf, C_buf, group_rows))
    assert str(group_rows.dtype) == "torch.int32" and group_rows.numel() == desc1.c.G + 1 and group_rows.is_contiguous()
    _check(lib().axe_gemm_grouped_pair_static(C.byref(desc1.c), C.byref(desc2.c), A_buf.data_ptr(), B1_buf.data_ptr(), H_buf.data_ptr(),
                                              B2_buf.data_ptr(), C_buf.data_ptr(), group_rows.data_ptr(), _stream_ptr(stream)))
    return C_buf


def axe_gemm_grouped_pair_fused(desc1: GroupedGemmDesc, desc2: GroupedGemmDesc) -> bool:
    return _flag(lib().axe_gemm_grouped_pair_fused(C.byref(desc1.c), C.byref(desc2.c)))


def axe_gemm_grouped_pair_status(sync, M: int, stream=None) -> None:
    """Synchronises the stream; raises if a wait inside the last fused launch that used `sync` gave up
    (sync None: the library's own workspace on the current device)."""
    _check(lib().axe_gemm_grouped_pair_status(sync.data_ptr() if sync is not None else None, M, _stream_ptr(stream)))


def axe_gemm_grouped_check(desc: GroupedGemmDesc) -> None:
    _check(lib().axe_gemm_grouped_check(C.byref(desc.c)))


def axe_gemm_tile(desc: GemmDesc) -> int:
    rc = lib().axe_gemm_tile(C.byref(desc.c))
    if rc < 0:
        _check(rc)
    return rc


def _spec_of(out: axe_layout_t, names: Optional[Sequence[str]] = None) -> dict:
    """An axe_layout_t the library filled in, as plain data (the same form Layout() takes)."""
    if names is None:
        names = [out.axis_names[i].decode() for i in range(out.n_axes)]
    return {"D": [(out.d[i].extent, out.d[i].stride, names[out.d[i].axis]) for i in range(out.n_d)],
            "R": [(out.r[i].extent, out.r[i].stride, names[out.r[i].axis]) for i in range(out.n_r)],
            "O": {names[a]: out.offset[a] for a in range(out.n_axes) if out.offset and out.offset[a] != 0},
            "swizzle": (names[out.swz_axis], out.swz_bits, out.swz_base, out.swz_shift) if out.swz_axis >= 0 else None}


def axe_gemm_describe(desc: GemmDesc, which: int) -> Tuple[dict, Tuple[int, ...]]:
    """Returns (spec, shape): the layout of one tile movement as plain data."""
    out = axe_layout_t()
    shape = (C.c_int64 * AXE_MAX_RANK)()
    rank = C.c_int32(0)
    arena = C.create_string_buffer(4096)
    _check(lib().axe_gemm_describe(C.byref(desc.c), which, C.byref(out), shape, C.byref(rank), arena, len(arena)))
    return _spec_of(out), tuple(shape[i] for i in range(rank.value))


def axe_gemm_grouped_kernel(desc: GroupedGemmDesc) -> int:
    rc = lib().axe_gemm_grouped_kernel(C.byref(desc.c))
    if rc < 0:
        _check(rc)
    return rc


def axe_gemm_grouped_describe(desc: GroupedGemmDesc, which: int) -> Tuple[dict, Tuple[int, ...]]:
    """Returns (spec, shape): the layout of one tile movement of the grouped tile kernel as plain data."""
    out = axe_layout_t()
    shape = (C.c_int64 * AXE_MAX_RANK)()
    rank = C.c_int32(0)
    arena = C.create_string_buffer(4096)
    _check(lib().axe_gemm_grouped_describe(C.byref(desc.c), which, C.byref(out), shape, C.byref(rank), arena, len(arena)))
    return _spec_of(out), tuple(shape[i] for i in range(rank.value))


# ---- layout operators (host only; the library does the work, this only marshals)
def _same_axes(*Ls: Layout) -> None:
    for L in Ls[1:]:
        if L.axes != Ls[0].axes:
            raise ValueError("the operands must be built on one axis list (pass axes= to Layout)")


def layout_span(L: Layout) -> Dict[str, int]:
    sp = (C.c_int64 * len(L.axes))()
    _check(lib().axe_layout_span(C.byref(L.c), sp))
    return {a: sp[i] for i, a in enumerate(L.axes)}


def layout_canonicalize(L: Layout) -> dict:
    out, arena = axe_layout_t(), C.create_string_buffer(1024)
    _check(lib().axe_layout_canonicalize(C.byref(L.c), C.byref(out), arena, len(arena)))
    return _spec_of(out, L.axes)


def _flag(rc: int) -> bool:
    if rc < 0:
        _check(rc)
    return bool(rc)


def layout_gap_condition(L: Layout) -> bool:
    return _flag(lib().axe_layout_gap_condition(C.byref(L.c)))


def layout_equal(A: Layout, B: Layout) -> bool:
    _same_axes(A, B)
    return _flag(lib().axe_layout_equal(C.byref(A.c), C.byref(B.c)))


def layout_group(L: Layout, shape: Sequence[int]) -> Tuple[dict, List[int]]:
    out, arena = axe_layout_t(), C.create_string_buffer(1024)
    ends = (C.c_int32 * len(shape))()
    _check(lib().axe_layout_group(C.byref(L.c), len(shape), _shape_arr(shape), C.byref(out), ends, arena, len(arena)))
    return _spec_of(out, L.axes), list(ends)


def _binary(fn, A: Layout, SA: Sequence[int], B: Layout, SB: Sequence[int], n_out: int):
    _same_axes(A, B)
    if len(SA) != len(SB):
        raise ValueError("the two shapes must have the same rank")
    out, arena = axe_layout_t(), C.create_string_buffer(1024)
    shape = (C.c_int64 * n_out)()
    _check(fn(C.byref(A.c), len(SA), _shape_arr(SA), C.byref(B.c), _shape_arr(SB), C.byref(out), shape, arena, len(arena)))
    return _spec_of(out, A.axes), tuple(shape)


def layout_tile(A: Layout, SA: Sequence[int], B: Layout, SB: Sequence[int]) -> Tuple[dict, Tuple[int, ...]]:
    return _binary(lib().axe_layout_tile, A, SA, B, SB, 2 * len(SA))


def layout_direct_sum(A: Layout, SA: Sequence[int], B: Layout, SB: Sequence[int]) -> Tuple[dict, Tuple[int, ...]]:
    return _binary(lib().axe_layout_direct_sum, A, SA, B, SB, 2 * len(SA))


def layout_flatten(L: Layout, pitch: Dict[str, int], to_axis: str) -> dict:
    """All axes of L folded onto `to_axis`: coordinate c on axis a goes to c * pitch[a] (axes not named: pitch 0)."""
    out, arena = axe_layout_t(), C.create_string_buffer(2048)
    p = (C.c_int64 * len(L.axes))(*[int(pitch.get(a, 0)) for a in L.axes])
    _check(lib().axe_layout_flatten(C.byref(L.c), p, L.axis(to_axis), C.byref(out), arena, len(arena)))
    return _spec_of(out, L.axes)


def layout_tile_of(A: Layout, SA: Sequence[int], B: Layout, SB: Sequence[int]) -> Tuple[dict, Tuple[int, ...]]:
    return _binary(lib().axe_layout_tile_of, A, SA, B, SB, len(SA))


def layout_slice(L: Layout, shape: Sequence[int], begin: Sequence[int], size: Sequence[int]) -> dict:
    out, arena = axe_layout_t(), C.create_string_buffer(1024)
    _check(lib().axe_layout_slice(C.byref(L.c), len(shape), _shape_arr(shape), _shape_arr(begin), _shape_arr(size),
                                  C.byref(out), arena, len(arena)))
    return _spec_of(out, L.axes)


def version() -> int:
    return int(lib().axe_version())
