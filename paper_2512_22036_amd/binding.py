"""ctypes binding of libfusco.so: same names as the C boundary, argument marshalling only.

Every step of the shuffle runs in the library's HIP kernels.  This module checks tensor shapes
against the layout (the C side sees bare pointers), passes pointers and the current HIP stream,
and turns negative return codes into FuscoError.  It never computes on the data and has no
fallback path: a missing library is an error.
"""
from __future__ import annotations

import ctypes
import os
from types import SimpleNamespace
from typing import Optional

import torch

BF16, F32 = 0, 1
DISPATCH_EXPERT, DISPATCH_WIRE, DISPATCH_TWO_HOP, DISPATCH_STREAMING = 1, 2, 4, 8

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libfusco.so")

EXPORTS = ("fusco_version", "fusco_status_string", "fusco_layout_bytes", "fusco_scratch_bytes",
           "fusco_layout_bind", "fusco_plan", "fusco_plan_static", "fusco_dispatch", "fusco_dispatch_in_transfer_order", "fusco_combine", "fusco_plan_dispatch", "fusco_probe_copy", "fusco_probe_rows", "fusco_probe_pieces", "fusco_probe_consume_slices", "fusco_probe_time_next_call", "fusco_probe_source_chunk_bytes", "fusco_probe_dispatch_kernel", "fusco_probe_dispatch_occupancy", "fusco_probe_dispatch_pull", "fusco_probe_dispatch_walk",
           "fusco_combine_two_hop", "fusco_balance_groups", "fusco_cross_node_load", "fusco_segments_scan", "fusco_segments_copy",
           "fusco_disaggregated_plan", "fusco_disaggregated_dispatch", "fusco_disaggregated_combine")


class FuscoError(RuntimeError):
    pass


class _CLayout(ctypes.Structure):
    """Mirror of struct fusco_layout."""
    _fields_ = [("N", ctypes.c_int32), ("k", ctypes.c_int32), ("E", ctypes.c_int32), ("D", ctypes.c_int32),
                ("P", ctypes.c_int32), ("send_cap", ctypes.c_int32),
                ("exp_count", ctypes.c_void_p), ("exp_off", ctypes.c_void_p),
                ("send_count", ctypes.c_void_p), ("send_off", ctypes.c_void_p),
                ("pair_slot", ctypes.c_void_p), ("slot_pair", ctypes.c_void_p),
                ("slot_token", ctypes.c_void_p), ("send_src", ctypes.c_void_p),
                ("pair_send_row", ctypes.c_void_p), ("slot_send_row", ctypes.c_void_p),
                ("pair_first", ctypes.c_void_p), ("status", ctypes.c_void_p),
                ("tile_slots", ctypes.c_void_p), ("tile_tokens", ctypes.c_int32), ("tile_count", ctypes.c_int32)]


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Load libfusco.so (built by paper_2512_22036_amd.build / __graft_entry__.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FuscoError("libfusco.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                         "(there is no fallback path)")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, sz, u32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t, ctypes.c_uint32
    lib.fusco_version.restype = ctypes.c_int
    lib.fusco_version.argtypes = []
    lib.fusco_status_string.restype = ctypes.c_char_p
    lib.fusco_status_string.argtypes = [ctypes.c_int]
    lib.fusco_layout_bytes.restype = sz
    lib.fusco_layout_bytes.argtypes = [i32, i32, i32, i32]
    lib.fusco_scratch_bytes.restype = sz
    lib.fusco_scratch_bytes.argtypes = [i32, i32, i32, i32]
    lib.fusco_layout_bind.restype = ctypes.c_int
    lib.fusco_layout_bind.argtypes = [ctypes.POINTER(_CLayout), i32, i32, i32, i32, vp, sz]
    lib.fusco_plan.restype = ctypes.c_int
    lib.fusco_plan.argtypes = [ctypes.POINTER(_CLayout), vp, vp, sz, vp]
    lib.fusco_plan_static.restype = ctypes.c_int
    lib.fusco_plan_static.argtypes = [ctypes.POINTER(_CLayout), vp, vp]
    lib.fusco_dispatch.restype = ctypes.c_int
    lib.fusco_dispatch.argtypes = [ctypes.POINTER(_CLayout), vp, sz, vp, sz, vp, vp, vp, vp, u32, vp]
    lib.fusco_dispatch_in_transfer_order.restype = ctypes.c_int
    lib.fusco_dispatch_in_transfer_order.argtypes = [ctypes.POINTER(_CLayout), sz, sz, u32]
    lib.fusco_plan_dispatch.restype = ctypes.c_int
    lib.fusco_plan_dispatch.argtypes = [ctypes.POINTER(_CLayout), vp, vp, sz, vp, sz, vp, vp, vp]
    lib.fusco_combine.restype = ctypes.c_int
    lib.fusco_combine.argtypes = [ctypes.POINTER(_CLayout), vp, ctypes.c_int, vp, vp, ctypes.c_int, i32, u32, vp]
    lib.fusco_probe_copy.restype = ctypes.c_int
    lib.fusco_probe_copy.argtypes = [vp, vp, sz, vp]
    lib.fusco_probe_dispatch_kernel.restype = ctypes.c_int
    lib.fusco_probe_dispatch_kernel.argtypes = [ctypes.c_int]
    lib.fusco_probe_dispatch_occupancy.restype = ctypes.c_int
    lib.fusco_probe_dispatch_occupancy.argtypes = [ctypes.c_int]
    lib.fusco_probe_dispatch_walk.restype = ctypes.c_int
    lib.fusco_probe_dispatch_walk.argtypes = [ctypes.c_int]
    lib.fusco_probe_dispatch_pull.restype = ctypes.c_int
    lib.fusco_probe_dispatch_pull.argtypes = [ctypes.c_int]
    lib.fusco_probe_source_chunk_bytes.restype = ctypes.c_size_t
    lib.fusco_probe_source_chunk_bytes.argtypes = [sz]
    lib.fusco_probe_time_next_call.restype = ctypes.c_int
    lib.fusco_probe_time_next_call.argtypes = [vp, vp]
    lib.fusco_probe_rows.restype = ctypes.c_int
    lib.fusco_probe_rows.argtypes = [vp, u32, vp, u32, sz, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                     vp, vp]
    lib.fusco_probe_pieces.restype = ctypes.c_int
    lib.fusco_probe_pieces.argtypes = [vp, sz, ctypes.c_int, u32, ctypes.c_int, vp, vp]
    lib.fusco_probe_consume_slices.restype = ctypes.c_int
    lib.fusco_probe_consume_slices.argtypes = [vp, ctypes.c_uint64, ctypes.c_uint64, vp, u32, vp, vp]
    lp = ctypes.POINTER(_CLayout)
    u64, i64 = ctypes.c_uint64, ctypes.c_int64
    lib.fusco_segments_scan.restype = ctypes.c_int
    lib.fusco_segments_scan.argtypes = [vp, i64, vp, vp, vp]
    lib.fusco_segments_copy.restype = ctypes.c_int
    lib.fusco_segments_copy.argtypes = [vp, u64, vp, vp, u64, vp, vp, i64, u64, u64, vp, vp, vp]
    lib.fusco_cross_node_load.restype = ctypes.c_int
    lib.fusco_cross_node_load.argtypes = [ctypes.POINTER(_CLayout), i32, i32, sz, vp, vp]
    lib.fusco_balance_groups.restype = ctypes.c_int
    lib.fusco_balance_groups.argtypes = [vp, i32, i32, vp]
    lib.fusco_combine_two_hop.restype = ctypes.c_int
    lib.fusco_combine_two_hop.argtypes = [lp, vp, ctypes.c_int, vp, vp, vp, ctypes.c_int, i32, vp]
    lib.fusco_disaggregated_plan.restype = ctypes.c_int
    lib.fusco_disaggregated_plan.argtypes = [lp, lp, vp, vp, vp, sz, vp]
    lib.fusco_disaggregated_dispatch.restype = ctypes.c_int
    lib.fusco_disaggregated_dispatch.argtypes = [lp, lp, vp, sz, vp, vp, vp, vp]
    lib.fusco_disaggregated_combine.restype = ctypes.c_int
    lib.fusco_disaggregated_combine.argtypes = [lp, lp, vp, ctypes.c_int, vp, vp, vp, vp, ctypes.c_int, i32, vp]
    _lib = lib
    return lib


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise FuscoError("%s failed: %s (%d)" % (what, load_library().fusco_status_string(rc).decode(), rc))


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _rows(t: torch.Tensor, name: str, min_rows: int, row_bytes: Optional[int] = None) -> int:
    if not t.is_cuda or t.dim() != 2 or not t.is_contiguous():
        raise FuscoError("%s must be a contiguous 2-D device tensor" % name)
    if t.shape[0] < min_rows:
        raise FuscoError("%s has %d rows, needs %d" % (name, t.shape[0], min_rows))
    rb = t.shape[1] * t.element_size()
    if row_bytes is not None and rb != row_bytes:
        raise FuscoError("%s rows are %d bytes, expected %d" % (name, rb, row_bytes))
    return rb


def fusco_version() -> int:
    return load_library().fusco_version()


_I32_FIELDS = {"exp_count": "E", "exp_off": "E+1", "send_count": "D", "send_off": "D+1", "pair_slot": "P",
               "slot_pair": "P", "slot_token": "P", "send_src": "send_cap", "pair_send_row": "P",
               "slot_send_row": "P", "status": "1", "tile_slots": "tiles"}


class Layout:
    """Device-resident layout descriptor: owns the device block the C struct points into and the
    planner scratch.  Arrays are exposed as torch views of that block (no copies)."""

    def __init__(self, N: int, k: int, E: int, D: int, device="cuda"):
        lib = load_library()
        nbytes = lib.fusco_layout_bytes(N, k, E, D)
        if nbytes == 0:
            raise FuscoError("invalid layout sizes N=%d k=%d E=%d D=%d" % (N, k, E, D))
        self.mem = torch.empty(nbytes, dtype=torch.uint8, device=device)
        self.scratch = torch.empty(lib.fusco_scratch_bytes(N, k, E, D), dtype=torch.uint8, device=device)
        self.c = _CLayout()
        _check(lib.fusco_layout_bind(ctypes.byref(self.c), N, k, E, D, self.mem.data_ptr(), nbytes),
               "fusco_layout_bind")
        self.N, self.k, self.E, self.D = N, k, E, D
        self.P, self.send_cap = int(self.c.P), int(self.c.send_cap)
        self.tile_tokens, self.tile_count = int(self.c.tile_tokens), int(self.c.tile_count)

    def array(self, name: str) -> torch.Tensor:
        """Torch view of one descriptor array (int32, or uint8 for pair_first)."""
        sizes = {"E": self.E, "E+1": self.E + 1, "D": self.D, "D+1": self.D + 1, "P": self.P,
                 "send_cap": self.send_cap, "1": 1, "tiles": self.tile_count * self.tile_tokens * self.k}
        off = getattr(self.c, name) - self.mem.data_ptr()
        if name == "pair_first":
            return self.mem[off:off + self.P]
        n = sizes[_I32_FIELDS[name]]
        return self.mem[off:off + 4 * n].view(torch.int32)

    def to_host(self) -> SimpleNamespace:
        """Synchronising copy of every array to numpy (send_src cut to its U valid rows)."""
        out = {n: self.array(n).cpu().numpy() for n in list(_I32_FIELDS) + ["pair_first"]}
        U = int(out["send_off"][self.D])
        out["send_src"] = out["send_src"][:max(0, min(U, self.send_cap))]
        return SimpleNamespace(N=self.N, k=self.k, E=self.E, D=self.D, P=self.P, U=U, **out)


def fusco_plan(layout: Layout, topk_idx: torch.Tensor, stream=None) -> None:
    if (not topk_idx.is_cuda or topk_idx.dtype != torch.int32 or not topk_idx.is_contiguous()
            or tuple(topk_idx.shape) != (layout.N, layout.k)):
        raise FuscoError("topk_idx must be a contiguous int32 device tensor of shape [N, k]")
    _check(load_library().fusco_plan(ctypes.byref(layout.c), topk_idx.data_ptr(), layout.scratch.data_ptr(),
                                     layout.scratch.numel(), _stream(stream)), "fusco_plan")


def fusco_plan_static(layout: Layout, topk_idx: torch.Tensor, stream=None) -> None:
    """fusco_plan on the library's own static scratch array: nothing is allocated or passed in."""
    if (not topk_idx.is_cuda or topk_idx.dtype != torch.int32 or not topk_idx.is_contiguous()
            or tuple(topk_idx.shape) != (layout.N, layout.k)):
        raise FuscoError("topk_idx must be a contiguous int32 device tensor of shape [N, k]")
    _check(load_library().fusco_plan_static(ctypes.byref(layout.c), topk_idx.data_ptr(), _stream(stream)),
           "fusco_plan_static")


def fusco_dispatch(layout: Layout, x: torch.Tensor, expert_buf: Optional[torch.Tensor] = None,
                   x_aux: Optional[torch.Tensor] = None, expert_aux: Optional[torch.Tensor] = None,
                   send_buf: Optional[torch.Tensor] = None, send_aux: Optional[torch.Tensor] = None,
                   flags: int = 0, stream=None) -> None:
    rb = _rows(x, "x", layout.N)
    ab = _rows(x_aux, "x_aux", layout.N) if x_aux is not None else 0
    eff = (flags & ~DISPATCH_STREAMING) or DISPATCH_EXPERT
    if eff & DISPATCH_TWO_HOP:
        eff |= DISPATCH_EXPERT | DISPATCH_WIRE
    if eff & DISPATCH_EXPERT:
        if expert_buf is None:
            raise FuscoError("expert_buf is required")
        _rows(expert_buf, "expert_buf", layout.P, rb)
        if ab:
            if expert_aux is None:
                raise FuscoError("expert_aux is required")
            _rows(expert_aux, "expert_aux", layout.P, ab)
    if eff & DISPATCH_WIRE:
        if send_buf is None:
            raise FuscoError("send_buf is required")
        _rows(send_buf, "send_buf", layout.send_cap, rb)
        if ab:
            if send_aux is None:
                raise FuscoError("send_aux is required")
            _rows(send_aux, "send_aux", layout.send_cap, ab)
    _check(load_library().fusco_dispatch(ctypes.byref(layout.c), x.data_ptr(), rb, _ptr(x_aux), ab,
                                         _ptr(expert_buf), _ptr(expert_aux), _ptr(send_buf), _ptr(send_aux),
                                         flags, _stream(stream)), "fusco_dispatch")


def fusco_dispatch_in_transfer_order(layout: Layout, row_bytes: int, aux_row_bytes: int = 0, flags: int = 0) -> bool:
    rc = load_library().fusco_dispatch_in_transfer_order(ctypes.byref(layout.c), row_bytes, aux_row_bytes, flags)
    if rc < 0:
        _check(rc, "fusco_dispatch_in_transfer_order")
    return bool(rc)


def fusco_plan_dispatch(layout: Layout, topk_idx: torch.Tensor, x: torch.Tensor, expert_buf: torch.Tensor,
                        x_aux: Optional[torch.Tensor] = None, expert_aux: Optional[torch.Tensor] = None,
                        stream=None) -> None:
    """fusco_plan and fusco_dispatch (expert tensor only) in one launch; inputs of one planner tile only
    (N <= 2048 // k), FuscoError otherwise."""
    if (not topk_idx.is_cuda or topk_idx.dtype != torch.int32 or not topk_idx.is_contiguous()
            or tuple(topk_idx.shape) != (layout.N, layout.k)):
        raise FuscoError("topk_idx must be a contiguous int32 device tensor of shape [N, k]")
    rb = _rows(x, "x", layout.N)
    ab = _rows(x_aux, "x_aux", layout.N) if x_aux is not None else 0
    _rows(expert_buf, "expert_buf", layout.P, rb)
    if ab:
        if expert_aux is None:
            raise FuscoError("expert_aux is required")
        _rows(expert_aux, "expert_aux", layout.P, ab)
    _check(load_library().fusco_plan_dispatch(ctypes.byref(layout.c), topk_idx.data_ptr(), x.data_ptr(), rb,
                                              _ptr(x_aux), ab, expert_buf.data_ptr(), _ptr(expert_aux),
                                              _stream(stream)), "fusco_plan_dispatch")


def _dtype_code(t: torch.Tensor, name: str) -> int:
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float32:
        return F32
    raise FuscoError("%s must be bfloat16 or float32" % name)


def fusco_combine(layout: Layout, y: torch.Tensor, w: torch.Tensor, out: torch.Tensor, stream=None) -> None:
    _rows(y, "y", layout.P)
    H = y.shape[1]
    _rows(out, "out", layout.N)
    if out.shape[1] != H:
        raise FuscoError("out must have %d columns" % H)
    if (not w.is_cuda or w.dtype != torch.float32 or not w.is_contiguous()
            or tuple(w.shape) != (layout.N, layout.k)):
        raise FuscoError("w must be a contiguous float32 device tensor of shape [N, k]")
    _check(load_library().fusco_combine(ctypes.byref(layout.c), y.data_ptr(), _dtype_code(y, "y"), w.data_ptr(),
                                        out.data_ptr(), _dtype_code(out, "out"), H, 0, _stream(stream)),
           "fusco_combine")


def fusco_combine_two_hop(layout: Layout, y: torch.Tensor, w: torch.Tensor, partial: torch.Tensor,
                          out: torch.Tensor, stream=None) -> None:
    _rows(y, "y", layout.P)
    H = y.shape[1]
    _rows(out, "out", layout.N)
    _rows(partial, "partial", layout.send_cap, 4 * H)
    if partial.dtype != torch.float32:
        raise FuscoError("partial must be float32")
    if out.shape[1] != H or H % 4 != 0:
        raise FuscoError("out must have %d columns and H must be a multiple of 4" % H)
    if (not w.is_cuda or w.dtype != torch.float32 or not w.is_contiguous()
            or tuple(w.shape) != (layout.N, layout.k)):
        raise FuscoError("w must be a contiguous float32 device tensor of shape [N, k]")
    _check(load_library().fusco_combine_two_hop(ctypes.byref(layout.c), y.data_ptr(), _dtype_code(y, "y"),
                                                w.data_ptr(), partial.data_ptr(), out.data_ptr(),
                                                _dtype_code(out, "out"), H, _stream(stream)),
           "fusco_combine_two_hop")


def fusco_cross_node_load(layout: Layout, devices_per_node: int, home_node: int, row_bytes: int,
                          load: torch.Tensor, stream=None) -> None:
    """load: one-element int64 device tensor (e.g. a cell of the [nodes, gpus] load matrix)."""
    if not load.is_cuda or load.dtype != torch.int64 or load.numel() != 1:
        raise FuscoError("load must be a one-element int64 device tensor")
    _check(load_library().fusco_cross_node_load(ctypes.byref(layout.c), devices_per_node, home_node, row_bytes,
                                                load.data_ptr(), _stream(stream)), "fusco_cross_node_load")


def fusco_balance_groups(load) -> "numpy.ndarray":
    """Algorithm 1 on a host [nodes, gpus] int64 load matrix; returns group_gpu [gpus, nodes] int32."""
    import numpy as np
    load = np.ascontiguousarray(load, dtype=np.int64)
    if load.ndim != 2:
        raise FuscoError("load must be a [nodes, gpus] matrix")
    nodes, gpus = load.shape
    out = np.empty((gpus, nodes), dtype=np.int32)
    _check(load_library().fusco_balance_groups(load.ctypes.data, nodes, gpus, out.ctypes.data), "fusco_balance_groups")
    return out


def _desc_ok(desc: Optional[torch.Tensor], n: int, name: str) -> None:
    if desc is None:
        return
    if not desc.is_cuda or desc.dtype != torch.int64 or not desc.is_contiguous() or tuple(desc.shape) != (n, 2):
        raise FuscoError("%s must be a contiguous int64 device tensor of shape [n, 2] (offset, size)" % name)


def fusco_segments_scan(desc: torch.Tensor, cum: torch.Tensor, status: torch.Tensor, stream=None) -> None:
    """desc: int64 [n, 2] (offset, size) on the device; cum: int64 [n + 1]; status: int32 [1]."""
    n = desc.shape[0]
    _desc_ok(desc, n, "desc")
    if not cum.is_cuda or cum.dtype != torch.int64 or not cum.is_contiguous() or cum.numel() != n + 1:
        raise FuscoError("cum must be a contiguous int64 device tensor with n + 1 entries")
    if not status.is_cuda or status.dtype != torch.int32 or status.numel() != 1:
        raise FuscoError("status must be an int32 device tensor with one entry")
    _check(load_library().fusco_segments_scan(desc.data_ptr(), n, cum.data_ptr(), status.data_ptr(), _stream(stream)),
           "fusco_segments_scan")


def fusco_segments_copy(src: torch.Tensor, src_desc: Optional[torch.Tensor], dst: torch.Tensor,
                        dst_desc: Optional[torch.Tensor], cum: torch.Tensor, stream_capacity: int,
                        status: torch.Tensor, slice_bytes: int = 0, slice_fill: Optional[torch.Tensor] = None,
                        stream=None) -> None:
    """src / dst: contiguous device tensors viewed as bytes; a None descriptor list means that side is the
    contiguous stream.  slice_fill: int32 [ceil(stream_capacity / slice_bytes)] or None."""
    n = cum.numel() - 1
    _desc_ok(src_desc, n, "src_desc")
    _desc_ok(dst_desc, n, "dst_desc")
    if not (src.is_cuda and dst.is_cuda and src.is_contiguous() and dst.is_contiguous()):
        raise FuscoError("src and dst must be contiguous device tensors")
    if not cum.is_cuda or cum.dtype != torch.int64 or not cum.is_contiguous() or n < 0:
        raise FuscoError("cum must be a contiguous int64 device tensor with n + 1 entries")
    if not status.is_cuda or status.dtype != torch.int32 or status.numel() != 1:
        raise FuscoError("status must be an int32 device tensor with one entry")
    src_bytes, dst_bytes = src.numel() * src.element_size(), dst.numel() * dst.element_size()
    if src_desc is None and src_bytes < stream_capacity or dst_desc is None and dst_bytes < stream_capacity:
        raise FuscoError("the contiguous side is smaller than stream_capacity")
    if slice_fill is not None:
        if slice_bytes <= 0:
            raise FuscoError("slice_bytes must be positive with slice_fill")
        need = (stream_capacity + slice_bytes - 1) // slice_bytes
        if (not slice_fill.is_cuda or slice_fill.dtype != torch.int32 or not slice_fill.is_contiguous()
                or slice_fill.numel() < need):
            raise FuscoError("slice_fill must be a contiguous int32 device tensor with %d entries" % need)
    _check(load_library().fusco_segments_copy(src.data_ptr(), src_bytes, _ptr(src_desc), dst.data_ptr(), dst_bytes,
                                              _ptr(dst_desc), cum.data_ptr(), n, stream_capacity, slice_bytes,
                                              _ptr(slice_fill), status.data_ptr(), _stream(stream)),
           "fusco_segments_copy")


def fusco_probe_copy(dst: torch.Tensor, src: torch.Tensor, stream=None) -> None:
    nbytes = src.numel() * src.element_size()
    if not (dst.is_cuda and src.is_cuda and dst.is_contiguous() and src.is_contiguous()):
        raise FuscoError("probe copy needs contiguous device tensors")
    if dst.numel() * dst.element_size() < nbytes:
        raise FuscoError("dst is smaller than src")
    _check(load_library().fusco_probe_copy(dst.data_ptr(), src.data_ptr(), nbytes, _stream(stream)),
           "fusco_probe_copy")


def fusco_probe_dispatch_kernel(which: int = -1) -> int:
    """Which kernel fusco_dispatch uses where it has a choice: 0 automatic, 1 token walk, 2 transfer order wherever
    its shape allows; < 0 reads the setting.  Returns the previous setting."""
    rc = int(load_library().fusco_probe_dispatch_kernel(int(which)))
    if rc < 0:
        _check(rc, "fusco_probe_dispatch_kernel")
    return rc


def fusco_probe_dispatch_occupancy(wgs: int = -1) -> int:
    """Workgroups of the tiled dispatch per compute unit: 0 automatic, 3 ... 15 that many, 16 no cap; < 0 reads the
    setting.  Returns the previous setting."""
    rc = int(load_library().fusco_probe_dispatch_occupancy(int(wgs)))
    if rc < 0:
        _check(rc, "fusco_probe_dispatch_occupancy")
    return rc


def fusco_probe_dispatch_walk(which: int = -1) -> int:
    """Loads and stores of the token walk: 0 automatic, 1 non-temporal loads + plain stores, 2 cached loads + plain
    stores, 3 non-temporal loads and stores, 4 cached loads + non-temporal stores; < 0 reads the setting.  Returns the
    previous setting."""
    rc = int(load_library().fusco_probe_dispatch_walk(int(which)))
    if rc < 0:
        _check(rc, "fusco_probe_dispatch_walk")
    return rc


def fusco_probe_dispatch_pull(which: int = -1) -> int:
    """Whether the tiled dispatch pulls a tile's source rows towards the L2 at the start of the tile: 0 automatic,
    1 off, 2 on; < 0 reads the setting.  Returns the previous setting."""
    rc = int(load_library().fusco_probe_dispatch_pull(int(which)))
    if rc < 0:
        _check(rc, "fusco_probe_dispatch_pull")
    return rc


def fusco_probe_source_chunk_bytes(nbytes: int = 0) -> int:
    """Largest source tensor the tiled dispatch takes in one piece; a non-zero value replaces it (returns the
    previous one)."""
    return int(load_library().fusco_probe_source_chunk_bytes(int(nbytes)))


def fusco_probe_time_next_call(start: torch.cuda.Event, stop: torch.cuda.Event) -> None:
    """The next plan / dispatch / combine call of this thread records its own device time into the two events
    (created with enable_timing=True and recorded once before, so that their HIP handles exist)."""
    h0, h1 = int(start.cuda_event or 0), int(stop.cuda_event or 0)
    if not h0 or not h1:
        raise FuscoError("events must have been recorded once (torch creates the HIP event on first use)")
    _check(load_library().fusco_probe_time_next_call(h0, h1), "fusco_probe_time_next_call")


def fusco_probe_rows(src, dst, reads: int, writes: int, scatter: bool, write_through: bool = False,
                     sink: torch.Tensor | None = None, stream=None) -> None:
    """src / dst: 2-D contiguous device tensors of rows with the same row size in bytes (either may be None
    when its side is unused); sink: one int32 on the device, needed for the read-only shape."""
    rows, row_bytes = [0, 0], 0
    for i, t in enumerate((src, dst)):
        if t is None:
            continue
        if not t.is_cuda or t.dim() != 2 or not t.is_contiguous():
            raise FuscoError("probe rows needs 2-D contiguous device tensors")
        rb = t.shape[1] * t.element_size()
        if row_bytes and rb != row_bytes:
            raise FuscoError("src and dst rows differ in size")
        rows[i], row_bytes = t.shape[0], rb
    if sink is not None and (not sink.is_cuda or sink.numel() < 1 or sink.element_size() != 4):
        raise FuscoError("sink must be one 32-bit word on the device")
    _check(load_library().fusco_probe_rows(_ptr(src), rows[0], _ptr(dst), rows[1], row_bytes, int(reads), int(writes),
                                           int(bool(scatter)), int(bool(write_through)), _ptr(sink), _stream(stream)),
           "fusco_probe_rows")


def fusco_probe_pieces(buf: torch.Tensor, write: bool, run_pieces: int = 1, scatter: bool = False,
                       sink: torch.Tensor | None = None, stream=None) -> None:
    """buf: contiguous device tensor whose size is a multiple of 4096 bytes; see fusco_probe.h."""
    if not buf.is_cuda or not buf.is_contiguous():
        raise FuscoError("probe pieces needs a contiguous device tensor")
    if sink is not None and (not sink.is_cuda or sink.numel() < 1 or sink.element_size() != 4):
        raise FuscoError("sink must be one 32-bit word on the device")
    _check(load_library().fusco_probe_pieces(buf.data_ptr(), buf.numel() * buf.element_size(), int(bool(write)),
                                             int(run_pieces), int(bool(scatter)), _ptr(sink), _stream(stream)),
           "fusco_probe_pieces")


def fusco_probe_consume_slices(packed: torch.Tensor, total_bytes: int, slice_bytes: int, slice_fill: torch.Tensor,
                               max_polls: int, report: torch.Tensor, stream=None) -> None:
    """report: int32 [slices, 4] on the device (ready, polls, checksum low, checksum high per slice)."""
    slices = (total_bytes + slice_bytes - 1) // slice_bytes if slice_bytes > 0 else 0
    if not packed.is_cuda or not packed.is_contiguous() or packed.numel() * packed.element_size() < total_bytes:
        raise FuscoError("packed must be a contiguous device tensor of at least total_bytes")
    if not slice_fill.is_cuda or slice_fill.dtype != torch.int32 or slice_fill.numel() < slices:
        raise FuscoError("slice_fill must be an int32 device tensor with one entry per slice")
    if not report.is_cuda or report.dtype != torch.int32 or not report.is_contiguous() or report.numel() < 4 * slices:
        raise FuscoError("report must be a contiguous int32 device tensor of shape [slices, 4]")
    _check(load_library().fusco_probe_consume_slices(packed.data_ptr(), total_bytes, slice_bytes, slice_fill.data_ptr(),
                                                     max_polls, report.data_ptr(), _stream(stream)),
           "fusco_probe_consume_slices")


def fusco_disaggregated_plan(rank_layout: Layout, layout: Layout, topk_idx: torch.Tensor, topk_dev: torch.Tensor,
                             stream=None) -> None:
    """rank_layout must be Layout(N, k, D, D); topk_dev is an int32 [N, k] scratch tensor."""
    for t, name in ((topk_idx, "topk_idx"), (topk_dev, "topk_dev")):
        if (not t.is_cuda or t.dtype != torch.int32 or not t.is_contiguous()
                or tuple(t.shape) != (layout.N, layout.k)):
            raise FuscoError("%s must be a contiguous int32 device tensor of shape [N, k]" % name)
    _check(load_library().fusco_disaggregated_plan(ctypes.byref(rank_layout.c), ctypes.byref(layout.c),
                                                   topk_idx.data_ptr(), topk_dev.data_ptr(),
                                                   rank_layout.scratch.data_ptr(), rank_layout.scratch.numel(),
                                                   _stream(stream)), "fusco_disaggregated_plan")


def fusco_disaggregated_dispatch(layout: Layout, rank_layout: Layout, x: torch.Tensor, stage_a: torch.Tensor,
                                 stage_b: torch.Tensor, expert_buf: torch.Tensor, stream=None) -> None:
    rb = _rows(x, "x", layout.N)
    for t, name in ((stage_a, "stage_a"), (stage_b, "stage_b"), (expert_buf, "expert_buf")):
        _rows(t, name, layout.P, rb)
    _check(load_library().fusco_disaggregated_dispatch(ctypes.byref(layout.c), ctypes.byref(rank_layout.c),
                                                       x.data_ptr(), rb, stage_a.data_ptr(), stage_b.data_ptr(),
                                                       expert_buf.data_ptr(), _stream(stream)),
           "fusco_disaggregated_dispatch")


def fusco_disaggregated_combine(layout: Layout, rank_layout: Layout, y: torch.Tensor, w: torch.Tensor,
                                stage_a: torch.Tensor, stage_b: torch.Tensor, out: torch.Tensor, stream=None) -> None:
    rb = _rows(y, "y", layout.P)
    H = y.shape[1]
    for t, name in ((stage_a, "stage_a"), (stage_b, "stage_b")):
        _rows(t, name, layout.P, rb)
    _rows(out, "out", layout.N)
    if out.shape[1] != H:
        raise FuscoError("out must have %d columns" % H)
    if (not w.is_cuda or w.dtype != torch.float32 or not w.is_contiguous()
            or tuple(w.shape) != (layout.N, layout.k)):
        raise FuscoError("w must be a contiguous float32 device tensor of shape [N, k]")
    _check(load_library().fusco_disaggregated_combine(ctypes.byref(layout.c), ctypes.byref(rank_layout.c),
                                                      y.data_ptr(), _dtype_code(y, "y"), w.data_ptr(),
                                                      stage_a.data_ptr(), stage_b.data_ptr(), out.data_ptr(),
                                                      _dtype_code(out, "out"), H, _stream(stream)),
           "fusco_disaggregated_combine")
