"""ctypes binding of libmoe_hip.so (the C ABI of include/moe.h).

Only argument marshalling happens here: tensors are checked (device, dtype,
contiguity, shape), outputs and workspaces are allocated with torch, raw
pointers and the current HIP stream are handed to the library.  Every step of
the layer runs in the library's kernels.  If the library cannot be loaded the
import of a symbol fails loudly; there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

from . import build as _build

_i32, _i64, _vp, _sz = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t

DTYPE_F32, DTYPE_BF16 = 0, 1
MAX_EXPERTS = 64


class MoEShape(ctypes.Structure):
    """struct moe_shape: T, H (h1), F (h2), E (n_e), k, dtype, page_bytes."""
    _fields_ = [("T", _i32), ("H", _i32), ("F", _i32), ("E", _i32), ("k", _i32), ("dtype", _i32),
                ("page_bytes", _i64)]

    @property
    def R(self) -> int:
        return self.T * self.k

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == DTYPE_BF16 else torch.float32

    def with_tokens(self, T: int) -> "MoEShape":
        return MoEShape(T, self.H, self.F, self.E, self.k, self.dtype, self.page_bytes)


class WorkspaceLayout(ctypes.Structure):
    _fields_ = [(n, _sz) for n in ("status", "topk_ids", "topk_w", "counts", "offsets", "row_src", "row_of", "row_w",
                                   "scan", "x_perm", "h", "out", "total", "permute_bytes")]


class MoEError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = _lib().moe_status_string(status).decode()
        if status == -5:
            msg += " (hipError %d)" % _lib().moe_last_hip_error()
        super().__init__("%s: %s [%d]" % (where, msg, status))


ERR_INVALID_ARG, ERR_UNSUPPORTED_DTYPE, ERR_WORKSPACE_TOO_SMALL, ERR_PAGE_NOT_RESIDENT, ERR_HIP = -1, -2, -3, -4, -5

_SIGNATURES = {
    "moe_status_string": (ctypes.c_char_p, [ctypes.c_int]),
    "moe_last_hip_error": (ctypes.c_int, []),
    "moe_validate_shape": (ctypes.c_int, [_vp]),
    "moe_tile_bytes": (ctypes.c_int, [_vp, _vp]),
    "moe_pages_required": (ctypes.c_int, [_vp, _vp, _vp]),
    "moe_pack_weights": (ctypes.c_int, [_vp, _vp, _vp, _vp, _vp, _i64, _vp]),
    "moe_unpack_weights": (ctypes.c_int, [_vp, _vp, _vp, _i64, _vp, _vp, _vp]),
    "moe_page_table_validate": (ctypes.c_int, [_vp, _vp, _i64]),
    "moe_workspace_layout_get": (ctypes.c_int, [_vp, _vp]),
    "moe_route": (ctypes.c_int, [_vp] * 8),
    "moe_permute": (ctypes.c_int, [_vp] * 11 + [_sz, _vp]),
    "moe_expert_ffn": (ctypes.c_int, [_vp] * 5 + [_i64] + [_vp] * 5),
    "moe_combine": (ctypes.c_int, [_vp] * 6),
    "moe_layer": (ctypes.c_int, [_vp] * 6 + [_i64, _vp, _vp, _sz, _vp]),
    "moe_layer_static": (ctypes.c_int, [_vp] * 6 + [_i64, _vp, _vp]),
    "moe_stream_create": (ctypes.c_int, [_vp, _vp, _i64, _vp, _vp, _vp, _vp]),
    "moe_stream_destroy": (ctypes.c_int, [_vp]),
    "moe_expert_ffn_streamed": (ctypes.c_int, [_vp] * 9),
    "moe_layer_streamed": (ctypes.c_int, [_vp] * 6 + [_sz, _vp, _vp]),
    "moe_pipeline_pool_pages": (ctypes.c_int, [_vp, ctypes.c_int32, ctypes.c_int32, _vp]),
    "moe_pipeline_create": (ctypes.c_int, [_vp, ctypes.c_int32, ctypes.c_int32, _vp, _vp, _vp, ctypes.c_int32, _vp, _i64, _vp, _vp]),
    "moe_pipeline_destroy": (ctypes.c_int, [_vp]),
    "moe_pipeline_run": (ctypes.c_int, [_vp, ctypes.c_int32, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp, _vp]),
    "moe_linear_pages_required": (ctypes.c_int, [_vp, _vp]),
    "moe_linear_pack": (ctypes.c_int, [_vp, _vp, _vp, _i64, _vp]),
    "moe_linear": (ctypes.c_int, [_vp] * 4 + [_i64, _vp, _vp, _sz, _vp, _vp]),
    "moe_add_rmsnorm": (ctypes.c_int, [ctypes.c_int32, ctypes.c_int32, _vp, _vp, _vp, ctypes.c_float, _vp, _vp, _vp]),
    "moe_cast_bf16": (ctypes.c_int, [_i64, _vp, _vp, _vp]),
    "moe_post_attention_workspace_bytes": (ctypes.c_int, [_vp, _vp]),
    "moe_post_attention": (ctypes.c_int, [_vp] * 6 + [ctypes.c_float] + [_vp] * 4 + [_i64] + [_vp] * 4 + [_sz, _vp]),
    "moe_pre_attention": (ctypes.c_int, [_vp] * 4 + [ctypes.c_float, _vp, _vp, _i64] + [_vp] * 5 + [_sz, _vp]),
    "moe_set_option": (ctypes.c_int, [ctypes.c_char_p, ctypes.c_int]),
    "moe_get_option": (ctypes.c_int, [ctypes.c_char_p, _vp]),
    "moe_profile_read": (ctypes.c_int, [_vp, _vp]),
    "moe_probe_stream_read": (ctypes.c_int, [_vp, _sz, ctypes.c_int32, _vp, _vp]),
}
EXPORTED_SYMBOLS = tuple(_SIGNATURES)

_LIB = None


def library_path() -> str:
    return _build.LIB


def _lib():
    global _LIB
    if _LIB is None:
        path = os.environ.get("MOE_HIP_LIBRARY")     # override: an experimental build of the same ABI
        if path is not None:
            if not os.path.exists(path):
                raise FileNotFoundError(f"MOE_HIP_LIBRARY names {path!r}, which does not exist")
        else:
            path = _build.LIB
            if not os.path.exists(path):
                path = _build.build(force=True)      # raises if hipcc is missing or the build fails
        lib = ctypes.CDLL(path)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(lib, name)                   # AttributeError if a declared symbol is missing
            fn.restype, fn.argtypes = res, args
        _LIB = lib
    return _LIB


def _check(status: int, where: str):
    if status != 0:
        raise MoEError(status, where)


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _dev(t: Optional[torch.Tensor], dtype, shape, name: str) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name}: must be a CUDA/HIP device tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name}: expected {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name}: must be contiguous")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: expected shape {tuple(shape)}, got {tuple(t.shape)}")
    return t.data_ptr()


def make_shape(T, H, F, E, k, dtype, page_bytes) -> MoEShape:
    code = {"f32": 0, "bf16": 1, torch.float32: 0, torch.bfloat16: 1, 0: 0, 1: 1}[dtype]
    return MoEShape(int(T), int(H), int(F), int(E), int(k), code, int(page_bytes))


def validate_shape(s: MoEShape) -> int:
    return _lib().moe_validate_shape(ctypes.byref(s))


def tile_bytes(s: MoEShape) -> int:
    v = _i64(0)
    _check(_lib().moe_tile_bytes(ctypes.byref(s), ctypes.byref(v)), "moe_tile_bytes")
    return v.value


def pages_required(s: MoEShape):
    """(pages_gu, pages_d) per expert."""
    a, b = _i64(0), _i64(0)
    _check(_lib().moe_pages_required(ctypes.byref(s), ctypes.byref(a), ctypes.byref(b)), "moe_pages_required")
    return a.value, b.value


def workspace_layout(s: MoEShape) -> WorkspaceLayout:
    L = WorkspaceLayout()
    _check(_lib().moe_workspace_layout_get(ctypes.byref(s), ctypes.byref(L)), "moe_workspace_layout_get")
    return L


def set_option(name: str, value: int):
    _check(_lib().moe_set_option(name.encode(), int(value)), "moe_set_option(%s)" % name)


def get_option(name: str) -> int:
    v = ctypes.c_int(0)
    _check(_lib().moe_get_option(name.encode(), ctypes.byref(v)), "moe_get_option(%s)" % name)
    return v.value


PROFILE_STAGES = ("route", "permute", "gemm_gate_up", "gemm_down", "combine")


def profile_read():
    """Average stage durations (ms) of the moe_layer calls made while option "profile" was 1,
    as (dict stage -> ms, n_calls).  Synchronise the stream first."""
    arr = (ctypes.c_double * len(PROFILE_STAGES))()
    n = ctypes.c_int(0)
    _check(_lib().moe_profile_read(arr, ctypes.byref(n)), "moe_profile_read")
    return {name: arr[i] for i, name in enumerate(PROFILE_STAGES)}, n.value


# ----------------------------------------------------------------------------- paged weights

def _host(t: torch.Tensor, dtype, shape, name):
    if t.is_cuda:
        raise ValueError(f"{name}: must be a host tensor")
    if t.dtype != dtype or not t.is_contiguous() or tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: expected contiguous {dtype} of shape {tuple(shape)}")
    return t.data_ptr()


def page_table_validate(s: MoEShape, page_table_host: torch.Tensor, pool_pages: int):
    gu, d = pages_required(s)
    p = _host(page_table_host, torch.int32, (s.E, gu + d), "page_table")
    _check(_lib().moe_page_table_validate(ctypes.byref(s), p, int(pool_pages)), "moe_page_table_validate")


def pack_weights(s: MoEShape, W1, W3, W2, page_table: torch.Tensor, pool_pages: int, pin: bool = False) -> torch.Tensor:
    """Host packer: dense W1/W3 [E,F,H], W2 [E,H,F] -> uint8 [pool_pages, page_bytes] (optionally pinned)."""
    gu, d = pages_required(s)
    dt = s.torch_dtype
    p1 = _host(W1, dt, (s.E, s.F, s.H), "W1")
    p3 = _host(W3, dt, (s.E, s.F, s.H), "W3")
    p2 = _host(W2, dt, (s.E, s.H, s.F), "W2")
    pt = _host(page_table, torch.int32, (s.E, gu + d), "page_table")
    pages = torch.zeros((int(pool_pages), s.page_bytes), dtype=torch.uint8, pin_memory=pin)
    _check(_lib().moe_pack_weights(ctypes.byref(s), p1, p3, p2, pt, int(pool_pages), pages.data_ptr()), "moe_pack_weights")
    return pages


def unpack_weights(s: MoEShape, pages: torch.Tensor, page_table: torch.Tensor):
    gu, d = pages_required(s)
    dt = s.torch_dtype
    pool_pages = pages.shape[0]
    pg = _host(pages, torch.uint8, (pool_pages, s.page_bytes), "pages")
    pt = _host(page_table, torch.int32, (s.E, gu + d), "page_table")
    W1 = torch.zeros((s.E, s.F, s.H), dtype=dt)
    W3 = torch.zeros((s.E, s.F, s.H), dtype=dt)
    W2 = torch.zeros((s.E, s.H, s.F), dtype=dt)
    _check(_lib().moe_unpack_weights(ctypes.byref(s), pg, pt, int(pool_pages), W1.data_ptr(), W3.data_ptr(), W2.data_ptr()),
           "moe_unpack_weights")
    return W1, W3, W2


# ----------------------------------------------------------------------------- the five calls

def moe_route(s: MoEShape, x, Wr, bias=None, want_logits: bool = False, stream=None):
    """-> (topk_ids int32 [T,k], topk_w float32 [T,k], logits float32 [T,E] or None)"""
    dt = s.torch_dtype
    px = _dev(x, dt, (s.T, s.H), "x")
    pw = _dev(Wr, dt, (s.E, s.H), "Wr")
    pb = _dev(bias, torch.float32, (s.E,), "bias")
    ids = torch.empty((s.T, s.k), dtype=torch.int32, device=x.device)
    w = torch.empty((s.T, s.k), dtype=torch.float32, device=x.device)
    logits = torch.empty((s.T, s.E), dtype=torch.float32, device=x.device) if want_logits else None
    _check(_lib().moe_route(ctypes.byref(s), px, pw, pb, ids.data_ptr(), w.data_ptr(),
                            None if logits is None else logits.data_ptr(), _stream(stream)), "moe_route")
    return ids, w, logits


def moe_permute(s: MoEShape, topk_ids, x=None, topk_w=None, stream=None):
    """-> dict(counts[E], offsets[E+1], row_src[R], row_of[R], row_w[R] or None, x_perm[R,H] or None)"""
    dev = topk_ids.device
    pi = _dev(topk_ids, torch.int32, (s.T, s.k), "topk_ids")
    pw = _dev(topk_w, torch.float32, (s.T, s.k), "topk_w")
    px = _dev(x, s.torch_dtype, (s.T, s.H), "x")
    R = s.R
    counts = torch.empty(s.E, dtype=torch.int32, device=dev)
    offsets = torch.empty(s.E + 1, dtype=torch.int32, device=dev)
    row_src = torch.empty(R, dtype=torch.int32, device=dev)
    row_of = torch.empty(R, dtype=torch.int32, device=dev)
    row_w = torch.empty(R, dtype=torch.float32, device=dev) if topk_w is not None else None
    x_perm = torch.empty((R, s.H), dtype=s.torch_dtype, device=dev) if x is not None else None
    wsb = workspace_layout(s).permute_bytes
    ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device=dev)
    _check(_lib().moe_permute(ctypes.byref(s), pi, pw, px, counts.data_ptr(), offsets.data_ptr(), row_src.data_ptr(),
                              row_of.data_ptr(), None if row_w is None else row_w.data_ptr(),
                              None if x_perm is None else x_perm.data_ptr(), ws.data_ptr(), ws.numel(),
                              _stream(stream)), "moe_permute")
    return dict(counts=counts, offsets=offsets, row_src=row_src, row_of=row_of, row_w=row_w, x_perm=x_perm)


def moe_expert_ffn(s: MoEShape, x_perm, offsets, page_table, page_pool, row_w=None, status=None, stream=None):
    """-> (h [R,F] dtype, out [R,H] float32)"""
    dev = x_perm.device
    R = s.R
    gu, d = pages_required(s)
    px = _dev(x_perm, s.torch_dtype, (R, s.H), "x_perm")
    po = _dev(offsets, torch.int32, (s.E + 1,), "offsets")
    pt = _dev(page_table, torch.int32, (s.E, gu + d), "page_table")
    pp = _dev(page_pool, torch.uint8, None, "page_pool")
    if page_pool.dim() != 2 or page_pool.shape[1] != s.page_bytes:
        raise ValueError("page_pool: expected uint8 [pool_pages, page_bytes]")
    pr = _dev(row_w, torch.float32, (R,), "row_w")
    ps = _dev(status, torch.int32, (4,), "status")
    h = torch.empty((R, s.F), dtype=s.torch_dtype, device=dev)
    out = torch.empty((R, s.H), dtype=torch.float32, device=dev)
    _check(_lib().moe_expert_ffn(ctypes.byref(s), px, po, pt, pp, int(page_pool.shape[0]), pr, h.data_ptr(),
                                 out.data_ptr(), ps, _stream(stream)), "moe_expert_ffn")
    return h, out


def moe_combine(s: MoEShape, out, row_of, topk_w=None, stream=None):
    """-> y float32 [T,H]"""
    po = _dev(out, torch.float32, (s.R, s.H), "out")
    pr = _dev(row_of, torch.int32, (s.R,), "row_of")
    pw = _dev(topk_w, torch.float32, (s.T, s.k), "topk_w")
    y = torch.empty((s.T, s.H), dtype=torch.float32, device=out.device)
    _check(_lib().moe_combine(ctypes.byref(s), po, pr, pw, y.data_ptr(), _stream(stream)), "moe_combine")
    return y


class Workspace:
    """Device scratch of moe_layer plus typed views of the intermediates it leaves behind."""

    def __init__(self, s: MoEShape, device="cuda"):
        self.shape = s
        self.layout = workspace_layout(s)
        self.buf = torch.empty(max(self.layout.total, 256), dtype=torch.uint8, device=device)
        if self.buf.data_ptr() % 256:
            raise RuntimeError("allocator returned an unaligned workspace")

    def view(self, name: str) -> torch.Tensor:
        s, L = self.shape, self.layout
        R = s.R
        esz = 2 if s.dtype == DTYPE_BF16 else 4
        spec = {
            "status": (torch.int32, (4,), 16), "topk_ids": (torch.int32, (s.T, s.k), R * 4),
            "topk_w": (torch.float32, (s.T, s.k), R * 4), "counts": (torch.int32, (s.E,), s.E * 4),
            "offsets": (torch.int32, (s.E + 1,), (s.E + 1) * 4), "row_src": (torch.int32, (R,), R * 4),
            "row_of": (torch.int32, (R,), R * 4), "row_w": (torch.float32, (R,), R * 4),
            "x_perm": (s.torch_dtype, (R, s.H), R * s.H * esz), "h": (s.torch_dtype, (R, s.F), R * s.F * esz),
            "out": (torch.float32, (R, s.H), R * s.H * 4),
        }[name]
        off = getattr(L, name)
        return self.buf[off:off + spec[2]].view(spec[0]).view(spec[1])


def moe_layer(s: MoEShape, x, Wr, page_table, page_pool, bias=None, workspace: Optional[Workspace] = None,
              y: Optional[torch.Tensor] = None, stream=None):
    """-> (y float32 [T,H], workspace)"""
    gu, d = pages_required(s)
    dt = s.torch_dtype
    px = _dev(x, dt, (s.T, s.H), "x")
    pw = _dev(Wr, dt, (s.E, s.H), "Wr")
    pb = _dev(bias, torch.float32, (s.E,), "bias")
    pt = _dev(page_table, torch.int32, (s.E, gu + d), "page_table")
    pp = _dev(page_pool, torch.uint8, None, "page_pool")
    if page_pool.dim() != 2 or page_pool.shape[1] != s.page_bytes:
        raise ValueError("page_pool: expected uint8 [pool_pages, page_bytes]")
    if workspace is None:
        workspace = Workspace(s, x.device)
    if y is None:
        y = torch.empty((s.T, s.H), dtype=torch.float32, device=x.device)
    _dev(y, torch.float32, (s.T, s.H), "y")
    _check(_lib().moe_layer(ctypes.byref(s), px, pw, pb, pt, pp, int(page_pool.shape[0]), y.data_ptr(),
                            workspace.buf.data_ptr(), workspace.buf.numel(), _stream(stream)), "moe_layer")
    return y, workspace


def probe_stream_read(buf: torch.Tensor, blocks: int = 2048, stream=None):
    """Enqueues one launch that reads all of the device tensor buf once (measurement helper)."""
    nbytes = buf.numel() * buf.element_size()
    _check(_lib().moe_probe_stream_read(buf.data_ptr(), nbytes, int(blocks), None, _stream(stream)), "moe_probe_stream_read")


STATIC_SCRATCH_BYTES = 32 << 20


def moe_layer_static(s: MoEShape, x, Wr, page_table, page_pool, y: torch.Tensor, bias=None, stream=None):
    """moe_layer on the library's own device scratch: nothing is allocated, y is the caller's float32 [T,H]."""
    gu, d = pages_required(s)
    dt = s.torch_dtype
    px = _dev(x, dt, (s.T, s.H), "x")
    pw = _dev(Wr, dt, (s.E, s.H), "Wr")
    pb = _dev(bias, torch.float32, (s.E,), "bias")
    pt = _dev(page_table, torch.int32, (s.E, gu + d), "page_table")
    pp = _dev(page_pool, torch.uint8, None, "page_pool")
    if page_pool.dim() != 2 or page_pool.shape[1] != s.page_bytes:
        raise ValueError("page_pool: expected uint8 [pool_pages, page_bytes]")
    py = _dev(y, torch.float32, (s.T, s.H), "y")
    _check(_lib().moe_layer_static(ctypes.byref(s), px, pw, pb, pt, pp, int(page_pool.shape[0]), py, _stream(stream)),
           "moe_layer_static")
    return y


# ----------------------------------------------------------------------------- streamed pages

class Streamer:
    """Expert pages in pinned host memory, streamed through a two-slot device region."""

    def __init__(self, s: MoEShape, host_pages: torch.Tensor, host_page_table: torch.Tensor, device="cuda"):
        gu, d = pages_required(s)
        self.shape, self.ppe = s, gu + d
        if not host_pages.is_pinned():
            raise ValueError("host_pages must be pinned host memory")
        pg = _host(host_pages, torch.uint8, (host_pages.shape[0], s.page_bytes), "host_pages")
        pt = _host(host_page_table, torch.int32, (s.E, self.ppe), "host_page_table")
        self.host_pages, self.host_page_table = host_pages, host_page_table
        self.slots = torch.empty((2 * self.ppe, s.page_bytes), dtype=torch.uint8, device=device)
        self.slot_table = torch.empty((2, self.ppe), dtype=torch.int32, device=device)
        self.copy_stream = torch.cuda.Stream(device=device)
        handle = _vp(0)
        _check(_lib().moe_stream_create(ctypes.byref(s), pg, int(host_pages.shape[0]), pt, self.slots.data_ptr(),
                                        self.slot_table.data_ptr(), ctypes.byref(handle)), "moe_stream_create")
        self.handle = handle

    def close(self):
        if self.handle:
            torch.cuda.synchronize()
            _check(_lib().moe_stream_destroy(self.handle), "moe_stream_destroy")
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def moe_expert_ffn_streamed(st: Streamer, x_perm, offsets, row_w=None, status=None, stream=None):
    s = st.shape
    R = s.R
    px = _dev(x_perm, s.torch_dtype, (R, s.H), "x_perm")
    po = _dev(offsets, torch.int32, (s.E + 1,), "offsets")
    pr = _dev(row_w, torch.float32, (R,), "row_w")
    ps = _dev(status, torch.int32, (4,), "status")
    h = torch.empty((R, s.F), dtype=s.torch_dtype, device=x_perm.device)
    out = torch.empty((R, s.H), dtype=torch.float32, device=x_perm.device)
    _check(_lib().moe_expert_ffn_streamed(st.handle, px, po, pr, h.data_ptr(), out.data_ptr(), ps, _stream(stream),
                                          st.copy_stream.cuda_stream), "moe_expert_ffn_streamed")
    return h, out


def moe_layer_streamed(st: Streamer, x, Wr, bias=None, workspace: Optional[Workspace] = None,
                       y: Optional[torch.Tensor] = None, stream=None):
    s = st.shape
    dt = s.torch_dtype
    px = _dev(x, dt, (s.T, s.H), "x")
    pw = _dev(Wr, dt, (s.E, s.H), "Wr")
    pb = _dev(bias, torch.float32, (s.E,), "bias")
    if workspace is None:
        workspace = Workspace(s, x.device)
    if y is None:
        y = torch.empty((s.T, s.H), dtype=torch.float32, device=x.device)
    _dev(y, torch.float32, (s.T, s.H), "y")
    _check(_lib().moe_layer_streamed(st.handle, px, pw, pb, y.data_ptr(), workspace.buf.data_ptr(),
                                     workspace.buf.numel(), _stream(stream), st.copy_stream.cuda_stream),
           "moe_layer_streamed")
    return y, workspace


# ----------------------------------------------------------------------------- weight paging over several layers

def pipeline_pool_pages(s: MoEShape, n_layers: int, resident_pages_per_expert: int) -> int:
    v = _i64(0)
    _check(_lib().moe_pipeline_pool_pages(ctypes.byref(s), int(n_layers), int(resident_pages_per_expert), ctypes.byref(v)),
           "moe_pipeline_pool_pages")
    return int(v.value)


class Pipeline:
    """A stack of MoE layers whose non-resident pages are streamed layer by layer (include/moe.h,
    "weight paging over several layers").  ``layers``: one (host_pages pinned uint8 [pool, page_bytes],
    host_page_table int32 [E, pages_per_expert]) pair per layer."""

    def __init__(self, s: MoEShape, layers, resident_pages_per_expert: int, max_micro_batches: int, device="cuda"):
        gu, d = pages_required(s)
        self.shape, self.ppe, self.n_layers = s, gu + d, len(layers)
        self.max_micro = int(max_micro_batches)
        self.layers = list(layers)
        for hp, ht in self.layers:
            if not hp.is_pinned():
                raise ValueError("host pages must be pinned host memory")
            _host(hp, torch.uint8, (hp.shape[0], s.page_bytes), "host_pages")
            _host(ht, torch.int32, (s.E, self.ppe), "host_page_table")
        L = self.n_layers
        self.pool_pages = pipeline_pool_pages(s, L, resident_pages_per_expert)
        self.pool = torch.empty((self.pool_pages, s.page_bytes), dtype=torch.uint8, device=device)
        self.tables = torch.empty((L, 2, s.E, self.ppe), dtype=torch.int32, device=device)
        self.copy_stream = torch.cuda.Stream(device=device)
        pages = (_vp * L)(*[hp.data_ptr() for hp, _ in self.layers])
        counts = (_i64 * L)(*[int(hp.shape[0]) for hp, _ in self.layers])
        tables = (_vp * L)(*[ht.data_ptr() for _, ht in self.layers])
        handle = _vp(0)
        _check(_lib().moe_pipeline_create(ctypes.byref(s), L, self.max_micro, pages, counts, tables,
                                          int(resident_pages_per_expert), self.pool.data_ptr(), self.pool_pages,
                                          self.tables.data_ptr(), ctypes.byref(handle)), "moe_pipeline_create")
        self.handle = handle

    def run(self, x_host, Wr, y, x_dev: Optional[torch.Tensor] = None, bias=None,
            workspace: Optional[Workspace] = None, stream=None):
        """x_host[l][j]: pinned host [T,H]; Wr[l]: device [E,H]; y[l][j]: device float32 [T,H]."""
        s, L = self.shape, self.n_layers
        n = len(x_host[0])
        dt = s.torch_dtype
        if x_dev is None:
            x_dev = torch.empty((n, s.T, s.H), dtype=dt, device=self.pool.device)
        _dev(x_dev, dt, (n, s.T, s.H), "x_dev")
        if workspace is None:
            workspace = Workspace(s, self.pool.device)
        xs, ys = [], []
        for l in range(L):
            if len(x_host[l]) != n or len(y[l]) != n:
                raise ValueError("every layer needs the same number of micro-batches")
            for j in range(n):
                if not x_host[l][j].is_pinned():
                    raise ValueError("x_host must be pinned host memory")
                xs.append(_host(x_host[l][j], dt, (s.T, s.H), "x_host"))
                ys.append(_dev(y[l][j], torch.float32, (s.T, s.H), "y"))
        wr = [_dev(Wr[l], dt, (s.E, s.H), "Wr") for l in range(L)]
        pb = None
        if bias is not None:
            pb = (_vp * L)(*[_dev(b, torch.float32, (s.E,), "bias") for b in bias])
        _check(_lib().moe_pipeline_run(self.handle, n, (_vp * (L * n))(*xs), x_dev.data_ptr(), (_vp * L)(*wr), pb,
                                       (_vp * (L * n))(*ys), workspace.buf.data_ptr(), workspace.buf.numel(),
                                       _stream(stream), self.copy_stream.cuda_stream), "moe_pipeline_run")
        self._keep = (x_host, x_dev, workspace)      # the enqueued work reads these
        return workspace

    def close(self):
        if self.handle:
            torch.cuda.synchronize()
            _check(_lib().moe_pipeline_destroy(self.handle), "moe_pipeline_destroy")
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# ----------------------------------------------------------------------------- dense neighbours of the layer

class LinearShape(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int32), ("K", ctypes.c_int32), ("N", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("page_bytes", ctypes.c_int64)]


def make_linear_shape(T, K, N, page_bytes) -> LinearShape:
    return LinearShape(int(T), int(K), int(N), DTYPE_BF16, int(page_bytes))


def linear_pages_required(ls: LinearShape) -> int:
    v = _i64(0)
    _check(_lib().moe_linear_pages_required(ctypes.byref(ls), ctypes.byref(v)), "moe_linear_pages_required")
    return int(v.value)


def linear_pack(ls: LinearShape, W: torch.Tensor, page_table: torch.Tensor, pages_out: torch.Tensor):
    """Writes the pages of W (host bf16 [N,K]) into pages_out (host uint8 [pool_pages, page_bytes]) at the slots
    page_table (host int32 [pages]) names."""
    n = linear_pages_required(ls)
    pw = _host(W, torch.bfloat16, (ls.N, ls.K), "W")
    pt = _host(page_table, torch.int32, (n,), "page_table")
    pp = _host(pages_out, torch.uint8, (pages_out.shape[0], ls.page_bytes), "pages_out")
    _check(_lib().moe_linear_pack(ctypes.byref(ls), pw, pt, int(pages_out.shape[0]), pp), "moe_linear_pack")


def moe_linear(ls: LinearShape, x, page_table, page_pool, status=None, stream=None) -> torch.Tensor:
    px = _dev(x, torch.bfloat16, (ls.T, ls.K), "x")
    pt = _dev(page_table, torch.int32, (linear_pages_required(ls),), "page_table")
    pp = _dev(page_pool, torch.uint8, None, "page_pool")
    ps = _dev(status, torch.int32, (4,), "status")
    out = torch.empty((ls.T, ls.N), dtype=torch.float32, device=x.device)
    ws = torch.empty(16, dtype=torch.uint8, device=x.device)
    _check(_lib().moe_linear(ctypes.byref(ls), px, pt, pp, int(page_pool.shape[0]), out.data_ptr(), ws.data_ptr(), 16, ps,
                             _stream(stream)), "moe_linear")
    return out


def moe_add_rmsnorm(hidden, delta, gamma, eps: float, want_hidden: bool = True, stream=None):
    """-> (hidden + delta as float32 or None, bf16 normalised rows)"""
    T, H = delta.shape
    ph = _dev(hidden, torch.float32, (T, H), "hidden")
    pd = _dev(delta, torch.float32, (T, H), "delta")
    pg = _dev(gamma, torch.float32, (H,), "gamma")
    hs = torch.empty((T, H), dtype=torch.float32, device=delta.device) if want_hidden else None
    x = torch.empty((T, H), dtype=torch.bfloat16, device=delta.device)
    _check(_lib().moe_add_rmsnorm(T, H, ph, pd, pg, float(eps), None if hs is None else hs.data_ptr(), x.data_ptr(),
                                  _stream(stream)), "moe_add_rmsnorm")
    return hs, x


def moe_cast_bf16(t: torch.Tensor, stream=None) -> torch.Tensor:
    _dev(t, torch.float32, None, "in")
    out = torch.empty(t.shape, dtype=torch.bfloat16, device=t.device)
    _check(_lib().moe_cast_bf16(t.numel(), t.data_ptr(), out.data_ptr(), _stream(stream)), "moe_cast_bf16")
    return out


def post_attention_workspace_bytes(s: MoEShape) -> int:
    v = _sz(0)
    _check(_lib().moe_post_attention_workspace_bytes(ctypes.byref(s), ctypes.byref(v)), "moe_post_attention_workspace_bytes")
    return int(v.value)


def moe_post_attention(s: MoEShape, o_proj: LinearShape, attn, hidden, o_table, norm_gamma, eps, Wr, page_table, page_pool,
                       bias=None, stream=None):
    """-> (hidden_mid f32, x_moe bf16, y f32, workspace bytes tensor)"""
    gu, d = pages_required(s)
    pa = _dev(attn, torch.bfloat16, (s.T, o_proj.K), "attn")
    ph = _dev(hidden, torch.float32, (s.T, s.H), "hidden")
    po = _dev(o_table, torch.int32, (linear_pages_required(o_proj),), "o_table")
    pg = _dev(norm_gamma, torch.float32, (s.H,), "norm_gamma")
    pw = _dev(Wr, torch.bfloat16, (s.E, s.H), "Wr")
    pb = _dev(bias, torch.float32, (s.E,), "bias")
    pt = _dev(page_table, torch.int32, (s.E, gu + d), "page_table")
    pp = _dev(page_pool, torch.uint8, None, "page_pool")
    dev = attn.device
    hidden_mid = torch.empty((s.T, s.H), dtype=torch.float32, device=dev)
    x_moe = torch.empty((s.T, s.H), dtype=torch.bfloat16, device=dev)
    y = torch.empty((s.T, s.H), dtype=torch.float32, device=dev)
    nbytes = post_attention_workspace_bytes(s)
    ws = torch.empty(nbytes + 256, dtype=torch.uint8, device=dev)
    off = (-ws.data_ptr()) % 256
    _check(_lib().moe_post_attention(ctypes.byref(s), ctypes.byref(o_proj), pa, ph, po, pg, float(eps), pw, pb, pt, pp,
                                     int(page_pool.shape[0]), hidden_mid.data_ptr(), x_moe.data_ptr(), y.data_ptr(),
                                     ws.data_ptr() + off, nbytes, _stream(stream)), "moe_post_attention")
    return hidden_mid, x_moe, y, ws


def moe_pre_attention(qkv_proj: LinearShape, hidden, delta, norm_gamma, eps, qkv_table, page_pool, want_bf16=True, stream=None):
    """-> (hidden_out f32, x_norm bf16, qkv f32, qkv bf16 or None)"""
    T, H = delta.shape
    ph = _dev(hidden, torch.float32, (T, H), "hidden")
    pd = _dev(delta, torch.float32, (qkv_proj.T, qkv_proj.K), "delta")
    pg = _dev(norm_gamma, torch.float32, (H,), "norm_gamma")
    pt = _dev(qkv_table, torch.int32, (linear_pages_required(qkv_proj),), "qkv_table")
    pp = _dev(page_pool, torch.uint8, None, "page_pool")
    dev = delta.device
    hidden_out = torch.empty((T, H), dtype=torch.float32, device=dev)
    x_norm = torch.empty((T, H), dtype=torch.bfloat16, device=dev)
    qkv = torch.empty((T, qkv_proj.N), dtype=torch.float32, device=dev)
    qkv16 = torch.empty((T, qkv_proj.N), dtype=torch.bfloat16, device=dev) if want_bf16 else None
    ws = torch.empty(16, dtype=torch.uint8, device=dev)
    _check(_lib().moe_pre_attention(ctypes.byref(qkv_proj), ph, pd, pg, float(eps), pt, pp, int(page_pool.shape[0]),
                                    hidden_out.data_ptr(), x_norm.data_ptr(), qkv.data_ptr(),
                                    None if qkv16 is None else qkv16.data_ptr(), ws.data_ptr(), 16, _stream(stream)),
           "moe_pre_attention")
    return hidden_out, x_norm, qkv, qkv16
