"""ctypes binding of liblasnet's C ABI (include/lasnet.h): argument marshalling only.

Every step of the path runs in the library's HIP kernels; PyTorch supplies device memory
and the current stream.  There is no fallback: a missing library or a failing call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

# LASNET_LIBRARY overrides the in-tree library (e.g. an instrumented build of the same sources).
_LIB_PATH = os.environ.get("LASNET_LIBRARY") or os.path.join(
    os.path.dirname(os.path.abspath(__file__)), "liblasnet.so")
_lib = None

LASNET_F32, LASNET_BF16 = 0, 1
LASNET_POST_RELU, LASNET_FORCE_GENERIC, LASNET_SKIP_IDENTITY, LASNET_FORCE_FUSED, LASNET_FORCE_TILED = 1, 2, 4, 8, 16
LASNET_OK, LASNET_EINVAL, LASNET_ESHAPE, LASNET_EUNSUPPORTED, LASNET_EALIAS, LASNET_EHIP = 0, -1, -2, -3, -4, -5
LASNET_ETOOBIG = -6
LASNET_NOALLOC_MAX_PACKED_BYTES = 4 << 20

EXPORTS = (
    "lasnet_version", "lasnet_status_string", "lasnet_masker", "lasnet_masker_ex", "lasnet_masker_logits",
    "lasnet_sparse_bottleneck", "lasnet_sparse_bottleneck_ex", "lasnet_dense_bottleneck",
    "lasnet_has_fast_path", "lasnet_packed_weights_bytes", "lasnet_pack_weights",
    "lasnet_sparse_bottleneck_packed", "lasnet_sparse_bottleneck_noalloc",
    "lasnet_workspace_bytes", "lasnet_sparse_bottleneck_planned",
    "lasnet_microbench_mfma", "lasnet_microbench_copy", "lasnet_microbench_weight_stream",
)


class LasnetError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().lasnet_status_string(status).decode()
        super().__init__("%s failed: %s (status %d)" % (where, msg, status))


class lasnet_tensor(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("n", ctypes.c_int32), ("h", ctypes.c_int32),
                ("w", ctypes.c_int32), ("c", ctypes.c_int32), ("dtype", ctypes.c_int32)]


def load_library(path: str) -> ctypes.CDLL:
    """Loads one build of the library and declares the argument types of its entry points."""
    if not os.path.exists(path):
        raise RuntimeError(
            "liblasnet.so is not built (%s missing): run `python -m paper_2210_06223_amd.build`; "
            "there is no CPU fallback" % path)
    L = ctypes.CDLL(path)
    vp, ip, tp = ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(lasnet_tensor)
    L.lasnet_version.restype = ip
    L.lasnet_version.argtypes = []
    L.lasnet_status_string.restype = ctypes.c_char_p
    L.lasnet_status_string.argtypes = [ip]
    L.lasnet_masker.restype = ip
    L.lasnet_masker.argtypes = [tp, vp, ctypes.c_float, ip, ctypes.c_float, vp, vp, vp, vp]
    L.lasnet_masker_ex.restype = ip
    L.lasnet_masker_ex.argtypes = [tp, vp, ctypes.c_float, ip, ctypes.c_float, vp, vp, vp, tp, vp]
    L.lasnet_masker_logits.restype = ip
    L.lasnet_masker_logits.argtypes = [tp, vp, ctypes.c_float, ip, vp, vp]
    L.lasnet_sparse_bottleneck.restype = ip
    L.lasnet_sparse_bottleneck.argtypes = [tp, vp, vp, ip, ip, vp, vp, vp, vp, vp, vp, tp, vp]
    L.lasnet_sparse_bottleneck_ex.restype = ip
    L.lasnet_sparse_bottleneck_ex.argtypes = [tp, vp, vp, ip, ip, vp, vp, vp, vp, vp, vp, tp,
                                              ctypes.c_uint32, vp]
    L.lasnet_workspace_bytes.restype = ctypes.c_size_t
    L.lasnet_workspace_bytes.argtypes = [ip] * 7
    L.lasnet_sparse_bottleneck_planned.restype = ip
    L.lasnet_sparse_bottleneck_planned.argtypes = [tp, vp, vp, vp, ip, ip, vp, vp, vp, vp, tp, ctypes.c_uint32,
                                                   vp, ctypes.c_size_t, vp]
    L.lasnet_microbench_mfma.restype = ctypes.c_double
    L.lasnet_microbench_mfma.argtypes = [ip, vp, vp]
    L.lasnet_microbench_weight_stream.restype = ctypes.c_double
    L.lasnet_microbench_weight_stream.argtypes = [vp, ctypes.c_size_t, ip, vp, vp]
    L.lasnet_microbench_copy.restype = ip
    L.lasnet_microbench_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
    L.lasnet_sparse_bottleneck_noalloc.restype = ip
    L.lasnet_sparse_bottleneck_noalloc.argtypes = L.lasnet_sparse_bottleneck_ex.argtypes
    L.lasnet_dense_bottleneck.restype = ip
    L.lasnet_dense_bottleneck.argtypes = [tp, ip, vp, vp, vp, vp, vp, vp, tp, ctypes.c_uint32, vp]
    L.lasnet_has_fast_path.restype = ip
    L.lasnet_has_fast_path.argtypes = [ip, ip, ip, ip]
    L.lasnet_packed_weights_bytes.restype = ctypes.c_size_t
    L.lasnet_packed_weights_bytes.argtypes = [ip, ip, ip, ip]
    L.lasnet_pack_weights.restype = ip
    L.lasnet_pack_weights.argtypes = [ip, ip, ip, ip, vp, vp, vp, vp, vp]
    L.lasnet_sparse_bottleneck_packed.restype = ip
    L.lasnet_sparse_bottleneck_packed.argtypes = [tp, vp, vp, ip, ip, vp, vp, vp, vp, tp,
                                                  ctypes.c_uint32, vp]
    return L


def lib() -> ctypes.CDLL:
    """The in-tree liblasnet.so (built by paper_2210_06223_amd.build / __graft_entry__.build)."""
    global _lib
    if _lib is None:
        _lib = load_library(_LIB_PATH)
    return _lib


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _as_tensor_desc(x: torch.Tensor) -> lasnet_tensor:
    if x.dim() != 4 or not x.is_contiguous():
        raise ValueError("feature maps are contiguous NHWC tensors [N,H,W,C]")
    if x.dtype == torch.float32:
        dt = LASNET_F32
    elif x.dtype == torch.bfloat16:
        dt = LASNET_BF16
    else:
        raise ValueError("dtype must be float32 or bfloat16")
    if not x.is_cuda:
        raise ValueError("feature maps live in device memory")
    n, h, w, c = x.shape
    return lasnet_tensor(x.data_ptr() if x.numel() else None, n, h, w, c, dt)


def _check(status: int, where: str):
    if status != LASNET_OK:
        raise LasnetError(status, where)


def _f32(t: torch.Tensor, name: str) -> torch.Tensor:
    if t.dtype != torch.float32 or not t.is_contiguous() or not t.is_cuda:
        raise ValueError("%s must be a contiguous float32 device tensor" % name)
    return t


def lasnet_version() -> int:
    return lib().lasnet_version()


def lasnet_has_fast_path(dtype: torch.dtype, C: int, M: int, S: int) -> int:
    return lib().lasnet_has_fast_path(LASNET_BF16 if dtype == torch.bfloat16 else LASNET_F32, C, M, S)


def lasnet_masker(x: torch.Tensor, Wm: torch.Tensor, bm: float, S: int, thr: float = 0.0,
                  mask: Optional[torch.Tensor] = None, idx: Optional[torch.Tensor] = None,
                  count: Optional[torch.Tensor] = None, stream=None
                  ) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """mask uint8 [N,G,GW], idx int32 [N*G*GW] (first count valid), count int32 [1]; all on device."""
    d = _as_tensor_desc(x)
    N, H, W, _ = x.shape
    if S <= 0 or H % S or W % S:
        _check(LASNET_ESHAPE if S > 0 else LASNET_EINVAL, "lasnet_masker")
    G, GW = H // S, W // S
    if mask is None:
        mask = torch.empty((N, G, GW), dtype=torch.uint8, device=x.device)
    if idx is None:
        idx = torch.empty((N * G * GW,), dtype=torch.int32, device=x.device)
    if count is None:
        count = torch.empty((1,), dtype=torch.int32, device=x.device)
    st = lib().lasnet_masker(ctypes.byref(d), _ptr(_f32(Wm, "Wm")), float(bm), int(S), float(thr),
                             _ptr(mask), _ptr(idx), _ptr(count), _stream(stream))
    _check(st, "lasnet_masker")
    return mask, idx, count


def lasnet_masker_ex(x: torch.Tensor, Wm: torch.Tensor, bm: float, S: int, thr: float = 0.0,
                     mask: Optional[torch.Tensor] = None, idx: Optional[torch.Tensor] = None,
                     count: Optional[torch.Tensor] = None, pass_out: Optional[torch.Tensor] = None,
                     stream=None) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """lasnet_masker that also copies every inactive cell of x to pass_out (may be None)."""
    d = _as_tensor_desc(x)
    N, H, W, _ = x.shape
    if S <= 0 or H % S or W % S:
        _check(LASNET_ESHAPE if S > 0 else LASNET_EINVAL, "lasnet_masker_ex")
    G, GW = H // S, W // S
    if mask is None:
        mask = torch.empty((N, G, GW), dtype=torch.uint8, device=x.device)
    if idx is None:
        idx = torch.empty((N * G * GW,), dtype=torch.int32, device=x.device)
    if count is None:
        count = torch.empty((1,), dtype=torch.int32, device=x.device)
    po = None
    if pass_out is not None:
        po = _as_tensor_desc(pass_out)
    st = lib().lasnet_masker_ex(ctypes.byref(d), _ptr(_f32(Wm, "Wm")), float(bm), int(S), float(thr),
                                _ptr(mask), _ptr(idx), _ptr(count),
                                ctypes.byref(po) if po is not None else None, _stream(stream))
    _check(st, "lasnet_masker_ex")
    return mask, idx, count


def lasnet_masker_logits(x: torch.Tensor, Wm: torch.Tensor, bm: float, S: int,
                         logits: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    d = _as_tensor_desc(x)
    N, H, W, _ = x.shape
    if S <= 0 or H % S or W % S:
        _check(LASNET_ESHAPE if S > 0 else LASNET_EINVAL, "lasnet_masker_logits")
    if logits is None:
        logits = torch.empty((N, H // S, W // S), dtype=torch.float64, device=x.device)
    st = lib().lasnet_masker_logits(ctypes.byref(d), _ptr(_f32(Wm, "Wm")), float(bm), int(S),
                                    _ptr(logits), _stream(stream))
    _check(st, "lasnet_masker_logits")
    return logits


def _weights(x, W1, b1, W2, b2, W3, b3):
    for n, t in (("W1", W1), ("W2", W2), ("W3", W3)):
        if t.dtype != x.dtype or not t.is_contiguous() or not t.is_cuda:
            raise ValueError("%s must be a contiguous device tensor of x's dtype" % n)
    M, C = W1.shape
    if C != x.shape[3] or tuple(W2.shape) != (M, 3, 3, M) or tuple(W3.shape) != (C, M):
        raise ValueError("weights: W1 [M,C], W2 [M,3,3,M], W3 [C,M]")
    if b1.numel() != M or b2.numel() != M or b3.numel() != C:
        raise ValueError("biases: b1 [M], b2 [M], b3 [C]")
    return int(M), [_ptr(W1), _ptr(_f32(b1, "b1")), _ptr(W2), _ptr(_f32(b2, "b2")), _ptr(W3),
                    _ptr(_f32(b3, "b3"))]


def _check_list(x: torch.Tensor, idx: Optional[torch.Tensor], count: Optional[torch.Tensor], S: int) -> None:
    """The list's storage is what the masker writes to: room for every cell of the map (the kernels may read
    entries past count[0], which only the device knows; they never use them)."""
    for n, t in (("idx", idx), ("count", count)):
        if t is not None and (t.dtype != torch.int32 or not t.is_cuda or not t.is_contiguous()):
            raise ValueError("%s must be a contiguous int32 device tensor" % n)
    if idx is not None and int(S) > 0 and x.dim() == 4 and x.shape[1] % int(S) == 0 and x.shape[2] % int(S) == 0:
        cells = int(x.shape[0]) * (int(x.shape[1]) // int(S)) * (int(x.shape[2]) // int(S))
        if idx.numel() < cells:
            raise ValueError("idx must have room for all %d cells of the map (it holds %d entries)" % (cells, idx.numel()))


def lasnet_sparse_bottleneck(x: torch.Tensor, idx: Optional[torch.Tensor],
                             count: Optional[torch.Tensor], S: int, W1, b1, W2, b2, W3, b3,
                             out: Optional[torch.Tensor] = None, flags: int = 0,
                             stream=None) -> torch.Tensor:
    d = _as_tensor_desc(x)
    if out is None:
        out = torch.empty_like(x)
    o = _as_tensor_desc(out)
    M, w = _weights(x, W1, b1, W2, b2, W3, b3)
    _check_list(x, idx, count, S)
    if flags:
        st = lib().lasnet_sparse_bottleneck_ex(ctypes.byref(d), _ptr(idx), _ptr(count), int(S), M, *w,
                                               ctypes.byref(o), int(flags), _stream(stream))
    else:
        st = lib().lasnet_sparse_bottleneck(ctypes.byref(d), _ptr(idx), _ptr(count), int(S), M, *w,
                                            ctypes.byref(o), _stream(stream))
    _check(st, "lasnet_sparse_bottleneck")
    return out


def lasnet_workspace_bytes(x: torch.Tensor, M: int, S: int) -> int:
    """Device memory the tiled schedule needs for a call on x (0: the fused schedule runs, or no fast path)."""
    n, h, w, c = x.shape
    return int(lib().lasnet_workspace_bytes(LASNET_BF16 if x.dtype == torch.bfloat16 else LASNET_F32,
                                            int(n), int(h), int(w), int(c), int(M), int(S)))


def lasnet_sparse_bottleneck_planned(x: torch.Tensor, idx: Optional[torch.Tensor],
                                     count: Optional[torch.Tensor], mask: Optional[torch.Tensor], S: int, M: int,
                                     packed: torch.Tensor, b1, b2, b3, out: torch.Tensor,
                                     workspace: Optional[torch.Tensor], flags: int = 0, stream=None) -> torch.Tensor:
    """The explicit form: packed weights, workspace (a uint8 device tensor or None) and out are the caller's."""
    d = _as_tensor_desc(x)
    o = _as_tensor_desc(out)
    _check_list(x, idx, count, S)
    if mask is not None and (mask.dtype != torch.uint8 or not mask.is_cuda or not mask.is_contiguous()):
        raise ValueError("mask must be a contiguous uint8 device tensor")
    if b1.numel() != M or b2.numel() != M or b3.numel() != x.shape[3]:
        raise ValueError("biases: b1 [M], b2 [M], b3 [C]")
    wbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = lib().lasnet_sparse_bottleneck_planned(ctypes.byref(d), _ptr(idx), _ptr(count), _ptr(mask), int(S), int(M),
                                                _ptr(packed), _ptr(_f32(b1, "b1")), _ptr(_f32(b2, "b2")),
                                                _ptr(_f32(b3, "b3")), ctypes.byref(o), int(flags),
                                                _ptr(workspace), wbytes, _stream(stream))
    _check(st, "lasnet_sparse_bottleneck_planned")
    return out


def lasnet_sparse_bottleneck_noalloc(x: torch.Tensor, idx: Optional[torch.Tensor],
                                     count: Optional[torch.Tensor], S: int, W1, b1, W2, b2, W3, b3,
                                     out: torch.Tensor, flags: int = 0, stream=None) -> torch.Tensor:
    """lasnet_sparse_bottleneck_ex whose weight repack goes to the library's fixed scratch array; `out` is
    the caller's (this wrapper allocates nothing either)."""
    d = _as_tensor_desc(x)
    o = _as_tensor_desc(out)
    M, w = _weights(x, W1, b1, W2, b2, W3, b3)
    _check_list(x, idx, count, S)
    st = lib().lasnet_sparse_bottleneck_noalloc(ctypes.byref(d), _ptr(idx), _ptr(count), int(S), M, *w,
                                                ctypes.byref(o), int(flags), _stream(stream))
    _check(st, "lasnet_sparse_bottleneck_noalloc")
    return out


def lasnet_dense_bottleneck(x: torch.Tensor, W1, b1, W2, b2, W3, b3,
                            out: Optional[torch.Tensor] = None, flags: int = 0,
                            stream=None) -> torch.Tensor:
    d = _as_tensor_desc(x)
    if out is None:
        out = torch.empty_like(x)
    o = _as_tensor_desc(out)
    M, w = _weights(x, W1, b1, W2, b2, W3, b3)
    st = lib().lasnet_dense_bottleneck(ctypes.byref(d), M, *w, ctypes.byref(o), int(flags),
                                       _stream(stream))
    _check(st, "lasnet_dense_bottleneck")
    return out


def lasnet_pack_weights(S: int, W1: torch.Tensor, W2: torch.Tensor, W3: torch.Tensor,
                        packed: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Repack W1 [M,C], W2 [M,3,3,M], W3 [C,M] (bf16) for the matrix-core kernel of (C, M, S)."""
    M, C = W1.shape
    for n, t in (("W1", W1), ("W2", W2), ("W3", W3)):
        if t.dtype != torch.bfloat16 or not t.is_contiguous() or not t.is_cuda:
            raise ValueError("%s must be a contiguous bfloat16 device tensor" % n)
    if tuple(W2.shape) != (M, 3, 3, M) or tuple(W3.shape) != (C, M):
        raise ValueError("weights: W1 [M,C], W2 [M,3,3,M], W3 [C,M]")
    nbytes = lib().lasnet_packed_weights_bytes(LASNET_BF16, int(C), int(M), int(S))
    if nbytes == 0:
        _check(LASNET_EUNSUPPORTED, "lasnet_pack_weights")
    if packed is None:
        packed = torch.empty((nbytes // 2,), dtype=torch.bfloat16, device=W1.device)
    elif packed.numel() * packed.element_size() < nbytes or not packed.is_cuda:
        raise ValueError("packed buffer too small")
    st = lib().lasnet_pack_weights(LASNET_BF16, int(C), int(M), int(S), _ptr(W1), _ptr(W2), _ptr(W3),
                                   _ptr(packed), _stream(stream))
    _check(st, "lasnet_pack_weights")
    return packed


def lasnet_sparse_bottleneck_packed(x: torch.Tensor, idx: Optional[torch.Tensor],
                                    count: Optional[torch.Tensor], S: int, M: int,
                                    packed: torch.Tensor, b1, b2, b3,
                                    out: Optional[torch.Tensor] = None, flags: int = 0,
                                    stream=None) -> torch.Tensor:
    d = _as_tensor_desc(x)
    if out is None:
        out = torch.empty_like(x)
    o = _as_tensor_desc(out)
    _check_list(x, idx, count, S)
    need = lib().lasnet_packed_weights_bytes(LASNET_BF16, int(x.shape[3]), int(M), int(S))
    if need and packed.numel() * packed.element_size() < need:
        raise ValueError("packed buffer too small for this shape")
    if b1.numel() != M or b2.numel() != M or b3.numel() != x.shape[3]:
        raise ValueError("biases: b1 [M], b2 [M], b3 [C]")
    st = lib().lasnet_sparse_bottleneck_packed(ctypes.byref(d), _ptr(idx), _ptr(count), int(S), int(M),
                                               _ptr(packed), _ptr(_f32(b1, "b1")), _ptr(_f32(b2, "b2")),
                                               _ptr(_f32(b3, "b3")), ctypes.byref(o), int(flags),
                                               _stream(stream))
    _check(st, "lasnet_sparse_bottleneck_packed")
    return out


def lasnet_microbench_mfma(iters: int, sink: torch.Tensor, stream=None) -> float:
    """Launches the register-only bf16 MFMA loop; returns the FLOPs of the launch."""
    f = lib().lasnet_microbench_mfma(int(iters), _ptr(sink), _stream(stream))
    if f <= 0:
        raise LasnetError(LASNET_EHIP, "lasnet_microbench_mfma")
    return float(f)


def lasnet_microbench_weight_stream(buf: torch.Tensor, passes: int, sink: torch.Tensor, stream=None) -> float:
    """Every CU reads `buf` `passes` times the way the block kernels read their weights; returns the bytes read."""
    f = lib().lasnet_microbench_weight_stream(_ptr(buf), buf.numel() * buf.element_size(), int(passes), _ptr(sink),
                                              _stream(stream))
    if f <= 0:
        raise LasnetError(LASNET_EHIP, "lasnet_microbench_weight_stream")
    return float(f)


def lasnet_microbench_copy(src: torch.Tensor, dst: torch.Tensor, stream=None) -> int:
    """dst = src with the library's copy kernel; returns the bytes copied."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("src and dst must have the same size")
    _check(lib().lasnet_microbench_copy(_ptr(src), _ptr(dst), nbytes, _stream(stream)), "lasnet_microbench_copy")
    return nbytes
