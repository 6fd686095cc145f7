"""ctypes binding of librr_attn.so: same names as the C ABI, argument marshalling only.

torch is used for device memory and the current stream; every step of the path runs inside the
library's HIP kernels.  There is no fallback: if the shared library is missing, importing this
module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "librr_attn.so")

RR_OK = 0
RR_ERR_NULL, RR_ERR_SHAPE, RR_ERR_DTYPE, RR_ERR_PARAM, RR_ERR_WORKSPACE, RR_ERR_LAUNCH = -1, -2, -3, -4, -5, -6
RR_ERR_SCRATCH_LIMIT = -7
RR_STATIC_SCRATCH_BYTES = 32 << 20
RR_QUEUE_WORDS = 160          # int32 words of rr_mask.queue
RR_BF16, RR_F32 = 0, 1
RR_FLAG_PROTECT_LAST = 1
RR_FLAG_DIAGONAL_TOKEN = 2

RR_OFFSET_HEAD, RR_OFFSET_FIXED, RR_OFFSET_LAYER, RR_OFFSET_HYBRID = 0, 1, 2, 3
OFFSET_MODES = {"head": RR_OFFSET_HEAD, "fixed": RR_OFFSET_FIXED, "layer": RR_OFFSET_LAYER, "hybrid": RR_OFFSET_HYBRID}

EXPORTS = ("rr_version", "rr_status_string", "rr_workspace_bytes", "rr_estimate", "rr_estimate_ex",
           "rr_sparse_attn", "rr_dense_attn", "rr_accuracy_workspace_bytes", "rr_selection_accuracy",
           "rr_mask_from_dense", "rr_dense_attn_packed", "rr_estimate_static", "rr_attn_workspace_bytes",
           "rr_sparse_attn_ws", "rr_dense_attn_ws")


class rr_shape(C.Structure):
    _fields_ = [("batch", C.c_int32), ("L", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32),
                ("d", C.c_int32), ("dtype", C.c_int32),
                ("q_stride_b", C.c_int64), ("q_stride_h", C.c_int64), ("q_stride_l", C.c_int64),
                ("kv_stride_b", C.c_int64), ("kv_stride_h", C.c_int64), ("kv_stride_l", C.c_int64),
                ("Lq", C.c_int32)]


class rr_mask(C.Structure):
    _fields_ = [("dense", C.c_void_p), ("row_count", C.c_void_p), ("row_list", C.c_void_p),
                ("block_mass", C.c_void_p), ("Nb", C.c_int32), ("B", C.c_int32), ("row_order", C.c_void_p), ("queue", C.c_void_p)]


class rr_estimate_opts(C.Structure):
    _fields_ = [("flags", C.c_uint32), ("offset_mode", C.c_int32), ("layer", C.c_int32),
                ("sink_blocks", C.c_int32), ("recent_blocks", C.c_int32), ("seq_first", C.c_void_p),
                ("ksum_capacity", C.c_int32), ("ksum_valid", C.c_int32)]


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2602_05853_amd.build`")
    lib = C.CDLL(LIB_PATH)
    lib.rr_version.restype = C.c_int
    lib.rr_status_string.restype = C.c_char_p
    lib.rr_status_string.argtypes = [C.c_int]
    lib.rr_workspace_bytes.restype = C.c_size_t
    lib.rr_workspace_bytes.argtypes = [C.POINTER(rr_shape), C.c_int, C.c_int]
    lib.rr_estimate.restype = C.c_int
    lib.rr_estimate.argtypes = [C.POINTER(rr_shape), C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_float,
                                C.c_uint32, C.c_void_p, C.c_size_t, C.POINTER(rr_mask), C.c_void_p]
    lib.rr_estimate_static.restype = C.c_int
    lib.rr_estimate_static.argtypes = [C.POINTER(rr_shape), C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_float,
                                       C.c_uint32, C.POINTER(rr_mask), C.c_void_p]
    lib.rr_estimate_ex.restype = C.c_int
    lib.rr_estimate_ex.argtypes = [C.POINTER(rr_shape), C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_float,
                                   C.POINTER(rr_estimate_opts), C.c_void_p, C.c_size_t, C.POINTER(rr_mask),
                                   C.c_void_p]
    lib.rr_sparse_attn.restype = C.c_int
    lib.rr_sparse_attn.argtypes = [C.POINTER(rr_shape), C.c_void_p, C.c_void_p, C.c_void_p,
                                   C.POINTER(rr_mask), C.c_void_p, C.c_void_p, C.c_void_p]
    lib.rr_accuracy_workspace_bytes.restype = C.c_size_t
    lib.rr_accuracy_workspace_bytes.argtypes = [C.POINTER(rr_shape), C.c_int]
    lib.rr_selection_accuracy.restype = C.c_int
    lib.rr_selection_accuracy.argtypes = [C.POINTER(rr_shape), C.c_void_p, C.c_void_p, C.POINTER(rr_mask), C.c_float,
                                          C.c_int, C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
    lib.rr_mask_from_dense.restype = C.c_int
    lib.rr_mask_from_dense.argtypes = [C.POINTER(rr_shape), C.POINTER(rr_mask), C.c_void_p]
    lib.rr_dense_attn_packed.restype = C.c_int
    lib.rr_dense_attn_packed.argtypes = [C.POINTER(rr_shape), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                         C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.rr_attn_workspace_bytes.restype = C.c_size_t
    lib.rr_attn_workspace_bytes.argtypes = [C.POINTER(rr_shape), C.c_int]
    lib.rr_sparse_attn_ws.restype = C.c_int
    lib.rr_sparse_attn_ws.argtypes = [C.POINTER(rr_shape), C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(rr_mask),
                                      C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.rr_dense_attn_ws.restype = C.c_int
    lib.rr_dense_attn_ws.argtypes = [C.POINTER(rr_shape), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                     C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.rr_dense_attn.restype = C.c_int
    lib.rr_dense_attn.argtypes = [C.POINTER(rr_shape), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                  C.c_void_p, C.c_void_p, C.c_void_p]
    return lib


lib = _load()


class RRError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"rr_attn status {status}: {lib.rr_status_string(status).decode()}")


def _check(status: int) -> None:
    if status != RR_OK:
        raise RRError(status)


def rr_version() -> int:
    return lib.rr_version()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return RR_BF16
    if t.dtype == torch.float32:
        return RR_F32
    raise RRError(RR_ERR_DTYPE)


def make_shape(Q: torch.Tensor, K: torch.Tensor) -> rr_shape:
    """Q [batch, Hq, Lq, d], K [batch, Hkv, L, d] (any strides with the last dimension contiguous).
    Lq < L is chunked prefill: Q holds the last Lq positions of the L-token context."""
    if Q.dim() != 4 or K.dim() != 4 or Q.stride(3) != 1 or K.stride(3) != 1:
        raise RRError(RR_ERR_SHAPE)
    b, Hq, Lq, d = Q.shape
    L = K.shape[2]
    if K.shape[0] != b or K.shape[3] != d or Lq > L:
        raise RRError(RR_ERR_SHAPE)
    return rr_shape(b, L, Hq, K.shape[1], d, _dtype_code(Q),
                    Q.stride(0), Q.stride(1), Q.stride(2), K.stride(0), K.stride(1), K.stride(2), Lq)


def _stream_ptr(stream: Optional[torch.cuda.Stream]) -> int:
    return (stream or torch.cuda.current_stream()).cuda_stream


@dataclass
class BlockMask:
    """Device arrays of one block selection (the rr_mask of the C ABI)."""
    B: int
    Nb: int
    row_count: torch.Tensor               # int32 [batch, Hq, rows]       rows = Lq / B (= Nb unless chunked)
    row_list: torch.Tensor                # int32 [batch, Hq, rows, Nb]
    dense: Optional[torch.Tensor] = None  # uint8 [batch, Hq, rows, Nb]
    block_mass: Optional[torch.Tensor] = None  # float32 [batch, Hq, rows, Nb]
    row_order: Optional[torch.Tensor] = None   # int32 [batch, Hkv, G * rows], scheduling hint
    queue: Optional[torch.Tensor] = None       # int32 [RR_QUEUE_WORDS], zero: row counters of rr_sparse_attn's persistent form

    def c_struct(self) -> rr_mask:
        return rr_mask(self.dense.data_ptr() if self.dense is not None else None,
                       self.row_count.data_ptr(), self.row_list.data_ptr(),
                       self.block_mass.data_ptr() if self.block_mass is not None else None,
                       self.Nb, self.B,
                       self.row_order.data_ptr() if self.row_order is not None else None,
                       self.queue.data_ptr() if self.queue is not None else None)

    @staticmethod
    def allocate(batch: int, Hq: int, Nb: int, B: int, device, dense: bool = True,
                 block_mass: bool = False, Hkv: Optional[int] = None, rows: Optional[int] = None) -> "BlockMask":
        """With Hkv given, the row-order hint ([batch, Hkv, (Hq/Hkv) * rows]) is allocated too.
        rows = number of query blocks (Lq / B), Nb by default."""
        Nq = Nb if rows is None else rows
        return BlockMask(
            row_order=(torch.zeros((batch, Hkv, (Hq // Hkv) * Nq), dtype=torch.int32, device=device)
                       if Hkv else None),
            queue=torch.zeros(RR_QUEUE_WORDS, dtype=torch.int32, device=device) if Hkv else None,
            B=B, Nb=Nb,
            row_count=torch.zeros((batch, Hq, Nq), dtype=torch.int32, device=device),
            row_list=torch.zeros((batch, Hq, Nq, Nb), dtype=torch.int32, device=device),
            dense=torch.zeros((batch, Hq, Nq, Nb), dtype=torch.uint8, device=device) if dense else None,
            block_mass=torch.zeros((batch, Hq, Nq, Nb), dtype=torch.float32, device=device) if block_mass else None)


def rr_workspace_bytes(Q: torch.Tensor, K: torch.Tensor, S: int, B: int) -> int:
    shp = make_shape(Q, K)
    return lib.rr_workspace_bytes(C.byref(shp), S, B)


def rr_estimate(Q: torch.Tensor, K: torch.Tensor, S: int, B: int, tau: float,
                flags: int = RR_FLAG_PROTECT_LAST, out: Optional[BlockMask] = None,
                workspace: Optional[torch.Tensor] = None, block_mass: bool = False,
                stream: Optional[torch.cuda.Stream] = None, offset_mode="head", layer: int = 0,
                sink_blocks: int = 0, recent_blocks: int = 0,
                seq_first: Optional[torch.Tensor] = None, ksum_capacity: int = 0, ksum_valid: int = 0) -> BlockMask:
    """rr_estimate of the C ABI; with any of the last seven arguments given, rr_estimate_ex.  With ksum_capacity
    the workspace must be given (it carries the stride sums from call to call)."""
    shp = make_shape(Q, K)
    if ksum_capacity and workspace is None:
        raise RRError(RR_ERR_WORKSPACE)
    if seq_first is not None:
        _check_seq_first(seq_first, _blocks(shp.L, B), Q.device)
    need = lib.rr_workspace_bytes(C.byref(shp), S, B)
    if need == 0:
        raise RRError(RR_ERR_SHAPE)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=Q.device)
    if out is None:
        out = BlockMask.allocate(shp.batch, shp.Hq, _blocks(shp.L, B), B, Q.device, dense=True, block_mass=block_mass,
                                 Hkv=shp.Hkv, rows=_query_blocks(shp, B))
    cm = out.c_struct()
    mode = OFFSET_MODES[offset_mode] if isinstance(offset_mode, str) else int(offset_mode)
    if mode == RR_OFFSET_HEAD and not (layer or sink_blocks or recent_blocks or ksum_capacity) and seq_first is None:
        _check(lib.rr_estimate(C.byref(shp), Q.data_ptr(), K.data_ptr(), S, B, tau, flags,
                               workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                               C.byref(cm), _stream_ptr(stream)))
    else:
        opts = rr_estimate_opts(flags, mode, layer, sink_blocks, recent_blocks,
                                seq_first.data_ptr() if seq_first is not None else None, ksum_capacity, ksum_valid)
        _check(lib.rr_estimate_ex(C.byref(shp), Q.data_ptr(), K.data_ptr(), S, B, tau, C.byref(opts),
                                  workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                  C.byref(cm), _stream_ptr(stream)))
    return out


def rr_estimate_static(Q: torch.Tensor, K: torch.Tensor, S: int, B: int, tau: float, out: BlockMask,
                       flags: int = RR_FLAG_PROTECT_LAST, stream: Optional[torch.cuda.Stream] = None) -> BlockMask:
    """rr_estimate_static of the C ABI: the caller brings the mask arrays, the library its own fixed scratch."""
    shp = make_shape(Q, K)
    cm = out.c_struct()
    _check(lib.rr_estimate_static(C.byref(shp), Q.data_ptr(), K.data_ptr(), S, B, tau, flags, C.byref(cm),
                                  _stream_ptr(stream)))
    return out


def rr_attn_workspace_bytes(Q: torch.Tensor, K: torch.Tensor, B: int) -> int:
    """Bytes of scratch with which rr_sparse_attn / rr_dense_attn split the rows of a step (0: no split)."""
    shp = make_shape(Q, K)
    return lib.rr_attn_workspace_bytes(C.byref(shp), B)


def rr_sparse_attn(Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, mask: BlockMask,
                   O: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None,
                   stream: Optional[torch.cuda.Stream] = None,
                   workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """workspace (uint8, rr_attn_workspace_bytes): the entry point with a workspace, for steps."""
    shp = make_shape(Q, K)
    if V.stride() != K.stride() or V.shape != K.shape:
        raise RRError(RR_ERR_SHAPE)
    if O is None:
        O = torch.empty_strided(Q.shape, Q.stride(), dtype=Q.dtype, device=Q.device)
    cm = mask.c_struct()
    if workspace is not None:
        _check(lib.rr_sparse_attn_ws(C.byref(shp), Q.data_ptr(), K.data_ptr(), V.data_ptr(), C.byref(cm),
                                     O.data_ptr(), lse.data_ptr() if lse is not None else None,
                                     workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                     _stream_ptr(stream)))
        return O
    _check(lib.rr_sparse_attn(C.byref(shp), Q.data_ptr(), K.data_ptr(), V.data_ptr(), C.byref(cm),
                              O.data_ptr(), lse.data_ptr() if lse is not None else None,
                              _stream_ptr(stream)))
    return O


def rr_dense_attn(Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, B: int,
                  O: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None,
                  stream: Optional[torch.cuda.Stream] = None,
                  workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    shp = make_shape(Q, K)
    if V.stride() != K.stride() or V.shape != K.shape:
        raise RRError(RR_ERR_SHAPE)
    if O is None:
        O = torch.empty_strided(Q.shape, Q.stride(), dtype=Q.dtype, device=Q.device)
    if workspace is not None:
        _check(lib.rr_dense_attn_ws(C.byref(shp), Q.data_ptr(), K.data_ptr(), V.data_ptr(), B,
                                    O.data_ptr(), lse.data_ptr() if lse is not None else None,
                                    workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                    _stream_ptr(stream)))
        return O
    _check(lib.rr_dense_attn(C.byref(shp), Q.data_ptr(), K.data_ptr(), V.data_ptr(), B,
                             O.data_ptr(), lse.data_ptr() if lse is not None else None,
                             _stream_ptr(stream)))
    return O


def _blocks(length: int, B: int) -> int:
    """Blocks of B positions covering `length` positions (the last one may be partial)."""
    return -(-length // B)


def _query_blocks(shp: rr_shape, B: int) -> int:
    """Rows of the mask arrays: the query blocks that the last Lq positions of the context touch (the first
    one may begin in front of them when the step starts inside a block)."""
    Lq = shp.Lq if shp.Lq else shp.L
    return _blocks(shp.L, B) - (shp.L - Lq) // B


def _check_seq_first(seq_first: torch.Tensor, Nb: int, device) -> None:
    if seq_first.dtype != torch.int32 or tuple(seq_first.shape) != (Nb,) or not seq_first.is_contiguous() or \
            seq_first.device != device:
        raise RRError(RR_ERR_PARAM)


def packed_seq_first(blocks_per_sequence, device) -> torch.Tensor:
    """The seq_first table of the header for sequences of the given lengths in blocks, packed back to back."""
    table = []
    for nb in blocks_per_sequence:
        table += [len(table)] * int(nb)
    return torch.tensor(table, dtype=torch.int32, device=device)


def rr_dense_attn_packed(Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, B: int, seq_first: torch.Tensor,
                         O: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None,
                         stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    shp = make_shape(Q, K)
    if V.stride() != K.stride() or V.shape != K.shape:
        raise RRError(RR_ERR_SHAPE)
    _check_seq_first(seq_first, _blocks(shp.L, B), Q.device)
    if O is None:
        O = torch.empty_strided(Q.shape, Q.stride(), dtype=Q.dtype, device=Q.device)
    _check(lib.rr_dense_attn_packed(C.byref(shp), Q.data_ptr(), K.data_ptr(), V.data_ptr(), B, seq_first.data_ptr(),
                                    O.data_ptr(), lse.data_ptr() if lse is not None else None,
                                    _stream_ptr(stream)))
    return O


def rr_selection_accuracy(Q: torch.Tensor, K: torch.Tensor, mask: BlockMask, tau: float = 0.95, step: int = 1,
                          workspace: Optional[torch.Tensor] = None,
                          stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """Precision / recall / F1 of `mask` per head, [batch, Hq, 3] fp32 (see rr_selection_accuracy in the header)."""
    shp = make_shape(Q, K)
    need = lib.rr_accuracy_workspace_bytes(C.byref(shp), step)
    if need == 0:
        raise RRError(RR_ERR_PARAM)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=Q.device)
    out = torch.empty((shp.batch, shp.Hq, 3), dtype=torch.float32, device=Q.device)
    cm = mask.c_struct()
    _check(lib.rr_selection_accuracy(C.byref(shp), Q.data_ptr(), K.data_ptr(), C.byref(cm), tau, step,
                                     workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                     out.data_ptr(), _stream_ptr(stream)))
    return out


def rr_mask_from_dense(Q: torch.Tensor, K: torch.Tensor, dense: torch.Tensor, B: int,
                       stream: Optional[torch.cuda.Stream] = None) -> BlockMask:
    """BlockMask of a caller-made 0/1 matrix `dense` (uint8 [batch, Hq, Nb, Nb] on the device)."""
    shp = make_shape(Q, K)
    Nb = _blocks(shp.L, B)
    if dense.dtype != torch.uint8 or tuple(dense.shape) != (shp.batch, shp.Hq, _query_blocks(shp, B), Nb) or \
            not dense.is_contiguous():
        raise RRError(RR_ERR_PARAM)
    mask = BlockMask.allocate(shp.batch, shp.Hq, Nb, B, Q.device, dense=False, Hkv=shp.Hkv, rows=_query_blocks(shp, B))
    mask.dense = dense
    cm = mask.c_struct()
    _check(lib.rr_mask_from_dense(C.byref(shp), C.byref(cm), _stream_ptr(stream)))
    return mask
