"""ctypes binding of libmmsp.so: the same calls as include/mmsp.h, argument marshalling only.

Tensors are anything with `.data_ptr()` (torch tensors on the GPU); PyTorch is used by the
callers for device memory and streams, never for arithmetic on the attention path.
There is no fallback: if the library has not been built, importing this module raises.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmmsp.so")

MMSP_OK, MMSP_ERR_INVALID_ARG, MMSP_ERR_UNSUPPORTED, MMSP_ERR_WORKSPACE_TOO_SMALL, MMSP_ERR_DEVICE = range(5)
MMSP_MASK_FULL, MMSP_MASK_CAUSAL_DIAG, MMSP_MASK_NONE = 0, 1, 2
MMSP_BF16, MMSP_F32 = 0, 1

EXPORTS = ["mmsp_zigzag_layout", "mmsp_zigzag_plan", "mmsp_contiguous_plan", "mmsp_zigzag_plan_packed", "mmsp_2d_layout", "mmsp_workspace_bytes", "mmsp_attn_step_fwd",
           "mmsp_attn_merge", "mmsp_attn_delta", "mmsp_attn_step_bwd", "mmsp_attn_step_bwd_static", "mmsp_zigzag_gather", "mmsp_zigzag_scatter",
           "mmsp_a2a_pack_heads", "mmsp_a2a_unpack_heads", "mmsp_last_error"]


class MmspShape(ctypes.Structure):
    _fields_ = [("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("io_dtype", ctypes.c_int32), ("softmax_scale", ctypes.c_float),
                ("q_tok_stride", ctypes.c_int64), ("q_head_stride", ctypes.c_int64),
                ("kv_tok_stride", ctypes.c_int64), ("kv_head_stride", ctypes.c_int64),
                ("lse_head_stride", ctypes.c_int64)]


class MmspBlock(ctypes.Structure):
    _fields_ = [("q_row0", ctypes.c_int64), ("n_q", ctypes.c_int64), ("k_row0", ctypes.c_int64),
                ("n_k", ctypes.c_int64), ("q_pos0", ctypes.c_int64), ("k_pos0", ctypes.c_int64),
                ("mask", ctypes.c_int32), ("n_docs", ctypes.c_int32), ("cu_seqlens", ctypes.c_void_p)]


class Mmsp2dShare(ctypes.Structure):
    _fields_ = [("head_rank", ctypes.c_int32), ("ring_rank", ctypes.c_int32), ("q_head0", ctypes.c_int32),
                ("n_q_heads", ctypes.c_int32), ("kv_head0", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("chunk_ids", ctypes.c_int32 * 2), ("chunk_len", ctypes.c_int64)]


class MmspError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("mmsp status %d: %s" % (status, message))
        self.status = status


if not os.path.exists(LIB_PATH):
    raise ImportError("libmmsp.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                      "(or python paper_2408_10188_amd/build.py) first; there is no fallback path")
_lib = ctypes.CDLL(LIB_PATH)

_P, _I64, _I32, _INT, _SZ = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int, ctypes.c_size_t
_lib.mmsp_last_error.restype = ctypes.c_char_p
_lib.mmsp_last_error.argtypes = []
_lib.mmsp_zigzag_layout.argtypes = [_I64, _I32, _I32, ctypes.POINTER(_I32), ctypes.POINTER(_I64)]
_lib.mmsp_zigzag_plan.argtypes = [_I64, _I32, _I32, _I32, ctypes.POINTER(_I32), ctypes.POINTER(MmspBlock)]
_lib.mmsp_contiguous_plan.argtypes = [_I64, _I32, _I32, _I32, ctypes.POINTER(_I32), ctypes.POINTER(MmspBlock)]
_lib.mmsp_zigzag_plan_packed.argtypes = [_I64, _I32, _I32, _I32, ctypes.POINTER(_I32), _I32, ctypes.POINTER(_I32),
                                         ctypes.POINTER(MmspBlock), ctypes.POINTER(_I32)]
_lib.mmsp_2d_layout.argtypes = [_I64, _I32, _I32, _I32, _I32, _I32, ctypes.POINTER(Mmsp2dShare)]
_lib.mmsp_zigzag_gather.argtypes = [_I64, _I32, _I64, _P, _P, _P]
_lib.mmsp_zigzag_scatter.argtypes = [_I64, _I32, _I64, _P, _P, _P]
_lib.mmsp_a2a_pack_heads.argtypes = [_I64, _I32, _I64, _P, _P, _P]
_lib.mmsp_a2a_unpack_heads.argtypes = [_I64, _I32, _I64, _P, _P, _P]
_lib.mmsp_workspace_bytes.restype = _SZ
_lib.mmsp_workspace_bytes.argtypes = [ctypes.POINTER(MmspShape), _I64, _I64, _INT]
_lib.mmsp_attn_step_fwd.argtypes = [ctypes.POINTER(MmspShape), ctypes.POINTER(MmspBlock), _P, _P, _P, _P, _P, _INT,
                                    _P, _SZ, _P]
_lib.mmsp_attn_merge.argtypes = [ctypes.POINTER(MmspShape), _I64, _I64, _P, _P, _P, _P, _P, _P]
_lib.mmsp_attn_delta.argtypes = [ctypes.POINTER(MmspShape), _I64, _I64, _P, _P, _P, _P]
_lib.mmsp_attn_step_bwd.argtypes = [ctypes.POINTER(MmspShape), ctypes.POINTER(MmspBlock), _P, _P, _P, _P, _P, _P, _P,
                                    _INT, _P, _P, _P, _INT, _P, _SZ, _P]
_lib.mmsp_attn_step_bwd_static.argtypes = [ctypes.POINTER(MmspShape), ctypes.POINTER(MmspBlock), _P, _P, _P, _P, _P, _P,
                                           _P, _INT, _P, _P, _P, _INT, _P]
for _name in EXPORTS:
    if _name not in ("mmsp_last_error", "mmsp_workspace_bytes"):
        getattr(_lib, _name).restype = _INT


def _ptr(t):
    return None if t is None else (t if isinstance(t, int) else t.data_ptr())


def _check(status):
    if status != MMSP_OK:
        raise MmspError(status, _lib.mmsp_last_error().decode())


def mmsp_last_error():
    return _lib.mmsp_last_error().decode()


def make_shape(n_q_heads, n_kv_heads, head_dim, io_dtype, softmax_scale, q_strides, kv_strides, lse_head_stride):
    """q_strides / kv_strides = (token stride, head stride) in elements."""
    return MmspShape(n_q_heads, n_kv_heads, head_dim, io_dtype, softmax_scale, q_strides[0], q_strides[1],
                     kv_strides[0], kv_strides[1], lse_head_stride)


def make_block(q_row0, n_q, k_row0, n_k, mask, q_pos0=0, k_pos0=0, cu_seqlens=None, n_docs=0):
    return MmspBlock(q_row0, n_q, k_row0, n_k, q_pos0, k_pos0, mask, n_docs, _ptr(cu_seqlens))


def mmsp_zigzag_layout(T, N, rank, want_map=True):
    ids = (_I32 * 2)()
    l2g = np.empty(T // N if (N > 0 and T > 0) else 0, dtype=np.int64) if want_map else None
    p = l2g.ctypes.data_as(ctypes.POINTER(_I64)) if want_map else None
    _check(_lib.mmsp_zigzag_layout(T, N, rank, ids, p))
    return (ids[0], ids[1]), l2g


def mmsp_zigzag_plan(T, N, rank, step):
    src = _I32()
    blk = MmspBlock()
    _check(_lib.mmsp_zigzag_plan(T, N, rank, step, ctypes.byref(src), ctypes.byref(blk)))
    return src.value, blk


def mmsp_contiguous_plan(T, N, rank, step):
    src = _I32()
    blk = MmspBlock()
    _check(_lib.mmsp_contiguous_plan(T, N, rank, step, ctypes.byref(src), ctypes.byref(blk)))
    return src.value, blk


def mmsp_zigzag_plan_packed(T, N, rank, step, cu_seqlens=None, n_docs=0, cu_host=None):
    """Returns (src, [blocks]); cu_seqlens (device int32 tensor) / n_docs are filled into every
    block; cu_host (numpy int32 copy of cu_seqlens) lets the plan drop segment pairs no document spans."""
    src, n = _I32(), _I32()
    blks = (MmspBlock * 4)()
    hp, hn = None, 0
    if cu_host is not None:
        cu_host = np.ascontiguousarray(cu_host, dtype=np.int32)
        hp, hn = cu_host.ctypes.data_as(ctypes.POINTER(_I32)), len(cu_host) - 1
    _check(_lib.mmsp_zigzag_plan_packed(T, N, rank, step, hp, hn, ctypes.byref(src), blks, ctypes.byref(n)))
    out = []
    for i in range(n.value):
        b = MmspBlock.from_buffer_copy(blks[i])
        b.cu_seqlens, b.n_docs = _ptr(cu_seqlens), n_docs
        out.append(b)
    return src.value, out


def mmsp_2d_layout(T, U, R, gpu, n_q_heads, n_kv_heads):
    share = Mmsp2dShare()
    _check(_lib.mmsp_2d_layout(T, U, R, gpu, n_q_heads, n_kv_heads, ctypes.byref(share)))
    return share


def mmsp_zigzag_gather(T, N, row_bytes, seq, shards, stream=0):
    _check(_lib.mmsp_zigzag_gather(T, N, row_bytes, _ptr(seq), _ptr(shards), stream or None))


def mmsp_zigzag_scatter(T, N, row_bytes, shards, seq, stream=0):
    _check(_lib.mmsp_zigzag_scatter(T, N, row_bytes, _ptr(shards), _ptr(seq), stream or None))


def mmsp_a2a_pack_heads(n_tokens, U, slice_bytes, x, y, stream=0):
    _check(_lib.mmsp_a2a_pack_heads(n_tokens, U, slice_bytes, _ptr(x), _ptr(y), stream or None))


def mmsp_a2a_unpack_heads(n_tokens, U, slice_bytes, y, x, stream=0):
    _check(_lib.mmsp_a2a_unpack_heads(n_tokens, U, slice_bytes, _ptr(y), _ptr(x), stream or None))


def mmsp_workspace_bytes(shape, n_q_max, n_k_max, backward):
    return _lib.mmsp_workspace_bytes(ctypes.byref(shape), n_q_max, n_k_max, int(backward))


def mmsp_attn_step_fwd(shape, blk, q, k, v, o, lse, accumulate, workspace=None, workspace_bytes=0, stream=0):
    _check(_lib.mmsp_attn_step_fwd(ctypes.byref(shape), ctypes.byref(blk), _ptr(q), _ptr(k), _ptr(v), _ptr(o),
                                   _ptr(lse), int(accumulate), _ptr(workspace), workspace_bytes, stream or None))


def mmsp_attn_merge(shape, row0, n_rows, o_acc, lse_acc, o_part, lse_part, o_final=None, stream=0):
    _check(_lib.mmsp_attn_merge(ctypes.byref(shape), row0, n_rows, _ptr(o_acc), _ptr(lse_acc), _ptr(o_part),
                                _ptr(lse_part), _ptr(o_final), stream or None))


def mmsp_attn_delta(shape, row0, n_rows, o_final, d_o, delta, stream=0):
    _check(_lib.mmsp_attn_delta(ctypes.byref(shape), row0, n_rows, _ptr(o_final), _ptr(d_o), _ptr(delta),
                                stream or None))


def mmsp_attn_step_bwd_static(shape, blk, q, k, v, o_final, d_o, lse_final, delta, compute_delta, dq_acc, dk, dv,
                              accumulate_dkdv, stream=0):
    _check(_lib.mmsp_attn_step_bwd_static(ctypes.byref(shape), ctypes.byref(blk), _ptr(q), _ptr(k), _ptr(v),
                                          _ptr(o_final), _ptr(d_o), _ptr(lse_final), _ptr(delta), int(compute_delta),
                                          _ptr(dq_acc), _ptr(dk), _ptr(dv), int(accumulate_dkdv), stream or None))


def mmsp_attn_step_bwd(shape, blk, q, k, v, o_final, d_o, lse_final, delta, compute_delta, dq_acc, dk, dv,
                       accumulate_dkdv, workspace=None, workspace_bytes=0, stream=0):
    _check(_lib.mmsp_attn_step_bwd(ctypes.byref(shape), ctypes.byref(blk), _ptr(q), _ptr(k), _ptr(v), _ptr(o_final),
                                   _ptr(d_o), _ptr(lse_final), _ptr(delta), int(compute_delta), _ptr(dq_acc),
                                   _ptr(dk), _ptr(dv), int(accumulate_dkdv), _ptr(workspace), workspace_bytes,
                                   stream or None))
