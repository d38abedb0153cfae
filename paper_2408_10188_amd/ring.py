"""Host loop that drives one virtual rank through its N ring steps (zigzag mode) or through
the single step of the Ulysses head-shard mode.  It only sequences C-ABI calls on one HIP
stream; all arithmetic happens in the kernels.

Device buffers (torch tensors, allocated by the caller):
  q, d_o, o_final   [2C, Hq, d]      io dtype, the rank's local rows (chunk r then chunk 2N-1-r)
  k_zz, v_zz        [N, 2C, Hkv, d]  io dtype, every rank's K/V block in zigzag order
  o_acc, dq         [2C, Hq, d]      f32
  lse, delta        [Hq, 2C]         f32
  dk_zz, dv_zz      [N, 2C, Hkv, d]  f32; each step overwrites the rows it reaches, rows that no
                                     query of this rank can see are never written (caller zeroes once)
"""
import math

from . import binding as B


def shape_for(q, k, io_dtype, n_rows, scale=None):
    """mmsp_shape for dense token-major tensors q [rows,Hq,d] and k [..., rows,Hkv,d]."""
    Hq, d = q.shape[-2], q.shape[-1]
    Hkv = k.shape[-2]
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    return B.make_shape(Hq, Hkv, d, io_dtype, scale, (q.stride(-3), q.stride(-2)), (k.stride(-3), k.stride(-2)), n_rows)


def workspace_bytes(shape, n_q, n_k):
    """Workspace that serves both the forward and the backward steps of blocks up to n_q x n_k."""
    return max(B.mmsp_workspace_bytes(shape, n_q, n_k, False), B.mmsp_workspace_bytes(shape, n_q, n_k, True))


def rank_forward(shape, T, N, rank, q, k_zz, v_zz, o_acc, lse, o_final=None, stream=0, fused_merge=True,
                 o_part=None, lse_part=None, ws=None, ws_bytes=0):
    """All N forward steps of `rank`.  fused_merge=True merges in the step kernel's epilogue;
    otherwise every step writes (o_part, lse_part) and mmsp_attn_merge combines them."""
    n_rows = q.shape[0]
    for s in range(N):
        src, blk = B.mmsp_zigzag_plan(T, N, rank, s)
        if fused_merge or s == 0:
            B.mmsp_attn_step_fwd(shape, blk, q, k_zz[src], v_zz[src], o_acc, lse, s > 0, ws, ws_bytes, stream)
        else:
            B.mmsp_attn_step_fwd(shape, blk, q, k_zz[src], v_zz[src], o_part, lse_part, False, ws, ws_bytes, stream)
            B.mmsp_attn_merge(shape, blk.q_row0, blk.n_q, o_acc, lse, o_part, lse_part, None, stream=stream)
    if o_final is not None:
        B.mmsp_attn_merge(shape, 0, n_rows, o_acc, lse, None, None, o_final, stream=stream)


def rank_backward(shape, T, N, rank, q, k_zz, v_zz, o_final, d_o, lse, delta, dq, dk_zz, dv_zz, stream=0, ws=None,
                  ws_bytes=0):
    """delta pre-pass, then all N backward steps of `rank`.  dq must be zero on entry."""
    n_rows = q.shape[0]
    B.mmsp_attn_delta(shape, 0, n_rows, o_final, d_o, delta, stream=stream)
    for s in range(N):
        src, blk = B.mmsp_zigzag_plan(T, N, rank, s)
        B.mmsp_attn_step_bwd(shape, blk, q, k_zz[src], v_zz[src], None, d_o, lse, delta, False, dq,
                             dk_zz[src], dv_zz[src], False, ws, ws_bytes, stream)


def ulysses_forward(shape, T, q, k, v, cu_seqlens, n_docs, o_acc, lse, o_final=None, stream=0, ws=None, ws_bytes=0):
    """Head-shard mode: the whole packed sequence in one step under the document-causal mask."""
    blk = B.make_block(0, T, 0, T, B.MMSP_MASK_CAUSAL_DIAG, 0, 0, cu_seqlens, n_docs)
    B.mmsp_attn_step_fwd(shape, blk, q, k, v, o_acc, lse, False, ws, ws_bytes, stream)
    if o_final is not None:
        B.mmsp_attn_merge(shape, 0, T, o_acc, lse, None, None, o_final, stream=stream)


def ulysses_backward(shape, T, q, k, v, cu_seqlens, n_docs, o_final, d_o, lse, delta, dq, dk, dv, stream=0, ws=None,
                     ws_bytes=0):
    blk = B.make_block(0, T, 0, T, B.MMSP_MASK_CAUSAL_DIAG, 0, 0, cu_seqlens, n_docs)
    B.mmsp_attn_step_bwd(shape, blk, q, k, v, o_final, d_o, lse, delta, True, dq, dk, dv, False, ws, ws_bytes, stream)
