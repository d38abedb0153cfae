"""Host loop that drives one virtual rank through its N ring steps (zigzag mode) or through
the single step of the Ulysses head-shard mode.  It only sequences C-ABI calls on HIP
streams; all arithmetic happens in the kernels.

A step's grid rarely fills the 256 CUs a whole number of times, so the last round of its
workgroups leaves CUs idle.  With a `SideLane` the loop keeps two independent chains of
launches in flight on two streams, whose tails fill each other: forward steps alternate between
two (O, LSE) accumulators that one final merge combines (the merge is associative, so any
split of the ring steps gives the same result up to rounding); in the backward the dQ kernels
(chained through dq) run on one stream and the dK/dV kernels (independent per step) on the other.

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


class SideLane:
    """A second HIP stream (torch.cuda.Stream) with the buffers its launches need: an (O, LSE)
    accumulator pair like (o_acc, lse) and a workspace of its own."""

    def __init__(self, stream, o_acc, lse, ws, ws_bytes):
        self.stream, self.o_acc, self.lse, self.ws, self.ws_bytes = stream, o_acc, lse, ws, ws_bytes

    @property
    def handle(self):
        return self.stream.cuda_stream


def _fork(side):
    import torch
    main = torch.cuda.current_stream()
    side.stream.wait_stream(main)
    return main


def rank_forward(shape, T, N, rank, q, k_zz, v_zz, o_acc, lse, o_final=None, stream=0, fused_merge=True,
                 o_part=None, lse_part=None, ws=None, ws_bytes=0, side=None, plan=None):
    """All N forward steps of `rank`.  fused_merge=True merges in the step kernel's epilogue;
    otherwise every step writes (o_part, lse_part) and mmsp_attn_merge combines them.
    With `side` (fused merge only, launches on the current torch stream and on side.stream)
    odd steps accumulate into the side lane and the final merge folds it in.
    `plan` (default mmsp_zigzag_plan) maps (T, N, rank, step) to (src, block); with
    mmsp_contiguous_plan, q and k_zz[r] hold the contiguous chunk r instead of the zigzag pair."""
    n_rows = q.shape[0]
    plan = plan or B.mmsp_zigzag_plan
    if side is not None and N > 1:
        main = _fork(side)
        # rows that no odd step reaches must still hold an empty partial result
        B.mmsp_attn_step_fwd(shape, B.make_block(0, n_rows, 0, 0, B.MMSP_MASK_NONE, 0, 0), q, k_zz[0], v_zz[0],
                             side.o_acc, side.lse, False, side.ws, side.ws_bytes, side.handle)
        for s in range(N):
            src, blk = plan(T, N, rank, s)
            if s & 1:
                B.mmsp_attn_step_fwd(shape, blk, q, k_zz[src], v_zz[src], side.o_acc, side.lse, True, side.ws,
                                     side.ws_bytes, side.handle)
            else:
                B.mmsp_attn_step_fwd(shape, blk, q, k_zz[src], v_zz[src], o_acc, lse, s > 0, ws, ws_bytes,
                                     main.cuda_stream)
        main.wait_stream(side.stream)
        B.mmsp_attn_merge(shape, 0, n_rows, o_acc, lse, side.o_acc, side.lse, o_final, stream=main.cuda_stream)
        return
    for s in range(N):
        src, blk = plan(T, N, rank, s)
        if fused_merge or s == 0:
            B.mmsp_attn_step_fwd(shape, blk, q, k_zz[src], v_zz[src], o_acc, lse, s > 0, ws, ws_bytes, stream)
        else:
            B.mmsp_attn_step_fwd(shape, blk, q, k_zz[src], v_zz[src], o_part, lse_part, False, ws, ws_bytes, stream)
            B.mmsp_attn_merge(shape, blk.q_row0, blk.n_q, o_acc, lse, o_part, lse_part, None, stream=stream)
    if o_final is not None:
        B.mmsp_attn_merge(shape, 0, n_rows, o_acc, lse, None, None, o_final, stream=stream)


def rank_backward(shape, T, N, rank, q, k_zz, v_zz, o_final, d_o, lse, delta, dq, dk_zz, dv_zz, stream=0, ws=None,
                  ws_bytes=0, side=None, plan=None):
    """delta pre-pass, then all N backward steps of `rank`.  dq must be zero on entry.
    With `side` the dQ kernels run on the current torch stream and the dK/dV kernels on
    side.stream (with side's workspace).  `plan` as in rank_forward."""
    n_rows = q.shape[0]
    plan = plan or B.mmsp_zigzag_plan
    if side is not None:
        import torch
        main = torch.cuda.current_stream()
        B.mmsp_attn_delta(shape, 0, n_rows, o_final, d_o, delta, stream=main.cuda_stream)
        side.stream.wait_stream(main)
        for s in range(N):
            src, blk = plan(T, N, rank, s)
            B.mmsp_attn_step_bwd(shape, blk, q, k_zz[src], v_zz[src], None, d_o, lse, delta, False, dq, None, None,
                                 False, ws, ws_bytes, main.cuda_stream)
            B.mmsp_attn_step_bwd(shape, blk, q, k_zz[src], v_zz[src], None, d_o, lse, delta, False, None,
                                 dk_zz[src], dv_zz[src], False, side.ws, side.ws_bytes, side.handle)
        main.wait_stream(side.stream)
        return
    B.mmsp_attn_delta(shape, 0, n_rows, o_final, d_o, delta, stream=stream)
    for s in range(N):
        src, blk = plan(T, N, rank, s)
        B.mmsp_attn_step_bwd(shape, blk, q, k_zz[src], v_zz[src], None, d_o, lse, delta, False, dq,
                             dk_zz[src], dv_zz[src], False, ws, ws_bytes, stream)


def rank_forward_packed(shape, T, N, rank, q, k_zz, v_zz, cu_seqlens, n_docs, o_acc, lse, o_final=None, stream=0,
                        ws=None, ws_bytes=0, cu_host=None):
    """Zigzag ring steps of `rank` over a packed sequence (document-causal mask from cu_seqlens
    on global positions): the sub-blocks of mmsp_zigzag_plan_packed, merged in the step epilogue.
    cu_host (host copy of cu_seqlens) lets the plan skip segment pairs that no document spans."""
    n_rows = q.shape[0]
    B.mmsp_attn_step_fwd(shape, B.make_block(0, n_rows, 0, 0, B.MMSP_MASK_NONE, 0, 0), q, k_zz[0], v_zz[0], o_acc, lse,
                         False, ws, ws_bytes, stream)          # rows whose document lies in no visited segment stay empty
    for s in range(N):
        src, blks = B.mmsp_zigzag_plan_packed(T, N, rank, s, cu_seqlens, n_docs, cu_host)
        for blk in blks:
            B.mmsp_attn_step_fwd(shape, blk, q, k_zz[src], v_zz[src], o_acc, lse, True, ws, ws_bytes, stream)
    if o_final is not None:
        B.mmsp_attn_merge(shape, 0, n_rows, o_acc, lse, None, None, o_final, stream=stream)


def rank_backward_packed(shape, T, N, rank, q, k_zz, v_zz, cu_seqlens, n_docs, o_final, d_o, lse, delta, dq, dk_zz,
                         dv_zz, stream=0, ws=None, ws_bytes=0, cu_host=None):
    """Backward of rank_forward_packed.  dq must be zero on entry; the key rows a step reaches
    are overwritten by its first sub-block and accumulated into by the next one."""
    n_rows = q.shape[0]
    B.mmsp_attn_delta(shape, 0, n_rows, o_final, d_o, delta, stream=stream)
    for s in range(N):
        src, blks = B.mmsp_zigzag_plan_packed(T, N, rank, s, cu_seqlens, n_docs, cu_host)
        seen = set()
        for blk in blks:
            B.mmsp_attn_step_bwd(shape, blk, q, k_zz[src], v_zz[src], None, d_o, lse, delta, False, dq,
                                 dk_zz[src], dv_zz[src], blk.k_row0 in seen, ws, ws_bytes, stream)
            seen.add(blk.k_row0)


def ulysses_forward(shape, T, q, k, v, cu_seqlens, n_docs, o_acc, lse, o_final=None, stream=0, ws=None, ws_bytes=0):
    """Head-shard mode: the whole packed sequence in one step under the document-causal mask."""
    blk = B.make_block(0, T, 0, T, B.MMSP_MASK_CAUSAL_DIAG, 0, 0, cu_seqlens, n_docs)
    B.mmsp_attn_step_fwd(shape, blk, q, k, v, o_acc, lse, False, ws, ws_bytes, stream)
    if o_final is not None:
        B.mmsp_attn_merge(shape, 0, T, o_acc, lse, None, None, o_final, stream=stream)


def ulysses_blocks(T, cu_host, q_block):
    """Cuts the head-shard step into query blocks of q_block rows.  Yields (q_row0, n_q, k_row0,
    n_k, masked): the block's rows against the keys from the start of its first row's document
    up to the block's own start (every pair visible when the block lies inside one document:
    masked = False), then against its own rows (document-causal, masked = True).  Rows outside
    every document see nothing and are left to the masked call."""
    import bisect
    cu = [int(x) for x in cu_host]
    for r0 in range(0, T, q_block):
        r1 = min(T, r0 + q_block)
        i = bisect.bisect_right(cu, r0) - 1
        one_document = 0 <= i < len(cu) - 1 and r1 <= cu[i + 1]
        if one_document:
            if r0 > cu[i]:
                yield r0, r1 - r0, cu[i], r0 - cu[i], False
            yield r0, r1 - r0, r0, r1 - r0, True
        else:
            k0 = min(r0, max(0, cu[max(i, 0)])) if i >= 0 else r0
            yield r0, r1 - r0, k0, r1 - k0, True


def ulysses_backward(shape, T, q, k, v, cu_seqlens, n_docs, o_final, d_o, lse, delta, dq, dk, dv, stream=0, ws=None,
                     ws_bytes=0, side=None, cu_host=None, q_block=None):
    """dq must be zero on entry.  By default one launch per kernel covers the whole sequence.
    With cu_host (host copy of cu_seqlens) and q_block the step is cut into query blocks of
    q_block rows, launched one after the other: the workgroups of a launch then walk the same
    Q / dO rows (dK/dV kernel) at the same time and share them in L2, where one launch over a
    long document lets them drift apart and re-read the operands (measured: an order of
    magnitude less HBM traffic, but no shorter, because every block's launch ends in a partly
    filled round of workgroups).  dk / dv rows are overwritten by the first block that reaches
    them and added to by later ones.
    With `side` the dK/dV kernels run on the current torch stream and the dQ kernels on side.stream."""
    import torch
    main = torch.cuda.current_stream() if side is not None else None
    s_main = main.cuda_stream if side is not None else stream
    B.mmsp_attn_delta(shape, 0, T, o_final, d_o, delta, stream=s_main)
    if side is not None:
        side.stream.wait_stream(main)           # delta and the caller's zeroing of dq
    if cu_host is None or not q_block:
        blocks = [(0, T, 0, T, True)]
    else:
        blocks = list(ulysses_blocks(T, cu_host, q_block))
    written = 0                                 # dk / dv rows below this index hold a result already
    for r0, n_q, k0, n_k, masked in blocks:
        if masked:
            blk = B.make_block(r0, n_q, k0, n_k, B.MMSP_MASK_CAUSAL_DIAG, r0, k0, cu_seqlens, n_docs)
        else:
            blk = B.make_block(r0, n_q, k0, n_k, B.MMSP_MASK_FULL, r0, k0)
        # keys [k0, k0 + n_k): the part below `written` accumulates, the rest is new
        parts = []
        if k0 < written:
            parts.append((k0, min(written, k0 + n_k) - k0, True))
        if k0 + n_k > written:
            parts.append((max(k0, written), k0 + n_k - max(k0, written), False))
        if len(parts) == 1:
            B.mmsp_attn_step_bwd(shape, blk, q, k, v, None, d_o, lse, delta, False, None, dk, dv, parts[0][2],
                                 ws, ws_bytes, s_main)
        else:
            for kk, nn, accumulate in parts:
                sub = B.make_block(r0, n_q, kk, nn, blk.mask, r0, kk, cu_seqlens if masked else None, n_docs if masked else 0)
                B.mmsp_attn_step_bwd(shape, sub, q, k, v, None, d_o, lse, delta, False, None, dk, dv, accumulate,
                                     ws, ws_bytes, s_main)
        written = max(written, k0 + n_k)
        if side is not None:
            B.mmsp_attn_step_bwd(shape, blk, q, k, v, None, d_o, lse, delta, False, dq, None, None, False,
                                 side.ws, side.ws_bytes, side.handle)
        else:
            B.mmsp_attn_step_bwd(shape, blk, q, k, v, None, d_o, lse, delta, False, dq, None, None, False,
                                 ws, ws_bytes, s_main)
    if side is not None:
        main.wait_stream(side.stream)
