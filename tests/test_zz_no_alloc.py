"""The allocation-free backward entry point (mmsp_attn_step_bwd_static, scratch built into the
library's device image) against mmsp_attn_step_bwd with a caller workspace, through the C-ABI:
same kernels, so every output must agree bit for bit, on two calls in a row that share the
built-in scratch, the second on a smaller block (so stale contents of the first would show)."""
import math

import numpy as np
import pytest
import torch

from paper_2408_10188_amd import binding as B
from paper_2408_10188_amd import ring, synth
from tests.helpers import DEV, nans, to_dev

pytestmark = pytest.mark.gpu


def _problem(seed, n_q, n_k, Hq, Hkv, d, mask, bf16, k_pos0=0, q_pos0=0):
    rng = np.random.default_rng(seed)
    rnd = lambda *s: (synth.bf16_round(rng.standard_normal(s, dtype=np.float32) * 0.5) if bf16
                      else rng.standard_normal(s, dtype=np.float32))
    q, k, v, do = rnd(n_q, Hq, d), rnd(n_k, Hkv, d), rnd(n_k, Hkv, d), rnd(n_q, Hq, d)
    qd, kd, vd, dod = (to_dev(x, bf16) for x in (q, k, v, do))
    shape = ring.shape_for(qd, kd, B.MMSP_BF16 if bf16 else B.MMSP_F32, n_q, 1 / math.sqrt(d))
    blk = B.make_block(0, n_q, 0, n_k, mask, q_pos0, k_pos0)
    return shape, blk, qd, kd, vd, dod


def _both_ways(shape, blk, qd, kd, vd, dod, n_q, n_k, Hq, Hkv, d, calls=1):
    """Forward (to get LSE and O), then the backward through both entry points."""
    o = nans(n_q, Hq, d); lse = nans(Hq, n_q)
    ws_bytes = ring.workspace_bytes(shape, n_q, n_k)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=DEV)
    B.mmsp_attn_step_fwd(shape, blk, qd, kd, vd, o, lse, 0, ws, ws_bytes)
    o_final = torch.empty_like(qd)
    B.mmsp_attn_merge(shape, 0, n_q, o, lse, None, None, o_final)
    outs = []
    for static in (False, True):
        delta = nans(Hq, n_q)
        dq = torch.zeros(n_q, Hq, d, dtype=torch.float32, device=DEV)
        dk, dv = nans(n_k, Hkv, d), nans(n_k, Hkv, d)
        for c in range(calls):                            # second call: accumulate on top of the first
            if static:
                B.mmsp_attn_step_bwd_static(shape, blk, qd, kd, vd, o_final, dod, lse, delta, 1, dq, dk, dv, c > 0)
            else:
                B.mmsp_attn_step_bwd(shape, blk, qd, kd, vd, o_final, dod, lse, delta, 1, dq, dk, dv, c > 0, ws, ws_bytes)
        torch.cuda.synchronize()
        outs.append([t.cpu().numpy() for t in (delta, dq, dk, dv)])
    return outs


def _assert_identical(outs):
    for name, a, b in zip(("delta", "dq", "dk", "dv"), *outs):
        assert np.all(np.isfinite(a)), name
        assert np.array_equal(a, b), (name, float(np.abs(a - b).max()))
    assert float(np.abs(outs[0][1]).max()) > 0 and float(np.abs(outs[0][2]).max()) > 0


def test_static_scratch_matches_workspace_on_two_calls_in_a_row():
    Hq, Hkv, d = 4, 2, 128
    # 1) few key tiles: the dK/dV kernel cuts query ranges and sums partial results through the scratch
    big = dict(n_q=700, n_k=520, Hq=Hq, Hkv=Hkv, d=d)
    p = _problem(11, mask=B.MMSP_MASK_CAUSAL_DIAG, bf16=True, q_pos0=0, k_pos0=0, **big)
    _assert_identical(_both_ways(*p, **big, calls=2))
    # 2) right after it a smaller, ragged block whose statistics and partial sums cover only part of
    #    what call 1 left in the scratch
    small = dict(n_q=131, n_k=77, Hq=Hq, Hkv=Hkv, d=d)
    p = _problem(12, mask=B.MMSP_MASK_FULL, bf16=True, **small)
    _assert_identical(_both_ways(*p, **small))


def test_static_entry_serves_f32_without_scratch():
    cfg = dict(n_q=40, n_k=56, Hq=2, Hkv=1, d=64)
    p = _problem(13, mask=B.MMSP_MASK_CAUSAL_DIAG, bf16=False, **cfg)
    _assert_identical(_both_ways(*p, **cfg))
