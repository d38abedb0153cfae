"""Parity of the HIP path (through the C-ABI) with the fp64 oracle, element by element, on
seeded inputs small enough for the oracle to finish in seconds yet spanning several tiles
and ragged tails.  Tolerances are the ones the task fixes: max-abs 2e-2 on O/dQ/dK/dV and
1e-3 on LSE for bf16 inputs, 1e-5 on everything for the fp32 configuration."""
import math

import numpy as np
import pytest
import torch

from oracle import mmsp_oracle as orc
from paper_2408_10188_amd import binding as B
from paper_2408_10188_amd import ring, synth
from tests.helpers import DEV, NORTH_STAR_TOL, RankProblem, max_abs, nans, nans_like, to_dev, to_host64

pytestmark = pytest.mark.gpu

TOL_BF16 = NORTH_STAR_TOL["bf16"]
TOL_F32 = NORTH_STAR_TOL["f32"]


def _check_rank(prob, rank, tol, fused_merge=True, backward=True, two_streams=False):
    q, do = prob.rank_inputs(rank)
    out = prob.run_gpu(rank, q, do if backward else None, fused_merge=fused_merge, two_streams=two_streams)
    _, l2g = orc.zigzag_layout(prob.T, prob.N, rank)
    K, V = prob.K_full().astype(np.float64), prob.V_full().astype(np.float64)
    ref = orc.causal_attention(q.astype(np.float64), K, V, prob.scale, q_pos=l2g,
                               dO=do.astype(np.float64) if backward else None)
    errs = dict(o=max_abs(to_host64(out["o_acc"]), ref[0]), lse=max_abs(to_host64(out["lse"]), ref[1]),
                o_final=max_abs(to_host64(out["o_final"]), ref[0]))
    assert errs["o"] <= tol["o"] and errs["lse"] <= tol["lse"], errs
    assert errs["o_final"] <= tol["o"] + (2.0 ** -8 if prob.bf16 else 0) * np.abs(ref[0]).max(), errs
    if backward:
        d_ref = orc.delta(do.astype(np.float64), ref[0])
        errs["delta"] = max_abs(to_host64(out["delta"]), d_ref)
        errs["dq"] = max_abs(to_host64(out["dq"]), ref[2])
        errs["dk"] = max_abs(prob.unzigzag(to_host64(out["dk_zz"])), ref[3])
        errs["dv"] = max_abs(prob.unzigzag(to_host64(out["dv_zz"])), ref[4])
        # the kernel's delta uses the final O rounded to the io dtype (bf16: 2^-9 relative per element)
        assert errs["delta"] <= (5e-2 if prob.bf16 else 1e-4), errs
        assert max(errs["dq"], errs["dk"], errs["dv"]) <= tol["g"], errs
    print(f"rank {rank} errs {errs}", flush=True)
    return out


def test_tiny_fp32_rank0_fwd_merge_bwd():
    """Configuration 1: fp32, 2/1 heads, d 64, T 512, N 2, rank 0 -- both merge variants."""
    prob = RankProblem(synth.CONFIGS["tiny"])
    assert TOL_F32 == dict(o=1e-5, lse=1e-5, g=1e-5)           # the named configuration gets the unscaled bounds
    a = _check_rank(prob, 0, TOL_F32, fused_merge=True)
    b = _check_rank(prob, 0, TOL_F32, fused_merge=False)
    assert max_abs(to_host64(a["o_acc"]), to_host64(b["o_acc"])) <= 2e-6
    _check_rank(prob, 1, TOL_F32)


@pytest.mark.parametrize("Hq,Hkv,N,C", [(4, 2, 2, 160), (7, 1, 3, 96), (2, 2, 1, 200), (6, 3, 2, 96), (8, 8, 2, 64), (32, 16, 1, 96)])
def test_bf16_ring_small_ragged(Hq, Hkv, N, C):
    """bf16 matrix-core path: several 128-row / 64-key tiles plus ragged tails, every rank.  The
    head counts cover both workgroup orders (KV heads that divide the 8 XCDs and that do not)
    and group sizes 1, 2 and 7."""
    cfg = dict(dtype="bf16", Hq=Hq, Hkv=Hkv, d=128, N=N, C=C, sigma=0.5, seed=3)
    prob = RankProblem(cfg)
    for r in range(N):
        _check_rank(prob, r, TOL_BF16, fused_merge=(r % 2 == 0))


@pytest.mark.parametrize("dtype,N,C,d", [("bf16", 4, 160, 128), ("bf16", 1, 128, 128), ("f32", 3, 64, 64)])
def test_ring_on_two_launch_lanes(dtype, N, C, d):
    """Ring steps alternating between two streams and two (O, LSE) accumulators, dQ and dK/dV
    kernels on different streams: same results as the oracle, rows no odd step reaches included."""
    cfg = dict(dtype=dtype, Hq=4, Hkv=2, d=d, N=N, C=C, sigma=0.5, seed=11)
    prob = RankProblem(cfg)
    for r in range(N):
        _check_rank(prob, r, TOL_BF16 if dtype == "bf16" else TOL_F32, two_streams=True)


def test_bf16_ring_reassembles_unsharded_result():
    """All ranks' outputs, un-permuted, equal the unsharded causal result; sum of the ranks'
    dK/dV contributions equals the unsharded dK/dV."""
    cfg = dict(dtype="bf16", Hq=4, Hkv=2, d=128, N=4, C=64, sigma=0.5, seed=5)
    prob = RankProblem(cfg)
    T = prob.T
    O = np.zeros((T, 4, 128)); L = np.zeros((4, T)); dQ = np.zeros((T, 4, 128))
    dK = np.zeros((T, 2, 128)); dV = np.zeros((T, 2, 128))
    Q = np.zeros((T, 4, 128)); dO = np.zeros((T, 4, 128))
    for r in range(prob.N):
        q, do = prob.rank_inputs(r)
        out = prob.run_gpu(r, q, do)
        _, l2g = orc.zigzag_layout(T, prob.N, r)
        Q[l2g], dO[l2g] = q, do
        O[l2g], L[:, l2g], dQ[l2g] = to_host64(out["o_acc"]), to_host64(out["lse"]), to_host64(out["dq"])
        dK += prob.unzigzag(to_host64(out["dk_zz"])); dV += prob.unzigzag(to_host64(out["dv_zz"]))
    ref = orc.causal_attention(Q, prob.K_full().astype(np.float64), prob.V_full().astype(np.float64), prob.scale, dO=dO)
    errs = [max_abs(x, y) for x, y in zip((O, L, dQ, dK, dV), ref)]
    assert errs[0] <= 2e-2 and errs[1] <= 1e-3 and max(errs[2:]) <= 2e-2, errs


def _run_step(io_bf16, Hq, Hkv, d, nq_tot, nk_tot, blk_kw, cu=None, seed=7, accumulate_into=None):
    """One step_fwd + step_bwd call on arbitrary sub-blocks vs the oracle's block functions."""
    rng = np.random.default_rng(seed)
    rnd = lambda *s: (synth.bf16_round(rng.standard_normal(s, dtype=np.float32) * 0.5) if io_bf16
                      else rng.standard_normal(s, dtype=np.float32))
    q, k, v, do = rnd(nq_tot, Hq, d), rnd(nk_tot, Hkv, d), rnd(nk_tot, Hkv, d), rnd(nq_tot, Hq, d)
    scale = 1 / math.sqrt(d)
    qd, kd, vd, dod = (to_dev(x, io_bf16) for x in (q, k, v, do))
    shape = ring.shape_for(qd, kd, B.MMSP_BF16 if io_bf16 else B.MMSP_F32, nq_tot, scale)
    cud = None if cu is None else torch.tensor(cu, dtype=torch.int32, device=DEV)
    blk = B.make_block(cu_seqlens=cud, n_docs=0 if cu is None else len(cu) - 1, **blk_kw)
    sentinel = 123.0
    o = torch.full((nq_tot, Hq, d), sentinel, dtype=torch.float32, device=DEV)
    lse = torch.full((Hq, nq_tot), sentinel, dtype=torch.float32, device=DEV)
    ws_bytes = ring.workspace_bytes(shape, blk_kw["n_q"], blk_kw["n_k"])
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=DEV)
    B.mmsp_attn_step_fwd(shape, blk, qd, kd, vd, o, lse, 0, ws, ws_bytes)
    torch.cuda.synchronize()
    ob = dict(q_row0=blk_kw["q_row0"], n_q=blk_kw["n_q"], k_row0=blk_kw["k_row0"], n_k=blk_kw["n_k"],
              q_pos0=blk_kw.get("q_pos0", 0), k_pos0=blk_kw.get("k_pos0", 0), mask=blk_kw["mask"])
    q64, k64, v64, do64 = (x.astype(np.float64) for x in (q, k, v, do))
    O_ref, L_ref = orc.step_fwd(q64, k64, v64, ob, scale, cu)
    r0, r1 = ob["q_row0"], ob["q_row0"] + ob["n_q"]
    tol = TOL_BF16 if io_bf16 else TOL_F32
    og, lg = to_host64(o), to_host64(lse)
    assert max_abs(og[r0:r1], O_ref) <= tol["o"], max_abs(og[r0:r1], O_ref)
    assert max_abs(lg[:, r0:r1], L_ref) <= tol["lse"], max_abs(lg[:, r0:r1], L_ref)
    # rows outside the block are untouched
    assert np.all(og[:r0] == sentinel) and np.all(og[r1:] == sentinel)
    assert np.all(lg[:, :r0] == sentinel) and np.all(lg[:, r1:] == sentinel)
    # backward of the same block, treating this block as the whole problem
    D_ref = orc.delta(do64[r0:r1], O_ref)
    lse_full = torch.zeros((Hq, nq_tot), dtype=torch.float32, device=DEV)
    lse_full[:, r0:r1] = torch.from_numpy(L_ref.astype(np.float32)).to(DEV)
    delta = torch.zeros((Hq, nq_tot), dtype=torch.float32, device=DEV)
    delta[:, r0:r1] = torch.from_numpy(D_ref.astype(np.float32)).to(DEV)
    dq = torch.zeros((nq_tot, Hq, d), dtype=torch.float32, device=DEV)
    dk = torch.full((nk_tot, Hkv, d), sentinel, dtype=torch.float32, device=DEV)
    dv = torch.full((nk_tot, Hkv, d), sentinel, dtype=torch.float32, device=DEV)
    B.mmsp_attn_step_bwd(shape, blk, qd, kd, vd, None, dod, lse_full, delta, 0, dq, dk, dv, 0, ws, ws_bytes)
    torch.cuda.synchronize()
    Dfull = np.zeros((Hq, nq_tot)); Dfull[:, r0:r1] = D_ref
    Lfull = np.zeros((Hq, nq_tot)); Lfull[:, r0:r1] = L_ref
    dq_ref, dk_ref, dv_ref = orc.step_bwd(q64, k64, v64, do64, Lfull, Dfull, ob, scale, cu)
    k0, k1 = ob["k_row0"], ob["k_row0"] + ob["n_k"]
    dqg, dkg, dvg = to_host64(dq), to_host64(dk), to_host64(dv)
    errs = (max_abs(dqg[r0:r1], dq_ref), max_abs(dkg[k0:k1], dk_ref), max_abs(dvg[k0:k1], dv_ref))
    # fp32: 1e-5 is the bound for values of order one (the Tiny configuration); a gradient that sums hundreds of
    # terms into values of order ten carries fp32 rounding in proportion, so the bound scales with the magnitude
    mag = 1.0 if io_bf16 else max(1.0, float(np.abs(dq_ref).max(initial=0)), float(np.abs(dk_ref).max(initial=0)),
                                  float(np.abs(dv_ref).max(initial=0)))
    assert max(errs) <= tol["g"] * mag, errs
    assert np.all(dqg[:r0] == 0) and np.all(dqg[r1:] == 0)
    assert np.all(dkg[:k0] == sentinel) and np.all(dkg[k1:] == sentinel)
    assert np.all(dvg[:k0] == sentinel) and np.all(dvg[k1:] == sentinel)
    # accumulate_dkdv adds on top
    B.mmsp_attn_step_bwd(shape, blk, qd, kd, vd, None, dod, lse_full, delta, 0, dq, dk, dv, 1, ws, ws_bytes)
    torch.cuda.synchronize()
    assert max_abs(to_host64(dk)[k0:k1], 2 * dk_ref) <= 2 * tol["g"] * mag
    assert max_abs(to_host64(dq)[r0:r1], 2 * dq_ref) <= 2 * tol["g"] * mag
    return errs


STEP_CASES = [
    # ragged sub-blocks, all three masks, offsets that put the diagonal inside / before / after the block
    dict(q_row0=0, n_q=300, k_row0=0, n_k=300, mask=B.MMSP_MASK_CAUSAL_DIAG),
    dict(q_row0=37, n_q=150, k_row0=21, n_k=201, mask=B.MMSP_MASK_FULL),
    dict(q_row0=5, n_q=131, k_row0=64, n_k=190, mask=B.MMSP_MASK_CAUSAL_DIAG, q_pos0=100, k_pos0=40),
    dict(q_row0=0, n_q=129, k_row0=0, n_k=65, mask=B.MMSP_MASK_CAUSAL_DIAG, q_pos0=0, k_pos0=30),   # early rows see nothing
    dict(q_row0=10, n_q=1, k_row0=3, n_k=1, mask=B.MMSP_MASK_FULL),
    dict(q_row0=0, n_q=200, k_row0=0, n_k=100, mask=B.MMSP_MASK_NONE),
    dict(q_row0=0, n_q=64, k_row0=0, n_k=0, mask=B.MMSP_MASK_FULL),
]


@pytest.mark.parametrize("case", range(len(STEP_CASES)))
@pytest.mark.parametrize("io_bf16", [True, False])
def test_step_blocks_ragged_and_degenerate(case, io_bf16):
    d = 128 if io_bf16 else 64
    _run_step(io_bf16, 6, 2, d, 320, 320, STEP_CASES[case], seed=20 + case)


@pytest.mark.parametrize("io_bf16", [True, False])
@pytest.mark.parametrize("mask", [B.MMSP_MASK_CAUSAL_DIAG, B.MMSP_MASK_FULL])
def test_step_with_packed_documents(io_bf16, mask):
    """cu_seqlens: document boundaries inside tiles, a 1-token document, block offset into the pack."""
    cu = [0, 100, 101, 333, 400, 700]
    d = 128 if io_bf16 else 64
    _run_step(io_bf16, 4, 2, d, 700, 700, dict(q_row0=0, n_q=700, k_row0=0, n_k=700, mask=mask), cu=cu, seed=31)
    _run_step(io_bf16, 4, 2, d, 400, 500,
              dict(q_row0=50, n_q=300, k_row0=20, n_k=450, mask=mask, q_pos0=250, k_pos0=80), cu=cu, seed=32)


@pytest.mark.parametrize("n_k,n_q,documents", [
    (4261, 200, True),      # 34 key tiles x 8 KV heads = 272 workgroups: no cut, direct store (and its read-modify-write)
    (4224, 64, False),      # the same with whole tiles and one query tile
    (2811, 131, True),      # 22 key tiles -> query ranges cut in 2
    (2048, 200, False),     # 16 -> 4
    (1153, 77, True),       # 10 -> 6
    (1100, 200, True),      # 9 -> 7
])
def test_dkdv_with_and_without_cut_query_ranges(n_k, n_q, documents):
    """Many KV heads and a long key block with few query rows: the dK/dV kernel then runs one
    workgroup per key tile (storing its result directly, adding to dk/dv in place when asked to
    accumulate) or cuts the query range in 2..7 partial sums.  Causal mask with the block's rows
    near the end of the key range, with and without document boundaries; _run_step checks dK, dV
    (and dQ) element by element against the oracle for accumulate 0 and then 1."""
    q_pos0 = n_k - n_q // 2                     # the diagonal crosses the last key tiles; the last rows see every key
    cu = [0, 700, 701, n_k - 30, n_k + n_q] if documents else None   # the block's rows straddle the last boundary
    _run_step(True, 8, 8, 128, n_q, n_k, dict(q_row0=0, n_q=n_q, k_row0=0, n_k=n_k, mask=B.MMSP_MASK_CAUSAL_DIAG,
                                              q_pos0=q_pos0, k_pos0=0), cu=cu, seed=60 + n_q)
    if not documents:                           # every pair visible: the variant without masking
        _run_step(True, 8, 8, 128, n_q, n_k, dict(q_row0=0, n_q=n_q, k_row0=0, n_k=n_k, mask=B.MMSP_MASK_FULL),
                  seed=61 + n_q)


@pytest.mark.parametrize("two_streams", [False, True])
@pytest.mark.parametrize("cu", [[0, 100, 101, 333, 400, 700], [50, 300, 650], [0, 700]])
def test_head_shard_backward_in_query_blocks(cu, two_streams):
    """ring.ulysses_backward cut into 128-row query blocks (document boundaries inside blocks,
    blocks inside one document, rows outside every document): every dQ, dK and dV element
    against the oracle, and dK/dV written without relying on their previous contents."""
    T, Hq, Hkv, d = 700, 4, 2, 128
    scale = 1 / math.sqrt(d)
    rng = np.random.default_rng(90 + len(cu))
    rnd = lambda *s: synth.bf16_round(rng.standard_normal(s, dtype=np.float32) * 0.5)
    q, k, v, do = rnd(T, Hq, d), rnd(T, Hkv, d), rnd(T, Hkv, d), rnd(T, Hq, d)
    qd, kd, vd, dod = (to_dev(x, True) for x in (q, k, v, do))
    cua = np.asarray(cu, dtype=np.int32)
    cud = torch.from_numpy(cua).to(DEV)
    shape = ring.shape_for(qd, kd, B.MMSP_BF16, T, scale)
    o_acc, lse, o_final, delta = nans(T, Hq, d), nans(Hq, T), nans_like(qd), nans(Hq, T)
    dq = torch.zeros(T, Hq, d, dtype=torch.float32, device=DEV)
    dk, dv = nans(T, Hkv, d), nans(T, Hkv, d)
    ws_bytes = ring.workspace_bytes(shape, T, T)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=DEV)
    side = ring.SideLane(torch.cuda.Stream(), None, None, torch.empty_like(ws), ws_bytes) if two_streams else None
    ring.ulysses_forward(shape, T, qd, kd, vd, cud, len(cu) - 1, o_acc, lse, o_final, ws=ws, ws_bytes=ws_bytes)
    ring.ulysses_backward(shape, T, qd, kd, vd, cud, len(cu) - 1, o_final, dod, lse, delta, dq, dk, dv, ws=ws,
                          ws_bytes=ws_bytes, side=side, cu_host=cua, q_block=128)
    torch.cuda.synchronize()
    ref = orc.causal_attention(q.astype(np.float64), k.astype(np.float64), v.astype(np.float64), scale, cu_seqlens=cua,
                               dO=do.astype(np.float64))
    errs = [max_abs(to_host64(x), r) for x, r in zip((o_acc, lse, dq, dk, dv), ref)]
    assert errs[0] <= TOL_BF16["o"] and errs[1] <= TOL_BF16["lse"] and max(errs[2:]) <= TOL_BF16["g"], errs


def test_c_caller_runs_a_step(tmp_path):
    """A C99 translation unit that includes only the public header runs one forward and one
    backward step on this process's device buffers; its results equal the binding's bit for bit
    and match the oracle."""
    import ctypes
    import os
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    libdir = os.path.dirname(B.LIB_PATH)
    so = tmp_path / "libc_abi_step.so"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-shared", "-fPIC", "-I", os.path.join(root, "include"),
                    os.path.join(root, "tests", "c_abi_step.c"), "-o", str(so), "-L", libdir, "-lmmsp",
                    "-Wl,-rpath," + libdir], check=True)
    c = ctypes.CDLL(str(so))
    P, I, F = ctypes.c_void_p, ctypes.c_int, ctypes.c_float
    c.c_client_step_fwd.argtypes = [P] * 5 + [I] * 5 + [F]
    c.c_client_step_bwd.argtypes = [P] * 10 + [I] * 5 + [F]
    c.c_client_last_error.restype = ctypes.c_char_p
    n_q, n_k, Hq, Hkv, d = 150, 333, 4, 2, 128
    scale = 1 / math.sqrt(d)
    rng = np.random.default_rng(77)
    rnd = lambda *s: synth.bf16_round(rng.standard_normal(s, dtype=np.float32) * 0.5)
    q, k, v, do = rnd(n_q, Hq, d), rnd(n_k, Hkv, d), rnd(n_k, Hkv, d), rnd(n_q, Hq, d)
    qd, kd, vd, dod = (to_dev(x, True) for x in (q, k, v, do))
    ptr = lambda t: t.data_ptr()
    res = []
    for through_c in (True, False):
        o, lse, delta = nans(n_q, Hq, d), nans(Hq, n_q), nans(Hq, n_q)
        dq = torch.zeros(n_q, Hq, d, dtype=torch.float32, device=DEV)
        dk, dv = nans(n_k, Hkv, d), nans(n_k, Hkv, d)
        shape = ring.shape_for(qd, kd, B.MMSP_BF16, n_q, scale)
        blk = B.make_block(0, n_q, 0, n_k, B.MMSP_MASK_CAUSAL_DIAG, n_k - n_q, 0)
        if through_c:
            st = c.c_client_step_fwd(ptr(qd), ptr(kd), ptr(vd), ptr(o), ptr(lse), n_q, n_k, Hq, Hkv, d, scale)
            assert st == 0, c.c_client_last_error()
        else:
            B.mmsp_attn_step_fwd(shape, blk, qd, kd, vd, o, lse, 0)
        o_final = o.to(torch.bfloat16)
        if through_c:
            st = c.c_client_step_bwd(ptr(qd), ptr(kd), ptr(vd), ptr(o_final), ptr(dod), ptr(lse), ptr(delta), ptr(dq), ptr(dk),
                                     ptr(dv), n_q, n_k, Hq, Hkv, d, scale)
            assert st == 0, c.c_client_last_error()
        else:
            B.mmsp_attn_step_bwd_static(shape, blk, qd, kd, vd, o_final, dod, lse, delta, 1, dq, dk, dv, 0)
        torch.cuda.synchronize()
        res.append([t.cpu().numpy() for t in (o, lse, delta, dq, dk, dv)])
    for a, b in zip(*res):
        assert np.array_equal(a, b)
    ob = dict(q_row0=0, n_q=n_q, k_row0=0, n_k=n_k, q_pos0=n_k - n_q, k_pos0=0, mask=B.MMSP_MASK_CAUSAL_DIAG)
    q64, k64, v64, do64 = (x.astype(np.float64) for x in (q, k, v, do))
    O_ref, L_ref = orc.step_fwd(q64, k64, v64, ob, scale, None)
    assert max_abs(res[0][0], O_ref) <= TOL_BF16["o"] and max_abs(res[0][1], L_ref) <= TOL_BF16["lse"]
    dq_ref, dk_ref, dv_ref = orc.step_bwd(q64, k64, v64, do64, L_ref, orc.delta(do64, O_ref), ob, scale, None)
    assert max(max_abs(res[0][3], dq_ref), max_abs(res[0][4], dk_ref), max_abs(res[0][5], dv_ref)) <= TOL_BF16["g"]


def test_merge_and_cast_kernel():
    rng = np.random.default_rng(40)
    n, H, d = 70, 3, 128
    O1 = rng.standard_normal((n, H, d)).astype(np.float32); O2 = rng.standard_normal((n, H, d)).astype(np.float32)
    L1 = rng.standard_normal((H, n)).astype(np.float32) * 5; L2 = rng.standard_normal((H, n)).astype(np.float32) * 5
    L1[0, :5] = -np.inf; L2[0, 3:8] = -np.inf; L2[1, 10] = -np.inf
    O1[:5, 0] = 0; O2[3:8, 0] = 0
    o_acc, l_acc, o_p, l_p = (torch.from_numpy(x.copy()).to(DEV) for x in (O1, L1, O2, L2))
    shape = B.make_shape(H, H, d, B.MMSP_BF16, 0.1, (H * d, d), (H * d, d), n)
    o_fin = torch.zeros((n, H, d), dtype=torch.bfloat16, device=DEV)
    B.mmsp_attn_merge(shape, 8, 50, o_acc, l_acc, o_p, l_p, o_fin)
    torch.cuda.synchronize()
    O_ref, L_ref = orc.merge(O1[8:58].astype(np.float64), L1[:, 8:58].astype(np.float64),
                             O2[8:58].astype(np.float64), L2[:, 8:58].astype(np.float64))
    og, lg = to_host64(o_acc), to_host64(l_acc)
    assert max_abs(og[8:58], O_ref) <= 1e-5 and max_abs(lg[:, 8:58], L_ref) <= 1e-5
    assert np.array_equal(og[:8], O1[:8]) and np.array_equal(og[58:], O1[58:])      # untouched rows
    assert max_abs(to_host64(o_fin)[8:58], O_ref) <= 2.0 ** -8 * np.abs(O_ref).max()
    # both sides empty -> stays empty, no NaN
    B.mmsp_attn_merge(shape, 0, 8, o_acc, l_acc, o_p, l_p, None)
    torch.cuda.synchronize()
    assert not torch.isnan(o_acc).any() and not torch.isnan(l_acc).any()
    assert torch.isneginf(l_acc[0, 3:5]).all() and (o_acc[3:5, 0] == 0).all()


def test_delta_kernel():
    rng = np.random.default_rng(41)
    for bf16, d in ((True, 128), (False, 64), (False, 128)):
        n, H = 50, 5
        o = rng.standard_normal((n, H, d), dtype=np.float32); do = rng.standard_normal((n, H, d), dtype=np.float32)
        if bf16:
            o, do = synth.bf16_round(o), synth.bf16_round(do)
        od, dod = to_dev(o, bf16), to_dev(do, bf16)
        delta = torch.full((H, n), 9.0, dtype=torch.float32, device=DEV)
        shape = B.make_shape(H, H, d, B.MMSP_BF16 if bf16 else B.MMSP_F32, 0.1, (H * d, d), (H * d, d), n)
        B.mmsp_attn_delta(shape, 3, 40, od, dod, delta)
        torch.cuda.synchronize()
        ref = orc.delta(do.astype(np.float64), o.astype(np.float64))
        got = to_host64(delta)
        assert max_abs(got[:, 3:43], ref[:, 3:43]) <= 1e-4
        assert np.all(got[:, :3] == 9.0) and np.all(got[:, 43:] == 9.0)


def test_backward_is_bit_reproducible():
    """No floating-point atomics: two runs give identical bits."""
    cfg = dict(dtype="bf16", Hq=7, Hkv=1, d=128, N=2, C=192, sigma=0.5, seed=9)
    prob = RankProblem(cfg)
    q, do = prob.rank_inputs(1)
    a = prob.run_gpu(1, q, do)
    b = prob.run_gpu(1, q, do)
    for key in ("o_acc", "lse", "dq", "dk_zz", "dv_zz"):
        assert torch.equal(a[key], b[key]), key


def test_strided_q_and_kv_views():
    """Q and K/V given as head-major views (explicit strides) give the same result as dense,
    forward and backward (both backward kernels and their transposing pre-passes read Q, K, V
    through the strides)."""
    rng = np.random.default_rng(50)
    n, Hq, Hkv, d = 200, 4, 2, 128
    q = synth.bf16_round(rng.standard_normal((n, Hq, d), dtype=np.float32) * 0.5)
    k = synth.bf16_round(rng.standard_normal((n, Hkv, d), dtype=np.float32) * 0.5)
    v = synth.bf16_round(rng.standard_normal((n, Hkv, d), dtype=np.float32) * 0.5)
    do = synth.bf16_round(rng.standard_normal((n, Hq, d), dtype=np.float32))
    qd, kd, vd, dod = to_dev(q, True), to_dev(k, True), to_dev(v, True), to_dev(do, True)
    q_hm = qd.permute(1, 0, 2).contiguous().permute(1, 0, 2)       # [n,Hq,d] view of head-major storage
    k_hm = kd.permute(1, 0, 2).contiguous().permute(1, 0, 2)
    v_hm = vd.permute(1, 0, 2).contiguous().permute(1, 0, 2)
    blk = B.make_block(0, n, 0, n, B.MMSP_MASK_CAUSAL_DIAG)
    outs = []
    for qq, kk, vv in ((qd, kd, vd), (q_hm, k_hm, v_hm)):
        shape = ring.shape_for(qq, kk, B.MMSP_BF16, n)
        o = nans(n, Hq, d)
        lse = nans(Hq, n)
        of = nans(n, Hq, d, dtype=torch.bfloat16)
        delta, dq = nans_like(lse), torch.zeros_like(o)
        dk = torch.zeros((n, Hkv, d), dtype=torch.float32, device=DEV)
        dv = torch.zeros_like(dk)
        ws_bytes = ring.workspace_bytes(shape, n, n)
        ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=DEV)
        B.mmsp_attn_step_fwd(shape, blk, qq, kk, vv, o, lse, 0, ws, ws_bytes)
        B.mmsp_attn_merge(shape, 0, n, o, lse, None, None, of)
        B.mmsp_attn_step_bwd(shape, blk, qq, kk, vv, of, dod, lse, delta, 1, dq, dk, dv, 0, ws, ws_bytes)
        torch.cuda.synchronize()
        outs.append((o, lse, dq, dk, dv))
    for a, b in zip(outs[0], outs[1]):
        assert torch.equal(a, b)
    ref = orc.causal_attention(q.astype(np.float64), k.astype(np.float64), v.astype(np.float64), 1 / math.sqrt(d), dO=do.astype(np.float64))
    assert max_abs(to_host64(outs[1][2]), ref[2]) <= 2e-2 and max_abs(to_host64(outs[1][3]), ref[3]) <= 2e-2
    assert max_abs(to_host64(outs[1][4]), ref[4]) <= 2e-2


@pytest.mark.parametrize("U,R,Hq,Hkv", [(2, 2, 4, 2), (4, 2, 4, 2)])
def test_two_d_attention_shares(U, R, Hq, Hkv):
    """2D-attention: every GPU of a U x R mesh runs the ring steps of its ring rank on its own
    heads (strided head slices of the full tensors); together they must give the unsharded
    causal result of the oracle.  The second case has more head ranks than KV heads."""
    C, d = 96, 128
    cfg = dict(dtype="bf16", Hq=Hq, Hkv=Hkv, d=d, N=R, C=C, sigma=0.5, seed=17)
    prob = RankProblem(cfg)
    T, n = prob.T, 2 * C
    K64, V64 = prob.K_full().astype(np.float64), prob.V_full().astype(np.float64)
    dK_sum = np.zeros((T, Hkv, d)); dV_sum = np.zeros((T, Hkv, d))
    ref_by_rank = {}
    for g in range(U * R):
        sh = B.mmsp_2d_layout(T, U, R, g, Hq, Hkv)
        r, h0, nh, kv0, nkv = sh.ring_rank, sh.q_head0, sh.n_q_heads, sh.kv_head0, sh.n_kv_heads
        q, do = prob.rank_inputs(r)
        if r not in ref_by_rank:
            _, l2g = orc.zigzag_layout(T, R, r)
            ref_by_rank[r] = (l2g, orc.causal_attention(q.astype(np.float64), K64, V64, prob.scale, q_pos=l2g,
                                                        dO=do.astype(np.float64)))
        l2g, ref = ref_by_rank[r]
        qd = to_dev(q, True)[:, h0:h0 + nh]                         # strided views: heads of this GPU only
        k_zz, v_zz = prob.k_zz[:, :, kv0:kv0 + nkv], prob.v_zz[:, :, kv0:kv0 + nkv]
        dod = to_dev(do, True)[:, h0:h0 + nh].contiguous()
        shape = ring.shape_for(qd, k_zz, B.MMSP_BF16, n, prob.scale)
        o_acc = nans(n, nh, d)
        lse = nans(nh, n)
        o_final = nans(n, nh, d, dtype=torch.bfloat16)
        delta, dq = nans_like(lse), torch.zeros_like(o_acc)
        dk = torch.zeros(R, n, nkv, d, dtype=torch.float32, device=DEV)
        dv = torch.zeros_like(dk)
        ws_bytes = ring.workspace_bytes(shape, n, n)
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device=DEV)
        ring.rank_forward(shape, T, R, r, qd, k_zz, v_zz, o_acc, lse, o_final, ws=ws, ws_bytes=ws_bytes)
        ring.rank_backward(shape, T, R, r, qd, k_zz, v_zz, o_final, dod, lse, delta, dq, dk, dv, ws=ws, ws_bytes=ws_bytes)
        torch.cuda.synchronize()
        errs = dict(o=max_abs(to_host64(o_acc), ref[0][:, h0:h0 + nh]), lse=max_abs(to_host64(lse), ref[1][h0:h0 + nh]),
                    dq=max_abs(to_host64(dq), ref[2][:, h0:h0 + nh]))
        assert errs["o"] <= 2e-2 and errs["lse"] <= 1e-3 and errs["dq"] <= 2e-2, (g, errs)
        dK_sum[:, kv0:kv0 + nkv] += prob.unzigzag(to_host64(dk))
        dV_sum[:, kv0:kv0 + nkv] += prob.unzigzag(to_host64(dv))
    # dK / dV: sum over every GPU (ring ranks, and head ranks that share a KV head) = unsharded gradient
    dK_ref = sum(ref_by_rank[r][1][3] for r in range(R))
    dV_ref = sum(ref_by_rank[r][1][4] for r in range(R))
    assert max_abs(dK_sum, dK_ref) <= 2e-2 and max_abs(dV_sum, dV_ref) <= 2e-2


@pytest.mark.parametrize("dtype,N,C,d,cuts", [("bf16", 3, 96, 128, (1, 70, 96, 200, 333, 500)), ("bf16", 2, 160, 128, (320,)),
                                            ("f32", 2, 64, 64, (5, 130, 131))])
def test_zigzag_ring_over_packed_documents(dtype, N, C, d, cuts):
    """Zigzag ring steps with a document mask on global positions (sub-blocks of
    mmsp_zigzag_plan_packed): documents that start and end inside chunks, one that spans a
    chunk boundary, one that exactly fills the first rank's first chunk."""
    cfg = dict(dtype=dtype, Hq=4, Hkv=2, d=d, N=N, C=C, sigma=0.5, seed=23)
    prob = RankProblem(cfg)
    bf16 = dtype == "bf16"
    tol = TOL_BF16 if bf16 else TOL_F32
    T, n = prob.T, 2 * C
    cu = np.array([0, *cuts, T], dtype=np.int32)
    cud = torch.from_numpy(cu).to(DEV)
    K64, V64 = prob.K_full().astype(np.float64), prob.V_full().astype(np.float64)
    dK_sum = np.zeros_like(K64); dV_sum = np.zeros_like(V64)
    dK_ref = np.zeros_like(K64); dV_ref = np.zeros_like(V64)
    for r in range(N):
        q, do = prob.rank_inputs(r)
        _, l2g = orc.zigzag_layout(T, N, r)
        ref = orc.causal_attention(q.astype(np.float64), K64, V64, prob.scale, cu_seqlens=cu, q_pos=l2g, dO=do.astype(np.float64))
        qd, dod = to_dev(q, bf16), to_dev(do, bf16)
        shape = ring.shape_for(qd, prob.k_zz, B.MMSP_BF16 if bf16 else B.MMSP_F32, n, prob.scale)
        o_acc = nans(n, prob.Hq, d)
        lse = nans(prob.Hq, n)
        o_final = nans_like(qd)
        delta, dq = nans_like(lse), torch.zeros_like(o_acc)
        dk = torch.zeros(N, n, prob.Hkv, d, dtype=torch.float32, device=DEV)
        dv = torch.zeros_like(dk)
        ws_bytes = ring.workspace_bytes(shape, n, n)
        ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=DEV)
        cu_host = cu if r % 2 == 0 else None               # with and without the host-side pruning of empty segment pairs
        ring.rank_forward_packed(shape, T, N, r, qd, prob.k_zz, prob.v_zz, cud, len(cu) - 1, o_acc, lse, o_final, ws=ws,
                                 ws_bytes=ws_bytes, cu_host=cu_host)
        ring.rank_backward_packed(shape, T, N, r, qd, prob.k_zz, prob.v_zz, cud, len(cu) - 1, o_final, dod, lse, delta, dq,
                                  dk, dv, ws=ws, ws_bytes=ws_bytes, cu_host=cu_host)
        torch.cuda.synchronize()
        errs = dict(o=max_abs(to_host64(o_acc), ref[0]), lse=max_abs(to_host64(lse), ref[1]), dq=max_abs(to_host64(dq), ref[2]))
        assert errs["o"] <= tol["o"] and errs["lse"] <= tol["lse"] and errs["dq"] <= tol["g"], (r, errs)
        dK_sum += prob.unzigzag(to_host64(dk)); dV_sum += prob.unzigzag(to_host64(dv))
        dK_ref += ref[3]; dV_ref += ref[4]
    assert max_abs(dK_sum, dK_ref) <= tol["g"] and max_abs(dV_sum, dV_ref) <= tol["g"]


def test_contiguous_ring_layout():
    """Plain ring layout through the same calls (mmsp_contiguous_plan): every rank's merged rows
    equal the unsharded causal result; low ranks skip the rounds in which they see nothing."""
    N, L, Hq, Hkv, d = 3, 160, 4, 2, 128
    T = N * L
    rng = np.random.default_rng(61)
    g = lambda H, s: synth.bf16_round(rng.standard_normal((T, H, d), dtype=np.float32) * s)
    Q, K, V, dO = g(Hq, 0.5), g(Hkv, 0.5), g(Hkv, 0.5), g(Hq, 1.0)
    scale = 1 / math.sqrt(d)
    ref = orc.causal_attention(Q.astype(np.float64), K.astype(np.float64), V.astype(np.float64), scale, dO=dO.astype(np.float64))
    k_blk = to_dev(K, True).view(N, L, Hkv, d)
    v_blk = to_dev(V, True).view(N, L, Hkv, d)
    dK = np.zeros((T, Hkv, d)); dV = np.zeros((T, Hkv, d))
    for r in range(N):
        rows = slice(r * L, (r + 1) * L)
        qd, dod = to_dev(Q[rows], True), to_dev(dO[rows], True)
        shape = ring.shape_for(qd, k_blk, B.MMSP_BF16, L, scale)
        o_acc = nans(L, Hq, d)
        lse = nans(Hq, L)
        o_final = nans_like(qd)
        delta, dq = nans_like(lse), torch.zeros_like(o_acc)
        dk = torch.zeros(N, L, Hkv, d, dtype=torch.float32, device=DEV)
        dv = torch.zeros_like(dk)
        ws_bytes = ring.workspace_bytes(shape, L, L)
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device=DEV)
        ring.rank_forward(shape, T, N, r, qd, k_blk, v_blk, o_acc, lse, o_final, ws=ws, ws_bytes=ws_bytes, plan=B.mmsp_contiguous_plan)
        ring.rank_backward(shape, T, N, r, qd, k_blk, v_blk, o_final, dod, lse, delta, dq, dk, dv, ws=ws, ws_bytes=ws_bytes,
                           plan=B.mmsp_contiguous_plan)
        torch.cuda.synchronize()
        errs = dict(o=max_abs(to_host64(o_acc), ref[0][rows]), lse=max_abs(to_host64(lse), ref[1][:, rows]),
                    dq=max_abs(to_host64(dq), ref[2][rows]))
        assert errs["o"] <= 2e-2 and errs["lse"] <= 1e-3 and errs["dq"] <= 2e-2, (r, errs)
        dK += to_host64(dk).reshape(T, Hkv, d); dV += to_host64(dv).reshape(T, Hkv, d)
    assert max_abs(dK, ref[3]) <= 2e-2 and max_abs(dV, ref[4]) <= 2e-2


@pytest.mark.parametrize("T,N,H,d,dtype", [(8, 4, 1, 8, torch.bfloat16), (2304, 3, 7, 128, torch.bfloat16), (1024, 4, 4, 64, torch.float32)])
def test_zigzag_gather_scatter_bit_exact(T, N, H, d, dtype):
    x = torch.randn(T, H, d, device=DEV).to(dtype)
    row_bytes = H * d * x.element_size()
    shards = torch.empty(N, T // N, H, d, dtype=dtype, device=DEV)
    B.mmsp_zigzag_gather(T, N, row_bytes, x, shards)
    back = torch.empty_like(x)
    B.mmsp_zigzag_scatter(T, N, row_bytes, shards, back)
    torch.cuda.synchronize()
    ref = orc.zigzag_gather(x.view(torch.int16 if dtype == torch.bfloat16 else torch.int32).cpu().numpy(), N)
    got = shards.view(torch.int16 if dtype == torch.bfloat16 else torch.int32).cpu().numpy()
    assert np.array_equal(got, ref) and torch.equal(back, x)


@pytest.mark.parametrize("t,U,hh,d", [(5, 4, 2, 8), (1000, 4, 7, 128), (333, 7, 1, 128)])
def test_a2a_head_packing_bit_exact(t, U, hh, d):
    x = torch.randn(t, U * hh, d, device=DEV).bfloat16()
    y = nans(U, t, hh, d, dtype=torch.bfloat16)
    B.mmsp_a2a_pack_heads(t, U, hh * d * 2, x, y)
    back = torch.empty_like(x)
    B.mmsp_a2a_unpack_heads(t, U, hh * d * 2, y, back)
    torch.cuda.synchronize()
    ref = orc.a2a_pack_heads(x.view(torch.int16).cpu().numpy(), U)
    assert np.array_equal(y.view(torch.int16).cpu().numpy(), ref) and torch.equal(back, x)
    assert np.array_equal(orc.a2a_unpack_heads(ref), x.view(torch.int16).cpu().numpy())


@pytest.mark.parametrize("seed", range(64))
def test_random_step_blocks(seed, io_bf16=True, d=128):
    """Seeded random sub-blocks: sizes around the 32 / 64 / 128 / 256-row tile edges, random
    offsets into the tensors, positions that put the causal diagonal anywhere, optional random
    documents (some positions outside every document), random head grouping."""
    rng = np.random.default_rng(1000 + seed)
    edges = np.array([1, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257, 300, 511, 513])
    n_q, n_k = int(rng.choice(edges)), int(rng.choice(edges))
    q_row0, k_row0 = int(rng.integers(0, 70)), int(rng.integers(0, 70))
    Hkv = int(rng.choice([1, 2, 3]))
    Hq = Hkv * int(rng.choice([1, 2, 4]))
    mask = int(rng.choice([B.MMSP_MASK_CAUSAL_DIAG, B.MMSP_MASK_CAUSAL_DIAG, B.MMSP_MASK_FULL]))
    q_pos0, k_pos0 = int(rng.integers(0, 400)), int(rng.integers(0, 400))
    cu = None
    if rng.random() < 0.6:
        hi = max(q_pos0 + n_q, k_pos0 + n_k)
        cuts = np.unique(rng.integers(0, hi + 40, size=int(rng.integers(1, 6))))
        cu = [int(x) for x in cuts]
        if len(cu) < 2:
            cu = [0] + cu if cu[0] > 0 else cu + [hi]
    blk = dict(q_row0=q_row0, n_q=n_q, k_row0=k_row0, n_k=n_k, mask=mask, q_pos0=q_pos0, k_pos0=k_pos0)
    _run_step(io_bf16, Hq, Hkv, d, q_row0 + n_q + int(rng.integers(0, 9)), k_row0 + n_k + int(rng.integers(0, 9)), blk, cu=cu,
              seed=2000 + seed)


@pytest.mark.parametrize("seed", range(16))
def test_random_step_blocks_fp32(seed):
    """The same sweep through the fp32 kernels (head_dim 64 and 128, tolerance 1e-5)."""
    test_random_step_blocks(400 + seed, io_bf16=False, d=64 if seed % 2 else 128)


@pytest.mark.parametrize("seed", range(12))
def test_random_ring_configurations(seed):
    """Seeded random zigzag rings: ring size, chunk length (ragged against every tile size),
    head grouping, one or two launch lanes, with or without packed documents (which may leave
    positions outside every document), with or without host-side pruning of the sub-blocks."""
    rng = np.random.default_rng(5000 + seed)
    N = int(rng.integers(1, 5))
    C = int(rng.choice([16, 33, 64, 96, 130, 200]))
    Hkv = int(rng.choice([1, 2, 3]))
    Hq = Hkv * int(rng.choice([1, 2, 7]))
    cfg = dict(dtype="bf16", Hq=Hq, Hkv=Hkv, d=128, N=N, C=C, sigma=0.5, seed=100 + seed)
    prob = RankProblem(cfg)
    T, n = prob.T, 2 * C
    packed = rng.random() < 0.6
    cu = None
    if packed:
        cuts = np.unique(rng.integers(0, T + 1, size=int(rng.integers(2, 7))))
        cu = cuts.astype(np.int32) if len(cuts) >= 2 else np.array([0, T], dtype=np.int32)
    K64, V64 = prob.K_full().astype(np.float64), prob.V_full().astype(np.float64)
    dK_sum = np.zeros_like(K64); dV_sum = np.zeros_like(V64); dK_ref = np.zeros_like(K64); dV_ref = np.zeros_like(V64)
    for r in range(N):
        q, do = prob.rank_inputs(r)
        _, l2g = orc.zigzag_layout(T, N, r)
        ref = orc.causal_attention(q.astype(np.float64), K64, V64, prob.scale, cu_seqlens=cu, q_pos=l2g, dO=do.astype(np.float64))
        if not packed:
            out = prob.run_gpu(r, q, do, two_streams=bool(rng.integers(0, 2)))
            o_acc, lse, dq, dk, dv = out["o_acc"], out["lse"], out["dq"], out["dk_zz"], out["dv_zz"]
        else:
            qd, dod = to_dev(q, True), to_dev(do, True)
            cud = torch.from_numpy(cu).to(DEV)
            shape = ring.shape_for(qd, prob.k_zz, B.MMSP_BF16, n, prob.scale)
            o_acc = nans(n, Hq, 128)
            lse = nans(Hq, n)
            o_final = nans_like(qd)
            delta, dq = nans_like(lse), torch.zeros_like(o_acc)
            dk = torch.zeros(N, n, Hkv, 128, dtype=torch.float32, device=DEV)
            dv = torch.zeros_like(dk)
            ws_bytes = ring.workspace_bytes(shape, n, n)
            ws = torch.empty(ws_bytes, dtype=torch.uint8, device=DEV)
            cu_host = cu if rng.integers(0, 2) else None
            ring.rank_forward_packed(shape, T, N, r, qd, prob.k_zz, prob.v_zz, cud, len(cu) - 1, o_acc, lse, o_final, ws=ws,
                                     ws_bytes=ws_bytes, cu_host=cu_host)
            ring.rank_backward_packed(shape, T, N, r, qd, prob.k_zz, prob.v_zz, cud, len(cu) - 1, o_final, dod, lse, delta, dq,
                                      dk, dv, ws=ws, ws_bytes=ws_bytes, cu_host=cu_host)
            torch.cuda.synchronize()
        errs = dict(o=max_abs(to_host64(o_acc), ref[0]), lse=max_abs(to_host64(lse), ref[1]), dq=max_abs(to_host64(dq), ref[2]))
        assert errs["o"] <= 2e-2 and errs["lse"] <= 1e-3 and errs["dq"] <= 2e-2, (r, cfg, cu, errs)
        dK_sum += prob.unzigzag(to_host64(dk)); dV_sum += prob.unzigzag(to_host64(dv))
        dK_ref += ref[3]; dV_ref += ref[4]
    assert max_abs(dK_sum, dK_ref) <= 2e-2 and max_abs(dV_sum, dV_ref) <= 2e-2, (cfg, cu)


@pytest.mark.parametrize("sigma,ramp", [(2.0, 0.0), (1.0, 4.0), (3.0, 0.0), (8.0, 0.0)])
def test_large_scores_exercise_the_lazy_rescale(sigma, ramp):
    """Scores whose row maximum keeps growing along the keys (large sigma, or keys scaled up
    with their position), so that the forward's lazy running-maximum update and O rescale run
    many times and the softmax is nearly one-hot; forward and backward against the oracle."""
    rng = np.random.default_rng(77)
    n, Hq, Hkv, d = 700, 2, 1, 128
    q = synth.bf16_round(rng.standard_normal((n, Hq, d), dtype=np.float32) * sigma)
    k = rng.standard_normal((n, Hkv, d), dtype=np.float32) * sigma
    k = synth.bf16_round(k * (1.0 + ramp * np.arange(n, dtype=np.float32)[:, None, None] / n))
    v = synth.bf16_round(rng.standard_normal((n, Hkv, d), dtype=np.float32))
    do = synth.bf16_round(rng.standard_normal((n, Hq, d), dtype=np.float32))
    scale = 1 / math.sqrt(d)
    ref = orc.causal_attention(q.astype(np.float64), k.astype(np.float64), v.astype(np.float64), scale, dO=do.astype(np.float64))
    qd, kd, vd, dod = to_dev(q, True), to_dev(k, True), to_dev(v, True), to_dev(do, True)
    shape = ring.shape_for(qd, kd, B.MMSP_BF16, n, scale)
    blk = B.make_block(0, n, 0, n, B.MMSP_MASK_CAUSAL_DIAG)
    o = nans(n, Hq, d)
    lse = nans(Hq, n)
    of = nans(n, Hq, d, dtype=torch.bfloat16)
    delta, dq = nans_like(lse), torch.zeros_like(o)
    dk = torch.zeros((n, Hkv, d), dtype=torch.float32, device=DEV)
    dv = torch.zeros_like(dk)
    ws_bytes = ring.workspace_bytes(shape, n, n)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=DEV)
    B.mmsp_attn_step_fwd(shape, blk, qd, kd, vd, o, lse, 0, ws, ws_bytes)
    B.mmsp_attn_merge(shape, 0, n, o, lse, None, None, of)
    B.mmsp_attn_step_bwd(shape, blk, qd, kd, vd, of, dod, lse, delta, 1, dq, dk, dv, 0, ws, ws_bytes)
    torch.cuda.synchronize()
    assert float(np.abs(ref[1]).max()) > 10          # far above the lazy-update threshold (8 in the exponent of 2)
    # LSE values of order 100 carry fp32 rounding of order 1e-5 * 100; O and the gradients keep the bf16 bound,
    # scaled by the magnitude of the values they are built from where that exceeds one
    errs = dict(o=max_abs(to_host64(o), ref[0]), lse=max_abs(to_host64(lse), ref[1]), dq=max_abs(to_host64(dq), ref[2]),
                dk=max_abs(to_host64(dk), ref[3]), dv=max_abs(to_host64(dv), ref[4]))
    mags = dict(o=1.0, lse=1.0, dq=max(1.0, np.abs(ref[2]).max()), dk=max(1.0, np.abs(ref[3]).max()), dv=max(1.0, np.abs(ref[4]).max()))
    print("large-score errors", errs, "magnitudes", mags, flush=True)
    assert errs["o"] <= 2e-2 and errs["lse"] <= 1e-3 * max(1.0, np.abs(ref[1]).max() / 10)
    for g in ("dq", "dk", "dv"):
        assert errs[g] <= 2e-2 * mags[g], (g, errs, mags)


@pytest.mark.parametrize("io_bf16", [True, False])
def test_many_tiny_documents(io_bf16):
    """Hundreds of documents of 1 to 5 tokens (every tile cuts many document boundaries), and a
    one-token-per-document pack, where every row sees exactly itself (P = 1, O = V, LSE = s_ii)."""
    rng = np.random.default_rng(91)
    n = 600
    lens = rng.integers(1, 6, size=400)
    cu = np.concatenate([[0], np.cumsum(lens)])
    cu = cu[cu <= n].tolist()
    if cu[-1] != n:
        cu.append(n)
    d = 128 if io_bf16 else 64
    for mask in (B.MMSP_MASK_CAUSAL_DIAG, B.MMSP_MASK_FULL):
        _run_step(io_bf16, 4, 2, d, n, n, dict(q_row0=0, n_q=n, k_row0=0, n_k=n, mask=mask), cu=cu, seed=92)
    _run_step(io_bf16, 2, 1, d, 300, 300, dict(q_row0=0, n_q=300, k_row0=0, n_k=300, mask=B.MMSP_MASK_CAUSAL_DIAG),
              cu=list(range(301)), seed=93)
