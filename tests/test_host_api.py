"""CPU-side checks of the boundary: the library loads, exports everything the header
declares, lays out the zigzag shards exactly like the oracle, and rejects bad arguments with
a status (nothing here launches a kernel)."""
import os
import re

import numpy as np
import pytest

from oracle import mmsp_oracle as orc
from paper_2408_10188_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "mmsp.h")).read()
    declared = set(re.findall(r"\b(mmsp_[a-z0-9_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(B._lib, name), name


@pytest.mark.parametrize("T,N", [(8, 4), (512, 2), (16384, 4), (65536, 8), (262144, 32), (96, 3)])
def test_layout_and_plan_match_the_oracle_bit_for_bit(T, N):
    for r in range(N):
        ids, l2g = B.mmsp_zigzag_layout(T, N, r)
        ids_o, l2g_o = orc.zigzag_layout(T, N, r)
        assert list(ids) == ids_o.tolist()
        assert l2g.dtype == np.int64 and np.array_equal(l2g, l2g_o)
        for s in range(N):
            src, blk = B.mmsp_zigzag_plan(T, N, r, s)
            ref = orc.zigzag_plan(T, N, r, s)
            got = dict(src=src, q_row0=blk.q_row0, n_q=blk.n_q, k_row0=blk.k_row0, n_k=blk.n_k,
                       q_pos0=blk.q_pos0, k_pos0=blk.k_pos0, mask=blk.mask)
            assert got == ref
            assert blk.cu_seqlens is None and blk.n_docs == 0


@pytest.mark.parametrize("T,N", [(8, 4), (96, 3), (65536, 8), (262144, 32)])
def test_packed_plan_matches_the_oracle_bit_for_bit(T, N):
    for r in range(N):
        for s in range(N):
            src, blks = B.mmsp_zigzag_plan_packed(T, N, r, s)
            src_o, blks_o = orc.zigzag_plan_packed(T, N, r, s)
            assert src == src_o and len(blks) == len(blks_o)
            for blk, ref in zip(blks, blks_o):
                got = dict(src=src, q_row0=blk.q_row0, n_q=blk.n_q, k_row0=blk.k_row0, n_k=blk.n_k,
                           q_pos0=blk.q_pos0, k_pos0=blk.k_pos0, mask=blk.mask)
                assert got == ref and blk.cu_seqlens is None and blk.n_docs == 0
    with pytest.raises(B.MmspError):
        B.mmsp_zigzag_plan_packed(T, N, 0, N)


@pytest.mark.parametrize("T,N,cu", [(48, 3, [0, 5, 8, 9, 30, 48]), (64, 4, [0, 64]), (64, 4, [0, 8, 16, 24, 32, 40, 48, 56, 64]),
                                    (64, 2, [3, 20, 50]), (96, 3, [0, 16, 17, 33, 80, 96])])
def test_packed_plan_pruning_matches_the_oracle(T, N, cu):
    """With the host copy of cu_seqlens the plan drops exactly the segment pairs in which the
    oracle's visibility matrix is empty (documents aligned with chunks, spanning several, or
    leaving positions outside every document)."""
    cu = np.asarray(cu, dtype=np.int32)
    dropped = 0
    for r in range(N):
        for s in range(N):
            src, blks = B.mmsp_zigzag_plan_packed(T, N, r, s, cu_host=cu)
            src_o, blks_o = orc.zigzag_plan_packed(T, N, r, s, cu)
            got = [(b.q_row0, b.k_row0, b.q_pos0, b.k_pos0, b.n_q, b.n_k, b.mask) for b in blks]
            want = [(b["q_row0"], b["k_row0"], b["q_pos0"], b["k_pos0"], b["n_q"], b["n_k"], b["mask"]) for b in blks_o]
            assert src == src_o and got == want
            dropped += len(orc.zigzag_plan_packed(T, N, r, s)[1]) - len(blks)
    assert dropped > 0 or len(cu) == 2


@pytest.mark.parametrize("T,N", [(8, 4), (30, 3), (262144, 32)])
def test_contiguous_plan_matches_the_oracle_bit_for_bit(T, N):
    for r in range(N):
        for s in range(N):
            src, blk = B.mmsp_contiguous_plan(T, N, r, s)
            ref = orc.contiguous_plan(T, N, r, s)
            got = dict(src=src, q_row0=blk.q_row0, n_q=blk.n_q, k_row0=blk.k_row0, n_k=blk.n_k,
                       q_pos0=blk.q_pos0, k_pos0=blk.k_pos0, mask=blk.mask)
            assert got == ref
    for bad in [(10, 4, 0, 0), (8, 4, 4, 0), (8, 4, 0, 4), (0, 4, 0, 0), (8, 0, 0, 0)]:
        with pytest.raises(B.MmspError):
            B.mmsp_contiguous_plan(*bad)


def test_layout_of_the_papers_example():
    got = [B.mmsp_zigzag_layout(8, 4, r)[1].tolist() for r in range(4)]
    assert got == [[0, 7], [1, 6], [2, 5], [3, 4]]


@pytest.mark.parametrize("T,U,R,Hq,Hkv", [(8, 2, 2, 2, 2), (48, 4, 2, 8, 2), (262144, 4, 8, 28, 4), (24, 8, 1, 8, 2), (64, 1, 4, 6, 3)])
def test_two_d_layout_matches_the_oracle_bit_for_bit(T, U, R, Hq, Hkv):
    for g in range(U * R):
        sh = B.mmsp_2d_layout(T, U, R, g, Hq, Hkv)
        ref = orc.two_d_share(T, U, R, g, Hq, Hkv)
        assert (sh.head_rank, sh.ring_rank) == (ref["u"], ref["r"])
        assert list(range(sh.q_head0, sh.q_head0 + sh.n_q_heads)) == ref["q_heads"].tolist()
        assert list(range(sh.kv_head0, sh.kv_head0 + sh.n_kv_heads)) == ref["kv_heads"].tolist()
        assert list(sh.chunk_ids) == ref["chunk_ids"].tolist() and sh.chunk_len == T // (2 * R)


@pytest.mark.parametrize("args", [(8, 0, 2, 0, 2, 2), (8, 2, 2, 4, 2, 2), (8, 2, 2, -1, 2, 2), (10, 2, 2, 0, 2, 2),
                                  (8, 3, 2, 0, 4, 2), (8, 2, 2, 0, 6, 4), (24, 4, 1, 0, 12, 6)])
def test_two_d_layout_rejects_bad_arguments(args):
    with pytest.raises(B.MmspError) as e:
        B.mmsp_2d_layout(*args)
    assert e.value.status == B.MMSP_ERR_INVALID_ARG


@pytest.mark.parametrize("T,N,rank", [(10, 4, 0), (8, 0, 0), (8, 4, 4), (8, 4, -1), (0, 1, 0), (-8, 4, 0)])
def test_layout_rejects_bad_arguments(T, N, rank):
    with pytest.raises(B.MmspError) as e:
        B.mmsp_zigzag_layout(T, N, rank)
    assert e.value.status == B.MMSP_ERR_INVALID_ARG
    assert B.mmsp_last_error() != ""


def test_plan_rejects_bad_step():
    for step in (-1, 4):
        with pytest.raises(B.MmspError) as e:
            B.mmsp_zigzag_plan(8, 4, 0, step)
        assert e.value.status == B.MMSP_ERR_INVALID_ARG


def _shape(**kw):
    base = dict(n_q_heads=4, n_kv_heads=2, head_dim=128, io_dtype=B.MMSP_BF16, softmax_scale=0.1,
                q_strides=(512, 128), kv_strides=(256, 128), lse_head_stride=64)
    base.update(kw)
    return B.make_shape(**base)


FAKE = 0x1000  # a 16-byte aligned non-NULL value; never dereferenced because validation fails first


@pytest.mark.parametrize("shape_kw,blk_kw,status", [
    (dict(n_kv_heads=3), {}, B.MMSP_ERR_INVALID_ARG),
    (dict(head_dim=96), {}, B.MMSP_ERR_UNSUPPORTED),
    (dict(head_dim=64), {}, B.MMSP_ERR_UNSUPPORTED),               # bf16 needs 128
    (dict(io_dtype=7), {}, B.MMSP_ERR_INVALID_ARG),
    (dict(softmax_scale=0.0), {}, B.MMSP_ERR_INVALID_ARG),
    (dict(softmax_scale=float("nan")), {}, B.MMSP_ERR_INVALID_ARG),
    (dict(q_strides=(100, 128)), {}, B.MMSP_ERR_INVALID_ARG),
    (dict(kv_strides=(256, 4)), {}, B.MMSP_ERR_INVALID_ARG),
    ({}, dict(n_q=-1), B.MMSP_ERR_INVALID_ARG),
    ({}, dict(q_row0=60, n_q=8), B.MMSP_ERR_INVALID_ARG),           # beyond lse_head_stride
    ({}, dict(k_row0=-2), B.MMSP_ERR_INVALID_ARG),
    ({}, dict(mask=5), B.MMSP_ERR_INVALID_ARG),
    ({}, dict(n_docs=3), B.MMSP_ERR_INVALID_ARG),                   # n_docs without cu_seqlens
    ({}, dict(q_pos0=1 << 40), B.MMSP_ERR_INVALID_ARG),
    ({}, dict(q_pos0=(1 << 30) - 8), B.MMSP_ERR_INVALID_ARG),       # q_pos0 + n_q leaves the int32-safe range
    ({}, dict(k_pos0=(1 << 30) - 15), B.MMSP_ERR_INVALID_ARG),      # k_pos0 + n_k likewise
])
def test_step_calls_reject_bad_shapes_and_blocks(shape_kw, blk_kw, status):
    shape = _shape(**shape_kw)
    b = dict(q_row0=0, n_q=16, k_row0=0, n_k=16, mask=B.MMSP_MASK_FULL)
    b.update(blk_kw)
    blk = B.make_block(**b)
    with pytest.raises(B.MmspError) as e:
        B.mmsp_attn_step_fwd(shape, blk, FAKE, FAKE, FAKE, FAKE, FAKE, 0)
    assert e.value.status == status
    with pytest.raises(B.MmspError) as e:
        B.mmsp_attn_step_bwd(shape, blk, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 0, FAKE, FAKE, FAKE, 0)
    assert e.value.status == status


def test_null_and_misaligned_pointers_are_rejected():
    shape, blk = _shape(), B.make_block(0, 16, 0, 16, B.MMSP_MASK_FULL)
    with pytest.raises(B.MmspError) as e:
        B.mmsp_attn_step_fwd(shape, blk, None, FAKE, FAKE, FAKE, FAKE, 0)
    assert e.value.status == B.MMSP_ERR_INVALID_ARG
    with pytest.raises(B.MmspError) as e:
        B.mmsp_attn_step_fwd(shape, blk, FAKE + 2, FAKE, FAKE, FAKE, FAKE, 0)
    assert e.value.status == B.MMSP_ERR_INVALID_ARG
    with pytest.raises(B.MmspError) as e:
        B.mmsp_attn_merge(shape, 0, 16, FAKE, FAKE, FAKE, None, None)
    assert e.value.status == B.MMSP_ERR_INVALID_ARG
    with pytest.raises(B.MmspError) as e:
        B.mmsp_attn_merge(shape, 0, 16, FAKE, FAKE, None, None, None)        # nothing to do
    assert e.value.status == B.MMSP_ERR_INVALID_ARG
    with pytest.raises(B.MmspError) as e:
        B.mmsp_attn_delta(shape, 0, 16, None, FAKE, FAKE)
    assert e.value.status == B.MMSP_ERR_INVALID_ARG
    with pytest.raises(B.MmspError) as e:
        B.mmsp_attn_step_bwd(shape, blk, FAKE, FAKE, FAKE, None, FAKE, FAKE, FAKE, 1, FAKE, FAKE, FAKE, 0)
    assert e.value.status == B.MMSP_ERR_INVALID_ARG                       # compute_delta without o_final


def test_workspace_size_and_rejection():
    shape = _shape()
    assert B.mmsp_workspace_bytes(shape, 200, 130, 0) == 0    # the forward needs no scratch
    need = B.mmsp_workspace_bytes(shape, 200, 130, 1)
    # backward: two padded statistics rows per query head (4 heads x ceil(200/64) tiles x 64 floats each)
    # plus the fixed area for partial dK / dV sums
    assert need >= 2 * 4 * 4 * 64 * 4 and need % 16 == 0
    assert B.mmsp_workspace_bytes(_shape(io_dtype=B.MMSP_F32, head_dim=64), 200, 130, 1) == 0
    blk = B.make_block(0, 16, 0, 16, B.MMSP_MASK_FULL)
    for ws, nbytes in ((None, 0), (FAKE, 100)):
        with pytest.raises(B.MmspError) as e:
            B.mmsp_attn_step_bwd(shape, blk, FAKE, FAKE, FAKE, None, FAKE, FAKE, FAKE, 0, FAKE, FAKE, FAKE, 0, ws, nbytes)
        assert e.value.status == B.MMSP_ERR_WORKSPACE_TOO_SMALL


def test_backward_checks_the_workspace_before_it_launches_anything():
    """compute_delta with a short workspace: the call must fail on the workspace, not after the
    delta kernel has been enqueued.  Without a GPU a launch would come back as MMSP_ERR_DEVICE,
    so the status also shows that no launch was attempted."""
    shape, blk = _shape(), B.make_block(0, 16, 0, 16, B.MMSP_MASK_FULL)
    for ws, nbytes in ((None, 0), (FAKE, 64)):
        with pytest.raises(B.MmspError) as e:
            B.mmsp_attn_step_bwd(shape, blk, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 1, FAKE, FAKE, FAKE, 0, ws, nbytes)
        assert e.value.status == B.MMSP_ERR_WORKSPACE_TOO_SMALL


def test_data_movement_calls_reject_bad_arguments():
    ok = 4096                                          # any aligned non-NULL addresses: rejected before use
    for fn, args in [(B._lib.mmsp_zigzag_gather, (10, 4, 256, ok, 2 * ok, None)),       # T not a multiple of 2N
                     (B._lib.mmsp_zigzag_gather, (8, 4, 250, ok, 2 * ok, None)),        # row size not a multiple of 16
                     (B._lib.mmsp_zigzag_scatter, (8, 4, 256, ok, ok, None)),           # in place
                     (B._lib.mmsp_zigzag_scatter, (8, 4, 256, None, ok, None)),
                     (B._lib.mmsp_a2a_pack_heads, (8, 0, 256, ok, 2 * ok, None)),
                     (B._lib.mmsp_a2a_pack_heads, (8, 2, 256, ok + 8, 2 * ok, None)),   # misaligned
                     (B._lib.mmsp_a2a_unpack_heads, (-1, 2, 256, ok, 2 * ok, None))]:
        assert fn(*args) == B.MMSP_ERR_INVALID_ARG
        assert B.mmsp_last_error() != ""


def test_header_is_plain_c_and_usable_from_a_c_program(tmp_path):
    """gcc -std=c99 compiles a client of include/mmsp.h; run against the built library it gets
    the same integers as the Python binding."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    exe = tmp_path / "c_abi_check"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "c_abi_check.c"), "-o", str(exe), "-ldl"], check=True)
    out = subprocess.run([str(exe), B.LIB_PATH], check=True, capture_output=True, text=True).stdout.split("\n")
    ids, l2g = B.mmsp_zigzag_layout(8, 4, 1)
    assert out[0] == "layout %d %d %d %d" % (ids[0], ids[1], l2g[0], l2g[1])
    src, blk = B.mmsp_zigzag_plan(262144, 32, 0, 1)
    assert out[1] == "plan %d %d %d %d %d %d" % (src, blk.q_row0, blk.n_q, blk.k_row0, blk.n_k, blk.mask)
    sh = B.mmsp_2d_layout(262144, 4, 8, 13, 28, 4)
    assert out[2] == "2d %d %d %d %d %d %d %d" % (sh.head_rank, sh.ring_rank, sh.q_head0, sh.n_q_heads, sh.kv_head0, sh.n_kv_heads, sh.chunk_len)
    assert out[3] == "ws %d" % B.mmsp_workspace_bytes(B.make_shape(28, 4, 128, B.MMSP_BF16, 0.0883883, (28 * 128, 128), (4 * 128, 128), 8192), 8192, 8192, 1)
    assert out[4] == "bad %d message" % B.MMSP_ERR_INVALID_ARG


def test_static_backward_rejects_blocks_beyond_its_built_in_scratch():
    """4 heads x 300000 rows of statistics exceed the 72 MiB area: refused on the host, with the
    sizes in the message, before any device call (without a GPU one would give MMSP_ERR_DEVICE)."""
    n = 300000
    shape = _shape(lse_head_stride=n)
    blk = B.make_block(0, n, 0, 64, B.MMSP_MASK_FULL)
    with pytest.raises(B.MmspError) as e:
        B.mmsp_attn_step_bwd_static(shape, blk, FAKE, FAKE, FAKE, None, FAKE, FAKE, FAKE, 0, FAKE, FAKE, FAKE, 0)
    assert e.value.status == B.MMSP_ERR_WORKSPACE_TOO_SMALL
    assert "built-in" in str(e.value) and str(72 << 20) in str(e.value)
    # bad arguments are reported as such, as by mmsp_attn_step_bwd
    with pytest.raises(B.MmspError) as e:
        B.mmsp_attn_step_bwd_static(_shape(n_kv_heads=3), B.make_block(0, 16, 0, 16, B.MMSP_MASK_FULL), FAKE, FAKE, FAKE,
                                    None, FAKE, FAKE, FAKE, 0, FAKE, FAKE, FAKE, 0)
    assert e.value.status == B.MMSP_ERR_INVALID_ARG


def test_flop_convention_against_the_papers_complexity_table():
    """The benchmark's forward count for a whole causal sequence is twice the appendix table's
    attention entry (the table counts one operation per multiply-accumulate), apart from the
    diagonal's T / 2 pairs; a factor-of-two slip either way fails here."""
    import os
    from paper_2408_10188_amd import accounting as acc
    path = os.path.join(os.path.dirname(__file__), "golden", "attention_flops_table.txt")
    rows = [ln.split() for ln in open(path) if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 10
    for _, T, L, H, d, printed in rows:
        T, L, H, d, printed = int(T), int(L), int(H), int(d), float(printed)
        # the printed entries follow T^2 d H L to within 2e-4 (and two decimals)
        assert abs(acc.paper_table_tflops(T, d, H, L) - printed) <= 0.006 + 3e-4 * printed
        ours = L * acc.attention_flops(acc.causal_pairs(T), d, H, forward=True, backward=False) / 1e12
        assert abs(ours / (2 * printed) - 1) <= 1.0 / T + 0.006 / printed + 3e-4      # diagonal, print rounding
    # backward = 2.5 x forward; the zigzag ranks' pairs add up to the whole causal triangle
    assert acc.attention_flops(7, 128, 28, False, True) * 2 == acc.attention_flops(7, 128, 28, True, False) * 5
    for N, C in ((4, 2048), (8, 4096), (32, 4096)):
        assert N * acc.zigzag_pairs_of_rank(N, C) == acc.causal_pairs(2 * N * C)
        assert sum(acc.contiguous_pairs_of_rank(N, C, r) for r in range(N)) == acc.causal_pairs(2 * N * C)
    assert acc.packed_pairs([3, 1]) == 7
