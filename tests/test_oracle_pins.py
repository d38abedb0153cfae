"""Pins for the fp64 oracle: each test checks it against something other than itself --
a value the paper prints, a closed form, an invariant, a textbook/library special case,
brute force in pure Python, or finite differences -- chosen so that a dropped term, a
wrong sign or index, or a transposed operand fails at least one of them.
"""
import math
import os

import numpy as np
import pytest
import scipy.special

from oracle import mmsp_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(rng, *shape):
    return rng.standard_normal(shape)


def _read_rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


# ---------------------------------------------------------------- brute force, pure Python
def _brute_force(Q, K, V, scale, cu=None):
    """Scalar loops with math.exp; no numpy arithmetic shared with the oracle."""
    T, Hq, d = Q.shape
    g = Hq // K.shape[1]
    O = np.zeros((T, Hq, V.shape[2]))
    LSE = np.zeros((Hq, T))
    doc = [0] * T
    if cu is not None:
        for k in range(len(cu) - 1):
            for t in range(cu[k], cu[k + 1]):
                doc[t] = k
    for h in range(Hq):
        for i in range(T):
            scores = []
            for j in range(T):
                if j <= i and doc[i] == doc[j]:
                    scores.append((j, scale * sum(Q[i, h, c] * K[j, h // g, c] for c in range(d))))
            z = sum(math.exp(s) for _, s in scores)
            LSE[h, i] = math.log(z)
            for j, s in scores:
                w = math.exp(s) / z
                for c in range(V.shape[2]):
                    O[i, h, c] += w * V[j, h // g, c]
    return O, LSE


@pytest.mark.parametrize("cu", [None, [0, 5, 6, 13, 20]])
def test_forward_matches_pure_python_brute_force(cu):
    rng = np.random.default_rng(1)
    T, Hq, Hkv, d = 20, 4, 2, 5
    Q, K, V = _rand(rng, T, Hq, d), _rand(rng, T, Hkv, d), _rand(rng, T, Hkv, d)
    O, LSE = orc.causal_attention(Q, K, V, 0.37, cu_seqlens=cu)
    Ob, Lb = _brute_force(Q, K, V, 0.37, cu)
    np.testing.assert_allclose(O, Ob, rtol=0, atol=1e-13)
    np.testing.assert_allclose(LSE, Lb, rtol=0, atol=1e-13)


# ---------------------------------------------------------------- closed forms
def test_zero_queries_give_prefix_means_and_log_counts():
    """Q = 0 => all scores 0: LSE[i] = ln(#visible), O[i] = mean of visible V rows,
    dV[j] = sum_{i sees j} dO[i] / #visible(i).  Pins LSE base, diagonal inclusivity, doc mask."""
    rng = np.random.default_rng(2)
    T, H, d = 17, 2, 3
    cu = [0, 4, 11, 17]
    Q = np.zeros((T, H, d))
    K, V, dO = _rand(rng, T, H, d), _rand(rng, T, H, d), _rand(rng, T, H, d)
    O, LSE, dQ, dK, dV = orc.causal_attention(Q, K, V, 1.0, cu_seqlens=cu, dO=dO)
    start = np.concatenate([np.full(cu[k + 1] - cu[k], cu[k]) for k in range(len(cu) - 1)])
    for i in range(T):
        n = i - start[i] + 1
        assert abs(LSE[0, i] - math.log(n)) < 1e-14
        np.testing.assert_allclose(O[i], V[start[i]: i + 1].mean(axis=0), atol=1e-14)
    dV_ref = np.zeros_like(V)
    for i in range(T):
        dV_ref[start[i]: i + 1] += dO[i] / (i - start[i] + 1)
    np.testing.assert_allclose(dV, dV_ref, atol=1e-14)
    np.testing.assert_allclose(dK, 0, atol=1e-14)      # Q = 0 => dK = dS^T Q = 0


def test_scale_enters_the_scores_once():
    """Q and K rows all ones, scale 1/sqrt(d): every score is sqrt(d), LSE = sqrt(d)+ln(i+1)."""
    T, d = 9, 16
    Q = np.ones((T, 1, d)); K = np.ones((T, 1, d)); V = _rand(np.random.default_rng(3), T, 1, d)
    _, LSE = orc.causal_attention(Q, K, V, 1 / math.sqrt(d))
    np.testing.assert_allclose(LSE[0], math.sqrt(d) + np.log(np.arange(1, T + 1)), atol=1e-13)


def test_constant_values_and_constant_keys():
    """V constant => O is that constant; K constant => dS rows sum to 0 so dQ = 0."""
    rng = np.random.default_rng(4)
    T, H, d = 12, 3, 4
    Q, dO = _rand(rng, T, H, d), _rand(rng, T, H, d)
    K = np.tile(_rand(rng, 1, 1, d), (T, 1, 1)); V = np.tile(_rand(rng, 1, 1, d), (T, 1, 1))
    O, LSE, dQ, dK, dV = orc.causal_attention(Q, K, V, 0.5, dO=dO)
    np.testing.assert_allclose(O, np.broadcast_to(V[0], O.shape), atol=1e-14)
    np.testing.assert_allclose(dQ, 0, atol=1e-13)
    K2 = _rand(rng, T, 1, d)
    O2, _, dQ2, dK2, dV2 = orc.causal_attention(Q, K2, V, 0.5, dO=dO)
    np.testing.assert_allclose(O2, np.broadcast_to(V[0], O2.shape), atol=1e-14)


# ---------------------------------------------------------------- library special case
def test_full_mask_block_equals_library_softmax():
    """With everything visible the step is textbook softmax(QK^T*scale)V; scipy's softmax
    and logsumexp give it without any of the oracle's code."""
    rng = np.random.default_rng(5)
    nq, nk, H, d = 7, 11, 2, 6
    Q, K, V = _rand(rng, nq, H, d), _rand(rng, nk, H, d), _rand(rng, nk, H, d)
    blk = dict(q_row0=0, n_q=nq, k_row0=0, n_k=nk, q_pos0=0, k_pos0=0, mask=orc.MASK_FULL)
    O, L = orc.step_fwd(Q, K, V, blk, 0.3)
    for h in range(H):
        S = 0.3 * Q[:, h] @ K[:, h].T
        np.testing.assert_allclose(O[:, h], scipy.special.softmax(S, axis=1) @ V[:, h], atol=1e-13)
        np.testing.assert_allclose(L[h], scipy.special.logsumexp(S, axis=1), atol=1e-13)


def test_causal_diag_block_offsets():
    """CAUSAL_DIAG with position offsets: query at q_pos0+i sees key at k_pos0+j iff
    k_pos0+j <= q_pos0+i.  Checked against the unsharded result restricted to a window."""
    rng = np.random.default_rng(6)
    T, H, d = 24, 2, 4
    Q, K, V = _rand(rng, T, H, d), _rand(rng, T, H, d), _rand(rng, T, H, d)
    q0, k0, nq, nk = 10, 6, 9, 12
    blk = dict(q_row0=q0, n_q=nq, k_row0=k0, n_k=nk, q_pos0=q0, k_pos0=k0, mask=orc.MASK_CAUSAL_DIAG)
    O, L = orc.step_fwd(Q, K, V, blk, 0.4)
    for i in range(nq):
        hi = min(q0 + i, k0 + nk - 1)
        for h in range(H):
            s = 0.4 * K[k0: hi + 1, h] @ Q[q0 + i, h]
            np.testing.assert_allclose(L[h, i], scipy.special.logsumexp(s), atol=1e-13)
            np.testing.assert_allclose(O[i, h], scipy.special.softmax(s) @ V[k0: hi + 1, h], atol=1e-13)


# ---------------------------------------------------------------- merge invariants
def test_merge_over_any_partition_equals_monolithic():
    rng = np.random.default_rng(7)
    nq, nk, Hq, Hkv, d = 6, 40, 4, 2, 5
    Q, K, V = _rand(rng, nq, Hq, d), _rand(rng, nk, Hkv, d), _rand(rng, nk, Hkv, d)
    full = dict(q_row0=0, n_q=nq, k_row0=0, n_k=nk, q_pos0=0, k_pos0=0, mask=orc.MASK_FULL)
    O_ref, L_ref = orc.step_fwd(Q, K, V, full, 0.6)
    for trial in range(5):
        cuts = np.sort(rng.choice(np.arange(0, nk + 1), size=4))      # may repeat -> empty parts
        edges = [0, *cuts.tolist(), nk]
        parts = list(zip(edges[:-1], edges[1:]))
        rng.shuffle(parts)
        O = np.zeros_like(O_ref); L = np.full_like(L_ref, -np.inf)
        for a, b in parts:
            blk = dict(full, k_row0=a, n_k=b - a)
            O_p, L_p = orc.step_fwd(Q, K, V, blk, 0.6)
            O, L = orc.merge(O, L, O_p, L_p)
        np.testing.assert_allclose(O, O_ref, atol=1e-12)
        np.testing.assert_allclose(L, L_ref, atol=1e-12)


def test_merge_identity_and_symmetry():
    rng = np.random.default_rng(8)
    O1, O2 = _rand(rng, 5, 2, 3), _rand(rng, 5, 2, 3)
    L1, L2 = _rand(rng, 2, 5), _rand(rng, 2, 5)
    Z, NI = np.zeros_like(O1), np.full_like(L1, -np.inf)
    O, L = orc.merge(O1, L1, Z, NI)
    assert np.array_equal(O, O1) and np.array_equal(L, L1)
    O, L = orc.merge(Z, NI, Z, NI)
    assert np.all(O == 0) and np.all(np.isneginf(L))
    Oa, La = orc.merge(O1, L1, O2, L2); Ob, Lb = orc.merge(O2, L2, O1, L1)
    np.testing.assert_allclose(Oa, Ob, atol=1e-15); np.testing.assert_allclose(La, Lb, atol=1e-15)
    # two-element closed form: weights are the softmax of (L1, L2)
    w = scipy.special.softmax(np.stack([L1, L2]), axis=0)
    np.testing.assert_allclose(Oa, w[0].T[:, :, None] * O1 + w[1].T[:, :, None] * O2, atol=1e-14)
    np.testing.assert_allclose(La, np.logaddexp(L1, L2), atol=1e-14)


def test_mask_none_block_contributes_nothing():
    rng = np.random.default_rng(9)
    Q, K, V = _rand(rng, 4, 2, 3), _rand(rng, 6, 1, 3), _rand(rng, 6, 1, 3)
    blk = dict(q_row0=0, n_q=4, k_row0=0, n_k=6, q_pos0=0, k_pos0=0, mask=orc.MASK_NONE)
    O, L = orc.step_fwd(Q, K, V, blk, 1.0)
    assert np.all(O == 0) and np.all(np.isneginf(L))
    dq, dk, dv = orc.step_bwd(Q, K, V, _rand(rng, 4, 2, 3), np.zeros((2, 4)), np.zeros((2, 4)), blk, 1.0)
    assert np.all(dq == 0) and np.all(dk == 0) and np.all(dv == 0)


# ---------------------------------------------------------------- zigzag layout
def test_zigzag_matches_the_papers_worked_example():
    for r, t0, t1, pairs in _read_rows("zigzag_8_4.txt"):
        ids, l2g = orc.zigzag_layout(8, 4, int(r))
        assert l2g.tolist() == [int(t0), int(t1)]
        assert ids.tolist() == [int(t0), int(t1)]           # chunk length 1: chunk id == token id
        assert orc.causal_pairs_of_rank(8, 4, int(r)) == int(pairs)


@pytest.mark.parametrize("T,N", [(8, 4), (512, 2), (96, 3), (16384, 4), (262144, 32)])
def test_zigzag_is_a_balanced_bijection(T, N):
    C = T // (2 * N)
    seen = np.zeros(T, dtype=np.int64)
    total = 0
    for r in range(N):
        ids, l2g = orc.zigzag_layout(T, N, r)
        assert ids.tolist() == [r, 2 * N - 1 - r]
        assert np.all(np.diff(l2g[:C]) == 1) and np.all(np.diff(l2g[C:]) == 1) and l2g[C - 1] < l2g[C]
        seen[l2g] += 1
        p = orc.causal_pairs_of_rank(T, N, r)
        assert p == 2 * N * C * C + C                      # equal work on every rank
        total += p
    assert np.all(seen == 1)
    assert total == T * (T + 1) // 2


@pytest.mark.parametrize("T,N", [(8, 4), (48, 3), (64, 1)])
def test_plan_blocks_cover_exactly_the_visible_pairs(T, N):
    """The plan's (rows, mask) triples, laid back onto global positions, must equal the
    causal visibility of the rank's rows -- no pair missing, none extra, none twice."""
    for r in range(N):
        _, l2g = orc.zigzag_layout(T, N, r)
        truth = orc.visible(l2g, np.arange(T))
        got = np.zeros_like(truth, dtype=np.int64)
        srcs = []
        for s in range(N):
            blk = orc.zigzag_plan(T, N, r, s)
            srcs.append(blk["src"])
            _, kv_rows = orc.zigzag_layout(T, N, blk["src"])
            vis = orc.block_visibility(blk)
            qs = slice(blk["q_row0"], blk["q_row0"] + blk["n_q"])
            cols = kv_rows[blk["k_row0"]: blk["k_row0"] + blk["n_k"]]
            got[qs, cols] += vis
        assert sorted(srcs) == list(range(N))
        assert np.array_equal(got, truth.astype(np.int64))


def test_plain_ring_imbalance_example():
    """Contiguous layout, 8 tokens / 4 ranks: rank r has visible work in r+1 of 4 rounds."""
    T, N = 8, 4
    C = T // N
    for r, rounds in _read_rows("plain_ring_8_4.txt"):
        r = int(r)
        q_pos = np.arange(r * C, (r + 1) * C)
        busy = sum(orc.visible(q_pos, np.arange(((r - s) % N) * C, ((r - s) % N + 1) * C)).any() for s in range(N))
        assert busy == int(rounds)


@pytest.mark.parametrize("T,N", [(8, 4), (30, 3), (64, 8)])
def test_contiguous_plan_reproduces_the_imbalance_and_the_unsharded_result(T, N):
    """Plain ring layout: rank r has work in r+1 of N rounds and (r*L^2 + L(L+1)/2) pairs (the
    paper's imbalance); merging its rounds still gives the rows of the unsharded result."""
    rng = np.random.default_rng(T)
    L, Hq, Hkv, d = T // N, 2, 1, 4
    Q, K, V = _rand(rng, T, Hq, d), _rand(rng, T, Hkv, d), _rand(rng, T, Hkv, d)
    scale = 1 / math.sqrt(d)
    O_ref, L_ref = orc.causal_attention(Q, K, V, scale)[:2]
    for r in range(N):
        rows = np.arange(r * L, (r + 1) * L)
        O = np.zeros((L, Hq, d)); Ls = np.full((Hq, L), -np.inf)
        busy = pairs = 0
        for s in range(N):
            blk = orc.contiguous_plan(T, N, r, s)
            src_rows = np.arange(blk["src"] * L, (blk["src"] + 1) * L)
            vis = orc.block_visibility(blk)
            assert np.array_equal(vis, orc.visible(rows, src_rows))       # the mask kind equals the definition on global positions
            busy += bool(vis.any()); pairs += int(vis.sum())
            O, Ls = orc.merge(O, Ls, *orc.step_fwd(Q[rows], K[src_rows], V[src_rows], blk, scale))
        assert busy == r + 1 and pairs == r * L * L + L * (L + 1) // 2
        np.testing.assert_allclose(O, O_ref[rows], atol=1e-12)
        np.testing.assert_allclose(Ls, L_ref[:, rows], atol=1e-12)


# ---------------------------------------------------------------- 2D-attention shares
def test_two_d_share_matches_the_papers_example():
    for g, r, u, head, t0, t1, t2, t3, pairs in _read_rows("two_d_8_2x2.txt"):
        sh = orc.two_d_share(8, 2, 2, int(g), 2, 2)
        assert (sh["r"], sh["u"]) == (int(r), int(u))
        assert sh["q_heads"].tolist() == [int(head)] and sh["kv_heads"].tolist() == [int(head)]
        assert sh["l2g"].tolist() == [int(t0), int(t1), int(t2), int(t3)]
        assert orc.causal_pairs_of_rank(8, 2, sh["r"]) == int(pairs)


@pytest.mark.parametrize("T,U,R,Hq,Hkv", [(8, 2, 2, 2, 2), (48, 4, 2, 8, 2), (64, 2, 4, 4, 4), (262144, 4, 8, 28, 4), (24, 8, 1, 8, 2)])
def test_two_d_shares_partition_heads_and_tokens(T, U, R, Hq, Hkv):
    """Every (query head, token) belongs to exactly one GPU; a GPU holds the KV heads its query
    heads read and no others; GPUs of one all-to-all group share their tokens."""
    seen = np.zeros((Hq, T), dtype=np.int32)
    for g in range(U * R):
        sh = orc.two_d_share(T, U, R, g, Hq, Hkv)
        seen[np.ix_(sh["q_heads"], sh["l2g"])] += 1
        assert set(sh["kv_heads"].tolist()) == {h // (Hq // Hkv) for h in sh["q_heads"].tolist()}
        assert len(sh["q_heads"]) == Hq // U and len(sh["l2g"]) == T // R
        assert np.array_equal(sh["l2g"], orc.two_d_share(T, U, R, (g // U) * U, Hq, Hkv)["l2g"])
    assert np.all(seen == 1)


def test_two_d_sharded_attention_reassembles_the_unsharded_result():
    """Each GPU runs the ring emulation of its ring rank on its own heads only; together they
    give the unsharded O, LSE, dQ and (summed over ring ranks) dK, dV."""
    rng = np.random.default_rng(21)
    U, R, C, Hq, Hkv, d = 2, 2, 3, 4, 2, 5
    T = 2 * R * C
    Q, K, V, dO = _rand(rng, T, Hq, d), _rand(rng, T, Hkv, d), _rand(rng, T, Hkv, d), _rand(rng, T, Hq, d)
    scale = 1 / math.sqrt(d)
    O_ref, L_ref, dQ_ref, dK_ref, dV_ref = orc.causal_attention(Q, K, V, scale, dO=dO)
    O = np.zeros_like(O_ref); L = np.zeros_like(L_ref); dQ = np.zeros_like(Q)
    dK = np.zeros_like(K); dV = np.zeros_like(V)
    for g in range(U * R):
        sh = orc.two_d_share(T, U, R, g, Hq, Hkv)
        qh, kh, l2g, r = sh["q_heads"], sh["kv_heads"], sh["l2g"], sh["r"]
        o, l = orc.ring_rank_fwd(Q[:, qh], K[:, kh], V[:, kh], R, r, scale)
        dq, dk, dv = orc.ring_rank_bwd(Q[:, qh], K[:, kh], V[:, kh], dO[np.ix_(l2g, qh)], o, l, R, r, scale)
        O[np.ix_(l2g, qh)] = o; L[np.ix_(qh, l2g)] = l; dQ[np.ix_(l2g, qh)] = dq
        dK[:, kh] += dk; dV[:, kh] += dv
    for got, ref in [(O, O_ref), (L, L_ref), (dQ, dQ_ref), (dK, dK_ref), (dV, dV_ref)]:
        np.testing.assert_allclose(got, ref, atol=1e-12)


# ---------------------------------------------------------------- ring emulation
@pytest.mark.parametrize("N,C,Hq,Hkv", [(2, 4, 2, 1), (3, 5, 6, 2), (4, 3, 4, 4)])
def test_ring_emulation_reassembles_the_unsharded_result(N, C, Hq, Hkv):
    rng = np.random.default_rng(10)
    T, d = 2 * N * C, 6
    Q, K, V, dO = _rand(rng, T, Hq, d), _rand(rng, T, Hkv, d), _rand(rng, T, Hkv, d), _rand(rng, T, Hq, d)
    scale = 1 / math.sqrt(d)
    O_ref, L_ref, dQ_ref, dK_ref, dV_ref = orc.causal_attention(Q, K, V, scale, dO=dO)
    O = np.zeros_like(O_ref); L = np.zeros_like(L_ref); dQ = np.zeros_like(Q)
    dK = np.zeros_like(K); dV = np.zeros_like(V)
    for r in range(N):
        _, l2g = orc.zigzag_layout(T, N, r)
        o, l = orc.ring_rank_fwd(Q, K, V, N, r, scale)
        O[l2g], L[:, l2g] = o, l
        dq, dk, dv = orc.ring_rank_bwd(Q, K, V, dO[l2g], o, l, N, r, scale)
        dQ[l2g] = dq; dK += dk; dV += dv
        # path A restricted to the rank's rows gives the same contribution
        _, _, dq_a, dk_a, dv_a = orc.causal_attention(Q[l2g], K, V, scale, q_pos=l2g, dO=dO[l2g])
        np.testing.assert_allclose(dq, dq_a, atol=1e-12)
        np.testing.assert_allclose(dk, dk_a, atol=1e-12)
        np.testing.assert_allclose(dv, dv_a, atol=1e-12)
    for got, ref in [(O, O_ref), (L, L_ref), (dQ, dQ_ref), (dK, dK_ref), (dV, dV_ref)]:
        np.testing.assert_allclose(got, ref, atol=1e-12)


@pytest.mark.parametrize("T,N", [(8, 4), (48, 3), (64, 2)])
def test_packed_plan_covers_exactly_the_visible_pairs(T, N):
    """Brute force over every (query, key) token pair: the sub-blocks of the packed plan, with
    the document test applied, see each causal same-document pair of the rank's rows exactly once."""
    rng = np.random.default_rng(T + N)
    cuts = np.sort(rng.choice(np.arange(1, T), size=3, replace=False))
    cu = np.concatenate([[0], cuts, [T]]).astype(np.int32)
    doc = orc.doc_of(np.arange(T), cu)
    for r, pruned in [(r, p) for r in range(N) for p in (False, True)]:
        _, l2g = orc.zigzag_layout(T, N, r)
        count = np.zeros((len(l2g), T), dtype=np.int32)
        for s in range(N):
            src, blks = orc.zigzag_plan_packed(T, N, r, s, cu if pruned else None)
            _, src_rows = orc.zigzag_layout(T, N, src)
            assert len(blks) <= 3 and (pruned or len(blks) >= 2)
            for blk in blks:
                vis = orc.block_visibility(blk, cu)
                qs = np.arange(blk["q_row0"], blk["q_row0"] + blk["n_q"])
                ks = src_rows[blk["k_row0"]: blk["k_row0"] + blk["n_k"]]
                assert np.array_equal(l2g[qs], blk["q_pos0"] + np.arange(blk["n_q"]))     # positions are the global ones
                assert np.array_equal(ks, blk["k_pos0"] + np.arange(blk["n_k"]))
                count[np.ix_(qs, ks)] += vis
        want = (np.arange(T)[None, :] <= l2g[:, None]) & (doc[None, :] == doc[l2g][:, None])
        assert np.array_equal(count, want.astype(np.int32))


@pytest.mark.parametrize("with_docs", [True, False])
def test_packed_ring_emulation_reassembles_the_unsharded_result(with_docs):
    rng = np.random.default_rng(33)
    N, C, Hq, Hkv, d = 3, 4, 4, 2, 5
    T = 2 * N * C
    cu = np.array([0, 3, 4, 13, 19, T], dtype=np.int32) if with_docs else None
    Q, K, V, dO = _rand(rng, T, Hq, d), _rand(rng, T, Hkv, d), _rand(rng, T, Hkv, d), _rand(rng, T, Hq, d)
    scale = 1 / math.sqrt(d)
    O_ref, L_ref, dQ_ref, dK_ref, dV_ref = orc.causal_attention(Q, K, V, scale, cu_seqlens=cu, dO=dO)
    O = np.zeros_like(O_ref); L = np.zeros_like(L_ref); dQ = np.zeros_like(Q)
    dK = np.zeros_like(K); dV = np.zeros_like(V)
    for r in range(N):
        _, l2g = orc.zigzag_layout(T, N, r)
        o, l = orc.ring_rank_fwd_packed(Q, K, V, N, r, scale, cu)
        O[l2g], L[:, l2g] = o, l
        dq, dk, dv = orc.ring_rank_bwd_packed(Q, K, V, dO[l2g], o, l, N, r, scale, cu)
        dQ[l2g] = dq; dK += dk; dV += dv
        if not with_docs:                                  # without documents the packed plan is the plain one, regrouped
            o2, l2 = orc.ring_rank_fwd(Q, K, V, N, r, scale)
            np.testing.assert_allclose(o, o2, atol=1e-12); np.testing.assert_allclose(l, l2, atol=1e-12)
    for got, ref in [(O, O_ref), (L, L_ref), (dQ, dQ_ref), (dK, dK_ref), (dV, dV_ref)]:
        np.testing.assert_allclose(got, ref, atol=1e-12)


# ---------------------------------------------------------------- backward: finite differences
@pytest.mark.parametrize("cu", [None, [0, 3, 10, 14]])
def test_backward_matches_central_finite_differences(cu):
    rng = np.random.default_rng(11)
    T, Hq, Hkv, d = 14, 4, 2, 3
    Q, K, V, dO = _rand(rng, T, Hq, d), _rand(rng, T, Hkv, d), _rand(rng, T, Hkv, d), _rand(rng, T, Hq, d)
    scale = 0.45

    def f(q, k, v):
        return float((orc.causal_attention(q, k, v, scale, cu_seqlens=cu)[0] * dO).sum())

    _, _, dQ, dK, dV = orc.causal_attention(Q, K, V, scale, cu_seqlens=cu, dO=dO)
    eps = 1e-6
    for X, G, idx in [(Q, dQ, 0), (K, dK, 1), (V, dV, 2)]:
        num = np.zeros_like(X)
        it = np.nditer(X, flags=["multi_index"])
        for _ in it:
            mi = it.multi_index
            args = [Q.copy(), K.copy(), V.copy()]
            args[idx][mi] += eps
            fp = f(*args)
            args[idx][mi] -= 2 * eps
            fm = f(*args)
            num[mi] = (fp - fm) / (2 * eps)
        np.testing.assert_allclose(G, num, atol=2e-8)


# ---------------------------------------------------------------- GQA and varlen reductions
def test_gqa_equals_repeated_kv_heads():
    rng = np.random.default_rng(12)
    T, Hkv, g, d = 10, 2, 7, 4
    Q, K, V, dO = _rand(rng, T, Hkv * g, d), _rand(rng, T, Hkv, d), _rand(rng, T, Hkv, d), _rand(rng, T, Hkv * g, d)
    O, L, dQ, dK, dV = orc.causal_attention(Q, K, V, 0.5, dO=dO)
    Kr, Vr = np.repeat(K, g, axis=1), np.repeat(V, g, axis=1)
    O1, L1, dQ1, dK1, dV1 = orc.causal_attention(Q, Kr, Vr, 0.5, dO=dO)      # g = 1: plain MHA
    np.testing.assert_allclose(O, O1, atol=1e-14); np.testing.assert_allclose(L, L1, atol=1e-14)
    np.testing.assert_allclose(dQ, dQ1, atol=1e-14)
    np.testing.assert_allclose(dK, dK1.reshape(T, Hkv, g, d).sum(axis=2), atol=1e-13)
    np.testing.assert_allclose(dV, dV1.reshape(T, Hkv, g, d).sum(axis=2), atol=1e-13)


def test_packed_documents_equal_independent_calls():
    rng = np.random.default_rng(13)
    cu = [0, 7, 8, 20, 31]
    T, Hq, Hkv, d = cu[-1], 4, 2, 5
    Q, K, V, dO = _rand(rng, T, Hq, d), _rand(rng, T, Hkv, d), _rand(rng, T, Hkv, d), _rand(rng, T, Hq, d)
    got = orc.causal_attention(Q, K, V, 0.4, cu_seqlens=cu, dO=dO, row_block=6)
    for a, b in zip(cu[:-1], cu[1:]):
        ref = orc.causal_attention(Q[a:b], K[a:b], V[a:b], 0.4, dO=dO[a:b])
        np.testing.assert_allclose(got[0][a:b], ref[0], atol=1e-13)
        np.testing.assert_allclose(got[1][:, a:b], ref[1], atol=1e-13)
        for x, y in zip(got[2:], ref[2:]):
            np.testing.assert_allclose(x[a:b], y, atol=1e-13)


def test_row_blocking_does_not_change_the_result():
    rng = np.random.default_rng(14)
    T, H, d = 33, 2, 4
    Q, K, V, dO = _rand(rng, T, H, d), _rand(rng, T, H, d), _rand(rng, T, H, d), _rand(rng, T, H, d)
    a = orc.causal_attention(Q, K, V, 0.5, dO=dO, row_block=5)
    b = orc.causal_attention(Q, K, V, 0.5, dO=dO, row_block=1000)
    for x, y in zip(a, b):
        np.testing.assert_allclose(x, y, atol=1e-13)


def test_delta_is_rowwise_dot():
    rng = np.random.default_rng(15)
    dO, O = _rand(rng, 5, 3, 4), _rand(rng, 5, 3, 4)
    D = orc.delta(dO, O)
    for i in range(5):
        for h in range(3):
            assert abs(D[h, i] - sum(dO[i, h, c] * O[i, h, c] for c in range(4))) < 1e-14


# ---------------------------------------------------------------- data movement around attention
def test_zigzag_gather_matches_the_papers_example_and_inverts():
    """8 tokens / 4 ranks: shards are {0,7},{1,6},{2,5},{3,4} (the golden example); scatter inverts
    gather for any N, and gathering positions gives each rank's local_to_global map."""
    x = np.arange(8)
    rows = [[int(t0), int(t1)] for _, t0, t1, _ in _read_rows("zigzag_8_4.txt")]
    assert orc.zigzag_gather(x, 4).tolist() == rows
    rng = np.random.default_rng(3)
    for T, N in [(8, 4), (48, 3), (64, 1)]:
        x = rng.standard_normal((T, 3, 2))
        g = orc.zigzag_gather(x, N)
        assert g.shape == (N, T // N, 3, 2) and np.array_equal(orc.zigzag_scatter(g), x)
        pos = orc.zigzag_gather(np.arange(T), N)
        for r in range(N):
            assert np.array_equal(pos[r], orc.zigzag_layout(T, N, r)[1])


def test_a2a_head_packing_is_the_head_to_sequence_exchange():
    """Brute force: after packing on U GPUs, delivering message u of GPU g to GPU u and
    concatenating by source, GPU u holds head group u of the whole sequence; the return trip
    (messages per head group, unpack) restores the original token-sharded tensor."""
    rng = np.random.default_rng(4)
    U, t, H, d = 4, 5, 8, 3
    full = rng.standard_normal((U * t, H, d))
    local = [full[g * t:(g + 1) * t] for g in range(U)]                 # token-sharded, all heads
    packed = [orc.a2a_pack_heads(x, U) for x in local]
    for x, y in zip(local, packed):                                     # element by element
        for u in range(U):
            for i in range(t):
                assert np.array_equal(y[u, i], x[i, u * (H // U):(u + 1) * (H // U)])
    hh = H // U
    for u in range(U):
        recv = np.concatenate([packed[g][u] for g in range(U)])         # all-to-all: message u of every GPU, by source
        assert np.array_equal(recv, full[:, u * hh:(u + 1) * hh])
    for g in range(U):
        back = np.stack([full[g * t:(g + 1) * t, u * hh:(u + 1) * hh] for u in range(U)])   # one message per head group
        assert np.array_equal(orc.a2a_unpack_heads(back), local[g])


def test_positions_outside_every_document_see_nothing():
    """cu_seqlens that does not cover every position: a pair is visible only if one document
    [cu[k], cu[k+1]) holds both positions -- checked by plain loops over documents, for the
    causal and for the full mask kind, and through the attention result (rows outside every
    document come out empty: O = 0, LSE = -inf)."""
    cu = [3, 7, 8, 15]
    pos = np.arange(0, 20)
    def same_doc(a, b):
        return any(cu[k] <= a < cu[k + 1] and cu[k] <= b < cu[k + 1] for k in range(len(cu) - 1))
    want_causal = np.array([[b <= a and same_doc(a, b) for b in pos] for a in pos])
    want_full = np.array([[same_doc(a, b) for b in pos] for a in pos])
    assert np.array_equal(orc.visible(pos, pos, cu), want_causal)
    blk = dict(q_row0=0, n_q=20, k_row0=0, n_k=20, q_pos0=0, k_pos0=0, mask=orc.MASK_FULL)
    assert np.array_equal(orc.block_visibility(blk, cu), want_full)
    blk["mask"] = orc.MASK_CAUSAL_DIAG
    assert np.array_equal(orc.block_visibility(blk, cu), want_causal)
    assert orc.doc_of(pos, cu).tolist() == [-1] * 3 + [0] * 4 + [1] + [2] * 7 + [-1] * 5
    rng = np.random.default_rng(8)
    Q, K, V = _rand(rng, 20, 2, 4), _rand(rng, 20, 1, 4), _rand(rng, 20, 1, 4)
    O, L = orc.causal_attention(Q, K, V, 0.5, cu_seqlens=np.array(cu))[:2]
    outside = [0, 1, 2, 15, 16, 17, 18, 19]
    assert np.all(O[outside] == 0) and np.all(np.isneginf(L[:, outside]))
    assert np.all(np.isfinite(L[:, 3:15]))
