"""fp64 CPU oracle for one rank's attention under MM-SP (zigzag ring / Ulysses head shard).

TEST INFRASTRUCTURE ONLY.  Nothing on the product path may import this module; it
exists so that tests, the smoke check and the benchmark's cpu_baseline leg can
compare the HIP kernels with a plain, slow, obviously correct computation.  It shares
no code with the HIP path and never calls it.

The paper (Sec. 4.2, "MM-SP workflow"; Fig. "Comparison of RingAttention, ZigZag and
2D-Attention"; Fig. "Convergence evaluation") describes the system in prose and states
that sequence-parallel training reproduces the unsharded result, so the quantity being
computed has a plain definition -- causal softmax attention with grouped KV heads and an
optional packed-document mask -- and path A below is that definition written out.
Path B walks the method's own steps (per-ring-step partial attention, log-sum-exp merge,
per-step backward) so the two can be checked against each other.

Conventions that the paper leaves open are the readings listed in the design doc:
  * softmax scale is passed in (callers use 1/sqrt(d));
  * LSE is the natural log of the sum of exp of the scaled scores;
  * the diagonal is visible (key position <= query position);
  * a row that sees nothing has O = 0 and LSE = -inf;
  * query head h reads KV head h // (Hq // Hkv);
  * rank r of N holds chunks r and 2N-1-r of 2N equal chunks, in ascending order.

All arrays are numpy float64.  Shapes: Q [nq, Hq, d], K/V [nk, Hkv, d], O like Q,
LSE [Hq, nq].  Positions are integer arrays giving each row's index in the full packed
sequence; `cu_seqlens` (ascending, [n_docs + 1]) delimits documents [cu[k], cu[k+1]); a
position below cu[0] or from cu[n_docs] on belongs to no document and sees nothing.
"""
import numpy as np

NEG_INF = -np.inf

MASK_FULL = 0         # every query row of the block sees every key row of the block
MASK_CAUSAL_DIAG = 1  # key visible iff k_pos <= q_pos (and same document)
MASK_NONE = 2         # nothing visible


# --------------------------------------------------------------------------------------
# visibility (Sec. 4.2: causal attention; packed variable-length inputs, Sec. 4.1 end)
# --------------------------------------------------------------------------------------
def doc_of(pos, cu_seqlens):
    """Index of the document (interval [cu[k], cu[k+1])) that holds each position; -1 for a
    position below cu[0] or from cu[-1] on, which belongs to no document."""
    pos = np.asarray(pos, dtype=np.int64)
    if cu_seqlens is None:
        return np.zeros_like(pos)
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    doc = np.searchsorted(cu, pos, side="right") - 1
    return np.where(pos >= cu[-1], -1, doc)


def visible(q_pos, k_pos, cu_seqlens=None):
    """Boolean [nq, nk]: key j is visible to query i iff k_pos[j] <= q_pos[i] and both
    lie in the same document (a position outside every document sees nothing and is seen
    by nothing)."""
    q_pos = np.asarray(q_pos, dtype=np.int64)
    k_pos = np.asarray(k_pos, dtype=np.int64)
    vis = k_pos[None, :] <= q_pos[:, None]
    if cu_seqlens is not None:
        qd, kd = doc_of(q_pos, cu_seqlens), doc_of(k_pos, cu_seqlens)
        vis &= (qd[:, None] == kd[None, :]) & (qd[:, None] >= 0)
    return vis


# --------------------------------------------------------------------------------------
# Path A: the plain definition
# --------------------------------------------------------------------------------------
def _masked_forward_one_head(q, k, v, vis, scale):
    """q [nq,d], k,v [nk,d], vis bool [nq,nk] -> (O [nq,d], LSE [nq], P [nq,nk])."""
    s = scale * (q @ k.T)
    s = np.where(vis, s, NEG_INF)
    m = s.max(axis=1) if s.shape[1] else np.full(s.shape[0], NEG_INF)
    m_safe = np.where(np.isfinite(m), m, 0.0)
    e = np.exp(s - m_safe[:, None])            # exp(-inf) = 0 for hidden keys
    l = e.sum(axis=1)
    with np.errstate(divide="ignore"):
        lse = np.where(l > 0, m_safe + np.log(l), NEG_INF)
    p = np.where(l[:, None] > 0, e / np.where(l > 0, l, 1.0)[:, None], 0.0)
    return p @ v, lse, p


def attention_fwd(Q, K, V, vis, scale):
    """Softmax attention under an explicit visibility matrix.

    S_h = scale * Q_h K_kv(h)^T; LSE_h[i] = ln sum_{j visible} exp S_h[i,j];
    O[i,h] = sum_j exp(S_h[i,j] - LSE_h[i]) V[j,kv(h)].
    """
    nq, Hq, d = Q.shape
    Hkv = K.shape[1]
    g = Hq // Hkv
    O = np.zeros((nq, Hq, V.shape[2]))
    LSE = np.full((Hq, nq), NEG_INF)
    for h in range(Hq):
        O[:, h], LSE[h], _ = _masked_forward_one_head(Q[:, h], K[:, h // g], V[:, h // g], vis, scale)
    return O, LSE


def attention_bwd(Q, K, V, dO, vis, scale, LSE=None, D=None):
    """Gradients of sum(O * dO) for the query rows given, by the chain rule of softmax:

      P = exp(S - LSE);  D[i] = sum_c dO[i,c] O[i,c];
      dV[j] = sum_i P[i,j] dO[i];  dS = P * (dO V^T - D);
      dQ[i] = scale sum_j dS[i,j] K[j];  dK[j] = scale sum_i dS[i,j] Q[i].

    dK/dV are these query rows' contribution for every key row given, summed over the
    query heads of each KV group.  When LSE and D are passed (path B: a block of a larger
    problem) they are used as given; otherwise they come from this call's own forward.
    """
    nq, Hq, d = Q.shape
    Hkv = K.shape[1]
    g = Hq // Hkv
    dQ = np.zeros_like(Q)
    dK = np.zeros_like(K)
    dV = np.zeros_like(V)
    for h in range(Hq):
        kh = h // g
        q, k, v, do = Q[:, h], K[:, kh], V[:, kh], dO[:, h]
        if LSE is None:
            o, lse, p = _masked_forward_one_head(q, k, v, vis, scale)
            dvec = (do * o).sum(axis=1)
        else:
            lse = LSE[h]
            s = scale * (q @ k.T)
            lse_safe = np.where(np.isfinite(lse), lse, 0.0)
            p = np.where(vis & np.isfinite(lse)[:, None], np.exp(np.where(vis, s, NEG_INF) - lse_safe[:, None]), 0.0)
            dvec = D[h]
        dV[:, kh] += p.T @ do
        ds = p * (do @ v.T - dvec[:, None])
        dQ[:, h] = scale * (ds @ k)
        dK[:, kh] += scale * (ds.T @ q)
    return dQ, dK, dV


def causal_attention(Q, K, V, scale, cu_seqlens=None, q_pos=None, dO=None, row_block=1024):
    """Path A entry point: causal (optionally document-causal) attention of the query rows
    at positions `q_pos` (default: all positions) against the whole sequence K, V.

    Each query row is independent by definition, so rows are taken `row_block` at a time
    only to bound the size of the score matrix; dK/dV sum over rows.
    Returns (O, LSE) or, with dO, (O, LSE, dQ, dK, dV).
    """
    T = K.shape[0]
    k_pos = np.arange(T, dtype=np.int64)
    q_pos = k_pos if q_pos is None else np.asarray(q_pos, dtype=np.int64)
    nq, Hq, d = Q.shape
    O = np.zeros((nq, Hq, V.shape[2]))
    LSE = np.full((Hq, nq), NEG_INF)
    if dO is not None:
        dQ, dK, dV = np.zeros_like(Q), np.zeros_like(K), np.zeros_like(V)
    for a in range(0, nq, row_block):
        b = min(a + row_block, nq)
        # keys after the last query of the block are hidden from every row in it
        kmax = int(q_pos[a:b].max()) + 1 if b > a else 0
        vis = visible(q_pos[a:b], k_pos[:kmax], cu_seqlens)
        O[a:b], LSE[:, a:b] = attention_fwd(Q[a:b], K[:kmax], V[:kmax], vis, scale)
        if dO is not None:
            dq, dk, dv = attention_bwd(Q[a:b], K[:kmax], V[:kmax], dO[a:b], vis, scale)
            dQ[a:b] = dq
            dK[:kmax] += dk
            dV[:kmax] += dv
    if dO is None:
        return O, LSE
    return O, LSE, dQ, dK, dV


# --------------------------------------------------------------------------------------
# Zigzag ("both ends") layout and the ring plan (Sec. 4.2 "MM-SP workflow"; the
# 8-token / 4-rank example in Fig. "Comparison of RingAttention, ZigZag, 2D-Attention")
# --------------------------------------------------------------------------------------
def zigzag_layout(T, N, rank):
    """Rank `rank` of N holds chunk `rank` and chunk 2N-1-rank of 2N equal chunks.
    Returns (chunk_ids (2,), local_to_global int64 [T/N])."""
    if T % (2 * N) != 0 or not (0 <= rank < N):
        raise ValueError("T must divide by 2N and 0 <= rank < N")
    C = T // (2 * N)
    c0, c1 = rank, 2 * N - 1 - rank
    l2g = np.concatenate([np.arange(c0 * C, (c0 + 1) * C), np.arange(c1 * C, (c1 + 1) * C)]).astype(np.int64)
    return np.array([c0, c1], dtype=np.int32), l2g


def two_d_share(T, U, R, gpu, Hq, Hkv):
    """One GPU's share under 2D-attention (Sec. 4.2, the U x R mesh; the comparison figure's
    2D-Attention row): the all-to-all group is U consecutive GPUs and splits the heads, the
    ring group of R splits the sequence by the zigzag rule.  GPU g = r*U + u gets query
    heads [u*Hq/U, (u+1)*Hq/U), the KV heads those query heads read (head h reads KV head
    h // (Hq/Hkv)), and the two chunks of ring rank r.
    Returns dict(u, r, q_heads (array), kv_heads (array), chunk_ids, l2g)."""
    if not (0 <= gpu < U * R) or Hq % U or Hq % Hkv or (Hkv % U and U % Hkv):
        raise ValueError("invalid 2D mesh for these heads")
    u, r = gpu % U, gpu // U
    q_heads = np.arange(u * (Hq // U), (u + 1) * (Hq // U))
    kv_heads = np.unique(q_heads // (Hq // Hkv))
    chunk_ids, l2g = zigzag_layout(T, R, r)
    return dict(u=u, r=r, q_heads=q_heads, kv_heads=kv_heads, chunk_ids=chunk_ids, l2g=l2g)


def zigzag_plan(T, N, rank, step):
    """Which KV block visits rank `rank` at ring step `step`, and which (query rows, key
    rows, mask) sub-block of it holds every visible pair.

    Derived from the chunk order alone: with local rows = [chunk r | chunk 2N-1-r],
      * own block (src == r): local causal -- chunk r precedes chunk 2N-1-r, order kept;
      * src < r: chunk src precedes both local chunks, chunk 2N-1-src follows both
        -> all query rows x first half of the key rows, everything visible;
      * src > r: chunk src and chunk 2N-1-src both lie between the local chunks
        -> second half of the query rows x all key rows, everything visible.
    """
    C = T // (2 * N)
    src = (rank - step) % N
    if src == rank:
        return dict(src=src, q_row0=0, n_q=2 * C, k_row0=0, n_k=2 * C, q_pos0=0, k_pos0=0, mask=MASK_CAUSAL_DIAG)
    if src < rank:
        return dict(src=src, q_row0=0, n_q=2 * C, k_row0=0, n_k=C, q_pos0=0, k_pos0=0, mask=MASK_FULL)
    return dict(src=src, q_row0=C, n_q=C, k_row0=0, n_k=2 * C, q_pos0=0, k_pos0=0, mask=MASK_FULL)


def zigzag_gather(x, N):
    """[T, ...] in sequence order -> [N, 2C, ...]: every rank's local rows (chunk r | chunk 2N-1-r)."""
    T = x.shape[0]
    return np.stack([x[zigzag_layout(T, N, r)[1]] for r in range(N)])


def zigzag_scatter(shards):
    """Inverse of zigzag_gather."""
    N, n = shards.shape[0], shards.shape[1]
    out = np.empty((N * n, *shards.shape[2:]), dtype=shards.dtype)
    for r in range(N):
        out[zigzag_layout(N * n, N, r)[1]] = shards[r]
    return out


def a2a_pack_heads(x, U):
    """[tokens, H, d] -> [U, tokens, H/U, d]: message u holds head group u of every local token."""
    t, H, d = x.shape
    return np.ascontiguousarray(x.reshape(t, U, H // U, d).transpose(1, 0, 2, 3))


def a2a_unpack_heads(y):
    """[U, tokens, H/U, d] (one message per head group) -> [tokens, H, d]."""
    U, t, hh, d = y.shape
    return np.ascontiguousarray(y.transpose(1, 0, 2, 3)).reshape(t, U * hh, d)


def contiguous_plan(T, N, rank, step):
    """Plain RingAttention layout (the comparison figure's first row): rank r holds the
    contiguous chunk r of N; at step `step` the block of rank src = (r - step) mod N visits.
    Own block: causal; src < r: everything visible; src > r: nothing (the rank idles)."""
    L = T // N
    src = (rank - step) % N
    mask = MASK_CAUSAL_DIAG if src == rank else (MASK_FULL if src < rank else MASK_NONE)
    return dict(src=src, q_row0=0, n_q=L, k_row0=0, n_k=L, q_pos0=0, k_pos0=0, mask=mask)


def zigzag_plan_packed(T, N, rank, step, cu_seqlens=None):
    """Ring step `step` of rank `rank` for a packed sequence (document mask from cu_seqlens on
    global positions): the local rows are two segments with positions chunk_r*C.. and
    chunk_(2N-1-r)*C.., the visiting block likewise, so the step is cut into sub-blocks of one
    query segment x one key segment, inside which positions are consecutive.  A (query chunk a,
    key chunk b) pair holds visible pairs only if b <= a; it is emitted as a causal-diagonal
    block on global positions (for b < a every pair passes the causal test and only the
    document test remains).  With cu_seqlens, segment pairs without any same-document
    (query, key) pair are left out.  Returns (src, [blk, ...])."""
    C = T // (2 * N)
    src = (rank - step) % N
    q_chunks = (rank, 2 * N - 1 - rank)
    k_chunks = (src, 2 * N - 1 - src)
    blks = []
    for qi, a in enumerate(q_chunks):
        for ki, b in enumerate(k_chunks):
            if b <= a:
                if cu_seqlens is not None and b < a and not np.any(
                        visible(np.arange(a * C, (a + 1) * C), np.arange(b * C, (b + 1) * C), cu_seqlens)):
                    continue
                blks.append(dict(src=src, q_row0=qi * C, n_q=C, k_row0=ki * C, n_k=C, q_pos0=a * C, k_pos0=b * C,
                                 mask=MASK_CAUSAL_DIAG))
    return src, blks


def causal_pairs_of_rank(T, N, rank):
    """Exact number of visible (query, key) pairs for one query head of one rank."""
    _, l2g = zigzag_layout(T, N, rank)
    return int((l2g + 1).sum())


# --------------------------------------------------------------------------------------
# Path B: the method's own steps, still fp64 and still by the definition per block
# --------------------------------------------------------------------------------------
def block_visibility(blk, cu_seqlens=None):
    """Visibility matrix of one step's sub-block from its mask kind."""
    nq, nk = blk["n_q"], blk["n_k"]
    if blk["mask"] == MASK_NONE:
        return np.zeros((nq, nk), dtype=bool)
    q_pos = blk["q_pos0"] + np.arange(nq, dtype=np.int64)
    k_pos = blk["k_pos0"] + np.arange(nk, dtype=np.int64)
    if blk["mask"] == MASK_FULL:
        vis = np.ones((nq, nk), dtype=bool)
        if cu_seqlens is not None:
            qd, kd = doc_of(q_pos, cu_seqlens), doc_of(k_pos, cu_seqlens)
            vis &= (qd[:, None] == kd[None, :]) & (qd[:, None] >= 0)
        return vis
    return visible(q_pos, k_pos, cu_seqlens)


def step_fwd(Q_local, K_blk, V_blk, blk, scale, cu_seqlens=None):
    """One ring step: partial O and LSE of the block's query rows against its key rows.
    Returns (O_part [n_q,Hq,d], LSE_part [Hq,n_q]) for rows q_row0 .. q_row0+n_q."""
    q = Q_local[blk["q_row0"]: blk["q_row0"] + blk["n_q"]]
    k = K_blk[blk["k_row0"]: blk["k_row0"] + blk["n_k"]]
    v = V_blk[blk["k_row0"]: blk["k_row0"] + blk["n_k"]]
    return attention_fwd(q, k, v, block_visibility(blk, cu_seqlens), scale)


def merge(O, L, O_p, L_p):
    """Combine two partial results over disjoint key sets:
    L' = ln(e^L + e^Lp);  O' = e^(L-L') O + e^(Lp-L') Op;  a side with L = -inf adds nothing.
    O [n,Hq,d], L [Hq,n]."""
    m = np.maximum(L, L_p)
    m_safe = np.where(np.isfinite(m), m, 0.0)
    a = np.exp(L - m_safe)
    b = np.exp(L_p - m_safe)
    tot = a + b
    with np.errstate(divide="ignore"):
        L_new = np.where(tot > 0, m_safe + np.log(tot), NEG_INF)
    tot_safe = np.where(tot > 0, tot, 1.0)
    wa = (a / tot_safe).T[:, :, None]
    wb = (b / tot_safe).T[:, :, None]
    return wa * O + wb * O_p, L_new


def ring_rank_fwd(Q, K, V, N, rank, scale):
    """Forward of one virtual rank over N ring steps.  Q/K/V are the full sequence
    [T,H,d]; returns (O_local [2C,Hq,d], LSE_local [Hq,2C])."""
    T = Q.shape[0]
    _, l2g = zigzag_layout(T, N, rank)
    Ql = Q[l2g]
    Hq, dv = Q.shape[1], V.shape[2]
    O = np.zeros((len(l2g), Hq, dv))
    L = np.full((Hq, len(l2g)), NEG_INF)
    for s in range(N):
        blk = zigzag_plan(T, N, rank, s)
        _, src_rows = zigzag_layout(T, N, blk["src"])
        O_p, L_p = step_fwd(Ql, K[src_rows], V[src_rows], blk, scale)
        r0, r1 = blk["q_row0"], blk["q_row0"] + blk["n_q"]
        O[r0:r1], L[:, r0:r1] = merge(O[r0:r1], L[:, r0:r1], O_p, L_p)
    return O, L


def delta(dO, O):
    """D[h,i] = sum_c dO[i,h,c] O[i,h,c] with the final merged O."""
    return np.einsum("ihc,ihc->hi", dO, O)


def step_bwd(Q_local, K_blk, V_blk, dO_local, LSE_final, D, blk, scale, cu_seqlens=None):
    """One ring step of the backward, using the completed forward's LSE and D.
    Returns (dQ_part [n_q,Hq,d] for the block's query rows, dK, dV [n_k,Hkv,d] for its key rows)."""
    r0, r1 = blk["q_row0"], blk["q_row0"] + blk["n_q"]
    k0, k1 = blk["k_row0"], blk["k_row0"] + blk["n_k"]
    return attention_bwd(Q_local[r0:r1], K_blk[k0:k1], V_blk[k0:k1], dO_local[r0:r1],
                         block_visibility(blk, cu_seqlens), scale,
                         LSE=LSE_final[:, r0:r1], D=D[:, r0:r1])


def ring_rank_bwd(Q, K, V, dO_local, O_local, LSE_local, N, rank, scale):
    """Backward of one virtual rank: dQ for its 2C rows, and its contribution to dK/dV for
    all T key rows (zero where none of its queries can see the key)."""
    T = Q.shape[0]
    _, l2g = zigzag_layout(T, N, rank)
    Ql = Q[l2g]
    D = delta(dO_local, O_local)
    dQ = np.zeros_like(Ql)
    dK = np.zeros_like(K)
    dV = np.zeros_like(V)
    for s in range(N):
        blk = zigzag_plan(T, N, rank, s)
        _, src_rows = zigzag_layout(T, N, blk["src"])
        dq, dk, dv = step_bwd(Ql, K[src_rows], V[src_rows], dO_local, LSE_local, D, blk, scale)
        r0 = blk["q_row0"]
        dQ[r0:r0 + blk["n_q"]] += dq
        rows = src_rows[blk["k_row0"]: blk["k_row0"] + blk["n_k"]]
        dK[rows] += dk
        dV[rows] += dv
    return dQ, dK, dV


def ring_rank_fwd_packed(Q, K, V, N, rank, scale, cu_seqlens):
    """ring_rank_fwd for a packed sequence: the sub-blocks of zigzag_plan_packed, merged."""
    T = Q.shape[0]
    _, l2g = zigzag_layout(T, N, rank)
    Ql = Q[l2g]
    O = np.zeros((len(l2g), Q.shape[1], V.shape[2]))
    L = np.full((Q.shape[1], len(l2g)), NEG_INF)
    for s in range(N):
        src, blks = zigzag_plan_packed(T, N, rank, s)
        _, src_rows = zigzag_layout(T, N, src)
        for blk in blks:
            O_p, L_p = step_fwd(Ql, K[src_rows], V[src_rows], blk, scale, cu_seqlens)
            r0, r1 = blk["q_row0"], blk["q_row0"] + blk["n_q"]
            O[r0:r1], L[:, r0:r1] = merge(O[r0:r1], L[:, r0:r1], O_p, L_p)
    return O, L


def ring_rank_bwd_packed(Q, K, V, dO_local, O_local, LSE_local, N, rank, scale, cu_seqlens):
    """ring_rank_bwd for a packed sequence."""
    T = Q.shape[0]
    _, l2g = zigzag_layout(T, N, rank)
    Ql = Q[l2g]
    D = delta(dO_local, O_local)
    dQ, dK, dV = np.zeros_like(Ql), np.zeros_like(K), np.zeros_like(V)
    for s in range(N):
        src, blks = zigzag_plan_packed(T, N, rank, s)
        _, src_rows = zigzag_layout(T, N, src)
        for blk in blks:
            dq, dk, dv = step_bwd(Ql, K[src_rows], V[src_rows], dO_local, LSE_local, D, blk, scale, cu_seqlens)
            dQ[blk["q_row0"]: blk["q_row0"] + blk["n_q"]] += dq
            rows = src_rows[blk["k_row0"]: blk["k_row0"] + blk["n_k"]]
            dK[rows] += dk
            dV[rows] += dv
    return dQ, dK, dV
