"""Work counts that the benchmark reports: visible (query, key) pairs and the floating-point
operations credited for them.  Pure integer arithmetic, no device code.

Convention.  One multiply-accumulate = 2 flops.  Per visible pair and query head the forward
has two products of inner length d (S = Q K^T and O = P V): 4 d flops.  The backward is
credited with five (S and dP recomputed once, dV, dK, dQ): 10 d flops, whatever a kernel
really executes.  The appendix table "Detailed model complexity analysis" of the paper counts
the attention of a whole model as T^2 d H L, i.e. one operation per multiply-accumulate over
the T^2 / 2 causal pairs and the two forward products; twice that table's entry is this
module's forward count for L layers (up to the T / 2 pairs of the diagonal, which the table
leaves out)."""

FWD_FLOPS_PER_PAIR_PER_D = 4
BWD_FLOPS_PER_PAIR_PER_D = 10


def causal_pairs(T):
    """Visible pairs per head of a causal sequence of T tokens, diagonal included."""
    return T * (T + 1) // 2


def zigzag_pairs_of_rank(N, C):
    """Visible pairs per head of any rank of the both-ends (zigzag) layout, T = 2 N C: the rank
    holds chunks r and 2N-1-r, whose rows see r C + ... keys; the sum is 2 N C^2 + C for every r."""
    return 2 * N * C * C + C


def contiguous_pairs_of_rank(N, C, rank):
    """Visible pairs per head of rank `rank` when it holds the contiguous rows [2 C rank, 2 C (rank + 1))."""
    n = 2 * C
    return rank * n * n + n * (n + 1) // 2


def packed_pairs(doc_lengths):
    """Visible pairs per head of a packed sequence under the document-causal mask."""
    return sum(int(t) * (int(t) + 1) // 2 for t in doc_lengths)


def attention_flops(pairs, d, n_q_heads, forward=True, backward=True):
    """Flops credited for `pairs` visible pairs per head."""
    per_pair = (FWD_FLOPS_PER_PAIR_PER_D if forward else 0) + (BWD_FLOPS_PER_PAIR_PER_D if backward else 0)
    return per_pair * d * n_q_heads * pairs


def paper_table_tflops(T, d, n_heads, n_layers):
    """The appendix table's attention entry for a model: T^2 d H L operations, in units of 1e12."""
    return T * T * d * n_heads * n_layers / 1e12
