"""A deliberately literal, slow transcription of the paper's mask-estimation algorithm
(Alg. 1 with the block-wise changes of Sec. 3.2), used only to pin the oracle on tiny inputs.

It differs from the oracle in every implementation choice that should not matter:
1-based inclusive ranges (f, l) as in the paper, fixed arrays of kb nodes / 2*kb branches
that include EMPTY ranges (f > l), a score of -inf for an empty or fully masked branch,
exactly ceil(log2(Tb)) iterations whether or not they still change anything, exact
rational rounding, and arg-top-k by a full stable sort.  Ties go to the lower position.
"""
from fractions import Fraction
import math


def _round_half_up(x: Fraction) -> int:
    return math.floor(x + Fraction(1, 2))


def literal_mask_unit(score_fn, Tb: int, kb: int, rep_pos: int = 0):
    """score_fn(r) -> score of the 1-based key block r (max over the query block's rows and the
    block's keys of the admissible dot products; -inf if none).  Returns the sorted list of
    selected 1-based block numbers."""
    if Tb <= 0:
        return []
    nodes = []
    for j in range(1, kb + 1):
        f = _round_half_up(Fraction((j - 1) * Tb, kb)) + 1
        l = _round_half_up(Fraction(j * Tb, kb))
        nodes.append((f, l))
    n_it = math.ceil(math.log2(Tb)) if Tb > 1 else 0
    while 2 ** n_it < Tb:      # guard against floating point log2
        n_it += 1
    for _ in range(n_it):
        branches = []
        for (f, l) in nodes:
            m = _round_half_up(Fraction(f + l, 2))
            branches.append((f, m - 1))
            branches.append((m, l))
        scores = []
        for (f, l) in branches:
            if f > l:
                scores.append(-math.inf)
            else:
                r = f if rep_pos == 1 else l if rep_pos == 2 else _round_half_up(Fraction(f + l, 2))
                scores.append(score_fn(r))
        # an empty range (f > l) never displaces a real one, even one whose score is -inf because
        # stride sampling left it no admissible (row, key) pair
        order = sorted(range(len(branches)), key=lambda h: (-scores[h], branches[h][0] > branches[h][1], h))
        top = sorted(order[:kb])
        nodes = [branches[h] for h in top]
    out = sorted(f for (f, l) in nodes if f <= l)
    for (f, l) in nodes:
        assert f > l or f == l, "a node is still longer than one block after n_it iterations"
    return out
