"""An independent, slow restatement of the paper's mask estimation (Alg. 1 in the block form of Sec. 3.2) on
explicit SETS of key blocks, used only to pin the oracle on tiny inputs.  Nothing under oracle/ or the GPU
package imports it.

It differs from the oracle in every implementation choice that should not matter: groups are tuples of block
numbers rather than (start, end) ranges; bounds and midpoints come from exact rational arithmetic on the paper's
1-based inclusive numbering rather than from integer formulas; the search is a recursion of fixed depth
ceil(log2(Tb)) that carries EMPTY groups along (they rank below everything) rather than a loop that stops when
every group is a single block; and the best kb groups are taken from a full stable sort.
"""
from fractions import Fraction
import math

HALF = Fraction(1, 2)


def _nearest(x: Fraction) -> int:
    """Nearest integer, halves up."""
    return math.floor(x + HALF)


def _initial_groups(Tb: int, kb: int):
    """kb groups of consecutive blocks 0..Tb-1 whose boundaries are the rounded multiples of Tb/kb."""
    cuts = [_nearest(Fraction(j * Tb, kb)) for j in range(kb + 1)]
    return [tuple(range(cuts[j], cuts[j + 1])) for j in range(kb)]


def _halves(group):
    """Lower and upper part of a group, split at the rounded midpoint of its first and last block number
    (numbers counted from 1, both ends included, as the paper counts)."""
    if not group:
        return (), ()
    mid = _nearest(Fraction((group[0] + 1) + (group[-1] + 1), 2))
    return tuple(b for b in group if b + 1 < mid), tuple(b for b in group if b + 1 >= mid)


def _representative(group, rep_pos: int) -> int:
    """Block number (from 1) that stands for the group: its first, its last, or the rounded midpoint."""
    if rep_pos == 1:
        return group[0] + 1
    if rep_pos == 2:
        return group[-1] + 1
    return _nearest(Fraction((group[0] + 1) + (group[-1] + 1), 2))


def _refine(groups, depth: int, kb: int, score_fn, rep_pos: int, level: int = 0, adjust=None):
    if depth == 0:
        return groups
    parts = [h for g in groups for h in _halves(g)]
    score = [score_fn(_representative(h, rep_pos)) if h else -math.inf for h in parts]
    if adjust is not None:
        # what the selection of this level compares (an ensemble sample moves the scores of one level)
        score = [adjust(level, _representative(h, rep_pos), sc) if h else sc for h, sc in zip(parts, score)]
    # best first; a real group outranks an empty one even when stride sampling left it no admissible
    # (row, key) pair and its score is -inf too; equal scores: the part that comes first (lower position)
    ranked = sorted(range(len(parts)), key=lambda i: (-score[i], not parts[i], i))
    kept = sorted(ranked[:kb])
    return _refine([parts[i] for i in kept], depth - 1, kb, score_fn, rep_pos, level + 1, adjust)


def levels_that_split(Tb: int, kb: int) -> int:
    """Levels at which some group can still hold more than one block: the longest initial group halves, rounding
    up, until it is a single block."""
    longest = max((len(g) for g in _initial_groups(Tb, kb)), default=0)
    n = 0
    while longest > 1:
        longest = -(-longest // 2)
        n += 1
    return n


def set_search_mask_unit(score_fn, Tb: int, kb: int, rep_pos: int = 0, adjust=None):
    """score_fn(r) -> score of key block number r, counted from 1 (max over the query block's rows and the block's
    keys of the admissible dot products; -inf if none); adjust(level, r, score) -> the score the selection of that
    level (0 = first) compares, if given.  Returns the sorted block numbers (from 1) selected."""
    if Tb <= 0:
        return []
    depth = 0
    while 2 ** depth < Tb:
        depth += 1
    final = _refine(_initial_groups(Tb, kb), depth, kb, score_fn, rep_pos, 0, adjust)
    assert all(len(g) <= 1 for g in final), "a group still holds several blocks after ceil(log2(Tb)) levels"
    return sorted(g[0] + 1 for g in final if g)
