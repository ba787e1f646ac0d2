"""CPU oracle for the offline phase: hierarchical block extraction -- TEST INFRASTRUCTURE.

Only tests may import this module.  It shares no code with the library's encoder (csrc/encoder.cpp): it works on
Python sets, follows the steps of the paper's Algorithm 1 (hierarchical block extraction: multi-level aggregation
around multi-round extraction) and Algorithm 2 (greedy row matching) in the paper's order and notation, and applies
the rules of Sections 6.2 / 6.3.1 that bound what may be extracted.

The method is a greedy heuristic, so this oracle is "the algorithm's steps", not a closed form.  Where the paper
leaves a choice open, the reading taken is stated at the place it is used:

  * pop() of Algorithm 2 returns the remaining row with the most columns (ties: lower index);
  * argmax breaks ties towards the lower index; similarity = number of shared columns (Section 4.3's matching text);
  * a pair is formed only if it shares at least one unit (`unit` columns); otherwise the popped row stays single;
  * extractBlock keeps units of `unit` consecutive shared columns whose successive gaps are <= `max_delta`
    (Section 6.2: only adjacent columns within the delta range; Section 6.3.1: whole load quanta only);
  * leftover columns of a level >= 1 row that no longer form a unit fall back to the two rows it was made from.

Pins (tests/test_extraction_oracle.py): block sets derived by hand for constructed matrices (a row split between two
partners over two rounds as in the paper's Section 4.3 narrative, identical rows climbing every level, leftovers
below a unit, a gap wider than the delta range, tie-breaking, and leftovers of a block lifted to 8 rows that fall back
two levels and complete a unit there), the worked example the paper prints (tests/golden/), and the partition
invariant.  The library is also checked without this module (tests/test_extraction_invariants.py: the rules every
block set obeys, and greedy matching against a brute-force search over all matchings).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Set, Tuple


@dataclass
class LevelRow:
    """One row of a level matrix A_E / A_R: at level l it stands for 2^l original rows (`members`); a column in
    `cols` means every member row has a stored entry there (Section 4.2)."""
    cols: Set[int]
    members: Tuple[int, ...]
    children: Optional[Tuple[int, int]] = None     # indices of the two rows of the level below it came from


def form_units(cols: Sequence[int], unit: int, max_delta: int) -> Tuple[List[int], List[int]]:
    """Cut sorted columns into runs of `unit` columns with all successive gaps <= max_delta.
    Returns (columns taken, in order, a multiple of `unit`; columns left)."""
    taken: List[int] = []
    rest: List[int] = []
    run: List[int] = []
    for c in cols:
        if run and c - run[-1] > max_delta:
            rest.extend(run)                # the run cannot be completed: its columns stay
            run = []
        run.append(c)
        if len(run) == unit:
            taken.extend(run)
            run = []
    rest.extend(run)
    return taken, rest


def row_matching(A: List[LevelRow], unit: int) -> List[Tuple[int, int]]:
    """Algorithm 2.  W = similarity (shared column counts); rows are popped and matched greedily."""
    unselected = [i for i in range(len(A)) if len(A[i].cols) >= unit]   # a row below one unit can form no block
    pairs: List[Tuple[int, int]] = []
    while unselected:
        row = min(unselected, key=lambda i: (-len(A[i].cols), i))        # pop(): most columns, then lower index
        unselected.remove(row)
        best, best_sim = None, 0
        for cand in sorted(unselected):                                   # argmax, ties -> lower index
            sim = len(A[row].cols & A[cand].cols)
            if sim > best_sim:
                best, best_sim = cand, sim
        if best is not None and best_sim >= unit:
            pairs.append((row, best))
            unselected.remove(best)
    return pairs


def hierarchical_block_extraction(rows: Sequence[Set[int]], max_granularity: int = 8, unit: int = 64,
                                  max_delta: int = 255, max_rounds: int = 64):
    """Algorithm 1 on one group of rows (a panel, or the whole matrix).

    rows: the column set of every row of A.  Returns (block_sets, residual):
      block_sets[g] = list of units (member rows tuple, tuple of `unit` columns) for g = 2, 4, ...
      residual[i]   = sorted columns of row i left at granularity 1."""
    levels: List[List[LevelRow]] = [[LevelRow(set(c), (i,)) for i, c in enumerate(rows)]]   # A_E = A
    level = 0
    while (2 << level) <= max_granularity:                    # multi-level aggregation
        A_R = levels[level]                                   # A_R = A_E
        extracted_blocks: List[LevelRow] = []
        for _ in range(max_rounds):                           # multi-round extraction
            row_pairs = row_matching(A_R, unit)
            blocks_R: List[LevelRow] = []
            for a, b in row_pairs:                            # extractBlock
                taken, _ = form_units(sorted(A_R[a].cols & A_R[b].cols), unit, max_delta)
                if not taken:
                    continue
                A_R[a].cols -= set(taken)                     # extracted entries are set to zero
                A_R[b].cols -= set(taken)
                blocks_R.append(LevelRow(set(taken), A_R[a].members + A_R[b].members, (a, b)))
            if not blocks_R:
                break
            extracted_blocks.extend(blocks_R)
        if not extracted_blocks:
            break
        levels.append(extracted_blocks)                       # A_E = encode(extracted_blocks)
        level += 1

    # decode(A, A_R): what is left at each level becomes blocks of that level's granularity, coarsest first
    block_sets: Dict[int, List[Tuple[Tuple[int, ...], Tuple[int, ...]]]] = {}
    for lv in range(len(levels) - 1, 0, -1):
        g = 1 << lv
        for r in levels[lv]:
            taken, rest = form_units(sorted(r.cols), unit, max_delta)
            for c in rest:                                    # no longer a unit: back to the two parent rows
                levels[lv - 1][r.children[0]].cols.add(c)
                levels[lv - 1][r.children[1]].cols.add(c)
            for u in range(0, len(taken), unit):
                block_sets.setdefault(g, []).append((r.members, tuple(taken[u:u + unit])))
    residual = [sorted(r.cols) for r in levels[0]]
    return block_sets, residual
