"""CPU oracle for the reachable-only index.  TEST INFRASTRUCTURE ONLY (tests, smoke check,
benchmark's CPU leg); plain numpy and Python loops, nothing shared with the GPU path.

Paper, Section 3, the paragraph after Algorithm 4: the index needs memory for every state of the
automaton in principle, but in practice not every state is ever represented by a vocabulary string.
Section 2.2, Algorithm 2: generation starts in q_0 and moves, token by token, to the end state the
index stores with the sampled token.  So the states a generation can ever be in are exactly those
that are reachable from q_0 through vocabulary tokens, and only their rows are ever read.

``reachable_states``  The least set R of states with  starts in R  and  q in R, (v, s) in sigma(q)
    implies s in R:  the states some sequence of vocabulary tokens leads to from a start state.

``restrict_rows``  The index with the rows of the states outside a given set left empty.  State ids
    keep their meaning (rows are still addressed by state id), the kept rows are unchanged, the
    entries are stored side by side in state order.
"""
from __future__ import annotations

import numpy as np


def reachable_states(row_ptr, next_states, starts):
    """Returns reach [Q] uint8 (1: reachable from one of `starts` through rows of the index)."""
    n_states = row_ptr.size - 1
    reach = np.zeros(n_states, dtype=np.uint8)
    todo = []
    for s in starts:
        s = int(s)
        if s < 0 or s >= n_states:
            raise ValueError(f"start state {s} outside [0, {n_states})")
        if not reach[s]:
            reach[s] = 1
            todo.append(s)
    while todo:
        q = todo.pop()
        a, b = int(row_ptr[q]), int(row_ptr[q + 1])
        for s in np.unique(next_states[a:b]):
            s = int(s)
            if not reach[s]:
                reach[s] = 1
                todo.append(s)
    return reach


def restrict_rows(row_ptr, token_ids, next_states, keep):
    """Returns (row_ptr' [Q + 1] int64, token_ids', next_states'): rows q with keep[q] == 0 empty."""
    n_states = row_ptr.size - 1
    new_ptr = np.zeros(n_states + 1, dtype=np.int64)
    for q in range(n_states):
        length = int(row_ptr[q + 1] - row_ptr[q]) if keep[q] else 0
        new_ptr[q + 1] = new_ptr[q] + length
    tok = np.zeros(int(new_ptr[-1]), dtype=np.int32)
    nxt = np.zeros(int(new_ptr[-1]), dtype=np.int32)
    for q in range(n_states):
        if keep[q]:
            a, b = int(row_ptr[q]), int(row_ptr[q + 1])
            tok[new_ptr[q]:new_ptr[q + 1]] = token_ids[a:b]
            nxt[new_ptr[q]:new_ptr[q + 1]] = next_states[a:b]
    return new_ptr, tok, nxt
