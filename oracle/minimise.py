"""CPU oracle for automaton minimisation before indexing.  TEST INFRASTRUCTURE ONLY (tests, smoke
check, benchmark's CPU leg); plain numpy and Python loops, nothing shared with the GPU path.

Paper, Section 5 (Discussion): the indices measured there were built from un-reduced automata, whose
redundant states make the index larger than it has to be.  The remedy is the textbook one: merge
the states that no input can tell apart, then index the smaller automaton.

What "tell apart" means here is fixed by what the index records (Section 3, Algorithms 3 and 4, and
Section 2.1 for EOS): whether a walk meets the rejecting state, and whether the state it ends in
accepts (EOS is admissible exactly there).  So every state carries one of three labels -- the
rejecting state, accepting, neither -- and two states are equivalent iff every string of byte
classes leads them to states with the same label.  ``minimise`` computes these classes by
refinement (Moore): start from the labels, split any class whose members disagree, for some byte
class, on the class of their successor, and stop when nothing splits.  Classes are numbered in
order of their smallest state, so the result is unique.

The quotient automaton has one state per class.  Its index is the original's with state ids mapped
through ``block_of_state``: row q of the original holds the same tokens as row block_of_state[q] of
the quotient, and each end state s appears there as block_of_state[s].
"""
from __future__ import annotations

import numpy as np


def minimise(trans, accept, dead):
    """trans [Q, C] int32, accept [Q] uint8, dead int (-1: none).  Returns (block_of_state [Q]
    int32, trans_min [B, C] int32, accept_min [B] uint8, dead_min int)."""
    n_states, n_classes = trans.shape

    def renumber(keys):
        ids = {}
        out = np.zeros(n_states, dtype=np.int32)
        for q in range(n_states):                                  # in state order: numbered by smallest state
            if keys[q] not in ids:
                ids[keys[q]] = len(ids)
            out[q] = ids[keys[q]]
        return out, len(ids)

    label = [0 if q == dead else (1 if accept[q] else 2) for q in range(n_states)]
    block, n_blocks = renumber(label)
    while True:
        keys = [(int(block[q]),) + tuple(int(block[trans[q, c]]) for c in range(n_classes)) for q in range(n_states)]
        refined, n_refined = renumber(keys)
        if n_refined == n_blocks:
            break
        block, n_blocks = refined, n_refined
    rep = np.full(n_blocks, -1, dtype=np.int64)
    for q in range(n_states - 1, -1, -1):
        rep[block[q]] = q
    trans_min = np.zeros((n_blocks, n_classes), dtype=np.int32)
    accept_min = np.zeros(n_blocks, dtype=np.uint8)
    for b in range(n_blocks):
        accept_min[b] = 1 if accept[rep[b]] else 0
        for c in range(n_classes):
            trans_min[b, c] = block[trans[rep[b], c]]
    dead_min = int(block[dead]) if dead >= 0 else -1
    return block, trans_min, accept_min, dead_min
