"""CPU oracle for the index-size row: many automata in one index, and identical rows stored once.
TEST INFRASTRUCTURE ONLY (tests, smoke check, benchmark's CPU leg); plain numpy and Python loops,
nothing shared with the GPU path.

Paper, Section 5 (Discussion): the index of a large grammar is big because it is built from many
un-reduced automata with redundant states; the remedy named there is to reduce it.  Two plain
definitions, both exact:

``union_automaton``  The disjoint union of automata M_1 .. M_K (Section 3, Definition 1, each with
    its own byte classes) as one automaton over one alphabet partition: the states of M_k are
    renumbered ``state_base[k] + s``, and two bytes are in the same class of the union iff every
    M_k puts them in the same class (the coarsest partition that refines all of them).  Classes
    are numbered in order of their smallest byte.  All reject states become one: the union's dead
    state is the renumbered dead state of the first automaton that has one (-1 if none has), and
    every transition into any automaton's dead state leads there.  An index built from the union
    (Algorithms 3 and 4) is the K indices laid end to end: row ``state_base[k] + s`` holds what row
    s of M_k's own index holds, end states renumbered.  This is the serving workload (many regular
    expressions against one vocabulary) done in one build.

``dedupe_rows``  States whose rows sigma(q) are identical -- the same tokens with the same end
    states -- are interchangeable for masking and for the next state; their row is kept once.
    ``row_of_state[q]`` is the number of q's row among the distinct rows, numbered in order of the
    smallest state that has them, and the distinct rows are stored as a CSR of their own.
"""
from __future__ import annotations

import numpy as np


def union_automaton(automata):
    """automata: sequence of (trans [Q_k, C_k] int32, byte_to_class [256] uint8, accept [Q_k]
    uint8, dead int).  Returns (trans, byte_to_class, accept, dead, state_base)."""
    n = len(automata)
    state_base = np.zeros(n + 1, dtype=np.int64)
    for k, (trans, _b2c, _acc, _dead) in enumerate(automata):
        state_base[k + 1] = state_base[k] + trans.shape[0]
    # the union's classes: bytes that every automaton treats alike
    signature_of_class = {}
    byte_to_class = np.zeros(256, dtype=np.int64)
    for b in range(256):
        sig = tuple(int(a[1][b]) for a in automata)
        if sig not in signature_of_class:
            signature_of_class[sig] = len(signature_of_class)        # in order of the smallest byte
        byte_to_class[b] = signature_of_class[sig]
    n_classes = len(signature_of_class)
    representative = [int(np.flatnonzero(byte_to_class == c)[0]) for c in range(n_classes)]
    dead = -1
    for k, (_t, _b, _a, d) in enumerate(automata):
        if d >= 0:
            dead = int(state_base[k] + d)
            break
    total = int(state_base[n])
    trans_u = np.zeros((total, n_classes), dtype=np.int32)
    accept_u = np.zeros(total, dtype=np.uint8)
    for k, (trans, b2c, acc, d) in enumerate(automata):
        for s in range(trans.shape[0]):
            row = int(state_base[k] + s)
            accept_u[row] = 1 if acc[s] else 0
            for c in range(n_classes):
                target = int(trans[s, int(b2c[representative[c]])])
                trans_u[row, c] = dead if (d >= 0 and target == d) else int(state_base[k] + target)
    return trans_u, byte_to_class.astype(np.uint8), accept_u, dead, state_base


def dedupe_rows(row_ptr, token_ids, next_states):
    """Returns (row_of_state [Q] int32, unique_row_ptr [U + 1] int64, token_ids_u, next_states_u)."""
    n_states = row_ptr.size - 1
    seen = {}
    row_of_state = np.zeros(n_states, dtype=np.int32)
    kept = []
    for q in range(n_states):
        a, b = int(row_ptr[q]), int(row_ptr[q + 1])
        key = (token_ids[a:b].tobytes(), next_states[a:b].tobytes())
        if key not in seen:
            seen[key] = len(kept)
            kept.append(q)
        row_of_state[q] = seen[key]
    unique_row_ptr = np.zeros(len(kept) + 1, dtype=np.int64)
    for u, q in enumerate(kept):
        unique_row_ptr[u + 1] = unique_row_ptr[u] + (row_ptr[q + 1] - row_ptr[q])
    tok_u = np.zeros(int(unique_row_ptr[-1]), dtype=np.int32)
    nxt_u = np.zeros(int(unique_row_ptr[-1]), dtype=np.int32)
    for u, q in enumerate(kept):
        a, b = int(row_ptr[q]), int(row_ptr[q + 1])
        tok_u[unique_row_ptr[u]:unique_row_ptr[u + 1]] = token_ids[a:b]
        nxt_u[unique_row_ptr[u]:unique_row_ptr[u + 1]] = next_states[a:b]
    return row_of_state, unique_row_ptr, tok_u, nxt_u
