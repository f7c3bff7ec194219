"""CPU oracle for the scanner step of parser-guided generation.  TEST INFRASTRUCTURE ONLY (tests,
smoke check, benchmark's CPU leg); plain numpy and Python loops, nothing shared with the GPU path.

Paper, Section 4 and Section 4.1.  Every parse state reads an ordered list of terminal symbols, and
its scanner is the union of their automata.  Two things are said about such a scanner:

``terminal_sets``  While characters arrive, the scanner knows a set V of terminals that the
    characters read since the last complete symbol can still become; V shrinks until one terminal is
    left (Section 4.1, the paragraph with the ``"de"`` example: there V = {DEF, NAME}).  For a state q
    of the scanner that set is
        V(q) = { t : some string leads from q (possibly the empty one) to a state that completes t },
    the least solution of  V(q) = completes(q) | OR_c V(delta(q, c)).

``restart_table``  A vocabulary string may finish the terminal being read and begin the next one
    (Section 4, the two cases after the ``"def f"`` example and the strings ``" "`` and ``"oo("``): the
    automaton of the current terminal stops in a final state, the parser moves on, and the rest of
    the string is read by the scanner of the parse state that follows.  With the parser's shift
    moves given as a table, this is a transition function of its own:
        delta'(q, c) = delta(q, c)                      if that is not the rejecting state,
                     = delta(shift[p(q), t], c)         otherwise, for the first terminal t in the
                                                        order of the list that q completes, that parse
                                                        state p(q) may shift, and whose following
                                                        scanner reads c,
                     = the rejecting state              if there is no such terminal.
    Algorithms 3 and 4 applied to delta' give the index the section's illustration describes.
    (The stack, and with it REDUCE moves, are outside this step: shift[p, t] depends on p and t
    alone.)
"""
from __future__ import annotations

import numpy as np


def terminal_sets(trans, completes):
    """trans int32 [Q, C], completes uint64 [Q] -> V uint64 [Q]."""
    trans = np.asarray(trans)
    v = np.asarray(completes, dtype=np.uint64).copy()
    while True:
        new = np.asarray(completes, dtype=np.uint64).copy()
        for c in range(trans.shape[1]):
            new |= v[trans[:, c]]
        if np.array_equal(new, v):
            return v
        v = new


def restart_table(trans, dead, completes, scanner_of_state, shift):
    """-> delta' int32 [Q, C].  shift int32 [P, T] holds scanner states or -1; completes[q] has bit t
    set iff q completes terminal t; scanner_of_state[q] is p(q)."""
    trans = np.asarray(trans)
    n_states, n_classes = trans.shape
    n_terminals = shift.shape[1]
    out = trans.copy()
    if dead < 0:
        return out                                       # nothing ever rejects: nothing to restart
    for q in range(n_states):
        if q == dead or int(completes[q]) == 0:
            continue
        done = [t for t in range(n_terminals) if (int(completes[q]) >> t) & 1]
        p = int(scanner_of_state[q])
        for c in range(n_classes):
            if int(trans[q, c]) != dead:
                continue
            for t in done:
                r = int(shift[p, t])
                if r >= 0 and int(trans[r, c]) != dead:
                    out[q, c] = trans[r, c]
                    break
    return out
