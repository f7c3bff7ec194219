"""Scanner automata for parser-guided generation, used only to *produce inputs* (test and bench
tooling; Section 4.1 of the paper: every parse state has a list of terminal symbols it reads and an
automaton that is the union of their automata).

    tagged_union     several terminal automata -> one deterministic automaton that runs them side by
                     side, with the set of terminals each state completes (a 64-bit mask)
    scanner_layout   the scanners of all parse states laid out in one transition table over a common
                     set of byte classes, one shared rejecting state last
    toy_grammar      a seeded stand-in for a parse table restricted to its shift moves: which
                     terminals a parse state reads and which parse state follows each of them

Nothing here walks vocabulary tokens, follows completions or computes terminal sets: it holds none of
the method's arithmetic.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

from .regex_dfa import DFA, compile_regex


def tagged_union(dfas):
    """Product of the automata `dfas` (at most 64), explored from the tuple of their start states.

    Returns (DFA, completes): state ids in breadth-first order, byte classes = the coarsest common
    refinement of the inputs' classes, the all-rejecting tuple as the dead state (last id),
    completes[q] = mask with bit t set iff component t accepts in q.  accept[q] = completes[q] != 0.
    """
    assert 1 <= len(dfas) <= 64
    sig = np.stack([d.byte_to_class.astype(np.int64) for d in dfas], axis=1)
    _, first, inverse = np.unique(sig, axis=0, return_index=True, return_inverse=True)
    order = np.argsort(first)
    rank = np.empty_like(order); rank[order] = np.arange(len(order))
    b2c = rank[inverse.reshape(-1)].astype(np.uint8)
    n_classes = int(b2c.max()) + 1
    rep = [int(np.flatnonzero(b2c == c)[0]) for c in range(n_classes)]

    def dead_of(d):
        return d.dead if d.dead >= 0 else None

    start = tuple(d.start for d in dfas)
    all_dead = tuple(-1 for _ in dfas)
    ids = {start: 0}
    todo = [start]
    rows = []
    while todo:
        nxt_todo = []
        for tup in todo:
            row = []
            for c in range(n_classes):
                to = []
                for d, s in zip(dfas, tup):
                    if s < 0:
                        to.append(-1)
                        continue
                    v = int(d.trans[s, d.byte_to_class[rep[c]]])
                    to.append(-1 if v == dead_of(d) else v)
                to = tuple(to)
                if to != all_dead and to not in ids:
                    ids[to] = len(ids)
                    nxt_todo.append(to)
                row.append(to)
            rows.append(row)
        todo = nxt_todo
    n = len(ids)
    trans = np.full((n + 1, n_classes), n, dtype=np.int32)
    completes = np.zeros(n + 1, dtype=np.uint64)
    for tup, q in ids.items():
        for t, (d, s) in enumerate(zip(dfas, tup)):
            if s >= 0 and d.accept[s]:
                completes[q] |= np.uint64(1) << np.uint64(t)
    for q, row in enumerate(rows):
        for c, to in enumerate(row):
            trans[q, c] = n if to == all_dead else ids[to]
    accept = (completes != 0).astype(np.uint8)
    return DFA(trans, b2c, accept, dead=n, start=0), completes


@dataclass
class Scanners:
    """All parse states' scanners in one table."""

    dfa: DFA                      # shared classes; dead = last state; accept = completes != 0
    completes: np.ndarray         # uint64 [Q]   terminals completed in a state (global terminal ids)
    scanner_of_state: np.ndarray  # int32  [Q]   parse state whose scanner the state belongs to (-1: rejecting state)
    start_of_scanner: np.ndarray  # int32  [P]
    shift: np.ndarray             # int32  [P, T] state the scan goes on from after terminal t in parse state p, -1: not read
    n_terminals: int


def scanner_layout(parts, follows, n_terminals):
    """parts[p] = (DFA, completes, terminal ids of its components); follows[p][t] = parse state after
    terminal t is read in parse state p (or -1).  Component-local terminal bits are renamed to the
    global ids."""
    sig = np.stack([d.byte_to_class.astype(np.int64) for d, _, _ in parts], axis=1)
    _, first, inverse = np.unique(sig, axis=0, return_index=True, return_inverse=True)
    order = np.argsort(first)
    rank = np.empty_like(order); rank[order] = np.arange(len(order))
    b2c = rank[inverse.reshape(-1)].astype(np.uint8)
    n_classes = int(b2c.max()) + 1
    rep = [int(np.flatnonzero(b2c == c)[0]) for c in range(n_classes)]
    live = [d.n_states - 1 for d, _, _ in parts]          # each part's dead state is its last
    base = np.concatenate([[0], np.cumsum(live)]).astype(np.int64)
    n = int(base[-1])
    trans = np.full((n + 1, n_classes), n, dtype=np.int32)
    completes = np.zeros(n + 1, dtype=np.uint64)
    owner = np.full(n + 1, -1, dtype=np.int32)
    for p, (d, comp, terms) in enumerate(parts):
        assert d.dead == d.n_states - 1 and d.start == 0
        for s in range(live[p]):
            q = int(base[p]) + s
            owner[q] = p
            for c in range(n_classes):
                v = int(d.trans[s, d.byte_to_class[rep[c]]])
                trans[q, c] = n if v == d.dead else int(base[p]) + v
            m = int(comp[s])
            for local, t in enumerate(terms):
                if (m >> local) & 1:
                    completes[q] |= np.uint64(1) << np.uint64(t)
    starts = base[:-1].astype(np.int32)
    shift = np.full((len(parts), n_terminals), -1, dtype=np.int32)
    for p in range(len(parts)):
        for t in range(n_terminals):
            if follows[p][t] >= 0:
                shift[p, t] = starts[follows[p][t]]
    accept = (completes != 0).astype(np.uint8)
    return Scanners(DFA(trans, b2c, accept, dead=n, start=0), completes, owner, starts, shift, n_terminals)


# Terminals of a small programming-language-like grammar (regexes in the syntax of regex_dfa).
TOY_TERMINALS = [
    ("WS", r"[ \t\n]+"),
    ("NAME", r"[^\W\d]\w*"),
    ("NUMBER", r"[0-9]+(\.[0-9]+)?"),
    ("STRING", r'"[^"\\]*"'),
    ("LPAR", r"\("), ("RPAR", r"\)"), ("LSQB", r"\["), ("RSQB", r"\]"), ("LBRACE", r"\{"), ("RBRACE", r"\}"),
    ("COLON", r":"), ("COMMA", r","), ("SEMI", r";"), ("DOT", r"\."), ("EQUAL", r"="), ("EQEQ", r"=="),
    ("PLUS", r"\+"), ("MINUS", r"-"), ("STAR", r"\*"), ("SLASH", r"/"), ("ARROW", r"->"), ("LESS", r"<"),
    ("LESSEQ", r"<="), ("GREATER", r">"), ("NOTEQ", r"!="),
    ("DEF", "def"), ("RETURN", "return"), ("IF", "if"), ("ELSE", "else"), ("ELIF", "elif"), ("WHILE", "while"),
    ("FOR", "for"), ("IN", "in"), ("NOT", "not"), ("AND", "and"), ("OR", "or"), ("PASS", "pass"),
    ("CLASS", "class"), ("IMPORT", "import"), ("FROM", "from"), ("AS", "as"), ("NONE", "None"),
    ("TRUE", "True"), ("FALSE", "False"), ("LAMBDA", "lambda"), ("WITH", "with"), ("YIELD", "yield"),
]


def toy_grammar(rng: np.random.Generator, n_parse_states: int, terminals=None, min_read: int = 3,
                max_read: int = 12) -> Scanners:
    """Every parse state reads whitespace and a random handful of the other terminals; the parse
    state that follows a terminal is drawn uniformly (whitespace leaves the parse state as it is)."""
    terminals = TOY_TERMINALS if terminals is None else terminals
    n_t = len(terminals)
    compiled = [compile_regex(rx) for _, rx in terminals]
    parts, follows = [], []
    for p in range(n_parse_states):
        k = int(rng.integers(min_read, min(max_read, n_t - 1) + 1))
        others = sorted(int(t) for t in rng.choice(np.arange(1, n_t), size=k, replace=False))
        terms = [0] + others
        d, comp = tagged_union([compiled[t] for t in terms])
        parts.append((d, comp, terms))
        row = np.full(n_t, -1, dtype=np.int64)
        row[0] = p
        for t in others:
            row[t] = int(rng.integers(0, n_parse_states))
        follows.append(row)
    return scanner_layout(parts, follows, n_t)
