"""Pins for ``oracle/minimise.py``: the paper's float automaton, the table-filling algorithm as an
independent route to the same classes, brute force over strings, an independent minimiser, and the
relation between the indices of an automaton and of its quotient."""
import itertools

import numpy as np

from paper_2307_09702_amd.synth import workloads as W
from paper_2307_09702_amd.synth import regex_dfa
from paper_2307_09702_amd.synth.regex_dfa import DFA

from oracle import minimise as M


def label(d_accept, dead, q):
    return 0 if q == dead else (1 if d_accept[q] else 2)


def with_clones(rng, d, n_clones, n_unreachable_junk=0):
    """Copies of states (same outgoing transitions, same acceptance), with some transitions of the
    original redirected to a copy: an un-reduced automaton with the same behaviour."""
    # (not of the rejecting state: a copy of it is a state that is merely hopeless, which a walk may
    # enter without being rejected, so it is not equivalent to the original)
    live = np.array([q for q in range(d.n_states) if q != d.dead])
    src = live[rng.integers(0, live.size, size=n_clones)]
    trans = np.concatenate([d.trans, d.trans[src]], axis=0)
    accept = np.concatenate([d.accept, d.accept[src]])
    for k, s in enumerate(src):
        hits = np.argwhere(trans[:d.n_states] == s)
        for (q, c) in hits[rng.random(len(hits)) < 0.5]:
            trans[q, c] = d.n_states + k
    return DFA(np.ascontiguousarray(trans), d.byte_to_class, accept, dead=d.dead), src


def test_float_example_of_the_paper_has_two_live_classes():
    """Section 3's automaton: before the point (states 0, 1) and after it (2, 3) behave alike
    pairwise -- digits loop, a point moves from the first pair to the second -- so it reduces to
    two live states and the rejecting one."""
    d = W.float_dfa()
    block, trans, accept, dead = M.minimise(d.trans, d.accept, d.dead)
    assert block.tolist() == [0, 0, 1, 1, 2] and dead == 2
    assert accept.tolist() == [1, 1, 0]
    digit, point = int(d.byte_to_class[ord("7")]), int(d.byte_to_class[ord(".")])
    assert trans[0, digit] == 0 and trans[0, point] == 1 and trans[1, digit] == 1 and trans[1, point] == 2
    assert (trans[2] == 2).all()


def test_classes_equal_those_of_the_table_filling_algorithm():
    """Independent route: mark every pair of states with different labels, then every pair that
    some byte class sends to a marked pair, until nothing changes; unmarked pairs are equivalent."""
    for seed in range(8):
        rng = np.random.default_rng(seed)
        base = W.random_dfa(rng, int(rng.integers(4, 14)), int(rng.integers(1, 5)), 0.6)
        d, _ = with_clones(rng, base, int(rng.integers(0, 10)))
        n = d.n_states
        marked = np.zeros((n, n), dtype=bool)
        for p in range(n):
            for q in range(n):
                marked[p, q] = label(d.accept, d.dead, p) != label(d.accept, d.dead, q)
        changed = True
        while changed:
            changed = False
            for p in range(n):
                for q in range(n):
                    if not marked[p, q] and any(marked[d.trans[p, c], d.trans[q, c]] for c in range(d.n_classes)):
                        marked[p, q] = True
                        changed = True
        block, *_ = M.minimise(d.trans, d.accept, d.dead)
        for p in range(n):
            for q in range(n):
                assert (block[p] == block[q]) == (not marked[p, q]), (seed, p, q)
        # numbered in order of the smallest state
        firsts = [int(np.flatnonzero(block == b)[0]) for b in range(int(block.max()) + 1)]
        assert firsts == sorted(firsts)


def test_quotient_reads_every_string_like_the_original():
    for seed in range(5):
        rng = np.random.default_rng(50 + seed)
        base = W.random_dfa(rng, 7, 3, 0.6)
        d, _ = with_clones(rng, base, 6)
        block, trans, accept, dead = M.minimise(d.trans, d.accept, d.dead)
        for q in range(d.n_states):
            for length in range(0, 6):
                for word in itertools.product(range(d.n_classes), repeat=length):
                    s, t = q, int(block[q])
                    for c in word:
                        s, t = int(d.trans[s, c]), int(trans[t, c])
                    assert label(d.accept, d.dead, s) == label(accept, dead, t)
                    assert block[s] == t


def test_clones_are_merged_and_a_minimal_automaton_is_left_alone():
    rng = np.random.default_rng(7)
    regex = W.json_schema_regex(rng, 3, nested=False)
    small = regex_dfa.compile_regex(regex)                         # trimmed and minimised by an independent minimiser
    block, trans, accept, dead = M.minimise(small.trans, small.accept, small.dead)
    assert block.tolist() == list(range(small.n_states))           # nothing to merge, numbering kept
    assert np.array_equal(trans, small.trans) and np.array_equal(accept, small.accept) and dead == small.dead
    raw = regex_dfa.compile_regex(regex, minimise=False)           # the same language, un-reduced
    assert raw.n_states > small.n_states
    block, trans, accept, dead = M.minimise(raw.trans, raw.accept, raw.dead)
    assert int(block.max()) + 1 == small.n_states
    cloned, src = with_clones(rng, small, 25)
    block, *_ = M.minimise(cloned.trans, cloned.accept, cloned.dead)
    assert int(block.max()) + 1 == small.n_states
    assert block[:small.n_states].tolist() == list(range(small.n_states))
    assert block[small.n_states:].tolist() == src.tolist()


def test_a_hopeless_state_is_not_the_rejecting_state():
    """A state from which every byte leads to rejection is still a state a one-byte-short token can
    end in: only the rejecting state itself rejects (the walk of Algorithm 3 fails when delta is
    undefined, not when acceptance has become impossible)."""
    trans = np.array([[1, 2], [2, 2], [2, 2]], dtype=np.int32)      # 0 -a-> 1 (hopeless) ; 2 rejects
    block, *_ = M.minimise(trans, np.zeros(3, np.uint8), 2)
    assert block.tolist() == [0, 1, 2]
    block, *_ = M.minimise(trans, np.zeros(3, np.uint8), -1)        # no rejecting state: all three alike
    assert block.tolist() == [0, 0, 0]


def test_index_of_the_quotient_is_the_index_mapped_through_the_classes(oracle_mod):
    """Row q of the original index = row block[q] of the quotient's index with end states mapped."""
    for seed, eos in ((0, -1), (1, 5)):
        rng = np.random.default_rng(90 + seed)
        base = W.random_dfa(rng, 25, 5, 0.5)
        d, _ = with_clones(rng, base, 20)
        vocab = W.bpe_like_vocab(rng, 400, 2.5, 7)
        block, trans, accept, dead = M.minimise(d.trans, d.accept, d.dead)
        full = oracle_mod.build_index(d.trans, d.byte_to_class, d.accept, d.dead, vocab.bytes, vocab.offsets, eos)
        small = oracle_mod.build_index(trans, d.byte_to_class, accept, dead, vocab.bytes, vocab.offsets, eos)
        assert int(block.max()) + 1 < d.n_states
        for q in range(d.n_states):
            a, b = full.row_ptr[q], full.row_ptr[q + 1]
            u, v = small.row_ptr[block[q]], small.row_ptr[block[q] + 1]
            assert full.token_ids[a:b].tolist() == small.token_ids[u:v].tolist(), q
            assert block[full.next_states[a:b]].tolist() == small.next_states[u:v].tolist(), q
