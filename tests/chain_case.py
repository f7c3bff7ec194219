"""A chain automaton on which the search over the admissible tokens alone holds more pending
branch points than the search over all tokens (shared by the GPU parity tests).

States S_0 .. S_{k-1} each have three (target, class set) pairs, taken in this order:
{a} -> X, {b} -> S_{i+1}, {c, d} -> Z.  X reads only `a` (back to X) and Z reads nothing, so
b^i a b is rejected while b^i c and b^i d are admissible.  The search over all tokens descends into
X first and comes back before it follows b; restricted to admissible tokens nothing goes to X, so
the node decides {a} and {b} together and waits, with {c, d} still to do, while the search follows
b: one waiting node per level of the chain.
"""
import numpy as np

from paper_2307_09702_amd.synth import workloads as W
from paper_2307_09702_amd.synth.regex_dfa import DFA


def chain_problem(depth: int, replicas: int = 60):
    a, b, c, d, other = 0, 1, 2, 3, 4
    n_classes = 5
    x_state, z_state, dead = depth, depth + 1, depth + 2
    trans = np.full((depth + 3, n_classes), dead, np.int32)
    for i in range(depth):
        trans[i, a] = x_state
        trans[i, b] = i + 1 if i + 1 < depth else z_state
        trans[i, c] = z_state
        trans[i, d] = z_state
    trans[x_state, a] = x_state
    b2c = np.full(256, other, np.uint8)
    for ch, k in ((b"a", a), (b"b", b), (b"c", c), (b"d", d)):
        b2c[ch[0]] = k
    accept = np.zeros(depth + 3, np.uint8)
    accept[z_state] = 1
    accept[0] = 1
    toks = []
    for _ in range(replicas):
        for i in range(depth):
            toks += [b"b" * i + b"ab", b"b" * i + b"c", b"b" * i + b"d"]
    return DFA(trans, b2c, accept, dead=dead), W.Vocab.from_tokens(toks)
