"""GPU parity for minimisation before indexing: fsmidx_minimise_dfa through the C ABI against
``oracle/minimise.py`` (classes, quotient table, acceptance, rejecting state), and the index built
from the device-resident quotient against the index oracle.  Integer work: equality of every element."""
import numpy as np
import pytest

from paper_2307_09702_amd.synth import workloads as W
from paper_2307_09702_amd.synth import regex_dfa
from paper_2307_09702_amd.synth.regex_dfa import DFA

from test_oracle_minimise_pins import with_clones

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2307_09702_amd import binding
    binding.load()
    return binding


def check_minimise(B, d):
    import torch
    from oracle import minimise as M
    block, trans, accept, dead = M.minimise(d.trans, d.accept, d.dead)
    m = B.DeviceMinimised(d.trans, d.byte_to_class, d.accept, d.dead)
    torch.cuda.synchronize()
    assert (m.n_states, m.n_classes, m.dead_state) == (trans.shape[0], trans.shape[1], dead)
    assert np.array_equal(m.block_of_state.cpu().numpy(), block)
    assert np.array_equal(m.trans.cpu().numpy(), trans)
    assert np.array_equal(m.accept[:m.n_states].cpu().numpy(), accept)
    return m, (block, trans, accept, dead)


def test_float_example_of_the_paper(gpu):
    m, want = check_minimise(gpu, W.float_dfa())
    assert want[0].tolist() == [0, 0, 1, 1, 2]


@pytest.mark.parametrize("seed", range(10))
def test_random_automata_with_clones(gpu, seed):
    rng = np.random.default_rng([31, seed])
    n_classes = int(rng.choice([1, 2, 5, 64, 65, 200]))
    base = W.random_dfa(rng, int(rng.integers(2, 300)), n_classes, float(rng.uniform(0.1, 0.9)))
    d, _ = with_clones(rng, base, int(rng.integers(0, 200)))
    if seed % 3 == 0:                                             # rejecting state somewhere else than at the end
        perm = rng.permutation(d.n_states)
        inv = np.argsort(perm)
        d = DFA(perm[d.trans[inv]].astype(np.int32), d.byte_to_class, d.accept[inv], dead=int(perm[d.dead]))
    if seed % 4 == 1:                                             # no rejecting state: the old one is a state like any other
        d = DFA(d.trans, d.byte_to_class, d.accept, dead=-1)
    check_minimise(gpu, d)


def test_single_states_chains_and_an_automaton_that_is_minimal(gpu):
    one = DFA(np.zeros((1, 3), np.int32), (np.arange(256) % 3).astype(np.uint8), np.ones(1, np.uint8), dead=0)
    check_minimise(gpu, one)
    # a chain of 3,000 states ending in the only accepting one: every state is its own class, and the
    # refinement needs as many rounds as the chain is long
    n = 3000
    trans = np.array([[min(s + 1, n)] for s in range(n)] + [[n]], dtype=np.int32)
    accept = np.zeros(n + 1, np.uint8); accept[n - 1] = 1
    chain = DFA(trans, np.zeros(256, np.uint8), accept, dead=n)
    m, want = check_minimise(gpu, chain)
    assert m.n_states == n + 1
    # all states accepting on a ring: one live class however long the ring
    ring = DFA(np.array([[(s + 1) % n] for s in range(n)], dtype=np.int32), np.zeros(256, np.uint8), np.ones(n, np.uint8), dead=-1)
    m, want = check_minimise(gpu, ring)
    assert m.n_states == 1


def test_unreduced_schema_automaton_and_the_index_of_its_quotient(gpu, oracle_mod):
    """The serving case: a schema's automaton as it comes out of the subset construction, reduced on
    the device and indexed from there; the index is the original's mapped through the classes."""
    import torch
    rng = np.random.default_rng(5)
    regex = W.json_schema_regex(rng, 8, nested=False)
    raw = regex_dfa.compile_regex(regex, minimise=False)
    small = regex_dfa.compile_regex(regex)
    m, (block, trans, accept, dead) = check_minimise(gpu, raw)
    assert m.n_states == small.n_states < raw.n_states
    vocab = W.config_json().vocab
    ref = oracle_mod.build_index(trans, raw.byte_to_class, accept, dead, vocab.bytes, vocab.offsets, 50256, n_threads=8)
    prob = gpu.DeviceProblem(m.trans, m.byte_to_class, m.accept, m.dead_state, vocab.bytes, vocab.offsets, 50256)
    csr, tok, nxt = prob.build()
    torch.cuda.synchronize()
    assert np.array_equal(prob.row_ptr.cpu().numpy(), ref.row_ptr)
    assert np.array_equal(tok.cpu().numpy(), ref.token_ids) and np.array_equal(nxt.cpu().numpy(), ref.next_states)
    full = oracle_mod.build_index(raw.trans, raw.byte_to_class, raw.accept, raw.dead, vocab.bytes, vocab.offsets, 50256,
                                  n_threads=8)
    print(f"un-reduced {raw.n_states} states, {full.nnz} entries -> {m.n_states} states, {ref.nnz} entries", flush=True)
    tok_h, nxt_h, ptr = tok.cpu().numpy(), nxt.cpu().numpy(), prob.row_ptr.cpu().numpy()
    for q in rng.integers(0, raw.n_states, size=60):
        a, b = full.row_ptr[q], full.row_ptr[q + 1]
        u, v = ptr[block[q]], ptr[block[q] + 1]
        assert np.array_equal(full.token_ids[a:b], tok_h[u:v])
        assert np.array_equal(block[full.next_states[a:b]], nxt_h[u:v])


def test_bad_tables_are_reported_and_small_outputs_refused(gpu):
    import torch
    d = W.random_dfa(np.random.default_rng(2), 20, 4, 0.5)
    bad = d.trans.copy(); bad[3, 1] = d.n_states + 9
    with pytest.raises(gpu.FsmidxError) as e:
        gpu.DeviceMinimised(bad, d.byte_to_class, d.accept, d.dead)
    assert e.value.code == gpu.BAD_DEVICE_INPUT
    leaky = d.trans.copy(); leaky[d.dead, 0] = 0
    with pytest.raises(gpu.FsmidxError) as e:
        gpu.DeviceMinimised(leaky, d.byte_to_class, d.accept, d.dead)
    assert e.value.code == gpu.BAD_DEVICE_INPUT
    with pytest.raises(gpu.FsmidxError) as e:
        gpu.DeviceMinimised(d.trans, d.byte_to_class, d.accept, d.dead, trans_capacity=8)
    assert e.value.code == gpu.OUTPUT_TOO_SMALL
    torch.cuda.synchronize()
    gpu.DeviceMinimised(d.trans, d.byte_to_class, d.accept, d.dead)      # and the library still works
    torch.cuda.synchronize()
