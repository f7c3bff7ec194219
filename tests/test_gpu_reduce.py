"""GPU parity for the index-size row: fsmidx_union_dfa and fsmidx_dedupe_rows / _fill through the C
ABI against ``oracle/index_reduce.py`` (and, for the index built from a union, against the index
oracle on the oracle's own union).  Integer work: the bar is equality of every element."""
import numpy as np
import pytest

from paper_2307_09702_amd.synth import workloads as W
from paper_2307_09702_amd.synth.regex_dfa import DFA, compile_regex

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2307_09702_amd import binding
    binding.load()
    return binding


def as_tuple(d):
    return (d.trans, d.byte_to_class, d.accept, d.dead)


def schema_automata(n, seed):
    """JSON-object automata of different schemas with their natural byte classes."""
    out = []
    for k in range(n):
        rng = np.random.default_rng([seed, k])
        out.append(compile_regex(W.json_schema_regex(rng, 4, nested=False)))
    return out


def check_union(B, oracle_mod, autos, vocab, eos):
    import torch
    from oracle import index_reduce as R
    want = R.union_automaton([as_tuple(d) for d in autos])
    u = B.DeviceUnion([as_tuple(d) for d in autos])
    torch.cuda.synchronize()
    assert (u.n_states, u.n_classes, u.dead_state) == (want[0].shape[0], want[0].shape[1], want[3])
    assert np.array_equal(u.state_base, want[4])
    assert np.array_equal(u.trans.cpu().numpy(), want[0])
    assert np.array_equal(u.byte_to_class.cpu().numpy(), want[1])
    assert np.array_equal(u.accept[:u.n_states].cpu().numpy(), want[2])
    # the index of the union, built from the device-resident union, against the index oracle
    ref = oracle_mod.build_index(want[0], want[1], want[2], want[3], vocab.bytes, vocab.offsets, eos, n_threads=8)
    prob = B.DeviceProblem(u.trans, u.byte_to_class, u.accept, u.dead_state, vocab.bytes, vocab.offsets, eos)
    csr, tok, nxt = prob.build()
    torch.cuda.synchronize()
    assert np.array_equal(prob.row_ptr.cpu().numpy(), ref.row_ptr)
    assert np.array_equal(tok.cpu().numpy(), ref.token_ids) and np.array_equal(nxt.cpu().numpy(), ref.next_states)
    return u, ref, prob, csr, (tok, nxt)


def test_union_of_the_papers_examples_and_small_random_automata(gpu, oracle_mod):
    rng = np.random.default_rng(3)
    autos = [W.float_dfa(), W.name_dfa(), W.random_dfa(rng, 9, 5, 0.6),
             DFA(rng.integers(0, 6, size=(6, 4)).astype(np.int32), W.random_partition(rng, 4), np.ones(6, np.uint8), dead=-1),
             W.random_dfa(rng, 30, 64, 0.4)]
    vocab = W.Vocab.from_tokens(["A", ".", "42", ".2", "1", "d", "ef", "pass", " ", "oo(", "):"] +
                                [W.bpe_like_vocab(rng, 600, 2.5, 7).token(t) for t in range(600)])
    check_union(gpu, oracle_mod, autos, vocab, 3)
    check_union(gpu, oracle_mod, autos[3:4], vocab, -1)              # one automaton, no dead state
    check_union(gpu, oracle_mod, [autos[2]] * 3, vocab, -1)          # the same automaton three times


def test_union_of_schema_automata_goes_through_the_token_set_walk_and_masks_a_mixed_batch(gpu, oracle_mod):
    """The serving case: eight JSON-schema automata against one vocabulary, one build; a decode
    batch whose rows belong to different automata is masked with one call."""
    import torch
    autos = schema_automata(8, 17)
    w = W.config_json()
    u, ref, prob, csr, keep = check_union(gpu, oracle_mod, autos, w.vocab, -1)
    assert u.n_classes <= 64
    rng = np.random.default_rng(5)
    states = np.array([int(u.state_base[k] + rng.integers(0, autos[k].n_states)) for k in rng.integers(0, 8, size=32)],
                      dtype=np.int32)
    logits = (rng.standard_normal((32, w.vocab.n_tokens)) * 3).astype(np.float32)
    want = oracle_mod.mask_logits(ref, w.vocab.n_tokens, states, logits)
    x = torch.from_numpy(logits).cuda()
    gpu.mask_logits(csr, torch.from_numpy(states).cuda(), x)
    torch.cuda.synchronize()
    assert x.cpu().numpy().tobytes() == want.tobytes()


def test_union_argument_and_input_checks(gpu):
    import ctypes
    import torch
    lib = gpu.load()
    n = ctypes.c_size_t()
    assert lib.fsmidx_union_workspace_bytes(0, ctypes.byref(n)) == gpu.INVALID_ARG
    assert lib.fsmidx_union_workspace_bytes(65, ctypes.byref(n)) == gpu.INVALID_ARG
    d = W.float_dfa()
    with pytest.raises(gpu.FsmidxError) as e:                           # table does not fit
        gpu.DeviceUnion([as_tuple(d), as_tuple(d)], trans_capacity=10)
    assert e.value.code == gpu.OUTPUT_TOO_SMALL
    bad = d.trans.copy(); bad[1, 0] = 99
    with pytest.raises(gpu.FsmidxError) as e:
        gpu.DeviceUnion([as_tuple(d), (bad, d.byte_to_class, d.accept, d.dead)])
    assert e.value.code == gpu.BAD_DEVICE_INPUT
    b2c = d.byte_to_class.copy(); b2c[65] = 7
    with pytest.raises(gpu.FsmidxError) as e:
        gpu.DeviceUnion([(d.trans, b2c, d.accept, d.dead)])
    assert e.value.code == gpu.BAD_DEVICE_INPUT
    torch.cuda.synchronize()


def check_dedupe(B, ref, csr):
    from oracle import index_reduce as R
    want = R.dedupe_rows(ref.row_ptr, ref.token_ids, ref.next_states)
    row_of, urp, tok_u, nxt_u = B.dedupe_rows(csr)
    assert np.array_equal(row_of.cpu().numpy(), want[0])
    assert np.array_equal(urp.cpu().numpy(), want[1])
    assert np.array_equal(tok_u.cpu().numpy(), want[2]) and np.array_equal(nxt_u.cpu().numpy(), want[3])
    return row_of, urp, tok_u, nxt_u


def test_dedupe_float_example_clones_and_empty_rows(gpu, oracle_mod):
    import torch
    d = W.float_dfa()
    vocab = W.Vocab.from_tokens(["A", ".", "42", ".2", "1"])
    ref = oracle_mod.build_index(d.trans, d.byte_to_class, d.accept, d.dead, vocab.bytes, vocab.offsets, -1)
    prob = gpu.DeviceProblem(d.trans, d.byte_to_class, d.accept, d.dead, vocab.bytes, vocab.offsets, -1)
    csr, tok, nxt = prob.build()
    torch.cuda.synchronize()
    row_of, urp, *_ = check_dedupe(gpu, ref, csr)
    assert row_of.cpu().tolist() == [0, 0, 1, 1, 2] and urp.cpu().tolist() == [0, 4, 6, 6]
    # clones of states (same outgoing transitions), many empty rows, rows of very different length
    rng = np.random.default_rng(12)
    base = W.random_dfa(rng, 40, 6, 0.5)
    clones = rng.integers(0, 40, size=30)
    trans = np.concatenate([base.trans, base.trans[clones], np.full((25, 6), base.dead, np.int32)], axis=0)
    accept = np.concatenate([base.accept, base.accept[clones], np.zeros(25, np.uint8)])
    big = DFA(trans, base.byte_to_class, accept, dead=base.dead)
    vocab = W.bpe_like_vocab(rng, 20000, 2.0, 8)
    for eos in (-1, 11):
        ref = oracle_mod.build_index(big.trans, big.byte_to_class, big.accept, big.dead, vocab.bytes, vocab.offsets, eos)
        prob = gpu.DeviceProblem(big.trans, big.byte_to_class, big.accept, big.dead, vocab.bytes, vocab.offsets, eos)
        csr, tok, nxt = prob.build()
        torch.cuda.synchronize()
        row_of, urp, *_ = check_dedupe(gpu, ref, csr)
        if eos < 0:
            assert urp.numel() - 1 <= 42


def test_dedupe_on_a_union_with_repeated_automata_and_masking_through_row_of_state(gpu, oracle_mod):
    """A union that holds the same automata several times over has every row several times; the
    compact index, used with row_of_state[state] in the place of the state, masks the same."""
    import torch
    autos = schema_automata(3, 23)
    autos = autos + autos[:2] + autos
    w = W.config_json()
    vocab = W.Vocab.from_tokens([w.vocab.token(t) for t in range(12000)])
    u, ref, prob, csr, keep = check_union(gpu, oracle_mod, autos, vocab, -1)
    row_of, urp, tok_u, nxt_u = check_dedupe(gpu, ref, csr)
    n_unique = urp.numel() - 1
    # states of a repeated automaton are not merged with their twins (their rows name their own
    # automaton's states), but the dead rows and the rows that hold the same tokens and ends are
    assert n_unique < u.n_states
    compact = gpu.CCsr(n_unique, vocab.n_tokens, int(tok_u.numel()), urp.data_ptr(), tok_u.data_ptr(), nxt_u.data_ptr(),
                       None, 0)
    rng = np.random.default_rng(6)
    states = rng.integers(0, u.n_states, size=40).astype(np.int32)
    logits = (rng.standard_normal((40, vocab.n_tokens)) * 3).astype(np.float32)
    want = oracle_mod.mask_logits(ref, vocab.n_tokens, states, logits)
    rows = row_of[torch.from_numpy(states).cuda().long()].contiguous()
    x = torch.from_numpy(logits).cuda()
    gpu.mask_logits(compact, rows, x)
    torch.cuda.synchronize()
    assert x.cpu().numpy().tobytes() == want.tobytes()
    # and the greedy step: same tokens, same end states
    from oracle import decode_step
    want_t, want_s = decode_step.masked_argmax(ref.row_ptr, ref.token_ids, ref.next_states, vocab.n_tokens, states, logits)
    got_t, got_s = gpu.masked_argmax(compact, rows, torch.from_numpy(logits).cuda())
    torch.cuda.synchronize()
    got_t, got_s = got_t.cpu().numpy(), got_s.cpu().numpy()
    assert np.array_equal(got_t, want_t)
    chosen = want_t >= 0                        # (an empty row gives the id that names no row: the index's own n_states)
    assert np.array_equal(got_s[chosen], want_s[chosen]) and (got_s[~chosen] == n_unique).all()


def test_dedupe_on_the_large_config(gpu, oracle_mod):
    import torch
    w = W.config_large()
    d, v = w.dfa, w.vocab
    ref = oracle_mod.build_index(d.trans, d.byte_to_class, d.accept, d.dead, v.bytes, v.offsets, -1, n_threads=16)
    prob = gpu.DeviceProblem(d.trans, d.byte_to_class, d.accept, d.dead, v.bytes, v.offsets, -1)
    csr, tok, nxt = prob.build()
    torch.cuda.synchronize()
    row_of, urp, tok_u, nxt_u = check_dedupe(gpu, ref, csr)
    print(f"large config: {d.n_states} states, {urp.numel() - 1} distinct rows, {ref.nnz} -> {tok_u.numel()} entries", flush=True)
