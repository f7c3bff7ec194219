"""GPU parity for the reachable-only index: fsmidx_reachable_states and fsmidx_restrict_rows /
_fill through the C ABI against ``oracle/reachable.py``.  Integer and byte work: the bar is
equality of every element."""
import numpy as np
import pytest

from paper_2307_09702_amd.synth import workloads as W
from paper_2307_09702_amd.synth.regex_dfa import DFA

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2307_09702_amd import binding
    binding.load()
    return binding


def built(B, oracle_mod, d, vocab, eos=-1, threads=8):
    import torch
    ref = oracle_mod.build_index(d.trans, d.byte_to_class, d.accept, d.dead, vocab.bytes, vocab.offsets, eos,
                                 n_threads=threads)
    prob = B.DeviceProblem(d.trans, d.byte_to_class, d.accept, d.dead, vocab.bytes, vocab.offsets, eos)
    csr, tok, nxt = prob.build()
    torch.cuda.synchronize()
    return ref, prob, csr, (tok, nxt)


def check_reach(B, ref, csr, starts):
    from oracle import reachable as R
    want = R.reachable_states(ref.row_ptr, ref.next_states, starts)
    reach, n = B.reachable_states(csr, starts)
    assert np.array_equal(reach.cpu().numpy(), want), starts
    assert n == int(want.sum())
    return reach, want


def check_restrict(B, ref, csr, keep_dev, keep_host):
    from oracle import reachable as R
    want = R.restrict_rows(ref.row_ptr, ref.token_ids, ref.next_states, keep_host)
    ptr, tok, nxt = B.restrict_rows(csr, keep_dev)
    assert np.array_equal(ptr.cpu().numpy(), want[0])
    assert np.array_equal(tok.cpu().numpy(), want[1]) and np.array_equal(nxt.cpu().numpy(), want[2])
    return ptr, tok, nxt


def test_float_example_of_the_paper(gpu, oracle_mod):
    d = W.float_dfa()
    ref, prob, csr, keep = built(gpu, oracle_mod, d, W.Vocab.from_tokens(["A", ".", "42", ".2", "1"]))
    reach, want = check_reach(gpu, ref, csr, [0])
    assert want.tolist() == [1, 1, 1, 1, 0]
    check_reach(gpu, ref, csr, [2])
    check_reach(gpu, ref, csr, [])
    check_reach(gpu, ref, csr, [3, 3, 2])
    ref, prob, csr, keep = built(gpu, oracle_mod, d, W.Vocab.from_tokens(["A", "42", "1"]))
    reach, want = check_reach(gpu, ref, csr, [0])
    assert want.tolist() == [1, 1, 0, 0, 0]
    check_restrict(gpu, ref, csr, reach, want)


@pytest.mark.parametrize("seed", range(8))
def test_random_automata_reach_and_restrict(gpu, oracle_mod, seed):
    import torch
    rng = np.random.default_rng([77, seed])
    n_live = int(rng.integers(5, 400))
    d = W.random_dfa(rng, n_live, int(rng.integers(2, 20)), float(rng.uniform(0.05, 0.5)))
    if seed % 3 == 0:                                             # dead state somewhere else than at the end
        perm = rng.permutation(d.n_states)
        inv = np.argsort(perm)
        d = DFA(perm[d.trans[inv]].astype(np.int32), d.byte_to_class, d.accept[inv], dead=int(perm[d.dead]))
    vocab = W.bpe_like_vocab(rng, int(rng.integers(1, 3000)), 2.5, 8)
    eos = int(rng.integers(0, vocab.n_tokens)) if seed % 2 else -1
    ref, prob, csr, keep = built(gpu, oracle_mod, d, vocab, eos)
    for starts in ([0], [int(rng.integers(0, d.n_states))], list(rng.integers(0, d.n_states, size=5)), list(range(d.n_states))):
        reach, want = check_reach(gpu, ref, csr, starts)
        check_restrict(gpu, ref, csr, reach, want)
    # any choice of rows, none and all
    mask = (rng.random(d.n_states) < 0.4).astype(np.uint8)
    check_restrict(gpu, ref, csr, torch.from_numpy(mask).cuda(), mask)
    none = np.zeros(d.n_states, np.uint8)
    ptr, tok, nxt = check_restrict(gpu, ref, csr, torch.from_numpy(none).cuda(), none)
    assert tok.numel() == 0
    check_restrict(gpu, ref, csr, torch.ones(d.n_states, dtype=torch.uint8, device="cuda"), np.ones(d.n_states, np.uint8))


def test_ring_with_thousands_of_levels_and_the_gcd_closed_form(gpu, oracle_mod):
    """Every byte moves one state on, every token has six bytes: from state 0 the search needs
    n / gcd(n, 6) levels, one new state each, and finds the multiples of the gcd."""
    n = 3000 * 6 + 3                                              # gcd 3: 6001 levels
    trans = np.array([[(s + 1) % n] for s in range(n)] + [[n]], dtype=np.int32)
    d = DFA(trans, np.zeros(256, np.uint8), np.ones(n + 1, np.uint8), dead=n)
    vocab = W.Vocab.from_tokens([b"abcdef", b"", b"uvwxyz"])
    ref, prob, csr, keep = built(gpu, oracle_mod, d, vocab)
    reach, n_reached = gpu.reachable_states(csr, [0])
    got = reach.cpu().numpy()
    assert n_reached == n // 3
    assert np.array_equal(np.flatnonzero(got), np.arange(0, n, 3))


def test_large_config_from_its_start_state(gpu, oracle_mod):
    import torch
    w = W.config_large()
    d, v = w.dfa, w.vocab
    ref, prob, csr, keep = built(gpu, oracle_mod, d, v, -1, threads=16)
    reach, want = check_reach(gpu, ref, csr, [d.start])
    ptr, tok, nxt = check_restrict(gpu, ref, csr, reach, want)
    print(f"large config: {int(want.sum())} of {d.n_states} states reachable from the start state, "
          f"{ref.nnz} -> {tok.numel()} entries", flush=True)
    # a vocabulary without one-letter and one-digit tokens reaches far fewer states: inside a key or
    # a word a generation can only be where whole tokens end
    lens = np.diff(v.offsets)
    first = v.bytes[np.minimum(v.offsets[:-1], v.bytes.size - 1)]
    alnum = np.isin(first, np.frombuffer(b"abcdefghijklmnopqrstuvwxyzABCDEFGHIJKLMNOPQRSTUVWXYZ0123456789", np.uint8))
    vocab = W.Vocab.from_tokens([v.token(t) for t in np.flatnonzero((lens >= 2) | ((lens == 1) & ~alnum))])
    ref, prob, csr, keep = built(gpu, oracle_mod, d, vocab, -1, threads=16)
    reach, want = check_reach(gpu, ref, csr, [d.start])
    ptr, tok, nxt = check_restrict(gpu, ref, csr, reach, want)
    print(f"without one-letter and one-digit tokens: {int(want.sum())} of {d.n_states} states reachable, "
          f"{ref.nnz} -> {tok.numel()} entries", flush=True)
    assert 100 < want.sum() < d.n_states // 4
    # masks and greedy steps of a generation from the start state: the restricted index serves them all
    from oracle import decode_step
    restricted = gpu.CCsr(d.n_states, vocab.n_tokens, int(tok.numel()), ptr.data_ptr(), tok.data_ptr(), nxt.data_ptr(), None, 0)
    rng = np.random.default_rng(4)
    states = rng.choice(np.flatnonzero(want), size=64).astype(np.int32)
    logits = (rng.standard_normal((64, vocab.n_tokens)) * 3).astype(np.float32)
    want_masked = oracle_mod.mask_logits(ref, vocab.n_tokens, states, logits)
    x = torch.from_numpy(logits).cuda()
    gpu.mask_logits(restricted, torch.from_numpy(states).cuda(), x)
    torch.cuda.synchronize()
    assert x.cpu().numpy().tobytes() == want_masked.tobytes()
    want_t, want_s = decode_step.masked_argmax(ref.row_ptr, ref.token_ids, ref.next_states, vocab.n_tokens, states, logits)
    got_t, got_s = gpu.masked_argmax(restricted, torch.from_numpy(states).cuda(), torch.from_numpy(logits).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(got_t.cpu().numpy(), want_t)
    chosen = want_t >= 0
    assert np.array_equal(got_s.cpu().numpy()[chosen], want_s[chosen])
    assert want[want_s[chosen]].all()                             # every step stays inside the reachable set


def test_end_states_outside_the_automaton_are_ignored_and_bad_calls_refused(gpu, oracle_mod):
    """An index the library did not write: end states are range checked before they are used."""
    import torch
    from oracle import reachable as R
    row_ptr = np.array([0, 3, 5, 5, 6], dtype=np.int64)
    tok = np.array([0, 1, 2, 0, 2, 1], dtype=np.int32)
    nxt = np.array([1, 9, -1, 3, 4, 0], dtype=np.int32)          # 9, -1 and 4 name no state of four
    dev = [torch.from_numpy(a).cuda() for a in (row_ptr, tok, nxt)]
    csr = gpu.CCsr(4, 3, 6, dev[0].data_ptr(), dev[1].data_ptr(), dev[2].data_ptr(), None, 0)
    reach, n = gpu.reachable_states(csr, [0])
    assert reach.cpu().tolist() == [1, 1, 0, 1] and n == 3
    clean = np.where((nxt >= 0) & (nxt < 4), nxt, 0).astype(np.int32)
    assert R.reachable_states(row_ptr, clean, [0]).tolist() == [1, 1, 0, 1]
    for bad in ([4], [-1], [0, 7]):
        with pytest.raises(gpu.FsmidxError) as e:
            gpu.reachable_states(csr, bad)
        assert e.value.code == gpu.INVALID_ARG
    torch.cuda.synchronize()
