"""GPU parity: libfsmidx (through its C ABI) against the CPU oracle, element by element.

The index is integer work, so the bar is bit-exact equality of row_ptr, token_ids and
next_states; masked logits are bit copies or -inf, so they are compared as raw bits too.
"""
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


def oracle_index(oracle, dfa, vocab, eos=-1, threads=16):
    return oracle.build_index(dfa.trans, dfa.byte_to_class, dfa.accept, dfa.dead, vocab.bytes, vocab.offsets,
                              eos, n_threads=threads)


def gpu_index_device_flow(B, dfa, vocab, eos=-1):
    import torch
    prob = B.DeviceProblem(dfa.trans, dfa.byte_to_class, dfa.accept, dfa.dead, vocab.bytes, vocab.offsets, eos)
    csr, tok, nxt = prob.build()
    torch.cuda.synchronize()
    prob.keep_alive = (tok, nxt)                 # csr holds raw pointers into these tensors
    return prob, csr, prob.row_ptr.cpu().numpy(), tok.cpu().numpy(), nxt.cpu().numpy()


def assert_same_index(ref, row_ptr, tok, nxt, what=""):
    assert row_ptr.dtype == np.int64 and tok.dtype == np.int32 and nxt.dtype == np.int32
    assert np.array_equal(row_ptr, ref.row_ptr), f"{what}: row_ptr differs"
    assert np.array_equal(tok, ref.token_ids), f"{what}: token_ids differ"
    assert np.array_equal(nxt, ref.next_states), f"{what}: next_states differ"


# ----------------------------------------------------------------------------- the five configs

@pytest.mark.parametrize("cfg", [0, 1, 2, 3])
def test_index_bit_exact_on_config(gpu, oracle_mod, cfg):
    w = W.CONFIGS[cfg]()
    print(f"config {cfg}: Q={w.dfa.n_states} C={w.dfa.n_classes} N={w.vocab.n_tokens}", flush=True)
    ref = oracle_index(oracle_mod, w.dfa, w.vocab)
    _, _, row_ptr, tok, nxt = gpu_index_device_flow(gpu, w.dfa, w.vocab)
    assert_same_index(ref, row_ptr, tok, nxt, w.name)


@pytest.mark.parametrize("cfg", [0, 1])
def test_index_with_eos_on_small_configs(gpu, oracle_mod, cfg):
    w = W.CONFIGS[cfg]()
    eos = w.vocab.n_tokens - 1
    ref = oracle_index(oracle_mod, w.dfa, w.vocab, eos)
    _, _, row_ptr, tok, nxt = gpu_index_device_flow(gpu, w.dfa, w.vocab, eos)
    assert_same_index(ref, row_ptr, tok, nxt, w.name + "+eos")
    assert (tok == eos).sum() == int(w.dfa.accept.sum())


def test_host_flow_matches_oracle_and_device_flow(gpu, oracle_mod):
    w = W.config_random()
    d, v = w.dfa, w.vocab
    ref = oracle_index(oracle_mod, d, v, 17)
    h = gpu.build_index(d.trans, d.byte_to_class, d.accept, d.dead, v.bytes, v.offsets, 17)
    assert h.nnz == ref.nnz
    row_ptr, tok, nxt = h.to_host()
    assert_same_index(ref, row_ptr, tok, nxt, "host flow")
    h.free()
    h.free()                                     # idempotent


def test_big_random_config_bit_exact(gpu, oracle_mod):
    """Config 4's build (20,000 states x 128,256 tokens, 2.6e9 pairs, 2.2e8 entries), in the launch
    configuration the benchmark times: row_ptr, token_ids and next_states against the oracle's,
    element by element (in slices, so that one slice of each side is on the host at a time)."""
    import torch
    w = W.config_big_random()
    d, v = w.dfa, w.vocab
    print("C4-big: oracle ...", flush=True)
    ref = oracle_index(oracle_mod, d, v)
    print(f"C4-big: oracle nnz={ref.nnz} W_bf={ref.w_bf}; GPU build ...", flush=True)
    prob = gpu.DeviceProblem(d.trans, d.byte_to_class, d.accept, d.dead, v.bytes, v.offsets, -1)
    csr, tok, nxt = prob.build()
    torch.cuda.synchronize()
    row_ptr = prob.row_ptr.cpu().numpy()
    assert np.array_equal(row_ptr, ref.row_ptr), "C4-big: row_ptr differs"
    nnz = int(row_ptr[-1])
    assert nnz == tok.numel() == nxt.numel() == ref.nnz > 2 ** 27
    step = 1 << 25
    for a in range(0, nnz, step):
        b = min(a + step, nnz)
        assert np.array_equal(tok[a:b].cpu().numpy(), ref.token_ids[a:b]), f"C4-big: token_ids differ in [{a}, {b})"
        assert np.array_equal(nxt[a:b].cpu().numpy(), ref.next_states[a:b]), f"C4-big: next_states differ in [{a}, {b})"
    # the one-call build into the same arrays gives the same bits
    tok2 = torch.full_like(tok, -1)
    nxt2 = torch.full_like(nxt, -1)
    assert prob.build_into(tok2, nxt2) == nnz
    torch.cuda.synchronize()
    assert torch.equal(tok2, tok) and torch.equal(nxt2, nxt)
    # properties that hold at any size
    lens = np.diff(v.offsets)
    expect = 20000 * (0.3 ** lens).sum()         # a walk of L bytes survives with probability 0.3^L
    assert abs(nnz - expect) < 0.02 * expect
    assert row_ptr[d.dead + 1] == row_ptr[d.dead]
    assert not bool((nxt == d.dead).any())


# ----------------------------------------------------------------------------- edge cases

def tiny_random(seed, n_live, n_classes, p_live, n_tokens, mean_len, cap):
    rng = np.random.default_rng(seed)
    return W.random_dfa(rng, n_live, n_classes, p_live), W.bpe_like_vocab(rng, n_tokens, mean_len, cap)


@pytest.mark.parametrize("n_tokens", [0, 1, 63, 64, 65, 511, 512, 513, 1537])
def test_ragged_token_counts(gpu, oracle_mod, n_tokens):
    dfa, vocab = tiny_random(n_tokens, 19, 5, 0.7, n_tokens, 3.0, 12)
    ref = oracle_index(oracle_mod, dfa, vocab)
    _, _, row_ptr, tok, nxt = gpu_index_device_flow(gpu, dfa, vocab)
    assert_same_index(ref, row_ptr, tok, nxt, f"N={n_tokens}")


def test_empty_tokens_long_tokens_and_no_bytes(gpu, oracle_mod):
    rng = np.random.default_rng(1)
    dfa = W.random_dfa(rng, 12, 4, 0.95)
    toks = [b"", b"a", b"", b"x" * 9, b"ab" * 20, bytes(rng.integers(0, 256, 100).astype(np.uint8)), b"", b"q" * 8, b"r" * 7]
    vocab = W.Vocab.from_tokens(toks)
    ref = oracle_index(oracle_mod, dfa, vocab, 6)                 # EOS is an empty token here
    _, _, row_ptr, tok, nxt = gpu_index_device_flow(gpu, dfa, vocab, 6)
    assert_same_index(ref, row_ptr, tok, nxt, "mixed lengths")
    assert ref.nnz > 0
    vocab = W.Vocab.from_tokens([b"", b"", b""])                  # n_bytes == 0
    ref = oracle_index(oracle_mod, dfa, vocab, 1)
    _, _, row_ptr, tok, nxt = gpu_index_device_flow(gpu, dfa, vocab, 1)
    assert_same_index(ref, row_ptr, tok, nxt, "no bytes")


@pytest.mark.parametrize("n_live", [40, 9000])
def test_tokens_around_the_widths_of_the_length_fields(gpu, oracle_mod, n_live):
    """Runs of one byte that every state reads, 254 to 70,000 bytes long (lengths are kept in 8 bits
    in the tokens' short form and in 16 bits in the dense walk's staging, with the record behind
    both), among ordinary tokens; a small automaton and one large enough for the emit pass to take
    the short form first."""
    rng = np.random.default_rng(5 + n_live)
    n_classes = 8
    dfa = W.random_dfa(rng, n_live, n_classes, 0.5)
    c = int(dfa.byte_to_class[ord("x")])
    dfa.trans[:n_live, c] = rng.integers(0, n_live, n_live)         # "x" is read everywhere
    runs = [b"x" * n for n in (254, 255, 256, 300, 65534, 65535, 65536, 70000)]
    few = W.bpe_like_vocab(rng, 2000, 3.0, 12)
    toks = [few.token(t) for t in range(1000)] + runs + [few.token(t) for t in range(1000, 2000)]
    vocab = W.Vocab.from_tokens(toks)
    ref = oracle_index(oracle_mod, dfa, vocab, 3)
    _, _, row_ptr, tok, nxt = gpu_index_device_flow(gpu, dfa, vocab, 3)
    assert_same_index(ref, row_ptr, tok, nxt, "very long tokens")
    # every run is admissible from every live state
    assert all(np.isin(np.arange(1000, 1008), ref.token_ids[ref.row_ptr[q]:ref.row_ptr[q + 1]]).all() for q in (0, n_live - 1))


def test_no_dead_state_and_single_state(gpu, oracle_mod):
    rng = np.random.default_rng(8)
    trans = rng.integers(0, 7, size=(7, 3)).astype(np.int32)
    dfa = DFA(trans, W.random_partition(rng, 3), (rng.random(7) < 0.5).astype(np.uint8), dead=-1)
    vocab = W.bpe_like_vocab(rng, 700, 3.0, 10)
    ref = oracle_index(oracle_mod, dfa, vocab, 5)
    _, _, row_ptr, tok, nxt = gpu_index_device_flow(gpu, dfa, vocab, 5)
    assert_same_index(ref, row_ptr, tok, nxt, "no dead state")
    assert ref.nnz == 7 * 699 + int(dfa.accept.sum())
    one = DFA(np.zeros((1, 2), np.int32), (np.arange(256) % 2).astype(np.uint8), np.ones(1, np.uint8), dead=0)
    ref = oracle_index(oracle_mod, one, vocab)
    _, _, row_ptr, tok, nxt = gpu_index_device_flow(gpu, one, vocab)
    assert_same_index(ref, row_ptr, tok, nxt, "only a dead state")
    assert ref.nnz == 0


def test_dead_state_in_the_middle_and_all_dead(gpu, oracle_mod):
    rng = np.random.default_rng(9)
    dfa = W.random_dfa(rng, 30, 6, 0.6)
    perm = rng.permutation(31)                                   # move the dead state to a random id
    inv = np.argsort(perm)
    moved = DFA(perm[dfa.trans[inv]].astype(np.int32), dfa.byte_to_class, dfa.accept[inv], dead=int(perm[30]))
    vocab = W.bpe_like_vocab(rng, 2000, 3.0, 9)
    ref = oracle_index(oracle_mod, moved, vocab, 3)
    _, _, row_ptr, tok, nxt = gpu_index_device_flow(gpu, moved, vocab, 3)
    assert_same_index(ref, row_ptr, tok, nxt, "dead in the middle")
    alld = DFA(np.full((9, 4), 8, np.int32), W.random_partition(rng, 4), np.ones(9, np.uint8), dead=8)
    ref = oracle_index(oracle_mod, alld, vocab)
    _, _, row_ptr, tok, nxt = gpu_index_device_flow(gpu, alld, vocab)
    assert_same_index(ref, row_ptr, tok, nxt, "all dead")
    assert ref.nnz == 0


@pytest.mark.parametrize("n_classes", [1, 64, 65, 130, 256])
def test_class_counts_up_to_256(gpu, oracle_mod, n_classes):
    rng = np.random.default_rng(n_classes)
    dfa = W.random_dfa(rng, 50, n_classes, 0.8)
    data = rng.integers(0, 256, size=6000).astype(np.uint8)       # all 256 byte values occur
    lens = rng.integers(1, 5, size=2000)
    offsets = np.zeros(2001, np.int64); np.cumsum(lens, out=offsets[1:])
    vocab = W.Vocab(data[:offsets[-1]], offsets)
    ref = oracle_index(oracle_mod, dfa, vocab)
    _, _, row_ptr, tok, nxt = gpu_index_device_flow(gpu, dfa, vocab)
    assert_same_index(ref, row_ptr, tok, nxt, f"C={n_classes}")
    assert ref.nnz > 0


def test_more_than_65535_states_uses_wide_entries(gpu, oracle_mod):
    rng = np.random.default_rng(70)
    dfa = W.random_dfa(rng, 70000, 3, 0.8)
    vocab = W.bpe_like_vocab(rng, 300, 3.0, 8)
    ref = oracle_index(oracle_mod, dfa, vocab, 11)
    _, _, row_ptr, tok, nxt = gpu_index_device_flow(gpu, dfa, vocab, 11)
    assert_same_index(ref, row_ptr, tok, nxt, "Q=70001")
    assert ref.next_states.max() > 65535


def test_table_sizes_around_the_lds_limit(gpu, oracle_mod):
    """64 KiB is where the walk kernel stops copying the table to LDS."""
    for n_live in (1023, 1024, 1025):                            # x 32 classes x 2 bytes
        rng = np.random.default_rng(n_live)
        dfa = W.random_dfa(rng, n_live - 1, 32, 0.5)
        vocab = W.bpe_like_vocab(rng, 900, 3.0, 8)
        ref = oracle_index(oracle_mod, dfa, vocab)
        _, _, row_ptr, tok, nxt = gpu_index_device_flow(gpu, dfa, vocab)
        assert_same_index(ref, row_ptr, tok, nxt, f"Q={n_live}")


@pytest.mark.parametrize("n_live,n_classes,p_live,dead,what", [
    (300, 64, 0.3, "last", "a few live classes per state"),
    (300, 64, 0.5, "last", "half of the classes live"),
    (300, 64, 0.9, "last", "most pairs survive the first byte: a queue per state"),
    (150, 64, 1.0, "none", "no dead state: every class is live"),
    (300, 64, 0.4, "middle", "dead state in the middle"),
    (400, 33, 0.4, "last", "odd number of classes"),
    (7000, 2, 0.8, "last", "two classes, many states"),
])
def test_dense_walk_with_the_table_in_memory(gpu, oracle_mod, n_live, n_classes, p_live, dead, what):
    """16-bit states, at most 64 classes and a table beyond 12 KB: the lane-per-pair walk whose
    lookups after the first byte are gathers from memory, with few and with many survivors per state."""
    rng = np.random.default_rng([n_live, n_classes, int(p_live * 100)])
    dfa = W.random_dfa(rng, n_live, n_classes, p_live)
    if dead == "none":
        dfa = DFA(np.ascontiguousarray(dfa.trans[:n_live]), dfa.byte_to_class, dfa.accept[:n_live], dead=-1)
    elif dead == "middle":
        perm = rng.permutation(n_live + 1)
        inv = np.argsort(perm)
        dfa = DFA(perm[dfa.trans[inv]].astype(np.int32), dfa.byte_to_class, dfa.accept[inv], dead=int(perm[n_live]))
    assert dfa.trans.size * 2 > 12 * 1024
    vocab = W.bpe_like_vocab(rng, 2900, 4.0, 40)                  # three token groups, the last ragged; tokens past 8 bytes
    eos = 1500
    ref = oracle_index(oracle_mod, dfa, vocab, eos)
    _, _, row_ptr, tok, nxt = gpu_index_device_flow(gpu, dfa, vocab, eos)
    assert_same_index(ref, row_ptr, tok, nxt, what)
    assert ref.nnz > 0


def test_dense_walk_many_states_per_wave(gpu, oracle_mod):
    """Enough (state, token group) units that a wave walks more consecutive states than it keeps
    bitmap rows for at a time."""
    rng = np.random.default_rng(3000)
    dfa = W.random_dfa(rng, 3000, 64, 0.3)
    vocab = W.bpe_like_vocab(rng, 100_000, 4.5, 32)
    ref = oracle_index(oracle_mod, dfa, vocab, 77_777)
    _, _, row_ptr, tok, nxt = gpu_index_device_flow(gpu, dfa, vocab, 77_777)
    assert_same_index(ref, row_ptr, tok, nxt, "18 states per wave")


# ----------------------------------------------------------------------------- choice of the walk

def cyclic_dfa(n_live, steps, n_classes=None):
    """State s reads class k (k < len(steps)) and moves to (s + steps[k]) mod n_live; every other
    class leads to the dead state n_live.  One class per target, so len(steps) pairs per state."""
    n_classes = n_classes or len(steps) + 1
    trans = np.full((n_live + 1, n_classes), n_live, np.int32)
    for s in range(n_live):
        for k, d in enumerate(steps):
            trans[s, k] = (s + d) % n_live
    b2c = (np.arange(256) % n_classes).astype(np.uint8)
    return DFA(trans, b2c, (np.arange(n_live + 1) % 3 == 0).astype(np.uint8), dead=n_live)


def test_deep_branching_overflows_the_search_stack_and_is_redone(gpu, oracle_mod):
    # three pairs per state and tokens of up to 24 bytes over the three live classes: the token-set
    # search would need a frame per byte; the library has to notice and count with the other kernel
    dfa = cyclic_dfa(12, (1, 2, 3))
    rng = np.random.default_rng(31)
    toks = [bytes(rng.integers(0, 3, int(rng.integers(1, 25))).astype(np.uint8)) for _ in range(9000)]
    toks += [bytes([3]), b"", bytes([0, 1, 2, 3])]
    vocab = W.Vocab.from_tokens(toks)
    ref = oracle_index(oracle_mod, dfa, vocab, 9001)
    _, _, row_ptr, tok, nxt = gpu_index_device_flow(gpu, dfa, vocab, 9001)
    assert_same_index(ref, row_ptr, tok, nxt, "deep branching")
    assert ref.nnz >= 12 * 9000


def test_shallow_branching_stays_within_the_search_stack(gpu, oracle_mod):
    # same automaton, tokens of at most 6 bytes: at most 6 frames are ever needed -- more than the
    # first attempt's stack holds, so the count is redone with the deep stack, which suffices
    dfa = cyclic_dfa(12, (1, 2, 3))
    rng = np.random.default_rng(32)
    toks = [bytes(rng.integers(0, 4, int(rng.integers(1, 7))).astype(np.uint8)) for _ in range(9000)]
    vocab = W.Vocab.from_tokens(toks)
    for eos in (-1, 0, 4095, 4096, 8999):
        ref = oracle_index(oracle_mod, dfa, vocab, eos)
        _, _, row_ptr, tok, nxt = gpu_index_device_flow(gpu, dfa, vocab, eos)
        assert_same_index(ref, row_ptr, tok, nxt, f"shallow branching, eos={eos}")


def test_searched_segment_with_more_end_nodes_than_node_numbers(gpu, oracle_mod):
    # state 0 fans out over 64 classes to 64 states that loop on everything: a block of 4096 tokens
    # of 1..3 bytes, all admissible from state 0, ends in up to 3 x 64 different search nodes, more
    # than the emit kernel has numbers for; the surplus nodes are stored directly
    n_classes = 64
    trans = np.empty((66, n_classes), np.int32)
    trans[0] = 1 + np.arange(n_classes)
    for s in range(1, 65):
        trans[s] = s
    trans[65] = 65
    trans[7, 5] = 65                                                     # a little rejection as well
    b2c = (np.arange(256) % n_classes).astype(np.uint8)
    dfa = DFA(trans, b2c, (np.arange(66) % 2).astype(np.uint8), dead=65)
    rng = np.random.default_rng(35)
    toks = [bytes(rng.integers(0, 256, int(rng.integers(1, 4))).astype(np.uint8)) for _ in range(9000)]
    vocab = W.Vocab.from_tokens(toks)
    ref = oracle_index(oracle_mod, dfa, vocab, 4100)
    assert len(set(ref.row(0)[1][:4000].tolist())) == 64 and ref.row(0)[0].size > 8900
    _, _, row_ptr, tok, nxt = gpu_index_device_flow(gpu, dfa, vocab, 4100)
    assert_same_index(ref, row_ptr, tok, nxt, "fan-out 64")


@pytest.mark.parametrize("n_first", [513, 767, 768, 769, 1023, 1024, 1025, 2303, 2304, 4095, 4096])
def test_searched_segments_around_the_sizes_in_which_their_entries_leave(gpu, oracle_mod, n_first):
    """Entries of a searched segment (more than 512) are collected and stored 256 at a time.  Three
    blocks of one-byte tokens, admissible (class 0 or 1) or not (class 2): the first with exactly
    n_first admissible tokens at random places, the second full, the third with 600 crowded into
    its last chunks; two states that read them into different end states, one that reads nothing."""
    rng = np.random.default_rng(n_first)
    cls = np.full(3 * 4096, 2, np.uint8)
    first = rng.choice(4096, size=n_first, replace=False)
    cls[first] = rng.integers(0, 2, size=n_first)
    cls[4096:8192] = rng.integers(0, 2, size=4096)
    cls[3 * 4096 - 600:] = rng.integers(0, 2, size=600)
    vocab = W.Vocab.from_tokens([bytes([c]) for c in cls])
    trans = np.array([[1, 2, 4], [2, 2, 4], [0, 1, 4], [4, 4, 4], [4, 4, 4]], np.int32)
    b2c = np.minimum(np.arange(256), 2).astype(np.uint8)
    dfa = DFA(trans, b2c, np.array([1, 0, 1, 1, 0], np.uint8), dead=4)
    for eos in (-1, int(first[0])):
        ref = oracle_index(oracle_mod, dfa, vocab, eos)
        assert int(ref.row_ptr[1]) >= n_first + 4096 + 600
        _, _, row_ptr, tok, nxt = gpu_index_device_flow(gpu, dfa, vocab, eos)
        assert_same_index(ref, row_ptr, tok, nxt, f"n_first={n_first}, eos={eos}")


@pytest.mark.parametrize("depth,eos,replicas", [(10, -1, 60), (12, 1, 60), (8, -1, 60), (3, 0, 200)])
def test_emit_search_that_needs_more_frames_than_the_counting_walk(gpu, oracle_mod, depth, eos, replicas):
    """Restricted to the admissible tokens the search of the emitting pass can hold more waiting
    nodes than the counting walk did (see chain_case): the counting walk needs one frame on this
    automaton, the emitting search one per level of the chain, more than it has for depth > 8; those
    segments have to come out right all the same, in the two-call and in the one-call build."""
    import torch
    import chain_case
    dfa, vocab = chain_case.chain_problem(depth, replicas)
    ref = oracle_index(oracle_mod, dfa, vocab, eos)
    assert int(np.diff(ref.row_ptr)[0]) > 512                      # state 0's segment is a searched one
    _, _, row_ptr, tok, nxt = gpu_index_device_flow(gpu, dfa, vocab, eos)
    assert_same_index(ref, row_ptr, tok, nxt, f"chain depth {depth}, two calls")
    prob = gpu.DeviceProblem(dfa.trans, dfa.byte_to_class, dfa.accept, dfa.dead, vocab.bytes, vocab.offsets, eos)
    tok = torch.full((ref.nnz,), -7, dtype=torch.int32, device="cuda")
    nxt = torch.full((ref.nnz,), -7, dtype=torch.int32, device="cuda")
    assert prob.build_into(tok, nxt) == ref.nnz
    torch.cuda.synchronize()
    assert_same_index(ref, prob.row_ptr.cpu().numpy(), tok.cpu().numpy(), nxt.cpu().numpy(), f"chain depth {depth}, one call")


def test_token_longer_than_32_bytes_with_a_chain_automaton(gpu, oracle_mod):
    # a JSON-like automaton (the token-set walk's case) but one token of 40 bytes: lane-per-pair walk
    w = W.CONFIGS[2]()
    toks = [w.vocab.token(t) for t in range(3000)] + [b"a" * 40, b"a" * 32, b"a" * 33, b' ' * 31]
    vocab = W.Vocab.from_tokens(toks)
    ref = oracle_index(oracle_mod, w.dfa, vocab)
    _, _, row_ptr, tok, nxt = gpu_index_device_flow(gpu, w.dfa, vocab)
    assert_same_index(ref, row_ptr, tok, nxt, "40-byte token")
    short = W.Vocab.from_tokens(toks[:3000] + [b"a" * 32, b' ' * 31])   # longest token exactly 32 bytes
    ref = oracle_index(oracle_mod, w.dfa, short)
    _, _, row_ptr, tok, nxt = gpu_index_device_flow(gpu, w.dfa, short)
    assert_same_index(ref, row_ptr, tok, nxt, "32-byte token")


def test_more_distinct_class_sets_than_the_bitmap_table_holds(gpu, oracle_mod):
    # two targets per state, the 64 classes split differently in every state: > 128 distinct sets
    rng = np.random.default_rng(33)
    n_live, n_classes = 150, 64
    trans = np.empty((n_live + 1, n_classes), np.int32)
    for s in range(n_live):
        a, b = rng.integers(0, n_live, 2)
        trans[s] = np.where(rng.random(n_classes) < 0.5, a, b)
        trans[s, rng.integers(0, n_classes, 8)] = n_live
    trans[n_live] = n_live
    dfa = DFA(trans, W.random_partition(rng, n_classes), (rng.random(n_live + 1) < 0.3).astype(np.uint8), dead=n_live)
    vocab = W.bpe_like_vocab(rng, 6000, 3.0, 12)
    ref = oracle_index(oracle_mod, dfa, vocab, 17)
    _, _, row_ptr, tok, nxt = gpu_index_device_flow(gpu, dfa, vocab, 17)
    assert_same_index(ref, row_ptr, tok, nxt, "many class sets")


@pytest.mark.parametrize("n_live", [40, 63, 64, 65, 66, 100, 127, 128, 129, 130, 160])
def test_numbers_of_distinct_class_sets_around_every_word_of_the_set_masks(gpu, oracle_mod, n_live):
    # two targets per state, the 64 classes split differently in every state: about 2 n_live distinct
    # sets, i.e. one to four 64-bit words of sets per class, and just past what the table holds
    rng = np.random.default_rng(100 + n_live)
    n_classes = 64
    trans = np.empty((n_live + 1, n_classes), np.int32)
    for s in range(n_live):
        # (the other target reads nothing further, so that the search never has two ways to go on
        # and stays within its stack whatever the tokens' lengths)
        trans[s] = np.where(rng.random(n_classes) < 0.5, rng.integers(0, n_live - 1), n_live - 1)
    trans[n_live - 1] = n_live
    trans[n_live] = n_live
    dfa = DFA(trans, W.random_partition(rng, n_classes), (rng.random(n_live + 1) < 0.3).astype(np.uint8), dead=n_live)
    vocab = W.bpe_like_vocab(rng, 9000, 2.5, 10)
    ref = oracle_index(oracle_mod, dfa, vocab, 5)
    _, _, row_ptr, tok, nxt = gpu_index_device_flow(gpu, dfa, vocab, 5)
    assert_same_index(ref, row_ptr, tok, nxt, f"{n_live} states with two class sets each")


def test_vocabulary_of_more_than_64_blocks_on_the_token_set_walk(gpu, oracle_mod):
    # C2's automaton against 300,000 tokens: 74 blocks of 4096, more than a wave has lanes
    w = W.CONFIGS[2]()
    vocab = W.bpe_like_vocab(W.rng_for(2, 7), 300000, 4.0, 16)
    ref = oracle_index(oracle_mod, w.dfa, vocab, 299999)
    _, _, row_ptr, tok, nxt = gpu_index_device_flow(gpu, w.dfa, vocab, 299999)
    assert_same_index(ref, row_ptr, tok, nxt, "C2 x 300,000 tokens")


def test_chain_automaton_with_eos_in_every_kind_of_block(gpu, oracle_mod):
    # C2 goes through the token-set walk; 50,257 tokens = 12 full blocks and a ragged one
    w = W.CONFIGS[2]()
    n = w.vocab.n_tokens
    for eos in (0, 4095, 4096, 8191, n - 1):
        ref = oracle_index(oracle_mod, w.dfa, w.vocab, eos)
        _, _, row_ptr, tok, nxt = gpu_index_device_flow(gpu, w.dfa, w.vocab, eos)
        assert_same_index(ref, row_ptr, tok, nxt, f"C2 eos={eos}")


def test_single_call_build_with_capacity(gpu, oracle_mod):
    import torch
    for cfg, eos in ((1, 31999), (2, -1)):                          # lane-per-pair walk and token-set walk
        w = W.CONFIGS[cfg]()
        ref = oracle_index(oracle_mod, w.dfa, w.vocab, eos)
        prob = gpu.DeviceProblem(w.dfa.trans, w.dfa.byte_to_class, w.dfa.accept, w.dfa.dead, w.vocab.bytes,
                                 w.vocab.offsets, eos)
        # too small: reports the size, leaves the arrays alone, and fill can finish the build
        small_t = torch.full((ref.nnz - 1,), -7, dtype=torch.int32, device="cuda")
        small_n = torch.full((ref.nnz - 1,), -7, dtype=torch.int32, device="cuda")
        with pytest.raises(gpu.OutputTooSmall) as err:
            prob.build_into(small_t, small_n)
        assert err.value.nnz == ref.nnz
        torch.cuda.synchronize()
        assert bool((small_t == -7).all()) and bool((small_n == -7).all())
        tok = torch.empty(ref.nnz, dtype=torch.int32, device="cuda")
        nxt = torch.empty(ref.nnz, dtype=torch.int32, device="cuda")
        prob.fill(ref.nnz, tok, nxt)
        torch.cuda.synchronize()
        assert_same_index(ref, prob.row_ptr.cpu().numpy(), tok.cpu().numpy(), nxt.cpu().numpy(), f"cfg {cfg} fill after")
        # large enough (with slack): one call
        tok = torch.full((ref.nnz + 100,), -7, dtype=torch.int32, device="cuda")
        nxt = torch.full((ref.nnz + 100,), -7, dtype=torch.int32, device="cuda")
        assert prob.build_into(tok, nxt) == ref.nnz
        torch.cuda.synchronize()
        assert_same_index(ref, prob.row_ptr.cpu().numpy(), tok[:ref.nnz].cpu().numpy(), nxt[:ref.nnz].cpu().numpy(),
                          f"cfg {cfg} single call")
        assert bool((tok[ref.nnz:] == -7).all())
        # the emitting pass may be repeated on the same workspace, after either kind of build
        for again in range(2):
            tok.fill_(-7)
            nxt.fill_(-7)
            prob.fill(ref.nnz, tok, nxt)
            torch.cuda.synchronize()
            assert_same_index(ref, prob.row_ptr.cpu().numpy(), tok[:ref.nnz].cpu().numpy(),
                              nxt[:ref.nnz].cpu().numpy(), f"cfg {cfg} fill again {again}")


def test_single_call_build_when_the_search_stack_overflows(gpu, oracle_mod):
    import torch
    dfa = cyclic_dfa(12, (1, 2, 3))
    rng = np.random.default_rng(34)
    toks = [bytes(rng.integers(0, 3, int(rng.integers(1, 25))).astype(np.uint8)) for _ in range(5000)]
    vocab = W.Vocab.from_tokens(toks)
    ref = oracle_index(oracle_mod, dfa, vocab)
    prob = gpu.DeviceProblem(dfa.trans, dfa.byte_to_class, dfa.accept, dfa.dead, vocab.bytes, vocab.offsets, -1)
    tok = torch.empty(ref.nnz, dtype=torch.int32, device="cuda")
    nxt = torch.empty(ref.nnz, dtype=torch.int32, device="cuda")
    assert prob.build_into(tok, nxt) == ref.nnz
    torch.cuda.synchronize()
    assert_same_index(ref, prob.row_ptr.cpu().numpy(), tok.cpu().numpy(), nxt.cpu().numpy(), "overflow, single call")


def test_two_builds_under_way_at_a_time_on_two_streams(gpu, oracle_mod):
    """Two different problems, each with its own workspace, output arrays and stream, enqueued one
    after the other and only then waited for, several times over (the token-set walk and the
    lane-per-pair walk side by side; hints of earlier builds in use from the second time on)."""
    import torch
    cases = []
    for cfg, eos in ((2, 50256), (1, 31999)):
        w = W.CONFIGS[cfg]()
        d, v = w.dfa, w.vocab
        ref = oracle_index(oracle_mod, d, v, eos)
        prob = gpu.DeviceProblem(d.trans, d.byte_to_class, d.accept, d.dead, v.bytes, v.offsets, eos)
        tok = torch.empty(ref.nnz, dtype=torch.int32, device="cuda")
        nxt = torch.empty(ref.nnz, dtype=torch.int32, device="cuda")
        rng = np.random.default_rng(cfg)
        states = rng.integers(-1, d.n_states, size=8).astype(np.int32)
        logits = (rng.standard_normal((8, v.n_tokens)) * 3).astype(np.float32)
        want = oracle_mod.mask_logits(ref, v.n_tokens, states, logits)
        cases.append((prob, tok, nxt, ref, torch.cuda.Stream(), torch.from_numpy(states).cuda(), logits, want))
    for repeat in range(4):
        masked = []
        for prob, tok, nxt, ref, stream, st, logits, want in cases:
            tok.fill_(-7); nxt.fill_(-7)
            torch.cuda.synchronize()
        for prob, tok, nxt, ref, stream, st, logits, want in cases:
            x = torch.from_numpy(logits).cuda()
            torch.cuda.synchronize()
            prob.build_enqueue(tok, nxt, stream=stream)
            gpu.mask_logits(prob.csr(ref.nnz, tok, nxt), st, x, stream=stream)
            masked.append(x)
        for (prob, tok, nxt, ref, stream, st, logits, want), x in zip(cases, masked):
            got, redone = prob.build_finish(tok, nxt, stream=stream)
            assert got == ref.nnz
            if redone:                                              # (first build without a hint may be redone: mask again)
                gpu.mask_logits(prob.csr(ref.nnz, tok, nxt), st, x.copy_(torch.from_numpy(logits)), stream=stream)
            stream.synchronize()
            assert_same_index(ref, prob.row_ptr.cpu().numpy(), tok.cpu().numpy(), nxt.cpu().numpy(), f"repeat {repeat}")
            assert x.cpu().numpy().tobytes() == want.tobytes()


def test_build_in_two_halves_with_masks_enqueued_in_between(gpu, oracle_mod):
    """fsmidx_build_enqueue + fsmidx_build_finish: work enqueued between the two sees the finished
    index; a build whose counting pass has to be redone says so."""
    import torch
    w = W.CONFIGS[2]()
    d, v = w.dfa, w.vocab
    ref = oracle_index(oracle_mod, d, v, 50256)
    prob = gpu.DeviceProblem(d.trans, d.byte_to_class, d.accept, d.dead, v.bytes, v.offsets, 50256)
    tok = torch.full((ref.nnz + 7,), -7, dtype=torch.int32, device="cuda")
    nxt = torch.full((ref.nnz + 7,), -7, dtype=torch.int32, device="cuda")
    rng = np.random.default_rng(2)
    states = rng.integers(-1, d.n_states, size=16).astype(np.int32)
    logits = (rng.standard_normal((16, v.n_tokens)) * 3).astype(np.float32)
    want = oracle_mod.mask_logits(ref, v.n_tokens, states, logits)
    st = torch.from_numpy(states).cuda()
    for repeat in range(3):                                        # the first build has no hint, the later ones follow one
        tok.fill_(-7); nxt.fill_(-7)
        prob.row_ptr.fill_(-1)
        x = torch.from_numpy(logits).cuda()
        y = torch.from_numpy(logits).cuda()
        torch.cuda.synchronize()
        prob.build_enqueue(tok, nxt)
        gpu.mask_logits(prob.csr(ref.nnz, tok, nxt), st, x)                         # bitmap form
        gpu.mask_logits(prob.csr(ref.nnz, tok, nxt, with_bits=False), st, y)        # rows of the CSR
        nnz, redone = prob.build_finish(tok, nxt)
        torch.cuda.synchronize()
        assert nnz == ref.nnz and not redone
        assert_same_index(ref, prob.row_ptr.cpu().numpy(), tok[:nnz].cpu().numpy(), nxt[:nnz].cpu().numpy(), "two halves")
        assert bool((tok[nnz:] == -7).all())
        assert x.cpu().numpy().tobytes() == want.tobytes() and y.cpu().numpy().tobytes() == want.tobytes()
    # too small: finish reports the size needed
    small = torch.full((ref.nnz - 1,), -7, dtype=torch.int32, device="cuda")
    prob.build_enqueue(small, small.clone())
    with pytest.raises(gpu.OutputTooSmall) as err:
        prob.build_finish(small, small.clone())
    assert err.value.nnz == ref.nnz
    # a search that needs the deep stack: finish redoes the counting pass and says so
    dfa = cyclic_dfa(12, (1, 2, 3))
    toks = [bytes(rng.integers(0, 3, int(rng.integers(1, 25))).astype(np.uint8)) for _ in range(5000)]
    vocab = W.Vocab.from_tokens(toks)
    ref = oracle_index(oracle_mod, dfa, vocab)
    prob = gpu.DeviceProblem(dfa.trans, dfa.byte_to_class, dfa.accept, dfa.dead, vocab.bytes, vocab.offsets, -1)
    tok = torch.empty(ref.nnz, dtype=torch.int32, device="cuda")
    nxt = torch.empty(ref.nnz, dtype=torch.int32, device="cuda")
    prob.build_enqueue(tok, nxt)
    nnz, redone = prob.build_finish(tok, nxt)
    torch.cuda.synchronize()
    assert nnz == ref.nnz and redone
    assert_same_index(ref, prob.row_ptr.cpu().numpy(), tok.cpu().numpy(), nxt.cpu().numpy(), "two halves, redone")


@pytest.mark.parametrize("longest", [3, 4, 5, 6, 7, 8, 9])
def test_single_call_build_around_the_depths_of_both_search_stacks(gpu, oracle_mod, longest):
    """Three pairs per state and tokens of up to `longest` bytes need up to `longest` stack frames:
    within the first attempt's stack, beyond it but within the deep one, and beyond both."""
    import torch
    dfa = cyclic_dfa(12, (1, 2, 3))
    rng = np.random.default_rng(40 + longest)
    toks = [bytes(rng.integers(0, 4, int(rng.integers(1, longest + 1))).astype(np.uint8)) for _ in range(6000)]
    toks += [bytes([0, 1, 2] * 3)[:longest]] * 3                      # some tokens of full length that survive
    vocab = W.Vocab.from_tokens(toks)
    ref = oracle_index(oracle_mod, dfa, vocab, 5)
    prob = gpu.DeviceProblem(dfa.trans, dfa.byte_to_class, dfa.accept, dfa.dead, vocab.bytes, vocab.offsets, 5)
    tok = torch.empty(ref.nnz, dtype=torch.int32, device="cuda")
    nxt = torch.empty(ref.nnz, dtype=torch.int32, device="cuda")
    assert prob.build_into(tok, nxt) == ref.nnz
    torch.cuda.synchronize()
    assert_same_index(ref, prob.row_ptr.cpu().numpy(), tok.cpu().numpy(), nxt.cpu().numpy(), f"longest={longest}, single call")
    _, _, row_ptr, tok2, nxt2 = gpu_index_device_flow(gpu, dfa, vocab, 5)
    assert_same_index(ref, row_ptr, tok2, nxt2, f"longest={longest}, two calls")


def test_builds_that_follow_a_hint_from_the_previous_build(gpu, oracle_mod):
    """After a build the library remembers which counting kernel the device chose for these buffers
    and launches only that one the next time.  Two automata of one shape, one for each kernel, are
    written into the same device buffers in turn: a build that follows the wrong hint has to notice
    and still give the right index, and the one after it follows the corrected hint."""
    import torch
    rng = np.random.default_rng(91)
    chainy = few_target_dfa(rng, 120, 24, 2, 0.3)                     # token-set kernels
    dense = W.random_dfa(rng, 120, 24, 0.7)                           # ~17 targets per state: dense kernel
    assert chainy.n_states == dense.n_states and chainy.dead == dense.dead
    dense = DFA(dense.trans, chainy.byte_to_class, dense.accept, dense.dead)
    vocab = W.bpe_like_vocab(rng, 9000, 3.0, 12)
    refs = {"chainy": oracle_index(oracle_mod, chainy, vocab, 5), "dense": oracle_index(oracle_mod, dense, vocab, 5)}
    prob = gpu.DeviceProblem(chainy.trans, chainy.byte_to_class, chainy.accept, chainy.dead, vocab.bytes, vocab.offsets, 5)
    cap = max(r.nnz for r in refs.values())
    tok = torch.empty(cap, dtype=torch.int32, device="cuda")
    nxt = torch.empty(cap, dtype=torch.int32, device="cuda")
    for step, name in enumerate(["chainy", "chainy", "dense", "dense", "dense", "chainy", "chainy", "chainy", "dense"]):
        d = chainy if name == "chainy" else dense
        prob.trans.copy_(torch.from_numpy(d.trans))
        prob.accept.copy_(torch.from_numpy(d.accept))
        torch.cuda.synchronize()
        ref = refs[name]
        if step % 2 == 0:
            assert prob.build_into(tok, nxt) == ref.nnz
        else:
            assert prob.count() == ref.nnz
            prob.fill(ref.nnz, tok, nxt)
        torch.cuda.synchronize()
        assert_same_index(ref, prob.row_ptr.cpu().numpy(), tok[:ref.nnz].cpu().numpy(), nxt[:ref.nnz].cpu().numpy(),
                          f"step {step}: {name}")


def test_repeated_builds_are_identical(gpu):
    import torch
    w = W.config_json()
    d, v = w.dfa, w.vocab
    prob = gpu.DeviceProblem(d.trans, d.byte_to_class, d.accept, d.dead, v.bytes, v.offsets, -1)
    first = None
    for _ in range(3):
        _, tok, nxt = prob.build()
        torch.cuda.synchronize()
        cur = (prob.row_ptr.cpu().numpy().tobytes(), tok.cpu().numpy().tobytes(), nxt.cpu().numpy().tobytes())
        assert first is None or cur == first
        first = cur


# ----------------------------------------------------------------------------- device-side input checks

def test_bad_device_inputs_are_reported_not_dereferenced(gpu):
    w = W.config_tiny()
    d, v = w.dfa, w.vocab

    def expect_bad(trans=d.trans, b2c=d.byte_to_class, offsets=v.offsets, fragment=""):
        prob = gpu.DeviceProblem(trans, b2c, d.accept, d.dead, v.bytes, offsets, -1)
        with pytest.raises(gpu.FsmidxError) as e:
            prob.count()
        assert e.value.code == gpu.BAD_DEVICE_INPUT and fragment in str(e.value)

    t = d.trans.copy(); t[1, 0] = 1 << 20
    expect_bad(trans=t, fragment="transition")
    t = d.trans.copy(); t[2, 2] = -7
    expect_bad(trans=t, fragment="transition")
    t = d.trans.copy(); t[4, 0] = 0
    expect_bad(trans=t, fragment="dead state")
    b = d.byte_to_class.copy(); b[0x31] = 200
    expect_bad(b2c=b, fragment="byte_to_class")
    o = v.offsets.copy(); o[10] = 1 << 40
    expect_bad(offsets=o, fragment="offsets")
    o = v.offsets.copy(); o[5] = -3
    expect_bad(offsets=o, fragment="offsets")
    o = v.offsets.copy(); o[-1] -= 1
    expect_bad(offsets=o, fragment="offsets")
    # and the same problem object works again with good inputs afterwards
    prob = gpu.DeviceProblem(d.trans, d.byte_to_class, d.accept, d.dead, v.bytes, v.offsets, -1)
    assert prob.count() > 0


def many_three_way_states(n_live, seed):
    """n_live states with three targets each -- a random state, and two states that read nothing
    further -- over six fixed three-way splits of 48 classes: 3 pairs per state (the most the
    token-set walk accepts on average), 18 distinct class sets, searches that never branch."""
    rng = np.random.default_rng(seed)
    n_classes = 48
    # (the state that goes on has the widest class set: the search follows a node's last pair without
    # a stack frame, so it never needs more than one whatever the tokens' lengths)
    splits = [rng.permutation(np.repeat([0, 1, 2], [28, 10, 10])) for _ in range(6)]
    end_a, end_b = n_live - 2, n_live - 1
    trans = np.empty((n_live + 1, n_classes), np.int32)
    nxt = rng.integers(0, n_live - 2, n_live)
    which = rng.integers(0, 6, n_live)
    for s in range(n_live):
        trans[s] = np.choose(splits[which[s]], [nxt[s], end_a, end_b])
    trans[end_a] = n_live
    trans[end_b] = n_live
    trans[n_live] = n_live
    return DFA(trans, W.random_partition(rng, n_classes), (rng.random(n_live + 1) < 0.3).astype(np.uint8), dead=n_live)


def test_twenty_thousand_states_with_three_targets_each(gpu, oracle_mod):
    """More states with more than two pairs than the finishing workgroup's list holds at a time,
    three rounds of 8192 states in it, and more workgroups of check words than it reads in one go."""
    dfa = many_three_way_states(20000, 71)
    vocab = W.bpe_like_vocab(np.random.default_rng(72), 5000, 3.0, 12)
    ref = oracle_index(oracle_mod, dfa, vocab, 11)
    _, _, row_ptr, tok, nxt = gpu_index_device_flow(gpu, dfa, vocab, 11)
    assert_same_index(ref, row_ptr, tok, nxt, "20,000 three-way states")
    # a bad value in one of the last states is still found
    bad = dfa.trans.copy()
    bad[19990, 3] = 70000
    prob = gpu.DeviceProblem(bad, dfa.byte_to_class, dfa.accept, dfa.dead, vocab.bytes, vocab.offsets, 11)
    with pytest.raises(gpu.FsmidxError) as e:
        prob.count()
    assert e.value.code == gpu.BAD_DEVICE_INPUT and "transition" in str(e.value)


# ----------------------------------------------------------------------------- mask_logits

def without_bits(B, csr):
    """The same index without its bitmap form: mask_logits then searches the CSR rows."""
    return B.CCsr(csr.n_states, csr.n_tokens, csr.nnz, csr.row_ptr, csr.token_ids, csr.next_states, None, 0)


def run_mask(B, csr, states, logits_np, torch_dtype, in_place, stride=None):
    import torch
    n = logits_np.shape[1]
    stride = n if stride is None else stride
    dev = torch.device("cuda:0")
    st = torch.from_numpy(states).to(dev)
    buf = torch.zeros(logits_np.shape[0], stride, dtype=torch_dtype, device=dev)
    if torch_dtype == torch.bfloat16:
        host = torch.from_numpy(logits_np.view(np.int16)).view(torch.bfloat16)
    else:
        host = torch.from_numpy(logits_np)
    buf[:, :n] = host.to(dev)
    if stride > n:
        buf[:, n:] = 7.0                                          # must stay untouched
    if in_place:
        B.mask_logits(csr, st, buf, None, row_stride=stride)
        out = buf
    else:
        out = torch.full_like(buf, 5.0)
        B.mask_logits(csr, st, buf, out, row_stride=stride)
    torch.cuda.synchronize()
    if stride > n:
        assert bool((out[:, n:] == (7.0 if in_place else 5.0)).all())
    res = out[:, :n].contiguous().cpu()
    return res.view(torch.int16).numpy().view(np.uint16) if torch_dtype == torch.bfloat16 else res.numpy()


@pytest.mark.parametrize("bits", [True, False])
@pytest.mark.parametrize("in_place", [False, True])
@pytest.mark.parametrize("stride_pad", [0, 8, 3])
def test_mask_bit_exact_small(gpu, oracle_mod, in_place, stride_pad, bits):
    import torch
    w = W.config_tiny()
    d, v = w.dfa, w.vocab
    ref = oracle_index(oracle_mod, d, v)
    prob, csr, *_ = gpu_index_device_flow(gpu, d, v)
    assert csr.allow_bits
    if not bits:
        csr = without_bits(gpu, csr)
    n = v.n_tokens
    rng = np.random.default_rng(0)
    states = np.array([0, 1, 2, 3, 4, -1, 99, 0, 2 ** 31 - 1, -(2 ** 31)], dtype=np.int32)
    logits = (rng.standard_normal((states.size, n)) * 3).astype(np.float32)
    logits[7, :4] = np.array([np.nan, -0.0, np.inf, -np.inf], np.float32)
    logits.view(np.uint32)[7, 4] = 0x7FC12345
    want = oracle_mod.mask_logits(ref, n, states, logits)
    got = run_mask(gpu, csr, states, logits, torch.float32, in_place, n + stride_pad)
    assert got.view(np.uint32).tobytes() == want.view(np.uint32).tobytes()
    bits = W.f32_to_bf16_bits(np.nan_to_num(logits, nan=1.0))
    want16 = oracle_mod.mask_logits(ref, n, states, bits)
    got16 = run_mask(gpu, csr, states, bits, torch.bfloat16, in_place, n + stride_pad)
    assert got16.tobytes() == want16.tobytes()


def test_mask_bit_exact_on_decode_config(gpu, oracle_mod):
    """Config 4's decode step: 256 rows at random live states of config 3's index, fp32 and bf16,
    full width 128,256, in place and out of place."""
    import torch
    w = W.config_large()
    d, v = w.dfa, w.vocab
    ref = oracle_index(oracle_mod, d, v)
    prob, csr, row_ptr, tok, nxt = gpu_index_device_flow(gpu, d, v)
    assert_same_index(ref, row_ptr, tok, nxt, "C3")
    states, logits = W.decode_batch(d.n_states, d.dead, v.n_tokens)
    assert states.shape == (256,) and logits.shape == (256, 128256)
    want = oracle_mod.mask_logits(ref, v.n_tokens, states, logits)
    kept = (want != np.float32(-np.inf)).sum(axis=1)
    assert np.array_equal(kept, np.diff(ref.row_ptr)[states])
    bits = W.f32_to_bf16_bits(logits)
    want16 = oracle_mod.mask_logits(ref, v.n_tokens, states, bits)
    for index in (csr, without_bits(gpu, csr)):                   # bitmap kernel, then CSR-search kernel
        for in_place in (False, True):
            got = run_mask(gpu, index, states, logits, torch.float32, in_place)
            assert got.view(np.uint32).tobytes() == want.view(np.uint32).tobytes()
            got16 = run_mask(gpu, index, states, bits, torch.bfloat16, in_place)
            assert got16.tobytes() == want16.tobytes()


def test_mask_segment_boundaries(gpu, oracle_mod):
    """Vocabulary sizes around the 16,384-element segment handled by one workgroup, with a total
    automaton (every token allowed), a sparse one, and rows that are empty."""
    import torch
    for n in (16383, 16384, 16385, 32768 + 5):
        rng = np.random.default_rng(n)
        dfa = W.random_dfa(rng, 6, 4, 0.55)
        vocab = W.bpe_like_vocab(rng, n, 2.0, 6)
        ref = oracle_index(oracle_mod, dfa, vocab, n - 1)
        prob, csr, *_ = gpu_index_device_flow(gpu, dfa, vocab, n - 1)
        states = np.array([0, 1, 2, 3, 4, 5, 6, -1], dtype=np.int32)
        logits = rng.standard_normal((8, n)).astype(np.float32)
        want = oracle_mod.mask_logits(ref, n, states, logits)
        bits = W.f32_to_bf16_bits(logits)
        want16 = oracle_mod.mask_logits(ref, n, states, bits)
        for index in (csr, without_bits(gpu, csr)):
            for in_place in (False, True):
                got = run_mask(gpu, index, states, logits, torch.float32, in_place)
                assert got.view(np.uint32).tobytes() == want.view(np.uint32).tobytes(), (n, in_place)
            got16 = run_mask(gpu, index, states, bits, torch.bfloat16, True, n + 1)  # odd stride: scalar path
            assert got16.tobytes() == want16.tobytes()
            got16 = run_mask(gpu, index, states, bits, torch.bfloat16, False)
            assert got16.tobytes() == want16.tobytes()


# ----------------------------------------------------------------------------- randomised problems

def few_target_dfa(rng, n_live, n_classes, max_targets, p_dead):
    """Every state reads a random subset of the classes and sends it to at most ``max_targets``
    distinct states (the shape the token-set walk takes); the rest is rejected."""
    trans = np.full((n_live + 1, n_classes), n_live, np.int32)
    for s in range(n_live):
        targets = rng.integers(0, n_live, size=int(rng.integers(1, max_targets + 1)))
        reads = rng.random(n_classes) >= p_dead
        trans[s, reads] = targets[rng.integers(0, targets.size, size=int(reads.sum()))]
    accept = (rng.random(n_live + 1) < 0.3).astype(np.uint8)
    return DFA(trans, W.random_partition(rng, n_classes), accept, dead=n_live)


def relabel_states(rng, dfa):
    """The same automaton with its state ids permuted (the dead state lands anywhere)."""
    n = dfa.n_states
    perm = rng.permutation(n)                                          # old id -> new id
    inv = np.argsort(perm)
    trans = perm[dfa.trans[inv]].astype(np.int32)
    return DFA(trans, dfa.byte_to_class, dfa.accept[inv], dead=int(perm[dfa.dead]) if dfa.dead >= 0 else -1)


@pytest.mark.parametrize("seed", range(36))
def test_randomised_problem(gpu, oracle_mod, seed):
    """Shapes drawn at random around the limits of both walks: few or many targets per state, 1 to
    64 classes (sometimes more), empty tokens, tokens up to 32 bytes (sometimes longer), EOS
    anywhere or absent, the dead state anywhere or absent, ragged token counts.  Index, mask and
    greedy step against the oracle."""
    import torch
    rng = np.random.default_rng(7000 + seed)
    n_live = int(rng.integers(1, 240))
    n_classes = int(rng.choice([1, 2, 3, 7, 16, 33, 48, 64, 64, 64, 65, 100]))
    if seed % 3 == 0:
        dfa = W.random_dfa(rng, n_live, n_classes, float(rng.uniform(0.15, 0.95)))
    else:
        nc = min(n_classes, 64)
        dfa = few_target_dfa(rng, n_live, nc, int(rng.integers(1, 4)), float(rng.uniform(0.0, 0.7)))
    if seed % 4 == 1:
        dfa = relabel_states(rng, dfa)
    if seed % 7 == 3:                                                   # no dead state: nothing is rejected
        trans = dfa.trans.copy()
        trans[trans == dfa.dead] = 0
        dfa = DFA(trans, dfa.byte_to_class, dfa.accept, dead=-1)
    n_tokens = int(rng.choice([1, 63, 64, 65, 700, 4095, 4096, 4097, 9000, 20000]))
    cap = int(rng.choice([1, 2, 6, 12, 32, 32, 40]))
    vocab = W.bpe_like_vocab(rng, n_tokens, float(rng.uniform(1.2, 6.0)), cap)
    if seed % 5 == 2:                                                   # sprinkle empty tokens
        toks = [vocab.token(t) for t in range(n_tokens)]
        for t in rng.integers(0, n_tokens, size=max(1, n_tokens // 50)):
            toks[int(t)] = b""
        vocab = W.Vocab.from_tokens(toks)
    eos = int(rng.integers(0, n_tokens)) if seed % 2 == 0 else -1
    what = f"seed {seed}: Q={dfa.n_states} C={dfa.n_classes} N={n_tokens} cap={cap} eos={eos} dead={dfa.dead}"
    print(what, flush=True)
    ref = oracle_index(oracle_mod, dfa, vocab, eos)
    prob, csr, row_ptr, tok, nxt = gpu_index_device_flow(gpu, dfa, vocab, eos)
    assert_same_index(ref, row_ptr, tok, nxt, what)
    batch = 24
    states = rng.integers(-1, dfa.n_states + 1, size=batch).astype(np.int32)
    logits = (rng.standard_normal((batch, n_tokens)) * 3).astype(np.float32)
    want = oracle_mod.mask_logits(ref, n_tokens, states, logits)
    got = run_mask(gpu, csr, states, logits, torch.float32, bool(seed & 1))
    assert got.view(np.uint32).tobytes() == want.view(np.uint32).tobytes(), what
    bits = W.f32_to_bf16_bits(logits)
    want16 = oracle_mod.mask_logits(ref, n_tokens, states, bits)
    got16 = run_mask(gpu, without_bits(gpu, csr) if seed % 3 == 1 else csr, states, bits, torch.bfloat16, not (seed & 1))
    assert got16.tobytes() == want16.tobytes(), what
    from oracle import decode_step
    want_t, want_s = decode_step.masked_argmax(ref.row_ptr, ref.token_ids, ref.next_states, n_tokens, states, logits)
    got_t, got_s = gpu.masked_argmax(csr, torch.from_numpy(states).cuda(), torch.from_numpy(logits).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(got_t.cpu().numpy(), want_t) and np.array_equal(got_s.cpu().numpy(), want_s), what
