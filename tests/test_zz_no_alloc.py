"""fsmidx_masked_argmax_static (the entry point that allocates nothing) against
fsmidx_masked_argmax through the C ABI: two calls in a row, the second with a smaller input."""
import numpy as np
import pytest

from paper_2307_09702_amd.synth import workloads as W

pytestmark = pytest.mark.gpu


def test_static_scratch_argmax_equals_the_workspace_form(oracle_mod):
    import torch
    from oracle import decode_step
    from paper_2307_09702_amd import binding as B
    assert torch.cuda.is_available(), "this test needs the MI355X"
    B.load()
    w = W.config_json()
    d, v = w.dfa, w.vocab
    ref = oracle_mod.build_index(d.trans, d.byte_to_class, d.accept, d.dead, v.bytes, v.offsets, 7, n_threads=8)
    prob = B.DeviceProblem(d.trans, d.byte_to_class, d.accept, d.dead, v.bytes, v.offsets, 7)
    csr, tok, nxt = prob.build()
    torch.cuda.synchronize()
    rng = np.random.default_rng(11)
    for round_no, batch in enumerate((300, 37)):                      # the second call is the smaller one
        print(f"static argmax: call {round_no}, batch {batch}", flush=True)
        states_np = rng.integers(-1, d.n_states + 1, size=batch).astype(np.int32)
        logits_np = (rng.standard_normal((batch, v.n_tokens)) * 3).astype(np.float32)
        states = torch.from_numpy(states_np).cuda()
        want_t, want_s = decode_step.masked_argmax(ref.row_ptr, ref.token_ids, ref.next_states, v.n_tokens, states_np,
                                                   logits_np)
        for logits in (torch.from_numpy(logits_np).cuda(), torch.from_numpy(logits_np).cuda().to(torch.bfloat16)):
            t0, s0 = B.masked_argmax(csr, states, logits)
            t1 = torch.full((batch,), -5, dtype=torch.int32, device="cuda")
            s1 = torch.full((batch,), -5, dtype=torch.int32, device="cuda")
            B.masked_argmax_static(csr, states, logits, t1, s1)
            torch.cuda.synchronize()
            assert torch.equal(t0, t1) and torch.equal(s0, s1), (round_no, logits.dtype)
            if logits.dtype == torch.float32:
                assert np.array_equal(t1.cpu().numpy(), want_t) and np.array_equal(s1.cpu().numpy(), want_s)
    # beyond the fixed array: refused, nothing launched
    big = torch.zeros(4097, dtype=torch.int32, device="cuda")
    out = torch.zeros(4097, dtype=torch.int32, device="cuda")
    with pytest.raises(B.FsmidxError) as err:
        B.masked_argmax_static(csr, big, torch.zeros(1, v.n_tokens, device="cuda"), out, out, row_stride=v.n_tokens)
    assert err.value.code == B.INVALID_ARG and "4096" in str(err.value)
