"""Benchmark of the FSM-index hot path on one MI355X.

One step = one pass of the whole hot path over synthetic inputs that are already resident in
HBM: build_index for the large JSON-schema automaton against the 128,256-token vocabulary
(byte classification, table preparation, counting walk, scans, emitting walk: fsmidx_build_enqueue)
followed on the same stream by mask_logits over a [256 x 128,256] batch in binary32 and in
bfloat16, and one stream synchronisation at the end of the step (fsmidx_build_finish, which reads
the build's status).  The decode-step calls
next to the mask (masked_argmax, masked_sample, advance_states) are timed on their own and reported beside the
step.  Prints ONE JSON line.

Beside the step (none of it inside the timed region): mask_logits on its own, in place and out
of place, with a plain fill of the same size as the ceiling; the decode-step calls; the build of
the 20,000-state random automaton of the last config; the index-size calls (a union of eight
schema automata built at once, identical rows kept once).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline] [--workload C3|C4b|scanner]

``--workload C4b`` is for profilers: its step is the build of the 20,000-state automaton alone;
``--workload scanner`` likewise runs the parser extension's scanner calls and the two index builds that go with them.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

LDS_PEAK_LOOKUPS = 256 * 32 * 2.4e9      # CUs x LDS banks x clock: one 4-byte bank access per lookup
HBM_PEAK = 8.0e12                        # bytes / s


def cpu_baseline(w, n_threads):
    """The CPU oracle, as it stands, on the same workload (count + fill passes, all host threads)."""
    import oracle
    oracle.build()
    d, v = w.dfa, w.vocab
    t0 = time.perf_counter()
    ref = oracle.build_index(d.trans, d.byte_to_class, d.accept, d.dead, v.bytes, v.offsets, -1, n_threads=n_threads)
    dt = time.perf_counter() - t0
    return ref, dt


KERNEL_SOURCES = ("emit.hip", "walk_sets.hip", "search.h", "walk.hip", "mask.hip", "internal.h")
VALU_PEAK_LANE_OPS = 256 * 4 * 16 * 2.4e9   # CUs x SIMDs x lanes per clock x clock


def sources_digest():
    import hashlib
    src = b"".join(open(os.path.join(ROOT, "paper_2307_09702_amd", "csrc", f), "rb").read() for f in KERNEL_SOURCES)
    return hashlib.sha256(src).hexdigest()[:16]


def recorded(path, kernel):
    """The machine-readable line of `kernel` in a committed rocprofv3 counter summary as a dict, or
    None if the kernel sources changed since the counters were taken."""
    path = os.path.join(ROOT, "profiles", path)
    if not os.path.exists(path):
        return None
    digest = sources_digest()
    for line in open(path):
        parts = dict(kv.split("=", 1) for kv in line.split() if "=" in kv)
        if parts.get("kernel") == kernel and parts.get("sources") == digest:
            return parts
    return None


def recorded_traffic(kernel, path="hbm_traffic_C3-large.md"):
    """HBM bytes per launch of `kernel` (FETCH_SIZE + WRITE_SIZE, scaled), or None."""
    parts = recorded(path, kernel)
    return int(parts["fetch_bytes"]) + int(parts["write_bytes"]) if parts else None


def recorded_lds_lookups(kernel, path="sq_counters_C3-large.md"):
    """LDS lane accesses per launch that `kernel` really issued (SQ_LDS_IDX_ACTIVE is in cycles of an
    active LDS index unit; the summary converts), or None."""
    parts = recorded(path, kernel)
    return int(parts["lds_lane_accesses"]) if parts and "lds_lane_accesses" in parts else None


def time_calls(fn, n, n_warm=4):
    """Mean milliseconds of fn(i) over n back-to-back calls (torch events on the current stream,
    which is the stream the library launches on)."""
    import torch
    for i in range(n_warm):
        fn(i)
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for i in range(n):
        fn(i)
    stop.record()
    stop.synchronize()
    return start.elapsed_time(stop) / n


def big_config_block(B, W, torch, dev, with_oracle):
    """The last config's build (20,000 random states x 128,256 tokens), timed on its own."""
    import numpy as np
    w = W.config_big_random()
    d, v = w.dfa, w.vocab
    n_pairs = d.n_states * v.n_tokens
    ref = None
    if with_oracle:
        import oracle
        t0 = time.perf_counter()
        ref = oracle.build_index(d.trans, d.byte_to_class, d.accept, d.dead, v.bytes, v.offsets, -1,
                                 n_threads=len(os.sched_getaffinity(0)))
        oracle_s = time.perf_counter() - t0
    prob = B.DeviceProblem(d.trans, d.byte_to_class, d.accept, d.dead, v.bytes, v.offsets, -1)
    nnz = prob.count()
    tok = torch.empty(nnz, dtype=torch.int32, device=dev)
    nxt = torch.empty(nnz, dtype=torch.int32, device=dev)
    for _ in range(2):
        prob.build_into(tok, nxt)
    torch.cuda.synchronize()
    n = 5
    t0 = time.perf_counter()
    for _ in range(n):
        prob.build_into(tok, nxt)
    torch.cuda.synchronize()
    build_ms = (time.perf_counter() - t0) / n * 1e3
    B.profile_enable(True)
    for _ in range(n):
        prob.build_into(tok, nxt)
    torch.cuda.synchronize()
    prof = B.profile_read()
    B.profile_enable(False)
    ms = {k: prof[k][0] for k in ("prepare", "count_walk", "scan", "emit_walk")}
    out = {"workload": "C4b-big: random automaton, 20,000 states + dead, 64 classes, density 0.3, x the 128,256-token "
                       "vocabulary", "n_states": d.n_states, "pairs": n_pairs, "nnz": nnz, "build_ms": build_ms,
           "pairs_per_s": n_pairs / (build_ms * 1e-3), "kernels_ms": ms,
           "emit_hbm_frac": nnz * 8 / (ms["emit_walk"] * 1e-3) / HBM_PEAK}
    if ref is not None:
        same = np.array_equal(prob.row_ptr.cpu().numpy(), ref.row_ptr)
        step = 1 << 25
        for a in range(0, nnz, step):
            same = same and np.array_equal(tok[a:a + step].cpu().numpy(), ref.token_ids[a:a + step]) \
                and np.array_equal(nxt[a:a + step].cpu().numpy(), ref.next_states[a:a + step])
        assert same, "GPU index of the 20,000-state config differs from the oracle"
        out.update({"W_bf": ref.w_bf, "bytes_walked_per_s": ref.w_bf / (build_ms * 1e-3),
                    "walk_lds_frac_effective": ref.w_bf / (ms["count_walk"] * 1e-3) / LDS_PEAK_LOOKUPS,
                    "build_lds_frac_effective": ref.w_bf / (build_ms * 1e-3) / LDS_PEAK_LOOKUPS,
                    "bit_exact_vs_oracle": True,
                    "cpu_oracle": {"pairs_per_s": n_pairs / oracle_s, "seconds": oracle_s,
                                   "cores": len(os.sched_getaffinity(0))}})
    del prob, tok, nxt
    torch.cuda.empty_cache()
    return out


def scanner_block(B, W, torch, dev, with_oracle):
    """Scanner step of parser-guided generation (Section 4, 4.1) on a seeded toy grammar: terminal
    sets and the restart table for 2,000 parse states, and the index of 400 parse states' scanners,
    with and without restarts, against the large vocabulary."""
    import numpy as np
    from paper_2307_09702_amd.synth import grammar as G

    def timed(fn, n=5):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            out = fn()
        torch.cuda.synchronize()
        return out, (time.perf_counter() - t0) / n * 1e3

    sc = G.toy_grammar(W.rng_for(12, 0), 2000)
    d = sc.dfa
    dev_sc = B.DeviceScanner(d.trans, d.dead, sc.completes, sc.scanner_of_state, sc.shift)
    (sets, launches), sets_ms = timed(dev_sc.terminal_sets)
    table, table_ms = timed(dev_sc.restart_table)
    entries = d.n_states * d.n_classes
    out = {"grammar": "seeded toy grammar: %d terminals, every parse state reads whitespace and 3 to 12 others; shifts drawn "
                      "uniformly" % sc.n_terminals,
           "kernels": {"parse_states": 2000, "states": d.n_states, "classes": d.n_classes,
                       "terminal_sets_call_ms_host_clock": sets_ms, "terminal_sets_launches": launches,
                       "restart_table_call_ms_host_clock": table_ms,
                       "restart_table_bytes": entries * 8, "entries_rejecting_before": int((d.trans == d.dead).sum())}}
    if with_oracle:
        from oracle import scanner as S
        t0 = time.perf_counter()
        want_v = S.terminal_sets(d.trans, sc.completes)
        want_t = S.restart_table(d.trans, d.dead, sc.completes, sc.scanner_of_state, sc.shift)
        oracle_s = time.perf_counter() - t0
        assert np.array_equal(sets.cpu().numpy().view(np.uint64), want_v), "terminal sets differ from the oracle"
        assert np.array_equal(table.cpu().numpy(), want_t), "restart table differs from the oracle"
        out["kernels"].update({"bit_exact_vs_oracle": True, "cpu_oracle_seconds": oracle_s,
                               "entries_restarted": int((want_t != d.trans).sum())})
    del dev_sc, sets, table
    sc = G.toy_grammar(W.rng_for(12, 1), 400)
    d = sc.dfa
    vocab = W.large_vocab()
    dev_sc = B.DeviceScanner(d.trans, d.dead, sc.completes, sc.scanner_of_state, sc.shift)
    table = dev_sc.restart_table()
    b2c = torch.from_numpy(d.byte_to_class).to(dev)
    acc = torch.from_numpy(d.accept).to(dev)
    built = {}
    for name, trans in (("scanners_as_given", dev_sc.trans), ("with_restarts", table)):
        prob = B.DeviceProblem(trans, b2c, acc, d.dead, vocab.bytes, vocab.offsets, -1)
        nnz = prob.count()
        tok = torch.empty(max(nnz, 1), dtype=torch.int32, device=dev)
        nxt = torch.empty(max(nnz, 1), dtype=torch.int32, device=dev)
        _, ms = timed(lambda: prob.build_into(tok, nxt), n=10)
        built[name] = {"nnz": nnz, "build_ms": ms, "pairs_per_s": d.n_states * vocab.n_tokens / (ms * 1e-3)}
        del prob, tok, nxt
    out["index"] = {"parse_states": 400, "states": d.n_states, "classes": d.n_classes, "vocabulary": vocab.n_tokens,
                    "pairs": d.n_states * vocab.n_tokens, **built}
    torch.cuda.empty_cache()
    return out


def reduce_block(B, W, torch, dev, csr_large, n_states_large, nnz_large):
    """Index size (Section 5): eight schema automata in one build against one vocabulary, and
    identical rows kept once."""
    import numpy as np
    from paper_2307_09702_amd.synth.regex_dfa import compile_regex
    autos = []
    for k in range(8):
        rng = np.random.default_rng([2, k])
        d = compile_regex(W.json_schema_regex(rng, 8, nested=False))
        autos.append((d.trans, d.byte_to_class, d.accept, d.dead))
    vocab = W.config_json().vocab

    def build_time(trans, b2c, accept, dead, n=10):
        prob = B.DeviceProblem(trans, b2c, accept, dead, vocab.bytes, vocab.offsets, -1)
        nnz = prob.count()
        tok = torch.empty(nnz, dtype=torch.int32, device=dev)
        nxt = torch.empty(nnz, dtype=torch.int32, device=dev)
        for _ in range(3):
            prob.build_into(tok, nxt)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            prob.build_into(tok, nxt)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n * 1e3, nnz, prob, (tok, nxt)

    t0 = time.perf_counter()
    u = B.DeviceUnion(autos)
    torch.cuda.synchronize()
    union_call_ms = (time.perf_counter() - t0) * 1e3
    one_ms, union_nnz, prob, keep = build_time(u.trans, u.byte_to_class, u.accept, u.dead_state)
    separate = [build_time(*a)[:2] for a in autos]
    csr_u = prob.csr(union_nnz, keep[0], keep[1])
    t0 = time.perf_counter()
    row_of, urp, tok_u, nxt_u = B.dedupe_rows(csr_u)
    dedupe_union_ms = (time.perf_counter() - t0) * 1e3
    t0 = time.perf_counter()
    row_of_l, urp_l, tok_l, nxt_l = B.dedupe_rows(csr_large)
    dedupe_large_ms = (time.perf_counter() - t0) * 1e3
    # reachable-only index (Section 3, the remark after Algorithm 4): the large config from its start
    # state, with its whole vocabulary and with one that has no one-letter and one-digit tokens
    def reachable(csr, start, n=5):
        reach, n_reached = B.reachable_states(csr, [start])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            reach, n_reached = B.reachable_states(csr, [start])
        reach_ms = (time.perf_counter() - t0) / n * 1e3
        t0 = time.perf_counter()
        ptr, tok_r, nxt_r = B.restrict_rows(csr, reach)
        restrict_ms = (time.perf_counter() - t0) * 1e3
        return {"states": int(csr.n_states), "reachable": n_reached, "entries": int(csr.nnz), "entries_kept": int(tok_r.numel()),
                "reachable_states_call_ms_host_clock": reach_ms, "restrict_calls_ms_host_clock": restrict_ms}
    large = W.config_large()
    reach_large = reachable(csr_large, large.dfa.start)
    lens = np.diff(large.vocab.offsets)
    first = large.vocab.bytes[np.minimum(large.vocab.offsets[:-1], large.vocab.bytes.size - 1)]
    alnum = np.isin(first, np.frombuffer(b"abcdefghijklmnopqrstuvwxyzABCDEFGHIJKLMNOPQRSTUVWXYZ0123456789", np.uint8))
    some = W.Vocab.from_tokens([large.vocab.token(t) for t in np.flatnonzero((lens >= 2) | ((lens == 1) & ~alnum))])
    prob_s = B.DeviceProblem(large.dfa.trans, large.dfa.byte_to_class, large.dfa.accept, large.dfa.dead, some.bytes,
                             some.offsets, -1)
    csr_s, tok_s, nxt_s = prob_s.build()
    reach_some = reachable(csr_s, large.dfa.start)
    reach_some["vocabulary"] = "C3-large's tokens without the one-letter and one-digit ones (%d tokens)" % some.n_tokens
    # minimisation before indexing (Section 5): the union of the eight automata (states that read
    # the same continuations in different automata fall together), and one automaton un-reduced
    def minimised(trans, b2c, accept, dead, n=5):
        m = B.DeviceMinimised(trans, b2c, accept, dead)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            m = B.DeviceMinimised(trans, b2c, accept, dead)
        torch.cuda.synchronize()
        call_ms = (time.perf_counter() - t0) / n * 1e3
        pm = B.DeviceProblem(m.trans, m.byte_to_class, m.accept, m.dead_state, vocab.bytes, vocab.offsets, -1)
        return m, {"states": int(trans.shape[0]), "classes_of_equivalent_states": m.n_states, "entries_after": pm.count(),
                   "call_ms_host_clock": call_ms}
    _, min_union = minimised(u.trans, u.byte_to_class, u.accept, u.dead_state)
    min_union["entries_before"] = union_nnz
    raw = compile_regex(W.json_schema_regex(np.random.default_rng([2, 0]), 8, nested=False), minimise=False)
    _, min_raw = minimised(raw.trans, raw.byte_to_class, raw.accept, raw.dead)
    min_raw["entries_before"] = B.DeviceProblem(raw.trans, raw.byte_to_class, raw.accept, raw.dead, vocab.bytes,
                                                vocab.offsets, -1).count()
    return {
        "minimise": {"union_of_eight": min_union, "one_schema_automaton_as_the_subset_construction_leaves_it": min_raw},
        "reachable_only": {"C3-large": reach_large, "C3-large, no one-character alphanumeric tokens": reach_some},
        "union": {"automata": 8, "states": u.n_states, "classes": u.n_classes, "vocabulary": vocab.n_tokens,
                  "pairs": u.n_states * vocab.n_tokens, "nnz": union_nnz, "fsmidx_union_dfa_ms_host_clock": union_call_ms,
                  "one_build_ms": one_ms, "eight_builds_one_after_the_other_ms": sum(t for t, _ in separate),
                  "pairs_per_s": u.n_states * vocab.n_tokens / (one_ms * 1e-3)},
        "dedupe": {"union_of_eight": {"states": u.n_states, "distinct_rows": int(urp.numel() - 1), "entries": union_nnz,
                                      "entries_kept": int(tok_u.numel()), "call_ms_host_clock": dedupe_union_ms},
                   "C3-large": {"states": n_states_large, "distinct_rows": int(urp_l.numel() - 1), "entries": nnz_large,
                                "entries_kept": int(tok_l.numel()), "call_ms_host_clock": dedupe_large_ms,
                                "note": "the generator's automaton is minimal, so only the two empty rows coincide"}},
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true",
                    help="skip the oracle legs (the roofline then uses the pair count as work)")
    ap.add_argument("--step-only", action="store_true",
                    help="for profilers: leave out what is timed beside the step (other configs, index-size calls), so "
                         "that every kernel name in a trace belongs to the step's workload")
    ap.add_argument("--in-flight", type=int, default=1, choices=(1, 2, 3, 4),
                    help="steps under way at a time in the timed region, each on its own stream, workspace and output "
                         "arrays (the default run also times two in flight, beside the headline)")
    ap.add_argument("--workload", default="C3", choices=("C3", "C4b", "scanner"),
                    help="for profilers. C4b: only the build of the 20,000-state automaton; scanner: only the scanner "
                         "step of the parser extension")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this path runs on exactly one GPU (one process, no collectives); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2307_09702_amd import binding as B
    from paper_2307_09702_amd.synth import workloads as W

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    B.load()

    if args.workload == "C4b":
        out = big_config_block(B, W, torch, dev, with_oracle=False)
        print(json.dumps({"metric": "(state,token) pairs indexed/sec", "value": out["pairs_per_s"], "unit": "pairs/s",
                          "n_gpus": 1, "config": out}))
        return

    if args.workload == "scanner":
        out = scanner_block(B, W, torch, dev, with_oracle=False)
        print(json.dumps({"metric": "(state,token) pairs indexed/sec", "value": out["index"]["with_restarts"]["pairs_per_s"],
                          "unit": "pairs/s", "n_gpus": 1, "config": out}))
        return

    w = W.config_large()
    d, v = w.dfa, w.vocab
    n_pairs = d.n_states * v.n_tokens
    print(f"[bench] workload {w.name}: Q={d.n_states} C={d.n_classes} N={v.n_tokens} bytes={v.bytes.size} "
          f"pairs={n_pairs}", file=sys.stderr, flush=True)

    ref, cpu = None, None
    if not args.no_cpu_baseline:
        n_threads = len(os.sched_getaffinity(0))
        ref, cpu_s = cpu_baseline(w, n_threads)
        cpu = {"value": n_pairs / cpu_s, "unit": "pairs/s", "cores": n_threads, "kind": "oracle",
               "sample": f"the whole workload once (count pass + fill pass over all {n_pairs} pairs), "
                         f"{cpu_s:.2f} s wall on {n_threads} threads"}
        print(f"[bench] oracle: {cpu_s:.2f} s on {n_threads} threads, W_bf={ref.w_bf} nnz={ref.nnz}",
              file=sys.stderr, flush=True)

    prob = B.DeviceProblem(d.trans, d.byte_to_class, d.accept, d.dead, v.bytes, v.offsets, -1)
    nnz = prob.count()
    token_ids = torch.empty(nnz, dtype=torch.int32, device=dev)
    next_states = torch.empty(nnz, dtype=torch.int32, device=dev)
    prob.fill(nnz, token_ids, next_states)
    torch.cuda.synchronize()
    csr = prob.csr(nnz, token_ids, next_states)
    if ref is not None:
        same = (np.array_equal(prob.row_ptr.cpu().numpy(), ref.row_ptr)
                and np.array_equal(token_ids.cpu().numpy(), ref.token_ids)
                and np.array_equal(next_states.cpu().numpy(), ref.next_states))
        assert same, "GPU index differs from the oracle"

    states_np, logits_np = W.decode_batch(d.n_states, d.dead, v.n_tokens)
    states = torch.from_numpy(states_np).to(dev)
    n_rot = 4                                   # rotate buffers so the 256 MB last-level cache cannot hold them
    base32 = torch.from_numpy(logits_np).to(dev)
    logits32 = [base32.clone() for _ in range(n_rot)]
    logits16 = [base32.to(torch.bfloat16) for _ in range(n_rot)]
    row_nnz = np.diff(prob.row_ptr.cpu().numpy())[states_np]
    kept = int(row_nnz.sum())
    batch, n_vocab = logits_np.shape

    # A step: the whole build enqueued at once (the arrays are known to be large enough from the
    # first build), the two masks that use the index behind it on the same stream, and one wait at
    # the end of the step: build_finish reads the build's status there and would say so if the
    # counting pass had to be redone (then the masks would have to be enqueued again: not here).
    # Steps are independent of each other, so several can be under way at a time, each on a stream,
    # a workspace and output arrays of its own: the preparation and the scans of one step are single
    # workgroups waiting for memory, and run beside the emit pass and the masks of the step before,
    # which fill the chip.  The headline is measured one step at a time (`--in-flight 1`, so that a
    # kernel's duration is its own); two in flight are timed beside it.
    class Slot:
        def __init__(self, problem, tok, nxt, view):
            self.prob, self.tok, self.nxt, self.csr = problem, tok, nxt, view
            self.stream = torch.cuda.Stream()

        def enqueue(self, i):
            self.prob.build_enqueue(self.tok, self.nxt, stream=self.stream)
            B.mask_logits(self.csr, states, logits32[i % n_rot], stream=self.stream)
            B.mask_logits(self.csr, states, logits16[i % n_rot], stream=self.stream)

        def finish(self):
            got, redone = self.prob.build_finish(self.tok, self.nxt, stream=self.stream)
            assert got == nnz and not redone

    slots = [Slot(prob, token_ids, next_states, csr)]
    most_in_flight = args.in_flight if args.step_only else max(args.in_flight, 2)
    for _ in range(1, most_in_flight):
        p2 = B.DeviceProblem(d.trans, d.byte_to_class, d.accept, d.dead, v.bytes, v.offsets, -1)
        assert p2.count() == nnz
        t2 = torch.empty(nnz, dtype=torch.int32, device=dev)
        n2 = torch.empty(nnz, dtype=torch.int32, device=dev)
        slots.append(Slot(p2, t2, n2, p2.csr(nnz, t2, n2)))

    def run_steps(n_steps, in_flight):
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        for i in range(n_steps):
            slot = slots[i % in_flight]
            if i >= in_flight:
                slot.finish()
            slot.enqueue(i)
        for i in range(max(n_steps - in_flight, 0), n_steps):
            slots[i % in_flight].finish()
        torch.cuda.synchronize()
        return time.perf_counter() - t_start

    def profiled(in_flight):
        # per-kernel durations from an untimed pass: the events that bracket the phases put gaps
        # between the kernels, so they stay out of the timed steps
        B.profile_enable(True)
        run_steps(args.steps, in_flight)
        out = B.profile_read()
        B.profile_enable(False)
        return out

    run_steps(args.warmup, args.in_flight)
    elapsed = run_steps(args.steps, args.in_flight)
    prof = profiled(args.in_flight)
    # the same steps with two under way, for comparison
    piped = None
    if most_in_flight > args.in_flight:
        run_steps(min(args.warmup, 4), most_in_flight)
        piped_elapsed = run_steps(args.steps, most_in_flight)
        piped = {"steps_in_flight": most_in_flight, "ms_per_step": piped_elapsed / args.steps * 1e3,
                 "value": n_pairs / (piped_elapsed / args.steps),
                 "note": "the same steps, the next one enqueued on a second stream (own workspace and output arrays) "
                         "before the one before it has been waited for; its preparation and scans run beside the "
                         "other's emit pass and masks"}
    if ref is not None and most_in_flight > 1:
        for slot in slots[1:]:              # the other slots' indices are the same index
            assert np.array_equal(slot.prob.row_ptr.cpu().numpy(), ref.row_ptr)
            assert np.array_equal(slot.tok.cpu().numpy(), ref.token_ids) and np.array_equal(slot.nxt.cpu().numpy(), ref.next_states)

    # mask_logits on its own: 200 launches back to back per dtype over the rotating buffers, HIP
    # events on the launching stream around the lot (a decode step calls the mask without a build
    # in front of it; inside a step the mask also pays for the write-back of the build's output)
    def alone(buffers, n=200):
        return time_calls(lambda i: B.mask_logits(csr, states, buffers[i % n_rot]), n)
    alone_ms = {4: alone(logits32), 2: alone(logits16)}
    # out of place (every element written, kept ones read), into a second set of rotating buffers;
    # and the ceiling of this part for a kernel that only writes: a plain fill of the same buffers
    out32 = [torch.empty_like(base32) for _ in range(n_rot)]
    out16 = [torch.empty_like(logits16[0]) for _ in range(n_rot)]
    oop_ms = {4: time_calls(lambda i: B.mask_logits(csr, states, logits32[i % n_rot], out32[i % n_rot]), 200),
              2: time_calls(lambda i: B.mask_logits(csr, states, logits16[i % n_rot], out16[i % n_rot]), 200)}
    fill_ms = {4: time_calls(lambda i: out32[i % n_rot].fill_(0.0), 200),
               2: time_calls(lambda i: out16[i % n_rot].fill_(0.0), 200)}
    del out32, out16
    mask_traffic = {4: recorded_traffic("mask_rows_bits_f32"), 2: recorded_traffic("mask_rows_bits_bf16")}

    # The decode-step neighbours of the mask (not part of a step; reported beside it): the greedy
    # choice under the mask reads only the rows' entries, and advance_states is one search per row.
    def alone_call(fn, n=200):
        return time_calls(fn, n)
    argmax_ws = torch.empty(B.masked_argmax_workspace_bytes(batch), dtype=torch.uint8, device=dev)
    picked = torch.empty_like(states)
    moved = torch.empty_like(states)
    argmax_ms = {e: alone_call(lambda i, buf=buf: B.masked_argmax(csr, states, buf[i % n_rot], workspace=argmax_ws,
                                                                  tokens_out=picked, states_out=moved))
                 for e, buf in ((4, logits32), (2, logits16))}
    advance_ms = alone_call(lambda i: B.advance_states(csr, states, picked, states_out=moved))
    sample_ws = torch.empty(B.masked_sample_workspace_bytes(batch), dtype=torch.uint8, device=dev)
    uniforms_np = W.rng_for(4, W.STREAM_STATES + 10).random(batch, dtype=np.float32)
    uniforms = torch.from_numpy(uniforms_np).to(dev)
    sample_ms = {e: alone_call(lambda i, buf=buf: B.masked_sample(csr, states, buf[i % n_rot], uniforms, workspace=sample_ws,
                                                                  tokens_out=picked, states_out=moved))
                 for e, buf in ((4, logits32), (2, logits16))}
    # the same calls bracketed by the library's HIP events (the back-to-back figures above are bound
    # by the host's launch rate when a call's kernels are shorter than that)
    B.profile_enable(True)
    for i in range(50):
        B.masked_argmax(csr, states, logits32[i % n_rot], workspace=argmax_ws, tokens_out=picked, states_out=moved)
        B.masked_argmax(csr, states, logits16[i % n_rot], workspace=argmax_ws, tokens_out=picked, states_out=moved)
        B.advance_states(csr, states, picked, states_out=moved)
        B.masked_sample(csr, states, logits32[i % n_rot], uniforms, workspace=sample_ws, tokens_out=picked, states_out=moved)
        B.masked_sample(csr, states, logits16[i % n_rot], uniforms, workspace=sample_ws, tokens_out=picked, states_out=moved)
    torch.cuda.synchronize()
    decode_prof = B.profile_read()
    B.profile_enable(False)
    decode_exact, decode_cpu, sample_same = None, None, None
    if ref is not None:
        from oracle import decode_step as D
        B.masked_argmax(csr, states, base32, workspace=argmax_ws, tokens_out=picked, states_out=moved)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        want_t, want_s = D.masked_argmax(ref.row_ptr, ref.token_ids, ref.next_states, n_vocab, states_np, logits_np)
        decode_cpu = time.perf_counter() - t0
        decode_exact = bool(np.array_equal(picked.cpu().numpy(), want_t) and np.array_equal(moved.cpu().numpy(), want_s))
        assert decode_exact, "masked_argmax differs from the oracle"
        # draws: equal to the oracle's except where the threshold lies within rounding of a boundary
        # between two entries (the parity tests check those cases one by one)
        B.masked_sample(csr, states, base32, uniforms, workspace=sample_ws, tokens_out=picked, states_out=moved)
        torch.cuda.synchronize()
        want_t, want_s = D.masked_sample(ref.row_ptr, ref.token_ids, ref.next_states, n_vocab, states_np, logits_np,
                                         uniforms_np)
        sample_same = int((picked.cpu().numpy() == want_t).sum())
        assert sample_same >= batch - 2, "masked_sample differs from the oracle in more than two draws"
    # per call: the rows' token ids and the logits they point at, states in, (token, state) out
    argmax_bytes = {e: kept * (4 + e) + batch * (4 + 16 + 8) for e in (4, 2)}

    ms_per_step = elapsed / args.steps * 1e3
    ms = {k: prof[k][0] for k in prof if prof[k][1] > 0}
    build_ms = ms["prepare"] + ms["count_walk"] + ms["scan"] + ms["emit_walk"]
    work = ref.w_bf if ref is not None else n_pairs
    emit_s = ms["emit_walk"] * 1e-3
    # in-place masking writes -inf over every removed element and reads one bitmap bit per element
    mask_bytes = {e: (batch * n_vocab - kept) * e + batch * n_vocab // 8 for e in (4, 2)}
    oop_bytes = {e: batch * n_vocab * e + kept * e + batch * n_vocab // 8 for e in (4, 2)}
    big = None if args.step_only else big_config_block(B, W, torch, dev, with_oracle=ref is not None)
    reduced = None if args.step_only else reduce_block(B, W, torch, dev, csr, d.n_states, nnz)
    scanned = None if args.step_only else scanner_block(B, W, torch, dev, with_oracle=ref is not None)

    # The two heavy kernels of the build and what bounds each:
    #  - the counting walk decides all pairs: transition lookups of the early-exit walk (W_bf, from
    #    the oracle), one 4-byte LDS bank access each, against 256 CUs x 32 banks x 2.4 GHz;
    #  - the emit kernel writes 8 bytes per entry of the CSR: HBM.
    issued = recorded_lds_lookups("walk_sets")
    count_roof = {
        "kernel": "walk_sets (counting walk)", "bound": "lds",
        "achieved": work * 4 / (ms["count_walk"] * 1e-3) / 1e9,
        "peak": LDS_PEAK_LOOKUPS * 4 / 1e9, "unit": "GB/s",
        "frac": work / (ms["count_walk"] * 1e-3) / LDS_PEAK_LOOKUPS, "traffic": recorded_traffic("walk_sets"),
        "frac_kind": "effective: W_bf (the early-exit walk's lookups, from the oracle) over this kernel's time",
        "frac_issued": issued / (ms["count_walk"] * 1e-3) / LDS_PEAK_LOOKUPS if issued else None,
        "issued_lds_lane_accesses": issued,
        "note": "algorithmic work = W_bf lookups x 4 B; the kernel decides whole token sets with bitmap ANDs and "
                "never issues most of these lookups, so `frac` is an effective rate; `frac_issued` is what its LDS "
                "instructions really moved (rocprofv3 counters, profiles/sq_counters_C3-large.md)",
    }
    emit_bytes = nnz * 8
    emit_roof = {
        "kernel": "emit_csr (emit pass: search for long row segments, table walk for the rest)", "bound": "hbm",
        "achieved": emit_bytes / emit_s / 1e9, "peak": HBM_PEAK / 1e9, "unit": "GB/s",
        "frac": emit_bytes / emit_s / HBM_PEAK, "traffic": recorded_traffic("emit_csr"),
        "note": f"algorithmic bytes = 8 B x {nnz} entries (token id + end state)",
    }
    dominant, other = (emit_roof, count_roof) if ms["emit_walk"] >= ms["count_walk"] else (count_roof, emit_roof)
    out = {
        "metric": "(state,token) pairs indexed/sec + mask_logits GB/s, fraction of roofline",
        "value": n_pairs / (elapsed / args.steps),
        "unit": "pairs/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32 index built with u64 bitmap and u16 table arithmetic; f32/bf16 logits moved as raw bits",
        "data": "synthetic",
        "config": {"workload": "C3-large: seeded 40-field nested JSON-schema DFA x 128,256-token BPE-like vocabulary "
                               "(build_index) + 256 x 128,256 decode batch (mask_logits f32 and bf16, in place)",
                   "n_states": d.n_states, "n_classes": d.n_classes, "n_tokens": v.n_tokens,
                   "vocab_bytes": int(v.bytes.size), "pairs": n_pairs, "nnz": nnz,
                   "W_bf": ref.w_bf if ref else None, "W_inv": ref.w_inv if ref else None,
                   "mask_batch": batch, "steps_in_flight": args.in_flight},
        "roofline": dominant,
        "roofline_second_kernel": other,
        "kernels_ms": ms,
        "pipelined": piped,
        "build": {"ms": build_ms, "pairs_per_s": n_pairs / (build_ms * 1e-3),
                  "lookups_per_s": work / (build_ms * 1e-3),
                  "bytes_walked_per_s": work / (build_ms * 1e-3),
                  "lds_frac_effective": work / (build_ms * 1e-3) / LDS_PEAK_LOOKUPS,
                  "emit_GBps": (nnz * 8 + (d.n_states + 1) * 8) / emit_s / 1e9,
                  "roofline_time_ms": max(work / LDS_PEAK_LOOKUPS, (nnz * 8 + (d.n_states + 1) * 8) / HBM_PEAK) * 1e3,
                  "frac_of_roofline_time": max(work / LDS_PEAK_LOOKUPS, (nnz * 8 + (d.n_states + 1) * 8) / HBM_PEAK)
                  * 1e3 / build_ms,
                  "note": "the whole build against max(walk at the LDS rate, output at the HBM rate); the target of "
                          "half the LDS-bound walk rate for the build as a whole is not met"},
        "configs": {"C4b-big": big},
        "index_size": reduced,
        "parser_scanner": scanned,
        "mask": {
            "mode": "in place, 4 rotating buffers per dtype",
            "algorithmic_bytes": "removed entries x element size + one bitmap bit per element",
            "out_of_place": {
                "algorithmic_bytes": "every element written + kept elements read + one bitmap bit per element",
                "f32": {"back_to_back_ms": oop_ms[4], "hbm_frac": oop_bytes[4] / (oop_ms[4] * 1e-3) / HBM_PEAK},
                "bf16": {"back_to_back_ms": oop_ms[2], "hbm_frac": oop_bytes[2] / (oop_ms[2] * 1e-3) / HBM_PEAK}},
            "fill_of_the_same_buffers": {
                "note": "a plain fill (torch) of the same rotating buffers in the same run: what a kernel that only "
                        "writes reaches on this part",
                "f32": {"back_to_back_ms": fill_ms[4], "hbm_frac": batch * n_vocab * 4 / (fill_ms[4] * 1e-3) / HBM_PEAK},
                "bf16": {"back_to_back_ms": fill_ms[2], "hbm_frac": batch * n_vocab * 2 / (fill_ms[2] * 1e-3) / HBM_PEAK}},
            "f32": {"back_to_back_ms": alone_ms[4], "GBps": mask_bytes[4] / (alone_ms[4] * 1e-3) / 1e9,
                    "hbm_frac": mask_bytes[4] / (alone_ms[4] * 1e-3) / HBM_PEAK,
                    "in_step_ms": ms["mask_f32"], "in_step_hbm_frac": mask_bytes[4] / (ms["mask_f32"] * 1e-3) / HBM_PEAK,
                    "traffic": mask_traffic[4]},
            "bf16": {"back_to_back_ms": alone_ms[2], "GBps": mask_bytes[2] / (alone_ms[2] * 1e-3) / 1e9,
                     "hbm_frac": mask_bytes[2] / (alone_ms[2] * 1e-3) / HBM_PEAK,
                     "in_step_ms": ms["mask_bf16"], "in_step_hbm_frac": mask_bytes[2] / (ms["mask_bf16"] * 1e-3) / HBM_PEAK,
                     "traffic": mask_traffic[2]},
        },
        "decode_step": {
            "note": "next to the mask, outside the timed step: greedy choice and sampling under the mask over the rows' "
                    "entries only, and state tracking; 200 launches back to back each; algorithmic bytes count the rows' "
                    "entries once (token id + logit), whatever passes a kernel makes",
            "entries_read": kept, "of_logits": batch * n_vocab,
            "masked_argmax_f32": {"back_to_back_ms": argmax_ms[4], "kernels_ms": decode_prof["masked_argmax_f32"][0],
                                  "algorithmic_bytes": argmax_bytes[4],
                                  "hbm_frac": argmax_bytes[4] / (decode_prof["masked_argmax_f32"][0] * 1e-3) / HBM_PEAK},
            "masked_argmax_bf16": {"back_to_back_ms": argmax_ms[2], "kernels_ms": decode_prof["masked_argmax_bf16"][0],
                                   "algorithmic_bytes": argmax_bytes[2],
                                   "hbm_frac": argmax_bytes[2] / (decode_prof["masked_argmax_bf16"][0] * 1e-3) / HBM_PEAK},
            "advance_states": {"back_to_back_ms": advance_ms, "kernels_ms": decode_prof["advance_states"][0]},
            "masked_sample_f32": {"back_to_back_ms": sample_ms[4], "kernels_ms": decode_prof["masked_sample_f32"][0],
                                  "algorithmic_bytes": argmax_bytes[4],
                                  "hbm_frac": argmax_bytes[4] / (decode_prof["masked_sample_f32"][0] * 1e-3) / HBM_PEAK},
            "masked_sample_bf16": {"back_to_back_ms": sample_ms[2], "kernels_ms": decode_prof["masked_sample_bf16"][0],
                                   "algorithmic_bytes": argmax_bytes[2],
                                   "hbm_frac": argmax_bytes[2] / (decode_prof["masked_sample_bf16"][0] * 1e-3) / HBM_PEAK},
            "masked_sample_draws_equal_to_oracle": sample_same,
            "cpu_oracle_masked_argmax_s": decode_cpu, "bit_exact_vs_oracle": decode_exact,
        },
        "cpu_baseline": cpu,
        "bit_exact_vs_oracle": True if ref is not None else None,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
