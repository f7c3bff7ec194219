/*
 * CPU oracle for FSM vocabulary indexing and logit masking.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition that the GPU library's results are compared with.
 * It is used by the tests, by the smoke check and by the benchmark's CPU-baseline leg and by
 * nothing else; it shares no code, header or table with the GPU path.
 *
 * What it computes (Willard & Louf, "Efficient Guided Generation for Large Language Models"):
 *
 *  - Section 3, Algorithm 3 (find_sub_sequences): for a vocabulary string v and a start state
 *    q, walk the automaton's transition function over the characters of v; the walk is
 *    dropped as soon as the automaton cannot read a character.  The printed listing starts
 *    its inner loop at the second character; the worked examples (the float example of
 *    Section 3 and the "f" example of Section 4, whose state sequences have |v|+1 entries)
 *    fix the reading used here: every character of v, the first included, is applied to the
 *    state, so the sequence is (q, delta(q,v0), ..., delta*(q,v)).  Looping over all q instead
 *    of only the states that read v0 gives the same result, because a q that does not read
 *    v0 fails on the first character.
 *  - Section 3, Algorithm 4 (map_states_to_vocab): sigma(q) collects every v whose walk from
 *    q survives.  sigma(q) is a set; it is emitted here in ascending token id.
 *  - Section 3, the paragraph before the worked example: the state in which the walk stops is
 *    kept next to the token, so that generation resumes from it.
 *  - Section 2.2, the masking equation and Algorithm 2: the mask of state q keeps the tokens of
 *    sigma(q) and removes all others; on logits, "remove" is -inf and "keep" is a bit copy.
 *
 * Readings where the paper is silent: the automaton is a dense table over byte classes
 * (delta(s,b) = trans[s*n_classes + byte_to_class[b]]) with one absorbing dead state standing
 * for "cannot read" (dead = -1: no such state); the end state need not be accepting
 * (Algorithm 3 never consults F); the EOS token (Section 2.1) is admissible, by id, exactly
 * from accepting states and leaves the state unchanged; empty tokens are never admissible; the
 * dead state's own row is empty.
 */
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    const int32_t *trans;
    int32_t n_states;
    int32_t n_classes;
    const uint8_t *byte_to_class;
    const uint8_t *accept;
    int32_t dead;
    const uint8_t *bytes;
    const int64_t *offsets;
    int32_t n_tokens;
    int32_t eos;
} problem_t;

/* One (state, token) pair.  Returns 1 and the end state if the token is admissible from q.
 * *steps counts transition-function evaluations, including the one that lands in dead. */
static int walk_pair(const problem_t *p, int32_t q, int32_t t, int32_t *end, int64_t *steps,
                     int *died_on_first)
{
    *died_on_first = 0;
    if (q == p->dead)
        return 0;
    if (t == p->eos) {
        if (p->accept[q]) { *end = q; return 1; }
        return 0;
    }
    int64_t lo = p->offsets[t], hi = p->offsets[t + 1];
    if (hi <= lo)
        return 0;
    int32_t s = q;
    for (int64_t i = lo; i < hi; ++i) {
        s = p->trans[(int64_t)s * p->n_classes + p->byte_to_class[p->bytes[i]]];
        ++*steps;
        if (s == p->dead) {
            if (i == lo) *died_on_first = 1;
            return 0;
        }
    }
    *end = s;
    return 1;
}

typedef struct {
    const problem_t *p;
    int32_t q_lo, q_hi;
    int64_t *row_count;          /* [n_states], count pass */
    const int64_t *row_ptr;      /* fill pass */
    int32_t *token_ids, *next_states;
    int64_t w_bf, w_first_fail;
} job_t;

static void *row_job(void *arg)
{
    job_t *j = (job_t *)arg;
    const problem_t *p = j->p;
    for (int32_t q = j->q_lo; q < j->q_hi; ++q) {
        int64_t n = 0;
        for (int32_t t = 0; t < p->n_tokens; ++t) {
            int32_t end = 0;
            int died0 = 0;
            int64_t steps = 0;
            int ok = walk_pair(p, q, t, &end, &steps, &died0);
            j->w_bf += steps;
            j->w_first_fail += died0;
            if (ok) {
                if (j->token_ids) {
                    j->token_ids[j->row_ptr[q] + n] = t;
                    j->next_states[j->row_ptr[q] + n] = end;
                }
                ++n;
            }
        }
        if (j->row_count)
            j->row_count[q] = n;
    }
    return NULL;
}

static void run_rows(const problem_t *p, int n_threads, int64_t *row_count, const int64_t *row_ptr,
                     int32_t *token_ids, int32_t *next_states, int64_t *w_bf, int64_t *w_first_fail)
{
    if (n_threads < 1) n_threads = 1;
    if (n_threads > p->n_states) n_threads = p->n_states > 0 ? p->n_states : 1;
    job_t *jobs = (job_t *)calloc((size_t)n_threads, sizeof(job_t));
    pthread_t *tid = (pthread_t *)calloc((size_t)n_threads, sizeof(pthread_t));
    for (int k = 0; k < n_threads; ++k) {
        jobs[k].p = p;
        jobs[k].q_lo = (int32_t)((int64_t)p->n_states * k / n_threads);
        jobs[k].q_hi = (int32_t)((int64_t)p->n_states * (k + 1) / n_threads);
        jobs[k].row_count = row_count;
        jobs[k].row_ptr = row_ptr;
        jobs[k].token_ids = token_ids;
        jobs[k].next_states = next_states;
    }
    if (n_threads == 1) {
        row_job(&jobs[0]);
    } else {
        for (int k = 0; k < n_threads; ++k) pthread_create(&tid[k], NULL, row_job, &jobs[k]);
        for (int k = 0; k < n_threads; ++k) pthread_join(tid[k], NULL);
    }
    int64_t a = 0, b = 0;
    for (int k = 0; k < n_threads; ++k) { a += jobs[k].w_bf; b += jobs[k].w_first_fail; }
    if (w_bf) *w_bf = a;
    if (w_first_fail) *w_first_fail = b;
    free(jobs);
    free(tid);
}

/*
 * Pass 1: row_ptr[0..n_states] (exclusive prefix sums of the row sizes, row_ptr[n_states] = nnz).
 * counters[0] = W_bf   transition evaluations of the early-exit walk over all pairs,
 * counters[1] = W_inv  the same minus the walks that fail on their first byte (the walks
 *                      that Algorithm 3's restriction to start states able to read v0 never
 *                      starts).
 * States are statically split over n_threads threads; every thread runs the same loops.
 */
int64_t oracle_index_count(const int32_t *trans, int32_t n_states, int32_t n_classes,
                           const uint8_t *byte_to_class, const uint8_t *accept, int32_t dead,
                           const uint8_t *bytes, const int64_t *offsets, int32_t n_tokens,
                           int32_t eos, int32_t n_threads, int64_t *row_ptr, int64_t *counters)
{
    problem_t p = { trans, n_states, n_classes, byte_to_class, accept, dead, bytes, offsets, n_tokens, eos };
    int64_t *cnt = (int64_t *)calloc((size_t)(n_states > 0 ? n_states : 1), sizeof(int64_t));
    int64_t w_bf = 0, w_ff = 0;
    run_rows(&p, n_threads, cnt, NULL, NULL, NULL, &w_bf, &w_ff);
    row_ptr[0] = 0;
    for (int32_t q = 0; q < n_states; ++q) row_ptr[q + 1] = row_ptr[q] + cnt[q];
    free(cnt);
    if (counters) { counters[0] = w_bf; counters[1] = w_bf - w_ff; }
    return row_ptr[n_states];
}

/* Pass 2: the entries of row q go to [row_ptr[q], row_ptr[q+1]) in ascending token id. */
void oracle_index_fill(const int32_t *trans, int32_t n_states, int32_t n_classes,
                       const uint8_t *byte_to_class, const uint8_t *accept, int32_t dead,
                       const uint8_t *bytes, const int64_t *offsets, int32_t n_tokens,
                       int32_t eos, int32_t n_threads, const int64_t *row_ptr,
                       int32_t *token_ids, int32_t *next_states)
{
    problem_t p = { trans, n_states, n_classes, byte_to_class, accept, dead, bytes, offsets, n_tokens, eos };
    run_rows(&p, n_threads, NULL, row_ptr, token_ids, next_states, NULL, NULL);
}

/* One row of the index: sigma(q) in ascending token id with the end states.  Returns its size;
 * the output arrays need room for n_tokens entries.  (Spot checks at sizes where indexing every
 * state on the CPU would take too long.) */
int64_t oracle_index_row(const int32_t *trans, int32_t n_states, int32_t n_classes,
                         const uint8_t *byte_to_class, const uint8_t *accept, int32_t dead,
                         const uint8_t *bytes, const int64_t *offsets, int32_t n_tokens, int32_t eos,
                         int32_t q, int32_t *token_ids, int32_t *next_states)
{
    problem_t p = { trans, n_states, n_classes, byte_to_class, accept, dead, bytes, offsets, n_tokens, eos };
    int64_t n = 0;
    if (q < 0 || q >= n_states) return 0;
    for (int32_t t = 0; t < n_tokens; ++t) {
        int32_t end = 0;
        int64_t steps = 0;
        int d0 = 0;
        if (walk_pair(&p, q, t, &end, &steps, &d0)) {
            token_ids[n] = t;
            next_states[n] = end;
            ++n;
        }
    }
    return n;
}

/* End state of one walk, or -1 if the token is not admissible from q (spot checks). */
int32_t oracle_walk(const int32_t *trans, int32_t n_states, int32_t n_classes,
                    const uint8_t *byte_to_class, const uint8_t *accept, int32_t dead,
                    const uint8_t *bytes, const int64_t *offsets, int32_t n_tokens, int32_t eos,
                    int32_t q, int32_t t)
{
    problem_t p = { trans, n_states, n_classes, byte_to_class, accept, dead, bytes, offsets, n_tokens, eos };
    int32_t end = -1;
    int64_t steps = 0;
    int d0 = 0;
    if (q < 0 || q >= n_states || t < 0 || t >= n_tokens) return -1;
    return walk_pair(&p, q, t, &end, &steps, &d0) ? end : -1;
}

/*
 * Mask (Section 2.2): out[b][t] = in[b][t] for t in sigma(states[b]), -inf otherwise.
 * elem_size 4: IEEE binary32 (-inf = 0xFF800000); elem_size 2: bfloat16 (-inf = 0xFF80).
 * A negative state leaves the row unmasked; a state outside [0, n_states) that is not negative
 * has no row, so everything is removed.  Rows are stride elements apart in both buffers.
 */
void oracle_mask_logits(const int64_t *row_ptr, const int32_t *token_ids, int32_t n_states,
                        int32_t n_vocab, const int32_t *states, int32_t batch,
                        const void *in, void *out, int64_t stride, int32_t elem_size)
{
    uint8_t *allowed = (uint8_t *)malloc((size_t)(n_vocab > 0 ? n_vocab : 1));
    for (int32_t b = 0; b < batch; ++b) {
        const uint8_t *src = (const uint8_t *)in + (size_t)b * (size_t)stride * (size_t)elem_size;
        uint8_t *dst = (uint8_t *)out + (size_t)b * (size_t)stride * (size_t)elem_size;
        if (dst != src)
            memmove(dst, src, (size_t)n_vocab * (size_t)elem_size);
        int32_t s = states[b];
        if (s < 0)
            continue;
        memset(allowed, 0, (size_t)n_vocab);
        if (s < n_states)
            for (int64_t k = row_ptr[s]; k < row_ptr[s + 1]; ++k)
                allowed[token_ids[k]] = 1;
        for (int32_t t = 0; t < n_vocab; ++t) {
            if (allowed[t])
                continue;
            if (elem_size == 4) {
                uint32_t ninf = 0xFF800000u;
                memcpy(dst + (size_t)t * 4, &ninf, 4);
            } else {
                uint16_t ninf = 0xFF80u;
                memcpy(dst + (size_t)t * 2, &ninf, 2);
            }
        }
    }
    free(allowed);
}
