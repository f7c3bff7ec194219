/*
 * fsmidx -- FSM vocabulary index construction and logit masking on AMD MI355X (gfx950).
 *
 * C ABI of the data-parallel hot path of FSM-guided generation (Willard & Louf, "Efficient
 * Guided Generation for Large Language Models", Section 3): for every pair (automaton state
 * q, vocabulary string v) walk v through the transition function, keep v in sigma(q) if the
 * walk never reaches the reject state, and remember the state in which it stops.  sigma is
 * stored as a CSR over states; a second call applies sigma(q) as a mask to logits
 * (Section 2.2).
 *
 * Conventions that hold for every function
 *   - "host" pointers are ordinary process memory, "device" pointers are HIP device memory of
 *     the current device.  The library never takes ownership of caller memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - Return value: FSMIDX_OK (0) or a negative fsmidx_status.  A human-readable message for
 *     the last failure on the calling thread is available from fsmidx_last_error().
 *   - Integers are little-endian two's complement; no function is re-entrant on the same
 *     workspace, all are re-entrant across different workspaces / streams.
 */
#ifndef FSMIDX_H
#define FSMIDX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FSMIDX_OK = 0,
    FSMIDX_INVALID_ARG = -1,      /* null pointer, size out of range, malformed automaton/vocabulary */
    FSMIDX_OUT_OF_MEMORY = -2,    /* device or host allocation failed                                */
    FSMIDX_HIP_ERROR = -3,        /* a HIP runtime call failed (message holds the HIP error string)  */
    FSMIDX_UNSUPPORTED = -4,      /* unknown dtype                                                   */
    FSMIDX_BAD_DEVICE_INPUT = -5, /* device-resident inputs failed the on-device checks              */
    FSMIDX_WORKSPACE_TOO_SMALL = -6,
    FSMIDX_OUTPUT_TOO_SMALL = -7  /* fsmidx_build_into: more entries than the caller's capacity        */
} fsmidx_status;

/*
 * The automaton (Q, Sigma, delta, q0, F) of Section 3, Definition 1, as a dense table over byte
 * classes: delta(s, b) = trans[s * n_classes + byte_to_class[b]].  q0 is not needed: every state
 * is indexed as a possible starting point (Section 3: a walk may begin in any state).
 * The paper's "delta(r, v_i) = empty" (Algorithm 3) is encoded by one absorbing state
 * `dead_state`; -1 means the automaton is total and nothing is ever rejected.
 */
typedef struct {
    const int32_t *trans;          /* [n_states * n_classes] row-major, every value in [0, n_states)   */
    int32_t        n_states;       /* 1 .. 2^31-1, includes the dead state if there is one             */
    int32_t        n_classes;      /* 1 .. 256                                                         */
    const uint8_t *byte_to_class;  /* [256], every value < n_classes                                   */
    const uint8_t *accept;         /* [n_states], nonzero for states in F (used for EOS only)          */
    int32_t        dead_state;     /* id of the absorbing reject state (trans[dead][*] == dead), or -1 */
} fsmidx_dfa;

/*
 * The vocabulary V (Section 2): token t is bytes[offsets[t] .. offsets[t+1]).  Empty tokens are
 * legal and never admissible.  `eos_token_id` names the EOS token of Section 2.1: it is
 * admissible, whatever its bytes, exactly from accepting states and leaves the state unchanged;
 * -1 = no such token.
 */
typedef struct {
    const uint8_t *bytes;          /* [n_bytes]                                                        */
    const int64_t *offsets;        /* [n_tokens + 1], offsets[0] = 0, non-decreasing, last = n_bytes   */
    int32_t        n_tokens;       /* 0 .. 2^30                                                        */
    int32_t        eos_token_id;   /* -1 or in [0, n_tokens)                                           */
    int64_t        n_bytes;        /* 0 .. 2^31-1                                                      */
} fsmidx_vocab;

/*
 * The index sigma: Q -> P(V) of Section 3 (Algorithm 4) with the end state of every walk kept
 * beside the token (Section 3, paragraph on tracking the state reached after a sampled token).
 * Row q is [row_ptr[q], row_ptr[q+1]); inside a row token ids ascend strictly.  All arrays are
 * DEVICE pointers.
 *
 * `allow_bits` is the same sigma as a bitmap -- the mask m of Section 2.2, one bit per (state,
 * token): bit (t mod 64) of word allow_bits[q * allow_stride + t / 64] is set iff token t is in row
 * q.  It is optional (NULL = absent).  The build produces it as a by-product and mask_logits is
 * faster with it; it costs n_states * allow_stride * 8 bytes.
 */
typedef struct {
    int32_t         n_states;
    int32_t         n_tokens;
    int64_t         nnz;
    const int64_t  *row_ptr;       /* [n_states + 1]                                                   */
    const int32_t  *token_ids;     /* [nnz]                                                            */
    const int32_t  *next_states;   /* [nnz]                                                            */
    const uint64_t *allow_bits;    /* [n_states * allow_stride] or NULL                                */
    int64_t         allow_stride;  /* words per state, >= ceil(n_tokens / 64)                          */
} fsmidx_csr;

typedef struct fsmidx_index fsmidx_index;   /* opaque owner of a CSR in device memory */

/* Message of the last failing call on this thread; valid until the next call on this thread. */
const char *fsmidx_last_error(void);

/*
 * Check an automaton and a vocabulary given by HOST pointers against every rule stated in the
 * struct comments above (value ranges, dead state absorbing, offsets monotone and consistent with
 * n_bytes, eos id in range).  Touches no GPU.  FSMIDX_OK or FSMIDX_INVALID_ARG.
 */
int fsmidx_validate_host(const fsmidx_dfa *dfa, const fsmidx_vocab *vocab);

/*
 * build_index, one call (Section 3, Algorithms 3 and 4).  `dfa` and `vocab` hold HOST pointers;
 * they are validated, copied to the device and may be freed when the call returns.  The call
 * allocates the result with hipMalloc, enqueues all kernels on `stream`, synchronises the stream
 * once (to learn nnz) and again before returning.  *out is owned by the library until
 * fsmidx_free_index.  On error *out is NULL and nothing is leaked.
 */
int fsmidx_build_index(const fsmidx_dfa *dfa, const fsmidx_vocab *vocab, void *stream, fsmidx_index **out);

/* Device-pointer view of an index (valid until the index is freed). */
int fsmidx_index_csr(const fsmidx_index *index, fsmidx_csr *view);

/* Copy an index to HOST arrays of sizes [n_states+1], [nnz], [nnz] (synchronous). */
int fsmidx_index_to_host(const fsmidx_index *index, int64_t *row_ptr, int32_t *token_ids, int32_t *next_states);

void fsmidx_free_index(fsmidx_index *index);

/*
 * build_index in two steps on DEVICE-resident inputs with caller-owned memory (the form to use
 * when torch or another allocator owns every byte, and the one the benchmark times):
 *
 *   fsmidx_build_workspace_bytes  -> size of the scratch area
 *   fsmidx_build_count            -> classifies bytes, prepares the table, walks all pairs, writes
 *                                    row_ptr and returns nnz (one stream synchronisation; an
 *                                    automaton that branches deeply makes the walk count again
 *                                    another way, at most twice, with one more each time)
 *   caller allocates token_ids[nnz], next_states[nnz]
 *   fsmidx_build_fill             -> walks again and writes the entries (asynchronous; `nnz` must be the
 *                                    count fsmidx_build_count returned: the call cannot wait for the
 *                                    device, so with a smaller nnz it returns FSMIDX_OK and the kernel,
 *                                    which checks the count against nnz itself, writes nothing)
 *
 * In fsmidx_build_count / fsmidx_build_fill the POINTER members of `dfa` and `vocab` are device
 * pointers; the scalar members are read on the host.  The host cannot inspect device data, so
 * range checks run on the device: a transition outside [0, n_states), a class id >= n_classes,
 * offsets that decrease or leave [0, n_bytes], or a dead state that is not absorbing make
 * fsmidx_build_count return FSMIDX_BAD_DEVICE_INPUT; the offending values are neutralised before
 * any kernel uses them as an address, so no out-of-bounds access happens.  row_ptr is then
 * unspecified.
 *
 * `workspace` (device, 256-byte aligned, at least the queried size) carries state from count to
 * fill and must not be touched in between; the inputs must not change either.
 */
int fsmidx_build_workspace_bytes(int32_t n_states, int32_t n_classes, int32_t n_tokens, int64_t n_bytes,
                                 size_t *bytes);
int fsmidx_build_count(const fsmidx_dfa *dfa_dev, const fsmidx_vocab *vocab_dev,
                       void *workspace, size_t workspace_bytes,
                       int64_t *row_ptr_dev /* [n_states + 1] */, int64_t *nnz_host, void *stream);
int fsmidx_build_fill(const fsmidx_dfa *dfa_dev, const fsmidx_vocab *vocab_dev,
                      void *workspace, size_t workspace_bytes, const int64_t *row_ptr_dev,
                      int64_t nnz /* as returned by build_count */,
                      int32_t *token_ids_dev, int32_t *next_states_dev, void *stream);

/*
 * build_index in ONE step for a caller that can bound nnz (say, from the last build of the same
 * automaton against the same vocabulary): counting pass, scans and emitting pass are enqueued back
 * to back, with no host round trip in between, and the stream is synchronised once at the end
 * (an automaton that branches deeply: up to two further rounds of the same, as in build_count).
 * token_ids_dev / next_states_dev hold `capacity` entries each.  Returns FSMIDX_OK with *nnz_host
 * entries written, or FSMIDX_OUTPUT_TOO_SMALL with *nnz_host = the number needed: then row_ptr
 * and the workspace are complete, nothing was written to the two arrays, and fsmidx_build_fill
 * with large enough arrays finishes the build.  Everything else as for count + fill.
 */
int fsmidx_build_into(const fsmidx_dfa *dfa_dev, const fsmidx_vocab *vocab_dev,
                      void *workspace, size_t workspace_bytes, int64_t *row_ptr_dev /* [n_states + 1] */,
                      int32_t *token_ids_dev, int32_t *next_states_dev, int64_t capacity,
                      int64_t *nnz_host, void *stream);

/*
 * fsmidx_build_into in two halves, for a caller that has more work for the stream before it wants
 * to wait (the masks of a decode batch that use the index, Section 2.2; the next build).
 * fsmidx_build_enqueue launches the counting pass, the scans and the emitting pass (Section 3,
 * Algorithms 3 and 4) and returns without waiting: it synchronises nothing, copies nothing and
 * allocates nothing.  Work enqueued on the same stream after it sees the finished index -- row_ptr,
 * the two arrays and the bitmap form in the workspace -- unless the build has to be repeated, which
 * only fsmidx_build_finish can find out: it waits for the stream, reads the status and returns
 * what fsmidx_build_into returns (same arguments, same error codes, *nnz_host).  If the counting
 * pass had to be redone (an automaton that branches deeper than the first attempt's stack holds, or
 * a build whose launch sequence followed a hint that no longer applies) it does that, waits again
 * and sets *redone_host = 1 (else 0; may be NULL): whatever was enqueued between the two calls has
 * then read an unfinished index and has to be enqueued again.  Input errors found on the device
 * are reported by fsmidx_build_finish as well.  Both calls take the same arguments; the workspace
 * and the inputs must not change in between.
 */
int fsmidx_build_enqueue(const fsmidx_dfa *dfa_dev, const fsmidx_vocab *vocab_dev,
                         void *workspace, size_t workspace_bytes, int64_t *row_ptr_dev /* [n_states + 1] */,
                         int32_t *token_ids_dev, int32_t *next_states_dev, int64_t capacity, void *stream);
int fsmidx_build_finish(const fsmidx_dfa *dfa_dev, const fsmidx_vocab *vocab_dev,
                        void *workspace, size_t workspace_bytes, int64_t *row_ptr_dev,
                        int32_t *token_ids_dev, int32_t *next_states_dev, int64_t capacity,
                        int64_t *nnz_host, int32_t *redone_host, void *stream);

/*
 * Where fsmidx_build_count left the bitmap form of the index inside `workspace` (for the
 * allow_bits / allow_stride members of fsmidx_csr).  Valid from the return of fsmidx_build_count
 * until the workspace is written again; touches no GPU.
 */
int fsmidx_build_allow_bits(int32_t n_states, int32_t n_classes, int32_t n_tokens, int64_t n_bytes,
                            const void *workspace, const uint64_t **allow_bits, int64_t *allow_stride);

/*
 * mask_logits (Section 2.2, "alpha~ = m (.) alpha", Algorithm 2): for every batch row b,
 *     out[b][t] = in[b][t]   if token t is in row states[b] of the index   (bit copy)
 *               = -inf       otherwise                                     (0xFF800000 / 0xFF80)
 * for t in [0, index->n_tokens).  Rows are `row_stride` ELEMENTS apart in both buffers
 * (row_stride >= n_tokens); elements past n_tokens in a row are not touched.
 *   dtype 0 = IEEE binary32, 1 = bfloat16.
 *   states[b] <  0                 -> the row is passed through unmasked
 *   states[b] >= index->n_states   -> no such row: everything becomes -inf
 *   a state with an empty row (e.g. the dead state) -> everything becomes -inf
 * With index->allow_bits the kernel reads one bitmap word per 64 tokens; without it, it locates
 * the row's token ids by search.  Both give the same result.
 * `logits_out` may be the same pointer as `logits_in` but must not overlap it in any other way.
 * In place the result is the same bits; which bytes are stored differs by type: binary32 stores
 * -inf over removed tokens only and reads no logits; bfloat16 also reads and rewrites, unchanged,
 * the kept tokens that share a 16-byte vector with removed ones (eight 2-byte stores cost more than
 * the read), so in place no other stream may write kept bfloat16 logits meanwhile.  All pointers are DEVICE pointers; buffers must be aligned to
 * the element size.  Asynchronous on `stream`.
 */
int fsmidx_mask_logits(const fsmidx_csr *index, const int32_t *states_dev, int32_t batch,
                       const void *logits_in, void *logits_out, int64_t row_stride,
                       int32_t dtype, void *stream);

/*
 * advance_states (Section 3: the index keeps, beside every token of sigma(q), the state in which
 * the automaton stops after reading it, so the state of a sequence is tracked from one step of
 * Algorithm 2 to the next without re-reading the sequence):
 *     states_out[b] = the end state stored with tokens[b] in row states[b] of the index.
 *   states[b] < 0 (no guidance)                          -> copied through unchanged
 *   tokens[b] not in the row, or either id out of range  -> index->n_states: an id that names no
 *       row, for which mask_logits removes everything and from which advancing stays put (a
 *       token sampled under the mask is always in the row, so this marks a caller's mistake)
 * One binary search per sequence in the row's ascending token ids; index->allow_bits is not
 * used.  `states_out` may be the same pointer as `states`.  All pointers are DEVICE pointers.
 * Asynchronous on `stream`.
 */
int fsmidx_advance_states(const fsmidx_csr *index, const int32_t *states_dev, const int32_t *tokens_dev,
                          int32_t batch, int32_t *states_out_dev, void *stream);

/*
 * masked_argmax: greedy decoding (Section 2.1) on the masked logits of Section 2.2, Algorithm 2,
 * together with the state update of Section 3.  Masked logits are -inf outside sigma(q), so
 *     tokens_out[b] = the token of row states[b] with the largest logits[b][token]
 *     states_out[b] = the end state stored with that token
 * and only the row's entries are read: the work follows |sigma(q)|, not |V| (Section 3).
 *   ties go to the lowest token id; a NaN logit counts as -inf; -0.0 equals +0.0
 *   states[b] < 0 (no guidance)      -> the choice ranges over all of [0, n_tokens); the state is
 *                                       copied through
 *   a state with an empty row, or states[b] >= index->n_states
 *                                    -> tokens_out[b] = -1, states_out[b] = index->n_states
 * `logits` is [batch] rows of `row_stride` elements (>= n_tokens), dtype as for mask_logits; it
 * is only read.  `workspace` is device memory of at least
 * fsmidx_masked_argmax_workspace_bytes(batch) bytes, 8-byte aligned, that the call may overwrite
 * (partial results; nothing is kept between calls).  batch <= 2^24.  `states_out` may be the same
 * pointer as `states`.  All pointers are DEVICE pointers.  Asynchronous on `stream`.
 */
int fsmidx_masked_argmax_workspace_bytes(int32_t batch, size_t *bytes);
int fsmidx_masked_argmax(const fsmidx_csr *index, const int32_t *states_dev, int32_t batch,
                         const void *logits, int64_t row_stride, int32_t dtype,
                         void *workspace, size_t workspace_bytes,
                         int32_t *tokens_out_dev, int32_t *states_out_dev, void *stream);

/*
 * masked_argmax without a workspace, for callers that cannot allocate device memory: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels and same results as fsmidx_masked_argmax; the partial results go to a fixed array of
 * 2 MiB inside the library (one copy per GPU, held until the process ends), which limits a call
 * to batch <= 4096: a larger batch is FSMIDX_INVALID_ARG.  The call allocates and frees nothing.
 * All calls on one GPU share that array: calls that overlap in time on one GPU (different streams
 * or threads) race and give undefined results; calls on one stream are ordered and safe.  Nothing
 * is carried over from one call to the next.  Asynchronous on `stream`.
 */
int fsmidx_masked_argmax_static(const fsmidx_csr *index, const int32_t *states_dev, int32_t batch,
                                const void *logits, int64_t row_stride, int32_t dtype,
                                int32_t *tokens_out_dev, int32_t *states_out_dev, void *stream);

/*
 * masked_sample: the sampling step of Algorithm 2 (Section 2.2), s ~ Categorical(alpha~), with the
 * state update of Section 3.  On logits the masked distribution alpha~ is the softmax over the
 * tokens of row states[b]; the random number is the caller's: uniforms[b] in [0, 1).  The draw is
 * by inversion over the row's entries in ascending token id, with weights
 *     w = 1 for a logit equal to the row's largest, exp(logit - largest) otherwise
 * (binary32 exponentials, binary64 sums):
 *     tokens_out[b] = the first entry whose cumulative weight exceeds uniforms[b] * (sum of all weights)
 *     states_out[b] = the end state stored with that token
 * Only the row's entries are read (three passes over them).
 *   a NaN logit counts as -inf (weight 0); +inf logits share the whole mass among themselves;
 *   nothing but -inf in the row -> the row's first entry
 *   uniforms[b] is clamped into [0, 1 - 2^-24], NaN counts as 0
 *   states[b] < 0 (no guidance)      -> the draw ranges over all of [0, n_tokens); state copied through
 *   a state with an empty row, or states[b] >= index->n_states
 *                                    -> tokens_out[b] = -1, states_out[b] = index->n_states
 * The cumulative weights carry rounding errors of a few 2^-24 of the total; when the threshold
 * lies that close to a boundary between two entries, either may be returned (never an entry of
 * weight 0).  Otherwise as fsmidx_masked_argmax: `workspace` of at least
 * fsmidx_masked_sample_workspace_bytes(batch) bytes, batch <= 2^24, `states_out` may alias
 * `states`, all pointers DEVICE pointers, asynchronous on `stream`.
 */
int fsmidx_masked_sample_workspace_bytes(int32_t batch, size_t *bytes);
int fsmidx_masked_sample(const fsmidx_csr *index, const int32_t *states_dev, int32_t batch,
                         const void *logits, int64_t row_stride, int32_t dtype,
                         const float *uniforms_dev, void *workspace, size_t workspace_bytes,
                         int32_t *tokens_out_dev, int32_t *states_out_dev, void *stream);

/*
 * Many automata in one index (Section 5: the index of a large grammar is built from many
 * automata; also the serving case of many regular expressions against one vocabulary).
 * fsmidx_union_dfa forms, on the device, the disjoint union of `n_dfas` automata (1..64) as ONE
 * automaton that the build calls above take like any other:
 *   - state s of automaton k becomes state  state_base[k] + s,  state_base[k] = the number of states
 *     of the automata before it (state_base[n_dfas] = all states);
 *   - two bytes are in one class of the union iff every automaton has them in one class; classes
 *     are numbered in order of their smallest byte;
 *   - every automaton's dead state becomes one: the union's dead state is the renumbered dead state
 *     of the first automaton that has one (-1 if none has), and every transition into any
 *     automaton's dead state leads there.
 * The index of the union is the automata's own indices laid end to end (rows state_base[k] ..
 * state_base[k+1] - 1 are automaton k's rows, end states renumbered the same way), built with the
 * vocabulary's share of the work done once; a decode batch that mixes sequences of different
 * automata is then masked with one fsmidx_mask_logits call on union state ids.
 *   `dfas` is a HOST array of structs whose pointer members are DEVICE pointers.  The three output
 * arrays are DEVICE memory of the caller: trans_out [trans_capacity] int32 (needs all states x the
 * union's classes, at most 256 per state), byte_to_class_out [256], accept_out [all states].
 * `workspace`: device, 256-byte aligned, fsmidx_union_workspace_bytes(n_dfas) bytes.  On success
 * *union_out describes the union (its pointers are the output arrays) and state_base_host
 * [n_dfas + 1] is filled.  The call synchronises the stream twice (the class count, then the
 * device-side range checks of the inputs: FSMIDX_BAD_DEVICE_INPUT as for fsmidx_build_count);
 * FSMIDX_OUTPUT_TOO_SMALL if trans_capacity does not hold the table (the message says how much).
 */
int fsmidx_union_workspace_bytes(int32_t n_dfas, size_t *bytes);
int fsmidx_union_dfa(const fsmidx_dfa *dfas, int32_t n_dfas, int32_t *trans_out_dev, int64_t trans_capacity,
                     uint8_t *byte_to_class_out_dev, uint8_t *accept_out_dev, void *workspace, size_t workspace_bytes,
                     fsmidx_dfa *union_out, int32_t *state_base_host /* [n_dfas + 1] */, void *stream);

/*
 * Identical rows kept once (Section 5: redundant states make the index larger than it has to be).
 * States whose rows of sigma are identical -- the same tokens with the same end states -- are
 * interchangeable for masking and for tracking the state.  fsmidx_dedupe_rows finds them:
 *     row_of_state[q]   = the number of q's row among the distinct rows, which are numbered in
 *                         order of the smallest state that has them
 *     unique_row_ptr[u] = first entry of distinct row u in the compact arrays that
 *                         fsmidx_dedupe_fill writes ([n_unique + 1] entries are set; the array
 *                         must hold n_states + 1)
 * and returns the number of distinct rows and of their entries (one stream synchronisation; rows
 * are grouped by a 64-bit hash and then compared entry by entry, so the result is exact).
 * fsmidx_dedupe_fill then copies the distinct rows side by side into token_ids_out /
 * next_states_out [nnz_unique] (asynchronous).  End states stay state ids: the row of an end state
 * s is distinct row row_of_state[s].  {n_states = n_unique, row_ptr = unique_row_ptr, the compact
 * arrays} is an fsmidx_csr that mask_logits, advance_states and the masked choices accept with
 * row_of_state[state] in the place of the state.
 *   `workspace`: device, 256-byte aligned, fsmidx_dedupe_workspace_bytes(n_states) bytes; it
 * carries state from dedupe_rows to dedupe_fill.  index->allow_bits is not used.  n_states <= 2^26.
 */
int fsmidx_dedupe_workspace_bytes(int32_t n_states, size_t *bytes);
int fsmidx_dedupe_rows(const fsmidx_csr *index, void *workspace, size_t workspace_bytes,
                       int32_t *row_of_state_dev /* [n_states] */, int64_t *unique_row_ptr_dev /* [n_states + 1] */,
                       int32_t *n_unique_host, int64_t *nnz_unique_host, void *stream);
int fsmidx_dedupe_fill(const fsmidx_csr *index, const void *workspace, size_t workspace_bytes,
                       const int64_t *unique_row_ptr_dev, int32_t *token_ids_out_dev, int32_t *next_states_out_dev,
                       void *stream);

/*
 * Minimisation before indexing (Section 5: the paper's indices come from un-reduced automata, whose
 * redundant states make them larger than they have to be).  What the index records about a walk is
 * whether it meets the rejecting state and whether the state it ends in accepts (Section 3,
 * Algorithms 3 and 4; Section 2.1 for EOS), so every state has one of three labels -- rejecting
 * state, accepting, neither -- and two states are equivalent iff every string of byte classes leads
 * them to equally labelled states.  A state from which nothing can be accepted any more is NOT the
 * rejecting state: only `dead_state` rejects.  fsmidx_minimise_dfa finds the classes by refinement
 * (exact: signatures are grouped by hash, then compared) and writes
 *     block_of_state[q] = the class of q; classes are numbered in order of their smallest state
 *     the quotient automaton: one state per class (trans_out [classes x n_classes], accept_out
 *     [classes], the class of the rejecting state as its dead_state), described by *min_out, whose
 *     byte_to_class is the input's pointer.
 * The index of the quotient is the original's with state ids mapped through block_of_state: row q
 * of the original holds the tokens of row block_of_state[q] of the quotient, and each end state s
 * appears there as block_of_state[s].
 *   `dfa`: DEVICE pointers, as for fsmidx_build_count; its table is range checked on the device
 * (FSMIDX_BAD_DEVICE_INPUT).  Outputs are DEVICE memory of the caller: block_of_state [n_states],
 * trans_out [trans_capacity] (n_states x n_classes always suffices; FSMIDX_OUTPUT_TOO_SMALL says
 * how much is needed), accept_out [n_states].  `workspace`: device, 256-byte aligned,
 * fsmidx_minimise_workspace_bytes(n_states) bytes.  The stream is synchronised once per 8 to 64
 * rounds of refinement and once at the end.  n_states <= 2^26.
 */
int fsmidx_minimise_workspace_bytes(int32_t n_states, size_t *bytes);
int fsmidx_minimise_dfa(const fsmidx_dfa *dfa, void *workspace, size_t workspace_bytes,
                        int32_t *block_of_state_dev /* [n_states] */, int32_t *trans_out_dev, int64_t trans_capacity,
                        uint8_t *accept_out_dev /* [n_states] */, fsmidx_dfa *min_out, void *stream);

/*
 * The reachable-only index (Section 3, the paragraph after Algorithm 4: the index needs a row per
 * state in principle, but not every state is ever represented by a vocabulary string; Section 2.2,
 * Algorithm 2: a generation starts in q_0 and moves to the end state stored with each sampled
 * token).  The states a generation can be in are those reachable from q_0 through rows of the
 * index; only their rows are ever read.
 *   fsmidx_reachable_states marks them: reach_out[q] = 1 if some sequence of vocabulary tokens
 * leads from one of the start states to q (the start states themselves included), else 0, and
 * *n_reached_host = their number.  `start_states_host` is a HOST array of n_starts state ids in
 * [0, n_states) (FSMIDX_INVALID_ARG otherwise); `index` is a complete index (device pointers,
 * allow_bits not used); reach_out_dev [n_states] is DEVICE memory.  A breadth-first search on the
 * device; the call synchronises the stream once per 8 to 64 levels and once at the end.  End states
 * outside [0, n_states) (an index the library did not write) are ignored, never dereferenced.
 *   fsmidx_restrict_rows / _fill write the index with the rows of all states q with keep[q] == 0
 * left empty (keep = reach_out, or any other choice): state ids keep their meaning, the kept rows
 * are unchanged and lie side by side in state order.  restrict_rows fills row_ptr_out_dev
 * [n_states + 1] and returns the number of entries kept (one synchronisation); restrict_fill copies
 * them into token_ids_out / next_states_out, which hold `capacity` >= that number of entries
 * (asynchronous; a row that would not fit is not written).  {row_ptr_out, the new arrays} is an
 * fsmidx_csr for mask_logits, advance_states and the masked choices; a generation that starts in a
 * start state never meets a missing row.
 *   `workspace`: device, 256-byte aligned, fsmidx_reach_workspace_bytes(n_states) bytes.
 * n_states <= 2^26.
 */
int fsmidx_reach_workspace_bytes(int32_t n_states, size_t *bytes);
int fsmidx_reachable_states(const fsmidx_csr *index, const int32_t *start_states_host, int32_t n_starts,
                            void *workspace, size_t workspace_bytes, uint8_t *reach_out_dev /* [n_states] */,
                            int32_t *n_reached_host, void *stream);
int fsmidx_restrict_rows(const fsmidx_csr *index, const uint8_t *keep_dev /* [n_states] */, void *workspace,
                         size_t workspace_bytes, int64_t *row_ptr_out_dev /* [n_states + 1] */, int64_t *nnz_out_host,
                         void *stream);
int fsmidx_restrict_fill(const fsmidx_csr *index, const uint8_t *keep_dev, const int64_t *row_ptr_out_dev,
                         int32_t *token_ids_out_dev, int32_t *next_states_out_dev, int64_t capacity, void *stream);

/*
 * The scanner step of parser-guided generation (Section 4 and Section 4.1).  Every parse state
 * reads an ordered list of terminal symbols and scans with the union of their automata.  A front
 * end (not part of this library) supplies all these scanners side by side in one automaton
 * `scanner` (DEVICE pointers as for fsmidx_build_count; only n_states, n_classes, trans and
 * dead_state are read), and for every state q
 *     completes[q]         uint64: bit t set iff q is a final state of terminal t (t < 64; the
 *                          terminals are numbered in the order of the parser's lists)
 *     scanner_of_state[q]  the parse state whose scanner q belongs to (read only for states that
 *                          complete a terminal)
 * and the parser's shift moves as a table
 *     shift[p * n_terminals + t]  the state in which scanning goes on after terminal t has been
 *                          read in parse state p (the start state of the following parse state's
 *                          scanner), or -1 if parse state p does not read t.
 * The stack of the pushdown automaton, its pre-image and the trie index over stack values
 * (Section 4.1, last paragraphs) are outside this step.
 *
 * fsmidx_scanner_terminal_sets writes possible_out[q] = the terminals that the characters read so
 * far can still become: bit t is set iff some string, possibly empty, leads from q to a state that
 * completes t (the set V of Section 4.1, which shrinks while characters arrive).  The stream is
 * synchronised once per 4 to 64 launches; *launches_host (may be NULL) receives the number of
 * launches up to and including the first that changed nothing.
 *
 * fsmidx_scanner_restart_table writes the transition function that lets a vocabulary string finish
 * one terminal and begin the next (Section 4, the strings " " and "oo(" after "def f"):
 *     trans_out[q][c] = trans[q][c]                       if that is not dead_state,
 *                     = trans[shift[p(q)][t]][c]          otherwise, for the lowest t that q
 *                                                         completes with shift[p(q)][t] >= 0 and
 *                                                         trans[shift[p(q)][t]][c] != dead_state,
 *                     = dead_state                        if there is no such t.
 * An automaton with trans_out in place of trans (same byte_to_class, accept, dead_state) is indexed
 * by the build calls like any other.  With dead_state = -1 the table is copied.  The stream is
 * synchronised once.
 *
 *   `workspace`: device, 256-byte aligned, fsmidx_scanner_workspace_bytes(n_states, n_classes)
 * bytes; both calls overwrite it.  All arrays are DEVICE memory of the caller: completes and
 * possible_out [n_states] (different arrays), scanner_of_state [n_states], shift [n_parse_states x
 * n_terminals], trans_out [n_states x n_classes] (not the scanner's own table).  Values that would
 * serve as addresses are range checked on the device (FSMIDX_BAD_DEVICE_INPUT; the outputs are
 * then unspecified but every access stayed in bounds).
 */
int fsmidx_scanner_workspace_bytes(int32_t n_states, int32_t n_classes, size_t *bytes);
int fsmidx_scanner_terminal_sets(const fsmidx_dfa *scanner, const uint64_t *completes_dev, void *workspace,
                                 size_t workspace_bytes, uint64_t *possible_out_dev /* [n_states] */,
                                 int32_t *launches_host, void *stream);
int fsmidx_scanner_restart_table(const fsmidx_dfa *scanner, const uint64_t *completes_dev,
                                 const int32_t *scanner_of_state_dev, const int32_t *shift_dev, int32_t n_parse_states,
                                 int32_t n_terminals, void *workspace, size_t workspace_bytes,
                                 int32_t *trans_out_dev /* [n_states x n_classes] */, void *stream);

/*
 * Kernel timing for benchmarks.  After fsmidx_profile_enable(1) the calling thread's build,
 * mask_logits, advance_states, masked_argmax and masked_sample calls bracket each phase's kernels
 * with HIP events on the stream they are given (enable(0) stops that; either call resets the
 * statistics).  fsmidx_profile_read waits for the recorded events and writes, per phase, the mean
 * duration in milliseconds over the phase's launches since enabling (the most recent 128 at most)
 * and the number of launches; mean -1 = never launched.  Phases:
 *   [0] input preparation (byte classes, token records, table narrowing; Section 3, Definition 1)
 *   [1] the counting walk (Algorithm 3)          [2] the scans (bookkeeping of Algorithm 4)
 *   [3] the emitting walk (Algorithms 3 and 4)   [4] mask_logits binary32  [5] mask_logits bfloat16
 *   [6] advance_states   [7] masked_argmax binary32   [8] masked_argmax bfloat16
 *   [9] masked_sample binary32   [10] masked_sample bfloat16
 */
int fsmidx_profile_enable(int enabled);
int fsmidx_profile_read(double *mean_ms /* [11] */, int64_t *calls /* [11] */);

#ifdef __cplusplus
}
#endif
#endif /* FSMIDX_H */
