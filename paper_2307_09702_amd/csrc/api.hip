// C ABI of libfsmidx: argument checks, workspace layout, and the sequence of kernel launches that
// makes up build_index (Section 3, Algorithms 3 and 4) and mask_logits (Section 2.2).
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>

#include "internal.h"

namespace fsmidx {

static thread_local char g_error[512] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
    return code;
}

static int hip_fail(hipError_t e, const char *what)
{
    if (e == hipErrorOutOfMemory)
        return fail(FSMIDX_OUT_OF_MEMORY, "%s: %s", what, hipGetErrorString(e));
    return fail(FSMIDX_HIP_ERROR, "%s: %s", what, hipGetErrorString(e));
}

#define FSMIDX_HIP(call)                                  \
    do {                                                  \
        hipError_t e_ = (call);                           \
        if (e_ != hipSuccess) return hip_fail(e_, #call); \
    } while (0)

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

static int check_sizes(int32_t n_states, int32_t n_classes, int32_t n_tokens, int64_t n_bytes)
{
    if (n_states < 1)
        return fail(FSMIDX_INVALID_ARG, "n_states must be >= 1 (got %d)", n_states);
    if (n_classes < 1 || n_classes > 256)
        return fail(FSMIDX_INVALID_ARG, "n_classes must be in 1..256 (got %d)", n_classes);
    if ((int64_t)n_states * n_classes > 0x7FFFFFFFll)
        return fail(FSMIDX_INVALID_ARG, "transition table too large: n_states*n_classes must be < 2^31");
    if (n_tokens < 0 || n_tokens > (1 << 30))
        return fail(FSMIDX_INVALID_ARG, "n_tokens must be in 0..2^30 (got %d)", n_tokens);
    if (n_bytes < 0 || n_bytes > 0x7FFFFFFFll)
        return fail(FSMIDX_INVALID_ARG, "n_bytes must be in 0..2^31-1 (got %lld)", (long long)n_bytes);
    return FSMIDX_OK;
}

int make_plan(int32_t n_states, int32_t n_classes, int32_t n_tokens, int64_t n_bytes, Plan *p)
{
    int rc = check_sizes(n_states, n_classes, n_tokens, n_bytes);
    if (rc)
        return rc;
    p->n_states = n_states;
    p->n_classes = n_classes;
    p->n_tokens = n_tokens;
    p->n_bytes = n_bytes;
    p->entry_bytes = n_states <= 65535 ? 2 : 4;
    p->live_words = (n_classes + 63) / 64;
    p->n_blocks = (n_tokens + kBlockTokens - 1) / kBlockTokens;
    p->n_chunks = p->n_blocks * kBlockChunks;
    p->n_groups = p->n_blocks * kGroupsPerBlock;
    // Dense path: aim at ~16k units of (token group, state range) so that small problems still
    // fill the chip and the tail of large ones is short.
    int64_t spw = ((int64_t)n_states * (p->n_groups > 0 ? p->n_groups : 1) + 16383) / 16384;
    if (spw < 1) spw = 1;
    if (spw > n_states) spw = n_states;
    p->states_per_wave = (int32_t)spw;
    p->n_ranges = (n_states + p->states_per_wave - 1) / p->states_per_wave;
    if ((int64_t)p->n_groups * p->n_ranges > 0x7FFFFFFFll)
        return fail(FSMIDX_INVALID_ARG, "problem too large for one launch");
    {
        const int64_t want = (n_bytes / 16 + 255) / 256;
        p->cls_groups = (int32_t)(want < 1 ? 1 : (want > 2048 ? 2048 : want));
        p->pack_groups = (p->n_chunks * kChunkTokens + 255) / 256;
        p->narrow_groups = (n_states + 3) / 4;
    }
    size_t o = 0;
    p->off_status = o; o = align256(o + sizeof(Status));
    p->off_badw = o;   o = align256(o + ((size_t)p->cls_groups + p->pack_groups + p->narrow_groups) * 4);
    p->off_sync = o;   o = align256(o + sizeof(SyncWords));
    p->off_cls = o;    o = align256(o + (size_t)n_bytes + 16);
    p->off_tok = o;    o = align256(o + (size_t)p->n_chunks * kChunkTokens * sizeof(TokenRecord));
    p->off_key = o;    o = align256(o + (size_t)p->n_chunks * kChunkTokens * 4);
    p->off_tab = o;    o = align256(o + (size_t)n_states * n_classes * p->entry_bytes + 16);
    p->off_live = o;   o = align256(o + (size_t)n_states * p->live_words * 8);
    p->off_cnt = o;    o = align256(o + (size_t)n_states * (size_t)p->n_groups * 4);
    p->off_rowtot = o; o = align256(o + (size_t)n_states * 8);
    p->off_allow = o;  o = align256(o + (size_t)n_states * (size_t)p->n_chunks * 8);
    // The token-set path needs 64-bit class masks and 16-bit state ids; whether the automaton has
    // few enough distinct (target, class set) pairs and the vocabulary short enough tokens is
    // decided on the device.
    p->sets_possible = n_classes <= 64 && n_states <= 65535 && p->n_blocks > 0 && p->n_blocks <= kMaxSetBlocks;
    if (p->sets_possible) {
        const size_t max_pairs = (size_t)n_states * n_classes;
        p->off_npairs = o;  o = align256(o + (size_t)n_states * 4);
        p->off_pmask = o;   o = align256(o + max_pairs * 8);
        p->off_pslot = o;   o = align256(o + max_pairs * 4);
        p->off_pairs = o;   o = align256(o + max_pairs * 4 + 16);
        p->off_srec = o;    o = align256(o + (size_t)n_states * sizeof(StateRecord));
        p->off_order = o;   o = align256(o + (size_t)n_states * 4);
        p->off_clsets = o;  o = align256(o + (size_t)64 * (kSetCap / 64) * 8);
        p->off_U = o;       o = align256(o + (size_t)kMaxSetDepth * kSetCap * p->n_chunks * 8);
        p->off_E = o;       o = align256(o + (size_t)kMaxSetDepth * p->n_chunks * 8);
        p->off_long = o;    o = align256(o + (size_t)n_states * (size_t)p->n_blocks * 4);
        p->off_queue = o;   o = align256(o + (size_t)kQueues * 4);
    }
    p->total = o;
    return FSMIDX_OK;
}

static int check_structs(const fsmidx_dfa *dfa, const fsmidx_vocab *vocab)
{
    if (!dfa || !vocab)
        return fail(FSMIDX_INVALID_ARG, "dfa and vocab must not be NULL");
    int rc = check_sizes(dfa->n_states, dfa->n_classes, vocab->n_tokens, vocab->n_bytes);
    if (rc)
        return rc;
    if (!dfa->trans || !dfa->byte_to_class || !dfa->accept)
        return fail(FSMIDX_INVALID_ARG, "dfa.trans, dfa.byte_to_class and dfa.accept must not be NULL");
    if (!vocab->offsets)
        return fail(FSMIDX_INVALID_ARG, "vocab.offsets must not be NULL");
    if (vocab->n_bytes > 0 && !vocab->bytes)
        return fail(FSMIDX_INVALID_ARG, "vocab.bytes must not be NULL when n_bytes > 0");
    if (dfa->dead_state < -1 || dfa->dead_state >= dfa->n_states)
        return fail(FSMIDX_INVALID_ARG, "dead_state must be -1 or in [0, n_states) (got %d)", dfa->dead_state);
    if (vocab->eos_token_id < -1 || vocab->eos_token_id >= vocab->n_tokens)
        return fail(FSMIDX_INVALID_ARG, "eos_token_id must be -1 or in [0, n_tokens) (got %d)", vocab->eos_token_id);
    return FSMIDX_OK;
}

static const char *flag_text(uint32_t flags)
{
    if (flags & kBadTransition) return "a transition lies outside [0, n_states)";
    if (flags & kBadClass) return "a byte_to_class value is >= n_classes";
    if (flags & kBadOffsets) return "offsets are not 0 = o[0] <= o[1] <= ... <= o[n_tokens] = n_bytes";
    if (flags & kDeadNotAbsorbing) return "the dead state has a transition that leaves it";
    if (flags & 32u) return "scanner_of_state lies outside [0, n_parse_states) for a state that completes a terminal";
    if (flags & 64u) return "a shift value lies outside [-1, n_states)";
    if (flags & 128u) return "completes has a bit at or above n_terminals";
    return "unknown";
}

// Optional per-thread kernel timing with HIP events on the caller's stream.  Every phase has a
// ring of (start, stop) event pairs; each launch of the phase takes the next pair.
constexpr int kProfPhases = 11;       // prepare, count walk, scans, emit walk, mask f32, mask bf16,
                                      // advance_states, masked_argmax f32, masked_argmax bf16,
                                      // masked_sample f32, masked_sample bf16
constexpr int kProfRing = 128;
struct ProfilePhase {
    hipEvent_t start[kProfRing], stop[kProfRing];
    int created = 0;                  // event pairs that exist
    int64_t calls = 0;                // launches since profiling was enabled
};
struct Profile {
    bool enabled = false;
    ProfilePhase phase[kProfPhases];
};
static thread_local Profile g_prof;

// which = 0: record the start event of the phase's next slot; which = 1: record its stop event.
static void prof_mark(int phase, int which, hipStream_t stream)
{
    if (!g_prof.enabled)
        return;
    ProfilePhase &ph = g_prof.phase[phase];
    const int slot = (int)(ph.calls % kProfRing);
    if (slot >= ph.created) {
        if (hipEventCreate(&ph.start[slot]) != hipSuccess || hipEventCreate(&ph.stop[slot]) != hipSuccess)
            return;
        ph.created = slot + 1;
    }
    if (which == 0) {
        (void)hipEventRecord(ph.start[slot], stream);
    } else {
        (void)hipEventRecord(ph.stop[slot], stream);
        ++ph.calls;
    }
}

struct Index {
    fsmidx_csr csr;
    char *stage = nullptr;         // inputs + workspace; kept because the bitmap lives in it
    int64_t *row_ptr = nullptr;
    int32_t *token_ids = nullptr;
    int32_t *next_states = nullptr;
};

// The one value the host needs back from a counting pass.  Read through a pinned buffer (allocated
// once per thread): a copy into pageable memory goes through a staging kernel.
static hipError_t read_status(const char *ws, const Plan &p, hipStream_t stream, Status *out)
{
    static thread_local Status *pinned = nullptr;
    if (!pinned && hipHostMalloc(reinterpret_cast<void **>(&pinned), sizeof(Status), hipHostMallocDefault) != hipSuccess) {
        pinned = nullptr;
        (void)hipGetLastError();
    }
    Status *dst = pinned ? pinned : out;
    hipError_t e = hipMemcpyAsync(dst, ws + p.off_status, sizeof(Status), hipMemcpyDeviceToHost, stream);
    if (e != hipSuccess)
        return e;
    e = hipStreamSynchronize(stream);
    if (e == hipSuccess && pinned)
        *out = *pinned;
    return e;
}

// What advance_states, masked_argmax and masked_sample need of an index.
int check_rows(const fsmidx_csr *index)
{
    if (!index)
        return fail(FSMIDX_INVALID_ARG, "index must not be NULL");
    if (index->n_states < 1 || index->n_tokens < 0 || index->nnz < 0)
        return fail(FSMIDX_INVALID_ARG, "index sizes are inconsistent");
    if (!index->row_ptr)
        return fail(FSMIDX_INVALID_ARG, "index.row_ptr must not be NULL");
    if (index->nnz > 0 && (!index->token_ids || !index->next_states))
        return fail(FSMIDX_INVALID_ARG, "index.token_ids and index.next_states must not be NULL when nnz > 0");
    return FSMIDX_OK;
}

// The argument checks that both masked_argmax entry points share (everything but where the partial
// results go); *partial_bytes = the size of those partial results.
int check_argmax_call(const fsmidx_csr *index, const int32_t *states_dev, int32_t batch, const void *logits,
                      int64_t row_stride, int32_t dtype, const int32_t *tokens_out_dev, const int32_t *states_out_dev,
                      size_t *partial_bytes)
{
    if (int rc = check_rows(index))
        return rc;
    if (dtype != 0 && dtype != 1)
        return fail(FSMIDX_UNSUPPORTED, "dtype %d is not supported (0 = binary32, 1 = bfloat16)", dtype);
    if (batch < 0 || batch > kArgmaxMaxBatch)
        return fail(FSMIDX_INVALID_ARG, "batch must be in [0, %d]", kArgmaxMaxBatch);
    *partial_bytes = align256((size_t)batch * kArgmaxSplits * sizeof(uint64_t));
    if (batch == 0)
        return FSMIDX_OK;
    if (!states_dev || !logits || !tokens_out_dev || !states_out_dev)
        return fail(FSMIDX_INVALID_ARG, "states, logits, tokens_out and states_out must not be NULL");
    if (row_stride < index->n_tokens)
        return fail(FSMIDX_INVALID_ARG, "row_stride (%lld) is smaller than n_tokens (%d)", (long long)row_stride,
                    index->n_tokens);
    const size_t elem = dtype == 0 ? 4 : 2;
    if (reinterpret_cast<uintptr_t>(logits) & (elem - 1))
        return fail(FSMIDX_INVALID_ARG, "logits must be aligned to the element size");
    return FSMIDX_OK;
}

}  // namespace fsmidx

using namespace fsmidx;

struct fsmidx_index : fsmidx::Index {};

extern "C" {

const char *fsmidx_last_error(void) { return g_error; }

int fsmidx_validate_host(const fsmidx_dfa *dfa, const fsmidx_vocab *vocab)
{
    int rc = check_structs(dfa, vocab);
    if (rc)
        return rc;
    const int32_t q = dfa->n_states, c = dfa->n_classes;
    for (int b = 0; b < 256; ++b)
        if (dfa->byte_to_class[b] >= c)
            return fail(FSMIDX_INVALID_ARG, "byte_to_class[%d] = %d is >= n_classes = %d", b, dfa->byte_to_class[b], c);
    const int64_t n = (int64_t)q * c;
    for (int64_t i = 0; i < n; ++i)
        if (dfa->trans[i] < 0 || dfa->trans[i] >= q)
            return fail(FSMIDX_INVALID_ARG, "trans[%lld][%lld] = %d lies outside [0, %d)", (long long)(i / c),
                        (long long)(i % c), dfa->trans[i], q);
    if (dfa->dead_state >= 0)
        for (int32_t k = 0; k < c; ++k)
            if (dfa->trans[(int64_t)dfa->dead_state * c + k] != dfa->dead_state)
                return fail(FSMIDX_INVALID_ARG, "dead state %d is not absorbing (class %d leads to %d)", dfa->dead_state,
                            k, dfa->trans[(int64_t)dfa->dead_state * c + k]);
    const int64_t *o = vocab->offsets;
    if (o[0] != 0)
        return fail(FSMIDX_INVALID_ARG, "offsets[0] must be 0 (got %lld)", (long long)o[0]);
    for (int32_t t = 0; t < vocab->n_tokens; ++t)
        if (o[t + 1] < o[t])
            return fail(FSMIDX_INVALID_ARG, "offsets decrease at token %d", t);
    if (o[vocab->n_tokens] != vocab->n_bytes)
        return fail(FSMIDX_INVALID_ARG, "offsets[n_tokens] = %lld differs from n_bytes = %lld",
                    (long long)o[vocab->n_tokens], (long long)vocab->n_bytes);
    return FSMIDX_OK;
}

int fsmidx_profile_enable(int enabled)
{
    g_prof.enabled = enabled != 0;
    for (auto &ph : g_prof.phase)
        ph.calls = 0;
    return FSMIDX_OK;
}

int fsmidx_profile_read(double *mean_ms, int64_t *calls)
{
    if (!mean_ms || !calls)
        return fail(FSMIDX_INVALID_ARG, "mean_ms and calls must not be NULL");
    for (int k = 0; k < kProfPhases; ++k) {
        ProfilePhase &ph = g_prof.phase[k];
        calls[k] = ph.calls;
        mean_ms[k] = -1.0;
        const int n = (int)(ph.calls < kProfRing ? ph.calls : kProfRing);
        if (n == 0)
            continue;
        double sum = 0.0;
        for (int i = 0; i < n; ++i) {
            FSMIDX_HIP(hipEventSynchronize(ph.stop[i]));
            float t = 0.f;
            FSMIDX_HIP(hipEventElapsedTime(&t, ph.start[i], ph.stop[i]));
            sum += t;
        }
        mean_ms[k] = sum / n;
    }
    return FSMIDX_OK;
}

int fsmidx_build_workspace_bytes(int32_t n_states, int32_t n_classes, int32_t n_tokens, int64_t n_bytes,
                                 size_t *bytes)
{
    if (!bytes)
        return fail(FSMIDX_INVALID_ARG, "bytes must not be NULL");
    Plan p;
    int rc = make_plan(n_states, n_classes, n_tokens, n_bytes, &p);
    if (rc)
        return rc;
    *bytes = p.total;
    return FSMIDX_OK;
}

static int plan_for(const fsmidx_dfa *dfa, const fsmidx_vocab *vocab, void *workspace, size_t workspace_bytes, Plan *p)
{
    int rc = check_structs(dfa, vocab);
    if (rc)
        return rc;
    rc = make_plan(dfa->n_states, dfa->n_classes, vocab->n_tokens, vocab->n_bytes, p);
    if (rc)
        return rc;
    if (!workspace)
        return fail(FSMIDX_INVALID_ARG, "workspace must not be NULL");
    if (reinterpret_cast<uintptr_t>(workspace) & 255)
        return fail(FSMIDX_INVALID_ARG, "workspace must be 256-byte aligned");
    if (workspace_bytes < p->total)
        return fail(FSMIDX_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", workspace_bytes, p->total);
    return FSMIDX_OK;
}

// Which counting kernel the device chose the last time this thread built an index from the same
// inputs in the same workspace.  Only a hint for what to launch: the device decides afresh in every
// build, and a launch sequence that left out the kernel it then wanted is noticed (Status::overflow
// == 2) and the count is redone.  0 = unknown, 1 = token-set kernels, 2 = dense kernels.
struct PathHint {
    const void *ws = nullptr, *trans = nullptr, *bytes = nullptr;
    int32_t n_states = 0, n_classes = 0, n_tokens = 0;
    int path = 0;
};
constexpr int kPathHints = 8;
static thread_local PathHint g_hints[kPathHints];
static thread_local int g_next_hint = 0;

static PathHint *find_hint(const fsmidx_dfa *dfa, const fsmidx_vocab *vocab, const char *ws, bool create)
{
    for (PathHint &h : g_hints)
        if (h.ws == ws && h.trans == dfa->trans && h.bytes == vocab->bytes && h.n_states == dfa->n_states &&
            h.n_classes == dfa->n_classes && h.n_tokens == vocab->n_tokens)
            return &h;
    if (!create)
        return nullptr;
    PathHint &h = g_hints[g_next_hint];
    g_next_hint = (g_next_hint + 1) % kPathHints;
    h.ws = ws;
    h.trans = dfa->trans;
    h.bytes = vocab->bytes;
    h.n_states = dfa->n_states;
    h.n_classes = dfa->n_classes;
    h.n_tokens = vocab->n_tokens;
    h.path = 0;
    return &h;
}

static void remember_path(const fsmidx_dfa *dfa, const fsmidx_vocab *vocab, const char *ws, const Status &st)
{
    find_hint(dfa, vocab, ws, true)->path = (st.use_sets || st.feasible) ? 1 : 2;
}

// Everything of the counting pass, enqueued.  Without a hint both counting kernels are launched
// and the one the device did not choose returns at once; with one, only the expected kernel.
static int enqueue_count(const Plan &p, const fsmidx_dfa *dfa, const fsmidx_vocab *vocab, char *ws,
                         int64_t *row_ptr_dev, hipStream_t stream)
{
    const PathHint *hint = find_hint(dfa, vocab, ws, false);
    const int path = !p.sets_possible ? 2 : (hint ? hint->path : 0);
    prof_mark(0, 0, stream);
    FSMIDX_HIP(launch_prepare(p, *dfa, *vocab, ws, path, stream));
    if (path != 2)
        FSMIDX_HIP(launch_token_sets(p, *dfa, *vocab, ws, stream));
    prof_mark(0, 1, stream);
    prof_mark(1, 0, stream);
    if (path != 2)
        FSMIDX_HIP(launch_walk_sets(p, *dfa, *vocab, ws, false, stream));
    if (path != 1)
        FSMIDX_HIP(launch_walk(p, *dfa, *vocab, ws, stream));
    prof_mark(1, 1, stream);
    prof_mark(2, 0, stream);
    FSMIDX_HIP(launch_scan(p, ws, row_ptr_dev, stream));
    prof_mark(2, 1, stream);
    return FSMIDX_OK;
}

// The counting pass has to be redone.  A token-set walk needed more branch points than its stack
// holds (overflow 1): the first time with the deep stack, and if that overflows too (an automaton
// with deep branching) with the workspace switched to the dense kernels.  The device decided
// against the token-set kernels and the dense one had not been launched (overflow 2): the dense
// kernels at once.
static int enqueue_recount(const Plan &p, const fsmidx_dfa *dfa, const fsmidx_vocab *vocab, char *ws,
                           int64_t *row_ptr_dev, int attempt, uint32_t why, hipStream_t stream)
{
    if (attempt == 0 && why == 1) {
        FSMIDX_HIP(launch_retry_sets(p, ws, stream));
        FSMIDX_HIP(launch_walk_sets(p, *dfa, *vocab, ws, true, stream));
    } else {
        FSMIDX_HIP(launch_disable_sets(p, ws, stream));
    }
    FSMIDX_HIP(launch_walk(p, *dfa, *vocab, ws, stream));
    FSMIDX_HIP(launch_scan(p, ws, row_ptr_dev, stream));
    return FSMIDX_OK;
}

static int enqueue_emit(const Plan &p, const fsmidx_vocab *vocab, char *ws, const int64_t *row_ptr_dev,
                        int32_t *token_ids_dev, int32_t *next_states_dev, int64_t capacity, bool queues_clear,
                        hipStream_t stream)
{
    prof_mark(3, 0, stream);
    FSMIDX_HIP(launch_emit(p, *vocab, ws, row_ptr_dev, token_ids_dev, next_states_dev, capacity, queues_clear,
                           stream));
    prof_mark(3, 1, stream);
    return FSMIDX_OK;
}

int fsmidx_build_count(const fsmidx_dfa *dfa, const fsmidx_vocab *vocab, void *workspace, size_t workspace_bytes,
                       int64_t *row_ptr_dev, int64_t *nnz_host, void *stream_v)
{
    Plan p;
    int rc = plan_for(dfa, vocab, workspace, workspace_bytes, &p);
    if (rc)
        return rc;
    if (!row_ptr_dev || !nnz_host)
        return fail(FSMIDX_INVALID_ARG, "row_ptr_dev and nnz_host must not be NULL");
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    char *ws = static_cast<char *>(workspace);
    rc = enqueue_count(p, dfa, vocab, ws, row_ptr_dev, stream);
    if (rc)
        return rc;
    Status st;
    FSMIDX_HIP(read_status(ws, p, stream, &st));
    if (st.flags)
        return fail(FSMIDX_BAD_DEVICE_INPUT, "device input rejected: %s (flags 0x%x)", flag_text(st.flags), st.flags);
    for (int attempt = 0; st.overflow && attempt < 2; ++attempt) {
        rc = enqueue_recount(p, dfa, vocab, ws, row_ptr_dev, attempt, st.overflow, stream);
        if (rc)
            return rc;
        FSMIDX_HIP(read_status(ws, p, stream, &st));
    }
    remember_path(dfa, vocab, ws, st);
    *nnz_host = st.nnz;
    return FSMIDX_OK;
}

int fsmidx_build_fill(const fsmidx_dfa *dfa, const fsmidx_vocab *vocab, void *workspace, size_t workspace_bytes,
                      const int64_t *row_ptr_dev, int64_t nnz, int32_t *token_ids_dev, int32_t *next_states_dev,
                      void *stream_v)
{
    Plan p;
    int rc = plan_for(dfa, vocab, workspace, workspace_bytes, &p);
    if (rc)
        return rc;
    if (!row_ptr_dev)
        return fail(FSMIDX_INVALID_ARG, "row_ptr_dev must not be NULL");
    if (nnz < 0)
        return fail(FSMIDX_INVALID_ARG, "nnz must be >= 0");
    if (nnz == 0)
        return FSMIDX_OK;
    if (!token_ids_dev || !next_states_dev)
        return fail(FSMIDX_INVALID_ARG, "token_ids_dev and next_states_dev must not be NULL when nnz > 0");
    // a second fill on the same workspace is legitimate, so the work counters are zeroed each time
    return enqueue_emit(p, vocab, static_cast<char *>(workspace), row_ptr_dev, token_ids_dev, next_states_dev, nnz,
                        false, static_cast<hipStream_t>(stream_v));
}

static int check_build_outputs(const int64_t *row_ptr_dev, const int32_t *token_ids_dev, const int32_t *next_states_dev,
                               int64_t capacity)
{
    if (!row_ptr_dev)
        return fail(FSMIDX_INVALID_ARG, "row_ptr_dev must not be NULL");
    if (capacity < 0 || (capacity > 0 && (!token_ids_dev || !next_states_dev)))
        return fail(FSMIDX_INVALID_ARG, "capacity must be >= 0, and the two arrays must not be NULL when it is > 0");
    return FSMIDX_OK;
}

int fsmidx_build_enqueue(const fsmidx_dfa *dfa, const fsmidx_vocab *vocab, void *workspace, size_t workspace_bytes,
                         int64_t *row_ptr_dev, int32_t *token_ids_dev, int32_t *next_states_dev, int64_t capacity,
                         void *stream_v)
{
    Plan p;
    int rc = plan_for(dfa, vocab, workspace, workspace_bytes, &p);
    if (rc)
        return rc;
    if ((rc = check_build_outputs(row_ptr_dev, token_ids_dev, next_states_dev, capacity)))
        return rc;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    char *ws = static_cast<char *>(workspace);
    rc = enqueue_count(p, dfa, vocab, ws, row_ptr_dev, stream);
    if (rc)
        return rc;
    // the emit kernel itself checks, on the device, that the counting pass was clean and that the
    // entries fit; otherwise it writes nothing
    if (capacity > 0)
        rc = enqueue_emit(p, vocab, ws, row_ptr_dev, token_ids_dev, next_states_dev, capacity, true, stream);
    return rc;
}

int fsmidx_build_finish(const fsmidx_dfa *dfa, const fsmidx_vocab *vocab, void *workspace, size_t workspace_bytes,
                        int64_t *row_ptr_dev, int32_t *token_ids_dev, int32_t *next_states_dev, int64_t capacity,
                        int64_t *nnz_host, int32_t *redone_host, void *stream_v)
{
    Plan p;
    int rc = plan_for(dfa, vocab, workspace, workspace_bytes, &p);
    if (rc)
        return rc;
    if ((rc = check_build_outputs(row_ptr_dev, token_ids_dev, next_states_dev, capacity)))
        return rc;
    if (!nnz_host)
        return fail(FSMIDX_INVALID_ARG, "nnz_host must not be NULL");
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    char *ws = static_cast<char *>(workspace);
    if (redone_host)
        *redone_host = 0;
    Status st;
    FSMIDX_HIP(read_status(ws, p, stream, &st));
    if (st.flags)
        return fail(FSMIDX_BAD_DEVICE_INPUT, "device input rejected: %s (flags 0x%x)", flag_text(st.flags), st.flags);
    for (int attempt = 0; st.overflow && attempt < 2; ++attempt) {
        if (redone_host)
            *redone_host = 1;
        rc = enqueue_recount(p, dfa, vocab, ws, row_ptr_dev, attempt, st.overflow, stream);
        if (rc)
            return rc;
        if (capacity > 0) {
            rc = enqueue_emit(p, vocab, ws, row_ptr_dev, token_ids_dev, next_states_dev, capacity, true, stream);
            if (rc)
                return rc;
        }
        FSMIDX_HIP(read_status(ws, p, stream, &st));
    }
    remember_path(dfa, vocab, ws, st);
    *nnz_host = st.nnz;
    if (st.nnz > capacity)
        return fail(FSMIDX_OUTPUT_TOO_SMALL, "the index has %lld entries, the arrays hold %lld", (long long)st.nnz,
                    (long long)capacity);
    return FSMIDX_OK;
}

int fsmidx_build_into(const fsmidx_dfa *dfa, const fsmidx_vocab *vocab, void *workspace, size_t workspace_bytes,
                      int64_t *row_ptr_dev, int32_t *token_ids_dev, int32_t *next_states_dev, int64_t capacity,
                      int64_t *nnz_host, void *stream_v)
{
    if (!nnz_host)
        return fail(FSMIDX_INVALID_ARG, "row_ptr_dev and nnz_host must not be NULL");
    int rc = fsmidx_build_enqueue(dfa, vocab, workspace, workspace_bytes, row_ptr_dev, token_ids_dev, next_states_dev,
                                  capacity, stream_v);
    if (rc)
        return rc;
    return fsmidx_build_finish(dfa, vocab, workspace, workspace_bytes, row_ptr_dev, token_ids_dev, next_states_dev,
                               capacity, nnz_host, nullptr, stream_v);
}

int fsmidx_build_index(const fsmidx_dfa *dfa, const fsmidx_vocab *vocab, void *stream_v, fsmidx_index **out)
{
    if (!out)
        return fail(FSMIDX_INVALID_ARG, "out must not be NULL");
    *out = nullptr;
    int rc = fsmidx_validate_host(dfa, vocab);
    if (rc)
        return rc;
    Plan p;
    rc = make_plan(dfa->n_states, dfa->n_classes, vocab->n_tokens, vocab->n_bytes, &p);
    if (rc)
        return rc;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    const size_t n_trans = (size_t)dfa->n_states * dfa->n_classes;
    // one staging allocation: inputs followed by the workspace
    size_t o = 0;
    const size_t o_trans = o; o = align256(o + n_trans * 4);
    const size_t o_b2c = o;   o = align256(o + 256);
    const size_t o_acc = o;   o = align256(o + (size_t)dfa->n_states);
    const size_t o_bytes = o; o = align256(o + (size_t)vocab->n_bytes + 16);
    const size_t o_offs = o;  o = align256(o + ((size_t)vocab->n_tokens + 1) * 8);
    const size_t o_ws = o;    o += p.total;
    char *stage = nullptr;
    fsmidx_index *idx = new (std::nothrow) fsmidx_index();
    if (!idx)
        return fail(FSMIDX_OUT_OF_MEMORY, "host allocation failed");
    auto cleanup = [&](int code) {
        if (code != FSMIDX_OK) {
            if (stage) (void)hipFree(stage);
            if (idx->row_ptr) (void)hipFree(idx->row_ptr);
            if (idx->token_ids) (void)hipFree(idx->token_ids);
            if (idx->next_states) (void)hipFree(idx->next_states);
            delete idx;
        }
        return code;
    };
#define FSMIDX_TRY(call)                                                \
    do {                                                                \
        hipError_t e_ = (call);                                         \
        if (e_ != hipSuccess) return cleanup(hip_fail(e_, #call));      \
    } while (0)
    FSMIDX_TRY(hipMalloc(reinterpret_cast<void **>(&stage), o));
    FSMIDX_TRY(hipMalloc(reinterpret_cast<void **>(&idx->row_ptr), ((size_t)dfa->n_states + 1) * 8));
    FSMIDX_TRY(hipMemcpyAsync(stage + o_trans, dfa->trans, n_trans * 4, hipMemcpyHostToDevice, stream));
    FSMIDX_TRY(hipMemcpyAsync(stage + o_b2c, dfa->byte_to_class, 256, hipMemcpyHostToDevice, stream));
    FSMIDX_TRY(hipMemcpyAsync(stage + o_acc, dfa->accept, (size_t)dfa->n_states, hipMemcpyHostToDevice, stream));
    if (vocab->n_bytes > 0)
        FSMIDX_TRY(hipMemcpyAsync(stage + o_bytes, vocab->bytes, (size_t)vocab->n_bytes, hipMemcpyHostToDevice, stream));
    FSMIDX_TRY(hipMemcpyAsync(stage + o_offs, vocab->offsets, ((size_t)vocab->n_tokens + 1) * 8, hipMemcpyHostToDevice,
                              stream));
    fsmidx_dfa d = *dfa;
    d.trans = reinterpret_cast<const int32_t *>(stage + o_trans);
    d.byte_to_class = reinterpret_cast<const uint8_t *>(stage + o_b2c);
    d.accept = reinterpret_cast<const uint8_t *>(stage + o_acc);
    fsmidx_vocab v = *vocab;
    v.bytes = reinterpret_cast<const uint8_t *>(stage + o_bytes);
    v.offsets = reinterpret_cast<const int64_t *>(stage + o_offs);
    int64_t nnz = 0;
    rc = fsmidx_build_count(&d, &v, stage + o_ws, p.total, idx->row_ptr, &nnz, stream);
    if (rc)
        return cleanup(rc);
    if (nnz > 0) {
        FSMIDX_TRY(hipMalloc(reinterpret_cast<void **>(&idx->token_ids), (size_t)nnz * 4));
        FSMIDX_TRY(hipMalloc(reinterpret_cast<void **>(&idx->next_states), (size_t)nnz * 4));
        rc = fsmidx_build_fill(&d, &v, stage + o_ws, p.total, idx->row_ptr, nnz, idx->token_ids, idx->next_states, stream);
        if (rc)
            return cleanup(rc);
    }
    FSMIDX_TRY(hipStreamSynchronize(stream));
#undef FSMIDX_TRY
    idx->csr.n_states = dfa->n_states;
    idx->csr.n_tokens = vocab->n_tokens;
    idx->csr.nnz = nnz;
    idx->csr.row_ptr = idx->row_ptr;
    idx->csr.token_ids = idx->token_ids;
    idx->csr.next_states = idx->next_states;
    idx->csr.allow_bits = reinterpret_cast<const uint64_t *>(stage + o_ws + p.off_allow);
    idx->csr.allow_stride = p.n_chunks;
    idx->stage = stage;
    *out = idx;
    return cleanup(FSMIDX_OK);
}

int fsmidx_index_csr(const fsmidx_index *index, fsmidx_csr *view)
{
    if (!index || !view)
        return fail(FSMIDX_INVALID_ARG, "index and view must not be NULL");
    *view = index->csr;
    return FSMIDX_OK;
}

int fsmidx_index_to_host(const fsmidx_index *index, int64_t *row_ptr, int32_t *token_ids, int32_t *next_states)
{
    if (!index || !row_ptr)
        return fail(FSMIDX_INVALID_ARG, "index and row_ptr must not be NULL");
    const fsmidx_csr &c = index->csr;
    FSMIDX_HIP(hipMemcpy(row_ptr, c.row_ptr, ((size_t)c.n_states + 1) * 8, hipMemcpyDeviceToHost));
    if (c.nnz > 0) {
        if (!token_ids || !next_states)
            return fail(FSMIDX_INVALID_ARG, "token_ids and next_states must not be NULL when nnz > 0");
        FSMIDX_HIP(hipMemcpy(token_ids, c.token_ids, (size_t)c.nnz * 4, hipMemcpyDeviceToHost));
        FSMIDX_HIP(hipMemcpy(next_states, c.next_states, (size_t)c.nnz * 4, hipMemcpyDeviceToHost));
    }
    return FSMIDX_OK;
}

void fsmidx_free_index(fsmidx_index *index)
{
    if (!index)
        return;
    if (index->stage) (void)hipFree(index->stage);
    if (index->row_ptr) (void)hipFree(index->row_ptr);
    if (index->token_ids) (void)hipFree(index->token_ids);
    if (index->next_states) (void)hipFree(index->next_states);
    delete index;
}

int fsmidx_build_allow_bits(int32_t n_states, int32_t n_classes, int32_t n_tokens, int64_t n_bytes,
                            const void *workspace, const uint64_t **allow_bits, int64_t *allow_stride)
{
    if (!workspace || !allow_bits || !allow_stride)
        return fail(FSMIDX_INVALID_ARG, "workspace, allow_bits and allow_stride must not be NULL");
    Plan p;
    int rc = make_plan(n_states, n_classes, n_tokens, n_bytes, &p);
    if (rc)
        return rc;
    *allow_bits = reinterpret_cast<const uint64_t *>(static_cast<const char *>(workspace) + p.off_allow);
    *allow_stride = p.n_chunks;
    return FSMIDX_OK;
}

int fsmidx_mask_logits(const fsmidx_csr *index, const int32_t *states_dev, int32_t batch, const void *logits_in,
                       void *logits_out, int64_t row_stride, int32_t dtype, void *stream_v)
{
    if (!index)
        return fail(FSMIDX_INVALID_ARG, "index must not be NULL");
    if (dtype != 0 && dtype != 1)
        return fail(FSMIDX_UNSUPPORTED, "dtype %d is not supported (0 = binary32, 1 = bfloat16)", dtype);
    if (batch < 0)
        return fail(FSMIDX_INVALID_ARG, "batch must be >= 0");
    if (index->n_states < 1 || index->n_tokens < 0 || index->nnz < 0)
        return fail(FSMIDX_INVALID_ARG, "index sizes are inconsistent");
    if (batch == 0 || index->n_tokens == 0)
        return FSMIDX_OK;
    if (!states_dev || !logits_in || !logits_out || !index->row_ptr)
        return fail(FSMIDX_INVALID_ARG, "states, logits and index.row_ptr must not be NULL");
    if (index->nnz > 0 && !index->token_ids)
        return fail(FSMIDX_INVALID_ARG, "index.token_ids must not be NULL when nnz > 0");
    if (index->allow_bits && index->allow_stride < ((int64_t)index->n_tokens + 63) / 64)
        return fail(FSMIDX_INVALID_ARG, "index.allow_stride is smaller than ceil(n_tokens / 64)");
    if (row_stride < index->n_tokens)
        return fail(FSMIDX_INVALID_ARG, "row_stride (%lld) is smaller than n_tokens (%d)", (long long)row_stride,
                    index->n_tokens);
    const size_t elem = dtype == 0 ? 4 : 2;
    if ((reinterpret_cast<uintptr_t>(logits_in) | reinterpret_cast<uintptr_t>(logits_out)) & (elem - 1))
        return fail(FSMIDX_INVALID_ARG, "logits buffers must be aligned to the element size");
    const int64_t segs = ((int64_t)index->n_tokens + 511) / 512;       // smallest segment of any mask kernel
    if (segs * batch > 0x7FFFFFFFll)
        return fail(FSMIDX_INVALID_ARG, "batch * ceil(n_tokens / 512) must be < 2^31");
    prof_mark(4 + dtype, 0, static_cast<hipStream_t>(stream_v));
    FSMIDX_HIP(launch_mask(*index, states_dev, batch, logits_in, logits_out, row_stride, dtype,
                           static_cast<hipStream_t>(stream_v)));
    prof_mark(4 + dtype, 1, static_cast<hipStream_t>(stream_v));
    return FSMIDX_OK;
}

int fsmidx_advance_states(const fsmidx_csr *index, const int32_t *states_dev, const int32_t *tokens_dev,
                          int32_t batch, int32_t *states_out_dev, void *stream_v)
{
    if (int rc = check_rows(index))
        return rc;
    if (batch < 0)
        return fail(FSMIDX_INVALID_ARG, "batch must be >= 0");
    if (batch == 0)
        return FSMIDX_OK;
    if (!states_dev || !tokens_dev || !states_out_dev)
        return fail(FSMIDX_INVALID_ARG, "states, tokens and states_out must not be NULL");
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    prof_mark(6, 0, stream);
    FSMIDX_HIP(launch_advance(*index, states_dev, tokens_dev, batch, states_out_dev, stream));
    prof_mark(6, 1, stream);
    return FSMIDX_OK;
}

int fsmidx_masked_argmax_workspace_bytes(int32_t batch, size_t *bytes)
{
    if (!bytes)
        return fail(FSMIDX_INVALID_ARG, "bytes must not be NULL");
    if (batch < 0 || batch > kArgmaxMaxBatch)
        return fail(FSMIDX_INVALID_ARG, "batch must be in [0, %d]", kArgmaxMaxBatch);
    *bytes = align256((size_t)batch * kArgmaxSplits * sizeof(uint64_t));
    return FSMIDX_OK;
}

int fsmidx_masked_argmax(const fsmidx_csr *index, const int32_t *states_dev, int32_t batch, const void *logits,
                         int64_t row_stride, int32_t dtype, void *workspace, size_t workspace_bytes,
                         int32_t *tokens_out_dev, int32_t *states_out_dev, void *stream_v)
{
    size_t need = 0;
    if (int rc = check_argmax_call(index, states_dev, batch, logits, row_stride, dtype, tokens_out_dev, states_out_dev,
                                   &need))
        return rc;
    if (batch == 0)
        return FSMIDX_OK;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 7))
        return fail(FSMIDX_INVALID_ARG, "workspace must be a device pointer aligned to 8 bytes");
    if (workspace_bytes < need)
        return fail(FSMIDX_WORKSPACE_TOO_SMALL, "workspace holds %zu bytes, %zu are needed", workspace_bytes, need);
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    prof_mark(7 + dtype, 0, stream);
    FSMIDX_HIP(launch_argmax(*index, states_dev, batch, logits, row_stride, dtype, static_cast<uint64_t *>(workspace),
                             tokens_out_dev, states_out_dev, stream));
    prof_mark(7 + dtype, 1, stream);
    return FSMIDX_OK;
}

int fsmidx_union_workspace_bytes(int32_t n_dfas, size_t *bytes)
{
    if (!bytes)
        return fail(FSMIDX_INVALID_ARG, "bytes must not be NULL");
    if (n_dfas < 1 || n_dfas > kMaxUnion)
        return fail(FSMIDX_INVALID_ARG, "n_dfas must be in 1..%d (got %d)", kMaxUnion, n_dfas);
    *bytes = 256 + (size_t)kMaxUnion * 256;
    return FSMIDX_OK;
}

int fsmidx_union_dfa(const fsmidx_dfa *dfas, int32_t n_dfas, int32_t *trans_out_dev, int64_t trans_capacity,
                     uint8_t *byte_to_class_out_dev, uint8_t *accept_out_dev, void *workspace, size_t workspace_bytes,
                     fsmidx_dfa *union_out, int32_t *state_base_host, void *stream_v)
{
    size_t need = 0;
    if (int rc = fsmidx_union_workspace_bytes(n_dfas, &need))
        return rc;
    if (!dfas || !trans_out_dev || !byte_to_class_out_dev || !accept_out_dev || !union_out || !state_base_host)
        return fail(FSMIDX_INVALID_ARG, "dfas, the three output arrays, union_out and state_base_host must not be NULL");
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255))
        return fail(FSMIDX_INVALID_ARG, "workspace must be a 256-byte aligned device pointer");
    if (workspace_bytes < need)
        return fail(FSMIDX_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
    int64_t total = 0;
    int32_t union_dead = -1;
    for (int32_t k = 0; k < n_dfas; ++k) {
        const fsmidx_dfa &d = dfas[k];
        if (int rc = check_sizes(d.n_states, d.n_classes, 0, 0))
            return rc;
        if (!d.trans || !d.byte_to_class || !d.accept)
            return fail(FSMIDX_INVALID_ARG, "automaton %d: trans, byte_to_class and accept must not be NULL", k);
        if (d.dead_state < -1 || d.dead_state >= d.n_states)
            return fail(FSMIDX_INVALID_ARG, "automaton %d: dead_state must be -1 or in [0, n_states)", k);
        state_base_host[k] = (int32_t)total;
        if (union_dead < 0 && d.dead_state >= 0)
            union_dead = (int32_t)total + d.dead_state;
        total += d.n_states;
        if (total > 0x7FFFFFFFll)
            return fail(FSMIDX_INVALID_ARG, "the union has more than 2^31 - 1 states");
    }
    state_base_host[n_dfas] = (int32_t)total;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    char *ws = static_cast<char *>(workspace);
    FSMIDX_HIP(launch_union_classes(dfas, n_dfas, byte_to_class_out_dev, ws, stream));
    uint32_t words[2] = {0, 0};
    FSMIDX_HIP(hipMemcpyAsync(words, ws, sizeof(words), hipMemcpyDeviceToHost, stream));
    FSMIDX_HIP(hipStreamSynchronize(stream));
    if (words[1])
        return fail(FSMIDX_BAD_DEVICE_INPUT, "device input rejected: %s (flags 0x%x)", flag_text(words[1]), words[1]);
    const int32_t n_classes = (int32_t)words[0];
    if (n_classes < 1 || n_classes > 256)
        return fail(FSMIDX_HIP_ERROR, "the union's class count came back as %d", n_classes);
    if (total * n_classes > trans_capacity)
        return fail(FSMIDX_OUTPUT_TOO_SMALL, "the union's table has %lld x %d entries, trans_out holds %lld",
                    (long long)total, n_classes, (long long)trans_capacity);
    if (total * n_classes > 0x7FFFFFFFll)
        return fail(FSMIDX_INVALID_ARG, "transition table too large: n_states*n_classes must be < 2^31");
    FSMIDX_HIP(launch_union_table(dfas, n_dfas, state_base_host, union_dead, n_classes, trans_out_dev, accept_out_dev, ws,
                                  stream));
    FSMIDX_HIP(hipMemcpyAsync(words, ws, sizeof(words), hipMemcpyDeviceToHost, stream));
    FSMIDX_HIP(hipStreamSynchronize(stream));
    if (words[1])
        return fail(FSMIDX_BAD_DEVICE_INPUT, "device input rejected: %s (flags 0x%x)", flag_text(words[1]), words[1]);
    union_out->trans = trans_out_dev;
    union_out->n_states = (int32_t)total;
    union_out->n_classes = n_classes;
    union_out->byte_to_class = byte_to_class_out_dev;
    union_out->accept = accept_out_dev;
    union_out->dead_state = union_dead;
    return FSMIDX_OK;
}

int fsmidx_dedupe_workspace_bytes(int32_t n_states, size_t *bytes)
{
    if (!bytes)
        return fail(FSMIDX_INVALID_ARG, "bytes must not be NULL");
    if (n_states < 1 || n_states > kDedupeMaxStates)
        return fail(FSMIDX_INVALID_ARG, "n_states must be in 1..%d (got %d)", kDedupeMaxStates, n_states);
    *bytes = align256(dedupe_workspace_bytes(n_states));
    return FSMIDX_OK;
}

int fsmidx_dedupe_rows(const fsmidx_csr *index, void *workspace, size_t workspace_bytes, int32_t *row_of_state_dev,
                       int64_t *unique_row_ptr_dev, int32_t *n_unique_host, int64_t *nnz_unique_host, void *stream_v)
{
    if (int rc = check_rows(index))
        return rc;
    size_t need = 0;
    if (int rc = fsmidx_dedupe_workspace_bytes(index->n_states, &need))
        return rc;
    if (!row_of_state_dev || !unique_row_ptr_dev || !n_unique_host || !nnz_unique_host)
        return fail(FSMIDX_INVALID_ARG, "row_of_state, unique_row_ptr, n_unique_host and nnz_unique_host must not be NULL");
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255))
        return fail(FSMIDX_INVALID_ARG, "workspace must be a 256-byte aligned device pointer");
    if (workspace_bytes < need)
        return fail(FSMIDX_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    char *ws = static_cast<char *>(workspace);
    // Rows are grouped by a 64-bit hash and then compared entry by entry; two different rows with
    // one hash (a chance of about states^2 / 2^64) make the pass start again with another seed.
    for (uint64_t attempt = 0; attempt < 4; ++attempt) {
        FSMIDX_HIP(launch_dedupe(*index, ws, 0x243F6A8885A308D3ull + attempt * 0x9E3779B97F4A7C15ull, row_of_state_dev,
                                 unique_row_ptr_dev, stream));
        int64_t result[3] = {0, 0, 0};
        FSMIDX_HIP(hipMemcpyAsync(result, ws, sizeof(result), hipMemcpyDeviceToHost, stream));
        FSMIDX_HIP(hipStreamSynchronize(stream));
        if (result[2] == 0) {
            *n_unique_host = (int32_t)result[0];
            *nnz_unique_host = result[1];
            return FSMIDX_OK;
        }
    }
    return fail(FSMIDX_HIP_ERROR, "row hashes collided four times in a row");
}

int fsmidx_dedupe_fill(const fsmidx_csr *index, const void *workspace, size_t workspace_bytes,
                       const int64_t *unique_row_ptr_dev, int32_t *token_ids_out_dev, int32_t *next_states_out_dev,
                       void *stream_v)
{
    if (int rc = check_rows(index))
        return rc;
    size_t need = 0;
    if (int rc = fsmidx_dedupe_workspace_bytes(index->n_states, &need))
        return rc;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) || workspace_bytes < need)
        return fail(FSMIDX_INVALID_ARG, "workspace must be the one fsmidx_dedupe_rows has filled");
    if (!unique_row_ptr_dev)
        return fail(FSMIDX_INVALID_ARG, "unique_row_ptr must not be NULL");
    if (index->nnz == 0)
        return FSMIDX_OK;
    if (!token_ids_out_dev || !next_states_out_dev)
        return fail(FSMIDX_INVALID_ARG, "token_ids_out and next_states_out must not be NULL when the index has entries");
    FSMIDX_HIP(launch_dedupe_copy(*index, const_cast<char *>(static_cast<const char *>(workspace)), unique_row_ptr_dev,
                                  token_ids_out_dev, next_states_out_dev, static_cast<hipStream_t>(stream_v)));
    return FSMIDX_OK;
}

static int check_scanner(const fsmidx_dfa *dfa, const uint64_t *completes_dev, void *workspace, size_t workspace_bytes)
{
    if (!dfa)
        return fail(FSMIDX_INVALID_ARG, "scanner must not be NULL");
    if (int rc = check_sizes(dfa->n_states, dfa->n_classes, 0, 0))
        return rc;
    if (!dfa->trans)
        return fail(FSMIDX_INVALID_ARG, "scanner.trans must not be NULL");
    if (dfa->dead_state < -1 || dfa->dead_state >= dfa->n_states)
        return fail(FSMIDX_INVALID_ARG, "dead_state must be -1 or in [0, n_states) (got %d)", dfa->dead_state);
    if (!completes_dev)
        return fail(FSMIDX_INVALID_ARG, "completes must not be NULL");
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255))
        return fail(FSMIDX_INVALID_ARG, "workspace must be a 256-byte aligned device pointer");
    const size_t need = scanner_workspace_bytes(dfa->n_states, dfa->n_classes);
    if (workspace_bytes < need)
        return fail(FSMIDX_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
    return FSMIDX_OK;
}

int fsmidx_scanner_workspace_bytes(int32_t n_states, int32_t n_classes, size_t *bytes)
{
    if (!bytes)
        return fail(FSMIDX_INVALID_ARG, "bytes must not be NULL");
    if (int rc = check_sizes(n_states, n_classes, 0, 0))
        return rc;
    *bytes = scanner_workspace_bytes(n_states, n_classes);
    return FSMIDX_OK;
}

int fsmidx_scanner_terminal_sets(const fsmidx_dfa *scanner, const uint64_t *completes_dev, void *workspace,
                                 size_t workspace_bytes, uint64_t *possible_out_dev, int32_t *launches_host,
                                 void *stream_v)
{
    if (int rc = check_scanner(scanner, completes_dev, workspace, workspace_bytes))
        return rc;
    if (!possible_out_dev)
        return fail(FSMIDX_INVALID_ARG, "possible_out must not be NULL");
    if (static_cast<const void *>(possible_out_dev) == static_cast<const void *>(completes_dev))
        return fail(FSMIDX_INVALID_ARG, "possible_out must not be the completes array");
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    char *ws = static_cast<char *>(workspace);
    FSMIDX_HIP(launch_scanner_start(*scanner, completes_dev, ws, possible_out_dev, stream));
    // Launches are enqueued in batches (4, then twice as many each time, 64 at most); one that finds
    // nothing to change makes those after it return at once, and tells the host that the sets are
    // final.  Every launch before that one moves some terminal at least one state further back, so
    // 64 n_states launches are always enough.
    int batch = 4;
    int64_t launched = 0;
    uint32_t flags = 0;
    for (;;) {
        FSMIDX_HIP(launch_scanner_sweeps(*scanner, ws, possible_out_dev, batch, stream));
        uint32_t changed[64];
        FSMIDX_HIP(hipMemcpyAsync(changed, scanner_changed(ws), (size_t)batch * 4, hipMemcpyDeviceToHost, stream));
        FSMIDX_HIP(hipMemcpyAsync(&flags, scanner_flags(ws), 4, hipMemcpyDeviceToHost, stream));
        FSMIDX_HIP(hipStreamSynchronize(stream));
        if (flags)
            return fail(FSMIDX_BAD_DEVICE_INPUT, "device input rejected: %s (flags 0x%x)", flag_text(flags), flags);
        bool done = false;
        for (int i = 0; i < batch && !done; ++i) {
            ++launched;
            done = changed[i] == 0;
        }
        if (done)
            break;
        if (launched > 64ll * scanner->n_states + 64)
            return fail(FSMIDX_HIP_ERROR, "the terminal sets did not settle");
        if (batch < scanner_launches_max())
            batch *= 2;
    }
    if (launches_host)
        *launches_host = (int32_t)(launched > 0x7FFFFFFF ? 0x7FFFFFFF : launched);
    return FSMIDX_OK;
}

int fsmidx_scanner_restart_table(const fsmidx_dfa *scanner, const uint64_t *completes_dev,
                                 const int32_t *scanner_of_state_dev, const int32_t *shift_dev, int32_t n_parse_states,
                                 int32_t n_terminals, void *workspace, size_t workspace_bytes, int32_t *trans_out_dev,
                                 void *stream_v)
{
    if (int rc = check_scanner(scanner, completes_dev, workspace, workspace_bytes))
        return rc;
    if (n_terminals < 1 || n_terminals > 64)
        return fail(FSMIDX_INVALID_ARG, "n_terminals must be in [1, 64] (got %d)", n_terminals);
    if (n_parse_states < 1 || (int64_t)n_parse_states * n_terminals > 0x7FFFFFFFll)
        return fail(FSMIDX_INVALID_ARG, "n_parse_states must be at least 1 and n_parse_states x n_terminals below 2^31");
    if (!scanner_of_state_dev || !shift_dev || !trans_out_dev)
        return fail(FSMIDX_INVALID_ARG, "scanner_of_state, shift and trans_out must not be NULL");
    if (trans_out_dev == scanner->trans)
        return fail(FSMIDX_INVALID_ARG, "trans_out must not be the scanner's own table");
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    char *ws = static_cast<char *>(workspace);
    FSMIDX_HIP(launch_scanner_restarts(*scanner, completes_dev, scanner_of_state_dev, shift_dev, n_parse_states, n_terminals,
                                       trans_out_dev, ws, stream));
    uint32_t flags = 0;
    FSMIDX_HIP(hipMemcpyAsync(&flags, scanner_flags(ws), 4, hipMemcpyDeviceToHost, stream));
    FSMIDX_HIP(hipStreamSynchronize(stream));
    if (flags)
        return fail(FSMIDX_BAD_DEVICE_INPUT, "device input rejected: %s (flags 0x%x)", flag_text(flags), flags);
    return FSMIDX_OK;
}

int fsmidx_minimise_workspace_bytes(int32_t n_states, size_t *bytes)
{
    if (!bytes)
        return fail(FSMIDX_INVALID_ARG, "bytes must not be NULL");
    if (n_states < 1 || n_states > kDedupeMaxStates)
        return fail(FSMIDX_INVALID_ARG, "n_states must be in [1, %d]", kDedupeMaxStates);
    *bytes = minimise_workspace_bytes(n_states);
    return FSMIDX_OK;
}

int fsmidx_minimise_dfa(const fsmidx_dfa *dfa, void *workspace, size_t workspace_bytes, int32_t *block_of_state_dev,
                        int32_t *trans_out_dev, int64_t trans_capacity, uint8_t *accept_out_dev, fsmidx_dfa *min_out,
                        void *stream_v)
{
    if (!dfa || !min_out)
        return fail(FSMIDX_INVALID_ARG, "dfa and min_out must not be NULL");
    if (int rc = check_sizes(dfa->n_states, dfa->n_classes, 0, 0))
        return rc;
    size_t need = 0;
    if (int rc = fsmidx_minimise_workspace_bytes(dfa->n_states, &need))
        return rc;
    if (!dfa->trans || !dfa->byte_to_class || !dfa->accept)
        return fail(FSMIDX_INVALID_ARG, "dfa.trans, dfa.byte_to_class and dfa.accept must not be NULL");
    if (dfa->dead_state < -1 || dfa->dead_state >= dfa->n_states)
        return fail(FSMIDX_INVALID_ARG, "dead_state must be -1 or in [0, n_states) (got %d)", dfa->dead_state);
    if (!block_of_state_dev || !trans_out_dev || !accept_out_dev || trans_capacity < 0)
        return fail(FSMIDX_INVALID_ARG, "block_of_state, trans_out and accept_out must not be NULL");
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255))
        return fail(FSMIDX_INVALID_ARG, "workspace must be a 256-byte aligned device pointer");
    if (workspace_bytes < need)
        return fail(FSMIDX_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    char *ws = static_cast<char *>(workspace);
    // Signatures are grouped by a 64-bit hash and then compared class by class; two different
    // signatures with one hash make the whole refinement start again with another seed.
    for (uint64_t attempt = 0; attempt < 4; ++attempt) {
        const uint64_t seed = 0x452821E638D01377ull + attempt * 0x9E3779B97F4A7C15ull;
        FSMIDX_HIP(launch_min_start(*dfa, ws, attempt == 0, stream));
        // Rounds are enqueued in batches (8, 8, 16, 32, then 64 at a time); after each the host reads
        // the class counts of its rounds.  The partition is final once a round leaves the count
        // unchanged; rounds enqueued after that one change nothing.  Every round before splits a
        // class, so n_states rounds are always enough.
        int64_t classes = -1;
        bool collided = false, done = false;
        uint32_t round = 0;
        int batch = 8;
        while (!done && !collided) {
            FSMIDX_HIP(launch_min_rounds(*dfa, ws, seed, round, batch, stream));
            int64_t result[3] = {0, 0, 0};
            uint32_t counts[64];
            FSMIDX_HIP(hipMemcpyAsync(result, min_result(ws, dfa->n_states), sizeof(result), hipMemcpyDeviceToHost, stream));
            FSMIDX_HIP(hipMemcpyAsync(counts, min_counts(ws, dfa->n_states) + round % (uint32_t)min_rounds_max(),
                                      (size_t)batch * 4, hipMemcpyDeviceToHost, stream));
            FSMIDX_HIP(hipStreamSynchronize(stream));
            if (result[1])
                return fail(FSMIDX_BAD_DEVICE_INPUT, "device input rejected: %s (flags 0x%x)", flag_text((uint32_t)result[1]),
                            (uint32_t)result[1]);
            collided = result[2] != 0;
            for (int r = 0; r < batch && !done; ++r) {
                done = (int64_t)counts[r] == classes;
                classes = counts[r];
            }
            round += (uint32_t)batch;
            if (round >= 16 && batch < 64)
                batch *= 2;
            if (!done && round > (uint32_t)dfa->n_states + 128u)
                return fail(FSMIDX_HIP_ERROR, "the refinement did not end");
        }
        if (collided)
            continue;
        if (classes < 1 || classes > dfa->n_states)
            return fail(FSMIDX_HIP_ERROR, "the class count came back as %lld", (long long)classes);
        if (classes * dfa->n_classes > trans_capacity)
            return fail(FSMIDX_OUTPUT_TOO_SMALL, "the quotient's table has %lld x %d entries, trans_out holds %lld",
                        (long long)classes, dfa->n_classes, (long long)trans_capacity);
        FSMIDX_HIP(launch_min_quotient(*dfa, ws, block_of_state_dev, trans_out_dev, trans_capacity, accept_out_dev, stream));
        uint32_t dead_class = 0;
        if (dfa->dead_state >= 0)
            FSMIDX_HIP(hipMemcpyAsync(&dead_class, min_block(ws, dfa->n_states) + dfa->dead_state, 4, hipMemcpyDeviceToHost,
                                      stream));
        FSMIDX_HIP(hipStreamSynchronize(stream));
        min_out->trans = trans_out_dev;
        min_out->n_states = (int32_t)classes;
        min_out->n_classes = dfa->n_classes;
        min_out->byte_to_class = dfa->byte_to_class;
        min_out->accept = accept_out_dev;
        min_out->dead_state = dfa->dead_state >= 0 ? (int32_t)dead_class : -1;
        return FSMIDX_OK;
    }
    return fail(FSMIDX_HIP_ERROR, "signature hashes collided four times in a row");
}

int fsmidx_reach_workspace_bytes(int32_t n_states, size_t *bytes)
{
    if (!bytes)
        return fail(FSMIDX_INVALID_ARG, "bytes must not be NULL");
    if (n_states < 1 || n_states > kDedupeMaxStates)
        return fail(FSMIDX_INVALID_ARG, "n_states must be in [1, %d]", kDedupeMaxStates);
    *bytes = reach_workspace_bytes(n_states);
    return FSMIDX_OK;
}

static int check_reach_workspace(const fsmidx_csr *index, const void *workspace, size_t workspace_bytes)
{
    if (int rc = check_rows(index))
        return rc;
    size_t need = 0;
    if (int rc = fsmidx_reach_workspace_bytes(index->n_states, &need))
        return rc;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255))
        return fail(FSMIDX_INVALID_ARG, "workspace must be a 256-byte aligned device pointer");
    if (workspace_bytes < need)
        return fail(FSMIDX_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
    return FSMIDX_OK;
}

int fsmidx_reachable_states(const fsmidx_csr *index, const int32_t *start_states_host, int32_t n_starts, void *workspace,
                            size_t workspace_bytes, uint8_t *reach_out_dev, int32_t *n_reached_host, void *stream_v)
{
    if (int rc = check_reach_workspace(index, workspace, workspace_bytes))
        return rc;
    if (!reach_out_dev || !n_reached_host)
        return fail(FSMIDX_INVALID_ARG, "reach_out and n_reached_host must not be NULL");
    if (n_starts < 0 || n_starts > index->n_states || (n_starts > 0 && !start_states_host))
        return fail(FSMIDX_INVALID_ARG, "n_starts must be in [0, n_states] and start_states must not be NULL");
    for (int32_t i = 0; i < n_starts; ++i)
        if (start_states_host[i] < 0 || start_states_host[i] >= index->n_states)
            return fail(FSMIDX_INVALID_ARG, "start state %d lies outside [0, %d)", start_states_host[i], index->n_states);
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    char *ws = static_cast<char *>(workspace);
    FSMIDX_HIP(launch_reach_start(*index, ws, start_states_host, n_starts, stream));
    // A level is one launch that reads its frontier's length from memory, so several are enqueued
    // before the host looks whether the search has ended (a level with an empty frontier does
    // nothing, and neither does any level after it): 8 at first, then twice as many each time, 64
    // at most.  Every level but the last reaches a new state, so n_states levels are always enough.
    int batch = 8;
    uint32_t level = 0, pending = (uint32_t)n_starts;
    for (;;) {
        FSMIDX_HIP(launch_reach_levels(*index, ws, level, batch, pending, stream));
        level += (uint32_t)batch;
        FSMIDX_HIP(hipMemcpyAsync(&pending, reach_next_count(ws, index->n_states, level), 4, hipMemcpyDeviceToHost, stream));
        FSMIDX_HIP(hipStreamSynchronize(stream));
        if (pending == 0)
            break;
        if (level > (uint32_t)index->n_states + 64u)
            return fail(FSMIDX_HIP_ERROR, "the search for reachable states did not end");
        if (batch < 64)
            batch *= 2;
    }
    FSMIDX_HIP(launch_reach_finish(*index, ws, reach_out_dev, stream));
    int64_t reached = 0;
    FSMIDX_HIP(hipMemcpyAsync(&reached, ws, 8, hipMemcpyDeviceToHost, stream));
    FSMIDX_HIP(hipStreamSynchronize(stream));
    *n_reached_host = (int32_t)reached;
    return FSMIDX_OK;
}

int fsmidx_restrict_rows(const fsmidx_csr *index, const uint8_t *keep_dev, void *workspace, size_t workspace_bytes,
                         int64_t *row_ptr_out_dev, int64_t *nnz_out_host, void *stream_v)
{
    if (int rc = check_reach_workspace(index, workspace, workspace_bytes))
        return rc;
    if (!keep_dev || !row_ptr_out_dev || !nnz_out_host)
        return fail(FSMIDX_INVALID_ARG, "keep, row_ptr_out and nnz_out_host must not be NULL");
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    char *ws = static_cast<char *>(workspace);
    FSMIDX_HIP(launch_restrict_scan(*index, keep_dev, ws, row_ptr_out_dev, stream));
    int64_t result[2] = {0, 0};
    FSMIDX_HIP(hipMemcpyAsync(result, ws, sizeof(result), hipMemcpyDeviceToHost, stream));
    FSMIDX_HIP(hipStreamSynchronize(stream));
    *nnz_out_host = result[1];
    return FSMIDX_OK;
}

int fsmidx_restrict_fill(const fsmidx_csr *index, const uint8_t *keep_dev, const int64_t *row_ptr_out_dev,
                         int32_t *token_ids_out_dev, int32_t *next_states_out_dev, int64_t capacity, void *stream_v)
{
    if (int rc = check_rows(index))
        return rc;
    if (!keep_dev || !row_ptr_out_dev)
        return fail(FSMIDX_INVALID_ARG, "keep and row_ptr_out must not be NULL");
    if (capacity < 0)
        return fail(FSMIDX_INVALID_ARG, "capacity must not be negative");
    if (index->nnz == 0 || capacity == 0)
        return FSMIDX_OK;
    if (!token_ids_out_dev || !next_states_out_dev)
        return fail(FSMIDX_INVALID_ARG, "token_ids_out and next_states_out must not be NULL when there are entries to copy");
    if (index->n_states > kDedupeMaxStates)
        return fail(FSMIDX_INVALID_ARG, "n_states must be at most %d", kDedupeMaxStates);
    FSMIDX_HIP(launch_restrict_copy(*index, keep_dev, row_ptr_out_dev, token_ids_out_dev, next_states_out_dev, capacity,
                                    static_cast<hipStream_t>(stream_v)));
    return FSMIDX_OK;
}

int fsmidx_masked_sample_workspace_bytes(int32_t batch, size_t *bytes)
{
    if (!bytes)
        return fail(FSMIDX_INVALID_ARG, "bytes must not be NULL");
    if (batch < 0 || batch > kArgmaxMaxBatch)
        return fail(FSMIDX_INVALID_ARG, "batch must be in [0, %d]", kArgmaxMaxBatch);
    *bytes = align256((size_t)batch * kArgmaxSplits * (sizeof(uint64_t) + sizeof(double)));
    return FSMIDX_OK;
}

int fsmidx_masked_sample(const fsmidx_csr *index, const int32_t *states_dev, int32_t batch, const void *logits,
                         int64_t row_stride, int32_t dtype, const float *uniforms_dev, void *workspace,
                         size_t workspace_bytes, int32_t *tokens_out_dev, int32_t *states_out_dev, void *stream_v)
{
    if (int rc = check_rows(index))
        return rc;
    if (dtype != 0 && dtype != 1)
        return fail(FSMIDX_UNSUPPORTED, "dtype %d is not supported (0 = binary32, 1 = bfloat16)", dtype);
    size_t need = 0;
    if (int rc = fsmidx_masked_sample_workspace_bytes(batch, &need))
        return rc;
    if (batch == 0)
        return FSMIDX_OK;
    if (!states_dev || !logits || !uniforms_dev || !tokens_out_dev || !states_out_dev)
        return fail(FSMIDX_INVALID_ARG, "states, logits, uniforms, tokens_out and states_out must not be NULL");
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 7))
        return fail(FSMIDX_INVALID_ARG, "workspace must be a device pointer aligned to 8 bytes");
    if (workspace_bytes < need)
        return fail(FSMIDX_WORKSPACE_TOO_SMALL, "workspace holds %zu bytes, %zu are needed", workspace_bytes, need);
    if (row_stride < index->n_tokens)
        return fail(FSMIDX_INVALID_ARG, "row_stride (%lld) is smaller than n_tokens (%d)", (long long)row_stride,
                    index->n_tokens);
    const size_t elem = dtype == 0 ? 4 : 2;
    if (reinterpret_cast<uintptr_t>(logits) & (elem - 1))
        return fail(FSMIDX_INVALID_ARG, "logits must be aligned to the element size");
    if (reinterpret_cast<uintptr_t>(uniforms_dev) & 3)
        return fail(FSMIDX_INVALID_ARG, "uniforms must be aligned to 4 bytes");
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    uint64_t *partial = static_cast<uint64_t *>(workspace);
    double *sums = reinterpret_cast<double *>(partial + (size_t)batch * kArgmaxSplits);
    prof_mark(9 + dtype, 0, stream);
    FSMIDX_HIP(launch_sample(*index, states_dev, batch, logits, row_stride, dtype, uniforms_dev, partial, sums,
                             tokens_out_dev, states_out_dev, stream));
    prof_mark(9 + dtype, 1, stream);
    return FSMIDX_OK;
}

}  // extern "C"
