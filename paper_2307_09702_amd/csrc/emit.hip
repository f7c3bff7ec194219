// Second pass of the build: sigma (Algorithm 4) written out as a CSR.
//
// The counting pass has left the index as a bitmap (one bit per (state, token): admissible or
// not), the number of admissible tokens per (state, token group) turned into offsets by the scans,
// and row_ptr.  What is missing is the end state of every admissible pair, the last element of
// Algorithm 3's state sequence.  This kernel walks exactly the admissible pairs, one lane per pair,
// through the narrowed transition table and stores (token id, end state) at
// row_ptr[q] + offset[q][block] + rank.  None of these walks can meet the dead state.
//
// Two ways to find the end states, one kernel (every workgroup is one wave):
//
//  walking   A wave owns one state q and kWalkBlocks consecutive blocks of 4096 tokens (most
//      segments have a dozen entries, and a wave costs the same few memory round trips whatever
//      it carries):
//   1. per block, lane l loads the admissibility word of tokens [64 l, 64 l + 64); prefix sums
//      over the lanes give every word's first rank and the number n of entries of the span;
//   2. the words are expanded into a list of token numbers in rank order (LDS; a part of at most
//      kEmitPart entries at a time);
//   3. lanes take ranks, two at a time so that two table lookups are in flight per lane: load the
//      token's record, walk its classes through the narrowed table (read through L1/L2: it is
//      small and hot), store.  Consecutive lanes hold consecutive ranks, so every store is
//      coalesced and every output line is written once.  The EOS token and empty tokens have
//      length 0, so an admissible EOS comes out with the state itself as its end state.
//
//  searching (token-set path only)  A segment (state, block) with more than kLongRow entries costs
//      the walk one table lookup per byte of every token, and lookups are 4 lanes per clock.  The
//      token-set search finds the same end states for whole sets of tokens at once: it is repeated
//      restricted to the admissible tokens; a node's end state is the same for all tokens that end
//      there, so a token only has to remember the number of its node (six bit planes in
//      registers; number 0, no bits, for the end state expected to be the most common), and a last
//      step turns the planes into (token id, end state) in token order.  The entries leave
//      through LDS, 16 bytes per lane and with the non-temporal hint: this output is most of what
//      the kernel writes, and written the ordinary way it passes through the L2s and evicts the
//      bitmaps, records and table that the searches and walks read again and again.
//      The scan has listed these segments; the first workgroups of the grid take them from the
//      list one by one, so the longest work starts first, and the walking workgroups skip them.
#include "search.h"

namespace fsmidx {

constexpr int kLongGrid = 256 * 14;    // workgroups that share out the list of searched segments
constexpr int kNodeBits = 6;           // bit planes of a token's node number in a searched segment
constexpr int kDirectNode = (1 << kNodeBits) - 1;   // the number that says: stored directly, not through a node
constexpr int kFlush = 4 * kWave;      // entries of a searched segment that leave LDS together
constexpr int kEmitPart = 1024;        // entries expanded into LDS at a time
constexpr int kEmitK = 2;              // ranks per lane in flight
constexpr int kDeferCap = 256;         // walks of more than two bytes put aside at a time (dense path)
constexpr int kSpanTarget = 8192;      // walked spans (times parts) a launch should at least have
constexpr int kMaxParts = 16;
constexpr int kWalkBlocks = 4;         // consecutive blocks of a row that one wave walks (token numbers fit 16 bits)

// four 32-bit values stored with one instruction at an address that is only 4-byte aligned
typedef int32_t Int4 __attribute__((ext_vector_type(4), aligned(4)));

struct EmitArgs {
    const Status *st;
    uint32_t *queue;             // [kQueues] work counters of the searched segments, zero at launch
    const uint32_t *cnt;       // offsets of the token groups within a row (after the scans)
    const int64_t *row_ptr;
    int32_t *token_ids;
    int32_t *next_states;
    const uint32_t *long_items;  // [Status::n_long] state << 12 | block: segments emitted by search
    const uint32_t *order;       // [n_states] token-set path: the states, those with most pairs first
    int32_t n_states, n_classes, n_blocks, n_chunks, n_groups, eos;
    uint32_t n_long_groups;      // workgroups at the front of the grid that take the searched segments
    uint32_t parts;              // waves that share one walked span (1 unless the problem is small)
    int64_t capacity;            // entries the output arrays hold
};

// LDS of one workgroup (= wave); the two ways of working never meet in one workgroup.
union alignas(16) EmitShared {
    struct {
        uint16_t list[kEmitPart];             // walking: token numbers of a part, rank order
        uint32_t row[256];                    //          row q of the table: the state after a token's first byte
        uint32_t later_state[kDeferCap];      //          walks put aside: state after two bytes ...
        uint16_t later_rank[kDeferCap];       //          ... and rank within the part
    } walk;
    struct {
        uint32_t node_state[kDirectNode + 1]; // searching: end state of every node
        uint32_t spread[16];                  //            byte i of entry x = bit i of x
        union {
            uint8_t node_of[kBlockTokens];    //            per token of the block, the node it ended in
            uint64_t stack[kStackFrames * kWave];   //        (before that: the search's stack)
        };
        alignas(16) uint32_t stage[kFlush + kWave];   //     entries on their way out, rank order
        uint32_t next;                        //            the segment this wave works on
    } search;
};

// Where the ranks of a walked span of kWalkBlocks blocks go: block w holds ranks
// [start[w], start[w + 1]) of the span and writes them from position base[w] of the output.
struct SpanOut {
    uint32_t start[kWalkBlocks + 1];
    int64_t base[kWalkBlocks];
};

// Where entry r of the span goes.
__device__ __forceinline__ int64_t span_pos(const SpanOut &out, const uint32_t r)
{
    int64_t pos = out.base[0] + r;
#pragma unroll
    for (int w = 1; w < kWalkBlocks; ++w)
        if (r >= out.start[w])
            pos = out.base[w] + (r - out.start[w]);
    return pos;
}

// Ranks g0 + k * 64 + lane (k < K) of the list: load the token records, walk, store.  The first
// byte is looked up in row q, which is in LDS; the next two bytes are looked up by every lane, and
// the bytes after them only if some token of the wave is that long.
template <typename E, int K>
__device__ __forceinline__ void walk_ranks(const EmitArgs &a, const TokenRecord *__restrict__ tok_b,
                                           const uint8_t *__restrict__ cls, const E *__restrict__ tab,
                                           const uint16_t *list, const uint32_t *row_q, const int32_t q,
                                           const int32_t token0, const int lane,
                                           const SpanOut &out, const uint32_t r0, const uint32_t g0, const uint32_t r1,
                                           const uint32_t n_classes)
{
    uint32_t t[K], s[K], len[K], kk[K];
    uint32_t off[K];
    uint64_t pk[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const uint32_t r = g0 + (uint32_t)(k * kWave + lane);
        t[k] = r < r1 ? (uint32_t)list[r - r0] : 0u;
    }
    // the record, and from it the short form the first bytes are read from: the classes of the
    // first three bytes and the length (255: 255 bytes or more)
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const TokenRecord rec = tok_b[t[k]];
        pk[k] = ((uint64_t)rec.cls_hi << 32) | rec.cls_lo;
        off[k] = rec.offset;
        kk[k] = (rec.cls_lo & 0xFFFFFFu) | (rec.length < 255u ? rec.length : 255u) << 24;
        len[k] = rec.length;                                // (kept for the long ones below)
    }
    uint32_t real_len[K];
#pragma unroll
    for (int k = 0; k < K; ++k)
        real_len[k] = len[k];
    bool any_long = false;
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const uint32_t r = g0 + (uint32_t)(k * kWave + lane);
        len[k] = r < r1 ? kk[k] >> 24 : 0u;                 // (255: more than 254 bytes, see the record)
        // (EOS and empty tokens have length 0: the end state is the state itself)
        s[k] = len[k] != 0u ? row_q[kk[k] & 255u] : (uint32_t)q;
        any_long = any_long || len[k] > 3u;
    }
    // bytes 1 and 2: every lane looks up (a walk that is over reads entry 0, one cache line for all
    // such lanes, and drops the result), so the K loads of a step are issued together
#pragma unroll
    for (int i = 1; i < 3; ++i) {
        bool some = false;
#pragma unroll
        for (int k = 0; k < K; ++k)
            some = some || len[k] > (uint32_t)i;
        if (__ballot(some) == 0)
            break;
        uint32_t next[K];
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const uint32_t c = (kk[k] >> (8 * i)) & 255u;
            next[k] = (uint32_t)tab[(uint32_t)i < len[k] ? s[k] * n_classes + c : 0u];
        }
#pragma unroll
        for (int k = 0; k < K; ++k)
            s[k] = (uint32_t)i < len[k] ? next[k] : s[k];
    }
    if (__ballot(any_long) != 0) {
        // tokens of more than three bytes: bytes 3 .. 7 from the record and the rest from the class
        // string
        uint32_t longest = 0;
#pragma unroll
        for (int k = 0; k < K; ++k) {
            if (len[k] > 3u) {
                len[k] = real_len[k];
                longest = max(longest, len[k]);
            } else {
                len[k] = 0;                                 // finished
            }
        }
#pragma unroll
        for (int i = 3; i < kPackedClasses; ++i) {
            if (__ballot((uint32_t)i < longest) == 0)
                break;
            uint32_t next[K];
#pragma unroll
            for (int k = 0; k < K; ++k) {
                const uint32_t half = i < 4 ? (uint32_t)pk[k] : (uint32_t)(pk[k] >> 32);
                const uint32_t c = (half >> (8 * (i & 3))) & 255u;
                next[k] = (uint32_t)tab[(uint32_t)i < len[k] ? s[k] * n_classes + c : 0u];
            }
#pragma unroll
            for (int k = 0; k < K; ++k)
                s[k] = (uint32_t)i < len[k] ? next[k] : s[k];
        }
        for (uint32_t i = (uint32_t)kPackedClasses; __ballot(i < longest) != 0; ++i) {
            uint32_t c[K], next[K];
#pragma unroll
            for (int k = 0; k < K; ++k)
                c[k] = i < len[k] ? (uint32_t)cls[off[k] + i] : 0u;
#pragma unroll
            for (int k = 0; k < K; ++k)
                next[k] = (uint32_t)tab[i < len[k] ? s[k] * n_classes + c[k] : 0u];
#pragma unroll
            for (int k = 0; k < K; ++k)
                s[k] = i < len[k] ? next[k] : s[k];
        }
    }
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const uint32_t r = g0 + (uint32_t)(k * kWave + lane);
        if (r < r1) {
            int64_t pos = out.base[0] + r;
#pragma unroll
            for (int w = 1; w < kWalkBlocks; ++w)
                if (r >= out.start[w])
                    pos = out.base[w] + (r - out.start[w]);
            a.token_ids[pos] = token0 + (int32_t)t[k];
            a.next_states[pos] = (int32_t)s[k];
        }
    }
}

// The same for large automata without structure, where the texture addresser is what bounds the
// walk and most admissible tokens are short.  A token is read in its four-byte form (the classes
// of its first three bytes and its length): consecutive ranks are tokens a few ids apart, and their
// short forms share cache lines where their 16-byte records do not.  Byte 0 comes from row q in
// LDS, byte 1 from the table; the few walks that are longer are put aside -- (rank, state so far)
// in LDS -- and finished together by walk_deferred, so that their look-ups are issued by full
// waves instead of by every wave that holds one of them.
struct Deferred {
    uint16_t *rank;            // [kDeferCap] rank within the part
    uint32_t *state;           // [kDeferCap] state after two bytes
};

template <typename E>
__device__ __forceinline__ void walk_deferred(const EmitArgs &a, const TokenRecord *__restrict__ tok_b,
                                              const uint8_t *__restrict__ cls, const E *__restrict__ tab,
                                              const uint16_t *list, const Deferred &d, const uint32_t n_def,
                                              const int lane, const SpanOut &out, const uint32_t r0,
                                              const uint32_t n_classes)
{
    for (uint32_t e0 = 0; e0 < n_def; e0 += kWave) {
        const bool valid = e0 + (uint32_t)lane < n_def;
        const uint32_t rel = valid ? (uint32_t)d.rank[e0 + lane] : 0u;
        uint32_t s = valid ? d.state[e0 + lane] : 0u;
        const TokenRecord rec = tok_b[list[rel]];
        const uint64_t pk = ((uint64_t)rec.cls_hi << 32) | rec.cls_lo;
        const uint32_t len = valid ? rec.length : 0u;
#pragma unroll
        for (int i = 2; i < kPackedClasses; ++i) {
            if (__ballot((uint32_t)i < len) == 0)
                break;
            const uint32_t half = i < 4 ? (uint32_t)pk : (uint32_t)(pk >> 32);
            const uint32_t c = (half >> (8 * (i & 3))) & 255u;
            const uint32_t next = (uint32_t)tab[(uint32_t)i < len ? s * n_classes + c : 0u];
            s = (uint32_t)i < len ? next : s;
        }
        for (uint32_t i = (uint32_t)kPackedClasses; __ballot(i < len) != 0; ++i) {
            const uint32_t c = i < len ? (uint32_t)cls[rec.offset + i] : 0u;
            const uint32_t next = (uint32_t)tab[i < len ? s * n_classes + c : 0u];
            s = i < len ? next : s;
        }
        if (valid)
            a.next_states[span_pos(out, r0 + rel)] = (int32_t)s;
    }
}

template <typename E, int K>
__device__ __forceinline__ void walk_ranks_short(const EmitArgs &a, const uint32_t *__restrict__ key_b,
                                                 const E *__restrict__ tab, const uint16_t *list,
                                                 const uint32_t *row_q, const int32_t q, const int32_t token0,
                                                 const int lane, const SpanOut &out, const uint32_t r0,
                                                 const uint32_t g0, const uint32_t r1, const uint32_t n_classes,
                                                 const Deferred &d, uint32_t &n_def)
{
    uint32_t t[K], s[K], len[K], kk[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const uint32_t r = g0 + (uint32_t)(k * kWave + lane);
        t[k] = r < r1 ? (uint32_t)list[r - r0] : 0u;
    }
#pragma unroll
    for (int k = 0; k < K; ++k)
        kk[k] = key_b[t[k]];
    bool some = false;
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const uint32_t r = g0 + (uint32_t)(k * kWave + lane);
        len[k] = r < r1 ? kk[k] >> 24 : 0u;                 // (255: 255 bytes or more, the record knows)
        s[k] = len[k] != 0u ? row_q[kk[k] & 255u] : (uint32_t)q;
        some = some || len[k] > 1u;
    }
    if (__ballot(some) != 0) {
        uint32_t next[K];
#pragma unroll
        for (int k = 0; k < K; ++k)
            next[k] = (uint32_t)tab[len[k] > 1u ? s[k] * n_classes + ((kk[k] >> 8) & 255u) : 0u];
#pragma unroll
        for (int k = 0; k < K; ++k)
            s[k] = len[k] > 1u ? next[k] : s[k];
    }
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const uint32_t r = g0 + (uint32_t)(k * kWave + lane);
        const bool later = len[k] > 2u;
        if (r < r1) {
            const int64_t pos = span_pos(out, r);
            a.token_ids[pos] = token0 + (int32_t)t[k];
            if (!later)
                a.next_states[pos] = (int32_t)s[k];
        }
        const uint64_t m = __ballot(later);
        if (later) {
            const uint32_t at = n_def + __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
            d.rank[at] = (uint16_t)(r - r0);
            d.state[at] = s[k];
        }
        n_def += (uint32_t)__popcll(m);
    }
}

// Searched segments: this workgroup's share of the list.
template <typename TabE>
__device__ __forceinline__ void emit_by_search(const EmitArgs &a, const uint64_t *__restrict__ allow,
                                               const TokenRecord *__restrict__ tok, const uint8_t *__restrict__ cls,
                                               const TabE *__restrict__ tab, const StateRecord *__restrict__ srec,
                                               const uint32_t *__restrict__ pairs, const uint64_t *__restrict__ U,
                                               const uint64_t *__restrict__ E, const int lane, EmitShared *sh)
{
    uint32_t *node_state = sh->search.node_state;
    uint8_t *node_of = sh->search.node_of;
    if (!a.st->use_sets)
        return;
    const uint32_t n_items = a.st->n_long;
    const uint32_t ch = (uint32_t)a.n_chunks;
    // Segments differ a lot in cost, so the waves take them one by one.  Atomics on one address
    // are served one after the other, so there are kQueues counters: counter c hands out segments
    // c, c + kQueues, c + 2 kQueues, ...  Lane 0 fetches, the others learn the number through LDS:
    // a read of lane 0's register behind a lane-dependent branch could be moved by the compiler
    // to where the lanes run apart.
    volatile uint32_t *slot = &sh->search.next;
    uint32_t *spread = sh->search.spread;
    if (lane < 16)
        spread[lane] = ((uint32_t)lane & 1u) | ((uint32_t)lane & 2u) << 7 | ((uint32_t)lane & 4u) << 14 |
                       ((uint32_t)lane & 8u) << 21;
    const uint32_t c = blockIdx.x % (uint32_t)kQueues;
    for (;;) {
        if (lane == 0)
            *slot = atomicAdd(&a.queue[c], 1u);
        __builtin_amdgcn_wave_barrier();
        const uint32_t item = c + (uint32_t)kQueues * sgpr(*slot);
        __builtin_amdgcn_wave_barrier();
        if (item >= n_items)
            break;                                                  // every wave gets here
        const uint32_t packed = a.long_items[item];
        const int32_t q = (int32_t)sgpr(packed >> 12);
        const int32_t b = (int32_t)sgpr(packed & 0xFFFu);
        uint32_t chunk[1] = {(uint32_t)b * kBlockChunks + (uint32_t)lane};
        const uint64_t A = allow[(int64_t)q * a.n_chunks + chunk[0]];
        const uint32_t own = (uint32_t)__popcll(A);
        uint32_t incl = own;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            const uint32_t up = __shfl_up(incl, d, kWave);
            if (lane >= d)
                incl += up;
        }
        const uint32_t first = incl - own;
        const int64_t base_v = a.row_ptr[q] + (int64_t)a.cnt[(int64_t)q * a.n_blocks + b];
        const int64_t base = (int64_t)(((uint64_t)sgpr((uint32_t)((uint64_t)base_v >> 32)) << 32) | sgpr((uint32_t)base_v));
        uint64_t T[1] = {A};
        // Number 0 needs no plane bits, so it goes to an end state that many tokens are expected to
        // have: the target of the state's widest class set (its last pair: where a string state
        // loops on ordinary characters, the state itself; where it counts them, the next count).
        // The choice affects speed only.
        uint64_t node_bit[kNodeBits] = {};
        uint32_t n_nodes = 1;
        const StateRecord start = srec[q];
        const uint32_t start_pairs = sgpr(start.n_pairs);
        uint32_t common = (uint32_t)q;
        if (start_pairs == 1)
            common = sgpr(start.pair0) & 0xFFFFu;
        else if (start_pairs == 2)
            common = sgpr(start.pair1) & 0xFFFFu;
        else if (start_pairs > 2)
            common = sgpr(pairs[sgpr(start.ext) + start_pairs - 3]) & 0xFFFFu;
        // EOS has no bytes: it is not walked, and its end state is the start state, which takes
        // number 0 in the block that holds EOS
        if (a.eos >= 0 && a.eos / kBlockTokens == b) {
            common = (uint32_t)q;
            if (lane == (a.eos % kBlockTokens) / kChunkTokens)
                T[0] &= ~(1ull << (a.eos & (kChunkTokens - 1)));
        }
        node_state[0] = common;
        // The counting walk that found this segment did not overflow, but that says nothing about
        // this search: a pair that leads somewhere for all tokens and nowhere for the admissible
        // ones is decided together with the pair after it here, and the node then waits on the
        // stack while the search follows that second pair, where the counting walk had already
        // come back from the first.  A chain of such nodes holds one frame per level.
        const bool searched = search<1, kStackFrames>(q, T, chunk, ch, srec, pairs, U, E, sh->search.stack,
                        [&](int, uint64_t fin, uint32_t target) {
                            if (target == common || __ballot(fin != 0) == 0)
                                return;
                            // Once the numbers are used up, further nodes store their entries directly
                            // and give their tokens the number kDirectNode = already stored.
                            const bool direct = n_nodes >= (uint32_t)kDirectNode;
                            const uint32_t number = direct ? (uint32_t)kDirectNode : n_nodes;
#pragma unroll
                            for (int k = 0; k < kNodeBits; ++k)
                                if ((number >> k) & 1u)
                                    node_bit[k] |= fin;
                            if (!direct) {
                                node_state[n_nodes] = target;               // every lane, same value
                                ++n_nodes;
                                return;
                            }
                            while (__ballot(fin != 0) != 0) {
                                if (fin != 0) {
                                    const int bit = __builtin_ctzll(fin);
                                    fin &= fin - 1;
                                    const int64_t p = base + first + __popcll(A & ((1ull << bit) - 1ull));
                                    a.token_ids[p] = b * kBlockTokens + lane * kChunkTokens + bit;
                                    a.next_states[p] = (int32_t)target;
                                }
                            }
                        });
        if (!searched) {
            // Out of frames (rare): every lane walks the tokens of its own word one after the other
            // through the table, which needs no stack.  Slow, but short and small; entries that nodes
            // have stored directly are written again with the same values.  (EOS and empty tokens
            // have length 0: the end state is the state itself.)
            uint64_t rest = A;
            int64_t at = base + first;
            while (rest != 0) {
                const int bit = __builtin_ctzll(rest);
                rest &= rest - 1;
                const int32_t t = b * kBlockTokens + lane * kChunkTokens + bit;
                const TokenRecord rec = tok[t];
                const uint64_t pk = ((uint64_t)rec.cls_hi << 32) | rec.cls_lo;
                uint32_t s = (uint32_t)q;
                for (uint32_t i = 0; i < rec.length; ++i) {
                    const uint32_t c = i < (uint32_t)kPackedClasses ? (uint32_t)(pk >> (8 * i)) & 255u
                                                                    : (uint32_t)cls[rec.offset + i];
                    s = (uint32_t)tab[s * (uint32_t)a.n_classes + c];
                }
                a.token_ids[at] = t;
                a.next_states[at] = (int32_t)s;
                ++at;
            }
            __builtin_amdgcn_wave_barrier();
            continue;
        }
        // (numbers are below n_nodes)
        const int planes =
            (int)sgpr(n_nodes >= (uint32_t)kDirectNode ? (uint32_t)kNodeBits : 32u - (uint32_t)__builtin_clz(n_nodes));
        // ---- every lane turns the planes of its word into one byte per token, the number of the
        //      token's node, four tokens at a time: a 16-entry table spreads four bits of a plane
        //      over four bytes, and plane k goes in shifted left by k.  The row of a chunk is 64
        //      bytes; its four 16-byte pieces are stored rotated by a quarter of the chunk's number,
        //      so that the lanes' stores spread over the LDS banks: token t of chunk c lives at
        //      c * 64 + (t + 16 (c / 4)) % 64.
        {
            uint32_t four[kChunkTokens / 4] = {};                    // byte i of four[n]: number of token 4 n + i
#pragma unroll
            for (int k = 0; k < kNodeBits; ++k) {
                if (k >= planes)
                    break;
                const uint32_t lo = (uint32_t)node_bit[k], hi = (uint32_t)(node_bit[k] >> 32);
#pragma unroll
                for (int n = 0; n < 8; ++n) {
                    four[n] |= spread[(lo >> (4 * n)) & 15u] << k;
                    four[8 + n] |= spread[(hi >> (4 * n)) & 15u] << k;
                }
            }
#pragma unroll
            for (int p = 0; p < 4; ++p)
                *reinterpret_cast<uint4 *>(node_of + lane * kChunkTokens + (((p + (lane >> 2)) & 3) << 4)) =
                    make_uint4(four[4 * p], four[4 * p + 1], four[4 * p + 2], four[4 * p + 3]);
        }
        __builtin_amdgcn_wave_barrier();
        // ---- token order, 64 consecutive tokens per step: the lanes with an admissible token have
        //      consecutive ranks.  What steers a step is wave-uniform and stays in scalar
        //      registers: the chunk's admissibility word (read again from the bitmap with a scalar
        //      load) is the mask of the active lanes, and the rank of the chunk's first entry is a
        //      running sum of the words' popcounts.  The entries are first collected in LDS (end
        //      state << 16 | token number within the block) and leave kFlush at a time, four
        //      consecutive entries per lane and array: runs of 1 KB, mostly whole cache lines, which
        //      is what lets them bypass the cache (a store of a few lanes' worth that does so is
        //      written to memory as a partial line, and again when its neighbour comes).
        //      Positions are 32-bit offsets from the segment's first entry.
        char *const tok_out = reinterpret_cast<char *>(a.token_ids + base);
        char *const st_out = reinterpret_cast<char *>(a.next_states + base);
        const uint64_t *const words = allow + ((int64_t)q * a.n_chunks + (int64_t)b * kBlockChunks);
        const uint32_t block_token0 = (uint32_t)b * kBlockTokens;
        //      (the words of four steps and their two LDS reads, node number and then its state, are
        //      issued together; four rows in a row share their rotation)
        constexpr int kSteps = 4;
        static_assert(kSteps == 4, "the statement that pins the LDS reads names every step");
        if (n_nodes < (uint32_t)kDirectNode) {
            uint32_t *const stage = sh->search.stage;
            uint32_t numbered = (uint32_t)lane;                      // token number within the block
            uint32_t fill = 0, flushed = 0;                          // entries in the stage / already stored
#pragma unroll 1
            for (int j0 = 0; j0 < kBlockChunks; j0 += kSteps) {
                uint64_t word[kSteps];
                uint32_t node[kSteps], state[kSteps];
#pragma unroll
                for (int k = 0; k < kSteps; ++k)
                    word[k] = words[j0 + k];
                const uint8_t *const rows = node_of + j0 * kChunkTokens + ((lane + 4 * j0) & (kChunkTokens - 1));
#pragma unroll
                for (int k = 0; k < kSteps; ++k)
                    node[k] = rows[k * kChunkTokens];
#pragma unroll
                for (int k = 0; k < kSteps; ++k)
                    state[k] = node_state[node[k]];
                asm volatile("" ::"v"(state[0]), "v"(state[1]), "v"(state[2]),
                             "v"(state[3]));                         // all read here, not behind the branches below
#pragma unroll
                for (int k = 0; k < kSteps; ++k) {
                    if (word[k] == 0)
                        continue;
                    if (__builtin_amdgcn_inverse_ballot_w64(word[k])) {
                        const uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(word[k] >> 32),
                                                                        __builtin_amdgcn_mbcnt_lo((uint32_t)word[k], 0u));
                        stage[fill + rank] = state[k] << 16 | (numbered + (uint32_t)k * kChunkTokens);
                    }
                    fill += (uint32_t)__popcll(word[k]);
                    if (fill < (uint32_t)kFlush)
                        continue;
                    __builtin_amdgcn_wave_barrier();
                    const uint4 e = reinterpret_cast<const uint4 *>(stage)[lane];
                    const uint32_t off = (flushed + 4u * (uint32_t)lane) << 2;
                    const Int4 tokens = {(int32_t)(block_token0 + (e.x & 0xFFFFu)),
                                         (int32_t)(block_token0 + (e.y & 0xFFFFu)),
                                         (int32_t)(block_token0 + (e.z & 0xFFFFu)),
                                         (int32_t)(block_token0 + (e.w & 0xFFFFu))};
                    const Int4 states = {(int32_t)(e.x >> 16), (int32_t)(e.y >> 16), (int32_t)(e.z >> 16),
                                         (int32_t)(e.w >> 16)};
                    __builtin_nontemporal_store(tokens, reinterpret_cast<Int4 *>(tok_out + off));
                    __builtin_nontemporal_store(states, reinterpret_cast<Int4 *>(st_out + off));
                    // what is left (fewer than 64 entries) moves to the front
                    fill -= (uint32_t)kFlush;
                    flushed += (uint32_t)kFlush;
                    const uint32_t left = (uint32_t)lane < fill ? stage[kFlush + lane] : 0u;
                    if ((uint32_t)lane < fill)
                        stage[lane] = left;
                    __builtin_amdgcn_wave_barrier();
                }
                numbered += kSteps * kChunkTokens;
            }
            __builtin_amdgcn_wave_barrier();
            for (uint32_t i = (uint32_t)lane; i < fill; i += (uint32_t)kWave) {
                const uint32_t e = stage[i];
                const uint32_t off = (flushed + i) << 2;
                *reinterpret_cast<int32_t *>(tok_out + off) = (int32_t)(block_token0 + (e & 0xFFFFu));
                *reinterpret_cast<int32_t *>(st_out + off) = (int32_t)(e >> 16);
            }
        } else {
            // (rare) some nodes have stored their entries themselves: every step stores its own
            // entries and leaves those out
            uint32_t token = block_token0 + (uint32_t)lane;
            uint32_t before = 0;                                     // entries of the chunks so far
#pragma unroll 1
            for (int j0 = 0; j0 < kBlockChunks; j0 += kSteps) {
                uint64_t word[kSteps];
                uint32_t node[kSteps], state[kSteps];
#pragma unroll
                for (int k = 0; k < kSteps; ++k)
                    word[k] = words[j0 + k];
                const uint8_t *const rows = node_of + j0 * kChunkTokens + ((lane + 4 * j0) & (kChunkTokens - 1));
#pragma unroll
                for (int k = 0; k < kSteps; ++k)
                    node[k] = rows[k * kChunkTokens];
#pragma unroll
                for (int k = 0; k < kSteps; ++k)
                    state[k] = node_state[node[k]];                  // (the last number has no state: unused)
#pragma unroll
                for (int k = 0; k < kSteps; ++k) {
                    if (word[k] != 0 && __builtin_amdgcn_inverse_ballot_w64(word[k]) && node[k] != (uint32_t)kDirectNode) {
                        const uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(word[k] >> 32),
                                                                        __builtin_amdgcn_mbcnt_lo((uint32_t)word[k], 0u));
                        const uint32_t off = (rank + before) << 2;
                        *reinterpret_cast<int32_t *>(tok_out + off) = (int32_t)(token + (uint32_t)k * kChunkTokens);
                        *reinterpret_cast<int32_t *>(st_out + off) = (int32_t)state[k];
                    }
                    before += (uint32_t)__popcll(word[k]);
                }
                token += kSteps * kChunkTokens;
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
}

// Row q, blocks [b0, b0 + kWalkBlocks): the segments of these blocks that are walked (all but the
// searched ones) as one span of ranks.
template <typename E>
__device__ __forceinline__ void emit_span(const EmitArgs &a, const uint64_t *__restrict__ allow,
                                          const TokenRecord *__restrict__ tok,
                                          const uint8_t *__restrict__ cls, const E *__restrict__ tab,
                                          const uint32_t *__restrict__ key,
                                          const int32_t q, const int32_t b0, const uint32_t part,
                                          const uint32_t parts, const int lane, uint16_t *list, uint32_t *row_q,
                                          const Deferred later)
{
    uint64_t A[kWalkBlocks];
    uint32_t own[kWalkBlocks], first[kWalkBlocks], n_w[kWalkBlocks];
    // row q of the table, what the first byte of every token of the span is looked up in: loaded
    // together with the admissibility words, put into LDS once the span is known to have entries
    const uint32_t n_classes = (uint32_t)a.n_classes;
    uint32_t row_ahead[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t c = (uint32_t)(j * kWave + lane);
        row_ahead[j] = (uint32_t)(j * kWave) < n_classes && c < n_classes ? (uint32_t)tab[(uint32_t)q * n_classes + c] : 0u;
    }
#pragma unroll
    for (int w = 0; w < kWalkBlocks; ++w) {
        A[w] = b0 + w < a.n_blocks ? allow[(int64_t)q * a.n_chunks + (int64_t)(b0 + w) * kBlockChunks + lane] : 0ull;
        own[w] = (uint32_t)__popcll(A[w]);
    }
    // prefix sums over the lanes, two blocks per scan (a block has at most 4096 entries)
#pragma unroll
    for (int w = 0; w < kWalkBlocks; w += 2) {
        const uint32_t both = own[w] | (w + 1 < kWalkBlocks ? own[w + 1] << 16 : 0u);
        uint32_t incl = both;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            const uint32_t up = __shfl_up(incl, d, kWave);
            if (lane >= d)
                incl += up;
        }
        const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)incl, kWave - 1);
        const uint32_t excl = incl - both;
        first[w] = excl & 0xFFFFu;
        n_w[w] = total & 0xFFFFu;
        if (w + 1 < kWalkBlocks) {
            first[w + 1] = excl >> 16;
            n_w[w + 1] = total >> 16;
        }
    }
    // the count matrix has one column per block (token-set walk) or four (dense walk)
    const bool per_block = a.st->use_sets != 0;
    SpanOut out;
    uint32_t n = 0;
    const int64_t row = a.row_ptr[q];
#pragma unroll
    for (int w = 0; w < kWalkBlocks; ++w) {
        if (per_block && n_w[w] > (uint32_t)kLongRow) {             // emitted by search
            n_w[w] = 0;
            A[w] = 0;
            own[w] = 0;
        }
        out.start[w] = n;
        first[w] += n;                                              // rank within the span
        n += n_w[w];
        out.base[w] = 0;
        if (n_w[w] != 0) {
            const int64_t col = per_block ? (int64_t)q * a.n_blocks + (b0 + w)
                                          : (int64_t)q * a.n_groups + (int64_t)(b0 + w) * kGroupsPerBlock;
            // (uniform values: keep them in scalar registers)
            const int64_t pos = row + (int64_t)a.cnt[col];
            out.base[w] = (int64_t)(((uint64_t)sgpr((uint32_t)((uint64_t)pos >> 32)) << 32) | sgpr((uint32_t)pos));
        }
    }
    out.start[kWalkBlocks] = n;
    if (n == 0)
        return;
    const int32_t token0 = b0 * kBlockTokens;
    const TokenRecord *tok_b = tok + (size_t)token0;
    const uint32_t *key_b = key + (size_t)token0;
#pragma unroll
    for (int j = 0; j < 4; ++j)
        if ((uint32_t)(j * kWave) < n_classes)
            row_q[j * kWave + lane] = row_ahead[j];
    __builtin_amdgcn_wave_barrier();

    // The short form of the tokens first where the texture addresser is what bounds the walk: a large
    // automaton without structure, whose admissible tokens are mostly short.  Small problems are
    // bound by their round trips, and the walked rows of JSON-like automata hold whole keys: there
    // the record is read at once.
    const bool short_first = !per_block && parts == 1u;
    // (small problems have few spans: then `parts` waves share a span, taking its parts of
    // kEmitPart ranks in turn)
    for (uint32_t r0 = part * (uint32_t)kEmitPart; r0 < n; r0 += parts * (uint32_t)kEmitPart) {
        const uint32_t r1 = min(r0 + (uint32_t)kEmitPart, n);
        // ---- expand the words into token numbers, ranks [r0, r1)
#pragma unroll
        for (int w = 0; w < kWalkBlocks; ++w) {
            uint64_t rest = A[w];
            uint32_t r = first[w];
            if (first[w] + own[w] <= r0 || first[w] >= r1)
                rest = 0;
            while (__ballot(rest != 0) != 0) {
                if (rest != 0) {
                    const int bit = __builtin_ctzll(rest);
                    rest &= rest - 1;
                    if (r >= r0 && r < r1)
                        list[r - r0] = (uint16_t)(w * kBlockTokens + lane * kChunkTokens + bit);
                    ++r;
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
        // ---- walk, up to kEmitK ranks per lane at a time
        if (short_first) {
            uint32_t n_def = 0;
            for (uint32_t g0 = r0; g0 < r1;) {
                if (n_def + (uint32_t)(kWave * kEmitK) > (uint32_t)kDeferCap) {
                    __builtin_amdgcn_wave_barrier();
                    walk_deferred<E>(a, tok_b, cls, tab, list, later, n_def, lane, out, r0, n_classes);
                    n_def = 0;
                    __builtin_amdgcn_wave_barrier();
                }
                const uint32_t left = r1 - g0;
                if (left > (uint32_t)kWave) {
                    walk_ranks_short<E, kEmitK>(a, key_b, tab, list, row_q, q, token0, lane, out, r0, g0, r1, n_classes,
                                                later, n_def);
                    g0 += (uint32_t)(kWave * kEmitK);
                } else {
                    walk_ranks_short<E, 1>(a, key_b, tab, list, row_q, q, token0, lane, out, r0, g0, r1, n_classes, later,
                                           n_def);
                    g0 += (uint32_t)kWave;
                }
            }
            __builtin_amdgcn_wave_barrier();
            walk_deferred<E>(a, tok_b, cls, tab, list, later, n_def, lane, out, r0, n_classes);
        } else {
            for (uint32_t g0 = r0; g0 < r1;) {
                const uint32_t left = r1 - g0;
                if (left > (uint32_t)kWave) {
                    walk_ranks<E, kEmitK>(a, tok_b, cls, tab, list, row_q, q, token0, lane, out, r0, g0, r1, n_classes);
                    g0 += (uint32_t)(kWave * kEmitK);
                } else {
                    walk_ranks<E, 1>(a, tok_b, cls, tab, list, row_q, q, token0, lane, out, r0, g0, r1, n_classes);
                    g0 += (uint32_t)kWave;
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
}

// grid: n_long_groups workgroups for the searched segments, then one workgroup per (span of
// kWalkBlocks blocks, state), span fastest (in rounds if there are more than the grid holds).
__global__ void reset_queues(uint32_t *queue)
{
    if (blockIdx.x == 0 && threadIdx.x < kQueues)
        queue[threadIdx.x] = 0;
}

template <typename E>
__global__ __launch_bounds__(kWave) void emit_csr(const EmitArgs a, const uint64_t *__restrict__ allow,
                                                  const TokenRecord *__restrict__ tok,
                                                  const uint8_t *__restrict__ cls, const E *__restrict__ tab,
                                                  const uint32_t *__restrict__ key,
                                                  const StateRecord *__restrict__ srec,
                                                  const uint32_t *__restrict__ pairs, const uint64_t *__restrict__ U,
                                                  const uint64_t *__restrict__ Ebits)
{
    __shared__ EmitShared shared;
    const int lane = threadIdx.x;
    // nothing to emit from a counting pass that has to be redone or was refused, and nothing if
    // the entries do not fit (uniform over the grid)
    if (a.st->overflow != 0 || a.st->flags != 0 || a.st->nnz > a.capacity)
        return;
    if (blockIdx.x < a.n_long_groups) {
        emit_by_search<E>(a, allow, tok, cls, tab, srec, pairs, U, Ebits, lane, &shared);
        return;
    }
    const uint32_t n_spans = ((uint32_t)a.n_blocks + kWalkBlocks - 1) / kWalkBlocks;
    const uint64_t n_items = (uint64_t)a.n_states * n_spans * a.parts;
    for (uint64_t item = blockIdx.x - a.n_long_groups; item < n_items; item += gridDim.x - a.n_long_groups) {
        const uint64_t whole = item / a.parts;
        const uint32_t part = (uint32_t)(item - whole * a.parts);
        const uint32_t slot = (uint32_t)(whole / n_spans);
        const uint32_t span = (uint32_t)(whole - (uint64_t)slot * n_spans);
        // token-set path: the states with several pairs first, as in the counting walk (their rows
        // are the long ones, and what starts last is what the kernel ends with)
        const uint32_t q = a.st->use_sets != 0 ? a.order[slot] : slot;
        emit_span<E>(a, allow, tok, cls, tab, key, (int32_t)q, (int32_t)(span * kWalkBlocks), part, a.parts, lane,
                     shared.walk.list, shared.walk.row, Deferred{shared.walk.later_rank, shared.walk.later_state});
    }
}

hipError_t launch_emit(const Plan &p, const fsmidx_vocab &vocab, char *ws, const int64_t *row_ptr, int32_t *token_ids,
                       int32_t *next_states, int64_t capacity, bool queues_clear, hipStream_t stream)
{
    if (p.n_blocks == 0 || p.n_states == 0)
        return hipSuccess;
    EmitArgs a;
    a.st = reinterpret_cast<const Status *>(ws + p.off_status);
    a.queue = reinterpret_cast<uint32_t *>(ws + p.off_queue);
    a.cnt = reinterpret_cast<const uint32_t *>(ws + p.off_cnt);
    const uint64_t *allow = reinterpret_cast<const uint64_t *>(ws + p.off_allow);   // [n_states][n_chunks]
    a.row_ptr = row_ptr;
    a.token_ids = token_ids;
    a.next_states = next_states;
    a.long_items = reinterpret_cast<const uint32_t *>(ws + p.off_long);
    a.order = reinterpret_cast<const uint32_t *>(ws + p.off_order);
    a.n_states = p.n_states;
    a.n_classes = p.n_classes;
    a.n_blocks = p.n_blocks;
    a.n_chunks = p.n_chunks;
    a.n_groups = p.n_groups;
    a.eos = vocab.eos_token_id;
    a.capacity = capacity;
    const int64_t items = (int64_t)p.n_states * p.n_blocks;
    a.n_long_groups = p.sets_possible ? (uint32_t)(items < kLongGrid ? items : kLongGrid) : 0u;
    const TokenRecord *tok = reinterpret_cast<const TokenRecord *>(ws + p.off_tok);
    const uint32_t *key = reinterpret_cast<const uint32_t *>(ws + p.off_key);
    const uint8_t *cls = reinterpret_cast<const uint8_t *>(ws + p.off_cls);
    const StateRecord *srec = reinterpret_cast<const StateRecord *>(ws + p.off_srec);
    const uint32_t *pairs = reinterpret_cast<const uint32_t *>(ws + p.off_pairs);
    const uint64_t *U = reinterpret_cast<const uint64_t *>(ws + p.off_U);
    const uint64_t *Ebits = reinterpret_cast<const uint64_t *>(ws + p.off_E);
    int64_t spans = (int64_t)p.n_states * ((p.n_blocks + kWalkBlocks - 1) / kWalkBlocks);
    // fewer spans than the chip holds waves: several waves per span
    a.parts = 1;
    if (spans < kSpanTarget)
        a.parts = (uint32_t)((kSpanTarget + spans - 1) / spans < kMaxParts ? (kSpanTarget + spans - 1) / spans : kMaxParts);
    spans *= a.parts;
    const int64_t cap = 0x7FFFFFFFll - a.n_long_groups;
    const dim3 grid((unsigned)((spans < cap ? spans : cap) + a.n_long_groups));
    if (a.n_long_groups != 0 && !queues_clear)
        hipLaunchKernelGGL(reset_queues, dim3(1), dim3(kQueues), 0, stream, a.queue);
    if (p.entry_bytes == 2)
        hipLaunchKernelGGL(emit_csr<uint16_t>, grid, dim3(kWave), 0, stream, a, allow, tok, cls,
                           reinterpret_cast<const uint16_t *>(ws + p.off_tab), key, srec, pairs, U, Ebits);
    else
        hipLaunchKernelGGL(emit_csr<uint32_t>, grid, dim3(kWave), 0, stream, a, allow, tok, cls,
                           reinterpret_cast<const uint32_t *>(ws + p.off_tab), key, srec, pairs, U, Ebits);
    return hipGetLastError();
}

}  // namespace fsmidx
