// Input preparation for the index build: the alphabet of V is mapped to byte classes and the
// transition function delta (Section 3, Definition 1) is narrowed, summarised and, for the
// token-set walk, regrouped by target.  Two launches here (a third, token_sets, has a file of its own):
//
//  prepare_all, one launch for three jobs that need nothing from each other:
//    classify_bytes : class string of the whole vocabulary, one byte per vocabulary byte
//    pack_token     : one 16-byte record per token (leading classes, start, length) and its
//                     four-byte short form
//    narrow_state   : int32 table -> uint16/uint32 table + per-state mask of the classes a state
//                     can read (the SIMD form of Algorithm 3's restriction to the states that can
//                     read the first symbol); for automata with at most 64 classes also the state's
//                     (target, class set) pairs, smallest class set first
//  finish_sets      : one workgroup gathers the check bits, numbers the distinct class sets, decides
//                     whether the token-set kernels run and writes the status words of the build;
//                     a second one orders the states for the counting walk
//
// Every value that later serves as an address (class id, transition target, offset) is range
// checked here; bad values raise a flag bit and are replaced by harmless ones.
#include "internal.h"

namespace fsmidx {

// The byte-to-class map in LDS, every value range checked (a bad one counts as class 0).
// Returns kBadClass if this thread's entry was bad.  256 threads.
__device__ __forceinline__ uint32_t load_class_map(const uint8_t *__restrict__ byte_to_class, int32_t n_classes,
                                                   uint8_t *map)
{
    uint32_t bad = 0;
    uint32_t c = byte_to_class[threadIdx.x];
    if (c >= (uint32_t)n_classes) {
        bad = kBadClass;
        c = 0;
    }
    map[threadIdx.x] = (uint8_t)c;
    return bad;
}

// Workgroup `group` of `n_groups`: its share of the class string.
__device__ __forceinline__ void classify_bytes(const uint8_t *__restrict__ bytes, int64_t n_bytes, const uint8_t *map,
                                               uint8_t *__restrict__ cls, int32_t group, int32_t n_groups)
{
    // 16 bytes per thread per step, tail byte-wise
    const int64_t n_vec = n_bytes / 16;
    const uint4 *src = reinterpret_cast<const uint4 *>(bytes);
    uint4 *dst = reinterpret_cast<uint4 *>(cls);
    const bool aligned = ((reinterpret_cast<uintptr_t>(bytes) | reinterpret_cast<uintptr_t>(cls)) & 15) == 0;
    const int64_t stride = (int64_t)n_groups * blockDim.x;
    const int64_t tid = (int64_t)group * blockDim.x + threadIdx.x;
    if (aligned) {
        for (int64_t i = tid; i < n_vec; i += stride) {
            uint4 v = src[i];
            uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                uint32_t x = w[k];
                w[k] = (uint32_t)map[x & 255] | ((uint32_t)map[(x >> 8) & 255] << 8) |
                       ((uint32_t)map[(x >> 16) & 255] << 16) | ((uint32_t)map[x >> 24] << 24);
            }
            dst[i] = make_uint4(w[0], w[1], w[2], w[3]);
        }
        for (int64_t i = n_vec * 16 + tid; i < n_bytes; i += stride)
            cls[i] = map[bytes[i]];
    } else {
        for (int64_t i = tid; i < n_bytes; i += stride)
            cls[i] = map[bytes[i]];
    }
}

// The record of token slot t (slots past the last token get an empty record).
__device__ __forceinline__ uint32_t pack_token(int32_t t, const int64_t *__restrict__ offsets, int32_t n_tokens,
                                               int64_t n_bytes, int32_t eos, int32_t n_slots,
                                               const uint8_t *__restrict__ bytes, const uint8_t *map,
                                               TokenRecord *__restrict__ tok, uint32_t *__restrict__ key)
{
    if (t >= n_slots)
        return 0;
    uint32_t bad = 0;
    TokenRecord r = {0, 0, 0, 0};
    if (t < n_tokens) {
        const int64_t a = offsets[t], b = offsets[t + 1];
        bool ok = a >= 0 && a <= b && b <= n_bytes;
        if (t == 0 && a != 0) ok = false;
        if (t == n_tokens - 1 && b != n_bytes) ok = false;
        if (!ok) {
            bad = kBadOffsets;
        } else if (t != eos) {
            const uint32_t len = (uint32_t)(b - a);
            r.offset = (uint32_t)a;
            r.length = len;
            // eight independent loads (classified here, straight from the vocabulary's bytes: the
            // class string is being written by other workgroups of the same launch), then the bytes
            // past the end are masked away: a loop to the token's own length would be eight
            // dependent round trips
            uint64_t pk = 0;
#pragma unroll
            for (int i = 0; i < kPackedClasses; ++i)
                pk |= (uint64_t)(a + i < n_bytes ? map[bytes[a + i]] : 0) << (8 * i);
            if (len < (uint32_t)kPackedClasses)
                pk &= (1ull << (8 * len)) - 1ull;
            r.cls_lo = (uint32_t)pk;
            r.cls_hi = (uint32_t)(pk >> 32);
        }
    }
    tok[t] = r;
    // the short form for the passes that mostly meet short tokens: three classes and the length in
    // one word (a length of 255 says: look at the record)
    key[t] = (r.cls_lo & 0xFFFFFFu) | (r.length < 255u ? r.length : 255u) << 24;
    // the token-set path handles tokens of up to kMaxSetDepth bytes
    if (r.length > (uint32_t)kMaxSetDepth)
        bad |= kLongTokens;
    return bad;
}

__device__ __forceinline__ uint32_t hash_mask(uint64_t m)
{
    m ^= m >> 29;
    m *= 0x9E3779B97F4A7C15ull;
    m ^= m >> 32;
    return (uint32_t)m & (kSetHashSlots - 1);
}

// One wave per state.  E is the narrowed entry type; `dead_e` is the dead state's id in that type
// (all-ones if the automaton has no dead state, which no valid id equals).  With npairs != NULL
// (at most 64 classes, at most 65535 states) the state's transitions are also grouped by target:
// pairs[q * n_classes + i] = target, pmask[i * n_states + q] = the class set that leads to it
// (the layout in which one workgroup reads all of them next), smallest class set first (ties by
// lowest class), so that the widest set -- typically the one that keeps a token set walking -- is
// last and can be followed without a stack frame.
template <typename E>
__device__ __forceinline__ uint32_t narrow_state(const int32_t q, const int lane, const int32_t *__restrict__ trans,
                                                 int32_t n_states, int32_t n_classes, int32_t dead, int32_t live_words,
                                                 E *__restrict__ tab, uint64_t *__restrict__ live,
                                                 uint32_t *__restrict__ npairs, uint32_t *__restrict__ pairs,
                                                 uint64_t *__restrict__ pmask)
{
    const E dead_e = dead >= 0 ? (E)dead : (E)~(E)0;
    uint32_t flags = 0;
    for (int32_t w = 0; w < live_words; ++w) {
        const int32_t c = w * 64 + lane;
        bool is_live = false;
        uint32_t mine = 0;
        if (c < n_classes) {
            int32_t v = trans[(int64_t)q * n_classes + c];
            E e;
            if (v < 0 || v >= n_states) {
                flags |= kBadTransition;
                e = dead >= 0 ? dead_e : (E)q;      // neutralise: reject, or stay put if nothing rejects
            } else {
                e = (E)v;
            }
            if (q == dead && v != dead)
                flags |= kDeadNotAbsorbing;
            tab[(int64_t)q * n_classes + c] = e;
            is_live = (e != dead_e) && (q != dead);
            mine = (uint32_t)e;
        }
        const uint64_t m = __ballot(is_live);
        if (lane == 0)
            live[(int64_t)q * live_words + w] = m;
        if (npairs != nullptr) {
            // (one word: at most 64 classes)  lane k ends up with the k-th distinct target, in the
            // order of the targets' lowest classes, and the set of classes that lead to it
            uint64_t remaining = m;
            uint32_t k = 0, my_t = 0;
            uint64_t my_m = 0;
            while (remaining) {
                const uint32_t t = (uint32_t)__builtin_amdgcn_readlane((int)mine, __builtin_ctzll(remaining));
                const uint64_t grp = __ballot(is_live && mine == t);
                remaining &= ~grp;
                if ((uint32_t)lane == k) {
                    my_t = t;
                    my_m = grp;
                }
                ++k;
            }
            const uint32_t key = (uint32_t)__popcll(my_m) * 64u + (uint32_t)(my_m ? __builtin_ctzll(my_m) : 0);
            uint32_t rank = 0;
            for (uint32_t j = 0; j < k; ++j) {
                const uint32_t kj = (uint32_t)__builtin_amdgcn_readlane((int)key, (int)j);
                rank += kj < key ? 1u : 0u;
            }
            if ((uint32_t)lane < k) {
                pairs[(int64_t)q * n_classes + rank] = my_t;
                pmask[(int64_t)rank * n_states + q] = my_m;
            }
            if (lane == 0)
                npairs[q] = k;
        }
    }
    return flags;
}

struct FinishArgs {
    SyncWords *sy;
    const uint32_t *npairs;       // [n_states]
    const uint64_t *pmask;        // [n_classes][n_states]
    uint32_t *pslot;              // [n_classes][n_states]
    uint32_t *order;              // [n_states]
    uint64_t *class_sets;         // [64][kSetCap / 64]
    int32_t n_states, n_classes;
    uint32_t expect;              // the counting kernels the host launches: 0 both, 1 token-set only, 2 dense only
    const uint32_t *badw;         // [n_badw] check bits of the preparation kernel's workgroups
    int32_t n_badw;
};

// The part of the preparation that needs every state's pairs (two workgroups of kFinishThreads,
// one for each of the first two jobs below; the third belongs to the second).
//  - the order in which the counting walk takes the states: those with two or more pairs first
//    (ascending), the others after them (descending, filled from the end).  Searches from branching
//    states are the long ones, and a long one that starts last is what the whole kernel waits for;
//  - the distinct class sets are collected in a table in LDS, its occupied slots are numbered
//    0 .. n_sets - 1 in slot order, every pair's slot is noted (token_sets turns slots into
//    numbers), and for every class the sets that contain it are written as a bit mask (what
//    token_sets looks up);
//  - the decision: the token-set kernels count if there are at most kSetCap class sets, at most
//    three pairs per state on average and no token longer than kMaxSetDepth bytes.
constexpr int kFinishThreads = 1024;
constexpr int kFinishStates = 8;       // states per thread whose loads are issued together

// The slot of class set `key` in the LDS table (entered if new); every lane of the wave may call
// with its own set.  Returns kSetHashSlots if the table is full.
__device__ __forceinline__ uint32_t table_slot(unsigned long long *keys, unsigned long long key)
{
    uint32_t h = hash_mask(key);
    for (int probe = 0; probe < kSetHashSlots; ++probe) {
        // Looked at before it is claimed: an automaton has few distinct class sets, so nearly every
        // call finds its set entered already, and lanes reading one address are served together
        // while their atomics on it would take turns.
        unsigned long long old = __hip_atomic_load(&keys[h], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (old == 0ull)
            old = atomicCAS(&keys[h], 0ull, key);
        if (old == 0ull || old == key)
            return h;
        h = (h + 1) & (kSetHashSlots - 1);
    }
    return kSetHashSlots;
}

// One workgroup on its own pays the full memory latency for every dependent load, so a thread
// issues the loads of kFinishStates states together: first their pair counts, then the class sets
// of their first two pairs.  The few states with more pairs are taken by their wave as a whole
// afterwards, lane j loading the state's pair j.
__global__ __launch_bounds__(kFinishThreads) void finish_sets(const FinishArgs f, Status *st)
{
    constexpr int kWaves = kFinishThreads / kWave;
    static_assert(kSetHashSlots <= kFinishThreads, "one thread per slot of the class-set table");
    __shared__ unsigned long long keys[kSetHashSlots];
    __shared__ uint64_t by_id[kSetCap];
    __shared__ uint32_t wave_sum[kWaves], wave_many[kWaves];
    __shared__ uint32_t carry_s, carry_many_s, failed, pairs_s;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int32_t n = f.n_states;
    // Two workgroups, two jobs that need nothing from each other: the class sets with the decision
    // and the status words (workgroup 0; the only one when the token-set kernels are out of the
    // question), and the order of the states (workgroup 1).
    if (blockIdx.x == 1) {
        if (threadIdx.x == 0)
            carry_many_s = 0;
        __syncthreads();
        for (int32_t c0 = 0; c0 < n; c0 += kFinishThreads * kFinishStates) {
            uint32_t k[kFinishStates];
#pragma unroll
            for (int u = 0; u < kFinishStates; ++u) {
                const int32_t i = c0 + u * kFinishThreads + (int32_t)threadIdx.x;
                k[u] = i < n ? f.npairs[i] : 0u;
            }
#pragma unroll
            for (int u = 0; u < kFinishStates; ++u) {
                const int32_t i0 = c0 + u * kFinishThreads;
                if (i0 >= n)
                    break;                                       // uniform
                const int32_t i = i0 + (int32_t)threadIdx.x;
                const uint32_t x = k[u];
                const uint64_t many = __ballot(i < n && x >= 2u);
                if (lane == 0)
                    wave_many[wave] = (uint32_t)__popcll(many);
                __syncthreads();
                uint32_t many_before = carry_many_s, all = 0;
                for (int w = 0; w < kWaves; ++w) {
                    if (w < wave)
                        many_before += wave_many[w];
                    all += wave_many[w];
                }
                if (i < n) {
                    const uint32_t rank = many_before + __builtin_amdgcn_mbcnt_hi((uint32_t)(many >> 32),
                                                                                  __builtin_amdgcn_mbcnt_lo((uint32_t)many, 0u));
                    f.order[x >= 2u ? rank : (uint32_t)n - 1u - ((uint32_t)i - rank)] = (uint32_t)i;
                }
                __syncthreads();
                if (threadIdx.x == 0)
                    carry_many_s += all;
                __syncthreads();
            }
        }
        return;
    }
    constexpr int kHeavyCap = 1024;
    __shared__ uint32_t checks_s, heavy_n;
    __shared__ uint32_t heavy_list[kHeavyCap];
    if (threadIdx.x == 0) {
        heavy_n = 0;
        carry_s = 0;
        failed = 0;
        pairs_s = 0;
        checks_s = 0;
    }
    if (threadIdx.x < kSetHashSlots)
        keys[threadIdx.x] = 0ull;
    __syncthreads();
    // What the preparation kernel's workgroups found wrong with the input (and whether some token
    // is too long for the token-set walk).  The words are asked for here and looked at after the
    // first states' loads have been issued: one trip to memory for both.
    uint32_t my_checks = 0;
    for (int32_t i0 = 0; i0 < f.n_badw; i0 += 4 * kFinishThreads) {
        uint32_t w[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {                            // four loads in flight
            const int32_t i = i0 + u * kFinishThreads + (int32_t)threadIdx.x;
            w[u] = i < f.n_badw ? f.badw[i] : 0u;
        }
        my_checks |= (w[0] | w[1]) | (w[2] | w[3]);
    }
    const bool with_sets = f.npairs != nullptr;
    if (!with_sets) {
        if (my_checks)
            atomicOr(&checks_s, my_checks);
        __syncthreads();
    }
    for (int32_t c0 = 0; with_sets && c0 < n; c0 += kFinishThreads * kFinishStates) {
        // pair counts and the class sets of the first two pairs, none of the loads waiting for
        // another (a set that does not exist is whatever the array held: masked right below)
        uint32_t k[kFinishStates];
        unsigned long long m0[kFinishStates], m1[kFinishStates];
        uint32_t mine = 0;
#pragma unroll
        for (int u = 0; u < kFinishStates; ++u) {
            const int32_t i = c0 + u * kFinishThreads + (int32_t)threadIdx.x;
            k[u] = i < n ? f.npairs[i] : 0u;
            m0[u] = i < n ? f.pmask[i] : 0ull;
            m1[u] = i < n && f.n_classes > 1 ? f.pmask[(int64_t)n + i] : 0ull;
        }
#pragma unroll
        for (int u = 0; u < kFinishStates; ++u) {
            mine += k[u];
            if (k[u] < 1u)
                m0[u] = 0ull;
            if (k[u] < 2u)
                m1[u] = 0ull;
        }
        if (c0 == 0 && my_checks)
            atomicOr(&checks_s, my_checks);
        // ---- the number of pairs so far
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1)
            mine += __shfl_xor(mine, o, kWave);
        if (lane == 0)
            atomicAdd(&pairs_s, mine);
        __syncthreads();
        if (threadIdx.x == 0)
            carry_s = pairs_s;
        __syncthreads();
        // ---- the class sets into the table (an automaton with more than three pairs per state on
        //      average is not for the token-set walk: its sets may be too many to be worth entering;
        //      the decision below looks at the final count)
        if (carry_s > 3u * (uint32_t)n || (checks_s & kLongTokens) != 0)
            continue;                                            // uniform
#pragma unroll
        for (int u = 0; u < kFinishStates; ++u) {
            const int32_t i = c0 + u * kFinishThreads + (int32_t)threadIdx.x;
            if (k[u] > 0u) {
                const uint32_t h = table_slot(keys, m0[u]);
                if (h == (uint32_t)kSetHashSlots)
                    failed = 1;
                f.pslot[i] = h;
            }
            if (k[u] > 1u) {
                const uint32_t h = table_slot(keys, m1[u]);
                if (h == (uint32_t)kSetHashSlots)
                    failed = 1;
                f.pslot[(int64_t)n + i] = h;
            }
            // a state with more pairs goes on a list (or, if the list is full, is taken by its wave
            // as a whole right away, lane j loading the state's pair j: one state after the other)
            bool listed = false;
            if (k[u] > 2u) {
                const uint32_t at = atomicAdd(&heavy_n, 1u);
                listed = at < (uint32_t)kHeavyCap;
                if (listed)
                    heavy_list[at] = (uint32_t)i | k[u] << 16;   // (at most 65535 states and 64 classes here)
            }
            uint64_t heavy = __ballot(k[u] > 2u && !listed);
            while (heavy != 0) {
                const int src = __builtin_ctzll(heavy);
                heavy &= heavy - 1;
                const uint32_t kk = (uint32_t)__builtin_amdgcn_readlane((int)k[u], src);
                const int32_t ii = c0 + u * kFinishThreads + (wave << 6) + src;
                for (uint32_t j = 2u + (uint32_t)lane; j < kk; j += (uint32_t)kWave) {
                    const int64_t at = (int64_t)j * n + ii;
                    const uint32_t h = table_slot(keys, f.pmask[at]);
                    if (h == (uint32_t)kSetHashSlots)
                        failed = 1;
                    f.pslot[at] = h;
                }
            }
        }
        // the listed states, sixteen lanes to a state, so that the loads of 64 states are in flight
        // together
        __syncthreads();
        const uint32_t n_listed = heavy_n < (uint32_t)kHeavyCap ? heavy_n : (uint32_t)kHeavyCap;
        for (uint32_t h0 = threadIdx.x >> 4; h0 < n_listed; h0 += kFinishThreads / 16) {
            const uint32_t e = heavy_list[h0];
            const int32_t ii = (int32_t)(e & 0xFFFFu);
            for (uint32_t j = 2u + (threadIdx.x & 15u); j < e >> 16; j += 16u) {
                const int64_t at = (int64_t)j * n + ii;
                const uint32_t h = table_slot(keys, f.pmask[at]);
                if (h == (uint32_t)kSetHashSlots)
                    failed = 1;
                f.pslot[at] = h;
            }
        }
        __syncthreads();
        if (threadIdx.x == 0)
            heavy_n = 0;
    }
    __syncthreads();
    const uint32_t n_pairs = carry_s;
    const uint32_t checks = checks_s;
    const uint32_t long_tokens = (checks & kLongTokens) != 0 ? 1u : 0u;
    bool ok = with_sets && n_pairs <= 3u * (uint32_t)n && long_tokens == 0;      // uniform over the workgroup
    uint32_t n_sets = 0;
    if (ok) {
        // number the occupied slots
        const int slot = (int)threadIdx.x;
        const unsigned long long key = slot < kSetHashSlots ? keys[slot] : 0ull;
        const uint64_t b = __ballot(key != 0ull);
        const uint32_t below = __builtin_amdgcn_mbcnt_hi((uint32_t)(b >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)b, 0u));
        if (lane == 0)
            wave_sum[wave] = (uint32_t)__popcll(b);
        __syncthreads();
        uint32_t before = 0;
        for (int w = 0; w < kWaves; ++w) {
            if (w < wave)
                before += wave_sum[w];
            n_sets += wave_sum[w];
        }
        if (key != 0ull) {
            const uint32_t id = before + below;
            f.sy->ids[slot] = id;
            if (id < (uint32_t)kSetCap)
                by_id[id] = key;
        }
        __syncthreads();
        ok = failed == 0 && n_sets <= (uint32_t)kSetCap;
        // the transpose: for every class, the sets that contain it (bit k of word k / 64 = set k).
        // Wave w holds the class sets of sets 64 w .. 64 w + 63, one per lane, as a 64 x 64 bit
        // matrix; transposed, lane c has word w of class c.
        static_assert(kSetCap % kWave == 0 && kSetCap <= kFinishThreads, "whole waves hold the sets");
        if (ok && threadIdx.x < kSetCap)
            f.class_sets[lane * (kSetCap / 64) + wave] =
                transpose_bits(threadIdx.x < n_sets ? by_id[threadIdx.x] : 0ull, lane);
    }
    // every status word of the build is written here, once: nothing before this kernel touches them
    if (threadIdx.x == 0) {
        st->nnz = 0;
        st->flags = checks & kInputFlags;
        st->long_tokens = long_tokens;
        st->n_long = 0;
        st->n_sets = n_sets;
        st->n_pairs = n_pairs;
        st->use_sets = ok && f.expect != 2u ? 1u : 0u;
        st->feasible = ok && f.expect == 2u ? 1u : 0u;           // the dense kernel counts; the host learns for next time
        st->overflow = !ok && f.expect == 1u ? 2u : 0u;          // nobody else will count: the host has to ask again
    }
}

// One launch for three jobs that need nothing from each other: the first cls_groups workgroups
// write the class string, the next pack_groups pack 256 token slots each (classifying the bytes
// they need themselves), the others narrow four states each, one wave per state.  Every workgroup
// leaves its check bits in a word of its own: the status words are written by the kernel after
// this one, so nothing here has to be ordered against their reset.
template <typename E>
__global__ __launch_bounds__(256) void prepare_all(int32_t cls_groups, int32_t pack_groups,
                                                   const uint8_t *__restrict__ bytes, int64_t n_bytes,
                                                   const uint8_t *__restrict__ byte_to_class, uint8_t *__restrict__ cls,
                                                   const int64_t *__restrict__ offsets, int32_t n_tokens, int32_t eos,
                                                   int32_t n_slots, TokenRecord *__restrict__ tok,
                                                   uint32_t *__restrict__ key,
                                                   const int32_t *__restrict__ trans, int32_t n_states,
                                                   int32_t n_classes, int32_t dead, int32_t live_words,
                                                   E *__restrict__ tab, uint64_t *__restrict__ live,
                                                   uint32_t *__restrict__ npairs, uint32_t *__restrict__ pairs,
                                                   uint64_t *__restrict__ pmask, uint32_t *__restrict__ badw)
{
    __shared__ uint8_t map[256];
    __shared__ uint32_t bad_s;
    if (threadIdx.x == 0)
        bad_s = 0;
    uint32_t bad = 0;
    const int32_t group = (int32_t)blockIdx.x;
    if (group < cls_groups + pack_groups) {
        bad = load_class_map(byte_to_class, n_classes, map);
        __syncthreads();
        if (group < cls_groups)
            classify_bytes(bytes, n_bytes, map, cls, group, cls_groups);
        else
            bad |= pack_token((group - cls_groups) * 256 + (int32_t)threadIdx.x, offsets, n_tokens, n_bytes, eos, n_slots,
                              bytes, map, tok, key);
    } else {
        __syncthreads();
        const int32_t q = (group - cls_groups - pack_groups) * 4 + (int32_t)(threadIdx.x >> 6);
        if (q < n_states)
            bad = narrow_state<E>(q, threadIdx.x & (kWave - 1), trans, n_states, n_classes, dead, live_words, tab, live,
                                  npairs, pairs, pmask);
    }
    if (bad)
        atomicOr(&bad_s, bad);
    __syncthreads();
    if (threadIdx.x == 0)
        badw[group] = bad_s;
}

hipError_t launch_prepare(const Plan &p, const fsmidx_dfa &dfa, const fsmidx_vocab &vocab, char *ws, int expect,
                          hipStream_t stream)
{
    Status *st = reinterpret_cast<Status *>(ws + p.off_status);
    SyncWords *sy = reinterpret_cast<SyncWords *>(ws + p.off_sync);
    uint8_t *cls = reinterpret_cast<uint8_t *>(ws + p.off_cls);
    TokenRecord *tok = reinterpret_cast<TokenRecord *>(ws + p.off_tok);
    uint32_t *key = reinterpret_cast<uint32_t *>(ws + p.off_key);
    uint64_t *live = reinterpret_cast<uint64_t *>(ws + p.off_live);
    uint32_t *badw = reinterpret_cast<uint32_t *>(ws + p.off_badw);
    const bool with_sets = p.sets_possible;
    uint32_t *npairs = with_sets ? reinterpret_cast<uint32_t *>(ws + p.off_npairs) : nullptr;
    uint32_t *pairs = with_sets ? reinterpret_cast<uint32_t *>(ws + p.off_pairs) : nullptr;
    uint64_t *pmask = with_sets ? reinterpret_cast<uint64_t *>(ws + p.off_pmask) : nullptr;
    FinishArgs f;
    f.sy = sy;
    f.npairs = npairs;
    f.pmask = pmask;
    f.pslot = with_sets ? reinterpret_cast<uint32_t *>(ws + p.off_pslot) : nullptr;
    f.order = with_sets ? reinterpret_cast<uint32_t *>(ws + p.off_order) : nullptr;
    f.class_sets = with_sets ? reinterpret_cast<uint64_t *>(ws + p.off_clsets) : nullptr;
    f.n_states = p.n_states;
    f.n_classes = p.n_classes;
    f.expect = (uint32_t)expect;
    f.badw = badw;
    f.n_badw = p.cls_groups + p.pack_groups + p.narrow_groups;

    const int32_t n_slots = p.n_chunks * kChunkTokens;
    const dim3 grid((unsigned)f.n_badw);
    if (p.entry_bytes == 2)
        hipLaunchKernelGGL(prepare_all<uint16_t>, grid, dim3(256), 0, stream, p.cls_groups, p.pack_groups, vocab.bytes,
                           p.n_bytes, dfa.byte_to_class, cls, vocab.offsets, p.n_tokens, vocab.eos_token_id, n_slots, tok,
                           key, dfa.trans, p.n_states, p.n_classes, dfa.dead_state, p.live_words,
                           reinterpret_cast<uint16_t *>(ws + p.off_tab), live, npairs, pairs, pmask, badw);
    else
        hipLaunchKernelGGL(prepare_all<uint32_t>, grid, dim3(256), 0, stream, p.cls_groups, p.pack_groups, vocab.bytes,
                           p.n_bytes, dfa.byte_to_class, cls, vocab.offsets, p.n_tokens, vocab.eos_token_id, n_slots, tok,
                           key, dfa.trans, p.n_states, p.n_classes, dfa.dead_state, p.live_words,
                           reinterpret_cast<uint32_t *>(ws + p.off_tab), live, static_cast<uint32_t *>(nullptr),
                           static_cast<uint32_t *>(nullptr), static_cast<uint64_t *>(nullptr), badw);
    // (without the token-set kernels: one workgroup, which gathers the check bits and writes the status)
    hipLaunchKernelGGL(finish_sets, dim3(with_sets ? 2 : 1), dim3(kFinishThreads), 0, stream, f, st);
    return hipGetLastError();
}

}  // namespace fsmidx
