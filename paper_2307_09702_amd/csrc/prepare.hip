// Input preparation for the index build: the alphabet of V is mapped to byte classes and the
// transition function delta (Section 3, Definition 1) is narrowed, summarised and, for the
// token-set walk, regrouped by target.  Three launches:
//
//  classify_bytes : class string of the whole vocabulary, one byte per vocabulary byte; also resets
//                   the status words of the build and the words its later launches meet through
//  pack_and_narrow, one launch for two jobs:
//    pack_token   : one 16-byte record per token (leading classes, start, length)
//    narrow_state : int32 table -> uint16/uint32 table + per-state mask of the classes a state
//                   can read (the SIMD form of Algorithm 3's restriction to the states that can
//                   read the first symbol); for automata with at most 64 classes also the state's
//                   (target, class set) pairs, smallest class set first
//  finish_sets    : one workgroup numbers the distinct class sets, orders the states for the
//                   counting walk and decides whether the token-set kernels run
//
// Every value that later serves as an address (class id, transition target, offset) is range
// checked here; bad values raise a flag bit and are replaced by harmless ones.
#include "internal.h"

namespace fsmidx {

__global__ __launch_bounds__(256) void classify_bytes(const uint8_t *__restrict__ bytes, int64_t n_bytes,
                                                      const uint8_t *__restrict__ byte_to_class,
                                                      int32_t n_classes, uint8_t *__restrict__ cls,
                                                      Status *st)
{
    __shared__ uint8_t map[256];
    // The first kernel of a build: its first workgroup resets the status words before it (and only
    // it, in this kernel) reports into them; every later kernel finds them reset.
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        {
            st->nnz = 0;
            st->flags = 0;
            st->use_sets = 0;
            st->n_sets = 0;
            st->n_pairs = 0;
            st->long_tokens = 0;
            st->overflow = 0;
            st->n_long = 0;
            st->feasible = 0;
        }
    }
    uint32_t bad = 0;
    {
        uint32_t c = byte_to_class[threadIdx.x];
        if (c >= (uint32_t)n_classes) {
            bad = 1;
            c = 0;
        }
        map[threadIdx.x] = (uint8_t)c;
    }
    __syncthreads();
    if (bad && blockIdx.x == 0)
        atomicOr(&st->flags, kBadClass);
    // 16 bytes per thread per step, tail byte-wise
    const int64_t n_vec = n_bytes / 16;
    const uint4 *src = reinterpret_cast<const uint4 *>(bytes);
    uint4 *dst = reinterpret_cast<uint4 *>(cls);
    const bool aligned = ((reinterpret_cast<uintptr_t>(bytes) | reinterpret_cast<uintptr_t>(cls)) & 15) == 0;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
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
__device__ __forceinline__ void pack_token(int32_t t, const int64_t *__restrict__ offsets, int32_t n_tokens,
                                           int64_t n_bytes, int32_t eos, int32_t n_slots,
                                           const uint8_t *__restrict__ cls, TokenRecord *__restrict__ tok,
                                           uint32_t *__restrict__ key, Status *st)
{
    if (t >= n_slots)
        return;
    TokenRecord r = {0, 0, 0, 0};
    if (t < n_tokens) {
        const int64_t a = offsets[t], b = offsets[t + 1];
        bool ok = a >= 0 && a <= b && b <= n_bytes;
        if (t == 0 && a != 0) ok = false;
        if (t == n_tokens - 1 && b != n_bytes) ok = false;
        if (!ok) {
            atomicOr(&st->flags, kBadOffsets);
        } else if (t != eos) {
            const uint32_t len = (uint32_t)(b - a);
            r.offset = (uint32_t)a;
            r.length = len;
            // eight independent loads (the class string is padded), then the bytes past the end are
            // masked away: a loop to the token's own length would be eight dependent round trips
            uint64_t pk = 0;
#pragma unroll
            for (int i = 0; i < kPackedClasses; ++i)
                pk |= (uint64_t)cls[a + i] << (8 * i);
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
    // the token-set path handles tokens of up to kMaxSetDepth bytes (a plain store: every writer
    // writes the same value)
    if (r.length > (uint32_t)kMaxSetDepth)
        st->long_tokens = 1;
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
__device__ __forceinline__ void narrow_state(const int32_t q, const int lane, const int32_t *__restrict__ trans,
                                             int32_t n_states, int32_t n_classes, int32_t dead, int32_t live_words,
                                             E *__restrict__ tab, uint64_t *__restrict__ live,
                                             uint32_t *__restrict__ npairs, uint32_t *__restrict__ pairs,
                                             uint64_t *__restrict__ pmask, Status *st)
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
    if (flags)
        atomicOr(&st->flags, flags);
}

struct FinishArgs {
    SyncWords *sy;
    const uint32_t *npairs;       // [n_states]
    const uint64_t *pmask;        // [n_classes][n_states]
    uint32_t *pslot;              // [n_classes][n_states]
    uint32_t *order;              // [n_states]
    uint64_t *class_sets;         // [64][kSetCap / 64]
    int32_t n_states;
    uint32_t expect;              // the counting kernels the host launches: 0 both, 1 token-set only, 2 dense only
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
        const unsigned long long old = atomicCAS(&keys[h], 0ull, key);
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
    // Two workgroups, two jobs that need nothing from each other: the order of the states
    // (workgroup 0), and the class sets with the decision (workgroup 1).
    if (blockIdx.x == 0) {
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
    if (threadIdx.x == 0) {
        carry_s = 0;
        failed = 0;
        pairs_s = 0;
    }
    if (threadIdx.x < kSetHashSlots)
        keys[threadIdx.x] = 0ull;
    const uint32_t long_tokens = st->long_tokens;
    __syncthreads();
    for (int32_t c0 = 0; c0 < n; c0 += kFinishThreads * kFinishStates) {
        uint32_t k[kFinishStates];
        unsigned long long m0[kFinishStates], m1[kFinishStates];
        uint32_t mine = 0;
#pragma unroll
        for (int u = 0; u < kFinishStates; ++u) {
            const int32_t i = c0 + u * kFinishThreads + (int32_t)threadIdx.x;
            k[u] = i < n ? f.npairs[i] : 0u;
            mine += k[u];
        }
#pragma unroll
        for (int u = 0; u < kFinishStates; ++u) {
            const int32_t i = c0 + u * kFinishThreads + (int32_t)threadIdx.x;
            m0[u] = k[u] > 0u ? f.pmask[i] : 0ull;
            m1[u] = k[u] > 1u ? f.pmask[(int64_t)n + i] : 0ull;
        }
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
        if (carry_s > 3u * (uint32_t)n || long_tokens != 0)
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
            uint64_t heavy = __ballot(k[u] > 2u);
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
    }
    __syncthreads();
    const uint32_t n_pairs = carry_s;
    bool ok = n_pairs <= 3u * (uint32_t)n && long_tokens == 0;       // uniform over the workgroup
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
        // the transpose: for every class, the sets that contain it (bit k of word k / 64 = set k)
        if (ok && threadIdx.x < 64) {
            uint64_t w[kSetCap / 64] = {};
            for (uint32_t k2 = 0; k2 < n_sets; ++k2)
                if ((by_id[k2] >> threadIdx.x) & 1ull)
                    w[k2 / 64] |= 1ull << (k2 & 63);
            for (int j = 0; j < kSetCap / 64; ++j)
                f.class_sets[threadIdx.x * (kSetCap / 64) + j] = w[j];
        }
    }
    if (threadIdx.x == 0) {
        st->n_sets = n_sets;
        st->n_pairs = n_pairs;
        st->use_sets = ok && f.expect != 2u ? 1u : 0u;
        if (ok && f.expect == 2u)
            st->feasible = 1;                                    // the dense kernel counts; the host learns for next time
        if (!ok && f.expect == 1u)
            st->overflow = 2;                                    // nobody else will count: the host has to ask again
    }
}

// The first `pack_groups` workgroups pack 256 token slots each, the others narrow four states
// each, one wave per state (neither job needs the other; both need classify_bytes to have run).
template <typename E>
__global__ __launch_bounds__(256) void pack_and_narrow(int32_t pack_groups, const int64_t *__restrict__ offsets,
                                                       int32_t n_tokens, int64_t n_bytes, int32_t eos, int32_t n_slots,
                                                       const uint8_t *__restrict__ cls, TokenRecord *__restrict__ tok,
                                                       uint32_t *__restrict__ key,
                                                       const int32_t *__restrict__ trans, int32_t n_states,
                                                       int32_t n_classes, int32_t dead, int32_t live_words,
                                                       E *__restrict__ tab, uint64_t *__restrict__ live,
                                                       uint32_t *__restrict__ npairs, uint32_t *__restrict__ pairs,
                                                       uint64_t *__restrict__ pmask, Status *st)
{
    if ((int32_t)blockIdx.x < pack_groups) {
        pack_token((int32_t)(blockIdx.x * blockDim.x + threadIdx.x), offsets, n_tokens, n_bytes, eos, n_slots, cls, tok, key, st);
        return;
    }
    const int32_t q = ((int32_t)blockIdx.x - pack_groups) * 4 + (int32_t)(threadIdx.x >> 6);
    if (q < n_states)
        narrow_state<E>(q, threadIdx.x & (kWave - 1), trans, n_states, n_classes, dead, live_words, tab, live, npairs,
                        pairs, pmask, st);
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
    f.expect = (uint32_t)expect;

    {
        int64_t want = (p.n_bytes / 16 + 255) / 256;
        int blocks = (int)(want < 1 ? 1 : (want > 2048 ? 2048 : want));
        hipLaunchKernelGGL(classify_bytes, dim3(blocks), dim3(256), 0, stream, vocab.bytes, p.n_bytes,
                           dfa.byte_to_class, p.n_classes, cls, st);
    }
    const int32_t n_slots = p.n_chunks * kChunkTokens;
    const int32_t pack_groups = (n_slots + 255) / 256;
    const dim3 grid((unsigned)(pack_groups + (p.n_states + 3) / 4));
    if (p.entry_bytes == 2)
        hipLaunchKernelGGL(pack_and_narrow<uint16_t>, grid, dim3(256), 0, stream, pack_groups, vocab.offsets, p.n_tokens,
                           p.n_bytes, vocab.eos_token_id, n_slots, cls, tok, key, dfa.trans, p.n_states, p.n_classes,
                           dfa.dead_state, p.live_words, reinterpret_cast<uint16_t *>(ws + p.off_tab), live, npairs, pairs,
                           pmask, st);
    else
        hipLaunchKernelGGL(pack_and_narrow<uint32_t>, grid, dim3(256), 0, stream, pack_groups, vocab.offsets, p.n_tokens,
                           p.n_bytes, vocab.eos_token_id, n_slots, cls, tok, key, dfa.trans, p.n_states, p.n_classes,
                           dfa.dead_state, p.live_words, reinterpret_cast<uint32_t *>(ws + p.off_tab), live,
                           static_cast<uint32_t *>(nullptr), static_cast<uint32_t *>(nullptr), static_cast<uint64_t *>(nullptr), st);
    if (with_sets)
        hipLaunchKernelGGL(finish_sets, dim3(2), dim3(kFinishThreads), 0, stream, f, st);
    return hipGetLastError();
}

}  // namespace fsmidx
