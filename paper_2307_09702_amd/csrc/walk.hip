// The DFA walk (Section 3, Algorithm 3) over every (state, token) pair: the counting pass for
// automata that the token-set walk does not take (many classes, many targets per state, long
// tokens, more than 65535 states).
//
// Work decomposition.  A workgroup of four waves owns one token group (1024 tokens, 16 chunks of
// 64) and four ranges of consecutive states, one per wave.  The group's leading byte classes and
// lengths are staged in LDS once per workgroup.  For each state q of its range a wave decides the
// 1024 pairs (q, token):
//
//   byte 0   row q of the narrowed table is put into LDS (one coalesced load), and every lane
//            looks up its token's first class there: no memory gather at all.  This is Algorithm
//            3's restriction to the states that can read the first symbol, turned around: for most
//            automata most pairs end here.
//   survivors (the walk goes on: not rejected, token longer than one byte) are compacted into a
//            queue in LDS -- (state reached, token) -- so that the table lookups of the following
//            bytes, which are gathers from memory, are issued by full waves however few pairs
//            survive: a wave-wide gather costs the same whether one lane or all of them need it.
//            The queue is compacted again after every byte, in place.
//   finished pairs (token read to its end without meeting the dead state) set their bit in the
//            wave's 1024-bit admissibility row in LDS; the row is the index as a bitmap, and its
//            popcount is the length of the group's segment of row q.
//
// The end states are not kept: after the scans the emitting pass walks the admissible pairs again
// and writes them in ascending token id.  Nothing here depends on the order in which atomics are
// served (the only ones are ORs into the wave's own bitmap), so the CSR is deterministic.
#include <type_traits>

#include "internal.h"

namespace fsmidx {

constexpr int kWalkBatch = 4;          // gathers a lane has in flight when working off the queue
constexpr int kWalkSlots = 8;          // most states whose survivors share one queue

struct WalkArgs {
    const TokenRecord *tok;
    const uint8_t *cls;
    const void *tab;
    const uint8_t *accept;
    uint32_t *cnt;             // [n_states][n_groups]
    int32_t n_states, n_classes, n_tokens, n_groups, n_ranges, states_per_wave;
    int32_t dead, eos;
    uint32_t tab_bytes;        // size of the narrowed table (LDS variant)
    const Status *status;      // use_sets != 0: the token-set kernels do this pass instead
    uint64_t *allow;           // [n_states][n_chunks] admissibility words
    int32_t n_chunks;
};

// Queue entries of one wave: one and a half states' worth.  A larger queue lets more states share
// a round of lookups, a smaller one lets more waves share a compute unit (LDS per workgroup is
// what limits them, and this kernel lives on overlapping the waits of many waves); measured on a
// 20,000-state automaton with 64 classes: 1024 entries 4.1 ms, 1280 3.7, 1536 3.3, 2048 4.0.
template <typename E> struct QueueCap { static constexpr int value = kGroupTokens + kGroupTokens / 2; };

// LDS of one workgroup, after the table copy (TAB_LDS only).
template <typename E>
struct alignas(16) WalkShared {
    uint64_t packed[kGroupTokens];                    // leading byte classes of the group's tokens, 8 bits each
    uint16_t length[kGroupTokens];                    // their lengths (clamped to 65535: see the kernel)
    struct PerWave {
        E row[256];                                   // row q of the table
        E state[QueueCap<E>::value];                  // queue: state reached ...
        uint16_t token[QueueCap<E>::value];           //        ... by this token of the group | slot of the start state << 10
        uint64_t bits[kWalkSlots][kChunksPerWave];    // per slot: admissible tokens of the group from that state
    } wave[kWavesPerBlock];
};

// E: narrowed entry type.  TAB_LDS: the whole table is first copied to LDS.
//
// The bytes after the first are a chain of dependent memory round trips, one per byte position,
// each for ever fewer pairs.  So the survivors of several consecutive states share one queue
// (as many states as leave room for a whole group of survivors of the next one, at most
// kWalkSlots): the chain is then paid once for all of them.
template <typename E, bool TAB_LDS>
__global__ __launch_bounds__(kWave *kWavesPerBlock) void walk_pairs(const WalkArgs a)
{
    constexpr int kCap = QueueCap<E>::value;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    if (a.status->use_sets)
        return;                                                // uniform over the grid
    const E *tab = static_cast<const E *>(a.tab);
    uint32_t tab_lds = 0;
    if (TAB_LDS) {
        const uint32_t n16 = a.tab_bytes / 16;                 // table bytes are padded to 16
        const uint4 *src = static_cast<const uint4 *>(a.tab);
        uint4 *dst = reinterpret_cast<uint4 *>(lds_raw);
        for (uint32_t i = threadIdx.x; i < n16; i += blockDim.x)
            dst[i] = src[i];
        tab = reinterpret_cast<const E *>(lds_raw);
        tab_lds = a.tab_bytes;
    }
    WalkShared<E> &sh = *reinterpret_cast<WalkShared<E> *>(lds_raw + tab_lds);
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    typename WalkShared<E>::PerWave &my = sh.wave[wave];
    const E dead_e = a.dead >= 0 ? (E)a.dead : (E) ~(E)0;
    const uint32_t n_classes = (uint32_t)a.n_classes;
    // the grid is capped: a workgroup takes units blockIdx.x, + gridDim.x, ...; a unit is one token
    // group and kWavesPerBlock state ranges
    const int32_t range_sets = (a.n_ranges + kWavesPerBlock - 1) / kWavesPerBlock;
    const int64_t n_units = (int64_t)a.n_groups * range_sets;
    for (int64_t unit = blockIdx.x; unit < n_units; unit += gridDim.x) {
        const int32_t g = (int32_t)(unit % a.n_groups);
        const int32_t r = (int32_t)(unit / a.n_groups) * kWavesPerBlock + wave;
        const int32_t q_lo = (int32_t)min((int64_t)r * a.states_per_wave, (int64_t)a.n_states);
        const int32_t q_hi = (int32_t)min((int64_t)q_lo + a.states_per_wave, (int64_t)a.n_states);
        const int32_t t_base = g * kGroupTokens;
        __syncthreads();                                       // the last unit's tokens are no longer read (and, the
                                                               // first time, the table copy is complete)
        uint32_t first[kChunksPerWave];                        // per chunk, this lane's token: first class | length << 8
#pragma unroll
        for (int k = 0; k < kChunksPerWave; ++k) {
            const TokenRecord rec = a.tok[t_base + k * kWave + lane];
            // (16 bits of length are enough here: they are only compared with the first eight byte
            // positions; from the ninth byte on a walk reads the real length from the token's record)
            const uint32_t len = min(rec.length, 65535u);
            first[k] = (rec.cls_lo & 255u) | len << 8;
            if (k % kWavesPerBlock == wave) {                  // every wave stages a quarter of the group
                sh.packed[k * kWave + lane] = ((uint64_t)rec.cls_hi << 32) | rec.cls_lo;
                sh.length[k * kWave + lane] = (uint16_t)len;
            }
        }
        __syncthreads();
        const bool group_has_eos = a.eos >= t_base && a.eos < t_base + kGroupTokens;

        // One byte position of the queue's pairs [b0, b0 + U * 64): look up, finish or keep.
        // Compaction is in place: a pair is written at or before the place it was read from, and
        // the reads of a call are issued before its writes.
        auto advance = [&](auto batch, const uint32_t d, const uint32_t b0, const uint32_t n, uint32_t &kept) {
            constexpr int U = decltype(batch)::value;
            uint32_t s[U], t[U], c[U], len[U];
            E s2[U];
            bool valid[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t at = b0 + (uint32_t)(u * kWave + lane);
                valid[u] = at < n;
                s[u] = valid[u] ? (uint32_t)my.state[at] : 0u;
                t[u] = valid[u] ? (uint32_t)my.token[at] : 0u;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t tt = t[u] & (uint32_t)(kGroupTokens - 1);
                len[u] = sh.length[tt];
                if (d < (uint32_t)kPackedClasses) {
                    c[u] = (uint32_t)(sh.packed[tt] >> (8 * d)) & 255u;
                } else {
                    // (few walks get this far) the class string; the real length, which may exceed 16 bits
                    c[u] = 0;
                    if (valid[u]) {
                        const TokenRecord rec = a.tok[t_base + (int32_t)tt];
                        c[u] = a.cls[rec.offset + d];
                        len[u] = rec.length;
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
                s2[u] = valid[u] ? tab[s[u] * n_classes + c[u]] : dead_e;
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const bool alive = valid[u] && s2[u] != dead_e;
                const bool done = alive && len[u] == d + 1u;
                const bool more = alive && !done;
                if (done) {
                    const uint32_t tt = t[u] & (uint32_t)(kGroupTokens - 1);
                    atomicOr(reinterpret_cast<unsigned long long *>(&my.bits[t[u] >> 10][tt >> 6]), 1ull << (tt & 63u));
                }
                const uint64_t m = __ballot(more);
                if (more) {
                    const uint32_t at = kept + __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32),
                                                                         __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
                    my.state[at] = s2[u];
                    my.token[at] = (uint16_t)t[u];
                }
                kept += (uint32_t)__popcll(m);
            }
            __builtin_amdgcn_wave_barrier();
        };

        for (int32_t q0 = q_lo; q0 < q_hi;) {
            // ---- byte 0 of the next states, from their table rows in LDS, while the queue has room
            //      for all 1024 pairs of one more state
            uint32_t n = 0;                                        // pairs in the queue
            int slots = 0;
            while (q0 + slots < q_hi && slots < kWalkSlots && n + (uint32_t)kGroupTokens <= (uint32_t)kCap) {
                const int32_t q = q0 + slots;
                const bool is_dead = q == a.dead;                  // the dead state's row is empty
                for (uint32_t c = (uint32_t)lane; c < n_classes; c += kWave)
                    my.row[c] = tab[(uint32_t)q * n_classes + c];
                __builtin_amdgcn_wave_barrier();
                // (all look-ups of the state first: one wait for sixteen reads instead of sixteen waits)
                E after[kChunksPerWave];
#pragma unroll
                for (int k = 0; k < kChunksPerWave; ++k)
                    after[k] = my.row[first[k] & 255u];
#pragma unroll
                for (int k = 0; k < kChunksPerWave; ++k) {
                    const uint32_t len = first[k] >> 8;
                    const E s1 = after[k];
                    const bool alive = len != 0 && s1 != dead_e && !is_dead;
                    const uint64_t done = __ballot(alive && len == 1u);
                    const uint64_t more = __ballot(alive && len > 1u);
                    if (lane == 0)
                        my.bits[slots][k] = done;
                    if (alive && len > 1u) {
                        const uint32_t at = n + __builtin_amdgcn_mbcnt_hi((uint32_t)(more >> 32),
                                                                          __builtin_amdgcn_mbcnt_lo((uint32_t)more, 0u));
                        my.state[at] = s1;
                        my.token[at] = (uint16_t)((uint32_t)(k * kWave + lane) | (uint32_t)slots << 10);
                    }
                    n += (uint32_t)__popcll(more);
                }
                // EOS has no bytes: admissible exactly from accepting states
                if (group_has_eos && !is_dead && a.accept[q] != 0 && lane == 0) {
                    const int32_t e = a.eos - t_base;
                    my.bits[slots][e >> 6] |= 1ull << (e & 63);
                }
                __builtin_amdgcn_wave_barrier();                   // the row is read before the next state's is written
                ++slots;
            }
            // ---- bytes 1, 2, ...
            for (uint32_t d = 1; n != 0; ++d) {
                uint32_t kept = 0;
                for (uint32_t b0 = 0; b0 < n;) {
                    if (n - b0 > (uint32_t)kWave) {
                        advance(std::integral_constant<int, kWalkBatch>{}, d, b0, n, kept);
                        b0 += kWalkBatch * kWave;
                    } else {
                        advance(std::integral_constant<int, 1>{}, d, b0, n, kept);
                        b0 += kWave;
                    }
                }
                n = kept;
            }
            __builtin_amdgcn_wave_barrier();
            // ---- the bitmap rows of (state, group) and their popcounts
            for (int j = 0; j < slots; ++j) {
                const int32_t q = q0 + j;
                uint32_t count = 0;
                if (lane < kChunksPerWave) {
                    const uint64_t word = my.bits[j][lane];
                    a.allow[(int64_t)q * a.n_chunks + g * kChunksPerWave + lane] = word;
                    count = (uint32_t)__popcll(word);
                }
#pragma unroll
                for (int o = kChunksPerWave / 2; o >= 1; o >>= 1)
                    count += __shfl_xor(count, o, kWave);
                if (lane == 0)
                    a.cnt[(int64_t)q * a.n_groups + g] = count;
            }
            __builtin_amdgcn_wave_barrier();
            q0 += slots;
        }
    }
}

template <typename E, bool TAB_LDS>
static void launch_variant(const WalkArgs &a, int64_t n_units, size_t lds, hipStream_t stream)
{
    // a few workgroups per compute unit: when the token-set kernel does the work instead, these have
    // nothing to do but to find that out
    const dim3 grid((unsigned)(n_units < 4096 ? n_units : 4096));
    const dim3 block(kWave * kWavesPerBlock);
    hipLaunchKernelGGL((walk_pairs<E, TAB_LDS>), grid, block, lds + sizeof(WalkShared<E>), stream, a);
}

hipError_t launch_walk(const Plan &p, const fsmidx_dfa &dfa, const fsmidx_vocab &vocab, char *ws, hipStream_t stream)
{
    if (p.n_groups == 0 || p.n_states == 0)
        return hipSuccess;
    WalkArgs a;
    a.tok = reinterpret_cast<const TokenRecord *>(ws + p.off_tok);
    a.cls = reinterpret_cast<const uint8_t *>(ws + p.off_cls);
    a.tab = ws + p.off_tab;
    a.accept = dfa.accept;
    a.cnt = reinterpret_cast<uint32_t *>(ws + p.off_cnt);
    a.n_states = p.n_states;
    a.n_classes = p.n_classes;
    a.n_tokens = p.n_tokens;
    a.n_groups = p.n_groups;
    a.n_ranges = p.n_ranges;
    a.states_per_wave = p.states_per_wave;
    a.dead = dfa.dead_state;
    a.eos = vocab.eos_token_id;
    a.status = reinterpret_cast<const Status *>(ws + p.off_status);
    a.allow = reinterpret_cast<uint64_t *>(ws + p.off_allow);
    a.n_chunks = p.n_chunks;
    const size_t tab_bytes = ((size_t)p.n_states * p.n_classes * p.entry_bytes + 15) / 16 * 16;
    a.tab_bytes = (uint32_t)(tab_bytes <= 0xFFFFFFFFu ? tab_bytes : 0);
    const int64_t n_units = (int64_t)p.n_groups * ((p.n_ranges + kWavesPerBlock - 1) / kWavesPerBlock);
    const bool lds = tab_bytes <= 12 * 1024;                       // beside the queues, within 64 KB per workgroup
    const size_t lds_bytes = lds ? tab_bytes : 0;
    if (p.entry_bytes == 2) {
        if (lds) launch_variant<uint16_t, true>(a, n_units, lds_bytes, stream);
        else launch_variant<uint16_t, false>(a, n_units, 0, stream);
    } else {
        launch_variant<uint32_t, false>(a, n_units, 0, stream);
    }
    return hipGetLastError();
}

}  // namespace fsmidx
