// Minimisation of the automaton before it is indexed (Section 5: the indices measured in the paper
// come from un-reduced automata, whose redundant states make them larger than they have to be).
//
// What the index records about a walk is whether it meets the rejecting state and whether the state
// it ends in accepts (Section 3, Algorithms 3 and 4; Section 2.1 for EOS), so a state has one of
// three labels -- rejecting state, accepting, neither -- and two states are equivalent iff every
// string of byte classes leads them to equally labelled states.  The classes are found by
// refinement (Moore): start from the labels; a round gives every state the signature (its class,
// the classes of its successors), groups equal signatures and numbers the groups in order of their
// smallest state; when a round leaves the number of classes unchanged, the partition is final.
//
//  min_start      labels as the first classes, input range checks
//  per round:
//   min_clear     the hash table of the round
//   min_group     a wave per state: 64-bit hash of the signature; the state joins the group of its
//                 hash (open addressing), the group keeps its smallest state
//   min_verify    a wave per state: the signature is compared, class by class, with that of the
//                 group's smallest state: exact, a collision of hashes is noticed (the host starts
//                 again with another seed)
//   min_number    one workgroup: groups numbered in order of their smallest state; the new classes
//  min_quotient   the quotient automaton: one state per class, taken from the class's smallest state
//
// Rounds are enqueued without waiting for each other (the class counts go to a list that the host
// reads once per batch); a round on a final partition changes nothing.
#include "internal.h"

namespace fsmidx {

constexpr int kMinRoundsMax = 1 << 16;     // class counts kept (the list is reused in turns of this many rounds)

__device__ __forceinline__ uint64_t min_mix(uint64_t x)
{
    x ^= x >> 33;
    x *= 0xFF51AFD7ED558CCDull;
    x ^= x >> 33;
    x *= 0xC4CEB9FE1A85EC53ull;
    x ^= x >> 33;
    return x;
}

struct MinBuffers {
    int64_t *result;            // [0] classes after the last round, [1] input check flags, [2] != 0: hashes collided
    uint32_t *counts;           // [kMinRoundsMax] classes after round r at r % kMinRoundsMax
    uint32_t *block;            // [n_states] class of a state
    uint32_t *slot_of;          // [n_states] the state's slot in the table
    uint32_t *canon;            // [n_states] smallest state of the state's group
    uint32_t *number;           // [n_states] for the smallest state of a group: the group's number
    uint32_t *rep_state;        // [n_states] class -> its smallest state
    unsigned long long *keys;   // [table] 0 = free
    uint32_t *rep;              // [table] smallest state of the group
    uint32_t table_mask;
};

static uint32_t min_table_slots(int32_t n_states)
{
    uint32_t t = 64;
    while (t < 2u * (uint32_t)n_states)
        t <<= 1;
    return t;
}

static size_t up256(size_t x) { return (x + 255) / 256 * 256; }

size_t minimise_workspace_bytes(int32_t n_states)
{
    const size_t q = up256((size_t)n_states * 4), t = min_table_slots(n_states);
    return 256 + up256((size_t)kMinRoundsMax * 4) + 5 * q + up256(t * 8) + up256(t * 4);
}

static MinBuffers min_buffers(char *ws, int32_t n_states)
{
    const size_t q = up256((size_t)n_states * 4), t = min_table_slots(n_states);
    MinBuffers b;
    size_t o = 0;
    b.result = reinterpret_cast<int64_t *>(ws + o);            o += 256;
    b.counts = reinterpret_cast<uint32_t *>(ws + o);           o += up256((size_t)kMinRoundsMax * 4);
    b.block = reinterpret_cast<uint32_t *>(ws + o);            o += q;
    b.slot_of = reinterpret_cast<uint32_t *>(ws + o);          o += q;
    b.canon = reinterpret_cast<uint32_t *>(ws + o);            o += q;
    b.number = reinterpret_cast<uint32_t *>(ws + o);           o += q;
    b.rep_state = reinterpret_cast<uint32_t *>(ws + o);        o += q;
    b.keys = reinterpret_cast<unsigned long long *>(ws + o);   o += up256(t * 8);
    b.rep = reinterpret_cast<uint32_t *>(ws + o);
    b.table_mask = (uint32_t)t - 1u;
    return b;
}

// successor of q under class c, range checked (a bad entry raises a flag and stays put)
__device__ __forceinline__ uint32_t min_next(const int32_t *__restrict__ trans, int32_t n_states, int32_t n_classes,
                                             uint32_t q, uint32_t c, uint32_t &bad)
{
    const int32_t v = trans[(int64_t)q * n_classes + c];
    if (v < 0 || v >= n_states) {
        bad |= kBadTransition;
        return q;
    }
    return (uint32_t)v;
}

__global__ __launch_bounds__(256) void min_start(const int32_t *__restrict__ trans, const uint8_t *__restrict__ accept,
                                                 int32_t n_states, int32_t n_classes, int32_t dead, const MinBuffers b)
{
    const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q == 0) {
        b.result[0] = 0;
        b.result[2] = 0;
    }
    if (q >= n_states)
        return;
    b.block[q] = q == dead ? 0u : (accept[q] != 0 ? 1u : 2u);
    if (q == dead) {
        uint32_t bad = 0;
        for (int32_t c = 0; c < n_classes; ++c)
            if (trans[q * n_classes + c] != dead)
                bad = kDeadNotAbsorbing;
        if (bad)
            atomicOr(reinterpret_cast<unsigned long long *>(&b.result[1]), (unsigned long long)bad);
    }
}

__global__ __launch_bounds__(256) void min_reset_flags(const MinBuffers b)
{
    if (blockIdx.x == 0 && threadIdx.x == 0)
        b.result[1] = 0;
}

__global__ __launch_bounds__(256) void min_clear(const MinBuffers b)
{
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i <= (uint64_t)b.table_mask) {
        b.keys[i] = 0ull;
        b.rep[i] = 0xFFFFFFFFu;
    }
}

// grid: one wave per state
__global__ __launch_bounds__(kWave) void min_group(const int32_t *__restrict__ trans, int32_t n_states, int32_t n_classes,
                                                   uint64_t seed, const MinBuffers b)
{
    const uint32_t q = blockIdx.x;
    const int lane = threadIdx.x;
    uint32_t bad = 0;
    uint64_t sum = 0;
    for (uint32_t c = (uint32_t)lane; c < (uint32_t)n_classes; c += kWave) {
        const uint32_t s = min_next(trans, n_states, n_classes, q, c, bad);
        sum += min_mix(((uint64_t)b.block[s] << 32 | c) ^ seed);          // the position counts: a signature is a sequence
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1)
        sum += __shfl_xor(sum, o, kWave);
    if (__ballot(bad != 0) != 0 && lane == 0)
        atomicOr(reinterpret_cast<unsigned long long *>(&b.result[1]), (unsigned long long)kBadTransition);
    if (lane != 0)
        return;
    const unsigned long long key = min_mix(sum + (uint64_t)b.block[q] * 0x9E3779B97F4A7C15ull + seed) | 1ull;   // never 0
    uint32_t h = (uint32_t)(key >> 20) & b.table_mask;
    for (;;) {                                                     // the table has at least twice as many slots as states
        const unsigned long long old = atomicCAS(&b.keys[h], 0ull, key);
        if (old == 0ull || old == key)
            break;
        h = (h + 1) & b.table_mask;
    }
    atomicMin(&b.rep[h], q);
    b.slot_of[q] = h;
}

// grid: one wave per state
__global__ __launch_bounds__(kWave) void min_verify(const int32_t *__restrict__ trans, int32_t n_states, int32_t n_classes,
                                                    const MinBuffers b)
{
    const uint32_t q = blockIdx.x;
    const int lane = threadIdx.x;
    const uint32_t r = b.rep[b.slot_of[q]];
    if (lane == 0)
        b.canon[q] = r;
    if (r == q)
        return;
    uint32_t bad = 0;
    bool differ = b.block[q] != b.block[r];
    for (uint32_t c = (uint32_t)lane; c < (uint32_t)n_classes; c += kWave)
        differ = differ || b.block[min_next(trans, n_states, n_classes, q, c, bad)] !=
                               b.block[min_next(trans, n_states, n_classes, r, c, bad)];
    if (__ballot(differ) != 0 && lane == 0)
        b.result[2] = 1;
}

// one workgroup: the groups numbered in order of their smallest state; every state's new class
__global__ __launch_bounds__(1024) void min_number(int32_t n_states, const MinBuffers b, uint32_t round)
{
    __shared__ uint32_t wave_cnt[16];
    __shared__ uint32_t carry;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    if (threadIdx.x == 0)
        carry = 0;
    __syncthreads();
    for (int32_t q0 = 0; q0 < n_states; q0 += 1024) {
        const int32_t q = q0 + (int32_t)threadIdx.x;
        const bool is_rep = q < n_states && b.canon[q] == (uint32_t)q;
        const uint64_t m = __ballot(is_rep);
        if (lane == 0)
            wave_cnt[wave] = (uint32_t)__popcll(m);
        __syncthreads();
        uint32_t before = carry;
        for (int w = 0; w < wave; ++w)
            before += wave_cnt[w];
        if (is_rep) {
            const uint32_t u = before + __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
            b.number[q] = u;
            b.rep_state[u] = (uint32_t)q;
        }
        __syncthreads();
        if (threadIdx.x == 1023)
            carry = before + (uint32_t)__popcll(m);
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        b.result[0] = (int64_t)carry;
        b.counts[round % (uint32_t)kMinRoundsMax] = carry;
    }
    __threadfence();
    __syncthreads();
    for (int32_t q = threadIdx.x; q < n_states; q += 1024)
        b.block[q] = b.number[b.canon[q]];
}

// grid: one wave per state slot; waves past the number of classes have nothing to do
__global__ __launch_bounds__(kWave) void min_quotient(const int32_t *__restrict__ trans, const uint8_t *__restrict__ accept,
                                                      int32_t n_states, int32_t n_classes, const MinBuffers b,
                                                      int32_t *__restrict__ block_of_state, int32_t *__restrict__ trans_out,
                                                      int64_t trans_capacity, uint8_t *__restrict__ accept_out)
{
    const uint32_t u = blockIdx.x;
    const int lane = threadIdx.x;
    if (lane == 0)
        block_of_state[u] = (int32_t)b.block[u];                   // (u is a state here)
    if ((int64_t)u >= b.result[0] || ((int64_t)u + 1) * n_classes > trans_capacity)
        return;
    const uint32_t q = b.rep_state[u];
    uint32_t bad = 0;
    for (uint32_t c = (uint32_t)lane; c < (uint32_t)n_classes; c += kWave)
        trans_out[(int64_t)u * n_classes + c] = (int32_t)b.block[min_next(trans, n_states, n_classes, q, c, bad)];
    if (lane == 0)
        accept_out[u] = accept[q] != 0 ? 1 : 0;
}

hipError_t launch_min_start(const fsmidx_dfa &dfa, char *ws, bool first_attempt, hipStream_t stream)
{
    const MinBuffers b = min_buffers(ws, dfa.n_states);
    if (first_attempt)
        hipLaunchKernelGGL(min_reset_flags, dim3(1), dim3(256), 0, stream, b);
    hipLaunchKernelGGL(min_start, dim3((unsigned)((dfa.n_states + 255) / 256)), dim3(256), 0, stream, dfa.trans, dfa.accept,
                       dfa.n_states, dfa.n_classes, dfa.dead_state, b);
    return hipGetLastError();
}

hipError_t launch_min_rounds(const fsmidx_dfa &dfa, char *ws, uint64_t seed, uint32_t first_round, int n_rounds,
                             hipStream_t stream)
{
    const MinBuffers b = min_buffers(ws, dfa.n_states);
    const unsigned table_blocks = (unsigned)(((uint64_t)b.table_mask + 256) / 256);
    for (int r = 0; r < n_rounds; ++r) {
        hipLaunchKernelGGL(min_clear, dim3(table_blocks), dim3(256), 0, stream, b);
        hipLaunchKernelGGL(min_group, dim3((unsigned)dfa.n_states), dim3(kWave), 0, stream, dfa.trans, dfa.n_states,
                           dfa.n_classes, seed, b);
        hipLaunchKernelGGL(min_verify, dim3((unsigned)dfa.n_states), dim3(kWave), 0, stream, dfa.trans, dfa.n_states,
                           dfa.n_classes, b);
        hipLaunchKernelGGL(min_number, dim3(1), dim3(1024), 0, stream, dfa.n_states, b, first_round + (uint32_t)r);
    }
    return hipGetLastError();
}

// what the host reads after a batch of rounds: result words and the class counts of rounds [first, first + n)
const int64_t *min_result(char *ws, int32_t n_states) { return min_buffers(ws, n_states).result; }
const uint32_t *min_counts(char *ws, int32_t n_states) { return min_buffers(ws, n_states).counts; }
const uint32_t *min_block(char *ws, int32_t n_states) { return min_buffers(ws, n_states).block; }
int min_rounds_max() { return kMinRoundsMax; }

hipError_t launch_min_quotient(const fsmidx_dfa &dfa, char *ws, int32_t *block_of_state, int32_t *trans_out,
                               int64_t trans_capacity, uint8_t *accept_out, hipStream_t stream)
{
    const MinBuffers b = min_buffers(ws, dfa.n_states);
    hipLaunchKernelGGL(min_quotient, dim3((unsigned)dfa.n_states), dim3(kWave), 0, stream, dfa.trans, dfa.accept,
                       dfa.n_states, dfa.n_classes, b, block_of_state, trans_out, trans_capacity, accept_out);
    return hipGetLastError();
}

}  // namespace fsmidx
