// Preparation for the token-set walk (automata with at most 64 byte classes).
//
// The table narrowing kernel has regrouped the transition function delta (Section 3, Definition 1)
// by target: state s has a list of pairs (target, class set), one per distinct non-rejecting
// target, smallest class set first, and the class sets that occur anywhere in the automaton are
// numbered.  Here, for every set S and byte position d, a bitmap over the vocabulary says which
// tokens are longer than d bytes and have their d-th byte in S.  With these bitmaps "which tokens of
// this token set can state s read next" -- the test inside Algorithm 3's inner loop, for a whole
// set of tokens at once -- is one AND.
//
//  token_sets  : bitmaps U[d][set][chunk] and the end-of-token bitmaps E[d][chunk]; also one
//                16-byte record per state (pair count, first two pairs, start of the rest), the
//                pairs' class sets renamed from table slots to set numbers on the way
#include "internal.h"

namespace fsmidx {

// The record of state q (the caller checks q < n_states).  The state's pairs start at q * n_classes
// and hold their targets: here they get the numbers of their class sets (pslot: the sets' slots in
// the table, pair i of state q at i * n_states + q; ids: slot -> number).
__device__ __forceinline__ void state_record(const uint32_t *__restrict__ npairs, uint32_t *__restrict__ pairs,
                                             const uint32_t *__restrict__ pslot, const uint32_t *__restrict__ ids,
                                             int32_t n_states, int32_t n_classes, int32_t q,
                                             StateRecord *__restrict__ srec)
{
    const uint32_t b = (uint32_t)q * (uint32_t)n_classes, n = npairs[q];
    StateRecord r;
    r.n_pairs = n;
    r.pair0 = 0u;
    r.pair1 = 0u;
    for (uint32_t i = 0; i < n; ++i) {
        const uint32_t slot = pslot[(int64_t)i * n_states + q] & (uint32_t)(kSetHashSlots - 1);
        const uint32_t named = (pairs[b + i] & 0xFFFFu) | ids[slot] << 16;
        pairs[b + i] = named;
        if (i == 0)
            r.pair0 = named;
        if (i == 1)
            r.pair1 = named;
    }
    r.ext = b + 2;
    srec[q] = r;
}

// One wave per (group of kSetChunks consecutive chunks of 64 tokens, byte position d): if some
// token of the group has a byte at position d, the end-of-token words E[d] of the group's chunks
// and one word U[d][set] per chunk and class set.  Lane k ends up with the words of set k for all
// chunks of the group, 64 contiguous bytes.  Positions past the group's longest token are not
// written: the walks only ever look at bits of tokens that are that long (position 0 is always
// written, there a walk starts with every token).
//
// The workgroups past the last group (blockIdx.x >= n_chunks / kSetChunks, blockIdx.y == 0) write
// the state records instead, 64 states each: both jobs wait for the same kernel and for nothing
// else.
constexpr int kSetChunks = 8;

__global__ __launch_bounds__(kWave) void token_sets(const TokenRecord *__restrict__ tok, const uint8_t *__restrict__ cls,
                                                    const uint64_t *__restrict__ class_sets, int32_t n_chunks,
                                                    uint64_t *__restrict__ U, uint64_t *__restrict__ E,
                                                    const uint32_t *__restrict__ npairs, uint32_t *__restrict__ pairs,
                                                    const uint32_t *__restrict__ pslot,
                                                    const uint32_t *__restrict__ ids, int32_t n_states,
                                                    int32_t n_classes, StateRecord *__restrict__ srec, const Status *st)
{
    static_assert(kBlockChunks % kSetChunks == 0, "n_chunks is a multiple of the group size");
    if (!st->use_sets)
        return;
    const uint32_t n_sets = st->n_sets;
    const int lane = threadIdx.x;
    const int32_t n_chunk_groups = n_chunks / kSetChunks;
    if ((int32_t)blockIdx.x >= n_chunk_groups) {
        const int32_t q = ((int32_t)blockIdx.x - n_chunk_groups) * kWave + lane;
        if (blockIdx.y == 0 && q < n_states)
            state_record(npairs, pairs, pslot, ids, n_states, n_classes, q, srec);
        return;
    }
    const uint32_t d = blockIdx.y;
    const int32_t chunk0 = (int32_t)blockIdx.x * kSetChunks;
    uint32_t len[kSetChunks], c[kSetChunks];
    bool any = false;
#pragma unroll
    for (int i = 0; i < kSetChunks; ++i) {
        const TokenRecord r = tok[(int64_t)(chunk0 + i) * kChunkTokens + lane];
        len[i] = r.length;
        c[i] = 0;
        if (r.length > d) {
            any = true;
            if (d < (uint32_t)kPackedClasses)
                c[i] = ((d < 4 ? r.cls_lo >> (8 * d) : r.cls_hi >> (8 * (d - 4))) & 255u);
            else
                c[i] = cls[r.offset + d];
        }
        c[i] &= 63u;
    }
    if (d > 0 && __ballot(any) == 0)
        return;
    uint64_t ends = 0;                                           // lane i keeps the word of chunk i
#pragma unroll
    for (int i = 0; i < kSetChunks; ++i) {
        const uint64_t w = __ballot(len[i] == d + 1);
        if (lane == i)
            ends = w;
    }
    if (lane < kSetChunks)
        E[(int64_t)d * n_chunks + chunk0 + lane] = ends;
#pragma unroll
    for (int j = 0; j < kSetCap / 64; ++j) {
        const uint32_t s0 = (uint32_t)j * 64u;
        if (s0 >= n_sets)
            break;
        // Lane t holds, as bits, the sets s0.. that contain the class of token t; lane k must
        // store, as bits, the tokens whose class is in set s0 + k: a 64 x 64 bit transpose.
        uint64_t mine[kSetChunks];
#pragma unroll
        for (int i = 0; i < kSetChunks; ++i)
            mine[i] = transpose_bits(len[i] > d ? class_sets[c[i] * (kSetCap / 64) + j] : 0ull, lane);
        if (s0 + (uint32_t)lane < n_sets) {
            uint4 *dst = reinterpret_cast<uint4 *>(U + ((int64_t)d * kSetCap + s0 + lane) * n_chunks + chunk0);
#pragma unroll
            for (int i = 0; i < kSetChunks; i += 2)
                dst[i / 2] = make_uint4((uint32_t)mine[i], (uint32_t)(mine[i] >> 32), (uint32_t)mine[i + 1],
                                        (uint32_t)(mine[i + 1] >> 32));
        }
    }
}

hipError_t launch_token_sets(const Plan &p, const fsmidx_dfa &dfa, const fsmidx_vocab &vocab, char *ws,
                             hipStream_t stream)
{
    if (!p.sets_possible)
        return hipSuccess;
    const Status *st = reinterpret_cast<const Status *>(ws + p.off_status);
    SyncWords *sy = reinterpret_cast<SyncWords *>(ws + p.off_sync);
    hipLaunchKernelGGL(token_sets, dim3(p.n_chunks / kSetChunks + (p.n_states + kWave - 1) / kWave, kMaxSetDepth),
                       dim3(kWave), 0, stream, reinterpret_cast<const TokenRecord *>(ws + p.off_tok),
                       reinterpret_cast<const uint8_t *>(ws + p.off_cls),
                       reinterpret_cast<const uint64_t *>(ws + p.off_clsets), p.n_chunks,
                       reinterpret_cast<uint64_t *>(ws + p.off_U), reinterpret_cast<uint64_t *>(ws + p.off_E),
                       reinterpret_cast<const uint32_t *>(ws + p.off_npairs),
                       reinterpret_cast<uint32_t *>(ws + p.off_pairs),
                       reinterpret_cast<const uint32_t *>(ws + p.off_pslot), sy->ids, p.n_states, p.n_classes,
                       reinterpret_cast<StateRecord *>(ws + p.off_srec), st);
    return hipGetLastError();
}

}  // namespace fsmidx
