// Index size (Section 5: the index of a big grammar comes from many un-reduced automata with
// redundant states).  Two tools:
//
//  union      Many automata against one vocabulary in ONE build: the disjoint union of the automata
//      as a single automaton over the coarsest byte-class partition that refines all of theirs.
//      State s of automaton k becomes state_base[k] + s; every automaton's reject state becomes the
//      union's single dead state.  The ordinary build then indexes all of them at once, and the
//      vocabulary-only work (class string, token records, token bitmaps) is done once.
//        union_classes : one workgroup, thread = byte value: bytes are in one class iff every
//                        automaton puts them in one class; classes numbered by smallest byte
//        union_table   : one workgroup per state of the union: its row, renumbered
//
//  dedupe     States whose rows of sigma (Algorithm 4) are identical -- same tokens, same end states
//      -- need the row only once.  Rows are hashed (a sum over the entries, so slices of a row
//      are added up in any order with the same result), the states are grouped by hash in a table,
//      every state's row is compared entry by entry with the row of the smallest state of its
//      group (a difference would mean two different rows with one hash: reported, the host
//      starts again with another seed), and the distinct rows are numbered in order of their
//      smallest state.
//        dedupe_init, dedupe_hash, dedupe_group, dedupe_verify, dedupe_number, dedupe_copy
#include "internal.h"

namespace fsmidx {

// ------------------------------------------------------------------------------------- union

struct UnionArgs {
    const int32_t *trans[kMaxUnion];
    const uint8_t *accept[kMaxUnion];
    const uint8_t *byte_to_class[kMaxUnion];
    int32_t n_states[kMaxUnion], n_classes[kMaxUnion], dead[kMaxUnion];
    int32_t base[kMaxUnion + 1];
    int32_t n_dfas;
    int32_t union_dead;
};

// words[0] = number of classes of the union, words[1] = input check flags
__global__ __launch_bounds__(256) void union_classes(const UnionArgs a, uint8_t *__restrict__ union_b2c,
                                                     uint8_t *__restrict__ class_of, uint32_t *__restrict__ words)
{
    __shared__ uint8_t cls[kMaxUnion][256];
    __shared__ uint32_t wave_sum[4];
    __shared__ uint8_t id_of_first[256];
    const int b = threadIdx.x;
    const int lane = b & (kWave - 1), wave = b >> 6;
    uint32_t bad = 0;
    if (b == 0)
        words[1] = 0;                                              // (flags are raised after the barrier below)
    for (int k = 0; k < a.n_dfas; ++k) {
        uint32_t c = a.byte_to_class[k][b];
        if (c >= (uint32_t)a.n_classes[k]) {
            bad = kBadClass;
            c = 0;
        }
        cls[k][b] = (uint8_t)c;
    }
    __syncthreads();
    // the smallest byte that every automaton treats like this one
    int first = b;
    for (int other = 0; other < b; ++other) {
        bool same = true;
        for (int k = 0; k < a.n_dfas && same; ++k)
            same = cls[k][other] == cls[k][b];
        if (same) {
            first = other;
            break;
        }
    }
    const bool is_first = first == b;
    const uint64_t m = __ballot(is_first);
    if (lane == 0)
        wave_sum[wave] = (uint32_t)__popcll(m);
    __syncthreads();
    uint32_t before = 0, total = 0;
    for (int w = 0; w < 4; ++w) {
        if (w < wave)
            before += wave_sum[w];
        total += wave_sum[w];
    }
    const uint32_t id = before + __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
    if (is_first) {
        id_of_first[b] = (uint8_t)id;                              // at most 256 classes: ids 0 .. 255
        for (int k = 0; k < a.n_dfas; ++k)
            class_of[k * 256 + (int)id] = cls[k][b];
    }
    __syncthreads();
    union_b2c[b] = id_of_first[first];
    if (bad)
        atomicOr(&words[1], bad);
    if (b == 0)
        words[0] = total;
}

__global__ __launch_bounds__(256) void union_table(const UnionArgs a, const uint8_t *__restrict__ class_of,
                                                   int32_t n_union_classes, int32_t *__restrict__ trans_out,
                                                   uint8_t *__restrict__ accept_out, uint32_t *__restrict__ words)
{
    const int32_t row = blockIdx.x;
    int k = 0;
    while (k + 1 < a.n_dfas && row >= a.base[k + 1])
        ++k;
    const int32_t s = row - a.base[k];
    const int32_t n_states = a.n_states[k], n_classes = a.n_classes[k], dead = a.dead[k];
    uint32_t bad = 0;
    for (int32_t c = threadIdx.x; c < n_union_classes; c += blockDim.x) {
        const int32_t own = class_of[k * 256 + c];                 // checked: < n_classes
        int32_t t = a.trans[k][(int64_t)s * n_classes + own];
        if (t < 0 || t >= n_states) {
            bad = kBadTransition;
            t = s;
        }
        trans_out[(int64_t)row * n_union_classes + c] = (dead >= 0 && t == dead) ? a.union_dead : a.base[k] + t;
    }
    if (threadIdx.x == 0)
        accept_out[row] = a.accept[k][s] != 0 ? 1 : 0;
    if (bad)
        atomicOr(&words[1], bad);
}

hipError_t launch_union_classes(const fsmidx_dfa *dfas, int32_t n_dfas, uint8_t *union_b2c, char *ws,
                                hipStream_t stream)
{
    UnionArgs a = {};
    a.n_dfas = n_dfas;
    for (int k = 0; k < n_dfas; ++k) {
        a.byte_to_class[k] = dfas[k].byte_to_class;
        a.n_classes[k] = dfas[k].n_classes;
    }
    uint32_t *words = reinterpret_cast<uint32_t *>(ws);
    hipLaunchKernelGGL(union_classes, dim3(1), dim3(256), 0, stream, a, union_b2c, reinterpret_cast<uint8_t *>(ws + 256),
                       words);
    return hipGetLastError();
}

hipError_t launch_union_table(const fsmidx_dfa *dfas, int32_t n_dfas, const int32_t *state_base, int32_t union_dead,
                              int32_t n_union_classes, int32_t *trans_out, uint8_t *accept_out, char *ws,
                              hipStream_t stream)
{
    UnionArgs a = {};
    a.n_dfas = n_dfas;
    a.union_dead = union_dead;
    for (int k = 0; k < n_dfas; ++k) {
        a.trans[k] = dfas[k].trans;
        a.accept[k] = dfas[k].accept;
        a.n_states[k] = dfas[k].n_states;
        a.n_classes[k] = dfas[k].n_classes;
        a.dead[k] = dfas[k].dead_state;
        a.base[k] = state_base[k];
    }
    a.base[n_dfas] = state_base[n_dfas];
    hipLaunchKernelGGL(union_table, dim3((unsigned)state_base[n_dfas]), dim3(256), 0, stream, a,
                       reinterpret_cast<const uint8_t *>(ws + 256), n_union_classes, trans_out, accept_out,
                       reinterpret_cast<uint32_t *>(ws));
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------- dedupe

constexpr int kRowSlices = 16;         // waves that share a row (rows differ in length by four orders of magnitude)

__device__ __forceinline__ uint64_t mix64(uint64_t x)
{
    x ^= x >> 33;
    x *= 0xFF51AFD7ED558CCDull;
    x ^= x >> 33;
    x *= 0xC4CEB9FE1A85EC53ull;
    x ^= x >> 33;
    return x;
}

// entries [i0, i1) of a row of n entries that belong to `slice`: whole multiples of a wave
__device__ __forceinline__ void row_slice(int64_t n, int32_t slice, int64_t &i0, int64_t &i1)
{
    int64_t per = (n + kRowSlices - 1) / kRowSlices;
    per = (per + kWave - 1) / kWave * kWave;
    i0 = min(n, (int64_t)slice * per);
    i1 = min(n, i0 + per);
}

struct DedupeBuffers {
    uint64_t *hash;        // [n_states]  sum over the row's entries
    unsigned long long *keys;   // [table]  0 = free
    uint32_t *rep;         // [table]     smallest state of the group
    uint32_t *slot_of;     // [n_states]  the state's slot; later, for the smallest state of a distinct row, the row's number
    uint32_t *canon;       // [n_states]  smallest state with the same row
    uint32_t *rep_state;   // [n_states]  distinct row -> its smallest state
    int64_t *result;       // [0] distinct rows, [1] their entries, [2] != 0: two different rows with one hash
    uint32_t table_mask;
};

__global__ __launch_bounds__(256) void dedupe_init(const DedupeBuffers d, int32_t n_states)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_states)
        d.hash[i] = 0;
    if (i <= (int64_t)d.table_mask) {
        d.keys[i] = 0ull;
        d.rep[i] = 0xFFFFFFFFu;
    }
    if (i < 3)
        d.result[i] = 0;
}

// grid: n_states * kRowSlices single-wave workgroups
__global__ __launch_bounds__(kWave) void dedupe_hash(const int64_t *__restrict__ row_ptr,
                                                     const int32_t *__restrict__ token_ids,
                                                     const int32_t *__restrict__ next_states, uint64_t seed,
                                                     const DedupeBuffers d)
{
    const int32_t q = blockIdx.x / kRowSlices, slice = blockIdx.x % kRowSlices;
    const int64_t lo = row_ptr[q], n = row_ptr[q + 1] - lo;
    int64_t i0, i1;
    row_slice(n, slice, i0, i1);
    if (i0 >= i1)
        return;
    uint64_t sum = 0;
    for (int64_t i = i0 + threadIdx.x; i < i1; i += kWave) {
        const uint64_t entry = (uint64_t)(uint32_t)token_ids[lo + i] << 32 | (uint32_t)next_states[lo + i];
        sum += mix64(entry ^ mix64((uint64_t)i + seed));           // the position counts: a row is a sequence
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1)
        sum += __shfl_xor(sum, o, kWave);
    if (threadIdx.x == 0)
        atomicAdd(reinterpret_cast<unsigned long long *>(&d.hash[q]), (unsigned long long)sum);
}

// one thread per state: the state joins the group of its (hash, length)
__global__ __launch_bounds__(256) void dedupe_group(const int64_t *__restrict__ row_ptr, int32_t n_states,
                                                    const DedupeBuffers d)
{
    const int32_t q = blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= n_states)
        return;
    const uint64_t n = (uint64_t)(row_ptr[q + 1] - row_ptr[q]);
    const unsigned long long key = mix64(d.hash[q] + n * 0x9E3779B97F4A7C15ull) | 1ull;     // never 0
    uint32_t h = (uint32_t)(key >> 20) & d.table_mask;
    for (;;) {                                                     // the table has at least twice as many slots as states
        const unsigned long long old = atomicCAS(&d.keys[h], 0ull, key);
        if (old == 0ull || old == key)
            break;
        h = (h + 1) & d.table_mask;
    }
    atomicMin(&d.rep[h], (uint32_t)q);
    d.slot_of[q] = h;
}

// grid as for dedupe_hash: is the state's row the row of its group's smallest state?
__global__ __launch_bounds__(kWave) void dedupe_verify(const int64_t *__restrict__ row_ptr,
                                                       const int32_t *__restrict__ token_ids,
                                                       const int32_t *__restrict__ next_states, const DedupeBuffers d)
{
    const int32_t q = blockIdx.x / kRowSlices, slice = blockIdx.x % kRowSlices;
    const uint32_t r = d.rep[d.slot_of[q]];
    if (slice == 0 && threadIdx.x == 0)
        d.canon[q] = r;
    if (r == (uint32_t)q)
        return;
    const int64_t lo = row_ptr[q], n = row_ptr[q + 1] - lo;
    const int64_t lo_r = row_ptr[r], n_r = row_ptr[r + 1] - lo_r;
    bool differ = n != n_r;
    if (!differ) {
        int64_t i0, i1;
        row_slice(n, slice, i0, i1);
        for (int64_t i = i0 + threadIdx.x; i < i1; i += kWave)
            differ = differ || token_ids[lo + i] != token_ids[lo_r + i] || next_states[lo + i] != next_states[lo_r + i];
    }
    if (__ballot(differ) != 0 && threadIdx.x == 0)
        d.result[2] = 1;
}

// one workgroup: the distinct rows numbered in order of their smallest state, their row_ptr
__global__ __launch_bounds__(1024) void dedupe_number(const int64_t *__restrict__ row_ptr, int32_t n_states,
                                                      const DedupeBuffers d, int32_t *__restrict__ row_of_state,
                                                      int64_t *__restrict__ unique_row_ptr)
{
    __shared__ uint32_t wave_cnt[16];
    __shared__ int64_t wave_len[16];
    __shared__ uint32_t carry_cnt;
    __shared__ int64_t carry_len;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    if (threadIdx.x == 0) {
        carry_cnt = 0;
        carry_len = 0;
    }
    __syncthreads();
    for (int32_t q0 = 0; q0 < n_states; q0 += 1024) {
        const int32_t q = q0 + (int32_t)threadIdx.x;
        const bool is_rep = q < n_states && d.canon[q] == (uint32_t)q;
        const int64_t len = is_rep ? row_ptr[q + 1] - row_ptr[q] : 0;
        const uint64_t m = __ballot(is_rep);
        int64_t incl = len;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
            const int64_t up = __shfl_up(incl, o, kWave);
            if (lane >= o)
                incl += up;
        }
        if (lane == kWave - 1) {
            wave_cnt[wave] = (uint32_t)__popcll(m);
            wave_len[wave] = incl;
        }
        __syncthreads();
        uint32_t cnt_before = carry_cnt;
        int64_t len_before = carry_len;
        for (int w = 0; w < wave; ++w) {
            cnt_before += wave_cnt[w];
            len_before += wave_len[w];
        }
        if (is_rep) {
            const uint32_t u = cnt_before + __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32),
                                                                      __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
            d.slot_of[q] = u;                                        // from here on: the row's number
            d.rep_state[u] = (uint32_t)q;
            unique_row_ptr[u] = len_before + incl - len;
        }
        __syncthreads();
        if (threadIdx.x == 1023) {
            carry_cnt = cnt_before + (uint32_t)__popcll(m);
            carry_len = len_before + incl;
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        unique_row_ptr[carry_cnt] = carry_len;
        d.result[0] = carry_cnt;
        d.result[1] = carry_len;
    }
    __threadfence();
    __syncthreads();
    for (int32_t q = threadIdx.x; q < n_states; q += 1024)
        row_of_state[q] = (int32_t)d.slot_of[d.canon[q]];
}

// grid: n_states * kRowSlices (an upper bound for the distinct rows): the distinct rows side by side
__global__ __launch_bounds__(kWave) void dedupe_copy(const int64_t *__restrict__ row_ptr,
                                                     const int32_t *__restrict__ token_ids,
                                                     const int32_t *__restrict__ next_states, const DedupeBuffers d,
                                                     const int64_t *__restrict__ unique_row_ptr,
                                                     int32_t *__restrict__ token_ids_out,
                                                     int32_t *__restrict__ next_states_out)
{
    const int32_t u = blockIdx.x / kRowSlices, slice = blockIdx.x % kRowSlices;
    if ((int64_t)u >= d.result[0])
        return;
    const uint32_t q = d.rep_state[u];
    const int64_t lo = row_ptr[q], n = row_ptr[q + 1] - lo, out = unique_row_ptr[u];
    int64_t i0, i1;
    row_slice(n, slice, i0, i1);
    for (int64_t i = i0 + threadIdx.x; i < i1; i += kWave) {
        token_ids_out[out + i] = token_ids[lo + i];
        next_states_out[out + i] = next_states[lo + i];
    }
}

static uint32_t table_slots(int32_t n_states)
{
    uint32_t t = 64;
    while (t < 2u * (uint32_t)n_states)
        t <<= 1;
    return t;
}

size_t dedupe_workspace_bytes(int32_t n_states)
{
    const size_t q = (size_t)n_states, t = table_slots(n_states);
    return 256 + q * 8 + t * 8 + t * 4 + q * 4 * 3 + 256;
}

static DedupeBuffers dedupe_buffers(char *ws, int32_t n_states)
{
    const size_t q = (size_t)n_states, t = table_slots(n_states);
    DedupeBuffers d;
    d.result = reinterpret_cast<int64_t *>(ws);
    char *p = ws + 256;
    d.hash = reinterpret_cast<uint64_t *>(p); p += q * 8;
    d.keys = reinterpret_cast<unsigned long long *>(p); p += t * 8;
    d.rep = reinterpret_cast<uint32_t *>(p); p += t * 4;
    d.slot_of = reinterpret_cast<uint32_t *>(p); p += q * 4;
    d.canon = reinterpret_cast<uint32_t *>(p); p += q * 4;
    d.rep_state = reinterpret_cast<uint32_t *>(p);
    d.table_mask = (uint32_t)t - 1;
    return d;
}

hipError_t launch_dedupe(const fsmidx_csr &csr, char *ws, uint64_t seed, int32_t *row_of_state,
                         int64_t *unique_row_ptr, hipStream_t stream)
{
    const int32_t n = csr.n_states;
    const DedupeBuffers d = dedupe_buffers(ws, n);
    const unsigned cover = (unsigned)(((size_t)d.table_mask + 1 + 255) / 256);      // table >= 2 * states >= 3
    hipLaunchKernelGGL(dedupe_init, dim3(cover), dim3(256), 0, stream, d, n);
    const dim3 per_slice((unsigned)n * kRowSlices);
    hipLaunchKernelGGL(dedupe_hash, per_slice, dim3(kWave), 0, stream, csr.row_ptr, csr.token_ids, csr.next_states, seed,
                       d);
    hipLaunchKernelGGL(dedupe_group, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, csr.row_ptr, n, d);
    hipLaunchKernelGGL(dedupe_verify, per_slice, dim3(kWave), 0, stream, csr.row_ptr, csr.token_ids, csr.next_states, d);
    hipLaunchKernelGGL(dedupe_number, dim3(1), dim3(1024), 0, stream, csr.row_ptr, n, d, row_of_state, unique_row_ptr);
    return hipGetLastError();
}

hipError_t launch_dedupe_copy(const fsmidx_csr &csr, char *ws, const int64_t *unique_row_ptr, int32_t *token_ids_out,
                              int32_t *next_states_out, hipStream_t stream)
{
    const DedupeBuffers d = dedupe_buffers(ws, csr.n_states);
    hipLaunchKernelGGL(dedupe_copy, dim3((unsigned)csr.n_states * kRowSlices), dim3(kWave), 0, stream, csr.row_ptr,
                       csr.token_ids, csr.next_states, d, unique_row_ptr, token_ids_out, next_states_out);
    return hipGetLastError();
}

}  // namespace fsmidx
