// The two per-step neighbours of the mask in Algorithm 2 (Section 2.2), both working on the rows
// of the index instead of on the vocabulary:
//
//  advance_states   Section 3: the end state of every admissible (state, token) walk is stored
//      beside the token, so the state after a sampled token is one lookup in the state's row (a
//      binary search; token ids ascend).  One lane per sequence.
//
//  masked_argmax    greedy decoding (Section 2.1) on the masked logits of Section 2.2.  Outside the
//      row everything is -inf, so the choice is the largest logit among the row's entries: the
//      kernel reads the row's token ids and gathers those logits only.  Rows differ in length by
//      four orders of magnitude, so every row is cut into kArgmaxSplits slices, one wave
//      each; a slice's best entry is one 64-bit word (order-preserving image of the logit in the
//      high half, complement of the entry's position in the low half, so the maximum of the words is
//      the largest logit and, among equals, the lowest token id), and a second small kernel takes
//      the maximum over the slices and looks up token and end state.  No atomics, deterministic.
//
//  masked_sample    the sampling step of Algorithm 2: one draw per sequence from the softmax over the
//      row's entries, by inversion with a uniform number the caller supplies.  One pass over the
//      row gives every slice's maximum and the sum of its weights relative to that maximum (a
//      running maximum, the sum rescaled when it rises); a second kernel, one wave per sequence,
//      brings the slice sums to the row's maximum, finds the slice in which the cumulative weight
//      crosses u * total and walks that slice in order with w = exp(logit - max).  Weights are
//      binary32 exponentials, every sum is binary64.
#include "internal.h"

namespace fsmidx {

constexpr int kArgmaxThreads = kWave;   // a slice is one wave: most slices are empty and only have to find that out

__global__ __launch_bounds__(256) void advance_rows(const int64_t *__restrict__ row_ptr,
                                                    const int32_t *__restrict__ token_ids,
                                                    const int32_t *__restrict__ next_states, int32_t n_states,
                                                    const int32_t *states, const int32_t *__restrict__ tokens,
                                                    int32_t batch, int32_t *states_out)
{
    const int32_t b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= batch)
        return;
    const int32_t s = states[b];
    int32_t result = s;                                   // negative: no guidance, nothing to track
    if (s >= 0) {
        result = n_states;                                // names no row: the sequence has left the automaton
        if (s < n_states) {
            const int32_t t = tokens[b];
            int64_t lo = row_ptr[s], hi = row_ptr[s + 1];
            while (lo < hi) {                             // first entry with token id >= t
                const int64_t mid = lo + ((hi - lo) >> 1);
                if (token_ids[mid] < t)
                    lo = mid + 1;
                else
                    hi = mid;
            }
            if (lo < row_ptr[s + 1] && token_ids[lo] == t)
                result = next_states[lo];
        }
    }
    states_out[b] = result;
}

// Order-preserving image of a binary32 bit pattern in the unsigned integers, with NaN taken as
// -inf and -0.0 as +0.0.  Never 0, so that 0 can stand for "no entry".
__device__ __forceinline__ uint32_t logit_key(uint32_t u)
{
    if ((u & 0x7FFFFFFFu) > 0x7F800000u)
        u = 0xFF800000u;
    if (u == 0x80000000u)
        u = 0u;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

template <typename T>
__device__ __forceinline__ uint32_t logit_bits(const T *p);
template <>
__device__ __forceinline__ uint32_t logit_bits<uint32_t>(const uint32_t *p) { return *p; }
template <>
__device__ __forceinline__ uint32_t logit_bits<uint16_t>(const uint16_t *p) { return (uint32_t)*p << 16; }

__device__ __forceinline__ uint64_t wave_max_u64(uint64_t v)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const uint64_t o = __shfl_xor(v, d, kWave);
        v = o > v ? o : v;
    }
    return v;
}

// Entries [i0, i1) of a row of n entries that belong to `slice`: whole multiples of a wave.
__device__ __forceinline__ void slice_range(int64_t n, int32_t slice, int64_t &i0, int64_t &i1)
{
    int64_t per = (n + kArgmaxSplits - 1) / kArgmaxSplits;
    per = (per + kWave - 1) / kWave * kWave;
    i0 = min(n, (int64_t)slice * per);
    i1 = min(n, i0 + per);
}

// The candidates of sequence b: the row of its state (lo = first entry, n = entries), or the whole
// vocabulary (whole = true) for a negative state; n = 0 for a state that names no row.
__device__ __forceinline__ void row_of(const int64_t *__restrict__ row_ptr, int32_t n_states, int32_t n_tokens,
                                       int32_t s, int64_t &lo, int64_t &n, bool &whole)
{
    lo = 0;
    n = 0;
    whole = s < 0;
    if (whole) {
        n = n_tokens;
    } else if (s < n_states) {
        lo = row_ptr[s];
        n = row_ptr[s + 1] - lo;
    }
}

// grid: batch * kArgmaxSplits workgroups, the slices of a sequence side by side; T = storage type of
// a logit (uint32_t: binary32, uint16_t: bfloat16)
template <typename T>
__global__ __launch_bounds__(kArgmaxThreads) void argmax_slices(const int64_t *__restrict__ row_ptr,
                                                                const int32_t *__restrict__ token_ids,
                                                                int32_t n_states, int32_t n_tokens,
                                                                const int32_t *__restrict__ states,
                                                                const T *__restrict__ logits, int64_t row_stride,
                                                                uint64_t *__restrict__ partial)
{
    const int32_t b = blockIdx.x / kArgmaxSplits;
    const int32_t slice = blockIdx.x % kArgmaxSplits;
    const int32_t s = states[b];
    int64_t lo, n;
    bool whole;                                           // no guidance: every token is a candidate
    row_of(row_ptr, n_states, n_tokens, s, lo, n, whole);
    int64_t i0, i1;
    slice_range(n, slice, i0, i1);
    const T *row = logits + (int64_t)b * row_stride;
    uint64_t best = 0;
    // kUnroll entries per lane and round: all token ids first, then all logits, so a slice of a
    // long row is two memory round trips
    constexpr int kUnroll = 16;
    for (int64_t i = i0 + threadIdx.x; i < i1; i += kUnroll * kArgmaxThreads) {
        uint32_t t[kUnroll], u[kUnroll];
#pragma unroll
        for (int k = 0; k < kUnroll; ++k) {
            const int64_t at = i + k * kArgmaxThreads;
            t[k] = 0xFFFFFFFFu;                                  // past the slice: reads nothing, never wins
            if (at < i1)
                t[k] = whole ? (uint32_t)at : (uint32_t)token_ids[lo + at];
        }
#pragma unroll
        for (int k = 0; k < kUnroll; ++k)
            u[k] = t[k] < (uint32_t)n_tokens ? logit_bits<T>(row + t[k]) : 0xFF800000u;
#pragma unroll
        for (int k = 0; k < kUnroll; ++k) {
            const int64_t at = i + k * kArgmaxThreads;
            const uint64_t w = ((uint64_t)logit_key(u[k]) << 32) | (0xFFFFFFFFu - (uint32_t)at);
            if (at < i1)
                best = w > best ? w : best;
        }
    }
    best = wave_max_u64(best);
    if (threadIdx.x == 0)
        partial[(int64_t)b * kArgmaxSplits + slice] = best;
}

// one wave per sequence
__global__ __launch_bounds__(kWave) void argmax_pick(const int64_t *__restrict__ row_ptr,
                                                     const int32_t *__restrict__ token_ids,
                                                     const int32_t *__restrict__ next_states, int32_t n_states,
                                                     const int32_t *states, const uint64_t *__restrict__ partial,
                                                     int32_t *__restrict__ tokens_out, int32_t *states_out)
{
    static_assert(kArgmaxSplits <= kWave, "one lane per slice");
    const int32_t b = blockIdx.x;
    const int lane = threadIdx.x;
    uint64_t best = lane < kArgmaxSplits ? partial[(int64_t)b * kArgmaxSplits + lane] : 0;
    best = wave_max_u64(best);
    if (lane != 0)
        return;
    const int32_t s = states[b];
    int32_t token = -1, state = n_states;
    if (best != 0) {
        const uint32_t i = 0xFFFFFFFFu - (uint32_t)best;
        if (s < 0) {
            token = (int32_t)i;
            state = s;
        } else {
            const int64_t at = row_ptr[s] + i;
            token = token_ids[at];
            state = next_states[at];
        }
    }
    tokens_out[b] = token;
    states_out[b] = state;
}

// ---- sampling

constexpr int kSampleRun = 32;        // consecutive entries of a slice that one lane adds up

__device__ __forceinline__ double wave_sum_f64(double v)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1)
        v += __shfl_xor(v, d, kWave);
    return v;
}

// The largest logit of a sequence from its slice words (0 = the sequence has no candidates), as a
// binary32 value: the inverse of logit_key.
__device__ __forceinline__ uint64_t row_best(const uint64_t *__restrict__ partial, int32_t b, int lane)
{
    return wave_max_u64(lane < kArgmaxSplits ? partial[(int64_t)b * kArgmaxSplits + lane] : 0);
}

__device__ __forceinline__ float key_value(uint32_t key)
{
    return __uint_as_float((key & 0x80000000u) ? (key & 0x7FFFFFFFu) : ~key);
}

// Weight of a logit (bit pattern u) under the maximum `top`: 1 for the maximum itself whatever it is,
// exp(x - top) otherwise (0 for -inf and for NaN, which counts as -inf).
__device__ __forceinline__ double logit_weight(uint32_t u, float top)
{
    if ((u & 0x7FFFFFFFu) > 0x7F800000u)
        return 0.0;
    const float x = __uint_as_float(u);
    if (x == top)
        return 1.0;
    return (double)expf(x - top);
}

// grid as for argmax_slices: the largest logit of every slice and the sum of the slice's weights
// relative to it, in ONE pass over the slice's entries: a lane keeps a running maximum and
// rescales its sum whenever the maximum rises, and the lanes' pairs are merged the same way.
// partial = the maximum's key << 32 (0: the slice has no entries), sums = sum of exp(logit - slice
// maximum) (1 for a logit equal to it).
template <typename T>
__global__ __launch_bounds__(kWave) void sample_slices(const int64_t *__restrict__ row_ptr,
                                                       const int32_t *__restrict__ token_ids, int32_t n_states,
                                                       int32_t n_tokens, const int32_t *__restrict__ states,
                                                       const T *__restrict__ logits, int64_t row_stride,
                                                       uint64_t *__restrict__ partial, double *__restrict__ sums)
{
    const int lane = threadIdx.x;
    const int32_t b = blockIdx.x / kArgmaxSplits;
    const int32_t slice = blockIdx.x % kArgmaxSplits;
    int64_t lo, n, i0, i1;
    bool whole;
    row_of(row_ptr, n_states, n_tokens, states[b], lo, n, whole);
    slice_range(n, slice, i0, i1);
    const T *row = logits + (int64_t)b * row_stride;
    float top = -INFINITY;                                 // of this lane's entries so far
    double sum = 0.0;                                      // of their weights relative to `top`
    constexpr int kUnroll = 8;
    for (int64_t i = i0 + lane; i < i1; i += kUnroll * kWave) {
        uint32_t t[kUnroll], u[kUnroll];
#pragma unroll
        for (int k = 0; k < kUnroll; ++k) {
            const int64_t at = i + k * kWave;
            t[k] = 0xFFFFFFFFu;
            if (at < i1)
                t[k] = whole ? (uint32_t)at : (uint32_t)token_ids[lo + at];
        }
#pragma unroll
        for (int k = 0; k < kUnroll; ++k)
            u[k] = t[k] < (uint32_t)n_tokens ? logit_bits<T>(row + t[k]) : 0xFF800000u;
#pragma unroll
        for (int k = 0; k < kUnroll; ++k) {
            if ((u[k] & 0x7FFFFFFFu) > 0x7F800000u || u[k] == 0xFF800000u)
                continue;                                  // NaN counts as -inf, and -inf weighs nothing
            const float x = __uint_as_float(u[k]);
            if (x > top) {
                sum = (top == -INFINITY ? 0.0 : sum * (double)expf(top - x)) + 1.0;
                top = x;
            } else {
                sum += x == top ? 1.0 : (double)expf(x - top);
            }
        }
    }
    // merge the lanes: the slice's maximum, every lane's sum rescaled to it
    float all = top;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1)
        all = fmaxf(all, __shfl_xor(all, d, kWave));
    if (top != all)
        sum = top == -INFINITY ? 0.0 : sum * (double)expf(top - all);
    sum = wave_sum_f64(sum);
    if (lane == 0) {
        const bool any = i1 > i0;
        // (a slice of nothing but -inf and NaN reports -inf as its maximum, with weight 0)
        partial[(int64_t)b * kArgmaxSplits + slice] = any ? (uint64_t)logit_key(__float_as_uint(all)) << 32 | 1u : 0ull;
        sums[(int64_t)b * kArgmaxSplits + slice] = sum;
    }
}

// one wave per sequence: the slice in which the cumulative weight crosses the threshold, then the
// entry inside that slice
template <typename T>
__global__ __launch_bounds__(kWave) void sample_pick(const int64_t *__restrict__ row_ptr,
                                                     const int32_t *__restrict__ token_ids,
                                                     const int32_t *__restrict__ next_states, int32_t n_states,
                                                     int32_t n_tokens, const int32_t *states,
                                                     const T *__restrict__ logits, int64_t row_stride,
                                                     const float *__restrict__ uniforms,
                                                     const uint64_t *__restrict__ partial,
                                                     const double *__restrict__ sums,
                                                     int32_t *__restrict__ tokens_out, int32_t *states_out)
{
    static_assert(kArgmaxSplits == kWave, "one lane per slice");
    const int lane = threadIdx.x;
    const int32_t b = blockIdx.x;
    const int32_t s = states[b];
    const uint64_t best = row_best(partial, b, lane);
    if (best == 0) {                                       // no candidates (uniform over the wave)
        if (lane == 0) {
            tokens_out[b] = -1;
            states_out[b] = n_states;
        }
        return;
    }
    int64_t lo, n;
    bool whole;
    row_of(row_ptr, n_states, n_tokens, s, lo, n, whole);
    const float top = key_value((uint32_t)(best >> 32));
    // inclusive prefix sums of the slice sums, each brought from its slice's maximum to the row's
    const uint64_t own_word = partial[(int64_t)b * kArgmaxSplits + lane];
    const float own_top = key_value((uint32_t)(own_word >> 32));
    double mine = own_word != 0 ? sums[(int64_t)b * kArgmaxSplits + lane] : 0.0;
    if (mine != 0.0 && own_top != top)
        mine *= (double)expf(own_top - top);
    double incl = mine;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const double up = __shfl_up(incl, d, kWave);
        if (lane >= d)
            incl += up;
    }
    const double total = __shfl(incl, kWave - 1, kWave);
    int64_t position = 0;                                  // nothing but -inf: the first entry
    if (total > 0.0) {
        float u = uniforms[b];
        u = u >= 0.0f ? fminf(u, 0x1.fffffep-1f) : 0.0f;   // clamped into [0, 1 - 2^-24]; NaN -> 0
        const double threshold = (double)u * total;
        uint64_t over = __ballot(incl > threshold);
        if (over == 0)                                     // cannot happen (threshold < total); stay in bounds anyway:
            over = 1ull << (63 - __builtin_clzll(__ballot(mine > 0.0)));   // the last slice with a weight (total > 0)
        const int slice = __builtin_ctzll(over);
        double carry = __shfl(incl - mine, slice, kWave);
        int64_t i0, i1;
        slice_range(n, slice, i0, i1);
        const T *row = logits + (int64_t)b * row_stride;
        // The slice, kSampleRun consecutive entries per lane and 64 lanes at a time: all loads of a
        // round are independent; a scan over the lanes' sums finds the lane in which the threshold
        // is crossed, and that lane's own entries are then added up one by one.  The sums were
        // added in another order by sample_sums (and by the scan), so a walk may end a rounding
        // error short of the threshold: then the last entry with a weight is the one.
        int64_t last_weighted = i0;
        bool found = false;
        for (int64_t r0 = i0; r0 < i1 && !found; r0 += (int64_t)kSampleRun * kWave) {
            const int64_t first = r0 + (int64_t)lane * kSampleRun;
            uint32_t t[kSampleRun];
            float w[kSampleRun];
#pragma unroll
            for (int k = 0; k < kSampleRun; ++k) {
                t[k] = 0xFFFFFFFFu;
                if (first + k < i1)
                    t[k] = whole ? (uint32_t)(first + k) : (uint32_t)token_ids[lo + first + k];
            }
#pragma unroll
            for (int k = 0; k < kSampleRun; ++k)
                w[k] = (float)logit_weight(t[k] < (uint32_t)n_tokens ? logit_bits<T>(row + t[k]) : 0xFF800000u, top);
            double own = 0.0;
            int last_k = -1;
#pragma unroll
            for (int k = 0; k < kSampleRun; ++k) {
                own += (double)w[k];
                if (w[k] > 0.0f)
                    last_k = k;
            }
            double run = own;
#pragma unroll
            for (int d = 1; d < kWave; d <<= 1) {
                const double up = __shfl_up(run, d, kWave);
                if (lane >= d)
                    run += up;
            }
            const uint64_t weighted = __ballot(last_k >= 0);
            if (weighted != 0) {
                const int top_lane = 63 - __builtin_clzll(weighted);
                last_weighted = r0 + (int64_t)top_lane * kSampleRun + __shfl(last_k, top_lane, kWave);
            }
            const uint64_t crossed = __ballot(own > 0.0 && carry + run > threshold);
            if (crossed != 0) {
                const int at_lane = __builtin_ctzll(crossed);
                double c = carry + (run - own);
                int hit = last_k;                                  // short of the threshold by rounding
                bool done = false;
#pragma unroll
                for (int k = 0; k < kSampleRun; ++k) {
                    c += (double)w[k];
                    if (!done && w[k] > 0.0f && c > threshold) {
                        hit = k;
                        done = true;
                    }
                }
                position = r0 + (int64_t)at_lane * kSampleRun + __shfl(hit, at_lane, kWave);
                found = true;
            }
            carry += __shfl(run, kWave - 1, kWave);
        }
        if (!found)
            position = last_weighted;
    }
    if (lane == 0) {
        if (whole) {
            tokens_out[b] = (int32_t)position;
            states_out[b] = s;
        } else {
            tokens_out[b] = token_ids[lo + position];
            states_out[b] = next_states[lo + position];
        }
    }
}

hipError_t launch_advance(const fsmidx_csr &csr, const int32_t *states, const int32_t *tokens, int32_t batch,
                          int32_t *states_out, hipStream_t stream)
{
    hipLaunchKernelGGL(advance_rows, dim3((batch + 255) / 256), dim3(256), 0, stream, csr.row_ptr, csr.token_ids,
                       csr.next_states, csr.n_states, states, tokens, batch, states_out);
    return hipGetLastError();
}

hipError_t launch_argmax(const fsmidx_csr &csr, const int32_t *states, int32_t batch, const void *logits,
                         int64_t row_stride, int32_t dtype, uint64_t *partial, int32_t *tokens_out,
                         int32_t *states_out, hipStream_t stream)
{
    const dim3 grid((unsigned)batch * kArgmaxSplits);
    if (dtype == 0)
        hipLaunchKernelGGL(argmax_slices<uint32_t>, grid, dim3(kArgmaxThreads), 0, stream, csr.row_ptr, csr.token_ids,
                           csr.n_states, csr.n_tokens, states, static_cast<const uint32_t *>(logits), row_stride,
                           partial);
    else
        hipLaunchKernelGGL(argmax_slices<uint16_t>, grid, dim3(kArgmaxThreads), 0, stream, csr.row_ptr, csr.token_ids,
                           csr.n_states, csr.n_tokens, states, static_cast<const uint16_t *>(logits), row_stride,
                           partial);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return e;
    hipLaunchKernelGGL(argmax_pick, dim3(batch), dim3(kWave), 0, stream, csr.row_ptr, csr.token_ids, csr.next_states,
                       csr.n_states, states, partial, tokens_out, states_out);
    return hipGetLastError();
}

hipError_t launch_sample(const fsmidx_csr &csr, const int32_t *states, int32_t batch, const void *logits,
                         int64_t row_stride, int32_t dtype, const float *uniforms, uint64_t *partial, double *sums,
                         int32_t *tokens_out, int32_t *states_out, hipStream_t stream)
{
    const dim3 grid((unsigned)batch * kArgmaxSplits);
    if (dtype == 0) {
        const uint32_t *x = static_cast<const uint32_t *>(logits);
        hipLaunchKernelGGL(sample_slices<uint32_t>, grid, dim3(kWave), 0, stream, csr.row_ptr, csr.token_ids,
                           csr.n_states, csr.n_tokens, states, x, row_stride, partial, sums);
        hipLaunchKernelGGL(sample_pick<uint32_t>, dim3(batch), dim3(kWave), 0, stream, csr.row_ptr, csr.token_ids,
                           csr.next_states, csr.n_states, csr.n_tokens, states, x, row_stride, uniforms, partial, sums,
                           tokens_out, states_out);
    } else {
        const uint16_t *x = static_cast<const uint16_t *>(logits);
        hipLaunchKernelGGL(sample_slices<uint16_t>, grid, dim3(kWave), 0, stream, csr.row_ptr, csr.token_ids,
                           csr.n_states, csr.n_tokens, states, x, row_stride, partial, sums);
        hipLaunchKernelGGL(sample_pick<uint16_t>, dim3(batch), dim3(kWave), 0, stream, csr.row_ptr, csr.token_ids,
                           csr.next_states, csr.n_states, csr.n_tokens, states, x, row_stride, uniforms, partial, sums,
                           tokens_out, states_out);
    }
    return hipGetLastError();
}

}  // namespace fsmidx
