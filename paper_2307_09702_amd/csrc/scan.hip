// Prefix sums that turn the per-(state, token group) counts into CSR positions (the bookkeeping
// behind Algorithm 4's union of v into sigma(z_0), made order-preserving).
//
//  scan_groups : one wave per state; exclusive scan of that state's counts over the token groups,
//                written back in place, and the row total.
//  scan_rows   : one workgroup; exclusive scan of the row totals into row_ptr (int64) and nnz.
#include "internal.h"

namespace fsmidx {

template <typename T>
__device__ __forceinline__ T wave_inclusive_scan(T v, int lane)
{
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        T up = __shfl_up(v, d, kWave);
        if (lane >= d)
            v += up;
    }
    return v;
}

__global__ __launch_bounds__(256) void scan_groups(uint32_t *__restrict__ cnt, int32_t n_states,
                                                   int32_t n_groups_dense, int32_t n_groups_sets,
                                                   int64_t *__restrict__ rowtot, uint32_t *__restrict__ long_items,
                                                   Status *st)
{
    // the two walk variants count per 1024-token group and per 4096-token block respectively
    const bool sets = st->use_sets != 0;
    const int32_t n_groups = sets ? n_groups_sets : n_groups_dense;
    const int lane = threadIdx.x & (kWave - 1);
    const int32_t q = blockIdx.x * (blockDim.x / kWave) + (threadIdx.x >> 6);
    if (q >= n_states)
        return;
    uint32_t *row = cnt + (int64_t)q * n_groups;
    uint32_t carry = 0;
    for (int32_t j0 = 0; j0 < n_groups; j0 += kWave) {
        const int32_t j = j0 + lane;
        const uint32_t v = j < n_groups ? row[j] : 0u;
        const uint32_t incl = wave_inclusive_scan(v, lane);
        if (j < n_groups)
            row[j] = carry + incl - v;
        carry += __shfl(incl, kWave - 1, kWave);
        // token-set path: the emit pass handles (state, block) segments with many entries by
        // search; list them (one atomic per wave; the order of the list does not matter)
        const uint64_t is_long = __ballot(sets && v > (uint32_t)kLongRow);
        if (is_long != 0) {
            uint32_t at = 0;
            if (lane == 0)
                at = atomicAdd(&st->n_long, (uint32_t)__popcll(is_long));
            at = (uint32_t)__shfl((int)at, 0, kWave);
            if ((is_long >> lane) & 1ull)
                long_items[at + __builtin_amdgcn_mbcnt_hi((uint32_t)(is_long >> 32),
                                                          __builtin_amdgcn_mbcnt_lo((uint32_t)is_long, 0u))] =
                    (uint32_t)q << 12 | (uint32_t)j;
        }
    }
    if (lane == 0)
        rowtot[q] = (int64_t)carry;
}

// Also zeroes the work counters of the emit kernel that follows (token-set path: queue != NULL).
// A thread takes kScanRows consecutive rows, so that a round of the workgroup covers 8192 rows: a
// round costs three barriers and a trip to memory whatever it covers.
constexpr int kScanRows = 8;

__global__ __launch_bounds__(1024) void scan_rows(const int64_t *__restrict__ rowtot, int32_t n_states,
                                                  int64_t *__restrict__ row_ptr, uint32_t *__restrict__ queue,
                                                  Status *st)
{
    if (queue != nullptr && threadIdx.x < kQueues)
        queue[threadIdx.x] = 0;
    __shared__ int64_t wave_sum[16];
    __shared__ int64_t carry_s;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    if (threadIdx.x == 0)
        carry_s = 0;
    __syncthreads();
    for (int32_t q0 = 0; q0 < n_states; q0 += 1024 * kScanRows) {
        const int32_t q = q0 + (int32_t)threadIdx.x * kScanRows;
        int64_t v[kScanRows];
#pragma unroll
        for (int i = 0; i < kScanRows; ++i)
            v[i] = q + i < n_states ? rowtot[q + i] : 0;
        int64_t mine = 0;
#pragma unroll
        for (int i = 0; i < kScanRows; ++i)
            mine += v[i];
        const int64_t incl = wave_inclusive_scan(mine, lane);
        if (lane == kWave - 1)
            wave_sum[wave] = incl;
        __syncthreads();
        int64_t at = carry_s + incl - mine;
        for (int w = 0; w < wave; ++w)
            at += wave_sum[w];
#pragma unroll
        for (int i = 0; i < kScanRows; ++i) {
            if (q + i < n_states)
                row_ptr[q + i] = at;
            at += v[i];
        }
        __syncthreads();
        if (threadIdx.x == 1023)
            carry_s = at;
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        row_ptr[n_states] = carry_s;
        st->nnz = carry_s;
    }
}

hipError_t launch_scan(const Plan &p, char *ws, int64_t *row_ptr, hipStream_t stream)
{
    uint32_t *cnt = reinterpret_cast<uint32_t *>(ws + p.off_cnt);
    int64_t *rowtot = reinterpret_cast<int64_t *>(ws + p.off_rowtot);
    Status *st = reinterpret_cast<Status *>(ws + p.off_status);
    if (p.n_states > 0)
        hipLaunchKernelGGL(scan_groups, dim3((p.n_states + 3) / 4), dim3(256), 0, stream, cnt, p.n_states,
                           p.n_groups, p.n_blocks, rowtot, reinterpret_cast<uint32_t *>(ws + p.off_long), st);
    hipLaunchKernelGGL(scan_rows, dim3(1), dim3(1024), 0, stream, rowtot, p.n_states, row_ptr,
                       p.sets_possible ? reinterpret_cast<uint32_t *>(ws + p.off_queue) : nullptr, st);
    return hipGetLastError();
}

}  // namespace fsmidx
