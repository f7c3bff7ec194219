// The reachable-only index (Section 3, the paragraph after Algorithm 4: not every state of the
// automaton is ever represented by a vocabulary string; Section 2.2, Algorithm 2: a generation
// starts in q_0 and moves to the end state stored with the sampled token).  The states a
// generation can be in are those reachable from q_0 through rows of the index, and only their
// rows are ever read.
//
// Building rows is cheap here, so nothing is built lazily: the whole index is built as usual, and
// these kernels find the reachable states in it and write the index without the other rows.
//
//  reach_clear, reach_seed   marks cleared, the start states marked and put on the first frontier
//  reach_level               one level of a breadth-first search: the rows of the frontier's states
//                            are read (kReachSlices waves share a row), every end state not yet
//                            marked is marked with an atomic exchange, and the wave that wins the
//                            exchange puts it on the next frontier (one counter update per wave
//                            and step: atomics on one address are served one after the other).
//                            The launch is a fixed grid that strides over (state, slice) items and
//                            reads the frontier's length from memory, so the host can enqueue
//                            several levels without waiting for any of them.
//  reach_finish              marks as bytes
//  restrict_scan, restrict_copy   row_ptr of the kept rows (one workgroup), and the rows themselves
#include "internal.h"

namespace fsmidx {

constexpr int kReachSlices = 64;       // waves that share one row
constexpr int kReachRecent = 64;       // end states a wave remembers having seen marked
constexpr int kCopySlices = 16;        // waves that share one row when the kept rows are copied
static_assert(kReachRecent == kWave, "every lane clears one entry of the table");
static_assert((int64_t)kDedupeMaxStates * kCopySlices <= 0x7FFFFFFFll, "one workgroup per (state, slice) must fit a grid");
constexpr int kReachGrid = 4096;       // most waves of one level's launch

struct ReachBuffers {
    int64_t *result;       // [0] states reached so far, [1] entries of the restricted index
    uint32_t *count;       // [3] frontier lengths: level l reads [l % 3], fills [(l + 1) % 3], clears [(l + 2) % 3]
    uint32_t *flag;        // [n_states] 1: reached
    uint32_t *front[2];    // [n_states] each: the frontier of even / odd levels
};

static ReachBuffers reach_buffers(char *ws, int32_t n_states)
{
    const size_t q = ((size_t)n_states * 4 + 255) / 256 * 256;
    ReachBuffers b;
    b.result = reinterpret_cast<int64_t *>(ws);
    b.count = reinterpret_cast<uint32_t *>(ws + 64);
    b.flag = reinterpret_cast<uint32_t *>(ws + 256);
    b.front[0] = reinterpret_cast<uint32_t *>(ws + 256 + q);
    b.front[1] = reinterpret_cast<uint32_t *>(ws + 256 + 2 * q);
    return b;
}

size_t reach_workspace_bytes(int32_t n_states)
{
    return 256 + 3 * (((size_t)n_states * 4 + 255) / 256 * 256);
}

__global__ __launch_bounds__(256) void reach_clear(const ReachBuffers b, int32_t n_states)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_states)
        b.flag[i] = 0;
    if (i == 0) {
        b.result[0] = 0;
        b.result[1] = 0;
        b.count[0] = 0;
        b.count[1] = 0;
        b.count[2] = 0;
    }
}

// one workgroup; the start states (already range checked by the host) lie in front[1]
__global__ __launch_bounds__(256) void reach_seed(const ReachBuffers b, int32_t n_starts)
{
    for (int32_t i = threadIdx.x; i < n_starts; i += blockDim.x) {
        const uint32_t s = b.front[1][i];
        if (atomicExch(&b.flag[s], 1u) == 0u)
            b.front[0][atomicAdd(&b.count[0], 1u)] = s;
    }
}

// entries [i0, i1) of a row of n entries that belong to `slice`: whole multiples of a wave
__device__ __forceinline__ void reach_slice(int64_t n, int32_t slice, int32_t n_slices, int64_t &i0, int64_t &i1)
{
    int64_t per = (n + n_slices - 1) / n_slices;
    per = (per + kWave - 1) / kWave * kWave;
    i0 = min(n, (int64_t)slice * per);
    i1 = min(n, i0 + per);
}

__global__ __launch_bounds__(kWave) void reach_level(const int64_t *__restrict__ row_ptr,
                                                     const int32_t *__restrict__ next_states, int32_t n_states,
                                                     int64_t nnz, const ReachBuffers b, uint32_t level)
{
    const uint32_t n_in = b.count[level % 3u];
    uint32_t *const n_out = &b.count[(level + 1u) % 3u];
    const uint32_t *const in = b.front[level & 1u];
    uint32_t *const out = b.front[(level + 1u) & 1u];
    const int lane = threadIdx.x;
    // Rows repeat their end states (a row of 80,000 entries may name five states), and a mark set
    // by a wave on another die may not be visible to a plain read for the rest of the launch: every
    // one of those entries would then go to the atomic unit, which serves one address at a time.
    // So a wave remembers the states it has seen marked (a direct-mapped table; a lost entry only
    // costs another look).
    __shared__ uint32_t recent[kReachRecent];
    recent[lane] = ~0u;
    __builtin_amdgcn_wave_barrier();
    if (blockIdx.x == 0 && lane == 0) {
        b.count[(level + 2u) % 3u] = 0;                              // the level after this one fills it
        b.result[0] += (int64_t)n_in;                                // (one writer per launch)
    }
    const uint64_t n_items = (uint64_t)n_in * kReachSlices;
    for (uint64_t item = blockIdx.x; item < n_items; item += gridDim.x) {
        const uint32_t q = in[item / kReachSlices];
        const int32_t slice = (int32_t)(item % kReachSlices);
        // (the index is the caller's memory: nothing read from it is used as an address unchecked)
        const int64_t lo = max((int64_t)0, min(row_ptr[q], nnz));
        const int64_t hi = max(lo, min(row_ptr[q + 1], nnz));
        int64_t i0, i1;
        reach_slice(hi - lo, slice, kReachSlices, i0, i1);
        for (int64_t base = i0; base < i1; base += kWave) {
            const int64_t i = base + lane;
            bool won = false;
            uint32_t s = 0;
            if (i < i1) {
                s = (uint32_t)next_states[lo + i];
                // (the plain read may be stale, another wave may be marking s right now: the exchange decides)
                if (s < (uint32_t)n_states && recent[s % (uint32_t)kReachRecent] != s) {
                    if (b.flag[s] == 0u)
                        won = atomicExch(&b.flag[s], 1u) == 0u;
                    recent[s % (uint32_t)kReachRecent] = s;
                }
            }
            const uint64_t m = __ballot(won);
            if (m != 0) {
                uint32_t at = 0;
                if (lane == 0)
                    at = atomicAdd(n_out, (uint32_t)__popcll(m));
                at = (uint32_t)__shfl((int)at, 0, kWave);
                if (won)
                    out[at + __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u))] = s;
            }
        }
    }
}

__global__ __launch_bounds__(256) void reach_finish(const ReachBuffers b, int32_t n_states, uint8_t *__restrict__ reach_out)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_states)
        reach_out[i] = b.flag[i] != 0u ? 1 : 0;
}

hipError_t launch_reach_start(const fsmidx_csr &csr, char *ws, const int32_t *starts_host, int32_t n_starts,
                              hipStream_t stream)
{
    const ReachBuffers b = reach_buffers(ws, csr.n_states);
    hipLaunchKernelGGL(reach_clear, dim3((unsigned)((csr.n_states + 255) / 256)), dim3(256), 0, stream, b, csr.n_states);
    if (n_starts > 0) {
        hipError_t e = hipMemcpyAsync(b.front[1], starts_host, (size_t)n_starts * 4, hipMemcpyHostToDevice, stream);
        if (e != hipSuccess)
            return e;
        hipLaunchKernelGGL(reach_seed, dim3(1), dim3(256), 0, stream, b, n_starts);
    }
    return hipGetLastError();
}

// `expected`: the length of the last frontier the host has seen (the grid is sized for a few times
// that; any grid gives the same result, a frontier that has grown is only taken in more rounds)
hipError_t launch_reach_levels(const fsmidx_csr &csr, char *ws, uint32_t first_level, int n_levels, uint32_t expected,
                               hipStream_t stream)
{
    const ReachBuffers b = reach_buffers(ws, csr.n_states);
    uint64_t waves = (uint64_t)(expected < 4u ? 4u : expected) * kReachSlices * 4u;
    if (waves > (uint64_t)kReachGrid)
        waves = kReachGrid;
    for (int l = 0; l < n_levels; ++l)
        hipLaunchKernelGGL(reach_level, dim3((unsigned)waves), dim3(kWave), 0, stream, csr.row_ptr, csr.next_states,
                           csr.n_states, csr.nnz, b, first_level + (uint32_t)l);
    return hipGetLastError();
}

// where the host reads, after `level` levels, the length of the frontier the next level would take
const uint32_t *reach_next_count(char *ws, int32_t n_states, uint32_t level)
{
    return &reach_buffers(ws, n_states).count[level % 3u];
}

hipError_t launch_reach_finish(const fsmidx_csr &csr, char *ws, uint8_t *reach_out, hipStream_t stream)
{
    const ReachBuffers b = reach_buffers(ws, csr.n_states);
    hipLaunchKernelGGL(reach_finish, dim3((unsigned)((csr.n_states + 255) / 256)), dim3(256), 0, stream, b, csr.n_states,
                       reach_out);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------- restricted index

// one workgroup: row_ptr of the index whose rows outside `keep` are empty
__global__ __launch_bounds__(1024) void restrict_scan(const int64_t *__restrict__ row_ptr, const uint8_t *__restrict__ keep,
                                                      int32_t n_states, int64_t nnz, int64_t *__restrict__ row_ptr_out,
                                                      int64_t *__restrict__ result)
{
    __shared__ int64_t wave_sum[16];
    __shared__ int64_t carry_s;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    if (threadIdx.x == 0)
        carry_s = 0;
    __syncthreads();
    for (int32_t q0 = 0; q0 < n_states; q0 += 1024) {
        const int32_t q = q0 + (int32_t)threadIdx.x;
        int64_t len = 0;
        if (q < n_states && keep[q] != 0) {
            const int64_t lo = max((int64_t)0, min(row_ptr[q], nnz));
            len = max(lo, min(row_ptr[q + 1], nnz)) - lo;
        }
        int64_t incl = len;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
            const int64_t up = __shfl_up(incl, o, kWave);
            if (lane >= o)
                incl += up;
        }
        if (lane == kWave - 1)
            wave_sum[wave] = incl;
        __syncthreads();
        int64_t before = carry_s;
        for (int w = 0; w < wave; ++w)
            before += wave_sum[w];
        if (q < n_states)
            row_ptr_out[q] = before + incl - len;
        __syncthreads();
        if (threadIdx.x == 1023)
            carry_s = before + incl;
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        row_ptr_out[n_states] = carry_s;
        result[1] = carry_s;
    }
}

// grid: n_states * kCopySlices
__global__ __launch_bounds__(kWave) void restrict_copy(const int64_t *__restrict__ row_ptr,
                                                       const int32_t *__restrict__ token_ids,
                                                       const int32_t *__restrict__ next_states,
                                                       const uint8_t *__restrict__ keep, int64_t nnz,
                                                       const int64_t *__restrict__ row_ptr_out, int64_t capacity,
                                                       int32_t *__restrict__ token_ids_out,
                                                       int32_t *__restrict__ next_states_out)
{
    const int32_t q = blockIdx.x / kCopySlices, slice = blockIdx.x % kCopySlices;
    if (keep[q] == 0)
        return;
    const int64_t lo = max((int64_t)0, min(row_ptr[q], nnz));
    const int64_t n = max(lo, min(row_ptr[q + 1], nnz)) - lo;
    const int64_t out = row_ptr_out[q];
    if (out < 0 || out > capacity - n)
        return;                                                    // (row_ptr_out is the caller's memory too)
    int64_t i0, i1;
    reach_slice(n, slice, kCopySlices, i0, i1);
    for (int64_t i = i0 + threadIdx.x; i < i1; i += kWave) {
        token_ids_out[out + i] = token_ids[lo + i];
        next_states_out[out + i] = next_states[lo + i];
    }
}

hipError_t launch_restrict_scan(const fsmidx_csr &csr, const uint8_t *keep, char *ws, int64_t *row_ptr_out,
                                hipStream_t stream)
{
    hipLaunchKernelGGL(restrict_scan, dim3(1), dim3(1024), 0, stream, csr.row_ptr, keep, csr.n_states, csr.nnz,
                       row_ptr_out, reinterpret_cast<int64_t *>(ws));
    return hipGetLastError();
}

hipError_t launch_restrict_copy(const fsmidx_csr &csr, const uint8_t *keep, const int64_t *row_ptr_out,
                                int32_t *token_ids_out, int32_t *next_states_out, int64_t capacity, hipStream_t stream)
{
    hipLaunchKernelGGL(restrict_copy, dim3((unsigned)csr.n_states * kCopySlices), dim3(kWave), 0, stream, csr.row_ptr,
                       csr.token_ids, csr.next_states, keep, csr.nnz, row_ptr_out, capacity, token_ids_out,
                       next_states_out);
    return hipGetLastError();
}

}  // namespace fsmidx
