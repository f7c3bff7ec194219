// Internal declarations shared by the translation units of libfsmidx (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "fsmidx.h"

namespace fsmidx {

constexpr int kWave = 64;              // gfx950 wavefront width

// Token geometry shared by all kernels: a chunk is 64 consecutive tokens (one 64-bit
// admissibility word per state), a block is 64 chunks (one word per lane of a wave).
constexpr int kChunkTokens = 64;
constexpr int kBlockChunks = 64;
constexpr int kBlockTokens = kChunkTokens * kBlockChunks;   // 4096

// Dense-table path (any automaton): one wave walks 16 chunks of tokens against a range of states.
constexpr int kChunksPerWave = 16;
constexpr int kGroupTokens = kWave * kChunksPerWave;        // 1024 tokens per count-matrix column
constexpr int kGroupsPerBlock = kBlockTokens / kGroupTokens;
constexpr int kWavesPerBlock = 4;
constexpr int kPackedClasses = 8;      // leading byte classes of a token packed into its record

// Token-set path (automata with <= 64 classes and few distinct targets per state).
constexpr int kMaxSetDepth = 32;       // longest token (bytes) the path handles
constexpr int kSetCap = 256;           // distinct class sets (one bitmap family each)
// most token blocks: the bitmaps U[kMaxSetDepth][kSetCap][64 per block] of 8-byte words stay below 4 GB
constexpr int kMaxSetBlocks = 2047;
constexpr int kSetHashSlots = 512;
constexpr int kStackFrames = 7;        // pending branch points a wave can hold (8 lanes of a register each)
constexpr int kShallowFrames = 4;      // ... in the counting walk's first attempt (less LDS, more waves per CU)
constexpr int kSetWaves = 1;           // waves per workgroup of the token-set kernels
constexpr int kQueues = 256;           // work counters the emit kernel's searching workgroups draw from
constexpr int kLongRow = 512;         // entries of one (state, block) above which the token-set path emits it by search

// Greedy choice under the mask: slices a row is cut into (one workgroup and one 64-bit partial
// result each).
constexpr int kArgmaxSplits = 64;
constexpr int kArgmaxMaxBatch = 1 << 24;   // batch * kArgmaxSplits workgroups must fit a grid

constexpr int kMaxUnion = 64;              // automata that one union call takes (their pointers travel as kernel arguments)
constexpr int kDedupeMaxStates = 1 << 26;  // states * 16 workgroups must fit a grid

// Bits of the device-side input check word.
enum : uint32_t {
    kBadTransition = 1u,   // table entry outside [0, n_states)
    kBadClass = 2u,        // byte_to_class value >= n_classes
    kBadOffsets = 4u,      // offsets decreasing / outside [0, n_bytes] / not starting at 0
    kDeadNotAbsorbing = 8u,
    kInputFlags = 15u,
    kLongTokens = 16u,     // (not an error) some token is longer than kMaxSetDepth bytes; travels with the check bits
};

// One vocabulary token as the walk kernels read it: 16 bytes, loaded as one dwordx4.
struct __attribute__((aligned(16))) TokenRecord {
    uint32_t cls_lo;   // byte classes 0..3 of the token, 8 bits each
    uint32_t cls_hi;   // byte classes 4..7
    uint32_t offset;   // start of the token in the class string
    uint32_t length;   // number of bytes; 0 for empty tokens and for the EOS token
};

// A state as the token-set walk reads it (one 16-byte uniform load).  Its outgoing transitions
// are grouped by target: pair = target | set id << 16, where the set id names the class set that
// leads to the target.  The first two pairs are inline, the rest start at `ext`.
struct __attribute__((aligned(16))) StateRecord {
    uint32_t n_pairs;
    uint32_t pair0, pair1;
    uint32_t ext;
};

// Where everything lives inside the caller's workspace.  All offsets are multiples of 256.
struct Plan {
    int32_t n_states = 0, n_classes = 0, n_tokens = 0;
    int64_t n_bytes = 0;
    int32_t entry_bytes = 2;       // width of a narrowed table entry: 2 (n_states <= 65535) or 4
    int32_t live_words = 1;        // 64-bit words of the per-state live-class mask
    int32_t n_blocks = 0;          // token blocks of 4096
    int32_t n_chunks = 0;          // n_blocks * 64 (padded)
    int32_t n_groups = 0;          // n_blocks * 4: columns of the dense path's count matrix
    int32_t states_per_wave = 0;   // dense path: consecutive states one wave walks
    int32_t n_ranges = 0;          // ceil(n_states / states_per_wave)
    bool sets_possible = false;    // host-side necessary conditions for the token-set path
    // the preparation kernel's workgroups: first those that classify bytes, then those that pack
    // tokens, then those that narrow states; each leaves one word of check bits
    int32_t cls_groups = 0, pack_groups = 0, narrow_groups = 0;
    size_t off_status = 0;         // Status
    size_t off_badw = 0;           // uint32 [cls_groups + pack_groups + narrow_groups] check bits per workgroup
    size_t off_sync = 0;           // SyncWords
    size_t off_cls = 0;            // uint8  [n_bytes]            class of every vocabulary byte
    size_t off_tok = 0;            // TokenRecord [n_chunks * 64]
    size_t off_key = 0;            // uint32 [n_chunks * 64] a token in four bytes: classes of its first three bytes, min(length, 255)
    size_t off_tab = 0;            // uint16/uint32 [n_states * n_classes]
    size_t off_live = 0;           // uint64 [n_states * live_words]
    size_t off_cnt = 0;            // uint32 [n_states * n_groups]  counts, then exclusive offsets
    size_t off_rowtot = 0;         // int64  [n_states]
    size_t off_allow = 0;          // uint64 [n_states][n_chunks] admissibility bitmap
    // token-set path only
    size_t off_npairs = 0;         // uint32 [n_states]  pairs per state
    size_t off_pmask = 0;          // uint64 [n_classes][n_states] class set of pair i of state q at i * n_states + q
    size_t off_pslot = 0;          // uint32 [n_classes][n_states] its slot in the class-set table, same layout
    size_t off_pairs = 0;          // uint32 [n_states][n_classes] target | set id << 16, state q's from q * n_classes
    size_t off_srec = 0;           // StateRecord [n_states]
    size_t off_order = 0;          // uint32 [n_states] the states, those with most pairs first
    size_t off_clsets = 0;         // uint64 [64][kSetCap / 64]  for every class, the sets that contain it
    size_t off_U = 0;              // uint64 [kMaxSetDepth][kSetCap][n_chunks]
    size_t off_E = 0;              // uint64 [kMaxSetDepth][n_chunks]
    size_t off_long = 0;           // uint32 [n_states * n_blocks] long segments: state << 12 | block
    size_t off_queue = 0;          // uint32 [256] work counters of the emit kernel
    size_t total = 0;
};

// What the numbering of the class sets leaves for the kernel that follows it.
struct SyncWords {
    uint32_t ids[kSetHashSlots];              // slot of the class-set table -> number of the set (0 .. n_sets - 1)
};

struct Status {       // mirrored at off_status
    int64_t nnz;
    uint32_t flags;
    uint32_t use_sets;     // decided on the device: the token-set kernels do the walk
    uint32_t n_sets;       // distinct class sets
    uint32_t n_pairs;      // (state, target) pairs
    uint32_t long_tokens;  // some token is longer than kMaxSetDepth bytes
    uint32_t overflow;     // the counting pass has to be redone: 1 = a token-set walk ran out of stack frames,
                           // 2 = the host expected the token-set kernels to count, the device decided against them
    uint32_t n_long;       // length of the list of long (state, block) segments (token-set path)
    uint32_t feasible;     // the token-set kernels could have counted, but the host had launched only the dense one
};

// Transpose of the 64 x 64 bit matrix whose row i is the word x of lane i: afterwards bit i of
// lane k's word is what bit k of lane i's word was.  Six rounds; round j swaps, between lanes
// that differ in bit j of their number, the blocks of bits whose position differs in bit j.
__device__ __forceinline__ uint64_t transpose_bits(uint64_t x, int lane)
{
    constexpr uint64_t kLow[6] = {0x5555555555555555ull, 0x3333333333333333ull, 0x0F0F0F0F0F0F0F0Full,
                                  0x00FF00FF00FF00FFull, 0x0000FFFF0000FFFFull, 0x00000000FFFFFFFFull};
#pragma unroll
    for (int r = 5; r >= 0; --r) {
        const int j = 1 << r;
        const uint64_t low = kLow[r];                            // positions b with (b & j) == 0
        const uint64_t other = __shfl_xor(x, j, kWave);
        x = (lane & j) == 0 ? (x & low) | ((other << j) & ~low) : (x & ~low) | ((other >> j) & low);
    }
    return x;
}

int make_plan(int32_t n_states, int32_t n_classes, int32_t n_tokens, int64_t n_bytes, Plan *plan);

// Kernel launchers (each enqueues on `stream` and returns the launch error, if any).
// expect: which counting kernel the host is going to launch: 0 = both (the device's choice runs,
// the other returns at once), 1 = the token-set kernels only, 2 = the dense kernel only (see
// Status::overflow and Status::feasible for what happens when the device would choose otherwise)
hipError_t launch_prepare(const Plan &p, const fsmidx_dfa &dfa, const fsmidx_vocab &vocab, char *ws, int expect,
                          hipStream_t stream);
hipError_t launch_token_sets(const Plan &p, const fsmidx_dfa &dfa, const fsmidx_vocab &vocab, char *ws,
                             hipStream_t stream);
// counting pass, either of two kernels (the choice is made on the device, see Status::use_sets)
hipError_t launch_walk(const Plan &p, const fsmidx_dfa &dfa, const fsmidx_vocab &vocab, char *ws, hipStream_t stream);
hipError_t launch_walk_sets(const Plan &p, const fsmidx_dfa &dfa, const fsmidx_vocab &vocab, char *ws, bool deep,
                            hipStream_t stream);
// emitting pass; writes nothing if the counting pass overflowed its stack, flagged bad input or
// found more than `capacity` entries
// (queues_clear: the scans have just run on this stream and no emit since, so the work counters
// are still zero; otherwise they are zeroed first)
hipError_t launch_emit(const Plan &p, const fsmidx_vocab &vocab, char *ws, const int64_t *row_ptr, int32_t *token_ids,
                       int32_t *next_states, int64_t capacity, bool queues_clear, hipStream_t stream);
hipError_t launch_disable_sets(const Plan &p, char *ws, hipStream_t stream);
hipError_t launch_retry_sets(const Plan &p, char *ws, hipStream_t stream);
hipError_t launch_scan(const Plan &p, char *ws, int64_t *row_ptr, hipStream_t stream);
hipError_t launch_mask(const fsmidx_csr &csr, const int32_t *states, int32_t batch, const void *in, void *out,
                       int64_t row_stride, int32_t dtype, hipStream_t stream);

hipError_t launch_advance(const fsmidx_csr &csr, const int32_t *states, const int32_t *tokens, int32_t batch,
                          int32_t *states_out, hipStream_t stream);
hipError_t launch_argmax(const fsmidx_csr &csr, const int32_t *states, int32_t batch, const void *logits,
                         int64_t row_stride, int32_t dtype, uint64_t *partial, int32_t *tokens_out,
                         int32_t *states_out, hipStream_t stream);

hipError_t launch_sample(const fsmidx_csr &csr, const int32_t *states, int32_t batch, const void *logits,
                         int64_t row_stride, int32_t dtype, const float *uniforms, uint64_t *partial, double *sums,
                         int32_t *tokens_out, int32_t *states_out, hipStream_t stream);

// union of automata; ws: 256 bytes of words ([0] classes of the union, [1] check flags) + kMaxUnion * 256 class ids
hipError_t launch_union_classes(const fsmidx_dfa *dfas, int32_t n_dfas, uint8_t *union_b2c, char *ws,
                                hipStream_t stream);
hipError_t launch_union_table(const fsmidx_dfa *dfas, int32_t n_dfas, const int32_t *state_base, int32_t union_dead,
                              int32_t n_union_classes, int32_t *trans_out, uint8_t *accept_out, char *ws,
                              hipStream_t stream);
// identical rows; ws starts with int64 [3]: distinct rows, their entries, collision flag
// minimisation of an automaton (minimise.hip)
// scanner step of parser-guided generation (scanner.hip)
size_t scanner_workspace_bytes(int32_t n_states, int32_t n_classes);
uint32_t *scanner_flags(char *ws);
uint32_t *scanner_changed(char *ws);
int scanner_launches_max();
hipError_t launch_scanner_start(const fsmidx_dfa &dfa, const uint64_t *completes, char *ws, uint64_t *V,
                                hipStream_t stream);
hipError_t launch_scanner_sweeps(const fsmidx_dfa &dfa, char *ws, uint64_t *V, int n, hipStream_t stream);
hipError_t launch_scanner_restarts(const fsmidx_dfa &dfa, const uint64_t *completes, const int32_t *scanner_of_state,
                                   const int32_t *shift, int32_t n_parse_states, int32_t n_terminals, int32_t *out,
                                   char *ws, hipStream_t stream);

size_t minimise_workspace_bytes(int32_t n_states);
hipError_t launch_min_start(const fsmidx_dfa &dfa, char *ws, bool first_attempt, hipStream_t stream);
hipError_t launch_min_rounds(const fsmidx_dfa &dfa, char *ws, uint64_t seed, uint32_t first_round, int n_rounds,
                             hipStream_t stream);
const int64_t *min_result(char *ws, int32_t n_states);
const uint32_t *min_counts(char *ws, int32_t n_states);
const uint32_t *min_block(char *ws, int32_t n_states);
int min_rounds_max();
hipError_t launch_min_quotient(const fsmidx_dfa &dfa, char *ws, int32_t *block_of_state, int32_t *trans_out,
                               int64_t trans_capacity, uint8_t *accept_out, hipStream_t stream);
// reachable states of an index and the index restricted to a set of states (reach.hip)
size_t reach_workspace_bytes(int32_t n_states);
hipError_t launch_reach_start(const fsmidx_csr &csr, char *ws, const int32_t *starts_host, int32_t n_starts,
                              hipStream_t stream);
hipError_t launch_reach_levels(const fsmidx_csr &csr, char *ws, uint32_t first_level, int n_levels, uint32_t expected,
                               hipStream_t stream);
const uint32_t *reach_next_count(char *ws, int32_t n_states, uint32_t level);
hipError_t launch_reach_finish(const fsmidx_csr &csr, char *ws, uint8_t *reach_out, hipStream_t stream);
hipError_t launch_restrict_scan(const fsmidx_csr &csr, const uint8_t *keep, char *ws, int64_t *row_ptr_out,
                                hipStream_t stream);
hipError_t launch_restrict_copy(const fsmidx_csr &csr, const uint8_t *keep, const int64_t *row_ptr_out,
                                int32_t *token_ids_out, int32_t *next_states_out, int64_t capacity, hipStream_t stream);
size_t dedupe_workspace_bytes(int32_t n_states);
hipError_t launch_dedupe(const fsmidx_csr &csr, char *ws, uint64_t seed, int32_t *row_of_state,
                         int64_t *unique_row_ptr, hipStream_t stream);
hipError_t launch_dedupe_copy(const fsmidx_csr &csr, char *ws, const int64_t *unique_row_ptr, int32_t *token_ids_out,
                              int32_t *next_states_out, hipStream_t stream);

int fail(int code, const char *fmt, ...);   // records the thread's last error, returns code

// Argument checks shared by the entry points that read rows of an index (api.hip).
int check_rows(const fsmidx_csr *index);
int check_argmax_call(const fsmidx_csr *index, const int32_t *states_dev, int32_t batch, const void *logits,
                      int64_t row_stride, int32_t dtype, const int32_t *tokens_out_dev, const int32_t *states_out_dev,
                      size_t *partial_bytes);

}  // namespace fsmidx
