// The scanner step of parser-guided generation (Section 4 and Section 4.1): every parse state reads
// a list of terminal symbols and scans with the union of their automata; all these scanners lie
// side by side in one transition table.
//
//  terminal sets   V(q): the terminals that the characters read so far can still become (the set
//      that Section 4.1 sees shrink while characters arrive) = the terminals completed in q or in
//      any state reachable from q: the least solution of V(q) = completes(q) | OR_c V(delta(q, c)).
//      Found by iteration.  A launch takes tiles of kTile consecutive states, one per workgroup, and
//      iterates inside the tile (sets of the tile's states in LDS, the others' read from memory as
//      they are) until the tile is stable or kSweeps sweeps are done; launches follow each other
//      until one changes nothing.  Automata compiled from grammars number the states of a literal
//      one after the other, so most chains close within a tile, in one launch.  The iteration is
//      chaotic (a sweep may or may not see what another thread has just written), which is fine:
//      the sets only grow, towards the one least solution.
//        scanner_start  : the table transposed ([class][state], so that a thread per state reads it
//                         coalesced) and range checked, V = completes
//        scanner_sweeps : one launch as described; returns at once if the launch before it changed
//                         nothing, so the host can enqueue several and look afterwards
//
//  restart table   delta'(q, c) = delta(q, c) where the scanner reads on; where it rejects, the
//      first terminal (in the order of the list) that q completes, that q's parse state may shift
//      and whose following scanner reads c decides: delta'(q, c) = delta(shift[p(q)][t], c).  This
//      is what lets a vocabulary string finish one terminal and begin the next (Section 4: " " and
//      "oo(" after "def f"); Algorithms 3 and 4 then index delta' like any automaton.
//        scanner_restarts : one thread per table entry
#include "internal.h"

namespace fsmidx {

constexpr int kTile = 1024;            // states per workgroup, one thread each
constexpr int kSweeps = 64;            // sweeps inside a tile per launch, at most
constexpr int kScannerLaunches = 64;   // launches the host may enqueue before it looks

enum : uint32_t {
    kBadParseState = 32u,              // scanner_of_state outside [0, n_parse_states) for a state that completes a terminal
    kBadShift = 64u,                   // shift value outside [-1, n_states)
    kBadTerminal = 128u,               // completes has a bit at or above n_terminals
};

struct ScannerHeader {                 // first 512 bytes of the workspace
    uint32_t flags;                    // check bits
    uint32_t pad[63];
    uint32_t changed[kScannerLaunches]; // launch i of a batch changed a set
};
static_assert(sizeof(ScannerHeader) == 512, "layout");

size_t scanner_workspace_bytes(int32_t n_states, int32_t n_classes)
{
    return sizeof(ScannerHeader) + ((size_t)n_states * (size_t)n_classes * 4 + 255) / 256 * 256;
}

uint32_t *scanner_flags(char *ws) { return &reinterpret_cast<ScannerHeader *>(ws)->flags; }
uint32_t *scanner_changed(char *ws) { return reinterpret_cast<ScannerHeader *>(ws)->changed; }
int scanner_launches_max() { return kScannerLaunches; }

__global__ __launch_bounds__(256) void scanner_clear(ScannerHeader *h, bool all)
{
    if (all && threadIdx.x == 0)
        h->flags = 0;
    if (threadIdx.x < kScannerLaunches)
        h->changed[threadIdx.x] = 0;
}

// One workgroup per 64 states x 64 classes: read along the rows, written along the columns.  A
// target outside the automaton is flagged and replaced by the state itself (which adds nothing to
// its own set).
__global__ __launch_bounds__(256) void scanner_start(const int32_t *__restrict__ trans, int32_t n_states,
                                                     int32_t n_classes, const uint64_t *__restrict__ completes,
                                                     uint32_t *__restrict__ tr, uint64_t *__restrict__ V,
                                                     ScannerHeader *h)
{
    __shared__ uint32_t tile[64][65];
    const int32_t q0 = (int32_t)blockIdx.x * 64, c0 = (int32_t)blockIdx.y * 64;
    const int x = threadIdx.x & 63, y0 = threadIdx.x >> 6;
    bool bad = false;
    for (int y = y0; y < 64; y += 4) {
        const int32_t q = q0 + y, c = c0 + x;
        if (q < n_states && c < n_classes) {
            int32_t v = trans[(int64_t)q * n_classes + c];
            if (v < 0 || v >= n_states) {
                bad = true;
                v = q;
            }
            tile[y][x] = (uint32_t)v;
        }
    }
    if (bad)
        atomicOr(&h->flags, kBadTransition);
    __syncthreads();
    for (int y = y0; y < 64; y += 4) {
        const int32_t q = q0 + x, c = c0 + y;
        if (q < n_states && c < n_classes)
            tr[(int64_t)c * n_states + q] = tile[x][y];
    }
    if (blockIdx.y == 0 && threadIdx.x < 64 && q0 + (int32_t)threadIdx.x < n_states)
        V[q0 + threadIdx.x] = completes[q0 + threadIdx.x];
}

__global__ __launch_bounds__(kTile) void scanner_sweeps(const uint32_t *__restrict__ tr, int32_t n_states,
                                                        int32_t n_classes, uint64_t *V, ScannerHeader *h, int launch)
{
    if (launch > 0 && h->changed[launch - 1] == 0)
        return;                                                   // uniform over the grid: the sets are final
    __shared__ uint64_t mine_s[kTile];
    __shared__ uint32_t changed_s;
    const int32_t q0 = (int32_t)blockIdx.x * kTile;
    const int32_t q = q0 + (int32_t)threadIdx.x;
    const bool live = q < n_states;
    const uint64_t at_start = live ? V[q] : 0ull;
    uint64_t mine = at_start;
    mine_s[threadIdx.x] = mine;
    for (int sweep = 0; sweep < kSweeps; ++sweep) {
        __syncthreads();
        if (threadIdx.x == 0)
            changed_s = 0;
        __syncthreads();
        uint64_t now = mine;
        if (live) {
            for (int32_t c = 0; c < n_classes; ++c) {
                const uint32_t s = tr[(int64_t)c * n_states + q];
                const uint32_t local = s - (uint32_t)q0;
                // (a set of another tile: whatever memory holds now; the launches to come see the rest)
                now |= local < (uint32_t)kTile ? mine_s[local] : __builtin_nontemporal_load(&V[s]);
            }
        }
        if (now != mine) {
            mine = now;
            mine_s[threadIdx.x] = now;
            changed_s = 1;
        }
        __syncthreads();
        if (changed_s == 0)
            break;                                                // uniform over the workgroup
    }
    if (mine != at_start) {
        V[q] = mine;
        h->changed[launch] = 1;
    }
}

__global__ __launch_bounds__(256) void scanner_restarts(const int32_t *__restrict__ trans, int32_t n_states,
                                                        int32_t n_classes, int32_t dead,
                                                        const uint64_t *__restrict__ completes,
                                                        const int32_t *__restrict__ scanner_of_state,
                                                        const int32_t *__restrict__ shift, int32_t n_parse_states,
                                                        int32_t n_terminals, int32_t *__restrict__ out, ScannerHeader *h)
{
    // (the table has fewer than 2^31 entries: 32-bit index arithmetic)
    const uint32_t total = (uint32_t)n_states * (uint32_t)n_classes;
    const uint64_t known = n_terminals >= 64 ? ~0ull : (1ull << n_terminals) - 1ull;
    uint32_t bad = 0;
    for (uint64_t at = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; at < total; at += (uint64_t)gridDim.x * blockDim.x) {
        const uint32_t i = (uint32_t)at;
        const int32_t q = (int32_t)(i / (uint32_t)n_classes), c = (int32_t)(i - (uint32_t)q * (uint32_t)n_classes);
        int32_t e = trans[i];
        if (e < 0 || e >= n_states) {
            bad |= kBadTransition;
            e = dead >= 0 ? dead : q;
        }
        if (dead >= 0 && e == dead && q != dead) {
            uint64_t done = completes[q];
            if (done & ~known) {
                bad |= kBadTerminal;
                done &= known;
            }
            if (done != 0) {
                const int32_t p = scanner_of_state[q];
                if (p < 0 || p >= n_parse_states) {
                    bad |= kBadParseState;
                    done = 0;
                }
                while (done != 0) {
                    const int t = __builtin_ctzll(done);
                    done &= done - 1;
                    const int32_t r = shift[(int64_t)p * n_terminals + t];
                    if (r < -1 || r >= n_states) {
                        bad |= kBadShift;
                        continue;
                    }
                    if (r < 0)
                        continue;
                    const int32_t v = trans[(int64_t)r * n_classes + c];
                    if (v < 0 || v >= n_states) {
                        bad |= kBadTransition;
                        continue;
                    }
                    if (v != dead) {
                        e = v;
                        break;
                    }
                }
            }
        }
        out[i] = e;
    }
    if (bad)
        atomicOr(&h->flags, bad);
}

hipError_t launch_scanner_start(const fsmidx_dfa &dfa, const uint64_t *completes, char *ws, uint64_t *V,
                                hipStream_t stream)
{
    ScannerHeader *h = reinterpret_cast<ScannerHeader *>(ws);
    uint32_t *tr = reinterpret_cast<uint32_t *>(ws + sizeof(ScannerHeader));
    hipLaunchKernelGGL(scanner_clear, dim3(1), dim3(256), 0, stream, h, true);
    hipLaunchKernelGGL(scanner_start, dim3((unsigned)((dfa.n_states + 63) / 64), (unsigned)((dfa.n_classes + 63) / 64)),
                       dim3(256), 0, stream, dfa.trans, dfa.n_states, dfa.n_classes, completes, tr, V, h);
    return hipGetLastError();
}

// `n` launches, numbered from 0 (the marks of the batch before are cleared first).
hipError_t launch_scanner_sweeps(const fsmidx_dfa &dfa, char *ws, uint64_t *V, int n, hipStream_t stream)
{
    ScannerHeader *h = reinterpret_cast<ScannerHeader *>(ws);
    const uint32_t *tr = reinterpret_cast<const uint32_t *>(ws + sizeof(ScannerHeader));
    hipLaunchKernelGGL(scanner_clear, dim3(1), dim3(256), 0, stream, h, false);
    for (int i = 0; i < n; ++i)
        hipLaunchKernelGGL(scanner_sweeps, dim3((unsigned)((dfa.n_states + kTile - 1) / kTile)), dim3(kTile), 0, stream, tr,
                           dfa.n_states, dfa.n_classes, V, h, i);
    return hipGetLastError();
}

hipError_t launch_scanner_restarts(const fsmidx_dfa &dfa, const uint64_t *completes, const int32_t *scanner_of_state,
                                   const int32_t *shift, int32_t n_parse_states, int32_t n_terminals, int32_t *out,
                                   char *ws, hipStream_t stream)
{
    ScannerHeader *h = reinterpret_cast<ScannerHeader *>(ws);
    hipLaunchKernelGGL(scanner_clear, dim3(1), dim3(256), 0, stream, h, true);
    const int64_t total = (int64_t)dfa.n_states * dfa.n_classes;
    const int64_t want = (total + 255) / 256;
    hipLaunchKernelGGL(scanner_restarts, dim3((unsigned)(want < 1 ? 1 : (want > 65536 ? 65536 : want))), dim3(256), 0, stream,
                       dfa.trans, dfa.n_states, dfa.n_classes, dfa.dead_state, completes, scanner_of_state, shift,
                       n_parse_states, n_terminals, out, h);
    return hipGetLastError();
}

}  // namespace fsmidx
