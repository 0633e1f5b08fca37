// Maximum-weight bipartite matching of the scored graph (paper: Algorithm
// "Scheduling algorithm", GetMatching; Section "Matching-based scheduling"
// states the problem and asks for the optimal matching).
//
// The paper solves it with the sequential Kuhn-Munkres algorithm.  Here the
// same optimum is reached by an epsilon-scaling forward/reverse auction, whose
// unit of work - "scan one line of the weight matrix against the current duals
// and keep the best two" - is a coalesced streaming read, and whose updates are
// 64-bit atomic maxima.  Weights are multiplied by K = min(n, m) + 1 so that the final
// epsilon = 1 is below 1/min(n, m) of a weight unit: the matching is then exactly
// optimal, and the duals it leaves behind prove it (see certificate_kernel).
//
// Formulation.  maximise sum W_ij x_ij, every row and column used at most
// once.  Dual: minimise sum pi_i + sum p_j with pi_i + p_j >= K W_ij, pi, p >= 0.
// The auction keeps, for the current epsilon,
//   (I1) pi_i + p_j >= K W_ij - eps on every feasible pair,
//   (I2) pi_i + p_j  = K W_ij      on every assigned pair,
// and stops a phase when every unassigned row has pi_i = 0 and every
// unassigned column has p_j = 0; then the assignment is within min(n, m)*eps of the
// optimum.  A forward round lets unassigned rows raise prices p; a reverse
// round lets unassigned columns that still carry a positive price raise
// profits pi (and lower their own price).  Both are the same computation with
// the roles of rows and columns exchanged, so one pair of kernels serves both,
// reading W for forward rounds and its transpose for reverse rounds.
//
// All dual values are integers below 2^43; the scans evaluate K*w - dual in
// double precision, where such integers and their differences are exact, so
// that they run at the full rate of the FP64 vector units.
#include "internal.h"
#include <math.h>

namespace {

constexpr int BID_THREADS = 256;
constexpr int MAX_GRID = 8192;
constexpr double NEG_HUGE = -1.0e300;

__device__ inline unsigned long long pack_word(double dual, int id_plus_one)
{
    return ((unsigned long long)(long long)dual << MF_ID_BITS) | (unsigned long long)id_plus_one;
}
__device__ inline double word_dual(unsigned long long w) { return (double)(long long)(w >> MF_ID_BITS); }
__device__ inline int word_id(unsigned long long w) { return (int)(w & MF_ID_MASK) - 1; }

struct Top2 {
    double b1, b2;      // best and second-best value
    int idx, w;         // position and weight of the best
};

__device__ inline void top2_merge(Top2 &t, const Top2 &o)
{
    const double nb2 = fmax(fmax(t.b2, o.b2), fmin(t.b1, o.b1));
    const bool take = (o.b1 > t.b1) || (o.b1 == t.b1 && o.idx < t.idx);
    t.idx = take ? o.idx : t.idx;
    t.w = take ? o.w : t.w;
    t.b1 = fmax(t.b1, o.b1);
    t.b2 = nb2;
}

struct SideArgs {
    const int32_t *A;                   // the bidding side's lines (W for rows, W^T for columns)
    long long pitch;
    int len;
    double *other_dual;                 // opposite duals as doubles, raised with atomicMax on the bits
    unsigned long long *otherword;      // opposite packed (dual, holder): the authoritative copy
    double eps, Kd;
    const int *line_len;                // optional: every entry of line b at or beyond line_len[b] is infeasible
    int typical_len;                    // what a scan reads on average (host-side choice of kernels only)
};

// How much of line b a scan has to read.
__device__ __forceinline__ int line_length(const SideArgs &s, int b)
{
    return s.line_len ? min(s.line_len[b], s.len) : s.len;
}

// Loads that must observe values other wavefronts produced during this kernel:
// they bypass the caches that atomics performed at the memory side do not update.
__device__ inline unsigned long long load_fresh_u64(const unsigned long long *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline unsigned load_fresh_u32(const unsigned *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void store_through(unsigned long long *p, unsigned long long v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline double load_fresh(const double *p)
{
    return __longlong_as_double((long long)__hip_atomic_load((const unsigned long long *)p, __ATOMIC_RELAXED,
                                                             __HIP_MEMORY_SCOPE_AGENT));
}

// Folds four consecutive entries (values v0..v3 at index j) into a running
// top-2: a min/max network finds the group's best two, and only a group that
// beats the running best pays for locating the entry.
//
// Ties.  Any entry attaining the best value is a correct choice, and "the
// smallest index" sends every one of a set of identical bidders to the same
// entry, where all but one lose.  Indices are therefore compared through a
// per-bidder key, index ^ salt (salt below 2^20, so keys stay below 2^20 too):
// identical bidders spread over tied entries.  Scans return the key; callers
// undo it with the same xor.
__device__ __forceinline__ int tie_salt(int bidder)
{
    return (int)(((unsigned)bidder * 2654435761u) >> 12) & 0xfffff;
}

__device__ __forceinline__ void top2_push4(double &b1, double &b2, int &idx, int &wbest, double v0,
                                           double v1, double v2, double v3, int j, const int4 &w, int salt)
{
    const double hi0 = fmax(v0, v1), lo0 = fmin(v0, v1);
    const double hi1 = fmax(v2, v3), lo1 = fmin(v2, v3);
    const double g1 = fmax(hi0, hi1);
    const double g2 = fmax(fmin(hi0, hi1), fmax(lo0, lo1));
    if (g1 > b1) {                                      // smallest index attaining the group's best
        const bool a0 = v0 == g1, a1 = v1 == g1, a2 = v2 == g1;
        idx = (j + (a0 ? 0 : a1 ? 1 : a2 ? 2 : 3)) ^ salt;
        wbest = a0 ? w.x : a1 ? w.y : a2 ? w.z : w.w;
    }
    b2 = fmax(fmax(b2, g2), fmin(b1, g1));
    b1 = fmax(b1, g1);
}

// Wavefront-wide reductions by data-parallel-primitive moves (row shifts
// within each row of 16 lanes, then row broadcasts), which cost a few cycles
// per step where a cross-lane permute through LDS costs a hundred.  Lanes a
// step has no source for keep their own value; maximum and minimum do not mind
// seeing a value twice.  The total lands in lane 63 and is read from there.
template <int CTRL>
__device__ __forceinline__ int dpp_move(int v)
{
    return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xf, 0xf, false);
}
template <int CTRL>
__device__ __forceinline__ double dpp_move(double v)
{
    return __hiloint2double(dpp_move<CTRL>(__double2hiint(v)), dpp_move<CTRL>(__double2loint(v)));
}
constexpr int DPP_ROW_SHR1 = 0x111, DPP_ROW_SHR2 = 0x112, DPP_ROW_SHR4 = 0x114, DPP_ROW_SHR8 = 0x118,
              DPP_ROW_BCAST15 = 0x142, DPP_ROW_BCAST31 = 0x143;

__device__ __forceinline__ double wave_max(double v)
{
    v = fmax(v, dpp_move<DPP_ROW_SHR1>(v));
    v = fmax(v, dpp_move<DPP_ROW_SHR2>(v));
    v = fmax(v, dpp_move<DPP_ROW_SHR4>(v));
    v = fmax(v, dpp_move<DPP_ROW_SHR8>(v));
    v = fmax(v, dpp_move<DPP_ROW_BCAST15>(v));
    v = fmax(v, dpp_move<DPP_ROW_BCAST31>(v));
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), 63),
                            __builtin_amdgcn_readlane(__double2loint(v), 63));
}

__device__ __forceinline__ int wave_min(int v)
{
    v = min(v, dpp_move<DPP_ROW_SHR1>(v));
    v = min(v, dpp_move<DPP_ROW_SHR2>(v));
    v = min(v, dpp_move<DPP_ROW_SHR4>(v));
    v = min(v, dpp_move<DPP_ROW_SHR8>(v));
    v = min(v, dpp_move<DPP_ROW_BCAST15>(v));
    v = min(v, dpp_move<DPP_ROW_BCAST31>(v));
    return __builtin_amdgcn_readlane(v, 63);
}

// Wavefront-wide top-2 of per-lane top-2s, as two plain maximum reductions: the
// best value, the first lane holding it (its index and weight are then read
// from that lane), and the best of everything else.
__device__ __forceinline__ Top2 wave_top2(const Top2 &t)
{
    Top2 r;
    r.b1 = wave_max(t.b1);
    // among lanes attaining the best, the smallest index wins (ties between lanes are rare)
    const bool hit = t.b1 == r.b1;
    const int idx = wave_min(hit ? t.idx : 0x7fffffff);
    r.idx = idx;
    const bool owner = hit && t.idx == idx;
    const unsigned long long own = __ballot(owner);
    const int src = own ? (int)__ffsll((long long)own) - 1 : 0;
    r.w = __builtin_amdgcn_readlane(t.w, src);
    r.b2 = wave_max(owner ? t.b2 : t.b1);
    return r;
}

// Scans line A[0..len) against dual[0..len): best and second-best value of
// K*w - dual, the entry attaining the best (as the key (index_base + position)
// ^ salt, smallest key among ties) and its weight.  Every thread of the
// NT-thread block must call it; the result is valid in thread 0.
// A is 16-byte aligned and padded to a multiple of four entries, dual
// likewise.  `fresh` re-reads the duals past the caches (block-uniform).
template <int NT>
__device__ inline Top2 block_scan(const int32_t *__restrict__ A, const double *__restrict__ dual,
                                  int len, double Kd, bool fresh, Top2 *red, int index_base, int salt)
{
    constexpr int UN = 4;               // independent load batches in flight per thread
    Top2 t{NEG_HUGE, NEG_HUGE, 0x7fffffff, 0};
    const int full = len & ~3;          // whole groups of four
    for (int j0 = threadIdx.x * 4; j0 < full; j0 += NT * 4 * UN) {
        int4 w[UN];
        double p[UN][4];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int j = j0 + u * NT * 4;
            if (j < full) {
                w[u] = *(const int4 *)(A + j);
                if (fresh) {
                    p[u][0] = load_fresh(dual + j); p[u][1] = load_fresh(dual + j + 1);
                    p[u][2] = load_fresh(dual + j + 2); p[u][3] = load_fresh(dual + j + 3);
                } else {
                    const double2 p01 = *(const double2 *)(dual + j);
                    const double2 p23 = *(const double2 *)(dual + j + 2);
                    p[u][0] = p01.x; p[u][1] = p01.y; p[u][2] = p23.x; p[u][3] = p23.y;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int j = j0 + u * NT * 4;
            if (j < full)
                top2_push4(t.b1, t.b2, t.idx, t.w, fma(Kd, (double)w[u].x, -p[u][0]),
                           fma(Kd, (double)w[u].y, -p[u][1]), fma(Kd, (double)w[u].z, -p[u][2]),
                           fma(Kd, (double)w[u].w, -p[u][3]), j + index_base, w[u], salt);
        }
    }
    if (full < len && (int)threadIdx.x == (full / 4) % NT) {   // the last, partial group
        const int4 w = *(const int4 *)(A + full);
        double p[3];
        for (int e = 0; e < 3; ++e) p[e] = fresh ? load_fresh(dual + full + e) : dual[full + e];
        top2_push4(t.b1, t.b2, t.idx, t.w, fma(Kd, (double)w.x, -p[0]),
                   full + 1 < len ? fma(Kd, (double)w.y, -p[1]) : NEG_HUGE,
                   full + 2 < len ? fma(Kd, (double)w.z, -p[2]) : NEG_HUGE, NEG_HUGE, full + index_base, w, salt);
    }
    // waves that saw no entry skip the reduction (they share SIMDs with the busy ones)
    const bool busy = (int)(threadIdx.x & ~63u) * 4 < len;
    if (busy) t = wave_top2(t);
    if (NT == 64) return t;
    __syncthreads();                       // protect `red` from its previous use
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = t;
    __syncthreads();
    if (threadIdx.x < 64) {
        t = threadIdx.x < NT / 64 ? red[threadIdx.x] : Top2{NEG_HUGE, NEG_HUGE, 0x7fffffff, 0};
        t = wave_top2(t);
    }
    return t;
}

// Whole-line scan of RB lines at once: the opposite duals are loaded once per
// four entries and applied to all RB lines, which cuts the on-chip traffic per
// entry (duals are 8 bytes, weights 4) and keeps RB + 2 loads in flight per
// thread.  On return red[r] holds line r's result (a barrier has been passed).
template <int NT, int RB>
__device__ __forceinline__ void block_scan_rows(const int32_t *const (&rows)[RB], const int (&salt)[RB],
                                                const double *__restrict__ dual, int len, double Kd,
                                                Top2 *red)
{
    double b1[RB], b2[RB];
    int idx[RB], wb[RB];
#pragma unroll
    for (int r = 0; r < RB; ++r) { b1[r] = NEG_HUGE; b2[r] = NEG_HUGE; idx[r] = 0x7fffffff; wb[r] = 0; }
    const int full = len & ~3;                          // whole groups of four
#pragma unroll 2
    for (int j = threadIdx.x * 4; j < full; j += NT * 4) {
        int4 w[RB];
#pragma unroll
        for (int r = 0; r < RB; ++r) w[r] = *(const int4 *)(rows[r] + j);
        const double2 p01 = *(const double2 *)(dual + j);
        const double2 p23 = *(const double2 *)(dual + j + 2);
#pragma unroll
        for (int r = 0; r < RB; ++r)
            top2_push4(b1[r], b2[r], idx[r], wb[r], fma(Kd, (double)w[r].x, -p01.x),
                       fma(Kd, (double)w[r].y, -p01.y), fma(Kd, (double)w[r].z, -p23.x),
                       fma(Kd, (double)w[r].w, -p23.y), j, w[r], salt[r]);
    }
    if (full < len && (int)threadIdx.x == (full / 4) % NT) {   // the last, partial group
        const double2 p01 = *(const double2 *)(dual + full);
        const double2 p23 = *(const double2 *)(dual + full + 2);
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            const int4 w = *(const int4 *)(rows[r] + full);
            top2_push4(b1[r], b2[r], idx[r], wb[r], fma(Kd, (double)w.x, -p01.x),
                       full + 1 < len ? fma(Kd, (double)w.y, -p01.y) : NEG_HUGE,
                       full + 2 < len ? fma(Kd, (double)w.z, -p23.x) : NEG_HUGE, NEG_HUGE, full, w, salt[r]);
        }
    }
    __syncthreads();                       // protect `red` from its previous use
#pragma unroll
    for (int r = 0; r < RB; ++r) {
        const Top2 t = wave_top2(Top2{b1[r], b2[r], idx[r], wb[r]});
        if ((threadIdx.x & 63) == 0) red[RB + r * (NT / 64) + (threadIdx.x >> 6)] = t;
    }
    __syncthreads();
    if (threadIdx.x < RB) {                // thread r folds the per-wave results of line r
        Top2 t = red[RB + threadIdx.x * (NT / 64)];
        for (int wv = 1; wv < NT / 64; ++wv) top2_merge(t, red[RB + threadIdx.x * (NT / 64) + wv]);
        red[threadIdx.x] = t;
    }
    __syncthreads();
}

// One thread: bidder b has seen best value t.b1 at column/row t.idx and
// second-best t.b2.  A bidder whose best value is at most eps rests with dual
// 0.  (A bidder's own dual is implied by what it holds - K*w minus the dual it
// offered, or 0 when it holds nothing - and is written out once the run is
// over; nothing reads it while bids are flying.)  Otherwise it offers the opposite workload the highest dual at which that
// workload is still within eps of the bidder's best alternative; the offer is
// an atomicMax on the packed (dual, holder) word, so the highest offer wins
// whatever the order.  The offer is formed from the weight itself, not from the
// dual the scan happened to read, which may have moved since.
// Returns the workload that has to bid next because of this bid (the bidder
// itself if it was outbid in the meantime, the previous holder if it won), or -1.
__device__ inline int decide_and_bid(const SideArgs &s, int b, const Top2 &t)
{
    if (t.b1 <= s.eps) return -1;
    const double keep = fmax(t.b2 - s.eps, 0.0);
    const double offer = s.Kd * (double)t.w - keep;
    const unsigned long long mine = pack_word(offer, b + 1);
    const unsigned long long old = atomicMax(&s.otherword[t.idx], mine);
    unsigned long long *dual_bits = (unsigned long long *)&s.other_dual[t.idx];
    if (old < mine) {
        atomicMax(dual_bits, (unsigned long long)__double_as_longlong(offer));
        return word_id(old);
    }
    atomicMax(dual_bits, (unsigned long long)__double_as_longlong(word_dual(old)));
    return b;
}

// One round for many bidders: a workgroup per bidder, bids taking effect at
// once.  Later bidders of the same round may already see them (or a slightly
// older dual): the auction tolerates both because duals only move one way and a
// bid computed from an outdated dual simply fails to win.  The counters form a
// ring: round r reads cnt[r], fills cnt[r+1] and clears cnt[r+2].
template <int NT, int RB>
__global__ __launch_bounds__(NT) void round_kernel(SideArgs s, const int *__restrict__ list,
                                                   int *__restrict__ next, mf_device_stats *stats,
                                                   int ring)
{
    __shared__ Top2 red[RB + RB * (NT / 64)];
    const int count = stats->cnt[ring & 3];
    int *ncnt = &stats->cnt[(ring + 1) & 3];
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        stats->cnt[(ring + 2) & 3] = 0;
        stats->head = 0;
        if (count > 0) {
            stats->rounds += 1ull;
            stats->bids += (unsigned long long)count;
        }
    }
    unsigned long long entries = 0;                         // scanned by this workgroup (thread 0 keeps count)
    for (int item = blockIdx.x * RB; item < count; item += gridDim.x * RB) {
        int salt[RB];
        const int32_t *rows[RB];
        int len = 0;                                        // the group scans as far as its longest line
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            const int b = list[min(item + r, count - 1)];   // a short last group repeats its last line
            rows[r] = s.A + (size_t)b * s.pitch;
            salt[r] = tie_salt(b);
            const int lb = line_length(s, b);
            len = max(len, lb);
            if (item + r < count) entries += (unsigned long long)lb;
        }
        block_scan_rows<NT, RB>(rows, salt, s.other_dual, len, s.Kd, red);
        if (threadIdx.x < 64) {                                      // first wavefront: one lane bids per line
            int again = -1;
            if (threadIdx.x < RB && item + (int)threadIdx.x < count) {
                const int b = list[item + threadIdx.x];
                Top2 t = red[threadIdx.x];
                t.idx ^= tie_salt(b);
                again = decide_and_bid(s, b, t);
            }
            // one counter update per workgroup: the list counter is a single hot address
            const unsigned long long pushing = __ballot(again >= 0);
            if (pushing) {
                int base = 0;
                if (threadIdx.x == 0) base = atomicAdd(ncnt, __popcll(pushing));
                base = __shfl(base, 0);
                if (again >= 0) next[base + __popcll(pushing & ((1ull << threadIdx.x) - 1ull))] = again;
            }
        }
    }
    if (threadIdx.x == 0 && entries) atomicAdd(&stats->bytes, entries * 4ull);
}

// The tail of a run.  When few bidders are left, rounds are bound by launch
// latency and the work is a handful of chains: a bid evicts a holder, who bids
// next, and so on.  Each workgroup takes a pending bidder and then follows its
// chain - after every bid it goes on with whoever has to bid because of it -
// so no workgroup creates work for another, none waits for another, and each
// stops as soon as the list is used up.  `stats->active` counts the workgroups
// still following a chain; once it is at most `hand_back_at` the rest hand their
// bidders back, so that the host can put several workgroups on each chain.
constexpr int CHAIN_THREADS = 1024;

__global__ __launch_bounds__(CHAIN_THREADS) void chain_kernel(SideArgs s, const int *__restrict__ list,
                                                              int *__restrict__ out_list,
                                                              mf_device_stats *stats, int ring,
                                                              long long step_cap, int hand_back_at)
{
    __shared__ Top2 red[CHAIN_THREADS / 64];
    __shared__ int s_next, s_active;
    if (threadIdx.x == 0) s_active = 0x7fffffff;
    const int count = stats->cnt[ring & 3];
    unsigned long long steps = 0, retries = 0, scanned = 0;
    for (;;) {
        __syncthreads();
        if (threadIdx.x == 0) s_next = atomicAdd(&stats->head, 1);
        __syncthreads();
        const int item = s_next;
        if (item >= count) break;
        int b = list[item];
        bool fresh = false;                 // re-read the duals past the caches after a bid that lost
        while (b >= 0) {
            if ((steps & 3) == 0) {         // now and then: how many workgroups still follow a chain?
                __syncthreads();
                if (threadIdx.x == 0)
                    s_active = __hip_atomic_load(&stats->active, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __syncthreads();
            }
            if ((long long)steps >= step_cap || s_active <= hand_back_at) {
                if (threadIdx.x == 0) out_list[atomicAdd(&stats->cnt[(ring + 1) & 3], 1)] = b;
                break;
            }
            ++steps;
            const int len = line_length(s, b);
            scanned += (unsigned long long)len;
            Top2 t = block_scan<CHAIN_THREADS>(s.A + (size_t)b * s.pitch, s.other_dual, len, s.Kd, fresh, red,
                                               0, tie_salt(b));
            t.idx ^= tie_salt(b);
            if (threadIdx.x == 0) s_next = decide_and_bid(s, b, t);
            __syncthreads();
            fresh = (s_next == b);
            if (fresh && threadIdx.x == 0) ++retries;
            b = s_next;
        }
        if (b >= 0) break;                  // handed back: take no further bidder
    }
    if (threadIdx.x == 0) {
        atomicAdd(&stats->active, -1);      // this workgroup follows no chain any more
        if (steps) {
            atomicAdd(&stats->bids, steps);
            atomicAdd(&stats->chain_bids, steps);
            atomicAdd(&stats->bytes, scanned * 4ull);
            atomicMax(&stats->launch_max, steps);
            if (retries) atomicAdd(&stats->chain_retries, retries);
        }
    }
}

__global__ void chain_begin_kernel(mf_device_stats *stats, int ring, int workgroups)
{
    stats->head = 0;
    stats->active = workgroups;
    stats->cnt[(ring + 1) & 3] = 0;
    stats->cnt[(ring + 2) & 3] = 0;
    stats->rounds += 1ull;
    stats->chain_depth += stats->launch_max;     // of the previous chain kernel
    stats->launch_max = 0;
}

// The last few chains.  One compute unit cannot keep enough memory requests in
// flight to read a 100 KB line in much under ten microseconds, and with one
// or two chains left that latency is all there is.  Here TEAM_SIZE workgroups
// (on as many compute units) share each step of one chain: the leader
// publishes the bidder, every member scans its slice of the line and posts
// its top-2, the leader merges them, bids and publishes the next bidder.
// Members only ever wait for their leader and the leader for its members;
// every wait is bounded, and a wait that runs out raises `abort` so that all
// workgroups leave and the host falls back to chain_kernel.
constexpr int TEAM_SIZE_MAX = 32;        // workgroups per chain (run-time choice up to this)
constexpr int TEAM_MAX = 64;             // chains served at once
constexpr int TEAM_WIDE_MIN_LINE = 8192; // shortest line for which many small teams pay
constexpr unsigned TEAM_SPIN_LIMIT = 1u << 21;

struct alignas(128) TeamCtl {
    unsigned long long cmd;             // sequence << 32 | fresh << 31 | (bidder + 1); bidder + 1 == 0: stop
    unsigned int abort;
    unsigned int pad0;
    unsigned long long pad[14];
    // a member's result: three words, each carrying the low 8 bits of the step's sequence number,
    // so that the leader can tell a word of this step from the previous one without any fence:
    // best << 8 | tag, second << 8 | tag, index << 40 | (weight & 0xffffffff) << 8 | tag
    unsigned long long partial[TEAM_SIZE_MAX][4];
};

__device__ inline unsigned long long tag_value(double v, unsigned tag)
{
    const double c = fmin(fmax(v, -4.0e15), 4.0e15);        // integers up to 2^52 in magnitude
    return ((unsigned long long)(long long)c << 8) | (unsigned long long)(tag & 0xffu);
}
__device__ inline double untag_value(unsigned long long w)
{
    return (double)((long long)w >> 8);
}

__global__ void team_begin_kernel(mf_device_stats *stats, TeamCtl *ctl, int ring)
{
    const int t = threadIdx.x;
    if (t < TEAM_MAX) {
        ctl[t].cmd = 0ull; ctl[t].abort = 0u;
        for (int k = 0; k < TEAM_SIZE_MAX; ++k) { ctl[t].partial[k][0] = 0ull; ctl[t].partial[k][1] = 0ull; ctl[t].partial[k][2] = 0ull; }
    }
    if (t == 0) {
        stats->head = 0;
        stats->cnt[(ring + 1) & 3] = 0;
        stats->cnt[(ring + 2) & 3] = 0;
        stats->rounds += 1ull;
        stats->chain_depth += stats->launch_max;
        stats->launch_max = 0;
    }
}

template <int NT>
__global__ __launch_bounds__(NT) void team_kernel(SideArgs s, const int *__restrict__ list,
                                                  int *__restrict__ out_list, mf_device_stats *stats,
                                                  TeamCtl *ctl_all, int ring, long long step_cap,
                                                  int TEAM_SIZE)
{
    __shared__ Top2 red[NT / 64];
    __shared__ long long s_word;
    TeamCtl *ctl = ctl_all + blockIdx.x / TEAM_SIZE;
    const int member = blockIdx.x % TEAM_SIZE;
    const int count = stats->cnt[ring & 3];
    // the members share a line in equal slices of what has to be read of it
    auto slice_of = [&](int b, int &off) {
        const int len = line_length(s, b);
        const int slice = (((len + TEAM_SIZE - 1) / TEAM_SIZE) + 3) & ~3;
        off = member * slice;
        return max(0, min(slice, len - off));
    };

    if (member != 0) {
        // ---- member: wait for the leader's next command, scan, post ----
        unsigned expect = 1;
        for (;;) {
            __syncthreads();
            if (threadIdx.x == 0) {
                unsigned long long c = 0ull;
                unsigned spins = 0;
                for (;;) {
                    c = load_fresh_u64(&ctl->cmd);
                    if ((unsigned)(c >> 32) == expect) break;
                    ++spins;
                    if (spins > TEAM_SPIN_LIMIT || ((spins & 255u) == 0u && load_fresh_u32(&ctl->abort))) { c = 0ull; break; }
                }
                if (c == 0ull) atomicExch(&ctl->abort, 1u);
                s_word = (long long)c;
            }
            __syncthreads();
            const unsigned long long c = (unsigned long long)s_word;
            const int b = (int)(c & 0x7fffffffull) - 1;
            if (b < 0) break;                                   // stop (or abort)
            // a slice is small enough to stay in this compute unit's cache from step to step, so the
            // duals are always read past the caches here
            int off;
            const int my_len = slice_of(b, off);
            const Top2 t = block_scan<NT>(s.A + (size_t)b * s.pitch + off, s.other_dual + off, my_len, s.Kd,
                                          true, red, off, tie_salt(b));
            if (threadIdx.x == 0) {
                const int idx = t.idx == 0x7fffffff ? 0 : t.idx;      // already a key on the global index
                store_through(&ctl->partial[member][0], tag_value(t.b1, expect));
                store_through(&ctl->partial[member][1], tag_value(t.b2, expect));
                store_through(&ctl->partial[member][2], ((unsigned long long)(unsigned)idx << 40) |
                                                            ((unsigned long long)(unsigned)t.w << 8) | (expect & 0xffu));
            }
            ++expect;
        }
        return;
    }

    // ---- leader: follow chains, one command per step ----
    unsigned seq = 0;
    unsigned long long steps = 0, retries = 0, scanned = 0;
    bool dead = false;
    while (!dead) {
        __syncthreads();
        if (threadIdx.x == 0) s_word = atomicAdd(&stats->head, 1);
        __syncthreads();
        const int item = (int)s_word;
        if (item >= count) break;
        int b = list[item];
        bool fresh = false;
        while (b >= 0) {
            if ((long long)steps >= step_cap) {
                if (threadIdx.x == 0) out_list[atomicAdd(&stats->cnt[(ring + 1) & 3], 1)] = b;
                dead = true;
                break;
            }
            ++steps;
            ++seq;
            if (threadIdx.x == 0)
                store_through(&ctl->cmd, ((unsigned long long)seq << 32) | (fresh ? 0x80000000ull : 0ull) |
                                             (unsigned long long)(b + 1));
            int off;
            const int my_len = slice_of(b, off);                       // member 0: off == 0
            scanned += (unsigned long long)line_length(s, b);
            const Top2 t = block_scan<NT>(s.A + (size_t)b * s.pitch, s.other_dual, my_len, s.Kd, true, red, 0,
                                          tie_salt(b));
            if (threadIdx.x < 64) {                         // first wavefront: one lane per member
                const int k = threadIdx.x;
                Top2 mine = t;                              // lane 0: the leader's own slice
                int ok = 1;
                if (k >= TEAM_SIZE) {
                    mine = Top2{NEG_HUGE, NEG_HUGE, 0x7fffffff, 0};
                } else if (k >= 1) {                        // wait for member k's three words of this step
                    const unsigned tag = seq & 0xffu;
                    unsigned long long w0, w1, w2;
                    unsigned spins = 0;
                    for (;;) {
                        w0 = load_fresh_u64(&ctl->partial[k][0]);
                        w1 = load_fresh_u64(&ctl->partial[k][1]);
                        w2 = load_fresh_u64(&ctl->partial[k][2]);
                        if ((w0 & 0xffu) == tag && (w1 & 0xffu) == tag && (w2 & 0xffu) == tag) break;
                        ++spins;
                        if (spins > TEAM_SPIN_LIMIT || ((spins & 255u) == 0u && load_fresh_u32(&ctl->abort))) { ok = 0; break; }
                    }
                    mine.b1 = untag_value(w0);
                    mine.b2 = untag_value(w1);
                    mine.idx = (int)(w2 >> 40);
                    mine.w = (int)(unsigned)((w2 >> 8) & 0xffffffffull);
                }
                ok = __all(ok);
                if (ok) {
                    mine = wave_top2(mine);
                    mine.idx ^= tie_salt(b);
                    if (threadIdx.x == 0) s_word = decide_and_bid(s, b, mine);
                } else if (threadIdx.x == 0) {
                    atomicExch(&ctl->abort, 1u);
                    out_list[atomicAdd(&stats->cnt[(ring + 1) & 3], 1)] = b;
                    s_word = -2;
                }
            }
            __syncthreads();
            const int next = (int)s_word;
            if (next == -2) { dead = true; break; }
            fresh = (next == b);
            retries += fresh;
            b = next;
        }
    }
    if (threadIdx.x == 0) {
        store_through(&ctl->cmd, (unsigned long long)(seq + 1) << 32);      // stop
        if (load_fresh_u32(&ctl->abort)) atomicExch(&stats->team_abort, 1);
        if (steps) {
            atomicAdd(&stats->bids, steps);
            atomicAdd(&stats->chain_bids, steps);
            atomicAdd(&stats->team_bids, steps);
            atomicAdd(&stats->bytes, scanned * 4ull);
            atomicMax(&stats->launch_max, steps);
            if (retries) atomicAdd(&stats->chain_retries, retries);
        }
    }
}

// The last bidders of a run, placed by shortest augmenting paths.
//
// A chain of bids is a greedy walk: every evicted holder moves to its own best
// alternative, and with one or two bidders left such a walk takes thousands of
// dependent steps to reach a free line.  The shortest way to make room is far
// shorter in hops, and finding it is a breadth-type search whose every step is
// wide.  For a bidder r, in the notation of the header of this file with
// "rows" the bidding side, let rc(i,k) = pi_i + p_k - K W_ik + eps >= 0 (I1)
// for every assigned row i and for r (pi_r = best value of r - eps); assigned
// pairs have rc = eps.  A path r -> k1, holder(k1) -> k2, ... that ends in a
// column nobody holds, or in a row giving up its column for profit 0 (at extra
// length pi_i), frees a place for r; label(k) is the length sum(rc) of the
// shortest such path to column k and d the length of the shortest complete
// one.  Raising p_k by d - label(k) on every column with label(k) < d (their
// holders' profits drop by as much) keeps I1 and I2 and makes the shortest
// path tight; re-assigning along it, each row paying eps more for its new
// column, keeps them too and leaves one bidder fewer.  Prices only rise, so
// this mixes freely with bids.  (The successive-shortest-path step of the
// Hungarian method, on costs relaxed by eps.)
//
// All compute units run the search together: labels are corrected in
// super-steps - every row whose column's label dropped into the current
// window [low, low + width) is scanned against all columns, in parallel, with
// an atomic minimum per improved label - separated by grid-wide barriers.
// Data shared between workgroups moves only through atomics and uncached
// loads/stores.  Every wait is bounded; if one runs out all workgroups leave,
// nothing half-done (the price update alone is a valid state), and the host
// falls back to the chain kernels.
constexpr int PATH_THREADS = 1024;
constexpr int PATH_MAX_SLICES = 1024;
constexpr int PATH_GROUP = 16, PATH_MAX_GROUPS = 64;      // up to 1024 workgroups
constexpr int PATH_SEGMENTS = 16, PATH_PUSH_BUFFER = 4096;
constexpr unsigned long long PATH_INF = ~0ull;
constexpr int PATH_FRONTIER_LOW = 128, PATH_FRONTIER_HIGH = 1024;

struct alignas(128) PathCtl {
    unsigned long long sink;        // shortest complete path: length << 21 | kind << 20 | id (kind 1: row id gives up)
    unsigned long long low[3];      // smallest label still to be expanded, per slot
    // best value of the current bidder (bits of a double), by parity of its position in the list:
    // when a bidder rests, workgroup 0 may already be writing the next bidder's value while a
    // slower workgroup has yet to read this one
    unsigned long long first_value[2];
    unsigned int arrive, pad[3];    // whole groups that have arrived at barriers so far | PATH_GAVE_UP
    unsigned long long steps, scans, entries;
    struct alignas(128) { unsigned int arrive; } group[PATH_MAX_GROUPS];
    // Frontier lengths: one counter per segment (a segment collects the pushes of sixteen
    // workgroups, so no counter is hit by more than sixteen atomics per step), in three slots:
    // step t reads slot t % 3, fills slot (t + 1) % 3 and clears slot (t + 2) % 3, which every
    // workgroup finished reading before the barrier that ended step t - 1.
    struct alignas(128) { unsigned int count; } seg[3][PATH_SEGMENTS];
};

struct PathBuffers {
    unsigned long long *label;      // [len] length << 20 | predecessor row
    unsigned long long *expanded;   // [len] label at which the column's holder was last scanned
    unsigned int *stamp;            // [len] last step in which the column was put on a frontier
    int *fr_col[2];                 // frontiers (by step parity): PATH_SEGMENTS segments of len columns each
    int *held;                      // [rows] column a frontier row holds
};

// Grid-wide barrier in two levels: workgroups arrive at their group's counter, the last of a
// group at the top counter, and everybody waits until the top counter shows that all groups have
// arrived for the so-many-th time.  (Hundreds of atomics on one address take turns; sixteen
// groups of sixteen do not.)  Counters only ever grow.  The top bit of the top counter says that
// somebody's wait ran out: whoever sees it leaves, so one load tells a waiting workgroup both.
// Returns false when the wait ran out or another workgroup gave up.
constexpr unsigned PATH_GAVE_UP = 0x80000000u;

__device__ inline bool grid_barrier(PathCtl *ctl, unsigned workgroups, unsigned &generation, unsigned spin_limit)
{
    __shared__ int s_ok;
    // every thread's writes (uncached stores and atomics) are acknowledged by memory before its
    // workgroup reports in
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned groups = (workgroups + PATH_GROUP - 1) / PATH_GROUP;
        const unsigned g = blockIdx.x / PATH_GROUP;
        const unsigned size = min((unsigned)PATH_GROUP, workgroups - g * PATH_GROUP);
        const unsigned target = (generation + 1u) * groups;      // whole groups arrived once this barrier is complete
        unsigned seen = 0u;
        if ((atomicAdd(&ctl->group[g].arrive, 1u) + 1u) % size == 0u) seen = atomicAdd(&ctl->arrive, 1u) + 1u;
        unsigned spins = 0;
        while (!(seen & PATH_GAVE_UP) && seen < target) {
            if (++spins > spin_limit) { seen = atomicOr(&ctl->arrive, PATH_GAVE_UP) | PATH_GAVE_UP; break; }
            seen = load_fresh_u32(&ctl->arrive);
        }
        s_ok = (seen & PATH_GAVE_UP) ? 0 : 1;
    }
    ++generation;
    __syncthreads();
    return s_ok != 0;
}

__global__ void path_begin_kernel(mf_device_stats *stats, PathCtl *ctl, int ring)
{
    ctl->arrive = 0u; ctl->steps = 0ull; ctl->scans = 0ull; ctl->entries = 0ull;
    for (int g = 0; g < PATH_MAX_GROUPS; ++g) ctl->group[g].arrive = 0u;
    stats->cnt[(ring + 1) & 3] = 0;
    stats->cnt[(ring + 2) & 3] = 0;
    stats->rounds += 1ull;
    stats->chain_depth += stats->launch_max;
    stats->launch_max = 0;
}

__device__ inline void store_dual(const SideArgs &s, int k, double dual, int holder_plus_one)
{
    store_through(&s.otherword[k], pack_word(dual, holder_plus_one));
    store_through((unsigned long long *)&s.other_dual[k], (unsigned long long)__double_as_longlong(dual));
}

__global__ __launch_bounds__(PATH_THREADS) void path_kernel(SideArgs s, const int *__restrict__ list,
                                                            int *__restrict__ out_list, mf_device_stats *stats,
                                                            PathCtl *ctl, PathBuffers buf, int ring, int rows,
                                                            double width_max, unsigned spin_limit)
{
    __shared__ Top2 red[PATH_THREADS / 64];
    __shared__ unsigned s_pushes, s_base, s_first[PATH_SEGMENTS + 1];
    __shared__ unsigned long long s_sink, s_low;
    __shared__ int s_list[PATH_PUSH_BUFFER];
    const unsigned G = gridDim.x;
    const int wg = blockIdx.x, tid = threadIdx.x;
    const int gtid = wg * PATH_THREADS + tid, gsize = (int)G * PATH_THREADS;
    const int count = stats->cnt[ring & 3];
    unsigned generation = 0;
    int item = 0;
    bool alive = true;
    for (; item < count && alive; ++item) {
        const int r0 = list[item];
        // ---- clear the labels; workgroup 0 finds the bidder's best value ----
        for (int k = gtid; k < s.len; k += gsize) {
            store_through(&buf.label[k], PATH_INF);
            store_through(&buf.expanded[k], PATH_INF);
            __hip_atomic_store(&buf.stamp[k], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (wg == 0) {
            const Top2 t = block_scan<PATH_THREADS>(s.A + (size_t)r0 * s.pitch, s.other_dual, line_length(s, r0),
                                                    s.Kd, true, red, 0, 0);
            if (tid < 3 * PATH_SEGMENTS)
                __hip_atomic_store(&ctl->seg[tid / PATH_SEGMENTS][tid % PATH_SEGMENTS].count, 0u, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            if (tid == 0) {
                const double v1 = t.b1;
                store_through(&ctl->first_value[item & 1], (unsigned long long)__double_as_longlong(v1));
                store_through(&ctl->low[0], PATH_INF);
                store_through(&ctl->low[1], PATH_INF);
                store_through(&ctl->low[2], PATH_INF);
                if (v1 > s.eps) {                                       // pi_r = v1 - eps: rc(r, best column) = 0
                    store_through(&ctl->sink, ((unsigned long long)(long long)(v1 - s.eps) << 21) | (1ull << 20) |
                                                  (unsigned long long)r0);
                    __hip_atomic_store(&buf.held[r0], -1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
        if (!grid_barrier(ctl, G, generation, spin_limit)) { alive = false; break; }
        // duals stand still during a search: drop what the caches hold of them from before the
        // last re-assignment once, then read them through the caches
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        const double v1 = __longlong_as_double((long long)load_fresh_u64(&ctl->first_value[item & 1]));
        if (v1 <= s.eps) continue;                                      // rests with dual 0: nothing to move
        const double first_profit = v1 - s.eps;

        // ---- label-correcting search, one grid barrier per super-step ----
        // A step scans the rows on the current frontier; a label that falls inside the window
        // puts its column on the next frontier at once (claimed through a per-step stamp, so once
        // per step), whose holder is scanned in the next step from the label the column has by
        // then.  Only when a frontier comes up empty does a pass over all columns pick up the
        // labels that fell outside earlier windows, or move the window on.
        double low = 0.0;
        // The window adapts to what it yields: wide enough to keep the device busy, narrow enough
        // that rows are not scanned long before their label is final (every workgroup derives the
        // same width from the same counters).
        double width = 4.0 * s.eps;
        unsigned long long my_steps = 0, my_scans = 0, my_entries = 0;
        const int segment = wg / PATH_GROUP % PATH_SEGMENTS;
        unsigned step = 0;
        bool swept = false;                      // the previous step was a pass over all columns
        for (;;) {
            // far more steps than a search over sound duals can take: give the bidder back to the
            // chains (every workgroup counts the same steps, so all leave here together)
            if (++step > 4u * (unsigned)s.len + 4096u) { alive = false; break; }
            const unsigned c = step % 3u, p = (step + 1u) % 3u, z = (step + 2u) % 3u;
            // frontier of this step: its segments' lengths (the very first holds just the bidder)
            if (tid < 64) {
                unsigned n_seg = 0;
                if (tid < PATH_SEGMENTS && step > 1u) n_seg = load_fresh_u32(&ctl->seg[c][tid].count);
                unsigned run = n_seg;                               // inclusive prefix sums over 16 lanes
                for (int d = 1; d < PATH_SEGMENTS; d <<= 1) {
                    const unsigned o = __shfl_up(run, d);
                    if ((int)tid >= d) run += o;
                }
                if (tid < PATH_SEGMENTS) s_first[tid + 1] = run;
                if (tid == 0) { s_first[0] = 0u; s_pushes = 0u; s_sink = PATH_INF; s_low = PATH_INF; }
            }
            __syncthreads();
            const int nf = step == 1u ? 1 : (int)s_first[PATH_SEGMENTS];
            const unsigned long long sink_word = load_fresh_u64(&ctl->sink);
            const double bound = (double)(long long)(sink_word >> 21);
            if (step > 1u && swept && nf == 0) {
                const unsigned long long lo = load_fresh_u64(&ctl->low[c]);
                if (lo == PATH_INF || lo >= (sink_word >> 21)) break;       // every label below the sink is final
                low = (double)(long long)lo;                                // move the window to the next label
            }
            if (nf > PATH_FRONTIER_HIGH) width = fmax(s.eps, width * 0.5);
            else if (nf < PATH_FRONTIER_LOW) width = fmin(width_max, width * 2.0);
            const double limit = fmin(low + width, bound);
            if (gtid < PATH_SEGMENTS)
                __hip_atomic_store(&ctl->seg[z][gtid].count, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (gtid == 0) store_through(&ctl->low[z], PATH_INF);
            const int *frontier = buf.fr_col[step & 1u];
            int *next_frontier = buf.fr_col[(step + 1u) & 1u];

            // puts column k on the next frontier (through the workgroup's LDS list while it has room)
            auto push = [&](int k) {
                const unsigned slot = atomicAdd(&s_pushes, 1u);
                if (slot < (unsigned)PATH_PUSH_BUFFER) s_list[slot] = k;
                else {
                    const unsigned pos = atomicAdd(&ctl->seg[p][segment].count, 1u);
                    __hip_atomic_store(&next_frontier[(size_t)segment * s.len + pos], k, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                }
            };

            if (nf > 0) {
                swept = false;
                // one wavefront per (row, slice of columns): enough independent loads in flight to
                // stream the rows at memory speed whether the frontier holds one row or thousands
                constexpr int WAVES = PATH_THREADS / 64;
                const int total_waves = (int)G * WAVES, wave_id = wg * WAVES + (tid >> 6), lane = tid & 63;
                int slices = total_waves / nf;
                slices = slices < 1 ? 1 : (slices > PATH_MAX_SLICES ? PATH_MAX_SLICES : slices);
                const int span = (((s.len + slices - 1) / slices) + 255) & ~255;
                slices = (s.len + span - 1) / span;
                const int items = nf * slices;
                for (int it = wave_id; it < items; it += total_waves) {
                    const int e = it / slices, sl = it - e * slices;
                    int i, mine_col;
                    double dist, profit;
                    if (step == 1u) {
                        i = r0; mine_col = -1; dist = 0.0; profit = first_profit;
                    } else {
                        int g = 0;
                        while ((unsigned)e >= s_first[g + 1]) ++g;
                        mine_col = __hip_atomic_load(&frontier[(size_t)g * s.len + (e - s_first[g])], __ATOMIC_RELAXED,
                                                     __HIP_MEMORY_SCOPE_AGENT);
                        const unsigned long long lw = load_fresh_u64(&buf.label[mine_col]);
                        i = word_id(load_fresh_u64(&s.otherword[mine_col]));
                        dist = (double)(long long)(lw >> MF_ID_BITS);
                        // the row's profit: what it holds minus that column's dual
                        profit = s.Kd * (double)s.A[(size_t)i * s.pitch + mine_col] - s.other_dual[mine_col];
                        if (sl == 0 && lane == 0) {
                            store_through(&buf.expanded[mine_col], lw >> MF_ID_BITS);
                            __hip_atomic_store(&buf.held[i], mine_col, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            if (dist + profit < bound)                      // it may also give up and rest
                                atomicMin(&ctl->sink, ((unsigned long long)(long long)(dist + profit) << 21) |
                                                          (1ull << 20) | (unsigned long long)i);
                        }
                    }
                    const int32_t *row = s.A + (size_t)i * s.pitch;
                    const double base = dist + profit + s.eps;
                    const int from = sl * span, to = min(line_length(s, i), from + span);
#pragma unroll 2
                    for (int k = from + lane * 4; k < to; k += 256) {
                        const int4 w4 = *(const int4 *)(row + k);
                        const double2 p01 = *(const double2 *)(s.other_dual + k);
                        const double2 p23 = *(const double2 *)(s.other_dual + k + 2);
                        const int32_t w[4] = {w4.x, w4.y, w4.z, w4.w};
                        const double pr[4] = {p01.x, p01.y, p23.x, p23.y};
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const double cand = base - fma(s.Kd, (double)w[q], -pr[q]);
                            if (k + q < to && w[q] != MF_INFEASIBLE && cand < bound) {
                                const unsigned long long mine = ((unsigned long long)(long long)cand << MF_ID_BITS) |
                                                                (unsigned long long)i;
                                // a cached label is never below the true one (labels only fall during a
                                // search and the caches were emptied at its start): a safe first test
                                if (mine < buf.label[k + q] && atomicMin(&buf.label[k + q], mine) > mine && cand < limit &&
                                    atomicExch(&buf.stamp[k + q], step) != step) {
                                    if (word_id(load_fresh_u64(&s.otherword[k + q])) < 0)    // a column nobody holds ends a path
                                        atomicMin(&ctl->sink, (unsigned long long)(long long)cand << 21 |
                                                                  (unsigned long long)(k + q));
                                    else push(k + q);
                                }
                            }
                        }
                    }
                    if (sl == 0 && lane == 0) { ++my_scans; my_entries += (unsigned long long)line_length(s, i); }
                }
            } else {
                // ---- nothing on the frontier: look at every column ----
                swept = true;
                for (int first = 0; first < s.len; first += gsize) {
                    const int k = first + gtid;
                    if (k < s.len) {
                        const unsigned long long lw = load_fresh_u64(&buf.label[k]);
                        const unsigned long long ex = load_fresh_u64(&buf.expanded[k]);
                        const unsigned long long d_int = lw >> MF_ID_BITS;
                        const double d = (double)(long long)d_int;
                        if (lw != PATH_INF && d < bound && d_int < ex) {
                            if (d >= limit) atomicMin(&s_low, d_int);
                            else if (word_id(load_fresh_u64(&s.otherword[k])) < 0)
                                atomicMin(&s_sink, (d_int << 21) | (unsigned long long)k);
                            else push(k);
                        }
                    }
                }
            }
            // ---- hand the workgroup's pushes, sink and window candidates over ----
            __syncthreads();
            const unsigned pushed = min(s_pushes, (unsigned)PATH_PUSH_BUFFER);
            if (tid == 0) {
                s_base = pushed ? atomicAdd(&ctl->seg[p][segment].count, pushed) : 0u;
                if (s_sink != PATH_INF) atomicMin(&ctl->sink, s_sink);
                if (s_low != PATH_INF) atomicMin(&ctl->low[p], s_low);
            }
            __syncthreads();
            for (unsigned t = tid; t < pushed; t += PATH_THREADS)
                __hip_atomic_store(&next_frontier[(size_t)segment * s.len + s_base + t], s_list[t], __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            ++my_steps;
            if (!grid_barrier(ctl, G, generation, spin_limit)) { alive = false; break; }
        }
        if (!alive) break;

        // ---- make the shortest path tight, then re-assign along it ----
        // Workgroup 0 does both on its own, and only behind one more barrier: passing it proves
        // that every workgroup finished its share of the search, so no wait that runs out can
        // leave the duals half-updated or updated from incomplete labels.
        if (!grid_barrier(ctl, G, generation, spin_limit)) { alive = false; break; }      // r0 not placed: handed back below
        if (wg == 0) {
            const unsigned long long sink = load_fresh_u64(&ctl->sink);
            const unsigned long long d_star = sink >> 21;
            for (int k = tid; k < s.len; k += PATH_THREADS) {
                const unsigned long long lw = load_fresh_u64(&buf.label[k]);
                if (lw == PATH_INF) continue;
                const unsigned long long d_int = lw >> MF_ID_BITS;
                if (d_int < d_star) {
                    const unsigned long long cw = load_fresh_u64(&s.otherword[k]);
                    store_dual(s, k, word_dual(cw) + (double)(long long)(d_star - d_int), (int)(cw & MF_ID_MASK));
                }
            }
            __threadfence();
            __syncthreads();
            if (tid == 0) {
                const int id = (int)(sink & 0xfffffull);
                int k = ((sink >> 20) & 1ull) ? (id == r0 ? -1 : __hip_atomic_load(&buf.held[id], __ATOMIC_RELAXED,
                                                                                     __HIP_MEMORY_SCOPE_AGENT))
                                              : id;
                int guard = 0;
                while (k >= 0 && guard++ <= rows) {
                    const int i = (int)(load_fresh_u64(&buf.label[k]) & MF_ID_MASK);
                    const int before = __hip_atomic_load(&buf.held[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    store_dual(s, k, word_dual(load_fresh_u64(&s.otherword[k])) + s.eps, i + 1);
                    k = (i == r0) ? -1 : before;
                }
                atomicAdd(&ctl->steps, my_steps);
            }
        }
        if ((tid & 63) == 0 && my_scans) { atomicAdd(&ctl->scans, my_scans); atomicAdd(&ctl->entries, my_entries); }
        if (!grid_barrier(ctl, G, generation, spin_limit)) { alive = false; ++item; break; }   // r0 is placed
    }
    if (gtid == 0) {
        for (int rest = item; rest < count; ++rest)                         // whoever was not served bids again
            out_list[atomicAdd(&stats->cnt[(ring + 1) & 3], 1)] = list[rest];
        if (!alive) atomicExch(&stats->team_abort, 2);
        const unsigned long long steps = load_fresh_u64(&ctl->steps), scans = load_fresh_u64(&ctl->scans);
        stats->launch_max = steps;
        stats->bids += scans;
        stats->chain_bids += scans;
        stats->path_steps += steps;
        stats->path_scans += scans;
        stats->bytes += load_fresh_u64(&ctl->entries) * 4ull;
    }
}

// Start of an epsilon phase: drop the assignment, keep the duals, all rows bid.
__global__ void reset_kernel(int n, int m, const double *__restrict__ price,
                             unsigned long long *colword, int *row2col, int *col2row, int *list,
                             mf_device_stats *stats)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) { row2col[i] = -1; list[i] = i; }
    if (i < m) { col2row[i] = -1; colword[i] = pack_word(price[i], 0); }
    if (i == 0) { stats->cnt[0] = n; stats->cnt[1] = 0; stats->cnt[2] = 0; stats->cnt[3] = 0; }
}

// After the forward rounds the price words name every column's holder, and a
// row's profit is whatever its column leaves it (0 for a row that rests).
__global__ void forward_done_rows_kernel(int n, double *__restrict__ profit,
                                         unsigned long long *roword, int *row2col)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) { row2col[i] = -1; profit[i] = 0.0; roword[i] = 0ull; }
}

__global__ void forward_done_cols_kernel(int m, const int32_t *__restrict__ W, int64_t ldw, double Kd,
                                         const unsigned long long *__restrict__ colword,
                                         const double *__restrict__ price, double *__restrict__ profit,
                                         unsigned long long *roword, int *row2col, int *col2row,
                                         int *list, mf_device_stats *stats)
{
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= m) return;
    const unsigned long long word = colword[j];
    const int r = word_id(word);
    col2row[j] = r;
    if (r >= 0) {
        const double pi = Kd * (double)W[(size_t)r * ldw + j] - word_dual(word);
        row2col[r] = j;
        profit[r] = pi;
        roword[r] = pack_word(pi, j + 1);
    } else if (price[j] > 0.0) {
        list[atomicAdd(&stats->cnt[0], 1)] = j;    // an unassigned column that still carries a price must bid
    }
}

// A forward side that was stopped early leaves rows that still wanted to bid.  Before the other
// side runs, each gets the profit that covers all of its pairs at the current prices (its best
// value, or 0), held by nobody: then pi_i + p_j >= K W_ij - eps holds on every feasible pair
// again, which the bids and searches of the other side rely on.
__global__ __launch_bounds__(BID_THREADS) void settle_unplaced_kernel(
    const int32_t *__restrict__ W, int64_t ldw, int n, int m, const double *__restrict__ price,
    const int *__restrict__ row2col, double Kd, double *__restrict__ profit, unsigned long long *roword,
    const int *__restrict__ line_len)
{
    __shared__ Top2 red[BID_THREADS / 64];
    for (int i = blockIdx.x; i < n; i += gridDim.x) {
        if (row2col[i] >= 0) continue;                               // block-uniform
        const int len = line_len ? min(line_len[i], m) : m;
        const Top2 t = block_scan<BID_THREADS>(W + (size_t)i * ldw, price, len, Kd, false, red, 0, 0);
        if (threadIdx.x == 0) {
            const double pi = fmax(t.b1, 0.0);
            profit[i] = pi;
            roword[i] = pack_word(pi, 0);
        }
        __syncthreads();
    }
}

// After the reverse rounds the profit words name every row's holder; a column's
// price is whatever its row leaves it (0 for a column that rests).
__global__ void reverse_done_cols_kernel(int m, double *__restrict__ price, int *col2row)
{
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j < m) { col2row[j] = -1; price[j] = 0.0; }
}

__global__ void reverse_done_rows_kernel(int n, const int32_t *__restrict__ W, int64_t ldw, double Kd,
                                         const unsigned long long *__restrict__ roword,
                                         double *__restrict__ price, int *row2col, int *col2row)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const unsigned long long word = roword[i];
    const int c = word_id(word);
    row2col[i] = c;
    if (c >= 0) {
        col2row[c] = i;
        price[c] = Kd * (double)W[(size_t)i * ldw + c] - word_dual(word);
    }
}

__global__ void clear_counts_kernel(mf_device_stats *stats)
{
    stats->cnt[0] = 0; stats->cnt[1] = 0; stats->cnt[2] = 0; stats->cnt[3] = 0;
}

// W^T (for the reverse rounds' coalesced column scans) and the largest weight.
// 64 x 64 tiles through LDS, 16-byte loads and stores on both sides.  wide: both
// matrices allow 16-byte accesses (pitches multiples of four, bases aligned).
__global__ __launch_bounds__(256) void transpose_kernel(const int32_t *__restrict__ W, int n, int m, int64_t ldw,
                                                        int32_t *__restrict__ WT, int64_t ldt,
                                                        mf_device_stats *stats)
{
    __shared__ int32_t tile[64][65];
    const int bx = blockIdx.x * 64, by = blockIdx.y * 64;
    const int q4 = (threadIdx.x & 15) * 4, rr = threadIdx.x >> 4;       // 16 threads per line, 16 lines per pass
    int mx = 0;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int r = p * 16 + rr, i = by + r, j = bx + q4;
        int32_t w[4] = {MF_INFEASIBLE, MF_INFEASIBLE, MF_INFEASIBLE, MF_INFEASIBLE};
        if (i < n) {
            const int32_t *src = W + (size_t)i * ldw + j;
            if (j + 3 < m) { const int4 v = *(const int4 *)src; w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w; }
            else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (j + e < m) w[e] = src[e];
            }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) { tile[r][q4 + e] = w[e]; mx = max(mx, w[e]); }
    }
    __syncthreads();
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int r = p * 16 + rr, j = bx + r, i = by + q4;
        if (j < m && i < n) {
            int32_t *dst = WT + (size_t)j * ldt + i;
            if (i + 3 < n) *(int4 *)dst = make_int4(tile[q4][r], tile[q4 + 1][r], tile[q4 + 2][r], tile[q4 + 3][r]);
            else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (i + e < n) dst[e] = tile[q4 + e][r];
            }
        }
    }
    for (int off = 32; off >= 1; off >>= 1) mx = max(mx, __shfl_xor(mx, off));
    // the maximum only grows, so an outdated (smaller) cached value at worst costs a redundant atomic
    if ((threadIdx.x & 63) == 0 && mx > stats->max_weight) atomicMax(&stats->max_weight, mx);
}

// The largest weight alone (it sets the first epsilon), for solves that may never need W^T.
__global__ __launch_bounds__(256) void max_weight_kernel(const int32_t *__restrict__ W, int n, int m, int64_t ldw,
                                                         mf_device_stats *stats)
{
    int mx = 0;
    for (int i = blockIdx.y; i < n; i += gridDim.y) {
        const int32_t *row = W + (size_t)i * ldw;
        for (int j = (blockIdx.x * 256 + threadIdx.x) * 4; j < m; j += gridDim.x * 1024) {
            const int4 v = *(const int4 *)(row + j);            // the pitch is a multiple of four
            mx = max(mx, v.x);
            if (j + 1 < m) mx = max(mx, v.y);
            if (j + 2 < m) mx = max(mx, v.z);
            if (j + 3 < m) mx = max(mx, v.w);
        }
    }
    for (int off = 32; off >= 1; off >>= 1) mx = max(mx, __shfl_xor(mx, off));
    if ((threadIdx.x & 63) == 0 && mx > stats->max_weight) atomicMax(&stats->max_weight, mx);
}

// Duals handed to the caller: v_j = p_j and the tightest row dual the prices
// allow, u_i = max(0, max_j (K W_ij - p_j)).
// RB rows per workgroup share every load of the prices (8 bytes per entry against 4 for a
// weight), as in the bulk bidding rounds.
template <int NT, int RB>
__global__ __launch_bounds__(NT) void duals_kernel(
    const int32_t *__restrict__ W, int64_t ldw, int n, int m, const double *__restrict__ price,
    const int *__restrict__ row2col, double Kd, int32_t *__restrict__ out_row2col,
    int64_t *__restrict__ u, int64_t *__restrict__ v, const int *__restrict__ line_len)
{
    __shared__ Top2 red[RB + RB * (NT / 64)];
    for (int i0 = blockIdx.x * RB; i0 < n; i0 += gridDim.x * RB) {
        const int32_t *rows[RB];
        int salt[RB];
        int len = 0;                                        // the group scans as far as its longest row
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            const int i = min(i0 + r, n - 1);               // a short last group repeats its last row
            rows[r] = W + (size_t)i * ldw;
            salt[r] = 0;
            len = max(len, line_len ? min(line_len[i], m) : m);
        }
        block_scan_rows<NT, RB>(rows, salt, price, len, Kd, red);
        if (threadIdx.x < RB && i0 + (int)threadIdx.x < n) {
            const int i = i0 + threadIdx.x;
            u[i] = (int64_t)fmax(red[threadIdx.x].b1, 0.0);
            out_row2col[i] = row2col[i];
        }
    }
    for (int j = blockIdx.x * blockDim.x + threadIdx.x; j < m; j += gridDim.x * blockDim.x)
        v[j] = (int64_t)price[j];
}

// The proof of optimality, evaluated for arbitrary caller-supplied integers:
// matching valid, duals non-negative, every feasible pair covered
// (min reduced cost), primal and dual totals.
// K32: K fits a signed 32-bit integer, so K*w is one 32 x 32 -> 64-bit multiply-add.
// A workgroup takes CERT_ROWS rows at a time: each column dual (8 bytes, against 4 for a weight)
// is loaded once for all of them.
constexpr int CERT_ROWS = 4;

template <bool K32>
__global__ __launch_bounds__(BID_THREADS) void certificate_kernel(
    const int32_t *__restrict__ W, int64_t ldw, int n, int m, const int32_t *__restrict__ row2col,
    const int64_t *__restrict__ u, const int64_t *__restrict__ v, long long K, int *colmark,
    mf_cert_out *out)
{
    __shared__ long long red[BID_THREADS / 64];
    constexpr int UN = 2;               // column groups of four in flight per thread
    long long dual_part = 0, primal_part = 0;
    int flags = 0, matched = 0;
    long long min_rc = INT64_MAX;
    const int k32 = (int)K;
    for (int i0 = blockIdx.x * CERT_ROWS; i0 < n; i0 += gridDim.x * CERT_ROWS) {
        long long ui[CERT_ROWS];
        const int32_t *rows[CERT_ROWS];
#pragma unroll
        for (int r = 0; r < CERT_ROWS; ++r) {
            const int i = min(i0 + r, n - 1);               // a short last group repeats its last row
            ui[r] = u[i];
            rows[r] = W + (size_t)i * ldw;
        }
        for (int j0 = threadIdx.x * 4; j0 < m; j0 += BID_THREADS * 4 * UN) {
            // every load is issued before any comparison: the column duals whatever the weights
            // turn out to be (index clamped into the array), the weights of all the rows
            long long vj[UN][4];
            int4 w4[UN][CERT_ROWS];
#pragma unroll
            for (int q = 0; q < UN; ++q) {
                const int j = j0 + q * BID_THREADS * 4;
#pragma unroll
                for (int e = 0; e < 4; ++e) vj[q][e] = v[min(j + e, m - 1)];
#pragma unroll
                for (int r = 0; r < CERT_ROWS; ++r)
                    w4[q][r] = j < m ? *(const int4 *)(rows[r] + j)
                                     : make_int4(MF_INFEASIBLE, MF_INFEASIBLE, MF_INFEASIBLE, MF_INFEASIBLE);
            }
#pragma unroll
            for (int q = 0; q < UN; ++q) {
                const int j = j0 + q * BID_THREADS * 4;
#pragma unroll
                for (int r = 0; r < CERT_ROWS; ++r) {
                    const int32_t w[4] = {w4[q][r].x, w4[q][r].y, w4[q][r].z, w4[q][r].w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const long long cover = ui[r] + vj[q][e];
                        const long long rc = K32 ? cover - (long long)w[e] * (long long)k32 : cover - K * (long long)w[e];
                        const bool counts = j + e < m && w[e] != MF_INFEASIBLE;
                        min_rc = counts && rc < min_rc ? rc : min_rc;
                    }
                }
            }
        }
        if (threadIdx.x < CERT_ROWS && i0 + (int)threadIdx.x < n) {          // one thread per row of the group
            const int i = i0 + threadIdx.x;
            const long long mine = u[i];
            if (mine < 0) flags |= 4;
            dual_part += mine;
            const int j = row2col[i];
            if (j != -1) {
                if (j < 0 || j >= m) flags |= 1;
                else {
                    if (atomicAdd(&colmark[j], 1) != 0) flags |= 1;
                    const int32_t w = W[(size_t)i * ldw + j];
                    if (w == MF_INFEASIBLE || w < 0) flags |= 2;
                    else { primal_part += w; matched += 1; }
                }
            }
        }
    }
    for (int j = blockIdx.x * blockDim.x + threadIdx.x; j < m; j += gridDim.x * blockDim.x) {
        const long long vj = v[j];
        if (vj < 0) flags |= 4;
        dual_part += vj;
    }
    // block reductions
    for (int off = 32; off >= 1; off >>= 1) {
        const long long o = __shfl_xor(min_rc, off);
        min_rc = o < min_rc ? o : min_rc;
        dual_part += __shfl_xor(dual_part, off);
        primal_part += __shfl_xor(primal_part, off);
        matched += __shfl_xor(matched, off);
        flags |= __shfl_xor(flags, off);
    }
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (lane == 0) red[wave] = min_rc;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int wv = 1; wv < BID_THREADS / 64; ++wv) min_rc = red[wv] < min_rc ? red[wv] : min_rc;
        atomicMin(&out->min_rc, min_rc);
        if (primal_part) atomicAdd((unsigned long long *)&out->primal, (unsigned long long)primal_part);
        if (matched) atomicAdd(&out->matched, matched);
    }
    if (lane == 0) {
        if (dual_part) atomicAdd((unsigned long long *)&out->dual, (unsigned long long)dual_part);
        if (flags) atomicOr(&out->flags, flags);
    }
}

__global__ void fill_int_kernel(int *p, int count, int value)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = value;
}

// Results of a solve that ran in other coordinates (rows and columns in memory order, and/or
// the transposed problem) handed to the caller: internal row k is the caller's row_ids[k]
// (k itself without a map), likewise columns; with `flipped` the internal rows are the caller's
// columns.  d_row2col was filled with -1 before.
__global__ void map_back_kernel(int rn, int rm, const int32_t *__restrict__ r2c, const int64_t *__restrict__ u,
                                const int64_t *__restrict__ v, const int32_t *__restrict__ row_ids,
                                const int32_t *__restrict__ col_ids, int flipped, int32_t *d_row2col,
                                int64_t *d_u, int64_t *d_v)
{
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k < rn) {
        const int rid = row_ids ? row_ids[k] : k;
        const int c = r2c[k];
        const int cid = c < 0 ? -1 : (col_ids ? col_ids[c] : c);
        if (!flipped) { d_row2col[rid] = cid; d_u[rid] = u[k]; }
        else { d_v[rid] = u[k]; if (cid >= 0) d_row2col[cid] = rid; }
    }
    if (k < rm) {
        const int cid = col_ids ? col_ids[k] : k;
        if (!flipped) d_v[cid] = v[k]; else d_u[cid] = v[k];
    }
}

__global__ void init_cert_kernel(mf_cert_out *out)
{
    out->primal = 0; out->dual = 0; out->min_rc = INT64_MAX; out->matched = 0; out->flags = 0;
}

__global__ void zero_listed_kernel(double *price, const int32_t *__restrict__ which, int count, int m)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count && which[i] >= 0 && which[i] < m) price[which[i]] = 0.0;
}

__global__ void init_solver_kernel(int n, int m, double *price, double *profit, mf_device_stats *stats,
                                   int keep_prices)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n + 4) profit[i] = 0.0;
    if (i < m + 4 && (!keep_prices || i >= m)) price[i] = 0.0;
    if (i == 0) {
        stats->rounds = 0; stats->bids = 0; stats->bytes = 0; stats->head = 0;
        stats->chain_bids = 0; stats->chain_depth = 0; stats->launch_max = 0; stats->chain_retries = 0; stats->team_bids = 0; stats->path_steps = 0; stats->path_scans = 0; stats->team_abort = 0; stats->active = 0; stats->max_weight = 0;
        stats->cnt[0] = 0; stats->cnt[1] = 0; stats->cnt[2] = 0; stats->cnt[3] = 0;
    }
}

template <int NT, int RB>
void launch_round_shape(mf_ctx *ctx, const SideArgs &s, int count, int ring)
{
    int grid = (count + RB - 1) / RB;
    if (grid > MAX_GRID) grid = MAX_GRID;
    hipLaunchKernelGGL((round_kernel<NT, RB>), dim3(grid), dim3(NT), 0, ctx->stream, s, ctx->list[ring & 1],
                       ctx->list[(ring + 1) & 1], ctx->stats, ring);
}

void launch_round(mf_ctx *ctx, const SideArgs &s, int count, int ring)
{
    switch (count >= 2048 ? ctx->bulk_shape : 0) {      // small rounds: one line per workgroup
    case 1: launch_round_shape<64, 4>(ctx, s, count, ring); break;
    case 2: launch_round_shape<64, 2>(ctx, s, count, ring); break;
    case 3: launch_round_shape<128, 4>(ctx, s, count, ring); break;
    case 4: launch_round_shape<256, 4>(ctx, s, count, ring); break;
    default: launch_round_shape<256, 1>(ctx, s, count, ring); break;
    }
}

// Runs one side until at most `stop_at` bidders are left (0: until nobody is left to bid).
// list[0] / cnt[0] hold the first bidders (`count` of them).  Returns MF_OK or an error;
// *left_over is the number of bidders still unplaced.
int run_side(mf_ctx *ctx, const SideArgs &s, int count, bool time_first, int stop_at, int *left_over)
{
    int ring = 0;
    // Short chains are cheapest followed step by step; a chain that is still going after
    // `path_after` steps is ended by shortest-path searches instead.
    long long team_steps = 0;
    *left_over = count;
    while (count > stop_at) {
        bool timed = false, counted_teams = false;
        const unsigned long long bytes_before = ctx->h_stats->bytes;
        const bool paths_ok = ctx->path_max > 0 && !ctx->path_off && ctx->n_cus > 0;
        const bool teams_ok = ctx->team_max > 0 && !ctx->team_off;
        const int cus = ctx->n_cus > 0 ? ctx->n_cus : 256;
        // chains at or below which teams take over from one workgroup per chain
        // (lines short enough for one compute unit to read in a couple of microseconds gain nothing
        // from being split: there the teams wait for the last few chains)
        int team_from = (ctx->team_wide > ctx->team_max && s.typical_len >= TEAM_WIDE_MIN_LINE) ? ctx->team_wide : ctx->team_max;
        if (team_from > TEAM_MAX) team_from = TEAM_MAX;
        if (team_from * 2 > cus) team_from = cus / 2;
        const long long left = ctx->max_rounds - (long long)ctx->h_stats->bids;
        if (left <= 0) return MF_ERR_NOT_CONVERGED;
        if (count > ctx->tail_max) {
            const int batch = (count > 4096 || time_first) ? 1 : 3;     // the timed round stands alone
            for (int r = 0; r < batch; ++r) {
                if (time_first && r == 0) { MF_HIP(hipEventRecord(ctx->ev[6], ctx->stream)); timed = true; }
                launch_round(ctx, s, count, ring);
                if (time_first && r == 0) MF_HIP(hipEventRecord(ctx->ev[7], ctx->stream));
                ++ring;
            }
        } else if (paths_ok && count <= ctx->path_max && (team_steps >= ctx->path_after || !teams_ok)) {
            // few enough bidders, and chains long enough, to place each bidder by a shortest-path
            // search over the whole device
            PathBuffers buf{ctx->path_label, ctx->path_expanded, ctx->path_stamp,
                            {ctx->path_frontier[0], ctx->path_frontier[1]}, ctx->path_held};
            hipLaunchKernelGGL(path_begin_kernel, dim3(1), dim3(1), 0, ctx->stream, ctx->stats,
                               (PathCtl *)ctx->path_ctl, ring);
            const int path_wgs = ctx->path_grid > 0 && ctx->path_grid < ctx->n_cus ? ctx->path_grid : ctx->n_cus;
            hipLaunchKernelGGL(path_kernel, dim3(path_wgs), dim3(PATH_THREADS), 0, ctx->stream, s,
                               ctx->list[ring & 1], ctx->list[(ring + 1) & 1], ctx->stats, (PathCtl *)ctx->path_ctl,
                               buf, ring, ctx->max_n > ctx->max_m ? ctx->max_n : ctx->max_m,
                               (double)ctx->path_width * s.eps, ctx->path_spin_limit);
            ++ring;
        } else if (!teams_ok || count > team_from) {
            const int grid = count < ctx->chain_grid ? count : ctx->chain_grid;
            const int hand_back = teams_ok ? team_from : (paths_ok ? ctx->path_max : -1);
            hipLaunchKernelGGL(chain_begin_kernel, dim3(1), dim3(1), 0, ctx->stream, ctx->stats, ring, grid);
            hipLaunchKernelGGL(chain_kernel, dim3(grid), dim3(CHAIN_THREADS), 0, ctx->stream, s,
                               ctx->list[ring & 1], ctx->list[(ring + 1) & 1], ctx->stats, ring,
                               left / grid + 1, hand_back);
            ++ring;
        } else {
            // every remaining chain gets a team: the fewer chains, the more workgroups on each
            const int teams = count;
            int size = cus / teams;
            size = size < 2 ? 2 : (size > ctx->team_size ? ctx->team_size : size);
            const bool before_paths = paths_ok && count <= ctx->path_max;
            long long team_cap = left / teams + 1;
            // many chains: stop after a while to regroup the ones still going into larger teams;
            // few: until the searches' turn
            const long long stop_after = before_paths ? ctx->path_after - team_steps
                                                      : (count > ctx->team_max ? ctx->team_regroup : team_cap);
            if (stop_after < team_cap) team_cap = stop_after;
            counted_teams = before_paths;
            hipLaunchKernelGGL(team_begin_kernel, dim3(1), dim3(64), 0, ctx->stream, ctx->stats,
                               (TeamCtl *)ctx->team_ctl, ring);
            const dim3 grid(teams * size);
            using TeamKernel = void (*)(SideArgs, const int *, int *, mf_device_stats *, TeamCtl *, int, long long, int);
            const int threads = ctx->team_threads;
            const TeamKernel kernel = threads == 64 ? team_kernel<64> : threads == 128 ? team_kernel<128>
                                    : threads == 256 ? team_kernel<256> : threads == 512 ? team_kernel<512>
                                                                                         : team_kernel<1024>;
            hipLaunchKernelGGL(kernel, grid, dim3(threads == 64 || threads == 128 || threads == 256 || threads == 512 ? threads : 1024),
                               0, ctx->stream, s, ctx->list[ring & 1], ctx->list[(ring + 1) & 1], ctx->stats,
                               (TeamCtl *)ctx->team_ctl, ring, team_cap, size);
            ++ring;
        }
        MF_HIP(hipGetLastError());
        MF_HIP(hipMemcpyAsync(ctx->h_stats, ctx->stats, sizeof(mf_device_stats), hipMemcpyDeviceToHost, ctx->stream));
        MF_HIP(hipStreamSynchronize(ctx->stream));
        if (timed) {
            float ms = 0.0f;
            MF_HIP(hipEventElapsedTime(&ms, ctx->ev[6], ctx->ev[7]));
            ctx->timings[T_BID_BULK] += ms;
            ctx->timings[T_BID_BULK_LAUNCHES] += 1.0f;
            ctx->timings[T_BID_BULK_BYTES] += (float)((double)(ctx->h_stats->bytes - bytes_before));
        }
        time_first = false;
        count = ctx->h_stats->cnt[ring & 3];
        if (counted_teams) team_steps += (long long)ctx->h_stats->launch_max;     // the longest any leader went
        if (ctx->h_stats->team_abort == 1) ctx->team_off = true;   // a bounded wait ran out: one workgroup per chain from now on
        if (ctx->h_stats->team_abort == 2) ctx->path_off = true;   // ... or no more shortest-path searches
        *left_over = count;
    }
    return MF_OK;
}

}  // namespace

int mf_run_certificate(mf_ctx *ctx, const int32_t *d_W, int n, int m, int64_t ldw,
                       const int32_t *d_row2col, const int64_t *d_u, const int64_t *d_v,
                       int64_t K, mf_result *h_res)
{
    hipLaunchKernelGGL(init_cert_kernel, dim3(1), dim3(1), 0, ctx->stream, ctx->cert);
    hipLaunchKernelGGL(fill_int_kernel, dim3((m + 255) / 256), dim3(256), 0, ctx->stream, ctx->colmark, m, 0);
    const int groups = (n + CERT_ROWS - 1) / CERT_ROWS, grid = groups < MAX_GRID ? groups : MAX_GRID;
    hipLaunchKernelGGL(K >= INT32_MIN && K <= INT32_MAX ? certificate_kernel<true> : certificate_kernel<false>,
                       dim3(grid), dim3(BID_THREADS), 0, ctx->stream, d_W, ldw, n, m,
                       d_row2col, d_u, d_v, (long long)K, ctx->colmark, ctx->cert);
    MF_HIP(hipGetLastError());
    MF_HIP(hipMemcpyAsync(ctx->h_cert, ctx->cert, sizeof(mf_cert_out), hipMemcpyDeviceToHost, ctx->stream));
    MF_HIP(hipStreamSynchronize(ctx->stream));
    const mf_cert_out &c = *ctx->h_cert;
    h_res->primal = c.primal;
    h_res->dual = c.dual;
    h_res->K = K;
    h_res->min_reduced_cost = c.min_rc == INT64_MAX ? 0 : c.min_rc;
    h_res->matched = c.matched;
    const long long gap = c.dual - K * c.primal;
    h_res->cert_ok = (c.flags == 0 && h_res->min_reduced_cost >= 0 && gap >= 0 && gap < K) ? 1 : 0;
    return MF_OK;
}

// `warm`: start from the prices the previous solve of the same shape left in
// the context (those of the columns listed in d_reset_cols set to 0) and from a
// small epsilon.  Any non-negative starting prices are valid - every phase
// drops the assignment and re-establishes its invariants - so this changes
// only how much work the phases have to do.
int mf_run_solver(mf_ctx *ctx, const int32_t *d_W, int n, int m, int64_t ldw,
                  int32_t *d_row2col, int64_t *d_u, int64_t *d_v, mf_result *h_res,
                  bool warm, const int32_t *d_reset_cols, int n_reset_cols, bool may_use_staged)
{
    // When the matrix was just scored here, the context still holds it with rows and columns in
    // order of memory fraction, where the pairs that can share are a prefix of every row and of
    // every column: the auction then runs on that copy and reads only the prefixes; the
    // certificate below is still evaluated on the caller's matrix, in the caller's coordinates.
    const bool candidate = may_use_staged && ctx->fit_prefix && ctx->staged_n == n && ctx->staged_m == m;
    const bool flip = n > m;
    warm = warm && !flip && !candidate && ctx->warm_n == n && ctx->warm_m == m;
    ctx->warm_n = ctx->warm_m = 0;
    const int64_t ldt = ((int64_t)n + 3) & ~3ll;
    const int rn = flip ? m : n, rm = flip ? n : m;
    const long long K = (long long)rn + 1;
    const double Kd = (double)K;
    const int nm = rm;

    MF_HIP(hipEventRecord(ctx->ev[3], ctx->stream));
    {
        // the largest weight sets the first epsilon
        const int chunks = (m + 4095) / 4096 < 4 ? (m + 4095) / 4096 : 4;
        hipLaunchKernelGGL(init_solver_kernel, dim3((nm + 4 + 255) / 256), dim3(256), 0, ctx->stream, rn, rm,
                           ctx->price, ctx->profit, ctx->stats, warm ? 1 : 0);
        hipLaunchKernelGGL(max_weight_kernel, dim3(chunks, n < 1024 ? n : 1024), dim3(256), 0, ctx->stream, d_W, n, m,
                           ldw, ctx->stats);
        MF_HIP(hipGetLastError());
    }
    *ctx->h_feasible_pairs = ~0ull;
    if (candidate)
        MF_HIP(hipMemcpyAsync(ctx->h_feasible_pairs, ctx->feasible_pairs, sizeof(unsigned long long),
                              hipMemcpyDeviceToHost, ctx->stream));
    MF_HIP(hipMemcpyAsync(ctx->h_stats, ctx->stats, sizeof(mf_device_stats), hipMemcpyDeviceToHost, ctx->stream));
    MF_HIP(hipStreamSynchronize(ctx->stream));
    const long long cmax = K * (long long)ctx->h_stats->max_weight;
    if (cmax >= MF_MAX_DUAL) return MF_ERR_RANGE;
    // ... worth it when most of the matrix can be left unread
    const bool staged = candidate && (double)*ctx->h_feasible_pairs * 100.0 < (double)ctx->fit_prefix_below * (double)n * (double)m;
    const int32_t *M = staged ? ctx->staged : d_W;
    const int64_t ldm = staged ? (((int64_t)m + 3) & ~3ll) : ldw;
    const int *len_rows = staged ? ctx->fit_len_on : nullptr, *len_cols = staged ? ctx->fit_len_off : nullptr;
    const int32_t *A = flip ? ctx->wt : M;
    const int64_t lda = flip ? ldt : ldm;
    const int32_t *At = flip ? M : ctx->wt;
    const int64_t ldat = flip ? ldm : ldt;
    if (warm && n_reset_cols > 0)
        hipLaunchKernelGGL(zero_listed_kernel, dim3((n_reset_cols + 255) / 256), dim3(256), 0, ctx->stream,
                           ctx->price, d_reset_cols, n_reset_cols, m);
    // W^T serves the second side of a phase (unassigned columns that still carry a price), which a
    // square, fully matched problem may never enter: it is made when first needed, unless the
    // transposed problem is the one being solved
    bool have_transpose = false;
    auto make_transpose = [&]() {
        hipLaunchKernelGGL(transpose_kernel, dim3((m + 63) / 64, (n + 63) / 64), dim3(256), 0, ctx->stream,
                           M, n, m, ldm, ctx->wt, ldt, ctx->stats);
        have_transpose = true;
    };
    if (flip) make_transpose();
    MF_HIP(hipGetLastError());
    MF_HIP(hipEventRecord(ctx->ev[4], ctx->stream));
    MF_HIP(hipStreamSynchronize(ctx->stream));
    {
        float ms = 0.0f;
        MF_HIP(hipEventElapsedTime(&ms, ctx->ev[3], ctx->ev[4]));
        ctx->timings[T_TRANSPOSE] = ms;
    }

    // with per-line lengths a scan reads, on average, the pairs that can share divided by the lines
    const double feasible = staged ? (double)*ctx->h_feasible_pairs : (double)n * (double)m;
    SideArgs fwd{A, (long long)lda, rm, ctx->price, ctx->colword, 0.0, Kd, flip ? len_cols : len_rows,
                 (int)(feasible / (double)rn)};
    SideArgs rev{At, (long long)ldat, rn, ctx->profit, ctx->roword, 0.0, Kd, flip ? len_rows : len_cols,
                 (int)(feasible / (double)rm)};

    long long eps = cmax / ctx->theta;
    if (warm && ctx->warm_eps_units * K < eps) eps = ctx->warm_eps_units * K;
    if (eps < 1) eps = 1;
    int phases = 0;
    for (;;) {
        ++phases;
        fwd.eps = rev.eps = (double)eps;
        hipLaunchKernelGGL(reset_kernel, dim3((nm + 255) / 256), dim3(256), 0, ctx->stream, rn, rm, ctx->price,
                           ctx->colword, ctx->row2col, ctx->col2row, ctx->list[0], ctx->stats);
        // A phase at a coarse epsilon only prepares prices for the later ones (each drops the
        // assignment anyway), so either of its sides may end while a few bidders are still
        // unplaced: their long chains of dependent bids, and the searches that would end them, are
        // then never run at that epsilon.  The last phase_keep phases run to the end: the first of
        // them settles what was left open, the last one is what makes the result exact.  The
        // second side runs whenever more columns than that are unused and still priced - skipping
        // it would carry their prices into ever finer phases, where taking them off costs far more.
        int left_over = 0, phases_after = 0;
        for (long long e = eps; e > 1; ++phases_after) { e /= ctx->theta; if (e < 1) e = 1; }
        // The coarser the phase, the more may be left (phase_growth times more per phase), but
        // never more than one bidder in 64: small problems complete every phase.
        long long stop_ll = 0;
        if (phases_after >= ctx->phase_keep) {
            stop_ll = ctx->phase_stop;
            for (int k = ctx->phase_keep; k < phases_after && stop_ll < rn; ++k) stop_ll *= ctx->phase_growth;
            // the searches are for the phases that have to finish: a coarse one ends at the latest
            // where they would take over
            if (ctx->path_max > 0 && !ctx->path_off && stop_ll > 0 && stop_ll < ctx->path_max) stop_ll = ctx->path_max;
            if (stop_ll > rn / 64) stop_ll = rn / 64;
        }
        const int stop_at = (int)stop_ll;
        int rc = run_side(ctx, fwd, rn, true, stop_at, &left_over);
        if (rc != MF_OK) return rc;
        // who holds what after the forward rounds; unassigned priced columns go to list[0]
        hipLaunchKernelGGL(clear_counts_kernel, dim3(1), dim3(1), 0, ctx->stream, ctx->stats);
        hipLaunchKernelGGL(forward_done_rows_kernel, dim3((rn + 255) / 256), dim3(256), 0, ctx->stream, rn,
                           ctx->profit, ctx->roword, ctx->row2col);
        hipLaunchKernelGGL(forward_done_cols_kernel, dim3((rm + 255) / 256), dim3(256), 0, ctx->stream, rm,
                           A, lda, Kd, ctx->colword, ctx->price, ctx->profit, ctx->roword, ctx->row2col,
                           ctx->col2row, ctx->list[0], ctx->stats);
        if (left_over > 0)
            hipLaunchKernelGGL(settle_unplaced_kernel, dim3(rn < MAX_GRID ? rn : MAX_GRID), dim3(BID_THREADS), 0,
                               ctx->stream, A, lda, rn, rm, ctx->price, ctx->row2col, Kd, ctx->profit, ctx->roword,
                               fwd.line_len);
        MF_HIP(hipGetLastError());
        MF_HIP(hipMemcpyAsync(ctx->h_stats, ctx->stats, sizeof(mf_device_stats), hipMemcpyDeviceToHost, ctx->stream));
        MF_HIP(hipStreamSynchronize(ctx->stream));
        const int rev_count = ctx->h_stats->cnt[0];
        if (rev_count > stop_at) {
            if (!have_transpose) make_transpose();
            rc = run_side(ctx, rev, rev_count, false, stop_at, &left_over);
            if (rc != MF_OK) return rc;
            hipLaunchKernelGGL(reverse_done_cols_kernel, dim3((rm + 255) / 256), dim3(256), 0, ctx->stream, rm,
                               ctx->price, ctx->col2row);
            hipLaunchKernelGGL(reverse_done_rows_kernel, dim3((rn + 255) / 256), dim3(256), 0, ctx->stream, rn,
                               A, lda, Kd, ctx->roword, ctx->price, ctx->row2col, ctx->col2row);
            MF_HIP(hipGetLastError());
        }
        if (eps == 1) break;
        eps /= ctx->theta;
        if (eps < 1) eps = 1;
    }
    MF_HIP(hipEventRecord(ctx->ev[4], ctx->stream));
    {
        const int groups = (rn + 3) / 4, grid = groups < MAX_GRID ? groups : MAX_GRID;
        if (!flip && !staged) {
            hipLaunchKernelGGL((duals_kernel<64, 4>), dim3(grid), dim3(64), 0, ctx->stream, A, lda, rn, rm,
                               ctx->price, ctx->row2col, Kd, d_row2col, d_u, d_v, fwd.line_len);
        } else {
            // the solve ran in other coordinates: results go through scratch (the searches' label
            // arrays are idle now) and are mapped to the caller's rows and columns
            int64_t *u_int = (int64_t *)ctx->path_label, *v_int = (int64_t *)ctx->path_expanded;
            hipLaunchKernelGGL((duals_kernel<64, 4>), dim3(grid), dim3(64), 0, ctx->stream, A, lda, rn, rm,
                               ctx->price, ctx->row2col, Kd, ctx->list[0], u_int, v_int, fwd.line_len);
            hipLaunchKernelGGL(fill_int_kernel, dim3((n + 255) / 256), dim3(256), 0, ctx->stream, d_row2col, n, -1);
            const int32_t *row_ids = staged ? (flip ? ctx->order_off : ctx->order_on) : nullptr;
            const int32_t *col_ids = staged ? (flip ? ctx->order_on : ctx->order_off) : nullptr;
            hipLaunchKernelGGL(map_back_kernel, dim3((nm + 255) / 256), dim3(256), 0, ctx->stream, rn, rm, ctx->list[0],
                               u_int, v_int, row_ids, col_ids, flip ? 1 : 0, d_row2col, d_u, d_v);
        }
        MF_HIP(hipGetLastError());
    }
    MF_HIP(hipEventRecord(ctx->ev[5], ctx->stream));
    MF_HIP(hipMemcpyAsync(ctx->h_stats, ctx->stats, sizeof(mf_device_stats), hipMemcpyDeviceToHost, ctx->stream));
    int rc = mf_run_certificate(ctx, d_W, n, m, ldw, d_row2col, d_u, d_v, K, h_res);
    if (rc != MF_OK) return rc;
    MF_HIP(hipEventRecord(ctx->ev[6], ctx->stream));
    MF_HIP(hipStreamSynchronize(ctx->stream));
    float ms_solve = 0.0f, ms_duals = 0.0f, ms_cert = 0.0f;
    MF_HIP(hipEventElapsedTime(&ms_solve, ctx->ev[3], ctx->ev[4]));
    MF_HIP(hipEventElapsedTime(&ms_duals, ctx->ev[4], ctx->ev[5]));
    MF_HIP(hipEventElapsedTime(&ms_cert, ctx->ev[5], ctx->ev[6]));
    ctx->timings[T_SOLVE] = ms_solve;
    ctx->timings[T_DUALS] = ms_duals;
    ctx->timings[T_CERT] = ms_cert;
    h_res->rounds = (int64_t)ctx->h_stats->rounds;
    h_res->bids = (int64_t)ctx->h_stats->bids;
    h_res->bytes_scanned = (int64_t)ctx->h_stats->bytes;
    h_res->chain_bids = (int64_t)ctx->h_stats->chain_bids;
    h_res->chain_retries = (int64_t)ctx->h_stats->chain_retries;
    h_res->team_bids = (int64_t)ctx->h_stats->team_bids;
    h_res->path_steps = (int64_t)ctx->h_stats->path_steps;
    h_res->path_scans = (int64_t)ctx->h_stats->path_scans;
    h_res->chain_depth = (int64_t)(ctx->h_stats->chain_depth + ctx->h_stats->launch_max);
    h_res->phases = phases;
    h_res->ms_solve = ms_solve;
    h_res->ms_certify = ms_duals + ms_cert;
    if (h_res->cert_ok && !staged) { ctx->warm_n = n; ctx->warm_m = m; }      // these prices may seed the next solve
    return h_res->cert_ok ? MF_OK : MF_ERR_CERT;
}
