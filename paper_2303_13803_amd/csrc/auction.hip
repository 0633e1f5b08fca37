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
#include "scan.h"

namespace {

// One round for many bidders: a workgroup per bidder, bids taking effect at
// once.  Later bidders of the same round may already see them (or a slightly
// older dual): the auction tolerates both because duals only move one way and a
// bid computed from an outdated dual simply fails to win.  The counters form a
// ring: round r reads cnt[r], fills cnt[r+1] and clears cnt[r+2].
constexpr int ROUND_GROUPS_PER_WORKGROUP = 128;

template <int NT, int RB>
__global__ __launch_bounds__(NT, 3) void round_kernel(SideArgs s, const int *__restrict__ list,
                                                   int *__restrict__ next, mf_device_stats *stats,
                                                   int ring)
{
    // Bidders this workgroup has to pass on are collected here and handed over together: the
    // list counter is a single address, every atomic on it takes its turn, and thousands of
    // workgroups that finish at the same moment would queue up behind it (measured: one such
    // atomic per group of four lines costs a full-matrix round a fifth of its time).
    // The launch gives every workgroup at most ROUND_GROUPS_PER_WORKGROUP groups of lines.
    __shared__ Top2 red[RB + RB * (NT / 64)];
    __shared__ int s_hold[RB * ROUND_GROUPS_PER_WORKGROUP];
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
    int held = 0;                                           // entries of s_hold in use (first wavefront, same in every lane)
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
                again = decide_and_bid<true>(s, b, t);
            }
            const unsigned long long pushing = __ballot(again >= 0);
            if (pushing) {
                if (again >= 0) s_hold[held + __popcll(pushing & ((1ull << threadIdx.x) - 1ull))] = again;
                held += __popcll(pushing);
            }
        }
    }
    if (threadIdx.x < 64 && held > 0) {
        int base = 0;
        if (threadIdx.x == 0) base = atomicAdd(ncnt, held);
        base = __shfl(base, 0);
        for (int k = threadIdx.x; k < held; k += 64) next[base + k] = s_hold[k];
    }
    // (a word with a cache line to itself: not behind the list counter)
    if (threadIdx.x == 0 && entries) atomicAdd(&stats->round_bytes, entries * 4ull);
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
    bool handing_back = false;              // block-uniform
    for (;;) {
        __syncthreads();
        if (threadIdx.x == 0) s_next = atomicAdd(&stats->head, 1);
        __syncthreads();
        const int item = s_next;
        if (item >= count) break;
        int b = list[item];
        if (handing_back) {                 // pass on what nobody will bid for in this launch
            if (threadIdx.x == 0) out_list[atomicAdd(&stats->cnt[(ring + 1) & 3], 1)] = b;
            continue;
        }
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
                handing_back = true;
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
        // handed back: follow no further chain, but keep emptying the list - if every workgroup
        // stopped here, entries nobody had claimed yet would never reach the next launch
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

__global__ void known_weight_kernel(const int *largest, mf_device_stats *stats) { stats->max_weight = *largest; }
__global__ void fill_counter_kernel(unsigned long long *counter) { *counter = 0ull; }

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
        stats->rounds = 0; stats->bids = 0; stats->bytes = 0; stats->round_bytes = 0; stats->head = 0;
        stats->chain_bids = 0; stats->chain_depth = 0; stats->launch_max = 0; stats->chain_retries = 0; stats->team_bids = 0; stats->path_steps = 0; stats->path_scans = 0; stats->team_abort = 0; stats->rested = 0; stats->active = 0; stats->max_weight = 0;
        stats->cnt[0] = 0; stats->cnt[1] = 0; stats->cnt[2] = 0; stats->cnt[3] = 0;
    }
}

template <int NT, int RB>
void launch_round_shape(mf_ctx *ctx, const SideArgs &s, int count, int ring)
{
    int grid = (count + RB - 1) / RB;
    if (grid > MAX_GRID) grid = MAX_GRID;
    // ten workgroups per compute unit read a matrix faster than one per group of lines: those that
    // finish early take another group, and fewer of them queue for the list counter at the end
    const int cap = ctx->bulk_grid > 0 ? ctx->bulk_grid : 10 * (ctx->n_cus > 0 ? ctx->n_cus : 256);
    if (grid > cap) grid = cap;
    const int groups = (count + RB - 1) / RB;               // (a workgroup's list of bidders to pass on holds so many groups)
    if ((long long)grid * ROUND_GROUPS_PER_WORKGROUP < groups) grid = (groups + ROUND_GROUPS_PER_WORKGROUP - 1) / ROUND_GROUPS_PER_WORKGROUP;
    hipLaunchKernelGGL((round_kernel<NT, RB>), dim3(grid), dim3(NT), 0, ctx->stream, s, ctx->list[ring & 1],
                       ctx->list[(ring + 1) & 1], ctx->stats, ring);
}

void launch_round(mf_ctx *ctx, const SideArgs &s, int count, int ring)
{
    if (s.edge_start && count >= 2048) { mf_launch_list_round(ctx, s, count, ring); return; }
    // Lines in groups per wavefront read the matrix fastest, and that is what counts when (nearly)
    // every line bids: the first round of a phase.  In the rounds after it, one line per workgroup
    // does better although it reads more slowly: bids land sooner, later bidders of the same round
    // see them, and fewer bids are wasted (measured on cluster-scale rounds: a fifth fewer bids).
    const bool grouped = count >= 2048 && (long long)count * 100 >= (long long)ctx->bulk_share * (long long)s.len_t;
    switch (grouped ? ctx->bulk_shape : 0) {
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
int run_side(mf_ctx *ctx, const SideArgs &s, int count, bool time_first, int stop_at, long long tail_budget, int *left_over)
{
    int ring = 0;
    // Short chains are cheapest followed step by step; a chain that is still going after
    // `path_after` steps is ended by shortest-path searches instead.
    long long team_steps = 0;
    int idle_launches = 0;
    long long tail_steps = 0;               // dependent steps of the chain kernels of this run, longest workgroup of each
    *left_over = count;
    // Bulk rounds do not wait for their own outcome: the next round is launched for at most as many
    // bidders as the last count the host has seen (a round never leaves more bidders than it
    // found: each bid displaces at most one holder), the kernel reads the true count on the
    // device, and the host reads the count of a round while the one after it runs.  `unread` says
    // that such a round is in flight; every other kind of launch waits for the exact count first.
    bool unread = false;
    int unread_ring = 0, unread_slot = 0, slot = 0;
    bool counted_teams = false, chained = false;
    unsigned long long bids_before = ctx->h_stats->bids;
    // takes in the statistics copied after the launch that left the lists at position `at`
    auto absorb = [&](int at) -> int {
        if ((long long)ctx->h_stats->bids == (long long)bids_before && ctx->h_stats->cnt[at & 3] >= count) {
            // a launch that neither evaluated a bid nor placed anybody must not repeat for ever
            if (++idle_launches > 64) return MF_ERR_NOT_CONVERGED;
        } else idle_launches = 0;
        bids_before = ctx->h_stats->bids;
        count = ctx->h_stats->cnt[at & 3];
        if (counted_teams) team_steps += (long long)ctx->h_stats->launch_max;     // the longest any leader went
        if (chained) tail_steps += (long long)ctx->h_stats->launch_max;
        // a bounded wait ran out: one workgroup per chain, or no more searches, for the rest of this solve
        if (ctx->h_stats->team_abort == 1) { ctx->team_off = true; ctx->fallbacks |= MF_FALLBACK_TEAMS; }
        if (ctx->h_stats->team_abort == 2) { ctx->path_off = true; ctx->fallbacks |= MF_FALLBACK_SEARCHES; }
        *left_over = count;
        return MF_OK;
    };
    auto read_unread = [&]() -> int {
        MF_HIP(hipEventSynchronize(ctx->ev_stats[unread_slot]));
        *ctx->h_stats = *ctx->h_stats_slot[unread_slot];
        unread = false;
        return absorb(unread_ring);
    };
    while (count > stop_at) {
        // a side that only prepares prices (stop_at > 0) does not follow chains for ever
        if (stop_at > 0 && tail_budget > 0 && tail_steps >= tail_budget) break;
        const bool bulk = count > ctx->tail_max;
        if (unread && !bulk) {
            // chains, teams and searches are laid out for the exact number of bidders
            const int rc = read_unread();
            if (rc != MF_OK) return rc;
            continue;
        }
        bool timed = false;
        counted_teams = false; chained = false;
        const unsigned long long bytes_before = ctx->h_stats->bytes + ctx->h_stats->round_bytes;
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
        if (bulk) {
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
            const int rc = mf_launch_path_search(ctx, s, ring);
            if (rc != MF_OK) return rc;
            ++ring;
        } else if (!teams_ok || count > team_from) {
            const int grid = count < ctx->chain_grid ? count : ctx->chain_grid;
            // Workgroups hand their bidders back once so few chains are left that teams (or searches)
            // do better.  Never at a count the grid starts below: then every workgroup would hand
            // back before its first bid and the same launch would repeat for ever.
            int hand_back = teams_ok ? team_from : (paths_ok ? ctx->path_max : -1);
            if (hand_back >= grid) hand_back = grid - 1;
            chained = true;
            hipLaunchKernelGGL(chain_begin_kernel, dim3(1), dim3(1), 0, ctx->stream, ctx->stats, ring, grid);
            // (the budget of a side that only prepares prices is checked between launches, not inside
            // this one: where rows that will end up unmatched fight over every column they fit
            // beside, cutting this launch short leaves hundreds of them to the finer phases, which
            // then take seconds - measured)
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
            chained = true;
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
        if (bulk && !timed && ctx->round_lag && count > 4096) {     // (smaller rounds go three to a read, above)
            MF_HIP(hipMemcpyAsync(ctx->h_stats_slot[slot], ctx->stats, sizeof(mf_device_stats), hipMemcpyDeviceToHost, ctx->stream));
            MF_HIP(hipEventRecord(ctx->ev_stats[slot], ctx->stream));
            if (unread) {
                const int rc = read_unread();           // the round before this one, while this one runs
                if (rc != MF_OK) return rc;
            }
            unread = true;
            unread_ring = ring;
            unread_slot = slot;
            slot ^= 1;
            continue;
        }
        MF_HIP(hipMemcpyAsync(ctx->h_stats, ctx->stats, sizeof(mf_device_stats), hipMemcpyDeviceToHost, ctx->stream));
        MF_HIP(hipStreamSynchronize(ctx->stream));
        unread = false;                                  // (a later copy on the same stream: it covers the round in flight too)
        if (timed) {
            float ms = 0.0f;
            MF_HIP(hipEventElapsedTime(&ms, ctx->ev[6], ctx->ev[7]));
            ctx->timings[T_BID_BULK] += ms;
            ctx->timings[T_BID_BULK_LAUNCHES] += 1.0f;
            ctx->timings[T_BID_BULK_BYTES] += (float)((double)(ctx->h_stats->bytes + ctx->h_stats->round_bytes - bytes_before));
        }
        time_first = false;
        const int rc = absorb(ring);
        if (rc != MF_OK) return rc;
    }
    if (unread) {
        const int rc = read_unread();
        if (rc != MF_OK) return rc;
    }
    return MF_OK;
}

}  // namespace

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
    ctx->team_off = ctx->path_off = false;      // every solve starts with all of its kernels
    ctx->fallbacks = 0;
    const bool candidate = may_use_staged && ctx->fit_prefix && ctx->staged_n == n && ctx->staged_m == m;
    const bool flip = n > m;
    warm = warm && !flip && !candidate && ctx->warm_n == n && ctx->warm_m == m;
    ctx->warm_n = ctx->warm_m = 0;
    const int64_t ldt = ((int64_t)n + 3) & ~3ll;
    const int rn = flip ? m : n, rm = flip ? n : m;
    const long long K = (long long)rn + 1;
    const double Kd = (double)K;
    const int nm = rm;

    // A matrix the caller brings (no memory-ordered copy, no prefixes) may still be mostly
    // infeasible pairs, in any pattern: its rows are then also kept as lists of feasible pairs.
    const bool lists_possible = !candidate && !flip && !warm && ctx->edge_lists_from > 0 && n >= ctx->edge_lists_from &&
                                ctx->fit_prefix_below > 0;
    MF_HIP(hipEventRecord(ctx->ev[3], ctx->stream));
    {
        // the largest weight sets the first epsilon
        const int chunks = (m + 4095) / 4096 < 4 ? (m + 4095) / 4096 : 4;
        hipLaunchKernelGGL(init_solver_kernel, dim3((nm + 4 + 255) / 256), dim3(256), 0, ctx->stream, rn, rm,
                           ctx->price, ctx->profit, ctx->stats, warm ? 1 : 0);
        // (when the matrix was scored here a moment ago its largest weight was noted on the way)
        if (candidate && ctx->largest_weight_known)
            hipLaunchKernelGGL(known_weight_kernel, dim3(1), dim3(1), 0, ctx->stream, ctx->largest_weight, ctx->stats);
        else if (lists_possible) {
            // the same pass also counts the feasible pairs of every row: with few of them the rounds read lists
            hipLaunchKernelGGL(fill_counter_kernel, dim3(1), dim3(1), 0, ctx->stream, ctx->feasible_pairs);
            const int rc = mf_count_edges(ctx, d_W, n, m, ldw);
            if (rc != MF_OK) return rc;
        } else
            hipLaunchKernelGGL(max_weight_kernel, dim3(chunks, n < 1024 ? n : 1024), dim3(256), 0, ctx->stream, d_W, n,
                               m, ldw, ctx->stats);
        MF_HIP(hipGetLastError());
    }
    *ctx->h_feasible_pairs = ~0ull;
    if (candidate || lists_possible)
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
                 (int)(feasible / (double)rn), nullptr, (long long)ldat, rn, flip ? len_rows : len_cols,
                 nullptr, nullptr, nullptr, &ctx->stats->rested};
    SideArgs rev{At, (long long)ldat, rn, ctx->profit, ctx->roword, 0.0, Kd, flip ? len_rows : len_cols,
                 (int)(feasible / (double)rm), A, (long long)lda, rm, flip ? len_cols : len_rows,
                 nullptr, nullptr, nullptr, nullptr};
    if (flip) fwd.T = At;                       // (the other copy of the matrix: made on demand unless it is the one solved on)
    if (lists_possible && (double)*ctx->h_feasible_pairs * 100.0 < (double)ctx->fit_prefix_below * (double)n * (double)m &&
        *ctx->h_feasible_pairs + 4ull * (unsigned long long)n <= (unsigned long long)mf_edge_capacity(ctx)) {
        const int rc = mf_build_edge_lists(ctx, d_W, n, m, ldw, &fwd);
        if (rc != MF_OK) return rc;
    }

    // The ladder of epsilons: divided by theta per phase down to 1.  Once epsilon is at most
    // final_jump weight units (final_jump * K in dual units) the next phase is the last one:
    // prices that good leave the phase at epsilon = 1 about one bid per row, and the phases in
    // between would each cost a full re-bid and a tail of their own.
    long long ladder[64];
    int n_phases = 0;
    {
        long long e = cmax / ctx->theta;
        if (warm && ctx->warm_eps_units * K < e) e = ctx->warm_eps_units * K;
        if (e < 1) e = 1;
        for (;;) {
            ladder[n_phases++] = e;
            if (e == 1 || n_phases == 64) break;
            long long next = e / ctx->theta;
            if (next < 1 || (ctx->final_jump > 0 && e <= ctx->final_jump * K) || n_phases == 63) next = 1;
            e = next;
        }
    }
    int phases = 0;
    for (int ph = 0; ph < n_phases; ++ph) {
        const long long eps = ladder[ph];
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
        int left_over = 0;
        const int phases_after = n_phases - 1 - ph;
        // The coarser the phase, the more may be left (phase_growth times more per phase), but
        // never more than one bidder in 64: small problems complete every phase.
        long long stop_ll = 0;
        if (phases_after >= ctx->phase_keep) {
            stop_ll = ctx->phase_stop;
            // ... unless bidders have been giving up (best value at most epsilon) in this solve: then
            // workloads stay unmatched at the optimum, the bidders left over would be the ones that
            // end up resting, and the finer the epsilon at which they fight it out the longer it takes
            const int growth = ctx->h_stats->rested < ctx->phase_growth_rest ? ctx->phase_growth : 1;
            for (int k = ctx->phase_keep; k < phases_after && stop_ll < rn; ++k) stop_ll *= growth;
            // the searches are for the phases that have to finish: a coarse one ends at the latest
            // where they would take over
            if (ctx->path_max > 0 && !ctx->path_off && stop_ll > 0 && stop_ll < ctx->path_max) stop_ll = ctx->path_max;
            if (stop_ll > rn / 64) stop_ll = rn / 64;
        }
        const int stop_at = (int)stop_ll;
        // a phase that runs to the end places its last bidders by a search, which re-labels the
        // columns of a served tree from the other copy of the matrix
        if (!have_transpose && stop_at == 0 && ctx->path_max > 1 && rn > 1) make_transpose();
        if (have_transpose) fwd.T = At;
        int rc = run_side(ctx, fwd, rn, true, stop_at, (ctx->phase_tail_sides & 1) && rn >= ctx->phase_tail_from ? ctx->phase_tail_steps : 0, &left_over);
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
            rc = run_side(ctx, rev, rev_count, false, stop_at, (ctx->phase_tail_sides & 2) && rn >= ctx->phase_tail_from ? ctx->phase_tail_steps : 0, &left_over);
            if (rc != MF_OK) return rc;
            hipLaunchKernelGGL(reverse_done_cols_kernel, dim3((rm + 255) / 256), dim3(256), 0, ctx->stream, rm,
                               ctx->price, ctx->col2row);
            hipLaunchKernelGGL(reverse_done_rows_kernel, dim3((rn + 255) / 256), dim3(256), 0, ctx->stream, rn,
                               A, lda, Kd, ctx->roword, ctx->price, ctx->row2col, ctx->col2row);
            MF_HIP(hipGetLastError());
        }
    }
    MF_HIP(hipEventRecord(ctx->ev[4], ctx->stream));
    {
        const int rc = mf_extract_duals(ctx, A, lda, rn, rm, Kd, fwd.line_len, n, flip, staged, d_row2col, d_u, d_v);
        if (rc != MF_OK) return rc;
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
    h_res->bytes_scanned = (int64_t)(ctx->h_stats->bytes + ctx->h_stats->round_bytes);
    h_res->chain_bids = (int64_t)ctx->h_stats->chain_bids;
    h_res->chain_retries = (int64_t)ctx->h_stats->chain_retries;
    h_res->team_bids = (int64_t)ctx->h_stats->team_bids;
    h_res->path_steps = (int64_t)ctx->h_stats->path_steps;
    h_res->path_scans = (int64_t)ctx->h_stats->path_scans;
    h_res->chain_depth = (int64_t)(ctx->h_stats->chain_depth + ctx->h_stats->launch_max);
    h_res->phases = phases;
    h_res->fallbacks = ctx->fallbacks;
    h_res->ms_solve = ms_solve;
    h_res->ms_certify = ms_duals + ms_cert;
    if (h_res->cert_ok && !staged) { ctx->warm_n = n; ctx->warm_m = m; }      // these prices may seed the next solve
    return h_res->cert_ok ? MF_OK : MF_ERR_CERT;
}
