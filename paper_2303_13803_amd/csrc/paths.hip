// The last bidders of an auction run, placed by shortest-augmenting-path searches that the
// whole device runs together (paper: Algorithm "Scheduling algorithm", GetMatching; the
// searches are the successive-shortest-path step of the Hungarian method the paper uses,
// applied to the few bidders whose chains of bids would otherwise go on for thousands of steps).
#include "scan.h"
#include <limits.h>

namespace {

// A chain of bids is a greedy walk: every evicted holder moves to its own best
// alternative, and with a few bidders left such a walk takes thousands of
// dependent steps to reach a free line.  The shortest way to make room is far
// shorter in hops, and finding it is a breadth-type search whose every step is
// wide.  In the notation of the header of auction.hip with "rows" the bidding
// side, let rc(i,k) = pi_i + p_k - K W_ik + eps >= 0 (I1) for every assigned
// row i and for every bidder r (pi_r = best value of r - eps); assigned pairs
// have rc = eps.  A path r -> k1, holder(k1) -> k2, ... that ends in a column
// nobody holds, or in a row giving up its column for profit 0 (at extra length
// pi_i), frees a place for r; label(k) is the length sum(rc) of the shortest
// such path to column k from ANY bidder still to be placed, and the columns
// whose shortest path starts at bidder a form a's tree.  When the nearest end
// of a path, at length d, is final, it belongs to one tree: raising p_k by
// d - label(k) on that tree's columns with label(k) < d (their holders' profits
// drop by as much) keeps I1 and I2 and makes the path tight; re-assigning
// along it, each row paying eps more for its new column, keeps them too and
// leaves one bidder fewer.  (The successive-shortest-path step of the Hungarian
// method, on costs relaxed by eps, with every unplaced bidder a root at once.)
// The search then goes on for the others: their trees, labels and pending
// updates stay as they are - a later, longer path only raises what an earlier
// one left - while the served tree's columns lose their labels and are reached
// again, at prices already raised, from the rows the other trees have scanned
// (all of which are scanned once more).  Searching for one bidder after another
// instead would label the same few thousand columns again for each of them:
// measured on cluster-scale rounds, successive trees share nine columns in ten.
// Prices only rise, so this mixes freely with bids.
//
// All compute units run the search together: labels are corrected in
// super-steps - every row whose column's label dropped into the current
// window [low, low + width) is scanned against all columns, in parallel, with
// an atomic compare-and-swap per improved label - separated by grid-wide
// barriers.  Data shared between workgroups moves only through atomics and
// uncached loads/stores.  Every wait is bounded; if one runs out all
// workgroups leave, nothing half-done, and the host falls back to the chain
// kernels.
constexpr int PATH_THREADS = 1024;
constexpr int PATH_MAX_SLICES = 1024;
constexpr int PATH_GROUP = 16, PATH_MAX_GROUPS = 64;      // up to 1024 workgroups
constexpr int PATH_SEGMENTS = 16, PATH_PUSH_BUFFER = 4096;
constexpr unsigned long long PATH_INF = ~0ull;
constexpr int PATH_MAX_SOURCES = 64;                      // bidders one search places
constexpr unsigned PATH_IN_TREE = 0xffffffffu;            // stamp of a column of the tree being served
constexpr int PATH_NO_LABEL = INT_MIN;                    // in PathBuffers::jump: the column has no label
constexpr int PATH_JUMP_HOPS = 4, PATH_JUMP_PASSES = 48;  // hops a column follows per pass; passes before the search gives up

struct alignas(128) PathCtl {
    unsigned long long sink;        // nearest end of a path found so far: length << 21 | kind << 20 | id (kind 1: row id gives up)
    unsigned long long low[3];      // smallest label still to be expanded, per slot
    // Ends of paths found during a step, per slot like `low`: `sink` above moves while a step
    // runs, so two workgroups reading it at the top of the same step may see different values;
    // what all workgroups must decide alike (a path end is final) must not depend on that, or
    // they would arrive at different barriers.  Every workgroup folds the slot the previous step
    // filled (nobody writes it any more) into a running minimum of its own and decides from that.
    unsigned long long sink_found[3];
    unsigned long long src_profit[PATH_MAX_SOURCES];     // bits of a double: best value - eps of each bidder (<= 0: it rests)
    // The barrier's two hot words each have a cache line to themselves: hundreds of polling loads
    // on the line of a counter that is being incremented (or of the sink above) slow both down.
    struct alignas(128) { unsigned int count; } arrive;       // whole groups that have arrived at barriers so far
    struct alignas(128) { unsigned int number; } open;        // barriers completed so far | PATH_GAVE_UP
    alignas(128) unsigned long long steps;
    unsigned long long scans, entries;
    alignas(128) unsigned int tree_count;                     // columns of the tree being served (list in PathBuffers::tree)
    // pass q of finding every column's root left some column short of it (zero between uses)
    alignas(128) unsigned int jump_pending[PATH_JUMP_PASSES + 1];
    struct alignas(128) { unsigned int arrive; } group[PATH_MAX_GROUPS];
    // Frontier lengths: one counter per segment (a segment collects the pushes of sixteen
    // workgroups, so no counter is hit by more than sixteen atomics per step), in three slots:
    // step t reads slot t % 3, fills slot (t + 1) % 3 and clears slot (t + 2) % 3, which every
    // workgroup finished reading before the barrier that ended step t - 1.
    struct alignas(128) { unsigned int count; } seg[3][PATH_SEGMENTS];
};
static_assert(sizeof(PathCtl) <= 32768, "the context allocates 32 KiB for this block");

struct PathBuffers {
    unsigned long long *label;      // [len] length << 20 | predecessor row
    unsigned long long *expanded;   // [len] label at which the column's holder was last scanned
    unsigned int *stamp;            // [len] last step in which the column was put on a frontier
    unsigned long long *fr_col[2];  // frontiers (by step parity): PATH_SEGMENTS segments of len entries each; an entry
                                    // is a column and, in the upper half, the row that holds it (holders change only
                                    // between searches' re-assignments, and no frontier outlives one)
    int *held;                      // [rows] column a frontier row holds (-1 - index for a bidder)
    double *base;                   // [rows + 8] for a row that has been scanned: its path length + its profit + eps
                                    // (a column's label through that row is base - K w + the column's dual); else PATH_FAR
    int *tree;                      // [len] columns of the tree being served
    int *parent;                    // [len] while a tree is served: the column whose holder gave this column its label
                                    // (-1 - index of a bidder if that row is a bidder)
    int *jump;                      // [len] ... and a column further up the same chain, in the end the bidder at its root
};
constexpr double PATH_FAR = 1.0e300;

// Grid-wide barrier in two levels: workgroups arrive at their group's counter, the last of a
// group at the top counter, and the last of all publishes the barrier's number in a word that
// everybody else polls.  (Hundreds of atomics on one address take turns; sixteen groups of
// sixteen do not.  The polled word sits on a cache line of its own: timed alone, 256 workgroups
// pass this barrier in 1.5 us, in 2.7 us when they poll the counter the arrivals increment, in
// 3.8 us when that counter shares its line with other shared words.)  Counters only ever grow.
// The top bit of the polled word says that somebody's wait ran out: whoever sees it leaves.
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
        const unsigned number = generation + 1u;                 // this barrier's number
        unsigned seen = 0u;
        if ((atomicAdd(&ctl->group[g].arrive, 1u) + 1u) % size == 0u &&
            atomicAdd(&ctl->arrive.count, 1u) + 1u == number * groups)
            // the last of all: the old value tells whether somebody had given up before
            seen = (atomicMax(&ctl->open.number, number) & PATH_GAVE_UP) | number;
        unsigned spins = 0;
        while (!(seen & PATH_GAVE_UP) && seen < number) {
            if (++spins > spin_limit) { seen = atomicOr(&ctl->open.number, PATH_GAVE_UP) | PATH_GAVE_UP; break; }
            seen = load_fresh_u32(&ctl->open.number);
        }
        s_ok = (seen & PATH_GAVE_UP) ? 0 : 1;
    }
    ++generation;
    __syncthreads();
    return s_ok != 0;
}

__global__ void path_begin_kernel(mf_device_stats *stats, PathCtl *ctl, int ring)
{
    ctl->arrive.count = 0u; ctl->open.number = 0u; ctl->steps = 0ull; ctl->scans = 0ull; ctl->entries = 0ull; ctl->tree_count = 0u;
    for (int q = 0; q <= PATH_JUMP_PASSES; ++q) ctl->jump_pending[q] = 0u;
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

// Lowers label[k] to `mine` if that is a strictly shorter length (a tie keeps the predecessor
// it has: swapping predecessors at equal length could close a cycle of zero-length edges).
// `seen` is what the caller has read of the word, possibly outdated but never below the true word:
// a safe first test.
__device__ inline bool lower_label(unsigned long long *word, unsigned long long seen, unsigned long long mine)
{
    while ((mine >> MF_ID_BITS) < (seen >> MF_ID_BITS)) {
        const unsigned long long was = atomicCAS(word, seen, mine);
        if (was == seen) return true;
        seen = was;
    }
    return false;
}

__global__ __launch_bounds__(PATH_THREADS) void path_kernel(SideArgs s, const int *__restrict__ list,
                                                            int *__restrict__ out_list, mf_device_stats *stats,
                                                            PathCtl *ctl, PathBuffers buf, int ring, int rows,
                                                            double width_max, unsigned spin_limit, int frontier_high)
{
    __shared__ Top2 red[PATH_THREADS / 64];
    __shared__ unsigned s_pushes, s_base, s_first[PATH_SEGMENTS + 1];
    __shared__ unsigned long long s_sink, s_low;
    __shared__ unsigned long long s_list[PATH_PUSH_BUFFER];
    __shared__ double s_profit[PATH_MAX_SOURCES];       // of each bidder: best value - eps
    __shared__ int s_row[PATH_MAX_SOURCES];
    __shared__ int s_alive[PATH_MAX_SOURCES], s_n_alive;
    const unsigned G = gridDim.x;
    const int wg = blockIdx.x, tid = threadIdx.x;
    const int gtid = wg * PATH_THREADS + tid, gsize = (int)G * PATH_THREADS;
    const int listed = stats->cnt[ring & 3];
    const int count = min(listed, PATH_MAX_SOURCES);
    unsigned generation = 0;
    unsigned long long my_steps = 0, my_scans = 0, my_entries = 0;
    bool ok = true;

    // ---- set-up: no labels; one workgroup per bidder finds its best value ----
    for (int k = gtid; k < s.len; k += gsize) {
        store_through(&buf.label[k], PATH_INF);
        store_through(&buf.expanded[k], PATH_INF);
        __hip_atomic_store(&buf.stamp[k], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    for (int i = gtid; i < ((s.len_t + 7) & ~3); i += gsize)
        store_through((unsigned long long *)&buf.base[i], (unsigned long long)__double_as_longlong(PATH_FAR));
    // (a barrier of its own: the bidders' entries below must not be overwritten by a late clearing store)
    const bool cleared = grid_barrier(ctl, G, generation, spin_limit);
    for (int item = wg; item < count; item += (int)G) {
        const int r = list[item];
        const Top2 t = block_scan<PATH_THREADS>(s.A + (size_t)r * s.pitch, s.other_dual, line_length(s, r), s.Kd,
                                                true, red, 0, 0);
        if (tid == 0) {
            store_through(&ctl->src_profit[item], (unsigned long long)__double_as_longlong(t.b1 - s.eps));
            __hip_atomic_store(&buf.held[r], -1 - item, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (t.b1 > s.eps) store_through((unsigned long long *)&buf.base[r], (unsigned long long)__double_as_longlong(t.b1));
        }
    }
    if (wg == 0) {
        if (tid < 3 * PATH_SEGMENTS)
            __hip_atomic_store(&ctl->seg[tid / PATH_SEGMENTS][tid % PATH_SEGMENTS].count, 0u, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        if (tid == 0) {
            store_through(&ctl->sink, PATH_INF);
            for (int q = 0; q < 3; ++q) { store_through(&ctl->low[q], PATH_INF); store_through(&ctl->sink_found[q], PATH_INF); }
        }
    }
    const bool started = grid_barrier(ctl, G, generation, spin_limit) && cleared;   // false: nobody's best value can be trusted
    ok = started;
    // duals stand still between two re-assignments: drop what the caches hold of them from before
    // once, then read them through the caches
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    if (tid < count) {
        s_profit[tid] = __longlong_as_double((long long)load_fresh_u64(&ctl->src_profit[tid]));
        s_row[tid] = list[tid];
    }
    __syncthreads();
    // Every workgroup keeps its own copy of the list of bidders still to be placed; all copies
    // change alike because every decision below is taken from the same published words.
    if (tid == 0) {
        int n = 0;
        for (int j = 0; j < count; ++j)
            if (s_profit[j] > 0.0) s_alive[n++] = j;        // a bidder whose best value is at most eps rests with dual 0
        s_n_alive = n;
    }
    __syncthreads();
    int n_alive = s_n_alive;

    // what "the bidder rests after all" costs, the nearest of them: the first path ends every workgroup agrees on
    auto resting_bidders = [&]() {
        unsigned long long best = PATH_INF;
        for (int e = 0; e < n_alive; ++e) {
            const int j = s_alive[e];
            const unsigned long long w = ((unsigned long long)(long long)s_profit[j] << 21) | (1ull << 20) |
                                         (unsigned long long)s_row[j];
            best = w < best ? w : best;
        }
        return best;
    };
    unsigned long long agreed_sink = resting_bidders();
    // ... and the farthest: no bidder's path is longer than what resting costs it, so labels at or
    // beyond that are of no use to anybody
    auto farthest_rest = [&]() {
        double far = 0.0;
        for (int e = 0; e < n_alive; ++e) far = fmax(far, s_profit[s_alive[e]]);
        return far;
    };
    double far_bound = farthest_rest();
    // With the other copy of the matrix at hand, the columns of a served tree get their new labels
    // by one look each at all scanned rows; without it, every scanned row is scanned again.
    const bool pull = s.T != nullptr;

    // ---- label-correcting search, one grid barrier per super-step ----
    // A step scans the rows on the current frontier; a label that falls inside the window puts
    // its column on the next frontier at once (claimed through a per-step stamp, so once per
    // step), whose holder is scanned in the next step from the label the column has by then.
    // Only when a frontier comes up empty does a pass over all columns pick up the labels that
    // fell outside earlier windows, or move the window on, or find that the nearest path end is final.
    double low = 0.0;
    // The window adapts to what it yields: wide enough to keep the device busy, narrow enough
    // that rows are not scanned long before their label is final (every workgroup derives the
    // same width from the same counters).
    double width = 4.0 * s.eps;
    const int segment = wg / PATH_GROUP % PATH_SEGMENTS;
    unsigned step = 0, since_served = 0;
    bool swept = false;                      // the previous step was a pass over all columns
    bool from_bidders = true;                // this step scans the bidders themselves (the first, and the one after a re-assignment)
    bool sweep_next = false;                 // ... and the step after that looks at every column
    while (ok && n_alive > 0) {
        // far more steps than a search over sound duals can take: give the bidders back to the
        // chains (every workgroup counts the same steps, so all leave here together)
        if (++since_served > 4u * (unsigned)s.len + 4096u) { ok = false; break; }
        ++step;
        const unsigned c = step % 3u, p = (step + 1u) % 3u, z = (step + 2u) % 3u;
        // frontier of this step: its segments' lengths
        if (tid < 64) {
            unsigned n_seg = 0;
            if (tid < PATH_SEGMENTS && !from_bidders) n_seg = load_fresh_u32(&ctl->seg[c][tid].count);
            unsigned run = n_seg;                               // inclusive prefix sums over 16 lanes
            for (int d = 1; d < PATH_SEGMENTS; d <<= 1) {
                const unsigned o = __shfl_up(run, d);
                if ((int)tid >= d) run += o;
            }
            if (tid < PATH_SEGMENTS) s_first[tid + 1] = run;
            if (tid == 0) { s_first[0] = 0u; s_pushes = 0u; s_sink = PATH_INF; s_low = PATH_INF; }
        }
        __syncthreads();
        const bool sweeping = !from_bidders && (sweep_next || s_first[PATH_SEGMENTS] == 0u);
        const int nf = from_bidders ? n_alive : (sweeping ? 0 : (int)s_first[PATH_SEGMENTS]);
        {
            const unsigned long long found = load_fresh_u64(&ctl->sink_found[c]);
            agreed_sink = found < agreed_sink ? found : agreed_sink;
        }
        if (!from_bidders && !sweep_next && swept && nf == 0) {
            const unsigned long long lo = load_fresh_u64(&ctl->low[c]);
            if (lo == PATH_INF || lo >= (agreed_sink >> 21)) {
                // ---- every label below the nearest path end is final: serve its tree ----
                // Nothing the others can see changes before the barrier that proves every
                // workgroup got here (a wait that runs out before it leaves the state as it
                // was); then workgroup 0 alone raises the tree's prices and re-assigns along the
                // path, so no wait that runs out later can leave that half-done.
                const unsigned long long sink = agreed_sink, d_star = sink >> 21;
                const int sink_id = (int)(sink & 0xfffffull);
                const bool gives_up = ((sink >> 20) & 1ull) != 0;
                // Which bidder's tree is it, and which columns belong to that tree?  A column's root
                // lies at the end of its chain of predecessors, dozens to hundreds of hops away,
                // every hop two dependent loads; instead of every column walking its chain, all
                // columns shorten their pointers together (pointer jumping): first every labelled
                // column notes the column above it (or the bidder, if its predecessor is one), then
                // in every pass it moves its pointer up to the pointer of the column it points to, a
                // few hops at a time, until all point at bidders.  Labels stand still meanwhile.
                for (int k = gtid; k < s.len; k += gsize) {
                    const unsigned long long lw = load_fresh_u64(&buf.label[k]);
                    int up = PATH_NO_LABEL;
                    if (lw != PATH_INF)
                        up = __hip_atomic_load(&buf.held[(int)(lw & MF_ID_MASK)], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(&buf.parent[k], up, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(&buf.jump[k], up, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                if (!grid_barrier(ctl, G, generation, spin_limit)) { ok = false; break; }
                int passes = 0;
                for (;;) {
                    bool short_of_it = false;
                    for (int k = gtid; k < s.len; k += gsize) {
                        int up = __hip_atomic_load(&buf.jump[k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        if (up < 0) continue;                       // a bidder, or no label
                        for (int hop = 0; hop < PATH_JUMP_HOPS && up >= 0; ++hop)
                            up = __hip_atomic_load(&buf.jump[up], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        // (a pointer to a column without a label cannot be, with sound labels: it stays
                        // as it is and reads as "no bidder" below)
                        __hip_atomic_store(&buf.jump[k], up, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        short_of_it |= up >= 0;
                    }
                    if (__syncthreads_or(short_of_it) && tid == 0) atomicOr(&ctl->jump_pending[passes], 1u);
                    if (!grid_barrier(ctl, G, generation, spin_limit)) { ok = false; break; }
                    if (load_fresh_u32(&ctl->jump_pending[passes]) == 0u) break;
                    if (++passes >= PATH_JUMP_PASSES) { ok = false; break; }        // (the same in every workgroup)
                }
                if (!ok) break;
                int root = -1;
                {
                    // where the path ends: a free column, or the column its last row gives up (none: the bidder itself rests)
                    int at = sink_id;
                    if (gives_up) at = __hip_atomic_load(&buf.held[sink_id], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if (at >= 0) at = __hip_atomic_load(&buf.jump[at], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if (at < 0 && at != PATH_NO_LABEL) root = -1 - at;
                }
                if (root < 0 || root >= count) { ok = false; break; }          // (the same in every workgroup)
                if (tid == 0) s_pushes = 0u;
                __syncthreads();
                for (int k = gtid; k < s.len; k += gsize) {
                    if (__hip_atomic_load(&buf.jump[k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == -1 - root) {
                        __hip_atomic_store(&buf.stamp[k], PATH_IN_TREE, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        if (pull) {
                            // its holder's scan no longer counts (workgroup 0 is about to change what it holds and pays)
                            const int holder = word_id(load_fresh_u64(&s.otherword[k]));
                            if (holder >= 0)
                                store_through((unsigned long long *)&buf.base[holder], (unsigned long long)__double_as_longlong(PATH_FAR));
                            const unsigned slot = atomicAdd(&s_pushes, 1u);
                            if (slot < (unsigned)PATH_PUSH_BUFFER) s_list[slot] = (unsigned long long)k;
                            else __hip_atomic_store(&buf.tree[atomicAdd(&ctl->tree_count, 1u)], k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        }
                    }
                }
                __syncthreads();
                if (pull) {
                    const unsigned mine = min(s_pushes, (unsigned)PATH_PUSH_BUFFER);
                    if (tid == 0) s_base = mine ? atomicAdd(&ctl->tree_count, mine) : 0u;
                    __syncthreads();
                    for (unsigned t = tid; t < mine; t += PATH_THREADS)
                        __hip_atomic_store(&buf.tree[s_base + t], (int)s_list[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if (gtid == 0)          // the bidder itself is no root any more
                        store_through((unsigned long long *)&buf.base[s_row[root]], (unsigned long long)__double_as_longlong(PATH_FAR));
                }
                if (!grid_barrier(ctl, G, generation, spin_limit)) { ok = false; break; }
                if (wg == 0) {
                    for (int k = tid; k < s.len; k += PATH_THREADS) {
                        if (__hip_atomic_load(&buf.stamp[k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != PATH_IN_TREE) continue;
                        const unsigned long long d_int = load_fresh_u64(&buf.label[k]) >> MF_ID_BITS;
                        if (d_int < d_star) {
                            const unsigned long long cw = load_fresh_u64(&s.otherword[k]);
                            store_dual(s, k, word_dual(cw) + (double)(long long)(d_star - d_int), (int)(cw & MF_ID_MASK));
                        }
                    }
                    __threadfence();
                    __syncthreads();
                    if (tid == 0) {
                        // the column the path ends in: a free one, or the one its last row gives up (none if the bidder itself rests)
                        int k = sink_id;
                        if (gives_up) {
                            const int h = __hip_atomic_load(&buf.held[sink_id], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            k = h < 0 ? -1 : h;
                        }
                        int guard = 0;
                        while (k >= 0 && guard++ <= rows) {
                            // (the three loads of a hop go out together; the next hop needs `before` alone)
                            const int before = __hip_atomic_load(&buf.parent[k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            const int i = (int)(load_fresh_u64(&buf.label[k]) & MF_ID_MASK);
                            store_dual(s, k, word_dual(load_fresh_u64(&s.otherword[k])) + s.eps, i + 1);
                            k = before;                     // negative: i is the bidder, the path is done
                        }
                        for (int q = 0; q <= PATH_JUMP_PASSES; ++q)
                            __hip_atomic_store(&ctl->jump_pending[q], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        // path ends found so far may belong to the tree that is gone: start again from
                        // "a bidder rests"; the pass over all columns below finds the others again
                        store_through(&ctl->sink, PATH_INF);
                        for (int q = 0; q < 3; ++q) store_through(&ctl->sink_found[q], PATH_INF);
                    }
                }
                if (!grid_barrier(ctl, G, generation, spin_limit)) {
                    // the bidder is placed; whoever leaves here must not hand it back
                    if (tid == 0) {
                        int n = 0;
                        for (int e = 0; e < n_alive; ++e) if (s_alive[e] != root) s_alive[n++] = s_alive[e];
                        s_n_alive = n;
                    }
                    __syncthreads();
                    n_alive = s_n_alive;
                    ok = false;
                    break;
                }
                // The served tree's columns lose their labels; every other labelled column is due
                // for another scan of its holder: columns of the served tree may now be nearer
                // through it, and labels beyond the old path end were never recorded.
                for (int k = gtid; k < s.len; k += gsize) {
                    const bool in_tree = __hip_atomic_load(&buf.stamp[k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == PATH_IN_TREE;
                    if (in_tree) {
                        store_through(&buf.label[k], PATH_INF);
                        __hip_atomic_store(&buf.stamp[k], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                    if (in_tree || !pull) store_through(&buf.expanded[k], PATH_INF);
                }
                if (tid == 0) {
                    int n = 0;
                    for (int e = 0; e < n_alive; ++e) if (s_alive[e] != root) s_alive[n++] = s_alive[e];
                    s_n_alive = n;
                }
                if (!grid_barrier(ctl, G, generation, spin_limit)) { __syncthreads(); n_alive = s_n_alive; ok = false; break; }
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");     // prices and labels changed: nothing cached is good any more
                n_alive = s_n_alive;
                agreed_sink = resting_bidders();
                far_bound = farthest_rest();
                since_served = 0;
                --step;                                                // this was no step: the slots keep their turn
                if (!pull) { from_bidders = true; sweep_next = false; swept = false; continue; }
                if (n_alive > 0) {
                    // ---- new labels for the served tree's columns: one wavefront per column looks at
                    // every row that has been scanned (and at the bidders) in the other copy of the matrix ----
                    const unsigned n_tree = load_fresh_u32(&ctl->tree_count);
                    constexpr int WAVES = PATH_THREADS / 64;
                    const int lane = tid & 63;
                    for (unsigned it = (unsigned)(wg * WAVES + (tid >> 6)); it < n_tree; it += G * WAVES) {
                        const int k = __hip_atomic_load(&buf.tree[it], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        const int32_t *line = s.T + (size_t)k * s.pitch_t;
                        const int to = s.line_len_t ? min(s.line_len_t[k], s.len_t) : s.len_t;
                        double best = PATH_FAR;
                        int who = 0x7fffffff;
#pragma unroll 2
                        for (int i = lane * 4; i < to; i += 256) {
                            const int4 w4 = *(const int4 *)(line + i);
                            const double2 b01 = *(const double2 *)(buf.base + i);
                            const double2 b23 = *(const double2 *)(buf.base + i + 2);
                            const int32_t w[4] = {w4.x, w4.y, w4.z, w4.w};
                            const double bs[4] = {b01.x, b01.y, b23.x, b23.y};
#pragma unroll
                            for (int q = 0; q < 4; ++q) {
                                const double cand = fma(-s.Kd, (double)w[q], bs[q]);
                                if (i + q < to && w[q] != MF_INFEASIBLE && bs[q] < PATH_FAR && cand < best) { best = cand; who = i + q; }
                            }
                        }
                        const double least = -wave_max(-best);
                        const int row = wave_min(best == least ? who : 0x7fffffff);
                        if (lane == 0 && least < PATH_FAR) {
                            const double length = least + s.other_dual[k];          // >= 0: a path length plus a reduced cost
                            store_through(&buf.label[k], ((unsigned long long)(long long)length << MF_ID_BITS) | (unsigned long long)row);
                        }
                    }
                }
                if (gtid == 0) __hip_atomic_store(&ctl->tree_count, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (!grid_barrier(ctl, G, generation, spin_limit)) { ok = false; break; }
                from_bidders = false; sweep_next = true; swept = false;    // next: a pass over all columns picks them up
                continue;
            }
            low = (double)(long long)lo;                                // move the window to the next label
        }
        // pruning may use whatever is known by now; decisions all workgroups must share may not
        // Labels beyond the nearest path end are of no use to the last bidder; with more bidders to
        // place they are what the search goes on from, and only what lies beyond every bidder's
        // own way out is left out.
        const double bound = (n_alive == 1 || !pull) ? (double)(long long)(min(agreed_sink, load_fresh_u64(&ctl->sink)) >> 21)
                                                     : far_bound;
        if (nf > frontier_high) width = fmax(s.eps, width * 0.5);
        else if (nf < frontier_high / 8) width = fmin(width_max, width * 2.0);
        const double limit = fmin(low + width, bound);
        if (gtid < PATH_SEGMENTS)
            __hip_atomic_store(&ctl->seg[z][gtid].count, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (gtid == 0) { store_through(&ctl->low[z], PATH_INF); store_through(&ctl->sink_found[z], PATH_INF); }
        const unsigned long long *frontier = buf.fr_col[step & 1u];
        unsigned long long *next_frontier = buf.fr_col[(step + 1u) & 1u];

        // puts column k, held by row `holder`, on the next frontier (through the workgroup's LDS
        // list while it has room)
        auto push = [&](int k, int holder) {
            const unsigned long long entry = ((unsigned long long)(unsigned)holder << 32) | (unsigned long long)(unsigned)k;
            const unsigned slot = atomicAdd(&s_pushes, 1u);
            if (slot < (unsigned)PATH_PUSH_BUFFER) s_list[slot] = entry;
            else {
                const unsigned pos = atomicAdd(&ctl->seg[p][segment].count, 1u);
                store_through(&next_frontier[(size_t)segment * s.len + pos], entry);
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
                int i, mine_col = -1;
                if (from_bidders) {
                    i = s_row[s_alive[e]];
                } else {
                    int g = 0;
                    while ((unsigned)e >= s_first[g + 1]) ++g;
                    // the entry names the column and the row that holds it: everything else the
                    // scan needs can be requested at once, one memory round trip after this one
                    const unsigned long long entry = load_fresh_u64(&frontier[(size_t)g * s.len + (e - s_first[g])]);
                    mine_col = (int)(unsigned)(entry & 0xffffffffull);
                    i = (int)(unsigned)(entry >> 32);
                }
                const int32_t *row = s.A + (size_t)i * s.pitch;
                const int from = sl * span, reach = min(s.len, from + span);
                // requested together: the column's label, what its holder pays for it, the line's
                // length and the first entries of the slice (a line is allocated to its full
                // length; what lies beyond its feasible part is marked infeasible)
                unsigned long long lw = 0ull;
                int32_t w_held = 0;
                double p_held = 0.0;
                if (!from_bidders) {
                    lw = load_fresh_u64(&buf.label[mine_col]);
                    w_held = row[mine_col];
                    p_held = s.other_dual[mine_col];
                }
                const int k0 = from + lane * 4;
                // (the labels of the slice's columns as well: whether a candidate improves one is then
                // known without a further load per candidate)
                int4 w4 = make_int4(MF_INFEASIBLE, MF_INFEASIBLE, MF_INFEASIBLE, MF_INFEASIBLE);
                double2 p01 = make_double2(0.0, 0.0), p23 = make_double2(0.0, 0.0);
                ulonglong2 l01 = make_ulonglong2(0ull, 0ull), l23 = make_ulonglong2(0ull, 0ull);
                if (k0 < reach) {
                    w4 = *(const int4 *)(row + k0);
                    p01 = *(const double2 *)(s.other_dual + k0);
                    p23 = *(const double2 *)(s.other_dual + k0 + 2);
                    l01 = *(const ulonglong2 *)(buf.label + k0);
                    l23 = *(const ulonglong2 *)(buf.label + k0 + 2);
                }
                const int to = min(line_length(s, i), reach);
                double dist, profit;
                if (from_bidders) {
                    dist = 0.0; profit = s_profit[s_alive[e]];
                } else {
                    if (lw == PATH_INF) continue;               // (cannot be: a column on a frontier has a label)
                    dist = (double)(long long)(lw >> MF_ID_BITS);
                    // the row's profit: what it holds minus that column's dual
                    profit = s.Kd * (double)w_held - p_held;
                    if (sl == 0 && lane == 0) {
                        store_through(&buf.expanded[mine_col], lw >> MF_ID_BITS);
                        __hip_atomic_store(&buf.held[i], mine_col, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        store_through((unsigned long long *)&buf.base[i], (unsigned long long)__double_as_longlong(dist + profit + s.eps));
                        if (dist + profit < bound) {                    // it may also give up and rest
                            const unsigned long long rests = ((unsigned long long)(long long)(dist + profit) << 21) |
                                                             (1ull << 20) | (unsigned long long)i;
                            atomicMin(&ctl->sink, rests);
                            atomicMin(&ctl->sink_found[p], rests);
                        }
                    }
                }
                const double base = dist + profit + s.eps;
                for (int k = k0; k < to; k += 256) {
                    if (k != k0) {
                        w4 = *(const int4 *)(row + k);
                        p01 = *(const double2 *)(s.other_dual + k);
                        p23 = *(const double2 *)(s.other_dual + k + 2);
                        l01 = *(const ulonglong2 *)(buf.label + k);
                        l23 = *(const ulonglong2 *)(buf.label + k + 2);
                    }
                    const int32_t w[4] = {w4.x, w4.y, w4.z, w4.w};
                    const double pr[4] = {p01.x, p01.y, p23.x, p23.y};
                    const unsigned long long seen[4] = {l01.x, l01.y, l23.x, l23.y};
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const double cand = base - fma(s.Kd, (double)w[q], -pr[q]);
                        if (k + q < to && w[q] != MF_INFEASIBLE && cand < bound) {
                            const unsigned long long mine = ((unsigned long long)(long long)cand << MF_ID_BITS) |
                                                            (unsigned long long)i;
                            if (lower_label(&buf.label[k + q], seen[q], mine) && cand < limit) {
                                // (both requested before either is looked at)
                                const unsigned stamped = atomicExch(&buf.stamp[k + q], step);
                                const int holder = word_id(load_fresh_u64(&s.otherword[k + q]));
                                if (stamped != step) {
                                    if (holder < 0) {                      // a column nobody holds ends a path
                                        const unsigned long long ends = (unsigned long long)(long long)cand << 21 |
                                                                        (unsigned long long)(k + q);
                                        atomicMin(&ctl->sink, ends);
                                        atomicMin(&ctl->sink_found[p], ends);
                                    } else push(k + q, holder);
                                }
                            }
                        }
                    }
                }
                if (sl == 0 && lane == 0) { ++my_scans; my_entries += (unsigned long long)line_length(s, i); }
            }
            sweep_next = from_bidders && step > 1u;     // after a re-assignment: every labelled column is due
            from_bidders = false;
        } else {
            // ---- nothing on the frontier (or everything is due): look at every column ----
            swept = true;
            sweep_next = false;
            for (int first = 0; first < s.len; first += gsize) {
                const int k = first + gtid;
                if (k < s.len) {
                    const unsigned long long lw = load_fresh_u64(&buf.label[k]);
                    const unsigned long long ex = load_fresh_u64(&buf.expanded[k]);
                    const unsigned long long d_int = lw >> MF_ID_BITS;
                    const double d = (double)(long long)d_int;
                    const int holder = lw != PATH_INF ? word_id(load_fresh_u64(&s.otherword[k])) : -1;
                    if (lw != PATH_INF && d < bound && d_int < ex) {
                        if (holder < 0)
                            atomicMin(&s_sink, (d_int << 21) | (unsigned long long)k);
                        else if (d >= limit) atomicMin(&s_low, d_int);
                        else push(k, holder);
                    }
                    // a row that has been scanned may also give its column up and rest (found when it was
                    // scanned, but path ends found before a re-assignment are forgotten with it)
                    if (pull && holder >= 0 && ex != PATH_INF) {
                        const double rests = __longlong_as_double((long long)load_fresh_u64((const unsigned long long *)&buf.base[holder])) - s.eps;
                        if (rests < bound)
                            atomicMin(&s_sink, ((unsigned long long)(long long)rests << 21) | (1ull << 20) | (unsigned long long)holder);
                    }
                }
            }
        }
        // ---- hand the workgroup's pushes, path ends and window candidates over ----
        __syncthreads();
        const unsigned pushed = min(s_pushes, (unsigned)PATH_PUSH_BUFFER);
        if (tid == 0) {
            s_base = pushed ? atomicAdd(&ctl->seg[p][segment].count, pushed) : 0u;
            if (s_sink != PATH_INF) { atomicMin(&ctl->sink, s_sink); atomicMin(&ctl->sink_found[p], s_sink); }
            if (s_low != PATH_INF) atomicMin(&ctl->low[p], s_low);
        }
        __syncthreads();
        for (unsigned t = tid; t < pushed; t += PATH_THREADS)
            store_through(&next_frontier[(size_t)segment * s.len + s_base + t], s_list[t]);
        ++my_steps;
        if (!grid_barrier(ctl, G, generation, spin_limit)) { ok = false; break; }
    }

    if ((tid & 63) == 0 && my_scans) { atomicAdd(&ctl->scans, my_scans); atomicAdd(&ctl->entries, my_entries); }
    if (gtid == 0) atomicAdd(&ctl->steps, my_steps);
    // the totals below are read by one thread after everybody's additions: one more barrier, whose
    // outcome no longer matters
    (void)grid_barrier(ctl, G, generation, spin_limit);
    if (gtid == 0) {
        if (started)
            for (int e = 0; e < n_alive; ++e)                               // whoever was not served bids again
                out_list[atomicAdd(&stats->cnt[(ring + 1) & 3], 1)] = s_row[s_alive[e]];
        for (int rest = started ? count : 0; rest < listed; ++rest)
            out_list[atomicAdd(&stats->cnt[(ring + 1) & 3], 1)] = list[rest];
        if (!ok) atomicExch(&stats->team_abort, 2);
        const unsigned long long steps = load_fresh_u64(&ctl->steps), scans = load_fresh_u64(&ctl->scans);
        stats->launch_max = steps;
        stats->bids += scans;
        stats->chain_bids += scans;
        stats->path_steps += steps;
        stats->path_scans += scans;
        stats->bytes += load_fresh_u64(&ctl->entries) * 4ull;
    }
}

}  // namespace

// Places the bidders listed in list[ring & 1] (stats->cnt[ring & 3] of them) by one search from
// all of them; whoever is not served (a wait ran out) is handed on in list[(ring + 1) & 1].
int mf_launch_path_search(mf_ctx *ctx, const SideArgs &s, int ring)
{
    PathBuffers buf{ctx->path_label, ctx->path_expanded, ctx->path_stamp,
                    {ctx->path_frontier[0], ctx->path_frontier[1]}, ctx->path_held, ctx->path_base, ctx->path_tree,
                    ctx->path_parent, ctx->path_jump};
    hipLaunchKernelGGL(path_begin_kernel, dim3(1), dim3(1), 0, ctx->stream, ctx->stats, (PathCtl *)ctx->path_ctl, ring);
    const int path_wgs = ctx->path_grid > 0 && ctx->path_grid < ctx->n_cus ? ctx->path_grid : ctx->n_cus;
    SideArgs side = s;
    if (!ctx->path_pull) side.T = nullptr;
    hipLaunchKernelGGL(path_kernel, dim3(path_wgs), dim3(PATH_THREADS), 0, ctx->stream, side,
                       ctx->list[ring & 1], ctx->list[(ring + 1) & 1], ctx->stats, (PathCtl *)ctx->path_ctl,
                       buf, ring, ctx->max_n > ctx->max_m ? ctx->max_n : ctx->max_m,
                       (double)ctx->path_width * s.eps, ctx->path_spin_limit, ctx->path_frontier_rows);
    MF_HIP(hipGetLastError());
    return MF_OK;
}
