// The last bidders of an auction run, placed by shortest-augmenting-path searches that the
// whole device runs together (paper: Algorithm "Scheduling algorithm", GetMatching; the
// searches are the successive-shortest-path step of the Hungarian method the paper uses,
// applied to the few bidders whose chains of bids would otherwise go on for thousands of steps).
#include "scan.h"

namespace {

// A chain of bids is a greedy walk: every evicted holder moves to its own best
// alternative, and with one or two bidders left such a walk takes thousands of
// dependent steps to reach a free line.  The shortest way to make room is far
// shorter in hops, and finding it is a breadth-type search whose every step is
// wide.  For a bidder r, in the notation of the header of auction.hip with
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
    // Complete paths found during a step, per slot like `low`: `sink` above moves while a step
    // runs, so two workgroups reading it at the top of the same step may see different values;
    // whether the search is over must not depend on that, or they would leave it at different
    // barriers.  Every workgroup folds the slot the previous step filled (nobody writes it any
    // more) into a running minimum of its own, and all take the decision from that.
    unsigned long long sink_found[3];
    // best value of the current bidder (bits of a double), by parity of its position in the list:
    // when a bidder rests, workgroup 0 may already be writing the next bidder's value while a
    // slower workgroup has yet to read this one
    unsigned long long first_value[2];
    // The barrier's two hot words each have a cache line to themselves: hundreds of polling loads
    // on the line of a counter that is being incremented (or of the sink above) slow both down.
    struct alignas(128) { unsigned int count; } arrive;       // whole groups that have arrived at barriers so far
    struct alignas(128) { unsigned int number; } open;        // barriers completed so far | PATH_GAVE_UP
    alignas(128) unsigned long long steps;
    unsigned long long scans, entries;
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
    ctl->arrive.count = 0u; ctl->open.number = 0u; ctl->steps = 0ull; ctl->scans = 0ull; ctl->entries = 0ull;
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
                store_through(&ctl->sink_found[0], PATH_INF);
                store_through(&ctl->sink_found[1], PATH_INF);
                store_through(&ctl->sink_found[2], PATH_INF);
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
        // shortest complete path every workgroup agrees on: first "the bidder rests", as workgroup 0 wrote it
        unsigned long long agreed_sink = ((unsigned long long)(long long)first_profit << 21) | (1ull << 20) |
                                         (unsigned long long)r0;

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
            if (step > 1u) {
                const unsigned long long found = load_fresh_u64(&ctl->sink_found[c]);
                agreed_sink = found < agreed_sink ? found : agreed_sink;
            }
            // pruning may use whatever is known by now; decisions all workgroups must share may not
            const unsigned long long sink_word = min(agreed_sink, load_fresh_u64(&ctl->sink));
            const double bound = (double)(long long)(sink_word >> 21);
            if (step > 1u && swept && nf == 0) {
                const unsigned long long lo = load_fresh_u64(&ctl->low[c]);
                if (lo == PATH_INF || lo >= (agreed_sink >> 21)) break;     // every label below the sink is final
                low = (double)(long long)lo;                                // move the window to the next label
            }
            if (nf > PATH_FRONTIER_HIGH) width = fmax(s.eps, width * 0.5);
            else if (nf < PATH_FRONTIER_LOW) width = fmin(width_max, width * 2.0);
            const double limit = fmin(low + width, bound);
            if (gtid < PATH_SEGMENTS)
                __hip_atomic_store(&ctl->seg[z][gtid].count, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (gtid == 0) { store_through(&ctl->low[z], PATH_INF); store_through(&ctl->sink_found[z], PATH_INF); }
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
                            if (dist + profit < bound) {                    // it may also give up and rest
                                const unsigned long long rests = ((unsigned long long)(long long)(dist + profit) << 21) |
                                                                 (1ull << 20) | (unsigned long long)i;
                                atomicMin(&ctl->sink, rests);
                                atomicMin(&ctl->sink_found[p], rests);
                            }
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
                                    if (word_id(load_fresh_u64(&s.otherword[k + q])) < 0) {  // a column nobody holds ends a path
                                        const unsigned long long ends = (unsigned long long)(long long)cand << 21 |
                                                                        (unsigned long long)(k + q);
                                        atomicMin(&ctl->sink, ends);
                                        atomicMin(&ctl->sink_found[p], ends);
                                    } else push(k + q);
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
                if (s_sink != PATH_INF) { atomicMin(&ctl->sink, s_sink); atomicMin(&ctl->sink_found[p], s_sink); }
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

}  // namespace

// Places the bidders listed in list[ring & 1] (stats->cnt[ring & 3] of them) one after another;
// whoever is not served (a wait ran out) is handed on in list[(ring + 1) & 1].
int mf_launch_path_search(mf_ctx *ctx, const SideArgs &s, int ring)
{
    PathBuffers buf{ctx->path_label, ctx->path_expanded, ctx->path_stamp,
                    {ctx->path_frontier[0], ctx->path_frontier[1]}, ctx->path_held};
    hipLaunchKernelGGL(path_begin_kernel, dim3(1), dim3(1), 0, ctx->stream, ctx->stats, (PathCtl *)ctx->path_ctl, ring);
    const int path_wgs = ctx->path_grid > 0 && ctx->path_grid < ctx->n_cus ? ctx->path_grid : ctx->n_cus;
    hipLaunchKernelGGL(path_kernel, dim3(path_wgs), dim3(PATH_THREADS), 0, ctx->stream, s,
                       ctx->list[ring & 1], ctx->list[(ring + 1) & 1], ctx->stats, (PathCtl *)ctx->path_ctl,
                       buf, ring, ctx->max_n > ctx->max_m ? ctx->max_n : ctx->max_m,
                       (double)ctx->path_width * s.eps, ctx->path_spin_limit);
    MF_HIP(hipGetLastError());
    return MF_OK;
}
