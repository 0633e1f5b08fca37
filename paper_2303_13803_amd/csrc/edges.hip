// The graph as edge lists (paper: Algorithm "Scheduling algorithm" builds its bipartite graph
// edge by edge with AddEdge, and which pairs may share a GPU need not follow any pattern -
// offline workloads only go to healthy GPUs, Section "Efficient and safe space-sharing").
//
// A caller-brought weight matrix in which most pairs are marked infeasible is turned into one list
// per row of (column, weight) for the pairs that remain, and the bidding rounds with many bidders -
// the part of the matching that is bound by memory bandwidth - read those lists instead of the
// rows: 8 bytes per feasible pair instead of 4 bytes per pair.  The few bidders at the end of a
// run, whose steps are bound by latency, and the final passes (duals, certificate) keep reading
// the matrix itself.
#include "scan.h"

namespace {

constexpr int LIST_LINES_PER_WORKGROUP = 128;

// Per row: how many pairs are feasible (rounded up to a multiple of four: lists are read 16 bytes
// at a time); the total, and the largest weight (which sets the first epsilon).
__global__ __launch_bounds__(256) void edge_count_kernel(const int32_t *__restrict__ W, int n, int m, int64_t ldw,
                                                         int *__restrict__ padded_count, unsigned long long *total,
                                                         mf_device_stats *stats)
{
    __shared__ int s_part[4];
    __shared__ unsigned long long s_total;
    if (threadIdx.x == 0) s_total = 0ull;
    int mx = 0;
    for (int i = blockIdx.x; i < n; i += gridDim.x) {
        const int32_t *row = W + (size_t)i * ldw;
        int mine = 0;
        for (int j = threadIdx.x * 4; j < m; j += 1024) {
            const int4 v = *(const int4 *)(row + j);               // the pitch is a multiple of four
            const int32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (j + e < m && w[e] != MF_INFEASIBLE) { ++mine; mx = max(mx, w[e]); }
        }
        for (int off = 32; off >= 1; off >>= 1) mine += __shfl_xor(mine, off);
        __syncthreads();
        if ((threadIdx.x & 63) == 0) s_part[threadIdx.x >> 6] = mine;
        __syncthreads();
        if (threadIdx.x == 0) {
            const int count = s_part[0] + s_part[1] + s_part[2] + s_part[3];
            padded_count[i] = (count + 3) & ~3;
            s_total += (unsigned long long)count;
        }
    }
    for (int off = 32; off >= 1; off >>= 1) mx = max(mx, __shfl_xor(mx, off));
    if ((threadIdx.x & 63) == 0 && mx > stats->max_weight) atomicMax(&stats->max_weight, mx);
    __syncthreads();
    if (threadIdx.x == 0 && s_total) atomicAdd(total, s_total);
}

// Where each row's list starts: running sums of the padded counts (one workgroup).
__global__ __launch_bounds__(1024) void edge_offsets_kernel(const int *__restrict__ padded_count, int n, long long *__restrict__ start)
{
    __shared__ long long s_sum[1024];
    const int per = (n + 1023) / 1024, first = threadIdx.x * per;
    long long mine = 0;
    for (int i = first; i < min(first + per, n); ++i) mine += padded_count[i];
    s_sum[threadIdx.x] = mine;
    __syncthreads();
    if (threadIdx.x == 0) {
        long long run = 0;
        for (int t = 0; t < 1024; ++t) { const long long v = s_sum[t]; s_sum[t] = run; run += v; }
        start[n] = run;
    }
    __syncthreads();
    long long run = s_sum[threadIdx.x];
    for (int i = first; i < min(first + per, n); ++i) { start[i] = run; run += padded_count[i]; }
}

// The lists themselves, columns in ascending order; the padding of a list holds (0, infeasible).
__global__ __launch_bounds__(256) void edge_fill_kernel(const int32_t *__restrict__ W, int n, int m, int64_t ldw,
                                                        const long long *__restrict__ start, int *__restrict__ col,
                                                        int32_t *__restrict__ weight)
{
    __shared__ int s_wave[4];
    __shared__ long long s_at;
    for (int i = blockIdx.x; i < n; i += gridDim.x) {
        const int32_t *row = W + (size_t)i * ldw;
        __syncthreads();
        if (threadIdx.x == 0) s_at = start[i];
        __syncthreads();
        for (int j0 = 0; j0 < m; j0 += 1024) {
            const int j = j0 + threadIdx.x * 4;
            int32_t w[4] = {MF_INFEASIBLE, MF_INFEASIBLE, MF_INFEASIBLE, MF_INFEASIBLE};
            if (j < m) { const int4 v = *(const int4 *)(row + j); w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w; }
            int mine = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) mine += (j + e < m && w[e] != MF_INFEASIBLE) ? 1 : 0;
            int before = mine;                                  // inclusive sums within the wavefront
            for (int d = 1; d < 64; d <<= 1) { const int o = __shfl_up(before, d); if ((int)(threadIdx.x & 63) >= d) before += o; }
            if ((threadIdx.x & 63) == 63) s_wave[threadIdx.x >> 6] = before;
            __syncthreads();
            int ahead = 0;
            for (int wv = 0; wv < (int)(threadIdx.x >> 6); ++wv) ahead += s_wave[wv];
            long long at = s_at + ahead + before - mine;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (j + e < m && w[e] != MF_INFEASIBLE) { col[at] = j + e; weight[at] = w[e]; ++at; }
            __syncthreads();
            if (threadIdx.x == 0) s_at += s_wave[0] + s_wave[1] + s_wave[2] + s_wave[3];
            __syncthreads();
        }
        const long long end = start[i + 1];
        for (long long at = s_at + threadIdx.x; at < end; at += 256) { col[at] = 0; weight[at] = MF_INFEASIBLE; }
    }
}

__device__ __forceinline__ void top2_push4_at(double &b1, double &b2, int &idx, int &wbest, double v0, double v1,
                                              double v2, double v3, const int4 &c, const int4 &w, int salt)
{
    const double hi0 = fmax(v0, v1), lo0 = fmin(v0, v1);
    const double hi1 = fmax(v2, v3), lo1 = fmin(v2, v3);
    const double g1 = fmax(hi0, hi1);
    const double g2 = fmax(fmin(hi0, hi1), fmax(lo0, lo1));
    if (g1 > b1) {                                      // the first entry attaining the group's best
        const bool a0 = v0 == g1, a1 = v1 == g1, a2 = v2 == g1;
        idx = (a0 ? c.x : a1 ? c.y : a2 ? c.z : c.w) ^ salt;
        wbest = a0 ? w.x : a1 ? w.y : a2 ? w.z : w.w;
    }
    b2 = fmax(fmax(b2, g2), fmin(b1, g1));
    b1 = fmax(b1, g1);
}

// One round for many bidders, each reading its list: one wavefront per bidder.  Otherwise as
// round_kernel (same bids, same lists of bidders to pass on, same ring of counters).
__global__ __launch_bounds__(64) void round_lists_kernel(SideArgs s, const int *__restrict__ list,
                                                         int *__restrict__ next, mf_device_stats *stats, int ring)
{
    __shared__ int s_hold[LIST_LINES_PER_WORKGROUP];
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
    int held = 0;
    unsigned long long entries = 0;
    const int lane = threadIdx.x;
    for (int item = blockIdx.x; item < count; item += gridDim.x) {
        const int b = list[item];
        const int salt = tie_salt(b);
        const long long from = s.edge_start[b], to = s.edge_start[b + 1];
        entries += (unsigned long long)(to - from);
        Top2 t{NEG_HUGE, NEG_HUGE, 0x7fffffff, 0};
#pragma unroll 2
        for (long long e = from + lane * 4; e < to; e += 256) {
            const int4 c = *(const int4 *)(s.edge_col + e);
            const int4 w = *(const int4 *)(s.edge_weight + e);
            const double p0 = s.other_dual[c.x], p1 = s.other_dual[c.y], p2 = s.other_dual[c.z], p3 = s.other_dual[c.w];
            top2_push4_at(t.b1, t.b2, t.idx, t.w, fma(s.Kd, (double)w.x, -p0), fma(s.Kd, (double)w.y, -p1),
                          fma(s.Kd, (double)w.z, -p2), fma(s.Kd, (double)w.w, -p3), c, w, salt);
        }
        t = wave_top2(t);
        int again = -1;
        if (lane == 0) {
            t.idx ^= salt;
            again = decide_and_bid<true>(s, b, t);
            if (again >= 0) s_hold[held] = again;
        }
        held += __shfl(again >= 0 ? 1 : 0, 0);
    }
    if (held > 0) {
        int base = 0;
        if (lane == 0) base = atomicAdd(ncnt, held);
        base = __shfl(base, 0);
        for (int k = lane; k < held; k += 64) next[base + k] = s_hold[k];
    }
    if (lane == 0 && entries) atomicAdd(&stats->round_bytes, entries * 8ull);
}

}  // namespace

// First pass over a matrix the caller brings: per-row counts of feasible pairs, their total (left
// in ctx->feasible_pairs) and the largest weight (in the statistics block, as max_weight_kernel
// leaves it).
int mf_count_edges(mf_ctx *ctx, const int32_t *d_W, int n, int m, int64_t ldw)
{
    hipLaunchKernelGGL(edge_count_kernel, dim3(n < 4096 ? n : 4096), dim3(256), 0, ctx->stream, d_W, n, m, ldw,
                       ctx->edge_count, ctx->feasible_pairs, ctx->stats);
    MF_HIP(hipGetLastError());
    return MF_OK;
}

// The lists, in the memory of the context's memory-ordered copy of the matrix (which a matrix the
// caller brings has no use for): columns in its first half, weights in its second.
int mf_build_edge_lists(mf_ctx *ctx, const int32_t *d_W, int n, int m, int64_t ldw, SideArgs *side)
{
    const size_t capacity = mf_edge_capacity(ctx);
    int *col = (int *)ctx->staged;
    int32_t *weight = ctx->staged + capacity;
    ctx->staged_n = ctx->staged_m = 0;                          // whatever was staged there is gone
    hipLaunchKernelGGL(edge_offsets_kernel, dim3(1), dim3(1024), 0, ctx->stream, ctx->edge_count, n, ctx->edge_start);
    hipLaunchKernelGGL(edge_fill_kernel, dim3(n < 8192 ? n : 8192), dim3(256), 0, ctx->stream, d_W, n, m, ldw,
                       ctx->edge_start, col, weight);
    MF_HIP(hipGetLastError());
    side->edge_start = ctx->edge_start;
    side->edge_col = col;
    side->edge_weight = weight;
    return MF_OK;
}

void mf_launch_list_round(mf_ctx *ctx, const SideArgs &s, int count, int ring)
{
    int grid = count < MAX_GRID ? count : MAX_GRID;
    if ((long long)grid * LIST_LINES_PER_WORKGROUP < count) grid = (count + LIST_LINES_PER_WORKGROUP - 1) / LIST_LINES_PER_WORKGROUP;
    hipLaunchKernelGGL(round_lists_kernel, dim3(grid), dim3(64), 0, ctx->stream, s, ctx->list[ring & 1],
                       ctx->list[(ring + 1) & 1], ctx->stats, ring);
}
