// Maximum-weight bipartite matching of the scored graph (paper: Algorithm
// "Scheduling algorithm", GetMatching; Section "Matching-based scheduling"
// states the problem and asks for the optimal matching).
//
// The paper solves it with the sequential Kuhn-Munkres algorithm.  Here the
// same optimum is reached by an epsilon-scaling forward/reverse auction, whose
// unit of work - "scan one line of the weight matrix against the current duals
// and keep the best two" - is a coalesced streaming read, and whose updates are
// 64-bit atomic maxima.  Weights are multiplied by K = n + 1 so that the final
// epsilon = 1 is below 1/n of a weight unit: the matching is then exactly
// optimal, and the duals it leaves behind prove it (see certificate_kernel).
//
// Formulation.  maximise sum W_ij x_ij, every row and column used at most
// once.  Dual: minimise sum pi_i + sum p_j with pi_i + p_j >= K W_ij, pi, p >= 0.
// The auction keeps, for the current epsilon,
//   (I1) pi_i + p_j >= K W_ij - eps on every feasible pair,
//   (I2) pi_i + p_j  = K W_ij      on every assigned pair,
// and stops a phase when every unassigned row has pi_i = 0 and every
// unassigned column has p_j = 0; then the assignment is within n*eps of the
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
    double b1, b2;
    int idx;
};

__device__ inline void top2_push(Top2 &t, double val, int j)
{
    t.b2 = fmax(t.b2, fmin(val, t.b1));
    t.idx = val > t.b1 ? j : t.idx;
    t.b1 = fmax(t.b1, val);
}

__device__ inline void top2_merge(Top2 &t, double ob1, double ob2, int oidx)
{
    const double nb2 = fmax(fmax(t.b2, ob2), fmin(t.b1, ob1));
    const bool take = (ob1 > t.b1) || (ob1 == t.b1 && oidx < t.idx);
    t.idx = take ? oidx : t.idx;
    t.b1 = fmax(t.b1, ob1);
    t.b2 = nb2;
}

// Scans line `A[0..len)` against `dual[0..len)` and leaves, in every thread of
// the block, the best and second-best value of K*w - dual and the smallest
// index attaining the best.  `A` is 16-byte aligned and padded to a multiple
// of four entries; `dual` likewise.
__device__ inline Top2 scan_line(const int32_t *__restrict__ A, const double *__restrict__ dual,
                                 int len, double Kd, Top2 *red)
{
    Top2 t{NEG_HUGE, NEG_HUGE, 0x7fffffff};
    for (int j = threadIdx.x * 4; j < len; j += BID_THREADS * 4) {
        const int4 w = *(const int4 *)(A + j);
        const double2 p01 = *(const double2 *)(dual + j);
        const double2 p23 = *(const double2 *)(dual + j + 2);
        double v0 = fma(Kd, (double)w.x, -p01.x);
        double v1 = fma(Kd, (double)w.y, -p01.y);
        double v2 = fma(Kd, (double)w.z, -p23.x);
        double v3 = fma(Kd, (double)w.w, -p23.y);
        if (j + 3 >= len) {
            if (j + 1 >= len) v1 = NEG_HUGE;
            if (j + 2 >= len) v2 = NEG_HUGE;
            v3 = NEG_HUGE;
        }
        top2_push(t, v0, j);
        top2_push(t, v1, j + 1);
        top2_push(t, v2, j + 2);
        top2_push(t, v3, j + 3);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const double ob1 = __shfl_xor(t.b1, off);
        const double ob2 = __shfl_xor(t.b2, off);
        const int oidx = __shfl_xor(t.idx, off);
        top2_merge(t, ob1, ob2, oidx);
    }
    const int wave = threadIdx.x >> 6;
    __syncthreads();                       // protect `red` from the previous line
    if ((threadIdx.x & 63) == 0) red[wave] = t;
    __syncthreads();
    Top2 r = red[0];
#pragma unroll
    for (int wv = 1; wv < BID_THREADS / 64; ++wv) top2_merge(r, red[wv].b1, red[wv].b2, red[wv].idx);
    return r;
}

// One bidding round for the side whose members are listed in `list`.
//   A          that side's lines of the weight matrix (W for rows, W^T for columns)
//   other_dual duals of the opposite side (read), otherword their packed (dual, holder)
//   own_*      this side's dual, packed word and partner index
// A bidder whose best value is at most eps rests with dual 0.  Otherwise it
// offers the opposite workload the highest dual at which that workload is
// still within eps of the bidder's best alternative.
__global__ __launch_bounds__(BID_THREADS) void bid_kernel(
    const int32_t *__restrict__ A, int64_t pitch, int len, const double *__restrict__ other_dual,
    unsigned long long *__restrict__ otherword, double *__restrict__ own_dual,
    unsigned long long *__restrict__ ownword, int *__restrict__ own2other,
    int *__restrict__ tent_tgt, double *__restrict__ tent_keep, const int *__restrict__ list,
    int *__restrict__ cnt, int cur, double eps, double Kd, mf_device_stats *stats)
{
    __shared__ Top2 red[BID_THREADS / 64];
    const int count = cnt[cur];
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        cnt[cur ^ 1] = 0;                  // the list the settle step of this round will fill
        if (count > 0) {
            stats->rounds += 1ull;
            stats->bids += (unsigned long long)count;
            stats->bytes += (unsigned long long)count * (unsigned long long)len * 4ull;
        }
    }
    for (int item = blockIdx.x; item < count; item += gridDim.x) {
        const int b = list[item];
        const Top2 t = scan_line(A + (size_t)b * pitch, other_dual, len, Kd, red);
        if (threadIdx.x == 0) {
            if (t.b1 <= eps) {
                own_dual[b] = 0.0;
                ownword[b] = 0ull;
                own2other[b] = -1;
                tent_tgt[b] = -1;
            } else {
                const double keep = fmax(t.b2 - eps, 0.0);
                const double offer = t.b1 + other_dual[t.idx] - keep;    // K*w - keep
                atomicMax(&otherword[t.idx], pack_word(offer, b + 1));
                tent_tgt[b] = t.idx;
                tent_keep[b] = keep;
            }
        }
    }
}

// Resolves a bidding round: the holder recorded in the target's word won.
__global__ void settle_kernel(const unsigned long long *__restrict__ otherword,
                              double *__restrict__ other_dual, int *__restrict__ other2own,
                              double *__restrict__ own_dual, unsigned long long *__restrict__ ownword,
                              int *__restrict__ own2other, const int *__restrict__ tent_tgt,
                              const double *__restrict__ tent_keep, const int *__restrict__ list,
                              int *__restrict__ next, int *__restrict__ cnt, int cur)
{
    const int count = cnt[cur];
    for (int item = blockIdx.x * blockDim.x + threadIdx.x; item < count; item += gridDim.x * blockDim.x) {
        const int b = list[item];
        const int tgt = tent_tgt[b];
        if (tgt < 0) continue;                                   // resting
        const unsigned long long word = otherword[tgt];
        if (word_id(word) == b) {
            const int old = other2own[tgt];
            if (old >= 0) {
                own2other[old] = -1;
                const double d = own_dual[old];
                ownword[old] = pack_word(d, 0);
                if (d > 0.0) next[atomicAdd(&cnt[cur ^ 1], 1)] = old;
            }
            other2own[tgt] = b;
            own2other[b] = tgt;
            other_dual[tgt] = word_dual(word);
            own_dual[b] = tent_keep[b];
            ownword[b] = pack_word(tent_keep[b], tgt + 1);
        } else {
            next[atomicAdd(&cnt[cur ^ 1], 1)] = b;
        }
    }
}

// Start of an epsilon phase: drop the assignment, keep the duals, all rows bid.
__global__ void reset_kernel(int n, int m, const double *__restrict__ price,
                             const double *__restrict__ profit, unsigned long long *colword,
                             unsigned long long *roword, int *row2col, int *col2row, int *list,
                             int *cnt)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) { row2col[i] = -1; roword[i] = pack_word(profit[i], 0); list[i] = i; }
    if (i < m) { col2row[i] = -1; colword[i] = pack_word(price[i], 0); }
    if (i == 0) { cnt[0] = n; cnt[1] = 0; }
}

// After the forward rounds: unassigned columns that still carry a price must bid.
__global__ void reverse_list_kernel(int m, const double *__restrict__ price,
                                    const int *__restrict__ col2row, int *list, int *cnt)
{
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j < m && col2row[j] < 0 && price[j] > 0.0) list[atomicAdd(&cnt[0], 1)] = j;
}

__global__ void clear_counts_kernel(int *cnt) { cnt[0] = 0; cnt[1] = 0; }

// W^T (for the reverse rounds' coalesced column scans) and the largest weight.
__global__ void transpose_kernel(const int32_t *__restrict__ W, int n, int m, int64_t ldw,
                                 int32_t *__restrict__ WT, int64_t ldt, mf_device_stats *stats)
{
    __shared__ int32_t tile[64][65];
    const int bx = blockIdx.x * 64, by = blockIdx.y * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;     // 256 threads: 4 rows per pass
    int mx = 0;
    for (int r = ty; r < 64; r += 4) {
        const int i = by + r, j = bx + tx;
        int32_t w = MF_INFEASIBLE;
        if (i < n && j < m) w = W[(size_t)i * ldw + j];
        tile[r][tx] = w;
        mx = max(mx, w);
    }
    __syncthreads();
    for (int r = ty; r < 64; r += 4) {
        const int j = bx + r, i = by + tx;
        if (j < m && i < n) WT[(size_t)j * ldt + i] = tile[tx][r];
    }
    for (int off = 32; off >= 1; off >>= 1) mx = max(mx, __shfl_xor(mx, off));
    if ((threadIdx.x & 63) == 0 && mx > 0) atomicMax(&stats->max_weight, mx);
}

// Duals handed to the caller: v_j = p_j and the tightest row dual the prices
// allow, u_i = max(0, max_j (K W_ij - p_j)).
__global__ __launch_bounds__(BID_THREADS) void duals_kernel(
    const int32_t *__restrict__ W, int64_t ldw, int n, int m, const double *__restrict__ price,
    const int *__restrict__ row2col, double Kd, int32_t *__restrict__ out_row2col,
    int64_t *__restrict__ u, int64_t *__restrict__ v)
{
    __shared__ Top2 red[BID_THREADS / 64];
    for (int i = blockIdx.x; i < n; i += gridDim.x) {
        const Top2 t = scan_line(W + (size_t)i * ldw, price, m, Kd, red);
        if (threadIdx.x == 0) {
            u[i] = (int64_t)fmax(t.b1, 0.0);
            out_row2col[i] = row2col[i];
        }
    }
    for (int j = blockIdx.x * blockDim.x + threadIdx.x; j < m; j += gridDim.x * blockDim.x)
        v[j] = (int64_t)price[j];
}

// The proof of optimality, evaluated for arbitrary caller-supplied integers:
// matching valid, duals non-negative, every feasible pair covered
// (min reduced cost), primal and dual totals.
__global__ __launch_bounds__(BID_THREADS) void certificate_kernel(
    const int32_t *__restrict__ W, int64_t ldw, int n, int m, const int32_t *__restrict__ row2col,
    const int64_t *__restrict__ u, const int64_t *__restrict__ v, long long K, int *colmark,
    mf_cert_out *out)
{
    __shared__ long long red[BID_THREADS / 64];
    long long dual_part = 0, primal_part = 0;
    int flags = 0, matched = 0;
    long long min_rc = INT64_MAX;
    for (int i = blockIdx.x; i < n; i += gridDim.x) {
        const long long ui = u[i];
        const int32_t *row = W + (size_t)i * ldw;
        for (int j = threadIdx.x * 4; j < m; j += BID_THREADS * 4) {
            const int4 w4 = *(const int4 *)(row + j);
            const int32_t w[4] = {w4.x, w4.y, w4.z, w4.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (j + e < m && w[e] != MF_INFEASIBLE) {
                    const long long rc = ui + v[j + e] - K * (long long)w[e];
                    min_rc = rc < min_rc ? rc : min_rc;
                }
            }
        }
        if (threadIdx.x == 0) {
            if (ui < 0) flags |= 4;
            dual_part += ui;
            const int j = row2col[i];
            if (j != -1) {
                if (j < 0 || j >= m) flags |= 1;
                else {
                    if (atomicAdd(&colmark[j], 1) != 0) flags |= 1;
                    const int32_t w = row[j];
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

__global__ void init_cert_kernel(mf_cert_out *out)
{
    out->primal = 0; out->dual = 0; out->min_rc = INT64_MAX; out->matched = 0; out->flags = 0;
}

__global__ void init_solver_kernel(int n, int m, double *price, double *profit, mf_device_stats *stats)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n + 4) profit[i] = 0.0;
    if (i < m + 4) price[i] = 0.0;
    if (i == 0) { stats->rounds = 0; stats->bids = 0; stats->bytes = 0; stats->max_weight = 0; }
}

struct Side {
    const int32_t *A;
    int64_t pitch;
    int len;
    double *own_dual, *other_dual;
    unsigned long long *ownword, *otherword;
    int *own2other, *other2own;
};

// Runs bidding rounds for one side until nobody is left to bid.  `count` is
// the number of bidders in list[0].  Returns MF_OK or an error.
int run_side(mf_ctx *ctx, const Side &s, int count, double eps, double Kd, int64_t *rounds_left,
             bool time_first)
{
    int cur = 0;
    while (count > 0) {
        const int batch = count > 2048 ? 1 : (count > 128 ? 4 : 16);
        if (*rounds_left < batch) return MF_ERR_NOT_CONVERGED;
        *rounds_left -= batch;
        const int grid = count < MAX_GRID ? count : MAX_GRID;
        const int sgrid = (count + 255) / 256 < 64 ? (count + 255) / 256 : 64;
        for (int r = 0; r < batch; ++r) {
            if (time_first && r == 0) MF_HIP(hipEventRecord(ctx->ev[6], ctx->stream));
            hipLaunchKernelGGL(bid_kernel, dim3(grid), dim3(BID_THREADS), 0, ctx->stream, s.A, s.pitch,
                               s.len, s.other_dual, s.otherword, s.own_dual, s.ownword, s.own2other,
                               ctx->tent_tgt, ctx->tent_keep, ctx->list[cur], ctx->cnt, cur, eps, Kd,
                               ctx->stats);
            if (time_first && r == 0) MF_HIP(hipEventRecord(ctx->ev[7], ctx->stream));
            hipLaunchKernelGGL(settle_kernel, dim3(sgrid), dim3(256), 0, ctx->stream, s.otherword,
                               s.other_dual, s.other2own, s.own_dual, s.ownword, s.own2other,
                               ctx->tent_tgt, ctx->tent_keep, ctx->list[cur], ctx->list[cur ^ 1],
                               ctx->cnt, cur);
            cur ^= 1;
        }
        MF_HIP(hipGetLastError());
        MF_HIP(hipMemcpyAsync(ctx->h_cnt, ctx->cnt, 2 * sizeof(int), hipMemcpyDeviceToHost, ctx->stream));
        MF_HIP(hipStreamSynchronize(ctx->stream));
        if (time_first) {
            float ms = 0.0f;
            MF_HIP(hipEventElapsedTime(&ms, ctx->ev[6], ctx->ev[7]));
            ctx->timings[T_BID_BULK] += ms;
            ctx->timings[T_BID_BULK_LAUNCHES] += 1.0f;
            ctx->timings[T_BID_BULK_BYTES] += (float)((double)count * s.len * 4.0);
            time_first = false;
        }
        count = ctx->h_cnt[cur];
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
    const int grid = n < MAX_GRID ? n : MAX_GRID;
    hipLaunchKernelGGL(certificate_kernel, dim3(grid), dim3(BID_THREADS), 0, ctx->stream, d_W, ldw, n, m,
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

int mf_run_solver(mf_ctx *ctx, const int32_t *d_W, int n, int m, int64_t ldw,
                  int32_t *d_row2col, int64_t *d_u, int64_t *d_v, mf_result *h_res)
{
    const int64_t ldt = ((int64_t)n + 3) & ~3ll;
    const long long K = (long long)n + 1;
    const double Kd = (double)K;
    const int nm = n > m ? n : m;

    MF_HIP(hipEventRecord(ctx->ev[3], ctx->stream));
    hipLaunchKernelGGL(init_solver_kernel, dim3((nm + 4 + 255) / 256), dim3(256), 0, ctx->stream, n, m,
                       ctx->price, ctx->profit, ctx->stats);
    hipLaunchKernelGGL(transpose_kernel, dim3((m + 63) / 64, (n + 63) / 64), dim3(256), 0, ctx->stream,
                       d_W, n, m, ldw, ctx->wt, ldt, ctx->stats);
    MF_HIP(hipGetLastError());
    MF_HIP(hipEventRecord(ctx->ev[4], ctx->stream));
    MF_HIP(hipMemcpyAsync(ctx->h_stats, ctx->stats, sizeof(mf_device_stats), hipMemcpyDeviceToHost, ctx->stream));
    MF_HIP(hipStreamSynchronize(ctx->stream));
    {
        float ms = 0.0f;
        MF_HIP(hipEventElapsedTime(&ms, ctx->ev[3], ctx->ev[4]));
        ctx->timings[T_TRANSPOSE] = ms;
    }
    const long long cmax = K * (long long)ctx->h_stats->max_weight;
    if (cmax >= MF_MAX_DUAL) return MF_ERR_RANGE;

    const Side fwd{d_W, ldw, m, ctx->profit, ctx->price, ctx->roword, ctx->colword, ctx->row2col, ctx->col2row};
    const Side rev{ctx->wt, ldt, n, ctx->price, ctx->profit, ctx->colword, ctx->roword, ctx->col2row, ctx->row2col};

    long long eps = cmax / ctx->theta;
    if (eps < 1) eps = 1;
    int64_t rounds_left = ctx->max_rounds;
    int phases = 0;
    for (;;) {
        ++phases;
        hipLaunchKernelGGL(reset_kernel, dim3((nm + 255) / 256), dim3(256), 0, ctx->stream, n, m, ctx->price,
                           ctx->profit, ctx->colword, ctx->roword, ctx->row2col, ctx->col2row,
                           ctx->list[0], ctx->cnt);
        int rc = run_side(ctx, fwd, n, (double)eps, Kd, &rounds_left, true);
        if (rc != MF_OK) return rc;
        hipLaunchKernelGGL(clear_counts_kernel, dim3(1), dim3(1), 0, ctx->stream, ctx->cnt);
        hipLaunchKernelGGL(reverse_list_kernel, dim3((m + 255) / 256), dim3(256), 0, ctx->stream, m,
                           ctx->price, ctx->col2row, ctx->list[0], ctx->cnt);
        MF_HIP(hipMemcpyAsync(ctx->h_cnt, ctx->cnt, 2 * sizeof(int), hipMemcpyDeviceToHost, ctx->stream));
        MF_HIP(hipStreamSynchronize(ctx->stream));
        rc = run_side(ctx, rev, ctx->h_cnt[0], (double)eps, Kd, &rounds_left, false);
        if (rc != MF_OK) return rc;
        if (eps == 1) break;
        eps /= ctx->theta;
        if (eps < 1) eps = 1;
    }
    MF_HIP(hipEventRecord(ctx->ev[4], ctx->stream));
    {
        const int grid = n < MAX_GRID ? n : MAX_GRID;
        hipLaunchKernelGGL(duals_kernel, dim3(grid), dim3(BID_THREADS), 0, ctx->stream, d_W, ldw, n, m,
                           ctx->price, ctx->row2col, Kd, d_row2col, d_u, d_v);
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
    h_res->phases = phases;
    h_res->ms_solve = ms_solve;
    h_res->ms_certify = ms_duals + ms_cert;
    return h_res->cert_ok ? MF_OK : MF_ERR_CERT;
}
