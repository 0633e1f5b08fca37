// What a solve hands to the caller and how it is proved: the LP duals of the matching
// problem (paper: Section "Matching-based scheduling" states the problem whose optimum is asked
// for) and the certificate that matching and duals are optimal together.
#include "scan.h"
#include <mutex>

namespace {

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
// is loaded once for all of them.  The grid is capped at what the chip holds at once (8 workgroups
// on each of 256 compute units) and every workgroup walks over its share of the rows: measured on
// a 20,000 x 20,000 matrix the scan then runs at 0.70-0.73 of the HBM peak, against 0.60 with one
// workgroup per group of rows.
constexpr int CERT_ROWS = 8;
constexpr int CERT_GRID = 2048;

template <bool K32>
__global__ __launch_bounds__(BID_THREADS) void certificate_kernel(
    const int32_t *__restrict__ W, int64_t ldw, int n, int m, const int32_t *__restrict__ row2col,
    const int64_t *__restrict__ u, const int64_t *__restrict__ v, long long K, int *colmark,
    mf_cert_out *out)
{
    __shared__ long long red[BID_THREADS / 64];
    constexpr int UN = 1;               // column groups of four in flight per thread
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

}  // namespace

int mf_run_certificate(mf_ctx *ctx, const int32_t *d_W, int n, int m, int64_t ldw,
                       const int32_t *d_row2col, const int64_t *d_u, const int64_t *d_v,
                       int64_t K, mf_result *h_res)
{
    hipLaunchKernelGGL(init_cert_kernel, dim3(1), dim3(1), 0, ctx->stream, ctx->cert);
    hipLaunchKernelGGL(fill_int_kernel, dim3((m + 255) / 256), dim3(256), 0, ctx->stream, ctx->colmark, m, 0);
    const int groups = (n + CERT_ROWS - 1) / CERT_ROWS, grid = groups < CERT_GRID ? groups : CERT_GRID;
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

// Writes the caller's row2col, u and v from the solver's state.  The solve may have run in other
// coordinates (rows and columns in memory order: `staged`; the transposed problem: `flip`): the
// results then go through scratch (the searches' label arrays are idle by now) and are mapped to
// the caller's rows and columns.
int mf_extract_duals(mf_ctx *ctx, const int32_t *A, int64_t lda, int rn, int rm, double Kd, const int *line_len,
                     int n, bool flip, bool staged, int32_t *d_row2col, int64_t *d_u, int64_t *d_v)
{
    const int groups = (rn + 3) / 4, grid = groups < MAX_GRID ? groups : MAX_GRID;
    if (!flip && !staged) {
        hipLaunchKernelGGL((duals_kernel<64, 4>), dim3(grid), dim3(64), 0, ctx->stream, A, lda, rn, rm,
                           ctx->price, ctx->row2col, Kd, d_row2col, d_u, d_v, line_len);
    } else {
        int64_t *u_int = (int64_t *)ctx->path_label, *v_int = (int64_t *)ctx->path_expanded;
        hipLaunchKernelGGL((duals_kernel<64, 4>), dim3(grid), dim3(64), 0, ctx->stream, A, lda, rn, rm,
                           ctx->price, ctx->row2col, Kd, ctx->list[0], u_int, v_int, line_len);
        hipLaunchKernelGGL(fill_int_kernel, dim3((n + 255) / 256), dim3(256), 0, ctx->stream, d_row2col, n, -1);
        const int32_t *row_ids = staged ? (flip ? ctx->order_off : ctx->order_on) : nullptr;
        const int32_t *col_ids = staged ? (flip ? ctx->order_on : ctx->order_off) : nullptr;
        const int most = rn > rm ? rn : rm;
        hipLaunchKernelGGL(map_back_kernel, dim3((most + 255) / 256), dim3(256), 0, ctx->stream, rn, rm, ctx->list[0],
                           u_int, v_int, row_ids, col_ids, flip ? 1 : 0, d_row2col, d_u, d_v);
    }
    MF_HIP(hipGetLastError());
    return MF_OK;
}

namespace {

// ---- the same certificate for callers that cannot allocate ----
// Everything mf_check_certificate keeps in context scratch (the partial sums and the per-column
// use marks) lives here in one array that is part of the library's image on every device.
// In host code the array's name is only a handle: what kernels, copies and fills get is the
// device address looked up once per device.
constexpr int NOALLOC_HEADER_BYTES = 256;           // an mf_cert_out, padded
static __device__ __align__(256) unsigned char scratch[NOALLOC_HEADER_BYTES + 4 * MF_NOALLOC_MAX_COLS];

constexpr int NOALLOC_MAX_DEVICES = 64;
std::mutex noalloc_lock;
unsigned char *noalloc_ptr[NOALLOC_MAX_DEVICES];    // scratch's address on each device (null: not looked up yet)

__global__ void noalloc_begin_kernel(mf_cert_out *out, int *colmark, int m)
{
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j < m) colmark[j] = 0;
    if (j == 0) { out->primal = 0; out->dual = 0; out->min_rc = INT64_MAX; out->matched = 0; out->flags = 0; }
}

__global__ void noalloc_finish_kernel(const mf_cert_out *in, long long K, mf_certificate *d_out)
{
    const long long min_rc = in->min_rc == INT64_MAX ? 0 : in->min_rc;
    const long long gap = in->dual - K * in->primal;
    d_out->primal = in->primal;
    d_out->dual = in->dual;
    d_out->K = K;
    d_out->min_reduced_cost = min_rc;
    d_out->matched = in->matched;
    d_out->flags = in->flags;
    d_out->cert_ok = (in->flags == 0 && min_rc >= 0 && gap >= 0 && gap < K) ? 1 : 0;
    d_out->reserved = 0;
}

}  // namespace

extern "C" int mf_check_certificate_noalloc(void *hip_stream, const int32_t *d_W, int n, int m, int64_t ldw,
                                            const int32_t *d_row2col, const int64_t *d_u, const int64_t *d_v,
                                            int64_t K, mf_certificate *d_out)
{
    if (!d_W || !d_row2col || !d_u || !d_v || !d_out || n <= 0 || m <= 0 || ldw < m || (ldw & 3) ||
        ((uintptr_t)d_W & 15u) || K < 1)
        return MF_ERR_ARG;
    if (m > MF_NOALLOC_MAX_COLS || n > MF_MAX_DIM) return MF_ERR_SHAPE;
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= NOALLOC_MAX_DEVICES) return MF_ERR_HIP;
    unsigned char *base = nullptr;
    {
        std::lock_guard<std::mutex> hold(noalloc_lock);
        if (!noalloc_ptr[device]) {
            void *p = nullptr;
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return MF_ERR_HIP;
            noalloc_ptr[device] = (unsigned char *)p;
        }
        base = noalloc_ptr[device];
    }
    mf_cert_out *out = (mf_cert_out *)base;
    int *colmark = (int *)(base + NOALLOC_HEADER_BYTES);
    hipStream_t stream = (hipStream_t)hip_stream;
    // the array keeps what the previous call left: both parts are cleared by a kernel (no
    // memset node, so the sequence can be captured into a graph)
    hipLaunchKernelGGL(noalloc_begin_kernel, dim3((m + 255) / 256), dim3(256), 0, stream, out, colmark, m);
    const int groups = (n + CERT_ROWS - 1) / CERT_ROWS, grid = groups < CERT_GRID ? groups : CERT_GRID;
    hipLaunchKernelGGL(K <= INT32_MAX ? certificate_kernel<true> : certificate_kernel<false>, dim3(grid),
                       dim3(BID_THREADS), 0, stream, d_W, ldw, n, m, d_row2col, d_u, d_v, (long long)K, colmark, out);
    hipLaunchKernelGGL(noalloc_finish_kernel, dim3(1), dim3(1), 0, stream, out, (long long)K, d_out);
    return hipGetLastError() == hipSuccess ? MF_OK : MF_ERR_HIP;
}
