// Edge weights for every online x offline pair (paper: Algorithm "Scheduling
// algorithm", the loop that calls CalcNormTput and AddEdge; Section
// "Matching-based scheduling" for the predictor's inputs and output).
//
// The predictor is an MLP 2F -> H -> H -> 1 over [online ; offline] features.
// Its first layer is linear in the concatenation, so it splits exactly into a
// per-online and a per-offline projection that are computed once per workload:
//     W1 [x_u ; x_v] + b1 = (W1[:, :F] x_u + b1) + (W1[:, F:] x_v).
// The pair kernel then only adds the two projections, applies ReLU, and runs
// the H x H hidden layer on the matrix cores with pairs along the N axis of
// the MFMA tile, so each lane ends up owning whole pairs and the output layer,
// logistic, quantisation and memory-fit mask run in registers before one
// coalesced int32 store.
#include "internal.h"
#include <math.h>
#include <type_traits>

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
union Half8Words { half8 v; unsigned int u[4]; uint4 q; };

namespace {

__global__ void project_kernel(const float *__restrict__ X, int rows, int F,
                               const float *__restrict__ W1, int col_off,
                               const float *__restrict__ bias, int H, float *__restrict__ P)
{
    long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long)rows * H) return;
    int r = (int)(idx / H), k = (int)(idx % H);
    const float *x = X + (size_t)r * F;
    const float *w = W1 + (size_t)k * 2 * F + col_off;
    float s = bias ? bias[k] : 0.0f;
    for (int t = 0; t < F; ++t) s = fmaf(x[t], w[t], s);
    P[idx] = s;
}

// order[k] = the workload with the k-th smallest key (ties by index).  Keys are
// compared through the usual order-preserving map of float bits to unsigned
// integers, so the result is a permutation whatever the keys hold.  A plain
// rank count: count^2 comparisons, staged through LDS, is microseconds at the
// sizes a weight matrix fits in memory for.
__device__ __forceinline__ unsigned ordered_bits(float x)
{
    const unsigned b = __float_as_uint(x);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

constexpr int RANK_THREADS = 256, RANK_TILE = 2048;

// rank[i] += number of keys in [first, last) that sort before key i.  The y
// extent of the grid splits the comparisons into slices so that a few thousand
// keys still fill the device; rank[] starts at zero.  With GROUPED the order is
// by group first (group[i] in [0, 2^15)) and by key within a group.
template <bool GROUPED>
__global__ __launch_bounds__(RANK_THREADS) void rank_count_kernel(const float *__restrict__ key,
                                                                  const int32_t *__restrict__ group, int count,
                                                                  int slice, int32_t *__restrict__ rank)
{
    __shared__ __align__(16) unsigned tile[RANK_TILE];
    __shared__ __align__(16) int gtile[GROUPED ? RANK_TILE : 4];
    const int i = blockIdx.x * RANK_THREADS + threadIdx.x;
    const unsigned mine = i < count ? ordered_bits(key[i]) : 0u;
    const int gmine = (GROUPED && i < count) ? group[i] : 0;
    const int first = blockIdx.y * slice, last = min(count, first + slice);
    const int ties_upto = min(i, last);                 // equal keys count when they sit earlier; padding never does
    int before = 0;
    for (int base = first; base < last; base += RANK_TILE) {
        const int lim = min(RANK_TILE, last - base);
        __syncthreads();
        for (int t = threadIdx.x; t < RANK_TILE; t += RANK_THREADS) {
            tile[t] = t < lim ? ordered_bits(key[base + t]) : 0xffffffffu;      // padding sorts after everything
            if (GROUPED) gtile[t] = t < lim ? group[base + t] : 0x7fffffff;
        }
        __syncthreads();
        const int upto = (lim + 3) & ~3;
        for (int t = 0; t < upto; t += 4) {
            const uint4 v = *(const uint4 *)(tile + t);
            const int at = base + t;
            int c0 = (v.x < mine) + ((v.x == mine) & (at < ties_upto));
            int c1 = (v.y < mine) + ((v.y == mine) & (at + 1 < ties_upto));
            int c2 = (v.z < mine) + ((v.z == mine) & (at + 2 < ties_upto));
            int c3 = (v.w < mine) + ((v.w == mine) & (at + 3 < ties_upto));
            if (GROUPED) {
                const int4 g = *(const int4 *)(gtile + t);
                c0 = (g.x < gmine) + ((g.x == gmine) & c0);
                c1 = (g.y < gmine) + ((g.y == gmine) & c1);
                c2 = (g.z < gmine) + ((g.z == gmine) & c2);
                c3 = (g.w < gmine) + ((g.w == gmine) & c3);
            }
            before += c0 + c1 + c2 + c3;
        }
    }
    if (i < count && before) atomicAdd(&rank[i], before);
}

__global__ void order_from_rank_kernel(const int32_t *__restrict__ rank, int count, int32_t *__restrict__ order)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) order[rank[i]] = i;
}

// The staged matrix: rows and columns of the weight matrix in order of memory fraction.  Before
// the pair kernel runs it is filled, in whole lines, with MF_INFEASIBLE where the memory rule
// (paper: Section "Implementation", the memory quota; one float32 addition) says the pair cannot
// share and 0 elsewhere, so that what the kernel skips is already marked.
__global__ __launch_bounds__(256) void stage_marks_kernel(const float *__restrict__ mem_on_sorted,
                                                          const float *__restrict__ mem_off_sorted, int n, int m,
                                                          float mem_limit, int32_t *__restrict__ S, int64_t lds,
                                                          const int32_t *__restrict__ fit_len)
{
    const int i = blockIdx.x;
    const float mon = mem_on_sorted[i];
    int32_t *row = S + (size_t)i * lds;                    // lds is a multiple of four, S 16-byte aligned
    // the pairs before fit_len[i] can share and are all written by the scoring kernel: only the
    // rest of the line needs marks (from the group of four the boundary falls in)
    const int first = fit_len[i] & ~3;
    for (int j = first + (blockIdx.y * 256 + threadIdx.x) * 4; j < m; j += gridDim.y * 1024) {
        int32_t w[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = (j + e < m && mon + mem_off_sorted[j + e] > mem_limit) ? MF_INFEASIBLE : 0;
        *(int4 *)(row + j) = make_int4(w[0], w[1], w[2], w[3]);
    }
}

// *total += sum of len[0..count): how many pairs can share at all.
__global__ void sum_lengths_kernel(const int32_t *__restrict__ len, int count, unsigned long long *total)
{
    unsigned long long t = 0;
    for (int k = blockIdx.x * blockDim.x + threadIdx.x; k < count; k += gridDim.x * blockDim.x) t += (unsigned)len[k];
    for (int off = 32; off >= 1; off >>= 1) t += __shfl_xor(t, off);
    if ((threadIdx.x & 63) == 0 && t) atomicAdd(total, t);
}

__global__ void gather_by_order_kernel(const float *__restrict__ value, const int32_t *__restrict__ order, int count,
                                       float *__restrict__ out)
{
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k < count) out[k] = value[order[k]];
}

// In memory order the pairs that can share form, in every row, a prefix of the columns (and in
// every column a prefix of the rows): len[k] = how many entries of `other` (ascending) fit next
// to mine[k].  A binary search on the same float32 rule the marks were written with.
__global__ void fit_prefix_kernel(const float *__restrict__ mine, int count, const float *__restrict__ other,
                                  int other_count, float mem_limit, int32_t *__restrict__ len)
{
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= count) return;
    const float a = mine[k];
    int lo = 0, hi = other_count;                          // first position that does not fit
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (a + other[mid] > mem_limit) hi = mid; else lo = mid + 1;
    }
    len[k] = lo;
}

// The placement kernels see every weight once more: they note the largest on the way (the
// matching's first epsilon is set by it), at most one atomic per workgroup and only when it has
// news.  Every thread of the NT-thread workgroup calls this.
template <int NT>
__device__ inline void note_largest(int mx, int *largest)
{
    __shared__ int wave_largest[NT / 64];
    for (int off = 32; off >= 1; off >>= 1) mx = max(mx, __shfl_xor(mx, off));
    if ((threadIdx.x & 63) == 0) wave_largest[threadIdx.x >> 6] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int wv = 1; wv < NT / 64; ++wv) mx = max(mx, wave_largest[wv]);
        // the maximum only grows, so an outdated (smaller) cached value at worst costs a redundant atomic
        if (mx > *largest) atomicMax(largest, mx);
    }
}

// Puts the staged scores in place: W[i][j] = S[rank_on[i]][rank_off[j]].  General form: a row of
// S is read back in scattered 4-byte pieces, every piece of it by the same workgroup while it
// sits in the caches.
__global__ __launch_bounds__(256) void place_kernel(const int32_t *__restrict__ S, int64_t lds,
                                                    const int32_t *__restrict__ rank_on,
                                                    const int32_t *__restrict__ rank_off, int n, int m,
                                                    int32_t *__restrict__ W, int64_t ldw, int wide_stores,
                                                    int *largest)
{
    const int i = blockIdx.x;
    const int32_t *src = S + (size_t)rank_on[i] * lds;
    int32_t *row = W + (size_t)i * ldw;
    int mx = 0;                                             // "cannot share" is the smallest integer
    for (int j = (blockIdx.y * 256 + threadIdx.x) * 4; j < m; j += gridDim.y * 1024) {
        int32_t w[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) { w[e] = j + e < m ? src[rank_off[j + e]] : 0; mx = max(mx, w[e]); }
        if (wide_stores && j + 3 < m) {
            *(int4 *)(row + j) = make_int4(w[0], w[1], w[2], w[3]);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (j + e < m) row[j + e] = w[e];
        }
    }
    note_largest<256>(mx, largest);
}

// The same through LDS, for rows that fit there (measured faster than the kernel above): a
// workgroup per row loads the staged row in whole lines - only as far as its pairs can share,
// everything beyond is a mark anyway - picks each output's entry out of LDS, and stores the row
// in whole lines: no scattered access reaches the caches.
constexpr int PLACE_THREADS = 1024;
constexpr size_t PLACE_LDS_BYTES = 159 * 1024;            // of the 160 KB a gfx950 workgroup can have

__global__ __launch_bounds__(PLACE_THREADS) void place_lds_kernel(
    const int32_t *__restrict__ S, int64_t lds, const int32_t *__restrict__ rank_on,
    const int32_t *__restrict__ rank_off, const int32_t *__restrict__ fit_len, int n, int m,
    int32_t *__restrict__ W, int64_t ldw, int wide_stores, int *largest)
{
    extern __shared__ int32_t staged[];
    const int i = blockIdx.x, tid = threadIdx.x;
    const int from = rank_on[i];
    const int32_t *src = S + (size_t)from * lds;
    const int len = fit_len[from];                          // staged entries at or beyond it are marks
    int32_t *row = W + (size_t)i * ldw;
    int mx = 0;                                             // "cannot share" is the smallest integer
    for (int t = tid * 4; t < len; t += PLACE_THREADS * 4) {
        const int4 v = *(const int4 *)(src + t);            // the last group may reach into the marks
        *(int4 *)(staged + t) = v;
        mx = max(max(mx, max(v.x, v.y)), max(v.z, v.w));
    }
    note_largest<PLACE_THREADS>(mx, largest);               // passes a barrier: the staged row is complete
    for (int j = tid * 4; j < m; j += PLACE_THREADS * 4) {
        int32_t w[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int p = rank_off[min(j + e, m - 1)];
            w[e] = j + e < m ? (p < len ? staged[p] : MF_INFEASIBLE) : 0;
        }
        if (wide_stores && j + 3 < m) {
            *(int4 *)(row + j) = make_int4(w[0], w[1], w[2], w[3]);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (j + e < m) row[j + e] = w[e];
        }
    }
}

__global__ void clear_counter_kernel(unsigned long long *c) { *c = 0ull; }

__global__ void fill_flag_kernel(int *flag) { *flag = 0; }

__global__ void fill_value_kernel(int32_t *p, int count, int value)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = value;
}

__global__ void fill_zero_kernel(int32_t *p, int count)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = 0;
}

// Largest magnitudes of up to five arrays (blockIdx.y picks one), as bit patterns of non-negative
// floats, which order like unsigned integers: slots[y] = max |a_y[i]|.  The slots start at zero.
__global__ void range_clear_kernel(unsigned *slots)
{
    if (threadIdx.x < 8) slots[threadIdx.x] = 0u;
}

struct RangeArrays { const float *a[5]; long long count[5]; };

__global__ __launch_bounds__(256) void range_kernel(RangeArrays arrays, unsigned *slots)
{
    const float *a = arrays.a[blockIdx.y];
    if (!a) return;
    const long long count = arrays.count[blockIdx.y];
    float mx = 0.0f;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < count; i += (long long)gridDim.x * 256)
        mx = fmaxf(mx, fabsf(a[i]));
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    if ((threadIdx.x & 63) == 0 && mx > 0.0f) atomicMax(&slots[blockIdx.y], __float_as_uint(mx));
}

constexpr int PAIR_THREADS = 512;   // 8 wavefronts: two per SIMD share one LDS copy of W2
constexpr int PAIR_WAVES = PAIR_THREADS / 64;
constexpr int PAIR_COLS = PAIR_WAVES * 32;

template <int H, bool SPLIT> struct PairShape {
    static constexpr int ROWS = 64;                        // online rows per workgroup (128 with the fp16 pieces: measured slower)
    static constexpr int KS = H / 2;                       // k-steps of the 32x32x2 tile
    static constexpr int MB = H / 32;                      // 32-row blocks of the hidden layer
    static constexpr size_t LDS_BYTES = sizeof(float) * ((size_t)H * H + (size_t)ROWS * H + 4 * H + 2 * ROWS);
};

// One wavefront owns 32 offline columns (lane & 31) and walks down the online
// rows of the tile.  n and m count the rows and columns to score; with
// row_map / col_map (either may be null) entry t of the map names the online
// row / offline column that tile position t stands for, so a scattered subset
// of rows or columns can be re-scored in place.  v_mfma_f32_32x32x2_f32 computes D[32x32] += A[32x2] B[2x32]
// with lane l supplying A[l%32][l/32] and B[l/32][l%32]; we let the two k
// slots of step s be hidden features s and H/2 + s, so each half-wave streams
// a contiguous half of the projections.  Accumulator register r of lane l is
// D[8*(r/4) + 4*(l/32) + r%4][l%32].
// PAIR_SM: the predictor has a third input, the SM share of the pair
// min(1 - sm_on[i], sm_off[j]); its layer-1 weights w_sm[H] add w_sm[k] * share to hidden unit k.
// SLOWDOWN: a second output unit on the same hidden layers (weights w3_slow[H], b3_slow) predicts
// how much the online workload of the pair slows down; a pair above slow_limit is infeasible.
// SPLIT: the hidden layer's products are formed from half-precision pieces.  Every fp32 operand is
// x = hi + lo with hi = x rounded to fp16 and lo = the fp16 of the exact remainder (together 22
// significant bits; the hardware keeps fp16 subnormals), and w * h = w_hi h_hi + w_hi h_lo + w_lo h_hi
// up to 2^-22 relative, accumulated in fp32 by v_mfma_f32_32x32x16_f16: three matrix instructions
// of 16,384 multiply-adds in 8 passes each where fp32 operands need eight of 2,048 in 16 passes
// each.  Measured against the fp64 reference the scores are as close as those of the fp32 products
// (largest relative error 3-4e-7 on every benchmark configuration).  fp16 ends at 65,504 and
// thins out below 6e-5, so both operands are first scaled by powers of two (exact) that bring the
// largest weight, and the largest value a layer-1 unit can take, to about 2^13: `range` holds the
// largest magnitudes of the projections, of W2 and of the SM term, found by range_kernel; the
// accumulators then carry the product of the two scales, which b2 is given on the way in and W3
// takes out again.  The result therefore does not depend on the size of the numbers.
// For lane l, element t of its operand of k-block kb is hidden unit (l / 32) * H/2 + 8 kb + t, for
// A (rows of W2) and B (pairs) alike.
template <int H, bool PAIR_SM, bool SLOWDOWN, bool SPLIT>
__global__ __launch_bounds__(PAIR_THREADS) void pair_mlp_kernel(
    const float *__restrict__ P_on, const float *__restrict__ P_off,
    const float *__restrict__ W2, const float *__restrict__ b2, const float *__restrict__ W3,
    const float *__restrict__ b3, const float *__restrict__ mem_on,
    const float *__restrict__ mem_off, int n, int m, float scale, float mem_limit,
    int32_t *__restrict__ W, int64_t ldw, float *__restrict__ sigma,
    const int32_t *__restrict__ row_map, const int32_t *__restrict__ col_map, int by_memory,
    unsigned long long *__restrict__ evaluated, const int32_t *__restrict__ segment,
    const float *__restrict__ w_sm, const float *__restrict__ sm_on, const float *__restrict__ sm_off,
    const float *__restrict__ w3_slow, const float *__restrict__ b3_slow, float slow_limit,
    const unsigned *__restrict__ range)
{
    using S = PairShape<H, SPLIT>;
    constexpr int KS = S::KS, MB = S::MB, ROWS = S::ROWS, Q = KS / 4, KB = H / 16;
    extern __shared__ float4 lds4[];
    float4 *a_lds = lds4;                                  // [MB][Q][64] float4: MFMA A operand order
    uint4 *a16_lds = (uint4 *)lds4;                        // SPLIT: [2 pieces][MB][KB][64] eight fp16 each (the same bytes)
    float *pon_lds = (float *)(lds4) + H * H;              // [ROWS][H]
    float *b2_lds = pon_lds + ROWS * H;
    float *w3_lds = b2_lds + H;
    float *mon_lds = w3_lds + H;                           // [ROWS] memory fraction of the tile's rows
    float *wsm_lds = mon_lds + ROWS;                       // [H] layer-1 weights of the SM share
    float *son_lds = wsm_lds + H;                          // [ROWS] 1 - SM activity of the tile's rows
    float *w3s_lds = son_lds + ROWS;                       // [H] output weights of the slowdown unit

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int hh = lane >> 5, nn = lane & 31;
    int staged_row0 = 0;                    // where the row map's entry 0 sits in the staged matrix
    if (segment) {                          // only entries [segment[0], segment[1]) of the row map
        row_map += segment[0];
        staged_row0 = segment[0];
        n = segment[1] - segment[0];
    }
    // consecutive workgroups (which the hardware deals out to the eight XCDs in turn) share one
    // tile of offline columns and walk down the online rows, so that tile stays in every L2
    // and each XCD keeps re-reading the same eighth of the online projections
    // The row tile also shifts by one per column tile: in memory order the tiles with work
    // are the first so-many of each column tile, and without the shift the low XCDs would
    // collect the odd one out every time.
    const int row0 = (int)((blockIdx.x + blockIdx.y) % gridDim.x) * ROWS;
    if (row0 >= n) return;                  // the grid's x extent is padded to a multiple of eight
    const int nrows = min(ROWS, n - row0);
    const int j0 = (blockIdx.y * PAIR_WAVES + wave) * 32;
    // in memory order the tile's first row and first column are its smallest: if they do not
    // fit together, nothing in the tile does
    if (by_memory && mem_on[row_map[row0]] + mem_off[col_map[blockIdx.y * PAIR_COLS]] > mem_limit) return;

    // SPLIT: the powers of two that scale layer-1 values and W2 into fp16's comfortable range
    float scale_p = 1.0f, scale_w = 1.0f;
    if (SPLIT) {
        auto toward_8192 = [](float largest) {
            if (!(largest > 0.0f) || !(largest < 3.0e38f)) return 1.0f;
            return ldexpf(1.0f, max(-60, min(60, 13 - ilogbf(largest))));
        };
        const float sm_term = PAIR_SM ? __uint_as_float(range[3]) * fmaxf(1.0f, __uint_as_float(range[4])) : 0.0f;
        scale_p = toward_8192(__uint_as_float(range[0]) + __uint_as_float(range[1]) + sm_term);
        scale_w = toward_8192(__uint_as_float(range[2]));
    }
    const float scale_acc = scale_p * scale_w, unscale_acc = 1.0f / scale_acc;
    if (SPLIT) {
        for (int idx = tid; idx < MB * KB * 64; idx += PAIR_THREADS) {
            const int ln = idx & 63, kb = (idx >> 6) % KB, mb = idx / (64 * KB);
            const float *src = W2 + (size_t)(mb * 32 + (ln & 31)) * H + (ln >> 5) * KS + kb * 8;
            const float4 w0 = *(const float4 *)src, w1 = *(const float4 *)(src + 4);
            const float w[8] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w};
            Half8Words hi, lo;
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const float ws = w[t] * scale_w;
                const _Float16 h = (_Float16)ws;
                hi.v[t] = h;
                lo.v[t] = (_Float16)(ws - (float)h);
            }
            a16_lds[(mb * KB + kb) * 64 + ln] = hi.q;
            a16_lds[((MB + mb) * KB + kb) * 64 + ln] = lo.q;
        }
    } else {
        for (int idx = tid; idx < MB * Q * 64; idx += PAIR_THREADS) {
            int ln = idx & 63, s4 = (idx >> 6) % Q, mb = idx / (64 * Q);
            a_lds[idx] = *(const float4 *)(W2 + (size_t)(mb * 32 + (ln & 31)) * H + (ln >> 5) * KS + s4 * 4);
        }
    }
    for (int idx = tid; idx < nrows * (H / 4); idx += PAIR_THREADS) {
        const int r = idx / (H / 4), q = idx % (H / 4);
        const int gi = row_map ? row_map[row0 + r] : row0 + r;
        float4 v = ((const float4 *)(P_on + (size_t)gi * H))[q];
        if (SPLIT) { v.x *= scale_p; v.y *= scale_p; v.z *= scale_p; v.w *= scale_p; }
        ((float4 *)pon_lds)[idx] = v;
    }
    if (tid < H) { b2_lds[tid] = b2[tid] * scale_acc; w3_lds[tid] = W3[tid] * unscale_acc; }
    if (tid < nrows) mon_lds[tid] = mem_on[row_map ? row_map[row0 + tid] : row0 + tid];
    if (PAIR_SM) {
        if (tid < H) wsm_lds[tid] = w_sm[tid] * scale_p;
        if (tid < nrows) son_lds[tid] = 1.0f - sm_on[row_map ? row_map[row0 + tid] : row0 + tid];
    }
    if (SLOWDOWN && tid < H) w3s_lds[tid] = w3_slow[tid] * unscale_acc;
    __syncthreads();
    if (j0 >= m) return;

    const int j = j0 + nn;
    const int jc = col_map ? col_map[min(j, m - 1)] : min(j, m - 1);     // the column this lane scores
    float poff[KS];
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        float4 t = *(const float4 *)(P_off + (size_t)jc * H + hh * KS + q * 4);
        poff[4 * q] = t.x * scale_p; poff[4 * q + 1] = t.y * scale_p; poff[4 * q + 2] = t.z * scale_p; poff[4 * q + 3] = t.w * scale_p;
    }
    const float moff = mem_off[jc];
    const float soff = PAIR_SM ? sm_off[jc] : 0.0f;
    const float bias3 = b3[0];
    const float bias3_slow = SLOWDOWN ? b3_slow[0] : 0.0f;
    // by_memory: the maps list rows and columns by ascending memory fraction, so this
    // wavefront's first column has its smallest one, and once a row does not fit next to
    // that column (float addition is monotone) no later row of the tile fits any of its columns
    const float moff_least = by_memory ? __shfl(moff, 0) : 0.0f;

    // NR rows of the tile at once against this wavefront's 32 columns.  Two rows share every
    // W2 operand fetched from LDS and give the matrix pipe two independent accumulator sets.
    auto score_rows = [&](auto nr_tag, auto split_tag, const int r) {
        constexpr int NR = decltype(nr_tag)::value;
        constexpr bool SPLIT_HERE = decltype(split_tag)::value;
        floatx16 acc[NR][MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                float4 bv = *(const float4 *)(b2_lds + mb * 32 + 8 * g + 4 * hh);
#pragma unroll
                for (int x = 0; x < NR; ++x) {
                    acc[x][mb][4 * g] = bv.x; acc[x][mb][4 * g + 1] = bv.y;
                    acc[x][mb][4 * g + 2] = bv.z; acc[x][mb][4 * g + 3] = bv.w;
                }
            }
        float share[NR];
#pragma unroll
        for (int x = 0; x < NR; ++x) share[x] = PAIR_SM ? fminf(son_lds[r + x], soff) : 0.0f;
        if constexpr (SPLIT_HERE) {
            float minus_one = -1.0f;
            asm volatile("" : "+s"(minus_one));             // no instruction: only hides the constant from the optimiser
            // the two fp16 pieces of this lane's eight layer-1 values of k-block kb, for row r + x
            auto pieces = [&](const int kb, const int x, const float4 &p0, const float4 &p1, Half8Words &hi, Half8Words &lo) {
                const float pq[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
                float y[8];
                if (PAIR_SM) {
                    const float4 s0 = *(const float4 *)(wsm_lds + hh * KS + 8 * kb);
                    const float4 s1 = *(const float4 *)(wsm_lds + hh * KS + 8 * kb + 4);
                    const float ws[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
#pragma unroll
                    for (int t = 0; t < 8; ++t) y[t] = fmaxf(fmaf(ws[t], share[x], pq[t] + poff[8 * kb + t]), 0.0f);
                } else {
#pragma unroll
                    for (int t = 0; t < 8; ++t) y[t] = fmaxf(pq[t] + poff[8 * kb + t], 0.0f);
                }
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    // toward zero, so the remainder keeps the sign; it is exact in fp32
                    const auto h2 = __builtin_amdgcn_cvt_pkrtz(y[2 * t], y[2 * t + 1]);
                    hi.u[t] = __builtin_bit_cast(unsigned int, h2);
                    // y - hi written as a fused multiply-add by a -1 the optimiser cannot see: it is then
                    // selected as the mixed-precision instruction that reads the fp16 piece itself, one
                    // instruction per value instead of a conversion and a subtraction (same value: the
                    // remainder is exact either way)
                    const auto l2 = __builtin_amdgcn_cvt_pkrtz(__builtin_fmaf((float)h2[0], minus_one, y[2 * t]),
                                                               __builtin_fmaf((float)h2[1], minus_one, y[2 * t + 1]));
                    lo.u[t] = __builtin_bit_cast(unsigned int, l2);
                }
            };
            // W2's pieces for step (kb, mb) + 1 are requested from LDS before the matrix instructions of
            // step (kb, mb) are issued, so that their latency passes behind those instructions (the
            // scheduling fences keep the compiler from moving the requests back next to their use)
            Half8Words ahi[2], alo[2];
            ahi[0].q = a16_lds[lane];
            alo[0].q = a16_lds[(MB * KB) * 64 + lane];
            // ... and the rows' projections for k-block kb + 1 before the last step of k-block kb
            float4 pn[NR][2];
#pragma unroll
            for (int x = 0; x < NR; ++x) {
                pn[x][0] = *(const float4 *)(pon_lds + (r + x) * H + hh * KS);
                pn[x][1] = *(const float4 *)(pon_lds + (r + x) * H + hh * KS + 4);
            }
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
                Half8Words bhi[NR], blo[NR];
#pragma unroll
                for (int x = 0; x < NR; ++x) pieces(kb, x, pn[x][0], pn[x][1], bhi[x], blo[x]);
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    const int step = kb * MB + mb, cur = step & 1, nxt = cur ^ 1;
                    if (step + 1 < KB * MB) {
                        const int kb1 = (step + 1) / MB, mb1 = (step + 1) % MB;
                        ahi[nxt].q = a16_lds[(mb1 * KB + kb1) * 64 + lane];
                        alo[nxt].q = a16_lds[((MB + mb1) * KB + kb1) * 64 + lane];
                        if (mb == MB - 1) {
#pragma unroll
                            for (int x = 0; x < NR; ++x) {
                                pn[x][0] = *(const float4 *)(pon_lds + (r + x) * H + hh * KS + 8 * (kb + 1));
                                pn[x][1] = *(const float4 *)(pon_lds + (r + x) * H + hh * KS + 8 * (kb + 1) + 4);
                            }
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    // hi x hi, then the two cross terms; consecutive instructions alternate between the rows' accumulators
#pragma unroll
                    for (int x = 0; x < NR; ++x)
                        acc[x][mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ahi[cur].v, bhi[x].v, acc[x][mb], 0, 0, 0);
#pragma unroll
                    for (int x = 0; x < NR; ++x)
                        acc[x][mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ahi[cur].v, blo[x].v, acc[x][mb], 0, 0, 0);
#pragma unroll
                    for (int x = 0; x < NR; ++x)
                        acc[x][mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(alo[cur].v, bhi[x].v, acc[x][mb], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        } else {
        // operands of step q + 1 are fetched from LDS before the matrix instructions of step q are
        // issued, so that their latency hides behind those instead of in front of the next ones
        float4 av[2][MB], pv[2][NR];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) av[0][mb] = a_lds[(mb * Q) * 64 + lane];
#pragma unroll
        for (int x = 0; x < NR; ++x) pv[0][x] = *(const float4 *)(pon_lds + (r + x) * H + hh * KS);
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            const int cur = q & 1, nxt = cur ^ 1;
            if (q + 1 < Q) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) av[nxt][mb] = a_lds[(mb * Q + q + 1) * 64 + lane];
#pragma unroll
                for (int x = 0; x < NR; ++x)
                    pv[nxt][x] = *(const float4 *)(pon_lds + (r + x) * H + hh * KS + 4 * (q + 1));
            }
            float h1[NR][4];
#pragma unroll
            for (int x = 0; x < NR; ++x) {
                const float4 pq = pv[cur][x];
                if (PAIR_SM) {
                    const float4 ws = *(const float4 *)(wsm_lds + hh * KS + 4 * q);
                    h1[x][0] = fmaxf(fmaf(ws.x, share[x], pq.x + poff[4 * q]), 0.0f);
                    h1[x][1] = fmaxf(fmaf(ws.y, share[x], pq.y + poff[4 * q + 1]), 0.0f);
                    h1[x][2] = fmaxf(fmaf(ws.z, share[x], pq.z + poff[4 * q + 2]), 0.0f);
                    h1[x][3] = fmaxf(fmaf(ws.w, share[x], pq.w + poff[4 * q + 3]), 0.0f);
                } else {
                    h1[x][0] = fmaxf(pq.x + poff[4 * q], 0.0f);
                    h1[x][1] = fmaxf(pq.y + poff[4 * q + 1], 0.0f);
                    h1[x][2] = fmaxf(pq.z + poff[4 * q + 2], 0.0f);
                    h1[x][3] = fmaxf(pq.w + poff[4 * q + 3], 0.0f);
                }
            }
            // consecutive matrix instructions go to different accumulators: none waits for the one before
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int x = 0; x < NR; ++x)
                    acc[x][mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[cur][mb].x, h1[x][0], acc[x][mb], 0, 0, 0);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int x = 0; x < NR; ++x)
                    acc[x][mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[cur][mb].y, h1[x][1], acc[x][mb], 0, 0, 0);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int x = 0; x < NR; ++x)
                    acc[x][mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[cur][mb].z, h1[x][2], acc[x][mb], 0, 0, 0);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int x = 0; x < NR; ++x)
                    acc[x][mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[cur][mb].w, h1[x][3], acc[x][mb], 0, 0, 0);
        }
        }
        // max(v, 0) as the median of (v, 0, +inf): one instruction.  fmaxf costs two on values that
        // come out of the matrix pipe, because the compiler first has to make sure of a quiet NaN
        // (same result: the median of a NaN, 0 and +inf is 0 as well).
        // The +inf is hidden from the optimiser (an empty asm, no instruction), or it would turn the
        // median back into fmaxf.
        float plus_inf = __builtin_inff();
        asm volatile("" : "+s"(plus_inf));
        auto relu = [plus_inf](const float v) { return __builtin_amdgcn_fmed3f(v, 0.0f, plus_inf); };
#pragma unroll
        for (int x = 0; x < NR; ++x) {
            // output layer on this lane's 16*MB hidden units, then add the other half-wave's
            float zp = 0.0f;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    float4 wv = *(const float4 *)(w3_lds + mb * 32 + 8 * g + 4 * hh);
                    zp = fmaf(wv.x, relu(acc[x][mb][4 * g]), zp);
                    zp = fmaf(wv.y, relu(acc[x][mb][4 * g + 1]), zp);
                    zp = fmaf(wv.z, relu(acc[x][mb][4 * g + 2]), zp);
                    zp = fmaf(wv.w, relu(acc[x][mb][4 * g + 3]), zp);
                }
            const float z = zp + __shfl_xor(zp, 32) + bias3;
            const float sg = 1.0f / (1.0f + expf(-z));
            bool too_slow = false;
            if (SLOWDOWN) {                 // the same output layer once more with the other unit's weights
                float sp = 0.0f;
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        float4 wv = *(const float4 *)(w3s_lds + mb * 32 + 8 * g + 4 * hh);
                        sp = fmaf(wv.x, relu(acc[x][mb][4 * g]), sp);
                        sp = fmaf(wv.y, relu(acc[x][mb][4 * g + 1]), sp);
                        sp = fmaf(wv.z, relu(acc[x][mb][4 * g + 2]), sp);
                        sp = fmaf(wv.w, relu(acc[x][mb][4 * g + 3]), sp);
                    }
                const float zs = sp + __shfl_xor(sp, 32) + bias3_slow;
                too_slow = 1.0f / (1.0f + expf(-zs)) > slow_limit;
            }
            if (hh == 0 && j < m) {
                float qv = rintf(sg * scale);
                qv = fminf(fmaxf(qv, 0.0f), scale);
                int32_t w = (int32_t)qv;
                const float memsum = mon_lds[r + x] + moff;
                if (memsum > mem_limit || too_slow) w = MF_INFEASIBLE;
                if (by_memory) {
                    // the staged matrix: rows and columns both in memory order, one whole line per wave
                    W[(size_t)(staged_row0 + row0 + r + x) * ldw + j] = w;
                } else {
                    // (looked up here, not above: a load still in flight at the end of a row makes
                    // the next row wait for it and for every store issued after it)
                    const int i = row_map ? row_map[row0 + r + x] : row0 + r + x;
                    W[(size_t)i * ldw + jc] = w;
                    if (sigma) sigma[(size_t)i * m + jc] = sg;
                }
            }
        }
    };

    int r = 0;
    while (r < nrows) {
        // W2 does not fit in registers next to the accumulators: keep its loads inside the row loop
        asm volatile("" ::: "memory");
        if (by_memory && mon_lds[r] + moff_least > mem_limit) break;
        const bool pair_of_rows = r + 1 < nrows && !(by_memory && mon_lds[r + 1] + moff_least > mem_limit);
        if (pair_of_rows) { score_rows(std::integral_constant<int, 2>{}, std::integral_constant<bool, SPLIT>{}, r); r += 2; }
        else { score_rows(std::integral_constant<int, 1>{}, std::integral_constant<bool, SPLIT>{}, r); r += 1; }
    }
    // rows the loop left early keep the "cannot fit" marks the staged matrix was filled with
    if (evaluated && lane == 0 && r > 0) atomicAdd(evaluated, (unsigned long long)r * (unsigned)min(32, m - j0));
}

template <int H, bool PAIR_SM, bool SLOWDOWN, bool SPLIT>
int launch_pair_variant(mf_ctx *ctx, const mf_predictor *p, int n, int m, int32_t *d_W, int64_t ldw,
                        float *d_sigma, const int32_t *row_map, const int32_t *col_map, bool by_memory,
                        const int32_t *segment, int grid_rows)
{
    using S = PairShape<H, SPLIT>;
    // (the attribute belongs to the device, so what has been set is remembered per context)
    const unsigned flag = 1u << (5 + (H == 128 ? 8 : 0) + (PAIR_SM ? 4 : 0) + (SLOWDOWN ? 2 : 0) + (SPLIT ? 1 : 0));
    if (!(ctx->kernels_configured & flag)) {
        MF_HIP(hipFuncSetAttribute((const void *)pair_mlp_kernel<H, PAIR_SM, SLOWDOWN, SPLIT>,
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)S::LDS_BYTES));
        ctx->kernels_configured |= flag;
    }
    // x covers the rows this launch scores (a segment of the row map, or all n), padded to a
    // multiple of 8: every XCD then meets the same row tiles for each column tile
    dim3 grid((((grid_rows + S::ROWS - 1) / S::ROWS) + 7) & ~7, (m + PAIR_COLS - 1) / PAIR_COLS);
    hipLaunchKernelGGL((pair_mlp_kernel<H, PAIR_SM, SLOWDOWN, SPLIT>), grid, dim3(PAIR_THREADS), S::LDS_BYTES, ctx->stream,
                       ctx->proj_on, ctx->proj_off, p->d_W2, p->d_b2, p->d_W3, p->d_b3,
                       ctx->mem_on, ctx->mem_off, n, m, p->scale, p->mem_limit, d_W, ldw, d_sigma, row_map, col_map,
                       by_memory ? 1 : 0, ctx->pairs_evaluated, segment, p->d_W1sm, ctx->sm_on, ctx->sm_off,
                       p->d_W3_slow, p->d_b3_slow, p->slow_limit, SPLIT ? ctx->score_range : nullptr);
    MF_HIP(hipGetLastError());
    return MF_OK;
}

template <int H>
int launch_pair(mf_ctx *ctx, const mf_predictor *p, int n, int m, int32_t *d_W, int64_t ldw,
                float *d_sigma, const int32_t *row_map, const int32_t *col_map, bool by_memory,
                const int32_t *segment = nullptr, int segment_rows = -1)
{
    const int grid_rows = segment_rows >= 0 ? segment_rows : n;
    const int which = (p->d_W1sm ? 4 : 0) + (p->d_W3_slow ? 2 : 0) + (ctx->score_split ? 1 : 0);
#define MF_PAIR_CASE(SM, SLOW, SPL) \
    return launch_pair_variant<H, SM, SLOW, SPL>(ctx, p, n, m, d_W, ldw, d_sigma, row_map, col_map, by_memory, segment, grid_rows)
    switch (which) {
    case 0: MF_PAIR_CASE(false, false, false);
    case 1: MF_PAIR_CASE(false, false, true);
    case 2: MF_PAIR_CASE(false, true, false);
    case 3: MF_PAIR_CASE(false, true, true);
    case 4: MF_PAIR_CASE(true, false, false);
    case 5: MF_PAIR_CASE(true, false, true);
    case 6: MF_PAIR_CASE(true, true, false);
    default: MF_PAIR_CASE(true, true, true);
    }
#undef MF_PAIR_CASE
}

// What the fp16 pieces of the scorer's hidden layer are scaled by depends on the largest
// projections and weights: found here, after the projections, before the pair kernel.
void launch_score_range(mf_ctx *ctx, const mf_predictor *p, int n, int m)
{
    if (!ctx->score_split) return;
    RangeArrays arrays{};
    arrays.a[0] = ctx->proj_on;  arrays.count[0] = (long long)n * p->H;
    arrays.a[1] = ctx->proj_off; arrays.count[1] = (long long)m * p->H;
    arrays.a[2] = p->d_W2;       arrays.count[2] = (long long)p->H * p->H;
    arrays.a[3] = p->d_W1sm;     arrays.count[3] = p->H;
    arrays.a[4] = p->d_W1sm ? ctx->sm_off : nullptr; arrays.count[4] = m;
    hipLaunchKernelGGL(range_clear_kernel, dim3(1), dim3(64), 0, ctx->stream, ctx->score_range);
    hipLaunchKernelGGL(range_kernel, dim3(64, 5), dim3(256), 0, ctx->stream, arrays, ctx->score_range);
}

// order[k] = the workload with the k-th smallest (group, key); rank[i] = its position k
void order_by_memory(mf_ctx *ctx, const float *key, const int32_t *group, int count, int32_t *order,
                     int32_t *rank)
{
    const int blocks = (count + RANK_THREADS - 1) / RANK_THREADS;
    int split = 2048 / blocks;
    split = split < 1 ? 1 : (split > 64 ? 64 : split);
    const int slice = ((count + split - 1) / split + 3) & ~3;
    const dim3 grid(blocks, (count + slice - 1) / slice);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(RANK_THREADS), 0, ctx->stream, rank, count);
    if (group)
        hipLaunchKernelGGL(rank_count_kernel<true>, grid, dim3(RANK_THREADS), 0, ctx->stream, key, group, count,
                           slice, rank);
    else
        hipLaunchKernelGGL(rank_count_kernel<false>, grid, dim3(RANK_THREADS), 0, ctx->stream, key, group, count,
                           slice, rank);
    hipLaunchKernelGGL(order_from_rank_kernel, dim3(blocks), dim3(RANK_THREADS), 0, ctx->stream, rank,
                       count, order);
}

__global__ void gather_feature_kernel(const float *__restrict__ X, int rows, int F, int feature,
                                      float *__restrict__ out)
{
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r < rows) out[r] = X[(size_t)r * F + feature];
}

// segment[t] = number of workloads whose type is below t (t = 0..n_types); *bad is raised for
// a type outside [0, n_types).  One workgroup: the type counts are a few dozen integers.
__global__ __launch_bounds__(1024) void type_segments_kernel(const int32_t *__restrict__ type, int count,
                                                             int n_types, int32_t *__restrict__ segment, int *bad)
{
    __shared__ int hist[MF_MAX_TYPES];
    for (int t = threadIdx.x; t < MF_MAX_TYPES; t += blockDim.x) hist[t] = 0;
    __syncthreads();
    for (int i = threadIdx.x; i < count; i += blockDim.x) {
        const int t = type[i];
        if (t < 0 || t >= n_types) atomicExch(bad, 1);
        else atomicAdd(&hist[t], 1);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int run = 0;
        for (int t = 0; t <= n_types; ++t) { segment[t] = run; if (t < n_types) run += hist[t]; }
    }
}

}  // namespace

// preds[0..n_types): with d_type == nullptr there is one predictor for everybody; otherwise
// online workload i is scored by preds[d_type[i]] (all of them agree on F, the memory feature,
// the memory limit and the scale; the hidden width may differ).  Per type: project everybody
// with that type's first layer, then run the pair kernel on that type's rows - a contiguous
// segment of the row map, which lists the online workloads by (type, memory fraction).
int mf_launch_score(mf_ctx *ctx, const mf_predictor *preds, int n_types, const int32_t *d_type,
                    const float *d_on, int n, const float *d_off, int m, int32_t *d_W, int64_t ldw,
                    float *d_sigma)
{
    const mf_predictor *p0 = &preds[0];
    const int F = p0->F;
    const bool typed = d_type != nullptr;
    int32_t type_first[MF_MAX_TYPES + 1] = {0};
    if (typed) {
        hipLaunchKernelGGL(fill_flag_kernel, dim3(1), dim3(1), 0, ctx->stream, ctx->colmark);
        hipLaunchKernelGGL(type_segments_kernel, dim3(1), dim3(1024), 0, ctx->stream, d_type, n, n_types,
                           ctx->type_segment, ctx->colmark);
        MF_HIP(hipGetLastError());
        int bad = 0;
        MF_HIP(hipMemcpyAsync(&bad, ctx->colmark, sizeof(int), hipMemcpyDeviceToHost, ctx->stream));
        // the host sizes each type's launch by its number of rows
        MF_HIP(hipMemcpyAsync(type_first, ctx->type_segment, sizeof(int32_t) * (size_t)(n_types + 1),
                              hipMemcpyDeviceToHost, ctx->stream));
        MF_HIP(hipStreamSynchronize(ctx->stream));
        if (bad) return MF_ERR_ARG;
    }
    MF_HIP(hipEventRecord(ctx->ev[0], ctx->stream));
    hipLaunchKernelGGL(gather_feature_kernel, dim3((n + 255) / 256), dim3(256), 0, ctx->stream, d_on, n, F,
                       p0->mem_feature, ctx->mem_on);
    hipLaunchKernelGGL(gather_feature_kernel, dim3((m + 255) / 256), dim3(256), 0, ctx->stream, d_off, m, F,
                       p0->mem_feature, ctx->mem_off);
    if (p0->d_W1sm) {
        hipLaunchKernelGGL(gather_feature_kernel, dim3((n + 255) / 256), dim3(256), 0, ctx->stream, d_on, n, F,
                           p0->sm_on_feature, ctx->sm_on);
        hipLaunchKernelGGL(gather_feature_kernel, dim3((m + 255) / 256), dim3(256), 0, ctx->stream, d_off, m, F,
                           p0->sm_off_feature, ctx->sm_off);
    }
    // Pairs whose memory fractions do not fit get no score, so unless the caller wants every
    // score, walk rows and columns in memory order: the pairs that cannot fit then form one
    // corner of the tile grid and the kernel leaves them out.  Results land at the same places.
    const bool by_memory = ctx->fit_order && !d_sigma;
    hipLaunchKernelGGL(clear_counter_kernel, dim3(1), dim3(1), 0, ctx->stream, ctx->pairs_evaluated);
    hipLaunchKernelGGL(fill_flag_kernel, dim3(1), dim3(1), 0, ctx->stream, ctx->largest_weight);
    ctx->largest_weight_known = false;
    if (by_memory || typed) order_by_memory(ctx, ctx->mem_on, d_type, n, ctx->order_on, ctx->rank_on);
    const int64_t lds = ((int64_t)m + 3) & ~3ll;
    ctx->staged_n = ctx->staged_m = 0;
    if (by_memory) {
        order_by_memory(ctx, ctx->mem_off, nullptr, m, ctx->order_off, ctx->rank_off);
        hipLaunchKernelGGL(gather_by_order_kernel, dim3((n + 255) / 256), dim3(256), 0, ctx->stream, ctx->mem_on,
                           ctx->order_on, n, ctx->mem_on_sorted);
        hipLaunchKernelGGL(gather_by_order_kernel, dim3((m + 255) / 256), dim3(256), 0, ctx->stream, ctx->mem_off,
                           ctx->order_off, m, ctx->mem_off_sorted);
        const int chunks = (m + 4095) / 4096 < 16 ? (m + 4095) / 4096 : 16;
        // feasibility is a prefix of every staged row (columns are in memory order) and, when the
        // rows are in memory order too - one predictor - of every staged column; with several
        // predictors the rows are ordered by type first and columns are read whole
        hipLaunchKernelGGL(fit_prefix_kernel, dim3((n + 255) / 256), dim3(256), 0, ctx->stream, ctx->mem_on_sorted,
                           n, ctx->mem_off_sorted, m, p0->mem_limit, ctx->fit_len_on);
        hipLaunchKernelGGL(stage_marks_kernel, dim3(n, chunks), dim3(256), 0, ctx->stream, ctx->mem_on_sorted,
                           ctx->mem_off_sorted, n, m, p0->mem_limit, ctx->staged, lds, ctx->fit_len_on);
        if (!typed)
            hipLaunchKernelGGL(fit_prefix_kernel, dim3((m + 255) / 256), dim3(256), 0, ctx->stream, ctx->mem_off_sorted,
                               m, ctx->mem_on_sorted, n, p0->mem_limit, ctx->fit_len_off);
        else
            hipLaunchKernelGGL(fill_value_kernel, dim3((m + 255) / 256), dim3(256), 0, ctx->stream, ctx->fit_len_off, m, n);
        hipLaunchKernelGGL(clear_counter_kernel, dim3(1), dim3(1), 0, ctx->stream, ctx->feasible_pairs);
        hipLaunchKernelGGL(sum_lengths_kernel, dim3(64), dim3(256), 0, ctx->stream, ctx->fit_len_on, n,
                           ctx->feasible_pairs);
        ctx->staged_n = n;
        ctx->staged_m = m;
    }
    MF_HIP(hipGetLastError());
    ctx->pairs_total = (double)n * (double)m;
    const int32_t *rmap = (by_memory || typed) ? ctx->order_on : nullptr, *cmap = by_memory ? ctx->order_off : nullptr;
    // in memory order the scores go to the staged matrix
    int32_t *out = by_memory ? ctx->staged : d_W;
    const int64_t ldo = by_memory ? lds : ldw;
    for (int t = 0; t < n_types; ++t) {
        const mf_predictor *p = &preds[t];
        const int H = p->H;
        long tot = (long)n * H;
        hipLaunchKernelGGL(project_kernel, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, ctx->stream,
                           d_on, n, F, p->d_W1, 0, p->d_b1, H, ctx->proj_on);
        tot = (long)m * H;
        hipLaunchKernelGGL(project_kernel, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, ctx->stream,
                           d_off, m, F, p->d_W1, F, (const float *)nullptr, H, ctx->proj_off);
        launch_score_range(ctx, p, n, m);
        MF_HIP(hipGetLastError());
        if (t == 0) MF_HIP(hipEventRecord(ctx->ev[1], ctx->stream));      // later types' projections count as scoring
        const int32_t *segment = typed ? ctx->type_segment + t : nullptr;
        const int segment_rows = typed ? type_first[t + 1] - type_first[t] : -1;
        if (segment_rows == 0) continue;                                   // no workload of this type
        int rc = (H == 64) ? launch_pair<64>(ctx, p, n, m, out, ldo, d_sigma, rmap, cmap, by_memory, segment, segment_rows)
                           : launch_pair<128>(ctx, p, n, m, out, ldo, d_sigma, rmap, cmap, by_memory, segment, segment_rows);
        if (rc != MF_OK) return rc;
    }
    MF_HIP(hipEventRecord(ctx->ev[2], ctx->stream));
    if (by_memory) {
        const int chunks = (m + 4095) / 4096 < 16 ? (m + 4095) / 4096 : 16;
        const int wide = ((uintptr_t)d_W & 15u) == 0 && (ldw & 3) == 0;
        if ((size_t)lds * sizeof(int32_t) <= PLACE_LDS_BYTES) {
            if (!(ctx->kernels_configured & 16u)) {
                MF_HIP(hipFuncSetAttribute((const void *)place_lds_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)PLACE_LDS_BYTES));
                ctx->kernels_configured |= 16u;
            }
            hipLaunchKernelGGL(place_lds_kernel, dim3(n), dim3(PLACE_THREADS), sizeof(int32_t) * (size_t)lds, ctx->stream,
                               ctx->staged, lds, ctx->rank_on, ctx->rank_off, ctx->fit_len_on, n, m, d_W, ldw, wide,
                               ctx->largest_weight);
        } else {
            hipLaunchKernelGGL(place_kernel, dim3(n, chunks), dim3(256), 0, ctx->stream, ctx->staged, lds,
                               ctx->rank_on, ctx->rank_off, n, m, d_W, ldw, wide, ctx->largest_weight);
        }
        MF_HIP(hipGetLastError());
        ctx->largest_weight_known = true;
    }
    MF_HIP(hipEventRecord(ctx->ev[8], ctx->stream));
    ctx->score_pending = true;
    return MF_OK;
}

namespace {

__global__ void check_indices_kernel(const int32_t *__restrict__ list, int count, int limit, int *bad)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count && (list[i] < 0 || list[i] >= limit)) atomicExch(bad, 1);
}

}  // namespace

// Re-scores, in place, the rows of the listed online workloads and the columns
// of the listed offline workloads (device index lists).  Projections are
// recomputed for everybody (they cost 2(n+m)FH flop); the pair kernel then runs
// on `n_rows x m` and `n x n_cols` through its index maps.
int mf_launch_rescore(mf_ctx *ctx, const mf_predictor *p, const float *d_on, int n, const float *d_off,
                      int m, int32_t *d_W, int64_t ldw, const int32_t *d_rows, int n_rows,
                      const int32_t *d_cols, int n_cols)
{
    const int H = p->H, F = p->F;
    ctx->staged_n = ctx->staged_m = 0;       // the staged copy no longer matches the matrix
    ctx->largest_weight_known = false;
    // the lists index device arrays: refuse anything out of range before a kernel trusts it
    hipLaunchKernelGGL(fill_flag_kernel, dim3(1), dim3(1), 0, ctx->stream, ctx->colmark);
    if (n_rows > 0)
        hipLaunchKernelGGL(check_indices_kernel, dim3((n_rows + 255) / 256), dim3(256), 0, ctx->stream, d_rows,
                           n_rows, n, ctx->colmark);
    if (n_cols > 0)
        hipLaunchKernelGGL(check_indices_kernel, dim3((n_cols + 255) / 256), dim3(256), 0, ctx->stream, d_cols,
                           n_cols, m, ctx->colmark);
    MF_HIP(hipGetLastError());
    int bad = 0;
    MF_HIP(hipMemcpyAsync(&bad, ctx->colmark, sizeof(int), hipMemcpyDeviceToHost, ctx->stream));
    MF_HIP(hipStreamSynchronize(ctx->stream));
    if (bad) return MF_ERR_ARG;
    MF_HIP(hipEventRecord(ctx->ev[0], ctx->stream));
    long tot = (long)n * H;
    hipLaunchKernelGGL(project_kernel, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, ctx->stream,
                       d_on, n, F, p->d_W1, 0, p->d_b1, H, ctx->proj_on);
    tot = (long)m * H;
    hipLaunchKernelGGL(project_kernel, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, ctx->stream,
                       d_off, m, F, p->d_W1, F, (const float *)nullptr, H, ctx->proj_off);
    hipLaunchKernelGGL(gather_feature_kernel, dim3((n + 255) / 256), dim3(256), 0, ctx->stream, d_on, n, F,
                       p->mem_feature, ctx->mem_on);
    hipLaunchKernelGGL(gather_feature_kernel, dim3((m + 255) / 256), dim3(256), 0, ctx->stream, d_off, m, F,
                       p->mem_feature, ctx->mem_off);
    if (p->d_W1sm) {
        hipLaunchKernelGGL(gather_feature_kernel, dim3((n + 255) / 256), dim3(256), 0, ctx->stream, d_on, n, F,
                           p->sm_on_feature, ctx->sm_on);
        hipLaunchKernelGGL(gather_feature_kernel, dim3((m + 255) / 256), dim3(256), 0, ctx->stream, d_off, m, F,
                           p->sm_off_feature, ctx->sm_off);
    }
    launch_score_range(ctx, p, n, m);       // over everybody, as a full scoring pass would find it
    MF_HIP(hipGetLastError());
    hipLaunchKernelGGL(clear_counter_kernel, dim3(1), dim3(1), 0, ctx->stream, ctx->pairs_evaluated);
    ctx->pairs_total = (double)n_rows * (double)m + (double)n * (double)n_cols;
    MF_HIP(hipEventRecord(ctx->ev[1], ctx->stream));
    int rc = MF_OK;
    if (n_rows > 0)
        rc = (H == 64) ? launch_pair<64>(ctx, p, n_rows, m, d_W, ldw, nullptr, d_rows, nullptr, false)
                       : launch_pair<128>(ctx, p, n_rows, m, d_W, ldw, nullptr, d_rows, nullptr, false);
    if (rc == MF_OK && n_cols > 0)
        rc = (H == 64) ? launch_pair<64>(ctx, p, n, n_cols, d_W, ldw, nullptr, nullptr, d_cols, false)
                       : launch_pair<128>(ctx, p, n, n_cols, d_W, ldw, nullptr, nullptr, d_cols, false);
    if (rc != MF_OK) return rc;
    MF_HIP(hipEventRecord(ctx->ev[2], ctx->stream));
    MF_HIP(hipEventRecord(ctx->ev[8], ctx->stream));
    ctx->score_pending = true;
    return MF_OK;
}
