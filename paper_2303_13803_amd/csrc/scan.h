// Building blocks shared by the kernels of the assignment solver: the packed (dual, holder)
// word, loads and stores that must be seen across workgroups, wavefront reductions, the
// line scans (best and second-best value of K*w - dual) and the bid itself.
// Everything here is device code with internal linkage; each translation unit gets its own copy.
#pragma once
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
// LOOK_FIRST: read the word before bidding and do without the atomic when the bid has lost
// already.  For rounds in which thousands bid at once, many of them for the same few entries; a
// bidder following a chain on its own would only wait one more memory round trip per step.
template <bool LOOK_FIRST = false>
__device__ inline int decide_and_bid(const SideArgs &s, int b, const Top2 &t)
{
    if (t.b1 <= s.eps) {
        if (s.rested) atomicAdd(s.rested, 1);
        return -1;
    }
    const double keep = fmax(t.b2 - s.eps, 0.0);
    const double offer = s.Kd * (double)t.w - keep;
    const unsigned long long mine = pack_word(offer, b + 1);
    unsigned long long *dual_bits = (unsigned long long *)&s.other_dual[t.idx];
    unsigned long long old = LOOK_FIRST ? load_fresh_u64(&s.otherword[t.idx]) : 0ull;
    if (old < mine) old = atomicMax(&s.otherword[t.idx], mine);
    if (old < mine) {
        atomicMax(dual_bits, (unsigned long long)__double_as_longlong(offer));
        return word_id(old);
    }
    // Outbid: whoever holds the word now has written, or is about to write, at least its dual to
    // the copy the scans read; make sure of it, but without an atomic when it is there already -
    // hundreds of bidders may lose on the same popular entry in one round, and every atomic on a
    // line that all scans are reading holds those reads up.
    const unsigned long long least = (unsigned long long)__double_as_longlong(word_dual(old));
    if (load_fresh_u64(dual_bits) < least) atomicMax(dual_bits, least);
    return b;
}

}  // namespace
