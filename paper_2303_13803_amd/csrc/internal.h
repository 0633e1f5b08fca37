// Internal declarations shared by the library's translation units (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "muxmatch.h"

#define MF_HIP(call)                                                            \
    do {                                                                        \
        hipError_t e_ = (call);                                                 \
        if (e_ != hipSuccess) {                                                 \
            ctx->hip_error = e_;                                                \
            return MF_ERR_HIP;                                                  \
        }                                                                       \
    } while (0)

// A dual value and the index of the workload holding the other end share one
// 64-bit word so that a single atomicMax both raises the dual and records
// who raised it: word = dual << MF_ID_BITS | (id + 1), id + 1 == 0 meaning "nobody".
#define MF_ID_BITS 20
#define MF_ID_MASK ((1ull << MF_ID_BITS) - 1ull)
#define MF_MAX_DIM ((1 << MF_ID_BITS) - 2)
#define MF_MAX_DUAL (1ll << 43)
#define MF_MAX_TYPES 64

enum { T_PROJ = 0, T_PAIR, T_BID_BULK, T_BID_BULK_LAUNCHES, T_TRANSPOSE, T_DUALS, T_CERT, T_SOLVE,
       T_BID_BULK_BYTES, T_PAIR_EVALUATED, T_COUNT = 16 };

struct mf_device_stats {            // lives in device memory, cleared per solve
    unsigned long long rounds;      // bidding rounds
    unsigned long long bids;        // bids evaluated (one line scan each)
    unsigned long long bytes;       // weight bytes those scans read
    unsigned long long chain_bids;  // bids evaluated by chain kernels
    unsigned long long chain_depth; // sum over chain kernels of the most bids any one workgroup evaluated
    unsigned long long chain_retries; // chain bids that lost and were redone with uncached dual reads
    unsigned long long team_bids;   // chain bids evaluated by several workgroups together
    unsigned long long path_steps;  // super-steps of the shortest-path searches
    unsigned long long path_scans;  // line scans those searches made
    unsigned long long launch_max;  // scratch: that maximum for the chain kernel in flight
    int max_weight;
    int cnt[4];                     // ring of bidder-list lengths: round r reads cnt[r & 3]
    int head;                       // next unclaimed entry of the list a chain kernel works through
    int active;                     // workgroups of the running chain kernel still following a chain
    int team_abort;                 // a bounded wait between cooperating workgroups ran out (1: chain teams, 2: path search)
    int rested;                     // bidders of the side on which rows bid that gave up with best value <= eps, this solve
    // weight bytes the rounds with many bidders read: every workgroup of such a round adds to it as
    // it leaves, so it sits on a cache line of its own, away from the list counters above
    alignas(128) unsigned long long round_bytes;
};

struct mf_cert_out {                // lives in device memory, cleared per check
    long long primal;
    long long dual;
    long long min_rc;
    int matched;
    int flags;                      // bit0 bad index/duplicate, bit1 infeasible pair, bit2 negative dual
};

struct mf_ctx {
    int device;
    hipStream_t stream;
    int max_n, max_m;
    hipError_t hip_error;
    unsigned kernels_configured;    // kernels whose dynamic shared memory limit has been raised on this device (bits)
    // scoring scratch
    float *proj_on, *proj_off;      // [max_n][H], [max_m][H]
    float *mem_on, *mem_off;        // [max_n], [max_m]
    float *sm_on, *sm_off;          // SM activity / SM demand features (pair-dependent SM input)
    int32_t *order_on, *order_off;  // workloads by ascending memory fraction (online: by type first)
    int32_t *rank_on, *rank_off;    // position of each workload in its order
    float *mem_on_sorted, *mem_off_sorted;
    int32_t *staged;                // [max_n][pad4(max_m)] the last scored matrix with rows and columns in memory order
    int32_t *fit_len_on, *fit_len_off;   // per staged row / column: how many entries from the start can share
    unsigned long long *feasible_pairs, *h_feasible_pairs;    // how many pairs of the staged matrix can share (device, pinned)
    int fit_prefix_below;           // percent of pairs that can share below which the solve uses the staged matrix
    int *edge_count;                // [max(max_n, max_m)] feasible pairs per row of a matrix the caller brought, padded to 4
    long long *edge_start;          // [max(max_n, max_m) + 1] where each row's list starts
    int edge_lists_from;            // rows from which such a matrix is turned into lists when few pairs are feasible (0: never)
    int staged_n, staged_m;         // shape of the staged matrix the solver may use (0: none)
    int *largest_weight;            // largest weight of the matrix just scored (device), noted while it was put in place
    bool largest_weight_known;      // ... and whether it is that of the matrix the staged copy belongs to
    int32_t *type_segment;          // [MF_MAX_TYPES + 1] first position of each type in order_on
    unsigned long long *pairs_evaluated, *h_pairs_evaluated;   // pairs the last scoring pass ran the MLP on (device, pinned)
    double pairs_total;             // ... out of this many
    bool fit_prefix;                // solve on the staged matrix, reading only the prefixes that can share
    bool fit_order;                 // score in memory order and skip pairs that cannot fit
    // solver scratch
    int32_t *wt;                    // transposed weights [max_m][ldt]
    double *price, *profit;         // [max_m+4], [max_n+4]: exact integers held in doubles
    unsigned long long *colword, *roword;
    int *row2col, *col2row;
    int warm_n, warm_m;             // shape of the solve whose prices the context still holds (0: none)
    bool warm_reset_cols;           // start replaced columns at price 0 instead of their predecessor's price
    int64_t warm_eps_units;         // first epsilon of a warm-started solve, in weight units
    int phase_stop;                 // unplaced bidders at or below which a phase that only prepares prices ends
    int phase_growth;               // ... times this for every phase further from the ones that run to the end
    int phase_growth_rest;               // bidders that may have given up before coarse phases stop leaving more
    int phase_keep;                 // the last so many phases always run to the end
    long long phase_tail_steps;     // dependent chain steps after which a side that only prepares prices ends (0: no limit)
    int phase_tail_from;            // ... for problems with at least this many bidding lines
    int phase_tail_sides;           // ... on which sides: bit 0 the first (rows bid), bit 1 the second
    long long final_jump;           // epsilon (weight units) at or below which the next phase is the last (0: never)
    int tail_max;                   // bidder count at or below which chains are followed in one kernel
    int bulk_grid;                  // most workgroups of such a round (0: one per group of lines, up to 8192)
    int bulk_shape;                 // workgroup shape of rounds with many bidders (see launch_round)
    int bulk_share;                 // ... "many": at least 2048 and this share (percent) of the side's lines
    int team_max;                   // chains at or below which several workgroups share each chain (0: never)
    int team_size, team_threads;    // most workgroups per chain, threads per such workgroup
    int team_wide;                  // chains at or below which smaller teams already take over from chain_kernel
    long long team_regroup;         // steps after which such teams stop so that the chains left can be regrouped
    bool team_off;                  // set after a team wait ran out, for the rest of the solve
    int fallbacks;                  // MF_FALLBACK_* bits of the running solve
    void *team_ctl;                 // control blocks of the cooperating workgroups
    void *path_ctl;                 // control block of the shortest-path search
    unsigned long long *path_label, *path_expanded;   // [max(max_n, max_m)] each
    unsigned int *path_stamp;
    unsigned long long *path_frontier[2];   // 16 segments of max(max_n, max_m) entries (column, holder) each
    int *path_held;
    double *path_base;              // per bidding line: length of the shortest path to it plus what it would pay, or +inf
    int *path_tree;                 // columns of the tree being served
    int *path_parent, *path_jump;   // [max(max_n, max_m)] each: predecessor columns while a tree is served
    int path_max;                   // bidders at or below which shortest-path searches place them (0: never)
    long long path_after;           // chain steps per run after which the searches take over
    int path_grid;                  // workgroups of a search (0: one per compute unit)
    int path_width;                 // label window of one super-step, in epsilons
    bool path_pull;                 // re-label a served tree's columns from the other copy of the matrix
    int path_frontier_rows;         // frontier above which the window is halved (doubled below an eighth of it)
    unsigned path_spin_limit;       // polls a workgroup waits at a barrier of the search before it gives up
    bool path_off;                  // set after a wait of the search ran out, for the rest of the solve
    int n_cus;                      // compute units of the device
    int chain_grid;                 // workgroups of that kernel
    int *list[2];
    int *colmark;                   // [max_m]
    mf_device_stats *stats;
    mf_cert_out *cert;
    // pinned host mirrors
    mf_device_stats *h_stats;
    mf_device_stats *h_stats_slot[2];   // pinned: where the counts of bulk rounds land while the next round runs
    hipEvent_t ev_stats[2];
    unsigned *score_range;              // device: largest magnitudes the scorer's fp16 pieces are scaled by (range_kernel)
    int score_split;                    // 1: the scorer's hidden layer multiplies fp16 pieces of its fp32 operands
    int round_lag;                      // 1: bulk rounds are launched one ahead of the host's reads
    mf_cert_out *h_cert;
    // options
    int64_t theta, max_rounds;
    // timing
    hipEvent_t ev[10];              // 0..2 and 8: scoring stages; 3..7: solver stages
    float timings[T_COUNT];
    bool score_pending;             // score events recorded but not yet read
};

// One side of the auction as its kernels see it (rows bidding for columns, or the reverse).
struct SideArgs {
    const int32_t *A;                   // the bidding side's lines (W for rows, W^T for columns)
    long long pitch;
    int len;
    double *other_dual;                 // opposite duals as doubles, raised with atomicMax on the bits
    unsigned long long *otherword;      // opposite packed (dual, holder): the authoritative copy
    double eps, Kd;
    const int *line_len;                // optional: every entry of line b at or beyond line_len[b] is infeasible
    int typical_len;                    // what a scan reads on average (host-side choice of kernels only)
    // the same matrix by lines of the other side (line k of T is entry k of every line of A), when
    // that copy exists (else null): lets a search look at one entry of all bidding lines at once
    const int32_t *T;
    long long pitch_t;
    int len_t;                          // entries of a line of T = lines of A
    const int *line_len_t;              // optional, as line_len
    // optional: every line of A once more as a list of its feasible entries (position, weight),
    // list b at [edge_start[b], edge_start[b + 1]), both multiples of four, padding (0, infeasible)
    const long long *edge_start;
    const int *edge_col;
    const int32_t *edge_weight;
    int *rested;                        // optional: counts the bidders that rest (best value at most eps)
};

// score.hip
int mf_launch_score(mf_ctx *ctx, const mf_predictor *preds, int n_types, const int32_t *d_type,
                    const float *d_on, int n, const float *d_off, int m, int32_t *d_W, int64_t ldw,
                    float *d_sigma);
int mf_launch_rescore(mf_ctx *ctx, const mf_predictor *pred, const float *d_on, int n, const float *d_off,
                      int m, int32_t *d_W, int64_t ldw, const int32_t *d_rows, int n_rows,
                      const int32_t *d_cols, int n_cols);
// auction.hip
int mf_run_solver(mf_ctx *ctx, const int32_t *d_W, int n, int m, int64_t ldw,
                  int32_t *d_row2col, int64_t *d_u, int64_t *d_v, mf_result *h_res,
                  bool warm, const int32_t *d_reset_cols, int n_reset_cols, bool may_use_staged);
// edges.hip
int mf_count_edges(mf_ctx *ctx, const int32_t *d_W, int n, int m, int64_t ldw);
int mf_build_edge_lists(mf_ctx *ctx, const int32_t *d_W, int n, int m, int64_t ldw, SideArgs *side);
void mf_launch_list_round(mf_ctx *ctx, const SideArgs &s, int count, int ring);
inline size_t mf_edge_capacity(const mf_ctx *ctx)      // entries the lists may hold: half the staged copy's words each for columns and weights
{
    return ((size_t)ctx->max_n * ((((size_t)ctx->max_m + 3) & ~(size_t)3)) / 2) & ~(size_t)3;
}
// paths.hip
int mf_launch_path_search(mf_ctx *ctx, const SideArgs &s, int ring);
// certificate.hip
int mf_extract_duals(mf_ctx *ctx, const int32_t *A, int64_t lda, int rn, int rm, double Kd, const int *line_len,
                     int n, bool flip, bool staged, int32_t *d_row2col, int64_t *d_u, int64_t *d_v);
int mf_run_certificate(mf_ctx *ctx, const int32_t *d_W, int n, int m, int64_t ldw,
                       const int32_t *d_row2col, const int64_t *d_u, const int64_t *d_v,
                       int64_t K, mf_result *h_res);
