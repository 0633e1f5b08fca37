/*
 * muxmatch - the data-parallel core of matching-based GPU-sharing scheduling
 * on one AMD MI355X (gfx950).
 *
 * One scheduling round (paper: Section "Matching-based scheduling", Algorithm
 * "Scheduling algorithm") builds a bipartite graph between n online and m
 * offline workloads whose edge (u, v) carries the predicted normalised
 * throughput of v when it shares a GPU with u, and then takes the maximum
 * weighted matching of that graph as the sharing plan.  This library does the
 * two heavy steps on the GPU:
 *
 *   mf_score_pairs       every edge weight, from the speed-predictor MLP
 *   mf_solve_assignment  the maximum-weight matching, with a proof of optimality
 *   mf_check_certificate re-verifies such a proof on the device
 *   mf_schedule_round    the two steps back to back (one call per round)
 *   mf_*_typed           the same with one predictor per GPU type
 *   mf_schedule_round_update  the next periodic round: re-scores what changed
 *
 * Conventions shared by every call
 *   - Pointers named d_* are DEVICE pointers (HIP global memory on the device
 *     the context was created for); pointers named h_* are HOST pointers.
 *   - The caller owns every buffer it passes.  The library allocates nothing
 *     in these calls (all scratch lives in the context, sized at mf_create),
 *     never frees a caller buffer and keeps no caller pointer after return.
 *   - Matrices are row-major.  The weight matrix W has n rows (online) and m
 *     columns (offline) of int32 with a row pitch of ldw elements (ldw >= m).
 *     An entry equal to MF_INFEASIBLE means "this pair must not share a GPU";
 *     every other entry is a weight in [0, 2^30].  The calls that READ a
 *     matrix (mf_solve_assignment, mf_check_certificate*, mf_schedule_round*,
 *     which solves on what it scored) also need ldw to be a multiple of 4 and
 *     d_W 16-byte aligned (MF_ERR_ARG otherwise); mf_score_pairs* alone
 *     writes any pitch and alignment.
 *   - Work is enqueued on the stream given to mf_create.  mf_score_pairs*
 *     returns without waiting for its kernels (the typed variant waits once, to
 *     check the types; the next call on the same
 *     stream, or a synchronisation of it, orders after them); every call
 *     that takes an mf_result *h_res (required, not NULL) steers its
 *     iteration from the host, waits for its own work and fills *h_res.
 *     mf_check_certificate_noalloc takes its own stream and never waits.
 *   - Return value: MF_OK (0) or a negative MF_ERR_* code; nothing is thrown
 *     across this boundary.  On error the output buffers are unspecified.
 *   - A context may be used by one thread at a time.
 */
#ifndef MUXMATCH_H
#define MUXMATCH_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MF_INFEASIBLE INT32_MIN

enum {
    MF_OK = 0,
    MF_ERR_ARG = -1,            /* null pointer, non-positive size, bad pitch or alignment   */
    MF_ERR_SHAPE = -2,          /* a size beyond what the context was created for            */
    MF_ERR_HIP = -3,            /* a HIP runtime call failed (see mf_last_hip_error)         */
    MF_ERR_NOT_CONVERGED = -4,  /* the solver hit its round limit                            */
    MF_ERR_CERT = -5,           /* the optimality certificate did not verify                 */
    MF_ERR_RANGE = -6           /* weights too large for exact arithmetic at this n          */
};

typedef struct mf_ctx mf_ctx;

/*
 * The speed predictor P of the scheduling algorithm: an MLP with two hidden
 * layers of width H over the concatenated features [online ; offline] of a
 * pair (paper: Section "Matching-based scheduling" for the inputs and the
 * regression target; Section "Implementation" for the shape).  Hidden
 * activations are ReLU; the output goes through a logistic function and is
 * quantised to round-half-even(sigma * scale) as int32.
 * A pair whose memory fractions add up (one float32 addition) to more than
 * mem_limit is infeasible: feature index mem_feature of each side is that
 * fraction (paper: Section "Implementation", the offline memory quota).
 * Optional third input (paper: Algorithm "Scheduling algorithm", sm = DynamicSM(u, v)
 * is an argument of CalcNormTput; Section "Dynamic SM allocation"): with d_W1sm
 * not NULL the SM share of the pair,
 *   sm(u, v) = min(1 - x_u[sm_on_feature], x_v[sm_off_feature])   (float32),
 * the complement of the online workload's SM activity capped by what the
 * offline workload can use, enters layer 1 with weights d_W1sm[H] (the column
 * 2F of a [H][2F+1] first layer).  With d_W1sm NULL the two indices are ignored
 * and the SM share is whatever feature of the online workload carries it.
 * Optional second constraint (paper: Section "Lessons and future direction",
 * paragraph "Slowdown of online workloads": sharing must not slow the online
 * workload down too much, and what "too much" is stays the operator's choice):
 * with d_W3_slow not NULL the predictor has a second output unit on the same
 * hidden layers, logistic(d_W3_slow . h2 + d_b3_slow), read as the predicted
 * slowdown of the online workload of the pair as a fraction in (0, 1); a pair
 * whose prediction exceeds slow_limit is infeasible like one that does not fit
 * in memory.
 * All parameter pointers are DEVICE pointers to float32, row-major.
 */
typedef struct {
    int32_t F;                  /* features per workload (1..256)                       */
    int32_t H;                  /* hidden width: 64 or 128                              */
    float   scale;              /* S > 0; weights land in [0, S], S <= 2^30             */
    int32_t mem_feature;        /* 0 <= mem_feature < F                                 */
    float   mem_limit;          /* e.g. 1.0f                                            */
    const float *d_W1;          /* [H][2F]: columns [0,F) online, [F,2F) offline        */
    const float *d_b1;          /* [H]                                                  */
    const float *d_W2;          /* [H][H]                                               */
    const float *d_b2;          /* [H]                                                  */
    const float *d_W3;          /* [H]                                                  */
    const float *d_b3;          /* [1]                                                  */
    const float *d_W1sm;        /* [H] or NULL: weights of the pair-dependent SM input  */
    int32_t sm_on_feature;      /* online feature: SM activity of the online workload   */
    int32_t sm_off_feature;     /* offline feature: SM share the offline one can use    */
    const float *d_W3_slow;     /* [H] or NULL: output weights of the slowdown unit     */
    const float *d_b3_slow;     /* [1]  (with d_W3_slow)                                */
    float   slow_limit;         /* pairs predicted above it are infeasible              */
} mf_predictor;

/* Filled on the host by the solving calls. */
typedef struct {
    int64_t primal;             /* P: sum of matched weights (weight units)             */
    int64_t dual;               /* D: sum u + sum v (1/K weight units)                  */
    int64_t K;                  /* dual scale, K = min(n, m) + 1                        */
    int64_t min_reduced_cost;   /* min over feasible (i,j) of u_i + v_j - K*W_ij        */
    int64_t rounds;             /* bidding kernels run (forward + reverse)              */
    int64_t bids;               /* bids evaluated: each scans one row or column         */
    int64_t bytes_scanned;      /* weight-matrix bytes those scans read                 */
    int64_t chain_bids;         /* bids evaluated by the chain-following kernels        */
    int64_t chain_depth;        /* longest per-workgroup bid sequence, summed over them */
    int64_t chain_retries;      /* chain bids that lost and were redone                 */
    int64_t team_bids;          /* chain bids evaluated by several workgroups together  */
    int64_t path_steps;         /* super-steps of the shortest-augmenting-path searches */
    int64_t path_scans;         /* line scans those searches made                       */
    int32_t matched;            /* rows with a partner                                  */
    int32_t phases;             /* epsilon-scaling phases                               */
    int32_t cert_ok;            /* 1: matching valid, duals feasible, 0 <= D - K*P < K  */
    int32_t status;             /* same code the call returned                          */
    float   ms_solve;           /* device time of the auction (HIP events)              */
    float   ms_certify;         /* device time of dual extraction + certificate         */
    int32_t fallbacks;          /* MF_FALLBACK_* bits: kernels this solve had to do without */
} mf_result;

/* A bounded wait between cooperating workgroups ran out during the solve, and from then on it
 * went without the kernels that use such waits (every solve starts with all of them again).  The
 * result is exact either way; a set bit says the solve was slower than it should have been. */
#define MF_FALLBACK_TEAMS    1  /* several workgroups per chain of bids          */
#define MF_FALLBACK_SEARCHES 2  /* shortest-augmenting-path searches             */

/*
 * Creates a context bound to HIP device `device` and to `hip_stream` (a
 * hipStream_t passed as void*, NULL = the default stream).  Allocates all
 * scratch for problems up to max_n x max_m (each at most 2^20 - 2):
 * layer-1 projections, a transposed copy of the weight matrix and a copy with
 * rows and columns in order of memory fraction (4*max_n*max_m bytes each) and
 * O(max_n + max_m) solver state.
 * Fails with MF_ERR_HIP when no such device exists or memory runs out.
 */
int mf_create(mf_ctx **out, int device, void *hip_stream, int max_n, int max_m);
int mf_destroy(mf_ctx *ctx);

/*
 * Edge-building loop of the scheduling algorithm: for every pair (i, j)
 *   d_W[i*ldw + j] = quantised predictor output, or MF_INFEASIBLE.
 * d_on is [n][F], d_off is [m][F] float32 (device).  If d_sigma is not NULL
 * it must hold n*m floats and receives the unquantised score of every pair
 * (pitch m).  Padding columns [m, ldw) are left untouched.
 * Without d_sigma the kernel walks rows and columns in order of their memory
 * fraction and leaves out the MLP for pairs that cannot fit (option
 * "fit_order", default 1); d_W is the same either way.
 */
int mf_score_pairs(mf_ctx *ctx, const mf_predictor *pred,
                   const float *d_on, int n, const float *d_off, int m,
                   int32_t *d_W, int64_t ldw, float *d_sigma);

/*
 * GetMatching of the scheduling algorithm: a maximum-weight matching of the
 * bipartite graph given by d_W (any n, m: when there are more online than
 * offline workloads the solver works on the transposed problem and maps the
 * result back).  A matching is a set of feasible
 * pairs using each row and each column at most once; it need not be perfect.
 * Outputs (device): d_row2col[n] (partner column, -1 = none) and integral
 * duals d_u[n], d_v[m] in units of 1/K of a weight unit that satisfy
 *   u, v >= 0,  u_i + v_j >= K*W_ij on every feasible pair,
 *   0 <= sum u + sum v - K * (matched weight) < K,
 * which by LP duality proves the matching optimal.  The certificate is
 * evaluated on the device and reported in *h_res (host, required).
 * The optimum weight is unique; which optimal matching is returned is not.
 */
int mf_solve_assignment(mf_ctx *ctx, const int32_t *d_W, int n, int m, int64_t ldw,
                        int32_t *d_row2col, int64_t *d_u, int64_t *d_v, mf_result *h_res);

/*
 * Evaluates the certificate above for caller-supplied (row2col, u, v, K) on
 * the device: fills primal, dual, K, min_reduced_cost, matched and cert_ok of
 * *h_res.  Returns MF_OK when the check ran (look at cert_ok), an error code
 * when it could not.
 */
int mf_check_certificate(mf_ctx *ctx, const int32_t *d_W, int n, int m, int64_t ldw,
                         const int32_t *d_row2col, const int64_t *d_u, const int64_t *d_v,
                         int64_t K, mf_result *h_res);

/*
 * The same check for callers that cannot allocate device memory or create a
 * context at the point of the call: code running under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  It needs no context
 * and calls no allocating routine: the partial sums and the per-column marks
 * live in an array that is part of the library's image on every device
 * (256 bytes + 4 bytes per column, 256 KiB in all, held until the process
 * ends), so m is limited to MF_NOALLOC_MAX_COLS (MF_ERR_SHAPE beyond it, and
 * for n above 2^20 - 2); arguments are otherwise as above (MF_ERR_ARG for a
 * null pointer, a pitch that is not a multiple of 4, a d_W that is not
 * 16-byte aligned, K < 1).  The work is enqueued on `hip_stream` (a
 * hipStream_t, NULL = the default stream) of the CURRENT device and the call
 * returns without waiting; the result is written to *d_out, a DEVICE buffer
 * the caller owns, once the stream gets there.  The array is cleared by a
 * kernel at the start of each call (no memset node is recorded).  All calls
 * on one device share the one array: calls that overlap on a device (two
 * streams, two threads) race and must be serialised by the caller.
 */
#define MF_NOALLOC_MAX_COLS 65536
typedef struct {
    int64_t primal;             /* sum of matched weights                               */
    int64_t dual;               /* sum u + sum v                                        */
    int64_t K;                  /* as passed                                            */
    int64_t min_reduced_cost;   /* min over feasible (i,j) of u_i + v_j - K*W_ij        */
    int32_t matched;            /* rows with a partner                                  */
    int32_t flags;              /* bit 0 bad or duplicate column, 1 infeasible pair, 2 negative dual */
    int32_t cert_ok;            /* 1: matching valid, duals feasible, 0 <= D - K*P < K  */
    int32_t reserved;
} mf_certificate;
int mf_check_certificate_noalloc(void *hip_stream, const int32_t *d_W, int n, int m, int64_t ldw,
                                 const int32_t *d_row2col, const int64_t *d_u, const int64_t *d_v,
                                 int64_t K, mf_certificate *d_out);

/*
 * One scheduling round: mf_score_pairs into d_W, then mf_solve_assignment on
 * it.  Returns MF_ERR_CERT if the certificate does not verify.
 */
int mf_schedule_round(mf_ctx *ctx, const mf_predictor *pred,
                      const float *d_on, int n, const float *d_off, int m,
                      int32_t *d_W, int64_t ldw,
                      int32_t *d_row2col, int64_t *d_u, int64_t *d_v, mf_result *h_res);

/*
 * The next scheduling round.  The scheduler is invoked periodically on a
 * workload set that changes slowly (paper: Section "Implementation", "invokes
 * the scheduler periodically to schedule all offline workloads"; Section
 * "Evaluation", the 15-minute interval).  d_W must hold the matrix the previous
 * round on this context scored for the same n and m; d_on / d_off hold the
 * current features of all workloads; d_changed_on[n_changed_on] and
 * d_changed_off[n_changed_off] (device arrays of distinct indices, may be
 * empty) name the online / offline workloads whose features differ from that
 * round (changed or replaced).  Only their rows and columns of d_W are
 * re-scored; the matching is then solved again.  Outputs, certificate and
 * error codes are those of mf_schedule_round: the result is the exact optimum
 * of the updated matrix.  By default the matching starts from scratch; with
 * the option "warm_eps_units" > 0 it starts from the previous round's column
 * prices (those of the listed offline workloads reset to 0, unless
 * "warm_reset_cols" is 0) at epsilon = warm_eps_units weight units - still
 * exact, since every phase re-establishes its invariants from any non-negative
 * prices, but measured no faster on the benchmark workloads.
 * Index lists are checked on the device before use (MF_ERR_ARG if out of range).
 */
int mf_schedule_round_update(mf_ctx *ctx, const mf_predictor *pred,
                             const float *d_on, int n, const float *d_off, int m,
                             const int32_t *d_changed_on, int n_changed_on,
                             const int32_t *d_changed_off, int n_changed_off,
                             int32_t *d_W, int64_t ldw,
                             int32_t *d_row2col, int64_t *d_u, int64_t *d_v, mf_result *h_res);

/*
 * One predictor per GPU type (paper: Section "Matching-based scheduling": GPU
 * types perform differently, so an MLP is trained for each).  Online workload
 * i runs on a GPU of type d_type_on[i] in [0, n_types) (device array of n
 * int32) and every pair in its row is scored by preds[d_type_on[i]]
 * (host array of n_types predictors, 1 <= n_types <= 64).  The predictors
 * must agree on F, mem_feature, mem_limit and scale (else MF_ERR_ARG); their
 * hidden widths may differ.  Everything else is as in mf_score_pairs /
 * mf_schedule_round; a type out of range gives MF_ERR_ARG (checked on the
 * device before use, which waits for the stream once).
 */
int mf_score_pairs_typed(mf_ctx *ctx, const mf_predictor *preds, int n_types, const int32_t *d_type_on,
                         const float *d_on, int n, const float *d_off, int m,
                         int32_t *d_W, int64_t ldw, float *d_sigma);
int mf_schedule_round_typed(mf_ctx *ctx, const mf_predictor *preds, int n_types, const int32_t *d_type_on,
                            const float *d_on, int n, const float *d_off, int m, int32_t *d_W, int64_t ldw,
                            int32_t *d_row2col, int64_t *d_u, int64_t *d_v, mf_result *h_res);

/*
 * Options of a context, by name.  Unknown names and values out of range give MF_ERR_ARG.
 *
 * STABLE (what they mean will not change):
 *   "theta"            epsilon divisor per phase of the matching, 2..1024, default 24
 *   "max_rounds"       limit on evaluated bids per solve (MF_ERR_NOT_CONVERGED beyond), default 4e9
 *   "score_split"      1 (default): the scorer's hidden layer multiplies fp16 pieces of its fp32
 *                      operands (two pieces each, three products, fp32 accumulation: the scores
 *                      stay as close to an fp64 evaluation as with fp32 products, about 3e-7
 *                      relative, at a third of the time); 0: fp32 products
 *   "fit_order"        1 (default): scoring walks workloads in order of memory fraction and runs no
 *                      MLP for pairs that cannot fit; 0: every pair goes through the MLP
 *   "fit_prefix"       1 (default) / 0: allow mf_schedule_round to match on the context's
 *                      memory-ordered copy of the matrix, reading only each line's feasible prefix
 *   "fit_prefix_below" percent (default 50): ... when fewer of the pairs just scored can share; 0: never
 *   "edge_lists_from"  rows (default 4096) from which mf_solve_assignment keeps a matrix with fewer
 *                      than fit_prefix_below percent of feasible pairs also as per-row lists of
 *                      them, which its bidding rounds then read instead of whole rows; 0: never
 *   "warm_eps_units"   0 (default): mf_schedule_round_update matches from scratch; > 0: from the
 *                      previous prices at that epsilon, in weight units
 *   "warm_reset_cols"  1 (default): such a start takes replaced columns at price 0
 *
 * TUNING (defaults were measured on the benchmark rounds; names and meanings may change with
 * the kernels they steer; every setting leaves the result exactly optimal):
 *   phases   "phase_stop" (16) / "phase_keep" (4) / "phase_growth" (2): either side of a phase that
 *            only prepares prices ends once at most phase_stop bidders are unplaced (times
 *            phase_growth per phase before, while fewer than "phase_growth_rest" (32) bidders have
 *            given up in this solve; never more than one bidder in 64, at least path_max);
 *            the last phase_keep phases run until nobody is left to bid.  "phase_tail_steps" (64) /
 *            "phase_tail_sides" (1: rows bidding; 2: columns; 3: both) / "phase_tail_from" (8192
 *            lines): such a side also ends after that many dependent chain steps.  "final_jump" (0:
 *            off): epsilon in weight units at or below which the next phase is the last.
 *   rounds   "tail_max" (1024 bidders: below, one kernel follows the eviction chains), "bulk_shape"
 *            (0..4: threads x lines per workgroup with many bidders: 256x1, 64x4 (default), 64x2,
 *            128x4, 256x4), "bulk_share" (95: "many" is at least that share, in percent, of the
 *            side's lines and at least 2048; other rounds take one line per workgroup),
 *            "bulk_grid" (0: ten workgroups per compute unit), "round_lag" (1: the host
 *            reads a round's bidder count while the next round already runs; 0: after every round)
 *   chains   "chain_grid" (256 workgroups), "team_wide" (64) / "team_max" (8) / "team_size" (16) /
 *            "team_threads" (1024) / "team_regroup" (128): several workgroups per chain once so few
 *            chains are left
 *   searches "path_max" (16, at most 64; 0: none): bidders at or below which one device-wide
 *            shortest-augmenting-path search places them all, after "path_after" (256) chain
 *            steps; "path_grid" (0: one workgroup per compute unit), "path_width" (1024 epsilons),
 *            "path_frontier_rows" (1024), "path_pull" (0), "path_spin_limit" (2^22 polls a workgroup
 *            waits for the others before all give up; see mf_result.fallbacks)
 */
int mf_set_option(mf_ctx *ctx, const char *name, int64_t value);

/*
 * Device time, in milliseconds, of the kernels the last call on this context
 * launched, by stage, measured with HIP events on the context's stream:
 * what[0] layer-1 projections (and the memory ordering), [1] pair scoring,
 * [2] the bidding rounds in which every line of the bidding side scans (the
 * first of each phase), [3] how many of those ran, [4] preparation of the solve (largest
 * weight; the transposed copy when it is needed up front - otherwise it is made inside [7] when a
 * phase first needs it),
 * [5] dual extraction, [6] certificate, [7] the whole auction, [8] weight
 * bytes the rounds of [2] scanned, [9] the fraction of the n*m pairs the pair
 * kernel ran the MLP on (the rest could not fit in memory and were marked
 * infeasible without being scored).  Entries of stages that did not run are 0.
 */
int mf_last_timings(mf_ctx *ctx, float what[16]);

/*
 * Measured ceilings of the device, as second denominators next to the
 * published peaks (diagnostic; the scheduling round does not use it):
 * out[0] = TFLOP/s of a dependency-free stream of v_mfma_f32_32x32x2_f32 on
 * every compute unit (the matrix instruction of the scoring kernel), out[1] its
 * duration in ms; with d_buffer (device, 16-byte aligned, `bytes` long, only
 * read) out[2] = GB/s of a plain streaming read of it and out[3] its duration;
 * out[4], out[5] = the same as out[0], out[1] for v_mfma_f32_32x32x16_f16 (the
 * instruction of the default scoring path); out[6], out[7] = 0.  Waits for the stream.
 */
int mf_measure_ceilings(mf_ctx *ctx, const void *d_buffer, int64_t bytes, float out[8]);

const char *mf_strerror(int code);
const char *mf_last_hip_error(mf_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* MUXMATCH_H */
