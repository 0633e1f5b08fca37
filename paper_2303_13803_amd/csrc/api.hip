// C entry points: argument checks, context life cycle, stage timing.
#include "internal.h"
#include <stdlib.h>
#include <string.h>
#include <new>

namespace {

template <typename T> hipError_t dev_alloc(T **p, size_t count)
{
    return hipMalloc((void **)p, count * sizeof(T));
}

bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

int check_matrix(const mf_ctx *ctx, const void *d_W, int n, int m, int64_t ldw)
{
    if (!ctx || !d_W || n <= 0 || m <= 0 || ldw < m || (ldw & 3) || !aligned16(d_W)) return MF_ERR_ARG;
    if (n > ctx->max_n || m > ctx->max_m) return MF_ERR_SHAPE;
    return MF_OK;
}

int check_predictor(const mf_predictor *p)
{
    if (!p || !p->d_W1 || !p->d_b1 || !p->d_W2 || !p->d_b2 || !p->d_W3 || !p->d_b3) return MF_ERR_ARG;
    if (p->F < 1 || p->F > 256 || (p->H != 64 && p->H != 128)) return MF_ERR_ARG;
    if (!(p->scale > 0.0f) || p->scale > 1073741824.0f) return MF_ERR_ARG;
    if (p->mem_feature < 0 || p->mem_feature >= p->F) return MF_ERR_ARG;
    if (!aligned16(p->d_W2) || !aligned16(p->d_b2) || !aligned16(p->d_W3)) return MF_ERR_ARG;
    if (p->d_W3_slow && (!aligned16(p->d_W3_slow) || !p->d_b3_slow || !(p->slow_limit == p->slow_limit))) return MF_ERR_ARG;
    if (p->d_W1sm && (!aligned16(p->d_W1sm) || p->sm_on_feature < 0 || p->sm_on_feature >= p->F ||
                      p->sm_off_feature < 0 || p->sm_off_feature >= p->F))
        return MF_ERR_ARG;
    return MF_OK;
}

// one predictor per GPU type: same inputs, same quantisation, same memory rule
int check_predictors(const mf_predictor *preds, int n_types)
{
    if (!preds || n_types < 1 || n_types > MF_MAX_TYPES) return MF_ERR_ARG;
    for (int t = 0; t < n_types; ++t) {
        const int rc = check_predictor(&preds[t]);
        if (rc != MF_OK) return rc;
        if (preds[t].F != preds[0].F || preds[t].mem_feature != preds[0].mem_feature ||
            preds[t].mem_limit != preds[0].mem_limit || preds[t].scale != preds[0].scale ||
            (preds[t].d_W1sm != nullptr) != (preds[0].d_W1sm != nullptr) ||
            (preds[t].d_W3_slow != nullptr) != (preds[0].d_W3_slow != nullptr) ||
            (preds[0].d_W1sm && (preds[t].sm_on_feature != preds[0].sm_on_feature ||
                                 preds[t].sm_off_feature != preds[0].sm_off_feature)))
            return MF_ERR_ARG;
    }
    return MF_OK;
}

void clear_timings(mf_ctx *ctx)
{
    memset(ctx->timings, 0, sizeof(ctx->timings));
    ctx->score_pending = false;
}

int finish_score_timing(mf_ctx *ctx)
{
    MF_HIP(hipMemcpyAsync(ctx->h_pairs_evaluated, ctx->pairs_evaluated, sizeof(unsigned long long),
                          hipMemcpyDeviceToHost, ctx->stream));
    MF_HIP(hipStreamSynchronize(ctx->stream));
    float a = 0.0f, b = 0.0f;
    float c = 0.0f;
    MF_HIP(hipEventElapsedTime(&a, ctx->ev[0], ctx->ev[1]));
    MF_HIP(hipEventElapsedTime(&b, ctx->ev[1], ctx->ev[2]));
    MF_HIP(hipEventElapsedTime(&c, ctx->ev[2], ctx->ev[8]));      // putting the columns back in place
    ctx->timings[T_PROJ] = a + c;
    ctx->timings[T_PAIR] = b;
    ctx->timings[T_PAIR_EVALUATED] = ctx->pairs_total > 0 ? (float)((double)*ctx->h_pairs_evaluated / ctx->pairs_total) : 0.0f;
    ctx->score_pending = false;
    return MF_OK;
}

}  // namespace

extern "C" {

int mf_create(mf_ctx **out, int device, void *hip_stream, int max_n, int max_m)
{
    if (!out || max_n <= 0 || max_m <= 0 || max_n > MF_MAX_DIM || max_m > MF_MAX_DIM) return MF_ERR_ARG;
    *out = nullptr;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || device < 0 || device >= ndev) return MF_ERR_HIP;
    if (hipSetDevice(device) != hipSuccess) return MF_ERR_HIP;
    mf_ctx *ctx = new (std::nothrow) mf_ctx();
    if (!ctx) return MF_ERR_HIP;
    memset(ctx, 0, sizeof(*ctx));
    ctx->device = device;
    ctx->stream = (hipStream_t)hip_stream;
    ctx->max_n = max_n;
    ctx->max_m = max_m;
    ctx->theta = 24;
    ctx->max_rounds = 4000000000ll;
    ctx->tail_max = 1024;
    ctx->round_lag = 1;
    ctx->score_split = 1;
    ctx->phase_stop = 16;
    ctx->phase_keep = 4;
    ctx->phase_growth = 2;
    ctx->phase_growth_rest = 32;
    ctx->final_jump = 0;
    ctx->phase_tail_steps = 64;
    ctx->phase_tail_sides = 1;
    ctx->phase_tail_from = 8192;
    ctx->warm_eps_units = 0;
    ctx->warm_reset_cols = true;
    ctx->chain_grid = 256;
    ctx->bulk_shape = 1;
    ctx->bulk_grid = 0;
    ctx->bulk_share = 95;
    ctx->team_max = 8;
    ctx->team_size = 16;
    ctx->team_wide = 64;
    ctx->team_regroup = 128;
    ctx->team_threads = 1024;
    ctx->fit_order = true;
    ctx->fit_prefix = true;
    ctx->fit_prefix_below = 50;
    ctx->edge_lists_from = 4096;
    ctx->path_max = 16;
    ctx->path_width = 1024;
    ctx->path_frontier_rows = 1024;
    ctx->path_pull = false;
    ctx->path_grid = 0;
    ctx->path_after = 256;
    ctx->path_spin_limit = 1u << 22;
    {
        hipDeviceProp_t prop;
        ctx->n_cus = hipGetDeviceProperties(&prop, device) == hipSuccess ? prop.multiProcessorCount : 0;
    }
    const size_t nm = (size_t)(max_n > max_m ? max_n : max_m);   // either side may be the one that bids first
    const size_t ldt = ((size_t)max_n + 3) & ~(size_t)3;
    hipError_t e = hipSuccess;
#define TRY(x) do { if (e == hipSuccess) e = (x); } while (0)
    TRY(dev_alloc(&ctx->proj_on, (size_t)max_n * 128));
    TRY(dev_alloc(&ctx->proj_off, (size_t)max_m * 128));
    TRY(dev_alloc(&ctx->mem_on, (size_t)max_n));
    TRY(dev_alloc(&ctx->mem_off, (size_t)max_m));
    TRY(dev_alloc(&ctx->sm_on, (size_t)max_n));
    TRY(dev_alloc(&ctx->sm_off, (size_t)max_m));
    TRY(dev_alloc(&ctx->order_on, (size_t)max_n));
    TRY(dev_alloc(&ctx->order_off, (size_t)max_m));
    TRY(dev_alloc(&ctx->rank_off, (size_t)max_m));
    TRY(dev_alloc(&ctx->rank_on, (size_t)max_n));
    TRY(dev_alloc(&ctx->mem_on_sorted, (size_t)max_n));
    TRY(dev_alloc(&ctx->mem_off_sorted, (size_t)max_m + 4));
    TRY(dev_alloc(&ctx->fit_len_on, (size_t)max_n));
    TRY(dev_alloc(&ctx->fit_len_off, (size_t)max_m));
    TRY(dev_alloc(&ctx->staged, (size_t)max_n * ((((size_t)max_m + 3) & ~(size_t)3))));
    TRY(dev_alloc(&ctx->type_segment, (size_t)MF_MAX_TYPES + 1));
    TRY(dev_alloc(&ctx->pairs_evaluated, 1));
    TRY(dev_alloc(&ctx->feasible_pairs, 1));
    TRY(dev_alloc(&ctx->largest_weight, 1));
    TRY(hipHostMalloc((void **)&ctx->h_feasible_pairs, sizeof(unsigned long long)));
    TRY(hipHostMalloc((void **)&ctx->h_pairs_evaluated, sizeof(unsigned long long)));
    TRY(dev_alloc(&ctx->wt, (size_t)max_m * ldt));
    TRY(dev_alloc(&ctx->price, nm + 8));
    TRY(dev_alloc(&ctx->profit, nm + 8));
    TRY(dev_alloc(&ctx->colword, nm));
    TRY(dev_alloc(&ctx->roword, nm));
    TRY(dev_alloc(&ctx->row2col, nm));
    TRY(dev_alloc(&ctx->col2row, nm));
    TRY(hipMalloc(&ctx->team_ctl, 128 * 1024));
    TRY(hipMalloc(&ctx->path_ctl, 32768));
    TRY(dev_alloc(&ctx->path_label, nm + 8));      // (read in groups of four, like the duals)
    TRY(dev_alloc(&ctx->path_expanded, nm));
    for (int k = 0; k < 2; ++k) {
        TRY(dev_alloc(&ctx->path_frontier[k], nm * 16));
    }
    TRY(dev_alloc(&ctx->path_held, nm));
    TRY(dev_alloc(&ctx->path_base, nm + 8));
    TRY(dev_alloc(&ctx->edge_count, nm));
    TRY(dev_alloc(&ctx->edge_start, nm + 1));
    TRY(dev_alloc(&ctx->path_tree, nm));
    TRY(dev_alloc(&ctx->path_parent, nm));
    TRY(dev_alloc(&ctx->path_jump, nm));
    TRY(dev_alloc(&ctx->path_stamp, nm));
    TRY(dev_alloc(&ctx->list[0], nm));
    TRY(dev_alloc(&ctx->list[1], nm));
    TRY(dev_alloc(&ctx->colmark, (size_t)max_m));
    TRY(dev_alloc(&ctx->stats, 1));
    TRY(dev_alloc(&ctx->cert, 1));
    TRY(hipMalloc((void **)&ctx->score_range, 8 * sizeof(unsigned)));
    TRY(hipHostMalloc((void **)&ctx->h_stats, sizeof(mf_device_stats)));
    for (int i = 0; i < 2; ++i) {
        TRY(hipHostMalloc((void **)&ctx->h_stats_slot[i], sizeof(mf_device_stats)));
        TRY(hipEventCreate(&ctx->ev_stats[i]));
    }
    TRY(hipHostMalloc((void **)&ctx->h_cert, sizeof(mf_cert_out)));
    for (int i = 0; i < 10; ++i) TRY(hipEventCreate(&ctx->ev[i]));
#undef TRY
    if (e != hipSuccess) {
        ctx->hip_error = e;
        mf_destroy(ctx);
        return MF_ERR_HIP;
    }
    *out = ctx;
    return MF_OK;
}

int mf_destroy(mf_ctx *ctx)
{
    if (!ctx) return MF_ERR_ARG;
    (void)hipSetDevice(ctx->device);
    (void)hipStreamSynchronize(ctx->stream);
    void *dev[] = {ctx->score_range, ctx->proj_on, ctx->proj_off, ctx->mem_on, ctx->mem_off, ctx->sm_on, ctx->sm_off, ctx->order_on, ctx->order_off, ctx->rank_off, ctx->rank_on, ctx->mem_on_sorted, ctx->mem_off_sorted, ctx->fit_len_on, ctx->fit_len_off, ctx->staged, ctx->type_segment, ctx->pairs_evaluated, ctx->feasible_pairs, ctx->largest_weight, ctx->wt, ctx->price,
                   ctx->profit, ctx->colword, ctx->roword, ctx->row2col, ctx->col2row, ctx->team_ctl, ctx->path_ctl, ctx->path_label, ctx->path_expanded, ctx->path_frontier[0], ctx->path_frontier[1], ctx->path_stamp, ctx->path_held, ctx->path_base, ctx->path_tree, ctx->path_parent, ctx->path_jump, ctx->edge_count, ctx->edge_start, ctx->list[0], ctx->list[1], ctx->colmark, ctx->stats,
                   ctx->cert};
    for (void *p : dev) if (p) (void)hipFree(p);
    if (ctx->h_stats) (void)hipHostFree(ctx->h_stats);
    for (int i = 0; i < 2; ++i) {
        if (ctx->h_stats_slot[i]) (void)hipHostFree(ctx->h_stats_slot[i]);
        if (ctx->ev_stats[i]) (void)hipEventDestroy(ctx->ev_stats[i]);
    }
    if (ctx->h_cert) (void)hipHostFree(ctx->h_cert);
    if (ctx->h_pairs_evaluated) (void)hipHostFree(ctx->h_pairs_evaluated);
    if (ctx->h_feasible_pairs) (void)hipHostFree(ctx->h_feasible_pairs);
    for (int i = 0; i < 10; ++i) if (ctx->ev[i]) (void)hipEventDestroy(ctx->ev[i]);
    delete ctx;
    return MF_OK;
}

int mf_score_pairs(mf_ctx *ctx, const mf_predictor *pred, const float *d_on, int n,
                   const float *d_off, int m, int32_t *d_W, int64_t ldw, float *d_sigma)
{
    if (!ctx || !d_on || !d_off || !d_W || n <= 0 || m <= 0 || ldw < m) return MF_ERR_ARG;
    int rc = check_predictor(pred);
    if (rc != MF_OK) return rc;
    if (n > ctx->max_n || m > ctx->max_m) return MF_ERR_SHAPE;
    MF_HIP(hipSetDevice(ctx->device));
    clear_timings(ctx);
    return mf_launch_score(ctx, pred, 1, nullptr, d_on, n, d_off, m, d_W, ldw, d_sigma);
}

int mf_solve_assignment(mf_ctx *ctx, const int32_t *d_W, int n, int m, int64_t ldw,
                        int32_t *d_row2col, int64_t *d_u, int64_t *d_v, mf_result *h_res)
{
    if (!d_row2col || !d_u || !d_v || !h_res) return MF_ERR_ARG;
    int rc = check_matrix(ctx, d_W, n, m, ldw);
    if (rc != MF_OK) return rc;
    MF_HIP(hipSetDevice(ctx->device));
    clear_timings(ctx);
    memset(h_res, 0, sizeof(*h_res));
    rc = mf_run_solver(ctx, d_W, n, m, ldw, d_row2col, d_u, d_v, h_res, false, nullptr, 0, false);
    h_res->status = rc;
    return rc;
}

int mf_check_certificate(mf_ctx *ctx, const int32_t *d_W, int n, int m, int64_t ldw,
                         const int32_t *d_row2col, const int64_t *d_u, const int64_t *d_v,
                         int64_t K, mf_result *h_res)
{
    if (!d_row2col || !d_u || !d_v || !h_res || K < 1) return MF_ERR_ARG;
    int rc = check_matrix(ctx, d_W, n, m, ldw);
    if (rc != MF_OK) return rc;
    MF_HIP(hipSetDevice(ctx->device));
    clear_timings(ctx);
    memset(h_res, 0, sizeof(*h_res));
    MF_HIP(hipEventRecord(ctx->ev[5], ctx->stream));
    rc = mf_run_certificate(ctx, d_W, n, m, ldw, d_row2col, d_u, d_v, K, h_res);
    if (rc == MF_OK) {
        MF_HIP(hipEventRecord(ctx->ev[6], ctx->stream));
        MF_HIP(hipStreamSynchronize(ctx->stream));
        MF_HIP(hipEventElapsedTime(&ctx->timings[T_CERT], ctx->ev[5], ctx->ev[6]));
        h_res->ms_certify = ctx->timings[T_CERT];
    }
    h_res->status = rc;
    return rc;
}

int mf_schedule_round(mf_ctx *ctx, const mf_predictor *pred, const float *d_on, int n,
                      const float *d_off, int m, int32_t *d_W, int64_t ldw,
                      int32_t *d_row2col, int64_t *d_u, int64_t *d_v, mf_result *h_res)
{
    if (!d_on || !d_off || !d_row2col || !d_u || !d_v || !h_res) return MF_ERR_ARG;
    int rc = check_matrix(ctx, d_W, n, m, ldw);
    if (rc != MF_OK) return rc;
    rc = check_predictor(pred);
    if (rc != MF_OK) return rc;
    MF_HIP(hipSetDevice(ctx->device));
    clear_timings(ctx);
    memset(h_res, 0, sizeof(*h_res));
    rc = mf_launch_score(ctx, pred, 1, nullptr, d_on, n, d_off, m, d_W, ldw, nullptr);
    if (rc == MF_OK) rc = mf_run_solver(ctx, d_W, n, m, ldw, d_row2col, d_u, d_v, h_res, false, nullptr, 0, true);
    if (rc == MF_OK || rc == MF_ERR_CERT) {
        int rt = finish_score_timing(ctx);
        if (rt != MF_OK) rc = rt;
    }
    h_res->status = rc;
    return rc;
}

int mf_score_pairs_typed(mf_ctx *ctx, const mf_predictor *preds, int n_types, const int32_t *d_type_on,
                         const float *d_on, int n, const float *d_off, int m,
                         int32_t *d_W, int64_t ldw, float *d_sigma)
{
    if (!ctx || !d_type_on || !d_on || !d_off || !d_W || n <= 0 || m <= 0 || ldw < m) return MF_ERR_ARG;
    int rc = check_predictors(preds, n_types);
    if (rc != MF_OK) return rc;
    if (n > ctx->max_n || m > ctx->max_m) return MF_ERR_SHAPE;
    MF_HIP(hipSetDevice(ctx->device));
    clear_timings(ctx);
    return mf_launch_score(ctx, preds, n_types, d_type_on, d_on, n, d_off, m, d_W, ldw, d_sigma);
}

int mf_schedule_round_typed(mf_ctx *ctx, const mf_predictor *preds, int n_types, const int32_t *d_type_on,
                            const float *d_on, int n, const float *d_off, int m, int32_t *d_W, int64_t ldw,
                            int32_t *d_row2col, int64_t *d_u, int64_t *d_v, mf_result *h_res)
{
    if (!d_type_on || !d_on || !d_off || !d_row2col || !d_u || !d_v || !h_res) return MF_ERR_ARG;
    int rc = check_matrix(ctx, d_W, n, m, ldw);
    if (rc != MF_OK) return rc;
    rc = check_predictors(preds, n_types);
    if (rc != MF_OK) return rc;
    MF_HIP(hipSetDevice(ctx->device));
    clear_timings(ctx);
    memset(h_res, 0, sizeof(*h_res));
    rc = mf_launch_score(ctx, preds, n_types, d_type_on, d_on, n, d_off, m, d_W, ldw, nullptr);
    if (rc == MF_OK) rc = mf_run_solver(ctx, d_W, n, m, ldw, d_row2col, d_u, d_v, h_res, false, nullptr, 0, true);
    if (rc == MF_OK || rc == MF_ERR_CERT) {
        int rt = finish_score_timing(ctx);
        if (rt != MF_OK) rc = rt;
    }
    h_res->status = rc;
    return rc;
}

int mf_schedule_round_update(mf_ctx *ctx, const mf_predictor *pred, const float *d_on, int n,
                             const float *d_off, int m, const int32_t *d_changed_on, int n_changed_on,
                             const int32_t *d_changed_off, int n_changed_off, int32_t *d_W, int64_t ldw,
                             int32_t *d_row2col, int64_t *d_u, int64_t *d_v, mf_result *h_res)
{
    if (!d_on || !d_off || !d_row2col || !d_u || !d_v || !h_res) return MF_ERR_ARG;
    if (n_changed_on < 0 || n_changed_off < 0 || (n_changed_on > 0 && !d_changed_on) ||
        (n_changed_off > 0 && !d_changed_off))
        return MF_ERR_ARG;
    int rc = check_matrix(ctx, d_W, n, m, ldw);
    if (rc != MF_OK) return rc;
    rc = check_predictor(pred);
    if (rc != MF_OK) return rc;
    if (n_changed_on > n || n_changed_off > m) return MF_ERR_SHAPE;
    MF_HIP(hipSetDevice(ctx->device));
    clear_timings(ctx);
    memset(h_res, 0, sizeof(*h_res));
    rc = mf_launch_rescore(ctx, pred, d_on, n, d_off, m, d_W, ldw, d_changed_on, n_changed_on,
                           d_changed_off, n_changed_off);
    if (rc == MF_OK)
        rc = mf_run_solver(ctx, d_W, n, m, ldw, d_row2col, d_u, d_v, h_res, ctx->warm_eps_units > 0, d_changed_off,
                           ctx->warm_reset_cols ? n_changed_off : 0, false);
    if (rc == MF_OK || rc == MF_ERR_CERT) {
        int rt = finish_score_timing(ctx);
        if (rt != MF_OK) rc = rt;
    }
    h_res->status = rc;
    return rc;
}

int mf_set_option(mf_ctx *ctx, const char *name, int64_t value)
{
    if (!ctx || !name) return MF_ERR_ARG;
    if (!strcmp(name, "theta")) { if (value < 2 || value > 1024) return MF_ERR_ARG; ctx->theta = value; return MF_OK; }
    if (!strcmp(name, "phase_keep")) { if (value < 1 || value > 64) return MF_ERR_ARG; ctx->phase_keep = (int)value; return MF_OK; }
    if (!strcmp(name, "phase_tail_steps")) { if (value < 0) return MF_ERR_ARG; ctx->phase_tail_steps = value; return MF_OK; }
    if (!strcmp(name, "phase_tail_from")) { if (value < 0 || value > (1 << 20)) return MF_ERR_ARG; ctx->phase_tail_from = (int)value; return MF_OK; }
    if (!strcmp(name, "phase_tail_sides")) { if (value < 0 || value > 3) return MF_ERR_ARG; ctx->phase_tail_sides = (int)value; return MF_OK; }
    if (!strcmp(name, "final_jump")) { if (value < 0 || value > (1 << 30)) return MF_ERR_ARG; ctx->final_jump = value; return MF_OK; }
    if (!strcmp(name, "phase_growth_rest")) { if (value < 0 || value > (1 << 20)) return MF_ERR_ARG; ctx->phase_growth_rest = (int)value; return MF_OK; }
    if (!strcmp(name, "phase_growth")) { if (value < 1 || value > 64) return MF_ERR_ARG; ctx->phase_growth = (int)value; return MF_OK; }
    if (!strcmp(name, "phase_stop")) { if (value < 0 || value > (1 << 20)) return MF_ERR_ARG; ctx->phase_stop = (int)value; return MF_OK; }
    if (!strcmp(name, "score_split")) { if (value < 0 || value > 1) return MF_ERR_ARG; ctx->score_split = (int)value; return MF_OK; }
    if (!strcmp(name, "round_lag")) { if (value < 0 || value > 1) return MF_ERR_ARG; ctx->round_lag = (int)value; return MF_OK; }
    if (!strcmp(name, "tail_max")) { if (value < 0 || value > (1 << 20)) return MF_ERR_ARG; ctx->tail_max = (int)value; return MF_OK; }
    if (!strcmp(name, "bulk_grid")) { if (value < 0 || value > 8192) return MF_ERR_ARG; ctx->bulk_grid = (int)value; return MF_OK; }
    if (!strcmp(name, "bulk_share")) { if (value < 0 || value > 100) return MF_ERR_ARG; ctx->bulk_share = (int)value; return MF_OK; }
    if (!strcmp(name, "bulk_shape")) { if (value < 0 || value > 4) return MF_ERR_ARG; ctx->bulk_shape = (int)value; return MF_OK; }
    if (!strcmp(name, "warm_reset_cols")) { ctx->warm_reset_cols = value != 0; return MF_OK; }
    if (!strcmp(name, "warm_eps_units")) { if (value < 0 || value > (1 << 30)) return MF_ERR_ARG; ctx->warm_eps_units = value; return MF_OK; }
    if (!strcmp(name, "team_max")) { if (value < 0 || value > 16) return MF_ERR_ARG; ctx->team_max = (int)value; return MF_OK; }
    if (!strcmp(name, "team_wide")) { if (value < 0 || value > 64) return MF_ERR_ARG; ctx->team_wide = (int)value; return MF_OK; }
    if (!strcmp(name, "team_regroup")) { if (value < 1) return MF_ERR_ARG; ctx->team_regroup = value; return MF_OK; }
    if (!strcmp(name, "team_size")) { if (value < 2 || value > 32) return MF_ERR_ARG; ctx->team_size = (int)value; return MF_OK; }
    if (!strcmp(name, "team_threads")) { if (value != 64 && value != 128 && value != 256 && value != 512 && value != 1024) return MF_ERR_ARG; ctx->team_threads = (int)value; return MF_OK; }
    if (!strcmp(name, "chain_grid")) { if (value < 1 || value > 4096) return MF_ERR_ARG; ctx->chain_grid = (int)value; return MF_OK; }
    if (!strcmp(name, "path_max")) { if (value < 0 || value > 64) return MF_ERR_ARG; ctx->path_max = (int)value; return MF_OK; }
    if (!strcmp(name, "path_spin_limit")) { if (value < 0 || value > (1ll << 30)) return MF_ERR_ARG; ctx->path_spin_limit = (unsigned)value; return MF_OK; }
    if (!strcmp(name, "path_after")) { if (value < 0) return MF_ERR_ARG; ctx->path_after = value; return MF_OK; }
    if (!strcmp(name, "path_grid")) { if (value < 0 || value > 1024) return MF_ERR_ARG; ctx->path_grid = (int)value; return MF_OK; }
    if (!strcmp(name, "path_pull")) { ctx->path_pull = value != 0; return MF_OK; }
    if (!strcmp(name, "path_frontier_rows")) { if (value < 8 || value > (1 << 20)) return MF_ERR_ARG; ctx->path_frontier_rows = (int)value; return MF_OK; }
    if (!strcmp(name, "path_width")) { if (value < 1 || value > (1 << 30)) return MF_ERR_ARG; ctx->path_width = (int)value; return MF_OK; }
    if (!strcmp(name, "edge_lists_from")) { if (value < 0 || value > (1 << 20)) return MF_ERR_ARG; ctx->edge_lists_from = (int)value; return MF_OK; }
    if (!strcmp(name, "fit_prefix_below")) { if (value < 0 || value > 101) return MF_ERR_ARG; ctx->fit_prefix_below = (int)value; return MF_OK; }
    if (!strcmp(name, "fit_prefix")) { ctx->fit_prefix = value != 0; return MF_OK; }
    if (!strcmp(name, "fit_order")) { ctx->fit_order = value != 0; return MF_OK; }
    if (!strcmp(name, "max_rounds")) { if (value < 1) return MF_ERR_ARG; ctx->max_rounds = value; return MF_OK; }
    return MF_ERR_ARG;
}

int mf_last_timings(mf_ctx *ctx, float what[16])
{
    if (!ctx || !what) return MF_ERR_ARG;
    if (ctx->score_pending) {           // a bare mf_score_pairs does not wait for its events
        int rc = finish_score_timing(ctx);
        if (rc != MF_OK) return rc;
    }
    memcpy(what, ctx->timings, sizeof(float) * 16);
    return MF_OK;
}

const char *mf_strerror(int code)
{
    switch (code) {
    case MF_OK: return "ok";
    case MF_ERR_ARG: return "bad argument (null pointer, non-positive size, pitch or alignment)";
    case MF_ERR_SHAPE: return "shape larger than the context was created for (or than the call supports)";
    case MF_ERR_HIP: return "HIP runtime error";
    case MF_ERR_NOT_CONVERGED: return "round limit reached before the auction finished";
    case MF_ERR_CERT: return "optimality certificate did not verify";
    case MF_ERR_RANGE: return "weights too large for exact arithmetic at this size";
    default: return "unknown error";
    }
}

const char *mf_last_hip_error(mf_ctx *ctx)
{
    return ctx ? hipGetErrorString(ctx->hip_error) : "no context";
}

}  // extern "C"
