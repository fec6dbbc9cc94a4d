// C-ABI entry points: host-side argument checks, workspace layout, launch sequences.
#include "internal.hpp"
#include <string.h>
#include <mutex>

namespace ab {

ab_trace_fn g_trace_fn = nullptr;
void *g_trace_user = nullptr;

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
static inline int round_up(int x, int a) { return (x + a - 1) / a * a; }

static int pick_tile(int64_t M, int N)
{
    for (int tile = TILE_BIG; tile > TILE_SMALL; --tile) {
        const int edge = tile_edge(tile);
        if (N % edge != 0) continue;
        if (((M + edge - 1) / edge) * (N / edge) >= 512) return tile;
    }
    return TILE_SMALL;
}

static ab_status check_desc(const ab_model_desc *d)
{
    if (!d) return AB_ERR_NULL;
    if (d->compute_dtype != AB_F32 && d->compute_dtype != AB_BF16) return AB_ERR_DTYPE;
    if (d->n_layers <= 0 || d->n_stats <= 0 || d->n_stats > AB_MAX_STATS) return AB_ERR_SHAPE;
    if (d->n_scalars < 0 || d->n_scalars > AB_MAX_SCALARS) return AB_ERR_SHAPE;
    if (d->n_hidden < 0 || d->n_hidden > AB_MAX_HIDDEN) return AB_ERR_SHAPE;
    if (d->n_hidden == 0 && d->tensor_encoder) return AB_ERR_UNSUPPORTED;   // the linear scorer takes flat statistics only
    for (int k = 0; k < d->n_hidden; ++k) {
        if (d->hidden[k] <= 0) return AB_ERR_SHAPE;
        if (d->hidden[k] % 64 != 0 || d->hidden[k] > 4096) return AB_ERR_UNSUPPORTED;
    }
    for (int k = 0; k < d->n_stats; ++k)
        if (d->enc_stat[k].kind != AB_ENC_LINEAR && d->enc_stat[k].kind != AB_ENC_LOG) return AB_ERR_SHAPE;
    for (int k = 0; k < d->n_scalars; ++k)
        if (d->enc_scalar[k].kind != AB_ENC_LINEAR && d->enc_scalar[k].kind != AB_ENC_LOG) return AB_ERR_SHAPE;
    if (d->n_outputs < 0 || d->n_outputs > AB_MAX_OUTPUTS) return AB_ERR_SHAPE;
    if (d->loss_kind != AB_LOSS_MSE && d->loss_kind != AB_LOSS_L2NORM) return AB_ERR_SHAPE;
    if (d->tensor_encoder < 0 || d->tensor_encoder > 2) return AB_ERR_SHAPE;
    if (d->tensor_encoder) {
        if (d->enc_hidden[0] <= 0 || d->enc_hidden[1] <= 0) return AB_ERR_SHAPE;
        if (d->n_stats > AB_MAX_ENCODER_STATS) return AB_ERR_UNSUPPORTED;
        if (d->tensor_encoder == 1 && (d->enc_hidden[0] != 128 || d->enc_hidden[1] != 128)) return AB_ERR_UNSUPPORTED;
        if (d->tensor_encoder == 2 && (d->enc_hidden[0] != 32 || d->enc_hidden[1] != 64)) return AB_ERR_UNSUPPORTED;
        if (d->compute_dtype != AB_BF16) return AB_ERR_UNSUPPORTED;
    } else if ((int64_t)d->n_layers * d->n_stats > (1 << 20)) {
        return AB_ERR_UNSUPPORTED;
    }
    return AB_OK;
}

struct ScorePlan {
    int dtype, Fs, F, Kp, D, base;
    int H[AB_MAX_HIDDEN];
    int tile[AB_MAX_HIDDEN];      // tile of hidden GEMM k (k >= 1)
    int big[AB_MAX_HIDDEN];       // hidden GEMM k runs on the 256x256 bf16 kernel
    int tile_a;                   // tile of the scenario-term GEMM
    int nt_last;
    int64_t chunk_scen, chunk_rows;
    size_t off_xs, off_w1s, off_aterm, off_bterm, off_cfgv, off_wout, off_xrow, off_partial, off_act0, off_act1, total;
    // second pass for the chosen candidate's prediction vector: one row per scenario, kVChunk scenarios at a time
    int64_t v_chunk;
    int v_tile[AB_MAX_HIDDEN];
    size_t off_vx, off_vact0, off_vact1, off_vlast;
};

static const int64_t kTargetChunkRows = 1 << 20;
static const int64_t kVChunk = 4096;

static ab_status plan_scoring(const ab_model_desc *d, int64_t S, int32_t C, ScorePlan *p)
{
    memset(p, 0, sizeof(*p));
    p->dtype = d->compute_dtype;
    p->base = d->tensor_encoder == 2 ? 3 : d->tensor_encoder ? 2 : 0;
    p->Fs = (d->tensor_encoder ? d->enc_hidden[1] : d->n_layers * d->n_stats) + d->n_scalars;
    p->F = p->Fs + 2;
    p->Kp = round_up(p->Fs, 64);
    p->D = d->n_hidden;
    int hmax = 0;
    for (int k = 0; k < p->D; ++k) { p->H[k] = d->hidden[k]; if (p->H[k] > hmax) hmax = p->H[k]; }
    if ((int64_t)C * p->H[0] >= (1LL << 31)) return AB_ERR_UNSUPPORTED;
    int64_t cs = kTargetChunkRows / C;
    if (cs < 1) cs = 1;
    if (cs > S) cs = S > 0 ? S : 1;
    const int64_t cap = ((1LL << 31) - 1) / p->H[0];
    if (cs > cap) cs = cap;
    p->chunk_scen = cs;
    p->chunk_rows = cs * C;
    p->tile_a = pick_tile(S, p->H[0]);
    for (int k = 1; k < p->D; ++k) {
        p->tile[k] = pick_tile(p->chunk_rows, p->H[k]);
        p->big[k] = p->dtype == AB_BF16 && p->H[k] % 256 == 0 && (k > 1 || C % 256 == 0) &&
                    ((p->chunk_rows + 255) / 256) * (p->H[k] / 256) >= 64;   // (measured crossover against the generic tiles)
    }
    p->nt_last = 1;
    if (p->D >= 2) {
        const int kl = p->D - 1;
        p->nt_last = p->big[kl] ? p->H[kl] / 256 : p->H[kl] / tile_edge(p->tile[kl]);
    }
    const size_t es = elem_size(p->dtype);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    p->off_xs = take((size_t)(S > 0 ? S : 1) * p->Kp * es);
    p->off_w1s = take((size_t)p->H[0] * p->Kp * es);
    p->off_aterm = take((size_t)(S > 0 ? S : 1) * p->H[0] * 4);
    p->off_bterm = take((size_t)C * p->H[0] * 4);
    p->off_cfgv = take(((size_t)2 * p->H[0] + 2 * (size_t)C) * 4);
    p->off_wout = take((size_t)(p->H[p->D - 1] + 1) * 4);     // folded output weights, then the folded bias
    p->off_xrow = take((size_t)p->chunk_rows * 2 * 4);          // per-scenario grids: (phi(S_p), phi(S_c)) of a chunk's rows
    p->off_partial = take((size_t)p->chunk_rows * p->nt_last * 4);
    p->off_act0 = p->off_act1 = 0;
    if (p->D >= 3) p->off_act0 = take((size_t)p->chunk_rows * hmax * es);
    if (p->D >= 4) p->off_act1 = take((size_t)p->chunk_rows * hmax * es);
    p->v_chunk = S < kVChunk ? (S > 0 ? S : 1) : kVChunk;
    for (int k = 1; k < p->D; ++k) p->v_tile[k] = pick_tile(p->v_chunk, p->H[k]);
    p->off_vx = take((size_t)p->v_chunk * 2 * 4);
    p->off_vact0 = p->off_vact1 = p->off_vlast = 0;
    if (p->D >= 2) p->off_vlast = take((size_t)p->v_chunk * p->H[p->D - 1] * 4);
    if (p->D >= 3) p->off_vact0 = take((size_t)p->v_chunk * hmax * es);
    if (p->D >= 4) p->off_vact1 = take((size_t)p->v_chunk * hmax * es);
    p->total = off;
    return AB_OK;
}

#define AB_HIP(expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) return AB_ERR_DEVICE; } while (0)

static inline bool misaligned(const void *p, size_t a) { return ((uintptr_t)p % a) != 0; }

// defined in update.hip
size_t update_workspace_bytes(const ab_model_desc *d, int64_t B);
hipError_t launch_replay_mix(const float *x_new, const float *t_new, int64_t n_new, const float *x_old,
                             const float *t_old, int64_t n_old, const int32_t *pick, int64_t B, int32_t F,
                             int32_t n_out, float *x_out, float *t_out, hipStream_t st);
ab_status online_update(const ab_model_desc *d, ab_params *params, const float *x_raw, const float *target,
                        int64_t B, float lr, float beta1, float beta2, float eps, float *loss_out,
                        void *workspace, size_t ws_bytes, int first_trainable, hipStream_t st);

}  // namespace ab

using namespace ab;

extern "C" {

int32_t ab_version(void) { return 109; }

void ab_set_trace(ab_trace_fn fn, void *user) { g_trace_fn = fn; g_trace_user = user; }

const char *ab_status_string(ab_status s)
{
    switch (s) {
    case AB_OK: return "ok";
    case AB_ERR_NULL: return "a required pointer is NULL";
    case AB_ERR_SHAPE: return "a size is non-positive or inconsistent";
    case AB_ERR_DTYPE: return "unknown compute dtype";
    case AB_ERR_ALIGN: return "a pointer misses its required alignment";
    case AB_ERR_WORKSPACE: return "workspace missing or too small";
    case AB_ERR_UNSUPPORTED: return "description not supported by this library";
    case AB_ERR_DEVICE: return "HIP reported an error";
    default: return "unknown status";
    }
}

size_t ab_workspace_bytes(const ab_model_desc *desc, int64_t S, int32_t C, int64_t B)
{
    if (check_desc(desc) != AB_OK || S < 0 || C < 0 || B < 0) return 0;
    size_t need = 0;
    if (C > 0 && desc->n_hidden == 0) {
        need = 256;                        // the linear scorer runs in one launch and uses no workspace
    } else if (C > 0) {
        ScorePlan p;
        if (plan_scoring(desc, S, C, &p) != AB_OK) return 0;
        need = p.total;
    }
    if (B > 0) {
        const size_t u = update_workspace_bytes(desc, B);
        if (u == 0) return 0;
        if (u > need) need = u;
    }
    return need;
}

}  // extern "C"

// Scoring with the workspace given by address: the body of both scoring entry points.
static ab_status score_candidates_in(const ab_model_desc *desc, const ab_params *params,
                                     const ab_stats *stats, const ab_grid *grid,
                                     float *scores, int32_t *best_idx, float *best_score, float *v_best,
                                     void *workspace, size_t workspace_bytes, void *stream)
{
    ab_status rc = check_desc(desc);
    if (rc != AB_OK) return rc;
    if (!params || !stats || !grid) return AB_ERR_NULL;
    if (stats->S == 0) return AB_OK;      // nothing to score: valid no-op, no pointer is looked at
    if (!scores && !best_idx) return AB_ERR_NULL;
    if (best_score && !best_idx) return AB_ERR_NULL;
    if (v_best && !best_idx) return AB_ERR_NULL;
    if (stats->S < 0 || grid->P <= 0 || grid->Q <= 0) return AB_ERR_SHAPE;
    if ((int64_t)grid->P * grid->Q > (1 << 24)) return AB_ERR_SHAPE;
    if (!grid->partition_bytes || !grid->credit_mult) return AB_ERR_NULL;
    if (grid->per_scenario != 0 && grid->per_scenario != 1) return AB_ERR_SHAPE;
    if (misaligned(grid->partition_bytes, 4) || misaligned(grid->credit_mult, 4)) return AB_ERR_ALIGN;
    const int64_t S = stats->S;
    const int32_t C = grid->P * grid->Q;
    if (S > 0 && (!stats->dyn || (desc->n_scalars > 0 && !stats->scalars))) return AB_ERR_NULL;
    if (stats->layers_of && !desc->tensor_encoder) return AB_ERR_UNSUPPORTED;   // the flat layout has one width
    if (misaligned(stats->layers_of, 4)) return AB_ERR_ALIGN;
    if (desc->n_hidden == 0) {
        // no hidden layer: V = W x + b, one launch, no workspace
        if (!params->W[0] || !params->b[0]) return AB_ERR_NULL;
        if (misaligned(params->W[0], 16) || misaligned(params->b[0], 4)) return AB_ERR_ALIGN;
        if (misaligned(stats->dyn, 4) || misaligned(stats->scalars, 4) || misaligned(scores, 4) ||
            misaligned(best_idx, 4) || misaligned(best_score, 4) || misaligned(v_best, 4)) return AB_ERR_ALIGN;
        hipStream_t st0 = (hipStream_t)stream;
        const double Fs0 = (double)desc->n_layers * desc->n_stats + desc->n_scalars;
        TraceScope ts("score_linear", (double)S * (Fs0 * 4.0 + (scores ? C * 4.0 : 0.0) + 8.0), 1, st0);
        AB_HIP(launch_score_linear(desc->compute_dtype, desc, params, stats->dyn, stats->scalars, grid, S, scores,
                                   best_idx, best_score, v_best, st0));
        return AB_OK;
    }
    ScorePlan p;
    rc = plan_scoring(desc, S, C, &p);
    if (rc != AB_OK) return rc;
    const int n_layers_total = p.base + p.D + 1;
    for (int k = 0; k < n_layers_total; ++k) {
        if (!params->W[k] || !params->b[k]) return AB_ERR_NULL;
        if (misaligned(params->W[k], 16) || misaligned(params->b[k], 4)) return AB_ERR_ALIGN;
    }
    if (misaligned(stats->dyn, 4) || misaligned(stats->scalars, 4) || misaligned(scores, 4) ||
        misaligned(best_idx, 4) || misaligned(best_score, 4) || misaligned(v_best, 4)) return AB_ERR_ALIGN;
    if (!workspace || workspace_bytes < p.total) return AB_ERR_WORKSPACE;
    if (misaligned(workspace, 256)) return AB_ERR_ALIGN;
    if (S == 0) return AB_OK;

    hipStream_t st = (hipStream_t)stream;
    if (!v_best && score_tiny_supported(desc, S, C)) {
        // the paper's own operating point (a job, tens of candidates, a small scorer): one launch does everything
        double fl = (double)p.H[0] * p.Fs * 2.0 * S;
        for (int k = 0; k < p.D; ++k) fl += 2.0 * S * C * p.H[k] * (k ? p.H[k - 1] : 3);
        TraceScope ts("score_tiny", fl, 0, st);
        AB_HIP(launch_score_tiny(p.dtype, desc, params, stats->dyn, stats->scalars, grid->partition_bytes,
                                 grid->credit_mult, grid->P, grid->Q, grid->per_scenario, S, scores, best_idx,
                                 best_score, st));
        return AB_OK;
    }
    unsigned char *ws = (unsigned char *)workspace;
    void *xs = ws + p.off_xs, *w1s = ws + p.off_w1s;
    float *a_term = (float *)(ws + p.off_aterm), *b_term = (float *)(ws + p.off_bterm);
    float *w_out_f = (float *)(ws + p.off_wout), *partial = (float *)(ws + p.off_partial);
    float *cfg_vec = (float *)(ws + p.off_cfgv);
    float *xp_row = (float *)(ws + p.off_xrow), *xc_row = xp_row + p.chunk_rows;
    const int per_scenario = grid->per_scenario;
    void *act[2] = {ws + p.off_act0, ws + p.off_act1};
    const int dt = p.dtype;

    // 1. scenario rows: transformed statistics (or pooled tensor embedding) + scalars, K-padded
    const double es = (double)elem_size(dt);
    bool prep_done = false;
    if (desc->tensor_encoder == 2) {
        {
            // per scenario and layer: two gate products (256 x 96 and 256 x 128) and the K -> 32 embedding
            TraceScope ts("lstm_encoder", (double)S * desc->n_layers * 2.0 * (256.0 * 224.0 + 32.0 * desc->n_stats), 0, st);
            AB_HIP(launch_lstm_encoder(desc, stats->dyn, params->W[0], params->b[0], params->W[1], params->b[1],
                                       params->W[2], params->b[2], xs, p.Kp, S, stats->layers_of, st));
        }
        TraceScope ts("encode_stats", (double)S * (desc->n_scalars * 4.0 + (p.Kp - desc->enc_hidden[1]) * es), 1, st);
        AB_HIP(launch_encode_stats(dt, desc, stats->dyn, stats->scalars, xs, S, p.Kp,
                                   desc->enc_hidden[1], 0, st));
    } else if (desc->tensor_encoder) {
        {
            TraceScope ts("tensor_encoder", (double)S * desc->n_layers * 2.0 * (desc->n_stats * 128.0 + 128.0 * 128.0),
                          0, st);
            AB_HIP(launch_tensor_encoder(dt, desc, stats->dyn, params->W[0], params->b[0], params->W[1],
                                         params->b[1], xs, p.Kp, S, stats->layers_of, st));
        }
        TraceScope ts("encode_stats", (double)S * (desc->n_scalars * 4.0 + (p.Kp - desc->enc_hidden[1]) * es), 1, st);
        AB_HIP(launch_encode_stats(dt, desc, stats->dyn, stats->scalars, xs, S, p.Kp,
                                   desc->enc_hidden[1], 0, st));
    } else {
        // flat statistics: transform and layer-1 preparation (step 2) share one launch where the layout allows
        const double prep_bytes = (double)p.H[0] * (p.F * es + p.Kp * es) + (double)C * p.H[0] * 4.0;
        TraceScope ts("encode_and_prep", (double)S * (p.Fs * 4.0 + p.Kp * es) + prep_bytes, 1, st);
        AB_HIP(launch_encode_and_prep(dt, desc, stats->dyn, stats->scalars, xs, S, p.Kp, params->W[p.base],
                                      params->b[p.base], p.F, p.Fs, p.H[0], w1s, grid, b_term, cfg_vec,
                                      params->W[p.base + p.D], params->b[p.base + p.D], p.H[p.D - 1], w_out_f,
                                      &prep_done, st));
        if (!prep_done) AB_HIP(launch_encode_stats(dt, desc, stats->dyn, stats->scalars, xs, S, p.Kp, 0, 1, st));
    }
    // 2. layer-1 split: packed statistics columns of W1, candidate term B[c], fp32 output weights
    if (!prep_done) {
        TraceScope ts("prep_layer1", (double)p.H[0] * (p.F * es + p.Kp * es) + (double)C * p.H[0] * 4.0, 1, st);
        AB_HIP(launch_prep_layer1(dt, desc, params->W[p.base], params->b[p.base], p.F, p.Fs, p.H[0], p.Kp, w1s,
                                  grid, b_term, cfg_vec, params->W[p.base + p.D], params->b[p.base + p.D],
                                  p.H[p.D - 1], w_out_f, st));
    }
    // 3. scenario term A[s] = x_s W1_s^T + b1 (fp32 out)
    {
        GemmArgs g;
        memset(&g, 0, sizeof(g));
        g.A = xs; g.lda = p.Kp; g.B = w1s; g.ldb = p.Kp;
        g.M = S; g.N = p.H[0]; g.K = p.Kp;
        g.out = a_term; g.ldo = p.H[0]; g.out_f32 = 1;
        g.bias = params->b[p.base];
        TraceScope ts("gemm_scenario_term", 2.0 * S * p.H[0] * p.Kp, 0, st);
        AB_HIP(launch_gemm(dt, p.tile_a, AMODE_LOAD, EPI_STORE, g, st));
    }
    // 4. candidate rows, a chunk of scenarios at a time
    for (int64_t s0 = 0; s0 < S; s0 += p.chunk_scen) {
        const int64_t ns = (S - s0 < p.chunk_scen) ? S - s0 : p.chunk_scen;
        const int64_t rows = ns * C;
        const float *a_chunk = a_term + s0 * p.H[0];
        int nt = 1;
        if (per_scenario) {
            TraceScope ts("grid_rows", (double)rows * 8.0, 1, st);
            AB_HIP(launch_grid_rows(desc, grid->partition_bytes + s0 * grid->P, grid->credit_mult + s0 * grid->Q,
                                    grid->P, grid->Q, xp_row, xc_row, rows, st));
        }
        if (p.D == 1) {
            TraceScope ts("score_single_hidden", 3.0 * rows * p.H[0], 0, st);
            AB_HIP(launch_score_single_hidden(a_chunk, b_term, w_out_f, partial, rows, C, p.H[0], cfg_vec,
                                              cfg_vec + p.H[0], per_scenario ? xp_row : nullptr,
                                              per_scenario ? xc_row : nullptr, st));
        } else {
            for (int k = 1; k < p.D; ++k) {
                GemmArgs g;
                memset(&g, 0, sizeof(g));
                if (k == 1) {
                    g.a_term = a_chunk; g.b_term = b_term; g.ldt = p.H[0]; g.C = C;
                    g.wp = cfg_vec; g.wc = cfg_vec + p.H[0]; g.xp = cfg_vec + 2 * p.H[0]; g.xc = cfg_vec + 2 * p.H[0] + C;
                    if (per_scenario) { g.xp = xp_row; g.xc = xc_row; g.x_per_row = 1; }
                    g.xp_runs4 = grid->Q % 4 == 0;          // (row = s C + p Q + q and 4 | Q: four adjacent rows, one p)
                }
                else { g.A = act[k & 1]; g.lda = p.H[k - 1]; }
                g.B = params->W[p.base + k]; g.ldb = p.H[k - 1];
                g.M = rows; g.N = p.H[k]; g.K = p.H[k - 1];
                g.bias = params->b[p.base + k]; g.relu = 1;
                const bool last = (k == p.D - 1);
                if (last) { g.w_out = w_out_f; g.partial = partial; nt = p.nt_last; }
                else { g.out = act[(k + 1) & 1]; g.ldo = p.H[k]; }
                TraceScope ts(k == 1 ? (last ? "gemm_hidden_first_last" : "gemm_hidden_first")
                                     : (last ? "gemm_hidden_last" : "gemm_hidden_mid"),
                              2.0 * rows * p.H[k] * p.H[k - 1], 0, st);
                const int amode = k == 1 ? AMODE_GEN : AMODE_LOAD, epi = last ? EPI_SCORE : EPI_STORE;
                if (p.big[k] && gemm_big_supported(dt, amode, epi, g))
                    AB_HIP(launch_gemm_big(amode, epi, g, st));
                else if (p.big[k])
                    return AB_ERR_UNSUPPORTED;     // cannot happen: the plan checked the same conditions
                else    // the generic tiles take a per-scenario grid's operand in its factored form
                    AB_HIP(launch_gemm(dt, p.tile[k], amode == AMODE_GEN && per_scenario ? AMODE_GENV : amode, epi, g, st));
            }
        }
        TraceScope ts("finish_select", (double)rows * (nt * 4.0 + (scores ? 4.0 : 0.0)) + ns * 8.0, 1, st);
        AB_HIP(launch_finish_select(partial, nt, C, w_out_f + p.H[p.D - 1],
                                    scores ? scores + s0 * C : nullptr, C,
                                    best_idx ? best_idx + s0 : nullptr,
                                    best_score ? best_score + s0 : nullptr, ns, C, st));
    }
    // 5. the chosen candidate's prediction vector: the hidden chain once more on one row per scenario (the row's
    // candidate values are those of best_idx), then the output layer unit by unit
    if (v_best) {
        const int n_out = desc->n_outputs > 0 ? desc->n_outputs : 1;
        float *xp_sel = (float *)(ws + p.off_vx), *xc_sel = xp_sel + p.v_chunk;
        float *h_last = (float *)(ws + p.off_vlast);
        void *vact[2] = {ws + p.off_vact0, ws + p.off_vact1};
        for (int64_t s0 = 0; s0 < S; s0 += p.v_chunk) {
            const int64_t ns = (S - s0 < p.v_chunk) ? S - s0 : p.v_chunk;
            ab_grid gsub = *grid;
            if (per_scenario) { gsub.partition_bytes += s0 * grid->P; gsub.credit_mult += s0 * grid->Q; }
            {
                TraceScope ts("chosen_pair", (double)ns * 20.0, 1, st);
                AB_HIP(launch_chosen_pair(desc, &gsub, best_idx + s0, xp_sel, xc_sel, ns, st));
            }
            for (int k = 1; k < p.D; ++k) {
                GemmArgs g;
                memset(&g, 0, sizeof(g));
                if (k == 1) {
                    g.a_term = a_term + s0 * p.H[0]; g.ldt = p.H[0]; g.C = 1;
                    g.wp = cfg_vec; g.wc = cfg_vec + p.H[0]; g.xp = xp_sel; g.xc = xc_sel; g.x_per_row = 1;
                } else { g.A = vact[k & 1]; g.lda = p.H[k - 1]; }
                g.B = params->W[p.base + k]; g.ldb = p.H[k - 1];
                g.M = ns; g.N = p.H[k]; g.K = p.H[k - 1];
                g.bias = params->b[p.base + k]; g.relu = 1;
                if (k == p.D - 1) { g.out = h_last; g.ldo = p.H[k]; g.out_f32 = 1; }
                else { g.out = vact[(k + 1) & 1]; g.ldo = p.H[k]; }
                TraceScope ts("gemm_chosen_rows", 2.0 * ns * p.H[k] * p.H[k - 1], 0, st);
                AB_HIP(launch_gemm(dt, p.v_tile[k], k == 1 ? AMODE_GENV : AMODE_LOAD, EPI_STORE, g, st));
            }
            TraceScope ts("output_v", (double)ns * (p.H[p.D - 1] * 4.0 + n_out * 4.0), 1, st);
            AB_HIP(launch_output_v(dt, p.D >= 2 ? h_last : nullptr, a_term + s0 * p.H[0], cfg_vec, cfg_vec + p.H[0],
                                   xp_sel, xc_sel, params->W[p.base + p.D], params->b[p.base + p.D], p.H[p.D - 1],
                                   n_out, best_idx + s0, v_best + s0 * n_out, ns, st));
        }
    }
    return AB_OK;
}

// Workspace of ab_score_candidates_static: lives in the code object, one copy per device.  The name is a
// host-side stand-in only; the device address is looked up once per device and kept in g_scratch_ptr.
static __device__ __align__(256) unsigned char scratch[AB_STATIC_SCRATCH_BYTES];
static const int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mutex;

static ab_status static_scratch(void **out)
{
    int dev = -1;
    AB_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return AB_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        AB_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return AB_ERR_DEVICE;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return AB_OK;
}

extern "C" {

ab_status ab_score_candidates(const ab_model_desc *desc, const ab_params *params,
                              const ab_stats *stats, const ab_grid *grid,
                              float *scores, int32_t *best_idx, float *best_score,
                              void *workspace, size_t workspace_bytes, void *stream)
{
    return score_candidates_in(desc, params, stats, grid, scores, best_idx, best_score, nullptr,
                               workspace, workspace_bytes, stream);
}

ab_status ab_score_candidates_v(const ab_model_desc *desc, const ab_params *params,
                                const ab_stats *stats, const ab_grid *grid,
                                float *scores, int32_t *best_idx, float *best_score, float *v_best,
                                void *workspace, size_t workspace_bytes, void *stream)
{
    return score_candidates_in(desc, params, stats, grid, scores, best_idx, best_score, v_best,
                               workspace, workspace_bytes, stream);
}

size_t ab_static_scratch_bytes(void) { return AB_STATIC_SCRATCH_BYTES; }

ab_status ab_score_candidates_static(const ab_model_desc *desc, const ab_params *params,
                                     const ab_stats *stats, const ab_grid *grid,
                                     float *scores, int32_t *best_idx, float *best_score, void *stream)
{
    ab_status rc = check_desc(desc);
    if (rc != AB_OK) return rc;
    if (!params || !stats || !grid) return AB_ERR_NULL;
    if (desc->n_hidden > 0 && stats->S > 0 && grid->P > 0 && grid->Q > 0 && (int64_t)grid->P * grid->Q <= (1 << 24)) {
        // refuse what does not fit before anything else is looked at
        ScorePlan p;
        rc = plan_scoring(desc, stats->S, grid->P * grid->Q, &p);
        if (rc != AB_OK) return rc;
        if (p.total > AB_STATIC_SCRATCH_BYTES) return AB_ERR_WORKSPACE;
    }
    void *ptr = nullptr;
    rc = static_scratch(&ptr);
    if (rc != AB_OK) return rc;
    return score_candidates_in(desc, params, stats, grid, scores, best_idx, best_score, nullptr,
                               ptr, AB_STATIC_SCRATCH_BYTES, stream);
}

ab_status ab_select_best(const float *scores, int64_t S, int32_t C, int64_t row_stride,
                         int32_t *best_idx, float *best_score, void *stream)
{
    if (!scores || !best_idx) return AB_ERR_NULL;
    if (S < 0 || C <= 0 || row_stride < C) return AB_ERR_SHAPE;
    if (misaligned(scores, 4) || misaligned(best_idx, 4) || misaligned(best_score, 4)) return AB_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    for (int64_t s0 = 0; s0 < S; s0 += (1 << 30)) {
        const int64_t ns = (S - s0 < (1 << 30)) ? S - s0 : (1 << 30);
        TraceScope ts("select_best", (double)ns * (C * 4.0 + 8.0), 1, st);
        AB_HIP(launch_finish_select(scores + s0 * row_stride, 1, row_stride, nullptr, nullptr, 0,
                                    best_idx + s0, best_score ? best_score + s0 : nullptr, ns, C, st));
    }
    return AB_OK;
}

ab_status ab_trigger(const float *scores, int64_t S, int32_t C, int64_t row_stride,
                     const int32_t *current_idx, const float *observed,
                     float gain_threshold, float error_threshold,
                     int32_t *best_idx, float *gain, uint8_t *reconfigure, uint8_t *adapt, void *stream)
{
    if (!scores || !current_idx || !best_idx || !reconfigure) return AB_ERR_NULL;
    if (adapt && !observed) return AB_ERR_NULL;
    if (S < 0 || C <= 0 || row_stride < C) return AB_ERR_SHAPE;
    if (misaligned(scores, 4) || misaligned(current_idx, 4) || misaligned(observed, 4) ||
        misaligned(best_idx, 4) || misaligned(gain, 4)) return AB_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    for (int64_t s0 = 0; s0 < S; s0 += (1 << 30)) {
        const int64_t ns = (S - s0 < (1 << 30)) ? S - s0 : (1 << 30);
        TraceScope ts("trigger", (double)ns * (C * 4.0 + 16.0), 1, st);
        AB_HIP(launch_trigger(scores + s0 * row_stride, ns, C, row_stride, current_idx + s0,
                              observed ? observed + s0 : nullptr, gain_threshold, error_threshold,
                              best_idx + s0, gain ? gain + s0 : nullptr, reconfigure + s0,
                              adapt ? adapt + s0 : nullptr, st));
    }
    return AB_OK;
}

ab_status ab_online_update(const ab_model_desc *desc, ab_params *params,
                           const float *x_raw, const float *target, int64_t B,
                           float lr, float beta1, float beta2, float eps,
                           float *loss_out, void *workspace, size_t workspace_bytes, void *stream)
{
    ab_status rc = check_desc(desc);
    if (rc != AB_OK) return rc;
    if (desc->tensor_encoder) return AB_ERR_UNSUPPORTED;
    if (!params || !x_raw || !target) return AB_ERR_NULL;
    if (B <= 0) return AB_ERR_SHAPE;
    return online_update(desc, params, x_raw, target, B, lr, beta1, beta2, eps, loss_out,
                         workspace, workspace_bytes, 0, (hipStream_t)stream);
}

ab_status ab_online_update_tail(const ab_model_desc *desc, ab_params *params,
                                const float *x_raw, const float *target, int64_t B, int32_t first_trainable,
                                float lr, float beta1, float beta2, float eps,
                                float *loss_out, void *workspace, size_t workspace_bytes, void *stream)
{
    ab_status rc = check_desc(desc);
    if (rc != AB_OK) return rc;
    if (desc->tensor_encoder) return AB_ERR_UNSUPPORTED;
    if (!params || !x_raw || !target) return AB_ERR_NULL;
    if (B <= 0 || first_trainable < 0 || first_trainable > desc->n_hidden) return AB_ERR_SHAPE;
    return online_update(desc, params, x_raw, target, B, lr, beta1, beta2, eps, loss_out,
                         workspace, workspace_bytes, first_trainable, (hipStream_t)stream);
}

ab_status ab_replay_mix(const float *x_new, const float *target_new, int64_t n_new,
                        const float *x_old, const float *target_old, int64_t n_old,
                        const int32_t *pick, int64_t B, int32_t F, int32_t n_outputs,
                        float *x_out, float *target_out, void *stream)
{
    if (n_new < 0 || n_old < 0 || B < 0 || F <= 0 || n_outputs < 1 || n_outputs > AB_MAX_OUTPUTS) return AB_ERR_SHAPE;
    if (B == 0) return AB_OK;
    if (!pick || !x_out || !target_out) return AB_ERR_NULL;
    if ((n_new > 0 && (!x_new || !target_new)) || (n_old > 0 && (!x_old || !target_old))) return AB_ERR_NULL;
    if (n_new > 0x7fffffffLL || n_old > 0x7fffffffLL || (B + 3) / 4 > 0x7fffffffLL) return AB_ERR_UNSUPPORTED;
    if (misaligned(x_new, 4) || misaligned(x_old, 4) || misaligned(x_out, 4) || misaligned(pick, 4) ||
        misaligned(target_new, 4) || misaligned(target_old, 4) || misaligned(target_out, 4)) return AB_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    TraceScope ts("replay_mix", (double)B * (F + n_outputs) * 8.0 + (double)B * 4.0, 1, st);
    AB_HIP(launch_replay_mix(x_new, target_new, n_new, x_old, target_old, n_old, pick, B, F, n_outputs, x_out,
                             target_out, st));
    return AB_OK;
}

}  // extern "C"
