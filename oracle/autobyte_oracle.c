/*
 * AutoByte meta-network: plain fp64 CPU oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement of what the
 * meta-network pass computes.  It is used by the test-suite, by the smoke check and by the
 * benchmark's CPU-baseline leg; the GPU product never calls it and shares no code with it.
 *
 * What it follows (arXiv 2112.13509):
 *   - Table 1 / Section 3.1 "Input runtime metrics": the input record (layer-wise computation
 *     time and other per-layer statistics, bandwidth, worker count, model / architecture type,
 *     and the candidate pair <S_p, S_c>).
 *   - Section 3.1 "Meta network architecture": the four feature groups are concatenated and
 *     dense layers map the concatenation to the predicted training speed V (Eq. 1).
 *   - Section 3 (intro) and Eq. 1: the pair with the maximum predicted V is chosen.
 *   - Eq. 2: L2 loss between predicted and observed speed, used for (online) training.
 *
 * Every function takes the steps in that order with no factorisation, blocking or fusion:
 * for each scenario and each candidate the full input vector is materialised and pushed
 * through every layer.  Floating point is fp64 throughout.  OpenMP, where present, only
 * distributes independent scenarios (rows) over threads.
 *
 * Pins: see tests/test_oracle_*.py (brute force on tiny grids, library matmul chain,
 * one-layer closed form, permutation invariance, finite differences, autograd, reference Adam;
 * for the per-worker output, the norm loss and per-scenario grids: library chain and linearity of
 * the mean, finite differences, autograd, the absolute-error closed form, scenario-by-scenario calls;
 * integer-valued networks against int64 arithmetic; the diagnostic rounding against the bfloat16 format).
 * Nothing here is pinned against numbers printed in the paper, because the paper prints no
 * numeric example of the meta-network.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_OK 0
#define ORC_ERR_ARG (-1)
#define ORC_ERR_MEM (-2)

/* ---- feature transform: phi(x) = (g(x) - shift) * scale, g = identity (kind 0) or ln (kind 1).
 * The paper only says the metrics are turned into vector inputs (Section 3.3, "Meta network
 * optimizer"); the per-feature affine / log-affine normalisation is this implementation's reading. */
static double orc_phi(double x, int kind, double shift, double scale)
{
    double g = (kind == 1) ? log(x) : x;
    return (g - shift) * scale;
}

/* Diagnostic only: nearest bfloat16 (ties to even) of a value, via its nearest float.  Used when a
 * test wants the oracle to round stored activations where a bf16 implementation stores them, so
 * that implementation bugs can be told apart from rounding noise.  Off by default. */
static double orc_round_bf16(double v)
{
    float f = (float)v;
    uint32_t u;
    if (f != f) return v;
    memcpy(&u, &f, 4);
    u = (u + 0x7FFFu + ((u >> 16) & 1u)) & 0xFFFF0000u;
    memcpy(&f, &u, 4);
    return (double)f;
}

double orc_encode_value(double x, int kind, double shift, double scale)
{
    return orc_phi(x, kind, shift, scale);
}

/* The diagnostic rounding alone, so that a test can hold it against a library conversion. */
double orc_round_bf16_value(double v) { return orc_round_bf16(v); }

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* y = W x + b, W is [n_out, n_in] row-major; optional ReLU. */
static void orc_dense(const double *W, const double *b, int n_out, int n_in,
                      const double *x, double *y, int relu)
{
    for (int o = 0; o < n_out; ++o) {
        double acc = b ? b[o] : 0.0;
        const double *w = W + (size_t)o * (size_t)n_in;
        for (int i = 0; i < n_in; ++i)
            acc += w[i] * x[i];
        if (relu && !(acc > 0.0))
            acc = (acc != acc) ? acc : 0.0; /* NaN stays NaN so bad inputs remain visible */
        y[o] = acc;
    }
}

/*
 * Description of one model, flattened to plain arrays.
 *
 *  L, K, Ns          : layers (tensors) per scenario, statistics per layer, scalar features
 *  stat_* [K]        : transform of each per-layer statistic
 *  scal_* [Ns]       : transform of each scalar feature
 *  cfg_*  [2]        : transform of partition size (0) and credit multiple (1)
 *  tensor_encoder    : 0 -> the L*K statistics are laid side by side (layer-major, stat-minor);
 *                      1 -> a shared two-layer MLP (K -> te_h0 -> te_h1, ReLU after both) is
 *                           applied to each layer's K statistics and the results are averaged
 *                           over the L layers (Section 3.1 "Meta network architecture": the per-layer
 *                           times are first mapped to a feature space of fixed width)
 *                      2 -> each layer's K statistics are embedded linearly into te_h0 values and a
 *                           two-layer LSTM of te_h1 units per layer runs over the L layers in order;
 *                           the second layer's last hidden state is the statistics block
 *                           (Section 3.1 "Meta network architecture": after the embedding a two-layer LSTM
 *                           reads the layer sequence)
 *  te_W[2], te_b[2]  : tensor-encoder weights ([te_h0,K], [te_h1,te_h0]) and biases; for the LSTM
 *                      te_W[3] = {[te_h0,K], [4*te_h1, te_h0+te_h1], [4*te_h1, 2*te_h1]} and te_b[3]
 *                      = {[te_h0], [4*te_h1], [4*te_h1]}: the recurrent matrices act on
 *                      [input ; previous hidden state], gate blocks in the order input, forget,
 *                      candidate, output
 *  n_hidden, hidden[]: widths of the scorer's hidden layers (ReLU after each)
 *  W[n_hidden+1], b[]: scorer weights, W[k] is [out,in] row-major; the last one has out = n_out and
 *                      is linear (V is a regression target)
 *  n_out             : width of V (Table 1 gives V one entry per worker); 0 or 1 -> a single value.
 *                      The speed a configuration is ranked by is the mean of the n_out predictions
 *                      (Eq. 1 ranks configurations by V without saying how a vector is ordered: in
 *                      synchronous data-parallel training the job advances at one rate, of which the
 *                      per-worker entries are n_out measurements -- this implementation's reading)
 *  loss_kind         : 0 -> mean over the minibatch of the squared error summed over the n_out entries;
 *                      1 -> mean over the minibatch of the Euclidean norm of the error vector (Eq. 2 as
 *                           printed: an unsquared L2 norm)
 *
 * Input vector order: [statistics block | scalars | phi(partition) | phi(credit)].
 */
typedef struct {
    int L, K, Ns;
    const int *stat_kind; const double *stat_shift; const double *stat_scale;
    const int *scal_kind; const double *scal_shift; const double *scal_scale;
    const int *cfg_kind;  const double *cfg_shift;  const double *cfg_scale;
    int tensor_encoder, te_h0, te_h1;
    const double *const *te_W; const double *const *te_b;
    int n_hidden; const int *hidden;
    const double *const *W; const double *const *b;
    int round_stored_bf16;   /* diagnostic, default 0: round to bf16 the values a bf16 pipeline keeps in
                                memory (scoring: statistics block + scalars, tensor-encoder hidden layer, every
                                hidden activation except the last; update: the transformed row, every hidden
                                activation and every hidden layer's delta) */
    int n_out, loss_kind;
} orc_model;

static int orc_n_out(const orc_model *m) { return m->n_out > 1 ? m->n_out : 1; }

static int orc_stats_width(const orc_model *m)
{
    return (m->tensor_encoder ? m->te_h1 : m->L * m->K) + m->Ns;
}

int orc_input_width(const orc_model *m) { return orc_stats_width(m) + 2; }

static double orc_sigmoid(double x) { return 1.0 / (1.0 + exp(-x)); }

/*
 * One LSTM cell step (Hochreiter & Schmidhuber's cell with forget gate, the form every library uses):
 *   z = W [x ; h] + b,  i = s(z[0:H]), f = s(z[H:2H]), g = tanh(z[2H:3H]), o = s(z[3H:4H]),
 *   c <- f*c + i*g,  h <- o*tanh(c).
 * xh holds [x (nx values) ; h (H values)], z is scratch of 4H values.
 */
static void orc_lstm_step(const double *W, const double *b, int nx, int H, const double *xh,
                          double *c, double *h_out, double *z)
{
    orc_dense(W, b, 4 * H, nx + H, xh, z, 0);
    for (int u = 0; u < H; ++u) {
        const double i = orc_sigmoid(z[u]), f = orc_sigmoid(z[H + u]);
        const double g = tanh(z[2 * H + u]), o = orc_sigmoid(z[3 * H + u]);
        c[u] = f * c[u] + i * g;
        h_out[u] = o * tanh(c[u]);
    }
}

/*
 * The temporal encoder of Section 3.1: linear embedding of each layer's statistics, two stacked LSTM
 * layers over the L layers (zero initial state), last hidden state of the second layer -> out[te_h1].
 * tmp holds K + te_h0 + 11*te_h1 doubles.
 */
static void orc_lstm_encode_one(const orc_model *m, const double *dyn_s, int Ls, double *out, double *tmp)
{
    const int E = m->te_h0, H = m->te_h1;
    double *in = tmp, *xh1 = in + m->K, *xh2 = xh1 + E + H, *c1 = xh2 + 2 * H, *c2 = c1 + H, *z = c2 + H;
    double *h1 = xh1 + E, *h2 = xh2 + H;                 /* the recurrent halves of the two inputs */
    for (int u = 0; u < H; ++u) h1[u] = h2[u] = c1[u] = c2[u] = 0.0;
    for (int l = 0; l < Ls; ++l) {
        for (int k = 0; k < m->K; ++k)
            in[k] = orc_phi(dyn_s[l * m->K + k], m->stat_kind[k], m->stat_shift[k], m->stat_scale[k]);
        orc_dense(m->te_W[0], m->te_b[0], E, m->K, in, xh1, 0);
        if (m->round_stored_bf16) for (int j = 0; j < E; ++j) xh1[j] = orc_round_bf16(xh1[j]);
        orc_lstm_step(m->te_W[1], m->te_b[1], E, H, xh1, c1, h1, z);
        if (m->round_stored_bf16) for (int u = 0; u < H; ++u) h1[u] = orc_round_bf16(h1[u]);
        for (int u = 0; u < H; ++u) xh2[u] = h1[u];
        orc_lstm_step(m->te_W[2], m->te_b[2], H, H, xh2, c2, h2, z);
        if (m->round_stored_bf16) for (int u = 0; u < H; ++u) h2[u] = orc_round_bf16(h2[u]);
    }
    for (int u = 0; u < H; ++u) out[u] = h2[u];
}

/* Scratch doubles orc_scenario_features needs behind xs. */
static int orc_feature_scratch(const orc_model *m) { return m->K + m->te_h0 + 11 * m->te_h1 + 8; }

/*
 * Layers a scenario really has: jobs differ in their number of layers (Section 3.1 "Meta network
 * architecture" notes that the layer count varies from one training task to the next), the statistics
 * tensor is padded to L.  layers_of == NULL: all L; values are clamped to [1, L].
 */
static int orc_layers_of(const orc_model *m, const int32_t *layers_of, int64_t s)
{
    if (!layers_of) return m->L;
    int n = layers_of[s];
    return n < 1 ? 1 : (n > m->L ? m->L : n);
}

/* The LSTM encoder alone: out[S, te_h1] (lets tests hold it against a library LSTM). */
int orc_lstm_encode(const orc_model *m, const double *dyn, int64_t S, const int32_t *layers_of, double *out)
{
    if (!m || m->tensor_encoder != 2 || !out || S < 0) return ORC_ERR_ARG;
    double *tmp = (double *)malloc(sizeof(double) * (size_t)orc_feature_scratch(m));
    if (!tmp) return ORC_ERR_MEM;
    for (int64_t s = 0; s < S; ++s)
        orc_lstm_encode_one(m, dyn + (size_t)s * m->L * m->K, orc_layers_of(m, layers_of, s),
                            out + (size_t)s * m->te_h1, tmp);
    free(tmp);
    return ORC_OK;
}

/* Statistics block + scalars of one scenario -> xs[orc_stats_width]. tmp holds orc_feature_scratch doubles. */
static void orc_scenario_features(const orc_model *m, const double *dyn_s, const double *scal_s, int Ls,
                                  double *xs, double *tmp)
{   /* Ls = layers of this scenario (<= L; only the encoders can take fewer than L) */
    int off;
    if (!m->tensor_encoder) {
        for (int l = 0; l < m->L; ++l)
            for (int k = 0; k < m->K; ++k)
                xs[l * m->K + k] = orc_phi(dyn_s[l * m->K + k], m->stat_kind[k],
                                           m->stat_shift[k], m->stat_scale[k]);
        off = m->L * m->K;
    } else if (m->tensor_encoder == 2) {
        orc_lstm_encode_one(m, dyn_s, Ls, xs, tmp);
        off = m->te_h1;
    } else {
        double *in = tmp, *h0 = tmp + m->K, *h1 = h0 + m->te_h0;
        for (int j = 0; j < m->te_h1; ++j) xs[j] = 0.0;
        for (int l = 0; l < Ls; ++l) {
            for (int k = 0; k < m->K; ++k)
                in[k] = orc_phi(dyn_s[l * m->K + k], m->stat_kind[k],
                                m->stat_shift[k], m->stat_scale[k]);
            orc_dense(m->te_W[0], m->te_b[0], m->te_h0, m->K, in, h0, 1);
            if (m->round_stored_bf16) for (int j = 0; j < m->te_h0; ++j) h0[j] = orc_round_bf16(h0[j]);
            orc_dense(m->te_W[1], m->te_b[1], m->te_h1, m->te_h0, h0, h1, 1);
            for (int j = 0; j < m->te_h1; ++j) xs[j] += h1[j];
        }
        for (int j = 0; j < m->te_h1; ++j) xs[j] /= (double)Ls;
        off = m->te_h1;
    }
    for (int j = 0; j < m->Ns; ++j)
        xs[off + j] = orc_phi(scal_s[j], m->scal_kind[j], m->scal_shift[j], m->scal_scale[j]);
    if (m->round_stored_bf16) for (int j = 0; j < off + m->Ns; ++j) xs[j] = orc_round_bf16(xs[j]);
}

/* Scorer MLP on one full input vector x[F]; buf holds 2*maxwidth doubles.  Returns the score (mean of V);
 * v_out, if given, receives the n_out entries of V themselves. */
static double orc_mlp_forward_v(const orc_model *m, const double *x, int F, double *buf, int maxw, double *v_out)
{
    const double *cur = x;
    int n_in = F;
    double *a = buf, *bb = buf + maxw;
    for (int k = 0; k < m->n_hidden; ++k) {
        double *out = (k & 1) ? bb : a;
        orc_dense(m->W[k], m->b[k], m->hidden[k], n_in, cur, out, 1);
        if (m->round_stored_bf16 && k < m->n_hidden - 1)
            for (int j = 0; j < m->hidden[k]; ++j) out[j] = orc_round_bf16(out[j]);
        cur = out;
        n_in = m->hidden[k];
    }
    /* V has n_out entries; the configuration's score is their mean */
    double v_local[64], score = 0.0;
    double *v = v_out ? v_out : v_local;
    const int no = orc_n_out(m);
    orc_dense(m->W[m->n_hidden], m->b[m->n_hidden], no, n_in, cur, v, 0);
    for (int w = 0; w < no; ++w) score += v[w];
    return score / (double)no;
}

static double orc_mlp_forward(const orc_model *m, const double *x, int F, double *buf, int maxw)
{
    return orc_mlp_forward_v(m, x, F, buf, maxw, NULL);
}

/*
 * Score every candidate of every scenario (Eq. 1 evaluated on the whole <S_p,S_c> grid).
 *   dyn  [S, L, K]   raw per-layer statistics
 *   scal [S, Ns]     raw scalar features
 *   part [P], cred [Q]   raw partition sizes and credit multiples; candidate c = p*Q + q
 *   scores [S, P*Q]  predicted V
 */
/* grid_per_scenario != 0: part is [S, P] and cred is [S, Q], every scenario brings its own candidate values
 * (Table 1 lists S_p and S_c as inputs of the one job being tuned; a batch of jobs need not share a grid). */
int orc_score_grids(const orc_model *m, const double *dyn, const double *scal, int64_t S,
                    const int32_t *layers_of, const double *part, int P, const double *cred, int Q,
                    int grid_per_scenario, double *scores)
{
    if (!m || !scores || S < 0 || P <= 0 || Q <= 0 || orc_n_out(m) > 64) return ORC_ERR_ARG;
    if (layers_of && !m->tensor_encoder) return ORC_ERR_ARG;      /* the flat layout has one width */
    const int Fs = orc_stats_width(m), F = Fs + 2;
    int maxw = 1;
    for (int k = 0; k < m->n_hidden; ++k) if (m->hidden[k] > maxw) maxw = m->hidden[k];
    const int tmpw = orc_feature_scratch(m);
    int err = 0;
#pragma omp parallel
    {
        double *x = (double *)malloc(sizeof(double) * (size_t)(F + 2 * maxw + tmpw));
        if (!x) {
#pragma omp atomic write
            err = 1;
        } else {
            double *buf = x + F, *tmp = buf + 2 * maxw;
#pragma omp for schedule(dynamic, 1)
            for (int64_t s = 0; s < S; ++s) {
                orc_scenario_features(m, dyn + (size_t)s * m->L * m->K, scal + (size_t)s * m->Ns,
                                      orc_layers_of(m, layers_of, s), x, tmp);
                const double *part_s = grid_per_scenario ? part + (size_t)s * P : part;
                const double *cred_s = grid_per_scenario ? cred + (size_t)s * Q : cred;
                for (int p = 0; p < P; ++p)
                    for (int q = 0; q < Q; ++q) {
                        x[Fs]     = orc_phi(part_s[p], m->cfg_kind[0], m->cfg_shift[0], m->cfg_scale[0]);
                        x[Fs + 1] = orc_phi(cred_s[q], m->cfg_kind[1], m->cfg_shift[1], m->cfg_scale[1]);
                        scores[(size_t)s * P * Q + (size_t)p * Q + q] = orc_mlp_forward(m, x, F, buf, maxw);
                    }
            }
            free(x);
        }
    }
    return err ? ORC_ERR_MEM : ORC_OK;
}

/*
 * The predicted speed vector V itself (Table 1: one entry per worker; Eq. 1 returns V) for ONE candidate per
 * scenario: cand[s] = p*Q + q, e.g. the chosen one.  V is [S, n_out]; a scenario with cand[s] outside [0, P*Q)
 * (no valid choice) gets NaN.  Same steps as orc_score_grids, nothing folded: the output layer is applied unit
 * by unit.
 */
int orc_predict_v(const orc_model *m, const double *dyn, const double *scal, int64_t S,
                  const int32_t *layers_of, const double *part, int P, const double *cred, int Q,
                  int grid_per_scenario, const int32_t *cand, double *V)
{
    if (!m || !V || !cand || S < 0 || P <= 0 || Q <= 0 || orc_n_out(m) > 64) return ORC_ERR_ARG;
    if (layers_of && !m->tensor_encoder) return ORC_ERR_ARG;
    const int Fs = orc_stats_width(m), F = Fs + 2, no = orc_n_out(m);
    int maxw = 1;
    for (int k = 0; k < m->n_hidden; ++k) if (m->hidden[k] > maxw) maxw = m->hidden[k];
    const int tmpw = orc_feature_scratch(m);
    double *x = (double *)malloc(sizeof(double) * (size_t)(F + 2 * maxw + tmpw));
    if (!x) return ORC_ERR_MEM;
    double *buf = x + F, *tmp = buf + 2 * maxw;
    for (int64_t s = 0; s < S; ++s) {
        double *v = V + (size_t)s * no;
        if (cand[s] < 0 || cand[s] >= P * Q) {
            for (int w = 0; w < no; ++w) v[w] = NAN;
            continue;
        }
        const int p = cand[s] / Q, q = cand[s] % Q;
        orc_scenario_features(m, dyn + (size_t)s * m->L * m->K, scal + (size_t)s * m->Ns,
                              orc_layers_of(m, layers_of, s), x, tmp);
        const double *part_s = grid_per_scenario ? part + (size_t)s * P : part;
        const double *cred_s = grid_per_scenario ? cred + (size_t)s * Q : cred;
        x[Fs]     = orc_phi(part_s[p], m->cfg_kind[0], m->cfg_shift[0], m->cfg_scale[0]);
        x[Fs + 1] = orc_phi(cred_s[q], m->cfg_kind[1], m->cfg_shift[1], m->cfg_scale[1]);
        (void)orc_mlp_forward_v(m, x, F, buf, maxw, v);
    }
    free(x);
    return ORC_OK;
}

int orc_score_layers(const orc_model *m, const double *dyn, const double *scal, int64_t S,
                     const int32_t *layers_of, const double *part, int P, const double *cred, int Q, double *scores)
{
    return orc_score_grids(m, dyn, scal, S, layers_of, part, P, cred, Q, 0, scores);
}

int orc_score(const orc_model *m, const double *dyn, const double *scal, int64_t S,
              const double *part, int P, const double *cred, int Q, double *scores)
{
    return orc_score_layers(m, dyn, scal, S, NULL, part, P, cred, Q, scores);
}

/* The full input vectors themselves, [S, P*Q, F]: lets tests feed a library matmul chain. */
int orc_materialise_inputs(const orc_model *m, const double *dyn, const double *scal, int64_t S,
                           const double *part, int P, const double *cred, int Q, double *X)
{
    if (!m || !X || S < 0 || P <= 0 || Q <= 0) return ORC_ERR_ARG;
    const int Fs = orc_stats_width(m), F = Fs + 2;
    double *xs = (double *)malloc(sizeof(double) * (size_t)(Fs + orc_feature_scratch(m)));
    if (!xs) return ORC_ERR_MEM;
    for (int64_t s = 0; s < S; ++s) {
        orc_scenario_features(m, dyn + (size_t)s * m->L * m->K, scal + (size_t)s * m->Ns, m->L, xs, xs + Fs);
        for (int p = 0; p < P; ++p)
            for (int q = 0; q < Q; ++q) {
                double *x = X + ((size_t)s * P * Q + (size_t)p * Q + q) * (size_t)F;
                memcpy(x, xs, sizeof(double) * (size_t)Fs);
                x[Fs]     = orc_phi(part[p], m->cfg_kind[0], m->cfg_shift[0], m->cfg_scale[0]);
                x[Fs + 1] = orc_phi(cred[q], m->cfg_kind[1], m->cfg_shift[1], m->cfg_scale[1]);
            }
    }
    free(xs);
    return ORC_OK;
}

/*
 * Pick the candidate with the largest predicted V per scenario (Section 3, introduction: of all candidate
 * pairs the one whose predicted speed is highest is applied).  Sequential scan: the lowest index wins exact ties.
 * NaN never wins; a scenario whose scores are all NaN gets index -1 and a NaN best score.
 * second[s] is the runner-up value (-inf if C == 1 or no second non-NaN score).
 */
int orc_select(const double *scores, int64_t S, int C, int64_t row_stride,
               int32_t *best_idx, double *best_score, double *second)
{
    if (!scores || !best_idx || S < 0 || C <= 0 || row_stride < C) return ORC_ERR_ARG;
    for (int64_t s = 0; s < S; ++s) {
        const double *r = scores + (size_t)s * (size_t)row_stride;
        int bi = -1;
        double bv = -INFINITY, sv = -INFINITY;
        for (int c = 0; c < C; ++c) {
            double v = r[c];
            if (v != v) continue;
            if (bi < 0 || v > bv) { if (bi >= 0) sv = bv; bv = v; bi = c; }
            else if (v > sv) sv = v;
        }
        best_idx[s] = bi;
        if (best_score) best_score[s] = (bi < 0) ? NAN : bv;
        if (second) second[s] = sv;
    }
    return ORC_OK;
}

/*
 * Optimization Trigger (Section 3.3 "Optimization trigger") on a stored score matrix:
 *   best    = candidate with the largest predicted V (rules of orc_select)
 *   gain    = (V_best - V_cur) / |V_cur|, V_cur = score of the configuration the job runs now
 *   reconf  = 1 if gain >= gain_threshold (the paper skips the attempt when the gain is below 5 %)
 *   adapt   = 1 if |V_cur - V_obs| / |V_obs| > error_threshold (the paper starts online adaptation when
 *             prediction and observed speed differ by more than 10 %)
 * The two decisions are taken in single precision on single-precision scores, the precision in which
 * the scores are stored, so that an implementation can agree bit for bit.  A scenario without a valid
 * best candidate, or whose current index is outside [0, C), gets gain = NaN and reconf = 0; adapt is 0
 * when its ratio is NaN.
 */
int orc_trigger(const float *scores, int64_t S, int C, int64_t row_stride, const int32_t *cur_idx,
                const float *observed, float gain_threshold, float error_threshold,
                int32_t *best_idx, float *gain, uint8_t *reconf, uint8_t *adapt)
{
    if (!scores || !cur_idx || !best_idx || !reconf || S < 0 || C <= 0 || row_stride < C) return ORC_ERR_ARG;
    for (int64_t s = 0; s < S; ++s) {
        const float *r = scores + (size_t)s * (size_t)row_stride;
        int bi = -1;
        float bv = -INFINITY;
        for (int c = 0; c < C; ++c) {
            float v = r[c];
            if (v != v) continue;
            if (bi < 0 || v > bv) { bv = v; bi = c; }
        }
        best_idx[s] = bi;
        const int ci = cur_idx[s];
        const int cur_ok = ci >= 0 && ci < C;
        const float vc = cur_ok ? r[ci] : NAN;
        float g = NAN;
        if (bi >= 0 && cur_ok) g = (bv - vc) / fabsf(vc);
        if (gain) gain[s] = g;
        reconf[s] = (uint8_t)(g >= gain_threshold);          /* false for NaN */
        if (adapt) {
            float e = NAN;
            if (observed && cur_ok) e = fabsf(vc - observed[s]) / fabsf(observed[s]);
            adapt[s] = (uint8_t)(e > error_threshold);
        }
    }
    return ORC_OK;
}

/*
 * One online-adaptation step of the flat-feature scorer (Section 3.2 "Offline training online
 * adapting"; loss per Eq. 2 read as the mean squared error over the minibatch).
 *
 *   x_raw [B, F]   raw rows: L*K statistics, Ns scalars, partition size, credit multiple
 *   target [B, n_out]  observed speed (one value per row, or one per worker)
 *   Wf[k]          weights used by forward/backward (pass the master weights, or a rounded copy
 *                  of them to reproduce a reduced-precision forward); bf[k] biases
 *   Wm,bm          master parameters updated in place by Adam; mW,vW,mb,vb its moments
 *   t              1-based step number used for bias correction
 *   gW,gb          optional outputs: the gradients (may be NULL)
 *   do_adam        0 -> only loss and gradients
 *
 * Backward is exact back-propagation of the loss.  With e_i = yhat_i - y_i (a vector of n_out entries):
 *   loss_kind 0:  loss = (1/B) sum_i |e_i|^2 ,  d_out_i = 2 e_i / B
 *   loss_kind 1:  loss = (1/B) sum_i |e_i|   ,  d_out_i = e_i / (|e_i| B)   (zero where e_i = 0)
 * then dW = d^T h_prev ; db = sum_i d_i ; d_prev = (d W) * [pre > 0].
 * Adam follows Kingma & Ba, Algorithm 1, with bias correction and epsilon outside the root.
 *
 * Transfer-learning form (Section 3.2 "Offline training online adapting" updates the offline-trained model by
 * transfer learning; the workflow of Section 3.3 adapts the trained network online): layers below first_trainable keep their
 * parameters and moments; back-propagation stops at the first trainable layer.  first_trainable = 0 is
 * the full update, first_trainable = n_hidden updates the output layer alone.  Frozen layers report
 * zero gradients.
 */
int orc_update_tail(const orc_model *m, const double *x_raw, const double *target, int64_t B,
                    const double *const *Wf, const double *const *bf,
                    double *const *Wm, double *const *bm,
                    double *const *mW, double *const *vW, double *const *mb, double *const *vb,
                    int64_t t, double lr, double beta1, double beta2, double eps, int do_adam,
                    double *loss_out, double *const *gW, double *const *gb, double *yhat_out,
                    int first_trainable)
{
    if (!m || !x_raw || !target || B <= 0 || m->tensor_encoder) return ORC_ERR_ARG;
    if (first_trainable < 0 || first_trainable > m->n_hidden) return ORC_ERR_ARG;
    const int nl = m->n_hidden + 1;
    const int F = m->L * m->K + m->Ns + 2;
    int width[16];
    if (nl > 15) return ORC_ERR_ARG;
    width[0] = F;
    for (int k = 0; k < m->n_hidden; ++k) width[k + 1] = m->hidden[k];
    width[nl] = orc_n_out(m);

    /* activations h[k]: [B, width[k]] (h[0] = encoded input), deltas d[k]: [B, width[k]] */
    double **h = (double **)calloc((size_t)nl + 1, sizeof(double *));
    double **d = (double **)calloc((size_t)nl + 1, sizeof(double *));
    double **gWl = (double **)calloc((size_t)nl, sizeof(double *));
    double **gbl = (double **)calloc((size_t)nl, sizeof(double *));
    int fail = (!h || !d || !gWl || !gbl);
    for (int k = 0; !fail && k <= nl; ++k) {
        h[k] = (double *)malloc(sizeof(double) * (size_t)B * (size_t)width[k]);
        d[k] = (double *)malloc(sizeof(double) * (size_t)B * (size_t)width[k]);
        if (!h[k] || !d[k]) fail = 1;
    }
    for (int k = 0; !fail && k < nl; ++k) {
        gWl[k] = (double *)calloc((size_t)width[k + 1] * (size_t)width[k], sizeof(double));
        gbl[k] = (double *)calloc((size_t)width[k + 1], sizeof(double));
        if (!gWl[k] || !gbl[k]) fail = 1;
    }
    if (fail) goto cleanup;

    /* encode */
    for (int64_t i = 0; i < B; ++i) {
        const double *r = x_raw + (size_t)i * F;
        double *e = h[0] + (size_t)i * F;
        int nstat = m->L * m->K;
        for (int j = 0; j < nstat; ++j) {
            int k = j % m->K;
            e[j] = orc_phi(r[j], m->stat_kind[k], m->stat_shift[k], m->stat_scale[k]);
        }
        for (int j = 0; j < m->Ns; ++j)
            e[nstat + j] = orc_phi(r[nstat + j], m->scal_kind[j], m->scal_shift[j], m->scal_scale[j]);
        e[F - 2] = orc_phi(r[F - 2], m->cfg_kind[0], m->cfg_shift[0], m->cfg_scale[0]);
        e[F - 1] = orc_phi(r[F - 1], m->cfg_kind[1], m->cfg_shift[1], m->cfg_scale[1]);
        if (m->round_stored_bf16) for (int j = 0; j < F; ++j) e[j] = orc_round_bf16(e[j]);
    }
    /* forward: h[k+1] = relu(W_k h[k] + b_k), last layer linear */
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < B; ++i)
        for (int k = 0; k < nl; ++k) {
            double *out = h[k + 1] + (size_t)i * width[k + 1];
            orc_dense(Wf[k], bf[k], width[k + 1], width[k], h[k] + (size_t)i * width[k], out, k < nl - 1);
            if (m->round_stored_bf16 && k < nl - 1)
                for (int j = 0; j < width[k + 1]; ++j) out[j] = orc_round_bf16(out[j]);
        }
    /* loss and output delta */
    {
        double loss = 0.0;
        const int no = width[nl];
        for (int64_t i = 0; i < B; ++i) {
            double sq = 0.0;
            for (int w = 0; w < no; ++w) {
                double e = h[nl][(size_t)i * no + w] - target[(size_t)i * no + w];
                sq += e * e;
                if (yhat_out) yhat_out[(size_t)i * no + w] = h[nl][(size_t)i * no + w];
            }
            const double nrm = sqrt(sq);
            loss += m->loss_kind == 1 ? nrm : sq;
            for (int w = 0; w < no; ++w) {
                double e = h[nl][(size_t)i * no + w] - target[(size_t)i * no + w];
                if (m->loss_kind == 1) d[nl][(size_t)i * no + w] = nrm > 0.0 ? e / (nrm * (double)B) : 0.0;
                else d[nl][(size_t)i * no + w] = 2.0 * e / (double)B;
            }
        }
        if (loss_out) *loss_out = loss / (double)B;
    }
    /* backward */
    for (int k = nl - 1; k >= first_trainable; --k) {
        const int no = width[k + 1], ni = width[k];
        /* dW[o,i] = sum_rows d[o] * h_prev[i]; db[o] = sum_rows d[o] */
#pragma omp parallel for schedule(static)
        for (int o = 0; o < no; ++o) {
            double *g = gWl[k] + (size_t)o * ni;
            double sb = 0.0;
            for (int64_t r = 0; r < B; ++r) {
                double dv = d[k + 1][(size_t)r * no + o];
                const double *hp = h[k] + (size_t)r * ni;
                sb += dv;
                for (int i = 0; i < ni; ++i) g[i] += dv * hp[i];
            }
            gbl[k][o] = sb;
        }
        if (k > first_trainable) {
#pragma omp parallel for schedule(static)
            for (int64_t r = 0; r < B; ++r) {
                const double *dn = d[k + 1] + (size_t)r * no;
                double *dp = d[k] + (size_t)r * ni;
                const double *hp = h[k] + (size_t)r * ni;
                for (int i = 0; i < ni; ++i) {
                    double acc = 0.0;
                    for (int o = 0; o < no; ++o) acc += dn[o] * Wf[k][(size_t)o * ni + i];
                    dp[i] = (hp[i] > 0.0) ? acc : 0.0; /* h = relu(pre): h > 0 <=> pre > 0 */
                    if (m->round_stored_bf16) dp[i] = orc_round_bf16(dp[i]);
                }
            }
        }
    }
    for (int k = 0; k < nl; ++k) {
        if (gW && gW[k]) memcpy(gW[k], gWl[k], sizeof(double) * (size_t)width[k + 1] * width[k]);
        if (gb && gb[k]) memcpy(gb[k], gbl[k], sizeof(double) * (size_t)width[k + 1]);
    }
    if (do_adam) {
        const double c1 = 1.0 - pow(beta1, (double)t), c2 = 1.0 - pow(beta2, (double)t);
        for (int k = first_trainable; k < nl; ++k) {
            size_t nw = (size_t)width[k + 1] * width[k], nb = (size_t)width[k + 1];
            for (size_t j = 0; j < nw + nb; ++j) {
                int isb = j >= nw;
                size_t q = isb ? j - nw : j;
                double g = isb ? gbl[k][q] : gWl[k][q];
                double *pm = isb ? &mb[k][q] : &mW[k][q];
                double *pv = isb ? &vb[k][q] : &vW[k][q];
                double *pw = isb ? &bm[k][q] : &Wm[k][q];
                *pm = beta1 * *pm + (1.0 - beta1) * g;
                *pv = beta2 * *pv + (1.0 - beta2) * g * g;
                *pw -= lr * (*pm / c1) / (sqrt(*pv / c2) + eps);
            }
        }
    }
cleanup:
    for (int k = 0; h && d && k <= nl; ++k) { free(h[k]); free(d[k]); }
    for (int k = 0; gWl && gbl && k < nl; ++k) { free(gWl[k]); free(gbl[k]); }
    free(h); free(d); free(gWl); free(gbl);
    return fail ? ORC_ERR_MEM : ORC_OK;
}

int orc_update(const orc_model *m, const double *x_raw, const double *target, int64_t B,
               const double *const *Wf, const double *const *bf,
               double *const *Wm, double *const *bm,
               double *const *mW, double *const *vW, double *const *mb, double *const *vb,
               int64_t t, double lr, double beta1, double beta2, double eps, int do_adam,
               double *loss_out, double *const *gW, double *const *gb, double *yhat_out)
{
    return orc_update_tail(m, x_raw, target, B, Wf, bf, Wm, bm, mW, vW, mb, vb, t, lr, beta1, beta2, eps,
                           do_adam, loss_out, gW, gb, yhat_out, 0);
}
