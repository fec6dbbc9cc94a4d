/*
 * autobyte.h - C ABI of the MI355X (gfx950) implementation of the AutoByte meta-network hot path.
 *
 * AutoByte (arXiv 2112.13509) tunes two ByteScheduler knobs, the partition size S_p and the credit
 * size S_c, with a meta-network f : (T, B, S_c, S_p) -> V (Eq. 1) that predicts the training speed V
 * of a job from its runtime statistics (Table 1) for a candidate pair <S_p, S_c>.  The pair with the
 * largest predicted V is applied (Section 3, introduction; Section 3.3 "Meta network optimizer"),
 * and the network keeps being adapted online on freshly observed speeds (Section 3.2 "Offline
 * training online adapting"; loss of Eq. 2).
 *
 * This library is that hot path, batched: many scenarios (one scenario = the statistics of one job
 * at one moment) times a whole grid of candidates.
 *
 *   ab_score_candidates  predicted V for every (scenario, candidate), optionally fused with the choice
 *   ab_select_best       per-scenario argmax over a stored score matrix
 *   ab_online_update     one forward + backward + Adam step on explicit (statistics, candidate, V) rows
 *   ab_online_update_tail, ab_replay_mix   the same step with frozen lower layers; minibatch from two pools
 *   ab_trigger           the choice plus the two threshold tests of the Optimization Trigger
 *
 * General rules
 *   - Every pointer marked DEVICE is HIP device memory on the current device, owned by the caller.  The
 *     library never allocates, frees or retains device memory.  It keeps no state between calls apart from
 *     the tracing hook (ab_set_trace), per-device launch attributes it looks up once, and the fixed scratch
 *     array of ab_score_candidates_static.
 *   - Every pointer marked HOST is ordinary host memory, read during the call only.
 *   - Work is enqueued on the HIP stream passed as `stream` (a hipStream_t cast to void*, NULL = the
 *     default stream).  Calls return as soon as the work is enqueued; nothing synchronises.
 *   - The workspace is DEVICE scratch of at least ab_workspace_bytes(...) bytes, 256-byte aligned, owned
 *     by the caller; its contents are undefined after the call and two calls that share it must be
 *     ordered on one stream.
 *   - Errors are returned as negative ab_status values after host-side checks of the arguments (null
 *     pointers, sizes, widths, alignment, workspace size) and of the launch status.  Nothing is thrown
 *     and nothing aborts.  Data-dependent trouble (a non-finite statistic) cannot be seen by the host
 *     and shows up in the outputs: a NaN score, and best_idx = -1 if a scenario has no non-NaN score.
 *   - Output buffers must not overlap inputs, weights or the workspace.
 *
 * Feature layout (Table 1; Section 3.1 "Meta network architecture": the feature groups are concatenated)
 *   x = [ statistics block | scalars | phi(S_p) | phi(S_c) ]
 *   statistics block: L*K transformed per-layer statistics, layer-major / statistic-minor (flat model),
 *   or the mean over the L layers of a shared two-layer MLP applied to each layer's K transformed
 *   statistics (tensor-encoder model: the paper maps the per-layer times to a feature space of fixed
 *   width before anything else reads them).  Every raw value x is transformed as phi(x) = (g(x) - shift) * scale with
 *   g = identity or natural logarithm; S_c is expressed as a multiple of S_p (Section 2.4).
 *
 * Network: hidden dense layers with ReLU, then a linear output layer of n_outputs units (V is a regression target).
 */
#ifndef AUTOBYTE_H
#define AUTOBYTE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define AB_MAX_STATS   16   /* statistics per layer (K): Table 1's T has one backward time per layer and worker;
                               the two encoders take at most AB_MAX_ENCODER_STATS of them                   */
#define AB_MAX_ENCODER_STATS 8
#define AB_MAX_SCALARS 40   /* scalar features per scenario (Table 1: n, l, type vectors, B_d and B_u per worker) */
#define AB_MAX_HIDDEN  8    /* hidden layers of the scorer                 */
#define AB_MAX_OUTPUTS 16   /* entries of the predicted speed V            */
#define AB_MAX_LAYERS  12   /* encoder (up to 3) + hidden (8) + output (1)                */

typedef int32_t ab_status;
enum {
    AB_OK = 0,
    AB_ERR_NULL = -1,         /* a required pointer is NULL                                   */
    AB_ERR_SHAPE = -2,        /* a size is non-positive or inconsistent (e.g. C != P*Q)        */
    AB_ERR_DTYPE = -3,        /* compute_dtype is not AB_F32 / AB_BF16                         */
    AB_ERR_ALIGN = -4,        /* a pointer misses its required alignment                       */
    AB_ERR_WORKSPACE = -5,    /* workspace is NULL or smaller than ab_workspace_bytes(...)     */
    AB_ERR_UNSUPPORTED = -6,  /* valid description that this library has no kernel for         */
    AB_ERR_DEVICE = -7        /* HIP reported a launch / runtime error                         */
};

enum { AB_F32 = 0, AB_BF16 = 1 };          /* arithmetic type of weights and activations; accumulation is fp32 */
enum { AB_ENC_LINEAR = 0, AB_ENC_LOG = 1 };
enum { AB_LOSS_MSE = 0, AB_LOSS_L2NORM = 1 };

/* phi(x) = (g(x) - shift) * scale, g(x) = x (AB_ENC_LINEAR) or ln x (AB_ENC_LOG). */
typedef struct { int32_t kind; float shift; float scale; } ab_enc;

/*
 * Model description (HOST, plain data, read during the call).
 *   n_layers, n_stats      L and K of the statistics tensor dyn[S, L, K]; K <= AB_MAX_STATS for the flat layout,
 *                          K <= AB_MAX_ENCODER_STATS with an encoder (more is AB_ERR_UNSUPPORTED)
 *   n_scalars              scalar features per scenario (worker count, bandwidth, type one-hots ...)
 *   enc_*                  transform of each statistic kind, each scalar, the partition size and the
 *                          credit multiple
 *   n_hidden, hidden[]     scorer hidden widths.  Supported: 0 <= n_hidden <= 8, every width a multiple
 *                          of 64 and <= 4096.  n_hidden = 0 is the linear scorer V = W x + b (flat statistics
 *                          only; one launch, no workspace needed beyond the 256 bytes ab_workspace_bytes reports)
 *   tensor_encoder         0: flat statistics block (width L*K); 1: shared per-layer MLP
 *                          K -> enc_hidden[0] -> enc_hidden[1] (ReLU after both), mean over the L layers
 *                          (width enc_hidden[1]).  Supported: enc_hidden = {128, 128};
 *                          2: the temporal encoder of Section 3.1 "Meta network architecture": each layer's
 *                          K statistics are embedded linearly into enc_hidden[0] values and a two-layer
 *                          LSTM of enc_hidden[1] units per layer runs over the L layers in order (zero
 *                          initial state); the second layer's last hidden state is the statistics block
 *                          (width enc_hidden[1]).  Supported: enc_hidden = {32, 64}.
 *                          Both encoders need compute_dtype = AB_BF16
 *   compute_dtype          AB_F32: fp32 weights, activations and fp32 MFMA; AB_BF16: bf16 weights and
 *                          activations with fp32 accumulation
 *   n_outputs              entries of the predicted speed V (Table 1 gives V one entry per worker); 0 or 1:
 *                          a single value; at most AB_MAX_OUTPUTS.  A candidate's score is the mean of the
 *                          n_outputs predictions (Eq. 1 ranks candidates by V; for a vector the mean is this
 *                          library's reading: a synchronous job advances at one rate, which the per-worker
 *                          entries measure n_outputs times)
 *   loss_kind              loss of ab_online_update: AB_LOSS_MSE: mean over the minibatch of the squared
 *                          error summed over the n_outputs entries; AB_LOSS_L2NORM: mean over the minibatch
 *                          of the Euclidean norm of the error vector (Eq. 2 as printed; a row predicted
 *                          exactly contributes no gradient)
 * The scorer's input width is F = (L*K or enc_hidden[1]) + n_scalars + 2.
 */
typedef struct {
    int32_t n_layers, n_stats, n_scalars;
    ab_enc  enc_stat[AB_MAX_STATS];
    ab_enc  enc_scalar[AB_MAX_SCALARS];
    ab_enc  enc_partition, enc_credit;
    int32_t n_hidden;
    int32_t hidden[AB_MAX_HIDDEN];
    int32_t tensor_encoder;
    int32_t enc_hidden[2];
    int32_t compute_dtype;
    int32_t n_outputs;
    int32_t loss_kind;
} ab_model_desc;

/*
 * Parameters (the struct is HOST, every pointer in it is DEVICE).
 * Layer order: the encoder's layers first (two if tensor_encoder = 1; three if tensor_encoder = 2: the
 * embedding [E, K], then per LSTM layer one matrix [4H, n_in + H] = [W_ih | W_hh] acting on
 * [input ; previous hidden state] with gate blocks in the order input, forget, candidate, output and one
 * bias [4H], n_in = E for the first and H for the second layer), then the scorer's hidden layers, then
 * the output layer (n_outputs x last hidden width).
 *   W[k]         [out, in] row-major in compute_dtype (bf16 = upper 16 bits of an fp32), 16-byte aligned
 *   b[k]         [out] fp32
 * Only ab_online_update uses the rest (flat model, so index k counts scorer layers from 0):
 *   W_master[k]  fp32 master copy of W[k]; b[k] is its own master
 *   adam_mW/vW   first / second moment of W[k], fp32; adam_mb/vb the same for b[k]
 *   step         one int64: number of update steps taken so far (0 before the first step)
 */
typedef struct {
    const void  *W[AB_MAX_LAYERS];
    float       *b[AB_MAX_LAYERS];
    float       *W_master[AB_MAX_LAYERS];
    float       *adam_mW[AB_MAX_LAYERS], *adam_vW[AB_MAX_LAYERS];
    float       *adam_mb[AB_MAX_LAYERS], *adam_vb[AB_MAX_LAYERS];
    int64_t     *step;
} ab_params;

/* Runtime statistics of S scenarios (struct HOST, pointers DEVICE, fp32, densely packed). */
typedef struct {
    const float *dyn;       /* [S, L, K] raw per-layer statistics (computation times, tensor bytes ...) */
    const float *scalars;   /* [S, n_scalars] raw scalars                                                */
    int64_t      S;
    const int32_t *layers_of; /* [S] or NULL: how many of the L layers scenario s really has (jobs differ in
                                 their number of layers, Section 3.1 "Meta network architecture"); rows of dyn
                                 past that count never influence a result; values are clamped to [1, L].  Needs an
                                 encoder (tensor_encoder = 1: mean over the scenario's own layers; 2: the LSTM
                                 stops after them); must be NULL for the flat layout                       */
} ab_stats;

/* Candidate grid (struct HOST, pointers DEVICE). Candidate c = p*Q + q.
 * per_scenario = 0: one grid shared by all scenarios.  per_scenario = 1: every scenario brings its own P
 * partition sizes and Q credit multiples (Table 1 lists S_p and S_c as inputs of the one job being tuned; jobs
 * of different models need not be offered the same values): partition_bytes is [S, P], credit_mult [S, Q]. */
typedef struct {
    const float *partition_bytes;  int32_t P;   /* [P] or [S, P] partition sizes S_p                    */
    const float *credit_mult;      int32_t Q;   /* [Q] or [S, Q] credit sizes as multiples of S_p       */
    int32_t      per_scenario;
} ab_grid;

/*
 * Bytes of workspace needed.  Pass S and C = P*Q for ab_score_candidates (B = 0), or B for
 * ab_online_update (S = C = 0); with all three set the result covers both.  Returns 0 for an
 * unsupported description.
 */
size_t ab_workspace_bytes(const ab_model_desc *desc, int64_t S, int32_t C, int64_t B);

/*
 * Predicted V of every candidate for every scenario (Eq. 1 over the <S_p, S_c> grid), and / or the
 * predicted-best candidate per scenario (Section 3: the pair with the maximum predicted speed).
 *   scores      DEVICE [S, C] fp32, or NULL when only the choice is wanted
 *   best_idx    DEVICE [S] int32 index c = p*Q+q of the largest score (lowest index on exact ties,
 *               NaN never wins, -1 if every score of the scenario is NaN), or NULL
 *   best_score  DEVICE [S] fp32 score of that candidate (NaN where best_idx = -1), or NULL
 * At least one of scores / best_idx must be given.  S = 0 is a valid no-op.
 */
ab_status ab_score_candidates(const ab_model_desc *desc, const ab_params *params,
                              const ab_stats *stats, const ab_grid *grid,
                              float *scores, int32_t *best_idx, float *best_score,
                              void *workspace, size_t workspace_bytes, void *stream);

/*
 * ab_score_candidates that also returns the predicted speed vector itself for the chosen candidate (Table 1: V has
 * one entry per worker; Eq. 1 returns V, of which ab_score_candidates only reports the mean it ranks by).
 *   v_best      DEVICE [S, n_outputs] fp32: V of candidate best_idx[s] (NaN where best_idx[s] = -1), or NULL;
 *               needs best_idx.  mean_o v_best[s, o] equals best_score[s] up to fp32 summation order.
 * Everything else as ab_score_candidates (same workspace size).  With v_best given the hidden chain runs once
 * more on one row per scenario (1/C of the scoring work) and the output layer is applied unit by unit.
 */
ab_status ab_score_candidates_v(const ab_model_desc *desc, const ab_params *params,
                                const ab_stats *stats, const ab_grid *grid,
                                float *scores, int32_t *best_idx, float *best_score, float *v_best,
                                void *workspace, size_t workspace_bytes, void *stream);

/*
 * ab_score_candidates for callers that cannot allocate device memory or hand over a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The workspace is a fixed array of
 * AB_STATIC_SCRATCH_BYTES inside the library's code object (every device the library runs on holds its own
 * copy until the process ends); the call allocates nothing, on the device or through any library.
 * Arguments, outputs and results as ab_score_candidates (the same kernels run).  A problem whose
 * ab_workspace_bytes(desc, S, C, 0) exceeds AB_STATIC_SCRATCH_BYTES is refused with AB_ERR_WORKSPACE before
 * anything is enqueued.  All calls on one device share the one array: calls that may overlap in time on a
 * device (different streams, different host threads) race and must be ordered by the caller; the array's
 * contents are undefined between calls and nothing in it has to be cleared (every kernel writes what it later
 * reads).  ab_static_scratch_bytes returns AB_STATIC_SCRATCH_BYTES.
 */
#define AB_STATIC_SCRATCH_BYTES (32u << 20)
size_t ab_static_scratch_bytes(void);
ab_status ab_score_candidates_static(const ab_model_desc *desc, const ab_params *params,
                                     const ab_stats *stats, const ab_grid *grid,
                                     float *scores, int32_t *best_idx, float *best_score, void *stream);

/*
 * Per-scenario argmax over a stored score matrix (same rules as above).
 *   scores      DEVICE fp32, row s starts at scores + s*row_stride (row_stride >= C, in elements)
 *   best_idx    DEVICE [S] int32;  best_score DEVICE [S] fp32 or NULL
 */
ab_status ab_select_best(const float *scores, int64_t S, int32_t C, int64_t row_stride,
                         int32_t *best_idx, float *best_score, void *stream);

/*
 * Optimization Trigger (Section 3.3 "Optimization trigger"), fused with the choice, on a stored score matrix.
 * Per scenario s, with V_cur = scores[s, current_idx[s]] and V_best the largest non-NaN score:
 *   best_idx[s]     as ab_select_best
 *   gain[s]         (V_best - V_cur) / |V_cur|                      (optional)
 *   reconfigure[s]  1 if gain >= gain_threshold, else 0             (the paper skips attempts below 5 %)
 *   adapt[s]        1 if |V_cur - observed[s]| / |observed[s]| > error_threshold, else 0 (the paper starts
 *                   online adaptation above 10 %); optional, needs `observed`
 * All arithmetic is IEEE single precision.  No valid best candidate, or current_idx[s] outside [0, C):
 * gain = NaN, reconfigure = 0, adapt = 0.
 *   scores DEVICE fp32 (row s at scores + s*row_stride), current_idx DEVICE [S] int32, observed DEVICE [S] fp32
 *   or NULL, best_idx DEVICE [S] int32, gain DEVICE [S] fp32 or NULL, reconfigure DEVICE [S] uint8,
 *   adapt DEVICE [S] uint8 or NULL (must be NULL when observed is NULL).
 */
ab_status ab_trigger(const float *scores, int64_t S, int32_t C, int64_t row_stride,
                     const int32_t *current_idx, const float *observed,
                     float gain_threshold, float error_threshold,
                     int32_t *best_idx, float *gain, uint8_t *reconfigure, uint8_t *adapt, void *stream);

/*
 * One online-adaptation step of the flat model (tensor_encoder = 0) on a minibatch of B observed rows:
 * forward, the loss of desc->loss_kind (mean_i |V_hat_i - V_i|^2, or Eq. 2's unsquared norm mean_i |V_hat_i - V_i|),
 * exact back-propagation, Adam with bias correction (epsilon outside the square root).
 *   x_raw     DEVICE [B, F] fp32 raw rows: L*K statistics, n_scalars scalars, partition bytes, credit
 *             multiple (transformed on the device with the description's constants)
 *   target    DEVICE [B, n_outputs] fp32 observed speed V (one value per row, or one per worker)
 *   loss_out  DEVICE one fp32 (loss before the step), or NULL
 * Mutates W_master, b, the Adam moments, *step (incremented by one) and refreshes W[k] (the
 * compute_dtype copy used by scoring).  With AB_BF16 the GEMMs run on bf16 copies of the masters.
 */
ab_status ab_online_update(const ab_model_desc *desc, ab_params *params,
                           const float *x_raw, const float *target, int64_t B,
                           float lr, float beta1, float beta2, float eps,
                           float *loss_out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Transfer-learning form of the online step (Section 3.2 "Offline training online adapting": the offline
 * trained model is updated by transfer learning): scorer layers below first_trainable are frozen: they are
 * only run forward, their parameters, master copies and moments are not touched (and need not be given,
 * beyond W[k] and b[k]); back-propagation stops at layer first_trainable.  0 <= first_trainable <= n_hidden;
 * 0 is ab_online_update, n_hidden trains the output layer alone.  Everything else as ab_online_update
 * (same workspace size).
 */
ab_status ab_online_update_tail(const ab_model_desc *desc, ab_params *params,
                                const float *x_raw, const float *target, int64_t B, int32_t first_trainable,
                                float lr, float beta1, float beta2, float eps,
                                float *loss_out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Minibatch assembly for online adaptation (Section 3.2: the newly observed samples also extend the
 * dataset the model was trained on, so a step mixes both): output row i is row pick[i] of the new pool
 * if pick[i] >= 0, else row -pick[i] - 1 of the old pool; the targets follow.  Which rows to mix is the
 * caller's draw.  An index outside its pool yields a NaN row and NaN targets (no memory is read).
 *   x_new [n_new, F], target_new [n_new, n_outputs], x_old [n_old, F], target_old [n_old, n_outputs]  DEVICE fp32
 *   pick [B] DEVICE int32;  x_out [B, F], target_out [B, n_outputs] DEVICE fp32 (must not overlap the pools)
 * n_outputs >= 1 is the number of observed speeds per row (one, or one per worker as ab_online_update takes them),
 * at most AB_MAX_OUTPUTS.  A pool of size 0 may be NULL.
 */
ab_status ab_replay_mix(const float *x_new, const float *target_new, int64_t n_new,
                        const float *x_old, const float *target_old, int64_t n_old,
                        const int32_t *pick, int64_t B, int32_t F, int32_t n_outputs,
                        float *x_out, float *target_out, void *stream);

const char *ab_status_string(ab_status status);

/*
 * Optional launch tracing, for measurement (the paper times computation and communication per
 * mini-batch, Section 3.1 "Input runtime metrics"; this is the library's counterpart for its own
 * kernels).  When a callback is installed, every kernel launch made by the entry points above is
 * bracketed by two calls on the launching host thread: phase 0 just before the launch is enqueued
 * and phase 1 just after.  A caller that records an event on `stream` in both gets the kernel's
 * device time.  `kernel` is a static string naming the launch's role, `work` its algorithmic
 * floating-point operations (matrix products) or bytes moved (streaming kernels), `work_is_bytes`
 * tells which.  Pass fn = NULL to switch tracing off (the default).  Process-wide, not thread-safe
 * against concurrent entry-point calls.
 */
typedef void (*ab_trace_fn)(const char *kernel, int32_t phase, double work, int32_t work_is_bytes,
                            void *stream, void *user);
void ab_set_trace(ab_trace_fn fn, void *user);

/* Library version as major*10000 + minor*100 + patch. */
int32_t ab_version(void);

#ifdef __cplusplus
}
#endif
#endif /* AUTOBYTE_H */
