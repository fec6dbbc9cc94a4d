// Streaming kernels around the matrix-core GEMMs of the scoring path: feature transform, layer-1
// candidate term, weight packing, the shared per-tensor encoder, score assembly and argmax.
#include "internal.hpp"

namespace ab {

// ------------------------------------------------------------------------------------------------
// Feature transform (Section 3.3 "Meta network optimizer": runtime statistics are turned into the
// network's input vector).  One thread produces two adjacent columns of one scenario's row.
//   xs[s, col0 + j]            j in [0, n_stat)            <- phi_stat(dyn[s, j])      (flat model only)
//   xs[s, col0 + n_stat + j]   j in [0, n_scal)            <- phi_scal(scal[s, j])
//   xs[s, ...up to ld)                                      <- 0   (K padding for the GEMM)
// ------------------------------------------------------------------------------------------------
struct EncodeArgs {
    const float *dyn; const float *scal;
    void *xs; int64_t S; int32_t ld;
    int32_t col0, n_stat, n_stats_per_layer, n_scal;
    ab_enc enc_stat[AB_MAX_STATS];
    ab_enc enc_scal[AB_MAX_SCALARS];
};

template <typename T>
__global__ __launch_bounds__(256) void encode_stats_kernel(const EncodeArgs a)
{
    const int pairs = (a.ld - a.col0) >> 1;
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t s = gid / pairs;
    if (s >= a.S) return;
    const int j0 = (int)(gid - s * pairs) * 2;
    float v[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int j = j0 + e;
        float x = 0.f;
        if (j < a.n_stat) {
            x = phi(a.dyn[s * a.n_stat + j], a.enc_stat[j % a.n_stats_per_layer]);
        } else if (j < a.n_stat + a.n_scal) {
            const int q = j - a.n_stat;
            x = phi(a.scal[s * a.n_scal + q], a.enc_scal[q]);
        }
        v[e] = x;
    }
    const int64_t o = s * a.ld + a.col0 + j0;
    if constexpr (sizeof(T) == 2) ((uint32_t *)a.xs)[o >> 1] = pack_bf16x2(v[0], v[1]);
    else ((f32x2 *)a.xs)[o >> 1] = f32x2{v[0], v[1]};
}

// The same transform, four adjacent columns per thread (16-byte loads, 8- or 16-byte stores), for rows
// whose statistics part is a multiple of four columns and 16-byte aligned.  A work-group takes `rpb`
// rows; lane -> (row, quad) by a multiply-high with magic = floor(2^32 / q4) + 1 (exact while
// index * q4 < 2^32), likewise column -> statistic index.  The transform constants sit in LDS so that a
// lane can pick its own.  With bf16 as compute type the logarithm is the hardware's log2 (1 ulp, far
// below what the rounding to bf16 keeps) times ln 2.
template <typename T>
__device__ __forceinline__ float phi_tab(float x, const f32x4 *tab, int i)
{
    float lg;
    if constexpr (sizeof(T) == 2) lg = __builtin_amdgcn_logf(x) * 0.69314718056f;
    else lg = logf(x);
    const f32x4 t = tab[i];                        // (kind, shift, scale, -)
    return ((t.x != 0.f ? lg : x) - t.y) * t.z;
}

template <typename T>
__device__ __forceinline__ void store_quad(void *xs, int64_t o, const float (&v)[4])
{
    if constexpr (sizeof(T) == 2) {
        typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
        *(u32x2 *)((uint16_t *)xs + o) = u32x2{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
    } else {
        *(f32x4 *)((float *)xs + o) = f32x4{v[0], v[1], v[2], v[3]};
    }
}

struct QuadSplit { int q4s, q4t; uint32_t magic_q4s, magic_q4t, magic_k; int rpb; };

template <typename T>
__device__ __forceinline__ void encode_stats_quad_block(const EncodeArgs &a, const QuadSplit &g, unsigned block)
{
    __shared__ f32x4 tab[AB_MAX_STATS + AB_MAX_SCALARS];     // statistics first, then the scalars
    if (threadIdx.x < AB_MAX_STATS + AB_MAX_SCALARS) {
        const int i = threadIdx.x;
        const ab_enc *e = i < AB_MAX_STATS ? &a.enc_stat[i] : &a.enc_scal[i - AB_MAX_STATS];
        tab[i] = f32x4{e->kind == AB_ENC_LOG ? 1.f : 0.f, e->shift, e->scale, 0.f};
    }
    __syncthreads();
    const int64_t row0 = (int64_t)block * g.rpb;
    const int rows = (int)((a.S - row0 < g.rpb) ? a.S - row0 : g.rpb);

    // the statistics columns: q4s quads a row, a thread's four loads issued before the first value is used
    const uint32_t n_a = (uint32_t)rows * (uint32_t)g.q4s;
    for (uint32_t base = 0; base < n_a; base += 1024) {
        f32x4 x[4];
        uint32_t r[4];
        int col[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t i = base + u * 256 + threadIdx.x;
            r[u] = __umulhi(i, g.magic_q4s);
            col[u] = (int)(i - r[u] * (uint32_t)g.q4s) * 4;
            if (i < n_a) x[u] = __builtin_nontemporal_load((const f32x4 *)(a.dyn + (row0 + r[u]) * a.n_stat + col[u]));
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (base + u * 256 + threadIdx.x >= n_a) break;
            int k = a.n_stats_per_layer == 1
                        ? 0 : col[u] - (int)__umulhi((uint32_t)col[u], g.magic_k) * a.n_stats_per_layer;
            float v[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                v[e] = phi_tab<T>(x[u][e], tab, k);
                k = (k + 1 == a.n_stats_per_layer) ? 0 : k + 1;
            }
            store_quad<T>(a.xs, (row0 + r[u]) * a.ld + a.col0 + col[u], v);
        }
    }

    // the scalars and the zero padding behind them: q4t quads a row
    const uint32_t n_b = (uint32_t)rows * (uint32_t)g.q4t;
    for (uint32_t i = threadIdx.x; i < n_b; i += 256) {
        const uint32_t r = __umulhi(i, g.magic_q4t);
        const int q0 = (int)(i - r * (uint32_t)g.q4t) * 4;
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int q = q0 + e;
            v[e] = q < a.n_scal ? phi_tab<T>(a.scal[(row0 + r) * a.n_scal + q], tab, AB_MAX_STATS + q) : 0.f;
        }
        store_quad<T>(a.xs, (row0 + r) * a.ld + a.col0 + a.n_stat + q0, v);
    }
}

template <typename T>
__global__ __launch_bounds__(256) void encode_stats_quad_kernel(const EncodeArgs a, const QuadSplit g)
{
    encode_stats_quad_block<T>(a, g, blockIdx.x);
}

// ------------------------------------------------------------------------------------------------
// Layer-1 preparation.  The first dense layer acts on [statistics | S_p | S_c]; its statistics
// columns are shared by all candidates of a scenario and its two configuration columns by all
// scenarios, so W1 x + b1 = A[s] + B[c] with A[s] = W1_s x_s + b1 (the bias rides in the A[s] GEMM's
// epilogue) and B[c] = wp * phi(S_p) + wc * phi(S_c).  This kernel packs the statistics columns of W1
// into a K-padded matrix for the A[s] GEMM, builds B[c] both as a [C, H1] matrix (generic kernels) and
// as its four generating vectors wp[H1], wc[H1], phi_p[C], phi_c[C] (the 256x256 kernel rebuilds B[c]
// from them with two FMAs instead of fetching 4 bytes per element), and widens the output weights.
// ------------------------------------------------------------------------------------------------
struct PrepArgs {
    const void *W1; int32_t F, Fs, H1, ld;      // W1[H1, F]; packed copy w1s[H1, ld]
    void *w1s;
    const float *b1;
    const float *part; const float *cred; int32_t P, Q;
    ab_enc enc_part, enc_cred;
    float *b_term;                               // [P*Q, H1]
    float *wp_f, *wc_f, *xp_f, *xc_f;            // [H1], [H1], [P*Q], [P*Q]
    const void *Wout; const float *b_out; int32_t H_last, n_out; float *w_out_f;   // w_out_f[H_last + 1]
};

template <typename T>
__device__ __forceinline__ float load_as_f32(const void *p, int64_t i)
{
    if constexpr (sizeof(T) == 2) return bf16_bits_to_f32(((const uint16_t *)p)[i]);
    else return ((const float *)p)[i];
}

template <typename T>
__device__ __forceinline__ void prep_layer1_block(const PrepArgs &a, unsigned block)
{
    const int64_t gid = (int64_t)block * 256 + threadIdx.x;
    const int64_t n_pack = (int64_t)a.H1 * a.ld;
    const int64_t n_bt = (int64_t)a.P * a.Q * a.H1;
    if (gid < n_pack) {
        const int h = (int)(gid / a.ld), k = (int)(gid - (int64_t)h * a.ld);
        if constexpr (sizeof(T) == 2) {
            uint16_t v = (k < a.Fs) ? ((const uint16_t *)a.W1)[(int64_t)h * a.F + k] : (uint16_t)0;
            ((uint16_t *)a.w1s)[gid] = v;
        } else {
            ((float *)a.w1s)[gid] = (k < a.Fs) ? ((const float *)a.W1)[(int64_t)h * a.F + k] : 0.f;
        }
    } else if (gid < n_pack + n_bt) {
        const int64_t e = gid - n_pack;
        const int c = (int)(e / a.H1), h = (int)(e - (int64_t)c * a.H1);
        const float xp = phi(a.part[c / a.Q], a.enc_part), xc = phi(a.cred[c % a.Q], a.enc_cred);
        const float wp = load_as_f32<T>(a.W1, (int64_t)h * a.F + a.Fs);
        const float wc = load_as_f32<T>(a.W1, (int64_t)h * a.F + a.Fs + 1);
        a.b_term[e] = wp * xp + wc * xc;
    } else if (gid < n_pack + n_bt + a.H_last) {
        const int h = (int)(gid - n_pack - n_bt);
        // the output layer folded to one unit: the mean over its n_out rows (a candidate's score is the mean
        // of the per-worker predictions); the folded bias follows the weights
        float acc = 0.f, bacc = 0.f;
        for (int w = 0; w < a.n_out; ++w) acc += load_as_f32<T>(a.Wout, (int64_t)w * a.H_last + h);
        a.w_out_f[h] = acc / (float)a.n_out;
        if (h == 0) {
            for (int w = 0; w < a.n_out; ++w) bacc += a.b_out[w];
            a.w_out_f[a.H_last] = bacc / (float)a.n_out;
        }
    } else if (gid < n_pack + n_bt + a.H_last + a.H1) {
        const int h = (int)(gid - n_pack - n_bt - a.H_last);
        a.wp_f[h] = load_as_f32<T>(a.W1, (int64_t)h * a.F + a.Fs);
        a.wc_f[h] = load_as_f32<T>(a.W1, (int64_t)h * a.F + a.Fs + 1);
    } else if (gid < n_pack + n_bt + a.H_last + a.H1 + (int64_t)a.P * a.Q) {
        const int c = (int)(gid - n_pack - n_bt - a.H_last - a.H1);
        a.xp_f[c] = phi(a.part[c / a.Q], a.enc_part);
        a.xc_f[c] = phi(a.cred[c % a.Q], a.enc_cred);
    }
}

template <typename T>
__global__ __launch_bounds__(256) void prep_layer1_kernel(const PrepArgs a)
{
    prep_layer1_block<T>(a, blockIdx.x);
}

// The two launches that open a scoring pass of the flat model are independent of each other (the transform reads
// the statistics, the preparation reads the model and the grid), so they share one launch: the first
// `enc_blocks` work-groups do the feature transform (the long, memory-bound part starts at once), the short
// work-groups of the layer-1 preparation fill in behind them.
template <typename T>
__global__ __launch_bounds__(256) void encode_and_prep_kernel(const EncodeArgs a, const QuadSplit g, const PrepArgs p,
                                                              unsigned enc_blocks)
{
    if (blockIdx.x < enc_blocks) encode_stats_quad_block<T>(a, g, blockIdx.x);
    else prep_layer1_block<T>(p, blockIdx.x - enc_blocks);
}

// Per-scenario candidate grids: the transformed pair (phi(S_p), phi(S_c)) of every (scenario, candidate) row
// of a chunk, row = s * P * Q + p * Q + q, from part[S, P] and cred[S, Q].
struct GridRowsArgs { const float *part, *cred; int32_t P, Q; ab_enc enc_part, enc_cred; float *xp_row, *xc_row; int64_t rows; };
__global__ __launch_bounds__(256) void grid_rows_kernel(const GridRowsArgs a)
{
    const int64_t row = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (row >= a.rows) return;
    const int Cn = a.P * a.Q;
    const int64_t s = row / Cn;
    const int c = (int)(row - s * Cn);
    a.xp_row[row] = phi(a.part[s * a.P + c / a.Q], a.enc_part);
    a.xc_row[row] = phi(a.cred[s * a.Q + c % a.Q], a.enc_cred);
}

hipError_t launch_grid_rows(const ab_model_desc *d, const float *part, const float *cred, int P, int Q,
                            float *xp_row, float *xc_row, int64_t rows, hipStream_t st)
{
    if (rows == 0) return hipSuccess;
    GridRowsArgs a{part, cred, P, Q, d->enc_partition, d->enc_credit, xp_row, xc_row, rows};
    grid_rows_kernel<<<(unsigned)((rows + 255) / 256), 256, 0, st>>>(a);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// The predicted speed vector V of the chosen candidate (Table 1: V has one entry per worker; Eq. 1 returns V).
// Scoring ranks candidates by the mean of V through a folded output unit; for the one chosen candidate per
// scenario the hidden chain is run once more (one row per scenario) and the output layer applied unit by unit.
// ------------------------------------------------------------------------------------------------
// The chosen candidate's transformed pair (phi(S_p), phi(S_c)) per scenario; NaN where nothing was chosen.
struct ChosenArgs { const float *part, *cred; int32_t P, Q, per_scenario; ab_enc enc_part, enc_cred;
                    const int32_t *best_idx; float *xp_sel, *xc_sel; int64_t S; };
__global__ __launch_bounds__(256) void chosen_pair_kernel(const ChosenArgs a)
{
    const int64_t s = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (s >= a.S) return;
    const int c = a.best_idx[s];
    float xp = __builtin_nanf(""), xc = __builtin_nanf("");
    if (c >= 0 && c < a.P * a.Q) {
        const int p = c / a.Q, q = c - p * a.Q;
        xp = phi(a.part[(a.per_scenario ? s * a.P : 0) + p], a.enc_part);
        xc = phi(a.cred[(a.per_scenario ? s * a.Q : 0) + q], a.enc_cred);
    }
    a.xp_sel[s] = xp;
    a.xc_sel[s] = xc;
}

hipError_t launch_chosen_pair(const ab_model_desc *d, const ab_grid *grid, const int32_t *best_idx,
                              float *xp_sel, float *xc_sel, int64_t S, hipStream_t st)
{
    if (S == 0) return hipSuccess;
    ChosenArgs a{grid->partition_bytes, grid->credit_mult, grid->P, grid->Q, grid->per_scenario,
                 d->enc_partition, d->enc_credit, best_idx, xp_sel, xc_sel, S};
    chosen_pair_kernel<<<(unsigned)((S + 255) / 256), 256, 0, st>>>(a);
    return hipGetLastError();
}

// V[s, o] = b[o] + sum_j W[o, j] * h[s, j]: a wavefront per scenario, lanes over j, up to AB_MAX_OUTPUTS sums.
// h is the last hidden activation in fp32 (h_last), or, for a scorer with one hidden layer, generated here as
// relu(a_term[s, j] + wp[j] * xp[s] + wc[j] * xc[s]).  A scenario without a choice (best_idx < 0) gets NaN.
struct OutputVArgs { const float *h_last; const float *a_term, *wp, *wc, *xp_sel, *xc_sel;
                     const void *W; const float *b; int32_t H, n_out; const int32_t *best_idx; float *V; int64_t S; };
template <typename T>
__global__ __launch_bounds__(256) void output_v_kernel(const OutputVArgs a)
{
    const int lane = threadIdx.x & 63;
    const int64_t s = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (s >= a.S) return;
    float acc[AB_MAX_OUTPUTS];
#pragma unroll
    for (int o = 0; o < AB_MAX_OUTPUTS; ++o) acc[o] = 0.f;
    const float xp = a.h_last ? 0.f : a.xp_sel[s], xc = a.h_last ? 0.f : a.xc_sel[s];
    for (int j = lane; j < a.H; j += 64) {
        float h;
        if (a.h_last) h = a.h_last[s * a.H + j];
        else {
            h = relu_keep_nan(fmaf(a.wc[j], xc, fmaf(a.wp[j], xp, a.a_term[s * a.H + j])));   // (the last hidden
        }                                                       // activation stays fp32 in the scoring pass too)
#pragma unroll
        for (int o = 0; o < AB_MAX_OUTPUTS; ++o) {
            if (o < a.n_out) {
                float w;
                if constexpr (sizeof(T) == 2) w = bf16_bits_to_f32(((const uint16_t *)a.W)[(int64_t)o * a.H + j]);
                else w = ((const float *)a.W)[(int64_t)o * a.H + j];
                acc[o] = fmaf(w, h, acc[o]);
            }
        }
    }
    const bool none = a.best_idx[s] < 0;
#pragma unroll
    for (int o = 0; o < AB_MAX_OUTPUTS; ++o) {
        if (o < a.n_out) {
            const float v = wave_sum(acc[o]) + a.b[o];
            if (lane == 0) a.V[s * a.n_out + o] = none ? __builtin_nanf("") : v;
        }
    }
}

hipError_t launch_output_v(int dtype, const float *h_last, const float *a_term, const float *wp, const float *wc,
                           const float *xp_sel, const float *xc_sel, const void *W, const float *b, int H, int n_out,
                           const int32_t *best_idx, float *V, int64_t S, hipStream_t st)
{
    if (S == 0) return hipSuccess;
    OutputVArgs a{h_last, a_term, wp, wc, xp_sel, xc_sel, W, b, H, n_out, best_idx, V, S};
    const unsigned blocks = (unsigned)((S + 3) / 4);
    if (dtype == AB_BF16) output_v_kernel<bf16_t><<<blocks, 256, 0, st>>>(a);
    else                  output_v_kernel<float><<<blocks, 256, 0, st>>>(a);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Argmax helpers: (value, index) pairs, larger value wins, lower index wins ties, NaN never wins.
// "Nothing yet" is (-inf, INT_MAX).
// ------------------------------------------------------------------------------------------------
#define AB_NONE 0x7fffffff
__device__ __forceinline__ void amax_take(float &bv, int &bi, float v, int i)
{
    if (!(v != v) && (v > bv || (v == bv && i < bi))) { bv = v; bi = i; }
}
// Over the 64 lanes of a wavefront, result in every lane: the exchanges of wave_sum (no LDS round trips); a lane
// that an exchange does not reach takes "nothing yet", which changes nothing.
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ void amax_dpp(float &bv, int &bi)
{
    const float ov = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp((int)0xff800000u, __builtin_bit_cast(int, bv),
                                                                           CTRL, ROW_MASK, 0xF, false));
    const int oi = __builtin_amdgcn_update_dpp(AB_NONE, bi, CTRL, ROW_MASK, 0xF, false);
    amax_take(bv, bi, ov, oi);
}
__device__ __forceinline__ void amax_wave(float &bv, int &bi)
{
    amax_dpp<0xB1>(bv, bi);
    amax_dpp<0x4E>(bv, bi);
    amax_dpp<0x141>(bv, bi);
    amax_dpp<0x140>(bv, bi);
    amax_dpp<0x142, 0xA>(bv, bi);    // row_bcast:15
    amax_dpp<0x143, 0xC>(bv, bi);    // row_bcast:31
    bv = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, bv), 63));
    bi = __builtin_amdgcn_readlane(bi, 63);
}

// One work-group per scenario.  score[c] = b_out + sum_t partial[(row0 + c)*nt + t]  (nt = 1 and
// b_out = 0 turn this into a plain argmax over stored scores with a row stride).
struct FinishArgs {
    const float *partial; int32_t nt; int64_t row_stride;   // elements between scenarios in `partial` (per nt)
    const float *b_out;                                      // one fp32 or NULL
    float *scores; int64_t score_stride;                     // NULL: do not store
    int32_t *best_idx; float *best_score;                    // may be NULL
    int32_t C;
};

__global__ __launch_bounds__(256) void finish_select_kernel(const FinishArgs a)
{
    const int64_t s = blockIdx.x;
    const float *p = a.partial + s * a.row_stride * a.nt;
    const float b = a.b_out ? a.b_out[0] : 0.f;
    float bv = -INFINITY;
    int bi = AB_NONE;
    for (int c0 = threadIdx.x; c0 < a.C; c0 += 1024) {      // four candidates per thread at a time, loads together
        float v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int c = c0 + 256 * u;
            v[u] = c < a.C ? p[(int64_t)c * a.nt] : 0.f;
        }
        for (int t = 1; t < a.nt; ++t) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int c = c0 + 256 * u;
                if (c < a.C) v[u] += p[(int64_t)c * a.nt + t];
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int c = c0 + 256 * u;
            if (c < a.C) {
                const float x = v[u] + b;
                if (a.scores) a.scores[s * a.score_stride + c] = x;
                amax_take(bv, bi, x, c);
            }
        }
    }
    if (!a.best_idx) return;
    amax_wave(bv, bi);
    __shared__ float sv[4];
    __shared__ int si[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) { sv[wave] = bv; si[wave] = bi; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 4; ++w) amax_take(bv, bi, sv[w], si[w]);
        a.best_idx[s] = (bi == AB_NONE) ? -1 : bi;
        if (a.best_score) a.best_score[s] = (bi == AB_NONE) ? __uint_as_float(0x7fc00000u) : bv;
    }
}

// The same for short rows (C <= 1024): a wavefront per scenario, four scenarios per work-group, no LDS
// and no barrier.  NT fixes the number of partial sums per candidate (one 4*NT-byte load each).
template <int NT>
__global__ __launch_bounds__(256) void finish_select_wave_kernel(const FinishArgs a, int64_t S)
{
    const int lane = threadIdx.x & 63;
    const int64_t s = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (s >= S) return;
    const float *p = a.partial + s * a.row_stride * NT;
    const float b = a.b_out ? a.b_out[0] : 0.f;
    float bv = -INFINITY;
    int bi = AB_NONE;
    {
        // four candidates of this lane at a time, their loads issued together
        typedef __attribute__((ext_vector_type(NT))) float vec_t;
        for (int c0 = lane; c0 < a.C; c0 += 256) {
            vec_t x[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int c = c0 + 64 * u;
                if (c < a.C) {
                    if constexpr (NT == 1) x[u] = vec_t(__builtin_nontemporal_load(p + c));
                    else x[u] = __builtin_nontemporal_load((const vec_t *)(p + (int64_t)c * NT));
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int c = c0 + 64 * u;
                if (c < a.C) {
                    float v = x[u][0];
#pragma unroll
                    for (int t = 1; t < NT; ++t) v += x[u][t];
                    v += b;
                    if (a.scores) a.scores[s * a.score_stride + c] = v;
                    amax_take(bv, bi, v, c);
                }
            }
        }
    }
    if (!a.best_idx) return;
    amax_wave(bv, bi);
    if (lane == 0) {
        a.best_idx[s] = (bi == AB_NONE) ? -1 : bi;
        if (a.best_score) a.best_score[s] = (bi == AB_NONE) ? __uint_as_float(0x7fc00000u) : bv;
    }
}

// Plain argmax over stored rows (C <= 1024, a multiple of 4, 16-byte aligned rows): sixteen lanes per
// scenario, four scenarios per wavefront, all of a lane's 16-byte loads issued up front; the lanes of a
// row of sixteen combine through four DPP exchanges (no LDS).
template <int NLOAD>
__global__ __launch_bounds__(256) void select_rows16_kernel(const FinishArgs a, int64_t S)
{
    const int l16 = threadIdx.x & 15;
    const int64_t s = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
    const bool live = s < S;
    const float *p = a.partial + (live ? s : 0) * a.row_stride;
    f32x4 x[NLOAD];
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) {
        const int c = (i * 16 + l16) * 4;
        x[i] = (live && c < a.C) ? __builtin_nontemporal_load((const f32x4 *)(p + c))
                                 : f32x4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
    }
    float bv = -INFINITY;
    int bi = AB_NONE;
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) {
        const int c = (i * 16 + l16) * 4;
#pragma unroll
        for (int e = 0; e < 4; ++e) if (c < a.C) amax_take(bv, bi, x[i][e], c + e);
    }
    amax_dpp<0xB1>(bv, bi);      // lanes ^ 1   (quad_perm 1,0,3,2)
    amax_dpp<0x4E>(bv, bi);      // lanes ^ 2   (quad_perm 2,3,0,1)
    amax_dpp<0x141>(bv, bi);     // the other quad of the half row (row_half_mirror)
    amax_dpp<0x140>(bv, bi);     // the other half of the row (row_mirror)
    if (live && l16 == 0) {
        a.best_idx[s] = (bi == AB_NONE) ? -1 : bi;
        if (a.best_score) a.best_score[s] = (bi == AB_NONE) ? __uint_as_float(0x7fc00000u) : bv;
    }
}

// ------------------------------------------------------------------------------------------------
// The whole pass in one launch for the size the paper runs it at (one job, tens of candidates, a small
// scorer; Section 3.3 "Meta network optimizer"): at that size the chain of launches of the batched path
// costs more than the arithmetic.  One work-group per scenario:
//   transformed features -> LDS; scenario term A[j] = W1[j, :Fs] x + b1[j] (a wavefront per output,
//   lanes over the inputs); then 64 candidates at a time, a candidate per lane and a sixteenth of a layer's
//   outputs per wavefront: h1 = relu(A + wp phi(S_p) + wc phi(S_c)), the further layers as dot products
//   whose weights are staged in LDS (wave-uniform broadcast reads) against the candidate's activations
//   (read once per layer into registers from LDS rows of stride H + 4 floats: no bank conflicts), the output unit, and
//   the running argmax.  With bf16 as compute type the values the batched path keeps in memory in bf16 (the
//   scenario's features, every hidden activation but the last layer's) are rounded to bf16 here too, so a
//   model scores the same whichever path a call takes.
// ------------------------------------------------------------------------------------------------
struct TinyArgs {
    const float *dyn, *scal, *part, *cred;
    int32_t part_stride, cred_stride;            // elements between two scenarios' grids (0: one shared grid)
    int32_t L, K, Ns, Q, C, F, Fs, D;
    int32_t H[AB_MAX_HIDDEN];
    const void *W[AB_MAX_HIDDEN + 1];
    const float *b[AB_MAX_HIDDEN + 1];
    ab_enc enc_stat[AB_MAX_STATS], enc_scalar[AB_MAX_SCALARS], enc_part, enc_cred;
    float *scores; int32_t *best_idx; float *best_score;
};

template <typename T>
__device__ __forceinline__ float as_stored(float v)        // what a value becomes when kept in the compute type
{
    if constexpr (sizeof(T) == 2) return bf16_bits_to_f32(pack_bf16x2(v, 0.f) & 0xffffu);
    else return v;
}

// One work-group = one scenario = one CU, so the kernel is a chain of short stages and its time is the sum of
// their latencies.  What does not depend on an earlier stage is done at the start (transformed grid values,
// hidden biases and the output unit -> LDS, each by a thread of its own instead of once per wavefront), and
// the hidden layers run on the matrix cores in fp32: 16 x 16 output blocks (outputs x candidates), one or two
// per wavefront, operands read from LDS as 16-byte pieces with one K order for both sides (piece q of a lane
// holds k = 16q + 4 (lane / 16) + e for the e-th instruction of the piece).
template <typename T>
__global__ __launch_bounds__(1024) void score_tiny_kernel(const TinyArgs a)
{
    constexpr int HM = 128, G = 64, STR = HM + 4, FS_MAX = 2048, NW = 16, CM = 256;   // sixteen wavefronts
    __shared__ float xs[FS_MAX];
    __shared__ float A1[HM], wp[HM], wc[HM];
    __shared__ __attribute__((aligned(16))) float b_s[AB_MAX_HIDDEN - 1][HM];   // biases of the hidden layers after the first
    __shared__ float wo_s[HM + 1];                                        // output unit: weights, then its bias
    __shared__ float xp_s[CM], xc_s[CM];                                  // transformed grid values per candidate
    __shared__ float red[NW][G];
    extern __shared__ __attribute__((aligned(16))) float tiny_dyn[];      // two activation buffers, one weight matrix
    float (*hb)[G * STR] = (float (*)[G * STR])tiny_dyn;
    float *w_lds = tiny_dyn + 2 * G * STR;                                // rows of hin + 4 floats
    const int64_t s = blockIdx.x;
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int hl = a.H[a.D - 1];

    auto load_w4 = [&](const void *W, int e) {                 // four adjacent weights as fp32
        if constexpr (sizeof(T) == 2) {
            const uint2 r = *(const uint2 *)((const uint16_t *)W + e);
            return f32x4{__uint_as_float(r.x << 16), __uint_as_float(r.x & 0xffff0000u),
                         __uint_as_float(r.y << 16), __uint_as_float(r.y & 0xffff0000u)};
        } else {
            return *(const f32x4 *)((const float *)W + e);
        }
    };
    auto park_w4 = [&](int hin, int e, f32x4 w) {              // ... to their place in the padded LDS rows
        const int j = hin == 64 ? e >> 6 : e >> 7;
        *(f32x4 *)(w_lds + j * (hin + 4) + (e & (hin - 1))) = w;
    };

    // transformed statistics and scalars of the scenario (threads from the front), everything else that only
    // depends on the arguments (threads from the back); the raw statistics are requested first, the second
    // layer's weights and this wavefront's first layer-1 rows right behind them
    const int n_stat = a.L * a.K;
    const int H1 = a.H[0];
    const bool first_x = t < a.Fs;
    float raw0 = 0.f;
    if (first_x) raw0 = t < n_stat ? a.dyn[s * n_stat + t] : a.scal[s * a.Ns + (t - n_stat)];
    const int n_w1 = a.D > 1 ? a.H[1] * H1 : 0;
    f32x4 w_pre[4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
        if (t * 4 + u * 4096 < n_w1) w_pre[u] = load_w4(a.W[1], t * 4 + u * 4096);
    float w0_pre[4] = {0.f, 0.f, 0.f, 0.f};
    if (wave * 4 < H1 && lane < a.Fs) {
#pragma unroll
        for (int u = 0; u < 4; ++u) w0_pre[u] = load_as_f32<T>(a.W[0], (int64_t)(wave * 4 + u) * a.F + lane);
    }
    if (first_x) xs[t] = as_stored<T>(phi(raw0, t < n_stat ? a.enc_stat[t % a.K] : a.enc_scalar[t - n_stat]));
    for (int i = t + 64 * NW; i < a.Fs; i += 64 * NW)
        xs[i] = as_stored<T>(i < n_stat ? phi(a.dyn[s * n_stat + i], a.enc_stat[i % a.K])
                                        : phi(a.scal[s * a.Ns + (i - n_stat)], a.enc_scalar[i - n_stat]));
    {
        const int r = 64 * NW - 1 - t;
        if (r < a.C) xp_s[r] = phi(a.part[(int64_t)blockIdx.x * a.part_stride + r / a.Q], a.enc_part);
        else if (r >= CM && r - CM < a.C) xc_s[r - CM] = phi(a.cred[(int64_t)blockIdx.x * a.cred_stride + (r - CM) % a.Q], a.enc_cred);
        else if (r >= 2 * CM && r - 2 * CM <= hl)
            wo_s[r - 2 * CM] = r - 2 * CM < hl ? load_as_f32<T>(a.W[a.D], r - 2 * CM) : a.b[a.D][0];
        for (int q = t; q < (a.D - 1) * HM; q += 64 * NW) {
            const int k = 1 + q / HM, jx = q % HM;
            if (jx < a.H[k]) b_s[k - 1][jx] = a.b[k][jx];
        }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
        if (t * 4 + u * 4096 < n_w1) park_w4(H1, t * 4 + u * 4096, w_pre[u]);
    __syncthreads();
    // scenario term of layer 1 and its two configuration columns
    for (int j0 = wave * 4; j0 < H1; j0 += 4 * NW) {           // four outputs at a time: four loads in flight
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
        int i_from = lane;
        if (j0 == wave * 4 && lane < a.Fs) {                    // (the piece requested at the start)
            const float x = xs[lane];
#pragma unroll
            for (int u = 0; u < 4; ++u) acc[u] = w0_pre[u] * x;
            i_from = lane + 64;
        }
        for (int i = i_from; i < a.Fs; i += 64) {
            const float x = xs[i];
#pragma unroll
            for (int u = 0; u < 4; ++u) acc[u] = fmaf(load_as_f32<T>(a.W[0], (int64_t)(j0 + u) * a.F + i), x, acc[u]);
        }
        float mine = 0.f, mp = 0.f, mc = 0.f;                  // (requested before the sums are formed)
        if (lane < 4) {
            const int j = j0 + lane;
            mine = a.b[0][j];
            mp = load_as_f32<T>(a.W[0], (int64_t)j * a.F + a.Fs);
            mc = load_as_f32<T>(a.W[0], (int64_t)j * a.F + a.Fs + 1);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) acc[u] = wave_sum(acc[u]);
        if (lane < 4) {
            const int j = j0 + lane;
            const float av = lane == 0 ? acc[0] : lane == 1 ? acc[1] : lane == 2 ? acc[2] : acc[3];
            A1[j] = av + mine;
            wp[j] = mp;
            wc[j] = mc;
        }
    }
    __syncthreads();

    float bv = -INFINITY;
    int bi = AB_NONE;
    for (int c0 = 0; c0 < a.C; c0 += G) {
        const int c = c0 + lane;
        const int cc = c < a.C ? c : a.C - 1;
        const float xp = xp_s[cc], xc = xc_s[cc];
        {
            float *mine = &hb[0][lane * STR];
            const int hq = H1 / NW;
            for (int jj = 0; jj < hq; ++jj) {
                const int j = wave * hq + jj;
                const float h = relu_keep_nan(fmaf(wc[j], xc, fmaf(wp[j], xp, A1[j])));
                mine[j] = a.D > 1 ? as_stored<T>(h) : h;
            }
        }
        int cur = 0;
        for (int k = 1; k < a.D; ++k) {
            const int hin = a.H[k - 1], hout = a.H[k], ws = hin + 4;
            // the layer's weights -> LDS as fp32, once the layer before has read its own (the last layer of the
            // group before is behind the output unit's barriers); the second layer's are there from the start
            // and, being the only ones, stay for every group of candidates
            if (k > 1) __syncthreads();
            if (!(k == 1 && (c0 == 0 || a.D == 2))) {           // (the second layer's were parked at the start)
                for (int e = t * 4; e < hout * hin; e += 256 * NW) park_w4(hin, e, load_w4(a.W[k], e));
            }
            __syncthreads();                                    // weights and the layer's inputs are in place
            const bool keep = k == a.D - 1;                     // the last hidden layer is not kept in the compute type
            for (int blk = wave; blk < 4 * (hout >> 4); blk += NW) {
                const int cb = blk & 3, ob = blk >> 2;
                const int row = lane & 15, kq = (lane >> 4) * 4;
                const float *pw = w_lds + (16 * ob + row) * ws + kq;
                const float *ph = &hb[cur][(16 * cb + row) * STR + kq];
                f32x4 acc = *(const f32x4 *)&b_s[k - 1][16 * ob + kq];     // lane: outputs 16 ob + kq .. + 3 of candidate 16 cb + row
                for (int q = 0; q < hin; q += 16) {
                    const f32x4 wv = *(const f32x4 *)(pw + q), hv = *(const f32x4 *)(ph + q);
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(wv.x, hv.x, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(wv.y, hv.y, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(wv.z, hv.z, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(wv.w, hv.w, acc, 0, 0, 0);
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float v = relu_keep_nan(acc[e]);
                    acc[e] = keep ? v : as_stored<T>(v);
                }
                *(f32x4 *)&hb[cur ^ 1][(16 * cb + row) * STR + 16 * ob + kq] = acc;
            }
            cur ^= 1;
        }
        __syncthreads();
        {   // output unit: each wavefront its share of the dot product
            const int hq = hl / NW;
            const float *src = &hb[cur][lane * STR + wave * hq];
            const float *wo = wo_s + wave * hq;
            float acc = 0.f;
            for (int i = 0; i < hq; i += 4) {
                const f32x4 h = *(const f32x4 *)(src + i);
                acc = fmaf(wo[i + 3], h.w, fmaf(wo[i + 2], h.z, fmaf(wo[i + 1], h.y, fmaf(wo[i], h.x, acc))));
            }
            red[wave][lane] = acc;
        }
        __syncthreads();
        if (wave == 0 && c < a.C) {
            float v = wo_s[hl];
#pragma unroll
            for (int w = 0; w < NW; ++w) v += red[w][lane];
            if (a.scores) a.scores[s * a.C + c] = v;
            amax_take(bv, bi, v, c);
        }
        // (the next group's first writes go to hb[0]: its last readers, the first hidden layer's matrix
        // instructions or the output unit, are behind a barrier; red is rewritten two barriers later)
    }
    if (wave == 0 && a.best_idx) {
        amax_wave(bv, bi);
        if (lane == 0) {
            a.best_idx[s] = (bi == AB_NONE) ? -1 : bi;
            if (a.best_score) a.best_score[s] = (bi == AB_NONE) ? __uint_as_float(0x7fc00000u) : bv;
        }
    }
}

// Optimization Trigger (Section 3.3): argmax of a stored score row, relative gain over the configuration in
// use, and the two threshold tests.  One work-group per scenario; IEEE single precision throughout.
struct TriggerArgs {
    const float *scores; int64_t row_stride; int32_t C;
    const int32_t *cur_idx; const float *observed;
    float gain_threshold, error_threshold;
    int32_t *best_idx; float *gain; uint8_t *reconf; uint8_t *adapt;
};

__global__ __launch_bounds__(256) void trigger_kernel(const TriggerArgs a)
{
    const int64_t s = blockIdx.x;
    const float *p = a.scores + s * a.row_stride;
    float bv = -INFINITY;
    int bi = AB_NONE;
    for (int c = threadIdx.x; c < a.C; c += 256) amax_take(bv, bi, p[c], c);
    amax_wave(bv, bi);
    __shared__ float sv[4];
    __shared__ int si[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) { sv[wave] = bv; si[wave] = bi; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 4; ++w) amax_take(bv, bi, sv[w], si[w]);
        const bool has_best = bi != AB_NONE;
        a.best_idx[s] = has_best ? bi : -1;
        const int ci = a.cur_idx[s];
        const bool cur_ok = ci >= 0 && ci < a.C;
        const float nan = __uint_as_float(0x7fc00000u);
        const float vc = cur_ok ? p[ci] : nan;
        float g = nan;
        if (has_best && cur_ok) g = (bv - vc) / fabsf(vc);
        if (a.gain) a.gain[s] = g;
        a.reconf[s] = (uint8_t)(g >= a.gain_threshold);
        if (a.adapt) {
            float e = nan;
            if (a.observed && cur_ok) e = fabsf(vc - a.observed[s]) / fabsf(a.observed[s]);
            a.adapt[s] = (uint8_t)(e > a.error_threshold);
        }
    }
}

// Scorer with a single hidden layer: score = w_out . relu(A[s] + B[c]) + b_out, one wavefront per
// (scenario, candidate) row, written into the same partial buffer layout (nt = 1, no bias yet).
struct ScoreD1Args {
    const float *a_term, *b_term, *w_out_f; float *partial; int64_t rows; int32_t C, H;
    const float *wp, *wc, *xp_row, *xc_row;      // xp_row != NULL: B = wp * xp_row[row] + wc * xc_row[row] instead of b_term[c]
};
__global__ __launch_bounds__(256) void score_single_hidden_kernel(const ScoreD1Args a)
{
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= a.rows) return;
    const int lane = threadIdx.x & 63;
    const int64_t s = row / a.C;
    const int c = (int)(row - s * a.C);
    float acc = 0.f;
    if (a.xp_row) {
        const float xp = a.xp_row[row], xc = a.xc_row[row];
        for (int h = lane; h < a.H; h += 64)
            acc += relu_keep_nan(fmaf(a.wc[h], xc, fmaf(a.wp[h], xp, a.a_term[s * a.H + h]))) * a.w_out_f[h];
    } else {
        for (int h = lane; h < a.H; h += 64)
            acc += relu_keep_nan(a.a_term[s * a.H + h] + a.b_term[(int64_t)c * a.H + h]) * a.w_out_f[h];
    }
    acc = wave_sum(acc);
    if (lane == 0) a.partial[row] = acc;
}

// ------------------------------------------------------------------------------------------------
// Shared per-tensor encoder (Section 3.1 "Meta network architecture": the layer-wise statistics are
// embedded into a fixed-dimension feature space so that models with different layer counts can be
// handled).  A work-group takes scenarios blockIdx.x, blockIdx.x + gridDim.x, ... (two work-groups per CU):
//   e[l] = relu(W_b relu(W_a phi(stat[l]) + b_a) + b_b)   (K -> 128 on the vector ALUs, 128 -> 128 on
//   the matrix cores), pooled[s] = mean_l e[l], written as the first 128 columns of the scenario row.
// W_b (bf16, 32 KB) is staged once per work-group in LDS.  After that the four wavefronts work on
// their own 32-tensor blocks without meeting, each block's raw statistics fetched while the block before
// is computed: a wavefront transforms its block's statistics, runs
// the first layer (a lane owns two of the 128 units, weights in registers), parks the bf16 result in
// its private 8 KB of LDS, multiplies it with W_b (32 matrix instructions) and adds relu(. + b_b) of the
// valid tensors to per-lane column sums.  One reduction over the wavefronts at the end.
// LDS rows are 256 bytes; 16-byte chunk c of row r sits at position c ^ (r & 15).
// Both layers' products use bf16 operands with fp32 accumulation.
// ------------------------------------------------------------------------------------------------
struct TensorEncArgs {
    const float *dyn; int32_t L, K;
    const void *Wa; const float *ba;     // [128, K]
    const void *Wb; const float *bb;     // [128, 128]
    void *xs; int32_t ld;                // scenario rows; columns [0,128) written here
    const int32_t *layers_of;            // [S] or NULL: layers the scenario really has (clamped to [1, L])
    int64_t S;
    ab_enc enc_stat[AB_MAX_ENCODER_STATS];
};

template <typename T>
__global__ __launch_bounds__(256) void tensor_encoder_kernel(const TensorEncArgs a)
{
    constexpr int H = 128;
    __shared__ __attribute__((aligned(16))) unsigned char wb_s[H * 256];        // W_b, bf16, swizzled rows
    __shared__ __attribute__((aligned(16))) unsigned char hbuf[4][32 * 256];    // per wavefront: 32 tensors x 128 bf16
    __shared__ __attribute__((aligned(16))) float xin[4][32 * AB_MAX_ENCODER_STATS];    // per wavefront: transformed statistics
    __shared__ __attribute__((aligned(16))) float wa_s[H * AB_MAX_ENCODER_STATS];       // [unit][AB_MAX_ENCODER_STATS], zero padded
    __shared__ float ba_s[H];
    __shared__ float red[4][H];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, half = lane >> 5, l31 = lane & 31;
    auto layers = [&](int64_t sc) {                        // a scenario's own layer count
        int n = a.L;
        if (a.layers_of) { n = a.layers_of[sc]; n = n < 1 ? 1 : (n > a.L ? a.L : n); }
        return n;
    };

    for (int i = t; i < H * AB_MAX_ENCODER_STATS; i += 256) {
        const int o = i / AB_MAX_ENCODER_STATS, k = i % AB_MAX_ENCODER_STATS;
        wa_s[i] = (k < a.K) ? load_as_f32<T>(a.Wa, o * a.K + k) : 0.f;
    }
    if (t < H) ba_s[t] = a.ba[t];
    for (int i = t; i < H * 16; i += 256) {                 // 16-byte chunks of W_b
        const int n = i >> 4, c = i & 15;
        i32x4 v;
        if constexpr (sizeof(T) == 2) {
            v = *(const i32x4 *)((const uint16_t *)a.Wb + n * H + c * 8);
        } else {
            const float *w = (const float *)a.Wb + n * H + c * 8;
            v.x = (int)pack_bf16x2(w[0], w[1]); v.y = (int)pack_bf16x2(w[2], w[3]);
            v.z = (int)pack_bf16x2(w[4], w[5]); v.w = (int)pack_bf16x2(w[6], w[7]);
        }
        *(i32x4 *)(wb_s + n * 256 + ((c ^ (n & 15)) << 4)) = v;
    }
    __syncthreads();

    float bb[4], colsum[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int jn = 0; jn < 4; ++jn) bb[jn] = a.bb[jn * 32 + l31];
    unsigned char *hb = hbuf[wave];
    float *xw = xin[wave];
    float wa0[AB_MAX_ENCODER_STATS], wa1[AB_MAX_ENCODER_STATS];             // first layer: rows 2*lane and 2*lane+1 of W_a
#pragma unroll
    for (int k = 0; k < AB_MAX_ENCODER_STATS; ++k) {
        wa0[k] = wa_s[(2 * lane) * AB_MAX_ENCODER_STATS + k];
        wa1[k] = wa_s[(2 * lane + 1) * AB_MAX_ENCODER_STATS + k];
    }
    const float ba0 = ba_s[2 * lane], ba1 = ba_s[2 * lane + 1];

    // this lane's slots of a block's statistics: element i = lane + 64 j of [32 tensors][AB_MAX_ENCODER_STATS], i.e.
    // tensor (lane >> 3) + 8 j, statistic lane & 7 (the same statistic for all four: one transform)
    const int my_k = lane & (AB_MAX_ENCODER_STATS - 1);
    const ab_enc my_enc = a.enc_stat[my_k];
    auto fetch_raw = [&](int64_t sc, int n_layers, int l0, float (&raw)[4]) {
        const float *dyn = a.dyn + sc * (int64_t)a.L * a.K;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int l = l0 + (lane >> 3) + 8 * j;
            raw[j] = (sc < a.S && l < n_layers && my_k < a.K) ? dyn[(int64_t)l * a.K + my_k] : 1.f;
        }
    };

    int64_t sc = blockIdx.x;
    int Ls = sc < a.S ? layers(sc) : 0;
    int l0 = wave * 32;
    float raw[4];
    fetch_raw(sc, Ls, l0, raw);
    for (; sc < a.S; ) {
      const bool has_block = l0 < Ls;                        // (its last block fetches the next scenario's first)
      for (; l0 < Ls; ) {
        // the block after this one (of this scenario, or the first of this wavefront in the next scenario)
        int64_t sc_n = sc;
        int Ls_n = Ls, l0_n = l0 + 128;
        if (l0_n >= Ls) { sc_n = sc + gridDim.x; Ls_n = sc_n < a.S ? layers(sc_n) : 0; l0_n = wave * 32; }
        float raw_n[4];
        fetch_raw(sc_n, Ls_n, l0_n, raw_n);
        // transformed statistics of the block's 32 tensors (zero rows past the end)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int l = l0 + (lane >> 3) + 8 * j;
            float lg;
            if constexpr (sizeof(T) == 2) lg = __builtin_amdgcn_logf(raw[j]) * 0.69314718056f;
            else lg = logf(raw[j]);
            const float y = ((my_enc.kind == AB_ENC_LOG ? lg : raw[j]) - my_enc.shift) * my_enc.scale;
            xw[lane + 64 * j] = (l < Ls && my_k < a.K) ? y : 0.f;
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // same wavefront: LDS ops are in order
        // first layer: this lane owns units 2*lane and 2*lane+1 (weights in registers) for all 32 tensors;
        // a tensor's statistics are one broadcast LDS read, its two results one packed 4-byte write
#pragma unroll 8
        for (int r = 0; r < 32; ++r) {
            const f32x4 x0 = *(const f32x4 *)(xw + r * AB_MAX_ENCODER_STATS);
            float h0 = fmaf(wa0[3], x0.w, fmaf(wa0[2], x0.z, fmaf(wa0[1], x0.y, fmaf(wa0[0], x0.x, ba0))));
            float h1 = fmaf(wa1[3], x0.w, fmaf(wa1[2], x0.z, fmaf(wa1[1], x0.y, fmaf(wa1[0], x0.x, ba1))));
            if (a.K > 4) {
                const f32x4 x1 = *(const f32x4 *)(xw + r * AB_MAX_ENCODER_STATS + 4);
                h0 = fmaf(wa0[7], x1.w, fmaf(wa0[6], x1.z, fmaf(wa0[5], x1.y, fmaf(wa0[4], x1.x, h0))));
                h1 = fmaf(wa1[7], x1.w, fmaf(wa1[6], x1.z, fmaf(wa1[5], x1.y, fmaf(wa1[4], x1.x, h1))));
            }
            const uint32_t pk = pack_bf16x2(relu_keep_nan(h0), relu_keep_nan(h1));
            *(uint32_t *)(hb + r * 256 + (((lane >> 2) ^ (r & 15)) << 4) + (lane & 3) * 4) = pk;
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        f32x16 acc[4];
#pragma unroll
        for (int jn = 0; jn < 4; ++jn)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[jn][r] = 0.f;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int chunk = q * 2 + half;
            const i32x4 fa = *(const i32x4 *)(hb + l31 * 256 + ((chunk ^ (l31 & 15)) << 4));
#pragma unroll
            for (int jn = 0; jn < 4; ++jn) {
                const int n = jn * 32 + l31;
                const i32x4 fb = *(const i32x4 *)(wb_s + n * 256 + ((chunk ^ (n & 15)) << 4));
                // rows = tensors (first operand), columns = units (second operand)
                acc[jn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa),
                                                                  __builtin_bit_cast(bf16x8, fb), acc[jn], 0, 0, 0);
            }
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int l = l0 + (r >> 2) * 8 + half * 4 + (r & 3);
            if (l < Ls) {
#pragma unroll
                for (int jn = 0; jn < 4; ++jn) colsum[jn] += relu_keep_nan(acc[jn][r] + bb[jn]);
            }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // fragment reads done before the block buffer is reused
#pragma unroll
        for (int j = 0; j < 4; ++j) raw[j] = raw_n[j];
        l0 += 128;
      }
      // the scenario is complete for this wavefront: combine the four wavefronts' column sums
#pragma unroll
      for (int jn = 0; jn < 4; ++jn) {
          const float v = colsum[jn] + __shfl_xor(colsum[jn], 32, 64);
          if (half == 0) red[wave][jn * 32 + l31] = v;
          colsum[jn] = 0.f;
      }
      __syncthreads();
      if (t < H) {
          const float pooled = ((red[0][t] + red[1][t]) + (red[2][t] + red[3][t])) / (float)Ls;
          const int64_t o = sc * a.ld + t;
          if constexpr (sizeof(T) == 2) ((uint16_t *)a.xs)[o] = (uint16_t)(pack_bf16x2(pooled, 0.f) & 0xffffu);
          else ((float *)a.xs)[o] = pooled;
      }
      __syncthreads();                                       // `red` may be written again
      sc += gridDim.x;
      Ls = sc < a.S ? layers(sc) : 0;
      l0 = wave * 32;
      if (!has_block) fetch_raw(sc, Ls, l0, raw);
    }
}

// ------------------------------------------------------------------------------------------------
// host-side launch wrappers
// ------------------------------------------------------------------------------------------------
static inline unsigned blocks_for(int64_t n) { return (unsigned)((n + 255) / 256); }

static void fill_encode_args(EncodeArgs &a, const ab_model_desc *d, const float *dyn, const float *scal,
                             void *xs, int64_t S, int ld, int col0, int with_stats)
{
    a.dyn = dyn; a.scal = scal; a.xs = xs; a.S = S; a.ld = ld; a.col0 = col0;
    a.n_stat = with_stats ? d->n_layers * d->n_stats : 0;
    a.n_stats_per_layer = d->n_stats; a.n_scal = d->n_scalars;
    for (int i = 0; i < AB_MAX_STATS; ++i) a.enc_stat[i] = d->enc_stat[i];
    for (int i = 0; i < AB_MAX_SCALARS; ++i) a.enc_scal[i] = d->enc_scalar[i];
}

// Whether the four-columns-per-thread form of the transform takes this layout; fills its index constants.
static bool quad_split(int dtype, const ab_model_desc *d, const EncodeArgs &a, QuadSplit &g)
{
    const int width = a.ld - a.col0;
    if (!(width % 4 == 0 && a.col0 % 4 == 0 && a.n_stat % 4 == 0 && a.n_stat != 4 && width - a.n_stat >= 8 &&
          width / 4 < 65536 && ((uintptr_t)a.dyn & 15) == 0 && ((uintptr_t)a.xs & 15) == 0 &&
          (a.ld * elem_size(dtype)) % 16 == 0))
        return false;
    // magic = floor(2^32 / n) + 1 turns index / n into a multiply-high, exact while index * n < 2^32
    auto magic = [](int n) { return n >= 2 ? (uint32_t)(0x100000000ull / (uint32_t)n) + 1u : 0u; };
    g.q4s = a.n_stat / 4; g.q4t = (width - a.n_stat) / 4;
    g.rpb = width / 4 >= 1792 ? 1 : 1792 / (width / 4);      // seven quads per thread (measured: 1000-2000 quads per
                                                             // work-group are alike, more are slower)
    g.magic_q4s = magic(g.q4s); g.magic_q4t = magic(g.q4t); g.magic_k = magic(d->n_stats);
    return true;
}

hipError_t launch_encode_stats(int dtype, const ab_model_desc *d, const float *dyn, const float *scal,
                               void *xs, int64_t S, int ld, int col0, int with_stats, hipStream_t st)
{
    if (S == 0) return hipSuccess;
    EncodeArgs a;
    fill_encode_args(a, d, dyn, scal, xs, S, ld, col0, with_stats);
    const int width = ld - col0;
    QuadSplit g;
    if (quad_split(dtype, d, a, g)) {
        const unsigned blocks = (unsigned)((S + g.rpb - 1) / g.rpb);
        if (dtype == AB_BF16) encode_stats_quad_kernel<bf16_t><<<blocks, 256, 0, st>>>(a, g);
        else encode_stats_quad_kernel<float><<<blocks, 256, 0, st>>>(a, g);
        return hipGetLastError();
    }
    const int64_t n = S * (width / 2);
    if (dtype == AB_BF16) encode_stats_kernel<bf16_t><<<blocks_for(n), 256, 0, st>>>(a);
    else encode_stats_kernel<float><<<blocks_for(n), 256, 0, st>>>(a);
    return hipGetLastError();
}

static int64_t fill_prep_args(PrepArgs &a, const ab_model_desc *d, const void *W1, const float *b1, int F, int Fs,
                              int H1, int ld, void *w1s, const ab_grid *grid, float *b_term, float *cfg_vec,
                              const void *Wout, const float *b_out, int H_last, float *w_out_f);

hipError_t launch_prep_layer1(int dtype, const ab_model_desc *d, const void *W1, const float *b1, int F, int Fs,
                              int H1, int ld, void *w1s, const ab_grid *grid, float *b_term, float *cfg_vec,
                              const void *Wout, const float *b_out, int H_last, float *w_out_f, hipStream_t st)
{
    PrepArgs a;
    const int64_t n = fill_prep_args(a, d, W1, b1, F, Fs, H1, ld, w1s, grid, b_term, cfg_vec, Wout, b_out, H_last, w_out_f);
    if (dtype == AB_BF16) prep_layer1_kernel<bf16_t><<<blocks_for(n), 256, 0, st>>>(a);
    else prep_layer1_kernel<float><<<blocks_for(n), 256, 0, st>>>(a);
    return hipGetLastError();
}

// Transform of the flat model's statistics and layer-1 preparation in one launch.  *done = false (and nothing
// launched) when the layout needs the general form of the transform; the caller then makes the two launches.
hipError_t launch_encode_and_prep(int dtype, const ab_model_desc *d, const float *dyn, const float *scal, void *xs,
                                  int64_t S, int ld, const void *W1, const float *b1, int F, int Fs, int H1, void *w1s,
                                  const ab_grid *grid, float *b_term, float *cfg_vec, const void *Wout,
                                  const float *b_out, int H_last, float *w_out_f, bool *done, hipStream_t st)
{
    *done = false;
    if (S == 0) return hipSuccess;
    EncodeArgs a;
    fill_encode_args(a, d, dyn, scal, xs, S, ld, 0, 1);
    QuadSplit g;
    if (!quad_split(dtype, d, a, g)) return hipSuccess;
    PrepArgs p;
    const int64_t n = fill_prep_args(p, d, W1, b1, F, Fs, H1, ld, w1s, grid, b_term, cfg_vec, Wout, b_out, H_last, w_out_f);
    const int64_t enc_blocks = (S + g.rpb - 1) / g.rpb, prep_blocks = (n + 255) / 256;
    if (enc_blocks + prep_blocks > 0x7fffffffLL) return hipSuccess;
    *done = true;
    if (dtype == AB_BF16)
        encode_and_prep_kernel<bf16_t><<<(unsigned)(enc_blocks + prep_blocks), 256, 0, st>>>(a, g, p, (unsigned)enc_blocks);
    else
        encode_and_prep_kernel<float><<<(unsigned)(enc_blocks + prep_blocks), 256, 0, st>>>(a, g, p, (unsigned)enc_blocks);
    return hipGetLastError();
}

static int64_t fill_prep_args(PrepArgs &a, const ab_model_desc *d, const void *W1, const float *b1, int F, int Fs,
                              int H1, int ld, void *w1s, const ab_grid *grid, float *b_term, float *cfg_vec,
                              const void *Wout, const float *b_out, int H_last, float *w_out_f)
{
    a.W1 = W1; a.F = F; a.Fs = Fs; a.H1 = H1; a.ld = ld; a.w1s = w1s; a.b1 = b1;
    a.part = grid->partition_bytes; a.cred = grid->credit_mult; a.P = grid->P; a.Q = grid->Q;
    a.enc_part = d->enc_partition; a.enc_cred = d->enc_credit; a.b_term = b_term;
    const int Cn = grid->P * grid->Q;
    a.wp_f = cfg_vec; a.wc_f = cfg_vec + H1; a.xp_f = cfg_vec + 2 * H1; a.xc_f = cfg_vec + 2 * H1 + Cn;
    a.Wout = Wout; a.b_out = b_out; a.H_last = H_last; a.n_out = d->n_outputs > 1 ? d->n_outputs : 1; a.w_out_f = w_out_f;
    return (int64_t)H1 * ld + (int64_t)Cn * H1 + H_last + H1 + Cn;
}

hipError_t launch_finish_select(const float *partial, int nt, int64_t row_stride, const float *b_out,
                                float *scores, int64_t score_stride, int32_t *best_idx, float *best_score,
                                int64_t S, int C, hipStream_t st)
{
    if (S == 0) return hipSuccess;
    FinishArgs a;
    a.partial = partial; a.nt = nt; a.row_stride = row_stride; a.b_out = b_out; a.scores = scores;
    a.score_stride = score_stride; a.best_idx = best_idx; a.best_score = best_score; a.C = C;
    const unsigned wave_blocks = (unsigned)((S + 3) / 4);
    if (C <= 1024 && nt == 1 && !b_out && !scores && best_idx && C % 4 == 0 && row_stride % 4 == 0 &&
        ((uintptr_t)partial & 15) == 0) {
        const unsigned blocks = (unsigned)((S + 15) / 16);
        if (C <= 256) select_rows16_kernel<4><<<blocks, 256, 0, st>>>(a, S);
        else if (C <= 512) select_rows16_kernel<8><<<blocks, 256, 0, st>>>(a, S);
        else select_rows16_kernel<16><<<blocks, 256, 0, st>>>(a, S);
    } else if (C <= 1024 && nt == 1)
        finish_select_wave_kernel<1><<<wave_blocks, 256, 0, st>>>(a, S);
    else if (C <= 1024 && nt == 2 && ((uintptr_t)partial & 7) == 0)
        finish_select_wave_kernel<2><<<wave_blocks, 256, 0, st>>>(a, S);
    else if (C <= 1024 && nt == 4 && ((uintptr_t)partial & 15) == 0)
        finish_select_wave_kernel<4><<<wave_blocks, 256, 0, st>>>(a, S);
    else
        finish_select_kernel<<<(unsigned)S, 256, 0, st>>>(a);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// A scorer without hidden layers (Section 3.1 leaves the depth open; with none the network is the linear map
// V = W x + b): a candidate's score is  mean_o W[o, :Fs] . x_s + mean_o b[o]  +  wp phi(S_p) + wc phi(S_c),
// wp / wc the means of W's two configuration columns.  One work-group per scenario: its wavefronts share the
// dot product over the transformed statistics (values kept as the compute type keeps them), then every thread
// takes candidates.  With v_out the per-output dot products of the chosen candidate are written as well.
// ------------------------------------------------------------------------------------------------
struct LinearArgs {
    const float *dyn, *scal, *part, *cred; int32_t part_stride, cred_stride;
    int32_t n_stat, K, Ns, Q, C, F, n_out;
    const void *W; const float *b;
    ab_enc enc_stat[AB_MAX_STATS], enc_scalar[AB_MAX_SCALARS], enc_part, enc_cred;
    float *scores; int32_t *best_idx; float *best_score; float *v_best;
};

template <typename T>
__global__ __launch_bounds__(256) void score_linear_kernel(const LinearArgs a)
{
    __shared__ float red[4][AB_MAX_OUTPUTS + 2];
    __shared__ float sv[4];
    __shared__ int si[4];
    const int64_t s = blockIdx.x;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int Fs = a.n_stat + a.Ns;
    // per output: the dot product over the statistics block and the scalars
    float acc[AB_MAX_OUTPUTS];
#pragma unroll
    for (int o = 0; o < AB_MAX_OUTPUTS; ++o) acc[o] = 0.f;
    for (int j = t; j < Fs; j += 256) {
        float x = j < a.n_stat ? phi(a.dyn[s * a.n_stat + j], a.enc_stat[j % a.K])
                               : phi(a.scal[s * a.Ns + (j - a.n_stat)], a.enc_scalar[j - a.n_stat]);
        x = as_stored<T>(x);
#pragma unroll
        for (int o = 0; o < AB_MAX_OUTPUTS; ++o)
            if (o < a.n_out) acc[o] = fmaf(load_as_f32<T>(a.W, (int64_t)o * a.F + j), x, acc[o]);
    }
#pragma unroll
    for (int o = 0; o < AB_MAX_OUTPUTS; ++o) {
        if (o < a.n_out) {
            const float v = wave_sum(acc[o]);
            if (lane == 0) red[wave][o] = v;
        }
    }
    __syncthreads();
    float a0 = 0.f, wp = 0.f, wc = 0.f;                    // folded over the outputs: mean of the rows, mean of the biases
    for (int o = 0; o < a.n_out; ++o) {
        a0 += ((red[0][o] + red[1][o]) + (red[2][o] + red[3][o])) + a.b[o];
        wp += load_as_f32<T>(a.W, (int64_t)o * a.F + Fs);
        wc += load_as_f32<T>(a.W, (int64_t)o * a.F + Fs + 1);
    }
    const float inv = 1.f / (float)a.n_out;
    a0 *= inv; wp *= inv; wc *= inv;
    const float *part = a.part + s * a.part_stride, *cred = a.cred + s * a.cred_stride;
    float bv = -INFINITY;
    int bi = AB_NONE;
    for (int c = t; c < a.C; c += 256) {
        const float xp = phi(part[c / a.Q], a.enc_part), xc = phi(cred[c % a.Q], a.enc_cred);
        const float v = fmaf(wc, xc, fmaf(wp, xp, a0));
        if (a.scores) a.scores[s * a.C + c] = v;
        amax_take(bv, bi, v, c);
    }
    if (!a.best_idx) return;
    amax_wave(bv, bi);
    if (lane == 0) { sv[wave] = bv; si[wave] = bi; }
    __syncthreads();
    for (int w = 0; w < 4; ++w) if (w != wave) amax_take(bv, bi, sv[w], si[w]);     // every thread ends with the block's choice
    if (t == 0) {
        a.best_idx[s] = (bi == AB_NONE) ? -1 : bi;
        if (a.best_score) a.best_score[s] = (bi == AB_NONE) ? __uint_as_float(0x7fc00000u) : bv;
    }
    if (a.v_best && t < a.n_out) {
        float v = __uint_as_float(0x7fc00000u);
        if (bi != AB_NONE) {
            const float xp = phi(part[bi / a.Q], a.enc_part), xc = phi(cred[bi % a.Q], a.enc_cred);
            const float d = ((red[0][t] + red[1][t]) + (red[2][t] + red[3][t])) + a.b[t];
            v = fmaf(load_as_f32<T>(a.W, (int64_t)t * a.F + Fs + 1), xc, fmaf(load_as_f32<T>(a.W, (int64_t)t * a.F + Fs), xp, d));
        }
        a.v_best[s * a.n_out + t] = v;
    }
}

hipError_t launch_score_linear(int dtype, const ab_model_desc *d, const ab_params *prm, const float *dyn,
                               const float *scal, const ab_grid *grid, int64_t S, float *scores, int32_t *best_idx,
                               float *best_score, float *v_best, hipStream_t st)
{
    if (S == 0) return hipSuccess;
    if (S > 0x7fffffffLL) return hipErrorInvalidValue;
    LinearArgs a = {};
    a.dyn = dyn; a.scal = scal; a.part = grid->partition_bytes; a.cred = grid->credit_mult;
    a.part_stride = grid->per_scenario ? grid->P : 0; a.cred_stride = grid->per_scenario ? grid->Q : 0;
    a.n_stat = d->n_layers * d->n_stats; a.K = d->n_stats; a.Ns = d->n_scalars; a.Q = grid->Q; a.C = grid->P * grid->Q;
    a.F = a.n_stat + a.Ns + 2; a.n_out = d->n_outputs > 1 ? d->n_outputs : 1;
    a.W = prm->W[0]; a.b = prm->b[0];
    for (int i = 0; i < AB_MAX_STATS; ++i) a.enc_stat[i] = d->enc_stat[i];
    for (int i = 0; i < AB_MAX_SCALARS; ++i) a.enc_scalar[i] = d->enc_scalar[i];
    a.enc_part = d->enc_partition; a.enc_cred = d->enc_credit;
    a.scores = scores; a.best_idx = best_idx; a.best_score = best_score; a.v_best = v_best;
    if (dtype == AB_BF16) score_linear_kernel<bf16_t><<<(unsigned)S, 256, 0, st>>>(a);
    else                  score_linear_kernel<float><<<(unsigned)S, 256, 0, st>>>(a);
    return hipGetLastError();
}

bool score_tiny_supported(const ab_model_desc *d, int64_t S, int32_t C)
{
    if (d->tensor_encoder || d->n_hidden < 1 || d->n_outputs > 1) return false;
    for (int k = 0; k < d->n_hidden; ++k) if (d->hidden[k] > 128) return false;     // (multiples of 64 already)
    const int64_t Fs = (int64_t)d->n_layers * d->n_stats + d->n_scalars;
    return Fs <= 2048 && C <= 256 && S >= 1 && S * C <= 16384;
}

hipError_t launch_score_tiny(int dtype, const ab_model_desc *d, const ab_params *prm, const float *dyn,
                             const float *scal, const float *part, const float *cred, int32_t P, int32_t Q,
                             int per_scenario, int64_t S, float *scores, int32_t *best_idx, float *best_score,
                             hipStream_t st)
{
    TinyArgs a = {};
    a.dyn = dyn; a.scal = scal; a.part = part; a.cred = cred;
    a.part_stride = per_scenario ? P : 0; a.cred_stride = per_scenario ? Q : 0;
    a.L = d->n_layers; a.K = d->n_stats; a.Ns = d->n_scalars; a.Q = Q; a.C = P * Q;
    a.Fs = d->n_layers * d->n_stats + d->n_scalars; a.F = a.Fs + 2; a.D = d->n_hidden;
    for (int k = 0; k < d->n_hidden; ++k) a.H[k] = d->hidden[k];
    for (int k = 0; k <= d->n_hidden; ++k) { a.W[k] = prm->W[k]; a.b[k] = prm->b[k]; }
    for (int i = 0; i < AB_MAX_STATS; ++i) a.enc_stat[i] = d->enc_stat[i];
    for (int i = 0; i < AB_MAX_SCALARS; ++i) a.enc_scalar[i] = d->enc_scalar[i];
    a.enc_part = d->enc_partition; a.enc_cred = d->enc_credit;
    a.scores = scores; a.best_idx = best_idx; a.best_score = best_score;
    constexpr int smem = (2 * 64 * 132 + 128 * 132) * 4;       // activation buffers + one weight matrix as fp32, padded rows
    hipError_t e;
    if (dtype == AB_BF16) {
        static DeviceOnce once;
        e = ensure_dynamic_lds((const void *)score_tiny_kernel<bf16_t>, smem, once);
        if (e != hipSuccess) return e;
        score_tiny_kernel<bf16_t><<<(unsigned)S, 1024, smem, st>>>(a);
    } else {
        static DeviceOnce once;
        e = ensure_dynamic_lds((const void *)score_tiny_kernel<float>, smem, once);
        if (e != hipSuccess) return e;
        score_tiny_kernel<float><<<(unsigned)S, 1024, smem, st>>>(a);
    }
    return hipGetLastError();
}

hipError_t launch_trigger(const float *scores, int64_t S, int C, int64_t row_stride, const int32_t *cur_idx,
                          const float *observed, float gain_threshold, float error_threshold, int32_t *best_idx,
                          float *gain, uint8_t *reconf, uint8_t *adapt, hipStream_t st)
{
    if (S == 0) return hipSuccess;
    TriggerArgs a{scores, row_stride, C, cur_idx, observed, gain_threshold, error_threshold, best_idx, gain, reconf, adapt};
    trigger_kernel<<<(unsigned)S, 256, 0, st>>>(a);
    return hipGetLastError();
}

hipError_t launch_score_single_hidden(const float *a_term, const float *b_term, const float *w_out_f,
                                      float *partial, int64_t rows, int C, int H, const float *wp, const float *wc,
                                      const float *xp_row, const float *xc_row, hipStream_t st)
{
    if (rows == 0) return hipSuccess;
    ScoreD1Args a{a_term, b_term, w_out_f, partial, rows, C, H, wp, wc, xp_row, xc_row};
    score_single_hidden_kernel<<<(unsigned)((rows + 3) / 4), 256, 0, st>>>(a);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Temporal encoder (Section 3.1 "Meta network architecture": the layer-wise statistics are embedded into
// a fixed width and a two-layer LSTM extracts the sequential features): e_t = W_e phi(stat[t]) + b_e
// (K -> 32), two stacked LSTM layers of 64 units over t = 0..L-1 with zero initial state, gate blocks in
// the order input, forget, candidate, output; the second layer's last hidden state becomes the first 64
// columns of the scenario row.
// One work-group of eight wavefronts per 32 scenarios, the whole sequence in one launch; four wavefronts run
// the first layer, four the second one step behind (two wavefronts per SIMD hide each other's latencies):
//   - a wavefront owns 16 units of its layer and keeps their rows of [W_ih | W_hh] (bf16) in registers
//     as matrix-instruction operands, permuted so that the four gates of a unit land in one lane:
//     column 8g + 4h + j of output block b is gate g of unit 16w + 8b + 4h + j;  the bias is the
//     addend of the first matrix instruction;
//   - the recurrent operands live in LDS as rows [e | h1 | h2] (bf16), double-buffered by iteration parity:
//     in iteration t layer 1 makes h1_t from (e_t, h1_{t-1}) and layer 2 makes h2_{t-1} from (h1_{t-1},
//     h2_{t-2}), all read from buffer t&1 and written to the other one: one barrier per iteration;
//   - cell states stay in fp32 registers; sigmoid and tanh through exp2 and reciprocal;
//   - the statistics come in chunks of 16 steps (transformed once, one chunk ahead in registers).
// The step is bound by the transcendental rate of the vector ALUs (10 per unit and step), not by the
// matrix cores.
// ------------------------------------------------------------------------------------------------
struct LstmEncArgs {
    const float *dyn; int32_t L, K; int64_t S;
    const void *We; const float *be;      // [32, K]
    const void *W1; const float *b1;      // [256, 32 + 64]
    const void *W2; const float *b2;      // [256, 64 + 64]
    void *xs; int32_t ld;                 // scenario rows; columns [0, 64) written here
    const int32_t *layers_of;             // [S] or NULL: layers the scenario really has (clamped to [1, L])
    ab_enc enc_stat[AB_MAX_ENCODER_STATS];
};

__device__ __forceinline__ float fast_sigmoid(float x)
{
    return __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.44269504088896f * x));
}
__device__ __forceinline__ float fast_tanh(float x)
{
    return 1.f - 2.f * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(2.88539008177793f * x));
}

__global__ __launch_bounds__(512) void lstm_encoder_kernel(const LstmEncArgs a)
{
    constexpr int E = 32, H = 64, R = 32, TC = 16;
    constexpr int STRIDE = 336;                    // bytes per row: (32 + 64 + 64) bf16 + 16 (bank spread)
    constexpr int COL_H1 = E, COL_H2 = E + H;
    __shared__ __attribute__((aligned(16))) unsigned char act[2][R * STRIDE];
    __shared__ __attribute__((aligned(16))) float stat[2][R][TC][AB_MAX_ENCODER_STATS];

    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int role = wave >> 2, wu = wave & 3;     // role 0: first LSTM layer, 1: second; wu: which 16 units
    // Of the two wavefronts of a SIMD the one of the second layer has more to do per step (eight k steps against six,
    // and the next step's embedding) and, being the younger one, would be served last: it gets the higher priority.
    if (role) __builtin_amdgcn_s_setprio(2);
    const int l31 = lane & 31, hf = lane >> 5;
    const int64_t s0 = (int64_t)blockIdx.x * R;
    const int L = a.L, K = a.K;

    // ---- this wavefront's weights as first operands: lane -> row (l31 = output column) and 8 k values (hf);
    // layer 1 has 6 k steps (32 + 64 inputs), layer 2 has 8 (64 + 64)
    i32x4 wf[2][8];
    f32x16 bias[2];
    {
        const int g = l31 >> 3, hp = (l31 >> 2) & 1, j = l31 & 3;
        const uint16_t *W = (const uint16_t *)(role ? a.W2 : a.W1);
        const float *bsrc = role ? a.b2 : a.b1;
        const int kin = role ? 2 * H : E + H;
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int wrow = g * H + 16 * wu + 8 * b + 4 * hp + j;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                wf[b][ks] = i32x4{0, 0, 0, 0};
                if (ks * 16 < kin) wf[b][ks] = *(const i32x4 *)(W + (size_t)wrow * kin + ks * 16 + 8 * hf);
            }
#pragma unroll
            for (int r = 0; r < 16; ++r)          // register r of the result: gate r / 4, unit offset r & 3 (+ 4 hf)
                bias[b][r] = bsrc[(r >> 2) * H + 16 * wu + 8 * b + 4 * hf + (r & 3)];
        }
    }
    // ---- embedding (the second layer's wavefronts do it): thread -> row te >> 3, outputs 4 (te & 7) .. + 3
    // (W_e and b_e sit in LDS: 33 values per output would crowd the registers that hold the gate weights)
    __shared__ __attribute__((aligned(16))) float we_s[E][AB_MAX_ENCODER_STATS];
    __shared__ float be_s[E];
    const int te = t & 255, erow = te >> 3, ej = (te & 7) * 4;
    if (t < E * AB_MAX_ENCODER_STATS) {
        const int o = t / AB_MAX_ENCODER_STATS, k = t % AB_MAX_ENCODER_STATS;
        we_s[o][k] = k < K ? bf16_bits_to_f32(((const uint16_t *)a.We)[o * K + k]) : 0.f;
    }
    if (t < E) be_s[t] = a.be[t];
    // ---- statistics chunks: 32 rows x TC steps x K values, element idx = t + 512 i
    constexpr int PRE = R * TC * AB_MAX_ENCODER_STATS / 512;     // 8 registers at K = 8
    float pre[PRE];
    const int per_row = TC * K;
    auto fetch_chunk = [&](int n) {
#pragma unroll
        for (int i = 0; i < PRE; ++i) {
            const int idx = t + 512 * i;
            pre[i] = 0.f;
            if (idx < R * per_row) {
                const int row = idx / per_row, o = idx - row * per_row;
                int step = n * TC + o / K;
                if (step > L - 1) step = L - 1;
                int64_t sc = s0 + row;
                if (sc > a.S - 1) sc = a.S - 1;
                const int k = o % K;
                pre[i] = phi(a.dyn[(sc * L + step) * K + k], a.enc_stat[k]);
            }
        }
    };
    auto put_chunk = [&](int buf) {
#pragma unroll
        for (int i = 0; i < PRE; ++i) {
            const int idx = t + 512 * i;
            if (idx < R * per_row) {
                const int row = idx / per_row, o = idx - row * per_row;
                stat[buf][row][o / K][o % K] = pre[i];
            }
        }
    };
    auto embed_step = [&](int step, int buf) {           // e_step -> act[buf], columns [0, 32)
        const float *sp = &stat[(step / TC) & 1][erow][step % TC][0];
        float e[4] = {be_s[ej], be_s[ej + 1], be_s[ej + 2], be_s[ej + 3]};
#pragma unroll
        for (int k = 0; k < AB_MAX_ENCODER_STATS; ++k)
            if (k < K) {
                const float x = sp[k];
#pragma unroll
                for (int i = 0; i < 4; ++i) e[i] = fmaf(we_s[ej + i][k], x, e[i]);
            }
        uint2 pk = {pack_bf16x2(e[0], e[1]), pack_bf16x2(e[2], e[3])};
        *(uint2 *)(&act[buf][erow * STRIDE + ej * 2]) = pk;
    };

    // ---- start: zero state, first chunk, e_0
    for (int i = t; i < 2 * R * STRIDE / 4; i += 512) ((uint32_t *)&act[0][0])[i] = 0u;
    fetch_chunk(0);
    put_chunk(0);
    __syncthreads();
    if (role == 1) embed_step(0, 0);

    float c[2][4], hv[2][4], hlast[2][4];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int j = 0; j < 4; ++j) c[b][j] = hv[b][j] = hlast[b][j] = 0.f;
    // this lane's scenario (row l31) may have fewer layers than the block runs for: its result is the second
    // layer's hidden state after its own last layer; what the recurrence does to that row afterwards is unused
    int my_len = L;
    if (a.layers_of) {
        int64_t sc = s0 + l31;
        if (sc > a.S - 1) sc = a.S - 1;
        my_len = a.layers_of[sc];
        my_len = my_len < 1 ? 1 : (my_len > L ? L : my_len);
    }

    const int frag_rd = l31 * STRIDE + 16 * hf;          // + column * 2
    const int h_wr = l31 * STRIDE + (16 * wu + 4 * hf) * 2;     // + (field column + 8 b) * 2
    auto cell = [&](const f32x16 &z, float (&cs)[4], float (&h)[4]) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float ig = fast_sigmoid(z[j]), fg = fast_sigmoid(z[4 + j]);
            const float gg = fast_tanh(z[8 + j]), og = fast_sigmoid(z[12 + j]);
            cs[j] = fmaf(fg, cs[j], ig * gg);
            h[j] = og * fast_tanh(cs[j]);
        }
    };

    // Iteration tau: the first layer makes h1_tau from (e_tau, h1_{tau-1}) while the second layer makes
    // h2_{tau-1} from (h1_{tau-1}, h2_{tau-2}); all of these sit in buffer tau & 1 and every result (with
    // e_{tau+1}) goes to the other buffer, so one barrier per iteration orders everything.
    for (int tau = 0; tau <= L; ++tau) {
        const int p = tau & 1;
        __syncthreads();
        const int tc = tau % TC, n = tau / TC;
        if (tc == 0 && (n + 1) * TC < L) fetch_chunk(n + 1);
        if (tc == TC - 2 && (n + 1) * TC < L) put_chunk((n + 1) & 1);
        f32x16 z[2];
        if (role == 0) {
            if (tau < L) {
#pragma unroll
                for (int ks = 0; ks < 6; ++ks) {
                    const i32x4 xf = *(const i32x4 *)(&act[p][frag_rd + ks * 32]);
#pragma unroll
                    for (int b = 0; b < 2; ++b)
                        z[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wf[b][ks]),
                                                                       __builtin_bit_cast(bf16x8, xf),
                                                                       ks == 0 ? bias[b] : z[b], 0, 0, 0);
                }
#pragma unroll
                for (int b = 0; b < 2; ++b) {
                    cell(z[b], c[b], hv[b]);
                    uint2 pk = {pack_bf16x2(hv[b][0], hv[b][1]), pack_bf16x2(hv[b][2], hv[b][3])};
                    *(uint2 *)(&act[p ^ 1][h_wr + (COL_H1 + 8 * b) * 2]) = pk;
                }
            }
        } else {
            if (tau + 1 < L) embed_step(tau + 1, p ^ 1);
            if (tau >= 1) {
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) {
                    const i32x4 xf = *(const i32x4 *)(&act[p][frag_rd + (COL_H1 + ks * 16) * 2]);
#pragma unroll
                    for (int b = 0; b < 2; ++b)
                        z[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wf[b][ks]),
                                                                       __builtin_bit_cast(bf16x8, xf),
                                                                       ks == 0 ? bias[b] : z[b], 0, 0, 0);
                }
#pragma unroll
                for (int b = 0; b < 2; ++b) {
                    cell(z[b], c[b], hv[b]);
                    uint2 pk = {pack_bf16x2(hv[b][0], hv[b][1]), pack_bf16x2(hv[b][2], hv[b][3])};
                    *(uint2 *)(&act[p ^ 1][h_wr + (COL_H2 + 8 * b) * 2]) = pk;
                    if (tau == my_len) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) hlast[b][j] = hv[b][j];
                    }
                }
            }
        }
    }
    // ---- second layer's hidden state after the scenario's last layer -> columns 16 wu + 8 b + 4 hf .. + 3
    if (role == 1 && s0 + l31 < a.S) {
        uint16_t *row = (uint16_t *)a.xs + (s0 + l31) * (int64_t)a.ld + 16 * wu + 4 * hf;
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            uint2 pk = {pack_bf16x2(hlast[b][0], hlast[b][1]), pack_bf16x2(hlast[b][2], hlast[b][3])};
            *(uint2 *)(row + 8 * b) = pk;
        }
    }
}

hipError_t launch_lstm_encoder(const ab_model_desc *d, const float *dyn, const void *We, const float *be,
                               const void *W1, const float *b1, const void *W2, const float *b2, void *xs,
                               int ld, int64_t S, const int32_t *layers_of, hipStream_t st)
{
    if (S == 0) return hipSuccess;
    LstmEncArgs a;
    a.layers_of = layers_of;
    a.dyn = dyn; a.L = d->n_layers; a.K = d->n_stats; a.S = S;
    a.We = We; a.be = be; a.W1 = W1; a.b1 = b1; a.W2 = W2; a.b2 = b2; a.xs = xs; a.ld = ld;
    for (int i = 0; i < AB_MAX_ENCODER_STATS; ++i) a.enc_stat[i] = d->enc_stat[i];
    const int64_t blocks = (S + 31) / 32;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    lstm_encoder_kernel<<<(unsigned)blocks, 512, 0, st>>>(a);
    return hipGetLastError();
}

hipError_t launch_tensor_encoder(int dtype, const ab_model_desc *d, const float *dyn, const void *Wa,
                                 const float *ba, const void *Wb, const float *bb, void *xs, int ld,
                                 int64_t S, const int32_t *layers_of, hipStream_t st)
{
    if (S == 0) return hipSuccess;
    TensorEncArgs a;
    a.layers_of = layers_of;
    a.dyn = dyn; a.L = d->n_layers; a.K = d->n_stats; a.Wa = Wa; a.ba = ba; a.Wb = Wb; a.bb = bb;
    a.xs = xs; a.ld = ld; a.S = S;
    for (int i = 0; i < AB_MAX_ENCODER_STATS; ++i) a.enc_stat[i] = d->enc_stat[i];
    int cus = 0;
    hipError_t e;
    if ((e = compute_units(&cus)) != hipSuccess) return e;
    const int64_t grid = S < 2 * (int64_t)cus ? S : 2 * (int64_t)cus;      // two work-groups fit a CU's LDS
    if (dtype == AB_BF16) tensor_encoder_kernel<bf16_t><<<(unsigned)grid, 256, 0, st>>>(a);
    else tensor_encoder_kernel<float><<<(unsigned)grid, 256, 0, st>>>(a);
    return hipGetLastError();
}

}  // namespace ab
