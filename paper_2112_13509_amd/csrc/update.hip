// Online adaptation step (Section 3.2 "Offline training online adapting"; loss of Eq. 2 as mean
// squared error): forward with saved activations, exact back-propagation, Adam.
//
// Every matrix product is brought to the K-contiguous form of gemm_core.hpp by keeping transposed
// copies next to the row-major ones (written by the producing kernel's epilogue):
//   forward   h_k      = relu(h_{k-1} W_k^T + b_k)          A = h_{k-1} [B, in],   B-op = W_k [out, in]
//   dW_k      = d_k^T h_{k-1}                               A = d_k^T [out, B],    B-op = h_{k-1}^T [in, B]   (split over B)
//   d_{k-1}   = (d_k W_k) * [h_{k-1} > 0]                   A = d_k [B, out],      B-op = W_k^T [in, out]
// The batch dimension is padded to a multiple of 64 in the transposed buffers (zero columns).
#include "internal.hpp"
#include <string.h>

namespace ab {

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
static inline int round_up(int x, int a) { return (x + a - 1) / a * a; }

#define AB_HIP(expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) return AB_ERR_DEVICE; } while (0)

struct UpdatePlan {
    int dtype, F, Kp, D, n_out;
    int H[AB_MAX_HIDDEN];
    int64_t B, Bp;
    int in_w[AB_MAX_HIDDEN + 1];        // padded input width of layer k (Kp for k = 0)
    int splits[AB_MAX_HIDDEN];
    size_t off_scal, off_x, off_xt, off_w1p, off_yhat, off_dout, off_lossrow, off_gwout, off_gbout;
    size_t off_wt[AB_MAX_HIDDEN], off_h[AB_MAX_HIDDEN], off_ht[AB_MAX_HIDDEN];
    size_t off_d[AB_MAX_HIDDEN], off_dt[AB_MAX_HIDDEN], off_gw[AB_MAX_HIDDEN], off_gb[AB_MAX_HIDDEN];
    size_t total;
};

static int update_tile(int64_t M, int N)
{
    if (N % 128 == 0 && ((M + 127) / 128) * (N / 128) >= 256) return TILE_MID;
    return TILE_SMALL;
}

static void plan_update(const ab_model_desc *d, int64_t B, UpdatePlan *p)
{
    memset(p, 0, sizeof(*p));
    p->dtype = d->compute_dtype;
    p->F = d->n_layers * d->n_stats + d->n_scalars + 2;
    p->Kp = round_up(p->F, 64);
    p->D = d->n_hidden;
    p->n_out = d->n_outputs > 1 ? d->n_outputs : 1;
    p->B = B;
    p->Bp = (B + 63) / 64 * 64;
    const size_t es = elem_size(p->dtype);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    p->off_scal = take(64);
    p->off_x = take((size_t)B * p->Kp * es);
    p->off_xt = take((size_t)p->Kp * p->Bp * es);
    p->off_yhat = take((size_t)B * p->n_out * 4);
    p->off_dout = take((size_t)p->Bp * p->n_out * 4);
    p->off_lossrow = take((size_t)p->Bp * 4);
    for (int k = 0; k < p->D; ++k) {
        p->H[k] = d->hidden[k];
        p->in_w[k] = (k == 0) ? p->Kp : d->hidden[k - 1];
        const int tiles = (p->H[k] / 64) * (p->in_w[k] / 64);
        const int slabs = (int)(p->Bp / slab_k(p->dtype));
        int s = 512 / tiles;
        if (s > 8) s = 8;
        if (s > slabs) s = slabs;
        if (s < 1) s = 1;
        p->splits[k] = s;
        p->off_wt[k] = take((size_t)p->H[k] * p->in_w[k] * es);     // k = 0: padded copy of W_1; else W_k^T
        p->off_h[k] = take((size_t)B * p->H[k] * es);
        p->off_ht[k] = take((size_t)p->H[k] * p->Bp * es);
        p->off_d[k] = take((size_t)B * p->H[k] * es);
        p->off_dt[k] = take((size_t)p->H[k] * p->Bp * es);
        p->off_gw[k] = take((size_t)s * p->H[k] * p->in_w[k] * 4);
        p->off_gb[k] = take((size_t)p->H[k] * 4);
    }
    p->off_gwout = take((size_t)p->n_out * (p->D > 0 ? p->H[p->D - 1] : p->F) * 4);   // no hidden layer: the output layer reads x
    p->off_gbout = take((size_t)AB_MAX_OUTPUTS * 4);
    p->total = off;
}

size_t update_workspace_bytes(const ab_model_desc *d, int64_t B)
{
    if (d->tensor_encoder || d->n_hidden < 0) return 0;
    UpdatePlan p;
    plan_update(d, B, &p);
    return p.total;
}

// ---------------------------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ float ld_f32(const void *p, int64_t i)
{
    if constexpr (sizeof(T) == 2) return bf16_bits_to_f32(((const uint16_t *)p)[i]);
    else return ((const float *)p)[i];
}
template <typename T>
__device__ __forceinline__ void st_T(void *p, int64_t i, float v)
{
    if constexpr (sizeof(T) == 2) ((uint16_t *)p)[i] = (uint16_t)(pack_bf16x2(v, 0.f) & 0xffffu);
    else ((float *)p)[i] = v;
}

// Per call: padded copy of W_1, transposes of the other hidden weights, zero padding columns of
// the transposed batch buffers.
struct UpdPrepArgs {
    int64_t *step; float *scal; float beta1, beta2;      // the step counter and Adam's bias corrections ride along
    int n_jobs;
    struct Job { const void *src; void *dst; int rows, cols, ld_src, ld_dst, kind; int64_t start; } job[2 + 3 * AB_MAX_HIDDEN];
    int64_t total;
};
enum { JOB_PAD_COPY = 0, JOB_TRANSPOSE = 1, JOB_ZERO_COLS = 2 };

template <typename T>
__device__ __forceinline__ void update_prep_block(const UpdPrepArgs &a, unsigned id)
{
    const int64_t gid = (int64_t)id * 256 + threadIdx.x;
    if (gid == 0) {                            // step counter and Adam bias corrections 1 - beta^t
        const int64_t t = *a.step + 1;
        *a.step = t;
        a.scal[0] = (float)(1.0 - pow((double)a.beta1, (double)t));
        a.scal[1] = (float)(1.0 - pow((double)a.beta2, (double)t));
    }
    if (gid >= a.total) return;
    int j = 0;
    while (j + 1 < a.n_jobs && gid >= a.job[j + 1].start) ++j;
    const UpdPrepArgs::Job &jb = a.job[j];
    const int64_t e = gid - jb.start;
    if (jb.kind == JOB_PAD_COPY) {            // dst[rows, ld_dst] <- src[rows, cols], zero padded
        const int r = (int)(e / jb.ld_dst), c = (int)(e % jb.ld_dst);
        if constexpr (sizeof(T) == 2)
            ((uint16_t *)jb.dst)[e] = c < jb.cols ? ((const uint16_t *)jb.src)[(int64_t)r * jb.ld_src + c] : (uint16_t)0;
        else
            ((float *)jb.dst)[e] = c < jb.cols ? ((const float *)jb.src)[(int64_t)r * jb.ld_src + c] : 0.f;
    } else if (jb.kind == JOB_TRANSPOSE) {    // dst[cols, rows] <- src[rows, cols]
        const int c = (int)(e / jb.rows), r = (int)(e % jb.rows);
        if constexpr (sizeof(T) == 2)
            ((uint16_t *)jb.dst)[e] = ((const uint16_t *)jb.src)[(int64_t)r * jb.ld_src + c];
        else
            ((float *)jb.dst)[e] = ((const float *)jb.src)[(int64_t)r * jb.ld_src + c];
    } else {                                  // zero columns [cols, ld_dst) of dst[rows, ld_dst]
        const int w = jb.ld_dst - jb.cols;
        const int r = (int)(e / w), c = jb.cols + (int)(e % w);
        if constexpr (sizeof(T) == 2) ((uint16_t *)jb.dst)[(int64_t)r * jb.ld_dst + c] = 0;
        else ((float *)jb.dst)[(int64_t)r * jb.ld_dst + c] = 0.f;
    }
}

// Output layer forward and its delta: one wavefront per sample.  With e = yhat - y (n_out entries):
//   squared loss:  dout = 2 e / B ;   norm loss (Eq. 2):  dout = e / (|e| B), zero where e = 0
//   d[r, :] = (sum_w dout[w] W_out[w, :]) * [h > 0]
struct OutFwdArgs {
    const void *h; const void *w_out; const float *b_out; const float *target;
    float *yhat; float *dout; float *lossrow; void *d; int64_t B; int32_t H, n_out, loss_kind;
};
// Eight consecutive elements of the compute type as fp32 (i a multiple of 8 on a 16-byte aligned base).
template <typename T>
__device__ __forceinline__ void load8(const void *p, int64_t i, float (&v)[8])
{
    if constexpr (sizeof(T) == 2) {
        const i32x4 x = *(const i32x4 *)((const uint16_t *)p + i);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            v[2 * q] = __uint_as_float((uint32_t)x[q] << 16);
            v[2 * q + 1] = __uint_as_float((uint32_t)x[q] & 0xffff0000u);
        }
    } else {
        const f32x4 x = *(const f32x4 *)((const float *)p + i), y = *(const f32x4 *)((const float *)p + i + 4);
#pragma unroll
        for (int q = 0; q < 4; ++q) { v[q] = x[q]; v[4 + q] = y[q]; }
    }
}
template <typename T>
__device__ __forceinline__ void store8(void *p, int64_t i, const float (&v)[8])
{
    if constexpr (sizeof(T) == 2) {
        i32x4 x;
#pragma unroll
        for (int q = 0; q < 4; ++q) x[q] = (int)pack_bf16x2(v[2 * q], v[2 * q + 1]);
        *(i32x4 *)((uint16_t *)p + i) = x;
    } else {
        *(f32x4 *)((float *)p + i) = f32x4{v[0], v[1], v[2], v[3]};
        *(f32x4 *)((float *)p + i + 4) = f32x4{v[4], v[5], v[6], v[7]};
    }
}

// A lane takes eight adjacent columns per 512 (the widths are multiples of 64, so a group of eight is inside
// the row or outside it as a whole); the hidden row is read once for all outputs.
template <typename T>
__global__ __launch_bounds__(256) void output_forward_kernel(const OutFwdArgs a)
{
    const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= a.B) return;
    const int lane = threadIdx.x & 63;
    float dv[AB_MAX_OUTPUTS];
#pragma unroll
    for (int w = 0; w < AB_MAX_OUTPUTS; ++w) dv[w] = 0.f;
    for (int c0 = lane * 8; c0 < a.H; c0 += 512) {
        float hv[8];
        load8<T>(a.h, r * a.H + c0, hv);
#pragma unroll
        for (int w = 0; w < AB_MAX_OUTPUTS; ++w) {
            if (w < a.n_out) {
                float wv[8];
                load8<T>(a.w_out, (int64_t)w * a.H + c0, wv);
#pragma unroll
                for (int e = 0; e < 8; ++e) dv[w] = fmaf(hv[e], wv[e], dv[w]);
            }
        }
    }
    float sq = 0.f;
#pragma unroll
    for (int w = 0; w < AB_MAX_OUTPUTS; ++w) {
        if (w < a.n_out) {
            const float acc = wave_sum(dv[w]);
            const float yh = acc + a.b_out[w];
            if (lane == 0) a.yhat[r * a.n_out + w] = yh;
            dv[w] = yh - a.target[r * a.n_out + w];
            sq += dv[w] * dv[w];
        }
    }
    const float nrm = sqrtf(sq);
    const float f = a.loss_kind == AB_LOSS_L2NORM ? (nrm > 0.f ? 1.f / (nrm * (float)a.B) : 0.f) : 2.f / (float)a.B;
    if (lane == 0) a.lossrow[r] = a.loss_kind == AB_LOSS_L2NORM ? nrm : sq;       // this row's term of the loss
#pragma unroll
    for (int w = 0; w < AB_MAX_OUTPUTS; ++w) {
        dv[w] *= f;
        if (w < a.n_out && lane == 0) a.dout[r * a.n_out + w] = dv[w];
    }
    for (int c0 = lane * 8; c0 < a.H; c0 += 512) {
        float hv[8], acc[8];
        load8<T>(a.h, r * a.H + c0, hv);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = 0.f;
#pragma unroll
        for (int w = 0; w < AB_MAX_OUTPUTS; ++w) {
            if (w < a.n_out) {
                float wv[8];
                load8<T>(a.w_out, (int64_t)w * a.H + c0, wv);
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[e] = fmaf(dv[w], wv[e], acc[e]);
            }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = hv[e] > 0.f ? acc[e] : 0.f;
        store8<T>(a.d, r * a.H + c0, acc);
    }
}

// The scorer without hidden layers: yhat = W x + b on the transformed rows x[B, ld] (W is [n_out, F], F <= ld),
// the loss terms and the output deltas as in output_forward_kernel; a wavefront per sample.
struct LinFwdArgs {
    const void *x; const void *w; const float *b; const float *target;
    float *yhat; float *dout; float *lossrow; int64_t B; int32_t ld, F, n_out, loss_kind;
};
template <typename T>
__global__ __launch_bounds__(256) void linear_forward_kernel(const LinFwdArgs a)
{
    const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= a.B) return;
    const int lane = threadIdx.x & 63;
    float dv[AB_MAX_OUTPUTS];
#pragma unroll
    for (int w = 0; w < AB_MAX_OUTPUTS; ++w) dv[w] = 0.f;
    for (int j = lane; j < a.F; j += 64) {
        const float xv = ld_f32<T>(a.x, r * a.ld + j);
#pragma unroll
        for (int w = 0; w < AB_MAX_OUTPUTS; ++w)
            if (w < a.n_out) dv[w] = fmaf(xv, ld_f32<T>(a.w, (int64_t)w * a.F + j), dv[w]);
    }
    float sq = 0.f;
#pragma unroll
    for (int w = 0; w < AB_MAX_OUTPUTS; ++w) {
        if (w < a.n_out) {
            const float yh = wave_sum(dv[w]) + a.b[w];
            if (lane == 0) a.yhat[r * a.n_out + w] = yh;
            dv[w] = yh - a.target[r * a.n_out + w];
            sq += dv[w] * dv[w];
        }
    }
    const float nrm = sqrtf(sq);
    const float f = a.loss_kind == AB_LOSS_L2NORM ? (nrm > 0.f ? 1.f / (nrm * (float)a.B) : 0.f) : 2.f / (float)a.B;
    if (lane == 0) {
        a.lossrow[r] = a.loss_kind == AB_LOSS_L2NORM ? nrm : sq;
#pragma unroll
        for (int w = 0; w < AB_MAX_OUTPUTS; ++w)
            if (w < a.n_out) a.dout[r * a.n_out + w] = dv[w] * f;
    }
}

// Output layer gradients: block c < H handles column c of the last hidden layer:
//   gw_out[w, c] = sum_r dout[r, w] h[r, c]  and  d^T[c, r] = (sum_w dout[r, w] W_out[w, c]) [h^T[c, r] > 0];
// block H + w (w < n_out) reduces the bias gradient sum_r dout[r, w], block H + n_out the loss.
struct OutGradArgs {
    const void *ht; const void *w_out; const float *dout; const float *lossrow;
    void *dt; float *gw_out; float *gb_out; float *loss_out; int64_t B, Bp; int32_t H, n_out, loss_kind;
};
__device__ __forceinline__ float block_sum_256(float v, float *sh)      // sh: four floats of LDS
{
    v = wave_sum(v);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    const float r = (sh[0] + sh[1]) + (sh[2] + sh[3]);
    __syncthreads();
    return r;
}
template <typename T>
__device__ __forceinline__ void output_grad_block(const OutGradArgs &a, unsigned id, float *sh)
{
    const int c = (int)id;
    if (c < a.H) {
        // a thread takes eight adjacent rows per 2048 of column c of h^T (the batch is padded to a multiple of
        // 64 with zero columns, whose deltas are taken as zero)
        float wv[AB_MAX_OUTPUTS], acc[AB_MAX_OUTPUTS];
#pragma unroll
        for (int w = 0; w < AB_MAX_OUTPUTS; ++w) {
            wv[w] = w < a.n_out ? ld_f32<T>(a.w_out, (int64_t)w * a.H + c) : 0.f;
            acc[w] = 0.f;
        }
        for (int64_t r0 = (int64_t)threadIdx.x * 8; r0 < a.Bp; r0 += 2048) {
            float hv[8], ds[8];
            load8<T>(a.ht, (int64_t)c * a.Bp + r0, hv);
#pragma unroll
            for (int e = 0; e < 8; ++e) ds[e] = 0.f;
            // (dout is allocated for the padded batch; what lies beyond B is read and discarded)
            if ((a.n_out & 3) == 0) {          // four outputs of a row per 16-byte load
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float live = r0 + e < a.B ? 1.f : 0.f;
#pragma unroll
                    for (int w4 = 0; w4 < AB_MAX_OUTPUTS / 4; ++w4) {
                        if (w4 * 4 < a.n_out) {
                            const f32x4 dv = *(const f32x4 *)(a.dout + (r0 + e) * a.n_out + w4 * 4);
#pragma unroll
                            for (int q = 0; q < 4; ++q) {
                                const float v = live != 0.f ? dv[q] : 0.f;
                                acc[w4 * 4 + q] = fmaf(v, hv[e], acc[w4 * 4 + q]);
                                ds[e] = fmaf(v, wv[w4 * 4 + q], ds[e]);
                            }
                        }
                    }
                }
            } else {
#pragma unroll
                for (int w = 0; w < AB_MAX_OUTPUTS; ++w) {
                    if (w < a.n_out) {
                        float dv[8];
                        if (a.n_out == 1) {
                            const f32x4 x = *(const f32x4 *)(a.dout + r0), y = *(const f32x4 *)(a.dout + r0 + 4);
#pragma unroll
                            for (int q = 0; q < 4; ++q) { dv[q] = x[q]; dv[4 + q] = y[q]; }
                        } else {
#pragma unroll
                            for (int e = 0; e < 8; ++e) dv[e] = a.dout[(r0 + e) * a.n_out + w];
                        }
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const float v = r0 + e < a.B ? dv[e] : 0.f;
                            acc[w] = fmaf(v, hv[e], acc[w]);
                            ds[e] = fmaf(v, wv[w], ds[e]);
                        }
                    }
                }
            }
            if (a.dt) {                  // (no layer below the output layer: nothing to hand down)
#pragma unroll
                for (int e = 0; e < 8; ++e) ds[e] = hv[e] > 0.f ? ds[e] : 0.f;
                store8<T>(a.dt, (int64_t)c * a.Bp + r0, ds);
            }
        }
#pragma unroll
        for (int w = 0; w < AB_MAX_OUTPUTS; ++w) {
            if (w < a.n_out) {
                const float s = block_sum_256(acc[w], sh);
                if (threadIdx.x == 0) a.gw_out[(int64_t)w * a.H + c] = s;
            }
        }
    } else if (c < a.H + a.n_out) {
        const int w = c - a.H;
        float sd = 0.f;
#pragma unroll 4
        for (int64_t r = threadIdx.x; r < a.B; r += 256) sd += a.dout[r * a.n_out + w];
        const float s1 = block_sum_256(sd, sh);
        if (threadIdx.x == 0) a.gb_out[w] = s1;
    } else {
        float sl = 0.f;
#pragma unroll 4
        for (int64_t r = threadIdx.x; r < a.B; r += 256) sl += a.lossrow[r];
        const float s2 = block_sum_256(sl, sh);
        if (threadIdx.x == 0 && a.loss_out) a.loss_out[0] = s2 / (float)a.B;
    }
}

// Bias gradients of the hidden layers: gb_k[c] = sum_r d_k^T[c, r], one block per (layer, unit).
struct BiasGradArgs {
    int n; struct L { const void *dt; float *gb; int H; int start; } l[AB_MAX_HIDDEN];
    int64_t B, Bp;
};
template <typename T>
__device__ __forceinline__ void bias_grad_block(const BiasGradArgs &a, unsigned id, float *sh)
{
    int k = 0;
    while (k + 1 < a.n && (int)id >= a.l[k + 1].start) ++k;
    const int c = (int)id - a.l[k].start;
    float acc = 0.f;                 // (the padding columns of d^T beyond B are zero)
    for (int64_t r0 = (int64_t)threadIdx.x * 8; r0 < a.Bp; r0 += 2048) {
        float v[8];
        load8<T>(a.l[k].dt, (int64_t)c * a.Bp + r0, v);
        acc += ((v[0] + v[1]) + (v[2] + v[3])) + ((v[4] + v[5]) + (v[6] + v[7]));
    }
    const float s = block_sum_256(acc, sh);
    if (threadIdx.x == 0) a.l[k].gb[c] = s;
}

// Raw update rows x_raw[B, F] (statistics, scalars, partition, credit) -> transformed x[B, ld] (zero in the
// padding columns) and its transpose x_t[ld, ld_t].  A work-group takes a tile of 64 rows x 64 columns: a
// thread transforms one pair of columns for eight rows (so it looks its two transforms up once), writes the
// row-major pairs, and parks the values in LDS, from which the transposed tile leaves as 32- or 64-byte
// pieces of a row of x_t.  Rows at and beyond B of the tile are written as zeros into x_t (ld_t is the batch
// rounded up to 64).
struct EncodeRowsArgs {
    const float *x_raw; void *x; void *x_t; int64_t B, ld_t; int32_t F, ld, col_tiles;
    int32_t n_stat, n_stats_per_layer, n_scal;
    ab_enc enc_stat[AB_MAX_STATS];
    ab_enc enc_scal[AB_MAX_SCALARS];
    ab_enc enc_part, enc_cred;
};

template <typename T>
__device__ __forceinline__ void encode_rows_block(const EncodeRowsArgs &a, unsigned id, unsigned char *smem)
{
    constexpr int LD_TILE = sizeof(T) == 2 ? 66 : 65;          // elements per tile row (one column of x, 64 rows)
    T *tile = (T *)smem;
    const int c0 = (int)(id % (unsigned)a.col_tiles) * 64;
    const int64_t r0 = (int64_t)(id / (unsigned)a.col_tiles) * 64;
    const int t = threadIdx.x, cp = t & 31, rr = t >> 5;
    const int j0 = c0 + 2 * cp;
    ab_enc e[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const int j = j0 + q;
        const ab_enc *src = j < a.n_stat ? &a.enc_stat[j % a.n_stats_per_layer]
                          : j < a.n_stat + a.n_scal ? &a.enc_scal[j - a.n_stat]
                          : j == a.F - 2 ? &a.enc_part : &a.enc_cred;
        e[q] = *src;
    }
    float raw0[8], raw1[8];                       // all of the thread's loads first: eight rows x two columns
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int64_t row = r0 + rr + 8 * i;
        raw0[i] = (row < a.B && j0 < a.F) ? a.x_raw[row * a.F + j0] : 1.f;
        raw1[i] = (row < a.B && j0 + 1 < a.F) ? a.x_raw[row * a.F + j0 + 1] : 1.f;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int rl = rr + 8 * i;
        const int64_t row = r0 + rl;
        float v0 = 0.f, v1 = 0.f;
        if (row < a.B) {
            if (j0 < a.F) v0 = phi(raw0[i], e[0]);
            if (j0 + 1 < a.F) v1 = phi(raw1[i], e[1]);
            const int64_t o = row * a.ld + j0;
            if constexpr (sizeof(T) == 2) ((uint32_t *)a.x)[o >> 1] = pack_bf16x2(v0, v1);
            else ((f32x2 *)a.x)[o >> 1] = f32x2{v0, v1};
        }
        if constexpr (sizeof(T) == 2) {
            const uint32_t pk = pack_bf16x2(v0, v1);
            ((uint16_t *)tile)[(2 * cp) * LD_TILE + rl] = (uint16_t)(pk & 0xffffu);
            ((uint16_t *)tile)[(2 * cp + 1) * LD_TILE + rl] = (uint16_t)(pk >> 16);
        } else {
            ((float *)tile)[(2 * cp) * LD_TILE + rl] = v0;
            ((float *)tile)[(2 * cp + 1) * LD_TILE + rl] = v1;
        }
    }
    __syncthreads();
    if (!a.x_t) return;
    const int col = t >> 2, rc = (t & 3) * 16;
    const int64_t o = (int64_t)(c0 + col) * a.ld_t + r0 + rc;
    if constexpr (sizeof(T) == 2) {
        const uint32_t *src = (const uint32_t *)((const uint16_t *)tile + col * LD_TILE + rc);
        i32x4 lo = {(int)src[0], (int)src[1], (int)src[2], (int)src[3]};
        i32x4 hi = {(int)src[4], (int)src[5], (int)src[6], (int)src[7]};
        i32x4 *dst = (i32x4 *)((uint16_t *)a.x_t + o);
        dst[0] = lo; dst[1] = hi;
    } else {
        const float *src = (const float *)tile + col * LD_TILE + rc;
        f32x4 *dst = (f32x4 *)((float *)a.x_t + o);
#pragma unroll
        for (int q = 0; q < 4; ++q) dst[q] = f32x4{src[4 * q], src[4 * q + 1], src[4 * q + 2], src[4 * q + 3]};
    }
}

// First launch of a step: the row transform and, next to it, the weight copies and the step counter.
template <typename T>
__global__ __launch_bounds__(256) void update_first_kernel(const EncodeRowsArgs e, const UpdPrepArgs p, unsigned enc_blocks)
{
    __shared__ __attribute__((aligned(16))) unsigned char smem[64 * 66 * 4];
    if (blockIdx.x < enc_blocks) encode_rows_block<T>(e, blockIdx.x, smem);
    else update_prep_block<T>(p, blockIdx.x - enc_blocks);
}

// Several independent pieces of the backward pass in one launch (each launch of this chain costs about as
// much as the piece itself): up to two matrix products on 64 x 64 tiles (delta of the layer below, split-K
// weight gradient) and either the output unit's gradients or the hidden layers' bias gradients.
enum { UJ_NONE = 0, UJ_GEMM_DRELU = 1, UJ_GEMM_SPLITK = 2, UJ_OUT_GRAD = 3, UJ_BIAS_GRAD = 4 };
struct GroupArgs {
    unsigned start[4];            // slot s owns work-groups [start[s], start[s + 1])
    int kind[3];                  // slots 0 and 1: matrix products; slot 2: output-unit or bias gradients
    GemmArgs gemm[2];
    OutGradArgs og;
    BiasGradArgs bg;
};

template <typename T>
__global__ __launch_bounds__(256) void update_group_kernel(const GroupArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const unsigned b = blockIdx.x;
    if (b < a.start[2]) {
        const int s = b < a.start[1] ? 0 : 1;
        if (a.kind[s] == UJ_GEMM_DRELU)
            gemm_tn_tile<T, 1, 1, AMODE_LOAD, EPI_DRELU>(a.gemm[s], b - a.start[s], smem);
        else
            gemm_tn_tile<T, 1, 1, AMODE_LOAD, EPI_SPLITK>(a.gemm[s], b - a.start[s], smem);
    } else if (a.kind[2] == UJ_OUT_GRAD) {
        output_grad_block<T>(a.og, b - a.start[2], (float *)smem);
    } else {
        bias_grad_block<T>(a.bg, b - a.start[2], (float *)smem);
    }
}

// Adam (Kingma & Ba, Algorithm 1; bias-corrected, epsilon outside the root) over every parameter
// tensor in one launch; also refreshes the compute-type copy of each weight matrix.
struct AdamArgs {
    int n;
    struct Tn {
        float *w, *m, *v; void *w_compute;        // master, moments, compute-type copy (NULL for biases)
        const float *g; int rows, cols, ldg, splits, vw; int64_t split_stride;
        int64_t start;                            // in threads: a thread takes vw adjacent elements
    } tn[2 * (AB_MAX_HIDDEN + 1)];
    int64_t total;
    const float *scal;                            // {1 - beta1^t, 1 - beta2^t}
    float lr, beta1, beta2, eps;
};
// VW adjacent elements of one tensor (VW divides the row length, so they share a row of the gradient buffer).
template <typename T, int VW>
__device__ __forceinline__ void adam_elems(const AdamArgs &a, const AdamArgs::Tn &tn, int64_t e)
{
    typedef __attribute__((ext_vector_type(VW))) float vec;
    const uint32_t r = (uint32_t)e / (uint32_t)tn.cols, c = (uint32_t)e - r * (uint32_t)tn.cols;
    // the split-K partial sums (at most eight): eight loads without a branch between them (splits past the last
    // one read the last one again and are not added), then the sum in split order
    vec gs[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        const int se = s < tn.splits ? s : tn.splits - 1;
        gs[s] = *(const vec *)(tn.g + se * tn.split_stride + (int64_t)r * tn.ldg + c);
    }
    vec g = gs[0];
#pragma unroll
    for (int s = 1; s < 8; ++s) {
        const vec sum = g + gs[s];
#pragma unroll
        for (int q = 0; q < VW; ++q) g[q] = s < tn.splits ? sum[q] : g[q];
    }
    vec m = *(const vec *)(tn.m + e), v = *(const vec *)(tn.v + e), w = *(const vec *)(tn.w + e);
    const float c1 = a.scal[0], c2 = a.scal[1];
#pragma unroll
    for (int q = 0; q < VW; ++q) {
        m[q] = a.beta1 * m[q] + (1.f - a.beta1) * g[q];
        v[q] = a.beta2 * v[q] + (1.f - a.beta2) * g[q] * g[q];
        w[q] = w[q] - a.lr * (m[q] / c1) / (sqrtf(v[q] / c2) + a.eps);
    }
    *(vec *)(tn.m + e) = m;
    *(vec *)(tn.v + e) = v;
    *(vec *)(tn.w + e) = w;
    if (tn.w_compute) {
        if constexpr (sizeof(T) == 2 && VW >= 2) {
#pragma unroll
            for (int q = 0; q < VW; q += 2) ((uint32_t *)tn.w_compute)[(e + q) >> 1] = pack_bf16x2(w[q], w[q + 1]);
        } else {
#pragma unroll
            for (int q = 0; q < VW; ++q) st_T<T>(tn.w_compute, e + q, w[q]);
        }
    }
}
template <typename T>
__global__ __launch_bounds__(256) void adam_kernel(const AdamArgs a)
{
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;       // one thread per group of tn.vw elements
    if (gid >= a.total) return;
    int j = 0;
    while (j + 1 < a.n && gid >= a.tn[j + 1].start) ++j;
    const AdamArgs::Tn &tn = a.tn[j];
    const int64_t e = (gid - tn.start) * tn.vw;
    if (tn.vw == 4) adam_elems<T, 4>(a, tn, e);
    else if (tn.vw == 2) adam_elems<T, 2>(a, tn, e);
    else adam_elems<T, 1>(a, tn, e);
}

template <typename T>
static ab_status run_update(const ab_model_desc *d, ab_params *prm, const UpdatePlan &p, const float *x_raw,
                            const float *target, float lr, float beta1, float beta2, float eps,
                            float *loss_out, unsigned char *ws, int k0, hipStream_t st)
{
    // k0 = first trainable scorer layer (0: all; D: the output layer alone): layers below it are only run forward
    const int dt = p.dtype, D = p.D;
    const int64_t B = p.B, Bp = p.Bp;
    float *scal = (float *)(ws + p.off_scal);
    void *x = ws + p.off_x, *xt = ws + p.off_xt;
    float *yhat = (float *)(ws + p.off_yhat), *dout = (float *)(ws + p.off_dout);
    float *gw_out = (float *)(ws + p.off_gwout), *gb_out = (float *)(ws + p.off_gbout);

    const double esz = (double)elem_size(dt);
    {   // launch 1: rows -> x, x^T; padded copy of W_1, transposed hidden weights, zero padding; step counter
        EncodeRowsArgs e;
        memset(&e, 0, sizeof(e));
        e.x_raw = x_raw; e.x = x; e.x_t = xt; e.B = B; e.ld_t = Bp; e.F = p.F; e.ld = p.Kp; e.col_tiles = p.Kp / 64;
        e.n_stat = d->n_layers * d->n_stats; e.n_stats_per_layer = d->n_stats; e.n_scal = d->n_scalars;
        for (int i = 0; i < AB_MAX_STATS; ++i) e.enc_stat[i] = d->enc_stat[i];
        for (int i = 0; i < AB_MAX_SCALARS; ++i) e.enc_scal[i] = d->enc_scalar[i];
        e.enc_part = d->enc_partition; e.enc_cred = d->enc_credit;
        const unsigned enc_blocks = (unsigned)(Bp / 64) * (unsigned)e.col_tiles;

        UpdPrepArgs a;
        memset(&a, 0, sizeof(a));
        int64_t start = 0;
        auto add = [&](int kind, const void *src, void *dst, int rows, int cols, int ld_src, int ld_dst, int64_t n) {
            if (n <= 0) return;
            UpdPrepArgs::Job &j = a.job[a.n_jobs++];
            j.src = src; j.dst = dst; j.rows = rows; j.cols = cols; j.ld_src = ld_src; j.ld_dst = ld_dst;
            j.kind = kind; j.start = start; start += n;
        };
        add(JOB_PAD_COPY, prm->W[0], ws + p.off_wt[0], p.H[0], p.F, p.F, p.Kp, (int64_t)p.H[0] * p.Kp);
        for (int k = (k0 > 0 ? k0 + 1 : 1); k < D; ++k)      // W_k^T is the operand of the delta of layer k - 1
            add(JOB_TRANSPOSE, prm->W[k], ws + p.off_wt[k], p.H[k], p.H[k - 1], p.H[k - 1], p.H[k],
                (int64_t)p.H[k] * p.H[k - 1]);
        if (Bp > B) {                                        // (x^T gets its zero columns from the row transform)
            for (int k = 0; k < D; ++k) {
                add(JOB_ZERO_COLS, nullptr, ws + p.off_ht[k], p.H[k], (int)B, 0, (int)Bp, (int64_t)p.H[k] * (Bp - B));
                add(JOB_ZERO_COLS, nullptr, ws + p.off_dt[k], p.H[k], (int)B, 0, (int)Bp, (int64_t)p.H[k] * (Bp - B));
            }
        }
        a.total = start;
        a.step = prm->step; a.scal = scal; a.beta1 = beta1; a.beta2 = beta2;
        const unsigned prep_blocks = (unsigned)((start + 255) / 256 > 0 ? (start + 255) / 256 : 1);
        TraceScope ts("upd_encode_prep", (double)B * (p.F * 4.0 + 2.0 * p.Kp * esz) + 2.0 * (double)start * esz, 1, st);
        update_first_kernel<T><<<enc_blocks + prep_blocks, 256, 0, st>>>(e, a, enc_blocks);
        AB_HIP(hipGetLastError());
    }
    if (D == 0) {
        // no hidden layer: the output layer acts on the transformed rows themselves.  Forward + deltas, then the
        // weight and bias gradients from x^T (one work-group per input column), then Adam: four launches in all.
        {
            LinFwdArgs a{x, prm->W[0], prm->b[0], target, yhat, dout, (float *)(ws + p.off_lossrow), B, p.Kp, p.F, p.n_out,
                         d->loss_kind};
            TraceScope ts("upd_output_forward", (double)B * p.Kp * esz, 1, st);
            linear_forward_kernel<T><<<(unsigned)((B + 3) / 4), 256, 0, st>>>(a);
            AB_HIP(hipGetLastError());
        }
        {
            GroupArgs ga;
            memset(&ga, 0, sizeof(ga));
            ga.kind[2] = UJ_OUT_GRAD;
            ga.og = OutGradArgs{xt, prm->W[0], dout, (const float *)(ws + p.off_lossrow), nullptr, gw_out, gb_out, loss_out,
                                B, Bp, p.F, p.n_out, d->loss_kind};
            ga.start[3] = (unsigned)p.F + (unsigned)p.n_out + 1;
            TraceScope ts("upd_output_grad", (double)B * p.Kp * esz, 1, st);
            update_group_kernel<T><<<ga.start[3], 256, 2 * 128 * 128, st>>>(ga);
            AB_HIP(hipGetLastError());
        }
        AdamArgs a;
        memset(&a, 0, sizeof(a));
        auto add = [&](float *w, float *m, float *v, void *wc, const float *g, int rows, int cols, int64_t start) {
            AdamArgs::Tn &t = a.tn[a.n++];
            t.w = w; t.m = m; t.v = v; t.w_compute = wc; t.g = g; t.rows = rows; t.cols = cols; t.ldg = cols;
            t.splits = 1; t.split_stride = 0; t.vw = 1; t.start = start;
        };
        add(prm->W_master[0], prm->adam_mW[0], prm->adam_vW[0], (void *)prm->W[0], gw_out, p.n_out, p.F, 0);
        add(prm->b[0], prm->adam_mb[0], prm->adam_vb[0], nullptr, gb_out, 1, p.n_out, (int64_t)p.n_out * p.F);
        a.total = (int64_t)p.n_out * p.F + p.n_out; a.scal = scal; a.lr = lr; a.beta1 = beta1; a.beta2 = beta2; a.eps = eps;
        TraceScope ts("upd_adam", (double)a.total * (28.0 + esz), 1, st);
        adam_kernel<T><<<(unsigned)((a.total + 255) / 256), 256, 0, st>>>(a);
        AB_HIP(hipGetLastError());
        return AB_OK;
    }
    // forward
    for (int k = 0; k < D; ++k) {
        GemmArgs g;
        memset(&g, 0, sizeof(g));
        g.A = (k == 0) ? x : (void *)(ws + p.off_h[k - 1]);
        g.lda = p.in_w[k];
        g.B = (k == 0) ? (const void *)(ws + p.off_wt[0]) : prm->W[k];
        g.ldb = p.in_w[k];
        g.M = B; g.N = p.H[k]; g.K = p.in_w[k];
        g.bias = prm->b[k]; g.relu = 1;
        g.out = ws + p.off_h[k]; g.ldo = p.H[k];
        g.out_t = ws + p.off_ht[k]; g.ldo_t = Bp;
        TraceScope ts("upd_gemm_fwd", 2.0 * B * p.H[k] * p.in_w[k], 0, st);
        AB_HIP(launch_gemm(dt, update_tile(B, p.H[k]), AMODE_LOAD, EPI_STORE, g, st));
    }
    {
        OutFwdArgs a{ws + p.off_h[D - 1], prm->W[D], prm->b[D], target, yhat, dout, (float *)(ws + p.off_lossrow),
                     ws + p.off_d[D - 1], B, p.H[D - 1], p.n_out, d->loss_kind};
        TraceScope ts("upd_output_forward", (double)B * p.H[D - 1] * 3.0 * esz, 1, st);
        output_forward_kernel<T><<<(unsigned)((B + 3) / 4), 256, 0, st>>>(a);
        AB_HIP(hipGetLastError());
    }

    // backward: the chain delta_{D-1} -> delta_{D-2} -> ... sets the number of launches; everything else rides
    // along.  Launch i holds the delta product of layer D-1-i (while that layer is above k0), the weight gradient
    // of layer D-i (its delta^T was written one launch earlier) and, in launch 0, the output unit's gradients;
    // the last launch holds the weight gradients still open and the bias gradients.
    auto dw_args = [&](int k) {
        GemmArgs g;
        memset(&g, 0, sizeof(g));
        g.A = ws + p.off_dt[k]; g.lda = Bp;
        g.B = (k == 0) ? xt : (void *)(ws + p.off_ht[k - 1]); g.ldb = Bp;
        g.M = p.H[k]; g.N = p.in_w[k]; g.K = (int32_t)Bp;
        g.out = ws + p.off_gw[k]; g.ldo = p.in_w[k];
        g.k_splits = p.splits[k]; g.split_stride = (int64_t)p.H[k] * p.in_w[k];
        return g;
    };
    auto dx_args = [&](int k) {                 // d_{k-1} = (d_k W_k) * [h_{k-1} > 0]
        GemmArgs g;
        memset(&g, 0, sizeof(g));
        g.A = ws + p.off_d[k]; g.lda = p.H[k];
        g.B = ws + p.off_wt[k]; g.ldb = p.H[k];
        g.M = B; g.N = p.H[k - 1]; g.K = p.H[k];
        g.mask = ws + p.off_h[k - 1]; g.ldmask = p.H[k - 1];
        g.out = ws + p.off_d[k - 1]; g.ldo = p.H[k - 1];
        g.out_t = ws + p.off_dt[k - 1]; g.ldo_t = Bp;
        return g;
    };
    struct Group {
        GroupArgs a; int n_gemm; double flops, bytes;
        Group() { memset(&a, 0, sizeof(a)); n_gemm = 0; flops = bytes = 0.0; }
    };
    // a product on 64 x 64 tiles joins the group; one that wants larger tiles (large batches) is launched alone
    auto add_gemm = [&](Group &gr, int kind, GemmArgs g, int tile, const char *name) -> hipError_t {
        const double fl = 2.0 * (double)g.M * g.N * g.K;
        if (tile != TILE_SMALL) {
            TraceScope ts(name, fl, 0, st);
            return launch_gemm(dt, tile, AMODE_LOAD, kind == UJ_GEMM_DRELU ? EPI_DRELU : EPI_SPLITK, g, st);
        }
        g.m_tiles = (g.M + 63) / 64;
        g.n_tiles = g.N / 64;
        int64_t blocks = (g.m_tiles + 7) / 8 * 8 * g.n_tiles;
        if (kind == UJ_GEMM_SPLITK) blocks *= g.k_splits;
        if (blocks > 0x3fffffffLL) return hipErrorInvalidValue;
        const int s = gr.n_gemm++;
        gr.a.kind[s] = kind; gr.a.gemm[s] = g;
        gr.a.start[s + 1] = gr.a.start[s] + (unsigned)blocks;
        gr.flops += fl;
        return hipSuccess;
    };
    auto launch_group = [&](Group &gr, const char *name) -> hipError_t {
        for (int s = gr.n_gemm; s < 2; ++s) gr.a.start[s + 1] = gr.a.start[s];
        unsigned extra = 0;
        if (gr.a.kind[2] == UJ_OUT_GRAD) extra = (unsigned)gr.a.og.H + (unsigned)gr.a.og.n_out + 1;
        else if (gr.a.kind[2] == UJ_BIAS_GRAD) extra = (unsigned)gr.a.bg.l[gr.a.bg.n - 1].start + (unsigned)gr.a.bg.l[gr.a.bg.n - 1].H;
        gr.a.start[3] = gr.a.start[2] + extra;
        if (gr.a.start[3] == 0) return hipSuccess;
        TraceScope ts(name, gr.n_gemm ? gr.flops : gr.bytes, gr.n_gemm ? 0 : 1, st);
        update_group_kernel<T><<<gr.a.start[3], 256, 2 * 128 * 128, st>>>(gr.a);
        return hipGetLastError();
    };

    const int n_dx = D - 1 - k0 > 0 ? D - 1 - k0 : 0;       // delta products: layers D-1 ... k0+1
    int next_dw = D - 1;                                    // weight gradients are taken in the order D-1, D-2, ...
    {
        Group gr;
        if (n_dx > 0) AB_HIP(add_gemm(gr, UJ_GEMM_DRELU, dx_args(D - 1), update_tile(B, p.H[D - 2]), "upd_gemm_dx"));
        gr.a.kind[2] = UJ_OUT_GRAD;
        gr.a.og = OutGradArgs{ws + p.off_ht[D - 1], prm->W[D], dout, (const float *)(ws + p.off_lossrow), ws + p.off_dt[D - 1], gw_out, gb_out,
                              loss_out, B, Bp, p.H[D - 1], p.n_out, d->loss_kind};
        gr.bytes = (double)B * p.H[D - 1] * 2.0 * esz;
        AB_HIP(launch_group(gr, n_dx > 0 ? "upd_gemm_dx_outgrad" : "upd_output_grad"));
    }
    for (int i = 1; i < n_dx; ++i) {
        Group gr;
        AB_HIP(add_gemm(gr, UJ_GEMM_DRELU, dx_args(D - 1 - i), update_tile(B, p.H[D - 2 - i]), "upd_gemm_dx"));
        AB_HIP(add_gemm(gr, UJ_GEMM_SPLITK, dw_args(next_dw), TILE_SMALL, "upd_gemm_dw"));
        --next_dw;
        AB_HIP(launch_group(gr, "upd_gemm_dx_dw"));
    }
    while (next_dw >= k0) {                                 // at most two products are still open here
        Group gr;
        AB_HIP(add_gemm(gr, UJ_GEMM_SPLITK, dw_args(next_dw), TILE_SMALL, "upd_gemm_dw"));
        --next_dw;
        if (next_dw >= k0) { AB_HIP(add_gemm(gr, UJ_GEMM_SPLITK, dw_args(next_dw), TILE_SMALL, "upd_gemm_dw")); --next_dw; }
        if (next_dw < k0) {
            BiasGradArgs &a = gr.a.bg;
            a.n = D - k0; a.B = B; a.Bp = Bp;
            int start = 0;
            for (int k = k0; k < D; ++k) {
                a.l[k - k0].dt = ws + p.off_dt[k]; a.l[k - k0].gb = (float *)(ws + p.off_gb[k]); a.l[k - k0].H = p.H[k];
                a.l[k - k0].start = start; start += p.H[k];
            }
            gr.a.kind[2] = UJ_BIAS_GRAD;
        }
        AB_HIP(launch_group(gr, "upd_gemm_dw_bias"));
    }
    {
        AdamArgs a;
        memset(&a, 0, sizeof(a));
        int64_t start = 0;
        auto add = [&](float *w, float *m, float *v, void *wc, const float *g, int rows, int cols, int ldg,
                       int splits, int64_t stride) {
            AdamArgs::Tn &t = a.tn[a.n++];
            t.w = w; t.m = m; t.v = v; t.w_compute = wc; t.g = g; t.rows = rows; t.cols = cols; t.ldg = ldg;
            t.splits = splits; t.split_stride = stride;
            // widest vector that divides the row length and the gradient rows' pitch and that every pointer is aligned to
            const uintptr_t ptrs = (uintptr_t)w | (uintptr_t)m | (uintptr_t)v | (uintptr_t)g | (uintptr_t)wc;
            t.vw = (cols % 4 == 0 && ldg % 4 == 0 && stride % 4 == 0 && ptrs % 16 == 0) ? 4
                 : (cols % 2 == 0 && ldg % 2 == 0 && stride % 2 == 0 && ptrs % 8 == 0) ? 2 : 1;
            t.start = start; start += (int64_t)rows * cols / t.vw;
        };
        for (int k = k0; k < D; ++k) {
            const int cols = (k == 0) ? p.F : p.H[k - 1];
            add(prm->W_master[k], prm->adam_mW[k], prm->adam_vW[k], (void *)prm->W[k], (float *)(ws + p.off_gw[k]),
                p.H[k], cols, p.in_w[k], p.splits[k], (int64_t)p.H[k] * p.in_w[k]);
            add(prm->b[k], prm->adam_mb[k], prm->adam_vb[k], nullptr, (float *)(ws + p.off_gb[k]), 1, p.H[k], p.H[k], 1, 0);
        }
        add(prm->W_master[D], prm->adam_mW[D], prm->adam_vW[D], (void *)prm->W[D], gw_out, p.n_out, p.H[D - 1], p.H[D - 1], 1, 0);
        add(prm->b[D], prm->adam_mb[D], prm->adam_vb[D], nullptr, gb_out, 1, p.n_out, p.n_out, 1, 0);
        a.total = start; a.scal = scal; a.lr = lr; a.beta1 = beta1; a.beta2 = beta2; a.eps = eps;
        double n_param = 0.0;
        for (int i = 0; i < a.n; ++i) n_param += (double)a.tn[i].rows * a.tn[i].cols;
        TraceScope ts("upd_adam", n_param * (28.0 + esz), 1, st);
        adam_kernel<T><<<(unsigned)((start + 255) / 256), 256, 0, st>>>(a);
        AB_HIP(hipGetLastError());
    }
    return AB_OK;
}

// Minibatch assembled from two pools of raw rows (fresh observations and the offline set): one wavefront per
// output row, 16-byte pieces where the row width allows.  An index outside its pool gives a NaN row.
struct ReplayMixArgs {
    const float *x_new, *t_new, *x_old, *t_old; const int32_t *pick;
    float *x_out, *t_out; int64_t n_new, n_old, B; int32_t F, n_out;
};
__global__ __launch_bounds__(256) void replay_mix_kernel(const ReplayMixArgs a)
{
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= a.B) return;
    const int lane = threadIdx.x & 63;
    const int64_t pk = a.pick[row];
    const float *src = nullptr, *ts = nullptr;
    if (pk >= 0) { if (pk < a.n_new) { src = a.x_new + pk * a.F; ts = a.t_new + pk * a.n_out; } }
    else { const int64_t o = -pk - 1; if (o < a.n_old) { src = a.x_old + o * a.F; ts = a.t_old + o * a.n_out; } }
    float *dst = a.x_out + row * a.F;
    const float nanv = __uint_as_float(0x7fc00000u);
    if ((a.F & 3) == 0 && src && (((uintptr_t)src | (uintptr_t)dst) & 15) == 0) {
        for (int j = lane; j < a.F / 4; j += 64) ((f32x4 *)dst)[j] = ((const f32x4 *)src)[j];
    } else {
        for (int j = lane; j < a.F; j += 64) dst[j] = src ? src[j] : nanv;
    }
    if (lane < a.n_out) a.t_out[row * a.n_out + lane] = ts ? ts[lane] : nanv;
}

hipError_t launch_replay_mix(const float *x_new, const float *t_new, int64_t n_new, const float *x_old,
                             const float *t_old, int64_t n_old, const int32_t *pick, int64_t B, int32_t F,
                             int32_t n_out, float *x_out, float *t_out, hipStream_t st)
{
    if (B == 0) return hipSuccess;
    ReplayMixArgs a{x_new, t_new, x_old, t_old, pick, x_out, t_out, n_new, n_old, B, F, n_out};
    replay_mix_kernel<<<(unsigned)((B + 3) / 4), 256, 0, st>>>(a);
    return hipGetLastError();
}

ab_status online_update(const ab_model_desc *d, ab_params *prm, const float *x_raw, const float *target,
                        int64_t B, float lr, float beta1, float beta2, float eps, float *loss_out,
                        void *workspace, size_t ws_bytes, int first_trainable, hipStream_t st)
{
    if (B > (1 << 24)) return AB_ERR_UNSUPPORTED;
    UpdatePlan p;
    plan_update(d, B, &p);
    // the Adam launch numbers a tensor's elements with 32 bits: the first layer's weight matrix must stay below 2^32
    if ((int64_t)d->hidden[0] * ((int64_t)d->n_layers * d->n_stats + d->n_scalars + 2) >= (1LL << 32))
        return AB_ERR_UNSUPPORTED;
    if (first_trainable < 0 || first_trainable > p.D) return AB_ERR_SHAPE;
    if (!prm->step) return AB_ERR_NULL;
    for (int k = 0; k <= p.D; ++k) {
        if (!prm->W[k] || !prm->b[k]) return AB_ERR_NULL;
        if ((uintptr_t)prm->W[k] % 16) return AB_ERR_ALIGN;
        if (k < first_trainable) continue;                 // frozen layers need no master copy and no moments
        if (!prm->W_master[k] || !prm->adam_mW[k] || !prm->adam_vW[k] || !prm->adam_mb[k] || !prm->adam_vb[k])
            return AB_ERR_NULL;
        if ((uintptr_t)prm->W_master[k] % 4) return AB_ERR_ALIGN;
    }
    if (((uintptr_t)prm->step % 8) || ((uintptr_t)x_raw % 4) || ((uintptr_t)target % 4) ||
        ((uintptr_t)loss_out % 4)) return AB_ERR_ALIGN;
    if (!workspace || ws_bytes < p.total) return AB_ERR_WORKSPACE;
    if ((uintptr_t)workspace % 256) return AB_ERR_ALIGN;
    if (!(beta1 >= 0.f && beta1 < 1.f && beta2 >= 0.f && beta2 < 1.f)) return AB_ERR_SHAPE;
    unsigned char *ws = (unsigned char *)workspace;
    if (p.dtype == AB_BF16)
        return run_update<bf16_t>(d, prm, p, x_raw, target, lr, beta1, beta2, eps, loss_out, ws, first_trainable, st);
    return run_update<float>(d, prm, p, x_raw, target, lr, beta1, beta2, eps, loss_out, ws, first_trainable, st);
}

}  // namespace ab
