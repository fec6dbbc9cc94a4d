// Tiled C = A * B^T on the CDNA4 matrix cores, shared by the scoring and the update kernels.
//
// Both operands are "K-contiguous": A is [M, K] row-major (activations), B is [N, K] row-major
// (a dense layer's weight matrix W[out, in]), so a layer h W^T needs no transposition anywhere.
//
// Work-group: 256 threads = 4 wavefronts in a 2 x 2 arrangement; each wavefront owns WMB x WNB
// blocks of 32 x 32 outputs, i.e. the work-group tile is (64*WMB) x (64*WNB).  A K-slab is 128 bytes
// per row (64 bf16 or 32 fp32) and is kept in LDS as rows of eight 16-byte chunks; chunk c of row r
// sits at position c ^ ((r >> 1) & 7), which makes both the 16-byte row-wise writes and the
// 16-byte column-of-rows operand reads spread over all banks.
//
// Matrix-core operand convention used here: for the 32x32 instructions lane l supplies row
// (l & 31) of its operand and the K positions selected by (l >> 5); since both operands use the
// same K assignment any consistent assignment is valid, so each lane simply takes one 16-byte
// chunk (8 bf16 -> one 32x32x16 instruction, 4 fp32 -> four 32x32x2 instructions).
// The 32x32 result holds, in register r of lane l, row 8*(r/4) + 4*(l>>5) + (r&3) and column (l&31).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ab {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) int i32x4;

struct bf16_t { uint16_t bits; };   // storage type of a bfloat16 value

// ReLU that lets NaN through, so a non-finite statistic stays visible in the scores.
// max(v, 0) that hands a NaN on (IEEE 754-2019 maximum; one v_maximum3_f32 on this target)
__device__ __forceinline__ float relu_keep_nan(float v) { return __builtin_elementwise_maximum(v, 0.f); }

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    f32x2 v = {lo, hi};
    bf16x2 b = __builtin_convertvector(v, bf16x2);   // round to nearest even
    return __builtin_bit_cast(uint32_t, b);
}
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

enum { AMODE_LOAD = 0, AMODE_GEN = 1, AMODE_GENV = 2 };
enum { EPI_STORE = 0, EPI_SCORE = 1, EPI_DRELU = 2, EPI_SPLITK = 3 };

struct GemmArgs {
    // A operand, AMODE_LOAD: A[M, K] with leading dimension lda (elements of the compute type)
    const void *A; int64_t lda;
    // A operand, AMODE_GEN: row r stands for (scenario s = r / C, candidate c = r % C) and
    // A[r, k] = relu(a_term[s*ldt + k] + b_term[c*ldt + k]) rounded to the compute type
    const float *a_term; const float *b_term; int32_t ldt; int32_t C;
    // the same b_term in factored form, b_term[c*ldt + k] = wp[k]*xp[c] + wc[k]*xc[c] (256x256 kernel);
    // with x_per_row the two candidate vectors are indexed by the row r instead (xp[r], xc[r]: every scenario
    // has its own candidate values).  AMODE_GENV: the generic tiles' form of the factored operand
    const float *wp, *wc, *xp, *xc; int32_t x_per_row;
    int32_t xp_runs4;                         // rows 4j .. 4j+3 of the product take the same xp (the grid's credit
                                              // count is a multiple of 4): lets a thread share wp*xp + a_term over them
    // B operand: B[N, K], leading dimension ldb
    const void *B; int64_t ldb;
    int64_t M; int32_t N; int32_t K;          // K is a multiple of the K-slab; N a multiple of the tile width
    int64_t m_tiles; int32_t n_tiles;
    // epilogue
    const float *bias; int32_t relu;          // EPI_STORE: out = act(acc + bias)
    void *out; int64_t ldo; int32_t out_f32;  // EPI_STORE / EPI_DRELU: compute type or fp32 output
    void *out_t; int64_t ldo_t;               // optional transposed copy out_t[col, row] (compute type);
                                              // ldo_t a multiple of 4 and out_t 16-byte aligned
    const float *w_out; float *partial;       // EPI_SCORE: partial[row*n_tiles + tile_n] = sum_col relu(acc+bias)*w_out
    const void *mask; int64_t ldmask;         // EPI_DRELU: out = acc * (mask[row, col] > 0)
    int32_t k_splits; int64_t split_stride;   // EPI_SPLITK: fp32 out + split*split_stride, K range split evenly
};

template <typename T> struct TileTraits;
template <> struct TileTraits<bf16_t> { static constexpr int BK = 64, EPC = 8; };
template <> struct TileTraits<float>  { static constexpr int BK = 32, EPC = 4; };

template <typename T>
__device__ __forceinline__ void mma_chunk(const i32x4 &a, const i32x4 &b, f32x16 &acc)
{
    if constexpr (sizeof(T) == 2) {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                      __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
    } else {
        f32x4 fa = __builtin_bit_cast(f32x4, a), fb = __builtin_bit_cast(f32x4, b);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa.x, fb.x, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa.y, fb.y, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa.z, fb.z, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa.w, fb.w, acc, 0, 0, 0);
    }
}

// relu(a + b) for one 16-byte chunk of the generated operand.
template <typename T>
__device__ __forceinline__ i32x4 gen_chunk(const float *pa, const float *pb)
{
    if constexpr (sizeof(T) == 2) {
        f32x4 a0 = *(const f32x4 *)pa, a1 = *(const f32x4 *)(pa + 4);
        f32x4 b0 = *(const f32x4 *)pb, b1 = *(const f32x4 *)(pb + 4);
        i32x4 r;
        r.x = (int)pack_bf16x2(relu_keep_nan(a0.x + b0.x), relu_keep_nan(a0.y + b0.y));
        r.y = (int)pack_bf16x2(relu_keep_nan(a0.z + b0.z), relu_keep_nan(a0.w + b0.w));
        r.z = (int)pack_bf16x2(relu_keep_nan(a1.x + b1.x), relu_keep_nan(a1.y + b1.y));
        r.w = (int)pack_bf16x2(relu_keep_nan(a1.z + b1.z), relu_keep_nan(a1.w + b1.w));
        return r;
    } else {
        f32x4 a0 = *(const f32x4 *)pa, b0 = *(const f32x4 *)pb;
        f32x4 v = {relu_keep_nan(a0.x + b0.x), relu_keep_nan(a0.y + b0.y),
                   relu_keep_nan(a0.z + b0.z), relu_keep_nan(a0.w + b0.w)};
        return __builtin_bit_cast(i32x4, v);
    }
}

// relu(a + wp * xp + wc * xc) for one 16-byte chunk of the generated operand in its factored form.
template <typename T>
__device__ __forceinline__ i32x4 gen_chunk_v(const float *pa, const float *pp, const float *pc, float xp, float xc)
{
    if constexpr (sizeof(T) == 2) {
        float h[8];
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const f32x4 a = *(const f32x4 *)(pa + 4 * q), wp = *(const f32x4 *)(pp + 4 * q), wc = *(const f32x4 *)(pc + 4 * q);
#pragma unroll
            for (int e = 0; e < 4; ++e) h[4 * q + e] = relu_keep_nan(fmaf(wc[e], xc, fmaf(wp[e], xp, a[e])));
        }
        i32x4 r;
        r.x = (int)pack_bf16x2(h[0], h[1]); r.y = (int)pack_bf16x2(h[2], h[3]);
        r.z = (int)pack_bf16x2(h[4], h[5]); r.w = (int)pack_bf16x2(h[6], h[7]);
        return r;
    } else {
        const f32x4 a = *(const f32x4 *)pa, wp = *(const f32x4 *)pp, wc = *(const f32x4 *)pc;
        f32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = relu_keep_nan(fmaf(wc[e], xc, fmaf(wp[e], xp, a[e])));
        return __builtin_bit_cast(i32x4, v);
    }
}

// The value another lane holds, by a DPP control word; lanes of rows not in ROW_MASK receive 0.
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ float dpp_move(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xF, false));
}

// Sum over the 64 lanes of a wavefront, returned to every lane: four exchanges inside the rows of sixteen, two
// row broadcasts, one read of lane 63 (no LDS round trips).
__device__ __forceinline__ float wave_sum(float v)
{
    v += dpp_move<0xB1>(v);
    v += dpp_move<0x4E>(v);
    v += dpp_move<0x141>(v);
    v += dpp_move<0x140>(v);
    v += dpp_move<0x142, 0xA>(v);    // row_bcast:15
    v += dpp_move<0x143, 0xC>(v);    // row_bcast:31
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

template <typename T>
__device__ __forceinline__ void store_elem(void *base, int64_t idx, float v, int as_f32)
{
    if (sizeof(T) == 4 || as_f32) ((float *)base)[idx] = v;
    else ((uint16_t *)base)[idx] = (uint16_t)(pack_bf16x2(v, 0.f) & 0xffffu);
}

// One work-group's tile of the product: `id` is the work-group's number within the product's launch (or
// within its share of a launch that holds several products), `smem` 2 * (BM + BN) * 128 bytes of LDS.
template <typename T, int WMB, int WNB, int AMODE, int EPI>
__device__ __forceinline__ void gemm_tn_tile(const GemmArgs &g, int64_t id, unsigned char *smem)
{
    constexpr int BM = 64 * WMB, BN = 64 * WNB;
    constexpr int BK = TileTraits<T>::BK, EPC = TileTraits<T>::EPC;
    constexpr int A_CH = BM / 32, B_CH = BN / 32;        // 16-byte chunks per thread per slab
    constexpr int STAGE_BYTES = (BM + BN) * 128;

    // Work-group -> tile.  Consecutive work-group ids go to consecutive XCDs, so the n_tiles tiles
    // that share one panel of A are given ids that land on the same XCD (same L2) back to back.
    int split = 0;
    if constexpr (EPI == EPI_SPLITK) { split = (int)(id % g.k_splits); id /= g.k_splits; }
    const int xcd = (int)(id & 7);
    const int64_t local = id >> 3;
    const int tn = (int)(local % g.n_tiles);
    const int64_t tm = (local / g.n_tiles) * 8 + xcd;
    if (tm >= g.m_tiles) return;

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wave_m = wave >> 1, wave_n = wave & 1;
    const int64_t m0 = tm * BM;
    const int n0 = tn * BN;
    const int ld_row = t >> 3, ld_cc = t & 7;

    int kt_begin = 0, kt_end = g.K / BK;
    if constexpr (EPI == EPI_SPLITK) {
        const int per = (kt_end + g.k_splits - 1) / g.k_splits;
        kt_begin = split * per;
        kt_end = min(kt_end, kt_begin + per);
    }

    // per-thread source offsets (elements) of its chunks within the A panel / B panel
    int32_t a_off[A_CH], a2_off[A_CH], b_off[B_CH];
    float gx_p[A_CH], gx_c[A_CH];             // AMODE_GENV: this thread's rows' candidate values
    const T *Ab = nullptr;
    if constexpr (AMODE == AMODE_LOAD) {
        Ab = (const T *)g.A + m0 * g.lda;
#pragma unroll
        for (int i = 0; i < A_CH; ++i) {
            int64_t r = min((int64_t)(ld_row + i * 32), g.M - 1 - m0);
            a_off[i] = (int32_t)(r * g.lda) + ld_cc * EPC;
            a2_off[i] = 0;
        }
    } else {
#pragma unroll
        for (int i = 0; i < A_CH; ++i) {
            int64_t r = min(m0 + ld_row + i * 32, g.M - 1);
            int64_t s = r / g.C;
            int32_t c = (int32_t)(r - s * g.C);
            a_off[i] = (int32_t)s * g.ldt + ld_cc * EPC;
            a2_off[i] = c * g.ldt + ld_cc * EPC;
            if constexpr (AMODE == AMODE_GENV) {
                gx_p[i] = g.xp[g.x_per_row ? r : (int64_t)c];
                gx_c[i] = g.xc[g.x_per_row ? r : (int64_t)c];
            }
        }
    }
    const T *Bb = (const T *)g.B + (int64_t)n0 * g.ldb;
#pragma unroll
    for (int i = 0; i < B_CH; ++i) b_off[i] = (int32_t)((ld_row + i * 32) * g.ldb) + ld_cc * EPC;

    // LDS positions
    int32_t st_off[(A_CH > B_CH ? A_CH : B_CH)];
#pragma unroll
    for (int i = 0; i < (A_CH > B_CH ? A_CH : B_CH); ++i) {
        const int r = ld_row + i * 32;
        st_off[i] = r * 128 + ((ld_cc ^ ((r >> 1) & 7)) << 4);
    }
    const int sw = ((lane & 31) >> 1) & 7, half = lane >> 5;
    int32_t rd_off[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) rd_off[q] = (lane & 31) * 128 + ((((q << 1) | half) ^ sw) << 4);
    const int a_rd_base = wave_m * (WMB * 32) * 128;
    const int b_rd_base = BM * 128 + wave_n * (WNB * 32) * 128;

    f32x16 acc[WMB][WNB];
#pragma unroll
    for (int i = 0; i < WMB; ++i)
#pragma unroll
        for (int j = 0; j < WNB; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // With fp32 the generated operand is kept raw in registers (its two addends, or the scenario term and
    // the slab's wp / wc chunks) and combined when the slab is written to LDS, after the matrix work of the
    // slab before: all of a slab's loads are then in flight together instead of being waited for one by one.
    constexpr bool RAW_GEN = AMODE != AMODE_LOAD && sizeof(T) == 4;
    i32x4 ra[A_CH], rb[B_CH];
    i32x4 ra2[RAW_GEN && AMODE == AMODE_GEN ? A_CH : 1];
    f32x4 rwp = {0.f, 0.f, 0.f, 0.f}, rwc = {0.f, 0.f, 0.f, 0.f};

    auto load_slab = [&](int kt) {
        const int k0 = kt * BK;
        if constexpr (AMODE == AMODE_LOAD) {
#pragma unroll
            for (int i = 0; i < A_CH; ++i) ra[i] = *(const i32x4 *)(Ab + a_off[i] + k0);
        } else if constexpr (RAW_GEN) {
#pragma unroll
            for (int i = 0; i < A_CH; ++i) ra[i] = *(const i32x4 *)(g.a_term + a_off[i] + k0);
            if constexpr (AMODE == AMODE_GEN) {
#pragma unroll
                for (int i = 0; i < A_CH; ++i) ra2[i] = *(const i32x4 *)(g.b_term + a2_off[i] + k0);
            } else {
                rwp = *(const f32x4 *)(g.wp + ld_cc * EPC + k0);
                rwc = *(const f32x4 *)(g.wc + ld_cc * EPC + k0);
            }
        } else if constexpr (AMODE == AMODE_GEN) {
#pragma unroll
            for (int i = 0; i < A_CH; ++i)
                ra[i] = gen_chunk<T>(g.a_term + a_off[i] + k0, g.b_term + a2_off[i] + k0);
        } else {
#pragma unroll
            for (int i = 0; i < A_CH; ++i)
                ra[i] = gen_chunk_v<T>(g.a_term + a_off[i] + k0, g.wp + ld_cc * EPC + k0, g.wc + ld_cc * EPC + k0,
                                       gx_p[i], gx_c[i]);
        }
#pragma unroll
        for (int i = 0; i < B_CH; ++i) rb[i] = *(const i32x4 *)(Bb + b_off[i] + k0);
    };
    auto store_slab = [&](int stage) {
        unsigned char *sa = smem + stage * STAGE_BYTES, *sb = sa + BM * 128;
#pragma unroll
        for (int i = 0; i < A_CH; ++i) {
            i32x4 v = ra[i];
            if constexpr (RAW_GEN) {
                const f32x4 a = __builtin_bit_cast(f32x4, ra[i]);
                f32x4 h;
                if constexpr (AMODE == AMODE_GEN) {
                    const f32x4 b = __builtin_bit_cast(f32x4, ra2[i]);
#pragma unroll
                    for (int e = 0; e < 4; ++e) h[e] = relu_keep_nan(a[e] + b[e]);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) h[e] = relu_keep_nan(fmaf(rwc[e], gx_c[i], fmaf(rwp[e], gx_p[i], a[e])));
                }
                v = __builtin_bit_cast(i32x4, h);
            }
            *(i32x4 *)(sa + st_off[i]) = v;
        }
#pragma unroll
        for (int i = 0; i < B_CH; ++i) *(i32x4 *)(sb + st_off[i]) = rb[i];
    };
    auto compute_slab = [&](int stage) {
        const unsigned char *sa = smem + stage * STAGE_BYTES + a_rd_base;
        const unsigned char *sb = smem + stage * STAGE_BYTES + b_rd_base;
        if constexpr (sizeof(T) == 4 && WMB * WNB == 16) {
            // one wavefront per SIMD here, so nothing else hides the LDS latency: the operands of quarter q + 1
            // are requested before the matrix instructions of quarter q (two register sets)
            i32x4 fa[2][WMB], fb[2][WNB];
            auto fetch = [&](int q, int set) {
#pragma unroll
                for (int i = 0; i < WMB; ++i) fa[set][i] = *(const i32x4 *)(sa + i * 4096 + rd_off[q]);
#pragma unroll
                for (int j = 0; j < WNB; ++j) fb[set][j] = *(const i32x4 *)(sb + j * 4096 + rd_off[q]);
            };
            fetch(0, 0);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (q < 3) fetch(q + 1, (q + 1) & 1);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < WMB; ++i)
#pragma unroll
                    for (int j = 0; j < WNB; ++j) mma_chunk<T>(fa[q & 1][i], fb[q & 1][j], acc[i][j]);
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                i32x4 fa[WMB], fb[WNB];
#pragma unroll
                for (int i = 0; i < WMB; ++i) fa[i] = *(const i32x4 *)(sa + i * 4096 + rd_off[q]);
#pragma unroll
                for (int j = 0; j < WNB; ++j) fb[j] = *(const i32x4 *)(sb + j * 4096 + rd_off[q]);
#pragma unroll
                for (int i = 0; i < WMB; ++i)
#pragma unroll
                    for (int j = 0; j < WNB; ++j) mma_chunk<T>(fa[i], fb[j], acc[i][j]);
            }
        }
    };

    const int row_l0 = wave_m * (WMB * 32) + half * 4;        // + i*32 + (r>>2)*8 + (r&3)
    const int col_l0 = wave_n * (WNB * 32) + (lane & 31);     // + j*32
    // What the epilogue of the 64 x 64 tile needs from memory is requested before the K loop (these launches are
    // short chains of memory round trips): the bias, or the sixteen mask values of this lane.
    constexpr bool PRE = WMB * WNB == 1 && (EPI == EPI_STORE || EPI == EPI_DRELU);
    float pre_bias = 0.f, pre_mask[PRE && EPI == EPI_DRELU ? 16 : 1];
    if constexpr (PRE && EPI == EPI_STORE) pre_bias = g.bias ? g.bias[n0 + col_l0] : 0.f;
    // the output unit's epilogue: bias and output weight of this lane's columns, likewise asked for up front
    float pre_b[EPI == EPI_SCORE ? WNB : 1], pre_w[EPI == EPI_SCORE ? WNB : 1];
    if constexpr (EPI == EPI_SCORE) {
#pragma unroll
        for (int j = 0; j < WNB; ++j) {
            pre_b[j] = g.bias[n0 + col_l0 + j * 32];
            pre_w[j] = g.w_out[n0 + col_l0 + j * 32];
        }
    }
    if constexpr (PRE && EPI == EPI_DRELU) {
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const int64_t row = min(m0 + row_l0 + (q >> 2) * 8 + (q & 3), g.M - 1);
            if constexpr (sizeof(T) == 2) pre_mask[q] = bf16_bits_to_f32(((const uint16_t *)g.mask)[row * g.ldmask + n0 + col_l0]);
            else pre_mask[q] = ((const float *)g.mask)[row * g.ldmask + n0 + col_l0];
        }
    }

    if (kt_begin < kt_end) {
        load_slab(kt_begin);
        store_slab(0);
        __syncthreads();
        for (int kt = kt_begin; kt < kt_end; ++kt) {
            const int cur = (kt - kt_begin) & 1;
            if (kt + 1 < kt_end) load_slab(kt + 1);
            compute_slab(cur);
            if (kt + 1 < kt_end) store_slab(cur ^ 1);
            __syncthreads();
        }
    }

    // ---------------------------------------------------------------- epilogues
    if constexpr (EPI == EPI_STORE || EPI == EPI_DRELU || EPI == EPI_SPLITK) {
        float *out_split = nullptr;
        if constexpr (EPI == EPI_SPLITK) out_split = (float *)g.out + (int64_t)split * g.split_stride;
#pragma unroll
        for (int j = 0; j < WNB; ++j) {
            const int col = n0 + col_l0 + j * 32;
            float bv = 0.f;
            if constexpr (EPI == EPI_STORE) { if constexpr (PRE) bv = pre_bias; else bv = g.bias ? g.bias[col] : 0.f; }
#pragma unroll
            for (int i = 0; i < WMB; ++i)
#pragma unroll
                for (int rg = 0; rg < 4; ++rg) {
                    // registers 4*rg .. 4*rg+3 of this block are four consecutive rows of one column
                    const int64_t row0 = m0 + row_l0 + i * 32 + rg * 8;
                    float v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        v[e] = acc[i][j][rg * 4 + e];
                        const int64_t row = row0 + e;
                        if constexpr (EPI == EPI_STORE) {
                            v[e] += bv;
                            if (g.relu) v[e] = relu_keep_nan(v[e]);
                        } else if constexpr (EPI == EPI_DRELU) {
                            if constexpr (PRE) {
                                v[e] = pre_mask[rg * 4 + e] > 0.f ? v[e] : 0.f;
                            } else if (row < g.M) {
                                float mk;
                                if constexpr (sizeof(T) == 2)
                                    mk = bf16_bits_to_f32(((const uint16_t *)g.mask)[row * g.ldmask + col]);
                                else
                                    mk = ((const float *)g.mask)[row * g.ldmask + col];
                                v[e] = mk > 0.f ? v[e] : 0.f;
                            }
                        }
                        if (row < g.M) {
                            if constexpr (EPI == EPI_SPLITK) out_split[row * g.ldo + col] = v[e];
                            else store_elem<T>(g.out, row * g.ldo + col, v[e], g.out_f32);
                        }
                    }
                    if constexpr (EPI != EPI_SPLITK) {
                        if (g.out_t) {
                            const int64_t o = (int64_t)col * g.ldo_t + row0;   // four rows are contiguous here
                            if (row0 + 3 < g.M) {
                                if constexpr (sizeof(T) == 2) {
                                    uint2 pk = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
                                    *(uint2 *)((uint16_t *)g.out_t + o) = pk;
                                } else {
                                    *(f32x4 *)((float *)g.out_t + o) = f32x4{v[0], v[1], v[2], v[3]};
                                }
                            } else {
#pragma unroll
                                for (int e = 0; e < 4; ++e)
                                    if (row0 + e < g.M) store_elem<T>(g.out_t, o + e, v[e], 0);
                            }
                        }
                    }
                }
        }
    } else {   // EPI_SCORE: per-row dot of relu(acc + bias) with w_out over this tile's columns
        float rs[WMB][16];
#pragma unroll
        for (int i = 0; i < WMB; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) rs[i][r] = 0.f;
#pragma unroll
        for (int j = 0; j < WNB; ++j) {
            const float bv = pre_b[j], wv = pre_w[j];
#pragma unroll
            for (int i = 0; i < WMB; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) rs[i][r] += relu_keep_nan(acc[i][j][r] + bv) * wv;
        }
        float *red = (float *)smem;    // [2][BM]; the K loop ended with a barrier, LDS is free
#pragma unroll
        for (int i = 0; i < WMB; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                // sum over the 32 lanes of a half (one row's columns) by DPP exchanges, no LDS round trips:
                // within a row of sixteen lanes every lane ends up with the row's sum, then lanes 16..31 of a
                // half take in the sum of lanes 0..15
                float v = rs[i][r];
                v += dpp_move<0xB1>(v);          // quad_perm 1,0,3,2
                v += dpp_move<0x4E>(v);          // quad_perm 2,3,0,1
                v += dpp_move<0x141>(v);         // row_half_mirror
                v += dpp_move<0x140>(v);         // row_mirror
                v += dpp_move<0x142, 0xA>(v);    // row_bcast:15 into the odd rows of sixteen
                if ((lane & 31) == 31) red[wave_n * BM + row_l0 + i * 32 + (r >> 2) * 8 + (r & 3)] = v;
            }
        __syncthreads();
        if (t < BM && m0 + t < g.M)
            g.partial[(m0 + t) * g.n_tiles + tn] = red[t] + red[BM + t];
    }
}

template <typename T, int WMB, int WNB, int AMODE, int EPI>
__global__ __launch_bounds__(256) void gemm_tn_kernel(const GemmArgs g)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    gemm_tn_tile<T, WMB, WNB, AMODE, EPI>(g, blockIdx.x, smem);
}

}  // namespace ab
