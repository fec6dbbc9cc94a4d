// The bf16 256 x 256 x 64 work-horse of the hidden-layer chain: C = A * B^T with A [M, K] (activations,
// or generated on the fly as relu(A[s] + B[c])) and B = W [N, K], both K-contiguous.
//
// Shape of the kernel
//   - 512 threads = 8 wavefronts (2 per SIMD, so one wavefront's LDS / global phases overlap the other's
//     matrix-core phase), arranged 2 (rows) x 4 (columns); each wavefront owns 128 rows x 64 columns.
//   - LDS holds a ring of three A slabs and a ring of two W slabs (256 rows x 128 bytes = 32 KB each,
//     160 KB in all).  A slab's stage is refilled right after the barrier that retires it, so W slabs
//     (L2 hits) are requested one slab ahead and A slabs (HBM / Infinity Cache) two slabs ahead.
//     Slabs that come straight from memory are written by the global->LDS DMA path (no registers, no
//     ds_write) in whole 128-byte row segments (64-byte segments halve the DMA rate); the generated
//     operand goes through registers.  Rows are eight 16-byte chunks; chunk c of row r sits at
//     position c ^ ((r >> 1) & 7).
//   - Operand roles are swapped with respect to the textbook order: the weight fragment is the matrix
//     instruction's first operand and the activation fragment its second, so in the 32x32 result a
//     lane holds ONE output row (lane & 31) and 16 output columns (register r -> column
//     8*(r/4) + 4*(lane>>5) + (r&3)).  Four consecutive registers are four consecutive columns: the
//     bf16 store packs them into 8 bytes, and the output-unit dot product is a per-lane sum.
//   - Fragments are double-buffered in registers; the barrier of a slab sits before its last quarter
//     so that the first fragments of the next slab are fetched under the last quarter's matrix work.
//     Waits on the DMA use exact vmcnt counts (loads retire in issue order), never a full drain.
//   - Stores go through an LDS staging tile (row stride 528 bytes) and leave as 16-byte, fully
//     coalesced writes.
#include "internal.hpp"

namespace ab {

typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void global_void;

// 64 lanes x 16 bytes; lane l's data lands at lds_uniform_dst + 16*l.  STREAM marks the access
// non-temporal: activation panels and outputs pass through L2 once per XCD and should not push the
// weight matrix (re-read by every tile) out of it.
template <bool STREAM>
__device__ __forceinline__ void dma16(const void *gsrc, void *lds_uniform_dst)
{
    __builtin_amdgcn_global_load_lds((global_void *)gsrc, (lds_void *)lds_uniform_dst, 16, 0, STREAM ? 2 : 0);
}

template <int AMODE, int EPI>
__global__ __launch_bounds__(512) void gemm_big_kernel(const GemmArgs g)
{
    constexpr int BM = 256, BN = 256, BK = 64;
    constexpr int SLAB = BM * 128;                         // 32 KB; BN == BM
    constexpr int W_BASE = 3 * SLAB;                       // A ring: stages 0..2, W ring: stages 0..1
    constexpr int OUT_STRIDE = 528;                       // bytes per staged output row (512 + 16 pad)
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    int64_t id = blockIdx.x;
    const int xcd = (int)(id & 7);
    const int64_t local = id >> 3;
    const int tn = (int)(local % g.n_tiles);
    const int64_t tm = (local / g.n_tiles) * 8 + xcd;
    if (tm >= g.m_tiles) return;

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wave_m = wave >> 2, wave_n = wave & 3;
    const int half = lane >> 5, l31 = lane & 31;
    const int64_t m0 = tm * BM;
    const int n0 = tn * BN;
    const int KT = g.K / BK;

    // ---- sources of this wavefront's DMA rows: row groups rg = wave + 8 i (8 rows each), i < 4
    const int dma_cc = (lane & 7) ^ ((wave & 1) * 4 + (lane >> 4));     // logical chunk this lane fetches
    const uint16_t *a_src[4];
    const uint16_t *w_src[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = (wave + 8 * i) * 8 + (lane >> 3);
        if constexpr (AMODE == AMODE_LOAD) {
            int64_t gr = m0 + r;
            if (gr > g.M - 1) gr = g.M - 1;
            a_src[i] = (const uint16_t *)g.A + gr * g.lda + dma_cc * 8;
        } else {
            a_src[i] = nullptr;
        }
        w_src[i] = (const uint16_t *)g.B + (int64_t)(n0 + r) * g.ldb + dma_cc * 8;
    }
    // ---- generated operand: thread -> chunks (row = t/8 + 64 i, logical chunk t & 7); one scenario per tile
    // A[r, k] = relu(a_term[s, k] + wp[k] * xp[c] + wc[k] * xc[c]): the per-row pair (xp, xc) stays in
    // registers, the three per-k vectors are fetched per slab (the same 8 values for all of a thread's rows)
    const float *gen_a = nullptr, *gen_wp = nullptr, *gen_wc = nullptr;
    float gen_xp[4], gen_xc[4];
    int gen_st[4];
    if constexpr (AMODE == AMODE_GEN) {
        const int64_t s = m0 / g.C;
        const int c0 = (int)(m0 - s * g.C);
        const int cc = t & 7;
        gen_a = g.a_term + s * g.ldt + cc * 8;
        gen_wp = g.wp + cc * 8;
        gen_wc = g.wc + cc * 8;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = (t >> 3) + 64 * i;
            gen_xp[i] = g.xp[c0 + r];
            gen_xc[i] = g.xc[c0 + r];
            gen_st[i] = r * 128 + ((cc ^ ((r >> 1) & 7)) << 4);
        }
    }

    // ---- fragment read offsets
    const int sw = (l31 >> 1) & 7;
    int rd[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) rd[q] = l31 * 128 + ((((q << 1) | half) ^ sw) << 4);
    const int a_rd = wave_m * 128 * 128;                   // + stage * SLAB + im * 4096
    const int w_rd = W_BASE + wave_n * 64 * 128;           // + stage * SLAB + jn * 4096

    f32x16 acc[2][4];
#pragma unroll
    for (int jn = 0; jn < 2; ++jn)
#pragma unroll
        for (int im = 0; im < 4; ++im)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[jn][im][r] = 0.f;

    f32x4 raw_a[2], raw_p[2], raw_c[2];
    auto dma_w = [&](int kt) {
        unsigned char *sb = smem + W_BASE + (kt & 1) * SLAB;
#pragma unroll
        for (int i = 0; i < 4; ++i) dma16<false>(w_src[i] + kt * BK, sb + (wave + 8 * i) * 1024);
    };
    auto dma_a = [&](int kt) {
        if constexpr (AMODE == AMODE_LOAD) {
            unsigned char *sb = smem + (kt % 3) * SLAB;
#pragma unroll
            for (int i = 0; i < 4; ++i) dma16<true>(a_src[i] + kt * BK, sb + (wave + 8 * i) * 1024);
        }
    };
    auto issue_raw = [&](int kt) {
        if constexpr (AMODE == AMODE_GEN) {
            const int k0 = kt * BK;
            raw_a[0] = *(const f32x4 *)(gen_a + k0);
            raw_a[1] = *(const f32x4 *)(gen_a + k0 + 4);
            raw_p[0] = *(const f32x4 *)(gen_wp + k0);
            raw_p[1] = *(const f32x4 *)(gen_wp + k0 + 4);
            raw_c[0] = *(const f32x4 *)(gen_wc + k0);
            raw_c[1] = *(const f32x4 *)(gen_wc + k0 + 4);
        }
    };
    auto write_generated = [&](int kt) {
        if constexpr (AMODE == AMODE_GEN) {
            unsigned char *sa = smem + (kt % 3) * SLAB;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float xp = gen_xp[i], xc = gen_xc[i];
                float h[8];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    h[e] = relu_keep_nan(fmaf(raw_c[0][e], xc, fmaf(raw_p[0][e], xp, raw_a[0][e])));
                    h[4 + e] = relu_keep_nan(fmaf(raw_c[1][e], xc, fmaf(raw_p[1][e], xp, raw_a[1][e])));
                }
                i32x4 v;
                v.x = (int)pack_bf16x2(h[0], h[1]);
                v.y = (int)pack_bf16x2(h[2], h[3]);
                v.z = (int)pack_bf16x2(h[4], h[5]);
                v.w = (int)pack_bf16x2(h[6], h[7]);
                *(i32x4 *)(sa + gen_st[i]) = v;
            }
        }
    };

    i32x4 fa[2][4], fw[2][2];
    auto load_frags = [&](int kt, int q, int set) {
        const unsigned char *sa = smem + (kt % 3) * SLAB + a_rd;
        const unsigned char *sw_ = smem + (kt & 1) * SLAB + w_rd;
#pragma unroll
        for (int jn = 0; jn < 2; ++jn) fw[set][jn] = *(const i32x4 *)(sw_ + jn * 4096 + rd[q]);
#pragma unroll
        for (int im = 0; im < 4; ++im) fa[set][im] = *(const i32x4 *)(sa + im * 4096 + rd[q]);
    };
    auto mma = [&](int set) {
#pragma unroll
        for (int jn = 0; jn < 2; ++jn)
#pragma unroll
            for (int im = 0; im < 4; ++im)
                acc[jn][im] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    __builtin_bit_cast(bf16x8, fw[set][jn]), __builtin_bit_cast(bf16x8, fa[set][im]),
                    acc[jn][im], 0, 0, 0);
    };

    // Scheduling hints: keep the source order of the phases (fence) and, inside a phase, alternate one
    // matrix instruction with one LDS fragment read so the reads for the next quarter are issued under
    // the current quarter's matrix work instead of being sunk in front of their first use.
#define AB_FENCE() __builtin_amdgcn_sched_barrier(0)
#define AB_MFMA_DS_PAIR() do { __builtin_amdgcn_sched_group_barrier(0x008, 1, 0); \
                               __builtin_amdgcn_sched_group_barrier(0x100, 1, 0); } while (0)
#define AB_INTERLEAVE_6() do { AB_MFMA_DS_PAIR(); AB_MFMA_DS_PAIR(); AB_MFMA_DS_PAIR(); AB_MFMA_DS_PAIR(); \
                               AB_MFMA_DS_PAIR(); AB_MFMA_DS_PAIR(); \
                               __builtin_amdgcn_sched_group_barrier(0x008, 2, 0); } while (0)

    // ---- prologue.  Issue order fixes what a vmcnt(n) wait leaves outstanding (loads retire in order).
    if constexpr (AMODE == AMODE_LOAD) {
        dma_a(0); dma_w(0);
        if (KT > 1) { dma_a(1); dma_w(1); }
        if (KT > 2) dma_a(2);
        if (KT > 2)      asm volatile("s_waitcnt vmcnt(12)" ::: "memory");
        else if (KT > 1) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        else             asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    } else {
        issue_raw(0);
        write_generated(0);                                // (the compiler waits for the raw loads it uses)
        dma_w(0);
        if (KT > 1) { dma_w(1); issue_raw(1); }
        if (KT > 1) asm volatile("s_waitcnt vmcnt(10)" ::: "memory");   // W(1): 4 DMA, raw(1): 6 loads
        else        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    AB_FENCE();
    load_frags(0, 0, 0);

    for (int kt = 0; kt < KT; ++kt) {
        AB_FENCE();
        load_frags(kt, 1, 1);
        mma(0);
        AB_INTERLEAVE_6();
        AB_FENCE();
        load_frags(kt, 2, 0);
        mma(1);
        AB_INTERLEAVE_6();
        AB_FENCE();
        load_frags(kt, 3, 1);
        mma(0);
        AB_INTERLEAVE_6();
        AB_FENCE();
        if constexpr (AMODE == AMODE_GEN) {
            if (kt + 1 < KT) write_generated(kt + 1);      // raw(kt+1) was requested one slab ago
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        } else {
            // slab kt+1 (both operands) must have landed; A(kt+2), issued last, may still be in flight
            if (kt + 2 < KT) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
            else             asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
        // own fragment reads of this slab returned; then meet: slab kt+1 is complete and visible to
        // everybody and slab kt's stages may be refilled
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        AB_FENCE();
        if (kt + 2 < KT) dma_w(kt + 2);
        if constexpr (AMODE == AMODE_LOAD) { if (kt + 3 < KT) dma_a(kt + 3); }
        else                               { if (kt + 2 < KT) issue_raw(kt + 2); }
        AB_FENCE();
        load_frags(kt + 1, 0, 0);                          // (after the last slab: a stale stage, unused)
        mma(1);
        AB_INTERLEAVE_6();
        AB_FENCE();
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __syncthreads();                           // everybody is done with the operand stages

    // ---------------------------------------------------------------- epilogues
    const int ncol0 = wave_n * 64 + half * 4;              // + jn*32 + rg*8 + e   (column within the tile)
    const int mrow0 = wave_m * 128 + l31;                  // + im*32              (row within the tile)
    if constexpr (EPI == EPI_STORE) {
#pragma unroll
        for (int jn = 0; jn < 2; ++jn)
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                const int nc = ncol0 + jn * 32 + rg * 8;
                f32x4 bv = {0.f, 0.f, 0.f, 0.f};
                if (g.bias) bv = *(const f32x4 *)(g.bias + n0 + nc);
#pragma unroll
                for (int im = 0; im < 4; ++im) {
                    float v0 = acc[jn][im][rg * 4 + 0] + bv.x, v1 = acc[jn][im][rg * 4 + 1] + bv.y;
                    float v2 = acc[jn][im][rg * 4 + 2] + bv.z, v3 = acc[jn][im][rg * 4 + 3] + bv.w;
                    if (g.relu) {
                        v0 = relu_keep_nan(v0); v1 = relu_keep_nan(v1);
                        v2 = relu_keep_nan(v2); v3 = relu_keep_nan(v3);
                    }
                    uint2 pk = {pack_bf16x2(v0, v1), pack_bf16x2(v2, v3)};
                    *(uint2 *)(smem + (mrow0 + im * 32) * OUT_STRIDE + nc * 2) = pk;
                }
            }
        __syncthreads();
        // thread -> 16-byte chunk (t & 31) of rows (t >> 5) + 16 it: all LDS reads first, then the stores
        {
            const unsigned char *src = smem + (t >> 5) * OUT_STRIDE + (t & 31) * 16;
            uint16_t *dst = (uint16_t *)g.out + (m0 + (t >> 5)) * g.ldo + n0 + (t & 31) * 8;
            const int64_t step = 16 * g.ldo;
            i32x4 v[16];
#pragma unroll
            for (int it = 0; it < 16; ++it) v[it] = *(const i32x4 *)(src + it * 16 * OUT_STRIDE);
            if (m0 + BM <= g.M) {
#pragma unroll
                for (int it = 0; it < 16; ++it) __builtin_nontemporal_store(v[it], (i32x4 *)(dst + it * step));
            } else {
#pragma unroll
                for (int it = 0; it < 16; ++it)
                    if (m0 + (t >> 5) + 16 * it < g.M) __builtin_nontemporal_store(v[it], (i32x4 *)(dst + it * step));
            }
        }
    } else {   // EPI_SCORE
        float ps[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int jn = 0; jn < 2; ++jn)
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                const int nc = n0 + ncol0 + jn * 32 + rg * 8;
                const f32x4 bv = *(const f32x4 *)(g.bias + nc);
                const f32x4 wv = *(const f32x4 *)(g.w_out + nc);
#pragma unroll
                for (int im = 0; im < 4; ++im) {
                    ps[im] += relu_keep_nan(acc[jn][im][rg * 4 + 0] + bv.x) * wv.x;
                    ps[im] += relu_keep_nan(acc[jn][im][rg * 4 + 1] + bv.y) * wv.y;
                    ps[im] += relu_keep_nan(acc[jn][im][rg * 4 + 2] + bv.z) * wv.z;
                    ps[im] += relu_keep_nan(acc[jn][im][rg * 4 + 3] + bv.w) * wv.w;
                }
            }
        float *red = (float *)smem;            // [4 column-waves][256 rows]
#pragma unroll
        for (int im = 0; im < 4; ++im) {
            const float v = ps[im] + __shfl_xor(ps[im], 32, 64);
            if (half == 0) red[wave_n * BM + mrow0 + im * 32] = v;
        }
        __syncthreads();
        if (t < BM && m0 + t < g.M)
            g.partial[(m0 + t) * g.n_tiles + tn] = (red[t] + red[BM + t]) + (red[2 * BM + t] + red[3 * BM + t]);
    }
}

template <int AMODE, int EPI>
static hipError_t launch_big_one(const GemmArgs &g, hipStream_t st)
{
    constexpr int smem = 5 * 256 * 128;   // 163840: three A slabs + two W slabs; the staged output tile (135168) reuses them
    auto kern = gemm_big_kernel<AMODE, EPI>;
    hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    const int64_t blocks = (g.m_tiles + 7) / 8 * 8 * g.n_tiles;
    if (blocks <= 0) return hipSuccess;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    kern<<<(unsigned)blocks, 512, smem, st>>>(g);
    return hipGetLastError();
}

bool gemm_big_supported(int dtype, int amode, int epi, const GemmArgs &g)
{
    if (dtype != AB_BF16 || (epi != EPI_STORE && epi != EPI_SCORE)) return false;
    if (g.N <= 0 || g.N % 256 != 0 || g.K <= 0 || g.K % 64 != 0 || g.M <= 0) return false;
    if (epi == EPI_STORE && (g.out_f32 || g.out_t || g.ldo % 8 != 0)) return false;
    if (amode == AMODE_GEN) {
        if (g.C % 256 != 0 || g.M % g.C != 0 || g.ldt % 4 != 0 || !g.wp || !g.wc || !g.xp || !g.xc) return false;
    } else if (g.lda % 8 != 0) {
        return false;
    }
    return g.ldb % 8 == 0;
}

hipError_t launch_gemm_big(int amode, int epi, GemmArgs g, hipStream_t st)
{
    g.m_tiles = (g.M + 255) / 256;
    g.n_tiles = g.N / 256;
    if (amode == AMODE_LOAD)
        return epi == EPI_STORE ? launch_big_one<AMODE_LOAD, EPI_STORE>(g, st)
                                : launch_big_one<AMODE_LOAD, EPI_SCORE>(g, st);
    return epi == EPI_STORE ? launch_big_one<AMODE_GEN, EPI_STORE>(g, st)
                            : launch_big_one<AMODE_GEN, EPI_SCORE>(g, st);
}

}  // namespace ab
