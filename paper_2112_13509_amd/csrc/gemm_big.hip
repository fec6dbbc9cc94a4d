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
#include <type_traits>

namespace ab {

typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void global_void;
typedef float f32x8_unaligned __attribute__((ext_vector_type(8), aligned(4)));

typedef __attribute__((address_space(4))) f32x8_unaligned const_f32x8;   // read-only for the whole launch: scalar loads
// Eight consecutive floats at a wave-uniform address, fetched through the scalar cache into scalar registers.
__device__ __forceinline__ f32x8_unaligned scalar_load8(const float *p)
{
    f32x8_unaligned v = *(const const_f32x8 *)(uintptr_t)p;
    asm volatile("" : "+s"(v));
    return v;
}

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
            gen_xp[i] = g.xp[(g.x_per_row ? m0 : (int64_t)c0) + r];
            gen_xc[i] = g.xc[(g.x_per_row ? m0 : (int64_t)c0) + r];
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


// ------------------------------------------------------------------------------------------------
// Streaming form of the same tile for operands that are read from memory: a grid of one work-group
// per compute unit, each walking its tiles in the order the one-tile-per-work-group launch would have
// handed them out (id = block + q * grid; id & 7 = XCD).  The slab rings run on across tile borders, so
// the first three slabs of the next tile are already under way while the current tile finishes, and
// the stores of a tile drain under the next tile's matrix work:
//   - at the last slab of a tile the W stage is refilled as usual, the A stage that was just retired
//     serves as staging room for the output (4 KB private to each wavefront: 32 rows x 64 columns per
//     pass, four passes, no work-group barrier in between) and is refilled after the epilogue;
//   - every slab fetch is issued unconditionally (past the end of the stream the last tile is
//     fetched again into stages nobody reads), so the number of memory operations between any two
//     points is fixed and every wait can name exactly how many younger operations may stay in
//     flight: 4 (the A slab two ahead) in a tile, plus the stores of the epilogue and the next tile's
//     bias fetch at the first slab after it.  Loads and stores retire in issue order.
//   - bias (and output weights) are read through the scalar cache in the epilogue, so no ordinary
//     vector load has to be waited for while slab fetches are in flight.
//
// LDS stores the compiler does not see as such: it orders every LDS store it knows of behind all
// global->LDS DMA in flight (a full vmcnt drain), which the staging writes of the epilogue must not do;
// the stage they go to has been retired by the barrier before.  LDS operations of a wavefront execute
// in order, so the reads that follow see the data.
__device__ __forceinline__ void lds_write8(void *p, uint2 v)
{
    asm volatile("ds_write_b64 %0, %1" ::"v"((uint32_t)(uintptr_t)(lds_void *)p), "v"(v) : "memory");
}
__device__ __forceinline__ void lds_write4(void *p, float v)
{
    asm volatile("ds_write_b32 %0, %1" ::"v"((uint32_t)(uintptr_t)(lds_void *)p), "v"(v) : "memory");
}

template <int EPI, bool COL_REGS>
__global__ __launch_bounds__(512) void gemm_stream_kernel(const GemmArgs g)
{
    // (the storing epilogue's staging areas fill the idle stage; with it the scalar loads hide under the draining stores anyway)
    static_assert(!(COL_REGS && EPI == EPI_STORE), "COL_REGS goes with the fused output unit only");
    constexpr int BM = 256, BK = 64;
    constexpr int SLAB = BM * 128;
    constexpr int W_BASE = 3 * SLAB;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);           // (scalar: addresses and branches on it stay scalar)
    const int wave_m = wave >> 2, wave_n = wave & 3;
    const int half = lane >> 5, l31 = lane & 31;
    const int KT = g.K / BK;
    // Values that are only needed once per tile are derived from an opaque copy of the lane id at the
    // place of use, so that they do not occupy registers during the matrix loop.
    auto opaque_lane = [&]() { int v = lane; asm volatile("" : "+v"(v)); return v; };

    // ---- this work-group's tiles: local index l0 + q * G8 on XCD xcd, q < n_my
    const unsigned G8 = gridDim.x >> 3, xcd = blockIdx.x & 7, l0 = blockIdx.x >> 3;
    const unsigned n_tiles = (unsigned)g.n_tiles;
    const unsigned panels = (unsigned)g.m_tiles > xcd ? ((unsigned)g.m_tiles - xcd + 7) / 8 : 0;
    const unsigned n_local = panels * n_tiles;
    if (l0 >= n_local) return;
    const unsigned n_my = (n_local - l0 + G8 - 1) / G8;

    // ---- DMA sources: a wave-uniform byte pointer per operand (advanced per slab on the scalar unit) plus
    // four 32-bit per-lane byte offsets (row dma_r0 + 64 i, chunk dma_cc)
    // lane l of wavefront w fetches logical chunk (l & 7) ^ ((w & 1) * 4 + (l >> 4)) of row w * 8 + (l >> 3) + 64 i
    const unsigned char *a_base, *w_base;
    uint32_t a_off[4], w_off[4];
    auto set_w = [&](unsigned q) {
        const unsigned local = l0 + q * G8;
        w_base = (const unsigned char *)g.B + (int64_t)(local % n_tiles) * 256 * g.ldb * 2;
        const int ln = opaque_lane();
        const int dma_cc = (ln & 7) ^ ((wave & 1) * 4 + (ln >> 4)), dma_r0 = wave * 8 + (ln >> 3);
#pragma unroll
        for (int i = 0; i < 4; ++i) w_off[i] = (uint32_t)(dma_r0 + 64 * i) * (uint32_t)g.ldb * 2u + dma_cc * 16;
    };
    auto set_a = [&](unsigned q) {
        const unsigned local = l0 + q * G8;
        const int64_t m0 = ((int64_t)(local / n_tiles) * 8 + xcd) * BM;
        a_base = (const unsigned char *)g.A + m0 * g.lda * 2;
        const int64_t rows_left = g.M - m0;                 // >= 1; rows past the end re-read the last row
        const int ln = opaque_lane();
        const int dma_cc = (ln & 7) ^ ((wave & 1) * 4 + (ln >> 4)), dma_r0 = wave * 8 + (ln >> 3);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int r = dma_r0 + 64 * i;
            if (r > rows_left - 1) r = (int)(rows_left - 1);
            a_off[i] = (uint32_t)r * (uint32_t)g.lda * 2u + dma_cc * 16;
        }
    };
    unsigned wq = 0, aq = 0;
    int wkt = 0, akt = 0;
    // A slab is fetched as two halves (row groups i0, i0 + 1 of four) so that the requests can be spread
    // over the quarters of a slab's matrix work instead of queueing up behind the barrier.
    auto dma_w_rows = [&](int slot, int i0) {
        unsigned char *sb = smem + W_BASE + slot * SLAB;
        dma16<false>(w_base + w_off[i0], sb + (wave + 8 * i0) * 1024);
        dma16<false>(w_base + w_off[i0 + 1], sb + (wave + 8 * (i0 + 1)) * 1024);
    };
    auto dma_a_rows = [&](int slot, int i0) {
        unsigned char *sb = smem + slot * SLAB;
        dma16<true>(a_base + a_off[i0], sb + (wave + 8 * i0) * 1024);
        dma16<true>(a_base + a_off[i0 + 1], sb + (wave + 8 * (i0 + 1)) * 1024);
    };
    auto advance_w = [&]() {
        w_base += BK * 2;
        if (++wkt == KT) { wkt = 0; if (wq + 1 < n_my) ++wq; set_w(wq); }
    };
    auto advance_a = [&]() {
        a_base += BK * 2;
        if (++akt == KT) { akt = 0; if (aq + 1 < n_my) ++aq; set_a(aq); }
    };

    // ---- fragment read offsets
    const int sw = (l31 >> 1) & 7;
    int rd[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) rd[q] = l31 * 128 + ((((q << 1) | half) ^ sw) << 4);
    const int a_rd = wave_m * 128 * 128;
    const int w_rd = W_BASE + wave_n * 64 * 128;

    f32x16 acc[2][4];
    f32x16 cinit[2];                                       // the tile's bias in accumulator layout (same for all four row blocks)
    i32x4 fa[2][4], fw[2][2];
    auto load_frags = [&](int a_slot, int w_slot, int q, int set) {
        const unsigned char *sa = smem + a_slot * SLAB + a_rd;
        const unsigned char *sw_ = smem + w_slot * SLAB + w_rd;
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
    auto mma_first = [&](int set) {                        // a tile's first quarter: the accumulators start at the bias
#pragma unroll
        for (int jn = 0; jn < 2; ++jn)
#pragma unroll
            for (int im = 0; im < 4; ++im)
                acc[jn][im] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    __builtin_bit_cast(bf16x8, fw[set][jn]), __builtin_bit_cast(bf16x8, fa[set][im]),
                    cinit[jn], 0, 0, 0);
    };

    // per-tile state of the computing side
    int64_t m0 = 0;
    int n0 = 0;
    unsigned tn = 0;
    // COL_REGS (at most four column tiles): a lane keeps, per column tile, the bias (and the output weight) of
    // column `lane` of this wavefront's 64, read once before any slab fetch is in flight.  A tile's values in
    // accumulator layout are then one 4-byte LDS write and eight 16-byte reads through 256 bytes private to the
    // wavefront, in an A stage that is idle at that moment (LDS serves a wavefront's requests in order), instead
    // of eight scalar loads in a row (about 2 k cycles per tile).  Otherwise they come through the scalar cache:
    // no vector-memory traffic either way.
    float bias_v[4] = {0.f, 0.f, 0.f, 0.f}, wout_v[4] = {0.f, 0.f, 0.f, 0.f};
    if constexpr (COL_REGS) {
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
            if ((unsigned)tt < n_tiles) {
                bias_v[tt] = g.bias[tt * 256 + wave_n * 64 + lane];
                if constexpr (EPI == EPI_SCORE) wout_v[tt] = g.w_out[tt * 256 + wave_n * 64 + lane];
            }
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) { asm volatile("" : "+v"(bias_v[tt])); asm volatile("" : "+v"(wout_v[tt])); }
    }
    // bias (and output weights) of this wavefront's 64 columns arrive through the scalar cache: no
    // vector-memory traffic, so nothing has to wait for the slab fetches in flight.  The bias is the
    // accumulators' starting value, in their layout: register rg*4+e of column block jn is column
    // jn*32 + rg*8 + (lane>>5)*4 + e.
    auto begin_tile = [&](unsigned q, int idle_stage) {
        const unsigned local = l0 + q * G8;
        tn = local % n_tiles;
        n0 = (int)tn * 256;
        m0 = ((int64_t)(local / n_tiles) * 8 + xcd) * BM;
        const int ln = opaque_lane();
        const int hf = ln >> 5;
        const unsigned char *scr = smem + idle_stage * SLAB + 4096 + wave * 256;     // behind the row sums' exchange area
        if constexpr (COL_REGS) {
            const float bsel = tn == 0 ? bias_v[0] : tn == 1 ? bias_v[1] : tn == 2 ? bias_v[2] : bias_v[3];
            lds_write4((void *)(scr + ln * 4), bsel);
        }
#pragma unroll
        for (int jn = 0; jn < 2; ++jn)
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                if constexpr (COL_REGS) {
                    const f32x4 b4 = *(const f32x4 *)(scr + (jn * 32 + rg * 8 + hf * 4) * 4);
#pragma unroll
                    for (int e = 0; e < 4; ++e) cinit[jn][rg * 4 + e] = b4[e];
                } else {
                    const f32x8_unaligned b8 = scalar_load8(g.bias + n0 + wave_n * 64 + jn * 32 + rg * 8);
#pragma unroll
                    for (int e = 0; e < 4; ++e) cinit[jn][rg * 4 + e] = hf ? b8[4 + e] : b8[e];
                }
            }
    };

    // Scheduling inside a quarter that also issues slab fetches: 8 matrix instructions, 6 fragment reads and
    // 2 (or 4) DMA requests, spread evenly.
#define AB_MFMA_VMEM_PAIR() do { __builtin_amdgcn_sched_group_barrier(0x008, 1, 0); \
                                 __builtin_amdgcn_sched_group_barrier(0x010, 1, 0); } while (0)
#define AB_INTERLEAVE_6_V2() do { AB_MFMA_DS_PAIR(); AB_MFMA_DS_PAIR(); AB_MFMA_VMEM_PAIR(); AB_MFMA_DS_PAIR(); \
                                  AB_MFMA_DS_PAIR(); AB_MFMA_VMEM_PAIR(); AB_MFMA_DS_PAIR(); AB_MFMA_DS_PAIR(); } while (0)
#define AB_INTERLEAVE_6_V4() do { __builtin_amdgcn_sched_group_barrier(0x100, 2, 0); \
                                  AB_MFMA_VMEM_PAIR(); AB_MFMA_DS_PAIR(); AB_MFMA_VMEM_PAIR(); AB_MFMA_DS_PAIR(); \
                                  AB_MFMA_VMEM_PAIR(); AB_MFMA_DS_PAIR(); AB_MFMA_VMEM_PAIR(); AB_MFMA_DS_PAIR(); } while (0)

    // Order of the memory operations of a wavefront (loads and stores retire in order).  The quarters are
    // straight-line code on purpose: a branch around matrix instructions makes the compiler copy accumulators.
    //   quarter 3 of slab j-1 (after its barrier): W(j+1), into the stage just retired (at a tile's last slab
    //                                              the epilogue's stores follow)
    //   quarter 0 of slab j:                       A(j+2), into the stage retired one slab ago (as early as the
    //                                              epilogue's use of that stage allows: measured best)
    //   wait before the barrier of slab j:         slab j+1 must be complete -> only A(j+2) (4 operations) and,
    //                                              at a tile's first slab, the previous tile's stores in front
    //                                              of it may still be in flight.
    // A stricter wait than needed is always safe.
    constexpr int EPI_OPS_LOW = EPI == EPI_STORE ? 16 : 1;              // wavefronts 0..3
    constexpr int EPI_OPS_HIGH = EPI == EPI_STORE ? 16 : 0;             // wavefronts 4..7 (no partial store)
    static_assert(EPI_OPS_LOW + 4 == (EPI == EPI_STORE ? 20 : 5) && EPI_OPS_HIGH + 4 == (EPI == EPI_STORE ? 20 : 4), "");

    // ---- prologue: slabs 0 and 1 whole
    set_w(0); set_a(0);
    dma_a_rows(0, 0); dma_a_rows(0, 2); advance_a();
    dma_w_rows(0, 0); dma_w_rows(0, 2); advance_w();
    dma_a_rows(1, 0); dma_a_rows(1, 2); advance_a();
    dma_w_rows(1, 0); dma_w_rows(1, 2); advance_w();
    begin_tile(0, 2);                                      // (stage 2 is first written in the first slab)
    asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    AB_FENCE();
    load_frags(0, 0, 0, 0);

    int a_slot = 0, w_slot = 0;
    unsigned q = 0;
    // One slab.  A tile's first slab is its own copy of the code (its first matrix instructions take the bias
    // as their addend, its wait knows of the stores in front), so that no branch sits inside a quarter.
    // Wave priority by progress: among equal priorities a SIMD serves its older wavefront first, so of the two
    // wavefronts of a SIMD the older one would run through its three quarters at full rate, wait at the barrier for
    // about 900 cycles of a 2400-cycle slab (measured with clock stamps around the barrier) while the younger one
    // runs alone, and each would expose its own fragment-read latencies.  With the priority falling from quarter
    // to quarter the wavefront that is behind wins, the two stay within one quarter of each other (the wait falls
    // to about 400 cycles) and fill each other's gaps.
    auto slab = [&](auto first_tag) {
        constexpr bool FIRST = decltype(first_tag)::value;
        const int pa = a_slot == 0 ? 2 : a_slot - 1;       // the A stage retired one slab ago
        AB_FENCE();
        __builtin_amdgcn_s_setprio(2);
        load_frags(a_slot, w_slot, 1, 1);
        dma_a_rows(pa, 0);
        dma_a_rows(pa, 2);
        if constexpr (FIRST) mma_first(0); else mma(0);
        AB_INTERLEAVE_6_V4();
        AB_FENCE();
        advance_a();
        AB_FENCE();
        __builtin_amdgcn_s_setprio(1);
        load_frags(a_slot, w_slot, 2, 0);
        mma(1);
        AB_INTERLEAVE_6();
        AB_FENCE();
        __builtin_amdgcn_s_setprio(0);
        load_frags(a_slot, w_slot, 3, 1);
        mma(0);
        AB_INTERLEAVE_6();
        AB_FENCE();
        if (!FIRST || q == 0) {
            asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        } else if (wave < 4) {
            if constexpr (EPI == EPI_STORE) asm volatile("s_waitcnt vmcnt(20)" ::: "memory");
            else                            asm volatile("s_waitcnt vmcnt(5)" ::: "memory");
        } else {
            if constexpr (EPI == EPI_STORE) asm volatile("s_waitcnt vmcnt(20)" ::: "memory");
            else                            asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        }
        // own fragment reads of this slab returned; then meet: slab j+1 is complete and visible to
        // everybody and slab j's stages may be refilled
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        AB_FENCE();
        __builtin_amdgcn_s_setprio(3);
        const int na = a_slot == 2 ? 0 : a_slot + 1, nw = w_slot ^ 1;
        load_frags(na, nw, 0, 0);
        dma_w_rows(w_slot, 0);
        dma_w_rows(w_slot, 2);
        mma(1);
        AB_INTERLEAVE_6_V4();
        AB_FENCE();
        advance_w();
        a_slot = na;
        w_slot = nw;
    };
    while (true) {
        slab(std::true_type{});
        for (int kt = 1; kt < KT; ++kt) slab(std::false_type{});
        {
            // ------------------------------------------------------------ epilogue of tile q
            // staging room: the A stage retired by the last barrier; A(j+3) goes there later
            unsigned char *stage = smem + (a_slot == 0 ? 2 : a_slot - 1) * SLAB;
            const bool ragged = m0 + BM > g.M;
            const int ln = opaque_lane();
            const int half = ln >> 5, l31 = ln & 31, sw = (l31 >> 1) & 7;
            if constexpr (EPI == EPI_STORE) {
                unsigned char *mine = stage + wave * 4096;
                const int rrow = ln >> 3, rch = ln & 7;
                uint16_t *dst = (uint16_t *)g.out + (m0 + wave_m * 128 + rrow) * g.ldo + n0 + wave_n * 64 + rch * 8;
                auto store_tile = [&](auto relu_tag) {
#pragma unroll
                    for (int im = 0; im < 4; ++im) {
#pragma unroll
                        for (int jn = 0; jn < 2; ++jn)
#pragma unroll
                            for (int rg = 0; rg < 4; ++rg) {
                                float v[4];
#pragma unroll
                                for (int e = 0; e < 4; ++e) {
                                    v[e] = acc[jn][im][rg * 4 + e];
                                    if constexpr (decltype(relu_tag)::value) v[e] = relu_keep_nan(v[e]);
                                }
                                uint2 pk = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
                                lds_write8(mine + l31 * 128 + (((jn * 4 + rg) ^ sw) << 4) + half * 8, pk);
                            }
                        i32x4 o[4];
#pragma unroll
                        for (int it = 0; it < 4; ++it) {
                            const int row = rrow + 8 * it;
                            o[it] = *(const i32x4 *)(mine + row * 128 + ((rch ^ ((row >> 1) & 7)) << 4));
                        }
                        uint16_t *d = dst + (int64_t)(im * 32) * g.ldo;
                        if (!ragged) {
#pragma unroll
                            for (int it = 0; it < 4; ++it)
                                __builtin_nontemporal_store(o[it], (i32x4 *)(d + (int64_t)(8 * it) * g.ldo));
                        } else {
#pragma unroll
                            for (int it = 0; it < 4; ++it)
                                if (m0 + wave_m * 128 + im * 32 + rrow + 8 * it < g.M)
                                    __builtin_nontemporal_store(o[it], (i32x4 *)(d + (int64_t)(8 * it) * g.ldo));
                        }
                    }
                };
                if (g.relu) store_tile(std::true_type{});
                else        store_tile(std::false_type{});
            } else {   // EPI_SCORE
                float ps[4] = {0.f, 0.f, 0.f, 0.f};
                const unsigned char *scr = stage + 4096 + wave * 256;      // behind the row sums' exchange area
                if constexpr (COL_REGS) {
                    const float wsel = tn == 0 ? wout_v[0] : tn == 1 ? wout_v[1] : tn == 2 ? wout_v[2] : wout_v[3];
                    lds_write4((void *)(scr + ln * 4), wsel);
                }
#pragma unroll
                for (int jn = 0; jn < 2; ++jn)
#pragma unroll
                    for (int rg = 0; rg < 4; ++rg) {
                        f32x8_unaligned w8;
                        f32x4 w4;
                        if constexpr (COL_REGS) w4 = *(const f32x4 *)(scr + (jn * 32 + rg * 8 + half * 4) * 4);
                        else w8 = scalar_load8(g.w_out + n0 + wave_n * 64 + jn * 32 + rg * 8);
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            float wv;
                            if constexpr (COL_REGS) wv = w4[e];
                            else wv = half ? w8[4 + e] : w8[e];
#pragma unroll
                            for (int im = 0; im < 4; ++im)
                                ps[im] += relu_keep_nan(acc[jn][im][rg * 4 + e]) * wv;
                        }
                    }
                float *red = (float *)stage;               // [4 column-waves][256 rows]
#pragma unroll
                for (int im = 0; im < 4; ++im) {
                    const float v = ps[im] + __shfl_xor(ps[im], 32, 64);
                    if (half == 0) lds_write4(red + wave_n * BM + wave_m * 128 + l31 + im * 32, v);
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();
                if (wave < 4) {
                    const int tt = wave * 64 + ln;
                    const float v = (red[tt] + red[BM + tt]) + (red[2 * BM + tt] + red[3 * BM + tt]);
                    if (!ragged) g.partial[(m0 + tt) * g.n_tiles + tn] = v;
                    else if (m0 + tt < g.M) g.partial[(m0 + tt) * g.n_tiles + tn] = v;
                }
            }
            // a ragged tile may have issued fewer stores than the counts assume: drain instead
            if (ragged) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            if (q + 1 == n_my) break;
            ++q;
            // the next tile's coordinates and bias: through the staging room, which this wavefront is done with,
            // or by scalar loads, which are better left to return under the draining stores behind the barrier
            if constexpr (COL_REGS) begin_tile(q, a_slot == 0 ? 2 : a_slot - 1);
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();                  // everybody has read the staging room back
            AB_FENCE();
            if constexpr (!COL_REGS) begin_tile(q, 0);
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");       // no DMA may still target LDS when the group ends
}


// ------------------------------------------------------------------------------------------------
// Streaming kernel for the first hidden layer: the activation operand is not read but generated,
// A[r, k] = relu(a_term[s, k] + wp[k] * xp[c] + wc[k] * xc[c]) for row r = (scenario s, candidate c), one
// scenario per 256-row tile.  Same walk over the tiles and same W ring as gemm_stream_kernel; differences:
//   - the A ring has two stages; while slab j is multiplied, slab j+1 is generated into the other
//     stage by the vector ALUs (a thread owns one 8-wide k chunk of four adjacent rows: two row chunks
//     in the first quarter, one in each of the next two), next to the matrix instructions;
//   - everything the generation reads comes from LDS: wp and wc (whole, fetched once), the scenario's
//     a_term row and the tile's xp / xc slices (double-buffered per tile, fetched one tile ahead by
//     DMA, 3 requests per wavefront), 20 KB behind the rings.  No ordinary vector load is in flight
//     next to the DMA, so no wait ever has to drain the queue.
//   - memory operations of a wavefront: W(j+2) x4 in the last quarter of slab j; at a tile border
//     the stores x16 and the vector fetch x3 follow.  Inside a tile the wait before a slab's barrier
//     is therefore for everything, at a tile's first slab 19 operations may stay in flight.
// Needs K <= 1024 (vector area) and at least two slabs.
__device__ __forceinline__ void lds_write16(void *p, i32x4 v)
{
    asm volatile("ds_write_b128 %0, %1" ::"v"((uint32_t)(uintptr_t)(lds_void *)p), "v"(v) : "memory");
}
__device__ __forceinline__ void dma4(const void *gsrc, void *lds_uniform_dst)   // 64 lanes x 4 bytes
{
    __builtin_amdgcn_global_load_lds((global_void *)gsrc, (lds_void *)lds_uniform_dst, 4, 0, 0);
}

template <int EPI, bool COL_REGS, bool SHARE>
__global__ __launch_bounds__(512) void gemm_stream_gen_kernel(const GemmArgs g)
{
    constexpr int BM = 256, BK = 64;
    constexpr int SLAB = BM * 128;
    constexpr int W_BASE = 2 * SLAB;
    constexpr int V_WP = 4 * SLAB, V_WC = V_WP + 4096, V_AT = V_WC + 4096, V_XP = V_AT + 8192;   // + 4096: 151552
    constexpr int V_BIAS = V_XP + 4096, V_WOUT = V_BIAS + 4096;   // COL_REGS: fp32 [4][256] each, + 4096: 159744
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wave_m = wave >> 2, wave_n = wave & 3;
    const int half = lane >> 5, l31 = lane & 31;
    const int KT = g.K / BK;
    auto opaque_lane = [&]() { int v = lane; asm volatile("" : "+v"(v)); return v; };

    const unsigned G8 = gridDim.x >> 3, xcd = blockIdx.x & 7, l0 = blockIdx.x >> 3;
    const unsigned n_tiles = (unsigned)g.n_tiles;
    const unsigned panels = (unsigned)g.m_tiles > xcd ? ((unsigned)g.m_tiles - xcd + 7) / 8 : 0;
    const unsigned n_local = panels * n_tiles;
    if (l0 >= n_local) return;
    const unsigned n_my = (n_local - l0 + G8 - 1) / G8;

    // ---- W slabs by DMA
    const unsigned char *w_base;
    uint32_t w_off[4];
    auto set_w = [&](unsigned q) {
        const unsigned local = l0 + q * G8;
        w_base = (const unsigned char *)g.B + (int64_t)(local % n_tiles) * 256 * g.ldb * 2;
        const int ln = opaque_lane();
        const int dma_cc = (ln & 7) ^ ((wave & 1) * 4 + (ln >> 4)), dma_r0 = wave * 8 + (ln >> 3);
#pragma unroll
        for (int i = 0; i < 4; ++i) w_off[i] = (uint32_t)(dma_r0 + 64 * i) * (uint32_t)g.ldb * 2u + dma_cc * 16;
    };
    unsigned wq = 0;
    int wkt = 0;
    auto dma_w_rows = [&](int slot, int i0) {
        unsigned char *sb = smem + W_BASE + slot * SLAB;
        dma16<false>(w_base + w_off[i0], sb + (wave + 8 * i0) * 1024);
        dma16<false>(w_base + w_off[i0 + 1], sb + (wave + 8 * (i0 + 1)) * 1024);
    };
    auto advance_w = [&]() {
        w_base += BK * 2;
        if (++wkt == KT) { wkt = 0; if (wq + 1 < n_my) ++wq; set_w(wq); }
    };

    // ---- what the generation reads, by DMA: 3 requests per wavefront and tile (past the end the last tile again)
    auto fetch_vec = [&](unsigned qq) {
        const int b = (int)(qq & 1);
        if (qq > n_my - 1) qq = n_my - 1;
        const unsigned local = l0 + qq * G8;
        const unsigned m0u = ((local / n_tiles) * 8 + xcd) * BM;
        const unsigned s = m0u / (unsigned)g.C, c0 = m0u - s * (unsigned)g.C;
        const int ln = opaque_lane();
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            int i = wave + 8 * h;
            if (i > KT - 1) i = KT - 1;
            dma4(g.a_term + (int64_t)s * g.ldt + i * 64 + ln, smem + V_AT + b * 4096 + i * 256);
        }
        dma4((wave < 4 ? g.xp : g.xc) + (g.x_per_row ? m0u : c0) + (wave & 3) * 64 + ln,
             smem + V_XP + b * 2048 + (wave >> 2) * 1024 + (wave & 3) * 256);
    };
    auto fetch_wp_wc = [&]() {                              // 4 requests per wavefront, once
        const int ln = opaque_lane();
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            int i = wave + 8 * h;
            if (i > KT - 1) i = KT - 1;
            dma4(g.wp + i * 64 + ln, smem + V_WP + i * 256);
            dma4(g.wc + i * 64 + ln, smem + V_WC + i * 256);
        }
    };

    // ---- generation: thread -> k chunk t & 7 of the four adjacent rows 4 (t >> 3) + i.  With SHARE (the rows of
    // such a group take the same xp, GemmArgs::xp_runs4) the inner term wp * xp + a_term is formed once for the
    // four rows: 5 instead of 8 fused multiply-adds per row chunk, the same values bit for bit.
    const int gcc = t & 7, grow4 = (t >> 3) * 4;
    int gen_st[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) gen_st[i] = (grow4 + i) * 128 + ((gcc ^ (((grow4 + i) >> 1) & 7)) << 4);
    f32x4 gxp, gxc;
    auto load_xpc = [&](int b) {
        gxp = *(const f32x4 *)(smem + V_XP + b * 2048 + grow4 * 4);
        gxc = *(const f32x4 *)(smem + V_XP + b * 2048 + 1024 + grow4 * 4);
    };
    f32x4 va[2], vp[2], vc[2];
    auto load_slices = [&](int b, int gk) {
        const int o = (gk * 64 + gcc * 8) * 4;
        va[0] = *(const f32x4 *)(smem + V_AT + b * 4096 + o);
        va[1] = *(const f32x4 *)(smem + V_AT + b * 4096 + o + 16);
        vp[0] = *(const f32x4 *)(smem + V_WP + o);
        vp[1] = *(const f32x4 *)(smem + V_WP + o + 16);
        vc[0] = *(const f32x4 *)(smem + V_WC + o);
        vc[1] = *(const f32x4 *)(smem + V_WC + o + 16);
    };
    auto gen_chunk = [&](int slot, int i) {
        const float xp = SHARE ? gxp[0] : gxp[i], xc = gxc[i];
        float h[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            h[e] = relu_keep_nan(fmaf(vc[0][e], xc, fmaf(vp[0][e], xp, va[0][e])));
            h[4 + e] = relu_keep_nan(fmaf(vc[1][e], xc, fmaf(vp[1][e], xp, va[1][e])));
        }
        i32x4 v;
        v.x = (int)pack_bf16x2(h[0], h[1]);
        v.y = (int)pack_bf16x2(h[2], h[3]);
        v.z = (int)pack_bf16x2(h[4], h[5]);
        v.w = (int)pack_bf16x2(h[6], h[7]);
        lds_write16(smem + slot * SLAB + gen_st[i], v);
    };

    // ---- fragment read offsets
    const int sw = (l31 >> 1) & 7;
    int rd[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) rd[q] = l31 * 128 + ((((q << 1) | half) ^ sw) << 4);
    const int a_rd = wave_m * 128 * 128;
    const int w_rd = W_BASE + wave_n * 64 * 128;

    f32x16 acc[2][4];
    f32x16 cinit[2];                                       // the tile's bias in accumulator layout
    i32x4 fa[2][4], fw[2][2];
    auto load_frags = [&](int a_slot, int w_slot, int q, int set) {
        const unsigned char *sa = smem + a_slot * SLAB + a_rd;
        const unsigned char *sw_ = smem + w_slot * SLAB + w_rd;
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

    auto mma_first = [&](int set) {                        // a tile's first quarter: the accumulators start at the bias
#pragma unroll
        for (int jn = 0; jn < 2; ++jn)
#pragma unroll
            for (int im = 0; im < 4; ++im)
                acc[jn][im] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    __builtin_bit_cast(bf16x8, fw[set][jn]), __builtin_bit_cast(bf16x8, fa[set][im]),
                    cinit[jn], 0, 0, 0);
    };

    int64_t m0 = 0;
    int n0 = 0;
    unsigned tn = 0;
    // COL_REGS (at most four column tiles): the bias and the output weights of all columns are put into LDS
    // once, before any slab fetch is in flight; a tile's values in accumulator layout (register rg*4+e of column
    // block jn is column jn*32 + rg*8 + (lane>>5)*4 + e of the wavefront's 64) are then eight 16-byte LDS reads,
    // the same addresses for all lanes of a half.  Otherwise they come through the scalar cache.
    if constexpr (COL_REGS) {
        const float *src = t < 256 ? g.bias : g.w_out;
        const bool mine = t < 256 || EPI == EPI_SCORE;
        float tv[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int tt = 0; tt < 4; ++tt)
            if (mine && (unsigned)tt < n_tiles) tv[tt] = src[tt * 256 + (t & 255)];
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
            asm volatile("" : "+v"(tv[tt]));
            if (mine) lds_write4(smem + (t < 256 ? V_BIAS : V_WOUT) + (tt * 256 + (t & 255)) * 4, tv[tt]);
        }
    }
    auto load_cinit = [&]() {
        const int hf = opaque_lane() >> 5;
#pragma unroll
        for (int jn = 0; jn < 2; ++jn)
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                if constexpr (COL_REGS) {
                    const f32x4 b4 = *(const f32x4 *)(smem + V_BIAS + ((int)tn * 256 + wave_n * 64 + jn * 32 + rg * 8 + hf * 4) * 4);
#pragma unroll
                    for (int e = 0; e < 4; ++e) cinit[jn][rg * 4 + e] = b4[e];
                } else {
                    const f32x8_unaligned b8 = scalar_load8(g.bias + n0 + wave_n * 64 + jn * 32 + rg * 8);
#pragma unroll
                    for (int e = 0; e < 4; ++e) cinit[jn][rg * 4 + e] = hf ? b8[4 + e] : b8[e];
                }
            }
    };
    auto begin_tile = [&](unsigned q) {
        const unsigned local = l0 + q * G8;
        tn = local % n_tiles;
        n0 = (int)tn * 256;
        m0 = ((int64_t)(local / n_tiles) * 8 + xcd) * BM;
    };

    // ---- prologue
    set_w(0);
    fetch_wp_wc();
    fetch_vec(0);
    fetch_vec(1);
    dma_w_rows(0, 0); dma_w_rows(0, 2); advance_w();
    dma_w_rows(1, 0); dma_w_rows(1, 2); advance_w();
    begin_tile(0);
    asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();                          // vectors, column tables and W(0) are in LDS for everybody
    AB_FENCE();
    load_cinit();
    load_xpc(0);
    load_slices(0, 0);
    gen_chunk(0, 0); gen_chunk(0, 1); gen_chunk(0, 2); gen_chunk(0, 3);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();                          // A(0) is complete
    AB_FENCE();
    load_frags(0, 0, 0, 0);

    int a_slot = 0, w_slot = 0, gpar = 0;
    unsigned q = 0;
    // One slab (kt = its place in the tile).  A tile's first slab is its own copy of the code, so that no
    // branch sits inside a quarter.
    // Wave priority: here the older wavefront of a SIMD does not expose latencies when it runs ahead (its vector
    // work fills them), so taking turns by progress as in the stored-operand kernel changes nothing; what the clock
    // stamps show is the younger wavefront held up in the first quarter, the one with two row chunks to generate
    // (990 cycles against 510).  It goes first there (3 against 0), after that the priority falls with progress.
    auto slab = [&](auto first_tag, int kt) {
        constexpr bool FIRST = decltype(first_tag)::value;
        const int nxt = a_slot ^ 1;                        // retired one slab ago: slab j+1 is generated there
        int gk = kt + 1;                                   // its place in its tile
        if (gk == KT) { gk = 0; gpar ^= 1; load_xpc(gpar); }
        load_slices(gpar, gk);
        AB_FENCE();
        if (wave_m) __builtin_amdgcn_s_setprio(3); else __builtin_amdgcn_s_setprio(0);
        load_frags(a_slot, w_slot, 1, 1);
        gen_chunk(nxt, 0);
        gen_chunk(nxt, 1);
        if constexpr (FIRST) mma_first(0); else mma(0);
        AB_INTERLEAVE_6();
        AB_FENCE();
        __builtin_amdgcn_s_setprio(1);
        load_frags(a_slot, w_slot, 2, 0);
        gen_chunk(nxt, 2);
        mma(1);
        AB_INTERLEAVE_6();
        AB_FENCE();
        __builtin_amdgcn_s_setprio(0);
        load_frags(a_slot, w_slot, 3, 1);
        gen_chunk(nxt, 3);
        mma(0);
        AB_INTERLEAVE_6();
        AB_FENCE();
        if (!FIRST || q == 0) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        } else if constexpr (EPI == EPI_STORE) {
            asm volatile("s_waitcnt vmcnt(19)" ::: "memory");          // 16 stores + 3 vector fetches
        } else {
            if (wave < 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");   // 1 store of partial sums + 3
            else          asm volatile("s_waitcnt vmcnt(3)" ::: "memory");
        }
        // own LDS traffic of this slab is done (fragment reads, generated chunks); then meet: slab j+1 is
        // complete and visible to everybody and slab j's stages may be refilled
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        AB_FENCE();
        __builtin_amdgcn_s_setprio(2);
        const int nw = w_slot ^ 1;
        load_frags(nxt, nw, 0, 0);
        dma_w_rows(w_slot, 0);
        dma_w_rows(w_slot, 2);
        mma(1);
        AB_INTERLEAVE_6_V4();
        AB_FENCE();
        advance_w();
        a_slot = nxt;
        w_slot = nw;
    };
    while (true) {
        slab(std::true_type{}, 0);
        for (int kt = 1; kt < KT; ++kt) slab(std::false_type{}, kt);
        {
            // ------------------------------------------------------------ epilogue of tile q (never ragged)
            unsigned char *stage = smem + (a_slot ^ 1) * SLAB;            // the A stage retired by the last barrier
            const int ln = opaque_lane();
            const int half = ln >> 5, l31 = ln & 31, sw = (l31 >> 1) & 7;
            if constexpr (EPI == EPI_STORE) {
                unsigned char *mine = stage + wave * 4096;
                const int rrow = ln >> 3, rch = ln & 7;
                uint16_t *dst = (uint16_t *)g.out + (m0 + wave_m * 128 + rrow) * g.ldo + n0 + wave_n * 64 + rch * 8;
                auto store_tile = [&](auto relu_tag) {
#pragma unroll
                    for (int im = 0; im < 4; ++im) {
#pragma unroll
                        for (int jn = 0; jn < 2; ++jn)
#pragma unroll
                            for (int rg = 0; rg < 4; ++rg) {
                                float v[4];
#pragma unroll
                                for (int e = 0; e < 4; ++e) {
                                    v[e] = acc[jn][im][rg * 4 + e];
                                    if constexpr (decltype(relu_tag)::value) v[e] = relu_keep_nan(v[e]);
                                }
                                uint2 pk = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
                                lds_write8(mine + l31 * 128 + (((jn * 4 + rg) ^ sw) << 4) + half * 8, pk);
                            }
                        i32x4 o[4];
#pragma unroll
                        for (int it = 0; it < 4; ++it) {
                            const int row = rrow + 8 * it;
                            o[it] = *(const i32x4 *)(mine + row * 128 + ((rch ^ ((row >> 1) & 7)) << 4));
                        }
                        uint16_t *d = dst + (int64_t)(im * 32) * g.ldo;
#pragma unroll
                        for (int it = 0; it < 4; ++it)
                            __builtin_nontemporal_store(o[it], (i32x4 *)(d + (int64_t)(8 * it) * g.ldo));
                    }
                };
                if (g.relu) store_tile(std::true_type{});
                else        store_tile(std::false_type{});
            } else {   // EPI_SCORE: the output unit as a per-lane dot product, reduced over the four column wavefronts
                float ps[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int jn = 0; jn < 2; ++jn)
#pragma unroll
                    for (int rg = 0; rg < 4; ++rg) {
                        f32x8_unaligned w8;
                        f32x4 w4;
                        if constexpr (COL_REGS) w4 = *(const f32x4 *)(smem + V_WOUT + ((int)tn * 256 + wave_n * 64 + jn * 32 + rg * 8 + half * 4) * 4);
                        else w8 = scalar_load8(g.w_out + n0 + wave_n * 64 + jn * 32 + rg * 8);
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            float wv;
                            if constexpr (COL_REGS) wv = w4[e];
                            else wv = half ? w8[4 + e] : w8[e];
#pragma unroll
                            for (int im = 0; im < 4; ++im)
                                ps[im] += relu_keep_nan(acc[jn][im][rg * 4 + e]) * wv;
                        }
                    }
                float *red = (float *)stage;               // [4 column-waves][256 rows]
#pragma unroll
                for (int im = 0; im < 4; ++im) {
                    const float v = ps[im] + __shfl_xor(ps[im], 32, 64);
                    if (half == 0) lds_write4(red + wave_n * BM + wave_m * 128 + l31 + im * 32, v);
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();
                if (wave < 4) {
                    const int tt = wave * 64 + ln;
                    const float v = (red[tt] + red[BM + tt]) + (red[2 * BM + tt] + red[3 * BM + tt]);
                    g.partial[(m0 + tt) * g.n_tiles + tn] = v;
                }
            }
            if (q + 1 == n_my) break;
            ++q;
            begin_tile(q);
            if constexpr (COL_REGS) load_cinit();          // (a fixed table: its reads may return under the wait below)
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();                  // everybody has read the staging room back
            AB_FENCE();
            if constexpr (!COL_REGS) load_cinit();
            fetch_vec(q + 1);
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");       // no DMA may still target LDS when the group ends
}

template <int EPI, bool COL_REGS, bool SHARE>
static hipError_t launch_stream_gen_impl(const GemmArgs &g, hipStream_t st);
template <int EPI>
static hipError_t launch_stream_gen(const GemmArgs &g, hipStream_t st)
{
    // at most four column tiles: bias and output weights sit in LDS tables (8 KB behind the vector area); otherwise
    // they come by scalar loads
    if (g.xp_runs4)
        return g.n_tiles <= 4 ? launch_stream_gen_impl<EPI, true, true>(g, st) : launch_stream_gen_impl<EPI, false, true>(g, st);
    return g.n_tiles <= 4 ? launch_stream_gen_impl<EPI, true, false>(g, st) : launch_stream_gen_impl<EPI, false, false>(g, st);
}
template <int EPI, bool COL_REGS, bool SHARE>
static hipError_t launch_stream_gen_impl(const GemmArgs &g, hipStream_t st)
{
    constexpr int smem = 4 * 256 * 128 + 20480 + (COL_REGS ? 8192 : 0);
    auto kern = gemm_stream_gen_kernel<EPI, COL_REGS, SHARE>;
    static DeviceOnce once;
    hipError_t e = ensure_dynamic_lds((const void *)kern, smem, once);
    if (e != hipSuccess) return e;
    int cus = 0;
    if ((e = compute_units(&cus)) != hipSuccess) return e;
    const int64_t ids = (g.m_tiles + 7) / 8 * 8 * g.n_tiles;
    if (ids <= 0) return hipSuccess;
    if (ids > 0x7fffffffLL) return hipErrorInvalidValue;
    int64_t grid = ids < cus ? ids : cus;
    grid = grid / 8 * 8;
    if (grid < 8) grid = 8;
    kern<<<(unsigned)grid, 512, smem, st>>>(g);
    return hipGetLastError();
}

template <int EPI, bool COL_REGS>
static hipError_t launch_stream_one_impl(const GemmArgs &g, hipStream_t st);
template <int EPI>
static hipError_t launch_stream_one(const GemmArgs &g, hipStream_t st)
{
    // at most four column tiles: bias and output weights live in registers and reach the accumulator layout through
    // a small LDS exchange; otherwise they come by scalar loads.  Measured at 16.8 M rows x 1024 x 1024: with the
    // fused output unit 1.58 -> 1.50 ms per launch (1.54 with lane reads in place of the exchange); with the
    // stored output nothing is gained (there the scalar loads already hide under the draining stores), so the
    // storing kernel keeps the scalar loads.
    if constexpr (EPI == EPI_SCORE) {
        if (g.n_tiles <= 4) return launch_stream_one_impl<EPI, true>(g, st);
    }
    return launch_stream_one_impl<EPI, false>(g, st);
}
template <int EPI, bool COL_REGS>
static hipError_t launch_stream_one_impl(const GemmArgs &g, hipStream_t st)
{
    constexpr int smem = 5 * 256 * 128;
    auto kern = gemm_stream_kernel<EPI, COL_REGS>;
    static DeviceOnce once;
    hipError_t e = ensure_dynamic_lds((const void *)kern, smem, once);
    if (e != hipSuccess) return e;
    int cus = 0;
    if ((e = compute_units(&cus)) != hipSuccess) return e;
    const int64_t ids = (g.m_tiles + 7) / 8 * 8 * g.n_tiles;
    if (ids <= 0) return hipSuccess;
    if (ids > 0x7fffffffLL) return hipErrorInvalidValue;
    int64_t grid = ids < cus ? ids : cus;
    grid = grid / 8 * 8;
    if (grid < 8) grid = 8;
    kern<<<(unsigned)grid, 512, smem, st>>>(g);
    return hipGetLastError();
}

template <int AMODE, int EPI>
static hipError_t launch_big_one(const GemmArgs &g, hipStream_t st)
{
    constexpr int smem = 5 * 256 * 128;   // 163840: three A slabs + two W slabs; the staged output tile (135168) reuses them
    auto kern = gemm_big_kernel<AMODE, EPI>;
    static DeviceOnce once;
    hipError_t e = ensure_dynamic_lds((const void *)kern, smem, once);
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
    } else if (g.lda % 8 != 0 || g.lda > (1 << 22)) {     // (row offsets inside a tile are kept in 32 bits)
        return false;
    }
    return g.ldb % 8 == 0 && g.ldb <= (1 << 22);
}

hipError_t launch_gemm_big(int amode, int epi, GemmArgs g, hipStream_t st)
{
    g.m_tiles = (g.M + 255) / 256;
    g.n_tiles = g.N / 256;
    if (amode == AMODE_LOAD) {
        if (g.bias)
            return epi == EPI_STORE ? launch_stream_one<EPI_STORE>(g, st) : launch_stream_one<EPI_SCORE>(g, st);
        return epi == EPI_STORE ? launch_big_one<AMODE_LOAD, EPI_STORE>(g, st)
                                : launch_big_one<AMODE_LOAD, EPI_SCORE>(g, st);
    }
    // generated operand: the streaming kernel needs the bias, the vector area bounds K, two slabs at least,
    // 32-bit row arithmetic and 4-byte DMA sources
    if (g.bias && g.K <= 1024 && g.K >= 128 && g.M < (1LL << 31))
        return epi == EPI_STORE ? launch_stream_gen<EPI_STORE>(g, st) : launch_stream_gen<EPI_SCORE>(g, st);
    return epi == EPI_STORE ? launch_big_one<AMODE_GEN, EPI_STORE>(g, st)
                            : launch_big_one<AMODE_GEN, EPI_SCORE>(g, st);
}

}  // namespace ab
