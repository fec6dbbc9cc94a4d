// Instantiations and host-side dispatch of the tiled matrix-core GEMM.
#include "internal.hpp"

namespace ab {

template <typename T, int WB, int AMODE, int EPI>
static hipError_t launch_one(const GemmArgs &g, hipStream_t st)
{
    constexpr int BM = 64 * WB, BN = 64 * WB;
    constexpr int smem = 2 * (BM + BN) * 128;
    auto kern = gemm_tn_kernel<T, WB, WB, AMODE, EPI>;
    if (smem > 48 * 1024) {
        static DeviceOnce once;
        hipError_t e = ensure_dynamic_lds((const void *)kern, smem, once);
        if (e != hipSuccess) return e;
    }
    const int64_t m_pad = (g.m_tiles + 7) / 8 * 8;
    int64_t blocks = m_pad * g.n_tiles;
    if (EPI == EPI_SPLITK) blocks *= g.k_splits;
    if (blocks <= 0) return hipSuccess;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    kern<<<(unsigned)blocks, 256, smem, st>>>(g);
    return hipGetLastError();
}

template <typename T, int WB>
static hipError_t launch_tile(int amode, int epi, const GemmArgs &g, hipStream_t st)
{
    if (amode == AMODE_LOAD) {
        switch (epi) {
        case EPI_STORE:  return launch_one<T, WB, AMODE_LOAD, EPI_STORE>(g, st);
        case EPI_SCORE:  return launch_one<T, WB, AMODE_LOAD, EPI_SCORE>(g, st);
        case EPI_DRELU:  if constexpr (WB <= 2) return launch_one<T, WB, AMODE_LOAD, EPI_DRELU>(g, st); break;
        case EPI_SPLITK: if constexpr (WB <= 2) return launch_one<T, WB, AMODE_LOAD, EPI_SPLITK>(g, st); break;
        }
    } else if (amode == AMODE_GEN) {
        switch (epi) {
        case EPI_STORE:  return launch_one<T, WB, AMODE_GEN, EPI_STORE>(g, st);
        case EPI_SCORE:  return launch_one<T, WB, AMODE_GEN, EPI_SCORE>(g, st);
        }
    } else {
        switch (epi) {
        case EPI_STORE:  return launch_one<T, WB, AMODE_GENV, EPI_STORE>(g, st);
        case EPI_SCORE:  return launch_one<T, WB, AMODE_GENV, EPI_SCORE>(g, st);
        }
    }
    return hipErrorInvalidValue;
}

hipError_t launch_gemm(int dtype, int tile, int amode, int epi, GemmArgs g, hipStream_t st)
{
    const int edge = tile_edge(tile);
    if (g.M <= 0) return hipSuccess;
    if (g.N <= 0 || g.N % edge != 0 || g.K <= 0 || g.K % slab_k(dtype) != 0) return hipErrorInvalidValue;
    g.m_tiles = (g.M + edge - 1) / edge;
    g.n_tiles = g.N / edge;
    if (dtype == AB_BF16) {
        switch (tile) {
        case TILE_SMALL: return launch_tile<bf16_t, 1>(amode, epi, g, st);
        case TILE_MID:   return launch_tile<bf16_t, 2>(amode, epi, g, st);
        case TILE_BIG:   return launch_tile<bf16_t, 4>(amode, epi, g, st);
        }
    } else {
        switch (tile) {
        case TILE_SMALL: return launch_tile<float, 1>(amode, epi, g, st);
        case TILE_MID:   return launch_tile<float, 2>(amode, epi, g, st);
        case TILE_BIG:   return launch_tile<float, 4>(amode, epi, g, st);
        }
    }
    return hipErrorInvalidValue;
}

}  // namespace ab
