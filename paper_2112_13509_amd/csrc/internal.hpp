// Internal declarations shared by the translation units of the library (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <atomic>
#include "../../include/autobyte.h"
#include "gemm_core.hpp"

namespace ab {

// Launch tracing (see ab_set_trace): brackets one launch with the two callback phases.
extern ab_trace_fn g_trace_fn;
extern void *g_trace_user;
struct TraceScope {
    const char *name; double work; int bytes; hipStream_t st;
    TraceScope(const char *n, double w, int is_bytes, hipStream_t s) : name(n), work(w), bytes(is_bytes), st(s)
    { if (g_trace_fn) g_trace_fn(name, 0, work, bytes, (void *)st, g_trace_user); }
    ~TraceScope() { if (g_trace_fn) g_trace_fn(name, 1, work, bytes, (void *)st, g_trace_user); }
};

// Feature transform phi(x) = (g(x) - shift) * scale with g the identity or the natural logarithm.
__device__ __forceinline__ float phi(float x, const ab_enc &e)
{
    const float gx = (e.kind == AB_ENC_LOG) ? logf(x) : x;
    return (gx - e.shift) * e.scale;
}

// Launch attributes that do not change while the process lives are looked up once per device: a kernel's
// dynamic-LDS limit (one DeviceOnce per kernel instantiation, a function-local static of its launcher) and the
// device's compute-unit count.  Devices beyond 63 are simply set up at every launch.
struct DeviceOnce { std::atomic<uint64_t> done{0}; };
inline hipError_t ensure_dynamic_lds(const void *kern, int bytes, DeviceOnce &once)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = (dev >= 0 && dev < 64) ? (1ull << dev) : 0;
    if (bit && (once.done.load(std::memory_order_acquire) & bit)) return hipSuccess;
    e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess && bit) once.done.fetch_or(bit, std::memory_order_release);
    return e;
}
inline hipError_t compute_units(int *cus)
{
    static std::atomic<int> cached[64];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 64) {
        const int c = cached[dev].load(std::memory_order_relaxed);
        if (c > 0) { *cus = c; return hipSuccess; }
    }
    e = hipDeviceGetAttribute(cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e == hipSuccess && dev >= 0 && dev < 64) cached[dev].store(*cus, std::memory_order_relaxed);
    return e;
}

enum { TILE_SMALL = 0, TILE_MID = 1, TILE_BIG = 2 };   // 64x64, 128x128, 256x256 work-group tiles

static inline int tile_edge(int tile) { return 64 << tile; }
static inline int slab_k(int dtype) { return dtype == AB_BF16 ? 64 : 32; }
static inline size_t elem_size(int dtype) { return dtype == AB_BF16 ? 2 : 4; }

// Fills m_tiles / n_tiles from M, N and the tile, then launches.  N must be a multiple of the tile edge.
hipError_t launch_gemm(int dtype, int tile, int amode, int epi, GemmArgs g, hipStream_t st);

// The 256x256 bf16 kernel (gemm_big.hip): EPI_STORE (bf16 out) or EPI_SCORE, AMODE_LOAD or AMODE_GEN.
bool gemm_big_supported(int dtype, int amode, int epi, const GemmArgs &g);
hipError_t launch_gemm_big(int amode, int epi, GemmArgs g, hipStream_t st);

hipError_t launch_encode_stats(int dtype, const ab_model_desc *d, const float *dyn, const float *scal,
                               void *xs, int64_t S, int ld, int col0, int with_stats, hipStream_t st);
hipError_t launch_prep_layer1(int dtype, const ab_model_desc *d, const void *W1, const float *b1, int F, int Fs,
                              int H1, int ld, void *w1s, const ab_grid *grid, float *b_term, float *cfg_vec,
                              const void *Wout, const float *b_out, int H_last, float *w_out_f, hipStream_t st);
hipError_t launch_encode_and_prep(int dtype, const ab_model_desc *d, const float *dyn, const float *scal, void *xs,
                                  int64_t S, int ld, const void *W1, const float *b1, int F, int Fs, int H1, void *w1s,
                                  const ab_grid *grid, float *b_term, float *cfg_vec, const void *Wout,
                                  const float *b_out, int H_last, float *w_out_f, bool *done, hipStream_t st);
hipError_t launch_finish_select(const float *partial, int nt, int64_t row_stride, const float *b_out,
                                float *scores, int64_t score_stride, int32_t *best_idx, float *best_score,
                                int64_t S, int C, hipStream_t st);
hipError_t launch_trigger(const float *scores, int64_t S, int C, int64_t row_stride, const int32_t *cur_idx,
                          const float *observed, float gain_threshold, float error_threshold, int32_t *best_idx,
                          float *gain, uint8_t *reconf, uint8_t *adapt, hipStream_t st);
hipError_t launch_score_single_hidden(const float *a_term, const float *b_term, const float *w_out_f,
                                      float *partial, int64_t rows, int C, int H, const float *wp, const float *wc,
                                      const float *xp_row, const float *xc_row, hipStream_t st);
hipError_t launch_grid_rows(const ab_model_desc *d, const float *part, const float *cred, int P, int Q,
                            float *xp_row, float *xc_row, int64_t rows, hipStream_t st);
hipError_t launch_chosen_pair(const ab_model_desc *d, const ab_grid *grid, const int32_t *best_idx,
                              float *xp_sel, float *xc_sel, int64_t S, hipStream_t st);
hipError_t launch_output_v(int dtype, const float *h_last, const float *a_term, const float *wp, const float *wc,
                           const float *xp_sel, const float *xc_sel, const void *W, const float *b, int H, int n_out,
                           const int32_t *best_idx, float *V, int64_t S, hipStream_t st);
hipError_t launch_score_linear(int dtype, const ab_model_desc *d, const ab_params *prm, const float *dyn,
                               const float *scal, const ab_grid *grid, int64_t S, float *scores, int32_t *best_idx,
                               float *best_score, float *v_best, hipStream_t st);
bool score_tiny_supported(const ab_model_desc *d, int64_t S, int32_t C);
hipError_t launch_score_tiny(int dtype, const ab_model_desc *d, const ab_params *prm, const float *dyn,
                             const float *scal, const float *part, const float *cred, int32_t P, int32_t Q,
                             int per_scenario, int64_t S, float *scores, int32_t *best_idx, float *best_score,
                             hipStream_t st);
hipError_t launch_lstm_encoder(const ab_model_desc *d, const float *dyn, const void *We, const float *be,
                               const void *W1, const float *b1, const void *W2, const float *b2, void *xs,
                               int ld, int64_t S, const int32_t *layers_of, hipStream_t st);
hipError_t launch_tensor_encoder(int dtype, const ab_model_desc *d, const float *dyn, const void *Wa,
                                 const float *ba, const void *Wb, const float *bb, void *xs, int ld,
                                 int64_t S, const int32_t *layers_of, hipStream_t st);

}  // namespace ab
