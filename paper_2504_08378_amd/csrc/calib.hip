// Threshold calibration for the threshold form of activation selection (Section 6: the index
// kernel keeps one activation threshold per sparsity level; Section 2.1 names the result
// Top-K sparsity).  The magnitudes of a calibration stream are counted exactly, one counter
// per 15-bit fp16 magnitude key, and a threshold is read off the counts: with N values pooled
// and m = N - floor(sp * N / 100) to keep, the threshold is the (m+1)-th largest magnitude.
#include "af_internal.h"

__global__ __launch_bounds__(256) void calib_hist_kernel(const unsigned short* x, int n,
                                                         unsigned* hist) {
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= n) return;
  const unsigned key = x[j] & 0x7FFFu;
  if (key <= 0x7C00u) atomicAdd(&hist[key], 1u);  // NaN stays out of the pool
}

#define CALIB_THREADS 1024
#define CALIB_PER_THREAD (AF_CALIB_BINS / CALIB_THREADS)  // 32 consecutive keys per thread

struct CalibLevels {
  int n;
  int sp[AF_CALIB_MAX_LEVELS];
};

__global__ __launch_bounds__(CALIB_THREADS) void calib_threshold_kernel(const unsigned* hist,
                                                                        CalibLevels lv, float* t_out) {
  __shared__ unsigned long long s_sum[CALIB_THREADS];
  __shared__ unsigned long long s_chunk[CALIB_THREADS / 64];
  const int tid = threadIdx.x;
  const int base = tid * CALIB_PER_THREAD;
  unsigned long long mine = 0;
  for (int b = 0; b < CALIB_PER_THREAD; ++b) mine += hist[base + b];
  s_sum[tid] = mine;
  __syncthreads();
  if (tid < CALIB_THREADS / 64) {
    unsigned long long c = 0;
    for (int u = 0; u < 64; ++u) c += s_sum[tid * 64 + u];
    s_chunk[tid] = c;
  }
  __syncthreads();
  unsigned long long N = 0, above = 0;  // above: values whose key lies beyond this thread's keys
  for (int c = 0; c < CALIB_THREADS / 64; ++c) {
    N += s_chunk[c];
    if (c > tid / 64) above += s_chunk[c];
  }
  for (int u = tid + 1; u < (tid / 64 + 1) * 64; ++u) above += s_sum[u];

  for (int l = 0; l < lv.n; ++l) {
    const unsigned long long m = N - (unsigned long long)lv.sp[l] * N / 100ull;
    if (m >= N) {  // nothing to drop: every magnitude exceeds -1
      if (tid == 0) t_out[l] = -1.0f;
      continue;
    }
    const unsigned long long want = m + 1;
    unsigned long long a = above;
    for (int b = CALIB_PER_THREAD - 1; b >= 0; --b) {
      const unsigned long long c = hist[base + b];
      if (a < want && want <= a + c)
        t_out[l] = (float)__builtin_bit_cast(half_t, (unsigned short)(base + b));
      a += c;
    }
  }
}

extern "C" int af_calib_accumulate(af_ctx* ctx, const void* x_f16, int n, uint32_t* hist) {
  if (!ctx || !hist || (!x_f16 && n > 0)) return AF_ENULL;
  if (n < 0) return AF_EINVAL;
  if (n == 0) return AF_OK;
  hipLaunchKernelGGL(calib_hist_kernel, dim3((n + 255) / 256), dim3(256), 0, ctx->stream,
                     (const unsigned short*)x_f16, n, hist);
  AF_LAUNCH_CHECK();
  return AF_OK;
}

extern "C" int af_calib_accumulate_layer(af_ctx* ctx, const af_layer_cfg* cfg, uint32_t* const* hist) {
  if (!ctx || !cfg || !hist) return AF_ENULL;
  if (!ctx->ws) return AF_EWORKSPACE;
  const int widths[4] = {cfg->d_model, cfg->n_heads * cfg->head_dim, cfg->d_model, cfg->d_ffn};
  const int tap[4] = {0, 2, 4, 6};
  for (int p = 0; p < 4; ++p) {
    if (!hist[p]) return AF_ENULL;
    if (widths[p] <= 0 || widths[p] > ctx->max_in) return AF_EWORKSPACE;
  }
  for (int p = 0; p < 4; ++p) {
    const int rc = af_calib_accumulate(ctx, ctx->ws + ctx->lay.act[tap[p]], widths[p], hist[p]);
    if (rc) return rc;
  }
  return AF_OK;
}

extern "C" int af_calib_thresholds(af_ctx* ctx, const uint32_t* hist, const int* sparsity_pct,
                                   int n_levels, float* t_out) {
  if (!ctx || !hist || !sparsity_pct || !t_out) return AF_ENULL;
  if (n_levels < 1 || n_levels > AF_CALIB_MAX_LEVELS) return AF_EINVAL;
  CalibLevels lv{};
  lv.n = n_levels;
  for (int l = 0; l < n_levels; ++l) {
    if (sparsity_pct[l] < 0 || sparsity_pct[l] > 100) return AF_EINVAL;
    lv.sp[l] = sparsity_pct[l];
  }
  hipLaunchKernelGGL(calib_threshold_kernel, dim3(1), dim3(CALIB_THREADS), 0, ctx->stream, hist, lv,
                     t_out);
  AF_LAUNCH_CHECK();
  return AF_OK;
}
