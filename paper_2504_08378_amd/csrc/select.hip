// Stand-alone activation selection (Section 2.1 Top-K sparsity; Section 4 operation T;
// Section 6 threshold form): one 1024-thread workgroup per vector, the same exact radix
// select as the GEMV front end (row_prologue.h), writing the ascending index list.
//
// The vector (n <= 32768 fp16 = 64 KB) is copied to LDS, padded to a multiple of eight
// elements with values that can never be selected ahead of a real element: zeros for top-k
// (equal to the smallest magnitude, but with a higher index than every real element) and NaN
// for the threshold rule (NaN never passes a threshold).
#include "af_internal.h"
#include "row_prologue.h"

#define SEL_THREADS 1024

__global__ __launch_bounds__(SEL_THREADS) void select_kernel(af_row_src r, int n_valid) {
  typedef RowPrologue<SEL_THREADS> RP;
  extern __shared__ __align__(16) unsigned short xs[];
  __shared__ __align__(16) unsigned s_scratch[RP_SCRATCH_WORDS];
  __shared__ typename RP::Smem s_rp;
  const int tid = threadIdx.x;
  const unsigned short* src = reinterpret_cast<const unsigned short*>(r.src);
  const unsigned short pad = r.sel == AF_SEL_TOPK ? 0 : 0x7E00;
  // r.n is n_valid rounded up to a multiple of 8; four scalar loads in flight per thread
  for (int j0 = tid; j0 < r.n; j0 += 4 * SEL_THREADS) {
    unsigned short t[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int j = j0 + u * SEL_THREADS;
      t[u] = j < n_valid ? src[j] : pad;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int j = j0 + u * SEL_THREADS;
      if (j < r.n) xs[j] = t[u];
    }
  }
  __syncthreads();
  int nidx;
  RP::select_split(r, xs, s_scratch, s_rp, nullptr, 1, 0, true, true, &nidx);
}

static int launch_select(af_ctx* ctx, const half_t* x, int n, int mode, int k, float t, int32_t* idx,
                         int32_t* count) {
  static bool attr_done = false;
  if (!attr_done) {  // the vector can need more dynamic LDS than the 64 KB a kernel gets by default
    attr_done = true;
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(select_kernel),
                              hipFuncAttributeMaxDynamicSharedMemorySize, 2 * AF_MAX_N);
  }
  af_row_src r{};
  r.pro = AF_PRO_NONE;
  r.src = x;
  r.n = (n + 7) & ~7;
  r.sel = mode;
  r.k = k;
  r.t = t;
  r.idx_out = idx;
  r.count_out = count;
  const size_t lds = af_align((size_t)r.n * 2, 16);
  hipLaunchKernelGGL(select_kernel, dim3(1), dim3(SEL_THREADS), lds, ctx->stream, r, n);
  AF_LAUNCH_CHECK();
  return AF_OK;
}

extern "C" int af_select_topk(af_ctx* ctx, const void* x_f16, int n, int k, int32_t* idx) {
  if (!ctx || !x_f16 || (!idx && k > 0)) return AF_ENULL;
  if (n < 0 || n > AF_MAX_N || k < 0 || k > n) return AF_EINVAL;
  if (n == 0 || k == 0) return AF_OK;
  return launch_select(ctx, (const half_t*)x_f16, n, AF_SEL_TOPK, k, 0.f, idx, nullptr);
}

extern "C" int af_select_threshold(af_ctx* ctx, const void* x_f16, int n, float t, int32_t* idx,
                                   int32_t* count) {
  if (!ctx || !x_f16 || !idx || !count) return AF_ENULL;
  if (n < 0 || n > AF_MAX_N) return AF_EINVAL;
  if (t != t) return AF_EINVAL;  // NaN threshold
  // n == 0 still has to write count = 0: the kernel handles an empty vector
  return launch_select(ctx, (const half_t*)x_f16, n, AF_SEL_THRESHOLD, 0, t, idx, count);
}
