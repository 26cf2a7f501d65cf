// Active-channel selection (Section 2.1 Top-K sparsity; Section 4 operation T; Section 6
// threshold form) as one 1024-thread workgroup per vector.
//
// The vector (n <= 32768 fp16 = 64 KB) lives in LDS for the whole kernel.  Top-k is an exact
// two-digit radix select on the 15-bit magnitude key (fp16 bits with the sign cleared):
//   pass 1  histogram of the high 8 bits  -> digit d1 that holds the k-th largest key
//   pass 2  histogram of the low 7 bits of the keys whose high digit is d1 -> digit d2
//   pass 3  keys > T are kept, keys == T are kept while the tie quota lasts, in index
//           order; an ordered block scan turns the flags into ascending positions.
// Histograms are replicated 16x (lane & 15 picks the copy) so that equal keys inside one
// wave do not serialise on a single LDS address.  Each thread owns a contiguous chunk of the
// vector in pass 3, which makes the scan order the index order.
#include "af_internal.h"

#define SEL_THREADS 1024
#define SEL_WAVES (SEL_THREADS / AF_WAVE)
#define HIST_COPIES 16

struct SelSmem {
  unsigned hist[256 * HIST_COPIES];  // 16 KB
  unsigned merged[256];
  unsigned wave_tot[SEL_WAVES];
  float red[SEL_WAVES];
  unsigned digit, above;             // result of a digit search
  unsigned total;
};

__device__ __forceinline__ unsigned wave_incl_scan(unsigned v, int) { return af_wave_incl_scan(v); }

// Exclusive prefix of v over the block in thread order; total in sm.total.
__device__ __forceinline__ unsigned block_excl_scan(unsigned v, SelSmem& sm) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  unsigned inc = wave_incl_scan(v, lane);
  if (lane == 63) sm.wave_tot[wave] = inc;
  __syncthreads();
  unsigned base = 0;
#pragma unroll
  for (int w = 0; w < SEL_WAVES; ++w) {
    unsigned t = sm.wave_tot[w];
    if (w < wave) base += t;
  }
  if (threadIdx.x == SEL_THREADS - 1) sm.total = base + inc;
  __syncthreads();
  return base + inc - v;
}

// Find the digit d (0..nbins-1, nbins <= 256) with  count(digit > d) < want <= count(digit >= d)
// from the replicated histogram.  Needs want >= 1 and want <= total count.
__device__ __forceinline__ void find_digit(SelSmem& sm, int nbins, unsigned want) {
  const int tid = threadIdx.x;
  if (tid < 256) {
    unsigned s = 0;
    if (tid < nbins) {
#pragma unroll
      for (int c = 0; c < HIST_COPIES; ++c) s += sm.hist[tid * HIST_COPIES + c];
    }
    sm.merged[tid] = s;
  }
  __syncthreads();
  if (tid < AF_WAVE) {
    // lane l owns bins 4l..4l+3; suffix sums via a reversed inclusive scan
    unsigned b0 = sm.merged[4 * tid], b1 = sm.merged[4 * tid + 1], b2 = sm.merged[4 * tid + 2],
             b3 = sm.merged[4 * tid + 3];
    unsigned mine = b0 + b1 + b2 + b3;
    const unsigned pre = af_wave_incl_scan(mine);
    unsigned above = (unsigned)__builtin_amdgcn_readlane((int)pre, 63) - pre;  // bins of higher lanes
    // walk my four bins from the top
    unsigned cnt[4] = {b0, b1, b2, b3};
#pragma unroll
    for (int q = 3; q >= 0; --q) {
      if (above < want && want <= above + cnt[q]) {
        sm.digit = 4 * tid + q;
        sm.above = above;
      }
      above += cnt[q];
    }
  }
  __syncthreads();
}

__device__ __forceinline__ void zero_hist(SelSmem& sm) {
  for (int i = threadIdx.x; i < 256 * HIST_COPIES; i += SEL_THREADS) sm.hist[i] = 0;
}

template <int PRODUCER>
__global__ __launch_bounds__(SEL_THREADS) void select_kernel(af_select_args a) {
  extern __shared__ unsigned short xs[];  // n fp16 bit patterns (padded to a multiple of 8)
  __shared__ SelSmem sm;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = a.n;

  // ---- producer: bring x into LDS (and to x_out when it is computed here) --------------
  if (PRODUCER == AF_PRO_NONE) {
    const unsigned short* src = reinterpret_cast<const unsigned short*>(a.src);
    for (int j0 = tid; j0 < n; j0 += 4 * SEL_THREADS) {  // four loads in flight per thread
      unsigned short t[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) t[u] = (j0 + u * SEL_THREADS < n) ? src[j0 + u * SEL_THREADS] : 0;
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (j0 + u * SEL_THREADS < n) xs[j0 + u * SEL_THREADS] = t[u];
    }
  } else if (PRODUCER == AF_PRO_RMSNORM) {
    float ss = 0.f;
    for (int j = tid; j < n; j += SEL_THREADS) {
      float v = (float)a.src[j];
      ss += v * v;
    }
    ss = af_wave_sum(ss);
    if (lane == 0) sm.red[wave] = ss;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < SEL_WAVES; ++w) tot += sm.red[w];
    const float scale = 1.0f / sqrtf(tot / (float)n + a.eps);
    for (int j = tid; j < n; j += SEL_THREADS) {
      half_t h = (half_t)((float)a.src[j] * scale * (float)a.gain[j]);
      a.x_out[j] = h;
      xs[j] = __builtin_bit_cast(unsigned short, h);
    }
  } else {  // AF_PRO_SILUMUL
    for (int j = tid; j < n; j += SEL_THREADS) {
      float g = (float)a.src[j], u = (float)a.src[n + j];
      half_t h = (half_t)(g / (1.0f + expf(-g)) * u);
      a.x_out[j] = h;
      xs[j] = __builtin_bit_cast(unsigned short, h);
    }
  }
  if (a.mode == AF_SEL_DENSE) return;  // producer only
  zero_hist(sm);
  __syncthreads();

  // contiguous chunk of this thread for the ordered pass
  const int c = (n + SEL_THREADS - 1) / SEL_THREADS;
  const int j0 = min(tid * c, n), j1 = min(j0 + c, n);

  unsigned T = 0x8000u;  // keys are < 0x8000: nothing is above T until it is lowered
  unsigned quota = 0;
  if (a.mode == AF_SEL_TOPK && a.k > 0) {
    // pass 1: high 8 bits
    for (int j = tid; j < n; j += SEL_THREADS) {
      unsigned key = xs[j] & 0x7FFFu;
      atomicAdd(&sm.hist[(key >> 7) * HIST_COPIES + (lane & (HIST_COPIES - 1))], 1u);
    }
    __syncthreads();
    find_digit(sm, 256, (unsigned)a.k);
    const unsigned d1 = sm.digit, above1 = sm.above;
    __syncthreads();
    zero_hist(sm);
    __syncthreads();
    // pass 2: low 7 bits of the keys in bin d1
    for (int j = tid; j < n; j += SEL_THREADS) {
      unsigned key = xs[j] & 0x7FFFu;
      if ((key >> 7) == d1)
        atomicAdd(&sm.hist[(key & 127u) * HIST_COPIES + (lane & (HIST_COPIES - 1))], 1u);
    }
    __syncthreads();
    find_digit(sm, 128, (unsigned)a.k - above1);
    T = (d1 << 7) | sm.digit;
    quota = (unsigned)a.k - above1 - sm.above;  // how many keys equal to T are kept
    __syncthreads();
  }

  // pass 3: count, scan, write (ascending by construction)
  unsigned gt = 0, eq = 0;
  if (a.mode == AF_SEL_TOPK) {
    for (int j = j0; j < j1; ++j) {
      unsigned key = xs[j] & 0x7FFFu;
      gt += key > T;
      eq += key == T;
    }
  } else {
    for (int j = j0; j < j1; ++j) {
      float v = fabsf((float)__builtin_bit_cast(half_t, xs[j]));
      gt += v > a.t;
    }
  }
  // both counts stay below 2^16, so one scan carries them in the two halves of a word
  unsigned pre = block_excl_scan(gt | (eq << 16), sm);
  unsigned gt_before = pre & 0xFFFFu, eq_before = pre >> 16;
  unsigned pos = gt_before + min(eq_before, quota);
  unsigned eq_seen = eq_before;
  if (a.mode == AF_SEL_TOPK) {
    for (int j = j0; j < j1; ++j) {
      unsigned key = xs[j] & 0x7FFFu;
      bool keep = key > T;
      if (key == T) {
        keep = eq_seen < quota;
        ++eq_seen;
      }
      if (keep) a.idx[pos++] = j;
    }
  } else {
    for (int j = j0; j < j1; ++j) {
      float v = fabsf((float)__builtin_bit_cast(half_t, xs[j]));
      if (v > a.t) a.idx[pos++] = j;
    }
  }
  if (a.count != nullptr && tid == 0) {
    unsigned tot = sm.total;
    *a.count = (int)((tot & 0xFFFFu) + min(tot >> 16, quota));
  }
}

// The vector can need more dynamic LDS than the 64 KB a kernel gets by default.
static void allow_large_lds() {
  static bool done = false;
  if (done) return;
  done = true;
  const int bytes = 2 * AF_MAX_N;
  (void)hipFuncSetAttribute(reinterpret_cast<const void*>(select_kernel<AF_PRO_NONE>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  (void)hipFuncSetAttribute(reinterpret_cast<const void*>(select_kernel<AF_PRO_RMSNORM>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  (void)hipFuncSetAttribute(reinterpret_cast<const void*>(select_kernel<AF_PRO_SILUMUL>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

int af_launch_select(af_ctx* ctx, int producer, const af_select_args& a) {
  const size_t lds = af_align((size_t)a.n * 2, 16);
  allow_large_lds();
  dim3 grid(1), block(SEL_THREADS);
  switch (producer) {
    case AF_PRO_NONE:
      hipLaunchKernelGGL(select_kernel<AF_PRO_NONE>, grid, block, lds, ctx->stream, a);
      break;
    case AF_PRO_RMSNORM:
      hipLaunchKernelGGL(select_kernel<AF_PRO_RMSNORM>, grid, block, lds, ctx->stream, a);
      break;
    default:
      hipLaunchKernelGGL(select_kernel<AF_PRO_SILUMUL>, grid, block, lds, ctx->stream, a);
      break;
  }
  AF_LAUNCH_CHECK();
  return AF_OK;
}

extern "C" int af_select_topk(af_ctx* ctx, const void* x_f16, int n, int k, int32_t* idx) {
  if (!ctx || !x_f16 || (!idx && k > 0)) return AF_ENULL;
  if (n < 0 || n > AF_MAX_N || k < 0 || k > n) return AF_EINVAL;
  if (n == 0 || k == 0) return AF_OK;
  af_select_args a{};
  a.src = (const half_t*)x_f16;
  a.n = n;
  a.mode = AF_SEL_TOPK;
  a.k = k;
  a.idx = idx;
  return af_launch_select(ctx, AF_PRO_NONE, a);
}

extern "C" int af_select_threshold(af_ctx* ctx, const void* x_f16, int n, float t, int32_t* idx,
                                   int32_t* count) {
  if (!ctx || !x_f16 || !idx || !count) return AF_ENULL;
  if (n < 0 || n > AF_MAX_N) return AF_EINVAL;
  if (t != t) return AF_EINVAL;  // NaN threshold
  af_select_args a{};
  a.src = (const half_t*)x_f16;
  a.n = n;
  a.mode = AF_SEL_THRESHOLD;
  a.t = t;
  a.idx = idx;
  a.count = count;
  // n == 0 still has to write count = 0: the kernel handles an empty vector
  return af_launch_select(ctx, AF_PRO_NONE, a);
}
