// Small-batch decode over the union of the tokens' active sets (extension of Section 4's
// operation C from one token to B <= 8 tokens; the paper itself decodes one token at a time).
//
//   Y[b][o] = sum_{j in idx_b[b]} Wt[j][o] * X[b][j]
//
// Step 1 (three small launches): set bit b of channel j's word in a device-memory mask for every
// entry j of token b's list (the batched decoder layer does this inside its selection launch
// instead); per 256 channels, turn the mask words into Xm[j][b] = X[b][j] if
// token b keeps channel j else 0 (fp16, 8 tokens per row = one 16-byte load in the GEMV) and into
// the range's part of the ascending union U; move the parts into place behind the lower ranges.
// Step 2: the gathered GEMV of gemv_f16.hip over U with B accumulator sets per lane; every
// weight row of the union is read once for all tokens.
#include "af_internal.h"

#define UB_THREADS 1024
#define UB_WAVES (UB_THREADS / AF_WAVE)
#define UB_RANGE 256   // channels per workgroup of the builder
#define UB_MAX_RANGES (AF_MAX_N / UB_RANGE)

struct UnionBuildParams {
  const half_t* X;         // [B][in]
  const int32_t* idx_b;    // [B][idx_stride], k entries used (or counts[b] of them)
  const int32_t* counts;   // per-token list lengths on the device, or null: k for every token
  unsigned* mask;          // [in]: bit b of word j = token b keeps channel j; zero between calls
  int32_t* range_list;     // [ranges][UB_RANGE]: the union's channels of each range, ascending
  int32_t* range_cnt;      // [ranges]
  int32_t* union_idx;      // [in]
  int32_t* union_n;        // [1]
  half_t* Xm;              // [in][8]
  int B, k, in, idx_stride, ranges;
  int* tickets;            // the device error word lies behind them
};

// Builder, first launch: every list entry is looked at once.  Grid (chunks of a list, tokens);
// a thread takes up to four entries of its token's list and sets the token's bit in the
// channel's word of a mask in device memory (all zero between calls).  An entry outside [0, in)
// is dropped and reported.
__global__ __launch_bounds__(UB_THREADS) void union_mark_kernel(UnionBuildParams p) {
  const int b = blockIdx.y;
  const int kb = p.counts ? min(max(p.counts[b], 0), p.k) : p.k;
  const int32_t* list = p.idx_b + (size_t)b * p.idx_stride;
  const int t0 = blockIdx.x * (4 * UB_THREADS) + threadIdx.x;
  int j[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) j[u] = t0 + u * UB_THREADS < kb ? list[t0 + u * UB_THREADS] : -1;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    if (t0 + u * UB_THREADS >= kb) continue;
    if ((unsigned)j[u] < (unsigned)p.in)
      __hip_atomic_fetch_or(p.mask + j[u], 1u << b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else
      af_report_bad_index(p.tickets);  // broken precondition
  }
}

// Builder, second launch: workgroup r owns the channels [r * UB_RANGE, (r + 1) * UB_RANGE): it
// takes their mask words (and clears them for the next call), writes their masked, transposed
// token values and leaves its part of the union, in ascending order, in range_list.
__global__ __launch_bounds__(UB_RANGE) void union_gather_kernel(UnionBuildParams p) {
  __shared__ unsigned s_wtot[UB_RANGE / AF_WAVE];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = blockIdx.x;
  const int c0 = r * UB_RANGE, cn = min(UB_RANGE, p.in - c0);
  const bool in_range = tid < cn;
  unsigned m = 0;
  if (in_range) {
    m = __hip_atomic_load(p.mask + c0 + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (m) __hip_atomic_store(p.mask + c0 + tid, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    half8 v;
#pragma unroll
    for (int b = 0; b < 8; ++b)
      v[b] = (b < p.B && ((m >> b) & 1u)) ? p.X[(size_t)b * p.in + c0 + tid] : (half_t)0;
    *reinterpret_cast<half8*>(p.Xm + (size_t)(c0 + tid) * 8) = v;
  }
  const unsigned flag = m != 0;
  const unsigned inc = af_wave_incl_scan(flag);
  if (lane == 63) s_wtot[wave] = inc;
  __syncthreads();
  unsigned base = 0, total = 0;
#pragma unroll
  for (int w = 0; w < UB_RANGE / AF_WAVE; ++w) {
    const unsigned t = s_wtot[w];
    if (w < wave) base += t;
    total += t;
  }
  if (flag) p.range_list[(size_t)r * UB_RANGE + base + inc - 1] = c0 + tid;
  if (tid == 0) p.range_cnt[r] = (int)total;
}

// Builder, third launch: workgroup r moves its range's channels to their place in the union
// (behind the channels of all lower ranges); workgroup 0 also writes the union's size.
#define UP_THREADS 256
__global__ __launch_bounds__(UP_THREADS) void union_place_kernel(UnionBuildParams p) {
  __shared__ int s_base, s_total;
  const int tid = threadIdx.x, r = blockIdx.x;
  if (tid < AF_WAVE) {  // the first wave adds up the range counts (at most 128 of them)
    int below = 0, all = 0;
    for (int q = tid; q < p.ranges; q += AF_WAVE) {
      const int c = p.range_cnt[q];
      all += c;
      if (q < r) below += c;
    }
    below = (int)af_wave_sum((unsigned)below);
    all = (int)af_wave_sum((unsigned)all);
    if (tid == 0) {
      s_base = below;
      s_total = all;
    }
  }
  __syncthreads();
  const int cnt = p.range_cnt[r];
  if (tid < cnt) p.union_idx[s_base + tid] = p.range_list[(size_t)r * UB_RANGE + tid];
  if (r == 0 && tid == 0) *p.union_n = s_total;
}

#define UG_THREADS 256
#define UG_WAVES (UG_THREADS / AF_WAVE)
#define UG_CHUNK 512

struct UnionGemvParams {
  const half_t* W;
  const half_t* Xm;        // [in][8]
  const int32_t* idx;      // union
  const int32_t* nidx_dev;
  float* partials;         // [S][B][out_pad]
  int* tickets;
  void* Y;                 // [B][out]
  const half_t* residual;  // [B][out] added to the product, or null
  int out, ld, nidx_host, y_kind, out_pad, B;
};

// U rows times NB tokens into the accumulators.  NB >= 4: the rows are taken in pairs through
// v_dot2_f32_f16 (two products and the add in one instruction; 16 packs + 64 dot instructions per
// row pair instead of 128 multiply-adds at NB = 8), because at eight tokens the multiply-adds, not
// the weight stream, were what the kernel waited for (vector ALU busy 59 %; gate|up of the 70B
// shape 188 -> 172 us; at four tokens the change is neutral).  Zero rows may be
// passed for the masked end of a list.
template <int NB, int U>
__device__ __forceinline__ void union_accumulate(float (&acc)[NB][8], const half8 (&w)[U], const half8 (&xm)[U]) {
  if constexpr (NB >= 4 && U % 2 == 0) {
#pragma unroll
    for (int u = 0; u < U; u += 2) {
      half2v wp[8];
#pragma unroll
      for (int c = 0; c < 8; ++c) wp[c] = half2v{w[u][c], w[u + 1][c]};
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        const half2v xp = half2v{xm[u][b], xm[u + 1][b]};
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[b][c] = __builtin_amdgcn_fdot2(wp[c], xp, acc[b][c], false);
      }
    }
  } else {
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        const float xv = (float)xm[u][b];
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[b][c] += (float)w[u][c] * xv;
      }
    }
  }
}

template <int NB, int LX, int U>
__global__ __launch_bounds__(UG_THREADS) void gemv_union_kernel(UnionGemvParams p) {
  constexpr int LY = AF_WAVE / LX;
  constexpr int TW = LX * 8;
  constexpr int STEP = UG_WAVES * LY;
  __shared__ int s_idx[UG_CHUNK];
  __shared__ half8 s_xm[UG_CHUNK];
  __shared__ float s_red[UG_WAVES][NB][TW];
  __shared__ int s_last;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lx = lane % LX, ly = lane / LX;
  const int col = blockIdx.x * TW + lx * 8;
  const int col_ld = col < p.out ? col : 0;
  const int S = gridDim.y, s = blockIdx.y;

  const int nidx = min(*p.nidx_dev, p.nidx_host);
  const int R = af_ceil_div_small(nidx, S);
  const int r0 = min(s * R, nidx), r1 = min(r0 + R, nidx);

  float acc[NB][8];
#pragma unroll
  for (int b = 0; b < NB; ++b)
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[b][c] = 0.f;
  const half_t* wcol = p.W + col_ld;

  for (int base = r0; base < r1; base += UG_CHUNK) {
    const int cnt = min(UG_CHUNK, r1 - base);
    __syncthreads();
    for (int i = tid; i < cnt; i += UG_THREADS) {
      const int j = p.idx[base + i];
      s_idx[i] = j;
      s_xm[i] = *reinterpret_cast<const half8*>(p.Xm + (size_t)j * 8);
    }
    __syncthreads();
    int i = wave * LY + ly;
    half8 zero8;
#pragma unroll
    for (int c = 0; c < 8; ++c) zero8[c] = (half_t)0;
    for (; i + (U - 1) * STEP < cnt; i += U * STEP) {
      half8 w[U], xm[U];
#pragma unroll
      for (int u = 0; u < U; ++u)
        w[u] = af_load_once(reinterpret_cast<const half8*>(wcol + (size_t)s_idx[i + u * STEP] * p.ld));
#pragma unroll
      for (int u = 0; u < U; ++u) xm[u] = s_xm[i + u * STEP];
      union_accumulate<NB, U>(acc, w, xm);
    }
    // ragged end: one masked batch of the same depth, its loads in flight together
    if (i < cnt) {
      half8 w[U], xm[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const bool ok = i + u * STEP < cnt;
        w[u] = ok ? af_load_once(reinterpret_cast<const half8*>(wcol + (size_t)s_idx[i + u * STEP] * p.ld)) : zero8;
        xm[u] = ok ? s_xm[i + u * STEP] : zero8;
      }
      union_accumulate<NB, U>(acc, w, xm);
    }
  }

#pragma unroll
  for (int off = LX; off < AF_WAVE; off <<= 1)
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int c = 0; c < 8; ++c) acc[b][c] += __shfl_xor(acc[b][c], off, AF_WAVE);
  if (ly == 0) {
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int c = 0; c < 8; ++c) s_red[wave][b][lx * 8 + c] = acc[b][c];
  }
  __syncthreads();

  const int tile0 = blockIdx.x * TW;
  auto store = [&](int b, int colg, float v) {
    if (b < p.B && colg < p.out) {
      if (p.residual) v += (float)p.residual[(size_t)b * p.out + colg];
      if (p.y_kind == AF_F16)
        reinterpret_cast<half_t*>(p.Y)[(size_t)b * p.out + colg] = (half_t)v;
      else
        reinterpret_cast<float*>(p.Y)[(size_t)b * p.out + colg] = v;
    }
  };
  if (S == 1) {
    for (int e = tid; e < NB * TW; e += UG_THREADS) {
      const int b = e / TW, c = e % TW;
      float v = 0.f;
#pragma unroll
      for (int w = 0; w < UG_WAVES; ++w) v += s_red[w][b][c];
      store(b, tile0 + c, v);
    }
    return;
  }
  float* mine = p.partials + (size_t)s * NB * p.out_pad;
  for (int e = tid; e < NB * TW; e += UG_THREADS) {
    const int b = e / TW, c = e % TW;
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < UG_WAVES; ++w) v += s_red[w][b][c];
    af_store_agent(mine + (size_t)b * p.out_pad + tile0 + c, v);
  }
  af_stores_done();
  __syncthreads();
  if (tid == 0) {
    int old = af_ticket_take(&p.tickets[blockIdx.x]);
    s_last = (old == S - 1);
  }
  __syncthreads();
  if (!s_last) return;
  for (int e = tid; e < NB * TW; e += UG_THREADS) {
    const int b = e / TW, c = e % TW;
    store(b, tile0 + c,
          af_sum_partials(p.partials + (size_t)b * p.out_pad + tile0 + c, (size_t)NB * p.out_pad, S));
  }
  if (tid == 0) af_ticket_reset(&p.tickets[blockIdx.x]);
}

int af_launch_union_f16(af_ctx* ctx, const af_union_args& u) {
  const int in = u.in, out = u.out, B = u.B, k = u.k;
  UnionBuildParams bp;
  bp.X = u.X;
  bp.idx_b = u.idx_b;
  bp.counts = u.counts;
  bp.range_list = (int32_t*)(ctx->ws + ctx->lay.union_ranges);
  bp.range_cnt = (int32_t*)(ctx->ws + ctx->lay.union_range_cnt);
  bp.union_idx = u.union_idx;
  bp.union_n = u.union_n;
  bp.Xm = (half_t*)(ctx->ws + ctx->lay.union_x);
  bp.B = B;
  bp.k = k;
  bp.in = in;
  bp.idx_stride = u.idx_stride;
  bp.ranges = (in + UB_RANGE - 1) / UB_RANGE;
  bp.tickets = (int*)(ctx->ws + ctx->lay.tickets);
  bp.mask = (unsigned*)(ctx->ws + ctx->lay.union_mask);
  if (k > 0 && !u.marked) {
    hipLaunchKernelGGL(union_mark_kernel, dim3((k + 4 * UB_THREADS - 1) / (4 * UB_THREADS), B), dim3(UB_THREADS), 0,
                       ctx->stream, bp);
    AF_LAUNCH_CHECK();
  }
  hipLaunchKernelGGL(union_gather_kernel, dim3(bp.ranges), dim3(UB_RANGE), 0, ctx->stream, bp);
  AF_LAUNCH_CHECK();
  hipLaunchKernelGGL(union_place_kernel, dim3(bp.ranges), dim3(UP_THREADS), 0, ctx->stream, bp);
  AF_LAUNCH_CHECK();

  const int NB = B == 1 ? 1 : (B == 2 ? 2 : (B <= 4 ? 4 : 8));
  const int lx = (out <= 2048) ? 16 : 32;
  const int tw = lx * 8;
  const int tiles = (out + tw - 1) / tw;
  const int out_pad = tiles * tw;
  if (tiles > AF_TICKET_ATTN) return AF_ESHAPE;
  const int nidx_max = (long long)B * k < in ? B * k : in;
  int S = (ctx->n_cu * 8 + tiles - 1) / tiles;
  int max_s = (nidx_max + 31) / 32;
  if (max_s < 1) max_s = 1;
  if (S > max_s) S = max_s;
  if (S > 256) S = 256;
  while (S > 1 && (size_t)S * NB * out_pad > ctx->lay.partial_floats) --S;

  UnionGemvParams p;
  p.W = (const half_t*)u.Wt;
  p.Xm = bp.Xm;
  p.idx = u.union_idx;
  p.nidx_dev = u.union_n;
  p.partials = (float*)(ctx->ws + ctx->lay.partials);
  p.tickets = (int*)(ctx->ws + ctx->lay.tickets);
  p.Y = u.Y;
  p.residual = u.residual;
  p.out = out;
  p.ld = u.ld;
  p.nidx_host = nidx_max;
  p.y_kind = u.y_kind;
  p.out_pad = out_pad;
  p.B = B;
  dim3 grid(tiles, S), block(UG_THREADS);
#define UNION_LAUNCH(NBV, LXV, UV) \
  hipLaunchKernelGGL((gemv_union_kernel<NBV, LXV, UV>), grid, block, 0, ctx->stream, p)
  if (lx == 16) {
    if (NB == 1) UNION_LAUNCH(1, 16, 8);
    else if (NB == 2) UNION_LAUNCH(2, 16, 8);
    else if (NB == 4) UNION_LAUNCH(4, 16, 4);
    else UNION_LAUNCH(8, 16, 4);
  } else {
    if (NB == 1) UNION_LAUNCH(1, 32, 8);
    else if (NB == 2) UNION_LAUNCH(2, 32, 8);
    else if (NB == 4) UNION_LAUNCH(4, 32, 4);
    else UNION_LAUNCH(8, 32, 4);
  }
#undef UNION_LAUNCH
  AF_LAUNCH_CHECK();
  return AF_OK;
}

extern "C" int af_sparse_gemv_union_f16(af_ctx* ctx, const void* Wt, int in, int out, int ld,
                                        const void* X_f16, int B, const int32_t* idx_b, int k,
                                        int32_t* union_idx, int32_t* union_n, void* Y, int y_kind) {
  if (!ctx || !Wt || !X_f16 || !union_idx || !union_n || !Y || (!idx_b && k > 0)) return AF_ENULL;
  if (in <= 0 || out <= 0 || in > AF_MAX_N || B < 1 || B > AF_MAX_BATCH || k < 0 || k > in)
    return AF_EINVAL;
  if (out % 8 || ld % 8 || ld < out) return AF_ESHAPE;
  if (y_kind != AF_F16 && y_kind != AF_F32) return AF_EINVAL;
  if (!ctx->ws) return AF_EWORKSPACE;
  if (in > ctx->max_in || out > ctx->max_out || B > ctx->max_batch) return AF_EWORKSPACE;
  if (ctx->validate)
    for (int b = 0; b < B; ++b) {
      const int rc = af_validate_idx(ctx, idx_b + (size_t)b * k, k, nullptr, in);
      if (rc) return rc;
    }
  af_union_args u{};
  u.Wt = Wt;
  u.in = in;
  u.out = out;
  u.ld = ld;
  u.X = (const half_t*)X_f16;
  u.B = B;
  u.idx_b = idx_b;
  u.idx_stride = k;
  u.k = k;
  u.union_idx = union_idx;
  u.union_n = union_n;
  u.Y = Y;
  u.y_kind = y_kind;
  return af_launch_union_f16(ctx, u);
}
