// Gathered-row sparse GEMV over an input-channel-major fp16 matrix (Section 4, operation C;
// layout of Section 6 "Flash loading").
//
//   y[o] = sum_{t < nidx} Wt[idx[t]][o] * x[idx[t]]  (+ residual[o])
//
// Decomposition.  The output columns are cut into tiles of TW = 8*LX columns; the index list
// is cut into S contiguous splits; workgroup (tile, split) streams its rows.  Inside a wave,
// LX lanes span the tile (16 bytes = 8 columns per lane, one global_load_dwordx4) and the
// remaining 64/LX lane groups take different rows, so one wave instruction fetches 64/LX
// rows x (16*LX) contiguous bytes.  The row loop is unrolled U deep to keep U independent
// 16-byte loads per lane in flight.  idx[t] and x[idx[t]] of the split are staged in LDS
// first, so the weight addresses never wait on a dependent global load.
// Reduction: lane groups by wave shuffles, waves through LDS, splits through an fp32
// partials buffer; the workgroup that arrives last at a tile's ticket adds the S partials in
// split order, so the result does not depend on scheduling.
#include "af_internal.h"

#define GEMV_THREADS 256
#define GEMV_WAVES (GEMV_THREADS / AF_WAVE)
#define GEMV_CHUNK 1024  // staged (idx, x) pairs per pass

struct GemvParams {
  const half_t* W;
  const half_t* x;
  const int32_t* idx;
  const int32_t* nidx_dev;
  float* partials;
  int* tickets;
  void* y;
  const half_t* residual;
  int out, ld, nidx_host, y_kind, out_pad;
};

__device__ __forceinline__ void store_out(const GemvParams& p, int col, float v) {
  if (p.residual) v += (float)p.residual[col];
  if (p.y_kind == AF_F16)
    reinterpret_cast<half_t*>(p.y)[col] = (half_t)v;
  else
    reinterpret_cast<float*>(p.y)[col] = v;
}

template <int LX, int U, bool HAS_IDX>
__global__ __launch_bounds__(GEMV_THREADS) void gemv_f16_kernel(GemvParams p) {
  constexpr int LY = AF_WAVE / LX;
  constexpr int TW = LX * 8;
  constexpr int STEP = GEMV_WAVES * LY;  // rows taken per workgroup iteration
  __shared__ int s_idx[GEMV_CHUNK];
  __shared__ float s_x[GEMV_CHUNK];
  __shared__ float s_red[GEMV_WAVES][TW];
  __shared__ int s_last;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lx = lane % LX, ly = lane / LX;
  const int col = blockIdx.x * TW + lx * 8;
  const int col_ld = col < p.out ? col : 0;  // lanes past the edge read column 0 and are dropped
  const int S = gridDim.y, s = blockIdx.y;

  int nidx = p.nidx_host;
  if (p.nidx_dev) nidx = min(*p.nidx_dev, nidx);
  const int R = (nidx + S - 1) / S;
  const int r0 = min(s * R, nidx), r1 = min(r0 + R, nidx);

  float acc[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) acc[c] = 0.f;
  const half_t* wcol = p.W + col_ld;

  for (int base = r0; base < r1; base += GEMV_CHUNK) {
    const int cnt = min(GEMV_CHUNK, r1 - base);
    __syncthreads();
    for (int i = tid; i < cnt; i += GEMV_THREADS) {
      int j = HAS_IDX ? p.idx[base + i] : base + i;
      s_idx[i] = j;
      s_x[i] = (float)p.x[j];
    }
    __syncthreads();
    int i = wave * LY + ly;
    for (; i + (U - 1) * STEP < cnt; i += U * STEP) {
      half8 w[U];
      float xv[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int j = s_idx[i + u * STEP];
        xv[u] = s_x[i + u * STEP];
        w[u] = *reinterpret_cast<const half8*>(wcol + (size_t)j * p.ld);
      }
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[c] += (float)w[u][c] * xv[u];
    }
    for (; i < cnt; i += STEP) {
      const int j = s_idx[i];
      const float xv = s_x[i];
      half8 w = *reinterpret_cast<const half8*>(wcol + (size_t)j * p.ld);
#pragma unroll
      for (int c = 0; c < 8; ++c) acc[c] += (float)w[c] * xv;
    }
  }

  // lane groups -> one row of sums per wave
#pragma unroll
  for (int off = LX; off < AF_WAVE; off <<= 1)
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[c] += __shfl_xor(acc[c], off, AF_WAVE);
  if (ly == 0) {
#pragma unroll
    for (int c = 0; c < 8; ++c) s_red[wave][lx * 8 + c] = acc[c];
  }
  __syncthreads();

  const int tile0 = blockIdx.x * TW;
  if (S == 1) {
    for (int c = tid; c < TW; c += GEMV_THREADS) {
      if (tile0 + c < p.out) {
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < GEMV_WAVES; ++w) v += s_red[w][c];
        store_out(p, tile0 + c, v);
      }
    }
    return;
  }

  float* mine = p.partials + (size_t)s * p.out_pad;
  for (int c = tid; c < TW; c += GEMV_THREADS) {
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < GEMV_WAVES; ++w) v += s_red[w][c];
    af_store_agent(mine + tile0 + c, v);  // out_pad covers whole tiles
  }
  af_stores_done();
  __syncthreads();
  if (tid == 0) {
    int old = af_ticket_take(&p.tickets[blockIdx.x]);
    s_last = (old == S - 1);
  }
  __syncthreads();
  if (!s_last) return;
  for (int c = tid; c < TW; c += GEMV_THREADS) {
    if (tile0 + c < p.out) {
      store_out(p, tile0 + c, af_sum_partials(p.partials + tile0 + c, p.out_pad, S));
    }
  }
  if (tid == 0) af_ticket_reset(&p.tickets[blockIdx.x]);  // ready for the next launch
}

template <int LX, int U>
static void launch_variant(bool has_idx, dim3 grid, hipStream_t st, const GemvParams& p) {
  if (has_idx)
    hipLaunchKernelGGL((gemv_f16_kernel<LX, U, true>), grid, dim3(GEMV_THREADS), 0, st, p);
  else
    hipLaunchKernelGGL((gemv_f16_kernel<LX, U, false>), grid, dim3(GEMV_THREADS), 0, st, p);
}

// Tile width and split count for a shape.  AF_GEMV_LX / AF_GEMV_SPLIT / AF_GEMV_WGS in the
// environment override the heuristic (used by the tuning sweeps of the benchmark).
static void choose_config(const af_ctx* ctx, int out, int nidx, int* lx_out, int* s_out) {
  // Measured on the 7B operators (cold matrices): 128-column tiles (256 B per row and
  // workgroup) win up to ~16K columns, 256-column tiles beyond; narrow outputs want about one
  // workgroup per CU (long row loops, few partials), wide ones about four.
  int lx = out <= 16384 ? 16 : 32;
  int target_wgs = out <= 4096 ? ctx->n_cu : ctx->n_cu * 4;
  if (const char* e = getenv("AF_GEMV_LX")) {
    int v = atoi(e);
    if (v == 16 || v == 32 || v == 64) lx = v;
  }
  if (const char* e = getenv("AF_GEMV_WGS")) {
    int v = atoi(e);
    if (v > 0) target_wgs = v;
  }
  const int tiles = (out + lx * 8 - 1) / (lx * 8);
  int S = (target_wgs + tiles - 1) / tiles;
  if (const char* e = getenv("AF_GEMV_SPLIT")) {
    int v = atoi(e);
    if (v > 0) S = v;
  }
  const int min_rows = 32;  // a split shorter than this is mostly reduction overhead
  int max_s = (nidx + min_rows - 1) / min_rows;
  if (max_s < 1) max_s = 1;
  if (S > max_s) S = max_s;
  if (S > 256) S = 256;
  if (S < 1) S = 1;
  *lx_out = lx;
  *s_out = S;
}

int af_launch_gemv_f16(af_ctx* ctx, const af_gemv_args& a) {
  int lx, S;
  choose_config(ctx, a.out, a.nidx_host, &lx, &S);
  const int tw = lx * 8;
  const int tiles = (a.out + tw - 1) / tw;
  const int out_pad = tiles * tw;
  if (tiles > AF_TICKET_ATTN) return AF_ESHAPE;
  while (S > 1 && (size_t)S * out_pad > ctx->lay.partial_floats) --S;
  GemvParams p;
  p.W = (const half_t*)a.W;
  p.x = a.x;
  p.idx = a.idx;
  p.nidx_dev = a.nidx_dev;
  p.partials = (float*)(ctx->ws + ctx->lay.partials);
  p.tickets = (int*)(ctx->ws + ctx->lay.tickets);
  p.y = a.y;
  p.residual = a.residual;
  p.out = a.out;
  p.ld = a.ld;
  p.nidx_host = a.nidx_host;
  p.y_kind = a.y_kind;
  p.out_pad = out_pad;
  dim3 grid(tiles, S);
  const bool has_idx = a.idx != nullptr;
  if (lx == 64)
    launch_variant<64, 8>(has_idx, grid, ctx->stream, p);
  else if (lx == 32)
    launch_variant<32, 8>(has_idx, grid, ctx->stream, p);
  else
    launch_variant<16, 8>(has_idx, grid, ctx->stream, p);
  AF_LAUNCH_CHECK();
  return AF_OK;
}

extern "C" int af_sparse_gemv_f16(af_ctx* ctx, const void* Wt, int in, int out, int ld,
                                  const void* x_f16, const int32_t* idx, int nidx_host,
                                  const int32_t* nidx_dev, void* y, int y_kind,
                                  const void* residual_f16) {
  if (!ctx || !Wt || !x_f16 || !y) return AF_ENULL;
  if (in <= 0 || out <= 0 || in > AF_MAX_N) return AF_EINVAL;
  if (out % 8 || ld % 8 || ld < out) return AF_ESHAPE;
  if (y_kind != AF_F16 && y_kind != AF_F32) return AF_EINVAL;
  if (idx == nullptr) {
    nidx_host = in;
    nidx_dev = nullptr;
  }
  if (nidx_host < 0 || nidx_host > in) return AF_EINVAL;
  if (!ctx->ws) return AF_EWORKSPACE;
  if (in > ctx->max_in || out > ctx->max_out) return AF_EWORKSPACE;
  af_gemv_args a{};
  a.W = Wt;
  a.in = in;
  a.out = out;
  a.ld = ld;
  a.x = (const half_t*)x_f16;
  a.idx = idx;
  a.nidx_host = nidx_host;
  a.nidx_dev = nidx_dev;
  a.y = y;
  a.y_kind = y_kind;
  a.residual = (const half_t*)residual_f16;
  return af_launch_gemv_f16(ctx, a);
}
