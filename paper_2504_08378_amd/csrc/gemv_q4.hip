// Gathered-row sparse GEMV over 4-bit group-quantised weights with the dequantisation fused
// into the row loop (Section 4 operation C on the 4-bit weights of Section 7.1; the layout
// keeps a channel's nibbles contiguous as in Section 6 "Flash loading").
//
//   y[o] = sum_{t} (nib[idx[t]][o] - 8) * s[idx[t] / 32][o] * x[idx[t]]
//
// Layout: packed u8 [in][ld/2] (byte i of a row = columns 2i, 2i+1), scales fp16 [in/32][ld].
// The scale of a group does not depend on the row inside the group, so it is factored out:
// each lane keeps  acc_g[c] = sum_{t in group} q * x  and folds  y[c] += s[c] * acc_g[c]  when
// its rows move on to the next group (the index list is ascending, so groups are visited in
// order).  A lane's rows are a contiguous slice of the split, which makes group changes rare.
//
// Unpacking: a dword holds 8 nibbles (columns c..c+7).  Masking two nibbles into the mantissa
// of the fp16 constant 1024 gives the pair (1024 + n_a, 1024 + n_b) in one and-or; a packed
// fp16 subtract of 1032 leaves the exact integers q = n - 8.  Nibbles sitting four bits higher
// come out as 16*q and are multiplied with x/16 instead.  Accumulation is fp32.
#include "af_internal.h"

#define Q4_THREADS 256
#define Q4_WAVES (Q4_THREADS / AF_WAVE)
#define Q4_CHUNK 1024

struct Q4Params {
  const unsigned char* packed;
  const half_t* scales;
  const half_t* x;
  const int32_t* idx;
  const int32_t* nidx_dev;
  float* partials;
  int* tickets;
  void* y;
  const half_t* residual;
  int out, ld, nidx_host, y_kind, out_pad;
};

__device__ __forceinline__ void q4_store_out(const Q4Params& p, int col, float v) {
  if (p.residual) v += (float)p.residual[col];
  if (p.y_kind == AF_F16)
    reinterpret_cast<half_t*>(p.y)[col] = (half_t)v;
  else
    reinterpret_cast<float*>(p.y)[col] = v;
}

// acc[0..7] += q[c] * x for the 8 nibbles of w; column order inside the dword is
// (0,4),(1,5),(2,6),(3,7) -> acc slots {0,4,1,5,2,6,3,7}.
__device__ __forceinline__ void q4_fma8(float* acc, unsigned w, float x, float x16) {
  const unsigned magic = 0x64006400u;  // fp16 1024.0 twice
  const half2v off_lo = {(half_t)1032.0f, (half_t)1032.0f};
  const half2v off_hi = {(half_t)1152.0f, (half_t)1152.0f};  // 1024 + 16*8
  const unsigned w2 = w >> 8;
  half2v a = __builtin_bit_cast(half2v, (w & 0x000F000Fu) | magic) - off_lo;   // cols 0,4
  half2v b = __builtin_bit_cast(half2v, (w & 0x00F000F0u) | magic) - off_hi;   // 16 * cols 1,5
  half2v c = __builtin_bit_cast(half2v, (w2 & 0x000F000Fu) | magic) - off_lo;  // cols 2,6
  half2v d = __builtin_bit_cast(half2v, (w2 & 0x00F000F0u) | magic) - off_hi;  // 16 * cols 3,7
  acc[0] += (float)a[0] * x;
  acc[4] += (float)a[1] * x;
  acc[1] += (float)b[0] * x16;
  acc[5] += (float)b[1] * x16;
  acc[2] += (float)c[0] * x;
  acc[6] += (float)c[1] * x;
  acc[3] += (float)d[0] * x16;
  acc[7] += (float)d[1] * x16;
}

template <int LX, int U, bool HAS_IDX>
__global__ __launch_bounds__(Q4_THREADS) void gemv_q4_kernel(Q4Params p) {
  constexpr int LY = AF_WAVE / LX;
  constexpr int TW = LX * 8;
  constexpr int NSLOT = Q4_WAVES * LY;  // row slices per workgroup
  __shared__ int s_idx[Q4_CHUNK];
  __shared__ float s_x[Q4_CHUNK];
  __shared__ float s_red[Q4_WAVES][TW];
  __shared__ int s_last;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lx = lane % LX, ly = lane / LX;
  const int col = blockIdx.x * TW + lx * 8;
  const int col_ld = col < p.out ? col : 0;
  const int S = gridDim.y, s = blockIdx.y;
  const int slot = wave * LY + ly;

  int nidx = p.nidx_host;
  if (p.nidx_dev) nidx = min(*p.nidx_dev, nidx);
  const int R = (nidx + S - 1) / S;
  const int r0 = min(s * R, nidx), r1 = min(r0 + R, nidx);

  float yacc[8], acc[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) yacc[c] = acc[c] = 0.f;
  int cur_g = -1;
  half8 sc;
#pragma unroll
  for (int c = 0; c < 8; ++c) sc[c] = (half_t)0;
  const size_t row_bytes = (size_t)(p.ld / 2);
  const unsigned char* wcol = p.packed + col_ld / 2;

  auto consume = [&](int j, unsigned w, float xv) {
    const int g = j >> 5;
    if (g != cur_g) {
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        yacc[c] += (float)sc[c] * acc[c];
        acc[c] = 0.f;
      }
      cur_g = g;
      sc = *reinterpret_cast<const half8*>(p.scales + (size_t)g * p.ld + col_ld);
    }
    q4_fma8(acc, w, xv, xv * 0.0625f);
  };

  for (int base = r0; base < r1; base += Q4_CHUNK) {
    const int cnt = min(Q4_CHUNK, r1 - base);
    __syncthreads();
    for (int i = tid; i < cnt; i += Q4_THREADS) {
      int j = HAS_IDX ? p.idx[base + i] : base + i;
      s_idx[i] = j;
      s_x[i] = (float)p.x[j];
    }
    __syncthreads();
    const int per = (cnt + NSLOT - 1) / NSLOT;
    int i = min(slot * per, cnt);
    const int iend = min(i + per, cnt);
    for (; i + U <= iend; i += U) {
      unsigned w[U];
      float xv[U];
      int jj[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        jj[u] = s_idx[i + u];
        xv[u] = s_x[i + u];
        w[u] = *reinterpret_cast<const unsigned*>(wcol + (size_t)jj[u] * row_bytes);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) consume(jj[u], w[u], xv[u]);
    }
    for (; i < iend; ++i) {
      const int j = s_idx[i];
      unsigned w = *reinterpret_cast<const unsigned*>(wcol + (size_t)j * row_bytes);
      consume(j, w, s_x[i]);
    }
  }
#pragma unroll
  for (int c = 0; c < 8; ++c) yacc[c] += (float)sc[c] * acc[c];

#pragma unroll
  for (int off = LX; off < AF_WAVE; off <<= 1)
#pragma unroll
    for (int c = 0; c < 8; ++c) yacc[c] += __shfl_xor(yacc[c], off, AF_WAVE);
  if (ly == 0) {
#pragma unroll
    for (int c = 0; c < 8; ++c) s_red[wave][lx * 8 + c] = yacc[c];
  }
  __syncthreads();

  const int tile0 = blockIdx.x * TW;
  if (S == 1) {
    for (int c = tid; c < TW; c += Q4_THREADS) {
      if (tile0 + c < p.out) {
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < Q4_WAVES; ++w) v += s_red[w][c];
        q4_store_out(p, tile0 + c, v);
      }
    }
    return;
  }
  float* mine = p.partials + (size_t)s * p.out_pad;
  for (int c = tid; c < TW; c += Q4_THREADS) {
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < Q4_WAVES; ++w) v += s_red[w][c];
    af_store_agent(mine + tile0 + c, v);
  }
  af_stores_done();
  __syncthreads();
  if (tid == 0) {
    int old = af_ticket_take(&p.tickets[blockIdx.x]);
    s_last = (old == S - 1);
  }
  __syncthreads();
  if (!s_last) return;
  for (int c = tid; c < TW; c += Q4_THREADS) {
    if (tile0 + c < p.out) {
      q4_store_out(p, tile0 + c, af_sum_partials(p.partials + tile0 + c, p.out_pad, S));
    }
  }
  if (tid == 0) af_ticket_reset(&p.tickets[blockIdx.x]);
}

template <int LX, int U>
static void launch_q4(bool has_idx, dim3 grid, hipStream_t st, const Q4Params& p) {
  if (has_idx)
    hipLaunchKernelGGL((gemv_q4_kernel<LX, U, true>), grid, dim3(Q4_THREADS), 0, st, p);
  else
    hipLaunchKernelGGL((gemv_q4_kernel<LX, U, false>), grid, dim3(Q4_THREADS), 0, st, p);
}

int af_launch_gemv_q4(af_ctx* ctx, const af_gemv_args& a) {
  int lx = a.out <= 4096 ? 16 : (a.out <= 16384 ? 32 : 64);
  if (const char* e = getenv("AF_Q4_LX")) {
    int v = atoi(e);
    if (v == 16 || v == 32 || v == 64) lx = v;
  }
  const int tw = lx * 8;
  const int tiles = (a.out + tw - 1) / tw;
  const int out_pad = tiles * tw;
  if (tiles > AF_TICKET_ATTN) return AF_ESHAPE;
  int target = ctx->n_cu * 8;
  if (const char* e = getenv("AF_Q4_WGS")) {
    int v = atoi(e);
    if (v > 0) target = v;
  }
  int S = (target + tiles - 1) / tiles;
  if (a.rows.pro != AF_PRO_NONE || a.rows.sel != AF_ROWS_GIVEN) return AF_EINVAL;  // no fused front end yet
  int max_s = (a.rows.nidx_host + 63) / 64;
  if (max_s < 1) max_s = 1;
  if (S > max_s) S = max_s;
  if (S > 256) S = 256;
  while (S > 1 && (size_t)S * out_pad > ctx->lay.partial_floats) --S;
  Q4Params p;
  p.packed = (const unsigned char*)a.W;
  p.scales = a.scales;
  p.x = a.rows.src;
  p.idx = a.rows.idx;
  p.nidx_dev = a.rows.nidx_dev;
  p.partials = (float*)(ctx->ws + ctx->lay.partials);
  p.tickets = (int*)(ctx->ws + ctx->lay.tickets);
  p.y = a.y;
  p.residual = a.residual;
  p.out = a.out;
  p.ld = a.ld;
  p.nidx_host = a.rows.nidx_host;
  p.y_kind = a.y_kind;
  p.out_pad = out_pad;
  dim3 grid(tiles, S);
  const bool has_idx = a.rows.idx != nullptr;
  if (lx == 64)
    launch_q4<64, 8>(has_idx, grid, ctx->stream, p);
  else if (lx == 32)
    launch_q4<32, 8>(has_idx, grid, ctx->stream, p);
  else
    launch_q4<16, 8>(has_idx, grid, ctx->stream, p);
  AF_LAUNCH_CHECK();
  return AF_OK;
}

extern "C" int af_sparse_gemv_q4(af_ctx* ctx, const void* packed, const void* scales_f16, int in,
                                 int out, int ld, const void* x_f16, const int32_t* idx,
                                 int nidx_host, const int32_t* nidx_dev, void* y, int y_kind,
                                 const void* residual_f16) {
  if (!ctx || !packed || !scales_f16 || !x_f16 || !y) return AF_ENULL;
  if (in <= 0 || out <= 0 || in > AF_MAX_N) return AF_EINVAL;
  if (in % 32 || out % 8 || ld % 8 || ld < out) return AF_ESHAPE;
  if (y_kind != AF_F16 && y_kind != AF_F32) return AF_EINVAL;
  if (idx == nullptr) {
    nidx_host = in;
    nidx_dev = nullptr;
  }
  if (nidx_host < 0 || nidx_host > in) return AF_EINVAL;
  if (!ctx->ws) return AF_EWORKSPACE;
  if (in > ctx->max_in || out > ctx->max_out) return AF_EWORKSPACE;
  af_gemv_args a{};
  a.W = packed;
  a.scales = (const half_t*)scales_f16;
  a.in = in;
  a.out = out;
  a.ld = ld;
  a.rows.pro = AF_PRO_NONE;
  a.rows.src = (const half_t*)x_f16;
  a.rows.n = in;
  a.rows.sel = AF_ROWS_GIVEN;
  a.rows.idx = idx;
  a.rows.nidx_host = nidx_host;
  a.rows.nidx_dev = nidx_dev;
  a.y = y;
  a.y_kind = y_kind;
  a.residual = (const half_t*)residual_f16;
  return af_launch_gemv_q4(ctx, a);
}
