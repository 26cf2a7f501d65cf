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
#include "row_prologue.h"

#define Q4_LIST 2048  // rows given by the caller are staged this many at a time

struct Q4Params {
  const unsigned char* packed;
  const half_t* scales;
  af_row_src rows;
  float* partials;
  int* tickets;
  void* y;
  const half_t* residual;
  int out, ld, y_kind, out_pad, use_lds_x;
  int range_sel;  // threshold selection per channel range, no list for the whole vector
  int list_off;   // byte offset of the staged-row list in dynamic LDS (behind x)
  // output slots over device-selected matrices, as in the fp16 kernel: slot s reads the packed
  // rows at packed + w_sel[s] * w_stride bytes and the scales at scales + w_sel[s] * s_stride
  int cols_per_slot, tiles_per_slot;
  const int* w_sel;
  long long w_stride, s_stride;
  const float* y_scale;
  // in-kernel router of a mixture-of-experts block, as in the fp16 kernel
  const half_t* router_Wr;
  int router_E, router_top;
  int32_t* router_experts;
  float* router_weights;
  float* router_logits;
  long long* prof;  // time stamps of this launch (af_profile_set), or null
};

__device__ __forceinline__ void q4_store_out(const Q4Params& p, int col, float v) {
  if (p.y_scale) v *= *p.y_scale;
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

// CL = false: scales [in/32][ld], one per (group of 32 input channels, column);
// CL = true:  scales [in][ld/32], one per (input channel, group of 32 columns).
// MODE: producer and row source as compile-time constants (pro | kind << 2; kind 0 rows given,
// 1 top-k, 2 threshold with a list, 3 threshold per channel range), or -1 for the generic kernel
// that reads them from its arguments; see gemv_f16_body.h for what this buys.
#define Q4_MODE(pro, kind) ((pro) | ((kind) << 2))
template <int LX, int U, int NW, bool CL, bool ROUTED, int MODE = -1>
__global__ __launch_bounds__(NW * AF_WAVE) void gemv_q4_kernel(Q4Params p_in) {
  Q4Params p = p_in;
  if constexpr (MODE >= 0) {
    constexpr int pro = MODE & 3, kind = MODE >> 2;
    p.rows.pro = pro;
    p.rows.sel = kind == 0 ? (int)AF_ROWS_GIVEN : (kind == 1 ? (int)AF_SEL_TOPK : (int)AF_SEL_THRESHOLD);
    p.use_lds_x = (pro != AF_PRO_NONE || kind != 0) ? 1 : 0;
    p.range_sel = kind == 3 ? 1 : 0;
  }
  constexpr int THREADS = NW * AF_WAVE;
  constexpr int LY = AF_WAVE / LX;
  constexpr int TW = LX * 8;
  constexpr int NSLOT = NW * LY;  // row slices per workgroup
  constexpr int SCRATCH = RP_SCRATCH_WORDS > NW * TW ? RP_SCRATCH_WORDS : NW * TW;
  typedef RowPrologue<THREADS> RP;
  extern __shared__ __align__(16) unsigned short xs[];
  __shared__ __align__(16) unsigned s_scratch[SCRATCH];  // histograms, later the wave sums
  __shared__ typename RP::Smem s_rp;
  __shared__ int s_last;
  float(*s_red)[TW] = reinterpret_cast<float(*)[TW]>(s_scratch);
  // staged rows, (index << 16 | fp16 bits of x)
  unsigned* s_list = reinterpret_cast<unsigned*>(reinterpret_cast<char*>(xs) + p.list_off);

  af_prof_begin(p.prof);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lx = lane % LX, ly = lane / LX;
  // one slot (a plain GEMV): no division
  const int slot_o = p.tiles_per_slot >= (int)gridDim.x ? 0 : (int)blockIdx.x / p.tiles_per_slot;
  const int tile_in = blockIdx.x - slot_o * p.tiles_per_slot;
  const int col = tile_in * TW + lx * 8;  // column inside the slot
  const int col_ld = col < p.cols_per_slot ? col : tile_in * TW;
  const int S = gridDim.y, s = blockIdx.y;
  const int slot = wave * LY + ly;
  const af_row_src& r = p.rows;

  constexpr int RE = 8;  // experts the in-kernel router handles
  constexpr bool routed = ROUTED;
  half8 wr[routed ? RE : 1];
  if constexpr (routed) {  // this thread's router weights do not depend on x: fetch them first
#pragma unroll
    for (int e = 0; e < RE; ++e) {
#pragma unroll
      for (int c = 0; c < 8; ++c) wr[e][c] = (half_t)0;
      if (e < p.router_E && tid < (r.n >> 3))
        wr[e] = *reinterpret_cast<const half8*>(p.router_Wr + (size_t)e * r.n + (size_t)tid * 8);
    }
  }
  if (p.use_lds_x && (!p.range_sel || routed))
    RP::produce(r, xs, s_rp, s == 0, blockIdx.x, gridDim.x,
                r.sel == AF_SEL_TOPK ? s_scratch : nullptr);
  if constexpr (routed) {
    RP::template router_in_lds<RE>(xs, r.n, s_rp, wr, p.router_E, p.router_top);
    if (blockIdx.x == 0 && s == 0) {
      if (tid < p.router_top) {
        p.router_experts[tid] = s_rp.experts[tid];
        p.router_weights[tid] = s_rp.weights[tid];
      }
      if (tid < p.router_E) p.router_logits[tid] = s_rp.logit[tid];
    }
  }

  float yacc[8], acc[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) yacc[c] = acc[c] = 0.f;
  int cur_g = -1;
  half8 sc;
#pragma unroll
  for (int c = 0; c < 8; ++c) sc[c] = (half_t)0;
  const size_t row_bytes = (size_t)(p.ld / 2);
  const unsigned char* wcol = p.packed + col_ld / 2;
  const half_t* sbase = p.scales;
  if (routed || p.w_sel) {
    const int e_sel = routed ? s_rp.experts[slot_o] : p.w_sel[slot_o];
    wcol += (size_t)e_sel * (size_t)p.w_stride;
    sbase += (size_t)e_sel * (size_t)p.s_stride;
  }

  auto consume = [&](unsigned e, unsigned w) {
    const int g = (int)(e >> 21);  // (index >> 5)
    if (g != cur_g) {
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        yacc[c] += (float)sc[c] * acc[c];
        acc[c] = 0.f;
      }
      cur_g = g;
      sc = *reinterpret_cast<const half8*>(sbase + (size_t)g * p.ld + col_ld);
    }
    const float xv = (float)__builtin_bit_cast(half_t, (unsigned short)(e & 0xFFFFu));
    q4_fma8(acc, w, xv, xv * 0.0625f);
  };
  // channel-local scales: the row's scale of this lane's column group multiplies x
  const size_t srow = (size_t)(p.ld / 32);
  const half_t* scol = sbase + col_ld / 32;
  auto consume_cl = [&](unsigned e, unsigned w, half_t s_row) {
    const float xv = (float)__builtin_bit_cast(half_t, (unsigned short)(e & 0xFFFFu)) * (float)s_row;
    q4_fma8(yacc, w, xv, xv * 0.0625f);
  };
  // One pass over `cnt` staged rows: every (wave, lane group) slot takes a contiguous slice,
  // so it crosses few group boundaries.
  auto stream = [&](int cnt) {
    const int per = (cnt + NSLOT - 1) / NSLOT;
    int i = min(slot * per, cnt);
    const int iend = min(i + per, cnt);
    for (; i + U <= iend; i += U) {
      unsigned w[U], e[U];
      half_t sr[U];
      half8 sg[U];  // group-32 layout: the scales of a row that opens a new group, fetched with the batch
      int gprev = cur_g;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        e[u] = s_list[i + u];
        w[u] = af_load_once(reinterpret_cast<const unsigned*>(wcol + (size_t)(e[u] >> 16) * row_bytes));
        if (CL) {
          sr[u] = scol[(size_t)(e[u] >> 16) * srow];
        } else {
          const int g = (int)(e[u] >> 21);
          if (g != gprev) sg[u] = *reinterpret_cast<const half8*>(sbase + (size_t)g * p.ld + col_ld);
          gprev = g;
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (CL) {
          consume_cl(e[u], w[u], sr[u]);
        } else {
          const int g = (int)(e[u] >> 21);
          if (g != cur_g) {  // fold the finished group, switch to the scales that came with the batch
#pragma unroll
            for (int c = 0; c < 8; ++c) {
              yacc[c] += (float)sc[c] * acc[c];
              acc[c] = 0.f;
            }
            cur_g = g;
            sc = sg[u];
          }
          const float xv = (float)__builtin_bit_cast(half_t, (unsigned short)(e[u] & 0xFFFFu));
          q4_fma8(acc, w[u], xv, xv * 0.0625f);
        }
      }
    }
    // Ragged end: one more batch of the same depth with the missing rows masked off, so its
    // loads are in flight together instead of one memory round trip per row.
    if (i < iend) {
      unsigned w[U], e[U];
      half_t sr[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const bool ok = i + u < iend;
        e[u] = ok ? s_list[i + u] : 0u;
        w[u] = ok ? af_load_once(reinterpret_cast<const unsigned*>(wcol + (size_t)(e[u] >> 16) * row_bytes)) : 0u;
        if (CL) sr[u] = ok ? scol[(size_t)(e[u] >> 16) * srow] : (half_t)0;
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (i + u < iend) {
          if (CL)
            consume_cl(e[u], w[u], sr[u]);
          else
            consume(e[u], w[u]);
        }
      }
    }
  };

  if (p.range_sel) {
    stream(routed ? RP::threshold_range_of_full(r, xs, s_rp, s_list, S, s)
                  : RP::threshold_range(r, xs, s_rp, s_list, S, s, blockIdx.x == 0));
  } else if (r.sel != AF_ROWS_GIVEN) {
    int nidx_total;
    const int cnt = RP::select_split(r, xs, s_scratch, s_rp, s_list, S, s, blockIdx.x == 0,
                                     blockIdx.x == 0 && s == 0, &nidx_total, p.use_lds_x != 0);
    stream(cnt);
  } else {
    int nidx = r.nidx_host;
    if (r.nidx_dev) nidx = min(*r.nidx_dev, nidx);
    const int R = af_ceil_div_small(nidx, S);
    const int r0 = min(s * R, nidx), r1 = min(r0 + R, nidx);
    const unsigned short* xg = reinterpret_cast<const unsigned short*>(r.src);
    for (int base = r0; base < r1; base += Q4_LIST) {
      const int cnt = min(Q4_LIST, r1 - base);
      __syncthreads();
      for (int i = tid; i < cnt; i += THREADS) {
        const int j = r.idx ? r.idx[base + i] : base + i;
        if ((unsigned)j < (unsigned)r.n) {
          const unsigned bits = p.use_lds_x ? xs[j] : xg[j];
          s_list[i] = ((unsigned)j << 16) | bits;
        } else {  // broken precondition: row 0 times zero, and the error word
          s_list[i] = 0u;
          af_report_bad_index(p.tickets);
        }
      }
      __syncthreads();
      stream(cnt);
    }
  }
  if (!CL) {
#pragma unroll
    for (int c = 0; c < 8; ++c) yacc[c] += (float)sc[c] * acc[c];
  }
  __syncthreads();  // s_scratch changes its role: histograms -> wave sums

#pragma unroll
  for (int off = LX; off < AF_WAVE; off <<= 1)
#pragma unroll
    for (int c = 0; c < 8; ++c) yacc[c] += __shfl_xor(yacc[c], off, AF_WAVE);
  if (ly == 0) {
#pragma unroll
    for (int c = 0; c < 8; ++c) s_red[wave][lx * 8 + c] = yacc[c];
  }
  __syncthreads();

  const int tile0 = blockIdx.x * TW;                        // in the padded column space
  const int out0 = slot_o * p.cols_per_slot + tile_in * TW;  // first output column of the tile
  const int valid = min(TW, p.cols_per_slot - tile_in * TW);
  if (S == 1) {
    for (int c = tid; c < valid; c += THREADS) {
      float v = 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) v += s_red[w][c];
      q4_store_out(p, out0 + c, v);
    }
    af_prof_end(p.prof);
    return;
  }
  float* mine = p.partials + (size_t)s * p.out_pad;
  for (int c = tid; c < TW; c += THREADS) {
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) v += s_red[w][c];
    af_store_agent(mine + tile0 + c, v);
  }
  af_stores_done();
  __syncthreads();
  if (tid == 0) {
    int old = af_ticket_take(&p.tickets[blockIdx.x]);
    s_last = (old == S - 1);
  }
  __syncthreads();
  if (!s_last) {
    af_prof_end(p.prof);
    return;
  }
  for (int c = tid; c < valid; c += THREADS)
    q4_store_out(p, out0 + c, af_sum_partials(p.partials + tile0 + c, p.out_pad, S));
  if (tid == 0) af_ticket_reset(&p.tickets[blockIdx.x]);
  af_prof_end(p.prof);
}

template <int LX, int NW, bool CL, bool ROUTED, int MODE>
static void q4_launch_one(dim3 grid, size_t lds, hipStream_t st, const Q4Params& p) {
  static bool attr_done = false;
  if (!attr_done) {  // the input vector and the staged rows can need more than the default 64 KB
    attr_done = true;
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(gemv_q4_kernel<LX, 8, NW, CL, ROUTED, MODE>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, AF_GEMV_LDS_BUDGET);
  }
  hipLaunchKernelGGL((gemv_q4_kernel<LX, 8, NW, CL, ROUTED, MODE>), grid, dim3(NW * AF_WAVE), lds, st, p);
}

// the (producer, selection) pairs of a decoder layer get an instantiation of their own
template <int LX, bool CL>
static void q4_launch_mode(dim3 grid, size_t lds, hipStream_t st, const Q4Params& p) {
  const int kind = p.rows.sel == AF_ROWS_GIVEN ? 0 : (p.rows.sel == AF_SEL_TOPK ? 1 : (p.range_sel ? 3 : 2));
  switch (Q4_MODE(p.rows.pro, kind)) {
#define AF_MODE_CASE(pro, kind_) \
  case Q4_MODE(pro, kind_):      \
    q4_launch_one<LX, 16, CL, false, Q4_MODE(pro, kind_)>(grid, lds, st, p); \
    break;
    AF_MODE_CASE(AF_PRO_RMSNORM, 1)
    AF_MODE_CASE(AF_PRO_NONE, 1)
    AF_MODE_CASE(AF_PRO_SILUMUL, 1)
    AF_MODE_CASE(AF_PRO_RMSNORM, 3)
    AF_MODE_CASE(AF_PRO_NONE, 3)
    AF_MODE_CASE(AF_PRO_SILUMUL, 3)
    AF_MODE_CASE(AF_PRO_RMSNORM, 0)
    AF_MODE_CASE(AF_PRO_NONE, 0)
    AF_MODE_CASE(AF_PRO_SILUMUL, 0)
#undef AF_MODE_CASE
    default:
      q4_launch_one<LX, 16, CL, false, -1>(grid, lds, st, p);
  }
}

template <int LX>
static void q4_launch_lx(int nw, bool cl, dim3 grid, size_t lds, hipStream_t st, const Q4Params& p) {
  if (p.router_Wr != nullptr) {  // the launcher has made sure of nw == 16
    if (cl)
      q4_launch_one<LX, 16, true, true, -1>(grid, lds, st, p);
    else
      q4_launch_one<LX, 16, false, true, -1>(grid, lds, st, p);
  } else if (nw == 16) {
    if (cl)
      q4_launch_mode<LX, true>(grid, lds, st, p);
    else
      q4_launch_mode<LX, false>(grid, lds, st, p);
  } else {
    if (cl)
      q4_launch_one<LX, 4, true, false, -1>(grid, lds, st, p);
    else
      q4_launch_one<LX, 4, false, false, -1>(grid, lds, st, p);
  }
}

int af_launch_gemv_q4(af_ctx* ctx, const af_gemv_args& a) {
  const af_row_src& r = a.rows;
  const bool selects = r.sel != AF_ROWS_GIVEN;
  const int max_rows = r.sel == AF_SEL_TOPK ? r.k : (r.sel == AF_SEL_THRESHOLD ? r.n : r.nidx_host);
  // a lane covers 8 columns = 4 bytes of a packed row; tiles of 8*LX columns
  int lx = a.out <= 4096 ? 16 : (a.out <= 16384 ? 32 : 64);
  // one 1024-thread workgroup per compute unit measured faster than four 256-thread ones for
  // every form of this kernel (with or without the selecting front end)
  int nw = 16;
  if (ctx->tune_lx == 16 || ctx->tune_lx == 32 || ctx->tune_lx == 64) lx = ctx->tune_lx;
  if (ctx->tune_nw == 4 || ctx->tune_nw == 16) nw = ctx->tune_nw;
  const int tw = lx * 8;
  const int n_slots = a.w_sel ? a.n_slots : 1;
  if (n_slots < 1 || a.out % n_slots) return AF_EINVAL;
  const int cols_per_slot = a.out / n_slots;
  if (cols_per_slot % (a.q4_channel_local ? 32 : 8)) return AF_ESHAPE;
  const int tiles_per_slot = (cols_per_slot + tw - 1) / tw;
  const int tiles = n_slots * tiles_per_slot;
  const int out_pad = tiles * tw;
  if (tiles > AF_TICKET_ATTN) return AF_ESHAPE;
  int target = nw == 16 ? ctx->n_cu : ctx->n_cu * 4;
  if (ctx->tune_wgs > 0) target = ctx->tune_wgs;
  int S = target / tiles;
  int max_s = (max_rows + 63) / 64;
  if (max_s < 1) max_s = 1;
  if (S > max_s) S = max_s;
  if (S > 256) S = 256;
  if (S < 1) S = 1;
  const bool range_sel = r.sel == AF_SEL_THRESHOLD && !r.idx_out && !r.count_out;
  const bool use_lds_x = r.pro != AF_PRO_NONE || selects;
  size_t xs_bytes;
  int list_cap;
  // the split partial sums have to fit the workspace, the staged rows of a split the LDS
  while (S > 1 && (size_t)S * out_pad > ctx->lay.partial_floats) --S;
  if (a.router_Wr && (r.pro != AF_PRO_RMSNORM || a.router_E > 8 || r.n > 8192 || nw != 16 || !use_lds_x))
    return AF_EINVAL;  // the in-kernel router's preconditions (the caller falls back to the router kernel)
  if (!af_plan_gemv_lds(r, max_rows, use_lds_x, range_sel, Q4_LIST, &S, &xs_bytes, &list_cap,
                        a.router_Wr != nullptr))
    return AF_EWORKSPACE;
  if (S > 1 && (size_t)S * out_pad > ctx->lay.partial_floats) return AF_EWORKSPACE;
  Q4Params p;
  p.packed = (const unsigned char*)a.W;
  p.scales = a.scales;
  p.rows = r;
  p.partials = (float*)(ctx->ws + ctx->lay.partials);
  p.tickets = (int*)(ctx->ws + ctx->lay.tickets);
  p.y = a.y;
  p.residual = a.residual;
  p.out = a.out;
  p.ld = a.ld;
  p.y_kind = a.y_kind;
  p.out_pad = out_pad;
  p.use_lds_x = use_lds_x ? 1 : 0;
  p.range_sel = range_sel ? 1 : 0;
  p.list_off = (int)xs_bytes;
  p.cols_per_slot = cols_per_slot;
  p.tiles_per_slot = tiles_per_slot;
  p.w_sel = a.w_sel;
  p.w_stride = a.w_stride;      // bytes of packed nibbles per matrix
  p.s_stride = a.w_stride_scales;  // scale elements per matrix
  p.y_scale = a.y_scale;
  p.router_Wr = a.router_Wr;
  p.router_E = a.router_E;
  p.router_top = a.router_top;
  p.router_experts = a.router_experts;
  p.router_weights = a.router_weights;
  p.router_logits = a.router_logits;
  p.prof = af_prof_take(ctx);
  const size_t lds = xs_bytes + (size_t)list_cap * 4;
  dim3 grid(tiles, S);
  if (lx == 64)
    q4_launch_lx<64>(nw, a.q4_channel_local, grid, lds, ctx->stream, p);
  else if (lx == 32)
    q4_launch_lx<32>(nw, a.q4_channel_local, grid, lds, ctx->stream, p);
  else
    q4_launch_lx<16>(nw, a.q4_channel_local, grid, lds, ctx->stream, p);
  AF_LAUNCH_CHECK();
  return AF_OK;
}

static int sparse_gemv_q4_any(af_ctx* ctx, bool cl, const void* packed, const void* scales_f16,
                              int in, int out, int ld, const void* x_f16, const int32_t* idx,
                              int nidx_host, const int32_t* nidx_dev, void* y, int y_kind,
                              const void* residual_f16) {
  if (!ctx || !packed || !scales_f16 || !x_f16 || !y) return AF_ENULL;
  if (in <= 0 || out <= 0 || in > AF_MAX_N) return AF_EINVAL;
  if (cl ? (out % 32 || ld % 32 || ld < out) : (in % 32 || out % 8 || ld % 8 || ld < out))
    return AF_ESHAPE;
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
  a.q4_channel_local = cl;
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
  if (ctx->validate) {
    const int rc = af_validate_idx(ctx, idx, nidx_host, nidx_dev, in);
    if (rc) return rc;
  }
  return af_launch_gemv_q4(ctx, a);
}

extern "C" int af_sparse_gemv_q4(af_ctx* ctx, const void* packed, const void* scales_f16, int in,
                                 int out, int ld, const void* x_f16, const int32_t* idx,
                                 int nidx_host, const int32_t* nidx_dev, void* y, int y_kind,
                                 const void* residual_f16) {
  return sparse_gemv_q4_any(ctx, false, packed, scales_f16, in, out, ld, x_f16, idx, nidx_host,
                            nidx_dev, y, y_kind, residual_f16);
}

extern "C" int af_sparse_gemv_q4_cl(af_ctx* ctx, const void* packed, const void* scales_f16, int in,
                                    int out, int ld, const void* x_f16, const int32_t* idx,
                                    int nidx_host, const int32_t* nidx_dev, void* y, int y_kind,
                                    const void* residual_f16) {
  return sparse_gemv_q4_any(ctx, true, packed, scales_f16, in, out, ld, x_f16, idx, nidx_host,
                            nidx_dev, y, y_kind, residual_f16);
}
