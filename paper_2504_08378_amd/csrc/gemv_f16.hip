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
// 16-byte loads per lane in flight.  The rows of the split are staged in LDS first as
// (index, x) pairs, so the weight addresses never wait on a dependent global load.
// Front end (row_prologue.h): the kernel can build its input vector itself (RMSNorm of the
// residual stream, SiLU(gate)*up) and run the top-k / threshold selection on it, each
// workgroup for itself, which removes the separate selection kernels from a decoder layer.
// With thresholds and no index list asked for, a workgroup decides only the channels of its
// own range (split by channel position instead of list position).
// Matrices picked on the device (mixture of experts): the output columns form slots of whole
// tiles and slot s reads W + w_sel[s] * w_stride, w_sel being device memory.
// Reduction: lane groups by wave shuffles, waves through LDS, splits through an fp32
// partials buffer; the workgroup that arrives last at a tile's ticket adds the S partials in
// split order, so the result does not depend on scheduling.
#include "af_internal.h"
#include "row_prologue.h"

#define GEMV_LIST 2048  // rows given by the caller are staged this many at a time

struct GemvParams {
  const half_t* W;
  af_row_src rows;
  float* partials;
  int* tickets;
  void* y;
  const half_t* residual;
  int out, ld, y_kind, out_pad, use_lds_x;
  int range_sel;  // threshold selection per channel range, no list for the whole vector
  int list_off;   // byte offset of the staged-row list in dynamic LDS (behind x)
  // Output columns come in `slots` of cols_per_slot columns, each covered by tiles_per_slot
  // tiles.  A plain GEMV has one slot.  With w_sel, slot s multiplies by the matrix
  // W + w_sel[s] * w_stride (leading dimension ld), so the experts a router picked on the
  // device are reached without a host round trip.  y_scale (device, one float) scales the
  // product before the residual is added.
  int cols_per_slot, tiles_per_slot;
  const int* w_sel;
  long long w_stride;
  const float* y_scale;
  // Router of a mixture-of-experts block run in this launch's front end (gate|up): every
  // workgroup works out the experts itself from x and uses them for its slot; workgroup
  // (0, 0) publishes them for the launches that follow.  Null router_Wr: no router.
  const half_t* router_Wr;  // [router_E][in]
  int router_E, router_top;
  int32_t* router_experts;
  float* router_weights;
  float* router_logits;
  long long* prof;  // time stamps of this launch (af_profile_set), or null
};

__device__ __forceinline__ void store_out(const GemvParams& p, int col, float v) {
  if (p.y_scale) v *= *p.y_scale;
  if (p.residual) v += (float)p.residual[col];
  if (p.y_kind == AF_F16)
    reinterpret_cast<half_t*>(p.y)[col] = (half_t)v;
  else
    reinterpret_cast<float*>(p.y)[col] = v;
}

// ROUTED: the instantiation that runs a mixture-of-experts router in its front end (kept apart
// so that the plain launches do not carry its registers).
template <int LX, int U, int NW, bool ROUTED>
__global__ __launch_bounds__(NW * AF_WAVE) void gemv_f16_kernel(GemvParams p) {
  constexpr int GEMV_THREADS = NW * AF_WAVE;
  constexpr int GEMV_WAVES = NW;
  constexpr int LY = AF_WAVE / LX;
  constexpr int TW = LX * 8;
  constexpr int STEP = GEMV_WAVES * LY;  // rows taken per workgroup iteration
  constexpr int SCRATCH = RP_SCRATCH_WORDS > NW * TW ? RP_SCRATCH_WORDS : NW * TW;
  typedef RowPrologue<GEMV_THREADS> RP;
  extern __shared__ __align__(16) unsigned short xs[];  // the operator input, when built here
  __shared__ __align__(16) unsigned s_scratch[SCRATCH];  // histograms, later the wave sums
  __shared__ typename RP::Smem s_rp;
  __shared__ int s_last;
  float(*s_red)[TW] = reinterpret_cast<float(*)[TW]>(s_scratch);
  // staged rows, (index << 16 | fp16 bits of x)
  unsigned* s_list = reinterpret_cast<unsigned*>(reinterpret_cast<char*>(xs) + p.list_off);

  af_prof_begin(p.prof);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lx = lane % LX, ly = lane / LX;
  const int slot = blockIdx.x / p.tiles_per_slot;
  const int tile_in = blockIdx.x - slot * p.tiles_per_slot;   // tile inside the slot
  const int col = tile_in * TW + lx * 8;                       // column inside the slot
  // lanes past the slot's edge read the tile's first column and are dropped at the store
  const int col_ld = col < p.cols_per_slot ? col : tile_in * TW;
  const int S = gridDim.y, s = blockIdx.y;
  const af_row_src& r = p.rows;

  // Rows given and their number known on the host: fetch this thread's share of the first
  // staging pass now, so that the index round trip overlaps the construction of x.
  constexpr int PF = GEMV_LIST / GEMV_THREADS;
  int pre[PF];
  const bool prefetched = r.sel == AF_ROWS_GIVEN && r.idx != nullptr && r.nidx_dev == nullptr;
  if (prefetched) {
    const int R = (r.nidx_host + S - 1) / S;
    const int r0 = min(s * R, r.nidx_host), r1 = min(r0 + R, r.nidx_host);
#pragma unroll
    for (int u = 0; u < PF; ++u) {
      const int i = r0 + tid + u * GEMV_THREADS;
      pre[u] = i < r1 ? r.idx[i] : 0;
    }
  }

  constexpr int RE = 8;  // experts the in-kernel router handles
  constexpr bool routed = ROUTED;
  half8 wr[routed ? RE : 1];
  if constexpr (routed) {  // this thread's router weights do not depend on x: fetch them before x is built
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

  float acc[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) acc[c] = 0.f;
  const half_t* wcol = p.W + col_ld;
  if (routed)
    wcol += (size_t)s_rp.experts[slot] * (size_t)p.w_stride;
  else if (p.w_sel)
    wcol += (size_t)p.w_sel[slot] * (size_t)p.w_stride;

  // One pass over `cnt` staged rows of s_list.
  auto stream = [&](int cnt) {
    int i = wave * LY + ly;
    for (; i + (U - 1) * STEP < cnt; i += U * STEP) {
      half8 w[U];
      unsigned e[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        e[u] = s_list[i + u * STEP];
        w[u] = *reinterpret_cast<const half8*>(wcol + (size_t)(e[u] >> 16) * p.ld);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const float xv = (float)__builtin_bit_cast(half_t, (unsigned short)(e[u] & 0xFFFFu));
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[c] += (float)w[u][c] * xv;
      }
    }
    // Ragged end: one more batch of the same depth with the missing rows masked off, so its
    // loads are all in flight together (a row-at-a-time loop would pay one memory round trip
    // per row, up to U - 1 of them in a row).
    if (i < cnt) {
      half8 w[U];
      unsigned e[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const bool ok = i + u * STEP < cnt;
        e[u] = ok ? s_list[i + u * STEP] : 0u;
        if (ok) {
          w[u] = *reinterpret_cast<const half8*>(wcol + (size_t)(e[u] >> 16) * p.ld);
        } else {
#pragma unroll
          for (int c = 0; c < 8; ++c) w[u][c] = (half_t)0;
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const float xv = (float)__builtin_bit_cast(half_t, (unsigned short)(e[u] & 0xFFFFu));
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[c] += (float)w[u][c] * xv;
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
    const int R = (nidx + S - 1) / S;
    const int r0 = min(s * R, nidx), r1 = min(r0 + R, nidx);
    const unsigned short* xg = reinterpret_cast<const unsigned short*>(r.src);
    for (int base = r0; base < r1; base += GEMV_LIST) {
      const int cnt = min(GEMV_LIST, r1 - base);
      __syncthreads();
      if (prefetched && base == r0) {
#pragma unroll
        for (int u = 0; u < PF; ++u) {
          const int i = tid + u * GEMV_THREADS;
          if (i < cnt) {
            const int j = pre[u];
            const unsigned bits = p.use_lds_x ? xs[j] : xg[j];
            s_list[i] = ((unsigned)j << 16) | bits;
          }
        }
      } else {
        for (int i = tid; i < cnt; i += GEMV_THREADS) {
          const int j = r.idx ? r.idx[base + i] : base + i;
          const unsigned bits = p.use_lds_x ? xs[j] : xg[j];
          s_list[i] = ((unsigned)j << 16) | bits;
        }
      }
      __syncthreads();
      stream(cnt);
    }
  }
  __syncthreads();  // s_scratch changes its role: histograms -> wave sums

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

  const int tile0 = blockIdx.x * TW;                      // in the padded column space
  const int out0 = slot * p.cols_per_slot + tile_in * TW;  // first output column of the tile
  const int valid = min(TW, p.cols_per_slot - tile_in * TW);
  if (S == 1) {
    for (int c = tid; c < valid; c += GEMV_THREADS) {
      float v = 0.f;
#pragma unroll
      for (int w = 0; w < GEMV_WAVES; ++w) v += s_red[w][c];
      store_out(p, out0 + c, v);
    }
    af_prof_end(p.prof);
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
  if (!s_last) {
    af_prof_end(p.prof);
    return;
  }
  for (int c = tid; c < valid; c += GEMV_THREADS)
    store_out(p, out0 + c, af_sum_partials(p.partials + tile0 + c, p.out_pad, S));
  if (tid == 0) af_ticket_reset(&p.tickets[blockIdx.x]);  // ready for the next launch
  af_prof_end(p.prof);
}

// Tile width, waves per workgroup and split count for a shape.  AF_GEMV_LX / AF_GEMV_NW /
// AF_GEMV_SPLIT / AF_GEMV_WGS in the environment override the heuristic (tuning sweeps).
static void choose_config(const af_ctx* ctx, int out, int nidx, bool selects, int* lx_out,
                          int* nw_out, int* s_out) {
  // Measured on the 7B and 13B operators (cold matrices): 128-column tiles (256 B per row and
  // workgroup) win up to ~16K columns, 512-column tiles (1 KB) beyond.  With 256-column tiles
  // on a row stride that is a multiple of 1 KB every workgroup stays on one value of address
  // bit 9 for all its rows, and the half of the workgroups on one of the two values finished
  // ~2 us after the other half.  A kernel that selects for itself (or builds its input
  // vector) repeats that work in every workgroup, so it runs few, large workgroups (one per
  // CU); a plain GEMV prefers several small ones per CU.
  int lx = out <= 16384 ? 16 : 64;
  int nw = selects ? 16 : 4;
  if (const char* e = getenv("AF_GEMV_LX")) {
    int v = atoi(e);
    if (v == 16 || v == 32 || v == 64) lx = v;
  }
  if (const char* e = getenv("AF_GEMV_NW")) {
    int v = atoi(e);
    if (v == 4 || v == 8 || v == 16) nw = v;
  }
  const int per_cu = 16 / nw;  // workgroups of nw waves that one CU holds at a time
  int target_wgs = nw == 4 ? (out <= 4096 ? ctx->n_cu : ctx->n_cu * 4) : ctx->n_cu * per_cu;
  if (const char* e = getenv("AF_GEMV_WGS")) {
    int v = atoi(e);
    if (v > 0) target_wgs = v;
  }
  const int tiles = (out + lx * 8 - 1) / (lx * 8);
  int S = target_wgs / tiles;  // never more workgroups than the chip holds at once
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
  *nw_out = nw;
  *s_out = S;
}

template <int LX, int NW, bool ROUTED>
static void launch_one(dim3 grid, size_t lds, hipStream_t st, const GemvParams& p) {
  static bool attr_done = false;
  if (!attr_done) {  // the input vector and the staged rows can need more than the default 64 KB
    attr_done = true;
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(gemv_f16_kernel<LX, 8, NW, ROUTED>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, AF_GEMV_LDS_BUDGET);
  }
  hipLaunchKernelGGL((gemv_f16_kernel<LX, 8, NW, ROUTED>), grid, dim3(NW * AF_WAVE), lds, st, p);
}

template <int LX>
static void launch_lx(int nw, dim3 grid, size_t lds, hipStream_t st, const GemvParams& p) {
  if (p.router_Wr != nullptr)  // the launcher has made sure of nw == 16
    launch_one<LX, 16, true>(grid, lds, st, p);
  else if (nw == 16)
    launch_one<LX, 16, false>(grid, lds, st, p);
  else if (nw == 8)
    launch_one<LX, 8, false>(grid, lds, st, p);
  else
    launch_one<LX, 4, false>(grid, lds, st, p);
}

int af_launch_gemv_f16(af_ctx* ctx, const af_gemv_args& a) {
  const af_row_src& r = a.rows;
  // the largest index set this launch can meet (the count of a threshold set is only known
  // on the device)
  int max_rows = r.sel == AF_SEL_TOPK ? r.k : (r.sel == AF_SEL_THRESHOLD ? r.n : r.nidx_host);
  int lx, nw, S;
  choose_config(ctx, a.out, max_rows, r.sel != AF_ROWS_GIVEN || r.pro != AF_PRO_NONE, &lx, &nw, &S);
  const int tw = lx * 8;
  // output slots (one per device-selected matrix; a single one otherwise), whole tiles each
  const int n_slots = a.w_sel ? a.n_slots : 1;
  if (n_slots < 1 || a.out % n_slots) return AF_EINVAL;
  const int cols_per_slot = a.out / n_slots;
  if (cols_per_slot % 8) return AF_ESHAPE;
  const int tiles_per_slot = (cols_per_slot + tw - 1) / tw;
  const int tiles = n_slots * tiles_per_slot;
  const int out_pad = tiles * tw;
  if (tiles > AF_TICKET_ATTN) return AF_ESHAPE;
  S = (int)((long long)S * ((a.out + tw - 1) / tw) / tiles);  // padding adds tiles: keep the grid size
  if (S < 1) S = 1;
  const bool range_sel = r.sel == AF_SEL_THRESHOLD && !r.idx_out && !r.count_out;
  const bool use_lds_x = r.pro != AF_PRO_NONE || r.sel != AF_ROWS_GIVEN;
  size_t xs_bytes;
  int list_cap;
  // the split partial sums have to fit the workspace, the staged rows of a split the LDS
  while (S > 1 && (size_t)S * out_pad > ctx->lay.partial_floats) --S;
  if (a.router_Wr && (r.pro != AF_PRO_RMSNORM || a.router_E > 8 || r.n > 8192 || nw != 16 || !use_lds_x))
    return AF_EINVAL;  // the in-kernel router's preconditions (the caller falls back to the router kernel)
  if (!af_plan_gemv_lds(r, max_rows, use_lds_x, range_sel, GEMV_LIST, &S, &xs_bytes, &list_cap,
                        a.router_Wr != nullptr))
    return AF_EWORKSPACE;
  if (S > 1 && (size_t)S * out_pad > ctx->lay.partial_floats) return AF_EWORKSPACE;
  GemvParams p;
  p.W = (const half_t*)a.W;
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
  p.w_stride = a.w_stride;
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
    launch_lx<64>(nw, grid, lds, ctx->stream, p);
  else if (lx == 32)
    launch_lx<32>(nw, grid, lds, ctx->stream, p);
  else
    launch_lx<16>(nw, grid, lds, ctx->stream, p);
  AF_LAUNCH_CHECK();
  return AF_OK;
}

// Argument checks of af_sparse_gemv_f16 (nothing is launched), and the launch itself.
static int sparse_gemv_f16_check(const af_ctx* ctx, const void* Wt, int in, int out, int ld,
                                 const void* x_f16, const int32_t* idx, int* nidx_host,
                                 const int32_t** nidx_dev, const void* y, int y_kind) {
  if (!ctx || !Wt || !x_f16 || !y) return AF_ENULL;
  if (in <= 0 || out <= 0 || in > AF_MAX_N) return AF_EINVAL;
  if (out % 8 || ld % 8 || ld < out) return AF_ESHAPE;
  if (y_kind != AF_F16 && y_kind != AF_F32) return AF_EINVAL;
  if (idx == nullptr) {
    *nidx_host = in;
    *nidx_dev = nullptr;
  }
  if (*nidx_host < 0 || *nidx_host > in) return AF_EINVAL;
  if (!ctx->ws) return AF_EWORKSPACE;
  if (in > ctx->max_in || out > ctx->max_out) return AF_EWORKSPACE;
  return AF_OK;
}

static int sparse_gemv_f16_launch(af_ctx* ctx, const void* Wt, int in, int out, int ld,
                                  const void* x_f16, const int32_t* idx, int nidx_host,
                                  const int32_t* nidx_dev, void* y, int y_kind,
                                  const void* residual_f16) {
  af_gemv_args a{};
  a.W = Wt;
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
  return af_launch_gemv_f16(ctx, a);
}

extern "C" int af_sparse_gemv_f16(af_ctx* ctx, const void* Wt, int in, int out, int ld,
                                  const void* x_f16, const int32_t* idx, int nidx_host,
                                  const int32_t* nidx_dev, void* y, int y_kind,
                                  const void* residual_f16) {
  const int rc = sparse_gemv_f16_check(ctx, Wt, in, out, ld, x_f16, idx, &nidx_host, &nidx_dev, y, y_kind);
  if (rc) return rc;
  return sparse_gemv_f16_launch(ctx, Wt, in, out, ld, x_f16, idx, nidx_host, nidx_dev, y, y_kind,
                                residual_f16);
}

// ---- the same operation for callers that cannot allocate ---------------------------------
// The tickets and split partials live in a device array of the library image instead of the
// caller's workspace.  Every GPU that loads the library holds its own copy of the array at its
// own address; the name below is only the host-side handle of the symbol, the address comes
// from hipGetSymbolAddress once per device.
#define AF_NOALLOC_PARTIAL_FLOATS (1u << 20)
#define AF_NOALLOC_BYTES (sizeof(int) * AF_N_TICKETS + sizeof(float) * AF_NOALLOC_PARTIAL_FLOATS)
#define AF_NOALLOC_MAX_DEVICES 64
static __device__ __align__(256) unsigned char scratch[AF_NOALLOC_BYTES];
static void* g_scratch_ptr[AF_NOALLOC_MAX_DEVICES];  // per device, filled on first use

__global__ void noalloc_clear_kernel(int* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

extern "C" int af_sparse_gemv_f16_noalloc(af_ctx* ctx, const void* Wt, int in, int out, int ld,
                                          const void* x_f16, const int32_t* idx, int nidx_host,
                                          const int32_t* nidx_dev, void* y, int y_kind,
                                          const void* residual_f16) {
  if (!ctx) return AF_ENULL;
  if (out > AF_NOALLOC_MAX_OUT) return AF_ENOALLOC_LIMIT;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return AF_EHIP;
  if (dev != ctx->device || dev < 0 || dev >= AF_NOALLOC_MAX_DEVICES) return AF_EINVAL;
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return AF_EHIP;
    g_scratch_ptr[dev] = ptr;
  }
  char* base = (char*)g_scratch_ptr[dev];
  // a shallow copy of the context whose scratch is the device array: same stream, same device
  af_ctx local = *ctx;
  local.ws = base;
  local.ws_bytes = AF_NOALLOC_BYTES;
  local.max_in = AF_MAX_N;
  local.max_out = AF_NOALLOC_MAX_OUT;
  local.max_batch = 1;
  local.lay = af_ws_layout{};
  local.lay.tickets = 0;
  local.lay.partials = sizeof(int) * AF_N_TICKETS;
  local.lay.partial_floats = AF_NOALLOC_PARTIAL_FLOATS;
  local.lay.total = AF_NOALLOC_BYTES;
  const int rc = sparse_gemv_f16_check(&local, Wt, in, out, ld, x_f16, idx, &nidx_host, &nidx_dev, y, y_kind);
  if (rc) return rc;
  // The array keeps what the last call left.  A completed call leaves its tickets at zero, but
  // a call that was cut short does not, so the tickets are cleared in front of every launch
  // (a fill kernel, not a memset node: the call may be under stream capture).
  hipLaunchKernelGGL(noalloc_clear_kernel, dim3(AF_TICKET_ATTN / 256), dim3(256), 0, ctx->stream,
                     (int*)base, (int)AF_TICKET_ATTN);
  AF_LAUNCH_CHECK();
  return sparse_gemv_f16_launch(&local, Wt, in, out, ld, x_f16, idx, nidx_host, nidx_dev, y,
                                y_kind, residual_f16);
}

static int select_gemv_any(af_ctx* ctx, const int32_t* expert_sel, int n_slots,
                           long long expert_stride, const float* y_scale, const void* Wt, int in,
                           int out, int ld, int producer,
                                  const void* src_f16, const void* gain_f16, float eps,
                                  int sel_mode, int k, float t, void* x_out, int32_t* idx_out,
                                  int32_t* count_out, void* y, int y_kind,
                                  const void* residual_f16) {
  if (!ctx || !Wt || !src_f16 || !y) return AF_ENULL;
  if (producer != AF_PRO_NONE && producer != AF_PRO_RMSNORM && producer != AF_PRO_SILUMUL)
    return AF_EINVAL;
  if (producer == AF_PRO_RMSNORM && !gain_f16) return AF_ENULL;
  if (in <= 0 || out <= 0 || in > AF_MAX_N) return AF_EINVAL;
  if (expert_sel && (n_slots < 1 || out % n_slots)) return AF_EINVAL;
  const int cols = expert_sel ? out / n_slots : out;  // columns of one matrix
  if (in % 8 || cols % 8 || ld % 8 || ld < cols) return AF_ESHAPE;
  if (y_kind != AF_F16 && y_kind != AF_F32) return AF_EINVAL;
  if (sel_mode != AF_SEL_TOPK && sel_mode != AF_SEL_THRESHOLD && sel_mode != AF_SEL_DENSE)
    return AF_EINVAL;
  if (sel_mode == AF_SEL_TOPK && (k < 0 || k > in)) return AF_EINVAL;
  if (sel_mode == AF_SEL_THRESHOLD && t != t) return AF_EINVAL;
  if (!ctx->ws) return AF_EWORKSPACE;
  if (in > ctx->max_in || out > ctx->max_out) return AF_EWORKSPACE;
  af_gemv_args a{};
  a.W = Wt;
  a.in = in;
  a.out = out;
  a.ld = ld;
  a.rows.pro = producer;
  a.rows.src = (const half_t*)src_f16;
  a.rows.gain = (const half_t*)gain_f16;
  a.rows.eps = eps;
  a.rows.x_out = (half_t*)x_out;
  a.rows.n = in;
  if (sel_mode == AF_SEL_DENSE) {
    a.rows.sel = AF_ROWS_GIVEN;
    a.rows.idx = nullptr;
    a.rows.nidx_host = in;
  } else {
    a.rows.sel = sel_mode;
    a.rows.k = k;
    a.rows.t = t;
    a.rows.idx_out = idx_out;
    a.rows.count_out = count_out;
  }
  a.y = y;
  a.y_kind = y_kind;
  a.residual = (const half_t*)residual_f16;
  a.w_sel = expert_sel;
  a.n_slots = n_slots;
  a.w_stride = expert_stride;
  a.y_scale = y_scale;
  return af_launch_gemv_f16(ctx, a);
}

extern "C" int af_select_gemv_f16(af_ctx* ctx, const void* Wt, int in, int out, int ld, int producer,
                                  const void* src_f16, const void* gain_f16, float eps,
                                  int sel_mode, int k, float t, void* x_out, int32_t* idx_out,
                                  int32_t* count_out, void* y, int y_kind,
                                  const void* residual_f16) {
  return select_gemv_any(ctx, nullptr, 1, 0, nullptr, Wt, in, out, ld, producer, src_f16, gain_f16,
                         eps, sel_mode, k, t, x_out, idx_out, count_out, y, y_kind, residual_f16);
}

extern "C" int af_select_gemv_experts_f16(af_ctx* ctx, const void* Wt_all, const int32_t* expert_sel,
                                          int n_slots, long long expert_stride, const float* y_scale,
                                          int in, int out, int ld, int producer, const void* src_f16,
                                          const void* gain_f16, float eps, int sel_mode, int k,
                                          float t, void* x_out, int32_t* idx_out, int32_t* count_out,
                                          void* y, int y_kind, const void* residual_f16) {
  if (!expert_sel) return AF_ENULL;
  if (expert_stride < 0) return AF_EINVAL;
  return select_gemv_any(ctx, expert_sel, n_slots, expert_stride, y_scale, Wt_all, in, out, ld,
                         producer, src_f16, gain_f16, eps, sel_mode, k, t, x_out, idx_out, count_out,
                         y, y_kind, residual_f16);
}
