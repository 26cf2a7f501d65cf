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
#include "gemv_f16_body.h"

// Tile width, waves per workgroup and split count for a shape.  The AF_OPT_TUNE_* options of
// the context override the heuristic (tuning sweeps).
static void choose_config(const af_ctx* ctx, int out, int nidx, bool selects, bool whole_layer,
                          int* lx_out, int* nw_out, int* s_out) {
  // A kernel that selects for itself (or builds its input vector) repeats that work in every
  // workgroup, so it runs few, large workgroups (one 1024-thread workgroup per CU); a plain
  // GEMV prefers several small ones per CU.
  //
  // Selecting launches, measured over the q|k|v, o, gate|up and down operators of the 7B, 13B
  // and 70B shapes with cold matrices and non-temporal row loads:
  //  * tile width: 128 columns up to ~6K output columns, 256 up to ~12K, 512 beyond (within
  //    1-2 % of the best of the three for every operator);
  //  * splits: between three quarters of the CUs and all of them, the most that leave every
  //    workgroup 320 rows (128-column tiles) or 500 rows (wider tiles); below that a workgroup
  //    is mostly front end and reduction.  13B: o 13.1 against 14.6 us, gate|up 31.0 against
  //    33.5 us, down 24.4 against 26.4 us for 240 against 160 workgroups; 70B down 54.9 against
  //    58.9 us; Mixtral gate|up of two experts 43 against 53 us (224 against 112 workgroups);
  //    7B o: 11.7 us with 6 splits, 12.1 with 8; 7B gate|up inside the stack: 21.8 us with 4
  //    splits, 22.2 with 5.
  // Plain launches: 128-column tiles up to 16K columns and 512 beyond; with 256-column tiles on
  // a row stride that is a multiple of 1 KB every workgroup stays on one value of address bit 9
  // for all its rows, and the half of the workgroups on one of the two values finished ~2 us
  // after the other half.
  int lx = out <= 16384 ? 16 : 64;
  int nw = selects ? 16 : 4;
  if (selects && !whole_layer) lx = out <= 6144 ? 16 : (out <= 12288 ? 32 : 64);
  if (selects && whole_layer && out > 8192 && out <= 16384) lx = 32;  // the shapes that kernel is built for
  if (ctx->tune_lx == 16 || ctx->tune_lx == 32 || ctx->tune_lx == 64) lx = ctx->tune_lx;
  if (ctx->tune_nw == 4 || ctx->tune_nw == 8 || ctx->tune_nw == 16) nw = ctx->tune_nw;
  const int per_cu = 16 / nw;  // workgroups of nw waves that one CU holds at a time
  int target_wgs = nw == 4 ? (out <= 4096 ? ctx->n_cu : ctx->n_cu * 4) : ctx->n_cu * per_cu;
  if (nw == 16 && selects && whole_layer) target_wgs = ctx->n_cu * 3 / 4;
  if (ctx->tune_wgs > 0) target_wgs = ctx->tune_wgs;
  const int tiles = (out + lx * 8 - 1) / (lx * 8);
  int S = target_wgs / tiles;  // never more workgroups than the chip holds at once
  if (nw == 16 && selects && !whole_layer && ctx->tune_wgs <= 0) {
    int s_min = ctx->n_cu * 3 / 4 / tiles;
    if (s_min < 1) s_min = 1;
    if (tiles * s_min < ctx->n_cu * 6 / 10 && tiles * (s_min + 1) <= ctx->n_cu) ++s_min;
    const int rows_min = lx == 16 ? 320 : 500;
    while (S > s_min && nidx / S < rows_min) --S;
    if (S < s_min) S = s_min;
  }
  if (ctx->tune_split > 0) S = ctx->tune_split;
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

template <int LX, int NW, bool ROUTED, int MODE>
static void launch_one(dim3 grid, size_t lds, hipStream_t st, const GemvParams& p) {
  static bool attr_done = false;
  if (!attr_done) {  // the input vector and the staged rows can need more than the default 64 KB
    attr_done = true;
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(gemv_f16_kernel<LX, 8, NW, ROUTED, MODE>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, AF_GEMV_LDS_BUDGET);
  }
  hipLaunchKernelGGL((gemv_f16_kernel<LX, 8, NW, ROUTED, MODE>), grid, dim3(NW * AF_WAVE), lds, st, p);
}

// The 1024-thread launches that build or select their input come in one instantiation per
// (producer, selection) pair of a decoder layer; anything else runs the generic kernel.
template <int LX>
static void launch_lx(int nw, dim3 grid, size_t lds, hipStream_t st, const GemvParams& p) {
  if (p.router_Wr != nullptr) {  // the launcher has made sure of nw == 16 and of an RMSNorm producer
    const int mode = gemv_mode_of(p);
    if (mode == GEMV_MODE(AF_PRO_RMSNORM, 1))
      launch_one<LX, 16, true, GEMV_MODE(AF_PRO_RMSNORM, 1)>(grid, lds, st, p);
    else if (mode == GEMV_MODE(AF_PRO_RMSNORM, 3))
      launch_one<LX, 16, true, GEMV_MODE(AF_PRO_RMSNORM, 3)>(grid, lds, st, p);
    else
      launch_one<LX, 16, true, -1>(grid, lds, st, p);
  } else if (nw == 16) {
    switch (gemv_mode_of(p)) {
#define AF_MODE_CASE(pro, kind) \
  case GEMV_MODE(pro, kind):    \
    launch_one<LX, 16, false, GEMV_MODE(pro, kind)>(grid, lds, st, p); \
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
        launch_one<LX, 16, false, -1>(grid, lds, st, p);
    }
  } else if (nw == 8) {
    launch_one<LX, 8, false, -1>(grid, lds, st, p);
  } else {
    launch_one<LX, 4, false, -1>(grid, lds, st, p);
  }
}

int af_plan_gemv_f16(af_ctx* ctx, const af_gemv_args& a, bool whole_layer, GemvPlan* plan) {
  const af_row_src& r = a.rows;
  // the largest index set this launch can meet (the count of a threshold set is only known
  // on the device)
  int max_rows = r.sel == AF_SEL_TOPK ? r.k : (r.sel == AF_SEL_THRESHOLD ? r.n : r.nidx_host);
  int lx, nw, S;
  // inside the whole-layer kernel every operator runs on the kernel's 1024-thread workgroups,
  // one per compute unit
  // a threshold keeps an unknown number of rows: plan the launch for half of them
  choose_config(ctx, a.out, r.sel == AF_SEL_THRESHOLD ? (r.n + 1) / 2 : max_rows,
                whole_layer || r.sel != AF_ROWS_GIVEN || r.pro != AF_PRO_NONE, whole_layer, &lx, &nw, &S);
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
  GemvParams& p = plan->p;
  p = GemvParams{};
  p.W = (const half_t*)a.W;
  p.rows = r;
  p.partials = (float*)(ctx->ws + ctx->lay.partials);
  p.tickets = (int*)(ctx->ws + ctx->lay.tickets);
  p.y = a.y;
  p.residual = a.residual;
  p.out = a.out;
  p.ld = a.ld;
  p.out_pad = out_pad;
  p.flags = (a.y_kind == AF_F32 ? GEMV_F_F32 : 0) | (use_lds_x ? GEMV_F_LDS_X : 0) |
            (range_sel ? GEMV_F_RANGE_SEL : 0);
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
  plan->tiles = tiles;
  plan->S = S;
  plan->lx = lx;
  plan->nw = nw;
  plan->lds = xs_bytes + (size_t)list_cap * 4;
  return AF_OK;
}

int af_launch_gemv_f16(af_ctx* ctx, const af_gemv_args& a) {
  GemvPlan plan;
  const int rc = af_plan_gemv_f16(ctx, a, false, &plan);
  if (rc) return rc;
  plan.p.prof = af_prof_take(ctx);
  dim3 grid(plan.tiles, plan.S);
  if (plan.lx == 64)
    launch_lx<64>(plan.nw, grid, plan.lds, ctx->stream, plan.p);
  else if (plan.lx == 32)
    launch_lx<32>(plan.nw, grid, plan.lds, ctx->stream, plan.p);
  else
    launch_lx<16>(plan.nw, grid, plan.lds, ctx->stream, plan.p);
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
  int rc = sparse_gemv_f16_check(ctx, Wt, in, out, ld, x_f16, idx, &nidx_host, &nidx_dev, y, y_kind);
  if (rc) return rc;
  if (ctx->validate && (rc = af_validate_idx(ctx, idx, nidx_host, nidx_dev, in))) return rc;
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
