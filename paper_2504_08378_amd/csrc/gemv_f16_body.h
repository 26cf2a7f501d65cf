// Body of the gathered-row sparse GEMV over an input-channel-major fp16 matrix (Section 4,
// operation C), shared by the stand-alone kernel (gemv_f16.hip) and the whole-layer kernel
// (layer.hip).  See gemv_f16.hip for the decomposition.
#pragma once
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
  // The argument block stays within 248 bytes: launches of this kernel were measured 0.3-0.4 us
  // slower once it grew to 280 bytes (the launch itself does not care: near-empty kernels take
  // the same time with 16 bytes or 1 KB of arguments; the cost was in this kernel's start-up).
  // Hence the flag word.
  int out, ld, out_pad;
  int flags;  // GEMV_F_*
  int list_off;   // byte offset of the staged-row list in dynamic LDS (behind x)
  // Output columns come in `slots` of cols_per_slot columns, each covered by tiles_per_slot
  // tiles.  A plain GEMV has one slot.  With w_sel, slot s multiplies by the matrix
  // W + w_sel[s] * w_stride (leading dimension ld), so the experts a router picked on the
  // device are reached without a host round trip.  y_scale (device, one float) scales the
  // product before the residual is added.
  int cols_per_slot, tiles_per_slot;
  int done_total;  // see `done` below
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
  // Whole-layer kernel only (null otherwise): the operator is one phase of a kernel whose
  // workgroups go on to the next operator.  Results are then stored through to memory (agent
  // scope) and every workgroup that has finished a tile adds one to *done; the workgroup that
  // brings it to done_total clears *done_prev, the counter of the phase before (all of its
  // waiters have passed it by then).
  // GEMV_F_DONE_PREV: the counter of the phase before is done[-1]; GEMV_F_DONE_LAST: the
  // kernel's last phase, nobody waits on *done and it is cleared as well.
  int* done;
  __host__ __device__ bool f32_out() const { return flags & 1; }
  __host__ __device__ bool use_lds_x() const { return flags & 2; }
  __host__ __device__ bool range_sel() const { return flags & 4; }
};
enum { GEMV_F_F32 = 1, GEMV_F_LDS_X = 2, GEMV_F_RANGE_SEL = 4, GEMV_F_DONE_PREV = 8, GEMV_F_DONE_LAST = 16 };
static_assert(sizeof(GemvParams) <= 248, "keep the kernel argument block small (see above)");

// One finished tile of a whole-layer phase: the results are acknowledged, then counted.
__device__ __forceinline__ void gemv_phase_signal(const GemvParams& p) {
  af_stores_done();
  __syncthreads();
  if (threadIdx.x == 0) {
    const int old = __hip_atomic_fetch_add(p.done, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old == p.done_total - 1) {
      if (p.flags & GEMV_F_DONE_PREV) __hip_atomic_store(p.done - 1, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (p.flags & GEMV_F_DONE_LAST) __hip_atomic_store(p.done, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

// Whole-layer kernel: the finished tile is read by other workgroups of the same launch, so it
// is written through to memory (agent scope).  Two-byte write-through stores would each cost a
// read-modify-write in the memory controller; the tile is therefore put together in LDS
// (`stage`, free at this point) and leaves as 8-byte stores of neighbouring lanes.
// valid % 8 == 0, (y + out0) 8-byte aligned.  v_of(c) yields the sum of column c.
template <int THREADS, typename F>
__device__ __forceinline__ void store_tile_through(const GemvParams& p, int out0, int valid,
                                                   unsigned short* stage, F v_of) {
  const float scale = p.y_scale ? *p.y_scale : 1.0f;
  if (!p.f32_out()) {
    for (int c = threadIdx.x; c < valid; c += THREADS) {
      float v = v_of(c) * scale;
      if (p.residual) v += (float)p.residual[out0 + c];
      stage[c] = __builtin_bit_cast(unsigned short, (half_t)v);
    }
    __syncthreads();
    unsigned long long* dst = reinterpret_cast<unsigned long long*>(reinterpret_cast<half_t*>(p.y) + out0);
    const unsigned long long* src = reinterpret_cast<const unsigned long long*>(stage);
    for (int q = threadIdx.x; q < (valid >> 2); q += THREADS)
      __hip_atomic_store(dst + q, src[q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  } else {
    for (int c = threadIdx.x; c < valid; c += THREADS) {
      float v = v_of(c) * scale;
      if (p.residual) v += (float)p.residual[out0 + c];
      af_store_agent(reinterpret_cast<float*>(p.y) + out0 + c, v);
    }
  }
}

__device__ __forceinline__ void store_out(const GemvParams& p, int col, float v) {
  if (p.y_scale) v *= *p.y_scale;
  if (p.residual) v += (float)p.residual[col];
  if (!p.f32_out())
    reinterpret_cast<half_t*>(p.y)[col] = (half_t)v;
  else
    reinterpret_cast<float*>(p.y)[col] = v;
}

// Launch shape and parameters of one fp16 GEMV as the host plans it: tiles x S workgroups of
// nw waves, lx lanes across a tile, `lds` bytes of dynamic LDS.
struct GemvPlan {
  GemvParams p;
  int tiles, S, lx, nw;
  size_t lds;
};
// whole_layer: the operator runs as a phase of the whole-layer kernel (1024-thread workgroups,
// at most one per compute unit).  Defined in gemv_f16.hip.
int af_plan_gemv_f16(af_ctx* ctx, const af_gemv_args& a, bool whole_layer, GemvPlan* plan);

// Virtual launch position of a workgroup: the stand-alone kernel passes blockIdx / gridDim, the
// whole-layer kernel the position it has given the workgroup in the current operator.
struct GemvPos {
  int bx, by, gx, gy;
};
// LDS of one workgroup that the GEMV bodies need besides the dynamic region: declared once by
// the kernel and shared by all the operators it runs.
template <int NW, int TWMAX = 512>
struct GemvLds {
  static constexpr int SCRATCH = RP_SCRATCH_WORDS > NW * TWMAX ? RP_SCRATCH_WORDS : NW * TWMAX;
  __align__(16) unsigned scratch[SCRATCH];  // histograms, later the wave sums
  typename RowPrologue<NW * AF_WAVE>::Smem rp;
  int last;
};

// PHASE: the operator is a phase of the whole-layer kernel (p.done is set).
template <int LX, int U, int NW, bool ROUTED, bool PHASE, typename LDS_T>
__device__ __forceinline__ void gemv_f16_body(const GemvParams& p, const GemvPos vb,
                                              unsigned short* xs, LDS_T& lds) {
  constexpr int GEMV_THREADS = NW * AF_WAVE;
  constexpr int GEMV_WAVES = NW;
  constexpr int LY = AF_WAVE / LX;
  constexpr int TW = LX * 8;
  constexpr int STEP = GEMV_WAVES * LY;  // rows taken per workgroup iteration
  typedef RowPrologue<GEMV_THREADS> RP;
  unsigned* s_scratch = lds.scratch;
  typename RP::Smem& s_rp = lds.rp;
  int& s_last = lds.last;
  float(*s_red)[TW] = reinterpret_cast<float(*)[TW]>(s_scratch);
  // staged rows, (index << 16 | fp16 bits of x)
  unsigned* s_list = reinterpret_cast<unsigned*>(reinterpret_cast<char*>(xs) + p.list_off);

  af_prof_begin(p.prof);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lx = lane % LX, ly = lane / LX;
  // one slot (a plain GEMV): no division
  const int slot = p.tiles_per_slot >= vb.gx ? 0 : vb.bx / p.tiles_per_slot;
  const int tile_in = vb.bx - slot * p.tiles_per_slot;   // tile inside the slot
  const int col = tile_in * TW + lx * 8;                       // column inside the slot
  // lanes past the slot's edge read the tile's first column and are dropped at the store
  const int col_ld = col < p.cols_per_slot ? col : tile_in * TW;
  const int S = vb.gy, s = vb.by;
  const af_row_src& r = p.rows;

  // Rows given and their number known on the host: fetch this thread's share of the first
  // staging pass now, so that the index round trip overlaps the construction of x.
  constexpr int PF = GEMV_LIST / GEMV_THREADS;
  int pre[PF];
  const bool prefetched = r.sel == AF_ROWS_GIVEN && r.idx != nullptr && r.nidx_dev == nullptr;
  if (prefetched) {
    const int R = af_ceil_div_small(r.nidx_host, S);
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
  if (p.use_lds_x() && (!p.range_sel() || routed))
    RP::produce(r, xs, s_rp, s == 0, vb.bx, vb.gx,
                r.sel == AF_SEL_TOPK ? s_scratch : nullptr);
  if constexpr (routed) {
    RP::template router_in_lds<RE>(xs, r.n, s_rp, wr, p.router_E, p.router_top);
    if (vb.bx == 0 && s == 0) {
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
        w[u] = af_load_once(reinterpret_cast<const half8*>(wcol + (size_t)(e[u] >> 16) * p.ld));
      }
      // All U loads are issued before the first product: without this fence the instruction
      // scheduler has, in some instantiations, paired every load with its own wait (one row in
      // flight instead of U), which halves the streaming rate.
      __builtin_amdgcn_sched_barrier(0);
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
          w[u] = af_load_once(reinterpret_cast<const half8*>(wcol + (size_t)(e[u] >> 16) * p.ld));
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

  if (p.range_sel()) {
    stream(routed ? RP::threshold_range_of_full(r, xs, s_rp, s_list, S, s)
                  : RP::threshold_range(r, xs, s_rp, s_list, S, s, vb.bx == 0));
  } else if (r.sel != AF_ROWS_GIVEN) {
    int nidx_total;
    const int cnt = RP::select_split(r, xs, s_scratch, s_rp, s_list, S, s, vb.bx == 0,
                                     vb.bx == 0 && s == 0, &nidx_total, p.use_lds_x());
    stream(cnt);
  } else {
    int nidx = r.nidx_host;
    if (r.nidx_dev) nidx = min(*r.nidx_dev, nidx);
    const int R = af_ceil_div_small(nidx, S);
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
            if ((unsigned)j < (unsigned)r.n) {
              const unsigned bits = p.use_lds_x() ? xs[j] : xg[j];
              s_list[i] = ((unsigned)j << 16) | bits;
            } else {  // broken precondition: row 0 times zero, and the error word
              s_list[i] = 0u;
              af_report_bad_index(p.tickets);
            }
          }
        }
      } else {
        for (int i = tid; i < cnt; i += GEMV_THREADS) {
          const int j = r.idx ? r.idx[base + i] : base + i;
          if ((unsigned)j < (unsigned)r.n) {
            const unsigned bits = p.use_lds_x() ? xs[j] : xg[j];
            s_list[i] = ((unsigned)j << 16) | bits;
          } else {
            s_list[i] = 0u;
            af_report_bad_index(p.tickets);
          }
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

  const int tile0 = vb.bx * TW;                      // in the padded column space
  const int out0 = slot * p.cols_per_slot + tile_in * TW;  // first output column of the tile
  const int valid = min(TW, p.cols_per_slot - tile_in * TW);
  if (S == 1) {
    if constexpr (PHASE) {
      store_tile_through<GEMV_THREADS>(p, out0, valid, xs, [&](int c) {
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < GEMV_WAVES; ++w) v += s_red[w][c];
        return v;
      });
      gemv_phase_signal(p);
    } else {
      for (int c = tid; c < valid; c += GEMV_THREADS) {
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < GEMV_WAVES; ++w) v += s_red[w][c];
        store_out(p, out0 + c, v);
      }
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
    int old = af_ticket_take(&p.tickets[vb.bx]);
    s_last = (old == S - 1);
  }
  __syncthreads();
  if (!s_last) {
    af_prof_end(p.prof);
    return;
  }
  if constexpr (PHASE) {
    store_tile_through<GEMV_THREADS>(p, out0, valid, xs, [&](int c) {
      return af_sum_partials(p.partials + tile0 + c, p.out_pad, S);
    });
  } else {
    for (int c = tid; c < valid; c += GEMV_THREADS)
      store_out(p, out0 + c, af_sum_partials(p.partials + tile0 + c, p.out_pad, S));
  }
  if (tid == 0) af_ticket_reset(&p.tickets[vb.bx]);  // ready for the next launch
  if constexpr (PHASE) gemv_phase_signal(p);
  af_prof_end(p.prof);
}

// GEMV_MODE(pro, kind): the producer and the way the rows are found as compile-time constants
// (kind: 0 rows given, 1 top-k, 2 threshold with an index list, 3 threshold per channel range).
// A kernel instantiated for one mode carries none of the other modes' code and branches, which
// measured 0.4-0.5 us per launch (q|k|v 16.7 -> 16.3 us, gate|up 23.5 -> 23.0 us); mode -1 is
// the generic kernel that reads both from its arguments.
#define GEMV_MODE(pro, kind) ((pro) | ((kind) << 2))
template <int MODE>
__device__ __forceinline__ GemvParams gemv_fix_mode(const GemvParams& p) {
  GemvParams q = p;
  if constexpr (MODE >= 0) {
    constexpr int pro = MODE & 3, kind = MODE >> 2;
    q.rows.pro = pro;
    q.rows.sel = kind == 0 ? (int)AF_ROWS_GIVEN : (kind == 1 ? (int)AF_SEL_TOPK : (int)AF_SEL_THRESHOLD);
    q.flags = (p.flags & ~(GEMV_F_LDS_X | GEMV_F_RANGE_SEL)) |
              ((pro != AF_PRO_NONE || kind != 0) ? GEMV_F_LDS_X : 0) | (kind == 3 ? GEMV_F_RANGE_SEL : 0);
  }
  return q;
}
// The mode the generic kernel would find in these arguments.
static inline int gemv_mode_of(const GemvParams& p) {
  const int kind = p.rows.sel == AF_ROWS_GIVEN ? 0 : (p.rows.sel == AF_SEL_TOPK ? 1 : (p.range_sel() ? 3 : 2));
  return GEMV_MODE(p.rows.pro, kind);
}

// ROUTED: the instantiation that runs a mixture-of-experts router in its front end (kept apart
// so that the plain launches do not carry its registers).
template <int LX, int U, int NW, bool ROUTED, int MODE = -1>
__global__ __launch_bounds__(NW * AF_WAVE) void gemv_f16_kernel(GemvParams p) {
  extern __shared__ __align__(16) unsigned short xs[];  // the operator input, when built here
  __shared__ GemvLds<NW, LX * 8> lds;
  const GemvPos vb = {(int)blockIdx.x, (int)blockIdx.y, (int)gridDim.x, (int)gridDim.y};
  if constexpr (MODE >= 0) {
    const GemvParams q = gemv_fix_mode<MODE>(p);
    gemv_f16_body<LX, U, NW, ROUTED, false>(q, vb, xs, lds);
  } else {
    gemv_f16_body<LX, U, NW, ROUTED, false>(p, vb, xs, lds);
  }
}
