// Internal declarations shared by the library's translation units (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "activeflow.h"

typedef _Float16 half_t;
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));

#define AF_WAVE 64

// Workspace carve-up (byte offsets from the caller's buffer), fixed by the limits given to
// af_set_workspace.
struct af_ws_layout {
  size_t tickets;       // int32[AF_N_TICKETS], zero between kernels
  size_t partials;      // float[partial_floats]: split partial sums of the GEMVs
  size_t attn_part;     // float[attn_floats]: per-(head, key split) softmax partials
  size_t act[7];        // fp16 inter-operator tensors of a layer, [max_batch] rows each (see af_layer_tap)
  size_t union_x;       // fp16 [max_in][8]: masked, transposed token values of the union GEMV
  size_t union_idx;     // int32 [max_in]: union of the tokens' sets (af_decode_layer_batch)
  size_t union_n;       // int32 [4]: its size per selection point
  size_t union_ranges;  // int32 [max_in rounded up to 256]: the union builder's per-range lists
  size_t union_range_cnt; // int32 [AF_MAX_N / 256]
  size_t union_mask;    // uint32 [max_in]: per-channel token bits of the union builder, zero between calls
  size_t total;
  size_t partial_floats;
  size_t attn_floats;
};
enum {
  AF_N_TICKETS = 8192,
  AF_TICKET_ATTN = 4096,  // first ticket used by attention
  AF_TICKET_PHASE = 8160, // five phase counters of the whole-layer kernel
  AF_TICKET_ERR = 8176    // device error word (af_last_device_error)
};


af_ws_layout af_layout(int max_in, int max_out, int max_batch);

struct af_ctx {
  int device;
  hipStream_t stream;
  char* ws;
  size_t ws_bytes;
  int max_in, max_out, max_batch;
  af_ws_layout lay;
  int n_cu;
  // af_profile_set: device stamps [2 * prof_slots], next slot to hand to a layer kernel
  long long* prof;
  int prof_slots, prof_next;
  int use_layer_kernel;   // af_set_option(AF_OPT_LAYER_KERNEL, 1): one launch per layer
  int validate;           // af_set_option(AF_OPT_VALIDATE, 1): check caller index lists on the device
  // launch-shape overrides for tuning sweeps (af_set_option; 0 = the built-in heuristic)
  int tune_lx, tune_nw, tune_split, tune_wgs, moe_router_kernel, tune_attn_splits;
  int layer_kernel_state; // 0 not probed yet, 1 usable, -1 not usable on this device
};

// Slot of the next layer kernel's time stamps (null: profiling off or slots used up).
static inline long long* af_prof_take(af_ctx* ctx) {
  if (!ctx->prof || ctx->prof_next >= ctx->prof_slots) return nullptr;
  return ctx->prof + 2 * (size_t)(ctx->prof_next++);
}

struct af_graph {
  hipGraph_t graph;
  hipGraphExec_t exec;
};

static inline int af_hip(hipError_t e) { return e == hipSuccess ? AF_OK : AF_EHIP; }
#define AF_LAUNCH_CHECK()                          \
  do {                                             \
    if (hipGetLastError() != hipSuccess) return AF_EHIP; \
  } while (0)

// ---- internal launchers (host) -----------------------------------------------------------
enum { AF_ROWS_GIVEN = 3 };  // rows come from memory (idx list) or are all channels (dense)

// Where a fused GEMV gets its input vector and its rows from (see row_prologue.h).
struct af_row_src {
  int pro;              // AF_PRO_NONE | AF_PRO_RMSNORM | AF_PRO_SILUMUL
  const half_t* src;    // NONE: x[n]; RMSNORM: hidden[n]; SILUMUL: gate|up [2n]
  const half_t* gain;   // RMSNORM
  float eps;
  half_t* x_out;        // produced x is also stored here (null: not stored)
  int n;
  int sel;              // AF_SEL_TOPK | AF_SEL_THRESHOLD | AF_ROWS_GIVEN
  int k;
  float t;
  const int32_t* idx;   // AF_ROWS_GIVEN: list (null = dense)
  int nidx_host;
  const int32_t* nidx_dev;
  int32_t* idx_out;     // selection result (null: not stored)
  int32_t* count_out;
};

// Dynamic LDS of a fused GEMV workgroup: [x as fp16 | staged rows as uint32].  A workgroup that
// selects keeps its whole share of the rows staged, so the share has to fit: *S (the number
// of row splits) is raised until it does.  Rows given by the caller are staged `chunk` at a
// time instead.  Returns false if nothing fits.
#define AF_GEMV_LDS_BUDGET (120u * 1024u)  // leaves room for the kernels' static LDS in 160 KB
static inline bool af_plan_gemv_lds(const af_row_src& r, int max_rows, bool use_lds_x,
                                    bool range_sel, int chunk, int* S, size_t* xs_bytes,
                                    int* list_cap, bool full_x = false) {
  for (int s = *S < 1 ? 1 : *S; s <= 4096; ++s) {
    size_t xb;
    int cap;
    if (range_sel) {
      cap = 8 * ((r.n / 8 + s - 1) / s);  // a channel range, whole 8-element vectors
      xb = full_x ? (size_t)r.n * 2 : (size_t)cap * 2;  // an in-kernel router wants all of x
    } else if (r.sel != AF_ROWS_GIVEN) {
      cap = (max_rows + s - 1) / s;
      xb = (size_t)r.n * 2;
    } else {
      cap = chunk;
      xb = use_lds_x ? (size_t)r.n * 2 : 0;
    }
    xb = (xb + 15) / 16 * 16;
    if (cap < 64) cap = 64;
    if (xb + (size_t)cap * 4 <= AF_GEMV_LDS_BUDGET) {
      *S = s;
      *xs_bytes = xb;
      *list_cap = cap;
      return true;
    }
    if (r.sel == AF_ROWS_GIVEN) return false;
  }
  return false;
}

struct af_gemv_args {
  const void* W;          // fp16 in-major, or packed nibbles
  const half_t* scales;   // q4 only
  bool q4_channel_local;  // q4: scales [in][ld/32] instead of [in/32][ld]
  int in, out, ld;
  af_row_src rows;
  void* y;
  int y_kind;
  const half_t* residual;
  // Device-selected matrices (mixture of experts): the out columns form n_slots equal slots;
  // slot s uses the matrix at W + w_sel[s] * w_stride elements (leading dimension ld), w_sel
  // being device memory.  w_sel == null: one matrix, one slot.
  const int32_t* w_sel;
  long long w_stride;         // fp16: elements per matrix; q4: bytes of packed nibbles per matrix
  long long w_stride_scales;  // q4: scale elements per matrix
  int n_slots;
  const float* y_scale;  // device scalar multiplying the product before the residual (null: 1)
  // Router run inside this launch (see the kernels): valid for a norm producer, at most 8
  // experts and in <= 8192; the slots then follow the experts found in the kernel (w_sel is
  // not read) and the results are published to the three device arrays.
  const half_t* router_Wr;
  int router_E, router_top;
  int32_t* router_experts;
  float* router_weights;
  float* router_logits;
};
int af_launch_gemv_f16(af_ctx* ctx, const af_gemv_args& a);
// AF_OPT_VALIDATE: queue the check of a caller's index list (ascending, unique, inside [0, n))
int af_validate_idx(af_ctx* ctx, const int32_t* idx, int nidx_host, const int32_t* nidx_dev, int n);
int af_launch_gemv_q4(af_ctx* ctx, const af_gemv_args& a);

// Union GEMV over B tokens (union.hip): builds the union of the tokens' index lists and runs
// the gathered GEMV once for all of them.  Arguments are taken as checked by the caller.
struct af_union_args {
  const void* Wt;
  int in, out, ld;
  const half_t* X;          // [B][in]
  int B;
  const int32_t* idx_b;     // [B][idx_stride]
  int idx_stride, k;        // k entries per list, or counts[b] <= k of them
  const int32_t* counts;    // device int32[B] or null
  int32_t* union_idx;       // [in]
  int32_t* union_n;         // [1]
  bool marked;              // the context's channel mask already holds the tokens' bits
  void* Y;                  // [B][out]
  int y_kind;
  const half_t* residual;   // [B][out] or null
};
int af_launch_union_f16(af_ctx* ctx, const af_union_args& u);
// Rotary embedding, KV append and attention of one token (layer.hip).
int af_launch_attention(af_ctx* ctx, const af_layer_cfg* cfg, const half_t* qkv, void* kc, void* vc,
                        int kv_len, int kv_cap, int pos, half_t* out);
// The same for B tokens in one launch; token b's qkv / out lie b * stride elements further.
int af_launch_attention_batch(af_ctx* ctx, const af_layer_cfg* cfg, int B, const half_t* qkv,
                              long long qkv_stride, void* const* kcs, void* const* vcs, const int* kv_len,
                              int kv_cap, const int* pos, half_t* out, long long out_stride);

// ---- cross-workgroup hand-off without cache-wide fences ------------------------------------
// Partial results travel between workgroups (possibly on different XCDs, each with its own
// L2) through agent-scope relaxed atomics: such a store is written through to memory, such a
// load does not hit a stale L2 line.  A full agent-scope fence would write back and invalidate
// the whole L2 of the XCD on every call, which serialises thousands of workgroups.
// Protocol: every thread stores its partials with af_store_agent, waits for its own stores
// (af_stores_done), the workgroup barriers, one thread takes a ticket; the workgroup whose
// ticket is the last one reads all partials with af_load_agent.
#ifdef __HIPCC__
__device__ __forceinline__ void af_store_agent(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float af_load_agent(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Sum of S partials p[0], p[stride], ... in index order, with up to 16 loads in flight.
__device__ __forceinline__ float af_sum_partials(const float* p, size_t stride, int S) {
  float v = 0.f;
  int q = 0;
  for (; q + 16 <= S; q += 16) {
    float t[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) t[u] = af_load_agent(p + (size_t)(q + u) * stride);
#pragma unroll
    for (int u = 0; u < 16; ++u) v += t[u];
  }
  float t[16];
#pragma unroll
  for (int u = 0; u < 16; ++u) t[u] = (q + u < S) ? af_load_agent(p + (size_t)(q + u) * stride) : 0.f;
#pragma unroll
  for (int u = 0; u < 16; ++u) v += t[u];
  return v;
}
__device__ __forceinline__ void af_stores_done() {
  // Keep the compiler from moving the stores, then wait until this wave's vector memory
  // operations (gfx9 counts stores in vmcnt) have been acknowledged: s_waitcnt vmcnt(0) with
  // expcnt and lgkmcnt left at their maxima (gfx9 encoding 0x0F70).
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_s_waitcnt(0x0F70);
}
__device__ __forceinline__ void af_ticket_reset(int* t) {
  __hip_atomic_store(t, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// -DAF_TICKET_ACQ_REL builds the form that is ordered by the language's memory model alone
// (the release writes the XCD's L2 back, the acquire invalidates it).  Measured: about 2 us
// more per kernel (7B stack 2.49 -> 2.76 ms per token), so the default relies on the
// write-through / acknowledged-store behaviour described above.
__device__ __forceinline__ int af_ticket_take(int* t) {
#ifdef AF_TICKET_ACQ_REL
  return __hip_atomic_fetch_add(t, 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
#else
  return __hip_atomic_fetch_add(t, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#endif
}
#endif

#ifdef __HIPCC__
// A caller-supplied channel index outside [0, n): reported in the device error word (which lies
// AF_TICKET_ERR ints behind the ticket area the kernel already knows) and replaced by a row
// that contributes nothing, so no access ever leaves the caller's buffers.
__device__ __forceinline__ void af_report_bad_index(int* tickets) {
  __hip_atomic_fetch_or(tickets + AF_TICKET_ERR, (int)AF_DEVERR_IDX, __ATOMIC_RELAXED,
                        __HIP_MEMORY_SCOPE_AGENT);
}

// ceil(a / s) for 0 <= a < 2^22 and 1 <= s <= 4096 without the integer-division sequence (some
// forty dependent instructions on this chip, in the start-up path of every workgroup): one
// float reciprocal and a correction step.
__device__ __forceinline__ int af_ceil_div_small(int a, int s) {
  const int b = a + s - 1;
  int q = (int)((float)b * __builtin_amdgcn_rcpf((float)s));
  const int r = b - q * s;
  q += (r >= s) - (r < 0);
  return q;
}

// A load of data that is used once (weight rows): marked non-temporal so that it does not
// displace lines that are used again; a plain streaming read of HBM measured about 10 % faster
// with this mark (6.7 against 6.05 TB/s).
template <typename T>
__device__ __forceinline__ T af_load_once(const T* p) {
  return __builtin_nontemporal_load(p);
}

// Time stamps of a layer kernel (af_profile_set): slot[0] = earliest entry, slot[1] = latest
// exit over its workgroups, in ticks of the device's constant-rate wall clock.
__device__ __forceinline__ void af_prof_begin(long long* slot) {
  if (slot && threadIdx.x == 0) atomicMin((unsigned long long*)slot, (unsigned long long)wall_clock64());
}
__device__ __forceinline__ void af_prof_end(long long* slot) {
  if (slot && threadIdx.x == 0) atomicMax((unsigned long long*)slot + 1, (unsigned long long)wall_clock64());
}


// ---- wave64 scans and sums on the DPP data path ------------------------------------------
// Inclusive prefix sum over the 64 lanes of a wave: four row_shr steps scan each row of 16
// lanes (lanes shifted in from outside the row read 0), row_bcast:15 adds a row's total to
// the next row (rows 1 and 3), row_bcast:31 adds the total of rows 0-1 to rows 2-3.  These
// are VALU operations; the shuffle intrinsics go through the LDS crossbar instead and cost
// several hundred cycles for the same scan.
__device__ __forceinline__ unsigned af_wave_incl_scan(unsigned v) {
  v += (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, false);  // row_shr:1
  v += (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, false);  // row_shr:2
  v += (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, false);  // row_shr:4
  v += (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, false);  // row_shr:8
  v += (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xa, 0xf, false);  // row_bcast:15
  v += (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xc, 0xf, false);  // row_bcast:31
  return v;
}
__device__ __forceinline__ float af_wave_incl_scan(float v) {
#define AF_DPP_F(ctrl, rmask) \
  __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), ctrl, rmask, 0xf, false))
  v += AF_DPP_F(0x111, 0xf);
  v += AF_DPP_F(0x112, 0xf);
  v += AF_DPP_F(0x114, 0xf);
  v += AF_DPP_F(0x118, 0xf);
  v += AF_DPP_F(0x142, 0xa);
  v += AF_DPP_F(0x143, 0xc);
#undef AF_DPP_F
  return v;
}
// Sum over the wave, returned to every lane (lane 63 of the scan holds it).
__device__ __forceinline__ unsigned af_wave_sum(unsigned v) {
  return (unsigned)__builtin_amdgcn_readlane((int)af_wave_incl_scan(v), 63);
}
__device__ __forceinline__ float af_wave_sum(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, af_wave_incl_scan(v)), 63));
}
#endif

static inline size_t af_align(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }
