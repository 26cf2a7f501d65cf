// Batch-1 decode step of a pre-norm decoder layer (block structure: Fig. "simplified
// transformer layer", Section 2.2) with activation selection (operation T) in front of every
// linear operator and the gathered GEMV (operation C) behind it; Section 3's reuse of a
// group leader's index sets is a bit mask over the four selection points.
//
// Launch sequence of one layer (all on the context's stream, no host synchronisation); the
// norm / SwiGLU producers and the selections run inside the GEMV kernels'
// front end, so a layer is five launches:
//   1 gemv  Wqkv     on rmsnorm(hidden), selecting        -> x_qkv, idx0, qkv
//   2 rope + kv append + attention                        -> attn
//   3 gemv  Wo       on attn, selecting, + hidden         -> idx1, h_mid
//   4 gemv  Wgateup  on rmsnorm(h_mid), selecting         -> x_gateup, idx2, gateup
//   5 gemv  Wdown    on silu(gate)*up, selecting, + h_mid -> x_down, idx3, hidden_out
// (the same holds for 4-bit weights: gemv_q4.hip shares the front end).
#include <math.h>
#include <stdlib.h>

#include "af_internal.h"
#include "row_prologue.h"
#include "gemv_f16_body.h"

#define ATT_THREADS 256
#define ATT_WAVES (ATT_THREADS / AF_WAVE)
#define ATT_MAX_KEYS 2048  // cache keys per (head, split) workgroup

struct AttnParams {
  const half_t* qkv;   // [q | k | v] of the new token, before rotation
  half_t* k_cache;     // [n_kv][cap][HD]
  half_t* v_cache;
  half_t* out;         // [n_heads*HD]
  float* part;         // [n_heads][KS][HD+2]
  int* tickets;        // [n_heads]
  int n_heads, n_kv, kv_len, kv_cap, head_dim;
  long long* prof;     // time stamps of this launch (af_profile_set), or null
  float cs[64], sn[64];  // cos / sin of pos * theta^(-2i/HD), i < HD/2, formed in fp64 on the host
};

// Output element `c` of one head from the partial results of its KS key splits
// ([KS][HD + 2]: running maximum, sum of weights, weighted values), summed in split order.  The
// partials come from other XCDs, so every batch of loads is a trip to memory: sixteen splits go
// out together (one trip for the usual split counts), and a running maximum rescales what
// earlier batches summed.
template <int HD>
__device__ __forceinline__ float attn_combine(const float* base, const int KS, const int c) {
  float M = -INFINITY, L = 0.f, v = 0.f;
  for (int q0 = 0; q0 < KS; q0 += 16) {
    float ms[16], ls[16], av[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const bool ok = q0 + u < KS;
      const float* pp = base + (size_t)(q0 + u) * (HD + 2);
      ms[u] = ok ? af_load_agent(pp) : -INFINITY;
      ls[u] = ok ? af_load_agent(pp + 1) : 0.f;
      av[u] = ok ? af_load_agent(pp + 2 + c) : 0.f;
    }
    float mb = M;
#pragma unroll
    for (int u = 0; u < 16; ++u) mb = fmaxf(mb, ms[u]);
    if (mb == -INFINITY) continue;  // nothing but empty splits so far
    const float keep = (M == -INFINITY) ? 0.f : expf(M - mb);
    L *= keep;
    v *= keep;
    M = mb;
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      if (ms[u] != -INFINITY) {  // an empty split has nothing to add
        const float wgt = expf(ms[u] - M);
        L += wgt * ls[u];
        v += wgt * av[u];
      }
    }
  }
  return v / L;
}

// One (head, key split) workgroup of the decode attention.  cs / sn: the rotary table of the
// token's position (kernel arguments for the single-token launch, LDS for the batched one).
template <int HD>
__device__ __forceinline__ void attn_decode_body(const AttnParams& p, const float* cs_tab,
                                                 const float* sn_tab, const int h, const int s,
                                                 const int KS) {
  constexpr int LPK = HD / 8;             // lanes per key (8 dims = 16 bytes each)
  constexpr int KPB = ATT_THREADS / LPK;  // keys per workgroup iteration
  constexpr int NB = 4;                   // iterations whose loads are issued together
  __shared__ float s_q[HD];
  __shared__ float s_knew[HD];
  __shared__ float s_vnew[HD];
  __shared__ float s_sc[ATT_MAX_KEYS + 1];
  __shared__ float s_pv[KPB][HD];
  __shared__ float s_red[ATT_WAVES];
  __shared__ int s_last;

  af_prof_begin(p.prof);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int rep = p.n_heads / p.n_kv, kvh = h / rep;
  const int T = p.kv_len;
  const int KP = (T + KS - 1) / KS;
  const int t0 = min(s * KP, T), t1 = min(t0 + KP, T);
  const int cnt = t1 - t0;
  const bool owns_new = (s == KS - 1);
  const int total = cnt + (owns_new ? 1 : 0);

  const half_t* q = p.qkv + (size_t)h * HD;
  const half_t* kn = p.qkv + (size_t)(p.n_heads + kvh) * HD;
  const half_t* vn = p.qkv + (size_t)(p.n_heads + p.n_kv + kvh) * HD;
  half_t* Kc = p.k_cache + (size_t)kvh * p.kv_cap * HD;
  half_t* Vc = p.v_cache + (size_t)kvh * p.kv_cap * HD;
  const int lk = tid % LPK, kq = tid / LPK;  // my slice of the head dim, my key slot
  half8 zero8;
#pragma unroll
  for (int c = 0; c < 8; ++c) zero8[c] = (half_t)0;

  // the first NB key/value rows of this thread go out before anything else needs them
  half8 kv[NB], vv[NB];
#pragma unroll
  for (int u = 0; u < NB; ++u) {
    const int i = kq + u * KPB;
    const bool ok = i < cnt;
    kv[u] = ok ? af_load_once(reinterpret_cast<const half8*>(Kc + (size_t)(t0 + i) * HD + lk * 8)) : zero8;
    vv[u] = ok ? af_load_once(reinterpret_cast<const half8*>(Vc + (size_t)(t0 + i) * HD + lk * 8)) : zero8;
  }

  if (tid < HD / 2) {
    const float a = (float)q[tid], b = (float)q[tid + HD / 2];
    const float cs = cs_tab[tid], sn = sn_tab[tid];
    const float sc = 1.0f / sqrtf((float)HD);
    s_q[tid] = (a * cs - b * sn) * sc;
    s_q[tid + HD / 2] = (b * cs + a * sn) * sc;
  } else if (owns_new && tid >= 64 && tid < 64 + HD / 2) {
    const int i = tid - 64;
    const float a = (float)kn[i], b = (float)kn[i + HD / 2];
    const float cs = cs_tab[i], sn = sn_tab[i];
    const half_t ha = (half_t)(a * cs - b * sn), hb = (half_t)(b * cs + a * sn);  // cache is fp16
    s_knew[i] = (float)ha;
    s_knew[i + HD / 2] = (float)hb;
    if (h % rep == 0) {
      Kc[(size_t)p.kv_len * HD + i] = ha;
      Kc[(size_t)p.kv_len * HD + i + HD / 2] = hb;
    }
  } else if (owns_new && tid >= 128 && tid < 128 + HD) {
    const int i = tid - 128;
    const half_t v = vn[i];
    s_vnew[i] = (float)v;
    if (h % rep == 0) Vc[(size_t)p.kv_len * HD + i] = v;
  }
  __syncthreads();

  // ---- scores ------------------------------------------------------------------------
  float qr[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) qr[c] = s_q[lk * 8 + c];
  auto score = [&](const half8& k8, int i) {
    float d = 0.f;
#pragma unroll
    for (int c = 0; c < 8; ++c) d += (float)k8[c] * qr[c];
#pragma unroll
    for (int off = 1; off < LPK; off <<= 1) d += __shfl_xor(d, off, AF_WAVE);
    if (lk == 0 && i < cnt) s_sc[i] = d;
  };
#pragma unroll
  for (int u = 0; u < NB; ++u) score(kv[u], kq + u * KPB);
  for (int i0 = kq + NB * KPB; i0 < cnt; i0 += NB * KPB) {  // long caches: further batches
    half8 k2[NB];
#pragma unroll
    for (int u = 0; u < NB; ++u) {
      const int i = i0 + u * KPB;
      k2[u] = i < cnt ? af_load_once(reinterpret_cast<const half8*>(Kc + (size_t)(t0 + i) * HD + lk * 8)) : zero8;
    }
#pragma unroll
    for (int u = 0; u < NB; ++u) score(k2[u], i0 + u * KPB);
  }
  if (owns_new && wave == 0) {
    float d = 0.f;
    for (int c = lane; c < HD; c += AF_WAVE) d += s_q[c] * s_knew[c];
    d = af_wave_sum(d);
    if (lane == 0) s_sc[cnt] = d;
  }
  __syncthreads();

  // ---- local softmax -----------------------------------------------------------------
  float m = -INFINITY;
  for (int i = tid; i < total; i += ATT_THREADS) m = fmaxf(m, s_sc[i]);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, AF_WAVE));
  if (lane == 0) s_red[wave] = m;
  __syncthreads();
  m = s_red[0];
#pragma unroll
  for (int w = 1; w < ATT_WAVES; ++w) m = fmaxf(m, s_red[w]);
  __syncthreads();
  float l = 0.f;
  for (int i = tid; i < total; i += ATT_THREADS) {
    float e = expf(s_sc[i] - m);
    s_sc[i] = e;
    l += e;
  }
  l = af_wave_sum(l);
  if (lane == 0) s_red[wave] = l;
  __syncthreads();
  l = 0.f;
#pragma unroll
  for (int w = 0; w < ATT_WAVES; ++w) l += s_red[w];

  // ---- weighted values ---------------------------------------------------------------
  float acc[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) acc[c] = 0.f;
#pragma unroll
  for (int u = 0; u < NB; ++u) {
    const int i = kq + u * KPB;
    const float pw = i < cnt ? s_sc[i] : 0.f;
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[c] += pw * (float)vv[u][c];
  }
  for (int i0 = kq + NB * KPB; i0 < cnt; i0 += NB * KPB) {
    half8 v2[NB];
#pragma unroll
    for (int u = 0; u < NB; ++u) {
      const int i = i0 + u * KPB;
      v2[u] = i < cnt ? af_load_once(reinterpret_cast<const half8*>(Vc + (size_t)(t0 + i) * HD + lk * 8)) : zero8;
    }
#pragma unroll
    for (int u = 0; u < NB; ++u) {
      const int i = i0 + u * KPB;
      const float pw = i < cnt ? s_sc[i] : 0.f;
#pragma unroll
      for (int c = 0; c < 8; ++c) acc[c] += pw * (float)v2[u][c];
    }
  }
#pragma unroll
  for (int c = 0; c < 8; ++c) s_pv[kq][lk * 8 + c] = acc[c];
  __syncthreads();
  float* mine = p.part + ((size_t)h * KS + s) * (HD + 2);
  if (tid < HD) {
    float v = 0.f;
#pragma unroll 4
    for (int g = 0; g < KPB; ++g) v += s_pv[g][tid];
    if (owns_new) v += s_sc[cnt] * s_vnew[tid];
    if (KS == 1) {
      p.out[(size_t)h * HD + tid] = (half_t)(v / l);
    } else {
      af_store_agent(mine + 2 + tid, v);
    }
  }
  if (KS == 1) {
    af_prof_end(p.prof);
    return;
  }
  if (tid == 0) {
    af_store_agent(mine, m);
    af_store_agent(mine + 1, l);
  }
  af_stores_done();
  __syncthreads();
  if (tid == 0) {
    int old = af_ticket_take(&p.tickets[h]);
    s_last = (old == KS - 1);
  }
  __syncthreads();
  if (!s_last) {
    af_prof_end(p.prof);
    return;
  }
  const float* base = p.part + (size_t)h * KS * (HD + 2);
  if (tid < HD) p.out[(size_t)h * HD + tid] = (half_t)attn_combine<HD>(base, KS, tid);
  if (tid == 0) af_ticket_reset(&p.tickets[h]);
  af_prof_end(p.prof);
}

template <int HD>
__global__ __launch_bounds__(ATT_THREADS) void attn_decode_kernel(AttnParams p) {
  attn_decode_body<HD>(p, p.cs, p.sn, blockIdx.x, blockIdx.y, gridDim.y);
}

// The same for B tokens in one launch (af_decode_layer_batch): grid (heads, key splits, tokens);
// every token has its own caches, length, position and number of key splits.  The rotary table
// of a token is formed here, in fp64 like the host does for the single-token launch
// (angle = pos * theta^(-2i/HD) with the host's theta^(-2i/HD)).
struct AttnBatchParams {
  AttnParams base;          // token 0's qkv / out, the shared sizes; cs / sn unused
  half_t* k_caches[AF_MAX_BATCH];
  half_t* v_caches[AF_MAX_BATCH];
  int kv_lens[AF_MAX_BATCH];
  int poss[AF_MAX_BATCH];
  int splits[AF_MAX_BATCH];  // key splits of each token
  double inv_freq[64];
  long long qkv_stride, out_stride, part_stride;  // elements between the tokens
};

template <int HD>
__global__ __launch_bounds__(ATT_THREADS) void attn_decode_batch_kernel(AttnBatchParams bp) {
  __shared__ float s_cs[HD / 2], s_sn[HD / 2];
  const int b = blockIdx.z;
  const int KS = bp.splits[b];
  if ((int)blockIdx.y >= KS) return;  // uniform for the workgroup: this token has fewer splits
  AttnParams p = bp.base;
  p.qkv += (size_t)b * bp.qkv_stride;
  p.out += (size_t)b * bp.out_stride;
  p.part += (size_t)b * bp.part_stride;
  p.tickets += b * p.n_heads;
  p.k_cache = bp.k_caches[b];
  p.v_cache = bp.v_caches[b];
  p.kv_len = bp.kv_lens[b];
  if (threadIdx.x < HD / 2) {
    const double ang = (double)bp.poss[b] * bp.inv_freq[threadIdx.x];
    s_cs[threadIdx.x] = (float)cos(ang);
    s_sn[threadIdx.x] = (float)sin(ang);
  }
  __syncthreads();
  attn_decode_body<HD>(p, s_cs, s_sn, blockIdx.x, blockIdx.y, KS);
}

int af_launch_attention(af_ctx* ctx, const af_layer_cfg* cfg, const half_t* qkv, void* kc, void* vc,
                        int kv_len, int kv_cap, int pos, half_t* out) {
  // One split per 64 keys up to two workgroups per compute unit over all heads; beyond that
  // more splits only lengthen the combine (7B shape, 2048 keys: 32 splits 86.4 us per layer,
  // 16 splits 80.5 us).
  int KS = (kv_len + 63) / 64;
  const int ks_cap = 2 * ctx->n_cu / cfg->n_heads > 1 ? 2 * ctx->n_cu / cfg->n_heads : 1;
  if (KS > ks_cap) KS = ks_cap;
  if (KS < (kv_len + ATT_MAX_KEYS - 1) / ATT_MAX_KEYS) KS = (kv_len + ATT_MAX_KEYS - 1) / ATT_MAX_KEYS;  // very long caches
  if (ctx->tune_attn_splits > 0) KS = ctx->tune_attn_splits;
  if (KS < 1) KS = 1;
  if (KS > 64) KS = 64;
  while ((size_t)cfg->n_heads * KS * (cfg->head_dim + 2) > ctx->lay.attn_floats && KS > 1) --KS;
  if ((kv_len + KS - 1) / KS > ATT_MAX_KEYS) return AF_EINVAL;
  AttnParams p;
  p.qkv = qkv;
  p.k_cache = (half_t*)kc;
  p.v_cache = (half_t*)vc;
  p.out = out;
  p.part = (float*)(ctx->ws + ctx->lay.attn_part);
  p.tickets = (int*)(ctx->ws + ctx->lay.tickets) + AF_TICKET_ATTN;
  p.n_heads = cfg->n_heads;
  p.n_kv = cfg->n_kv_heads;
  p.kv_len = kv_len;
  p.kv_cap = kv_cap;
  p.head_dim = cfg->head_dim;
  p.prof = af_prof_take(ctx);
  for (int i = 0; i < cfg->head_dim / 2; ++i) {
    const double ang = (double)pos * pow((double)cfg->rope_theta, -2.0 * (double)i / (double)cfg->head_dim);
    p.cs[i] = (float)cos(ang);
    p.sn[i] = (float)sin(ang);
  }
  dim3 grid(cfg->n_heads, KS);
  if (cfg->head_dim == 128)
    hipLaunchKernelGGL(attn_decode_kernel<128>, grid, dim3(ATT_THREADS), 0, ctx->stream, p);
  else
    hipLaunchKernelGGL(attn_decode_kernel<64>, grid, dim3(ATT_THREADS), 0, ctx->stream, p);
  AF_LAUNCH_CHECK();
  return AF_OK;
}

int af_launch_attention_batch(af_ctx* ctx, const af_layer_cfg* cfg, int B, const half_t* qkv,
                              long long qkv_stride, void* const* kcs, void* const* vcs, const int* kv_len,
                              int kv_cap, const int* pos, half_t* out, long long out_stride) {
  AttnBatchParams bp{};
  AttnParams& p = bp.base;
  int ks_max = 1;
  const size_t per_split = (size_t)cfg->n_heads * (cfg->head_dim + 2);
  for (int b = 0; b < B; ++b) {
    int KS = (kv_len[b] + 63) / 64;
    const int ks_cap = 2 * ctx->n_cu / cfg->n_heads > 1 ? 2 * ctx->n_cu / cfg->n_heads : 1;
    if (KS > ks_cap) KS = ks_cap;
    if (KS < (kv_len[b] + ATT_MAX_KEYS - 1) / ATT_MAX_KEYS) KS = (kv_len[b] + ATT_MAX_KEYS - 1) / ATT_MAX_KEYS;
    if (KS < 1) KS = 1;
    if (KS > 64) KS = 64;
    while (KS > 1 && (size_t)B * KS * per_split > ctx->lay.attn_floats) --KS;
    if ((kv_len[b] + KS - 1) / KS > ATT_MAX_KEYS) return AF_EINVAL;
    bp.splits[b] = KS;
    if (KS > ks_max) ks_max = KS;
    bp.k_caches[b] = (half_t*)kcs[b];
    bp.v_caches[b] = (half_t*)vcs[b];
    bp.kv_lens[b] = kv_len[b];
    bp.poss[b] = pos[b];
  }
  if ((size_t)B * ks_max * per_split > ctx->lay.attn_floats) return AF_EWORKSPACE;
  p.qkv = qkv;
  p.out = out;
  p.part = (float*)(ctx->ws + ctx->lay.attn_part);
  p.tickets = (int*)(ctx->ws + ctx->lay.tickets) + AF_TICKET_ATTN;
  p.n_heads = cfg->n_heads;
  p.n_kv = cfg->n_kv_heads;
  p.kv_cap = kv_cap;
  p.head_dim = cfg->head_dim;
  p.prof = nullptr;
  for (int i = 0; i < cfg->head_dim / 2; ++i)
    bp.inv_freq[i] = pow((double)cfg->rope_theta, -2.0 * (double)i / (double)cfg->head_dim);
  bp.qkv_stride = qkv_stride;
  bp.out_stride = out_stride;
  bp.part_stride = (long long)ks_max * (long long)per_split;
  dim3 grid(cfg->n_heads, ks_max, B);
  if (cfg->head_dim == 128)
    hipLaunchKernelGGL(attn_decode_batch_kernel<128>, grid, dim3(ATT_THREADS), 0, ctx->stream, bp);
  else
    hipLaunchKernelGGL(attn_decode_batch_kernel<64>, grid, dim3(ATT_THREADS), 0, ctx->stream, bp);
  AF_LAUNCH_CHECK();
  return AF_OK;
}

// ---- whole-layer kernel -------------------------------------------------------------------
// The five operators of a layer as phases of ONE launch of 1024-thread workgroups, one per
// compute unit, all resident at once.  A phase hands its result to the next one through
// memory: the workgroup that completes a tile (or a head) stores it through to memory, waits
// for the acknowledgement and adds one to the phase's counter; a workgroup enters a phase once
// the counter of the phase before has reached its total.  Every address a phase reads with
// plain loads is written at most once per launch and only before that phase starts, so no
// compute unit can hold a stale copy.  Waits are bounded: a wait that does not end sets the
// device error word and the workgroup leaves the kernel, so the grid always drains.
// What the phases do not depend on is fetched before the wait (the attention phase loads its
// share of the KV cache while the qkv projection is still being reduced).
#define LAYER_THREADS 1024
#define LAYER_WAVES (LAYER_THREADS / AF_WAVE)
#define LAYER_SPIN_LIMIT (1 << 21)
#define LAYER_ATT_MAX_KEYS 2048

struct LayerParams {
  GemvParams g[4];  // qkv, o, gate|up, down
  int tiles[4], S[4], lx[4];
  AttnParams at;
  int KS;           // key splits per head
  int* done;        // [5] phase counters: qkv, attention, o, gate|up, down
  int* err;
};

// All threads of the workgroup wait until *counter >= target (polled by one thread); false if
// the bounded wait ran out (the error word is set, the caller leaves the kernel).
__device__ __forceinline__ bool layer_wait(const int* counter, int target, int* err, int& s_flag) {
  if (threadIdx.x == 0) {
    int ok = 0;
    for (int i = 0; i < LAYER_SPIN_LIMIT; ++i) {
      if (__hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= target) {
        ok = 1;
        break;
      }
      __builtin_amdgcn_s_sleep(2);
    }
    if (!ok) __hip_atomic_fetch_or(err, (int)AF_DEVERR_SPIN, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_flag = ok;
  }
  __syncthreads();
  const bool ok = s_flag != 0;
  __syncthreads();  // s_flag may be rewritten by the next wait
  return ok;
}

// LDS of the attention phase, carved from the dynamic region (floats).
template <int HD>
struct AttnLds {
  static constexpr int LPK = HD / 8;
  static constexpr int KPB = LAYER_THREADS / LPK;
  static constexpr int PARTS = LAYER_THREADS / HD;
  static constexpr int Q = 0, KNEW = HD, VNEW = 2 * HD, RED = 3 * HD, SC = 3 * HD + 32,
                       PV = SC + LAYER_ATT_MAX_KEYS + 16, PV2 = PV + KPB * HD, END = PV2 + PARTS * HD;
};
#define LAYER_ATT_LDS_BYTES (4 * (AttnLds<128>::END > AttnLds<64>::END ? AttnLds<128>::END : AttnLds<64>::END))

// Attention of (head h, key split s) by one 1024-thread workgroup; same arithmetic as
// attn_decode_kernel.  The cached keys and values of the split are requested first, then the
// workgroup waits for the qkv projection (counter `ready` reaching `ready_total`).
template <int HD>
__device__ __forceinline__ bool attn_phase(const AttnParams& p, int h, int s, int KS, float* lds,
                                           int& s_last, int& s_flag, const int* ready, int ready_total,
                                           int* done, int* done_prev, int* err) {
  typedef AttnLds<HD> L;
  constexpr int LPK = L::LPK, KPB = L::KPB, NB = 2, PARTS = L::PARTS;
  float* s_q = lds + L::Q;
  float* s_knew = lds + L::KNEW;
  float* s_vnew = lds + L::VNEW;
  float* s_red = lds + L::RED;
  float* s_sc = lds + L::SC;
  float(*s_pv)[HD] = reinterpret_cast<float(*)[HD]>(lds + L::PV);
  float(*s_pv2)[HD] = reinterpret_cast<float(*)[HD]>(lds + L::PV2);
  unsigned short* s_out = reinterpret_cast<unsigned short*>(lds + L::KNEW);  // reused for the result

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int rep = p.n_heads / p.n_kv, kvh = h / rep;
  const int T = p.kv_len;
  const int KP = (T + KS - 1) / KS;
  const int t0 = min(s * KP, T), t1 = min(t0 + KP, T);
  const int cnt = t1 - t0;
  const bool owns_new = (s == KS - 1);
  const int total = cnt + (owns_new ? 1 : 0);

  const half_t* q = p.qkv + (size_t)h * HD;
  const half_t* kn = p.qkv + (size_t)(p.n_heads + kvh) * HD;
  const half_t* vn = p.qkv + (size_t)(p.n_heads + p.n_kv + kvh) * HD;
  half_t* Kc = p.k_cache + (size_t)kvh * p.kv_cap * HD;
  half_t* Vc = p.v_cache + (size_t)kvh * p.kv_cap * HD;
  const int lk = tid % LPK, kq = tid / LPK;  // my slice of the head dim, my key slot
  half8 zero8;
#pragma unroll
  for (int c = 0; c < 8; ++c) zero8[c] = (half_t)0;

  // cached rows first: they do not depend on this token
  half8 kv[NB], vv[NB];
#pragma unroll
  for (int u = 0; u < NB; ++u) {
    const int i = kq + u * KPB;
    const bool ok = i < cnt;
    kv[u] = ok ? af_load_once(reinterpret_cast<const half8*>(Kc + (size_t)(t0 + i) * HD + lk * 8)) : zero8;
    vv[u] = ok ? af_load_once(reinterpret_cast<const half8*>(Vc + (size_t)(t0 + i) * HD + lk * 8)) : zero8;
  }
  if (!layer_wait(ready, ready_total, err, s_flag)) return false;
  af_prof_begin(p.prof);

  if (tid < HD / 2) {
    const float a = (float)q[tid], b = (float)q[tid + HD / 2];
    const float cs = p.cs[tid], sn = p.sn[tid];
    const float sc = 1.0f / sqrtf((float)HD);
    s_q[tid] = (a * cs - b * sn) * sc;
    s_q[tid + HD / 2] = (b * cs + a * sn) * sc;
  } else if (owns_new && tid >= 64 && tid < 64 + HD / 2) {
    const int i = tid - 64;
    const float a = (float)kn[i], b = (float)kn[i + HD / 2];
    const float cs = p.cs[i], sn = p.sn[i];
    const half_t ha = (half_t)(a * cs - b * sn), hb = (half_t)(b * cs + a * sn);  // cache is fp16
    s_knew[i] = (float)ha;
    s_knew[i + HD / 2] = (float)hb;
    if (h % rep == 0) {
      Kc[(size_t)p.kv_len * HD + i] = ha;
      Kc[(size_t)p.kv_len * HD + i + HD / 2] = hb;
    }
  } else if (owns_new && tid >= 128 && tid < 128 + HD) {
    const int i = tid - 128;
    const half_t v = vn[i];
    s_vnew[i] = (float)v;
    if (h % rep == 0) Vc[(size_t)p.kv_len * HD + i] = v;
  }
  __syncthreads();

  // ---- scores ------------------------------------------------------------------------
  float qr[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) qr[c] = s_q[lk * 8 + c];
  auto score = [&](const half8& k8, int i) {
    float d = 0.f;
#pragma unroll
    for (int c = 0; c < 8; ++c) d += (float)k8[c] * qr[c];
#pragma unroll
    for (int off = 1; off < LPK; off <<= 1) d += __shfl_xor(d, off, AF_WAVE);
    if (lk == 0 && i < cnt) s_sc[i] = d;
  };
#pragma unroll
  for (int u = 0; u < NB; ++u) score(kv[u], kq + u * KPB);
  for (int i0 = kq + NB * KPB; i0 < cnt; i0 += NB * KPB) {  // long caches: further batches
    half8 k2[NB];
#pragma unroll
    for (int u = 0; u < NB; ++u) {
      const int i = i0 + u * KPB;
      k2[u] = i < cnt ? af_load_once(reinterpret_cast<const half8*>(Kc + (size_t)(t0 + i) * HD + lk * 8)) : zero8;
    }
#pragma unroll
    for (int u = 0; u < NB; ++u) score(k2[u], i0 + u * KPB);
  }
  if (owns_new && wave == 0) {
    float d = 0.f;
    for (int c = lane; c < HD; c += AF_WAVE) d += s_q[c] * s_knew[c];
    d = af_wave_sum(d);
    if (lane == 0) s_sc[cnt] = d;
  }
  __syncthreads();

  // ---- local softmax -----------------------------------------------------------------
  float m = -INFINITY;
  for (int i = tid; i < total; i += LAYER_THREADS) m = fmaxf(m, s_sc[i]);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, AF_WAVE));
  if (lane == 0) s_red[wave] = m;
  __syncthreads();
  m = s_red[0];
#pragma unroll
  for (int w = 1; w < LAYER_WAVES; ++w) m = fmaxf(m, s_red[w]);
  __syncthreads();
  float l = 0.f;
  for (int i = tid; i < total; i += LAYER_THREADS) {
    float e = expf(s_sc[i] - m);
    s_sc[i] = e;
    l += e;
  }
  l = af_wave_sum(l);
  if (lane == 0) s_red[wave] = l;
  __syncthreads();
  l = 0.f;
#pragma unroll
  for (int w = 0; w < LAYER_WAVES; ++w) l += s_red[w];

  // ---- weighted values ---------------------------------------------------------------
  float acc[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) acc[c] = 0.f;
#pragma unroll
  for (int u = 0; u < NB; ++u) {
    const int i = kq + u * KPB;
    const float pw = i < cnt ? s_sc[i] : 0.f;
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[c] += pw * (float)vv[u][c];
  }
  for (int i0 = kq + NB * KPB; i0 < cnt; i0 += NB * KPB) {
    half8 v2[NB];
#pragma unroll
    for (int u = 0; u < NB; ++u) {
      const int i = i0 + u * KPB;
      v2[u] = i < cnt ? af_load_once(reinterpret_cast<const half8*>(Vc + (size_t)(t0 + i) * HD + lk * 8)) : zero8;
    }
#pragma unroll
    for (int u = 0; u < NB; ++u) {
      const int i = i0 + u * KPB;
      const float pw = i < cnt ? s_sc[i] : 0.f;
#pragma unroll
      for (int c = 0; c < 8; ++c) acc[c] += pw * (float)v2[u][c];
    }
  }
#pragma unroll
  for (int c = 0; c < 8; ++c) s_pv[kq][lk * 8 + c] = acc[c];
  __syncthreads();
  {  // key slots -> PARTS partial rows -> one row, always in slot order
    const int c = tid % HD, part = tid / HD;
    constexpr int PER = KPB / PARTS;
    float v = 0.f;
#pragma unroll 4
    for (int g = 0; g < PER; ++g) v += s_pv[part * PER + g][c];
    s_pv2[part][c] = v;
  }
  __syncthreads();
  float* mine = p.part + ((size_t)h * KS + s) * (HD + 2);
  unsigned short* outp = reinterpret_cast<unsigned short*>(p.out) + (size_t)h * HD;
  if (tid < HD) {
    float v = 0.f;
#pragma unroll
    for (int g = 0; g < PARTS; ++g) v += s_pv2[g][tid];
    if (owns_new) v += s_sc[cnt] * s_vnew[tid];
    if (KS == 1) {
      s_out[tid] = __builtin_bit_cast(unsigned short, (half_t)(v / l));
    } else {
      af_store_agent(mine + 2 + tid, v);
    }
  }
  bool finisher = KS == 1;
  if (KS > 1) {
    if (tid == 0) {
      af_store_agent(mine, m);
      af_store_agent(mine + 1, l);
    }
    af_stores_done();
    __syncthreads();
    if (tid == 0) {
      int old = af_ticket_take(&p.tickets[h]);
      s_last = (old == KS - 1);
    }
    __syncthreads();
    finisher = s_last != 0;
    if (finisher) {
      const float* base = p.part + (size_t)h * KS * (HD + 2);
      if (tid < HD) s_out[tid] = __builtin_bit_cast(unsigned short, (half_t)attn_combine<HD>(base, KS, tid));
      if (tid == 0) af_ticket_reset(&p.tickets[h]);
    }
  }
  if (finisher) {  // one finished head: stored through as 8-byte pieces, acknowledged, then counted
    __syncthreads();
    if (tid < HD / 4)
      __hip_atomic_store(reinterpret_cast<unsigned long long*>(outp) + tid,
                         reinterpret_cast<const unsigned long long*>(s_out)[tid], __ATOMIC_RELAXED,
                         __HIP_MEMORY_SCOPE_AGENT);
    af_stores_done();
    __syncthreads();
    if (tid == 0) {
      const int old = __hip_atomic_fetch_add(done, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (old == p.n_heads - 1)
        __hip_atomic_store(done_prev, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  af_prof_end(p.prof);
  return true;
}

// One GEMV phase: operator OP of the layer (0 qkv, 1 o, 2 gate|up, 3 down) in phase PH.
template <int LX, int OP, int PH>
__device__ __forceinline__ bool layer_gemv_phase(const LayerParams& P, int w, unsigned short* xs,
                                                 GemvLds<LAYER_WAVES>& lds, int& s_flag) {
  const int tiles = P.tiles[OP], S = P.S[OP];
  if (w >= tiles * S) return true;
  if (PH > 0) {
    const int need = PH == 2 ? P.at.n_heads : P.tiles[OP - 1];
    if (!layer_wait(P.done + PH - 1, need, P.err, s_flag)) return false;
  }
  const GemvPos vb = {w % tiles, w / tiles, tiles, S};
  const GemvParams g = P.g[OP];  // a copy of its own: the fields settle in scalar registers
  gemv_f16_body<LX, 8, LAYER_WAVES, false, true>(g, vb, xs, lds);
  __syncthreads();  // the next phase reuses the workgroup's LDS
  return true;
}

// LX_QKV, LX_GU: lanes across a tile of the q|k|v and the gate|up operator (the wide ones); o and
// down use 16 (128-column tiles).
template <int LX_QKV, int LX_GU>
__global__ __launch_bounds__(LAYER_THREADS) void layer_f16_kernel(LayerParams P) {
  extern __shared__ __align__(16) unsigned short xs[];
  __shared__ GemvLds<LAYER_WAVES> lds;
  __shared__ int s_flag;
  const int w = blockIdx.x;
  if (!layer_gemv_phase<LX_QKV, 0, 0>(P, w, xs, lds, s_flag)) return;
  if (w < P.at.n_heads * P.KS) {
    const int h = w % P.at.n_heads, s = w / P.at.n_heads;
    bool ok;
    if (P.at.head_dim == 128)
      ok = attn_phase<128>(P.at, h, s, P.KS, reinterpret_cast<float*>(xs), lds.last, s_flag, P.done + 0,
                           P.tiles[0], P.done + 1, P.done + 0, P.err);
    else
      ok = attn_phase<64>(P.at, h, s, P.KS, reinterpret_cast<float*>(xs), lds.last, s_flag, P.done + 0,
                          P.tiles[0], P.done + 1, P.done + 0, P.err);
    if (!ok) return;
    __syncthreads();
  }
  if (!layer_gemv_phase<16, 1, 2>(P, w, xs, lds, s_flag)) return;
  if (!layer_gemv_phase<LX_GU, 2, 3>(P, w, xs, lds, s_flag)) return;
  layer_gemv_phase<16, 3, 4>(P, w, xs, lds, s_flag);
}

static int check_layer_args(const af_ctx* ctx, const af_layer_cfg* cfg, const af_select_cfg* sel,
                            int kv_len, int kv_cap, int pos) {
  if (cfg->d_model <= 0 || cfg->n_heads <= 0 || cfg->n_kv_heads <= 0 || cfg->d_ffn <= 0)
    return AF_EINVAL;
  if (cfg->head_dim != 128 && cfg->head_dim != 64) return AF_ESHAPE;
  if (cfg->n_heads % cfg->n_kv_heads) return AF_ESHAPE;
  if (cfg->n_heads > AF_TICKET_PHASE - AF_TICKET_ATTN) return AF_ESHAPE;
  if (cfg->d_model % 8 || cfg->d_ffn % 8) return AF_ESHAPE;
  if (cfg->weight_kind != AF_W_F16 && cfg->weight_kind != AF_W_Q4G32 &&
      cfg->weight_kind != AF_W_Q4CL)
    return AF_EINVAL;
  const int qdim = cfg->n_heads * cfg->head_dim;
  if (cfg->weight_kind == AF_W_Q4G32 && (cfg->d_model % 32 || cfg->d_ffn % 32 || qdim % 32))
    return AF_ESHAPE;
  // channel-local groups run along the (fused) output columns
  if (cfg->weight_kind == AF_W_Q4CL &&
      (cfg->d_model % 32 || (2 * cfg->d_ffn) % 32 || ((cfg->n_heads + 2 * cfg->n_kv_heads) * cfg->head_dim) % 32))
    return AF_ESHAPE;
  if (kv_len < 0 || kv_cap <= 0 || kv_len >= kv_cap || pos < 0) return AF_EINVAL;
  if (sel->mode != AF_SEL_TOPK && sel->mode != AF_SEL_THRESHOLD && sel->mode != AF_SEL_DENSE)
    return AF_EINVAL;
  const int widths[4] = {cfg->d_model, qdim, cfg->d_model, cfg->d_ffn};
  for (int p = 0; p < 4; ++p) {
    if (widths[p] > AF_MAX_N) return AF_ESHAPE;
    if (sel->mode == AF_SEL_TOPK && (sel->k[p] < 0 || sel->k[p] > widths[p])) return AF_EINVAL;
    if (sel->mode == AF_SEL_THRESHOLD && sel->t[p] != sel->t[p]) return AF_EINVAL;
  }
  if (!ctx->ws) return AF_EWORKSPACE;
  const int qkv_out = (cfg->n_heads + 2 * cfg->n_kv_heads) * cfg->head_dim;
  int max_w = qkv_out > 2 * cfg->d_ffn ? qkv_out : 2 * cfg->d_ffn;
  int max_i = cfg->d_ffn > qdim ? cfg->d_ffn : qdim;
  if (cfg->d_model > max_i) max_i = cfg->d_model;
  if (max_w > ctx->max_out || max_i > ctx->max_in) return AF_EWORKSPACE;
  return AF_OK;
}

// The layer as one launch (fp16 weights).  Returns 1 if the configuration does not fit the
// whole-layer kernel (the caller then launches the operators one by one), else a status.
static int launch_layer_kernel(af_ctx* ctx, const af_layer_cfg* cfg, const af_gemv_args* ga,
                               const half_t* qkv, void* kc, void* vc, int kv_len, int kv_cap, int pos,
                               half_t* attn) {
  if (!ctx->use_layer_kernel || ctx->layer_kernel_state < 0) return 1;
  if (ctx->layer_kernel_state == 0) {
    // every workgroup of the grid has to be resident at the same time: one per compute unit
    int per_cu = 0;
    bool ok = true;
    const void* fns[3] = {reinterpret_cast<const void*>(layer_f16_kernel<16, 16>),
                          reinterpret_cast<const void*>(layer_f16_kernel<16, 64>),
                          reinterpret_cast<const void*>(layer_f16_kernel<32, 64>)};
    for (const void* fn : fns) {
      per_cu = 0;
      if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, AF_GEMV_LDS_BUDGET) != hipSuccess ||
          hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, LAYER_THREADS, AF_GEMV_LDS_BUDGET) != hipSuccess ||
          per_cu < 1)
        ok = false;
    }
    if (!ok) {
      (void)hipGetLastError();
      ctx->layer_kernel_state = -1;
      return 1;
    }
    ctx->layer_kernel_state = 1;
  }
  if (cfg->n_heads > ctx->n_cu) return 1;
  for (int op = 0; op < 4; ++op)
    if ((uintptr_t)ga[op].y & 7u) return 1;  // results leave as 8-byte stores
  LayerParams P{};
  size_t lds = LAYER_ATT_LDS_BYTES;
  int n_wg = 0;
  for (int op = 0; op < 4; ++op) {
    if (ga[op].w_sel || ga[op].y_scale || ga[op].router_Wr) return 1;
    GemvPlan plan;
    if (af_plan_gemv_f16(ctx, ga[op], true, &plan) != AF_OK) return 1;  // the per-operator path reports it
    if (plan.nw != LAYER_WAVES || plan.tiles * plan.S > ctx->n_cu) return 1;
    P.g[op] = plan.p;
    P.tiles[op] = plan.tiles;
    P.S[op] = plan.S;
    P.lx[op] = plan.lx;
    if ((op == 1 || op == 3) && plan.lx != 16) return 1;  // the tile shapes the kernel is built for
    if (plan.lds > lds) lds = plan.lds;
    if (plan.tiles * plan.S > n_wg) n_wg = plan.tiles * plan.S;
  }
  if (lds > AF_GEMV_LDS_BUDGET) return 1;
  int KS = (kv_len + 63) / 64;
  if (KS < 1) KS = 1;
  if (KS > 64) KS = 64;
  if (KS > ctx->n_cu / cfg->n_heads) KS = ctx->n_cu / cfg->n_heads;
  while ((size_t)cfg->n_heads * KS * (cfg->head_dim + 2) > ctx->lay.attn_floats && KS > 1) --KS;
  if ((kv_len + KS - 1) / KS > LAYER_ATT_MAX_KEYS) return 1;
  if (cfg->n_heads * KS > n_wg) n_wg = cfg->n_heads * KS;
  int* counters = (int*)(ctx->ws + ctx->lay.tickets);
  P.done = counters + AF_TICKET_PHASE;
  P.err = counters + AF_TICKET_ERR;
  P.KS = KS;
  AttnParams& a = P.at;
  a.qkv = qkv;
  a.k_cache = (half_t*)kc;
  a.v_cache = (half_t*)vc;
  a.out = attn;
  a.part = (float*)(ctx->ws + ctx->lay.attn_part);
  a.tickets = counters + AF_TICKET_ATTN;
  a.n_heads = cfg->n_heads;
  a.n_kv = cfg->n_kv_heads;
  a.kv_len = kv_len;
  a.kv_cap = kv_cap;
  a.head_dim = cfg->head_dim;
  for (int i = 0; i < cfg->head_dim / 2; ++i) {
    const double ang = (double)pos * pow((double)cfg->rope_theta, -2.0 * (double)i / (double)cfg->head_dim);
    a.cs[i] = (float)cos(ang);
    a.sn[i] = (float)sin(ang);
  }
  // phase counters: qkv 0, attention 1, o 2, gate|up 3, down 4 (time stamps in the same order)
  const int phase_of[4] = {0, 2, 3, 4};
  for (int op = 0; op < 4; ++op) {
    const int ph = phase_of[op];
    P.g[op].done = P.done + ph;
    P.g[op].done_total = P.tiles[op];
    P.g[op].flags |= (ph > 0 ? GEMV_F_DONE_PREV : 0) | (ph == 4 ? GEMV_F_DONE_LAST : 0);
  }
  P.g[0].prof = af_prof_take(ctx);
  a.prof = af_prof_take(ctx);
  for (int op = 1; op < 4; ++op) P.g[op].prof = af_prof_take(ctx);
  if (P.lx[0] == 16 && P.lx[2] == 16)
    hipLaunchKernelGGL((layer_f16_kernel<16, 16>), dim3(n_wg), dim3(LAYER_THREADS), lds, ctx->stream, P);
  else if (P.lx[0] == 16 && P.lx[2] == 64)
    hipLaunchKernelGGL((layer_f16_kernel<16, 64>), dim3(n_wg), dim3(LAYER_THREADS), lds, ctx->stream, P);
  else if (P.lx[0] == 32 && P.lx[2] == 64)
    hipLaunchKernelGGL((layer_f16_kernel<32, 64>), dim3(n_wg), dim3(LAYER_THREADS), lds, ctx->stream, P);
  else
    return 1;
  AF_LAUNCH_CHECK();
  return AF_OK;
}

// One layer.  `own` receives the sets of the selecting points named in write_sets; `src`
// provides the sets of points whose bit is set in reuse (own == src unless the layer follows
// a group leader).
static int run_layer(af_ctx* ctx, const af_layer_cfg* cfg, const af_layer_weights* w,
                     const half_t* h_in, half_t* h_out, void* kc, void* vc, int kv_len,
                     int kv_cap, int pos, const af_select_cfg* sel, unsigned reuse,
                     unsigned write_sets, const af_idx_sets* own, const af_idx_sets* src) {
  const int d = cfg->d_model, f = cfg->d_ffn, hd = cfg->head_dim;
  const int qdim = cfg->n_heads * hd, qkv_out = (cfg->n_heads + 2 * cfg->n_kv_heads) * hd;
  half_t* act[7];
  for (int i = 0; i < 7; ++i) act[i] = (half_t*)(ctx->ws + ctx->lay.act[i]);
  half_t *x0 = act[0], *qkv = act[1], *attn = act[2], *hmid = act[3], *x2 = act[4], *gu = act[5],
         *x3 = act[6];
  const bool q4 = cfg->weight_kind != AF_W_F16;
  int rc;

  struct Point {
    const int32_t* idx;
    int nidx_host;
    const int32_t* nidx_dev;
  } pt[4];
  const int widths[4] = {d, qdim, d, f};
  for (int p = 0; p < 4; ++p) {
    const bool reused = (reuse >> p) & 1u;
    const af_idx_sets* ss = reused ? src : own;
    if (!reused && (sel->mode == AF_SEL_DENSE || !((write_sets >> p) & 1u))) {
      pt[p] = {nullptr, widths[p], nullptr};  // not read: the point is dense or selects for itself
    } else if (sel->mode == AF_SEL_TOPK) {
      pt[p] = {ss->idx[p], sel->k[p], nullptr};
    } else {  // threshold, or a reused set under dense/threshold: the count lives on the device
      pt[p] = {ss->idx[p], widths[p], ss->count[p]};
    }
  }

  // GEMV at selection point p.  fused: the kernel builds x from `src_v` (producer) and selects
  // for itself; otherwise x is ready in `x` and the rows come from pt[p].
  auto make = [&](int p, const void* W, const void* Sc, int in, int out, int producer,
                  const half_t* src_v, const half_t* gain, half_t* x, half_t* y,
                  const half_t* res) -> af_gemv_args {
    af_gemv_args a{};
    a.W = W;
    a.scales = (const half_t*)Sc;
    a.q4_channel_local = cfg->weight_kind == AF_W_Q4CL;
    a.in = in;
    a.out = out;
    a.ld = out;
    a.y = y;
    a.y_kind = AF_F16;
    a.residual = res;
    af_row_src& r = a.rows;
    r.n = in;
    r.eps = cfg->rms_eps;
    const bool reused = (reuse >> p) & 1u;
    const bool selects = !reused && sel->mode != AF_SEL_DENSE;
    r.pro = producer;
    r.src = src_v;
    r.gain = gain;
    r.x_out = x;
    if (selects) {
      r.sel = sel->mode;
      r.k = sel->k[p];
      r.t = sel->t[p];
      if ((write_sets >> p) & 1u) {
        r.idx_out = own->idx[p];
        r.count_out = own->count[p];
      }
    } else {
      r.sel = AF_ROWS_GIVEN;
      r.idx = pt[p].idx;
      r.nidx_host = pt[p].nidx_host;
      r.nidx_dev = pt[p].nidx_dev;
    }
    return a;
  };
  const af_gemv_args ga[4] = {
      make(0, w->Wqkv, w->Sqkv, d, qkv_out, AF_PRO_RMSNORM, h_in, (const half_t*)w->g_attn_norm, x0, qkv, nullptr),
      make(1, w->Wo, w->So, qdim, d, AF_PRO_NONE, attn, nullptr, nullptr, hmid, h_in),
      make(2, w->Wgateup, w->Sgateup, d, 2 * f, AF_PRO_RMSNORM, hmid, (const half_t*)w->g_ffn_norm, x2, gu, nullptr),
      make(3, w->Wdown, w->Sdown, f, d, AF_PRO_SILUMUL, gu, nullptr, x3, h_out, hmid)};
  if (!q4) {
    rc = launch_layer_kernel(ctx, cfg, ga, qkv, kc, vc, kv_len, kv_cap, pos, attn);
    if (rc != 1) return rc;
  }
  auto gemv = [&](const af_gemv_args& a) { return q4 ? af_launch_gemv_q4(ctx, a) : af_launch_gemv_f16(ctx, a); };
  if ((rc = gemv(ga[0]))) return rc;
  if ((rc = af_launch_attention(ctx, cfg, qkv, kc, vc, kv_len, kv_cap, pos, attn))) return rc;
  if ((rc = gemv(ga[1]))) return rc;
  if ((rc = gemv(ga[2]))) return rc;
  if ((rc = gemv(ga[3]))) return rc;
  return AF_OK;
}

static int check_layer_ptrs(const af_layer_cfg* cfg, const af_layer_weights* w,
                            const af_select_cfg* sel, unsigned reuse, unsigned write_sets,
                            const af_idx_sets* own, const af_idx_sets* src) {
  if (!w->Wqkv || !w->Wo || !w->Wgateup || !w->Wdown || !w->g_attn_norm || !w->g_ffn_norm)
    return AF_ENULL;
  if (cfg->weight_kind != AF_W_F16 && (!w->Sqkv || !w->So || !w->Sgateup || !w->Sdown))
    return AF_ENULL;
  for (int p = 0; p < 4; ++p) {
    const bool reused = (reuse >> p) & 1u;
    if (!reused && (sel->mode == AF_SEL_DENSE || !((write_sets >> p) & 1u))) continue;
    const af_idx_sets* ss = reused ? src : own;
    if (!ss || !ss->idx[p]) return AF_ENULL;
    if (sel->mode != AF_SEL_TOPK && !ss->count[p]) return AF_ENULL;
  }
  return AF_OK;
}

extern "C" int af_decode_layer(af_ctx* ctx, const af_layer_cfg* cfg, const af_layer_weights* w,
                               const void* hidden_in, void* hidden_out, void* k_cache,
                               void* v_cache, int kv_len, int kv_cap, int pos,
                               const af_select_cfg* sel, af_idx_sets* sets) {
  if (!ctx || !cfg || !w || !hidden_in || !hidden_out || !k_cache || !v_cache || !sel)
    return AF_ENULL;
  int rc = check_layer_args(ctx, cfg, sel, kv_len, kv_cap, pos);
  if (rc) return rc;
  static const af_idx_sets none = {};
  const unsigned write_sets = (sel->flags & AF_SEL_SKIP_SETS) ? 0u : 15u;
  const af_idx_sets* ss = sets ? sets : &none;
  if ((rc = check_layer_ptrs(cfg, w, sel, sel->reuse_mask & 15u, write_sets, ss, ss))) return rc;
  return run_layer(ctx, cfg, w, (const half_t*)hidden_in, (half_t*)hidden_out, k_cache, v_cache,
                   kv_len, kv_cap, pos, sel, sel->reuse_mask & 15u, write_sets, ss, ss);
}

// Points of layer l whose freshly selected sets have to reach memory: all of them, unless the
// configuration asks to skip sets nobody reads; then only what a follower of l reuses.
static unsigned stack_write_sets(const af_select_cfg* sel, int l, int n_layers, int group,
                                 unsigned reuse_points) {
  if (!(sel->flags & AF_SEL_SKIP_SETS)) return 15u;
  const bool leader_with_followers = group > 1 && (l % group) == 0 && l + 1 < n_layers;
  return leader_with_followers ? (reuse_points & 15u) : 0u;
}

extern "C" int af_decode_stack(af_ctx* ctx, const af_layer_cfg* cfg, const af_layer_weights* w,
                               int n_layers, const void* hidden_in, void* hidden_out,
                               void* const* k_caches, void* const* v_caches, int kv_len,
                               int kv_cap, int pos, const af_select_cfg* sel, int n_sel, int group,
                               unsigned reuse_points, af_idx_sets* sets) {
  if (!ctx || !cfg || !w || !hidden_in || !hidden_out || !k_caches || !v_caches || !sel)
    return AF_ENULL;
  if (n_layers <= 0 || group < 1) return AF_EINVAL;
  if (n_sel != 1 && n_sel != n_layers) return AF_EINVAL;
  static const af_idx_sets none = {};
  int rc;
  // validate every layer before the first launch
  for (int l = 0; l < n_layers; ++l) {
    const af_select_cfg* sl = &sel[n_sel == 1 ? 0 : l];
    if ((rc = check_layer_args(ctx, cfg, sl, kv_len, kv_cap, pos))) return rc;
    if (!k_caches[l] || !v_caches[l]) return AF_ENULL;
    const bool follower = group > 1 && (l % group) != 0;
    const unsigned reuse = (sl->reuse_mask | (follower ? reuse_points : 0u)) & 15u;
    const unsigned write_sets = stack_write_sets(sl, l, n_layers, group, reuse_points);
    const af_idx_sets* own = sets ? &sets[l] : &none;
    const af_idx_sets* src = sets ? &sets[follower ? l - l % group : l] : &none;
    if ((rc = check_layer_ptrs(cfg, &w[l], sl, reuse, write_sets, own, src))) return rc;
  }
  for (int l = 0; l < n_layers; ++l) {
    const af_select_cfg* sl = &sel[n_sel == 1 ? 0 : l];
    const bool follower = group > 1 && (l % group) != 0;
    const unsigned reuse = (sl->reuse_mask | (follower ? reuse_points : 0u)) & 15u;
    const unsigned write_sets = stack_write_sets(sl, l, n_layers, group, reuse_points);
    const af_idx_sets* own = sets ? &sets[l] : &none;
    const af_idx_sets* src = sets ? &sets[follower ? l - l % group : l] : &none;
    const half_t* hin = (const half_t*)(l == 0 ? hidden_in : hidden_out);
    rc = run_layer(ctx, cfg, &w[l], hin, (half_t*)hidden_out, k_caches[l], v_caches[l], kv_len,
                   kv_cap, pos, sl, reuse, write_sets, own, src);
    if (rc) return rc;
  }
  return AF_OK;
}

// ---- mixture-of-experts block ------------------------------------------------------------
#define MOE_THREADS 1024
struct RouterParams {
  af_row_src rows;  // RMSNorm of h_mid: the same x the gate/up GEMV builds
  const half_t* Wr;
  int n_experts, top;
  int32_t* experts;
  float* weights;
  float* logits;
};

// Router of one token: x in LDS, one fp32 dot product per expert (lanes -> waves -> one
// thread, fixed order), then the `top` largest logits and their softmax.
__global__ __launch_bounds__(MOE_THREADS) void moe_router_kernel(RouterParams p) {
  typedef RowPrologue<MOE_THREADS> RP;
  extern __shared__ __align__(16) unsigned short xs[];
  __shared__ typename RP::Smem s_rp;
  __shared__ float s_part[MOE_THREADS / AF_WAVE][AF_MOE_MAX_EXPERTS];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nvec = p.rows.n >> 3;
  half8 zero8;
#pragma unroll
  for (int c = 0; c < 8; ++c) zero8[c] = (half_t)0;
  // the router rows of this thread's first vector do not depend on x: fetch them before x is
  // built, so the two global round trips overlap
  half8 w0[AF_MOE_MAX_EXPERTS];
#pragma unroll
  for (int e = 0; e < AF_MOE_MAX_EXPERTS; ++e)
    w0[e] = (e < p.n_experts && tid < nvec)
                ? *reinterpret_cast<const half8*>(p.Wr + (size_t)e * p.rows.n + (size_t)tid * 8)
                : zero8;
  RP::produce(p.rows, xs, s_rp, false, 0, 1);
  const half8* xv = reinterpret_cast<const half8*>(xs);
  float acc[AF_MOE_MAX_EXPERTS];
#pragma unroll
  for (int e = 0; e < AF_MOE_MAX_EXPERTS; ++e) acc[e] = 0.f;
  if (tid < nvec) {
    const half8 x8 = xv[tid];
#pragma unroll
    for (int e = 0; e < AF_MOE_MAX_EXPERTS; ++e)
#pragma unroll
      for (int c = 0; c < 8; ++c) acc[e] += (float)w0[e][c] * (float)x8[c];
  }
  for (int v = tid + MOE_THREADS; v < nvec; v += MOE_THREADS) {  // inputs wider than 8192
    const half8 x8 = xv[v];
#pragma unroll
    for (int e = 0; e < AF_MOE_MAX_EXPERTS; ++e) {
      if (e < p.n_experts) {
        const half8 w8 = *reinterpret_cast<const half8*>(p.Wr + (size_t)e * p.rows.n + (size_t)v * 8);
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[e] += (float)w8[c] * (float)x8[c];
      }
    }
  }
#pragma unroll
  for (int e = 0; e < AF_MOE_MAX_EXPERTS; ++e) {
    const float t = af_wave_sum(acc[e]);
    if (lane == 0) s_part[wave][e] = t;
  }
  __syncthreads();
  if (tid >= AF_WAVE) return;
  // lane e adds the wave sums of expert e in wave order; thread 0 then picks
  __shared__ float s_logit[AF_MOE_MAX_EXPERTS];
  if (lane < p.n_experts) {
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < MOE_THREADS / AF_WAVE; ++w) t += s_part[w][lane];
    s_logit[lane] = t;
    p.logits[lane] = t;
  }
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  if (tid != 0) return;
  const float* logit = s_logit;  // indexed at run time: stays in LDS
  int chosen[AF_MOE_MAX_TOP];
  float z[AF_MOE_MAX_TOP];
  unsigned taken = 0;
  for (int s = 0; s < p.top; ++s) {  // largest remaining logit, ties to the lower expert
    int best = -1;
    for (int e = 0; e < p.n_experts; ++e)
      if (!((taken >> e) & 1u) && (best < 0 || logit[e] > logit[best])) best = e;
    taken |= 1u << best;
    chosen[s] = best;
    z[s] = logit[best];
  }
  float den = 0.f;
  for (int s = 0; s < p.top; ++s) {
    z[s] = expf(z[s] - logit[chosen[0]]);
    den += z[s];
  }
  for (int s = 0; s < p.top; ++s) {
    p.experts[s] = chosen[s];
    p.weights[s] = z[s] / den;
  }
}

extern "C" int af_decode_moe_layer(af_ctx* ctx, const af_moe_cfg* mcfg, const af_moe_weights* w,
                                   const void* hidden_in, void* hidden_out, void* k_cache,
                                   void* v_cache, int kv_len, int kv_cap, int pos,
                                   const af_select_cfg* sel, const af_moe_sets* sets,
                                   const af_moe_route* route) {
  if (!ctx || !mcfg || !w || !hidden_in || !hidden_out || !k_cache || !v_cache || !sel || !route)
    return AF_ENULL;
  const af_layer_cfg* cfg = &mcfg->base;
  int rc = check_layer_args(ctx, cfg, sel, kv_len, kv_cap, pos);
  if (rc) return rc;
  const bool q4 = cfg->weight_kind != AF_W_F16;
  const bool cl = cfg->weight_kind == AF_W_Q4CL;
  if (mcfg->n_experts < 1 || mcfg->n_experts > AF_MOE_MAX_EXPERTS) return AF_EINVAL;
  if (mcfg->top < 1 || mcfg->top > AF_MOE_MAX_TOP || mcfg->top > mcfg->n_experts) return AF_EINVAL;
  if (sel->reuse_mask & 15u) return AF_EINVAL;
  if (!w->Wqkv || !w->Wo || !w->g_attn_norm || !w->g_ffn_norm || !w->Wr || !w->Wgateup || !w->Wdown)
    return AF_ENULL;
  if (q4 && (!w->Sqkv || !w->So || !w->Sgateup || !w->Sdown)) return AF_ENULL;
  if (!route->experts || !route->weights || !route->logits) return AF_ENULL;
  const int d = cfg->d_model, f = cfg->d_ffn, hd = cfg->head_dim, top = mcfg->top;
  const int qdim = cfg->n_heads * hd, qkv_out = (cfg->n_heads + 2 * cfg->n_kv_heads) * hd;
  if ((long long)top * 2 * f > ctx->max_out || (long long)top * f > ctx->max_in) return AF_EWORKSPACE;
  const bool selects = sel->mode != AF_SEL_DENSE;
  const bool write_sets = selects && !(sel->flags & AF_SEL_SKIP_SETS);
  if (write_sets) {
    if (!sets) return AF_ENULL;
    for (int p = 0; p < 3 + top; ++p)
      if (!sets->idx[p] || !sets->count[p]) return AF_ENULL;
  }
  half_t* act[7];
  for (int i = 0; i < 7; ++i) act[i] = (half_t*)(ctx->ws + ctx->lay.act[i]);
  half_t *x0 = act[0], *qkv = act[1], *attn = act[2], *hmid = act[3], *x2 = act[4], *gu = act[5],
         *x3 = act[6];
  const half_t* h_in = (const half_t*)hidden_in;
  half_t* h_out = (half_t*)hidden_out;

  // GEMV at selection point `point` (its k / threshold come from sel slot `cfg_p`)
  auto gemv = [&](int point, int cfg_p, af_gemv_args& a, int producer, const half_t* src_v,
                  const half_t* gain, half_t* x) -> int {
    a.y_kind = AF_F16;
    a.q4_channel_local = cl;
    af_row_src& r = a.rows;
    r.n = a.in;
    r.eps = cfg->rms_eps;
    r.pro = producer;
    r.src = src_v;
    r.gain = gain;
    r.x_out = x;
    if (selects) {
      r.sel = sel->mode;
      r.k = sel->k[cfg_p];
      r.t = sel->t[cfg_p];
      if (write_sets) {
        r.idx_out = sets->idx[point];
        r.count_out = sets->count[point];
      }
    } else {
      r.sel = AF_ROWS_GIVEN;
      r.idx = nullptr;
      r.nidx_host = a.in;
    }
    return q4 ? af_launch_gemv_q4(ctx, a) : af_launch_gemv_f16(ctx, a);
  };
  // per-expert strides of a bank [E][in][cols]: fp16 elements, or packed bytes + scale elements
  auto bank = [&](af_gemv_args& a, int in, int cols) {
    if (!q4) {
      a.w_stride = (long long)in * cols;
    } else {
      a.w_stride = (long long)in * (cols / 2);
      a.w_stride_scales = cl ? (long long)in * (cols / 32) : (long long)(in / 32) * cols;
    }
  };

  {
    af_gemv_args a{};
    a.W = w->Wqkv; a.scales = (const half_t*)w->Sqkv; a.in = d; a.out = qkv_out; a.ld = qkv_out; a.y = qkv;
    if ((rc = gemv(0, 0, a, AF_PRO_RMSNORM, h_in, (const half_t*)w->g_attn_norm, x0))) return rc;
  }
  if ((rc = af_launch_attention(ctx, cfg, qkv, k_cache, v_cache, kv_len, kv_cap, pos, attn))) return rc;
  {
    af_gemv_args a{};
    a.W = w->Wo; a.scales = (const half_t*)w->So; a.in = qdim; a.out = d; a.ld = d; a.y = hmid; a.residual = h_in;
    if ((rc = gemv(1, 1, a, AF_PRO_NONE, attn, nullptr, nullptr))) return rc;
  }
  // The router runs inside the gate|up launch when that kernel can take it (up to 8 experts,
  // d <= 8192); otherwise as a launch of its own in front of it.
  const bool fuse_router = mcfg->n_experts <= 8 && d <= 8192 && !ctx->moe_router_kernel;
  if (!fuse_router) {
    RouterParams rp{};
    rp.rows.pro = AF_PRO_RMSNORM;
    rp.rows.src = hmid;
    rp.rows.gain = (const half_t*)w->g_ffn_norm;
    rp.rows.eps = cfg->rms_eps;
    rp.rows.n = d;
    rp.Wr = (const half_t*)w->Wr;
    rp.n_experts = mcfg->n_experts;
    rp.top = top;
    rp.experts = route->experts;
    rp.weights = route->weights;
    rp.logits = route->logits;
    static bool attr_done = false;
    if (!attr_done) {
      attr_done = true;
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(moe_router_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 2 * AF_MAX_N);
    }
    hipLaunchKernelGGL(moe_router_kernel, dim3(1), dim3(MOE_THREADS), af_align((size_t)d * 2, 16),
                       ctx->stream, rp);
    AF_LAUNCH_CHECK();
  }
  {
    af_gemv_args a{};
    a.W = w->Wgateup; a.scales = (const half_t*)w->Sgateup; a.in = d; a.out = top * 2 * f; a.ld = 2 * f; a.y = gu;
    a.w_sel = route->experts; a.n_slots = top;
    bank(a, d, 2 * f);
    if (fuse_router) {
      a.router_Wr = (const half_t*)w->Wr;
      a.router_E = mcfg->n_experts;
      a.router_top = top;
      a.router_experts = route->experts;
      a.router_weights = route->weights;
      a.router_logits = route->logits;
    }
    if ((rc = gemv(2, 2, a, AF_PRO_RMSNORM, hmid, (const half_t*)w->g_ffn_norm, x2))) return rc;
  }
  for (int s = 0; s < top; ++s) {
    af_gemv_args a{};
    a.W = w->Wdown; a.scales = (const half_t*)w->Sdown; a.in = f; a.out = d; a.ld = d; a.y = h_out;
    a.residual = s == 0 ? hmid : h_out;
    a.w_sel = route->experts + s; a.n_slots = 1;
    bank(a, f, d);
    a.y_scale = route->weights + s;
    if ((rc = gemv(3 + s, 3, a, AF_PRO_SILUMUL, gu + (size_t)s * 2 * f, nullptr, x3 + (size_t)s * f)))
      return rc;
  }
  return AF_OK;
}

extern "C" int af_layer_tap(af_ctx* ctx, int which, const void** dev_ptr) {
  if (!ctx || !dev_ptr) return AF_ENULL;
  if (which < 0 || which > 6) return AF_EINVAL;
  if (!ctx->ws) return AF_EWORKSPACE;
  *dev_ptr = ctx->ws + ctx->lay.act[which];
  return AF_OK;
}
