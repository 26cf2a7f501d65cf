// Decoder layer for a small batch of tokens (B <= 8), each with its own KV cache and position:
// the block of Fig. "simplified transformer layer" (Section 2.2) with operations T and C of
// Section 4 in front of every linear operator, where operation C runs ONCE over the union of the
// tokens' active sets (union.hip) instead of once per token.  The paper decodes one token at a
// time; this is the batched extension of the same layer: every token's result is what the
// single-token layer gives for that token alone.
//
// Per selection point: one launch of B workgroups builds each token's operator input (RMSNorm,
// copy, or SiLU(gate)*up), selects on it (the front end of row_prologue.h, one workgroup per
// token) and sets the token's bit in the channel mask for every channel it keeps; one launch
// turns the mask into the union and the masked token values; one launch streams the union's
// weight rows for all tokens.  Attention is one launch over (head, key split, token); each token has its own cache,
// length and position.
#include <math.h>

#include "af_internal.h"
#include "row_prologue.h"

#define BS_THREADS 1024

struct BatchSelectParams {
  af_row_src r;          // token 0; token b lies the strides below further
  long long src_stride;  // elements between the tokens' sources
  long long x_stride;    // ... their produced inputs (x_out)
  long long idx_stride;  // ... their index lists
  unsigned* mask;        // [n] channel mask of the union builder (bit b: token b keeps the channel)
};

__global__ __launch_bounds__(BS_THREADS) void batch_select_kernel(BatchSelectParams p) {
  typedef RowPrologue<BS_THREADS> RP;
  extern __shared__ __align__(16) unsigned short xs[];
  __shared__ __align__(16) unsigned s_scratch[RP_SCRATCH_WORDS];
  __shared__ typename RP::Smem s_rp;
  af_row_src r = p.r;
  const int b = blockIdx.x;
  r.src += (size_t)b * p.src_stride;
  if (r.x_out) r.x_out += (size_t)b * p.x_stride;
  r.idx_out += (size_t)b * p.idx_stride;
  r.count_out += b;
  const bool topk = r.sel == AF_SEL_TOPK;
  RP::produce(r, xs, s_rp, true, 0, 1, topk ? s_scratch : nullptr);
  int nidx;
  RP::select_split(r, xs, s_scratch, s_rp, nullptr, 1, 0, true, true, &nidx, topk);
  // the list just written (its stores were waited for at the barrier that ends the selection),
  // read back past the CU's cache: every kept channel gets this token's bit
  for (int i0 = threadIdx.x; i0 < nidx; i0 += 8 * BS_THREADS) {
    int j[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int i = i0 + u * BS_THREADS;
      j[u] = i < nidx ? __hip_atomic_load(r.idx_out + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : -1;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if ((unsigned)j[u] < (unsigned)r.n)
        __hip_atomic_fetch_or(p.mask + j[u], 1u << b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

static int launch_batch_select(af_ctx* ctx, int B, int producer, const half_t* src, long long src_stride,
                               const half_t* gain, float eps, int n, const af_select_cfg* sel, int point,
                               half_t* x_out, int32_t* idx_out, int32_t* count_out) {
  static bool attr_done = false;
  if (!attr_done) {  // the vector can need more dynamic LDS than the 64 KB a kernel gets by default
    attr_done = true;
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(batch_select_kernel),
                              hipFuncAttributeMaxDynamicSharedMemorySize, 2 * AF_MAX_N);
  }
  BatchSelectParams p{};
  af_row_src& r = p.r;
  r.pro = producer;
  r.src = src;
  r.gain = gain;
  r.eps = eps;
  r.x_out = x_out;
  r.n = n;
  r.sel = sel->mode;
  r.k = sel->k[point];
  r.t = sel->t[point];
  r.idx_out = idx_out;
  r.count_out = count_out;
  p.src_stride = src_stride;
  p.x_stride = n;
  p.idx_stride = n;
  p.mask = (unsigned*)(ctx->ws + ctx->lay.union_mask);
  const size_t lds = af_align((size_t)n * 2, 16);
  hipLaunchKernelGGL(batch_select_kernel, dim3(B), dim3(BS_THREADS), lds, ctx->stream, p);
  AF_LAUNCH_CHECK();
  return AF_OK;
}

extern "C" int af_decode_layer_batch(af_ctx* ctx, const af_layer_cfg* cfg, const af_layer_weights* w,
                                     int B, const void* hidden_in, void* hidden_out,
                                     void* const* k_caches, void* const* v_caches, const int* kv_len,
                                     int kv_cap, const int* pos, const af_select_cfg* sel,
                                     af_idx_sets* sets, int32_t* union_n) {
  if (!ctx || !cfg || !w || !hidden_in || !hidden_out || !k_caches || !v_caches || !kv_len || !pos ||
      !sel || !sets)
    return AF_ENULL;
  if (B < 1 || B > AF_MAX_BATCH) return AF_EINVAL;
  if (cfg->d_model <= 0 || cfg->n_heads <= 0 || cfg->n_kv_heads <= 0 || cfg->d_ffn <= 0) return AF_EINVAL;
  if (cfg->head_dim != 128 && cfg->head_dim != 64) return AF_ESHAPE;
  if (cfg->n_heads % cfg->n_kv_heads || cfg->d_model % 8 || cfg->d_ffn % 8) return AF_ESHAPE;
  if (cfg->n_heads > AF_TICKET_PHASE - AF_TICKET_ATTN) return AF_ESHAPE;
  if (cfg->weight_kind != AF_W_F16) return AF_EINVAL;  // the union GEMV reads fp16 weights
  if (sel->mode != AF_SEL_TOPK && sel->mode != AF_SEL_THRESHOLD) return AF_EINVAL;
  if (sel->reuse_mask) return AF_EINVAL;
  if (!w->Wqkv || !w->Wo || !w->Wgateup || !w->Wdown || !w->g_attn_norm || !w->g_ffn_norm) return AF_ENULL;
  const int d = cfg->d_model, f = cfg->d_ffn, hd = cfg->head_dim;
  const int qdim = cfg->n_heads * hd, qkv_out = (cfg->n_heads + 2 * cfg->n_kv_heads) * hd;
  const int widths[4] = {d, qdim, d, f};
  for (int p = 0; p < 4; ++p) {
    if (widths[p] > AF_MAX_N) return AF_ESHAPE;
    if (!sets->idx[p] || !sets->count[p]) return AF_ENULL;
    if (sel->mode == AF_SEL_TOPK && (sel->k[p] < 0 || sel->k[p] > widths[p])) return AF_EINVAL;
    if (sel->mode == AF_SEL_THRESHOLD && sel->t[p] != sel->t[p]) return AF_EINVAL;
  }
  if (kv_cap <= 0) return AF_EINVAL;
  for (int b = 0; b < B; ++b) {
    if (!k_caches[b] || !v_caches[b]) return AF_ENULL;
    if (kv_len[b] < 0 || kv_len[b] >= kv_cap || pos[b] < 0) return AF_EINVAL;
  }
  if (!ctx->ws) return AF_EWORKSPACE;
  const int max_w = qkv_out > 2 * f ? qkv_out : 2 * f;
  const int max_i = f > qdim ? f : qdim;
  if (max_i > ctx->max_in || d > ctx->max_in || max_w > ctx->max_out || B > ctx->max_batch)
    return AF_EWORKSPACE;

  half_t* act[7];
  for (int i = 0; i < 7; ++i) act[i] = (half_t*)(ctx->ws + ctx->lay.act[i]);
  half_t *x0 = act[0], *qkv = act[1], *attn = act[2], *hmid = act[3], *x2 = act[4], *gu = act[5],
         *x3 = act[6];
  int32_t* un_idx = (int32_t*)(ctx->ws + ctx->lay.union_idx);
  int32_t* un_n = union_n ? union_n : (int32_t*)(ctx->ws + ctx->lay.union_n);
  const half_t* h_in = (const half_t*)hidden_in;
  half_t* h_out = (half_t*)hidden_out;
  int rc;

  // operation C for all tokens over the union of the sets of point p
  auto gemv = [&](int p, const void* W, int in, int out, const half_t* X, half_t* Y,
                  const half_t* residual) {
    af_union_args u{};
    u.Wt = W;
    u.in = in;
    u.out = out;
    u.ld = out;
    u.X = X;
    u.B = B;
    u.idx_b = sets->idx[p];
    u.idx_stride = in;
    u.k = sel->mode == AF_SEL_TOPK ? sel->k[p] : in;
    u.counts = sel->mode == AF_SEL_TOPK ? nullptr : sets->count[p];
    u.union_idx = un_idx;
    u.union_n = un_n + p;
    u.marked = true;        // by the selection launch
    u.Y = Y;
    u.y_kind = AF_F16;
    u.residual = residual;
    return af_launch_union_f16(ctx, u);
  };

  // q | k | v
  if ((rc = launch_batch_select(ctx, B, AF_PRO_RMSNORM, h_in, d, (const half_t*)w->g_attn_norm,
                                cfg->rms_eps, d, sel, 0, x0, sets->idx[0], sets->count[0])))
    return rc;
  if ((rc = gemv(0, w->Wqkv, d, qkv_out, x0, qkv, nullptr))) return rc;
  if ((rc = af_launch_attention_batch(ctx, cfg, B, qkv, qkv_out, k_caches, v_caches, kv_len, kv_cap, pos,
                                      attn, qdim)))
    return rc;
  // o + residual
  if ((rc = launch_batch_select(ctx, B, AF_PRO_NONE, attn, qdim, nullptr, 0.f, qdim, sel, 1, nullptr,
                                sets->idx[1], sets->count[1])))
    return rc;
  if ((rc = gemv(1, w->Wo, qdim, d, attn, hmid, h_in))) return rc;
  // gate | up
  if ((rc = launch_batch_select(ctx, B, AF_PRO_RMSNORM, hmid, d, (const half_t*)w->g_ffn_norm,
                                cfg->rms_eps, d, sel, 2, x2, sets->idx[2], sets->count[2])))
    return rc;
  if ((rc = gemv(2, w->Wgateup, d, 2 * f, x2, gu, nullptr))) return rc;
  // down + residual
  if ((rc = launch_batch_select(ctx, B, AF_PRO_SILUMUL, gu, 2 * f, nullptr, 0.f, f, sel, 3, x3,
                                sets->idx[3], sets->count[3])))
    return rc;
  if ((rc = gemv(3, w->Wdown, f, d, x3, h_out, hmid))) return rc;
  return AF_OK;
}
