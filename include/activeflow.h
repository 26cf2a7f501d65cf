/*
 * activeflow.h -- C ABI of the MI355X (gfx950) active-weight decode library.
 *
 * The library implements the compute half of ActiveFlow's active-weight
 * inference (arXiv 2504.08378) for batch-1 decode on one GPU:
 *   T  (Section 4, "Top-K"):     activation -> indices of the active input channels
 *   C  (Section 4, "Computing"): the linear operator over those channels only
 *   Section 3: the index set of one layer reused by the next layers of its group
 * Weights are stored input-channel-major (Section 6, "Flash loading": the
 * matrix is transposed so that reading one channel returns everything that
 * channel needs), so an active channel is one contiguous row in HBM.
 *
 * Conventions (all entry points)
 *   - Every tensor pointer is a DEVICE pointer owned by the caller unless the
 *     argument comment says "host".  The library never frees caller memory
 *     and allocates no device memory of its own; scratch comes from the
 *     caller through af_set_workspace().
 *   - Every call only enqueues work on the context's HIP stream (borrowed from
 *     the caller) and returns; nothing synchronises.  Results are valid once
 *     the caller has synchronised that stream.  Calls on one context must not
 *     overlap on different streams: they share the workspace.
 *   - Return value: AF_OK (0) or a negative af_status.  All argument checks
 *     happen on the host before anything is launched; a failing call has
 *     launched nothing.  af_strerror() names a code.
 *   - fp16 tensors are IEEE binary16; index lists are int32, ascending, unique.
 *   - "in-major" matrix: Wt[in][ld] fp16, row j holds the weights of input
 *     channel j for all outputs (ld >= out, ld % 8 == 0, out % 8 == 0).
 */
#ifndef ACTIVEFLOW_H
#define ACTIVEFLOW_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  AF_OK = 0,
  AF_EINVAL = -1,     /* a scalar argument is out of range                    */
  AF_ENULL = -2,      /* a required pointer is NULL                           */
  AF_ESHAPE = -3,     /* a dimension violates the layout rules stated below   */
  AF_EWORKSPACE = -4, /* no workspace set, or it is too small for this call   */
  AF_EHIP = -5,       /* the HIP runtime reported an error (launch, stream)   */
  AF_ENOALLOC_LIMIT = -6 /* af_sparse_gemv_f16_noalloc: out exceeds AF_NOALLOC_MAX_OUT */
} af_status;

enum { AF_F16 = 0, AF_F32 = 1 };                              /* y_kind            */
enum { AF_W_F16 = 0, AF_W_Q4G32 = 1, AF_W_Q4CL = 2 };          /* weight_kind       */
enum { AF_SEL_TOPK = 0, AF_SEL_THRESHOLD = 1, AF_SEL_DENSE = 2 }; /* selection mode */
enum { AF_MAX_N = 32768, AF_MAX_BATCH = 8 };

typedef struct af_ctx af_ctx; /* opaque */

/* Context. `device` is the HIP device ordinal, `hip_stream` a hipStream_t (may be 0 for
 * the default stream); the stream is borrowed, never destroyed. */
int af_create(af_ctx** out, int device, void* hip_stream);
int af_destroy(af_ctx* ctx);
int af_set_stream(af_ctx* ctx, void* hip_stream);
const char* af_strerror(int status);

/* Options of a context.  AF_OPT_LAYER_KERNEL (default 0): with 1, af_decode_layer /
 * af_decode_stack run a layer with fp16 weights as ONE launch whose workgroups (one per compute
 * unit, all resident together) go through the five operators and hand results on through
 * memory and counters in the workspace, instead of one launch per operator.  Both give the same
 * results; on the hardware measured the single launch is the slower of the two (a counter
 * hand-off costs what a kernel boundary costs in a replayed graph), which is why it is off by
 * default.  It needs the GPU to itself for its duration (another kernel that occupies compute
 * units only delays it); configurations it does not cover (4-bit weights, more heads than
 * compute units, very long caches) take the per-operator path by themselves. */
/* AF_OPT_VALIDATE (default 0): with 1, every entry point that takes an index list from the caller
 * (af_sparse_gemv_f16 / _q4 / _q4_cl, af_sparse_gemv_union_f16) first queues a check of the
 * list's precondition (entries ascending, unique, inside [0, in)) on the stream; a violation
 * sets AF_DEVERR_IDX in the device error word (af_last_device_error).  Independently of this
 * option no kernel ever follows an index outside [0, in): such an entry contributes nothing to
 * the result and sets the same bit.  A list that is in range but unsorted or repeated is only
 * detected in validate mode; the GEMV then adds a repeated row twice.
 * AF_OPT_TUNE_*: launch-shape overrides for tuning sweeps, 0 = the built-in choice: lanes across
 * a tile (16, 32, 64), waves per workgroup (4, 8, 16), splits of the row list, workgroups
 * aimed at; AF_OPT_TUNE_ATTN_SPLITS: key splits of the attention launch (0 = one per 64 keys).
 * AF_OPT_MOE_ROUTER_KERNEL: 1 runs the router of af_decode_moe_layer as a launch of
 * its own instead of inside the gate|up launch. */
enum {
  AF_OPT_LAYER_KERNEL = 1,
  AF_OPT_VALIDATE = 2,
  AF_OPT_TUNE_LX = 3,
  AF_OPT_TUNE_WAVES = 4,
  AF_OPT_TUNE_SPLIT = 5,
  AF_OPT_TUNE_WORKGROUPS = 6,
  AF_OPT_MOE_ROUTER_KERNEL = 7,
  AF_OPT_TUNE_ATTN_SPLITS = 8
};
int af_set_option(af_ctx* ctx, int option, int value);

/* Device error word of the context's workspace (host call; waits for the context's stream):
 * *flags receives the OR of AF_DEVERR_* bits set by kernels since the word was last cleared;
 * clear != 0 resets it.  AF_DEVERR_SPIN: a bounded wait inside the single-launch layer kernel
 * ran out (its results are invalid; set the workspace again before further calls).
 * AF_DEVERR_IDX: an index list broke its precondition (see af_set_validate). */
enum { AF_DEVERR_SPIN = 1, AF_DEVERR_IDX = 2 };
int af_last_device_error(af_ctx* ctx, int* flags, int clear);

/* Scratch memory.  af_workspace_bytes() gives the size that serves every call whose
 * dimensions stay within max_in input channels, max_out output columns (of the widest
 * fused matrix) and max_batch tokens; 0 if an argument is invalid.
 * af_set_workspace() hands the buffer over for those limits (256-byte aligned, at least
 * af_workspace_bytes() long; the caller keeps ownership and must keep it alive while the
 * context uses it) and enqueues the clearing of its counter areas on the stream (they stay
 * cleared between calls: a call that is not allowed to finish leaves them undefined, set the
 * workspace again then).  Later calls whose dimensions exceed the limits return AF_EWORKSPACE. */
size_t af_workspace_bytes(int max_in, int max_out, int max_batch);
int af_set_workspace(af_ctx* ctx, void* dev_ptr, size_t bytes, int max_in, int max_out,
                     int max_batch);

/* ---- selection: Section 2.1 (Top-K sparsity) and Section 4, operation T ----------------
 * af_select_topk: idx[0..k) = the k channels of largest |x_j|, ascending.  Magnitude order
 *   is the integer order of the fp16 bits with the sign cleared (+0 == -0, Inf above all
 *   finite values, NaN above Inf); equal magnitudes go to the lower index.
 *   x fp16 [n], 0 <= k <= n <= AF_MAX_N.  k == 0 writes nothing.
 * af_select_threshold: idx = { j : |x_j| > t } (strict, compared in fp32, NaN never
 *   passes), ascending; *count receives the number written.  idx must hold n entries.
 *   This is the form the paper's own index kernel takes (Section 6, "Caching": one
 *   preloaded threshold per sparsity level). */
int af_select_topk(af_ctx* ctx, const void* x_f16, int n, int k, int32_t* idx);
int af_select_threshold(af_ctx* ctx, const void* x_f16, int n, float t, int32_t* idx,
                        int32_t* count);

/* ---- weight layout: Section 6 "Flash loading" (channel-major storage) -------------------
 * af_pack_inmajor_f16: W[out][in] fp16 (row-major, out-major) -> Wt[in][ld] at column
 *   offset col0 (so several operators that share an input can be fused side by side:
 *   q|k|v and gate|up).  Columns outside [col0, col0+out) are left untouched.
 * af_pack_q4_g32: quantise W[out][in] fp16 to 4 bits in groups of 32 consecutive input
 *   channels per output: s = fp16(max|w| / 7), q = clamp(rint(w / s), -7, 7) (fp32
 *   arithmetic, ties to even, s == 0 -> q = 0), nibble = q + 8.
 *   packed u8 [in][ld/2]: byte i of row j = columns 2i (low nibble) and 2i+1 (high);
 *   scales fp16 [in/32][ld].  in % 32 == 0, out % 8 == 0, col0 % 8 == 0, ld % 8 == 0.
 * af_pack_q4_cl: the channel-local arrangement (Section 6: the transposed matrix lets the
 *   read of a channel bring all the scales it needs): the same quantiser with groups of 32
 *   consecutive output columns inside one input channel's row.  packed as above; scales fp16
 *   [in][ld/32].  out % 32 == 0, col0 % 32 == 0, ld % 32 == 0.  The bytes of an inactive
 *   channel, scales included, are never read. */
int af_pack_inmajor_f16(af_ctx* ctx, const void* W_f16, int out, int in, void* Wt, int ld,
                        int col0);
int af_pack_q4_g32(af_ctx* ctx, const void* W_f16, int out, int in, void* packed,
                   void* scales_f16, int ld, int col0);
int af_pack_q4_cl(af_ctx* ctx, const void* W_f16, int out, int in, void* packed,
                  void* scales_f16, int ld, int col0);
/* af_unpack_q4_g32 (for tests): the inverse of af_pack_q4_g32 on the device, which pins the
 * nibble order and the scale indexing the GEMV kernel relies on.  Reads the `out` columns at
 * col0 of packed / scales (layout as above) and writes, in the out-major arrangement of the
 * original matrix, q_i8 [out][in] = nibble - 8 (int8) and / or w_f32 [out][in] = (nibble - 8) *
 * scale of the entry's group, exact in fp32.  Either output may be NULL. */
int af_unpack_q4_g32(af_ctx* ctx, const void* packed, const void* scales_f16, int out, int in,
                     int ld, int col0, void* q_i8, void* w_f32);

/* ---- sparse GEMV: Section 4, operation C -----------------------------------------------
 * y[o] = sum over t < nidx of Wt[idx[t]][o] * x[idx[t]]  (+ residual[o] if given),
 * fp32 accumulation, o in [0, out).  Only the rows named by idx are read.
 *   idx == NULL means all channels 0..in-1 (dense).  Otherwise idx holds nidx entries
 *   (ascending, unique, in [0, in) -- a precondition; see AF_OPT_VALIDATE for what happens to
 *   a list that breaks it); nidx is *nidx_dev if
 *   nidx_dev != NULL (a device int32 written by af_select_threshold, must be <= nidx_host)
 *   else nidx_host.  nidx == 0 gives y = residual (or 0).
 *   y: fp16 or fp32 [out] by y_kind; residual: fp16 [out] or NULL; y may alias residual.
 * The result is deterministic: partial sums are combined in a fixed order.
 * af_sparse_gemv_q4: same with W = (nibble - 8) * scale of the row's group (layout of
 *   af_pack_q4_g32); af_sparse_gemv_q4_cl: layout of af_pack_q4_cl. */
int af_sparse_gemv_f16(af_ctx* ctx, const void* Wt, int in, int out, int ld, const void* x_f16,
                       const int32_t* idx, int nidx_host, const int32_t* nidx_dev, void* y,
                       int y_kind, const void* residual_f16);
int af_sparse_gemv_q4(af_ctx* ctx, const void* packed, const void* scales_f16, int in, int out,
                      int ld, const void* x_f16, const int32_t* idx, int nidx_host,
                      const int32_t* nidx_dev, void* y, int y_kind, const void* residual_f16);
int af_sparse_gemv_q4_cl(af_ctx* ctx, const void* packed, const void* scales_f16, int in, int out,
                      int ld, const void* x_f16, const int32_t* idx, int nidx_host,
                      const int32_t* nidx_dev, void* y, int y_kind, const void* residual_f16);

/* The same operation for callers that cannot allocate device memory or hand over a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same
 * arguments, same kernels and same results as af_sparse_gemv_f16, but the tickets and split
 * partial sums live in a device array that is part of the library image (about 4.03 MB on every
 * GPU that loads the library, held until the process ends) instead of the workspace, and the
 * call allocates nothing.  The context needs no workspace; its device must be the current HIP
 * device (else AF_EINVAL).  Limits: in <= AF_MAX_N, out <= AF_NOALLOC_MAX_OUT (beyond that:
 * AF_ENOALLOC_LIMIT, nothing launched).  The array keeps the last call's contents; the call
 * clears the counters it needs with a fill kernel on the context's stream before the GEMV.
 * All calls on one GPU share that GPU's array: calls that overlap on one GPU (different streams,
 * different contexts or processes do not matter: the array is per process and GPU) race; issue
 * them on one stream or order them with events.  The first call on a device looks the array's
 * address up (no allocation, no stream work). */
enum { AF_NOALLOC_MAX_OUT = 65536 };
int af_sparse_gemv_f16_noalloc(af_ctx* ctx, const void* Wt, int in, int out, int ld,
                               const void* x_f16, const int32_t* idx, int nidx_host,
                               const int32_t* nidx_dev, void* y, int y_kind,
                               const void* residual_f16);

/* ---- fused front end: operations T and C of Section 4 in one launch --------------------
 * The GEMV kernel builds its own input vector and selects on it, so no activation or index
 * list has to travel through memory between a producer, a selection and the GEMV:
 *   producer AF_PRO_NONE    x = src                      (src fp16 [in])
 *            AF_PRO_RMSNORM x = fp16(src * rsqrt(mean(src^2) + eps) * gain)   (src, gain [in])
 *            AF_PRO_SILUMUL x = fp16(silu(src[j]) * src[in + j])              (src [2*in])
 *   sel_mode AF_SEL_TOPK (k) | AF_SEL_THRESHOLD (t) | AF_SEL_DENSE (all channels)
 *   y = Wt[idx][:]^T x[idx] (+ residual), idx = select(x) as af_select_topk/_threshold define it.
 * Optional outputs (NULL to skip): x_out fp16 [in] the produced vector; idx_out int32 [in]
 * and count_out int32 [1] the index set.  in % 8 == 0; other rules as af_sparse_gemv_f16. */
enum { AF_PRO_NONE = 0, AF_PRO_RMSNORM = 1, AF_PRO_SILUMUL = 2 };
int af_select_gemv_f16(af_ctx* ctx, const void* Wt, int in, int out, int ld, int producer,
                       const void* src_f16, const void* gain_f16, float eps, int sel_mode, int k,
                       float t, void* x_out, int32_t* idx_out, int32_t* count_out, void* y,
                       int y_kind, const void* residual_f16);

/* The same launch over matrices picked on the device (mixture of experts): the out columns
 * are n_slots equal slots; slot s multiplies by the in-major matrix that starts
 * expert_sel[s] * expert_stride elements behind Wt_all (leading dimension ld >= out/n_slots);
 * expert_sel is device memory (written by the router), so no host round trip is needed.
 * All slots share the input vector and its selection.  y_scale (device, one float, or NULL)
 * multiplies the product before the residual is added.  (out / n_slots) % 8 == 0. */
int af_select_gemv_experts_f16(af_ctx* ctx, const void* Wt_all, const int32_t* expert_sel,
                               int n_slots, long long expert_stride, const float* y_scale, int in,
                               int out, int ld, int producer, const void* src_f16,
                               const void* gain_f16, float eps, int sel_mode, int k, float t,
                               void* x_out, int32_t* idx_out, int32_t* count_out, void* y,
                               int y_kind, const void* residual_f16);

/* ---- small-batch union GEMV (extension of operation C to B tokens) ----------------------
 * Each of the B <= AF_MAX_BATCH tokens has its own index set idx_b[b][0..k); the kernel
 * reads every row of the union once and applies each token's mask:
 *   Y[b][o] = sum over j in idx_b[b] of Wt[j][o] * X[b][j].
 * X fp16 [B][in]; idx_b int32 [B][k], every row ascending, unique, inside [0, in) (precondition
 * as for af_sparse_gemv_f16; an entry out of range is dropped and reported, see
 * AF_OPT_VALIDATE); union_idx int32 [in] and union_n int32 [1] receive the ascending union and
 * its size; Y [B][out] fp16 or fp32. */
int af_sparse_gemv_union_f16(af_ctx* ctx, const void* Wt, int in, int out, int ld,
                             const void* X_f16, int B, const int32_t* idx_b, int k,
                             int32_t* union_idx, int32_t* union_n, void* Y, int y_kind);

/* ---- decoder layer: block of Fig. "simplified transformer layer" (Section 2.2) with
 * operations T and C at the inputs of qkv, o, gate/up and down ---------------------------- */
typedef struct {
  int d_model, n_heads, n_kv_heads, head_dim, d_ffn; /* head_dim must be 128 or 64 */
  float rms_eps, rope_theta;
  int weight_kind; /* AF_W_F16 | AF_W_Q4G32 | AF_W_Q4CL */
} af_layer_cfg;

/* In-major, fused: Wqkv [d][(h+2kv)*hd] (q|k|v), Wo [h*hd][d], Wgateup [d][2*ffn]
 * (gate|up), Wdown [ffn][d]; leading dimension == number of columns.  For AF_W_Q4G32 and
 * AF_W_Q4CL the W* pointers are packed nibbles and S* their scales (in the layout of the
 * respective packer); S* are NULL for fp16 weights.
 * g_*: fp16 [d] RMSNorm gains. */
typedef struct {
  const void *Wqkv, *Wo, *Wgateup, *Wdown;
  const void *Sqkv, *So, *Sgateup, *Sdown;
  const void *g_attn_norm, *g_ffn_norm;
} af_layer_weights;

/* Index sets of the four selection points (0 qkv, 1 o, 2 gate/up, 3 down).  idx[p] holds
 * n_p entries (n_p = input width of the point), count[p] one int32; both device memory.
 * A point that selects writes them; a point whose reuse bit is set reads them. */
typedef struct {
  int32_t* idx[4];
  int32_t* count[4];
} af_idx_sets;

typedef struct {
  int mode;            /* AF_SEL_TOPK | AF_SEL_THRESHOLD | AF_SEL_DENSE */
  int k[4];            /* top-k mode: channels kept at each point        */
  float t[4];          /* threshold mode: threshold at each point        */
  unsigned reuse_mask; /* bit p set: do not select at p, use sets (Section 3) */
  unsigned flags;      /* AF_SEL_SKIP_SETS or 0 */
} af_select_cfg;
/* AF_SEL_SKIP_SETS: a selecting point does not write its index set and count (the GEMV uses
 * them on the fly) unless a later layer of the same af_decode_stack call reuses them; `sets`
 * entries that are neither written nor read may then be NULL.  In threshold mode this is the
 * fully fused form: each workgroup of the GEMV compares only the channels of its own range
 * against the threshold (Section 6), and no index list is built for the whole vector. */
enum { AF_SEL_SKIP_SETS = 1 };

/* One batch-1 decode step of one layer.  hidden_in/hidden_out fp16 [d] (may alias).
 * k_cache/v_cache fp16 [n_kv][kv_cap][hd]; the new (rotated) key and the value are
 * written at slot kv_len (< kv_cap) and attention runs over slots 0..kv_len; `pos` is
 * the rotary position.  Inter-operator tensors are fp16. */
int af_decode_layer(af_ctx* ctx, const af_layer_cfg* cfg, const af_layer_weights* w,
                    const void* hidden_in, void* hidden_out, void* k_cache, void* v_cache,
                    int kv_len, int kv_cap, int pos, const af_select_cfg* sel,
                    af_idx_sets* sets);

/* The same layer for a small batch of B <= AF_MAX_BATCH tokens that are decoded together, each
 * with its own KV cache, length and position (small-batch extension of the layer above; the
 * paper decodes one token at a time, Section 2.1).  Every token selects its own active channels
 * at the four points; each linear operator then reads the union of the tokens' sets once
 * (af_sparse_gemv_union_f16) with every token's own mask applied, so token b's result is what
 * af_decode_layer gives for token b alone (up to the order of the fp32 sums).
 * hidden_in / hidden_out: fp16 [B][d_model], device (may be the same buffer).  k_caches,
 * v_caches: HOST arrays of B device pointers, each a cache [n_kv_heads][kv_cap][head_dim] of its
 * own; kv_len, pos: HOST arrays of B ints (kv_len[b] < kv_cap).  sel: one configuration for all
 * tokens, AF_SEL_TOPK or AF_SEL_THRESHOLD, reuse_mask 0.  sets (required): idx[p] int32
 * [B][n_p] (row b = token b's ascending list, n_p = input width of point p), count[p] int32 [B];
 * both are written.  union_n: device int32 [4] that receives the size of the union at each point,
 * or NULL.  fp16 weights only (AF_EINVAL for the 4-bit kinds).  Needs a workspace set for
 * max_batch >= B; afterwards af_layer_tap(which) points at the [B][width] tensor of all tokens. */
int af_decode_layer_batch(af_ctx* ctx, const af_layer_cfg* cfg, const af_layer_weights* w, int B,
                          const void* hidden_in, void* hidden_out, void* const* k_caches,
                          void* const* v_caches, const int* kv_len, int kv_cap, const int* pos,
                          const af_select_cfg* sel, af_idx_sets* sets, int32_t* union_n);

/* n_layers layers in sequence.  w, k_caches, v_caches, sets: host arrays of n_layers
 * entries.  With group > 1, layer l with l % group != 0 reuses the sets of its group's
 * first layer at the points named by reuse_points (Section 3, N = 4); sets[l] of a
 * follower is not touched at those points.  sel: n_sel configurations, n_sel == 1 (shared by
 * all layers) or n_sel == n_layers (one per layer: calibrated thresholds differ from operator
 * to operator); a configuration's reuse_mask applies on top of the group rule. */
int af_decode_stack(af_ctx* ctx, const af_layer_cfg* cfg, const af_layer_weights* w, int n_layers,
                    const void* hidden_in, void* hidden_out, void* const* k_caches,
                    void* const* v_caches, int kv_len, int kv_cap, int pos,
                    const af_select_cfg* sel, int n_sel, int group, unsigned reuse_points,
                    af_idx_sets* sets);

/* ---- mixture-of-experts block (the Mixtral-8x7B deployment reported in Sections 1 and 7):
 * the feed-forward half is n_experts experts of width d_ffn, of which a router picks `top`
 * per token.  The paper gives no MoE-specific rule; the dense block's rules are carried over:
 * operations T and C sit in front of every linear operator; the normed input is shared by the
 * router (dense: it is tiny) and by the gate/up projections of all chosen experts, so one
 * selection (point 2) serves them all; every chosen expert's down projection selects on its
 * own silu(gate)*up with sel->k[3] / sel->t[3].  Router: logits = Wr x in fp32, the `top`
 * largest (ties to the lower expert), slot 0 the largest; weights = softmax over the chosen
 * logits.  hidden <- fp16(hidden + weight_s * down_s(...)), one slot after the other.
 * The experts are reached on the device (no host round trip): the call can be captured. */
enum { AF_MOE_MAX_EXPERTS = 16, AF_MOE_MAX_TOP = 4 };
typedef struct {
  af_layer_cfg base; /* d_ffn: width of one expert */
  int n_experts, top;
} af_moe_cfg;
/* Wqkv, Wo, g_*: as af_layer_weights.  Wr fp16 [n_experts][d] (one row per expert).
 * Wgateup [n_experts][d][2*ffn]: expert e's in-major gate|up matrix behind expert e-1's;
 * Wdown [n_experts][ffn][d] likewise.  For 4-bit weight kinds W* are packed nibbles and S*
 * their scales, every expert's matrix packed on its own (af_pack_q4_g32 / af_pack_q4_cl with
 * ld = the matrix's own width) and the banks stored expert after expert; S* are NULL for fp16. */
typedef struct {
  const void *Wqkv, *Wo, *g_attn_norm, *g_ffn_norm;
  const void *Wr, *Wgateup, *Wdown;
  const void *Sqkv, *So, *Sgateup, *Sdown;
} af_moe_weights;
/* Index sets: points 0 qkv, 1 o, 2 gate/up (shared by the chosen experts), 3+s the down
 * projection of slot s.  Written unless sel->flags has AF_SEL_SKIP_SETS (then they may be
 * NULL).  idx[p] holds as many entries as the point has input channels. */
typedef struct {
  int32_t* idx[3 + AF_MOE_MAX_TOP];
  int32_t* count[3 + AF_MOE_MAX_TOP];
} af_moe_sets;
/* Router results of the call (device memory, all required): experts int32 [top] in slot
 * order, weights fp32 [top], logits fp32 [n_experts]. */
typedef struct {
  int32_t* experts;
  float* weights;
  float* logits;
} af_moe_route;
/* One batch-1 decode step of such a block; arguments as af_decode_layer.  sel->reuse_mask
 * must be 0.  af_layer_tap afterwards: 5 = gate|up of the chosen experts [top][2*ffn],
 * 6 = x_down [top][ffn]; the workspace limits must cover top*2*ffn outputs. */
int af_decode_moe_layer(af_ctx* ctx, const af_moe_cfg* cfg, const af_moe_weights* w,
                        const void* hidden_in, void* hidden_out, void* k_cache, void* v_cache,
                        int kv_len, int kv_cap, int pos, const af_select_cfg* sel,
                        const af_moe_sets* sets, const af_moe_route* route);

/* Device address of an inter-operator tensor of the most recent af_decode_layer call on
 * this context (for tests): which = 0 x_qkv [d], 1 qkv [(h+2kv)*hd], 2 attn [h*hd],
 * 3 h_mid [d], 4 x_gateup [d], 5 gateup [2*ffn], 6 x_down [ffn].  fp16. */
int af_layer_tap(af_ctx* ctx, int which, const void** dev_ptr);

/* ---- threshold calibration (Section 6, "Caching": the index kernel keeps one activation
 * threshold per sparsity level; the paper does not say how they are found) ----------------
 * Reading built here: pool the magnitudes of a calibration stream of one operator's input
 * vectors in an exact histogram over the 15-bit fp16 magnitude key (NaN left out); for
 * sparsity sp with N pooled values, m = N - floor(sp*N/100) are to be kept and the threshold
 * is the (m+1)-th largest pooled magnitude, so the strict rule |x| > t keeps at most m of
 * them (exactly the pooled top-m when nothing ties with the boundary); m == N gives -1.
 *   af_calib_accumulate        adds the n values of x (device fp16) to hist (device,
 *                              AF_CALIB_BINS uint32 counters, zeroed by the caller before the
 *                              first call; a counter wraps at 2^32).
 *   af_calib_accumulate_layer  adds the four operator inputs of the most recent
 *                              af_decode_layer call on this context (x_qkv, attn, x_gateup,
 *                              x_down) to hist[0..3] (host array of four device pointers).
 *   af_calib_thresholds        writes the thresholds of n_levels <= AF_CALIB_MAX_LEVELS
 *                              sparsity levels (host int array, percent 0..100) to t_out
 *                              (device, n_levels floats; each an fp16 magnitude or -1). */
#define AF_CALIB_BINS 32768
#define AF_CALIB_MAX_LEVELS 16
int af_calib_accumulate(af_ctx* ctx, const void* x_f16, int n, uint32_t* hist);
int af_calib_accumulate_layer(af_ctx* ctx, const af_layer_cfg* cfg, uint32_t* const* hist);
int af_calib_thresholds(af_ctx* ctx, const uint32_t* hist, const int* sparsity_pct, int n_levels,
                        float* t_out);

/* ---- host-side tools (host memory only; no GPU work) --------------------------------------
 * Dynamic weight caching, Section 4.2: one usage counter per channel of a tensor (zero at the
 * start), a cache of at most `capacity` channels.  af_lfu_step takes the ascending, unique
 * channels one token needs: those found in the cache are hits; every needed channel's counter
 * goes up; then the missed channels, in ascending order, enter a free slot, or replace the
 * least-used cached channel the token does not need (ties: lower channel) when their own
 * count is >= that channel's (the paper's worked example fixes >= over the ">" of its text);
 * otherwise they pass by uncached.  evicted (capacity entries, may be NULL) receives the
 * channels that left; hits / loaded / n_evicted may be NULL. */
typedef struct af_lfu af_lfu;
int af_lfu_create(af_lfu** out, int n_channels, int capacity, const int32_t* initial, int n_initial);
int af_lfu_destroy(af_lfu* c);
int af_lfu_step(af_lfu* c, const int32_t* idx, int nidx, int* hits, int* loaded, int32_t* evicted,
                int* n_evicted);
int af_lfu_stats(const af_lfu* c, long long* tokens, long long* needed, long long* hits,
                 long long* evictions);
int af_lfu_cached(const af_lfu* c, int32_t* channels /* capacity entries or NULL */, int* n_cached);

/* Cost model, Section 4.1, Eq. 1-9 as printed (bytes, bytes/s, seconds):
 *   M_cl = S_l (1-sp) N;  T_load = M_cl (1-hr) / bw_flash_small;  T_comp = M_cl / bw_mem;
 *   T_onload = S_l (1-sp)(1-hr)(1-si) / bw_flash_small;  T_preload = M_cl (1-hr) / bw_flash_large;
 *   T_overlap = T_onload + max(T_preload, T_comp);  T_decode = T_load + T_overlap + T_comp;
 *   M = M_cl + M_cache + M_kv.
 * "flash" is whatever tier lies below the memory the GEMVs stream from (on an MI355X: host
 * memory behind the HBM). */
typedef struct {
  double sp, hr, si;
  double bw_mem, bw_flash_small, bw_flash_large;
  double S_l, N, M_cache, M_kv;
} af_cost_in;
typedef struct {
  double M_cl, M, T_load, T_comp, T_onload, T_preload, T_overlap, T_decode;
} af_cost_out;
int af_cost_eval(const af_cost_in* in, af_cost_out* out);

/* Greedy search of Section 4.1: sp = 1 - M_max / S_m (clamped to [0, 1)); N = 1, 2, ... with
 * the cache taking what the budget leaves (M_cache = M_max - M_cl - M_kv) and its hit rate read
 * off the caller's curve at M_cache / (S_m (1-sp)) (n_hr points, ascending fractions, linear in
 * between, flat outside); stops when the budget is exhausted, when T_preload <= T_comp, or when
 * T_preload changed by less than min_gain; returns the visited candidate of lowest T_decode
 * (N == 0: none fits). */
enum { AF_PLAN_MAX_HR = 64 };
typedef struct {
  double M_max, S_m, S_l, M_kv, si;
  double bw_mem, bw_flash_small, bw_flash_large;
  const double* hr_fraction;
  const double* hr_value;
  int n_hr, n_max;
  double min_gain;
} af_plan_in;
typedef struct {
  double sp;
  int N, visited;
  double M_cache, hr;
  af_cost_out cost;
} af_plan_out;
int af_plan_search(const af_plan_in* in, af_plan_out* out);

/* Measurement aid (the Eq. 4 memory-bandwidth term BW_mem of this device): one plain
 * streaming-read kernel over `bytes` of device memory at dev_ptr (16-byte aligned; bytes a
 * multiple of 16) with 16-byte loads, queued on the context's stream, in a grid of
 * wgs_per_cu (1..32) 256-thread workgroups per compute unit.  Every workgroup stores one
 * float fold of what it read to sink_f32 (device, af_probe_sink_floats() floats), so no
 * load can be dropped.  The caller times it with events. */
int af_probe_sink_floats(af_ctx* ctx);
int af_probe_stream_read(af_ctx* ctx, const void* dev_ptr, size_t bytes, void* sink_f32,
                         int wgs_per_cu);
/* Other shapes of the same reader, so that the yardstick does not rest on one of them: threads
 * per workgroup (256 or 1024), 16-byte loads in flight per lane (4, 8, 16; non-temporal: 8, 16),
 * loads marked non-temporal or not; wgs_per_cu * threads <= 8192.  AF_EINVAL for a combination
 * that is not built. */
int af_probe_stream_read_variant(af_ctx* ctx, const void* dev_ptr, size_t bytes, void* sink_f32,
                                 int wgs_per_cu, int threads, int in_flight, int nontemporal);

/* Measurement aid: time stamps of the layer kernels.  While a stamp buffer is set, every kernel
 * that af_decode_layer / af_decode_stack / af_decode_moe_layer and the GEMV entry points launch
 * takes the next free slot, in launch order (slot i = int64 pair dev_stamps[2i], [2i+1]); its
 * workgroups write the earliest kernel entry (atomic min) and the latest exit (atomic max), in
 * ticks of the device's constant-rate wall clock (hipDeviceAttributeWallClockRate, kHz).  A
 * phase of the single-launch layer kernel counts as a kernel.  The caller fills the buffer with
 * INT64_MAX (even entries) and 0 (odd entries) before each run and reads it after
 * synchronising.  Launches beyond n_slots are not stamped.  af_profile_set
 * restarts at slot 0; NULL switches the stamps off.  A captured graph keeps the slots it was
 * recorded with.  dev_stamps: device memory, 8-byte aligned, 2 * n_slots int64. */
int af_profile_set(af_ctx* ctx, void* dev_stamps, int n_slots);
int af_wall_clock_khz(af_ctx* ctx); /* tick rate of those stamps; 0 if unknown */

/* Stream capture helpers: record the calls made between begin and end into a HIP graph
 * and replay it.  The graph holds the pointers and scalars of the recorded calls: a captured
 * decode call is valid for the one (pos, kv_len) and the buffers it was recorded with. */
typedef struct af_graph af_graph;
int af_capture_begin(af_ctx* ctx);
int af_capture_end(af_ctx* ctx, af_graph** out);
int af_graph_launch(af_ctx* ctx, af_graph* g);
int af_graph_destroy(af_graph* g);

#ifdef __cplusplus
}
#endif
#endif /* ACTIVEFLOW_H */
