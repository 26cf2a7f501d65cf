// Context, workspace, weight packing and graph helpers of the C ABI.
#include <stdlib.h>
#include <string.h>

#include "af_internal.h"

af_ws_layout af_layout(int max_in, int max_out, int max_batch) {
  af_ws_layout L{};
  size_t off = 0;
  L.tickets = off;
  off = af_align(off + sizeof(int) * AF_N_TICKETS);
  // split partials: S * out_pad floats per launch; the launchers shrink S to fit.
  L.partial_floats = (size_t)(1u << 20) + (size_t)4 * max_out * max_batch;
  L.partials = off;
  off = af_align(off + L.partial_floats * sizeof(float));
  L.attn_floats = (size_t)(1u << 18) * (size_t)max_batch;
  L.attn_part = off;
  off = af_align(off + L.attn_floats * sizeof(float));
  const size_t act_halves = (size_t)(max_in > max_out ? max_in : max_out);
  for (int i = 0; i < 7; ++i) {
    L.act[i] = off;
    off = af_align(off + act_halves * sizeof(half_t) * (size_t)max_batch);
  }
  L.union_x = off;
  off = af_align(off + (size_t)max_in * 8 * sizeof(half_t));
  L.union_idx = off;
  off = af_align(off + (size_t)max_in * sizeof(int32_t));
  L.union_n = off;
  off = af_align(off + 4 * sizeof(int32_t));
  L.union_ranges = off;
  off = af_align(off + ((size_t)max_in + 256) * sizeof(int32_t));
  L.union_range_cnt = off;
  off = af_align(off + (AF_MAX_N / 256) * sizeof(int32_t));
  L.union_mask = off;
  off = af_align(off + (size_t)max_in * sizeof(uint32_t));
  L.total = off;
  return L;
}

extern "C" size_t af_workspace_bytes(int max_in, int max_out, int max_batch) {
  if (max_in <= 0 || max_out <= 0 || max_batch <= 0) return 0;
  if (max_in > AF_MAX_N || max_batch > AF_MAX_BATCH) return 0;
  return af_layout(max_in, max_out, max_batch).total;
}

extern "C" int af_create(af_ctx** out, int device, void* hip_stream) {
  if (!out) return AF_ENULL;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || device < 0 || device >= ndev) return AF_EHIP;
  if (hipSetDevice(device) != hipSuccess) return AF_EHIP;
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, device) != hipSuccess) return AF_EHIP;
  af_ctx* c = (af_ctx*)calloc(1, sizeof(af_ctx));
  if (!c) return AF_EINVAL;
  c->device = device;
  c->stream = (hipStream_t)hip_stream;
  c->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  *out = c;
  return AF_OK;
}

extern "C" int af_destroy(af_ctx* ctx) {
  if (!ctx) return AF_ENULL;
  free(ctx);
  return AF_OK;
}

extern "C" int af_set_option(af_ctx* ctx, int option, int value) {
  if (!ctx) return AF_ENULL;
  switch (option) {
    case AF_OPT_LAYER_KERNEL:
      ctx->use_layer_kernel = value ? 1 : 0;
      return AF_OK;
    case AF_OPT_VALIDATE:
      ctx->validate = value ? 1 : 0;
      return AF_OK;
    case AF_OPT_TUNE_LX:
      ctx->tune_lx = value;
      return AF_OK;
    case AF_OPT_TUNE_WAVES:
      ctx->tune_nw = value;
      return AF_OK;
    case AF_OPT_TUNE_SPLIT:
      ctx->tune_split = value;
      return AF_OK;
    case AF_OPT_TUNE_WORKGROUPS:
      ctx->tune_wgs = value;
      return AF_OK;
    case AF_OPT_MOE_ROUTER_KERNEL:
      ctx->moe_router_kernel = value ? 1 : 0;
      return AF_OK;
    case AF_OPT_TUNE_ATTN_SPLITS:
      ctx->tune_attn_splits = value;
      return AF_OK;
    default:
      return AF_EINVAL;
  }
}

// The device error word is part of the workspace; reading it waits for the context's stream.
extern "C" int af_last_device_error(af_ctx* ctx, int* flags, int clear) {
  if (!ctx || !flags) return AF_ENULL;
  if (!ctx->ws) return AF_EWORKSPACE;
  int* word = (int*)(ctx->ws + ctx->lay.tickets) + AF_TICKET_ERR;
  if (hipStreamSynchronize(ctx->stream) != hipSuccess) return AF_EHIP;
  if (hipMemcpy(flags, word, sizeof(int), hipMemcpyDeviceToHost) != hipSuccess) return AF_EHIP;
  if (clear && *flags) {
    const int zero = 0;
    if (hipMemcpy(word, &zero, sizeof(int), hipMemcpyHostToDevice) != hipSuccess) return AF_EHIP;
  }
  return AF_OK;
}

// AF_OPT_VALIDATE: every entry of the list inside [0, n) and larger than the one before it.
__global__ void validate_idx_kernel(const int32_t* idx, int nidx_host, const int32_t* nidx_dev, int n,
                                    int* err) {
  int nidx = nidx_host;
  if (nidx_dev) nidx = min(*nidx_dev, nidx);
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= nidx) return;
  const int j = idx[i];
  const bool bad = (unsigned)j >= (unsigned)n || (i > 0 && idx[i - 1] >= j);
  if (bad) __hip_atomic_fetch_or(err, (int)AF_DEVERR_IDX, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

int af_validate_idx(af_ctx* ctx, const int32_t* idx, int nidx_host, const int32_t* nidx_dev, int n) {
  if (!idx || nidx_host <= 0) return AF_OK;
  if (!ctx->ws) return AF_EWORKSPACE;
  int* err = (int*)(ctx->ws + ctx->lay.tickets) + AF_TICKET_ERR;
  hipLaunchKernelGGL(validate_idx_kernel, dim3((nidx_host + 255) / 256), dim3(256), 0, ctx->stream, idx,
                     nidx_host, nidx_dev, n, err);
  AF_LAUNCH_CHECK();
  return AF_OK;
}

// Device-side inverse of af_pack_q4_g32: one thread per (input channel, column pair).
__global__ __launch_bounds__(256) void unpack_q4_kernel(const unsigned char* packed, const half_t* scales,
                                                        int in, int out, int ld, int col0, signed char* q_out,
                                                        float* w_out) {
  const int pair = blockIdx.x * blockDim.x + threadIdx.x;
  const int j = blockIdx.y;
  if (pair * 2 >= out) return;
  const unsigned char b = packed[(size_t)j * (ld / 2) + col0 / 2 + pair];
  for (int e = 0; e < 2; ++e) {
    const int o = pair * 2 + e;
    const int q = (int)((b >> (4 * e)) & 15u) - 8;
    if (q_out) q_out[(size_t)o * in + j] = (signed char)q;
    if (w_out) w_out[(size_t)o * in + j] = (float)q * (float)scales[(size_t)(j / 32) * ld + col0 + o];
  }
}

extern "C" int af_unpack_q4_g32(af_ctx* ctx, const void* packed, const void* scales_f16, int out, int in,
                                int ld, int col0, void* q_i8, void* w_f32) {
  if (!ctx || !packed || !scales_f16 || (!q_i8 && !w_f32)) return AF_ENULL;
  if (out <= 0 || in <= 0 || col0 < 0) return AF_EINVAL;
  if (in % 32 || out % 8 || col0 % 8 || ld % 8 || col0 + out > ld || in > 65535) return AF_ESHAPE;
  dim3 grid((out / 2 + 255) / 256, in);
  hipLaunchKernelGGL(unpack_q4_kernel, grid, dim3(256), 0, ctx->stream, (const unsigned char*)packed,
                     (const half_t*)scales_f16, in, out, ld, col0, (signed char*)q_i8, (float*)w_f32);
  AF_LAUNCH_CHECK();
  return AF_OK;
}

extern "C" int af_profile_set(af_ctx* ctx, void* dev_stamps, int n_slots) {
  if (!ctx) return AF_ENULL;
  if (dev_stamps != nullptr && n_slots <= 0) return AF_EINVAL;
  if ((uintptr_t)dev_stamps & 7u) return AF_ESHAPE;
  ctx->prof = (long long*)dev_stamps;
  ctx->prof_slots = dev_stamps ? n_slots : 0;
  ctx->prof_next = 0;
  return AF_OK;
}

extern "C" int af_wall_clock_khz(af_ctx* ctx) {
  if (!ctx) return 0;
  int khz = 0;
  if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, ctx->device) != hipSuccess) return 0;
  return khz;
}

extern "C" int af_set_stream(af_ctx* ctx, void* hip_stream) {
  if (!ctx) return AF_ENULL;
  ctx->stream = (hipStream_t)hip_stream;
  return AF_OK;
}

extern "C" const char* af_strerror(int status) {
  switch (status) {
    case AF_OK: return "ok";
    case AF_EINVAL: return "argument out of range";
    case AF_ENULL: return "required pointer is null";
    case AF_ESHAPE: return "dimension violates the layout rules";
    case AF_EWORKSPACE: return "workspace missing or too small";
    case AF_EHIP: return "HIP runtime error";
    case AF_ENOALLOC_LIMIT: return "size beyond the limit of the allocation-free entry point";
    default: return "unknown status";
  }
}

__global__ void fill_int_kernel(int* p, int n, int v) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

extern "C" int af_set_workspace(af_ctx* ctx, void* dev_ptr, size_t bytes, int max_in, int max_out,
                                int max_batch) {
  if (!ctx || !dev_ptr) return AF_ENULL;
  const size_t need = af_workspace_bytes(max_in, max_out, max_batch);
  if (need == 0) return AF_EINVAL;
  if (bytes < need || ((uintptr_t)dev_ptr & 255u)) return AF_EWORKSPACE;
  ctx->ws = (char*)dev_ptr;
  ctx->ws_bytes = bytes;
  ctx->max_in = max_in;
  ctx->max_out = max_out;
  ctx->max_batch = max_batch;
  ctx->lay = af_layout(max_in, max_out, max_batch);
  // a fill kernel rather than a memset node, so the call is also safe under stream capture
  hipLaunchKernelGGL(fill_int_kernel, dim3((AF_N_TICKETS + 255) / 256), dim3(256), 0, ctx->stream,
                     (int*)(ctx->ws + ctx->lay.tickets), (int)AF_N_TICKETS, 0);
  AF_LAUNCH_CHECK();
  // the union builder's channel mask is all zero between calls
  hipLaunchKernelGGL(fill_int_kernel, dim3((max_in + 255) / 256), dim3(256), 0, ctx->stream,
                     (int*)(ctx->ws + ctx->lay.union_mask), max_in, 0);
  AF_LAUNCH_CHECK();
  return AF_OK;
}

// ---- packing -----------------------------------------------------------------------------
// W[out][in] -> Wt[in][ld] at column col0, 32x32 tiles through LDS so both sides coalesce.
__global__ __launch_bounds__(256) void transpose_kernel(const half_t* W, int out, int in, half_t* Wt,
                                                        int ld, int col0) {
  __shared__ half_t tile[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
  const int i0 = blockIdx.x * 32, o0 = blockIdx.y * 32;
  for (int r = ty; r < 32; r += 8) {
    const int o = o0 + r, i = i0 + tx;
    tile[r][tx] = (o < out && i < in) ? W[(size_t)o * in + i] : (half_t)0;
  }
  __syncthreads();
  for (int r = ty; r < 32; r += 8) {
    const int i = i0 + r, o = o0 + tx;
    if (i < in && o < out) Wt[(size_t)i * ld + col0 + o] = tile[tx][r];
  }
}

extern "C" int af_pack_inmajor_f16(af_ctx* ctx, const void* W_f16, int out, int in, void* Wt,
                                   int ld, int col0) {
  if (!ctx || !W_f16 || !Wt) return AF_ENULL;
  if (out <= 0 || in <= 0 || col0 < 0) return AF_EINVAL;
  if (ld % 8 || col0 + out > ld) return AF_ESHAPE;
  dim3 grid((in + 31) / 32, (out + 31) / 32);
  hipLaunchKernelGGL(transpose_kernel, grid, dim3(256), 0, ctx->stream, (const half_t*)W_f16, out,
                     in, (half_t*)Wt, ld, col0);
  AF_LAUNCH_CHECK();
  return AF_OK;
}

// One thread quantises one group (32 input channels) of two neighbouring output columns, so
// it owns whole bytes of the packed rows.
__global__ __launch_bounds__(256) void pack_q4_kernel(const half_t* W, int out, int in,
                                                      unsigned char* packed, half_t* scales, int ld,
                                                      int col0) {
  const int pair = blockIdx.x * blockDim.x + threadIdx.x;  // output column pair
  const int g = blockIdx.y;                                // group along the input dim
  if (pair * 2 >= out) return;
  unsigned char nib[2][32];
  for (int e = 0; e < 2; ++e) {
    const int o = pair * 2 + e;
    const half_t* src = W + (size_t)o * in + (size_t)g * 32;
    float w[32];
    float amax = 0.f;
    for (int i = 0; i < 32; ++i) {
      w[i] = (float)src[i];
      amax = fmaxf(amax, fabsf(w[i]));
    }
    const half_t sh = (half_t)(amax / 7.0f);
    const float s = (float)sh;
    scales[(size_t)g * ld + col0 + o] = sh;
    for (int i = 0; i < 32; ++i) {
      float q = 0.f;
      if (s != 0.f) q = fminf(7.f, fmaxf(-7.f, rintf(w[i] / s)));
      nib[e][i] = (unsigned char)((int)q + 8);
    }
  }
  for (int i = 0; i < 32; ++i)
    packed[((size_t)g * 32 + i) * (ld / 2) + (col0 / 2) + pair] =
        (unsigned char)(nib[0][i] | (nib[1][i] << 4));
}

extern "C" int af_pack_q4_g32(af_ctx* ctx, const void* W_f16, int out, int in, void* packed,
                              void* scales_f16, int ld, int col0) {
  if (!ctx || !W_f16 || !packed || !scales_f16) return AF_ENULL;
  if (out <= 0 || in <= 0 || col0 < 0) return AF_EINVAL;
  if (in % 32 || out % 8 || col0 % 8 || ld % 8 || col0 + out > ld) return AF_ESHAPE;
  dim3 grid((out / 2 + 255) / 256, in / 32);
  hipLaunchKernelGGL(pack_q4_kernel, grid, dim3(256), 0, ctx->stream, (const half_t*)W_f16, out,
                     in, (unsigned char*)packed, (half_t*)scales_f16, ld, col0);
  AF_LAUNCH_CHECK();
  return AF_OK;
}

// Channel-local groups: one thread quantises one (input channel, group of 32 output columns)
// and writes the 16 packed bytes and the one scale of that group.  Consecutive threads take
// consecutive input channels, so the reads of W[o][j] coalesce along j.
__global__ __launch_bounds__(256) void pack_q4_cl_kernel(const half_t* W, int out, int in,
                                                         unsigned char* packed, half_t* scales,
                                                         int ld, int col0) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;  // input channel
  const int g = blockIdx.y;                             // group of 32 output columns
  if (j >= in) return;
  float w[32];
  float amax = 0.f;
  for (int i = 0; i < 32; ++i) {
    w[i] = (float)W[(size_t)(g * 32 + i) * in + j];
    amax = fmaxf(amax, fabsf(w[i]));
  }
  const half_t sh = (half_t)(amax / 7.0f);
  const float s = (float)sh;
  scales[(size_t)j * (ld / 32) + col0 / 32 + g] = sh;
  unsigned char* dst = packed + (size_t)j * (ld / 2) + (col0 + g * 32) / 2;
  for (int i = 0; i < 32; i += 2) {
    int q[2];
    for (int e = 0; e < 2; ++e) {
      float v = 0.f;
      if (s != 0.f) v = fminf(7.f, fmaxf(-7.f, rintf(w[i + e] / s)));
      q[e] = (int)v + 8;
    }
    dst[i / 2] = (unsigned char)(q[0] | (q[1] << 4));
  }
}

extern "C" int af_pack_q4_cl(af_ctx* ctx, const void* W_f16, int out, int in, void* packed,
                             void* scales_f16, int ld, int col0) {
  if (!ctx || !W_f16 || !packed || !scales_f16) return AF_ENULL;
  if (out <= 0 || in <= 0 || col0 < 0) return AF_EINVAL;
  if (out % 32 || col0 % 32 || ld % 32 || col0 + out > ld) return AF_ESHAPE;
  dim3 grid((in + 255) / 256, out / 32);
  hipLaunchKernelGGL(pack_q4_cl_kernel, grid, dim3(256), 0, ctx->stream, (const half_t*)W_f16, out,
                     in, (unsigned char*)packed, (half_t*)scales_f16, ld, col0);
  AF_LAUNCH_CHECK();
  return AF_OK;
}

// ---- bandwidth probe ---------------------------------------------------------------------
typedef float probe_f4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void stream_read_kernel(const probe_f4* __restrict__ p, size_t n16,
                                                          float* sink) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  probe_f4 acc = {0.f, 0.f, 0.f, 0.f};
  for (; i + 7 * stride < n16; i += 8 * stride) {
    probe_f4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = p[i + u * stride];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc += v[u];
  }
  for (; i < n16; i += stride) acc += p[i];
  float s = af_wave_sum(acc.x + acc.y + acc.z + acc.w);
  if (threadIdx.x == 0) sink[blockIdx.x] = s;
}

// Variants of the plain reader: THREADS per workgroup, U 16-byte loads in flight per lane,
// NT = loads marked non-temporal (the data is used once).
template <int THREADS, int U, bool NT>
__global__ __launch_bounds__(THREADS) void stream_read_variant_kernel(const probe_f4* __restrict__ p,
                                                                      size_t n16, float* sink) {
  const size_t stride = (size_t)gridDim.x * THREADS;
  size_t i = (size_t)blockIdx.x * THREADS + threadIdx.x;
  probe_f4 acc = {0.f, 0.f, 0.f, 0.f};
  for (; i + (U - 1) * stride < n16; i += U * stride) {
    probe_f4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = NT ? __builtin_nontemporal_load(p + i + u * stride) : p[i + u * stride];
#pragma unroll
    for (int u = 0; u < U; ++u) acc += v[u];
  }
  for (; i < n16; i += stride) acc += p[i];
  float s = af_wave_sum(acc.x + acc.y + acc.z + acc.w);
  if ((threadIdx.x & 63) == 0) atomicAdd(&sink[blockIdx.x], s);
}

extern "C" int af_probe_stream_read_variant(af_ctx* ctx, const void* dev_ptr, size_t bytes, void* sink_f32,
                                            int wgs_per_cu, int threads, int in_flight, int nontemporal) {
  if (!ctx || !dev_ptr || !sink_f32) return AF_ENULL;
  if (wgs_per_cu < 1 || wgs_per_cu * threads > 8192) return AF_EINVAL;
  if (bytes == 0 || bytes % 16 || ((uintptr_t)dev_ptr & 15u)) return AF_ESHAPE;
  const dim3 grid(ctx->n_cu * wgs_per_cu);
  const probe_f4* p = (const probe_f4*)dev_ptr;
  float* sink = (float*)sink_f32;
  const size_t n16 = bytes / 16;
#define AF_PROBE(T, U, N)                                                                            \
  if (threads == T && in_flight == U && (nontemporal != 0) == N) {                                   \
    hipLaunchKernelGGL((stream_read_variant_kernel<T, U, N>), grid, dim3(T), 0, ctx->stream, p, n16, \
                       sink);                                                                        \
    AF_LAUNCH_CHECK();                                                                               \
    return AF_OK;                                                                                    \
  }
  AF_PROBE(256, 4, false) AF_PROBE(256, 8, false) AF_PROBE(256, 16, false)
  AF_PROBE(1024, 4, false) AF_PROBE(1024, 8, false) AF_PROBE(1024, 16, false)
  AF_PROBE(256, 8, true) AF_PROBE(256, 16, true) AF_PROBE(1024, 8, true) AF_PROBE(1024, 16, true)
#undef AF_PROBE
  return AF_EINVAL;
}

extern "C" int af_probe_sink_floats(af_ctx* ctx) {
  if (!ctx) return 0;
  return ctx->n_cu * 32;
}

extern "C" int af_probe_stream_read(af_ctx* ctx, const void* dev_ptr, size_t bytes, void* sink_f32,
                                    int wgs_per_cu) {
  if (!ctx || !dev_ptr || !sink_f32) return AF_ENULL;
  if (wgs_per_cu < 1 || wgs_per_cu > 32) return AF_EINVAL;
  if (bytes == 0 || bytes % 16 || ((uintptr_t)dev_ptr & 15u)) return AF_ESHAPE;
  hipLaunchKernelGGL(stream_read_kernel, dim3(ctx->n_cu * wgs_per_cu), dim3(256), 0, ctx->stream,
                     (const probe_f4*)dev_ptr, bytes / 16, (float*)sink_f32);
  AF_LAUNCH_CHECK();
  return AF_OK;
}

// ---- graph capture -----------------------------------------------------------------------
extern "C" int af_capture_begin(af_ctx* ctx) {
  if (!ctx) return AF_ENULL;
  if (ctx->stream == nullptr) return AF_EINVAL;  // the default stream cannot be captured
  return af_hip(hipStreamBeginCapture(ctx->stream, hipStreamCaptureModeThreadLocal));
}

extern "C" int af_capture_end(af_ctx* ctx, af_graph** out) {
  if (!ctx || !out) return AF_ENULL;
  hipGraph_t g = nullptr;
  if (hipStreamEndCapture(ctx->stream, &g) != hipSuccess || !g) return AF_EHIP;
  hipGraphExec_t ex = nullptr;
  if (hipGraphInstantiate(&ex, g, nullptr, nullptr, 0) != hipSuccess) {
    (void)hipGraphDestroy(g);
    return AF_EHIP;
  }
  af_graph* r = (af_graph*)calloc(1, sizeof(af_graph));
  if (!r) return AF_EINVAL;
  r->graph = g;
  r->exec = ex;
  *out = r;
  return AF_OK;
}

extern "C" int af_graph_launch(af_ctx* ctx, af_graph* g) {
  if (!ctx || !g) return AF_ENULL;
  return af_hip(hipGraphLaunch(g->exec, ctx->stream));
}

extern "C" int af_graph_destroy(af_graph* g) {
  if (!g) return AF_ENULL;
  (void)hipGraphExecDestroy(g->exec);
  (void)hipGraphDestroy(g->graph);
  free(g);
  return AF_OK;
}
