// Workgroup-local front end of the fused GEMV kernels: produce the operator's input vector in
// LDS (plain copy, RMSNorm, or SiLU(gate)*up) and, when asked, run the activation selection
// (Section 2.1 Top-K sparsity / Section 6 threshold form; Section 4 operation T) right there,
// so that operation T needs no kernel of its own: every workgroup of the GEMV repeats the
// cheap O(n) selection on its own copy of the vector and keeps only its split of the
// ascending index list.  The arithmetic is the same as in select.hip (exact two-digit radix
// select on the 15-bit magnitude key, ties to the lower index).
#pragma once
#include "af_internal.h"

// Replicas of the digit histograms.  Measured 1 / 2 / 4 / 8 / 16 on the synthetic activations:
// 2.360 / 2.364 / 2.367 / 2.378 / 2.411 ms per 7B token (zeroing and merging the replicas cost
// more than the atomic conflicts they avoid); 4 keeps a vector of equal magnitudes, which sends
// every lane to one bin, at a quarter of the serialisation a single table would see.
#ifndef RP_HIST_COPIES
#define RP_HIST_COPIES 4
#endif
#define RP_SCRATCH_WORDS (384 * RP_HIST_COPIES)  // both digit tables; reused by the caller afterwards
// Elements per LDS / global access of the element passes.  With 4 a 4096-wide input gives every
// one of 1024 threads one vector; with 8 half of the threads would idle while the others walk
// twice as many elements one after the other, and those serial walks are what the front end
// spends its time in.
#ifndef RP_EV
#define RP_EV 4
#endif
typedef _Float16 rp_half __attribute__((ext_vector_type(RP_EV)));
typedef unsigned short rp_u16 __attribute__((ext_vector_type(RP_EV)));

template <int THREADS>
struct RowPrologue {
  static constexpr int WAVES = THREADS / AF_WAVE;

  struct Smem {
    unsigned wave_tot[WAVES];
    float red[WAVES];
    unsigned digit, above;
    // router of a mixture-of-experts block run inside the gate|up launch
    float rpart[WAVES][AF_MOE_MAX_EXPERTS];
    float logit[AF_MOE_MAX_EXPERTS];
    int experts[AF_MOE_MAX_TOP];
    float weights[AF_MOE_MAX_TOP];
  };

  // Histogram scratch: RP_HIST_COPIES replicas, replica-major (replica r of bin b at
  // r * 256 + b): lanes of one replica that hit different bins hit different banks, and the
  // merge reads 256 consecutive words per replica.  First 256-bin table at word 0, the
  // 128-bin table of the second digit behind it.
  static constexpr int H1 = 0;
  static constexpr int H2 = 256 * RP_HIST_COPIES;

  static __device__ __forceinline__ void zero_hist(unsigned* hist) {
    for (int i = threadIdx.x; i < RP_SCRATCH_WORDS; i += THREADS) hist[i] = 0;
  }

  // first-digit counts of one vector into this lane's replica
  static __device__ __forceinline__ void count_digit1(unsigned* hist, const rp_half& h) {
    const rp_u16 b = __builtin_bit_cast(rp_u16, h);
    const int rep = threadIdx.x & (RP_HIST_COPIES - 1);
#pragma unroll
    for (int c = 0; c < RP_EV; ++c) atomicAdd(&hist[H1 + rep * 256 + ((b[c] & 0x7FFFu) >> 7)], 1u);
  }

  // Fill xs[0..n) with the fp16 bits of the operator input (n % 8 == 0).  Global reads are
  // RP_EV-element vectors issued four at a time, so a thread waits for memory once per batch and
  // not once per element.
  // `hist`, when given (top-k selection follows), receives the histogram of the first radix
  // digit on the way: the values are counted while they are still in registers, which saves
  // the selection a pass over LDS and two barriers (select_split is told so).
  static __device__ __forceinline__ void produce(const af_row_src& r, unsigned short* xs, Smem& sm,
                                                 bool store_x, int store_phase, int store_stride,
                                                 unsigned* hist = nullptr) {
    // RMSNorm of a vector of at most one access per thread (n <= RP_EV * THREADS: 4096 channels
    // for the 1024-thread kernels) takes the copy of the code without the batch of four and its
    // masks: the front end is bound by the instructions its waves issue, and that copy issues
    // fewer (q|k|v 15.7 -> 15.4 us, gate|up 21.2 -> 20.8 us at the 7B shape).  The other two
    // producers measured no better with a second copy, so they keep the one.
    if (r.pro == AF_PRO_RMSNORM && r.n <= RP_EV * THREADS)
      produce_batched<1>(r, xs, sm, store_x, store_phase, store_stride, hist);
    else
      produce_batched<4>(r, xs, sm, store_x, store_phase, store_stride, hist);
  }

  template <int B>
  static __device__ __forceinline__ void produce_batched(const af_row_src& r, unsigned short* xs, Smem& sm,
                                                         bool store_x, int store_phase, int store_stride,
                                                         unsigned* hist) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = r.n, nvec = n / RP_EV;
    rp_half* xv = reinterpret_cast<rp_half*>(xs);
    const rp_half* src = reinterpret_cast<const rp_half*>(r.src);
    rp_half zero;
#pragma unroll
    for (int c = 0; c < RP_EV; ++c) zero[c] = (half_t)0;
    if (hist != nullptr) {
      zero_hist(hist);
      if (r.pro != AF_PRO_RMSNORM) __syncthreads();  // the norm has a barrier of its own before it counts
    }
    if (r.pro == AF_PRO_NONE) {
      for (int v0 = tid; v0 < nvec; v0 += B * THREADS) {
        rp_half t[B];
#pragma unroll
        for (int u = 0; u < B; ++u) t[u] = (v0 + u * THREADS < nvec) ? src[v0 + u * THREADS] : zero;
#pragma unroll
        for (int u = 0; u < B; ++u)
          if (v0 + u * THREADS < nvec) {
            xv[v0 + u * THREADS] = t[u];
            if (hist != nullptr) count_digit1(hist, t[u]);
          }
      }
    } else if (r.pro == AF_PRO_RMSNORM) {
      const rp_half* gain = reinterpret_cast<const rp_half*>(r.gain);
      // When one batch per thread covers the vector (the usual case) the gains are fetched
      // together with the source, so the sum-of-squares reduction does not sit between two
      // dependent global round trips.
      const bool single = nvec <= B * THREADS;
      rp_half g[B];
      float ss = 0.f;
      for (int v0 = tid; v0 < nvec; v0 += B * THREADS) {
        rp_half t[B];
#pragma unroll
        for (int u = 0; u < B; ++u) t[u] = (v0 + u * THREADS < nvec) ? src[v0 + u * THREADS] : zero;
        if (single) {
#pragma unroll
          for (int u = 0; u < B; ++u) g[u] = (v0 + u * THREADS < nvec) ? gain[v0 + u * THREADS] : zero;
        }
#pragma unroll
        for (int u = 0; u < B; ++u) {
#pragma unroll
          for (int c = 0; c < RP_EV; ++c) ss += (float)t[u][c] * (float)t[u][c];
          if (v0 + u * THREADS < nvec) xv[v0 + u * THREADS] = t[u];  // raw; normalised below
        }
      }
      ss = af_wave_sum(ss);
      if (lane == 0) sm.red[wave] = ss;
      __syncthreads();
      float tot = 0.f;
#pragma unroll
      for (int w = 0; w < WAVES; ++w) tot += sm.red[w];
      const float scale = 1.0f / sqrtf(tot / (float)n + r.eps);
      for (int v0 = tid; v0 < nvec; v0 += B * THREADS) {
        if (!single) {
#pragma unroll
          for (int u = 0; u < B; ++u) g[u] = (v0 + u * THREADS < nvec) ? gain[v0 + u * THREADS] : zero;
        }
#pragma unroll
        for (int u = 0; u < B; ++u) {
          if (v0 + u * THREADS < nvec) {
            rp_half h = xv[v0 + u * THREADS];   // each thread revisits the vectors it wrote
#pragma unroll
            for (int c = 0; c < RP_EV; ++c) h[c] = (half_t)((float)h[c] * scale * (float)g[u][c]);
            xv[v0 + u * THREADS] = h;
            if (hist != nullptr) count_digit1(hist, h);
          }
        }
      }
    } else {  // AF_PRO_SILUMUL: src = gate[n] | up[n]
      const rp_half* up = reinterpret_cast<const rp_half*>(r.src + n);
      for (int v0 = tid; v0 < nvec; v0 += B * THREADS) {
        rp_half g[B], u8[B];
#pragma unroll
        for (int u = 0; u < B; ++u) {
          const bool ok = v0 + u * THREADS < nvec;
          g[u] = ok ? src[v0 + u * THREADS] : zero;
          u8[u] = ok ? up[v0 + u * THREADS] : zero;
        }
#pragma unroll
        for (int u = 0; u < B; ++u) {
          if (v0 + u * THREADS < nvec) {
            rp_half h;
#pragma unroll
            for (int c = 0; c < RP_EV; ++c) {
              const float gg = (float)g[u][c];
              h[c] = (half_t)(gg * __builtin_amdgcn_rcpf(1.0f + __expf(-gg)) * (float)u8[u][c]);
            }
            xv[v0 + u * THREADS] = h;
            if (hist != nullptr) count_digit1(hist, h);
          }
        }
      }
    }
    __syncthreads();
    if (store_x && r.x_out != nullptr) {
      rp_half* dst = reinterpret_cast<rp_half*>(r.x_out);
      for (int v = store_phase * THREADS + tid; v < nvec; v += store_stride * THREADS) dst[v] = xv[v];
    }
  }

  // digit d with count(digit > d) < want <= count(digit >= d); result in sm.digit / sm.above
  static __device__ __forceinline__ void find_digit(const unsigned* hist, Smem& sm, int nbins,
                                                    unsigned want) {
    // The first wave sums the replicas itself, four neighbouring bins per lane and 16 bytes
    // per LDS read, and scans them; the others only wait for the answer (one barrier).
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    const int tid = threadIdx.x;
    if (tid < AF_WAVE) {
      unsigned cnt[4] = {0u, 0u, 0u, 0u};
      if (4 * tid < nbins) {
#pragma unroll
        for (int c = 0; c < RP_HIST_COPIES; ++c) {
          const u32x4 v = *reinterpret_cast<const u32x4*>(hist + c * nbins + 4 * tid);
          cnt[0] += v[0];
          cnt[1] += v[1];
          cnt[2] += v[2];
          cnt[3] += v[3];
        }
      }
      const unsigned mine = cnt[0] + cnt[1] + cnt[2] + cnt[3];
      const unsigned pre = af_wave_incl_scan(mine);                       // bins of lanes <= mine
      const unsigned all = (unsigned)__builtin_amdgcn_readlane((int)pre, 63);
      unsigned above = all - pre;                                         // bins of higher lanes
#pragma unroll
      for (int q = 3; q >= 0; --q) {
        if (above < want && want <= above + cnt[q]) {
          sm.digit = 4 * tid + q;
          sm.above = above;
        }
        above += cnt[q];
      }
    }
    __syncthreads();
  }

  // exclusive prefix over the workgroup in thread order; *total gets the sum over all threads.
  // sm.wave_tot must not be rewritten before the next barrier of the caller.
  static __device__ __forceinline__ unsigned excl_scan(unsigned v, Smem& sm, unsigned* total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned inc = af_wave_incl_scan(v);
    if (lane == 63) sm.wave_tot[wave] = inc;
    __syncthreads();
    unsigned base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
      const unsigned t = sm.wave_tot[w];
      if (w < wave) base += t;
      tot += t;
    }
    *total = tot;
    return base + inc - v;
  }

  // |x| > t as an integer test on the magnitude key: key > bits(largest fp16 <= t) for t >= 0;
  // -1 lets every key pass for t < 0.  (NaN is kept out by the separate key <= 0x7C00 test.)
  static __device__ __forceinline__ int threshold_key(float t) {
    if (t < 0.f) return -1;
    typedef __fp16 fp16x2 __attribute__((ext_vector_type(2)));
    const fp16x2 h = __builtin_amdgcn_cvt_pkrtz(t, 0.f);  // toward zero = downward for t >= 0
    return (int)(__builtin_bit_cast(unsigned, h) & 0x7FFFu);
  }

  // Threshold selection without an index list for the whole vector (Section 6: a channel is
  // active iff its magnitude passes the preloaded threshold, which needs no look at any other
  // channel).  The channels are cut into S contiguous ranges of whole RP_EV-element vectors;
  // workgroup s builds x only for its range, in xs[0 .. RP_EV * vectors of the range), and lists
  // the channels of that range that pass, as (index << 16 | fp16 bits).  RMSNorm still reads
  // the whole source once for the sum of squares.  Returns the number of list entries.
  // The caller guarantees RP_EV * ceil(n / RP_EV / S) <= capacity of `list` (8 * ceil(n / 8 / S)
  // is at least that).
  static __device__ __forceinline__ int threshold_range(const af_row_src& r, unsigned short* xs,
                                                        Smem& sm, unsigned* list, int S, int s,
                                                        bool store_x) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = r.n, nvec = n / RP_EV;
    const int V = af_ceil_div_small(nvec, S);
    const int vs0 = min(s * V, nvec), vs1 = min(vs0 + V, nvec), nv = vs1 - vs0;
    constexpr int B = 4;
    rp_half* xv = reinterpret_cast<rp_half*>(xs);
    const rp_half* src = reinterpret_cast<const rp_half*>(r.src);
    rp_half zero;
#pragma unroll
    for (int c = 0; c < RP_EV; ++c) zero[c] = (half_t)0;

    if (r.pro == AF_PRO_NONE) {
      for (int i0 = tid; i0 < nv; i0 += B * THREADS) {
        rp_half t[B];
#pragma unroll
        for (int u = 0; u < B; ++u) t[u] = (i0 + u * THREADS < nv) ? src[vs0 + i0 + u * THREADS] : zero;
#pragma unroll
        for (int u = 0; u < B; ++u)
          if (i0 + u * THREADS < nv) xv[i0 + u * THREADS] = t[u];
      }
    } else if (r.pro == AF_PRO_SILUMUL) {
      const rp_half* up = reinterpret_cast<const rp_half*>(r.src + n);
      for (int i0 = tid; i0 < nv; i0 += B * THREADS) {
        rp_half g[B], u8[B];
#pragma unroll
        for (int u = 0; u < B; ++u) {
          const bool ok = i0 + u * THREADS < nv;
          g[u] = ok ? src[vs0 + i0 + u * THREADS] : zero;
          u8[u] = ok ? up[vs0 + i0 + u * THREADS] : zero;
        }
#pragma unroll
        for (int u = 0; u < B; ++u) {
          if (i0 + u * THREADS < nv) {
            rp_half h;
#pragma unroll
            for (int c = 0; c < RP_EV; ++c) {
              const float gg = (float)g[u][c];
              h[c] = (half_t)(gg * __builtin_amdgcn_rcpf(1.0f + __expf(-gg)) * (float)u8[u][c]);
            }
            xv[i0 + u * THREADS] = h;
          }
        }
      }
    } else {  // AF_PRO_RMSNORM
      const rp_half* gain = reinterpret_cast<const rp_half*>(r.gain);
      // the range's own vectors (raw) and their gains travel with the first batch of the
      // full pass, so there is one global round trip before the reduction
      const bool single = nv <= B * THREADS;
      rp_half g[B];
      if (single) {
        rp_half t[B];
#pragma unroll
        for (int u = 0; u < B; ++u) {
          const bool ok = tid + u * THREADS < nv;
          t[u] = ok ? src[vs0 + tid + u * THREADS] : zero;
          g[u] = ok ? gain[vs0 + tid + u * THREADS] : zero;
        }
#pragma unroll
        for (int u = 0; u < B; ++u)
          if (tid + u * THREADS < nv) xv[tid + u * THREADS] = t[u];
      } else {
        for (int i = tid; i < nv; i += THREADS) xv[i] = src[vs0 + i];
      }
      float ss = 0.f;
      for (int v0 = tid; v0 < nvec; v0 += B * THREADS) {
        rp_half t[B];
#pragma unroll
        for (int u = 0; u < B; ++u) t[u] = (v0 + u * THREADS < nvec) ? src[v0 + u * THREADS] : zero;
#pragma unroll
        for (int u = 0; u < B; ++u) {
#pragma unroll
          for (int c = 0; c < RP_EV; ++c) ss += (float)t[u][c] * (float)t[u][c];
        }
      }
      ss = af_wave_sum(ss);
      if (lane == 0) sm.red[wave] = ss;
      __syncthreads();
      float tot = 0.f;
#pragma unroll
      for (int w = 0; w < WAVES; ++w) tot += sm.red[w];
      const float scale = 1.0f / sqrtf(tot / (float)n + r.eps);
      for (int i0 = tid; i0 < nv; i0 += B * THREADS) {
        if (!single) {
#pragma unroll
          for (int u = 0; u < B; ++u) g[u] = (i0 + u * THREADS < nv) ? gain[vs0 + i0 + u * THREADS] : zero;
        }
#pragma unroll
        for (int u = 0; u < B; ++u) {
          if (i0 + u * THREADS < nv) {
            rp_half h = xv[i0 + u * THREADS];   // each thread revisits the vectors it wrote
#pragma unroll
            for (int c = 0; c < RP_EV; ++c) h[c] = (half_t)((float)h[c] * scale * (float)g[u][c]);
            xv[i0 + u * THREADS] = h;
          }
        }
      }
    }
    __syncthreads();
    if (store_x && r.x_out != nullptr) {
      rp_half* dst = reinterpret_cast<rp_half*>(r.x_out);
      for (int i = tid; i < nv; i += THREADS) dst[vs0 + i] = xv[i];
    }

    return range_list(r, xs, sm, list, vs0, nv);
  }

  // Threshold compare, scan and list over nv vectors of x that lie in LDS at xs; the first of
  // them is vector vs0 of the operator input.  Every thread owns a contiguous run.
  static __device__ __forceinline__ int range_list(const af_row_src& r, const unsigned short* xs,
                                                   Smem& sm, unsigned* list, int vs0, int nv) {
    const int tid = threadIdx.x;
    const int T = threshold_key(r.t);
    const int cv = (nv + THREADS - 1) / THREADS;
    const int v0 = min(tid * cv, nv), v1 = min(v0 + cv, nv);
    const rp_u16* xb = reinterpret_cast<const rp_u16*>(xs);
    unsigned gt = 0;
    for (int v = v0; v < v1; ++v) {
      const rp_u16 b = xb[v];
#pragma unroll
      for (int c = 0; c < RP_EV; ++c) {
        const unsigned key = b[c] & 0x7FFFu;
        gt += ((int)key > T) & (key <= 0x7C00u);
      }
    }
    unsigned tot;
    unsigned pos = excl_scan(gt, sm, &tot);
    if (gt != 0) {
      for (int v = v0; v < v1; ++v) {
        const rp_u16 b = xb[v];
#pragma unroll
        for (int c = 0; c < RP_EV; ++c) {
          const unsigned bits = b[c];
          const unsigned key = bits & 0x7FFFu;
          if (((int)key > T) & (key <= 0x7C00u)) {
            list[pos] = ((unsigned)((vs0 + v) * RP_EV + c) << 16) | bits;
            ++pos;
          }
        }
      }
    }
    __syncthreads();
    return (int)tot;
  }

  // Threshold selection of split s's channel range when the whole x already lies in LDS (the
  // router below needs all of it): the compare / scan / list part of threshold_range alone.
  static __device__ __forceinline__ int threshold_range_of_full(const af_row_src& r,
                                                                const unsigned short* xs, Smem& sm,
                                                                unsigned* list, int S, int s) {
    const int nvec = r.n / RP_EV;
    const int V = af_ceil_div_small(nvec, S);
    const int vs0 = min(s * V, nvec), vs1 = min(vs0 + V, nvec);
    return range_list(r, xs + (size_t)vs0 * RP_EV, sm, list, vs0, vs1 - vs0);
  }

  // The `top` largest of E logits (ties to the lower expert, slot 0 the largest) and the
  // softmax over them; one thread.
  static __device__ __forceinline__ void router_pick(const float* logit, int E, int top, int* experts,
                                                     float* weights) {
    unsigned taken = 0;
    float z0 = 0.f, den = 0.f;
    for (int s = 0; s < top; ++s) {
      int best = -1;
      for (int e = 0; e < E; ++e)
        if (!((taken >> e) & 1u) && (best < 0 || logit[e] > logit[best])) best = e;
      taken |= 1u << best;
      experts[s] = best;
      if (s == 0) z0 = logit[best];
      weights[s] = expf(logit[best] - z0);
      den += weights[s];
    }
    for (int s = 0; s < top; ++s) weights[s] /= den;
  }

  // Router of a mixture-of-experts block inside the GEMV's front end: logits[e] = Wr[e] . x over
  // the x in LDS (n <= 8 * THREADS; wr[e] holds this thread's 8 router weights of expert e,
  // fetched by the caller before x was built), reduced lanes -> waves -> one lane per expert in a
  // fixed order, then the pick.  Leaves sm.experts / sm.weights / sm.logit for every thread.
  template <int E_MAX>
  static __device__ __forceinline__ void router_in_lds(const unsigned short* xs, int n, Smem& sm,
                                                       const half8 (&wr)[E_MAX], int E, int top) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const half8* xv = reinterpret_cast<const half8*>(xs);
    float acc[E_MAX];
#pragma unroll
    for (int e = 0; e < E_MAX; ++e) acc[e] = 0.f;
    if (tid < (n >> 3)) {
      const half8 x8 = xv[tid];
#pragma unroll
      for (int e = 0; e < E_MAX; ++e)
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[e] += (float)wr[e][c] * (float)x8[c];
    }
#pragma unroll
    for (int e = 0; e < E_MAX; ++e) {
      const float t = af_wave_sum(acc[e]);
      if (lane == 0) sm.rpart[wave][e] = t;
    }
    __syncthreads();
    if (tid < E) {
      float t = 0.f;
#pragma unroll
      for (int w = 0; w < WAVES; ++w) t += sm.rpart[w][tid];
      sm.logit[tid] = t;
    }
    __syncthreads();
    if (tid == 0) router_pick(sm.logit, E, top, sm.experts, sm.weights);
    __syncthreads();
  }

  // Select on xs[0..n) (n % 8 == 0) and keep the entries of split s of S in list[] as
  // (index << 16 | fp16 bits).  Returns the number of entries kept by this workgroup;
  // *nidx_total is the size of the whole index set.  `hist` is RP_SCRATCH_WORDS words of LDS.
  // `list` may be null (only idx_out / count_out are wanted).
  // Every thread owns a contiguous run of RP_EV-element vectors, read from LDS one vector at a
  // time in each pass; the thread order is therefore the index order.
  static __device__ __forceinline__ int select_split(const af_row_src& r, const unsigned short* xs,
                                                     unsigned* hist, Smem& sm, unsigned* list,
                                                     int S, int s, bool store_idx, bool store_count,
                                                     int* nidx_total, bool digit1_counted = false) {
    const int tid = threadIdx.x, lane = tid & 63;
    const int nvec = r.n / RP_EV;
    const int cv = (nvec + THREADS - 1) / THREADS;  // vectors per thread
    const int v0 = min(tid * cv, nvec), v1 = min(v0 + cv, nvec);
    const rp_u16* xv = reinterpret_cast<const rp_u16*>(xs);
    const int rep = lane & (RP_HIST_COPIES - 1);
    // Both selection rules become integer tests on the magnitude key:
    //   kept outright  <=>  (int)key > T  and  key <= kmax
    //   tie candidates <=>  key == T, kept while the quota lasts (top-k only)
    // top-k: T from the radix select below, kmax = 0x7FFF.  threshold: |x| > t  <=>  key >
    // bits(largest fp16 <= t) for t >= 0 (T = -1 passes everything for t < 0); kmax = 0x7C00
    // keeps NaN out, quota = 0.
    int T = 0x8000;
    unsigned quota = 0, kmax = 0x7FFFu;
    const bool topk = r.sel == AF_SEL_TOPK;
    if (!topk) {
      kmax = 0x7C00u;
      T = threshold_key(r.t);
    }
    if (topk && r.k > 0) {
      if (!digit1_counted) {
        zero_hist(hist);
        __syncthreads();
        for (int v = v0; v < v1; ++v) {
          const rp_u16 b = xv[v];
#pragma unroll
          for (int c = 0; c < RP_EV; ++c)
            atomicAdd(&hist[H1 + rep * 256 + ((b[c] & 0x7FFFu) >> 7)], 1u);
        }
        __syncthreads();
      }
      find_digit(hist + H1, sm, 256, (unsigned)r.k);
      const unsigned d1 = sm.digit, above1 = sm.above;
      for (int v = v0; v < v1; ++v) {
        const rp_u16 b = xv[v];
#pragma unroll
        for (int c = 0; c < RP_EV; ++c) {
          const unsigned key = b[c] & 0x7FFFu;
          if ((key >> 7) == d1) atomicAdd(&hist[H2 + rep * 128 + (key & 127u)], 1u);
        }
      }
      __syncthreads();
      find_digit(hist + H2, sm, 128, (unsigned)r.k - above1);
      T = (int)((d1 << 7) | sm.digit);
      quota = (unsigned)r.k - above1 - sm.above;
    }
    unsigned gt = 0, eq = 0;
    for (int v = v0; v < v1; ++v) {
      const rp_u16 b = xv[v];
#pragma unroll
      for (int c = 0; c < RP_EV; ++c) {
        const unsigned key = b[c] & 0x7FFFu;
        gt += ((int)key > T) & (key <= kmax);
        eq += (int)key == T;
      }
    }
    unsigned tot;
    const unsigned pre = excl_scan(gt | (eq << 16), sm, &tot);
    const int nidx = (int)((tot & 0xFFFFu) + min(tot >> 16, quota));
    *nidx_total = nidx;
    const int R = af_ceil_div_small(nidx, S);
    const int r0 = min(s * R, nidx), r1 = min(r0 + R, nidx);
    unsigned pos = (pre & 0xFFFFu) + min(pre >> 16, quota);
    unsigned eq_seen = pre >> 16;
    // only threads whose run overlaps the split's positions need the second look
    const unsigned my_kept = gt + (min(eq_seen + eq, quota) - min(eq_seen, quota));
    if ((int)(pos + my_kept) > r0 && (int)pos < r1) {
      const bool to_mem = store_idx && r.idx_out != nullptr;
      for (int v = v0; v < v1; ++v) {
        const rp_u16 b = xv[v];
#pragma unroll
        for (int c = 0; c < RP_EV; ++c) {
          const unsigned bits = b[c];
          const unsigned key = bits & 0x7FFFu;
          const bool is_eq = (int)key == T;
          const bool keep = (((int)key > T) & (key <= kmax)) | (is_eq & (eq_seen < quota));
          eq_seen += is_eq;
          if (keep & ((int)pos >= r0) & ((int)pos < r1)) {
            const int j = v * RP_EV + c;
            if (list != nullptr) list[pos - r0] = ((unsigned)j << 16) | bits;
            if (to_mem) r.idx_out[pos] = j;
          }
          pos += keep;
        }
      }
    }
    if (store_count && r.count_out != nullptr && tid == 0) *r.count_out = nidx;
    __syncthreads();
    return r1 - r0;
  }
};
