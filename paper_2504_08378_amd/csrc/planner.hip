// Host-side tools around the hot path: the dynamic weight-cache simulator of Section 4.2 and the
// cost model with its greedy parameter search of Section 4.1 (Eq. 1-9).  Plain C++ on host
// memory; no device code.
#include <algorithm>
#include <math.h>
#include <new>
#include <stdlib.h>
#include <vector>

#include "activeflow.h"

// ---- LFU cache of weight channels (Section 4.2, "Dynamic LLM Weight Caching") --------------
struct af_lfu {
  int n, capacity;
  std::vector<long long> count;
  std::vector<unsigned char> cached, needed;
  int n_cached;
  long long tokens, needed_total, hits_total, evictions_total;
};

extern "C" int af_lfu_create(af_lfu** out, int n_channels, int capacity, const int32_t* initial,
                             int n_initial) {
  if (!out) return AF_ENULL;
  if (n_channels <= 0 || capacity < 0 || n_initial < 0 || n_initial > capacity) return AF_EINVAL;
  if (n_initial > 0 && !initial) return AF_ENULL;
  af_lfu* c = new (std::nothrow) af_lfu();
  if (!c) return AF_EINVAL;
  c->n = n_channels;
  c->capacity = capacity;
  c->count.assign(n_channels, 0);
  c->cached.assign(n_channels, 0);
  c->needed.assign(n_channels, 0);
  c->n_cached = 0;
  c->tokens = c->needed_total = c->hits_total = c->evictions_total = 0;
  for (int i = 0; i < n_initial; ++i) {
    const int j = initial[i];
    if (j < 0 || j >= n_channels || c->cached[j]) {
      delete c;
      return AF_EINVAL;
    }
    c->cached[j] = 1;
    ++c->n_cached;
  }
  *out = c;
  return AF_OK;
}

extern "C" int af_lfu_destroy(af_lfu* c) {
  if (!c) return AF_ENULL;
  delete c;
  return AF_OK;
}

extern "C" int af_lfu_step(af_lfu* c, const int32_t* idx, int nidx, int* hits, int* loaded,
                           int32_t* evicted, int* n_evicted) {
  if (!c || (nidx > 0 && !idx)) return AF_ENULL;
  if (nidx < 0) return AF_EINVAL;
  for (int i = 0; i < nidx; ++i)
    if (idx[i] < 0 || idx[i] >= c->n || (i > 0 && idx[i] <= idx[i - 1])) return AF_EINVAL;  // ascending, unique
  int h = 0;
  for (int i = 0; i < nidx; ++i) {
    const int j = idx[i];
    c->needed[j] = 1;
    ++c->count[j];
    h += c->cached[j];
  }
  // cached channels this token does not need, least used first (ties: lower channel first)
  std::vector<int> victims;
  if (c->n_cached + (nidx - h) > c->capacity) {
    for (int j = 0; j < c->n; ++j)
      if (c->cached[j] && !c->needed[j]) victims.push_back(j);
    std::stable_sort(victims.begin(), victims.end(),
                     [&](int a, int b) { return c->count[a] < c->count[b]; });
  }
  size_t next = 0;
  int ev = 0;
  for (int i = 0; i < nidx; ++i) {
    const int j = idx[i];
    if (c->cached[j]) continue;
    if (c->n_cached < c->capacity) {
      c->cached[j] = 1;
      ++c->n_cached;
      continue;
    }
    if (next >= victims.size()) continue;  // everything cached is needed now: j passes by
    const int m = victims[next];
    if (c->count[j] >= c->count[m]) {  // the worked example of Section 4.2 needs >=, not >
      c->cached[m] = 0;
      c->cached[j] = 1;
      ++next;
      if (evicted) evicted[ev] = m;
      ++ev;
    }
  }
  for (int i = 0; i < nidx; ++i) c->needed[idx[i]] = 0;
  ++c->tokens;
  c->needed_total += nidx;
  c->hits_total += h;
  c->evictions_total += ev;
  if (hits) *hits = h;
  if (loaded) *loaded = nidx - h;
  if (n_evicted) *n_evicted = ev;
  return AF_OK;
}

extern "C" int af_lfu_stats(const af_lfu* c, long long* tokens, long long* needed, long long* hits,
                            long long* evictions) {
  if (!c) return AF_ENULL;
  if (tokens) *tokens = c->tokens;
  if (needed) *needed = c->needed_total;
  if (hits) *hits = c->hits_total;
  if (evictions) *evictions = c->evictions_total;
  return AF_OK;
}

extern "C" int af_lfu_cached(const af_lfu* c, int32_t* channels, int* n_cached) {
  if (!c || !n_cached) return AF_ENULL;
  int k = 0;
  for (int j = 0; j < c->n; ++j)
    if (c->cached[j]) {
      if (channels) channels[k] = j;
      ++k;
    }
  *n_cached = k;
  return AF_OK;
}

// ---- cost model (Section 4.1, Eq. 1-9) ---------------------------------------------------------
extern "C" int af_cost_eval(const af_cost_in* in, af_cost_out* out) {
  if (!in || !out) return AF_ENULL;
  if (!(in->bw_mem > 0) || !(in->bw_flash_small > 0) || !(in->bw_flash_large > 0)) return AF_EINVAL;
  if (in->sp < 0 || in->sp > 1 || in->hr < 0 || in->hr > 1 || in->si < 0 || in->si > 1) return AF_EINVAL;
  if (in->S_l < 0 || in->N < 0 || in->M_cache < 0 || in->M_kv < 0) return AF_EINVAL;
  out->M_cl = in->S_l * (1.0 - in->sp) * in->N;                                            // Eq. 9
  out->T_load = out->M_cl * (1.0 - in->hr) / in->bw_flash_small;                            // Eq. 3
  out->T_comp = out->M_cl / in->bw_mem;                                                     // Eq. 4
  out->T_onload = in->S_l * (1.0 - in->sp) * (1.0 - in->hr) * (1.0 - in->si) / in->bw_flash_small;  // Eq. 6
  out->T_preload = out->M_cl * (1.0 - in->hr) / in->bw_flash_large;                         // Eq. 7
  out->T_overlap = out->T_onload + fmax(out->T_preload, out->T_comp);                       // Eq. 5
  out->M = out->M_cl + in->M_cache + in->M_kv;                                              // Eq. 8
  out->T_decode = out->T_load + out->T_overlap + out->T_comp;                               // Eq. 1
  return AF_OK;
}

// hit rate at a cache fraction: piecewise linear through the caller's points (ascending fractions),
// flat outside them
static double hr_at(const af_plan_in* p, double frac) {
  if (p->n_hr <= 0) return 0.0;
  if (frac <= p->hr_fraction[0]) return p->hr_value[0];
  for (int i = 1; i < p->n_hr; ++i) {
    if (frac <= p->hr_fraction[i]) {
      const double w = (frac - p->hr_fraction[i - 1]) / (p->hr_fraction[i] - p->hr_fraction[i - 1]);
      return p->hr_value[i - 1] + w * (p->hr_value[i] - p->hr_value[i - 1]);
    }
  }
  return p->hr_value[p->n_hr - 1];
}

extern "C" int af_plan_search(const af_plan_in* p, af_plan_out* out) {
  if (!p || !out) return AF_ENULL;
  if (!(p->M_max > 0) || !(p->S_m > 0) || !(p->S_l > 0) || p->M_kv < 0 || p->n_max < 1) return AF_EINVAL;
  if (p->n_hr < 1 || p->n_hr > AF_PLAN_MAX_HR || !p->hr_fraction || !p->hr_value) return AF_EINVAL;
  for (int i = 1; i < p->n_hr; ++i)
    if (!(p->hr_fraction[i] > p->hr_fraction[i - 1])) return AF_EINVAL;
  double sp = 1.0 - p->M_max / p->S_m;
  if (sp < 0) sp = 0;
  if (sp > 1.0 - 1e-12) sp = 1.0 - 1e-12;
  out->sp = sp;
  out->N = 0;
  out->M_cache = 0;
  out->hr = 0;
  out->visited = 0;
  double prev = -1.0;
  bool have = false;
  for (int N = 1; N <= p->n_max; ++N) {
    af_cost_in in;
    in.sp = sp;
    in.si = p->si;
    in.bw_mem = p->bw_mem;
    in.bw_flash_small = p->bw_flash_small;
    in.bw_flash_large = p->bw_flash_large;
    in.S_l = p->S_l;
    in.N = N;
    in.M_kv = p->M_kv;
    in.M_cache = p->M_max - p->S_l * (1.0 - sp) * N - p->M_kv;  // the cache takes what the budget leaves
    if (in.M_cache < 0) break;
    in.hr = hr_at(p, in.M_cache / (p->S_m * (1.0 - sp)));
    af_cost_out c;
    const int rc = af_cost_eval(&in, &c);
    if (rc) return rc;
    ++out->visited;
    if (!have || c.T_decode < out->cost.T_decode) {
      have = true;
      out->N = N;
      out->M_cache = in.M_cache;
      out->hr = in.hr;
      out->cost = c;
    }
    if (c.T_preload <= c.T_comp) break;                                  // preloading hides behind compute
    if (prev >= 0 && fabs(prev - c.T_preload) < p->min_gain) break;      // no longer worth a larger group
    prev = c.T_preload;
  }
  return AF_OK;
}
