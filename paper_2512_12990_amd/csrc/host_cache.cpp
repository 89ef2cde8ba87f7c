// Host-only bookkeeping that produces the slice mask: the unified slice LRU (paper Sections 4.1
// and 6.1 item 3) and the post-prefill retention order (Section 4.3).  No device work.
#include "../../include/slicemoe.h"
#include <algorithm>
#include <new>
#include <vector>

struct smoe_cache {
  int L, E, cap, count;
  // intrusive doubly linked list over slice ids; head = most recently used, tail = next victim
  std::vector<int> prev, next;
  std::vector<uint8_t> resident;
  int head, tail;
  smoe_cache_stats st;

  void unlink(int s) {
    const int p = prev[s], n = next[s];
    if (p >= 0) next[p] = n; else head = n;
    if (n >= 0) prev[n] = p; else tail = p;
    resident[s] = 0; count--;
  }
  void push_front(int s) {
    prev[s] = -1; next[s] = head;
    if (head >= 0) prev[head] = s; else tail = s;
    head = s; resident[s] = 1; count++;
  }
  void push_back(int s) {
    next[s] = -1; prev[s] = tail;
    if (tail >= 0) next[tail] = s; else head = s;
    tail = s; resident[s] = 1; count++;
  }
  void make_room() { if (count >= cap && tail >= 0) unlink(tail); }
};

extern "C" int smoe_cache_create(int L, int E, int capacity_slices, smoe_cache** out) {
  if (!out) return SMOE_EINVAL;
  *out = nullptr;
  if (L <= 0 || E <= 0 || capacity_slices < 2) return SMOE_ESHAPE;
  smoe_cache* c = new (std::nothrow) smoe_cache();
  if (!c) return SMOE_EINVAL;
  const size_t n = (size_t)2 * L * E;
  c->L = L; c->E = E; c->cap = capacity_slices; c->count = 0; c->head = c->tail = -1;
  c->prev.assign(n, -1); c->next.assign(n, -1); c->resident.assign(n, 0);
  c->st = smoe_cache_stats{0, 0, 0, 0};
  *out = c;
  return SMOE_OK;
}

extern "C" int smoe_cache_destroy(smoe_cache* c) {
  if (!c) return SMOE_EINVAL;
  delete c;
  return SMOE_OK;
}

extern "C" int smoe_cache_init_order(smoe_cache* c, const uint32_t* slice_ids, int n) {
  if (!c || (n > 0 && !slice_ids) || n < 0) return SMOE_EINVAL;
  const uint32_t lim = (uint32_t)(2 * c->L * c->E);
  std::vector<uint8_t> seen(lim, 0);
  const int m = std::min(n, c->cap);
  for (int i = 0; i < m; i++) {
    if (slice_ids[i] >= lim || seen[slice_ids[i]]) return SMOE_EINVAL;
    seen[slice_ids[i]] = 1;
  }
  while (c->tail >= 0) c->unlink(c->tail);
  for (int i = 0; i < m; i++) c->push_back((int)slice_ids[i]);
  return SMOE_OK;
}

extern "C" int smoe_cache_snapshot(const smoe_cache* c, int layer, float beta, uint8_t* slice_mask_host, float* bias_host) {
  if (!c || !slice_mask_host) return SMOE_EINVAL;
  if (layer < 0 || layer >= c->L) return SMOE_ESHAPE;
  for (int e = 0; e < c->E; e++) {
    const int s = (layer * c->E + e) << 1;
    const uint8_t m = (uint8_t)(c->resident[s] | (c->resident[s | 1] << 1));
    slice_mask_host[e] = m;
    if (bias_host) bias_host[e] = (m & 1) ? beta : 0.0f;
  }
  return SMOE_OK;
}

extern "C" int smoe_cache_access(smoe_cache* c, int layer, int k, const int32_t* idx_host, const uint8_t* want_high_host) {
  if (!c || !idx_host || k < 0) return SMOE_EINVAL;
  if (layer < 0 || layer >= c->L) return SMOE_ESHAPE;
  for (int j = 0; j < k; j++)
    if (idx_host[j] < 0 || idx_host[j] >= c->E) return SMOE_ESHAPE;
  for (int j = 0; j < k; j++) {
    const int s = (layer * c->E + idx_host[j]) << 1;
    if (c->resident[s]) { c->st.msb_hit++; c->unlink(s); }
    else { c->st.msb_miss++; c->make_room(); }
    c->push_front(s);
    if (want_high_host && want_high_host[j]) {
      const int l = s | 1;
      if (c->resident[l]) c->st.lsb_hit++;
      else { c->st.lsb_miss++; c->make_room(); c->push_back(l); }
    }
  }
  return SMOE_OK;
}

extern "C" int smoe_cache_snapshot_all(const smoe_cache* c, float beta, uint8_t* slice_mask_host, float* bias_host) {
  if (!c || !slice_mask_host) return SMOE_EINVAL;
  for (int l = 0; l < c->L; l++) {
    const int rc = smoe_cache_snapshot(c, l, beta, slice_mask_host + (size_t)l * c->E, bias_host ? bias_host + (size_t)l * c->E : nullptr);
    if (rc) return rc;
  }
  return SMOE_OK;
}

extern "C" int smoe_cache_access_all(smoe_cache* c, int k, const int32_t* idx_host, int idx_stride, const uint8_t* want_high_host) {
  if (!c || !idx_host || k < 0 || idx_stride < k) return SMOE_EINVAL;
  for (int l = 0; l < c->L; l++)                      // nothing is applied unless every index is valid
    for (int j = 0; j < k; j++) {
      const int32_t e = idx_host[(size_t)l * idx_stride + j];
      if (e < 0 || e >= c->E) return SMOE_ESHAPE;
    }
  for (int l = 0; l < c->L; l++) {
    const int rc = smoe_cache_access(c, l, k, idx_host + (size_t)l * idx_stride, want_high_host ? want_high_host + (size_t)l * k : nullptr);
    if (rc) return rc;
  }
  return SMOE_OK;
}

extern "C" int smoe_cache_stats_get(const smoe_cache* c, smoe_cache_stats* out) {
  if (!c || !out) return SMOE_EINVAL;
  *out = c->st;
  return SMOE_OK;
}

extern "C" int smoe_cache_order(const smoe_cache* c, uint32_t* slice_ids_host, int max_n, int* n_out) {
  if (!c || !n_out || (max_n > 0 && !slice_ids_host)) return SMOE_EINVAL;
  int n = 0;
  for (int s = c->head; s >= 0 && n < max_n; s = c->next[s]) slice_ids_host[n++] = (uint32_t)s;
  *n_out = n;
  return SMOE_OK;
}

extern "C" int smoe_topn_slices(const uint32_t* hist_host, int L, int E, int N, uint32_t* slice_ids_host, int* n_out) {
  if (!hist_host || !n_out || (N > 0 && !slice_ids_host)) return SMOE_EINVAL;
  if (L <= 0 || E <= 0 || N < 0) return SMOE_ESHAPE;
  const int LE = L * E;
  std::vector<int> order(LE);
  for (int i = 0; i < LE; i++) order[i] = i;
  // higher count first; the flat (layer, expert) index breaks ties, which a stable sort keeps
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return hist_host[a] > hist_host[b]; });
  int n = 0;
  for (int plane = 0; plane < 2 && n < N; plane++)
    for (int i = 0; i < LE && n < N; i++) slice_ids_host[n++] = ((uint32_t)order[i] << 1) | (uint32_t)plane;
  *n_out = n;
  return SMOE_OK;
}

// ---- modeled cost on the paper's target system (Section 5) ---------------------------------
extern "C" int smoe_system_spec_paper(smoe_system_spec* out) {
  if (!out) return SMOE_EINVAL;
  out->flash_gbit_s = 10.0; out->dram_gbit_s = 104.0; out->xpu_tops = 16.4;
  out->flash_pj_bit = 103.0; out->dram_pj_bit = 1.5; out->xpu_tops_w = 3.18;
  return SMOE_OK;
}

extern "C" int smoe_cost_model(const smoe_system_spec* spec, const smoe_cache_stats* stats, uint64_t msb_slice_bytes,
                               uint64_t lsb_slice_bytes, double ops, smoe_cost* out) {
  if (!spec || !stats || !out) return SMOE_EINVAL;
  if (!(spec->flash_gbit_s > 0) || !(spec->dram_gbit_s > 0) || !(spec->xpu_tops > 0) || !(spec->xpu_tops_w > 0) || ops < 0)
    return SMOE_EINVAL;
  const double bm = (double)msb_slice_bytes, bl = (double)lsb_slice_bytes;
  const double miss_bytes = (double)stats->msb_miss * bm + (double)stats->lsb_miss * bl;
  const double used_bytes = (double)(stats->msb_hit + stats->msb_miss) * bm + (double)(stats->lsb_hit + stats->lsb_miss) * bl;
  out->flash_bits = 8.0 * miss_bytes;
  out->dram_bits = 8.0 * (used_bytes + miss_bytes);
  out->ops = ops;
  out->energy_j = out->flash_bits * spec->flash_pj_bit * 1e-12 + out->dram_bits * spec->dram_pj_bit * 1e-12 +
                  ops / (spec->xpu_tops_w * 1e12);
  out->latency_s = out->flash_bits / (spec->flash_gbit_s * 1e9) + out->dram_bits / (spec->dram_gbit_s * 1e9) +
                   ops / (spec->xpu_tops * 1e12);
  const double req = (double)(stats->msb_hit + stats->msb_miss);
  out->miss_rate_high = req > 0 ? miss_bytes / (req * (bm + bl)) : 0.0;
  return SMOE_OK;
}
