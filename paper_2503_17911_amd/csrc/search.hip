// Host entry point of the batched graph search: argument checks, choice of the
// visited set and of the kernel family, launch (kernels: search_kernel.hpp).
#include "search_kernel.hpp"


#include <mutex>

using namespace ann;

namespace {

// What the argument checks settle before anything is launched.
struct SearchPlan {
  uint32_t p = 1, vis_log2 = 0;
  bool cache = false, wide = false;
};

ann_status check_search_args(const char *fn, const ann_index *index, const float *q, uint32_t nq,
                             const ann_search_params *params, const uint32_t *entry_ids, uint32_t n_entry,
                             const uint32_t *out_ids, SearchPlan &plan) {

  if (!index || !q || !params || !out_ids) return fail(ANN_EINVAL, "%s: NULL argument", fn);
  if (nq == 0) return fail(ANN_EINVAL, "%s: nq == 0", fn);
  if (params->k == 0) return fail(ANN_EINVAL, "%s: k == 0", fn);
  if (params->ef < params->k) return fail(ANN_EINVAL, "%s: ef = %u < k = %u", fn, params->ef, params->k);
  if (params->ef > ANN_MAX_EF) return fail(ANN_ECAPACITY, "%s: ef = %u exceeds ANN_MAX_EF = %u", fn, params->ef, ANN_MAX_EF);
  if (params->layout > 2) return fail(ANN_EINVAL, "%s: unknown layout %u", fn, params->layout);
  if (params->layout == 2 && !index->adjacency_norms) return fail(ANN_EINVAL, "%s: layout 2 needs ann_build_row_norms first", fn);
  if (params->layout == 1 && !index->prs_codes) return fail(ANN_EINVAL, "%s: layout 1 needs ann_build_prs first", fn);
  if (params->layout == 1 && (params->alpha_s > 0.0f || (params->m_s != 0 && params->m_s < index->degree)))
    return fail(ANN_EUNSUPPORTED, "%s: the edge filter is not available with the redundant layout", fn);
  if (!(params->alpha_s >= 0.0f)) return fail(ANN_EINVAL, "%s: alpha_s must be >= 0", fn);
  if (params->alpha_s > 0.0f && !index->labels) return fail(ANN_EINVAL, "%s: alpha_s given but the index was uploaded without edge labels", fn);
  if (params->mode > 1) return fail(ANN_EINVAL, "%s: unknown mode %u", fn, params->mode);
  if (params->mode == 0 && params->expansions_per_step > 1) return fail(ANN_EINVAL, "%s: expansions_per_step needs mode 1", fn);
  if (params->expansions_per_step > (uint32_t)kMaxExpansionsPerStep) return fail(ANN_ECAPACITY, "%s: expansions_per_step = %u exceeds %d", fn, params->expansions_per_step, kMaxExpansionsPerStep);
  const uint32_t p = params->mode == 0 ? 1u : (params->expansions_per_step ? params->expansions_per_step : ann_default_expansions_per_step(params->ef, index->degree));
  if (entry_ids && n_entry == 0) return fail(ANN_EINVAL, "%s: entry_ids given with n_entry == 0", fn);
  if (entry_ids && n_entry > ANN_MAX_ENTRIES) return fail(ANN_ECAPACITY, "%s: n_entry = %u exceeds ANN_MAX_ENTRIES = %u", fn, n_entry, ANN_MAX_ENTRIES);

  const uint32_t ef = params->ef;
  const bool capped = params->m_s != 0 && params->m_s < index->degree;
  if (params->visited_kind > ANN_VISITED_CACHE_WIDE) return fail(ANN_EINVAL, "%s: unknown visited_kind %u", fn, params->visited_kind);
  const bool wide = params->visited_kind == ANN_VISITED_CACHE_WIDE;
  if ((params->visited_kind == ANN_VISITED_CACHE || wide) && capped)
    return fail(ANN_EINVAL, "%s: the cap m_s needs ANN_VISITED_TABLE (its choice of neighbours depends on the visited set)", fn);
  const bool cache = params->visited_kind == ANN_VISITED_CACHE || wide || (params->visited_kind == ANN_VISITED_AUTO && !capped);
  // the table must hold the pool and one step's candidates below 3/4 load
  // after a rebuild; the cache has no such minimum
  uint32_t need = cache ? 64u : 2 * (ef + 64 * p), min_log2 = 0;
  while ((1u << min_log2) < need) ++min_log2;
  uint32_t vis_log2;
  if (params->visited_slots == 0) {
    // defaults: a small cache, so that many queries are resident per compute
    // unit (1024 slots measured fastest on 1M x 128 SQ8 for ef 64..256; with
    // wide code rows a repeated evaluation costs more, 2048 slots measured
    // fastest on 200k x 960 SQ4); the largest table when the cap is active, so
    // that rebuilds are rare
    const uint32_t want = cache ? (index->level[0].row_stride >= 256 ? 2048u : 1024u) : (capped ? 8192u : 1024u);
    vis_log2 = 0;
    while ((1u << vis_log2) < want) ++vis_log2;
    if (vis_log2 < min_log2) vis_log2 = min_log2;
  } else {
    uint32_t v = params->visited_slots;
    if (v & (v - 1)) return fail(ANN_EINVAL, "%s: visited_slots = %u is not a power of two", fn, v);
    vis_log2 = 0;
    while ((1u << vis_log2) < v) ++vis_log2;
    if (vis_log2 < min_log2) return fail(ANN_EINVAL, "%s: visited_slots = %u is below the minimum %u for ef = %u", fn, v, 1u << min_log2, ef);
  }
  if (vis_log2 > 13) return fail(ANN_ECAPACITY, "%s: the visited set would need more than 8192 slots", fn);
  plan.p = p;
  plan.vis_log2 = vis_log2;
  plan.cache = cache;
  plan.wide = wide;
  return ANN_OK;
}

// Launch of the search kernel for a batch whose folded queries are in `w`.
ann_status launch_search_with(const ann_index *index, uint32_t nq, const ann_search_params *params,
                              const SearchPlan &plan, const uint32_t *entry_ids, uint32_t n_entry, uint32_t *out_ids,
                              float *out_keys, int32_t *out_idot, uint32_t *out_counts, const Workspace &w,
                              hipStream_t st) {
  const uint32_t ef = params->ef, p = plan.p, vis_log2 = plan.vis_log2;
  const bool cache = plan.cache, wide = plan.wide;
  const LevelDev &L = index->level[0];
  if (index->query_bits == 15 && out_idot)
    return fail(ANN_EINVAL, "out_idot is not available with the 15-bit query (the dot products exceed 32 bits)");
  SearchArgs a{};
  a.codes = L.codes;
  a.norm_term = index->key_metric == ANN_L2 ? L.norm_term : nullptr;
  a.adj_norms = params->layout == 2 ? 1u : 0u;
  a.adjacency = a.adj_norms ? index->adjacency_norms : index->adjacency;
  a.adj_stride = a.adj_norms ? 2 * index->degree : index->degree;
  a.tq = w.tq;
  a.s = w.s;
  a.qlo = w.qlo;
  a.sum_t = w.sum_t;
  a.sum_t_lo = index->query_bits == 15 ? w.sum_t + w.nq_cap : nullptr;
  a.tq_plane = w.tq_plane;
  a.q15 = index->query_bits == 15 ? 1u : 0u;
  a.entry_ids = entry_ids;
  a.order = params->query_order;
  a.ef_per_query = params->ef_per_query;
  a.prs_codes = params->layout == 1 ? index->prs_codes : nullptr;
  a.prs_norm = params->layout == 1 && index->key_metric == ANN_L2 ? index->prs_norm : nullptr;
  a.prs_slots = index->prs_slots;
  a.labels = params->alpha_s > 0.0f ? index->labels : nullptr;
  a.alpha_s = params->alpha_s;
  a.m_s = params->m_s == 0 || params->m_s > index->degree ? index->degree : params->m_s;
  a.filtered = (a.labels != nullptr || a.m_s < index->degree) ? 1u : 0u;
  a.out_ids = out_ids;
  a.out_keys = out_keys;
  a.out_idot = out_idot;
  a.out_counts = out_counts;
  a.n = index->n;
  a.row_stride = L.row_stride;
  a.n_chunks = L.row_stride / 16;
  a.degree = index->degree;
  a.metric = index->key_metric;  // the form of the traversal key
  a.tq_stride = w.tq_stride;
  a.n_entry = entry_ids ? n_entry : 0;
  a.entry_point = index->entry_point;
  a.ef = ef;
  a.vis_log2 = vis_log2;
  a.vis_cache = cache ? 1u : 0u;
  // 16-bit tags (twice the entries in the same memory) while (set, tag) can name every node
  const bool packed = cache && !wide && ((index->n - 1) >> vis_log2) + 1 < 0xFFFFu;
  a.vis_packed = packed ? 1u : 0u;
  a.nq = nq;
  a.p = p;
  int m = 1;
  while (64 * m < (int)ef) m <<= 1;
  const bool multi = params->mode != 0;
  // more than the default number of expansions per step: the kernels built for the maximum
  const bool wide_step = multi && p > (uint32_t)kDefaultExpansionsPerStep;
  const uint32_t p_built = wide_step ? (uint32_t)kMaxExpansionsPerStep : (uint32_t)kDefaultExpansionsPerStep;
  // FAST multi-expansion kernels: the staging area (64 m entries, at least 32 per expansion) must hold a step's ids
  const bool ids_fit = index->degree <= 32 || 64 * m >= (int)(64 * p_built);
  const bool fast = packed && !a.filtered && !a.prs_codes && !a.q15 && (!multi || (ids_fit && p == p_built));
  if (wide_step)
    return fast ? launch_search_fast_wide(a, L.bits, L.search_lanes, m, st)
                : launch_search_general_wide(a, L.bits, L.search_lanes, m, st);
  return fast ? launch_search_fast(a, L.bits, L.search_lanes, m, multi, st)
              : launch_search_general(a, L.bits, L.search_lanes, m, multi, st);
}

}  // namespace



extern "C" uint32_t ann_default_expansions_per_step(uint32_t ef, uint32_t degree) {
  // pools of more than 256 entries take eight registers per lane: their staging area holds 8 x 64 ids
  const bool folded_kernel_for_eight = degree <= 32 || ef > 256;
  return ef > 128 && folded_kernel_for_eight ? (uint32_t)kMaxExpansionsPerStep : (uint32_t)kDefaultExpansionsPerStep;
}

extern "C" ann_status ann_search_batch(ann_index *index, const float *q, uint32_t nq, const ann_search_params *params,
                                       const uint32_t *entry_ids, uint32_t n_entry, uint32_t *out_ids, float *out_keys,
                                       int32_t *out_idot, uint32_t *out_counts, void *stream) {
  hipStream_t st = (hipStream_t)stream;
  SearchPlan plan;
  ann_status rc = check_search_args("ann_search_batch", index, q, nq, params, entry_ids, n_entry, out_ids, plan);
  if (rc != ANN_OK) return rc;
  WorkspaceLease lease;  // held until the search kernel is enqueued
  if (params->reuse_folded_queries) {
    rc = workspace_for(index, 0, nq, st, lease);
    if (rc != ANN_OK) return rc;
    if (lease.ws->folded_q != q || lease.ws->folded_nq != nq)
      return fail(ANN_EINVAL, "ann_search_batch: reuse_folded_queries, but the last folding for this index on this stream was of another batch");
  } else {
    rc = launch_query_prep(index, 0, q, nq, nullptr, nullptr, nullptr, st, lease);
    if (rc != ANN_OK) return rc;
  }
  return launch_search_with(index, nq, params, plan, entry_ids, n_entry, out_ids, out_keys, out_idot, out_counts,
                            *lease.ws, st);
}

// ---------------------------------------------------------------- no allocation
// The folded queries of ann_search_batch_static live here instead of in a
// workspace from hipMalloc.  In host code the array's name is only a handle:
// the address the kernels use comes from hipGetSymbolAddress, once per device.
static __device__ __align__(256) unsigned char scratch[ANN_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
unsigned char *g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device.
ann_status scratch_address(unsigned char **out) {
  int dev = 0;
  ANN_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(ANN_ECAPACITY, "ann_search_batch_static: device %d is beyond the %d devices the library tracks", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *ptr = nullptr;
    ANN_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return fail(ANN_EDEVICE, "ann_search_batch_static: hipGetSymbolAddress returned no address");
    g_scratch_ptr[dev] = static_cast<unsigned char *>(ptr);
  }
  *out = g_scratch_ptr[dev];
  return ANN_OK;
}

inline size_t round_up_256(size_t v) { return (v + 255) & ~(size_t)255; }

}  // namespace

extern "C" ann_status ann_search_batch_static(ann_index *index, const float *q, uint32_t nq,
                                              const ann_search_params *params, const uint32_t *entry_ids,
                                              uint32_t n_entry, uint32_t *out_ids, float *out_keys, int32_t *out_idot,
                                              uint32_t *out_counts, void *stream) {
  hipStream_t st = (hipStream_t)stream;
  SearchPlan plan;
  ann_status rc = check_search_args("ann_search_batch_static", index, q, nq, params, entry_ids, n_entry, out_ids, plan);
  if (rc != ANN_OK) return rc;
  if (params->reuse_folded_queries)
    return fail(ANN_EINVAL, "ann_search_batch_static: reuse_folded_queries is not available (the static scratch is shared by every index)");
  // carve the folded-query buffers out of the static array
  Workspace w;
  w.tq_plane = tq_plane_for(index->level[0]);
  w.tq_stride = w.tq_plane * (index->query_bits == 15 ? 2u : 1u);
  const size_t tq_bytes = round_up_256((size_t)nq * w.tq_stride), word_bytes = round_up_256((size_t)nq * 4);
  const size_t need = tq_bytes + 4 * word_bytes;
  if (need > (size_t)ANN_STATIC_SCRATCH_BYTES)
    return fail(ANN_ECAPACITY, "ann_search_batch_static: %u queries of %u folded bytes need %zu bytes of scratch, the static buffer holds %zu",
                nq, w.tq_stride, need, (size_t)ANN_STATIC_SCRATCH_BYTES);
  unsigned char *base = nullptr;
  rc = scratch_address(&base);
  if (rc != ANN_OK) return rc;
  w.nq_cap = nq;
  w.tq = base;
  w.s = reinterpret_cast<float *>(base + tq_bytes);
  w.qlo = reinterpret_cast<float *>(base + tq_bytes + word_bytes);
  w.sum_t = reinterpret_cast<int32_t *>(base + tq_bytes + 2 * word_bytes);  // two planes of nq sums
  // the folding writes every byte the search reads (rows are written whole,
  // zero padding included), so nothing of an earlier call has to be cleared
  rc = launch_query_prep_into(index, 0, q, nq, w, nullptr, nullptr, nullptr, st);
  if (rc != ANN_OK) return rc;
  return launch_search_with(index, nq, params, plan, entry_ids, n_entry, out_ids, out_keys, out_idot, out_counts, w,
                            st);
}
