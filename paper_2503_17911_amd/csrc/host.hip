// Host side of the library: error reporting, index upload/packing, workspace.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <new>
#include <vector>

#include "ann_internal.hpp"

namespace ann {

static thread_local char g_err[512] = "";

ann_status fail(ann_status code, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

ann_status hip_fail(hipError_t e, const char *what) {
  ann_status code = (e == hipErrorOutOfMemory) ? ANN_ENOMEM : ANN_EDEVICE;
  return fail(code, "%s: %s", what, hipGetErrorString(e));
}

// ---------------------------------------------------------------- pack kernels
// codes [n][row_bytes] -> [n][row_stride]; 8-bit codes are stored biased by
// 128 (c ^ 0x80 read as int8 is c - 128) so the signed packed-dot instruction
// applies; padding bytes are never multiplied by a non-zero query byte.
__global__ void pack_codes_kernel(const uint8_t *__restrict__ in, uint8_t *__restrict__ out, uint64_t n,
                                  uint32_t row_bytes, uint32_t row_stride, uint32_t flip) {
  uint64_t total = n * row_stride;
  for (uint64_t e = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; e < total; e += (uint64_t)gridDim.x * blockDim.x) {
    uint64_t i = e / row_stride;
    uint32_t b = (uint32_t)(e - i * row_stride);
    uint8_t v = (b < row_bytes) ? in[i * row_bytes + b] : 0;
    out[e] = (uint8_t)(v ^ flip);
  }
}

// CSR -> [n][degree] with padding; sets *bad if a row is too long.
template <typename T>
__global__ void pack_csr_kernel(const T *__restrict__ cols, const uint64_t *__restrict__ offsets,
                                T *__restrict__ out, uint64_t n, uint32_t degree, T pad, uint32_t *bad) {
  uint64_t total = n * degree;
  for (uint64_t e = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; e < total; e += (uint64_t)gridDim.x * blockDim.x) {
    uint64_t i = e / degree;
    uint32_t t = (uint32_t)(e - i * degree);
    uint64_t b = offsets[i], len = offsets[i + 1] - b;
    if (t == 0 && len > degree) atomicOr(bad, 1u);
    out[e] = (t < len) ? cols[b + t] : pad;
  }
}

// A row must not name the same neighbour twice.
__global__ void check_rows_distinct_kernel(const uint32_t *__restrict__ adj, uint64_t n, uint32_t degree,
                                           uint32_t *bad) {
  for (uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; i < n; i += (uint64_t)gridDim.x * blockDim.x) {
    const uint32_t *row = adj + i * degree;
    for (uint32_t t = 1; t < degree; ++t) {
      const uint32_t v = row[t];
      if (v == ANN_PAD_ID) continue;
      for (uint32_t u = 0; u < t; ++u)
        if (row[u] == v) atomicOr(bad, 4u);
    }
  }
}

// Redundant layout: entry (i, t), t < stored, receives a copy of the code row
// (and norm term) of neighbour adjacency[i][t]; padding slots are zero.
__global__ void build_prs_kernel(const uint32_t *__restrict__ adj, const uint8_t *__restrict__ codes,
                                 const float *__restrict__ norm, uint64_t n, uint32_t degree, uint32_t stored,
                                 uint32_t row_stride, uint8_t *__restrict__ out_codes, float *__restrict__ out_norm) {
  const uint32_t cpr = row_stride / 16;
  const uint64_t total = n * stored * cpr;
  for (uint64_t e = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; e < total; e += (uint64_t)gridDim.x * blockDim.x) {
    const uint64_t entry = e / cpr;
    const uint32_t c = (uint32_t)(e - entry * cpr);
    const uint64_t node = entry / stored;
    const uint32_t t = (uint32_t)(entry - node * stored);
    const uint32_t v = adj[node * degree + t];
    const bool real = v != ANN_PAD_ID && v < n;
    reinterpret_cast<uint4 *>(out_codes)[e] =
        real ? reinterpret_cast<const uint4 *>(codes + (uint64_t)v * row_stride)[c] : make_uint4(0, 0, 0, 0);
    if (c == 0 && out_norm) out_norm[entry] = real ? norm[v] : 0.0f;
  }
}

// Adjacency rows with the neighbours' norm terms behind them: row i is
// adjacency[i][0 .. degree) followed by norm[adjacency[i][t]] for t in
// 0 .. degree (zero for padding slots).
__global__ void build_row_norms_kernel(const uint32_t *__restrict__ adj, const float *__restrict__ norm, uint64_t n,
                                       uint32_t degree, uint32_t *__restrict__ out) {
  const uint64_t total = n * degree;
  for (uint64_t e = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; e < total; e += (uint64_t)gridDim.x * blockDim.x) {
    const uint64_t node = e / degree;
    const uint32_t t = (uint32_t)(e - node * degree);
    const uint32_t v = adj[e];
    const bool real = v != ANN_PAD_ID && v < n;
    out[node * 2 * degree + t] = v;
    out[node * 2 * degree + degree + t] = real ? __float_as_uint(norm[v]) : 0u;
  }
}

__global__ void check_adjacency_kernel(const uint32_t *__restrict__ adj, uint64_t total, uint64_t n, uint32_t *bad) {
  for (uint64_t e = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; e < total; e += (uint64_t)gridDim.x * blockDim.x) {
    uint32_t v = adj[e];
    if (v != ANN_PAD_ID && v >= n) atomicOr(bad, 2u);
  }
}

namespace {

// Device buffer holding a copy of `count` elements from host or device memory.
template <typename T>
ann_status dev_copy(T **dst, const T *src, size_t count, bool src_on_host, hipStream_t st) {
  *dst = nullptr;
  if (count == 0) return ANN_OK;
  ANN_HIP(hipMalloc((void **)dst, count * sizeof(T)));
  ANN_HIP(hipMemcpyAsync(*dst, src, count * sizeof(T), src_on_host ? hipMemcpyHostToDevice : hipMemcpyDeviceToDevice,
                         st));
  return ANN_OK;
}

void free_workspace(Workspace &w) {
  (void)hipFree(w.tq);
  (void)hipFree(w.s);
  (void)hipFree(w.qlo);
  (void)hipFree(w.sum_t);
  w = Workspace{};
}

void destroy(ann_index *ix) {
  if (!ix) return;
  (void)hipFree(ix->vectors);
  (void)hipFree(ix->adjacency);
  (void)hipFree(ix->labels);
  (void)hipFree(ix->adjacency_norms);
  (void)hipFree(ix->pivot_codes);
  (void)hipFree(ix->prs_codes);
  (void)hipFree(ix->prs_norm);
  (void)hipFree(ix->pivot_norm);
  (void)hipFree(ix->pivot_ids);
  for (int l = 0; l < ANN_MAX_LEVELS; ++l) {
    (void)hipFree(ix->level[l].codes);
    (void)hipFree(ix->level[l].lo);
    (void)hipFree(ix->level[l].delta);
    (void)hipFree(ix->level[l].norm_term);
  }
  for (StreamWorkspaces &sw : ix->stream_ws)
    for (Workspace &w : sw.ws) free_workspace(w);
  delete ix;
}

inline int grid_for(uint64_t total, int block) {
  uint64_t g = (total + block - 1) / block;
  return (int)(g > 65535 * 16 ? 65535 * 16 : (g ? g : 1));
}

}  // namespace

ann_status workspace_for(ann_index *ix, uint32_t level, uint32_t nq, hipStream_t st, WorkspaceLease &lease) {
  if (!lease.lock.owns_lock()) lease.lock = std::unique_lock<std::mutex>(ix->ws_mutex);
  StreamWorkspaces *sw = nullptr, *free_slot = nullptr, *oldest = nullptr;
  for (StreamWorkspaces &c : ix->stream_ws) {
    if (c.used && c.stream == st) {
      sw = &c;
      break;
    }
    if (!c.used && !free_slot) free_slot = &c;
    if (c.used && (!oldest || c.last_use < oldest->last_use)) oldest = &c;
  }
  if (!sw) {
    if (free_slot) {
      sw = free_slot;
    } else {
      // every set is taken: hand the least recently used one to this stream,
      // once nothing on the device can still be reading it
      ANN_HIP(hipDeviceSynchronize());
      sw = oldest;
      for (Workspace &w : sw->ws) w.folded_q = nullptr, w.folded_nq = 0;
    }
    sw->used = true;
    sw->stream = st;
  }
  sw->last_use = ++ix->ws_clock;
  Workspace &w = sw->ws[level];
  lease.ws = &w;
  if (nq <= w.nq_cap) return ANN_OK;
  // growth is the only allocation on the search path (ann_reserve_workspace
  // moves it out of the path); it waits for work that may still be using the
  // old buffers
  ANN_HIP(hipDeviceSynchronize());
  free_workspace(w);
  uint32_t cap = nq < 1024 ? 1024 : nq;
  w.tq_plane = tq_plane_for(ix->level[level]);
  w.tq_stride = w.tq_plane * (ix->query_bits == 15 ? 2u : 1u);
  ANN_HIP(hipMalloc((void **)&w.tq, (size_t)cap * w.tq_stride));
  ANN_HIP(hipMalloc((void **)&w.s, (size_t)cap * sizeof(float)));
  ANN_HIP(hipMalloc((void **)&w.qlo, (size_t)cap * sizeof(float)));
  ANN_HIP(hipMalloc((void **)&w.sum_t, (size_t)cap * 2 * sizeof(int32_t)));
  w.nq_cap = cap;
  return ANN_OK;
}

}  // namespace ann

using namespace ann;

extern "C" {

const char *ann_last_error(void) { return g_err; }
const char *ann_version(void) { return "ann-gfx950 0.1"; }

ann_status ann_upload_index(const ann_index_desc *desc, void *stream, ann_index **out) {
  hipStream_t st = (hipStream_t)stream;
  if (!out) return fail(ANN_EINVAL, "ann_upload_index: out is NULL");
  *out = nullptr;
  if (!desc) return fail(ANN_EINVAL, "ann_upload_index: desc is NULL");
  if (desc->n == 0 || desc->n >= (1ull << 31)) return fail(ANN_EINVAL, "n must be in [1, 2^31), got %llu", (unsigned long long)desc->n);
  if (desc->d == 0) return fail(ANN_EINVAL, "d must be positive");
  if (desc->d > 2048) return fail(ANN_ECAPACITY, "d = %u exceeds the supported maximum 2048", desc->d);
  if (desc->degree == 0) return fail(ANN_EINVAL, "degree must be positive");
  if (desc->degree > ANN_MAX_DEGREE) return fail(ANN_ECAPACITY, "degree = %u exceeds ANN_MAX_DEGREE = %u", desc->degree, ANN_MAX_DEGREE);
  if (desc->metric != ANN_L2 && desc->metric != ANN_IP) return fail(ANN_EINVAL, "unknown metric %u", desc->metric);
  if ((desc->flags & ANN_DESC_UNIT_NORM_L2_KEYS) && desc->metric != ANN_IP)
    return fail(ANN_EINVAL, "ANN_DESC_UNIT_NORM_L2_KEYS is for ANN_IP indexes");
  if (desc->n_levels < 1 || desc->n_levels > ANN_MAX_LEVELS) return fail(ANN_EINVAL, "n_levels must be 1..%d", ANN_MAX_LEVELS);
  if (!desc->adjacency) return fail(ANN_EINVAL, "adjacency is NULL");
  if (desc->entry_point >= desc->n) return fail(ANN_EINVAL, "entry_point %u is not a node", desc->entry_point);
  for (uint32_t l = 0; l < desc->n_levels; ++l) {
    const ann_sq_level &L = desc->level[l];
    if (L.bits != 8 && L.bits != 4) return fail(ANN_EINVAL, "level %u: bits must be 4 or 8, got %u", l, L.bits);
    if (L.bits == 4 && (desc->d & 1)) return fail(ANN_EINVAL, "level %u: 4-bit codes need an even d", l);
    if (!L.codes || !L.lo || !L.delta) return fail(ANN_EINVAL, "level %u: codes, lo and delta must be given", l);
    if ((desc->metric == ANN_L2 || (desc->flags & ANN_DESC_UNIT_NORM_L2_KEYS)) && !L.norm_term)
      return fail(ANN_EINVAL, "level %u: norm_term is required for ANN_L2 and for ANN_DESC_UNIT_NORM_L2_KEYS", l);
  }
  const bool host = (desc->flags & ANN_DESC_HOST_POINTERS) != 0;
  const uint64_t n = desc->n;

  ann_index *ix = new (std::nothrow) ann_index();
  if (!ix) return fail(ANN_ENOMEM, "host allocation failed");
  ix->n = n;
  ix->d = desc->d;
  ix->degree = desc->degree;
  ix->metric = desc->metric;
  ix->query_bits = (desc->flags & ANN_DESC_QUERY_15BIT) ? 15u : 8u;
  ix->key_metric = (desc->flags & ANN_DESC_UNIT_NORM_L2_KEYS) ? (uint32_t)ANN_L2 : desc->metric;
  ix->n_levels = desc->n_levels;
  ix->entry_point = desc->entry_point;
  (void)hipGetDevice(&ix->device);

  ann_status rc = ANN_OK;
  uint32_t *bad_dev = nullptr;
  uint8_t *raw_codes = nullptr;
  uint32_t *raw_cols = nullptr;
  uint64_t *raw_offs = nullptr;
  float *raw_labels = nullptr;
  auto cleanup = [&](ann_status r) {
    (void)hipFree(bad_dev);
    (void)hipFree(raw_codes);
    (void)hipFree(raw_cols);
    (void)hipFree(raw_offs);
    (void)hipFree(raw_labels);
    if (r != ANN_OK) destroy(ix);
    return r;
  };
#define ANN_TRY(expr)                      \
  do {                                     \
    rc = (expr);                           \
    if (rc != ANN_OK) return cleanup(rc);  \
  } while (0)
#define ANN_TRY_HIP(call)                                         \
  do {                                                            \
    hipError_t e_ = (call);                                       \
    if (e_ != hipSuccess) return cleanup(hip_fail(e_, #call));    \
  } while (0)

  ANN_TRY_HIP(hipMalloc((void **)&bad_dev, sizeof(uint32_t)));
  ANN_TRY_HIP(hipMemsetAsync(bad_dev, 0, sizeof(uint32_t), st));

  if (desc->vectors) ANN_TRY(dev_copy(&ix->vectors, desc->vectors, (size_t)n * desc->d, host, st));

  for (uint32_t l = 0; l < desc->n_levels; ++l) {
    const ann_sq_level &S = desc->level[l];
    LevelDev &L = ix->level[l];
    L.bits = S.bits;
    L.row_bytes = S.bits == 8 ? desc->d : desc->d / 2;
    // Rows start on 16-byte boundaries.  Where it costs at most a third more
    // memory they are also laid out so that no row crosses more 128-byte lines
    // than it must: a stride that divides 128 or is a multiple of it (96-byte
    // rows at stride 128 touch one line each instead of one or two; 480-byte
    // rows at stride 512 four instead of four or five).
    L.row_stride = (L.row_bytes + 15u) & ~15u;
    {
      uint32_t aligned = L.row_bytes <= 16 ? 16u : L.row_bytes <= 32 ? 32u : L.row_bytes <= 64 ? 64u : (L.row_bytes + 127u) & ~127u;
      if ((aligned - L.row_bytes) * 3u <= L.row_bytes) L.row_stride = aligned;
    }
    uint32_t chunks = L.row_stride / 16u, lpr = 8;
    while (lpr < chunks) lpr <<= 1;
    if (lpr > 64) return cleanup(fail(ANN_ECAPACITY, "level %u: code rows of %u bytes exceed 1024", l, L.row_bytes));
    L.lanes_per_row = lpr;
    uint32_t sl = 1;
    while (sl * 4 < chunks) sl <<= 1;
    L.search_lanes = sl;
    ANN_TRY(dev_copy(&L.lo, S.lo, desc->d, host, st));
    ANN_TRY(dev_copy(&L.delta, S.delta, desc->d, host, st));
    if (S.norm_term) ANN_TRY(dev_copy(&L.norm_term, S.norm_term, (size_t)n, host, st));
    const uint8_t *src = S.codes;
    if (host) {
      ANN_TRY(dev_copy(&raw_codes, S.codes, (size_t)n * L.row_bytes, true, st));
      src = raw_codes;
    }
    ANN_TRY_HIP(hipMalloc((void **)&L.codes, (size_t)n * L.row_stride));
    uint64_t total = n * L.row_stride;
    pack_codes_kernel<<<grid_for(total, 256), 256, 0, st>>>(src, L.codes, n, L.row_bytes, L.row_stride,
                                                            S.bits == 8 ? 0x80u : 0u);
    ANN_TRY_HIP(hipGetLastError());
    if (host) {
      ANN_TRY_HIP(hipStreamSynchronize(st));
      (void)hipFree(raw_codes);
      raw_codes = nullptr;
    }
  }

  const uint64_t total_adj = n * desc->degree;
  if (desc->csr_offsets) {
    const uint64_t *offs = desc->csr_offsets;
    const uint32_t *cols = desc->adjacency;
    uint64_t nnz = 0;
    if (host) {
      nnz = desc->csr_offsets[n];
      ANN_TRY(dev_copy(&raw_offs, desc->csr_offsets, (size_t)n + 1, true, st));
      ANN_TRY(dev_copy(&raw_cols, desc->adjacency, (size_t)nnz, true, st));
      offs = raw_offs;
      cols = raw_cols;
    }
    ANN_TRY_HIP(hipMalloc((void **)&ix->adjacency, total_adj * sizeof(uint32_t)));
    pack_csr_kernel<uint32_t><<<grid_for(total_adj, 256), 256, 0, st>>>(cols, offs, ix->adjacency, n, desc->degree,
                                                                         ANN_PAD_ID, bad_dev);
    ANN_TRY_HIP(hipGetLastError());
    if (desc->edge_labels) {
      const float *lab = desc->edge_labels;
      if (host) {
        ANN_TRY(dev_copy(&raw_labels, desc->edge_labels, (size_t)nnz, true, st));
        lab = raw_labels;
      }
      ANN_TRY_HIP(hipMalloc((void **)&ix->labels, total_adj * sizeof(float)));
      pack_csr_kernel<float><<<grid_for(total_adj, 256), 256, 0, st>>>(lab, offs, ix->labels, n, desc->degree, 0.0f,
                                                                        bad_dev);
      ANN_TRY_HIP(hipGetLastError());
    }
  } else {
    ANN_TRY(dev_copy(&ix->adjacency, desc->adjacency, (size_t)total_adj, host, st));
    if (desc->edge_labels) ANN_TRY(dev_copy(&ix->labels, desc->edge_labels, (size_t)total_adj, host, st));
  }
  check_rows_distinct_kernel<<<grid_for(n, 256), 256, 0, st>>>(ix->adjacency, n, desc->degree, bad_dev);
  ANN_TRY_HIP(hipGetLastError());
  check_adjacency_kernel<<<grid_for(total_adj, 256), 256, 0, st>>>(ix->adjacency, total_adj, n, bad_dev);
  ANN_TRY_HIP(hipGetLastError());
  uint32_t bad = 0;
  ANN_TRY_HIP(hipMemcpyAsync(&bad, bad_dev, sizeof(bad), hipMemcpyDeviceToHost, st));
  ANN_TRY_HIP(hipStreamSynchronize(st));
  if (bad & 1u) return cleanup(fail(ANN_EINVAL, "a CSR row has more than degree = %u neighbours", desc->degree));
  if (bad & 2u) return cleanup(fail(ANN_EINVAL, "adjacency holds a neighbour id >= n"));
  if (bad & 4u) return cleanup(fail(ANN_EINVAL, "an adjacency row names the same neighbour twice"));
#undef ANN_TRY
#undef ANN_TRY_HIP
  cleanup(ANN_OK);
  *out = ix;
  return ANN_OK;
}

ann_status ann_build_prs_ratio(ann_index *index, float ratio, void *stream) {
  hipStream_t st = (hipStream_t)stream;
  if (!index) return fail(ANN_EINVAL, "ann_build_prs_ratio: index is NULL");
  if (!(ratio > 0.0f && ratio <= 1.0f)) return fail(ANN_EINVAL, "ann_build_prs_ratio: the ratio must be in (0, 1]");
  uint32_t stored = (uint32_t)((double)ratio * index->degree + 0.999999);
  if (stored < 1) stored = 1;
  if (stored > index->degree) stored = index->degree;
  if (index->prs_codes && index->prs_slots == stored) return ANN_OK;
  if (index->prs_codes) {
    ANN_HIP(hipDeviceSynchronize());  // a search may still be reading the old copy
    (void)hipFree(index->prs_codes);
    (void)hipFree(index->prs_norm);
    index->prs_codes = nullptr;
    index->prs_norm = nullptr;
    index->prs_slots = 0;
  }
  const LevelDev &L = index->level[0];
  const uint64_t entries = index->n * stored;
  ANN_HIP(hipMalloc((void **)&index->prs_codes, (size_t)entries * L.row_stride));
  if (index->key_metric == ANN_L2) {
    hipError_t e = hipMalloc((void **)&index->prs_norm, (size_t)entries * sizeof(float));
    if (e != hipSuccess) {
      (void)hipFree(index->prs_codes);
      index->prs_codes = nullptr;
      return hip_fail(e, "hipMalloc");
    }
  }
  const uint64_t total = entries * (L.row_stride / 16);
  build_prs_kernel<<<grid_for(total, 256), 256, 0, st>>>(index->adjacency, L.codes, index->prs_norm ? L.norm_term : nullptr,
                                                         index->n, index->degree, stored, L.row_stride, index->prs_codes,
                                                         index->prs_norm);
  ANN_HIP(hipGetLastError());
  ANN_HIP(hipStreamSynchronize(st));
  index->prs_slots = stored;
  return ANN_OK;
}

ann_status ann_build_row_norms(ann_index *index, void *stream) {
  hipStream_t st = (hipStream_t)stream;
  if (!index) return fail(ANN_EINVAL, "ann_build_row_norms: index is NULL");
  if (index->adjacency_norms) return ANN_OK;
  const LevelDev &L = index->level[0];
  if (index->key_metric != ANN_L2 || !L.norm_term)
    return fail(ANN_EINVAL, "ann_build_row_norms: the index's keys use no norm term (inner-product keys)");
  ANN_HIP(hipMalloc((void **)&index->adjacency_norms, (size_t)index->n * index->degree * 2 * sizeof(uint32_t)));
  build_row_norms_kernel<<<grid_for(index->n * index->degree, 256), 256, 0, st>>>(index->adjacency, L.norm_term, index->n,
                                                                                  index->degree, index->adjacency_norms);
  hipError_t e = hipGetLastError();
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  if (e != hipSuccess) {
    (void)hipFree(index->adjacency_norms);
    index->adjacency_norms = nullptr;
    return hip_fail(e, "build_row_norms_kernel");
  }
  return ANN_OK;
}

ann_status ann_build_prs(ann_index *index, void *stream) {
  if (!index) return fail(ANN_EINVAL, "ann_build_prs: index is NULL");
  return ann_build_prs_ratio(index, 1.0f, stream);
}

ann_status ann_reserve_workspace(ann_index *index, uint32_t max_nq, void *stream) {
  if (!index) return fail(ANN_EINVAL, "ann_reserve_workspace: index is NULL");
  if (max_nq == 0) return fail(ANN_EINVAL, "ann_reserve_workspace: max_nq == 0");
  WorkspaceLease lease;
  for (uint32_t l = 0; l < index->n_levels; ++l) {
    ann_status rc = workspace_for(index, l, max_nq, (hipStream_t)stream, lease);
    if (rc != ANN_OK) return rc;
  }
  return ANN_OK;
}

ann_status ann_free_index(ann_index *index) {
  if (!index) return ANN_OK;
  (void)hipDeviceSynchronize();
  destroy(index);
  return ANN_OK;
}

}  // extern "C"
