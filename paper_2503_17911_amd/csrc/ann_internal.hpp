// Internal declarations shared by the translation units of the library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "ann.h"

namespace ann {

constexpr int kWave = 64;

// Device copy of one code level, in the layout the kernels read.
struct LevelDev {
  uint32_t bits = 0;
  uint32_t row_bytes = 0;    // d or d/2: the bytes that carry codes
  uint32_t row_stride = 0;   // row_bytes rounded up to 16
  uint32_t lanes_per_row = 0;  // rescore kernel: one 16-byte chunk per lane; power of two >= row_stride/16, in {8,..,64}
  uint32_t search_lanes = 0;   // search kernel: four chunks per lane; power of two >= row_stride/64, in {1,..,16}
  uint8_t *codes = nullptr;  // [n][row_stride]; 8-bit codes stored as (c ^ 0x80), 4-bit codes as given
  float *lo = nullptr;       // [d]
  float *delta = nullptr;    // [d]
  float *norm_term = nullptr;  // [n] or nullptr
};

// Scratch for the folded queries of one batch (one per code level and stream).
struct Workspace {
  uint32_t nq_cap = 0;
  uint8_t *tq = nullptr;   // [nq_cap][tq_stride] folded query in kernel layout
  float *s = nullptr;      // [nq_cap]
  float *qlo = nullptr;    // [nq_cap]
  int32_t *sum_t = nullptr;  // [2][nq_cap]: sums of the folded bytes, first plane then second
  uint32_t tq_stride = 0;   // bytes per query: one plane, or two for the 15-bit query (high bytes, then low bytes)
  uint32_t tq_plane = 0;    // bytes of one plane
  const float *folded_q = nullptr;  // the batch whose folded form the buffers hold (as last launched)
  uint32_t folded_nq = 0;
};

// The workspaces of the calls issued on one stream.  Work on a stream runs in
// order, so calls on the same stream may share them; calls on different
// streams get different sets and may be in flight together.
constexpr int kMaxStreamWorkspaces = 8;
struct StreamWorkspaces {
  hipStream_t stream = nullptr;
  bool used = false;
  uint64_t last_use = 0;
  Workspace ws[ANN_MAX_LEVELS];
};

}  // namespace ann

struct ann_index {
  uint64_t n = 0;
  uint32_t d = 0, degree = 0, metric = 0, n_levels = 0, entry_point = 0;
  uint32_t query_bits = 8;  // width of the folded query: 8, or 15 (two byte planes)
  uint32_t key_metric = 0;  // form of the low-precision keys: the metric, or ANN_L2 for unit-norm inner-product data
  float *vectors = nullptr;    // [n][d] or nullptr
  uint32_t *adjacency = nullptr;  // [n][degree]
  float *labels = nullptr;        // [n][degree] edge labels or nullptr
  uint32_t *adjacency_norms = nullptr;  // [n][2 * degree]: every adjacency row followed by its neighbours' level-0 norm terms (bits), or nullptr
  uint8_t *prs_codes = nullptr;    // redundant layout: [n][prs_slots][row_stride] level-0 code rows of each node's first neighbours
  float *prs_norm = nullptr;       // [n][prs_slots] their norm terms (L2)
  uint32_t prs_slots = 0;          // slots per node stored that way (redundancy ratio = prs_slots / degree)
  uint8_t *pivot_codes = nullptr;  // entry-point stage: [n_pivots][row_stride] level-0 codes of the sampled nodes
  float *pivot_norm = nullptr;     // [n_pivots] their norm terms (L2)
  uint32_t *pivot_ids = nullptr;   // [n_pivots] their node ids
  uint32_t n_pivots = 0;
  ann::LevelDev level[ANN_MAX_LEVELS];
  ann::StreamWorkspaces stream_ws[ann::kMaxStreamWorkspaces];
  uint64_t ws_clock = 0;
  std::mutex ws_mutex;  // guards the stream -> workspace table
  int device = 0;
};

namespace ann {

// Error reporting (thread-local message behind ann_last_error()).
ann_status fail(ann_status code, const char *fmt, ...);
ann_status hip_fail(hipError_t e, const char *what);
#define ANN_HIP(call)                                        \
  do {                                                       \
    hipError_t e_ = (call);                                  \
    if (e_ != hipSuccess) return ::ann::hip_fail(e_, #call); \
  } while (0)

// Kernel-layout length of one byte plane of a folded query for a level: every 16-byte chunk of
// codes needs 16 (8-bit) or 32 (4-bit) query bytes; zero-padded to the number
// of chunks the kernels' lanes cover.
inline uint32_t tq_plane_for(const LevelDev &L) {
  uint32_t chunks = L.search_lanes * 4 > L.lanes_per_row ? L.search_lanes * 4 : L.lanes_per_row;
  return chunks * (L.bits == 8 ? 16u : 32u);
}

// A workspace together with the lock on the index's stream -> workspace
// table.  The holder keeps it until everything that reads or writes the
// workspace has been enqueued: a stream beyond kMaxStreamWorkspaces takes a
// set over only under this lock and after a device-wide wait, so work that was
// enqueued while a lease was held never sees its buffers change hands.
struct WorkspaceLease {
  std::unique_lock<std::mutex> lock;
  Workspace *ws = nullptr;
};

// The workspace of (level, stream), holding at least nq queries.
ann_status workspace_for(ann_index *index, uint32_t level, uint32_t nq, hipStream_t stream, WorkspaceLease &lease);
// Folds a batch into the given buffers (no allocation, no table lookup).
ann_status launch_query_prep_into(const ann_index *index, uint32_t level, const float *q, uint32_t nq,
                                  const Workspace &w, int8_t *t_plain, float *s_out, float *qlo_out,
                                  hipStream_t stream);
// Folds a batch into the workspace of (level, stream), which `lease` then holds.
ann_status launch_query_prep(ann_index *index, uint32_t level, const float *q, uint32_t nq, int8_t *t_plain,
                             float *s_out, float *qlo_out, hipStream_t stream, WorkspaceLease &lease);

}  // namespace ann
