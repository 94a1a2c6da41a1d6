// Exact k nearest neighbours by exhaustive search: the ground truth NN_k of
// the paper's recall measure (Section 6.1).  The Q.X^T contraction runs on the
// matrix cores (fp32 MFMA 32x32x2); a threshold-and-buffer top-k in LDS keeps
// k + margin candidates per (query, base slab); the candidates of all slabs
// are then re-evaluated directly in fp64 (rerank kernel) and sorted by
// (distance, id), so the decomposed fp32 scores only ever select candidates.
//
// Three tile kernels, chosen by ann_bruteforce_topk: bf_own_kernel (k <= 16,
// d % 4 == 0: 128 x 128 tiles, eight wavefronts, per-wavefront candidate
// lists), bf_block_kernel (k <= 152: 128 x 128 or 64 x 256 tiles, four
// wavefronts, one buffer per query) and bf_tile_kernel (anything: 32 x 128
// tiles, scalar staging).  In the first two the slabs of a query publish their
// kp-th best score in global memory and every slab filters with the smallest:
// the kp-th best of a part bounds the kp-th best of the whole.
#include "ann_internal.hpp"
#include "device_utils.hpp"

namespace ann {

ann_status rerank_device(const float *X, uint64_t n, uint32_t d, uint32_t metric, const float *Q, uint32_t nq,
                         const uint32_t *cand, uint32_t n_cand, uint32_t stride, uint32_t k, uint32_t *out_ids,
                         float *out_dist, hipStream_t st, const float *cand_keys = nullptr, uint32_t n_min = 0,
                         float gamma = 0.0f, uint32_t *out_n = nullptr);

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kQT = 32;    // queries per workgroup
constexpr int kBT = 128;   // base vectors per tile (4 wavefronts x 32)
constexpr int kKC = 32;    // K chunk staged in LDS
constexpr int kLd = kKC + 1;  // padded row length (floats): conflict-free column reads

__global__ void fill_u32_kernel(uint32_t *__restrict__ p, uint32_t n, uint32_t v) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

__global__ void row_norm_kernel(const float *__restrict__ x, uint64_t n, uint32_t d, float *__restrict__ out) {
  const int lane = threadIdx.x % kWave;
  const uint64_t wave = ((uint64_t)blockIdx.x * blockDim.x + threadIdx.x) / kWave;
  const uint64_t n_waves = (uint64_t)gridDim.x * blockDim.x / kWave;
  for (uint64_t i = wave; i < n; i += n_waves) {
    float acc = 0.f;
    for (uint32_t j = lane; j < d; j += kWave) {
      float v = x[i * d + j];
      acc = fmaf(v, v, acc);
    }
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) acc += __int_as_float(xor_lane_i32(__float_as_int(acc), m));
    if (lane == 0) out[i] = acc;
  }
}

// One workgroup: kQT queries against base rows [slab*rows_per_slab, ...).
// The K dimension is walked in chunks of kKC; the next chunk of Q and X is
// fetched into registers while the matrix cores work on the current one, then
// written to the other half of a double-buffered LDS tile (one barrier per
// chunk).  LDS: Qs[2][kQT][kLd], Xs[2][kBT][kLd], thr[kQT], cnt[kQT],
// buf[kQT][cb] (u64).
// VEC4: rows are read as float4 (needs d % 4 == 0).
template <bool VEC4>
__global__ __launch_bounds__(256) void bf_tile_kernel(const float *__restrict__ X, const float *__restrict__ xnorm,
                                                      uint64_t n, uint32_t d, const float *__restrict__ Q, uint32_t nq,
                                                      uint32_t metric, uint64_t rows_per_slab, uint32_t kp, uint32_t cb,
                                                      uint32_t *__restrict__ cand_out /*[nq][slabs][kp]*/) {
  extern __shared__ float smem_f[];
  float *Qs = smem_f;                    // [2][kQT][kLd]
  float *Xs = Qs + 2 * kQT * kLd;        // [2][kBT][kLd]
  float *thr = Xs + 2 * kBT * kLd;
  uint32_t *cnt = reinterpret_cast<uint32_t *>(thr + kQT);
  uint64_t *buf = reinterpret_cast<uint64_t *>(cnt + kQT);  // offset is a multiple of 8 bytes

  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const uint32_t q0 = blockIdx.x * kQT;
  const uint32_t slab = blockIdx.y, n_slabs = gridDim.y;
  const uint64_t b_begin = (uint64_t)slab * rows_per_slab;
  const uint64_t b_end = b_begin + rows_per_slab < n ? b_begin + rows_per_slab : n;

  if (tid < kQT) {
    thr[tid] = INFINITY;
    cnt[tid] = 0;
  }

  // staging registers: one float4 of Q and four of X per thread and chunk
  // (kQT*kKC = 1024 and kBT*kKC = 4096 floats over 256 threads)
  const int sc = (tid % 8) * 4;  // column inside the chunk
  const int sr = tid / 8;        // row 0..31 (+32 i for X)
  float4 rq, rx[4];
  auto fetch = [&](uint64_t t0, uint32_t k0) {
    const uint32_t kk = k0 + sc;
    const uint32_t qi = q0 + sr;
    rq = make_float4(0.f, 0.f, 0.f, 0.f);
    if (qi < nq) {
      const float *p = Q + (uint64_t)qi * d + kk;
      if (VEC4) {
        if (kk < d) rq = *reinterpret_cast<const float4 *>(p);
      } else {
        if (kk + 0 < d) rq.x = p[0];
        if (kk + 1 < d) rq.y = p[1];
        if (kk + 2 < d) rq.z = p[2];
        if (kk + 3 < d) rq.w = p[3];
      }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint64_t bi = t0 + sr + 32 * i;
      rx[i] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (bi < b_end) {
        const float *p = X + bi * d + kk;
        if (VEC4) {
          if (kk < d) rx[i] = *reinterpret_cast<const float4 *>(p);
        } else {
          if (kk + 0 < d) rx[i].x = p[0];
          if (kk + 1 < d) rx[i].y = p[1];
          if (kk + 2 < d) rx[i].z = p[2];
          if (kk + 3 < d) rx[i].w = p[3];
        }
      }
    }
  };
  auto stage = [&](int b) {
    float *qd = Qs + (b * kQT + sr) * kLd + sc;
    qd[0] = rq.x;
    qd[1] = rq.y;
    qd[2] = rq.z;
    qd[3] = rq.w;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float *xd = Xs + (b * kBT + sr + 32 * i) * kLd + sc;
      xd[0] = rx[i].x;
      xd[1] = rx[i].y;
      xd[2] = rx[i].z;
      xd[3] = rx[i].w;
    }
  };

  const uint32_t n_chunks = (d + kKC - 1) / kKC;
  int cur = 0;
  if (b_begin < b_end) {
    fetch(b_begin, 0);
    stage(0);
  }
  __syncthreads();

  for (uint64_t t0 = b_begin; t0 < b_end; t0 += kBT) {
    floatx16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
    for (uint32_t c = 0; c < n_chunks; ++c) {
      // next chunk (of this tile, or the first of the next tile) on its way
      const bool last_chunk = c + 1 == n_chunks;
      const uint64_t nt0 = last_chunk ? t0 + kBT : t0;
      const bool more = nt0 < b_end;
      if (more) fetch(nt0, last_chunk ? 0 : (c + 1) * kKC);
      const float *ap = Qs + (cur * kQT + lane % 32) * kLd + lane / 32;
      const float *bp = Xs + (cur * kBT + wave * 32 + lane % 32) * kLd + lane / 32;
#pragma unroll
      for (int kk = 0; kk < kKC; kk += 2) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(ap[kk], bp[kk], acc, 0, 0, 0);
      if (more) stage(cur ^ 1);
      __syncthreads();
      cur ^= 1;
    }
    // scores and threshold filter.  acc[i] belongs to query row
    // 8*(i/4) + 4*(lane/32) + i%4 and base column lane%32 of this wave.
    const uint64_t bi = t0 + wave * 32 + lane % 32;
    const bool live = bi < b_end;
    const float xn = (live && metric == ANN_L2) ? xnorm[bi] : 0.f;
    bool pushed = false;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int row = 8 * (i / 4) + 4 * (lane / 32) + (i % 4);
      const float score = metric == ANN_L2 ? fmaf(-2.0f, acc[i], xn) : -acc[i];
      if (live && q0 + row < nq && score < thr[row]) {
        uint32_t pos = atomicAdd(&cnt[row], 1u);
        buf[(size_t)row * cb + pos] = ((uint64_t)order_u32(score) << 32) | (uint32_t)bi;
        pushed = true;
      }
    }
    // tiles that pushed nothing (the common case once the thresholds have
    // settled) skip the compaction pass
    if (__syncthreads_or(pushed ? 1 : 0) == 0) continue;
    // keep the kp best of every row that grew beyond kp (each wave owns 8 rows)
    for (int row = wave; row < kQT; row += 4) {
      const uint32_t c = cnt[row];
      if (c <= kp) continue;
      uint64_t *list = buf + (size_t)row * cb;
      uint64_t mine[8];
      uint32_t rank[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const uint32_t i = lane + u * kWave;
        mine[u] = i < c ? list[i] : ~0ull;
        rank[u] = 0;
      }
      for (uint32_t j = 0; j < c; ++j) {
        const uint64_t o = list[j];
#pragma unroll
        for (int u = 0; u < 8; ++u) rank[u] += o < mine[u] ? 1u : 0u;   // ids differ, so no ties
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const uint32_t i = lane + u * kWave;
        if (i < c && rank[u] < kp) {
          list[rank[u]] = mine[u];
          if (rank[u] == kp - 1) thr[row] = unorder_f32((uint32_t)(mine[u] >> 32));
        }
      }
      if (lane == 0) cnt[row] = kp;
    }
    __syncthreads();
  }
  // hand the survivors of this slab to the exact stage
  for (int e = tid; e < kQT * (int)kp; e += 256) {
    const int row = e / kp, j = e % kp;
    const uint32_t qi = q0 + row;
    if (qi < nq)
      cand_out[((uint64_t)qi * n_slabs + slab) * kp + j] = (uint32_t)j < cnt[row] ? (uint32_t)buf[(size_t)row * cb + j] : ANN_PAD_ID;
  }
}


// The part_lists-th smallest of n_vals published values (+inf in score order:
// nothing published): with every part (a slab's buffer, a wavefront's list)
// publishing its part_rank-th best score, that many parts hold part_rank
// entries each at or below it, so the query has part_lists * part_rank >= kp
// entries at or below it - a bound on its kp-th best.
__device__ __forceinline__ uint32_t bound_over_parts(const uint32_t *vals, uint32_t n_vals, uint32_t part_lists) {
  constexpr int kMaxLists = 8;
  uint32_t low[kMaxLists];   // the smallest published values, ascending
#pragma unroll
  for (int j = 0; j < kMaxLists; ++j) low[j] = 0xFFFFFFFFu;
  for (uint32_t i = 0; i < n_vals; ++i) {
    uint32_t v = vals[i];
#pragma unroll
    for (int j = 0; j < kMaxLists; ++j) {
      const uint32_t lo_ = v < low[j] ? v : low[j];
      v = v < low[j] ? low[j] : v;
      low[j] = lo_;
    }
  }
  uint32_t t = 0xFFFFFFFFu;
#pragma unroll
  for (int j = 0; j < kMaxLists; ++j) t = (uint32_t)j == part_lists - 1 ? low[j] : t;
  return t;
}
// tiles 3, 7, 15, 31, ... of a slab: often while the thresholds still move fast, rarely later
__device__ __forceinline__ bool bound_refresh_due(uint32_t tile_no) { return tile_no >= 3 && (tile_no & (tile_no + 1)) == 0; }

// Global -> LDS staging of one K chunk of a tile (QT query rows, then BT base
// rows) by NT threads.  Rows are staged K-contiguous with pitch KC + 4 floats:
// LDS is written and read 16 bytes at a time without bank conflicts.  The loads
// are unconditional, with addresses clamped into the arrays (conditional loads
// make the compiler wait for every outstanding load at each of them), and are
// issued back to back; what lies outside the arrays is zeroed when the
// registers are written to LDS.  An address is a base common to the workgroup
// (the tile's first row) plus a 32-bit offset of the thread.
template <int QT, int BT, int KC, int NT>
struct TileStager {
  static constexpr int ROWS = QT + BT, P = KC + 4;
  static constexpr int C4 = KC / 4;      // float4 per staged row
  static constexpr int RP = NT / C4;     // rows staged per pass of the workgroup
  static constexpr int NLD = ROWS / RP;  // passes
  static_assert(ROWS % RP == 0 && QT % RP == 0, "a pass is all queries or all base rows");
  const float *q_base, *x;
  float *stage_buf;   // [2][ROWS][P]
  uint64_t b_end;     // end of the slab
  uint32_t d, q_last; // q_last: last row of the batch, counted from the tile's first
  int s_row, s_col;

  __device__ __forceinline__ TileStager(const float *Q, const float *X, float *lds, uint32_t q0, uint32_t nq, uint32_t dim,
                                        uint64_t slab_end, int tid)
      : q_base(Q + (uint64_t)q0 * dim), x(X), stage_buf(lds), b_end(slab_end), d(dim), q_last(nq - 1 - q0),
        s_row(tid / C4), s_col((tid % C4) * 4) {}

  // rows of the tile that starts at base row t0 (at or past the slab's end: clamped loads, nothing kept), columns k0 ..
  __device__ __forceinline__ void fetch(float4 (&reg)[NLD], uint32_t &keep, uint64_t t0, uint32_t k0) const {
    const uint32_t kk = k0 + s_col;
    const bool k_in = kk < d;
    const uint32_t kc = k_in ? kk : 0;
    const uint64_t t0c = t0 < b_end ? t0 : b_end - 1;
    const float *x_base = x + t0c * d;
    const uint64_t left = b_end - 1 - t0c;
    const uint32_t x_last = left < (uint64_t)BT ? (uint32_t)left : (uint32_t)BT;   // last row of the slab, counted from the tile's first
    keep = 0;
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const uint32_t row = (uint32_t)(s_row + RP * i);
      if (row < (uint32_t)QT) {
        const bool in = row <= q_last && k_in;
        reg[i] = *reinterpret_cast<const float4 *>(q_base + ((row < q_last ? row : q_last) * d + kc));
        keep |= in ? 1u << i : 0u;
      } else {
        const uint32_t r = row - QT;
        const bool in = t0 < b_end && r <= x_last && k_in;
        reg[i] = *reinterpret_cast<const float4 *>(x_base + ((r < x_last ? r : x_last) * d + kc));
        keep |= in ? 1u << i : 0u;
      }
    }
  }
  __device__ __forceinline__ void stage(const float4 (&reg)[NLD], uint32_t keep, int b) const {
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const bool in = (keep >> i) & 1u;
      const float4 v = make_float4(in ? reg[i].x : 0.f, in ? reg[i].y : 0.f, in ? reg[i].z : 0.f, in ? reg[i].w : 0.f);
      *reinterpret_cast<float4 *>(stage_buf + ((size_t)b * ROWS + s_row + RP * i) * P + s_col) = v;
    }
  }
};

// ---------------------------------------------------------------------------
// Larger tiles for the common case (d a multiple of 4, moderate k): a
// workgroup of four wavefronts computes 64 WR queries x 64 WC base rows per
// tile, every wavefront a 64 x 64 block as 2 x 2 MFMA 32x32 accumulators, so
// four matrix instructions in a row never wait for each other and one LDS read
// feeds two of them.  Rows are staged K-contiguous (pitch KC + 4 floats: 16-byte
// LDS reads and writes without bank conflicts); the two halves of a wavefront
// take the two halves of a K chunk, which only changes the order in which the
// products are added.  The next chunk is fetched into registers before the
// chunk's matrix work and written to the other LDS buffer after it: one barrier
// per chunk.
//
// Top-k: per query a threshold and a buffer of cb (score, id) entries.  A score
// below the threshold is appended; a row whose buffer is more than half way
// from kp to cb is cut back to its kp best (threshold = the kp-th), by the
// wavefront that owns the row.  An append that finds the buffer full stays
// pending and is tried again after the cut.
template <int WR, int WC, int KC, int EPL>
__global__ __launch_bounds__(256) void bf_block_kernel(const float *__restrict__ X, const float *__restrict__ xnorm,
                                                       uint64_t n, uint32_t d, const float *__restrict__ Q, uint32_t nq,
                                                       uint32_t metric, uint64_t rows_per_slab, uint32_t kp, uint32_t cb,
                                                       uint32_t *__restrict__ bound /*[nq]*/,
                                                       uint32_t *__restrict__ part_best /*[nq][slabs]*/, uint32_t part_rank,
                                                       uint32_t part_lists,
                                                       uint32_t *__restrict__ cand_out /*[nq][slabs][kp]*/) {
  constexpr int QT = 64 * WR, BT = 64 * WC;
  using Stager = TileStager<QT, BT, KC, 256>;
  constexpr int ROWS = Stager::ROWS, P = Stager::P, NLD = Stager::NLD;
  static_assert(WR * WC == 4, "four wavefronts");
  extern __shared__ float smem_f[];
  float *stage_buf = smem_f;                                // [2][ROWS][P]
  float *thr = stage_buf + 2 * ROWS * P;                    // [QT]
  uint32_t *cnt = reinterpret_cast<uint32_t *>(thr + QT);   // [QT]
  uint64_t *buf = reinterpret_cast<uint64_t *>(cnt + QT);   // [QT][cb]

  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const int wr = wave / WC, wc = wave % WC, half = lane / 32, l32 = lane % 32;
  const uint32_t q0 = blockIdx.x * QT;
  const uint32_t slab = blockIdx.y, n_slabs = gridDim.y;
  const uint64_t b_begin = (uint64_t)slab * rows_per_slab;
  const uint64_t b_end = b_begin + rows_per_slab < n ? b_begin + rows_per_slab : n;
  const uint32_t limit = kp + (cb - kp) / 2;   // a longer buffer is cut back

  for (int r = tid; r < QT; r += 256) {
    thr[r] = q0 + r < nq ? INFINITY : -INFINITY;   // rows past the batch never take anything
    cnt[r] = 0;
  }

  const Stager stager(Q, X, stage_buf, q0, nq, d, b_end, tid);
  float4 reg[NLD];
  uint32_t keep = 0;
  // Cut row `row` back to its kp smallest entries (ids differ, so no ties).
  auto cut = [&](int row) {
    const uint32_t c = cnt[row] < cb ? cnt[row] : cb;
    if (c <= kp) {
      if (lane == 0) cnt[row] = c;
      return;
    }
    uint64_t *list = buf + (size_t)row * cb;
    uint64_t mine[EPL];
    uint32_t rank[EPL];
#pragma unroll
    for (int u = 0; u < EPL; ++u) {
      const uint32_t i = lane + u * kWave;
      mine[u] = i < c ? list[i] : ~0ull;
      rank[u] = 0;
    }
    for (uint32_t j = 0; j < c; ++j) {
      const uint64_t o = list[j];
#pragma unroll
      for (int u = 0; u < EPL; ++u) rank[u] += o < mine[u] ? 1u : 0u;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int u = 0; u < EPL; ++u) {
      const uint32_t i = lane + u * kWave;
      if (i < c && rank[u] < kp) {
        list[rank[u]] = mine[u];
        // this slab's part_rank-th best, for the bound over several slabs (see the tile loop)
        if (rank[u] == part_rank - 1 && q0 + row < nq) part_best[(uint64_t)(q0 + row) * n_slabs + slab] = (uint32_t)(mine[u] >> 32);
        if (rank[u] == kp - 1) {
          thr[row] = unorder_f32((uint32_t)(mine[u] >> 32));
          // the kp-th best of one slab bounds the kp-th best overall: the slabs of a query share the smallest
          if (q0 + row < nq) atomicMin(&bound[q0 + row], (uint32_t)(mine[u] >> 32));
        }
      }
    }
    if (lane == 0) cnt[row] = kp;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  };
  // every row over `over` entries is cut by the wavefront that owns it (row % 4 == wave)
  auto cut_rows_over = [&](uint32_t over) {
    const int mine_row = wave + 4 * lane;   // lanes 0 .. QT/4-1 each look at one row
    const bool need = lane < QT / 4 && cnt[mine_row] > over;
    for (uint64_t m = __ballot(need); m; m &= m - 1) cut(wave + 4 * __builtin_ctzll(m));
  };

  const uint32_t n_chunks = (d + KC - 1) / KC;
  const float scale = metric == ANN_L2 ? -2.0f : -1.0f;
  int cur = 0;
  if (b_begin < b_end) {
    stager.fetch(reg, keep, b_begin, 0);
    stager.stage(reg, keep, 0);
  }
  __syncthreads();

  uint32_t tile_no = 0;
  for (uint64_t t0 = b_begin; t0 < b_end; t0 += BT, ++tile_no) {
    // a tighter bound from several slabs' part_rank-th best scores joins the shared bound
    if (bound_refresh_due(tile_no) && tid < QT && q0 + tid < nq) {
      const uint32_t t = bound_over_parts(part_best + (uint64_t)(q0 + tid) * n_slabs, n_slabs, part_lists);
      if (t < 0xFF800000u) atomicMin(&bound[q0 + tid], t);
    }
    floatx16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;
    // norm terms of this lane's two columns; +inf keeps columns past the end out
    float xn[2];
    uint64_t col_id[2];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      col_id[b] = t0 + wc * 64 + b * 32 + l32;
      xn[b] = col_id[b] < b_end ? (metric == ANN_L2 ? xnorm[col_id[b]] : 0.f) : INFINITY;
    }
    // what the other slabs of this thread's query have published (used after the matrix work)
    const uint32_t shared_thr = bound[q0 + tid < nq ? q0 + tid : nq - 1];
    for (uint32_t c = 0; c < n_chunks; ++c) {
      const bool last_chunk = c + 1 == n_chunks;
      const uint64_t nt0 = last_chunk ? t0 + BT : t0;
      const bool more = nt0 < b_end;
      stager.fetch(reg, keep, nt0, last_chunk ? 0 : (c + 1) * KC);   // (no tile left: clamped loads that are never staged)
      const float *ap = stage_buf + ((size_t)cur * ROWS + wr * 64 + l32) * P + half * (KC / 2);
      const float *bp = stage_buf + ((size_t)cur * ROWS + QT + wc * 64 + l32) * P + half * (KC / 2);
#pragma unroll
      for (int j = 0; j < KC / 8; ++j) {
        const float4 a0 = *reinterpret_cast<const float4 *>(ap + 4 * j);
        const float4 a1 = *reinterpret_cast<const float4 *>(ap + 32 * P + 4 * j);
        const float4 b0 = *reinterpret_cast<const float4 *>(bp + 4 * j);
        const float4 b1 = *reinterpret_cast<const float4 *>(bp + 32 * P + 4 * j);
        const float av0[4] = {a0.x, a0.y, a0.z, a0.w}, av1[4] = {a1.x, a1.y, a1.z, a1.w};
        const float bv0[4] = {b0.x, b0.y, b0.z, b0.w}, bv1[4] = {b1.x, b1.y, b1.z, b1.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(av0[e], bv0[e], acc[0][0], 0, 0, 0);
          acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(av0[e], bv1[e], acc[0][1], 0, 0, 0);
          acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(av1[e], bv0[e], acc[1][0], 0, 0, 0);
          acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(av1[e], bv1[e], acc[1][1], 0, 0, 0);
        }
      }
      if (more) stager.stage(reg, keep, cur ^ 1);
      __syncthreads();
      cur ^= 1;
    }

    // acc[a][b][i] is query row wr*64 + a*32 + 8*(i/4) + 4*half + i%4 against
    // base column col_id[b].  Bit b*16 + i of pend[a]: that score is below its
    // row's threshold and not yet in the buffer.
    if (tid < QT && q0 + tid < nq && unorder_f32(shared_thr) < thr[tid]) thr[tid] = unorder_f32(shared_thr);
    __syncthreads();
    uint32_t pend[2] = {0u, 0u};
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float4 t4 = *reinterpret_cast<const float4 *>(thr + wr * 64 + a * 32 + 8 * g + 4 * half);
        const float tv[4] = {t4.x, t4.y, t4.z, t4.w};
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
          for (int b = 0; b < 2; ++b)
            pend[a] |= fmaf(scale, acc[a][b][4 * g + e], xn[b]) < tv[e] ? 1u << (b * 16 + 4 * g + e) : 0u;
      }
    bool any = (pend[0] | pend[1]) != 0;
    if (__syncthreads_or(any ? 1 : 0) == 0) continue;   // nothing for any row of the tile
    for (;;) {
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const uint32_t bit = 1u << (b * 16 + i);
            if (pend[a] & bit) {
              const int row = wr * 64 + a * 32 + 8 * (i / 4) + 4 * half + (i % 4);
              const float score = fmaf(scale, acc[a][b][i], xn[b]);
              if (score < thr[row]) {   // the threshold may have dropped since the bit was set
                const uint32_t pos = atomicAdd(&cnt[row], 1u);
                if (pos < cb) {
                  buf[(size_t)row * cb + pos] = ((uint64_t)order_u32(score) << 32) | (uint32_t)col_id[b];
                  pend[a] &= ~bit;
                }
              } else {
                pend[a] &= ~bit;
              }
            }
          }
      __syncthreads();
      cut_rows_over(limit);
      any = (pend[0] | pend[1]) != 0;
      if (__syncthreads_or(any ? 1 : 0) == 0) break;
    }
  }
  __syncthreads();
  cut_rows_over(kp);
  __syncthreads();
  // hand the survivors of this slab to the exact stage
  for (int e = tid; e < QT * (int)kp; e += 256) {
    const int row = e / kp, j = e % kp;
    const uint32_t qi = q0 + row;
    if (qi < nq)
      cand_out[((uint64_t)qi * n_slabs + slab) * kp + j] = (uint32_t)j < cnt[row] ? (uint32_t)buf[(size_t)row * cb + j] : ANN_PAD_ID;
  }
}


// ---------------------------------------------------------------------------
// Small k: a 128 x 128 tile per workgroup of eight wavefronts (two per SIMD, so
// that one's LDS and barrier waits are covered by the other's matrix work),
// every wavefront a 32 x 64 block (two MFMA 32x32 accumulators), with the top-k
// state owned by single wavefronts so that nothing after the matrix work needs
// a barrier.  Each wavefront keeps, for each of its 32 query rows, its own list
// of the best candidates among the base columns it has seen (two lists per
// query and slab, both handed to the exact stage).
//
// The accumulators take one more matrix step per tile whose only non-zero
// products are 1 x (-|x|^2 / 2) (L2; 0 for inner product; -inf for columns past
// the end), so that score = scale * acc with scale = -2 / -1, and "score below
// the row's threshold" is one compare, acc > u[row] with u = thr / scale.
// Hits are rare once the thresholds have settled: every lane collects a bit
// mask of its hits and the wavefront takes them one per lane and round into
// their rows' lists (LDS atomic for the slot); a list found full is cut back to
// its kp best (rank counting over lanes), which lowers the row's threshold, and
// the hit is tried again.  The lists of one query (its slabs, its two
// wavefronts) publish their thresholds in global memory and use the smallest.
//
// QRES: for rows of up to 128 dimensions the query tile is read into LDS once
// and stays there (K padded to whole chunks, row pitch + 4); only base rows are
// staged with every chunk.  LIST: entries per (row, wavefront) list.
constexpr int kOwnList = 32;     // entries per (row, wavefront) list
constexpr int kOwnListRes = 24;  // the same when the query tile stays in LDS (d <= 128, k <= 10), which leaves less room
constexpr int kOwnWaves = 8, kOwnRows = 32;   // wavefronts per workgroup, query rows per wavefront

// number of set bits of mask below this lane's
__device__ __forceinline__ int bf_lanes_below(uint64_t mask) {
  return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

template <int KC, bool QRES, int LIST>
__global__ __launch_bounds__(512) void bf_own_kernel(const float *__restrict__ X, const float *__restrict__ xnorm,
                                                     uint64_t n, uint32_t d, const float *__restrict__ Q, uint32_t nq,
                                                     uint32_t metric, uint64_t rows_per_slab, uint32_t kp,
                                                     uint32_t *__restrict__ bound /*[nq]*/,
                                                     uint32_t *__restrict__ cand_out /*[nq][slabs][2][kp]*/) {
  constexpr int WC = 2, QT = 128, BT = 128;
  constexpr int QS = QRES ? 0 : QT;   // query rows staged with every chunk (none when the query tile stays in LDS)
  using Stager = TileStager<QS, BT, KC, 64 * kOwnWaves>;
  constexpr int ROWS = Stager::ROWS, P = Stager::P, NLD = Stager::NLD;
  constexpr int NR = kOwnWaves * kOwnRows;   // (row, wavefront) lists per workgroup
  static_assert(kOwnWaves / WC * kOwnRows == QT, "tile shape");
  extern __shared__ float smem_f[];
  // QRES: the 128 queries of the tile stay in LDS for the whole kernel, K padded to whole chunks, row pitch + 4
  const uint32_t q_pitch = (d + KC - 1) / KC * KC + 4;
  float *q_res = smem_f;                                                      // [QT][q_pitch] (QRES)
  float *stage_buf = smem_f + (QRES ? QT * q_pitch : 0);                      // [2][ROWS][P]
  float *u_all = stage_buf + 2 * ROWS * P;                                    // [NR]  acc must exceed this
  uint32_t *thr_all = reinterpret_cast<uint32_t *>(u_all + NR);               // [NR]  ordered score an entry must be below
  uint32_t *cnt_all = thr_all + NR;                                           // [NR]
  uint64_t *list_all = reinterpret_cast<uint64_t *>(cnt_all + NR);            // [NR][LIST]

  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const int wr = wave / WC, wc = wave % WC, half = lane / 32, l32 = lane % 32;
  const uint32_t q0 = blockIdx.x * QT;
  const uint32_t slab = blockIdx.y, n_slabs = gridDim.y;
  const uint64_t b_begin = (uint64_t)slab * rows_per_slab;
  const uint64_t b_end = b_begin + rows_per_slab < n ? b_begin + rows_per_slab : n;
  const float scale = metric == ANN_L2 ? -2.0f : -1.0f;
  const float inv_scale = metric == ANN_L2 ? -0.5f : -1.0f;

  // this wavefront's state (its rows are queries q0 + wr*32 + 0..31)
  float *u = u_all + wave * kOwnRows;
  uint32_t *thr = thr_all + wave * kOwnRows;
  uint32_t *cnt = cnt_all + wave * kOwnRows;
  uint64_t *list = list_all + (size_t)wave * kOwnRows * LIST;
  if (lane < kOwnRows) {
    const bool live = q0 + wr * kOwnRows + lane < nq;
    u[lane] = live ? -INFINITY : INFINITY;   // rows past the batch never take anything
    thr[lane] = order_u32(INFINITY);
    cnt[lane] = 0;
  }

  if (QRES) {
    const uint32_t p4 = (q_pitch - 4) / 4, d4 = d / 4;   // float4 per padded row, per row of Q
    for (uint32_t e = tid; e < QT * p4; e += 64 * kOwnWaves) {
      const uint32_t row = e / p4, c4 = e % p4;
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (q0 + row < nq && c4 < d4) v = reinterpret_cast<const float4 *>(Q + (uint64_t)(q0 + row) * d)[c4];
      *reinterpret_cast<float4 *>(q_res + row * q_pitch + 4 * c4) = v;
    }
  }
  // two sets of staging registers: a chunk is fetched two steps before it is
  // multiplied, so that a row that comes from HBM has two steps to arrive
  const Stager stager(Q, X, stage_buf, q0, nq, d, b_end, tid);
  float4 reg_a[NLD], reg_b[NLD];
  uint32_t keep_a = 0, keep_b = 0;   // bit i: reg[i] lies inside the arrays
  auto wave_sync = [&]() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  };

  // Cut list `row` (c entries, c <= LIST) back to its kp smallest; returns the new length.
  auto cut = [&](int row, uint32_t c) -> uint32_t {
    uint64_t *l = list + (size_t)row * LIST;
    const uint64_t mine = (uint32_t)lane < c ? l[lane < LIST ? lane : 0] : ~0ull;
    const uint32_t mhi = (uint32_t)(mine >> 32), mlo = (uint32_t)mine;
    uint32_t rank = 0;
#pragma unroll
    for (int j = 0; j < LIST; ++j) {
      const uint64_t o = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)mhi, j) << 32) |
                         (uint32_t)__builtin_amdgcn_readlane((int)mlo, j);
      rank += o < mine ? 1u : 0u;   // ids differ, so no two entries are equal
    }
    wave_sync();
    if ((uint32_t)lane < c && rank < kp) {
      l[rank] = mine;
      if (rank == kp - 1) {
        thr[row] = mhi;
        u[row] = unorder_f32(mhi) * inv_scale;
        atomicMin(&bound[q0 + wr * kOwnRows + row], mhi);   // (a list is only ever filled for a query of the batch)
      }
    }
    wave_sync();
    return c < kp ? c : kp;
  };

  const uint32_t n_chunks = (d + KC - 1) / KC;
  int cur = 0;
  // the next (tile, chunk) to fetch; at the top of a step it is two steps ahead
  // and the other register set holds the step in between
  uint64_t f_t0 = b_begin;
  uint32_t f_c = 0;
  auto advance = [&]() {
    if (++f_c == n_chunks) {
      f_c = 0;
      f_t0 += BT;
    }
  };
  if (b_begin < b_end) {
    stager.fetch(reg_a, keep_a, f_t0, 0);
    advance();
    stager.stage(reg_a, keep_a, 0);
    stager.fetch(reg_a, keep_a, f_t0, f_c * KC);   // (past the end: clamped loads that are never staged)
    advance();
  }
  __syncthreads();

  // the tile being multiplied, its chunk, its accumulators
  uint64_t t0 = b_begin;
  uint32_t c = 0;
  floatx16 acc[2];
  float xn[2];         // norm terms of this lane's two columns (loaded at the start of a tile, used at its end)
  uint32_t col_id[2];  // their ids
  uint32_t shared_thr;  // lanes 0..31: the bound other lists have published for this lane's row (same timing)
  const uint32_t my_q = q0 + wr * kOwnRows + (lane < kOwnRows ? lane : 0);
  auto begin_tile = [&]() {
    shared_thr = bound[my_q < nq ? my_q : nq - 1];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[b][i] = 0.f;
      const uint64_t ci = t0 + wc * 64 + b * 32 + l32;
      col_id[b] = (uint32_t)ci;
      xn[b] = xnorm[ci < b_end ? ci : b_end - 1];   // (any readable array of n floats when the metric has no norm term)
    }
  };

  auto finish_tile = [&]() {
    {
      // the extra matrix step: (1, 0) x (ext, 0) over its two K slots
      const float one = half ? 0.f : 1.f;
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        float ext = col_id[b] < b_end ? (metric == ANN_L2 ? -0.5f * xn[b] : 0.f) : -INFINITY;
        if (half) ext = 0.f;
        acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(one, ext, acc[b], 0, 0, 0);
      }
    }
    // The kp-th best score of any list of a query bounds the query's kp-th best
    // overall, so the lists of a query (other slabs, the other wavefront) share
    // the smallest threshold any of them has reached.
    if (lane < kOwnRows && my_q < nq && shared_thr < thr[lane]) {
      thr[lane] = shared_thr;
      u[lane] = unorder_f32(shared_thr) * inv_scale;
    }
    wave_sync();
    // acc[b][i]: row 8*(i/4) + 4*half + i%4 of this wavefront against column col_id[b].
    // Bit 2*i + b of hits: that score is below its row's threshold.
    uint32_t hits = 0;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const float4 u4 = *reinterpret_cast<const float4 *>(u + 8 * g + 4 * half);
      const float uv[4] = {u4.x, u4.y, u4.z, u4.w};
#pragma unroll
      for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int b = 0; b < 2; ++b) hits |= acc[b][4 * g + e] > uv[e] ? 1u << (2 * (4 * g + e) + b) : 0u;
    }
    // One hit per lane and round: into the row's list (LDS atomic for the
    // slot); a list found full is cut back to its kp best, which lowers the
    // row's threshold, and the hit is tried again.
    while (__ballot(hits != 0)) {
      const bool active = hits != 0;
      const int bit = active ? __builtin_ctz(hits) : 0;
      hits &= hits - 1;
      float v = 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int b = 0; b < 2; ++b) v = bit == 2 * i + b ? acc[b][i] : v;
      const int i_el = bit >> 1;
      const int erow = 8 * (i_el >> 2) + 4 * half + (i_el & 3);
      const uint64_t ent = ((uint64_t)order_u32(scale * v) << 32) | (col_id[0] + ((uint32_t)(bit & 1) << 5));   // column b is col_id[0] + 32 b (a select between the two array elements became an indexed read from scratch memory)
      bool pending = active && (uint32_t)(ent >> 32) < thr[erow];
      while (__ballot(pending)) {
        if (pending) {
          const uint32_t pos = atomicAdd(&cnt[erow], 1u);
          if (pos < (uint32_t)LIST) {
            list[(size_t)erow * LIST + pos] = ent;
            pending = false;
          }
        }
        wave_sync();
        uint64_t todo = __ballot(pending);
        if (todo == 0) break;
        while (todo) {
          const int row = __builtin_amdgcn_readlane(erow, __builtin_ctzll(todo));
          todo &= ~__ballot(pending && erow == row);
          const uint32_t left = cut(row, LIST);   // the count ran past the list's end: the list is full
          if (lane == 0) cnt[row] = left;
        }
        wave_sync();
        pending = pending && (uint32_t)(ent >> 32) < thr[erow];
      }
    }
  };

  // One chunk: fetch the chunk two steps ahead into r_fetch, multiply the
  // staged one, stage the next from r_stage.  Returns whether a step follows.
  auto one_step = [&](const float4 (&r_stage)[NLD], uint32_t k_stage, float4 (&r_fetch)[NLD], uint32_t &k_fetch) -> bool {
    const bool last_chunk = c + 1 == n_chunks;
    const bool more = !last_chunk || t0 + BT < b_end;
    stager.fetch(r_fetch, k_fetch, f_t0, f_c * KC);   // (past the end: clamped loads that are never staged)
    advance();
    const float *ap = QRES ? q_res + (size_t)(wr * kOwnRows + l32) * q_pitch + c * KC + half * (KC / 2)
                           : stage_buf + ((size_t)cur * ROWS + wr * kOwnRows + l32) * P + half * (KC / 2);
    const float *bp = stage_buf + ((size_t)cur * ROWS + QS + wc * 64 + l32) * P + half * (KC / 2);
#pragma unroll
    for (int j = 0; j < KC / 8; ++j) {
      const float4 a0 = *reinterpret_cast<const float4 *>(ap + 4 * j);
      const float4 b0 = *reinterpret_cast<const float4 *>(bp + 4 * j);
      const float4 b1 = *reinterpret_cast<const float4 *>(bp + 32 * P + 4 * j);
      const float av0[4] = {a0.x, a0.y, a0.z, a0.w};
      const float bv0[4] = {b0.x, b0.y, b0.z, b0.w}, bv1[4] = {b1.x, b1.y, b1.z, b1.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(av0[e], bv0[e], acc[0], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(av0[e], bv1[e], acc[1], 0, 0, 0);
      }
    }
    if (more) stager.stage(r_stage, k_stage, cur ^ 1);
    __syncthreads();
    cur ^= 1;
    if (last_chunk) {
      finish_tile();
      t0 += BT;
      c = 0;
      if (more) begin_tile();
    } else {
      ++c;
    }
    return more;
  };
  if (b_begin < b_end) {
    begin_tile();
    for (;;) {
      if (!one_step(reg_a, keep_a, reg_b, keep_b)) break;
      if (!one_step(reg_b, keep_b, reg_a, keep_a)) break;
    }
  }
  // every list down to kp, then to the exact stage
  wave_sync();
  for (int row = 0; row < kOwnRows; ++row) {
    uint32_t c = cnt[row] < (uint32_t)LIST ? cnt[row] : (uint32_t)LIST;
    if (c > kp) c = cut(row, c);
    const uint32_t qi = q0 + wr * kOwnRows + row;
    if (qi < nq && (uint32_t)lane < kp) {
      // an entry above what the query's lists have agreed on by now is not among its kp best
      const uint64_t ent = list[(size_t)row * LIST + lane];
      const bool keep = (uint32_t)lane < c && (uint32_t)(ent >> 32) <= bound[qi];
      cand_out[(((uint64_t)qi * n_slabs + slab) * WC + wc) * kp + lane] = keep ? (uint32_t)ent : ANN_PAD_ID;
    }
  }
}

}  // namespace ann

using namespace ann;

extern "C" ann_status ann_bruteforce_topk(const float *x, uint64_t n, uint32_t d, const float *q, uint32_t nq, uint32_t k,
                                          uint32_t metric, uint32_t *out_ids, float *out_dist, void *stream) {
  hipStream_t st = (hipStream_t)stream;
  if (!x || !q || !out_ids || !out_dist) return fail(ANN_EINVAL, "ann_bruteforce_topk: NULL argument");
  if (n == 0 || n >= (1ull << 31) || d == 0 || nq == 0 || k == 0) return fail(ANN_EINVAL, "ann_bruteforce_topk: empty input or n >= 2^31");
  if (metric != ANN_L2 && metric != ANN_IP) return fail(ANN_EINVAL, "ann_bruteforce_topk: unknown metric %u", metric);
  if (k > 256) return fail(ANN_ECAPACITY, "ann_bruteforce_topk: k = %u exceeds 256", k);
  if (d > 2048) return fail(ANN_ECAPACITY, "ann_bruteforce_topk: d = %u exceeds 2048", d);

  const uint32_t kp = k + 8;               // candidates kept per (query, slab): k plus a margin for fp32 score error
  // Tile shape: 128 queries x 128 base rows, with lists owned by single
  // wavefronts for k up to 16 and a shared 64-entry buffer per query for k up
  // to 24; 64 x 256 with a longer buffer for larger k; and the 32 x 128 kernel with scalar staging for what is left (d not a multiple of
  // 4, k above 152).
  int shape = 0;
  uint32_t cb = kp + kBT, q_rows = kQT, b_rows = kBT;
  // rows can be read 16 bytes at a time
  const bool vec4 = d % 4 == 0 && (reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(q)) % 16 == 0;
  uint32_t lists = 1;   // candidate lists per (query, slab)
  if (vec4 && kp + 8 <= (uint32_t)kOwnList) {
    shape = 3;
    cb = kOwnList;
    q_rows = 128;
    b_rows = 128;
    lists = 2;
  } else if (vec4 && kp + 32 <= 64) {
    shape = 1;
    cb = 64;
    q_rows = 128;
    b_rows = 128;
  } else if (vec4 && kp + 32 <= 192) {
    shape = 2;
    cb = kp + 48 <= 192 ? kp + 48 : 192;
    q_rows = 64;
    b_rows = 256;
  }
  if (shape == 0 && cb > 8 * kWave) return fail(ANN_ECAPACITY, "ann_bruteforce_topk: internal buffer too small for k = %u", k);
  const uint32_t q_tiles = (nq + q_rows - 1) / q_rows;
  const uint64_t tiles = (n + b_rows - 1) / b_rows;
  // Slabs of base rows: the grid (query tiles x slabs) should fill the chip a
  // whole number of times - workgroups take equal time, so three left over for
  // a fifth turn cost as much as a full one.  Among 3 to 8 turns take the one
  // whose last turn is fullest (one workgroup per compute unit with the large
  // tiles' LDS, two with the small tile).
  int n_cu = 256;
  {
    int dev = 0;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev);
    if (n_cu <= 0) n_cu = 256;
  }
  const uint32_t slots = (uint32_t)n_cu * (shape == 0 ? 2u : 1u);
  uint32_t slabs = 1;
  double best_fill = 0.0;
  for (uint32_t turns = 3; turns <= 8; ++turns) {
    const uint32_t s_ = slots * turns / q_tiles;
    if (s_ == 0) continue;
    const double fill = (double)q_tiles * s_ / ((double)slots * turns);
    if (fill > best_fill + 0.01) {
      best_fill = fill;
      slabs = s_;
    }
  }
  if (slabs > tiles) slabs = (uint32_t)tiles;
  if (slabs * lists * kp > 4096) slabs = 4096 / (lists * kp);
  if (slabs < 1) slabs = 1;
  uint64_t rows_per_slab = ((tiles + slabs - 1) / slabs) * b_rows;
  slabs = (uint32_t)((n + rows_per_slab - 1) / rows_per_slab);

  float *xnorm = nullptr;
  uint32_t *cand = nullptr;
  size_t smem;
  const void *fn;
  // (short rows and small k: the query tile stays in LDS and only base rows are staged)
  const bool q_res = shape == 3 && d <= 128 && kp + 6 <= (uint32_t)kOwnListRes;
  if (q_res) {
    smem = (size_t)128 * ((d + 31) / 32 * 32 + 4) * sizeof(float) + (size_t)2 * 128 * (32 + 4) * sizeof(float) + 3 * 256 * 4 +
           (size_t)256 * kOwnListRes * sizeof(uint64_t);
    fn = reinterpret_cast<const void *>(bf_own_kernel<32, true, kOwnListRes>);
  } else if (shape == 3) {
    smem = (size_t)2 * 256 * (32 + 4) * sizeof(float) + 3 * 256 * 4 + (size_t)256 * kOwnList * sizeof(uint64_t);
    fn = reinterpret_cast<const void *>(bf_own_kernel<32, false, kOwnList>);
  } else if (shape == 1) {
    smem = (size_t)2 * 256 * (32 + 4) * sizeof(float) + 128 * 8 + (size_t)128 * cb * sizeof(uint64_t);
    fn = reinterpret_cast<const void *>(bf_block_kernel<2, 2, 32, 1>);
  } else if (shape == 2) {
    smem = (size_t)2 * 320 * (16 + 4) * sizeof(float) + 64 * 8 + (size_t)64 * cb * sizeof(uint64_t);
    fn = reinterpret_cast<const void *>(bf_block_kernel<1, 4, 16, 3>);
  } else {
    smem = (size_t)2 * (kQT + kBT) * kLd * sizeof(float) + kQT * (sizeof(float) + sizeof(uint32_t)) +
           (size_t)kQT * cb * sizeof(uint64_t);
    fn = vec4 ? reinterpret_cast<const void *>(bf_tile_kernel<true>) : reinterpret_cast<const void *>(bf_tile_kernel<false>);
  }
  hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (e != hipSuccess) return hip_fail(e, "hipFuncSetAttribute");
  // candidates, then one shared bound per query (the large-tile kernels)
  const size_t n_cand_words = (size_t)nq * slabs * lists * kp;
  // (then, for the 4-wavefront kernels, every slab's part_rank-th best per query: see bound_over_parts; in the
  // 8-wavefront kernel the loads of that bound cost more than the few hits it would save)
  const uint32_t part_lists = slabs < 8 ? slabs : 8;
  const uint32_t part_rank = (kp + part_lists - 1) / part_lists;
  const size_t n_part_words = shape == 1 || shape == 2 ? (size_t)nq * slabs : 0;
  ANN_HIP(hipMalloc((void **)&cand, (n_cand_words + nq + n_part_words) * sizeof(uint32_t)));
  uint32_t *bound = cand + n_cand_words;
  uint32_t *part_best = bound + nq;
  if (shape != 0) {
    const size_t n_fill = nq + n_part_words;
    fill_u32_kernel<<<(uint32_t)((n_fill + 255) / 256), 256, 0, st>>>(bound, (uint32_t)n_fill, 0xFF800000u);   // +inf in score order
  }
  if (metric == ANN_L2) {
    e = hipMalloc((void **)&xnorm, (size_t)n * sizeof(float));
    if (e != hipSuccess) {
      (void)hipFree(cand);
      return hip_fail(e, "hipMalloc");
    }
    row_norm_kernel<<<2048, 256, 0, st>>>(x, n, d, xnorm);
  }
  const dim3 grid(q_tiles, slabs);
  if (q_res)
    bf_own_kernel<32, true, kOwnListRes><<<grid, 64 * kOwnWaves, smem, st>>>(x, metric == ANN_L2 ? xnorm : x, n, d, q, nq, metric,
                                                                             rows_per_slab, kp, bound, cand);
  else if (shape == 3)
    bf_own_kernel<32, false, kOwnList><<<grid, 64 * kOwnWaves, smem, st>>>(x, metric == ANN_L2 ? xnorm : x, n, d, q, nq, metric,
                                                                            rows_per_slab, kp, bound, cand);
  else if (shape == 1)
    bf_block_kernel<2, 2, 32, 1><<<grid, 256, smem, st>>>(x, xnorm, n, d, q, nq, metric, rows_per_slab, kp, cb, bound, part_best,
                                                          part_rank, part_lists, cand);
  else if (shape == 2)
    bf_block_kernel<1, 4, 16, 3><<<grid, 256, smem, st>>>(x, xnorm, n, d, q, nq, metric, rows_per_slab, kp, cb, bound, part_best,
                                                          part_rank, part_lists, cand);
  else if (vec4)
    bf_tile_kernel<true><<<grid, 256, smem, st>>>(x, xnorm, n, d, q, nq, metric, rows_per_slab, kp, cb, cand);
  else
    bf_tile_kernel<false><<<grid, 256, smem, st>>>(x, xnorm, n, d, q, nq, metric, rows_per_slab, kp, cb, cand);
  e = hipGetLastError();
  ann_status rc = e == hipSuccess ? rerank_device(x, n, d, metric, q, nq, cand, slabs * lists * kp, slabs * lists * kp, k, out_ids,
                                                  out_dist, st)
                                  : hip_fail(e, "brute-force tile kernel launch");
  hipError_t e2 = hipStreamSynchronize(st);
  (void)hipFree(cand);
  (void)hipFree(xnorm);
  if (rc != ANN_OK) return rc;
  if (e2 != hipSuccess) return hip_fail(e2, "hipStreamSynchronize");
  return ANN_OK;
}
