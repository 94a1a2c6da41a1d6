// Batched best-first graph search: Algorithm 1 of the paper ("Deterministic
// Access Greedy Search"), one query per wavefront.
//
// Mapping of the algorithm's steps onto a 64-lane wavefront:
//   pool C          sorted array of (key, id) pairs spread over the lanes'
//                   registers (lane l holds entries l*M .. l*M+M-1); the
//                   "expanded" mark is bit 31 of the id.
//   visited set V   open-addressing hash table in LDS, test-and-set by CAS.
//   for j in G_i    one lane per adjacency slot: all ids of the row are
//                   tested against V first, survivors are compacted (the
//                   "deterministic access" batch filter), and only their code
//                   rows are fetched.
//   tau_l           LPR lanes share one code row, 16 bytes per lane; packed
//                   int8 dot products, reduced across the lanes with DPP.
//   insert          candidates are inserted one at a time, each by a
//                   wave-wide compare and a one-position shift.
// The pool after a step is the ef smallest (key, id) pairs among the old pool
// and the row's new candidates, which is what sequential insertion in row
// order gives; so results equal a sequential execution bit for bit.
#include "ann_internal.hpp"
#include "device_utils.hpp"

namespace ann {

constexpr uint32_t kEmpty = 0xFFFFFFFFu;
constexpr uint32_t kFlag = 0x80000000u;
constexpr uint32_t kIdMask = 0x7FFFFFFFu;

struct SearchArgs {
  const uint8_t *codes;
  const float *norm_term;
  const uint32_t *adjacency;
  const uint8_t *tq;
  const float *s;
  const float *qlo;
  const int32_t *sum_t;
  const uint32_t *entry_ids;
  uint32_t *out_ids;
  float *out_keys;
  int32_t *out_idot;
  uint32_t *out_counts;
  uint64_t n;
  uint32_t row_stride, n_chunks, degree, metric, tq_stride, n_entry, entry_point, ef, vis_log2, nq;
};

__device__ __forceinline__ uint64_t pack64(uint32_t hi, uint32_t lo) { return ((uint64_t)hi << 32) | lo; }

template <int BITS, int LPR, int M>
struct SearchWave {
  static constexpr int G = kWave / LPR;  // code rows evaluated side by side
  static constexpr int U = 4;            // row loads in flight per lane
  static constexpr int TQW = TqRegs<BITS>::kWords;

  const SearchArgs &a;
  uint32_t *vis;   // LDS [cap]
  uint32_t *cand;  // LDS [64]
  int lane, chunk, grp;
  uint32_t vis_mask, vis_shift, vis_limit;
  int tq[TQW];
  float s, qlo;
  int bias;
  uint32_t pk[M], pid[M];  // pool: ordered key bits, id | expanded flag
  uint64_t worst;          // (key,id) of pool entry ef-1
  uint32_t n_exp = 0, n_dist = 0, n_vis = 0, n_rebuild = 0;

  __device__ SearchWave(const SearchArgs &args, uint32_t *smem) : a(args) {
    lane = lane_id();
    chunk = lane % LPR;
    grp = lane / LPR;
    const uint32_t cap = 1u << a.vis_log2;
    vis = smem;
    cand = smem + cap;
    vis_mask = cap - 1;
    vis_shift = 32 - a.vis_log2;
    vis_limit = cap - cap / 4;
  }

  __device__ __forceinline__ void clear_table() {
    for (uint32_t i = lane; i <= vis_mask; i += kWave) vis[i] = kEmpty;
  }

  // true if id was not in the table (and now is)
  __device__ __forceinline__ bool test_and_set(uint32_t id) {
    uint32_t slot = (id * 0x9E3779B1u) >> vis_shift;
    for (;;) {
      uint32_t old = atomicCAS(&vis[slot], kEmpty, id);
      if (old == kEmpty) return true;
      if (old == id) return false;
      slot = (slot + 1) & vis_mask;
    }
  }

  // The table holds every node whose key has been evaluated, as long as it
  // fits.  When it is about to pass 3/4 load it is rebuilt from the pool.  A
  // forgotten node is outside the pool, so it was rejected or evicted by a
  // pool maximum that has only decreased since: re-evaluating it yields the
  // same key and the same rejection.  Results do not change; work is repeated.
  __device__ __forceinline__ void rebuild_table() {
    __syncthreads();
    clear_table();
    __syncthreads();
    int kept = 0;
#pragma unroll
    for (int r = 0; r < M; ++r)
      if (pk[r] != kEmpty) {
        test_and_set(pid[r] & kIdMask);
        ++kept;
      }
    n_vis = (uint32_t)group_sum_i32<64>(kept);
    ++n_rebuild;
    __syncthreads();
  }

  __device__ __forceinline__ void refresh_worst() {
    const int g = (int)a.ef - 1, rl = g / M, rr = g % M;
    uint32_t k_ = pk[0], i_ = pid[0];
#pragma unroll
    for (int r = 1; r < M; ++r) {
      k_ = (rr == r) ? pk[r] : k_;
      i_ = (rr == r) ? pid[r] : i_;
    }
    worst = pack64(__builtin_amdgcn_readlane(k_, rl), __builtin_amdgcn_readlane(i_, rl) & kIdMask);
  }

  // Insert (cku, cid), known to be smaller than `worst`; all arguments are
  // wave-uniform.
  __device__ __forceinline__ void insert(uint32_t cku, uint32_t cid) {
    const uint64_t c64 = pack64(cku, cid);
    int cnt = 0;
#pragma unroll
    for (int r = 0; r < M; ++r) cnt += (pack64(pk[r], pid[r] & kIdMask) < c64) ? 1 : 0;
    const uint64_t open = __ballot(cnt < M);  // lanes that hold an entry >= candidate
    const int L = __builtin_ctzll(open);
    const int p = L * M + __builtin_amdgcn_readlane(cnt, L);
    const uint32_t upk = (uint32_t)dpp_i32<kDppWaveShr1>((int)pk[M - 1]);
    const uint32_t upid = (uint32_t)dpp_i32<kDppWaveShr1>((int)pid[M - 1]);
#pragma unroll
    for (int r = M - 1; r >= 0; --r) {
      const int g = lane * M + r;
      const uint32_t sk = r > 0 ? pk[r > 0 ? r - 1 : 0] : upk;
      const uint32_t si = r > 0 ? pid[r > 0 ? r - 1 : 0] : upid;
      uint32_t nk = g > p ? sk : pk[r];
      uint32_t ni = g > p ? si : pid[r];
      nk = g == p ? cku : nk;
      ni = g == p ? cid : ni;
      const bool beyond = g >= (int)a.ef;  // the entry pushed past ef is dropped
      pk[r] = beyond ? kEmpty : nk;
      pid[r] = beyond ? kEmpty : ni;
    }
    refresh_worst();
  }

  __device__ __forceinline__ void insert_candidates(bool have, uint32_t ku, uint32_t id) {
    uint64_t m = __ballot(have && pack64(ku, id) < worst);
    while (m) {
      const int l = __builtin_ctzll(m);
      m &= m - 1;
      const uint32_t k_ = __builtin_amdgcn_readlane(ku, l), i_ = __builtin_amdgcn_readlane(id, l);
      if (pack64(k_, i_) < worst) insert(k_, i_);
    }
  }

  // Integer dot products for the code rows of up to G*U nodes listed in
  // cand[base ..]; lane (grp, chunk 0) of each group gets the full sum.
  __device__ __forceinline__ void row_dots(int base, int count, int (&dot)[U], float (&nrm)[U], uint32_t (&vid)[U]) {
    uint4 rows[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int ci = base + u * G + grp;
      vid[u] = ci < count ? cand[ci] : kEmpty;
      rows[u] = make_uint4(0, 0, 0, 0);
      nrm[u] = 0.0f;
      if (vid[u] != kEmpty) {
        if (chunk < (int)a.n_chunks)
          rows[u] = *reinterpret_cast<const uint4 *>(a.codes + (uint64_t)vid[u] * a.row_stride + (uint32_t)chunk * 16u);
        if (a.norm_term && chunk == 0) nrm[u] = a.norm_term[vid[u]];
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) dot[u] = group_sum_i32<LPR>(chunk_dot<BITS>(rows[u], tq)) + bias;
  }

  // Visited filter, compaction, distance evaluation and pool insertion for one
  // list of node ids (an adjacency row or the initial nodes), one id per lane.
  __device__ __forceinline__ void process_ids(uint32_t nb) {
    bool valid = nb != kEmpty && nb < a.n;
    const uint32_t incoming = (uint32_t)__popcll(__ballot(valid));
    if (n_vis + incoming > vis_limit) rebuild_table();
    const bool fresh = valid && test_and_set(nb);
    const uint64_t fm = __ballot(fresh);
    const int count = __popcll(fm);
    if (count == 0) return;
    n_vis += count;
    n_dist += count;
    const int rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(fm >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)fm, 0));
    if (fresh) cand[rank] = nb;
    __syncthreads();
    for (int base = 0; base < count; base += G * U) {
      int dot[U];
      float nrm[U];
      uint32_t vid[U];
      row_dots(base, count, dot, nrm, vid);
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const float key = key_from_idot(a.metric, s, qlo, dot[u], nrm[u]);
        insert_candidates(chunk == 0 && vid[u] != kEmpty, order_u32(key), vid[u]);
      }
    }
    __syncthreads();
  }

  __device__ void run(uint32_t qi) {
    // this lane's share of the folded query
    const int *tqp = reinterpret_cast<const int *>(a.tq + (uint64_t)qi * a.tq_stride + (uint32_t)chunk * (TQW * 4u));
#pragma unroll
    for (int w = 0; w < TQW; ++w) tq[w] = tqp[w];
    s = a.s[qi];
    qlo = a.qlo[qi];
    bias = BITS == 8 ? 128 * a.sum_t[qi] : 0;
#pragma unroll
    for (int r = 0; r < M; ++r) {
      pk[r] = kEmpty;
      pid[r] = kEmpty;
    }
    worst = pack64(kEmpty, kIdMask);
    clear_table();
    __syncthreads();

    // initial nodes I: into the pool and into V
    uint32_t nb = kEmpty;
    if (a.entry_ids) {
      if (lane < (int)a.n_entry) nb = a.entry_ids[(uint64_t)qi * a.n_entry + lane];
    } else if (lane == 0) {
      nb = a.entry_point;
    }
    process_ids(nb);

    for (;;) {
      // closest un-expanded pool entry
      int first = M;
#pragma unroll
      for (int r = M - 1; r >= 0; --r) first = (pid[r] & kFlag) ? first : r;
      const uint64_t has = __ballot(first < M);
      if (has == 0) break;
      const int L = __builtin_ctzll(has);
      const int rr = __builtin_amdgcn_readlane(first, L);
      uint32_t sel = pid[0];
#pragma unroll
      for (int r = 1; r < M; ++r) sel = (rr == r) ? pid[r] : sel;
      const uint32_t uid = __builtin_amdgcn_readlane(sel, L);
#pragma unroll
      for (int r = 0; r < M; ++r)
        if (lane == L && r == rr) pid[r] |= kFlag;
      ++n_exp;
      nb = lane < (int)a.degree ? a.adjacency[(uint64_t)uid * a.degree + lane] : kEmpty;
      process_ids(nb);
    }

    // results: stage the pool through LDS (the visited table is dead now) so
    // that global writes are coalesced
    __syncthreads();
    uint32_t *st_id = vis, *st_key = vis + a.ef;
    int kept = 0;
#pragma unroll
    for (int r = 0; r < M; ++r) {
      const int g = lane * M + r;
      if (g < (int)a.ef) {
        st_id[g] = pk[r] == kEmpty ? kEmpty : (pid[r] & kIdMask);
        st_key[g] = pk[r];
      }
      kept += pk[r] != kEmpty ? 1 : 0;
    }
    kept = group_sum_i32<64>(kept);
    __syncthreads();
    for (uint32_t i = lane; i < a.ef; i += kWave) {
      a.out_ids[(uint64_t)qi * a.ef + i] = st_id[i];
      if (a.out_keys) a.out_keys[(uint64_t)qi * a.ef + i] = st_key[i] == kEmpty ? INFINITY : unorder_f32(st_key[i]);
    }
    if (a.out_idot) {
      for (int base = 0; base < (int)a.ef; base += G * U) {
        // same arithmetic as during traversal, over the final pool
        uint4 rows[U];
        uint32_t vid[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int ci = base + u * G + grp;
          vid[u] = ci < (int)a.ef ? st_id[ci] : kEmpty;
          rows[u] = make_uint4(0, 0, 0, 0);
          if (vid[u] != kEmpty && chunk < (int)a.n_chunks)
            rows[u] = *reinterpret_cast<const uint4 *>(a.codes + (uint64_t)vid[u] * a.row_stride + (uint32_t)chunk * 16u);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int dot = group_sum_i32<LPR>(chunk_dot<BITS>(rows[u], tq)) + bias;
          const int ci = base + u * G + grp;
          if (chunk == 0 && ci < (int)a.ef) a.out_idot[(uint64_t)qi * a.ef + ci] = vid[u] != kEmpty ? dot : 0;
        }
      }
    }
    if (a.out_counts && lane == 0) {
      uint32_t *c = a.out_counts + (uint64_t)qi * 4;
      c[0] = n_exp;
      c[1] = n_dist;
      c[2] = (uint32_t)kept;
      c[3] = n_rebuild;
    }
  }
};

template <int BITS, int LPR, int M>
__global__ __launch_bounds__(64) void search_exact_kernel(SearchArgs args) {
  extern __shared__ uint32_t smem[];
  const uint32_t qi = blockIdx.x;
  if (qi >= args.nq) return;
  SearchWave<BITS, LPR, M> w(args, smem);
  w.run(qi);
}

template <int BITS, int LPR>
static ann_status launch_m(const SearchArgs &args, int m, size_t smem, hipStream_t st) {
  switch (m) {
    case 1: search_exact_kernel<BITS, LPR, 1><<<args.nq, 64, smem, st>>>(args); break;
    case 2: search_exact_kernel<BITS, LPR, 2><<<args.nq, 64, smem, st>>>(args); break;
    case 4: search_exact_kernel<BITS, LPR, 4><<<args.nq, 64, smem, st>>>(args); break;
    case 8: search_exact_kernel<BITS, LPR, 8><<<args.nq, 64, smem, st>>>(args); break;
    default: return fail(ANN_EUNSUPPORTED, "no kernel for pool registers per lane = %d", m);
  }
  ANN_HIP(hipGetLastError());
  return ANN_OK;
}

template <int BITS>
static ann_status launch_lpr(const SearchArgs &args, uint32_t lpr, int m, size_t smem, hipStream_t st) {
  switch (lpr) {
    case 8: return launch_m<BITS, 8>(args, m, smem, st);
    case 16: return launch_m<BITS, 16>(args, m, smem, st);
    case 32: return launch_m<BITS, 32>(args, m, smem, st);
    case 64: return launch_m<BITS, 64>(args, m, smem, st);
    default: return fail(ANN_EUNSUPPORTED, "no kernel for %u lanes per code row", lpr);
  }
}

}  // namespace ann

using namespace ann;

extern "C" ann_status ann_search_batch(ann_index *index, const float *q, uint32_t nq, const ann_search_params *params,
                                       const uint32_t *entry_ids, uint32_t n_entry, uint32_t *out_ids, float *out_keys,
                                       int32_t *out_idot, uint32_t *out_counts, void *stream) {
  hipStream_t st = (hipStream_t)stream;
  if (!index || !q || !params || !out_ids) return fail(ANN_EINVAL, "ann_search_batch: NULL argument");
  if (nq == 0) return fail(ANN_EINVAL, "ann_search_batch: nq == 0");
  if (params->k == 0) return fail(ANN_EINVAL, "ann_search_batch: k == 0");
  if (params->ef < params->k) return fail(ANN_EINVAL, "ann_search_batch: ef = %u < k = %u", params->ef, params->k);
  if (params->ef > ANN_MAX_EF) return fail(ANN_ECAPACITY, "ann_search_batch: ef = %u exceeds ANN_MAX_EF = %u", params->ef, ANN_MAX_EF);
  if (params->reserved[0] || params->reserved[1] || params->reserved[2]) return fail(ANN_EINVAL, "ann_search_batch: reserved fields must be zero");
  if (params->mode > 1) return fail(ANN_EINVAL, "ann_search_batch: unknown mode %u", params->mode);
  if (params->mode == 1) return fail(ANN_EUNSUPPORTED, "ann_search_batch: multi-expansion mode is not built yet");
  if (entry_ids && n_entry == 0) return fail(ANN_EINVAL, "ann_search_batch: entry_ids given with n_entry == 0");
  if (entry_ids && n_entry > ANN_MAX_ENTRIES) return fail(ANN_ECAPACITY, "ann_search_batch: n_entry = %u exceeds ANN_MAX_ENTRIES = %u", n_entry, ANN_MAX_ENTRIES);

  const uint32_t ef = params->ef;
  uint32_t need = 2 * (ef + 64), min_log2 = 0;
  while ((1u << min_log2) < need) ++min_log2;
  uint32_t vis_log2;
  if (params->visited_slots == 0) {
    // default: room for the evaluations a search of this ef typically makes
    uint32_t want = 16 * ef < 4096 ? 4096 : 16 * ef;
    vis_log2 = 0;
    while ((1u << vis_log2) < want) ++vis_log2;
    if (vis_log2 < min_log2) vis_log2 = min_log2;
  } else {
    uint32_t v = params->visited_slots;
    if (v & (v - 1)) return fail(ANN_EINVAL, "ann_search_batch: visited_slots = %u is not a power of two", v);
    vis_log2 = 0;
    while ((1u << vis_log2) < v) ++vis_log2;
    if (vis_log2 < min_log2) return fail(ANN_EINVAL, "ann_search_batch: visited_slots = %u is below the minimum %u for ef = %u", v, 1u << min_log2, ef);
    if (vis_log2 > 13) return fail(ANN_ECAPACITY, "ann_search_batch: visited_slots = %u exceeds 8192", v);
  }

  ann_status rc = launch_query_prep(index, 0, q, nq, nullptr, nullptr, nullptr, st);
  if (rc != ANN_OK) return rc;

  const LevelDev &L = index->level[0];
  const Workspace &w = index->ws[0];
  SearchArgs a{};
  a.codes = L.codes;
  a.norm_term = index->metric == ANN_L2 ? L.norm_term : nullptr;
  a.adjacency = index->adjacency;
  a.tq = w.tq;
  a.s = w.s;
  a.qlo = w.qlo;
  a.sum_t = w.sum_t;
  a.entry_ids = entry_ids;
  a.out_ids = out_ids;
  a.out_keys = out_keys;
  a.out_idot = out_idot;
  a.out_counts = out_counts;
  a.n = index->n;
  a.row_stride = L.row_stride;
  a.n_chunks = L.row_stride / 16;
  a.degree = index->degree;
  a.metric = index->metric;
  a.tq_stride = w.tq_stride;
  a.n_entry = entry_ids ? n_entry : 0;
  a.entry_point = index->entry_point;
  a.ef = ef;
  a.vis_log2 = vis_log2;
  a.nq = nq;
  int m = 1;
  while (64 * m < (int)ef) m <<= 1;
  const size_t smem = ((size_t)(1u << vis_log2) + 64) * sizeof(uint32_t);
  return L.bits == 8 ? launch_lpr<8>(a, L.lanes_per_row, m, smem, st) : launch_lpr<4>(a, L.lanes_per_row, m, smem, st);
}
