// Batched best-first graph search: Algorithm 1 of the paper ("Deterministic
// Access Greedy Search"), one query per wavefront.
//
// Mapping of the algorithm's steps onto a 64-lane wavefront:
//   pool C          sorted array of (key, id) pairs in registers, striped:
//                   entry i lives in register i/64 of lane i%64.  The low word
//                   is (id << 1) | expanded, so pairs compare as plain u64.
//   visited set V   in LDS, either a two-way cache of node ids (one or two
//                   exchanges per test, may forget) or an open-addressing hash
//                   table with test-and-set by CAS (complete while it fits).
//   for j in G_i    one lane per adjacency slot: all ids of the row are
//                   tested against V first, survivors are compacted (the
//                   "deterministic access" batch filter), and only their code
//                   rows are fetched.
//   tau_l           LPR lanes share one code row, four 16-byte chunks per lane
//                   (interleaved, so one load instruction reads LPR*16
//                   contiguous bytes of each row); packed int8 dot products,
//                   reduced across the LPR lanes with DPP.  128-byte rows: two
//                   lanes per row, 32 rows per instruction group.
//   insert          all candidates of a step that beat the pool's last entry
//                   are merged at once: each candidate finds its rank among
//                   the pool entries by binary search in a sorted LDS copy of
//                   the pool and its rank among the other candidates by
//                   counting; each pool entry moves up by the number of
//                   candidates below it (prefix sums over a histogram of the
//                   candidates' ranks); both scatter to their final positions
//                   through LDS, which leaves the next sorted copy behind.
// The pool after a step is the ef smallest (key, id) pairs among the old pool
// and the step's new candidates, which is what sequential insertion in row
// order gives; so with one expansion per step results equal a sequential
// execution bit for bit.  With P > 1 expansions per step the P closest
// un-expanded entries are expanded together (rows filtered in that order).
#pragma once
// Tuning constants (measured on the 1M x 128 8-bit workload; a build may override them):
// Wavefronts per SIMD a kernel is compiled for set its register budget (512 / n, in eights).  LDS is handed
// out in blocks of 1,280 bytes, 128 to a compute unit: 5 blocks (up to 6,400 B) let 25 one-wavefront workgroups
// stay resident, 6 blocks 21, 4 blocks 32.  Measured: the multi-expansion kernels need their 80 (four
// expansions) and 96 (eight) registers - compiled for one wavefront more they spill and run 15-17 % slower.
#ifndef ANN_WPE_EXACT
#define ANN_WPE_EXACT 7  // one expansion per step, FAST kernels (72 registers)
#endif
#ifndef ANN_WPE_WIDE
#define ANN_WPE_WIDE 5  // eight expansions per step, FAST kernels (96 registers)
#endif
#ifndef ANN_U
#define ANN_U 2  // groups of code rows requested together in the multi-expansion kernels
#endif
#ifndef ANN_FEW
#define ANN_FEW 4  // up to this many candidates are merged by merge_few(), more by merge()
#endif
#ifndef ANN_WPE
#define ANN_WPE 6  // wavefronts per SIMD the 8-bit multi-expansion FAST kernels are compiled for
#endif
#include "ann_internal.hpp"
#include "device_utils.hpp"

namespace ann {

constexpr uint32_t kEmpty = 0xFFFFFFFFu;

struct SearchArgs {
  const uint8_t *codes;
  const float *norm_term;
  const uint32_t *adjacency;
  const uint8_t *tq;
  const float *s;
  const float *qlo;
  const int32_t *sum_t;
  const int32_t *sum_t_lo;  // second plane's sums (15-bit query) or nullptr
  const uint32_t *entry_ids;
  const uint32_t *order;  // processing order (workgroup -> query) or nullptr
  const uint32_t *ef_per_query;  // [nq] pool size of each query (<= ef) or nullptr
  const float *labels;  // [n][degree] edge labels or nullptr
  const uint8_t *prs_codes;  // [n][degree][row_stride] code rows of every node's neighbours, or nullptr
  const float *prs_norm;     // [n][degree] their norm terms (L2), or nullptr
  uint32_t *out_ids;
  float *out_keys;
  int32_t *out_idot;
  uint32_t *out_counts;
  uint64_t n;
  uint32_t row_stride, n_chunks, degree, metric, tq_stride, n_entry, entry_point, ef, vis_log2, nq, p;
  uint32_t filtered;  // the label test and/or the per-expansion cap m_s is active
  uint32_t vis_cache;  // visited set is the two-way cache
  uint32_t vis_packed;  // the cache keeps 16-bit tags, two ways to a word (needs (n - 1 >> vis_log2) + 1 < 0xFFFF)
  uint32_t m_s;
  uint32_t tq_plane;   // bytes of one plane of a folded query (tq_stride: one plane, or two for the 15-bit query)
  uint32_t q15;        // the folded query has 15 bits: two byte planes, keys from both dot products
  uint32_t prs_slots;  // slots of every adjacency row whose code rows are in prs_codes (the first prs_slots)
  uint32_t adj_stride;  // words from one adjacency row to the next: degree, or 2 * degree with adj_norms
  uint32_t adj_norms;   // every adjacency row is followed by the norm terms of its neighbours, in slot order
  float alpha_s;
};

// A workgroup of these kernels is one wavefront, and a wavefront's LDS
// instructions are carried out in the order they were issued: what one lane
// wrote is there for any lane's later read.  So all that is needed between a
// write and a dependent read by another lane is that the compiler keeps the
// two in program order - no barrier instruction and no wait for global loads
// that are still in flight (which a workgroup barrier implies).
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

__device__ __forceinline__ uint64_t pack64(uint32_t hi, uint32_t lo) { return ((uint64_t)hi << 32) | lo; }

__device__ __forceinline__ int lanes_below(uint64_t mask) {
  return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
}

// The merge scatter buffer: the sorted pool, 64 m slots.  A merge scatters the
// old entries and the candidates to their new ranks (ranks past the buffer
// are dropped) and so leaves the new pool in order.
__host__ __device__ constexpr int merge_buf_entries(int m) { return 64 * m; }
// Staging area of a step's qualifying candidates; during a merge (candidates
// are in registers then) it serves as integer counters.  In the FAST kernels
// it also holds the step's unvisited ids, in the upper word of entry i (the
// lower word: the node's norm term where it came with the adjacency row):
// entry j is written only after id j has been read.
// With one expansion per step a step has at most ANN_MAX_DEGREE = 64 candidates.
__host__ __device__ constexpr int stage_entries(int m, int pmax, bool fast) {
  return pmax == 1 ? 64 : (fast && 32 * pmax > 64 * m ? 32 * pmax : 64 * m);
}
// During a merge the area holds 64 m integer counters (32 m entries).  The
// list of the batch's candidates (64 and 4 of padding) lies in the merge
// buffer itself when that has 128 entries or more: the buffer's old contents
// are not read again once the candidates are ranked, and the scatter that
// ends the merge rewrites every slot of it.  With 64 entries the list follows
// the counters.
__host__ __device__ constexpr int merge_list_at(int m) { return 32 * m; }
__host__ __device__ constexpr int stage_area_entries(int m, int pmax, bool fast) {
  const int need = m >= 2 ? merge_list_at(m) : merge_list_at(m) + 68;
  return stage_entries(m, pmax, fast) > need ? stage_entries(m, pmax, fast) : need;
}

// Ids of one step's unvisited neighbours: up to pmax rows of `degree` ids.
__host__ __device__ inline uint32_t cand_entries(uint32_t degree, int pmax) {
  return (degree <= 32 ? 32u : 64u) * (uint32_t)pmax;
}

// LDS bytes for one query: merge buffer, staging, visited set, candidate ids, folded query.
__host__ __device__ inline size_t search_smem_bytes(int m, int pmax, bool fast, uint32_t vis_log2, uint32_t degree,
                                                    uint32_t tq_stride) {
  return (size_t)(merge_buf_entries(m) + stage_area_entries(m, pmax, fast)) * 8 + ((size_t)1 << vis_log2) * 4 +
         (fast ? 0 : (size_t)cand_entries(degree, pmax) * 8) + tq_stride;
}

// FAST: the configuration that matters for throughput, with the run-time
// switches folded away (two-way visited cache, no edge filter, plain
// layout, PMAX expansions per step; degree <= 32 when PMAX > 1, degree <= 64
// with four or more pool registers per lane).  The general
// kernel (FAST = false) takes every switch from SearchArgs.
template <int BITS, int LPR, int M, int PMAX, bool FAST>
struct SearchWave {
  static constexpr int G = kWave / LPR;      // code rows evaluated side by side
  static constexpr int CPL = 4;              // 16-byte chunks of a row per lane
  // groups of G rows in flight.  With one expansion per step and wide rows
  // (eight or more lanes to a row) a group is fewer rows than a step has
  // candidates, so two are requested together (1M x 960 4-bit: 6 % faster;
  // four groups, or four in the multi-expansion kernels, cost more in
  // registers than they gain)
  static constexpr int U = PMAX > 1 ? ANN_U : (LPR >= 8 ? 2 : 1);
  static constexpr int TQW = TqRegs<BITS>::kWords;

  // the i-th unvisited neighbour of the current step: id in the upper word,
  // in the lower one the bits of its norm term if that came with the row
  __device__ __forceinline__ uint64_t &cand_at(int i) const { return cand[i]; }
  // Slot `slot` of node u's adjacency row: the neighbour's id and, where the
  // rows carry them, the bits of its norm term.  The norm terms follow the ids
  // as a block of their own (ids first: the visited filter can start when the
  // first 4 * degree bytes have arrived; measured against (id, norm) pairs, which
  // cost the one-expansion-per-step kernel 4 % more).
  __device__ __forceinline__ void load_slot(uint32_t u, int slot, uint32_t &id, uint32_t &nrm) const {
    const uint32_t *row = a.adjacency + (uint64_t)u * a.adj_stride;
    id = row[slot];
    nrm = a.adj_norms ? row[a.degree + slot] : 0u;
  }

  __device__ __forceinline__ bool use_cache() const { return FAST || a.vis_cache != 0; }
  __device__ __forceinline__ bool use_packed() const { return FAST || a.vis_packed != 0; }
  __device__ __forceinline__ bool use_prs() const { return !FAST && a.prs_codes != nullptr; }
  __device__ __forceinline__ bool use_filter() const { return !FAST && a.filtered != 0; }
  // two adjacency rows of at most 32 slots per pass (FAST kernels with up to
  // two pool registers per lane are only launched for such degrees: their
  // staging area holds 32 PMAX ids; with four or more it holds 64 PMAX)
  __device__ __forceinline__ bool use_pairs() const { return PMAX > 1 && ((FAST && M < 4) || a.degree <= 32); }

  const SearchArgs &a;
  uint64_t *mbuf;   // LDS: sorted copy of the pool as of the last merge; merge scatter buffer
  uint64_t *stage;  // LDS: a step's qualifying candidates; counters during a merge
  uint32_t *vis;   // LDS [cap]
  uint64_t *cand;  // LDS: unvisited neighbours of this step
  const int *tql;  // LDS: the folded query, TQW words per 16-byte code chunk
  int lane, sub, grp;
  uint32_t coff[CPL];  // byte offsets of this lane's chunks inside a code row
  uint32_t vis_mask, vis_shift, vis_limit;
  float s, qlo;
  int bias, bias_lo;
  uint32_t pk[M], pv[M];  // pool: ordered key bits; (id << 1) | expanded
  uint64_t worst;         // pool entry ef_q-1 (all ones while the pool is not full)
  int ef_q;               // this query's pool size
  uint32_t n_exp = 0, n_dist = 0, n_vis = 0, n_rebuild = 0;

  __device__ __forceinline__ SearchWave(const SearchArgs &args, uint64_t *smem) : a(args) {
    lane = lane_id();
    sub = lane % LPR;
    grp = lane / LPR;
#pragma unroll
    for (int j = 0; j < CPL; ++j) {
      // chunks past the end of the row are read from the last chunk instead;
      // their share of the folded query is zero
      const uint32_t c = (uint32_t)(sub + j * LPR);
      coff[j] = (c < a.n_chunks ? c : a.n_chunks - 1) * 16u;
    }
    const uint32_t cap = 1u << a.vis_log2;
    mbuf = smem;
    stage = mbuf + merge_buf_entries(M);
    vis = reinterpret_cast<uint32_t *>(stage + stage_area_entries(M, PMAX, FAST));
    cand = FAST ? stage : reinterpret_cast<uint64_t *>(vis + cap);
    tql = reinterpret_cast<const int *>(vis + cap + (FAST ? 0 : 2 * cand_entries(a.degree, PMAX)));
    vis_mask = cap - 1;
    vis_shift = 32 - a.vis_log2;
    vis_limit = use_cache() ? 0xFFFFFFFFu : cap - cap / 4;  // the cache is never rebuilt
  }

  // This lane's part of the code/query dot product of one row: its four
  // chunks against the matching words of the folded query.
  __device__ __forceinline__ int row_dot(const uint4 (&row)[CPL], const int *plane) const {
    int dot = 0;
#pragma unroll
    for (int j = 0; j < CPL; ++j) {
      int t[TQW];
      const int4 *tp = reinterpret_cast<const int4 *>(plane + (sub + j * LPR) * TQW);
#pragma unroll
      for (int w = 0; w < TQW / 4; ++w) {
        const int4 v = tp[w];
        t[4 * w] = v.x;
        t[4 * w + 1] = v.y;
        t[4 * w + 2] = v.z;
        t[4 * w + 3] = v.w;
      }
      dot += chunk_dot<BITS>(row[j], t);
    }
    return dot;
  }

  __device__ __forceinline__ int row_dot(const uint4 (&row)[CPL]) const { return row_dot(row, tql); }

  // tau_l of one code row (shared by the LPR lanes that hold its chunks).
  __device__ __forceinline__ float row_key(const uint4 (&row)[CPL], float nrm) const {
    const int dot = group_sum_i32<LPR>(row_dot(row, tql)) + bias;
    if (FAST || !a.q15) return key_from_idot(a.metric, s, qlo, dot, nrm);
    const int dot_lo = group_sum_i32<LPR>(row_dot(row, tql + a.tq_plane / 4)) + bias_lo;
    return key_from_idot15(a.metric, s, qlo, dot, dot_lo, nrm);
  }

  __device__ __forceinline__ void clear_table() {
    for (uint32_t i = lane; i <= vis_mask; i += kWave) vis[i] = kEmpty;
  }

  // Two-way cache of node ids with full-width entries: a set is two adjacent
  // slots, way 0 the more recently tested.  The id goes into way 0; what it
  // displaces moves to way 1, and what that displaces is forgotten.  The
  // exchanges make lanes that test the same id in one instruction see each
  // other (in almost every interleaving; the merge copes with the rest).  A
  // forgotten id may come back as a candidate and is then recognised when it
  // is merged (it equals a pool entry or another candidate) or rejected again
  // by the pool's last entry.
  __device__ __forceinline__ bool wide_cache_test_and_set(uint32_t id) {
    uint32_t *set = &vis[((id * 0x9E3779B1u) >> vis_shift) & ~1u];
    const uint32_t o0 = atomicExch(set, id);
    if (o0 == id) return false;
    if (o0 == kEmpty) return true;  // way 1 is filled only from way 0
    return atomicExch(set + 1, o0) != id;
  }

  // The same cache with twice the entries in the same memory: a set is one
  // word, way 0 its low half and way 1 its high half, and an entry is the
  // 16-bit tag (id >> log2 sets) + 1.  The set index is the id's low bits
  // mixed with a hash of the tag, so (set, tag) still names exactly one id:
  // a hit is never a different node.  0xFFFF marks an empty way.
  __device__ __forceinline__ uint32_t *packed_set(uint32_t id, uint32_t &tag) const {
    const uint32_t hi = id >> a.vis_log2;
    tag = hi + 1u;
    return &vis[(id ^ ((hi * 0x9E3779B1u) >> vis_shift)) & vis_mask];
  }
  static __device__ __forceinline__ bool packed_hit(uint32_t word, uint32_t tag) {
    return (word & 0xFFFFu) == tag || (word >> 16) == tag;
  }
  __device__ __forceinline__ bool packed_cache_test_and_set(uint32_t id) {
    uint32_t tag;
    uint32_t *set = packed_set(id, tag);
    uint32_t seen = *set;
    for (;;) {
      if (packed_hit(seen, tag)) return false;
      // the new tag becomes way 0, way 0 moves to way 1, way 1 is forgotten;
      // a lane that lost the word to another lane looks at what that one wrote
      const uint32_t was = atomicCAS(set, seen, (seen << 16) | tag);
      if (was == seen) return true;
      seen = was;
    }
  }

  __device__ __forceinline__ bool cache_test_and_set(uint32_t id) {
    return use_packed() ? packed_cache_test_and_set(id) : wide_cache_test_and_set(id);
  }

  // true if id was not in the table (and now is)
  __device__ __forceinline__ bool test_and_set(uint32_t id) {
    if (use_cache()) return cache_test_and_set(id);
    // double hashing: the probe stride is odd, so every slot is reached
    const uint32_t h = id * 0x9E3779B1u;
    uint32_t slot = h >> vis_shift;
    const uint32_t stride = ((h >> 4) | 1u) & vis_mask;
    for (;;) {
      uint32_t old = atomicCAS(&vis[slot], kEmpty, id);
      if (old == kEmpty) return true;
      if (old == id) return false;
      slot = (slot + stride) & vis_mask;
    }
  }

  // Membership test without insertion.
  __device__ __forceinline__ bool lookup(uint32_t id) {
    if (use_cache()) {
      if (use_packed()) {
        uint32_t tag;
        const uint32_t *set = packed_set(id, tag);
        return packed_hit(*set, tag);
      }
      const uint32_t *set = &vis[((id * 0x9E3779B1u) >> vis_shift) & ~1u];
      return set[0] == id || set[1] == id;
    }
    const uint32_t h = id * 0x9E3779B1u;
    uint32_t slot = h >> vis_shift;
    const uint32_t stride = ((h >> 4) | 1u) & vis_mask;
    for (;;) {
      const uint32_t cur = vis[slot];
      if (cur == id) return true;
      if (cur == kEmpty) return false;
      slot = (slot + stride) & vis_mask;
    }
  }

  // Two ids per lane at once: the two probe sequences advance together, so
  // the latency of the LDS atomics overlaps.  Bit 0 / bit 1 of the result: id0
  // / id1 was not in the table (and now is).  A lane's two ids may be equal.
  __device__ __forceinline__ int test_and_set2(bool v0, uint32_t id0, bool v1, uint32_t id1) {
    if (use_cache() && use_packed()) {
      uint32_t t0, t1;
      uint32_t *set0 = packed_set(id0, t0), *set1 = packed_set(id1, t1);
      uint32_t seen0 = v0 ? *set0 : 0u, seen1 = v1 ? *set1 : 0u;
      int fresh = 0;
      while (v0 || v1) {
        v0 = v0 && !packed_hit(seen0, t0);
        v1 = v1 && !packed_hit(seen1, t1);
        uint32_t was0 = seen0, was1 = seen1;
        if (v0) was0 = atomicCAS(set0, seen0, (seen0 << 16) | t0);
        if (v1) was1 = atomicCAS(set1, seen1, (seen1 << 16) | t1);
        if (v0 && was0 == seen0) {
          fresh |= 1;
          v0 = false;
        }
        if (v1 && was1 == seen1) {
          fresh |= 2;
          v1 = false;
        }
        seen0 = was0;
        seen1 = was1;
      }
      return fresh;
    }
    if (use_cache()) {
      uint32_t *set0 = &vis[((id0 * 0x9E3779B1u) >> vis_shift) & ~1u];
      uint32_t *set1 = &vis[((id1 * 0x9E3779B1u) >> vis_shift) & ~1u];
      uint32_t o0 = id0, o1 = id1;
      if (v0) o0 = atomicExch(set0, id0);
      if (v1) o1 = atomicExch(set1, id1);
      bool f0 = o0 != id0, f1 = o1 != id1;
      if (f0 && o0 != kEmpty) f0 = atomicExch(set0 + 1, o0) != id0;
      if (f1 && o1 != kEmpty) f1 = atomicExch(set1 + 1, o1) != id1;
      return (f0 ? 1 : 0) | (f1 ? 2 : 0);
    }
    const uint32_t h0 = id0 * 0x9E3779B1u, h1 = id1 * 0x9E3779B1u;
    uint32_t s0 = h0 >> vis_shift, s1 = h1 >> vis_shift;
    const uint32_t st0 = ((h0 >> 4) | 1u) & vis_mask, st1 = ((h1 >> 4) | 1u) & vis_mask;
    int fresh = 0;
    while (v0 || v1) {
      uint32_t o0 = 0, o1 = 0;
      if (v0) o0 = atomicCAS(&vis[s0], kEmpty, id0);
      if (v1) o1 = atomicCAS(&vis[s1], kEmpty, id1);
      if (v0) {
        if (o0 == kEmpty) {
          fresh |= 1;
          v0 = false;
        } else if (o0 == id0) {
          v0 = false;
        } else {
          s0 = (s0 + st0) & vis_mask;
        }
      }
      if (v1) {
        if (o1 == kEmpty) {
          fresh |= 2;
          v1 = false;
        } else if (o1 == id1) {
          v1 = false;
        } else {
          s1 = (s1 + st1) & vis_mask;
        }
      }
    }
    return fresh;
  }

  // The table holds every node whose key has been evaluated, as long as it
  // fits.  When it is about to pass 3/4 load it is rebuilt from the pool.  A
  // forgotten node is outside the pool, so it was rejected or evicted by a
  // pool maximum that has only decreased since: re-evaluating it yields the
  // same key and the same rejection.  Results do not change; work is repeated.
  __device__ __forceinline__ void rebuild_table() {
    wave_sync();
    clear_table();
    wave_sync();
    int kept = 0;
#pragma unroll
    for (int r = 0; r < M; ++r)
      if (pk[r] != kEmpty) {
        test_and_set(pv[r] >> 1);
        ++kept;
      }
    n_vis = (uint32_t)group_sum_i32<64>(kept);
    ++n_rebuild;
    wave_sync();
  }

  __device__ __forceinline__ void refresh_worst() {
    const int g = ef_q - 1, rr = g / kWave, rl = g % kWave;
    uint32_t k_ = pk[0], v_ = pv[0];
#pragma unroll
    for (int r = 1; r < M; ++r) {
      k_ = (rr == r) ? pk[r] : k_;
      v_ = (rr == r) ? pv[r] : v_;
    }
    worst = pack64(__builtin_amdgcn_readlane(k_, rl), __builtin_amdgcn_readlane(v_, rl));
  }

  // Merge up to 64 candidates (one per lane where `have`) into the pool.
  //
  // mbuf[0 .. 64 M) is the pool in order as the last merge left it (expanded
  // marks may be out of date, which no comparison below depends on); slots
  // behind the pool hold all-ones or entries that were pushed out, all of them
  // above any candidate that beats the pool's last entry.
  __device__ __forceinline__ void merge(bool have, uint32_t ck, uint32_t cv) {
    const uint64_t c64 = pack64(ck, cv);
    bool mine = have && c64 < worst;
    if (__ballot(mine) == 0) return;
    // number of pool entries below the candidate: lower bound over slots
    // 0 .. 64 M - 2 (a candidate that beats the last entry ranks below 64 M).
    // Two levels of the bisection per round: the probe of the first level and
    // both possible probes of the second are read together, so a round costs
    // one LDS latency instead of two.
    uint32_t pos = 0;  // byte offset into mbuf
    {
      const char *mb = reinterpret_cast<const char *>(mbuf);
      int step = 32 * M;
#pragma unroll
      for (; step >= 2; step >>= 2) {
        const uint64_t ea = *reinterpret_cast<const uint64_t *>(mb + pos + (step - 1) * 8);
        const uint64_t eb = *reinterpret_cast<const uint64_t *>(mb + pos + (step / 2 - 1) * 8);
        const uint64_t ec = *reinterpret_cast<const uint64_t *>(mb + pos + (step + step / 2 - 1) * 8);
        const bool up = ea < c64;
        const uint64_t second = up ? ec : eb;
        pos += (up ? (uint32_t)step * 8u : 0u) + (second < c64 ? (uint32_t)(step / 2) * 8u : 0u);
      }
      if (step == 1) {
        const uint64_t e = *reinterpret_cast<const uint64_t *>(mb + pos);
        pos += e < c64 ? 8u : 0u;
      }
    }
    // A node the visited set has forgotten can come back.  If it is in the
    // pool, the entry found is that node (ids are unique in the pool): dropped.
    const uint32_t at_id = (uint32_t)*reinterpret_cast<const uint64_t *>(reinterpret_cast<const char *>(mbuf) + pos);
    mine = mine && (at_id | 1u) != (cv | 1u);
    uint64_t km = __ballot(mine);
    if (km == 0) return;
    const int rank_p = (int)(pos >> 3);
    int *cnt = reinterpret_cast<int *>(stage);
    uint64_t *lst = M >= 2 ? mbuf : stage + merge_list_at(M);
    int shift[M];
    int dest;
    for (;;) {
      // pool entry i moves up by the number of candidates with rank <= i
#pragma unroll
      for (int r = 0; r < M; ++r) cnt[r * kWave + lane] = 0;
      // the batch's candidates side by side, padded to a multiple of four with
      // values above every candidate
      const int n_l = __popcll(km);
      if (mine) lst[lanes_below(km)] = c64;
      if (lane < 4) lst[n_l + lane] = ~0ull;
      wave_sync();
      if (mine) atomicAdd(&cnt[rank_p], 1);
      wave_sync();
      int carry = 0;
#pragma unroll
      for (int r = 0; r < M; ++r) {
        shift[r] = wave_inclusive_scan_i32(cnt[r * kWave + lane]) + carry;
        carry = __builtin_amdgcn_readlane(shift[r], kWave - 1);
      }
      // candidates below this lane's candidate: every lane walks the list
      // (all lanes read the same entry: one LDS access each, four in flight)
      int below_c = 0;
      for (int i = 0; i < n_l; i += 4) {
        const uint64_t e0 = lst[i], e1 = lst[i + 1], e2 = lst[i + 2], e3 = lst[i + 3];
        below_c += (e0 < c64 ? 1 : 0) + (e1 < c64 ? 1 : 0) + (e2 < c64 ? 1 : 0) + (e3 < c64 ? 1 : 0);
      }
      dest = rank_p + below_c;
      // The same forgotten node twice among the candidates: equal values get
      // equal destinations.  One of them stays, the count starts over (rare).
      // (candidates ranked past the buffer are dropped anyway)
      const bool lands = mine && dest < 64 * M;
      wave_sync();
      if (lands) cnt[dest] = lane;
      wave_sync();
      const uint64_t lose = __ballot(lands && cnt[dest] != lane);
      if (lose == 0) break;
      km &= ~lose;
      mine = mine && ((lose >> lane) & 1ull) == 0;
      wave_sync();
    }
    const int n_m = __popcll(km);
    // no two (key, id) pairs are equal: the destinations are a permutation
#pragma unroll
    for (int r = 0; r < M; ++r) {
      const int to = r * kWave + lane + shift[r];
      if (to < 64 * M) mbuf[to] = pack64(pk[r], pv[r]);
    }
    if (mine && dest < 64 * M) mbuf[dest] = c64;
    wave_sync();
#pragma unroll
    for (int r = 0; r < M; ++r) {
      const uint64_t v = mbuf[r * kWave + lane];
      const bool beyond = r * kWave + lane >= ef_q;  // entries pushed past the pool size are dropped
      pk[r] = beyond ? kEmpty : (uint32_t)(v >> 32);
      pv[r] = beyond ? kEmpty : (uint32_t)v;
    }
    wave_sync();
    (void)n_m;
    refresh_worst();
  }

  // Merge of a few candidates (lanes 0 .. n-1 hold them, all below the pool's
  // last entry): one pass per candidate, its value broadcast to all lanes.
  // Every pool entry counts the candidates below it (it moves up by that
  // many), the candidate gets the number of pool entries and of other
  // candidates below it; a candidate that names a node of the pool, or the same
  // node as an earlier candidate (both: forgotten by the visited cache and
  // evaluated again), is left out.  Then the scatter through the sorted copy as
  // in merge().  No search, no counters, no prefix sums: cheaper than merge()
  // while the candidates are few, and the result is the same pool.
  __device__ __forceinline__ void merge_few(int n, uint64_t c64) {
    uint64_t pool64[M];
    int shift[M];
#pragma unroll
    for (int r = 0; r < M; ++r) {
      pool64[r] = pack64(pk[r], pv[r]);
      shift[r] = 0;
    }
    int dest = 0;
    bool in = false;
    int n_in = 0;
#pragma nounroll
    for (int j = 0; j < n; ++j) {
      const uint32_t ck = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(c64 >> 32), j);
      const uint32_t cv = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)c64, j);
      const uint64_t cj = pack64(ck, cv);
      uint64_t same = __ballot(lane < j && c64 == cj);
#pragma unroll
      for (int r = 0; r < M; ++r) same |= __ballot((pv[r] | 1u) == (cv | 1u));
      if (same != 0) continue;
      int below = 0;
#pragma unroll
      for (int r = 0; r < M; ++r) {
        const bool lt = pool64[r] < cj;
        below += __popcll(__ballot(lt));
        shift[r] += lt ? 0 : 1;
      }
      if (lane == j) {
        dest += below;
        in = true;
      }
      if (lane < n && cj < c64) ++dest;
      ++n_in;
    }
    if (n_in == 0) return;
#pragma unroll
    for (int r = 0; r < M; ++r) {
      const int to = r * kWave + lane + shift[r];
      if (to < 64 * M) mbuf[to] = pool64[r];
    }
    if (in && dest < 64 * M) mbuf[dest] = c64;
    wave_sync();
#pragma unroll
    for (int r = 0; r < M; ++r) {
      const uint64_t v = mbuf[r * kWave + lane];
      const bool beyond = r * kWave + lane >= ef_q;  // entries pushed past the pool size are dropped
      pk[r] = beyond ? kEmpty : (uint32_t)(v >> 32);
      pv[r] = beyond ? kEmpty : (uint32_t)v;
    }
    wave_sync();
    refresh_worst();
  }

  // Visited filter and compaction for one list of node ids (one per lane):
  // unvisited ids are marked and appended to cand[n_cand ..].
  __device__ __forceinline__ void filter_ids(uint32_t nb, uint32_t nrm, int &n_cand) {
    const bool valid = nb != kEmpty && nb < a.n;
    const bool fresh = valid && test_and_set(nb);
    const uint64_t fm = __ballot(fresh);
    if (fresh) cand_at(n_cand + lanes_below(fm)) = pack64(nb, nrm);
    n_cand += __popcll(fm);
  }

  // The same with the cap of Algorithm 1's inner condition |N| < m_s: only the
  // first m_s unvisited ids (in lane = stored order) are taken and marked;
  // the others stay unvisited.
  __device__ __forceinline__ void filter_ids_capped(uint32_t nb, uint32_t nrm, uint32_t m_s, int &n_cand) {
    const bool valid = nb != kEmpty && nb < a.n;
    const bool open = valid && !lookup(nb);
    const uint64_t om = __ballot(open);
    const bool take = open && (uint32_t)lanes_below(om) < m_s;
    wave_sync();
    const bool fresh = take && test_and_set(nb);
    const uint64_t fm = __ballot(fresh);
    if (fresh) cand_at(n_cand + lanes_below(fm)) = pack64(nb, nrm);
    n_cand += __popcll(fm);
  }

  // Same for two lists at once (list 0's survivors are appended first).
  __device__ __forceinline__ void filter_ids2(uint32_t nb0, uint32_t nrm0, uint32_t nb1, uint32_t nrm1, int &n_cand) {
    const int f = test_and_set2(nb0 != kEmpty && nb0 < a.n, nb0, nb1 != kEmpty && nb1 < a.n, nb1);
    const uint64_t fm0 = __ballot(f & 1), fm1 = __ballot(f & 2);
    const int c0 = __popcll(fm0);
    if (f & 1) cand_at(n_cand + lanes_below(fm0)) = pack64(nb0, nrm0);
    if (f & 2) cand_at(n_cand + c0 + lanes_below(fm1)) = pack64(nb1, nrm1);
    n_cand += c0 + __popcll(fm1);
  }

  // Merge the n_q staged candidates into the pool, 64 at a time (they are
  // copied to registers first: a merge uses the staging area for its counters).
  static constexpr int kStage = stage_entries(M, PMAX, FAST);
  __device__ __forceinline__ void merge_staged(int &n_q) {
    if (n_q == 0) return;
    wave_sync();
    if (n_q <= ANN_FEW) {
      const uint64_t c = lane < n_q ? stage[lane] : 0;
      wave_sync();
      merge_few(n_q, c);
      n_q = 0;
      return;
    }
    constexpr int kBatches = kStage / kWave;
    uint64_t batch[kBatches];
#pragma unroll
    for (int b = 0; b < kBatches; ++b) batch[b] = b * kWave + lane < n_q ? stage[b * kWave + lane] : 0;
    wave_sync();
    // one copy of the merge code, however many batches: the batch is picked by selects
#pragma nounroll
    for (int b = 0; b * kWave < n_q; ++b) {
      uint64_t c = batch[0];
#pragma unroll
      for (int t = 1; t < kBatches; ++t) c = b == t ? batch[t] : c;
      merge(b * kWave + lane < n_q, (uint32_t)(c >> 32), (uint32_t)c);
    }
    n_q = 0;
  }

  // tau_l for the n_cand nodes in cand[], then merge the ones that can enter
  // the pool.
  __device__ __forceinline__ void evaluate_and_merge(int n_cand) {
    if (n_cand == 0) return;
    n_vis += n_cand;
    n_dist += n_cand;
    wave_sync();
    int n_q = 0;
    for (int base = 0; base < n_cand; base += G * U) {
      uint4 rows[U][CPL];
      float nrm[U];
      uint32_t vid[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (base + u * G < n_cand) {
          // lanes past the end of the list recompute its last node; the
          // duplicate is ignored below, and no branch is needed around loads
          const int ci = base + u * G + grp;
          const uint64_t ce = cand_at(ci < n_cand ? ci : n_cand - 1);
          vid[u] = (uint32_t)(ce >> 32);
          const uint8_t *rp = a.codes + (uint64_t)vid[u] * a.row_stride;
#pragma unroll
          for (int j = 0; j < CPL; ++j) rows[u][j] = *reinterpret_cast<const uint4 *>(rp + coff[j]);
          nrm[u] = a.adj_norms ? __uint_as_float((uint32_t)ce) : (a.norm_term ? a.norm_term[vid[u]] : 0.0f);
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (base + u * G < n_cand) {
          const float key = row_key(rows[u], nrm[u]);
          const uint64_t c64 = pack64(order_u32(key), vid[u] << 1);
          const bool q = sub == 0 && base + u * G + grp < n_cand && c64 < worst;
          const uint64_t bm = __ballot(q);
          if (!FAST && n_q + G > kStage) merge_staged(n_q);  // rare: make room (FAST: the area holds a whole step)
          if (q) stage[n_q + lanes_below(bm)] = c64;
          n_q += __popcll(bm);
        }
      }
    }
    merge_staged(n_q);
  }

  // Expansion with redundantly stored neighbour vectors (the paper's PRS
  // layout, Section 3.3): the code rows and norm terms of u's first prs_slots
  // neighbours (redundancy ratio = prs_slots / degree) lie next to each other
  // in slot order, so they are requested together with the id row - one memory
  // round trip instead of two, sequential instead of scattered reads, and no
  // compaction.  Rows of visited neighbours among them are fetched as well;
  // only unvisited ones are counted and can enter the pool.  The unvisited
  // neighbours in the remaining slots go to the list cand[n_cand ..] and are
  // gathered from the code table the usual way by the caller.
  __device__ __forceinline__ void expand_prs(uint32_t uid, int &n_q, int &n_cand) {
    const int S = (int)a.prs_slots;
    uint32_t nb = kEmpty, nb_nrm = 0;
    if (lane < (int)a.degree) load_slot(uid, lane, nb, nb_nrm);
    const uint64_t rowbase = (uint64_t)uid * (uint32_t)S;
    uint64_t fm = 0;
    for (int sg = 0; sg < S; sg += G) {
      const int slot = sg + grp;
      const uint64_t at = rowbase + (uint32_t)(slot < S ? slot : S - 1);
      const uint8_t *rp = a.prs_codes + at * a.row_stride;
      uint4 rows[CPL];
#pragma unroll
      for (int j = 0; j < CPL; ++j) rows[j] = *reinterpret_cast<const uint4 *>(rp + coff[j]);
      const float nrm = a.prs_norm ? a.prs_norm[at] : 0.0f;
      if (sg == 0) {
        // all ids of the row against the visited set, while the rows are on their way
        if (PMAX == 1) {
          const uint32_t incoming = (uint32_t)__popcll(__ballot(nb != kEmpty));
          if (n_vis + incoming > vis_limit) rebuild_table();
        }
        const bool fresh = nb != kEmpty && nb < a.n && test_and_set(nb);
        fm = __ballot(fresh);
        const uint64_t stored = S >= 64 ? ~0ull : ((1ull << S) - 1ull);
        const int n_new = __popcll(fm & stored);
        n_vis += n_new;
        n_dist += n_new;
        // the rest of the row: unvisited neighbours whose rows are not stored with u
        const uint64_t rest = fm & ~stored;
        if ((rest >> lane) & 1ull) cand_at(n_cand + lanes_below(rest)) = pack64(nb, nb_nrm);
        n_cand += __popcll(rest);
      }
      const uint32_t vid = (uint32_t)__shfl((int)nb, slot & 63);
      const float key = row_key(rows, nrm);
      const uint64_t c64 = pack64(order_u32(key), vid << 1);
      const bool q = sub == 0 && slot < S && ((fm >> (slot & 63)) & 1ull) && c64 < worst;
      const uint64_t bm = __ballot(q);
      if (n_q + G > kStage) merge_staged(n_q);
      if (q) stage[n_q + lanes_below(bm)] = c64;
      n_q += __popcll(bm);
    }
  }

  __device__ __forceinline__ void run(uint32_t qi) {
    // the folded query goes to LDS: it is read again for every group of rows
    // (keeping it in registers costs a wavefront of occupancy)
    {
      const int *src = reinterpret_cast<const int *>(a.tq + (uint64_t)qi * a.tq_stride);
      int *dst = const_cast<int *>(tql);
      for (uint32_t i = lane; i < a.tq_stride / 4; i += kWave) dst[i] = src[i];
    }
    ef_q = (int)a.ef;
    if (a.ef_per_query) {
      const uint32_t e = a.ef_per_query[qi];
      ef_q = e == 0 ? 1 : (e < a.ef ? (int)e : (int)a.ef);
    }
    s = a.s[qi];
    qlo = a.qlo[qi];
    bias = BITS == 8 ? 128 * a.sum_t[qi] : 0;
    bias_lo = BITS == 8 && a.sum_t_lo ? 128 * a.sum_t_lo[qi] : 0;
#pragma unroll
    for (int r = 0; r < M; ++r) {
      pk[r] = kEmpty;
      pv[r] = kEmpty;
    }
    worst = ~0ull;
#pragma unroll
    for (int r = 0; r < M; ++r) mbuf[r * kWave + lane] = ~0ull;  // the empty pool, in order
    clear_table();
    wave_sync();

    // initial nodes I: into the pool and into V
    {
      uint32_t nb = kEmpty;
      if (a.entry_ids) {
        if (lane < (int)a.n_entry) nb = a.entry_ids[(uint64_t)qi * a.n_entry + lane];
      } else if (lane == 0) {
        nb = a.entry_point;
      }
      uint32_t nrm = 0;
      if (a.adj_norms && nb != kEmpty && nb < a.n) nrm = __float_as_uint(a.norm_term[nb]);
      int n_cand = 0;
      filter_ids(nb, nrm, n_cand);
      evaluate_and_merge(n_cand);
    }

    const int p = PMAX == 1 || FAST ? PMAX : (int)a.p;
    uint32_t pre_id = kEmpty, pre_row = kEmpty, pre_nrm = 0;  // adjacency row fetched ahead (PMAX == 1)
    for (;;) {
      // the p closest un-expanded pool entries, in pool order: their ids as
      // wave-uniform values, their expanded marks set in one pass per register
      uint32_t uid[PMAX];
      uint32_t next_id = kEmpty;
      int got = 0;
      if constexpr (PMAX > 1) {
        // every lane ranks its own entries among the un-expanded ones (pool
        // order: register by register); the first p mark themselves and leave
        // their ids in LDS, where all lanes read them back
        uint32_t *picked = reinterpret_cast<uint32_t *>(stage);
        int before = 0;
#pragma unroll
        for (int r = 0; r < M; ++r) {
          const bool open = (pv[r] & 1u) == 0;
          const uint64_t um = __ballot(open);
          const int rank = before + lanes_below(um);
          if (open && rank < p) {
            picked[rank] = pv[r] >> 1;
            pv[r] |= 1u;
          }
          before += __popcll(um);
        }
        got = before < p ? before : p;
        wave_sync();
#pragma unroll
        for (int e = 0; e < PMAX; ++e) uid[e] = e < got ? picked[e] : kEmpty;
        wave_sync();
      } else {
        uint64_t um[M], mark[M];
#pragma unroll
        for (int r = 0; r < M; ++r) {
          um[r] = __ballot((pv[r] & 1u) == 0);
          mark[r] = 0;
        }
#pragma unroll
        for (int e = 0; e < PMAX; ++e) {
          uid[e] = kEmpty;
          bool found = false;
#pragma unroll
          for (int r = 0; r < M; ++r) {
            if (!found && e < p && um[r] != 0) {
              const int L = __builtin_ctzll(um[r]);
              um[r] &= um[r] - 1;
              mark[r] |= 1ull << L;
              uid[e] = (uint32_t)__builtin_amdgcn_readlane(pv[r], L) >> 1;
              found = true;
            }
          }
          got += found ? 1 : 0;
        }
#pragma unroll
        for (int r = M - 1; r >= 0; --r)
          if (um[r] != 0) next_id = (uint32_t)__builtin_amdgcn_readlane(pv[r], __builtin_ctzll(um[r])) >> 1;
#pragma unroll
        for (int r = 0; r < M; ++r) pv[r] |= (uint32_t)((mark[r] >> lane) & 1ull);
      }
      if (got == 0) break;
      n_exp += got;
      if (PMAX > 1 && !use_cache() && n_vis + (uint32_t)(got * kWave) > vis_limit) rebuild_table();

      if (use_prs()) {
        int n_q = 0, n_rest = 0;
#pragma unroll
        for (int e = 0; e < PMAX; ++e)
          if (e < got) expand_prs(uid[e], n_q, n_rest);
        merge_staged(n_q);
        evaluate_and_merge(n_rest);  // neighbours beyond the stored slots (none at ratio 1)
        continue;
      }
      int n_cand = 0;
      if (use_filter()) {
        // label test and per-expansion cap: rows one after the other, in
        // the order of the picked entries
#pragma unroll
        for (int e = 0; e < PMAX; ++e) {
          if (e >= got) break;
          uint32_t nb = kEmpty, nrm = 0;
          if (lane < (int)a.degree) {
            load_slot(uid[e], lane, nb, nrm);
            if (a.labels && !(a.labels[(uint64_t)uid[e] * a.degree + lane] <= a.alpha_s)) nb = kEmpty;
          }
          if (PMAX == 1) {
            const uint32_t incoming = (uint32_t)__popcll(__ballot(nb != kEmpty));
            if (n_vis + incoming > vis_limit) rebuild_table();
          }
          filter_ids_capped(nb, nrm, a.m_s, n_cand);
        }
      } else if (use_pairs()) {
        // two adjacency rows per pass: lanes 0-31 take one, lanes 32-63 the next
        const int slot = lane & 31;
        uint32_t rows[PMAX / 2 > 0 ? PMAX / 2 : 1], nrms[PMAX / 2 > 0 ? PMAX / 2 : 1];
#pragma unroll
        for (int t = 0; t < PMAX / 2; ++t) {
          rows[t] = kEmpty;
          nrms[t] = 0;
          if (2 * t < got) {
            const uint32_t u = lane < 32 ? uid[2 * t] : uid[2 * t + 1 < PMAX ? 2 * t + 1 : 2 * t];
            if (u != kEmpty && slot < (int)a.degree) load_slot(u, slot, rows[t], nrms[t]);
          }
        }
#pragma unroll
        for (int t = 0; t < PMAX / 2; t += 2) {
          constexpr int kLast = PMAX / 2 > 0 ? PMAX / 2 - 1 : 0;
          const int t1 = t + 1 < PMAX / 2 ? t + 1 : kLast;
          if (t + 1 < PMAX / 2 && 2 * (t + 1) < got)
            filter_ids2(rows[t], nrms[t], rows[t1], nrms[t1], n_cand);
          else if (2 * t < got)
            filter_ids(rows[t], nrms[t], n_cand);
        }
      } else {
        uint32_t rows[PMAX], nrms[PMAX];
#pragma unroll
        for (int e = 0; e < PMAX; ++e) {
          rows[e] = kEmpty;
          nrms[e] = 0;
          if (e < got) {
            if (PMAX == 1 && uid[e] == pre_id) {
              rows[e] = pre_row;
              nrms[e] = pre_nrm;
            } else if (lane < (int)a.degree) {
              load_slot(uid[e], lane, rows[e], nrms[e]);
            }
          }
        }
        if (PMAX == 1) {
          // fetch ahead the row of the entry that is expanded next unless a
          // candidate of this step overtakes it
          pre_id = next_id;
          pre_row = kEmpty;
          pre_nrm = 0;
          if (next_id != kEmpty && lane < (int)a.degree) load_slot(next_id, lane, pre_row, pre_nrm);
        }
#pragma unroll
        for (int e = 0; e < PMAX; ++e) {
          if (e < got) {
            if (PMAX == 1) {
              const uint32_t incoming = (uint32_t)__popcll(__ballot(rows[e] != kEmpty));
              if (n_vis + incoming > vis_limit) rebuild_table();
            }
            filter_ids(rows[e], nrms[e], n_cand);
          }
        }
      }
      evaluate_and_merge(n_cand);
    }

    // results (pool index r*64 + lane: coalesced)
    int kept = 0;
#pragma unroll
    for (int r = 0; r < M; ++r) {
      const uint32_t i = r * kWave + lane;
      const bool live = pk[r] != kEmpty;
      kept += __popcll(__ballot(live));
      if (i < a.ef) {
        a.out_ids[(uint64_t)qi * a.ef + i] = live ? (pv[r] >> 1) : kEmpty;
        if (a.out_keys) a.out_keys[(uint64_t)qi * a.ef + i] = live ? unorder_f32(pk[r]) : INFINITY;
      }
    }
    if (a.out_idot) {
      // same arithmetic as during traversal, over the final pool
      wave_sync();
      uint32_t *st_id = reinterpret_cast<uint32_t *>(mbuf);
#pragma unroll
      for (int r = 0; r < M; ++r) st_id[r * kWave + lane] = pk[r] != kEmpty ? (pv[r] >> 1) : kEmpty;
      wave_sync();
      for (int base = 0; base < (int)a.ef; base += G) {
        const int ci = base + grp;
        const uint32_t v = ci < (int)a.ef ? st_id[ci] : kEmpty;
        int dot = 0;
        if (v != kEmpty) {
          const uint8_t *rp = a.codes + (uint64_t)v * a.row_stride;
          uint4 row[CPL];
#pragma unroll
          for (int j = 0; j < CPL; ++j) row[j] = *reinterpret_cast<const uint4 *>(rp + coff[j]);
          dot = row_dot(row);
        }
        dot = group_sum_i32<LPR>(dot) + bias;
        if (sub == 0 && ci < (int)a.ef) a.out_idot[(uint64_t)qi * a.ef + ci] = v != kEmpty ? dot : 0;
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

template <int BITS, int LPR, int M, int PMAX, bool FAST>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(M <= 2 ? (FAST ? (PMAX > 4 ? ANN_WPE_WIDE : (PMAX > 1 ? (BITS == 8 ? ANN_WPE : 5) : ANN_WPE_EXACT)) : 5) : (M == 4 ? 4 : 3)))) void search_kernel(SearchArgs args) {
  extern __shared__ uint64_t smem[];
  if (blockIdx.x >= args.nq) return;
  const uint32_t qi = args.order ? args.order[blockIdx.x] : blockIdx.x;
  if (qi >= args.nq) return;  // not a permutation: skip rather than write out of bounds
  SearchWave<BITS, LPR, M, PMAX, FAST> w(args, smem);
  w.run(qi);
}

template <int BITS, int LPR, int PMAX, bool FAST>
static ann_status launch_m(const SearchArgs &args, int m, hipStream_t st) {
  const size_t smem = search_smem_bytes(m, PMAX, FAST, args.vis_log2, args.degree, args.tq_stride);
  switch (m) {
    case 1: search_kernel<BITS, LPR, 1, PMAX, FAST><<<args.nq, 64, smem, st>>>(args); break;
    case 2: search_kernel<BITS, LPR, 2, PMAX, FAST><<<args.nq, 64, smem, st>>>(args); break;
    case 4: search_kernel<BITS, LPR, 4, PMAX, FAST><<<args.nq, 64, smem, st>>>(args); break;
    case 8: search_kernel<BITS, LPR, 8, PMAX, FAST><<<args.nq, 64, smem, st>>>(args); break;
    default: return fail(ANN_EUNSUPPORTED, "no kernel for pool registers per lane = %d", m);
  }
  ANN_HIP(hipGetLastError());
  return ANN_OK;
}

template <int BITS, int PMAX, bool FAST>
static ann_status launch_lpr(const SearchArgs &args, uint32_t lpr, int m, hipStream_t st) {
  switch (lpr) {
    case 1: return launch_m<BITS, 1, PMAX, FAST>(args, m, st);
    case 2: return launch_m<BITS, 2, PMAX, FAST>(args, m, st);
    case 4: return launch_m<BITS, 4, PMAX, FAST>(args, m, st);
    case 8: return launch_m<BITS, 8, PMAX, FAST>(args, m, st);
    case 16: return launch_m<BITS, 16, PMAX, FAST>(args, m, st);
    default: return fail(ANN_EUNSUPPORTED, "no kernel for %u lanes per code row", lpr);
  }
}

// Expansions per step: any count up to kMaxExpansionsPerStep; the kernels are
// built for 1, 4 and 8 picked entries (a count in between runs in the next
// larger general kernel).  The library default stays at 4: eight shorten a
// query's chain of dependent steps (fewer, wider steps: better when the batch
// is too small to fill the chip) but evaluate more nodes (worse when it does).
constexpr int kMaxExpansionsPerStep = 8;
constexpr int kDefaultExpansionsPerStep = 4;

// One translation unit per (FAST, PMAX > 4) instantiates its kernels through this.
template <bool FAST, bool WIDE_STEP>
static ann_status launch_search(const SearchArgs &a, uint32_t bits, uint32_t lpr, int m, bool multi, hipStream_t st) {
  if constexpr (WIDE_STEP) {
    return bits == 8 ? launch_lpr<8, kMaxExpansionsPerStep, FAST>(a, lpr, m, st)
                     : launch_lpr<4, kMaxExpansionsPerStep, FAST>(a, lpr, m, st);
  } else {
    if (!multi) return bits == 8 ? launch_lpr<8, 1, FAST>(a, lpr, m, st) : launch_lpr<4, 1, FAST>(a, lpr, m, st);
    return bits == 8 ? launch_lpr<8, kDefaultExpansionsPerStep, FAST>(a, lpr, m, st)
                     : launch_lpr<4, kDefaultExpansionsPerStep, FAST>(a, lpr, m, st);
  }
}

ann_status launch_search_fast(const SearchArgs &a, uint32_t bits, uint32_t lpr, int m, bool multi, hipStream_t st);
ann_status launch_search_general(const SearchArgs &a, uint32_t bits, uint32_t lpr, int m, bool multi, hipStream_t st);
ann_status launch_search_fast_wide(const SearchArgs &a, uint32_t bits, uint32_t lpr, int m, hipStream_t st);
ann_status launch_search_general_wide(const SearchArgs &a, uint32_t bits, uint32_t lpr, int m, hipStream_t st);

}  // namespace ann
