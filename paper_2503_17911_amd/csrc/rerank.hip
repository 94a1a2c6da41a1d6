// Candidate re-evaluation: the exact fp32 rerank that ends Algorithm 1 (its
// last step orders the pool by the high-precision distance; here that is done
// over a fixed-length prefix of the pool) and the rescore with a finer code
// level.  One query per
// wavefront; candidates are ordered by ranking every (value, id) pair against
// all others in LDS.
#include "ann_internal.hpp"
#include "device_utils.hpp"

namespace ann {

constexpr uint32_t kNone = 0xFFFFFFFFu;

__device__ __forceinline__ uint64_t pack_vi(uint32_t hi, uint32_t lo) { return ((uint64_t)hi << 32) | lo; }

// Rank of every element of list[0..n) under (value, position) order, written
// to out positions; elements equal to the all-ones sentinel sort last.
// `emit(rank, index)` is called for every element by the lane that owns it.
template <int T, typename Emit>
__device__ __forceinline__ void rank_blocks(const uint64_t *list, uint32_t n, int lane, Emit emit) {
  // a lane ranks T of its elements per sweep over the list: one (broadcast)
  // LDS read serves T comparisons
  for (uint32_t i0 = 0; i0 < n; i0 += kWave * T) {
    uint64_t e[T];
    uint32_t rank[T], idx[T];
#pragma unroll
    for (int t = 0; t < T; ++t) {
      idx[t] = i0 + t * kWave + lane;
      e[t] = idx[t] < n ? list[idx[t]] : ~0ull;
      rank[t] = 0;
    }
    for (uint32_t j = 0; j < n; ++j) {
      const uint64_t o = list[j];
#pragma unroll
      for (int t = 0; t < T; ++t) rank[t] += (o < e[t] || (o == e[t] && j < idx[t])) ? 1u : 0u;
    }
#pragma unroll
    for (int t = 0; t < T; ++t)
      if (idx[t] < n) emit(rank[t], idx[t], e[t]);
  }
}

template <typename Emit>
__device__ __forceinline__ void rank_all(const uint64_t *list, uint32_t n, int lane, Emit emit) {
  if (n <= (uint32_t)kWave)
    rank_blocks<1>(list, n, lane, emit);
  else
    rank_blocks<4>(list, n, lane, emit);
}

// ------------------------------------------------------------------ rerank
// tau_h on the original vectors.  L2: sum (q - x)^2; IP: -(q . x).  Products
// and sums in fp64 (each lane sums a strided share, then a butterfly), one
// rounding to fp32 at the end.
template <int LPR, bool VEC4>
__global__ __launch_bounds__(64) void rerank_kernel(const float *__restrict__ X, uint32_t d, uint32_t metric,
                                                    const float *__restrict__ Q, uint32_t nq, uint64_t n,
                                                    const uint32_t *__restrict__ cand_ids, uint32_t n_max,
                                                    uint32_t cand_stride, uint32_t k, uint32_t *__restrict__ out_ids,
                                                    float *__restrict__ out_dist,
                                                    const float *__restrict__ cand_keys, uint32_t n_min, float gamma,
                                                    uint32_t *__restrict__ out_n) {
  extern __shared__ uint64_t smem64[];
  float *qs = reinterpret_cast<float *>(smem64);             // [d], 16-byte aligned
  uint64_t *list = smem64 + ((d + 3) / 4) * 2;               // [n_max]
  // [n_max] the candidates' ids (padding and ids >= n as kNone), in the upper
  // half of the list's memory: result j is written after id j has been read
  // (results come in order, at most one per id), and result j ends at byte
  // 8 j + 8 <= 4 n_max + 4 i, where id i >= j + 1 begins, as long as j < n_max
  uint32_t *ids_s = reinterpret_cast<uint32_t *>(list) + n_max;
  const uint32_t qi = blockIdx.x;
  if (qi >= nq) return;
  const int lane = threadIdx.x, chunk = lane % LPR, grp = lane / LPR;
  constexpr int G = kWave / LPR;
  // Length of the prefix that is re-evaluated.  Fixed (n_max), or chosen per
  // query from the low-precision keys: every candidate whose key is not above
  // key[k-1] + gamma * (key[k-1] - key[0]), at least n_min, at most n_max.
  uint32_t n_cand = n_max;
  if (cand_keys) {
    const float *keys = cand_keys + (uint64_t)qi * cand_stride;
    const float k0 = keys[0], kk = keys[k - 1 < n_max ? k - 1 : n_max - 1];
    if (isfinite(kk)) {
      const float thr = __fmaf_rn(gamma, __fsub_rn(kk, k0), kk);
      uint32_t cnt = 0;
      for (uint32_t i = lane; i < n_max; i += kWave) cnt += keys[i] <= thr ? 1u : 0u;
      n_cand = (uint32_t)group_sum_i32<64>((int)cnt);
      n_cand = n_cand < n_min ? n_min : n_cand;
    }
    if (out_n && lane == 0) out_n[qi] = n_cand;
  }
  for (uint32_t j = lane; j < d; j += kWave) qs[j] = Q[(uint64_t)qi * d + j];
  // the ids go to LDS with the query, so that a round of rows costs one
  // memory round trip instead of two (id, then row)
  const uint32_t *cand = cand_ids + (uint64_t)qi * cand_stride;
  for (uint32_t i = lane; i < n_cand; i += kWave) {
    const uint32_t v = cand[i];
    ids_s[i] = v >= n ? kNone : v;   // (padding is 0xFFFFFFFF >= n)
  }
  __syncthreads();
  uint32_t n_valid = 0;   // candidates that name a node: their entries are kept in order at the front of the list
  // the row sums of one round (G candidates side by side) go to the list; acc is this lane's share of candidate v
  auto append = [&](uint32_t v, double acc) {
    acc = group_sum_f64<LPR>(acc);
    const bool have = chunk == 0 && v != kNone;
    const uint64_t hm = __ballot(have);
    if (have) {
      float dist = (float)(metric == ANN_L2 ? acc : -acc);
      uint32_t b = __float_as_uint(dist);
      if ((b & 0x7FFFFFFFu) == 0) dist = 0.0f;
      const uint32_t below = __builtin_amdgcn_mbcnt_hi((uint32_t)(hm >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)hm, 0u));
      list[n_valid + below] = pack_vi(order_u32(dist), v);
    }
    n_valid += (uint32_t)__popcll(hm);
  };
  bool done = false;
  if constexpr (VEC4) {
    const uint32_t d4 = d / 4;
    if (d4 <= 4 * (uint32_t)LPR) {
      // Short rows (at most four 16-byte pieces per lane): three rounds at a
      // time - their ids first, then all their rows, so that one memory latency
      // covers the three rounds; the sums are formed in the order of the loop below.
      constexpr int kRounds = 3;
      const float4 *x4 = reinterpret_cast<const float4 *>(X);
      for (uint32_t base = 0; base < n_cand; base += kRounds * G) {
        uint32_t vv[kRounds];
        float4 xr[kRounds][4];
#pragma unroll
        for (int r = 0; r < kRounds; ++r) {
          const uint32_t ci = base + r * G + grp;
          vv[r] = ci < n_cand ? ids_s[ci] : kNone;
        }
#pragma unroll
        for (int r = 0; r < kRounds; ++r) {
          const float4 *row = x4 + (uint64_t)(vv[r] != kNone ? vv[r] : 0) * d4;
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            const uint32_t c = (uint32_t)(chunk + LPR * t);
            xr[r][t] = row[c < d4 ? c : 0];
          }
        }
#pragma unroll
        for (int r = 0; r < kRounds; ++r) {
          if (base + r * G >= n_cand) break;
          double acc = 0.0;
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            const uint32_t c = (uint32_t)(chunk + LPR * t);
            if (c < d4 && vv[r] != kNone) {
              const float4 xv = xr[r][t];
              const float4 qv = *reinterpret_cast<const float4 *>(qs + 4 * c);
              if (metric == ANN_L2) {
                const double t0 = (double)qv.x - (double)xv.x, t1 = (double)qv.y - (double)xv.y;
                const double t2 = (double)qv.z - (double)xv.z, t3 = (double)qv.w - (double)xv.w;
                acc += t0 * t0;
                acc += t1 * t1;
                acc += t2 * t2;
                acc += t3 * t3;
              } else {
                acc += (double)qv.x * (double)xv.x;
                acc += (double)qv.y * (double)xv.y;
                acc += (double)qv.z * (double)xv.z;
                acc += (double)qv.w * (double)xv.w;
              }
            }
          }
          append(vv[r], acc);
        }
      }
      done = true;
    }
  }
  for (uint32_t base = 0; !done && base < n_cand; base += G) {
    const uint32_t ci = base + grp;
    const uint32_t v = ci < n_cand ? ids_s[ci] : kNone;
    double acc = 0.0;
    if (v != kNone) {
      const float *x = X + (uint64_t)v * d;
      if constexpr (VEC4) {
        for (uint32_t c = chunk; c < d / 4; c += LPR) {
          const float4 xv = *reinterpret_cast<const float4 *>(x + 4 * c);
          const float4 qv = *reinterpret_cast<const float4 *>(qs + 4 * c);
          if (metric == ANN_L2) {
            const double t0 = (double)qv.x - (double)xv.x, t1 = (double)qv.y - (double)xv.y;
            const double t2 = (double)qv.z - (double)xv.z, t3 = (double)qv.w - (double)xv.w;
            acc += t0 * t0;
            acc += t1 * t1;
            acc += t2 * t2;
            acc += t3 * t3;
          } else {
            acc += (double)qv.x * (double)xv.x;
            acc += (double)qv.y * (double)xv.y;
            acc += (double)qv.z * (double)xv.z;
            acc += (double)qv.w * (double)xv.w;
          }
        }
      } else {
        for (uint32_t j = chunk; j < d; j += LPR) {
          if (metric == ANN_L2) {
            const double t = (double)qs[j] - (double)x[j];
            acc += t * t;
          } else {
            acc += (double)qs[j] * (double)x[j];
          }
        }
      }
    }
    append(v, acc);
  }
  __syncthreads();
  // only the entries that name a node are ranked (padding sorts last anyway)
  rank_all(list, n_valid, lane, [&](uint32_t rank, uint32_t, uint64_t e) {
    if (rank < k) {
      out_ids[(uint64_t)qi * k + rank] = (uint32_t)e;
      out_dist[(uint64_t)qi * k + rank] = unorder_f32((uint32_t)(e >> 32));
    }
  });
  for (uint32_t r = n_valid + lane; r < k; r += kWave) {
    out_ids[(uint64_t)qi * k + r] = kNone;
    out_dist[(uint64_t)qi * k + r] = INFINITY;
  }
}

// ------------------------------------------------------------------ rescore
// Keys of the candidates under another code level, then a full sort.
template <int BITS, int LPR>
__global__ __launch_bounds__(64) void rescore_kernel(const uint8_t *__restrict__ codes, uint32_t row_stride,
                                                     uint32_t n_chunks, const float *__restrict__ norm_term,
                                                     uint32_t metric, uint64_t n, const uint8_t *__restrict__ tq,
                                                     uint32_t tq_stride, uint32_t tq_plane,
                                                     const int32_t *__restrict__ sum_t_lo,
                                                     const float *__restrict__ s_arr,
                                                     const float *__restrict__ qlo_arr,
                                                     const int32_t *__restrict__ sum_t, uint32_t nq,
                                                     const uint32_t *__restrict__ cand_ids, uint32_t n_cand,
                                                     uint32_t cand_stride, uint32_t *__restrict__ out_ids,
                                                     float *__restrict__ out_keys, int32_t *__restrict__ out_idot) {
  extern __shared__ uint64_t smem64[];
  uint64_t *list = smem64;                                     // [n_cand]
  int32_t *dots = reinterpret_cast<int32_t *>(smem64 + n_cand);  // [n_cand]
  const uint32_t qi = blockIdx.x;
  if (qi >= nq) return;
  const int lane = threadIdx.x, chunk = lane % LPR, grp = lane / LPR;
  constexpr int G = kWave / LPR;
  constexpr int TQW = TqRegs<BITS>::kWords;
  // sum_t_lo given: the query has 15 bits, its low bytes are a second plane
  const bool q15 = sum_t_lo != nullptr;
  int tqr[TQW], tqr_lo[TQW];
  const int *tqp = reinterpret_cast<const int *>(tq + (uint64_t)qi * tq_stride + (uint32_t)chunk * (TQW * 4u));
#pragma unroll
  for (int w = 0; w < TQW; ++w) {
    tqr[w] = tqp[w];
    tqr_lo[w] = q15 ? tqp[tq_plane / 4 + w] : 0;
  }
  const float s = s_arr[qi], qlo = qlo_arr[qi];
  const int bias = BITS == 8 ? 128 * sum_t[qi] : 0;
  const int bias_lo = BITS == 8 && q15 ? 128 * sum_t_lo[qi] : 0;
  const uint32_t *cand = cand_ids + (uint64_t)qi * cand_stride;
  // the candidate ids go to LDS first (they share the words of `dots`: entry i
  // is read before dot product i is written), so that the rows of several
  // groups can be requested together instead of one id and one row at a time
  uint32_t *ids_s = reinterpret_cast<uint32_t *>(dots);
  for (uint32_t i = lane; i < n_cand; i += kWave) {
    const uint32_t v = cand[i];
    ids_s[i] = v != kNone && v >= n ? kNone : v;
  }
  __syncthreads();
  constexpr int UNR = 8;  // groups of G rows in flight
  for (uint32_t base = 0; base < n_cand; base += G * UNR) {
    uint32_t vs[UNR];
    uint4 rows[UNR];
    float nrms[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const uint32_t ci = base + u * G + grp;
      vs[u] = ci < n_cand ? ids_s[ci] : kNone;
      rows[u] = make_uint4(0, 0, 0, 0);
      nrms[u] = 0.0f;
      if (vs[u] != kNone) {
        if (chunk < (int)n_chunks)
          rows[u] = *reinterpret_cast<const uint4 *>(codes + (uint64_t)vs[u] * row_stride + (uint32_t)chunk * 16u);
        if (norm_term && chunk == 0) nrms[u] = norm_term[vs[u]];
      }
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const uint32_t ci = base + u * G + grp;
      const uint32_t v = vs[u];
      const int dot = group_sum_i32<LPR>(chunk_dot<BITS>(rows[u], tqr)) + bias;
      int dot_lo = 0;
      if (q15) dot_lo = group_sum_i32<LPR>(chunk_dot<BITS>(rows[u], tqr_lo)) + bias_lo;
      if (chunk == 0 && ci < n_cand) {
        const float key = q15 ? key_from_idot15(metric, s, qlo, dot, dot_lo, nrms[u]) : key_from_idot(metric, s, qlo, dot, nrms[u]);
        list[ci] = v == kNone ? ~0ull : pack_vi(order_u32(key), v);
        dots[ci] = v == kNone || q15 ? 0 : dot;
      }
    }
  }
  __syncthreads();
  rank_all(list, n_cand, lane, [&](uint32_t rank, uint32_t i, uint64_t e) {
    const bool none = e == ~0ull;
    out_ids[(uint64_t)qi * n_cand + rank] = none ? kNone : (uint32_t)e;
    if (out_keys) out_keys[(uint64_t)qi * n_cand + rank] = none ? INFINITY : unorder_f32((uint32_t)(e >> 32));
    if (out_idot) out_idot[(uint64_t)qi * n_cand + rank] = dots[i];
  });
}

template <bool VEC4>
static void launch_rerank(uint32_t lpr, const float *X, uint32_t d, uint32_t metric, const float *Q, uint32_t nq,
                          uint64_t n, const uint32_t *cand, uint32_t n_cand, uint32_t stride, uint32_t k,
                          uint32_t *out_ids, float *out_dist, size_t smem, hipStream_t st, const float *cand_keys,
                          uint32_t n_min, float gamma, uint32_t *out_n) {
#define ANN_RR(L) rerank_kernel<L, VEC4><<<nq, 64, smem, st>>>(X, d, metric, Q, nq, n, cand, n_cand, stride, k, out_ids, out_dist, cand_keys, n_min, gamma, out_n)
  switch (lpr) {
    case 8: ANN_RR(8); break;
    case 16: ANN_RR(16); break;
    case 32: ANN_RR(32); break;
    default: ANN_RR(64); break;
  }
#undef ANN_RR
}

// Shared by ann_rerank and the final stage of ann_bruteforce_topk.
ann_status rerank_device(const float *X, uint64_t n, uint32_t d, uint32_t metric, const float *Q, uint32_t nq,
                         const uint32_t *cand, uint32_t n_cand, uint32_t stride, uint32_t k, uint32_t *out_ids,
                         float *out_dist, hipStream_t st, const float *cand_keys, uint32_t n_min, float gamma,
                         uint32_t *out_n) {
  // four 16-byte pieces of a row per lane: 128 dimensions -> 8 lanes per row, 8 rows side by side
  uint32_t chunks = (d + 3) / 4, lpr = 8;
  while (lpr * 4 < chunks && lpr < 64) lpr <<= 1;
  const size_t smem = (size_t)n_cand * sizeof(uint64_t) + (size_t)((d + 3) / 4) * 16;
  if (d % 4 == 0)
    launch_rerank<true>(lpr, X, d, metric, Q, nq, n, cand, n_cand, stride, k, out_ids, out_dist, smem, st, cand_keys, n_min, gamma, out_n);
  else
    launch_rerank<false>(lpr, X, d, metric, Q, nq, n, cand, n_cand, stride, k, out_ids, out_dist, smem, st, cand_keys, n_min, gamma, out_n);
  ANN_HIP(hipGetLastError());
  return ANN_OK;
}

}  // namespace ann

using namespace ann;

extern "C" {

ann_status ann_rerank(ann_index *index, const float *q, uint32_t nq, const uint32_t *cand_ids, uint32_t n_cand,
                      uint32_t cand_stride, uint32_t k, uint32_t *out_ids, float *out_dist, void *stream) {
  if (!index || !q || !cand_ids || !out_ids || !out_dist) return fail(ANN_EINVAL, "ann_rerank: NULL argument");
  if (!index->vectors) return fail(ANN_EINVAL, "ann_rerank: the index was uploaded without fp32 vectors");
  if (nq == 0 || n_cand == 0 || k == 0) return fail(ANN_EINVAL, "ann_rerank: nq, n_cand and k must be positive");
  if (k > n_cand) return fail(ANN_EINVAL, "ann_rerank: k = %u > n_cand = %u", k, n_cand);
  if (cand_stride < n_cand) return fail(ANN_EINVAL, "ann_rerank: cand_stride = %u < n_cand = %u", cand_stride, n_cand);
  if (n_cand > 4096) return fail(ANN_ECAPACITY, "ann_rerank: n_cand = %u exceeds 4096", n_cand);
  return rerank_device(index->vectors, index->n, index->d, index->metric, q, nq, cand_ids, n_cand, cand_stride, k,
                       out_ids, out_dist, (hipStream_t)stream, nullptr, 0, 0.0f, nullptr);
}

ann_status ann_rerank_adaptive(ann_index *index, const float *q, uint32_t nq, const uint32_t *cand_ids,
                               const float *cand_keys, uint32_t n_min, uint32_t n_max, uint32_t cand_stride,
                               float gamma, uint32_t k, uint32_t *out_ids, float *out_dist, uint32_t *out_n,
                               void *stream) {
  if (!index || !q || !cand_ids || !cand_keys || !out_ids || !out_dist)
    return fail(ANN_EINVAL, "ann_rerank_adaptive: NULL argument");
  if (!index->vectors) return fail(ANN_EINVAL, "ann_rerank_adaptive: the index was uploaded without fp32 vectors");
  if (nq == 0 || n_max == 0 || k == 0) return fail(ANN_EINVAL, "ann_rerank_adaptive: nq, n_max and k must be positive");
  if (k > n_min || n_min > n_max) return fail(ANN_EINVAL, "ann_rerank_adaptive: need k <= n_min <= n_max, got %u, %u, %u", k, n_min, n_max);
  if (cand_stride < n_max) return fail(ANN_EINVAL, "ann_rerank_adaptive: cand_stride = %u < n_max = %u", cand_stride, n_max);
  if (n_max > 4096) return fail(ANN_ECAPACITY, "ann_rerank_adaptive: n_max = %u exceeds 4096", n_max);
  if (!(gamma >= 0.0f)) return fail(ANN_EINVAL, "ann_rerank_adaptive: gamma must be >= 0");
  return rerank_device(index->vectors, index->n, index->d, index->metric, q, nq, cand_ids, n_max, cand_stride, k,
                       out_ids, out_dist, (hipStream_t)stream, cand_keys, n_min, gamma, out_n);
}

ann_status ann_rescore(ann_index *index, uint32_t level, const float *q, uint32_t nq, const uint32_t *cand_ids,
                       uint32_t n_cand, uint32_t cand_stride, uint32_t *out_ids, float *out_keys, int32_t *out_idot,
                       void *stream) {
  hipStream_t st = (hipStream_t)stream;
  if (!index || !q || !cand_ids || !out_ids) return fail(ANN_EINVAL, "ann_rescore: NULL argument");
  if (level >= index->n_levels) return fail(ANN_EINVAL, "ann_rescore: level %u not in the index", level);
  if (nq == 0 || n_cand == 0) return fail(ANN_EINVAL, "ann_rescore: nq and n_cand must be positive");
  if (cand_stride < n_cand) return fail(ANN_EINVAL, "ann_rescore: cand_stride = %u < n_cand = %u", cand_stride, n_cand);
  if (n_cand > 4096) return fail(ANN_ECAPACITY, "ann_rescore: n_cand = %u exceeds 4096", n_cand);
  WorkspaceLease lease;
  ann_status rc = launch_query_prep(index, level, q, nq, nullptr, nullptr, nullptr, st, lease);
  if (rc != ANN_OK) return rc;
  const LevelDev &L = index->level[level];
  const Workspace &w = *lease.ws;
  const float *norm = index->key_metric == ANN_L2 ? L.norm_term : nullptr;
  const size_t smem = (size_t)n_cand * (sizeof(uint64_t) + sizeof(int32_t));
#define ANN_RS(B, P)                                                                                              \
  rescore_kernel<B, P><<<nq, 64, smem, st>>>(L.codes, L.row_stride, L.row_stride / 16, norm, index->key_metric,   \
                                             index->n, w.tq, w.tq_stride, w.tq_plane,                             \
                                             index->query_bits == 15 ? w.sum_t + w.nq_cap : nullptr, w.s, w.qlo,  \
                                             w.sum_t, nq, cand_ids,                                               \
                                             n_cand, cand_stride, out_ids, out_keys, out_idot)
  if (L.bits == 8) {
    switch (L.lanes_per_row) {
      case 8: ANN_RS(8, 8); break;
      case 16: ANN_RS(8, 16); break;
      case 32: ANN_RS(8, 32); break;
      default: ANN_RS(8, 64); break;
    }
  } else {
    switch (L.lanes_per_row) {
      case 8: ANN_RS(4, 8); break;
      case 16: ANN_RS(4, 16); break;
      case 32: ANN_RS(4, 32); break;
      default: ANN_RS(4, 64); break;
    }
  }
#undef ANN_RS
  ANN_HIP(hipGetLastError());
  return ANN_OK;
}

}  // extern "C"
