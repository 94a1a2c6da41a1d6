// Entry-point stage: choose the initial nodes I of Algorithm 1 per query.
// The paper takes I as an input of the search ("initial nodes I"); a fixed
// sample of base vectors (pivots) is scanned with the same low-precision
// distance tau_l as the traversal, and the closest few become the query's
// initial nodes.  One query per wavefront; the pivot codes are a compact copy,
// read sequentially.
#include "ann_internal.hpp"
#include "device_utils.hpp"

namespace ann {

constexpr int kScanKeep = 4;  // best pivots kept per lane and returned at most

__device__ __forceinline__ uint64_t pack_ki(uint32_t hi, uint32_t lo) { return ((uint64_t)hi << 32) | lo; }

template <int BITS, int LPR>
__global__ __launch_bounds__(64) void entry_scan_kernel(const uint8_t *__restrict__ pcodes,
                                                        const float *__restrict__ pnorm,
                                                        const uint32_t *__restrict__ pids, uint32_t n_pivots,
                                                        uint32_t row_stride, uint32_t n_chunks, uint32_t metric,
                                                        const uint8_t *__restrict__ tq, uint32_t tq_stride,
                                                        uint32_t tq_plane, const int32_t *__restrict__ sum_t_lo,
                                                        const float *__restrict__ s_arr,
                                                        const float *__restrict__ qlo_arr,
                                                        const int32_t *__restrict__ sum_t, uint32_t nq,
                                                        uint32_t n_entry, uint32_t *__restrict__ out) {
  const bool q15 = sum_t_lo != nullptr;  // 15-bit query: a second plane of low bytes
  constexpr int G = kWave / LPR, CPL = 4, TQW = TqRegs<BITS>::kWords;
  const uint32_t qi = blockIdx.x;
  if (qi >= nq) return;
  const int lane = threadIdx.x, sub = lane % LPR, grp = lane / LPR;
  int tqr[CPL][TQW], tqr_lo[CPL][TQW];
  uint32_t coff[CPL];
#pragma unroll
  for (int j = 0; j < CPL; ++j) {
    const uint32_t c = (uint32_t)(sub + j * LPR);
    coff[j] = (c < n_chunks ? c : n_chunks - 1) * 16u;
    const int *tqp = reinterpret_cast<const int *>(tq + (uint64_t)qi * tq_stride + c * (TQW * 4u));
#pragma unroll
    for (int w = 0; w < TQW; ++w) {
      tqr[j][w] = tqp[w];
      tqr_lo[j][w] = q15 ? tqp[tq_plane / 4 + w] : 0;
    }
  }
  const float s = s_arr[qi], qlo = qlo_arr[qi];
  const int bias = BITS == 8 ? 128 * sum_t[qi] : 0;
  const int bias_lo = BITS == 8 && q15 ? 128 * sum_t_lo[qi] : 0;
  uint64_t best[kScanKeep];
#pragma unroll
  for (int t = 0; t < kScanKeep; ++t) best[t] = ~0ull;
  // four groups of G pivots per round: their rows are requested together, so
  // that a round costs one trip to the pivot table (it stays in the L2s)
  constexpr int UNR = 4;
  for (uint32_t base = 0; base < n_pivots; base += G * UNR) {
    uint4 rows[UNR][CPL];
    float pn[UNR];
    uint32_t pid[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const uint32_t pi = base + u * G + grp;
      const uint32_t pc = pi < n_pivots ? pi : n_pivots - 1;
      const uint8_t *rp = pcodes + (uint64_t)pc * row_stride;
#pragma unroll
      for (int j = 0; j < CPL; ++j) rows[u][j] = *reinterpret_cast<const uint4 *>(rp + coff[j]);
      pn[u] = pnorm ? pnorm[pc] : 0.0f;
      pid[u] = pids[pc];
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const uint32_t pi = base + u * G + grp;
      int dot = 0, dot_lo = 0;
#pragma unroll
      for (int j = 0; j < CPL; ++j) {
        dot += chunk_dot<BITS>(rows[u][j], tqr[j]);
        if (q15) dot_lo += chunk_dot<BITS>(rows[u][j], tqr_lo[j]);
      }
      dot = group_sum_i32<LPR>(dot) + bias;
      if (q15) dot_lo = group_sum_i32<LPR>(dot_lo) + bias_lo;
      const float key = q15 ? key_from_idot15(metric, s, qlo, dot, dot_lo, pn[u]) : key_from_idot(metric, s, qlo, dot, pn[u]);
      uint64_t c = (sub == 0 && pi < n_pivots) ? pack_ki(order_u32(key), pid[u]) : ~0ull;
      // sorted insertion into this lane's short list
#pragma unroll
      for (int t = 0; t < kScanKeep; ++t) {
        const uint64_t lo = c < best[t] ? c : best[t];
        c = c < best[t] ? best[t] : c;
        best[t] = lo;
      }
    }
  }
  // the n_entry smallest over all lanes, one at a time: every lane offers the
  // head of its sorted list, the wave takes the minimum, its owner moves on
  // ((key, id) pairs are distinct except for the all-ones filler)
  for (uint32_t r = 0; r < n_entry; ++r) {
    uint64_t m = best[0];
#pragma unroll
    for (int x = 1; x < kWave; x <<= 1) {
      const uint32_t ohi = (uint32_t)xor_lane_i32((int)(uint32_t)(m >> 32), x);
      const uint32_t olo = (uint32_t)xor_lane_i32((int)(uint32_t)m, x);
      const uint64_t o = pack_ki(ohi, olo);
      m = o < m ? o : m;
    }
    if (best[0] == m && m != ~0ull) {
#pragma unroll
      for (int t = 0; t + 1 < kScanKeep; ++t) best[t] = best[t + 1];
      best[kScanKeep - 1] = ~0ull;
    }
    if (lane == 0) out[(uint64_t)qi * n_entry + r] = m == ~0ull ? ANN_PAD_ID : (uint32_t)m;
  }
}

// The same scan for the common case (8-bit codes, one entry per query, d <=
// 256) as a dense contraction on the matrix cores, with the query folding in
// front of it: a workgroup of four wavefronts takes 32 queries, folds them
// (the arithmetic of query_prep_kernel, step for step, so the folded queries
// it leaves in the workspace are the same bytes), and multiplies them against
// the pivot table with v_mfma_i32_32x32x16_i8 (integer, hence exact: the keys
// and the choice are those of entry_scan_kernel).  Wavefront w takes the pivot
// blocks w, w + 4, ...; every lane keeps the best pivot of its column for its
// 16 rows; the columns are reduced by lane exchanges, the wavefronts in LDS.
typedef int intx16 __attribute__((ext_vector_type(16)));
constexpr int kFsQueries = 32, kFsThreads = 256, kFsMaxD = 256;

__global__ __launch_bounds__(kFsThreads) void fold_scan_kernel(
    const float *__restrict__ q, uint32_t nq, uint32_t d, const float *__restrict__ lo, const float *__restrict__ delta,
    uint8_t *__restrict__ tq, uint32_t tq_stride, float *__restrict__ s_ws, float *__restrict__ qlo_ws,
    int32_t *__restrict__ sum_t_ws, const uint8_t *__restrict__ pcodes, const float *__restrict__ pnorm,
    const uint32_t *__restrict__ pids, uint32_t n_pivots, uint32_t row_stride, uint32_t metric,
    uint32_t *__restrict__ out) {
  extern __shared__ double smem_d[];
  const uint32_t pp = d + 1;                       // row pitch of prod (doubles): the serial sums of 32 lanes hit 32 banks
  const uint32_t tp = row_stride + 8;              // row pitch of tql (bytes)
  double *prod = smem_d;                                             // [32][pp]
  uint64_t *red = reinterpret_cast<uint64_t *>(prod + kFsQueries * pp);  // [4][32]
  float *s_l = reinterpret_cast<float *>(red + 4 * kFsQueries);      // [32]
  float *qlo_l = s_l + kFsQueries;                                   // [32]
  int *bias_l = reinterpret_cast<int *>(qlo_l + kFsQueries);         // [32]
  uint8_t *tql = reinterpret_cast<uint8_t *>(bias_l + kFsQueries);   // [32][tp], 8-byte aligned rows

  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const uint32_t q0 = blockIdx.x * kFsQueries;

  // ---- folding: eight threads per query, dimension j of thread part p: j % 8 == p
  {
    const int qr = tid / 8, part = tid % 8;
    const uint32_t qi = q0 + qr < nq ? q0 + qr : nq - 1;
    const float *qrow = q + (uint64_t)qi * d;
    float amax = 0.0f;
    for (uint32_t j = part; j < d; j += 8) amax = fmaxf(amax, fabsf(__fmul_rn(delta[j], qrow[j])));
#pragma unroll
    for (int m = 1; m < 8; m <<= 1) amax = fmaxf(amax, __int_as_float(xor_lane_i32(__float_as_int(amax), m)));
    float s = 1.0f, r = 0.0f;
    if (amax > 0.0f) {
      s = __fdiv_rn(amax, 127.0f);
      r = __fdiv_rn(127.0f, amax);
    }
    int sum = 0;
    for (uint32_t j = part; j < row_stride; j += 8) {
      int ti = 0;
      if (j < d) {
        const float a = __fmul_rn(delta[j], qrow[j]);
        ti = __float2int_rn(__fmul_rn(a, r));  // round half to even
        ti = ti > 127 ? 127 : (ti < -127 ? -127 : ti);
        prod[qr * pp + j] = (double)qrow[j] * (double)lo[j];
      }
      tql[qr * tp + j] = (uint8_t)(int8_t)ti;
      sum += ti;
    }
#pragma unroll
    for (int m = 1; m < 8; m <<= 1) sum += xor_lane_i32(sum, m);
    if (part == 0) {
      s_l[qr] = s;
      bias_l[qr] = 128 * sum;
      if (q0 + qr < nq) {
        s_ws[q0 + qr] = s;
        sum_t_ws[q0 + qr] = sum;
      }
    }
  }
  __syncthreads();
  if (tid < kFsQueries) {
    // every product of two floats is exact in fp64; added in dimension order, which fixes the rounding
    double acc = 0.0;
    for (uint32_t j = 0; j < d; ++j) acc += prod[tid * pp + j];
    const float qlo = (float)acc;
    qlo_l[tid] = qlo;
    if (q0 + tid < nq) qlo_ws[q0 + tid] = qlo;
  }
  // the folded queries in the layout the search kernels load (8-bit: dimension order, zero-padded)
  for (uint32_t e = tid; e < kFsQueries * (tq_stride / 8); e += kFsThreads) {
    const uint32_t qr = e / (tq_stride / 8), c8 = e % (tq_stride / 8);
    if (q0 + qr < nq) {
      const uint64_t v = c8 * 8 < row_stride ? *reinterpret_cast<const uint64_t *>(tql + qr * tp + c8 * 8) : 0ull;
      *reinterpret_cast<uint64_t *>(tq + (uint64_t)(q0 + qr) * tq_stride + c8 * 8) = v;
    }
  }
  __syncthreads();

  // ---- scan.  acc[i] is query row 8*(i/4) + 4*half + i%4 against the pivot of column lane % 32.
  const int half = lane / 32, l32 = lane % 32;
  float s_r[16], qlo_r[16];
  int bias_r[16];
  uint64_t best[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int row = 8 * (i / 4) + 4 * half + (i % 4);
    s_r[i] = s_l[row];
    qlo_r[i] = qlo_l[row];
    bias_r[i] = bias_l[row];
    best[i] = ~0ull;
  }
  const uint32_t steps = row_stride / 16;
  const uint32_t p_blocks = (n_pivots + 31) / 32;
  for (uint32_t pb = wave; pb < p_blocks; pb += 4) {
    const uint32_t pi = pb * 32 + l32;
    const uint32_t pc = pi < n_pivots ? pi : n_pivots - 1;
    const uint8_t *prow = pcodes + (uint64_t)pc * row_stride + 8 * half;
    const uint8_t *arow = tql + l32 * tp + 8 * half;
    intx16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0;
    for (uint32_t st = 0; st < steps; ++st) {
      const long a = *reinterpret_cast<const long *>(arow + 16 * st);
      const long b = *reinterpret_cast<const long *>(prow + 16 * st);
      acc = __builtin_amdgcn_mfma_i32_32x32x16_i8(a, b, acc, 0, 0, 0);
    }
    const float norm = pnorm ? pnorm[pc] : 0.0f;
    const uint32_t id = pids[pc];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float key = key_from_idot(metric, s_r[i], qlo_r[i], acc[i] + bias_r[i], norm);
      const uint64_t c = pi < n_pivots ? pack_ki(order_u32(key), id) : ~0ull;
      best[i] = c < best[i] ? c : best[i];
    }
  }
  // the best over the 32 columns of a half, then over the wavefronts
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    uint64_t m = best[i];
#pragma unroll
    for (int x = 1; x < 32; x <<= 1) {
      const uint64_t o = pack_ki((uint32_t)xor_lane_i32((int)(uint32_t)(m >> 32), x), (uint32_t)xor_lane_i32((int)(uint32_t)m, x));
      m = o < m ? o : m;
    }
    if (l32 == 0) red[wave * kFsQueries + 8 * (i / 4) + 4 * half + (i % 4)] = m;
  }
  __syncthreads();
  if (tid < kFsQueries && q0 + tid < nq) {
    uint64_t m = red[tid];
#pragma unroll
    for (int w = 1; w < 4; ++w) m = red[w * kFsQueries + tid] < m ? red[w * kFsQueries + tid] : m;
    out[q0 + tid] = m == ~0ull ? ANN_PAD_ID : (uint32_t)m;
  }
}

__global__ void gather_pivots_kernel(const uint8_t *__restrict__ codes, const float *__restrict__ norm,
                                     uint64_t n, uint32_t n_pivots, uint32_t row_stride,
                                     uint8_t *__restrict__ pcodes, float *__restrict__ pnorm,
                                     uint32_t *__restrict__ pids) {
  const uint64_t total = (uint64_t)n_pivots * (row_stride / 16);
  for (uint64_t e = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; e < total; e += (uint64_t)gridDim.x * blockDim.x) {
    const uint32_t p = (uint32_t)(e / (row_stride / 16)), c = (uint32_t)(e % (row_stride / 16));
    const uint64_t id = (uint64_t)p * n / n_pivots;  // evenly spaced sample of the base set
    reinterpret_cast<uint4 *>(pcodes)[e] = reinterpret_cast<const uint4 *>(codes + id * row_stride)[c];
    if (c == 0) {
      pids[p] = (uint32_t)id;
      if (pnorm) pnorm[p] = norm[id];
    }
  }
}

}  // namespace ann

using namespace ann;

extern "C" {

ann_status ann_build_entry_table(ann_index *index, uint32_t n_pivots, void *stream) {
  hipStream_t st = (hipStream_t)stream;
  if (!index) return fail(ANN_EINVAL, "ann_build_entry_table: index is NULL");
  if (n_pivots == 0 || n_pivots > index->n) return fail(ANN_EINVAL, "ann_build_entry_table: n_pivots must be in [1, n]");
  ANN_HIP(hipDeviceSynchronize());
  (void)hipFree(index->pivot_codes);
  (void)hipFree(index->pivot_norm);
  (void)hipFree(index->pivot_ids);
  index->pivot_codes = nullptr;
  index->pivot_norm = nullptr;
  index->pivot_ids = nullptr;
  index->n_pivots = 0;
  const LevelDev &L = index->level[0];
  ANN_HIP(hipMalloc((void **)&index->pivot_codes, (size_t)n_pivots * L.row_stride));
  ANN_HIP(hipMalloc((void **)&index->pivot_ids, (size_t)n_pivots * sizeof(uint32_t)));
  if (index->key_metric == ANN_L2) ANN_HIP(hipMalloc((void **)&index->pivot_norm, (size_t)n_pivots * sizeof(float)));
  const uint64_t total = (uint64_t)n_pivots * (L.row_stride / 16);
  const int grid = (int)((total + 255) / 256 > 65535 ? 65535 : (total + 255) / 256);
  gather_pivots_kernel<<<grid, 256, 0, st>>>(L.codes, index->key_metric == ANN_L2 ? L.norm_term : nullptr, index->n, n_pivots,
                                             L.row_stride, index->pivot_codes, index->pivot_norm, index->pivot_ids);
  ANN_HIP(hipGetLastError());
  ANN_HIP(hipStreamSynchronize(st));
  index->n_pivots = n_pivots;
  return ANN_OK;
}

ann_status ann_entry_scan(ann_index *index, const float *q, uint32_t nq, uint32_t n_entry, uint32_t *out_entry_ids,
                          void *stream) {
  hipStream_t st = (hipStream_t)stream;
  if (!index || !q || !out_entry_ids) return fail(ANN_EINVAL, "ann_entry_scan: NULL argument");
  if (index->n_pivots == 0) return fail(ANN_EINVAL, "ann_entry_scan: call ann_build_entry_table first");
  if (nq == 0 || n_entry == 0) return fail(ANN_EINVAL, "ann_entry_scan: nq and n_entry must be positive");
  if (n_entry > (uint32_t)kScanKeep) return fail(ANN_ECAPACITY, "ann_entry_scan: n_entry = %u exceeds %d", n_entry, kScanKeep);
  WorkspaceLease lease;
  const LevelDev &L = index->level[0];
  if (L.bits == 8 && n_entry == 1 && index->d <= (uint32_t)kFsMaxD && index->query_bits == 8) {
    // folding and scan in one launch, on the matrix cores
    ann_status rc = workspace_for(index, 0, nq, st, lease);
    if (rc != ANN_OK) return rc;
    Workspace *fw = lease.ws;
    const size_t smem = (size_t)kFsQueries * (index->d + 1) * sizeof(double) + 4 * kFsQueries * sizeof(uint64_t) +
                        3 * kFsQueries * 4 + (size_t)kFsQueries * (L.row_stride + 8);
    if (smem > 48 * 1024) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(fold_scan_kernel),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
      if (e != hipSuccess) return hip_fail(e, "hipFuncSetAttribute");
    }
    fold_scan_kernel<<<(nq + kFsQueries - 1) / kFsQueries, kFsThreads, smem, st>>>(
        q, nq, index->d, L.lo, L.delta, fw->tq, fw->tq_stride, fw->s, fw->qlo, fw->sum_t, index->pivot_codes,
        index->pivot_norm, index->pivot_ids, index->n_pivots, L.row_stride, index->key_metric, out_entry_ids);
    ANN_HIP(hipGetLastError());
    fw->folded_q = q;
    fw->folded_nq = nq;
    return ANN_OK;
  }
  ann_status rc = launch_query_prep(index, 0, q, nq, nullptr, nullptr, nullptr, st, lease);
  if (rc != ANN_OK) return rc;
  const Workspace &w = *lease.ws;
#define ANN_ES(B, P)                                                                                                   \
  entry_scan_kernel<B, P><<<nq, 64, 0, st>>>(index->pivot_codes, index->pivot_norm, index->pivot_ids, index->n_pivots,   \
                                             L.row_stride, L.row_stride / 16, index->key_metric, w.tq, w.tq_stride,      \
                                             w.tq_plane, index->query_bits == 15 ? w.sum_t + w.nq_cap : nullptr, w.s,  \
                                             w.qlo, w.sum_t, nq, n_entry, out_entry_ids)
  if (L.bits == 8) {
    switch (L.search_lanes) {
      case 1: ANN_ES(8, 1); break;
      case 2: ANN_ES(8, 2); break;
      case 4: ANN_ES(8, 4); break;
      case 8: ANN_ES(8, 8); break;
      default: ANN_ES(8, 16); break;
    }
  } else {
    switch (L.search_lanes) {
      case 1: ANN_ES(4, 1); break;
      case 2: ANN_ES(4, 2); break;
      case 4: ANN_ES(4, 4); break;
      case 8: ANN_ES(4, 8); break;
      default: ANN_ES(4, 16); break;
    }
  }
#undef ANN_ES
  ANN_HIP(hipGetLastError());
  return ANN_OK;
}

}  // extern "C"
