// Exact k nearest neighbours by exhaustive search: the ground truth NN_k of
// the paper's recall measure (Section 6.1).  The Q.X^T contraction runs on the
// matrix cores (fp32 MFMA 32x32x2); a threshold-and-buffer top-k in LDS keeps
// k + margin candidates per (query, base slab); the candidates of all slabs
// are then re-evaluated directly in fp64 (rerank kernel) and sorted by
// (distance, id), so the decomposed fp32 scores only ever select candidates.
#include "ann_internal.hpp"
#include "device_utils.hpp"

namespace ann {

ann_status rerank_device(const float *X, uint64_t n, uint32_t d, uint32_t metric, const float *Q, uint32_t nq,
                         const uint32_t *cand, uint32_t n_cand, uint32_t stride, uint32_t k, uint32_t *out_ids,
                         float *out_dist, hipStream_t st);

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kQT = 32;    // queries per workgroup
constexpr int kBT = 128;   // base vectors per tile (4 wavefronts x 32)
constexpr int kKC = 32;    // K chunk staged in LDS
constexpr int kLd = kKC + 1;  // padded row length (floats): conflict-free column reads

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
  const uint32_t cb = kp + kBT;            // buffer: survivors plus one tile of pushes
  if (cb > 8 * kWave) return fail(ANN_ECAPACITY, "ann_bruteforce_topk: internal buffer too small for k = %u", k);
  const uint32_t q_tiles = (nq + kQT - 1) / kQT;
  // enough workgroups to fill the chip, at most 4096 exact re-evaluations per query
  uint32_t slabs = (1024 + q_tiles - 1) / q_tiles;
  const uint64_t tiles = (n + kBT - 1) / kBT;
  if (slabs > tiles) slabs = (uint32_t)tiles;
  if (slabs * kp > 4096) slabs = 4096 / kp;
  if (slabs < 1) slabs = 1;
  uint64_t rows_per_slab = ((tiles + slabs - 1) / slabs) * kBT;
  slabs = (uint32_t)((n + rows_per_slab - 1) / rows_per_slab);

  float *xnorm = nullptr;
  uint32_t *cand = nullptr;
  const size_t smem = (size_t)2 * (kQT + kBT) * kLd * sizeof(float) + kQT * (sizeof(float) + sizeof(uint32_t)) +
                      (size_t)kQT * cb * sizeof(uint64_t);
  const bool vec4 = d % 4 == 0;
  hipError_t e = hipFuncSetAttribute(vec4 ? reinterpret_cast<const void *>(bf_tile_kernel<true>)
                                          : reinterpret_cast<const void *>(bf_tile_kernel<false>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (e != hipSuccess) return hip_fail(e, "hipFuncSetAttribute");
  ANN_HIP(hipMalloc((void **)&cand, (size_t)nq * slabs * kp * sizeof(uint32_t)));
  if (metric == ANN_L2) {
    e = hipMalloc((void **)&xnorm, (size_t)n * sizeof(float));
    if (e != hipSuccess) {
      (void)hipFree(cand);
      return hip_fail(e, "hipMalloc");
    }
    row_norm_kernel<<<2048, 256, 0, st>>>(x, n, d, xnorm);
  }
  if (vec4)
    bf_tile_kernel<true><<<dim3(q_tiles, slabs), 256, smem, st>>>(x, xnorm, n, d, q, nq, metric, rows_per_slab, kp, cb, cand);
  else
    bf_tile_kernel<false><<<dim3(q_tiles, slabs), 256, smem, st>>>(x, xnorm, n, d, q, nq, metric, rows_per_slab, kp, cb, cand);
  e = hipGetLastError();
  ann_status rc = e == hipSuccess ? rerank_device(x, n, d, metric, q, nq, cand, slabs * kp, slabs * kp, k, out_ids,
                                                  out_dist, st)
                                  : hip_fail(e, "bf_tile_kernel launch");
  hipError_t e2 = hipStreamSynchronize(st);
  (void)hipFree(cand);
  (void)hipFree(xnorm);
  if (rc != ANN_OK) return rc;
  if (e2 != hipSuccess) return hip_fail(e2, "hipStreamSynchronize");
  return ANN_OK;
}
