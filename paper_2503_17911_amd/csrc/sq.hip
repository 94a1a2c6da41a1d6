// Scalar quantization: codebook training, encoding, and query folding.
// Paper Appendix G (SQ-b: uniform levels over the value range of a dimension)
// and Section 5.2 (stored squared norm; query terms precomputed before search).
#include <math.h>

#include <vector>

#include "ann_internal.hpp"
#include "device_utils.hpp"

namespace ann {

// ------------------------------------------------------------- codebook
// Column-wise min/max over a slab of rows.  Thread t of a block walks columns
// t, t+blockDim, ... so that a wavefront reads consecutive floats of one row.
__global__ void sq_minmax_partial_kernel(const float *__restrict__ x, uint64_t n, uint32_t d, uint32_t rows_per_block,
                                         float *__restrict__ pmin, float *__restrict__ pmax) {
  uint64_t r0 = (uint64_t)blockIdx.x * rows_per_block;
  uint64_t r1 = r0 + rows_per_block < n ? r0 + rows_per_block : n;
  for (uint32_t j = threadIdx.x; j < d; j += blockDim.x) {
    float mn = INFINITY, mx = -INFINITY;
    for (uint64_t i = r0; i < r1; ++i) {
      float v = x[i * d + j];
      mn = fminf(mn, v);
      mx = fmaxf(mx, v);
    }
    pmin[(uint64_t)blockIdx.x * d + j] = mn;
    pmax[(uint64_t)blockIdx.x * d + j] = mx;
  }
}

__global__ void sq_minmax_final_kernel(const float *__restrict__ pmin, const float *__restrict__ pmax, uint32_t nblocks,
                                       uint32_t d, float levels, float *__restrict__ lo, float *__restrict__ delta) {
  uint32_t j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= d) return;
  float mn = INFINITY, mx = -INFINITY;
  for (uint32_t b = 0; b < nblocks; ++b) {
    mn = fminf(mn, pmin[(uint64_t)b * d + j]);
    mx = fmaxf(mx, pmax[(uint64_t)b * d + j]);
  }
  lo[j] = mn;
  delta[j] = (mx > mn) ? __fdiv_rn(__fsub_rn(mx, mn), levels) : 1.0f;
}

// ------------------------------------------------------------- truncated range
// Exact order statistics of every column by radix selection on the ordered
// bit pattern of the floats: four passes of 8 bits; each pass histograms the
// next digit of the elements that still match the prefix found so far.  Two
// selections per column run side by side (lower and upper end of the range).
constexpr int kSelCols = 32;  // columns per workgroup

__global__ __launch_bounds__(256) void radix_hist_kernel(const float *__restrict__ x, uint64_t n, uint32_t d,
                                                         uint32_t rows_per_block, int shift,
                                                         const uint32_t *__restrict__ prefix /*[2][d]*/,
                                                         uint32_t *__restrict__ hist /*[2][d][256]*/) {
  __shared__ uint32_t lh[2][kSelCols][256];
  for (int e = threadIdx.x; e < 2 * kSelCols * 256; e += 256) (&lh[0][0][0])[e] = 0;
  __syncthreads();
  const uint32_t c = threadIdx.x % kSelCols, col = blockIdx.y * kSelCols + c;
  const uint64_t r0 = (uint64_t)blockIdx.x * rows_per_block;
  const uint64_t r1 = r0 + rows_per_block < n ? r0 + rows_per_block : n;
  if (col < d) {
    const uint32_t p0 = prefix[col], p1 = prefix[d + col];
    for (uint64_t i = r0 + threadIdx.x / kSelCols; i < r1; i += 256 / kSelCols) {
      const uint32_t key = order_u32(x[i * d + col]);
      const uint32_t digit = (key >> shift) & 255u;
      const uint32_t high = shift == 24 ? 0u : key >> (shift + 8);
      if (high == p0) atomicAdd(&lh[0][c][digit], 1u);
      if (high == p1) atomicAdd(&lh[1][c][digit], 1u);
    }
  }
  __syncthreads();
  for (int e = threadIdx.x; e < 2 * kSelCols * 256; e += 256) {
    const int sel = e / (kSelCols * 256), cc = (e / 256) % kSelCols, b = e % 256;
    const uint32_t v = lh[sel][cc][b], gc = blockIdx.y * kSelCols + cc;
    if (v != 0 && gc < d) atomicAdd(&hist[((size_t)sel * d + gc) * 256 + b], v);
  }
}

// One thread per (selection, column): the digit whose bucket holds the wanted rank.
__global__ void radix_pick_kernel(const uint32_t *__restrict__ hist, uint32_t d, uint32_t *__restrict__ prefix,
                                  uint32_t *__restrict__ rank) {
  const uint32_t t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= 2 * d) return;
  const uint32_t *h = hist + (size_t)t * 256;
  uint32_t want = rank[t], cum = 0, b = 0;
  for (; b < 255; ++b) {
    if (want < cum + h[b]) break;
    cum += h[b];
  }
  rank[t] = want - cum;
  prefix[t] = (prefix[t] << 8) | b;
}

__global__ void truncated_range_kernel(const uint32_t *__restrict__ prefix, uint32_t d, float levels,
                                       float *__restrict__ lo, float *__restrict__ delta) {
  const uint32_t j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= d) return;
  const float mn = unorder_f32(prefix[j]), mx = unorder_f32(prefix[d + j]);
  lo[j] = mn;
  delta[j] = (mx > mn) ? __fdiv_rn(__fsub_rn(mx, mn), levels) : 1.0f;
}

// ------------------------------------------------------------- encoder
// One wavefront per row.  Lanes quantize strided dimensions; the squared norm
// of the decoded row is summed by one lane in dimension order in fp64 so that
// it is reproducible bit for bit (each product of two floats is exact in fp64).
template <int BITS>
__global__ __launch_bounds__(256) void sq_encode_kernel(const float *__restrict__ x, uint64_t n, uint32_t d,
                                                        const float *__restrict__ lo, const float *__restrict__ delta,
                                                        uint8_t *__restrict__ codes, float *__restrict__ norm_term) {
  extern __shared__ float xhat_smem[];  // [waves per block][d]
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const int waves_per_block = blockDim.x / kWave;
  float *xhat = xhat_smem + (size_t)wave * d;
  const uint32_t row_bytes = BITS == 8 ? d : d / 2;
  const int maxc = (1 << BITS) - 1;
  for (uint64_t i = (uint64_t)blockIdx.x * waves_per_block + wave; i < n; i += (uint64_t)gridDim.x * waves_per_block) {
    const float *xr = x + i * d;
    uint8_t *cr = codes + i * row_bytes;
    if constexpr (BITS == 8) {
      for (uint32_t j = lane; j < d; j += kWave) {
        float u = __fadd_rn(__fdiv_rn(__fsub_rn(xr[j], lo[j]), delta[j]), 0.5f);
        int c = !(u > 0.0f) ? 0 : (u >= (float)(maxc + 1) ? maxc : (int)floorf(u));
        cr[j] = (uint8_t)c;
        xhat[j] = __fadd_rn(lo[j], __fmul_rn(delta[j], (float)c));
      }
    } else {
      for (uint32_t b = lane; b < row_bytes; b += kWave) {
        int cc[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          uint32_t j = 2 * b + h;
          float u = __fadd_rn(__fdiv_rn(__fsub_rn(xr[j], lo[j]), delta[j]), 0.5f);
          int c = !(u > 0.0f) ? 0 : (u >= (float)(maxc + 1) ? maxc : (int)floorf(u));
          cc[h] = c;
          xhat[j] = __fadd_rn(lo[j], __fmul_rn(delta[j], (float)c));
        }
        cr[b] = (uint8_t)(cc[0] | (cc[1] << 4));
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    if (norm_term && lane == 0) {
      double acc = 0.0;
      for (uint32_t j = 0; j < d; ++j) acc += (double)xhat[j] * (double)xhat[j];
      norm_term[i] = (float)acc;
    }
    __builtin_amdgcn_wave_barrier();
  }
}

// ------------------------------------------------------------- query folding
// One wavefront per query.  a_j = delta_j q_j; s = max|a|/127; t_j =
// rint(a_j * (127/max|a|)) in [-127,127]; qlo = sum_j q_j lo_j in fp64 in
// dimension order.  Writes the folded query in the layout the
// search kernels load (see chunk_dot) and optionally as plain [nq][d] int8.
template <int BITS>
__global__ __launch_bounds__(64) void query_prep_kernel(const float *__restrict__ q, uint32_t nq, uint32_t d,
                                                        const float *__restrict__ lo, const float *__restrict__ delta,
                                                        uint8_t *__restrict__ tq, uint32_t tq_stride,
                                                        uint32_t tq_plane, uint32_t nq_cap,
                                                        float *__restrict__ s_ws, float *__restrict__ qlo_ws,
                                                        int32_t *__restrict__ sum_t_ws, int8_t *__restrict__ t_plain,
                                                        float *__restrict__ s_out, float *__restrict__ qlo_out) {
  // One plane: the int8 query.  Two planes (tq_stride == 2 * tq_plane): the
  // 15-bit query t = 128 * hi + lo with lo in [-64, 63], high bytes first.
  const bool q15 = tq_stride != tq_plane;
  const float top = q15 ? 16256.0f : 127.0f;
  const uint32_t qi = blockIdx.x;
  if (qi >= nq) return;
  const int lane = threadIdx.x;
  const float *qr = q + (uint64_t)qi * d;
  float amax = 0.0f;
  for (uint32_t j = lane; j < d; j += kWave) amax = fmaxf(amax, fabsf(__fmul_rn(delta[j], qr[j])));
  amax = wave_max_f32(amax);
  float s = 1.0f, r = 0.0f;
  if (amax > 0.0f) {
    s = __fdiv_rn(amax, top);
    r = __fdiv_rn(top, amax);
  }
  uint8_t *tq_row = tq + (uint64_t)qi * tq_stride;
  int sum = 0, sum_lo = 0;
  const int limit = q15 ? 16256 : 127;
  for (uint32_t j = lane; j < tq_plane; j += kWave) {
    // byte j of the kernel layout holds dimension dim(j)
    uint32_t dim;
    if constexpr (BITS == 8) {
      dim = j;
    } else {
      uint32_t chunk = j / 32, within = j % 32, word = (within % 16) / 4, byte = within % 4, odd = within / 16;
      dim = chunk * 32 + word * 8 + byte * 2 + odd;
    }
    int ti = 0;
    if (dim < d) {
      float a = __fmul_rn(delta[dim], qr[dim]);
      ti = __float2int_rn(__fmul_rn(a, r));  // round half to even
      ti = ti > limit ? limit : (ti < -limit ? -limit : ti);
      if (t_plain) {
        if (q15)
          reinterpret_cast<int16_t *>(t_plain)[(uint64_t)qi * d + dim] = (int16_t)ti;
        else
          t_plain[(uint64_t)qi * d + dim] = (int8_t)ti;
      }
    }
    if (q15) {
      const int low = ((ti + 64) & 127) - 64, high = (ti - low) >> 7;
      tq_row[j] = (uint8_t)(int8_t)high;
      tq_row[tq_plane + j] = (uint8_t)(int8_t)low;
      sum += high;
      sum_lo += low;
    } else {
      tq_row[j] = (uint8_t)(int8_t)ti;
      sum += ti;
    }
  }
  sum = group_sum_i32<64>(sum);
  sum_lo = group_sum_i32<64>(sum_lo);
  // every product of two floats is exact in fp64; they are formed by all lanes
  // and then added by one lane in dimension order, which fixes the rounding
  extern __shared__ double prod[];
  for (uint32_t j = lane; j < d; j += kWave) prod[j] = (double)qr[j] * (double)lo[j];
  __syncthreads();
  if (lane == 0) {
    double acc = 0.0;
    for (uint32_t j = 0; j < d; ++j) acc += prod[j];
    float qlo = (float)acc;
    s_ws[qi] = s;
    qlo_ws[qi] = qlo;
    sum_t_ws[qi] = sum;
    sum_t_ws[nq_cap + qi] = sum_lo;
    if (s_out) s_out[qi] = s;
    if (qlo_out) qlo_out[qi] = qlo;
  }
}

ann_status launch_query_prep_into(const ann_index *ix, uint32_t level, const float *q, uint32_t nq, const Workspace &w,
                                  int8_t *t_plain, float *s_out, float *qlo_out, hipStream_t st) {
  const LevelDev &L = ix->level[level];
  const size_t smem = (size_t)ix->d * sizeof(double);
  if (L.bits == 8)
    query_prep_kernel<8><<<nq, 64, smem, st>>>(q, nq, ix->d, L.lo, L.delta, w.tq, w.tq_stride, w.tq_plane, w.nq_cap, w.s, w.qlo, w.sum_t,
                                               t_plain, s_out, qlo_out);
  else
    query_prep_kernel<4><<<nq, 64, smem, st>>>(q, nq, ix->d, L.lo, L.delta, w.tq, w.tq_stride, w.tq_plane, w.nq_cap, w.s, w.qlo, w.sum_t,
                                               t_plain, s_out, qlo_out);
  ANN_HIP(hipGetLastError());
  return ANN_OK;
}

ann_status launch_query_prep(ann_index *ix, uint32_t level, const float *q, uint32_t nq, int8_t *t_plain, float *s_out,
                             float *qlo_out, hipStream_t st, WorkspaceLease &lease) {
  ann_status rc = workspace_for(ix, level, nq, st, lease);
  if (rc != ANN_OK) return rc;
  rc = launch_query_prep_into(ix, level, q, nq, *lease.ws, t_plain, s_out, qlo_out, st);
  if (rc != ANN_OK) return rc;
  lease.ws->folded_q = q;
  lease.ws->folded_nq = nq;
  return ANN_OK;
}

}  // namespace ann

using namespace ann;

extern "C" {

ann_status ann_sq_train(const float *x, uint64_t n, uint32_t d, uint32_t bits, float *lo, float *delta, void *stream) {
  hipStream_t st = (hipStream_t)stream;
  if (!x || !lo || !delta) return fail(ANN_EINVAL, "ann_sq_train: NULL argument");
  if (n == 0 || d == 0) return fail(ANN_EINVAL, "ann_sq_train: empty input");
  if (bits != 8 && bits != 4) return fail(ANN_EINVAL, "ann_sq_train: bits must be 4 or 8");
  const uint32_t rows_per_block = 512;
  const uint32_t nblocks = (uint32_t)((n + rows_per_block - 1) / rows_per_block);
  float *pmin = nullptr, *pmax = nullptr;
  ANN_HIP(hipMalloc((void **)&pmin, (size_t)nblocks * d * sizeof(float)));
  hipError_t e = hipMalloc((void **)&pmax, (size_t)nblocks * d * sizeof(float));
  if (e != hipSuccess) {
    (void)hipFree(pmin);
    return hip_fail(e, "hipMalloc");
  }
  sq_minmax_partial_kernel<<<nblocks, 256, 0, st>>>(x, n, d, rows_per_block, pmin, pmax);
  sq_minmax_final_kernel<<<(d + 255) / 256, 256, 0, st>>>(pmin, pmax, nblocks, d, (float)((1u << bits) - 1u), lo, delta);
  e = hipGetLastError();
  hipError_t e2 = hipStreamSynchronize(st);
  (void)hipFree(pmin);
  (void)hipFree(pmax);
  if (e != hipSuccess) return hip_fail(e, "sq_minmax launch");
  if (e2 != hipSuccess) return hip_fail(e2, "hipStreamSynchronize");
  return ANN_OK;
}

ann_status ann_sq_train_truncated(const float *x, uint64_t n, uint32_t d, uint32_t bits, double coverage, float *lo,
                                  float *delta, void *stream) {
  hipStream_t st = (hipStream_t)stream;
  if (!x || !lo || !delta) return fail(ANN_EINVAL, "ann_sq_train_truncated: NULL argument");
  if (n == 0 || n >= (1ull << 31) || d == 0) return fail(ANN_EINVAL, "ann_sq_train_truncated: empty input or n >= 2^31");
  if (bits != 8 && bits != 4) return fail(ANN_EINVAL, "ann_sq_train_truncated: bits must be 4 or 8");
  if (!(coverage > 0.5 && coverage <= 1.0)) return fail(ANN_EINVAL, "ann_sq_train_truncated: coverage must be in (0.5, 1]");
  const uint64_t k = (uint64_t)floor((1.0 - coverage) * (double)(n - 1));
  uint32_t *hist = nullptr, *state = nullptr;  // state: prefix[2][d], rank[2][d]
  ANN_HIP(hipMalloc((void **)&hist, (size_t)2 * d * 256 * sizeof(uint32_t)));
  hipError_t e = hipMalloc((void **)&state, (size_t)4 * d * sizeof(uint32_t));
  if (e != hipSuccess) {
    (void)hipFree(hist);
    return hip_fail(e, "hipMalloc");
  }
  std::vector<uint32_t> init((size_t)4 * d, 0u);
  for (uint32_t j = 0; j < d; ++j) {
    init[(size_t)2 * d + j] = (uint32_t)k;
    init[(size_t)3 * d + j] = (uint32_t)(n - 1 - k);
  }
  e = hipMemcpyAsync(state, init.data(), init.size() * sizeof(uint32_t), hipMemcpyHostToDevice, st);
  const uint32_t rows_per_block = 4096;
  const dim3 grid((uint32_t)((n + rows_per_block - 1) / rows_per_block), (d + kSelCols - 1) / kSelCols);
  for (int shift = 24; shift >= 0 && e == hipSuccess; shift -= 8) {
    e = hipMemsetAsync(hist, 0, (size_t)2 * d * 256 * sizeof(uint32_t), st);
    if (e != hipSuccess) break;
    radix_hist_kernel<<<grid, 256, 0, st>>>(x, n, d, rows_per_block, shift, state, hist);
    radix_pick_kernel<<<(2 * d + 255) / 256, 256, 0, st>>>(hist, d, state, state + (size_t)2 * d);
    e = hipGetLastError();
  }
  if (e == hipSuccess) {
    truncated_range_kernel<<<(d + 255) / 256, 256, 0, st>>>(state, d, (float)((1u << bits) - 1u), lo, delta);
    e = hipGetLastError();
  }
  hipError_t e2 = hipStreamSynchronize(st);  // also keeps `init` alive until the copy is done
  (void)hipFree(hist);
  (void)hipFree(state);
  if (e != hipSuccess) return hip_fail(e, "ann_sq_train_truncated");
  if (e2 != hipSuccess) return hip_fail(e2, "hipStreamSynchronize");
  return ANN_OK;
}

ann_status ann_sq_encode(const float *x, uint64_t n, uint32_t d, uint32_t bits, const float *lo, const float *delta,
                         uint8_t *codes, float *norm_term, void *stream) {
  hipStream_t st = (hipStream_t)stream;
  if (!x || !lo || !delta || !codes) return fail(ANN_EINVAL, "ann_sq_encode: NULL argument");
  if (n == 0 || d == 0) return fail(ANN_EINVAL, "ann_sq_encode: empty input");
  if (bits != 8 && bits != 4) return fail(ANN_EINVAL, "ann_sq_encode: bits must be 4 or 8");
  if (bits == 4 && (d & 1)) return fail(ANN_EINVAL, "ann_sq_encode: 4-bit codes need an even d");
  if (d > 2048) return fail(ANN_ECAPACITY, "ann_sq_encode: d = %u exceeds 2048", d);
  const int block = 256, waves = block / kWave;
  uint64_t want = (n + waves - 1) / waves;
  int grid = (int)(want > 16384 ? 16384 : want);
  size_t smem = (size_t)waves * d * sizeof(float);
  if (bits == 8)
    sq_encode_kernel<8><<<grid, block, smem, st>>>(x, n, d, lo, delta, codes, norm_term);
  else
    sq_encode_kernel<4><<<grid, block, smem, st>>>(x, n, d, lo, delta, codes, norm_term);
  ANN_HIP(hipGetLastError());
  ANN_HIP(hipStreamSynchronize(st));
  return ANN_OK;
}

ann_status ann_query_prep(ann_index *index, uint32_t level, const float *q, uint32_t nq, int8_t *t, float *s, float *qlo,
                          void *stream) {
  if (!index || !q) return fail(ANN_EINVAL, "ann_query_prep: NULL argument");
  if (level >= index->n_levels) return fail(ANN_EINVAL, "ann_query_prep: level %u not in the index", level);
  if (nq == 0) return fail(ANN_EINVAL, "ann_query_prep: nq == 0");
  WorkspaceLease lease;
  return launch_query_prep(index, level, q, nq, t, s, qlo, (hipStream_t)stream, lease);
}

}  // extern "C"
