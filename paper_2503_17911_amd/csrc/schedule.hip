// Processing order of a batch: queries that will walk the same part of the
// graph are run at the same time on the same XCD (accelerator die), so that
// the code rows and adjacency rows they share are fetched into that die's L2
// once.  Results do not depend on the order; only the time does.
//
// The caller supplies one 32-bit key per query that is equal or close for
// similar queries (the node id of the closest of a few scanned pivots, as
// written by ann_entry_scan, serves).  Queries are grouped by key bucket
// (counting sort in LDS, one workgroup), and the grouped list is dealt out so
// that workgroup b - which the dispatcher places on die b mod 8 - takes the
// next query of the b mod 8-th eighth of the list.
#include "ann_internal.hpp"
#include "device_utils.hpp"

namespace ann {

constexpr int kDies = 8;             // XCDs of the MI355X; workgroups are dealt to them round-robin
constexpr int kBuckets = 4096;       // key buckets (LDS histogram)
constexpr int kScheduleThreads = 1024;

__global__ __launch_bounds__(kScheduleThreads) void schedule_kernel(const uint32_t *__restrict__ keys, uint32_t nq,
                                                                    uint32_t key_range, uint32_t *__restrict__ order) {
  __shared__ uint32_t count[kBuckets];
  __shared__ uint32_t partial[kScheduleThreads / kWave];
  const uint32_t tid = threadIdx.x;
  for (uint32_t b = tid; b < kBuckets; b += kScheduleThreads) count[b] = 0;
  __syncthreads();
  // floor(key * kBuckets / key_range) in fp64: both operands are integers below
  // 2^53 and the quotient, when not an integer, is at least 2^-32 away from one,
  // far more than the rounding of the division, so the floor is the exact one
  // (an integer division of 64-bit values costs ten times as many instructions).
  auto bucket_of = [&](uint32_t key) {
    const uint32_t kc = key < key_range ? key : key_range - 1;
    return (uint32_t)((double)((uint64_t)kc * kBuckets) / (double)key_range);
  };
  // (keys are read eight at a time per thread, so that the loads are in flight together)
  constexpr int kBatch = 8;
  for (uint32_t base = 0; base < nq; base += kBatch * kScheduleThreads) {
    uint32_t kv[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const uint32_t i = base + u * kScheduleThreads + tid;
      kv[u] = i < nq ? keys[i] : 0u;
    }
#pragma unroll
    for (int u = 0; u < kBatch; ++u)
      if (base + u * kScheduleThreads + tid < nq) atomicAdd(&count[bucket_of(kv[u])], 1u);
  }
  __syncthreads();
  // exclusive prefix sums over the buckets: four per thread, then over threads
  constexpr int kPer = kBuckets / kScheduleThreads;
  uint32_t local[kPer], sum = 0;
#pragma unroll
  for (int j = 0; j < kPer; ++j) {
    local[j] = sum;
    sum += count[tid * kPer + j];
  }
  // prefix over the threads: inside a wavefront by lane exchanges, then the 16 wavefront totals
  const uint32_t in_wave = (uint32_t)wave_inclusive_scan_i32((int)sum);
  if (tid % kWave == kWave - 1) partial[tid / kWave] = in_wave;
  __syncthreads();
  uint32_t waves_before = 0;
  for (uint32_t w = 0; w < tid / kWave; ++w) waves_before += partial[w];
  const uint32_t before = waves_before + in_wave - sum;
#pragma unroll
  for (int j = 0; j < kPer; ++j) count[tid * kPer + j] = before + local[j];  // now: next free rank of the bucket
  __syncthreads();
  // Rank g in the grouped list belongs to the die whose run contains it: die x
  // owns ceil((nq - x) / 8) consecutive ranks, and its t-th rank is searched by
  // workgroup 8 t + x.
  for (uint32_t base = 0; base < nq; base += kBatch * kScheduleThreads) {
    uint32_t kv[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const uint32_t i = base + u * kScheduleThreads + tid;
      kv[u] = i < nq ? keys[i] : 0u;
    }
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const uint32_t i = base + u * kScheduleThreads + tid;
      if (i >= nq) continue;
      const uint32_t g = atomicAdd(&count[bucket_of(kv[u])], 1u);
      uint32_t x = 0, start = 0;
      for (uint32_t y = 0; y + 1 < (uint32_t)kDies && y < nq; ++y) {
        const uint32_t owned = (nq - y + kDies - 1) / kDies;
        if (g < start + owned) break;
        start += owned;
        x = y + 1;
      }
      order[(g - start) * kDies + x] = i;
    }
  }
}

}  // namespace ann

using namespace ann;

extern "C" ann_status ann_schedule_queries(const uint32_t *keys, uint32_t nq, uint32_t key_range, uint32_t *out_order,
                                           void *stream) {
  if (!keys || !out_order) return fail(ANN_EINVAL, "ann_schedule_queries: NULL argument");
  if (nq == 0) return fail(ANN_EINVAL, "ann_schedule_queries: nq == 0");
  if (key_range == 0) return fail(ANN_EINVAL, "ann_schedule_queries: key_range == 0");
  schedule_kernel<<<1, kScheduleThreads, 0, (hipStream_t)stream>>>(keys, nq, key_range, out_order);
  ANN_HIP(hipGetLastError());
  return ANN_OK;
}
