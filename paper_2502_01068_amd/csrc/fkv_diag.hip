// Diagnostics of Sec. 3 on device-resident selection results: how many indices two kept sets
// share (the overlap of critical-token sets between layers, Sec. 3.1) and which share of a score
// row's mass a kept set covers (the attention recall of a token subset, Sec. 3.2).  One block per
// row; integer counts are exact, mass sums are accumulated in fp64 in a fixed order.
#include "fkv_internal.h"

namespace fkv {

constexpr int kDiagThreads = 1024;
constexpr int kDiagWaves = kDiagThreads / 64;

// a, b ascending and duplicate-free: every element of a is looked up in b by binary search.
__global__ __launch_bounds__(kDiagThreads) void k_index_overlap(DiagOverlapArgs p) {
  __shared__ unsigned wcount[kDiagWaves];
  const int row = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int32_t *a = p.a + (int64_t)row * p.a_stride;
  const int32_t *b = p.b + (int64_t)row * p.b_stride;
  unsigned mine = 0;
  for (int i = threadIdx.x; i < p.n_a; i += kDiagThreads) {
    const int32_t x = a[i];
    int lo = 0, hi = p.n_b;  // first position of b with b[pos] >= x
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (b[mid] < x) lo = mid + 1; else hi = mid;
    }
    mine += (lo < p.n_b && b[lo] == x) ? 1u : 0u;
  }
  for (int off = 32; off > 0; off >>= 1) mine += __shfl_down(mine, off);
  if (lane == 0) wcount[wave] = mine;
  __syncthreads();
  if (threadIdx.x == 0) {
    unsigned tot = 0;
    for (int w = 0; w < kDiagWaves; ++w) tot += wcount[w];
    p.count_out[row] = (int32_t)tot;
  }
}

// Fixed-order block sum: thread-strided partial sums, a shuffle tree per wave, waves in order.
__device__ __forceinline__ double block_sum(double x, double *wsum) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int off = 32; off > 0; off >>= 1) x += __shfl_down(x, off);
  __syncthreads();  // wsum may still be read from the previous use
  if (lane == 0) wsum[wave] = x;
  __syncthreads();
  double tot = 0.0;
  for (int w = 0; w < kDiagWaves; ++w) tot += wsum[w];
  return tot;
}

__global__ __launch_bounds__(kDiagThreads) void k_mass_recall(DiagRecallArgs p) {
  __shared__ double wsum[kDiagWaves];
  const int row = blockIdx.x;
  const float *sc = p.scores + (int64_t)row * p.row_stride;
  const int32_t *idx = p.idx + (int64_t)row * p.idx_stride;
  double total = 0.0, kept = 0.0;
  for (int j = threadIdx.x; j < p.n_scores; j += kDiagThreads) total += (double)sc[j];
  for (int t = threadIdx.x; t < p.n_idx; t += kDiagThreads) {
    const int32_t j = idx[t];
    if (j >= 0 && j < p.n_scores) kept += (double)sc[j];  // window positions carry no score
  }
  total = block_sum(total, wsum);
  kept = block_sum(kept, wsum);
  if (threadIdx.x == 0) p.recall_out[row] = total > 0.0 ? (float)(kept / total) : 0.f;
}

hipError_t launch_index_overlap(const DiagOverlapArgs &p, int n_rows, hipStream_t s) {
  hipLaunchKernelGGL(k_index_overlap, dim3(n_rows), dim3(kDiagThreads), 0, s, p);
  return hipGetLastError();
}
hipError_t launch_mass_recall(const DiagRecallArgs &p, int n_rows, hipStream_t s) {
  hipLaunchKernelGGL(k_mass_recall, dim3(n_rows), dim3(kDiagThreads), 0, s, p);
  return hipGetLastError();
}

}  // namespace fkv
