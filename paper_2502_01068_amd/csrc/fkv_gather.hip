// Index-driven row gathers (HiddenCompress / KVCompress, App. B.1): bit-exact copies of the
// kept rows into compacted buffers.  Up to three jobs (hidden rows, K rows, V rows) share one
// launch so the small K/V jobs fill the machine alongside the large hidden-row job.
//
// The unit of work is one 16-byte chunk; consecutive lanes take consecutive chunks of a row,
// so a 256-byte K/V head row is one 16-lane segment and an 8 KiB hidden row is 512 lanes.
#include "fkv_internal.h"

namespace fkv {

constexpr int kGatherThreads = 256;
constexpr int kGatherUnroll = 4;  // 16-byte chunks in flight per thread

int gather_blocks(const GatherJob &j) {
  const int64_t chunks = (int64_t)j.n_heads * j.total_rows * (j.row_bytes / 16);
  const int64_t per_block = (int64_t)kGatherThreads * kGatherUnroll;
  return (int)((chunks + per_block - 1) / per_block);
}

__global__ __launch_bounds__(kGatherThreads) void k_gather(GatherArgs a) {
  int ji = 0;
  while (ji + 1 < a.n_jobs && (int)blockIdx.x >= a.job[ji + 1].blk0) ++ji;
  const GatherJob &job = a.job[ji];
  const int cpr = job.row_bytes >> 4;  // chunks per row
  const int64_t n_chunks = (int64_t)job.n_heads * job.total_rows * cpr;
  const int64_t c0 = ((int64_t)((int)blockIdx.x - job.blk0) * kGatherUnroll) * kGatherThreads + threadIdx.x;

  u32x4 val[kGatherUnroll];
  int64_t dst_off[kGatherUnroll];
#pragma unroll
  for (int u = 0; u < kGatherUnroll; ++u) {
    const int64_t c = c0 + (int64_t)u * kGatherThreads;
    dst_off[u] = -1;
    if (c < n_chunks) {
      const int64_t rowi = c / cpr;            // h * total_rows + t
      const int col = (int)(c - rowi * cpr);
      const int h = (int)(rowi / job.total_rows);
      const int t = (int)(rowi - (int64_t)h * job.total_rows);
      int b = 0;
      while (b + 1 < a.n_seq && t >= job.cnt_off[b + 1]) ++b;
      const int tok = a.cu[b] + job.idx[rowi];
      const uint8_t *src = job.src + (size_t)tok * job.src_row_stride + (size_t)h * job.row_bytes;
      val[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src) + col);
      dst_off[u] = c;
    }
  }
#pragma unroll
  for (int u = 0; u < kGatherUnroll; ++u)
    if (dst_off[u] >= 0) __builtin_nontemporal_store(val[u], reinterpret_cast<u32x4 *>(job.dst) + dst_off[u]);
}

hipError_t launch_gather(const GatherArgs &a, int n_blocks, hipStream_t s) {
  if (n_blocks <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_gather, dim3(n_blocks), dim3(kGatherThreads), 0, s, a);
  return hipGetLastError();
}

}  // namespace fkv
