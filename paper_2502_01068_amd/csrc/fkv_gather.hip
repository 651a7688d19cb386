// Index-driven row gathers (HiddenCompress / KVCompress, App. B.1): bit-exact copies of the
// kept rows into compacted buffers.  Up to three jobs (hidden rows, K rows, V rows) share one
// launch so the small K/V jobs fill the machine alongside the large hidden-row job.
//
// The unit of work is one 16-byte chunk; consecutive lanes take consecutive chunks of a row,
// so a 256-byte K/V head row is one 16-lane segment and an 8 KiB hidden row is 512 lanes.
// Each (job, head) owns a contiguous range of blocks, so the head and job lookups are scalar.
#include "fkv_internal.h"

namespace fkv {

constexpr int kGatherThreads = 256;
constexpr int kGatherUnroll = 2;  // 16-byte chunks in flight per thread

int gather_blocks_per_head(const GatherJob &j) {
  const int64_t chunks = (int64_t)j.total_rows * (j.row_bytes / 16);
  const int64_t per_block = (int64_t)kGatherThreads * kGatherUnroll;
  return (int)((chunks + per_block - 1) / per_block);
}

__global__ __launch_bounds__(kGatherThreads) void k_gather(GatherArgs a) {
  int ji = 0;
  while (ji + 1 < a.n_jobs && (int)blockIdx.x >= a.job[ji + 1].blk0) ++ji;
  const GatherJob &job = a.job[ji];
  const uint32_t rel = blockIdx.x - job.blk0;
  const uint32_t h = rel / (uint32_t)job.blocks_per_head;  // uniform: scalar division
  const uint32_t hb = rel - h * job.blocks_per_head;
  const uint32_t cpr = (uint32_t)job.row_bytes >> 4;       // chunks per row
  const uint32_t n_chunks = (uint32_t)job.total_rows * cpr; // per head; host guarantees < 2^31
  const uint32_t c0 = hb * (kGatherUnroll * kGatherThreads) + threadIdx.x;
  const int32_t *idx = job.idx + (size_t)h * job.total_rows;
  const uint8_t *src_h = job.src + (size_t)(h / (uint32_t)job.head_div) * job.row_bytes;
  u32x4 *dst_h = reinterpret_cast<u32x4 *>(job.dst + (size_t)h * job.total_rows * job.row_bytes);

  u32x4 val[kGatherUnroll];
  bool live[kGatherUnroll];
#pragma unroll
  for (int u = 0; u < kGatherUnroll; ++u) {
    const uint32_t c = c0 + u * kGatherThreads;
    live[u] = c < n_chunks;
    if (live[u]) {
      uint32_t t, col;
      if (job.cpr_shift >= 0) { t = c >> job.cpr_shift; col = c & (cpr - 1u); }
      else { t = c / cpr; col = c - t * cpr; }
      int b = 0;
      while (b + 1 < a.n_seq && (int)t >= job.cnt_off[b + 1]) ++b;
      // an index beyond its sequence is clamped into it: a wrong row, never an out-of-bounds read;
      // a negative index (the mark of an invalid selection) copies nothing
      const int raw = idx[t];
      live[u] = raw >= 0;
      const int local = min(max(raw, 0), a.cu[b + 1] - a.cu[b] - 1);
      const size_t tok = (size_t)a.cu[b] + (size_t)local;
      // rows are read once and written once: non-temporal both ways (plain stores leave the L2 dirty and
      // measurably slow the next score launch)
      val[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src_h + tok * job.src_row_stride) + col);
    }
  }
#pragma unroll
  for (int u = 0; u < kGatherUnroll; ++u)
    if (live[u]) __builtin_nontemporal_store(val[u], dst_h + (c0 + u * kGatherThreads));
}

// Paged destination: chunk c of the launch is 16 bytes of (kept slot t, KV head g), heads fastest,
// so the 16*Hkv lanes of one slot write one contiguous [Hkv][d] page entry.  blockIdx.y picks K or V.
// A block-table entry outside [0, n_pages) writes nothing.
__global__ __launch_bounds__(kGatherThreads) void k_gather_paged(PagedGatherArgs a) {
  const int which = blockIdx.y;
  const uint8_t *src = a.src[which];
  uint8_t *pages = a.pages[which];
  constexpr uint32_t kCpr = kHeadDim * 2 / 16;  // 16 chunks per head row
  const uint32_t n_chunks = (uint32_t)a.total_rows * a.Hkv * kCpr;
  const uint32_t c0 = blockIdx.x * (kGatherUnroll * kGatherThreads) + threadIdx.x;
  u32x4 val[kGatherUnroll];
  u32x4 *dst[kGatherUnroll];
#pragma unroll
  for (int u = 0; u < kGatherUnroll; ++u) {
    const uint32_t c = c0 + u * kGatherThreads;
    dst[u] = nullptr;
    if (c < n_chunks) {
      const uint32_t col = c & (kCpr - 1u), r = c / kCpr;
      const uint32_t t = r / (uint32_t)a.Hkv, g = r - t * a.Hkv;
      int b = 0;
      while (b + 1 < a.n_seq && (int)t >= a.cnt_off[b + 1]) ++b;
      const uint32_t tl = t - a.cnt_off[b];
      const int page = a.block_table[(size_t)b * a.max_pages + (tl >> a.page_shift)];
      const int raw = a.idx[(size_t)g * a.total_rows + t];
      const int local = min(max(raw, 0), a.cu[b + 1] - a.cu[b] - 1);
      const size_t tok = (size_t)a.cu[b] + (size_t)local;
      val[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src + (tok * a.Hkv + g) * (kHeadDim * 2)) + col);
      if (raw >= 0 && page >= 0 && page < a.n_pages) {
        const size_t slot = ((size_t)page << a.page_shift) + (tl & ((1u << a.page_shift) - 1u));
        dst[u] = reinterpret_cast<u32x4 *>(pages + (slot * a.Hkv + g) * (kHeadDim * 2)) + col;
      }
    }
  }
#pragma unroll
  for (int u = 0; u < kGatherUnroll; ++u)
    if (dst[u]) __builtin_nontemporal_store(val[u], dst[u]);
}

hipError_t launch_gather_paged(const PagedGatherArgs &a, hipStream_t s) {
  const int64_t chunks = (int64_t)a.total_rows * a.Hkv * (kHeadDim * 2 / 16);
  const int64_t per_block = (int64_t)kGatherThreads * kGatherUnroll;
  const int n_blocks = (int)((chunks + per_block - 1) / per_block);
  if (n_blocks <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_gather_paged, dim3(n_blocks, a.src[1] ? 2 : 1), dim3(kGatherThreads), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_gather(const GatherArgs &a, int n_blocks, hipStream_t s) {
  if (n_blocks <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_gather, dim3(n_blocks), dim3(kGatherThreads), 0, s, a);
  return hipGetLastError();
}

}  // namespace fkv
