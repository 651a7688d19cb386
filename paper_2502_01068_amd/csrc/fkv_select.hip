// Top-k of one score row with the window merged in (Sec. 4.2): exact radix select on the
// order-preserving integer image of the fp32 scores, then an ordered compaction, so the
// output is ascending, has exactly k entries and equal scores go to the lower index.
//
// One 1024-thread block per (row, sequence).  Thread t owns 32 consecutive keys of each
// 32768-key chunk ("blocked" layout), read with 128-bit loads.  Rows of up to one chunk stay
// in registers for the whole kernel; longer rows are re-read from L2 per pass.
//   1. three histogram passes (11 + 11 + 10 bits, most significant first) over an LDS
//      histogram narrow down the key T of the (k-W)-th largest prefix score; runs of equal
//      digits inside a thread are merged before the LDS atomic (pooled scores are smooth, so
//      neighbours mostly share a digit);
//   2. one block-wide exclusive scan of the per-thread keep counts gives every thread its
//      output offset; it then writes its kept indices in order: all keys > T and the first
//      `need_eq` keys == T by index.
#include "fkv_internal.h"

namespace fkv {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kKpt = 32;                          // keys per thread per chunk
constexpr int kChunk = kSelThreads * kKpt;        // 32768
constexpr int kBins = 2048;

// Monotone map fp32 -> uint32 (larger float <=> larger key), valid for any non-NaN input;
// -0.0 and +0.0 compare equal as floats, so both get the key of +0.0.  No valid key is 0.
__device__ __forceinline__ uint32_t order_key(float f) {
  uint32_t u = __float_as_uint(f);
  if (u == 0x80000000u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Keys of virtual positions v0 .. v0+31 of the row, where position v holds score v - mis
// (`base` = row pointer - mis is 16-byte aligned).  Positions outside [mis, mis+P) get key 0.
__device__ __forceinline__ void load_keys(const float *base, int mis, int P, int v0, uint32_t (&key)[kKpt]) {
  typedef float f32x4 __attribute__((ext_vector_type(4)));
#pragma unroll
  for (int q = 0; q < kKpt / 4; ++q) {
    const int v = v0 + 4 * q;
    if (v >= mis && v + 3 < mis + P) {
      const f32x4 f = *reinterpret_cast<const f32x4 *>(base + v);
      key[4 * q + 0] = order_key(f[0]);
      key[4 * q + 1] = order_key(f[1]);
      key[4 * q + 2] = order_key(f[2]);
      key[4 * q + 3] = order_key(f[3]);
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int vv = v + e;
        key[4 * q + e] = (vv >= mis && vv < mis + P) ? order_key(base[vv]) : 0u;
      }
    }
  }
}

template <bool kResident>
__device__ __forceinline__ void select_row(const float *sc, int P, int kp, int W, int32_t *out, uint32_t *hist,
                                           uint32_t *wsum, uint32_t *bcast) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int mis = (int)((reinterpret_cast<uintptr_t>(sc) >> 2) & 3);
  const float *base = sc - mis;
  const int n_chunks = kResident ? 1 : (P + mis + kChunk - 1) / kChunk;
  uint32_t key[kKpt];
  if (kResident) load_keys(base, mis, P, tid * kKpt, key);

  uint32_t prefix = 0, mask = 0, remaining = (uint32_t)kp;
  uint32_t need_eq = 0;
  bool done = false;
  for (int pass = 0; pass < 3 && !done; ++pass) {
    const int shift = pass == 0 ? 21 : (pass == 1 ? 10 : 0);
    const uint32_t nb = pass == 2 ? 1024u : 2048u;
    for (int i = tid; i < kBins; i += kSelThreads) hist[i] = 0;
    __syncthreads();
    for (int ch = 0; ch < n_chunks; ++ch) {
      if (!kResident) load_keys(base, mis, P, ch * kChunk + tid * kKpt, key);
      uint32_t cur = 0, cnt = 0;
#pragma unroll
      for (int e = 0; e < kKpt; ++e) {
        const uint32_t kk = key[e];
        if (kk != 0u && (kk & mask) == prefix) {
          const uint32_t bin = (kk >> shift) & (nb - 1u);
          if (bin != cur && cnt) { atomicAdd(&hist[cur], cnt); cnt = 0; }
          cur = bin;
          ++cnt;
        }
      }
      if (cnt) atomicAdd(&hist[cur], cnt);
    }
    __syncthreads();
    // thread owns bins 2*tid, 2*tid+1; suffix sums from the top bin down
    const uint32_t h0 = hist[2 * tid], h1 = hist[2 * tid + 1];
    const uint32_t mine = h0 + h1;
    uint32_t run = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const uint32_t v = __shfl_down(run, off);
      if (lane + off < 64) run += v;
    }
    if (lane == 0) wsum[wave] = run;
    __syncthreads();
    uint32_t above = run - mine;
    for (int w = wave + 1; w < kSelWaves; ++w) above += wsum[w];
    if (above < remaining && remaining <= above + mine) {
      const bool top = remaining <= above + h1;
      const uint32_t digit = 2 * tid + (top ? 1 : 0);
      const uint32_t in_bin = top ? h1 : h0;
      const uint32_t rem = remaining - above - (top ? 0u : h1);
      bcast[0] = prefix | (digit << shift);
      bcast[1] = rem;
      bcast[2] = (in_bin == rem) ? 1u : 0u;  // the whole bin is kept: no need to refine further
    }
    __syncthreads();
    prefix = bcast[0];
    remaining = bcast[1];
    mask |= (nb - 1u) << shift;
    if (bcast[2]) { done = true; need_eq = 0xFFFFFFFFu; } else need_eq = remaining;
    // (bcast is rewritten only after the next pass's two barriers)
  }
  // keep key > T, and key == T while fewer than need_eq equal keys came before it.  When a whole
  // bin is kept, T is the smallest key the bin could hold and every key == T is kept.
  const uint32_t T = prefix;

  uint32_t run_gt = 0, run_eq = 0;
  for (int ch = 0; ch < n_chunks; ++ch) {
    if (!kResident) load_keys(base, mis, P, ch * kChunk + tid * kKpt, key);
    uint32_t cg = 0, ce = 0;
#pragma unroll
    for (int e = 0; e < kKpt; ++e) {
      cg += (key[e] > T) ? 1u : 0u;
      ce += (key[e] == T) ? 1u : 0u;
    }
    // block-wide exclusive scan of (cg, ce); both fit 16 bits within a chunk
    const uint32_t packed = cg | (ce << 16);
    uint32_t inc = packed;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const uint32_t v = __shfl_up(inc, off);
      if (lane >= off) inc += v;
    }
    __syncthreads();  // wsum is free (previous readers are past their loop)
    if (lane == 63) wsum[wave] = inc;
    __syncthreads();
    uint32_t before = inc - packed, total = 0;
    for (int w = 0; w < kSelWaves; ++w) {
      const uint32_t v = wsum[w];
      if (w < wave) before += v;
      total += v;
    }
    uint32_t gt_before = run_gt + (before & 0xFFFFu);
    uint32_t eq_before = run_eq + (before >> 16);
    const int i0 = ch * kChunk + tid * kKpt - mis;
    if (cg | ce) {
#pragma unroll
      for (int e = 0; e < kKpt; ++e) {
        const uint32_t kk = key[e];
        if (kk > T) {
          out[gt_before + min(eq_before, need_eq)] = i0 + e;
          ++gt_before;
        } else if (kk == T) {
          if (eq_before < need_eq) out[gt_before + eq_before] = i0 + e;
          ++eq_before;
        }
      }
    }
    run_gt += total & 0xFFFFu;
    run_eq += total >> 16;
  }
  (void)W;
}

__global__ __launch_bounds__(kSelThreads) void k_select(SelectArgs a) {
  __shared__ uint32_t hist[kBins];
  __shared__ uint32_t wsum[kSelWaves];
  __shared__ uint32_t bcast[4];

  int row = blockIdx.x;
  const int set_id = (a.n_sets > 1 && row >= a.set[0].n_rows) ? 1 : 0;
  if (set_id) row -= a.set[0].n_rows;
  const SelectRowSet &rs = a.set[set_id];
  const int b = blockIdx.y;
  const int Lb = a.cu[b + 1] - a.cu[b];
  const int P = Lb - a.W;
  const int k = rs.cnt_off[b + 1] - rs.cnt_off[b];
  const int kp = k - a.W;  // prefix tokens to keep
  const float *sc = rs.scores + (size_t)row * rs.row_stride + (a.cu[b] - b * a.W);
  int32_t *out = rs.idx_out + (size_t)row * rs.cnt_off[a.n_seq] + rs.cnt_off[b];

  if ((int)threadIdx.x < a.W) out[kp + threadIdx.x] = P + threadIdx.x;  // window tokens are always kept
  if (kp <= 0) return;
  if (P + 3 <= kChunk)
    select_row<true>(sc, P, kp, a.W, out, hist, wsum, bcast);
  else
    select_row<false>(sc, P, kp, a.W, out, hist, wsum, bcast);
}

hipError_t launch_select(const SelectArgs &a, hipStream_t s) {
  int rows = 0;
  for (int i = 0; i < a.n_sets; ++i) rows += a.set[i].n_rows;
  hipLaunchKernelGGL(k_select, dim3(rows, a.n_seq), dim3(kSelThreads), 0, s, a);
  return hipGetLastError();
}

}  // namespace fkv
