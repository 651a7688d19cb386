// Top-k of one score row with the window merged in (Sec. 4.2): exact radix select on the
// order-preserving integer image of the fp32 scores, then an ordered compaction, so the
// output is ascending, has exactly k entries and equal scores go to the lower index.
//
// One 1024-thread block per (row, sequence).  Each thread holds 8, 16 or 32 keys (by row
// length) read with coalesced 128-bit loads.  Rows of up to 32768 keys stay in registers for
// the whole kernel; longer rows are processed in 32768-key chunks re-read from L2 per pass.
//   1. the row's smallest and largest key bound the search interval [lo, lo + 2^s); histogram
//      passes of up to 11 bits of (key - lo), most significant first, narrow it down to the key
//      T of the (k-W)-th largest prefix score.  Taking digits relative to the row's own range
//      spreads the keys over the 2048 LDS bins (fp32 exponents would crowd them into a few
//      dozen) and makes a constant row cost no pass at all.  After the first pass the few keys
//      left in the interval are collected into LDS, one per thread, and the remaining passes
//      run on that list.  Keys equal to the interval's lower end are never histogrammed (a row
//      may hold thousands of them: probabilities that underflowed to zero); their count is the
//      difference between the interval's key count and the histogram's total;
//   2. a scan of the per-item keep counts (in-wave through an LDS table, across waves through
//      wave totals) gives every kept key its output offset in index order: all keys > T and
//      the first `need_eq` keys == T by index.
#include "fkv_select_common.h"

namespace fkv {

template <bool kResident, int kKpt>
__device__ __forceinline__ void select_row(const float *sc, int P, int kp, int32_t *out, uint32_t *hist,
                                           uint32_t *wsum, uint32_t *bcast, uint32_t *scan_tbl) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int mis = (int)((reinterpret_cast<uintptr_t>(sc) >> 2) & 3);
  const float *base = sc - mis;
  constexpr int kChunk = kSelThreads * kKpt;
  const int n_chunks = kResident ? 1 : (P + mis + kChunk - 1) / kChunk;
  uint32_t key[kKpt];
  FKV_TICK(0);
  FKV_BTICK(0);

  // ---- key range of the row: the radix digits are taken relative to the smallest key, so
  // the bins spread over the values the row really holds instead of over fp32's exponent
  uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
  for (int ch = 0; ch < n_chunks; ++ch) {
    load_keys<kKpt>(base, mis, P, ch * kChunk, wave, lane, key);
#pragma unroll
    for (int e = 0; e < kKpt; ++e) {
      kmax = max(kmax, key[e]);
      kmin = min(kmin, key[e] - 1u);  // key 0 (no element) wraps to the largest value
    }
  }
  kmax = wave_max_to_last(kmax);
  kmin = wave_min_to_last(kmin);
  if (lane == 63) { wsum[wave] = kmin; wsum[kSelWaves + wave] = kmax; }
  __syncthreads();
  for (int w = 0; w < kSelWaves; ++w) {
    kmin = min(kmin, wsum[w]);
    kmax = max(kmax, wsum[kSelWaves + w]);
  }
  kmin += 1u;

  FKV_TICK(1);
  FKV_BTICK(1);
  // ---- narrow [lo, lo + 2^s) down to the key T of the kp-th largest score
  uint32_t lo = kmin, remaining = (uint32_t)kp, need_eq = remaining;
  uint32_t n_in = (uint32_t)P;  // keys in the current interval [lo, lo + 2^s)
  int s = (kmax == kmin) ? 0 : 32 - __clz(kmax - kmin);  // kmax - kmin < 2^s
  bool whole_bin = false;

  // Picks the histogram bin that holds the `remaining`-th largest candidate and narrows the
  // interval to it.  Expects hist filled and a barrier passed; leaves a barrier behind.
  auto narrow = [&](int shift) {
    const BinPick p = pick_bin(hist, wsum, bcast, remaining, n_in);
    n_in = p.in_bin;
    lo += p.digit << shift;
    remaining = p.remaining;
    need_eq = remaining;
    s = shift;
    whole_bin = p.in_bin == p.remaining;  // the whole bin is kept: no need to refine further
    return p.in_bin;                      // candidates left
  };
  auto clear_hist = [&]() {
    __syncthreads();  // wsum / hist / bcast readers of the previous round are done
    for (int i = tid; i < kBins; i += kSelThreads) hist[i] = 0;
    if (tid == 0) bcast[4] = 0;  // candidate-list length
    __syncthreads();
  };

  uint32_t n_cand = 0xFFFFFFFFu;
  if (s > 0) {
    // first pass: every key of the row
    const int shift = s - min(11, s);
    clear_hist();
    for (int ch = 0; ch < n_chunks; ++ch) {
      if (!kResident) load_keys<kKpt>(base, mis, P, ch * kChunk, wave, lane, key);
      const uint32_t span = s >= 32 ? 0xFFFFFFFFu : ((1u << s) - 1u);
#pragma unroll
      for (int e = 0; e < kKpt; ++e) {
        // branch-free: what is not counted goes to a spare word per bank.  Not counted: empty slots (key 0)
        // and the keys equal to lo, whose number pick_bin recovers from the histogram's total
        const uint32_t rel = key[e] - lo;
        atomicAdd(&hist[(key[e] > lo && rel <= span) ? rel >> shift : (uint32_t)kBins + (lane & 31)], 1u);
      }
    }
    __syncthreads();
    FKV_TICK(8);
    n_cand = narrow(shift);
    FKV_TICK(9);
  }
  if (s > 0 && !whole_bin && n_cand <= (uint32_t)kSelThreads) {
    // Few keys are left in the interval (typically ~1 %): collect them into LDS, one per thread, and
    // finish the search on that list instead of sweeping all register keys again.
    uint32_t *cand = scan_tbl;  // free until the compaction
    const uint32_t span = (1u << s) - 1u;  // s <= 21 here
    for (int ch = 0; ch < n_chunks; ++ch) {
      if (!kResident) load_keys<kKpt>(base, mis, P, ch * kChunk, wave, lane, key);
      // Valid keys lie in [0x007FFFFF, 0xFF800000] and span < 2^21, so a key below lo (or an empty
      // slot) wraps above span: one unsigned compare per key.  A wave reserves list space for all its
      // candidates with one LDS atomic (a scan over the lanes' counts gives each lane its place).
      uint32_t mine = 0;
#pragma unroll
      for (int e = 0; e < kKpt; ++e) mine += (key[e] - lo <= span) ? 1u : 0u;
      const uint32_t inc = wave_scan_add(mine);
      const uint32_t wave_n = wave_last(inc);
      if (wave_n == 0) continue;
      uint32_t wave_base = 0;
      if (lane == 63) wave_base = atomicAdd(&bcast[4], wave_n);
      wave_base = wave_last(wave_base);
      if (mine != 0) {
        uint32_t at = wave_base + inc - mine;
#pragma unroll
        for (int e = 0; e < kKpt; ++e) {
          const uint32_t rel = key[e] - lo;
          if (rel <= span) cand[at++] = rel;
        }
      }
    }
    __syncthreads();
    FKV_TICK(10);
    const uint32_t my_rel = (uint32_t)tid < n_cand ? cand[tid] : 0xFFFFFFFFu;
    uint32_t base_rel = 0;  // lo advanced since the list was built
    while (s > 0 && !whole_bin) {
      const int shift = s - min(11, s);
      const uint32_t span2 = (1u << s) - 1u;
      clear_hist();
      const uint32_t rel = my_rel - base_rel;
      if (my_rel >= base_rel && rel <= span2) atomicAdd(&hist[rel >> shift], 1u);
      __syncthreads();
      const uint32_t lo_before = lo;
      narrow(shift);
      base_rel += lo - lo_before;
    }
  } else {
    while (s > 0 && !whole_bin) {
      const int shift = s - min(11, s);
      const uint32_t span = (s >= 32) ? 0xFFFFFFFFu : ((1u << s) - 1u);  // candidates: key - lo <= span
      clear_hist();
      for (int ch = 0; ch < n_chunks; ++ch) {
        if (!kResident) load_keys<kKpt>(base, mis, P, ch * kChunk, wave, lane, key);
#pragma unroll
        for (int e = 0; e < kKpt; ++e) {  // keys equal to lo are left to pick_bin's total, as in the first pass
          const uint32_t rel = key[e] - lo;
          atomicAdd(&hist[(key[e] > lo && rel <= span) ? rel >> shift : (uint32_t)kBins + (lane & 31)], 1u);
        }
      }
      __syncthreads();
      narrow(shift);
    }
  }
  if (whole_bin) need_eq = 0xFFFFFFFFu;
  __syncthreads();  // the candidate list (scan table) is free again
  // keep key > T, and key == T while fewer than need_eq equal keys came before it.  When a whole
  // bin is kept, T is the smallest key the bin could hold and every key == T is kept.
  const uint32_t T = lo;
  FKV_TICK(2);
  FKV_BTICK(2);

  // ---- ordered compaction.  Index order inside a wave is (q, lane, e).
  uint32_t run_gt = 0, run_eq = 0;
  for (int ch = 0; ch < n_chunks; ++ch) {
    if (!kResident) load_keys<kKpt>(base, mis, P, ch * kChunk, wave, lane, key);
    compact_chunk<kKpt>(key, T, need_eq, run_gt, run_eq, ch * kChunk - mis, out, scan_tbl, wsum, bcast + 8);
  }
  FKV_TICK(3);
  FKV_BTICK(3);
}

__global__ __launch_bounds__(kSelThreads) void k_select(SelectArgs a) {
  __shared__ uint32_t hist[kBins + 32];  // + spare words for key slots that are not counted (never read; one
                                         // per bank, so they do not pile onto one address)
  __shared__ __attribute__((aligned(16))) uint32_t scan_tbl[kSelWaves * 64 * kMaxKpt];  // 128 KiB: scan tables / output staging
  __shared__ uint32_t wsum[2 * kSelWaves];
  __shared__ uint32_t bcast[8 + 64];  // broadcast slots, then one sink word per lane

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

  if (a.long_state != nullptr && P + 3 > kSelThreads * kMaxKpt) return;  // taken by the multi-block chain
  if (a.err != nullptr && *a.err != 0u) {  // the scores are invalid: no index may look usable
    for (int i = threadIdx.x; i < k; i += kSelThreads) out[i] = -1;
    return;
  }
  if ((int)threadIdx.x < a.W) out[kp + threadIdx.x] = P + threadIdx.x;  // window tokens are always kept
  if (kp <= 0) return;
  if (P + 3 <= kSelThreads * 8)
    select_row<true, 8>(sc, P, kp, out, hist, wsum, bcast, scan_tbl);
  else if (P + 3 <= kSelThreads * 16)
    select_row<true, 16>(sc, P, kp, out, hist, wsum, bcast, scan_tbl);
  else if (P + 3 <= kSelThreads * 32)
    select_row<true, 32>(sc, P, kp, out, hist, wsum, bcast, scan_tbl);
  else
    select_row<false, 32>(sc, P, kp, out, hist, wsum, bcast, scan_tbl);
}

hipError_t launch_select(SelectArgs a, uint32_t *long_state, const SelectCoop *coop, hipStream_t s) {
  int rows = 0;
  for (int i = 0; i < a.n_sets; ++i) rows += a.set[i].n_rows;
  {
    hipError_t e = hipSuccess;
    a.long_state = nullptr;
    if (coop != nullptr && try_launch_select_coop(a, rows, *coop, s, &e)) return e;
  }
  // Rows over one chunk go to the multi-block chain when the call's row instances fit its state.
  int max_slices = 0;
  bool any_short = false;
  for (int b = 0; b < a.n_seq; ++b) {
    const int P = a.cu[b + 1] - a.cu[b] - a.W;
    if (P + 3 > select_long_threshold())
      max_slices = max(max_slices, (P + 3 + select_long_chunk() - 1) / select_long_chunk());
    else
      any_short = true;
  }
  const bool use_long = long_state != nullptr && max_slices > 0 && max_slices <= kLongMaxSlices &&
                        (int64_t)rows * a.n_seq <= kLongMaxInst;
  a.long_state = use_long ? long_state : nullptr;
  hipError_t e = hipSuccess;
  if (!use_long || any_short) {
    hipLaunchKernelGGL(k_select, dim3(rows, a.n_seq), dim3(kSelThreads), 0, s, a);
    e = hipGetLastError();
  }
  if (e == hipSuccess && use_long) e = launch_select_long(a, rows, max_slices, s);
  return e;
}

}  // namespace fkv
