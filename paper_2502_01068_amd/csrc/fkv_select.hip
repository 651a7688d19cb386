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
//      dozen) and makes a constant row cost no pass at all;
//   2. a scan of the per-item keep counts (in-wave through an LDS table, across waves through
//      wave totals) gives every kept key its output offset in index order: all keys > T and
//      the first `need_eq` keys == T by index.
#include "fkv_internal.h"

namespace fkv {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kMaxKpt = 32;                       // keys per thread per chunk (8, 16 or 32)
constexpr int kBins = 2048;

// Monotone map fp32 -> uint32 (larger float <=> larger key), valid for any non-NaN input;
// -0.0 and +0.0 compare equal as floats, so both get the key of +0.0.  No valid key is 0.
__device__ __forceinline__ uint32_t order_key(float f) {
  uint32_t u = __float_as_uint(f);
  if (u == 0x80000000u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Key layout of a chunk of 1024*kKpt keys (kKpt keys per thread): wave w owns virtual positions
// [64 kKpt w, 64 kKpt (w+1)); its q-th 128-bit load covers positions 64 kKpt w + 256 q + 4 lane
// + {0..3}, so every load instruction reads 1 KiB of consecutive memory.  Position v holds
// score v - mis (`base` = row pointer - mis is 16-byte aligned); positions outside
// [mis, mis+P) get key 0.  Short rows use fewer keys per thread: the kernel is bound by the
// instructions it spends per key slot.
template <int kKpt>
__device__ __forceinline__ int slot_pos(int wave, int lane, int q) { return wave * (64 * kKpt) + q * 256 + lane * 4; }

template <int kKpt>
__device__ __forceinline__ void load_keys(const float *base, int mis, int P, int v_chunk, int wave, int lane,
                                          uint32_t (&key)[kKpt]) {
  typedef float f32x4 __attribute__((ext_vector_type(4)));
#pragma unroll
  for (int q = 0; q < kKpt / 4; ++q) {
    const int v = v_chunk + slot_pos<kKpt>(wave, lane, q);
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

__device__ __forceinline__ void wave_sync_lds() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <bool kResident, int kKpt>
__device__ __forceinline__ void select_row(const float *sc, int P, int kp, int32_t *out, uint32_t *hist,
                                           uint32_t *wsum, uint32_t *bcast, uint32_t *scan_tbl) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int mis = (int)((reinterpret_cast<uintptr_t>(sc) >> 2) & 3);
  const float *base = sc - mis;
  constexpr int kChunk = kSelThreads * kKpt;
  constexpr int kQ = kKpt / 4;  // 128-bit loads (scan items) per thread
  const int n_chunks = kResident ? 1 : (P + mis + kChunk - 1) / kChunk;
  uint32_t key[kKpt];
  FKV_TICK(0);

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
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, off));
    kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, off));
  }
  if (lane == 0) { wsum[wave] = kmin; wsum[kSelWaves + wave] = kmax; }
  __syncthreads();
  for (int w = 0; w < kSelWaves; ++w) {
    kmin = min(kmin, wsum[w]);
    kmax = max(kmax, wsum[kSelWaves + w]);
  }
  kmin += 1u;

  FKV_TICK(1);
  // ---- narrow [lo, lo + 2^s) down to the key T of the kp-th largest score
  uint32_t lo = kmin, remaining = (uint32_t)kp, need_eq = remaining;
  int s = (kmax == kmin) ? 0 : 32 - __clz(kmax - kmin);  // kmax - kmin < 2^s
  while (s > 0) {
    const int bits = min(11, s);
    const int shift = s - bits;
    const uint32_t span = (s >= 32) ? 0xFFFFFFFFu : ((1u << s) - 1u);  // candidates: key - lo <= span
    __syncthreads();  // wsum / hist / bcast readers of the previous round are done
    for (int i = tid; i < kBins; i += kSelThreads) hist[i] = 0;
    __syncthreads();
    for (int ch = 0; ch < n_chunks; ++ch) {
      if (!kResident) load_keys<kKpt>(base, mis, P, ch * kChunk, wave, lane, key);
#pragma unroll
      for (int e = 0; e < kKpt; ++e) {
        const uint32_t rel = key[e] - lo;  // keys below lo (and key 0) wrap far above span
        if (key[e] >= lo && rel <= span) atomicAdd(&hist[rel >> shift], 1u);
      }
    }
    __syncthreads();
    FKV_TICK(8 + 2 * (s > 22 ? 0 : (s > 11 ? 1 : 2)));
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
      bcast[0] = lo + (digit << shift);
      bcast[1] = rem;
      bcast[2] = (in_bin == rem) ? 1u : 0u;  // the whole bin is kept: no need to refine further
    }
    __syncthreads();
    lo = bcast[0];
    remaining = bcast[1];
    need_eq = remaining;
    s = shift;
    if (bcast[2]) { need_eq = 0xFFFFFFFFu; break; }
  }
  // keep key > T, and key == T while fewer than need_eq equal keys came before it.  When a whole
  // bin is kept, T is the smallest key the bin could hold and every key == T is kept.
  const uint32_t T = lo;
  FKV_TICK(2);

  // ---- ordered compaction.  Index order inside a wave is (q, lane, e).
  uint32_t run_gt = 0, run_eq = 0;
  for (int ch = 0; ch < n_chunks; ++ch) {
    if (!kResident) load_keys<kKpt>(base, mis, P, ch * kChunk, wave, lane, key);
    uint32_t gt_mask = 0, eq_mask = 0;
#pragma unroll
    for (int e = 0; e < kKpt; ++e) {
      gt_mask |= (key[e] > T) ? (1u << e) : 0u;
      eq_mask |= (key[e] == T) ? (1u << e) : 0u;
    }
    // Kept counts per (q, lane) item, packed (low 16 bits: keys > T, high 16 bits: keys == T).
    // Index order inside the wave is item order q*64 + lane; lane l scans items 8l .. 8l+7 from a
    // wave-private LDS table, the 64 lanes scan their sums, and the table is overwritten with the
    // exclusive prefix of every item.
    uint32_t *tbl = scan_tbl + wave * (64 * kQ);
#pragma unroll
    for (int q = 0; q < kQ; ++q)
      tbl[q * 64 + lane] = (uint32_t)__popc((gt_mask >> (4 * q)) & 15u) | ((uint32_t)__popc((eq_mask >> (4 * q)) & 15u) << 16);
    wave_sync_lds();
    uint32_t item[kQ];
#pragma unroll
    for (int i = 0; i < kQ; ++i) item[i] = tbl[kQ * lane + i];
    uint32_t mine = 0;
#pragma unroll
    for (int i = 0; i < kQ; ++i) mine += item[i];
    uint32_t inc = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const uint32_t v = (uint32_t)__shfl_up((int)inc, off);
      if (lane >= off) inc += v;
    }
    const uint32_t wave_tot = (uint32_t)__shfl((int)inc, 63);
    uint32_t pre = inc - mine;
    wave_sync_lds();
#pragma unroll
    for (int i = 0; i < kQ; ++i) {
      tbl[kQ * lane + i] = pre;
      pre += item[i];
    }
    __syncthreads();  // wsum is free (previous readers are past their loop); tables are complete
    if (lane == 0) wsum[wave] = wave_tot;
    __syncthreads();
    uint32_t before_w = 0, total = 0;
    for (int w = 0; w < kSelWaves; ++w) {
      const uint32_t v = wsum[w];
      if (w < wave) before_w += v;
      total += v;
    }
    const uint32_t gt0 = run_gt + (before_w & 0xFFFFu), eq0 = run_eq + (before_w >> 16);
    const int i_chunk = ch * kChunk - mis;
#pragma unroll
    for (int q = 0; q < kQ; ++q) {
      const uint32_t gq = (gt_mask >> (4 * q)) & 15u, eqq = (eq_mask >> (4 * q)) & 15u;
      if (gq | eqq) {
        const uint32_t pq = tbl[q * 64 + lane];
        uint32_t gt_before = gt0 + (pq & 0xFFFFu);
        uint32_t eq_before = eq0 + (pq >> 16);
        const int i0 = i_chunk + slot_pos<kKpt>(wave, lane, q);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if ((gq >> e) & 1u) {
            out[gt_before + min(eq_before, need_eq)] = i0 + e;
            ++gt_before;
          } else if ((eqq >> e) & 1u) {
            if (eq_before < need_eq) out[gt_before + eq_before] = i0 + e;
            ++eq_before;
          }
        }
      }
    }
    __syncthreads();  // the tables are rewritten by the next chunk
    run_gt += total & 0xFFFFu;
    run_eq += total >> 16;
  }
  FKV_TICK(3);
}

__global__ __launch_bounds__(kSelThreads) void k_select(SelectArgs a) {
  __shared__ uint32_t hist[kBins];
  __shared__ __attribute__((aligned(16))) uint32_t scan_tbl[kSelWaves * 64 * (kMaxKpt / 4)];
  __shared__ uint32_t wsum[2 * kSelWaves];
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
  if (P + 3 <= kSelThreads * 8)
    select_row<true, 8>(sc, P, kp, out, hist, wsum, bcast, scan_tbl);
  else if (P + 3 <= kSelThreads * 16)
    select_row<true, 16>(sc, P, kp, out, hist, wsum, bcast, scan_tbl);
  else if (P + 3 <= kSelThreads * 32)
    select_row<true, 32>(sc, P, kp, out, hist, wsum, bcast, scan_tbl);
  else
    select_row<false, 32>(sc, P, kp, out, hist, wsum, bcast, scan_tbl);
}

hipError_t launch_select(const SelectArgs &a, hipStream_t s) {
  int rows = 0;
  for (int i = 0; i < a.n_sets; ++i) rows += a.set[i].n_rows;
  hipLaunchKernelGGL(k_select, dim3(rows, a.n_seq), dim3(kSelThreads), 0, s, a);
  return hipGetLastError();
}

}  // namespace fkv
