// Device helpers shared by the top-k kernels: order-preserving keys, the coalesced key layout,
// the histogram bin search and the ordered compaction of one 1024-thread chunk.
#pragma once

#include "fkv_dpp.h"
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

// Result of a bin search over a 2048-bin LDS histogram of the current candidates.
struct BinPick {
  uint32_t digit;      // bin that holds the `remaining`-th largest candidate
  uint32_t remaining;  // rank of the wanted key inside that bin (1 = largest)
  uint32_t in_bin;     // candidates in that bin
};

// Expects hist[0..kBins) filled and a block barrier passed; every thread gets the same result and a
// barrier is left behind.  wsum: kSelWaves words, bcast: 4 words of LDS.
// n_total: number of keys in the interval the histogram covers, or kNoDeficit.  A fill may leave out
// the keys equal to the interval's lower end (they all fall into bin 0): what is missing from the
// histogram's total is credited to bin 0 here.  Mass ties sit at the smallest key in practice (scores
// that underflowed to zero), and thousands of atomics on one LDS word would serialise.
constexpr uint32_t kNoDeficit = 0xFFFFFFFFu;
__device__ __forceinline__ BinPick pick_bin(const uint32_t *hist, uint32_t *wsum, uint32_t *bcast, uint32_t remaining,
                                            uint32_t n_total = kNoDeficit) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // thread t owns the bin pair 2*(1023-t), 2*(1023-t)+1: thread order runs from the top bin down, so
  // an inclusive prefix sum over threads counts the candidates in this pair and above it
  const int pair = kSelThreads - 1 - tid;
  uint32_t h0 = hist[2 * pair];
  const uint32_t h1 = hist[2 * pair + 1];
  uint32_t mine = h0 + h1;
  const uint32_t run = wave_scan_add(mine);
  if (lane == 63) wsum[wave] = run;
  __syncthreads();
  uint32_t above = run - mine;
  for (int w = 0; w < wave; ++w) above += wsum[w];
  if (pair == 0 && n_total != kNoDeficit) {  // the last thread in scan order sees the histogram's total
    const uint32_t deficit = n_total - (above + mine);
    h0 += deficit;
    mine += deficit;
  }
  if (above < remaining && remaining <= above + mine) {
    const bool top = remaining <= above + h1;
    bcast[0] = 2 * pair + (top ? 1 : 0);
    bcast[1] = remaining - above - (top ? 0u : h1);
    bcast[2] = top ? h1 : h0;
  }
  __syncthreads();
  BinPick p;
  p.digit = bcast[0];
  p.remaining = bcast[1];
  p.in_bin = bcast[2];
  return p;
}

// Ordered compaction of one chunk of 1024*kKpt keys held in registers: appends to `out` the
// chunk-local indices (+ i_chunk) of all keys > T and of keys == T while fewer than need_eq equal
// keys came before, in index order.  run_gt / run_eq count what earlier chunks kept / saw and are
// advanced.  scan_tbl: kSelWaves*64*kMaxKpt words, wsum: kSelWaves words, sink: 64 words of LDS.
// Index order inside a wave is (q, lane, e).  Contains block barriers.
// kCoherentOut: the indices leave as agent-scope atomic stores (straight to device memory instead of
// resting in the writing CU's L2), for kernels whose blocks order their output among themselves.
template <int kKpt, bool kCoherentOut = false>
__device__ __forceinline__ void compact_chunk(const uint32_t (&key)[kKpt], uint32_t T, uint32_t need_eq,
                                              uint32_t &run_gt, uint32_t &run_eq, int i_chunk, int32_t *out,
                                              uint32_t *scan_tbl, uint32_t *wsum, uint32_t *sink) {
  constexpr int kQ = kKpt / 4;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t cnt[kQ];   // per 4-key item: keys > T (low 16 bits), keys == T (high 16 bits)
#pragma unroll
    for (int q = 0; q < kQ; ++q) {
      uint32_t c = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) c += (key[4 * q + e] > T ? 1u : 0u) + (key[4 * q + e] == T ? 0x10000u : 0u);
      cnt[q] = c;
    }
    // Kept counts per (q, lane) item, packed (low 16 bits: keys > T, high 16 bits: keys == T; a wave holds
    // at most 2048 keys, so neither field overflows).  Index order inside the wave is item order
    // q*64 + lane: the exclusive prefix of item (q, lane) is the total of the items of all q' < q plus
    // an in-wave scan over the lanes of q, all on DPP lane routing (no LDS round trip).
    uint32_t *tbl = scan_tbl + wave * (64 * kMaxKpt);  // up to 64*kKpt staged outputs of this wave
    uint32_t pq[kQ];
    uint32_t wave_tot = 0;
#pragma unroll
    for (int q = 0; q < kQ; ++q) {
      const uint32_t inc = wave_scan_add(cnt[q]);
      pq[q] = wave_tot + inc - cnt[q];
      wave_tot += wave_last(inc);
    }
    if (lane == 0) wsum[wave] = wave_tot;  // free: every caller leaves a barrier behind its last use of wsum
    __syncthreads();
    uint32_t before_w = 0, total = 0;
    for (int w = 0; w < kSelWaves; ++w) {
      const uint32_t v = wsum[w];
      if (w < wave) before_w += v;
      total += v;
    }
    // Kept indices are first placed in the wave's LDS region (its outputs are consecutive in the
    // result because index order is kept), then written out with full 64-lane stores.
    const uint32_t gt0 = run_gt + (before_w & 0xFFFFu), eq0 = run_eq + (before_w >> 16);
    const uint32_t wave_base = gt0 + min(eq0, need_eq);
    const uint32_t wave_end = gt0 + (wave_tot & 0xFFFFu) + min(eq0 + (wave_tot >> 16), need_eq);
    int32_t *stg = reinterpret_cast<int32_t *>(tbl);
    int32_t *dummy = reinterpret_cast<int32_t *>(sink) + lane;  // sink for keys that are dropped
#pragma unroll
    for (int q = 0; q < kQ; ++q) {
      uint32_t gt_before = gt0 + (pq[q] & 0xFFFFu);
      uint32_t eq_before = eq0 + (pq[q] >> 16);
      const int i0 = i_chunk + slot_pos<kKpt>(wave, lane, q);
      if (cnt[q] == 0) continue;  // most items keep nothing
      if ((cnt[q] >> 16) == 0) {
        // no key of this item ties with T: branch-free placement
        int32_t *dst = stg + (gt_before + min(eq_before, need_eq) - wave_base);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const bool kept = key[4 * q + e] > T;
          *(kept ? dst : dummy) = i0 + e;
          dst += kept ? 1 : 0;
        }
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const uint32_t kk = key[4 * q + e];
          if (kk > T) {
            stg[gt_before + min(eq_before, need_eq) - wave_base] = i0 + e;
            ++gt_before;
          } else if (kk == T) {
            if (eq_before < need_eq) stg[gt_before + eq_before - wave_base] = i0 + e;
            ++eq_before;
          }
        }
      }
    }
    wave_sync_lds();
    for (uint32_t o = lane; o < wave_end - wave_base; o += 64) {
      if (kCoherentOut)
        __hip_atomic_store(out + wave_base + o, stg[o], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      else
        out[wave_base + o] = stg[o];
    }
    __syncthreads();  // the tables are rewritten by the next chunk
    run_gt += total & 0xFFFFu;
    run_eq += total >> 16;
}

}  // namespace fkv
