// Top-k of long score rows with several blocks per row (Sec. 4.2: the same exact selection as
// fkv_select.hip, window merged in, output ascending, equal scores to the lower index).
//
// A row is cut into at most 8 slices of 8192, 16384 or 32768 keys (by row length), one block each; the
// blocks of a row agree on the threshold key through tagged mailbox words (fkv_mailbox.h), all of them
// resident at once.  Every step is the one-block kernel's, with an exchange where that kernel has a
// block-wide reduction:
//   range     every block posts its slice's smallest and largest key and reads the others': the radix
//             digits are taken relative to the row's smallest key
//   rounds    every block histograms its slice's keys of the current interval (2048 bins), posts the
//             histogram and reads the other slices'.  Every block then knows, identically, the bin that
//             holds the (k-W)-th largest score, how many keys of each slice fall into it and how many
//             keys of the slices before its own lie above it
//   list      once the interval holds at most 1024 keys (after one round, usually) every block posts
//             its keys of the interval, all blocks read the whole list and finish the search on it,
//             each for itself and with the same result
//   compact   with the threshold and the per-slice counts every block knows where its kept indices
//             start in the output and writes them in index order.
// Three exchanges in the usual case, 2-4 us each (a post and a poll are one trip through device memory
// each, and a poll that comes too early costs another), against one launch per step (5 us each) in the
// launch chain this kernel replaces where the rows fit.  Histogram region 0 of the mailboxes is unused
// (rounds count from 1).
//
// Every wait is bounded.  A block that gives up raises the context's error flag and marks the launch
// as failed; the block that finishes last then overwrites every index of the launch with -1.  So
// that this overwrite is ordered after the other blocks' indices, all indices leave as agent-scope
// stores and each block waits for their acknowledgement before it counts itself as finished.
#include "fkv_mailbox.h"
#include "fkv_select_common.h"

namespace fkv {

constexpr int kCoopCandCap = kSelThreads;  // longest list the blocks exchange (one key per thread)

// mailbox regions of a block, in words
constexpr int kCoopList = kCoopHistRounds * kSelThreads;  // keys of the agreed interval
constexpr int kCoopHeader = kCoopList + kSelThreads;      // (smallest key - 1, largest key) of the slice
static_assert(kCoopHeader + 2 <= kCoopWords, "mailbox regions");

__host__ __device__ inline int coop_slices(int P, int chunk) { return P + 3 <= chunk ? 1 : (P + 3 + chunk - 1) / chunk; }

// kKpt: keys per thread; kSl: most slices a row of the launch has (sizes the unrolled exchange code)
template <int kKpt, int kSl>
__global__ __launch_bounds__(kSelThreads) void k_select_coop(SelectArgs a, CoopArgs c) {
  constexpr int kChunk = kSelThreads * kKpt;  // keys per block
  __shared__ uint32_t hist[kBins + 32];  // + one spare word per bank for key slots that are not counted
  __shared__ __attribute__((aligned(16))) uint32_t scan_tbl[kSelWaves * 64 * kMaxKpt];  // 128 KiB: peers' histogram words [slice][thread], then scan tables / output staging
  __shared__ uint32_t wsum[2 * kSelWaves];
  __shared__ uint32_t bcast[8 + 64];
  __shared__ uint32_t slice_cnt[kCoopMaxSlices];  // keys of each slice inside the current interval
  __shared__ uint32_t hdr[2 * kCoopMaxSlices];    // (smallest key - 1, largest key) of each slice
  __shared__ uint32_t misc[8];  // 0 keys counted into the histogram, 1 kept / 2 tied list keys of earlier slices,
                                // 3 a wave gave up, 4 outcome of the finish count, 5 list length of this slice
  static_assert(kCoopMaxSlices * kSelThreads <= kSelWaves * 64 * kMaxKpt, "peer staging fits the scan table");

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  FKV_TICK(6);
  int b = 0;
  while (b + 1 < a.n_seq && (int)blockIdx.x >= c.blk[b + 1]) ++b;
  const int P = a.cu[b + 1] - a.cu[b] - a.W;
  const int M = coop_slices(P, kChunk);
  const int local = (int)blockIdx.x - c.blk[b];
  int row = local / M;
  const int s = local - row * M;          // this block's slice
  const int blk0 = (int)blockIdx.x - s;   // block of the row's slice 0
  const int set_id = (a.n_sets > 1 && row >= a.set[0].n_rows) ? 1 : 0;
  if (set_id) row -= a.set[0].n_rows;
  const SelectRowSet &rs = a.set[set_id];
  const int k = rs.cnt_off[b + 1] - rs.cnt_off[b];
  const int kp = k - a.W;  // prefix tokens to keep
  const float *sc = rs.scores + (size_t)row * rs.row_stride + (a.cu[b] - b * a.W);
  int32_t *out = rs.idx_out + (size_t)row * rs.cnt_off[a.n_seq] + rs.cnt_off[b];
  const int mis = (int)((reinterpret_cast<uintptr_t>(sc) >> 2) & 3);
  const int v0 = s * kChunk;
  // the keys, the epoch and the flag are on their way while the tables are cleared
  // (in the order they are needed: loads return in order, the epoch comes from device memory)
  const unsigned poisoned = a.err != nullptr ? *a.err : 0u;
  uint32_t key[kKpt];
  load_keys<kKpt>(sc - mis, mis, P, v0, wave, lane, key);
  const unsigned epoch = __hip_atomic_load(c.state + 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  unsigned long long *const my_box = c.boxes + (size_t)blockIdx.x * kCoopWords;
  const unsigned long long *const row_box = c.boxes + (size_t)blk0 * kCoopWords;
  for (int i = tid; i < kBins + 32; i += kSelThreads) hist[i] = 0;
  if (tid < 8) misc[tid] = 0;
  __syncthreads();
  FKV_TICK(7);

  // The search and the compaction of this block's slice; false if a wait ran out.  Block-uniform.
  auto run = [&]() -> bool {
    const uint32_t own_len = (uint32_t)max(0, min(v0 + kChunk, mis + P) - max(v0, mis));
    uint32_t own_in = own_len;               // this slice's keys in the interval
    uint32_t in_before = (uint32_t)min(max(v0 - mis, 0), P);  // keys of earlier slices in the interval
    uint32_t gt_before = 0;                  // keys of earlier slices above the interval
    uint32_t remaining = (uint32_t)kp, n_in = (uint32_t)P;
    uint32_t lo = 1u, span = 0xFFFFFFFEu;    // interval [lo, lo + span]
    if (tid < M) slice_cnt[tid] = (uint32_t)max(0, min(tid * kChunk + kChunk, mis + P) - max(tid * kChunk, mis));
    FKV_TICK(0);
    FKV_BTICK(0);

    auto clear_hist = [&]() {
      __syncthreads();
      for (int i = tid; i < kBins + 32; i += kSelThreads) hist[i] = 0;
      if (tid == 0) misc[0] = 0;
      __syncthreads();
    };
    auto count_in = [&](uint32_t n) {  // adds this thread's number of histogrammed keys to misc[0]
      n = wave_sum_to_last(n);
      if (lane == 63 && n != 0) atomicAdd(&misc[0], n);
    };
    const int pair = kSelThreads - 1 - tid;  // histogram bins 2*pair, 2*pair+1: thread order runs from the top bin down
    // This thread's bin pair of the slice's histogram as a mailbox payload (a slice has at most 32768 keys;
    // the keys a fill left out belong to bin 0).
    auto own_word = [&]() {
      uint32_t h0 = hist[2 * pair];
      const uint32_t h1 = hist[2 * pair + 1];
      if (pair == 0) h0 += own_in - misc[0];
      return (h1 << 16) | h0;
    };
    // Polls tagged words (addresses from `slot(i)`, i < the length of `got`; skip(i) = nothing to fetch)
    // until all carry this launch's epoch; payloads to `got`.  Wave-uniform result.
    auto fetch = [&](auto slot, auto skip, auto &got) -> bool {
      constexpr int kN = (int)(sizeof(got) / sizeof(got[0]));
      BoundedWait wait(c.timeout_ticks);
      if constexpr (kKpt >= 32 && kN > 4) {
        // 32 keys per thread leave few registers: four words in flight at a time
#pragma unroll
        for (int p0 = 0; p0 < kN; p0 += 4) {
          unsigned pending = 0;
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (p0 + i < kN && !skip(p0 + i)) pending |= 1u << i;
          while (true) {
            unsigned long long v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
              if (pending & (1u << i)) v[i] = tag_peek(slot(p0 + i));
#pragma unroll
            for (int i = 0; i < 4; ++i)
              if ((pending & (1u << i)) && tag_is(v[i], epoch)) {
                got[p0 + i] = (uint32_t)v[i];
                pending &= ~(1u << i);
              }
            if (!__any(pending != 0u)) break;
            if (wait.expired()) return false;
          }
        }
        return true;
      } else {
        unsigned pending = 0;
#pragma unroll
        for (int i = 0; i < kN; ++i)
          if (!skip(i)) pending |= 1u << i;
        while (true) {
          unsigned long long v[kN];
#pragma unroll
          for (int i = 0; i < kN; ++i)
            if (pending & (1u << i)) v[i] = tag_peek(slot(i));
#pragma unroll
          for (int i = 0; i < kN; ++i)
            if ((pending & (1u << i)) && tag_is(v[i], epoch)) {
              got[i] = (uint32_t)v[i];
              pending &= ~(1u << i);
            }
          if (!__any(pending != 0u)) return true;
          if (wait.expired()) return false;
        }
      }
    };
    // With every slice's histogram word of this thread's bin pair in w[] (own slice included): stages them,
    // picks the bin of the `remaining`-th largest key of the row and updates remaining, n_in, own_in,
    // in_before, gt_before.  `failed`: this wave's fetch ran out.  False if any wave's did.
    auto pick = [&](const uint32_t (&w)[kSl], bool failed, uint32_t &digit) -> bool {
      uint32_t *stage = scan_tbl;
      uint32_t tot0 = 0, tot1 = 0, bef0 = 0, bef1 = 0;
#pragma unroll
      for (int j = 0; j < kSl; ++j)
        if (j < M) {
          stage[j * kSelThreads + tid] = w[j];
          tot0 += w[j] & 0xFFFFu;
          tot1 += w[j] >> 16;
          if (j < s) { bef0 += w[j] & 0xFFFFu; bef1 += w[j] >> 16; }
        }
      if (failed && lane == 0) misc[3] = 1u;
      // inclusive scans from the top bin down: keys of the row / of the earlier slices in this pair and above
      const uint32_t both = tot0 + tot1, befb = bef0 + bef1;
      const uint32_t run_t = wave_scan_add(both), run_b = wave_scan_add(befb);
      if (lane == 63) { wsum[wave] = run_t; wsum[kSelWaves + wave] = run_b; }
      __syncthreads();
      if (misc[3] != 0u) return false;
      uint32_t above = run_t - both, above_b = run_b - befb;
      for (int i = 0; i < wave; ++i) { above += wsum[i]; above_b += wsum[kSelWaves + i]; }
      if (above < remaining && remaining <= above + both) {
        const bool top = remaining <= above + tot1;
        bcast[0] = 2 * pair + (top ? 1 : 0);
        bcast[1] = remaining - above - (top ? 0u : tot1);
        bcast[2] = top ? tot1 : tot0;
        bcast[3] = above_b + (top ? 0u : bef1);
        for (int j = 0; j < M; ++j) {
          const uint32_t x = stage[j * kSelThreads + tid];
          slice_cnt[j] = top ? x >> 16 : x & 0xFFFFu;
        }
      }
      __syncthreads();
      digit = bcast[0];
      remaining = bcast[1];
      n_in = bcast[2];
      gt_before += bcast[3];
      own_in = slice_cnt[s];
      in_before = 0;
      for (int j = 0; j < s; ++j) in_before += slice_cnt[j];
      return true;
    };
    // Finishes the search inside [lo, lo + span] on the list (one key per thread; 0 = none, keys outside the
    // interval take no part): sets lo to the threshold key; whole = every key >= lo is kept.
    auto finish_on_list = [&](uint32_t cand, bool &whole) {
      whole = false;
      if (span > 0u) {
        // first pass over 8192 bins (behind the staged histogram words): with a few hundred keys in the interval
        // the threshold's bin then holds one key, or only ties, and the search is over
        uint32_t *wide = scan_tbl + kCoopMaxSlices * kSelThreads;
        const int shift = max(32 - __clz(span) - 13, 0);
        const int grp = kSelThreads - 1 - tid;  // bins 8*grp .. 8*grp+7: thread order runs from the top bin down
        __syncthreads();
        *reinterpret_cast<u32x4 *>(wide + 8 * tid) = u32x4{0u, 0u, 0u, 0u};
        *reinterpret_cast<u32x4 *>(wide + 8 * tid + 4) = u32x4{0u, 0u, 0u, 0u};
        __syncthreads();
        {
          const uint32_t rel = cand - lo;  // below lo, or an empty slot (key 0): wraps above span
          if (rel <= span) atomicAdd(&wide[rel >> shift], 1u);
        }
        __syncthreads();
        const u32x4 lo4 = *reinterpret_cast<const u32x4 *>(wide + 8 * grp), hi4 = *reinterpret_cast<const u32x4 *>(wide + 8 * grp + 4);
        const uint32_t hb[8] = {lo4[0], lo4[1], lo4[2], lo4[3], hi4[0], hi4[1], hi4[2], hi4[3]};
        uint32_t sum8 = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) sum8 += hb[i];
        const uint32_t run_t = wave_scan_add(sum8);
        if (lane == 63) wsum[wave] = run_t;
        __syncthreads();
        uint32_t above = run_t - sum8;
        for (int i = 0; i < wave; ++i) above += wsum[i];
        if (above < remaining && remaining <= above + sum8) {
#pragma unroll
          for (int i = 7; i >= 0; --i) {
            if (above < remaining && remaining <= above + hb[i]) {
              bcast[0] = 8 * grp + i;
              bcast[1] = remaining - above;
              bcast[2] = hb[i];
            }
            above += hb[i];
          }
        }
        __syncthreads();
        const uint32_t digit = bcast[0];
        lo += digit << shift;
        span = shift == 0 ? 0u : min(span - (digit << shift), (1u << shift) - 1u);
        remaining = bcast[1];
        whole = bcast[2] == remaining;
      }
      while (span > 0u && !whole) {
        const int shift = max(32 - __clz(span) - 11, 0);
        clear_hist();
        {
          const uint32_t rel = cand - lo;
          if (rel <= span) atomicAdd(&hist[rel >> shift], 1u);
        }
        __syncthreads();
        const BinPick p = pick_bin(hist, wsum, bcast, remaining);
        lo += p.digit << shift;
        span = shift == 0 ? 0u : min(span - (p.digit << shift), (1u << shift) - 1u);
        remaining = p.remaining;
        whole = p.in_bin == p.remaining;
      }
    };

    // ---- the row's key range: the radix digits are taken relative to the smallest key, so the bins
    // spread over the values the row really holds (fp32 exponents would crowd them into a few dozen)
    {
      uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
#pragma unroll
      for (int e = 0; e < kKpt; ++e) {
        kmax = max(kmax, key[e]);
        kmin = min(kmin, key[e] - 1u);  // key 0 (no element) wraps to the largest value
      }
      kmax = wave_max_to_last(kmax);
      kmin = wave_min_to_last(kmin);
      if (lane == 63) { wsum[wave] = kmin; wsum[kSelWaves + wave] = kmax; }
      __syncthreads();
      if (tid < 2) {  // thread 0: smallest key - 1, thread 1: largest key of the slice
        uint32_t v = wsum[tid * kSelWaves];
        for (int i = 1; i < kSelWaves; ++i) v = tid == 0 ? min(v, wsum[i]) : max(v, wsum[kSelWaves + i]);
        tag_post(my_box + kCoopHeader + tid, epoch, v);
        bcast[5 + tid] = v;
      }
      uint32_t got[1] = {0u};
      const int peer = tid >> 1;
      const bool mine_to_fetch = wave == 0 && peer < M && peer != s;
      bool wave_ok = true;
      if (wave == 0) wave_ok = fetch([&](int) { return row_box + (size_t)min(peer, M - 1) * kCoopWords + kCoopHeader + (tid & 1); },
                                     [&](int) { return !mine_to_fetch; }, got);
      if (!wave_ok && lane == 0) misc[3] = 1u;
      if (mine_to_fetch) hdr[tid] = got[0];
      __syncthreads();
      if (misc[3] != 0u) return false;
      kmin = bcast[5];
      kmax = bcast[6];
      for (int j = 0; j < M; ++j)
        if (j != s) {
          kmin = min(kmin, hdr[2 * j]);
          kmax = max(kmax, hdr[2 * j + 1]);
        }
      kmin += 1u;
      lo = kmin;
      span = kmax - kmin;  // every key of the row lies in [lo, lo + span]
    }
    FKV_TICK(1);
    uint32_t w[kSl];
    uint32_t digit;

    uint32_t T, need_eq, eq_before = 0;
    int round = 0;
    while (true) {
      if (n_in == remaining) {  // the whole interval is kept: every key >= lo
        gt_before += in_before;
        T = lo - 1u;
        need_eq = 0;
        break;
      }
      if (span == 0u) {         // one key value left: the first `remaining` of its holders are kept
        T = lo;
        need_eq = remaining;
        eq_before = in_before;
        break;
      }
      if (n_in <= (uint32_t)kCoopCandCap) {
        uint32_t cand = 0;  // this thread's key of the list
        int my_sl = 0;      // and the slice it came from
        const uint32_t lo_list = lo, span_list = span;
        {
          // ---- the list: every slice posts its keys of the interval, every block reads them all
          uint32_t mine_n = 0;
#pragma unroll
          for (int e = 0; e < kKpt; ++e) mine_n += (key[e] - lo <= span) ? 1u : 0u;  // keys below lo and empty slots wrap above span
          const uint32_t inc = wave_scan_add(mine_n);
          const uint32_t wave_n = wave_last(inc);
          if (wave_n != 0u) {
            uint32_t wave_base = 0;
            if (lane == 63) wave_base = atomicAdd(&misc[5], wave_n);
            wave_base = wave_last(wave_base);
            uint32_t at = wave_base + inc - mine_n;
#pragma unroll
            for (int e = 0; e < kKpt; ++e)
              if (key[e] - lo <= span && at < (uint32_t)kCoopCandCap) tag_post(my_box + kCoopList + at++, epoch, key[e]);
          }
          const bool valid = (uint32_t)tid < n_in;
          uint32_t off = 0;
          if (valid)
            for (; my_sl < M - 1; ++my_sl) {
              const uint32_t n = slice_cnt[my_sl];
              if ((uint32_t)tid < off + n) break;
              off += n;
            }
          uint32_t one[1] = {0u};
          const bool got_it = fetch([&](int) { return row_box + (size_t)my_sl * kCoopWords + kCoopList + ((uint32_t)tid - off); },
                                    [&](int) { return !valid; }, one);
          cand = one[0];
          if (!got_it && lane == 0) misc[3] = 1u;
          __syncthreads();
          if (misc[3] != 0u) return false;
        }
        FKV_TICK(3);
        FKV_BTICK(2);
        bool whole;
        finish_on_list(cand, whole);
        // list keys of the earlier slices (inside the interval the list was made for) that are kept for sure /
        // that tie with the threshold
        const bool early = my_sl < s && cand - lo_list <= span_list;
        uint32_t n_kept = (early && (whole ? cand >= lo : cand > lo)) ? 1u : 0u;
        const uint32_t n_tied = (early && !whole && cand == lo) ? 1u : 0u;
        n_kept = wave_sum_to_last(n_kept | (n_tied << 16));
        if (lane == 63 && n_kept != 0u) {
          atomicAdd(&misc[1], n_kept & 0xFFFFu);
          atomicAdd(&misc[2], n_kept >> 16);
        }
        __syncthreads();
        gt_before += misc[1];
        eq_before = misc[2];
        T = whole ? lo - 1u : lo;
        need_eq = whole ? 0u : remaining;
        break;
      }
      // ---- another histogram round: the interval cut into equal parts
      ++round;
      if (round >= kCoopHistRounds) return false;  // (cannot happen: three rounds resolve 32 bits)
      const int shift = max(32 - __clz(span) - 11, 0);
      clear_hist();
      {
        uint32_t n = 0;
#pragma unroll
        for (int e = 0; e < kKpt; ++e) {  // keys equal to lo (there may be thousands) go to bin 0 by count
          const uint32_t rel = key[e] - lo;
          const bool counted = key[e] > lo && rel <= span;
          atomicAdd(&hist[counted ? rel >> shift : (uint32_t)kBins + (lane & 31)], 1u);
          n += counted ? 1u : 0u;
        }
        count_in(n);
      }
      __syncthreads();
      const uint32_t mine_r = own_word();
      tag_post(my_box + round * kSelThreads + tid, epoch, mine_r);
      const bool got_all = fetch([&](int j) { return row_box + (size_t)j * kCoopWords + round * kSelThreads + tid; },
                                 [&](int j) { return j >= M || j == s; }, w);
#pragma unroll
      for (int j = 0; j < kSl; ++j)
        if (j == s) w[j] = mine_r;
      if (!pick(w, !got_all, digit)) return false;
      lo += digit << shift;
      span = shift == 0 ? 0u : min(span - (digit << shift), (1u << shift) - 1u);
    }
    FKV_TICK(4);

    // ---- ordered compaction of this slice; earlier slices' kept / tied keys give the start
    __syncthreads();
    uint32_t run_gt = gt_before, run_eq = eq_before;
    compact_chunk<kKpt, true>(key, T, need_eq, run_gt, run_eq, v0 - mis, out, scan_tbl, wsum, bcast + 8);
    FKV_TICK(5);
    FKV_BTICK(3);
    return true;
  };

  bool ok = poisoned == 0u;  // invalid scores: no index may look usable
  if (ok) {
    if (s == 0 && tid < a.W) __hip_atomic_store(out + kp + tid, P + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // window tokens are always kept
    if (kp > 0) {
      ok = run();
      if (!ok && tid == 0) __hip_atomic_store(c.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }

  // ---- finish count.  Every block counts itself exactly once, after its stores have been acknowledged;
  // the last one closes the launch: -1 over every index if any block failed, next epoch.
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  FKV_TICK(8);
  if (tid == 0) {
    const unsigned add = ok ? 1u : 0x10001u;
    const unsigned now = __hip_atomic_fetch_add(c.state + 1, add, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + add;
    misc[4] = (now & 0xFFFFu) == gridDim.x ? (1u | ((now >> 16) != 0u ? 2u : 0u)) : 0u;
  }
  __syncthreads();
  const unsigned verdict = misc[4];
  FKV_TICK(9);
  if (verdict == 0u) return;
  if (verdict & 2u) {
    for (int i = 0; i < a.n_sets; ++i) {
      const int64_t n = (int64_t)a.set[i].n_rows * a.set[i].cnt_off[a.n_seq];
      for (int64_t j = tid; j < n; j += kSelThreads)
        __hip_atomic_store(a.set[i].idx_out + j, -1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  if (tid == 0) {
    __hip_atomic_store(c.state + 1, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(c.state + 0, epoch + 1u == 0u ? 1u : epoch + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

int select_coop_max_blocks_per_cu(void) {
  int n = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, k_select_coop<32, kCoopMaxSlices>, kSelThreads, 0) != hipSuccess) return 0;
  return n;
}

// Takes the launch if every row instance gets its blocks resident at once and rows are long enough for
// the exchanges to pay (mode 0), or whenever it fits (mode 2).  *e receives the launch result.
bool try_launch_select_coop(const SelectArgs &a, int rows, const SelectCoop &coop, hipStream_t s, hipError_t *e) {
  if (coop.boxes == nullptr || coop.mode == 1 || coop.max_blocks <= 0 || rows <= 0 || a.n_seq <= 0) return false;
  CoopArgs c{};
  int max_p = 0;
  for (int b = 0; b < a.n_seq; ++b) max_p = max(max_p, a.cu[b + 1] - a.cu[b] - a.W);
  // keys per thread: the fewest that keep the longest row within kCoopMaxSlices blocks
  int kpt = 8;
  while (kpt < kMaxKpt && coop_slices(max_p, kSelThreads * kpt) > kCoopMaxSlices) kpt *= 2;
  if (coop_slices(max_p, kSelThreads * kpt) > kCoopMaxSlices) return false;
  int64_t total = 0;
  for (int b = 0; b < a.n_seq; ++b) {
    const int P = a.cu[b + 1] - a.cu[b] - a.W;
    if (coop.mode != 2 && P + 3 <= kCoopMinKeys) return false;
    c.blk[b] = (int)total;
    total += (int64_t)rows * coop_slices(P, kSelThreads * kpt);
    if (total > coop.max_blocks) return false;
  }
  c.blk[a.n_seq] = (int)total;
  c.boxes = coop.boxes;
  c.state = coop.state;
  c.err = coop.err;
  c.timeout_ticks = coop.timeout_ticks;
  if (kpt == 8 && coop_slices(max_p, kSelThreads * kpt) <= 4)
    hipLaunchKernelGGL((k_select_coop<8, 4>), dim3((unsigned)total), dim3(kSelThreads), 0, s, a, c);
  else if (kpt == 8)
    hipLaunchKernelGGL((k_select_coop<8, kCoopMaxSlices>), dim3((unsigned)total), dim3(kSelThreads), 0, s, a, c);
  else if (kpt == 16)
    hipLaunchKernelGGL((k_select_coop<16, kCoopMaxSlices>), dim3((unsigned)total), dim3(kSelThreads), 0, s, a, c);
  else
    hipLaunchKernelGGL((k_select_coop<32, kCoopMaxSlices>), dim3((unsigned)total), dim3(kSelThreads), 0, s, a, c);
  *e = hipGetLastError();
  return true;
}

}  // namespace fkv
