// Top-k of rows longer than one block's register-resident chunk (32768 keys): the row is cut into
// 8192-key slices, one 1024-thread block each, and the radix search runs as a short chain of
// launches with per-row state in global memory (kernel boundaries are the only grid-wide
// synchronisation; a launch costs far less than one more sweep of the row by a single block):
//
//   prep      zero the row's histograms, fold the row's smallest / largest key (atomic max),
//             write the window indices
//   hist<1>   digits of (key - smallest), up to 11 bits, of every key       -> histogram 1
//   hist<2>   pick the bin from histogram 1; candidates' next digits        -> histogram 2
//   hist<3>   pick the bin from histogram 2; candidates' last digits        -> histogram 3
//   count     pick the bin from histogram 3: T and how many keys == T are kept; per-slice counts
//             of keys > T and == T
//   compact   prefix of the slice counts, then the same ordered compaction as the one-block
//             kernel; zeroes the min / max words for the next call
//
// Every block of a launch derives the same interval from the same global histogram, so no value
// crosses blocks inside a launch except through atomic adds / maxes on the row state.
#include "fkv_select_common.h"

namespace fkv {

constexpr int kLongKpt = 8;
constexpr int kLongChunk = kSelThreads * kLongKpt;  // 8192 keys per block
constexpr int kOneBlockMax = kSelThreads * kMaxKpt; // rows up to this stay on the one-block kernel

int select_long_threshold(void) { return kOneBlockMax; }
int select_long_chunk(void) { return kLongChunk; }

// info words of a row's state
// Launch R (2..4) writes the interval it derived to words 4(R-2).. and reads what launch R-1 wrote,
// so no launch reads words another block of the same launch writes.
enum { kInfLo = 0, kInfS = 1, kInfRem = 2, kInfCount = 3, kInfSlot = 4, kInfMax = 12, kInfNotMin = 13 };

struct LongRow {
  const float *base;  // row pointer rounded down to 16 bytes
  int mis, P, kp, slice, W;
  int32_t *out;
  uint32_t *st;       // this row instance's state block
  bool is_long;       // row is handled by this chain
  bool active;        // ... and this block has keys and something to select
};

__device__ __forceinline__ LongRow locate_long(const SelectArgs &a) {
  LongRow r;
  int row = blockIdx.x;
  const int set_id = (a.n_sets > 1 && row >= a.set[0].n_rows) ? 1 : 0;
  const int row_global = row;
  if (set_id) row -= a.set[0].n_rows;
  const SelectRowSet &rs = a.set[set_id];
  const int b = blockIdx.y;
  const int Lb = a.cu[b + 1] - a.cu[b];
  r.W = a.W;
  r.P = Lb - a.W;
  r.kp = rs.cnt_off[b + 1] - rs.cnt_off[b] - a.W;
  const float *sc = rs.scores + (size_t)row * rs.row_stride + (a.cu[b] - b * a.W);
  r.mis = (int)((reinterpret_cast<uintptr_t>(sc) >> 2) & 3);
  r.base = sc - r.mis;
  r.out = rs.idx_out + (size_t)row * rs.cnt_off[a.n_seq] + rs.cnt_off[b];
  r.st = a.long_state + (size_t)(row_global * a.n_seq + b) * kLongStateWords;
  r.slice = blockIdx.z;
  const int n_slices = (r.P + r.mis + kLongChunk - 1) / kLongChunk;
  r.is_long = r.P + 3 > kOneBlockMax;
  r.active = r.is_long && r.kp > 0 && r.slice < n_slices;
  return r;
}

// Interval [lo, lo + 2^s) and rank after `rounds` completed rounds, from the state the previous
// launches left: the first histogram launch starts from the row's key range.
struct Interval { uint32_t lo, remaining, count; int s; };  // count: keys of the row inside the interval
__device__ __forceinline__ Interval initial_interval(const LongRow &r) {
  Interval v;
  const uint32_t kmax = r.st[kLongInfo + kInfMax], kmin = ~r.st[kLongInfo + kInfNotMin];
  v.lo = kmin;
  v.s = kmax == kmin ? 0 : 32 - __clz(kmax - kmin);
  v.remaining = (uint32_t)r.kp;
  v.count = (uint32_t)r.P;
  return v;
}

__global__ __launch_bounds__(kSelThreads) void k_sel_long_prep(SelectArgs a) {
  __shared__ uint32_t red[2 * kSelWaves];
  const LongRow r = locate_long(a);
  if (!r.is_long) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (r.slice == 0) {
    if (tid < r.W) r.out[r.kp + tid] = r.P + tid;  // window tokens are always kept
    for (int i = tid; i < 3 * kBins; i += kSelThreads) r.st[i] = 0u;
  }
  if (!r.active) return;
  uint32_t key[kLongKpt];
  load_keys<kLongKpt>(r.base, r.mis, r.P, r.slice * kLongChunk, wave, lane, key);
  uint32_t kmax = 0u, nmin = 0u;  // nmin = max over valid keys of ~key (empty slots give ~(0-1)... excluded)
#pragma unroll
  for (int e = 0; e < kLongKpt; ++e) {
    kmax = max(kmax, key[e]);
    nmin = max(nmin, key[e] ? ~key[e] : 0u);
  }
  kmax = wave_max_to_last(kmax);
  nmin = wave_max_to_last(nmin);
  if (lane == 63) { red[wave] = kmax; red[kSelWaves + wave] = nmin; }
  __syncthreads();
  if (tid == 0) {
    kmax = 0u, nmin = 0u;
    for (int w = 0; w < kSelWaves; ++w) { kmax = max(kmax, red[w]); nmin = max(nmin, red[kSelWaves + w]); }
    atomicMax(&r.st[kLongInfo + kInfMax], kmax);
    atomicMax(&r.st[kLongInfo + kInfNotMin], nmin);
  }
}

// Round kRound (1..3) of the search; kRound == 4 is the counting launch.
template <int kRound>
__global__ __launch_bounds__(kSelThreads) void k_sel_long_round(SelectArgs a) {
  __shared__ uint32_t hist[kBins];
  __shared__ uint32_t wsum[kSelWaves];
  __shared__ uint32_t bcast[4];
  const LongRow r = locate_long(a);
  if (!r.active) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  uint32_t key[kLongKpt];
  load_keys<kLongKpt>(r.base, r.mis, r.P, r.slice * kLongChunk, wave, lane, key);

  // interval before this round: from the key range (first histogram launch) or from what launch kRound-1 stored,
  // narrowed by the bin picked from that round's histogram
  Interval v;
  if (kRound <= 2) {
    v = initial_interval(r);
  } else {
    const uint32_t *prev = r.st + kLongInfo + kInfSlot * (kRound - 3);
    v.lo = prev[kInfLo];
    v.s = (int)prev[kInfS];
    v.remaining = prev[kInfRem];
    v.count = prev[kInfCount];
  }
  if (kRound > 1 && v.s > 0) {
    const uint32_t *gh = r.st + (kRound - 2) * kBins;
    for (int i = tid; i < kBins; i += kSelThreads) hist[i] = gh[i];
    __syncthreads();
    // the histograms leave out the keys equal to the interval's lower end; pick_bin credits them to bin 0
    const BinPick p = pick_bin(hist, wsum, bcast, v.remaining, v.count);
    const int shift = v.s - min(11, v.s);
    v.lo += p.digit << shift;
    v.s = shift;
    v.remaining = p.remaining;
    v.count = p.in_bin;
  }
  if (kRound > 1 && r.slice == 0 && tid == 0) {  // read by the next launch
    uint32_t *mine = r.st + kLongInfo + kInfSlot * (kRound - 2);
    mine[kInfLo] = v.lo;
    mine[kInfS] = (uint32_t)v.s;
    mine[kInfRem] = v.remaining;
    mine[kInfCount] = v.count;
  }
  if (kRound <= 3) {
    if (v.s == 0) return;  // the interval is a single key already
    const int shift = v.s - min(11, v.s);
    const uint32_t span = v.s >= 32 ? 0xFFFFFFFFu : ((1u << v.s) - 1u);
    for (int i = tid; i < kBins; i += kSelThreads) hist[i] = 0;
    __syncthreads();
#pragma unroll
    for (int e = 0; e < kLongKpt; ++e) {
      const uint32_t rel = key[e] - v.lo;
      if (key[e] > v.lo && rel <= span) atomicAdd(&hist[rel >> shift], 1u);  // key 0 (empty) is below lo; keys == lo
                                                                             // are recovered from the total
    }
    __syncthreads();
    uint32_t *gh = r.st + (kRound - 1) * kBins;
    for (int i = tid; i < kBins; i += kSelThreads) {
      const uint32_t c = hist[i];
      if (c) atomicAdd(&gh[i], c);
    }
  } else {
    // v.lo is T (s == 0 after at most three rounds of 11 bits), v.remaining the equal keys kept
    const uint32_t T = v.lo;
    uint32_t cg = 0, ce = 0;
#pragma unroll
    for (int e = 0; e < kLongKpt; ++e) {
      cg += key[e] > T ? 1u : 0u;
      ce += key[e] == T ? 1u : 0u;
    }
    cg = wave_sum_to_last(cg);
    ce = wave_sum_to_last(ce);
    __syncthreads();  // pick_bin's readers of wsum are done
    if (lane == 63) { wsum[wave] = cg; hist[wave] = ce; }
    __syncthreads();
    if (tid == 0) {
      uint32_t tg = 0, te = 0;
      for (int w = 0; w < kSelWaves; ++w) { tg += wsum[w]; te += hist[w]; }
      r.st[kLongCnt + 2 * r.slice] = tg;
      r.st[kLongCnt + 2 * r.slice + 1] = te;
    }
  }
}

__global__ __launch_bounds__(kSelThreads) void k_sel_long_compact(SelectArgs a) {
  __shared__ __attribute__((aligned(16))) uint32_t scan_tbl[kSelWaves * 64 * kMaxKpt];
  __shared__ uint32_t wsum[kSelWaves];
  __shared__ uint32_t sink[64];
  __shared__ uint32_t pre[2];
  const LongRow r = locate_long(a);
  if (!r.is_long) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (a.err != nullptr && *a.err != 0u) {  // the scores are invalid: no index may look usable
    if (r.slice == 0) {
      for (int i = tid; i < r.kp + r.W; i += kSelThreads) r.out[i] = -1;
      if (tid == 0) {
        r.st[kLongInfo + kInfMax] = 0u;
        r.st[kLongInfo + kInfNotMin] = 0u;
      }
    }
    return;
  }
  if (!r.active) return;
  uint32_t key[kLongKpt];
  load_keys<kLongKpt>(r.base, r.mis, r.P, r.slice * kLongChunk, wave, lane, key);
  if (tid < 2) pre[tid] = 0;
  __syncthreads();
  if (tid < r.slice) {  // slices before this one (at most kLongMaxSlices <= blockDim)
    atomicAdd(&pre[0], r.st[kLongCnt + 2 * tid]);
    atomicAdd(&pre[1], r.st[kLongCnt + 2 * tid + 1]);
  }
  __syncthreads();
  uint32_t run_gt = pre[0], run_eq = pre[1];
  const uint32_t *fin = r.st + kLongInfo + kInfSlot * 2;  // written by the counting launch
  const uint32_t T = fin[kInfLo], need_eq = fin[kInfRem];
  if (r.slice == 0 && tid == 0) {  // min / max must be zero when the next call's prep launch folds into them
    r.st[kLongInfo + kInfMax] = 0u;
    r.st[kLongInfo + kInfNotMin] = 0u;
  }
  compact_chunk<kLongKpt>(key, T, need_eq, run_gt, run_eq, r.slice * kLongChunk - r.mis, r.out, scan_tbl, wsum, sink);
}

hipError_t launch_select_long(const SelectArgs &a, int rows, int max_slices, hipStream_t s) {
  const dim3 grid(rows, a.n_seq, max_slices), block(kSelThreads);
  hipLaunchKernelGGL(k_sel_long_prep, grid, block, 0, s, a);
  hipLaunchKernelGGL(k_sel_long_round<1>, grid, block, 0, s, a);
  hipLaunchKernelGGL(k_sel_long_round<2>, grid, block, 0, s, a);
  hipLaunchKernelGGL(k_sel_long_round<3>, grid, block, 0, s, a);
  hipLaunchKernelGGL(k_sel_long_round<4>, grid, block, 0, s, a);
  hipLaunchKernelGGL(k_sel_long_compact, grid, block, 0, s, a);
  return hipGetLastError();
}

}  // namespace fkv
