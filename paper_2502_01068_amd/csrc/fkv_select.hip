// Top-k of one score row with the window merged in (Sec. 4.2): exact radix select on the
// order-preserving integer image of the fp32 scores, then an ordered compaction, so the
// output is ascending, has exactly k entries and equal scores go to the lower index.
//
// One block per (row, sequence).  Four 8-bit passes narrow down the key T of the
// (k-W)-th largest prefix score; the compaction keeps every key > T and the first
// `need_eq` keys == T in index order, using wave ballots for the in-wave rank.
#include "fkv_internal.h"

namespace fkv {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;

// Monotone map fp32 -> uint32 (larger float <=> larger key), valid for any non-NaN input;
// -0.0 and +0.0 compare equal as floats, so both get the key of +0.0.
__device__ __forceinline__ uint32_t order_key(float f) {
  uint32_t u = __float_as_uint(f);
  if (u == 0x80000000u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__global__ __launch_bounds__(kSelThreads) void k_select(SelectArgs a) {
  __shared__ uint32_t hist[256];
  __shared__ uint32_t sh_prefix, sh_remaining;
  __shared__ uint32_t wave_gt[2][kSelWaves], wave_eq[2][kSelWaves];

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
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  if (tid < a.W) out[kp + tid] = P + tid;  // window tokens are always kept
  if (kp <= 0) return;

  uint32_t prefix = 0, mask = 0, remaining = (uint32_t)kp;
  for (int shift = 24; shift >= 0; shift -= 8) {
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    for (int i = tid; i < P; i += kSelThreads) {
      const uint32_t key = order_key(sc[i]);
      if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (wave == 0) {
      // lane owns bins 4*lane .. 4*lane+3; suffix counts from the top bin down
      const uint32_t h0 = hist[4 * lane], h1 = hist[4 * lane + 1], h2 = hist[4 * lane + 2],
                     h3 = hist[4 * lane + 3];
      const uint32_t mine = h0 + h1 + h2 + h3;
      uint32_t above = 0;  // count in lanes > lane
      uint32_t run = mine;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const uint32_t v = __shfl_down(run, off);
        if (lane + off < 64) run += v;
      }
      above = run - mine;
      // the digit is in this lane iff above < remaining <= above + mine
      if (above < remaining && remaining <= above + mine) {
        uint32_t acc = above;
        int digit;
        if (remaining <= acc + h3) digit = 3;
        else if (remaining <= (acc += h3) + h2) digit = 2;
        else if (remaining <= (acc += h2) + h1) digit = 1;
        else { acc += h1; digit = 0; }
        sh_prefix = prefix | ((uint32_t)(4 * lane + digit) << shift);
        sh_remaining = remaining - acc;
      }
    }
    __syncthreads();
    prefix = sh_prefix;
    remaining = sh_remaining;
    mask |= 255u << shift;
  }
  const uint32_t T = prefix;            // key of the kp-th largest score
  const uint32_t need_eq = remaining;   // how many keys == T are kept (>= 1)

  uint32_t run_gt = 0, run_eq = 0;      // kept-so-far counters, identical in every thread
  int buf = 0;
  for (int base = 0; base < P; base += kSelThreads, buf ^= 1) {
    const int i = base + tid;
    uint32_t key = 0;
    bool gt = false, eq = false;
    if (i < P) {
      key = order_key(sc[i]);
      gt = key > T;
      eq = key == T;
    }
    const uint64_t bg = __ballot(gt), be = __ballot(eq);
    if (lane == 0) {
      wave_gt[buf][wave] = (uint32_t)__popcll(bg);
      wave_eq[buf][wave] = (uint32_t)__popcll(be);
    }
    __syncthreads();
    uint32_t gt_before = run_gt, eq_before = run_eq, tot_gt = 0, tot_eq = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) {
      const uint32_t cg = wave_gt[buf][w], ce = wave_eq[buf][w];
      if (w < wave) { gt_before += cg; eq_before += ce; }
      tot_gt += cg;
      tot_eq += ce;
    }
    const uint64_t lower = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    gt_before += (uint32_t)__popcll(bg & lower);
    eq_before += (uint32_t)__popcll(be & lower);
    if (gt || (eq && eq_before < need_eq)) out[gt_before + min(eq_before, need_eq)] = i;
    run_gt += tot_gt;
    run_eq += tot_eq;
  }
}

hipError_t launch_select(const SelectArgs &a, hipStream_t s) {
  int rows = 0;
  for (int i = 0; i < a.n_sets; ++i) rows += a.set[i].n_rows;
  hipLaunchKernelGGL(k_select, dim3(rows, a.n_seq), dim3(kSelThreads), 0, s, a);
  return hipGetLastError();
}

}  // namespace fkv
