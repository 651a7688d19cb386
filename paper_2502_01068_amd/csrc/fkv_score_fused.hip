// Single-pass window-attention scores (Sec. 4.2 Eq. 1-2, App. B.1): K is read from HBM once.
//
// The softmax normaliser of every window row depends on all keys, so a block cannot turn its
// logits into probabilities until every block has seen its share of K.  Here the logits wait in
// registers: each block owns a contiguous token range small enough that its logits (up to 8 MFMA
// sub-tiles x 16 accumulator registers per lane) stay on chip, all blocks are resident at once
// (one per CU), and a grid-wide exchange of the per-row (max, sum) pairs sits between the K
// stream and the probability / pooling / averaging phase:
//
//   phase 1  stream the block's K rows (owned range plus pooling halo), keep raw logits in
//            registers, fold running (max, sum) of the owned tokens per softmax row
//   phase 2  publish the block's partials; the last block to arrive in each cluster of 16
//            folds the cluster; when all clusters are done every block folds the <= 16 cluster
//            results of its sequence in a fixed order (bit-reproducible)
//   phase 3  probabilities from the kept logits, window sum, LDS pooling, head means, write
//
// Used when the batch fits the resident grid (about 64K tokens on 256 CUs); longer inputs take
// the two-pass kernels.  The wait in phase 2 is bounded: a block that does not see the grid
// complete within the time limit raises the context's error flag and skips phase 3.
#include "fkv_score_common.h"

namespace fkv {

constexpr int kFusedSubShort = 5;  // sub-tiles (of 32 tokens) a block keeps in registers: the variant for inputs
constexpr int kFusedSubLong = 8;   // that fit 5 per block carries less register-select work per logit
constexpr int kFusedSlotsMax = kFusedSubLong * kSub;
constexpr int kClusterSize = 16;

int fused_slots(void) { return kFusedSlotsMax; }
int fused_cluster_size(void) { return kClusterSize; }

// Cross-block exchange without cache maintenance.  The L2 caches of the chip's XCDs are not
// coherent with each other, and an agent-scope release / acquire fence writes back / invalidates
// a whole L2 (tens of microseconds here).  Instead every value another block reads is written
// with an agent-scope atomic exchange (performed at the coherence point, complete when its
// result returns) and read with an agent-scope atomic load (which bypasses the local L2); a
// workgroup-scope fence (wait for outstanding memory operations, no cache action) plus the
// block barrier orders them before the counter update.  These buffers are touched by nothing else.
__device__ __forceinline__ void st_coherent(float2 *p, float2 v) {
  unsigned long long bits;
  __builtin_memcpy(&bits, &v, sizeof bits);
  const unsigned long long old = __hip_atomic_exchange(reinterpret_cast<unsigned long long *>(p), bits,
                                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  asm volatile("" ::"v"(old));  // keep the returning form: its completion is what the fence waits for
}
__device__ __forceinline__ float2 ld_coherent(const float2 *p) {
  const unsigned long long bits = __hip_atomic_load(reinterpret_cast<const unsigned long long *>(p),
                                                    __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  float2 v;
  __builtin_memcpy(&v, &bits, sizeof v);
  return v;
}
__device__ __forceinline__ unsigned ld_counter(const unsigned *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void block_publish() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __syncthreads();
}

template <int kFusedSub>
__global__ __launch_bounds__(kThreads) void k_score_fused(ScoreArgs a, FusedArgs f) {
  constexpr int kFusedSlots = kFusedSub * kSub;
  __shared__ __attribute__((aligned(16))) uint8_t lds_all[kWaves * kStageBytes];
  __shared__ float cst_lds[kWaves][kRowsPerGroup];
  __shared__ unsigned flag_lds[2];
  float(*s_head)[kFusedSlots] = reinterpret_cast<float(*)[kFusedSlots]>(lds_all);  // [Hkv*4][slots]
  float(*g_sum)[kFusedSlots] =
      reinterpret_cast<float(*)[kFusedSlots]>(lds_all + kMaxKvHeads * kMaxGroup * kFusedSlots * 4);
  static_assert((kMaxKvHeads * kMaxGroup + kMaxKvHeads) * kFusedSlots * 4 <= kWaves * kStageBytes, "LDS reuse");

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 31, hi = lane >> 5;
  const int b = find_seq(a.map, blockIdx.x);
  const int tok_base = a.map.cu[b];
  const int Lb = a.map.cu[b + 1] - tok_base;
  const int P = Lb - a.W;
  const int r = a.pool_r;
  const int local = (int)blockIdx.x - a.map.blk[b];
  const int n_ranges = a.map.blk[b + 1] - a.map.blk[b];
  const int o0 = local * f.own[b], o1 = min(P, o0 + f.own[b]);  // owned prefix tokens
  const bool last = local == n_ranges - 1;                      // also owns the window columns
  const int c0 = o0 - r;                                        // first computed token (may be < 0)
  const int c1 = last ? max(Lb, o1 + r) : o1 + r;               // the pooling halo may reach past the window (r > W)
  const int n_sub = (c1 - c0 + kSub - 1) / kSub;                // <= kFusedSub (host guarantees)
  uint8_t *stage = lds_all + wave * kStageBytes;
  const int g = wave;
  const bool has_group = g < a.V;  // the host takes this kernel only for V <= 8 (one wave per virtual group)

  FKV_TICK(32);
  FKV_BTICK(0);
  // ---- phase 1: logits into registers, running statistics of the owned tokens
  float z[kFusedSub][16], mloc[16];
  float2 ms = make_float2(kNegBig, 0.f);
  if (has_group) {
    bf16x8 qa[8];
    load_q(a, b, g, lane, qa);
    float mx[16], sm[16];
#pragma unroll
    for (int q = 0; q < 16; ++q) { mx[q] = kNegBig; sm[q] = 0.f; }
    stream_head_direct(a, qa, tok_base, Lb, g, c0, n_sub, stage, lane, [&](int st, const floatx16 &acc) {
      const int tok = c0 + st * kSub + n;
      const bool counted = (tok >= o0 && tok < o1) || (last && tok >= P && tok < Lb);
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int w = hi * 4 + (q & 3);
        const bool ok = counted && (!a.causal || tok <= P + w);
        const float zz = acc[q] * a.scale_log2e;
#pragma unroll
        for (int t = 0; t < kFusedSub; ++t)
          if (t == st) z[t][q] = zz;
        // running reference = max over every computed logit (counted or not), so that
        // 2^(z - reference) <= 1 for all of them; only counted keys enter the sum
        const float d = zz - mx[q];
        const float e = fast_exp2(-fabsf(d));
        const float one = ok ? 1.f : 0.f;
        sm[q] = d > 0.f ? sm[q] * e + one : sm[q] + one * e;
        mx[q] = fmaxf(mx[q], zz);
      }
    });
    FKV_TICK(33);
    ms = fold_rows(mx, sm, reinterpret_cast<float *>(stage), lane);
    if (lane < 32) st_coherent(f.bpartial + (size_t)(g * kRowsPerGroup + lane) * f.bpartial_stride + blockIdx.x, ms);
    // While the exchange is in flight: turn the kept logits into 2^(z - block reference).  The
    // global normaliser then costs one multiply per value instead of an exponential.
    const float *mrow = reinterpret_cast<const float *>(stage) + kFoldMaxOffset;
#pragma unroll
    for (int q = 0; q < 16; ++q) mloc[q] = mrow[(q >> 2) * 8 + hi * 4 + (q & 3)];
#pragma unroll
    for (int st = 0; st < kFusedSub; ++st)
      if (st < n_sub) {
#pragma unroll
        for (int q = 0; q < 16; ++q) z[st][q] = fast_exp2(z[st][q] - mloc[q]);
      }
  }

  FKV_TICK(34);
  FKV_BTICK(1);
  // ---- phase 2: grid-wide fold of the row statistics
  const int cl_local = local / kClusterSize;
  const int cluster = f.cl0[b] + cl_local;
  const int cl_first = a.map.blk[b] + cl_local * kClusterSize;  // first block of the cluster
  const int cl_size = min(kClusterSize, n_ranges - cl_local * kClusterSize);
  block_publish();
  FKV_TICK(35);
  if (threadIdx.x == 0) {
    const unsigned ticket =
        __hip_atomic_fetch_add(&f.counters[cluster], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    flag_lds[0] = (ticket == (unsigned)cl_size - 1u) ? 1u : 0u;
  }
  __syncthreads();
  if (flag_lds[0]) {  // this block closes its cluster
    if ((int)threadIdx.x < a.V * kRowsPerGroup) {
      const float2 *src = f.bpartial + (size_t)threadIdx.x * f.bpartial_stride + cl_first;
      float2 v[kClusterSize];  // all loads in flight before the (ordered) fold
#pragma unroll
      for (int i = 0; i < kClusterSize; ++i) v[i] = ld_coherent(src + (i < cl_size ? i : 0));
      float2 acc = v[0];
#pragma unroll
      for (int i = 1; i < kClusterSize; ++i)
        if (i < cl_size) acc = merge_stats(acc, v[i]);
      st_coherent(f.cpartial + (size_t)threadIdx.x * f.cpartial_stride + cluster, acc);
    }
    block_publish();
    if (threadIdx.x == 0) {
      __hip_atomic_store(&f.counters[cluster], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_fetch_add(&f.counters[kCtrDone], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  FKV_TICK(36);
  if (threadIdx.x == 0) {
    const unsigned long long t0 = wall_clock64();
    unsigned ok = 1u;
    while (ld_counter(&f.counters[kCtrDone]) < (unsigned)f.n_clusters) {
      __builtin_amdgcn_s_sleep(2);
      if (wall_clock64() - t0 > f.timeout_ticks) { ok = 0u; break; }
    }
    flag_lds[1] = ok;
  }
  __syncthreads();
  const bool grid_ok = flag_lds[1] != 0u;
  FKV_TICK(37);
  FKV_BTICK(2);
  FKV_TICK(38);

  if (grid_ok && has_group) {
    // lanes l and l+32 fold the even / odd clusters of this sequence for row l, then merge
    const int row = lane & 31, half = lane >> 5;
    const float2 *src = f.cpartial + (size_t)(g * kRowsPerGroup + row) * f.cpartial_stride;
    float2 acc = make_float2(kNegBig, 0.f);
    const int c_lo = f.cl0[b] + half, c_hi = f.cl0[b + 1];
    for (int cb = c_lo; cb < c_hi; cb += 16) {  // 8 loads in flight per round, folded in order
      float2 v[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = ld_coherent(src + (cb + 2 * i < c_hi ? cb + 2 * i : c_lo));
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (cb + 2 * i < c_hi) acc = merge_stats(acc, v[i]);
    }
    float2 oth;
    oth.x = __shfl_xor(acc.x, 32);
    oth.y = __shfl_xor(acc.y, 32);
    const float2 lo2 = half ? oth : acc, hi2 = half ? acc : oth;
    const float2 tot = merge_stats(lo2, hi2);
    const bool row_ok = (row >> 3) < vg_heads(a, g) && (row & 7) < a.W;
    if (lane < 32) cst_lds[wave][row] = row_ok ? (tot.x + __log2f(tot.y)) : 0.f;
  }
  __syncthreads();  // all staging tiles are dead, cst_lds is visible
  FKV_TICK(39);

  // ---- phase 3: probabilities from the kept logits, window sums into LDS
  if (grid_ok && has_group) {
    float fac[16];  // 2^(block reference - global log-sum-exp) per row
#pragma unroll
    for (int q = 0; q < 16; ++q) fac[q] = fast_exp2(mloc[q] - cst_lds[wave][(q >> 2) * 8 + hi * 4 + (q & 3)]);
#pragma unroll
    for (int st = 0; st < kFusedSub; ++st) {
      if (st < n_sub) {
        const int tok = c0 + st * kSub + n;
        const bool inb = tok >= 0 && tok < P;  // only prefix tokens are scored
#pragma unroll
        for (int hl = 0; hl < 4; ++hl) {
          float sum = 0.f;
#pragma unroll
          for (int rr = 0; rr < 4; ++rr) sum += (hi * 4 + rr < a.W) ? z[st][hl * 4 + rr] * fac[hl * 4 + rr] : 0.f;
          sum = add_across_halves(sum);  // other half of the window rows
          if (hi == 0 && hl < vg_heads(a, g)) s_head[g * kMaxGroup + hl][st * kSub + n] = inb ? sum : 0.f;
        }
      }
    }
  }
  __syncthreads();
  FKV_TICK(40);
  if (grid_ok) pool_and_write<kFusedSlots>(a, s_head, g_sum, c0, o0, o1, tok_base - b * a.W);
  FKV_TICK(41);
  FKV_BTICK(3);

  // ---- leave the grid: the last block out re-arms the counters for the next launch
  if (threadIdx.x == 0) {
    if (!grid_ok) __hip_atomic_store(&f.counters[kCtrError], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned e = __hip_atomic_fetch_add(&f.counters[kCtrExit], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (e == (unsigned)f.n_wg - 1u) {
      __hip_atomic_store(&f.counters[kCtrDone], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(&f.counters[kCtrExit], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

hipError_t launch_score_fused(const ScoreArgs &a, const FusedArgs &f, hipStream_t s) {
  if (f.n_sub_max <= kFusedSubShort)
    hipLaunchKernelGGL(k_score_fused<kFusedSubShort>, dim3(f.n_wg), dim3(kThreads), 0, s, a, f);
  else
    hipLaunchKernelGGL(k_score_fused<kFusedSubLong>, dim3(f.n_wg), dim3(kThreads), 0, s, a, f);
  return hipGetLastError();
}

int score_fused_max_blocks_per_cu(void) {
  int n = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, k_score_fused<kFusedSubLong>, kThreads, 0) != hipSuccess) return 0;
  return n;
}

}  // namespace fkv
