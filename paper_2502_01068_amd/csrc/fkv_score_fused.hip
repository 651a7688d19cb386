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
//   phase 2  every block posts its 256 row partials; each softmax row has one owner wave somewhere
//            in the grid that collects the row's partials from all blocks of the sequence, folds
//            them in a fixed order (bit-reproducible) and posts the row's log-sum-exp to every
//            block of the sequence
//   phase 3  probabilities from the kept logits, window sum, LDS pooling, head means, write
//
// Used when the batch fits the resident grid (about 64K tokens on 256 CUs); longer inputs take
// the two-pass kernels.  Every wait in phase 2 is bounded: a wave that does not get what it waits
// for within the time limit raises the context's error flag, and its block writes NaN scores.
#include "fkv_dpp.h"
#include "fkv_mailbox.h"
#include "fkv_score_common.h"

namespace fkv {

constexpr int kFusedSubShort = 5;  // sub-tiles (of 32 tokens) a block keeps in registers: the variant for inputs
constexpr int kFusedSubLong = 8;   // that fit 5 per block carries less register-select work per logit
constexpr int kFusedSlotsMax = kFusedSubLong * kSub;
constexpr int kBoxChunks = kMaxFusedBlocks / 64;  // 64-block chunks an owner wave collects

int fused_slots(void) { return kFusedSlotsMax; }
// Block count up to which a layout of n_sub full sub-tiles per block is preferred over one more
// sub-tile per block (fewer, longer blocks): the exchange gets slower with the number of blocks.
// Swept over 2048 .. 49152 tokens (e.g. 6554 tokens: 64 blocks 21.1 us, 113 blocks 18.0, 160 blocks
// 18.6, 256 blocks 18.4; 32768 tokens: 213 blocks 28.3, 256 blocks 28.7).
int fused_preferred_blocks(int n_sub) { return n_sub == 1 ? 128 : 224; }

// Writes NaN into every score this block owns: a call whose exchange failed must not leave
// plausible numbers behind.
__device__ __forceinline__ void poison_scores(const ScoreArgs &a, int col0, int o0, int o1) {
  const float nan = __uint_as_float(0x7FC00000u);
  const int own = o1 - o0;
  for (int i = threadIdx.x; i < own; i += blockDim.x) {
    const size_t col = (size_t)col0 + o0 + i;
    if (a.scores_group)
      for (int g = 0; g < a.Hkv; ++g) a.scores_group[(size_t)g * a.sum_p + col] = nan;
    if (a.scores_head)
      for (int h = 0; h < a.Hq; ++h) a.scores_head[(size_t)h * a.sum_p + col] = nan;
    if (a.scores_tsp) a.scores_tsp[col] = nan;
  }
}

template <int kFusedSub>
__global__ __launch_bounds__(kThreads) void k_score_fused(ScoreArgs a, FusedArgs f) {
  constexpr int kFusedSlots = kFusedSub * kSub;
  __shared__ __attribute__((aligned(16))) uint8_t lds_all[kWaves * kStageBytes];
  __shared__ float cst_lds[kWaves][kRowsPerGroup];
  __shared__ unsigned flag_lds[1];
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
  const int col0 = tok_base - b * a.W;
  uint8_t *stage = lds_all + wave * kStageBytes;
  const int g = wave;
  const bool has_group = g < a.V;  // the host takes this kernel only for V <= 8 (one wave per virtual group)

  // A failed exchange leaves mailboxes in an unknown state: until the host has reset them
  // (fkv_clear_error) every launch only marks its scores invalid.
  if (*f.err != 0u) {
    poison_scores(a, col0, o0, o1);
    return;
  }
  if (threadIdx.x == 0) flag_lds[0] = 1u;

  FKV_TICK(32);
  FKV_BTICK(0);
  // ---- phase 1: logits into registers, running statistics of the owned tokens
  float z[kFusedSub][16], mloc[16];
  if (has_group) {
    bf16x8 qa[8];
    load_q(a, b, g, lane, qa);
    float mx[16], sm[16];
#pragma unroll
    for (int q = 0; q < 16; ++q) { mx[q] = kNegBig; sm[q] = 0.f; }
    stream_head_direct(a, qa, tok_base, Lb, g, c0, c1 - c0, stage, lane, [&](int st, const floatx16 &acc) {
      const int tok = c0 + st * kSub + n;
      const bool counted = (tok >= o0 && tok < o1) || (last && tok >= P && tok < Lb);
      const bool scored = tok >= 0 && tok < min(P, c1);  // a prefix token (owned or halo): its probability is formed in phase 3
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int w = hi * 4 + (q & 3);
        const bool ok = counted && (!a.causal || tok <= P + w);
        const float zz = acc[q] * a.scale_log2e;
#pragma unroll
        for (int t = 0; t < kFusedSub; ++t)
          if (t == st) z[t][q] = zz;
        // running reference = max over every logit that is counted or later scored, so that
        // 2^(z - reference) <= 1 for all of them; only counted keys enter the sum.  Masked window
        // keys and clamped slots outside the sequence are neither: they must not move the reference.
        const float zr = (ok || scored) ? zz : kNegBig;
        const float d = zr - mx[q];
        const float e = fast_exp2(-fabsf(d));
        const float one = ok ? 1.f : 0.f;
        sm[q] = d > 0.f ? sm[q] * e + one : sm[q] + one * e;
        mx[q] = fmaxf(mx[q], zr);
      }
    });
    FKV_TICK(33);
    FKV_WTICK(0);
    // fold over the 32 token lanes of each wave half: registers only
    float srow[16];
#pragma unroll
    for (int q = 0; q < 16; ++q) mloc[q] = half_max(mx[q]);
#pragma unroll
    for (int q = 0; q < 16; ++q) srow[q] = half_sum(sm[q] * fast_exp2(mx[q] - mloc[q]));
    // lanes 0-15 post the 16 rows of the low half, lanes 32-47 those of the high half
    float pm = mloc[0], ps = srow[0];
#pragma unroll
    for (int q = 1; q < 16; ++q)
      if ((lane & 15) == q) { pm = mloc[q]; ps = srow[q]; }
    if ((lane & 31) < 16) {
      const int q = lane & 15;
      const int row = g * kRowsPerGroup + (q >> 2) * 8 + hi * 4 + (q & 3);
      box_post(f.part + (size_t)row * kMaxFusedBlocks + blockIdx.x, make_float2(pm, ps));
    }
  }
  FKV_TICK(34);
  FKV_BTICK(1);
  FKV_WTICK(1);

  // ---- phase 2a: owner duty.  Softmax row t = (sequence, row) belongs to block t mod n_wg; a block
  // spreads its rows over its waves.  The owner collects the row's partial from every block of the
  // sequence, folds them and posts the log-sum-exp into each of those blocks' result boxes.
  bool wave_ok = true;
  {
    const int rows_per_seq = a.V * kRowsPerGroup;
    const int n_tasks = a.map.n_seq * rows_per_seq;
    for (int t = (int)blockIdx.x + wave * f.n_wg; t < n_tasks; t += kWaves * f.n_wg) {
      const int tb = t / rows_per_seq, row = t - tb * rows_per_seq;
      const int blk0 = a.map.blk[tb], nb = a.map.blk[tb + 1] - blk0;
      float2 *src = f.part + (size_t)row * kMaxFusedBlocks + blk0;
      const int n_it = (nb + 63) >> 6;
      unsigned long long v[kBoxChunks];
#pragma unroll
      for (int i = 0; i < kBoxChunks; ++i) v[i] = kEmpty64;
      BoundedWait wait(f.timeout_ticks);
      while (true) {
        bool missing = false;
#pragma unroll
        for (int i = 0; i < kBoxChunks; ++i)
          if (i < n_it && i * 64 + lane < nb && v[i] == kEmpty64) v[i] = box_peek(src + i * 64 + lane);
#pragma unroll
        for (int i = 0; i < kBoxChunks; ++i)
          if (i < n_it && i * 64 + lane < nb && v[i] == kEmpty64) missing = true;
        if (!__any(missing)) break;
        if (wait.expired()) { wave_ok = false; break; }
      }
      if (!wave_ok) break;
      float m = kNegBig, s = 0.f;
#pragma unroll
      for (int i = 0; i < kBoxChunks; ++i)
        if (i < n_it && i * 64 + lane < nb) {
          box_clear(src + i * 64 + lane);
          float2 pv;
          __builtin_memcpy(&pv, &v[i], sizeof pv);
          const float mn = fmaxf(m, pv.x);
          s = s * fast_exp2(m - mn) + pv.y * fast_exp2(pv.x - mn);
          m = mn;
        }
      const float mw = wave_fmax(m);
      const float sw = wave_fsum(s * fast_exp2(m - mw));
      const int vg = row >> 5, rr = row & 31;
      const bool row_ok = (rr >> 3) < vg_heads(a, vg) && (rr & 7) < a.W;
      const float lse = row_ok ? mw + __log2f(sw) : 0.f;
#pragma unroll
      for (int i = 0; i < kBoxChunks; ++i)
        if (i < n_it && i * 64 + lane < nb) box_post(f.lse + (size_t)(blk0 + i * 64 + lane) * kLseRowsPerBlock + row, lse);
    }
  }
  FKV_TICK(35);
  FKV_WTICK(2);

  // While the exchange is in flight: turn the kept logits into 2^(z - block reference).  The
  // global normaliser then costs one multiply per value instead of an exponential.
  if (has_group) {
#pragma unroll
    for (int st = 0; st < kFusedSub; ++st)
      if (st < n_sub) {
#pragma unroll
        for (int q = 0; q < 16; ++q) z[st][q] = fast_exp2(z[st][q] - mloc[q]);
      }
  }
  FKV_TICK(36);

  // ---- phase 2b: collect the log-sum-exp of this wave's 32 rows from the block's result box
  if (has_group && wave_ok) {
    float *box = f.lse + (size_t)blockIdx.x * kLseRowsPerBlock + g * kRowsPerGroup + (lane & 31);
    unsigned bits = kEmpty32;
    BoundedWait wait(f.timeout_ticks);
    while (true) {
      if (lane < 32 && bits == kEmpty32) bits = box_peek(box);
      if (!__any(lane < 32 && bits == kEmpty32)) break;
      if (wait.expired()) { wave_ok = false; break; }
    }
    if (wave_ok && lane < 32) {
      box_clear(box);
      cst_lds[wave][lane] = __uint_as_float(bits);
    }
  }
  FKV_BTICK(2);
  FKV_WTICK(3);
  __syncthreads();  // every wave has left its staging tile (phase 3 reuses them); flag_lds is initialised
  if (!wave_ok && lane == 0) flag_lds[0] = 0u;
  FKV_TICK(37);

  // ---- phase 3: probabilities from the kept logits, window sums into LDS
  if (has_group && wave_ok) {
    float fac[16];  // 2^(block reference - global log-sum-exp) per row
#pragma unroll
    for (int q = 0; q < 16; ++q) fac[q] = fast_exp2(mloc[q] - cst_lds[wave][(q >> 2) * 8 + hi * 4 + (q & 3)]);
#pragma unroll
    for (int st = 0; st < kFusedSub; ++st) {
      if (st < n_sub) {
        const int tok = c0 + st * kSub + n;
        const bool inb = tok >= 0 && tok < min(P, c1);  // only prefix tokens are scored; slots past c1 were never loaded
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
  const bool grid_ok = flag_lds[0] != 0u;
  if (grid_ok) {
    pool_and_write<kFusedSlots>(a, s_head, g_sum, c0, o0, o1, col0);
  } else {
    poison_scores(a, col0, o0, o1);
    if (threadIdx.x == 0) __hip_atomic_store(f.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  FKV_TICK(41);
  FKV_BTICK(3);
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
