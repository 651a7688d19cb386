// Window-attention saliency scores (Sec. 4.2 Eq. 1-2, App. B.1) for gfx950.
//
// Three launches, K streamed twice (the softmax normaliser of each of the Hq*W window rows
// depends on every key, so the rows' log-sum-exp must exist before any score does):
//   k_stats    one pass over K: per block, running (max, sum) of every softmax row
//   k_combine  folds the per-block partials into one log2-domain normaliser per row
//   k_scores   second pass over K: probabilities, window sum, per-head pooling in LDS,
//              group mean and all-head mean, written once
//
// The logits of one KV group are a [32 x 128] x [128 x 32 tokens] product: the 32 rows are
// the G<=4 heads of the group times the W<=8 window queries, exactly one 32x32x16 bf16 MFMA
// tile in M.  Tokens sit on the MFMA N axis, i.e. on lanes, so the per-row softmax statistics
// stay in registers per lane and are only reduced across lanes once per block.
//
// K path: one wave per KV head.  A wave reads its head's 32 x 256 B sub-tile with fully
// coalesced 128-bit loads (16 lanes cover one token's 256-byte row), parks it in a private
// 8 KiB LDS tile with an XOR swizzle on the 16-byte column, and reads it back in the MFMA
// operand layout (lane = token).  The next sub-tile's global loads are issued before the
// current one is consumed.
#include "fkv_score_common.h"

namespace fkv {

int stats_chunk_tokens(void) { return kStatsChunk; }
int scores_sub_short(void) { return kScoresSubShort; }
int scores_sub_long(void) { return kScoresSubLong; }
int scores_sub_wide(void) { return kScoresSubWide; }

__global__ __launch_bounds__(kThreads) void k_stats(ScoreArgs a) {
  __shared__ __attribute__((aligned(16))) uint8_t stage_all[kWaves * kStageBytes];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 31, hi = lane >> 5;
  const int b = find_seq(a.map, blockIdx.x);
  const int tok_base = a.map.cu[b];
  const int Lb = a.map.cu[b + 1] - tok_base;
  const int P = Lb - a.W;
  const int t0 = ((int)blockIdx.x - a.map.blk[b]) * a.chunk;
  const int t1 = min(Lb, t0 + a.chunk);
  const int n_sub = (t1 - t0 + kSub - 1) / kSub;
  uint8_t *stage = stage_all + wave * kStageBytes;

  FKV_TICK(16);
  for (int g = wave; g < a.V; g += kWaves) {
    bf16x8 qa[8];
    load_q(a, b, g, lane, qa);
    float mx[16], sm[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) { mx[r] = kNegBig; sm[r] = 0.f; }

    stream_head<true>(a, qa, tok_base, Lb, g, t0, n_sub, stage, lane, [&](int st, const floatx16 &acc) {
      const int tok = t0 + st * kSub + n;
      const bool valid = tok < t1;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int w = hi * 4 + (r & 3);
        const bool ok = valid && (!a.causal || tok <= P + w);
        // online softmax with one exponential per element: e = 2^-|z - max|
        const float z = ok ? acc[r] * a.scale_log2e : kNegBig;
        const float d = z - mx[r];
        const float e = fast_exp2(-fabsf(d));
        sm[r] = d > 0.f ? sm[r] * e + 1.f : sm[r] + (ok ? e : 0.f);
        mx[r] = fmaxf(mx[r], z);
      }
    });
    FKV_TICK(17);
    const float2 ms = fold_rows(mx, sm, reinterpret_cast<float *>(stage), lane);
    if (lane < 32)
      a.partial[(size_t)(g * kRowsPerGroup + lane) * a.partial_stride + blockIdx.x] = ms;
    FKV_TICK(18);
  }
}

// One wave per softmax row: grid.x = ceil(B*Hkv*32 / 4), 256 threads.  Lane l folds partials
// l, l+64, ... in order, then the 64 lanes are folded by a fixed butterfly.
__global__ __launch_bounds__(256) void k_combine(ScoreArgs a) {
  const int lane = threadIdx.x & 63;
  const int rid = blockIdx.x * 4 + (threadIdx.x >> 6);  // (b, g, m)
  const int rows_per_seq = a.V * kRowsPerGroup;
  if (rid >= a.map.n_seq * rows_per_seq) return;
  const int b = rid / rows_per_seq, gm = rid - b * rows_per_seq;
  const int p0 = a.map.blk[b], p1 = a.map.blk[b + 1];
  const float2 *src = a.partial + (size_t)gm * a.partial_stride;
  float M = kNegBig, S = 0.f;
  for (int p = p0 + lane; p < p1; p += 64) {
    const float2 v = src[p];
    const float mn = fmaxf(M, v.x);
    S = S * fast_exp2(M - mn) + v.y * fast_exp2(v.x - mn);
    M = mn;
  }
  float Mx = M;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) Mx = fmaxf(Mx, __shfl_xor(Mx, off));
  S *= fast_exp2(M - Mx);
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) S += __shfl_xor(S, off);
  if (lane == 0) {
    const int row = gm & 31;
    const bool ok = (row >> 3) < vg_heads(a, gm >> 5) && (row & 7) < a.W;
    // probability = exp2(z*scale*log2e - (Mx + log2 S))
    a.rowstat[(size_t)b * rows_per_seq + gm] = ok ? (Mx + __log2f(S)) : 0.f;
  }
}

// kMaxSub 32-token sub-tiles per block at most; a.tile_sub of them are used (host-chosen so that
// the launch is about one block per CU).  The window sums go straight into their own LDS array,
// next to the waves' staging tiles.
template <int kMaxSub, int kGroups, bool kStreaming = true>
__global__ __launch_bounds__(kThreads) void k_scores(ScoreArgs a) {
  constexpr int kSlots = kMaxSub * kSub;
  __shared__ __attribute__((aligned(16))) uint8_t stage_all[kWaves * kStageBytes];
  __shared__ float s_head[kGroups * kMaxGroup][kSlots];  // window-summed probabilities per head
  __shared__ float g_sum[kGroups][kSlots];               // per virtual group sums of pooled head scores

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 31, hi = lane >> 5;
  const int b = find_seq(a.map, blockIdx.x);
  const int tok_base = a.map.cu[b];
  const int Lb = a.map.cu[b + 1] - tok_base;
  const int P = Lb - a.W;
  const int r = a.pool_r;
  const int n_sub = a.tile_sub;
  const int tout = n_sub * kSub - 2 * r;
  const int j0 = ((int)blockIdx.x - a.map.blk[b]) * tout - r;  // first computed token (may be < 0)
  uint8_t *stage = stage_all + wave * kStageBytes;

  FKV_TICK(24);
  for (int g = wave; g < a.V; g += kWaves) {
    bf16x8 qa[8];
    load_q(a, b, g, lane, qa);
    float cst[16];
    const float *rs = a.rowstat + ((size_t)b * a.V + g) * kRowsPerGroup;
#pragma unroll
    for (int q = 0; q < 16; ++q) cst[q] = rs[(q >> 2) * 8 + hi * 4 + (q & 3)];

    stream_head<kStreaming>(a, qa, tok_base, Lb, g, j0, n_sub, stage, lane, [&](int st, const floatx16 &acc) {
      const int tok = j0 + st * kSub + n;
      const bool inb = tok >= 0 && tok < P;  // only prefix tokens are scored
#pragma unroll
      for (int hl = 0; hl < 4; ++hl) {
        float sum = 0.f;
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
          const float e = fast_exp2(acc[hl * 4 + rr] * a.scale_log2e - cst[hl * 4 + rr]);
          sum += (hi * 4 + rr < a.W) ? e : 0.f;
        }
        sum = add_across_halves(sum);  // other half of the window rows
        if (hi == 0 && hl < vg_heads(a, g)) s_head[g * kMaxGroup + hl][st * kSub + n] = inb ? sum : 0.f;
      }
    });
  }
  FKV_TICK(25);
  __syncthreads();
  FKV_TICK(26);

  const int col0 = tok_base - b * a.W;  // column of this sequence's token 0 in the score rows
  pool_and_write<kSlots>(a, s_head, g_sum, j0, j0 + r, min(j0 + r + tout, P), col0);
  FKV_TICK(27);
}

hipError_t launch_stats(const ScoreArgs &a, int n_blocks, hipStream_t s) {
  hipLaunchKernelGGL(k_stats, dim3(n_blocks), dim3(kThreads), 0, s, a);
  return hipGetLastError();
}
hipError_t launch_combine(const ScoreArgs &a, hipStream_t s) {
  const int rows = a.map.n_seq * a.V * kRowsPerGroup;
  hipLaunchKernelGGL(k_combine, dim3((rows + 3) / 4), dim3(256), 0, s, a);
  return hipGetLastError();
}
hipError_t launch_scores(const ScoreArgs &a, int n_blocks, hipStream_t s) {
  if (a.V > kMaxKvHeads)  // twice the heads in LDS: half the tile
    hipLaunchKernelGGL((k_scores<kScoresSubWide, kMaxVGroups>), dim3(n_blocks), dim3(kThreads), 0, s, a);
  else if (a.tile_sub <= kScoresSubShort && !a.k_cached)
    hipLaunchKernelGGL((k_scores<kScoresSubShort, kMaxKvHeads>), dim3(n_blocks), dim3(kThreads), 0, s, a);
  else if (!a.k_cached)
    hipLaunchKernelGGL((k_scores<kScoresSubLong, kMaxKvHeads>), dim3(n_blocks), dim3(kThreads), 0, s, a);
  else  // K was just read by the launch before: plain loads, so that what the caches still hold is used
    hipLaunchKernelGGL((k_scores<kScoresSubLong, kMaxKvHeads, false>), dim3(n_blocks), dim3(kThreads), 0, s, a);
  return hipGetLastError();
}

}  // namespace fkv
