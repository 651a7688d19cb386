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
#include "fkv_internal.h"

namespace fkv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float floatx16;

constexpr int kWaves = 8;            // one wave per KV head
constexpr int kThreads = kWaves * 64;
constexpr int kStatsChunk = 128;     // tokens per block in k_stats
constexpr int kTile = 128;           // tokens computed per block in k_scores (incl. pooling halo)
constexpr float kNegBig = -1.0e30f;

int stats_chunk_tokens(void) { return kStatsChunk; }
int scores_tile_out(int pool_r) { return kTile - 2 * pool_r; }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ int find_seq(const SeqMap &map, int block) {
  int b = 0;
  while (b + 1 < map.n_seq && block >= map.blk[b + 1]) ++b;
  return b;
}

// MFMA A operand for KV group g: lane (m = lane%32, hi = lane/32) holds, for step s, the 8
// values d = hi*64 + s*8 .. +7 of query row m (head g*G + m/8, window row m%8).  The
// contraction index may be permuted freely as long as K uses the same permutation; this one
// lets each lane read 128 contiguous bytes of a key row.
__device__ __forceinline__ void load_q(const ScoreArgs &a, int b, int g, int lane, bf16x8 (&qa)[8]) {
  const int m = lane & 31, hi = lane >> 5;
  const int hl = m >> 3, w = m & 7;
  const bool ok = hl < a.G && w < a.W;
  const u32x4 *src = reinterpret_cast<const u32x4 *>(
      a.q_win + (((size_t)b * a.W + (ok ? w : 0)) * a.Hq + (size_t)g * a.G + (ok ? hl : 0)) * kHeadDim + hi * 64);
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    u32x4 v = src[s];
    if (!ok) v = (u32x4){0u, 0u, 0u, 0u};
    qa[s] = __builtin_bit_cast(bf16x8, v);
  }
}

// Raw logits (before scale) of 32 tokens x 32 rows.  Lane (n = lane%32, hi) supplies token
// row `krow` (already offset to this lane's 128-byte half).  Result: acc[r] is row
// m = (r/4)*8 + hi*4 + r%4 (head r/4, window row hi*4 + r%4) of token n.
__device__ __forceinline__ floatx16 logits_tile(const bf16x8 (&qa)[8], const u32x4 *krow) {
  u32x4 kb[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) kb[s] = krow[s];
  floatx16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int s = 0; s < 8; ++s)
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa[s], __builtin_bit_cast(bf16x8, kb[s]), acc, 0, 0, 0);
  return acc;
}

__global__ __launch_bounds__(kThreads) void k_stats(ScoreArgs a) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 31, hi = lane >> 5;
  const int b = find_seq(a.map, blockIdx.x);
  const int tok_base = a.map.cu[b];
  const int Lb = a.map.cu[b + 1] - tok_base;
  const int P = Lb - a.W;
  const int t0 = ((int)blockIdx.x - a.map.blk[b]) * a.chunk;
  const int t1 = min(Lb, t0 + a.chunk);

  for (int g = wave; g < a.Hkv; g += kWaves) {
    bf16x8 qa[8];
    load_q(a, b, g, lane, qa);
    float mx[16], sm[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) { mx[r] = kNegBig; sm[r] = 0.f; }

    for (int tb = t0; tb < t1; tb += 32) {
      const int tok = tb + n;
      const bool valid = tok < t1;
      const int tl = valid ? tok : (t1 - 1);
      const u32x4 *krow = reinterpret_cast<const u32x4 *>(
          a.k + ((size_t)(tok_base + tl) * a.Hkv + g) * kHeadDim + hi * 64);
      const floatx16 acc = logits_tile(qa, krow);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int w = hi * 4 + (r & 3);
        const bool ok = valid && (!a.causal || tok <= P + w);
        const float z = ok ? acc[r] * a.scale_log2e : kNegBig;
        const float mn = fmaxf(mx[r], z);
        sm[r] = sm[r] * fast_exp2(mx[r] - mn) + (ok ? fast_exp2(z - mn) : 0.f);
        mx[r] = mn;
      }
    }
    // fold the 32 lanes that share `hi` (fixed butterfly order: deterministic)
    float2 *dst = a.partial + (size_t)blockIdx.x * (a.Hkv * kRowsPerGroup) + g * kRowsPerGroup;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float M = mx[r];
#pragma unroll
      for (int off = 1; off < 32; off <<= 1) M = fmaxf(M, __shfl_xor(M, off));
      float S = sm[r] * fast_exp2(mx[r] - M);
#pragma unroll
      for (int off = 1; off < 32; off <<= 1) S += __shfl_xor(S, off);
      if (n == 0) dst[(r >> 2) * 8 + hi * 4 + (r & 3)] = make_float2(M, S);
    }
  }
}

// grid = (Hkv, B); 256 threads: row = tid % 32, slice = tid / 32.  Partials are folded in
// block order within a slice, then slices in order.
__global__ __launch_bounds__(256) void k_combine(ScoreArgs a) {
  __shared__ float2 part[8][kRowsPerGroup];
  const int g = blockIdx.x, b = blockIdx.y;
  const int row = threadIdx.x & 31, slice = threadIdx.x >> 5;
  const int p0 = a.map.blk[b], p1 = a.map.blk[b + 1];
  float M = kNegBig, S = 0.f;
  for (int p = p0 + slice; p < p1; p += 8) {
    const float2 v = a.partial[(size_t)p * (a.Hkv * kRowsPerGroup) + g * kRowsPerGroup + row];
    const float mn = fmaxf(M, v.x);
    S = S * fast_exp2(M - mn) + v.y * fast_exp2(v.x - mn);
    M = mn;
  }
  part[slice][row] = make_float2(M, S);
  __syncthreads();
  if (slice == 0) {
    for (int sl = 1; sl < 8; ++sl) {
      const float2 v = part[sl][row];
      const float mn = fmaxf(M, v.x);
      S = S * fast_exp2(M - mn) + v.y * fast_exp2(v.x - mn);
      M = mn;
    }
    const bool ok = (row >> 3) < a.G && (row & 7) < a.W;
    // probability = exp2(z*scale*log2e - (M + log2 S))
    a.rowstat[((size_t)b * a.Hkv + g) * kRowsPerGroup + row] = ok ? (M + __log2f(S)) : 0.f;
  }
}

__global__ __launch_bounds__(kThreads) void k_scores(ScoreArgs a) {
  __shared__ float s_head[kMaxKvHeads * kMaxGroup][kTile];  // window-summed probabilities per head
  __shared__ float g_sum[kMaxKvHeads][kTile];               // per-group sums of pooled head scores
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 31, hi = lane >> 5;
  const int b = find_seq(a.map, blockIdx.x);
  const int tok_base = a.map.cu[b];
  const int Lb = a.map.cu[b + 1] - tok_base;
  const int P = Lb - a.W;
  const int r = a.pool_r;
  const int tout = kTile - 2 * r;
  const int j0 = ((int)blockIdx.x - a.map.blk[b]) * tout - r;  // first computed token (may be < 0)

  for (int g = wave; g < a.Hkv; g += kWaves) {
    bf16x8 qa[8];
    load_q(a, b, g, lane, qa);
    float cst[16];
    const float *rs = a.rowstat + ((size_t)b * a.Hkv + g) * kRowsPerGroup;
#pragma unroll
    for (int q = 0; q < 16; ++q) cst[q] = rs[(q >> 2) * 8 + hi * 4 + (q & 3)];

#pragma unroll 2
    for (int st = 0; st < kTile / 32; ++st) {
      const int tok = j0 + st * 32 + n;
      const bool inb = tok >= 0 && tok < P;  // only prefix tokens are scored
      const int tl = min(max(tok, 0), Lb - 1);
      const u32x4 *krow = reinterpret_cast<const u32x4 *>(
          a.k + ((size_t)(tok_base + tl) * a.Hkv + g) * kHeadDim + hi * 64);
      const floatx16 acc = logits_tile(qa, krow);
#pragma unroll
      for (int hl = 0; hl < 4; ++hl) {
        float sum = 0.f;
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
          const float e = fast_exp2(acc[hl * 4 + rr] * a.scale_log2e - cst[hl * 4 + rr]);
          sum += (hi * 4 + rr < a.W) ? e : 0.f;
        }
        sum += __shfl_xor(sum, 32);  // other half of the window rows
        if (hi == 0 && hl < a.G) s_head[g * kMaxGroup + hl][st * 32 + n] = inb ? sum : 0.f;
      }
    }
  }
  __syncthreads();

  // Pool each head over the token axis (Eq. 1), then mean over the group's heads (App. B.1).
  // Taps outside [0,P) hold 0: neutral for max (scores are >= 0) and the zero padding of avg.
  const int col0 = tok_base - b * a.W;  // column of this sequence's token 0 in the score rows
  const float inv_k = 1.0f / (float)(2 * r + 1);
  (void)inv_k;
  for (int i = threadIdx.x; i < tout * a.Hkv; i += kThreads) {
    const int g = i / tout, jj = i - g * tout;
    const int c = jj + r;
    float gs = 0.f;
    for (int hl = 0; hl < a.G; ++hl) {
      const float *row = s_head[g * kMaxGroup + hl];
      float p;
      if (a.pool_mode == FKV_POOL_MAX) {
        p = row[c];
        for (int t = -r; t <= r; ++t) p = fmaxf(p, row[c + t]);
      } else {
        p = 0.f;
        for (int t = -r; t <= r; ++t) p += row[c + t];
        p = p / (float)(2 * r + 1);
      }
      gs += p;
    }
    g_sum[g][jj] = gs;
    const int j = j0 + c;
    if (j < P) a.scores_group[(size_t)g * a.sum_p + col0 + j] = gs / (float)a.G;
  }
  if (a.scores_tsp == nullptr) return;
  __syncthreads();
  for (int jj = threadIdx.x; jj < tout; jj += kThreads) {
    const int j = j0 + r + jj;
    if (j >= P) break;
    float tot = 0.f;
    for (int g = 0; g < a.Hkv; ++g) tot += g_sum[g][jj];
    a.scores_tsp[col0 + j] = tot / (float)a.Hq;  // Eq. 2
  }
}

hipError_t launch_stats(const ScoreArgs &a, int n_blocks, hipStream_t s) {
  hipLaunchKernelGGL(k_stats, dim3(n_blocks), dim3(kThreads), 0, s, a);
  return hipGetLastError();
}
hipError_t launch_combine(const ScoreArgs &a, hipStream_t s) {
  hipLaunchKernelGGL(k_combine, dim3(a.Hkv, a.map.n_seq), dim3(256), 0, s, a);
  return hipGetLastError();
}
hipError_t launch_scores(const ScoreArgs &a, int n_blocks, hipStream_t s) {
  hipLaunchKernelGGL(k_scores, dim3(n_blocks), dim3(kThreads), 0, s, a);
  return hipGetLastError();
}

}  // namespace fkv
