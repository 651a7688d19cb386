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
#include "fkv_internal.h"

namespace fkv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float floatx16;

constexpr int kWaves = 8;            // one wave per KV head
constexpr int kThreads = kWaves * 64;
constexpr int kStatsChunk = 128;     // tokens per block in k_stats
constexpr int kTile = 128;           // tokens computed per block in k_scores (incl. pooling halo)
constexpr int kSub = 32;             // tokens per MFMA sub-tile
constexpr int kStageBytes = kSub * kHeadDim * 2;  // 8 KiB per wave
constexpr float kNegBig = -1.0e30f;

int stats_chunk_tokens(void) { return kStatsChunk; }
int scores_tile_out(int pool_r) { return kTile - 2 * pool_r; }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ int find_seq(const SeqMap &map, int block) {
  int b = 0;
  while (b + 1 < map.n_seq && block >= map.blk[b + 1]) ++b;
  return b;
}

// Orders this wave's LDS traffic (writes of one layout, reads of another) without a block barrier.
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// MFMA A operand for KV group g: lane (m = lane%32, hi = lane/32) holds, for step s, the 8
// values d = hi*64 + s*8 .. +7 of query row m (head g*G + m/8, window row m%8).  The
// contraction index may be permuted freely as long as K uses the same permutation.
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

// Streams the K rows of one KV head for `n_sub` consecutive 32-token sub-tiles starting at
// sequence-local token `first` (tokens are clamped into [0, Lb-1] for the load; the caller masks
// what lies outside its range).  fn(st, acc) receives the raw logits of sub-tile st:
// acc[r] = q_row(m) . k(token first + st*32 + lane%32) with m = (r/4)*8 + (lane/32)*4 + r%4,
// i.e. head r/4 of the group and window row (lane/32)*4 + r%4.
template <typename F>
__device__ __forceinline__ void stream_head(const ScoreArgs &a, const bf16x8 (&qa)[8], int tok_base, int Lb, int g,
                                            int first, int n_sub, uint8_t *stage, int lane, F fn) {
  const int c = lane & 15;        // 16-byte column of the 256-byte head row
  const int tq = lane >> 4;       // token within a quad of 4 tokens per load instruction
  const int n = lane & 31, hi = lane >> 5;
  const uint16_t *kbase = a.k + (size_t)g * kHeadDim + c * 8;
  const size_t tok_stride = (size_t)a.Hkv * kHeadDim;

  u32x4 nxt[8];
  auto issue = [&](int st) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      int t = first + st * kSub + i * 4 + tq;
      t = min(max(t, 0), Lb - 1);
      nxt[i] = *reinterpret_cast<const u32x4 *>(kbase + (size_t)(tok_base + t) * tok_stride);
    }
  };
  issue(0);
  for (int st = 0; st < n_sub; ++st) {
    wave_lds_sync();  // previous sub-tile's reads are done before the tile is overwritten
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int t = i * 4 + tq;  // token slot in the tile
      *reinterpret_cast<u32x4 *>(stage + t * 256 + ((c ^ (t & 15)) << 4)) = nxt[i];
    }
    if (st + 1 < n_sub) issue(st + 1);
    wave_lds_sync();
    floatx16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const u32x4 kb = *reinterpret_cast<const u32x4 *>(stage + n * 256 + (((hi * 8 + s) ^ (n & 15)) << 4));
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa[s], __builtin_bit_cast(bf16x8, kb), acc, 0, 0, 0);
    }
    fn(st, acc);
  }
}

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

  for (int g = wave; g < a.Hkv; g += kWaves) {
    bf16x8 qa[8];
    load_q(a, b, g, lane, qa);
    float mx[16], sm[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) { mx[r] = kNegBig; sm[r] = 0.f; }

    stream_head(a, qa, tok_base, Lb, g, t0, n_sub, stage, lane, [&](int st, const floatx16 &acc) {
      const int tok = t0 + st * kSub + n;
      const bool valid = tok < t1;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int w = hi * 4 + (r & 3);
        const bool ok = valid && (!a.causal || tok <= P + w);
        const float z = ok ? acc[r] * a.scale_log2e : kNegBig;
        const float mn = fmaxf(mx[r], z);
        sm[r] = sm[r] * fast_exp2(mx[r] - mn) + (ok ? fast_exp2(z - mn) : 0.f);
        mx[r] = mn;
      }
    });
    // fold the 32 lanes that share `hi` (fixed butterfly order: deterministic)
    float2 *dst = a.partial + (size_t)(g * kRowsPerGroup) * a.partial_stride + blockIdx.x;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float M = mx[r];
#pragma unroll
      for (int off = 1; off < 32; off <<= 1) M = fmaxf(M, __shfl_xor(M, off));
      float S = sm[r] * fast_exp2(mx[r] - M);
#pragma unroll
      for (int off = 1; off < 32; off <<= 1) S += __shfl_xor(S, off);
      if (n == 0) dst[(size_t)((r >> 2) * 8 + hi * 4 + (r & 3)) * a.partial_stride] = make_float2(M, S);
    }
  }
}

// One wave per softmax row: grid.x = ceil(B*Hkv*32 / 4), 256 threads.  Lane l folds partials
// l, l+64, ... in order, then the 64 lanes are folded by a fixed butterfly.
__global__ __launch_bounds__(256) void k_combine(ScoreArgs a) {
  const int lane = threadIdx.x & 63;
  const int rid = blockIdx.x * 4 + (threadIdx.x >> 6);  // (b, g, m)
  const int rows_per_seq = a.Hkv * kRowsPerGroup;
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
    const bool ok = (row >> 3) < a.G && (row & 7) < a.W;
    // probability = exp2(z*scale*log2e - (Mx + log2 S))
    a.rowstat[(size_t)b * rows_per_seq + gm] = ok ? (Mx + __log2f(S)) : 0.f;
  }
}

__global__ __launch_bounds__(kThreads) void k_scores(ScoreArgs a) {
  // The staging tiles are dead once every wave has left its K loop; the per-head window sums
  // then reuse the same LDS.
  __shared__ __attribute__((aligned(16))) uint8_t lds_all[kWaves * kStageBytes];
  float(*s_head)[kTile] = reinterpret_cast<float(*)[kTile]>(lds_all);  // [Hkv*4][kTile]
  float(*g_sum)[kTile] = reinterpret_cast<float(*)[kTile]>(lds_all + kMaxKvHeads * kMaxGroup * kTile * 4);
  static_assert((kMaxKvHeads * kMaxGroup + kMaxKvHeads) * kTile * 4 <= kWaves * kStageBytes, "LDS reuse");

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 31, hi = lane >> 5;
  const int b = find_seq(a.map, blockIdx.x);
  const int tok_base = a.map.cu[b];
  const int Lb = a.map.cu[b + 1] - tok_base;
  const int P = Lb - a.W;
  const int r = a.pool_r;
  const int tout = kTile - 2 * r;
  const int j0 = ((int)blockIdx.x - a.map.blk[b]) * tout - r;  // first computed token (may be < 0)
  uint8_t *stage = lds_all + wave * kStageBytes;
  constexpr int kNSub = kTile / kSub;

  // window-summed probabilities of this wave's group: hsum[st][hl] for token j0 + st*32 + n
  float hsum[kNSub][4];
  int g_mine = -1;
  for (int g = wave; g < a.Hkv; g += kWaves) {  // Hkv <= kWaves: at most one group per wave
    g_mine = g;
    bf16x8 qa[8];
    load_q(a, b, g, lane, qa);
    float cst[16];
    const float *rs = a.rowstat + ((size_t)b * a.Hkv + g) * kRowsPerGroup;
#pragma unroll
    for (int q = 0; q < 16; ++q) cst[q] = rs[(q >> 2) * 8 + hi * 4 + (q & 3)];

    stream_head(a, qa, tok_base, Lb, g, j0, kNSub, stage, lane, [&](int st, const floatx16 &acc) {
#pragma unroll
      for (int hl = 0; hl < 4; ++hl) {
        float sum = 0.f;
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
          const float e = fast_exp2(acc[hl * 4 + rr] * a.scale_log2e - cst[hl * 4 + rr]);
          sum += (hi * 4 + rr < a.W) ? e : 0.f;
        }
        sum += __shfl_xor(sum, 32);  // other half of the window rows
#pragma unroll
        for (int q = 0; q < kNSub; ++q)
          if (q == st) hsum[q][hl] = sum;
      }
    });
  }
  __syncthreads();
  if (g_mine >= 0 && hi == 0) {
#pragma unroll
    for (int st = 0; st < kNSub; ++st) {
      const int tok = j0 + st * kSub + n;
      const bool inb = tok >= 0 && tok < P;  // only prefix tokens are scored
#pragma unroll
      for (int hl = 0; hl < 4; ++hl)
        if (hl < a.G) s_head[g_mine * kMaxGroup + hl][st * kSub + n] = inb ? hsum[st][hl] : 0.f;
    }
  }
  __syncthreads();

  // Pool each head over the token axis (Eq. 1), then mean over the group's heads (App. B.1).
  // Taps outside [0,P) hold 0: neutral for max (scores are >= 0) and the zero padding of avg.
  const int col0 = tok_base - b * a.W;  // column of this sequence's token 0 in the score rows
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
  const int rows = a.map.n_seq * a.Hkv * kRowsPerGroup;
  hipLaunchKernelGGL(k_combine, dim3((rows + 3) / 4), dim3(256), 0, s, a);
  return hipGetLastError();
}
hipError_t launch_scores(const ScoreArgs &a, int n_blocks, hipStream_t s) {
  hipLaunchKernelGGL(k_scores, dim3(n_blocks), dim3(kThreads), 0, s, a);
  return hipGetLastError();
}

}  // namespace fkv
