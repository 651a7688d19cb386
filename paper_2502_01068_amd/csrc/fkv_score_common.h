// Device helpers shared by the score kernels: MFMA operand loads and the K streaming loop.
#pragma once

#include "fkv_internal.h"

namespace fkv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float floatx16;

constexpr int kWaves = 8;            // one wave per KV head
constexpr int kThreads = kWaves * 64;
constexpr int kScoresSubShort = 4;   // k_scores: sub-tiles per block (incl. pooling halo), short inputs
constexpr int kScoresSubLong = 18;   // ... and the most for long inputs (LDS bound)
constexpr int kScoresSubWide = 9;    // ... when more than 8 virtual groups keep their window sums in LDS
constexpr int kSub = 32;             // tokens per MFMA sub-tile
constexpr int kStageBytes = kSub * kHeadDim * 2;  // 8 KiB per wave
constexpr float kNegBig = -1.0e30f;

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

// MFMA A operand for virtual group g: lane (m = lane%32, hi = lane/32) holds, for step s, the 8
// values d = hi*64 + s*8 .. +7 of query row m (head vg_head0(g) + m/8, window row m%8).  The
// contraction index may be permuted freely as long as K uses the same permutation.
template <typename A>
__device__ __forceinline__ void load_q(const A &a, int b, int g, int lane, bf16x8 (&qa)[8]) {
  const int m = lane & 31, hi = lane >> 5;
  const int hl = m >> 3, w = m & 7;
  const bool ok = hl < vg_heads(a, g) && w < a.W;
  const u32x4 *src = reinterpret_cast<const u32x4 *>(
      a.q_win + (((size_t)b * a.W + (ok ? w : 0)) * a.Hq + (size_t)vg_head0(a, g) + (ok ? hl : 0)) * kHeadDim + hi * 64);
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    u32x4 v = src[s];
    if (!ok) v = (u32x4){0u, 0u, 0u, 0u};
    qa[s] = __builtin_bit_cast(bf16x8, v);
  }
}

// Streams the K rows of virtual group g's KV head for `n_sub` consecutive 32-token sub-tiles starting at
// sequence-local token `first` (tokens are clamped into [0, Lb-1] for the load; the caller masks
// what lies outside its range).  fn(st, acc) receives the raw logits of sub-tile st:
// acc[r] = q_row(m) . k(token first + st*32 + lane%32) with m = (r/4)*8 + (lane/32)*4 + r%4,
// i.e. head r/4 of the group and window row (lane/32)*4 + r%4.
// kStreaming marks the loads non-temporal.  Measured at 131072 tokens: both passes of the two-pass
// kernels gain from it together (-6 us per layer), the single-pass kernel does not.
template <bool kStreaming = false, typename F>
__device__ __forceinline__ void stream_head(const ScoreArgs &a, const bf16x8 (&qa)[8], int tok_base, int Lb, int g,
                                            int first, int n_sub, uint8_t *stage, int lane, F fn) {
  const int c = lane & 15;        // 16-byte column of the 256-byte head row
  const int tq = lane >> 4;       // token within a quad of 4 tokens per load instruction
  const int n = lane & 31, hi = lane >> 5;
  const uint16_t *kbase = a.k + (size_t)vg_kv_head(a, g) * kHeadDim + c * 8;
  const size_t tok_stride = (size_t)a.Hkv * kHeadDim;

  u32x4 nxt[8];
  auto issue = [&](int st) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      int t = first + st * kSub + i * 4 + tq;
      t = min(max(t, 0), Lb - 1);
      const u32x4 *src = reinterpret_cast<const u32x4 *>(kbase + (size_t)(tok_base + t) * tok_stride);
      nxt[i] = kStreaming ? __builtin_nontemporal_load(src) : *src;
    }
  };
  issue(0);
#pragma unroll 1
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

// The same stream with the sub-tiles loaded straight from global memory into the wave's LDS tile
// (gfx950's 128-bit LDS-direct loads: lane l of a load instruction lands at tile offset 16 l), so no
// registers hold a tile while the previous one is being consumed.  The XOR swizzle moves to the global
// side: the lane that owns LDS column c' of token slot t fetches the row's column c' ^ (t & 15).
// Per sub-tile: wait for its loads, run the MFMAs off the tile, start the next sub-tile's loads into
// the same (now free) tile, run fn while they are in flight.
// Only the first n_slots token slots (counted from `first`) are loaded: the rest of the last sub-tile
// keeps whatever the LDS tile held, and the caller ignores those tokens' logits (they may be anything,
// NaN included; a token is one MFMA column, so nothing spreads to other tokens).
template <typename F>
__device__ __forceinline__ void stream_head_direct(const ScoreArgs &a, const bf16x8 (&qa)[8], int tok_base, int Lb,
                                                   int g, int first, int n_slots, uint8_t *stage, int lane, F fn) {
  const int n_sub = (n_slots + kSub - 1) / kSub;
  const int c = lane & 15;        // LDS column of this lane within a token slot
  const int tq = lane >> 4;       // token within the quad of 4 tokens one load instruction covers
  const int n = lane & 31, hi = lane >> 5;
  const uint16_t *kbase = a.k + (size_t)vg_kv_head(a, g) * kHeadDim;
  const size_t tok_stride = (size_t)a.Hkv * kHeadDim;
  typedef __attribute__((address_space(1))) const void *gptr_t;
  typedef __attribute__((address_space(3))) void *lptr_t;

  auto issue = [&](int st) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (st * kSub + i * 4 >= n_slots) break;  // wave-uniform: this instruction's 4 tokens are all beyond the range
      const int slot = i * 4 + tq;
      int t = first + st * kSub + slot;
      t = min(max(t, 0), Lb - 1);
      const uint16_t *src = kbase + (size_t)(tok_base + t) * tok_stride + ((c ^ (slot & 15)) << 3);
      __builtin_amdgcn_global_load_lds((gptr_t)src, (lptr_t)(stage + i * 1024), 16, 0, 0);
    }
  };
  issue(0);
#pragma unroll 1
  for (int st = 0; st < n_sub; ++st) {
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the tile has landed in LDS
    wave_lds_sync();
    floatx16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const u32x4 kb = *reinterpret_cast<const u32x4 *>(stage + n * 256 + (((hi * 8 + s) ^ (n & 15)) << 4));
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa[s], __builtin_bit_cast(bf16x8, kb), acc, 0, 0, 0);
    }
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): every lane's operands have left the tile
    wave_lds_sync();
    if (st + 1 < n_sub) issue(st + 1);   // in flight while fn runs
    fn(st, acc);
  }
}

// Folds the per-lane running (max, sum) pairs of a wave's 32 softmax rows over the 32 token
// lanes, through a wave-private LDS transpose (`scratch` >= 4480 bytes, 4-byte aligned).
// In: mx[r], sm[r] of row m = (r/4)*8 + (lane/32)*4 + r%4 for token lane%32.
// Out (every lane; lanes l and l+32 agree): (M, S) of row lane%32, S relative to M.
// On return scratch[32*33 + m] still holds M of row m (kFoldMaxOffset floats into scratch).
// The summation order is fixed, so results are reproducible.
constexpr int kFoldMaxOffset = 32 * 33;
__device__ __forceinline__ float2 fold_rows(const float (&mx)[16], const float (&sm)[16], float *scratch, int lane) {
  const int n = lane & 31, hi = lane >> 5;
  float *T = scratch;             // [32 rows][33]
  float *Mrow = scratch + 32 * 33;
  wave_lds_sync();
#pragma unroll
  for (int r = 0; r < 16; ++r) T[((r >> 2) * 8 + hi * 4 + (r & 3)) * 33 + n] = mx[r];
  wave_lds_sync();
  const int row = lane & 31, half = lane >> 5;
  float M = kNegBig;
#pragma unroll
  for (int j = 0; j < 16; ++j) M = fmaxf(M, T[row * 33 + half * 16 + j]);
  M = fmaxf(M, __shfl_xor(M, 32));
  if (lane < 32) Mrow[row] = M;
  wave_lds_sync();
  float scaled[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) scaled[r] = sm[r] * fast_exp2(mx[r] - Mrow[(r >> 2) * 8 + hi * 4 + (r & 3)]);
#pragma unroll
  for (int r = 0; r < 16; ++r) T[((r >> 2) * 8 + hi * 4 + (r & 3)) * 33 + n] = scaled[r];
  wave_lds_sync();
  float S = 0.f;
#pragma unroll
  for (int j = 0; j < 16; ++j) S += T[row * 33 + half * 16 + j];
  S += __shfl_xor(S, 32);
  return make_float2(M, S);
}

// x(lane) + x(lane ^ 32) in every lane, low half first (one VALU lane swap, no LDS round trip).
__device__ __forceinline__ float add_across_halves(float x) {
  const unsigned u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Merges two (max, sum) pairs of the same softmax row (log2 domain).
__device__ __forceinline__ float2 merge_stats(float2 x, float2 y) {
  const float mn = fmaxf(x.x, y.x);
  return make_float2(mn, x.y * fast_exp2(x.x - mn) + y.y * fast_exp2(y.x - mn));
}

// Pools the per-head window sums along tokens (Eq. 1), averages the heads of each KV group
// (App. B.1) and all heads (Eq. 2) and writes the scores of the owned tokens [o0, o1).
// s_head[4 v + i][slot] holds the window-summed probability of head i of virtual group v at token j0 + slot, 0 outside the
// prefix: neutral for max pooling (scores are >= 0) and the zero padding of avg pooling.
// Slots o0 - r - j0 .. o1 + r - 1 - j0 must be filled.  Contains block barriers.
template <int kStride>
__device__ __forceinline__ void pool_and_write(const ScoreArgs &a, const float (*s_head)[kStride],
                                               float (*g_sum)[kStride], int j0, int o0, int o1, int col0) {
  const int r = a.pool_r;
  const int own = o1 - o0;
  const float inv_k = 1.0f / (float)(2 * r + 1), inv_g = 1.0f / (float)a.G, inv_h = 1.0f / (float)a.Hq;
  const bool is_max = a.pool_mode == FKV_POOL_MAX;
  const int lane = threadIdx.x & 63, n_waves = blockDim.x >> 6;
  const bool split = a.vsh != 0;  // a KV group spans two virtual groups: its mean is formed after the barrier
  for (int g = threadIdx.x >> 6; g < a.V; g += n_waves) {  // one wave per virtual group
    const int n_h = vg_heads(a, g), h0 = vg_head0(a, g);
    if (r == 3) {
      // kernel 7 (the paper's): the 7 taps of all heads of the group are independent LDS reads, in flight together
#pragma unroll 1
      for (int jj = lane; jj < own; jj += 64) {
        const int c = o0 + jj - j0;  // slot of the pooled token
        float p[kMaxGroup];
#pragma unroll
        for (int hl = 0; hl < kMaxGroup; ++hl) {
          const float *row = s_head[g * kMaxGroup + (hl < n_h ? hl : 0)] + c;
          const float v0 = row[-3], v1 = row[-2], v2 = row[-1], v3 = row[0], v4 = row[1], v5 = row[2], v6 = row[3];
          p[hl] = is_max ? fmaxf(fmaxf(fmaxf(v0, v1), fmaxf(v2, v3)), fmaxf(fmaxf(v4, v5), v6))
                         : ((((((v0 + v1) + v2) + v3) + v4) + v5) + v6) * inv_k;
        }
        float gs = 0.f;
#pragma unroll
        for (int hl = 0; hl < kMaxGroup; ++hl)
          if (hl < n_h) {
            if (a.scores_head) a.scores_head[(size_t)(h0 + hl) * a.sum_p + col0 + o0 + jj] = p[hl];
            gs += p[hl];
          }
        g_sum[g][jj] = gs;
        if (a.scores_group && !split) a.scores_group[(size_t)g * a.sum_p + col0 + o0 + jj] = gs * inv_g;
      }
      continue;
    }
#pragma unroll 1
    for (int jj = lane; jj < own; jj += 64) {
      const int c = o0 + jj - j0;  // slot of the pooled token
      float gs = 0.f;
#pragma unroll 1
      for (int hl = 0; hl < n_h; ++hl) {
        const float *row = s_head[g * kMaxGroup + hl] + c;
        float p;
        if (is_max) {
          p = row[0];
          for (int t = -r; t <= r; ++t) p = fmaxf(p, row[t]);
        } else {
          p = 0.f;
          for (int t = -r; t <= r; ++t) p += row[t];
          p *= inv_k;
        }
        if (a.scores_head) a.scores_head[(size_t)(h0 + hl) * a.sum_p + col0 + o0 + jj] = p;
        gs += p;
      }
      g_sum[g][jj] = gs;
      if (a.scores_group && !split) a.scores_group[(size_t)g * a.sum_p + col0 + o0 + jj] = gs * inv_g;
    }
  }
  if (a.scores_tsp == nullptr && !(split && a.scores_group)) return;
  __syncthreads();
  if (split && a.scores_group) {
    for (int i = threadIdx.x; i < own * a.Hkv; i += blockDim.x) {
      const int kv = i / own, jj = i - kv * own;
      a.scores_group[(size_t)kv * a.sum_p + col0 + o0 + jj] = (g_sum[2 * kv][jj] + g_sum[2 * kv + 1][jj]) * inv_g;
    }
  }
  if (a.scores_tsp == nullptr) return;
  for (int jj = threadIdx.x; jj < own; jj += blockDim.x) {
    float tot = 0.f;
    for (int g = 0; g < a.V; ++g) tot += g_sum[g][jj];
    a.scores_tsp[col0 + o0 + jj] = tot * inv_h;
  }
}

}  // namespace fkv
