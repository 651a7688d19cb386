// Attention output of the observation-window rows: out[w][h] = sum_j Att[h, P+w, j] * V[j, g(h)], with
// the probabilities Att of Eq. 1 (Sec. 4.2).  The layer's fused attention kernel does not hand these
// probabilities out (Sec. 5.1), so the estimation step forms them itself; forming the window rows'
// output from them here lets the layer skip those rows.
//
// One wave works on 32-token tiles of one (sequence, virtual group): both contractions run on the
// matrix cores with the 32 softmax rows (4 heads x 8 window rows) of the group on the N side.
//   S^T = K . Q^T : A operand = K rows of the tile (token on the lane), B operand = Q rows.  The
//     result leaves softmax row n = lane % 32 on the lane and 16 tokens of the tile in its
//     registers, so the running maximum, the exponentials and the rescale factor are per-lane
//     scalars (two lanes share a row and meet once per tile).
//   O^T += V^T . P : B operand = the probabilities exactly as the first contraction left them
//     (the token order inside the contraction may be permuted freely as long as V uses the same
//     order); A operand = V transposed through the LDS tile: the lane reads the 8 bytes
//     d = 4m .. 4m+3 of each of its 8 tokens and feeds one 16-bit piece to each of the four
//     32-row output tiles, whose row m therefore stands for d = 4m + tile.
// The probabilities enter the second contraction as a bf16 pair (rounded value + remainder), which
// keeps 16 bits of them; fp32 accumulation throughout.
// K and V tiles go straight from global memory into the wave's two 8 KiB LDS tiles (128-bit
// LDS-direct loads); a tile's next load is issued as soon as its operands sit in registers.
// Tokens are split over blocks (8 waves each); a block merges its waves' running states through
// LDS and leaves one partial (max, sum, 32 x 128 accumulator) per (sequence, group, split); a second
// launch folds the splits in a fixed order.
#include "fkv_score_common.h"

namespace fkv {

constexpr int kWoWaves = 8;
constexpr int kWoThreads = kWoWaves * 64;
constexpr int kWoTileBytes = 2 * kStageBytes;       // K tile + V tile per wave
constexpr int kWoRowFloats = kRowsPerGroup * kHeadDim;  // 4096 accumulator values per partial
constexpr float kWoEmpty = -5.0e29f;                // running maximum before any visible key (> masked logits)

int wout_tiles_per_block_min(void) { return kWoWaves; }

__device__ __forceinline__ float max_across_halves(float x) {
  const unsigned u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

template <bool kKeepK>
__global__ __launch_bounds__(kWoThreads) void k_wout_partial(WoutArgs a) {
  __shared__ __attribute__((aligned(16))) uint8_t lds_all[kWoWaves * kWoTileBytes];
  __shared__ float2 ms_lds[kWoWaves][kRowsPerGroup];
  typedef __attribute__((address_space(1))) const void *gptr_t;
  typedef __attribute__((address_space(3))) void *lptr_t;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 31, hi = lane >> 5;
  const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
  const int tok_base = a.cu[b];
  const int Lb = a.cu[b + 1] - tok_base;
  const int P = Lb - a.W;
  const int n_tiles = (Lb + kSub - 1) / kSub;
  const int per = (n_tiles + a.n_split - 1) / a.n_split;
  const int t0 = split * per, t1 = min(n_tiles, t0 + per);
  uint8_t *ktile = lds_all + wave * kWoTileBytes, *vtile = ktile + kStageBytes;

  const int blk_id = (blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x;  // timing builds only
  (void)blk_id;
  FKV_BTICK_AT(blk_id, 0);
  bf16x8 qa[8];
  load_q(a, b, g, lane, qa);

  // direct-to-LDS tile loads: lane l of load i lands at tile offset i*1024 + 16 l, i.e. token slot
  // 4 i + l/16, 16-byte column l%16.  The K tile is XOR-swizzled (from the global side), V is plain.
  // Both streams are read once: the loads are marked non-temporal (measured 34.3 instead of 38.6 us per call at
  // 32768 tokens), except K when the caller reads it again right after this launch (kKeepK).
  const int c = lane & 15, tq = lane >> 4;
  const size_t tok_stride = (size_t)a.Hkv * kHeadDim;
  const uint16_t *kbase = a.k + (size_t)vg_kv_head(a, g) * kHeadDim;
  const uint16_t *vbase = a.v + (size_t)vg_kv_head(a, g) * kHeadDim + c * 8;
  auto issue_k = [&](int tile) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int slot = i * 4 + tq;
      const int t = min(tile * kSub + slot, Lb - 1);
      const uint16_t *src = kbase + (size_t)(tok_base + t) * tok_stride + ((c ^ (slot & 15)) << 3);
      __builtin_amdgcn_global_load_lds((gptr_t)src, (lptr_t)(ktile + i * 1024), 16, 0, kKeepK ? 0 : 2);
    }
  };
  auto issue_v = [&](int tile) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int t = min(tile * kSub + i * 4 + tq, Lb - 1);
      const uint16_t *src = vbase + (size_t)(tok_base + t) * tok_stride;
      __builtin_amdgcn_global_load_lds((gptr_t)src, (lptr_t)(vtile + i * 1024), 16, 0, 2);
    }
  };

  floatx16 o[4];
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int q = 0; q < 16; ++q) o[t][q] = 0.f;
  float m = kWoEmpty, s = 0.f;
  const int vis_last = a.causal ? P + (n & 7) : Lb - 1;  // last key softmax row n may see

  int tile = t0 + wave;
  if (tile < t1) {
    issue_k(tile);
    issue_v(tile);
  }
#pragma unroll 1
  for (; tile < t1; tile += kWoWaves) {
    const bool more = tile + kWoWaves < t1;
    __builtin_amdgcn_s_waitcnt(0x0F78);  // vmcnt(8): the K tile has landed (V may still be on its way)
    wave_lds_sync();
    u32x4 kb[8];
#pragma unroll
    for (int s8 = 0; s8 < 8; ++s8)
      kb[s8] = *reinterpret_cast<const u32x4 *>(ktile + n * 256 + (((hi * 8 + s8) ^ (n & 15)) << 4));
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
    wave_lds_sync();
    if (more) issue_k(tile + kWoWaves);
    floatx16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s8 = 0; s8 < 8; ++s8)
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kb[s8]), qa[s8], acc, 0, 0, 0);

    // acc[q] = logit of softmax row n and token slot 8*(q/4) + 4*hi + q%4 of the tile
    const int tok0 = tile * kSub;
    const bool edge = tok0 + kSub - 1 > (a.causal ? P : Lb - 1);  // some (row, token) pair of the tile is masked
    float z[16];
    float tmax = kNegBig;
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const int tok = tok0 + 8 * (q >> 2) + 4 * hi + (q & 3);
      z[q] = acc[q] * a.scale_log2e;
      if (edge && tok > vis_last) z[q] = kNegBig;
      tmax = fmaxf(tmax, z[q]);
    }
    tmax = max_across_halves(tmax);
    const float m_new = fmaxf(m, tmax);
    const float alpha = fast_exp2(m - m_new);
    m = m_new;
    float psum = 0.f;
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      z[q] = fast_exp2(z[q] - m_new);  // masked: 2^(-1e30 - m_new) = 0 because m_new >= kWoEmpty
      psum += z[q];
    }
    s = s * alpha + psum;
    if (__builtin_amdgcn_ballot_w64(alpha != 1.f) != 0ull) {
#pragma unroll
      for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int q = 0; q < 16; ++q) o[t][q] *= alpha;
    }
    bf16x8 ph[2], pl[2];
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const __bf16 h = (__bf16)z[q];
      ph[q >> 3][q & 7] = h;
      pl[q >> 3][q & 7] = (__bf16)(z[q] - (float)h);
    }

    if (more) __builtin_amdgcn_s_waitcnt(0x0F78);  // the V tile has landed (the next K tile may be in flight)
    else __builtin_amdgcn_s_waitcnt(0x0F70);
    wave_lds_sync();
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
      uint2 r[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int slot = 16 * s2 + 8 * (i >> 2) + 4 * hi + (i & 3);  // the token acc register 8*s2 + i stands for
        r[i] = *reinterpret_cast<const uint2 *>(vtile + slot * 256 + n * 8);
      }
      u32x4 va[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint2 e = r[2 * j], f = r[2 * j + 1];
        va[0][j] = (e.x & 0xffffu) | (f.x << 16);
        va[1][j] = (e.x >> 16) | (f.x & 0xffff0000u);
        va[2][j] = (e.y & 0xffffu) | (f.y << 16);
        va[3][j] = (e.y >> 16) | (f.y & 0xffff0000u);
      }
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        o[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, va[t]), ph[s2], o[t], 0, 0, 0);
        o[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, va[t]), pl[s2], o[t], 0, 0, 0);
      }
    }
    __builtin_amdgcn_s_waitcnt(0xC07F);
    wave_lds_sync();
    if (more) issue_v(tile + kWoWaves);
  }

  FKV_BTICK_AT(blk_id, 1);
  // ---- the wave's state into its own (now idle) LDS tiles: O[row n][d], 16-byte chunks XOR-swizzled by row
  s = add_across_halves(s);
  float *ow = reinterpret_cast<float *>(ktile);
#pragma unroll
  for (int q = 0; q < 16; ++q) {
    const int mrow = 8 * (q >> 2) + 4 * hi + (q & 3);  // output row of the tiles; d = 4*mrow + tile
    *reinterpret_cast<float4 *>(ow + n * kHeadDim + ((mrow ^ n) << 2)) = make_float4(o[0][q], o[1][q], o[2][q], o[3][q]);
  }
  if (hi == 0) ms_lds[wave][n] = make_float2(m, s);
  __syncthreads();
  FKV_BTICK_AT(blk_id, 2);

  // ---- merge the waves in a fixed order and write the block's partial
  const size_t slot = ((size_t)b * a.V + g) * a.n_split + split;
  float *po = a.part_o + slot * kWoRowFloats;
#pragma unroll
  for (int j = 0; j < kWoRowFloats / 4 / kWoThreads; ++j) {
    const int idx = threadIdx.x + j * kWoThreads;
    const int row = idx >> 5, chunk = idx & 31;
    float M = ms_lds[0][row].x;
#pragma unroll
    for (int w = 1; w < kWoWaves; ++w) M = fmaxf(M, ms_lds[w][row].x);
    float4 accv = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int w = 0; w < kWoWaves; ++w) {
      const float f = fast_exp2(ms_lds[w][row].x - M);
      const float4 x = *reinterpret_cast<const float4 *>(reinterpret_cast<const float *>(lds_all + w * kWoTileBytes) +
                                                         row * kHeadDim + ((chunk ^ row) << 2));
      accv.x += f * x.x; accv.y += f * x.y; accv.z += f * x.z; accv.w += f * x.w;
    }
    *reinterpret_cast<float4 *>(po + row * kHeadDim + chunk * 4) = accv;
  }
  if (threadIdx.x < kRowsPerGroup) {
    const int row = threadIdx.x;
    float M = ms_lds[0][row].x;
#pragma unroll
    for (int w = 1; w < kWoWaves; ++w) M = fmaxf(M, ms_lds[w][row].x);
    float S = 0.f;
#pragma unroll
    for (int w = 0; w < kWoWaves; ++w) S += ms_lds[w][row].y * fast_exp2(ms_lds[w][row].x - M);
    a.part_ms[slot * kRowsPerGroup + row] = make_float2(M, S);
  }
  FKV_BTICK_AT(blk_id, 3);
}

// Folds the splits of one (sequence, group).  Four lanes share one float4 of the output and take
// every fourth split each (eight loads in flight per lane), then meet through two lane exchanges;
// the order of the sums is fixed.  Grid (n_seq * V, 16), 256 threads.
constexpr int kWoMergeOutputs = 64;  // float4 outputs per block
__global__ __launch_bounds__(256) void k_wout_merge(WoutArgs a) {
  const int bg = blockIdx.x, b = bg / a.V, g = bg - b * a.V;
  const int j = threadIdx.x & 3;
  const int idx = blockIdx.y * kWoMergeOutputs + (threadIdx.x >> 2);
  const int row = idx >> 5, chunk = idx & 31;
  const int hl = row >> 3, w = row & 7;
  const bool first = j == 0 && chunk == 0;        // the lane that reports the row's normaliser
  if (hl >= vg_heads(a, g) || w >= a.W) {         // the four lanes of an output leave together
    if (first && a.rowstat) a.rowstat[(size_t)bg * kRowsPerGroup + row] = 0.f;
    return;
  }
  const float2 *ms = a.part_ms + (size_t)bg * a.n_split * kRowsPerGroup + row;
  const float *po = a.part_o + (size_t)bg * a.n_split * kWoRowFloats + row * kHeadDim + chunk * 4;
  constexpr int kBatch = 8;
  const int per = (a.n_split + 3) >> 2;  // splits j, j+4, ... of this lane
  float M = kNegBig;
  for (int i0 = 0; i0 < per; i0 += kBatch) {
    float mx[kBatch];
#pragma unroll
    for (int i = 0; i < kBatch; ++i) mx[i] = ms[min(4 * (i0 + i) + j, a.n_split - 1) * kRowsPerGroup].x;
#pragma unroll
    for (int i = 0; i < kBatch; ++i) M = fmaxf(M, mx[i]);
  }
  M = fmaxf(M, __shfl_xor(M, 1));
  M = fmaxf(M, __shfl_xor(M, 2));
  float den = 0.f;
  float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int i0 = 0; i0 < per; i0 += kBatch) {
    float2 st[kBatch];
    float4 x[kBatch];
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      const int sp = min(4 * (i0 + i) + j, a.n_split - 1);
      st[i] = ms[sp * kRowsPerGroup];
      x[i] = *reinterpret_cast<const float4 *>(po + (size_t)sp * kWoRowFloats);
    }
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      const float f = 4 * (i0 + i) + j < a.n_split ? fast_exp2(st[i].x - M) : 0.f;
      den += f * st[i].y;
      num.x += f * x[i].x; num.y += f * x[i].y; num.z += f * x[i].z; num.w += f * x[i].w;
    }
  }
#pragma unroll
  for (int d = 1; d <= 2; d <<= 1) {
    den += __shfl_xor(den, d);
    num.x += __shfl_xor(num.x, d); num.y += __shfl_xor(num.y, d);
    num.z += __shfl_xor(num.z, d); num.w += __shfl_xor(num.w, d);
  }
  if (j != 0) return;
  if (first && a.rowstat) a.rowstat[(size_t)bg * kRowsPerGroup + row] = M + __log2f(den);
  const float inv = 1.f / den;
  float *dst = a.out + (((size_t)b * a.W + w) * a.Hq + vg_head0(a, g) + hl) * kHeadDim + chunk * 4;
  *reinterpret_cast<float4 *>(dst) = make_float4(num.x * inv, num.y * inv, num.z * inv, num.w * inv);
}

hipError_t launch_wout(const WoutArgs &a, hipStream_t s) {
  if (a.keep_k)
    hipLaunchKernelGGL(k_wout_partial<true>, dim3(a.n_split, a.V, a.n_seq), dim3(kWoThreads), 0, s, a);
  else
    hipLaunchKernelGGL(k_wout_partial<false>, dim3(a.n_split, a.V, a.n_seq), dim3(kWoThreads), 0, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_wout_merge, dim3(a.n_seq * a.V, kWoRowFloats / 4 / kWoMergeOutputs), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace fkv
