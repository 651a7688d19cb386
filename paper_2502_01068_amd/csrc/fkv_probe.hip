// Measurement aid: a launch that only reads device memory, with the access pattern of the K stream
// of the score kernels (8 waves per block, wave w reads the w-th 256-byte piece of each 2 KiB token
// row, 8 x 128-bit loads in flight per lane).  Timing it on cold data gives the read bandwidth a
// score pass could reach at best on the machine at hand.
#include "fkv_score_common.h"
#include "fkv_select_common.h"

namespace fkv {

template <bool kStreaming>
__global__ __launch_bounds__(512) void k_probe_read(const uint8_t *p, int n_tiles, int tiles_per_block, uint32_t *sink) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = lane & 15, tq = lane >> 4;
  u32x4 acc = {0u, 0u, 0u, 0u};
  const int t0 = blockIdx.x * tiles_per_block, t1 = min(n_tiles, t0 + tiles_per_block);
  for (int t = t0; t < t1; ++t) {
    const uint8_t *tile = p + (size_t)t * 65536;  // 32 token rows of 2 KiB
    u32x4 v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const u32x4 *src = reinterpret_cast<const u32x4 *>(tile + (size_t)(i * 4 + tq) * 2048 + wave * 256 + c * 16);
      v[i] = kStreaming ? __builtin_nontemporal_load(src) : *src;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) acc ^= v[i];
  }
  // keeps the loads alive; all four words equal to this pattern does not occur for xor-folded data in practice,
  // and the store is harmless if it does
  if (acc[0] == 0x9E3779B9u && acc[1] == 0x7F4A7C15u && acc[2] == 0xF39CC060u && acc[3] == 0x5CEDC834u) sink[0] = 1u;
}

hipError_t launch_probe_read(const void *src, int64_t bytes, bool streaming, int n_blocks, uint32_t *sink, hipStream_t s) {
  const int n_tiles = (int)(bytes / 65536);
  if (n_tiles <= 0) return hipSuccess;
  if (n_blocks > n_tiles) n_blocks = n_tiles;
  const int tpb = (n_tiles + n_blocks - 1) / n_blocks;
  const uint8_t *p = static_cast<const uint8_t *>(src);
  if (streaming)
    hipLaunchKernelGGL(k_probe_read<true>, dim3(n_blocks), dim3(512), 0, s, p, n_tiles, tpb, sink);
  else
    hipLaunchKernelGGL(k_probe_read<false>, dim3(n_blocks), dim3(512), 0, s, p, n_tiles, tpb, sink);
  return hipGetLastError();
}

// ---- logits probe -------------------------------------------------------------------------
// The window-logits contraction alone (Eq. 1's q.k products for the 32 rows of a KV group and every
// token), once on the matrix cores exactly as the score kernels run it and once as wavefront FMAs, so
// the two can be timed against each other on the same K stream.  Each variant folds the largest
// raw logit of every (head, window row) over all tokens into row_max (as order-preserving integer
// keys, by atomic max), which keeps the arithmetic alive and lets the caller check that both variants
// computed the same products.
//
// FMA variant: same coalesced loads and swizzled LDS tile; lane (n, hi) takes token n's half row
// hi (64 values, unpacked to fp32 once per sub-tile), reads each query row's matching half from an
// LDS copy of Q (bf16, unpacked as it is read) and accumulates 64 FMAs per row; the two halves meet
// through one lane swap.
// Folds per-lane row maxima into the wave's LDS keys and from there into the global row keys.
template <int kN, typename RowOf>
__device__ __forceinline__ void probe_fold_rows(const float (&mx)[kN], RowOf row_of, uint32_t *rowkeys, int g,
                                                uint32_t *lds_keys, int lane) {
  if (lane < 32) lds_keys[lane] = 0u;
  wave_lds_sync();
#pragma unroll
  for (int i = 0; i < kN; ++i) atomicMax(&lds_keys[row_of(i)], order_key(mx[i]));
  wave_lds_sync();
  if (lane < kRowsPerGroup) atomicMax(&rowkeys[g * kRowsPerGroup + lane], lds_keys[lane]);
}

template <bool kMfma>
__global__ __launch_bounds__(kThreads) void k_probe_logits(ScoreArgs a, uint32_t *rowkeys, int tokens_per_block) {
  __shared__ __attribute__((aligned(16))) uint8_t stage_all[kWaves * kStageBytes];
  __shared__ __attribute__((aligned(16))) uint16_t q_lds[kMfma ? 1 : kWaves][kMfma ? 8 : kRowsPerGroup * kHeadDim];
  __shared__ uint32_t keys_lds[kWaves][32];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 31, hi = lane >> 5;
  const int Lb = a.map.cu[1];
  const int t0 = blockIdx.x * tokens_per_block, t1 = min(Lb, t0 + tokens_per_block);
  if (t0 >= t1) return;
  const int n_sub = (t1 - t0 + kSub - 1) / kSub;
  uint8_t *stage = stage_all + wave * kStageBytes;
  for (int g = wave; g < a.V; g += kWaves) {
    if (kMfma) {
      bf16x8 qa[8];
      load_q(a, 0, g, lane, qa);
      float mx[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) mx[r] = kNegBig;
      stream_head(a, qa, 0, Lb, g, t0, n_sub, stage, lane, [&](int, const floatx16 &acc) {
#pragma unroll
        for (int r = 0; r < 16; ++r) mx[r] = fmaxf(mx[r], acc[r]);
      });
      probe_fold_rows(mx, [&](int r) { return (r >> 2) * 8 + hi * 4 + (r & 3); }, rowkeys, g, keys_lds[wave], lane);
    } else {
      // Q rows of this group into LDS (rows of heads or window positions the shape does not have stay zero)
      uint16_t *ql = q_lds[wave];
      for (int i = lane; i < kRowsPerGroup * kHeadDim / 8; i += 64) {
        const int m = i >> 4, cc = i & 15, hl = m >> 3, w = m & 7;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (hl < vg_heads(a, g) && w < a.W)
          v = *reinterpret_cast<const u32x4 *>(a.q_win + ((size_t)w * a.Hq + vg_head0(a, g) + hl) * kHeadDim + cc * 8);
        *reinterpret_cast<u32x4 *>(ql + m * kHeadDim + cc * 8) = v;
      }
      wave_lds_sync();
      float mx[32];
#pragma unroll
      for (int m = 0; m < 32; ++m) mx[m] = kNegBig;
      const int c = lane & 15, tq = lane >> 4;
      const uint16_t *kbase = a.k + (size_t)vg_kv_head(a, g) * kHeadDim + c * 8;
      const size_t tok_stride = (size_t)a.Hkv * kHeadDim;
#pragma unroll 1
      for (int st = 0; st < n_sub; ++st) {
        u32x4 ld[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int t = min(t0 + st * kSub + i * 4 + tq, Lb - 1);
          ld[i] = *reinterpret_cast<const u32x4 *>(kbase + (size_t)t * tok_stride);
        }
        wave_lds_sync();
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int t = i * 4 + tq;
          *reinterpret_cast<u32x4 *>(stage + t * 256 + ((c ^ (t & 15)) << 4)) = ld[i];
        }
        wave_lds_sync();
        float kf[64];  // token n, values hi*64 .. hi*64 + 63
#pragma unroll
        for (int s = 0; s < 8; ++s) {
          const u32x4 kb = *reinterpret_cast<const u32x4 *>(stage + n * 256 + (((hi * 8 + s) ^ (n & 15)) << 4));
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            kf[s * 8 + 2 * j] = __uint_as_float(kb[j] << 16);
            kf[s * 8 + 2 * j + 1] = __uint_as_float(kb[j] & 0xFFFF0000u);
          }
        }
#pragma unroll 1
        for (int m = 0; m < 32; ++m) {
          float dot = 0.f;
#pragma unroll
          for (int s = 0; s < 8; ++s) {
            const u32x4 qb = *reinterpret_cast<const u32x4 *>(ql + m * kHeadDim + hi * 64 + s * 8);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              dot = fmaf(__uint_as_float(qb[j] << 16), kf[s * 8 + 2 * j], dot);
              dot = fmaf(__uint_as_float(qb[j] & 0xFFFF0000u), kf[s * 8 + 2 * j + 1], dot);
            }
          }
          dot = add_across_halves(dot);
          // mx is indexed at compile time in the other variant; here a small select chain keeps it in registers
#pragma unroll
          for (int mm = 0; mm < 32; ++mm)
            if (mm == m) mx[mm] = fmaxf(mx[mm], dot);
        }
      }
      probe_fold_rows(mx, [](int m) { return m; }, rowkeys, g, keys_lds[wave], lane);
    }
  }
}

__global__ void k_probe_zero(uint32_t *p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}

hipError_t launch_probe_logits(const ScoreArgs &a, uint32_t *rowkeys, int n_blocks, bool mfma, hipStream_t s) {
  const int Lb = a.map.cu[1];
  int per = (Lb + n_blocks - 1) / n_blocks;
  per = (per + kSub - 1) / kSub * kSub;
  const int blocks = (Lb + per - 1) / per;
  const int n_keys = a.V * kRowsPerGroup;
  hipLaunchKernelGGL(k_probe_zero, dim3((n_keys + 255) / 256), dim3(256), 0, s, rowkeys, n_keys);
  if (mfma)
    hipLaunchKernelGGL(k_probe_logits<true>, dim3(blocks), dim3(kThreads), 0, s, a, rowkeys, per);
  else
    hipLaunchKernelGGL(k_probe_logits<false>, dim3(blocks), dim3(kThreads), 0, s, a, rowkeys, per);
  return hipGetLastError();
}

}  // namespace fkv
