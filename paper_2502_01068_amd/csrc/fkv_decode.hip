// Decode-step attention of one new query token per sequence over a KV cache, in particular the
// compacted cache KVCompress leaves behind (Algorithm 1 returns it; Sec. 5.3 measures decoding over
// it).  out[h] = sum_t softmax_t(scale * q[h].k[g(h),t]) * v[g(h),t], every cached token visible.
//
// The work is a pure stream of K and V (512 B per cached token and KV head, ~1 flop per byte), so
// it runs on the vector ALUs: 16 lanes cover one token's 256-byte row with one 128-bit load each,
// a wave takes 4 tokens per step, the G query heads of the KV group share every K / V load.  Tokens
// are split over blocks (flash-decoding style); each block keeps a running (max, sum, weighted V
// sum) per head, and a second small launch merges the splits in a fixed order.
#include "fkv_internal.h"

namespace fkv {

constexpr int kDecThreads = 256;
constexpr int kDecWaves = kDecThreads / 64;
constexpr float kDecNegBig = -1.0e30f;

int decode_max_splits(void) { return kDecodeMaxSplits; }

__device__ __forceinline__ float dec_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }
__device__ __forceinline__ void unpack8(const u32x4 &w, float (&f)[8]) {
  f[0] = bf16_lo(w[0]); f[1] = bf16_hi(w[0]); f[2] = bf16_lo(w[1]); f[3] = bf16_hi(w[1]);
  f[4] = bf16_lo(w[2]); f[5] = bf16_hi(w[2]); f[6] = bf16_lo(w[3]); f[7] = bf16_hi(w[3]);
}

// Sum over the 16 lanes of a DPP row (= the lanes that share a token), result in every lane of the
// row, on the vector ALU (row rotations; no LDS crossbar traffic).  Every lane adds the same pairs
// at every level, so the 16 results are bit-identical.
__device__ __forceinline__ float row_sum16(float x) {
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x128, 0xF, 0xF, false));  // row_ror:8
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x124, 0xF, 0xF, false));  // row_ror:4
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x122, 0xF, 0xF, false));  // row_ror:2
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x121, 0xF, 0xF, false));  // row_ror:1
  return x;
}

struct DecState {  // running softmax of one head over this lane's tokens, for the lane's 8 columns
  float m, l, acc[8];
};
__device__ __forceinline__ void dec_merge(DecState &a, float m2, float l2, const float (&acc2)[8]) {
  const float mn = fmaxf(a.m, m2);
  const float ca = dec_exp2(a.m - mn), cb = dec_exp2(m2 - mn);
  a.l = a.l * ca + l2 * cb;
#pragma unroll
  for (int i = 0; i < 8; ++i) a.acc[i] = a.acc[i] * ca + acc2[i] * cb;
  a.m = mn;
}

// grid (n_split, V, B), one block per split and virtual group; partial results part[((b*Hq + h)*n_split + s)*(128+2)]: 128 weighted sums, max, sum
template <bool kPaged>
__global__ __launch_bounds__(kDecThreads) void k_decode_partial(DecodeArgs a) {
  __shared__ float lds[kDecWaves][kMaxGroup][16][10];
  const int s = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = lane & 15, tq = lane >> 4;
  const int n = a.off[b + 1] - a.off[b];
  int chunk = (n + a.n_split - 1) / a.n_split;
  chunk = (chunk + 15) / 16 * 16;
  const int t0 = s * chunk, t1 = min(n, t0 + chunk);
  const int kvh = vg_kv_head(a, g), h0 = vg_head0(a, g), n_h = vg_heads(a, g);

  float qf[kMaxGroup][8];
#pragma unroll
  for (int hl = 0; hl < kMaxGroup; ++hl) {
    if (hl < n_h) {
      const u32x4 w = *reinterpret_cast<const u32x4 *>(a.q + ((size_t)b * a.Hq + h0 + hl) * kHeadDim + c * 8);
      unpack8(w, qf[hl]);
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) qf[hl][i] = 0.f;
    }
  }
  DecState st[kMaxGroup];
#pragma unroll
  for (int hl = 0; hl < kMaxGroup; ++hl) {
    st[hl].m = kDecNegBig;
    st[hl].l = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) st[hl].acc[i] = 0.f;
  }
  const size_t first = kPaged ? 0 : (size_t)a.off[b];  // a paged sequence is addressed through its block table
  const uint16_t *kb = a.k + (size_t)kvh * a.head_stride + first * a.tok_stride + c * 8;
  const uint16_t *vb = a.v + (size_t)kvh * a.head_stride + first * a.tok_stride + c * 8;
  const int32_t *table = kPaged ? a.block_table + (size_t)b * a.max_pages : nullptr;

  constexpr int kU = 4;  // token steps whose loads are in flight together
  for (int tb = t0 + wave * 4; tb < t1; tb += kDecWaves * 4 * kU) {  // uniform per wave
    u32x4 kw[kU], vw[kU];
#pragma unroll
    for (int u = 0; u < kU; ++u) {
      int t = min(tb + u * kDecWaves * 4 + tq, t1 - 1);
      if (kPaged) {  // physical slot; an entry outside the pool is clamped into it (never out of bounds)
        const int page = min(max(table[t >> a.page_shift], 0), a.n_pages - 1);
        t = (page << a.page_shift) + (t & ((1 << a.page_shift) - 1));
      }
      kw[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(kb + (size_t)t * a.tok_stride));
      vw[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(vb + (size_t)t * a.tok_stride));
    }
#pragma unroll
    for (int u = 0; u < kU; ++u) {
      const bool valid = tb + u * kDecWaves * 4 + tq < t1;
      float kf[8], vf[8];
      unpack8(kw[u], kf);
      unpack8(vw[u], vf);
#pragma unroll
      for (int hl = 0; hl < kMaxGroup; ++hl) {
        float dot = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) dot += qf[hl][i] * kf[i];
        dot = row_sum16(dot);  // the 16 lanes of this token
        const float z = dot * a.scale_log2e;
        const float mn = valid ? fmaxf(st[hl].m, z) : st[hl].m;
        const float corr = dec_exp2(st[hl].m - mn);
        const float p = valid ? dec_exp2(z - mn) : 0.f;
        st[hl].l = st[hl].l * corr + p;
#pragma unroll
        for (int i = 0; i < 8; ++i) st[hl].acc[i] = st[hl].acc[i] * corr + p * vf[i];
        st[hl].m = mn;
      }
    }
  }
  // merge the 4 token groups of the wave (same columns, lanes 16 and 32 apart), fixed order
#pragma unroll
  for (int off = 16; off < 64; off <<= 1) {
#pragma unroll
    for (int hl = 0; hl < kMaxGroup; ++hl) {
      const float m2 = __shfl_xor(st[hl].m, off), l2 = __shfl_xor(st[hl].l, off);
      float acc2[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) acc2[i] = __shfl_xor(st[hl].acc[i], off);
      // both partners compute merge(lower, upper) so that they agree bit for bit
      DecState lo = st[hl];
      if (lane & off) {
        DecState up = st[hl];
        lo.m = m2; lo.l = l2;
#pragma unroll
        for (int i = 0; i < 8; ++i) lo.acc[i] = acc2[i];
        dec_merge(lo, up.m, up.l, up.acc);
      } else {
        dec_merge(lo, m2, l2, acc2);
      }
      st[hl] = lo;
    }
  }
  if (tq == 0) {
#pragma unroll
    for (int hl = 0; hl < kMaxGroup; ++hl) {
#pragma unroll
      for (int i = 0; i < 8; ++i) lds[wave][hl][c][i] = st[hl].acc[i];
      lds[wave][hl][c][8] = st[hl].m;
      lds[wave][hl][c][9] = st[hl].l;
    }
  }
  __syncthreads();
  if (wave == 0 && tq == 0) {
#pragma unroll
    for (int hl = 0; hl < kMaxGroup; ++hl) {
      if (hl >= n_h) continue;
      DecState r = st[hl];
      for (int w = 1; w < kDecWaves; ++w) {
        float acc2[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc2[i] = lds[w][hl][c][i];
        dec_merge(r, lds[w][hl][c][8], lds[w][hl][c][9], acc2);
      }
      float *dst = a.part + (((size_t)b * a.Hq + h0 + hl) * a.n_split + s) * (kHeadDim + 2);
#pragma unroll
      for (int i = 0; i < 8; ++i) dst[c * 8 + i] = r.acc[i];
      if (c == 0) { dst[kHeadDim] = r.m; dst[kHeadDim + 1] = r.l; }
    }
  }
}

// grid (Hq, B), 512 threads: 4 split groups x 128 output columns.  Every thread first learns the
// splits' (max, sum) pairs (one load each, all in flight together), then sums its share of the
// splits' weighted rows with the loads of a round issued together; the 4 groups meet in LDS.
__global__ __launch_bounds__(4 * kHeadDim) void k_decode_combine(DecodeArgs a) {
  __shared__ float w_lds[kDecodeMaxSplits];
  __shared__ float o_lds[4][kHeadDim];
  __shared__ float l_tot;
  const int h = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const int col = tid & (kHeadDim - 1), grp = tid >> 7;
  const float *src = a.part + ((size_t)b * a.Hq + h) * a.n_split * (kHeadDim + 2);
  if (tid < 64) {  // one wave: lane = split
    const bool live = tid < a.n_split;
    const float m = live ? src[tid * (kHeadDim + 2) + kHeadDim] : kDecNegBig;
    const float l = live ? src[tid * (kHeadDim + 2) + kHeadDim + 1] : 0.f;
    float M = m;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) M = fmaxf(M, __shfl_xor(M, off));
    const float w = dec_exp2(m - M);
    float L = l * w;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) L += __shfl_xor(L, off);
    w_lds[tid] = w;
    if (tid == 0) l_tot = L;
  }
  __syncthreads();
  float o = 0.f;
  const int per = (a.n_split + 3) / 4;
  const int s0 = grp * per, s1 = min(a.n_split, s0 + per);
  for (int sb = s0; sb < s1; sb += 8) {
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = src[(size_t)min(sb + i, s1 - 1) * (kHeadDim + 2) + col];
#pragma unroll
    for (int i = 0; i < 8; ++i)
      if (sb + i < s1) o += v[i] * w_lds[sb + i];
  }
  o_lds[grp][col] = o;
  __syncthreads();
  if (grp == 0)
    a.out[((size_t)b * a.Hq + h) * kHeadDim + col] = (((o_lds[0][col] + o_lds[1][col]) + o_lds[2][col]) + o_lds[3][col]) / l_tot;
}

hipError_t launch_decode(const DecodeArgs &a, hipStream_t s) {
  if (a.block_table)
    hipLaunchKernelGGL(k_decode_partial<true>, dim3(a.n_split, a.V, a.n_seq), dim3(kDecThreads), 0, s, a);
  else
    hipLaunchKernelGGL(k_decode_partial<false>, dim3(a.n_split, a.V, a.n_seq), dim3(kDecThreads), 0, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_decode_combine, dim3(a.Hq, a.n_seq), dim3(4 * kHeadDim), 0, s, a);
  return hipGetLastError();
}

}  // namespace fkv
