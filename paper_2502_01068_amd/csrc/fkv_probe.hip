// Measurement aid: a launch that only reads device memory, with the access pattern of the K stream
// of the score kernels (8 waves per block, wave w reads the w-th 256-byte piece of each 2 KiB token
// row, 8 x 128-bit loads in flight per lane).  Timing it on cold data gives the read bandwidth a
// score pass could reach at best on the machine at hand.
#include "fkv_internal.h"

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

}  // namespace fkv
