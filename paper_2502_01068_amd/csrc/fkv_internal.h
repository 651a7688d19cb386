// Internal declarations shared by the HIP translation units of libfastkv_select.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fastkv_select.h"

namespace fkv {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));  // one 128-bit load / store

constexpr int kHeadDim = 128;     // d: one KV-head row is 256 bytes = 16 lanes x 16 B
constexpr int kMaxWindow = 8;     // W <= 8: window index is the low 3 bits of an MFMA row
constexpr int kMaxGroup = 4;      // query heads per MFMA row tile: head-in-tile is the high 2 bits of a row
constexpr int kMaxKvHeads = 8;
// A KV group of more than 4 query heads is processed as two "virtual groups" of up to 4 heads that
// read the same K rows: virtual group v serves KV head v >> vsh and query heads
// (v >> vsh) * G + (v & (vg - 1)) * 4 + {0..3} (those below G).  vg = 1 << vsh is 1 for G <= 4, else 2.
constexpr int kMaxReal = 8;       // G <= 8
constexpr int kMaxVGroups = 16;   // Hkv * vg
constexpr int kRowsPerGroup = 32; // MFMA M: row m = head_in_group * 8 + w
constexpr int kMaxPoolKernel = 31;
constexpr int kStatsChunk = 128;  // fewest tokens per block in the statistics pass of the two-pass score kernels

// Phase timestamps for kernel tuning builds (-DFKV_TIMING): block (0,0), thread 0 stores the
// 100 MHz wall clock into fkv_ticks[i].  Compiles to nothing in the product build.
#ifdef FKV_TIMING
extern __device__ unsigned long long fkv_ticks[64];
#define FKV_TICK(i)                                                                         \
  do {                                                                                      \
    if (threadIdx.x == 0 && blockIdx.x == FKV_TIMING_BLOCK && blockIdx.y == 0) fkv::fkv_ticks[i] = wall_clock64(); \
  } while (0)
extern __device__ unsigned long long fkv_block_ticks[1024 * 4];
#define FKV_BTICK(i)                                                                        \
  do {                                                                                      \
    if (threadIdx.x == 0 && blockIdx.x < 1024) fkv::fkv_block_ticks[blockIdx.x * 4 + (i)] = wall_clock64(); \
  } while (0)
#define FKV_BTICK_AT(blk, i)                                                                \
  do {                                                                                      \
    if (threadIdx.x == 0 && (blk) < 1024) fkv::fkv_block_ticks[(blk) * 4 + (i)] = wall_clock64(); \
  } while (0)
extern __device__ unsigned long long fkv_wave_ticks[1024 * 8 * 4];
#define FKV_WTICK(i)                                                                        \
  do {                                                                                      \
    if ((threadIdx.x & 63) == 0 && blockIdx.x < 1024 && blockDim.x <= 512)                  \
      fkv::fkv_wave_ticks[(blockIdx.x * 8 + (threadIdx.x >> 6)) * 4 + (i)] = wall_clock64(); \
  } while (0)
#else
#define FKV_TICK(i) ((void)0)
#define FKV_BTICK(i) ((void)0)
#define FKV_BTICK_AT(blk, i) ((void)0)
#define FKV_WTICK(i) ((void)0)
#endif
#ifndef FKV_TIMING_BLOCK
#define FKV_TIMING_BLOCK 0
#endif

// Kernel ids for the per-kernel timing facility.
enum KernelId { KID_STATS = 0, KID_COMBINE, KID_SCORES, KID_SELECT, KID_GATHER, KID_SCORE_FUSED, KID_DECODE, KID_DIAG, KID_PROBE, KID_WOUT, KID_COUNT };

// Sequence map passed by value in the kernel arguments: where each sequence's tokens
// start and which block range of the launch works on it.
struct SeqMap {
  int n_seq;
  int cu[FKV_MAX_SEQS + 1];   // token offset of sequence b in the packed tensors
  int blk[FKV_MAX_SEQS + 1];  // first block of sequence b in this launch
};

// ---- score ------------------------------------------------------------------------------
struct ScoreArgs {
  const uint16_t *q_win;  // [B][W][Hq][d]
  const uint16_t *k;      // [sum L][Hkv][d]
  float2 *partial;        // [Hkv*32][partial_stride]: per stats block (running max, sum), log2 units
  int partial_stride;     // blocks the workspace was sized for
  float *rowstat;         // [B][Hkv*32]: log2-domain max + log2(sum) per softmax row
  float *scores_group;    // [Hkv][sum P] or nullptr
  float *scores_head;     // [Hq][sum P] or nullptr: pooled per-head scores before any head averaging
  float *scores_tsp;      // [sum P] or nullptr
  SeqMap map;
  int Hq, Hkv, G, W;
  int V, vsh;             // virtual groups (Hkv << vsh) and their shift, see kMaxVGroups
  float scale_log2e;      // softmax scale * log2(e)
  int causal;
  int pool_r;             // pooling radius (kernel = 2r+1)
  int pool_mode;          // FKV_POOL_AVG / FKV_POOL_MAX
  int chunk;              // tokens per block in the stats launch (multiple of 32)
  int tile_sub;           // 32-token sub-tiles per block in the scores launch
  int k_cached;           // scores launch: K was streamed by the launch just before (read it with plain loads)
  int64_t sum_p;          // row stride of scores_group
};

// Single-pass (resident grid) score kernel: per-launch plan and the mailboxes of its grid exchange.
constexpr int kMaxFusedBlocks = 256;  // upper bound on resident blocks (one per CU) the mailboxes hold
constexpr int kLseRowsPerBlock = kMaxKvHeads * kRowsPerGroup;  // result boxes per block: one per softmax row
constexpr int kCtrError = 0;          // sticky error flag of the context
constexpr int kNumCounters = 64;
struct FusedArgs {
  float2 *part;            // [Hkv*32][kMaxFusedBlocks]: (max, sum) of a softmax row over one block's tokens, log2 units
  float *lse;              // [kMaxFusedBlocks][kLseRowsPerBlock]: log-sum-exp of each row, one copy per block
  unsigned *err;           // the context's sticky error flag
  int n_wg;                // blocks of the launch (all resident at once)
  int n_sub_max;           // most 32-token sub-tiles any block of the launch computes
  unsigned long long timeout_ticks;  // bound of every wait of the exchange, 100 MHz ticks
  int own[FKV_MAX_SEQS];             // prefix tokens owned by each block of sequence b
};
constexpr size_t kFusedPartBytes = (size_t)kMaxKvHeads * kRowsPerGroup * kMaxFusedBlocks * sizeof(float2);
constexpr size_t kFusedLseBytes = (size_t)kMaxFusedBlocks * kLseRowsPerBlock * sizeof(float);
// Virtual-group helpers (a = any args struct with Hkv, G, vsh).
template <typename A> __host__ __device__ inline int vg_kv_head(const A &a, int v) { return v >> a.vsh; }
template <typename A> __host__ __device__ inline int vg_head0(const A &a, int v) {
  return (v >> a.vsh) * a.G + (v & ((1 << a.vsh) - 1)) * kMaxGroup;
}
template <typename A> __host__ __device__ inline int vg_heads(const A &a, int v) {
  const int left = a.G - (v & ((1 << a.vsh) - 1)) * kMaxGroup;
  return left < kMaxGroup ? left : kMaxGroup;
}
int fused_slots(void);
int fused_preferred_blocks(int n_sub);
int score_fused_max_blocks_per_cu(void);
hipError_t launch_score_fused(const ScoreArgs &a, const FusedArgs &f, hipStream_t s);

int stats_chunk_tokens(void);
int scores_sub_short(void);
int scores_sub_long(void);
int scores_sub_wide(void);
hipError_t launch_stats(const ScoreArgs &a, int n_blocks, hipStream_t s);
hipError_t launch_combine(const ScoreArgs &a, hipStream_t s);
hipError_t launch_scores(const ScoreArgs &a, int n_blocks, hipStream_t s);

// ---- select -----------------------------------------------------------------------------
struct SelectRowSet {
  const float *scores;  // rows of length sum P, sequence b at column cu[b] - b*W
  int64_t row_stride;   // floats between rows
  int n_rows;
  int32_t *idx_out;     // [n_rows][cnt_off[n_seq]]
  int cnt_off[FKV_MAX_SEQS + 1];  // prefix sums of the per-sequence keep counts
};
// Rows longer than 32768 keys are selected by a chain of launches that keeps per-row state here.
constexpr int kLongMaxInst = 256;    // (row, sequence) instances one call may have on that path (8.4 MB of state)
constexpr int kLongMaxSlices = 1024; // 8192-key slices per row (8.4M keys)
constexpr int kLongInfo = 3 * 2048;  // words: [3][2048] histograms, 16 info words, 2 counts per slice
constexpr int kLongCnt = kLongInfo + 16;
constexpr int kLongStateWords = kLongCnt + 2 * kLongMaxSlices;
struct SelectArgs {
  SelectRowSet set[2];
  int n_sets;
  int W;
  int n_seq;
  int cu[FKV_MAX_SEQS + 1];
  uint32_t *long_state;  // [kLongMaxInst][kLongStateWords], or nullptr: long rows stay on the one-block kernel
  const unsigned *err;   // sticky error flag of the score pass that produced the rows, or nullptr: while it is
                         // set every index written is -1 (the scores are invalid)
};
// Several blocks per row (fkv_select_coop.hip): the blocks of a row exchange histograms and a key list
// through tagged mailbox words; all blocks of the launch are resident at once.
constexpr int kCoopHistRounds = 4;    // histogram exchanges a search can need (fixed map, then 3 x 11 bits)
constexpr int kCoopWords = (kCoopHistRounds + 1) * 1024 + 64;  // mailbox words per block: one region per round, the list, the key range
constexpr int kCoopMaxSlices = 8;     // slices (blocks) per row; 8192, 16384 or 32768 keys each
constexpr int kCoopMaxBlocks = 256;   // blocks per launch the mailboxes hold
constexpr int kCoopMinKeys = 16384;   // rows up to here stay on the one-block kernel (measured: there the exchanges cost more than they save)
constexpr size_t kCoopBoxBytes = (size_t)kCoopMaxBlocks * kCoopWords * sizeof(unsigned long long);
constexpr int kCtrSelEpoch = 1;       // context counters: epoch of the next launch (never 0),
constexpr int kCtrSelDone = 2;        // finish count of the running launch
struct CoopArgs {
  unsigned long long *boxes;  // [blocks][kCoopWords]
  unsigned *state;            // [0] epoch, [1] finish count (low half: blocks done, high half: blocks that failed)
  unsigned *err;              // the context's sticky error flag
  unsigned long long timeout_ticks;
  int blk[FKV_MAX_SEQS + 1];  // first block of sequence b's rows; a row's slices are consecutive blocks
};
struct SelectCoop {           // what a context lends to that kernel
  unsigned long long *boxes;
  unsigned *state, *err;
  unsigned long long timeout_ticks;
  int max_blocks;             // resident blocks (0: the kernel is not used)
  int mode;                   // 0 rows over kCoopMinKeys keys, 1 never, 2 whenever the launch fits
};
int select_coop_max_blocks_per_cu(void);
bool try_launch_select_coop(const SelectArgs &a, int rows, const SelectCoop &coop, hipStream_t s, hipError_t *e);
// `long_state` is the context's state buffer for the launch chain that takes rows over 32768 keys (may be
// nullptr), `coop` what the several-blocks-per-row kernel needs (may be nullptr).
hipError_t launch_select(SelectArgs a, uint32_t *long_state, const SelectCoop *coop, hipStream_t s);
int select_long_chunk(void);
int select_long_threshold(void);
hipError_t launch_select_long(const SelectArgs &a, int rows, int max_slices, hipStream_t s);

// ---- decode attention over the cache ----------------------------------------------------
constexpr int kDecodeMaxSplits = 64;
struct DecodeArgs {
  const uint16_t *q;     // [B][Hq][d]
  const uint16_t *k, *v; // element (b, g, t) at g*head_stride + (off[b] + t)*tok_stride
  float *out;            // [B][Hq][d]
  float *part;           // [B][Hq][n_split][d + 2]
  int64_t tok_stride, head_stride;
  int Hq, Hkv, G, n_split, n_seq;
  int V, vsh;            // virtual groups, as in ScoreArgs
  float scale_log2e;
  int off[FKV_MAX_SEQS + 1];
  // paged cache (block_table != nullptr): k, v are page pools [n_pages][page_size][Hkv][d]; logical
  // token t of sequence b lives in page block_table[b*max_pages + t/page_size], slot t % page_size
  const int32_t *block_table;
  int max_pages, page_shift, n_pages;
};
int decode_max_splits(void);
hipError_t launch_decode(const DecodeArgs &a, hipStream_t s);

// ---- attention output of the window rows ------------------------------------------------
constexpr int kWoutBlocks = 256;  // blocks a launch aims for (one per CU: 128 KiB of LDS each)
struct WoutArgs {
  const uint16_t *q_win;  // [B][W][Hq][d]
  const uint16_t *k, *v;  // [sum L][Hkv][d]
  float *part_o;          // [n_seq * V][n_split][32][d]: per block, accumulator relative to its own maximum
  float2 *part_ms;        // [n_seq * V][n_split][32]: per block (max, sum), log2 units
  float *out;             // [B][W][Hq][d]
  int cu[FKV_MAX_SEQS + 1];
  int n_seq, Hq, Hkv, G, W;
  int V, vsh;             // virtual groups, as in ScoreArgs
  int n_split;            // blocks per (sequence, virtual group)
  int causal;
  float scale_log2e;
  float *rowstat;         // [n_seq][V*32] or nullptr: receives each softmax row's log-sum-exp (log2 units), the
                          // normaliser the second pass of the two-pass score kernels reads
  int keep_k;             // K is read with plain loads (it will be read again soon) instead of non-temporal ones
};
int wout_tiles_per_block_min(void);
hipError_t launch_wout(const WoutArgs &a, hipStream_t s);

// ---- diagnostics ------------------------------------------------------------------------
struct DiagOverlapArgs {
  const int32_t *a, *b;   // row r at a + r*a_stride / b + r*b_stride, ascending and duplicate-free
  int64_t a_stride, b_stride;
  int n_a, n_b;
  int32_t *count_out;     // [n_rows]
};
struct DiagRecallArgs {
  const float *scores;    // row r at scores + r*row_stride, n_scores entries
  int64_t row_stride;
  int n_scores;
  const int32_t *idx;     // row r at idx + r*idx_stride, n_idx entries
  int64_t idx_stride;
  int n_idx;
  float *recall_out;      // [n_rows]
};
hipError_t launch_index_overlap(const DiagOverlapArgs &p, int n_rows, hipStream_t s);
hipError_t launch_mass_recall(const DiagRecallArgs &p, int n_rows, hipStream_t s);

// ---- read-bandwidth probe -----------------------------------------------------------------
hipError_t launch_probe_read(const void *src, int64_t bytes, bool streaming, int n_blocks, uint32_t *sink, hipStream_t s);
struct ScoreArgs;
hipError_t launch_probe_logits(const ScoreArgs &a, uint32_t *rowkeys, int n_blocks, bool mfma, hipStream_t s);

// ---- gather -----------------------------------------------------------------------------
struct GatherJob {
  const uint8_t *src;
  uint8_t *dst;
  const int32_t *idx;     // [n_heads][total_rows]
  int64_t src_row_stride; // bytes between consecutive tokens in src
  int row_bytes;          // bytes copied per (head, kept token); multiple of 16
  int n_heads;            // output heads; head h reads source head h / head_div
  int head_div;           // src offset of source head s inside a token row is s*row_bytes
  int total_rows;         // kept rows per head over all sequences
  int blk0;               // first block of this job in the launch
  int blocks_per_head;    // blocks that cover one head's kept rows
  int cpr_shift;          // log2(row_bytes/16) when that is a power of two, else -1
  int cnt_off[FKV_MAX_SEQS + 1];
};
struct GatherArgs {
  GatherJob job[3];
  int n_jobs;
  int n_seq;
  int cu[FKV_MAX_SEQS + 1];
};
// KVCompress straight into a paged cache [n_pages][page_size][Hkv][d] through a block table.
struct PagedGatherArgs {
  const uint8_t *src[2];        // K, V: [sum L][Hkv][d] bf16 (V may be nullptr)
  uint8_t *pages[2];            // K, V page pools
  const int32_t *idx;           // [Hkv][total_rows]
  const int32_t *block_table;   // [n_seq][max_pages]
  int max_pages, page_shift, n_pages;
  int Hkv, total_rows, n_seq;
  int cu[FKV_MAX_SEQS + 1];
  int cnt_off[FKV_MAX_SEQS + 1];
};
hipError_t launch_gather_paged(const PagedGatherArgs &a, hipStream_t s);
int gather_blocks_per_head(const GatherJob &j);
hipError_t launch_gather(const GatherArgs &a, int n_blocks, hipStream_t s);

}  // namespace fkv
