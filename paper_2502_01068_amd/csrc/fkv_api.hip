// C ABI of libfastkv_select: host-side validation, workspace carving and launch sequencing.
// Every entry point validates on the host first, then only enqueues kernels on the caller's
// stream; nothing here synchronises or allocates after fkv_create.
#include <math.h>
#include <mutex>
#include <new>
#include <string.h>
#include <vector>

#include "fkv_internal.h"

using namespace fkv;

namespace {

thread_local int g_last_hip_error = 0;

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct WsLayout {
  size_t partial, rowstat, scores_group, scores_tsp, counters, fused_part, fused_lse, sel_long, sel_coop, dec_part, wout_o, wout_ms, total;
  int max_stat_blocks;
};

WsLayout ws_layout(int64_t max_tokens, int32_t max_seqs) {
  WsLayout w{};
  const int chunk = stats_chunk_tokens();
  w.max_stat_blocks = (int)((max_tokens + chunk - 1) / chunk) + max_seqs;
  size_t off = 0;
  w.partial = off;      off += align_up((size_t)w.max_stat_blocks * kMaxVGroups * kRowsPerGroup * sizeof(float2));
  w.rowstat = off;      off += align_up((size_t)max_seqs * kMaxVGroups * kRowsPerGroup * sizeof(float));
  w.scores_group = off; off += align_up((size_t)max_tokens * kMaxKvHeads * sizeof(float));
  w.scores_tsp = off;   off += align_up((size_t)max_tokens * sizeof(float));
  w.counters = off;     off += align_up((size_t)kNumCounters * sizeof(unsigned));
  w.fused_part = off;   off += align_up(kFusedPartBytes);
  w.fused_lse = off;    off += align_up(kFusedLseBytes);
  w.sel_long = off;     off += align_up((size_t)kLongMaxInst * kLongStateWords * sizeof(uint32_t));
  w.sel_coop = off;     off += align_up(kCoopBoxBytes);
  w.dec_part = off;     off += align_up((size_t)max_seqs * kMaxKvHeads * kMaxReal * kDecodeMaxSplits * (kHeadDim + 2) * sizeof(float));
  const size_t wout_slots = (size_t)kWoutBlocks + (size_t)kMaxVGroups * max_seqs;
  w.wout_o = off;       off += align_up(wout_slots * kRowsPerGroup * kHeadDim * sizeof(float));
  w.wout_ms = off;      off += align_up(wout_slots * kRowsPerGroup * sizeof(float2));
  w.total = off;
  return w;
}

// The single-pass score kernel needs its whole grid resident at once (one block per CU).  Two such
// launches from different streams could each get part of the CUs and wait for the rest until their
// time limit, so when more than one context lives on a device their single-pass launches are chained
// on the GPU through an event (no host wait): each waits for the previous one to finish.  Creating
// the second context of a device synchronises the device once, so that every launch made while
// only one context existed (those are not followed by an event record) has finished before the
// first chained launch is enqueued.
struct FusedGate {
  std::mutex mu;
  int n_ctx = 0;
  hipEvent_t last = nullptr;
  bool recorded = false;
};
FusedGate g_gate[16];

// Enqueues a launch whose blocks must all be resident at once, under the device's gate.
template <typename F>
hipError_t gated_launch(int device, hipStream_t st, F &&launch) {
  FusedGate &gate = g_gate[device & 15];
  std::lock_guard<std::mutex> lock(gate.mu);
  const bool chained = gate.n_ctx > 1 && gate.last != nullptr;
  hipError_t e = hipSuccess;
  if (chained && gate.recorded) e = hipStreamWaitEvent(st, gate.last, 0);
  if (e == hipSuccess) e = launch();
  if (e == hipSuccess && chained) {
    e = hipEventRecord(gate.last, st);
    gate.recorded = true;
  }
  return e;
}

// Scratch memory and launch parameters the score kernels need besides the caller's tensors: a
// view of a context's workspace, or of the library's static scratch array.
struct ScoreWs {
  float2 *partial;      // two-pass kernels: per stats block (max, sum) of every softmax row
  int partial_stride;   // stats blocks `partial` has room for
  float *rowstat;       // [n_seq][V*32] log-sum-exp per softmax row
  float2 *fused_part;   // single-pass kernel's mailboxes, nullptr: that kernel is not available
  float *fused_lse;
  unsigned *err;
  int n_cu;             // resident blocks the single-pass kernel may use; also the block-count target of the two-pass launches
  int score_path;       // 0 auto, 1 two-pass, 2 single-pass or fail
  unsigned long long wait_ticks;
  int device;
  fkv_ctx *prof;        // context whose timing facility brackets the launches, may be nullptr
};

struct EventPair { hipEvent_t a, b, start; int kid; };  // start = own `a` or the previous launch's `b`

}  // namespace

struct fkv_ctx {
  int device;
  int64_t max_tokens;
  int32_t max_seqs;
  WsLayout lay;
  uint8_t *ws;
  int n_cu;            // compute units x resident blocks per CU of the single-pass score kernel
  int score_path;      // 0 auto, 1 two-pass kernels, 2 single-pass resident grid
  int n_cu_select;     // resident blocks of the several-blocks-per-row select kernel (0: not available)
  int select_path;     // 0 auto, 1 never several blocks per row, 2 several blocks per row whenever the launch fits
  unsigned long long wait_ticks;  // bound of every wait inside a kernel, 100 MHz ticks
  bool prof_on;
  std::vector<EventPair> ev_pool;
  size_t ev_used;
  EventPair *ev_prev;  // previous launch of the current API call (its end event starts the next)
  float ms_acc[KID_COUNT];
  int32_t n_acc[KID_COUNT];
};

namespace {

const char *kKernelNames[KID_COUNT] = {"k_stats", "k_combine", "k_scores", "k_select", "k_gather", "k_score_fused", "k_decode", "k_diag", "k_probe_read", "k_wout"};

int hip_fail(hipError_t e) {
  g_last_hip_error = (int)e;
  return FKV_EHIP;
}

// Resolved view of a shape: per-sequence token offsets.
struct Resolved {
  int n_seq;
  int cu[FKV_MAX_SEQS + 1];
  int W, Hq, Hkv, G;
  int V, vsh;  // virtual groups of at most 4 query heads (two per KV head when G > 4)
  int64_t total, sum_p;
};

int resolve(const fkv_shape *s, Resolved *r) {
  if (!s) return FKV_ENULL;
  if (s->n_seq < 1) return FKV_EINVAL;
  if (s->window < 1 || s->n_q_heads < 1 || s->n_kv_heads < 1 || s->head_dim < 1) return FKV_EINVAL;
  if (s->n_q_heads % s->n_kv_heads != 0) return FKV_EINVAL;
  if (s->pool_kernel < 1 || (s->pool_kernel & 1) == 0) return FKV_EINVAL;
  if (s->pool_mode != FKV_POOL_AVG && s->pool_mode != FKV_POOL_MAX) return FKV_EINVAL;
  if (s->causal != 0 && s->causal != 1) return FKV_EINVAL;
  if (!(s->softmax_scale >= 0.0f) || !isfinite(s->softmax_scale)) return FKV_EINVAL;
  if (!s->cu_seqlens && s->n_seq != 1) return FKV_ENULL;
  if (s->n_seq > FKV_MAX_SEQS) return FKV_EUNSUPPORTED;
  if (s->head_dim != kHeadDim) return FKV_EUNSUPPORTED;
  if (s->window > kMaxWindow) return FKV_EUNSUPPORTED;
  if (s->n_kv_heads > kMaxKvHeads || s->n_q_heads / s->n_kv_heads > kMaxReal) return FKV_EUNSUPPORTED;
  if (s->pool_kernel > kMaxPoolKernel) return FKV_EUNSUPPORTED;
  r->n_seq = s->n_seq;
  if (s->cu_seqlens) {
    if (s->cu_seqlens[0] != 0) return FKV_EINVAL;
    for (int b = 0; b <= s->n_seq; ++b) r->cu[b] = s->cu_seqlens[b];
  } else {
    r->cu[0] = 0;
    r->cu[1] = s->L;
  }
  for (int b = 0; b < r->n_seq; ++b)
    if ((int64_t)r->cu[b + 1] - r->cu[b] < s->window) return FKV_EINVAL;  // also rejects non-monotone
  r->W = s->window;
  r->Hq = s->n_q_heads;
  r->Hkv = s->n_kv_heads;
  r->G = r->Hq / r->Hkv;
  r->vsh = r->G > kMaxGroup ? 1 : 0;
  r->V = r->Hkv << r->vsh;
  r->total = r->cu[r->n_seq];
  r->sum_p = r->total - (int64_t)r->n_seq * r->W;
  return FKV_OK;
}

int check_counts(const Resolved &r, const int32_t *cnt, int *off /*[n_seq+1]*/) {
  if (!cnt) return FKV_ENULL;
  int64_t acc = 0;
  off[0] = 0;
  for (int b = 0; b < r.n_seq; ++b) {
    const int Lb = r.cu[b + 1] - r.cu[b];
    if (cnt[b] < r.W || cnt[b] > Lb) return FKV_EINVAL;
    acc += cnt[b];
    if (acc > INT32_MAX) return FKV_EINVAL;
    off[b + 1] = (int)acc;
  }
  return FKV_OK;
}

inline bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

int check_ctx(fkv_ctx *ctx, const Resolved &r) {
  if (!ctx) return FKV_ENULL;
  ctx->ev_prev = nullptr;
  if (r.total > ctx->max_tokens || r.n_seq > ctx->max_seqs) return FKV_EWORKSPACE;
  return FKV_OK;
}

// Launch bracket for the timing facility.  Within one API call the end event of a launch is the
// start event of the next, so a launch is charged its duration plus the gap before it and only
// one event record sits between consecutive kernels.
struct Timed {
  fkv_ctx *ctx;
  hipStream_t s;
  EventPair *ev;
  Timed(fkv_ctx *c, hipStream_t st, int kid) : ctx(c), s(st), ev(nullptr) {
    if (c && c->prof_on && c->ev_used < c->ev_pool.size()) {
      ev = &c->ev_pool[c->ev_used++];
      ev->kid = kid;
      if (c->ev_prev) {
        ev->start = c->ev_prev->b;
      } else {
        ev->start = ev->a;
        (void)hipEventRecord(ev->a, s);
      }
    }
  }
  ~Timed() {
    if (ev) {
      (void)hipEventRecord(ev->b, s);
      ctx->ev_prev = ev;
    }
  }
};

void fill_map(const Resolved &r, SeqMap *m) {
  m->n_seq = r.n_seq;
  for (int b = 0; b <= r.n_seq; ++b) m->cu[b] = r.cu[b];
}

// Token ranges of the single-pass score kernel's resident grid.  Block i of sequence b owns the prefix
// tokens [i * own[b], min(P_b, (i + 1) * own[b])) and computes them plus the pooling halo of r tokens on
// both sides; the last block of a sequence also computes the W window columns, so for the same amount
// of work it owns max(0, W - r) tokens fewer.  A CU streams K at a fixed rate, so the time of the pass
// follows the most tokens any block computes; the share found below is evened out inside each sequence.  blk[b] = first
// block of sequence b (blk[n_seq] = blocks in all), n_sub_max = 32-token sub-tiles the largest block
// computes.  False if no layout fits (more than fused_slots() computed tokens per block needed).
bool plan_fused(const Resolved &r, int pool_r, int max_blocks, int *blk, int *own, int *n_sub_max) {
  const int last_less = r.W > pool_r ? r.W - pool_r : 0;
  const int own_cap = fused_slots() - 2 * pool_r;
  if (own_cap <= last_less || max_blocks < 1) return false;
  // fewest blocks of a sequence at a share of at most `share` tokens per block, and the share they get:
  // the largest o <= share whose remainder P - (nb - 1) o fits the last block
  auto layout = [&](int P, int share, int *own_out) {
    *own_out = 1;
    if (P <= 0) return 0;
    for (int o = share; o > last_less; --o) {
      const int nb = (P + o - 1) / o;
      if (P - (nb - 1) * o <= o - last_less) { *own_out = o; return nb; }
    }
    return 1 << 20;  // no layout at this share
  };
  auto need = [&](int share) {
    int64_t t = 0;
    int o;
    for (int b = 0; b < r.n_seq; ++b) t += layout(r.cu[b + 1] - r.cu[b] - r.W, share, &o);
    return t;
  };
  if (need(own_cap) > max_blocks) return false;
  // First choice: the fewest full sub-tiles per block whose block count stays within what the grid
  // exchange was measured to favour.  Otherwise the smallest share that fits max_blocks (the blocks
  // needed fall as the share grows: bisect).
  int lo = 0;
  for (int n_sub = 1; n_sub * 32 <= fused_slots() && lo == 0; ++n_sub) {
    const int share = n_sub * 32 - 2 * pool_r;
    if (share > last_less && need(share) <= std::min(max_blocks, fused_preferred_blocks(n_sub))) lo = share;
  }
  if (lo == 0) {
    int hi = own_cap;
    lo = last_less + 1;
    while (lo < hi) {
      const int mid = (lo + hi) / 2;
      if (need(mid) <= max_blocks) hi = mid; else lo = mid + 1;
    }
  }
  int total = 0, own_max = 0;
  for (int b = 0; b < r.n_seq; ++b) {
    blk[b] = total;
    total += layout(r.cu[b + 1] - r.cu[b] - r.W, lo, &own[b]);
    if (own[b] > own_max) own_max = own[b];
  }
  blk[r.n_seq] = total;
  if (total < 1 || total > max_blocks) return false;
  *n_sub_max = (own_max + 2 * pool_r + 31) / 32;
  return true;
}

ScoreWs ws_of(fkv_ctx *ctx) {
  ScoreWs w{};
  w.partial = reinterpret_cast<float2 *>(ctx->ws + ctx->lay.partial);
  w.partial_stride = ctx->lay.max_stat_blocks;
  w.rowstat = reinterpret_cast<float *>(ctx->ws + ctx->lay.rowstat);
  w.fused_part = reinterpret_cast<float2 *>(ctx->ws + ctx->lay.fused_part);
  w.fused_lse = reinterpret_cast<float *>(ctx->ws + ctx->lay.fused_lse);
  w.err = reinterpret_cast<unsigned *>(ctx->ws + ctx->lay.counters) + kCtrError;
  w.n_cu = ctx->n_cu;
  w.score_path = ctx->score_path;
  w.wait_ticks = ctx->wait_ticks;
  w.device = ctx->device;
  w.prof = ctx;
  return w;
}

// Second pass of the two-pass score kernels: probabilities from the per-row normalisers in
// a.rowstat, window sum, pooling, head means.  Tiles overlap by the pooling halo.
int enqueue_scores_pass2(const ScoreWs &w, ScoreArgs &a, const Resolved &r, hipStream_t st) {
  const int n_cu = w.n_cu > 0 ? w.n_cu : 256;
  {
    int sub = scores_sub_short();
    const int64_t per_cu = (r.sum_p + n_cu - 1) / n_cu + 2 * a.pool_r;
    if (per_cu > (int64_t)sub * 32) sub = (int)((per_cu + 31) / 32);
    const int sub_max = r.V > kMaxKvHeads ? scores_sub_wide() : scores_sub_long();
    if (sub > sub_max) sub = sub_max;
    while (sub * 32 - 2 * a.pool_r < 1) ++sub;
    a.tile_sub = sub;
  }
  const int tout = a.tile_sub * 32 - 2 * a.pool_r;
  int nb = 0;
  for (int b = 0; b < r.n_seq; ++b) {
    a.map.blk[b] = nb;
    const int P = r.cu[b + 1] - r.cu[b] - r.W;
    nb += (P + tout - 1) / tout;
  }
  a.map.blk[r.n_seq] = nb;
  if (nb > 0) {
    Timed t(w.prof, st, KID_SCORES);
    const hipError_t e = launch_scores(a, nb, st);
    if (e != hipSuccess) return hip_fail(e);
  }
  return FKV_OK;
}

void fill_score_args(ScoreArgs &a, const ScoreWs &w, const fkv_shape *sh, const Resolved &r, const void *q_win,
                     const void *k, float *scores_group, float *scores_tsp, float *scores_head) {
  a.q_win = static_cast<const uint16_t *>(q_win);
  a.k = static_cast<const uint16_t *>(k);
  a.partial = w.partial;
  a.partial_stride = w.partial_stride;
  a.rowstat = w.rowstat;
  a.scores_group = scores_group;
  a.scores_tsp = scores_tsp;
  a.scores_head = scores_head;
  a.Hq = r.Hq; a.Hkv = r.Hkv; a.G = r.G; a.W = r.W;
  a.V = r.V; a.vsh = r.vsh;
  const float scale = sh->softmax_scale > 0.f ? sh->softmax_scale : 1.0f / sqrtf((float)sh->head_dim);
  a.scale_log2e = scale * 1.4426950408889634f;
  a.causal = sh->causal;
  a.pool_r = sh->pool_kernel / 2;
  a.pool_mode = sh->pool_mode;
  a.sum_p = r.sum_p;
  fill_map(r, &a.map);
}

int enqueue_score(const ScoreWs &w, const fkv_shape *sh, const Resolved &r, const void *q_win, const void *k,
                  float *scores_group, float *scores_tsp, float *scores_head, hipStream_t st) {
  ScoreArgs a{};
  fill_score_args(a, w, sh, r, q_win, k, scores_group, scores_tsp, scores_head);

  // Single pass over K when every block of the batch can be resident at once.
  if (w.fused_part != nullptr) {
    FusedArgs f{};
    int total = 0;
    const bool fits = w.score_path != 1 && r.V <= kMaxKvHeads &&
                      plan_fused(r, a.pool_r, std::min(w.n_cu, kMaxFusedBlocks), a.map.blk, f.own, &f.n_sub_max);
    if (fits) total = a.map.blk[r.n_seq];
    if (w.score_path == 2 && !(fits && total > 0)) return FKV_EUNSUPPORTED;
    if (fits && total > 0) {
      f.part = w.fused_part;
      f.lse = w.fused_lse;
      f.err = w.err;
      f.n_wg = total;
      f.timeout_ticks = w.wait_ticks;
      const hipError_t e = gated_launch(w.device, st, [&] {
        Timed t(w.prof, st, KID_SCORE_FUSED);
        return launch_score_fused(a, f, st);
      });
      return e == hipSuccess ? FKV_OK : hip_fail(e);
    }
    if (r.sum_p == 0) return FKV_OK;  // no prefix token anywhere: nothing to score
  } else if (w.score_path == 2) {
    return FKV_EUNSUPPORTED;
  }
  if (r.sum_p == 0) return FKV_OK;

  // pass 1: softmax statistics of every window row over all L keys.  Blocks take at least
  // stats_chunk_tokens() tokens, more when that keeps the launch near one block per CU (the Q
  // load and the fold at the end of a block are paid once per block).
  const int n_cu = w.n_cu > 0 ? w.n_cu : 256;
  {
    const int64_t per_cu = (r.total + n_cu - 1) / n_cu;
    int chunk = (int)((per_cu + 31) / 32 * 32);
    if (chunk < stats_chunk_tokens()) chunk = stats_chunk_tokens();
    if (chunk > 1024) chunk = 1024;
    a.chunk = chunk;
  }
  int nb = 0;
  for (int b = 0; b < r.n_seq; ++b) {
    a.map.blk[b] = nb;
    nb += (r.cu[b + 1] - r.cu[b] + a.chunk - 1) / a.chunk;
  }
  a.map.blk[r.n_seq] = nb;
  if (nb > w.partial_stride) return FKV_EWORKSPACE;
  hipError_t e;
  { Timed t(w.prof, st, KID_STATS);   e = launch_stats(a, nb, st); }
  if (e != hipSuccess) return hip_fail(e);
  { Timed t(w.prof, st, KID_COMBINE); e = launch_combine(a, st); }
  if (e != hipSuccess) return hip_fail(e);

  return enqueue_scores_pass2(w, a, r, st);
}

// The select launch(es) of a call.  Rows long enough take the several-blocks-per-row kernel, whose
// blocks must all be resident at once (hence the gate).
hipError_t enqueue_select(fkv_ctx *ctx, const SelectArgs &a, hipStream_t st) {
  uint32_t *long_state = reinterpret_cast<uint32_t *>(ctx->ws + ctx->lay.sel_long);
  unsigned *counters = reinterpret_cast<unsigned *>(ctx->ws + ctx->lay.counters);
  SelectCoop coop{};
  coop.boxes = reinterpret_cast<unsigned long long *>(ctx->ws + ctx->lay.sel_coop);
  coop.state = counters + kCtrSelEpoch;
  coop.err = counters + kCtrError;
  coop.timeout_ticks = ctx->wait_ticks;
  coop.max_blocks = std::min(ctx->n_cu_select, kCoopMaxBlocks);
  coop.mode = ctx->select_path;
  Timed t(ctx, st, KID_SELECT);
  if (coop.max_blocks > 0 && coop.mode == 0) {
    // While several contexts exist on the device, resident launches are chained one after the other;
    // the select gains less from its resident kernel than concurrent calls lose by that.
    std::lock_guard<std::mutex> lock(g_gate[ctx->device & 15].mu);
    if (g_gate[ctx->device & 15].n_ctx > 1) coop.mode = 1;
  }
  if (coop.max_blocks <= 0 || coop.mode == 1) return launch_select(a, long_state, nullptr, st);
  return gated_launch(ctx->device, st, [&] { return launch_select(a, long_state, &coop, st); });
}

void fill_rowset(SelectRowSet *rs, const float *scores, int64_t stride, int n_rows, int32_t *out,
                 const int *off, int n_seq) {
  rs->scores = scores;
  rs->row_stride = stride;
  rs->n_rows = n_rows;
  rs->idx_out = out;
  for (int b = 0; b <= n_seq; ++b) rs->cnt_off[b] = off[b];
}

void fill_job(GatherJob *j, const void *src, void *dst, const int32_t *idx, int64_t stride, int row_bytes,
              int n_heads, const int *off, int n_seq, int head_div = 1) {
  j->head_div = head_div;
  j->src = static_cast<const uint8_t *>(src);
  j->dst = static_cast<uint8_t *>(dst);
  j->idx = idx;
  j->src_row_stride = stride;
  j->row_bytes = row_bytes;
  j->n_heads = n_heads;
  j->total_rows = off[n_seq];
  for (int b = 0; b <= n_seq; ++b) j->cnt_off[b] = off[b];
}

int enqueue_gather(fkv_ctx *ctx, GatherArgs &g, const Resolved &r, hipStream_t st) {
  g.n_seq = r.n_seq;
  for (int b = 0; b <= r.n_seq; ++b) g.cu[b] = r.cu[b];
  int nb = 0;
  for (int i = 0; i < g.n_jobs; ++i) {
    GatherJob &j = g.job[i];
    if ((int64_t)j.total_rows * (j.row_bytes / 16) >= (int64_t)1 << 31) return FKV_EUNSUPPORTED;
    const int cpr = j.row_bytes / 16;
    j.cpr_shift = -1;
    for (int sft = 0; sft < 31; ++sft)
      if ((1 << sft) == cpr) j.cpr_shift = sft;
    j.blk0 = nb;
    j.blocks_per_head = gather_blocks_per_head(j);
    nb += j.blocks_per_head * j.n_heads;
  }
  if (nb == 0) return FKV_OK;
  Timed t(ctx, st, KID_GATHER);
  const hipError_t e = launch_gather(g, nb, st);
  return e == hipSuccess ? FKV_OK : hip_fail(e);
}

}  // namespace

#ifdef FKV_TIMING
namespace fkv { __device__ unsigned long long fkv_ticks[64]; __device__ unsigned long long fkv_block_ticks[1024 * 4]; __device__ unsigned long long fkv_wave_ticks[1024 * 8 * 4]; }
extern "C" int fkv_debug_read_wave_ticks(unsigned long long *out) {
  return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(fkv::fkv_wave_ticks), sizeof(unsigned long long) * 1024 * 8 * 4);
}
extern "C" int fkv_debug_read_block_ticks(unsigned long long *out) {
  return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(fkv::fkv_block_ticks), sizeof(unsigned long long) * 4096);
}
extern "C" int fkv_debug_read_ticks(unsigned long long *out) {
  return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(fkv::fkv_ticks), sizeof(unsigned long long) * 64);
}
#endif

extern "C" {

int fkv_version(void) { return 100; }

const char *fkv_strerror(int status) {
  switch (status) {
    case FKV_OK: return "ok";
    case FKV_EINVAL: return "invalid argument (size, count or flag out of range)";
    case FKV_ENULL: return "required pointer is NULL";
    case FKV_EALIGN: return "device pointer or row size not a multiple of 16 bytes";
    case FKV_EUNSUPPORTED: return "shape not supported by the gfx950 kernels";
    case FKV_EWORKSPACE: return "problem exceeds the context's workspace";
    case FKV_EHIP: return "HIP runtime error (see fkv_last_hip_error)";
    default: return "unknown status";
  }
}

int fkv_last_hip_error(void) { return g_last_hip_error; }

int fkv_check_shape(const fkv_shape *shape) {
  Resolved r;
  return resolve(shape, &r);
}

int fkv_check_counts(const fkv_shape *shape, const int32_t *count_per_seq) {
  Resolved r;
  const int rc = resolve(shape, &r);
  if (rc != FKV_OK) return rc;
  int off[FKV_MAX_SEQS + 1];
  return check_counts(r, count_per_seq, off);
}

size_t fkv_workspace_bytes(int64_t max_total_tokens, int32_t max_seqs) {
  if (max_total_tokens < 1 || max_seqs < 1 || max_seqs > FKV_MAX_SEQS) return 0;
  return ws_layout(max_total_tokens, max_seqs).total;
}

namespace {
// Mailbox words of the several-blocks-per-row select all stale (tag 0), epoch 1, nobody counted as finished.
hipError_t reset_select_exchange(fkv_ctx *c) {
  hipError_t e = hipMemset(c->ws + c->lay.sel_coop, 0, kCoopBoxBytes);
  const unsigned init[2] = {1u, 0u};
  static_assert(kCtrSelDone == kCtrSelEpoch + 1, "epoch and finish count are adjacent");
  if (e == hipSuccess)
    e = hipMemcpy(c->ws + c->lay.counters + kCtrSelEpoch * sizeof(unsigned), init, sizeof init, hipMemcpyHostToDevice);
  return e;
}
}  // namespace

int fkv_create(fkv_ctx **out, int device, int64_t max_total_tokens, int32_t max_seqs) {
  if (!out) return FKV_ENULL;
  *out = nullptr;
  if (max_total_tokens < 1 || max_total_tokens > INT32_MAX || max_seqs < 1) return FKV_EINVAL;
  if (max_seqs > FKV_MAX_SEQS) return FKV_EUNSUPPORTED;
  // the caller's current device is put back before returning
  int caller_device = -1;
  hipError_t e = hipGetDevice(&caller_device);
  if (e != hipSuccess) return hip_fail(e);
  struct RestoreDevice {
    int dev;
    ~RestoreDevice() { (void)hipSetDevice(dev); }
  } restore{caller_device};
  e = hipSetDevice(device);
  if (e != hipSuccess) return hip_fail(e);
  fkv_ctx *c = new (std::nothrow) fkv_ctx();
  if (!c) return FKV_EINVAL;
  c->device = device;
  c->max_tokens = max_total_tokens;
  c->max_seqs = max_seqs;
  c->lay = ws_layout(max_total_tokens, max_seqs);
  c->ws = nullptr;
  c->score_path = 0;
  c->wait_ticks = 200000000ull;  // 2 s
  {
    hipDeviceProp_t prop;
    e = hipGetDeviceProperties(&prop, device);
    if (e != hipSuccess) { delete c; return hip_fail(e); }
    const int per_cu = score_fused_max_blocks_per_cu();
    c->n_cu = prop.multiProcessorCount * (per_cu > 0 ? 1 : 0);  // one resident block per CU
    c->n_cu_select = prop.multiProcessorCount * (select_coop_max_blocks_per_cu() > 0 ? 1 : 0);
  }
  c->select_path = 0;
  c->prof_on = false;
  c->ev_used = 0;
  c->ev_prev = nullptr;
  memset(c->ms_acc, 0, sizeof c->ms_acc);
  memset(c->n_acc, 0, sizeof c->n_acc);
  e = hipMalloc(reinterpret_cast<void **>(&c->ws), c->lay.total);
  {
    FusedGate &gate = g_gate[device & 15];
    std::lock_guard<std::mutex> lock(gate.mu);
    if (e == hipSuccess && gate.last == nullptr) e = hipEventCreateWithFlags(&gate.last, hipEventDisableTiming);
    // launches made while this was the device's only context carry no event: let them finish
    // before chained launches begin
    if (e == hipSuccess && gate.n_ctx >= 1) e = hipDeviceSynchronize();
    if (e == hipSuccess) ++gate.n_ctx;
  }
  const bool counted = e == hipSuccess;
  if (e == hipSuccess) e = hipMemset(c->ws + c->lay.counters, 0, kNumCounters * sizeof(unsigned));
  if (e == hipSuccess) e = hipMemset(c->ws + c->lay.fused_part, 0xFF, kFusedPartBytes);  // every mailbox empty
  if (e == hipSuccess) e = hipMemset(c->ws + c->lay.fused_lse, 0xFF, kFusedLseBytes);
  if (e == hipSuccess) e = reset_select_exchange(c);
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e == hipSuccess) e = hipMemset(c->ws + c->lay.sel_long, 0, (size_t)kLongMaxInst * kLongStateWords * sizeof(uint32_t));
  if (e != hipSuccess) {
    if (counted) {
      std::lock_guard<std::mutex> lock(g_gate[device & 15].mu);
      --g_gate[device & 15].n_ctx;
    }
    if (c->ws) (void)hipFree(c->ws);
    delete c;
    return hip_fail(e);
  }
  *out = c;
  return FKV_OK;
}

int fkv_destroy(fkv_ctx *ctx) {
  if (!ctx) return FKV_ENULL;
  for (auto &p : ctx->ev_pool) {
    (void)hipEventDestroy(p.a);
    (void)hipEventDestroy(p.b);
  }
  {
    std::lock_guard<std::mutex> lock(g_gate[ctx->device & 15].mu);
    --g_gate[ctx->device & 15].n_ctx;
  }
  const hipError_t e = hipFree(ctx->ws);
  delete ctx;
  return e == hipSuccess ? FKV_OK : hip_fail(e);
}

int fkv_score_window(fkv_ctx *ctx, const fkv_shape *shape, const void *q_win, const void *k,
                     float *scores_group, float *scores_tsp, void *stream) {
  Resolved r;
  int rc = resolve(shape, &r);
  if (rc != FKV_OK) return rc;
  if (!q_win || !k || (!scores_group && r.sum_p > 0)) return FKV_ENULL;
  if (misaligned(q_win) || misaligned(k) || misaligned(scores_group) || misaligned(scores_tsp)) return FKV_EALIGN;
  rc = check_ctx(ctx, r);
  if (rc != FKV_OK) return rc;
  return enqueue_score(ws_of(ctx), shape, r, q_win, k, scores_group, scores_tsp, nullptr, static_cast<hipStream_t>(stream));
}

int fkv_select_topk(fkv_ctx *ctx, const fkv_shape *shape, const float *scores, int32_t n_rows,
                    const int32_t *k_per_seq, int32_t *idx_out, void *stream) {
  Resolved r;
  int rc = resolve(shape, &r);
  if (rc != FKV_OK) return rc;
  if ((!scores && r.sum_p > 0) || !idx_out) return FKV_ENULL;
  int off[FKV_MAX_SEQS + 1];
  rc = check_counts(r, k_per_seq, off);
  if (rc != FKV_OK) return rc;
  if (n_rows < 1 || n_rows > 65535) return FKV_EINVAL;
  if (misaligned(scores) || misaligned(idx_out)) return FKV_EALIGN;
  rc = check_ctx(ctx, r);
  if (rc != FKV_OK) return rc;
  SelectArgs a{};
  a.n_sets = 1;
  a.W = r.W;
  a.n_seq = r.n_seq;
  for (int b = 0; b <= r.n_seq; ++b) a.cu[b] = r.cu[b];
  fill_rowset(&a.set[0], scores, r.sum_p, n_rows, idx_out, off, r.n_seq);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const hipError_t e = enqueue_select(ctx, a, st);
  return e == hipSuccess ? FKV_OK : hip_fail(e);
}

int fkv_gather_rows(fkv_ctx *ctx, const fkv_shape *shape, const void *x, size_t row_bytes,
                    const int32_t *idx, const int32_t *k_per_seq, void *out, void *stream) {
  Resolved r;
  int rc = resolve(shape, &r);
  if (rc != FKV_OK) return rc;
  if (!x || !idx || !out) return FKV_ENULL;
  int off[FKV_MAX_SEQS + 1];
  rc = check_counts(r, k_per_seq, off);
  if (rc != FKV_OK) return rc;
  if (row_bytes == 0 || row_bytes > (1u << 30)) return FKV_EINVAL;
  if (row_bytes % 16 != 0 || misaligned(x) || misaligned(out) || misaligned(idx)) return FKV_EALIGN;
  rc = check_ctx(ctx, r);
  if (rc != FKV_OK) return rc;
  GatherArgs g{};
  g.n_jobs = 1;
  fill_job(&g.job[0], x, out, idx, (int64_t)row_bytes, (int)row_bytes, 1, off, r.n_seq);
  return enqueue_gather(ctx, g, r, static_cast<hipStream_t>(stream));
}

int fkv_gather_kv(fkv_ctx *ctx, const fkv_shape *shape, const void *k, const void *v,
                  const int32_t *idx_kv, const int32_t *budget_per_seq, void *k_out, void *v_out,
                  void *stream) {
  Resolved r;
  int rc = resolve(shape, &r);
  if (rc != FKV_OK) return rc;
  if (!k || !idx_kv || !k_out) return FKV_ENULL;
  if ((v == nullptr) != (v_out == nullptr)) return FKV_ENULL;
  int off[FKV_MAX_SEQS + 1];
  rc = check_counts(r, budget_per_seq, off);
  if (rc != FKV_OK) return rc;
  if (misaligned(k) || misaligned(v) || misaligned(k_out) || misaligned(v_out) || misaligned(idx_kv)) return FKV_EALIGN;
  rc = check_ctx(ctx, r);
  if (rc != FKV_OK) return rc;
  const int row_bytes = kHeadDim * 2;
  GatherArgs g{};
  g.n_jobs = 0;
  fill_job(&g.job[g.n_jobs++], k, k_out, idx_kv, (int64_t)r.Hkv * row_bytes, row_bytes, r.Hkv, off, r.n_seq);
  if (v) fill_job(&g.job[g.n_jobs++], v, v_out, idx_kv, (int64_t)r.Hkv * row_bytes, row_bytes, r.Hkv, off, r.n_seq);
  return enqueue_gather(ctx, g, r, static_cast<hipStream_t>(stream));
}

int fkv_score_heads(fkv_ctx *ctx, const fkv_shape *shape, const void *q_win, const void *k, float *scores_head,
                    void *stream) {
  Resolved r;
  int rc = resolve(shape, &r);
  if (rc != FKV_OK) return rc;
  if (!q_win || !k || (!scores_head && r.sum_p > 0)) return FKV_ENULL;
  if (misaligned(q_win) || misaligned(k) || misaligned(scores_head)) return FKV_EALIGN;
  rc = check_ctx(ctx, r);
  if (rc != FKV_OK) return rc;
  return enqueue_score(ws_of(ctx), shape, r, q_win, k, nullptr, nullptr, scores_head, static_cast<hipStream_t>(stream));
}

int fkv_gather_kv_per_head(fkv_ctx *ctx, const fkv_shape *shape, const void *k, const void *v,
                           const int32_t *idx_head, const int32_t *budget_per_seq, void *k_out, void *v_out,
                           void *stream) {
  Resolved r;
  int rc = resolve(shape, &r);
  if (rc != FKV_OK) return rc;
  if (!k || !idx_head || !k_out) return FKV_ENULL;
  if ((v == nullptr) != (v_out == nullptr)) return FKV_ENULL;
  int off[FKV_MAX_SEQS + 1];
  rc = check_counts(r, budget_per_seq, off);
  if (rc != FKV_OK) return rc;
  if (misaligned(k) || misaligned(v) || misaligned(k_out) || misaligned(v_out) || misaligned(idx_head)) return FKV_EALIGN;
  rc = check_ctx(ctx, r);
  if (rc != FKV_OK) return rc;
  const int row_bytes = kHeadDim * 2;
  GatherArgs g{};
  g.n_jobs = 0;
  fill_job(&g.job[g.n_jobs++], k, k_out, idx_head, (int64_t)r.Hkv * row_bytes, row_bytes, r.Hq, off, r.n_seq, r.G);
  if (v) fill_job(&g.job[g.n_jobs++], v, v_out, idx_head, (int64_t)r.Hkv * row_bytes, row_bytes, r.Hq, off, r.n_seq, r.G);
  return enqueue_gather(ctx, g, r, static_cast<hipStream_t>(stream));
}

int fkv_score_plan(const fkv_shape *shape, int32_t max_blocks, int32_t *first_block, int32_t *own, int32_t *n_sub_max) {
  Resolved r;
  const int rc = resolve(shape, &r);
  if (rc != FKV_OK) return rc;
  if (!first_block || !own || !n_sub_max) return FKV_ENULL;
  if (max_blocks < 1) return FKV_EINVAL;
  int blk[FKV_MAX_SEQS + 1], o[FKV_MAX_SEQS], ns = 0;
  if (r.V > kMaxKvHeads || !plan_fused(r, shape->pool_kernel / 2, std::min(max_blocks, kMaxFusedBlocks), blk, o, &ns))
    return FKV_EUNSUPPORTED;
  for (int b = 0; b <= r.n_seq; ++b) first_block[b] = blk[b];
  for (int b = 0; b < r.n_seq; ++b) own[b] = o[b];
  *n_sub_max = ns;
  return FKV_OK;
}

int32_t fkv_count_from_rate(int32_t n_tokens, double rate) {
  if (n_tokens < 0 || !(rate >= 0.0)) return -1;
  const double x = floor(rate * (double)n_tokens + 0.5);
  if (x > (double)n_tokens) return n_tokens;
  return (int32_t)x;
}

int fkv_plan_layer(int32_t layer, int32_t n_layers, int32_t tsp_layer, int32_t n_tokens, double tsp_rate,
                   double kv_rate, int32_t window, fkv_layer_plan *out) {
  if (!out) return FKV_ENULL;
  if (n_layers < 1 || layer < 0 || layer >= n_layers || tsp_layer < 0 || tsp_layer >= n_layers) return FKV_EINVAL;
  if (window < 1 || n_tokens < window) return FKV_EINVAL;
  if (!(tsp_rate > 0.0) || !(kv_rate > 0.0) || tsp_rate > 1.0 || kv_rate > 1.0) return FKV_EINVAL;
  int32_t k = fkv_count_from_rate(n_tokens, tsp_rate);
  if (k < window) k = window;                       // the window is always propagated
  int32_t budget = fkv_count_from_rate(n_tokens, kv_rate);
  if (budget < window) budget = window;
  out->tokens_in = layer <= tsp_layer ? n_tokens : k;
  out->k_tsp = layer == tsp_layer ? k : 0;
  out->kv_budget = budget < out->tokens_in ? budget : out->tokens_in;
  return FKV_OK;
}

namespace {
struct Paging {  // block-table addressing of a paged cache; table == nullptr: none
  const int32_t *table;
  int max_pages, page_size;
  int64_t n_pages;
};
int page_shift_of(int page_size) {  // log2 of a power of two, else -1
  if (page_size < 1 || (page_size & (page_size - 1)) != 0) return -1;
  int sh = 0;
  while ((1 << sh) < page_size) ++sh;
  return sh;
}
int check_paging(const Paging &pg, int Hkv) {
  if (!pg.table) return FKV_ENULL;
  if (page_shift_of(pg.page_size) < 0 || pg.max_pages < 1 || pg.n_pages < 1) return FKV_EINVAL;
  if (pg.n_pages * pg.page_size > INT32_MAX / Hkv) return FKV_EINVAL;  // slot * Hkv stays below 2^31
  return FKV_OK;
}

int decode_common(fkv_ctx *ctx, const fkv_shape *shape, const void *q, const void *k, const void *v,
                  int32_t kv_layout, const Paging *pg, const int32_t *n_per_seq, float *out, void *stream) {
  Resolved r;
  int rc = resolve(shape, &r);
  if (rc != FKV_OK) return rc;
  if (!q || !k || !v || !n_per_seq || !out) return FKV_ENULL;
  if (pg) {
    rc = check_paging(*pg, r.Hkv);
    if (rc != FKV_OK) return rc;
  } else if (kv_layout != FKV_KV_COMPACT && kv_layout != FKV_KV_TOKEN_MAJOR) {
    return FKV_EINVAL;
  }
  DecodeArgs a{};
  int64_t tot = 0;
  int n_max = 0;
  a.off[0] = 0;
  for (int b = 0; b < r.n_seq; ++b) {
    if (n_per_seq[b] < 1) return FKV_EINVAL;
    if (pg && n_per_seq[b] > (int64_t)pg->max_pages * pg->page_size) return FKV_EINVAL;
    tot += n_per_seq[b];
    if (tot > INT32_MAX) return FKV_EINVAL;
    a.off[b + 1] = (int)tot;
    if (n_per_seq[b] > n_max) n_max = n_per_seq[b];
  }
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(out)) return FKV_EALIGN;
  if (!ctx) return FKV_ENULL;
  if (r.n_seq > ctx->max_seqs) return FKV_EWORKSPACE;
  ctx->ev_prev = nullptr;
  a.q = static_cast<const uint16_t *>(q);
  a.k = static_cast<const uint16_t *>(k);
  a.v = static_cast<const uint16_t *>(v);
  a.out = out;
  a.part = reinterpret_cast<float *>(ctx->ws + ctx->lay.dec_part);
  const bool token_major = pg || kv_layout == FKV_KV_TOKEN_MAJOR;
  a.tok_stride = token_major ? (int64_t)r.Hkv * kHeadDim : kHeadDim;
  a.head_stride = token_major ? kHeadDim : tot * kHeadDim;
  if (pg) {
    a.block_table = pg->table;
    a.max_pages = pg->max_pages;
    a.page_shift = page_shift_of(pg->page_size);
    a.n_pages = (int)pg->n_pages;
  }
  a.Hq = r.Hq; a.Hkv = r.Hkv; a.G = r.G; a.n_seq = r.n_seq;
  a.V = r.V; a.vsh = r.vsh;
  int splits = (n_max + 63) / 64;  // at least 64 tokens per block, at most decode_max_splits() blocks per head
  if (splits < 1) splits = 1;
  if (splits > decode_max_splits()) splits = decode_max_splits();
  a.n_split = splits;
  const float scale = shape->softmax_scale > 0.f ? shape->softmax_scale : 1.0f / sqrtf((float)shape->head_dim);
  a.scale_log2e = scale * 1.4426950408889634f;
  hipStream_t st = static_cast<hipStream_t>(stream);
  Timed t(ctx, st, KID_DECODE);
  const hipError_t e = launch_decode(a, st);
  return e == hipSuccess ? FKV_OK : hip_fail(e);
}
}  // namespace

namespace {
// Launches the window rows' attention output; rowstat != nullptr also stores every softmax row's
// log-sum-exp there and keeps K in the caches for the score pass that follows.
int enqueue_wout(fkv_ctx *ctx, const fkv_shape *shape, const Resolved &r, const void *q_win, const void *k, const void *v,
                 float *out, float *rowstat, hipStream_t st) {
  WoutArgs a{};
  a.q_win = static_cast<const uint16_t *>(q_win);
  a.k = static_cast<const uint16_t *>(k);
  a.v = static_cast<const uint16_t *>(v);
  a.part_o = reinterpret_cast<float *>(ctx->ws + ctx->lay.wout_o);
  a.part_ms = reinterpret_cast<float2 *>(ctx->ws + ctx->lay.wout_ms);
  a.out = out;
  a.rowstat = rowstat;
  a.keep_k = rowstat != nullptr;
  int tiles_max = 1;
  for (int b = 0; b <= r.n_seq; ++b) a.cu[b] = r.cu[b];
  for (int b = 0; b < r.n_seq; ++b) tiles_max = std::max(tiles_max, (r.cu[b + 1] - r.cu[b] + 31) / 32);
  a.n_seq = r.n_seq; a.Hq = r.Hq; a.Hkv = r.Hkv; a.G = r.G; a.W = r.W;
  a.V = r.V; a.vsh = r.vsh;
  // about one block per CU over all (sequence, group) pairs, and at least one tile per wave of a block
  int splits = kWoutBlocks / (r.V * r.n_seq);
  splits = std::min(splits, (tiles_max + wout_tiles_per_block_min() - 1) / wout_tiles_per_block_min());
  a.n_split = std::max(splits, 1);
  a.causal = shape->causal;
  const float scale = shape->softmax_scale > 0.f ? shape->softmax_scale : 1.0f / sqrtf((float)shape->head_dim);
  a.scale_log2e = scale * 1.4426950408889634f;
  Timed t(ctx, st, KID_WOUT);
  const hipError_t e = launch_wout(a, st);
  return e == hipSuccess ? FKV_OK : hip_fail(e);
}
}  // namespace

int fkv_window_output(fkv_ctx *ctx, const fkv_shape *shape, const void *q_win, const void *k, const void *v,
                      float *out, void *stream) {
  Resolved r;
  int rc = resolve(shape, &r);
  if (rc != FKV_OK) return rc;
  if (!q_win || !k || !v || !out) return FKV_ENULL;
  if (misaligned(q_win) || misaligned(k) || misaligned(v) || misaligned(out)) return FKV_EALIGN;
  rc = check_ctx(ctx, r);
  if (rc != FKV_OK) return rc;
  return enqueue_wout(ctx, shape, r, q_win, k, v, out, nullptr, static_cast<hipStream_t>(stream));
}

int fkv_score_window_output(fkv_ctx *ctx, const fkv_shape *shape, const void *q_win, const void *k, const void *v,
                            float *scores_group, float *scores_tsp, float *out, void *stream) {
  Resolved r;
  int rc = resolve(shape, &r);
  if (rc != FKV_OK) return rc;
  if (!q_win || !k || !v || !out || (!scores_group && r.sum_p > 0)) return FKV_ENULL;
  if (misaligned(q_win) || misaligned(k) || misaligned(v) || misaligned(out) || misaligned(scores_group) ||
      misaligned(scores_tsp))
    return FKV_EALIGN;
  rc = check_ctx(ctx, r);
  if (rc != FKV_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const ScoreWs w = ws_of(ctx);
  // one pass over K and V: the window rows' output and, as a by-product, every softmax row's normaliser
  rc = enqueue_wout(ctx, shape, r, q_win, k, v, out, w.rowstat, st);
  if (rc != FKV_OK || r.sum_p == 0) return rc;
  // second pass over K (what the first pass left in the caches is reused): the scores
  ScoreArgs a{};
  fill_score_args(a, w, shape, r, q_win, k, scores_group, scores_tsp, nullptr);
  a.k_cached = r.V <= kMaxKvHeads ? 1 : 0;
  return enqueue_scores_pass2(w, a, r, st);
}

int fkv_decode_attention(fkv_ctx *ctx, const fkv_shape *shape, const void *q, const void *k, const void *v,
                         int32_t kv_layout, const int32_t *n_per_seq, float *out, void *stream) {
  return decode_common(ctx, shape, q, k, v, kv_layout, nullptr, n_per_seq, out, stream);
}

int fkv_decode_attention_paged(fkv_ctx *ctx, const fkv_shape *shape, const void *q, const void *k_pages,
                               const void *v_pages, const int32_t *block_table, int32_t max_pages_per_seq,
                               int32_t page_size, int64_t n_pages, const int32_t *n_per_seq, float *out, void *stream) {
  const Paging pg{block_table, max_pages_per_seq, page_size, n_pages};
  return decode_common(ctx, shape, q, k_pages, v_pages, FKV_KV_TOKEN_MAJOR, &pg, n_per_seq, out, stream);
}

namespace {
// Validation shared by the paged gathers: counts, block table geometry, chunk-id range.
int check_paged_gather(const Resolved &r, const int32_t *budget_per_seq, const Paging &pg, PagedGatherArgs *g) {
  int rc = check_counts(r, budget_per_seq, g->cnt_off);
  if (rc != FKV_OK) return rc;
  rc = check_paging(pg, r.Hkv);
  if (rc != FKV_OK) return rc;
  for (int b = 0; b < r.n_seq; ++b)
    if (budget_per_seq[b] > (int64_t)pg.max_pages * pg.page_size) return FKV_EINVAL;
  if ((int64_t)g->cnt_off[r.n_seq] * r.Hkv > (INT32_MAX >> 5)) return FKV_EINVAL;  // 16-byte chunk ids stay below 2^31
  return FKV_OK;
}
int enqueue_gather_paged(fkv_ctx *ctx, const Resolved &r, PagedGatherArgs &g, const void *k, const void *v,
                         const int32_t *idx_kv, const Paging &pg, void *k_pages, void *v_pages, hipStream_t st) {
  g.src[0] = static_cast<const uint8_t *>(k);
  g.src[1] = static_cast<const uint8_t *>(v);
  g.pages[0] = static_cast<uint8_t *>(k_pages);
  g.pages[1] = static_cast<uint8_t *>(v_pages);
  g.idx = idx_kv;
  g.block_table = pg.table;
  g.max_pages = pg.max_pages;
  g.page_shift = page_shift_of(pg.page_size);
  g.n_pages = (int)pg.n_pages;
  g.Hkv = r.Hkv;
  g.total_rows = g.cnt_off[r.n_seq];
  g.n_seq = r.n_seq;
  for (int b = 0; b <= r.n_seq; ++b) g.cu[b] = r.cu[b];
  Timed t(ctx, st, KID_GATHER);
  const hipError_t e = launch_gather_paged(g, st);
  return e == hipSuccess ? FKV_OK : hip_fail(e);
}
}  // namespace

int fkv_gather_kv_paged(fkv_ctx *ctx, const fkv_shape *shape, const void *k, const void *v, const int32_t *idx_kv,
                        const int32_t *budget_per_seq, const int32_t *block_table, int32_t max_pages_per_seq,
                        int32_t page_size, int64_t n_pages, void *k_pages, void *v_pages, void *stream) {
  Resolved r;
  int rc = resolve(shape, &r);
  if (rc != FKV_OK) return rc;
  if (!k || !idx_kv || !k_pages) return FKV_ENULL;
  if ((v == nullptr) != (v_pages == nullptr)) return FKV_ENULL;
  PagedGatherArgs g{};
  const Paging pg{block_table, max_pages_per_seq, page_size, n_pages};
  rc = check_paged_gather(r, budget_per_seq, pg, &g);
  if (rc != FKV_OK) return rc;
  if (misaligned(k) || misaligned(v) || misaligned(k_pages) || misaligned(v_pages)) return FKV_EALIGN;
  rc = check_ctx(ctx, r);
  if (rc != FKV_OK) return rc;
  return enqueue_gather_paged(ctx, r, g, k, v, idx_kv, pg, k_pages, v_pages, static_cast<hipStream_t>(stream));
}

int fkv_compress_kv_paged(fkv_ctx *ctx, const fkv_shape *shape, const void *q_win, const void *k, const void *v,
                          const int32_t *budget_per_seq, const int32_t *block_table, int32_t max_pages_per_seq,
                          int32_t page_size, int64_t n_pages, void *k_pages, void *v_pages, int32_t *idx_kv,
                          void *stream) {
  Resolved r;
  int rc = resolve(shape, &r);
  if (rc != FKV_OK) return rc;
  if (!q_win || !k || !v || !k_pages || !v_pages || !idx_kv) return FKV_ENULL;
  PagedGatherArgs g{};
  const Paging pg{block_table, max_pages_per_seq, page_size, n_pages};
  rc = check_paged_gather(r, budget_per_seq, pg, &g);
  if (rc != FKV_OK) return rc;
  if (misaligned(q_win) || misaligned(k) || misaligned(v) || misaligned(k_pages) || misaligned(v_pages) || misaligned(idx_kv))
    return FKV_EALIGN;
  rc = check_ctx(ctx, r);
  if (rc != FKV_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  float *sg = reinterpret_cast<float *>(ctx->ws + ctx->lay.scores_group);
  rc = enqueue_score(ws_of(ctx), shape, r, q_win, k, sg, nullptr, nullptr, st);
  if (rc != FKV_OK) return rc;
  SelectArgs a{};
  a.W = r.W;
  a.n_seq = r.n_seq;
  for (int b = 0; b <= r.n_seq; ++b) a.cu[b] = r.cu[b];
  a.n_sets = 0;
  a.err = ws_of(ctx).err;
  fill_rowset(&a.set[a.n_sets++], sg, r.sum_p, r.Hkv, idx_kv, g.cnt_off, r.n_seq);
  {
    const hipError_t e = enqueue_select(ctx, a, st);
    if (e != hipSuccess) return hip_fail(e);
  }
  return enqueue_gather_paged(ctx, r, g, k, v, idx_kv, pg, k_pages, v_pages, st);
}

int fkv_probe_read(fkv_ctx *ctx, const void *src, int64_t bytes, int32_t streaming, void *stream) {
  if (bytes < 0 || (bytes & 65535) != 0 || bytes / 65536 > INT32_MAX) return FKV_EINVAL;
  if (!src && bytes > 0) return FKV_ENULL;
  if (misaligned(src)) return FKV_EALIGN;
  if (!ctx) return FKV_ENULL;
  ctx->ev_prev = nullptr;
  hipStream_t st = static_cast<hipStream_t>(stream);
  Timed t(ctx, st, KID_PROBE);
  const hipError_t e = launch_probe_read(src, bytes, streaming != 0, ctx->n_cu > 0 ? ctx->n_cu : 256,
                                         reinterpret_cast<uint32_t *>(ctx->ws), st);
  return e == hipSuccess ? FKV_OK : hip_fail(e);
}

int fkv_probe_logits(fkv_ctx *ctx, const fkv_shape *shape, const void *q_win, const void *k, int32_t use_mfma,
                     uint32_t *row_keys, void *stream) {
  Resolved r;
  int rc = resolve(shape, &r);
  if (rc != FKV_OK) return rc;
  if (r.n_seq != 1 || r.vsh != 0) return FKV_EUNSUPPORTED;
  if (!q_win || !k || !row_keys) return FKV_ENULL;
  if (misaligned(q_win) || misaligned(k) || misaligned(row_keys)) return FKV_EALIGN;
  rc = check_ctx(ctx, r);
  if (rc != FKV_OK) return rc;
  ScoreArgs a{};
  a.q_win = static_cast<const uint16_t *>(q_win);
  a.k = static_cast<const uint16_t *>(k);
  a.Hq = r.Hq; a.Hkv = r.Hkv; a.G = r.G; a.W = r.W;
  a.V = r.V; a.vsh = r.vsh;
  fill_map(r, &a.map);
  hipStream_t st = static_cast<hipStream_t>(stream);
  Timed t(ctx, st, KID_PROBE);
  const hipError_t e = launch_probe_logits(a, row_keys, ctx->n_cu > 0 ? ctx->n_cu : 256, use_mfma != 0, st);
  return e == hipSuccess ? FKV_OK : hip_fail(e);
}

int fkv_index_overlap(fkv_ctx *ctx, const int32_t *a, int64_t a_stride, int32_t n_a, const int32_t *b,
                      int64_t b_stride, int32_t n_b, int32_t n_rows, int32_t *count_out, void *stream) {
  if (n_rows < 0 || n_a < 0 || n_b < 0 || a_stride < 0 || b_stride < 0) return FKV_EINVAL;
  if (!ctx) return FKV_ENULL;
  if (n_rows == 0) return FKV_OK;
  if (!count_out || (n_a > 0 && !a) || (n_b > 0 && !b)) return FKV_ENULL;
  ctx->ev_prev = nullptr;
  DiagOverlapArgs p{a, b, a_stride, b_stride, n_a, n_b, count_out};
  hipStream_t st = static_cast<hipStream_t>(stream);
  Timed t(ctx, st, KID_DIAG);
  const hipError_t e = launch_index_overlap(p, n_rows, st);
  return e == hipSuccess ? FKV_OK : hip_fail(e);
}

int fkv_mass_recall(fkv_ctx *ctx, const float *scores, int64_t row_stride, int32_t n_scores, const int32_t *idx,
                    int64_t idx_stride, int32_t n_idx, int32_t n_rows, float *recall_out, void *stream) {
  if (n_rows < 0 || n_scores < 0 || n_idx < 0 || row_stride < 0 || idx_stride < 0) return FKV_EINVAL;
  if (!ctx) return FKV_ENULL;
  if (n_rows == 0) return FKV_OK;
  if (!recall_out || (n_scores > 0 && !scores) || (n_idx > 0 && !idx)) return FKV_ENULL;
  ctx->ev_prev = nullptr;
  DiagRecallArgs p{scores, row_stride, n_scores, idx, idx_stride, n_idx, recall_out};
  hipStream_t st = static_cast<hipStream_t>(stream);
  Timed t(ctx, st, KID_DIAG);
  const hipError_t e = launch_mass_recall(p, n_rows, st);
  return e == hipSuccess ? FKV_OK : hip_fail(e);
}

int fkv_compress_kv(fkv_ctx *ctx, const fkv_shape *shape, const void *q_win, const void *k,
                    const void *v, const int32_t *budget_per_seq, void *k_out, void *v_out,
                    int32_t *idx_kv, const void *x, size_t x_row_bytes,
                    const int32_t *k_tsp_per_seq, void *x_out, int32_t *idx_tsp, void *stream) {
  Resolved r;
  int rc = resolve(shape, &r);
  if (rc != FKV_OK) return rc;
  if (!q_win || !k || !v || !k_out || !v_out || !idx_kv) return FKV_ENULL;
  const bool tsp = x != nullptr;
  if (tsp != (k_tsp_per_seq != nullptr) || tsp != (x_out != nullptr) || tsp != (idx_tsp != nullptr)) return FKV_ENULL;
  int off_kv[FKV_MAX_SEQS + 1], off_tsp[FKV_MAX_SEQS + 1];
  rc = check_counts(r, budget_per_seq, off_kv);
  if (rc != FKV_OK) return rc;
  if (tsp) {
    rc = check_counts(r, k_tsp_per_seq, off_tsp);
    if (rc != FKV_OK) return rc;
    if (x_row_bytes == 0 || x_row_bytes > (1u << 30)) return FKV_EINVAL;
    if (x_row_bytes % 16 != 0) return FKV_EALIGN;
  }
  if (misaligned(q_win) || misaligned(k) || misaligned(v) || misaligned(k_out) || misaligned(v_out) ||
      misaligned(idx_kv) || misaligned(x) || misaligned(x_out) || misaligned(idx_tsp))
    return FKV_EALIGN;
  rc = check_ctx(ctx, r);
  if (rc != FKV_OK) return rc;

  hipStream_t st = static_cast<hipStream_t>(stream);
  float *sg = reinterpret_cast<float *>(ctx->ws + ctx->lay.scores_group);
  float *stp = tsp ? reinterpret_cast<float *>(ctx->ws + ctx->lay.scores_tsp) : nullptr;
  rc = enqueue_score(ws_of(ctx), shape, r, q_win, k, sg, stp, nullptr, st);
  if (rc != FKV_OK) return rc;

  SelectArgs a{};
  a.W = r.W;
  a.n_seq = r.n_seq;
  for (int b = 0; b <= r.n_seq; ++b) a.cu[b] = r.cu[b];
  a.n_sets = 0;
  a.err = ws_of(ctx).err;
  fill_rowset(&a.set[a.n_sets++], sg, r.sum_p, r.Hkv, idx_kv, off_kv, r.n_seq);
  if (tsp) fill_rowset(&a.set[a.n_sets++], stp, r.sum_p, 1, idx_tsp, off_tsp, r.n_seq);
  {
    const hipError_t e = enqueue_select(ctx, a, st);
    if (e != hipSuccess) return hip_fail(e);
  }

  const int row_bytes = kHeadDim * 2;
  GatherArgs g{};
  g.n_jobs = 0;
  if (tsp) fill_job(&g.job[g.n_jobs++], x, x_out, idx_tsp, (int64_t)x_row_bytes, (int)x_row_bytes, 1, off_tsp, r.n_seq);
  fill_job(&g.job[g.n_jobs++], k, k_out, idx_kv, (int64_t)r.Hkv * row_bytes, row_bytes, r.Hkv, off_kv, r.n_seq);
  fill_job(&g.job[g.n_jobs++], v, v_out, idx_kv, (int64_t)r.Hkv * row_bytes, row_bytes, r.Hkv, off_kv, r.n_seq);
  return enqueue_gather(ctx, g, r, st);
}

}  // extern "C"

// ---- the entry point that allocates nothing -------------------------------------------------
// Scratch of fkv_score_window_static: the two-pass score kernels' per-block row statistics and
// the per-row normalisers, for up to kStaticMaxTokens tokens in up to kStaticMaxSeqs sequences.
// Every GPU the library runs on holds its own copy of the array until the process ends.
namespace {
constexpr int64_t kStaticMaxTokens = 131072;
constexpr int kStaticMaxSeqs = 16;
constexpr int kStaticStatBlocks = (int)(kStaticMaxTokens / kStatsChunk) + kStaticMaxSeqs;
constexpr size_t kStaticPartialBytes = (size_t)kStaticStatBlocks * kMaxVGroups * kRowsPerGroup * sizeof(float2);
constexpr size_t kStaticRowstatBytes = (size_t)kStaticMaxSeqs * kMaxVGroups * kRowsPerGroup * sizeof(float);
constexpr size_t kStaticScratchBytes = kStaticPartialBytes + kStaticRowstatBytes;  // 4.3 MB
static_assert(kStaticPartialBytes % 256 == 0, "rowstat stays aligned");
}  // namespace

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
// `scratch` above is a host-side stand-in in host code, not an address a kernel can use: the device
// address is looked up once per device and kept here.
struct StaticDevice {
  unsigned char *ptr = nullptr;
  int n_cu = 0;
};
StaticDevice g_static[16];
std::mutex g_static_mu;

int static_device(StaticDevice *out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e);
  if (dev < 0 || dev >= 16) return FKV_EUNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_static_mu);
  StaticDevice &d = g_static[dev];
  if (d.ptr == nullptr) {
    unsigned char *p = nullptr;
    e = hipGetSymbolAddress(reinterpret_cast<void **>(&p), HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_fail(e);
    if (p == nullptr) return FKV_EHIP;
    int n_cu = 0;
    e = hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return hip_fail(e);
    d.n_cu = n_cu;
    d.ptr = p;
  }
  *out = d;
  return FKV_OK;
}
}  // namespace

extern "C" {

int fkv_score_window_static(const fkv_shape *shape, const void *q_win, const void *k, float *scores_group,
                            float *scores_tsp, void *stream) {
  Resolved r;
  int rc = resolve(shape, &r);
  if (rc != FKV_OK) return rc;
  if (!q_win || !k || (!scores_group && r.sum_p > 0)) return FKV_ENULL;
  if (misaligned(q_win) || misaligned(k) || misaligned(scores_group) || misaligned(scores_tsp)) return FKV_EALIGN;
  if (r.total > kStaticMaxTokens || r.n_seq > kStaticMaxSeqs) return FKV_EWORKSPACE;
  StaticDevice d;
  rc = static_device(&d);
  if (rc != FKV_OK) return rc;
  ScoreWs w{};
  w.partial = reinterpret_cast<float2 *>(d.ptr);
  w.partial_stride = kStaticStatBlocks;
  w.rowstat = reinterpret_cast<float *>(d.ptr + kStaticPartialBytes);
  w.n_cu = d.n_cu;
  w.score_path = 1;  // the two-pass kernels: no resident-grid requirement, nothing to reset between calls
  return enqueue_score(w, shape, r, q_win, k, scores_group, scores_tsp, nullptr, static_cast<hipStream_t>(stream));
}

int fkv_set_score_path(fkv_ctx *ctx, int mode) {
  if (!ctx) return FKV_ENULL;
  if (mode < 0 || mode > 2) return FKV_EINVAL;
  ctx->score_path = mode;
  return FKV_OK;
}

int fkv_set_select_path(fkv_ctx *ctx, int mode) {
  if (!ctx) return FKV_ENULL;
  if (mode < 0 || mode > 2) return FKV_EINVAL;
  ctx->select_path = mode;
  return FKV_OK;
}

int fkv_query_error(fkv_ctx *ctx, int32_t *flag_out) {
  if (!ctx || !flag_out) return FKV_ENULL;
  unsigned v = 0;
  hipError_t e = hipDeviceSynchronize();  // streams created non-blocking do not wait for the copy below
  if (e != hipSuccess) return hip_fail(e);
  e = hipMemcpy(&v, ctx->ws + ctx->lay.counters + kCtrError * sizeof(unsigned), sizeof v,
                                 hipMemcpyDeviceToHost);
  if (e != hipSuccess) return hip_fail(e);
  *flag_out = (int32_t)v;
  return FKV_OK;
}

int fkv_set_wait_limit(fkv_ctx *ctx, int64_t microseconds) {
  if (!ctx) return FKV_ENULL;
  if (microseconds < 0 || microseconds > 60000000) return FKV_EINVAL;
  ctx->wait_ticks = microseconds == 0 ? 200000000ull : (unsigned long long)microseconds * 100ull;
  return FKV_OK;
}

int fkv_clear_error(fkv_ctx *ctx) {
  if (!ctx) return FKV_ENULL;
  hipError_t e = hipDeviceSynchronize();
  // a failed exchange may have left values in the mailboxes: empty them all, then drop the flag
  if (e == hipSuccess) e = hipMemset(ctx->ws + ctx->lay.fused_part, 0xFF, kFusedPartBytes);
  if (e == hipSuccess) e = hipMemset(ctx->ws + ctx->lay.fused_lse, 0xFF, kFusedLseBytes);
  if (e == hipSuccess) e = reset_select_exchange(ctx);
  if (e == hipSuccess) e = hipMemset(ctx->ws + ctx->lay.counters + kCtrError * sizeof(unsigned), 0, sizeof(unsigned));
  if (e == hipSuccess) e = hipDeviceSynchronize();
  return e == hipSuccess ? FKV_OK : hip_fail(e);
}

int fkv_profile_kernels(void) { return KID_COUNT; }

const char *fkv_profile_kernel_name(int id) { return (id >= 0 && id < KID_COUNT) ? kKernelNames[id] : ""; }

int fkv_profile_enable(fkv_ctx *ctx, int on) {
  if (!ctx) return FKV_ENULL;
  if (on && ctx->ev_pool.empty()) {
    ctx->ev_pool.resize(4096);
    for (auto &p : ctx->ev_pool) {
      hipError_t e = hipEventCreate(&p.a);
      if (e == hipSuccess) e = hipEventCreate(&p.b);
      if (e != hipSuccess) return hip_fail(e);
    }
  }
  ctx->prof_on = on != 0;
  return FKV_OK;
}

int fkv_profile_read(fkv_ctx *ctx, float *ms_out, int32_t *launches_out, int32_t cap) {
  if (!ctx || !ms_out || !launches_out) return FKV_ENULL;
  if (cap < KID_COUNT) return FKV_EINVAL;
  for (size_t i = 0; i < ctx->ev_used; ++i) {
    EventPair &p = ctx->ev_pool[i];
    hipError_t e = hipEventSynchronize(p.b);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, p.start, p.b);
    if (e != hipSuccess) return hip_fail(e);
    ctx->ms_acc[p.kid] += ms;
    ctx->n_acc[p.kid] += 1;
  }
  ctx->ev_used = 0;
  for (int i = 0; i < KID_COUNT; ++i) {
    ms_out[i] = ctx->ms_acc[i];
    launches_out[i] = ctx->n_acc[i];
    ctx->ms_acc[i] = 0.f;
    ctx->n_acc[i] = 0;
  }
  return FKV_OK;
}

}  // extern "C"
