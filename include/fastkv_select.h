/*
 * libfastkv_select: token-importance selection of FastKV (arXiv 2502.01068) on MI355X (gfx950).
 *
 * What it computes (paper notation; L = N_I tokens, W = N_obs window queries, P = L - W):
 *   score   S^{l,h}_i = Pooling( sum_{w<W} Att_l[h, P+w, i+m] )            Sec. 4.2, Eq. 1
 *           group score = mean of S^{l,h} over the heads of a KV group     App. B.1, KVCompress
 *           TSP score   = mean of S^{l,h} over all H heads                 Sec. 4.2, Eq. 2
 *   select  indices of the top-ranked prefix tokens, window tokens always
 *           kept and merged in                                             Sec. 4.2
 *   gather  hidden rows (HiddenCompress) and per-KV-head K/V rows
 *           (KVCompress) of the kept tokens                                App. B.1, Algorithm 1
 *
 * Conventions for every call
 *   - C ABI, no exceptions.  Return value: FKV_OK (0) or a negative fkv_status.
 *   - Pointers named q_win, k, v, x, scores*, idx*, *_out are DEVICE pointers, 16-byte
 *     aligned, owned by the caller; the library never frees or keeps them.  Inputs are
 *     read-only and must not alias outputs.
 *   - fkv_shape and every *_per_seq / cu_seqlens array are HOST memory, read during the
 *     call only.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*, NULL = default
 *     stream).  Calls never synchronise, never allocate, and validate every argument on
 *     the host before the first launch, so a rejected call has no effect.
 *   - Two calls that share a context must be ordered on one stream (they share the
 *     context's workspace).  Calls on different contexts may run concurrently on different
 *     streams; while several contexts exist on a device, their single-pass score launches are
 *     chained on the GPU through an event (that event wait cannot be captured into a graph, and
 *     graphs that hold single-pass launches of different contexts must not be replayed
 *     concurrently; force the two-pass kernels with fkv_set_score_path for such use).
 *   - The calling thread's current HIP device must be the context's device and `stream` must
 *     belong to it; the compute calls do not switch devices (fkv_create makes `device` current for
 *     its own set-up and puts the caller's device back before it returns).
 *   - bf16 tensors are raw 16-bit patterns.  Scores are fp32, indices int32.
 *   - Score precision: fp32 accumulation of exact bf16 products; a score agrees with exact
 *     arithmetic to a few ulp, except that each of the W probabilities it sums is formed with the
 *     hardware exp2 and is taken as 0 when it lies below fp32's normal range (2^-126): a score may
 *     fall short by up to W * 2^-126 in absolute terms, and scores that small come out as 0.
 *
 * Tensor layouts (B = n_seq sequences packed along tokens, T_b = cu_seqlens[b], sum L = T_B)
 *   q_win        [B][W][Hq][d]      bf16   queries of the last W positions of each sequence
 *   k, v         [sum L][Hkv][d]    bf16   token-major
 *   x            [sum L][row_bytes]        hidden states (row_bytes = 2*hidden for bf16)
 *   scores_group [Hkv][sum P]       fp32   sequence b starts at column T_b - b*W
 *   scores_tsp   [sum P]            fp32
 *   idx (1 row set)  [n_rows][sum k]  int32  sequence-local token positions, ascending,
 *                                            sequence b starts at column sum_{b'<b} k_b'
 *   k_out, v_out [Hkv][sum budget][d] bf16
 *   x_out        [sum k][row_bytes]
 *
 * Supported shapes: head_dim = 128; 1 <= W <= 8; Hq = G*Hkv with 1 <= G <= 8;
 * 1 <= Hkv <= 8; odd pool_kernel <= 31; B <= FKV_MAX_SEQS.  Anything else returns
 * FKV_EUNSUPPORTED.  (Groups of more than 4 query heads take two passes of the matrix tile
 * per KV head; with more than 8 such half-groups the two-pass score kernels are used.)
 */
#ifndef FASTKV_SELECT_H
#define FASTKV_SELECT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FKV_MAX_SEQS 64

typedef enum {
  FKV_OK = 0,
  FKV_EINVAL = -1,       /* a size, count or flag is out of range */
  FKV_ENULL = -2,        /* a required pointer is NULL */
  FKV_EALIGN = -3,       /* a device pointer or row size is not a multiple of 16 bytes */
  FKV_EUNSUPPORTED = -4, /* valid problem, shape outside what the kernels cover */
  FKV_EWORKSPACE = -5,   /* problem larger than the context was created for */
  FKV_EHIP = -6          /* a HIP runtime call failed; see fkv_last_hip_error */
} fkv_status;

typedef enum { FKV_POOL_AVG = 0, FKV_POOL_MAX = 1 } fkv_pool_t;

/* Problem description (host struct). */
typedef struct fkv_shape {
  int32_t n_seq;             /* B >= 1 */
  const int32_t *cu_seqlens; /* host [B+1], cu[0] = 0, strictly increasing; may be NULL when B == 1 */
  int32_t L;                 /* tokens of the single sequence when cu_seqlens == NULL */
  int32_t n_q_heads;         /* Hq */
  int32_t n_kv_heads;        /* Hkv; query head h reads KV head h / (Hq/Hkv) */
  int32_t head_dim;          /* d */
  int32_t window;            /* W = N_obs (Sec. 5.1 uses 8) */
  int32_t pool_kernel;       /* odd; Sec. 5.1 uses 7 */
  int32_t pool_mode;         /* fkv_pool_t; App. D.4 names max pooling */
  float softmax_scale;       /* 0 means 1/sqrt(d) */
  int32_t causal;            /* 1: window query w sees keys j <= P + w; 0: all L keys */
} fkv_shape;

typedef struct fkv_ctx fkv_ctx;

/* Library version as major*10000 + minor*100 + patch. */
int fkv_version(void);
const char *fkv_strerror(int status);
/* hipError_t of the last failed HIP call on this thread (0 if none). */
int fkv_last_hip_error(void);

/* Host-only checks, usable without a GPU.  fkv_check_shape validates a shape;
 * fkv_check_counts validates a per-sequence keep count array (W <= count_b <= L_b). */
int fkv_check_shape(const fkv_shape *shape);
int fkv_check_counts(const fkv_shape *shape, const int32_t *count_per_seq);

/* Device workspace a context needs for problems of up to max_total_tokens tokens in up to
 * max_seqs sequences (Hkv <= 8). */
size_t fkv_workspace_bytes(int64_t max_total_tokens, int32_t max_seqs);

/* Create a context on HIP device `device`; allocates the workspace once (the only
 * allocation the library ever makes) and synchronises that device.  fkv_destroy frees it; the
 * caller must have synchronised the streams that used it. */
int fkv_create(fkv_ctx **out, int device, int64_t max_total_tokens, int32_t max_seqs);
int fkv_destroy(fkv_ctx *ctx);

/* score_window(Q_win, K) -> per-token scores (Eq. 1, Eq. 2, App. B.1 group mean).
 * scores_group is required (unless no sequence has a prefix token); scores_tsp may be NULL. */
int fkv_score_window(fkv_ctx *ctx, const fkv_shape *shape, const void *q_win, const void *k,
                     float *scores_group, float *scores_tsp, void *stream);

/* select_topk(scores, k) -> ascending kept indices (Sec. 4.2).  `scores` holds n_rows rows
 * laid out like scores_group (row stride = sum P floats).  For each row and sequence the
 * k_b - W largest prefix scores are kept (equal scores: lower index first) and the W window
 * positions P_b .. L_b-1 are appended, so exactly k_b indices come out.  Requires
 * W <= k_b <= L_b.  NaN scores are outside the contract. */
int fkv_select_topk(fkv_ctx *ctx, const fkv_shape *shape, const float *scores, int32_t n_rows,
                    const int32_t *k_per_seq, int32_t *idx_out, void *stream);

/* gather_rows(X, idx): out[o_b + t][:] = x[T_b + idx[o_b + t]][:] for t < k_b, where
 * o_b = sum_{b'<b} k_b' (HiddenCompress, App. B.1).  Rows are copied bit for bit.
 * Indices must lie in [0, L_b); the kernels clamp an index beyond the sequence into it (a wrong
 * row is copied, nothing is read out of bounds) and copy nothing for a negative index (the mark
 * fkv_compress_kv leaves when its score pass failed).  The same holds for every gather below. */
int fkv_gather_rows(fkv_ctx *ctx, const fkv_shape *shape, const void *x, size_t row_bytes,
                    const int32_t *idx, const int32_t *k_per_seq, void *out, void *stream);

/* Per-KV-head gather of KVCompress (App. B.1): for g < Hkv,
 * k_out[g][o_b + t][:] = k[T_b + idx_kv[g][o_b + t]][g][:], same for v.  v / v_out may both
 * be NULL to gather K only. */
int fkv_gather_kv(fkv_ctx *ctx, const fkv_shape *shape, const void *k, const void *v,
                  const int32_t *idx_kv, const int32_t *budget_per_seq, void *k_out, void *v_out,
                  void *stream);

/* fkv_score_window for callers that cannot allocate device memory or create a context: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (minus
 * the context), same outputs, computed by the two-pass score kernels; the scratch they need (the
 * per-block row statistics and the per-row normalisers) lives in a 4.3 MB array in the library's
 * device image instead of a context's workspace, so the call allocates nothing, frees nothing and
 * calls nothing that does.  Limits: at most 131072 tokens in at most 16 sequences per call, else
 * FKV_EWORKSPACE; devices 0..15.  Runs on the calling thread's current device, on `stream`.  All
 * calls on one GPU share that GPU's copy of the array: calls that overlap on one GPU (different
 * streams without an ordering between them) race; calls ordered on one stream, or by events, are
 * fine.  Nothing in the array has to be cleared between calls (every word a call reads, it has
 * written before).  The first call on a device looks up the array's device address (no
 * allocation); make that first call outside graph capture. */
int fkv_score_window_static(const fkv_shape *shape, const void *q_win, const void *k, float *scores_group,
                            float *scores_tsp, void *stream);

/* Per-head variant of the score (Eq. 1 alone, no averaging over heads): scores_head [Hq][sum P]
 * holds the pooled saliency S^{l,h} of every query head.  With fkv_select_topk (n_rows = Hq) and
 * fkv_gather_kv_per_head it gives head-wise KV retention, the layout Sec. 5.3 contrasts with the
 * group-wise one (it stores Hq instead of Hkv compacted copies). */
int fkv_score_heads(fkv_ctx *ctx, const fkv_shape *shape, const void *q_win, const void *k, float *scores_head,
                    void *stream);

/* k_out[h][o_b + t][:] = k[T_b + idx_head[h][o_b + t]][h / G][:] for every query head h < Hq (same
 * for v; v / v_out may both be NULL).  idx_head [Hq][sum budget], k_out, v_out [Hq][sum budget][d]. */
int fkv_gather_kv_per_head(fkv_ctx *ctx, const fkv_shape *shape, const void *k, const void *v,
                           const int32_t *idx_head, const int32_t *budget_per_seq, void *k_out, void *v_out,
                           void *stream);

/* Keep count for a rate ("top-{context length x R}", App. B.1): round-half-up of rate * n_tokens,
 * at most n_tokens (20 % of 32768 -> 6554); -1 for a negative length or rate.  Host only.  Callers
 * who read the paper's merge as "top-k plus the window" pass count + W to the calls above. */
int32_t fkv_count_from_rate(int32_t n_tokens, double rate);

/* The schedule of Algorithm 1 for one layer of an n_layers-deep prefill over n_tokens context
 * tokens: layers 0..tsp_layer see the whole context, later layers the k = round-half-up(tsp_rate *
 * n_tokens) tokens that the TSP layer propagates (Sec. 4.2); every layer keeps a KV budget of
 * round-half-up(kv_rate * n_tokens) tokens per KV head, counted on the original context length and
 * capped by the tokens the layer sees (Sec. 4.4, App. B.1); both counts include the window and are
 * never below it.  k_tsp is k at the TSP layer (run HiddenCompress there) and 0 elsewhere.
 * Rates in (0, 1].  Host only. */
typedef struct {
  int32_t tokens_in;  /* tokens this layer's attention and KVCompress run over */
  int32_t k_tsp;      /* rows HiddenCompress keeps after this layer, 0: none */
  int32_t kv_budget;  /* tokens KVCompress keeps per KV head */
} fkv_layer_plan;
int fkv_plan_layer(int32_t layer, int32_t n_layers, int32_t tsp_layer, int32_t n_tokens, double tsp_rate,
                   double kv_rate, int32_t window, fkv_layer_plan *out);

/* Decode-step attention of one new query token per sequence over a KV cache, every cached token
 * visible (the consumer of the compressed cache C of Algorithm 1; Sec. 5.3 measures decoding over
 * it): out[b][h][:] = sum_t softmax_t(scale * q[b][h].k[b][h/G][t]) * v[b][h/G][t].
 * q [B][Hq][d] bf16; out [B][Hq][d] fp32; n_per_seq host [B], each >= 1 (the window and any tokens
 * appended since are simply more cached tokens).  kv_layout FKV_KV_COMPACT: k, v [Hkv][sum n][d],
 * sequence b at token offset sum_{b'<b} n_b' (the k_out / v_out of fkv_compress_kv);
 * FKV_KV_TOKEN_MAJOR: k, v [sum n][Hkv][d] (an uncompressed cache).  Only n_seq, the head counts
 * and softmax_scale of `shape` are used. */
enum { FKV_KV_COMPACT = 0, FKV_KV_TOKEN_MAJOR = 1 };
int fkv_decode_attention(fkv_ctx *ctx, const fkv_shape *shape, const void *q, const void *k, const void *v,
                         int32_t kv_layout, const int32_t *n_per_seq, float *out, void *stream);

/* Attention output of the W window queries of each sequence, formed from the same probabilities
 * Eq. 1 (Sec. 4.2) sums: out[b][w][h][:] = sum over the keys j visible to position P+w of
 * Att[h, P+w, j] * v[j][h/G][:] (the layer's fused attention kernel does not expose Att, Sec. 5.1,
 * so the estimation step forms it; with this call the layer can skip those W rows).
 * q_win [B][W][Hq][d], k, v [sum L][Hkv][d] bf16 (device); out [B][W][Hq][d] fp32 (device, 16-byte
 * aligned, written completely).  Uses softmax_scale and causal of `shape` (causal = 0: every window
 * query sees every key of its sequence); the pooling fields are ignored.  Reads K and V once;
 * the probabilities enter the value contraction with 16 significant bits. */
int fkv_window_output(fkv_ctx *ctx, const fkv_shape *shape, const void *q_win, const void *k, const void *v,
                      float *out, void *stream);

/* Scores and the window rows' attention output from one set of probabilities: what fkv_score_window
 * and fkv_window_output compute (Sec. 4.2 Eq. 1-2, App. B.1; Sec. 5.1: the layer's fused attention
 * kernel does not expose Att, so the estimation step recomputes it), in one call that reads V once and
 * K twice and needs no grid-wide exchange: the pass that forms the output also leaves every softmax
 * row's normaliser, and a second pass over K (largely served by the caches the first one filled)
 * turns logits into pooled, head-averaged scores.  Arguments and outputs as in the two calls;
 * scores_tsp may be NULL. */
int fkv_score_window_output(fkv_ctx *ctx, const fkv_shape *shape, const void *q_win, const void *k, const void *v,
                            float *scores_group, float *scores_tsp, float *out, void *stream);

/* Paged cache layout (the serving layout the paper's Limitations section says the method has to
 * fit): a pool of pages [n_pages][page_size][Hkv][d] bf16 per tensor and a DEVICE block table
 * [B][max_pages_per_seq] int32; logical token t of sequence b lives in page
 * block_table[b][t / page_size], slot t % page_size.  page_size is a power of two;
 * n_pages * page_size * Hkv < 2^31; max_pages_per_seq * page_size covers every sequence's count.
 *
 * fkv_gather_kv_paged: KVCompress straight into the pages: the t-th kept row of KV head g of
 * sequence b (idx_kv as in fkv_gather_kv) goes to logical token t.  Other slots are not written; a
 * table entry outside [0, n_pages) writes nothing.  v / v_pages may both be NULL.
 *
 * fkv_compress_kv_paged: KVCompress of a layer in one call, as fkv_compress_kv without the TSP leg
 * but with the kept rows written into the pages; idx_kv [Hkv][sum budget] receives the kept
 * positions.
 *
 * fkv_decode_attention_paged: fkv_decode_attention over the first n_per_seq[b] logical tokens of
 * each sequence.  A table entry outside the pool is clamped into it (wrong result, no fault). */
int fkv_gather_kv_paged(fkv_ctx *ctx, const fkv_shape *shape, const void *k, const void *v, const int32_t *idx_kv,
                        const int32_t *budget_per_seq, const int32_t *block_table, int32_t max_pages_per_seq,
                        int32_t page_size, int64_t n_pages, void *k_pages, void *v_pages, void *stream);
int fkv_compress_kv_paged(fkv_ctx *ctx, const fkv_shape *shape, const void *q_win, const void *k, const void *v,
                          const int32_t *budget_per_seq, const int32_t *block_table, int32_t max_pages_per_seq,
                          int32_t page_size, int64_t n_pages, void *k_pages, void *v_pages, int32_t *idx_kv,
                          void *stream);
int fkv_decode_attention_paged(fkv_ctx *ctx, const fkv_shape *shape, const void *q, const void *k_pages,
                               const void *v_pages, const int32_t *block_table, int32_t max_pages_per_seq,
                               int32_t page_size, int64_t n_pages, const int32_t *n_per_seq, float *out, void *stream);

/* Measurement aid for callers that want the machine's achievable read bandwidth next to their
 * timings: one launch that only reads `bytes` (a multiple of 65536) of device memory at `src` with
 * the access pattern of the score kernels' K stream; streaming != 0 uses non-temporal loads.
 * Nothing is written.  Time it with events on `stream` or through fkv_profile_read
 * ("k_probe_read"). */
int fkv_probe_read(fkv_ctx *ctx, const void *src, int64_t bytes, int32_t streaming, void *stream);

/* Second measurement aid: the window-logits contraction of Eq. 1 alone (q.k for the Hq*W window rows
 * and every token of one sequence), on the matrix cores as the score kernels run it (use_mfma != 0)
 * or as wavefront FMAs (use_mfma == 0), for timing the two against each other on the same K stream.
 * row_keys [Hkv*32] uint32, device: entry g*32 + i*8 + w receives the largest raw logit (no scale, no
 * mask) of window row w of the i-th head of KV group g as an order-preserving key (larger float <=>
 * larger key; bit 31 set: key ^ 0x80000000 is the float's bits, else ~key), 0 for rows the shape
 * does not have.  Single sequence, G <= 4. */
int fkv_probe_logits(fkv_ctx *ctx, const fkv_shape *shape, const void *q_win, const void *k, int32_t use_mfma,
                     uint32_t *row_keys, void *stream);

/* Diagnostics of Sec. 3 on device-resident results.  Both run one block per row on `stream`.
 *
 * fkv_index_overlap: count_out[r] = number of indices A_r and B_r share, for n_rows pairs of
 * ascending, duplicate-free int32 index lists (Sec. 3.1: overlap of the critical-token sets of two layers; the overlap ratio is
 * the count over the set size).  Row r of a starts at a + r*a_stride (elements), likewise b; a
 * stride of 0 compares every row with the same list.  n_a, n_b >= 0.  count_out [n_rows] int32,
 * device.  Unsorted input gives an undefined count (never an out-of-bounds access).
 *
 * fkv_mass_recall: recall_out[r] = sum of scores_r[j] over the kept j in [0, n_scores) divided by
 * the sum of the whole row (Sec. 3.2: share of the attention mass a token subset covers); kept
 * indices outside the row (the window positions of a kept set) are skipped, a row without mass
 * gives 0.  scores row r at scores + r*row_stride (n_scores fp32), idx row r at idx + r*idx_stride
 * (n_idx int32, duplicate-free).  Sums are accumulated in fp64 in a fixed order; recall_out
 * [n_rows] fp32, device. */
int fkv_index_overlap(fkv_ctx *ctx, const int32_t *a, int64_t a_stride, int32_t n_a, const int32_t *b,
                      int64_t b_stride, int32_t n_b, int32_t n_rows, int32_t *count_out, void *stream);
int fkv_mass_recall(fkv_ctx *ctx, const float *scores, int64_t row_stride, int32_t n_scores, const int32_t *idx,
                    int64_t idx_stride, int32_t n_idx, int32_t n_rows, float *recall_out, void *stream);

/* compress_kv(K, V, budget): one layer's selection of Algorithm 1 in one call: score once,
 * select budget_b tokens per KV head, gather K/V; and, when x != NULL, also the TSP leg
 * (HiddenCompress): select k_tsp_b tokens on the all-head score and gather hidden rows.
 * idx_kv [Hkv][sum budget] and idx_tsp [sum k_tsp] are outputs.  x, k_tsp_per_seq, x_out,
 * idx_tsp are either all given or all NULL (x_row_bytes ignored then). */
int fkv_compress_kv(fkv_ctx *ctx, const fkv_shape *shape, const void *q_win, const void *k,
                    const void *v, const int32_t *budget_per_seq, void *k_out, void *v_out,
                    int32_t *idx_kv, const void *x, size_t x_row_bytes,
                    const int32_t *k_tsp_per_seq, void *x_out, int32_t *idx_tsp, void *stream);

/* Which kernels compute the scores.  0 (default): the single-pass kernel (K read once; all its
 * blocks must be resident at once, about 64K tokens per call on 256 CUs) when the batch fits,
 * else the two-pass kernels; 1: always two-pass; 2: single-pass or FKV_EUNSUPPORTED.  Both give
 * the same scores up to fp32 summation order. */
int fkv_set_score_path(fkv_ctx *ctx, int mode);

/* Which kernels select the top-k of a score row (Sec. 4.2).  0 (default): rows of more than 16384 keys
 * are cut into at most 8 slices (8192, 16384 or 32768 keys each, by row length), one block per slice,
 * and the blocks of a row agree on the threshold through device memory inside one launch, when every
 * block of the call can be resident at once (rows x slices x sequences <= compute units, rows up to
 * 262144 keys); other calls take one block per row (rows up to 32768 keys) or a chain of launches
 * (longer rows), and so do all calls while several contexts exist on the device (resident launches of
 * different contexts are chained, see above).  1: never several blocks per row inside one launch;
 * 2: several blocks per row whenever the call fits, whatever the row length and the number of
 * contexts.  All give the same indices.  The resident launch waits on other blocks with the bound of
 * fkv_set_wait_limit; a wait that runs out raises the context's error flag and the launch writes -1
 * into every index. */
int fkv_set_select_path(fkv_ctx *ctx, int mode);

/* How the single-pass score kernel would lay a batch out over at most max_blocks resident blocks
 * (host only; the library plans with the device's compute-unit count).  Block i of sequence b owns the
 * prefix tokens [i * own[b], min(P_b, (i + 1) * own[b])) and computes them plus pool_kernel / 2 halo
 * tokens on each side (the last block of a sequence: plus the W window columns instead of the right
 * halo when W is larger).  first_block [B + 1]: first block of each sequence, first_block[B] = blocks
 * in all; own [B]; n_sub_max: 32-token sub-tiles the largest block computes (at most 8).
 * FKV_EUNSUPPORTED if the batch does not fit (then the two-pass kernels run). */
int fkv_score_plan(const fkv_shape *shape, int32_t max_blocks, int32_t *first_block, int32_t *own, int32_t *n_sub_max);

/* Synchronises the device (hipDeviceSynchronize) and reports the context's sticky error flag: 0, or
 * 1 if a wave of the single-pass score kernel gave up waiting for the rest of its grid (2 s bound).
 * Cannot happen while the library's launches are the only work competing for the device's compute
 * units for that long.  The failure is visible on the device without this call: the blocks that
 * gave up write NaN scores, and while the flag is set every single-pass score launch of the context
 * writes only NaN scores, fkv_compress_kv / fkv_compress_kv_paged write -1 into every index and the
 * gathers copy nothing for those.  The flag stays set until fkv_clear_error. */
int fkv_query_error(fkv_ctx *ctx, int32_t *flag_out);

/* fkv_set_wait_limit: bound of every wait of the single-pass kernel's grid exchange in microseconds
 * (0 restores the 2 s default, at most 60 s).  A wave that gives up still leaves the kernel
 * normally; a tiny limit is how the failure path is exercised.  fkv_clear_error synchronises the
 * device, empties the exchange's mailboxes (a failed exchange may leave values in them) and resets
 * the flag; the next call works again. */
int fkv_set_wait_limit(fkv_ctx *ctx, int64_t microseconds);
int fkv_clear_error(fkv_ctx *ctx);

/* Per-kernel device timing for benchmarks.  While enabled, every launch is bracketed by
 * HIP events on the caller's stream (within one call the end event of a launch starts the next
 * launch's interval, so each figure includes the event record that precedes the launch: about
 * 2 us on MI355X, which a caller can estimate as the excess of the summed figures over the
 * un-profiled time of the same call).  fkv_profile_read synchronises those events, writes
 * the accumulated milliseconds and launch counts of kernel ids 0 .. n-1 (n =
 * fkv_profile_kernels()) and clears the accumulators.  Not for use under graph capture. */
int fkv_profile_kernels(void);
const char *fkv_profile_kernel_name(int id);
int fkv_profile_enable(fkv_ctx *ctx, int on);
int fkv_profile_read(fkv_ctx *ctx, float *ms_out, int32_t *launches_out, int32_t cap);

#ifdef __cplusplus
}
#endif
#endif /* FASTKV_SELECT_H */
