/*
 * FastKV token-importance selection: reference oracle (TEST INFRASTRUCTURE ONLY).
 *
 * A plain, slow, single-pass-per-step CPU implementation of the selection path of
 * FastKV (arXiv 2502.01068): window attention scores (Sec. 4.2, Eq. 1), pooling,
 * head / GQA-group averaging (Eq. 2; App. B.1 "KVCompress"), top-k with the window
 * tokens merged in (Sec. 4.2), and the row gathers of HiddenCompress / KVCompress
 * (App. B.1, Algorithm 1), plus the attention output of the window rows and the
 * decoding step over a cache.  It exists to check the GPU library and shares no code
 * with it.  Nothing in the product path may call it.
 *
 * Every step follows the paper's order: logits -> softmax ("attention score
 * matrix", Sec. 4.2) -> sum over the observation-window queries (Eq. 1) -> pooling
 * per head (Eq. 1) -> mean over the heads of a group (App. B.1) or over all heads
 * (Eq. 2) -> top-k + window merge -> gather.  No blocking, fusion or reordering.
 *
 * Precision: `real` is float by default (loops accumulate in fp32, left to right)
 * and double when compiled with -DORC_F64; the double build bounds the float
 * build's own rounding.  bf16 inputs are decoded exactly.
 *
 * Readings of the paper taken here (each one is a single switch or constant):
 *  - the window is exactly W rows, absolute positions L-W .. L-1; Eq. 1's printed
 *    limits (0..N_obs, row N_I) are off by one on both ends;
 *  - window scores are summed (not averaged) over w, as Eq. 1 prints;
 *  - softmax runs over every key the query may see (causal: j <= P+w), window
 *    columns included; only the prefix [0,P) is scored, pooled and ranked;
 *  - pooling taps outside [0,P) are ignored by max and count as zeros for avg
 *    (the avg divisor is always the kernel size);
 *  - head g*G .. g*G+G-1 share KV head g;
 *  - |kept| = k counts the W window tokens; ties go to the lower index.
 *
 * Pins: every function here is checked in tests/test_oracle_pins.py against something other
 * than itself (textbook softmax and library pooling / sort / index ops, closed forms for
 * equal keys, the causal corner by hand, exhaustive subset enumeration for the top-k).
 * Parity unpinned by the paper itself: it prints no value or worked example for the
 * selection, so the readings above about the pooling type and boundary, mean rather than
 * sum over heads, k counting the window and KVCompress keeping the window rest on the
 * text alone.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef ORC_F64
typedef double real;
#define REAL_EXP exp
#else
typedef float real;
#define REAL_EXP expf
#endif

#define ORC_POOL_AVG 0
#define ORC_POOL_MAX 1

int orc_real_bytes(void) { return (int)sizeof(real); }

#ifdef _OPENMP
#include <omp.h>
int orc_max_threads(void) { return omp_get_max_threads(); }
void orc_set_threads(int n) { if (n > 0) omp_set_num_threads(n); }
#else
int orc_max_threads(void) { return 1; }
void orc_set_threads(int n) { (void)n; }
#endif

static float bf16_to_f32(uint16_t b) {
  uint32_t u = ((uint32_t)b) << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return f;
}

/* Steps 1-3 (Sec. 4.2, Eq. 1 before "Pooling"): s[h][j] = sum_w Att[h, P+w, j], j in [0,P).
 * q_win [W][Hq][d] bf16 bits, k [L][Hkv][d] bf16 bits, s_head [Hq][P]. */
int orc_window_attention(const uint16_t *q_win, const uint16_t *k, int L, int Hq, int Hkv, int d,
                         int W, double scale, int causal, real *s_head) {
  if (L < W || W < 1 || Hq % Hkv != 0) return -1;
  const int P = L - W, G = Hq / Hkv;
  const real sc = (real)scale;
  int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int h = 0; h < Hq; ++h) {
    const int g = h / G;
    real *z = (real *)malloc((size_t)L * sizeof(real));
    real *row = s_head + (size_t)h * P;
    if (!z) { err = 1; continue; }
    for (int j = 0; j < P; ++j) row[j] = 0;
    for (int w = 0; w < W; ++w) {
      const int last = causal ? (P + w) : (L - 1); /* last visible key */
      const uint16_t *qv = q_win + ((size_t)w * Hq + h) * d;
      real m = 0;
      for (int j = 0; j <= last; ++j) {
        const uint16_t *kv = k + ((size_t)j * Hkv + g) * d;
        real acc = 0;
        for (int c = 0; c < d; ++c) acc += (real)bf16_to_f32(qv[c]) * (real)bf16_to_f32(kv[c]);
        z[j] = sc * acc;
        if (j == 0 || z[j] > m) m = z[j];
      }
      real Z = 0;
      for (int j = 0; j <= last; ++j) {
        z[j] = REAL_EXP(z[j] - m);
        Z += z[j];
      }
      for (int j = 0; j < P; ++j) row[j] += z[j] / Z;
    }
    free(z);
  }
  return err ? -2 : 0;
}

/* The layer's attention output at the W window positions, from the same probabilities Eq. 1 sums
 * (Sec. 4.2: Att_l is the layer's own attention matrix; Sec. 5.1 notes the fused attention kernel
 * does not hand them out, so the estimation step forms them itself):
 * out[w][h][c] = sum_{j visible to P+w} Att[h, P+w, j] * v[j][g(h)][c].
 * q_win [W][Hq][d], k, v [L][Hkv][d] bf16 bits; out [W][Hq][d]. */
int orc_window_output(const uint16_t *q_win, const uint16_t *k, const uint16_t *v, int L, int Hq, int Hkv, int d,
                      int W, double scale, int causal, real *out) {
  if (L < W || W < 1 || Hq % Hkv != 0) return -1;
  const int P = L - W, G = Hq / Hkv;
  const real sc = (real)scale;
  int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int h = 0; h < Hq; ++h) {
    const int g = h / G;
    real *a = (real *)malloc((size_t)L * sizeof(real));
    if (!a) { err = 1; continue; }
    for (int w = 0; w < W; ++w) {
      const int last = causal ? (P + w) : (L - 1);
      const uint16_t *qv = q_win + ((size_t)w * Hq + h) * d;
      real m = 0;
      for (int j = 0; j <= last; ++j) {
        const uint16_t *kv = k + ((size_t)j * Hkv + g) * d;
        real acc = 0;
        for (int c = 0; c < d; ++c) acc += (real)bf16_to_f32(qv[c]) * (real)bf16_to_f32(kv[c]);
        a[j] = sc * acc;
        if (j == 0 || a[j] > m) m = a[j];
      }
      real Z = 0;
      for (int j = 0; j <= last; ++j) { a[j] = REAL_EXP(a[j] - m); Z += a[j]; }
      real *o = out + ((size_t)w * Hq + h) * d;
      for (int c = 0; c < d; ++c) {
        real acc = 0;
        for (int j = 0; j <= last; ++j) acc += (a[j] / Z) * (real)bf16_to_f32(v[((size_t)j * Hkv + g) * d + c]);
        o[c] = acc;
      }
    }
    free(a);
  }
  return err ? -2 : 0;
}

/* Step 4 (Eq. 1 "Pooling", kernel size from Sec. 5.1; max per App. D.4): same-length
 * 1-D pooling of one row over the domain [0,P). */
int orc_pool_row(const real *s, int P, int kernel, int mode, real *p) {
  if (kernel < 1 || (kernel & 1) == 0) return -1;
  const int r = kernel / 2;
  for (int j = 0; j < P; ++j) {
    if (mode == ORC_POOL_MAX) {
      real best = s[j];
      for (int t = -r; t <= r; ++t) {
        int i = j + t;
        if (i < 0 || i >= P) continue;
        if (s[i] > best) best = s[i];
      }
      p[j] = best;
    } else {
      real sum = 0;
      for (int t = -r; t <= r; ++t) {
        int i = j + t;
        if (i < 0 || i >= P) continue;
        sum += s[i];
      }
      p[j] = sum / (real)kernel;
    }
  }
  return 0;
}

/* Step 5: S_group[g][j] = mean over the G heads of group g (App. B.1);
 * S_tsp[j] = mean over all Hq heads (Eq. 2).  Sums run in ascending head order. */
int orc_head_means(const real *p_head, int Hq, int Hkv, int P, real *s_group, real *s_tsp) {
  if (Hq % Hkv != 0) return -1;
  const int G = Hq / Hkv;
  for (int g = 0; g < Hkv; ++g)
    for (int j = 0; j < P; ++j) {
      real sum = 0;
      for (int h = g * G; h < (g + 1) * G; ++h) sum += p_head[(size_t)h * P + j];
      s_group[(size_t)g * P + j] = sum / (real)G;
    }
  for (int j = 0; j < P; ++j) {
    real sum = 0;
    for (int h = 0; h < Hq; ++h) sum += p_head[(size_t)h * P + j];
    s_tsp[j] = sum / (real)Hq;
  }
  return 0;
}

/* Step 6 (Sec. 4.2: top-ranked tokens up to the rate, window always kept and merged):
 * rank the P prefix tokens by (score descending, index ascending), keep the first
 * k-W, sort them ascending, then append P .. P+W-1.  scores are fp32: the ranking
 * is decided in the precision the GPU path ranks in. */
typedef struct { float s; int32_t i; } orc_item;
static int cmp_rank(const void *a, const void *b) {
  const orc_item *x = (const orc_item *)a, *y = (const orc_item *)b;
  if (x->s > y->s) return -1;
  if (x->s < y->s) return 1;
  return (x->i > y->i) - (x->i < y->i);
}
static int cmp_i32(const void *a, const void *b) {
  int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
  return (x > y) - (x < y);
}
int orc_select_topk(const float *scores, int P, int W, int k, int32_t *idx_out) {
  if (k < W || k > P + W || P < 0) return -1;
  const int kp = k - W;
  orc_item *it = (orc_item *)malloc((size_t)(P > 0 ? P : 1) * sizeof(orc_item));
  if (!it) return -2;
  for (int j = 0; j < P; ++j) { it[j].s = scores[j]; it[j].i = j; }
  qsort(it, (size_t)P, sizeof(orc_item), cmp_rank);
  for (int t = 0; t < kp; ++t) idx_out[t] = it[t].i;
  qsort(idx_out, (size_t)kp, sizeof(int32_t), cmp_i32);
  for (int w = 0; w < W; ++w) idx_out[kp + w] = P + w;
  free(it);
  return 0;
}

/* Step 7 (HiddenCompress / KVCompress, App. B.1): out[t] = the row_bytes bytes at
 * src + idx[t]*src_stride_bytes, copied bit for bit. */
int orc_gather_rows(const uint8_t *src, size_t src_stride_bytes, size_t row_bytes,
                    const int32_t *idx, int n, uint8_t *out) {
  for (int t = 0; t < n; ++t)
    memcpy(out + (size_t)t * row_bytes, src + (size_t)idx[t] * src_stride_bytes, row_bytes);
  return 0;
}

/* Decode-step attention over a (compressed) KV cache: the consumer of what KVCompress keeps
 * (Algorithm 1 returns the cache C; Sec. 5.3 measures decoding over it).  One new query token,
 * every cached token visible: out[h] = sum_t softmax_t(scale * q[h].k[g(h),t]) * v[g(h),t].
 * q [Hq][d] bf16 bits; k, v addressed as base + t*tok_stride + g*head_stride (in elements), so both
 * the compacted [Hkv][n][d] and the token-major [n][Hkv][d] layouts fit; out [Hq][d]. */
int orc_decode_attention(const uint16_t *q, const uint16_t *k, const uint16_t *v, int n, int Hq, int Hkv, int d,
                         long tok_stride, long head_stride, double scale, real *out) {
  if (n < 1 || Hq % Hkv != 0) return -1;
  const int G = Hq / Hkv;
  const real sc = (real)scale;
  real *p = (real *)malloc((size_t)n * sizeof(real));
  if (!p) return -2;
  for (int h = 0; h < Hq; ++h) {
    const int g = h / G;
    real m = 0;
    for (int t = 0; t < n; ++t) {
      const uint16_t *kv = k + (size_t)t * tok_stride + (size_t)g * head_stride;
      real acc = 0;
      for (int c = 0; c < d; ++c) acc += (real)bf16_to_f32(q[(size_t)h * d + c]) * (real)bf16_to_f32(kv[c]);
      p[t] = sc * acc;
      if (t == 0 || p[t] > m) m = p[t];
    }
    real Z = 0;
    for (int t = 0; t < n; ++t) { p[t] = REAL_EXP(p[t] - m); Z += p[t]; }
    for (int c = 0; c < d; ++c) {
      real acc = 0;
      for (int t = 0; t < n; ++t)
        acc += (p[t] / Z) * (real)bf16_to_f32(v[(size_t)t * tok_stride + (size_t)g * head_stride + c]);
      out[(size_t)h * d + c] = acc;
    }
  }
  free(p);
  return 0;
}
