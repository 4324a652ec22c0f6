/*
 * fp64 CPU oracle for span-restricted single-query (decode) attention.
 *
 * TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only the tests, the smoke check and the
 * benchmark's CPU-baseline leg may call this file.  It shares no code, header,
 * constant or helper with the HIP library, and nothing in the HIP library calls it.
 * It is deliberately plain and slow: no blocking, no fusion, no SIMD intrinsics.
 *
 * What it computes (Sec. 2.2 eqs. (4)-(6), restricted to the one query row of the
 * decoding phase, Sec. 2.2 "Token generation"; the additive mask of eq. (5) is 0 on
 * the span and -inf elsewhere, so the softmax normaliser runs over span positions
 * only, Sec. 3.3; Algorithm 1 is the blocked evaluation of the same quantity):
 *
 *   S_b      = union_i [starts[i], ends[i])  for i in [offsets[b], offsets[b+1])
 *   s_j      = scale * sum_t q[b,h,t] * K[b,h,j,t]                 j in S_b
 *   m        = max_j s_j ;  w_j = exp(s_j - m) ;  l = sum_j w_j
 *   out[b,h] = (1/l) * sum_j w_j * V[b,h,j,:]
 *
 * All arithmetic is IEEE double.  Inputs are the already-rounded fp32 / fp16 / bf16
 * values, widened exactly; `scale` is the fp32 value the library receives, widened.
 * The span is a SET of positions (a mask cannot count a position twice), so the
 * union is formed in a bitmap and positions are visited in ascending order.
 * A sequence whose span is empty gets an all-zero output row and its flag set.
 *
 * Pins (tests/test_oracle_pins.py): full cover == textbook softmax(qK^T*scale)V from a
 * library routine; single position -> that V row; brute-force additive-mask softmax over
 * all positions; closed forms (q = 0 -> mean of V rows, equal V rows, key shift
 * invariance, two-position logistic, dominant key); convexity; NaN outside the span has
 * no influence; group-wise (m, l, acc) states merged by log-sum-exp equal the one-shot
 * result; the validator is checked by exhaustive enumeration against a bitmap checker.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_F32 = 0, ORC_F16 = 1, ORC_BF16 = 2 };

/* Exact widening of one stored element to double. */
static double widen(const void* base, int dtype, size_t idx) {
  if (dtype == ORC_F32) return (double)((const float*)base)[idx];
  uint16_t h = ((const uint16_t*)base)[idx];
  if (dtype == ORC_BF16) {
    uint32_t u = (uint32_t)h << 16; /* bf16 is the top half of an IEEE binary32 */
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
  }
  /* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits */
  int sign = (h >> 15) & 1, e = (h >> 10) & 0x1f, frac = h & 0x3ff;
  double mag;
  if (e == 0) mag = ldexp((double)frac, -24);
  else if (e == 31) mag = frac ? NAN : INFINITY;
  else mag = ldexp(1.0 + (double)frac / 1024.0, e - 15);
  return sign ? -mag : mag;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Attention of one query row over an ascending list of positions of one (b,h) slab. */
static void attend_positions(int D, int dtype, const void* q, size_t q_off, const void* K, const void* V,
                             size_t slab_off, const int32_t* pos, int n, double scale, double* out) {
  for (int t = 0; t < D; ++t) out[t] = 0.0;
  if (n == 0) return;
  double* s = (double*)malloc(sizeof(double) * (size_t)n);
  double m = -INFINITY;
  for (int j = 0; j < n; ++j) {
    double dot = 0.0;
    size_t row = slab_off + (size_t)pos[j] * (size_t)D;
    for (int t = 0; t < D; ++t) dot += widen(q, dtype, q_off + t) * widen(K, dtype, row + t);
    s[j] = scale * dot;
    if (s[j] > m) m = s[j];
  }
  double l = 0.0;
  for (int j = 0; j < n; ++j) {
    s[j] = exp(s[j] - m);
    l += s[j];
  }
  for (int j = 0; j < n; ++j) {
    size_t row = slab_off + (size_t)pos[j] * (size_t)D;
    for (int t = 0; t < D; ++t) out[t] += s[j] * widen(V, dtype, row + t);
  }
  for (int t = 0; t < D; ++t) out[t] /= l;
  free(s);
}

/* Positions of the union of the intervals, ascending; positions outside [0, max_len) are dropped. */
static int span_positions(const int32_t* starts, const int32_t* ends, int lo, int hi, int max_len, int32_t* pos) {
  uint8_t* mark = (uint8_t*)calloc((size_t)max_len, 1);
  for (int i = lo; i < hi; ++i)
    for (int64_t p = starts[i]; p < ends[i]; ++p)
      if (p >= 0 && p < max_len) mark[p] = 1;
  int n = 0;
  for (int p = 0; p < max_len; ++p)
    if (mark[p]) pos[n++] = p;
  free(mark);
  return n;
}

/* q: [B,H,D]; K,V: [B,H,max_len,D]; out: [B,H,D] doubles; empty_flags: [B] or NULL. */
int oracle_span_attn(int B, int H, int D, int max_len, int dtype, const void* q, const void* K, const void* V,
                     const int32_t* offsets, const int32_t* starts, const int32_t* ends, float scale, double* out,
                     int32_t* empty_flags) {
  for (int b = 0; b < B; ++b) {
    int32_t* pos = (int32_t*)malloc(sizeof(int32_t) * (size_t)(max_len > 0 ? max_len : 1));
    int n = span_positions(starts, ends, offsets[b], offsets[b + 1], max_len, pos);
    if (empty_flags) empty_flags[b] = (n == 0);
#pragma omp parallel for schedule(dynamic)
    for (int h = 0; h < H; ++h) {
      size_t bh = (size_t)b * H + h;
      attend_positions(D, dtype, q, bh * D, K, V, bh * (size_t)max_len * D, pos, n, (double)scale, out + bh * D);
    }
    free(pos);
  }
  return 0;
}

/*
 * Few-query form: Qn query rows per sequence, one per consecutive new token, all sharing the sequence's
 * span.  Query j of sequence b attends the span positions p with p <= q_pos[b] + j: the causal mask of
 * Sec. 2.2 (a token never attends a later one) laid over the span mask of Sec. 3.3; eqs. (4)-(6) then
 * apply row by row.  q_pos NULL = no causal limit.  q, out: [B, Qn, H, D].
 */
int oracle_span_attn_multi(int B, int H, int D, int max_len, int dtype, int Qn, const void* q, const void* K,
                           const void* V, const int32_t* offsets, const int32_t* starts, const int32_t* ends,
                           const int32_t* q_pos, float scale, double* out) {
  for (int b = 0; b < B; ++b) {
    int32_t* pos = (int32_t*)malloc(sizeof(int32_t) * (size_t)(max_len > 0 ? max_len : 1));
    int n = span_positions(starts, ends, offsets[b], offsets[b + 1], max_len, pos);
    for (int j = 0; j < Qn; ++j) {
      int nj = n;  /* pos is ascending: the visible positions are a prefix of it */
      if (q_pos) {
        int64_t last = (int64_t)q_pos[b] + j;
        nj = 0;
        while (nj < n && pos[nj] <= last) ++nj;
      }
#pragma omp parallel for schedule(dynamic)
      for (int h = 0; h < H; ++h) {
        size_t row = ((size_t)b * Qn + j) * H + h;
        attend_positions(D, dtype, q, row * D, K, V, ((size_t)b * H + h) * (size_t)max_len * D, pos, nj,
                         (double)scale, out + row * D);
      }
    }
    free(pos);
  }
  return 0;
}

/* Dense control: S_b = [0, ctx_lens[b]). */
int oracle_dense_attn(int B, int H, int D, int max_len, int dtype, const void* q, const void* K, const void* V,
                      const int32_t* ctx_lens, float scale, double* out) {
  for (int b = 0; b < B; ++b) {
    int n = ctx_lens[b] < 0 ? 0 : (ctx_lens[b] > max_len ? max_len : ctx_lens[b]);
    int32_t* pos = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
    for (int p = 0; p < n; ++p) pos[p] = p;
#pragma omp parallel for schedule(dynamic)
    for (int h = 0; h < H; ++h) {
      size_t bh = (size_t)b * H + h;
      attend_positions(D, dtype, q, bh * D, K, V, bh * (size_t)max_len * D, pos, n, (double)scale, out + bh * D);
    }
    free(pos);
  }
  return 0;
}

/*
 * Softmax state of one (b,h) over the union of some intervals, un-normalised:
 *   m = max s_j, l = sum exp(s_j - m), acc = sum exp(s_j - m) V_j.
 * An empty group gives m = -inf, l = 0, acc = 0.
 */
int oracle_span_state(int H, int D, int max_len, int dtype, const void* q, const void* K, const void* V, int b, int h,
                      const int32_t* starts, const int32_t* ends, int n_intervals, float scale, double* m_out,
                      double* l_out, double* acc) {
  int32_t* pos = (int32_t*)malloc(sizeof(int32_t) * (size_t)(max_len > 0 ? max_len : 1));
  int n = span_positions(starts, ends, 0, n_intervals, max_len, pos);
  size_t bh = (size_t)b * H + h, slab = bh * (size_t)max_len * D;
  double m = -INFINITY, l = 0.0;
  for (int t = 0; t < D; ++t) acc[t] = 0.0;
  double* s = (double*)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
  for (int j = 0; j < n; ++j) {
    double dot = 0.0;
    for (int t = 0; t < D; ++t)
      dot += widen(q, dtype, bh * D + t) * widen(K, dtype, slab + (size_t)pos[j] * D + t);
    s[j] = (double)scale * dot;
    if (s[j] > m) m = s[j];
  }
  for (int j = 0; j < n; ++j) {
    double w = exp(s[j] - m);
    l += w;
    for (int t = 0; t < D; ++t) acc[t] += w * widen(V, dtype, slab + (size_t)pos[j] * D + t);
  }
  *m_out = m;
  *l_out = l;
  free(s);
  free(pos);
  return 0;
}

/*
 * Log-sum-exp merge of G group states into the normalised output:
 *   M = max_g m_g ;  out = sum_g e^{m_g - M} acc_g / sum_g e^{m_g - M} l_g.
 * This is the softmax of eq. (5) regrouped.  All groups empty -> zeros.
 */
int oracle_lse_merge(int G, int D, const double* m, const double* l, const double* acc, double* out) {
  double M = -INFINITY, L = 0.0;
  for (int g = 0; g < G; ++g)
    if (l[g] > 0.0 && m[g] > M) M = m[g];
  for (int t = 0; t < D; ++t) out[t] = 0.0;
  if (M == -INFINITY) return 0;
  for (int g = 0; g < G; ++g) {
    if (!(l[g] > 0.0)) continue;
    double w = exp(m[g] - M);
    L += w * l[g];
    for (int t = 0; t < D; ++t) out[t] += w * acc[(size_t)g * D + t];
  }
  for (int t = 0; t < D; ++t) out[t] /= L;
  return 0;
}

/*
 * Span-list validation.  Sequences are scanned in index order; within a sequence its
 * offsets are checked first, then its intervals in list order, each against the rules
 * in the order below; the first failure is reported as (code, sequence, interval index
 * within the sequence, or -1 when the failure is not tied to one interval).
 *   1 OFFSETS         offsets[0] != 0, or offsets[b+1] < offsets[b], or offsets[b+1] > num_intervals
 *                     (num_intervals = number of entries the starts / ends arrays hold)
 *   2 RANGE           start < 0 or end > ctx_lens[b]
 *   3 EMPTY_INTERVAL  start >= end
 *   4 OVERLAP         start_i >= start_{i-1} but start_i < end_{i-1}
 *   5 UNSORTED        start_i < start_{i-1}
 *   6 EMPTY_SPAN      the sequence has no interval
 * Adjacent intervals (start_i == end_{i-1}) are legal.  tokens_per_seq[b] (if given)
 * receives sum(end - start) for every sequence scanned before a failure, else all.
 */
int oracle_validate(int B, int num_intervals, const int32_t* offsets, const int32_t* starts, const int32_t* ends,
                    const int32_t* ctx_lens, int32_t* bad_seq, int32_t* bad_interval, int64_t* tokens_per_seq) {
  *bad_seq = -1;
  *bad_interval = -1;
  for (int b = 0; b < B; ++b) {
    if ((b == 0 && offsets[0] != 0) || offsets[b + 1] < offsets[b] || offsets[b + 1] > num_intervals) {
      *bad_seq = b;
      return 1;
    }
    int lo = offsets[b], hi = offsets[b + 1];
    if (hi == lo) {
      *bad_seq = b;
      return 6;
    }
    int64_t total = 0;
    for (int i = lo; i < hi; ++i) {
      int code = 0;
      if (starts[i] < 0 || ends[i] > ctx_lens[b]) code = 2;
      else if (starts[i] >= ends[i]) code = 3;
      else if (i > lo && starts[i] >= starts[i - 1] && starts[i] < ends[i - 1]) code = 4;
      else if (i > lo && starts[i] < starts[i - 1]) code = 5;
      if (code) {
        *bad_seq = b;
        *bad_interval = i - lo;
        return code;
      }
      total += (int64_t)ends[i] - (int64_t)starts[i];
    }
    if (tokens_per_seq) tokens_per_seq[b] = total;
  }
  return 0;
}
