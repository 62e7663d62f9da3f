/*
 * CPU oracle for the SparQ Attention single-token decode step.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the test-suite, the
 * smoke check and the benchmark's cpu_baseline leg may call it.  It shares no
 * code, header, table or helper with the HIP library, and it is written to be
 * checked against the paper by eye: one head at a time, the paper's steps in
 * the paper's order, fp64 arithmetic on the exactly-converted 16-bit inputs,
 * full sorts instead of selection, no blocking, no fusion.
 *
 * Equation numbers are the paper's own, counted from its first displayed equation: (2) dense
 * attention, (3) M_dense, (6) mean value reallocation, (7) approximate scores, (8) attention over
 * the selected positions, (9) temperature, (10) blend with the mean value vector.
 *
 * What each function follows:
 *   oracle_dense_decode      Section 3, Eq. (2)  (dense single-query attention)
 *   oracle_sparq_decode      Section 3 Eqs. (7)-(10), Section 4 Steps 1-3,
 *                            the GQA paragraph of Section 4, Appendix B
 *   oracle_mean_value        Section 3, "Mean value reallocation" (definition of v-bar)
 *   oracle_to_double         exact widening of IEEE binary16 / bfloat16
 *
 * Readings taken where the paper is silent (each also checked by a test):
 *   - top-r of |q| and top-k of the scores break ties towards the lower index;
 *   - selection is made on the approximate logit z (the softmax is monotone,
 *     so this is the ordering of s-hat without its underflow to zero);
 *   - k is clamped to the sequence length; an all-zero query gives tau = sqrt(d_h);
 *   - the current token has been appended before the step, rows >= S are invisible;
 *   - in grouped-query "shared" mode the group sum of s-hat decides the positions,
 *     tau and alpha stay per query head (Appendix B).
 *
 * Pins (tests/test_oracle_pins.py): r = d_h and k = S reproduces Eq. (2);
 * r = d_h with any k reproduces Eq. (6); the schematic's worked query; the
 * sqrt(r) <= tau <= sqrt(d_h) range; alpha = k/S for identical keys; brute
 * force on tiny inputs; permutation invariances; conversion of all 65536 codes.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F16 = 0, ORACLE_BF16 = 1 };
enum { ORACLE_NO_REALLOC = 1, ORACLE_GQA_SHARED = 2, ORACLE_TAU_SQRT_DH = 8, ORACLE_TAU_SQRT_R = 16 };

/* ---- exact widening of the 16-bit storage formats -------------------------------- */

static double f16_to_double(uint16_t h) {
  int sign = h >> 15, e = (h >> 10) & 31, m = h & 1023;
  double v;
  if (e == 0) v = ldexp((double)m, -24);                 /* subnormal: m * 2^-24 */
  else if (e == 31) v = m ? NAN : INFINITY;
  else v = ldexp((double)(1024 + m), e - 25);            /* (1 + m/1024) * 2^(e-15) */
  return sign ? -v : v;
}

static double bf16_to_double(uint16_t b) {
  int sign = b >> 15, e = (b >> 7) & 255, m = b & 127;
  double v;
  if (e == 0) v = ldexp((double)m, -133);                /* m/128 * 2^-126 */
  else if (e == 255) v = m ? NAN : INFINITY;
  else v = ldexp((double)(128 + m), e - 134);            /* (1 + m/128) * 2^(e-127) */
  return sign ? -v : v;
}

static double widen(uint16_t bits, int dtype) {
  return dtype == ORACLE_BF16 ? bf16_to_double(bits) : f16_to_double(bits);
}

int oracle_to_double(int dtype, const uint16_t* in, long n, double* out) {
  if (dtype != ORACLE_F16 && dtype != ORACLE_BF16) return -1;
  for (long i = 0; i < n; ++i) out[i] = widen(in[i], dtype);
  return 0;
}

/* ---- ranking: value descending, index ascending ---------------------------------- */

typedef struct { double v; int idx; } ranked;

static int by_value_desc_index_asc(const void* a, const void* b) {
  const ranked* x = (const ranked*)a; const ranked* y = (const ranked*)b;
  if (x->v > y->v) return -1;
  if (x->v < y->v) return 1;
  return (x->idx > y->idx) - (x->idx < y->idx);
}

static int by_int_asc(const void* a, const void* b) {
  int x = *(const int*)a, y = *(const int*)b;
  return (x > y) - (x < y);
}

/* indices of the `count` largest entries of v[0..n), ties to the lower index, returned ascending */
static void top_indices(const double* v, int n, int count, int* out) {
  ranked* order = (ranked*)malloc((size_t)n * sizeof(ranked));
  for (int i = 0; i < n; ++i) { order[i].v = v[i]; order[i].idx = i; }
  qsort(order, (size_t)n, sizeof(ranked), by_value_desc_index_asc);
  for (int i = 0; i < count; ++i) out[i] = order[i].idx;
  qsort(out, (size_t)count, sizeof(int), by_int_asc);
  free(order);
}

/* ---- Section 3, definition of the mean value vector ------------------------------ */

/* vbar[c] = (1/S) * sum_{i<S} V[i,c]   for one KV head; V is [S_max, d_h] */
static void mean_value(const uint16_t* V, int S, int d_h, int dtype, double* vbar) {
  for (int c = 0; c < d_h; ++c) vbar[c] = 0.0;
  for (int i = 0; i < S; ++i)
    for (int c = 0; c < d_h; ++c) vbar[c] += widen(V[(size_t)i * d_h + c], dtype);
  for (int c = 0; c < d_h; ++c) vbar[c] = S > 0 ? vbar[c] / (double)S : 0.0;
}

int oracle_mean_value(int B, int H_kv, int S_max, int d_h, int dtype, const uint16_t* V,
                      const int32_t* seq_lens, double* vbar /* [B,H_kv,d_h] */) {
  for (int b = 0; b < B; ++b)
    for (int h = 0; h < H_kv; ++h) {
      size_t u = (size_t)b * H_kv + h;
      mean_value(V + u * S_max * d_h, seq_lens[b], d_h, dtype, vbar + u * d_h);
    }
  return 0;
}

/* ---- Eq. (2): y = softmax(q K^T / sqrt(d_h)) V over the rows in `rows` ----------- */

/* exact attention restricted to the listed rows (all rows for the dense case) */
static void attention_over_rows(const double* q, const uint16_t* K, const uint16_t* V, int d_h,
                                int dtype, const int* rows, int n_rows, double* y) {
  double* logit = (double*)malloc((size_t)(n_rows > 0 ? n_rows : 1) * sizeof(double));
  double top = -INFINITY;
  for (int n = 0; n < n_rows; ++n) {
    const uint16_t* krow = K + (size_t)rows[n] * d_h;
    double dot = 0.0;
    for (int c = 0; c < d_h; ++c) dot += q[c] * widen(krow[c], dtype);
    logit[n] = dot / sqrt((double)d_h);
    if (logit[n] > top) top = logit[n];
  }
  double denom = 0.0;
  for (int n = 0; n < n_rows; ++n) { logit[n] = exp(logit[n] - top); denom += logit[n]; }
  for (int c = 0; c < d_h; ++c) y[c] = 0.0;
  for (int n = 0; n < n_rows; ++n) {
    const uint16_t* vrow = V + (size_t)rows[n] * d_h;
    double p = logit[n] / denom;
    for (int c = 0; c < d_h; ++c) y[c] += p * widen(vrow[c], dtype);
  }
  free(logit);
}

int oracle_dense_decode(int B, int H, int H_kv, int S_max, int d_h, int dtype,
                        const uint16_t* K, const uint16_t* V, const uint16_t* q,
                        const int32_t* seq_lens, double* y /* [B,H,d_h] */) {
  if (B < 1 || H < 1 || H_kv < 1 || H % H_kv || d_h < 1 || S_max < 1) return -1;
  int g = H / H_kv;
  int fail = 0;
#pragma omp parallel for collapse(2) schedule(dynamic) reduction(|:fail)
  for (int b = 0; b < B; ++b)
    for (int h = 0; h < H; ++h) {
      int S = seq_lens[b];
      double* yu = y + ((size_t)b * H + h) * d_h;
      if (S < 0 || S > S_max) { fail = 1; continue; }
      if (S == 0) { for (int c = 0; c < d_h; ++c) yu[c] = 0.0; continue; }
      size_t kv = ((size_t)b * H_kv + h / g) * S_max * d_h;
      double* qd = (double*)malloc((size_t)d_h * sizeof(double));
      int* rows = (int*)malloc((size_t)S * sizeof(int));
      for (int c = 0; c < d_h; ++c) qd[c] = widen(q[((size_t)b * H + h) * d_h + c], dtype);
      for (int i = 0; i < S; ++i) rows[i] = i;
      attention_over_rows(qd, K + kv, V + kv, d_h, dtype, rows, S, yu);
      free(rows); free(qd);
    }
  return fail ? -2 : 0;
}

/* ---- SparQ, one KV head with its g query heads ----------------------------------- */

typedef struct {
  int S_max, d_h, r, dtype, g, S, k_eff, k_stride, local_window;
  unsigned flags;
  const uint16_t *K, *V;          /* this KV head: [S_max, d_h] */
  const uint16_t* q;              /* the g query heads of the group: [g, d_h] */
  const int32_t* given_i2;        /* nullable, [g, k_stride], -1 padded */
  double *y, *alpha, *tau, *z;    /* [g,d_h], [g], [g], nullable [g,S_max] */
  int32_t *i1, *i2;               /* [g,r], [g,k_stride] */
} group_job;

static void sparq_group(const group_job* J) {
  const int g = J->g, d_h = J->d_h, r = J->r, S = J->S, dtype = J->dtype;
  const int shared = (J->flags & ORACLE_GQA_SHARED) != 0;
  double* qd = (double*)malloc((size_t)g * d_h * sizeof(double));
  double* shat = (double*)malloc((size_t)g * S * sizeof(double));
  double* zrow = (double*)malloc((size_t)g * S * sizeof(double));
  double* mag = (double*)malloc((size_t)d_h * sizeof(double));
  double* score = (double*)malloc((size_t)S * sizeof(double));
  double* vbar = (double*)malloc((size_t)d_h * sizeof(double));
  double* y3 = (double*)malloc((size_t)d_h * sizeof(double));
  int* chan = (int*)malloc((size_t)g * r * sizeof(int));
  int* pos = (int*)malloc((size_t)(J->k_eff > 0 ? J->k_eff : 1) * sizeof(int));

  for (int t = 0; t < g; ++t)
    for (int c = 0; c < d_h; ++c) qd[t * d_h + c] = widen(J->q[(size_t)t * d_h + c], dtype);

  /* Step 1: the r largest components of |q| (of the group sum of |q| in shared mode) */
  if (shared) {
    for (int c = 0; c < d_h; ++c) {
      mag[c] = 0.0;
      for (int t = 0; t < g; ++t) mag[c] += fabs(qd[t * d_h + c]);
    }
    top_indices(mag, d_h, r, chan);
    for (int t = 1; t < g; ++t) memcpy(chan + t * r, chan, (size_t)r * sizeof(int));
  } else {
    for (int t = 0; t < g; ++t) {
      for (int c = 0; c < d_h; ++c) mag[c] = fabs(qd[t * d_h + c]);
      top_indices(mag, d_h, r, chan + t * r);
    }
  }

  /* Step 1 continued: temperature (Eq. 9) and approximate scores (Eq. 7), per query head */
  for (int t = 0; t < g; ++t) {
    const double* qt = qd + t * d_h;
    const int* i1 = chan + t * r;
    double l1_all = 0.0, l1_sel = 0.0;
    for (int c = 0; c < d_h; ++c) l1_all += fabs(qt[c]);
    for (int j = 0; j < r; ++j) l1_sel += fabs(qt[i1[j]]);
    /* no mass on the selected channels (q = 0, or in shared mode a head that is zero on the group's
       channels): every logit is 0 whatever tau is; take sqrt(d_h) so that 0 / tau is defined */
    double tau = l1_sel > 0.0 ? sqrt((double)d_h * l1_sel / l1_all) : sqrt((double)d_h);
    /* the two fixed temperatures of the ablation (Section 5.3 'Approximate softmax temperature') */
    if (J->flags & ORACLE_TAU_SQRT_DH) tau = sqrt((double)d_h);
    if (J->flags & ORACLE_TAU_SQRT_R) tau = sqrt((double)r);
    J->tau[t] = tau;
    for (int j = 0; j < r; ++j) J->i1[t * r + j] = i1[j];

    double* z = zrow + (size_t)t * S;
    double top = -INFINITY;
    for (int i = 0; i < S; ++i) {
      const uint16_t* krow = J->K + (size_t)i * d_h;
      double dot = 0.0;
      for (int j = 0; j < r; ++j) dot += qt[i1[j]] * widen(krow[i1[j]], dtype);
      z[i] = dot / tau;
      if (z[i] > top) top = z[i];
    }
    double denom = 0.0;
    double* s = shat + (size_t)t * S;
    for (int i = 0; i < S; ++i) { s[i] = exp(z[i] - top); denom += s[i]; }
    for (int i = 0; i < S; ++i) s[i] /= denom;
    if (J->z) {
      for (int i = 0; i < S; ++i) J->z[(size_t)t * J->S_max + i] = z[i];
      for (int i = S; i < J->S_max; ++i) J->z[(size_t)t * J->S_max + i] = 0.0;
    }
  }

  if (!(J->flags & ORACLE_NO_REALLOC)) mean_value(J->V, S, d_h, dtype, vbar);

  /* Local window (Appendix 'Experimental setup', l): the l most recent positions are always selected,
     the other k - l are the best-scoring of the positions before them. */
  const int n_local = J->local_window < J->k_eff ? J->local_window : J->k_eff;
  const int n_top = J->k_eff - n_local, S_old = S - n_local;

  /* Steps 2 and 3, per query head; positions shared across the group in shared mode */
  for (int t = 0; t < g; ++t) {
    int n_pos = J->k_eff;
    if (J->given_i2) {
      n_pos = 0;
      for (int n = 0; n < J->k_stride; ++n) {
        int p = J->given_i2[(size_t)t * J->k_stride + n];
        if (p >= 0 && p < S && n_pos < J->k_eff) pos[n_pos++] = p;
      }
    } else if (shared) {
      if (t == 0) {
        for (int i = 0; i < S; ++i) {
          score[i] = 0.0;
          for (int u = 0; u < g; ++u) score[i] += shat[(size_t)u * S + i];
        }
        top_indices(score, S_old, n_top, pos);
        for (int i = 0; i < n_local; ++i) pos[n_top + i] = S_old + i;
      }
    } else {
      /* top-k of s-hat for one head == top-k of its logits z */
      top_indices(zrow + (size_t)t * S, S_old, n_top, pos);
      for (int i = 0; i < n_local; ++i) pos[n_top + i] = S_old + i;
    }
    for (int n = 0; n < J->k_stride; ++n)
      J->i2[(size_t)t * J->k_stride + n] = n < n_pos ? pos[n] : -1;

    /* Step 2: exact attention over the selected rows (Eq. 8 with epsilon -> 0) */
    attention_over_rows(qd + t * d_h, J->K, J->V, d_h, dtype, pos, n_pos, y3);

    /* Step 3: alpha = mass of the selected positions under s-hat; blend with v-bar (Eq. 10) */
    double alpha = 0.0;
    for (int n = 0; n < n_pos; ++n) alpha += shat[(size_t)t * S + pos[n]];
    J->alpha[t] = alpha;
    for (int c = 0; c < d_h; ++c)
      J->y[t * d_h + c] = (J->flags & ORACLE_NO_REALLOC) ? y3[c] : alpha * y3[c] + (1.0 - alpha) * vbar[c];
  }

  free(pos); free(chan); free(y3); free(vbar); free(score); free(mag); free(zrow); free(shat); free(qd);
}

/*
 * Whole batch.  All arrays are host memory.
 *   K, V      [B, H_kv, S_max, d_h]  raw 16-bit codes (dtype: 0 = binary16, 1 = bfloat16)
 *   q         [B, H, d_h]
 *   seq_lens  [B]; k_per_seq nullable [B] (overrides k); given_i2 nullable [B, H, k_stride]
 *   local_window  l >= 0: the min(l, k_b, S_b) most recent positions are selected unconditionally
 *   y [B,H,d_h], alpha [B,H], tau [B,H], i1 [B,H,r] ascending, i2 [B,H,k_stride] ascending, -1 padded,
 *   z nullable [B,H,S_max] (approximate logits; entries >= S set to 0)
 * Returns 0, or a negative code for invalid arguments.
 */
int oracle_sparq_decode(int B, int H, int H_kv, int S_max, int d_h, int r, int k, int local_window, int dtype,
                        unsigned flags, const uint16_t* K, const uint16_t* V, const uint16_t* q,
                        const int32_t* seq_lens, const int32_t* k_per_seq, const int32_t* given_i2,
                        int k_stride, double* y, double* alpha, double* tau, int32_t* i1,
                        int32_t* i2, double* z) {
  if (B < 1 || H < 1 || H_kv < 1 || H % H_kv || d_h < 1 || S_max < 1) return -1;
  if (r < 1 || r > d_h || k < 1 || k_stride < 1 || local_window < 0) return -1;
  if ((flags & ORACLE_TAU_SQRT_DH) && (flags & ORACLE_TAU_SQRT_R)) return -1;
  if (dtype != ORACLE_F16 && dtype != ORACLE_BF16) return -1;
  for (int b = 0; b < B; ++b) {
    int kb = k_per_seq ? k_per_seq[b] : k;
    int ke = kb < seq_lens[b] ? kb : seq_lens[b];
    if (seq_lens[b] < 0 || seq_lens[b] > S_max || kb < 1 || ke > k_stride) return -2;
  }
  const int g = H / H_kv;
#pragma omp parallel for collapse(2) schedule(dynamic)
  for (int b = 0; b < B; ++b)
    for (int hk = 0; hk < H_kv; ++hk) {
      size_t unit = (size_t)b * H + (size_t)hk * g;       /* first query head of the group */
      size_t kv = ((size_t)b * H_kv + hk) * S_max * d_h;
      int S = seq_lens[b];
      int kb = k_per_seq ? k_per_seq[b] : k;
      if (S == 0) {
        for (int t = 0; t < g; ++t) {
          for (int c = 0; c < d_h; ++c) y[(unit + t) * d_h + c] = 0.0;
          alpha[unit + t] = 0.0; tau[unit + t] = sqrt((double)d_h);
          for (int j = 0; j < r; ++j) i1[(unit + t) * r + j] = -1;
          for (int n = 0; n < k_stride; ++n) i2[(unit + t) * k_stride + n] = -1;
          if (z) for (int i = 0; i < S_max; ++i) z[(unit + t) * S_max + i] = 0.0;
        }
        continue;
      }
      group_job J;
      J.S_max = S_max; J.d_h = d_h; J.r = r; J.dtype = dtype; J.g = g; J.S = S;
      J.k_eff = kb < S ? kb : S; J.k_stride = k_stride; J.flags = flags; J.local_window = local_window;
      J.K = K + kv; J.V = V + kv; J.q = q + unit * d_h;
      J.given_i2 = given_i2 ? given_i2 + unit * k_stride : NULL;
      J.y = y + unit * d_h; J.alpha = alpha + unit; J.tau = tau + unit;
      J.z = z ? z + unit * S_max : NULL;
      J.i1 = i1 + unit * r; J.i2 = i2 + unit * k_stride;
      sparq_group(&J);
    }
  return 0;
}

int oracle_num_threads(void) {
  int n = 1;
#ifdef _OPENMP
#pragma omp parallel
  {
#pragma omp single
    n = omp_get_num_threads();
  }
#endif
  return n;
}
