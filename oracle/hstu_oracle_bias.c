/*
 * CPU oracle for jagged HSTU attention WITH the timestamp bias.  TEST INFRASTRUCTURE ONLY
 * (same rules as hstu_oracle.c: tests, smoke check and benchmark baseline only; nothing
 * shared with the GPU library).
 *
 * Paper, section 2.1: the attention equation has "+ Bias" inside the SiLU,
 *     HSTUAttention(Q,K,V) = Mask(SiLU((Q K^T + Bias)/sqrt(d_k))) V,
 * and the bias is described only in words: differences of the timestamps ts are taken (the
 * text speaks of consecutive elements), transformed, then grouped into bucket indices, which
 * select entries of a learnable table ts_weights.  The paper gives neither the transformation
 * nor the number of buckets, and a term added to Q K^T needs one value per (query, key) pair,
 * which differences of neighbouring rows alone do not give; the reading below takes the
 * difference of the pair's two timestamps (the sum of the consecutive differences between
 * them).  It is this build's own and PARITY WITH THE PAPER IS UNPINNED for it; what the pins
 * in tests/test_oracle_bias_pins.py fix is that this file computes the reading correctly.
 *
 * Reading.  Every row carries an int32 timestamp ts.  For a visible pair (query i, key j) of
 * one sequence
 *     delta  = |ts[i] - ts[j]|
 *     bucket = 0                                           if delta <= 1
 *            = min(NB-1, e*2^f + m)                        otherwise, with
 *                e = floor(log2(delta)),  m = the f bits below delta's leading one
 *                (delta >> (e-f) minus 2^f when e >= f, delta << (f-e) minus 2^f otherwise),
 * a logarithmic transformation with 2^f groups per octave, all in integer arithmetic (so that
 * no rounding decides a bucket).  Then, with the table w[NB] shared by all heads,
 *     x_ij = alpha * (<Q[i],K[j]> + w[bucket_ij])
 *     O[i] = (1/N) * sum_j silu(x_ij) * V[j]
 * and for a given dO, with sg = sigmoid(x), p = x*sg/N, dp = <dO[i],V[j]>/N, ds = dp*silu'(x):
 *     dV[j] += p*dO[i]   dQ[i] += alpha*ds*K[j]   dK[j] += alpha*ds*Q[i]
 *     dW[bucket_ij] += alpha*ds                      (summed over pairs and heads)
 * w = 0 gives hstu_oracle.c's results exactly.
 *
 * Double precision, one pair at a time, in the order of the definition.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static double sigmoid(double x) {
  if (x >= 0.0) return 1.0 / (1.0 + exp(-x));
  double e = exp(x);
  return e / (1.0 + e);
}

static double dot(const double* a, const double* b, int n) {
  double s = 0.0;
  for (int t = 0; t < n; ++t) s += a[t] * b[t];
  return s;
}

/* The bucket of a timestamp difference (see the header). */
int32_t hstu_oracle_bias_bucket(int64_t ts_i, int64_t ts_j, int32_t nb, int32_t f) {
  int64_t delta = ts_i - ts_j;
  if (delta < 0) delta = -delta;
  if (delta <= 1) return 0;
  int e = 0;
  while ((delta >> (e + 1)) != 0) ++e;          /* floor(log2(delta)) */
  int64_t top = e >= f ? (delta >> (e - f)) : (delta << (f - e));
  int64_t b = (int64_t)e * ((int64_t)1 << f) + (top - ((int64_t)1 << f));
  return (int32_t)(b < nb - 1 ? b : nb - 1);
}

/* Forward and, if d_o != NULL, backward over the whole jagged batch (single thread: the
 * table gradient is a sum over everything).  Any of o, dq, dk, dv_out, dw may be NULL. */
int hstu_oracle_bias(int32_t B, int32_t H, int32_t dqk, int32_t dv, int32_t max_len, double alpha,
                     int32_t causal, const int32_t* off, const int32_t* ts, int32_t nb, int32_t f,
                     const double* w, const double* q, const double* k, const double* v,
                     const double* d_o, double* o, double* dq, double* dk, double* dv_out,
                     double* dw) {
  if (B < 0 || H < 1 || dqk < 1 || dv < 1 || max_len < 1 || nb < 1 || f < 0 || f > 8) return -1;
  const double N = (double)max_len;
  const int64_t T = off[B];
  if (o) memset(o, 0, sizeof(double) * T * H * dv);
  if (dq) memset(dq, 0, sizeof(double) * T * H * dqk);
  if (dk) memset(dk, 0, sizeof(double) * T * H * dqk);
  if (dv_out) memset(dv_out, 0, sizeof(double) * T * H * dv);
  if (dw) memset(dw, 0, sizeof(double) * nb);
  for (int b = 0; b < B; ++b) {
    const int64_t s = off[b];
    const int L = off[b + 1] - off[b];
    if (L < 0) return -2;
    for (int i = 0; i < L; ++i) {
      const int jend = causal ? i : L - 1;
      for (int j = 0; j <= jend; ++j) {
        const int bucket = hstu_oracle_bias_bucket(ts[s + i], ts[s + j], nb, f);
        for (int h = 0; h < H; ++h) {
          const double* qi = q + ((s + i) * (int64_t)H + h) * dqk;
          const double* kj = k + ((s + j) * (int64_t)H + h) * dqk;
          const double* vj = v + ((s + j) * (int64_t)H + h) * dv;
          const double x = alpha * (dot(qi, kj, dqk) + w[bucket]);
          const double sg = sigmoid(x);
          const double p = x * sg / N;
          if (o) {
            double* oi = o + ((s + i) * (int64_t)H + h) * dv;
            for (int t = 0; t < dv; ++t) oi[t] += p * vj[t];
          }
          if (d_o) {
            const double* doi = d_o + ((s + i) * (int64_t)H + h) * dv;
            const double dp = dot(doi, vj, dv) / N;
            const double ds = dp * sg * (1.0 + x * (1.0 - sg));
            if (dv_out) {
              double* dvj = dv_out + ((s + j) * (int64_t)H + h) * dv;
              for (int t = 0; t < dv; ++t) dvj[t] += p * doi[t];
            }
            if (dq) {
              double* dqi = dq + ((s + i) * (int64_t)H + h) * dqk;
              for (int t = 0; t < dqk; ++t) dqi[t] += alpha * ds * kj[t];
            }
            if (dk) {
              double* dkj = dk + ((s + j) * (int64_t)H + h) * dqk;
              for (int t = 0; t < dqk; ++t) dkj[t] += alpha * ds * qi[t];
            }
            if (dw) dw[bucket] += alpha * ds;
          }
        }
      }
    }
  }
  return 0;
}

/* The same definition at chosen global rows only (rows do not interact): for row rows[r] of its
 * sequence, O and dQ of that row as a query, dK and dV of that row as a key; outputs are
 * [n, H, d].  d_o may be NULL (then only o is written).  Returns -3 if a row lies in no sequence. */
int hstu_oracle_bias_rows(int32_t B, int32_t H, int32_t dqk, int32_t dv, int32_t max_len,
                          double alpha, int32_t causal, const int32_t* off, const int32_t* ts,
                          int32_t nb, int32_t f, const double* w, const double* q, const double* k,
                          const double* v, const double* d_o, int32_t n, const int64_t* rows,
                          double* o, double* dq, double* dk, double* dv_out) {
  if (B < 0 || H < 1 || dqk < 1 || dv < 1 || max_len < 1 || nb < 1 || f < 0 || f > 8 || n < 0) return -1;
  const double N = (double)max_len;
  int bad = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int r = 0; r < n; ++r)
    for (int h = 0; h < H; ++h) {
      int b = -1;
      for (int c = 0; c < B; ++c)
        if (off[c] <= rows[r] && rows[r] < off[c + 1]) { b = c; break; }
      if (b < 0) {
#pragma omp atomic write
        bad = 1;
        continue;
      }
      const int64_t s = off[b];
      const int L = off[b + 1] - off[b];
      const int me = (int)(rows[r] - s);
      double* oi = o ? o + ((int64_t)r * H + h) * dv : NULL;
      double* dqi = (dq && d_o) ? dq + ((int64_t)r * H + h) * dqk : NULL;
      double* dkj = (dk && d_o) ? dk + ((int64_t)r * H + h) * dqk : NULL;
      double* dvj = (dv_out && d_o) ? dv_out + ((int64_t)r * H + h) * dv : NULL;
      if (oi) memset(oi, 0, sizeof(double) * dv);
      if (dqi) memset(dqi, 0, sizeof(double) * dqk);
      if (dkj) memset(dkj, 0, sizeof(double) * dqk);
      if (dvj) memset(dvj, 0, sizeof(double) * dv);
      /* the row as a query i = me against its visible keys */
      if (oi || dqi) {
        const double* qi = q + ((s + me) * (int64_t)H + h) * dqk;
        const double* doi = d_o ? d_o + ((s + me) * (int64_t)H + h) * dv : NULL;
        const int jend = causal ? me : L - 1;
        for (int j = 0; j <= jend; ++j) {
          const double* kj = k + ((s + j) * (int64_t)H + h) * dqk;
          const double* vj = v + ((s + j) * (int64_t)H + h) * dv;
          const double x = alpha * (dot(qi, kj, dqk) + w[hstu_oracle_bias_bucket(ts[s + me], ts[s + j], nb, f)]);
          const double sg = sigmoid(x);
          if (oi) {
            const double p = x * sg / N;
            for (int t = 0; t < dv; ++t) oi[t] += p * vj[t];
          }
          if (dqi) {
            const double ds = dot(doi, vj, dv) / N * sg * (1.0 + x * (1.0 - sg));
            for (int t = 0; t < dqk; ++t) dqi[t] += alpha * ds * kj[t];
          }
        }
      }
      /* the row as a key j = me against the queries that see it */
      if (dkj || dvj) {
        const double* kj = k + ((s + me) * (int64_t)H + h) * dqk;
        const double* vj = v + ((s + me) * (int64_t)H + h) * dv;
        for (int i = causal ? me : 0; i < L; ++i) {
          const double* qi = q + ((s + i) * (int64_t)H + h) * dqk;
          const double* doi = d_o + ((s + i) * (int64_t)H + h) * dv;
          const double x = alpha * (dot(qi, kj, dqk) + w[hstu_oracle_bias_bucket(ts[s + i], ts[s + me], nb, f)]);
          const double sg = sigmoid(x);
          if (dvj) {
            const double p = x * sg / N;
            for (int t = 0; t < dv; ++t) dvj[t] += p * doi[t];
          }
          if (dkj) {
            const double ds = dot(doi, vj, dv) / N * sg * (1.0 + x * (1.0 - sg));
            for (int t = 0; t < dqk; ++t) dkj[t] += alpha * ds * qi[t];
          }
        }
      }
    }
  return bad ? -3 : 0;
}
