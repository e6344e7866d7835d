/*
 * CPU oracle for jagged HSTU attention.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the yardstick the GPU library is checked against.  It may be
 * built and called from tests, from the smoke check and from the benchmark's
 * CPU-baseline leg, and from nowhere else; the GPU library never links it and
 * shares no header, helper or constant with it.
 *
 * What it computes (paper, section 2.1, the HSTU attention equation, with the
 * bias term taken as zero; section 2.2 for the jagged values + offsets
 * representation):
 *
 *     O[i] = (1/N) * sum over visible keys j of  silu(alpha * <Q[i],K[j]>) * V[j]
 *
 * per sequence and per head, silu(x) = x * sigmoid(x).  The mask sits outside
 * the SiLU: a masked pair contributes exactly nothing.  With causal != 0 key j
 * is visible to query i iff j <= i, positions counted inside the sequence;
 * with causal == 0 every key of the same sequence is visible.  N is the
 * caller's max_len scalar (a plain normaliser; N = 1 gives the equation as it
 * is printed).  alpha is the scale inside the SiLU (the equation's 1/sqrt(d_k)).
 *
 * The backward pass is the exact derivative of that sum for a given dO:
 *     x  = alpha*<Q[i],K[j]>,  sg = sigmoid(x),  p = x*sg/N
 *     dp = <dO[i],V[j]>/N,     ds = dp * sg*(1 + x*(1-sg))        (silu'(x))
 *     dV[j] += p*dO[i]    dQ[i] += alpha*ds*K[j]    dK[j] += alpha*ds*Q[i]
 *
 * The context-parallel partial (paper, section 2.3, the load-balancing
 * paragraph: every sequence is cut into 2*CP mini-chunks and rank r owns
 * mini-chunks r and 2*CP-1-r) is the same sum restricted to the query rows a
 * rank owns and to the key rows of one rank (or of all ranks), with the causal
 * test taken on positions inside the whole sequence.
 *
 * Everything is double precision, one (i, j) pair at a time, in the order of
 * the definition: no blocking, no fusion, no reordering.  Threads (OpenMP)
 * split only over independent output rows.
 *
 * Layouts: q, k: [T, H, d_qk]; v, o, d_o: [T, H, d_v]; row-major, contiguous;
 * row t belongs to sequence b iff off[b] <= t < off[b+1].
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Overflow-free logistic function. */
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

int hstu_oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* silu and its derivative, exported so tests can pin them to textbook values. */
double hstu_oracle_silu(double x) { return x * sigmoid(x); }
double hstu_oracle_silu_grad(double x) {
  double sg = sigmoid(x);
  return sg * (1.0 + x * (1.0 - sg));
}

/* ------------------------------------------------------------------------- */
/* Full attention, one query row.                                            */
/* ------------------------------------------------------------------------- */

/* O row (and, if d_o != NULL, dQ row) of query row i (in-sequence index) of
 * sequence [s, s+L), head h. */
static void query_row(int H, int dqk, int dv, double N, double alpha, int causal,
                      int64_t s, int L, int i, int h,
                      const double* q, const double* k, const double* v, const double* d_o,
                      double* o_row, double* dq_row) {
  const double* qi = q + ((s + i) * (int64_t)H + h) * dqk;
  const double* doi = d_o ? d_o + ((s + i) * (int64_t)H + h) * dv : NULL;
  if (o_row) memset(o_row, 0, sizeof(double) * dv);
  if (dq_row) memset(dq_row, 0, sizeof(double) * dqk);
  int jend = causal ? i : L - 1;
  for (int j = 0; j <= jend; ++j) {
    const double* kj = k + ((s + j) * (int64_t)H + h) * dqk;
    const double* vj = v + ((s + j) * (int64_t)H + h) * dv;
    double x = alpha * dot(qi, kj, dqk);
    double sg = sigmoid(x);
    double p = x * sg / N;
    if (o_row)
      for (int t = 0; t < dv; ++t) o_row[t] += p * vj[t];
    if (dq_row) {
      double dp = dot(doi, vj, dv) / N;
      double ds = dp * sg * (1.0 + x * (1.0 - sg));
      for (int t = 0; t < dqk; ++t) dq_row[t] += alpha * ds * kj[t];
    }
  }
}

/* dK row and dV row of key row j (in-sequence index). */
static void key_row(int H, int dqk, int dv, double N, double alpha, int causal,
                    int64_t s, int L, int j, int h,
                    const double* q, const double* k, const double* v, const double* d_o,
                    double* dk_row, double* dv_row) {
  const double* kj = k + ((s + j) * (int64_t)H + h) * dqk;
  const double* vj = v + ((s + j) * (int64_t)H + h) * dv;
  memset(dk_row, 0, sizeof(double) * dqk);
  memset(dv_row, 0, sizeof(double) * dv);
  int ibeg = causal ? j : 0;
  for (int i = ibeg; i < L; ++i) {
    const double* qi = q + ((s + i) * (int64_t)H + h) * dqk;
    const double* doi = d_o + ((s + i) * (int64_t)H + h) * dv;
    double x = alpha * dot(qi, kj, dqk);
    double sg = sigmoid(x);
    double p = x * sg / N;
    double dp = dot(doi, vj, dv) / N;
    double ds = dp * sg * (1.0 + x * (1.0 - sg));
    for (int t = 0; t < dv; ++t) dv_row[t] += p * doi[t];
    for (int t = 0; t < dqk; ++t) dk_row[t] += alpha * ds * qi[t];
  }
}

/* Forward over the whole jagged batch.  o: [T, H, d_v]. */
int hstu_oracle_fwd(int32_t B, int32_t H, int32_t dqk, int32_t dv, int32_t max_len,
                    double alpha, int32_t causal, const int32_t* off,
                    const double* q, const double* k, const double* v, double* o) {
  if (B < 0 || H < 1 || dqk < 1 || dv < 1 || max_len < 1) return -1;
  for (int b = 0; b < B; ++b) {
    int64_t s = off[b];
    int L = off[b + 1] - off[b];
    if (L < 0) return -2;
#pragma omp parallel for collapse(2) schedule(dynamic, 8)
    for (int i = 0; i < L; ++i)
      for (int h = 0; h < H; ++h)
        query_row(H, dqk, dv, (double)max_len, alpha, causal, s, L, i, h, q, k, v, NULL,
                  o + ((s + i) * (int64_t)H + h) * dv, NULL);
  }
  return 0;
}

/* Backward over the whole jagged batch.  dq, dk: [T, H, d_qk]; dv_out: [T, H, d_v]. */
int hstu_oracle_bwd(int32_t B, int32_t H, int32_t dqk, int32_t dv, int32_t max_len,
                    double alpha, int32_t causal, const int32_t* off,
                    const double* q, const double* k, const double* v, const double* d_o,
                    double* dq, double* dk, double* dv_out) {
  if (B < 0 || H < 1 || dqk < 1 || dv < 1 || max_len < 1) return -1;
  for (int b = 0; b < B; ++b) {
    int64_t s = off[b];
    int L = off[b + 1] - off[b];
    if (L < 0) return -2;
#pragma omp parallel for collapse(2) schedule(dynamic, 8)
    for (int i = 0; i < L; ++i)
      for (int h = 0; h < H; ++h) {
        query_row(H, dqk, dv, (double)max_len, alpha, causal, s, L, i, h, q, k, v, d_o, NULL,
                  dq + ((s + i) * (int64_t)H + h) * dqk);
        key_row(H, dqk, dv, (double)max_len, alpha, causal, s, L, i, h, q, k, v, d_o,
                dk + ((s + i) * (int64_t)H + h) * dqk, dv_out + ((s + i) * (int64_t)H + h) * dv);
      }
  }
  return 0;
}

/* Sequence that holds global row t, or -1. */
static int find_seq(int32_t B, const int32_t* off, int64_t t) {
  for (int b = 0; b < B; ++b)
    if (t >= off[b] && t < off[b + 1]) return b;
  return -1;
}

/* Exact values at chosen rows only.  Because the SiLU is pointwise there is no
 * coupling between rows: O[i], dQ[i] need only row i and its visible keys,
 * dK[j], dV[j] only column j and the queries that see it.  rows[] holds global
 * row indices; outputs are [n, H, d] in the order of rows[].  Any output
 * pointer may be NULL (d_o may be NULL when only o is wanted). */
int hstu_oracle_rows(int32_t B, int32_t H, int32_t dqk, int32_t dv, int32_t max_len,
                     double alpha, int32_t causal, const int32_t* off,
                     const double* q, const double* k, const double* v, const double* d_o,
                     int32_t n, const int64_t* rows,
                     double* o, double* dq, double* dk, double* dv_out) {
  if (B < 0 || H < 1 || dqk < 1 || dv < 1 || max_len < 1 || n < 0) return -1;
  int bad = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int r = 0; r < n; ++r)
    for (int h = 0; h < H; ++h) {
      int b = find_seq(B, off, rows[r]);
      if (b < 0) {
#pragma omp atomic write
        bad = 1;
        continue;
      }
      int64_t s = off[b];
      int L = off[b + 1] - off[b];
      int i = (int)(rows[r] - s);
      if (o || dq)
        query_row(H, dqk, dv, (double)max_len, alpha, causal, s, L, i, h, q, k, v,
                  dq ? d_o : NULL, o ? o + ((int64_t)r * H + h) * dv : NULL,
                  dq ? dq + ((int64_t)r * H + h) * dqk : NULL);
      if (dk && dv_out)
        key_row(H, dqk, dv, (double)max_len, alpha, causal, s, L, i, h, q, k, v, d_o,
                dk + ((int64_t)r * H + h) * dqk, dv_out + ((int64_t)r * H + h) * dv);
    }
  return bad ? -3 : 0;
}

/* ------------------------------------------------------------------------- */
/* Context-parallel partial.                                                 */
/* ------------------------------------------------------------------------- */

/* Mini-chunk m of a sequence of length L under a 2*CP-way split: chunk size
 * c = ceil(L / (2*CP)); chunk m covers in-sequence positions
 * [m*c, min((m+1)*c, L)), possibly fewer than c, possibly none. */
static void chunk_range(int L, int cp, int m, int* beg, int* end) {
  int c = (L + 2 * cp - 1) / (2 * cp);
  int64_t lo = (int64_t)m * c, hi = (int64_t)(m + 1) * c;
  if (lo > L) lo = L;
  if (hi > L) hi = L;
  *beg = (int)lo;
  *end = (int)hi;
}

/* Number of rows rank r owns in a sequence of length L. */
static int rank_rows(int L, int cp, int r) {
  int b0, e0, b1, e1;
  chunk_range(L, cp, r, &b0, &e0);
  chunk_range(L, cp, 2 * cp - 1 - r, &b1, &e1);
  return (e0 - b0) + (e1 - b1);
}

/* Rows a rank holds, in its local order: for each sequence in turn, the rows
 * of mini-chunk r and then those of mini-chunk 2*CP-1-r.  Writes, per local
 * row, the sequence index and the in-sequence position; returns the count.
 * rank < 0 means "all rows, global layout" (local row == global row). */
static int64_t local_rows(int32_t B, const int32_t* off, int cp, int rank,
                          int32_t* seq_of, int32_t* pos_of) {
  int64_t n = 0;
  for (int b = 0; b < B; ++b) {
    int L = off[b + 1] - off[b];
    if (rank < 0) {
      for (int p = 0; p < L; ++p) { if (seq_of) { seq_of[n] = b; pos_of[n] = p; } ++n; }
      continue;
    }
    int m[2] = {rank, 2 * cp - 1 - rank};
    for (int u = 0; u < 2; ++u) {
      int beg, end;
      chunk_range(L, cp, m[u], &beg, &end);
      for (int p = beg; p < end; ++p) { if (seq_of) { seq_of[n] = b; pos_of[n] = p; } ++n; }
    }
  }
  return n;
}

/* Row count of a rank's local layout (rank < 0: all rows). */
int64_t hstu_oracle_cp_local_rows(int32_t B, const int32_t* off, int32_t cp, int32_t rank) {
  return local_rows(B, off, cp, rank, NULL, NULL);
}

/* Fills seq_of[n], pos_of[n] for a rank's local layout; returns n. */
int64_t hstu_oracle_cp_local_map(int32_t B, const int32_t* off, int32_t cp, int32_t rank,
                                 int32_t* seq_of, int32_t* pos_of) {
  return local_rows(B, off, cp, rank, seq_of, pos_of);
}

/* One rank's partial result against one rank's keys (kv_rank >= 0) or against
 * all keys in the global layout (kv_rank < 0).
 *   q_local, d_o_local, o_local, dq_local : q_rank's local layout
 *   k_part, v_part, dk_part, dv_part      : kv_rank's local layout, or global
 * Outputs are overwritten with this partial alone (summing partials is the
 * caller's business).  d_o_local == NULL: forward only.  When n_sel_q >= 0
 * only the listed local query rows get o/dq (others are left untouched); the
 * same for n_sel_k and dk/dv.  A negative count means "all rows". */
int hstu_oracle_cp_partial(int32_t B, int32_t H, int32_t dqk, int32_t dv, int32_t max_len,
                           double alpha, int32_t causal, const int32_t* off,
                           int32_t cp, int32_t q_rank, int32_t kv_rank,
                           const double* q_local, const double* k_part, const double* v_part,
                           const double* d_o_local,
                           double* o_local, double* dq_local, double* dk_part, double* dv_part,
                           int64_t n_sel_q, const int64_t* sel_q,
                           int64_t n_sel_k, const int64_t* sel_k) {
  if (B < 0 || H < 1 || dqk < 1 || dv < 1 || max_len < 1) return -1;
  if (cp < 1 || q_rank < 0 || q_rank >= cp || kv_rank >= cp) return -4;
  int64_t T = off[B];
  int64_t cap = T + 1;
  int32_t* qseq = malloc(sizeof(int32_t) * cap);
  int32_t* qpos = malloc(sizeof(int32_t) * cap);
  int32_t* kseq = malloc(sizeof(int32_t) * cap);
  int32_t* kpos = malloc(sizeof(int32_t) * cap);
  int64_t* qbeg = malloc(sizeof(int64_t) * (B + 1)); /* first local q row of each sequence */
  int64_t* kbeg = malloc(sizeof(int64_t) * (B + 1));
  if (!qseq || !qpos || !kseq || !kpos || !qbeg || !kbeg) return -5;
  int64_t nq = local_rows(B, off, cp, q_rank, qseq, qpos);
  int64_t nk = local_rows(B, off, cp, kv_rank, kseq, kpos);
  qbeg[0] = kbeg[0] = 0;
  for (int b = 0; b < B; ++b) {
    int L = off[b + 1] - off[b];
    qbeg[b + 1] = qbeg[b] + rank_rows(L, cp, q_rank);
    kbeg[b + 1] = kbeg[b] + (kv_rank < 0 ? L : rank_rows(L, cp, kv_rank));
  }
  const double N = (double)max_len;

  /* query side: o and dq of every (selected) local query row */
  int64_t nqi = n_sel_q >= 0 ? n_sel_q : nq;
  if (o_local || dq_local) {
#pragma omp parallel for collapse(2) schedule(dynamic, 4)
    for (int64_t u = 0; u < nqi; ++u)
      for (int h = 0; h < H; ++h) {
        int64_t a = n_sel_q >= 0 ? sel_q[u] : u;
        if (a < 0 || a >= nq) continue;
        int b = qseq[a];
        const double* qi = q_local + (a * H + h) * dqk;
        const double* doi = d_o_local ? d_o_local + (a * H + h) * dv : NULL;
        double* orow = o_local ? o_local + (a * H + h) * dv : NULL;
        double* dqrow = (dq_local && doi) ? dq_local + (a * H + h) * dqk : NULL;
        if (orow) memset(orow, 0, sizeof(double) * dv);
        if (dqrow) memset(dqrow, 0, sizeof(double) * dqk);
        for (int64_t c = kbeg[b]; c < kbeg[b + 1]; ++c) {
          if (causal && kpos[c] > qpos[a]) continue;
          const double* kj = k_part + (c * H + h) * dqk;
          const double* vj = v_part + (c * H + h) * dv;
          double x = alpha * dot(qi, kj, dqk);
          double sg = sigmoid(x);
          double p = x * sg / N;
          if (orow)
            for (int t = 0; t < dv; ++t) orow[t] += p * vj[t];
          if (dqrow) {
            double dp = dot(doi, vj, dv) / N;
            double ds = dp * sg * (1.0 + x * (1.0 - sg));
            for (int t = 0; t < dqk; ++t) dqrow[t] += alpha * ds * kj[t];
          }
        }
      }
  }

  /* key side: dk and dv of every (selected) key row of the part */
  int64_t nki = n_sel_k >= 0 ? n_sel_k : nk;
  if (d_o_local && dk_part && dv_part) {
#pragma omp parallel for collapse(2) schedule(dynamic, 4)
    for (int64_t u = 0; u < nki; ++u)
      for (int h = 0; h < H; ++h) {
        int64_t c = n_sel_k >= 0 ? sel_k[u] : u;
        if (c < 0 || c >= nk) continue;
        int b = kseq[c];
        const double* kj = k_part + (c * H + h) * dqk;
        const double* vj = v_part + (c * H + h) * dv;
        double* dkrow = dk_part + (c * H + h) * dqk;
        double* dvrow = dv_part + (c * H + h) * dv;
        memset(dkrow, 0, sizeof(double) * dqk);
        memset(dvrow, 0, sizeof(double) * dv);
        for (int64_t a = qbeg[b]; a < qbeg[b + 1]; ++a) {
          if (causal && kpos[c] > qpos[a]) continue;
          const double* qi = q_local + (a * H + h) * dqk;
          const double* doi = d_o_local + (a * H + h) * dv;
          double x = alpha * dot(qi, kj, dqk);
          double sg = sigmoid(x);
          double p = x * sg / N;
          double dp = dot(doi, vj, dv) / N;
          double ds = dp * sg * (1.0 + x * (1.0 - sg));
          for (int t = 0; t < dv; ++t) dvrow[t] += p * doi[t];
          for (int t = 0; t < dqk; ++t) dkrow[t] += alpha * ds * qi[t];
        }
      }
  }
  free(qseq); free(qpos); free(kseq); free(kpos); free(qbeg); free(kbeg);
  return 0;
}
