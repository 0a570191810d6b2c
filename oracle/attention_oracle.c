/*
 * Standard (non-fused) scaled dot-product attention in fp64 -- TEST INFRASTRUCTURE ONLY.
 *
 * This file is the correctness oracle for the fused GPU forward pass.  It is the plain
 * definition of the operation, the paper's Algorithm 1 ("Standard Attention") together
 * with the formula of Section 2,
 *
 *      S = scale * Q K^T ,   P = softmax_rows(S) ,   O = P V ,
 *
 * evaluated head by head with S and P fully materialised, each row's softmax done in two
 * passes over the complete row (max, then exp and sum).  Nothing here is tiled, fused,
 * online or reordered; it shares no code, header, table or helper with the GPU library
 * and must never be linked into or called from the product path.  Only the tests, the
 * smoke check and the benchmark's cpu_baseline leg use it.
 *
 * The paper fixes no log-sum-exp output (Algorithm 2 writes only O).  LSE here is the
 * natural logarithm of the softmax denominator taken over the *scaled* logits,
 *      LSE_i = ln sum_j exp(S_ij) = m_i + ln(sum_j exp(S_ij - m_i)),
 * which is the quantity needed to merge attention over disjoint key sets.
 *
 * Tensor layout (Section 2: Q, K, V have shape (batch, seqlen, heads, headdim)):
 *      element (b, n, h, k) of Q/K/V/O lives at ((b*N + n)*H + h)*d + k,
 *      LSE (b, h, n) lives at (b*H + h)*N + n.
 * Q and O have Nq rows per head, K and V have Nk rows; the paper's workloads use Nq == Nk.
 *
 * Build:  gcc -O2 -fopenmp -shared -fPIC attention_oracle.c -o libattention_oracle.so -lm
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_ERR_ARG (-1)
#define ORACLE_ERR_NOMEM (-2)

static size_t qkv_index(int b, int n, int h, int k, int N, int H, int d) {
  return (((size_t)b * (size_t)N + (size_t)n) * (size_t)H + (size_t)h) * (size_t)d + (size_t)k;
}

/*
 * One block of `rows` complete rows [i0, i0+rows) of head (b, h).
 * S and P are caller-provided scratch of rows*Nk doubles each and hold, on return, the full
 * rows of the scaled logits and of the softmax.  Follows Algorithm 1 step by step.
 */
static void attention_row_block(const double* Q, const double* K, const double* V, int H, int Nq, int Nk,
                                int d, double scale, int causal, int b, int h, int i0, int rows, double* S,
                                double* P, double* O_rows /* rows*d */, double* LSE_rows /* rows */) {
  /* GEMM-I: S = scale * Q K^T  (Algorithm 1, "Compute S"; the scale sits inside S, Section 2). */
  for (int r = 0; r < rows; ++r) {
    const double* q = Q + qkv_index(b, i0 + r, h, 0, Nq, H, d);
    for (int j = 0; j < Nk; ++j) {
      const double* kj = K + qkv_index(b, j, h, 0, Nk, H, d);
      double acc = 0.0;
      for (int k = 0; k < d; ++k) acc += q[k] * kj[k];
      S[(size_t)r * Nk + j] = scale * acc;
    }
  }
  /* Optional masking of S (Section 2, footnote to the attention formula).  Causal mask: query row i sees
   * keys j <= i only; a masked logit is -infinity, so its softmax weight is exactly zero.  Key 0 is
   * visible to every row, hence every row keeps a finite maximum. */
  if (causal) {
    for (int r = 0; r < rows; ++r)
      for (int j = i0 + r + 1; j < Nk; ++j) S[(size_t)r * Nk + j] = -INFINITY;
  }
  /* Row softmax of the complete row, shifted by the row maximum (Algorithm 1, the "S - rowmax(S)"
   * and "P = softmax(S)" steps; the shift leaves the softmax unchanged, Section 2).  S itself is
   * kept unshifted so callers can inspect the logits. */
  for (int r = 0; r < rows; ++r) {
    double* s = S + (size_t)r * Nk;
    double* p = P + (size_t)r * Nk;
    double m = s[0];
    for (int j = 1; j < Nk; ++j)
      if (s[j] > m) m = s[j];
    double l = 0.0;
    for (int j = 0; j < Nk; ++j) {
      p[j] = exp(s[j] - m);
      l += p[j];
    }
    for (int j = 0; j < Nk; ++j) p[j] = p[j] / l;
    LSE_rows[r] = m + log(l);
  }
  /* GEMM-II: O = P V  (Algorithm 1, "Compute O"). */
  for (int r = 0; r < rows; ++r) {
    const double* p = P + (size_t)r * Nk;
    double* o = O_rows + (size_t)r * d;
    for (int k = 0; k < d; ++k) o[k] = 0.0;
    for (int j = 0; j < Nk; ++j) {
      const double* vj = V + qkv_index(b, j, h, 0, Nk, H, d);
      const double pj = p[j];
      for (int k = 0; k < d; ++k) o[k] += pj * vj[k];
    }
  }
}

static int check_shape(const void* Q, const void* K, const void* V, int B, int H, int Nq, int Nk, int d,
                       double scale) {
  if (!Q || !K || !V) return ORACLE_ERR_ARG;
  if (B <= 0 || H <= 0 || Nq <= 0 || Nk <= 0 || d <= 0) return ORACLE_ERR_ARG;
  if (!(scale == scale) || isinf(scale)) return ORACLE_ERR_ARG;
  return ORACLE_OK;
}

/*
 * Full forward: every (b, h, row).  O is [B][Nq][H][d] fp64 (never rounded to 16 bits), LSE is
 * [B][H][Nq].  Either output may be NULL.  Rows are processed in blocks of `row_block` complete
 * rows only to bound the memory of the materialised S and P (2 * row_block * Nk doubles per
 * thread); the arithmetic of a row does not depend on the block size.
 */
int fa_oracle_forward_masked(const double* Q, const double* K, const double* V, double* O, double* LSE, int B,
                             int H, int Nq, int Nk, int d, double scale, int causal, int row_block) {
  int rc = check_shape(Q, K, V, B, H, Nq, Nk, d, scale);
  if (rc != ORACLE_OK) return rc;
  if (causal && Nq != Nk) return ORACLE_ERR_ARG; /* the causal mask is defined for self-attention shapes */
  if (row_block <= 0) row_block = 32;
  if (row_block > Nq) row_block = Nq;
  const int nblk = (Nq + row_block - 1) / row_block;
  const long total = (long)B * H * nblk;
  int failed = 0;
#pragma omp parallel
  {
    double* S = (double*)malloc(sizeof(double) * (size_t)row_block * (size_t)Nk);
    double* P = (double*)malloc(sizeof(double) * (size_t)row_block * (size_t)Nk);
    double* Ob = (double*)malloc(sizeof(double) * (size_t)row_block * (size_t)d);
    double* Lb = (double*)malloc(sizeof(double) * (size_t)row_block);
    if (!S || !P || !Ob || !Lb) {
#pragma omp atomic write
      failed = 1;
    }
#pragma omp barrier
    int stop;
#pragma omp atomic read
    stop = failed;
    if (!stop) {
#pragma omp for schedule(dynamic, 1)
      for (long t = 0; t < total; ++t) {
        const int blk = (int)(t % nblk);
        const int h = (int)((t / nblk) % H);
        const int b = (int)(t / ((long)nblk * H));
        const int i0 = blk * row_block;
        const int rows = (i0 + row_block <= Nq) ? row_block : (Nq - i0);
        attention_row_block(Q, K, V, H, Nq, Nk, d, scale, causal, b, h, i0, rows, S, P, Ob, Lb);
        for (int r = 0; r < rows; ++r) {
          if (O) {
            double* dst = O + qkv_index(b, i0 + r, h, 0, Nq, H, d);
            for (int k = 0; k < d; ++k) dst[k] = Ob[(size_t)r * d + k];
          }
          if (LSE) LSE[((size_t)b * H + h) * (size_t)Nq + (size_t)(i0 + r)] = Lb[r];
        }
      }
    }
    free(S);
    free(P);
    free(Ob);
    free(Lb);
  }
  return failed ? ORACLE_ERR_NOMEM : ORACLE_OK;
}

/* Unmasked forward (the paper's workloads): fa_oracle_forward_masked without a mask. */
int fa_oracle_forward(const double* Q, const double* K, const double* V, double* O, double* LSE, int B,
                      int H, int Nq, int Nk, int d, double scale, int row_block) {
  return fa_oracle_forward_masked(Q, K, V, O, LSE, B, H, Nq, Nk, d, scale, 0, row_block);
}

/*
 * Sampled rows: for t in [0, n_rows) compute query row rows_bhi[3t+2] of head
 * (rows_bhi[3t], rows_bhi[3t+1]).  O_rows is [n_rows][d], LSE_rows is [n_rows].
 * Each sampled row is a complete, two-pass softmax over all Nk keys.
 */
int fa_oracle_rows_masked(const double* Q, const double* K, const double* V, const int* rows_bhi, int n_rows,
                          double* O_rows, double* LSE_rows, int B, int H, int Nq, int Nk, int d, double scale,
                          int causal) {
  int rc = check_shape(Q, K, V, B, H, Nq, Nk, d, scale);
  if (rc != ORACLE_OK) return rc;
  if (causal && Nq != Nk) return ORACLE_ERR_ARG;
  if (n_rows < 0 || (n_rows > 0 && (!rows_bhi || !O_rows || !LSE_rows))) return ORACLE_ERR_ARG;
  for (int t = 0; t < n_rows; ++t) {
    if (rows_bhi[3 * t] < 0 || rows_bhi[3 * t] >= B || rows_bhi[3 * t + 1] < 0 || rows_bhi[3 * t + 1] >= H ||
        rows_bhi[3 * t + 2] < 0 || rows_bhi[3 * t + 2] >= Nq)
      return ORACLE_ERR_ARG;
  }
  int failed = 0;
#pragma omp parallel
  {
    double* S = (double*)malloc(sizeof(double) * (size_t)Nk);
    double* P = (double*)malloc(sizeof(double) * (size_t)Nk);
    if (!S || !P) {
#pragma omp atomic write
      failed = 1;
    }
#pragma omp barrier
    int stop;
#pragma omp atomic read
    stop = failed;
    if (!stop) {
#pragma omp for schedule(dynamic, 1)
      for (int t = 0; t < n_rows; ++t) {
        attention_row_block(Q, K, V, H, Nq, Nk, d, scale, causal, rows_bhi[3 * t], rows_bhi[3 * t + 1],
                            rows_bhi[3 * t + 2], 1, S, P, O_rows + (size_t)t * d, LSE_rows + t);
      }
    }
    free(S);
    free(P);
  }
  return failed ? ORACLE_ERR_NOMEM : ORACLE_OK;
}

int fa_oracle_rows(const double* Q, const double* K, const double* V, const int* rows_bhi, int n_rows,
                   double* O_rows, double* LSE_rows, int B, int H, int Nq, int Nk, int d, double scale) {
  return fa_oracle_rows_masked(Q, K, V, rows_bhi, n_rows, O_rows, LSE_rows, B, H, Nq, Nk, d, scale, 0);
}

/*
 * The materialised intermediates of one head: S_out and P_out are [Nq][Nk] (either may be NULL).
 * S_out holds the scaled logits before the rowmax subtraction, P_out the softmax.
 */
int fa_oracle_head_probs(const double* Q, const double* K, const double* V, double* S_out, double* P_out,
                         int B, int H, int Nq, int Nk, int d, double scale, int b, int h) {
  int rc = check_shape(Q, K, V, B, H, Nq, Nk, d, scale);
  if (rc != ORACLE_OK) return rc;
  if (b < 0 || b >= B || h < 0 || h >= H) return ORACLE_ERR_ARG;
  double* S = (double*)malloc(sizeof(double) * (size_t)Nk);
  double* P = (double*)malloc(sizeof(double) * (size_t)Nk);
  double* o = (double*)malloc(sizeof(double) * (size_t)d);
  if (!S || !P || !o) {
    free(S);
    free(P);
    free(o);
    return ORACLE_ERR_NOMEM;
  }
  for (int i = 0; i < Nq; ++i) {
    double lse;
    /* recompute the raw scaled logits first: attention_row_block leaves S unshifted. */
    attention_row_block(Q, K, V, H, Nq, Nk, d, scale, 0, b, h, i, 1, S, P, o, &lse);
    for (int j = 0; j < Nk; ++j) {
      if (S_out) S_out[(size_t)i * Nk + j] = S[j];
      if (P_out) P_out[(size_t)i * Nk + j] = P[j];
    }
  }
  free(S);
  free(P);
  free(o);
  return ORACLE_OK;
}

/* Number of threads a parallel region of this library uses (1 without OpenMP). */
int fa_oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
