/*
 * CPU checker for message-passing Aggregation, chunk by chunk along the
 * feature dimension (the paper's Algorithm 1).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT A PRODUCT PATH.  It is slow on purpose:
 * scalar loops, fp64 accumulation, one rounding to fp32 at the end.  It shares
 * no code with the GPU library and nothing in the GPU library may call it.
 * Only the tests, the smoke check and the benchmark's CPU-baseline leg use it.
 *
 * Conventions (paper, Section II-C: the input is the COO edge set plus the
 * vertex feature matrix): messages flow src -> dst; CSR rows are destinations
 * and colidx holds sources.
 *
 * Every function here is pinned by tests that do not call it to produce the
 * expected value (dense brute force, scipy SpMM, closed forms): nothing is
 * "parity unpinned".
 *
 * The optional `threads` argument only spreads independent destination rows
 * over OpenMP threads for timing; each output element is still produced by the
 * same scalar loop, so results are identical for any thread count.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { REF_SUM = 0, REF_WSUM = 1, REF_MEAN = 2, REF_MAX = 3, REF_SUM_SCALED = 4 };
enum { REF_F32 = 0, REF_BF16 = 1 };
enum { REF_SELF_LOOPS = 1, REF_NORM_SYM = 2 };

/* feature element j*F+f widened to double; bf16 widening is exact */
static inline double x_at(const void* X, int x_dtype, int64_t idx) {
  if (x_dtype == REF_F32) return (double)((const float*)X)[idx];
  uint32_t bits = (uint32_t)((const uint16_t*)X)[idx] << 16;
  float f;
  memcpy(&f, &bits, 4);
  return (double)f;
}

/* ---------------------------------------------------------------------------
 * CSR construction (paper Section II-C / III: COO in, destination-indexed
 * neighbour lists out).  Edge k (k < E) is src[k] -> dst[k]; with SELF_LOOPS,
 * edges E..E+N-1 are i -> i.  Row i lists the sources of all edges whose
 * destination is i, ordered by (source ascending, input position ascending);
 * duplicates are kept.  perm[slot] = input position of the edge in that slot.
 * With NORM_SYM, edge_w[slot] = 1/sqrt(d_i * d_j) where d is the row length
 * (in-degree after self-loops), computed in fp64 and rounded once to fp32
 * (GCN's D^-1/2 (A+I) D^-1/2).
 * ------------------------------------------------------------------------- */
typedef struct { int32_t s; int64_t pos; } slot_t;

static int slot_cmp(const void* a, const void* b) {
  const slot_t* x = (const slot_t*)a;
  const slot_t* y = (const slot_t*)b;
  if (x->s != y->s) return x->s < y->s ? -1 : 1;
  if (x->pos != y->pos) return x->pos < y->pos ? -1 : 1;
  return 0;
}

int gnnagg_ref_build_csr(int64_t N, int64_t E, const int32_t* src, const int32_t* dst, uint32_t flags,
                         int64_t* rowptr, int32_t* colidx, float* edge_w, int64_t* perm, int threads) {
  if (N < 0 || E < 0 || !rowptr || (E > 0 && (!src || !dst))) return -1;
  const int64_t loops = (flags & REF_SELF_LOOPS) ? N : 0;
  const int64_t nnz = E + loops;
  if (nnz > 0 && !colidx) return -1;
  for (int64_t k = 0; k < E; ++k)
    if (src[k] < 0 || src[k] >= N || dst[k] < 0 || dst[k] >= N) return -1;

  for (int64_t i = 0; i <= N; ++i) rowptr[i] = 0;
  for (int64_t k = 0; k < E; ++k) rowptr[dst[k] + 1] += 1;
  for (int64_t i = 0; i < loops; ++i) rowptr[i + 1] += 1;
  for (int64_t i = 0; i < N; ++i) rowptr[i + 1] += rowptr[i];

  slot_t* slots = (slot_t*)malloc(sizeof(slot_t) * (size_t)(nnz > 0 ? nnz : 1));
  int64_t* fill = (int64_t*)malloc(sizeof(int64_t) * (size_t)(N > 0 ? N : 1));
  if (!slots || !fill) { free(slots); free(fill); return -2; }
  for (int64_t i = 0; i < N; ++i) fill[i] = rowptr[i];
  for (int64_t k = 0; k < E; ++k) {
    int64_t p = fill[dst[k]]++;
    slots[p].s = src[k];
    slots[p].pos = k;
  }
  for (int64_t i = 0; i < loops; ++i) {
    int64_t p = fill[i]++;
    slots[p].s = (int32_t)i;
    slots[p].pos = E + i;
  }
#pragma omp parallel for schedule(dynamic, 64) num_threads(threads > 1 ? threads : 1)
  for (int64_t i = 0; i < N; ++i)
    qsort(slots + rowptr[i], (size_t)(rowptr[i + 1] - rowptr[i]), sizeof(slot_t), slot_cmp);
  for (int64_t p = 0; p < nnz; ++p) {
    colidx[p] = slots[p].s;
    if (perm) perm[p] = slots[p].pos;
  }
  if (edge_w) {
    for (int64_t i = 0; i < N; ++i) {
      double di = (double)(rowptr[i + 1] - rowptr[i]);
      for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
        if (flags & REF_NORM_SYM) {
          int64_t j = colidx[p];
          double dj = (double)(rowptr[j + 1] - rowptr[j]);
          edge_w[p] = (float)(1.0 / sqrt(di * dj));
        } else {
          edge_w[p] = 1.0f;
        }
      }
    }
  }
  free(slots);
  free(fill);
  return 0;
}

/* ---------------------------------------------------------------------------
 * Columns [c0,c1) of one output row by the plain definition (Algorithm 1, the
 * Message and Aggregate steps): reduce over the in-edges of row i in CSR
 * order, one fp64 accumulator per column.
 *   sum / wsum : (float) sum_e w_e * X[colidx[e], f]   (w = 1 for sum)
 *   mean       : 0 if the row is empty, else (float)(sum / deg)
 *   scaled sum : (float)(s_i * sum_e X[colidx[e], f]), the N factors s passed as edge_w: a weighted sum
 *                whose weights are s_i times a factor of the source that X already carries (GCN,
 *                Section III, with s = d^-1/2 on both sides)
 *   max        : +0.0f if the row is empty, else the largest value, with
 *                -0 ordered below +0 so that the result is unique.
 * acc is scratch for c1-c0 doubles.
 * ------------------------------------------------------------------------- */
static void reduce_row(int op, const int64_t* rowptr, const int32_t* colidx, const float* edge_w,
                       const void* X, int x_dtype, int64_t F, int64_t i, int64_t c0, int64_t c1,
                       double* acc, float* out_row /* points at column c0 */) {
  const int64_t e0 = rowptr[i], e1 = rowptr[i + 1];
  const int64_t W = c1 - c0;
  if (e0 == e1) {
    for (int64_t f = 0; f < W; ++f) out_row[f] = 0.0f;
    return;
  }
  if (op == REF_MAX) {
    for (int64_t f = 0; f < W; ++f) acc[f] = x_at(X, x_dtype, (int64_t)colidx[e0] * F + c0 + f);
    for (int64_t e = e0 + 1; e < e1; ++e)
      for (int64_t f = 0; f < W; ++f) {
        double v = x_at(X, x_dtype, (int64_t)colidx[e] * F + c0 + f);
        if (v > acc[f] || (v == acc[f] && signbit(acc[f]) && !signbit(v))) acc[f] = v;
      }
    for (int64_t f = 0; f < W; ++f) out_row[f] = (float)acc[f];
    return;
  }
  for (int64_t f = 0; f < W; ++f) acc[f] = 0.0;
  for (int64_t e = e0; e < e1; ++e) {
    const double w = (op == REF_WSUM) ? (double)edge_w[e] : 1.0;
    for (int64_t f = 0; f < W; ++f) acc[f] += w * x_at(X, x_dtype, (int64_t)colidx[e] * F + c0 + f);
  }
  const double deg = (double)(e1 - e0);
  for (int64_t f = 0; f < W; ++f) {
    if (op == REF_MEAN) out_row[f] = (float)(acc[f] / deg);
    else if (op == REF_SUM_SCALED) out_row[f] = (float)((double)edge_w[i] * acc[f]);
    else out_row[f] = (float)acc[f];
  }
}

/* Whole-matrix aggregation.  form 0: destination-row outer loop over full
 * rows (the plain definition; f_chunk is ignored).  form 1: the loop nest of
 * Algorithm 1 - feature chunk outer, vertex inner - with chunks
 * [c*f_chunk, min(F,(c+1)*f_chunk)); f_chunk <= 0 or >= F means one chunk.
 * Both forms reduce every element over the same operands in the same order,
 * so they agree bit for bit (the paper's exactness argument, Section I). */
int gnnagg_ref_aggregate(int op, int64_t N, const int64_t* rowptr, const int32_t* colidx, const float* edge_w,
                         const void* X, int x_dtype, float* out, int32_t F, int32_t f_chunk, int form,
                         int threads) {
  if (op < 0 || op > 4 || N < 0 || F <= 0 || !rowptr || !out || !X) return -1;
  if ((op == REF_WSUM || op == REF_SUM_SCALED) && !edge_w) return -1;
  if (x_dtype != REF_F32 && x_dtype != REF_BF16) return -1;
  const int64_t width = (form == 0 || f_chunk <= 0 || f_chunk >= F) ? F : f_chunk;
  const int64_t P = (F + width - 1) / width;
  int fail = 0;
  for (int64_t p = 0; p < P; ++p) {
    const int64_t c0 = p * width, c1 = (c0 + width < F) ? c0 + width : F;
#pragma omp parallel num_threads(threads > 1 ? threads : 1)
    {
      double* acc = (double*)malloc(sizeof(double) * (size_t)(c1 - c0));
      if (!acc) {
#pragma omp atomic write
        fail = 1;
      }
#pragma omp for schedule(dynamic, 16)
      for (int64_t v = 0; v < N; ++v)
        if (acc) reduce_row(op, rowptr, colidx, edge_w, X, x_dtype, F, v, c0, c1, acc, out + v * F + c0);
      free(acc);
    }
  }
  return fail ? -2 : 0;
}

/* The same definition for a list of destination rows only: out is [nrows, F].
 * Used to check sampled rows of workloads too large to aggregate in full. */
int gnnagg_ref_aggregate_rows(int op, int64_t nrows, const int64_t* rows, const int64_t* rowptr,
                              const int32_t* colidx, const float* edge_w, const void* X, int x_dtype,
                              float* out, int32_t F, int threads) {
  if (op < 0 || op > 4 || nrows < 0 || F <= 0 || !rows || !rowptr || !out || !X) return -1;
  if ((op == REF_WSUM || op == REF_SUM_SCALED) && !edge_w) return -1;
  if (x_dtype != REF_F32 && x_dtype != REF_BF16) return -1;
  int fail = 0;
#pragma omp parallel num_threads(threads > 1 ? threads : 1)
  {
    double* acc = (double*)malloc(sizeof(double) * (size_t)F);
    if (!acc) {
#pragma omp atomic write
      fail = 1;
    }
#pragma omp for schedule(dynamic, 1)
    for (int64_t r = 0; r < nrows; ++r)
      if (acc) reduce_row(op, rowptr, colidx, edge_w, X, x_dtype, F, rows[r], 0, F, acc, out + r * F);
    free(acc);
  }
  return fail ? -2 : 0;
}

/* ---------------------------------------------------------------------------
 * Graph-attention aggregation (the paper evaluates GAT as one of its three
 * aggregate operators, Section III; the operator is the cited one).
 *   s_src[j,h] = sum_c a_src[h,c] H[j,h,c],  s_dst[i,h] likewise
 *   e_ij,h     = LeakyReLU_slope(s_src[j,h] + s_dst[i,h])
 *   alpha_ij,h = exp(e - m) / sum_k exp(e_ik,h - m),   m = max over row i
 *   out[i,h,c] = (float) sum_j alpha_ij,h H[j,h,c];  empty row -> 0
 * All in fp64.  alpha ([nnz, heads]) and out ([N, heads, C]) may be NULL.
 * ------------------------------------------------------------------------- */
int gnnagg_ref_gat_attention(int64_t N, const int64_t* rowptr, const int32_t* colidx, const float* H,
                             const float* a_src, const float* a_dst, int32_t heads, int32_t C,
                             float negative_slope, float* alpha, float* out, int threads) {
  if (N < 0 || heads <= 0 || C <= 0 || !rowptr || !H || !a_src || !a_dst) return -1;
  const int64_t HC = (int64_t)heads * C;
  double* ssrc = (double*)malloc(sizeof(double) * (size_t)(N * heads + 1));
  double* sdst = (double*)malloc(sizeof(double) * (size_t)(N * heads + 1));
  if (!ssrc || !sdst) { free(ssrc); free(sdst); return -2; }
  for (int64_t j = 0; j < N; ++j)
    for (int32_t h = 0; h < heads; ++h) {
      double a = 0.0, b = 0.0;
      for (int32_t c = 0; c < C; ++c) {
        double x = (double)H[j * HC + (int64_t)h * C + c];
        a += (double)a_src[h * C + c] * x;
        b += (double)a_dst[h * C + c] * x;
      }
      ssrc[j * heads + h] = a;
      sdst[j * heads + h] = b;
    }
  const double slope = (double)negative_slope;
#pragma omp parallel for schedule(dynamic, 16) num_threads(threads > 1 ? threads : 1)
  for (int64_t i = 0; i < N; ++i) {
    const int64_t e0 = rowptr[i], e1 = rowptr[i + 1];
    for (int32_t h = 0; h < heads; ++h) {
      if (e0 == e1) {
        if (out) for (int32_t c = 0; c < C; ++c) out[i * HC + (int64_t)h * C + c] = 0.0f;
        continue;
      }
      double m = -INFINITY;
      for (int64_t e = e0; e < e1; ++e) {
        double s = ssrc[(int64_t)colidx[e] * heads + h] + sdst[i * heads + h];
        double v = s >= 0.0 ? s : slope * s;
        if (v > m) m = v;
      }
      double z = 0.0;
      for (int64_t e = e0; e < e1; ++e) {
        double s = ssrc[(int64_t)colidx[e] * heads + h] + sdst[i * heads + h];
        double v = s >= 0.0 ? s : slope * s;
        z += exp(v - m);
      }
      if (alpha)
        for (int64_t e = e0; e < e1; ++e) {
          double s = ssrc[(int64_t)colidx[e] * heads + h] + sdst[i * heads + h];
          double v = s >= 0.0 ? s : slope * s;
          alpha[e * heads + h] = (float)(exp(v - m) / z);
        }
      if (out)
        for (int32_t c = 0; c < C; ++c) {
          double acc = 0.0;
          for (int64_t e = e0; e < e1; ++e) {
            double s = ssrc[(int64_t)colidx[e] * heads + h] + sdst[i * heads + h];
            double v = s >= 0.0 ? s : slope * s;
            acc += (exp(v - m) / z) * (double)H[(int64_t)colidx[e] * HC + (int64_t)h * C + c];
          }
          out[i * HC + (int64_t)h * C + c] = (float)acc;
        }
    }
  }
  free(ssrc);
  free(sdst);
  return 0;
}

/* The same attention definition for a list of destination rows only: out is [nrows, heads, C].
 * Scores are formed edge by edge from H (no score arrays), everything in fp64.  Used to check
 * sampled rows of graphs too large to run in full. */
int gnnagg_ref_gat_attention_rows(int64_t nrows, const int64_t* rows, const int64_t* rowptr,
                                  const int32_t* colidx, const float* H, const float* a_src, const float* a_dst,
                                  int32_t heads, int32_t C, float negative_slope, float* out, int threads) {
  if (nrows < 0 || heads <= 0 || C <= 0 || !rows || !rowptr || !H || !a_src || !a_dst || !out) return -1;
  const int64_t HC = (int64_t)heads * C;
  const double slope = (double)negative_slope;
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads > 1 ? threads : 1)
  for (int64_t q = 0; q < nrows; ++q) {
    const int64_t i = rows[q];
    const int64_t e0 = rowptr[i], e1 = rowptr[i + 1];
    for (int32_t h = 0; h < heads; ++h) {
      float* o = out + q * HC + (int64_t)h * C;
      for (int32_t c = 0; c < C; ++c) o[c] = 0.0f;
      if (e0 == e1) continue;
      double sdst = 0.0;
      for (int32_t c = 0; c < C; ++c) sdst += (double)a_dst[h * C + c] * (double)H[i * HC + (int64_t)h * C + c];
      double* logit = (double*)malloc(sizeof(double) * (size_t)(e1 - e0));
      double m = -INFINITY;
      for (int64_t e = e0; e < e1; ++e) {
        const int64_t j = colidx[e];
        double ssrc = 0.0;
        for (int32_t c = 0; c < C; ++c) ssrc += (double)a_src[h * C + c] * (double)H[j * HC + (int64_t)h * C + c];
        const double s = ssrc + sdst;
        logit[e - e0] = s >= 0.0 ? s : slope * s;
        if (logit[e - e0] > m) m = logit[e - e0];
      }
      double z = 0.0;
      for (int64_t e = e0; e < e1; ++e) z += exp(logit[e - e0] - m);
      for (int32_t c = 0; c < C; ++c) {
        double acc = 0.0;
        for (int64_t e = e0; e < e1; ++e)
          acc += (exp(logit[e - e0] - m) / z) * (double)H[(int64_t)colidx[e] * HC + (int64_t)h * C + c];
        o[c] = (float)acc;
      }
      free(logit);
    }
  }
  return 0;
}

/* Combination as one dense layer (paper Section I / Algorithm 1, Update):
 *   out[n,h] = act( sum_f X[n,f] * W[f,h] + bias[h] ),  act = max(0,.) if relu else identity,
 * by the definition: fp64 products and sum in ascending f, bias added in fp64, one rounding to fp32. */
int gnnagg_ref_combine(int64_t N, const void* X, int x_dtype, int32_t F, const float* W, const float* bias,
                       int32_t H, int relu, float* out, int threads) {
  if (N < 0 || F <= 0 || H <= 0 || !X || !W || !out) return -1;
  if (x_dtype != REF_F32 && x_dtype != REF_BF16) return -1;
#pragma omp parallel for schedule(static) num_threads(threads > 1 ? threads : 1)
  for (int64_t n = 0; n < N; ++n)
    for (int32_t h = 0; h < H; ++h) {
      double acc = 0.0;
      for (int32_t f = 0; f < F; ++f) acc += x_at(X, x_dtype, n * F + f) * (double)W[(int64_t)f * H + h];
      if (bias) acc += (double)bias[h];
      float y = (float)acc;
      if (relu && !(y > 0.0f)) y = 0.0f;
      out[n * H + h] = y;
    }
  return 0;
}

/* The Update step of Algorithm 1 without a weight matrix, applied to an aggregated matrix A [N,F]:
 *   out[n,f] = act( A[n,f] + bias[f] ),  the sum formed in fp64 and rounded once to fp32;
 * bias may be NULL. */
int gnnagg_ref_update(int64_t N, int32_t F, const float* A, const float* bias, int relu, float* out) {
  if (N < 0 || F <= 0 || !A || !out) return -1;
  for (int64_t n = 0; n < N; ++n)
    for (int32_t f = 0; f < F; ++f) {
      float y = (float)((double)A[n * F + f] + (bias ? (double)bias[f] : 0.0));
      if (relu && !(y > 0.0f)) y = 0.0f;
      out[n * F + f] = y;
    }
  return 0;
}

/* GCN's weights in factored form (the GCN operator of Section III): 1/sqrt(d_i d_j) = s_i s_j with
 *   s[i] = (float)(1/sqrt(d_i)), d_i the length of row i; 0 for an empty row. */
int gnnagg_ref_gcn_factors(int64_t N, const int64_t* rowptr, float* s) {
  if (N < 0 || !rowptr || !s) return -1;
  for (int64_t i = 0; i < N; ++i) {
    const int64_t d = rowptr[i + 1] - rowptr[i];
    s[i] = d > 0 ? (float)(1.0 / sqrt((double)d)) : 0.0f;
  }
  return 0;
}

/* out[j,f] = (float)(scale[j] * X[j,f]): the product of two fp32 values is exact in fp64, so this is the
 * correctly rounded fp32 product. */
int gnnagg_ref_scale_rows(int64_t N, int32_t F, const void* X, int x_dtype, const float* scale, float* out) {
  if (N < 0 || F <= 0 || !X || !scale || !out) return -1;
  if (x_dtype != REF_F32 && x_dtype != REF_BF16) return -1;
  for (int64_t j = 0; j < N; ++j)
    for (int32_t f = 0; f < F; ++f) out[j * F + f] = (float)((double)scale[j] * x_at(X, x_dtype, j * F + f));
  return 0;
}
