/*
 * CPU oracle for the MEFT sparse-adapter layer -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, fp64 restatement of what the layer computes, written from the
 * paper (MEFT: Memory-Efficient Fine-Tuning through Sparse Adapter).  It is
 * used by the tests, by the smoke check and by the CPU-baseline leg of the
 * benchmark; the product path never calls it.  It shares no code with the HIP
 * library.
 *
 * Notation follows the benchmark's problem statement (the paper's letters are
 * given in brackets):
 *   T tokens, hidden size d, N = n_blocks*block_size adapter neurons [r],
 *   n_blocks key experts [N], top_e experts per token [blackboard K],
 *   top_k neurons per token [K], keys K[N,d] (row j = column j of W_A),
 *   values V[N,d] (row j of W_B), router Wg[n_blocks,d].
 *
 * Per token t (Algorithm 1 applied to one token; Section 3.2 Eq. 5-7,
 * Section 3.1 Eq. 1-4):
 *   1. p[b]  = sum_c Wg[b,c] h[t,c] (+ bias[b])                      Eq. 5, no softmax
 *   2. tau   = the top_e blocks by p, ties to the lower block id
 *   3. cand  = all neurons of the blocks in tau; sc[j] = sum_c h[t,c] K[j,c]   Eq. 6
 *   4. I_t   = the top_k candidates by sc (pre-activation, Eq. 1), ties to the lower id
 *   5. out[t,:] = sum_{j in I_t} max(sc[j],0) V[j,:]                  Eq. 4, adapter term
 * Backward (Section 3.1, last paragraph: only activated neurons get gradient):
 *   6. g[j]  = sum_c dOut[t,c] V[j,c];  ds[j] = g[j] if sc[j] > 0 else 0
 *   7. dV[j,:] += max(sc[j],0) dOut[t,:];  dK[j,:] += ds[j] h[t,:];  dh[t,:] += ds[j] K[j,:]
 *   8. touched = sorted unique union of the I_t; every other row of dK, dV is zero.
 *
 * Batch-union evaluation (Algorithm 1 as printed, which evaluates the adapter over the union of all
 * tokens' selections rather than per token), meft_oracle_union_fwd / _bwd:
 *   S = sorted unique ids of all tokens' selections (built by the caller from step 4's lists)
 *   out[t,:] = sum_{j in S} max(h[t,:].K[j,:], 0) V[j,:]          for every token t
 *   backward over the same S with the rules of steps 6-7 applied to every (t, j in S).
 *
 * Optimizer step (Section 4.3 "Implementation Details": the Adam optimizer; Section 3.1, last
 * paragraph: only the activated rows have a gradient and are updated), meft_oracle_adam_rows:
 * for every row j of `touched` and every column c, with step count t >= 1,
 *   m = b1 m + (1-b1) g;  v = b2 v + (1-b2) g^2;
 *   w = w - lr (m / (1-b1^t)) / (sqrt(v / (1-b2^t)) + eps)            (Adam as published)
 * Rows outside `touched` keep weights and both moments unchanged (reading: a row without a
 * gradient in a step takes no part in that step; t counts steps of the layer, not of the row).
 *
 * Inputs are float32 arrays that hold exactly the stored values (bf16 values
 * are exactly representable); every product and sum is done in double, sums in
 * ascending index order.
 *
 * Readings where the paper is silent or inconsistent: the selection is per
 * token (Eq. 1-4), not the batch union of Algorithm 1; top-k ranks
 * pre-activation scores (Eq. 1); ties go to the lower index and +0 == -0 is a
 * tie; the ReLU derivative at 0 is 0; the router score only selects (no gate
 * multiply, Appendix "Negative Attempts"), so the router has no gradient;
 * experts are contiguous equal blocks: neuron j lies in block j / block_size.
 *
 * Pins (tests/test_oracle_*.py): dense equivalence against numpy matmul when
 * top_e = n_blocks and top_k = N (values and all three gradients), block-dense
 * and saturation cases, one-expert and one-neuron-per-expert special cases,
 * stable-argsort top-k, constructed ties, finite differences, linearity, a
 * hand-worked example (tests/golden/worked_example.txt).  Batch union: numpy matmul over the
 * compacted rows, the dense adapter when S is everything, the per-token result plus the extra
 * neurons' contributions, finite differences.  Adam: closed form of the first step,
 * torch.optim.Adam (all rows touched) and torch.optim.SparseAdam (row subsets, eps -> 0) over
 * several steps, untouched rows bit-identical.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
  int32_t T, d, n_blocks, block_size, top_e, top_k;
} oracle_shape;

typedef struct {
  double s;
  int32_t id;
} scored;

/* descending score, then ascending id: a total order, so qsort's instability does not matter */
static int by_score_desc_id_asc(const void* a, const void* b) {
  const scored* x = (const scored*)a;
  const scored* y = (const scored*)b;
  if (x->s > y->s) return -1;
  if (x->s < y->s) return 1;
  return (x->id > y->id) - (x->id < y->id);
}

static int by_id_asc(const void* a, const void* b) {
  const scored* x = (const scored*)a;
  const scored* y = (const scored*)b;
  return (x->id > y->id) - (x->id < y->id);
}

static double dot_f32(const float* a, const float* b, int32_t n) {
  double acc = 0.0;
  for (int32_t c = 0; c < n; ++c) acc += (double)a[c] * (double)b[c];
  return acc;
}

static int shape_ok(const oracle_shape* s) {
  return s && s->T >= 0 && s->d >= 1 && s->n_blocks >= 1 && s->block_size >= 1 && s->top_e >= 1 &&
         s->top_e <= s->n_blocks && s->top_k >= 1 &&
         (int64_t)s->top_k <= (int64_t)s->top_e * s->block_size;
}

int meft_oracle_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Steps 1-2.  block_idx[T,top_e] ordered by (p desc, block asc); block_score the matching p;
 * p_all[T,n_blocks] (may be NULL) every router score. */
int meft_oracle_route(const oracle_shape* s, const float* h, const float* Wg, const float* bias,
                      int32_t* block_idx, double* block_score, double* p_all) {
  if (!shape_ok(s)) return 1;
  const int32_t B = s->n_blocks, d = s->d, e = s->top_e;
#pragma omp parallel
  {
    scored* p = (scored*)malloc(sizeof(scored) * (size_t)B);
#pragma omp for schedule(static)
    for (int32_t t = 0; t < s->T; ++t) {
      for (int32_t b = 0; b < B; ++b) {
        p[b].s = dot_f32(Wg + (size_t)b * d, h + (size_t)t * d, d) + (bias ? (double)bias[b] : 0.0);
        p[b].id = b;
        if (p_all) p_all[(size_t)t * B + b] = p[b].s;
      }
      qsort(p, (size_t)B, sizeof(scored), by_score_desc_id_asc);
      for (int32_t q = 0; q < e; ++q) {
        block_idx[(size_t)t * e + q] = p[q].id;
        block_score[(size_t)t * e + q] = p[q].s;
      }
    }
    free(p);
  }
  return 0;
}

/* Steps 3-5.  idx[T,top_k] and score[T,top_k] ordered by (sc desc, id asc); score is the
 * PRE-activation value.  next_score[T] (may be NULL): the (top_k+1)-th candidate score, -inf if
 * there is none.  cand_id / cand_score [T, top_e*block_size] (may be NULL): every candidate in
 * ascending neuron id with its score.  out[T,d]. */
int meft_oracle_fwd(const oracle_shape* s, const float* h, const float* K, const float* V,
                    const int32_t* block_idx, double* out, int32_t* idx, double* score,
                    double* next_score, int32_t* cand_id, double* cand_score) {
  if (!shape_ok(s)) return 1;
  const int32_t d = s->d, e = s->top_e, bs = s->block_size, k = s->top_k;
  const int64_t C = (int64_t)e * bs;
  int bad = 0;
#pragma omp parallel
  {
    scored* cand = (scored*)malloc(sizeof(scored) * (size_t)C);
#pragma omp for schedule(dynamic, 1)
    for (int32_t t = 0; t < s->T; ++t) {
      const float* ht = h + (size_t)t * d;
      int64_t n = 0;
      for (int32_t q = 0; q < e; ++q) {
        const int32_t b = block_idx[(size_t)t * e + q];
        if (b < 0 || b >= s->n_blocks) { bad = 1; continue; }
        for (int32_t r = 0; r < bs; ++r) {
          const int32_t j = b * bs + r;
          cand[n].id = j;
          cand[n].s = dot_f32(ht, K + (size_t)j * d, d);
          ++n;
        }
      }
      if (n != C) continue;
      if (cand_id) {
        /* report candidates in ascending id */
        scored* tmp = (scored*)malloc(sizeof(scored) * (size_t)C);
        memcpy(tmp, cand, sizeof(scored) * (size_t)C);
        qsort(tmp, (size_t)C, sizeof(scored), by_id_asc);
        for (int64_t a = 0; a < C; ++a) {
          cand_id[(size_t)t * C + a] = tmp[a].id;
          cand_score[(size_t)t * C + a] = tmp[a].s;
        }
        free(tmp);
      }
      qsort(cand, (size_t)C, sizeof(scored), by_score_desc_id_asc);
      double* ot = out + (size_t)t * d;
      for (int32_t c = 0; c < d; ++c) ot[c] = 0.0;
      for (int32_t i = 0; i < k; ++i) {
        const int32_t j = cand[i].id;
        const double a = cand[i].s > 0.0 ? cand[i].s : 0.0;
        idx[(size_t)t * k + i] = j;
        score[(size_t)t * k + i] = cand[i].s;
        const float* vj = V + (size_t)j * d;
        for (int32_t c = 0; c < d; ++c) ot[c] += a * (double)vj[c];
      }
      if (next_score) next_score[t] = (k < C) ? cand[k].s : -INFINITY;
    }
    free(cand);
  }
  return bad;
}

/* Steps 6-8 for given selections.  score is pre-activation.  dh[T,d] (may be NULL).
 * If rows == NULL: dK, dV are dense [N,d] and are fully written (zero outside touched rows).
 * If rows != NULL: dK, dV are [n_rows,d] and hold the gradient rows of the neurons listed in
 * rows[] (any order, distinct).  touched (capacity min(N, T*top_k), may be NULL) ascending,
 * n_touched its length. */
int meft_oracle_bwd(const oracle_shape* s, const float* h, const float* K, const float* V,
                    const int32_t* idx, const double* score, const float* dOut, double* dh,
                    double* dK, double* dV, int32_t* touched, int32_t* n_touched,
                    const int32_t* rows, int32_t n_rows) {
  if (!shape_ok(s)) return 1;
  const int32_t d = s->d, k = s->top_k, T = s->T;
  const int64_t N = (int64_t)s->n_blocks * s->block_size;
  const int64_t P = (int64_t)T * k;
  for (int64_t p = 0; p < P; ++p)
    if (idx[p] < 0 || idx[p] >= N) return 2;

  /* ds[t,i] (step 6) and dh (step 7, the dh part): independent per token */
  double* ds = (double*)malloc(sizeof(double) * (size_t)(P > 0 ? P : 1));
#pragma omp parallel for schedule(static)
  for (int32_t t = 0; t < T; ++t) {
    double* dht = dh ? dh + (size_t)t * d : NULL;
    if (dht) for (int32_t c = 0; c < d; ++c) dht[c] = 0.0;
    for (int32_t i = 0; i < k; ++i) {
      const int64_t p = (int64_t)t * k + i;
      const int32_t j = idx[p];
      const double g = dot_f32(dOut + (size_t)t * d, V + (size_t)j * d, d);
      ds[p] = score[p] > 0.0 ? g : 0.0;
      if (dht) {
        const float* kj = K + (size_t)j * d;
        for (int32_t c = 0; c < d; ++c) dht[c] += ds[p] * (double)kj[c];
      }
    }
  }

  /* group the (token, neuron) pairs by neuron, tokens ascending inside a group */
  int64_t* seg = (int64_t*)calloc((size_t)N + 1, sizeof(int64_t));
  for (int64_t p = 0; p < P; ++p) seg[idx[p] + 1]++;
  int32_t nt = 0;
  for (int64_t j = 0; j < N; ++j) {
    if (seg[j + 1] > 0) {
      if (touched) touched[nt] = (int32_t)j;
      ++nt;
    }
    seg[j + 1] += seg[j];
  }
  if (n_touched) *n_touched = nt;
  int64_t* fill = (int64_t*)malloc(sizeof(int64_t) * (size_t)N);
  for (int64_t j = 0; j < N; ++j) fill[j] = seg[j];
  int64_t* pair = (int64_t*)malloc(sizeof(int64_t) * (size_t)(P > 0 ? P : 1));
  for (int64_t p = 0; p < P; ++p) pair[fill[idx[p]]++] = p; /* p ascending => token ascending */

  const int64_t n_out = rows ? n_rows : N;
#pragma omp parallel for schedule(dynamic, 16)
  for (int64_t o = 0; o < n_out; ++o) {
    const int64_t j = rows ? rows[o] : o;
    double* dKj = dK + (size_t)o * d;
    double* dVj = dV + (size_t)o * d;
    for (int32_t c = 0; c < d; ++c) { dKj[c] = 0.0; dVj[c] = 0.0; }
    if (j < 0 || j >= N) continue;
    for (int64_t q = seg[j]; q < seg[j + 1]; ++q) {
      const int64_t p = pair[q];
      const int32_t t = (int32_t)(p / k);
      const double a = score[p] > 0.0 ? score[p] : 0.0;
      const float* go = dOut + (size_t)t * d;
      const float* ht = h + (size_t)t * d;
      for (int32_t c = 0; c < d; ++c) {
        dVj[c] += a * (double)go[c];
        dKj[c] += ds[p] * (double)ht[c];
      }
    }
  }
  free(pair); free(fill); free(seg); free(ds);
  return 0;
}

/* Step 5 alone for selections given from outside (used by pins that fix the selection). */
int meft_oracle_apply(const oracle_shape* s, const float* h, const float* K, const float* V,
                      const int32_t* idx, double* out) {
  if (!shape_ok(s)) return 1;
  const int32_t d = s->d, k = s->top_k;
#pragma omp parallel for schedule(static)
  for (int32_t t = 0; t < s->T; ++t) {
    double* ot = out + (size_t)t * d;
    for (int32_t c = 0; c < d; ++c) ot[c] = 0.0;
    for (int32_t i = 0; i < k; ++i) {
      const int32_t j = idx[(size_t)t * k + i];
      const double sc = dot_f32(h + (size_t)t * d, K + (size_t)j * d, d);
      const double a = sc > 0.0 ? sc : 0.0;
      const float* vj = V + (size_t)j * d;
      for (int32_t c = 0; c < d; ++c) ot[c] += a * (double)vj[c];
    }
  }
  return 0;
}

/* Row-sparse Adam step on the rows listed in `touched` (ascending, unique).  All arrays [N, d], double. */
int meft_oracle_adam_rows(int32_t N, int32_t d, const int32_t* touched, int32_t n_touched, const double* g,
                          double* w, double* m, double* v, double lr, double b1, double b2, double eps,
                          int32_t step) {
  if (N < 1 || d < 1 || n_touched < 0 || n_touched > N || step < 1) return 1;
  for (int32_t i = 0; i < n_touched; ++i)
    if (touched[i] < 0 || touched[i] >= N || (i > 0 && touched[i] <= touched[i - 1])) return 2;
  const double c1 = 1.0 - pow(b1, (double)step), c2 = 1.0 - pow(b2, (double)step);
#pragma omp parallel for schedule(static)
  for (int32_t i = 0; i < n_touched; ++i) {
    const size_t o = (size_t)touched[i] * d;
    for (int32_t c = 0; c < d; ++c) {
      const double gr = g[o + c];
      const double mn = b1 * m[o + c] + (1.0 - b1) * gr;
      const double vn = b2 * v[o + c] + (1.0 - b2) * gr * gr;
      m[o + c] = mn;
      v[o + c] = vn;
      w[o + c] -= lr * (mn / c1) / (sqrt(vn / c2) + eps);
    }
  }
  return 0;
}

/* Batch-union forward: out[t,:] = sum over the nS listed neurons of max(h_t.K_j, 0) V_j (ascending j). */
int meft_oracle_union_fwd(int32_t T, int32_t d, int32_t N, const float* h, const float* K, const float* V,
                          const int32_t* S, int32_t nS, double* out) {
  if (T < 0 || d < 1 || N < 1 || nS < 0 || nS > N) return 1;
  for (int32_t i = 0; i < nS; ++i)
    if (S[i] < 0 || S[i] >= N || (i > 0 && S[i] <= S[i - 1])) return 2;
#pragma omp parallel for schedule(static)
  for (int32_t t = 0; t < T; ++t) {
    double* ot = out + (size_t)t * d;
    for (int32_t c = 0; c < d; ++c) ot[c] = 0.0;
    for (int32_t i = 0; i < nS; ++i) {
      const size_t j = (size_t)S[i];
      const double sc = dot_f32(h + (size_t)t * d, K + j * d, d);
      if (sc > 0.0)
        for (int32_t c = 0; c < d; ++c) ot[c] += sc * (double)V[j * d + c];
    }
  }
  return 0;
}

/* Batch-union backward.  dK, dV are [nS, d]: row i belongs to neuron S[i].  dh may be NULL. */
int meft_oracle_union_bwd(int32_t T, int32_t d, int32_t N, const float* h, const float* K, const float* V,
                          const int32_t* S, int32_t nS, const float* dOut, double* dh, double* dK, double* dV) {
  if (T < 0 || d < 1 || N < 1 || nS < 0 || nS > N) return 1;
  for (int32_t i = 0; i < nS; ++i)
    if (S[i] < 0 || S[i] >= N || (i > 0 && S[i] <= S[i - 1])) return 2;
  /* weight gradients: one neuron at a time, tokens in ascending order */
#pragma omp parallel for schedule(dynamic, 4)
  for (int32_t i = 0; i < nS; ++i) {
    const size_t j = (size_t)S[i];
    double* dk = dK + (size_t)i * d;
    double* dv = dV + (size_t)i * d;
    for (int32_t c = 0; c < d; ++c) { dk[c] = 0.0; dv[c] = 0.0; }
    for (int32_t t = 0; t < T; ++t) {
      const double sc = dot_f32(h + (size_t)t * d, K + j * d, d);
      if (!(sc > 0.0)) continue;                       /* a = 0 and ds = 0 */
      const double g = dot_f32(dOut + (size_t)t * d, V + j * d, d);
      for (int32_t c = 0; c < d; ++c) {
        dv[c] += sc * (double)dOut[(size_t)t * d + c];
        dk[c] += g * (double)h[(size_t)t * d + c];
      }
    }
  }
  if (dh) {
#pragma omp parallel for schedule(static)
    for (int32_t t = 0; t < T; ++t) {
      double* o = dh + (size_t)t * d;
      for (int32_t c = 0; c < d; ++c) o[c] = 0.0;
      for (int32_t i = 0; i < nS; ++i) {
        const size_t j = (size_t)S[i];
        const double sc = dot_f32(h + (size_t)t * d, K + j * d, d);
        if (!(sc > 0.0)) continue;
        const double g = dot_f32(dOut + (size_t)t * d, V + j * d, d);
        for (int32_t c = 0; c < d; ++c) o[c] += g * (double)K[j * d + c];
      }
    }
  }
  return 0;
}
