/*
 * Driver for tests/test_oracle_sanitizers.py -- TEST INFRASTRUCTURE ONLY.
 *
 * Compiled together with oracle/meft_oracle.c under -fsanitize=address,undefined.  It reads one seeded case from a
 * binary file, runs every entry point of the oracle on it (route, forward with the candidate lists, backward dense
 * and on a row subset, the replay of step 5, the batch-union pair, the optimizer step, and the argument checks that
 * must reject bad input) and writes the results to a second file, which the test compares with the results of the
 * ordinary build.  A sanitizer report ends the run with a non-zero status.
 *
 * File layout (little endian): int32 T, d, n_blocks, block_size, top_e, top_k, n_rows; then float32 h[T,d],
 * Wg[n_blocks,d], bias[n_blocks], K[N,d], V[N,d], dOut[T,d]; then int32 rows[n_rows].
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
  int32_t T, d, n_blocks, block_size, top_e, top_k;
} oracle_shape;

int meft_oracle_route(const oracle_shape*, const float*, const float*, const float*, int32_t*, double*, double*);
int meft_oracle_fwd(const oracle_shape*, const float*, const float*, const float*, const int32_t*, double*, int32_t*,
                    double*, double*, int32_t*, double*);
int meft_oracle_bwd(const oracle_shape*, const float*, const float*, const float*, const int32_t*, const double*,
                    const float*, double*, double*, double*, int32_t*, int32_t*, const int32_t*, int32_t);
int meft_oracle_apply(const oracle_shape*, const float*, const float*, const float*, const int32_t*, double*);
int meft_oracle_adam_rows(int32_t, int32_t, const int32_t*, int32_t, const double*, double*, double*, double*, double,
                          double, double, double, int32_t);
int meft_oracle_union_fwd(int32_t, int32_t, int32_t, const float*, const float*, const float*, const int32_t*, int32_t,
                          double*);
int meft_oracle_union_bwd(int32_t, int32_t, int32_t, const float*, const float*, const float*, const int32_t*, int32_t,
                          const float*, double*, double*, double*);

static void* xmalloc(size_t n) {
  void* p = malloc(n ? n : 1);
  if (!p) { fprintf(stderr, "out of memory\n"); exit(3); }
  return p;
}
static void rd(FILE* f, void* p, size_t n) {
  if (n && fread(p, 1, n, f) != n) { fprintf(stderr, "short input\n"); exit(3); }
}
static void wr(FILE* f, const void* p, size_t n) {
  if (n && fwrite(p, 1, n, f) != n) { fprintf(stderr, "short output\n"); exit(3); }
}

int main(int argc, char** argv) {
  if (argc != 3) { fprintf(stderr, "usage: driver in.bin out.bin\n"); return 2; }
  FILE* in = fopen(argv[1], "rb");
  if (!in) return 2;
  int32_t hd[7];
  rd(in, hd, sizeof hd);
  oracle_shape s = {hd[0], hd[1], hd[2], hd[3], hd[4], hd[5]};
  const int32_t n_rows = hd[6];
  const size_t T = (size_t)s.T, d = (size_t)s.d, B = (size_t)s.n_blocks, N = B * (size_t)s.block_size;
  const size_t e = (size_t)s.top_e, k = (size_t)s.top_k, C = e * (size_t)s.block_size;
  float* h = xmalloc(4 * T * d);     rd(in, h, 4 * T * d);
  float* Wg = xmalloc(4 * B * d);    rd(in, Wg, 4 * B * d);
  float* bias = xmalloc(4 * B);      rd(in, bias, 4 * B);
  float* K = xmalloc(4 * N * d);     rd(in, K, 4 * N * d);
  float* V = xmalloc(4 * N * d);     rd(in, V, 4 * N * d);
  float* dOut = xmalloc(4 * T * d);  rd(in, dOut, 4 * T * d);
  int32_t* rows = xmalloc(4 * (size_t)n_rows);  rd(in, rows, 4 * (size_t)n_rows);
  fclose(in);

  FILE* out = fopen(argv[2], "wb");
  if (!out) return 2;
  int rc = 0;

  int32_t* block_idx = xmalloc(4 * T * e);
  double* block_score = xmalloc(8 * T * e);
  double* p_all = xmalloc(8 * T * B);
  rc |= meft_oracle_route(&s, h, Wg, bias, block_idx, block_score, p_all);
  wr(out, block_idx, 4 * T * e); wr(out, block_score, 8 * T * e); wr(out, p_all, 8 * T * B);

  double* o = xmalloc(8 * T * d);
  int32_t* idx = xmalloc(4 * T * k);
  double* score = xmalloc(8 * T * k);
  double* next = xmalloc(8 * T);
  int32_t* cand_id = xmalloc(4 * T * C);
  double* cand_score = xmalloc(8 * T * C);
  rc |= meft_oracle_fwd(&s, h, K, V, block_idx, o, idx, score, next, cand_id, cand_score);
  wr(out, o, 8 * T * d); wr(out, idx, 4 * T * k); wr(out, score, 8 * T * k); wr(out, next, 8 * T);
  wr(out, cand_id, 4 * T * C); wr(out, cand_score, 8 * T * C);
  /* the optional outputs left out */
  rc |= meft_oracle_fwd(&s, h, K, V, block_idx, o, idx, score, NULL, NULL, NULL);

  double* dh = xmalloc(8 * T * d);
  double* dK = xmalloc(8 * N * d);
  double* dV = xmalloc(8 * N * d);
  const size_t cap = N < T * k ? N : T * k;
  int32_t* touched = xmalloc(4 * cap);
  int32_t nt = -1;
  rc |= meft_oracle_bwd(&s, h, K, V, idx, score, dOut, dh, dK, dV, touched, &nt, NULL, 0);
  wr(out, dh, 8 * T * d); wr(out, dK, 8 * N * d); wr(out, dV, 8 * N * d); wr(out, &nt, 4);
  wr(out, touched, 4 * (size_t)nt);
  /* row subset, no dh, no touched list */
  double* dKr = xmalloc(8 * (size_t)n_rows * d);
  double* dVr = xmalloc(8 * (size_t)n_rows * d);
  rc |= meft_oracle_bwd(&s, h, K, V, idx, score, dOut, NULL, dKr, dVr, NULL, NULL, rows, n_rows);
  wr(out, dKr, 8 * (size_t)n_rows * d); wr(out, dVr, 8 * (size_t)n_rows * d);

  rc |= meft_oracle_apply(&s, h, K, V, idx, o);
  wr(out, o, 8 * T * d);

  /* batch union over the touched list */
  rc |= meft_oracle_union_fwd(s.T, s.d, (int32_t)N, h, K, V, touched, nt, o);
  wr(out, o, 8 * T * d);
  double* dKs = xmalloc(8 * (size_t)nt * d);
  double* dVs = xmalloc(8 * (size_t)nt * d);
  rc |= meft_oracle_union_bwd(s.T, s.d, (int32_t)N, h, K, V, touched, nt, dOut, dh, dKs, dVs);
  wr(out, dh, 8 * T * d); wr(out, dKs, 8 * (size_t)nt * d); wr(out, dVs, 8 * (size_t)nt * d);

  /* optimizer step on the touched rows: weights K, gradient dK, moments from dV's magnitudes */
  double* w = xmalloc(8 * N * d);
  double* m = xmalloc(8 * N * d);
  double* v = xmalloc(8 * N * d);
  for (size_t i = 0; i < N * d; ++i) { w[i] = K[i]; m[i] = 0.1 * dV[i]; v[i] = 0.01 * dV[i] * dV[i]; }
  rc |= meft_oracle_adam_rows((int32_t)N, s.d, touched, nt, dK, w, m, v, 1e-3, 0.9, 0.999, 1e-8, 3);
  wr(out, w, 8 * N * d); wr(out, m, 8 * N * d); wr(out, v, 8 * N * d);

  /* argument checks: each must be refused (non-zero) without touching memory it should not */
  oracle_shape bad = s;
  bad.top_k = (int32_t)C + 1;
  int refused = meft_oracle_fwd(&bad, h, K, V, block_idx, o, idx, score, NULL, NULL, NULL) != 0;
  bad = s; bad.top_e = s.n_blocks + 1;
  refused += meft_oracle_route(&bad, h, Wg, NULL, block_idx, block_score, NULL) != 0;
  idx[0] = (int32_t)N;   /* out of range id */
  refused += meft_oracle_bwd(&s, h, K, V, idx, score, dOut, dh, dK, dV, touched, &nt, NULL, 0) != 0;
  block_idx[0] = -1;     /* out of range block */
  refused += meft_oracle_fwd(&s, h, K, V, block_idx, o, idx, score, NULL, NULL, NULL) != 0;
  int32_t unsorted[2] = {1, 0};
  refused += meft_oracle_union_fwd(s.T, s.d, (int32_t)N, h, K, V, unsorted, 2, o) != 0;
  refused += meft_oracle_adam_rows((int32_t)N, s.d, unsorted, 2, dK, w, m, v, 1e-3, 0.9, 0.999, 1e-8, 1) != 0;
  int32_t tail[2] = {rc, refused};
  wr(out, tail, sizeof tail);
  fclose(out);

  free(h); free(Wg); free(bias); free(K); free(V); free(dOut); free(rows); free(block_idx); free(block_score);
  free(p_all); free(o); free(idx); free(score); free(next); free(cand_id); free(cand_score); free(dh); free(dK);
  free(dV); free(touched); free(dKr); free(dVr); free(dKs); free(dVs); free(w); free(m); free(v);
  return rc ? 1 : 0;
}
