/* Runs every function of oracle/asa_ref.c on small ragged inputs.  Built by
 * tests/test_sanitizers.py with -fsanitize=address,undefined: any out-of-bounds access,
 * misaligned access, signed overflow or use of uninitialised heap that these sizes reach ends
 * the program with a report and a non-zero status.  Prints "ok" at the end. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int asa_ref_num_threads(void);
int asa_ref_sample_rows(int L, int b, int k, const int32_t *offs, int32_t *rows);
int asa_ref_p_imp_direct(const float *q, const float *k, int L, int d, int b, int ks, const int32_t *offs,
                         float scale, float *p_imp);
int asa_ref_p_imp_online(const float *q, const float *k, int L, int d, int b, int ks, const int32_t *offs,
                         float scale, float *p_imp);
int asa_ref_retention_bounds(int Nb, float r_min, float r_max, int32_t *m_min, int32_t *m_max);
int asa_ref_mask_rule_sort(const float *p_imp, int rows, int Nb, float tau, int m_min, int m_max,
                           uint8_t *mask, int32_t *m_out);
int asa_ref_mask_rule_orderfree(const float *p_imp, int rows, int Nb, float tau, int m_min, int m_max,
                                uint8_t *mask, int32_t *m_out);
int asa_ref_force_prefix(uint8_t *mask, int Nb, int b, int n_prefix);
int asa_ref_attn_fwd(const float *q, const float *k, const float *v, int L, int d, int b,
                     const uint8_t *mask, double scale, const int32_t *qblocks, int nq, double *o, double *lse);
int asa_ref_attn_delta(const float *d_o, const double *o, int L, int d, int b, const int32_t *qblocks, int nq,
                       double *delta);
int asa_ref_attn_bwd_dq(const float *q, const float *k, const float *v, const float *d_o, int L, int d, int b,
                        const uint8_t *mask, double scale, const double *lse, const double *delta,
                        const int32_t *qblocks, int nq, double *dq);
int asa_ref_attn_bwd_dkv(const float *q, const float *k, const float *v, const float *d_o, int L, int d, int b,
                         const uint8_t *mask, double scale, const double *lse, const double *delta,
                         const int32_t *kblocks, int nk, double *dk, double *dv);
int asa_ref_attn_bwd_dq_mag(const float *q, const float *k, const float *v, const float *d_o, int L, int d,
                            int b, const uint8_t *mask, double scale, const double *lse, const double *delta,
                            const int32_t *qblocks, int nq, double *dq);
int asa_ref_attn_bwd_dkv_mag(const float *q, const float *k, const float *v, const float *d_o, int L, int d,
                             int b, const uint8_t *mask, double scale, const double *lse, const double *delta,
                             const int32_t *kblocks, int nk, double *dk, double *dv);

static uint32_t rng_state = 12345u;
static float rnd(void) {   /* small deterministic generator: uniform in [-1, 1) */
  rng_state = rng_state * 1664525u + 1013904223u;
  return (float)((rng_state >> 8) & 0xFFFF) / 32768.0f - 1.0f;
}
#define CHECK(x) do { int rc_ = (x); if (rc_ != 0) { printf("%s -> %d\n", #x, rc_); return 1; } } while (0)

static int one_case(int L, int d, int b, int ks) {
  const int Nb = (L + b - 1) / b;
  float *q = malloc(sizeof(float) * L * d), *k = malloc(sizeof(float) * L * d);
  float *v = malloc(sizeof(float) * L * d), *g = malloc(sizeof(float) * L * d);
  for (int i = 0; i < L * d; ++i) { q[i] = rnd(); k[i] = rnd(); v[i] = rnd(); g[i] = rnd(); }
  int32_t *offs = malloc(sizeof(int32_t) * ks), *rows = malloc(sizeof(int32_t) * Nb * ks);
  for (int u = 0; u < ks; ++u) offs[u] = u * (b / ks);
  CHECK(asa_ref_sample_rows(L, b, ks, offs, rows));
  float *p1 = malloc(sizeof(float) * Nb * Nb), *p2 = malloc(sizeof(float) * Nb * Nb);
  CHECK(asa_ref_p_imp_direct(q, k, L, d, b, ks, offs, 0.25f, p1));
  CHECK(asa_ref_p_imp_online(q, k, L, d, b, ks, offs, 0.25f, p2));
  for (int i = 0; i < Nb * Nb; ++i)
    if (fabsf(p1[i] - p2[i]) > 1e-6f * fabsf(p1[i]) + 1e-30f) { printf("forms differ\n"); return 1; }
  p1[0] = NAN;   /* a NaN score counts as 0 */
  int32_t lo, hi;
  CHECK(asa_ref_retention_bounds(Nb, 0.1f, 0.9f, &lo, &hi));
  uint8_t *m1 = malloc(Nb * Nb), *m2 = malloc(Nb * Nb);
  int32_t *mo = malloc(sizeof(int32_t) * Nb);
  CHECK(asa_ref_mask_rule_sort(p1, Nb, Nb, 0.9f, lo, hi, m1, mo));
  CHECK(asa_ref_mask_rule_orderfree(p1, Nb, Nb, 0.9f, lo, hi, m2, mo));
  if (memcmp(m1, m2, Nb * Nb)) { printf("rule forms differ\n"); return 1; }
  CHECK(asa_ref_force_prefix(m1, Nb, b, b / 2 + 1));
  int32_t *blocks = malloc(sizeof(int32_t) * Nb);
  for (int i = 0; i < Nb; ++i) blocks[i] = i;
  double *o = malloc(sizeof(double) * L * d), *lse = malloc(sizeof(double) * L), *delta = malloc(sizeof(double) * L);
  double *dq = malloc(sizeof(double) * L * d), *dk = malloc(sizeof(double) * L * d), *dv = malloc(sizeof(double) * L * d);
  CHECK(asa_ref_attn_fwd(q, k, v, L, d, b, m1, 0.3, blocks, Nb, o, lse));
  CHECK(asa_ref_attn_delta(g, o, L, d, b, blocks, Nb, delta));
  CHECK(asa_ref_attn_bwd_dq(q, k, v, g, L, d, b, m1, 0.3, lse, delta, blocks, Nb, dq));
  CHECK(asa_ref_attn_bwd_dkv(q, k, v, g, L, d, b, m1, 0.3, lse, delta, blocks, Nb, dk, dv));
  CHECK(asa_ref_attn_bwd_dq_mag(q, k, v, g, L, d, b, m1, 0.3, lse, delta, blocks, Nb, dq));
  CHECK(asa_ref_attn_bwd_dkv_mag(q, k, v, g, L, d, b, m1, 0.3, lse, delta, blocks, Nb, dk, dv));
  double s = 0;
  for (int i = 0; i < L * d; ++i) s += o[i] + dq[i] + dk[i] + dv[i];
  if (!(s == s)) { printf("non-finite result\n"); return 1; }
  free(q); free(k); free(v); free(g); free(offs); free(rows); free(p1); free(p2); free(m1); free(m2);
  free(mo); free(blocks); free(o); free(lse); free(delta); free(dq); free(dk); free(dv);
  return 0;
}

int main(void) {
  if (asa_ref_num_threads() < 1) return 1;
  if (one_case(100, 16, 32, 8)) return 1;    /* ragged last block: 4 valid tokens */
  if (one_case(64, 8, 64, 64)) return 1;     /* one block, every token sampled */
  if (one_case(7, 4, 4, 2)) return 1;        /* tiny, ragged */
  if (one_case(1, 8, 8, 1)) return 1;        /* a single token */
  printf("ok\n");
  return 0;
}
