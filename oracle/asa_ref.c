/*
 * CPU oracle for Adaptive Block-Sparse Attention (ASA).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what
 * the HIP library must compute.  It is called from tests/, from the smoke
 * check and from the benchmark's cpu_baseline leg, and from nowhere else.
 * It shares no code, header, table or helper with the HIP path.
 *
 * Everything works on ONE (batch, head) slab: q, k, v, dO are fp32 arrays
 * [L][d] holding values that are exactly representable in bf16 (the bits
 * the GPU sees, widened).  Python loops over slabs.
 *
 * Precision.  Dot products, exponentials and sums are carried in fp64.
 * The mask path rounds to fp32 at the two places where the method's own
 * data type is fp32 (a logit of the probe, a probability of the probe), so
 * the importance map P_imp is an fp32 array: it is the input of an integer
 * decision (the block mask) and the HIP path holds it in fp32 too.  The
 * selection rule then works on those fp32 values in fp64, in the order the
 * paper's algorithm states.  Attention and its gradients are fp64 end to end.
 *
 * Parity status against the authors' own implementation: UNPINNED.  The
 * paper prints no numeric example of a mask, a score or an output, so no
 * value here can be checked against theirs.  What pins this file instead
 * (dense attention, the dense soft-max map when every token is sampled,
 * closed forms for uniform scores, brute-force subset search, finite
 * differences, library autograd) lives in tests/test_oracle_*.py.
 *
 * Passages followed (paper "BLADE", Sec. 3.3 and the appendix "Pseudocode"):
 *   block sampling            Alg. 2 steps 1-3, Alg. 3 steps 2-3
 *   probe soft-max + max-pool Alg. 3 steps 4-5 (direct), Alg. 1 (online form)
 *   selection rule            Alg. 3 steps 6-11, Sec. 3.3 "Step 2.1"
 *   masked attention          Sec. 3.3 "Step 2.2", variant 1 (standard ASA)
 *   gradients                 soft-max attention calculus on the kept pairs
 *                             (the mask is used "during both training and
 *                             inference", Sec. 3.3 Step 2.1)
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define ASA_REF_OK 0
#define ASA_REF_BAD_ARG (-1)
#define ASA_REF_NOMEM (-2)

int asa_ref_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

static int thread_id(void) {
#ifdef _OPENMP
  return omp_get_thread_num();
#else
  return 0;
#endif
}

/* fp64 dot product of two fp32 rows. */
static double dot_fd(const float *a, const float *b, int d) {
  double acc = 0.0;
#pragma omp simd reduction(+ : acc)
  for (int x = 0; x < d; ++x) acc += (double)a[x] * (double)b[x];
  return acc;
}

static int nblocks(int L, int b) { return (L + b - 1) / b; }

/* --------------------------------------------------------------------------
 * Block sampling (Alg. 2 steps 1-3; Alg. 3 steps 2-3).
 * Sample u of block t is token t*b + offs[u]; it exists iff that index is
 * below L (the sequence is conceptually padded to a multiple of b and padded
 * positions never take part).  The same offsets serve Q and K.
 * row_of[t*ks+u] = token index or -1.
 * ------------------------------------------------------------------------ */
int asa_ref_sample_rows(int L, int b, int ks, const int32_t *offs, int32_t *row_of) {
  if (L < 1 || b < 1 || ks < 1 || ks > b || !offs || !row_of) return ASA_REF_BAD_ARG;
  for (int u = 0; u < ks; ++u) {
    if (offs[u] < 0 || offs[u] >= b) return ASA_REF_BAD_ARG;
    if (u && offs[u] <= offs[u - 1]) return ASA_REF_BAD_ARG;
  }
  int Nb = nblocks(L, b);
  for (int t = 0; t < Nb; ++t)
    for (int u = 0; u < ks; ++u) {
      int p = t * b + offs[u];
      row_of[t * ks + u] = (p < L) ? p : -1;
    }
  return ASA_REF_OK;
}

/* --------------------------------------------------------------------------
 * Importance map, direct form (Alg. 3 steps 4-5).
 *   s[r][c]  = fp32( scale * <Qs[r], Ks[c]> )
 *   p[r][c]  = fp32( softmax over ALL sampled keys c of s[r][.] )
 *   P_imp[i][j] = max of p over the sampled rows of block i and the sampled
 *                 keys of block j   (0 where no such pair exists)
 * ------------------------------------------------------------------------ */
int asa_ref_p_imp_direct(const float *q, const float *k, int L, int d, int b, int ks,
                         const int32_t *offs, float scale, float *p_imp) {
  if (!q || !k || !p_imp || d < 1) return ASA_REF_BAD_ARG;
  int Nb = nblocks(L, b);
  int Nk = Nb * ks;
  int32_t *row_of = (int32_t *)malloc(sizeof(int32_t) * (size_t)Nk);
  if (!row_of) return ASA_REF_NOMEM;
  int rc = asa_ref_sample_rows(L, b, ks, offs, row_of);
  if (rc) { free(row_of); return rc; }
  for (size_t t = 0; t < (size_t)Nb * Nb; ++t) p_imp[t] = 0.0f;
  int nthr = asa_ref_num_threads();
  float *s_all = (float *)malloc(sizeof(float) * (size_t)Nk * nthr);
  float *p_all = (float *)malloc(sizeof(float) * (size_t)Nk * nthr);
  if (!s_all || !p_all) { free(s_all); free(p_all); free(row_of); return ASA_REF_NOMEM; }
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthr)
  for (int i = 0; i < Nb; ++i) {
    float *s = s_all + (size_t)Nk * thread_id();
    float *p = p_all + (size_t)Nk * thread_id();
    for (int u = 0; u < ks; ++u) {
      int r = row_of[i * ks + u];
      if (r < 0) continue;
      /* logits of this sampled query against every sampled key */
      double m = -INFINITY;
      for (int c = 0; c < Nk; ++c) {
        int kc = row_of[c];
        if (kc < 0) { s[c] = -INFINITY; continue; }
        s[c] = (float)((double)scale * dot_fd(q + (size_t)r * d, k + (size_t)kc * d, d));
        if ((double)s[c] > m) m = (double)s[c];
      }
      double ell = 0.0;
      for (int c = 0; c < Nk; ++c)
        if (row_of[c] >= 0) ell += exp((double)s[c] - m);
      for (int c = 0; c < Nk; ++c)
        p[c] = (row_of[c] >= 0) ? (float)(exp((double)s[c] - m) / ell) : 0.0f;
      /* k x k max-pool: fold this row into row i of P_imp */
      for (int j = 0; j < Nb; ++j) {
        float best = p_imp[(size_t)i * Nb + j];
        for (int w = 0; w < ks; ++w) {
          int c = j * ks + w;
          if (row_of[c] >= 0 && p[c] > best) best = p[c];
        }
        p_imp[(size_t)i * Nb + j] = best;
      }
    }
  }
  free(s_all);
  free(p_all);
  free(row_of);
  return ASA_REF_OK;
}

/* --------------------------------------------------------------------------
 * Importance map, online form (Alg. 1 applied to the sampled tokens with
 * pooling size ks, as Alg. 2 step 4 calls it).  For each query block: a
 * first sweep over key blocks keeps, per sampled query row, the running
 * maximum Mt, the running denominator lt and the per-key-block row maximum
 * Rt[.][j]; a second sweep turns Rt into the largest probability inside each
 * (row, key block) and takes the maximum over rows.
 * ------------------------------------------------------------------------ */
int asa_ref_p_imp_online(const float *q, const float *k, int L, int d, int b, int ks,
                         const int32_t *offs, float scale, float *p_imp) {
  if (!q || !k || !p_imp || d < 1) return ASA_REF_BAD_ARG;
  int Nb = nblocks(L, b);
  int Nk = Nb * ks;
  int32_t *row_of = (int32_t *)malloc(sizeof(int32_t) * (size_t)Nk);
  if (!row_of) return ASA_REF_NOMEM;
  int rc = asa_ref_sample_rows(L, b, ks, offs, row_of);
  if (rc) { free(row_of); return rc; }
  int nthr = asa_ref_num_threads();
  size_t per = (size_t)2 * ks + (size_t)ks * Nb;
  double *scratch = (double *)malloc(sizeof(double) * per * nthr);
  float *sij_all = (float *)malloc(sizeof(float) * (size_t)ks * nthr);
  if (!scratch || !sij_all) { free(scratch); free(sij_all); free(row_of); return ASA_REF_NOMEM; }
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthr)
  for (int i = 0; i < Nb; ++i) {
    double *Mt = scratch + per * thread_id();
    double *lt = Mt + ks;
    double *Rt = lt + ks;
    float *sij = sij_all + (size_t)ks * thread_id();
    for (int u = 0; u < ks; ++u) { Mt[u] = -INFINITY; lt[u] = 0.0; }
    for (int j = 0; j < Nb; ++j) {
      for (int u = 0; u < ks; ++u) {
        int r = row_of[i * ks + u];
        Rt[(size_t)u * Nb + j] = -INFINITY;
        if (r < 0) continue;
        double mij = -INFINITY;
        for (int w = 0; w < ks; ++w) {
          int kc = row_of[j * ks + w];
          if (kc < 0) { sij[w] = -INFINITY; continue; }
          sij[w] = (float)((double)scale * dot_fd(q + (size_t)r * d, k + (size_t)kc * d, d));
          if ((double)sij[w] > mij) mij = (double)sij[w];
        }
        if (mij == -INFINITY) continue; /* key block without a sample */
        double lij = 0.0;
        for (int w = 0; w < ks; ++w)
          if (sij[w] != -INFINITY) lij += exp((double)sij[w] - mij);
        double mnew = (Mt[u] > mij) ? Mt[u] : mij;
        lt[u] = exp(Mt[u] - mnew) * lt[u] + exp(mij - mnew) * lij;
        Mt[u] = mnew;
        Rt[(size_t)u * Nb + j] = mij;
      }
    }
    for (int j = 0; j < Nb; ++j) {
      float best = 0.0f;
      for (int u = 0; u < ks; ++u) {
        if (row_of[i * ks + u] < 0) continue;
        double rt = Rt[(size_t)u * Nb + j];
        if (rt == -INFINITY) continue;
        float a = (float)(exp(rt - Mt[u]) / lt[u]);
        if (a > best) best = a;
      }
      p_imp[(size_t)i * Nb + j] = best;
    }
  }
  free(scratch);
  free(sij_all);
  free(row_of);
  return ASA_REF_OK;
}

/* --------------------------------------------------------------------------
 * Retention clamps (Alg. 3 step 9, "minimum and maximum retention ratios").
 * The paper gives neither values nor rounding; the reading used here:
 *   m_min = max(1, ceil(r_min * Nb)),  m_max = max(m_min, floor(r_max * Nb)),
 * both products taken in fp64 from the fp32 ratios.
 * ------------------------------------------------------------------------ */
int asa_ref_retention_bounds(int Nb, float r_min, float r_max, int32_t *m_min, int32_t *m_max) {
  if (Nb < 1 || !(r_min >= 0.0f) || !(r_max <= 1.0f) || !(r_min <= r_max)) return ASA_REF_BAD_ARG;
  int lo = (int)ceil((double)r_min * (double)Nb);
  if (lo < 1) lo = 1;
  if (lo > Nb) lo = Nb;
  int hi = (int)floor((double)r_max * (double)Nb);
  if (hi < lo) hi = lo;
  if (hi > Nb) hi = Nb;
  *m_min = lo;
  *m_max = hi;
  return ASA_REF_OK;
}

/* key order of the rule: larger score first, equal scores by lower index */
static int precedes(float pa, int ja, float pb, int jb) {
  return (pa > pb) || (pa == pb && ja < jb);
}

/* --------------------------------------------------------------------------
 * Selection rule, sort form (Alg. 3 steps 6-11) for `rows` independent rows
 * of length Nb.  Normalising a row by its sum T and asking for a cumulative
 * normalised score >= tau is the same as asking for a cumulative raw score
 * >= tau*T; the raw form is used so that no rounded quotient is ever summed.
 *   order   : descending score, ties by ascending block index
 *   c_0 = 0, c_{r+1} = c_r + p_(r)    (fp64, in that order);  T = c_Nb
 *   m*  = number of ranks r with c_r < tau*T
 *         (= the smallest m >= 1 whose first m blocks reach tau*T, Nb if none)
 *   m   = clamp(m*, m_min, m_max); keep the m first ranks.
 * A NaN score counts as 0.
 * ------------------------------------------------------------------------ */
int asa_ref_mask_rule_sort(const float *p_imp, int rows, int Nb, float tau, int m_min, int m_max,
                           uint8_t *mask, int32_t *m_out) {
  if (!p_imp || !mask || rows < 0 || Nb < 1 || m_min < 1 || m_max < m_min || m_max > Nb ||
      tau != tau)
    return ASA_REF_BAD_ARG;
  int nthr = asa_ref_num_threads();
  float *p_all = (float *)malloc(sizeof(float) * (size_t)Nb * nthr);
  int *ord_all = (int *)malloc(sizeof(int) * (size_t)Nb * nthr);
  double *c_all = (double *)malloc(sizeof(double) * ((size_t)Nb + 1) * nthr);
  if (!p_all || !ord_all || !c_all) { free(p_all); free(ord_all); free(c_all); return ASA_REF_NOMEM; }
#pragma omp parallel for schedule(static) num_threads(nthr)
  for (int i = 0; i < rows; ++i) {
    float *p = p_all + (size_t)Nb * thread_id();
    int *ord = ord_all + (size_t)Nb * thread_id();
    double *c = c_all + ((size_t)Nb + 1) * thread_id();
    const float *src = p_imp + (size_t)i * Nb;
    for (int j = 0; j < Nb; ++j) { p[j] = (src[j] == src[j]) ? src[j] : 0.0f; ord[j] = j; }
    /* insertion sort: stable, plain, Nb is a few hundred */
    for (int a = 1; a < Nb; ++a) {
      int ja = ord[a];
      int t = a - 1;
      while (t >= 0 && precedes(p[ja], ja, p[ord[t]], ord[t])) { ord[t + 1] = ord[t]; --t; }
      ord[t + 1] = ja;
    }
    c[0] = 0.0;
    for (int r = 0; r < Nb; ++r) c[r + 1] = c[r] + (double)p[ord[r]];
    double thr = (double)tau * c[Nb];
    int mstar = 0;
    for (int r = 0; r < Nb; ++r) if (c[r] < thr) ++mstar;
    int m = mstar;
    if (m < m_min) m = m_min;
    if (m > m_max) m = m_max;
    uint8_t *dst = mask + (size_t)i * Nb;
    memset(dst, 0, (size_t)Nb);
    for (int r = 0; r < m; ++r) dst[ord[r]] = 1;
    if (m_out) m_out[i] = m;
  }
  free(p_all); free(ord_all); free(c_all);
  return ASA_REF_OK;
}

/* --------------------------------------------------------------------------
 * Selection rule, order-free form: the same decisions written without a sort.
 *   rank_j = #{ l : key_l precedes key_j },  c(j) = sum of p_l over those l
 *   keep_j = rank_j < m_max  and  ( c(j) < tau*T  or  rank_j < m_min )
 * with T the plain sum of the row.  (Sums run in index order, so the fp64
 * roundings differ from the sort form by an ulp or so; decisions agree unless
 * a cumulative score sits within that of tau*T.)
 * ------------------------------------------------------------------------ */
int asa_ref_mask_rule_orderfree(const float *p_imp, int rows, int Nb, float tau, int m_min,
                                int m_max, uint8_t *mask, int32_t *m_out) {
  if (!p_imp || !mask || rows < 0 || Nb < 1 || m_min < 1 || m_max < m_min || m_max > Nb ||
      tau != tau)
    return ASA_REF_BAD_ARG;
#pragma omp parallel for schedule(static)
  for (int i = 0; i < rows; ++i) {
    const float *src = p_imp + (size_t)i * Nb;
    double T = 0.0;
    for (int j = 0; j < Nb; ++j) T += (src[j] == src[j]) ? (double)src[j] : 0.0;
    double thr = (double)tau * T;
    int m = 0;
    for (int j = 0; j < Nb; ++j) {
      float pj = (src[j] == src[j]) ? src[j] : 0.0f;
      int rank = 0;
      double cj = 0.0;
      for (int l = 0; l < Nb; ++l) {
        float pl = (src[l] == src[l]) ? src[l] : 0.0f;
        if (precedes(pl, l, pj, j)) { ++rank; cj += (double)pl; }
      }
      int keep = (rank < m_max) && (cj < thr || rank < m_min);
      mask[(size_t)i * Nb + j] = (uint8_t)keep;
      m += keep;
    }
    if (m_out) m_out[i] = m;
  }
  return ASA_REF_OK;
}

/* --------------------------------------------------------------------------
 * Always-kept prefix (CogVideoX text tokens; a workload convention, not in
 * the paper): every block that holds one of the first n_prefix tokens is kept
 * as a row and as a column, OR-ed in after the rule.
 * ------------------------------------------------------------------------ */
int asa_ref_force_prefix(uint8_t *mask, int Nb, int b, int n_prefix) {
  if (!mask || Nb < 1 || b < 1 || n_prefix < 0) return ASA_REF_BAD_ARG;
  int npb = (n_prefix + b - 1) / b;
  if (npb > Nb) npb = Nb;
  for (int i = 0; i < Nb; ++i)
    for (int j = 0; j < Nb; ++j)
      if (i < npb || j < npb) mask[(size_t)i * Nb + j] = 1;
  return ASA_REF_OK;
}

/* --------------------------------------------------------------------------
 * Masked soft-max attention, forward (Sec. 3.3 Step 2.2, standard ASA), for
 * the query blocks listed in qblocks.  Row q of block i sees key c iff
 * c < L and mask[i][c / b] = 1:
 *   S_c = scale * <Q_q, K_c>,  LSE_q = log sum_c exp(S_c),
 *   O_q = sum_c exp(S_c - LSE_q) V_c.
 * o [L][d] and lse [L] are full-size; only rows of the listed blocks are
 * written.  A row that sees no key gets O = 0, LSE = -inf.
 * ------------------------------------------------------------------------ */
int asa_ref_attn_fwd(const float *q, const float *k, const float *v, int L, int d, int b,
                     const uint8_t *mask, double scale, const int32_t *qblocks, int nq, double *o,
                     double *lse) {
  if (!q || !k || !v || !mask || !o || !lse || L < 1 || d < 1 || b < 1 || nq < 0) return ASA_REF_BAD_ARG;
  int Nb = nblocks(L, b);
  for (int t = 0; t < nq; ++t)
    if (qblocks[t] < 0 || qblocks[t] >= Nb) return ASA_REF_BAD_ARG;
  int nthr = asa_ref_num_threads();
  double *s_all = (double *)malloc(sizeof(double) * (size_t)L * nthr);
  if (!s_all) return ASA_REF_NOMEM;
#pragma omp parallel for schedule(dynamic, 4) collapse(2) num_threads(nthr)
  for (int t = 0; t < nq; ++t) {
    for (int rr = 0; rr < b; ++rr) {
      double *s = s_all + (size_t)L * thread_id();
      int i = qblocks[t];
      int r = i * b + rr;
      if (r >= L) continue;
      const uint8_t *mrow = mask + (size_t)i * Nb;
      double mx = -INFINITY;
      for (int c = 0; c < L; ++c) {
        if (!mrow[c / b]) continue;
        s[c] = scale * dot_fd(q + (size_t)r * d, k + (size_t)c * d, d);
        if (s[c] > mx) mx = s[c];
      }
      double *orow = o + (size_t)r * d;
      for (int x = 0; x < d; ++x) orow[x] = 0.0;
      if (mx == -INFINITY) { lse[r] = -INFINITY; continue; }
      double sum = 0.0;
      for (int c = 0; c < L; ++c)
        if (mrow[c / b]) sum += exp(s[c] - mx);
      double l = mx + log(sum);
      lse[r] = l;
      for (int c = 0; c < L; ++c) {
        if (!mrow[c / b]) continue;
        double p = exp(s[c] - l);
        const float *vrow = v + (size_t)c * d;
        for (int x = 0; x < d; ++x) orow[x] += p * (double)vrow[x];
      }
    }
  }
  free(s_all);
  return ASA_REF_OK;
}

/* Delta_q = <dO_q, O_q> for the rows of the listed query blocks. */
int asa_ref_attn_delta(const float *d_o, const double *o, int L, int d, int b,
                       const int32_t *qblocks, int nq, double *delta) {
  if (!d_o || !o || !delta || L < 1 || d < 1 || b < 1) return ASA_REF_BAD_ARG;
  for (int t = 0; t < nq; ++t)
    for (int rr = 0; rr < b; ++rr) {
      int r = qblocks[t] * b + rr;
      if (r >= L) continue;
      double acc = 0.0;
      for (int x = 0; x < d; ++x) acc += (double)d_o[(size_t)r * d + x] * o[(size_t)r * d + x];
      delta[r] = acc;
    }
  return ASA_REF_OK;
}

/* --------------------------------------------------------------------------
 * Gradients of the masked attention with the mask held constant.  With
 *   P_qc = exp(S_qc - LSE_q),  dP_qc = <dO_q, V_c>,  dS_qc = P_qc (dP_qc - Delta_q):
 *   dQ_q = scale * sum_c dS_qc K_c        (rows of the listed query blocks)
 *   dK_c = scale * sum_q dS_qc Q_q,  dV_c = sum_q P_qc dO_q
 *                                          (rows of the listed key blocks)
 * lse and delta must hold valid values for every query row that is touched:
 * the listed query blocks for dQ; every query block that keeps a listed key
 * block for dK, dV.
 * ------------------------------------------------------------------------ */
int asa_ref_attn_bwd_dq(const float *q, const float *k, const float *v, const float *d_o, int L,
                        int d, int b, const uint8_t *mask, double scale, const double *lse,
                        const double *delta, const int32_t *qblocks, int nq, double *dq) {
  if (!q || !k || !v || !d_o || !mask || !lse || !delta || !dq) return ASA_REF_BAD_ARG;
  int Nb = nblocks(L, b);
#pragma omp parallel for schedule(dynamic, 4) collapse(2)
  for (int t = 0; t < nq; ++t) {
    for (int rr = 0; rr < b; ++rr) {
      int i = qblocks[t];
      int r = i * b + rr;
      if (r >= L) continue;
      const uint8_t *mrow = mask + (size_t)i * Nb;
      double *g = dq + (size_t)r * d;
      for (int x = 0; x < d; ++x) g[x] = 0.0;
      for (int c = 0; c < L; ++c) {
        if (!mrow[c / b]) continue;
        double s = scale * dot_fd(q + (size_t)r * d, k + (size_t)c * d, d);
        double p = exp(s - lse[r]);
        double dp = dot_fd(d_o + (size_t)r * d, v + (size_t)c * d, d);
        double ds = p * (dp - delta[r]);
        const float *krow = k + (size_t)c * d;
        for (int x = 0; x < d; ++x) g[x] += scale * ds * (double)krow[x];
      }
    }
  }
  return ASA_REF_OK;
}

int asa_ref_attn_bwd_dkv(const float *q, const float *k, const float *v, const float *d_o, int L,
                         int d, int b, const uint8_t *mask, double scale, const double *lse,
                         const double *delta, const int32_t *kblocks, int nk, double *dk,
                         double *dv) {
  if (!q || !k || !v || !d_o || !mask || !lse || !delta || !dk || !dv) return ASA_REF_BAD_ARG;
  int Nb = nblocks(L, b);
#pragma omp parallel for schedule(dynamic, 4) collapse(2)
  for (int t = 0; t < nk; ++t) {
    for (int cc = 0; cc < b; ++cc) {
      int j = kblocks[t];
      int c = j * b + cc;
      if (c >= L) continue;
      double *gk = dk + (size_t)c * d;
      double *gv = dv + (size_t)c * d;
      for (int x = 0; x < d; ++x) { gk[x] = 0.0; gv[x] = 0.0; }
      for (int r = 0; r < L; ++r) {
        if (!mask[(size_t)(r / b) * Nb + j]) continue;
        double s = scale * dot_fd(q + (size_t)r * d, k + (size_t)c * d, d);
        double p = exp(s - lse[r]);
        double dp = dot_fd(d_o + (size_t)r * d, v + (size_t)c * d, d);
        double ds = p * (dp - delta[r]);
        const float *qrow = q + (size_t)r * d;
        const float *grow = d_o + (size_t)r * d;
        for (int x = 0; x < d; ++x) {
          gk[x] += scale * ds * (double)qrow[x];
          gv[x] += p * (double)grow[x];
        }
      }
    }
  }
  return ASA_REF_OK;
}

/* --------------------------------------------------------------------------
 * Size of what the gradient sums add up, before cancellation (used by the
 * tests to bound the rounding error that a bf16 implementation may show on
 * an element; no part of the method):
 *   dq_mag[q][x] = scale * sum_c |dS_qc| |K_cx|     (listed query blocks)
 *   dk_mag[c][x] = scale * sum_q |dS_qc| |Q_qx|,
 *   dv_mag[c][x] =         sum_q  P_qc   |dO_qx|    (listed key blocks)
 * Same loops and the same P, dP, dS as the gradient functions above.
 * ------------------------------------------------------------------------ */
int asa_ref_attn_bwd_dq_mag(const float *q, const float *k, const float *v, const float *d_o, int L,
                            int d, int b, const uint8_t *mask, double scale, const double *lse,
                            const double *delta, const int32_t *qblocks, int nq, double *dq_mag) {
  if (!q || !k || !v || !d_o || !mask || !lse || !delta || !dq_mag) return ASA_REF_BAD_ARG;
  int Nb = nblocks(L, b);
#pragma omp parallel for schedule(dynamic, 4) collapse(2)
  for (int t = 0; t < nq; ++t) {
    for (int rr = 0; rr < b; ++rr) {
      int i = qblocks[t];
      int r = i * b + rr;
      if (r >= L) continue;
      const uint8_t *mrow = mask + (size_t)i * Nb;
      double *g = dq_mag + (size_t)r * d;
      for (int x = 0; x < d; ++x) g[x] = 0.0;
      for (int c = 0; c < L; ++c) {
        if (!mrow[c / b]) continue;
        double s = scale * dot_fd(q + (size_t)r * d, k + (size_t)c * d, d);
        double p = exp(s - lse[r]);
        double dp = dot_fd(d_o + (size_t)r * d, v + (size_t)c * d, d);
        double ds = p * (dp - delta[r]);
        const float *krow = k + (size_t)c * d;
        for (int x = 0; x < d; ++x) g[x] += fabs(scale * ds * (double)krow[x]);
      }
    }
  }
  return ASA_REF_OK;
}

int asa_ref_attn_bwd_dkv_mag(const float *q, const float *k, const float *v, const float *d_o, int L,
                             int d, int b, const uint8_t *mask, double scale, const double *lse,
                             const double *delta, const int32_t *kblocks, int nk, double *dk_mag,
                             double *dv_mag) {
  if (!q || !k || !v || !d_o || !mask || !lse || !delta || !dk_mag || !dv_mag) return ASA_REF_BAD_ARG;
  int Nb = nblocks(L, b);
#pragma omp parallel for schedule(dynamic, 4) collapse(2)
  for (int t = 0; t < nk; ++t) {
    for (int cc = 0; cc < b; ++cc) {
      int j = kblocks[t];
      int c = j * b + cc;
      if (c >= L) continue;
      double *gk = dk_mag + (size_t)c * d;
      double *gv = dv_mag + (size_t)c * d;
      for (int x = 0; x < d; ++x) { gk[x] = 0.0; gv[x] = 0.0; }
      for (int r = 0; r < L; ++r) {
        if (!mask[(size_t)(r / b) * Nb + j]) continue;
        double s = scale * dot_fd(q + (size_t)r * d, k + (size_t)c * d, d);
        double p = exp(s - lse[r]);
        double dp = dot_fd(d_o + (size_t)r * d, v + (size_t)c * d, d);
        double ds = p * (dp - delta[r]);
        const float *qrow = q + (size_t)r * d;
        const float *grow = d_o + (size_t)r * d;
        for (int x = 0; x < d; ++x) {
          gk[x] += fabs(scale * ds * (double)qrow[x]);
          gv[x] += fabs(p * (double)grow[x]);
        }
      }
    }
  }
  return ASA_REF_OK;
}
