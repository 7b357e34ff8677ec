/*
 * TEST INFRASTRUCTURE ONLY -- plain, slow, fp64 CPU definition of Spatial Sparse Attention (SSA).
 *
 * This file is the checker for the HIP library, not part of the product: only tests, the smoke check and
 * the benchmark's cpu_baseline leg may call it.  It shares no code with the HIP path.
 *
 * What it computes (paper: Sec. "Spatial Sparse Attention"):
 *   - every branch is the dense softmax attention of eq. (2)-(3) restricted to an explicit key set;
 *   - compression keys/values are the mean over the active tokens of each m_cmp^3 block (eq. (5), mean-pool
 *     part only);
 *   - a selection block's score is the sum of the post-softmax compression probabilities of its child
 *     compression blocks, summed over the query heads of a GQA group (eq. (6));
 *   - the T best-scoring selection blocks per (token, KV head) are kept, ties to the lowest block id, the
 *     decision being taken on the score rounded to fp32; all their tokens form the key set (Algorithm 1);
 *   - the window branch attends over the tokens of the query's own m_win^3 window;
 *   - the output is the gate-weighted sum of the three branch outputs (eq. (4)).
 * Backward is the textbook softmax-attention gradient of that forward with the selected indices held
 * constant (the paper gives no backward).
 *
 * No tiling, no online softmax, no reordering: logits of a whole key set are formed, then normalised.
 * OpenMP only spreads independent queries over cores.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
  int32_t N, B, Hq, Hkv, d, T;
  int32_t Nc, Ns, Nw, Smax; /* block counts; Smax = max selection blocks in one batch item */
  double scale;             /* softmax scale, 1/sqrt(d) in eq. (3) */
  const int32_t *tok_item;  /* [N] batch item of each token */
  const int32_t *cmp_id;    /* [N] dense compression-block id of each token */
  const int32_t *slc_id;    /* [N] dense selection-block id */
  const int32_t *win_id;    /* [N] dense window id */
  const int32_t *cmp_parent;     /* [Nc] selection block containing each compression block */
  const int32_t *cmp_item_start; /* [B+1] compression-block id range of each item */
  const int32_t *slc_item_start; /* [B+1] selection-block id range of each item */
  const int32_t *cmp_mem_start, *cmp_mem; /* CSR: member tokens (caller order) of each compression block */
  const int32_t *slc_mem_start, *slc_mem; /* same for selection blocks */
  const int32_t *win_mem_start, *win_mem; /* same for windows */
} ssa_oracle_problem;

int ssa_oracle_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* eq. (5), mean-pool part: Xc[c,g,:] = mean over the tokens of block c of X[tok,g,:]. */
void ssa_oracle_pool(const ssa_oracle_problem *p, const double *X, double *Xc) {
  const int64_t row = (int64_t)p->Hkv * p->d;
  for (int32_t c = 0; c < p->Nc; ++c) {
    double *dst = Xc + (int64_t)c * row;
    for (int64_t i = 0; i < row; ++i) dst[i] = 0.0;
    const int32_t b = p->cmp_mem_start[c], e = p->cmp_mem_start[c + 1];
    for (int32_t j = b; j < e; ++j) {
      const double *src = X + (int64_t)p->cmp_mem[j] * row;
      for (int64_t i = 0; i < row; ++i) dst[i] += src[i];
    }
    for (int64_t i = 0; i < row; ++i) dst[i] /= (double)(e - b);
  }
}

/* Dense softmax attention (eq. (2)-(3)) of one query vector over an explicit key list.
 * Kb/Vb: [rows, Hkv, d]; keys[j] is a row index.  Writes o[d], returns log-sum-exp of the scaled logits and
 * leaves the normalised probabilities in prob[0..n). */
static double attend(const ssa_oracle_problem *p, const double *q, const double *Kb, const double *Vb, int g,
                     const int32_t *keys, int64_t n, double *o, double *prob) {
  const int d = p->d;
  const int64_t row = (int64_t)p->Hkv * d;
  double mx = -INFINITY;
  for (int64_t j = 0; j < n; ++j) {
    const double *k = Kb + (int64_t)keys[j] * row + (int64_t)g * d;
    double s = 0.0;
    for (int i = 0; i < d; ++i) s += q[i] * k[i];
    s *= p->scale;
    prob[j] = s;
    if (s > mx) mx = s;
  }
  double den = 0.0;
  for (int64_t j = 0; j < n; ++j) den += exp(prob[j] - mx);
  const double lse = mx + log(den);
  for (int i = 0; i < d; ++i) o[i] = 0.0;
  for (int64_t j = 0; j < n; ++j) {
    const double w = exp(prob[j] - lse);
    prob[j] = w;
    const double *v = Vb + (int64_t)keys[j] * row + (int64_t)g * d;
    for (int i = 0; i < d; ++i) o[i] += w * v[i];
  }
  return lse;
}

/* Pick the T largest of s[0..n) (fp32), ties to the lowest index; ids written ascending, offset by base, -1 padded. */
static void select_topk(const float *s, int n, int T, int base, int32_t *out, char *taken) {
  int cnt = 0;
  memset(taken, 0, (size_t)n);
  for (int r = 0; r < T && r < n; ++r) {
    int best = -1;
    for (int j = 0; j < n; ++j) {
      if (taken[j]) continue;
      if (best < 0 || s[j] > s[best]) best = j; /* strict >: an equal score never displaces a lower id */
    }
    taken[best] = 1;
    ++cnt;
  }
  int w = 0;
  for (int j = 0; j < n; ++j)
    if (taken[j]) out[w++] = base + j;
  for (; w < T; ++w) out[w] = -1;
  (void)cnt;
}

/* Gather the tokens of the selected blocks (ascending block id) into keys[]; returns their number. */
static int64_t gather_selected(const ssa_oracle_problem *p, const int32_t *I, int32_t *keys) {
  int64_t n = 0;
  for (int j = 0; j < p->T; ++j) {
    const int32_t b = I[j];
    if (b < 0) continue;
    for (int32_t m = p->slc_mem_start[b]; m < p->slc_mem_start[b + 1]; ++m) keys[n++] = p->slc_mem[m];
  }
  return n;
}

/*
 * Forward for the queries listed in qidx[0..nq) (caller-order token indices); rows of other tokens are
 * left untouched.  I_in == NULL: compute the top-k sets (written to I_out); otherwise use I_in's rows and
 * copy them to I_out.  scores32 (optional): [N,Hkv,Smax] fp32 selection scores, column j = j-th selection
 * block of the row's batch item.
 * Outputs (caller order): O [N,Hq,d]; Ob [3,N,Hq,d] (cmp,slc,win); lse [3,N,Hq]; I_out [N,Hkv,T].
 */
void ssa_oracle_forward(const ssa_oracle_problem *p, const double *Q, const double *K, const double *V,
                        const double *gates, const double *Kc, const double *Vc, int64_t nq,
                        const int32_t *qidx, const int32_t *I_in, double *O, double *Ob, double *lse,
                        float *scores32, int32_t *I_out) {
  const int d = p->d, Hq = p->Hq, Hkv = p->Hkv, hs = Hq / Hkv, T = p->T;
  const int64_t N = p->N;
#pragma omp parallel
  {
    double *prob = (double *)malloc(sizeof(double) * (size_t)(N > p->Nc ? N : p->Nc) + 8);
    int32_t *keys = (int32_t *)malloc(sizeof(int32_t) * (size_t)(N > p->Nc ? N : p->Nc) + 8);
    double *S = (double *)malloc(sizeof(double) * (size_t)(p->Smax + 1));
    float *S32 = (float *)malloc(sizeof(float) * (size_t)(p->Smax + 1));
    char *taken = (char *)malloc((size_t)(p->Smax + 1));
    double *o3 = (double *)malloc(sizeof(double) * 3 * (size_t)d);
#pragma omp for schedule(dynamic, 8)
    for (int64_t qi = 0; qi < nq; ++qi) {
      const int64_t t = qidx[qi];
      const int item = p->tok_item[t];
      const int c0 = p->cmp_item_start[item], c1 = p->cmp_item_start[item + 1];
      const int s0 = p->slc_item_start[item], s1 = p->slc_item_start[item + 1];
      for (int g = 0; g < Hkv; ++g) {
        /* --- compression branch + selection scores (eq. (4) first term, eq. (6)) --- */
        for (int b = 0; b < s1 - s0; ++b) S[b] = 0.0;
        for (int hl = 0; hl < hs; ++hl) {
          const int h = g * hs + hl;
          const double *q = Q + ((int64_t)t * Hq + h) * d;
          for (int c = c0; c < c1; ++c) keys[c - c0] = c;
          double *oc = Ob + (((int64_t)0 * N + t) * Hq + h) * d;
          lse[((int64_t)0 * N + t) * Hq + h] = attend(p, q, Kc, Vc, g, keys, c1 - c0, oc, prob);
          for (int c = c0; c < c1; ++c) S[p->cmp_parent[c] - s0] += prob[c - c0];
        }
        int32_t *Irow = I_out + ((int64_t)t * Hkv + g) * T;
        for (int b = 0; b < s1 - s0; ++b) S32[b] = (float)S[b];
        if (scores32) {
          float *dst = scores32 + ((int64_t)t * Hkv + g) * p->Smax;
          for (int b = 0; b < s1 - s0; ++b) dst[b] = S32[b];
          for (int b = s1 - s0; b < p->Smax; ++b) dst[b] = 0.0f;
        }
        if (I_in) {
          memcpy(Irow, I_in + ((int64_t)t * Hkv + g) * T, sizeof(int32_t) * (size_t)T);
        } else {
          select_topk(S32, s1 - s0, T, s0, Irow, taken);
        }
        /* --- selection branch (Algorithm 1's key set, evaluated densely) --- */
        const int64_t ns = gather_selected(p, Irow, keys);
        for (int hl = 0; hl < hs; ++hl) {
          const int h = g * hs + hl;
          const double *q = Q + ((int64_t)t * Hq + h) * d;
          double *os = Ob + (((int64_t)1 * N + t) * Hq + h) * d;
          lse[((int64_t)1 * N + t) * Hq + h] = attend(p, q, K, V, g, keys, ns, os, prob);
        }
        /* --- window branch --- */
        const int w = p->win_id[t];
        const int32_t *wk = p->win_mem + p->win_mem_start[w];
        const int64_t nw = p->win_mem_start[w + 1] - p->win_mem_start[w];
        for (int hl = 0; hl < hs; ++hl) {
          const int h = g * hs + hl;
          const double *q = Q + ((int64_t)t * Hq + h) * d;
          double *ow = Ob + (((int64_t)2 * N + t) * Hq + h) * d;
          lse[((int64_t)2 * N + t) * Hq + h] = attend(p, q, K, V, g, wk, nw, ow, prob);
        }
      }
      /* --- gated sum, eq. (4) --- */
      for (int h = 0; h < Hq; ++h) {
        const double *w = gates + ((int64_t)t * Hq + h) * 3;
        double *o = O + ((int64_t)t * Hq + h) * d;
        for (int i = 0; i < d; ++i) {
          double acc = 0.0;
          for (int b = 0; b < 3; ++b) acc += w[b] * Ob[(((int64_t)b * N + t) * Hq + h) * d + i];
          o[i] = acc;
        }
      }
    }
    free(prob); free(keys); free(S); free(S32); free(taken); free(o3);
  }
}

/* Gradient of one (query row, key list) softmax attention.  gb = gate * dO row (d), ob = branch output row.
 * Adds into dq[d] and into dKacc/dVacc rows (same layout as Kb/Vb). */
static void attend_bwd(const ssa_oracle_problem *p, const double *q, const double *Kb, const double *Vb, int g,
                       const int32_t *keys, int64_t n, const double *gb, const double *ob, double *dq,
                       double *dKacc, double *dVacc, double *prob) {
  const int d = p->d;
  const int64_t row = (int64_t)p->Hkv * d;
  /* probabilities, recomputed from the definition */
  double mx = -INFINITY;
  for (int64_t j = 0; j < n; ++j) {
    const double *k = Kb + (int64_t)keys[j] * row + (int64_t)g * d;
    double s = 0.0;
    for (int i = 0; i < d; ++i) s += q[i] * k[i];
    s *= p->scale;
    prob[j] = s;
    if (s > mx) mx = s;
  }
  double den = 0.0;
  for (int64_t j = 0; j < n; ++j) den += exp(prob[j] - mx);
  const double lse = mx + log(den);
  double delta = 0.0; /* <gb, ob> */
  for (int i = 0; i < d; ++i) delta += gb[i] * ob[i];
  for (int64_t j = 0; j < n; ++j) {
    const double pj = exp(prob[j] - lse);
    const int64_t off = (int64_t)keys[j] * row + (int64_t)g * d;
    const double *k = Kb + off, *v = Vb + off;
    double dp = 0.0;
    for (int i = 0; i < d; ++i) dp += gb[i] * v[i];
    const double ds = pj * (dp - delta) * p->scale;
    for (int i = 0; i < d; ++i) {
      dVacc[off + i] += pj * gb[i];
      dq[i] += ds * k[i];
      dKacc[off + i] += ds * q[i];
    }
  }
}

/*
 * Backward for the queries in qidx (rows of dO outside the list are treated as zero: the gradient is linear
 * in dO).  I [N,Hkv,T] are the selected blocks of the forward pass (constants).  Ob [3,N,Hq,d] are the branch
 * outputs of ssa_oracle_forward on the same inputs.  Outputs are overwritten: dQ [N,Hq,d], dK,dV [N,Hkv,d],
 * dgates [N,Hq,3].
 */
void ssa_oracle_backward(const ssa_oracle_problem *p, const double *Q, const double *K, const double *V,
                         const double *gates, const double *Kc, const double *Vc, const double *Ob,
                         const double *dO, int64_t nq, const int32_t *qidx, const int32_t *I, double *dQ,
                         double *dK, double *dV, double *dgates, double *dKc_out, double *dVc_out) {
  const int d = p->d, Hq = p->Hq, Hkv = p->Hkv, hs = Hq / Hkv, T = p->T;
  const int64_t N = p->N;
  const int64_t kvsz = N * Hkv * d, csz = (int64_t)p->Nc * Hkv * d;
  memset(dQ, 0, sizeof(double) * (size_t)(N * Hq * d));
  memset(dK, 0, sizeof(double) * (size_t)kvsz);
  memset(dV, 0, sizeof(double) * (size_t)kvsz);
  memset(dgates, 0, sizeof(double) * (size_t)(N * Hq * 3));
  double *dKc = (double *)calloc((size_t)csz + 1, sizeof(double));
  double *dVc = (double *)calloc((size_t)csz + 1, sizeof(double));
#pragma omp parallel
  {
    double *prob = (double *)malloc(sizeof(double) * (size_t)(N > p->Nc ? N : p->Nc) + 8);
    int32_t *keys = (int32_t *)malloc(sizeof(int32_t) * (size_t)(N > p->Nc ? N : p->Nc) + 8);
    double *gb = (double *)malloc(sizeof(double) * (size_t)d);
    /* per-thread accumulators for the key-side gradients, summed at the end */
    double *tK = (double *)calloc((size_t)kvsz + 1, sizeof(double));
    double *tV = (double *)calloc((size_t)kvsz + 1, sizeof(double));
    double *tKc = (double *)calloc((size_t)csz + 1, sizeof(double));
    double *tVc = (double *)calloc((size_t)csz + 1, sizeof(double));
#pragma omp for schedule(dynamic, 8)
    for (int64_t qi = 0; qi < nq; ++qi) {
      const int64_t t = qidx[qi];
      const int item = p->tok_item[t];
      const int c0 = p->cmp_item_start[item], c1 = p->cmp_item_start[item + 1];
      for (int h = 0; h < Hq; ++h) {
        const int g = h / hs;
        const double *q = Q + ((int64_t)t * Hq + h) * d;
        const double *go = dO + ((int64_t)t * Hq + h) * d;
        const double *w = gates + ((int64_t)t * Hq + h) * 3;
        double *dq = dQ + ((int64_t)t * Hq + h) * d;
        for (int b = 0; b < 3; ++b) {
          const double *ob = Ob + (((int64_t)b * N + t) * Hq + h) * d;
          double acc = 0.0;
          for (int i = 0; i < d; ++i) acc += go[i] * ob[i];
          dgates[((int64_t)t * Hq + h) * 3 + b] = acc; /* d o / d gate_b = o_b */
          for (int i = 0; i < d; ++i) gb[i] = w[b] * go[i];
          if (b == 0) {
            for (int c = c0; c < c1; ++c) keys[c - c0] = c;
            attend_bwd(p, q, Kc, Vc, g, keys, c1 - c0, gb, ob, dq, tKc, tVc, prob);
          } else if (b == 1) {
            const int64_t ns = gather_selected(p, I + ((int64_t)t * Hkv + g) * T, keys);
            attend_bwd(p, q, K, V, g, keys, ns, gb, ob, dq, tK, tV, prob);
          } else {
            const int wdw = p->win_id[t];
            attend_bwd(p, q, K, V, g, p->win_mem + p->win_mem_start[wdw],
                       p->win_mem_start[wdw + 1] - p->win_mem_start[wdw], gb, ob, dq, tK, tV, prob);
          }
        }
      }
    }
#pragma omp critical
    {
      for (int64_t i = 0; i < kvsz; ++i) { dK[i] += tK[i]; dV[i] += tV[i]; }
      for (int64_t i = 0; i < csz; ++i) { dKc[i] += tKc[i]; dVc[i] += tVc[i]; }
    }
    free(prob); free(keys); free(gb); free(tK); free(tV); free(tKc); free(tVc);
  }
  /* block-level keys/values supplied from outside (Kc, Vc are then not the mean pool of K, V): hand their
   * gradients out and leave dK, dV with the selection and window branches only */
  if (dKc_out != NULL && dVc_out != NULL) {
    memcpy(dKc_out, dKc, sizeof(double) * (size_t)csz);
    memcpy(dVc_out, dVc, sizeof(double) * (size_t)csz);
    free(dKc); free(dVc);
    return;
  }
  /* gradient of the mean pool: every member token receives dXc / count */
  const int64_t row = (int64_t)Hkv * d;
  for (int32_t c = 0; c < p->Nc; ++c) {
    const int32_t b = p->cmp_mem_start[c], e = p->cmp_mem_start[c + 1];
    for (int32_t j = b; j < e; ++j) {
      const int64_t tok = p->cmp_mem[j];
      for (int64_t i = 0; i < row; ++i) {
        dK[tok * row + i] += dKc[(int64_t)c * row + i] / (double)(e - b);
        dV[tok * row + i] += dVc[(int64_t)c * row + i] / (double)(e - b);
      }
    }
  }
  free(dKc); free(dVc);
}

/* Top-k decision alone, on caller-supplied fp32 scores [rows, Smax]; n_valid[r] candidates in row r whose
 * block ids start at base[r].  Used to pin the tie-break rule. */
void ssa_oracle_topk(const float *scores, int64_t rows, int Smax, int T, const int32_t *n_valid,
                     const int32_t *base, int32_t *out) {
  char *taken = (char *)malloc((size_t)Smax + 1);
  for (int64_t r = 0; r < rows; ++r)
    select_topk(scores + r * Smax, n_valid[r], T, base[r], out + r * T, taken);
  free(taken);
}
