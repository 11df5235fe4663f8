/*
 * CPU oracle for the slow/fast decode-attention path of Slow-Fast Inference.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, fp64
 * implementation written from the paper's definitions so that a reader can
 * check it against the paper by eye.  It shares no code with the HIP library;
 * only tests, the smoke check and the benchmark's CPU-baseline leg call it.
 *
 * Inputs are bf16 bit patterns (uint16_t); bf16 -> double is exact.  All
 * arithmetic is double.  Loops follow the order of the definitions; the only
 * parallelism is an OpenMP loop over independent (sequence, head) problems.
 *
 * What each function follows:
 *   sfio_logits    scaled dot-product logits l(j) = scale * <q, k_j>
 *                  (Sec. 3.1 "Slow step": dense attention over the prefix).
 *   sfio_dense     softmax(l) V over the whole prefix [0, L)  (same passage).
 *   sfio_sparse    the same attention restricted to the index set
 *                  I = I_sink U I_recent U I_sel  (Eq. index_set, Eq. index_set_head,
 *                  Sec. 3.1 "Fast step").
 *   sfio_reorg     cache reorganisation Reorg_i: the sink rows and the selected rows
 *                  copied into a contiguous compact buffer (Sec. 4.1 dependency
 *                  structure and Sec. 4.2 two-segment KV layout).
 *   sfio_trigger_schedule
 *                  the slow/fast indicator g_t of one request (Sec. 3.1 "Training-free
 *                  trigger policy", Eq. trigger, with the forced refresh after T_max fast
 *                  steps; Algorithm 1: g_0 = 1).
 *   sfio_advance   the state update between two decode steps: the context grows by one row and the
 *                  recent window slides with it (Algorithm 1, "Update I_recent"; Sec. 3.1 "Fast step").
 *   sfio_decode_loop
 *                  Algorithm 1 for a batch of requests with a scripted indicator g_t: slow steps attend
 *                  densely and refresh I_sel through the Selector, fast steps attend over
 *                  I_sink U I_recent U I_sel and keep I_sel (Eq. freeze_sel).
 *   sfio_selector_from_logits / sfio_selector
 *                  Algorithm 2 step by step: allowed set J (Eq. allowed_set),
 *                  evidence p, mu, f (Eqs. selector_pt, selector_mu, selector_f),
 *                  prior r (Eqs. selector_prior_kn, selector_u, selector_prior_pos,
 *                  selector_r), lambda* and fusion (Eqs. selector_lambda_closed,
 *                  selector_closed), log-score (Eq. z_base), Soft-NMS (Eqs. nms_pool,
 *                  nms), cross-head exclusivity (Eqs. head_softmax, head_mutex) and
 *                  Top-K (Eq. topk_out).
 *
 * Readings of points the paper leaves open (each also listed in the design notes):
 *   - positions are 0-based; ctx_len counts the rows in the cache, current token included;
 *   - I_sink = [0, n_sink), I_recent = [max(n_sink, L - recent), L), J = [n_sink, L - recent);
 *   - the G query heads that share one KV head play the role of the W window queries
 *     of Eq. selector_mu (one evidence vector per KV head);
 *   - Top-K orders by (-score, index): equal scores -> lower index first; the selected
 *     set is emitted ascending by index and padded with -1;
 *   - a window of W > 1 queries (Eq. window_logits) is handed in as W * G vectors per KV head; a window
 *     query that sits before the end of the context sees only the rows up to its own ("masked attention
 *     logit"): its softmax runs over the part of J it sees and it contributes p = 0 elsewhere, while the
 *     mean of Eq. selector_mu still divides by the full number of window vectors.
 *
 * Pins: tests/test_oracle_*.py (brute force on tiny inputs, closed forms, invariants,
 * library special cases).  The hyper-parameters gamma, beta, p, eta, T and the Soft-NMS
 * radius are not given by the paper: "parity unpinned" against the authors' code for
 * mode 1; pinned only against the equations.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
  int32_t B, Hq, Hkv, d;
  int32_t n_sink, recent;
  double scale;                       /* logit scale, e.g. 1/sqrt(d) */
  int64_t k_stride_b, k_stride_h, k_stride_t; /* in elements; a row of d elements is contiguous */
  int64_t v_stride_b, v_stride_h, v_stride_t;
  /* Selector */
  int32_t mode;                       /* 0: evidence only (s = f); 1: prior + fusion + refinements */
  int32_t nms_radius;                 /* N(j) = {i in J : |i - j| <= nms_radius} */
  double alpha;                       /* power-mean exponent, (0, 1] */
  double gamma, beta, p, eta;         /* prior shape */
  double lambda_clip, alpha_soft, alpha_cross, temp, eps;
} sfio_cfg;

static inline double bf16_to_double(uint16_t u) {
  uint32_t w = ((uint32_t)u) << 16;
  float f;
  memcpy(&f, &w, sizeof f);
  return (double)f;
}

static inline const uint16_t* k_row(const sfio_cfg* c, const uint16_t* K, int b, int h, int64_t j) {
  return K + b * c->k_stride_b + h * c->k_stride_h + j * c->k_stride_t;
}
static inline const uint16_t* v_row(const sfio_cfg* c, const uint16_t* V, int b, int h, int64_t j) {
  return V + b * c->v_stride_b + h * c->v_stride_h + j * c->v_stride_t;
}

/* l(j) = scale * sum_c q[c] k_j[c] */
static double logit_of(const sfio_cfg* c, const uint16_t* qrow, const uint16_t* krow) {
  double s = 0.0;
  for (int t = 0; t < c->d; ++t) s += bf16_to_double(qrow[t]) * bf16_to_double(krow[t]);
  return c->scale * s;
}

/* logits[b][g][j] for j < ctx_len[b]; row stride ld (>= max ctx_len). */
int sfio_logits(const sfio_cfg* c, const uint16_t* q, const uint16_t* K, const int32_t* ctx_len,
                double* logits, int64_t ld) {
  const int G = c->Hq / c->Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic)
  for (int b = 0; b < c->B; ++b)
    for (int g = 0; g < c->Hq; ++g) {
      const int h = g / G;
      const uint16_t* qrow = q + ((int64_t)b * c->Hq + g) * c->d;
      double* out = logits + ((int64_t)b * c->Hq + g) * ld;
      for (int64_t j = 0; j < ctx_len[b]; ++j) out[j] = logit_of(c, qrow, k_row(c, K, b, h, j));
    }
  return 0;
}

/* Attention of one query head over the rows flagged in take[0..L) (take == NULL: all rows).
 * out[c] = sum_j w(j) v_j[c] / sum_j w(j),  w(j) = exp(l(j) - max l). */
static void attend_rows(const sfio_cfg* c, const uint16_t* qrow, const uint16_t* K, const uint16_t* V, int b,
                        int h, int64_t L, const uint8_t* take, double* out) {
  double M = -INFINITY;
  for (int64_t j = 0; j < L; ++j) {
    if (take && !take[j]) continue;
    double l = logit_of(c, qrow, k_row(c, K, b, h, j));
    if (l > M) M = l;
  }
  double Z = 0.0;
  for (int t = 0; t < c->d; ++t) out[t] = 0.0;
  for (int64_t j = 0; j < L; ++j) {
    if (take && !take[j]) continue;
    double w = exp(logit_of(c, qrow, k_row(c, K, b, h, j)) - M);
    Z += w;
    const uint16_t* vr = v_row(c, V, b, h, j);
    for (int t = 0; t < c->d; ++t) out[t] += w * bf16_to_double(vr[t]);
  }
  if (Z > 0.0)
    for (int t = 0; t < c->d; ++t) out[t] /= Z;
}

/* Dense attention over [0, ctx_len[b]) for every query head.  out: [B, Hq, d] */
int sfio_dense(const sfio_cfg* c, const uint16_t* q, const uint16_t* K, const uint16_t* V,
               const int32_t* ctx_len, double* out) {
  const int G = c->Hq / c->Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic)
  for (int b = 0; b < c->B; ++b)
    for (int g = 0; g < c->Hq; ++g) {
      const uint16_t* qrow = q + ((int64_t)b * c->Hq + g) * c->d;
      attend_rows(c, qrow, K, V, b, g / G, ctx_len[b], NULL, out + ((int64_t)b * c->Hq + g) * c->d);
    }
  return 0;
}

/* Sparse attention over I = [0, n_sink) U sel_idx[b,h,0:n_sel] U [recent_start[b], L).
 * I is a set: duplicated or overlapping entries count once.  Entries outside [0, L) are an error. */
int sfio_sparse(const sfio_cfg* c, const uint16_t* q, const uint16_t* K, const uint16_t* V,
                const int32_t* sel_idx, const int32_t* n_sel, int64_t sel_stride,
                const int32_t* recent_start, const int32_t* ctx_len, double* out) {
  const int G = c->Hq / c->Hkv;
  int bad = 0;
#pragma omp parallel for collapse(2) schedule(dynamic)
  for (int b = 0; b < c->B; ++b)
    for (int h = 0; h < c->Hkv; ++h) {
      const int64_t L = ctx_len[b];
      uint8_t* take = (uint8_t*)calloc((size_t)(L > 0 ? L : 1), 1);
      for (int64_t j = 0; j < c->n_sink && j < L; ++j) take[j] = 1;
      const int32_t* s = sel_idx + ((int64_t)b * c->Hkv + h) * sel_stride;
      for (int i = 0; i < n_sel[(int64_t)b * c->Hkv + h]; ++i) {
        if (s[i] < 0 || s[i] >= L) {
#pragma omp atomic write
          bad = 1;
        } else
          take[s[i]] = 1;
      }
      for (int64_t j = recent_start[b] < 0 ? 0 : recent_start[b]; j < L; ++j) take[j] = 1;
      for (int gg = 0; gg < G; ++gg) {
        const int g = h * G + gg;
        const uint16_t* qrow = q + ((int64_t)b * c->Hq + g) * c->d;
        attend_rows(c, qrow, K, V, b, h, L, take, out + ((int64_t)b * c->Hq + g) * c->d);
      }
      free(take);
    }
  return bad ? -1 : 0;
}

/* ------------------------------------------------------------------ Selector */

typedef struct {
  double z;
  int32_t j;
} zj_t;

/* ascending in (-z, j): larger score first, equal scores -> lower index first */
static int cmp_zj(const void* a, const void* b) {
  const zj_t* x = (const zj_t*)a;
  const zj_t* y = (const zj_t*)b;
  if (x->z > y->z) return -1;
  if (x->z < y->z) return 1;
  return (x->j > y->j) - (x->j < y->j);
}
static int cmp_i32(const void* a, const void* b) {
  int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
  return (x > y) - (x < y);
}

/*
 * Selector from logits (Algorithm 2).
 *   logits : [B, Hq, ld_l]   l_g(j) for j < ctx_len[b]
 *   knorm  : [B, Hkv, ld_l]  ||k_h(j)||_2 (mode 1 only; may be NULL in mode 0)
 *   vis    : [B, Hq] or NULL: vector (b, g) sees rows [0, vis[b][g]) only (a window query under the
 *            causal mask, Eq. window_logits); NULL: every vector sees the whole context
 *   sel_idx: [B, Hkv, budget] out, ascending, padded with -1;  n_sel: [B, Hkv] out
 *   z_out  : [B, Hkv, ld_z]  optional: final ranking score per absolute position j
 *            (-inf outside J)
 *   dbg_f, dbg_r, dbg_s, dbg_zbase, dbg_znms : optional [B, Hkv, ld_z] intermediates
 *            (0 outside J); dbg_lambda: optional [B, Hkv].
 */
int sfio_selector_from_logits(const sfio_cfg* c, const double* logits, const double* knorm, int64_t ld_l,
                              const int32_t* vis, const int32_t* ctx_len, int32_t budget, int32_t* sel_idx, int32_t* n_sel,
                              double* z_out, int64_t ld_z, double* dbg_f, double* dbg_r, double* dbg_s,
                              double* dbg_zbase, double* dbg_znms, double* dbg_lambda) {
  const int G = c->Hq / c->Hkv;
  const double eps = c->eps;
  for (int b = 0; b < c->B; ++b) {
    const int64_t L = ctx_len[b];
    const int64_t j_lo = c->n_sink;          /* J = [j_lo, j_hi) (Eq. allowed_set) */
    const int64_t j_hi = L - c->recent;
    const int64_t nJ = j_hi > j_lo ? j_hi - j_lo : 0;
    const int32_t k_take = (int32_t)(budget < nJ ? budget : nJ);
    for (int h = 0; h < c->Hkv; ++h) {
      int32_t* s = sel_idx + ((int64_t)b * c->Hkv + h) * budget;
      for (int i = 0; i < budget; ++i) s[i] = -1;
      n_sel[(int64_t)b * c->Hkv + h] = k_take;
      if (z_out)
        for (int64_t j = 0; j < ld_z; ++j) z_out[((int64_t)b * c->Hkv + h) * ld_z + j] = -INFINITY;
    }
    if (nJ == 0) continue;

    /* z[h][jj], jj = j - j_lo */
    double* z = (double*)malloc(sizeof(double) * (size_t)c->Hkv * (size_t)nJ);

    /* (A) continuous importance, per KV head */
#pragma omp parallel for schedule(dynamic)
    for (int h = 0; h < c->Hkv; ++h) {
      const int64_t bh = (int64_t)b * c->Hkv + h;
      double* mu = (double*)calloc((size_t)nJ, sizeof(double));
      double* f = (double*)malloc(sizeof(double) * (size_t)nJ);
      double* sc = (double*)malloc(sizeof(double) * (size_t)nJ);
      /* Eq. selector_pt: p_g = softmax over J;  Eq. selector_mu: mu = (1/G) sum_g p_g^alpha */
      for (int gg = 0; gg < G; ++gg) {
        const double* l = logits + ((int64_t)b * c->Hq + h * G + gg) * ld_l;
        /* the part of J this vector sees: all of it, or up to its own row under the causal mask */
        int64_t j_end = j_hi;
        if (vis && vis[(int64_t)b * c->Hq + h * G + gg] < j_end) j_end = vis[(int64_t)b * c->Hq + h * G + gg];
        double M = -INFINITY;
        for (int64_t j = j_lo; j < j_end; ++j)
          if (l[j] > M) M = l[j];
        double Z = 0.0;
        for (int64_t j = j_lo; j < j_end; ++j) Z += exp(l[j] - M);
        for (int64_t j = j_lo; j < j_end; ++j) {
          double p = exp(l[j] - M) / Z;
          mu[j - j_lo] += pow(p, c->alpha) / (double)G;
        }
      }
      /* Eq. selector_f: f = mu^(1/alpha) / sum mu^(1/alpha) */
      double fs = 0.0;
      for (int64_t i = 0; i < nJ; ++i) {
        f[i] = pow(mu[i], 1.0 / c->alpha);
        fs += f[i];
      }
      for (int64_t i = 0; i < nJ; ++i) f[i] /= fs;

      double lambda = 0.0;
      if (c->mode == 0) {
        for (int64_t i = 0; i < nJ; ++i) sc[i] = f[i];
      } else {
        /* Eqs. selector_prior_kn, selector_u, selector_prior_pos, selector_r */
        double* r = (double*)malloc(sizeof(double) * (size_t)nJ);
        const double jmin = (double)j_lo, jmax = (double)(j_hi - 1);
        double rs = 0.0;
        for (int64_t i = 0; i < nJ; ++i) {
          const double kn = knorm[bh * ld_l + (j_lo + i)];
          const double pi_kn = pow(kn + eps, -c->gamma);
          const double u = ((double)(j_lo + i) - jmin) / (jmax - jmin + eps);
          const double pi_pos = exp(-c->beta * pow(u, c->p)) * pow(1.0 - u + eps, c->eta);
          r[i] = pi_kn * pi_pos;
          rs += r[i];
        }
        for (int64_t i = 0; i < nJ; ++i) r[i] /= rs;
        /* Eq. selector_lambda_closed */
        double ff = 0.0, fr = 0.0, rr = 0.0;
        for (int64_t i = 0; i < nJ; ++i) {
          ff += f[i] * f[i];
          fr += f[i] * r[i];
          rr += r[i] * r[i];
        }
        const double den = ff - 2.0 * fr + rr;
        lambda = den > 1e-300 ? (ff - fr) / den : 0.0;
        if (lambda < 0.0) lambda = 0.0;
        if (lambda > c->lambda_clip) lambda = c->lambda_clip;
        /* Eq. selector_closed */
        for (int64_t i = 0; i < nJ; ++i) sc[i] = (1.0 - lambda) * f[i] + lambda * r[i];
        if (dbg_r)
          for (int64_t i = 0; i < nJ; ++i) dbg_r[bh * ld_z + j_lo + i] = r[i];
        free(r);
      }
      /* Eq. z_base */
      for (int64_t i = 0; i < nJ; ++i) z[(int64_t)h * nJ + i] = log(sc[i] + eps);
      if (dbg_f)
        for (int64_t i = 0; i < nJ; ++i) dbg_f[bh * ld_z + j_lo + i] = f[i];
      if (dbg_s)
        for (int64_t i = 0; i < nJ; ++i) dbg_s[bh * ld_z + j_lo + i] = sc[i];
      if (dbg_zbase)
        for (int64_t i = 0; i < nJ; ++i) dbg_zbase[bh * ld_z + j_lo + i] = z[(int64_t)h * nJ + i];
      if (dbg_lambda) dbg_lambda[bh] = lambda;
      free(mu);
      free(f);
      free(sc);
    }

    /* (B) refinements in log-score space (mode 1) */
    if (c->mode != 0) {
      /* Soft-NMS, one pass on the un-updated scores, neighbourhood clipped to J */
      for (int h = 0; h < c->Hkv; ++h) {
        double* zh = z + (int64_t)h * nJ;
        double* zn = (double*)malloc(sizeof(double) * (size_t)nJ);
        for (int64_t i = 0; i < nJ; ++i) {
          double m = -INFINITY;
          for (int64_t t = i - c->nms_radius; t <= i + c->nms_radius; ++t)
            if (t >= 0 && t < nJ && zh[t] > m) m = zh[t];
          const double gap = m - zh[i];
          zn[i] = zh[i] - c->alpha_soft * (gap > 0.0 ? gap : 0.0);
        }
        memcpy(zh, zn, sizeof(double) * (size_t)nJ);
        free(zn);
        if (dbg_znms)
          for (int64_t i = 0; i < nJ; ++i) dbg_znms[((int64_t)b * c->Hkv + h) * ld_z + j_lo + i] = zh[i];
      }
      /* cross-head exclusivity at each position */
      double* zc = (double*)malloc(sizeof(double) * (size_t)c->Hkv);
      for (int64_t i = 0; i < nJ; ++i) {
        double M = -INFINITY;
        for (int h = 0; h < c->Hkv; ++h) {
          zc[h] = z[(int64_t)h * nJ + i] / c->temp;
          if (zc[h] > M) M = zc[h];
        }
        double Z = 0.0;
        for (int h = 0; h < c->Hkv; ++h) Z += exp(zc[h] - M);
        for (int h = 0; h < c->Hkv; ++h) {
          double resp = exp(zc[h] - M) / Z;
          if (resp < eps) resp = eps;
          z[(int64_t)h * nJ + i] += c->alpha_cross * log(resp);
        }
      }
      free(zc);
    }

    /* Top-K per head (Eq. topk_out) */
#pragma omp parallel for schedule(dynamic)
    for (int h = 0; h < c->Hkv; ++h) {
      const int64_t bh = (int64_t)b * c->Hkv + h;
      zj_t* a = (zj_t*)malloc(sizeof(zj_t) * (size_t)nJ);
      for (int64_t i = 0; i < nJ; ++i) {
        a[i].z = z[(int64_t)h * nJ + i];
        a[i].j = (int32_t)(j_lo + i);
      }
      qsort(a, (size_t)nJ, sizeof(zj_t), cmp_zj);
      int32_t* s = sel_idx + bh * budget;
      for (int i = 0; i < k_take; ++i) s[i] = a[i].j;
      qsort(s, (size_t)k_take, sizeof(int32_t), cmp_i32);
      if (z_out)
        for (int64_t i = 0; i < nJ; ++i) z_out[bh * ld_z + j_lo + i] = z[(int64_t)h * nJ + i];
      free(a);
    }
    free(z);
  }
  return 0;
}

/* Selector from q and K: computes the logits and (mode 1) key norms, then Algorithm 2. */
int sfio_selector(const sfio_cfg* c, const uint16_t* q, const uint16_t* K, const int32_t* vis, const int32_t* ctx_len,
                  int32_t budget, int32_t* sel_idx, int32_t* n_sel, double* z_out, int64_t ld_z) {
  int64_t ld = 1;
  for (int b = 0; b < c->B; ++b)
    if (ctx_len[b] > ld) ld = ctx_len[b];
  double* logits = (double*)malloc(sizeof(double) * (size_t)c->B * c->Hq * (size_t)ld);
  double* knorm = NULL;
  sfio_logits(c, q, K, ctx_len, logits, ld);
  if (c->mode != 0) {
    knorm = (double*)calloc((size_t)c->B * c->Hkv * (size_t)ld, sizeof(double));
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < c->B; ++b)
      for (int h = 0; h < c->Hkv; ++h)
        for (int64_t j = 0; j < ctx_len[b]; ++j) {
          const uint16_t* kr = k_row(c, K, b, h, j);
          double s = 0.0;
          for (int t = 0; t < c->d; ++t) s += bf16_to_double(kr[t]) * bf16_to_double(kr[t]);
          knorm[((int64_t)b * c->Hkv + h) * ld + j] = sqrt(s);
        }
  }
  int rc = sfio_selector_from_logits(c, logits, knorm, ld, vis, ctx_len, budget, sel_idx, n_sel, z_out, ld_z, NULL,
                                     NULL, NULL, NULL, NULL, NULL);
  free(logits);
  free(knorm);
  return rc;
}

/* Reorg: Kc[b][h][i] = K[b][h][i] for i < min(n_sink, L_b);  Kc[b][h][n_sink + i] = K[b][h][sel_idx[b][h][i]]
 * for i < n_sel[b][h]; likewise Vc.  Kc, Vc: [B, Hkv, c_rows, d], rows not named here are left untouched.
 * Returns -1 if a selected index lies outside [0, L_b) or the buffer is too small. */
int sfio_reorg(const sfio_cfg* c, const uint16_t* K, const uint16_t* V, const int32_t* sel_idx, const int32_t* n_sel,
               int64_t sel_stride, const int32_t* ctx_len, uint16_t* Kc, uint16_t* Vc, int64_t c_rows) {
  for (int b = 0; b < c->B; ++b)
    for (int h = 0; h < c->Hkv; ++h) {
      const int64_t bh = (int64_t)b * c->Hkv + h;
      const int64_t L = ctx_len[b];
      uint16_t* kc = Kc + bh * c_rows * c->d;
      uint16_t* vc = Vc + bh * c_rows * c->d;
      if (c->n_sink + (int64_t)n_sel[bh] > c_rows) return -1;
      for (int64_t i = 0; i < c->n_sink && i < L; ++i) {
        memcpy(kc + i * c->d, k_row(c, K, b, h, i), sizeof(uint16_t) * (size_t)c->d);
        memcpy(vc + i * c->d, v_row(c, V, b, h, i), sizeof(uint16_t) * (size_t)c->d);
      }
      for (int64_t i = 0; i < n_sel[bh]; ++i) {
        const int64_t j = sel_idx[bh * sel_stride + i];
        if (j < 0 || j >= L) return -1;
        memcpy(kc + (c->n_sink + i) * c->d, k_row(c, K, b, h, j), sizeof(uint16_t) * (size_t)c->d);
        memcpy(vc + (c->n_sink + i) * c->d, v_row(c, V, b, h, j), sizeof(uint16_t) * (size_t)c->d);
      }
    }
  return 0;
}

/* g[t] for t = 0 .. n_steps-1.  x[t] is the token generated at step t; trig[0..n_trig) the trigger ids.
 * g[0] = 1; for t >= 1: g[t] = 1 if x[t-1] is a trigger token, or if the T_max steps before t were all fast. */
int sfio_trigger_schedule(const int32_t* x, int32_t n_steps, const int32_t* trig, int32_t n_trig, int32_t t_max,
                          uint8_t* g) {
  int32_t fast_run = 0; /* fast steps since the last slow step */
  for (int32_t t = 0; t < n_steps; ++t) {
    int slow = 0;
    if (t == 0) {
      slow = 1;
    } else {
      for (int32_t i = 0; i < n_trig; ++i)
        if (trig[i] == x[t - 1]) slow = 1;
      if (fast_run >= t_max) slow = 1;
    }
    g[t] = (uint8_t)slow;
    fast_run = slow ? 0 : fast_run + 1;
  }
  return 0;
}

/* State update between two decode steps (Algorithm 1, "Update I_recent"): the new token's row joins the cache,
 * L <- L + 1, and the recent window slides: I_recent = [max(n_sink, L - recent), L). */
int sfio_advance(const sfio_cfg* c, int32_t* ctx_len, int32_t* recent_start) {
  for (int b = 0; b < c->B; ++b) {
    const int32_t L = ctx_len[b] + 1;
    ctx_len[b] = L;
    recent_start[b] = L - c->recent > c->n_sink ? L - c->recent : c->n_sink;
  }
  return 0;
}

/*
 * Algorithm 1 for B requests over n_steps decode steps with a scripted indicator g[t][b] (1 = slow step).
 *   q        : [n_steps, B, Hq, d]  the query of every step
 *   K, V     : caches that already hold the rows of every step (row L0[b] + t - 1 is step t's own token)
 *   ctx_len, recent_start : [B] in / out: the state before step 0, left as after the last step
 *   sel_idx, n_sel : [B, Hkv, budget], [B, Hkv] in / out: I_sel before step 0 (n_sel = 0: empty), left as after
 *                    the last step
 *   out      : [n_steps, B, Hq, d]
 *   sel_hist : optional [n_steps, B, Hkv, budget], nsel_hist optional [n_steps, B, Hkv]: I_sel after each step
 *   ctx_hist, rs_hist : optional [n_steps, B]: the state each step ran on
 * Per step and request: fast -> attention over I_sink U I_recent U I_sel, I_sel kept (Eq. freeze_sel);
 * slow -> dense attention over the prefix, I_sel <- Selector on J (Algorithm 2); then the state update.
 */
int sfio_decode_loop(const sfio_cfg* c, const uint16_t* q, const uint16_t* K, const uint16_t* V, int32_t n_steps,
                     const uint8_t* g, int32_t budget, int32_t* ctx_len, int32_t* recent_start, int32_t* sel_idx,
                     int32_t* n_sel, double* out, int32_t* sel_hist, int32_t* nsel_hist, int32_t* ctx_hist,
                     int32_t* rs_hist) {
  const int64_t q_step = (int64_t)c->B * c->Hq * c->d;
  int rc = 0;
  for (int32_t t = 0; t < n_steps; ++t) {
    for (int b = 0; b < c->B; ++b) {
      /* request b on its own: a batch of one at the request's offsets */
      sfio_cfg c1 = *c;
      c1.B = 1;
      const uint16_t* qb = q + t * q_step + (int64_t)b * c->Hq * c->d;
      const uint16_t* Kb = K + b * c->k_stride_b;
      const uint16_t* Vb = V + b * c->v_stride_b;
      double* ob = out + t * q_step + (int64_t)b * c->Hq * c->d;
      int32_t* sel_b = sel_idx + (int64_t)b * c->Hkv * budget;
      int32_t* nsel_b = n_sel + (int64_t)b * c->Hkv;
      if (ctx_hist) ctx_hist[(int64_t)t * c->B + b] = ctx_len[b];
      if (rs_hist) rs_hist[(int64_t)t * c->B + b] = recent_start[b];
      if (g[(int64_t)t * c->B + b]) {
        rc |= sfio_dense(&c1, qb, Kb, Vb, ctx_len + b, ob);
        rc |= sfio_selector(&c1, qb, Kb, NULL, ctx_len + b, budget, sel_b, nsel_b, NULL, 0);
      } else {
        rc |= sfio_sparse(&c1, qb, Kb, Vb, sel_b, nsel_b, budget, recent_start + b, ctx_len + b, ob);
      }
    }
    if (sel_hist) memcpy(sel_hist + (int64_t)t * c->B * c->Hkv * budget, sel_idx, sizeof(int32_t) * (size_t)c->B * c->Hkv * budget);
    if (nsel_hist) memcpy(nsel_hist + (int64_t)t * c->B * c->Hkv, n_sel, sizeof(int32_t) * (size_t)c->B * c->Hkv);
    sfio_advance(c, ctx_len, recent_start);
  }
  return rc;
}

int sfio_num_threads(void) {
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
