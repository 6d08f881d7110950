/*
 * QSAC oracle: a plain, slow CPU statement of the per-decode-step QSAC path
 * (LiteCache, arXiv 2511.14510).
 *
 * THIS IS TEST INFRASTRUCTURE.  It exists to be compared against; nothing on
 * the product path may call it, and it shares no code with the HIP path.  It
 * widens the 16-bit inputs (IEEE binary16 or bfloat16 bit patterns) to fp64
 * and does every piece of arithmetic in fp64, one key, one head and one pair
 * at a time, with no blocking, fusion or reordering.
 *
 * Paper passages followed:
 *   CosSim                      - Section 3.1, unnumbered equation
 *   qkscore                     - Section 3.1, Eq. (1)
 *   per-step control flow       - Section 4, Algorithm 1 (lookup, miss path,
 *                                 label update only on miss, attention)
 *   GQA similarity aggregation  - Section 4.2, Eq. (2)
 *   adaptive thresholds         - Section 4.3, Eq. (3)-(5)
 *   reuse difficulty            - Section 4.4 (D_i)
 *   attention                   - Section 2.1, softmax(q K^T / sqrt(d_k)) V
 *
 * Readings taken where the paper is silent (they bind the HIP path too):
 *   - the gate compares with ">=" (equality reuses);
 *   - the cached query label q_c is rewritten only on a miss;
 *   - the gate is taken per KV head: per-query-head cosines are aggregated by
 *     Eq. (2); if any cosine of the group is <= 0 the aggregate is -1;
 *   - a zero-norm q or q_c has cosine -1;
 *   - a head with no valid cache (first step) always misses, hit_mask all 0;
 *   - the retrieval score of key n for a KV head is max over its query heads
 *     of the raw dot product q_g . k_n (Eq. (1) when the group has one head);
 *   - keys are ranked by (score descending, index ascending); -0.0 ranks as
 *     +0.0; the selected set is reported in ascending index order;
 *   - on a miss the cache ends up holding exactly Gather(K, V, index) as in
 *     Algorithm 1; rows already cached stay in their slots, the i-th slot
 *     (ascending) whose token left the set receives the i-th (ascending)
 *     token that entered it;
 *   - sink and recent tokens (Section 7.1: kept in the cache persistently): the
 *     first n_sink and the last n_recent of the N context tokens rank above
 *     every other token (score +infinity) in every retrieval;
 *   - append-only buffer (Sections 6.1, 6.2): the KV of tokens generated during
 *     decoding sit in a GPU buffer of which n_app rows are valid at a step; the
 *     attention runs over the k cached rows and all n_app appended rows.
 *
 * Parity pins (tests/test_oracle_*.py) cover every function below; no
 * function here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { QO_F16 = 0, QO_BF16 = 1 };

/* ---- 16-bit patterns -> fp64, exactly ---------------------------------- */

static double widen_f16(uint16_t h) {
  int sign = (h >> 15) & 1;
  int e = (h >> 10) & 0x1f;
  int m = h & 0x3ff;
  double v;
  if (e == 0) {
    v = ldexp((double)m, -24); /* subnormal or zero */
  } else if (e == 31) {
    v = m ? NAN : INFINITY;
  } else {
    v = ldexp((double)(m | 0x400), e - 25);
  }
  return sign ? -v : v;
}

static double widen_bf16(uint16_t b) {
  uint32_t u = ((uint32_t)b) << 16; /* bfloat16 is the top half of binary32 */
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

double qo_widen(uint16_t bits, int dtype) {
  return dtype == QO_F16 ? widen_f16(bits) : widen_bf16(bits);
}

static double dot16(const uint16_t *a, const uint16_t *b, int D, int dtype) {
  double s = 0.0;
  for (int d = 0; d < D; ++d) s += qo_widen(a[d], dtype) * qo_widen(b[d], dtype);
  return s;
}

/* ---- CosSim (Section 3.1) ---------------------------------------------- */

double qo_cossim(const uint16_t *a, const uint16_t *b, int D, int dtype) {
  double ab = dot16(a, b, D, dtype);
  double aa = dot16(a, a, D, dtype);
  double bb = dot16(b, b, D, dtype);
  if (aa == 0.0 || bb == 0.0) return -1.0;
  return ab / (sqrt(aa) * sqrt(bb));
}

/* ---- Eq. (2): importance-weighted harmonic aggregation ------------------ */

double qo_aggregate(const double *sim, const double *w, int m) {
  double num = 0.0, den = 0.0;
  for (int j = 0; j < m; ++j) {
    double wj = w ? w[j] : 1.0;
    if (sim[j] <= 0.0) return -1.0;
    num += wj;
    den += wj / sim[j];
  }
  return num / den;
}

/* ---- Eq. (3)-(5): adaptive threshold; Section 4.4: reuse difficulty ----- */

double qo_adaptive_tau(double importance, double eta, double p) {
  double theta_star = acos(eta);
  double lambda = pow(importance, p);
  double theta = lambda * theta_star + (1.0 - lambda) * M_PI;
  return cos(theta);
}

double qo_reuse_difficulty(double tau, double avg_sim, double eps) {
  return tau - (avg_sim - eps);
}

/* ---- Eq. (1) over a query group: S[n] = max_g q_g . k_n ----------------- */

void qo_scores(const uint16_t *q /*[G][D]*/, const uint16_t *K /*[N][D]*/,
               int G, int64_t N, int D, int dtype, double *S /*[N]*/) {
  for (int64_t n = 0; n < N; ++n) {
    double best = -INFINITY;
    for (int g = 0; g < G; ++g) {
      double s = dot16(q + (size_t)g * D, K + (size_t)n * D, D, dtype);
      if (s > best) best = s;
    }
    S[n] = best;
  }
}

/* ---- top-k under the total order (score desc, index asc) ---------------- */

typedef struct {
  double s;
  int32_t n;
} ranked;

static int rank_cmp(const void *pa, const void *pb) {
  const ranked *a = (const ranked *)pa, *b = (const ranked *)pb;
  if (a->s > b->s) return -1;
  if (a->s < b->s) return 1;
  return (a->n > b->n) - (a->n < b->n);
}

static int int_cmp(const void *pa, const void *pb) {
  int32_t a = *(const int32_t *)pa, b = *(const int32_t *)pb;
  return (a > b) - (a < b);
}

/* idx_out gets the k selected indices in ascending index order; if kth_score
 * is not NULL it receives the score of the last key admitted. */
int qo_topk(const double *S, int64_t N, int k, int32_t *idx_out, double *kth_score) {
  if (k < 0 || k > N) return -1;
  ranked *r = (ranked *)malloc(sizeof(ranked) * (size_t)(N > 0 ? N : 1));
  if (!r) return -2;
  for (int64_t n = 0; n < N; ++n) {
    r[n].s = (S[n] == 0.0) ? 0.0 : S[n]; /* -0.0 ranks as +0.0 */
    r[n].n = (int32_t)n;
  }
  qsort(r, (size_t)N, sizeof(ranked), rank_cmp);
  for (int j = 0; j < k; ++j) idx_out[j] = r[j].n;
  if (kth_score && k > 0) *kth_score = r[k - 1].s;
  free(r);
  qsort(idx_out, (size_t)k, sizeof(int32_t), int_cmp);
  return 0;
}

/* ---- attention over a set of rows (Section 2.1) ------------------------- */

/* out[D] = sum_j w_j V[j], w = softmax_j(q . K[j] / sqrt(D)); w_out optional. */
void qo_attention(const uint16_t *q, const uint16_t *Kc, const uint16_t *Vc,
                  int k, int D, int dtype, double *out, double *w_out) {
  double *x = (double *)malloc(sizeof(double) * (size_t)(k > 0 ? k : 1));
  double mx = -INFINITY;
  for (int j = 0; j < k; ++j) {
    x[j] = dot16(q, Kc + (size_t)j * D, D, dtype) / sqrt((double)D);
    if (x[j] > mx) mx = x[j];
  }
  double z = 0.0;
  for (int j = 0; j < k; ++j) {
    x[j] = exp(x[j] - mx);
    z += x[j];
  }
  for (int d = 0; d < D; ++d) out[d] = 0.0;
  for (int j = 0; j < k; ++j) {
    double w = x[j] / z;
    if (w_out) w_out[j] = w;
    for (int d = 0; d < D; ++d) out[d] += w * qo_widen(Vc[(size_t)j * D + d], dtype);
  }
  free(x);
}

/* ---- slot diff of Algorithm 1's "transfer" step ------------------------- */

/*
 * old set = slot_idx[0..k) (ignored when !valid), new set = topk_idx (ascending).
 * hit_mask[j] = valid && topk_idx[j] in old.  Slots whose token is not in the
 * new set (all slots when !valid), in ascending slot order, receive the new
 * tokens that are not in the old set, in ascending token order.
 * miss_slot/miss_tok (optional, length k) receive the pairs; returns the
 * number of pairs, or <0 on a malformed state.  slot_idx is updated in place.
 */
int qo_diff(int valid, int64_t N, int k, int32_t *slot_idx, const int32_t *topk_idx,
            uint8_t *hit_mask, int32_t *miss_slot, int32_t *miss_tok) {
  uint8_t *in_old = (uint8_t *)calloc((size_t)N, 1);
  uint8_t *in_new = (uint8_t *)calloc((size_t)N, 1);
  int32_t *slots = (int32_t *)malloc(sizeof(int32_t) * (size_t)(k > 0 ? k : 1));
  int32_t *toks = (int32_t *)malloc(sizeof(int32_t) * (size_t)(k > 0 ? k : 1));
  int ns = 0, nt = 0, rc = 0;
  if (valid)
    for (int j = 0; j < k; ++j) {
      if (slot_idx[j] < 0 || slot_idx[j] >= N || in_old[slot_idx[j]]) { rc = -3; goto done; }
      in_old[slot_idx[j]] = 1;
    }
  for (int j = 0; j < k; ++j) in_new[topk_idx[j]] = 1;
  for (int j = 0; j < k; ++j) {
    hit_mask[j] = (uint8_t)(valid && in_old[topk_idx[j]]);
    if (!hit_mask[j]) toks[nt++] = topk_idx[j];
  }
  for (int j = 0; j < k; ++j)
    if (!valid || !in_new[slot_idx[j]]) slots[ns++] = j;
  if (ns != nt) { rc = -4; goto done; }
  for (int i = 0; i < ns; ++i) {
    slot_idx[slots[i]] = toks[i];
    if (miss_slot) miss_slot[i] = slots[i];
    if (miss_tok) miss_tok[i] = toks[i];
  }
  rc = ns;
done:
  free(in_old); free(in_new); free(slots); free(toks);
  return rc;
}

/* ---- hybrid attention: cached rows plus the append-only buffer (Section 6.2) ---- */

/* softmax over the k cached rows followed by the n_app appended rows; w_out (optional) has k + n_app entries. */
void qo_attention_hybrid(const uint16_t *q, const uint16_t *Kc, const uint16_t *Vc, int k, const uint16_t *Ka,
                         const uint16_t *Va, int n_app, int D, int dtype, double *out, double *w_out) {
  if (n_app == 0) {
    qo_attention(q, Kc, Vc, k, D, dtype, out, w_out);
    return;
  }
  const size_t rows = (size_t)k + (size_t)n_app;
  uint16_t *Kall = (uint16_t *)malloc(sizeof(uint16_t) * rows * D);
  uint16_t *Vall = (uint16_t *)malloc(sizeof(uint16_t) * rows * D);
  memcpy(Kall, Kc, sizeof(uint16_t) * (size_t)k * D);
  memcpy(Vall, Vc, sizeof(uint16_t) * (size_t)k * D);
  memcpy(Kall + (size_t)k * D, Ka, sizeof(uint16_t) * (size_t)n_app * D);
  memcpy(Vall + (size_t)k * D, Va, sizeof(uint16_t) * (size_t)n_app * D);
  qo_attention(q, Kall, Vall, (int)rows, D, dtype, out, w_out);
  free(Kall);
  free(Vall);
}

/* Sink / recent tokens and the append-only buffer of a step (all zero / NULL = plain Algorithm 1). */
typedef struct {
  int32_t n_sink, n_recent; /* forced members of every retrieved set: tokens [0, n_sink) and [N - n_recent, N) */
  int32_t n_app, app_cap;   /* valid rows and row stride of the append-only buffer                             */
  const uint16_t *K_app;    /* [P, app_cap, D]                                                                 */
  const uint16_t *V_app;
} qo_ext;

/* ---- one QSAC step (Algorithm 1, one iteration of the loop over t) ------ */

typedef struct {
  int32_t B, Hq, Hkv, D;
  int64_t N;
  int32_t k;     /* slots in use per KV head */
  int32_t k_max; /* slot stride of K_slots / V_slots / slot_idx */
  int32_t dtype;
} qo_dims;

/*
 * State (in/out): valid[P], prev_q[B,Hq,D], slot_idx[P,k_max],
 * K_slots/V_slots[P,k_max,D].   Inputs: q[B,Hq,D], K[P,N,D] (scored),
 * K_src/V_src[P,N,D] (rows copied into the slots), tau[Hkv], importance[Hq]
 * or NULL.  Outputs: out[B,Hq,D], topk_idx[P,k], hit_mask[P,k],
 * reuse_flags[P], sim[B,Hq], s_agg[P]; optional (NULL ok): kth_score[P]
 * (score of the last admitted key, NaN on reuse), scores[P,N] (NaN on reuse),
 * weights[B,Hq,k+n_app], n_filled[P].  ext (NULL ok): sink / recent tokens and the append-only buffer.  pair_mask[P] (NULL = all) restricts the work
 * to the marked pairs; unmarked pairs are left untouched everywhere.
 * P = B*Hkv, pair p = b*Hkv + h; query head g of pair p is b*Hq + h*G + g.
 */
int qo_step(const qo_dims *dm, const uint16_t *q, const uint16_t *K,
            const uint16_t *K_src, const uint16_t *V_src, uint8_t *valid,
            uint16_t *prev_q, int32_t *slot_idx, uint16_t *K_slots,
            uint16_t *V_slots, const double *tau, const double *importance,
            double *out, int32_t *topk_idx, uint8_t *hit_mask,
            uint8_t *reuse_flags, double *sim, double *s_agg, double *kth_score,
            double *scores, double *weights, int32_t *n_filled,
            const uint8_t *pair_mask, const qo_ext *ext) {
  const int n_sink = ext ? ext->n_sink : 0, n_recent = ext ? ext->n_recent : 0;
  const int n_app = ext ? ext->n_app : 0;
  const int G = dm->Hq / dm->Hkv, D = dm->D, k = dm->k;
  const int64_t N = dm->N;
  const int P = dm->B * dm->Hkv;
  int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int p = 0; p < P; ++p) {
    if (pair_mask && !pair_mask[p]) continue;
    const int b = p / dm->Hkv, h = p % dm->Hkv;
    const size_t qoff = ((size_t)b * dm->Hq + (size_t)h * G) * D;
    const uint16_t *qg = q + qoff;
    uint16_t *qc = prev_q + qoff;
    int32_t *sl = slot_idx + (size_t)p * dm->k_max;
    uint16_t *Ks = K_slots + (size_t)p * dm->k_max * D;
    uint16_t *Vs = V_slots + (size_t)p * dm->k_max * D;
    int32_t *tk = topk_idx + (size_t)p * k;
    uint8_t *hm = hit_mask + (size_t)p * k;

    /* cache lookup: per-query-head CosSim, then Eq. (2) */
    double sg[64];
    for (int g = 0; g < G; ++g) {
      sg[g] = qo_cossim(qg + (size_t)g * D, qc + (size_t)g * D, D, dm->dtype);
      sim[(size_t)b * dm->Hq + (size_t)h * G + g] = sg[g];
    }
    double s = qo_aggregate(sg, importance ? importance + (size_t)h * G : NULL, G);
    s_agg[p] = s;
    int reuse = valid[p] && (s >= tau[h]);
    reuse_flags[p] = (uint8_t)reuse;

    if (reuse) {
      /* cache hit: the cached set is used as it stands */
      memcpy(tk, sl, sizeof(int32_t) * (size_t)k);
      qsort(tk, (size_t)k, sizeof(int32_t), int_cmp);
      for (int j = 0; j < k; ++j) hm[j] = 1;
      if (kth_score) kth_score[p] = NAN;
      if (scores) for (int64_t n = 0; n < N; ++n) scores[(size_t)p * N + n] = NAN;
      if (n_filled) n_filled[p] = 0;
    } else {
      /* cache miss: retrieve, gather, replace, relabel */
      double *S = scores ? scores + (size_t)p * N : (double *)malloc(sizeof(double) * (size_t)N);
      qo_scores(qg, K + (size_t)p * N * D, G, N, D, dm->dtype, S);
      for (int64_t n = 0; n < N; ++n)
        if (n < n_sink || n >= N - n_recent) S[n] = INFINITY; /* sink and recent tokens always belong */
      double kth = NAN;
      int rc = qo_topk(S, N, k, tk, &kth);
      if (kth_score) kth_score[p] = kth;
      if (!scores) free(S);
      int32_t *ms = (int32_t *)malloc(sizeof(int32_t) * (size_t)k);
      int32_t *mt = (int32_t *)malloc(sizeof(int32_t) * (size_t)k);
      int m = rc ? rc : qo_diff(valid[p], N, k, sl, tk, hm, ms, mt);
      if (m < 0) {
#pragma omp atomic write
        err = m;
        m = 0;
      }
      for (int i = 0; i < m; ++i) {
        memcpy(Ks + (size_t)ms[i] * D, K_src + ((size_t)p * N + mt[i]) * D, sizeof(uint16_t) * D);
        memcpy(Vs + (size_t)ms[i] * D, V_src + ((size_t)p * N + mt[i]) * D, sizeof(uint16_t) * D);
      }
      free(ms); free(mt);
      if (n_filled) n_filled[p] = m;
      memcpy(qc, qg, sizeof(uint16_t) * (size_t)G * D);
      valid[p] = 1;
    }

    /* attention over the cached rows, one query head at a time */
    for (int g = 0; g < G; ++g) {
      size_t hq = (size_t)b * dm->Hq + (size_t)h * G + g;
      qo_attention_hybrid(qg + (size_t)g * D, Ks, Vs, k,
                          n_app ? ext->K_app + (size_t)p * ext->app_cap * D : NULL,
                          n_app ? ext->V_app + (size_t)p * ext->app_cap * D : NULL, n_app, D, dm->dtype,
                          out + hq * D, weights ? weights + hq * ((size_t)k + n_app) : NULL);
    }
  }
  return err;
}

int qo_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void qo_set_num_threads(int n) {
#ifdef _OPENMP
  omp_set_num_threads(n);
#else
  (void)n;
#endif
}
