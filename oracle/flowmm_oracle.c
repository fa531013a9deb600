/*
 * FlowMM prefill-time KV-cache merge: plain CPU oracle, fp64.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call this file;
 * it exists so that tests, the smoke check and the benchmark's cpu_baseline leg
 * have an independent statement of what the method computes.  It shares no code
 * with the HIP path.  Inputs arrive as float (values already rounded to the
 * cache dtype); all arithmetic is double.  No blocking, fusion or reordering
 * beyond what the paper's equations state; OpenMP only across independent heads.
 *
 * Stages (one sequence, one layer per call):
 *   fmo_score  - attention of the proxy (observation-window) queries over the
 *                cached keys, eq. for o_t in Preliminary (softmax(q K^T / sqrt d));
 *                proxy importance I(i) = sum over proxies of alpha_{j->i}
 *                (Information Flow Guided Merging, importance equation), here
 *                normalised by the number of proxy rows so that sum_i I(i) = 1;
 *                per-head cross-modal attention share (the ratio inside the
 *                rho^l equation: mass sent to the other modality / total mass).
 *   fmo_flow   - rho^l = mean over heads; cross-modal merging iff rho^l > theta.
 *   fmo_select - top-B by importance = pivot set (same section); proxy tokens
 *                themselves are always pivots.
 *   fmo_match  - cosine similarity between non-pivot and pivot keys and the
 *                argmax over pivots whose importance does not exceed tau
 *                (Sensitivity-Adaptive Token Matching, both equations), restricted
 *                to the token's own modality when the layer is intra-modal.
 *   fmo_merge  - fold every matched non-pivot K/V row into its pivot by a
 *                uniform mean (the paper leaves f_merge/g_merge open; uniform
 *                weights are this build's reading).
 *
 * Variants of the paper's ablation study (Effectiveness of Each Component), same stages:
 *   fmo_flow with invert != 0 - the strategy misaligned with the measured flow
 *                (cross-modal merging exactly where the rule says intra-modal);
 *   fmo_merge_weighted        - f_merge/g_merge as a similarity-weighted mean: the pivot
 *                counts 1, a member counts max(u, 0) with u its cosine to the pivot.
 *   fmo_decode_attention      - one decode step of attention (the attention-output equation of
 *                the Preliminary section, o_t = softmax(q_t K^T / sqrt d) V) over a compacted cache:
 *                what the paper's decoding-latency table exercises on the compressed cache.
 *   fmo_cache_append          - the cache-append equation of the Preliminary section,
 *                K_t = [K_{t-1}, k_t], V_t = [V_{t-1}, v_t], on a cache with head room per sequence.
 *   fmo_cache_remerge         - this build's reading of what the paper leaves open (what to do when
 *                the compressed cache has outgrown its budget during decoding): the stages above run
 *                again on the valid rows of the cache as if they were a prompt of one modality, the
 *                last W rows being the proxies; the merged rows replace the head of the cache.
 *   ("Without sensitivity-adaptive matching" is tau = +inf; "without information flow
 *   guidance" is a theta below 0 or above 1; neither needs code of its own.)
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int fmo_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* K [Hkv][L][d], Q [Hq][W][d] (row r of the window is token L-W+r), mod [L].
 * I [Hkv][L], cross [Hq]. */
void fmo_score(int Hq, int Hkv, int L, int W, int d, double scale, const float *K, const float *Q,
               const int32_t *mod, double *I, double *cross) {
  const int G = Hq / Hkv;
#pragma omp parallel for schedule(dynamic, 1)
  for (int g = 0; g < Hkv; ++g) {
    double *Ig = I + (size_t)g * L;
    double *alpha = (double *)malloc(sizeof(double) * (size_t)L);
    for (int i = 0; i < L; ++i) Ig[i] = 0.0;
    for (int hh = 0; hh < G; ++hh) {
      const int h = g * G + hh;
      double cr = 0.0;
      for (int r = 0; r < W; ++r) {
        const int pos = L - W + r; /* causal: the query at pos sees keys 0..pos */
        const float *q = Q + ((size_t)h * W + r) * d;
        double mx = -INFINITY;
        for (int i = 0; i <= pos; ++i) {
          const float *k = K + ((size_t)g * L + i) * d;
          double s = 0.0;
          for (int c = 0; c < d; ++c) s += (double)q[c] * (double)k[c];
          s *= scale;
          alpha[i] = s;
          if (s > mx) mx = s;
        }
        double z = 0.0;
        for (int i = 0; i <= pos; ++i) {
          alpha[i] = exp(alpha[i] - mx);
          z += alpha[i];
        }
        for (int i = 0; i <= pos; ++i) {
          const double a = alpha[i] / z;
          Ig[i] += a;
          if (mod[i] != mod[pos]) cr += a;
        }
      }
      cross[h] = cr / (double)W;
    }
    for (int i = 0; i < L; ++i) Ig[i] /= (double)(G * W);
    free(alpha);
  }
}

/* rho = mean of the per-head shares; returns 1 (cross-modal) iff rho > theta.
 * invert != 0 gives the misaligned strategy: 1 iff NOT rho > theta. */
int fmo_flow(int Hq, const double *cross, double theta, int invert, double *rho) {
  double s = 0.0;
  for (int h = 0; h < Hq; ++h) s += cross[h];
  *rho = s / (double)Hq;
  const int cross_modal = (*rho > theta) ? 1 : 0;
  return invert ? 1 - cross_modal : cross_modal;
}

/* One KV head.  The last W positions are forced pivots; the remaining B-W pivots
 * are the largest I, ties to the smaller index.  kept_idx ascending. */
void fmo_select(int L, int W, int B, const double *I, int32_t *kept_idx) {
  char *chosen = (char *)calloc((size_t)L, 1);
  int n = 0;
  for (int i = L - W; i < L; ++i) {
    chosen[i] = 1;
    ++n;
  }
  while (n < B) {
    int best = -1;
    for (int i = 0; i < L - W; ++i) {
      if (chosen[i]) continue;
      if (best < 0 || I[i] > I[best]) best = i;
    }
    chosen[best] = 1;
    ++n;
  }
  int s = 0;
  for (int i = 0; i < L; ++i)
    if (chosen[i]) kept_idx[s++] = i;
  free(chosen);
}

/* One KV head.  K [L][d], I [L], kept_idx [B] ascending, mod [L].
 * assign [L]: pivots get their own slot, others the matched slot or -1.
 * u_best/u_second [L] (optional, may be NULL): best and runner-up cosine among
 * eligible pivots (-inf when absent), for margin-aware comparisons.
 * Returns the number of non-pivot tokens with no eligible pivot. */
int fmo_match(int L, int d, int B, const float *K, const double *I, const int32_t *kept_idx,
              const int32_t *mod, int mode_cross, double tau, int32_t *assign, double *u_best,
              double *u_second) {
  double *norm = (double *)malloc(sizeof(double) * (size_t)L);
  for (int i = 0; i < L; ++i) {
    double s = 0.0;
    for (int c = 0; c < d; ++c) s += (double)K[(size_t)i * d + c] * (double)K[(size_t)i * d + c];
    norm[i] = sqrt(s);
    assign[i] = -2;
  }
  for (int s = 0; s < B; ++s) assign[kept_idx[s]] = s;
  int dropped = 0;
  for (int i = 0; i < L; ++i) {
    if (assign[i] >= 0) {
      if (u_best) u_best[i] = -INFINITY;
      if (u_second) u_second[i] = -INFINITY;
      continue;
    }
    int best = -1;
    double ub = -INFINITY, us = -INFINITY;
    for (int s = 0; s < B; ++s) {
      const int j = kept_idx[s];
      if (I[j] > tau) continue;                       /* highly sensitive pivot: never a target */
      if (!mode_cross && mod[j] != mod[i]) continue;  /* intra-modal layer */
      double u = 0.0;
      if (norm[i] > 0.0 && norm[j] > 0.0) {
        double dot = 0.0;
        for (int c = 0; c < d; ++c) dot += (double)K[(size_t)i * d + c] * (double)K[(size_t)j * d + c];
        u = dot / (norm[i] * norm[j]);
      }
      if (u > ub) {
        us = ub;
        ub = u;
        best = s;
      } else if (u > us) {
        us = u;
      }
    }
    assign[i] = best;
    if (best < 0) ++dropped;
    if (u_best) u_best[i] = ub;
    if (u_second) u_second[i] = us;
  }
  free(norm);
  return dropped;
}

/* One KV head.  Kout, Vout [B][d] in double (unrounded); n_members [B]. */
void fmo_merge(int L, int d, int B, const float *K, const float *V, const int32_t *kept_idx,
               const int32_t *assign, double *Kout, double *Vout, int32_t *n_members) {
  for (int s = 0; s < B; ++s) {
    n_members[s] = 0;
    for (int c = 0; c < d; ++c) {
      Kout[(size_t)s * d + c] = (double)K[(size_t)kept_idx[s] * d + c];
      Vout[(size_t)s * d + c] = (double)V[(size_t)kept_idx[s] * d + c];
    }
  }
  for (int i = 0; i < L; ++i) {
    const int s = assign[i];
    if (s < 0 || kept_idx[s] == i) continue;
    n_members[s] += 1;
    for (int c = 0; c < d; ++c) {
      Kout[(size_t)s * d + c] += (double)K[(size_t)i * d + c];
      Vout[(size_t)s * d + c] += (double)V[(size_t)i * d + c];
    }
  }
  for (int s = 0; s < B; ++s) {
    const double w = 1.0 / (double)(1 + n_members[s]);
    for (int c = 0; c < d; ++c) {
      Kout[(size_t)s * d + c] *= w;
      Vout[(size_t)s * d + c] *= w;
    }
  }
}

/* Similarity-weighted variant of fmo_merge:
 *   out[s] = (row[pivot] + sum_i w_i row[i]) / (1 + sum_i w_i),  w_i = max(u_i, 0),
 * u_i the cosine between member key i and the pivot key (0 if either is a zero row); V rows take
 * the weights of their K rows.  wsum [B] receives 1 + sum_i w_i. */
void fmo_merge_weighted(int L, int d, int B, const float *K, const float *V, const int32_t *kept_idx,
                        const int32_t *assign, double *Kout, double *Vout, int32_t *n_members, double *wsum) {
  for (int s = 0; s < B; ++s) {
    n_members[s] = 0;
    wsum[s] = 1.0;
    for (int c = 0; c < d; ++c) {
      Kout[(size_t)s * d + c] = (double)K[(size_t)kept_idx[s] * d + c];
      Vout[(size_t)s * d + c] = (double)V[(size_t)kept_idx[s] * d + c];
    }
  }
  for (int i = 0; i < L; ++i) {
    const int s = assign[i];
    if (s < 0 || kept_idx[s] == i) continue;
    const float *ki = K + (size_t)i * d, *kj = K + (size_t)kept_idx[s] * d;
    double dot = 0.0, ni = 0.0, nj = 0.0;
    for (int c = 0; c < d; ++c) {
      dot += (double)ki[c] * (double)kj[c];
      ni += (double)ki[c] * (double)ki[c];
      nj += (double)kj[c] * (double)kj[c];
    }
    double w = (ni > 0.0 && nj > 0.0) ? dot / (sqrt(ni) * sqrt(nj)) : 0.0;
    if (w < 0.0) w = 0.0;
    n_members[s] += 1;
    wsum[s] += w;
    for (int c = 0; c < d; ++c) {
      Kout[(size_t)s * d + c] += w * (double)K[(size_t)i * d + c];
      Vout[(size_t)s * d + c] += w * (double)V[(size_t)i * d + c];
    }
  }
  for (int s = 0; s < B; ++s) {
    for (int c = 0; c < d; ++c) {
      Kout[(size_t)s * d + c] /= wsum[s];
      Vout[(size_t)s * d + c] /= wsum[s];
    }
  }
}

/* One KV head of one sequence: q [G][d] (the G query heads that read this KV head), Kc, Vc [B][d]
 * (the compacted cache).  out [G][d] = softmax_s(scale * <q_g, Kc_s>) Vc, in double. */
void fmo_decode_attention(int G, int B, int d, double scale, const float *q, const float *Kc, const float *Vc,
                          double *out) {
  double *p = (double *)malloc(sizeof(double) * (size_t)B);
  for (int g = 0; g < G; ++g) {
    double mx = -INFINITY;
    for (int s = 0; s < B; ++s) {
      double dot = 0.0;
      for (int c = 0; c < d; ++c) dot += (double)q[(size_t)g * d + c] * (double)Kc[(size_t)s * d + c];
      p[s] = scale * dot;
      if (p[s] > mx) mx = p[s];
    }
    double z = 0.0;
    for (int s = 0; s < B; ++s) {
      p[s] = exp(p[s] - mx);
      z += p[s];
    }
    for (int c = 0; c < d; ++c) {
      double acc = 0.0;
      for (int s = 0; s < B; ++s) acc += p[s] * (double)Vc[(size_t)s * d + c];
      out[(size_t)g * d + c] = acc / z;
    }
  }
  free(p);
}

/* Round-to-nearest-even of doubles to the output dtype (0 = fp32, 1 = bf16), result as float. */
void fmo_round(int64_t n, int dtype, const double *x, float *y) {
  for (int64_t i = 0; i < n; ++i) {
    if (dtype == 0 || x[i] == 0.0 || !isfinite(x[i])) {
      y[i] = (float)x[i];
      continue;
    }
    int e;
    double m = frexp(x[i], &e); /* x = m * 2^e, 0.5 <= |m| < 1 */
    if (e < -125) {             /* below the normal range of bf16: quantum is fixed at 2^-133 */
      y[i] = (float)ldexp(nearbyint(ldexp(x[i], 133)), -133);
    } else {
      y[i] = (float)ldexp(nearbyint(ldexp(m, 8)), e - 8); /* 8 significant bits */
    }
  }
}

/* Whole pass over one layer of one sequence, all heads (used for timing and end-to-end tests).
 * K, V [Hkv][L][d]; Q [Hq][W][d].  Outputs: I [Hkv][L], rho, mode, kept_idx [Hkv][B],
 * assign [Hkv][L], n_dropped [Hkv], Kout/Vout [Hkv][B][d] rounded to dtype. */
void fmo_layer(int Hq, int Hkv, int L, int W, int d, int B, int dtype, double scale, double theta,
               double tau, const float *K, const float *V, const float *Q, const int32_t *mod,
               double *I, double *rho, int32_t *mode, int32_t *kept_idx, int32_t *assign,
               int32_t *n_dropped, float *Kout, float *Vout) {
  double *cross = (double *)malloc(sizeof(double) * (size_t)Hq);
  fmo_score(Hq, Hkv, L, W, d, scale, K, Q, mod, I, cross);
  *mode = fmo_flow(Hq, cross, theta, 0, rho);
  free(cross);
  const int mode_cross = *mode;
#pragma omp parallel for schedule(dynamic, 1)
  for (int g = 0; g < Hkv; ++g) {
    const float *Kg = K + (size_t)g * L * d;
    const float *Vg = V + (size_t)g * L * d;
    int32_t *kept = kept_idx + (size_t)g * B;
    int32_t *asg = assign + (size_t)g * L;
    fmo_select(L, W, B, I + (size_t)g * L, kept);
    n_dropped[g] = fmo_match(L, d, B, Kg, I + (size_t)g * L, kept, mod, mode_cross, tau, asg, NULL, NULL);
    double *ko = (double *)malloc(sizeof(double) * (size_t)B * d);
    double *vo = (double *)malloc(sizeof(double) * (size_t)B * d);
    int32_t *nm = (int32_t *)malloc(sizeof(int32_t) * (size_t)B);
    fmo_merge(L, d, B, Kg, Vg, kept, asg, ko, vo, nm);
    fmo_round((int64_t)B * d, dtype, ko, Kout + (size_t)g * B * d);
    fmo_round((int64_t)B * d, dtype, vo, Vout + (size_t)g * B * d);
    free(ko);
    free(vo);
    free(nm);
  }
}

/* Cache-append equation (Preliminary): the new token's key and value become row `length` of every
 * kv head's cache.  Kc, Vc [Hkv][capacity][d]; k, v [Hkv][d].  Returns the new length, or -1 if full. */
int fmo_cache_append(int Hkv, int capacity, int d, int length, float *Kc, float *Vc, const float *k,
                     const float *v) {
  if (length < 0 || length >= capacity) return -1;
  for (int g = 0; g < Hkv; ++g)
    for (int c = 0; c < d; ++c) {
      Kc[((size_t)g * capacity + length) * d + c] = k[(size_t)g * d + c];
      Vc[((size_t)g * capacity + length) * d + c] = v[(size_t)g * d + c];
    }
  return length + 1;
}

/* Re-merge of one sequence's cache in one layer (reading of this build, the paper gives no policy):
 * the n valid rows are a prompt whose tokens all share one modality, the last W rows are the proxies
 * (Q [Hq][W][d] are their queries); score, flow, select, match and merge run as for a prompt, and the
 * B merged rows, rounded to the cache dtype, replace rows [0, B).  Rows from B on are left as they
 * were (stale).  Kc, Vc [Hkv][capacity][d].  Outputs as fmo_layer's, for n tokens.  Returns B. */
int fmo_cache_remerge(int Hq, int Hkv, int capacity, int n, int W, int d, int B, int dtype, double scale,
                      double tau, float *Kc, float *Vc, const float *Q, double *I, double *rho,
                      int32_t *mode, int32_t *kept_idx, int32_t *assign, int32_t *n_dropped) {
  float *K = (float *)malloc(sizeof(float) * (size_t)Hkv * n * d);
  float *V = (float *)malloc(sizeof(float) * (size_t)Hkv * n * d);
  float *Ko = (float *)malloc(sizeof(float) * (size_t)Hkv * B * d);
  float *Vo = (float *)malloc(sizeof(float) * (size_t)Hkv * B * d);
  int32_t *mod = (int32_t *)calloc((size_t)n, sizeof(int32_t)); /* one modality for every row */
  for (int g = 0; g < Hkv; ++g) {
    memcpy(K + (size_t)g * n * d, Kc + (size_t)g * capacity * d, sizeof(float) * (size_t)n * d);
    memcpy(V + (size_t)g * n * d, Vc + (size_t)g * capacity * d, sizeof(float) * (size_t)n * d);
  }
  /* with one modality rho is 0 and either strategy admits the same pivots; theta plays no part */
  fmo_layer(Hq, Hkv, n, W, d, B, dtype, scale, -1.0, tau, K, V, Q, mod, I, rho, mode, kept_idx, assign,
            n_dropped, Ko, Vo);
  for (int g = 0; g < Hkv; ++g) {
    memcpy(Kc + (size_t)g * capacity * d, Ko + (size_t)g * B * d, sizeof(float) * (size_t)B * d);
    memcpy(Vc + (size_t)g * capacity * d, Vo + (size_t)g * B * d, sizeof(float) * (size_t)B * d);
  }
  free(K); free(V); free(Ko); free(Vo); free(mod);
  return B;
}
