/*
 * ckv_oracle.c -- plain CPU oracle of CompilerKV's prefill-end retention step.
 *
 * TEST INFRASTRUCTURE ONLY. This file is the parity reference for the HIP library: it is called by
 * the tests, by the smoke check and by the benchmark's CPU-baseline leg, never by the product path.
 * It shares no code, header, table or helper with the HIP sources.
 *
 * Every function takes dense row-major arrays, widens inputs to double and does every sum in double.
 * The steps follow the paper's order (Alg. 1) and notation: T prompt length (window included),
 * W = |Omega| observation window, P = T - W, Hq / Hkv query / key-value heads, G = Hq / Hkv.
 * Nothing is blocked, fused or reordered; OpenMP only spreads independent (batch, head) units over
 * cores.
 *
 * What each function is pinned by (tests/test_oracle_*.py): see the comment above it. The budget
 * split (ckv_oracle_budgets) and the 1-D pooling are this build's workload definitions, absent from
 * the paper: "parity unpinned" by the paper itself, pinned by brute force and library routines.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------------------------------
 * Observation-window attention mass per query head (paper Sec. 3 attention definition; Eq. 4's
 * alpha_t before the layer/head mean; Alg. 1 step (A)).
 *
 * q [Bz,Hq,W,d], k [Bz,Hkv,T,d] (float, already exact images of the stored dtype).
 * Window row j sits at absolute position P + j and attends causally to keys t <= P + j.
 *   z[j,t]   = scale * <q_j, k_t>
 *   LSE_j    = log sum_{t <= P+j} exp z[j,t]
 *   A[j,t]   = exp(z[j,t] - LSE_j)   (0 for masked t)
 *   scores[t] = (T / W) * sum_j A[j,t]
 * scores [Bz,Hq,T] double; lse_out [Bz,Hq,W] double or NULL.
 * Pins: sum_t scores = T (Eq. 4's remark); constant keys => closed form harmonic sums;
 * W = 1 => T * softmax (library routine); fp64 library softmax on small cases.
 * ---------------------------------------------------------------------------------------------- */
int ckv_oracle_window_scores(int Bz, int Hq, int Hkv, int d, int T, int W, double scale,
                             const float *q, const float *k, double *scores, double *lse_out) {
  if (Bz < 1 || Hq < 1 || Hkv < 1 || Hq % Hkv || d < 1 || W < 1 || W > T) return 1;
  const int G = Hq / Hkv, P = T - W;
  int failed = 0;
#pragma omp parallel for collapse(2) schedule(dynamic)
  for (int b = 0; b < Bz; ++b) {
    for (int h = 0; h < Hq; ++h) {
      const int g = h / G;
      const float *kh = k + ((size_t)b * Hkv + g) * (size_t)T * d;
      const float *qh = q + ((size_t)b * Hq + h) * (size_t)W * d;
      double *s = scores + ((size_t)b * Hq + h) * (size_t)T;
      double *z = (double *)malloc((size_t)T * sizeof(double));
      if (!z) {
        failed = 1;
        continue;
      }
      for (int t = 0; t < T; ++t) s[t] = 0.0;
      for (int j = 0; j < W; ++j) {
        const int last = P + j; /* last visible key */
        double m = -INFINITY;
        for (int t = 0; t <= last; ++t) {
          double acc = 0.0;
          for (int c = 0; c < d; ++c) acc += (double)qh[(size_t)j * d + c] * (double)kh[(size_t)t * d + c];
          z[t] = scale * acc;
          if (z[t] > m) m = z[t];
        }
        double denom = 0.0;
        for (int t = 0; t <= last; ++t) denom += exp(z[t] - m);
        const double lse = m + log(denom);
        if (lse_out) lse_out[((size_t)b * Hq + h) * W + j] = lse;
        for (int t = 0; t <= last; ++t) s[t] += exp(z[t] - lse);
      }
      const double norm = (double)T / (double)W;
      for (int t = 0; t < T; ++t) s[t] *= norm;
      free(z);
    }
  }
  return failed ? 2 : 0;
}

/* ------------------------------------------------------------------------------------------------
 * Value-norm ratio (paper Eq. 4's rho; Alg. 1 Stage 1): r_t = ||v_t||_2, mu = mean_{t<T} r_t,
 * rho_t = r_t / (mu + eps).  v [Bz,Hkv,T,d] float -> rho [Bz,Hkv,T] double.
 * Pins: unit-norm rows => 1/(1+eps); invariance under v -> c*v up to eps; mean(rho) = mu/(mu+eps).
 * ---------------------------------------------------------------------------------------------- */
int ckv_oracle_value_norm_ratio(int Bz, int Hkv, int T, int d, double eps, const float *v,
                                double *rho) {
  if (Bz < 1 || Hkv < 1 || T < 1 || d < 1) return 1;
  for (int u = 0; u < Bz * Hkv; ++u) {
    const float *vu = v + (size_t)u * T * d;
    double *ru = rho + (size_t)u * T;
    double total = 0.0;
    for (int t = 0; t < T; ++t) {
      double sq = 0.0;
      for (int c = 0; c < d; ++c) sq += (double)vu[(size_t)t * d + c] * (double)vu[(size_t)t * d + c];
      ru[t] = sqrt(sq);
      total += ru[t];
    }
    const double mu = total / (double)T;
    for (int t = 0; t < T; ++t) ru[t] = ru[t] / (mu + eps);
  }
  return 0;
}

/* ------------------------------------------------------------------------------------------------
 * 1-D pooling of one row along the token axis (workload definition; the paper only says its scan is
 * that of window-based prefill compressors). Centred, stride 1, output length n.
 * mode 0: copy. mode 1 (avg): sum over |delta| <= kernel/2 of in-range entries, divided by kernel
 * (zeros outside). mode 2 (max): maximum over in-range entries.
 * Pins: library avg/max pooling with the same padding convention; hand cases at both edges.
 * ---------------------------------------------------------------------------------------------- */
static void pool_row(const double *x, int n, int mode, int kernel, double *y) {
  const int r = kernel / 2;
  for (int t = 0; t < n; ++t) {
    if (mode == 0) {
      y[t] = x[t];
    } else if (mode == 1) {
      double acc = 0.0;
      for (int dt = -r; dt <= r; ++dt)
        if (t + dt >= 0 && t + dt < n) acc += x[t + dt];
      y[t] = acc / (double)kernel;
    } else {
      double best = -INFINITY;
      for (int dt = -r; dt <= r; ++dt)
        if (t + dt >= 0 && t + dt < n && x[t + dt] > best) best = x[t + dt];
      y[t] = best;
    }
  }
}

int ckv_oracle_pool(int rows, int n, int mode, int kernel, const double *x, double *y) {
  if (rows < 0 || n < 0 || mode < 0 || mode > 2 || (mode != 0 && (kernel < 1 || kernel % 2 == 0)))
    return 1;
  for (int r = 0; r < rows; ++r) pool_row(x + (size_t)r * n, n, mode, kernel, y + (size_t)r * n);
  return 0;
}

/* ------------------------------------------------------------------------------------------------
 * Pooled mass -> utility per KV head (paper Eq. 4 u = alpha * rho; Eq. 6 weighted max over heads,
 * here over the query heads that share one KV head; Alg. 1 Stages 1-2).
 *   c[h,t] = pool(scores[b,h,0:P])[t];  u[h,t] = c[h,t] * rho[b,g,t] (rho NULL => 1)
 *   utility[b,g,t] = fp32( max_{h in g} w_head_row[h] * u[h,t] )
 * scores [Bz,Hq,T] double, rho [Bz,Hkv,T] double or NULL, w_head_row [Hq] float (the layer's row),
 * utility [Bz,Hkv,P] float (the ABI stores fp32, and selection decides on those fp32 values).
 * Pins: all weights 1 and G = 1 => pooled scores; one huge weight => that head decides every max.
 * ---------------------------------------------------------------------------------------------- */
int ckv_oracle_utility(int Bz, int Hq, int Hkv, int T, int W, int mode, int kernel,
                       const double *scores, const double *rho, const float *w_head_row,
                       float *utility) {
  if (Bz < 1 || Hq < 1 || Hkv < 1 || Hq % Hkv || W < 1 || W > T) return 1;
  if (mode < 0 || mode > 2 || (mode != 0 && (kernel < 1 || kernel % 2 == 0))) return 1;
  const int G = Hq / Hkv, P = T - W;
  if (P == 0) return 0;
  double *c = (double *)malloc((size_t)P * sizeof(double));
  double *best = (double *)malloc((size_t)P * sizeof(double));
  if (!c || !best) {
    free(c);
    free(best);
    return 2;
  }
  for (int b = 0; b < Bz; ++b) {
    for (int g = 0; g < Hkv; ++g) {
      for (int t = 0; t < P; ++t) best[t] = -INFINITY;
      for (int h = g * G; h < (g + 1) * G; ++h) {
        pool_row(scores + ((size_t)b * Hq + h) * T, P, mode, kernel, c);
        for (int t = 0; t < P; ++t) {
          double u = c[t];
          if (rho) u *= rho[((size_t)b * Hkv + g) * T + t];
          const double weighted = (double)w_head_row[h] * u;
          if (weighted > best[t]) best[t] = weighted;
        }
      }
      float *out = utility + ((size_t)b * Hkv + g) * P;
      for (int t = 0; t < P; ++t) out[t] = (float)best[t];
    }
  }
  free(c);
  free(best);
  return 0;
}

/* ------------------------------------------------------------------------------------------------
 * Per-KV-head budgets of one layer (workload definition; the paper has one B_l per layer).
 * share [Hkv] float or NULL. B = nominal budget per head (window included), B_tot = B * Hkv.
 *   NULL: b_g = B.  Else b_g = floor(share[g] * B_tot) in double, clamped to [W, T]; while the sum
 *   exceeds B_tot, the largest b_g that is > W (lowest g on ties) loses one.
 * Pins: sum <= B_tot, W <= b_g <= T, uniform shares => all B; brute-force re-derivation.
 * ---------------------------------------------------------------------------------------------- */
int ckv_oracle_budgets(int Hkv, int T, int W, int B, const float *share, int32_t *budget) {
  if (Hkv < 1 || W < 1 || W > T || B < W) return 1;
  const int64_t B_tot = (int64_t)B * Hkv;
  if (!share) {
    for (int g = 0; g < Hkv; ++g) budget[g] = B < T ? B : T;
    return 0;
  }
  int64_t total = 0;
  for (int g = 0; g < Hkv; ++g) {
    double want = floor((double)share[g] * (double)B_tot);
    if (!(want >= (double)W)) want = (double)W; /* also catches NaN */
    if (want > (double)T) want = (double)T;
    budget[g] = (int32_t)want;
    total += budget[g];
  }
  while (total > B_tot) {
    int arg = -1;
    for (int g = 0; g < Hkv; ++g)
      if (budget[g] > W && (arg < 0 || budget[g] > budget[arg])) arg = g;
    if (arg < 0) break; /* every head is at its floor W; cannot happen while B >= W */
    budget[arg] -= 1;
    total -= 1;
  }
  return 0;
}

/* ------------------------------------------------------------------------------------------------
 * Risk-gate lookup (paper Sec. 4.3, Alg. 1 Stage 3 first line): tau = T_gate[layer, b_ent, b_ppl],
 * with the budget coordinate already resolved by the caller. gate_layer [n_ent,n_ppl] float is the
 * layer's slice; NULL => gate off => 0. Bins are clamped into the table.
 * ---------------------------------------------------------------------------------------------- */
float ckv_oracle_tau(const float *gate_layer, int n_ent, int n_ppl, int b_ent, int b_ppl) {
  if (!gate_layer) return 0.0f;
  if (b_ent < 0) b_ent = 0;
  if (b_ent >= n_ent) b_ent = n_ent - 1;
  if (b_ppl < 0) b_ppl = 0;
  if (b_ppl >= n_ppl) b_ppl = n_ppl - 1;
  return gate_layer[(size_t)b_ent * n_ppl + b_ppl];
}

/* ------------------------------------------------------------------------------------------------
 * Elastic candidate pool with budget clamp (paper Eq. 8; Alg. 1 Select) for one (batch, KV head):
 *   cand = { t < P : u[t] >= tau };  kp = budget - W
 *   |cand| <= kp : keep cand;  else keep the kp first of cand under (u descending, t ascending)
 *   idx = kept in ascending t, then P..T-1;  returns count = |kept| + W.
 * The sort is a full sort of the candidate pool ("a single sort over the candidate pool").
 * Pins: brute force over all subsets on tiny inputs; tau = 0 => library top-k; tau above the
 * maximum => window only; count = min(budget, W + |cand|).
 * ---------------------------------------------------------------------------------------------- */
typedef struct {
  float u;
  int32_t t;
} cand_t;

static int by_utility_then_position(const void *pa, const void *pb) {
  const cand_t *a = (const cand_t *)pa, *b = (const cand_t *)pb;
  if (a->u > b->u) return -1;
  if (a->u < b->u) return 1;
  return (a->t > b->t) - (a->t < b->t);
}

static int by_position(const void *pa, const void *pb) {
  const cand_t *a = (const cand_t *)pa, *b = (const cand_t *)pb;
  return (a->t > b->t) - (a->t < b->t);
}

int ckv_oracle_select_one(int T, int W, const float *u, float tau, int budget, int32_t *idx) {
  const int P = T - W;
  int kp = budget - W;
  if (kp < 0) kp = 0;
  cand_t *cand = (cand_t *)malloc((size_t)(P > 0 ? P : 1) * sizeof(cand_t));
  if (!cand) return -1;
  int n = 0;
  for (int t = 0; t < P; ++t)
    if (u[t] >= tau) {
      cand[n].u = u[t];
      cand[n].t = t;
      ++n;
    }
  int kept = n;
  if (n > kp) {
    qsort(cand, (size_t)n, sizeof(cand_t), by_utility_then_position);
    kept = kp;
    qsort(cand, (size_t)kept, sizeof(cand_t), by_position);
  }
  for (int r = 0; r < kept; ++r) idx[r] = cand[r].t;
  for (int j = 0; j < W; ++j) idx[kept + j] = P + j;
  free(cand);
  return kept + W;
}

/* All (batch, KV head) units: utility [Bz,Hkv,P], tau [Bz], budget [Bz,Hkv] -> idx [Bz,Hkv,cap],
 * count [Bz,Hkv]. Entries of idx beyond count are left untouched. */
int ckv_oracle_select(int Bz, int Hkv, int T, int W, int cap, const float *utility, const float *tau,
                      const int32_t *budget, int32_t *idx, int32_t *count) {
  if (Bz < 1 || Hkv < 1 || W < 1 || W > T || cap < W) return 1;
  const int P = T - W;
  int failed = 0;
#pragma omp parallel for schedule(dynamic)
  for (int u = 0; u < Bz * Hkv; ++u) {
    int bud = budget[u];
    if (bud < W) bud = W;
    if (bud > cap) bud = cap;
    if (bud > T) bud = T;
    const int c = ckv_oracle_select_one(T, W, utility + (size_t)u * P, tau[u / Hkv], bud,
                                        idx + (size_t)u * cap);
    if (c < 0) failed = 1;
    count[u] = c;
  }
  return failed ? 2 : 0;
}

/* ------------------------------------------------------------------------------------------------
 * Token-axis gather (paper Sec. 3: K~ = K[S], V~ = V[S]; Alg. 1 Gather_tok): byte copies of rows.
 * src [units,T,row_bytes], idx [units,cap], count [units] -> dst [units,cap,row_bytes]; rows at and
 * beyond count are left untouched.
 * Pins: library index-select; identity index list => plain copy.
 * ---------------------------------------------------------------------------------------------- */
int ckv_oracle_gather(int units, int T, int cap, size_t row_bytes, const unsigned char *src,
                      const int32_t *idx, const int32_t *count, unsigned char *dst) {
  if (units < 0 || T < 1 || cap < 0) return 1;
  for (int u = 0; u < units; ++u)
    for (int r = 0; r < count[u] && r < cap; ++r) {
      const int32_t t = idx[(size_t)u * cap + r];
      if (t < 0 || t >= T) return 3;
      memcpy(dst + ((size_t)u * cap + r) * row_bytes, src + ((size_t)u * T + t) * row_bytes, row_bytes);
    }
  return 0;
}

/* Number of OpenMP threads the parallel loops above will use (1 when built without OpenMP). */
#ifdef _OPENMP
#include <omp.h>
int ckv_oracle_threads(void) { return omp_get_max_threads(); }
#else
int ckv_oracle_threads(void) { return 1; }
#endif
