/*
 * toma_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain, slow, fp64 CPU statement of what one ToMA layer computes, written from the paper
 * (ToMA: Token Merge with Attention for Diffusion Models): local regions (Sec. 4.3.1, Alg. 3),
 * cosine similarity and the facility-location objective (Sec. 4.1, Eq. 2), the greedy selection
 * with the cached marginal gain (Alg. 1, Alg. 2, App. A.1), the attention-like merge weights and
 * the merge (Sec. 4.2.1), scaled dot-product attention on the merged tokens (Eq. 1), and the
 * transpose unmerge (Sec. 4.2.2).  Only tests, the smoke check and the benchmark's CPU-baseline
 * leg may call it.  It shares no code, header, table or helper with the GPU library.
 *
 * Every function works on dense row-major double arrays.  Loops are written in the order the
 * definitions state; OpenMP only distributes independent (sample, region) pairs or output rows.
 *
 * Readings of points the paper leaves open are stated where they are used; all of them are also
 * listed in the design notes of the repository.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_API __attribute__((visibility("default")))

/* Shape of one layer call.  N = H*W tokens on a row-major H x W grid; regions are tile_h x tile_w
 * windows (a stripe region is tile_h rows by W columns).  merge_regions is 1 (merge weights over
 * all tokens: the variant the paper calls ToMA) or P (weights inside each region: ToMA_tile,
 * Alg. 3).  sim_bits > 0 rounds every similarity S_ij to the nearest multiple of 2^-sim_bits
 * before the greedy decisions are taken: it names the precision in which the argmax is decided
 * (sums of such values are exact in double, so ties are exact ties). */
typedef struct {
  int32_t B, H, W, C;
  int32_t tile_h, tile_w;
  int32_t d_loc;
  int32_t merge_regions;
  double scale; /* logit multiplier of the merge weights, 1/tau in Sec. 4.2.1's display formula */
  int32_t sim_bits;
} oracle_desc;

static int n_regions(const oracle_desc *d) { return (d->H / d->tile_h) * (d->W / d->tile_w); }
static int n_loc(const oracle_desc *d) { return d->tile_h * d->tile_w; }

/* Sec. 4.3.1 "Tile-shaped Regions" / Alg. 3 "Split into local regions": token n = r*W + c lies in
 * region p = (r / tile_h) * (W / tile_w) + (c / tile_w) at local position
 * l = (r % tile_h) * tile_w + (c % tile_w).  token_of[p * N_loc + l] is the inverse map. */
ORACLE_API void toma_oracle_region_map(int H, int W, int tile_h, int tile_w, int32_t *region,
                                       int32_t *local, int32_t *token_of) {
  int pw = W / tile_w, nl = tile_h * tile_w;
  for (int r = 0; r < H; r++)
    for (int c = 0; c < W; c++) {
      int n = r * W + c;
      int p = (r / tile_h) * pw + (c / tile_w);
      int l = (r % tile_h) * tile_w + (c % tile_w);
      if (region) region[n] = p;
      if (local) local[n] = l;
      if (token_of) token_of[p * nl + l] = n;
    }
}

/* Sec. 4.1: S_ij = cos(x_i, x_j) for the n tokens whose rows are listed in rows[] (row stride C).
 * A zero vector gets norm eps = 1e-12 so that its similarities are 0 rather than NaN. */
ORACLE_API void toma_oracle_cosine(const double *X, const int32_t *rows, int n, int C,
                                   int round_bits, double *S) {
  double *nrm = (double *)malloc(sizeof(double) * (size_t)n);
  for (int i = 0; i < n; i++) {
    const double *xi = X + (size_t)rows[i] * C;
    double s = 0.0;
    for (int c = 0; c < C; c++) s += xi[c] * xi[c];
    s = sqrt(s);
    nrm[i] = s > 1e-12 ? s : 1e-12;
  }
  for (int i = 0; i < n; i++) {
    const double *xi = X + (size_t)rows[i] * C;
    for (int j = 0; j < n; j++) {
      const double *xj = X + (size_t)rows[j] * C;
      double s = 0.0;
      for (int c = 0; c < C; c++) s += xi[c] * xj[c];
      s = s / (nrm[i] * nrm[j]);
      S[(size_t)i * n + j] = round_bits > 0 ? ldexp(nearbyint(ldexp(s, round_bits)), -round_bits) : s;
    }
  }
  free(nrm);
}

/* Eq. 2 shifted so that the empty set has value 0: f'(D) = sum_i max_{j in D} (S_ij + 1),
 * f'({}) = 0.  The shift adds the same constant to every non-empty set, so greedy on f' takes
 * Alg. 2's steps (its first step, the largest row sum, is the largest f'({v}); S is symmetric). */
ORACLE_API double toma_oracle_fl_value(const double *S, int n, const int32_t *set, int size) {
  if (size <= 0) return 0.0;
  double f = 0.0;
  for (int i = 0; i < n; i++) {
    double best = -INFINITY;
    for (int q = 0; q < size; q++) {
      double v = S[(size_t)i * n + set[q]];
      if (v > best) best = v;
    }
    f += best + 1.0;
  }
  return f;
}

/* Alg. 2 (greedy facility location with the coverage cache m of Sec. 4.1 / App. A.1).
 *   step 1: s_i = sum_j S_ij, t_1 = argmax_i s_i, m = S[t_1, :]
 *   step k: g_i = sum_j max(0, S_ij - m_j) for i not yet chosen, t_k = argmax g_i,
 *           m = max(m, S[t_k, :])
 * Re-selection is prevented by an explicit chosen-mask (zeroing a row, as the listing words it,
 * would not exclude it when some m_j is negative).  Ties go to the lowest index.
 * picks[k] = t_k, gains[k] = the winning value, gaps[k] = winning value minus the runner-up among
 * the not-yet-chosen (INFINITY when there is no runner-up). */
ORACLE_API void toma_oracle_greedy_fl(const double *S, int n, int k, int32_t *picks, double *gains,
                                      double *gaps) {
  double *m = (double *)malloc(sizeof(double) * (size_t)n);
  char *chosen = (char *)calloc((size_t)n, 1);
  for (int step = 0; step < k; step++) {
    int best = -1, have2 = 0;
    double gbest = 0.0, gsecond = 0.0;
    for (int i = 0; i < n; i++) {
      if (chosen[i]) continue;
      double g = 0.0;
      if (step == 0) {
        for (int j = 0; j < n; j++) g += S[(size_t)i * n + j];
      } else {
        for (int j = 0; j < n; j++) {
          double d = S[(size_t)i * n + j] - m[j];
          if (d > 0.0) g += d;
        }
      }
      if (best < 0) {
        best = i; gbest = g;
      } else if (g > gbest) {
        gsecond = gbest; have2 = 1; best = i; gbest = g;
      } else if (!have2 || g > gsecond) {
        gsecond = g; have2 = 1;
      }
    }
    picks[step] = best;
    if (gains) gains[step] = gbest;
    if (gaps) gaps[step] = have2 ? gbest - gsecond : INFINITY;
    chosen[best] = 1;
    for (int j = 0; j < n; j++) {
      double v = S[(size_t)best * n + j];
      m[j] = (step == 0) ? v : (v > m[j] ? v : m[j]);
    }
  }
  free(m);
  free(chosen);
}

/* Alg. 1 with the marginal gain taken literally as f'(A + v) - f'(A) from Eq. 2 (no cache).
 * Independent of toma_oracle_greedy_fl; the two must return the same picks (App. A.1). */
ORACLE_API void toma_oracle_greedy_direct(const double *S, int n, int k, int32_t *picks,
                                          double *gains) {
  int32_t *set = (int32_t *)malloc(sizeof(int32_t) * (size_t)(k + 1));
  char *chosen = (char *)calloc((size_t)n, 1);
  for (int step = 0; step < k; step++) {
    double fcur = toma_oracle_fl_value(S, n, set, step);
    int best = -1;
    double gbest = 0.0;
    for (int v = 0; v < n; v++) {
      if (chosen[v]) continue;
      set[step] = v;
      double g = toma_oracle_fl_value(S, n, set, step + 1) - fcur;
      if (best < 0 || g > gbest) { best = v; gbest = g; }
    }
    set[step] = best;
    picks[step] = best;
    chosen[best] = 1;
    if (gains) gains[step] = gbest;
  }
  free(set);
  free(chosen);
}

/* Teacher-forced check of a pick sequence produced elsewhere: at every step, with the prefix of
 * the GIVEN picks as the chosen set, evaluate Alg. 2's values for all candidates and report
 *   deficit[k] = (max value - value of the given pick) / max(max value, 1e-30)   (0 if it is a max)
 *   is_first[k] = 1 when the given pick is the lowest-index maximiser.
 * Returns -1 when the picks are distinct and in range, else the first offending step. */
ORACLE_API int toma_oracle_check_picks(const double *S, int n, int k, const int32_t *picks,
                                       double *deficit, int32_t *is_first) {
  double *m = (double *)malloc(sizeof(double) * (size_t)n);
  char *chosen = (char *)calloc((size_t)n, 1);
  int bad = -1;
  for (int step = 0; step < k; step++) {
    int t = picks[step];
    if (t < 0 || t >= n || chosen[t]) { bad = step; break; }
    int best = -1;
    double gbest = 0.0, gt = 0.0;
    for (int i = 0; i < n; i++) {
      if (chosen[i]) continue;
      double g = 0.0;
      if (step == 0) {
        for (int j = 0; j < n; j++) g += S[(size_t)i * n + j];
      } else {
        for (int j = 0; j < n; j++) {
          double d = S[(size_t)i * n + j] - m[j];
          if (d > 0.0) g += d;
        }
      }
      if (best < 0 || g > gbest) { best = i; gbest = g; }
      if (i == t) gt = g;
    }
    double den = gbest > 1e-30 ? gbest : 1e-30;
    deficit[step] = (gbest - gt) / den;
    is_first[step] = (best == t);
    chosen[t] = 1;
    for (int j = 0; j < n; j++) {
      double v = S[(size_t)t * n + j];
      m[j] = (step == 0) ? v : (v > m[j] ? v : m[j]);
    }
  }
  free(m);
  free(chosen);
  return bad;
}

/* Alg. 3 step 1 for every (sample, region): idx[b][p][k] = grid index of the k-th pick of region
 * p of sample b (pick order).  gain/gap may be NULL.  X is [B][N][C]. */
ORACLE_API void toma_oracle_select(const oracle_desc *d, const double *X, int32_t *idx,
                                   double *gain, double *gap) {
  int P = n_regions(d), nl = n_loc(d), N = d->H * d->W, k = d->d_loc;
  int32_t *token_of = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
  toma_oracle_region_map(d->H, d->W, d->tile_h, d->tile_w, NULL, NULL, token_of);
#pragma omp parallel for schedule(dynamic)
  for (int bp = 0; bp < d->B * P; bp++) {
    int b = bp / P, p = bp % P;
    double *S = (double *)malloc(sizeof(double) * (size_t)nl * nl);
    int32_t *t = (int32_t *)malloc(sizeof(int32_t) * (size_t)k);
    toma_oracle_cosine(X + (size_t)b * N * d->C, token_of + (size_t)p * nl, nl, d->C, d->sim_bits, S);
    toma_oracle_greedy_fl(S, nl, k, t, gain ? gain + (size_t)bp * k : NULL,
                          gap ? gap + (size_t)bp * k : NULL);
    for (int q = 0; q < k; q++) idx[(size_t)bp * k + q] = token_of[(size_t)p * nl + t[q]];
    free(S);
    free(t);
  }
  free(token_of);
}

/* Token list of merge region rho: all N tokens in grid order when merge_regions == 1, else the
 * tokens of selection region rho in local order. */
static void merge_region_tokens(const oracle_desc *d, const int32_t *token_of, int rho, int32_t *tok) {
  int N = d->H * d->W;
  if (d->merge_regions == 1) {
    for (int s = 0; s < N; s++) tok[s] = s;
  } else {
    int nl = n_loc(d);
    for (int s = 0; s < nl; s++) tok[s] = token_of[(size_t)rho * nl + s];
  }
}

/* Sec. 4.2.1.  Inside each merge region with destinations j (rows of X named by idx, in idx
 * order) and sources s:
 *   L_js = scale * <d_j, x_s>                     (raw tokens; scale = 1/tau)
 *   A_js = exp(L_js - max_j' L_j's) / sum_j' exp(L_j's - max)     softmax over DESTINATIONS for
 *          each source s, so that a source's shares add up to one ("column-wise")
 *   Z_j  = sum_s A_js                              row sums; A~ = A / Z row-normalises
 * A is [B][R][D/R][N/R], Z is [B][D].  A destination that no source chooses has Z_j -> 0; it is
 * clamped at 1e-20 when dividing and *clamps counts such rows (expected: none). */
ORACLE_API void toma_oracle_merge_weights(const oracle_desc *d, const double *X, const int32_t *idx,
                                          double *A, double *Z, int64_t *clamps) {
  int P = n_regions(d), N = d->H * d->W, C = d->C, R = d->merge_regions;
  int D = P * d->d_loc, Dr = D / R, Nr = N / R;
  int32_t *token_of = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
  toma_oracle_region_map(d->H, d->W, d->tile_h, d->tile_w, NULL, NULL, token_of);
  int64_t nclamp = 0;
#pragma omp parallel for schedule(dynamic) reduction(+ : nclamp)
  for (int br = 0; br < d->B * R; br++) {
    int b = br / R, rho = br % R;
    const double *Xb = X + (size_t)b * N * C;
    const int32_t *dst = idx + (size_t)b * D + (size_t)rho * Dr;
    double *Ar = A + (size_t)br * Dr * Nr;
    double *Zr = Z + (size_t)b * D + (size_t)rho * Dr;
    int32_t *tok = (int32_t *)malloc(sizeof(int32_t) * (size_t)Nr);
    merge_region_tokens(d, token_of, rho, tok);
    for (int j = 0; j < Dr; j++) {
      const double *dj = Xb + (size_t)dst[j] * C;
      for (int s = 0; s < Nr; s++) {
        const double *xs = Xb + (size_t)tok[s] * C;
        double acc = 0.0;
        for (int c = 0; c < C; c++) acc += dj[c] * xs[c];
        Ar[(size_t)j * Nr + s] = d->scale * acc;
      }
    }
    for (int s = 0; s < Nr; s++) {
      double mx = -INFINITY, den = 0.0;
      for (int j = 0; j < Dr; j++) if (Ar[(size_t)j * Nr + s] > mx) mx = Ar[(size_t)j * Nr + s];
      for (int j = 0; j < Dr; j++) {
        double e = exp(Ar[(size_t)j * Nr + s] - mx);
        Ar[(size_t)j * Nr + s] = e;
        den += e;
      }
      for (int j = 0; j < Dr; j++) Ar[(size_t)j * Nr + s] /= den;
    }
    for (int j = 0; j < Dr; j++) {
      double z = 0.0;
      for (int s = 0; s < Nr; s++) z += Ar[(size_t)j * Nr + s];
      Zr[j] = z;
      if (z < 1e-20) nclamp++;
    }
    free(tok);
  }
  if (clamps) *clamps = nclamp;
  free(token_of);
}

static double clampz(double z) { return z > 1e-20 ? z : 1e-20; }

/* Sec. 4.2.1: X_merged = A~ X with A~_js = A_js / Z_j.  Xm is [B][D][C], rows in idx order. */
ORACLE_API void toma_oracle_merge(const oracle_desc *d, const double *X, const double *A,
                                  const double *Z, double *Xm) {
  int P = n_regions(d), N = d->H * d->W, C = d->C, R = d->merge_regions;
  int D = P * d->d_loc, Dr = D / R, Nr = N / R;
  int32_t *token_of = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
  toma_oracle_region_map(d->H, d->W, d->tile_h, d->tile_w, NULL, NULL, token_of);
#pragma omp parallel for schedule(dynamic)
  for (int bj = 0; bj < d->B * D; bj++) {
    int b = bj / D, jg = bj % D, rho = jg / Dr, j = jg % Dr;
    const double *Xb = X + (size_t)b * N * C;
    const double *Aj = A + ((size_t)(b * R + rho) * Dr + j) * Nr;
    double z = clampz(Z[(size_t)b * D + jg]);
    double *out = Xm + (size_t)bj * C;
    int32_t *tok = (int32_t *)malloc(sizeof(int32_t) * (size_t)Nr);
    merge_region_tokens(d, token_of, rho, tok);
    for (int c = 0; c < C; c++) out[c] = 0.0;
    for (int s = 0; s < Nr; s++) {
      double w = Aj[s] / z;
      const double *xs = Xb + (size_t)tok[s] * C;
      for (int c = 0; c < C; c++) out[c] += w * xs[c];
    }
    free(tok);
  }
  free(token_of);
}

/* Eq. 1 with tau = 1 on the token set U = [X_merged ; X_extra] (L = D + T rows per sample):
 * Q = U Wq, K = U Wk, V = U Wv (weights [C][C], y = x W); head h owns channels
 * [h*dh, (h+1)*dh); P = softmax over keys of Q_h K_h^T / sqrt(dh); O_h = P V_h; heads are
 * concatenated; O = O Wo when Wo is given.  Xe may be NULL when T == 0.  O is [B][L][C]. */
ORACLE_API void toma_oracle_attend(int B, int D, int T, int C, int heads, const double *Xm,
                                   const double *Xe, const double *Wq, const double *Wk,
                                   const double *Wv, const double *Wo, double *O) {
  int L = D + T, dh = C / heads;
  size_t per = (size_t)L * C;
  double *U = (double *)malloc(sizeof(double) * per * B);
  double *Q = (double *)malloc(sizeof(double) * per * B);
  double *K = (double *)malloc(sizeof(double) * per * B);
  double *V = (double *)malloc(sizeof(double) * per * B);
  double *Oh = (double *)malloc(sizeof(double) * per * B);
  for (int b = 0; b < B; b++) {
    memcpy(U + b * per, Xm + (size_t)b * D * C, sizeof(double) * (size_t)D * C);
    if (T > 0) memcpy(U + b * per + (size_t)D * C, Xe + (size_t)b * T * C, sizeof(double) * (size_t)T * C);
  }
#pragma omp parallel for schedule(dynamic)
  for (int r = 0; r < B * L; r++) {
    const double *u = U + (size_t)r * C;
    double *q = Q + (size_t)r * C, *k = K + (size_t)r * C, *v = V + (size_t)r * C;
    for (int n = 0; n < C; n++) { q[n] = 0.0; k[n] = 0.0; v[n] = 0.0; }
    for (int c = 0; c < C; c++) {
      double uc = u[c];
      const double *wq = Wq + (size_t)c * C, *wk = Wk + (size_t)c * C, *wv = Wv + (size_t)c * C;
      for (int n = 0; n < C; n++) { q[n] += uc * wq[n]; k[n] += uc * wk[n]; v[n] += uc * wv[n]; }
    }
  }
  double inv = 1.0 / sqrt((double)dh);
#pragma omp parallel for schedule(dynamic)
  for (int r = 0; r < B * L; r++) {
    int b = r / L;
    double *p = (double *)malloc(sizeof(double) * (size_t)L);
    for (int h = 0; h < heads; h++) {
      const double *q = Q + (size_t)r * C + (size_t)h * dh;
      double mx = -INFINITY, den = 0.0;
      for (int j = 0; j < L; j++) {
        const double *k = K + ((size_t)b * L + j) * C + (size_t)h * dh;
        double s = 0.0;
        for (int c = 0; c < dh; c++) s += q[c] * k[c];
        p[j] = s * inv;
        if (p[j] > mx) mx = p[j];
      }
      for (int j = 0; j < L; j++) { p[j] = exp(p[j] - mx); den += p[j]; }
      double *o = Oh + (size_t)r * C + (size_t)h * dh;
      for (int c = 0; c < dh; c++) o[c] = 0.0;
      for (int j = 0; j < L; j++) {
        double w = p[j] / den;
        const double *v = V + ((size_t)b * L + j) * C + (size_t)h * dh;
        for (int c = 0; c < dh; c++) o[c] += w * v[c];
      }
    }
    free(p);
  }
  if (Wo) {
#pragma omp parallel for schedule(dynamic)
    for (int r = 0; r < B * L; r++) {
      const double *u = Oh + (size_t)r * C;
      double *o = O + (size_t)r * C;
      for (int n = 0; n < C; n++) o[n] = 0.0;
      for (int c = 0; c < C; c++) {
        double uc = u[c];
        const double *w = Wo + (size_t)c * C;
        for (int n = 0; n < C; n++) o[n] += uc * w[n];
      }
    }
  } else {
    memcpy(O, Oh, sizeof(double) * per * B);
  }
  free(U); free(Q); free(K); free(V); free(Oh);
}

/* The same attention (Eq. 1) evaluated only for the query rows listed in rows[] (indices into
 * the B*L rows of U); keys and values are still formed from every token.  out is [nrows][C].
 * Lets a test check sampled rows of a workload whose full attention is too slow in fp64. */
ORACLE_API void toma_oracle_attend_rows(int B, int D, int T, int C, int heads, const double *Xm,
                                        const double *Xe, const double *Wq, const double *Wk,
                                        const double *Wv, const int32_t *rows, int nrows, double *out) {
  int L = D + T, dh = C / heads;
  size_t per = (size_t)L * C;
  double *U = (double *)malloc(sizeof(double) * per * B);
  double *K = (double *)malloc(sizeof(double) * per * B);
  double *V = (double *)malloc(sizeof(double) * per * B);
  for (int b = 0; b < B; b++) {
    memcpy(U + b * per, Xm + (size_t)b * D * C, sizeof(double) * (size_t)D * C);
    if (T > 0) memcpy(U + b * per + (size_t)D * C, Xe + (size_t)b * T * C, sizeof(double) * (size_t)T * C);
  }
#pragma omp parallel for schedule(dynamic)
  for (int r = 0; r < B * L; r++) {
    const double *u = U + (size_t)r * C;
    double *k = K + (size_t)r * C, *v = V + (size_t)r * C;
    for (int n = 0; n < C; n++) { k[n] = 0.0; v[n] = 0.0; }
    for (int c = 0; c < C; c++) {
      double uc = u[c];
      const double *wk = Wk + (size_t)c * C, *wv = Wv + (size_t)c * C;
      for (int n = 0; n < C; n++) { k[n] += uc * wk[n]; v[n] += uc * wv[n]; }
    }
  }
  double inv = 1.0 / sqrt((double)dh);
#pragma omp parallel for schedule(dynamic)
  for (int i = 0; i < nrows; i++) {
    int r = rows[i], b = r / L;
    const double *u = U + (size_t)r * C;
    double *q = (double *)malloc(sizeof(double) * (size_t)C);
    double *p = (double *)malloc(sizeof(double) * (size_t)L);
    for (int n = 0; n < C; n++) q[n] = 0.0;
    for (int c = 0; c < C; c++) {
      double uc = u[c];
      const double *wq = Wq + (size_t)c * C;
      for (int n = 0; n < C; n++) q[n] += uc * wq[n];
    }
    for (int h = 0; h < heads; h++) {
      const double *qh = q + (size_t)h * dh;
      double mx = -INFINITY, den = 0.0;
      for (int j = 0; j < L; j++) {
        const double *k = K + ((size_t)b * L + j) * C + (size_t)h * dh;
        double sc = 0.0;
        for (int c = 0; c < dh; c++) sc += qh[c] * k[c];
        p[j] = sc * inv;
        if (p[j] > mx) mx = p[j];
      }
      for (int j = 0; j < L; j++) { p[j] = exp(p[j] - mx); den += p[j]; }
      double *o = out + (size_t)i * C + (size_t)h * dh;
      for (int c = 0; c < dh; c++) o[c] = 0.0;
      for (int j = 0; j < L; j++) {
        double wgt = p[j] / den;
        const double *v = V + ((size_t)b * L + j) * C + (size_t)h * dh;
        for (int c = 0; c < dh; c++) o[c] += wgt * v[c];
      }
    }
    free(q);
    free(p);
  }
  free(U); free(K); free(V);
}

/* Cross-attention with the merged tokens as queries (Sec. 5.1: in the ToMA_once variant every module
 * of a transformer block, cross-attention included, runs on the merged tokens between one merge and
 * one unmerge).  Eq. 1 with tau = 1 and separate token sets: Q = U Wq from the Lq query tokens
 * (U [B][Lq][C], Wq [C][C]); K = Ctx Wk, V = Ctx Wv from the Tc context tokens (Ctx [B][Tc][Cc],
 * Wk, Wv [Cc][C]); head h owns channels [h*dh, (h+1)*dh); P = softmax over the context tokens of
 * Q_h K_h^T / sqrt(dh); O_h = P V_h; heads concatenated; O = O Wo when Wo is given.  O is [B][Lq][C]. */
ORACLE_API void toma_oracle_cross_attend(int B, int Lq, int Tc, int C, int Cc, int heads, const double *U,
                                         const double *Ctx, const double *Wq, const double *Wk,
                                         const double *Wv, const double *Wo, double *O) {
  int dh = C / heads;
  double *Q = (double *)malloc(sizeof(double) * (size_t)B * Lq * C);
  double *K = (double *)malloc(sizeof(double) * (size_t)B * Tc * C);
  double *V = (double *)malloc(sizeof(double) * (size_t)B * Tc * C);
  double *Oh = (double *)malloc(sizeof(double) * (size_t)B * Lq * C);
#pragma omp parallel for schedule(dynamic)
  for (int r = 0; r < B * Lq; r++) {
    double *q = Q + (size_t)r * C;
    for (int n = 0; n < C; n++) q[n] = 0.0;
    for (int c = 0; c < C; c++)
      for (int n = 0; n < C; n++) q[n] += U[(size_t)r * C + c] * Wq[(size_t)c * C + n];
  }
#pragma omp parallel for schedule(dynamic)
  for (int r = 0; r < B * Tc; r++) {
    double *k = K + (size_t)r * C, *v = V + (size_t)r * C;
    for (int n = 0; n < C; n++) { k[n] = 0.0; v[n] = 0.0; }
    for (int c = 0; c < Cc; c++) {
      double x = Ctx[(size_t)r * Cc + c];
      for (int n = 0; n < C; n++) { k[n] += x * Wk[(size_t)c * C + n]; v[n] += x * Wv[(size_t)c * C + n]; }
    }
  }
  double inv = 1.0 / sqrt((double)dh);
#pragma omp parallel for schedule(dynamic)
  for (int r = 0; r < B * Lq; r++) {
    int b = r / Lq;
    double *p = (double *)malloc(sizeof(double) * (size_t)Tc);
    for (int h = 0; h < heads; h++) {
      const double *q = Q + (size_t)r * C + (size_t)h * dh;
      double mx = -INFINITY, den = 0.0;
      for (int j = 0; j < Tc; j++) {
        const double *k = K + ((size_t)b * Tc + j) * C + (size_t)h * dh;
        double s = 0.0;
        for (int c = 0; c < dh; c++) s += q[c] * k[c];
        p[j] = s * inv;
        if (p[j] > mx) mx = p[j];
      }
      for (int j = 0; j < Tc; j++) { p[j] = exp(p[j] - mx); den += p[j]; }
      double *o = Oh + (size_t)r * C + (size_t)h * dh;
      for (int c = 0; c < dh; c++) o[c] = 0.0;
      for (int j = 0; j < Tc; j++) {
        double wgt = p[j] / den;
        const double *v = V + ((size_t)b * Tc + j) * C + (size_t)h * dh;
        for (int c = 0; c < dh; c++) o[c] += wgt * v[c];
      }
    }
    free(p);
  }
  if (Wo) {
#pragma omp parallel for schedule(dynamic)
    for (int r = 0; r < B * Lq; r++) {
      double *o = O + (size_t)r * C;
      for (int n = 0; n < C; n++) o[n] = 0.0;
      for (int c = 0; c < C; c++)
        for (int n = 0; n < C; n++) o[n] += Oh[(size_t)r * C + c] * Wo[(size_t)c * C + n];
    }
  } else {
    memcpy(O, Oh, sizeof(double) * (size_t)B * Lq * C);
  }
  free(Q); free(K); free(V); free(Oh);
}

/* Sec. 4.2.2 (transpose unmerge): X'_unmerged = A~^T X', i.e. for source s of merge region rho
 * Y[token(rho, s)] = sum_{j in rho} A~_js O[j].  O is [B][o_rows][C] and only its first D rows
 * (the merged image tokens) are read; Y is [B][N][C] in grid order. */
ORACLE_API void toma_oracle_unmerge(const oracle_desc *d, const double *A, const double *Z,
                                    const double *O, int o_rows, double *Y) {
  int P = n_regions(d), N = d->H * d->W, C = d->C, R = d->merge_regions;
  int D = P * d->d_loc, Dr = D / R, Nr = N / R;
  int32_t *token_of = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
  toma_oracle_region_map(d->H, d->W, d->tile_h, d->tile_w, NULL, NULL, token_of);
#pragma omp parallel for schedule(dynamic)
  for (int bs = 0; bs < d->B * N; bs++) {
    int b = bs / N, sg = bs % N, rho = sg / Nr, s = sg % Nr;
    int tok = (R == 1) ? s : token_of[(size_t)rho * Nr + s];
    double *y = Y + ((size_t)b * N + tok) * C;
    for (int c = 0; c < C; c++) y[c] = 0.0;
    for (int j = 0; j < Dr; j++) {
      int jg = rho * Dr + j;
      double w = A[((size_t)(b * R + rho) * Dr + j) * Nr + s] / clampz(Z[(size_t)b * D + jg]);
      const double *o = O + ((size_t)b * o_rows + jg) * C;
      for (int c = 0; c < C; c++) y[c] += w * o[c];
    }
  }
  free(token_of);
}

/* Sec. 4.2.2 (Moore-Penrose unmerge, the alternative the paper measures against): in toma_oracle.py
 * (unmerge_pinv), where numpy's SVD-based pseudo-inverse serves as the step. */

/* ---------------------------------------------------------------------------------------------
 * A feed-forward core module (Sec. 4.2: the module between merge and unmerge may be attention
 * or an MLP; Sec. 5.1's ToMA_once runs every module of a block on the merged tokens):
 *   out = gelu(X W1) W2,   gelu(x) = x/2 (1 + erf(x / sqrt 2)),
 * X [rows, C], W1 [C, hidden], W2 [hidden, C], no biases.  (The paper does not fix the MLP's
 * form; this is the textbook two-layer GELU block.)
 * --------------------------------------------------------------------------------------------- */
ORACLE_API void toma_oracle_mlp(int rows, int C, int hidden, const double *X, const double *W1,
                                const double *W2, double *out) {
#pragma omp parallel for
  for (int r = 0; r < rows; r++) {
    double *h = (double *)malloc(sizeof(double) * (size_t)hidden);
    for (int j = 0; j < hidden; j++) {
      double acc = 0.0;
      for (int k = 0; k < C; k++) acc += X[(size_t)r * C + k] * W1[(size_t)k * hidden + j];
      h[j] = 0.5 * acc * (1.0 + erf(acc / sqrt(2.0)));
    }
    for (int c = 0; c < C; c++) {
      double acc = 0.0;
      for (int j = 0; j < hidden; j++) acc += h[j] * W2[(size_t)j * C + c];
      out[(size_t)r * C + c] = acc;
    }
    free(h);
  }
}
