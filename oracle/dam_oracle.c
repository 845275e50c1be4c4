/*
 * dam_oracle.c -- slow, plain CPU statement of what the DAM hot path computes.
 *
 * TEST INFRASTRUCTURE ONLY. This file is the checker the GPU library is compared against; nothing
 * in the product path may call it, and it shares no code, header, table or helper with the GPU
 * library. Every function follows one passage of the paper (arXiv 2506.11104) and says which.
 *
 * Precision: the mask rule is a fixed sequence of individually rounded fp32 operations (the paper
 * does not fix a precision; a bit-exact mask needs one). Attention is evaluated in fp64 from the
 * inputs as stored (fp32, or bf16 widened exactly to fp32 by the caller).
 *
 * Build: gcc -O2 -fopenmp -ffp-contract=off -fno-fast-math -shared -fPIC (see build.py).
 * OpenMP is used only over independent units (maps, rows); no loop is blocked, fused or reordered.
 *
 * Pins (tests/test_oracle_*.py): Box-Cox closed forms and the value 2.00 printed in the paper's
 * App. B table; threshold special cases; match scores against literally materialised pattern
 * matrices; the capture against closed-form uniform attention, row sums and a library softmax;
 * prefix stability of the extension; re-expansion of the block index; attention against
 * dense causal attention, a brute-force numpy softmax, convexity, single-key and LSE-merge
 * identities. No function here is "parity unpinned" for lambda in {0.5, 1}; lambda = 0 and general
 * lambda (logf / powf, not correctly rounded) are pinned only up to a few ulp at the threshold
 * boundary and are marked "parity unpinned" for bit-exactness. The same holds for the alternative
 * transforms of App. B: raw sum, average, min-max and square root are exact sequences; log,
 * Yeo-Johnson, arcsinh (library functions) and z-score (fp64 sums) are "parity unpinned" for
 * bit-exactness and compared up to a band around the threshold.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---------------------------------------------------------------------------------------------
 * Sec. 4.2.2, feature amplification.
 *   Abar = A / (C + eps)                      (first equation of the section)
 *   X    = max(Abar, eps)                     (the clamp stated before the Box-Cox equation)
 *   B    = (X^lambda - 1) / lambda, ln X at lambda = 0      (Box-Cox equation)
 * cnt == NULL means a single causal capture: C = 1 for j <= i; for j > i the pair was never
 * computed, so C = 0 and the accumulated attention is 0.
 * Writes B [H][L][L] and returns the minimum of B over every map and every entry, including
 * never-valid pairs (the "min over l', h', i', j'" of the shift equation).
 * ------------------------------------------------------------------------------------------- */
float dam_oracle_boxcox(const float *attn_sum, const float *attn_cnt, int32_t H, int32_t L,
                        float lambda, float eps, float *B) {
  float bmin = INFINITY;
#pragma omp parallel for reduction(min : bmin) schedule(static)
  for (int64_t h = 0; h < H; ++h)
    for (int64_t i = 0; i < L; ++i)
      for (int64_t j = 0; j < L; ++j) {
        const int64_t at = (h * L + i) * L + j;
        float a, c;
        if (attn_cnt) {
          a = attn_sum[at];
          c = attn_cnt[at];
        } else {
          a = (j <= i) ? attn_sum[at] : 0.0f;
          c = (j <= i) ? 1.0f : 0.0f;
        }
        const float denom = c + eps;
        const float abar = a / denom;
        const float x = fmaxf(abar, eps);
        float b;
        if (lambda == 0.5f) {
          const float root = sqrtf(x);
          const float num = root - 1.0f;
          b = num / 0.5f;
        } else if (lambda == 1.0f) {
          b = x - 1.0f;
        } else if (lambda == 0.0f) {
          b = logf(x);
        } else {
          const float p = powf(x, lambda);
          const float num = p - 1.0f;
          b = num / lambda;
        }
        B[at] = b;
        if (b < bmin) bmin = b;
      }
  return bmin;
}

/* App. B, "Feature Amplification Transformation Methods": the nine alternatives for the step
 * between the mean map and the threshold. With Abar = A / (C + eps) and X = max(Abar, eps):
 *   0 Box-Cox (lambda)  (X^lambda - 1) / lambda, ln X at lambda = 0      (the method's default)
 *   1 raw sum           A
 *   2 average           Abar
 *   3 log               ln X
 *   4 Yeo-Johnson (lambda)  ((X + 1)^lambda - 1) / lambda, ln(X + 1) at lambda = 0   (X >= eps > 0: the
 *                       branches for negative inputs never apply)
 *   5 z-score           (X - mu) / (sigma + eps), mu and sigma (population) over every stored entry of
 *                       every map of the call, accumulated in fp64 and rounded to fp32
 *   6 min-max           (X - min X) / ((max X - min X) + eps), min and max over the same scope
 *   7 square root       sqrt X
 *   8 arcsinh           asinh X
 * each an fp32 sequence of individually rounded operations, and "unless otherwise stated" the global
 * minimum of the result is subtracted afterwards (App. B): this function writes T and returns that
 * minimum, exactly like dam_oracle_boxcox. cnt == NULL as there (one causal capture). */
float dam_oracle_transform(const float *attn_sum, const float *attn_cnt, int32_t H, int32_t L,
                           int32_t kind, float lambda, float eps, float *T) {
  if (kind == 0) return dam_oracle_boxcox(attn_sum, attn_cnt, H, L, lambda, eps, T);
  const int64_t n = (int64_t)H * L * L;
  /* pass 1: X (into T), and the statistics of X that z-score and min-max need */
  double sum = 0.0, sumsq = 0.0;
  float xmin = INFINITY, xmax = -INFINITY;
  for (int64_t h = 0; h < H; ++h)
    for (int64_t i = 0; i < L; ++i)
      for (int64_t j = 0; j < L; ++j) {
        const int64_t at = (h * L + i) * L + j;
        float a, c;
        if (attn_cnt) {
          a = attn_sum[at];
          c = attn_cnt[at];
        } else {
          a = (j <= i) ? attn_sum[at] : 0.0f;
          c = (j <= i) ? 1.0f : 0.0f;
        }
        const float denom = c + eps;
        const float abar = a / denom;
        const float x = fmaxf(abar, eps);
        sum += (double)x;
        sumsq += (double)x * (double)x;
        if (x < xmin) xmin = x;
        if (x > xmax) xmax = x;
        T[at] = kind == 1 ? a : (kind == 2 ? abar : x);
      }
  const double mean = sum / (double)n;
  double var = sumsq / (double)n - mean * mean;
  if (var < 0.0) var = 0.0;
  const float mu = (float)mean, sigma = (float)sqrt(var);
  float tmin = INFINITY;
  for (int64_t at = 0; at < n; ++at) {
    const float x = T[at];
    float t = x; /* kinds 1 and 2 */
    if (kind == 3) {
      t = logf(x);
    } else if (kind == 4) {
      const float x1 = x + 1.0f;
      if (lambda == 0.0f) {
        t = logf(x1);
      } else {
        const float p = powf(x1, lambda);
        const float num = p - 1.0f;
        t = num / lambda;
      }
    } else if (kind == 5) {
      const float num = x - mu;
      const float den = sigma + eps;
      t = num / den;
    } else if (kind == 6) {
      const float num = x - xmin;
      const float range = xmax - xmin;
      const float den = range + eps;
      t = num / den;
    } else if (kind == 7) {
      t = sqrtf(x);
    } else if (kind == 8) {
      t = asinhf(x);
    }
    T[at] = t;
    if (t < tmin) tmin = t;
  }
  return tmin;
}

/* Sec. 4.2.2 last equation and Sec. 4.2.3: Bstar = B - bmin; m[i][j] = 1 iff Bstar >= tau.
 * Causality (j <= i) is part of every mask (the vertical pattern's "i >= c", Fig. 1). */
void dam_oracle_true_mask(const float *B, int32_t H, int32_t L, float bmin, float tau, uint8_t *m) {
#pragma omp parallel for schedule(static)
  for (int64_t h = 0; h < H; ++h)
    for (int64_t i = 0; i < L; ++i)
      for (int64_t j = 0; j < L; ++j) {
        const int64_t at = (h * L + i) * L + j;
        const float bstar = B[at] - bmin;
        m[at] = (uint8_t)((bstar >= tau) && (j <= i));
      }
}

/* Sec. 4.2.4. Diagonal pattern r holds the entries (i, i - r), i = r .. L-1 (L - r of them); the
 * vertical pattern c holds (i, c), i = c .. L-1 (L - c of them). gamma = kept / size; matched iff
 * gamma >= mu (the equations' ">="). */
void dam_oracle_match(const uint8_t *m, int32_t H, int32_t L, float mu, int32_t *diag_cnt,
                      int32_t *vert_cnt, uint8_t *diag_flag, uint8_t *vert_flag) {
#pragma omp parallel for schedule(static)
  for (int64_t h = 0; h < H; ++h) {
    const uint8_t *mh = m + h * (int64_t)L * L;
    for (int64_t r = 0; r < L; ++r) {
      int32_t kept = 0;
      for (int64_t i = r; i < L; ++i) kept += mh[i * L + (i - r)];
      const int32_t size = (int32_t)(L - r);
      const float gamma = (float)kept / (float)size;
      diag_cnt[h * L + r] = kept;
      diag_flag[h * L + r] = (uint8_t)(gamma >= mu);
    }
    for (int64_t c = 0; c < L; ++c) {
      int32_t kept = 0;
      for (int64_t i = c; i < L; ++i) kept += mh[i * L + c];
      const int32_t size = (int32_t)(L - c);
      const float gamma = (float)kept / (float)size;
      vert_cnt[h * L + c] = kept;
      vert_flag[h * L + c] = (uint8_t)(gamma >= mu);
    }
  }
}

/* One head's stored mask artefact: the true mask (side L, may be 0) and the matched pattern sets,
 * given as flags over offsets / columns 0 .. P-1. */
typedef struct {
  const uint8_t *true_mask; /* [L][L] or NULL when L == 0 */
  const uint8_t *diag_flag; /* [P] */
  const uint8_t *vert_flag; /* [P] */
  int32_t L, P;
} dam_oracle_head;

/* Sec. 4.3: entry (i, j) of the mask applied to a length-S problem.
 *   Case 1 (S <= L): the true mask (every i, j < S <= L falls in the first branch).
 *   Case 2 (S > L):  the true mask inside the top-left L x L block; elsewhere the union of the
 *                    matched patterns, continued at a fixed offset (diagonal) or a fixed column
 *                    (vertical) down to the last row. */
static int kept_entry(const dam_oracle_head *hd, int64_t i, int64_t j) {
  if (j > i) return 0;
  if (i < hd->L && j < hd->L) return hd->true_mask[i * hd->L + j];
  const int64_t r = i - j;
  const int on_diag = (r < hd->P) && hd->diag_flag[r];
  const int on_vert = (j < hd->P) && hd->vert_flag[j];
  return on_diag || on_vert;
}

int dam_oracle_kept(const uint8_t *true_mask, int32_t L, const uint8_t *diag_flag,
                    const uint8_t *vert_flag, int32_t P, int64_t i, int64_t j) {
  dam_oracle_head hd = {true_mask, diag_flag, vert_flag, L, P};
  return kept_entry(&hd, i, j);
}

/* Rows [i0, i1) of the S x S mask as bytes, [i1 - i0][S]. */
void dam_oracle_rows(const uint8_t *true_mask, int32_t L, const uint8_t *diag_flag,
                     const uint8_t *vert_flag, int32_t P, int64_t S, int64_t i0, int64_t i1,
                     uint8_t *out) {
  dam_oracle_head hd = {true_mask, diag_flag, vert_flag, L, P};
#pragma omp parallel for schedule(static)
  for (int64_t i = i0; i < i1; ++i)
    for (int64_t j = 0; j < S; ++j) out[(i - i0) * S + j] = (uint8_t)kept_entry(&hd, i, j);
}

/* Kept keys of row i, ascending. Returns the count; writes at most cap indices. */
int64_t dam_oracle_kept_list(const uint8_t *true_mask, int32_t L, const uint8_t *diag_flag,
                             const uint8_t *vert_flag, int32_t P, int64_t i, int32_t *idx,
                             int64_t cap) {
  dam_oracle_head hd = {true_mask, diag_flag, vert_flag, L, P};
  int64_t n = 0;
  for (int64_t j = 0; j <= i; ++j)
    if (kept_entry(&hd, i, j)) {
      if (n < cap) idx[n] = (int32_t)j;
      ++n;
    }
  return n;
}

/* Block index of one head for query tiles [qt0, qt1): a tile (qt, kt) of tile_m x tile_n entries is
 * listed iff it holds a kept entry; listed tiles of a query tile are in ascending kt.
 *   row_cnt[qt - qt0]   listed tiles of that query tile
 *   col / kind / tile_bits   per listed tile, in order; kind bit 0 = 1 iff all tile_m * tile_n
 *                       entries are kept (which needs the tile inside S and strictly below the
 *                       diagonal); kind bit 1 + q = 1 iff key quarter q of the tile, columns
 *                       [q tile_n / 4, (q + 1) tile_n / 4), holds a kept entry
 *   tile_bits           [tile][tile_m][tile_n / 64] words, bit (j % 64) of word j / 64 of row i
 * Returns the number of listed tiles; writes at most cap of them (col, kind, tile_bits may be
 * NULL to count only). */
int64_t dam_oracle_block_index(const uint8_t *true_mask, int32_t L, const uint8_t *diag_flag,
                               const uint8_t *vert_flag, int32_t P, int64_t S, int32_t tile_m,
                               int32_t tile_n, int64_t qt0, int64_t qt1, int32_t *row_cnt,
                               int32_t *col, uint8_t *kind, uint64_t *tile_bits, int64_t cap) {
  dam_oracle_head hd = {true_mask, diag_flag, vert_flag, L, P};
  const int64_t nKt = (S + tile_n - 1) / tile_n;
  const int64_t wpr = tile_n / 64; /* words per tile row */
  const int64_t tile_words = (int64_t)tile_m * wpr;
  uint64_t *bits = (uint64_t *)malloc((size_t)tile_words * sizeof(uint64_t));
  int64_t total = 0;
  for (int64_t qt = qt0; qt < qt1; ++qt) {
    int32_t listed = 0;
    for (int64_t kt = 0; kt < nKt; ++kt) {
      memset(bits, 0, (size_t)tile_words * sizeof(uint64_t));
      int64_t kept = 0;
      int quarters = 0;
      for (int64_t ii = 0; ii < tile_m; ++ii)
        for (int64_t jj = 0; jj < tile_n; ++jj) {
          const int64_t i = qt * tile_m + ii, j = kt * tile_n + jj;
          if (i < S && j < S && kept_entry(&hd, i, j)) {
            bits[ii * wpr + jj / 64] |= (uint64_t)1 << (jj % 64);
            quarters |= 1 << (jj / (tile_n / 4));
            ++kept;
          }
        }
      if (kept == 0) continue;
      if (total < cap) {
        if (col) col[total] = (int32_t)kt;
        if (kind) kind[total] = (uint8_t)((kept == (int64_t)tile_m * tile_n) | (quarters << 1));
        if (tile_bits)
          memcpy(tile_bits + total * tile_words, bits, (size_t)tile_words * sizeof(uint64_t));
      }
      ++total;
      ++listed;
    }
    row_cnt[qt - qt0] = listed;
  }
  free(bits);
  return total;
}

/* Block index with the matched columns gathered into tiles of their own (a layout of this build for
 * the attention kernel; the mask it describes is the one of Sec. 4.3, unchanged). gcols[n_g]: the
 * head's matched columns below S, ascending. For a query tile that lies wholly in the pattern region
 * (its first row >= L) the entries of a row i are split into two disjoint parts:
 *   diagonal part   key j <= i with i - j a matched diagonal              -> ordinary tiles kt < nKt
 *   column part     gathered column c = gcols[s], c <= i, i - c NOT a matched diagonal
 *                   -> gathered tiles nKt + v, v = s / tile_n, bit s % tile_n of the row
 * Query tiles that start inside the true-mask block are listed exactly as by dam_oracle_block_index.
 * Listing, order (ascending tile index, gathered tiles after the ordinary ones), kind and bits follow
 * the same rules as there. */
int64_t dam_oracle_block_index_gathered(const uint8_t *true_mask, int32_t L, const uint8_t *diag_flag,
                                        const uint8_t *vert_flag, int32_t P, int64_t S, int32_t tile_m,
                                        int32_t tile_n, int64_t qt0, int64_t qt1, const int32_t *gcols,
                                        int64_t n_g, int32_t *row_cnt, int32_t *col, uint8_t *kind,
                                        uint64_t *tile_bits, int64_t cap) {
  dam_oracle_head hd = {true_mask, diag_flag, vert_flag, L, P};
  const int64_t nKt = (S + tile_n - 1) / tile_n;
  const int64_t nGt = (n_g + tile_n - 1) / tile_n;
  const int64_t wpr = tile_n / 64;
  const int64_t tile_words = (int64_t)tile_m * wpr;
  uint64_t *bits = (uint64_t *)malloc((size_t)tile_words * sizeof(uint64_t));
  int64_t total = 0;
  for (int64_t qt = qt0; qt < qt1; ++qt) {
    int32_t listed = 0;
    const int split = qt * tile_m >= L;
    for (int64_t kt = 0; kt < nKt + (split ? nGt : 0); ++kt) {
      memset(bits, 0, (size_t)tile_words * sizeof(uint64_t));
      int64_t kept = 0;
      int quarters = 0;
      for (int64_t ii = 0; ii < tile_m; ++ii)
        for (int64_t jj = 0; jj < tile_n; ++jj) {
          const int64_t i = qt * tile_m + ii;
          int on = 0;
          if (i < S) {
            if (kt < nKt) {
              const int64_t j = kt * tile_n + jj;
              if (j < S) {
                if (!split) on = kept_entry(&hd, i, j);
                else on = j <= i && i - j < P && diag_flag[i - j];
              }
            } else {
              const int64_t s_at = (kt - nKt) * tile_n + jj;
              if (s_at < n_g) {
                const int64_t c = gcols[s_at];
                on = c <= i && !(i - c < P && diag_flag[i - c]);
              }
            }
          }
          if (on) {
            bits[ii * wpr + jj / 64] |= (uint64_t)1 << (jj % 64);
            quarters |= 1 << (jj / (tile_n / 4));
            ++kept;
          }
        }
      if (kept == 0) continue;
      if (total < cap) {
        if (col) col[total] = (int32_t)kt;
        if (kind) kind[total] = (uint8_t)((kept == (int64_t)tile_m * tile_n) | (quarters << 1));
        if (tile_bits)
          memcpy(tile_bits + total * tile_words, bits, (size_t)tile_words * sizeof(uint64_t));
      }
      ++total;
      ++listed;
    }
    row_cnt[qt - qt0] = listed;
  }
  free(bits);
  return total;
}

/* Sec. 3 with the -inf reading of Sec. 4.3's last paragraph: attention of one query over an explicit
 * list of kept keys.
 *   s_j = (q . k_j) * scale;  w_j = exp(s_j - max s);  O = sum w_j v_j / sum w_j;
 *   lse = max s + ln sum w_j.   Empty list: O = 0, lse = -inf.
 * q [d]; K, V rows of d floats at stride row_stride; idx[n] row numbers. fp64 throughout. */
static void attend_list(const float *q, const float *K, const float *V, int64_t row_stride,
                        int32_t d, const int32_t *idx, int64_t n, double scale, double *O,
                        double *lse) {
  for (int32_t t = 0; t < d; ++t) O[t] = 0.0;
  if (n == 0) {
    *lse = -INFINITY;
    return;
  }
  double *s = (double *)malloc((size_t)n * sizeof(double));
  double smax = -INFINITY;
  for (int64_t a = 0; a < n; ++a) {
    const float *k = K + (int64_t)idx[a] * row_stride;
    double dot = 0.0;
    for (int32_t t = 0; t < d; ++t) dot += (double)q[t] * (double)k[t];
    s[a] = dot * scale;
    if (s[a] > smax) smax = s[a];
  }
  double wsum = 0.0;
  for (int64_t a = 0; a < n; ++a) {
    const double w = exp(s[a] - smax);
    const float *v = V + (int64_t)idx[a] * row_stride;
    wsum += w;
    for (int32_t t = 0; t < d; ++t) O[t] += w * (double)v[t];
  }
  for (int32_t t = 0; t < d; ++t) O[t] /= wsum;
  *lse = smax + log(wsum);
  free(s);
}

/* Decode form: n_items independent (query, cache, list) triples.
 *   q [n_items][d];  kv_of[n_items]: which cache block each item reads; caches
 *   [n_blocks][T][d]; CSR kept_ptr [n_items + 1] / kept_idx.  out [n_items][d] f64, lse [n_items]. */
void dam_oracle_attend_lists(const float *q, const float *kcache, const float *vcache,
                             const int32_t *kv_of, int64_t T, int32_t d, const int64_t *kept_ptr,
                             const int32_t *kept_idx, int64_t n_items, double scale, double *out,
                             double *lse) {
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t it = 0; it < n_items; ++it) {
    const float *K = kcache + (int64_t)kv_of[it] * T * d;
    const float *V = vcache + (int64_t)kv_of[it] * T * d;
    attend_list(q + it * d, K, V, d, d, kept_idx + kept_ptr[it], kept_ptr[it + 1] - kept_ptr[it],
                scale, out + it * d, lse + it);
  }
}

/* Prefill form: rows (head[n], row[n]) of a causal self-attention layer with per-head masks.
 *   q_rows [n][d]: the query vectors of those rows (gathered by the caller);
 *   K, V [Hkv][S][d];  query head h reads KV head h / (Hq / Hkv);
 *   per-head artefacts: true_mask [Hq][L][L] (NULL when L == 0), diag_flag / vert_flag [Hq][P].
 * The kept set of a row is found by testing every key j <= i with the Sec. 4.3 rule. */
void dam_oracle_attend_rows(const float *q_rows, const float *K, const float *V, int32_t Hq,
                            int32_t Hkv, int64_t S, int32_t d, const uint8_t *true_mask, int32_t L,
                            const uint8_t *diag_flag, const uint8_t *vert_flag, int32_t P,
                            const int32_t *head, const int64_t *row, int64_t n, double scale,
                            double *out, double *lse) {
  const int32_t group = Hq / Hkv;
#pragma omp parallel for schedule(dynamic, 4)
  for (int64_t a = 0; a < n; ++a) {
    const int32_t h = head[a];
    const int64_t i = row[a];
    dam_oracle_head hd = {true_mask ? true_mask + (int64_t)h * L * L : NULL,
                          diag_flag + (int64_t)h * P, vert_flag + (int64_t)h * P, L, P};
    int32_t *idx = (int32_t *)malloc((size_t)(i + 1) * sizeof(int32_t));
    int64_t cnt = 0;
    for (int64_t j = 0; j <= i; ++j)
      if (kept_entry(&hd, i, j)) idx[cnt++] = (int32_t)j;
    const int64_t kvh = h / group;
    attend_list(q_rows + a * d, K + kvh * S * d, V + kvh * S * d, d, d, idx, cnt, scale,
                out + a * d, lse + a);
    free(idx);
  }
}

/* Sec. 4.2.1 / 4.2.2, pattern capture: one sequence of n <= L tokens is run with full causal
 * attention and its attention probabilities are added to the accumulated statistics,
 *   A[h][i][j] += softmax_j(q_i . k_j * scale)   and   C[h][i][j] += 1     for j <= i < n
 * ("attention weights summed over batches" and "the number of times a position pair was valid").
 * Q [Hq][n][d], K [Hkv][n][d] (query head h reads KV head h / (Hq / Hkv)); A, C [Hq][L][L] fp32,
 * C may be NULL. The softmax is evaluated in fp64 and rounded to fp32 once, then added to the fp32
 * sum (the paper fixes no storage precision; fp32 statistics is this build's reading). */
void dam_oracle_capture(const float *Q, const float *K, int32_t Hq, int32_t Hkv, int64_t n, int32_t d,
                        int64_t L, double scale, float *A, float *C) {
  const int32_t group = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic, 8)
  for (int64_t h = 0; h < Hq; ++h)
    for (int64_t i = 0; i < n; ++i) {
      const float *q = Q + (h * n + i) * d;
      const float *Kh = K + (int64_t)(h / group) * n * d;
      double *s = (double *)malloc((size_t)(i + 1) * sizeof(double));
      double smax = -INFINITY;
      for (int64_t j = 0; j <= i; ++j) {
        double dot = 0.0;
        for (int32_t t = 0; t < d; ++t) dot += (double)q[t] * (double)Kh[j * d + t];
        s[j] = dot * scale;
        if (s[j] > smax) smax = s[j];
      }
      double wsum = 0.0;
      for (int64_t j = 0; j <= i; ++j) {
        s[j] = exp(s[j] - smax);
        wsum += s[j];
      }
      for (int64_t j = 0; j <= i; ++j) {
        const int64_t at = (h * L + i) * L + j;
        A[at] = A[at] + (float)(s[j] / wsum);
        if (C) C[at] = C[at] + 1.0f;
      }
      free(s);
    }
}

/* Threads the parallel loops above use (reported next to every oracle timing). */
int dam_oracle_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
