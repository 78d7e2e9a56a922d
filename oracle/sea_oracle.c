/*
 * CPU oracle for the SEA attention forward pass (arXiv 2310.01777).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * path computes; it is called by the tests, by the smoke check and by the
 * benchmark's cpu_baseline leg, never by the product path.  It shares no code,
 * header, table or helper with the HIP library.
 *
 * Everything is fp64, naive loops, one head after the other, no blocking and no
 * reordering beyond what the method states.  Inputs are host arrays of double
 * holding the exact values of the fp32 or bf16 tensors the GPU sees.
 *
 * Passages followed (section names of the paper):
 *   Sec. 3 "Preliminaries"            A = softmax(Q K^T), C = A V
 *   Sec. 3 "Performer (FAVOR+)"       phi(Q) (phi(K)^T phi(V)), linear in T
 *   Sec. 3.1 "Attention Matrix Estimation"   V_I = nearest-neighbour stretched
 *        identity, "Performer output is the attention matrix when V = I"
 *   Sec. 3.1 "Grouped Top-k^ Selection"      per-query and causal-per-batch grouping
 *   Sec. 3.1 "Linear Sparse Attention Mask Generation" + App. A.5.3
 *        k^ = max(1, round(k K / T)), nearest-neighbour expansion of the
 *        compressed mask, replication cap with uniform spacing
 *   Sec. 3.1.1 "Sparse Attention Mechanism"  rho (masked QK^T on stored
 *        entries), sigma (softmax over stored entries), C = A* V
 *   Sec. 3.1.1 "Output Calculation"          C_sea = s_mix C + (1 - s_mix) C_avg
 *
 * Readings taken where the paper is silent (each also listed in the design
 * notes of the repository):
 *   - the feature map is the positive softmax-kernel map
 *       phi(x)[i] = exp(w_i.x - |x|^2/2),  x = sqrt(scale) * q  (same for keys)
 *     with the projection matrix W passed in by the caller;
 *   - the estimate has no learned decoder: V_I is the T x K nearest-neighbour
 *     stretch of I_K, so FAVOR+(Q,K,V_I) is itself a T x K matrix, normalised
 *     per row (linear-attention normaliser); causal rows only see keys j <= t;
 *   - key buckets are fixed: key j belongs to column floor(j K / T);
 *     geometry = 1 is the other reading, App. A.4 (figure of the masking
 *     process): a causal row t is resized to its own width, so its column c
 *     holds the keys [ceil(c (t+1) / K), ceil((c+1)(t+1) / K)) -- the whole
 *     method for that row is the bidirectional one on a sequence of t + 1 keys;
 *     in reduced-precision mode every column of such a row is summed key by
 *     key, as a fixed-bucket row's own column is: phi(q_t) and each phi(k_j)
 *     are rounded, nothing else;
 *   - masked-out keys are excluded from the softmax (not given logit zero);
 *   - right padding: keys and rows >= seq_len[b] are inactive;
 *   - ties in the selection go to the lower column; a column with no admissible
 *     key is never selected;
 *   - reduced-precision mode (bf16 inputs): phi(Q), the K x m key-side state
 *     phi(K)^T V_I and, for the keys of a causal row's own bucket, phi(k_j)
 *     are rounded to an 8-bit significand, round-to-nearest-even; products are
 *     summed without further rounding.
 *
 * Pins (tests, CPU only): k^ = K reproduces dense softmax attention computed by
 * a library softmax; the estimate converges to bucket sums of the exact softmax
 * matrix as m grows and equals a closed form for zero queries/keys; the
 * expansion equals a library nearest-neighbour resize of the dense mask and
 * hand-enumerated cases; the selection equals a full sort; causality and
 * padding invariances hold bit for bit.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
  int32_t B, H, T, d;
  int32_t m;        /* random features, W is [m][d]                          */
  int32_t K;        /* compressed width                                       */
  int32_t k_hat;    /* selections per query row in the compressed space       */
  int32_t k_budget; /* the paper's k: cap on keys per row, 0 = no cap         */
  int32_t causal;
  int32_t round8;   /* 1: apply the reduced-precision rounding points         */
  int32_t grouping; /* 0: per-query top-k^; 1: causal-per-batch (over heads)  */
  int32_t geometry; /* 0: key j belongs to column floor(j K / T) for every row;
                       1 (causal only): row t spreads its K columns over its own
                       t + 1 keys, column floor(j K / (t + 1))               */
  double scale;     /* logits = scale * q.k                                   */
} ref_params;

/* ---- small integer helpers (Sec. 3.1 "Mask Generation", App. A.5.3) ------ */

/* k^ = max(1, round(k K / T)); halves round up. */
int32_t ref_k_hat(int32_t k, int32_t K, int32_t T) {
  int64_t num = (int64_t)k * K;
  int64_t r = (2 * num + T) / (2 * (int64_t)T); /* floor(x + 1/2) */
  return r < 1 ? 1 : (int32_t)r;
}

/* first key of column c: ceil(c T / K) */
static int64_t block_start(int64_t c, int64_t T, int64_t K) {
  return (c * T + K - 1) / K;
}

/* column of key j: floor(j K / T) */
static int64_t bucket_of(int64_t j, int64_t T, int64_t K) { return (j * K) / T; }

/* keys emitted for a selected column of width w */
static int64_t replication(int64_t w, int64_t k_hat, int64_t k_budget) {
  if (k_budget <= 0) return w;
  int64_t cap = k_budget / k_hat;
  if (cap < 1) cap = 1;
  return w < cap ? w : cap;
}

/* most columns one row of one head can select: k^ per query; with the causal-per-batch
   grouping a single head may take up to H k^ of the time step's quota (never more than K) */
int32_t ref_sel_stride(const ref_params* p) {
  if (p->grouping == 0) return p->k_hat;
  int64_t q = (int64_t)p->H * p->k_hat;
  return (int32_t)(q < p->K ? q : p->K);
}

/* row stride of the index list: (columns per row) * replication of the widest column */
int32_t ref_row_stride(const ref_params* p) {
  int64_t wmax = ((int64_t)p->T + p->K - 1) / p->K;
  return (int32_t)(ref_sel_stride(p) * replication(wmax, p->k_hat, p->k_budget));
}

/* round to an 8-bit significand (bf16 precision, unbounded exponent), RNE */
double ref_round8(double x) {
  if (x == 0.0 || !isfinite(x)) return x;
  int e;
  double f = frexp(x, &e);          /* |f| in [0.5, 1) */
  double s = ldexp(f, 8);           /* |s| in [128, 256) */
  double r = nearbyint(s);          /* default mode: ties to even */
  return ldexp(r, e - 8);
}

static int32_t row_at(const int32_t* rows, int32_t r) { return rows ? rows[r] : r; }

/* ---- a1-a3: random-feature estimate of the compressed attention matrix ---- */
/*
 * Q, K: [B][H][T][d], W: [m][d], seq_len: [B] or NULL.
 * rows: n_rows query positions (ascending, same for every head) or NULL = all T.
 * A_hat out: [B][H][n_rows][K], rows sum to 1 (inactive rows all zero).
 */
int ref_estimate(const ref_params* p, const double* Q, const double* K,
                 const double* W, const int32_t* seq_len, const int32_t* rows,
                 int32_t n_rows, double* A_hat) {
  const int64_t T = p->T, d = p->d, m = p->m, KK = p->K;
  if (!rows) n_rows = p->T;
  const double rs = sqrt(p->scale);
  double* phiK = (double*)malloc(sizeof(double) * T * m);
  double* state = (double*)malloc(sizeof(double) * KK * m); /* phi(K)^T V_I */
  double* phiQ = (double*)malloc(sizeof(double) * m);
  double* arg = (double*)malloc(sizeof(double) * m);
  double* y = (double*)malloc(sizeof(double) * d);
  if (!phiK || !state || !phiQ || !arg || !y) return -1;

  for (int64_t b = 0; b < p->B; ++b) {
    const int64_t len = seq_len ? seq_len[b] : T;
    for (int64_t h = 0; h < p->H; ++h) {
      const double* Qh = Q + ((b * p->H + h) * T) * d;
      const double* Kh = K + ((b * p->H + h) * T) * d;
      double* Ah = A_hat + ((b * p->H + h) * (int64_t)n_rows) * KK;

      /* phi(K): positive softmax-kernel features of the scaled keys */
      for (int64_t j = 0; j < T; ++j) {
        double ny = 0.0;
        for (int64_t e = 0; e < d; ++e) { y[e] = rs * Kh[j * d + e]; ny += y[e] * y[e]; }
        for (int64_t i = 0; i < m; ++i) {
          double dot = 0.0;
          for (int64_t e = 0; e < d; ++e) dot += W[i * d + e] * y[e];
          phiK[j * m + i] = (j < len) ? exp(dot - 0.5 * ny) : 0.0;
        }
      }
      /* phi(K)^T V_I: V_I[j][c] = 1 iff c = floor(j K / T) */
      memset(state, 0, sizeof(double) * KK * m);
      for (int64_t j = 0; j < T; ++j) {
        int64_t c = bucket_of(j, T, KK);
        for (int64_t i = 0; i < m; ++i) state[c * m + i] += phiK[j * m + i];
      }
      if (p->round8)
        for (int64_t x = 0; x < KK * m; ++x) state[x] = ref_round8(state[x]);

      for (int32_t r = 0; r < n_rows; ++r) {
        const int64_t t = row_at(rows, r);
        double* Arow = Ah + (int64_t)r * KK;
        for (int64_t c = 0; c < KK; ++c) Arow[c] = 0.0;
        if (t >= len) continue;
        /* phi(q_t); a power-of-two row shift keeps the exponent in range and
           commutes with the rounding below, so it changes nothing */
        double nx = 0.0, amax = -INFINITY;
        for (int64_t e = 0; e < d; ++e) { y[e] = rs * Qh[t * d + e]; nx += y[e] * y[e]; }
        for (int64_t i = 0; i < m; ++i) {
          double dot = 0.0;
          for (int64_t e = 0; e < d; ++e) dot += W[i * d + e] * y[e];
          arg[i] = dot - 0.5 * nx;
          if (arg[i] > amax) amax = arg[i];
        }
        const double shift = ceil(amax / M_LN2) * M_LN2;
        for (int64_t i = 0; i < m; ++i) {
          phiQ[i] = exp(arg[i] - shift);
          if (p->round8) phiQ[i] = ref_round8(phiQ[i]);
        }
        const int64_t ct = bucket_of(t, T, KK);
        double rowsum = 0.0;
        if (p->geometry == 1) {
          /* the row's own width: FAVOR+ with V_I the (t+1) x K stretch of the identity */
          for (int64_t j = 0; j <= t; ++j) {
            double dotp = 0.0;
            for (int64_t i = 0; i < m; ++i) {
              /* key by key, as in the own column above: each phi(k_j) is rounded before its product */
              const double f = phiK[j * m + i];
              dotp += phiQ[i] * (p->round8 ? ref_round8(f) : f);
            }
            Arow[bucket_of(j, t + 1, KK)] += dotp;
            rowsum += dotp;
          }
          if (rowsum > 0.0)
            for (int64_t c = 0; c < KK; ++c) Arow[c] /= rowsum;
          continue;
        }
        for (int64_t c = 0; c < KK; ++c) {
          double acc = 0.0;
          if (!p->causal || c < ct) {
            /* every key of the column is admissible: phi(q_t) . (phi(K)^T V_I)[c] */
            const double* s = state + c * m;
            for (int64_t i = 0; i < m; ++i) acc += phiQ[i] * s[i];
          } else if (c == ct) {
            /* the row's own column: only its keys j <= t (causal FAVOR+ prefix), key by key */
            for (int64_t j = block_start(ct, T, KK); j <= t; ++j)
              for (int64_t i = 0; i < m; ++i) {
                const double f = phiK[j * m + i];
                acc += phiQ[i] * (p->round8 ? ref_round8(f) : f);
              }
          } else {
            continue;
          }
          Arow[c] = acc;
          rowsum += acc;
        }
        if (rowsum > 0.0)
          for (int64_t c = 0; c < KK; ++c) Arow[c] /= rowsum;
      }
    }
  }
  free(phiK); free(state); free(phiQ); free(arg); free(y);
  return 0;
}

/* ---- a4-a5: grouped top-k^ and expansion to key positions ------------------ */
/* expansion of the columns flagged in taken[0..ncand) of one row (App. A.5.3) */
static void expand_row(const ref_params* p, const uint8_t* taken, int64_t ncand, int64_t jmax,
                       int64_t T, int32_t* srow, int32_t* irow, int32_t* cnt_out) {
  const int64_t KK = p->K;  /* T: the width the row's columns are spread over */
  int64_t ns = 0, ni = 0;
  for (int64_t c = 0; c < ncand; ++c) {
    if (!taken[c]) continue;
    if (srow) srow[ns] = (int32_t)c;
    ++ns;
    const int64_t s0 = block_start(c, T, KK);
    const int64_t w = block_start(c + 1, T, KK) - s0;
    const int64_t rep = replication(w, p->k_hat, p->k_budget);
    for (int64_t i = 0; i < rep; ++i) {
      const int64_t j = s0 + (i * w) / rep;
      if (j <= jmax) irow[ni++] = (int32_t)j;
    }
  }
  *cnt_out = (int32_t)ni;
}

/*
 * A_hat: [B][H][n_rows][K].  sel out: [B][H][n_rows][S] ascending columns, -1 padded (may be
 * NULL), S = ref_sel_stride.  idx out: [B][H][n_rows][L] ascending key positions, -1 padded,
 * L = ref_row_stride.  cnt out: [B][H][n_rows].
 * grouping 0 (Sec. 3.1 "per-query"): each row of each head keeps its k^ largest entries.
 * grouping 1 (Sec. 3.1 "causal-per-batch"): A_hat is viewed as [T][H K]; each time step keeps
 * the H k^ largest entries of its H x K slab, so heads share the step's quota.  Ties go to the
 * lower flattened index h K + c.
 */
int ref_topk_mask(const ref_params* p, const double* A_hat, const int32_t* seq_len,
                  const int32_t* rows, int32_t n_rows, int32_t* sel, int32_t* idx,
                  int32_t* cnt) {
  const int64_t T = p->T, KK = p->K, H = p->H;
  if (!rows) n_rows = p->T;
  const int64_t L = ref_row_stride(p), S = ref_sel_stride(p);
  uint8_t* taken = (uint8_t*)malloc(H * KK);
  uint8_t* empty = (uint8_t*)malloc(KK);
  if (!taken || !empty) return -1;
  for (int64_t b = 0; b < p->B; ++b) {
    const int64_t len = seq_len ? seq_len[b] : T;
    for (int32_t r = 0; r < n_rows; ++r) {
      const int64_t t = row_at(rows, r);
      /* last admissible key of this row and its candidate columns 0..ncand-1 */
      const int64_t jmax = (p->causal && t < len - 1) ? t : len - 1;
      /* Tw: the width the row's K columns are spread over.  Columns 0..ncand-1 can hold an
         admissible key; with the row's own width (Tw = t + 1 < K) some of them are empty */
      const int64_t Tw = p->geometry == 1 ? t + 1 : T;
      const int64_t ncand = t < len ? bucket_of(jmax, Tw, KK) + 1 : 0;
      int64_t nfull = 0;
      for (int64_t c = 0; c < ncand; ++c) {
        empty[c] = block_start(c + 1, Tw, KK) <= block_start(c, Tw, KK);
        nfull += !empty[c];
      }
      memset(taken, 0, H * KK);
      if (p->grouping == 0) {
        const int64_t n = p->k_hat < nfull ? p->k_hat : nfull;
        for (int64_t h = 0; h < H; ++h) {
          const double* Arow = A_hat + ((b * H + h) * (int64_t)n_rows + r) * KK;
          /* n passes of "largest remaining, lowest column on ties" */
          for (int64_t s = 0; s < n; ++s) {
            int64_t best = -1;
            for (int64_t c = 0; c < ncand; ++c) {
              if (taken[h * KK + c] || empty[c]) continue;
              if (best < 0 || Arow[c] > Arow[best]) best = c;
            }
            taken[h * KK + best] = 1;
          }
        }
      } else {
        const int64_t quota = H * p->k_hat, total = H * nfull;
        const int64_t n = quota < total ? quota : total;
        for (int64_t s = 0; s < n; ++s) {
          int64_t bh = -1, bc = -1;
          double bv = 0.0;
          for (int64_t h = 0; h < H; ++h) {
            const double* Arow = A_hat + ((b * H + h) * (int64_t)n_rows + r) * KK;
            for (int64_t c = 0; c < ncand; ++c) {
              if (taken[h * KK + c] || empty[c]) continue;
              if (bh < 0 || Arow[c] > bv) { bh = h; bc = c; bv = Arow[c]; }
            }
          }
          taken[bh * KK + bc] = 1;
        }
      }
      for (int64_t h = 0; h < H; ++h) {
        const int64_t row = (b * H + h) * (int64_t)n_rows + r;
        int32_t* srow = sel ? sel + row * S : NULL;
        int32_t* irow = idx + row * L;
        for (int64_t x = 0; x < L; ++x) irow[x] = -1;
        if (srow) for (int64_t x = 0; x < S; ++x) srow[x] = -1;
        cnt[row] = 0;
        if (t >= len) continue;
        expand_row(p, taken + h * KK, ncand, jmax, Tw, srow, irow, &cnt[row]);
      }
    }
  }
  free(taken); free(empty);
  return 0;
}

/* ---- a6: sparse attention over the listed keys --------------------------- */
/*
 * Q, K, V: [B][H][T][d]; idx: [B][H][n_rows][L]; cnt: [B][H][n_rows];
 * O out: [B][H][n_rows][d].  Rows with cnt = 0 give zeros.
 */
int ref_sparse_attn(const ref_params* p, const double* Q, const double* K,
                    const double* V, const int32_t* idx, const int32_t* cnt,
                    const int32_t* rows, int32_t n_rows, int32_t L, double* O) {
  const int64_t T = p->T, d = p->d;
  if (!rows) n_rows = p->T;
  double* s = (double*)malloc(sizeof(double) * (L > 0 ? L : 1));
  if (!s) return -1;
  for (int64_t bh = 0; bh < (int64_t)p->B * p->H; ++bh) {
    const double* Qh = Q + bh * T * d;
    const double* Kh = K + bh * T * d;
    const double* Vh = V + bh * T * d;
    for (int32_t r = 0; r < n_rows; ++r) {
      const int64_t row = bh * (int64_t)n_rows + r;
      const int64_t t = row_at(rows, r);
      const int32_t* irow = idx + row * L;
      const int64_t n = cnt[row];
      double* Orow = O + row * d;
      for (int64_t e = 0; e < d; ++e) Orow[e] = 0.0;
      if (n <= 0) continue;
      double smax = -INFINITY;
      for (int64_t x = 0; x < n; ++x) {
        const double* kj = Kh + (int64_t)irow[x] * d;
        double dot = 0.0;
        for (int64_t e = 0; e < d; ++e) dot += Qh[t * d + e] * kj[e];
        s[x] = p->scale * dot;
        if (s[x] > smax) smax = s[x];
      }
      double z = 0.0;
      for (int64_t x = 0; x < n; ++x) { s[x] = exp(s[x] - smax); z += s[x]; }
      for (int64_t x = 0; x < n; ++x) {
        const double pj = s[x] / z;
        const double* vj = Vh + (int64_t)irow[x] * d;
        for (int64_t e = 0; e < d; ++e) Orow[e] += pj * vj[e];
      }
    }
  }
  free(s);
  return 0;
}

/* ---- output mixing (Sec. 3.1.1 "Output Calculation") ------------------------ */
/*
 * C_sea = s_mix * (s_prob * C) + (1 - s_mix) * C_avg, row by row.
 *   C: [B][H][T][d] sparse-attention output; s_prob (may be NULL = 1) rescales the sparse
 *   probabilities A* = s_prob * sigma(...), which by linearity rescales C; s_mix: [B][H][T].
 *   Bidirectional: importance i^ = mean over the active rows of A_hat (R^K), stretched to the
 *   keys by nearest neighbour (i_j = i^[floor(j K / T)]), C_avg = weighted average of the active
 *   value rows with weights i (one vector per head).  Causal: C_avg[t] = mean of v_0..v_t.
 *   The scalers are learned in the paper; here the caller supplies them.
 */
int ref_output_mix(const ref_params* p, const double* C, const double* V, const double* A_hat,
                   const double* s_prob, const double* s_mix, const int32_t* seq_len, double* O) {
  const int64_t T = p->T, d = p->d, KK = p->K;
  double* ihat = (double*)malloc(sizeof(double) * KK);
  double* avg = (double*)malloc(sizeof(double) * d);
  if (!ihat || !avg) return -1;
  for (int64_t bh = 0; bh < (int64_t)p->B * p->H; ++bh) {
    const int64_t len = seq_len ? seq_len[bh / p->H] : T;
    const double* Ch = C + bh * T * d;
    const double* Vh = V + bh * T * d;
    double* Oh = O + bh * T * d;
    for (int64_t e = 0; e < d; ++e) avg[e] = 0.0;
    if (!p->causal) {
      for (int64_t c = 0; c < KK; ++c) ihat[c] = 0.0;
      for (int64_t t = 0; t < len; ++t)
        for (int64_t c = 0; c < KK; ++c) ihat[c] += A_hat[(bh * T + t) * KK + c];
      for (int64_t c = 0; c < KK; ++c) ihat[c] /= (len > 0 ? (double)len : 1.0);
      double wsum = 0.0;
      for (int64_t j = 0; j < len; ++j) {
        const double wj = ihat[bucket_of(j, T, KK)];
        wsum += wj;
        for (int64_t e = 0; e < d; ++e) avg[e] += wj * Vh[j * d + e];
      }
      for (int64_t e = 0; e < d; ++e) avg[e] = wsum > 0.0 ? avg[e] / wsum : 0.0;
    }
    for (int64_t t = 0; t < T; ++t) {
      if (t >= len) {
        for (int64_t e = 0; e < d; ++e) Oh[t * d + e] = 0.0;
        continue;
      }
      if (p->causal)  /* running sum of the values; the mean divides by the count t + 1 */
        for (int64_t e = 0; e < d; ++e) avg[e] += Vh[t * d + e];
      const double sm = s_mix[bh * T + t], sp = s_prob ? s_prob[bh * T + t] : 1.0;
      for (int64_t e = 0; e < d; ++e) {
        const double ca = p->causal ? avg[e] / (double)(t + 1) : avg[e];
        Oh[t * d + e] = sm * sp * Ch[t * d + e] + (1.0 - sm) * ca;
      }
    }
  }
  free(ihat); free(avg);
  return 0;
}

/* ---- a7: the whole forward, one head range at a time ---------------------- */
/*
 * Runs a1..a6 for heads [head_lo, head_hi) of the flattened B*H axis, in
 * parallel over heads when built with OpenMP.  Outputs are laid out as in the
 * stage functions; A_hat, sel, idx, cnt may be NULL when not wanted.
 * Returns the number of threads used (>= 1) or a negative error.
 */
#ifdef _OPENMP
#include <omp.h>
#endif

int ref_forward(const ref_params* p, const double* Q, const double* K,
                const double* V, const double* W, const int32_t* seq_len,
                const int32_t* rows, int32_t n_rows, int32_t head_lo,
                int32_t head_hi, double* O, double* A_hat, int32_t* sel,
                int32_t* idx, int32_t* cnt, int32_t n_threads) {
  const int64_t T = p->T, d = p->d, KK = p->K;
  if (!rows) n_rows = p->T;
  const int64_t L = ref_row_stride(p), S = ref_sel_stride(p);
  /* unit of independent work: one head (per-query) or one batch element (causal-per-batch) */
  const int32_t G = p->grouping == 0 ? 1 : p->H;
  if (head_lo % G != 0 || head_hi % G != 0) return -2;
  int used = 1, err = 0;
#ifdef _OPENMP
  if (n_threads > 0) omp_set_num_threads(n_threads);
#pragma omp parallel
  {
#pragma omp single
    used = omp_get_num_threads();
#pragma omp for schedule(dynamic, 1)
#endif
    for (int32_t u = head_lo / G; u < head_hi / G; ++u) {
      const int32_t bh = u * G;  /* first head of the unit */
      ref_params q = *p;
      q.B = 1; q.H = G;
      const int32_t b = bh / p->H;
      const int32_t* sl = seq_len ? seq_len + b : NULL;
      const int64_t rowbase = (int64_t)bh * n_rows;
      const size_t nr = (size_t)G * n_rows;
      double* Ah = (double*)malloc(sizeof(double) * nr * KK);
      int32_t* ih = (int32_t*)malloc(sizeof(int32_t) * nr * (L > 0 ? L : 1));
      int32_t* ch = (int32_t*)malloc(sizeof(int32_t) * nr);
      if (!Ah || !ih || !ch) { err = -1; free(Ah); free(ih); free(ch); continue; }
      ref_estimate(&q, Q + (int64_t)bh * T * d, K + (int64_t)bh * T * d, W, sl, rows, n_rows, Ah);
      ref_topk_mask(&q, Ah, sl, rows, n_rows, sel ? sel + rowbase * S : NULL, ih, ch);
      ref_sparse_attn(&q, Q + (int64_t)bh * T * d, K + (int64_t)bh * T * d,
                      V + (int64_t)bh * T * d, ih, ch, rows, n_rows, (int32_t)L,
                      O + rowbase * d);
      if (A_hat) memcpy(A_hat + rowbase * KK, Ah, sizeof(double) * nr * KK);
      if (idx) memcpy(idx + rowbase * L, ih, sizeof(int32_t) * nr * L);
      if (cnt) memcpy(cnt + rowbase, ch, sizeof(int32_t) * nr);
      free(Ah); free(ih); free(ch);
    }
#ifdef _OPENMP
  }
#endif
  return err ? err : used;
}
