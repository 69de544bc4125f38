/*
 * fp64 CPU oracle for bidirectional cosine-similarity attention.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * GPU library must compute.  It shares no code with the HIP path and nothing in
 * the product path may call it; only the tests, the smoke check and the
 * benchmark's cpu_baseline leg do.
 *
 * What it follows (Cotten4Rec, section "Model Description"):
 *   - the CosineAttention definition, Sim(Q,K) V with Sim the product of the
 *     row-normalised Q and the transposed row-normalised K       (quadratic form);
 *   - the scaled variant, the same expression times the scalar 1/n^m, here a
 *     scalar `scale` handed in by the caller;
 *   - the reordered variant, Q_hat (K_hat^T V), a d x d state built first
 *     (linear form);
 *   - section "Cosine Similarity and CUDA Kernel": a row x is normalised as
 *     x / sqrt(sum_c x_c^2 + eps), eps INSIDE the square root.
 * Readings where the paper is silent: only Q and K are normalised (V never is);
 * the key-padding mask m_j in {0,1} removes key/value row j from the sum and
 * masks nothing on the query side; the backward is the chain rule applied to
 * the expressions above (the paper prints none).
 *
 * The learnable normaliser of the scaled variant (same section, the scaled
 * CosineAttention): s = 1 / n^m with a learnable exponent m.  Here one m per head
 * and one n per sequence (its valid length, or the padded length), so slice
 * (b,h) has s_bh = n_b^(-m_h).  cotten_oracle_normaliser evaluates it,
 * cotten_oracle_scaled_fwd / _bwd take one s per slice, the backward also
 * returns d/d(log s_bh) = sum_i dO_i . O_i (O is linear in s), and
 * cotten_oracle_normaliser_bwd turns that into dm_h = -sum_b ln(n_b) dlog_s_bh.
 *
 * The causal variant (what the paper's bidirectional model removes, "no causal mask": row i
 * attends keys j <= i only) is stated here from its definition with all N x N cosines,
 * cotten_oracle_causal_fwd / _bwd, so that the prefix-state kernels can be checked against
 * something that has no prefix state in it.
 *
 * The ELU + 1 feature map (section "Linear Attention Models": the linear-attention comparison
 * model applies ELU(x) + 1 element-wise to queries and keys, collapses keys and values into a
 * d x d product and multiplies the transformed queries with it).  Stated here from the N x N
 * scores A_ij = phi(q_i) . phi(k_j), O_i = scale * sum_j m_j A_ij v_j, phi(x) = x + 1 for x > 0
 * and exp(x) otherwise (ELU with alpha = 1), cotten_oracle_elu_fwd / _bwd.  Reading: the
 * section names no normalising denominator, so none is applied beyond the scalar `scale`.
 *
 * Pins (tests/test_oracle_pins.py): linear == quadratic on small inputs;
 * closed forms; unit norms; masked-key invariance; permutation equivariance;
 * fp64 autograd of the library expression; central finite differences and an
 * independently derived n x n route for the backward.
 *
 * Layout: Q,K,V,O,dO,dQ,dK,dV are [B,H,N,d] row-major doubles; mask is [B,N]
 * bytes (1 = valid key) or NULL for "all valid".  Slices (b,h) are independent
 * and are spread over OpenMP threads; inside a slice every loop is sequential.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int cotten_oracle_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* r(x) = sqrt(sum_c x_c^2 + eps) */
static double row_norm(const double* x, int d, double eps) {
  double ss = 0.0;
  for (int c = 0; c < d; ++c) ss += x[c] * x[c];
  return sqrt(ss + eps);
}

static int key_valid(const uint8_t* mask, int b, int N, int j) {
  return mask == NULL ? 1 : (mask[(size_t)b * N + j] != 0);
}

/* Definition: O_i = scale * sum_j m_j cos(q_i, k_j) v_j, forming every one of
 * the N x N cosines explicitly. */
void cotten_oracle_fwd_quadratic(const double* Q, const double* K, const double* V,
                                 const uint8_t* mask, double* O, int B, int H, int N,
                                 int d, double scale, double eps) {
#pragma omp parallel for schedule(dynamic)
  for (int bh = 0; bh < B * H; ++bh) {
    const int b = bh / H;
    const size_t off = (size_t)bh * N * d;
    const double *q = Q + off, *k = K + off, *v = V + off;
    double* o = O + off;
    double* rk = (double*)malloc(sizeof(double) * (size_t)N);
    for (int j = 0; j < N; ++j) rk[j] = row_norm(k + (size_t)j * d, d, eps);
    for (int i = 0; i < N; ++i) {
      const double rq = row_norm(q + (size_t)i * d, d, eps);
      for (int c = 0; c < d; ++c) o[(size_t)i * d + c] = 0.0;
      for (int j = 0; j < N; ++j) {
        if (!key_valid(mask, b, N, j)) continue;
        double dot = 0.0;
        for (int a = 0; a < d; ++a) dot += q[(size_t)i * d + a] * k[(size_t)j * d + a];
        const double cosine = dot / (rq * rk[j]);
        for (int c = 0; c < d; ++c) o[(size_t)i * d + c] += cosine * v[(size_t)j * d + c];
      }
      for (int c = 0; c < d; ++c) o[(size_t)i * d + c] *= scale;
    }
    free(rk);
  }
}

/* S[a][c] = sum_j m_j khat_j[a] v_j[c]   (the d x d state of the reordered form) */
static void build_state(const double* k, const double* v, const uint8_t* mask, int b,
                        int N, int d, double eps, double* S) {
  for (int a = 0; a < d * d; ++a) S[a] = 0.0;
  for (int j = 0; j < N; ++j) {
    if (!key_valid(mask, b, N, j)) continue;
    const double rk = row_norm(k + (size_t)j * d, d, eps);
    for (int a = 0; a < d; ++a) {
      const double kh = k[(size_t)j * d + a] / rk;
      for (int c = 0; c < d; ++c) S[(size_t)a * d + c] += kh * v[(size_t)j * d + c];
    }
  }
}

/* The state of the reordered form on its own, S[b,h] = Khat^T V under the key mask
 * ([B,H,d,d]): what a forward call may hand to its backward call. */
void cotten_oracle_state(const double* K, const double* V, const uint8_t* mask, double* S,
                         int B, int H, int N, int d, double eps) {
#pragma omp parallel for schedule(dynamic)
  for (int bh = 0; bh < B * H; ++bh) {
    const size_t off = (size_t)bh * N * d;
    build_state(K + off, V + off, mask, bh / H, N, d, eps, S + (size_t)bh * d * d);
  }
}

/* Reordered form: S = Khat^T V under the key mask, then O_i = scale * qhat_i S. */
void cotten_oracle_fwd_linear(const double* Q, const double* K, const double* V,
                              const uint8_t* mask, double* O, int B, int H, int N, int d,
                              double scale, double eps) {
#pragma omp parallel for schedule(dynamic)
  for (int bh = 0; bh < B * H; ++bh) {
    const int b = bh / H;
    const size_t off = (size_t)bh * N * d;
    const double *q = Q + off, *k = K + off, *v = V + off;
    double* o = O + off;
    double* S = (double*)malloc(sizeof(double) * (size_t)d * d);
    build_state(k, v, mask, b, N, d, eps, S);
    for (int i = 0; i < N; ++i) {
      const double rq = row_norm(q + (size_t)i * d, d, eps);
      for (int c = 0; c < d; ++c) {
        double acc = 0.0;
        for (int a = 0; a < d; ++a) acc += (q[(size_t)i * d + a] / rq) * S[(size_t)a * d + c];
        o[(size_t)i * d + c] = scale * acc;
      }
    }
    free(S);
  }
}

/* Backward of the reordered form, chain rule step by step.  With
 *   xhat = x / r(x),  r = sqrt(|x|^2 + eps)   =>   dx = (dxhat - xhat (xhat . dxhat)) / r
 * (exact also for eps > 0, because d r / d x = x / r):
 *   dS      = scale * sum_i qhat_i^T dO_i          (all N query rows)
 *   dqhat_i = scale * dO_i S^T
 *   dV_j    = m_j * khat_j dS
 *   dkhat_j = m_j * v_j dS^T
 * dK_j and dV_j are exactly zero at masked keys. */
void cotten_oracle_bwd(const double* Q, const double* K, const double* V,
                       const uint8_t* mask, const double* dO, double* dQ, double* dK,
                       double* dV, int B, int H, int N, int d, double scale, double eps) {
#pragma omp parallel for schedule(dynamic)
  for (int bh = 0; bh < B * H; ++bh) {
    const int b = bh / H;
    const size_t off = (size_t)bh * N * d;
    const double *q = Q + off, *k = K + off, *v = V + off, *go = dO + off;
    double *gq = dQ + off, *gk = dK + off, *gv = dV + off;
    double* S = (double*)malloc(sizeof(double) * (size_t)d * d);
    double* dS = (double*)malloc(sizeof(double) * (size_t)d * d);
    double* xh = (double*)malloc(sizeof(double) * (size_t)d);
    double* gh = (double*)malloc(sizeof(double) * (size_t)d);
    build_state(k, v, mask, b, N, d, eps, S);

    for (int a = 0; a < d * d; ++a) dS[a] = 0.0;
    for (int i = 0; i < N; ++i) {
      const double rq = row_norm(q + (size_t)i * d, d, eps);
      for (int a = 0; a < d; ++a) {
        const double qh = q[(size_t)i * d + a] / rq;
        for (int c = 0; c < d; ++c) dS[(size_t)a * d + c] += scale * qh * go[(size_t)i * d + c];
      }
    }

    for (int i = 0; i < N; ++i) {
      const double rq = row_norm(q + (size_t)i * d, d, eps);
      double proj = 0.0;
      for (int a = 0; a < d; ++a) {
        xh[a] = q[(size_t)i * d + a] / rq;
        double acc = 0.0;
        for (int c = 0; c < d; ++c) acc += go[(size_t)i * d + c] * S[(size_t)a * d + c];
        gh[a] = scale * acc;
        proj += xh[a] * gh[a];
      }
      for (int a = 0; a < d; ++a) gq[(size_t)i * d + a] = (gh[a] - xh[a] * proj) / rq;
    }

    for (int j = 0; j < N; ++j) {
      if (!key_valid(mask, b, N, j)) {
        for (int a = 0; a < d; ++a) gk[(size_t)j * d + a] = gv[(size_t)j * d + a] = 0.0;
        continue;
      }
      const double rk = row_norm(k + (size_t)j * d, d, eps);
      for (int a = 0; a < d; ++a) xh[a] = k[(size_t)j * d + a] / rk;
      for (int c = 0; c < d; ++c) {
        double acc = 0.0;
        for (int a = 0; a < d; ++a) acc += xh[a] * dS[(size_t)a * d + c];
        gv[(size_t)j * d + c] = acc;
      }
      double proj = 0.0;
      for (int a = 0; a < d; ++a) {
        double acc = 0.0;
        for (int c = 0; c < d; ++c) acc += v[(size_t)j * d + c] * dS[(size_t)a * d + c];
        gh[a] = acc;
        proj += xh[a] * gh[a];
      }
      for (int a = 0; a < d; ++a) gk[(size_t)j * d + a] = (gh[a] - xh[a] * proj) / rk;
    }
    free(S); free(dS); free(xh); free(gh);
  }
}

/* ---- the learnable normaliser 1 / n^m of the scaled variant ----------------- */

/* s[b*H+h] = n_b^(-m_h) */
void cotten_oracle_normaliser(const double* m, const double* n, double* s, int B, int H) {
  for (int b = 0; b < B; ++b)
    for (int h = 0; h < H; ++h) s[(size_t)b * H + h] = pow(n[b], -m[h]);
}

/* Forward with one scalar per slice: the reordered form, slice by slice. */
void cotten_oracle_scaled_fwd(const double* Q, const double* K, const double* V,
                              const uint8_t* mask, const double* s, double* O, int B, int H,
                              int N, int d, double eps) {
  for (int bh = 0; bh < B * H; ++bh) {
    const int b = bh / H;
    const size_t off = (size_t)bh * N * d;
    const uint8_t* mrow = mask == NULL ? NULL : mask + (size_t)b * N;
    cotten_oracle_fwd_linear(Q + off, K + off, V + off, mrow, O + off, 1, 1, N, d, s[bh], eps);
  }
}

/* Backward with one scalar per slice.  dQ, dK, dV as in cotten_oracle_bwd with
 * scale = s_bh.  O = s * U with U free of s, hence
 *   d loss / d log s_bh = s_bh * sum_i dO_i . U_i = sum_i dO_i . O_i. */
void cotten_oracle_scaled_bwd(const double* Q, const double* K, const double* V,
                              const uint8_t* mask, const double* s, const double* dO,
                              double* dQ, double* dK, double* dV, double* dlog_s, int B,
                              int H, int N, int d, double eps) {
  double* O = (double*)malloc(sizeof(double) * (size_t)N * d);
  for (int bh = 0; bh < B * H; ++bh) {
    const int b = bh / H;
    const size_t off = (size_t)bh * N * d;
    const uint8_t* mrow = mask == NULL ? NULL : mask + (size_t)b * N;
    cotten_oracle_bwd(Q + off, K + off, V + off, mrow, dO + off, dQ + off, dK + off, dV + off,
                      1, 1, N, d, s[bh], eps);
    cotten_oracle_fwd_linear(Q + off, K + off, V + off, mrow, O, 1, 1, N, d, s[bh], eps);
    double acc = 0.0;
    for (size_t e = 0; e < (size_t)N * d; ++e) acc += dO[off + e] * O[e];
    dlog_s[bh] = acc;
  }
  free(O);
}

/* s_bh = exp(-m_h ln n_b)  =>  d log s_bh / d m_h = -ln n_b  =>
 * dm_h = -sum_b ln(n_b) * dlog_s[b*H+h] */
void cotten_oracle_normaliser_bwd(const double* dlog_s, const double* n, double* dm, int B,
                                  int H) {
  for (int h = 0; h < H; ++h) {
    double acc = 0.0;
    for (int b = 0; b < B; ++b) acc += log(n[b]) * dlog_s[(size_t)b * H + h];
    dm[h] = -acc;
  }
}

/* ---- causal variant: row i sees keys j <= i ---------------------------------- */

/* P[i][j] = cos(q_i, k_j) for j <= i and valid key j, else 0 (row-major N x N). */
static void causal_cosines(const double* q, const double* k, const uint8_t* mask, int b, int N,
                           int d, double eps, double* P, double* rq, double* rk) {
  for (int i = 0; i < N; ++i) {
    rq[i] = row_norm(q + (size_t)i * d, d, eps);
    rk[i] = row_norm(k + (size_t)i * d, d, eps);
  }
  for (int i = 0; i < N; ++i)
    for (int j = 0; j < N; ++j) {
      double p = 0.0;
      if (j <= i && key_valid(mask, b, N, j)) {
        for (int a = 0; a < d; ++a) p += q[(size_t)i * d + a] * k[(size_t)j * d + a];
        p /= rq[i] * rk[j];
      }
      P[(size_t)i * N + j] = p;
    }
}

/* O_i = scale * sum_{j <= i} m_j cos(q_i, k_j) v_j */
void cotten_oracle_causal_fwd(const double* Q, const double* K, const double* V,
                              const uint8_t* mask, double* O, int B, int H, int N, int d,
                              double scale, double eps) {
#pragma omp parallel for schedule(dynamic)
  for (int bh = 0; bh < B * H; ++bh) {
    const size_t off = (size_t)bh * N * d;
    double* P = (double*)malloc(sizeof(double) * (size_t)N * N);
    double* rq = (double*)malloc(sizeof(double) * N);
    double* rk = (double*)malloc(sizeof(double) * N);
    causal_cosines(Q + off, K + off, mask, bh / H, N, d, eps, P, rq, rk);
    for (int i = 0; i < N; ++i)
      for (int c = 0; c < d; ++c) {
        double acc = 0.0;
        for (int j = 0; j <= i; ++j) acc += P[(size_t)i * N + j] * V[off + (size_t)j * d + c];
        O[off + (size_t)i * d + c] = scale * acc;
      }
    free(P); free(rq); free(rk);
  }
}

/* Backward of the same expression through the N x N matrix: with P as above and
 * G[i][j] = scale * (dO_i . v_j) on the same support,
 *   dV_j = scale * sum_i P[i][j] dO_i,  dqhat_i = sum_j G[i][j] khat_j,
 *   dkhat_j = sum_i G[i][j] qhat_i,  and  dx = (dxhat - xhat (xhat . dxhat)) / r. */
void cotten_oracle_causal_bwd(const double* Q, const double* K, const double* V,
                              const uint8_t* mask, const double* dO, double* dQ, double* dK,
                              double* dV, int B, int H, int N, int d, double scale,
                              double eps) {
#pragma omp parallel for schedule(dynamic)
  for (int bh = 0; bh < B * H; ++bh) {
    const int b = bh / H;
    const size_t off = (size_t)bh * N * d;
    const double *q = Q + off, *k = K + off, *v = V + off, *go = dO + off;
    double* P = (double*)malloc(sizeof(double) * (size_t)N * N);
    double* G = (double*)malloc(sizeof(double) * (size_t)N * N);
    double* rq = (double*)malloc(sizeof(double) * N);
    double* rk = (double*)malloc(sizeof(double) * N);
    double* xh = (double*)malloc(sizeof(double) * d);
    double* gh = (double*)malloc(sizeof(double) * d);
    causal_cosines(q, k, mask, b, N, d, eps, P, rq, rk);
    for (int i = 0; i < N; ++i)
      for (int j = 0; j < N; ++j) {
        double g = 0.0;
        if (j <= i && key_valid(mask, b, N, j)) {
          for (int c = 0; c < d; ++c) g += go[(size_t)i * d + c] * v[(size_t)j * d + c];
          g *= scale;
        }
        G[(size_t)i * N + j] = g;
      }
    for (int j = 0; j < N; ++j)
      for (int c = 0; c < d; ++c) {
        double acc = 0.0;
        for (int i = j; i < N; ++i) acc += P[(size_t)i * N + j] * go[(size_t)i * d + c];
        dV[off + (size_t)j * d + c] = scale * acc;
      }
    for (int i = 0; i < N; ++i) {
      double proj = 0.0;
      for (int a = 0; a < d; ++a) {
        xh[a] = q[(size_t)i * d + a] / rq[i];
        double acc = 0.0;
        for (int j = 0; j <= i; ++j) acc += G[(size_t)i * N + j] * k[(size_t)j * d + a] / rk[j];
        gh[a] = acc;
        proj += xh[a] * acc;
      }
      for (int a = 0; a < d; ++a) dQ[off + (size_t)i * d + a] = (gh[a] - xh[a] * proj) / rq[i];
    }
    for (int j = 0; j < N; ++j) {
      double proj = 0.0;
      for (int a = 0; a < d; ++a) {
        xh[a] = k[(size_t)j * d + a] / rk[j];
        double acc = 0.0;
        for (int i = j; i < N; ++i) acc += G[(size_t)i * N + j] * q[(size_t)i * d + a] / rq[i];
        gh[a] = acc;
        proj += xh[a] * acc;
      }
      for (int a = 0; a < d; ++a) dK[off + (size_t)j * d + a] = (gh[a] - xh[a] * proj) / rk[j];
    }
    free(P); free(G); free(rq); free(rk); free(xh); free(gh);
  }
}

/* ---- ELU + 1 feature map ("Linear Attention Models") ---------------------------------- */

/* phi(x) = ELU(x) + 1 with alpha = 1: x + 1 for x > 0, exp(x) otherwise; always positive. */
static double elu1(double x) { return x > 0.0 ? x + 1.0 : exp(x); }
/* its derivative: 1 for x > 0, exp(x) otherwise */
static double elu1_prime(double x) { return x > 0.0 ? 1.0 : exp(x); }

/* A[i][j] = m_j * phi(q_i) . phi(k_j) */
static void elu_scores(const double* q, const double* k, const uint8_t* mask, int b, int N,
                       int d, double* A) {
  for (int i = 0; i < N; ++i)
    for (int j = 0; j < N; ++j) {
      double a = 0.0;
      if (key_valid(mask, b, N, j))
        for (int c = 0; c < d; ++c) a += elu1(q[(size_t)i * d + c]) * elu1(k[(size_t)j * d + c]);
      A[(size_t)i * N + j] = a;
    }
}

/* O_i = scale * sum_j m_j (phi(q_i) . phi(k_j)) v_j */
void cotten_oracle_elu_fwd(const double* Q, const double* K, const double* V,
                           const uint8_t* mask, double* O, int B, int H, int N, int d,
                           double scale) {
#pragma omp parallel for schedule(dynamic)
  for (int bh = 0; bh < B * H; ++bh) {
    const size_t off = (size_t)bh * N * d;
    double* A = (double*)malloc(sizeof(double) * (size_t)N * N);
    elu_scores(Q + off, K + off, mask, bh / H, N, d, A);
    for (int i = 0; i < N; ++i)
      for (int c = 0; c < d; ++c) {
        double acc = 0.0;
        for (int j = 0; j < N; ++j) acc += A[(size_t)i * N + j] * V[off + (size_t)j * d + c];
        O[off + (size_t)i * d + c] = scale * acc;
      }
    free(A);
  }
}

/* Backward through the N x N scores: with G[i][j] = scale * m_j * (dO_i . v_j),
 *   dV_j = scale * sum_i A[i][j] dO_i,
 *   dq_i = phi'(q_i) * sum_j G[i][j] phi(k_j),   dk_j = phi'(k_j) * sum_i G[i][j] phi(q_i)
 * (element-wise products with phi').  Masked keys get exact zeros. */
void cotten_oracle_elu_bwd(const double* Q, const double* K, const double* V,
                           const uint8_t* mask, const double* dO, double* dQ, double* dK,
                           double* dV, int B, int H, int N, int d, double scale) {
#pragma omp parallel for schedule(dynamic)
  for (int bh = 0; bh < B * H; ++bh) {
    const int b = bh / H;
    const size_t off = (size_t)bh * N * d;
    const double *q = Q + off, *k = K + off, *v = V + off, *go = dO + off;
    double* A = (double*)malloc(sizeof(double) * (size_t)N * N);
    double* G = (double*)malloc(sizeof(double) * (size_t)N * N);
    elu_scores(q, k, mask, b, N, d, A);
    for (int i = 0; i < N; ++i)
      for (int j = 0; j < N; ++j) {
        double g = 0.0;
        if (key_valid(mask, b, N, j)) {
          for (int c = 0; c < d; ++c) g += go[(size_t)i * d + c] * v[(size_t)j * d + c];
          g *= scale;
        }
        G[(size_t)i * N + j] = g;
      }
    for (int j = 0; j < N; ++j)
      for (int c = 0; c < d; ++c) {
        double acc = 0.0;
        for (int i = 0; i < N; ++i) acc += A[(size_t)i * N + j] * go[(size_t)i * d + c];
        dV[off + (size_t)j * d + c] = scale * acc;
      }
    for (int i = 0; i < N; ++i)
      for (int a = 0; a < d; ++a) {
        double acc = 0.0;
        for (int j = 0; j < N; ++j) acc += G[(size_t)i * N + j] * elu1(k[(size_t)j * d + a]);
        dQ[off + (size_t)i * d + a] = elu1_prime(q[(size_t)i * d + a]) * acc;
      }
    for (int j = 0; j < N; ++j)
      for (int a = 0; a < d; ++a) {
        double acc = 0.0;
        for (int i = 0; i < N; ++i) acc += G[(size_t)i * N + j] * elu1(q[(size_t)i * d + a]);
        dK[off + (size_t)j * d + a] = elu1_prime(k[(size_t)j * d + a]) * acc;
      }
    free(A); free(G);
  }
}
