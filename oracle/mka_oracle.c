/*
 * fp64 CPU oracle for FastMKA route-fused attention.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * HIP library is checked against.  It shares no code with the GPU path and the
 * product never calls it; only the test-suite, the smoke check and the
 * CPU-baseline leg of the benchmark may load it.
 *
 * What is computed (paper: Algorithm 2 "FastMKA", steps 5-9, with Attention
 * defined by Eq. (1) of the "Hierarchical Block-wise MKA Algorithm" section
 * and the scale tau of Eq. (3)):
 *
 *   router   g[t,l]   = b_r[l] + sum_k Q[t,k] W_r[k,l]          (Alg. 2 step 5)
 *            lam[t,:] = softmax_3(g[t,:]),  idx[t] = argmax_l g[t,l]
 *   fusion   Kf[j,:]  = sum_l [j < len_l] G[j,l] K_l[j,:]       (Alg. 2 step 6-7)
 *            Vf[j,:]  likewise
 *   attention over the fused stream, causal, bottom-right aligned
 *            s[t,j] = tau Q[t].Kf[j],  p = softmax_j(s),  O = p Vf   (Alg. 2 step 9, Eq. 1)
 *   decode   = append one slot (Alg. 2 step 8) then one query row of the above
 *   backward = chain rule through all of the above (the paper prints none)
 *
 * Readings taken where the paper is silent: the gate of slot j is computed
 * from the query of the token that produced slot j and scales that slot's
 * memory entries (token-aligned product of Alg. 2 step 6); the routing "MLP"
 * is one linear map W_r[d,3] plus bias; a level that has no entry at a slot
 * contributes the zero vector (Alg. 1's M_3 <- 0) and the gates are not
 * renormalised; the fusion is applied to already-projected K/V, which equals
 * fusing before the projection because the projection is linear.
 *
 * Every tensor is a dense row-major array of doubles on the host:
 *   Q,O,dO,dQ [B,H,Tq,d]   K_l,V_l,dK_l,dV_l [B,H,S,d]   G [B,H,S,3]
 *   W_r [d,3]  b_r [3]  LSE [B,H,Tq]  idx [B,H,Tq] (int32)
 * The (b,h) pairs are independent and are spread over OpenMP threads; inside a
 * pair there is no blocking, fusion or reordering beyond the definitions.
 *
 * Pins (tests/test_oracle_*.py): brute-force nested sums on tiny shapes,
 * one-hot gates == textbook causal attention, equal memories == textbook
 * attention, zero keys == prefix means, rows of p summing to one, block-size
 * independence of the max-shift recursion, decode == last prefill row,
 * finite differences and an autograd second opinion for the backward.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int mka_oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ---- router: Alg. 2 step 5 ------------------------------------------------
 * Logits are an fma chain in ascending k starting from the bias, so that an
 * implementation using the same chain in fp64 gets bit-identical logits and
 * therefore the same argmax.  Ties go to the lowest level.  Rows of G for the
 * Tq new slots (slots S-Tq .. S-1) are written; older slots are left alone. */
void mka_oracle_route(const double* Q, const double* W_r, const double* b_r,
                      int B, int H, int Tq, int S, int d, double* G, int32_t* idx) {
  long n = (long)B * H;
#pragma omp parallel for schedule(static)
  for (long bh = 0; bh < n; ++bh) {
    for (int t = 0; t < Tq; ++t) {
      const double* q = Q + ((size_t)bh * Tq + t) * d;
      double g[3];
      for (int l = 0; l < 3; ++l) {
        double acc = b_r ? b_r[l] : 0.0;
        for (int k = 0; k < d; ++k) acc = fma(q[k], W_r[(size_t)k * 3 + l], acc);
        g[l] = acc;
      }
      int best = 0;
      for (int l = 1; l < 3; ++l)
        if (g[l] > g[best]) best = l;
      double e[3], z = 0.0;
      for (int l = 0; l < 3; ++l) {
        e[l] = exp(g[l] - g[best]);
        z += e[l];
      }
      if (G) {
        double* row = G + ((size_t)bh * S + (S - Tq + t)) * 3;
        for (int l = 0; l < 3; ++l) row[l] = e[l] / z;
      }
      if (idx) idx[(size_t)bh * Tq + t] = best;
    }
  }
}

/* ---- routing variants of the ablation (section "Routing Mechanism Ablation", table
 * "Routing mechanism ablation"): the paper names them without formulas.  Reading: mode 0 = the
 * learned soft gates of step 5; mode 1 = fixed lam = 1/3 for every level; mode 2 = hard top-2: the
 * level with the smallest logit is dropped and the other two soft gates are renormalised to sum
 * 1; mode 3 = hard top-1: the gate is the indicator of the largest logit.  Ties go to the lower
 * level (the argmax keeps the lowest index, the dropped level is the highest index among equal
 * minima). */
void mka_oracle_route_variant(const double* Q, const double* W_r, const double* b_r, int mode,
                              int B, int H, int Tq, int S, int d, double* G, int32_t* idx) {
  long n = (long)B * H;
#pragma omp parallel for schedule(static)
  for (long bh = 0; bh < n; ++bh) {
    for (int t = 0; t < Tq; ++t) {
      const double* q = Q + ((size_t)bh * Tq + t) * d;
      double g[3];
      for (int l = 0; l < 3; ++l) {
        double acc = b_r ? b_r[l] : 0.0;
        for (int k = 0; k < d; ++k) acc = fma(q[k], W_r[(size_t)k * 3 + l], acc);
        g[l] = acc;
      }
      int best = 0, drop = 0;
      for (int l = 1; l < 3; ++l) {
        if (g[l] > g[best]) best = l;
        if (g[l] <= g[drop]) drop = l;
      }
      double lam[3];
      if (mode == 1) {
        lam[0] = lam[1] = lam[2] = 1.0 / 3.0;
      } else if (mode == 3) {
        for (int l = 0; l < 3; ++l) lam[l] = (l == best) ? 1.0 : 0.0;
      } else {
        double e[3], z = 0.0;
        for (int l = 0; l < 3; ++l) {
          e[l] = (mode == 2 && l == drop) ? 0.0 : exp(g[l] - g[best]);
          z += e[l];
        }
        for (int l = 0; l < 3; ++l) lam[l] = e[l] / z;
      }
      if (G) {
        double* row = G + ((size_t)bh * S + (S - Tq + t)) * 3;
        for (int l = 0; l < 3; ++l) row[l] = lam[l];
      }
      if (idx) idx[(size_t)bh * Tq + t] = best;
    }
  }
}

/* ---- fusion: Alg. 2 step 6 (token-wise gate-weighted mix) ----------------- */
void mka_oracle_fuse(const double* X1, const double* X2, const double* X3, const double* G,
                     const int32_t* len, int B, int H, int S, int d, double* Xf) {
  const double* X[3] = {X1, X2, X3};
  long n = (long)B * H;
#pragma omp parallel for schedule(static)
  for (long bh = 0; bh < n; ++bh) {
    for (int j = 0; j < S; ++j) {
      size_t row = (size_t)bh * S + j;
      for (int k = 0; k < d; ++k) {
        double acc = 0.0;
        for (int l = 0; l < 3; ++l)
          if (X[l] && j < len[l]) acc += G[row * 3 + l] * X[l][row * d + k];
        Xf[row * d + k] = acc;
      }
    }
  }
}

static int visible_upto(int t, int Tq, int S, int causal) {
  /* number of visible slots for query row t: bottom-right aligned causal mask */
  return causal ? (t + (S - Tq) + 1) : S;
}

/* ---- attention: Eq. (1), direct two-pass softmax per row ------------------
 * P (optional) receives the full probability matrix [B,H,Tq,S] (zeros where
 * masked); only sensible for tiny shapes. */
void mka_oracle_attn_fwd(const double* Q, const double* Kf, const double* Vf, int B, int H, int Tq,
                         int S, int d, int causal, double tau, double* O, double* LSE, double* P) {
  long n = (long)B * H;
#pragma omp parallel for schedule(dynamic, 1)
  for (long bh = 0; bh < n; ++bh) {
    double* s = (double*)malloc(sizeof(double) * (size_t)S);
    for (int t = 0; t < Tq; ++t) {
      const double* q = Q + ((size_t)bh * Tq + t) * d;
      int nv = visible_upto(t, Tq, S, causal);
      double m = -INFINITY;
      for (int j = 0; j < nv; ++j) {
        const double* kf = Kf + ((size_t)bh * S + j) * d;
        double acc = 0.0;
        for (int k = 0; k < d; ++k) acc += q[k] * kf[k];
        s[j] = tau * acc;
        if (s[j] > m) m = s[j];
      }
      double z = 0.0;
      for (int j = 0; j < nv; ++j) {
        s[j] = exp(s[j] - m);
        z += s[j];
      }
      double* o = O + ((size_t)bh * Tq + t) * d;
      for (int k = 0; k < d; ++k) o[k] = 0.0;
      for (int j = 0; j < nv; ++j) {
        double p = s[j] / z;
        const double* vf = Vf + ((size_t)bh * S + j) * d;
        for (int k = 0; k < d; ++k) o[k] += p * vf[k];
        if (P) P[((size_t)bh * Tq + t) * S + j] = p;
      }
      if (P)
        for (int j = nv; j < S; ++j) P[((size_t)bh * Tq + t) * S + j] = 0.0;
      if (LSE) LSE[(size_t)bh * Tq + t] = m + log(z);
    }
    free(s);
  }
}

/* ---- gated mixture of exponentiated scores over the three memories -------
 * (paper: section "Theoretical Formulation: Recursive MKA with Online Softmax",
 * first equation and Theorem "Recursive MKA Computes Gated Mixture Attention"):
 *
 *   O[t] = sum_l lam[t,l] sum_j exp(s_l[t,j]) V_l[j]  /  sum_l lam[t,l] sum_j exp(s_l[t,j])
 *
 * with s_l[t,j] = tau Q[t].K_l[j], the gate indexed by the QUERY row, one
 * normalisation after the mix.  Written out directly: a first pass finds the
 * largest exponent of the row over the levels with a positive gate (only to
 * keep exp() in range; the quotient does not depend on it), a second pass
 * accumulates numerator and denominator.  Level l has S[l] slots (0 = absent)
 * and its own bottom-right aligned causal mask.  lam == NULL means lam = 1 for
 * every level (softmax attention over the concatenation of the memories).
 * LSE[t] = log of the denominator.  Rows that see nothing give O = 0, LSE = -inf. */
void mka_oracle_mixture_fwd(const double* Q, const double* K1, const double* K2, const double* K3,
                            const double* V1, const double* V2, const double* V3,
                            const double* lam, int B, int H, int Tq, const int* S, int d,
                            int causal, double tau, double* O, double* LSE) {
  const double* K[3] = {K1, K2, K3};
  const double* V[3] = {V1, V2, V3};
  long n = (long)B * H;
#pragma omp parallel for schedule(dynamic, 1)
  for (long bh = 0; bh < n; ++bh) {
    for (int t = 0; t < Tq; ++t) {
      const double* q = Q + ((size_t)bh * Tq + t) * d;
      const double* lt = lam ? lam + ((size_t)bh * Tq + t) * 3 : NULL;
      double m = -INFINITY;
      for (int l = 0; l < 3; ++l) {
        if (!K[l] || S[l] <= 0 || (lt && !(lt[l] > 0.0))) continue;
        int nv = visible_upto(t, Tq, S[l], causal);
        for (int j = 0; j < nv; ++j) {
          const double* kr = K[l] + ((size_t)bh * S[l] + j) * d;
          double acc = 0.0;
          for (int k = 0; k < d; ++k) acc += q[k] * kr[k];
          if (tau * acc > m) m = tau * acc;
        }
      }
      double* o = O + ((size_t)bh * Tq + t) * d;
      for (int k = 0; k < d; ++k) o[k] = 0.0;
      double z = 0.0;
      if (m > -INFINITY) {
        for (int l = 0; l < 3; ++l) {
          if (!K[l] || S[l] <= 0 || (lt && !(lt[l] > 0.0))) continue;
          double w = lt ? lt[l] : 1.0;
          int nv = visible_upto(t, Tq, S[l], causal);
          for (int j = 0; j < nv; ++j) {
            const double* kr = K[l] + ((size_t)bh * S[l] + j) * d;
            const double* vr = V[l] + ((size_t)bh * S[l] + j) * d;
            double acc = 0.0;
            for (int k = 0; k < d; ++k) acc += q[k] * kr[k];
            double e = w * exp(tau * acc - m);
            z += e;
            for (int k = 0; k < d; ++k) o[k] += e * vr[k];
          }
        }
        for (int k = 0; k < d; ++k) o[k] /= z;
      }
      if (LSE) LSE[(size_t)bh * Tq + t] = (z > 0.0) ? m + log(z) : -INFINITY;
    }
  }
}

/* ---- attention by the max-shift recursion over KV blocks of Bc slots ------
 * ("Numerical Stability via Max-Shift": running max mu, normaliser z and
 * numerator alpha, both rescaled by exp(mu_old - mu_new) before a block is
 * added).  Exists to check that the blocked schedule reaches Eq. (1). */
void mka_oracle_attn_fwd_blockwise(const double* Q, const double* Kf, const double* Vf, int B,
                                   int H, int Tq, int S, int d, int causal, double tau, int Bc,
                                   double* O, double* LSE) {
  long n = (long)B * H;
#pragma omp parallel for schedule(dynamic, 1)
  for (long bh = 0; bh < n; ++bh) {
    double* alpha = (double*)malloc(sizeof(double) * (size_t)d);
    double* sb = (double*)malloc(sizeof(double) * (size_t)Bc);
    for (int t = 0; t < Tq; ++t) {
      const double* q = Q + ((size_t)bh * Tq + t) * d;
      int nv = visible_upto(t, Tq, S, causal);
      double mu = -INFINITY, z = 0.0;
      for (int k = 0; k < d; ++k) alpha[k] = 0.0;
      for (int j0 = 0; j0 < nv; j0 += Bc) {
        int j1 = j0 + Bc < nv ? j0 + Bc : nv;
        double mu_new = mu;
        for (int j = j0; j < j1; ++j) {
          const double* kf = Kf + ((size_t)bh * S + j) * d;
          double acc = 0.0;
          for (int k = 0; k < d; ++k) acc += q[k] * kf[k];
          sb[j - j0] = tau * acc;
          if (sb[j - j0] > mu_new) mu_new = sb[j - j0];
        }
        double resc = exp(mu - mu_new); /* exp(-inf) = 0 on the first block */
        z *= resc;
        for (int k = 0; k < d; ++k) alpha[k] *= resc;
        for (int j = j0; j < j1; ++j) {
          double e = exp(sb[j - j0] - mu_new);
          const double* vf = Vf + ((size_t)bh * S + j) * d;
          z += e;
          for (int k = 0; k < d; ++k) alpha[k] += e * vf[k];
        }
        mu = mu_new;
      }
      double* o = O + ((size_t)bh * Tq + t) * d;
      for (int k = 0; k < d; ++k) o[k] = alpha[k] / z;
      if (LSE) LSE[(size_t)bh * Tq + t] = mu + log(z);
    }
    free(alpha);
    free(sb);
  }
}

/* ---- whole forward: Alg. 2 steps 6-9 on given gates ----------------------- */
void mka_oracle_fwd(const double* Q, const double* K1, const double* K2, const double* K3,
                    const double* V1, const double* V2, const double* V3, const double* G,
                    const int32_t* len, int B, int H, int Tq, int S, int d, int causal, double tau,
                    double* O, double* LSE) {
  size_t n = (size_t)B * H * S * d;
  double* Kf = (double*)malloc(sizeof(double) * n);
  double* Vf = (double*)malloc(sizeof(double) * n);
  mka_oracle_fuse(K1, K2, K3, G, len, B, H, S, d, Kf);
  mka_oracle_fuse(V1, V2, V3, G, len, B, H, S, d, Vf);
  mka_oracle_attn_fwd(Q, Kf, Vf, B, H, Tq, S, d, causal, tau, O, LSE, NULL);
  free(Kf);
  free(Vf);
}

/* ---- decode: Alg. 2 step 8 (append) then step 9 for the one new row -------
 * Caches are [B,H,cap_l,d] (gate cache [B,H,capG,3]); len[l] = valid slots of
 * level l before the call, updated on return.  The new token's slot is
 * j_new = max_l len[l]; a level whose k_new/v_new is given is written at that
 * slot (it must be complete up to there, i.e. len[l] == j_new) and its length
 * becomes j_new+1.  The new slot's gate is the router on q.  The new query
 * then attends over slots 0..j_new (it sees itself).  Returns 0, or -1 when
 * the append would be inconsistent or out of capacity. */
int mka_oracle_decode(const double* q, const double* const* k_new, const double* const* v_new,
                      double* const* Kc, double* const* Vc, double* Gc, int32_t* len,
                      const int32_t* cap, int capG, const double* W_r, const double* b_r, int B,
                      int H, int d, double tau, double* O, double* LSE, int32_t* idx) {
  int j_new = 0, any = 0;
  for (int l = 0; l < 3; ++l)
    if (len[l] > j_new) j_new = len[l];
  for (int l = 0; l < 3; ++l) {
    if (k_new[l] && v_new[l]) {
      if (len[l] != j_new || j_new >= cap[l]) return -1;
      any = 1;
    }
  }
  if (!any || j_new >= capG) return -1;
  long n = (long)B * H;
  /* append (step 8) and the new slot's gate (step 5 on the new query) */
#pragma omp parallel for schedule(static)
  for (long bh = 0; bh < n; ++bh) {
    for (int l = 0; l < 3; ++l) {
      if (k_new[l] && v_new[l]) {
        memcpy(Kc[l] + ((size_t)bh * cap[l] + j_new) * d, k_new[l] + (size_t)bh * d,
               sizeof(double) * (size_t)d);
        memcpy(Vc[l] + ((size_t)bh * cap[l] + j_new) * d, v_new[l] + (size_t)bh * d,
               sizeof(double) * (size_t)d);
      }
    }
  }
  for (long bh = 0; bh < n; ++bh) {
    /* one row per (b,h): reuse the router with Tq = S = 1 on a 3-vector */
    double g3[3];
    int32_t id;
    mka_oracle_route(q + (size_t)bh * d, W_r, b_r, 1, 1, 1, 1, d, g3, &id);
    for (int l = 0; l < 3; ++l) Gc[((size_t)bh * capG + j_new) * 3 + l] = g3[l];
    if (idx) idx[bh] = id;
  }
  for (int l = 0; l < 3; ++l)
    if (k_new[l] && v_new[l]) len[l] = j_new + 1;
  int S = j_new + 1;
  /* attention of the single new row over the fused stream (steps 6, 9) */
#pragma omp parallel for schedule(dynamic, 1)
  for (long bh = 0; bh < n; ++bh) {
    double* s = (double*)malloc(sizeof(double) * (size_t)S);
    double* vf = (double*)malloc(sizeof(double) * (size_t)d);
    const double* qq = q + (size_t)bh * d;
    double m = -INFINITY;
    for (int j = 0; j < S; ++j) {
      const double* g = Gc + ((size_t)bh * capG + j) * 3;
      double acc = 0.0;
      for (int k = 0; k < d; ++k) {
        double kf = 0.0;
        for (int l = 0; l < 3; ++l)
          if (j < len[l]) kf += g[l] * Kc[l][((size_t)bh * cap[l] + j) * d + k];
        acc += qq[k] * kf;
      }
      s[j] = tau * acc;
      if (s[j] > m) m = s[j];
    }
    double z = 0.0;
    for (int j = 0; j < S; ++j) {
      s[j] = exp(s[j] - m);
      z += s[j];
    }
    double* o = O + (size_t)bh * d;
    for (int k = 0; k < d; ++k) o[k] = 0.0;
    for (int j = 0; j < S; ++j) {
      const double* g = Gc + ((size_t)bh * capG + j) * 3;
      for (int k = 0; k < d; ++k) {
        double v = 0.0;
        for (int l = 0; l < 3; ++l)
          if (j < len[l]) v += g[l] * Vc[l][((size_t)bh * cap[l] + j) * d + k];
        vf[k] = v;
      }
      double p = s[j] / z;
      for (int k = 0; k < d; ++k) o[k] += p * vf[k];
    }
    if (LSE) LSE[bh] = m + log(z);
    free(s);
    free(vf);
  }
  return 0;
}

/* ---- backward: chain rule through steps 5-9 ---------------------------------
 * Given dO, returns dQ, dK_l, dV_l, dW_r, db_r for L = sum(dO * O).
 *   D[t]      = dO[t].O[t]
 *   dVf[j]    = sum_t p[t,j] dO[t]
 *   dp[t,j]   = dO[t].Vf[j]
 *   ds[t,j]   = p[t,j] (dp[t,j] - D[t])
 *   dQ[t]     = tau sum_j ds[t,j] Kf[j]        dKf[j] = tau sum_t ds[t,j] Q[t]
 *   dK_l[j]   = G[j,l] dKf[j],  dV_l[j] = G[j,l] dVf[j]       (0 where level absent)
 *   dlam[j,l] = dKf[j].K_l[j] + dVf[j].V_l[j]                 (0 where level absent)
 *   dg[j,l]   = G[j,l] (dlam[j,l] - sum_m G[j,m] dlam[j,m])   (softmax Jacobian)
 * and, for the slots whose gate was produced from this call's queries
 * (j = S-Tq+t):  dQ[t] += sum_l dg[j,l] W_r[:,l],  dW_r += Q[t]^T dg[j,:],
 * db_r += dg[j,:].  Older slots' gates are constants of this call.
 * dG (optional, [B,H,S,3]) receives dlam, the gradient w.r.t. the gates
 * themselves, for every slot.  dW_r/db_r are summed over (b,h) in index order. */
void mka_oracle_bwd(const double* dO, const double* Q, const double* K1, const double* K2,
                    const double* K3, const double* V1, const double* V2, const double* V3,
                    const double* G, const double* W_r, const int32_t* len, int B, int H, int Tq,
                    int S, int d, int causal, double tau, double* dQ, double* dK1, double* dK2,
                    double* dK3, double* dV1, double* dV2, double* dV3, double* dW_r, double* db_r,
                    double* dG) {
  const double* K[3] = {K1, K2, K3};
  const double* V[3] = {V1, V2, V3};
  double* dK[3] = {dK1, dK2, dK3};
  double* dV[3] = {dV1, dV2, dV3};
  long n = (long)B * H;
  size_t nf = (size_t)n * S * d;
  double* Kf = (double*)malloc(sizeof(double) * nf);
  double* Vf = (double*)malloc(sizeof(double) * nf);
  double* dKf = (double*)calloc(nf, sizeof(double));
  double* dVf = (double*)calloc(nf, sizeof(double));
  double* dWp = (double*)calloc((size_t)n * d * 3, sizeof(double)); /* per-(b,h) partials */
  double* dbp = (double*)calloc((size_t)n * 3, sizeof(double));
  mka_oracle_fuse(K1, K2, K3, G, len, B, H, S, d, Kf);
  mka_oracle_fuse(V1, V2, V3, G, len, B, H, S, d, Vf);

#pragma omp parallel for schedule(dynamic, 1)
  for (long bh = 0; bh < n; ++bh) {
    double* p = (double*)malloc(sizeof(double) * (size_t)S);
    double* o = (double*)malloc(sizeof(double) * (size_t)d);
    const double* kf = Kf + (size_t)bh * S * d;
    const double* vf = Vf + (size_t)bh * S * d;
    double* dkf = dKf + (size_t)bh * S * d;
    double* dvf = dVf + (size_t)bh * S * d;
    for (int t = 0; t < Tq; ++t) {
      const double* q = Q + ((size_t)bh * Tq + t) * d;
      const double* go = dO + ((size_t)bh * Tq + t) * d;
      double* dq = dQ + ((size_t)bh * Tq + t) * d;
      int nv = visible_upto(t, Tq, S, causal);
      /* recompute the row's probabilities and output from the definition */
      double m = -INFINITY, z = 0.0;
      for (int j = 0; j < nv; ++j) {
        double acc = 0.0;
        for (int k = 0; k < d; ++k) acc += q[k] * kf[(size_t)j * d + k];
        p[j] = tau * acc;
        if (p[j] > m) m = p[j];
      }
      for (int j = 0; j < nv; ++j) {
        p[j] = exp(p[j] - m);
        z += p[j];
      }
      for (int k = 0; k < d; ++k) o[k] = 0.0;
      for (int j = 0; j < nv; ++j) {
        p[j] /= z;
        for (int k = 0; k < d; ++k) o[k] += p[j] * vf[(size_t)j * d + k];
      }
      double D = 0.0;
      for (int k = 0; k < d; ++k) D += go[k] * o[k];
      for (int k = 0; k < d; ++k) dq[k] = 0.0;
      for (int j = 0; j < nv; ++j) {
        double dp = 0.0;
        for (int k = 0; k < d; ++k) dp += go[k] * vf[(size_t)j * d + k];
        double ds = p[j] * (dp - D);
        for (int k = 0; k < d; ++k) {
          dvf[(size_t)j * d + k] += p[j] * go[k];
          dq[k] += tau * ds * kf[(size_t)j * d + k];
          dkf[(size_t)j * d + k] += tau * ds * q[k];
        }
      }
    }
    /* un-fuse and router backward, slot by slot */
    for (int j = 0; j < S; ++j) {
      size_t row = (size_t)bh * S + j;
      const double* g = G + row * 3;
      double dlam[3] = {0.0, 0.0, 0.0};
      for (int l = 0; l < 3; ++l) {
        int present = K[l] && V[l] && j < len[l];
        for (int k = 0; k < d; ++k) {
          double gk = present ? g[l] * dkf[(size_t)j * d + k] : 0.0;
          double gv = present ? g[l] * dvf[(size_t)j * d + k] : 0.0;
          if (dK[l]) dK[l][row * d + k] = gk;
          if (dV[l]) dV[l][row * d + k] = gv;
          if (present)
            dlam[l] += dkf[(size_t)j * d + k] * K[l][row * d + k] +
                       dvf[(size_t)j * d + k] * V[l][row * d + k];
        }
      }
      if (dG)
        for (int l = 0; l < 3; ++l) dG[row * 3 + l] = dlam[l];
      int t = j - (S - Tq);
      if (t >= 0 && W_r) {
        double mean = 0.0;
        for (int l = 0; l < 3; ++l) mean += g[l] * dlam[l];
        const double* q = Q + ((size_t)bh * Tq + t) * d;
        double* dq = dQ + ((size_t)bh * Tq + t) * d;
        for (int l = 0; l < 3; ++l) {
          double dg = g[l] * (dlam[l] - mean);
          dbp[(size_t)bh * 3 + l] += dg;
          for (int k = 0; k < d; ++k) {
            dq[k] += dg * W_r[(size_t)k * 3 + l];
            dWp[((size_t)bh * d + k) * 3 + l] += q[k] * dg;
          }
        }
      }
    }
    free(p);
    free(o);
  }
  if (dW_r) {
    for (int i = 0; i < d * 3; ++i) dW_r[i] = 0.0;
    for (long bh = 0; bh < n; ++bh)
      for (int i = 0; i < d * 3; ++i) dW_r[i] += dWp[(size_t)bh * d * 3 + i];
  }
  if (db_r) {
    for (int l = 0; l < 3; ++l) db_r[l] = 0.0;
    for (long bh = 0; bh < n; ++bh)
      for (int l = 0; l < 3; ++l) db_r[l] += dbp[(size_t)bh * 3 + l];
  }
  free(Kf);
  free(Vf);
  free(dKf);
  free(dVf);
  free(dWp);
  free(dbp);
}
