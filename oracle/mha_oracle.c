/*
 * fp64 CPU oracle for multi-head attention forward and backward.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * HIP kernels are checked against.  It shares no code, header, table or helper
 * with the GPU path, and the GPU path never calls it.  Only the tests, the
 * smoke check and the benchmark's cpu_baseline leg may load it.
 *
 * What it computes, per (batch, head) independently, for row-major matrices
 * Q (Nq x d) and K, V (Nk x d).  Self-attention has Nq = Nk = N; the decoder's
 * second attention layer of Sec. 2.1 takes its queries from one sequence and its
 * keys and values from another, so the two lengths differ there.  The causal
 * mask is defined for Nq = Nk only.  (Paper Sec. 2.1, Eq. 1, with the scale applied to the logits
 * before the softmax, which is the only reading under which rows of P sum to
 * one and which every system the paper compares against computes):
 *
 *   S_ij   = scale * sum_k Q_ik K_jk                       (Eq. 1, first line)
 *   causal : keys j > i are excluded (S_ij = -inf)         (Sec. 2.1, masked MHA)
 *   m_i    = max_j S_ij,  f_ij = exp(S_ij - m_i),
 *   l_i    = sum_j f_ij,  P_ij = f_ij / l_i                (Sec. 3.2.1, Eq. 2, with
 *                                                           l = sum of f, the only
 *                                                           reading for which the
 *                                                           merge rule of Eq. 3 holds)
 *   LSE_i  = m_i + ln l_i    (the row statistic the forward saves for the
 *                             backward; Sec. 3.3 uses it as Exp(S_ij - L_i) = P_ij,
 *                             which holds only for the log-sum-exp)
 *   O_ik   = sum_j P_ij V_jk                               (Eq. 1, third line)
 *
 * Backward (Sec. 3.3, Eq. 4), given dO:
 *   D_i    = sum_k dO_ik O_ik           ("dPsum", with this oracle's own fp64 O)
 *   dV_jk  = sum_i P_ij dO_ik           (dV = P^T dO)
 *   dP_ij  = sum_k dO_ik V_jk           (dP = dO V^T)
 *   dS_ij  = P_ij (dP_ij - D_i)         (Jacobian-vector product of row softmax;
 *                                        sum_j P_ij dP_ij = D_i follows from O = P V)
 *   dQ_ik  = scale * sum_j dS_ij K_jk   (dQ = dS K)
 *   dK_jk  = scale * sum_i dS_ij Q_ik   (dK = dS^T Q; the printed "Q dS^T" has
 *                                        no consistent shape)
 *
 * Dropout (Sec. 4.1 runs every measurement with a dropout rate of 0.1; Sec. 4.2
 * says the backward applies the same dropout logic as the forward so that the
 * two agree).  The paper fixes neither where the mask is applied nor how it is
 * drawn.  Reading taken: the usual attention dropout, an independent keep/drop
 * decision per entry of P after the softmax, survivors scaled by r = 1/(1 - p)
 * so that the expectation is unchanged.  With a keep mask M (1 = keep):
 *   O_ik   = sum_j r M_ij P_ij V_jk           (LSE and P themselves unchanged)
 *   dV_jk  = sum_i r M_ij P_ij dO_ik
 *   dP_ij  = r M_ij sum_k dO_ik V_jk          (gradient w.r.t. P, through the mask)
 *   dS_ij  = P_ij (dP_ij - D_i), D_i = sum_k dO_ik O_ik as before (it still equals
 *            sum_j P_ij dP_ij, now with the dropped O)
 * The attention routines take M as an explicit array; oracle_dropout_mask draws
 * it with a counter-based generator (see there) so that a test can hand the
 * same (seed, offset) to the GPU library, which implements the generator itself.
 *
 * The Nq x Nk matrices are materialised per head.  There is no tiling, no online
 * softmax, no fusion: a reader can check every loop against the formulas above.
 * OpenMP only spreads independent rows (or independent output rows) over
 * threads; it reorders no sum.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/*
 * Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw: "Parallel random numbers:
 * as easy as 1, 2, 3", SC'11): a keyed bijection of a 128-bit counter.  One round
 * maps (c0, c1, c2, c3) to (hi(M1 c2) ^ c1 ^ k0, lo(M1 c2), hi(M0 c0) ^ c3 ^ k1,
 * lo(M0 c0)); the key grows by the two Weyl constants after every round.
 */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n1 = (uint32_t)p1;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    const uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/*
 * Keep mask of attention dropout, M [B*H][Nq][Nk] bytes (1 = keep, 0 = drop).
 * The decision for entry (head h, query i, key j) is one byte of a Philox output:
 *   x = Philox4x32-10(counter = (j / 4, i / 4, h, offset), key = (seed low, seed high))
 *   u = byte (j mod 4) of word x[i mod 4]   (byte 0 = least significant)
 *   keep iff u >= threshold
 * so one generator call decides a block of 4 queries x 4 keys, an entry is dropped
 * with probability threshold / 256 exactly, and survivors are to be scaled by
 * 256 / (256 - threshold).  `offset` distinguishes calls that share a seed.
 * Returns 0, or -1 on bad arguments (threshold outside 0..255).
 */
int oracle_dropout_mask(unsigned char *M, int BH, int Nq, int Nk, uint64_t seed,
                        uint32_t offset, int threshold) {
  if (!M || BH < 0 || Nq <= 0 || Nk <= 0 || threshold < 0 || threshold > 255) return -1;
  const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
#pragma omp parallel for schedule(static) collapse(2)
  for (int h = 0; h < BH; ++h)
    for (int i = 0; i < Nq; ++i)
      for (int j = 0; j < Nk; ++j) {
        const uint32_t ctr[4] = {(uint32_t)(j / 4), (uint32_t)(i / 4), (uint32_t)h, offset};
        uint32_t x[4];
        oracle_philox4x32_10(ctr, key, x);
        const unsigned u = (x[i % 4] >> (8 * (j % 4))) & 0xFFu;
        M[((size_t)h * Nq + i) * Nk + j] = u >= (unsigned)threshold ? 1 : 0;
      }
  return 0;
}

/* S and P for one head.  P is Nq x Nk row-major; masked entries are exactly 0. */
static void head_softmax(const double *Q, const double *K, int Nq, int Nk, int d,
                         double scale, int causal, double *P, double *LSE) {
#pragma omp parallel for schedule(dynamic, 8)
  for (int i = 0; i < Nq; ++i) {
    double *Pi = P + (size_t)i * Nk;
    const int jend = causal ? i + 1 : Nk;
    double m = -INFINITY;
    for (int j = 0; j < jend; ++j) {
      double s = 0.0;
      for (int k = 0; k < d; ++k) s += Q[(size_t)i * d + k] * K[(size_t)j * d + k];
      s *= scale;
      Pi[j] = s;
      if (s > m) m = s;
    }
    double l = 0.0;
    for (int j = 0; j < jend; ++j) {
      Pi[j] = exp(Pi[j] - m);
      l += Pi[j];
    }
    for (int j = 0; j < jend; ++j) Pi[j] /= l;
    for (int j = jend; j < Nk; ++j) Pi[j] = 0.0;
    LSE[i] = m + log(l);
  }
}

/* O = (r M o P) V for one head; keep == NULL means no dropout (M = 1, r = 1). */
static void head_pv(const double *P, const unsigned char *keep, double r, const double *V,
                    int Nq, int Nk, int d, double *O) {
#pragma omp parallel for schedule(dynamic, 8)
  for (int i = 0; i < Nq; ++i) {
    double *Oi = O + (size_t)i * d;
    for (int k = 0; k < d; ++k) Oi[k] = 0.0;
    for (int j = 0; j < Nk; ++j) {
      double p = P[(size_t)i * Nk + j];
      if (keep) p = keep[(size_t)i * Nk + j] ? r * p : 0.0;
      if (p == 0.0) continue; /* masked, dropped or underflowed: contributes exactly 0 */
      for (int k = 0; k < d; ++k) Oi[k] += p * V[(size_t)j * d + k];
    }
  }
}

/*
 * Forward for B*H heads.  Q: [B*H][Nq][d], K, V: [B*H][Nk][d] fp64 (the caller
 * widens the 16-bit inputs exactly).  Outputs O [B*H][Nq][d], LSE [B*H][Nq].
 * P_out, if not NULL, receives the full probability matrices [B*H][Nq][Nk]
 * (tests only; P before dropout).  keep: NULL, or the dropout keep mask
 * [B*H][Nq][Nk] with keep_scale = r.  Returns 0, or -1 on allocation failure /
 * bad arguments (causal with Nq != Nk is a bad argument).
 */
int oracle_mha_fwd(const double *Q, const double *K, const double *V, double *O,
                   double *LSE, double *P_out, int BH, int Nq, int Nk, int d,
                   double scale, int causal, const unsigned char *keep, double keep_scale) {
  if (!Q || !K || !V || !O || !LSE || BH < 0 || Nq <= 0 || Nk <= 0 || d <= 0) return -1;
  if (causal && Nq != Nk) return -1;
  double *Pbuf = P_out ? NULL : (double *)malloc((size_t)Nq * Nk * sizeof(double));
  if (!P_out && !Pbuf) return -1;
  for (int h = 0; h < BH; ++h) {
    const size_t offq = (size_t)h * Nq * d; /* Q, O */
    const size_t offk = (size_t)h * Nk * d; /* K, V */
    double *P = P_out ? P_out + (size_t)h * Nq * Nk : Pbuf;
    const unsigned char *keeph = keep ? keep + (size_t)h * Nq * Nk : NULL;
    head_softmax(Q + offq, K + offk, Nq, Nk, d, scale, causal, P, LSE + (size_t)h * Nq);
    head_pv(P, keeph, keep_scale, V + offk, Nq, Nk, d, O + offq);
  }
  free(Pbuf);
  return 0;
}

/*
 * Backward for B*H heads.  Recomputes the forward in fp64 itself (its own O
 * feeds D), then applies Eq. 4.  dO, dQ (and O_out): [B*H][Nq][d]; dK, dV:
 * [B*H][Nk][d]; LSE_out, D_out: [B*H][Nq]; the three *_out pointers may be NULL.
 * keep / keep_scale: as in oracle_mha_fwd.
 */
int oracle_mha_bwd(const double *Q, const double *K, const double *V,
                   const double *dO, double *dQ, double *dK, double *dV,
                   double *O_out, double *LSE_out, double *D_out, int BH, int Nq,
                   int Nk, int d, double scale, int causal, const unsigned char *keep,
                   double keep_scale) {
  if (!Q || !K || !V || !dO || !dQ || !dK || !dV || BH < 0 || Nq <= 0 || Nk <= 0 || d <= 0)
    return -1;
  if (causal && Nq != Nk) return -1;
  double *P = (double *)malloc((size_t)Nq * Nk * sizeof(double));
  double *dS = (double *)malloc((size_t)Nq * Nk * sizeof(double));
  double *O = (double *)malloc((size_t)Nq * d * sizeof(double));
  double *LSE = (double *)malloc((size_t)Nq * sizeof(double));
  double *D = (double *)malloc((size_t)Nq * sizeof(double));
  if (!P || !dS || !O || !LSE || !D) {
    free(P); free(dS); free(O); free(LSE); free(D);
    return -1;
  }
  for (int h = 0; h < BH; ++h) {
    const size_t offq = (size_t)h * Nq * d; /* Q, dO, dQ, O */
    const size_t offk = (size_t)h * Nk * d; /* K, V, dK, dV */
    const double *Qh = Q + offq, *Kh = K + offk, *Vh = V + offk, *dOh = dO + offq;
    const unsigned char *keeph = keep ? keep + (size_t)h * Nq * Nk : NULL;
    head_softmax(Qh, Kh, Nq, Nk, d, scale, causal, P, LSE);
    head_pv(P, keeph, keep_scale, Vh, Nq, Nk, d, O);
    /* D_i, dP_ij, dS_ij: independent per query row i */
#pragma omp parallel for schedule(dynamic, 8)
    for (int i = 0; i < Nq; ++i) {
      double Di = 0.0;
      for (int k = 0; k < d; ++k) Di += dOh[(size_t)i * d + k] * O[(size_t)i * d + k];
      D[i] = Di;
      const int jend = causal ? i + 1 : Nk;
      for (int j = 0; j < jend; ++j) {
        double dp = 0.0;
        for (int k = 0; k < d; ++k) dp += dOh[(size_t)i * d + k] * Vh[(size_t)j * d + k];
        if (keeph) dp = keeph[(size_t)i * Nk + j] ? keep_scale * dp : 0.0;
        dS[(size_t)i * Nk + j] = P[(size_t)i * Nk + j] * (dp - Di);
      }
      for (int j = jend; j < Nk; ++j) dS[(size_t)i * Nk + j] = 0.0;
      /* dQ_i = scale * sum_j dS_ij K_j */
      double *dQi = dQ + offq + (size_t)i * d;
      for (int k = 0; k < d; ++k) dQi[k] = 0.0;
      for (int j = 0; j < jend; ++j) {
        const double ds = dS[(size_t)i * Nk + j];
        for (int k = 0; k < d; ++k) dQi[k] += ds * Kh[(size_t)j * d + k];
      }
      for (int k = 0; k < d; ++k) dQi[k] *= scale;
    }
    /* dV_j = sum_i P_ij dO_i ;  dK_j = scale * sum_i dS_ij Q_i : independent per key row j */
#pragma omp parallel for schedule(dynamic, 8)
    for (int j = 0; j < Nk; ++j) {
      double *dVj = dV + offk + (size_t)j * d;
      double *dKj = dK + offk + (size_t)j * d;
      for (int k = 0; k < d; ++k) { dVj[k] = 0.0; dKj[k] = 0.0; }
      const int ibeg = causal ? j : 0;
      for (int i = ibeg; i < Nq; ++i) {
        const double p = P[(size_t)i * Nk + j];
        const double pm = keeph ? (keeph[(size_t)i * Nk + j] ? keep_scale * p : 0.0) : p;
        const double ds = dS[(size_t)i * Nk + j];
        for (int k = 0; k < d; ++k) {
          dVj[k] += pm * dOh[(size_t)i * d + k];
          dKj[k] += ds * Qh[(size_t)i * d + k];
        }
      }
      for (int k = 0; k < d; ++k) dKj[k] *= scale;
    }
    if (O_out) for (size_t t = 0; t < (size_t)Nq * d; ++t) O_out[offq + t] = O[t];
    if (LSE_out) for (int i = 0; i < Nq; ++i) LSE_out[(size_t)h * Nq + i] = LSE[i];
    if (D_out) for (int i = 0; i < Nq; ++i) D_out[(size_t)h * Nq + i] = D[i];
  }
  free(P); free(dS); free(O); free(LSE); free(D);
  return 0;
}
