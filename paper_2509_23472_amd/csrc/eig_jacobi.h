// Symmetric eigendecomposition of a small matrix (order <= LORACT_MAX_RANK) by the parallel cyclic
// Jacobi method, in float64, by one workgroup working in global (L2 resident) memory.
//
// Used only by the randomized-SVD comparator (Section 3.2) to truncate its l-column factor to
// rank k: with B = Q^T X (l x n) and B B^T = W diag(lambda) W^T, the k leading left singular
// vectors of B are the k leading columns of W.  Each round rotates l/2 disjoint index pairs
// (round-robin tournament order); a sweep is l-1 rounds.  Rotations are the classical
// symmetric Schur 2 x 2 ones.  The sweeps stop when the off-diagonal mass no longer matters at
// float64 precision, or after a fixed maximum.
#pragma once
#include "common.h"

#define EJ_THREADS 1024
#define EJ_MAX_SWEEPS 14

// A: l x l symmetric (overwritten, diagonal -> eigenvalues); W: l x l out (columns = eigenvectors);
// Wk: l x k out = the k eigenvectors of largest eigenvalue, in descending order.
// Adaptive rank (k_out != null): with s_i = sqrt(eigenvalue i) in descending order -- the singular
// values of the factor whose Gram matrix A is -- only the first k_eff columns of Wk are filled,
// k_eff = the smallest count with s_1 + ... + s_k_eff >= energy * (s_1 + ... + s_l), at most k;
// the other columns are zero and *k_out = k_eff (the retained-energy count of Section 2).
__global__ __launch_bounds__(EJ_THREADS) void jacobi_eig_kernel(double* A, double* W, double* Wk,
                                                                int l, int k, double energy,
                                                                int32_t* k_out) {
  __shared__ double cs_c[LORACT_MAX_RANK / 2 + 1], cs_s[LORACT_MAX_RANK / 2 + 1];
  __shared__ int pr_p[LORACT_MAX_RANK / 2 + 1], pr_q[LORACT_MAX_RANK / 2 + 1];
  __shared__ double red[EJ_THREADS / 64];
  __shared__ double off_norm, diag_norm;
  __shared__ int order[LORACT_MAX_RANK];

  const int t = threadIdx.x;
  const int n = l + (l & 1);          // even number of players; index l (if any) is a bye
  const int half = n / 2;
  for (int e = t; e < l * l; e += EJ_THREADS) W[e] = ((e / l) == (e % l)) ? 1.0 : 0.0;
  __syncthreads();

  for (int sweep = 0; sweep < EJ_MAX_SWEEPS; ++sweep) {
    // convergence test: sum of squares off the diagonal against the diagonal
    double so = 0.0, sd = 0.0;
    for (int e = t; e < l * l; e += EJ_THREADS) {
      const int i = e / l, j = e - i * l;
      const double v = A[e];
      if (i == j) sd += v * v; else so += v * v;
    }
    for (int pass = 0; pass < 2; ++pass) {
      double v = pass == 0 ? so : sd;
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
      if ((t & 63) == 0) red[t >> 6] = v;
      __syncthreads();
      if (t == 0) {
        double tot = 0.0;
        for (int w = 0; w < EJ_THREADS / 64; ++w) tot += red[w];
        if (pass == 0) off_norm = tot; else diag_norm = tot;
      }
      __syncthreads();
    }
    if (off_norm <= 1e-30 * diag_norm || off_norm == 0.0) break;

    for (int round = 0; round < n - 1; ++round) {
      // pairs of this round and their rotations
      if (t < half) {
        int p = (round + t) % (n - 1);
        int q = (t == 0) ? (n - 1) : (round + n - 1 - t) % (n - 1);
        if (p > q) { const int tmp = p; p = q; q = tmp; }
        double c = 1.0, s = 0.0;
        if (q < l) {
          const double app = A[(int64_t)p * l + p], aqq = A[(int64_t)q * l + q];
          const double apq = A[(int64_t)p * l + q];
          if (fabs(apq) > 1e-300 && fabs(apq) > 1e-18 * sqrt(fabs(app * aqq))) {
            const double tau = (aqq - app) / (2.0 * apq);
            const double tt = (tau >= 0.0 ? 1.0 : -1.0) / (fabs(tau) + sqrt(1.0 + tau * tau));
            c = 1.0 / sqrt(1.0 + tt * tt);
            s = tt * c;
          }
        } else {
          q = -1;     // bye
        }
        pr_p[t] = p; pr_q[t] = q; cs_c[t] = c; cs_s[t] = s;
      }
      __syncthreads();
      // columns: A <- A J, W <- W J
      for (int e = t; e < l * half; e += EJ_THREADS) {
        const int r = e / half, i = e - r * half;
        const int p = pr_p[i], q = pr_q[i];
        if (q < 0) continue;
        const double c = cs_c[i], s = cs_s[i];
        if (s == 0.0) continue;
        double* ar = A + (int64_t)r * l;
        const double ap = ar[p], aq = ar[q];
        ar[p] = c * ap - s * aq;
        ar[q] = s * ap + c * aq;
        double* wr = W + (int64_t)r * l;
        const double wp = wr[p], wq = wr[q];
        wr[p] = c * wp - s * wq;
        wr[q] = s * wp + c * wq;
      }
      __syncthreads();
      // rows: A <- J^T A
      for (int e = t; e < half * l; e += EJ_THREADS) {
        const int i = e / l, col = e - i * l;
        const int p = pr_p[i], q = pr_q[i];
        if (q < 0) continue;
        const double c = cs_c[i], s = cs_s[i];
        if (s == 0.0) continue;
        const double ap = A[(int64_t)p * l + col], aq = A[(int64_t)q * l + col];
        A[(int64_t)p * l + col] = c * ap - s * aq;
        A[(int64_t)q * l + col] = s * ap + c * aq;
      }
      __syncthreads();
    }
  }

  // rank the eigenvalues (descending, ties by index) and gather the k leading eigenvectors
  for (int i = t; i < l; i += EJ_THREADS) {
    const double li = A[(int64_t)i * l + i];
    int rank = 0;
    for (int j = 0; j < l; ++j) {
      const double lj = A[(int64_t)j * l + j];
      rank += (lj > li) || (lj == li && j < i);
    }
    order[rank] = i;
  }
  __syncthreads();
  __shared__ int k_eff;
  if (t == 0) {
    int keep = k;
    if (k_out) {
      double total = 0.0;
      for (int i = 0; i < l; ++i) total += sqrt(fmax(A[(int64_t)order[i] * l + order[i]], 0.0));
      double run = 0.0;
      keep = l;
      for (int i = 0; i < l; ++i) {
        run += sqrt(fmax(A[(int64_t)order[i] * l + order[i]], 0.0));
        if (run >= energy * total) { keep = i + 1; break; }
      }
      if (keep > k) keep = k;
      *k_out = keep;
    }
    k_eff = keep;
  }
  __syncthreads();
  for (int e = t; e < l * k; e += EJ_THREADS) {
    const int r = e / k, c = e - r * k;
    Wk[e] = c < k_eff ? W[(int64_t)r * l + order[c]] : 0.0;
  }
}

static int launch_jacobi_eig(hipStream_t s, double* A, double* W, double* Wk, int l, int k,
                             double energy = 1.0, int32_t* k_out = nullptr) {
  if (l < 1 || l > LORACT_MAX_RANK || k < 1 || k > l) return LORACT_ERR_INVALID_ARG;
  LORACT_LAUNCH("jacobi_eig", s, jacobi_eig_kernel, dim3(1), dim3(EJ_THREADS), 0, A, W, Wk, l, k, energy, k_out);
  return LORACT_OK;
}
