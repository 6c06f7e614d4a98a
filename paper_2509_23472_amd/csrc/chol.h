// Cholesky factorisation of a small Gram matrix and inversion of its triangular factor, in
// float64, by one workgroup.
//
// For a tall-skinny Y with Gram matrix G = Y^T Y = L L^T the orthonormal factor of the thin QR
// of Y is Q = Y L^{-T}; this kernel turns G into Rinv = L^{-T} (upper triangular) so that the
// factor can be applied as a plain matrix product.
//
// Two modes, used as the two rounds of a shifted Cholesky QR:
//  * shift_rel > 0 (first round): factor G + s I with s = shift_rel * trace(G).  The shift keeps
//    the factorisation defined when cond(Y)^2 exceeds what float64 resolves; Q1 = Y Rinv still
//    spans range(Y) exactly (Rinv is invertible) and has cond(Q1) ~ cond(Y) * sqrt(shift_rel),
//    small enough for an unshifted second round.
//  * shift_rel == 0 (second round): plain Cholesky.
// Breakdown rule (second round): after the first round the columns of Q1 are scaled to O(1) and
// stored in at most float32, so a pivot not larger than tol * G[j][j] with tol = (k 2^-24)^2 means
// column j depends on the earlier columns to within float32 resolution (exact duplicates among
// the sampled rows, or an all-zero sampled row).  Its reciprocal pivot is set to zero, which
// zeroes column j of L below the diagonal and the whole column j of Rinv: the matching column
// of Q becomes zero, the other columns are exactly what they would be with column j removed,
// and the status word gets LORACT_STATUS_RANK_DEFICIENT.  The shifted first round only clamps
// (and flags) a pivot that is not positive at all.
#pragma once
#include "common.h"

#define CH_NB 16

__global__ __launch_bounds__(256) void chol_inverse_kernel(double* G, double* Rinv, int k,
                                                           double tol, double shift_rel,
                                                           int32_t* status) {
  __shared__ double Ds[CH_NB][CH_NB + 1];
  __shared__ double Di[CH_NB][CH_NB + 1];
  __shared__ double Ps[LORACT_MAX_RANK * (CH_NB + 1)];  // panel [row][17], later W [16][k+1]
  __shared__ double dinv[LORACT_MAX_RANK];
  __shared__ double gdiag[LORACT_MAX_RANK];
  __shared__ int deficient;
  __shared__ double shift_s;

  const int t = threadIdx.x;
  const int tr = t >> 4, tc = t & 15;
  for (int i = t; i < k; i += 256) gdiag[i] = G[(int64_t)i * k + i];
  if (t == 0) deficient = 0;
  __syncthreads();
  if (t == 0) {
    double tr_sum = 0.0;
    for (int i = 0; i < k; ++i) tr_sum += gdiag[i];
    shift_s = shift_rel * tr_sum;
  }
  __syncthreads();
  const double shift = shift_s;

  // ---- phase A: G = L L^T, L left in the strict lower triangle of G, 1/L[j][j] in dinv.
  for (int jb = 0; jb < k; jb += CH_NB) {
    const int nb = (k - jb < CH_NB) ? (k - jb) : CH_NB;
    if (tr < nb && tc < nb)
      Ds[tr][tc] = G[(int64_t)(jb + tr) * k + jb + tc] + (tr == tc ? shift : 0.0);
    __syncthreads();
    for (int j = 0; j < nb; ++j) {
      const double piv = Ds[j][j];
      const bool usable = shift > 0.0 ? (piv > 0.0) : (piv > tol * gdiag[jb + j]);
      const bool bad = !usable;
      const double di = usable ? 1.0 / sqrt(piv) : 0.0;
      if (t == 0) {
        dinv[jb + j] = di;
        if (bad) deficient = 1;
      }
      if (t > j && t < nb) Ds[t][j] *= di;
      __syncthreads();
      if (tr < nb && tc > j && tc <= tr) Ds[tr][tc] -= Ds[tr][j] * Ds[tc][j];
      __syncthreads();
    }
    if (tr < nb && tc < tr) G[(int64_t)(jb + tr) * k + jb + tc] = Ds[tr][tc];

    // panel below the diagonal block: solve X * Lbb^T = G[i][jb..jb+nb) row by row
    const int below = jb + nb;
    for (int i = below + t; i < k; i += 256) {
      double x[CH_NB];
#pragma unroll
      for (int c = 0; c < CH_NB; ++c) x[c] = (c < nb) ? G[(int64_t)i * k + jb + c] : 0.0;
#pragma unroll
      for (int c = 0; c < CH_NB; ++c) {
        if (c < nb) {
          double s = x[c];
#pragma unroll
          for (int c2 = 0; c2 < CH_NB; ++c2)
            if (c2 < c) s -= x[c2] * Ds[c][c2];
          x[c] = s * dinv[jb + c];
        }
      }
#pragma unroll
      for (int c = 0; c < CH_NB; ++c) {
        if (c < nb) G[(int64_t)i * k + jb + c] = x[c];
        Ps[(i - below) * (CH_NB + 1) + c] = x[c];
      }
    }
    __syncthreads();
    // trailing update of the lower triangle
    const int nrem = k - below;
    for (int e = t; e < nrem * nrem; e += 256) {
      const int ri = e / nrem, ci = e - ri * nrem;
      if (ci <= ri) {
        double s = 0.0;
#pragma unroll
        for (int c = 0; c < CH_NB; ++c) s += Ps[ri * (CH_NB + 1) + c] * Ps[ci * (CH_NB + 1) + c];
        G[(int64_t)(below + ri) * k + below + ci] -= s;
      }
    }
    __syncthreads();
  }

  // ---- phase B: Linv = L^{-1} (lower), written transposed: Rinv[c][i] = Linv[i][c].
  for (int e = t; e < k * k; e += 256) Rinv[e] = 0.0;
  __syncthreads();
  double* Ws = Ps;  // [CH_NB][k + 1]
  const int wld = k + 1;
  for (int ib = 0; ib < k; ib += CH_NB) {
    const int nb = (k - ib < CH_NB) ? (k - ib) : CH_NB;
    if (tr < nb && tc < nb) {
      Ds[tr][tc] = (tc < tr) ? G[(int64_t)(ib + tr) * k + ib + tc] : 0.0;
      Di[tr][tc] = 0.0;
    }
    __syncthreads();
    // inverse of the diagonal block, one thread per column
    if (t < nb) {
      const int c = t;
      double x[CH_NB];
#pragma unroll
      for (int r = 0; r < CH_NB; ++r) x[r] = 0.0;
#pragma unroll
      for (int r = 0; r < CH_NB; ++r) {
        if (r == c) x[r] = dinv[ib + c];
        else if (r > c && r < nb) {
          double s = 0.0;
#pragma unroll
          for (int j = 0; j < CH_NB; ++j)
            if (j >= c && j < r) s += Ds[r][j] * x[j];
          x[r] = -s * dinv[ib + r];
        }
      }
#pragma unroll
      for (int r = 0; r < CH_NB; ++r)
        if (r < nb) Di[r][c] = x[r];
    }
    // W[r][c] = sum_{j=c}^{ib-1} L[ib+r][j] * Linv[j][c]   for c < ib
    for (int e = t; e < CH_NB * ib; e += 256) {
      const int c = e >> 4, r = e & 15;
      double s = 0.0;
      if (r < nb) {
        const double* lrow = G + (int64_t)(ib + r) * k;
        const double* icol = Rinv + (int64_t)c * k;
        for (int j = c; j < ib; ++j) s += lrow[j] * icol[j];
      }
      Ws[r * wld + c] = s;
    }
    __syncthreads();
    // Linv[ib+r][c] = - sum_{r2<=r} Di[r][r2] * W[r2][c]
    for (int e = t; e < CH_NB * ib; e += 256) {
      const int c = e >> 4, r = e & 15;
      if (r < nb) {
        double s = 0.0;
#pragma unroll
        for (int r2 = 0; r2 < CH_NB; ++r2)
          if (r2 <= r) s += Di[r][r2] * Ws[r2 * wld + c];
        Rinv[(int64_t)c * k + ib + r] = -s;
      }
    }
    if (tr < nb && tc <= tr) Rinv[(int64_t)(ib + tc) * k + ib + tr] = Di[tr][tc];
    __syncthreads();
  }
  if (t == 0 && deficient && status) atomicOr(status, LORACT_STATUS_RANK_DEFICIENT);
}

static int launch_chol_inverse(hipStream_t stream, double* G, double* Rinv, int k,
                               double shift_rel, int32_t* status) {
  if (k < 1 || k > LORACT_MAX_RANK) return LORACT_ERR_UNSUPPORTED;
  const double tol = ((double)k * 5.9604644775390625e-08) * ((double)k * 5.9604644775390625e-08);
  LORACT_LAUNCH("chol_inverse", stream, chol_inverse_kernel, dim3(1), dim3(256), 0, G, Rinv, k,
                tol, shift_rel, status);
  return LORACT_OK;
}
