// Symmetric positive semidefinite eigendecomposition of a small matrix (order <= LORACT_MAX_RANK)
// by the one-sided (Hestenes) Jacobi method in float64, one workgroup.
//
// Used where an l-column factor is cut to rank k (the randomized-SVD comparator of Section 3.2,
// more sampled rows than the rank, the adaptive rank): with B = Q^T X (l x n) and
// A = B B^T = W diag(lambda) W^T, the k leading left singular vectors of B are the k leading
// columns of W and its singular values are sqrt(lambda).
//
// Method.  A = L L^T is factored first (Cholesky without pivoting in place; a pivot at the rounding
// level of the largest diagonal entry ends its column with zeros, which is what a semidefinite
// matrix of that rank calls for), because the left singular vectors of L are the eigenvectors of A
// and its singular values their square roots: the iteration then works on a matrix with the
// condition number of B instead of its fourth power, and needs a third of the sweeps.  The columns
// of G = L are then orthogonalised by plane rotations from the right: for a pair (p, q) with
// a = |g_p|^2, b = |g_q|^2, c = g_p . g_q the rotation with tangent t = sign(z) / (|z| + sqrt(1 + z^2)),
// z = (b - a) / (2 c), makes the two columns orthogonal; the longer of the two results goes to the
// lower index (de Rijk's rule, which keeps the columns roughly sorted by length and speeds up the
// convergence on graded matrices).  When all pairs are orthogonal G = W diag(sigma) (up to the order
// and the signs of the columns): lambda_j = |g_j|^2 and w_j = g_j / |g_j|.  Nothing besides G is
// stored -- no accumulated rotation matrix -- and a round of l / 2 disjoint pairs (round-robin
// tournament order) needs no communication between pairs, only a barrier before the next round.
// Small columns keep their relative accuracy under rotations with large ones, which is what the
// graded spectra met here (eigenvalue ratios of 1e-12) need.
//
// Layout.  G is column-major with a pitch of EJ_PITCH(l) doubles; a pair is handled by 16 lanes,
// lane i of the group owning rows i, i + 16, ...; the dot product is summed inside the group by
// four exchange steps.  Up to l = 141 G lives in LDS (160 KB); above, in a global work buffer that
// stays in L2 (an order of magnitude slower: every round then moves the whole matrix through the
// CU once; measured 2.6 ms at l = 136, 13 sweeps, against 40 ms at l = 264).  A round moves every
// column through LDS once (2 l^2 x 8 bytes at 128 bytes per clock: about 1 us at l = 136), which
// is most of its cost; 8 lanes per pair, so that the 68 pairs of a round at l = 136 run in one
// pass instead of two, moves the same bytes with longer chains per lane and was slower (4.3 ms).
#pragma once
#include "common.h"

#define EJ_THREADS 1024
#define EJ_GROUPS (EJ_THREADS / 16)
#define EJ_MAX_SWEEPS 30
#define EJ_ROT_TOL 1e-11        // pairs with |c| <= tol sqrt(a b) count as orthogonal

// (an even pitch two rows longer than the matrix: 16-byte aligned columns whose offsets spread over
// the LDS banks)
static inline __host__ __device__ int ej_pitch(int l) { return l + (l & 1) + 2; }
static inline size_t ej_small_bytes(int l) { return ((size_t)2 * l + 8) * sizeof(double) + (size_t)(l + 4) * sizeof(int); }
static inline size_t ej_lds_bytes(int l) { return (size_t)ej_pitch(l) * l * sizeof(double) + ej_small_bytes(l); }
#define EJ_LDS_LIMIT (160 * 1024 - 256)     // dynamic LDS the kernel may ask for (it has a few static words too)
static inline bool ej_fits_lds(int l) { return ej_lds_bytes(l) <= EJ_LDS_LIMIT; }
// doubles of global work space the kernel needs when G does not fit in LDS
static inline size_t ej_work_doubles(int l) { return (size_t)ej_pitch(l) * l; }

// Sum over the 16 lanes of a group; every lane gets the total.  Four exchange steps inside a
// row of 16 lanes on the data-parallel-primitive path of the vector unit (no LDS round trip):
// mirror of the row, mirror of each half, reversal and pair swap inside each quad.
template <int CTRL>
__device__ inline double ej_dpp_add(double v) {
  union { double d; int i[2]; } a, b;
  a.d = v;
  b.i[0] = __builtin_amdgcn_update_dpp(0, a.i[0], CTRL, 0xf, 0xf, false);
  b.i[1] = __builtin_amdgcn_update_dpp(0, a.i[1], CTRL, 0xf, 0xf, false);
  return v + b.d;
}
__device__ inline double ej_group_sum(double v) {
  v = ej_dpp_add<0x140>(v);     // row_mirror:       lane i <- lane 15 - i
  v = ej_dpp_add<0x141>(v);     // row_half_mirror:  lane i <- lane 7 - i inside each half
  v = ej_dpp_add<0x1b>(v);      // quad_perm [3,2,1,0]
  v = ej_dpp_add<0xb1>(v);      // quad_perm [1,0,3,2]
  return v;
}

// cos and sin of the rotation that orthogonalises two columns with squared norms a, b and inner
// product c, and its tangent.  The tangent only has to be roughly right -- a pair that is left with
// a residual inner product is met again -- so it is formed from the hardware's reciprocal and square
// root estimates; what must be exact is cs^2 + sn^2 = 1 (else the columns would change length with
// every rotation), and cs = 1 / sqrt(1 + t^2) is therefore refined to float64 accuracy.
__device__ inline void ej_rotation(double a, double b, double c, double* cs, double* sn, double* tt) {
  const double z = (b - a) * (0.5 * __builtin_amdgcn_rcp(c));
  const double az = fabs(z);
  // |z| + sqrt(1 + z^2): for large |z| the square root is |z| itself
  const double den = az > 1e8 ? 2.0 * az : az + __builtin_amdgcn_sqrt(fma(z, z, 1.0));
  double t = __builtin_amdgcn_rcp(den);
  t = z >= 0.0 ? t : -t;
  const double x = fma(t, t, 1.0);
  double y = __builtin_amdgcn_rsq(x);
#pragma unroll
  for (int it = 0; it < 2; ++it) y = y * fma(-0.5 * x * y, y, 1.5);      // Newton steps for 1 / sqrt(x)
  *cs = y;
  *sn = t * y;
  *tt = t;
}

// A: l x l symmetric positive semidefinite, row-major (read only); work: ej_work_doubles(l) doubles
// (used when G does not fit in LDS); Wk: l x k out = the k eigenvectors of largest eigenvalue, in
// descending order (a column whose eigenvalue is zero comes out zero).
// Adaptive rank (k_out != null): with s_i = sqrt(lambda_i) in descending order -- the singular
// values of the factor whose Gram matrix A is -- only the first k_eff columns of Wk are filled,
// k_eff = the smallest count with s_1 + ... + s_k_eff >= energy * (s_1 + ... + s_l), at most k;
// the other columns are zero and *k_out = k_eff (the retained-energy count of Section 2).
// NR = rows per lane (pitch / 16 rounded up); IN_LDS selects where G lives.
template <int NR, bool IN_LDS>
__global__ __launch_bounds__(EJ_THREADS) void jacobi_eig_kernel(const double* A, double* work, double* Wk,
                                                                int l, int k, double energy,
                                                                int32_t* k_out) {
  extern __shared__ __attribute__((aligned(16))) double ej_smem[];
  const int pitch = ej_pitch(l);
  double* const G = IN_LDS ? ej_smem : work;
  double* const nrm2 = ej_smem + (IN_LDS ? (size_t)pitch * l : 0);     // squared column norms
  double* const lam = nrm2 + l;                                        // eigenvalues at the end
  int* const order = (int*)(lam + l + 8);
  __shared__ int rotated, k_eff;

  const int t = threadIdx.x;
  const int grp = t >> 4, li = t & 15;
  const int np = l + (l & 1);          // even number of players; index l (if any) is a bye
  const int half = np / 2;

  // G = A (column p of G = row p of A), rows past l zero
  for (int e = t; e < l * pitch; e += EJ_THREADS) {
    const int p = e / pitch, r = e - p * pitch;
    G[e] = r < l ? A[(int64_t)p * l + r] : 0.0;
  }
  __syncthreads();

  // ---- A = L L^T in place (column j of L in column j of G, rows j .. l-1); 16 lanes per column
  {
    double dmax = 0.0;
    for (int p = li; p < l; p += 16) dmax = fmax(dmax, G[p * pitch + p]);
#pragma unroll
    for (int off = 8; off > 0; off >>= 1) dmax = fmax(dmax, __shfl_xor(dmax, off, 16));
    const double thresh = (double)l * 2.220446049250313e-16 * dmax;
    for (int j = 0; j < l; ++j) {
      const double d = G[j * pitch + j];                  // final since the previous step's barrier
      const bool usable = d > thresh;
      const double rs = usable ? 1.0 / sqrt(d) : 0.0;
      __syncthreads();                                    // everyone has read the pivot
      for (int r = j + t; r < l; r += EJ_THREADS) {       // the diagonal becomes sqrt(d) = d / sqrt(d)
        const double v = G[j * pitch + r];
        G[j * pitch + r] = (r == j) ? d * rs : v * rs;
      }
      __syncthreads();
      if (usable) {
        for (int c = j + 1 + grp; c < l; c += EJ_GROUPS) {
          const double lcj = G[j * pitch + c];
          for (int r = c + li; r < l; r += 16) G[c * pitch + r] = fma(-lcj, G[j * pitch + r], G[c * pitch + r]);
        }
      }
      __syncthreads();
    }
    // the part above the diagonal still holds A: L is lower triangular
    for (int e = t; e < l * pitch; e += EJ_THREADS) {
      const int p = e / pitch, r = e - p * pitch;
      if (r < p) G[e] = 0.0;
    }
    __syncthreads();
  }

  for (int sweep = 0; sweep < EJ_MAX_SWEEPS; ++sweep) {
    // squared norms afresh once per sweep (they are updated by formula in between)
    for (int p = grp; p < l; p += EJ_GROUPS) {
      double s = 0.0;
      for (int r = li; r < l; r += 16) { const double v = G[p * pitch + r]; s += v * v; }
      s = ej_group_sum(s);
      if (li == 0) nrm2[p] = s;
    }
    if (t == 0) rotated = 0;
    __syncthreads();

    for (int round = 0; round < np - 1; ++round) {
      bool any = false;
      for (int i = grp; i < half; i += EJ_GROUPS) {
        int p = round + i;                          // both below 2 (np - 1): one subtraction reduces them
        if (p >= np - 1) p -= np - 1;
        int q = round + np - 1 - i;
        if (q >= np - 1) q -= np - 1;
        if (i == 0) q = np - 1;
        if (p > q) { const int tmp = p; p = q; q = tmp; }
        if (q >= l) continue;                       // bye
        double gp[NR], gq[NR];
        double c = 0.0;
#pragma unroll
        for (int j = 0; j < NR; ++j) {
          const int r = li + 16 * j;
          const bool on = r < pitch;
          gp[j] = on ? G[p * pitch + r] : 0.0;
          gq[j] = on ? G[q * pitch + r] : 0.0;
          c = fma(gp[j], gq[j], c);
        }
        c = ej_group_sum(c);
        const double a = nrm2[p], b = nrm2[q];
        // (every lane of the group holds the same bits of a, b and c: the test is uniform in the group)
        if (!(c * c > (EJ_ROT_TOL * EJ_ROT_TOL) * a * b) || a == 0.0 || b == 0.0) continue;
        double cs, sn, tt;
        ej_rotation(a, b, c, &cs, &sn, &tt);
        const double a2 = fmax(a - tt * c, 0.0), b2 = fmax(b + tt * c, 0.0);
        const bool swap = a2 < b2;                  // the longer column to the lower index
        const int pw = swap ? q : p, qw = swap ? p : q;
#pragma unroll
        for (int j = 0; j < NR; ++j) {
          const int r = li + 16 * j;
          if (r < pitch) {
            G[pw * pitch + r] = cs * gp[j] - sn * gq[j];
            G[qw * pitch + r] = sn * gp[j] + cs * gq[j];
          }
        }
        if (li == 0) {
          nrm2[pw] = a2;
          nrm2[qw] = b2;
        }
        any = true;
      }
      if (any && li == 0) rotated = 1;
      __syncthreads();
    }
    const int again = rotated;
    __syncthreads();
    if (!again) break;
  }

  // eigenvalues = squared column norms
  for (int p = grp; p < l; p += EJ_GROUPS) {
    double s = 0.0;
    for (int r = li; r < l; r += 16) { const double v = G[p * pitch + r]; s += v * v; }
    s = ej_group_sum(s);
    if (li == 0) lam[p] = s;                        // |g_p|^2 = sigma_p^2 = lambda_p
  }
  __syncthreads();
  // rank them (descending, ties by index)
  for (int i = t; i < l; i += EJ_THREADS) {
    const double vi = lam[i];
    int rank = 0;
    for (int j = 0; j < l; ++j) {
      const double vj = lam[j];
      rank += (vj > vi) || (vj == vi && j < i);
    }
    order[rank] = i;
  }
  __syncthreads();
  if (t == 0) {
    int keep = k;
    if (k_out) {
      double total = 0.0;
      for (int i = 0; i < l; ++i) total += sqrt(lam[order[i]]);
      double run = 0.0;
      keep = l;
      for (int i = 0; i < l; ++i) {
        run += sqrt(lam[order[i]]);
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
    double v = 0.0;
    if (c < k_eff) {
      const double nv = lam[order[c]];
      if (nv > 0.0) v = G[order[c] * pitch + r] / sqrt(nv);
    }
    Wk[e] = v;
  }
}

template <int NR>
static int launch_jacobi_nr(hipStream_t s, const double* A, double* work, double* Wk, int l, int k,
                            double energy, int32_t* k_out) {
  if (ej_fits_lds(l)) {
    const size_t lds = ej_lds_bytes(l);
    static std::atomic<bool> attr_done{false};
    if (lds > 64 * 1024 && !attr_done.load(std::memory_order_acquire)) {
      hipError_t e = hipFuncSetAttribute((const void*)jacobi_eig_kernel<NR, true>,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, EJ_LDS_LIMIT);
      if (e != hipSuccess) return hip_fail(e, "hipFuncSetAttribute(eigensolver LDS)");
      attr_done.store(true, std::memory_order_release);
    }
    LORACT_LAUNCH("jacobi_eig", s, (jacobi_eig_kernel<NR, true>), dim3(1), dim3(EJ_THREADS), lds, A, work, Wk,
                  l, k, energy, k_out);
  } else {
    const size_t lds = ej_small_bytes(l);
    LORACT_LAUNCH("jacobi_eig", s, (jacobi_eig_kernel<NR, false>), dim3(1), dim3(EJ_THREADS), lds, A, work, Wk,
                  l, k, energy, k_out);
  }
  return LORACT_OK;
}

// A (l x l, read only), work (ej_work_doubles(l) doubles, used above the LDS limit), Wk (l x k out).
static int launch_jacobi_eig(hipStream_t s, const double* A, double* work, double* Wk, int l, int k,
                             double energy = 1.0, int32_t* k_out = nullptr) {
  if (l < 1 || l > LORACT_MAX_RANK || k < 1 || k > l) return LORACT_ERR_INVALID_ARG;
  const int nr = (ej_pitch(l) + 15) / 16;
  if (nr <= 3) return launch_jacobi_nr<3>(s, A, work, Wk, l, k, energy, k_out);
  if (nr <= 6) return launch_jacobi_nr<6>(s, A, work, Wk, l, k, energy, k_out);
  if (nr <= 10) return launch_jacobi_nr<10>(s, A, work, Wk, l, k, energy, k_out);
  if (nr <= 15) return launch_jacobi_nr<15>(s, A, work, Wk, l, k, energy, k_out);
  return launch_jacobi_nr<21>(s, A, work, Wk, l, k, energy, k_out);
}
