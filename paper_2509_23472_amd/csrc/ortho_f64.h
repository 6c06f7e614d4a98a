// Tall-skinny orthonormalisation kernels of the bf16 path: Gram matrix, Cholesky factor and
// triangular solve, all accumulated in float64 on the gfx950 matrix cores
// (v_mfma_f64_16x16x4_f64) without LDS staging of the operands.
//
// Layout conventions used below (verified on the device):
//   A operand (16 x 4):  lane l holds A[m = l % 16][kk = l / 16]
//   B operand (4 x 16):  lane l holds B[kk = l / 16][n = l % 16]
//   C/D      (16 x 16):  register r of lane l holds D[m = 4 r + l / 16][n = l % 16]
// so an accumulator can be fed back as the B operand of a later product whose contraction
// index is the accumulator's row index: slice r (kk = 4 r .. 4 r + 3) is register r.
//
// The sketch Y and the intermediate Q1 are stored as m x kp float32 with kp = k rounded up to a
// multiple of 16; columns k..kp-1 are zero.  The Gram matrix / Cholesky factor is kp x kp.
#pragma once
#include "common.h"

#define OF_NB 16
#ifndef GRAM_TARGET_WGS
#define GRAM_TARGET_WGS 256
#endif
#ifndef OF_RSQ_STEPS
#define OF_RSQ_STEPS 1
#endif


__device__ inline f64x4 mfma_f64(double a, double b, f64x4 c) {
  return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
}

// ---------------------------------------------------------------------------------------------
// Gram matrix G = Y^T Y (lower 64 x 64 blocks only), rows split into chunks; one workgroup per
// (chunk, block), each of its 4 waves owning a 32 x 32 sub-block (2 x 2 MFMA tiles).
// part[(chunk * nblocks + block) * 4096 + i * 64 + j] holds the chunk's contribution.

struct GramArgs {
  const float* Y;
  int64_t ldy;
  int64_t m;
  int kp;
  int rows_per_chunk;   // multiple of 4
  int nb64;             // number of 64-wide block rows = ceil(kp / 64)
  double* part;
};

__device__ inline void gram_block_of(int b, int* bi, int* bj) {
  int i = 0;
  while ((i + 1) * (i + 2) / 2 <= b) ++i;
  *bi = i;
  *bj = b - i * (i + 1) / 2;
}

__global__ __launch_bounds__(256) void gram_mfma_kernel(GramArgs g) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int bi, bj;
  gram_block_of(blockIdx.y, &bi, &bj);
  const int wi = wave >> 1, wj = wave & 1;
  const int ca = bi * 64 + wi * 32;   // first Gram row (a column of Y) of this wave's sub-block
  const int cb = bj * 64 + wj * 32;
  const int64_t r_begin = (int64_t)blockIdx.x * g.rows_per_chunk;
  const int64_t r_end = (r_begin + g.rows_per_chunk < g.m) ? r_begin + g.rows_per_chunk : g.m;
  const int lc = lane & 15, lr = lane >> 4;

  f64x4 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = (f64x4){0.0, 0.0, 0.0, 0.0};

  const bool a_ok0 = ca + lc < g.kp, a_ok1 = ca + 16 + lc < g.kp;
  const bool b_ok0 = cb + lc < g.kp, b_ok1 = cb + 16 + lc < g.kp;
  const int ca_c0 = a_ok0 ? ca + lc : 0, ca_c1 = a_ok1 ? ca + 16 + lc : 0;
  const int cb_c0 = b_ok0 ? cb + lc : 0, cb_c1 = b_ok1 ? cb + 16 + lc : 0;
  // 16 rows per trip.  The 16 loads of a trip are unconditional, from clamped (in-bounds, hence
  // finite) addresses, and zeroed by a multiplication: a select would put the load under a
  // branch, where it is waited for on the spot.
  const float ma0 = a_ok0 ? 1.0f : 0.0f, ma1 = a_ok1 ? 1.0f : 0.0f;
  const float mb0 = b_ok0 ? 1.0f : 0.0f, mb1 = b_ok1 ? 1.0f : 0.0f;
  float fa0[4][4], fa1[4][4], fb0[4][4], fb1[4][4];
  auto load_trip = [&](int64_t r0, float* pa0, float* pa1, float* pb0, float* pb1) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int64_t row = r0 + 4 * u + lr;
      const bool rok = row < r_end;
      const float* yr = g.Y + (rok ? row : r_begin) * g.ldy;
      pa0[u] = yr[ca_c0];
      pa1[u] = yr[ca_c1];
      pb0[u] = yr[cb_c0];
      pb1[u] = yr[cb_c1];
    }
  };
  // the masks are applied here, at the point of use, so that nothing touches a loaded value
  // (and waits for it) before the trip that consumes it
  auto mac_trip = [&](int64_t r0, const float* pa0, const float* pa1, const float* pb0,
                      const float* pb1) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const float rm = (r0 + 4 * u + lr < r_end) ? 1.0f : 0.0f;
      const double a0 = (double)(pa0[u] * (rm * ma0)), a1 = (double)(pa1[u] * (rm * ma1));
      const double b0 = (double)(pb0[u] * (rm * mb0)), b1 = (double)(pb1[u] * (rm * mb1));
      acc[0][0] = mfma_f64(a0, b0, acc[0][0]);
      acc[0][1] = mfma_f64(a0, b1, acc[0][1]);
      acc[1][0] = mfma_f64(a1, b0, acc[1][0]);
      acc[1][1] = mfma_f64(a1, b1, acc[1][1]);
    }
  };
  // ring of 4 trips: the loads run 3 trips (48 rows) ahead of the matrix instructions.  Loads past
  // the end of the chunk are harmless (clamped addresses) and are not multiplied.
#pragma unroll
  for (int p = 0; p < 3; ++p) load_trip(r_begin + 16 * p, fa0[p], fa1[p], fb0[p], fb1[p]);
  for (int64_t r0 = r_begin; r0 < r_end; r0 += 64) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      load_trip(r0 + 16 * (q + 3), fa0[(q + 3) & 3], fa1[(q + 3) & 3], fb0[(q + 3) & 3], fb1[(q + 3) & 3]);
      if (r0 + 16 * q < r_end) mac_trip(r0 + 16 * q, fa0[q], fa1[q], fb0[q], fb1[q]);
    }
  }
  double* out = g.part + ((int64_t)blockIdx.x * gridDim.y + blockIdx.y) * 4096;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r)
        out[(wi * 32 + i * 16 + 4 * r + lr) * 64 + wj * 32 + j * 16 + lc] = acc[i][j][r];
}

// G[i][j] (lower triangle, kp x kp) = sum over chunks, ascending.  One thread per element.
// Optional by-products for the second round (ns_T != null): with E = G - I restricted to the
// live k x k part, T = -E/2 as a full symmetric bf16 matrix (pad rows/columns zero), and this
// workgroup's share of ||E||_F^2 in ns_e2[workgroup] (an off-diagonal block counts twice, for its
// mirror image).  The consumer adds the shares in index order.
__global__ __launch_bounds__(256) void gram_reduce_kernel(const double* part, int chunks,
                                                          int nblocks, int kp, int k, double* G,
                                                          double* G_copy, bf16_t* ns_T,
                                                          double* ns_e2, int32_t* clear_word) {
  __shared__ double red[4];
  // (the progress word of a fused factor-and-solve launch that follows starts at zero)
  if (clear_word && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *clear_word = 0;
  const int b = blockIdx.y;
  int bi, bj;
  gram_block_of(b, &bi, &bj);
  // four lanes per element: lane `sub` adds the chunks sub, sub + 4, ... in ascending order and the
  // four sums are combined as (s0 + s1) + (s2 + s3), a fixed order whatever the chunk count
  const int sub = threadIdx.x & 3;
  const int e = blockIdx.x * 64 + (threadIdx.x >> 2);     // gridDim.x = 64
  const int i = bi * 64 + (e >> 6), j = bj * 64 + (e & 63);
  double contrib = 0.0;
  if (i < kp && j < kp) {
    const double* src = part + (int64_t)b * 4096 + e;
    const int64_t stride = (int64_t)nblocks * 4096;
    double s = 0.0;
    int c = sub;
    for (; c + 28 < chunks; c += 32) {
      double v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = src[(int64_t)(c + 4 * u) * stride];
#pragma unroll
      for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; c < chunks; c += 4) s += src[(int64_t)c * stride];
    s += __shfl_xor(s, 1);
    s += __shfl_xor(s, 2);
    if (sub == 0) {
      G[(int64_t)i * kp + j] = s;
      if (G_copy) G_copy[(int64_t)i * kp + j] = s;
      if (ns_e2) {
        if (bi != bj) G[(int64_t)j * kp + i] = s;        // round 2 leaves the whole symmetric matrix

        double ev = 0.0;
        if (i < k && j < k) ev = s - (i == j ? 1.0 : 0.0);
        if (ns_T) {
          const bf16_t tv = (bf16_t)(float)(-0.5 * ev);
          ns_T[(int64_t)i * kp + j] = tv;
          if (bi != bj) ns_T[(int64_t)j * kp + i] = tv;
        }
        contrib = (bi == bj) ? ev * ev : 2.0 * ev * ev;
      }
    }
  }
  if (ns_e2) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) contrib += __shfl_xor(contrib, off);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = contrib;
    __syncthreads();
    if (threadIdx.x == 0) ns_e2[blockIdx.y * gridDim.x + blockIdx.x] = red[0] + red[1] + red[2] + red[3];
  }
}

// ---------------------------------------------------------------------------------------------
// Blocked Cholesky factorisation G (+ shift) = L L^T of the kp x kp Gram matrix by one workgroup.
// Two kernels: chol_reg_kernel (further down: kp <= 256, matrix in registers, what the benchmark
// shapes use) and chol_blocked_kernel (any kp, matrix updated in place in global memory).
//
// chol_blocked_kernel, per 16-column panel: every wave holds the 16 diagonal-block rows
// redundantly in lanes 0..15 and up to 48 rows below in lanes 16..63, one row per lane with its 16
// panel entries in registers; the 16 pivot steps then need no workgroup barrier, only wave-wide
// lane reads.  The trailing lower triangle is updated per 16 x 16 block on the matrix cores.
//
// Outputs: L in the strict lower triangle of G (global), and Dinv[b] = inverse of the b-th
// 16 x 16 diagonal block of L (row-major, lower triangular), which is what the triangular solve
// in trsm_apply_kernel consumes.
//
// Pivot rule: see chol.h.  Columns k..kp-1 are padding: their reciprocal pivot is whatever the
// rule gives (zero without a shift) and they never raise the status flag.

__device__ inline double readlane_f64(double v, int src_lane) {
  union { double d; int i[2]; } u;
  u.d = v;
  u.i[0] = __builtin_amdgcn_readlane(u.i[0], src_lane);
  u.i[1] = __builtin_amdgcn_readlane(u.i[1], src_lane);
  return u.d;
}

// 1 / sqrt(x) to float64 accuracy: the hardware estimate (relative error below ~2^-22) refined by
// third-order steps y <- y (1 + e/2 + 3 e^2/8), e = 1 - x y^2, each of which cubes the error.
template <int STEPS>
__device__ inline double rsqrt_f64(double x) {
  double y = __builtin_amdgcn_rsq(x);
#pragma unroll
  for (int it = 0; it < STEPS; ++it) {
    const double e = fma(-x * y, y, 1.0);
    y = fma(y * fma(0.375, e, 0.5), e, y);
  }
  return y;
}


// chol_blocked_kernel runs 8 waves to overlap the memory latency of the trailing-block updates.
//
// round == 1 (Gram matrix of the sketch): the factorisation is first attempted WITHOUT a shift;
//   a pivot that is not above unshifted_thresh * G[j][j] (a small multiple of the rounding level
//   k u) abandons the attempt and the matrix is factored again as G + s I, s = shift_rel * trace
//   (the matrix is restored from G_backup).  Unshifted factors leave
//   Q1 = Y R^{-1} orthonormal to ~u cond(G); shifted ones only well conditioned (see chol.h).
// round == 2 (Gram matrix of Q1): if ns_flag is given, E = G - I is measured first.  When
//   ||E||_F <= ns_tol the factorisation is skipped (T = -E/2 was already written by
//   gram_reduce_kernel) and *ns_flag = 1, so that the caller finishes with the first-order Newton-Schulz correction
//   Q = Q1 (I - E/2), whose defect is ~ (3/4) ||E||^2.  When ||E||_F <= ns_exact_tol, Q1 is taken as
//   it is (*ns_flag = 2: no second round at all).  Otherwise *ns_flag = 0 and the matrix is
//   factored unshifted with the clamping rule of chol.h.
struct CholArgs {
  double* G;
  const double* G_backup;
  double* Dinv;
  int k, kp;
  int round;
  double tol;               // round 2 clamping level
  double shift_rel;         // round 1 shift (second attempt)
  double unshifted_thresh;  // round 1 breakdown level of the unshifted attempt (0 = always shift)
  int32_t* status;
  const double* ns_e2;      // round 2: shares of ||E||_F^2 from gram_reduce_kernel
  int ns_e2_count;
  int32_t* ns_flag;
  double ns_tol;            // Newton-Schulz finish up to this ||E||_F (0 = not available)
  double ns_exact_tol;      // Q1 accepted unchanged up to this ||E||_F
  const double* poly_p4;    // optional: shares of ||E^4||_F^2 from ns_poly_finish_kernel
  int poly_count;
  double poly_hi_tol;       // the polynomial finish was attempted for ||E||_F in (ns_tol, poly_hi_tol]
  double poly_b4_tol;       // ... and is accepted when ||E^4||_F^(1/4) (>= ||E||_2) is at most this
  int32_t* ready;           // fused factor-and-solve launch only: progress word read by the solving workgroups
};

// Progress word of the fused factor-and-solve launch: (attempt << 16) | panels, where `panels` = p
// means that block rows 0 .. p-1 of L (left of the diagonal) and the inverted diagonal blocks
// 0 .. p-1 are complete in memory, and `attempt` counts restarts of the factorisation (a solving
// workgroup that sees it change starts over: what it consumed so far belongs to the abandoned
// attempt).  The producer writes L, Dinv and the word with device-scope write-through stores
// and waits for their completion before it advances the word; consumers read with device-scope
// loads.  No read-modify-write and no cache write-back is involved.
#define CF_ATTEMPT_SHIFT 16
__device__ inline void cf_store(double* p, double v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void cf_publish(int32_t* ready, int attempt, int panels) {
  __hip_atomic_store(ready, (attempt << CF_ATTEMPT_SHIFT) | panels, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline int cf_poll(const int32_t* ready) {
  return __hip_atomic_load(ready, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Round 2 decision, taken by the whole workgroup before any factorisation work: E = G - I has been
// measured by gram_reduce_kernel (||E||_F^2 in pieces, T = -E/2 already written).  Returns true,
// with *ns_flag set, when no second factorisation is needed; misc is an LDS scratch of 4 doubles.
__device__ inline bool chol_round2_exit(const CholArgs& g, double* misc, const bool write_flag = true) {
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  // wave 0 adds the shares (lane i takes shares i, i + 64, ...; butterfly sum, so every lane
  // ends with the same value) and hands the total to the other waves through LDS
  if (wave == 0) {
    double part_sum = 0.0;
    for (int w0 = lane; w0 < g.ns_e2_count; w0 += 256) {      // four loads in flight, no branch around them
      double v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int w = w0 + 64 * u;
        v[u] = g.ns_e2[w < g.ns_e2_count ? w : g.ns_e2_count - 1] * (w < g.ns_e2_count ? 1.0 : 0.0);
      }
      part_sum += (v[0] + v[1]) + (v[2] + v[3]);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) part_sum += __shfl_xor(part_sum, off);
    if (lane == 0) misc[1] = part_sum;
  }
  __syncthreads();
  const double tot = misc[1];
  if (tot <= g.ns_exact_tol * g.ns_exact_tol) {     // Q1 is orthonormal as it stands
    if (t == 0 && write_flag) *g.ns_flag = 2;
    return true;
  }
  if (g.ns_tol > 0.0 && tot <= g.ns_tol * g.ns_tol) {       // comparisons are false for NaN
    if (t == 0 && write_flag) *g.ns_flag = 1;
    return true;
  }
  if (g.ns_tol > 0.0 && g.poly_count > 0 && tot <= g.poly_hi_tol * g.poly_hi_tol) {
    // the degree-4 correction was prepared (T holds it): accept it if the spectral norm of E,
    // bounded by ||E^4||_F^(1/4), keeps the truncated series accurate
    if (wave == 0) {
      double part_sum = 0.0;
      for (int w = lane; w < g.poly_count; w += 64) part_sum += g.poly_p4[w];
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) part_sum += __shfl_xor(part_sum, off);
      if (lane == 0) misc[2] = part_sum;
    }
    __syncthreads();
    const double b4 = sqrt(sqrt(sqrt(misc[2])));
    if (b4 <= g.poly_b4_tol) {
      if (t == 0 && write_flag) *g.ns_flag = 1;
      return true;
    }
  }
  if (t == 0 && write_flag) *g.ns_flag = 0;
  return false;
}

__global__ __launch_bounds__(512) void chol_blocked_kernel(CholArgs g) {
  constexpr int CHOL_THREADS = 512;
  double* const G = g.G;
  double* const Dinv = g.Dinv;
  const int k = g.k, kp = g.kp;
  const double tol = g.tol;
  int32_t* const status = g.status;
  extern __shared__ double smem[];
  // layout: gdiag[kp] | dinv[kp] | misc[8] | Pt[16][kp - 16]
  double* gdiag = smem;            // original diagonal
  double* dinv = smem + kp;        // reciprocal pivots
  double* misc = smem + 2 * kp;    // [0] = shift
  const int ptld = kp > OF_NB ? kp - OF_NB : 2;
  double* Pt = smem + 2 * kp + 8;  // panel below the diagonal block, transposed: Pt[p][row - below]
  double* Am = G;
  const int lda = kp;
  __shared__ int deficient, restart;

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  if (t == 0) { deficient = 0; restart = 0; }
  __syncthreads();

  // ---- round 2: is Q1 already orthonormal enough for a Newton-Schulz finish?  On that branch
  // the kernel ends here.
  if (g.round == 2 && g.ns_flag && chol_round2_exit(g, misc)) return;

  for (int i = t; i < kp; i += CHOL_THREADS) gdiag[i] = G[(int64_t)i * kp + i];
  __syncthreads();

  double trace_sum = 0.0;
  if (wave == 0) {
    double tr = 0.0;
    for (int i = lane; i < kp; i += 64) tr += gdiag[i];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) tr += __shfl_xor(tr, off);
    if (lane == 0) misc[0] = tr;
  }
  __syncthreads();
  trace_sum = misc[0];

  const bool try_unshifted = g.round == 1 && g.unshifted_thresh > 0.0;
  for (int attempt = try_unshifted ? 0 : 1; attempt < 2; ++attempt) {
  const bool unshifted_attempt = g.round == 1 && attempt == 0;
  const double shift = (g.round == 1 && attempt == 1) ? g.shift_rel * trace_sum : 0.0;
  if (attempt == 1 && try_unshifted) {
    // the unshifted attempt broke down: restore the matrix and start over with the shift
      for (int e = t; e < kp * kp; e += CHOL_THREADS) G[e] = g.G_backup[e];
    
    if (t == 0) restart = 0;
    __syncthreads();
  }

  for (int jb = 0; jb < kp; jb += OF_NB) {
    const int below = jb + OF_NB;
    const int nrows_below = kp - below;

    // ---- panel: one row per lane, its 16 panel entries in registers.  Lanes 0..15 of every
    // wave hold the diagonal block (redundantly), lanes 16..63 hold 48 of the rows below.
    // 4 waves x 48 rows per pass; a second pass (kp > 208) reuses the saved diagonal block
    constexpr int NWAVES = CHOL_THREADS / 64;
    const int npass = nrows_below > 0 ? (nrows_below + 48 * NWAVES - 1) / (48 * NWAVES) : 1;
    double dsave[OF_NB];
    double thr[OF_NB], gdiag_reg[OF_NB];
#pragma unroll
    for (int c = 0; c < OF_NB; ++c) {
      double v = 0.0;
      if (lane < 16 && c <= lane) v = Am[(jb + lane) * lda + jb + c];
      if (lane < 16 && c == lane) v += shift;
      dsave[c] = v;
      gdiag_reg[c] = gdiag[jb + c];
      thr[c] = tol * gdiag_reg[c];
    }
    // the first pass's rows below are fetched together with the diagonal block, before the barrier:
    // one memory round trip per panel instead of two (they are written only after it)
    double afirst[OF_NB];
    {
      const int row = below + wave * 48 + lane - 16;
      const bool on = lane >= 16 && row < kp;
#pragma unroll
      for (int c = 0; c < OF_NB; ++c) afirst[c] = on ? Am[row * lda + jb + c] : 0.0;
    }
    __syncthreads();   // every wave has read the unfactored diagonal block
    for (int pass = 0; pass < npass; ++pass) {
    const int row = (lane < 16) ? (jb + lane) : (below + (pass * NWAVES + wave) * 48 + lane - 16);
    const bool row_ok = row < kp;
    double a[OF_NB];
    if (pass == 0) {
#pragma unroll
      for (int c = 0; c < OF_NB; ++c) a[c] = (lane < 16) ? dsave[c] : afirst[c];
    } else {
#pragma unroll
      for (int c = 0; c < OF_NB; ++c)
        a[c] = (lane < 16) ? dsave[c] : (row_ok ? Am[row * lda + jb + c] : 0.0);
    }
    double dval[OF_NB];
    bool any_bad = false;
#pragma unroll
    for (int j = 0; j < OF_NB; ++j) {
      const double piv = readlane_f64(a[j], j);
      const bool live = jb + j < k;                      // padding columns never count
      bool usable;
      if (unshifted_attempt) usable = piv > g.unshifted_thresh * gdiag_reg[j];
      else if (g.round == 1) usable = piv > 0.0;
      else usable = piv > thr[j];
      const double d = (usable && live) ? rsqrt_f64<OF_RSQ_STEPS>(piv) : 0.0;
      dval[j] = d;
      any_bad = any_bad || (!usable && live);
      a[j] *= d;
#pragma unroll
      for (int c = j + 1; c < OF_NB; ++c) {
        const double lcj = readlane_f64(a[j], c);
        a[c] = fma(-a[j], lcj, a[c]);
      }
    }
    if (lane >= 16) {
      if (row_ok) {
#pragma unroll
        for (int c = 0; c < OF_NB; ++c) {
          Am[row * lda + jb + c] = a[c];
          Pt[c * ptld + row - below] = a[c];
        }
      }
    } else if (wave == 0 && pass == 0) {   // wave 0 owns the diagonal block
#pragma unroll
      for (int c = 0; c < OF_NB; ++c)
        if (c < lane) Am[row * lda + jb + c] = a[c];
      if (lane == 0) {
#pragma unroll
        for (int j = 0; j < OF_NB; ++j) dinv[jb + j] = dval[j];
        if (any_bad) {
          if (unshifted_attempt) restart = 1; else deficient = 1;
        }
      }
    }
    }
    __syncthreads();
    if (restart) break;          // uniform: written before the barrier

    // ---- trailing update of the lower triangle: A[I][C] -= P_I P_C^T per 16 x 16 block (C <= I),
    // on the float64 matrix cores, the panel read from Pt.
    {
      const int nb16 = nrows_below / OF_NB;
      const int nblocks = nb16 * (nb16 + 1) / 2;
      const int lc = lane & 15, lr = lane >> 4;
      // Several blocks per wave and trip: the loads of all their accumulators are issued before
      // the first matrix instruction, so that their latency (LDS, or L2 when the matrix lives in
      // global memory) is paid once per trip.  The panel operands come from LDS at the point of use.
      constexpr int NWV = CHOL_THREADS / 64, TB = 4;
      for (int e0 = wave; e0 < nblocks; e0 += NWV * TB) {
        double* ablk[TB];
        int ta[TB], tb[TB];
        f64x4 acc[TB];
#pragma unroll
        for (int b = 0; b < TB; ++b) {
          const int e = e0 + b * NWV;
          const int ee = e < nblocks ? e : e0;            // idle slots redo the first block's loads
          int ti = (int)((sqrtf(8.0f * (float)ee + 1.0f) - 1.0f) * 0.5f);
          while (ti * (ti + 1) / 2 > ee) --ti;
          while ((ti + 1) * (ti + 2) / 2 <= ee) ++ti;
          const int tc = ee - ti * (ti + 1) / 2;
          ta[b] = OF_NB * ti + lc;
          tb[b] = OF_NB * tc + lc;
          ablk[b] = Am + (below + OF_NB * ti + lr) * lda + below + OF_NB * tc + lc;
#pragma unroll
          for (int r = 0; r < 4; ++r) acc[b][r] = ablk[b][4 * r * lda];
        }
#pragma unroll
        for (int b = 0; b < TB; ++b) {
#pragma unroll
          for (int r = 0; r < 4; ++r)
            acc[b] = mfma_f64(-Pt[(4 * r + lr) * ptld + ta[b]], Pt[(4 * r + lr) * ptld + tb[b]], acc[b]);
        }
#pragma unroll
        for (int b = 0; b < TB; ++b) {
          if (e0 + b * NWV < nblocks) {
#pragma unroll
            for (int r = 0; r < 4; ++r) ablk[b][4 * r * lda] = acc[b][r];
          }
        }
      }
    }
    __syncthreads();
  }
  if (!restart) break;
  __syncthreads();
  }

  // ---- inverses of the 16 x 16 diagonal blocks, one thread per (block, column c):
  // column c of L_bb^{-1} by forward substitution in update form (x_j is final after step j and
  // is then subtracted from all later rows at once, so the 15 steps carry a two-operation chain).
  const int nblk = kp / OF_NB;
  for (int e = t; e < nblk * OF_NB; e += CHOL_THREADS) {
    const int b = e >> 4, c = e & 15;
    const int base = b * OF_NB;
    double acc[OF_NB], x[OF_NB];
#pragma unroll
    for (int r = 0; r < OF_NB; ++r) acc[r] = (r == c) ? 1.0 : 0.0;
#pragma unroll
    for (int j = 0; j < OF_NB; ++j) {
      const double xj = (j >= c) ? acc[j] * dinv[base + j] : 0.0;
      x[j] = xj;
#pragma unroll
      for (int r = j + 1; r < OF_NB; ++r) acc[r] = fma(-Am[(base + r) * lda + base + j], xj, acc[r]);
    }
#pragma unroll
    for (int r = 0; r < OF_NB; ++r) Dinv[((int64_t)b * OF_NB + r) * OF_NB + c] = x[r];
  }
  if (t == 0 && deficient && status) atomicOr(status, LORACT_STATUS_RANK_DEFICIENT);
}

// ---------------------------------------------------------------------------------------------
// Register-resident blocked Cholesky for kp <= 256: one workgroup of 8 waves, the matrix never
// touches LDS or global memory between panels.
//
// Storage.  The symmetric matrix is kept as its UPPER 16 x 16 blocks U(C, I) = G[C rows][I cols],
// C <= I, each in the accumulator layout of the float64 matrix instruction, dealt round-robin in
// row-major order to the 7 worker waves (so every suffix C > j, the trailing matrix of panel j, and
// every block row C == j, the panel itself, are spread evenly).  In that layout register r of a
// block is at once slice r of the B operand of a product contracting over the block's rows, so
//   panel j:     P_I^T = Linv_j U(j, I)            (P_I = L[I rows][j cols], 4 matrix instructions)
//   trailing:    U(C, I) -= P_C P_I^T              (operands from LDS, accumulated in place)
// need no layout change at all.  P^T goes to LDS (Pt) for the trailing update and to global
// memory as L.  Within a block the rows are permuted: register r of lane group q holds row 4 q + r
// (the hardware's natural order would be q + 4 r), so that a lane's four registers are 32
// contiguous bytes of a row of G and the blocks are loaded with full cache lines; the permutation
// is undone where it matters, in the row index of the A operand of the trailing update.
//
// Look-ahead.  Wave 0 owns the serial part.  While the workers apply panel j to the trailing
// matrix, wave 0 takes the next diagonal block (staged in LDS by its owner one iteration earlier),
// applies panel j to it, factors it one row per lane, and leaves L_bb and Linv_bb in LDS, from
// where two workers copy them out.  Lanes 16..31 carry the rows of the identity through the same
// 16 pivot steps, which turns them into the rows of L^{-T}: the inverse costs nothing extra.
// Two workgroup barriers per panel; wave 0's pivot steps are the critical path and everything
// else hides behind them once the trailing matrix is small enough.
//
// In round 1 the original matrix is read from G_backup (required: the unshifted attempt may have
// to start over with the shift after L has begun to overwrite G), in round 2 from G.
// Pivot rules, outputs (L in the strict lower triangle of G, Dinv) and the round-2 early exits are
// those of chol_blocked_kernel, except that padding columns get a unit diagonal (their rows and
// columns of L are zero either way).
#define CR_THREADS 512
#define CR_WORKERS 7

static inline int chol_reg_ptld(int kp) {
  const int w = kp > OF_NB ? kp - OF_NB : OF_NB;
  return (w % 32 == 16) ? w : w + 16;        // consecutive panel rows start 128 bytes apart (mod 256)
}
// LDS doubles: misc[8] | LinvT[2][16][17] | Ltile[2][16][17] | Dstage[2][256] | Dtile[16][17] |
//              Colbuf[2][64] | gdiag[kp] | Pt[16][ptld]
static inline size_t chol_reg_lds_bytes(int kp) {
  return sizeof(double) * (size_t)(8 + 544 + 544 + 512 + 272 + 128 + kp + OF_NB * chol_reg_ptld(kp));
}

// PUB: the factor is published panel by panel for the solving workgroups of the same launch
// (chol_trsm_fused_kernel): write-through stores and the progress word g.ready.
template <int SLOTS, bool PUB>
__device__ inline void chol_reg_body(const CholArgs& g, const int ptld, double* smem) {
  double* const G = g.G;
  // (round 2 never starts over, and its caller's backup, if any, is round 1's matrix)
  const double* const src = (g.round == 1 && g.G_backup) ? g.G_backup : g.G;
  const int k = g.k, kp = g.kp, nb = kp / OF_NB;
  // (the fixed-size pieces come first, so that their addresses are compile-time constants)
  double* misc = smem;                 // [0] trace, [1], [2] round-2 decision
  double* LinvT = smem + 8;            // [b & 1][c * 17 + i] = Linv_bb[i][c]
  double* Ltile = LinvT + 544;         // [b & 1][r * 17 + c] = L_bb[r][c]
  double* Dstage = Ltile + 544;        // next diagonal blocks, accumulator layout, two buffers
  double* Dtile = Dstage + 512;        // wave 0: diagonal block turned to one row per lane
  double* Colbuf = Dtile + 272;        // wave 0: the two latest scaled columns of the diagonal block
  double* gdiag = Colbuf + 128;        // original diagonal (wave 0 only)
  double* Pt = gdiag + kp;             // Pt[p * ptld + x] = L[below + x][16 j + p]
  __shared__ int deficient, restart;

  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int lc = lane & 15, lr = lane >> 4;
  const int pm = 4 * (lc & 3) + (lc >> 2);   // accumulator row of logical row lc, and back
  if (t == 0) { deficient = 0; restart = 0; }
  __syncthreads();
  // (in the fused launch every workgroup has taken the round-2 decision before it got here)
  if (!PUB && g.round == 2 && g.ns_flag && chol_round2_exit(g, misc)) return;

  // ---- block ownership: worker w holds blocks e = s * 7 + w of the row-major upper triangle
  // without block (0, 0), which wave 0 reads itself
  // (packed as C | I << 8; an unused slot names block (0, 0), which no condition below selects)
  int ci[SLOTS];
  {
    const int total = nb * (nb + 1) / 2 - 1;
    int c = 0, rem = wave;                 // block e + 1 = rem-th of block row c, carried from slot to slot
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
      const int e = s * CR_WORKERS + wave - 1;
      while (c < nb && rem >= nb - c) { rem -= nb - c; ++c; }
      ci[s] = (wave > 0 && e < total) ? (c | ((c + rem) << 8)) : 0;
      rem += CR_WORKERS;
    }
  }
  // Unpacking goes through an empty volatile asm so that nothing derived from a slot's block
  // coordinates is hoisted out of the panel loop (20 slots' worth of addresses would spill).
#define CR_SLOT(s, C, I)                       \
  int ci_ = ci[s];                             \
  asm volatile("" : "+s"(ci_));                \
  const int C = ci_ & 255, I = ci_ >> 8
  // Block (C, I) as it lies in memory: lane (q, n) takes G[16 I + n][16 C + 4 q .. + 3]
#define CR_LOAD_BLOCK(dst, C, I)                                                              \
  {                                                                                           \
    const double* p_ = src + (int64_t)(OF_NB * (I) + lc) * kp + OF_NB * (C) + 4 * lr;          \
    const double2 v0_ = *(const double2*)p_, v1_ = *(const double2*)(p_ + 2);                  \
    dst[0] = v0_.x; dst[1] = v0_.y; dst[2] = v1_.x; dst[3] = v1_.y;                            \
  }
  // Diagonal entries of a diagonal block: the shift, and 1 on the padding columns
#define CR_FIX_DIAG(dst, C)                                                                   \
  _Pragma("unroll") for (int r_ = 0; r_ < 4; ++r_)                                            \
    if (4 * lr + r_ == lc) dst[r_] = (OF_NB * (C) + lc < k) ? dst[r_] + shift : 1.0;

  // Round 1 starts with the unshifted attempt (the launcher sends anything else to
  // chol_blocked_kernel), so the shift is needed on a second attempt only, long after wave 0 has
  // left the trace in LDS.
  const bool try_unshifted = g.round == 1;
  int attempt_pub = 0;                 // attempt number as the solving workgroups count it
  for (int attempt = try_unshifted ? 0 : 1; attempt < 2; ++attempt) {
    attempt_pub = (try_unshifted && attempt == 1) ? 1 : 0;
    const bool unshifted_attempt = g.round == 1 && attempt == 0;
    const double shift = (g.round == 1 && attempt == 1) ? g.shift_rel * misc[0] : 0.0;
    if (PUB && attempt_pub == 1 && t == 64) cf_publish(g.ready, 1, 0);   // the solvers start over

    // The two roles run separate loops with the same sequence of barriers, so that the workers'
    // blocks and wave 0's pivot rows never compete for registers.
    if (wave == 0) {
      // ---- wave 0: factor diagonal block b, given in the accumulator layout
      auto factor_diag = [&](const int b, const f64x4 dacc) {
#pragma unroll
        for (int r = 0; r < 4; ++r) Dtile[(4 * lr + r) * 17 + lc] = dacc[r];
        __builtin_amdgcn_wave_barrier();      // LDS operations of one wave complete in order
        double a[OF_NB];
#define CR_LOAD_ROWS()                                                           \
  _Pragma("unroll") for (int c = 0; c < OF_NB; ++c) {                            \
    const double v = Dtile[lc * 17 + c];                                         \
    a[c] = (lane < 16) ? v : ((lane < 32 && lc == c) ? 1.0 : 0.0);               \
  }
        CR_LOAD_ROWS();
        // lane c: the level pivot c has to exceed (one rule for the three cases)
        const double level = unshifted_attempt ? g.unshifted_thresh : (g.round == 1 ? 0.0 : g.tol);
        const double thl = level * gdiag[OF_NB * b + lc];
        // one opaque base register for all broadcast reads (otherwise every address becomes a
        // hoisted constant of its own)
        typedef const __attribute__((address_space(3))) double* lds_cptr;
        unsigned colofs = (unsigned)(uintptr_t)(lds_cptr)Colbuf;
        asm volatile("" : "+v"(colofs));
        const lds_cptr colbase = (lds_cptr)(uintptr_t)colofs;

        // ---- The 16 pivot steps, fast form.  One wave issues in order and a dependent float64
        // operation costs it tens of cycles, so what counts is the number of DEPENDENT operations
        // from one pivot to the next.  Here that chain is seven long and runs on wave-uniform
        // values held in vector registers:
        //   y = rsq(piv);  e = 1 - piv y^2;  q = e (1/2 + 3e/8)     (1/sqrt(piv) = y (1 + q))
        //   l = l0 y (1 + q)        l0 = entry (jj+1, jj), read from its lane BEFORE the step
        //   piv' = p0 - l^2         p0 = entry (jj+1, jj+1), likewise
        // while the lanes scale their own row entry the same way (bitwise the same arithmetic as
        // l) and apply the rank-1 update off the chain: columns jj+1 and jj+2 at once (with l and
        // one lane read), the others one step later with multipliers read back from LDS (column
        // jj is written there once scaled; one address for all lanes is a broadcast read).  Every
        // column is therefore complete two steps before it holds the pivot, which is what allows
        // l0 and p0 to be read early.  No operation on the chain tests the pivot: padding columns
        // carry a unit diagonal, and a pivot that fails its test is only recorded (the block is
        // then redone by the guarded form below).
        bool any_bad = false;
        {
          double pivv = readlane_f64(a[0], 0);
          double y = __builtin_amdgcn_rsq(pivv);
#pragma unroll
          for (int jj = 0; jj < OF_NB; ++jj) {
            const bool live = OF_NB * b + jj < k;
            any_bad = any_bad || (live && !(pivv > readlane_f64(thl, jj)));
            double l0 = 0.0, p0 = 0.0;
            if (jj + 1 < OF_NB) {
              l0 = readlane_f64(a[jj], jj + 1);
              p0 = readlane_f64(a[jj + 1], jj + 1);
            }
            double mult[OF_NB];
            if (jj > 0) {
              const lds_cptr col = colbase + ((jj - 1) & 1) * 64;
#pragma unroll
              for (int c = jj + 2; c < OF_NB; ++c) mult[c] = col[c];
            }
            const double s0 = a[jj] * y, ls0 = l0 * y;
            const double tq = pivv * y;
            const double eq = fma(-tq, y, 1.0);
            const double q = eq * fma(0.375, eq, 0.5);
            a[jj] = fma(s0, q, s0);
            if (jj + 1 < OF_NB) {
              const double l = fma(ls0, q, ls0);
              pivv = fma(-l, l, p0);
              y = __builtin_amdgcn_rsq(pivv);
              a[jj + 1] = fma(-a[jj], l, a[jj + 1]);
            }
            Colbuf[(jj & 1) * 64 + lane] = a[jj];
            if (jj + 2 < OF_NB) {
              const double ln2 = readlane_f64(a[jj], jj + 2);
              a[jj + 2] = fma(-a[jj], ln2, a[jj + 2]);
            }
            if (jj > 0) {
#pragma unroll
              for (int c = jj + 2; c < OF_NB; ++c) a[c] = fma(-a[jj - 1], mult[c], a[c]);
            }
          }
        }
        // ---- guarded form, only after a pivot failed its test (and the factorisation goes on:
        // an unshifted attempt is abandoned anyway): unusable and padding columns get a zero
        // reciprocal, so that they drop out of L and of Linv instead of spreading NaN.
        if (any_bad && !unshifted_attempt) {
          CR_LOAD_ROWS();
          double piv = readlane_f64(a[0], 0);
          double y = __builtin_amdgcn_rsq(piv);
#pragma unroll
          for (int jj = 0; jj < OF_NB; ++jj) {
            const bool live = OF_NB * b + jj < k;
            const bool usable = piv > readlane_f64(thl, jj);
            const double tq = piv * y;
            const double eq = fma(-tq, y, 1.0);
            const double hq = y * fma(0.375, eq, 0.5);
            const double d = (usable && live) ? fma(hq, eq, y) : 0.0;
            a[jj] *= d;
#pragma unroll
            for (int c = jj + 1; c < OF_NB; ++c) {
              const double lcj = readlane_f64(a[jj], c);
              a[c] = fma(-a[jj], lcj, a[c]);
            }
            if (jj + 1 < OF_NB) {
              piv = readlane_f64(a[jj + 1], jj + 1);
              y = __builtin_amdgcn_rsq(piv);
            }
          }
        }
#undef CR_LOAD_ROWS
        // lanes 0..15 hold the rows of L_bb, lanes 16..31 the rows of L_bb^{-T}: both to LDS, one
        // store instruction per column (two workers copy them to global memory later)
        if (lane < 32) {
          double* base = ((lane < 16) ? Ltile : LinvT) + (b & 1) * 272 + lc * 17;
#pragma unroll
          for (int c = 0; c < OF_NB; ++c) base[c] = a[c];
        }
        if (lane == 0 && any_bad) {
          if (unshifted_attempt) restart = 1; else deficient = 1;
        }
      };

      __builtin_amdgcn_s_setprio(3);
      {
        // block (0, 0), and on the first pass the diagonal (pivot thresholds) with its sum (the
        // shift of a second attempt), fetched in one memory round trip
        f64x4 first;
        if (attempt == 0 || !try_unshifted) {
          // (addresses are formed here, from a pitch the compiler cannot see through: hoisted out
          // of the attempt loop they are spilled, and every reload then drains the load queue)
          int kpo = kp;
          asm volatile("" : "+s"(kpo));
          double dg[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) {       // unconditional loads (a load under a branch is waited for on the spot)
            const int i = lane + 64 * q, ic = i < kp ? i : kp - 1;
            dg[q] = src[(int64_t)ic * kpo + ic];
          }
          CR_LOAD_BLOCK(first, 0, 0);
          double tr = 0.0;
#pragma unroll
          for (int q = 0; q < 4; ++q) {       // branch-free (a branch would pull the load into it): lanes
            const int i = lane + 64 * q;      // past the end rewrite the last entry with its own value
            gdiag[i < kp ? i : kp - 1] = dg[q];
            tr += dg[q] * (i < kp ? 1.0 : 0.0);
          }
#pragma unroll
          for (int off = 32; off > 0; off >>= 1) tr += __shfl_xor(tr, off);
          if (lane == 0) misc[0] = tr;
        } else {
          CR_LOAD_BLOCK(first, 0, 0);
        }
        CR_FIX_DIAG(first, 0);
        factor_diag(0, first);
      }
      __syncthreads();
      // (the flag is made wave-uniform for the compiler)
      for (int j = 0; j < nb - 1 && !__builtin_amdgcn_readfirstlane(restart); ++j) {
        __syncthreads();                      // panel j is in Pt
        const int b = j + 1;
        f64x4 dacc;
#pragma unroll
        for (int r = 0; r < 4; ++r) dacc[r] = Dstage[(b & 1) * 256 + r * 64 + lane];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          const double* prow = Pt + (4 * kk + lr) * ptld;
          dacc = mfma_f64(-prow[pm], prow[lc], dacc);
        }
        factor_diag(b, dacc);
        __syncthreads();                      // restart, if set, was written before this barrier
      }
      __builtin_amdgcn_s_setprio(0);
    } else {
      // ---- workers load their blocks (all loads are issued before the first use)
      f64x4 acc[SLOTS];
#pragma unroll
      for (int s = 0; s < SLOTS; ++s) {
        CR_SLOT(s, C, I);
        CR_LOAD_BLOCK(acc[s], C, I);
      }
#pragma unroll
      for (int s = 0; s < SLOTS; ++s) {
        CR_SLOT(s, C, I);
        if (C == I) {
          CR_FIX_DIAG(acc[s], C);
          if (C == 1) {                       // wave 0 takes it after block (0, 0)
#pragma unroll
            for (int r = 0; r < 4; ++r) Dstage[256 + r * 64 + lane] = acc[s][r];
          }
        }
      }
      // Block b's factors, left in LDS by wave 0, to global memory: Dinv by wave 1, L_bb by wave 2
      auto copy_out = [&](const int b) {
        if (wave == 1) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int e = lane + 64 * q;      // Dinv[b][c][i] = Linv[c][i] = LinvT[i][c]
            const double dv = LinvT[(b & 1) * 272 + (e & 15) * 17 + (e >> 4)];
            if (PUB) cf_store(g.Dinv + (int64_t)b * 256 + e, dv); else g.Dinv[(int64_t)b * 256 + e] = dv;
          }
        } else if (wave == 2) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int e = lane + 64 * q, r = e >> 4, c = e & 15;
            if (c < r) {
              const double lv = Ltile[(b & 1) * 272 + r * 17 + c];
              if (PUB) cf_store(G + (int64_t)(OF_NB * b + r) * kp + OF_NB * b + c, lv);
              else G[(int64_t)(OF_NB * b + r) * kp + OF_NB * b + c] = lv;
            }
          }
        }
      };
      __syncthreads();
      int jdone = -1;                         // last panel whose factors were copied out
      for (int j = 0; j < nb - 1 && !__builtin_amdgcn_readfirstlane(restart); ++j) {
        // (published factors leave first, so that their stores are old by the end of the trip)
        if (PUB) copy_out(j);
        // ---- phase A: the rows of panel j, P_I^T = Linv_j U(j, I), to LDS and to L
        double la[4];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) la[kk] = LinvT[(j & 1) * 272 + (4 * lr + kk) * 17 + lc];
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
          CR_SLOT(s, C, I);
          if (C == j && I > j) {
            f64x4 d = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) d = mfma_f64(la[kk], acc[s][kk], d);
            const int x0 = OF_NB * (I - j - 1) + lc;
            double* lrow = G + (int64_t)(OF_NB * I + lc) * kp + OF_NB * j + lr;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              Pt[(lr + 4 * r) * ptld + x0] = d[r];
              if (PUB) cf_store(lrow + 4 * r, d[r]); else lrow[4 * r] = d[r];
            }
          }
        }
        __syncthreads();

        // ---- phase B: panel j applied to the trailing matrix (wave 0 factors block j + 1)
        const int b = j + 1;
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
          CR_SLOT(s, C, I);
          if (C > j && !(C == b && I == b)) {
            const int xc = OF_NB * (C - j - 1) + pm, xi = OF_NB * (I - j - 1) + lc;
            // The product is formed on its own and then subtracted: accumulating into acc[s]
            // directly makes the compiler keep an old and a new copy of every block across this
            // branch (the matrix instruction's destination may not overlap a live source).
            f64x4 d = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
              d = mfma_f64(Pt[(4 * kk + lr) * ptld + xc], Pt[(4 * kk + lr) * ptld + xi], d);
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[s][r] -= d[r];
            if (C == I && C == b + 1) {       // the diagonal block wave 0 takes next
#pragma unroll
              for (int r = 0; r < 4; ++r) Dstage[(C & 1) * 256 + r * 64 + lane] = acc[s][r];
            }
          }
        }
        if (!PUB) copy_out(j);                // its LDS copy is overwritten two panels later
        jdone = j;
        if (PUB) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's share of panel j is in memory
        __syncthreads();
        // block row j + 1 of L (its last piece was panel j) and Dinv up to block j are complete
        if (PUB && t == 64 && !restart) cf_publish(g.ready, attempt_pub, j + 1);
      }
      // the blocks not copied yet: the last one factored, and the one before it if the loop did
      // not run for it (their LDS buffers differ)
      if (!__builtin_amdgcn_readfirstlane(restart)) {
        for (int b = jdone + 1; b < nb; ++b) copy_out(b);
      }
    }
    if (!__builtin_amdgcn_readfirstlane(restart)) break;
    __syncthreads();                          // everyone has seen the flag
    if (t == 0) restart = 0;
    __syncthreads();
  }
#undef CR_SLOT
#undef CR_LOAD_BLOCK
#undef CR_FIX_DIAG
  if (PUB) {
    // the last factors were copied out after the loop: once every wave's stores are complete the
    // whole of L and Dinv is published (attempt 1 if the unshifted one was abandoned)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (t == 64) cf_publish(g.ready, attempt_pub, nb);
  }
  if (t == 0 && deficient && g.status) atomicOr(g.status, LORACT_STATUS_RANK_DEFICIENT);
}

template <int SLOTS>
__global__ __launch_bounds__(CR_THREADS) void chol_reg_kernel(CholArgs g, int ptld) {
  extern __shared__ double smem[];
  chol_reg_body<SLOTS, false>(g, ptld, smem);
}

// ---------------------------------------------------------------------------------------------
// Q = Y R^{-1} with R = L^T, as a blocked triangular solve per 16-row strip (one wave each):
//   for J = 0 .. NJ-1:   T = Y[:, J] - sum_{I < J} Q[:, I] R[I, J];   Q[:, J] = T R[J, J]^{-1}
// evaluated transposed (Q_J^T = Linv_JJ (Y_J^T - sum_I L[J, I] Q_I^T)) so that each finished
// 16 x 16 block of Q^T stays in the accumulator layout and is reused directly as the B operand.

struct TrsmArgs {
  const float* Y;       // m x kp, ld = ldy
  int64_t ldy;
  const double* L;      // kp x kp, strict lower triangle valid
  const double* Dinv;   // NJ blocks of 16 x 16
  int64_t m;
  int kp;
  int k;
  void* Q;              // output
  int64_t ldq;
  int out_ek;           // EK_F32 (all kp columns written) or EK_BF16 / EK_F32 final (k columns)
  int out_cols;         // number of columns to write (kp or k)
  bf16_t* Qb;           // optional second bf16 copy (ld = ldqb, out_cols columns), may be null
  int64_t ldqb;
  const int32_t* skip_flag;   // optional: the launch does nothing when *skip_flag != 0
};

// Workgroup = WAVES waves = 16 WAVES rows of Y.  The operands every wave needs -- block row J of
// L left of the diagonal and the inverted diagonal block, together "panel J", 16 x 16 (J + 1)
// doubles -- are staged in LDS once per workgroup by asynchronous global -> LDS copies instead of
// being fetched by every wave:
//   panels 0 .. J0-1 (J0 = min(NJ, 8), 6 for the widest) are copied up front, side by side in one 16-row array;
//   panel J + 1 >= J0 is copied into the other half of a double buffer while step J runs.
// The LDS row pitches are 2 modulo 32 doubles (or 18), which spreads the 16 rows that one matrix
// instruction operand touches over distinct banks.
#define TRSM_J0(NJ) ((NJ) < 8 ? (NJ) : ((NJ) > 16 ? 6 : 8))
#define TRSM_TILE_FLOATS (16 * 20)     // per-wave staging tile for the stores: 16 rows, pitch 20 floats
#define TRSM_SPIN_LIMIT (1 << 22)      // polls of the progress word before a solving workgroup gives up

// FUSED = false: L and Dinv are complete when the kernel starts (a launch of its own).
// FUSED = true: the workgroup runs beside the factorisation (chol_trsm_fused_kernel) and takes
// panel J when the progress word says it is complete: no panel is copied up front, panel J goes to
// half J & 1 of the double buffer, and panel J + 1 is copied ahead only if it is complete already.
// A change of the attempt number sends the workgroup back to J = 0.  `wg` is the workgroup's index
// among the solving workgroups, `lds` its dynamic LDS.
template <int NJ, int WAVES, bool FUSED>
__device__ inline void trsm_body(const TrsmArgs& g, const int first_strip, const int strip_stride,
                                 double* trsm_lds, const int32_t* ready, int32_t* status) {
  constexpr int J0 = FUSED ? 0 : TRSM_J0(NJ);
  constexpr int PK = 8 * J0 * (J0 + 1) + 2;           // pitch of the side-by-side array, in doubles
  constexpr int PR = 16 * NJ + 2;                     // pitch of a double-buffer half
  double* const ring = trsm_lds + (FUSED ? 0 : 16 * PK);
  float* const tile = (float*)(ring + (NJ > J0 ? 32 * PR : 0)) + (threadIdx.x >> 6) * TRSM_TILE_FLOATS;
  int* const word = (int*)((float*)(ring + (NJ > J0 ? 32 * PR : 0)) + WAVES * TRSM_TILE_FLOATS);   // FUSED: the progress word as the workgroup saw it
  if (g.skip_flag && *g.skip_flag != 0) return;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int lc = lane & 15, lr = lane >> 4;
  const int nstrips = (int)((g.m + 16 * WAVES - 1) / (16 * WAVES));
  // 4 consecutive output columns per lane can be stored as one vector
  const bool vec_ok = (g.ldq & 3) == 0 && ((uintptr_t)g.Q & 15) == 0 &&
                      (!g.Qb || ((g.ldqb & 3) == 0 && ((uintptr_t)g.Qb & 7) == 0));

  // Copy of panel J to `dst` (pitch in doubles): one wave-wide instruction per (panel row, 64
  // pieces of 16 bytes), dealt round-robin to the waves; lanes past the row end stay idle.
  // (FUSED: device-scope loads, the panel was written by another workgroup of this launch.)
  auto copy_panel = [&](int J, double* dst, int pitch) {
    const int pieces = 8 * (J + 1);
    const int nq = (pieces + 63) / 64;
    for (int e = wave; e < 16 * nq; e += WAVES) {
      const int r = e / nq, q = e - r * nq;
      const int c = 2 * (64 * q + lane);
      if (c < 16 * (J + 1)) {
        const double* src = c < 16 * J ? g.L + (int64_t)(16 * J + r) * g.kp + c
                                        : g.Dinv + ((int64_t)J * 16 + r) * 16 + (c - 16 * J);
        if (FUSED) sb_async16_device(src, (unsigned char*)(dst + r * pitch) + q * 1024);
        else sb_async16(src, (unsigned char*)(dst + r * pitch) + q * 1024);
      }
    }
  };
  // FUSED: the whole workgroup learns the progress word (one poll per trip, shared through LDS);
  // returns it once panel J of attempt `att` is complete or the attempt has changed
  auto wait_panel = [&](int J, int att) -> int {
    int f = 0;
    for (int spin = 0; spin < TRSM_SPIN_LIMIT; ++spin) {
      if (t == 0) *word = cf_poll(ready);
      sb_barrier_lds();
      f = *word;
      sb_barrier_lds();                  // everyone has read the word before the next poll rewrites it
      if ((f >> CF_ATTEMPT_SHIFT) != att || (f & 0xffff) > J) return f;
      __builtin_amdgcn_s_sleep(8);
    }
    return -1;
  };

  if (!FUSED) {
#pragma unroll
    for (int J = 0; J < J0; ++J) copy_panel(J, trsm_lds + 8 * J * (J + 1), PK);
    SB_WAIT_VMCNT(0);
    __syncthreads();
  }

  f64x4 qb[NJ];
  float ycur[4], ynext[4];
  int att = 0;
  int known = 0;                       // FUSED: the progress word as last seen (uniform in the workgroup)
  bool restart_solve;
  // A workgroup takes the strips first_strip, first_strip + strip_stride, ... of 16 WAVES rows one
  // after the other (FUSED: fewer workgroups than strips when the matrix is tall; once the progress
  // word has been seen complete no strip polls again).  A restart of the factorisation sends the
  // workgroup back to its first strip: everything it wrote so far belongs to the abandoned attempt.
  for (int strip = first_strip; strip < nstrips; strip += strip_stride) {
  const int64_t row = (int64_t)strip * (16 * WAVES) + wave * 16 + lc;
  const bool rok = row < g.m;
  // every row of the wave exists: its store instructions per step can be counted
  const bool full_wave = (int64_t)strip * (16 * WAVES) + wave * 16 + 15 < g.m;
  const float* yrow = g.Y + (rok ? row : 0) * g.ldy;   // rows past m read row 0 and are never stored
  do {
    restart_solve = false;
    bool next_copied = false;
#pragma unroll
    for (int r = 0; r < 4; ++r) ycur[r] = yrow[4 * r + lr];
#pragma unroll
    for (int J = 0; J < NJ; ++J) {
      if (FUSED) {
        if (restart_solve) continue;                     // (uniform) the attempt changed: drain the unrolled loop
        int f = known;
        if ((f >> CF_ATTEMPT_SHIFT) != att || (f & 0xffff) <= J) {
          f = wait_panel(J, att);
          if (f < 0) {                                   // the factorisation never got here: give up, flagged
            if (t == 0 && status) atomicOr(status, LORACT_STATUS_INTERNAL);
            return;
          }
          known = f;
        }
        if ((f >> CF_ATTEMPT_SHIFT) != att) { att = f >> CF_ATTEMPT_SHIFT; restart_solve = true; continue; }
        if (!next_copied) copy_panel(J, ring + (J & 1) * 16 * PR, PR);
        next_copied = false;
        if (J + 1 < NJ) {
#pragma unroll
          for (int r = 0; r < 4; ++r) ynext[r] = yrow[16 * (J + 1) + 4 * r + lr];
        }
        SB_WAIT_VMCNT(4);                                 // the panel's copies are older than the 4 loads of ynext
        if (J + 1 >= NJ) SB_WAIT_VMCNT(0);
        sb_barrier_lds();                                // everyone's share of panel J landed
        if (J + 1 < NJ && (f & 0xffff) > J + 1) {        // the next panel is complete as well: copy it ahead
          copy_panel(J + 1, ring + ((J + 1) & 1) * 16 * PR, PR);
          next_copied = true;
        }
      } else {
        const bool ring_next = J + 1 >= J0 && J + 1 < NJ;
        if (ring_next) copy_panel(J + 1, ring + ((J + 1) & 1) * 16 * PR, PR);
        if (J + 1 < NJ) {
#pragma unroll
          for (int r = 0; r < 4; ++r) ynext[r] = yrow[16 * (J + 1) + 4 * r + lr];
        }
      }
      const double* pan = (!FUSED && J < J0) ? trsm_lds + lc * PK + 8 * J * (J + 1) : ring + (J & 1) * 16 * PR + lc * PR;
      f64x4 s = (f64x4){0.0, 0.0, 0.0, 0.0};
#pragma unroll
      for (int I = 0; I < J; ++I) {
#pragma unroll
        for (int r = 0; r < 4; ++r) s = mfma_f64(pan[16 * I + 4 * r + lr], qb[I][r], s);
      }
      f64x4 tt;
#pragma unroll
      for (int r = 0; r < 4; ++r) tt[r] = (double)ycur[r] - s[r];
      f64x4 o = (f64x4){0.0, 0.0, 0.0, 0.0};
#pragma unroll
      for (int r = 0; r < 4; ++r) o = mfma_f64(pan[16 * J + 4 * r + lr], tt[r], o);
      qb[J] = o;
      if (vec_ok && 16 * J + 16 <= g.out_cols) {
        // The 16 x 16 block is turned through a wave-private LDS tile (LDS operations of one wave
        // execute in order) so that every lane stores 4 consecutive columns at once.
#pragma unroll
        for (int r = 0; r < 4; ++r) tile[lc * 20 + 4 * r + lr] = (float)o[r];
        const f32x4 v = *(const f32x4*)(tile + lc * 20 + 4 * lr);
        bf16x4 vh;
#pragma unroll
        for (int u = 0; u < 4; ++u) vh[u] = (bf16_t)v[u];
        if (rok) {
          const int col = 16 * J + 4 * lr;
          if (g.out_ek == EK_F32) *(f32x4*)((float*)g.Q + row * g.ldq + col) = v;
          else *(bf16x4*)((bf16_t*)g.Q + row * g.ldq + col) = vh;
          if (g.Qb) *(bf16x4*)(g.Qb + row * g.ldqb + col) = vh;
        }
      } else if (rok) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int col = 16 * J + 4 * r + lr;
          if (col < g.out_cols) {
            if (g.out_ek == EK_F32) ((float*)g.Q)[row * g.ldq + col] = (float)o[r];
            else ((bf16_t*)g.Q)[row * g.ldq + col] = (bf16_t)(float)o[r];
            if (g.Qb) g.Qb[row * g.ldqb + col] = (bf16_t)(float)o[r];
          }
        }
      }
      if (J + 1 < NJ) {
#pragma unroll
        for (int r = 0; r < 4; ++r) ycur[r] = ynext[r];
      }
      if (FUSED) {
        // the stores of this step and a copy issued ahead may stay in flight; the next trip's
        // wait_panel barriers order this trip's reads of the buffer half before its refill
        if (next_copied) SB_WAIT_VMCNT(0);
      } else if (J + 1 >= J0 && J + 1 < NJ) {
        // The copies of panel J + 1 are older than this step's stores (1 per wave on the vector
        // path, 2 with the second output; every column of a step that is not the last lies inside
        // out_cols), so they have landed once at most that many operations are pending.  The barrier also orders this step's
        // reads of its buffer half before the copy that the next step issues into it.
        if (!full_wave || !vec_ok) SB_WAIT_VMCNT(0);
        else if (g.Qb) SB_WAIT_VMCNT(2);
        else SB_WAIT_VMCNT(1);
        sb_barrier_lds();
      }
    }
  } while (FUSED && restart_solve && strip == first_strip);
  if (FUSED) {
    sb_barrier_lds();                  // this strip's last reads of the buffer halves precede the next strip's copies
    if (restart_solve) strip = first_strip - strip_stride;      // (uniform) back to the first strip
  }
  }
}

template <int NJ, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void trsm_apply_kernel(TrsmArgs g) {
  extern __shared__ __attribute__((aligned(16))) double trsm_lds[];
  trsm_body<NJ, WAVES, false>(g, blockIdx.x, gridDim.x, trsm_lds, nullptr, nullptr);
}

template <int NJ, int WAVES, bool FUSED>
static constexpr size_t trsm_lds_bytes() {
  constexpr int J0 = FUSED ? 0 : TRSM_J0(NJ);
  return ((size_t)(FUSED ? 0 : 16 * (8 * J0 * (J0 + 1) + 2)) + (NJ > J0 ? (size_t)32 * (16 * NJ + 2) : 0)) *
             sizeof(double) + (size_t)WAVES * TRSM_TILE_FLOATS * sizeof(float) + 16;
}

template <int NJ, int WAVES>
static int launch_trsm_nj_waves(hipStream_t s, const TrsmArgs& g) {
  constexpr size_t lds = trsm_lds_bytes<NJ, WAVES, false>();
  static std::atomic<bool> attr_done{false};
  if (lds > 64 * 1024 && !attr_done.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute((const void*)trsm_apply_kernel<NJ, WAVES>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return hip_fail(e, "hipFuncSetAttribute(trsm LDS)");
    attr_done.store(true, std::memory_order_release);
  }
  LORACT_LAUNCH("trsm_apply", s, (trsm_apply_kernel<NJ, WAVES>),
                dim3((unsigned)ceil_div64(g.m, 16 * WAVES)), dim3(64 * WAVES), lds, g);
  return LORACT_OK;
}

// ---------------------------------------------------------------------------------------------
// Factorisation and triangular solve of round 1 in ONE launch: workgroup 0 factors the Gram
// matrix (chol_reg_body, publishing), workgroups 1 .. solve their 128 rows of Y panel by panel
// as the factor appears, so that the solve costs one panel step after the factorisation ends
// instead of a launch of its own after it.  Workgroup 0 waits for nobody, and is dispatched
// first, so the others' bounded waits cannot starve it.  The progress word must be zero when the
// launch starts (an earlier kernel of the same call clears it).
template <int SLOTS, int NJ>
__global__ __launch_bounds__(CR_THREADS) void chol_trsm_fused_kernel(CholArgs c, int ptld, TrsmArgs g) {
  extern __shared__ __attribute__((aligned(16))) double fused_lds[];
  // Round 2: whether Q1 needs a second factorisation at all is decided from the shares of
  // ||E||_F^2 that the Gram reduction left -- by every workgroup for itself, with the same
  // arithmetic in the same order, so that on the usual exits (Newton-Schulz finish, or Q1 accepted
  // as it is) the whole launch ends after one look at those few hundred numbers and nobody waits
  // for anybody.  Workgroup 0 records the decision in *ns_flag.
  if (c.round == 2 && c.ns_flag) {
    if (chol_round2_exit(c, fused_lds, blockIdx.x == 0)) return;
    __syncthreads();
  }
  if (blockIdx.x == 0) chol_reg_body<SLOTS, true>(c, ptld, fused_lds);
  else trsm_body<NJ, CR_THREADS / 64, true>(g, (int)blockIdx.x - 1, (int)gridDim.x - 1, fused_lds, c.ready, c.status);
}

// Few rows: 64 per workgroup so that more CUs take part; many rows: 128, which halves the panel
// traffic per row.
template <int NJ>
static int launch_trsm_nj(hipStream_t s, const TrsmArgs& g) {
  return g.m >= 32768 ? launch_trsm_nj_waves<NJ, 8>(s, g) : launch_trsm_nj_waves<NJ, 4>(s, g);
}

// ---------------------------------------------------------------------------------------------
// Higher-order finish of round 2.  With E = Q1^T Q1 - I symmetric and ||E||_2 < 1,
//   (I + E)^(-1/2) = I - E/2 + 3 E^2/8 - 5 E^3/16 + 35 E^4/128 - ...,
// so Q = Q1 (I + T) with T = -E/2 + 3 E^2/8 - 5 E^3/16 + 35 E^4/128 is orthonormal up to
// ~ (63/128) ||E||_2^5: 1.6e-4 at ||E||_2 = 0.2.  The first-order step T = -E/2 only serves
// ||E|| <= 0.015; with this one a sketch whose Gram matrix loses 14 digits (the long-context
// sites) still needs no second factorisation and no second triangular solve over the m rows.
// Two small launches on k x k matrices in float64: E^2, then E^3, E^4, T (bf16) and the shares of
// ||E^4||_F^2, from which the factorisation kernel bounds ||E||_2 before it accepts T.
// One 16 x 16 tile per wave.  The contraction index is dealt to the lanes in runs of four
// (lane group q of an operand holds columns 16 kb + 4 q .. + 3), the same way for both operands,
// so that every lane reads 32 contiguous bytes and a tile row is one 128-byte line; the second
// operand is read by rows too, all matrices involved being symmetric.

struct NsPolyArgs {
  const double* G;          // Q1^T Q1, full symmetric kp x kp
  double* P2;               // E^2 (kp x kp)
  bf16_t* T;                // out: the correction, kp x kp bf16
  const double* e2;         // shares of ||E||_F^2
  int e2_count;
  double* p4;               // out: one share of ||E^4||_F^2 per workgroup
  int k, kp;
  double lo_tol, hi_tol;    // active for ||E||_F in (lo_tol, hi_tol]
};

__device__ inline bool ns_poly_active(const NsPolyArgs& g, int lane) {
  // lane i adds shares i, i + 64, ... in that order; eight loads at a time are in flight (from
  // clamped indices, masked at use), or the loop is a chain of as many memory latencies
  double part_sum = 0.0;
  for (int w0 = lane; w0 < g.e2_count; w0 += 512) {
    double v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int w = w0 + 64 * u;
      v[u] = g.e2[w < g.e2_count ? w : g.e2_count - 1];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (w0 + 64 * u < g.e2_count) part_sum += v[u];
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) part_sum += __shfl_xor(part_sum, off);
  return part_sum > g.lo_tol * g.lo_tol && part_sum <= g.hi_tol * g.hi_tol;
}

// rows [16 t .. +15], four consecutive columns from c0 of E = G - I (live k x k part, else 0)
__device__ inline f64x4 ns_poly_e4(const NsPolyArgs& g, int row, int c0) {
  f64x4 v = *(const f64x4*)(g.G + (int64_t)row * g.kp + c0);
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    if (c0 + u == row) v[u] -= 1.0;
    if (row >= g.k || c0 + u >= g.k) v[u] = 0.0;
  }
  return v;
}

__global__ __launch_bounds__(256) void ns_poly_square_kernel(NsPolyArgs g) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (!ns_poly_active(g, lane)) return;
  const int nj = g.kp / 16;
  const int tile = blockIdx.x * 4 + wave;
  if (tile >= nj * nj) return;
  const int ti = tile / nj, tj = tile - ti * nj;
  const int lc = lane & 15, lr = lane >> 4;
  f64x4 acc = (f64x4){0.0, 0.0, 0.0, 0.0};
  for (int kb = 0; kb < nj; ++kb) {
    const f64x4 a = ns_poly_e4(g, 16 * ti + lc, 16 * kb + 4 * lr);
    const f64x4 b = ns_poly_e4(g, 16 * tj + lc, 16 * kb + 4 * lr);
#pragma unroll
    for (int r = 0; r < 4; ++r) acc = mfma_f64(a[r], b[r], acc);
  }
#pragma unroll
  for (int r = 0; r < 4; ++r) g.P2[(int64_t)(16 * ti + 4 * r + lr) * g.kp + 16 * tj + lc] = acc[r];
}

__global__ __launch_bounds__(256) void ns_poly_finish_kernel(NsPolyArgs g) {
  __shared__ double red[4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (!ns_poly_active(g, lane)) {                // uniform over the grid: every wave sums the same shares
    // Not prepared: say so in the share itself.  The factorisation kernel adds the shares of
    // ||E||_F^2 in another order and may land on the other side of a threshold by a rounding;
    // an infinite share makes it reject the series instead of reading a stale value.
    if (threadIdx.x == 0) g.p4[blockIdx.x] = __builtin_huge_val();
    return;
  }
  const int nj = g.kp / 16;
  const int tile = blockIdx.x * 4 + wave;
  const bool on = tile < nj * nj;
  const int ti = on ? tile / nj : 0, tj = on ? tile - ti * nj : 0;
  const int lc = lane & 15, lr = lane >> 4;
  f64x4 p3 = (f64x4){0.0, 0.0, 0.0, 0.0}, p4 = (f64x4){0.0, 0.0, 0.0, 0.0};
  for (int kb = 0; kb < nj; ++kb) {
    const f64x4 a = *(const f64x4*)(g.P2 + (int64_t)(16 * ti + lc) * g.kp + 16 * kb + 4 * lr);
    const f64x4 be = ns_poly_e4(g, 16 * tj + lc, 16 * kb + 4 * lr);
    const f64x4 bp = *(const f64x4*)(g.P2 + (int64_t)(16 * tj + lc) * g.kp + 16 * kb + 4 * lr);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      p3 = mfma_f64(a[r], be[r], p3);
      p4 = mfma_f64(a[r], bp[r], p4);
    }
  }
  double share = 0.0;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int row = 16 * ti + 4 * r + lr, col = 16 * tj + lc;
    double e = g.G[(int64_t)row * g.kp + col] - (row == col ? 1.0 : 0.0);
    if (row >= g.k || col >= g.k) e = 0.0;
    const double p2 = g.P2[(int64_t)row * g.kp + col];
    const double tv = -0.5 * e + 0.375 * p2 - 0.3125 * p3[r] + 0.2734375 * p4[r];
    if (on) g.T[(int64_t)row * g.kp + col] = (bf16_t)(float)tv;
    if (on) share += p4[r] * p4[r];
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) share += __shfl_xor(share, off);
  if (lane == 0) red[wave] = share;
  __syncthreads();
  if (threadIdx.x == 0) g.p4[blockIdx.x] = red[0] + red[1] + red[2] + red[3];
}

static inline int ns_poly_blocks(int kp) { return ((kp / 16) * (kp / 16) + 3) / 4; }
static int launch_ns_poly(hipStream_t s, const NsPolyArgs& g) {
  const dim3 grid((unsigned)ns_poly_blocks(g.kp));
  LORACT_LAUNCH("ns_poly_square", s, ns_poly_square_kernel, grid, dim3(256), 0, g);
  LORACT_LAUNCH("ns_poly_finish", s, ns_poly_finish_kernel, grid, dim3(256), 0, g);
  return LORACT_OK;
}

// ---------------------------------------------------------------------------------------------
// Newton-Schulz finish: Q = Q1 + C with C = Q1 (-E/2) (computed by the bf16 matrix-core product
// of the sketch kernel from the bf16 copy of Q1; the correction is O(||E||) small, so bf16 inputs
// cost nothing at the accuracy required).  Runs only when *flag != 0.
__global__ __launch_bounds__(256) void ns_finalize_kernel(const float* Q1, const float* C,
                                                          int64_t m, int kp, int l, void* Q,
                                                          int q_ek, bf16_t* Qb,
                                                          const int32_t* flag) {
  const int mode = *flag;            // 0: the second factorisation ran; 1: Q = Q1 + C; 2: Q = Q1
  if (mode == 0) return;
  const bool add_c = mode == 1;
  const int c4 = kp >> 2;
  const int64_t total = m * c4;
  const bool vec_ok = (l & 3) == 0 && ((uintptr_t)Q & 15) == 0 && ((uintptr_t)Qb & 7) == 0;
  for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256) {
    const int64_t r = e / c4;
    const int c = (int)(e - r * c4) << 2;
    f32x4 q = *(const f32x4*)(Q1 + r * kp + c);
    if (add_c) q += *(const f32x4*)(C + r * kp + c);
    if (vec_ok) {
      // the row pitch l and the base addresses keep groups of four aligned: vector stores
      if (c < l) {
        bf16x4 qh;
#pragma unroll
        for (int u = 0; u < 4; ++u) qh[u] = (bf16_t)q[u];
        if (q_ek == EK_F32) *(f32x4*)((float*)Q + r * l + c) = q;
        else *(bf16x4*)((bf16_t*)Q + r * l + c) = qh;
        if (Qb) *(bf16x4*)(Qb + r * l + c) = qh;
      }
      continue;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (c + u < l) {
        if (q_ek == EK_F32) ((float*)Q)[r * l + c + u] = q[u];
        else ((bf16_t*)Q)[r * l + c + u] = (bf16_t)q[u];
        if (Qb) Qb[r * l + c + u] = (bf16_t)q[u];
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Host-side launchers.

static int gram_rows_per_chunk(int64_t m, int nblocks) {
  // Whole multiples of the 256 CUs (a workgroup's four waves fill the four SIMDs of a CU), so
  // that no CU ends up with one workgroup more than its neighbour: one per CU for short
  // matrices, where the partial blocks are the cost, two for long ones.  At least 32 rows per
  // chunk, at most 256 chunks.
  const int64_t target = m >= 32768 ? 2 * GRAM_TARGET_WGS : GRAM_TARGET_WGS;
  int64_t chunks = std::max<int64_t>(1, target / std::max(1, nblocks));
  chunks = std::min<int64_t>(chunks, 256);
  int64_t rows = ceil_div64(m, chunks);
  rows = std::max<int64_t>(32, ceil_div64(rows, 16) * 16);
  return (int)rows;
}
static int gram_nblocks(int kp) {
  const int nb64 = (kp + 63) / 64;
  return nb64 * (nb64 + 1) / 2;
}
static size_t gram_partial_bytes(int64_t m, int kp) {
  const int nblocks = gram_nblocks(kp);
  const int rows = gram_rows_per_chunk(m, nblocks);
  return (size_t)ceil_div64(m, rows) * nblocks * 4096 * sizeof(double);
}

// ns_e2 needs 64 * gram_nblocks(kp) doubles.
static int launch_gram_mfma(hipStream_t s, const float* Y, int64_t ldy, int64_t m, int kp, int k,
                            double* part, double* G, double* G_copy = nullptr,
                            bf16_t* ns_T = nullptr, double* ns_e2 = nullptr, int32_t* clear_word = nullptr) {
  GramArgs g;
  g.Y = Y; g.ldy = ldy; g.m = m; g.kp = kp;
  g.nb64 = (kp + 63) / 64;
  const int nblocks = gram_nblocks(kp);
  g.rows_per_chunk = gram_rows_per_chunk(m, nblocks);
  g.part = part;
  const int chunks = (int)ceil_div64(m, g.rows_per_chunk);
  LORACT_LAUNCH("gram", s, gram_mfma_kernel, dim3(chunks, nblocks), dim3(256), 0, g);
  LORACT_LAUNCH("gram_reduce", s, gram_reduce_kernel, dim3(64, nblocks), dim3(256), 0,
                (const double*)part, chunks, nblocks, kp, k, G, G_copy, ns_T, ns_e2, clear_word);
  return LORACT_OK;
}

static size_t chol_lds_bytes(int kp) {
  const int ptld = kp > OF_NB ? kp - OF_NB : 2;
  return sizeof(double) * ((size_t)2 * kp + 8 + (size_t)OF_NB * ptld);
}

// Breakdown level of the unshifted first-round attempt: 16 k u (pivots below it are within a
// couple of digits of the rounding noise of the factorisation).
static inline double chol_unshifted_thresh(int k) { return 16.0 * (double)k * 1.1102230246251565e-16; }

static int launch_chol_blocked(hipStream_t s, CholArgs a) {
  a.tol = ((double)a.k * 5.9604644775390625e-08) * ((double)a.k * 5.9604644775390625e-08);
  if (a.round == 1 && a.unshifted_thresh > 0.0 && !a.G_backup) return LORACT_ERR_INVALID_ARG;
  if (a.kp <= 256 && (a.round == 2 || a.unshifted_thresh > 0.0)) {
    const int ptld = chol_reg_ptld(a.kp);
    const size_t lds = chol_reg_lds_bytes(a.kp);
    if (a.kp <= 128)
      LORACT_LAUNCH("chol", s, chol_reg_kernel<5>, dim3(1), dim3(CR_THREADS), lds, a, ptld);
    else
      LORACT_LAUNCH("chol", s, chol_reg_kernel<20>, dim3(1), dim3(CR_THREADS), lds, a, ptld);
    return LORACT_OK;
  }
  LORACT_LAUNCH("chol", s, chol_blocked_kernel, dim3(1), dim3(512), chol_lds_bytes(a.kp), a);
  return LORACT_OK;
}

template <int SLOTS, int NJ>
static int launch_chol_trsm_fused_nj(hipStream_t s, const CholArgs& c, const TrsmArgs& g) {
  const int ptld = chol_reg_ptld(c.kp);
  // At least 81 KB: one workgroup per CU, so that the factorising workgroup -- whose first wave is
  // the critical path of the whole launch -- never shares its CU's issue slots with solving
  // workgroups (measured at 65536 rows, 256 columns: 235 us with two workgroups per CU, 206 us with
  // one).
  const size_t lds = std::max<size_t>(std::max(chol_reg_lds_bytes(c.kp), trsm_lds_bytes<NJ, CR_THREADS / 64, true>()),
                                      81 * 1024);
  static std::atomic<bool> attr_done{false};
  if (!attr_done.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute((const void*)chol_trsm_fused_kernel<SLOTS, NJ>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return hip_fail(e, "hipFuncSetAttribute(fused factor-and-solve LDS)");
    attr_done.store(true, std::memory_order_release);
  }
  // one solving workgroup per CU beside the factorising one; a tall matrix gives each several strips
  const unsigned solvers = (unsigned)std::min<int64_t>(ceil_div64(g.m, 16 * (CR_THREADS / 64)), 255);
  LORACT_LAUNCH("chol_trsm", s, (chol_trsm_fused_kernel<SLOTS, NJ>), dim3(1 + solvers), dim3(CR_THREADS), lds,
                c, ptld, g);
  return LORACT_OK;
}

// One launch per round when the register-resident factorisation applies (kp <= 256; round 1:
// unshifted first attempt); c.ready must have been cleared by an earlier kernel.
// A solving workgroup works strip by strip and a strip needs every panel, so only its first strip
// overlaps the factorisation.  Beyond 32768 rows (more than eight strips per workgroup) that gain
// is smaller than what the one-workgroup-per-CU solver of the fused launch loses against the plain
// one (measured at 65536 rows, 256 columns: 206 us fused, 190 us as two launches).  Round 2
// normally has nothing to factor, and there the single launch that decides for itself always wins.
static bool chol_trsm_fusable(const CholArgs& c, int64_t m) {
  if (c.kp > 256 || !c.ready) return false;
  if (c.round == 2) return true;
  return m <= 32768 && c.unshifted_thresh > 0.0 && c.G_backup;
}
static int launch_chol_trsm_fused(hipStream_t s, CholArgs c, const TrsmArgs& g) {
  c.tol = ((double)c.k * 5.9604644775390625e-08) * ((double)c.k * 5.9604644775390625e-08);
  switch (c.kp / 16) {
#define CF_CASE(N, S) case N: return launch_chol_trsm_fused_nj<S, N>(s, c, g);
    CF_CASE(1, 5) CF_CASE(2, 5) CF_CASE(3, 5) CF_CASE(4, 5) CF_CASE(5, 5) CF_CASE(6, 5) CF_CASE(7, 5) CF_CASE(8, 5)
    CF_CASE(9, 20) CF_CASE(10, 20) CF_CASE(11, 20) CF_CASE(12, 20) CF_CASE(13, 20) CF_CASE(14, 20)
    CF_CASE(15, 20) CF_CASE(16, 20)
#undef CF_CASE
    default: return LORACT_ERR_UNSUPPORTED;
  }
}

static int launch_trsm_apply(hipStream_t s, const TrsmArgs& g) {
  switch (g.kp / 16) {
#define TRSM_CASE(N) case N: return launch_trsm_nj<N>(s, g);
    TRSM_CASE(1) TRSM_CASE(2) TRSM_CASE(3) TRSM_CASE(4) TRSM_CASE(5) TRSM_CASE(6) TRSM_CASE(7)
    TRSM_CASE(8) TRSM_CASE(9) TRSM_CASE(10) TRSM_CASE(11) TRSM_CASE(12) TRSM_CASE(13)
    TRSM_CASE(14) TRSM_CASE(15) TRSM_CASE(16) TRSM_CASE(17) TRSM_CASE(18) TRSM_CASE(19)
    TRSM_CASE(20)
#undef TRSM_CASE
    default: return LORACT_ERR_UNSUPPORTED;
  }
}
