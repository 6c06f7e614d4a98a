// General matrix product with float64 accumulation for the small, accuracy-critical
// contractions of the orthonormalisation (Gram matrices, triangular-factor application), for
// the fp32 input path, and for the thin contractions of the LoRA gradient.
//
//   C[i][j] = alpha * sum_kk opA(i, kk) * opB(j, kk)
//
// Operand addressing as in gemm_bf16.h (K-contiguous with optional row indirection for B, or
// K-strided); element types are chosen at run time (fp32, bf16 or fp64).  One 256-thread
// workgroup computes a 64 x 64 tile, K in slabs of 16 through LDS (the next slab is fetched into
// registers while the current one is multiplied), 4 x 4 outputs per thread.
// blockIdx.z splits K into fp64 partial tiles that reduce_partials_f64 sums in a fixed order.
#pragma once
#include "common.h"

struct GemmF64Args {
  const void* A;
  int64_t lda;
  const void* B;
  int64_t ldb;
  const int32_t* b_rows;
  void* C;
  int64_t ldc;
  double* Cpart;
  int64_t M, N, K;
  int64_t k_per_split;
  double alpha;
  int a_kc, b_kc;
  int a_ek, b_ek, out_ek;
};

#define GD_BM 64
#define GD_BN 64
#define GD_BK 16

// Element (i, kk) of a 64 x 16 operand slab that thread t handles in its step s; K-contiguous
// operands are walked along K by neighbouring threads, K-strided ones along the rows.
__device__ inline void gd_slot(int kc, int t, int s, int* i, int* kk) {
  const int e = t + 256 * s;
  if (kc) { *kk = e & 15; *i = e >> 4; } else { *i = e & 63; *kk = e >> 6; }
}
// The four elements of a slab that a thread brings in.  The loads are unconditional, from indices
// clamped into the matrix (a load under a branch would be waited for on the spot); what lies
// outside is replaced by zero when the values are put into LDS.
template <int EK>
__device__ inline double gd_load(const void* p, int64_t i) {
  if (EK == EK_F32) return (double)((const float*)p)[i];
  if (EK == EK_F64) return ((const double*)p)[i];
  return (double)(float)((const bf16_t*)p)[i];
}
template <int EK>
__device__ inline void gd_fetch_tile(double* v, const void* P, int64_t ld, const int32_t* rows, int kc,
                                     int64_t row0, int64_t nrows, int64_t k0, int64_t kend, int t) {
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    int i, kk;
    gd_slot(kc, t, s, &i, &kk);
    int64_t gr = row0 + i, gk = k0 + kk;
    if (gr > nrows - 1) gr = nrows - 1;
    if (gk > kend - 1) gk = kend - 1;
    const int64_t src_row = (kc && rows) ? (int64_t)rows[gr] : gr;     // (does not depend on the slab)
    v[s] = gd_load<EK>(P, kc ? src_row * ld + gk : gk * ld + gr);
  }
}
__device__ inline void gd_put_tile(double (*Ls)[GD_BM + 1], const double* v, int kc, int64_t row0,
                                   int64_t nrows, int64_t k0, int64_t kend, int t) {
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    int i, kk;
    gd_slot(kc, t, s, &i, &kk);
    Ls[kk][i] = (row0 + i < nrows && k0 + kk < kend) ? v[s] : 0.0;
  }
}

// AEK, BEK: element kinds of the operands (compiled in, so that the loads are not under a branch).
template <int AEK, int BEK>
__global__ __launch_bounds__(256) void gemm_f64_kernel(GemmF64Args g) {
  __shared__ double As[GD_BK][GD_BM + 1];
  __shared__ double Bs[GD_BK][GD_BN + 1];
  const int t = threadIdx.x;
  const int tx = t & 15, ty = t >> 4;
  const int64_t row0 = (int64_t)blockIdx.x * GD_BM;
  const int64_t col0 = (int64_t)blockIdx.y * GD_BN;
  const int64_t kbeg = (int64_t)blockIdx.z * g.k_per_split;
  const int64_t kend = (kbeg + g.k_per_split < g.K) ? kbeg + g.k_per_split : g.K;

  double acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.0;

  // the next slab is on its way to registers while the current one is multiplied
  double va[4], vb[4];
  gd_fetch_tile<AEK>(va, g.A, g.lda, nullptr, g.a_kc, row0, g.M, kbeg, kend, t);
  gd_fetch_tile<BEK>(vb, g.B, g.ldb, g.b_rows, g.b_kc, col0, g.N, kbeg, kend, t);
  for (int64_t k0 = kbeg; k0 < kend; k0 += GD_BK) {
    gd_put_tile(As, va, g.a_kc, row0, g.M, k0, kend, t);
    gd_put_tile(Bs, vb, g.b_kc, col0, g.N, k0, kend, t);
    __syncthreads();
    // (after the last slab this fetches clamped elements that nobody uses)
    gd_fetch_tile<AEK>(va, g.A, g.lda, nullptr, g.a_kc, row0, g.M, k0 + GD_BK, kend, t);
    gd_fetch_tile<BEK>(vb, g.B, g.ldb, g.b_rows, g.b_kc, col0, g.N, k0 + GD_BK, kend, t);
#pragma unroll
    for (int kk = 0; kk < GD_BK; ++kk) {
      double a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fma(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }

  const bool split = gridDim.z > 1;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t row = row0 + ty * 4 + i;
    if (row >= g.M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int64_t col = col0 + tx * 4 + j;
      if (col >= g.N) continue;
      if (split) g.Cpart[((int64_t)blockIdx.z * g.M + row) * g.N + col] = acc[i][j];
      else store_f64(g.C, row * g.ldc + col, g.out_ek, g.alpha * acc[i][j]);
    }
  }
}

// out = alpha * sum over splits (ascending); optionally a second bf16 copy of the result.
__global__ __launch_bounds__(256) void reduce_partials_f64(const double* part, int splits,
                                                           int64_t M, int64_t N, double alpha,
                                                           void* out, int64_t ldc, int out_ek) {
  const int64_t total = M * N;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (int64_t)gridDim.x * blockDim.x) {
    double s = 0.0;
    for (int z = 0; z < splits; ++z) s += part[(int64_t)z * total + i];
    const int64_t row = i / N, col = i - row * N;
    store_f64(out, row * ldc + col, out_ek, alpha * s);
  }
}

static inline int gemm_f64_effective_splits(int64_t K, int splits) {
  if (splits < 1) splits = 1;
  int64_t kps = ceil_div64(ceil_div64(K, splits), GD_BK) * GD_BK;
  return (int)ceil_div64(K, kps);
}

static int launch_gemm_f64(const char* name, hipStream_t stream, const void* A, int64_t lda,
                           int a_kc, int a_ek, const void* B, int64_t ldb, int b_kc, int b_ek,
                           const int32_t* b_rows, int64_t M, int64_t N, int64_t K, double alpha,
                           void* C, int64_t ldc, int out_ek, int splits, double* Cpart) {
  if (M <= 0 || N <= 0 || K <= 0) return LORACT_OK;
  GemmF64Args g;
  g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.b_rows = b_rows;
  g.C = C; g.ldc = ldc; g.Cpart = Cpart; g.M = M; g.N = N; g.K = K; g.alpha = alpha;
  g.a_kc = a_kc; g.b_kc = b_kc; g.a_ek = a_ek; g.b_ek = b_ek; g.out_ek = out_ek;
  if (splits < 1) splits = 1;
  int64_t kps = ceil_div64(ceil_div64(K, splits), GD_BK) * GD_BK;
  splits = (int)ceil_div64(K, kps);
  g.k_per_split = kps;
  dim3 grid((unsigned)ceil_div64(M, GD_BM), (unsigned)ceil_div64(N, GD_BN), (unsigned)splits);
  if (grid.y > 65535 || grid.z > 65535) return LORACT_ERR_UNSUPPORTED;
  // one instantiation per pair of operand kinds
#define GD_CASE(AE, BE) \
  if (a_ek == AE && b_ek == BE) { LORACT_LAUNCH(name, stream, (gemm_f64_kernel<AE, BE>), grid, dim3(256), 0, g); } else
  GD_CASE(EK_F32, EK_F32) GD_CASE(EK_F32, EK_F64) GD_CASE(EK_F32, EK_BF16)
  GD_CASE(EK_F64, EK_F32) GD_CASE(EK_F64, EK_F64) GD_CASE(EK_F64, EK_BF16)
  GD_CASE(EK_BF16, EK_F32) GD_CASE(EK_BF16, EK_F64) GD_CASE(EK_BF16, EK_BF16)
  return LORACT_ERR_INVALID_ARG;
#undef GD_CASE
  if (splits > 1) {
    const int64_t total = M * N;
    int blocks = (int)(ceil_div64(total, 256) < 2048 ? ceil_div64(total, 256) : 2048);
    LORACT_LAUNCH("reduce_partials_f64", stream, reduce_partials_f64, dim3(blocks), dim3(256), 0,
                  (const double*)Cpart, splits, M, N, alpha, C, ldc, out_ek);
  }
  return LORACT_OK;
}
