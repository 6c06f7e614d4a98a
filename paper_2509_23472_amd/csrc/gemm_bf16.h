// General bf16 x bf16 -> fp32 matrix product on the gfx950 matrix cores.
//
//   C[i][j] = sum_kk opA(i, kk) * opB(j, kk),   0 <= i < M, 0 <= j < N, 0 <= kk < K
//
// Each operand is addressed either "K-contiguous" (element (i, kk) at P[row(i) * ld + kk],
// i.e. a row-major M x K matrix, with an optional row indirection for B) or "K-strided"
// (element (i, kk) at P[kk * ld + i], i.e. the transpose of a row-major K x M matrix).
// This covers the sketch Y = X X_S^T (both K-contiguous, B rows gathered through the sample
// indices), the projection V = U^T X (both K-strided, long reduction over the tokens, split
// across workgroups) and the reconstruction Xhat = U V (A K-contiguous, B K-strided).
//
// Tiling: one 256-thread workgroup (4 wavefronts, 2 x 2) per 64 x 64 tile of C, K consumed in
// slabs of 32 staged through LDS as [row][K] so that every wave feeds
// v_mfma_f32_32x32x16_bf16 with 16-byte LDS reads.  blockIdx.z splits K; partial tiles go to
// an fp32 buffer that reduce_partials_f32 sums in a fixed order.
#pragma once
#include "common.h"

struct GemmBf16Args {
  const bf16_t* A;
  int64_t lda;
  const bf16_t* B;
  int64_t ldb;
  const int32_t* b_rows;  // optional row indirection for a K-contiguous B
  void* C;                // final output (out_kind) when gridDim.z == 1
  int64_t ldc;
  float* Cpart;           // [splits][M][N] partial sums when gridDim.z > 1
  int64_t M, N, K;
  int64_t n_pad;          // columns N..n_pad-1 of C are written as zero (unsplit launches only)
  int64_t k_per_split;    // multiple of 32
  int a_kc, b_kc;         // 1 = K-contiguous, 0 = K-strided
  int a_vec, b_vec;       // 16-byte vector loads are legal for this operand
  int out_kind;           // EK_F32 or EK_BF16
};

#define GB_BM 64
#define GB_BN 64
#define GB_BK 32
#define GB_LDS_STRIDE 40  // bf16 elements per LDS row: 32 + 8 pad, keeps 16-byte alignment

// Loads one 64 x 32 operand tile into LDS laid out [row][k].
__device__ inline void gb_load_tile(bf16_t (*Ls)[GB_LDS_STRIDE], const bf16_t* P, int64_t ld,
                                    const int32_t* rows, int kc, int vec, int64_t row0,
                                    int64_t nrows, int64_t k0, int64_t kend, int t) {
  const bf16_t zero = (bf16_t)0.0f;
  if (kc) {
    const int r = t >> 2, c = (t & 3) * 8;
    const int64_t gr = row0 + r;
    bf16x8 v;
    for (int e = 0; e < 8; ++e) v[e] = zero;
    if (gr < nrows) {
      const int64_t src_row = rows ? (int64_t)rows[gr] : gr;
      const bf16_t* src = P + src_row * ld + k0 + c;
      if (vec && k0 + c + 8 <= kend) {
        v = *(const bf16x8*)src;
      } else {
        for (int e = 0; e < 8; ++e)
          if (k0 + c + e < kend) v[e] = src[e];
      }
    }
    *(bf16x8*)&Ls[r][c] = v;
  } else {
    const int kk = t >> 3, rc = (t & 7) * 8;
    const int64_t gk = k0 + kk;
    bf16x8 v;
    for (int e = 0; e < 8; ++e) v[e] = zero;
    if (gk < kend) {
      const bf16_t* src = P + gk * ld + row0 + rc;
      if (vec && row0 + rc + 8 <= nrows) {
        v = *(const bf16x8*)src;
      } else {
        for (int e = 0; e < 8; ++e)
          if (row0 + rc + e < nrows) v[e] = src[e];
      }
    }
    for (int e = 0; e < 8; ++e) Ls[rc + e][kk] = v[e];
  }
}

__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmBf16Args g) {
  __shared__ __attribute__((aligned(16))) bf16_t As[GB_BM][GB_LDS_STRIDE];
  __shared__ __attribute__((aligned(16))) bf16_t Bs[GB_BN][GB_LDS_STRIDE];

  const int t = threadIdx.x;
  const int lane = t & 63, wave = t >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int64_t row0 = (int64_t)blockIdx.x * GB_BM;
  const int64_t col0 = (int64_t)blockIdx.y * GB_BN;
  const int64_t kbeg = (int64_t)blockIdx.z * g.k_per_split;
  const int64_t kend = (kbeg + g.k_per_split < g.K) ? kbeg + g.k_per_split : g.K;

  f32x16 acc;
  for (int i = 0; i < 16; ++i) acc[i] = 0.0f;

  for (int64_t k0 = kbeg; k0 < kend; k0 += GB_BK) {
    gb_load_tile(As, g.A, g.lda, nullptr, g.a_kc, g.a_vec, row0, g.M, k0, kend, t);
    gb_load_tile(Bs, g.B, g.ldb, g.b_rows, g.b_kc, g.b_vec, col0, g.N, k0, kend, t);
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < GB_BK; ks += 16) {
      const bf16x8 a = *(const bf16x8*)&As[wm * 32 + (lane & 31)][ks + 8 * (lane >> 5)];
      const bf16x8 b = *(const bf16x8*)&Bs[wn * 32 + (lane & 31)][ks + 8 * (lane >> 5)];
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
    }
    __syncthreads();
  }

  // 32x32 accumulator layout: register r of lane l holds
  // row 8*(r/4) + 4*(l/32) + r%4, column l%32 of the wave's sub-tile.
  const int64_t col = col0 + wn * 32 + (lane & 31);
  const bool split = gridDim.z > 1;
  if (col >= g.N) {
    if (!split && col < g.n_pad) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t row = row0 + wm * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (row >= g.M) continue;
        if (g.out_kind == EK_F32) ((float*)g.C)[row * g.ldc + col] = 0.0f;
        else ((bf16_t*)g.C)[row * g.ldc + col] = (bf16_t)0.0f;
      }
    }
    return;
  }
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int64_t row = row0 + wm * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
    if (row >= g.M) continue;
    if (split) {
      g.Cpart[((int64_t)blockIdx.z * g.M + row) * g.N + col] = acc[r];
    } else if (g.out_kind == EK_F32) {
      ((float*)g.C)[row * g.ldc + col] = acc[r];
    } else {
      ((bf16_t*)g.C)[row * g.ldc + col] = (bf16_t)acc[r];
    }
  }
}

// out[row][col] = sum over splits (ascending) of part[s][row][col], converted to out_kind.
__global__ __launch_bounds__(256) void reduce_partials_f32(const float* part, int splits,
                                                           int64_t M, int64_t N, void* out,
                                                           int64_t ldc, int out_kind) {
  const int64_t total = M * N;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (int64_t)gridDim.x * blockDim.x) {
    float s = 0.0f;
    for (int z = 0; z < splits; ++z) s += part[(int64_t)z * total + i];
    const int64_t row = i / N, col = i - row * N;
    if (out_kind == EK_F32) ((float*)out)[row * ldc + col] = s;
    else ((bf16_t*)out)[row * ldc + col] = (bf16_t)s;
  }
}

static inline bool gb_vec_ok(const void* p, int64_t ld) {
  return (((uintptr_t)p) % 16 == 0) && (ld % 8 == 0);
}

// Enqueue C = opA * opB^T.  `splits` > 1 requires Cpart with splits*M*N floats.
static int launch_gemm_bf16(const char* name, hipStream_t stream, const bf16_t* A, int64_t lda,
                            int a_kc, const bf16_t* B, int64_t ldb, int b_kc,
                            const int32_t* b_rows, int64_t M, int64_t N, int64_t K, void* C,
                            int64_t ldc, int out_kind, int splits, float* Cpart,
                            int64_t n_pad = 0) {
  if (M <= 0 || N <= 0 || K <= 0) return LORACT_OK;
  GemmBf16Args g;
  g.n_pad = n_pad;
  g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.b_rows = b_rows;
  g.C = C; g.ldc = ldc; g.Cpart = Cpart; g.M = M; g.N = N; g.K = K;
  g.a_kc = a_kc; g.b_kc = b_kc;
  g.a_vec = gb_vec_ok(A, lda); g.b_vec = gb_vec_ok(B, ldb);
  g.out_kind = out_kind;
  if (splits < 1) splits = 1;
  int64_t kps = ceil_div64(ceil_div64(K, splits), GB_BK) * GB_BK;
  splits = (int)ceil_div64(K, kps);
  g.k_per_split = kps;
  dim3 grid((unsigned)ceil_div64(M, GB_BM), (unsigned)ceil_div64(std::max(N, n_pad), GB_BN),
            (unsigned)splits);
  if (grid.y > 65535 || grid.z > 65535) return LORACT_ERR_UNSUPPORTED;
  LORACT_LAUNCH(name, stream, gemm_bf16_kernel, grid, dim3(256), 0, g);
  if (splits > 1) {
    const int64_t total = M * N;
    int blocks = (int)(ceil_div64(total, 256) < 2048 ? ceil_div64(total, 256) : 2048);
    LORACT_LAUNCH("reduce_partials_f32", stream, reduce_partials_f32, dim3(blocks), dim3(256), 0,
                  (const float*)Cpart, splits, M, N, C, ldc, out_kind);
  }
  return LORACT_OK;
}

// Number of K splits the launcher will actually use for a requested count.
static inline int gemm_bf16_effective_splits(int64_t K, int splits) {
  if (splits < 1) splits = 1;
  int64_t kps = ceil_div64(ceil_div64(K, splits), GB_BK) * GB_BK;
  return (int)ceil_div64(K, kps);
}
