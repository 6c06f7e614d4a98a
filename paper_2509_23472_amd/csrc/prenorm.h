// Pre-norm unit of Section 3.3: the RMS normalisation whose OUTPUT A = Norm(X) is the activation
// that gets stored (compressed) and shared by Norm and the sub-layer, and the backward step that
// recovers dL/dX from the stored A, the RMS vector and dL/dA (Eqs. 6-10):
//
//   forward   rms_i = sqrt(mean_j X_ij^2 + eps),  A_ij = X_ij / rms_i * gamma_j
//   backward  Xbar = A / gamma,  dXbar = dA * gamma,
//             dX_ij = (dXbar_ij - Xbar_ij * mean_j(dXbar_ij Xbar_ij)) / rms_i
//             (the mean is mean_j(dA_ij A_ij): gamma cancels in the product)
//
// Both are bandwidth-bound row kernels: one wavefront per row, two sweeps over the row (the
// second one is served by the caches), 16-byte accesses for bf16 rows that allow them.
#pragma once
#include "common.h"

struct PrenormArgs {
  const void* X;       // forward: X; backward: A (reconstructed activation)
  int64_t ldx;
  const void* dA;      // backward only
  int64_t ldda;
  const float* gamma;  // n
  float* rms;          // forward: out (m); backward: in
  void* out;           // forward: A; backward: dX
  int64_t ldo;
  int64_t m, n;
  int ek;              // element kind of X / dA / out (EK_F32 or EK_BF16)
  int vec;             // 16-byte accesses legal (bf16 only)
  float eps;
};

__device__ inline float pn_wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  return v;
}
__device__ inline float pn_load(const void* p, int64_t i, int ek) {
  return ek == EK_F32 ? ((const float*)p)[i] : (float)((const bf16_t*)p)[i];
}
__device__ inline void pn_store(void* p, int64_t i, int ek, float v) {
  if (ek == EK_F32) ((float*)p)[i] = v; else ((bf16_t*)p)[i] = (bf16_t)v;
}

__global__ __launch_bounds__(256) void prenorm_forward_kernel(PrenormArgs g) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= g.m) return;
  const int64_t xo = row * g.ldx, oo = row * g.ldo;
  float ss = 0.0f;
  if (g.vec) {
    const bf16_t* x = (const bf16_t*)g.X + xo;
    for (int64_t c = lane * 8; c < g.n; c += 512) {
      const bf16x8 v = *(const bf16x8*)(x + c);
#pragma unroll
      for (int e = 0; e < 8; ++e) { const float f = (float)v[e]; ss += f * f; }
    }
  } else {
    for (int64_t c = lane; c < g.n; c += 64) { const float f = pn_load(g.X, xo + c, g.ek); ss += f * f; }
  }
  ss = pn_wave_sum(ss);
  const float rms = sqrtf(ss / (float)g.n + g.eps);
  if (lane == 0) g.rms[row] = rms;
  const float inv = 1.0f / rms;
  if (g.vec) {
    const bf16_t* x = (const bf16_t*)g.X + xo;
    bf16_t* o = (bf16_t*)g.out + oo;
    for (int64_t c = lane * 8; c < g.n; c += 512) {
      const bf16x8 v = *(const bf16x8*)(x + c);
      const f32x4 g0 = *(const f32x4*)(g.gamma + c), g1 = *(const f32x4*)(g.gamma + c + 4);
      bf16x8 r;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        r[e] = (bf16_t)((float)v[e] * inv * g0[e]);
        r[e + 4] = (bf16_t)((float)v[e + 4] * inv * g1[e]);
      }
      *(bf16x8*)(o + c) = r;
    }
  } else {
    for (int64_t c = lane; c < g.n; c += 64)
      pn_store(g.out, oo + c, g.ek, pn_load(g.X, xo + c, g.ek) * inv * g.gamma[c]);
  }
}

__global__ __launch_bounds__(256) void prenorm_backward_kernel(PrenormArgs g) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= g.m) return;
  const int64_t ao = row * g.ldx, go = row * g.ldda, oo = row * g.ldo;
  float dot = 0.0f;
  if (g.vec) {
    const bf16_t* a = (const bf16_t*)g.X + ao;
    const bf16_t* d = (const bf16_t*)g.dA + go;
    for (int64_t c = lane * 8; c < g.n; c += 512) {
      const bf16x8 va = *(const bf16x8*)(a + c), vd = *(const bf16x8*)(d + c);
#pragma unroll
      for (int e = 0; e < 8; ++e) dot += (float)va[e] * (float)vd[e];
    }
  } else {
    for (int64_t c = lane; c < g.n; c += 64) dot += pn_load(g.X, ao + c, g.ek) * pn_load(g.dA, go + c, g.ek);
  }
  const float inner = pn_wave_sum(dot) / (float)g.n;
  const float inv = 1.0f / g.rms[row];
  if (g.vec) {
    const bf16_t* a = (const bf16_t*)g.X + ao;
    const bf16_t* d = (const bf16_t*)g.dA + go;
    bf16_t* o = (bf16_t*)g.out + oo;
    for (int64_t c = lane * 8; c < g.n; c += 512) {
      const bf16x8 va = *(const bf16x8*)(a + c), vd = *(const bf16x8*)(d + c);
      const f32x4 g0 = *(const f32x4*)(g.gamma + c), g1 = *(const f32x4*)(g.gamma + c + 4);
      bf16x8 r;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        r[e] = (bf16_t)(((float)vd[e] * g0[e] - (float)va[e] / g0[e] * inner) * inv);
        r[e + 4] = (bf16_t)(((float)vd[e + 4] * g1[e] - (float)va[e + 4] / g1[e] * inner) * inv);
      }
      *(bf16x8*)(o + c) = r;
    }
  } else {
    for (int64_t c = lane; c < g.n; c += 64) {
      const float gm = g.gamma[c];
      const float v = (pn_load(g.dA, go + c, g.ek) * gm - pn_load(g.X, ao + c, g.ek) / gm * inner) * inv;
      pn_store(g.out, oo + c, g.ek, v);
    }
  }
}
