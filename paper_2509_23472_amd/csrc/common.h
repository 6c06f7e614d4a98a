// Shared device helpers, launch bookkeeping and per-kernel event profiling.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include <atomic>
#include <map>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/loract.h"

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef double f64x4 __attribute__((ext_vector_type(4)));

// Element kinds used by the runtime-typed kernels (values match loract_dtype where they overlap).
enum { EK_F32 = 0, EK_BF16 = 1, EK_F64 = 2 };

__host__ __device__ inline int ek_size(int ek) { return ek == EK_F64 ? 8 : (ek == EK_F32 ? 4 : 2); }

__device__ inline double load_f64(const void* p, int64_t i, int ek) {
  if (ek == EK_F32) return (double)((const float*)p)[i];
  if (ek == EK_F64) return ((const double*)p)[i];
  return (double)(float)((const bf16_t*)p)[i];
}
__device__ inline void store_f64(void* p, int64_t i, int ek, double v) {
  if (ek == EK_F32) ((float*)p)[i] = (float)v;
  else if (ek == EK_F64) ((double*)p)[i] = v;
  else ((bf16_t*)p)[i] = (bf16_t)(float)v;
}

static inline int64_t ceil_div64(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---------------------------------------------------------------------------------------------
// Error state and profiling (host side).

struct LoractHostState {
  std::string last_hip_error;
};
static thread_local LoractHostState g_host;

static inline int hip_fail(hipError_t e, const char* what) {
  g_host.last_hip_error = std::string(what) + ": " + hipGetErrorString(e);
  return LORACT_ERR_HIP;
}

struct ProfRecord {
  const char* name;
  hipEvent_t start, stop;
};
// The per-kernel profile is one process-wide record; `mu` serialises the host threads that
// launch while it is on (launches from several threads are otherwise independent of each other).
struct ProfState {
  std::atomic<bool> on{false};
  std::mutex mu;
  std::vector<ProfRecord> recs;
  std::vector<hipEvent_t> pool;
  std::map<std::string, std::pair<double, int64_t>> agg;
  std::vector<std::string> order;
};
static ProfState g_prof;

static inline hipEvent_t prof_event() {   // caller holds g_prof.mu
  hipEvent_t e;
  if (!g_prof.pool.empty()) {
    e = g_prof.pool.back();
    g_prof.pool.pop_back();
    return e;
  }
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

struct KernelScope {
  hipStream_t stream;
  hipEvent_t start = nullptr, stop = nullptr;
  const char* name;
  KernelScope(const char* n, hipStream_t s) : stream(s), name(n) {
    if (g_prof.on.load(std::memory_order_acquire)) {
      {
        std::lock_guard<std::mutex> lock(g_prof.mu);
        start = prof_event();
        stop = prof_event();
      }
      if (start) (void)hipEventRecord(start, stream);
    }
  }
  ~KernelScope() {
    if (start && stop) {
      (void)hipEventRecord(stop, stream);
      std::lock_guard<std::mutex> lock(g_prof.mu);
      g_prof.recs.push_back({name, start, stop});
    }
  }
};

// Launch `kernel<<<grid, block, shmem, stream>>>(args...)`, timing it when profiling is on,
// and turn a launch failure into LORACT_ERR_HIP.
#define LORACT_LAUNCH(NAME, STREAM, KERNEL, GRID, BLOCK, SHMEM, ...)                      \
  do {                                                                                    \
    {                                                                                     \
      KernelScope scope_(NAME, STREAM);                                                   \
      hipLaunchKernelGGL(KERNEL, GRID, BLOCK, SHMEM, STREAM, __VA_ARGS__);                \
    }                                                                                     \
    hipError_t e_ = hipGetLastError();                                                    \
    if (e_ != hipSuccess) return hip_fail(e_, NAME);                                      \
  } while (0)

#define LORACT_TRY(EXPR)              \
  do {                                \
    int rc_ = (EXPR);                 \
    if (rc_ != LORACT_OK) return rc_; \
  } while (0)
// ---------------------------------------------------------------------------------------------
// Asynchronous global -> LDS copies (global_load_lds_dwordx4): every lane of a wave fetches 16
// bytes from its own global address and the wave's 64 pieces land contiguously (lane i at
// base + 16 i) in LDS, without passing through registers.  Several slabs can therefore be in
// flight from HBM per workgroup at no register cost; s_waitcnt vmcnt tracks their arrival.
// Because the LDS placement is fixed by the lane number, bank conflicts are avoided by choosing
// WHICH global chunk each lane fetches (an XOR swizzle on the chunk index), not by padding.

__device__ inline void sb_async16(const void* gsrc, void* lds_wave_base) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gsrc,
                                   (__attribute__((address_space(3))) void*)lds_wave_base, 16, 0, 0);
}
// The same copy with the non-temporal cache policy, for operands that are streamed once (the
// activation matrix): their lines are the first to leave L2, which keeps the small operands that
// every workgroup re-reads (sampled rows, Q, U) resident there.
#ifndef SB_STREAM_POLICY
#define SB_STREAM_POLICY 2    // "nt" bit of the gfx940+ cache-policy operand
#endif
__device__ inline void sb_async16_stream(const void* gsrc, void* lds_wave_base) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gsrc,
                                   (__attribute__((address_space(3))) void*)lds_wave_base, 16, 0,
                                   SB_STREAM_POLICY);
}
// The same copy as a device-scope load (sc1): for data another workgroup of the SAME launch wrote
// with device-scope stores; a line this compute die's L2 may still hold from before is refetched.
__device__ inline void sb_async16_device(const void* gsrc, void* lds_wave_base) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gsrc,
                                   (__attribute__((address_space(3))) void*)lds_wave_base, 16, 0, 16);
}
// s_waitcnt with only the vector-memory counter constrained (gfx9 encoding).
#define SB_WAIT_VMCNT(n) \
  __builtin_amdgcn_s_waitcnt(((n) & 15) | ((((n) >> 4) & 3) << 14) | (7 << 4) | (15 << 8))

// Workgroup barrier that orders LDS traffic for the compiler but does not drain the vector-memory
// queue: __syncthreads() would wait for every outstanding asynchronous copy and with it for the
// slabs that are meant to stay in flight.  Callers first wait (SB_WAIT_VMCNT) for the copies they
// are about to read; LDS reads of the slab being recycled have completed by then because their
// results were consumed by matrix instructions earlier in program order.
__device__ inline void sb_barrier_keep_copies() { asm volatile("s_barrier" ::: "memory"); }
// Workgroup barrier that first waits for this wave's LDS traffic but leaves vector-memory
// operations (asynchronous copies, stores) in flight.
__device__ inline void sb_barrier_lds() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

