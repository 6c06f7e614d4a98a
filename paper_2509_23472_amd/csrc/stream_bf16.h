// Streaming bf16 kernels of the hot path: the passes over the activation X (tokens x hidden)
// and the write of its reconstruction, on v_mfma_f32_32x32x16_bf16 with fp32 accumulation.
//
//   sketch       Y = X Bt^T          Algorithm 1: the sketch (Bt = sampled rows of X) and the power rounds
//   project      V = Q^T X           Algorithm 1: the projection onto the basis (and the power rounds)
//   reconstruct  Xhat = U V          Section 3.1 Eq. (4)
//
// All three fill LDS with asynchronous global -> LDS copies, several slabs or tiles ahead, and
// give each wave a strip of 32 x 32 accumulator tiles.  Operands whose contraction index is
// contiguous in memory (both operands of the sketch, the rows of U in the reconstruction) lie in
// LDS as [row][K] and are read back as 16-byte matrix-core fragments.  In the projection the
// contraction index is the ROW index of both row-major operands: the slabs are copied as they
// lie in memory and the fragments (8 consecutive rows of one column) come from the transposing
// LDS read ds_read_b64_tr_b16.  Only the V operand of the reconstruction, which is staged once per
// column block and then kept in registers, is stored "pair interleaved" (LDS word [p][c] holds
// rows 2p and 2p+1 of column c) and read with four 4-byte LDS reads per fragment.
//
// Fast-path requirements (checked by the host, which otherwise falls back to gemm_bf16.h):
// 16-byte aligned base pointers and leading dimensions that are multiples of 8 elements.
#pragma once
#include "common.h"

#define SB_BK 64     // contraction slab of the sketch and the projection

// Split reductions (over K in the sketch, over the rows in the projection) leave fp32 partial
// tiles in a scratch buffer; this kernel sums them in ascending split order, so the result does
// not depend on scheduling, and converts to the output type.  `ld*` in elements; the row length
// `cols` is a multiple of 4.  Output kinds: fp32, bf16, or EK_BF16_SPLIT: every value v is written
// as the bf16 pair hi = bf16(v), lo = bf16(v - hi) at columns c and cols + c of a row of 2 * cols
// bf16 values, so that a bf16 matrix product with the pair recovers ~16 mantissa bits of v.
#define EK_BF16_SPLIT 3
__global__ __launch_bounds__(256) void sum_partials_kernel(const float* part, int splits,
                                                           int64_t rows, int64_t cols,
                                                           int64_t ld_part, void* out,
                                                           int64_t ld_out, int out_ek) {
  const int64_t c4 = cols >> 2;
  const int64_t total = rows * c4;
  const int64_t split_stride = rows * ld_part;
  for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256) {
    const int64_t r = e / c4, c = (e - r * c4) << 2;
    const float* src = part + r * ld_part + c;
    // loads are issued in batches so that their latencies overlap; the additions keep the
    // ascending order of the splits
    f32x4 s4 = *(const f32x4*)src;
    int z = 1;
    for (; z + 8 <= splits; z += 8) {
      f32x4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = *(const f32x4*)(src + (int64_t)(z + u) * split_stride);
#pragma unroll
      for (int u = 0; u < 8; ++u) s4 += v[u];
    }
    if (z + 4 <= splits) {
      f32x4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = *(const f32x4*)(src + (int64_t)(z + u) * split_stride);
#pragma unroll
      for (int u = 0; u < 4; ++u) s4 += v[u];
      z += 4;
    }
    if (z + 2 <= splits) {
      const f32x4 v0 = *(const f32x4*)(src + (int64_t)z * split_stride);
      const f32x4 v1 = *(const f32x4*)(src + (int64_t)(z + 1) * split_stride);
      s4 += v0;
      s4 += v1;
      z += 2;
    }
    if (z < splits) s4 += *(const f32x4*)(src + (int64_t)z * split_stride);
    if (out_ek == EK_F32) {
      *(f32x4*)((float*)out + r * ld_out + c) = s4;
    } else if (out_ek == EK_BF16) {
      bf16x4 o;
#pragma unroll
      for (int u = 0; u < 4; ++u) o[u] = (bf16_t)s4[u];
      *(bf16x4*)((bf16_t*)out + r * ld_out + c) = o;
    } else {
      bf16x4 hi, lo;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        hi[u] = (bf16_t)s4[u];
        lo[u] = (bf16_t)(s4[u] - (float)hi[u]);
      }
      *(bf16x4*)((bf16_t*)out + r * ld_out + c) = hi;
      *(bf16x4*)((bf16_t*)out + r * ld_out + cols + c) = lo;
    }
  }
}

static int launch_sum_partials(hipStream_t s, const float* part, int splits, int64_t rows,
                               int64_t cols, int64_t ld_part, void* out, int64_t ld_out,
                               int out_ek) {
  const int64_t total = rows * (cols >> 2);
  const int blocks = (int)std::max<int64_t>(1, std::min<int64_t>(ceil_div64(total, 256), 2048));
  LORACT_LAUNCH("sum_partials", s, sum_partials_kernel, dim3(blocks), dim3(256), 0, part, splits,
                rows, cols, ld_part, out, ld_out, out_ek);
  return LORACT_OK;
}

// ---------------------------------------------------------------------------------------------
// sketch: Y (m x kp, fp32) = X (m x n) * Bt^T, Bt = l rows of length n (optionally gathered).
//
// LDS slab layout, both operands: [row][64 K] as 8 chunks of 16 bytes per 128-byte row, chunk c of
// row r stored at position c ^ (r & 7), so that the 16-byte fragment reads of 8 consecutive rows
// hit 8 different bank groups.  Requires n % 64 == 0 (no partial slab) on this path.

// Row ids passed by value inside kernel arguments (no host-to-device copy needed).
struct IdxPack {
  int32_t v[LORACT_MAX_RANK];
};

struct SketchArgs {
  const bf16_t* X;
  int64_t ldx;
  int64_t m, n;
  const bf16_t* B;
  int64_t ldb;
  const int32_t* b_rows;
  int l;                 // valid rows of Bt
  int kp;                // columns of Y (l rounded up to 16), columns >= l come out zero
  float* Y;
  float* part;           // [splits][m][kp], used when splits > 1
  int splits;
  int64_t k_per_split;   // multiple of SB_BK
  const int32_t* run_flag;   // optional: the launch does nothing unless *run_flag == 1
  int stream_x;              // set by the launcher: X is too large to stay cached, copy it non-temporally
  int ids_in_args;           // the gather ids are `ids` below (read from the kernel-argument segment), not b_rows
  int32_t* clear_status;     // optional: word that the first workgroup sets to zero
  // Optional fused finish (splits == 1 only).  With fin_q set the product is not stored: the
  // launch writes fin_q (and its bf16 copy fin_qb, if given) = fin_q1 + X Bt^T, both with row
  // pitch fin_ld and l valid columns, and run_flag selects 0: nothing, 1: as said, 2: no product,
  // fin_q1 alone is converted.
  const float* fin_q1;       // m x kp float32
  void* fin_q;
  bf16_t* fin_qb;
  int fin_ek;                // EK_F32 or EK_BF16
  int64_t fin_ld;
  IdxPack ids;
};

// WM = 64-row wave groups per workgroup: 2 (4 waves, 128 rows) or 4 (8 waves, 256 rows; halves the
// re-reads of Bt per row of X, for matrices tall enough to fill the CUs with 256-row tiles).
// ROLE only names the use in the kernel's symbol, so that a profile tells the uses apart:
// 0 the sketch of Algorithm 1, 1 the product dY B_lora^T of the LoRA gradient, 2 the finish of
// the orthonormalisation.  The code is the same.
enum { SK_SKETCH = 0, SK_LORA_DYB = 1, SK_NS_CORRECT = 2 };
// RT = 32-row tiles per wave: 2 (a wave owns 64 rows), or 1 (32 rows: twice the waves on the same
// tile -- half the accumulators per wave and the copies of a slab issued by twice as many waves;
// used for the 128-row tiles of up to 128 columns: sketch 23.1 -> 21.7 us and the Newton-Schulz
// finish 11.9 -> 9.2 us at 8192 x 4096 with 128 columns, dY B^T 16.5 -> 15.3 us; and for the
// finish on 256-row tiles, 42.6 -> 38.3 us at 65536 x 256, where the sketch itself is no faster
// on sixteen waves than on eight).
template <int NT, int STAGES, int WM, int ROLE, int RT = 2>
__global__ __launch_bounds__(256 * WM / RT) void sketch_mfma_kernel(SketchArgs g) {
  constexpr int BM = 64 * WM, BN = 64 * NT;
  constexpr int NWV = 4 * WM / RT;      // waves: BM / (32 RT) row groups x 2 column halves
  constexpr int NA = 8 * WM / NWV;      // X copy instructions per wave per slab (8 rows each)
  constexpr int NB = 8 * NT / NWV;      // Bt copy instructions per wave per slab
  constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128, STAGE_BYTES = A_BYTES + B_BYTES;
  constexpr int LOADS = NA + NB;        // wave-level copy instructions per slab per wave
  extern __shared__ __attribute__((aligned(16))) unsigned char sb_smem[];
  const int run_mode = g.run_flag ? *g.run_flag : 1;
  if (g.fin_q ? run_mode == 0 : run_mode != 1) return;
  if (g.fin_q && run_mode == 2) {
    // no product: the whole grid converts fin_q1, four columns per thread and step
    const int64_t nthreads = (int64_t)gridDim.x * gridDim.y * gridDim.z * (64 * NWV);
    const int64_t tid = (((int64_t)blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) * (64 * NWV) + threadIdx.x;
    const int c4 = g.kp >> 2;
    const bool vec_ok = (g.fin_ld & 3) == 0 && ((uintptr_t)g.fin_q & 15) == 0 && ((uintptr_t)g.fin_qb & 7) == 0;
    const int64_t total = g.m * c4;
    // four independent loads in flight per thread: the grid is sized for the product, not for a copy
    for (int64_t e0 = tid; e0 < total; e0 += 4 * nthreads) {
      f32x4 q[4];
      int64_t rr[4];
      int cc[4];
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int64_t e = e0 + v * nthreads;
        const int64_t ec = e < total ? e : tid;
        rr[v] = total < (1ll << 31) ? (int64_t)((unsigned)ec / (unsigned)c4) : ec / c4;
        cc[v] = (int)(ec - rr[v] * c4) << 2;
        q[v] = *(const f32x4*)(g.fin_q1 + rr[v] * g.kp + cc[v]);
      }
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        if (e0 + v * nthreads >= total) continue;
        const int64_t r = rr[v];
        const int c = cc[v];
        if (vec_ok && c + 4 <= g.l) {
          bf16x4 qh;
#pragma unroll
          for (int u = 0; u < 4; ++u) qh[u] = (bf16_t)q[v][u];
          if (g.fin_ek == EK_F32) *(f32x4*)((float*)g.fin_q + r * g.fin_ld + c) = q[v];
          else *(bf16x4*)((bf16_t*)g.fin_q + r * g.fin_ld + c) = qh;
          if (g.fin_qb) *(bf16x4*)(g.fin_qb + r * g.fin_ld + c) = qh;
          continue;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (c + u < g.l) {
            if (g.fin_ek == EK_F32) ((float*)g.fin_q)[r * g.fin_ld + c + u] = q[v][u];
            else ((bf16_t*)g.fin_q)[r * g.fin_ld + c + u] = (bf16_t)q[v][u];
            if (g.fin_qb) g.fin_qb[r * g.fin_ld + c + u] = (bf16_t)q[v][u];
          }
        }
      }
    }
    return;
  }
  if (g.clear_status && threadIdx.x == 0 && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0)
    *g.clear_status = 0;
  // ids carried in the arguments are read through the kernel-argument segment, which is ordinary
  // read-only memory and so can be indexed per lane (g is the kernel's only argument, offset 0)
  const int32_t* const gather =
      g.ids_in_args ? (const int32_t*)((const char*)__builtin_amdgcn_kernarg_segment_ptr() + offsetof(SketchArgs, ids))
                    : g.b_rows;

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int64_t row0 = (int64_t)blockIdx.y * BM;
  const int col0 = blockIdx.z * BN;
  // Split z owns a contiguous K range.  Each workgroup walks its slabs starting from a different
  // offset (rotated by its row-tile index): with a power-of-two row pitch, workgroups that all read
  // the same K offset at the same time would crowd a few memory channels.
  const int zsplit = blockIdx.x;
  const int64_t kbeg = (int64_t)zsplit * g.k_per_split;
  const int64_t kend = (kbeg + g.k_per_split < g.n) ? kbeg + g.k_per_split : g.n;
  const int nslab = (int)((kend - kbeg) / SB_BK);
  const int rot = nslab > 0 ? (int)(blockIdx.y % nslab) : 0;

  // global sources of this lane's chunks (rows past the end are clamped: they only feed
  // accumulator rows / columns that are never stored)
  const int sub = lane >> 3;                       // row within the 8-row group = row & 7
  const int kc = (lane & 7) ^ sub;                 // swizzled K chunk fetched by this lane
  const bf16_t* a_src[NA];
#pragma unroll
  for (int i = 0; i < NA; ++i) {
    int64_t r = row0 + (wave * NA + i) * 8 + sub;
    if (r >= g.m) r = g.m - 1;
    a_src[i] = g.X + r * g.ldx + kbeg + kc * 8;
  }
  const bf16_t* b_src[NB];
#pragma unroll
  for (int i = 0; i < NB; ++i) {
    const int j = col0 + (wave * NB + i) * 8 + sub;
    int64_t r = 0;
    if (j < g.l) r = gather ? (int64_t)gather[j] : (int64_t)j;
    else r = gather ? (int64_t)gather[0] : 0;
    b_src[i] = g.B + r * g.ldb + kbeg + kc * 8;
  }
  auto issue = [&](int slab) {
    unsigned char* st = sb_smem + (slab % STAGES) * STAGE_BYTES;
    int pos = slab + rot;
    if (pos >= nslab) pos -= nslab;
    const int64_t koff = (int64_t)pos * SB_BK;
#pragma unroll
    for (int i = 0; i < NA; ++i) {
      if (g.stream_x) sb_async16_stream(a_src[i] + koff, st + (wave * NA + i) * 1024);
      else sb_async16(a_src[i] + koff, st + (wave * NA + i) * 1024);
    }
#pragma unroll
    for (int i = 0; i < NB; ++i)
      sb_async16(b_src[i] + koff, st + A_BYTES + (wave * NB + i) * 1024);
  };

  f32x16 acc[RT][NT];
#pragma unroll
  for (int i = 0; i < RT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  // fragment addresses inside a stage
  int a_off[RT], b_off[NT];
#pragma unroll
  for (int i = 0; i < RT; ++i) a_off[i] = (wm * 32 * RT + 32 * i + (lane & 31)) * 128;
#pragma unroll
  for (int j = 0; j < NT; ++j) b_off[j] = A_BYTES + (wn * 32 * NT + 32 * j + (lane & 31)) * 128;
  const int rsw = lane & 7;                        // (row & 7) of every fragment row of this lane
  const int khalf = lane >> 5;

#pragma unroll
  for (int p = 0; p < STAGES - 1; ++p)
    if (p < nslab) issue(p);
  for (int s = 0; s < nslab; ++s) {
    // slab s has landed once at most the copies of the (STAGES - 2) younger slabs are pending
    if (s + STAGES - 1 <= nslab) SB_WAIT_VMCNT((STAGES - 2) * LOADS);
    else SB_WAIT_VMCNT(0);
    sb_barrier_keep_copies();                      // everyone's copies landed; slab s-1 is consumed
    if (s + STAGES - 1 < nslab) issue(s + STAGES - 1);
    const unsigned char* st = sb_smem + (s % STAGES) * STAGE_BYTES;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int pos = ((2 * ks + khalf) ^ rsw) << 4;
      bf16x8 a[RT], b[NT];
#pragma unroll
      for (int i = 0; i < RT; ++i) a[i] = *(const bf16x8*)(st + a_off[i] + pos);
#pragma unroll
      for (int j = 0; j < NT; ++j) b[j] = *(const bf16x8*)(st + b_off[j] + pos);
#pragma unroll
      for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
  }

  // epilogue: accumulator register r of lane l is row 8*(r/4) + 4*(l/32) + r%4, column l%32
  if (g.fin_q) {
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const int col = col0 + wn * 32 * NT + 32 * j + (lane & 31);
        if (col >= g.l) continue;
        float q1[16];
        int64_t rows[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int64_t row = row0 + wm * 32 * RT + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          rows[r] = row;
          q1[r] = g.fin_q1[(row < g.m ? row : g.m - 1) * g.kp + col];
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          if (rows[r] >= g.m) continue;
          const float q = q1[r] + acc[i][j][r];
          if (g.fin_ek == EK_F32) ((float*)g.fin_q)[rows[r] * g.fin_ld + col] = q;
          else ((bf16_t*)g.fin_q)[rows[r] * g.fin_ld + col] = (bf16_t)q;
          if (g.fin_qb) g.fin_qb[rows[r] * g.fin_ld + col] = (bf16_t)q;
        }
      }
    return;
  }
  float* dst = g.splits > 1 ? g.part + (int64_t)zsplit * g.m * g.kp : g.Y;
#pragma unroll
  for (int i = 0; i < RT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const int col = col0 + wn * 32 * NT + 32 * j + (lane & 31);
      if (col >= g.kp) continue;
      const bool live = col < g.l;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t row = row0 + wm * 32 * RT + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (row < g.m) dst[row * g.kp + col] = live ? acc[i][j][r] : 0.0f;
      }
    }
}

// Wide sketches of matrices with 8192 rows or more: 256-row tiles (8 waves: two per SIMD, one
// covering the other's LDS reads), with K splits while the row tiles alone do not fill the CUs.
// (measured at 8192 x 11008, 256 columns: 75 -> 64 us for the product, +5 us for the sum of the
// twice as many split partials)
static inline int sketch_wm_for(int64_t m, int nt) { return (nt == 4 && m >= 8192) ? 4 : 2; }
static inline int sketch_stages_for(int nt, int wm) { return wm == 4 ? 2 : (nt == 4 ? 3 : 4); }
static size_t sketch_lds_bytes(int nt, int wm) {
  return (size_t)sketch_stages_for(nt, wm) * (64 * wm + 64 * nt) * 128;
}

static inline int sketch_nt_for(int kp) { return kp <= 64 ? 1 : (kp <= 128 ? 2 : 4); }

// Number of K splits: fill ~256-512 workgroups, at least 512 columns per split.
static inline int sketch_splits_for(int64_t m, int64_t n, int kp) {
  const int nt = sketch_nt_for(kp);
  const int wm = sketch_wm_for(m, nt);
  const int64_t tiles = ceil_div64(m, 64 * wm) * ceil_div64(kp, 64 * nt);
  // one workgroup per CU (the multi-stage LDS pipeline fills a CU's LDS), at least 512 columns each
  int64_t s = std::max<int64_t>(1, 256 / std::max<int64_t>(1, tiles));
  s = std::min<int64_t>(s, std::max<int64_t>(1, n / 512));
  return (int)std::min<int64_t>(s, 16);
}

// A matrix of this many bytes does not survive in the 256 MB memory-side cache between two
// passes, so caching its lines only evicts the small operands that are re-read.
static inline int sb_streams_past_cache(int64_t bytes, int limit_mb = 192) { return bytes >= ((int64_t)limit_mb << 20); }

static inline bool sb_aligned(const void* p, int64_t ld) {
  return (((uintptr_t)p) % 16 == 0) && (ld % 8 == 0);
}

// Which share of the work a workgroup takes.  The projection and the reconstruction cut a list of
// (output tile, step) items, tile major, into equal contiguous shares, one per workgroup; at step i
// a share that begins at item b reads block (b + i) mod period of the operand every tile re-reads
// (the basis Q, the factor U).  Workgroups are handed to the eight XCDs in turn (workgroup B runs
// on XCD B mod 8) and each XCD has an L2 of its own, so the shares are sorted by b mod period and
// dealt out in eight consecutive runs: the workgroups of one XCD then walk through the same blocks
// of that operand at about the same time and fetch each of them into their L2 once, instead of once
// per workgroup.  share_of[B] = share of workgroup B; any permutation is correct, this one is fast.
#define SB_MAX_WGS 512
// Tuning knob for measurements: LORACT_XCD_ORDER=0 in the environment deals the shares out in
// their natural order instead.
static bool sb_xcd_order_enabled() {
  static const bool on = [] { const char* e = getenv("LORACT_XCD_ORDER"); return !(e && e[0] == '0'); }();
  return on;
}
static void sb_xcd_share_order(int64_t items, int wgs, int64_t period, unsigned short* share_of) {
  int order[SB_MAX_WGS];
  int64_t key[SB_MAX_WGS];
  for (int w = 0; w < wgs; ++w) {
    order[w] = w;
    key[w] = (items * w / wgs) % period;
  }
  if (sb_xcd_order_enabled())
    std::stable_sort(order, order + wgs, [&](int a, int b) { return key[a] < key[b]; });
  const int base = wgs / 8, extra = wgs % 8;
  for (int b = 0; b < wgs; ++b) {
    const int x = b % 8, j = b / 8;
    share_of[b] = (unsigned short)order[x * base + std::min(x, extra) + j];
  }
}

template <int NT, int WM, int ROLE, int RT = 2>
static int launch_sketch_nt(hipStream_t s, const SketchArgs& g, dim3 grid, const char* name) {
  constexpr int STAGES = WM == 4 ? 2 : (NT == 4 ? 3 : 4);
  static std::atomic<bool> attr_done{false};
  const size_t lds = sketch_lds_bytes(NT, WM);
  if (lds > 64 * 1024 && !attr_done.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute((const void*)sketch_mfma_kernel<NT, STAGES, WM, ROLE, RT>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return hip_fail(e, "hipFuncSetAttribute(sketch LDS)");
    attr_done.store(true, std::memory_order_release);
  }
  LORACT_LAUNCH(name, s, (sketch_mfma_kernel<NT, STAGES, WM, ROLE, RT>), grid, dim3(256 * WM / RT), lds, g);
  return LORACT_OK;
}

// part must hold splits * m * kp floats when splits > 1.  If `split_out` is given the result is
// (also for a single split) passed through the partial buffer and written there as the bf16 pair
// [hi | lo] (m x 2 kp) instead of fp32 Y.
static int launch_sketch_mfma(hipStream_t s, SketchArgs g, const char* name = "sketch",
                              bf16_t* split_out = nullptr) {
  int nt = sketch_nt_for(g.kp);
  // the fused finish contracts over kp only: with so little work per tile, narrower column tiles
  // (more workgroups) win as long as the wide ones leave CUs idle
  if (g.fin_q)
    while (nt > 1 && ceil_div64(g.m, 128) * ceil_div64(g.kp, 64 * nt) < 256) nt >>= 1;
  g.stream_x = sb_streams_past_cache(g.m * g.n * 2);
  int64_t kps = ceil_div64(ceil_div64(g.n, g.splits), SB_BK) * SB_BK;
  g.splits = (int)ceil_div64(g.n, kps);
  g.k_per_split = kps;
  const int wm = sketch_wm_for(g.m, nt);
  dim3 grid((unsigned)g.splits, (unsigned)ceil_div64(g.m, 64 * wm), (unsigned)ceil_div64(g.kp, 64 * nt));
  if (grid.y > 65535) return LORACT_ERR_UNSUPPORTED;
  if (split_out && g.splits == 1) g.Y = g.part;     // single split: Y itself is the "partial"
  int rc;
  const int role = g.fin_q ? SK_NS_CORRECT : (split_out ? SK_LORA_DYB : SK_SKETCH);
#define SK_LAUNCH(ROLE)                                                                                   \
  switch (nt) {                                                                                           \
    case 1: rc = launch_sketch_nt<1, 2, ROLE, 1>(s, g, grid, name); break;                                \
    case 2: rc = launch_sketch_nt<2, 2, ROLE, 1>(s, g, grid, name); break;                                \
    default: rc = wm == 4 ? launch_sketch_nt<4, 4, ROLE, (ROLE == SK_NS_CORRECT ? 1 : 2)>(s, g, grid, name) \
                          : launch_sketch_nt<4, 2, ROLE>(s, g, grid, name); break;                        \
  }
  if (role == SK_NS_CORRECT) { SK_LAUNCH(SK_NS_CORRECT) }
  else if (role == SK_LORA_DYB && nt == 1) rc = launch_sketch_nt<1, 2, SK_LORA_DYB, 1>(s, g, grid, name);
  else { SK_LAUNCH(SK_SKETCH) }
#undef SK_LAUNCH
  if (rc != LORACT_OK) return rc;
  if (split_out)
    return launch_sum_partials(s, g.part, g.splits, g.m, g.kp, g.kp, split_out, 2 * g.kp, EK_BF16_SPLIT);
  if (g.splits == 1) return rc;
  return launch_sum_partials(s, g.part, g.splits, g.m, g.kp, g.kp, g.Y, g.kp, EK_F32);
}

// ---------------------------------------------------------------------------------------------
// Pair-interleaved staging of a row-major slab whose rows are the contraction index.

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Rows 2p (lo) and 2p+1 (hi), 8 consecutive columns each -> 8 words (col c: lo[c] | hi[c] << 16).
__device__ inline void sb_interleave(const bf16x8 lo, const bf16x8 hi, u32x4* w0, u32x4* w1) {
  const u32x4 l = __builtin_bit_cast(u32x4, lo), h = __builtin_bit_cast(u32x4, hi);
  u32x4 a, b;
  a[0] = (l[0] & 0xffffu) | (h[0] << 16);  a[1] = (l[0] >> 16) | (h[0] & 0xffff0000u);
  a[2] = (l[1] & 0xffffu) | (h[1] << 16);  a[3] = (l[1] >> 16) | (h[1] & 0xffff0000u);
  b[0] = (l[2] & 0xffffu) | (h[2] << 16);  b[1] = (l[2] >> 16) | (h[2] & 0xffff0000u);
  b[2] = (l[3] & 0xffffu) | (h[3] << 16);  b[3] = (l[3] >> 16) | (h[3] & 0xffff0000u);
  *w0 = a;
  *w1 = b;
}

// MFMA fragment (8 consecutive-K values of one column) from a pair-interleaved tile:
// words [p0 .. p0+3][col], row stride ldw words.
__device__ inline bf16x8 sb_pair_frag(const unsigned int* tile, int ldw, int p0, int col) {
  u32x4 w;
  w[0] = tile[(p0 + 0) * ldw + col];
  w[1] = tile[(p0 + 1) * ldw + col];
  w[2] = tile[(p0 + 2) * ldw + col];
  w[3] = tile[(p0 + 3) * ldw + col];
  return __builtin_bit_cast(bf16x8, w);
}

// ---------------------------------------------------------------------------------------------
// project: V (l x n) = Q^T X with Q (m x l, bf16, ld = ldq) and X (m x n, bf16): a long reduction
// over the rows in which BOTH operands are stored with the reduction index as the slow one.
//
// Slabs of 64 rows of X (BNX columns) and of Q (BMQ columns) are brought into LDS exactly as they
// lie in memory, row major, by asynchronous global -> LDS copies, several slabs ahead.  The
// matrix-core fragments (8 consecutive reduction indices of one column) are produced by the
// transposing LDS read ds_read_b64_tr_b16: within a group of 16 lanes, lane s supplies the
// address of 4 consecutive columns of row s / 4, and lane j receives the 4 rows of column j.
// Chunk c (16 bytes) of slab row r is stored at chunk position c ^ 2 (r & 3), so that the four
// rows a 16-lane group reads fall into different banks.
//
// Work items are (output tile of BMQ x BNX, slab), tile major; every workgroup takes an equal
// contiguous share (share_of says which), writes one fp32 partial tile per output tile it touched,
// and project_sum_kernel adds the partial tiles of each output tile in the order of the shares.


struct ProjectArgs {
  const bf16_t* Q;
  int64_t ldq;
  const bf16_t* X;
  int64_t ldx;
  int64_t m, n;
  int l;                   // columns of Q = rows of V
  void* V;                 // l x n, ld = n
  int out_ek;              // EK_BF16 or EK_F32
  float* part;             // project_part_floats(m, n, l) floats
  // filled in by the launcher
  int slabs;               // ceil(m / 64)
  int col_blocks;          // ceil(n / bnx)
  int64_t items;           // output tiles * slabs
  int wgs;                 // workgroups sharing the items
  int segs_max;            // partial tiles reserved per workgroup
  int bmq, bnx;            // rows and columns of an output tile
  int stream_x;            // X is too large to stay cached: copy it non-temporally
  unsigned short share_of[SB_MAX_WGS];   // share of the items that workgroup B takes (wgs entries)
};

#define PJ_MAX_PARTS 72   // partial tiles per output tile: the launcher keeps it at 64 + 2 boundary shares
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

__device__ inline s16x4 sb_read_tr(const unsigned char* lds_ptr) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)lds_ptr);
}

// Output tile (32 NTQ WQ) x (32 NTX WN), waves WQ x WN, each with NTQ x NTX matrix-core tiles.
// WN = 4 (8 waves, 256 columns of X for NTX = 2) halves the re-reads of Q per byte of X.
// WQ = 4 (8 waves on the same tile as WQ = 2 with twice the NTQ): half the accumulators per wave,
// so two waves fit on a SIMD, and the copies of a slab are issued by eight waves side by side (a
// wave gets a 1 KB copy out only every ~150 clocks): 95 -> 81 us at 8192 x 11008 with 256 columns
// of Q, 24 -> 21.7 us at 8192 x 4096 with 128.
// ROLE only names the use in the kernel's symbol: 0 the projection V = Q^T X, 1 the product
// U^T [G_hi | G_lo] of the LoRA gradient.
enum { PJ_PROJECT = 0, PJ_LORA_UTG = 1 };
template <int NTQ, int NTX, int STAGES, int WN, int ROLE, int WQ = 2>
__global__ __launch_bounds__(64 * WQ * WN) void project_mfma_kernel(ProjectArgs g) {
  constexpr int NW = WQ * WN;                      // waves: WQ along the columns of Q x WN along those of X
  constexpr int BMQ = 32 * NTQ * WQ, BNX = 32 * NTX * WN;
  constexpr int CQ = BMQ / 8, CX = BNX / 8;        // 16-byte chunks per slab row
  constexpr int QPITCH = BMQ * 2, XPITCH = BNX * 2;
  constexpr int X_BYTES = SB_BK * XPITCH, Q_BYTES = SB_BK * QPITCH;
  constexpr int STAGE_BYTES = X_BYTES + Q_BYTES;
  constexpr int XI = CX / NW, QI = CQ / NW;        // copy instructions per wave per slab
  constexpr int LOADS = XI + QI;
  extern __shared__ __attribute__((aligned(16))) unsigned char sb_smem[];

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave / WN, wn = wave % WN;

  // fragment addresses inside a stage (for K step 0, first half): lane s of a 16-lane group points
  // at row s / 4, columns 4 (s % 4) .. + 3 of the group's 16 columns; lanes 32..63 take rows + 8
  const int s16 = lane & 15, cg = (lane >> 4) & 1, kg = lane >> 5;
  const int frow = 8 * kg + (s16 >> 2);
  int x_off[NTX], q_off[NTQ];
#pragma unroll
  for (int j = 0; j < NTX; ++j) {
    const int col = wn * 32 * NTX + 32 * j + 16 * cg + 4 * (s16 & 3);
    x_off[j] = frow * XPITCH + (((col >> 3) ^ (2 * (s16 >> 2))) << 4) + (col & 7) * 2;
  }
#pragma unroll
  for (int i = 0; i < NTQ; ++i) {
    const int col = wm * 32 * NTQ + 32 * i + 16 * cg + 4 * (s16 & 3);
    q_off[i] = X_BYTES + frow * QPITCH + (((col >> 3) ^ (2 * (s16 >> 2))) << 4) + (col & 7) * 2;
  }

  const int share = g.share_of[blockIdx.x];
  const int64_t item_begin = g.items * share / gridDim.x;
  const int64_t item_end = g.items * (share + 1) / gridDim.x;
  int64_t item = item_begin;
  int seg = 0;
  while (item < item_end) {
    // ---- segment: consecutive slabs of one output tile
    const int64_t tile = item / g.slabs;
    const int s_beg = (int)(item - tile * g.slabs);
    const int64_t s_stop = s_beg + (item_end - item);
    const int s_end = (int)(s_stop < g.slabs ? s_stop : g.slabs);     // exclusive
    const int nslab = s_end - s_beg;
    item += nslab;
    const int qb = (int)(tile / g.col_blocks), cb = (int)(tile - (int64_t)qb * g.col_blocks);
    const int64_t col0 = (int64_t)cb * BNX;
    const int q0 = qb * BMQ;

    // copies of slab sl of the segment; rows past m repeat the last row and are zeroed when the
    // fragments are read.  Addresses are rebuilt per copy from a few values to keep registers free.
    const bf16_t* const x_col = g.X + col0;
    const bf16_t* const q_col = g.Q + q0;
    auto issue = [&](int sl) {          // sl: slab index within the segment
      unsigned char* st = sb_smem + (sl % STAGES) * STAGE_BYTES;
      const int64_t r0 = (int64_t)(s_beg + sl) * SB_BK;
#pragma unroll
      for (int i = 0; i < XI; ++i) {
        const int row = (wave * XI + i) * (64 / CX) + lane / CX;
        const int ch = (lane % CX) ^ (2 * (row & 3));
        int64_t grow = r0 + row;
        if (grow > g.m - 1) grow = g.m - 1;
        if (col0 + ch * 8 + 8 <= g.n)
        {
          if (g.stream_x) sb_async16_stream(x_col + grow * g.ldx + ch * 8, st + (wave * XI + i) * 1024);
          else sb_async16(x_col + grow * g.ldx + ch * 8, st + (wave * XI + i) * 1024);
        }
      }
#pragma unroll
      for (int i = 0; i < QI; ++i) {
        const int row = (wave * QI + i) * (64 / CQ) + lane / CQ;
        const int ch = (lane % CQ) ^ (2 * (row & 3));
        int64_t grow = r0 + row;
        if (grow > g.m - 1) grow = g.m - 1;
        if (q0 + ch * 8 + 8 <= g.l)
          sb_async16(q_col + grow * g.ldq + ch * 8, st + X_BYTES + (wave * QI + i) * 1024);
      }
    };

    f32x16 acc[NTQ][NTX];
#pragma unroll
    for (int i = 0; i < NTQ; ++i)
#pragma unroll
      for (int j = 0; j < NTX; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // fragments of K step ks of a stage
    auto read_frags = [&](const unsigned char* st, int ks, s16x8* a, s16x8* b) {
#pragma unroll
      for (int i = 0; i < NTQ; ++i) {
        const s16x4 lo = sb_read_tr(st + q_off[i] + (16 * ks) * QPITCH);
        const s16x4 hi = sb_read_tr(st + q_off[i] + (16 * ks + 4) * QPITCH);
        a[i] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      }
#pragma unroll
      for (int j = 0; j < NTX; ++j) {
        const s16x4 lo = sb_read_tr(st + x_off[j] + (16 * ks) * XPITCH);
        const s16x4 hi = sb_read_tr(st + x_off[j] + (16 * ks + 4) * XPITCH);
        b[j] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      }
    };
    // one slab: 4 K steps of 16 rows, the fragments of a step read while the step before is multiplied
    auto slab_mac = [&](const unsigned char* st) {
      s16x8 a[2][NTQ], b[2][NTX];
      read_frags(st, 0, a[0], b[0]);
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        if (ks + 1 < 4) read_frags(st, ks + 1, a[(ks + 1) & 1], b[(ks + 1) & 1]);
#pragma unroll
        for (int i = 0; i < NTQ; ++i)
#pragma unroll
          for (int j = 0; j < NTX; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[ks & 1][i]),
                                                                __builtin_bit_cast(bf16x8, b[ks & 1][j]),
                                                                acc[i][j], 0, 0, 0);
      }
    };

#pragma unroll
    for (int p = 0; p < STAGES - 1; ++p)
      if (p < nslab) issue(p);
#pragma nounroll
    for (int sl = 0; sl < nslab; ++sl) {
      // slab sl has landed once at most the copies of the (STAGES - 2) younger slabs are pending
      if (sl + STAGES - 1 <= nslab) SB_WAIT_VMCNT((STAGES - 2) * LOADS);
      else SB_WAIT_VMCNT(0);
      sb_barrier_keep_copies();                      // everyone's copies landed; slab sl-1 is consumed
      if (sl + STAGES - 1 < nslab) issue(sl + STAGES - 1);
      unsigned char* st = sb_smem + (sl % STAGES) * STAGE_BYTES;
      const int64_t left = g.m - (int64_t)(s_beg + sl) * SB_BK;
      if (left < SB_BK) {
        // last slab of the matrix: its rows past m (copies of row m - 1) are cleared in LDS
        const u32x4 z = {0u, 0u, 0u, 0u};
        for (int e = (int)left * (XPITCH / 16) + t; e < SB_BK * (XPITCH / 16); e += 64 * NW)
          *(u32x4*)(st + e * 16) = z;
        for (int e = (int)left * (QPITCH / 16) + t; e < SB_BK * (QPITCH / 16); e += 64 * NW)
          *(u32x4*)(st + X_BYTES + e * 16) = z;
        sb_barrier_lds();
      }
      slab_mac(st);
    }
    sb_barrier_keep_copies();                        // the stages may be refilled by a next segment

    // partial tile: rows = columns of Q, columns = columns of X
    float* dst = g.part + ((int64_t)share * g.segs_max + seg) * (BMQ * BNX);
#pragma unroll
    for (int i = 0; i < NTQ; ++i)
#pragma unroll
      for (int j = 0; j < NTX; ++j) {
        const int colw = wn * 32 * NTX + 32 * j + (lane & 31);
        if (col0 + colw >= g.n) continue;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int qw = wm * 32 * NTQ + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          if (q0 + qw < g.l) dst[qw * BNX + colw] = acc[i][j][r];
        }
      }
    ++seg;
  }
}

// V tile blockIdx.y = sum of the partial tiles that cover it, in the order of the shares; a thread owns
// groups of 4 consecutive columns.  The range of shares of the tile is uniform per block.
template <int LPG>   // lanes per output group: 4 when an output tile has many partial tiles, else 1
__global__ __launch_bounds__(256) void project_sum_kernel(ProjectArgs g) {
  const int64_t tile = blockIdx.y;
  const int64_t lo_item = tile * g.slabs, hi_item = lo_item + g.slabs;
  // first share [items w / wgs, items (w+1) / wgs) that reaches into the tile
  int64_t w_lo = lo_item * g.wgs / g.items;
  while (g.items * (w_lo + 1) / g.wgs <= lo_item) ++w_lo;
  int64_t w_hi = w_lo;                               // exclusive
  while (w_hi < g.wgs && g.items * w_hi / g.wgs < hi_item) ++w_hi;
  const int64_t tile_floats = (int64_t)g.bmq * g.bnx;
  // offsets of the tile's partial tiles, worked out once per block (64-bit divisions)
  __shared__ int64_t slot_off[PJ_MAX_PARTS];
  const int nparts = (int)(w_hi - w_lo);               // <= PJ_MAX_PARTS by the launcher's cap
  for (int i = threadIdx.x; i < nparts; i += 256) {
    const int64_t w = w_lo + i;
    const int64_t first_tile = (g.items * w / g.wgs) / g.slabs;
    slot_off[i] = (w * g.segs_max + (tile - first_tile)) * tile_floats;
  }
  __syncthreads();
  const int qb = (int)(tile / g.col_blocks), cb = (int)(tile - (int64_t)qb * g.col_blocks);
  const int bnx4 = g.bnx >> 2;
  const int groups = g.bmq * bnx4;
  // LPG = 4 lanes per group of 4 columns: lane `sub` adds the partial tiles sub, sub + 4, ... in
  // ascending order and the four sums are combined as (s0 + s1) + (s2 + s3), a fixed order;
  // LPG = 1: one lane adds them all in ascending order
  constexpr int GPB = 256 / LPG;                         // groups per block and trip
  const int sub = threadIdx.x % LPG;
  for (int e0 = blockIdx.x * GPB; e0 < groups; e0 += gridDim.x * GPB) {
    const int e = e0 + threadIdx.x / LPG;
    const int ec = e < groups ? e : groups - 1;          // idle lanes redo the last group, never store
    const int qw = ec / bnx4, cw = (ec - qw * bnx4) << 2;
    const int64_t q = (int64_t)qb * g.bmq + qw, col = (int64_t)cb * g.bnx + cw;
    const float* base = g.part + (int64_t)qw * g.bnx + cw;
    f32x4 s4 = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int i = sub; i < nparts; i += 8 * LPG) {
      // up to eight partial tiles at a time: loads first (an unused slot re-reads a valid one)
      f32x4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = *(const f32x4*)(base + slot_off[(i + LPG * u < nparts) ? i + LPG * u : i]);
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (i + LPG * u < nparts) s4 += v[u];
    }
    if (LPG == 4) {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        s4[u] += __shfl_xor(s4[u], 1);
        s4[u] += __shfl_xor(s4[u], 2);
      }
    }
    if (sub != 0 || e >= groups || q >= g.l || col >= g.n) continue;
    if (g.out_ek == EK_F32) {
      *(f32x4*)((float*)g.V + q * g.n + col) = s4;
    } else {
      bf16x4 o;
#pragma unroll
      for (int u = 0; u < 4; ++u) o[u] = (bf16_t)s4[u];
      *(bf16x4*)((bf16_t*)g.V + q * g.n + col) = o;
    }
  }
}

// Tile shape and ring depth (bmq = 64 ntq whatever the wave layout is; the launcher picks the
// layout).  Up to 128 columns of Q: 128-column tiles with a two-stage ring, so that two workgroups
// share a CU (one hides the other's waits) and the partial tiles stay small.  Wider Q: one
// workgroup per CU, three stages of 128 columns, or for tall matrices (where the partial tiles
// are small against X) 256 columns with two stages.  All but the narrowest run eight waves.
static inline void project_shape_for(int l, int64_t m, int64_t n, int* ntq, int* ntx, int* stages, int* wn) {
  *wn = 2;
  // (a single column block, as in the LoRA gradient: 64-column tiles of Q, so that the workgroups
  // that share the rows of a tall Q are four times as many -- one CU pulls only about 28 GB/s)
  if (l <= 64 || n <= 128) { *ntq = 1; *ntx = 2; *stages = 2; }
  else if (l <= 128) { *ntq = 2; *ntx = 2; *stages = 2; }
  else if (m < 32768 || n < 1024) { *ntq = 4; *ntx = 2; *stages = 3; }   // (a narrow X, as in the LoRA gradient, has no use for 256-column tiles)
  else { *ntq = 4; *ntx = 2; *stages = 2; *wn = 4; }
}
static size_t project_lds_bytes(int ntq, int ntx, int stages, int wn) {
  return (size_t)stages * SB_BK * (64 * ntq + 32 * ntx * wn) * 2;
}
// Fills in the work split of a projection (everything the kernels derive their indexing from).
static void project_plan(ProjectArgs* g) {
  int ntq, ntx, stages, wn;
  project_shape_for(g->l, g->m, g->n, &ntq, &ntx, &stages, &wn);
  g->bmq = 64 * ntq;
  g->bnx = 32 * ntx * wn;
  g->slabs = (int)ceil_div64(g->m, SB_BK);
  g->col_blocks = (int)ceil_div64(g->n, g->bnx);
  const int64_t tiles = (int64_t)g->col_blocks * ceil_div64(g->l, g->bmq);
  g->items = tiles * g->slabs;
  const int64_t per_cu = std::max<int64_t>(1, std::min<int64_t>(2, (160 * 1024) / (int64_t)project_lds_bytes(ntq, ntx, stages, wn)));
  // at least 4 slabs per workgroup: a partial tile costs as much as a slab to write and sum
  int64_t wgs = std::min<int64_t>(256 * per_cu, ceil_div64(g->items, 4));
  // and at most 32 partial tiles per output tile (64 for a single column block, where the grid
  // would otherwise be a few dozen workgroups): the sum walks them one after the other
  wgs = std::min<int64_t>(wgs, (g->n <= 128 ? 64 : 32) * tiles);
  wgs = std::max<int64_t>(1, std::min<int64_t>(wgs, g->items));
  // hard bound the sum kernel relies on: shares of floor(items / wgs) slabs or more put at most
  // ceil(slabs / share) + 1 partial tiles on an output tile
  while (wgs > 1 && ceil_div64(g->slabs, std::max<int64_t>(1, g->items / wgs)) + 1 > PJ_MAX_PARTS)
    wgs = wgs * 3 / 4;
  g->wgs = (int)wgs;
  // a share of ceil(items / wgs) consecutive items touches at most this many output tiles
  g->segs_max = (int)(ceil_div64(ceil_div64(g->items, wgs), g->slabs) + 1);
}
static size_t project_part_floats(int64_t m, int64_t n, int l) {
  ProjectArgs g;
  g.m = m; g.n = n; g.l = l;
  project_plan(&g);
  return (size_t)g.wgs * g.segs_max * g.bmq * g.bnx;
}

template <int NTQ, int NTX, int STAGES, int WN, int ROLE, int WQ = 2>
static int launch_project_shape(hipStream_t s, const ProjectArgs& g, const char* name) {
  static std::atomic<bool> attr_done{false};
  const size_t lds = project_lds_bytes(NTQ * WQ / 2, NTX, STAGES, WN);
  if (lds > 64 * 1024 && !attr_done.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute((const void*)project_mfma_kernel<NTQ, NTX, STAGES, WN, ROLE, WQ>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return hip_fail(e, "hipFuncSetAttribute(project LDS)");
    attr_done.store(true, std::memory_order_release);
  }
  LORACT_LAUNCH(name, s, (project_mfma_kernel<NTQ, NTX, STAGES, WN, ROLE, WQ>), dim3((unsigned)g.wgs), dim3(64 * WQ * WN), lds, g);
  return LORACT_OK;
}

template <int ROLE>
static int launch_project_role(hipStream_t s, const ProjectArgs& g, const char* name) {
  if (g.l <= 64 || g.n <= 128) return launch_project_shape<1, 2, 2, 2, ROLE>(s, g, name);
  if (g.l <= 128) return launch_project_shape<1, 2, 2, 2, ROLE, 4>(s, g, name);
  if (g.m < 32768 || g.n < 1024) return launch_project_shape<2, 2, 3, 2, ROLE, 4>(s, g, name);
  return launch_project_shape<4, 2, 2, 4, ROLE>(s, g, name);
}
static int launch_project_main(hipStream_t s, const ProjectArgs& g, const char* name, int role) {
  return role == PJ_LORA_UTG ? launch_project_role<PJ_LORA_UTG>(s, g, name) : launch_project_role<PJ_PROJECT>(s, g, name);
}
static int launch_project_sum(hipStream_t s, const ProjectArgs& g) {
  const int64_t tiles = (int64_t)g.col_blocks * ceil_div64(g.l, g.bmq);
  const int groups = g.bmq * (g.bnx >> 2);
  // enough blocks per tile to occupy the machine, each thread at least one group
  // four lanes per group pay off when a tile has many partial tiles to walk through
  const bool wide = g.wgs >= 8 * tiles;
  const int gpb = wide ? 64 : 256;
  int bx = (int)std::max<int64_t>(1, std::min<int64_t>(ceil_div64(groups, gpb), ceil_div64(4096, tiles)));
  if (wide) LORACT_LAUNCH("project_sum", s, project_sum_kernel<4>, dim3((unsigned)bx, (unsigned)tiles), dim3(256), 0, g);
  else LORACT_LAUNCH("project_sum", s, project_sum_kernel<1>, dim3((unsigned)bx, (unsigned)tiles), dim3(256), 0, g);
  return LORACT_OK;
}

// Requires 16-byte aligned rows of Q, X and V (l, ldq, ldx, n multiples of 8; checked by the
// caller); part: project_part_floats(m, n, l) floats.
static int launch_project_mfma(hipStream_t s, ProjectArgs g, const char* name = "project", int role = PJ_PROJECT) {
  project_plan(&g);
  // (the projection is the last reader of X inside a compress: above 128 MB its lines only push the
  // basis, which every column block re-reads, out of L2 -- measured at 8192 x 11008: twice the
  // algorithmic bytes fetched, 108 -> 103 us)
  g.stream_x = sb_streams_past_cache(g.m * g.n * 2, 128);
  if (g.wgs > SB_MAX_WGS) return LORACT_ERR_UNSUPPORTED;
  sb_xcd_share_order(g.items, g.wgs, g.slabs, g.share_of);
  int rc = launch_project_main(s, g, name, role);
  if (rc != LORACT_OK) return rc;
  return launch_project_sum(s, g);
}

// ---------------------------------------------------------------------------------------------
// reconstruct: Xhat (m x n, bf16) = U (m x k) V (k x n), a product with a short inner dimension
// whose cost is the m x n write.
//
// Work items are (column block of 128, row tile of 64), column block major; every workgroup
// takes an equal contiguous share of them, so the grid always matches the machine.  For its
// column block a workgroup keeps the V operand stationary IN REGISTERS (staged once through
// LDS, pair interleaved, then read out as matrix-core fragments), and streams the U row tiles
// -- contiguous 64 x k blocks of memory -- through a double-buffered LDS ring with asynchronous
// global -> LDS copies, one tile ahead.  The product is formed transposed (rows of the MFMA tile
// = columns of Xhat) so that a U fragment is one 16-byte LDS read; the finished tile is turned
// back through LDS and written as full 256-byte row segments.  Stores are not waited for: they
// drain while the next tile is multiplied.
//
// U tile layout in LDS: [row][2 NKS chunks of 16 bytes], chunk c of row r stored at position
// (c + r) mod 2 NKS, which spreads the fragment reads of consecutive rows over the banks.

#define RC_BM 64
#define RC_LDV (128 + 4)     // words per pair-row of the V staging tile (128 columns at a time)

struct ReconArgs {
  const bf16_t* U;       // m x k, ld = k
  const bf16_t* V;       // k x n, ld = n
  int64_t m, n;
  int k;
  bf16_t* Xhat;
  int64_t ldxh;
  int row_tiles;         // ceil(m / 64)
  int64_t items;         // column blocks * row_tiles
  int bn;                // columns per block
  int stream_out;        // Xhat is too large to stay cached: store it non-temporally
  unsigned short share_of[SB_MAX_WGS];   // share of the items that workgroup B takes
};


// NKS = number of 16-deep K steps = ceil(k / 16).  WIDE = false: four waves, 128 columns per
// block, waves 2 (64-column groups) x 2 (32-row halves).  WIDE = true (for k > 128, where a
// workgroup fills a CU's LDS anyway): eight waves, 256 columns per block, every wave 32 columns and
// both row halves -- half the U traffic and half the barriers per byte written.  With 32 columns
// a wave's V fragments take 64 registers instead of 128, so that two waves fit on a SIMD, and the
// copies and stores of a tile are issued by eight waves side by side (a wave gets a 1 KB memory
// instruction out only every ~150 clocks): 77 -> 64 us at 8192 x 11008 against four waves of 64
// columns.  The price is that every U fragment read from LDS feeds two matrix instructions instead
// of four: at k = 256 the LDS reads of a tile (8 waves x 32 KB) take as long as its matrix
// instructions, which is what bounds this kernel now (two independent workgroups per CU on
// 128-column blocks, with the staging tile swizzled instead of padded to fit 2 x 80 KB, were slower:
// 204 against 170 us at 65536 x 4096).
template <int NKS, bool WIDE>
__global__ __launch_bounds__(WIDE ? 512 : 256) void reconstruct_mfma_kernel(ReconArgs g) {
  constexpr int NW = WIDE ? 8 : 4, NT = 64 * NW;   // waves, threads
  constexpr int WN = WIDE ? 4 : 2;              // 64-column groups of the block
  constexpr int CT = WIDE ? 1 : 2;              // 32-column tiles per wave
  constexpr int RH = WIDE ? 2 : 1;              // 32-row halves per wave
  constexpr int BN = 64 * WN;
  constexpr int NST = RC_BM * (BN / 8) / NT;    // 16-byte stores per thread and tile
  constexpr int LDC = BN + 8;                   // bf16 elements per row of the output staging tile
  constexpr int CS_BYTES = RC_BM * LDC * 2;
  constexpr int CPR = 2 * NKS;                  // 16-byte chunks per U row in LDS
  constexpr int UBUF = RC_BM * CPR * 16;        // bytes per U buffer = CPR wave-wide copies
  constexpr int NCOPY_MIN = CPR / NW;           // fewest copy instructions any wave issues per tile
  extern __shared__ __attribute__((aligned(16))) unsigned char sb_smem[];
  bf16_t* Cs = (bf16_t*)sb_smem;                                   // [64][LDC]
  unsigned char* Ub = sb_smem + CS_BYTES;                          // 2 x UBUF
  unsigned int* Vs = (unsigned int*)sb_smem;                       // [NKS * 8][RC_LDV], prologue only

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wc = WIDE ? wave * 32 : (wave >> 1) * 64;   // first column of the wave inside the block
  const int wn = WIDE ? 0 : wave & 1;           // first 32-row half
  const int cvalid = g.k >> 3;                  // valid chunks per row (k is a multiple of 8)
  const bf16x8 zero8 = {(bf16_t)0.0f, (bf16_t)0.0f, (bf16_t)0.0f, (bf16_t)0.0f,
                        (bf16_t)0.0f, (bf16_t)0.0f, (bf16_t)0.0f, (bf16_t)0.0f};

  // copy of U rows [rt * 64, +64) into buffer `buf`; rows past m repeat the last row (never stored)
  auto issue_copy = [&](int rt, int buf) {
    const int64_t r0 = (int64_t)rt * RC_BM;
#pragma unroll
    for (int i = 0; i < (CPR + NW - 1) / NW; ++i) {
      const int ins = wave + NW * i;
      if (ins < CPR) {
        const int p = ins * 64 + lane;
        const int row = p / CPR, pos = p % CPR;
        int c = pos - row % CPR;
        if (c < 0) c += CPR;
        int64_t grow = r0 + row;
        if (grow > g.m - 1) grow = g.m - 1;
        if (c < cvalid)
          sb_async16(g.U + grow * g.k + c * 8, Ub + buf * UBUF + ins * 1024);
      }
    }
  };

  const int share = g.share_of[blockIdx.x];
  const int64_t item_begin = g.items * share / gridDim.x;
  const int64_t item_end = g.items * (share + 1) / gridDim.x;
  int64_t item = item_begin;
  while (item < item_end) {
    // ---- segment: the items of one column block
    const int64_t cb = item / g.row_tiles;
    const int rt_first = (int)(item - cb * g.row_tiles);
    const int64_t rt_stop = rt_first + (item_end - item);
    const int rt_last = (int)(rt_stop < g.row_tiles ? rt_stop : g.row_tiles);   // exclusive
    item += rt_last - rt_first;
    const int64_t col0 = cb * BN;

    // this wave's V fragments (64 columns of Xhat, all K steps), staged 128 columns at a time
    bf16x8 a[NKS][CT];
#pragma unroll
    for (int h = 0; h < WN / 2; ++h) {
      __syncthreads();   // LDS is free: a previous segment (or half) is done with it
      for (int c = t; c < NKS * 8 * 16; c += NT) {
        const int p = c >> 4, ch = c & 15;
        const int64_t col = col0 + 128 * h + ch * 8;
        const bool cok = col + 8 <= g.n;
        const bf16_t* src = g.V + (int64_t)(2 * p) * g.n + col;
        const bf16x8 lo = (cok && 2 * p < g.k) ? *(const bf16x8*)src : zero8;
        const bf16x8 hi = (cok && 2 * p + 1 < g.k) ? *(const bf16x8*)(src + g.n) : zero8;
        u32x4 w0, w1;
        sb_interleave(lo, hi, &w0, &w1);
        unsigned int* d = Vs + p * RC_LDV + ch * 8;
        *(u32x4*)d = w0;
        *(u32x4*)(d + 4) = w1;
      }
      __syncthreads();
      if (WN == 2 || (wc >> 7) == h) {
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
          for (int i = 0; i < CT; ++i)
            a[ks][i] = sb_pair_frag(Vs, RC_LDV, ks * 8 + 4 * (lane >> 5), (wc & 127) + 32 * i + (lane & 31));
      }
    }
    __syncthreads();   // the V staging area is free: it overlaps Cs and the U buffers
    if ((g.k & 15) != 0 && t < 2 * RC_BM) {
      // k = 16 NKS - 8: the last chunk of every row is padding that no copy writes
      const int buf = t / RC_BM, row = t % RC_BM;
      *(bf16x8*)(Ub + buf * UBUF + (row * CPR + (CPR - 1 + row) % CPR) * 16) = zero8;
    }

    issue_copy(rt_first, 0);
    for (int rt = rt_first; rt < rt_last; ++rt) {
      const int it = rt - rt_first, cur = it & 1;
      const bool has_next = rt + 1 < rt_last;
      // next tile into the other buffer: its last readers (tile it-1) are past a barrier
      if (has_next) issue_copy(rt + 1, cur ^ 1);
      // Wait for this tile's copies.  Younger than them, and allowed to stay in flight: the NST
      // stores of the previous tile (every tile but the last of the matrix is full, so each
      // wave issued exactly NST) and the copies just issued (at least NCOPY_MIN per wave).
      if (has_next) {
        if (it > 0) SB_WAIT_VMCNT(NST + NCOPY_MIN); else SB_WAIT_VMCNT(NCOPY_MIN);
      } else {
        if (it > 0) SB_WAIT_VMCNT(NST); else SB_WAIT_VMCNT(0);
      }
      sb_barrier_lds();   // copies of all waves landed; previous tile's reads of Cs are complete

      const unsigned char* ub = Ub + cur * UBUF;
      f32x16 acc[CT][RH];
#pragma unroll
      for (int i = 0; i < CT; ++i)
#pragma unroll
        for (int j = 0; j < RH; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
      const int urow = wn * 32 + (lane & 31);
      // U fragments are read one group of K steps ahead of the matrix instructions that use them
      constexpr int GS = WIDE ? 2 : 4;
      constexpr int NG = (NKS + GS - 1) / GS;
      bf16x8 b[2][GS][RH];
      auto read_group = [&](int gi, bf16x8 (*dst)[RH]) {
#pragma unroll
        for (int u = 0; u < GS; ++u) {
          const int ks = GS * gi + u;
          if (ks < NKS) {
            const int c = 2 * ks + (lane >> 5);
#pragma unroll
            for (int j = 0; j < RH; ++j) {
              const int ur = urow + 32 * j;
              dst[u][j] = *(const bf16x8*)(ub + (ur * CPR + (c + ur) % CPR) * 16);
            }
          }
        }
      };
      read_group(0, b[0]);
#pragma unroll
      for (int gi = 0; gi < NG; ++gi) {
        if (gi + 1 < NG) read_group(gi + 1, b[(gi + 1) & 1]);
#pragma unroll
        for (int u = 0; u < GS; ++u) {
          const int ks = GS * gi + u;
          if (ks < NKS) {
#pragma unroll
            for (int j = 0; j < RH; ++j)
#pragma unroll
              for (int i = 0; i < CT; ++i)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks][i], b[gi & 1][u][j], acc[i][j], 0, 0, 0);
          }
        }
      }
      // accumulator register r of lane l: column 8*(r/4) + 4*(l/32) + r%4 of Xhat, row l%32
#pragma unroll
      for (int i = 0; i < CT; ++i)
#pragma unroll
        for (int j = 0; j < RH; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            bf16x4 o;
#pragma unroll
            for (int u = 0; u < 4; ++u) o[u] = (bf16_t)acc[i][j][4 * q + u];
            const int col = wc + 32 * i + 8 * q + 4 * (lane >> 5);
            *(bf16x4*)(Cs + (urow + 32 * j) * LDC + col) = o;
          }
      sb_barrier_lds();
      const int64_t r0 = (int64_t)rt * RC_BM;
#pragma unroll
      for (int q0 = 0; q0 < NST; q0 += 4) {
        bf16x8 o[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int e = t + NT * (q0 + q);
          o[q] = *(const bf16x8*)(Cs + (e / (BN / 8)) * LDC + (e % (BN / 8)) * 8);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int e = t + NT * (q0 + q);
          const int row = e / (BN / 8), ch = e % (BN / 8);
          const int64_t grow = r0 + row, col = col0 + ch * 8;
          if (grow < g.m && col + 8 <= g.n) {
            if (g.stream_out) __builtin_nontemporal_store(o[q], (bf16x8*)(g.Xhat + grow * g.ldxh + col));
            else *(bf16x8*)(g.Xhat + grow * g.ldxh + col) = o[q];
          }
        }
      }
    }
  }
}

static inline int reconstruct_wn_for(int nks) { return (nks > 8 && nks <= 16) ? 4 : 2; }
static size_t reconstruct_lds_bytes(int nks) {
  const int bn = 64 * reconstruct_wn_for(nks);
  const size_t run = (size_t)RC_BM * (bn + 8) * 2 + (size_t)2 * RC_BM * 2 * nks * 16;
  const size_t stage = (size_t)nks * 8 * RC_LDV * sizeof(unsigned int);
  return std::max(run, stage);
}

template <int NKS>
static int launch_reconstruct_nks(hipStream_t s, const ReconArgs& g, dim3 grid) {
  constexpr bool WIDE = NKS > 8 && NKS <= 16;    // beyond 16 K steps the V fragments leave no registers
  static std::atomic<bool> attr_done{false};
  const size_t lds = reconstruct_lds_bytes(NKS);
  if (lds > 64 * 1024 && !attr_done.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute((const void*)reconstruct_mfma_kernel<NKS, WIDE>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return hip_fail(e, "hipFuncSetAttribute(reconstruct LDS)");
    attr_done.store(true, std::memory_order_release);
  }
  LORACT_LAUNCH("reconstruct", s, (reconstruct_mfma_kernel<NKS, WIDE>), grid, dim3(WIDE ? 512 : 256), lds, g);
  return LORACT_OK;
}

// Requires k % 8 == 0 and 16-byte aligned U, V, Xhat rows (checked by the caller).
static int launch_reconstruct_mfma(hipStream_t s, ReconArgs g) {
  const int nks = (g.k + 15) / 16;
  g.stream_out = sb_streams_past_cache(g.m * g.n * 2);
  g.bn = 64 * reconstruct_wn_for(nks);
  g.row_tiles = (int)ceil_div64(g.m, RC_BM);
  g.items = ceil_div64(g.n, g.bn) * g.row_tiles;
  // as many workgroups as stay resident: LDS allows 160 KB per CU, registers about 2 per CU
  const int64_t per_cu = std::max<int64_t>(1, std::min<int64_t>(2, (160 * 1024) / (int64_t)reconstruct_lds_bytes(nks)));
  const int64_t wgs = std::min<int64_t>(g.items, 256 * per_cu);
  if (wgs > SB_MAX_WGS) return LORACT_ERR_UNSUPPORTED;     // (share_of has SB_MAX_WGS entries)
  sb_xcd_share_order(g.items, (int)wgs, g.row_tiles, g.share_of);
  dim3 grid((unsigned)wgs);
  switch (nks) {
#define RC_CASE(N) case N: return launch_reconstruct_nks<N>(s, g, grid);
    RC_CASE(1) RC_CASE(2) RC_CASE(3) RC_CASE(4) RC_CASE(5) RC_CASE(6) RC_CASE(7) RC_CASE(8)
    RC_CASE(9) RC_CASE(10) RC_CASE(11) RC_CASE(12) RC_CASE(13) RC_CASE(14) RC_CASE(15)
    RC_CASE(16) RC_CASE(17) RC_CASE(18) RC_CASE(19) RC_CASE(20)
#undef RC_CASE
    default: return LORACT_ERR_UNSUPPORTED;
  }
}

// ---------------------------------------------------------------------------------------------
// Last contraction of the LoRA gradient: dA (n x r) = scale * V^T (T_hi + T_lo), with V (k x n,
// bf16) and the k x 2rp fp32 matrix [T_hi | T_lo] produced by the split-bf16 projection.
// A workgroup owns 32 columns of V; its 256 threads are 32 columns x 8 groups of the contraction
// index, so that each thread's chain of loads is k / 8 long; the 8 partial sums of an output are
// added in a fixed order through LDS.  RP = 16 RP16 is the padded LoRA rank.

template <int RP16>
__global__ __launch_bounds__(256) void lora_vtt_kernel(const bf16_t* V, const float* Tsplit,
                                                       int k, int64_t n, int r, float scale,
                                                       float* dA) {
  constexpr int RP = 16 * RP16;
  extern __shared__ float lv_T[];   // T [k][RP], then partial sums [8][32][RP + 1]
  float* const red = lv_T + k * RP;
  for (int e = threadIdx.x; e < k * RP; e += 256) {
    const int q = e / RP, c = e - q * RP;
    lv_T[e] = Tsplit[(int64_t)q * 2 * RP + c] + Tsplit[(int64_t)q * 2 * RP + RP + c];
  }
  __syncthreads();
  const int cj = threadIdx.x & 31, kg = threadIdx.x >> 5;
  const int64_t j = (int64_t)blockIdx.x * 32 + cj;
  const int64_t jc = j < n ? j : n - 1;        // columns past the end repeat the last one, never stored
  const int per = (k + 7) >> 3;
  const int q_begin = kg * per, q_end = (q_begin + per < k) ? q_begin + per : k;
  f32x4 acc[RP / 4];
#pragma unroll
  for (int c = 0; c < RP / 4; ++c) acc[c] = (f32x4){0.0f, 0.0f, 0.0f, 0.0f};
  int q = q_begin;
  for (; q + 8 <= q_end; q += 8) {            // 8 independent loads in flight
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = (float)V[(int64_t)(q + u) * n + jc];
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
      for (int c = 0; c < RP / 4; ++c) acc[c] += v[u] * *(const f32x4*)(lv_T + (q + u) * RP + 4 * c);
  }
  for (; q < q_end; ++q) {
    const float v = (float)V[(int64_t)q * n + jc];
#pragma unroll
    for (int c = 0; c < RP / 4; ++c) acc[c] += v * *(const f32x4*)(lv_T + q * RP + 4 * c);
  }
#pragma unroll
  for (int c = 0; c < RP / 4; ++c)
#pragma unroll
    for (int u = 0; u < 4; ++u) red[(kg * 32 + cj) * (RP + 1) + 4 * c + u] = acc[c][u];
  __syncthreads();
  for (int o = threadIdx.x; o < 32 * RP; o += 256) {
    const int col = o / RP, c = o - col * RP;
    float sum = 0.0f;
#pragma unroll
    for (int g8 = 0; g8 < 8; ++g8) sum += red[(g8 * 32 + col) * (RP + 1) + c];
    const int64_t jo = (int64_t)blockIdx.x * 32 + col;
    if (jo < n && c < r) dA[jo * r + c] = scale * sum;
  }
}

template <int RP16>
static int launch_lora_vtt_rp(hipStream_t s, const bf16_t* V, const float* Tsplit, int k, int64_t n, int r,
                              float scale, float* dA) {
  const int rp = 16 * RP16;
  const size_t lds = ((size_t)k * rp + (size_t)8 * 32 * (rp + 1)) * sizeof(float);
  static std::atomic<size_t> attr_bytes{64 * 1024};
  if (lds > attr_bytes.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute((const void*)lora_vtt_kernel<RP16>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return hip_fail(e, "hipFuncSetAttribute(lora_vtt LDS)");
    attr_bytes.store(lds, std::memory_order_release);
  }
  LORACT_LAUNCH("lora_vtt", s, lora_vtt_kernel<RP16>, dim3((unsigned)ceil_div64(n, 32)), dim3(256), lds, V,
                Tsplit, k, n, r, scale, dA);
  return LORACT_OK;
}
static int launch_lora_vtt(hipStream_t s, const bf16_t* V, const float* Tsplit, int k, int64_t n, int r,
                           int rp, float scale, float* dA) {
  switch (rp / 16) {
    case 1: return launch_lora_vtt_rp<1>(s, V, Tsplit, k, n, r, scale, dA);
    case 2: return launch_lora_vtt_rp<2>(s, V, Tsplit, k, n, r, scale, dA);
    case 3: return launch_lora_vtt_rp<3>(s, V, Tsplit, k, n, r, scale, dA);
    case 4: return launch_lora_vtt_rp<4>(s, V, Tsplit, k, n, r, scale, dA);
    default: return LORACT_ERR_UNSUPPORTED;
  }
}
