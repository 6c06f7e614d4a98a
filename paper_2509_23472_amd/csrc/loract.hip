// libloract: C ABI entry points and host-side orchestration.  See include/loract.h.
#include "common.h"
#include "gemm_bf16.h"
#include "gemm_f64.h"
#include "chol.h"
#include "ortho_f64.h"
#include "stream_bf16.h"
#include "eig_jacobi.h"
#include "prenorm.h"

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <mutex>
#include <set>
#include <string>

// ---------------------------------------------------------------------------------------------
// Small utility kernels.

// Copies the sampled row ids (passed by value in the kernel arguments, so no host-to-device
// copy is needed) into the workspace and clears the status word.
__global__ void store_indices_kernel(IdxPack pack, int count, int32_t* dst, int32_t* status) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t < count) dst[t] = pack.v[t];
  if (t == 0 && status) *status = 0;
}

__global__ __launch_bounds__(256) void convert_kernel(const void* src, int src_ek, void* dst,
                                                      int dst_ek, int64_t count) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count;
       i += (int64_t)gridDim.x * blockDim.x)
    store_f64(dst, i, dst_ek, load_f64(src, i, src_ek));
}

static int launch_convert(hipStream_t s, const void* src, int src_ek, void* dst, int dst_ek,
                          int64_t count) {
  if (count <= 0) return LORACT_OK;
  int blocks = (int)std::min<int64_t>(ceil_div64(count, 256), 4096);
  LORACT_LAUNCH("convert", s, convert_kernel, dim3(blocks), dim3(256), 0, src, src_ek, dst, dst_ek,
                count);
  return LORACT_OK;
}

// splitmix64: state += golden; output = mix(state).
__host__ __device__ inline uint64_t splitmix64_mix(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
#define SPLITMIX_GOLDEN 0x9E3779B97F4A7C15ull

__global__ __launch_bounds__(256) void gaussian_kernel(void* dst, int ek, int64_t count,
                                                       uint64_t seed) {
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < count;
       e += (int64_t)gridDim.x * blockDim.x) {
    const uint64_t h = splitmix64_mix(seed + (uint64_t)(e + 1) * SPLITMIX_GOLDEN);
    const double u1 = ((double)(uint32_t)(h >> 32) + 1.0) * (1.0 / 4294967296.0);
    const double u2 = (double)(uint32_t)(h & 0xFFFFFFFFull) * (1.0 / 4294967296.0);
    const double z = sqrt(-2.0 * log(u1)) * cospi(2.0 * u2);
    store_f64(dst, e, ek, z);
  }
}

// ---------------------------------------------------------------------------------------------
// Host helpers.

static bool dtype_ok(int d) { return d == LORACT_F32 || d == LORACT_BF16; }

static int sample_indices_host(int64_t m, int32_t l, uint64_t seed, int32_t* out) {
  if (!out || l < 0 || m < 0 || l > m || m > 0x7fffffffLL) return LORACT_ERR_INVALID_ARG;
  std::set<int64_t> chosen;
  uint64_t state = seed;
  for (int64_t i = m - l; i < m; ++i) {
    state += SPLITMIX_GOLDEN;
    const uint64_t r = splitmix64_mix(state);
    const int64_t j = (int64_t)(r % (uint64_t)(i + 1));
    if (!chosen.insert(j).second) chosen.insert(i);
  }
  int32_t c = 0;
  for (int64_t v : chosen) out[c++] = (int32_t)v;
  return LORACT_OK;
}

// Workspace layout shared by loract_compress and loract_rsvd.
struct Plan {
  int bf16_path;
  int l;                 // sketch columns
  int kp;                // l rounded up to a multiple of 16 (column count of the fp32 work buffers)
  int gram_splits, proj_splits;
  size_t off_idx, off_a, off_b, off_ub, off_g, off_rinv, off_dpart, off_fpart, off_zt;
  size_t off_bmat, off_eig, off_omega, off_dinv, off_q1b, off_nsT, off_gbak, off_flag;
  int sketch_splits, bgram_splits;
  int sketch64_splits;    // K splits of the sketch on the float64 path
  size_t total;
};

static int pick_splits(int64_t tiles, int64_t K, int64_t min_k_per_split) {
  int64_t s = std::max<int64_t>(1, 1024 / std::max<int64_t>(1, tiles));
  s = std::min<int64_t>(s, std::max<int64_t>(1, K / min_k_per_split));
  return (int)std::min<int64_t>(s, 64);
}

static int validate_params(const loract_params* p, bool rsvd, int* l_out) {
  if (!p) return LORACT_ERR_INVALID_ARG;
  if (p->m < 1 || p->n < 1 || p->ldx < p->n || p->k < 1 || p->t < 0) return LORACT_ERR_INVALID_ARG;
  if (p->m > 0x7fffffffLL || p->n > 0x7fffffffLL) return LORACT_ERR_INVALID_ARG;
  if (!dtype_ok(p->x_dtype) || !dtype_ok(p->factor_dtype)) return LORACT_ERR_INVALID_ARG;
  if (p->k > p->m || p->k > p->n) return LORACT_ERR_INVALID_ARG;
  int l = p->l == 0 ? p->k : p->l;
  // l == k is Algorithm 1 (and the plain range finder); l > k (more sampled rows, or Gaussian
  // oversampling) ends with a truncation of the l x n factor to rank k
  if (l < p->k || l > p->m || l > p->n) return LORACT_ERR_INVALID_ARG;
  if (l > LORACT_MAX_RANK) return LORACT_ERR_UNSUPPORTED;
  if (p->x_dtype == LORACT_F32 && p->factor_dtype != LORACT_F32) return LORACT_ERR_UNSUPPORTED;
  *l_out = l;
  return LORACT_OK;
}

static int make_plan(const loract_params* p, bool rsvd, Plan* pl, bool truncate_always = false) {
  int l = 0;
  LORACT_TRY(validate_params(p, rsvd, &l));
  pl->l = l;
  pl->bf16_path = (p->x_dtype == LORACT_BF16);
  const int64_t m = p->m, n = p->n;
  pl->kp = (l + 15) / 16 * 16;
  const size_t ybytes = pl->bf16_path ? (size_t)m * pl->kp * 4 : (size_t)m * l * 8;
  const int64_t lt = ceil_div64(l, 64);
  pl->gram_splits = pick_splits(lt * lt, m, 64);
  pl->proj_splits = pick_splits(lt * ceil_div64(n, 64), m, 64);
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
  pl->off_idx = take(sizeof(int32_t) * LORACT_MAX_RANK);
  pl->off_a = take(ybytes);
  pl->off_b = take(ybytes);
  pl->off_ub = take(pl->bf16_path ? (size_t)m * l * 2 : 0);
  pl->off_g = take((size_t)pl->kp * pl->kp * 8);
  pl->off_rinv = take((size_t)l * l * 8);
  pl->off_dinv = take((size_t)pl->kp * 16 * 8);
  pl->off_q1b = take(pl->bf16_path ? (size_t)m * pl->kp * 2 : 0);
  pl->off_nsT = take(pl->bf16_path ? (size_t)pl->kp * pl->kp * 2 : 0);
  pl->off_gbak = take(pl->bf16_path ? (size_t)pl->kp * pl->kp * 8 : 0);
  pl->off_flag = take(64 + 8 * (64 * 16 + 128));   // flag word, up to 64 x 15 shares of ||E||^2, 100 of ||E^4||^2
  size_t dpart = (size_t)pl->gram_splits * l * l * 8;
  if (!pl->bf16_path) dpart = std::max(dpart, (size_t)pl->proj_splits * l * n * 8);
  // the float64 sketch splits the hidden dimension while the row tiles alone leave CUs idle
  pl->sketch64_splits = pl->bf16_path ? 1 : pick_splits(ceil_div64(m, 64) * lt, n, 64);
  if (pl->sketch64_splits > 1) dpart = std::max(dpart, (size_t)pl->sketch64_splits * m * l * 8);
  if (pl->bf16_path) dpart = std::max(dpart, gram_partial_bytes(m, pl->kp));
  if (pl->bf16_path) dpart = std::max(dpart, (size_t)pl->kp * pl->kp * 8);   // E^2 of the degree-4 finish
  const bool trunc = l > p->k || truncate_always;
  pl->bgram_splits = 1;
  if (trunc) {
    pl->bgram_splits = pick_splits(lt * lt, n, 256);
    dpart = std::max(dpart, (size_t)pl->bgram_splits * l * l * 8);
  }
  pl->off_dpart = take(dpart);
  size_t fpart = 0;
  pl->sketch_splits = 1;
  if (pl->bf16_path) {
    pl->sketch_splits = sketch_splits_for(m, n, pl->kp);
    // the matrix-core projection's partial tiles, or the generic product's split partials
    fpart = std::max(std::max(project_part_floats(m, n, l) * 4, (size_t)pl->proj_splits * l * n * 4),
                     pl->sketch_splits > 1 ? (size_t)pl->sketch_splits * m * pl->kp * 4 : (size_t)0);
  }
  pl->off_fpart = take(fpart);
  const bool need_zt = p->t > 0 || rsvd;
  pl->off_zt = take(need_zt ? (size_t)l * n * (pl->bf16_path ? 2 : 8) : 0);
  pl->off_bmat = take(trunc ? (size_t)l * n * (pl->bf16_path ? 4 : 8) : 0);
  // the Gram matrix of the l x n factor, the eigensolver's work matrix, the k leading eigenvectors
  pl->off_eig = take(trunc ? ((size_t)2 * l * l + ej_work_doubles(l)) * 8 : 0);
  pl->off_omega = take(rsvd ? (size_t)l * n * (pl->bf16_path ? 2 : 4) : 0);
  pl->total = off;
  return LORACT_OK;
}

// ---------------------------------------------------------------------------------------------
// Building blocks of Algorithm 1 on the device.

struct Ctx {
  hipStream_t s;
  const loract_params* p;
  Plan pl;
  char* ws;
  int32_t* status;
  const void* X;
  int x_ek;      // element kind of X
  int y_ek;      // element kind of the sketch / Q work buffers (fp32 on the bf16 path, fp64 otherwise)
};

template <typename T>
static T* ws_ptr(const Ctx& c, size_t off) { return (T*)(c.ws + off); }

// Y (m x l) = X * Bt^T where Bt is l x n, K-contiguous rows of length n (optionally gathered
// from X itself through the sampled row ids).  Algorithm 1: the sketch, and the second product of a power round.
// The matrix-core sketch can take the sampled row ids in its own kernel arguments (`pack`, and
// then also clears the status word), which saves the launch that stores them in the workspace.
static bool sketch_takes_ids(const Ctx& c) {
  return c.pl.bf16_path && sb_aligned(c.X, c.p->ldx) && c.p->n % 64 == 0;
}
static int sketch(const Ctx& c, const void* Bt, int64_t ldb, const int32_t* rows, void* Y,
                  const IdxPack* pack = nullptr) {
  const int64_t m = c.p->m, n = c.p->n;
  const int l = c.pl.l;
  if (c.pl.bf16_path) {
    if (sb_aligned(c.X, c.p->ldx) && sb_aligned(Bt, ldb) && n % 64 == 0) {
      SketchArgs a{};
      a.X = (const bf16_t*)c.X; a.ldx = c.p->ldx; a.m = m; a.n = n;
      a.B = (const bf16_t*)Bt; a.ldb = ldb; a.b_rows = rows; a.l = l; a.kp = c.pl.kp;
      a.Y = (float*)Y; a.part = ws_ptr<float>(c, c.pl.off_fpart); a.splits = c.pl.sketch_splits;
      a.k_per_split = 0; a.run_flag = nullptr;
      a.ids_in_args = 0; a.clear_status = nullptr;
      if (pack) { a.ids = *pack; a.ids_in_args = 1; a.clear_status = c.status; }
      return launch_sketch_mfma(c.s, a);
    }
    return launch_gemm_bf16("sketch_generic", c.s, (const bf16_t*)c.X, c.p->ldx, 1, (const bf16_t*)Bt,
                            ldb, 1, rows, m, l, n, Y, c.pl.kp, EK_F32, 1, nullptr, c.pl.kp);
  }
  return launch_gemm_f64("sketch_f64", c.s, c.X, c.p->ldx, 1, EK_F32, Bt, ldb, 1,
                         rows ? EK_F32 : EK_F64, rows, m, l, n, 1.0, Y, l, EK_F64, c.pl.sketch64_splits,
                         ws_ptr<double>(c, c.pl.off_dpart));
}

// Thin QR of Y (m x l) by two rounds of Cholesky QR with float64 Gram matrices (the orthonormalisations
// of Algorithm 1).  Y is overwritten; the orthonormal factor is written to Qout (element kind
// q_ek, leading dimension l).  `tmp` is a second m x l work buffer of Y's element kind.
static int orthonormalise(const Ctx& c, void* Y, void* tmp, void* Qout, int q_ek) {
  const int64_t m = c.p->m;
  const int l = c.pl.l;
  double* G = ws_ptr<double>(c, c.pl.off_g);
  double* Rinv = ws_ptr<double>(c, c.pl.off_rinv);
  double* dpart = ws_ptr<double>(c, c.pl.off_dpart);
  const void* src = Y;
  for (int round = 0; round < 2; ++round) {
    LORACT_TRY(launch_gemm_f64("gram", c.s, src, l, 0, c.y_ek, src, l, 0, c.y_ek, nullptr, l, l, m,
                               1.0, G, l, EK_F64, c.pl.gram_splits, dpart));
    // first round shifted by ~8 max(l, sqrt(m)) u trace(G), second round plain (see chol.h)
    const double shift_rel =
        round == 0 ? 8.0 * std::max((double)l, sqrt((double)m)) * 1.1102230246251565e-16 : 0.0;
    LORACT_TRY(launch_chol_inverse(c.s, G, Rinv, l, shift_rel, c.status));
    void* dst = round == 0 ? tmp : Qout;
    const int dst_ek = round == 0 ? c.y_ek : q_ek;
    LORACT_TRY(launch_gemm_f64("apply_rinv", c.s, src, l, 1, c.y_ek, Rinv, l, 0, EK_F64, nullptr, m,
                               l, l, 1.0, dst, l, dst_ek, 1, nullptr));
    src = dst;
  }
  return LORACT_OK;
}

// Tuning knob for measurements: LORACT_FUSED_SOLVE=0 in the environment runs the factorisation
// and the triangular solve of round 1 as two launches instead of one.
static bool fused_solve_enabled() {
  static const bool on = [] {
    const char* e = getenv("LORACT_FUSED_SOLVE");
    return !(e && e[0] == '0');
  }();
  return on;
}

// bf16 path: the same two rounds on the matrix cores.  Y is m x kp float32 (zero padded
// columns); round 1 factors the shifted Gram matrix and writes Q1 (float32) into tmp, round 2
// writes the orthonormal factor as `Q` (element kind q_ek, k columns, leading dimension k) and,
// if Qb is given, a bf16 copy with the same shape.
static int orthonormalise_mfma(const Ctx& c, const float* Y, float* tmp, void* Q, int q_ek,
                               bf16_t* Qb) {
  const int64_t m = c.p->m;
  const int l = c.pl.l, kp = c.pl.kp;
  double* G = ws_ptr<double>(c, c.pl.off_g);
  double* Dinv = ws_ptr<double>(c, c.pl.off_dinv);
  double* part = ws_ptr<double>(c, c.pl.off_dpart);
  double* Gbak = ws_ptr<double>(c, c.pl.off_gbak);
  bf16_t* Q1b = ws_ptr<bf16_t>(c, c.pl.off_q1b);
  bf16_t* nsT = ws_ptr<bf16_t>(c, c.pl.off_nsT);
  int32_t* ns_flag = ws_ptr<int32_t>(c, c.pl.off_flag);
  // the Newton-Schulz finish reuses the sketch kernel, which wants a K extent that is a multiple of 64
  const bool ns_ok = (kp % 64 == 0);
  CholArgs ch;
  ch.G = G; ch.G_backup = Gbak; ch.Dinv = Dinv; ch.k = l; ch.kp = kp; ch.tol = 0.0; ch.status = c.status;
  ch.shift_rel = 8.0 * std::max((double)l, sqrt((double)m)) * 1.1102230246251565e-16;
  ch.unshifted_thresh = chol_unshifted_thresh(l);
  ch.ns_e2 = nullptr; ch.ns_e2_count = 0; ch.ns_flag = nullptr; ch.ns_tol = 0.0; ch.ns_exact_tol = 0.0;
  ch.poly_p4 = nullptr; ch.poly_count = 0; ch.poly_hi_tol = 0.0; ch.poly_b4_tol = 0.0; ch.ready = nullptr;
  TrsmArgs t;
  t.L = G; t.Dinv = Dinv; t.m = m; t.kp = kp; t.k = l;
  // round 1: Q1 = Y R^{-1} (fp32, plus a bf16 copy for a possible Newton-Schulz finish)
  ch.round = 1;
  ch.ready = fused_solve_enabled() ? ns_flag + 1 : nullptr;     // progress word of the fused launch
  const bool fused = chol_trsm_fusable(ch, m);
  LORACT_TRY(launch_gram_mfma(c.s, Y, kp, m, kp, l, part, G, Gbak, nullptr, nullptr, fused ? ch.ready : nullptr));
  t.Y = Y; t.ldy = kp; t.Q = tmp; t.ldq = kp; t.out_ek = EK_F32; t.out_cols = kp;
  t.Qb = ns_ok ? Q1b : nullptr; t.ldqb = kp; t.skip_flag = nullptr;
  if (fused) {
    LORACT_TRY(launch_chol_trsm_fused(c.s, ch, t));
  } else {
    LORACT_TRY(launch_chol_blocked(c.s, ch));
    LORACT_TRY(launch_trsm_apply(c.s, t));
  }
  // round 2: either Q = Q1 (I - E/2) when E = Q1^T Q1 - I is small, or a second Cholesky QR
  double* ns_e2 = ws_ptr<double>(c, c.pl.off_flag) + 8;      // after the flag word
  ch.round = 2;
  const bool fused2 = chol_trsm_fusable(ch, m);
  LORACT_TRY(launch_gram_mfma(c.s, tmp, kp, m, kp, l, part, G, nullptr, ns_ok ? nsT : nullptr, ns_e2,
                              fused2 ? ch.ready : nullptr));
  ch.ns_e2 = ns_e2; ch.ns_e2_count = 64 * gram_nblocks(kp); ch.ns_flag = ns_flag;
  ch.ns_tol = ns_ok ? 0.015 : 0.0;
  // Tall matrices: when the first-order finish does not reach, a degree-4 correction is prepared
  // (two small launches on k x k matrices, which return at once when they are not needed; they
  // are only worth their fixed cost where a second factorisation and solve are expensive).
  if (ns_ok && m >= 32768) {
    NsPolyArgs np;
    np.G = G; np.P2 = part; np.T = nsT; np.e2 = ns_e2; np.e2_count = ch.ns_e2_count;
    np.p4 = ns_e2 + 64 * 16; np.k = l; np.kp = kp; np.lo_tol = ch.ns_tol; np.hi_tol = 2.0;
    LORACT_TRY(launch_ns_poly(c.s, np));
    ch.poly_p4 = np.p4; ch.poly_count = ns_poly_blocks(kp); ch.poly_hi_tol = np.hi_tol; ch.poly_b4_tol = 0.2;
  }
  ch.ns_exact_tol = 1e-6;             // Q1 is then orthonormal to 1e-6 already: nothing for round 2 to do
  t.Y = tmp; t.Q = Q; t.ldq = l; t.out_ek = q_ek; t.out_cols = l; t.Qb = Qb; t.ldqb = l;
  if (fused2) {
    t.skip_flag = nullptr;            // every workgroup of the fused launch takes the decision itself
    LORACT_TRY(launch_chol_trsm_fused(c.s, ch, t));
  } else {
    LORACT_TRY(launch_chol_blocked(c.s, ch));
    t.skip_flag = ns_flag;
    LORACT_TRY(launch_trsm_apply(c.s, t));
  }
  if (ns_ok) {
    // Q = Q1 + Q1b T^T (T symmetric) for flag 1, Q = Q1 for flag 2, nothing for flag 0: the
    // product kernel of the sketch with the finish fused into its epilogue
    SketchArgs a{};
    a.X = Q1b; a.ldx = kp; a.m = m; a.n = kp; a.B = nsT; a.ldb = kp; a.b_rows = nullptr; a.l = l; a.kp = kp;
    a.Y = nullptr; a.part = nullptr; a.splits = 1; a.k_per_split = 0; a.run_flag = ns_flag;
    a.fin_q1 = tmp; a.fin_q = Q; a.fin_qb = Qb; a.fin_ek = q_ek; a.fin_ld = l;
    LORACT_TRY(launch_sketch_mfma(c.s, a, "ns_correct"));
  } else {
    const int blocks = (int)std::min<int64_t>(ceil_div64(m * (kp / 4), 256), 2048);
    LORACT_LAUNCH("ns_finalize", c.s, ns_finalize_kernel, dim3(blocks), dim3(256), 0, (const float*)tmp,
                  (const float*)Y, m, kp, l, Q, q_ek, Qb, (const int32_t*)ns_flag);
  }
  return LORACT_OK;
}

// Bt (l x n) = Q^T X: the projection of Algorithm 1 (and the first product of a power round).
static int project(const Ctx& c, const void* Q, int q_ek, void* Bt, int out_ek) {
  const int64_t m = c.p->m, n = c.p->n;
  const int l = c.pl.l;
  if (c.pl.bf16_path) {
    if (sb_aligned(c.X, c.p->ldx) && sb_aligned(Q, l) && sb_aligned(Bt, n)) {
      ProjectArgs a;
      a.Q = (const bf16_t*)Q; a.ldq = l; a.X = (const bf16_t*)c.X; a.ldx = c.p->ldx; a.m = m; a.n = n;
      a.l = l; a.V = Bt; a.out_ek = out_ek; a.part = ws_ptr<float>(c, c.pl.off_fpart);
      return launch_project_mfma(c.s, a);
    }
    return launch_gemm_bf16("project_generic", c.s, (const bf16_t*)Q, l, 0, (const bf16_t*)c.X,
                            c.p->ldx, 0, nullptr, l, n, m, Bt, n, out_ek, c.pl.proj_splits,
                            ws_ptr<float>(c, c.pl.off_fpart));
  }
  return launch_gemm_f64("project_f64", c.s, Q, l, 0, q_ek, c.X, c.p->ldx, 0, EK_F32, nullptr, l, n,
                         m, 1.0, Bt, n, out_ek, c.pl.proj_splits, ws_ptr<double>(c, c.pl.off_dpart));
}

static int check_common(const void* X, const loract_params* p, void* U, void* V, void* ws,
                        size_t ws_bytes, bool rsvd, Ctx* c, hipStream_t s, int32_t* status,
                        bool truncate_always = false) {
  if (!X || !U || !V) return LORACT_ERR_INVALID_ARG;
  LORACT_TRY(make_plan(p, rsvd, &c->pl, truncate_always));
  if (!ws || ws_bytes < c->pl.total) return LORACT_ERR_WORKSPACE_TOO_SMALL;
  if (((uintptr_t)ws) % 16 != 0) return LORACT_ERR_INVALID_ARG;
  c->s = s;
  c->p = p;
  c->ws = (char*)ws;
  c->status = status;
  c->X = X;
  c->x_ek = p->x_dtype == LORACT_BF16 ? EK_BF16 : EK_F32;
  c->y_ek = c->pl.bf16_path ? EK_F32 : EK_F64;
  return LORACT_OK;
}

// Final orthonormalisation + projection shared by compress and the l == k case of rsvd:
// leaves U (m x l, factor dtype) and V (l x n, factor dtype).
static int finish_factors(const Ctx& c, void* Y, void* tmp, void* U, void* V) {
  const int64_t m = c.p->m;
  const int l = c.pl.l;
  const int f_ek = c.p->factor_dtype == LORACT_BF16 ? EK_BF16 : EK_F32;
  if (c.pl.bf16_path) {
    bf16_t* Ub = (bf16_t*)U;
    if (f_ek == EK_BF16) {
      LORACT_TRY(orthonormalise_mfma(c, (const float*)Y, (float*)tmp, U, EK_BF16, nullptr));
    } else {
      Ub = ws_ptr<bf16_t>(c, c.pl.off_ub);
      LORACT_TRY(orthonormalise_mfma(c, (const float*)Y, (float*)tmp, U, EK_F32, Ub));
    }
    return project(c, Ub, EK_BF16, V, f_ek);
  }
  // fp32 input: keep Q in float64 for the projection, hand out fp32 factors
  LORACT_TRY(orthonormalise(c, Y, tmp, Y, EK_F64));
  LORACT_TRY(launch_convert(c.s, Y, EK_F64, U, EK_F32, m * l));
  return project(c, Y, EK_F64, V, EK_F32);
}

// t rounds of [QR; Y = X (X^T Q)] (the power rounds of Algorithm 1).  Only Y is orthonormalised.
static int power_iterations(const Ctx& c, void* Y, void* tmp) {
  const int l = c.pl.l;
  for (int it = 0; it < c.p->t; ++it) {
    void* Zt = c.ws + c.pl.off_zt;
    if (c.pl.bf16_path) {
      bf16_t* Qb = ws_ptr<bf16_t>(c, c.pl.off_ub);
      LORACT_TRY(orthonormalise_mfma(c, (const float*)Y, (float*)tmp, Qb, EK_BF16, nullptr));
      LORACT_TRY(project(c, Qb, EK_BF16, Zt, EK_BF16));
    } else {
      LORACT_TRY(orthonormalise(c, Y, tmp, Y, EK_F64));
      LORACT_TRY(project(c, Y, EK_F64, Zt, EK_F64));
    }
    LORACT_TRY(sketch(c, Zt, c.p->n, nullptr, Y));
  }
  (void)l;
  return LORACT_OK;
}

// ---------------------------------------------------------------------------------------------
// Scratch memory owned by the library, for the one entry point that must not allocate
// (loract_lora_grad_static).  The array's name is only a host-side stand-in for the symbol: its
// device address is looked up once per device with hipGetSymbolAddress and that pointer is what
// kernels and copies receive.  Every GPU that loads the library holds its own copy until the
// process ends.

static __device__ __align__(256) unsigned char scratch[LORACT_STATIC_SCRATCH_BYTES];

#define LORACT_MAX_DEVICES 64
static std::mutex g_scratch_mu;
static void* g_scratch_ptr[LORACT_MAX_DEVICES];

// Device address of this GPU's `scratch` (looked up on the first call on each device).
static int static_scratch_ptr(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
  if (dev < 0 || dev >= LORACT_MAX_DEVICES) return LORACT_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
    if (!ptr) return LORACT_ERR_HIP;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return LORACT_OK;
}

// ---------------------------------------------------------------------------------------------
// C ABI.

extern "C" {

const char* loract_version(void) { return "loract-gfx950 0.1"; }

const char* loract_strerror(int code) {
  switch (code) {
    case LORACT_OK: return "ok";
    case LORACT_ERR_INVALID_ARG: return "invalid argument";
    case LORACT_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case LORACT_ERR_UNSUPPORTED: return "unsupported configuration";
    case LORACT_ERR_NOT_IMPLEMENTED: return "not implemented";
    case LORACT_ERR_HIP: return "HIP runtime error";
    default: return "unknown error";
  }
}

const char* loract_last_hip_error(void) { return g_host.last_hip_error.c_str(); }

int loract_sample_indices(int64_t m, int32_t l, uint64_t seed, int32_t* idx_host) {
  return sample_indices_host(m, l, seed, idx_host);
}

int loract_workspace_bytes(const loract_params* p, size_t* bytes) {
  if (!bytes) return LORACT_ERR_INVALID_ARG;
  Plan pl;
  // the RSVD layout with the truncation buffers is a superset of every other layout, so one
  // size serves loract_compress, loract_compress_adaptive and loract_rsvd
  loract_params q;
  if (!p) return LORACT_ERR_INVALID_ARG;
  q = *p;
  int rc = make_plan(&q, true, &pl, true);
  if (rc != LORACT_OK) return rc;
  *bytes = pl.total;
  return LORACT_OK;
}

// l > k: B = Q^T X (l x n) with Q an orthonormal basis of the l-column sketch Y, then the rank-k
// factors of the k leading singular triplets of B: U = Q W_k, V = W_k^T B, where the columns of
// W_k are the k leading eigenvectors of B B^T (Section 3.2; the setting of Theorem 4.3 when the
// sketch comes from l sampled rows).
static int truncate_factors(const Ctx& c, void* Y, void* tmp, void* U_dev, void* V_dev,
                            double energy = 1.0, int32_t* k_out = nullptr) {
  const loract_params* p = c.p;
  hipStream_t s = c.s;
  const int64_t m = p->m, n = p->n;
  const int k = p->k, l = c.pl.l;
  const int f_ek = p->factor_dtype == LORACT_BF16 ? EK_BF16 : EK_F32;
  void* Bmat = c.ws + c.pl.off_bmat;
  const void* Q;
  int q_ek, b_ek;
  if (c.pl.bf16_path) {
    // Q in fp32 (into the sketch buffer, free by the second round) for U = Q W_k, and its bf16
    // copy for the projection on the matrix cores
    bf16_t* Qb = ws_ptr<bf16_t>(c, c.pl.off_ub);
    LORACT_TRY(orthonormalise_mfma(c, (const float*)Y, (float*)tmp, Y, EK_F32, Qb));
    LORACT_TRY(project(c, Qb, EK_BF16, Bmat, EK_F32));
    Q = Y; q_ek = EK_F32; b_ek = EK_F32;
  } else {
    LORACT_TRY(orthonormalise(c, Y, tmp, Y, EK_F64));
    LORACT_TRY(project(c, Y, EK_F64, Bmat, EK_F64));
    Q = Y; q_ek = EK_F64; b_ek = EK_F64;
  }
  double* eigA = ws_ptr<double>(c, c.pl.off_eig);
  double* eigW = eigA + (size_t)l * l;
  double* Wk = eigW + ej_work_doubles(l);
  LORACT_TRY(launch_gemm_f64("truncate_bbt", s, Bmat, n, 1, b_ek, Bmat, n, 1, b_ek, nullptr, l, l, n, 1.0,
                             eigA, l, EK_F64, c.pl.bgram_splits, ws_ptr<double>(c, c.pl.off_dpart)));
  LORACT_TRY(launch_jacobi_eig(s, eigA, eigW, Wk, l, k, energy, k_out));
  // U = Q W_k (m x k),  V = W_k^T B (k x n)
  LORACT_TRY(launch_gemm_f64("truncate_qw", s, Q, l, 1, q_ek, Wk, k, 0, EK_F64, nullptr, m, k, l, 1.0,
                             U_dev, k, f_ek, 1, nullptr));
  return launch_gemm_f64("truncate_wtb", s, Wk, k, 0, EK_F64, Bmat, n, 0, b_ek, nullptr, k, n, l, 1.0,
                         V_dev, n, f_ek, 1, nullptr);
}

// Shared by loract_compress and loract_compress_adaptive (k_out != null: the rank is chosen from
// the singular values of the l x n factor, see loract.h).
static int compress_impl(const void* X_dev, const loract_params* p, const int32_t* idx_host,
                         void* U_dev, void* V_dev, void* ws_dev, size_t ws_bytes, void* stream,
                         int32_t* status_dev, double energy, int32_t* k_out) {
  Ctx c;
  hipStream_t s = (hipStream_t)stream;
  LORACT_TRY(check_common(X_dev, p, U_dev, V_dev, ws_dev, ws_bytes, false, &c, s, status_dev, k_out != nullptr));
  const int k = p->k, l = c.pl.l;
  IdxPack pack;
  memset(&pack, 0, sizeof(pack));
  if (idx_host) {
    for (int i = 0; i < l; ++i) {
      if (idx_host[i] < 0 || idx_host[i] >= p->m) return LORACT_ERR_INVALID_ARG;
      if (i > 0 && idx_host[i] <= idx_host[i - 1]) return LORACT_ERR_INVALID_ARG;
      pack.v[i] = idx_host[i];
    }
  } else {
    LORACT_TRY(sample_indices_host(p->m, l, p->seed, pack.v));
  }
  int32_t* idx_dev = ws_ptr<int32_t>(c, c.pl.off_idx);
  void* Y = c.ws + c.pl.off_a;
  void* tmp = c.ws + c.pl.off_b;
  if (sketch_takes_ids(c)) {
    LORACT_TRY(sketch(c, X_dev, p->ldx, nullptr, Y, &pack));   // Y = X X_S^T, ids in the arguments
  } else {
    LORACT_LAUNCH("store_indices", s, store_indices_kernel, dim3((l + 255) / 256), dim3(256), 0, pack,
                  l, idx_dev, status_dev);
    LORACT_TRY(sketch(c, X_dev, p->ldx, idx_dev, Y));          // Y = X X_S^T
  }
  LORACT_TRY(power_iterations(c, Y, tmp));                // t power rounds
  if (l == k && !k_out) return finish_factors(c, Y, tmp, U_dev, V_dev);   // U = orth(Y), V = U^T X
  return truncate_factors(c, Y, tmp, U_dev, V_dev, energy, k_out);  // l > k sampled rows, or adaptive rank
}

int loract_compress(const void* X_dev, const loract_params* p, const int32_t* idx_host,
                    void* U_dev, void* V_dev, void* ws_dev, size_t ws_bytes, void* stream,
                    int32_t* status_dev) {
  return compress_impl(X_dev, p, idx_host, U_dev, V_dev, ws_dev, ws_bytes, stream, status_dev, 1.0, nullptr);
}

int loract_compress_adaptive(const void* X_dev, const loract_params* p, const int32_t* idx_host,
                             double energy, void* U_dev, void* V_dev, int32_t* k_out_dev,
                             void* ws_dev, size_t ws_bytes, void* stream, int32_t* status_dev) {
  if (!k_out_dev || !(energy > 0.0 && energy <= 1.0)) return LORACT_ERR_INVALID_ARG;
  return compress_impl(X_dev, p, idx_host, U_dev, V_dev, ws_dev, ws_bytes, stream, status_dev, energy,
                       k_out_dev);
}

int loract_reconstruct(const void* U_dev, const void* V_dev, int64_t m, int64_t n, int32_t k,
                       int32_t factor_dtype, void* Xhat_dev, int64_t ldxh, int32_t out_dtype,
                       void* stream) {
  if (!U_dev || !V_dev || !Xhat_dev || m < 1 || n < 1 || k < 1 || ldxh < n)
    return LORACT_ERR_INVALID_ARG;
  if (!dtype_ok(factor_dtype) || !dtype_ok(out_dtype)) return LORACT_ERR_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  if (factor_dtype == LORACT_BF16 && out_dtype == LORACT_BF16 && k <= LORACT_MAX_RANK &&
      sb_aligned(U_dev, k) && sb_aligned(V_dev, n) && sb_aligned(Xhat_dev, ldxh)) {
    ReconArgs a;
    a.U = (const bf16_t*)U_dev; a.V = (const bf16_t*)V_dev; a.m = m; a.n = n; a.k = k;
    a.Xhat = (bf16_t*)Xhat_dev; a.ldxh = ldxh; a.row_tiles = 0;
    return launch_reconstruct_mfma(s, a);
  }
  if (factor_dtype == LORACT_BF16)
    return launch_gemm_bf16("reconstruct_generic", s, (const bf16_t*)U_dev, k, 1, (const bf16_t*)V_dev, n, 0,
                            nullptr, m, n, k, Xhat_dev, ldxh,
                            out_dtype == LORACT_BF16 ? EK_BF16 : EK_F32, 1, nullptr);
  return launch_gemm_f64("reconstruct_f64", s, U_dev, k, 1, EK_F32, V_dev, n, 0, EK_F32, nullptr, m,
                         n, k, 1.0, Xhat_dev, ldxh, out_dtype == LORACT_BF16 ? EK_BF16 : EK_F32, 1,
                         nullptr);
}

// Workspace of loract_lora_grad: G (m x r, fp32 or bf16), T (k x r, fp32), split partials.
struct LoraPlan {
  int t_splits;
  int rp;                 // r rounded up to 16
  int g_splits;           // K splits of dY B^T
  size_t off_g, off_t, off_dpart, off_gpart, off_gsplit, off_ppart, off_tsplit, total;
};
static int make_lora_plan(int64_t m, int64_t n, int32_t k, int64_t n_out, int32_t r, LoraPlan* lp) {
  if (m < 1 || n < 1 || k < 1 || n_out < 1 || r < 1 || r > 64) return LORACT_ERR_INVALID_ARG;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
  lp->t_splits = pick_splits(ceil_div64(k, 64), m, 64);
  lp->rp = (r + 15) / 16 * 16;
  lp->g_splits = sketch_splits_for(m, n_out, lp->rp);
  lp->off_g = take((size_t)m * lp->rp * 4);
  lp->off_t = take((size_t)k * r * 4);
  lp->off_dpart = take((size_t)lp->t_splits * k * r * 8);
  lp->off_gpart = take((size_t)lp->g_splits * m * lp->rp * 4);
  lp->off_gsplit = take((size_t)m * 2 * lp->rp * 2);
  lp->off_ppart = take(project_part_floats(m, 2 * lp->rp, k) * 4);
  lp->off_tsplit = take((size_t)k * 2 * lp->rp * 4);
  lp->total = off;
  return LORACT_OK;
}

int loract_lora_grad_workspace_bytes(int64_t m, int64_t n, int32_t k, int64_t n_out,
                                     int32_t r_lora, size_t* bytes) {
  if (!bytes) return LORACT_ERR_INVALID_ARG;
  LoraPlan lp;
  LORACT_TRY(make_lora_plan(m, n, k, n_out, r_lora, &lp));
  *bytes = lp.total;
  return LORACT_OK;
}

int loract_lora_grad(const void* U_dev, const void* V_dev, int64_t m, int64_t n, int32_t k,
                     int32_t factor_dtype, const void* dY_dev, int64_t n_out,
                     const void* Blora_dev, int32_t r_lora, int32_t grad_dtype, float scale,
                     float* dA_dev, void* ws_dev, size_t ws_bytes, void* stream) {
  if (!U_dev || !V_dev || !dY_dev || !Blora_dev || !dA_dev) return LORACT_ERR_INVALID_ARG;
  if (!dtype_ok(factor_dtype) || !dtype_ok(grad_dtype)) return LORACT_ERR_INVALID_ARG;
  LoraPlan lp;
  LORACT_TRY(make_lora_plan(m, n, k, n_out, r_lora, &lp));
  if (!ws_dev || ws_bytes < lp.total) return LORACT_ERR_WORKSPACE_TOO_SMALL;
  hipStream_t s = (hipStream_t)stream;
  char* ws = (char*)ws_dev;
  float* G = (float*)(ws + lp.off_g);
  float* T = (float*)(ws + lp.off_t);
  double* dpart = (double*)(ws + lp.off_dpart);
  const int f_ek = factor_dtype == LORACT_BF16 ? EK_BF16 : EK_F32;
  if (factor_dtype == LORACT_BF16 && grad_dtype == LORACT_BF16 && k <= LORACT_MAX_RANK &&
      n_out % 64 == 0 && sb_aligned(dY_dev, n_out) && sb_aligned(Blora_dev, n_out) &&
      sb_aligned(U_dev, k) && sb_aligned(V_dev, n)) {
    const int rp = lp.rp;
    // G = dY B_lora^T (m x rp), the one pass over dY, left as the bf16 pair [G_hi | G_lo]
    SketchArgs a{};
    a.X = (const bf16_t*)dY_dev; a.ldx = n_out; a.m = m; a.n = n_out;
    a.B = (const bf16_t*)Blora_dev; a.ldb = n_out; a.b_rows = nullptr; a.l = r_lora; a.kp = rp;
    a.Y = (float*)(ws + lp.off_g); a.part = (float*)(ws + lp.off_gpart); a.splits = lp.g_splits;
    a.k_per_split = 0; a.run_flag = nullptr;
    a.ids_in_args = 0; a.clear_status = nullptr;
    bf16_t* Gsplit = (bf16_t*)(ws + lp.off_gsplit);
    LORACT_TRY(launch_sketch_mfma(s, a, "lora_dyb", Gsplit));
    // [T_hi | T_lo] = U^T [G_hi | G_lo]  (k x 2rp)
    ProjectArgs pa;
    pa.Q = (const bf16_t*)U_dev; pa.ldq = k; pa.X = Gsplit; pa.ldx = 2 * rp; pa.m = m; pa.n = 2 * rp;
    pa.l = k; pa.V = ws + lp.off_tsplit; pa.out_ek = EK_F32; pa.part = (float*)(ws + lp.off_ppart);
    LORACT_TRY(launch_project_mfma(s, pa, "lora_utg", PJ_LORA_UTG));
    // dA = scale * V^T (T_hi + T_lo)
    return launch_lora_vtt(s, (const bf16_t*)V_dev, (const float*)(ws + lp.off_tsplit), (int)k, n,
                           (int)r_lora, rp, scale, dA_dev);
  }
  // G = dY B_lora^T  (m x r): the only pass over the large operand
  if (grad_dtype == LORACT_BF16)
    LORACT_TRY(launch_gemm_bf16("lora_dyb_generic", s, (const bf16_t*)dY_dev, n_out, 1,
                                (const bf16_t*)Blora_dev, n_out, 1, nullptr, m, r_lora, n_out, G,
                                r_lora, EK_F32, 1, nullptr));
  else
    LORACT_TRY(launch_gemm_f64("lora_dyb_f64", s, dY_dev, n_out, 1, EK_F32, Blora_dev, n_out, 1,
                               EK_F32, nullptr, m, r_lora, n_out, 1.0, G, r_lora, EK_F32, 1, nullptr));
  // T = U^T G  (k x r)
  LORACT_TRY(launch_gemm_f64("lora_utg_generic", s, U_dev, k, 0, f_ek, G, r_lora, 0, EK_F32, nullptr, k,
                             r_lora, m, 1.0, T, r_lora, EK_F32, lp.t_splits, dpart));
  // dA = V^T T * scale  (n x r)
  return launch_gemm_f64("lora_vtt_generic", s, V_dev, n, 0, f_ek, T, r_lora, 0, EK_F32, nullptr, n, r_lora,
                         k, (double)scale, dA_dev, r_lora, EK_F32, 1, nullptr);
}

size_t loract_static_scratch_bytes(void) { return (size_t)LORACT_STATIC_SCRATCH_BYTES; }

int loract_lora_grad_static(const void* U_dev, const void* V_dev, int64_t m, int64_t n, int32_t k,
                            int32_t factor_dtype, const void* dY_dev, int64_t n_out,
                            const void* Blora_dev, int32_t r_lora, int32_t grad_dtype, float scale,
                            float* dA_dev, void* stream) {
  LoraPlan lp;
  LORACT_TRY(make_lora_plan(m, n, k, n_out, r_lora, &lp));
  if (lp.total > (size_t)LORACT_STATIC_SCRATCH_BYTES) {
    g_host.last_hip_error = "loract_lora_grad_static: this shape needs " + std::to_string(lp.total) +
                            " bytes of scratch, the built-in buffer holds " +
                            std::to_string((size_t)LORACT_STATIC_SCRATCH_BYTES);
    return LORACT_ERR_WORKSPACE_TOO_SMALL;
  }
  void* ws = nullptr;
  LORACT_TRY(static_scratch_ptr(&ws));
  // the partial results every kernel of the gradient reads were written by an earlier kernel of
  // the same call, so nothing in the buffer has to start at zero
  return loract_lora_grad(U_dev, V_dev, m, n, k, factor_dtype, dY_dev, n_out, Blora_dev, r_lora,
                          grad_dtype, scale, dA_dev, ws, (size_t)LORACT_STATIC_SCRATCH_BYTES, stream);
}

int loract_gaussian_omega_t(void* omegaT_dev, int32_t l, int64_t n, int32_t dtype, uint64_t seed,
                            void* stream) {
  if (!omegaT_dev || l < 1 || n < 1 || !dtype_ok(dtype)) return LORACT_ERR_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  const int64_t count = (int64_t)l * n;
  int blocks = (int)std::min<int64_t>(ceil_div64(count, 256), 4096);
  LORACT_LAUNCH("gaussian", s, gaussian_kernel, dim3(blocks), dim3(256), 0, omegaT_dev,
                dtype == LORACT_BF16 ? EK_BF16 : EK_F32, count, seed);
  return LORACT_OK;
}

int loract_rsvd(const void* X_dev, const loract_params* p, const void* omegaT_dev, void* U_dev,
                void* V_dev, void* ws_dev, size_t ws_bytes, void* stream, int32_t* status_dev) {
  Ctx c;
  hipStream_t s = (hipStream_t)stream;
  LORACT_TRY(check_common(X_dev, p, U_dev, V_dev, ws_dev, ws_bytes, true, &c, s, status_dev));
  const int64_t m = p->m, n = p->n;
  const int k = p->k, l = c.pl.l;
  // clear the status word (no sampled rows on this path)
  IdxPack pack;
  memset(&pack, 0, sizeof(pack));
  LORACT_LAUNCH("store_indices", s, store_indices_kernel, dim3(1), dim3(256), 0, pack, 0,
                ws_ptr<int32_t>(c, c.pl.off_idx), status_dev);
  // Gaussian test matrix, stored transposed (l x n) in X's element type
  const void* omega = omegaT_dev;
  if (!omega) {
    void* om = c.ws + c.pl.off_omega;
    LORACT_TRY(loract_gaussian_omega_t(om, l, n, p->x_dtype, p->seed, stream));
    omega = om;
  }
  void* Y = c.ws + c.pl.off_a;
  void* tmp = c.ws + c.pl.off_b;
  if (c.pl.bf16_path) {
    LORACT_TRY(sketch(c, omega, n, nullptr, Y));                       // Y = X Omega
  } else {
    // fp32 input: the generic product reads Omega in its own element type
    LORACT_TRY(launch_gemm_f64("sketch_f64", s, X_dev, p->ldx, 1, EK_F32, omega, n, 1, EK_F32, nullptr,
                               m, l, n, 1.0, Y, l, EK_F64, 1, nullptr));
  }
  LORACT_TRY(power_iterations(c, Y, tmp));                             // t x [QR; Y = X (X^T Q)]
  if (l == k) return finish_factors(c, Y, tmp, U_dev, V_dev);          // no oversampling: U = Q, V = Q^T X

  return truncate_factors(c, Y, tmp, U_dev, V_dev);                   // oversampled: cut to rank k
}

static int prenorm_common(PrenormArgs* a, int64_t m, int64_t n, int32_t dtype) {
  if (m < 1 || n < 1 || !dtype_ok(dtype)) return LORACT_ERR_INVALID_ARG;
  if (a->ldx < n || a->ldo < n) return LORACT_ERR_INVALID_ARG;
  a->m = m; a->n = n;
  a->ek = dtype == LORACT_BF16 ? EK_BF16 : EK_F32;
  return LORACT_OK;
}

int loract_prenorm_forward(const void* X_dev, int64_t m, int64_t n, int64_t ldx, int32_t dtype,
                           const float* gamma_dev, float eps, void* A_dev, int64_t lda,
                           float* rms_dev, void* stream) {
  if (!X_dev || !gamma_dev || !A_dev || !rms_dev) return LORACT_ERR_INVALID_ARG;
  PrenormArgs a;
  a.X = X_dev; a.ldx = ldx; a.dA = nullptr; a.ldda = 0; a.gamma = gamma_dev; a.rms = rms_dev;
  a.out = A_dev; a.ldo = lda; a.eps = eps;
  LORACT_TRY(prenorm_common(&a, m, n, dtype));
  a.vec = dtype == LORACT_BF16 && n % 8 == 0 && sb_aligned(X_dev, ldx) && sb_aligned(A_dev, lda) &&
          ((uintptr_t)gamma_dev) % 16 == 0;
  LORACT_LAUNCH("prenorm_forward", (hipStream_t)stream, prenorm_forward_kernel,
                dim3((unsigned)ceil_div64(m, 4)), dim3(256), 0, a);
  return LORACT_OK;
}

int loract_prenorm_backward(const void* A_dev, int64_t m, int64_t n, int64_t lda, int32_t dtype,
                            const float* rms_dev, const float* gamma_dev, const void* dA_dev,
                            int64_t ldda, void* dX_dev, int64_t lddx, void* stream) {
  if (!A_dev || !rms_dev || !gamma_dev || !dA_dev || !dX_dev || ldda < n) return LORACT_ERR_INVALID_ARG;
  PrenormArgs a;
  a.X = A_dev; a.ldx = lda; a.dA = dA_dev; a.ldda = ldda; a.gamma = gamma_dev; a.rms = (float*)rms_dev;
  a.out = dX_dev; a.ldo = lddx; a.eps = 0.0f;
  LORACT_TRY(prenorm_common(&a, m, n, dtype));
  a.vec = dtype == LORACT_BF16 && n % 8 == 0 && sb_aligned(A_dev, lda) && sb_aligned(dA_dev, ldda) &&
          sb_aligned(dX_dev, lddx) && ((uintptr_t)gamma_dev) % 16 == 0;
  LORACT_LAUNCH("prenorm_backward", (hipStream_t)stream, prenorm_backward_kernel,
                dim3((unsigned)ceil_div64(m, 4)), dim3(256), 0, a);
  return LORACT_OK;
}

int loract_profile_begin(void) {
  std::lock_guard<std::mutex> lock(g_prof.mu);
  g_prof.recs.clear();
  g_prof.agg.clear();
  g_prof.order.clear();
  g_prof.on = true;
  return LORACT_OK;
}

int loract_profile_end(void) {
  g_prof.on = false;
  std::lock_guard<std::mutex> lock(g_prof.mu);
  for (auto& r : g_prof.recs) {
    hipError_t e = hipEventSynchronize(r.stop);
    if (e != hipSuccess) return hip_fail(e, "hipEventSynchronize");
    float ms = 0.0f;
    e = hipEventElapsedTime(&ms, r.start, r.stop);
    if (e != hipSuccess) return hip_fail(e, "hipEventElapsedTime");
    auto it = g_prof.agg.find(r.name);
    if (it == g_prof.agg.end()) {
      g_prof.agg[r.name] = std::make_pair((double)ms, (int64_t)1);
      g_prof.order.push_back(r.name);
    } else {
      it->second.first += ms;
      it->second.second += 1;
    }
    g_prof.pool.push_back(r.start);
    g_prof.pool.push_back(r.stop);
  }
  g_prof.recs.clear();
  return LORACT_OK;
}

int loract_profile_count(void) {
  std::lock_guard<std::mutex> lock(g_prof.mu);
  return (int)g_prof.order.size();
}

int loract_profile_get(int i, char* name_buf, int name_buf_len, double* total_ms,
                       int64_t* launches) {
  std::lock_guard<std::mutex> lock(g_prof.mu);
  if (i < 0 || i >= (int)g_prof.order.size() || !name_buf || name_buf_len < 1)
    return LORACT_ERR_INVALID_ARG;
  const std::string& nm = g_prof.order[i];
  strncpy(name_buf, nm.c_str(), (size_t)name_buf_len - 1);
  name_buf[name_buf_len - 1] = 0;
  auto& a = g_prof.agg[nm];
  if (total_ms) *total_ms = a.first;
  if (launches) *launches = a.second;
  return LORACT_OK;
}

}  // extern "C"
