/*
 * loract.h - C ABI of the LoRAct activation-compression library for AMD MI355X (gfx950).
 *
 * The library implements the data path of "LoRAct: low-rank activation compression"
 * (arXiv 2509.23472): the online compression of one saved activation matrix in the forward
 * pass (Section 3.1, Eqs. 2-3, by the sampling-based orthogonal decomposition of
 * Section 3.2, Algorithm 1) and the backward-side consumers of the factors (Section 3.1,
 * Eqs. 4-5), plus the randomized-SVD method the paper compares with (Section 3.2).
 *
 * Conventions shared by every entry point
 *   - Matrices are dense and row-major.  "dev" pointers are device (HBM) pointers owned by
 *     the caller; "host" pointers are ordinary host memory.  The library never allocates,
 *     frees or retains caller memory; scratch space is a caller-provided workspace.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All device
 *     work is enqueued on it in order; no entry point synchronises the device, except the
 *     loract_profile_* readers which wait for their own events.
 *   - Return value: LORACT_OK (0) or a negative loract_status.  Argument errors are detected
 *     on the host before anything is enqueued.  Numerical events on the device (a
 *     rank-deficient sketch) never abort; they are reported through the optional device
 *     status word.
 *   - Same inputs, parameters and seed give bit-identical outputs: all split reductions are
 *     combined in a fixed order, no floating-point atomics are used.
 *   - Element types: LORACT_BF16 is the 16-bit brain float (upper half of an IEEE binary32),
 *     LORACT_F32 is IEEE binary32.
 */
#ifndef LORACT_H
#define LORACT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  LORACT_OK = 0,
  LORACT_ERR_INVALID_ARG = -1,        /* null pointer, non-positive size, k out of range, ... */
  LORACT_ERR_WORKSPACE_TOO_SMALL = -2,
  LORACT_ERR_UNSUPPORTED = -3,        /* dtype combination, rank above LORACT_MAX_RANK, ... */
  LORACT_ERR_NOT_IMPLEMENTED = -4,
  LORACT_ERR_HIP = -5                 /* a HIP runtime call failed; see loract_last_hip_error */
} loract_status;

typedef enum { LORACT_F32 = 0, LORACT_BF16 = 1 } loract_dtype;

/* Largest number of sketch columns (k, or k + oversampling for RSVD) the kernels accept. */
#define LORACT_MAX_RANK 320
#define LORACT_STATIC_SCRATCH_BYTES (16u << 20)   /* scratch built into the library, see loract_lora_grad_static */

/* Bits of the device status word written by loract_compress / loract_rsvd. */
#define LORACT_STATUS_RANK_DEFICIENT 1   /* a direction of the sketch was numerically dependent on
                                            the others and was dropped: U has a zero column */
#define LORACT_STATUS_INTERNAL 2         /* a workgroup's bounded wait for another workgroup of the
                                            same launch ran out: the outputs are not valid */

/* Problem statement of Algorithm 1: A in R^{m x n}, expected rank k, iterations t. */
typedef struct {
  int64_t m;             /* rows of X (tokens) */
  int64_t n;             /* columns of X (hidden size) */
  int64_t ldx;           /* leading dimension of X in elements, >= n */
  int32_t k;             /* target rank, 1 <= k <= min(m, n) */
  int32_t l;             /* sketch columns, k <= l <= min(m, n, LORACT_MAX_RANK); 0 = k.
                            loract_compress: sampled rows (Algorithm 1 takes l = k; l > k is the
                            sample of Theorem 4.3).  loract_rsvd: k + oversampling.  With l > k the
                            l x n factor Q^T X is cut to its k leading singular triplets */
  int32_t t;             /* power iterations (the power rounds of Algorithm 1); 0 on the hot path */
  int32_t x_dtype;       /* loract_dtype of X */
  int32_t factor_dtype;  /* loract_dtype of U and V; F32 input requires F32 factors */
  uint64_t seed;         /* seed of the row sample (compress) or of the Gaussian test matrix (rsvd) */
} loract_params;

const char* loract_version(void);
const char* loract_strerror(int code);
/* Text of the most recent HIP error seen by this thread's calls ("" if none). Host. */
const char* loract_last_hip_error(void);

/*
 * Algorithm 1, row sampling: the l distinct row indices sampled uniformly without replacement from
 * [0, m), in ascending order.  Pure host function; this is the definition the device path
 * uses when no explicit indices are given: splitmix64 started at `seed` drives Floyd's subset
 * sampling (for i = m-l .. m-1: j = next() mod (i+1); take j, or i if j was already taken).
 * idx_host: out, l int32 values.  Errors: INVALID_ARG if l < 0, l > m, m > 2^31-1 or null.
 */
int loract_sample_indices(int64_t m, int32_t l, uint64_t seed, int32_t* idx_host);

/*
 * Bytes of device workspace loract_compress / loract_rsvd need for these parameters
 * (256-byte aligned base expected).  Host.  Errors as for the call itself.
 */
int loract_workspace_bytes(const loract_params* p, size_t* bytes);

/*
 * Forward pass, Section 3.1 Eqs. (2)-(3) by Algorithm 1 (Section 3.2):
 *   A_k = X[S, :] (k sampled rows), Y = X A_k^T, t x [Y = QR; Y = X (X^T Q)], Y = QR,
 *   U = Q (m x k, orthonormal columns), V = Q^T X (k x n).
 * With l > k sampled rows (Theorem 4.3) Q has l columns and the factors are those of the k
 * leading singular triplets of B = Q^T X: U = Q W_k, V = W_k^T B (W_k: k leading eigenvectors
 * of B B^T), still m x k and k x n with orthonormal U.
 * X_dev        in,  m x n (ld = ldx), dtype x_dtype.
 * idx_host     in,  l ascending distinct row ids in host memory, or NULL to derive them from
 *              p->seed with loract_sample_indices.  Read before the call returns.
 * U_dev, V_dev out, m x k and k x n, contiguous, dtype factor_dtype.
 * ws_dev       scratch of at least loract_workspace_bytes(p) bytes; contents undefined after.
 * status_dev   optional int32 in device memory; set to 0 or an OR of LORACT_STATUS_* bits.
 * If Y is rank deficient (X holds duplicate or all-zero rows and they were sampled) U V
 * remains the projection of X onto range(Y) to working accuracy and U stays finite: a
 * dependent direction is either replaced by an arbitrary orthonormal completion, or, when it
 * vanishes to within float32 resolution, dropped: then that column of U (and row of V) is
 * zero and the status bit is raised.
 */
int loract_compress(const void* X_dev, const loract_params* p, const int32_t* idx_host,
                    void* U_dev, void* V_dev, void* ws_dev, size_t ws_bytes,
                    void* stream, int32_t* status_dev);

/*
 * Algorithm 1 with the rank chosen from the data.  The paper fixes k by hand and leaves adaptive
 * rank selection to future work (Conclusion); the rule used here is the measure of Section 2: the
 * number of kept dimensions when `energy` (0 < energy <= 1, Section 2 uses 0.9) of the energy --
 * the sum of the singular values -- is retained.  It is evaluated inside the sketch: with Q an
 * orthonormal basis of the l-column sketch (l = p->l sampled rows, 0 = p->k) and s_1 >= ... >= s_l the
 * singular values of B = Q^T X, k_eff is the smallest count with s_1 + ... + s_k_eff >= energy *
 * (s_1 + ... + s_l), at most p->k, and the factors are the k_eff leading singular triplets of B as
 * in loract_compress with l > k.
 * U_dev, V_dev  out, m x p->k and p->k x n as for loract_compress: columns of U and rows of V from
 *               k_eff on are zero, so U V is the rank-k_eff product whatever slice the caller keeps.
 * k_out_dev     out, int32 in device memory: k_eff.
 * Workspace, indices, stream, status and errors as for loract_compress.
 */
int loract_compress_adaptive(const void* X_dev, const loract_params* p, const int32_t* idx_host,
                             double energy, void* U_dev, void* V_dev, int32_t* k_out_dev,
                             void* ws_dev, size_t ws_bytes, void* stream, int32_t* status_dev);

/*
 * Backward pass, Section 3.1 Eq. (4): Xhat = U V.
 * U_dev m x k, V_dev k x n (contiguous, dtype factor_dtype); Xhat_dev out, m x n with leading
 * dimension ldxh >= n, dtype out_dtype.  No workspace.
 */
int loract_reconstruct(const void* U_dev, const void* V_dev, int64_t m, int64_t n, int32_t k,
                       int32_t factor_dtype, void* Xhat_dev, int64_t ldxh, int32_t out_dtype,
                       void* stream);

/*
 * Backward pass, Section 3.1 Eqs. (4)-(5) specialised to a LoRA down-projection whose input
 * was compressed: dA = Xhat^T (dY B_lora^T) * scale  (n x r_lora, float32), evaluated as
 * V^T (U^T (dY B_lora^T)) without forming Xhat.
 * dY_dev m x n_out and Blora_dev r_lora x n_out have dtype grad_dtype (contiguous);
 * 1 <= r_lora <= 64.  Workspace: loract_lora_grad_workspace_bytes.
 */
int loract_lora_grad_workspace_bytes(int64_t m, int64_t n, int32_t k, int64_t n_out,
                                     int32_t r_lora, size_t* bytes);
int loract_lora_grad(const void* U_dev, const void* V_dev, int64_t m, int64_t n, int32_t k,
                     int32_t factor_dtype, const void* dY_dev, int64_t n_out,
                     const void* Blora_dev, int32_t r_lora, int32_t grad_dtype, float scale,
                     float* dA_dev, void* ws_dev, size_t ws_bytes, void* stream);

/*
 * loract_lora_grad for callers that cannot allocate or hand over device memory: code under HIP
 * graph capture, tight serving or training loops, harnesses that forbid hipMalloc.  Same
 * arguments, kernels and result (bit for bit) as loract_lora_grad, without the workspace: the
 * scratch is a buffer of LORACT_STATIC_SCRATCH_BYTES (16 MiB) built into the library's device
 * image, one copy per GPU, held until the process ends.  The call allocates nothing: no hipMalloc,
 * hipFree or allocating library routine is reached.
 * Limit: shapes whose loract_lora_grad_workspace_bytes exceeds LORACT_STATIC_SCRATCH_BYTES are
 * rejected with LORACT_ERR_WORKSPACE_TOO_SMALL (loract_last_hip_error names both sizes) before
 * anything is enqueued; 8192 x 4096, rank 128, LoRA rank 16 needs 8 MiB.
 * All calls on one GPU share that GPU's buffer, which keeps the previous call's contents (no kernel
 * of the gradient relies on them): calls that overlap on one GPU -- from two streams or two
 * threads -- race; serialise them on one stream.  The first call on a device looks up the
 * buffer's address (no allocation, but not a stream operation: make one call before capturing).
 * loract_static_scratch_bytes returns the built-in size.
 */
size_t loract_static_scratch_bytes(void);
int loract_lora_grad_static(const void* U_dev, const void* V_dev, int64_t m, int64_t n, int32_t k,
                            int32_t factor_dtype, const void* dY_dev, int64_t n_out,
                            const void* Blora_dev, int32_t r_lora, int32_t grad_dtype, float scale,
                            float* dA_dev, void* stream);

/*
 * The comparator of Section 3.2: randomized SVD with a Gaussian test matrix Omega (n x l),
 * the same procedure as Algorithm 1 with Omega in place of the sampled rows: Y = X Omega,
 * t x [QR; Y = X (X^T Q)], QR, B = Q^T X (l x n); for l > k the result is truncated to the k leading singular triplets
 * of B, so that U (m x k) and V (k x n) have the same shapes as loract_compress returns.
 * omegaT_dev   optional, Omega stored transposed (l x n, contiguous, dtype x_dtype); NULL =
 *              generate it on the device from p->seed (see loract_gaussian_omega_t).
 */
int loract_rsvd(const void* X_dev, const loract_params* p, const void* omegaT_dev,
                void* U_dev, void* V_dev, void* ws_dev, size_t ws_bytes,
                void* stream, int32_t* status_dev);

/*
 * Fills omegaT_dev (l x n, dtype) with the counter-based standard normal deviates the
 * comparator uses: element e = j*n + c takes h = the (e+1)-th splitmix64 output of `seed`,
 * u1 = (high32(h) + 1) / 2^32, u2 = low32(h) / 2^32, value sqrt(-2 ln u1) cos(2 pi u2).
 */
int loract_gaussian_omega_t(void* omegaT_dev, int32_t l, int64_t n, int32_t dtype,
                            uint64_t seed, void* stream);

/*
 * Pre-norm unit, Section 3.3.  The activation that is stored (and handed to loract_compress) is
 * the OUTPUT of the RMS normalisation, A = Norm(X) = X / RMS(X) * gamma (Eqs. 6-7), shared by
 * Norm and the sub-layer; only the RMS vector (m floats) is kept beside the factors.
 *
 * forward:  rms_i = sqrt(mean_j X_ij^2 + eps), A_ij = X_ij / rms_i * gamma_j.
 *   X_dev m x n (ld ldx), A_dev m x n out (ld lda), both of dtype; gamma_dev n floats;
 *   rms_dev m floats out.
 * backward (Eqs. 8-10): from the reconstructed A (= U V), the stored RMS vector and dA = dL/dA:
 *   Xbar = A / gamma, dXbar = dA * gamma,
 *   dX_ij = (dXbar_ij - Xbar_ij * mean_j(dXbar_ij Xbar_ij)) / rms_i.
 *   A_dev, dA_dev, dX_dev m x n of dtype (leading dimensions lda, ldda, lddx); gamma must be
 *   nonzero.  No workspace; enqueued on `stream`.
 */
int loract_prenorm_forward(const void* X_dev, int64_t m, int64_t n, int64_t ldx, int32_t dtype,
                           const float* gamma_dev, float eps, void* A_dev, int64_t lda,
                           float* rms_dev, void* stream);
int loract_prenorm_backward(const void* A_dev, int64_t m, int64_t n, int64_t lda, int32_t dtype,
                            const float* rms_dev, const float* gamma_dev, const void* dA_dev,
                            int64_t ldda, void* dX_dev, int64_t lddx, void* stream);

/*
 * Per-kernel timing with HIP events on the stream the kernels are launched on.
 * begin: start bracketing every kernel launch of this library with event records.
 * end:   stop, wait for the recorded events, and aggregate by kernel name.
 * count/get: read the aggregate (name, total milliseconds, number of launches).
 * Recording adds two event records per launch; leave it off when measuring end-to-end time.
 */
int loract_profile_begin(void);
int loract_profile_end(void);
int loract_profile_count(void);
int loract_profile_get(int i, char* name_buf, int name_buf_len, double* total_ms,
                       int64_t* launches);

#ifdef __cplusplus
}
#endif
#endif /* LORACT_H */
