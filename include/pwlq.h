/*
 * pwlq.h - C ABI of libpwlq: optimal-breakpoint search and quantizer of
 * Post-Training Piecewise Linear Quantization (Fang et al.) on one MI355X.
 *
 * Conventions for every call
 *   - Weight tensors are contiguous, row-major [C, K] binary32 in DEVICE
 *     memory; a conv weight [Cout, Cin, kh, kw] is passed with K = Cin*kh*kw.
 *     "Per channel" means per output channel (Section 2, Section 5).
 *   - A group is one row (PWLQ_PER_CHANNEL) or the whole tensor
 *     (PWLQ_PER_TENSOR, the paper's "per-layer", Section 5.2).
 *   - All array arguments except tensor-descriptor tables are DEVICE pointers
 *     owned by the caller.  The library allocates nothing; scratch comes from
 *     the caller's workspace.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL is the
 *     default stream) and the call returns without waiting for it.  Tensor
 *     descriptor tables are HOST arrays and are consumed before the call
 *     returns.
 *   - Stream capture: the calls only launch kernels (a list call writes its
 *     tensor table into the workspace through kernel arguments) and can be
 *     recorded into a HIP graph and replayed (same pointers, new contents).
 *     Exception: a list call whose table exceeds 63 KB (about 500 tensors)
 *     copies it from host memory instead, waits for that copy (and so for the
 *     work queued on `stream` before it) and returns PWLQ_EINVAL on a
 *     capturing stream.
 *   - Return value: a pwlq_status; pwlq_last_error() describes a failure.
 *     PWLQ_EINVAL, PWLQ_ENULL and PWLQ_EWORKSPACE are found before anything is
 *     launched: nothing was enqueued and no output is written.  PWLQ_EHIP
 *     reports a failure of the HIP runtime itself (a launch or copy it
 *     refused); kernels of the same call launched before it may already be
 *     queued, so the workspace and the outputs are then undefined.
 *   - Valid ranges: 2 <= bits <= 8, 1 <= n_cand <= 65535, C >= 1, K >= 1,
 *     at most 2^31-1 elements per group's tile set and per call 2^31-1 tiles.
 *   - A group whose absmax is NaN or infinite gets k_star = -1 and NaN in
 *     p_star and mse; quantizing such a group is unspecified.  Groups whose
 *     absmax is below 2^-100 or above 2^100 are outside the tested domain.
 */
#ifndef PWLQ_H
#define PWLQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PWLQ_OK = 0,
    PWLQ_EINVAL = 1,     /* argument out of range                     */
    PWLQ_ENULL = 2,      /* a required pointer is NULL                */
    PWLQ_EWORKSPACE = 3, /* workspace missing, misaligned or too small */
    PWLQ_EHIP = 4        /* a HIP runtime call failed                 */
} pwlq_status;

typedef enum { PWLQ_PER_CHANNEL = 0, PWLQ_PER_TENSOR = 1 } pwlq_mode;

/* One tensor of a model-level call.  w: device [C,K].  group_offset: index of
 * this tensor's first group in the per-group arrays.  elem_offset: index of
 * this tensor's first element in the per-element output arrays. */
typedef struct {
    const float *w;
    int64_t C, K;
    int64_t group_offset;
    int64_t elem_offset;
} pwlq_tensor_desc;

/*
 * Breakpoint search: Eq.7 (Section 3.3) solved on the group's own values.
 * For each group, m = max|w| and, for k = 1..n_cand, p_k = m*(k/n_cand); the
 * squared error of the b-bit piecewise quantizer of Eq.3 (Section 3.2: centre
 * [-p,p] and tails +-(p,m], each piece a (b-1)-bit uniform quantizer of Eq.1
 * with 2^(b-1) levels) is summed over the group, and the smallest k attaining
 * the minimum is returned.
 *
 * Outputs, device arrays of G entries (G = C per channel, 1 per tensor):
 *   p_star  the chosen breakpoint p_{k*}
 *   m_out   the group's absmax
 *   k_star  1-based index of the chosen candidate
 *   mse     SSE[k*] / (elements in the group), accumulated in binary64
 * workspace: device memory, 256-byte aligned, at least
 * pwlq_search_workspace_bytes(...) bytes; contents are scratch.
 */
size_t pwlq_search_workspace_bytes(int64_t C, int64_t K, int bits, int n_cand, int mode);

int pwlq_search(const float *w, int64_t C, int64_t K, int bits, int n_cand, int mode,
                float *p_star, float *m_out, int32_t *k_star, double *mse,
                void *workspace, size_t workspace_bytes, void *stream);

/*
 * pwlq_search for callers that cannot allocate device memory (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): the
 * same kernels, arguments and outputs as pwlq_search, with the scratch taken
 * from a buffer of PWLQ_STATIC_SCRATCH_BYTES that is part of the library's
 * device image (one copy per GPU, held until the process ends) instead of a
 * caller's workspace.  The call allocates and frees nothing on the device and
 * calls no allocating library routine.
 *   - A search whose pwlq_search_workspace_bytes(C, K, bits, n_cand, mode)
 *     exceeds PWLQ_STATIC_SCRATCH_BYTES returns PWLQ_EWORKSPACE and enqueues
 *     nothing (32 MiB holds, e.g., 3000 channels of 1000 weights with 1000
 *     candidates, or one group of 7 million weights with 100).
 *   - The buffer belongs to the device that is current at the call, which must
 *     be the device of `stream`.  Its address is looked up on the first call
 *     made on a device; make that call outside stream capture.
 *   - Every call on a GPU shares that GPU's buffer, which keeps the previous
 *     call's contents; the kernels read nothing from it that the same call has
 *     not written, so nothing is cleared.  Two calls that overlap in time on
 *     one GPU (different streams, or graphs replayed concurrently) race on it:
 *     the caller serialises them.
 */
#define PWLQ_STATIC_SCRATCH_BYTES (32u << 20)

int pwlq_search_static(const float *w, int64_t C, int64_t K, int bits, int n_cand, int mode,
                       float *p_star, float *m_out, int32_t *k_star, double *mse, void *stream);

/*
 * The same search with the same outputs, computed with less work: for tiles
 * long enough to pay for it, a candidate's squared error is obtained from
 * cumulative counts and sums of the magnitudes (2^b - 1 look-ups per
 * candidate, independent of the group's length) instead of a pass over the
 * group; the candidates this filter cannot tell apart are then re-evaluated
 * exactly as in pwlq_search, so k_star, p_star and mse follow the same
 * definition (Eq.7 on the group's own values).  Arguments and workspace size
 * as for pwlq_search / pwlq_search_list.
 */
int pwlq_search_fast(const float *w, int64_t C, int64_t K, int bits, int n_cand, int mode,
                     float *p_star, float *m_out, int32_t *k_star, double *mse,
                     void *workspace, size_t workspace_bytes, void *stream);

int pwlq_search_fast_list(const pwlq_tensor_desc *desc, int n_tensors, int bits, int n_cand,
                          int mode, float *p_star, float *m_out, int32_t *k_star, double *mse,
                          void *workspace, size_t workspace_bytes, void *stream);

/*
 * Quantizer: Eq.3 with given (m, p) per group.  Device outputs of C*K entries:
 *   codes  b-bit sign-magnitude in one byte: bit b-1 is the sign, bits 0..b-2
 *          the piece's code 0..2^(b-1)-1 (Section 3.2: b bits including sign)
 *   flags  0 = centre region, 1 = tail region (the extra stored bit of
 *          Section 4)
 *   w_hat  sign * (step*code + offset) in binary32; the top code of a piece
 *          decodes to the piece's end point (p or m) exactly; zero is +0
 * Values with |w| > m are clamped (Eq.1) to the top tail code.
 */
int pwlq_quantize(const float *w, int64_t C, int64_t K, int bits, int mode,
                  const float *p_star, const float *m, uint8_t *codes, uint8_t *flags,
                  float *w_hat, void *stream);

/*
 * Model-level variants: every tensor of `desc` (host array of n_tensors
 * entries) in one set of launches.  Per-group arrays are indexed by
 * group_offset (+ row, per channel); per-element arrays by elem_offset + the
 * element's row-major index.  The caller chooses offsets so that tensors do
 * not overlap.  Semantics per tensor are those of pwlq_search / pwlq_quantize.
 */
size_t pwlq_search_list_workspace_bytes(const pwlq_tensor_desc *desc, int n_tensors,
                                        int bits, int n_cand, int mode);

int pwlq_search_list(const pwlq_tensor_desc *desc, int n_tensors, int bits, int n_cand,
                     int mode, float *p_star, float *m_out, int32_t *k_star, double *mse,
                     void *workspace, size_t workspace_bytes, void *stream);

size_t pwlq_quantize_list_workspace_bytes(const pwlq_tensor_desc *desc, int n_tensors,
                                          int bits, int mode);

int pwlq_quantize_list(const pwlq_tensor_desc *desc, int n_tensors, int bits, int mode,
                       const float *p_star, const float *m, uint8_t *codes, uint8_t *flags,
                       float *w_hat, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Quantizer with bit-packed outputs: the storage format Section 4 argues for
 * (b bits per weight plus one region bit).  Same arithmetic as pwlq_quantize;
 * only the layout of codes and flags differs:
 *   packed_codes  one little-endian bit stream per tensor: the b-bit code of
 *                 row-major element i occupies stream bits [i*b, (i+1)*b),
 *                 where stream bit j is bit (j mod 8) of byte (j div 8);
 *                 pwlq_packed_code_bytes(C*K, bits) = ceil(C*K*b/8) bytes
 *   packed_flags  region flag of element i in stream bit i;
 *                 pwlq_packed_flag_bytes(C*K) = ceil(C*K/8) bytes
 *   w_hat         as in pwlq_quantize, or NULL to skip it
 * Unused bits of a stream's last byte are written as 0.  In the list variant
 * tensor t's streams start at packed_codes + code_byte_offset[t] and
 * packed_flags + flag_byte_offset[t] (host arrays of n_tensors entries chosen
 * by the caller so that streams do not overlap); w_hat, if given, is indexed by
 * the descriptors' elem_offset.  Workspace: as pwlq_quantize_list.
 */
size_t pwlq_packed_code_bytes(int64_t count, int bits);
size_t pwlq_packed_flag_bytes(int64_t count);

int pwlq_quantize_packed(const float *w, int64_t C, int64_t K, int bits, int mode,
                         const float *p_star, const float *m, uint8_t *packed_codes,
                         uint8_t *packed_flags, float *w_hat, void *stream);

int pwlq_quantize_packed_list(const pwlq_tensor_desc *desc, int n_tensors, int bits, int mode,
                              const float *p_star, const float *m, uint8_t *packed_codes,
                              const int64_t *code_byte_offset, uint8_t *packed_flags,
                              const int64_t *flag_byte_offset, float *w_hat, void *workspace,
                              size_t workspace_bytes, void *stream);

/*
 * The paper's own breakpoint selectors (Section 3.3, Section 5.1): the group is
 * assumed to follow a zero-mean Gaussian or Laplacian restricted to [-m, m],
 * m = max|w|, and p minimises the expected error of Eq.6 over (0, m/2), i.e.
 * solves Eq.11.  The scale is estimated about zero from the group itself
 * (sigma^2 = mean w^2, beta = mean |w|), in binary64.
 *   PWLQ_SELECT_GAUSS_FIT      Section 5.1's logarithmic fit for a normalized
 *                              Gaussian, with breakpoint and range in units of
 *                              sigma: p = sigma ln(0.8614 m/sigma + 0.6079)
 *   PWLQ_SELECT_GAUSS_SOLVE    Eq.11 with the truncated Gaussian's F and f
 *   PWLQ_SELECT_LAPLACE_SOLVE  Eq.11 with the truncated Laplacian's F and f
 * Outputs, device arrays of G entries: p_out (the solution rounded to
 * binary32) and m_out (absmax).  An all-zero group gets p = 0; a group whose
 * absmax is NaN or infinite gets p = NaN.  Workspace: device, 256-byte aligned,
 * at least pwlq_select[_list]_workspace_bytes(...) bytes.
 */
typedef enum {
    PWLQ_SELECT_GAUSS_FIT = 0,
    PWLQ_SELECT_GAUSS_SOLVE = 1,
    PWLQ_SELECT_LAPLACE_SOLVE = 2
} pwlq_selector;

size_t pwlq_select_workspace_bytes(int64_t C, int64_t K, int mode);
size_t pwlq_select_list_workspace_bytes(const pwlq_tensor_desc *desc, int n_tensors, int mode);

int pwlq_select_analytic(const float *w, int64_t C, int64_t K, int mode, int selector,
                         float *p_out, float *m_out, void *workspace, size_t workspace_bytes,
                         void *stream);

int pwlq_select_analytic_list(const pwlq_tensor_desc *desc, int n_tensors, int mode, int selector,
                              float *p_out, float *m_out, void *workspace,
                              size_t workspace_bytes, void *stream);

/*
 * Mean squared quantization error of Eq.3 at a given (m, p) per group (the
 * quantity Eq.7 minimises, for any breakpoint, not only a grid point): codes
 * decided in binary32 exactly as pwlq_quantize decides them, error
 * step*code + offset - |w| and its sum in binary64, divided by the number of
 * elements in the group.  p and m are device arrays of G entries indexed like
 * the search outputs; mse is a device array of G binary64 values.  Workspace:
 * device, 256-byte aligned, at least pwlq_mse[_list]_workspace_bytes(...) bytes.
 */
size_t pwlq_mse_workspace_bytes(int64_t C, int64_t K, int mode);
size_t pwlq_mse_list_workspace_bytes(const pwlq_tensor_desc *desc, int n_tensors, int mode);

int pwlq_mse(const float *w, int64_t C, int64_t K, int bits, int mode, const float *p,
             const float *m, double *mse, void *workspace, size_t workspace_bytes, void *stream);

int pwlq_mse_list(const pwlq_tensor_desc *desc, int n_tensors, int bits, int mode, const float *p,
                  const float *m, double *mse, void *workspace, size_t workspace_bytes,
                  void *stream);

/*
 * Consumer of the packed format: Y = X_hat W_hat^T on integer arithmetic
 * (Section 4).  Activations are uniformly quantized 8-bit values (Eq.1) with
 * one step and one offset for the call, X_hat = s_x * xq + z_x, xq int8 [M, K]
 * row-major.  Weights [N, K] are per-output-channel PWLQ weights in the packed
 * format of pwlq_quantize_packed (one tensor: element n*K + k of the streams),
 * with p and m the N per-channel parameters they were quantized with.  For
 * every output the three integer sums of Section 4 are formed on the int8
 * matrix cores,
 *     A1 = <xq, w_q>_R1,  A2 = <xq, w_q>_R2,  A3 = <xq, sigma>_R2
 * (w_q the signed code, sigma the sign of a tail weight, which the offset p
 * carries), and combined in binary32:
 *     y = s_x (s1 A1 + s2 A2 + p A3) + z_x (s1 sum_R1 w_q + s2 sum_R2 w_q + p sum_R2 sigma)
 * with s1 = p/L, s2 = (m - p)/L, L = 2^(bits-1) - 1: the constants C2..C6 of
 * Section 4.
 *   y    device [M, N] binary32, row-major
 *   acc  device [3, M, N] int32 receiving A1, A2, A3, or NULL
 * With acc NULL the library may form A1 + L A3 as one integer sum (p = s1 L, so
 * s1 A1 + p A3 = s1 (A1 + L A3); L sigma is an int8 like any code) and issue two
 * matrix products per weight instead of three; y then differs from the
 * three-sum form by binary32 rounding only.
 * Requirements: K a multiple of 16; xq and packed_codes 16-byte aligned,
 * packed_flags 2-byte aligned; K * 128 * L below 2^31.  Workspace: device,
 * 256-byte aligned, pwlq_linear_workspace_bytes(N) bytes.
 */
size_t pwlq_linear_workspace_bytes(int64_t N);

int pwlq_linear_i8(const int8_t *xq, int64_t M, int64_t K, float s_x, float z_x,
                   const uint8_t *packed_codes, const uint8_t *packed_flags, int64_t N, int bits,
                   const float *p, const float *m, float *y, int32_t *acc, void *workspace,
                   size_t workspace_bytes, void *stream);

/* Text of the calling thread's last non-OK status ("" if none).  The storage
 * is thread-local and owned by the library. */
const char *pwlq_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PWLQ_H */
