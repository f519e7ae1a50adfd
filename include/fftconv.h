/*
 * fftconv.h -- C ABI of the MI355X (gfx950) long FFT-convolution library.
 *
 * The operation (paper Section 2.1, Eq. 1; problem statement of Algorithm 1):
 * for every batch row b and channel h, independently,
 *
 *     y[b,h,:] = iFFT( FFT(zero-pad(u[b,h,:])) . k_f[h,:] )[0:N],
 *     k_f[h,:] = FFT(zero-pad(k[h,:])),
 *
 * with transforms of length fft_size.  The result is the circular convolution
 * of u and k modulo fft_size, truncated to N outputs; it equals the causal
 * convolution sum_{j<=i} u[j] k[i-j] whenever N + Nk - 1 <= fft_size.  k is
 * shared over the batch, so k_f is computed once per filter and reused
 * (Section 1).  The transforms are evaluated as chains of small DFT-matrix
 * products with twiddle scaling in between (order-p decomposition, Section
 * 2.1 and Algorithms 1, 3, 4); which factorisation is used is the plan's
 * business and never visible in the results.
 *
 * Conventions
 *  - Every pointer named u, k, k_f, y, workspace is DEVICE memory on the
 *    device that was current when the plan was created; the caller owns and
 *    frees it.  block_keep is HOST memory.
 *  - u and y are contiguous row-major (B, H, N) in the plan's I/O dtype;
 *    k is contiguous row-major (H, Nk) fp32.  u, y, the gates, k_f and the
 *    workspace must start on a 16-byte boundary (any device allocation does);
 *    k and dk on a 4-byte one.
 *  - k_f is an opaque buffer of fftconv_kf_bytes() bytes: spectrum in the
 *    plan's internal (permuted) order, pre-scaled by 1/fft_size.  It is only
 *    valid with the plan that produced it (or a plan created with identical
 *    arguments).
 *  - All *_filter_fft* and *_forward* calls are asynchronous on `stream`
 *    (a hipStream_t passed as void*, NULL = the default stream).  They do not
 *    allocate and do not synchronise, with one exception: the calls that take
 *    a mask or pattern in HOST memory (fftconv_filter_fft_sparse,
 *    fftconv_filter_fft_sparse_digits) copy it to the device from pageable
 *    memory, for which the runtime may make the calling thread wait until
 *    earlier work on `stream` has finished.
 *  - A plan is const in every call after its creation as far as its meaning
 *    goes, but the filter transforms use device scratch that the plan owns:
 *    calls of the *_filter_fft* family on ONE plan must not overlap (different
 *    streams or threads); forward and backward calls may.
 *  - Every call returns FFTCONV_OK (0) or a negative error code; on error no
 *    kernel has been launched by that call.  fftconv_last_error() returns a
 *    thread-local description of the most recent failure on this thread.
 *  - Arithmetic: 16-bit I/O plans multiply bf16/fp16 operands on the matrix
 *    cores with fp32 accumulation; fp32 I/O plans compute in fp32.  All
 *    16-bit roundings are round-to-nearest-even.
 */
#ifndef FFTCONV_H
#define FFTCONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fftconv_plan fftconv_plan; /* opaque */

enum { FFTCONV_F32 = 0, FFTCONV_F16 = 1, FFTCONV_BF16 = 2 }; /* I/O dtype of u and y */

enum {
    FFTCONV_OK = 0,
    FFTCONV_EINVAL = -1,       /* bad argument (size, NULL pointer, mismatch with the plan) */
    FFTCONV_EUNSUPPORTED = -2, /* valid request this build has no kernel for */
    FFTCONV_EHIP = -3,         /* a HIP runtime call failed */
    FFTCONV_ENOMEM = -4,       /* host or device allocation failed */
    FFTCONV_ENODEV = -5        /* no usable GPU */
};

/* Create a plan for sequences of length N, transform length fft_size, H
 * channels and the given I/O dtype (Section 3.1; the paper's range of
 * transform lengths, 256 .. 4M, Section 1).
 *   N >= 1; fft_size a power of two in [256, 2^22]; N <= fft_size; H >= 1.
 * Builds the DFT matrices and twiddle tables in fp64 on the host, uploads
 * them, chooses the factorisation and allocates the plan's private scratch.
 * Arguments are validated before any device is touched. */
int fftconv_plan_create(fftconv_plan **out, int64_t N, int64_t fft_size, int64_t H, int dtype);

/* As fftconv_plan_create, with the kernel family chosen by the caller instead of by the cost model:
 * path is one of the names fftconv_plan_path returns ("fused3", "small", "multipass", "staged"), or NULL /
 * "" for the model's choice.  Fails with FFTCONV_EUNSUPPORTED when that family has no kernel for the
 * shape.  Where several families can run a shape (16-bit causal shapes: "fused3" everywhere it exists,
 * "small" up to fft_size 4096, "multipass" from 8192), fftconv_plan_create evaluates Eq. 2 of Section 3.2
 * (fftconv_cost_model with the FFTCONV_MACHINE_MI355X constants) on each family's own factorisation --
 * matrix-unit rate for the families that multiply on the matrix cores, general arithmetic rate for the
 * vector-ALU family, one trip through HBM for every step that is a kernel of its own -- and takes the
 * cheapest. */
int fftconv_plan_create_path(fftconv_plan **out, int64_t N, int64_t fft_size, int64_t H, int dtype, const char *path);

/* Free the plan and everything it owns.  NULL is accepted. */
int fftconv_plan_destroy(fftconv_plan *plan);

/* Bytes of the opaque k_f buffer for the plan's H channels. */
size_t fftconv_kf_bytes(const fftconv_plan *plan);

/* Bytes of caller-provided workspace fftconv_forward* needs for batch size B
 * (0 when the whole transform is fused on chip). */
size_t fftconv_workspace_bytes(const fftconv_plan *plan, int64_t B);

/* k_f = FFT(zero-pad(k)) / fft_size in the plan's order (Section 1: the
 * filter transform is computed once and reused over the batch).
 *   k: device, (H, Nk) fp32, 1 <= Nk <= fft_size; taps t >= Nk are zero.
 * The transform runs on the device: in fp32 for plans whose k_f is stored as 16-bit constants (16-bit I/O
 * from fft_size 256 up with N <= fft_size / 2 and N a multiple of 8, and every 16-bit plan from 16384 up), in
 * fp64 otherwise.  Asynchronous on `stream`; uses scratch memory owned by the plan, so calls on one plan must
 * not overlap. */
int fftconv_filter_fft(const fftconv_plan *plan, const float *k, int64_t Nk, void *k_f, void *stream);

/* y = conv(u, k) as defined at the top (Algorithm 1 / 3 / 4 depending on
 * fft_size).  H and N must equal the plan's; B >= 0 is free.  y must not
 * alias u.  workspace: at least fftconv_workspace_bytes(plan, B) bytes, may
 * be NULL when that is 0. */
int fftconv_forward(const fftconv_plan *plan, const void *u, const void *k_f, void *y,
                    int64_t B, int64_t H, int64_t N, void *workspace, void *stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): fftconv_forward with the workspace taken from a fixed array inside
 * the library instead of from the caller.  The array holds FFTCONV_STATIC_WORKSPACE_BYTES bytes on every
 * GPU the library runs on, for as long as the process lives.  Same arguments, result and kernels as
 * fftconv_forward; the call allocates and frees nothing (no hipMalloc, hipFree or allocating library
 * routine), it only launches the plan's kernels on `stream`.
 *   Fails with FFTCONV_EINVAL, before anything is launched, when fftconv_workspace_bytes(plan, B)
 *   exceeds FFTCONV_STATIC_WORKSPACE_BYTES (plans that need no workspace always fit).
 *   All calls on one GPU share that GPU's array, which keeps the previous call's contents; every kernel
 *   writes what it later reads, so nothing has to be cleared between calls.  Calls that overlap on one
 *   GPU (different streams or threads) race on the array: serialise them. */
#define FFTCONV_STATIC_WORKSPACE_BYTES ((size_t)64 << 20)
int fftconv_forward_static(const fftconv_plan *plan, const void *u, const void *k_f, void *y,
                           int64_t B, int64_t H, int64_t N, void *stream);

/* Partial convolution (Section 3.3): the filter is zero for taps t >= Nk.
 * Same result as fftconv_forward on that k_f; the plan may skip the parts of the decomposition that a
 * short filter leaves unused: plans with 16-bit I/O, causal shapes (N <= fft_size / 2, N a multiple of 8)
 * and fft_size >= 16384 run filters of Nk <= 2049 taps as overlapping 8192-point segments (the outer
 * factors of the decomposition are never executed).  That route needs the second, 8192-point spectrum
 * which fftconv_filter_fft(plan, k, Nk, ...) stores behind the dense one when called with this same Nk,
 * together with a tag naming the Nk.  Any other k_f of the plan (built for another Nk -- for instance
 * from the full-length filter with its tail zeroed --, masked, or adjoint) carries another tag, and the
 * call then runs the plan's dense kernels on it: the choice is made on the device by the kernels
 * themselves (both routes are launched, the one whose tag test fails returns at once), so the result is
 * always the dense result and nothing synchronises with the host. */
int fftconv_forward_partial(const fftconv_plan *plan, const void *u, const void *k_f, void *y,
                            int64_t B, int64_t H, int64_t N, int64_t Nk, void *workspace, void *stream);

/* Frequency-sparse filter (Section 3.3, Appendix A.4): as fftconv_filter_fft,
 * then every frequency bin f whose block is dropped is set to zero.
 *   block_keep: host, n_blocks bytes, 1 = keep; n_blocks a power of two that
 *   divides fft_size; block j holds the natural-order frequencies
 *   f in [j * fft_size / n_blocks, (j+1) * fft_size / n_blocks).
 * The convolution with the masked spectrum K~ is defined as
 * y = Re(iFFT(K~ . FFT(u))).  For real u this equals iFFT(K' . FFT(u)) with
 * K'[f] = K[f] * (keep[f] + keep[fft_size - f]) / 2, and K' is what is stored:
 * a bin whose mirror bin is masked differently carries weight 1/2 (a block
 * mask is at most one bin per block edge away from mirror symmetry). */
int fftconv_filter_fft_sparse(const fftconv_plan *plan, const float *k, int64_t Nk,
                              const uint8_t *block_keep, int64_t n_blocks, void *k_f, void *stream);

/* Forward pass with a frequency-sparse k_f made by fftconv_filter_fft_sparse
 * with the same block_keep.  Same result as fftconv_forward on that k_f; the
 * matrix blocks that only meet zeroed bins may be skipped. */
int fftconv_forward_freq_sparse(const fftconv_plan *plan, const void *u, const void *k_f,
                                const uint8_t *block_keep, int64_t n_blocks, void *y,
                                int64_t B, int64_t H, int64_t N, void *workspace, void *stream);

/* Digit cut-off patterns (Appendix A.4: sparsity along each dimension of k_f viewed as an array over
 * the digits of the decomposition).  The digits are those of the plan's factorisation
 * (fftconv_plan_factors, outermost factor first): f = sum_i d_i w_i with w_0 = 1,
 * w_i = w_{i-1} * factors[i-1], so the outermost factor is the least significant digit and the innermost
 * one (the paper's first dimension, the last matrix of the forward transform) the most significant.
 *   digit_keep: host, ndigits = number of factors; digit i keeps digit_keep[i] in [1, factors[i]] of its
 *   values.  The paper cuts one-sided in the half spectrum of its real transform; two real rows share a
 *   complex transform here, which needs a set of bins that is mirror symmetric (f -> fft_size - f), so
 *   the low-pass set of that size is kept: for digit 0 the values nearest zero on the circle,
 *   d <= keep/2 or d >= factors[0] - (keep-1)/2; for the other digits the values nearest the two ends
 *   of the range, d < ceil(keep/2) or d >= factors[i] - keep/2 (the mirror image of a bin has digit
 *   factors[i] - 1 - d there unless all lower digits are zero).
 * A bin is kept when all of its digits are; the result is defined as for fftconv_filter_fft_sparse
 * (mirror bins carry weight 1/2 where the kept set is one bin off mirror symmetry).
 * fftconv_forward_freq_sparse_digits: same result as fftconv_forward on that k_f; digits whose kept set is
 * small let the plan skip work: planes of the per-plane loops (the paper's loop trip counts) and matrix
 * tiles that only meet zeroed bins. */
int fftconv_filter_fft_sparse_digits(const fftconv_plan *plan, const float *k, int64_t Nk,
                                     const int64_t *digit_keep, int ndigits, void *k_f, void *stream);
int fftconv_forward_freq_sparse_digits(const fftconv_plan *plan, const void *u, const void *k_f,
                                       const int64_t *digit_keep, int ndigits, void *y,
                                       int64_t B, int64_t H, int64_t N, void *workspace, void *stream);

/* Bytes of workspace fftconv_forward_gated needs for batch size B: fftconv_workspace_bytes plus,
 * for plans whose kernel does not fuse the gates, room for the gated input (B*H*N elements). */
size_t fftconv_workspace_bytes_gated(const fftconv_plan *plan, int64_t B);

/* Gated convolution (Section 3.1 "Domain-Specific Optimizations"; Section 4.1):
 *     y = v . ((u . w) * k)          (. elementwise, * the convolution of fftconv_forward)
 *   w, v: device, (B, H, N) in the plan's I/O dtype like u; either may be NULL (no gate on that
 *   side; both NULL is fftconv_forward).  v must not alias y.
 * Arithmetic: the product u . w is rounded to the I/O dtype (nearest even) before the transform
 * (it is what the matrix cores consume); the output gate multiplies the convolution result after
 * it has been rounded to the I/O dtype, and the product is rounded again.  Plans whose path
 * (fftconv_plan_path) is "fused3" or "multipass" apply both gates inside their kernels (u, w, v each read
 * once, y written once, no extra workspace); "small" and "staged" plans run one elementwise kernel per
 * gate around fftconv_forward.
 * workspace: at least fftconv_workspace_bytes_gated(plan, B) bytes, may be NULL when that is 0. */
int fftconv_forward_gated(const fftconv_plan *plan, const void *u, const void *w, const void *v, const void *k_f,
                          void *y, int64_t B, int64_t H, int64_t N, void *workspace, void *stream);

/* Backward pass (Section 3.1 "Kernel Fusion and Recomputation"; Section 4.1).  With dy = dL/dy of
 * y = fftconv_forward(u, k_f), nothing of the forward pass is kept; both gradients are recomputed
 * from u, k and dy:
 *     du[b,h,j] = sum_i dy[b,h,i] k[h,(i-j) mod fft_size]          = iFFT(FFT(pad(dy)) . conj(k_f))[0:N]
 *     dk[h,t]   = sum_b sum_i dy[b,h,i] u_pad[b,h,(i-t) mod fft_size] = Re iFFT(sum_b conj(FFT(pad(u))) . FFT(pad(dy)))[t]
 *
 * fftconv_filter_fft_adjoint: as fftconv_filter_fft, but the spectrum of the filter reversed in time
 * (the conjugate spectrum).  The buffer has fftconv_kf_bytes() bytes and is only meant for
 * fftconv_backward_input.
 * fftconv_backward_input: du from dy and the adjoint spectrum; arguments, layouts, workspace and
 * kernels are those of fftconv_forward (du must not alias dy).
 * fftconv_backward_filter: dk (device, (H, Nk) fp32, 1 <= Nk <= fft_size) from u and dy (device,
 * (B, H, N), plan dtype); the reduction over the batch runs in frequency space in fp32, in the
 * order of b (results are reproducible).  workspace: fftconv_workspace_bytes_backward_filter bytes. */
int fftconv_filter_fft_adjoint(const fftconv_plan *plan, const float *k, int64_t Nk, void *k_f, void *stream);
int fftconv_backward_input(const fftconv_plan *plan, const void *dy, const void *k_f_adjoint, void *du,
                           int64_t B, int64_t H, int64_t N, void *workspace, void *stream);
size_t fftconv_workspace_bytes_backward_filter(const fftconv_plan *plan, int64_t B);
int fftconv_backward_filter(const fftconv_plan *plan, const void *u, const void *dy, float *dk, int64_t Nk,
                            int64_t B, int64_t H, int64_t N, void *workspace, void *stream);

/* Fraction of k_f that a cut-off pattern zeroes (Appendix A.4): k_f is viewed
 * as an ndim-dimensional array of shape dims[0..ndim) and, in every dimension
 * i, the last cuts[i] indices are set to zero (cuts[i] = how much of that
 * dimension is removed).  Returns 1 - prod_i (dims[i] - cuts[i]) / dims[i],
 * or a negative value on bad arguments.  Host-only helper. */
double fftconv_sparsity_fraction(const int64_t *dims, const int64_t *cuts, int ndim);

/* Cost model of an order-p decomposition (Section 3.2, Eq. 2).  Host-only helpers.
 *     C = B H sum_{i=1..p} ( 16 N N_i / gamma(N_i) + 4 N / omega(i) )          [seconds]
 * gamma(N_i) = tau_M if N_i >= mu else tau_G; omega(i) = sigma_S when the intermediate of step i stays
 * on chip, sigma_H otherwise: the innermost three steps form one fused kernel whose first step reads
 * from HBM and whose later steps stay on chip iff the subsequence it works on (N over the outer
 * factors) is at most sram_seq; every step outside it goes through HBM.
 * fftconv_machine_preset: FFTCONV_MACHINE_MI355X = what fftconv_measure_machine returned on an MI355X
 * (python bench.py --constants prints a fresh measurement beside the preset), FFTCONV_MACHINE_A100_PAPER =
 * the paper's table for A100-40GB (Appendix C).
 * fftconv_measure_machine: measures the four rates on the current device with micro-benchmark kernels
 * inside the library, following Appendix C ("Empirical GPU Profiling"): sigma_H from a plain copy of 1 GiB
 * (bytes read + written per second), tau_M from 16-bit matrix-core products issued back to back on every
 * SIMD, tau_G from fp32 twiddle products applied over and over (6 operations per complex product),
 * sigma_S from the slow-down of a chain of matrix products when each intermediate result takes a trip
 * through LDS.  Synchronous; allocates and frees about 2 GiB of device memory; takes about a second.
 * fftconv_cost_model: C for factors[0..p) (outermost first, product N); negative on bad arguments.
 * fftconv_balanced_factors: power-of-two factors of N as equal as possible, larger first.
 * fftconv_plan_order: the order p in {2, 3, 4} with balanced factors that minimises C for B = H = 1;
 * writes p, its factors (room for 4) and the cost; any output pointer may be NULL. */
typedef struct fftconv_machine {
    double sigma_H;     /* achievable HBM bandwidth, bytes / s */
    double sigma_S;     /* achievable on-chip memory bandwidth, bytes / s */
    double tau_M;       /* achievable matrix-unit rate, FLOP / s */
    double tau_G;       /* achievable general arithmetic rate, FLOP / s */
    int mu;             /* size of the matrix-multiply unit */
    int64_t sram_seq;   /* longest sequence whose intermediates stay on chip */
} fftconv_machine;
#define FFTCONV_MACHINE_MI355X 0
#define FFTCONV_MACHINE_A100_PAPER 1
void fftconv_machine_preset(int which, fftconv_machine *m);
int fftconv_measure_machine(fftconv_machine *m);
double fftconv_cost_model(const fftconv_machine *m, int64_t B, int64_t H, int64_t N, int p, const int64_t *factors);
int fftconv_balanced_factors(int64_t N, int p, int64_t *factors);
int fftconv_plan_order(const fftconv_machine *m, int64_t N, int *p, int64_t *factors, double *cost);

/* Name of the kernel family the plan dispatches to ("staged", "fused3", ...);
 * for logs and benchmarks.  Never NULL for a valid plan. */
const char *fftconv_plan_path(const fftconv_plan *plan);

/* Factorisation of fft_size the plan uses: writes up to max_factors factors
 * (outermost first) and returns how many there are. */
int fftconv_plan_factors(const fftconv_plan *plan, int64_t *factors, int max_factors);

const char *fftconv_strerror(int code);
const char *fftconv_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* FFTCONV_H */
