/*
 * conv_oracle.c -- TEST INFRASTRUCTURE, not part of the product.
 *
 * A plain, slow, fp64 CPU statement of what the FFT-convolution path must
 * return, written from the definitions in the paper and from nothing else.
 * It shares no code, table or constant with the HIP library.  Only tests,
 * the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * What is computed (paper Section 2.1, "FFT Convolution"): a convolution is
 *     (u * k)[i] = sum_j u[j] k[i-j],
 * and the FFT route (Eq. 1) yields the CIRCULAR form of it, in which an index
 * i-j < 0 wraps round to the end of k; padding u and k with zeros up to the
 * transform length M makes the wrapped taps hit zeros, which gives the causal
 * convolution.  So the one definition that covers every case is
 *
 *     y[b,h,i] = sum_{j=0}^{N-1} u[b,h,j] * kext[h, (i-j) mod M],  0 <= i < N,
 *
 * kext = the filter laid out on M taps (zero beyond its support).  There is
 * no FFT in this file: the sum is evaluated term by term in double precision.
 *
 * Frequency-sparse filters (Section 3.3, Appendix A.4) are defined by zeroing
 * entries of k_f = DFT_M(kext).  oracle_mask_filter() applies such a 0/1 mask
 * with a naive O(M^2) DFT and inverse DFT and returns the real time-domain
 * filter the masked spectrum corresponds to; the convolution above then runs
 * on that filter.
 *
 * Every function here is pinned by tests/test_oracle_pins.py against things
 * it does not share code with: a dense DFT-matrix evaluation of Eq. 1 on tiny
 * inputs, closed forms, exact integer polynomial products, library routines.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* One output sample of one sequence: sum_j u[j] * kext[(i-j) mod M].
 * For j <= i the tap index is i-j; for j > i it wraps to M+i-j. */
static double conv_point(const double *u, const double *kext, int64_t N, int64_t M, int64_t i)
{
    double acc = 0.0;
    int64_t jmax = i < N - 1 ? i : N - 1;
    for (int64_t j = 0; j <= jmax; ++j)
        acc += u[j] * kext[i - j];
    for (int64_t j = i + 1; j < N; ++j)
        acc += u[j] * kext[M + i - j];
    return acc;
}

/* Full convolution.  u: (B,H,N); kext: (H,M); y: (B,H,N); all row-major fp64.
 * Requires 1 <= N <= M.  Returns 0, or -1 on bad sizes. */
int oracle_fftconv(const double *u, const double *kext, double *y,
                   int64_t B, int64_t H, int64_t N, int64_t M)
{
    if (B < 0 || H < 0 || N < 1 || M < N) return -1;
    int64_t nseq = B * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t s = 0; s < nseq; ++s) {
        int64_t h = s % H;
        const double *us = u + s * N;
        const double *ks = kext + h * M;
        double *ys = y + s * N;
        for (int64_t i = 0; i < N; ++i)
            ys[i] = conv_point(us, ks, N, M, i);
    }
    return 0;
}

/* The same sum at chosen output positions only.
 * u: (S,N) -- S sequences already gathered by the caller; kext: (S,M) -- the
 * filter row that belongs to each of them; idx: (S,P) output positions in
 * [0,N); out: (S,P).  Used where N is too long to evaluate every output. */
int oracle_fftconv_at(const double *u, const double *kext, const int64_t *idx, double *out,
                      int64_t S, int64_t N, int64_t M, int64_t P)
{
    if (S < 0 || N < 1 || M < N || P < 0) return -1;
    for (int64_t t = 0; t < S * P; ++t)
        if (idx[t] < 0 || idx[t] >= N) return -1;
    int64_t total = S * P;
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t t = 0; t < total; ++t) {
        int64_t s = t / P;
        out[t] = conv_point(u + s * N, kext + s * M, N, M, idx[t]);
    }
    return 0;
}

/* The same definition for a filter with few non-zero taps, given as a list: channel h has T taps,
 * tap t at position pos[h,t] in [0,M) with value val[h,t] (positions distinct within a channel), so
 * kext[h,p] = val[h,t] where p = pos[h,t] and zero elsewhere.  In the sum over j only the terms with
 * (i-j) mod M = pos[h,t] survive, i.e. j = (i - pos[h,t]) mod M, and only if that j is an input
 * sample (j < N):
 *     y[b,h,i] = sum_t val[h,t] * u[b,h,(i - pos[h,t]) mod M]   [(i - pos[h,t]) mod M < N].
 * O(T N) per sequence, which makes every output of a very long row checkable.
 * u: (B,H,N); pos, val: (H,T); y: (B,H,N).  Returns 0, or -1 on bad sizes or positions. */
int oracle_fftconv_taps(const double *u, const int64_t *pos, const double *val, double *y,
                        int64_t B, int64_t H, int64_t N, int64_t M, int64_t T)
{
    if (B < 0 || H < 0 || N < 1 || M < N || T < 0) return -1;
    for (int64_t h = 0; h < H; ++h)
        for (int64_t t = 0; t < T; ++t) {
            if (pos[h * T + t] < 0 || pos[h * T + t] >= M) return -1;
            for (int64_t t2 = 0; t2 < t; ++t2)
                if (pos[h * T + t2] == pos[h * T + t]) return -1;
        }
    int64_t nseq = B * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t s = 0; s < nseq; ++s) {
        int64_t h = s % H;
        const double *us = u + s * N;
        double *ys = y + s * N;
        for (int64_t i = 0; i < N; ++i) {
            double acc = 0.0;
            for (int64_t t = 0; t < T; ++t) {
                int64_t j = i - pos[h * T + t];
                if (j < 0) j += M;
                if (j < N) acc += val[h * T + t] * us[j];
            }
            ys[i] = acc;
        }
    }
    return 0;
}

/* Frequency masking of one or more filters.
 * kext: (H,M) real; keep: (M) bytes, 1 = keep DFT bin f, 0 = set it to zero,
 * indexed by the natural frequency f of X[f] = sum_t x[t] exp(-2 pi i f t / M)
 * (the convention of Appendix A.1); out: (H,M) real:
 *     out[t] = Re( (1/M) sum_f keep[f] X[f] exp(+2 pi i f t / M) ).
 * Phases are reduced exactly with integer arithmetic: p = f*t mod M is carried
 * along the inner loop (add the step, subtract M on overflow) and indexes a
 * table of the M roots of unity, so no large-argument sin/cos occurs. */
int oracle_mask_filter(const double *kext, const uint8_t *keep, double *out, int64_t H, int64_t M)
{
    if (H < 0 || M < 1) return -1;
    const double two_pi = 6.283185307179586476925286766559;
    double *wr = (double *)malloc(sizeof(double) * (size_t)M);
    double *wi = (double *)malloc(sizeof(double) * (size_t)M);
    if (!wr || !wi) { free(wr); free(wi); return -2; }
    for (int64_t j = 0; j < M; ++j) {           /* w[j] = exp(-2 pi i j / M) */
        wr[j] = cos(two_pi * (double)j / (double)M);
        wi[j] = -sin(two_pi * (double)j / (double)M);
    }
    int rc = 0;
#pragma omp parallel
    {
        double *Xr = (double *)malloc(sizeof(double) * (size_t)M);
        double *Xi = (double *)malloc(sizeof(double) * (size_t)M);
        if (!Xr || !Xi) {
#pragma omp atomic write
            rc = -2;
        }
#pragma omp barrier
        if (rc == 0) {
#pragma omp for schedule(dynamic, 1)
            for (int64_t h = 0; h < H; ++h) {
                const double *x = kext + h * M;
                for (int64_t f = 0; f < M; ++f) {
                    double sr = 0.0, si = 0.0;
                    if (keep[f]) {
                        int64_t p = 0;                    /* p = f*t mod M */
                        for (int64_t t = 0; t < M; ++t) {
                            sr += x[t] * wr[p];
                            si += x[t] * wi[p];
                            p += f;
                            if (p >= M) p -= M;
                        }
                    }
                    Xr[f] = sr;
                    Xi[f] = si;
                }
                for (int64_t t = 0; t < M; ++t) {
                    double sr = 0.0;
                    int64_t p = 0;                        /* p = f*t mod M */
                    for (int64_t f = 0; f < M; ++f) {
                        /* Re( X[f] * conj(w[p]) ) */
                        sr += Xr[f] * wr[p] + Xi[f] * wi[p];
                        p += t;
                        if (p >= M) p -= M;
                    }
                    out[h * M + t] = sr / (double)M;
                }
            }
        }
        free(Xr);
        free(Xi);
    }
    free(wr);
    free(wi);
    return rc;
}

/* Backward pass (Section 3.1 "Kernel Fusion and Recomputation"; Section 4.1 backward tables): for
 * a loss L with dy = dL/dy, the gradients of the definition at the top of this file are its
 * partial derivatives written out term by term,
 *     dy[i]/du[j]    = kext[(i-j) mod M]         =>  du[b,h,j] = sum_{i<N} dy[b,h,i] kext[h,(i-j) mod M]
 *     dy[i]/dkext[t] = u[j] where (i-j) mod M = t =>  dk[h,t]   = sum_b sum_{i<N} dy[b,h,i] upad[b,h,(i-t) mod M]
 * (upad = u laid out on M samples, zero beyond N).  No FFT, no reuse of the forward code.
 * dy, u, du: (B,H,N); kext: (H,M); dk: (H,Nk), the first Nk taps.  Returns 0, or -1 on bad sizes. */
int oracle_backward_u(const double *dy, const double *kext, double *du, int64_t B, int64_t H, int64_t N, int64_t M)
{
    if (B < 0 || H < 0 || N < 1 || M < N) return -1;
    int64_t nseq = B * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t s = 0; s < nseq; ++s) {
        const double *g = dy + s * N;
        const double *kr = kext + (s % H) * M;
        double *out = du + s * N;
        for (int64_t j = 0; j < N; ++j) {
            double acc = 0.0;
            for (int64_t i = 0; i < N; ++i) {
                int64_t t = i - j;
                if (t < 0) t += M;
                acc += g[i] * kr[t];
            }
            out[j] = acc;
        }
    }
    return 0;
}

int oracle_backward_k(const double *u, const double *dy, double *dk, int64_t B, int64_t H, int64_t N, int64_t M,
                      int64_t Nk)
{
    if (B < 0 || H < 0 || N < 1 || M < N || Nk < 1 || Nk > M) return -1;
    int64_t ntap = H * Nk;
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t e = 0; e < ntap; ++e) {
        int64_t h = e / Nk, t = e % Nk;
        double acc = 0.0;
        for (int64_t b = 0; b < B; ++b) {
            const double *ur = u + (b * H + h) * N;
            const double *g = dy + (b * H + h) * N;
            for (int64_t i = 0; i < N; ++i) {
                int64_t j = i - t;
                if (j < 0) j += M;
                if (j < N) acc += g[i] * ur[j];
            }
        }
        dk[e] = acc;
    }
    return 0;
}

/* Number of threads the parallel loops above run on. */
int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
