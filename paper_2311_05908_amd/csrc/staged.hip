// Generic transforms, one launch per stage of the order-p decomposition (paper
// Section 2.1: F_M as a chain of small DFT-matrix products with twiddle diagonals
// in between), intermediates in HBM; rows that fit in LDS run all stages in one
// kernel there (lds_fft.h).  Users: the fp64 filter transform k -> k_f of the
// plans without a fused one, the filter gradient of the plans below fft_size
// 16384 without a fused kernel, and the k_f layout of the fp32 plans, whose
// forward pass lives in long_fft.hip.
//
// Index maps.  M = N_1 * ... * N_p.  Time index n = sum_i n_i S_i with
// S_i = prod_{j>i} N_j (n_1 most significant); frequency f = sum_i k_i R_i with
// R_i = prod_{j<i} N_j (k_1 least significant).  Then
//   W_M^{n f} = prod_i W_{N_i}^{n_i k_i} * prod_i W_M^{k_i R_i (n mod S_i)},
// so stage i contracts digit i in place (position sum_i d_i S_i, d_i = n_i before
// and k_i after the stage) and is followed by the twiddle W_M^{k_i R_i r},
// r = the not-yet-transformed lower digits.  After the last stage position
// sum_i k_i S_i holds frequency sum_i k_i R_i; k_f is stored in that order so no
// permutation is ever executed.  The inverse runs the mirrored chain with
// conjugated factors; its 1/M lives in k_f.
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>

#include <cmath>
#include <type_traits>

#include "lds_fft.h"
#include "fftconv_internal.h"

namespace fftconv {

FacList staged_factors_for(int64_t M);

namespace {

template <typename T> struct C2;
template <> struct C2<float> { using type = float2; };
template <> struct C2<double> { using type = double2; };

__device__ __forceinline__ float load_real(const float *p, int64_t i) { return p[i]; }
__device__ __forceinline__ float load_real(const __half *p, int64_t i) { return __half2float(p[i]); }
__device__ __forceinline__ float load_real(const __hip_bfloat16 *p, int64_t i) { return __bfloat162float(p[i]); }

// Zero-padded real input -> complex buffer (imaginary part 0, zeros for n >= len).
template <typename V, typename In>
__global__ void k_load_padded(const In *src, V *dst, int64_t len, int64_t M, int64_t nrows, bool reversed = false)
{
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= nrows * M) return;
    int64_t row = idx / M, n = idx % M;
    // reversed: position n holds tap (M - n) mod M, the circularly time-reversed sequence, whose
    // spectrum is the conjugate of the original's (real input)
    if (reversed && n != 0) n = M - n;
    V v;
    v.x = n < len ? (decltype(v.x))load_real(src, row * len + n) : 0;
    v.y = 0;
    dst[idx] = v;
}

// Forward stage: out[prefix, k, r] = W_M^{k R r} * sum_n W_{Nj}^{n k} in[prefix, n, r].
// tws: stride of the twiddle table when it was built for a multiple tws*M of this transform length
template <typename V>
__global__ void k_stage_fwd(const V *in, V *out, const V *w, int64_t M, int Nj, int64_t Sj, int64_t Rj,
                            int64_t nrows, int64_t tws)
{
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= nrows * M) return;
    int64_t row = idx / M, p = idx % M;
    int64_t r = p % Sj;
    int k = (int)((p / Sj) % Nj);
    int64_t base = row * M + (p - (int64_t)k * Sj);
    int64_t step = M / Nj;
    V acc;
    acc.x = 0;
    acc.y = 0;
    int ph = 0;                                   // (n*k) mod Nj
    for (int n = 0; n < Nj; ++n) {
        V x = in[base + (int64_t)n * Sj];
        V t = cmul(x, w[(int64_t)ph * step * tws]);
        acc.x += t.x;
        acc.y += t.y;
        ph += k;
        if (ph >= Nj) ph -= Nj;
    }
    out[idx] = cmul(acc, w[(int64_t)k * Rj * r * tws]);  // k*Rj*r < Nj*Rj*Sj = M
}

// Inverse stage: out[prefix, n, r] = sum_k conj(W_{Nj}^{n k} W_M^{k R r}) in[prefix, k, r].
template <typename V>
__global__ void k_stage_inv(const V *in, V *out, const V *w, int64_t M, int Nj, int64_t Sj, int64_t Rj,
                            int64_t nrows)
{
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= nrows * M) return;
    int64_t row = idx / M, p = idx % M;
    int64_t r = p % Sj;
    int n = (int)((p / Sj) % Nj);
    int64_t base = row * M + (p - (int64_t)n * Sj);
    int64_t step = M / Nj;
    V acc;
    acc.x = 0;
    acc.y = 0;
    int ph = 0;                                   // (n*k) mod Nj
    for (int k = 0; k < Nj; ++k) {
        V x = in[base + (int64_t)k * Sj];
        int64_t e = (int64_t)ph * step + (int64_t)k * Rj * r;
        if (e >= M) e -= M;
        V t = cmul_conj(x, w[e]);
        acc.x += t.x;
        acc.y += t.y;
        ph += n;
        if (ph >= Nj) ph -= Nj;
    }
    out[idx] = acc;
}

// The same two stages with the length-R transform done in registers (R a power of two <= 32): one thread per
// (row, prefix, r) loads its R inputs once, instead of R loads per output.  The plain kernels above remain for
// factors these do not cover.
template <int R, typename V>
__global__ void k_stage_fwd_reg(const V *in, V *out, const V *w, int64_t M, int64_t Sj, int64_t Rj,
                                int64_t nrows, int64_t tws)
{
    const int64_t per_row = M / R;
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= nrows * per_row) return;
    const int64_t row = idx / per_row, q = idx % per_row;
    const int64_t r = q % Sj, prefix = q / Sj;
    const int64_t base = row * M + prefix * (R * Sj) + r;
    V x[R];
#pragma unroll
    for (int n = 0; n < R; ++n) x[n] = in[base + (int64_t)n * Sj];
    dft_reg<R, false>(x);
#pragma unroll
    for (int k = 0; k < R; ++k) out[base + (int64_t)k * Sj] = cmul(x[k], w[(int64_t)k * Rj * r * tws]);
}

template <int R, typename V>
__global__ void k_stage_inv_reg(const V *in, V *out, const V *w, int64_t M, int64_t Sj, int64_t Rj,
                                int64_t nrows)
{
    const int64_t per_row = M / R;
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= nrows * per_row) return;
    const int64_t row = idx / per_row, q = idx % per_row;
    const int64_t r = q % Sj, prefix = q / Sj;
    const int64_t base = row * M + prefix * (R * Sj) + r;
    V x[R];
#pragma unroll
    for (int k = 0; k < R; ++k) x[k] = cmul_conj(in[base + (int64_t)k * Sj], w[(int64_t)k * Rj * r]);   // k Rj r < M
    dft_reg<R, true>(x);
#pragma unroll
    for (int n = 0; n < R; ++n) out[base + (int64_t)n * Sj] = x[n];
}

// ---- Rows resident in LDS (lds_fft.h): one workgroup per row, HBM touched once each way.
// Forward transform of zero-padded real rows (the filter transform): src (nrows, len) fp32 -> spec
// (nrows, M) in position order.  reversed: see k_load_padded.
__global__ void __launch_bounds__(LDS_ROW_THREADS) k_rows_fwd_lds(const float *__restrict__ src, double2 *__restrict__ spec,
                                                                 const double2 *__restrict__ w, FacList fl, int M,
                                                                 int64_t len, int tws, bool reversed)
{
    extern __shared__ double2 XD[];
    const int64_t row = blockIdx.x;
    // (a tap beyond `len` reads tap 0 and is discarded: unconditional loads, several in flight per thread)
    for (int n0 = threadIdx.x; n0 < M; n0 += 8 * LDS_ROW_THREADS) {
        float v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int n = n0 + j * LDS_ROW_THREADS;
            const int t = (reversed && n != 0) ? M - n : n;
            v[j] = src[row * len + ((n < M && t < len) ? t : 0)];
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) asm volatile("" ::"v"(v[j]));
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int n = n0 + j * LDS_ROW_THREADS;
            const int t = (reversed && n != 0) ? M - n : n;
            if (n < M) XD[lds_slot(n)] = make_double2(t < len ? (double)v[j] : 0.0, 0.0);
        }
    }
    __syncthreads();
    lds_forward(XD, w, fl, M, tws);
#pragma unroll 8
    for (int n = threadIdx.x; n < M; n += LDS_ROW_THREADS) spec[row * M + n] = XD[lds_slot(n)];
}

// Unnormalised inverse transform of position-ordered spectra, real part of the first Nk samples times scale
// (the tail of the filter gradient).
__global__ void __launch_bounds__(LDS_ROW_THREADS) k_rows_inv_dk_lds(const float2 *__restrict__ spec, float *__restrict__ dk,
                                                                    const float2 *__restrict__ w, FacList fl, int M,
                                                                    int64_t Nk, float scale)
{
    extern __shared__ float2 XF[];
    const int64_t row = blockIdx.x;
#pragma unroll 8
    for (int n = threadIdx.x; n < M; n += LDS_ROW_THREADS) XF[lds_slot(n)] = spec[row * M + n];
    __syncthreads();
    lds_inverse(XF, w, fl, M, 1);
    for (int n = threadIdx.x; n < Nk; n += LDS_ROW_THREADS) dk[row * Nk + n] = XF[lds_slot(n)].x * scale;
}

inline unsigned grid_of(int64_t n, int bs) { return (unsigned)((n + bs - 1) / bs); }

// one stage, in registers when the factor allows; returns false if it does not
template <typename V>
bool launch_stage_reg(bool inverse, const V *src, V *dst, const V *w, int64_t M, int Nj, int64_t S,
                      int64_t R, int64_t nrows, int64_t tws, hipStream_t s)
{
    const int bs = 256;
    const unsigned grid = grid_of(nrows * (M / Nj), bs);
#define STAGE_REG(RR)                                                                                          \
    case RR:                                                                                                   \
        if (inverse)                                                                                           \
            hipLaunchKernelGGL((k_stage_inv_reg<RR, V>), dim3(grid), dim3(bs), 0, s, src, dst, w, M, S, R, nrows);   \
        else                                                                                                   \
            hipLaunchKernelGGL((k_stage_fwd_reg<RR, V>), dim3(grid), dim3(bs), 0, s, src, dst, w, M, S, R, nrows, tws); \
        return true;
    switch (Nj) {
        STAGE_REG(2)
        STAGE_REG(4)
        STAGE_REG(8)
        STAGE_REG(16)
        STAGE_REG(32)
    default: return false;
    }
#undef STAGE_REG
}

// spectra in position order (fp64) -> staged k_f (fp32 pairs, same position order), scaled 1/M,
// with dropped frequency blocks zeroed.
__global__ void k_pack_staged(const double2 *spec, float2 *kf, FacList fl, int64_t M, int64_t h0, int64_t nh,
                              const uint8_t *keep, int64_t n_blocks)
{
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= nh * M) return;
    int64_t h = idx / M, f = idx % M;
    int64_t p = freq_to_pos(f, fl, M);
    double2 v = spec[h * M + p];
    double sc = mask_weight(keep, n_blocks, f, M) / (double)M;
    kf[(h0 + h) * M + p] = make_float2((float)(v.x * sc), (float)(v.y * sc));
}

FacList fac_list(const fftconv_plan *p) { return staged_fac_list(p); }

inline unsigned grid_for(int64_t n, int bs) { return (unsigned)((n + bs - 1) / bs); }

template <typename V>
int run_stages_fwd(const FacList &fl, int64_t M, int64_t tws, V *a, V *b, const V *w, int64_t nrows, hipStream_t s,
                   V **result)
{
    const int bs = 256;
    int64_t S = M, R = 1;
    V *src = a, *dst = b;
    for (int i = 0; i < fl.nf; ++i) {
        int Nj = fl.fac[i];
        S /= Nj;
        if (!launch_stage_reg<V>(false, src, dst, w, M, Nj, S, R, nrows, tws, s))
            hipLaunchKernelGGL(k_stage_fwd<V>, dim3(grid_for(nrows * M, bs)), dim3(bs), 0, s, src, dst, w, M, Nj, S, R,
                               nrows, tws);
        FC_HIP(hipGetLastError());
        R *= Nj;
        V *t = src; src = dst; dst = t;
    }
    *result = src;
    return FFTCONV_OK;
}

}  // namespace

int staged_init(fftconv_plan *p)
{
    // factors of 16, remainder (2, 4 or 8) last; the fp32 plans from 32768 up keep k_f in the position order of
    // their two-kernel transforms (long_fft.hip)
    const FacList fl0 = (p->path == PATH_STAGED && p->M >= 32768) ? long_fft_factor_list(p->M) : staged_factors_for(p->M);
    p->st.nf = fl0.nf;
    for (int i = 0; i < MAX_FACTORS; ++i) p->st.fac[i] = fl0.fac[i];

    int64_t M = p->M;
    std::vector<double2> w64((size_t)M);
    std::vector<float2> w32((size_t)M);
    const double two_pi = 6.283185307179586476925286766559;
    for (int64_t t = 0; t < M; ++t) {
        // exact octant symmetry is not needed: libm is accurate to < 1 ulp for |x| <= 2 pi
        double a = two_pi * (double)t / (double)M;
        w64[t] = make_double2(std::cos(a), -std::sin(a));
        w32[t] = make_float2((float)w64[t].x, (float)w64[t].y);
    }
    FC_HIP(hipMalloc((void **)&p->st.w64, sizeof(double2) * M));
    FC_HIP(hipMalloc((void **)&p->st.w32, sizeof(float2) * M));
    FC_HIP(hipMemcpy(p->st.w64, w64.data(), sizeof(double2) * M, hipMemcpyHostToDevice));
    FC_HIP(hipMemcpy(p->st.w32, w32.data(), sizeof(float2) * M, hipMemcpyHostToDevice));

    // filter-transform scratch: two ping-pong buffers of at most 64 MiB, or 8 channels, each
    const int64_t cap = (int64_t)64 << 20;
    int64_t per_ch = M * (int64_t)sizeof(double2);
    int64_t chunk = cap / per_ch;
    if (chunk < 8) chunk = 8;
    if (chunk > p->H) chunk = p->H;
    p->filt_chunk = chunk;
    FC_HIP(hipMalloc((void **)&p->filt_a, (size_t)(chunk * per_ch)));
    FC_HIP(hipMalloc((void **)&p->filt_b, (size_t)(chunk * per_ch)));
    return FFTCONV_OK;
}

void staged_destroy(fftconv_plan *p)
{
    if (p->st.w64) (void)hipFree(p->st.w64);
    if (p->st.w32) (void)hipFree(p->st.w32);
    if (p->filt_a) (void)hipFree(p->filt_a);
    if (p->filt_b) (void)hipFree(p->filt_b);
    p->st.w64 = nullptr;
    p->st.w32 = nullptr;
    p->filt_a = p->filt_b = nullptr;
}

size_t staged_kf_bytes(const fftconv_plan *p) { return (size_t)(p->H * p->M) * sizeof(float2); }

size_t staged_workspace_bytes(const fftconv_plan *p, int64_t) { return long_forward_workspace_bytes(p); }

// fp32 I/O from fft_size 8192 up: the whole row in LDS up to 16384, three kernels above (long_fft.hip)
int staged_forward(const fftconv_plan *p, const void *u, const void *kf, void *y, int64_t B, void *workspace,
                   hipStream_t s)
{
    return long_forward(p, u, kf, y, B, workspace, s);
}

// Largest row the LDS-resident kernels take: 8192 fp64 or 16384 fp32 complex points with their padding.
constexpr size_t LDS_ROW_MAX = (8192 + 512) * sizeof(double2);

static int raise_lds_limit(const void *kern) { return raise_dynamic_lds(kern, (int)LDS_ROW_MAX); }

// Rows short enough for LDS take the one-kernel transform: *ran says whether this was one (otherwise the
// caller runs the stages through HBM).
static int rows_fwd_lds(const fftconv_plan *p, const FacList &fl, int64_t M, int64_t tws, const float *k, int64_t Nk,
                        int64_t nh, bool reversed, hipStream_t s, double2 **result, bool *ran)
{
    const size_t bytes = lds_row_bytes(M, sizeof(double2));
    *ran = bytes <= LDS_ROW_MAX && lds_factors_ok(fl);
    if (!*ran) return FFTCONV_OK;
    const int rc = raise_lds_limit((const void *)k_rows_fwd_lds);
    if (rc) return rc;
    hipLaunchKernelGGL(k_rows_fwd_lds, dim3((unsigned)nh), dim3(LDS_ROW_THREADS), bytes, s, k, p->filt_a, p->st.w64, fl,
                       (int)M, Nk, (int)tws, reversed);
    FC_HIP(hipGetLastError());
    *result = p->filt_a;
    return FFTCONV_OK;
}

int staged_filter_transform(const fftconv_plan *p, const float *k, int64_t Nk, int64_t h0, int64_t nh, hipStream_t s,
                            double2 **result, bool adjoint)
{
    bool ran = false;
    const int rc = rows_fwd_lds(p, fac_list(p), p->M, 1, k + h0 * Nk, Nk, nh, adjoint, s, result, &ran);
    if (rc || ran) return rc;
    const int bs = 256;
    hipLaunchKernelGGL((k_load_padded<double2, float>), dim3(grid_for(nh * p->M, bs)), dim3(bs), 0, s, k + h0 * Nk,
                       p->filt_a, Nk, p->M, nh, adjoint);
    FC_HIP(hipGetLastError());
    return run_stages_fwd<double2>(fac_list(p), p->M, 1, p->filt_a, p->filt_b, p->st.w64, nh, s, result);
}

FacList staged_factors_for(int64_t M)
{
    FacList fl;
    for (int i = 0; i < MAX_FACTORS; ++i) fl.fac[i] = 0;
    int lg = 0;
    while (((int64_t)1 << lg) < M) ++lg;
    int nf = 0, rem = lg;
    while (rem >= 4) { fl.fac[nf++] = 16; rem -= 4; }
    if (rem) fl.fac[nf++] = 1 << rem;
    fl.nf = nf;
    return fl;
}

int staged_pack_kf(const fftconv_plan *p, const double2 *spec, int64_t h0, int64_t nh, const uint8_t *keep_dev,
                   int64_t n_blocks, void *kf, hipStream_t s)
{
    const int bs = 256;
    hipLaunchKernelGGL(k_pack_staged, dim3(grid_for(nh * p->M, bs)), dim3(bs), 0, s, spec, (float2 *)kf, fac_list(p),
                       p->M, h0, nh, keep_dev, n_blocks);
    FC_HIP(hipGetLastError());
    return FFTCONV_OK;
}

FacList staged_fac_list(const fftconv_plan *p)
{
    FacList fl;
    fl.nf = p->st.nf;
    for (int i = 0; i < MAX_FACTORS; ++i) fl.fac[i] = (int)p->st.fac[i];
    return fl;
}

// ---- filter gradient (backward pass, Section 3.1 "Kernel Fusion and Recomputation"):
//   dk_f[h] = sum_b conj(FFT(pad(u[b,h]))) . FFT(pad(dy[b,h]))   (reduction over the batch in frequency space,
//   nothing of the forward pass is stored), dk[h] = Re(iFFT(dk_f[h]))[0:Nk].
// acc[h, p] (+)= conj(xu[r, p]) * xdy[r, p] for the rows r of one batch index (distinct channels, so no two
// threads meet and the sum over b runs in a fixed order)
__global__ void k_accumulate_corr(float2 *acc, const float2 *xu, const float2 *xdy, int64_t M, int64_t nrows, bool first)
{
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= nrows * M) return;
    const float2 a = xu[idx], b = xdy[idx];
    float2 v = make_float2(a.x * b.x + a.y * b.y, a.x * b.y - a.y * b.x);
    if (!first) {
        const float2 o = acc[idx];
        v.x += o.x;
        v.y += o.y;
    }
    acc[idx] = v;
}

__global__ void k_zero_f32(float *x, int64_t n)
{
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx < n) x[idx] = 0.f;
}

__global__ void k_store_dk(const float2 *x, float *dk, int64_t Nk, int64_t M, int64_t nrows, float scale)
{
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= nrows * Nk) return;
    int64_t row = idx / Nk, t = idx % Nk;
    dk[idx] = x[row * M + t].x * scale;
}

// channels per trip through the scratch of the filter gradient: buffers of at most 256 MiB
static int64_t bwd_chunk(const fftconv_plan *p)
{
    int64_t cap = ((int64_t)256 << 20) / (p->M * (int64_t)sizeof(float2));
    if (cap < 1) cap = 1;
    return p->H < cap ? p->H : cap;
}

// dk rows from position-ordered spectra: unnormalised inverse stages (ping-pong between spec and other,
// both nrows * M), real part of the first Nk samples, times 1/M.  spec is overwritten.
int staged_inverse_to_dk(const fftconv_plan *p, float2 *spec, float2 *other, int64_t nrows, float *dk, int64_t Nk,
                         hipStream_t s)
{
    const int bs = 256;
    const int64_t M = p->M;
    const size_t lds_bytes = lds_row_bytes(M, sizeof(float2));
    if (lds_bytes <= LDS_ROW_MAX && lds_factors_ok(fac_list(p))) {
        const int rc = raise_lds_limit((const void *)k_rows_inv_dk_lds);
        if (rc) return rc;
        hipLaunchKernelGGL(k_rows_inv_dk_lds, dim3((unsigned)nrows), dim3(LDS_ROW_THREADS), lds_bytes, s, spec, dk,
                           p->st.w32, fac_list(p), (int)M, Nk, 1.0f / (float)M);
        FC_HIP(hipGetLastError());
        return FFTCONV_OK;
    }
    float2 *src = spec, *dst = other;
    int64_t S = 1, R = M;
    for (int i = p->st.nf - 1; i >= 0; --i) {
        const int Nj = (int)p->st.fac[i];
        R /= Nj;
        if (!launch_stage_reg<float2>(true, src, dst, p->st.w32, M, Nj, S, R, nrows, 1, s))
            hipLaunchKernelGGL(k_stage_inv<float2>, dim3(grid_for(nrows * M, bs)), dim3(bs), 0, s, src, dst, p->st.w32, M,
                               Nj, S, R, nrows);
        FC_HIP(hipGetLastError());
        S *= Nj;
        float2 *t = src;
        src = dst;
        dst = t;
    }
    hipLaunchKernelGGL(k_store_dk, dim3(grid_for(nrows * Nk, bs)), dim3(bs), 0, s, src, dk, Nk, M, nrows,
                       1.0f / (float)M);
    FC_HIP(hipGetLastError());
    return FFTCONV_OK;
}

int64_t staged_backward_chunk(const fftconv_plan *p) { return bwd_chunk(p); }

size_t staged_backward_filter_bytes(const fftconv_plan *p)
{
    // dk_f accumulator for every channel + two ping-pong pairs (u and dy) of one chunk of channels
    return (size_t)((p->H + 4 * bwd_chunk(p)) * p->M) * sizeof(float2);
}

template <typename IO>
static int staged_backward_filter_t(const fftconv_plan *p, const IO *u, const IO *dy, float *dk, int64_t Nk, int64_t B,
                                    void *workspace, hipStream_t s)
{
    const int bs = 256;
    const int64_t M = p->M, N = p->N, H = p->H, chunk = bwd_chunk(p);
    float2 *acc = (float2 *)workspace;
    float2 *a1 = acc + H * M, *b1 = a1 + chunk * M, *a2 = b1 + chunk * M, *b2 = a2 + chunk * M;
    if (B == 0) {                                 // an empty batch: dk = 0
        hipLaunchKernelGGL(k_zero_f32, dim3(grid_for(H * Nk, bs)), dim3(bs), 0, s, dk, H * Nk);
        FC_HIP(hipGetLastError());
        return FFTCONV_OK;
    }
    for (int64_t b = 0; b < B; ++b)
        for (int64_t h0 = 0; h0 < H; h0 += chunk) {
            const int64_t nrows = H - h0 < chunk ? H - h0 : chunk;
            const int64_t row0 = b * H + h0;
            float2 *xu = nullptr, *xdy = nullptr;
            hipLaunchKernelGGL((k_load_padded<float2, IO>), dim3(grid_for(nrows * M, bs)), dim3(bs), 0, s, u + row0 * N,
                               a1, N, M, nrows, false);
            FC_HIP(hipGetLastError());
            int rc = run_stages_fwd<float2>(fac_list(p), M, 1, a1, b1, p->st.w32, nrows, s, &xu);
            if (rc) return rc;
            hipLaunchKernelGGL((k_load_padded<float2, IO>), dim3(grid_for(nrows * M, bs)), dim3(bs), 0, s, dy + row0 * N,
                               a2, N, M, nrows, false);
            FC_HIP(hipGetLastError());
            rc = run_stages_fwd<float2>(fac_list(p), M, 1, a2, b2, p->st.w32, nrows, s, &xdy);
            if (rc) return rc;
            hipLaunchKernelGGL(k_accumulate_corr, dim3(grid_for(nrows * M, bs)), dim3(bs), 0, s, acc + h0 * M, xu, xdy, M,
                               nrows, b == 0);
            FC_HIP(hipGetLastError());
        }
    for (int64_t h0 = 0; h0 < H; h0 += chunk) {
        const int64_t nrows = H - h0 < chunk ? H - h0 : chunk;
        int rc = staged_inverse_to_dk(p, acc + h0 * M, a1, nrows, dk + h0 * Nk, Nk, s);
        if (rc) return rc;
    }
    return FFTCONV_OK;
}

int staged_backward_filter(const fftconv_plan *p, const void *u, const void *dy, float *dk, int64_t Nk, int64_t B,
                           void *workspace, hipStream_t s)
{
    switch (p->dtype) {
    case FFTCONV_F32:
        return staged_backward_filter_t<float>(p, (const float *)u, (const float *)dy, dk, Nk, B, workspace, s);
    case FFTCONV_F16:
        return staged_backward_filter_t<__half>(p, (const __half *)u, (const __half *)dy, dk, Nk, B, workspace, s);
    default:
        return staged_backward_filter_t<__hip_bfloat16>(p, (const __hip_bfloat16 *)u, (const __hip_bfloat16 *)dy, dk, Nk,
                                                        B, workspace, s);
    }
}

// Elementwise gate of the gated convolution for plans without a fused-gate kernel:
// out = a * b, the fp32 product rounded to the I/O dtype (exact product for 16-bit inputs).
template <typename T> __global__ void k_gate_multiply(const T *a, const T *b, T *out, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    if constexpr (std::is_same<T, float>::value)
        out[i] = a[i] * b[i];
    else if constexpr (std::is_same<T, __half>::value)
        out[i] = __float2half_rn(__half2float(a[i]) * __half2float(b[i]));
    else
        out[i] = __float2bfloat16(__bfloat162float(a[i]) * __bfloat162float(b[i]));
}

int gate_multiply(int dtype, const void *a, const void *b, void *out, int64_t n, hipStream_t s)
{
    const int bs = 256;
    const unsigned grid = (unsigned)((n + bs - 1) / bs);
    if (dtype == FFTCONV_F32)
        hipLaunchKernelGGL(k_gate_multiply<float>, dim3(grid), dim3(bs), 0, s, (const float *)a, (const float *)b,
                           (float *)out, n);
    else if (dtype == FFTCONV_F16)
        hipLaunchKernelGGL(k_gate_multiply<__half>, dim3(grid), dim3(bs), 0, s, (const __half *)a, (const __half *)b,
                           (__half *)out, n);
    else
        hipLaunchKernelGGL(k_gate_multiply<__hip_bfloat16>, dim3(grid), dim3(bs), 0, s, (const __hip_bfloat16 *)a,
                           (const __hip_bfloat16 *)b, (__hip_bfloat16 *)out, n);
    FC_HIP(hipGetLastError());
    return FFTCONV_OK;
}

}  // namespace fftconv
