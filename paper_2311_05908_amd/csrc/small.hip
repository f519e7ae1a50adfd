// Fused FFT convolution for short transforms, fft_size M in {256, 512, 1024, 2048, 4096}, any I/O
// dtype, any N <= M (paper Section 2.1, Eq. 1; the fused single-kernel path of Section 3.1 for the
// short end of the paper's range).
//
// At these lengths the work per byte is small (O(log M) butterflies per point) and the path is bound
// by HBM, so it is not reshaped into matrix products: the transforms are radix-16/32 Cooley-Tukey
// passes on the vector ALUs in fp32 (in-register butterflies, dft_reg.h), in place in LDS, one HBM read of
// u and one HBM write of y.  fp32 arithmetic also serves fp32 I/O at its tolerance.
//  * Two batch rows of a channel share one complex transform, z = u[b] + i u[b+1] (real filter).
//  * A workgroup (256 threads) holds 4096 points = 4096/M pairs at a time, so every pass has 16 points
//    per thread whatever M is.
//  * Decimation in frequency forward, in place: after the passes with radices R0, R1, R2 position
//    p = k0 M/R0 + k1 M/(R0 R1) + k2 holds frequency f = k0 + R0 k1 + R0 R1 k2.  k_f is stored in that
//    order, the inverse runs the passes mirrored (decimation in time, conjugate twiddles) and lands in
//    natural time order: no permutation is executed.
//  * LDS index i is stored at i + i/16, so that the passes whose 16 points per thread are adjacent
//    (stride 1) and those whose threads are adjacent both spread over the banks.
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>

#include <type_traits>

#include "dft_reg.h"
#include "fftconv_internal.h"

namespace fftconv {

namespace {

constexpr int PTS = 4096;                     // points per workgroup pass
constexpr int NTS = 256;                      // threads
__device__ __forceinline__ int pad(int i) { return i + (i >> 4); }

template <typename IO> __device__ __forceinline__ float ld(const IO *p, int64_t i)
{
    if constexpr (std::is_same<IO, float>::value) return p[i];
    else if constexpr (std::is_same<IO, __half>::value) return __half2float(p[i]);
    else return __bfloat162float(p[i]);
}
template <typename IO> __device__ __forceinline__ void st(IO *p, int64_t i, float v)
{
    if constexpr (std::is_same<IO, float>::value) p[i] = v;
    else if constexpr (std::is_same<IO, __half>::value) p[i] = __float2half_rn(v);
    else p[i] = __float2bfloat16(v);
}
__device__ __forceinline__ float2 cmul2(float2 a, float2 b)
{
    return make_float2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x);
}
__device__ __forceinline__ float2 cmulc2(float2 a, float2 b)          // a * conj(b)
{
    return make_float2(a.x * b.x + a.y * b.y, a.y * b.x - a.x * b.y);
}

// One radix-R pass over all PTS points: blocks of length L (a divisor of M), sub-length Ls = L / R.
// Forward: y_k = W_L^{j k} sum_m x_m W_R^{m k} written back to slot k; inverse: the mirror image.
template <int R, bool INV>
__device__ __forceinline__ void radix_pass(float2 *z, const float2 *wt, int L, int wstride, int tid)
{
    const int Ls = L / R;
#pragma unroll 1
    for (int bi = tid; bi < PTS / R; bi += NTS) {
        const int blk = bi / Ls, j = bi - blk * Ls;
        const int base = blk * L + j;
        float2 x[R];
        if constexpr (!INV) {
#pragma unroll
            for (int m = 0; m < R; ++m) x[m] = z[pad(base + m * Ls)];
            dft_reg<R, false>(x);
#pragma unroll
            for (int k = 0; k < R; ++k) z[pad(base + k * Ls)] = (Ls == 1 || k == 0) ? x[k] : cmul2(x[k], wt[j * k * wstride]);
        } else {
#pragma unroll
            for (int k = 0; k < R; ++k) {
                const float2 v = z[pad(base + k * Ls)];
                x[k] = (Ls == 1 || k == 0) ? v : cmulc2(v, wt[j * k * wstride]);
            }
            dft_reg<R, true>(x);
#pragma unroll
            for (int m = 0; m < R; ++m) z[pad(base + m * Ls)] = x[m];
        }
    }
}

// The innermost pass of both directions in one go: blocks of R adjacent points; forward butterfly, product
// with k_f at the block's positions, inverse butterfly, written back in place (no twiddles at sub-length 1).
template <int R, int M>
__device__ __forceinline__ void middle_pass(float2 *z, const float2 *__restrict__ kf, const int *s_h, int tid)
{
#pragma unroll 1
    for (int bi = tid; bi < PTS / R; bi += NTS) {
        const int base = bi * R;
        const int slot = base / M, p = base - slot * M;
        const int h = s_h[slot];
        float2 x[R];
#pragma unroll
        for (int m = 0; m < R; ++m) x[m] = z[pad(base + m)];
        dft_reg<R, false>(x);
        if (h >= 0) {
            const float2 *kr = kf + (int64_t)h * M + p;
#pragma unroll
            for (int k = 0; k < R; ++k) x[k] = cmul2(x[k], kr[k]);
        }
        dft_reg<R, true>(x);
#pragma unroll
        for (int m = 0; m < R; ++m) z[pad(base + m)] = x[m];
    }
}

// kf: [h][position] fp32 pairs, scaled by 1/M; wtab: W_M^t, t < M.
template <int M, int R0, int R1, int R2, typename IO>
__global__ void __launch_bounds__(NTS) k_small(const IO *__restrict__ u, IO *__restrict__ y,
                                              const float2 *__restrict__ kf, const float2 *__restrict__ wtab, int B,
                                              int H, int N)
{
    static_assert(R0 * R1 * R2 == M, "radices must multiply to the transform length");
    constexpr int P = PTS / M;                                    // pairs per workgroup pass
    extern __shared__ float2 smem_small[];
    float2 *const z = smem_small;                                 // [PTS + PTS / 16]
    float2 *const wt = smem_small + PTS + PTS / 16;               // [M]
    __shared__ int s_h[P], s_pair[P];                             // channel and pair of each slot (-1: no work)
    const int tid = threadIdx.x;
    for (int t = tid; t < M; t += NTS) wt[t] = wtab[t];
    const int npairs = (B + 1) / 2;
    const long long T = (long long)H * npairs;                    // work items t = h * npairs + pair
    const long long groups = (T + P - 1) / P;
    // 16-byte accesses of 8 (16-bit) or 4 (fp32) consecutive samples when the rows allow it
    constexpr int VEC = sizeof(IO) == 2 ? 8 : 4;
    const bool vec_ok = (N % VEC == 0) && ((((uintptr_t)u | (uintptr_t)y) & 15) == 0);
    for (long long g = blockIdx.x; g < groups; g += gridDim.x) {
        __syncthreads();                                          // z and the slot table are free again (and wt is loaded)
        if (tid < P) {
            const long long t = g * P + tid;
            const int h = t < T ? (int)(t / npairs) : -1;
            s_h[tid] = h;
            s_pair[tid] = t < T ? (int)(t - (long long)h * npairs) : -1;
        }
        __syncthreads();
        // ---- load: point i = pair slot i / M, sample n = i % M; zeros for n >= N and for a missing row
        if (vec_ok) {
#pragma unroll
            for (int c = tid; c < PTS / VEC; c += NTS) {
                const int i = c * VEC, slot = i / M, n = i - slot * M;
                const int h = s_h[slot], pair = s_pair[slot];
                float re[VEC], im[VEC];
#pragma unroll
                for (int e = 0; e < VEC; ++e) re[e] = im[e] = 0.f;
                if (h >= 0 && n < N) {
                    const int64_t row = ((int64_t)(2 * pair) * H + h) * N + n;
                    const uint4 a = *(const uint4 *)(u + row);
                    uint4 b4 = make_uint4(0, 0, 0, 0);
                    if (2 * pair + 1 < B) b4 = *(const uint4 *)(u + row + (int64_t)H * N);
                    alignas(16) IO ta[VEC], tb[VEC];
                    *(uint4 *)ta = a;
                    *(uint4 *)tb = b4;
#pragma unroll
                    for (int e = 0; e < VEC; ++e) {
                        re[e] = ld(ta, e);
                        im[e] = ld(tb, e);
                    }
                }
#pragma unroll
                for (int e = 0; e < VEC; ++e) z[pad(i) + e] = make_float2(re[e], im[e]);
            }
        } else {
#pragma unroll 4
            for (int i = tid; i < PTS; i += NTS) {
                const int slot = i / M, n = i - slot * M;
                const int h = s_h[slot], pair = s_pair[slot];
                float2 v = make_float2(0.f, 0.f);
                if (h >= 0 && n < N) {
                    const int64_t row = ((int64_t)(2 * pair) * H + h) * N;
                    v.x = ld(u, row + n);
                    if (2 * pair + 1 < B) v.y = ld(u, row + (int64_t)H * N + n);
                }
                z[pad(i)] = v;
            }
        }
        __syncthreads();
        // ---- forward passes (decimation in frequency), the innermost pass of both directions fused
        //      with the product by k_f[h], inverse passes mirrored
        radix_pass<R0, false>(z, wt, M, 1, tid);
        __syncthreads();
        if constexpr (R2 > 1) {
            radix_pass<R1, false>(z, wt, M / R0, R0, tid);
            __syncthreads();
            middle_pass<R2, M>(z, kf, s_h, tid);
            __syncthreads();
            radix_pass<R1, true>(z, wt, M / R0, R0, tid);
            __syncthreads();
        } else {
            middle_pass<R1, M>(z, kf, s_h, tid);
            __syncthreads();
        }
        radix_pass<R0, true>(z, wt, M, 1, tid);
        __syncthreads();
        // ---- store: real part -> row b, imaginary part -> row b+1
        if (vec_ok) {
#pragma unroll
            for (int c = tid; c < PTS / VEC; c += NTS) {
                const int i = c * VEC, slot = i / M, n = i - slot * M;
                const int h = s_h[slot], pair = s_pair[slot];
                if (h >= 0 && n < N) {
                    alignas(16) IO ta[VEC], tb[VEC];
#pragma unroll
                    for (int e = 0; e < VEC; ++e) {
                        const float2 v = z[pad(i) + e];
                        st(ta, e, v.x);
                        st(tb, e, v.y);
                    }
                    const int64_t row = ((int64_t)(2 * pair) * H + h) * N + n;
                    *(uint4 *)(y + row) = *(const uint4 *)ta;
                    if (2 * pair + 1 < B) *(uint4 *)(y + row + (int64_t)H * N) = *(const uint4 *)tb;
                }
            }
        } else {
#pragma unroll 4
            for (int i = tid; i < PTS; i += NTS) {
                const int slot = i / M, n = i - slot * M;
                const int h = s_h[slot], pair = s_pair[slot];
                if (h >= 0 && n < N) {
                    const int64_t row = ((int64_t)(2 * pair) * H + h) * N;
                    const float2 v = z[pad(i)];
                    st(y, row + n, v.x);
                    if (2 * pair + 1 < B) st(y, row + (int64_t)H * N + n, v.y);
                }
            }
        }
    }
}

struct Radices { int r0, r1, r2; };
__host__ __device__ inline Radices small_radices(int64_t M)
{
    switch (M) {
    case 256: return {16, 16, 1};
    case 512: return {32, 16, 1};
    case 1024: return {32, 32, 1};
    case 2048: return {16, 16, 8};
    default: return {16, 16, 16};
    }
}

// position of frequency f after the forward passes (see the head of this file)
__host__ __device__ inline int64_t small_pos(int64_t f, int64_t M)
{
    const Radices r = small_radices(M);
    const int64_t k0 = f % r.r0, k1 = (f / r.r0) % r.r1, k2 = f / ((int64_t)r.r0 * r.r1);
    return k0 * (M / r.r0) + k1 * (M / ((int64_t)r.r0 * r.r1)) + k2;
}

__global__ void k_pack_small(const double2 *spec, float2 *kf, FacList fl, int64_t M, int64_t h0, int64_t nh,
                             const uint8_t *keep, int64_t n_blocks)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= nh * M) return;
    const int64_t h = idx / M, f = idx % M;
    const double2 v = spec[h * M + freq_to_pos(f, fl, M)];
    const double sc = mask_weight(keep, n_blocks, f, M) / (double)M;
    kf[(h0 + h) * M + small_pos(f, M)] = make_float2((float)(v.x * sc), (float)(v.y * sc));
}

template <int M, int R0, int R1, int R2, typename IO>
int launch_small(const fftconv_plan *p, const void *u, const void *kf, void *y, int64_t B, hipStream_t s)
{
    const int64_t T = p->H * ((B + 1) / 2);
    const int64_t groups = (T + PTS / M - 1) / (PTS / M);
    // a few workgroups per compute unit (LDS: 34 KB + the twiddle table), each looping over its groups
    const int64_t cap = (int64_t)p->f3.num_cu * 4;
    const unsigned grid = (unsigned)(groups < cap ? groups : cap);
    constexpr size_t lds = sizeof(float2) * (PTS + PTS / 16 + M);
    FC_TRY(raise_dynamic_lds((const void *)k_small<M, R0, R1, R2, IO>, (int)lds));
    hipLaunchKernelGGL((k_small<M, R0, R1, R2, IO>), dim3(grid), dim3(NTS), lds, s, (const IO *)u, (IO *)y,
                       (const float2 *)kf, (const float2 *)p->st.w32, (int)B, (int)p->H, (int)p->N);
    FC_HIP(hipGetLastError());
    return FFTCONV_OK;
}

template <typename IO> int dispatch_small(const fftconv_plan *p, const void *u, const void *kf, void *y, int64_t B, hipStream_t s)
{
    switch (p->M) {
    case 256: return launch_small<256, 16, 16, 1, IO>(p, u, kf, y, B, s);
    case 512: return launch_small<512, 32, 16, 1, IO>(p, u, kf, y, B, s);
    case 1024: return launch_small<1024, 32, 32, 1, IO>(p, u, kf, y, B, s);
    case 2048: return launch_small<2048, 16, 16, 8, IO>(p, u, kf, y, B, s);
    case 4096: return launch_small<4096, 16, 16, 16, IO>(p, u, kf, y, B, s);
    default:
        set_error("small-transform kernel: no instance for fft_size=%lld", (long long)p->M);
        return FFTCONV_EUNSUPPORTED;
    }
}

}  // namespace

FacList small_factor_list(int64_t M)
{
    const Radices r = small_radices(M);
    FacList fl;
    for (int i = 0; i < MAX_FACTORS; ++i) fl.fac[i] = 0;
    fl.fac[0] = r.r0;
    fl.fac[1] = r.r1;
    fl.fac[2] = r.r2;
    fl.nf = r.r2 > 1 ? 3 : 2;
    return fl;
}

bool small_supported(int64_t N, int64_t M, int dtype)
{
    (void)dtype;
    return M >= 256 && M <= 4096 && N <= M;
}

int small_init(fftconv_plan *p)
{
    hipDeviceProp_t prop;
    FC_HIP(hipGetDeviceProperties(&prop, p->device));
    p->f3.num_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    const Radices r = small_radices(p->M);
    p->f3.N1 = r.r0;
    p->f3.N2 = r.r1;
    p->f3.N3 = r.r2;
    return FFTCONV_OK;
}

size_t small_kf_bytes(const fftconv_plan *p) { return (size_t)(p->H * p->M) * sizeof(float2); }

int small_pack_kf(const fftconv_plan *p, const double2 *spec, int64_t h0, int64_t nh, const uint8_t *keep_dev,
                  int64_t n_blocks, void *kf, hipStream_t s)
{
    const int bs = 256;
    const unsigned grid = (unsigned)((nh * p->M + bs - 1) / bs);
    hipLaunchKernelGGL(k_pack_small, dim3(grid), dim3(bs), 0, s, spec, (float2 *)kf, staged_fac_list(p), p->M, h0, nh,
                       keep_dev, n_blocks);
    FC_HIP(hipGetLastError());
    return FFTCONV_OK;
}

int small_forward(const fftconv_plan *p, const void *u, const void *kf, void *y, int64_t B, hipStream_t s)
{
    if ((int64_t)((B + 1) / 2) * p->H >= ((int64_t)1 << 40)) {
        set_error("fftconv_forward: too many sequences for the small-transform kernel");
        return FFTCONV_EUNSUPPORTED;
    }
    switch (p->dtype) {
    case FFTCONV_F32: return dispatch_small<float>(p, u, kf, y, B, s);
    case FFTCONV_F16: return dispatch_small<__half>(p, u, kf, y, B, s);
    default: return dispatch_small<__hip_bfloat16>(p, u, kf, y, B, s);
    }
}

}  // namespace fftconv
