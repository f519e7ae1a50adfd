// Multi-pass causal FFT convolution for transforms too long to keep on chip
// (paper Algorithm 4 and Section 3.1 "Kernel Fusion": the outermost matrix
// operation of the forward and of the inverse transform takes one trip through
// HBM each, everything inside stays fused).  16-bit I/O, fft_size M = No * Mi with
// Mi = 8192 (the fused inner transform) and No = M / Mi in [4, 512].
//
// Index maps: time n = no*Mi + r, frequency f = ko + No*f'.  Then
//   W_M^{n f} = W_No^{no ko} * W_M^{r ko} * W_Mi^{r f'},
// so, with z = u[b] + i*u[b+1] (two batch rows share one complex transform because the
// filter is real),
//   pass A:  S[ko, r] = W_M^{r ko} * sum_{no < No/2} z[no*Mi + r] W_No^{no ko}     (zeros for no >= No/2
//            are implicit; the listing in the paper omits the twiddle, its prose names it)
//   pass B:  every row S[ko, :] is circularly convolved (length Mi, complex in / complex out,
//            fused kernel) with the spectrum row k_f[ko + No*f'] / M
//   pass C:  y[no*Mi + r] = sum_{ko} conj(W_M^{r ko} W_No^{no ko}) S[ko, r],  no < No/2;
//            real part -> row b, imaginary part -> row b+1.
// S lives in the caller's workspace as 16-bit (re, im) pairs, M per pair of rows, and is
// rewritten in place by pass B.  The outer DFT of length No is itself split in two
// (No = Ra * Rb, Ra = min(16, No)) inside one workgroup, on the vector ALUs in fp32.
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>

#include "fftconv_internal.h"

namespace fftconv {

namespace {

constexpr int MI = 8192;
constexpr int TB = 256;          // threads per block of the outer passes

__device__ __forceinline__ float2 cmulf(float2 a, float2 b)
{
    return make_float2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x);
}
__device__ __forceinline__ float2 cmulcf(float2 a, float2 b)      // a * conj(b)
{
    return make_float2(a.x * b.x + a.y * b.y, a.y * b.x - a.x * b.y);
}
// exp(-2 pi i e / M) for 0 <= e < M <= 2^22 (e / M is exact in fp32)
__device__ __forceinline__ float2 wm(int e, float inv_half_m)
{
    float s, c;
    sincospif((float)e * inv_half_m, &s, &c);
    return make_float2(c, -s);
}

template <bool F16> __device__ __forceinline__ uint16_t cv16(float v)
{
    if constexpr (F16) {
        __half hv = __float2half_rn(v);
        return *(uint16_t *)&hv;
    } else {
        __hip_bfloat16 bv = __float2bfloat16(v);
        return *(uint16_t *)&bv;
    }
}
template <bool F16> __device__ __forceinline__ float2 unpack2(uint32_t w)
{
    if constexpr (F16) {
        __half2 hv = *(__half2 *)&w;
        return make_float2(__low2float(hv), __high2float(hv));
    } else {
        return make_float2(__uint_as_float(w << 16), __uint_as_float(w & 0xffff0000u));
    }
}

struct OuterGeo {
    int No, Ra, Rb, CT;          // outer length, its two factors, columns per block
};

// ---- pass A: zero-padded pair of real rows -> outer forward DFT -> twiddle -> S
template <bool F16>
__global__ void __launch_bounds__(TB) k_outer_fwd(const uint16_t *__restrict__ u, uint32_t *__restrict__ S,
                                                 OuterGeo g, int B, int H, int N, int64_t M)
{
    extern __shared__ float2 sm[];
    const int No = g.No, Ra = g.Ra, Rb = g.Rb, CT = g.CT;
    float2 *wno = sm;                              // W_No^j, j < No
    float2 *T = sm + No;                           // [No][CT]
    uint32_t *zin = (uint32_t *)(T + (size_t)No * CT);   // [No/2][CT] packed (row b, row b+1) 16-bit
    const int tid = threadIdx.x;
    const int c = tid % CT, grp = tid / CT, G = TB / CT;
    const int r0 = blockIdx.x * CT;
    const int ph = blockIdx.y;                     // pair * H + h
    const int pair = ph / H, h = ph % H;
    for (int j = tid; j < No; j += TB) wno[j] = wm(j, 2.0f / (float)No);
    const int half = No / 2;
    for (int e = tid; e < half * CT; e += TB) {
        const int no = e / CT, cc = e % CT;
        const int64_t n = (int64_t)no * MI + r0 + cc;
        uint32_t lo = 0, hi = 0;
        if (n < N) {
            const int b0 = 2 * pair;
            lo = u[((size_t)b0 * H + h) * N + n];
            if (b0 + 1 < B) hi = u[((size_t)(b0 + 1) * H + h) * N + n];
        }
        zin[e] = lo | (hi << 16);
    }
    __syncthreads();
    // step 1: T[ka*Rb + b2] = W_No^{ka b2} * sum_{a < Ra/2} z[a*Rb + b2] W_Ra^{a ka}
    for (int o = grp; o < No; o += G) {
        const int ka = o / Rb, b2 = o % Rb;
        float2 acc = make_float2(0.f, 0.f);
        int ph2 = 0;                               // (a * ka) mod Ra
        for (int a = 0; a < Ra / 2; ++a) {
            const float2 z = unpack2<F16>(zin[(a * Rb + b2) * CT + c]);   // (row b, row b+1) = (re, im)
            const float2 t = cmulf(z, wno[ph2 * Rb]);
            acc.x += t.x;
            acc.y += t.y;
            ph2 += ka;
            if (ph2 >= Ra) ph2 -= Ra;
        }
        T[o * CT + c] = cmulf(acc, wno[ka * b2]);
    }
    __syncthreads();
    // step 2: A[ka + Ra*kb] = sum_{b2} T[ka*Rb + b2] W_Rb^{b2 kb};  S = A * W_M^{r ko}
    const float ihm = 2.0f / (float)M;
    for (int o = grp; o < No; o += G) {
        const int ka = o % Ra, kb = o / Ra;        // o = ko
        float2 acc = make_float2(0.f, 0.f);
        int ph2 = 0;                               // (b2 * kb) mod Rb
        for (int b2 = 0; b2 < Rb; ++b2) {
            const float2 t = cmulf(T[(ka * Rb + b2) * CT + c], wno[ph2 * Ra]);
            acc.x += t.x;
            acc.y += t.y;
            ph2 += kb;
            if (ph2 >= Rb) ph2 -= Rb;
        }
        const int r = r0 + c;
        const int e = (int)(((int64_t)r * o) % M);
        acc = cmulf(acc, wm(e, ihm));
        S[((size_t)ph * No + o) * MI + r] = (uint32_t)cv16<F16>(acc.x) | ((uint32_t)cv16<F16>(acc.y) << 16);
    }
}

// ---- pass C: S -> conjugate twiddle -> outer inverse DFT -> the two real rows of the pair
template <bool F16>
__global__ void __launch_bounds__(TB) k_outer_inv(const uint32_t *__restrict__ S, uint16_t *__restrict__ y,
                                                 OuterGeo g, int B, int H, int N, int64_t M)
{
    extern __shared__ float2 sm[];
    const int No = g.No, Ra = g.Ra, Rb = g.Rb, CT = g.CT;
    float2 *wno = sm;
    float2 *X = sm + No;                           // [No][CT] twiddled input
    float2 *T = X + (size_t)No * CT;               // [No][CT]
    const int tid = threadIdx.x;
    const int c = tid % CT, grp = tid / CT, G = TB / CT;
    const int r0 = blockIdx.x * CT;
    const int ph = blockIdx.y;
    const int pair = ph / H, h = ph % H;
    for (int j = tid; j < No; j += TB) wno[j] = wm(j, 2.0f / (float)No);
    const float ihm = 2.0f / (float)M;
    for (int e = tid; e < No * CT; e += TB) {
        const int ko = e / CT, cc = e % CT;
        const int r = r0 + cc;
        const float2 v = unpack2<F16>(S[((size_t)ph * No + ko) * MI + r]);
        X[e] = cmulcf(v, wm((int)(((int64_t)r * ko) % M), ihm));
    }
    __syncthreads();
    // step 1: T[ka*Rb + b2] = conj(W_No^{ka b2}) * sum_{kb} X[ka + Ra*kb] conj(W_Rb^{b2 kb})
    for (int o = grp; o < No; o += G) {
        const int ka = o / Rb, b2 = o % Rb;
        float2 acc = make_float2(0.f, 0.f);
        int ph2 = 0;                               // (b2 * kb) mod Rb
        for (int kb = 0; kb < Rb; ++kb) {
            const float2 t = cmulcf(X[(ka + Ra * kb) * CT + c], wno[ph2 * Ra]);
            acc.x += t.x;
            acc.y += t.y;
            ph2 += b2;
            if (ph2 >= Rb) ph2 -= Rb;
        }
        T[o * CT + c] = cmulcf(acc, wno[ka * b2]);
    }
    __syncthreads();
    // step 2: z[a*Rb + b2] = sum_{ka} T[ka*Rb + b2] conj(W_Ra^{a ka}),  a < Ra/2 (n < M/2)
    for (int o = grp; o < No / 2; o += G) {        // o = no = a*Rb + b2
        const int a = o / Rb, b2 = o % Rb;
        float2 acc = make_float2(0.f, 0.f);
        int ph2 = 0;                               // (a * ka) mod Ra
        for (int ka = 0; ka < Ra; ++ka) {
            const float2 t = cmulcf(T[(ka * Rb + b2) * CT + c], wno[ph2 * Rb]);
            acc.x += t.x;
            acc.y += t.y;
            ph2 += a;
            if (ph2 >= Ra) ph2 -= Ra;
        }
        const int64_t n = (int64_t)o * MI + r0 + c;
        if (n < N) {
            const int b0 = 2 * pair;
            y[((size_t)b0 * H + h) * N + n] = cv16<F16>(acc.x);
            if (b0 + 1 < B) y[((size_t)(b0 + 1) * H + h) * N + n] = cv16<F16>(acc.y);
        }
    }
}

// k_f for the multi-pass path: [h][ko][inner order of f'] fp32 pairs, f = ko + No*f', scaled 1/M.
__global__ void k_pack_multipass(const double2 *spec, float2 *kf, FacList fl, int64_t M, int No, int64_t h0,
                                 int64_t nh, const uint8_t *keep, int64_t n_blocks)
{
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= nh * M) return;
    const int64_t h = idx / M, f = idx % M;
    const int ko = (int)(f % No);
    const int64_t fi = f / No;
    const double2 v = spec[h * M + freq_to_pos(f, fl, M)];
    const double sc = mask_weight(keep, n_blocks, f, M) / (double)M;
    kf[((h0 + h) * No + ko) * (int64_t)MI + fused3_kf_slot_8192(fi)] =
        make_float2((float)(v.x * sc), (float)(v.y * sc));
}

OuterGeo outer_geo(int64_t M)
{
    OuterGeo g;
    g.No = (int)(M / MI);
    g.Ra = g.No < 16 ? g.No : 16;
    g.Rb = g.No / g.Ra;
    g.CT = MI / g.No < TB ? MI / g.No : TB;      // No * CT <= 8192 points per block, at most one column per thread
    return g;
}

}  // namespace

bool multipass_supported(int64_t N, int64_t M, int dtype)
{
    if (dtype != FFTCONV_F16 && dtype != FFTCONV_BF16) return false;
    if (M < 4 * MI || M > 512 * (int64_t)MI) return false;
    return N <= M / 2;
}

int multipass_init(fftconv_plan *p) { return fused3_init_inner(p); }

size_t multipass_kf_bytes(const fftconv_plan *p) { return (size_t)(p->H * p->M) * sizeof(float2); }

size_t multipass_workspace_bytes(const fftconv_plan *p, int64_t B)
{
    const int64_t npairs = (B + 1) / 2;
    return (size_t)(npairs * p->H * p->M) * sizeof(uint32_t);
}

int multipass_pack_kf(const fftconv_plan *p, const double2 *spec, int64_t h0, int64_t nh, const uint8_t *keep_dev,
                      int64_t n_blocks, void *kf, hipStream_t s)
{
    const int bs = 256;
    const unsigned grid = (unsigned)((nh * p->M + bs - 1) / bs);
    hipLaunchKernelGGL(k_pack_multipass, dim3(grid), dim3(bs), 0, s, spec, (float2 *)kf, staged_fac_list(p), p->M,
                       (int)(p->M / MI), h0, nh, keep_dev, n_blocks);
    FC_HIP(hipGetLastError());
    return FFTCONV_OK;
}

int multipass_forward(const fftconv_plan *p, const void *u, const void *kf, void *y, int64_t B, void *workspace,
                      hipStream_t s)
{
    const OuterGeo g = outer_geo(p->M);
    const int64_t npairs = (B + 1) / 2;
    const int64_t rows = npairs * p->H;
    if (rows > 65535) {
        set_error("fftconv_forward: ceil(B/2) * H = %lld exceeds the multi-pass grid limit 65535", (long long)rows);
        return FFTCONV_EUNSUPPORTED;
    }
    const bool f16 = p->dtype == FFTCONV_F16;
    uint32_t *S = (uint32_t *)workspace;
    const dim3 grid((unsigned)(MI / g.CT), (unsigned)rows);
    const size_t lds_a = sizeof(float2) * (g.No + (size_t)g.No * g.CT) + sizeof(uint32_t) * (size_t)(g.No / 2) * g.CT;
    const size_t lds_c = sizeof(float2) * (g.No + 2 * (size_t)g.No * g.CT);
    static bool attr_set = false;
    if (!attr_set) {
        FC_HIP(hipFuncSetAttribute((const void *)k_outer_fwd<true>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        FC_HIP(hipFuncSetAttribute((const void *)k_outer_fwd<false>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        FC_HIP(hipFuncSetAttribute((const void *)k_outer_inv<true>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        FC_HIP(hipFuncSetAttribute((const void *)k_outer_inv<false>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        attr_set = true;
    }
    if (f16)
        hipLaunchKernelGGL(k_outer_fwd<true>, grid, dim3(TB), lds_a, s, (const uint16_t *)u, S, g, (int)B, (int)p->H,
                           (int)p->N, p->M);
    else
        hipLaunchKernelGGL(k_outer_fwd<false>, grid, dim3(TB), lds_a, s, (const uint16_t *)u, S, g, (int)B, (int)p->H,
                           (int)p->N, p->M);
    FC_HIP(hipGetLastError());
    int rc = fused3_inner_rows(p, S, kf, npairs, p->H * g.No, s);
    if (rc) return rc;
    if (f16)
        hipLaunchKernelGGL(k_outer_inv<true>, grid, dim3(TB), lds_c, s, S, (uint16_t *)y, g, (int)B, (int)p->H,
                           (int)p->N, p->M);
    else
        hipLaunchKernelGGL(k_outer_inv<false>, grid, dim3(TB), lds_c, s, S, (uint16_t *)y, g, (int)B, (int)p->H,
                           (int)p->N, p->M);
    FC_HIP(hipGetLastError());
    return FFTCONV_OK;
}

}  // namespace fftconv
