// Fused causal FFT convolution for 16-bit I/O, fft_size M = N1*N2*N3 with N1 = 32
// (paper Algorithm 3: order-3 decomposition, whole sequence on chip, one HBM read
// of u and one HBM write of y).  gfx950 only.
//
// What is different from the paper's kernel, and why
//  * Two batch rows that share a channel are transformed together as one complex
//    sequence z = u[b] + i*u[b+1].  The filter is real, so
//    iFFT(FFT(z) . k_f) = conv(u[b],k) + i*conv(u[b+1],k): one complex transform
//    serves two sequences and no spectrum unpacking is needed.  This plays the role
//    of the paper's real-FFT trick (Section 3.1 "Domain-Specific Optimizations",
//    Appendix A.1): it halves the transform work per sequence.
//  * Implicit zero padding (Section 3.1): only the n1 < N1/2 half of the outermost
//    DFT matrix is multiplied in the forward transform and only the n1 < N1/2 output
//    rows (real and imaginary part = the two sequences) are formed in the inverse.
//  * Every DFT-matrix product is a v_mfma_f32_16x16x32 (bf16 or f16 operands, fp32
//    accumulate).  A complex Nx16 * 16x16 product is the real product
//    [Xr Xi] * [[Gr Gi], [-Gi Gr]] with K = 32.
//  * Stage-to-stage hand-off without a transpose (the paper's accumulator ->
//    matrix_a reuse, Appendix A.2): an MFMA result leaves each lane with 4
//    consecutive rows of one column; the next contraction runs over exactly those
//    rows, and since a contraction does not care about the order of K, the constant
//    matrix is stored with its K axis permuted to (4 rows) x (re, im) per lane.
//    Only two exchanges per pair go through LDS (before the innermost forward
//    stage and before the outermost inverse stage), both as packed 16-bit pairs.
//  * Twiddles that depend only on (contracted index, output index, tile constant)
//    are folded into per-tile DFT matrices; the others are fp32 multiplies on the
//    accumulators.
//
// Index maps (time n = (n1*N2 + n2)*N3 + n3, frequency f = k1 + N1*k2 + N1*N2*k3):
//   forward  A1[k1,n2,n3] = sum_{n1<N1/2} z[n1,n2,n3] W_N1^{n1 k1}
//            A1 *= W_M^{k1 (N3 n2 + n3)}
//            A2[k1,k2,n3] = sum_{n2} A1 W_N2^{n2 k2} W_{N2 N3}^{k2 n3}     (folded)
//            A3[k1,k2,k3] = sum_{n3} A2 W_N3^{n3 k3};   A3 *= k_f[k1,k2,k3]
//   inverse  B3[k1,k2,n3] = sum_{k3} A3 conj(W_N3^{k3 n3})
//            B3 *= conj(W_M^{(k1 + N1 k2) n3})
//            B2[k1,n2,n3] = sum_{k2} B3 conj(W_N2^{k2 n2} W_{N1 N2}^{k1 n2})  (folded)
//            y[n1,n2,n3]  = sum_{k1} B2 conj(W_N1^{k1 n1}),  n1 < N1/2
// Work split of a 512-thread workgroup (8 waves) on one work item:
//   phase A (per n3):  stage 1, twiddle, stage 2      -> LDS[k1,k2,n3]
//   phase B (per k1):  stage 3, k_f, inverse 3, twiddle, inverse 2 -> LDS in place
//   phase C (per n3):  inverse stage 1                -> HBM
// This file holds what the kernels of this family share on the host side: the per-lane operand tables, the
// filter transforms, the overlap-save route of short filters and the dispatch.  The kernels themselves:
// fused3_ws.hip (fft 8192 and the grouped shorter transforms), fused3_wsc.hip (complex rows of length 8192,
// the inner step of the multi-pass scheme), fused3_big.hip (fft 16384 and 32768).
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <vector>

#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>

#include <type_traits>

#include "fused3_common.h"
#include "lds_fft.h"

namespace fftconv {

namespace {

using namespace f3;

// Filter transform of the plans that run on the 8192-point kernel, one workgroup per channel and no
// intermediate in HBM: taps -> LDS (zero padded, fp32), forward transform of length Ms = 8192 / groups in
// LDS (the stages of the generic path, lds_fft.h; fp32 is ample for constants that are rounded to 16 bits),
// then k_f[h] in the kernel's per-lane order, scaled by 1/Ms:
//   slot d = (k1 * 4 + r) * 64 + lane holds k2 = lane % 16, k3 = k3_at_index(4 (lane / 16) + r), as 16-bit
//   constant pairs for TT::ctw (fmt 1: bf16 dot-product form, fmt 2: fp16 packed form).
// groups > 1: slot (k1, k2, k3) takes bin k1 % N1s + N1s (k2 + 16 k3) of the short spectrum, N1s = 32 / groups
// (the same spectrum for every group), see build_tables().  reversed: see the adjoint filter transform.
constexpr int FILT_THREADS = 512;
__global__ void __launch_bounds__(FILT_THREADS) k_filter_fused3(const float *__restrict__ k, uint2 *__restrict__ kf,
                                                               const float2 *__restrict__ w, FacList fl, int64_t Nk,
                                                               int tws, bool reversed, const uint8_t *__restrict__ keep,
                                                               int64_t n_blocks, int fmt, int groups)
{
    extern __shared__ float2 XF[];
    constexpr int M = 8192;
    const int Ms = M / groups, N1s = N1 / groups;
    const int64_t h = blockIdx.x;
    // all taps of the thread are requested before the first is used (a tap beyond Nk reads tap 0 and is discarded:
    // behind a branch every load would be waited for in turn)
    constexpr int TPT = M / FILT_THREADS;
    float tap[TPT];
#pragma unroll
    for (int j = 0; j < TPT; ++j) {
        const int n = threadIdx.x + j * FILT_THREADS;
        const int t = (reversed && n != 0) ? Ms - n : n;
        tap[j] = k[h * Nk + ((n < Ms && t < Nk) ? t : 0)];
    }
#pragma unroll
    for (int j = 0; j < TPT; ++j) asm volatile("" ::"v"(tap[j]));
#pragma unroll
    for (int j = 0; j < TPT; ++j) {
        const int n = threadIdx.x + j * FILT_THREADS;
        const int t = (reversed && n != 0) ? Ms - n : n;
        if (n < Ms) XF[lds_slot(n)] = make_float2(t < Nk ? tap[j] : 0.f, 0.f);
    }
    __syncthreads();
    lds_forward(XF, w, fl, Ms, tws);
    for (int d = threadIdx.x; d < M; d += FILT_THREADS) {
        const int lane = d % 64, r = (d / 64) % 4, k1 = d / 256;
        const int k2 = lane % 16, k3 = k3_at_index(4 * (lane / 16) + r, 16);
        const int fs = (k1 % N1s) + N1s * (k2 + 16 * k3);                      // bin of the (sub-)transform
        const float2 v = XF[lds_slot(lds_pos(fs, fl, Ms))];
        const double sc = (double)lds_mask_weight(keep, n_blocks, fs, Ms) / (double)Ms;
        uint2 c;
        if (fmt == 1)
            c = ctw_const(v.x * sc, v.y * sc, 1, [](double x) {
                __hip_bfloat16 b = __float2bfloat16((float)x);
                return *(uint16_t *)&b;
            });
        else
            c = ctw_const(v.x * sc, v.y * sc, 2, [](double x) {
                __half hv = __float2half_rn((float)x);
                return *(uint16_t *)&hv;
            });
        kf[h * M + d] = c;
    }
}

// ---------------------------------------------------------------- host side

uint16_t to_bf16(double x)
{
    float f = (float)x;
    uint32_t b;
    std::memcpy(&b, &f, 4);
    b += 0x7fffu + ((b >> 16) & 1u);       // round to nearest even (finite inputs only)
    return (uint16_t)(b >> 16);
}
uint16_t to_f16(double x)
{
    _Float16 hv = (_Float16)(float)x;
    uint16_t b;
    std::memcpy(&b, &hv, 2);
    return b;
}

struct Cplx { double re, im; };
Cplx wpow(int64_t M, int64_t e)             // exp(-2 pi i e / M)
{
    const double two_pi = 6.283185307179586476925286766559;
    e %= M;
    if (e < 0) e += M;
    double a = two_pi * (double)e / (double)M;
    return {std::cos(a), -std::sin(a)};
}
Cplx cmulh(Cplx a, Cplx b) { return {a.re * b.re - a.im * b.im, a.re * b.im + a.im * b.re}; }
Cplx conjh(Cplx a) { return {a.re, -a.im}; }

// One MFMA operand (64 lanes x 8 16-bit slots) of the real form of a complex matrix G:
// lane (c16, q), slot 2r+s multiplies data element e_in = 16 t + 4 q + r, part s (0 = re, 1 = im),
// and contributes to output e_out = 16 ct + c16, part `part`.
template <typename Fn>
void fill_operand(uint16_t *dst, bool f16, int t, int ct, int part, Fn G)
{
    for (int lane = 0; lane < 64; ++lane) {
        int c16 = lane % 16, q = lane / 16;
        for (int r = 0; r < 4; ++r) {
            Cplx g = G(16 * t + 4 * q + r, 16 * ct + c16);
            double v0 = part == 0 ? g.re : g.im;     // multiplies the real part of the data
            double v1 = part == 0 ? -g.im : g.re;    // multiplies the imaginary part
            dst[lane * 8 + 2 * r + 0] = f16 ? to_f16(v0) : to_bf16(v0);
            dst[lane * 8 + 2 * r + 1] = f16 ? to_f16(v1) : to_bf16(v1);
        }
    }
}

// groups > 1 (N2 = N3 = 16 only): the tables of `groups` independent transforms of length Ms = 8192 / groups
// = N1s * 16 * 16 (N1s = 32 / groups) that share one pass of the 8192-point kernel.  The outermost stage
// becomes block diagonal: input rows n1 < 16 are the causal halves (N1s / 2 rows each) of the groups,
// output k1 = g * N1s + k1' is frequency digit k1' of group g; the twiddles and the folded stage-2 inverse
// matrices are those of a length-Ms transform; stages 2 and 3 do not change (N2 N3 = 256 either way).
// groups = 32 (fft 256 = 1 * 16 * 16): the outer factor is 1 and a row n1 of the input slot holds the causal
// halves of two groups, group 2 n1 in n2 < 8 and group 2 n1 + 1 in n2 >= 8.  Stage 1 copies the row to both
// planes k1 = 2 n1, 2 n1 + 1, the elementwise twiddle zeroes the other group's half, and each plane runs its own
// circular transform of length 256: the odd group works in a frame shifted by 128 samples, where its N <= 128
// outputs still depend only on inputs at or before them.  The per-plane inverse stage-2 matrices keep only the
// plane's own half of n2, so that inverse stage 1 (a sum over the two planes) reassembles the row.
template <int N2, int N3>
int build_tables(fftconv_plan *p, void **dest, int groups = 1)
{
    using G = Geo<N2, N3>;
    constexpr int64_t M = G::M;
    const int N1s = N1 / groups, H1 = N1s / 2;                  // sub-transform: outer factor, its causal half
    const int64_t Ms = M / groups;
    const bool halves = groups == N1;                            // two groups per input row
    auto g_of_k1 = [&](int k1) { return halves ? k1 / 2 : k1 / N1s; };          // (row of the pair of groups when halves)
    auto g_of_n1 = [&](int n1) { return groups == 1 ? 0 : halves ? n1 : n1 / H1; };   // n1 < 16 when groups > 1
    auto sub_n1 = [&](int n1) { return groups == 1 ? n1 : halves ? 0 : n1 % H1; };
    auto own_half = [&](int k1, int n2) { return !halves || ((n2 >= N2 / 2) == ((k1 & 1) != 0)); };
    const Cplx zero_c = {0.0, 0.0};
    const bool f16 = p->dtype == FFTCONV_F16;
    const size_t n_u4 = (size_t)G::TAB1 + G::TAB2 + 2 * (size_t)G::TAB3 + G::TAB2I + G::TAB1I;
    const size_t n_f2 = (size_t)G::TWA + G::TWB;
    std::vector<uint16_t> ops(n_u4 * 8);
    std::vector<float2> tw(n_f2);
    std::vector<uint2> tw16(n_f2);
    const int cfmt = f16 ? 2 : 1;
    auto hi16 = [&](double v) { return f16 ? to_f16(v) : to_bf16(v); };
    size_t o = 0;
    auto next = [&]() { uint16_t *d = ops.data() + o * 8; o += 64; return d; };
    // tab1 [K step][ct][part]: W_N1^{n1 k1}; zero-padded real input only meets K step 0 (n1 < 16)
    for (int ks = 0; ks < 2; ++ks)
        for (int ct = 0; ct < 2; ++ct)
            for (int part = 0; part < 2; ++part)
                fill_operand(next(), f16, ks, ct, part, [&](int n1, int k1) {
                    if (groups > 1 && (n1 >= 16 || g_of_n1(n1) != g_of_k1(k1))) return zero_c;
                    return wpow(N1s, (int64_t)sub_n1(n1) * (k1 % N1s));
                });
    // tab2 [n3][t][ct][part]: W_N2^{n2 k2} W_{N2 N3}^{k2 n3}
    for (int n3 = 0; n3 < N3; ++n3)
        for (int t = 0; t < G::R2; ++t)
            for (int ct = 0; ct < G::R2; ++ct)
                for (int part = 0; part < 2; ++part)
                    fill_operand(next(), f16, t, ct, part, [&](int n2, int k2) {
                        return cmulh(wpow(N2, (int64_t)n2 * k2), wpow((int64_t)N2 * N3, (int64_t)k2 * n3));
                    });
    // tab3 [t][ct][part]: W_N3^{n3 k3}, output rows in the k3 order of k3_at_index()
    for (int t = 0; t < G::R3; ++t)
        for (int ct = 0; ct < G::R3; ++ct)
            for (int part = 0; part < 2; ++part)
                fill_operand(next(), f16, t, ct, part,
                             [&](int n3, int idx) { return wpow(N3, (int64_t)n3 * k3_at_index(idx, N3)); });
    // tab3i: conj(W_N3^{k3 n3}), contraction slots in the same k3 order
    for (int t = 0; t < G::R3; ++t)
        for (int ct = 0; ct < G::R3; ++ct)
            for (int part = 0; part < 2; ++part)
                fill_operand(next(), f16, t, ct, part,
                             [&](int idx, int n3) { return conjh(wpow(N3, (int64_t)n3 * k3_at_index(idx, N3))); });
    // tab2i [k1][t][ct][part]: conj(W_N2^{k2 n2} W_{N1 N2}^{k1 n2})
    for (int k1 = 0; k1 < N1; ++k1)
        for (int t = 0; t < G::R2; ++t)
            for (int ct = 0; ct < G::R2; ++ct)
                for (int part = 0; part < 2; ++part)
                    fill_operand(next(), f16, t, ct, part, [&](int k2, int n2) {
                        if (!own_half(k1, n2)) return zero_c;
                        return conjh(cmulh(wpow(N2, (int64_t)n2 * k2), wpow((int64_t)N1s * N2, (int64_t)(k1 % N1s) * n2)));
                    });
    // tab1i [K step][row tile][part]: conj(W_N1^{k1 n1}); the causal kernel only forms row tile 0 (n1 < 16)
    for (int t = 0; t < 2; ++t)
        for (int rt = 0; rt < 2; ++rt)
            for (int part = 0; part < 2; ++part)
                fill_operand(next(), f16, t, rt, part, [&](int k1, int n1) {
                    if (groups > 1 && (n1 >= 16 || g_of_n1(n1) != g_of_k1(k1))) return zero_c;
                    return conjh(wpow(N1s, (int64_t)sub_n1(n1) * (k1 % N1s)));
                });
    if (o != n_u4) {
        set_error("fused3: operand table size mismatch");
        return FFTCONV_EINVAL;
    }
    // twa [n3][rt][ct][r][lane]: W_M^{k1 (N3 n2 + n3)}, k1 = 16 ct + c16, n2 = 16 rt + 4 q + r
    size_t w = 0;
    for (int n3 = 0; n3 < N3; ++n3)
        for (int rt = 0; rt < G::R2; ++rt)
            for (int ct = 0; ct < 2; ++ct)
                for (int r = 0; r < 4; ++r)
                    for (int lane = 0; lane < 64; ++lane) {
                        int k1 = 16 * ct + lane % 16, n2 = 16 * rt + 4 * (lane / 16) + r;
                        Cplx v = own_half(k1, n2) ? wpow(Ms, (int64_t)(k1 % N1s) * ((int64_t)N3 * n2 + n3)) : zero_c;
                        tw16[w] = ctw_const(v.re, v.im, cfmt, hi16);
                        tw[w++] = make_float2((float)v.re, (float)v.im);
                    }
    // twb [k1][ct2][ct3][r][lane]: conj(W_M^{(k1 + N1 k2) n3}), n3 = 16 ct3 + c16, k2 = 16 ct2 + 4 q + r
    for (int k1 = 0; k1 < N1; ++k1)
        for (int ct2 = 0; ct2 < G::R2; ++ct2)
            for (int ct3 = 0; ct3 < G::R3; ++ct3)
                for (int r = 0; r < 4; ++r)
                    for (int lane = 0; lane < 64; ++lane) {
                        int n3 = 16 * ct3 + lane % 16, k2 = 16 * ct2 + 4 * (lane / 16) + r;
                        Cplx v = conjh(wpow(Ms, ((int64_t)(k1 % N1s) + (int64_t)N1s * k2) * n3));
                        tw16[w] = ctw_const(v.re, v.im, cfmt, hi16);
                        tw[w++] = make_float2((float)v.re, (float)v.im);
                    }
    const size_t bytes = n_u4 * 16 + 2 * n_f2 * 8;
    FC_HIP(hipMalloc(dest, bytes));
    p->f3.consts_bytes += bytes;
    FC_HIP(hipMemcpy(*dest, ops.data(), n_u4 * 16, hipMemcpyHostToDevice));
    FC_HIP(hipMemcpy((char *)*dest + n_u4 * 16, tw.data(), n_f2 * 8, hipMemcpyHostToDevice));
    FC_HIP(hipMemcpy((char *)*dest + n_u4 * 16 + n_f2 * 8, tw16.data(), n_f2 * 8, hipMemcpyHostToDevice));
    return FFTCONV_OK;
}

}  // namespace

bool fused3_supported(int64_t N, int64_t M, int dtype)
{
    if (dtype != FFTCONV_F16 && dtype != FFTCONV_BF16) return false;
    // 256 .. 4096: 8192 / fft_size transforms share one pass of the 8192-point kernel
    if (M != 256 && M != 512 && M != 1024 && M != 2048 && M != 4096 && M != 8192 && M != 16384 && M != 32768) return false;
    return N <= M / 2 && N % 8 == 0;
}

int fused3_init(fftconv_plan *p)
{
    p->f3.N1 = N1;
    hipDeviceProp_t prop;
    FC_HIP(hipGetDeviceProperties(&prop, p->device));
    p->f3.num_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    switch (p->M) {
    case 256:
    case 512:
    case 1024:
    case 2048:
    case 4096:
        p->f3.N1 = (int)(p->M / 256);
        p->f3.N2 = 16;
        p->f3.N3 = 16;
        return build_tables<16, 16>(p, &p->f3.consts, (int)(8192 / p->M));
    case 8192:
        p->f3.N2 = 16;
        p->f3.N3 = 16;
        return build_tables<16, 16>(p, &p->f3.consts);
    case 16384: {
        // 32 * 16 * 32 on the streamed-table kernel of fused3_big.hip: the per-plane stage-2 matrices are then
        // 16 x 16 (a quarter of the bytes of a 32 * 32 * 16 split)
        p->f3.N2 = 16;
        p->f3.N3 = 32;
        int rc = fused3_big_init(p);
        if (rc) return rc;
        return fused3_init_short(p);                             // for partial convolutions, see fused3_forward_short
    }
    case 32768: {
        p->f3.N2 = 32;
        p->f3.N3 = 32;
        int rc = fused3_big_init(p);
        if (rc) return rc;
        return fused3_init_short(p);
    }
    default:
        set_error("fused3: no kernel for fft_size=%lld", (long long)p->M);
        return FFTCONV_EUNSUPPORTED;
    }
}

// Frequency-sparse filter (Appendix A.4): live_k3 / live_k1 have a bit set for every value of the digit that
// can meet a non-zero bin of k_f.  The kernels for 16384 and 32768 skip the tile of the innermost digit k3, and
// (32768) of the middle digit k2, that only meets zeroed bins, and the k1 planes that are not live; the 8192
// kernel skips the k1 planes that are not live (the trip count of its per-plane loop).
int fused3_forward_sparse(const fftconv_plan *p, const void *u, const void *kf, void *y, int64_t B, uint32_t live_k3,
                          hipStream_t s, uint32_t live_k1, uint32_t live_k2)
{
    if (p->M == 16384 || p->M == 32768) {
        if (((uintptr_t)u | (uintptr_t)y) & 15) {
            set_error("fftconv_forward_freq_sparse: u and y must be 16-byte aligned for this plan");
            return FFTCONV_EINVAL;
        }
        return fused3_big_forward(p, u, kf, y, B, live_k3, s, live_k2, live_k1);
    }
    if (p->M == 8192 && live_k1 != 0xffffffffu) {
        if (((uintptr_t)u | (uintptr_t)y) & 15) {
            set_error("fftconv_forward_freq_sparse: u and y must be 16-byte aligned for this plan");
            return FFTCONV_EINVAL;
        }
        return fused3_ws_launch(p, p->f3.consts, u, kf, y, B, 1, 0, s, nullptr, nullptr, live_k1);
    }
    return fused3_forward(p, u, kf, y, B, s);
}

// Which values of the most significant frequency digit k3 (f = k1 + 32 k2 + 32 N2 k3) can meet a
// non-zero bin under a block mask: bit k3 of the result.  Mirror bins count: two real rows share
// one complex transform, so a bin keeps weight 1/2 when only its mirror image M - f is kept.
uint32_t fused3_live_k3(const fftconv_plan *p, const uint8_t *block_keep, int64_t n_blocks)
{
    const int N3 = p->f3.N3;
    const int64_t per_row = p->M / N3, per_blk = p->M / n_blocks;
    uint32_t live = 0;
    for (int k3 = 0; k3 < N3; ++k3) {
        bool kept = false;
        for (int side = 0; side < 2 && !kept; ++side) {
            // bins of this row, or their mirror images M - f
            int64_t lo = (int64_t)k3 * per_row, hi = lo + per_row - 1;
            if (side) {
                const int64_t mlo = (p->M - hi) % p->M, mhi = (p->M - lo) % p->M;
                if (lo == 0) {                  // row 0 mirrors to {0} and [M - per_row + 1, M - 1]
                    kept = block_keep[0] != 0;
                    lo = p->M - per_row + 1;
                    hi = p->M - 1;
                } else {
                    lo = mlo;
                    hi = mhi;
                }
            }
            for (int64_t b = lo / per_blk; b <= hi / per_blk && !kept; ++b) kept = block_keep[b] != 0;
        }
        if (kept) live |= 1u << k3;
    }
    return live;
}

int fused3_init_inner(fftconv_plan *p)
{
    p->f3.N1 = N1;
    p->f3.N2 = 16;
    p->f3.N3 = 16;
    hipDeviceProp_t prop;
    FC_HIP(hipGetDeviceProperties(&prop, p->device));
    p->f3.num_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    return build_tables<16, 16>(p, &p->f3.consts);
}

// ko_n > 0: the k_f rows come in groups of ko_n (outer frequency digit ko); only ko < ko_lo and ko >= ko_hi
// are processed (the others hold zero spectra and their rows are never touched).  ko_n = 0: every row.
int fused3_inner_rows(const fftconv_plan *p, void *rows, const void *kf, int64_t rows_per_kf, int64_t kf_rows,
                      hipStream_t s, int ko_n, int ko_lo, int ko_hi, bool quarter_rows)
{
    int64_t live_rows = kf_rows;
    if (ko_n > 0) {
        if (ko_lo >= ko_hi) ko_n = 0;                            // everything live
        else live_rows = kf_rows / ko_n * (ko_lo + ko_n - ko_hi);
    }
    return fused3_wsc_launch(p, rows, kf, rows_per_kf, live_rows, s, ko_n, ko_lo, ko_hi, quarter_rows);
}

int fused3_inner_whole(const fftconv_plan *p, const void *u, const void *kf, void *y, int64_t B, hipStream_t s)
{
    return fused3_wsc_real_launch(p, u, kf, y, B, s);
}

void fused3_destroy(fftconv_plan *p)
{
    if (p->f3.consts) (void)hipFree(p->f3.consts);
    if (p->f3.consts_short) (void)hipFree(p->f3.consts_short);
    p->f3.consts = nullptr;
    p->f3.consts_short = nullptr;
}

constexpr int64_t SHORT_M = 8192;          // transform length of the segments of a partial convolution
constexpr int64_t SHORT_MAX_P = 2048;      // most history a segment may carry (at least half of it is output)

// Plans for fft >= 16384 (the single-kernel ones and the multi-pass route) also carry the 8192-point tables:
// a short (partial) filter runs as overlapping 8192-point segments, and k_f then holds a second,
// 8192-point spectrum (8 bytes per bin) after the dense one.
int fused3_init_short(fftconv_plan *p)
{
    if (p->M < 2 * SHORT_M || p->N > p->M / 2 || p->N % 8 != 0) return FFTCONV_OK;      // no segmented route
    if (p->f3.num_cu == 0) {
        hipDeviceProp_t prop;
        FC_HIP(hipGetDeviceProperties(&prop, p->device));
        p->f3.num_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    }
    return build_tables<16, 16>(p, &p->f3.consts_short);
}

constexpr size_t SHORT_TAG_BYTES = 256;     // the tag word, padded so that whatever follows stays aligned

size_t fused3_short_kf_bytes(const fftconv_plan *p)
{
    return p->f3.consts_short ? (size_t)(p->H * SHORT_M) * sizeof(float2) + SHORT_TAG_BYTES : 0;
}

// bytes of the plan's dense spectrum, = offset of the short one
static size_t dense_kf_bytes(const fftconv_plan *p)
{
    if (p->path == PATH_MULTIPASS) return multipass_kf_bytes(p) - fused3_short_kf_bytes(p);
    return fused3_big_kf_bytes(p);
}

size_t fused3_kf_bytes(const fftconv_plan *p)
{
    if (p->M >= 16384) return fused3_big_kf_bytes(p) + fused3_short_kf_bytes(p);
    return (size_t)(p->H * 8192) * sizeof(float2);             // fft <= 8192: the 8192 slots of the wave-specialised kernel
}

const long long *fused3_short_tag(const fftconv_plan *p, const void *kf)
{
    return (const long long *)((const char *)kf + dense_kf_bytes(p) + (size_t)(p->H * SHORT_M) * sizeof(float2));
}

__global__ void k_set_tag(long long *tag, long long value) { *tag = value; }

int fused3_set_short_tag(const fftconv_plan *p, void *kf, int64_t Nk, hipStream_t s)
{
    hipLaunchKernelGGL(k_set_tag, dim3(1), dim3(1), 0, s, (long long *)fused3_short_tag(p, kf), (long long)Nk);
    FC_HIP(hipGetLastError());
    return FFTCONV_OK;
}

static int64_t history_of(int64_t Nk) { return (Nk - 1 + 7) / 8 * 8; }

bool fused3_short_ok(const fftconv_plan *p, int64_t Nk)
{
    return p->f3.consts_short != nullptr && Nk >= 1 && history_of(Nk) <= SHORT_MAX_P;
}

static int launch_filter_fused3(const float *k, int64_t Nk, int64_t H, uint2 *kf, const float2 *w, const FacList &fl,
                                int64_t Ms, int64_t tws, bool reversed, const uint8_t *keep_dev, int64_t n_blocks, int fmt,
                                hipStream_t s)
{
    const size_t bytes = lds_row_bytes(Ms, sizeof(float2));
    FC_TRY(raise_dynamic_lds((const void *)k_filter_fused3, (int)lds_row_bytes(8192, sizeof(float2))));
    hipLaunchKernelGGL(k_filter_fused3, dim3((unsigned)H), dim3(FILT_THREADS), bytes, s, k, kf, w, fl, Nk, (int)tws, reversed,
                       keep_dev, n_blocks, fmt, (int)(8192 / Ms));
    FC_HIP(hipGetLastError());
    return FFTCONV_OK;
}

// the 8192-point spectrum of a short filter, behind the dense one (see fused3_forward_short)
int fused3_filter_short(const fftconv_plan *p, const float *k, int64_t Nk, void *kf, hipStream_t s)
{
    uint2 *dst = (uint2 *)((char *)kf + dense_kf_bytes(p));
    return launch_filter_fused3(k, Nk, p->H, dst, p->st.w32, staged_factors_for(SHORT_M), SHORT_M, p->M / SHORT_M, false,
                                nullptr, 1, p->dtype == FFTCONV_F16 ? 2 : 1, s);
}

// Partial convolution (Section 3.3) of a plan for fft >= 16384: the filter covers Nk <= 2049 taps, so
// every output depends on at most P = Nk - 1 (rounded up to 8) earlier inputs and the row can be cut
// into overlapping windows that each fit the 8192-point kernel (overlap-save).  The outermost
// factor of the decomposition is skipped altogether: 8192-point transforms instead of 16384-point
// ones, register-resident tables, 1/2 of the k_f bytes.
int fused3_forward_short(const fftconv_plan *p, const void *u, const void *kf, void *y, int64_t B, int64_t Nk,
                         hipStream_t s)
{
    if (((uintptr_t)u | (uintptr_t)y) & 15) {
        set_error("fftconv_forward_partial: u and y must be 16-byte aligned for this plan");
        return FFTCONV_EINVAL;
    }
    const int P = (int)history_of(Nk);
    const int Lo = (int)(SHORT_M / 2) - P;
    const int nseg = p->N <= SHORT_M / 2 ? 1 : 1 + (int)((p->N - SHORT_M / 2 + Lo - 1) / Lo);
    const float2 *kf_short = (const float2 *)((const char *)kf + dense_kf_bytes(p));
    return fused3_ws_launch(p, p->f3.consts_short, u, kf_short, y, B, nseg, P, s);
}

// The filter transform of every plan on this path is one kernel from the taps to k_f.
int fused3_filter(const fftconv_plan *p, const float *k, int64_t Nk, bool adjoint, const uint8_t *keep_dev,
                  int64_t n_blocks, void *kf, hipStream_t s)
{
    if (p->M > 8192) return fused3_big_filter(p, k, Nk, adjoint, keep_dev, n_blocks, kf, s);
    // the 8192-point kernel takes k_f as 16-bit constant pairs; shorter transforms fill its 8192 slots with
    // 8192 / fft_size copies of their spectrum (see build_tables())
    return launch_filter_fused3(k, Nk, p->H, (uint2 *)kf, p->st.w32, staged_fac_list(p), p->M, 1, adjoint, keep_dev,
                                n_blocks, p->dtype == FFTCONV_F16 ? 2 : 1, s);
}

bool fused3_gates_fused(const fftconv_plan *p) { return p->path == PATH_FUSED3; }

int fused3_forward_gated(const fftconv_plan *p, const void *u, const void *w, const void *v, const void *kf, void *y,
                         int64_t B, hipStream_t s)
{
    if (((uintptr_t)u | (uintptr_t)y | (uintptr_t)w | (uintptr_t)v) & 15) {
        set_error("fftconv_forward_gated: u, w, v and y must be 16-byte aligned for this plan");
        return FFTCONV_EINVAL;
    }
    if (p->M > 8192) return fused3_big_forward_gated(p, u, w, v, kf, y, B, s);
    return fused3_ws_launch(p, p->f3.consts, u, kf, y, B, 1, 0, s, w, v);
}

int fused3_forward(const fftconv_plan *p, const void *u, const void *kf, void *y, int64_t B, hipStream_t s)
{
    if (((uintptr_t)u | (uintptr_t)y) & 15) {
        set_error("fftconv_forward: u and y must be 16-byte aligned for this plan");
        return FFTCONV_EINVAL;
    }
    switch (p->M) {
    case 256:
    case 512:
    case 1024:
    case 2048:
    case 4096:
    case 8192:
        return fused3_ws_launch(p, p->f3.consts, u, kf, y, B, 1, 0, s);     // wave-specialised schedule (fused3_ws.hip)
    case 16384:
    case 32768:
        return fused3_big_forward(p, u, kf, y, B, 0xffffffffu, s);
    default:
        set_error("fused3: no kernel for fft_size=%lld", (long long)p->M);
        return FFTCONV_EUNSUPPORTED;
    }
}

}  // namespace fftconv
