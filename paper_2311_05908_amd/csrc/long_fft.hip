// fp32 transforms of rows too long for LDS (fft_size 16384 .. 2^22), two kernels per direction instead of one
// per factor: the decomposition of the generic path (Section 3.2, order-p Monarch form; decimation in
// frequency, position order out) with fft_size = A * 8192.
//   forward:  "columns" - the factors of A act at stride 8192: a workgroup takes C = 8192 / A adjacent columns
//             of the (A, 8192) view of a row into LDS (8192 points), runs those stages there with the twiddles
//             W_M^{k R r} of the full length and writes the tile back in place;
//             "blocks"  - the remaining factors act inside contiguous blocks of 8192 positions: one workgroup
//             per block, the length-8192 forward transform of lds_fft.h (its own table of W_8192).
//   inverse:  the same two kernels mirrored (blocks first, then columns).
// Users: the filter transform of the multi-pass plans (taps -> spectrum -> k_f, fp32 is ample for constants
// that are rounded to 16 bits) and the filter gradient of every plan from fft_size 16384 up that has no
// fused kernel (Section 3.1 "Kernel Fusion and Recomputation": dk = Re iFFT(sum_b conj(FFT(u_b)) FFT(dy_b))[0:Nk]).
// Two batch rows share one complex transform there, z = x_b + i x_{b+1}: conj(Z_u) Z_dy is the wanted sum plus
// i times a cross term that is itself the spectrum of a real sequence, so it ends up in the imaginary part of
// the inverse transform, which is dropped.
#include <hip/hip_runtime.h>
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>

#include <cmath>
#include <type_traits>
#include <vector>

#include "fftconv_internal.h"
#include "lds_fft.h"

namespace fftconv {

namespace {

constexpr int LB = 8192;                       // block length: what one workgroup holds in LDS
constexpr int LT = 512;                        // threads per workgroup
constexpr size_t L_LDS = (size_t)(LB + LB / 16) * sizeof(float2);

struct LongGeo {
    int A = 0, C = 0;                          // outer length, columns per tile (A * C = 8192)
    FacList flA, flB, fl;                      // factors of A, of 8192, and all of them (the position order)
};

LongGeo long_geo(int64_t M)
{
    LongGeo g;
    g.A = (int)(M / LB);
    g.C = LB / g.A;
    int nf = 0, rem = g.A;
    for (int i = 0; i < MAX_FACTORS; ++i) g.flA.fac[i] = g.flB.fac[i] = g.fl.fac[i] = 0;
    while (rem >= 16) {
        g.flA.fac[nf++] = 16;
        rem /= 16;
    }
    if (rem > 1) g.flA.fac[nf++] = rem;
    g.flA.nf = nf;
    g.flB = staged_factors_for(LB);
    g.fl.nf = g.flA.nf + g.flB.nf;
    for (int i = 0; i < g.flA.nf; ++i) g.fl.fac[i] = g.flA.fac[i];
    for (int i = 0; i < g.flB.nf; ++i) g.fl.fac[g.flA.nf + i] = g.flB.fac[i];
    return g;
}

__device__ __forceinline__ float ld_real(const float *p, int64_t i) { return p[i]; }
__device__ __forceinline__ float ld_real(const __half *p, int64_t i) { return __half2float(p[i]); }
__device__ __forceinline__ float ld_real(const __hip_bfloat16 *p, int64_t i) { return __bfloat162float(p[i]); }
__device__ __forceinline__ void st_real(float *p, int64_t i, float v) { p[i] = v; }
__device__ __forceinline__ void st_real(__half *p, int64_t i, float v) { p[i] = __float2half_rn(v); }
__device__ __forceinline__ void st_real(__hip_bfloat16 *p, int64_t i, float v) { p[i] = __float2bfloat16(v); }

// W_M^e of the full length as a product of two small tables, e = 2048 e_hi + e_lo: the exponents of the outer
// stages are spread over the whole range, and gathers from a table of M entries (16 MB at 2^21) miss every cache
struct LongTw {
    const float2 *w8k;                         // W_8192^t, t < 8192: the table of the block transforms
    const float2 *lo, *hi;                     // W_M^t, t < 2048; W_M^{2048 t}, t < M / 2048
    __device__ __forceinline__ float2 operator()(int64_t e) const { return cmul(hi[e >> 11], lo[e & 2047]); }
};

// A thread's share of a tile of 8192 points: LPT points LT apart.  All loads of a thread are issued before the
// first value is used (a loop of load -> LDS write waits for every load in turn, and the round trip to HBM was most
// of these kernels' time); the launches use LT threads.
constexpr int LPT = LB / LT;
// contiguous block: src[i] -> slot i
__device__ __forceinline__ void load_block(float2 *XL, const float2 *__restrict__ src)
{
    float2 v[LPT];
#pragma unroll
    for (int j = 0; j < LPT; ++j) v[j] = src[threadIdx.x + j * LT];
#pragma unroll
    for (int j = 0; j < LPT; ++j) XL[lds_slot(threadIdx.x + j * LT)] = v[j];
}
__device__ __forceinline__ void store_block(const float2 *XL, float2 *__restrict__ dst)
{
#pragma unroll
    for (int j = 0; j < LPT; ++j) dst[threadIdx.x + j * LT] = XL[lds_slot(threadIdx.x + j * LT)];
}
// column tile: slot i = a * C + c <- row[a * 8192 + col0 + c] (C a power of two)
__device__ __forceinline__ void load_cols(float2 *XL, const float2 *__restrict__ row, int C, int col0)
{
    const int lgC = __ffs(C) - 1;
    float2 v[LPT];
#pragma unroll
    for (int j = 0; j < LPT; ++j) {
        const int i = threadIdx.x + j * LT;
        v[j] = row[(int64_t)(i >> lgC) * LB + col0 + (i & (C - 1))];
    }
#pragma unroll
    for (int j = 0; j < LPT; ++j) XL[lds_slot(threadIdx.x + j * LT)] = v[j];
}

// One stage of the outer part on a tile X[a][c] (a < A, c < C, slot a * C + c): factor R_ along a at stride
// Sp, for every column; the twiddle exponent k Rj r uses the position r = rp * 8192 + (first column + c)
// inside the full-length stage.
template <int R_, bool INV>
__device__ inline void cols_stage(float2 *X, const LongTw &w, int A, int C, int Sp, int Rj, int col0)
{
    const int nb = (A / R_) * C;
    const int lgC = __ffs(C) - 1, lgSp = __ffs(Sp) - 1;          // powers of two
    for (int t = threadIdx.x; t < nb; t += blockDim.x) {
        const int c = t & (C - 1), q = t >> lgC;
        const int rp = q & (Sp - 1), prefix = q >> lgSp;
        const int a0 = prefix * R_ * Sp + rp;
        const int64_t rg = (int64_t)rp * LB + col0 + c;
        float2 x[R_], tw[R_];
        stage_twiddles<R_>(tw, w, (int64_t)Rj * rg);
#pragma unroll
        for (int n = 0; n < R_; ++n) {
            x[n] = X[lds_slot((a0 + n * Sp) * C + c)];
            if (INV) x[n] = cmul_conj(x[n], tw[n]);
        }
        dft_reg<R_, INV>(x);
#pragma unroll
        for (int k = 0; k < R_; ++k) X[lds_slot((a0 + k * Sp) * C + c)] = INV ? x[k] : cmul(x[k], tw[k]);
    }
}

template <bool INV>
__device__ inline void cols_stage_any(float2 *X, const LongTw &w, int A, int C, int Nj, int Sp, int Rj, int col0)
{
    switch (Nj) {
    case 2: cols_stage<2, INV>(X, w, A, C, Sp, Rj, col0); break;
    case 4: cols_stage<4, INV>(X, w, A, C, Sp, Rj, col0); break;
    case 8: cols_stage<8, INV>(X, w, A, C, Sp, Rj, col0); break;
    default: cols_stage<16, INV>(X, w, A, C, Sp, Rj, col0); break;
    }
}

// Forward, columns: rows of real input (re from src_re, im from src_im or zero; `len` valid samples, zeros
// beyond; reversed: position n holds sample (M - n) mod M) -> tmp (rows, M) after the factors of A.
// half_rows (real input only, src_im == nullptr): only the blocks of the outer frequency digits ko <= A/2 are
// written; the others hold mirror images (see k_long_fwd_blocks_kf) and nobody reads them.
template <typename In>
__global__ void __launch_bounds__(LT) k_long_fwd_cols(const In *__restrict__ src_re, const In *__restrict__ src_im,
                                                     float2 *__restrict__ tmp, LongTw w, FacList flA, int A, int C, int64_t len,
                                                     bool reversed, bool half_rows)
{
    extern __shared__ float2 XL[];
    const int64_t M = (int64_t)A * LB, row = blockIdx.y;
    const int col0 = blockIdx.x * C;
    const int lgC = __ffs(C) - 1;
    // samples beyond `len` are zeros: their loads go to sample 0 instead and are discarded, so that every load of
    // the thread is unconditional and in flight at once (see load_block)
    float vr[LPT], vi[LPT];
#pragma unroll
    for (int j = 0; j < LPT; ++j) {
        const int i = threadIdx.x + j * LT;
        int64_t n = (int64_t)(i >> lgC) * LB + col0 + (i & (C - 1));
        if (reversed && n != 0) n = M - n;
        const int64_t at = row * len + (n < len ? n : 0);
        vr[j] = ld_real(src_re, at);
        vi[j] = src_im ? ld_real(src_im, at) : 0.f;
    }
#pragma unroll
    for (int j = 0; j < LPT; ++j) asm volatile("" ::"v"(vr[j]), "v"(vi[j]));      // keeps the loads unconditional
#pragma unroll
    for (int j = 0; j < LPT; ++j) {
        const int i = threadIdx.x + j * LT;
        int64_t n = (int64_t)(i >> lgC) * LB + col0 + (i & (C - 1));
        if (reversed && n != 0) n = M - n;
        XL[lds_slot(i)] = n < len ? make_float2(vr[j], vi[j]) : make_float2(0.f, 0.f);
    }
    __syncthreads();
    int Sp = A, R = 1;
    for (int i = 0; i < flA.nf; ++i) {
        const int Nj = flA.fac[i];
        Sp /= Nj;
        cols_stage_any<false>(XL, w, A, C, Nj, Sp, R, col0);
        __syncthreads();
        R *= Nj;
    }
#pragma unroll
    for (int j = 0; j < LPT; ++j) {
        const int i = threadIdx.x + j * LT;
        const int ap = i >> lgC;                              // position of the block; its digit: lds_freq()
        if (!half_rows || 2 * lds_freq(ap, flA, A) <= A)
            tmp[row * M + (int64_t)ap * LB + col0 + (i & (C - 1))] = XL[lds_slot(i)];
    }
}

// Forward, blocks: tmp -> spectrum in position order.  MODE 0: store to out.  MODE 1: acc (+)= conj(other) * X
// (other: the spectrum of the u rows, X: that of the dy rows; first: assign instead of add).
template <int MODE>
__global__ void __launch_bounds__(LT) k_long_fwd_blocks(const float2 *__restrict__ tmp, float2 *__restrict__ out,
                                                       const float2 *__restrict__ other, LongTw w, FacList flB, int A,
                                                       bool first)
{
    extern __shared__ float2 XL[];
    const int64_t base = ((int64_t)blockIdx.y * A + blockIdx.x) * LB;
    load_block(XL, tmp + base);
    __syncthreads();
    lds_forward(XL, w.w8k, flB, LB, 1);
    if (MODE == 0) {
        store_block(XL, out + base);
    } else {
        float2 a[LPT], o[LPT];
#pragma unroll
        for (int j = 0; j < LPT; ++j) a[j] = other[base + threadIdx.x + j * LT];
        if (!first) {
#pragma unroll
            for (int j = 0; j < LPT; ++j) o[j] = out[base + threadIdx.x + j * LT];
        }
#pragma unroll
        for (int j = 0; j < LPT; ++j) {
            const int i = threadIdx.x + j * LT;
            const float2 x = XL[lds_slot(i)];
            float2 v = make_float2(a[j].x * x.x + a[j].y * x.y, a[j].x * x.y - a[j].y * x.x);
            if (!first) {
                v.x += o[j].x;
                v.y += o[j].y;
            }
            out[base + i] = v;
        }
    }
}

// Forward, blocks, for the filter transform of the multi-pass plans: the block at position a' of a row holds the
// bins f = ko + A f' of one outer frequency digit ko (the digit reversal of a'), f' < 8192 in position order; they
// go straight to that digit's row of k_f, [h][ko][slot of f' in the 8192-point kernel's per-lane order] as 16-bit
// (re, im) pairs, scaled by 1/M (times the fp16 range boost, multipass_kf_boost) and by the frequency mask.
// The taps are real, so K[M - f] = conj K[f]: with f = ko + A f', M - f = (A - ko) + A (8191 - f') for ko >= 1.  Only the
// blocks of the digits ko <= A/2 are transformed (the column kernel wrote no others); a block with 0 < ko < A/2 also
// writes the row of the digit A - ko, bin g of which is the conjugate of this row's bin 8191 - g.  The rows ko = 0 and
// ko = A/2 are their own mirror images.
// natural: tmp holds the rows ko <= A/2 only, in the order of ko (A/2 + 1 blocks per channel: the output of
// k_filter_outer_real, multipass.hip) instead of all A blocks in position order.  conj_out: the conjugate spectrum
// (that of the circularly time-reversed taps, which are real).
template <bool F16>
__global__ void __launch_bounds__(LT) k_long_fwd_blocks_kf(const float2 *__restrict__ tmp, uint32_t *__restrict__ kf, LongTw w,
                                                          FacList flA, FacList flB, int A, int64_t h0,
                                                          const uint8_t *__restrict__ keep, int64_t n_blocks, bool natural,
                                                          bool conj_out)
{
    extern __shared__ float2 XL[];
    const int ko = natural ? (int)blockIdx.x : lds_freq(blockIdx.x, flA, A);
    if (2 * ko > A) return;                                   // written by the block of A - ko
    const int64_t base = natural ? ((int64_t)blockIdx.y * (A / 2 + 1) + ko) * LB : ((int64_t)blockIdx.y * A + blockIdx.x) * LB;
    load_block(XL, tmp + base);
    __syncthreads();
    lds_forward(XL, w.w8k, flB, LB, 1);
    const int M = A * LB;
    const float boost = (float)multipass_kf_boost(F16, A) / (float)M;
    typedef __attribute__((ext_vector_type(2))) float f32x2;
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
    auto pair16 = [](float re, float im) {                    // round to nearest even, one conversion instruction
        const f32x2 v = {re, im};
        if constexpr (F16) return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
        else return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
    };
    // position of inner frequency f after the block transform, for the factors 16, 16, 16, 2 of 8192 (lds_pos()
    // with the loop over the factor list folded; the launch checks the list)
    auto pos8k = [](int f) { return ((f & 15) << 9) | (((f >> 4) & 15) << 5) | (((f >> 8) & 15) << 1) | (f >> 12); };
    uint32_t *dst = kf + ((h0 + blockIdx.y) * A + ko) * (int64_t)LB;
    const bool mirror = ko > 0 && 2 * ko < A;
    uint32_t *dst_m = kf + ((h0 + blockIdx.y) * A + (mirror ? A - ko : ko)) * (int64_t)LB;
#pragma unroll 4
    for (int d = threadIdx.x; d < LB; d += LT) {
        const int lane = d % 64, r = (d / 64) % 4, k1 = d / 256;
        const int k2 = lane % 16, k3 = k3_at_index(4 * (lane / 16) + r, 16);
        const int fi = k1 + 32 * (k2 + 16 * k3);              // the inner frequency of slot d
        const float2 v = XL[lds_slot(pos8k(fi))];
        const float sc = keep ? lds_mask_weight(keep, n_blocks, ko + A * fi, M) * boost : boost;
        dst[d] = pair16(v.x * sc, conj_out ? -v.y * sc : v.y * sc);
        if (mirror) {
            const float2 vm = XL[lds_slot(pos8k(LB - 1 - fi))];
            const float scm = keep ? lds_mask_weight(keep, n_blocks, (A - ko) + A * fi, M) * boost : boost;
            dst_m[d] = pair16(vm.x * scm, conj_out ? vm.y * scm : -vm.y * scm);
        }
    }
}

// The same for the plans that keep k_f as fp32 pairs in position order (fp32 I/O from fft_size 32768 up): tmp
// holds the rows ko <= A/2 in the order of ko (k_filter_outer_real); row ko goes to the block at the position of
// digit ko, bins in the block transform's own order, scaled by 1/M and by the frequency mask; the mirror row
// A - ko likewise, bin g = conj of this row's bin 8191 - g.
__global__ void __launch_bounds__(LT) k_long_fwd_blocks_kf32(const float2 *__restrict__ tmp, float2 *__restrict__ kf, LongTw w,
                                                            FacList flA, FacList flB, int A, int64_t h0,
                                                            const uint8_t *__restrict__ keep, int64_t n_blocks, bool conj_out)
{
    extern __shared__ float2 XL[];
    const int ko = blockIdx.x;                                // <= A/2
    const int64_t base = ((int64_t)blockIdx.y * (A / 2 + 1) + ko) * LB;
    load_block(XL, tmp + base);
    __syncthreads();
    lds_forward(XL, w.w8k, flB, LB, 1);
    const int M = A * LB;
    const float inv = 1.0f / (float)M;
    // the factors 16, 16, 16, 2 of 8192 folded (the launch checks the list): position of a frequency and back
    auto pos8k = [](int f) { return ((f & 15) << 9) | (((f >> 4) & 15) << 5) | (((f >> 8) & 15) << 1) | (f >> 12); };
    auto freq8k = [](int i) { return (i >> 9) | (((i >> 5) & 15) << 4) | (((i >> 1) & 15) << 8) | ((i & 1) << 12); };
    const bool mirror = ko > 0 && 2 * ko < A;
    float2 *dst = kf + ((h0 + blockIdx.y) * A + lds_pos(ko, flA, A)) * (int64_t)LB;
    float2 *dst_m = kf + ((h0 + blockIdx.y) * A + lds_pos(mirror ? A - ko : ko, flA, A)) * (int64_t)LB;
    const float sgn = conj_out ? -1.f : 1.f;
#pragma unroll 4
    for (int i = threadIdx.x; i < LB; i += LT) {
        const int fi = freq8k(i);
        const float2 v = XL[lds_slot(i)];
        const float sc = keep ? lds_mask_weight(keep, n_blocks, ko + A * fi, M) * inv : inv;
        dst[i] = make_float2(v.x * sc, sgn * v.y * sc);
        if (mirror) {
            const float2 vm = XL[lds_slot(pos8k(LB - 1 - fi))];
            const float scm = keep ? lds_mask_weight(keep, n_blocks, (A - ko) + A * fi, M) * inv : inv;
            dst_m[i] = make_float2(vm.x * scm, -sgn * vm.y * scm);
        }
    }
}

// Inverse, blocks: spectrum in position order -> tmp after the factors of 8192 (unnormalised).
__global__ void __launch_bounds__(LT) k_long_inv_blocks(const float2 *__restrict__ spec, float2 *__restrict__ tmp, LongTw w,
                                                       FacList flB, int A)
{
    extern __shared__ float2 XL[];
    const int64_t base = ((int64_t)blockIdx.y * A + blockIdx.x) * LB;
    load_block(XL, spec + base);
    __syncthreads();
    lds_inverse(XL, w.w8k, flB, LB, 1);
    store_block(XL, tmp + base);
}

// Inverse, columns: the factors of A, then real part times scale of the samples n < Nk -> dk (rows, Nk).
__global__ void __launch_bounds__(LT) k_long_inv_cols_dk(const float2 *__restrict__ tmp, float *__restrict__ dk, LongTw w,
                                                        FacList flA, int A, int C, int64_t Nk, float scale)
{
    extern __shared__ float2 XL[];
    const int64_t M = (int64_t)A * LB, row = blockIdx.y;
    const int col0 = blockIdx.x * C;
    if (col0 >= Nk) return;                                 // every sample of this tile is n >= col0 >= Nk
    load_cols(XL, tmp + row * M, C, col0);
    __syncthreads();
    int Sp = 1, R = A;
    for (int i = flA.nf - 1; i >= 0; --i) {
        const int Nj = flA.fac[i];
        R /= Nj;
        cols_stage_any<true>(XL, w, A, C, Nj, Sp, R, col0);
        __syncthreads();
        Sp *= Nj;
    }
    for (int i = threadIdx.x; i < LB; i += LT) {
        const int a = i >> (__ffs(C) - 1), c = i & (C - 1);
        const int64_t n = (int64_t)a * LB + col0 + c;
        if (n < Nk) dk[row * Nk + n] = XL[lds_slot(i)].x * scale;
    }
}

// ---- The convolution itself in fp32 (plans with fp32 I/O from fft_size 8192 up): y = iFFT(FFT(pad(u)) . k_f)[0:N]
// with k_f as fp32 pairs in position order, already scaled by 1 / fft_size.  Two batch rows share a complex
// transform (re = row b, im = row b + 1; k is real, so the two convolutions come back as re and im).
//
// Rows that fit in LDS (fft_size <= 16384): one workgroup per (pair, channel) does everything.
template <typename IO>
__global__ void __launch_bounds__(LT) k_rows_conv_lds(const IO *__restrict__ u, const float2 *__restrict__ kf,
                                                     IO *__restrict__ y, const float2 *__restrict__ w, FacList fl, int M,
                                                     int64_t N, int B, int H)
{
    extern __shared__ float2 XL[];
    const int h = blockIdx.x, b0 = 2 * blockIdx.y;
    const bool two = b0 + 1 < B;
    const int64_t r0 = ((int64_t)b0 * H + h) * N, r1 = r0 + (int64_t)H * N;
    // (a sample beyond N, or of a missing second row, reads a valid one and is discarded: unconditional loads,
    //  several in flight per thread)
    const int64_t r1e = two ? r1 : r0;
#pragma unroll 8
    for (int n = threadIdx.x; n < M; n += LT) {
        const int64_t at = n < N ? n : 0;
        const float a = ld_real(u, r0 + at), b = ld_real(u, r1e + at);
        XL[lds_slot(n)] = n < N ? make_float2(a, two ? b : 0.f) : make_float2(0.f, 0.f);
    }
    __syncthreads();
    lds_forward(XL, w, fl, M, 1);
#pragma unroll 8
    for (int i = threadIdx.x; i < M; i += LT) XL[lds_slot(i)] = cmul(XL[lds_slot(i)], kf[(int64_t)h * M + i]);
    __syncthreads();
    lds_inverse(XL, w, fl, M, 1);
    for (int n = threadIdx.x; n < N; n += LT) {
        const float2 v = XL[lds_slot(n)];
        st_real(y, r0 + n, v.x);
        if (two) st_real(y, r1 + n, v.y);
    }
}

// Longer rows, middle kernel: a block of 8192 positions forward, times its piece of k_f, and back, in place in tmp.
// natural: tmp holds the rows ko <= A/2 of real sequences in the order of ko (A/2 + 1 blocks per channel, the output
// of k_filter_outer_real); the k_f of digit ko sits at that digit's position among the A blocks of the channel.
__global__ void __launch_bounds__(LT) k_long_conv_blocks(float2 *__restrict__ tmp, const float2 *__restrict__ kf, LongTw w,
                                                        FacList flA, FacList flB, int A, bool natural)
{
    extern __shared__ float2 XL[];
    const int64_t base = natural ? ((int64_t)blockIdx.y * (A / 2 + 1) + blockIdx.x) * LB
                                 : ((int64_t)blockIdx.y * A + blockIdx.x) * LB;
    const int64_t kbase = natural ? ((int64_t)blockIdx.y * A + lds_pos(blockIdx.x, flA, A)) * LB : base;
    load_block(XL, tmp + base);
    float2 kv[LPT];                                          // in flight during the forward transform
#pragma unroll
    for (int j = 0; j < LPT; ++j) kv[j] = kf[kbase + threadIdx.x + j * LT];
    __syncthreads();
    lds_forward(XL, w.w8k, flB, LB, 1);
#pragma unroll
    for (int j = 0; j < LPT; ++j) {
        const int i = threadIdx.x + j * LT;
        XL[lds_slot(i)] = cmul(XL[lds_slot(i)], kv[j]);
    }
    __syncthreads();
    lds_inverse(XL, w.w8k, flB, LB, 1);
    store_block(XL, tmp + base);
}

// Longer rows, last kernel: the outer factors back, real part -> row of y_re, imaginary part -> row of y_im
// (nullptr: no second row), the first N samples.
template <typename IO>
__global__ void __launch_bounds__(LT) k_long_inv_cols_y(const float2 *__restrict__ tmp, IO *__restrict__ y_re,
                                                       IO *__restrict__ y_im, LongTw w, FacList flA, int A, int C, int64_t N)
{
    extern __shared__ float2 XL[];
    const int64_t M = (int64_t)A * LB, row = blockIdx.y;
    const int col0 = blockIdx.x * C;
    if (col0 >= N) return;
    load_cols(XL, tmp + row * M, C, col0);
    __syncthreads();
    int Sp = 1, R = A;
    for (int i = flA.nf - 1; i >= 0; --i) {
        const int Nj = flA.fac[i];
        R /= Nj;
        cols_stage_any<true>(XL, w, A, C, Nj, Sp, R, col0);
        __syncthreads();
        Sp *= Nj;
    }
    for (int i = threadIdx.x; i < LB; i += LT) {
        const int a = i >> (__ffs(C) - 1), c = i & (C - 1);
        const int64_t n = (int64_t)a * LB + col0 + c;
        if (n < N) {
            const float2 v = XL[lds_slot(i)];
            st_real(y_re, row * N + n, v.x);
            if (y_im) st_real(y_im, row * N + n, v.y);
        }
    }
}

__global__ void k_zero_dk(float *x, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) x[i] = 0.f;
}

LongTw long_tw(const fftconv_plan *p)
{
    LongTw t;
    t.w8k = p->long_tw;
    t.lo = p->long_tw + LB;
    t.hi = t.lo + 2048;
    return t;
}

int raise_lds(const void *kern) { return raise_dynamic_lds(kern, (int)L_LDS); }

template <typename In>
int launch_fwd_cols(const LongGeo &g, const In *re, const In *im, float2 *tmp, const LongTw &w, int64_t rows, int64_t len,
                    bool reversed, hipStream_t s, bool half_rows = false)
{
    const int rc = raise_lds((const void *)k_long_fwd_cols<In>);
    if (rc) return rc;
    hipLaunchKernelGGL(k_long_fwd_cols<In>, dim3((unsigned)g.A, (unsigned)rows), dim3(LT), L_LDS, s, re, im, tmp, w, g.flA,
                       g.A, g.C, len, reversed, half_rows && im == nullptr);
    FC_HIP(hipGetLastError());
    return FFTCONV_OK;
}

template <int MODE>
int launch_fwd_blocks(const LongGeo &g, const float2 *tmp, float2 *out, const float2 *other, const LongTw &w, int64_t rows,
                      bool first, hipStream_t s)
{
    const int rc = raise_lds((const void *)k_long_fwd_blocks<MODE>);
    if (rc) return rc;
    hipLaunchKernelGGL(k_long_fwd_blocks<MODE>, dim3((unsigned)g.A, (unsigned)rows), dim3(LT), L_LDS, s, tmp, out, other, w,
                       g.flB, g.A, first);
    FC_HIP(hipGetLastError());
    return FFTCONV_OK;
}

template <typename IO>
int long_backward_filter_t(const fftconv_plan *p, const IO *u, const IO *dy, float *dk, int64_t Nk, int64_t B,
                           void *workspace, hipStream_t s)
{
    const LongGeo g = long_geo(p->M);
    const LongTw tw = long_tw(p);
    const int64_t M = p->M, N = p->N, H = p->H;
    float2 *acc = (float2 *)workspace, *spec_u = acc + H * M, *tmp = spec_u + H * M;
    if (B == 0) {
        const int bs = 256;
        hipLaunchKernelGGL(k_zero_dk, dim3((unsigned)((H * Nk + bs - 1) / bs)), dim3(bs), 0, s, dk, H * Nk);
        FC_HIP(hipGetLastError());
        return FFTCONV_OK;
    }
    if (multipass_filter_outer_ok(p)) {
        // Outer lengths with a register kernel for real rows (multipass.hip): every row of u and dy is transformed
        // as a real sequence -- outer pass on the rows ko <= A/2 only, 8192-point block transforms of those rows,
        // acc (+)= conj(U) DY on them -- and the sum, the spectrum of a real sequence again, goes back through the
        // inverse block transforms and the real inverse outer pass: half the intermediate traffic of the complex
        // pipeline below, and a row without a partner costs no more than half a pair.
        const int NR = g.A / 2 + 1;
        const int64_t RW = (int64_t)NR * LB;
        float2 *acc2 = (float2 *)workspace, *spec2 = acc2 + H * RW, *tmp2 = spec2 + H * RW;
        const dim3 grid((unsigned)NR, (unsigned)H);
        int rc = raise_lds((const void *)k_long_fwd_blocks<0>);
        if (!rc) rc = raise_lds((const void *)k_long_fwd_blocks<1>);
        if (!rc) rc = raise_lds((const void *)k_long_inv_blocks);
        if (rc) return rc;
        for (int64_t b = 0; b < B; ++b) {
            rc = multipass_filter_outer(p, u + b * H * N, p->dtype, N, H, tmp2, s);
            if (rc) return rc;
            hipLaunchKernelGGL(k_long_fwd_blocks<0>, grid, dim3(LT), L_LDS, s, tmp2, spec2, nullptr, tw, g.flB, NR, false);
            FC_HIP(hipGetLastError());
            rc = multipass_filter_outer(p, dy + b * H * N, p->dtype, N, H, tmp2, s);
            if (rc) return rc;
            hipLaunchKernelGGL(k_long_fwd_blocks<1>, grid, dim3(LT), L_LDS, s, tmp2, acc2, spec2, tw, g.flB, NR, b == 0);
            FC_HIP(hipGetLastError());
        }
        hipLaunchKernelGGL(k_long_inv_blocks, grid, dim3(LT), L_LDS, s, acc2, tmp2, tw, g.flB, NR);
        FC_HIP(hipGetLastError());
        return multipass_dk_outer_inv(p, tmp2, dk, Nk, H, 1.0f / (float)M, s);
    }
    for (int64_t b = 0; b < B; b += 2) {                      // rows b and b + 1 share a transform
        const IO *u0 = u + b * H * N, *u1 = b + 1 < B ? u0 + H * N : nullptr;
        const IO *d0 = dy + b * H * N, *d1 = b + 1 < B ? d0 + H * N : nullptr;
        int rc = launch_fwd_cols<IO>(g, u0, u1, tmp, tw, H, N, false, s);
        if (!rc) rc = launch_fwd_blocks<0>(g, tmp, spec_u, nullptr, tw, H, false, s);
        if (!rc) rc = launch_fwd_cols<IO>(g, d0, d1, tmp, tw, H, N, false, s);
        if (!rc) rc = launch_fwd_blocks<1>(g, tmp, acc, spec_u, tw, H, b == 0, s);
        if (rc) return rc;
    }
    int rc = raise_lds((const void *)k_long_inv_blocks);
    if (!rc) rc = raise_lds((const void *)k_long_inv_cols_dk);
    if (rc) return rc;
    hipLaunchKernelGGL(k_long_inv_blocks, dim3((unsigned)g.A, (unsigned)H), dim3(LT), L_LDS, s, acc, tmp, tw, g.flB,
                       g.A);
    FC_HIP(hipGetLastError());
    hipLaunchKernelGGL(k_long_inv_cols_dk, dim3((unsigned)g.A, (unsigned)H), dim3(LT), L_LDS, s, tmp, dk, tw, g.flA,
                       g.A, g.C, Nk, 1.0f / (float)M);
    FC_HIP(hipGetLastError());
    return FFTCONV_OK;
}

// channels per trip through the workspace of the long forward pass: at most 512 MiB of it
int64_t conv_chunk(const fftconv_plan *p)
{
    int64_t c = ((int64_t)512 << 20) / (p->M * (int64_t)sizeof(float2));
    if (c < 1) c = 1;
    return c < p->H ? c : p->H;
}

template <typename IO>
int long_forward_t(const fftconv_plan *p, const IO *u, const float2 *kf, IO *y, int64_t B, void *workspace, hipStream_t s)
{
    const int64_t M = p->M, N = p->N, H = p->H, npairs = (B + 1) / 2;
    if (M <= 2 * LB) {                                   // the whole row in LDS
        if (H > 2147483647 || npairs > 65535) {
            set_error("fftconv_forward: H = %lld or ceil(B/2) = %lld exceeds the grid limits of this plan", (long long)H,
                      (long long)npairs);
            return FFTCONV_EUNSUPPORTED;
        }
            FC_TRY(raise_dynamic_lds((const void *)k_rows_conv_lds<IO>, (int)lds_row_bytes(2 * LB, sizeof(float2))));
        hipLaunchKernelGGL(k_rows_conv_lds<IO>, dim3((unsigned)H, (unsigned)npairs), dim3(LT), lds_row_bytes(M, sizeof(float2)),
                           s, u, kf, y, (const float2 *)p->st.w32, staged_fac_list(p), (int)M, N, (int)B, (int)H);
        FC_HIP(hipGetLastError());
        return FFTCONV_OK;
    }
    const LongGeo g = long_geo(M);
    const LongTw tw = long_tw(p);
    float2 *tmp = (float2 *)workspace;
    const int64_t chunk = conv_chunk(p);
    int rc = raise_lds((const void *)k_long_conv_blocks);
    if (!rc) rc = raise_lds((const void *)k_long_inv_cols_y<IO>);
    if (rc) return rc;
    // fp32 rows at outer lengths with register kernels for real rows (multipass.hip) can go one row at a time as
    // real sequences: outer pass on the rows ko <= A/2, the blocks of those rows (forward, k_f, inverse), real inverse
    // outer pass (k_f is the spectrum of real taps, so the product is the spectrum of a real sequence again).  That is
    // half the blocks of a complex transform per row, the same as a pair's share, with cheaper outer kernels: measured
    // faster from A = 32 up (2.8 against 3.3 ms for 2^27 samples at fft 2^18, 1.9 against 2.2 ms at 2^21), slower
    // below, where the rows ko <= A/2 are well over half of all (3 of 4 at A = 4) -- except for a row without a
    // partner, which otherwise pays for a whole pair.
    const bool real_ok = std::is_same<IO, float>::value && multipass_filter_outer_ok(p);
    const int NR = g.A / 2 + 1;
    for (int64_t b = 0; b < B;) {
        const bool two = b + 1 < B;
        const bool as_real = real_ok && (g.A >= 32 || !two);
        for (int64_t h0 = 0; h0 < H; h0 += chunk) {
            const int64_t nh = H - h0 < chunk ? H - h0 : chunk;
            const int64_t o0 = (b * H + h0) * N;
            if (as_real) {
                rc = multipass_filter_outer(p, u + o0, FFTCONV_F32, N, nh, tmp, s);
                if (rc) return rc;
                hipLaunchKernelGGL(k_long_conv_blocks, dim3((unsigned)NR, (unsigned)nh), dim3(LT), L_LDS, s, tmp, kf + h0 * M,
                                   tw, g.flA, g.flB, g.A, true);
                FC_HIP(hipGetLastError());
                rc = multipass_dk_outer_inv(p, tmp, (float *)(y + o0), N, nh, 1.0f, s);
                if (rc) return rc;
                continue;
            }
            rc = launch_fwd_cols<IO>(g, u + o0, two ? u + o0 + H * N : nullptr, tmp, tw, nh, N, false, s);
            if (rc) return rc;
            hipLaunchKernelGGL(k_long_conv_blocks, dim3((unsigned)g.A, (unsigned)nh), dim3(LT), L_LDS, s, tmp, kf + h0 * M, tw,
                               g.flA, g.flB, g.A, false);
            FC_HIP(hipGetLastError());
            hipLaunchKernelGGL(k_long_inv_cols_y<IO>, dim3((unsigned)g.A, (unsigned)nh), dim3(LT), L_LDS, s,
                               (const float2 *)tmp, y + o0, two ? y + o0 + H * N : nullptr, tw, g.flA, g.A, g.C, N);
            FC_HIP(hipGetLastError());
        }
        b += as_real ? 1 : 2;
    }
    return FFTCONV_OK;
}

}  // namespace

// rows of fft_size = A * 8192, A = 2 .. 512; a row index must fit the grid's second dimension
bool long_fft_supported(const fftconv_plan *p) { return p->M >= 2 * LB && p->M <= 512 * (int64_t)LB && p->H <= 65535; }

int long_fft_init(fftconv_plan *p)
{
    const int64_t M = p->M, nhi = M / 2048;
    std::vector<float2> t((size_t)(LB + 2048 + nhi));
    const double two_pi = 6.283185307179586476925286766559;
    auto wpow = [&](double num, double den) {
        const double a = two_pi * num / den;
        return make_float2((float)std::cos(a), (float)-std::sin(a));
    };
    for (int64_t i = 0; i < LB; ++i) t[(size_t)i] = wpow((double)i, (double)LB);
    for (int64_t i = 0; i < 2048; ++i) t[(size_t)(LB + i)] = wpow((double)i, (double)M);
    for (int64_t i = 0; i < nhi; ++i) t[(size_t)(LB + 2048 + i)] = wpow((double)i, (double)nhi);
    FC_HIP(hipMalloc((void **)&p->long_tw, t.size() * sizeof(float2)));
    FC_HIP(hipMemcpy(p->long_tw, t.data(), t.size() * sizeof(float2), hipMemcpyHostToDevice));
    return FFTCONV_OK;
}

void long_fft_destroy(fftconv_plan *p)
{
    if (p->long_tw) (void)hipFree(p->long_tw);
    p->long_tw = nullptr;
}

// The filter transform of channels [h0, h0 + nh) of a multi-pass plan: taps (nh, Nk) -> their rows of k_f; tmp holds
// nh * M float2.  adjoint: the spectrum of the circularly time-reversed filter (the conjugate spectrum).
int long_filter_transform(const fftconv_plan *p, const float *k, int64_t Nk, int64_t h0, int64_t nh, bool adjoint,
                          const uint8_t *keep_dev, int64_t n_blocks, float2 *tmp, void *kf, hipStream_t s)
{
    const LongGeo g = long_geo(p->M);
    const LongTw tw = long_tw(p);
    if (g.flB.nf != 4 || g.flB.fac[0] != 16 || g.flB.fac[1] != 16 || g.flB.fac[2] != 16 || g.flB.fac[3] != 2) {
        set_error("multi-pass filter transform: the block transform's factors are not 16, 16, 16, 2");
        return FFTCONV_EUNSUPPORTED;
    }
    // outer factor: the register kernel of the multi-pass route where it exists for this outer length (rows ko <= A/2
    // in natural order; the adjoint spectrum is then the conjugate, taken on the way out), else the generic column kernel
    const bool natural = multipass_filter_outer_ok(p);
    int rc = natural ? multipass_filter_outer(p, k, FFTCONV_F32, Nk, nh, tmp, s)
                     : launch_fwd_cols<float>(g, k, nullptr, tmp, tw, nh, Nk, adjoint, s, true);
    if (rc) return rc;
    rc = raise_lds((const void *)k_long_fwd_blocks_kf<true>);
    if (!rc) rc = raise_lds((const void *)k_long_fwd_blocks_kf<false>);
    if (rc) return rc;
    const dim3 grid((unsigned)(natural ? g.A / 2 + 1 : g.A), (unsigned)nh);
    if (p->dtype == FFTCONV_F16)
        hipLaunchKernelGGL(k_long_fwd_blocks_kf<true>, grid, dim3(LT), L_LDS, s, tmp, (uint32_t *)kf, tw, g.flA, g.flB, g.A, h0,
                           keep_dev, n_blocks, natural, natural && adjoint);
    else
        hipLaunchKernelGGL(k_long_fwd_blocks_kf<false>, grid, dim3(LT), L_LDS, s, tmp, (uint32_t *)kf, tw, g.flA, g.flB, g.A, h0,
                           keep_dev, n_blocks, natural, natural && adjoint);
    FC_HIP(hipGetLastError());
    return FFTCONV_OK;
}

// The filter transform of channels [h0, h0 + nh) of a plan that keeps k_f as fp32 pairs in the position order of
// long_fft_factor_list() (fp32 I/O, fft_size 32768 .. 2^21): the real outer pass and the block transforms of the
// rows ko <= A/2, as above.  tmp holds nh * (A/2 + 1) * 8192 float2.  Needs multipass_filter_outer_ok(p).
int long_filter_transform_f32(const fftconv_plan *p, const float *k, int64_t Nk, int64_t h0, int64_t nh, bool adjoint,
                              const uint8_t *keep_dev, int64_t n_blocks, float2 *tmp, void *kf, hipStream_t s)
{
    const LongGeo g = long_geo(p->M);
    const LongTw tw = long_tw(p);
    if (g.flB.nf != 4 || g.flB.fac[0] != 16 || g.flB.fac[1] != 16 || g.flB.fac[2] != 16 || g.flB.fac[3] != 2) {
        set_error("long filter transform: the block transform's factors are not 16, 16, 16, 2");
        return FFTCONV_EUNSUPPORTED;
    }
    int rc = multipass_filter_outer(p, k, FFTCONV_F32, Nk, nh, tmp, s);
    if (rc) return rc;
    rc = raise_lds((const void *)k_long_fwd_blocks_kf32);
    if (rc) return rc;
    hipLaunchKernelGGL(k_long_fwd_blocks_kf32, dim3((unsigned)(g.A / 2 + 1), (unsigned)nh), dim3(LT), L_LDS, s, tmp,
                       (float2 *)kf, tw, g.flA, g.flB, g.A, h0, keep_dev, n_blocks, adjoint);
    FC_HIP(hipGetLastError());
    return FFTCONV_OK;
}

// The position order of the spectra of these transforms (k_f of the fp32 plans from fft_size 32768 up is stored in it)
FacList long_fft_factor_list(int64_t M) { return long_geo(M).fl; }

size_t long_forward_workspace_bytes(const fftconv_plan *p)
{
    return p->M <= 2 * LB ? 0 : (size_t)(conv_chunk(p) * p->M) * sizeof(float2);
}

// fp32 forward pass of the plans without a 16-bit kernel (fft_size >= 8192); kf: (H, fft_size) fp32 pairs in position order
int long_forward(const fftconv_plan *p, const void *u, const void *kf, void *y, int64_t B, void *workspace, hipStream_t s)
{
    switch (p->dtype) {
    case FFTCONV_F32: return long_forward_t<float>(p, (const float *)u, (const float2 *)kf, (float *)y, B, workspace, s);
    case FFTCONV_F16:
        return long_forward_t<__half>(p, (const __half *)u, (const float2 *)kf, (__half *)y, B, workspace, s);
    default:
        return long_forward_t<__hip_bfloat16>(p, (const __hip_bfloat16 *)u, (const float2 *)kf, (__hip_bfloat16 *)y, B,
                                              workspace, s);
    }
}

size_t long_backward_filter_bytes(const fftconv_plan *p) { return (size_t)(3 * p->H * p->M) * sizeof(float2); }

int long_backward_filter(const fftconv_plan *p, const void *u, const void *dy, float *dk, int64_t Nk, int64_t B,
                         void *workspace, hipStream_t s)
{
    switch (p->dtype) {
    case FFTCONV_F32: return long_backward_filter_t<float>(p, (const float *)u, (const float *)dy, dk, Nk, B, workspace, s);
    case FFTCONV_F16:
        return long_backward_filter_t<__half>(p, (const __half *)u, (const __half *)dy, dk, Nk, B, workspace, s);
    default:
        return long_backward_filter_t<__hip_bfloat16>(p, (const __hip_bfloat16 *)u, (const __hip_bfloat16 *)dy, dk, Nk, B,
                                                      workspace, s);
    }
}

}  // namespace fftconv
