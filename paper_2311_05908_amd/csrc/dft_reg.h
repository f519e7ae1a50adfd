// In-register DFTs of power-of-two length <= 32 on the vector ALUs, shared by the outer passes of the
// multi-pass path, the small-transform kernel (fp32) and the generic per-stage kernels (fp32, fp64).
#pragma once

#include <hip/hip_runtime.h>

namespace fftconv {

// cos / sin of 2 pi j / 32: every twiddle of the transforms below
__device__ constexpr float C32[32] = {1.000000000f, 0.980785280f, 0.923879533f, 0.831469612f, 0.707106781f, 0.555570233f, 0.382683432f, 0.195090322f, 0.000000000f, -0.195090322f, -0.382683432f, -0.555570233f, -0.707106781f, -0.831469612f, -0.923879533f, -0.980785280f, -1.000000000f, -0.980785280f, -0.923879533f, -0.831469612f, -0.707106781f, -0.555570233f, -0.382683432f, -0.195090322f, -0.000000000f, 0.195090322f, 0.382683432f, 0.555570233f, 0.707106781f, 0.831469612f, 0.923879533f, 0.980785280f};
__device__ constexpr float S32[32] = {0.000000000f, 0.195090322f, 0.382683432f, 0.555570233f, 0.707106781f, 0.831469612f, 0.923879533f, 0.980785280f, 1.000000000f, 0.980785280f, 0.923879533f, 0.831469612f, 0.707106781f, 0.555570233f, 0.382683432f, 0.195090322f, 0.000000000f, -0.195090322f, -0.382683432f, -0.555570233f, -0.707106781f, -0.831469612f, -0.923879533f, -0.980785280f, -1.000000000f, -0.980785280f, -0.923879533f, -0.831469612f, -0.707106781f, -0.555570233f, -0.382683432f, -0.195090322f};

// the first half in double precision, for the fp64 filter transform
__device__ constexpr double C32D[16] = {1.0, 0.9807852804032304, 0.9238795325112867, 0.8314696123025452, 0.7071067811865476, 0.5555702330196023, 0.38268343236508984, 0.19509032201612833, 0.0, -0.1950903220161282, -0.3826834323650897, -0.555570233019602, -0.7071067811865475, -0.8314696123025453, -0.9238795325112867, -0.9807852804032304};
__device__ constexpr double S32D[16] = {0.0, 0.19509032201612825, 0.3826834323650898, 0.5555702330196022, 0.7071067811865475, 0.8314696123025452, 0.9238795325112867, 0.9807852804032304, 1.0, 0.9807852804032304, 0.9238795325112867, 0.8314696123025455, 0.7071067811865476, 0.5555702330196022, 0.3826834323650899, 0.1950903220161286};

constexpr int bitrev(int v, int bits)
{
    int r = 0;
    for (int i = 0; i < bits; ++i) r |= ((v >> i) & 1) << (bits - 1 - i);
    return r;
}
constexpr int ilog2(int v) { return v <= 1 ? 0 : 1 + ilog2(v / 2); }

// In-register DFT of length R (power of two <= 32), natural order in and out, unnormalised;
// INV conjugates the kernel.  Radix-2 decimation in time, fully unrolled so every index and
// twiddle is a compile-time constant.
template <int R, bool INV> __device__ __forceinline__ void dft_reg(float2 (&x)[R])
{
    constexpr int LG = ilog2(R);
#pragma unroll
    for (int i = 0; i < R; ++i) {
        const int j = bitrev(i, LG);
        if (j > i) {
            const float2 t = x[i];
            x[i] = x[j];
            x[j] = t;
        }
    }
#pragma unroll
    for (int len = 2; len <= R; len *= 2) {
#pragma unroll
        for (int blk = 0; blk < R; blk += len) {
#pragma unroll
            for (int j = 0; j < len / 2; ++j) {
                const int q = j * (32 / len);                  // twiddle W_32^q, 0 <= q < 16
                const float2 a = x[blk + j], b = x[blk + j + len / 2];
                float2 t;
                if (q == 0) {
                    t = b;
                } else if (q == 8) {                           // -i forward, +i inverse
                    t = INV ? make_float2(-b.y, b.x) : make_float2(b.y, -b.x);
                } else {
                    const float wr = C32[q];
                    const float wi = INV ? S32[q] : -S32[q];
                    t = make_float2(b.x * wr - b.y * wi, b.x * wi + b.y * wr);
                }
                x[blk + j] = make_float2(a.x + t.x, a.y + t.y);
                x[blk + j + len / 2] = make_float2(a.x - t.x, a.y - t.y);
            }
        }
    }
}

// The same transform in double precision.
template <int R, bool INV> __device__ __forceinline__ void dft_reg(double2 (&x)[R])
{
    constexpr int LG = ilog2(R);
#pragma unroll
    for (int i = 0; i < R; ++i) {
        const int j = bitrev(i, LG);
        if (j > i) {
            const double2 t = x[i];
            x[i] = x[j];
            x[j] = t;
        }
    }
#pragma unroll
    for (int len = 2; len <= R; len *= 2) {
#pragma unroll
        for (int blk = 0; blk < R; blk += len) {
#pragma unroll
            for (int j = 0; j < len / 2; ++j) {
                const int q = j * (32 / len);                  // twiddle W_32^q, 0 <= q < 16
                const double2 a = x[blk + j], b = x[blk + j + len / 2];
                double2 t;
                if (q == 0) {
                    t = b;
                } else if (q == 8) {                           // -i forward, +i inverse
                    t = INV ? make_double2(-b.y, b.x) : make_double2(b.y, -b.x);
                } else {
                    const double wr = C32D[q];
                    const double wi = INV ? S32D[q] : -S32D[q];
                    t = make_double2(b.x * wr - b.y * wi, b.x * wi + b.y * wr);
                }
                x[blk + j] = make_double2(a.x + t.x, a.y + t.y);
                x[blk + j + len / 2] = make_double2(a.x - t.x, a.y - t.y);
            }
        }
    }
}

}  // namespace fftconv
