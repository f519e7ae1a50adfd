// Micro-benchmarks behind the machine constants of the cost model (paper Section 3.2, Eq. 2), measured the
// way Appendix C ("Empirical GPU Profiling") describes for its table of constants:
//   sigma_H  achievable HBM bandwidth: a plain copy of a large tensor (the paper clones a tensor), bytes
//            read plus bytes written per second;
//   tau_M    achievable matrix-unit rate: 16-bit matrix products issued back to back on every SIMD
//            (v_mfma_f32_16x16x32_bf16, the instruction every DFT-matrix product of the library uses);
//   tau_G    achievable general arithmetic rate: twiddle factors applied over and over (fp32 complex
//            products on the vector ALUs, 6 floating-point operations each);
//   sigma_S  achievable on-chip bandwidth: the slow-down from passing intermediate results through LDS
//            between matrix products (a chain of products whose 16-bit packed result goes straight into the
//            next product, against the same chain with a 16-byte-per-lane write and read of LDS in between).
// fftconv_measure_machine() runs them on the current device and fills an fftconv_machine.
#include <algorithm>

#include "fused3_common.h"

namespace fftconv {
namespace {

using f3::BF16;
using f3::f32x4;

constexpr int MB_THREADS = 256;             // 4 waves: one per SIMD of a compute unit
constexpr int MB_BLOCKS_PER_CU = 2;         // two waves per SIMD, as in the fused kernels

__global__ void __launch_bounds__(MB_THREADS) k_mb_copy(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

// MB_ACC independent accumulators per wave, `iters` rounds of MB_ACC products.  Sixteen, because a product
// that accumulates onto the result of an earlier one waits for it much longer than the 16 clocks between
// issues: with 8 accumulators the chip-wide rate measured 1.3 PFLOP/s, with 16 it is 2.26 (the fused
// kernels start nearly every product from a zero accumulator and do not meet this).
constexpr int MB_ACC = 16;
__global__ void __launch_bounds__(MB_THREADS) k_mb_mfma(float *__restrict__ out, int iters)
{
    const uint32_t l = threadIdx.x;
    const uint4 a = make_uint4(0x3f803f80u + l, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u);
    const uint4 b = make_uint4(0x3f803f80u, 0x3f803f80u + (l << 16), 0x3f803f80u, 0x3f803f80u);
    f32x4 acc[MB_ACC];
#pragma unroll
    for (int i = 0; i < MB_ACC; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < MB_ACC; ++i) acc[i] = BF16::mfma(a, b, acc[i]);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < MB_ACC; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// 8 complex values per thread, each multiplied by a unit-modulus twiddle `iters` times
__global__ void __launch_bounds__(MB_THREADS) k_mb_twiddle(float2 *__restrict__ out, int iters)
{
    const float ang = 1e-3f * (float)(threadIdx.x + 1);
    const float wr = cosf(ang), wi = sinf(ang);
    float zr[8], zi[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        zr[i] = 1.0f + 0.125f * i;
        zi[i] = 0.5f - 0.0625f * i;
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float r = zr[i] * wr - zi[i] * wi;
            const float m = zr[i] * wi + zi[i] * wr;
            zr[i] = r;
            zi[i] = m;
        }
    }
    float2 s = make_float2(0.f, 0.f);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        s.x += zr[i];
        s.y += zi[i];
    }
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// A chain of complex matrix products as the fused kernels run them: two products (real and imaginary part
// of the result), four packs to 16-bit (re, im) pairs, and the packed 16 bytes per lane become the operand of
// the next link.  VIA_LDS: the 16 bytes are written to LDS and read back from another lane's slot first.
template <bool VIA_LDS>
__global__ void __launch_bounds__(MB_THREADS) k_mb_chain(uint4 *__restrict__ out, int iters)
{
    __shared__ uint4 buf[MB_THREADS];
    const uint32_t t = threadIdx.x, l = t & 63u;
    const uint32_t partner = (t & ~63u) | ((l + 17u) & 63u);          // a slot of the same wave: no barrier needed
    const uint4 m0 = make_uint4(0x3d003d00u + l, 0x3d003d00u, 0x3d003d00u, 0x3d003d00u);
    const uint4 m1 = make_uint4(0x3d003d00u, 0x3d003d00u + l, 0x3d003d00u, 0x3d003d00u);
    uint4 x = make_uint4(0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u + l);
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
        const f32x4 dre = BF16::mfma(m0, x, zero);
        const f32x4 dim = BF16::mfma(m1, x, zero);
        x = make_uint4(BF16::pack(dre[0], dim[0]), BF16::pack(dre[1], dim[1]), BF16::pack(dre[2], dim[2]),
                       BF16::pack(dre[3], dim[3]));
        if constexpr (VIA_LDS) {
            buf[t] = x;
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");          // LDS operations of a wave complete in order
            x = buf[partner];
        }
    }
    out[(size_t)blockIdx.x * blockDim.x + t] = x;
}

// Shortest of `reps` timed launches, in seconds.  The core clock of this GPU needs tens of milliseconds of
// load to leave its idle state, so the same launch first runs back to back for about 150 ms, untimed.
template <typename Launch> int time_launch(Launch launch, int reps, double *seconds)
{
    hipEvent_t e0, e1;
    FC_HIP(hipEventCreate(&e0));
    FC_HIP(hipEventCreate(&e1));
    float spun = 0.f;
    while (spun < 150.f) {
        FC_HIP(hipEventRecord(e0, nullptr));
        for (int i = 0; i < 4; ++i) launch();
        FC_HIP(hipEventRecord(e1, nullptr));
        FC_HIP(hipEventSynchronize(e1));
        float ms = 0.f;
        FC_HIP(hipEventElapsedTime(&ms, e0, e1));
        spun += ms > 0.01f ? ms : 0.01f;
    }
    float best = 0.f;
    for (int r = 0; r < reps; ++r) {
        FC_HIP(hipEventRecord(e0, nullptr));
        launch();
        FC_HIP(hipEventRecord(e1, nullptr));
        FC_HIP(hipEventSynchronize(e1));
        float ms = 0.f;
        FC_HIP(hipEventElapsedTime(&ms, e0, e1));
        if (r == 0 || ms < best) best = ms;
    }
    FC_HIP(hipGetLastError());
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    *seconds = (double)best * 1e-3;
    return FFTCONV_OK;
}

}  // namespace
}  // namespace fftconv

using namespace fftconv;

extern "C" int fftconv_measure_machine(fftconv_machine *m)
{
    if (!m) {
        set_error("fftconv_measure_machine: m is NULL");
        return FFTCONV_EINVAL;
    }
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
        (void)hipGetLastError();
        set_error("fftconv_measure_machine: no usable GPU");
        return FFTCONV_ENODEV;
    }
    const int cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    const int grid = cus * MB_BLOCKS_PER_CU;
    const size_t copy_bytes = (size_t)1 << 30;
    const size_t out_bytes = (size_t)grid * MB_THREADS * sizeof(uint4);
    void *src = nullptr, *dst = nullptr, *out = nullptr;
    if (hipMalloc(&src, copy_bytes) != hipSuccess || hipMalloc(&dst, copy_bytes) != hipSuccess ||
        hipMalloc(&out, out_bytes) != hipSuccess) {
        (void)hipGetLastError();
        if (src) (void)hipFree(src);
        if (dst) (void)hipFree(dst);
        if (out) (void)hipFree(out);
        set_error("fftconv_measure_machine: device allocation failed");
        return FFTCONV_ENOMEM;
    }
    int rc = hipMemset(src, 1, copy_bytes) == hipSuccess ? FFTCONV_OK : FFTCONV_EHIP;
    double t_copy = 0, t_mfma = 0, t_tw = 0, t_chain = 0, t_chain_lds = 0;
    const int it_mfma = 16384, it_tw = 32768, it_chain = 32768;      // a few milliseconds per launch
    if (!rc)
        rc = time_launch([&] { hipLaunchKernelGGL(k_mb_copy, dim3(cus * 8), dim3(MB_THREADS), 0, nullptr, (const uint4 *)src,
                                                  (uint4 *)dst, copy_bytes / 16); }, 5, &t_copy);
    if (!rc)
        rc = time_launch([&] { hipLaunchKernelGGL(k_mb_mfma, dim3(grid), dim3(MB_THREADS), 0, nullptr, (float *)out, it_mfma); },
                         3, &t_mfma);
    if (!rc)
        rc = time_launch([&] { hipLaunchKernelGGL(k_mb_twiddle, dim3(grid), dim3(MB_THREADS), 0, nullptr, (float2 *)out, it_tw); },
                         3, &t_tw);
    if (!rc)
        rc = time_launch([&] { hipLaunchKernelGGL(k_mb_chain<false>, dim3(grid), dim3(MB_THREADS), 0, nullptr, (uint4 *)out,
                                                  it_chain); }, 3, &t_chain);
    if (!rc)
        rc = time_launch([&] { hipLaunchKernelGGL(k_mb_chain<true>, dim3(grid), dim3(MB_THREADS), 0, nullptr, (uint4 *)out,
                                                  it_chain); }, 3, &t_chain_lds);
    (void)hipFree(src);
    (void)hipFree(dst);
    (void)hipFree(out);
    if (rc) return rc;
    const double waves = (double)grid * (MB_THREADS / 64);
    m->sigma_H = 2.0 * (double)copy_bytes / t_copy;
    m->tau_M = waves * it_mfma * (double)MB_ACC * (2.0 * 16 * 16 * 32) / t_mfma;
    m->tau_G = (double)grid * MB_THREADS * it_tw * 8.0 * 6.0 / t_tw;
    // 16 bytes written and 16 bytes read per lane and link; the time they add to the chain
    const double lds_bytes = (double)grid * MB_THREADS * it_chain * 32.0;
    m->sigma_S = lds_bytes / std::max(t_chain_lds - t_chain, 1e-9);
    m->mu = 16;
    m->sram_seq = 32768;
    return FFTCONV_OK;
}
