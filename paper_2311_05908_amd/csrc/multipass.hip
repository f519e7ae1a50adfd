// Multi-pass causal FFT convolution for transforms too long to keep on chip
// (paper Algorithm 4 and Section 3.1 "Kernel Fusion": the outermost matrix
// operation of the forward and of the inverse transform takes one trip through
// HBM each, everything inside stays fused).  16-bit I/O, fft_size M = No * Mi with
// Mi = 8192 (the fused inner transform) and No = M / Mi in [1, 512].  Causal shapes (N <= M/2)
// of the sizes the single-kernel paths do not take, and every shape with N > M/2 (circular
// convolution, Section 2.1: the input fills the transform) from M = 8192 up: the kernels are
// instantiated with and without the implicit zero half (FULLN).  No = 1 has no outer transform:
// pass A only packs a pair of rows into a complex row, pass C unpacks it.
//
// Index maps: time n = no*Mi + r, frequency f = ko + No*f'.  Then
//   W_M^{n f} = W_No^{no ko} * W_M^{r ko} * W_Mi^{r f'},
// so, with z = u[b] + i*u[b+1] (two batch rows share one complex transform because the
// filter is real),
//   pass A:  S[ko, r] = W_M^{r ko} * sum_{no < No/2} z[no*Mi + r] W_No^{no ko}     (zeros for no >= No/2
//            are implicit; the listing in the paper omits the twiddle, its prose names it)
//   pass B:  every row S[ko, :] is circularly convolved (length Mi, complex in / complex out,
//            fused kernel) with the spectrum row k_f[ko + No*f'] / M
//   pass C:  y[no*Mi + r] = sum_{ko} conj(W_M^{r ko} W_No^{no ko}) S[ko, r] / boost,  no < No/2;
//            real part -> row b, imaginary part -> row b+1.
// S lives in the caller's workspace as 16-bit (re, im) pairs, M per pair of rows, and is
// rewritten in place by pass B.  The outer DFT of length No is itself split in two
// (No = Ra * Rb, Ra = min(16, No)) inside one workgroup: in-register radix-2 butterflies on the
// vector ALUs in fp32, one thread per column, so HBM sees rows of consecutive columns.
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>

#include "dft_reg.h"
#include "fftconv_internal.h"

#include <mutex>

namespace fftconv {

// ---- workspace for callers that cannot allocate (fftconv_forward_static): one array per GPU, part of the
// library's device image, held until the process ends.  Host code never uses the array's name as an
// address: static_workspace_init() asks the runtime for the array's device address once per device and
// every later use goes through that pointer.
static __device__ __align__(256) unsigned char scratch[FFTCONV_STATIC_WORKSPACE_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
void *g_scratch_ptr[MAX_DEVICES] = {};          // device address of `scratch` on each device, nullptr = not asked yet
std::mutex g_scratch_mu;
}  // namespace

// with `device` current; called from plan creation
int static_workspace_init(int device)
{
    if (device < 0 || device >= MAX_DEVICES) {
        set_error("static workspace: device index %d out of range", device);
        return FFTCONV_EUNSUPPORTED;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (g_scratch_ptr[device]) return FFTCONV_OK;
    void *ptr = nullptr;
    FC_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    g_scratch_ptr[device] = ptr;
    return FFTCONV_OK;
}

void *static_workspace(int device)
{
    if (device < 0 || device >= MAX_DEVICES) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    return g_scratch_ptr[device];
}

namespace {

constexpr int MI = 8192;
constexpr int TB = 512;          // threads per block of the outer passes

__device__ __forceinline__ float2 cmulf(float2 a, float2 b)
{
    return make_float2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x);
}
__device__ __forceinline__ float2 cmulcf(float2 a, float2 b)      // a * conj(b)
{
    return make_float2(a.x * b.x + a.y * b.y, a.y * b.x - a.x * b.y);
}
// exp(-2 pi i e / M) for 0 <= e < M <= 2^22, inv_half_m = 2 / M: e / M is exact in fp32 and goes straight to
// the hardware sine and cosine, which take their argument in revolutions (two quarter-rate instructions
// instead of the ~25 of the library routine).  Their absolute error over every e / 2^22 measures 1.3e-7, far
// below the 16-bit roundings of the values these twiddles multiply.
__device__ __forceinline__ float2 wm(int e, float inv_half_m)
{
    const float rev = (float)e * (0.5f * inv_half_m);
    return make_float2(__builtin_amdgcn_cosf(rev), -__builtin_amdgcn_sinf(rev));
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

// elementwise product of two packed pairs of 16-bit values, each product rounded to the I/O dtype (the
// gates of the gated form, Section 3.1: the rounded product is what the transform consumes / what is stored)
template <bool F16> __device__ __forceinline__ uint32_t mul_pair16(uint32_t a, uint32_t b)
{
    const float2 x = unpack2<F16>(a), g = unpack2<F16>(b);
    return (uint32_t)cv16<F16>(x.x * g.x) | ((uint32_t)cv16<F16>(x.y * g.y) << 16);
}

struct OuterGeo {
    int No, Ra, Rb, CT;          // outer length, its two factors, columns per block
};

// ---- pass A: zero-padded pair of real rows -> outer forward DFT (No = RA * RB) -> twiddle -> S.
// One block = CT consecutive columns r of one (pair, channel); one thread = CV adjacent columns of
// one butterfly, so that 16-bit input moves as 2*CV-byte and S as 4*CV-byte accesses.
// Step 1: for every b2 < RB the length-RA transform over a (unless FULLN, inputs a >= RA/2 are the
// implicit zeros), times W_No^{ka b2}, into the fp32 LDS tile T[ka*RB + b2][c].  Step 2: for every ka the
// length-RB transform over b2, times W_M^{r ko} (ko = ka + RA kb, by recurrence over kb), to S.
// EXACT (all four outer kernels): N is even and equals the input length the instantiation is for (M/2, or M
// with FULLN), so every load of u and store of y is in range, 4-byte aligned and unconditional: the compiler
// can then issue a thread's loads back to back instead of one guarded load at a time.
template <bool F16, int RA, int RB, int CV, bool FULLN, bool GATED, bool EXACT>
__global__ void __launch_bounds__(TB, 4) k_outer_fwd(const uint16_t *__restrict__ u, uint32_t *__restrict__ S, int CT,
                                                 int B, int H, int N, int64_t M, int ko_lo, int ko_hi,
                                                 const uint16_t *__restrict__ wg, LaunchGate gate)
{
    extern __shared__ float2 sm[];
    if (gate_closed(gate)) return;
    constexpr int No = RA * RB;
    constexpr int RAIN = FULLN ? RA : RA / 2;      // outer rows that can hold input
    float2 *wno = sm;                              // W_No^j, j < No
    float2 *T = sm + No;                           // [No][CT]
    const int tid = threadIdx.x;
    const int r0 = blockIdx.x * CT;
    const int ph = blockIdx.y;                     // pair * H + h
    const int pair = ph / H, h = ph % H;
    const int b0 = 2 * pair;
    const bool two = b0 + 1 < B;
    const uint16_t *row0 = u + ((size_t)b0 * H + h) * N;
    const uint16_t *row1 = u + ((size_t)(b0 + (two ? 1 : 0)) * H + h) * N;
    // input gate of the gated form (same shape as u), multiplied in as the samples arrive; nullptr = none
    const uint16_t *g0 = GATED ? wg + ((size_t)b0 * H + h) * N : nullptr;
    const uint16_t *g1 = GATED ? wg + ((size_t)(b0 + (two ? 1 : 0)) * H + h) * N : nullptr;
    const bool wide = CV == 2 && (EXACT || N % 2 == 0);       // rows start 4-byte aligned
    const int CG = CT / CV;                        // column groups, a power of two
    const int lgCG = 31 - __builtin_clz(CG);
    for (int j = tid; j < No; j += TB) wno[j] = wm(j, 2.0f / (float)No);
    __syncthreads();
    for (int e = tid; e < RB * CG; e += TB) {
        const int c = (e & (CG - 1)) * CV, b2 = e >> lgCG;
        uint32_t in0[RAIN], in1[RAIN];             // CV 16-bit values of row b / row b+1
        uint32_t gt0[GATED ? RAIN : 1], gt1[GATED ? RAIN : 1];
#pragma unroll
        for (int a = 0; a < RAIN; ++a) {
            const int64_t n = (int64_t)(a * RB + b2) * MI + r0 + c;
            in0[a] = in1[a] = 0;
            if constexpr (GATED) gt0[a] = gt1[a] = 0;
            if (wide) {
                // a pair beyond N (n and N are even: in or out as a whole) reads sample 0 and is discarded below, a
                // missing row b+1 reads row b: the loads need no branch and go out back to back
                const int64_t at = (EXACT || n < N) ? n : 0;
                in0[a] = *(const uint32_t *)(row0 + at);
                in1[a] = *(const uint32_t *)(row1 + at);
                if constexpr (GATED) {
                    gt0[a] = *(const uint32_t *)(g0 + at);
                    gt1[a] = *(const uint32_t *)(g1 + at);
                }
            } else {
#pragma unroll
                for (int v = 0; v < CV; ++v)
                    if (EXACT || n + v < N) {
                        in0[a] |= (uint32_t)row0[n + v] << (16 * v);
                        if (two) in1[a] |= (uint32_t)row1[n + v] << (16 * v);
                        if constexpr (GATED) {
                            gt0[a] |= (uint32_t)g0[n + v] << (16 * v);
                            if (two) gt1[a] |= (uint32_t)g1[n + v] << (16 * v);
                        }
                    }
            }
        }
        if (wide) {
#pragma unroll
            for (int a = 0; a < RAIN; ++a) {
                asm volatile("" ::"v"(in0[a]), "v"(in1[a]));             // keeps the loads unconditional
                if constexpr (GATED) asm volatile("" ::"v"(gt0[a]), "v"(gt1[a]));
            }
#pragma unroll
            for (int a = 0; a < RAIN; ++a) {
                const int64_t n = (int64_t)(a * RB + b2) * MI + r0 + c;
                const bool in = EXACT || n < N;
                if (!in) in0[a] = 0;
                if (!in || !two) in1[a] = 0;
                if constexpr (GATED) {                                    // (0 times a discarded gate must stay 0)
                    if (!in) gt0[a] = 0;
                    if (!in || !two) gt1[a] = 0;
                }
            }
        }
        if constexpr (GATED) {
#pragma unroll
            for (int a = 0; a < RAIN; ++a) {
                in0[a] = mul_pair16<F16>(in0[a], gt0[a]);
                in1[a] = mul_pair16<F16>(in1[a], gt1[a]);
            }
        }
        float2 o[RA][CV];
#pragma unroll
        for (int v = 0; v < CV; ++v) {
            float2 x[RA];
#pragma unroll
            for (int a = 0; a < RA; ++a) {
                x[a] = make_float2(0.f, 0.f);
                if (a < RAIN)                                        // (row b, row b+1) = (re, im)
                    x[a] = unpack2<F16>(((in0[a] >> (16 * v)) & 0xffffu) | ((in1[a] >> (16 * v)) << 16));
            }
            dft_reg<RA, false>(x);
#pragma unroll
            for (int ka = 0; ka < RA; ++ka) o[ka][v] = cmulf(x[ka], wno[ka * b2]);
        }
#pragma unroll
        for (int ka = 0; ka < RA; ++ka) {
            float2 *dst = &T[(ka * RB + b2) * CT + c];
            if constexpr (CV == 2)
                *(float4 *)dst = make_float4(o[ka][0].x, o[ka][0].y, o[ka][1].x, o[ka][1].y);
            else
                *dst = o[ka][0];
        }
    }
    __syncthreads();
    const float ihm = 2.0f / (float)M;
    const int Mmask = (int)M - 1;                  // M is a power of two, at most 2^22, and so is every r * ko
    for (int e = tid; e < RA * CG; e += TB) {
        const int c = (e & (CG - 1)) * CV, ka = e >> lgCG;
        uint32_t o[RB][CV];
#pragma unroll
        for (int v = 0; v < CV; ++v) {
            float2 x[RB];
#pragma unroll
            for (int b2 = 0; b2 < RB; ++b2) x[b2] = T[(ka * RB + b2) * CT + c + v];
            dft_reg<RB, false>(x);
            const int r = r0 + c + v;
            float2 w = wm((r * ka) & Mmask, ihm);                 // W_M^{r ka}
            const float2 step = wm((r * RA) & Mmask, ihm);        // W_M^{r RA}
#pragma unroll
            for (int kb = 0; kb < RB; ++kb) {
                const float2 t = cmulf(x[kb], w);
                o[kb][v] = (uint32_t)cv16<F16>(t.x) | ((uint32_t)cv16<F16>(t.y) << 16);
                w = cmulf(w, step);
            }
        }
        auto put = [&](int kb) {
            uint32_t *dst = &S[((size_t)ph * No + ka + RA * kb) * MI + multipass_row_slot(r0 + c, multipass_quarter_rows(No))];
            if constexpr (CV == 2)
                *(uint2 *)dst = make_uint2(o[kb][0], o[kb][1]);
            else
                *dst = o[kb][0];
        };
        if (ko_lo >= ko_hi) {                             // dense: unconditional stores, back to back
#pragma unroll
            for (int kb = 0; kb < RB; ++kb) put(kb);
        } else {
            // frequency-sparse filter: rows of a zeroed part of the spectrum are never used
#pragma unroll
            for (int kb = 0; kb < RB; ++kb) {
                const int ko = ka + RA * kb;
                if (ko < ko_lo || ko >= ko_hi) put(kb);
            }
        }
    }
}

// ---- pass C: S -> conjugate twiddle -> outer inverse DFT -> the two real rows of the pair
template <bool F16, int RA, int RB, int CV, bool FULLN, bool GATED, bool MIRROR, bool EXACT>
__global__ void __launch_bounds__(TB, 4) k_outer_inv(const uint32_t *__restrict__ S, uint16_t *__restrict__ y, int CT,
                                                 int B, int H, int N, int64_t M, int ko_lo, int ko_hi, int mirror_from,
                                                 const uint16_t *__restrict__ vg, LaunchGate gate)
{
    extern __shared__ float2 sm[];
    if (gate_closed(gate)) return;
    constexpr int No = RA * RB;
    constexpr int RAIN = FULLN ? RA : RA / 2;      // outer rows that are kept
    float2 *wno = sm;
    float2 *T = sm + No;                           // [No][CT]
    const int tid = threadIdx.x;
    const int r0 = blockIdx.x * CT;
    const int ph = blockIdx.y;
    const int pair = ph / H, h = ph % H;
    const int b0 = 2 * pair;
    const bool two = b0 + 1 < B;
    const bool wide = CV == 2 && (EXACT || N % 2 == 0);
    const int CG = CT / CV;
    const int lgCG = 31 - __builtin_clz(CG);
    for (int j = tid; j < No; j += TB) wno[j] = wm(j, 2.0f / (float)No);
    __syncthreads();
    const float ihm = 2.0f / (float)M;
    const int Mmask = (int)M - 1;                  // M is a power of two, at most 2^22, and so is every r * ko
    // step 1: T[ka*RB + b2] = conj(W_No^{ka b2}) * sum_{kb} conj(W_RB^{b2 kb}) conj(W_M^{r ko}) S[ko], ko = ka + RA kb
    // MIRROR (mirror_from == No/2 + 1): rows ko > No/2 were never computed (a lone real row, see multipass_forward): before the
    // twiddle row ko is the complex conjugate of row ko' = No - ko, i.e.
    //   conj(W_M^{r ko}) S[ko] = conj(conj(W_M^{r ko'}) S[ko']),   W_M^{r ko'} = W_Mi^{r} conj(W_M^{r ko}),
    // so the value that enters the inverse is conj(S[ko']) conj(conj(W_Mi^{r}) W_M^{r ko}): the mirror row is
    // read and conjugated (a sign flip on the packed word), and from the first mirrored row on the twiddle of the
    // recurrence carries the extra factor conj(W_Mi^{r}).
    for (int e = tid; e < RA * CG; e += TB) {
        const int c = (e & (CG - 1)) * CV, ka = e >> lgCG;
        uint32_t in[RB][CV];
#pragma unroll
        for (int kb = 0; kb < RB; ++kb) {
            const int ko = ka + RA * kb;
            // ko = ka + RA kb > No/2 = RA RB/2, written so that only kb == RB/2 depends on the thread
            const bool mir = MIRROR && (RB == 1 ? ka > RA / 2 : (kb > RB / 2 || (kb == RB / 2 && ka > 0)));
            // zeroed part of the spectrum: the row counts as zero and was never written.  The load stays
            // unconditional (of row 0 instead, its value discarded), so that a thread's loads go out back to
            // back: behind a branch each of them would be waited for before the next is issued.
            const bool dead = ko >= ko_lo && ko < ko_hi;
            const uint32_t *src = &S[((size_t)ph * No + (dead ? 0 : (mir ? No - ko : ko))) * MI + multipass_row_slot(r0 + c, multipass_quarter_rows(No))];
            if constexpr (CV == 2) {
                const uint2 t = *(const uint2 *)src;
                in[kb][0] = t.x;
                in[kb][1] = t.y;
            } else {
                in[kb][0] = *src;
            }
        }
        // (an empty statement that reads the loaded words: without it the compiler moves each load back under its
        //  condition)
#pragma unroll
        for (int kb = 0; kb < RB; ++kb)
#pragma unroll
            for (int v = 0; v < CV; ++v) asm volatile("" ::"v"(in[kb][v]));
#pragma unroll
        for (int kb = 0; kb < RB; ++kb) {
            const int ko = ka + RA * kb;
            const bool mir = MIRROR && (RB == 1 ? ka > RA / 2 : (kb > RB / 2 || (kb == RB / 2 && ka > 0)));
            if (ko >= ko_lo && ko < ko_hi) {
#pragma unroll
                for (int v = 0; v < CV; ++v) in[kb][v] = 0;
            }
            if (mir) {                                        // conjugate: the imaginary part is the upper half
#pragma unroll
                for (int v = 0; v < CV; ++v) in[kb][v] ^= 0x80000000u;
            }
        }
        float2 o[RB][CV];
#pragma unroll
        for (int v = 0; v < CV; ++v) {
            const int r = r0 + c + v;
            float2 w = wm((r * ka) & Mmask, ihm);
            const float2 step = wm((r * RA) & Mmask, ihm);
            constexpr float unboost = 1.0f / (float)multipass_kf_boost(F16, No);     // exact: a power of two
            w.x *= unboost;
            w.y *= unboost;
            float2 x[RB];
#pragma unroll
            for (int kb = 0; kb < RB; ++kb) {
                // the first mirrored row of this thread: kb = RB/2 (ka > 0) or RB/2 + 1 (ka == 0)
                const bool first_mirrored = RB == 1 ? ka > RA / 2
                                                    : ((kb == RB / 2 && ka > 0) || (kb == RB / 2 + 1 && ka == 0));
                if (MIRROR && first_mirrored)
                    w = cmulcf(w, wm((r * No) & Mmask, ihm));        // times conj(W_Mi^{r}), once
                x[kb] = cmulcf(unpack2<F16>(in[kb][v]), w);
                w = cmulf(w, step);
            }
            dft_reg<RB, true>(x);
#pragma unroll
            for (int b2 = 0; b2 < RB; ++b2) o[b2][v] = cmulcf(x[b2], wno[ka * b2]);
        }
#pragma unroll
        for (int b2 = 0; b2 < RB; ++b2) {
            float2 *dst = &T[(ka * RB + b2) * CT + c];
            if constexpr (CV == 2)
                *(float4 *)dst = make_float4(o[b2][0].x, o[b2][0].y, o[b2][1].x, o[b2][1].y);
            else
                *dst = o[b2][0];
        }
    }
    __syncthreads();
    // step 2: z[a*RB + b2] = sum_{ka} conj(W_RA^{a ka}) T[ka*RB + b2], kept for a < RAIN (n < M/2 unless FULLN)
    uint16_t *row0 = y + ((size_t)b0 * H + h) * N;
    uint16_t *row1 = y + ((size_t)(b0 + (two ? 1 : 0)) * H + h) * N;
    // output gate of the gated form: multiplies the result after its rounding to the I/O dtype; nullptr = none
    const uint16_t *g0 = GATED ? vg + ((size_t)b0 * H + h) * N : nullptr;
    const uint16_t *g1 = GATED ? vg + ((size_t)(b0 + (two ? 1 : 0)) * H + h) * N : nullptr;
    for (int e = tid; e < RB * CG; e += TB) {
        const int c = (e & (CG - 1)) * CV, b2 = e >> lgCG;
        uint32_t o0[RAIN], o1[RAIN];
#pragma unroll
        for (int a = 0; a < RAIN; ++a) o0[a] = o1[a] = 0;
#pragma unroll
        for (int v = 0; v < CV; ++v) {
            float2 x[RA];
#pragma unroll
            for (int ka = 0; ka < RA; ++ka) x[ka] = T[(ka * RB + b2) * CT + c + v];
            dft_reg<RA, true>(x);
#pragma unroll
            for (int a = 0; a < RAIN; ++a) {
                o0[a] |= (uint32_t)cv16<F16>(x[a].x) << (16 * v);
                o1[a] |= (uint32_t)cv16<F16>(x[a].y) << (16 * v);
            }
        }
#pragma unroll
        for (int a = 0; a < RAIN; ++a) {
            const int64_t n = (int64_t)(a * RB + b2) * MI + r0 + c;
            if (wide) {
                if (EXACT || n < N) {
                    if constexpr (GATED) {
                        o0[a] = mul_pair16<F16>(o0[a], *(const uint32_t *)(g0 + n));
                        if (two) o1[a] = mul_pair16<F16>(o1[a], *(const uint32_t *)(g1 + n));
                    }
                    *(uint32_t *)(row0 + n) = o0[a];
                    if (two) *(uint32_t *)(row1 + n) = o1[a];
                }
            } else {
#pragma unroll
                for (int v = 0; v < CV; ++v)
                    if (EXACT || n + v < N) {
                        uint32_t a0 = (o0[a] >> (16 * v)) & 0xffffu, a1 = (o1[a] >> (16 * v)) & 0xffffu;
                        if constexpr (GATED) {
                            a0 = mul_pair16<F16>(a0, g0[n + v]) & 0xffffu;
                            if (two) a1 = mul_pair16<F16>(a1, g1[n + v]) & 0xffffu;
                        }
                        row0[n + v] = (uint16_t)a0;
                        if (two) row1[n + v] = (uint16_t)a1;
                    }
            }
        }
    }
}

// ---- the outer passes of a LONE real row (B = 1, or the last row of an odd batch): two adjacent columns of
// the real row share one complex outer transform, z[no] = x[no, c] + i x[no, c+1] (Appendix A.1's point that a
// real transform costs half a complex one, taken on the column pairs of the outer factor), and only the
// outer frequencies ko <= No/2 are kept (the others are their conjugates, see multipass_forward).
//   pass A:  Z = DFT_No(z);  X_c[ko] = (Z[ko] + conj Z[No-ko]) / 2,  X_{c+1}[ko] = (Z[ko] - conj Z[No-ko]) / (2i);
//            S[ko, r] = W_M^{r ko} X_r[ko] for ko <= No/2.
//   pass C:  U_r[ko] = conj(W_M^{r ko}) S[ko, r] (ko <= No/2), U_r[ko] = conj(U_r[No-ko]) (ko > No/2);
//            z = IDFT_No(U_c + i U_{c+1}): its real part is column c of y, its imaginary part column c+1.
// One block = 2 CG consecutive columns of one channel, T[No][CG] in LDS; a 16-bit pair of adjacent samples
// is one 32-bit word, so a wave moves whole 128-byte lines of u and y.
template <bool F16, int RA, int RB, bool FULLN, bool GATED, bool EXACT>
__global__ void __launch_bounds__(TB, 4) k_outer_fwd_real(const uint16_t *__restrict__ u, uint32_t *__restrict__ S, int CG,
                                                      int H, int N, int64_t M, int ko_lo, const uint16_t *__restrict__ wg,
                                                      LaunchGate gate)
{
    extern __shared__ float2 sm[];
    if (gate_closed(gate)) return;
    constexpr int No = RA * RB;
    constexpr int RAIN = FULLN ? RA : RA / 2;      // outer rows that can hold input
    float2 *wno = sm;                              // W_No^j, j < No
    float2 *T = sm + No;                           // [No][CG]
    const int tid = threadIdx.x;
    const int r0 = blockIdx.x * 2 * CG;
    const int lgCG = 31 - __builtin_clz(CG);       // CG is a power of two
    const int h = blockIdx.y;
    const uint16_t *row0 = u + (size_t)h * N;
    const uint16_t *g0 = GATED ? wg + (size_t)h * N : nullptr;
    const bool wide = EXACT || N % 2 == 0;         // rows start 4-byte aligned
    for (int j = tid; j < No; j += TB) wno[j] = wm(j, 2.0f / (float)No);
    __syncthreads();
    // step 1: length-RA transforms over a, times W_No^{ka b2}
    for (int e = tid; e < RB * CG; e += TB) {
        const int cg = e & (CG - 1), b2 = e >> lgCG;
        float2 x[RA];
        uint32_t wd[RAIN], gt[GATED ? RAIN : 1];
#pragma unroll
        for (int a = 0; a < RAIN; ++a) {
            const int64_t n = (int64_t)(a * RB + b2) * MI + r0 + 2 * cg;
            wd[a] = 0;
            if constexpr (GATED) gt[a] = 0;
            if (wide) {
                // a pair beyond N (n and N are even: in or out as a whole) reads sample 0 and is discarded below: the
                // loads need no branch and go out back to back
                const int64_t at = (EXACT || n < N) ? n : 0;
                wd[a] = *(const uint32_t *)(row0 + at);
                if constexpr (GATED) gt[a] = *(const uint32_t *)(g0 + at);
            } else {
#pragma unroll
                for (int v = 0; v < 2; ++v)
                    if (EXACT || n + v < N) {
                        wd[a] |= (uint32_t)row0[n + v] << (16 * v);
                        if constexpr (GATED) gt[a] |= (uint32_t)g0[n + v] << (16 * v);
                    }
            }
        }
        if (wide && !EXACT) {
#pragma unroll
            for (int a = 0; a < RAIN; ++a) {
                asm volatile("" ::"v"(wd[a]));                           // keeps the loads unconditional
                if constexpr (GATED) asm volatile("" ::"v"(gt[a]));
            }
#pragma unroll
            for (int a = 0; a < RAIN; ++a) {
                const int64_t n = (int64_t)(a * RB + b2) * MI + r0 + 2 * cg;
                if (n >= N) {
                    wd[a] = 0;
                    if constexpr (GATED) gt[a] = 0;                      // (0 times a discarded gate must stay 0)
                }
            }
        }
#pragma unroll
        for (int a = 0; a < RA; ++a) {
            x[a] = make_float2(0.f, 0.f);
            if (a < RAIN) {
                if constexpr (GATED) wd[a] = mul_pair16<F16>(wd[a], gt[a]);
                x[a] = unpack2<F16>(wd[a]);        // (column c, column c+1) = (re, im)
            }
        }
        dft_reg<RA, false>(x);
#pragma unroll
        for (int ka = 0; ka < RA; ++ka) T[(ka * RB + b2) * CG + cg] = cmulf(x[ka], wno[ka * b2]);
    }
    __syncthreads();
    // step 2: length-RB transforms over b2, in place: slot ka*RB + kb then holds Z[ko], ko = ka + RA kb
    for (int e = tid; e < RA * CG; e += TB) {
        const int cg = e & (CG - 1), ka = e >> lgCG;
        float2 x[RB];
#pragma unroll
        for (int b2 = 0; b2 < RB; ++b2) x[b2] = T[(ka * RB + b2) * CG + cg];
        dft_reg<RB, false>(x);
#pragma unroll
        for (int kb = 0; kb < RB; ++kb) T[(ka * RB + kb) * CG + cg] = x[kb];
    }
    __syncthreads();
    // step 3: split the two columns, twiddle (by recurrence over kb), store the rows ko <= No/2
    const float ihm = 2.0f / (float)M;
    const int Mmask = (int)M - 1;                  // M is a power of two, at most 2^22, and so is every r * ko
    for (int e = tid; e < RA * CG; e += TB) {
        const int cg = e & (CG - 1), ka = e >> lgCG;
        const int r = r0 + 2 * cg;
        float2 w0 = wm((r * ka) & Mmask, ihm), w1 = wm(((r + 1) * ka) & Mmask, ihm);
        const float2 s0 = wm((r * RA) & Mmask, ihm), s1 = wm(((r + 1) * RA) & Mmask, ihm);
#pragma unroll
        for (int kb = 0; kb < RB && kb <= RB / 2; ++kb) {          // ko = ka + RA kb <= No/2 needs kb <= RB/2
            const int ko = ka + RA * kb;
            if (ko <= No / 2 && ko < ko_lo) {         // (rows from ko_lo on only meet zeroed bins of a sparse filter)
                const int km = (No - ko) % No;
                const float2 z = T[(ka * RB + kb) * CG + cg], zm = T[((km % RA) * RB + km / RA) * CG + cg];
                const float2 xa = make_float2(0.5f * (z.x + zm.x), 0.5f * (z.y - zm.y));      // (Z + conj Zm) / 2
                const float2 xb = make_float2(0.5f * (z.y + zm.y), -0.5f * (z.x - zm.x));     // (Z - conj Zm) / (2i)
                const float2 ta = cmulf(xa, w0), tb = cmulf(xb, w1);
                *(uint2 *)&S[((size_t)h * No + ko) * MI + multipass_row_slot(r, multipass_quarter_rows(No))] =
                    make_uint2((uint32_t)cv16<F16>(ta.x) | ((uint32_t)cv16<F16>(ta.y) << 16),
                               (uint32_t)cv16<F16>(tb.x) | ((uint32_t)cv16<F16>(tb.y) << 16));
            }
            w0 = cmulf(w0, s0);
            w1 = cmulf(w1, s1);
        }
    }
}

template <bool F16, int RA, int RB, bool FULLN, bool GATED, bool EXACT>
__global__ void __launch_bounds__(TB, 4) k_outer_inv_real(const uint32_t *__restrict__ S, uint16_t *__restrict__ y, int CG,
                                                      int H, int N, int64_t M, int ko_lo, const uint16_t *__restrict__ vg,
                                                      LaunchGate gate)
{
    extern __shared__ float2 sm[];
    if (gate_closed(gate)) return;
    constexpr int No = RA * RB;
    constexpr int RAIN = FULLN ? RA : RA / 2;      // outer rows that are kept
    float2 *wno = sm;
    float2 *T = sm + No;                           // [No][CG]
    const int tid = threadIdx.x;
    const int r0 = blockIdx.x * 2 * CG;
    const int lgCG = 31 - __builtin_clz(CG);       // CG is a power of two
    const int h = blockIdx.y;
    const bool wide = EXACT || N % 2 == 0;
    for (int j = tid; j < No; j += TB) wno[j] = wm(j, 2.0f / (float)No);
    __syncthreads();
    const float ihm = 2.0f / (float)M;
    const int Mmask = (int)M - 1;                  // M is a power of two, at most 2^22, and so is every r * ko
    constexpr float unboost = 1.0f / (float)multipass_kf_boost(F16, No);     // exact: a power of two
    // step 1: untwiddle both columns, complete the rows ko > No/2 from their mirror rows, combine the columns
    // into one complex sequence, length-RB inverse over kb, times conj(W_No^{ka b2})
    for (int e = tid; e < RA * CG; e += TB) {
        const int cg = e & (CG - 1), ka = e >> lgCG;
        const int r = r0 + 2 * cg;
        uint2 in[RB];
#pragma unroll
        for (int kb = 0; kb < RB; ++kb) {
            const int ko = ka + RA * kb;
            // ko > No/2, written so that only kb == RB/2 depends on the thread
            const bool mir = RB == 1 ? ka > RA / 2 : (kb > RB / 2 || (kb == RB / 2 && ka > 0));
            const int kr = mir ? No - ko : ko;                // the row that holds it, <= No/2
            // rows from ko_lo on: zeroed bins of a sparse filter, never written; they count as zero (the load stays
            // unconditional, of row 0 instead, see k_outer_inv)
            in[kb] = *(const uint2 *)&S[((size_t)h * No + (kr < ko_lo ? kr : 0)) * MI + multipass_row_slot(r, multipass_quarter_rows(No))];
        }
        // (an empty statement that reads the loaded words: without it the compiler moves each load back under its
        //  condition)
#pragma unroll
        for (int kb = 0; kb < RB; ++kb) asm volatile("" ::"v"(in[kb].x), "v"(in[kb].y));
#pragma unroll
        for (int kb = 0; kb < RB; ++kb) {
            const int ko = ka + RA * kb;
            const bool mir = RB == 1 ? ka > RA / 2 : (kb > RB / 2 || (kb == RB / 2 && ka > 0));
            const int kr = mir ? No - ko : ko;
            if (kr >= ko_lo) in[kb] = make_uint2(0, 0);
            if (mir) {                                        // conjugate: the imaginary part is the upper half
                in[kb].x ^= 0x80000000u;
                in[kb].y ^= 0x80000000u;
            }
        }
        float2 w0 = wm((r * ka) & Mmask, ihm), w1 = wm(((r + 1) * ka) & Mmask, ihm);
        const float2 s0 = wm((r * RA) & Mmask, ihm), s1 = wm(((r + 1) * RA) & Mmask, ihm);
        w0.x *= unboost, w0.y *= unboost, w1.x *= unboost, w1.y *= unboost;
        float2 x[RB];
#pragma unroll
        for (int kb = 0; kb < RB; ++kb) {
            // from the first mirrored row on the twiddle carries the extra factor conj(W_Mi^{r}) (see k_outer_inv)
            const bool first_mirrored = RB == 1 ? ka > RA / 2 : ((kb == RB / 2 && ka > 0) || (kb == RB / 2 + 1 && ka == 0));
            if (first_mirrored) {
                w0 = cmulcf(w0, wm((r * No) & Mmask, ihm));
                w1 = cmulcf(w1, wm(((r + 1) * No) & Mmask, ihm));
            }
            const float2 ua = cmulcf(unpack2<F16>(in[kb].x), w0), ub = cmulcf(unpack2<F16>(in[kb].y), w1);
            x[kb] = make_float2(ua.x - ub.y, ua.y + ub.x);               // U_c + i U_{c+1}
            w0 = cmulf(w0, s0);
            w1 = cmulf(w1, s1);
        }
        dft_reg<RB, true>(x);
#pragma unroll
        for (int b2 = 0; b2 < RB; ++b2) T[(ka * RB + b2) * CG + cg] = cmulcf(x[b2], wno[ka * b2]);
    }
    __syncthreads();
    // step 2: length-RA inverse over ka; real part -> column c, imaginary part -> column c+1
    uint16_t *row0 = y + (size_t)h * N;
    const uint16_t *g0 = GATED ? vg + (size_t)h * N : nullptr;
    for (int e = tid; e < RB * CG; e += TB) {
        const int cg = e & (CG - 1), b2 = e >> lgCG;
        float2 x[RA];
#pragma unroll
        for (int ka = 0; ka < RA; ++ka) x[ka] = T[(ka * RB + b2) * CG + cg];
        dft_reg<RA, true>(x);
#pragma unroll
        for (int a = 0; a < RAIN; ++a) {
            const int64_t n = (int64_t)(a * RB + b2) * MI + r0 + 2 * cg;
            uint32_t o = (uint32_t)cv16<F16>(x[a].x) | ((uint32_t)cv16<F16>(x[a].y) << 16);
            if (wide) {
                if (EXACT || n < N) {
                    if constexpr (GATED) o = mul_pair16<F16>(o, *(const uint32_t *)(g0 + n));
                    *(uint32_t *)(row0 + n) = o;
                }
            } else {
#pragma unroll
                for (int v = 0; v < 2; ++v)
                    if (EXACT || n + v < N) {
                        uint32_t a0 = (o >> (16 * v)) & 0xffffu;
                        if constexpr (GATED) a0 = mul_pair16<F16>(a0, g0[n + v]) & 0xffffu;
                        row0[n + v] = (uint16_t)a0;
                    }
            }
        }
    }
}

// ---- the outer pass of the FILTER transform of a multi-pass plan (fftconv_filter_fft: taps -> k_f): pass A of a
// lone real row (k_outer_fwd_real above) with fp32 taps in and fp32 rows out.  k_f holds 16-bit constants, so
// its transform runs in fp32 throughout: this kernel, then the 8192-point transform of every row in LDS
// (k_long_fwd_blocks_kf, long_fft.hip).  Rows ko <= No/2 only, T2[h][ko][r] (No/2 + 1 rows of 8192 fp32 pairs per
// channel): the taps are real, the other rows are mirror images that the second kernel writes from these.
// Taps at and beyond Nk are zeros (their loads read tap 0 and are discarded: no load sits behind a branch).
// The filter gradient of these plans (long_fft.hip) transforms its rows of u and dy the same way: IN = 0: fp32
// rows, 1: fp16, 2: bf16; row h starts at element h * Nk.
template <int IN, int RA, int RB, bool FULLN>
__global__ void __launch_bounds__(TB, 4) k_filter_outer_real(const void *__restrict__ src, float2 *__restrict__ T2, int CG,
                                                         int64_t Nk, int64_t M, bool wide)
{
    extern __shared__ float2 sm[];
    constexpr int No = RA * RB, NR = No / 2 + 1;
    constexpr int RAIN = FULLN ? RA : RA / 2;      // outer rows that can hold taps
    float2 *wno = sm;                              // W_No^j, j < No
    float2 *T = sm + No;                           // [No][CG]
    const int tid = threadIdx.x;
    const int r0 = blockIdx.x * 2 * CG;
    const int lgCG = 31 - __builtin_clz(CG);       // CG is a power of two
    const int64_t h = blockIdx.y;
    const float *row0 = (const float *)src + h * Nk;               // IN == 0
    const uint16_t *row16 = (const uint16_t *)src + h * Nk;        // IN != 0
    for (int j = tid; j < No; j += TB) wno[j] = wm(j, 2.0f / (float)No);
    __syncthreads();
    // step 1: length-RA transforms over a, times W_No^{ka b2}; (column c, column c+1) = (re, im)
    for (int e = tid; e < RB * CG; e += TB) {
        const int cg = e & (CG - 1), b2 = e >> lgCG;
        float2 x[RA];
#pragma unroll
        for (int a = 0; a < RA; ++a) x[a] = make_float2(0.f, 0.f);
#pragma unroll
        for (int a = 0; a < RAIN; ++a) {
            const int64_t n = (int64_t)(a * RB + b2) * MI + r0 + 2 * cg;
            if constexpr (IN == 0) {
                if (wide) {                        // Nk even, rows 8-byte aligned: a pair is inside or outside as a whole
                    x[a] = *(const float2 *)(row0 + (n < Nk ? n : 0));
                } else {
                    x[a].x = row0[n < Nk ? n : 0];
                    x[a].y = row0[n + 1 < Nk ? n + 1 : 0];
                }
            } else {
                uint32_t wd;
                if (wide)                          // Nk even, rows 4-byte aligned: one word holds the pair
                    wd = *(const uint32_t *)(row16 + (n < Nk ? n : 0));
                else
                    wd = (uint32_t)row16[n < Nk ? n : 0] | ((uint32_t)row16[n + 1 < Nk ? n + 1 : 0] << 16);
                x[a] = unpack2<IN == 1>(wd);
            }
        }
#pragma unroll
        for (int a = 0; a < RAIN; ++a) asm volatile("" ::"v"(x[a].x), "v"(x[a].y));      // keeps the loads unconditional
#pragma unroll
        for (int a = 0; a < RAIN; ++a) {
            const int64_t n = (int64_t)(a * RB + b2) * MI + r0 + 2 * cg;
            if (n >= Nk) x[a].x = 0.f;
            if (n + 1 >= Nk) x[a].y = 0.f;
        }
        dft_reg<RA, false>(x);
#pragma unroll
        for (int ka = 0; ka < RA; ++ka) T[(ka * RB + b2) * CG + cg] = cmulf(x[ka], wno[ka * b2]);
    }
    __syncthreads();
    // step 2: length-RB transforms over b2, in place: slot ka*RB + kb then holds Z[ko], ko = ka + RA kb
    for (int e = tid; e < RA * CG; e += TB) {
        const int cg = e & (CG - 1), ka = e >> lgCG;
        float2 x[RB];
#pragma unroll
        for (int b2 = 0; b2 < RB; ++b2) x[b2] = T[(ka * RB + b2) * CG + cg];
        dft_reg<RB, false>(x);
#pragma unroll
        for (int kb = 0; kb < RB; ++kb) T[(ka * RB + kb) * CG + cg] = x[kb];
    }
    __syncthreads();
    // step 3: split the two columns, twiddle (by recurrence over kb), store the rows ko <= No/2
    const float ihm = 2.0f / (float)M;
    const int Mmask = (int)M - 1;                  // M is a power of two, at most 2^22, and so is every r * ko
    for (int e = tid; e < RA * CG; e += TB) {
        const int cg = e & (CG - 1), ka = e >> lgCG;
        const int r = r0 + 2 * cg;
        float2 w0 = wm((r * ka) & Mmask, ihm), w1 = wm(((r + 1) * ka) & Mmask, ihm);
        const float2 s0 = wm((r * RA) & Mmask, ihm), s1 = wm(((r + 1) * RA) & Mmask, ihm);
#pragma unroll
        for (int kb = 0; kb < RB && kb <= RB / 2; ++kb) {          // ko = ka + RA kb <= No/2 needs kb <= RB/2
            const int ko = ka + RA * kb;
            if (ko <= No / 2) {
                const int km = (No - ko) % No;
                const float2 z = T[(ka * RB + kb) * CG + cg], zm = T[((km % RA) * RB + km / RA) * CG + cg];
                const float2 xa = make_float2(0.5f * (z.x + zm.x), 0.5f * (z.y - zm.y));      // (Z + conj Zm) / 2
                const float2 xb = make_float2(0.5f * (z.y + zm.y), -0.5f * (z.x - zm.x));     // (Z - conj Zm) / (2i)
                const float2 ta = cmulf(xa, w0), tb = cmulf(xb, w1);
                *(float4 *)&T2[((size_t)h * NR + ko) * MI + r] = make_float4(ta.x, ta.y, tb.x, tb.y);
            }
            w0 = cmulf(w0, s0);
            w1 = cmulf(w1, s1);
        }
    }
}

// ---- the last pass of the filter gradient of a multi-pass plan: pass C of a lone real row (k_outer_inv_real)
// with fp32 rows in and fp32 samples out.  T2[h][ko][r], ko <= No/2, holds the rows of sum_b conj(FFT u_b) FFT dy_b
// after their inverse 8192-point transforms (unnormalised); the spectrum is that of a real sequence, so the rows
// ko > No/2 are the mirror images described at k_outer_inv.  dk[h][n] = scale * (the inverse outer transform),
// n < Nk.
template <int RA, int RB, bool FULLN>
__global__ void __launch_bounds__(TB, 4) k_dk_outer_inv_real(const float2 *__restrict__ T2, float *__restrict__ dk, int CG,
                                                         int64_t Nk, int64_t M, float scale)
{
    extern __shared__ float2 sm[];
    constexpr int No = RA * RB, NR = No / 2 + 1;
    constexpr int RAIN = FULLN ? RA : RA / 2;      // outer rows that are kept
    constexpr int KBC = RB < 8 ? RB : 8;           // rows loaded at a time (16 bytes each per thread)
    float2 *wno = sm;
    float2 *T = sm + No;                           // [No][CG]
    const int tid = threadIdx.x;
    const int r0 = blockIdx.x * 2 * CG;
    const int lgCG = 31 - __builtin_clz(CG);       // CG is a power of two
    const int64_t h = blockIdx.y;
    for (int j = tid; j < No; j += TB) wno[j] = wm(j, 2.0f / (float)No);
    __syncthreads();
    const float ihm = 2.0f / (float)M;
    const int Mmask = (int)M - 1;                  // M is a power of two, at most 2^22, and so is every r * ko
    // step 1: untwiddle both columns, complete the rows ko > No/2 from their mirror rows, combine the columns
    // into one complex sequence, length-RB inverse over kb, times conj(W_No^{ka b2})
    for (int e = tid; e < RA * CG; e += TB) {
        const int cg = e & (CG - 1), ka = e >> lgCG;
        const int r = r0 + 2 * cg;
        float2 w0 = wm((r * ka) & Mmask, ihm), w1 = wm(((r + 1) * ka) & Mmask, ihm);
        const float2 s0 = wm((r * RA) & Mmask, ihm), s1 = wm(((r + 1) * RA) & Mmask, ihm);
        w0.x *= scale, w0.y *= scale, w1.x *= scale, w1.y *= scale;
        float2 x[RB];
#pragma unroll
        for (int kb0 = 0; kb0 < RB; kb0 += KBC) {
            float4 in[KBC];
#pragma unroll
            for (int kk = 0; kk < KBC; ++kk) {
                const int kb = kb0 + kk, ko = ka + RA * kb;
                // ko > No/2, written so that only kb == RB/2 depends on the thread
                const bool mir = RB == 1 ? ka > RA / 2 : (kb > RB / 2 || (kb == RB / 2 && ka > 0));
                const int kr = mir ? No - ko : ko;            // the row that holds it, <= No/2
                in[kk] = *(const float4 *)&T2[((size_t)h * NR + kr) * MI + r];
            }
#pragma unroll
            for (int kk = 0; kk < KBC; ++kk) {
                const int kb = kb0 + kk;
                const bool mir = RB == 1 ? ka > RA / 2 : (kb > RB / 2 || (kb == RB / 2 && ka > 0));
                // from the first mirrored row on the twiddle carries the extra factor conj(W_Mi^{r}) (see k_outer_inv)
                const bool first_mirrored = RB == 1 ? ka > RA / 2 : ((kb == RB / 2 && ka > 0) || (kb == RB / 2 + 1 && ka == 0));
                if (first_mirrored) {
                    w0 = cmulcf(w0, wm((r * No) & Mmask, ihm));
                    w1 = cmulcf(w1, wm(((r + 1) * No) & Mmask, ihm));
                }
                const float2 sa = make_float2(in[kk].x, mir ? -in[kk].y : in[kk].y);
                const float2 sb = make_float2(in[kk].z, mir ? -in[kk].w : in[kk].w);
                const float2 ua = cmulcf(sa, w0), ub = cmulcf(sb, w1);
                x[kb] = make_float2(ua.x - ub.y, ua.y + ub.x);               // U_c + i U_{c+1}
                w0 = cmulf(w0, s0);
                w1 = cmulf(w1, s1);
            }
        }
        dft_reg<RB, true>(x);
#pragma unroll
        for (int b2 = 0; b2 < RB; ++b2) T[(ka * RB + b2) * CG + cg] = cmulcf(x[b2], wno[ka * b2]);
    }
    __syncthreads();
    // step 2: length-RA inverse over ka; real part -> column c, imaginary part -> column c+1
    float *row0 = dk + h * Nk;
    const bool wide = Nk % 2 == 0 && ((uintptr_t)dk & 7) == 0;
    for (int e = tid; e < RB * CG; e += TB) {
        const int cg = e & (CG - 1), b2 = e >> lgCG;
        float2 x[RA];
#pragma unroll
        for (int ka = 0; ka < RA; ++ka) x[ka] = T[(ka * RB + b2) * CG + cg];
        dft_reg<RA, true>(x);
#pragma unroll
        for (int a = 0; a < RAIN; ++a) {
            const int64_t n = (int64_t)(a * RB + b2) * MI + r0 + 2 * cg;
            if (wide) {
                if (n < Nk) *(float2 *)(row0 + n) = x[a];
            } else {
                if (n < Nk) row0[n] = x[a].x;
                if (n + 1 < Nk) row0[n + 1] = x[a].y;
            }
        }
    }
}

template <int RA, int RB>
int launch_dk_outer_inv(const OuterGeo &g, const float2 *T2, float *dk, int64_t Nk, int64_t M, int64_t nh, float scale,
                        hipStream_t s)
{
    const size_t lds = sizeof(float2) * ((size_t)g.No + (size_t)g.No * g.CT);
    const dim3 grid((unsigned)(MI / (2 * g.CT)), (unsigned)nh);
    if (Nk > M / 2) {
        FC_TRY(raise_dynamic_lds((const void *)k_dk_outer_inv_real<RA, RB, true>, 160 * 1024));
        hipLaunchKernelGGL((k_dk_outer_inv_real<RA, RB, true>), grid, dim3(TB), lds, s, T2, dk, g.CT, Nk, M, scale);
    } else {
        FC_TRY(raise_dynamic_lds((const void *)k_dk_outer_inv_real<RA, RB, false>, 160 * 1024));
        hipLaunchKernelGGL((k_dk_outer_inv_real<RA, RB, false>), grid, dim3(TB), lds, s, T2, dk, g.CT, Nk, M, scale);
    }
    FC_HIP(hipGetLastError());
    return FFTCONV_OK;
}

template <int IN, int RA, int RB>
int launch_filter_outer_in(const OuterGeo &g, const void *k, float2 *T2, int64_t Nk, int64_t M, int64_t nh, hipStream_t s)
{
    const size_t lds = sizeof(float2) * ((size_t)g.No + (size_t)g.No * g.CT);
    const dim3 grid((unsigned)(MI / (2 * g.CT)), (unsigned)nh);
    const bool wide = Nk % 2 == 0 && ((uintptr_t)k & (IN == 0 ? 7 : 3)) == 0;
    if (Nk > M / 2) {
        FC_TRY(raise_dynamic_lds((const void *)k_filter_outer_real<IN, RA, RB, true>, 160 * 1024));
        hipLaunchKernelGGL((k_filter_outer_real<IN, RA, RB, true>), grid, dim3(TB), lds, s, k, T2, g.CT, Nk, M, wide);
    } else {
        FC_TRY(raise_dynamic_lds((const void *)k_filter_outer_real<IN, RA, RB, false>, 160 * 1024));
        hipLaunchKernelGGL((k_filter_outer_real<IN, RA, RB, false>), grid, dim3(TB), lds, s, k, T2, g.CT, Nk, M, wide);
    }
    FC_HIP(hipGetLastError());
    return FFTCONV_OK;
}
// dtype: FFTCONV_F32 / F16 / BF16 of the rows
template <int RA, int RB>
int launch_filter_outer(const OuterGeo &g, const void *k, int dtype, float2 *T2, int64_t Nk, int64_t M, int64_t nh, hipStream_t s)
{
    if (dtype == FFTCONV_F32) return launch_filter_outer_in<0, RA, RB>(g, k, T2, Nk, M, nh, s);
    if (dtype == FFTCONV_F16) return launch_filter_outer_in<1, RA, RB>(g, k, T2, Nk, M, nh, s);
    return launch_filter_outer_in<2, RA, RB>(g, k, T2, Nk, M, nh, s);
}

// k_f for the multi-pass path: [h][ko][inner order of f'] 16-bit (re, im) pairs, f = ko + No*f', scaled 1/M
// (fp16: boost/M, see multipass_kf_boost; pass C takes the boost out again).
template <bool F16>
__global__ void k_pack_multipass(const double2 *spec, uint32_t *kf, FacList fl, int64_t M, int No, int64_t h0,
                                 int64_t nh, const uint8_t *keep, int64_t n_blocks)
{
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= nh * M) return;
    const int64_t h = idx / M, f = idx % M;
    const int ko = (int)(f % No);
    const int64_t fi = f / No;
    const double2 v = spec[h * M + freq_to_pos(f, fl, M)];
    const double sc = mask_weight(keep, n_blocks, f, M) * (double)multipass_kf_boost(F16, No) / (double)M;
    kf[((h0 + h) * No + ko) * (int64_t)MI + fused3_kf_slot_8192(fi)] =
        (uint32_t)cv16<F16>((float)(v.x * sc)) | ((uint32_t)cv16<F16>((float)(v.y * sc)) << 16);
}

OuterGeo outer_geo(int64_t M)
{
    OuterGeo g;
    g.No = (int)(M / MI);
    g.Ra = g.No < 16 ? g.No : 16;
    g.Rb = g.No / g.Ra;
    // fp32 tile T[No][CT] of 64 KiB (two blocks per compute unit), at least 32 columns
    g.CT = MI / g.No < 32 ? 32 : MI / g.No;
    return g;
}

template <bool F16, int RA, int RB, bool FULLN, bool GATED, bool EXACT>
int launch_outer_t(bool inverse, const OuterGeo &g, dim3 grid, const void *src, void *dst, int B, int H, int N, int64_t M,
                   hipStream_t s, int ko_lo, int ko_hi, int mirror_from, const void *gate)
{
    // two columns per thread while the registers allow and while that still leaves an entry for every thread
    // (at No = 256 a block has 32 columns: 16 x 32 / 2 entries would keep half of its 512 threads idle)
    constexpr int CTC = MI / (RA * RB) < 32 ? 32 : MI / (RA * RB);
    constexpr int CV = (RB <= 16 && RA * CTC / 2 >= TB) ? 2 : 1;
    const size_t lds = sizeof(float2) * ((size_t)g.No + (size_t)g.No * g.CT);
    FC_TRY(raise_dynamic_lds((const void *)k_outer_fwd<F16, RA, RB, CV, FULLN, GATED, EXACT>, 160 * 1024));
    FC_TRY(raise_dynamic_lds((const void *)k_outer_inv<F16, RA, RB, CV, FULLN, GATED, false, EXACT>, 160 * 1024));
    FC_TRY(raise_dynamic_lds((const void *)k_outer_inv<F16, RA, RB, CV, FULLN, GATED, true, EXACT>, 160 * 1024));
    if (!inverse)
        hipLaunchKernelGGL((k_outer_fwd<F16, RA, RB, CV, FULLN, GATED, EXACT>), grid, dim3(TB), lds, s, (const uint16_t *)src,
                           (uint32_t *)dst, g.CT, B, H, N, M, ko_lo, ko_hi, (const uint16_t *)gate, launch_gate());
    else if (mirror_from < g.No)
        hipLaunchKernelGGL((k_outer_inv<F16, RA, RB, CV, FULLN, GATED, true, EXACT>), grid, dim3(TB), lds, s, (const uint32_t *)src,
                           (uint16_t *)dst, g.CT, B, H, N, M, ko_lo, ko_hi, mirror_from, (const uint16_t *)gate, launch_gate());
    else
        hipLaunchKernelGGL((k_outer_inv<F16, RA, RB, CV, FULLN, GATED, false, EXACT>), grid, dim3(TB), lds, s, (const uint32_t *)src,
                           (uint16_t *)dst, g.CT, B, H, N, M, ko_lo, ko_hi, mirror_from, (const uint16_t *)gate, launch_gate());
    FC_HIP(hipGetLastError());
    return FFTCONV_OK;
}

// the half-input instantiation needs an outer transform (No >= 2) and N <= M/2; EXACT: N is even and fills its
// half (or, FULLN, the whole transform), so that no load or store needs a range check (ungated calls only)
template <bool F16, int RA, int RB>
int launch_outer(bool inverse, const OuterGeo &g, dim3 grid, const void *src, void *dst, int B, int H, int N, int64_t M,
                 hipStream_t s, int ko_lo, int ko_hi, int mirror_from, const void *gate)
{
#define FFTCONV_OUTER(FULLN, GATED, EXACT) \
    launch_outer_t<F16, RA, RB, FULLN, GATED, EXACT>(inverse, g, grid, src, dst, B, H, N, M, s, ko_lo, ko_hi, mirror_from, gate)
    if constexpr (RA >= 2) {
        if ((int64_t)N <= M / 2) {
            if (gate) return FFTCONV_OUTER(false, true, false);
            return (int64_t)N == M / 2 && N % 2 == 0 ? FFTCONV_OUTER(false, false, true) : FFTCONV_OUTER(false, false, false);
        }
    }
    if (gate) return FFTCONV_OUTER(true, true, false);
    return (int64_t)N == M && N % 2 == 0 ? FFTCONV_OUTER(true, false, true) : FFTCONV_OUTER(true, false, false);
#undef FFTCONV_OUTER
}

template <bool F16>
int dispatch_outer(bool inverse, const OuterGeo &g, dim3 grid, const void *src, void *dst, int B, int H, int N,
                   int64_t M, hipStream_t s, int ko_lo, int ko_hi, int mirror_from, const void *gate)
{
    switch (g.No) {
    case 1: return launch_outer<F16, 1, 1>(inverse, g, grid, src, dst, B, H, N, M, s, ko_lo, ko_hi, mirror_from, gate);
    case 2: return launch_outer<F16, 2, 1>(inverse, g, grid, src, dst, B, H, N, M, s, ko_lo, ko_hi, mirror_from, gate);
    case 4: return launch_outer<F16, 4, 1>(inverse, g, grid, src, dst, B, H, N, M, s, ko_lo, ko_hi, mirror_from, gate);
    case 8: return launch_outer<F16, 8, 1>(inverse, g, grid, src, dst, B, H, N, M, s, ko_lo, ko_hi, mirror_from, gate);
    case 16: return launch_outer<F16, 16, 1>(inverse, g, grid, src, dst, B, H, N, M, s, ko_lo, ko_hi, mirror_from, gate);
    case 32: return launch_outer<F16, 16, 2>(inverse, g, grid, src, dst, B, H, N, M, s, ko_lo, ko_hi, mirror_from, gate);
    case 64: return launch_outer<F16, 16, 4>(inverse, g, grid, src, dst, B, H, N, M, s, ko_lo, ko_hi, mirror_from, gate);
    case 128: return launch_outer<F16, 16, 8>(inverse, g, grid, src, dst, B, H, N, M, s, ko_lo, ko_hi, mirror_from, gate);
    case 256: return launch_outer<F16, 16, 16>(inverse, g, grid, src, dst, B, H, N, M, s, ko_lo, ko_hi, mirror_from, gate);
    case 512: return launch_outer<F16, 16, 32>(inverse, g, grid, src, dst, B, H, N, M, s, ko_lo, ko_hi, mirror_from, gate);
    default:
        set_error("multipass: unsupported outer length %d", g.No);
        return FFTCONV_EUNSUPPORTED;
    }
}

template <bool F16, int RA, int RB>
int launch_outer_real(bool inverse, const OuterGeo &g, const void *src, void *dst, int H, int N, int64_t M, hipStream_t s,
                      int ko_lo, const void *gate)
{
    // a block takes 2 g.CT columns as g.CT pairs: the same tile T[No][g.CT] as the paired passes
    const size_t lds = sizeof(float2) * ((size_t)g.No + (size_t)g.No * g.CT);
    const dim3 grid((unsigned)(MI / (2 * g.CT)), (unsigned)H);
    const bool fulln = (int64_t)N > M / 2;
#define FFTCONV_REAL_LAUNCH(FULLN, GATED, EXACT)                                                                                  \
    do {                                                                                                                    \
        if (!inverse) {                                                                                                     \
            FC_TRY(raise_dynamic_lds((const void *)k_outer_fwd_real<F16, RA, RB, FULLN, GATED, EXACT>, 160 * 1024));               \
            hipLaunchKernelGGL((k_outer_fwd_real<F16, RA, RB, FULLN, GATED, EXACT>), grid, dim3(TB), lds, s, (const uint16_t *)src, \
                               (uint32_t *)dst, g.CT, H, N, M, ko_lo, (const uint16_t *)gate, launch_gate());               \
        } else {                                                                                                            \
            FC_TRY(raise_dynamic_lds((const void *)k_outer_inv_real<F16, RA, RB, FULLN, GATED, EXACT>, 160 * 1024));               \
            hipLaunchKernelGGL((k_outer_inv_real<F16, RA, RB, FULLN, GATED, EXACT>), grid, dim3(TB), lds, s, (const uint32_t *)src, \
                               (uint16_t *)dst, g.CT, H, N, M, ko_lo, (const uint16_t *)gate, launch_gate());               \
        }                                                                                                                   \
    } while (0)
    // exact: N is even and fills its half (or the whole transform): no range checks (ungated calls only)
    const bool exact = N % 2 == 0 && (int64_t)N == (fulln ? M : M / 2);
    if (fulln) {
        if (gate) FFTCONV_REAL_LAUNCH(true, true, false);
        else if (exact) FFTCONV_REAL_LAUNCH(true, false, true);
        else FFTCONV_REAL_LAUNCH(true, false, false);
    } else {
        if (gate) FFTCONV_REAL_LAUNCH(false, true, false);
        else if (exact) FFTCONV_REAL_LAUNCH(false, false, true);
        else FFTCONV_REAL_LAUNCH(false, false, false);
    }
#undef FFTCONV_REAL_LAUNCH
    FC_HIP(hipGetLastError());
    return FFTCONV_OK;
}

// outer lengths the packed real-row passes exist for
bool outer_real_ok(int No) { return No >= 4 && No <= 256; }

template <bool F16>
int dispatch_outer_real(bool inverse, const OuterGeo &g, const void *src, void *dst, int H, int N, int64_t M, hipStream_t s,
                        int ko_lo, const void *gate)
{
    switch (g.No) {
    case 4: return launch_outer_real<F16, 4, 1>(inverse, g, src, dst, H, N, M, s, ko_lo, gate);
    case 8: return launch_outer_real<F16, 8, 1>(inverse, g, src, dst, H, N, M, s, ko_lo, gate);
    case 16: return launch_outer_real<F16, 16, 1>(inverse, g, src, dst, H, N, M, s, ko_lo, gate);
    case 32: return launch_outer_real<F16, 16, 2>(inverse, g, src, dst, H, N, M, s, ko_lo, gate);
    case 64: return launch_outer_real<F16, 16, 4>(inverse, g, src, dst, H, N, M, s, ko_lo, gate);
    case 128: return launch_outer_real<F16, 16, 8>(inverse, g, src, dst, H, N, M, s, ko_lo, gate);
    case 256: return launch_outer_real<F16, 16, 16>(inverse, g, src, dst, H, N, M, s, ko_lo, gate);
    default:
        set_error("multipass: no real-row outer pass for outer length %d", g.No);
        return FFTCONV_EUNSUPPORTED;
    }
}

}  // namespace

bool multipass_supported(int64_t N, int64_t M, int dtype)
{
    if (dtype != FFTCONV_F16 && dtype != FFTCONV_BF16) return false;
    if (M < MI || M > 512 * (int64_t)MI) return false;
    return N >= 1 && N <= M;
}

int multipass_init(fftconv_plan *p)
{
    int rc = fused3_init_inner(p);
    if (rc) return rc;
    return fused3_init_short(p);      // short filters run as overlapping 8192-point segments (fused3.hip)
}

size_t multipass_kf_bytes(const fftconv_plan *p)
{
    return (size_t)(p->H * p->M) * sizeof(uint32_t) + fused3_short_kf_bytes(p);
}

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
    if (p->dtype == FFTCONV_F16)
        hipLaunchKernelGGL(k_pack_multipass<true>, dim3(grid), dim3(bs), 0, s, spec, (uint32_t *)kf, staged_fac_list(p),
                           p->M, (int)(p->M / MI), h0, nh, keep_dev, n_blocks);
    else
        hipLaunchKernelGGL(k_pack_multipass<false>, dim3(grid), dim3(bs), 0, s, spec, (uint32_t *)kf, staged_fac_list(p),
                           p->M, (int)(p->M / MI), h0, nh, keep_dev, n_blocks);
    FC_HIP(hipGetLastError());
    return FFTCONV_OK;
}

// Outer pass of the transform of nh real rows of Nk samples each (see k_filter_outer_real; dtype: FFTCONV_F32 / F16 /
// BF16 of the rows); T2 takes nh * (No/2 + 1) * 8192 fp32 pairs.  multipass_filter_outer_ok(): false = no such kernel
// for this outer length (the caller takes the generic column kernel instead).
bool multipass_filter_outer_ok(const fftconv_plan *p) { return outer_real_ok((int)(p->M / MI)); }

int multipass_filter_outer(const fftconv_plan *p, const void *rows, int dtype, int64_t Nk, int64_t nh, void *T2, hipStream_t s)
{
    const OuterGeo g = outer_geo(p->M);
    if (nh > 65535) {
        set_error("multipass: %lld rows per launch of the real outer pass exceed the grid limit", (long long)nh);
        return FFTCONV_EUNSUPPORTED;
    }
    float2 *t = (float2 *)T2;
    switch (g.No) {
    case 4: return launch_filter_outer<4, 1>(g, rows, dtype, t, Nk, p->M, nh, s);
    case 8: return launch_filter_outer<8, 1>(g, rows, dtype, t, Nk, p->M, nh, s);
    case 16: return launch_filter_outer<16, 1>(g, rows, dtype, t, Nk, p->M, nh, s);
    case 32: return launch_filter_outer<16, 2>(g, rows, dtype, t, Nk, p->M, nh, s);
    case 64: return launch_filter_outer<16, 4>(g, rows, dtype, t, Nk, p->M, nh, s);
    case 128: return launch_filter_outer<16, 8>(g, rows, dtype, t, Nk, p->M, nh, s);
    case 256: return launch_filter_outer<16, 16>(g, rows, dtype, t, Nk, p->M, nh, s);
    default:
        set_error("multipass: no real outer pass for outer length %d", g.No);
        return FFTCONV_EUNSUPPORTED;
    }
}

// Last pass of the filter gradient, and of the fp32 forward pass of long plans (see k_dk_outer_inv_real): T2 holds
// nh * (No/2 + 1) rows; dk (nh, Nk) = scale * the real inverse outer transform.
int multipass_dk_outer_inv(const fftconv_plan *p, const void *T2, float *dk, int64_t Nk, int64_t nh, float scale, hipStream_t s)
{
    const OuterGeo g = outer_geo(p->M);
    if (nh > 65535) {
        set_error("multipass: %lld rows per launch of the real outer pass exceed the grid limit", (long long)nh);
        return FFTCONV_EUNSUPPORTED;
    }
    const float2 *t = (const float2 *)T2;
    switch (g.No) {
    case 4: return launch_dk_outer_inv<4, 1>(g, t, dk, Nk, p->M, nh, scale, s);
    case 8: return launch_dk_outer_inv<8, 1>(g, t, dk, Nk, p->M, nh, scale, s);
    case 16: return launch_dk_outer_inv<16, 1>(g, t, dk, Nk, p->M, nh, scale, s);
    case 32: return launch_dk_outer_inv<16, 2>(g, t, dk, Nk, p->M, nh, scale, s);
    case 64: return launch_dk_outer_inv<16, 4>(g, t, dk, Nk, p->M, nh, scale, s);
    case 128: return launch_dk_outer_inv<16, 8>(g, t, dk, Nk, p->M, nh, scale, s);
    case 256: return launch_dk_outer_inv<16, 16>(g, t, dk, Nk, p->M, nh, scale, s);
    default:
        set_error("multipass: no real outer pass for outer length %d", g.No);
        return FFTCONV_EUNSUPPORTED;
    }
}

// One set of the three passes over rows [0, B) of u.  ko_lo, ko_hi: outer frequency digits ko in [ko_lo, ko_hi)
// only meet zeroed bins of k_f (frequency-sparse filters); their rows of the workspace are skipped by all three
// passes.  ko_lo >= ko_hi: none.  wg, vg: input / output gate of the gated form, fused into passes A and C.
// lone: B == 1 and the row is transformed as a REAL sequence (Appendix A.1's point -- a real input needs half
// of a complex transform -- taken at the outer factor): before the twiddle, row No - ko of the outer transform
// of a real sequence is the conjugate of row ko, its spectrum is the mirror image of row ko's, and since the
// filter is real the same holds after the inner convolutions.  So only the rows ko <= No/2 are written by pass A,
// convolved by pass B (which then reads only those rows of k_f) and read by pass C, which forms the others as
// conjugates: half of the workspace traffic, of the k_f traffic and of the inner transforms.
static int multipass_passes(const fftconv_plan *p, const void *u, const void *kf, void *y, int64_t B, uint32_t *S,
                            hipStream_t s, int ko_lo, int ko_hi, const void *wg, const void *vg, bool lone)
{
    const OuterGeo g = outer_geo(p->M);
    const int64_t npairs = (B + 1) / 2;
    const int64_t rows = npairs * p->H;
    if (rows > 65535) {
        set_error("fftconv_forward: ceil(B/2) * H = %lld exceeds the multi-pass grid limit 65535", (long long)rows);
        return FFTCONV_EUNSUPPORTED;
    }
    const bool f16 = p->dtype == FFTCONV_F16;
    const dim3 grid((unsigned)(MI / g.CT), (unsigned)rows);
    if (ko_lo >= ko_hi) ko_lo = ko_hi = g.No;            // nothing skipped
    // rows that passes A and B leave out, rows that pass C takes as zero, rows that pass C mirrors
    int ab_lo = ko_lo, ab_hi = ko_hi, c_lo = ko_lo, c_hi = ko_hi, mirror_from = g.No;
    const bool packed = lone && outer_real_ok(g.No);
    if (packed) {
        // a sparse filter keeps ko < ko_lo and ko >= ko_hi = No - (ko_lo - 1), mirror images of each other: of the rows
        // ko <= No/2 those below ko_lo are live
        ab_lo = ko_lo < g.No / 2 + 1 ? ko_lo : g.No / 2 + 1;
        ab_hi = g.No;
    } else if (lone && g.No >= 4 && ko_lo >= ko_hi) {     // outer length 512: paired kernels, pass C mirrors the rows
        mirror_from = ab_lo = g.No / 2 + 1;
        ab_hi = g.No;
    }
    // the lone row's outer passes pack two columns into one complex transform where such kernels exist
    // (outer lengths 4 .. 256); at 512 the paired kernels run with the missing partner and pass C mirrors the rows
    int rc;
    if (packed)
        rc = f16 ? dispatch_outer_real<true>(false, g, u, S, (int)p->H, (int)p->N, p->M, s, ab_lo, wg)
                 : dispatch_outer_real<false>(false, g, u, S, (int)p->H, (int)p->N, p->M, s, ab_lo, wg);
    else
        rc = f16 ? dispatch_outer<true>(false, g, grid, u, S, (int)B, (int)p->H, (int)p->N, p->M, s, ab_lo, ab_hi, g.No, wg)
                 : dispatch_outer<false>(false, g, grid, u, S, (int)B, (int)p->H, (int)p->N, p->M, s, ab_lo, ab_hi, g.No, wg);
    if (rc) return rc;
    rc = fused3_inner_rows(p, S, kf, npairs, p->H * g.No, s, g.No, ab_lo, ab_hi, multipass_quarter_rows(g.No));
    if (rc) return rc;
    if (packed)
        return f16 ? dispatch_outer_real<true>(true, g, S, y, (int)p->H, (int)p->N, p->M, s, ab_lo, vg)
                   : dispatch_outer_real<false>(true, g, S, y, (int)p->H, (int)p->N, p->M, s, ab_lo, vg);
    return f16 ? dispatch_outer<true>(true, g, grid, S, y, (int)B, (int)p->H, (int)p->N, p->M, s, c_lo, c_hi, mirror_from, vg)
               : dispatch_outer<false>(true, g, grid, S, y, (int)B, (int)p->H, (int)p->N, p->M, s, c_lo, c_hi, mirror_from, vg);
}

// Batch rows are transformed two at a time (one complex transform per pair, the filter being real); a row left
// over (odd B, B = 1) goes through a set of passes of its own as a real sequence (see above).
int multipass_forward(const fftconv_plan *p, const void *u, const void *kf, void *y, int64_t B, void *workspace,
                      hipStream_t s, int ko_lo, int ko_hi, const void *wg, const void *vg)
{
    uint32_t *S = (uint32_t *)workspace;
    // fft_size 8192 (outer length 1: a circular or ragged shape the causal kernel does not take): the inner kernel
    // reads u and writes y itself, nothing passes through the workspace.  Gated calls and N not a multiple of 4
    // (rows that start off an 8-byte boundary) keep the three passes.
    if (p->M == MI && p->N % 4 == 0 && !wg && !vg) return fused3_inner_whole(p, u, kf, y, B, s);
    const int64_t Be = B - B % 2;                        // rows in pairs
    if (Be > 0) {
        const int rc = multipass_passes(p, u, kf, y, Be, S, s, ko_lo, ko_hi, wg, vg, false);
        if (rc) return rc;
    }
    if (B % 2 == 0) return FFTCONV_OK;
    const size_t ofs = (size_t)Be * (size_t)p->H * (size_t)p->N;             // elements before the last row
    auto at = [&](const void *base) { return base ? (const void *)((const uint16_t *)base + ofs) : nullptr; };
    return multipass_passes(p, at(u), kf, (uint16_t *)y + ofs, 1, S + (size_t)(Be / 2) * p->H * p->M, s, ko_lo, ko_hi,
                            at(wg), at(vg), true);
}

}  // namespace fftconv
