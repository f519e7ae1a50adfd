// Definitions shared by the fused order-3 kernels (fused3_ws.hip, fused3_wsc.hip, fused3_big.hip): MFMA wrappers,
// tile geometry / LDS layouts of fft_size = 32 * N2 * N3, and the table pointers.
#pragma once

#include "fftconv_internal.h"

namespace fftconv {
namespace f3 {

constexpr int N1 = 32;
constexpr int NT = 512;
constexpr int NW = NT / 64;

typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;

// Wait states between the dot products of a hand-written block and the first conversion that reads
// one of them: none in the release build (the instruction order alone keeps every DOT result 3 issue
// slots away from its reader), eight extra in the checking build.
#ifdef FFTCONV_SYNC_CHECK
#define DOT_SLACK "s_nop 7\n\t"
#else
#define DOT_SLACK ""
#endif

struct BF16 {
    static __device__ __forceinline__ f32x4 mfma(uint4 a, uint4 b, f32x4 c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c,
                                                       0, 0, 0);
    }
    static __device__ __forceinline__ uint32_t pack(float lo, float hi)
    {
        f32x2 v = {lo, hi};
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
    }
    static __device__ __forceinline__ uint16_t cvt(float x) { return __builtin_bit_cast(uint16_t, (__bf16)x); }
    // Four complex products (re[r] + i im[r]) * w[r], each packed as a 16-bit (re, im) pair;
    // c[r] = { (wr, -wi), (wi, wr) } as bf16 pairs.  The operand is rounded to bf16 first, the two
    // dot products of each point accumulate in fp32: 4 vector ops per point instead of 5.
    // Written as one asm block because the compiler would pick the accumulate-only form of the dot
    // product (one extra move per product).  On this target a DOT result may be read by another
    // vector op only 3 issue slots later; the compiler cannot see into the block, so the order
    // below keeps every producer / consumer pair at least 3 instructions apart.  The packs that
    // read MFMA results stay outside the block, where the compiler places the MFMA wait states.
    static __device__ __forceinline__ uint4 ctw4(f32x4 re, f32x4 im, const uint2 (&c)[4])
    {
        const uint32_t p0 = pack(re[0], im[0]), p1 = pack(re[1], im[1]);
        const uint32_t p2 = pack(re[2], im[2]), p3 = pack(re[3], im[3]);
        uint32_t t0, t1, t2, t3, t4, t5, t6, t7;
        asm("v_dot2_f32_bf16 %0, %8, %12, 0\n\t"
            "v_dot2_f32_bf16 %1, %8, %13, 0\n\t"
            "v_dot2_f32_bf16 %2, %9, %14, 0\n\t"
            "v_dot2_f32_bf16 %3, %9, %15, 0\n\t"
            "v_dot2_f32_bf16 %4, %10, %16, 0\n\t"
            "v_dot2_f32_bf16 %5, %10, %17, 0\n\t"
            "v_dot2_f32_bf16 %6, %11, %18, 0\n\t"
            "v_dot2_f32_bf16 %7, %11, %19, 0\n\t"
            DOT_SLACK "v_cvt_pk_bf16_f32 %0, %0, %1\n\t"
            "v_cvt_pk_bf16_f32 %2, %2, %3\n\t"
            "v_cvt_pk_bf16_f32 %4, %4, %5\n\t"
            "v_cvt_pk_bf16_f32 %6, %6, %7"
            : "=&v"(t0), "=&v"(t1), "=&v"(t2), "=&v"(t3), "=&v"(t4), "=&v"(t5), "=&v"(t6), "=&v"(t7)
            : "v"(p0), "v"(p1), "v"(p2), "v"(p3), "v"(c[0].x), "v"(c[0].y), "v"(c[1].x), "v"(c[1].y),
              "v"(c[2].x), "v"(c[2].y), "v"(c[3].x), "v"(c[3].y));
        return make_uint4(t0, t2, t4, t6);
    }
    // Elementwise product of 8 bf16 values (a 16-byte chunk) with 8 others, rounded to bf16 (the gates of
    // the gated form).  Each element is widened to fp32 (a shift or a mask: bf16 is the upper half of fp32),
    // multiplied in fp32 -- exact for bf16 inputs -- and two products are rounded into one word: one rounding
    // per element, and a NaN or an infinity stays in its own element (a dot product against a half-zeroed
    // operand, four instructions cheaper per chunk, would turn 0 * inf of the neighbour into a NaN).
    static __device__ __forceinline__ uint4 mul8(uint4 a, uint4 b)
    {
        auto m = [](uint32_t x, uint32_t y) {
            const float lo = __uint_as_float(x << 16) * __uint_as_float(y << 16);
            const float hi = __uint_as_float(x & 0xffff0000u) * __uint_as_float(y & 0xffff0000u);
            return pack(lo, hi);
        };
        return make_uint4(m(a.x, b.x), m(a.y, b.y), m(a.z, b.z), m(a.w, b.w));
    }
    static constexpr int CFMT = 1;
};
struct F16 {
    static __device__ __forceinline__ f32x4 mfma(uint4 a, uint4 b, f32x4 c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0,
                                                      0, 0);
    }
    static __device__ __forceinline__ uint32_t pack(float lo, float hi)
    {
        f32x2 v = {lo, hi};
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
    }
    static __device__ __forceinline__ uint16_t cvt(float x) { return __builtin_bit_cast(uint16_t, (_Float16)x); }
    // Four complex products in packed fp16 arithmetic (3 vector ops per point);
    // c[r] = { (wr, wr), (-wi, wi) } as fp16 pairs.
    static __device__ __forceinline__ uint4 ctw4(f32x4 re, f32x4 im, const uint2 (&c)[4])
    {
        uint32_t o[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            f32x2 v = {re[r], im[r]};
            const f16x2 p = __builtin_convertvector(v, f16x2);
            const f16x2 t = p * __builtin_bit_cast(f16x2, c[r].x);
            const f16x2 sw = {p[1], p[0]};
            o[r] = __builtin_bit_cast(uint32_t, __builtin_elementwise_fma(sw, __builtin_bit_cast(f16x2, c[r].y), t));
        }
        return make_uint4(o[0], o[1], o[2], o[3]);
    }
    // Elementwise product of 8 fp16 values with 8 others in packed arithmetic (one rounding each).
    static __device__ __forceinline__ uint4 mul8(uint4 a, uint4 b)
    {
        auto m = [](uint32_t x, uint32_t y) {
            return __builtin_bit_cast(uint32_t, __builtin_bit_cast(f16x2, x) * __builtin_bit_cast(f16x2, y));
        };
        return make_uint4(m(a.x, b.x), m(a.y, b.y), m(a.z, b.z), m(a.w, b.w));
    }
    static constexpr int CFMT = 2;
};

// ---- complex products with 4-byte constants: the traits of the kernels that stream their tables
//      or reload them by the plane (fused3_big.hip, fused3_wsc.hip)

// bf16: dot-product form.  Constant of a factor: the pair (wr, wi), 4 bytes (every constant is
// streamed from L2 once per use by the kernels for the larger sizes, whose bound is the load
// path of a compute unit, and the others keep them in registers, where 4 bytes halve the cost:
// an 8-byte form ready for both dot products costs more than the one rotate that derives the
// swapped pair here).  With z = (zr, zi) rounded to bf16:
//   re = dot(z, (wr, wi)) with the high product negated      = zr wr - zi wi
//   im = dot(z, (wi, wr))                                    = zr wi + zi wr     CONJ negates both products.
// Results accumulate in fp32 and are rounded once into the packed pair.  One asm block: the
// compiler would pick the accumulate-only form of the dot product (an extra move each), and a
// DOT result may be read by another vector op only 3 issue slots later on this target, which the
// order below respects.
struct B16 {
    using CW = uint32_t;
    static __device__ __forceinline__ f32x4 mfma(uint4 a, uint4 b, f32x4 c) { return BF16::mfma(a, b, c); }
    static __device__ __forceinline__ uint32_t pack(float lo, float hi) { return BF16::pack(lo, hi); }
    // The matrix operand that yields the imaginary part of a complex product, from the one that yields the real
    // part: every 32-bit word (g.re, -g.im) becomes (g.im, g.re): halves swapped, sign of the new lower half flipped.
    static __device__ __forceinline__ uint4 imag_operand(uint4 a)
    {
        auto f = [](uint32_t x) { return __builtin_amdgcn_perm(x, x, 0x01000302u) ^ 0x00008000u; };
        return make_uint4(f(a.x), f(a.y), f(a.z), f(a.w));
    }
    template <bool CONJ> static __device__ __forceinline__ uint4 ctw4(f32x4 re, f32x4 im, const CW (&c)[4])
    {
        const uint32_t p0 = pack(re[0], im[0]), p1 = pack(re[1], im[1]);
        const uint32_t p2 = pack(re[2], im[2]), p3 = pack(re[3], im[3]);
        uint32_t t0, t1, t2, t3, t4, t5, t6, t7;
#define B16_CTW4(IMNEG)                                                                            \
        asm("v_alignbit_b32 %1, %12, %12, 16\n\t"                                                   \
            "v_alignbit_b32 %3, %13, %13, 16\n\t"                                                   \
            "v_alignbit_b32 %5, %14, %14, 16\n\t"                                                   \
            "v_alignbit_b32 %7, %15, %15, 16\n\t"                                                   \
            "v_dot2_f32_bf16 %0, %8, %12, 0 neg_hi:[0,1,0]\n\t"                                     \
            "v_dot2_f32_bf16 %1, %8, %1, 0" IMNEG "\n\t"                                            \
            "v_dot2_f32_bf16 %2, %9, %13, 0 neg_hi:[0,1,0]\n\t"                                     \
            "v_dot2_f32_bf16 %3, %9, %3, 0" IMNEG "\n\t"                                            \
            "v_dot2_f32_bf16 %4, %10, %14, 0 neg_hi:[0,1,0]\n\t"                                    \
            "v_dot2_f32_bf16 %5, %10, %5, 0" IMNEG "\n\t"                                           \
            "v_dot2_f32_bf16 %6, %11, %15, 0 neg_hi:[0,1,0]\n\t"                                    \
            "v_dot2_f32_bf16 %7, %11, %7, 0" IMNEG "\n\t"                                           \
            DOT_SLACK "v_cvt_pk_bf16_f32 %0, %0, %1\n\t"                                                      \
            "v_cvt_pk_bf16_f32 %2, %2, %3\n\t"                                                      \
            "v_cvt_pk_bf16_f32 %4, %4, %5\n\t"                                                      \
            "v_cvt_pk_bf16_f32 %6, %6, %7"                                                          \
            : "=&v"(t0), "=&v"(t1), "=&v"(t2), "=&v"(t3), "=&v"(t4), "=&v"(t5), "=&v"(t6), "=&v"(t7) \
            : "v"(p0), "v"(p1), "v"(p2), "v"(p3), "v"(c[0]), "v"(c[1]), "v"(c[2]), "v"(c[3]))
        if constexpr (CONJ)
            B16_CTW4(" neg_lo:[0,1,0] neg_hi:[0,1,0]");
        else
            B16_CTW4("");
#undef B16_CTW4
        return make_uint4(t0, t2, t4, t6);
    }
    static __host__ __device__ inline CW cconst(uint32_t re, uint32_t im, bool) { return re | (im << 16); }   // 16-bit patterns
    // the constant as an fp32 pair
    static __device__ __forceinline__ float2 widen(CW c)
    {
        return make_float2(__uint_as_float(c << 16), __uint_as_float(c & 0xffff0000u));
    }
    static __device__ __forceinline__ uint4 mul8(uint4 a, uint4 b) { return BF16::mul8(a, b); }
};

// fp16: packed arithmetic.  Constant of a factor: the pair (wr, wi); the operand selectors
// broadcast / swap halves and the neg modifiers supply the signs:
//   t   = (zr*wr, zi*wr)
//   out = (zi*(-wi) + t.lo, zr*wi + t.hi)            CONJ negates the high half of both steps.
struct H16 {
    using CW = uint32_t;
    static __device__ __forceinline__ f32x4 mfma(uint4 a, uint4 b, f32x4 c) { return F16::mfma(a, b, c); }
    static __device__ __forceinline__ uint32_t pack(float lo, float hi) { return F16::pack(lo, hi); }
    // The matrix operand that yields the imaginary part of a complex product, from the one that yields the real
    // part: every 32-bit word (g.re, -g.im) becomes (g.im, g.re).  One packed multiplication by (-1, 1) with the
    // halves of the source swapped: exact.
    static __device__ __forceinline__ uint4 imag_operand(uint4 a)
    {
        uint4 d;
        asm("v_pk_mul_f16 %0, %4, %8 op_sel:[1,0] op_sel_hi:[0,1]\n\t"
            "v_pk_mul_f16 %1, %5, %8 op_sel:[1,0] op_sel_hi:[0,1]\n\t"
            "v_pk_mul_f16 %2, %6, %8 op_sel:[1,0] op_sel_hi:[0,1]\n\t"
            "v_pk_mul_f16 %3, %7, %8 op_sel:[1,0] op_sel_hi:[0,1]"
            : "=&v"(d.x), "=&v"(d.y), "=&v"(d.z), "=&v"(d.w)
            : "v"(a.x), "v"(a.y), "v"(a.z), "v"(a.w), "s"(0x3C00BC00u));
        return d;
    }
    static __host__ __device__ inline CW cconst(uint32_t re, uint32_t im, bool) { return re | (im << 16); }
    // the constant as an fp32 pair
    static __device__ __forceinline__ float2 widen(CW c)
    {
        const f16x2 h = __builtin_bit_cast(f16x2, c);
        return make_float2((float)h[0], (float)h[1]);
    }
    static __device__ __forceinline__ uint4 mul8(uint4 a, uint4 b) { return F16::mul8(a, b); }
    template <bool CONJ> static __device__ __forceinline__ uint4 ctw4(f32x4 re, f32x4 im, const CW (&c)[4])
    {
        uint32_t o[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const uint32_t p = pack(re[r], im[r]);
            uint32_t t;
            if constexpr (!CONJ) {
                asm("v_pk_mul_f16 %0, %1, %2 op_sel:[0,0] op_sel_hi:[1,0]" : "=v"(t) : "v"(p), "v"(c[r]));
                asm("v_pk_fma_f16 %0, %1, %2, %3 op_sel:[1,1,0] op_sel_hi:[0,1,1] neg_lo:[0,1,0]"
                    : "=v"(o[r])
                    : "v"(p), "v"(c[r]), "v"(t));
            } else {
                asm("v_pk_mul_f16 %0, %1, %2 op_sel:[0,0] op_sel_hi:[1,0] neg_hi:[0,1]"
                    : "=v"(t)
                    : "v"(p), "v"(c[r]));
                asm("v_pk_fma_f16 %0, %1, %2, %3 op_sel:[1,1,0] op_sel_hi:[0,1,1] neg_lo:[0,1,0] neg_hi:[0,1,0]"
                    : "=v"(o[r])
                    : "v"(p), "v"(c[r]), "v"(t));
            }
        }
        return make_uint4(o[0], o[1], o[2], o[3]);
    }
};

// Workgroup barrier for exchanges through LDS only.  __syncthreads() also waits for every
// outstanding global load and store of the wave (its fence covers global memory), which would
// throw away the prefetches and stores these kernels keep in flight across barriers.  LDS
// operations of a wave complete in order, so once its LDS counter is zero its writes are visible
// to, and its reads are finished before, whatever the other waves do after the barrier.
// A build with FFTCONV_SYNC_CHECK defined (tests only) uses the full __syncthreads() instead and
// pads the hand-spaced dot-product blocks with wait states (DOT_SLACK); its results must be
// bit-identical to the release build's.
__device__ __forceinline__ void lds_barrier()
{
#ifdef FFTCONV_SYNC_CHECK
    __syncthreads();
#else
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
#endif
}

// Waits until every vector-memory operation of the wave has completed, as an instruction the compiler knows.
// Placed after the loads of a persistent kernel's prologue (register-resident tables, the first work item) and
// before its loop.  Without it the compiler's wait-count bookkeeping treats those registers as possibly still
// in flight at the head of every iteration (it merges the state before the loop with the state at the back edge)
// and re-issues the prologue's waits there, where they then wait for the loads that the previous iteration
// has just put in flight for a later work item.
// (The empty statements and scheduling barriers keep the compiler from moving loads across the wait.)
__device__ __forceinline__ void vmem_settled()
{
    asm volatile("" ::: "memory");                                // no load is moved below this point
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(0x0F70);                           // vmcnt(0)
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("" ::: "memory");
}

template <int N2, int N3> struct Geo {
    static constexpr int M = N1 * N2 * N3;
    static constexpr int R2 = N2 / 16, R3 = N3 / 16;
    // exchange buffer, 32-bit words: X(k1,k2,n3) = n3*PN3 + k1*PK1 + k2.
    // 4*PK1 and 4*PN3 are 16 mod 32, which spreads the 4 lane groups of a wave over the banks.
    static constexpr int PK1 = N2 + 4;
    static constexpr int PN3 = N1 * PK1 + 4;
    static constexpr int XB_WORDS = N3 * PN3;
    // staging of u / y, 16-bit elements: (s, n1, n2, n3) -> s*SU + n1*PQ1 + n2*PR + n3
    static constexpr int PR = N3 + 2;
    static constexpr int PQ1 = N2 * PR + 8;
    static constexpr int SU = (N1 / 2) * PQ1;
    static constexpr int UB_ELEMS = 2 * SU;
    // table sizes (entries)
    static constexpr int TAB1 = 2 * 2 * 2 * 64;             // [K step][ct][part][lane] uint4
    static constexpr int TAB2 = N3 * R2 * R2 * 2 * 64;      // [n3][t][ct][part][lane]
    static constexpr int TAB3 = R3 * R3 * 2 * 64;           // [t][ct][part][lane]
    static constexpr int TAB2I = N1 * R2 * R2 * 2 * 64;     // [k1][t][ct][part][lane]
    static constexpr int TAB1I = 2 * 2 * 2 * 64;            // [K step][row tile][part][lane]
    static constexpr int TWA = N3 * R2 * 2 * 4 * 64;        // [n3][rt][ct][r][lane] float2
    static constexpr int TWB = N1 * R2 * R3 * 4 * 64;       // [k1][ct2][ct3][r][lane] float2
    static constexpr int KF_PER_H = N1 * R2 * R3 * 4 * 64;  // == M
};

struct Consts {
    const uint4 *tab1, *tab2, *tab3, *tab3i, *tab2i, *tab1i;
    const float2 *twa, *twb;
    const uint2 *twa16, *twb16;       // the same twiddles as 16-bit constant pairs for TT::ctw
};

// 16-bit constant pair of a complex factor (wr, wi) in the form TT::ctw expects
// (fmt 1: bf16 dot-product form, fmt 2: fp16 packed-math form).  hi16(x) converts one value.
template <typename F> __host__ __device__ inline uint2 ctw_const(double wr, double wi, int fmt, F hi16)
{
    uint2 c;
    if (fmt == 1) {
        c.x = (uint32_t)hi16(wr) | ((uint32_t)hi16(-wi) << 16);
        c.y = (uint32_t)hi16(wi) | ((uint32_t)hi16(wr) << 16);
    } else {
        c.x = (uint32_t)hi16(wr) | ((uint32_t)hi16(wr) << 16);
        c.y = (uint32_t)hi16(-wi) | ((uint32_t)hi16(wi) << 16);
    }
    return c;
}

__device__ __forceinline__ void cmul_ip(float &re, float &im, float2 w)
{
    float r = re * w.x - im * w.y;
    float i = re * w.y + im * w.x;
    re = r;
    im = i;
}


template <int N2, int N3>
inline Consts consts_at(const void *base)
{
    using G = Geo<N2, N3>;
    Consts c;
    const uint4 *b = (const uint4 *)base;
    c.tab1 = b;
    c.tab2 = c.tab1 + G::TAB1;
    c.tab3 = c.tab2 + G::TAB2;
    c.tab3i = c.tab3 + G::TAB3;
    c.tab2i = c.tab3i + G::TAB3;
    c.tab1i = c.tab2i + G::TAB2I;
    c.twa = (const float2 *)(c.tab1i + G::TAB1I);
    c.twb = c.twa + G::TWA;
    c.twa16 = (const uint2 *)(c.twb + G::TWB);
    c.twb16 = c.twa16 + G::TWA;
    return c;
}


// wave-specialised kernel for fft_size 8192 (fused3_ws.hip)
template <int N2, int N3>
inline Consts consts_of(const fftconv_plan *p) { return consts_at<N2, N3>(p->f3.consts); }

// wg / vg: input / output gate of the gated form (nullptr = none; only with nseg == 1)
// live_k1: bit k1 clear = k_f is zero on that k1 plane (skipped; ungated calls only)
int fused3_ws_launch(const fftconv_plan *p, const void *consts, const void *u, const void *kf, void *y, int64_t B,
                     int nseg, int P, hipStream_t s, const void *wg = nullptr, const void *vg = nullptr,
                     uint32_t live_k1 = 0xffffffffu);

// wave-specialised kernel for complex rows of length 8192, in place (fused3_wsc.hip): the inner step of the
// multi-pass scheme
int fused3_wsc_launch(const fftconv_plan *p, void *rows, const void *kf, int64_t rows_per_kf, int64_t live_rows,
                      hipStream_t s, int ko_n, int ko_lo, int ko_hi, bool quarter_rows);
// the same kernel running a whole 8192-point convolution (u and y in place of the rows; N a multiple of 4)
int fused3_wsc_real_launch(const fftconv_plan *p, const void *u, const void *kf, void *y, int64_t B, hipStream_t s);

// fused kernel for fft_size 32768 (fused3_big.hip): own tables (in p->f3.consts) and k_f layout
int fused3_big_init(fftconv_plan *p);
size_t fused3_big_kf_bytes(const fftconv_plan *p);
int fused3_big_filter(const fftconv_plan *p, const float *k, int64_t Nk, bool adjoint, const uint8_t *keep_dev,
                      int64_t n_blocks, void *kf, hipStream_t s);
int fused3_big_forward(const fftconv_plan *p, const void *u, const void *kf, void *y, int64_t B, uint32_t live_k3,
                       hipStream_t s, uint32_t live_k2 = 0xffffffffu, uint32_t live_k1 = 0xffffffffu);
int fused3_big_forward_gated(const fftconv_plan *p, const void *u, const void *wg, const void *vg, const void *kf, void *y,
                             int64_t B, hipStream_t s);

}  // namespace f3
}  // namespace fftconv
