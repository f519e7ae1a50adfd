// Wave-specialised fused circular convolution of complex rows of length 8192 = 32*16*16, the inner step
// of the multi-pass scheme (paper Algorithm 4: everything inside the outermost matrix operation stays
// fused).  A row holds 8192 16-bit (re, im) pairs and is convolved in place with one row of k_f; a work
// item is one row.  Same arithmetic, tables and k_f order as the causal 8192-point kernel (fused3_ws.hip),
// without its implicit zeros: stage 1 contracts all 32 values of n1 and the inverse of stage 1 yields all 32.
//
// The workgroup is split by role and software-pipelined over work items, one workgroup barrier per step:
//   waves 0-3 ("outer"): phase C of item s-1 (inverse stage 1, straight from registers to HBM), phase A
//                        of item s+1 (stage 1, twiddle, stage 2 -> XB) from registers loaded a step
//                        earlier, then the loads of item s+2;
//   waves 4-7 ("inner"): phase B of item s (stage 3, k_f, inverse 3, twiddle, inverse 2, in place in XB),
//                        reloading the k_f constants of each plane for the next item as soon as the plane
//                        has used them.
// A row needs no staging through LDS: the operand of stage 1 for the planes n3 = 4w .. 4w+3 of wave w,
// row n2 and four consecutive n1 is four 16-byte pieces of the row (position n1*256 + n2*16 + n3), and
// the result of the inverse of stage 1 has the same shape.  With the row in natural order a wave takes a
// quarter of every line; QUARTER says the row is stored as four quarter rows, one per outer wave
// (multipass_row_slot(): outer lengths up to 64), and the pieces of a wave are then contiguous.  LDS holds
// only the exchange buffer XB, double buffered by item parity:
//   XB[t&1]: written by A(t) in step t-1, rewritten in place by B(t) in step t, read by C(t) in step t+1;
//            A(t+2) reuses it in step t+1, and every outer wave reads (C) and rewrites (A) only its own planes.
#include <type_traits>

#include "fused3_common.h"

namespace fftconv {
namespace f3 {

namespace {

using G = Geo<16, 16>;
constexpr int XBW = G::XB_WORDS;
constexpr size_t WSC_LDS_BYTES = (size_t)2 * XBW * 4;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));        // a 16-byte piece as one register tuple

// Four complex products (re[r] + i im[r]) * c[r] in fp32, each rounded once into a 16-bit (re, im) pair of
// the I/O type; CT is the type of the 4-byte constant.  The 16-bit forms TT::ctw4 round the operand before the
// product as well, and their twiddles carry 8 bits in bf16 plans; over the three products of an inner row,
// inside transforms of up to 2^22 points, that takes the bf16 error past the tolerance.  So here the twiddles
// are fp16 pairs for both I/O types (11 bits, converted from the fp32 tables when the kernel starts), k_f
// comes in the I/O type as stored, and the products of a bf16 plan run in fp32 (7 vector operations per point
// instead of 4.5; the kernel waits for memory more than for the vector ALUs).  An fp16 plan keeps the packed
// fp16 form (3 operations per point), whose roundings are 8 times smaller than the tolerance allows.
template <typename TT, typename CT> __device__ __forceinline__ uint4 cmul4(f32x4 re, f32x4 im, const uint32_t (&c)[4])
{
    if constexpr (std::is_same<TT, H16>::value) return H16::ctw4<false>(re, im, c);
    uint32_t o[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        float a = re[r], b = im[r];
        cmul_ip(a, b, CT::widen(c[r]));
        o[r] = TT::pack(a, b);
    }
    return make_uint4(o[0], o[1], o[2], o[3]);
}
__device__ __forceinline__ uint32_t tw_f16(float2 w) { return F16::pack(w.x, w.y); }
// Re-defines a register-resident constant in place (no instruction).  The bf16 products widen their fp16
// twiddles to fp32 at every use; seen as loop invariant, the widened values would be computed once before the
// loop and kept: twice the registers of the table, which the role does not have (they ended up in scratch
// memory, reloaded inside the loop).
__device__ __forceinline__ void redefine(uint32_t &c) { asm volatile("" : "+v"(c)); }

// Rows: `npairs` rows per k_f row, Hlive live k_f rows; row (pair, h) starts at word (pair * Hrows + row_of(h)) * 8192.
// Row skipping (frequency-sparse filters, Appendix A.4: the trip count of the outer loop): with KoN > 0 the
// rows come in groups of KoN (the outer frequency digit ko) of which only ko < ko_lo and ko >= ko_hi can
// meet a non-zero bin; Hlive counts the live rows only.  The other rows are neither read nor written.
//
// MODE: 0 = rows in natural order, 1 = quarter rows, 2 = no rows at all: the transform is 8192 points long (outer
// length 1), an item is a pair of batch rows of u (row 2*pair as the real, row 2*pair+1 as the imaginary part; samples
// from N on are zero and are not read) and the real / imaginary parts of the result are the first N samples of the two
// rows of y.  A lane's piece is then 4 consecutive samples (8 bytes) of either row; N is a multiple of 4, Hlive = H.
template <typename TT, int MODE>
__global__ void __launch_bounds__(NT) k_fused3_wsc(uint32_t *rows, const uint32_t *__restrict__ kf, Consts cs, int npairs,
                                                  int Hlive, int KoN, int ko_lo, int ko_hi, const uint16_t *__restrict__ u,
                                                  uint16_t *__restrict__ y, int B, int N, LaunchGate gate)
{
    constexpr bool QUARTER = MODE == 1, REAL = MODE == 2;
    extern __shared__ uint32_t smem[];
    if (gate_closed(gate)) return;
    uint32_t *const XBb = smem;                                   // [2][XBW]

    const int tid = threadIdx.x, l = tid & 63, q = l >> 4, c16 = l & 15;
    // the wave index as a scalar: the role branch is uniform and each wave runs exactly one of the two
    // loops (both execute the same number of workgroup barriers)
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const long long T = (long long)Hlive * npairs;
    const int t0 = (int)(T * blockIdx.x / gridDim.x);
    const int t1 = (int)(T * (blockIdx.x + 1) / gridDim.x);
    if (t0 >= t1) return;
    const int ko_live = KoN > 0 ? ko_lo + KoN - ko_hi : 1;
    const int Hrows = KoN > 0 ? (Hlive / ko_live) * KoN : Hlive;      // rows per pair in memory
    auto row_of = [&](int h) {                                          // live row -> row among all
        if (KoN <= 0) return h;
        const int g = h / ko_live, j = h - g * ko_live;
        return g * KoN + (j < ko_lo ? j : j - ko_lo + ko_hi);
    };
    const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};

    if (w < 4) {
        // =========================== outer role: phases C and A, all row traffic ===========================
        uint4 tab1[2][2][2], tab1i[2][2][2], tab2[4];             // tab2: the operand of the real part only
        uint32_t twa[4][2][4];                                    // fp16 pairs
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int p = 0; p < 2; ++p) {
                    tab1[a][b][p] = cs.tab1[((a * 2 + b) * 2 + p) * 64 + l];       // [K step][k1 tile][part]
                    tab1i[a][b][p] = cs.tab1i[((a * 2 + b) * 2 + p) * 64 + l];     // [K step][n1 tile][part]
                }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c = 4 * w + i;
            tab2[i] = cs.tab2[(c * 2 + 0) * 64 + l];
#pragma unroll
            for (int ct = 0; ct < 2; ++ct)
#pragma unroll
                for (int r = 0; r < 4; ++r) twa[i][ct][r] = tw_f16(cs.twa[((c * 2 + ct) * 4 + r) * 64 + l]);
        }
        // this lane's piece (tile k, register r) of a row: n1 = 16k + 4q + r, n2 = c16, n3 = 4w .. 4w+3
        // (words: multipass_row_slot() of (n1 = 4q, n2 = c16, n3 = 4w), and the distance between consecutive n1)
        const int lane_ofs = QUARTER ? w * 2048 + (4 * q) * 64 + c16 * 4 : (4 * q) * 256 + c16 * 16 + 4 * w;
        constexpr int n1_stride = QUARTER ? 64 : 256;
        auto row_ptr = [&](int t) {
            const int h = t / npairs, pair = t - h * npairs;
            return rows + ((size_t)pair * Hrows + row_of(h)) * (size_t)G::M + lane_ofs;
        };
        // MODE 2: first sample of this lane's piece (tile k, register r) is real_ofs + (16k + r) * 256; bit 4k + r
        // of in_range says that it lies below N (the piece then does entirely)
        const int real_ofs = (4 * q) * 256 + c16 * 16 + 4 * w;
        uint32_t in_range = 0;
        if constexpr (REAL) {
#pragma unroll
            for (int k = 0; k < 2; ++k)
#pragma unroll
                for (int r = 0; r < 4; ++r) in_range |= (real_ofs + (16 * k + r) * 256 < N ? 1u : 0u) << (4 * k + r);
        }
        auto real_rows = [&](int t, size_t &e0, size_t &e1, bool &has1) {   // first elements of the two rows of item t
            const int h = t / npairs, pair = t - h * npairs;
            has1 = 2 * pair + 1 < B;
            e0 = ((size_t)(2 * pair) * Hlive + h) * (size_t)N;
            e1 = ((size_t)(has1 ? 2 * pair + 1 : 2 * pair) * Hlive + h) * (size_t)N;
        };
        u32x4 L[2][4];                                            // the row being loaded / consumed by phase A
        bool L_has1 = true;                                       // MODE 2: the item in L has a second row
        auto issue_loads = [&](int t) {
            if constexpr (REAL) {
                // every load unconditional (a piece beyond N reads the row's first samples and is dropped in
                // phase A): behind a condition each would be waited for before the next one is issued
                size_t e0, e1;
                real_rows(t, e0, e1, L_has1);
#pragma unroll
                for (int k = 0; k < 2; ++k)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int n = (in_range >> (4 * k + r)) & 1u ? real_ofs + (16 * k + r) * 256 : 0;
                        const uint2 a = *(const uint2 *)(u + e0 + n), b = *(const uint2 *)(u + e1 + n);
                        L[k][r] = u32x4{a.x, a.y, b.x, b.y};
                    }
            } else {
                const uint32_t *src = row_ptr(t);
#pragma unroll
                for (int k = 0; k < 2; ++k)
#pragma unroll
                    for (int r = 0; r < 4; ++r) L[k][r] = *(const u32x4 *)(src + (16 * k + r) * n1_stride);
            }
        };

        issue_loads(t0);
        vmem_settled();
        // One step s: phase C of item s-1 (doC), phase A of item s+1 (doA), the loads of item s+2 (doL: only with
        // doA).  The steps in the middle of a workgroup's range have all three and are a loop of their own with
        // the flags as constants: the compiler's wait counts are exact only in straight-line code.  With the
        // three parts behind conditions it assumes at every join that the shorter path was taken -- no stores
        // issued in phase C, the row registers not yet consumed by phase A -- and then waits for the row loads
        // with a count that also drains the stores issued after them, and for everything before the next loads.
        auto step = [&](const int s, const bool doC, const bool doA, const bool doL) __attribute__((always_inline)) {
            if constexpr (!std::is_same<TT, H16>::value) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
                        for (int r = 0; r < 4; ++r) redefine(twa[i][ct][r]);
            }
            // ---- phase C of item s-1: inverse stage 1 -> the row, in place
            if (doC) {
                const uint32_t *XB = XBb + ((s - 1) & 1) * XBW;
                auto read_c = [&](int i, uint4 (&x)[2]) {
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks) {
                        const uint32_t *src = XB + (4 * w + i) * G::PN3 + (16 * ks + 4 * q) * G::PK1 + c16;
                        x[ks] = make_uint4(src[0], src[G::PK1], src[2 * G::PK1], src[3 * G::PK1]);
                    }
                };
                uint4 xc[2][2];                                   // [plane parity][K step], read one plane ahead
                read_c(0, xc[0]);
                uint32_t ow[2][4][4];                             // [n1 tile][r][plane]
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (i + 1 < 4) read_c(i + 1, xc[(i + 1) & 1]);
#pragma unroll
                    for (int rt = 0; rt < 2; ++rt) {
                        f32x4 dre = zero4, dim = zero4;
#pragma unroll
                        for (int ks = 0; ks < 2; ++ks) {
                            dre = TT::mfma(tab1i[ks][rt][0], xc[i & 1][ks], dre);
                            dim = TT::mfma(tab1i[ks][rt][1], xc[i & 1][ks], dim);
                        }
                        // lane: n2 = c16; reg r: n1 = 16 rt + 4q + r
#pragma unroll
                        for (int r = 0; r < 4; ++r) ow[rt][r][i] = TT::pack(dre[r], dim[r]);
                    }
                }
                if constexpr (REAL) {
                    size_t e0, e1;
                    bool has1;
                    real_rows(s - 1, e0, e1, has1);
#pragma unroll
                    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            if (!((in_range >> (4 * rt + r)) & 1u)) continue;
                            const int n = real_ofs + (16 * rt + r) * 256;
                            const uint32_t(&o)[4] = ow[rt][r];
                            // low halves = real parts = row 2*pair, high halves = row 2*pair + 1
                            *(uint2 *)(y + e0 + n) = make_uint2(__builtin_amdgcn_perm(o[1], o[0], 0x05040100u),
                                                                __builtin_amdgcn_perm(o[3], o[2], 0x05040100u));
                            if (has1)
                                *(uint2 *)(y + e1 + n) = make_uint2(__builtin_amdgcn_perm(o[1], o[0], 0x07060302u),
                                                                    __builtin_amdgcn_perm(o[3], o[2], 0x07060302u));
                        }
                } else {
                    uint32_t *dst = row_ptr(s - 1);
#pragma unroll
                    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            *(uint4 *)(dst + (16 * rt + r) * n1_stride) =
                                make_uint4(ow[rt][r][0], ow[rt][r][1], ow[rt][r][2], ow[rt][r][3]);
                }
            }
            // ---- phase A of item s+1: stage 1, twiddle, stage 2 -> XB
            if (doA) {
                uint32_t *XB = XBb + ((s + 1) & 1) * XBW;
                // the row registers are consumed from here on, not earlier: without this the compiler gathers
                // the operands (register moves) at the top of the step and waits there for the loads, which
                // were issued just before the barrier
#pragma unroll
                for (int k = 0; k < 2; ++k)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        asm volatile("" : "+v"(L[k][r])::"memory");       // as a tuple: it stays where the load put it
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int c = 4 * w + i;
                    uint4 x1[2];
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks) {
                        if constexpr (REAL) {
                            // sample i of the piece from either row -> one (re, im) word; zero beyond N
                            uint32_t d[4];
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                const u32x4 v = L[ks][r];
                                const uint32_t lo = i < 2 ? v.x : v.y, hi = L_has1 ? (i < 2 ? v.z : v.w) : 0u;
                                const uint32_t word = __builtin_amdgcn_perm(hi, lo, (i & 1) ? 0x07060302u : 0x05040100u);
                                d[r] = (in_range >> (4 * ks + r)) & 1u ? word : 0u;
                            }
                            x1[ks] = make_uint4(d[0], d[1], d[2], d[3]);
                        } else {
                            x1[ks] = make_uint4(L[ks][0][i], L[ks][1][i], L[ks][2][i], L[ks][3][i]);
                        }
                    }
                    uint4 x2[2];
#pragma unroll
                    for (int ct = 0; ct < 2; ++ct) {
                        f32x4 dre = zero4, dim = zero4;
#pragma unroll
                        for (int ks = 0; ks < 2; ++ks) {
                            dre = TT::mfma(x1[ks], tab1[ks][ct][0], dre);
                            dim = TT::mfma(x1[ks], tab1[ks][ct][1], dim);
                        }
                        x2[ct] = cmul4<TT, H16>(dre, dim, twa[i][ct]);
                    }
                    // the operand of the imaginary part is made from the other one (the same numbers in another
                    // arrangement) instead of being kept: 16 registers for a few vector operations per plane
                    const uint4 tab2_im = TT::imag_operand(tab2[i]);
#pragma unroll
                    for (int ct = 0; ct < 2; ++ct) {
                        const f32x4 dre = TT::mfma(tab2[i], x2[ct], zero4);
                        const f32x4 dim = TT::mfma(tab2_im, x2[ct], zero4);
                        // lane: k1 = 16 ct + c16; reg r: k2 = 4q + r
                        uint32_t *dst = XB + c * G::PN3 + (16 * ct + c16) * G::PK1 + 4 * q;
                        *(uint4 *)dst = make_uint4(TT::pack(dre[0], dim[0]), TT::pack(dre[1], dim[1]),
                                                   TT::pack(dre[2], dim[2]), TT::pack(dre[3], dim[3]));
                    }
                }
                // ---- the row of item s+2: in flight during the barrier and phase C of the next step
                if (doL) issue_loads(s + 2);
            }
            lds_barrier();
        };
        int s = t0 - 1;
        for (; s <= t0 && s <= t1; ++s) step(s, false, s + 1 < t1, s + 2 < t1);          // nothing to finish yet
        for (; s + 2 < t1; ++s) step(s, true, true, true);
        for (; s <= t1; ++s) step(s, true, s + 1 < t1, false);                           // nothing left to load
    } else {
        // =========================== inner role: phase B ===========================
        const int wq = w - 4;
        uint4 tab3[2], tab3i[2], tab2i[8][2];
        uint32_t twb[8][4], kfr[8][4];                            // fp16 pairs; pairs of the I/O type
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            tab3[p] = cs.tab3[p * 64 + l];
            tab3i[p] = cs.tab3i[p * 64 + l];
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int c = 8 * wq + i;
#pragma unroll
            for (int p = 0; p < 2; ++p) tab2i[i][p] = cs.tab2i[(c * 2 + p) * 64 + l];
#pragma unroll
            for (int r = 0; r < 4; ++r) twb[i][r] = tw_f16(cs.twb[(c * 4 + r) * 64 + l]);
        }
        // k_f of item t, plane i of this wave (k1 = 8 wq + i): four constants per lane
        auto kf_ptr = [&](int t) {
            return kf + (size_t)row_of(t / npairs) * G::KF_PER_H + (size_t)(8 * wq) * 256 + l;
        };
        {
            const uint32_t *src = kf_ptr(t0);
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int r = 0; r < 4; ++r) kfr[i][r] = src[(i * 4 + r) * 64];
        }
        vmem_settled();
        lds_barrier();                                            // step t0 - 1: nothing to do yet
        for (int s = t0; s < t1; ++s) {
            if constexpr (!std::is_same<TT, H16>::value) {
#pragma unroll
                for (int i = 0; i < 8; ++i)
#pragma unroll
                    for (int r = 0; r < 4; ++r) redefine(twb[i][r]);
            }
            {
                uint32_t *XB = XBb + (s & 1) * XBW;
                const bool more = s + 1 < t1;
                const uint32_t *kf_next = kf_ptr(more ? s + 1 : s);
                // operand of stage 3 for plane k1: columns k2 = c16, slots = (re, im) of n3 = 4q + r;
                // read two planes ahead of the one being computed
                auto read_plane = [&](int i) {
                    const uint32_t *src = XB + (4 * q) * G::PN3 + (8 * wq + i) * G::PK1 + c16;
                    return make_uint4(src[0], src[G::PN3], src[2 * G::PN3], src[3 * G::PN3]);
                };
                uint4 xq[3];
#pragma unroll
                for (int i = 0; i < 2; ++i) xq[i] = read_plane(i);
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int c = 8 * wq + i;
                    if (i + 2 < 8) xq[(i + 2) % 3] = read_plane(i + 2);
                    const uint4 x3v = xq[i % 3];
                    // stage 3: matrix rows k3, data columns k2
                    f32x4 dre = TT::mfma(tab3[0], x3v, zero4);
                    f32x4 dim = TT::mfma(tab3[1], x3v, zero4);
                    const uint4 x3i = cmul4<TT, TT>(dre, dim, kfr[i]);
                    // this plane's constants of the next item (the same row again while the item's k_f row stays)
#pragma unroll
                    for (int r = 0; r < 4; ++r) kfr[i][r] = kf_next[(i * 4 + r) * 64];
                    // inverse stage 3: rows k2, contraction over k3
                    dre = TT::mfma(x3i, tab3i[0], zero4);
                    dim = TT::mfma(x3i, tab3i[1], zero4);
                    const uint4 x2i = cmul4<TT, H16>(dre, dim, twb[i]);
                    // inverse stage 2: matrix rows n2, data columns n3
                    dre = TT::mfma(tab2i[i][0], x2i, zero4);
                    dim = TT::mfma(tab2i[i][1], x2i, zero4);
                    // lane: n3 = c16; reg r: n2 = 4q + r -> one 16-byte write, in place
                    uint32_t *dst = XB + c16 * G::PN3 + c * G::PK1 + 4 * q;
                    *(uint4 *)dst = make_uint4(TT::pack(dre[0], dim[0]), TT::pack(dre[1], dim[1]),
                                               TT::pack(dre[2], dim[2]), TT::pack(dre[3], dim[3]));
                }
            }
            lds_barrier();
        }
        lds_barrier();                                            // step t1: the outer role finishes the last item
    }
}

}  // namespace

// rows_per_kf rows per k_f row, `live_rows` live k_f rows (see the kernel for ko_n, ko_lo, ko_hi)
int fused3_wsc_launch(const fftconv_plan *p, void *rows, const void *kf, int64_t rows_per_kf, int64_t live_rows,
                      hipStream_t s, int ko_n, int ko_lo, int ko_hi, bool quarter_rows)
{
    const int64_t T = live_rows * rows_per_kf;
    if (T >= ((int64_t)1 << 31) - 8) {
        set_error("fftconv_forward: %lld inner rows exceed the fused kernel's limit", (long long)T);
        return FFTCONV_EUNSUPPORTED;
    }
    if (T <= 0) return FFTCONV_OK;
    const bool f16 = p->dtype == FFTCONV_F16;
    auto kern = f16 ? (quarter_rows ? k_fused3_wsc<H16, 1> : k_fused3_wsc<H16, 0>)
                    : (quarter_rows ? k_fused3_wsc<B16, 1> : k_fused3_wsc<B16, 0>);
    FC_TRY(raise_dynamic_lds((const void *)kern, (int)WSC_LDS_BYTES));
    const int grid = (int)(T < p->f3.num_cu ? T : p->f3.num_cu);
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(NT), WSC_LDS_BYTES, s, (uint32_t *)rows, (const uint32_t *)kf,
                       consts_at<16, 16>(p->f3.consts), (int)rows_per_kf, (int)live_rows, ko_n, ko_lo, ko_hi,
                       (const uint16_t *)nullptr, (uint16_t *)nullptr, 0, 0, launch_gate());
    FC_HIP(hipGetLastError());
    return FFTCONV_OK;
}

// The whole convolution of an 8192-point plan in this kernel (MODE 2): u (B, H, N) -> y, N <= 8192 a multiple of 4.
int fused3_wsc_real_launch(const fftconv_plan *p, const void *u, const void *kf, void *y, int64_t B, hipStream_t s)
{
    const int64_t npairs = (B + 1) / 2, T = npairs * p->H;
    if (p->M != G::M || p->N % 4 != 0 || p->N > G::M) {
        set_error("fftconv_forward: the single-kernel 8192-point route needs fft_size 8192 and N a multiple of 4");
        return FFTCONV_EINVAL;
    }
    if (T >= ((int64_t)1 << 31) - 8) {
        set_error("fftconv_forward: %lld row pairs exceed the fused kernel's limit", (long long)T);
        return FFTCONV_EUNSUPPORTED;
    }
    if (T <= 0) return FFTCONV_OK;
    auto kern = p->dtype == FFTCONV_F16 ? k_fused3_wsc<H16, 2> : k_fused3_wsc<B16, 2>;
    FC_TRY(raise_dynamic_lds((const void *)kern, (int)WSC_LDS_BYTES));
    const int grid = (int)(T < p->f3.num_cu ? T : p->f3.num_cu);
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(NT), WSC_LDS_BYTES, s, (uint32_t *)nullptr, (const uint32_t *)kf,
                       consts_at<16, 16>(p->f3.consts), (int)npairs, (int)p->H, 0, 0, 0, (const uint16_t *)u, (uint16_t *)y,
                       (int)B, (int)p->N, launch_gate());
    FC_HIP(hipGetLastError());
    return FFTCONV_OK;
}

}  // namespace f3
}  // namespace fftconv
