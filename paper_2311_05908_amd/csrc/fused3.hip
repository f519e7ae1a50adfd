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
// Work split of a 512-thread workgroup (8 waves) on one pair:
//   phase A (per n3):  stage 1, twiddle, stage 2      -> LDS[k1,k2,n3]
//   phase B (per k1):  stage 3, k_f, inverse 3, twiddle, inverse 2 -> LDS in place
//   phase C (per n3):  inverse stage 1                -> LDS staging -> HBM
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

// CPLX = false: u, y are (B, H, N) real rows; a work item is a pair of batch rows of one channel.
// CPLX = true : u, y are (B, H, M) rows of 16-bit (re, im) pairs (u may equal y); a work item is
//               one row, transformed in full (no implicit zeros), circular convolution of length M.
//               This is the inner step of the multi-pass scheme (Algorithm 4).
// LIVE: accumulator registers r < LIVE of stage 3 may meet non-zero k_f (frequency-sparse filters
//       ordered as in k3_at_index()); for r >= LIVE the product is zero and is not formed.
// Row skipping (CPLX, frequency-sparse filters, Appendix A.4: the trip count of the outer loop): with
// KoN > 0 the rows come in groups of KoN (the outer frequency digit ko) of which only ko < ko_lo and
// ko >= ko_hi can meet a non-zero bin; H then counts the live rows only and rows_of() maps a live row to its
// place among all rows.  The other rows are neither read nor written.
template <int N2, int N3, typename TT, bool REGC, bool CPLX, int LIVE = 4>
__global__ void __launch_bounds__(NT) k_fused3(const uint16_t *u, uint16_t *y,
                                              const uint32_t *__restrict__ kf, Consts cs, int B, int H, int N,
                                              int KoN, int ko_lo, int ko_hi, LaunchGate gate)
{
    using G = Geo<N2, N3>;
    if (gate_closed(gate)) return;
    constexpr int R2 = G::R2, R3 = G::R3, C3 = G::C3, C1 = G::C1;
    // streamed tables are requested one tile ahead of their use when two tiles' worth fits in registers
    constexpr bool AHEAD = !REGC && N2 == 16;
    constexpr int KS1 = CPLX ? 2 : 1;            // K steps of forward stage 1 (n1 < 16 only when zero padded)
    constexpr int RT1 = CPLX ? 2 : 1;            // output row tiles of inverse stage 1
    constexpr int NCH = CPLX ? G::CHUNKS_C : G::CHUNKS;
    extern __shared__ uint32_t smem[];
    uint32_t *XB = smem;
    uint16_t *UB = (uint16_t *)(smem + G::XB_WORDS);
    uint16_t *YB = UB + (CPLX ? 2 * G::UBC_WORDS : G::UB_ELEMS);
    uint32_t *UBC = (uint32_t *)UB, *YBC = (uint32_t *)YB;

    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, q = l >> 4, c16 = l & 15;
    // Persistent workgroup; a work item t = h * npairs + pair.
    //  REGC (k_f and tables in registers): a contiguous range of items, so k_f[h] is loaded once per
    //  channel the range touches.
    //  otherwise (k_f streamed from L2 for every item): workgroups are dealt to the 8 accelerator
    //  dies round-robin, each die has its own L2; die x = blockIdx % 8 takes the channels
    //  h = x mod 8 and its workgroups walk through them side by side, so that at any time a die
    //  works on a few channels only and their k_f stays in its L2.
    const int npairs = CPLX ? B : (B + 1) / 2;
    const long long T = (long long)H * npairs;
    const int nx = (!REGC && gridDim.x % 8 == 0) ? 8 : 1;
    const int x = blockIdx.x % nx, nb = gridDim.x / nx, jb = blockIdx.x / nx;
    int first, stride, cnt;                               // local item k is v = first + k * stride
    if constexpr (REGC) {
        const int t0 = (int)(T * blockIdx.x / gridDim.x), t1 = (int)(T * (blockIdx.x + 1) / gridDim.x);
        first = t0;
        stride = 1;
        cnt = t1 - t0;
    } else {
        const int n_local = ((H - x + nx - 1) / nx) * npairs;
        first = jb;
        stride = nb;
        cnt = jb < n_local ? (n_local - jb + nb - 1) / nb : 0;
    }
    if (cnt <= 0) return;
    auto item = [&](int k) {
        const int v = first + k * stride;
        return REGC ? v : ((v / npairs) * nx + x) * npairs + v % npairs;
    };
    const int ko_live = KoN > 0 ? ko_lo + KoN - ko_hi : 1;
    const int Hrows = KoN > 0 ? (H / ko_live) * KoN : H;        // rows per pair in memory
    auto row_of = [&](int h) {                                   // live row -> row among all
        if (KoN <= 0) return h;
        const int g = h / ko_live, j = h - g * ko_live;
        return g * KoN + (j < ko_lo ? j : j - ko_lo + ko_hi);
    };

    // ---------------- constants (per-lane operand tables) ----------------
    uint4 tab1[KS1][2][2], tab1i[2][RT1][2], tab3[R3][R3][2], tab3i[R3][R3][2];
    uint4 tab2[C3][R2][R2][2], tab2i[C1][R2][R2][2];
    float2 twa[C3][R2][2][4], twb[C1][R2][R3][4];
    // k_f: 4-byte 16-bit (re, im) constants (it is streamed for every row: as many bytes as the row itself at 8)
    using T4 = typename std::conditional<std::is_same<TT, F16>::value, H16, B16>::type;
    uint32_t kfr[C1][R2][R3][4];

#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int p = 0; p < 2; ++p) {
#pragma unroll
            for (int ks = 0; ks < KS1; ++ks) tab1[ks][a][p] = cs.tab1[((ks * 2 + a) * 2 + p) * 64 + l];
#pragma unroll
            for (int rt = 0; rt < RT1; ++rt) tab1i[a][rt][p] = cs.tab1i[((a * 2 + rt) * 2 + p) * 64 + l];
        }
#pragma unroll
    for (int t = 0; t < R3; ++t)
#pragma unroll
        for (int c = 0; c < R3; ++c)
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                tab3[t][c][p] = cs.tab3[((t * R3 + c) * 2 + p) * 64 + l];
                tab3i[t][c][p] = cs.tab3i[((t * R3 + c) * 2 + p) * 64 + l];
            }
    // When the tables are streamed (REGC false) the loads must stay inside the loop over work
    // items: an opaque zero added to the lane offset keeps the compiler from hoisting them.
    int lz = l;
    auto opaque = [&]() {
        if constexpr (!REGC) {
            int z = 0;
            asm volatile("" : "+v"(z));
            lz = l + z;
        }
    };
    auto load_A = [&](int i) {
        const int c = w * C3 + i;
#pragma unroll
        for (int t = 0; t < R2; ++t)
#pragma unroll
            for (int ct = 0; ct < R2; ++ct)
#pragma unroll
                for (int p = 0; p < 2; ++p)
                    tab2[i][t][ct][p] = cs.tab2[(((c * R2 + t) * R2 + ct) * 2 + p) * 64 + lz];
#pragma unroll
        for (int rt = 0; rt < R2; ++rt)
#pragma unroll
            for (int ct = 0; ct < 2; ++ct)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    twa[i][rt][ct][r] = cs.twa[(((c * R2 + rt) * 2 + ct) * 4 + r) * 64 + lz];
    };
    auto load_B = [&](int i) {
        const int c = w * C1 + i;
#pragma unroll
        for (int t = 0; t < R2; ++t)
#pragma unroll
            for (int ct = 0; ct < R2; ++ct)
#pragma unroll
                for (int p = 0; p < 2; ++p)
                    tab2i[i][t][ct][p] = cs.tab2i[(((c * R2 + t) * R2 + ct) * 2 + p) * 64 + lz];
#pragma unroll
        for (int a = 0; a < R2; ++a)
#pragma unroll
            for (int b = 0; b < R3; ++b)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    twb[i][a][b][r] = cs.twb[(((c * R2 + a) * R3 + b) * 4 + r) * 64 + lz];
    };
    auto load_kf = [&](int i, int h) {
        const int c = w * C1 + i;
#pragma unroll
        for (int a = 0; a < R2; ++a)
#pragma unroll
            for (int b = 0; b < R3; ++b)
#pragma unroll
                for (int r = 0; r < LIVE; ++r)
                    kfr[i][a][b][r] = kf[(size_t)h * G::KF_PER_H + (((c * R2 + a) * R3 + b) * 4 + r) * 64 + lz];
    };
    if constexpr (REGC) {
#pragma unroll
        for (int i = 0; i < C3; ++i) load_A(i);
#pragma unroll
        for (int i = 0; i < C1; ++i) load_B(i);
    }

    // ---------------- input prefetch (registers) ----------------
    uint4 pre[NCH];
    auto issue_loads = [&](int k) {
        const int t = item(k < cnt ? k : cnt - 1);
        const int h = t / npairs, pair = t - h * npairs;
        if constexpr (CPLX) {
            const uint16_t *row = u + ((size_t)pair * Hrows + row_of(h)) * (size_t)(2 * G::M);
#pragma unroll
            for (int j = 0; j < NCH; ++j) {
                uint4 v = make_uint4(0, 0, 0, 0);
                if (k < cnt) v = *(const uint4 *)(row + (size_t)(tid + NT * j) * 8);
                pre[j] = v;
            }
        } else
#pragma unroll
        for (int j = 0; j < G::CHUNKS; ++j) {
            const int s = j / G::CPS;                    // which row of the pair (wave-uniform)
            const int n = (tid + NT * (j % G::CPS)) * 8;
            const int b = 2 * pair + s;
            uint4 v = make_uint4(0, 0, 0, 0);
            const uint16_t *row = u + ((size_t)b * H + h) * N;
            if (k < cnt && b < B && n < N) v = *(const uint4 *)(row + n);
            pre[j] = v;
        }
    };
    // prefetched input -> UB (padded layout)
    auto stage_in = [&]() {
        if constexpr (CPLX) {
#pragma unroll
            for (int j = 0; j < NCH; ++j) {
                const int n = (tid + NT * j) * 4;
                const int n3 = n % N3, n2 = (n / N3) % N2, n1 = n / (N2 * N3);
                uint32_t *dst = UBC + n1 * G::PQ1C + n2 * G::PRC + n3;
                dst[0] = pre[j].x;
                dst[1] = pre[j].y;
                dst[2] = pre[j].z;
                dst[3] = pre[j].w;
            }
        } else
#pragma unroll
        for (int j = 0; j < G::CHUNKS; ++j) {
            const int s = j / G::CPS;
            const int n = (tid + NT * (j % G::CPS)) * 8;
            const int n3 = n % N3, n2 = (n / N3) % N2, n1 = n / (N2 * N3);
            uint32_t *dst = (uint32_t *)(UB + s * G::SU + n1 * G::PQ1 + n2 * G::PR + n3);
            dst[0] = pre[j].x;
            dst[1] = pre[j].y;
            dst[2] = pre[j].z;
            dst[3] = pre[j].w;
        }
    };
    // YB -> y, 16 bytes per lane, coalesced
    auto store_out = [&](int k) {
        const int t = item(k);
        const int h = t / npairs, pair = t - h * npairs;
        if constexpr (CPLX) {
            uint16_t *row = y + ((size_t)pair * Hrows + row_of(h)) * (size_t)(2 * G::M);
#pragma unroll
            for (int j = 0; j < NCH; ++j) {
                const int n = (tid + NT * j) * 4;
                const int n3 = n % N3, n2 = (n / N3) % N2, n1 = n / (N2 * N3);
                const uint32_t *src = YBC + n1 * G::PQ1C + n2 * G::PRC + n3;
                *(uint4 *)(row + (size_t)n * 2) = make_uint4(src[0], src[1], src[2], src[3]);
            }
        } else
#pragma unroll
        for (int j = 0; j < G::CHUNKS; ++j) {
            const int s = j / G::CPS;
            const int n = (tid + NT * (j % G::CPS)) * 8;
            const int b = 2 * pair + s;
            const int n3 = n % N3, n2 = (n / N3) % N2, n1 = n / (N2 * N3);
            const uint32_t *src = (const uint32_t *)(YB + s * G::SU + n1 * G::PQ1 + n2 * G::PR + n3);
            const uint4 v = make_uint4(src[0], src[1], src[2], src[3]);
            uint16_t *row = y + ((size_t)b * H + h) * N;
            if (b < B && n < N) *(uint4 *)(row + n) = v;
        }
    };

    // Pipeline over work items (3 barriers each):
    //   [A(t)] | [B(t) + store(t-1) + stage_in(t+1) + issue_loads(t+2)] | [C(t)] |
    // UB is read in A(t) and rewritten in B(t); YB is written in C(t) and read in B(t+1); XB planes
    // change owner only across barriers.
    issue_loads(0);
    stage_in();
    issue_loads(1);
    if constexpr (AHEAD) load_A(0);
    lds_barrier();

    const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};
    int h_cur = -1;
    for (int k = 0; k < cnt; ++k) {
        opaque();
        {
            const int h = row_of(item(k) / npairs);
            if (h != h_cur) {                             // new channel: fetch its k_f (used in phase B)
                h_cur = h;
                if constexpr (REGC) {
#pragma unroll
                    for (int i = 0; i < C1; ++i) load_kf(i, h);
                }
            }
        }
        // ================= phase A: per n3 = c: stage 1, twiddle, stage 2 -> XB
        // (all operand reads first, then tile by tile compute -> write, so that the LDS
        //  traffic of one tile drains while the next tile computes)
        {
            uint4 x1[C3][R2][KS1];
#pragma unroll
            for (int i = 0; i < C3; ++i) {
                const int c = w * C3 + i;
#pragma unroll
                for (int rt = 0; rt < R2; ++rt) {
                    if constexpr (CPLX) {
                        // row n2 = 16 rt + c16, slots (2r, 2r+1) = (re, im) of x[n1 = 16 ks + 4q + r]
#pragma unroll
                        for (int ks = 0; ks < KS1; ++ks) {
                            const uint32_t *p0 = UBC + (16 * ks + 4 * q) * G::PQ1C + (16 * rt + c16) * G::PRC + c;
                            x1[i][rt][ks] = make_uint4(p0[0], p0[G::PQ1C], p0[2 * G::PQ1C], p0[3 * G::PQ1C]);
                        }
                    } else {
                        // operand of stage 1: row n2 = 16 rt + c16, slots (2r+s) = u_s[n1 = 4q + r]
                        const uint16_t *p0 = UB + (4 * q) * G::PQ1 + (16 * rt + c16) * G::PR + c;
                        uint32_t d[4];
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            d[r] = (uint32_t)p0[r * G::PQ1] | ((uint32_t)p0[G::SU + r * G::PQ1] << 16);
                        x1[i][rt][0] = make_uint4(d[0], d[1], d[2], d[3]);
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < C3; ++i) {
                const int c = w * C3 + i;
                // streamed tables (L2-resident): requested one tile ahead where the registers allow
                if constexpr (AHEAD) {
                    if (i + 1 < C3) load_A(i + 1);
                } else if constexpr (!REGC) {
                    load_A(i);
                }
                uint4 x2[2][R2];                          // stage-2 operands [k1 tile][K step = n2 tile]
#pragma unroll
                for (int rt = 0; rt < R2; ++rt)
#pragma unroll
                    for (int ct = 0; ct < 2; ++ct) {
                        f32x4 dre = zero4, dim = zero4;
#pragma unroll
                        for (int ks = 0; ks < KS1; ++ks) {
                            dre = TT::mfma(x1[i][rt][ks], tab1[ks][ct][0], dre);
                            dim = TT::mfma(x1[i][rt][ks], tab1[ks][ct][1], dim);
                        }
                        uint32_t o[4];
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            float re = dre[r], im = dim[r];
                            cmul_ip(re, im, twa[i][rt][ct][r]);
                            o[r] = TT::pack(re, im);
                        }
                        x2[ct][rt] = make_uint4(o[0], o[1], o[2], o[3]);
                    }
#pragma unroll
                for (int ct = 0; ct < 2; ++ct)
#pragma unroll
                    for (int ct2 = 0; ct2 < R2; ++ct2) {
                        f32x4 dre = zero4, dim = zero4;
#pragma unroll
                        for (int ks = 0; ks < R2; ++ks) {   // matrix as the A operand: rows k2, data columns k1
                            dre = TT::mfma(tab2[i][ks][ct2][0], x2[ct][ks], dre);
                            dim = TT::mfma(tab2[i][ks][ct2][1], x2[ct][ks], dim);
                        }
                        // lane: k1 = 16 ct + c16; reg r: k2 = 16 ct2 + 4q + r -> 4 consecutive words, one 16-byte write
                        uint32_t *dst = XB + c * G::PN3 + (16 * ct + c16) * G::PK1 + 16 * ct2 + 4 * q;
                        *(uint4 *)dst = make_uint4(TT::pack(dre[0], dim[0]), TT::pack(dre[1], dim[1]),
                                                   TT::pack(dre[2], dim[2]), TT::pack(dre[3], dim[3]));
                    }
            }
            if constexpr (AHEAD) {                        // phase B's first tile: in flight across the barrier
                load_B(0);
                load_kf(0, h_cur);
            }
        }
        lds_barrier();

        // ================= phase B: per k1 = c: stage 3, k_f, inverse 3, twiddle, inverse 2 -> XB in place
        {
            uint4 x3[C1][R2][R3];
#pragma unroll
            for (int i = 0; i < C1; ++i) {
                const int c = w * C1 + i;
#pragma unroll
                for (int ct2 = 0; ct2 < R2; ++ct2)
#pragma unroll
                    for (int ks = 0; ks < R3; ++ks) {
                        const uint32_t *src = XB + (16 * ks + 4 * q) * G::PN3 + c * G::PK1 + 16 * ct2 + c16;
                        x3[i][ct2][ks] = make_uint4(src[0], src[G::PN3], src[2 * G::PN3], src[3 * G::PN3]);
                    }
            }
            // The staging traffic rides in this compute-heavy phase: the previous pair's output
            // (YB, complete since the last barrier) goes to HBM, the next pair's prefetched input
            // goes to UB (its readers finished before the last barrier), and the loads of the pair
            // after that start.
            // (stage_in first: it waits for the prefetch, and on this target loads and stores
            //  retire through one counter, so it must not sit behind freshly issued stores)
            stage_in();
            issue_loads(k + 2);
            if (k > 0) store_out(k - 1);
#pragma unroll
            for (int i = 0; i < C1; ++i) {
                const int c = w * C1 + i;
                if constexpr (AHEAD) {
                    if (i + 1 < C1) {
                        load_B(i + 1);
                        load_kf(i + 1, h_cur);
                    }
                } else if constexpr (!REGC) {
                    load_B(i);
                    load_kf(i, h_cur);
                }
                uint4 x3i[R2][R3];                        // [k2 tile][K step = k3 tile]
#pragma unroll
                for (int ct2 = 0; ct2 < R2; ++ct2)
#pragma unroll
                    for (int ct3 = 0; ct3 < R3; ++ct3) {
                        f32x4 dre = zero4, dim = zero4;
#pragma unroll
                        for (int ks = 0; ks < R3; ++ks) {  // matrix is the A operand: rows k3, data columns k2
                            dre = TT::mfma(tab3[ks][ct3][0], x3[i][ct2][ks], dre);
                            dim = TT::mfma(tab3[ks][ct3][1], x3[i][ct2][ks], dim);
                        }
                        // the product runs in fp32 (plain multiply-adds overlap with the matrix cores of the
                        // other wave, the 16-bit dot products do not); the constant is widened in two cheap ops
                        uint32_t o[4];
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            float re = dre[r], im = dim[r];
                            cmul_ip(re, im, T4::widen(kfr[i][ct2][ct3][r]));
                            o[r] = TT::pack(re, im);
                        }
                        x3i[ct2][ct3] = make_uint4(o[0], o[1], o[2], o[3]);
                    }
                uint4 x2i[R3][R2];                        // [n3 tile][K step = k2 tile]
#pragma unroll
                for (int ct2 = 0; ct2 < R2; ++ct2)
#pragma unroll
                    for (int cn3 = 0; cn3 < R3; ++cn3) {
                        f32x4 dre = zero4, dim = zero4;
#pragma unroll
                        for (int ks = 0; ks < R3; ++ks) {
                            dre = TT::mfma(x3i[ct2][ks], tab3i[ks][cn3][0], dre);
                            dim = TT::mfma(x3i[ct2][ks], tab3i[ks][cn3][1], dim);
                        }
                        uint32_t o[4];
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            float re = dre[r], im = dim[r];
                            cmul_ip(re, im, twb[i][ct2][cn3][r]);
                            o[r] = TT::pack(re, im);
                        }
                        x2i[cn3][ct2] = make_uint4(o[0], o[1], o[2], o[3]);
                    }
#pragma unroll
                for (int cn3 = 0; cn3 < R3; ++cn3)
#pragma unroll
                    for (int cn2 = 0; cn2 < R2; ++cn2) {
                        f32x4 dre = zero4, dim = zero4;
#pragma unroll
                        for (int ks = 0; ks < R2; ++ks) {   // matrix as the A operand: rows n2, data columns n3
                            dre = TT::mfma(tab2i[i][ks][cn2][0], x2i[cn3][ks], dre);
                            dim = TT::mfma(tab2i[i][ks][cn2][1], x2i[cn3][ks], dim);
                        }
                        // lane: n3 = 16 cn3 + c16; reg r: n2 = 16 cn2 + 4q + r -> one 16-byte write
                        uint32_t *dst = XB + (16 * cn3 + c16) * G::PN3 + c * G::PK1 + 16 * cn2 + 4 * q;
                        *(uint4 *)dst = make_uint4(TT::pack(dre[0], dim[0]), TT::pack(dre[1], dim[1]),
                                                   TT::pack(dre[2], dim[2]), TT::pack(dre[3], dim[3]));
                    }
            }
        }
        lds_barrier();

        // ================= phase C: per n3 = c: inverse stage 1 (n1 < 16; re -> row b, im -> row b+1) -> YB
        {
            uint4 x1i[C3][R2][2];
#pragma unroll
            for (int i = 0; i < C3; ++i) {
                const int c = w * C3 + i;
#pragma unroll
                for (int cn2 = 0; cn2 < R2; ++cn2)
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks) {
                        const uint32_t *src = XB + c * G::PN3 + (16 * ks + 4 * q) * G::PK1 + 16 * cn2 + c16;
                        x1i[i][cn2][ks] = make_uint4(src[0], src[G::PK1], src[2 * G::PK1], src[3 * G::PK1]);
                    }
            }
#pragma unroll
            for (int i = 0; i < C3; ++i) {
                const int c = w * C3 + i;
#pragma unroll
                for (int cn2 = 0; cn2 < R2; ++cn2)
#pragma unroll
                    for (int rt = 0; rt < RT1; ++rt) {
                        f32x4 dre = zero4, dim = zero4;
#pragma unroll
                        for (int ks = 0; ks < 2; ++ks) {
                            dre = TT::mfma(tab1i[ks][rt][0], x1i[i][cn2][ks], dre);
                            dim = TT::mfma(tab1i[ks][rt][1], x1i[i][cn2][ks], dim);
                        }
                        // lane: n2 = 16 cn2 + c16; reg r: n1 = 16 rt + 4q + r
                        if constexpr (CPLX) {
                            uint32_t *dst = YBC + (16 * rt + 4 * q) * G::PQ1C + (16 * cn2 + c16) * G::PRC + c;
#pragma unroll
                            for (int r = 0; r < 4; ++r) dst[r * G::PQ1C] = TT::pack(dre[r], dim[r]);
                        } else {
                            uint16_t *dst = YB + (4 * q) * G::PQ1 + (16 * cn2 + c16) * G::PR + c;
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                dst[r * G::PQ1] = TT::cvt(dre[r]);
                                dst[G::SU + r * G::PQ1] = TT::cvt(dim[r]);
                            }
                        }
                    }
            }
            if constexpr (AHEAD) load_A(0);               // the next item's first phase-A tile
        }
        lds_barrier();
    }
    store_out(cnt - 1);
}

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
    for (int n = threadIdx.x; n < Ms; n += FILT_THREADS) {
        const int t = (reversed && n != 0) ? Ms - n : n;
        XF[lds_slot(n)] = make_float2(t < Nk ? k[h * Nk + t] : 0.f, 0.f);
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

// Rows: for the causal kernel (CPLX false) B batch rows of H channels, N samples each; for the
// complex-row kernel B rows per k_f row, H k_f rows.
template <int N2, int N3, typename TT, bool REGC, bool CPLX, int LIVE = 4>
int launch(const fftconv_plan *p, const void *u, const void *kf, void *y, int64_t B, int64_t H, int64_t N,
           hipStream_t s, int KoN = 0, int ko_lo = 0, int ko_hi = 0)
{
    using G = Geo<N2, N3>;
    auto kern = k_fused3<N2, N3, TT, REGC, CPLX, LIVE>;
    constexpr size_t lds = CPLX ? G::LDS_BYTES_C : G::LDS_BYTES;
    FC_TRY(raise_dynamic_lds((const void *)kern, (int)lds));
    const int64_t npairs = CPLX ? B : (B + 1) / 2;
    const int64_t T = H * npairs;
    if (T >= ((int64_t)1 << 31)) {
        set_error("fftconv_forward: H * ceil(B/2) = %lld work items exceed the fused kernel's 2^31 limit", (long long)T);
        return FFTCONV_EUNSUPPORTED;
    }
    // one persistent workgroup per compute unit (fewer when there is less work than that); a
    // multiple of 8 for the streamed-table kernels (see the kernel's work split)
    int grid = (int)(T < p->f3.num_cu ? T : p->f3.num_cu);
    if (!REGC && grid >= 8) grid -= grid % 8;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(NT), lds, s, (const uint16_t *)u, (uint16_t *)y,
                       (const uint32_t *)kf, consts_of<N2, N3>(p), (int)B, (int)H, (int)N, KoN, ko_lo, ko_hi, launch_gate());
    FC_HIP(hipGetLastError());
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
                      hipStream_t s, int ko_n, int ko_lo, int ko_hi)
{
    int64_t live_rows = kf_rows;
    if (ko_n > 0) {
        if (ko_lo >= ko_hi) ko_n = 0;                            // everything live
        else live_rows = kf_rows / ko_n * (ko_lo + ko_n - ko_hi);
    }
    if (p->dtype == FFTCONV_F16)
        return launch<16, 16, F16, false, true>(p, rows, kf, rows, rows_per_kf, live_rows, Geo<16, 16>::M, s, ko_n, ko_lo,
                                                ko_hi);
    return launch<16, 16, BF16, false, true>(p, rows, kf, rows, rows_per_kf, live_rows, Geo<16, 16>::M, s, ko_n, ko_lo,
                                             ko_hi);
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
