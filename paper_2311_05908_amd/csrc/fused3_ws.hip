// Wave-specialised fused causal FFT convolution, fft_size 8192 = 32*16*16, 16-bit I/O
// (paper Algorithm 3; index maps, tables and k_f layout: see fused3.hip).
//
// Why a second schedule: with every wave running the same phase at the same time, all eight
// waves of a workgroup meet the same LDS latencies and barriers together and the SIMDs idle
// ~40 % of the time.  Here the workgroup is split by role and software-pipelined over work
// items (a work item = one pair of batch rows of one channel):
//   waves 0-3 ("outer"): phase A of item s+1 (stage 1, twiddle, stage 2 -> XB), phase C of
//                        item s-1 (inverse stage 1 -> YB), and all staging: prefetch of item
//                        s+3 from HBM, input of item s+2 into UB, output of item s-2 to HBM;
//   waves 4-7 ("inner"): phase B of item s (stage 3, k_f, inverse 3, twiddle, inverse 2, in place).
// Each SIMD holds one wave of each role, so while one waits on LDS the other computes, and a
// step needs ONE workgroup barrier.  XB, UB and YB are double buffered by item parity:
//   XB[t&1]: written by A(t) in step t-1, rewritten in place by B(t) in step t, read by C(t) in step t+1;
//            A(t+2) reuses it in step t+1, and every outer wave reads (C) and rewrites (A) only its own n3 planes.
//   UB[t&1]: written in step t-2, read by A(t) in step t-1.   YB[t&1]: written by C(t) in step t+1, read in step t+2.
// Each role keeps only its own constant tables in registers (outer: stage-1/2 matrices and the
// forward twiddles of its 4 n3 planes; inner: stage-3 matrices, k_f[h], inverse twiddles and
// per-k1 inverse matrices of its 8 k1 planes).
#include "fused3_common.h"


namespace fftconv {
namespace f3 {

namespace {

using G = Geo<16, 16>;
constexpr int XBW = G::XB_WORDS;
constexpr int UBE = G::UB_ELEMS;
constexpr size_t WS_LDS_BYTES = (size_t)2 * XBW * 4 + (size_t)4 * UBE * 2;
constexpr int PT = 256;                       // threads per role
constexpr int PCH = G::M / 8 / PT;            // 16-byte input chunks per outer-role thread and item (4)

// FULL: B even and N == fft_size/2, so every load and store of a work item is in range and
// unconditional (the compiler can then count outstanding memory operations exactly).
// groups > 1 (nseg == 1): a work item holds `groups` pairs of rows of a transform of length 8192 / groups (tables
// from build_tables(..., groups)): positions [g * half, (g + 1) * half) of its 4096-sample input / output slot,
// half = 2^lg_half = fft_size / 2, belong to the pair 2 (pair * groups + g), of which the first N are real samples.
// GATE (gated form y = v . ((u . w) * k), Section 3.1 / 4.1; needs nseg == 1): bit 0 = the input gate
// wg multiplies u on its way into LDS, bit 1 = the output gate vg multiplies y on its way out; the
// gates travel with the staging traffic of the outer role (16-byte chunks, one item ahead / behind).
// SKIP1 (frequency-sparse filters, Appendix A.4: the trip count of the per-plane loop): bit k1 of live_k1
// clear means k_f is zero on the whole plane k1; phase B then writes zeros for it instead of computing.
template <typename TT, bool FULL, int GATE, bool SKIP1 = false>
__global__ void __launch_bounds__(NT) k_fused3_ws(const uint16_t *__restrict__ u, uint16_t *__restrict__ y,
                                                 const uint2 *__restrict__ kf, Consts cs, int B, int H, int N, int nseg, int P, int Lo,
                                                 const uint16_t *__restrict__ wg, const uint16_t *__restrict__ vg,
                                                 uint32_t live_k1, int groups, int lg_half, LaunchGate gate)
{
    extern __shared__ uint32_t smem[];
    if (gate_closed(gate)) return;
    uint32_t *const XBb = smem;                                   // [2][XBW]
    uint16_t *const UBb = (uint16_t *)(smem + 2 * XBW);           // [2][UBE]
    uint16_t *const YBb = UBb + 2 * UBE;                          // [2][UBE]

    const int tid = threadIdx.x, l = tid & 63, q = l >> 4, c16 = l & 15;
    // the wave index as a scalar, so that the role branch is a uniform branch and each wave runs
    // exactly one of the two loops (both execute the same number of workgroup barriers)
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    // A work item is (channel h, pair of batch rows, segment).  Segments exist only for partial
    // convolutions (a filter much shorter than the sequence): the row is cut into overlapping
    // windows of at most fft/2 samples, segment 0 yields outputs [0, fft/2), segment j >= 1 yields Lo
    // outputs and reads P samples of history before them (P >= filter length - 1), i.e. overlap-save.
    const int npairs = (B + 2 * groups - 1) / (2 * groups);
    const int per_h = npairs * nseg;
    const long long T = (long long)H * per_h;
    const int t0 = (int)(T * blockIdx.x / gridDim.x);
    const int t1 = (int)(T * (blockIdx.x + 1) / gridDim.x);
    if (t0 >= t1) return;
    const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};
    // (channel, pair, segment) of a work item, t = (h * npairs + pair) * nseg + seg.  Every loop below walks its
    // items one by one, so the three digits are counted up (a few scalar adds and compares per step) instead of
    // divided out of t at every use.
    struct Item {
        int h, pair, seg;
    };
    auto item_at = [&](int t) {
        Item it;
        it.h = t / per_h;
        const int rem = t - it.h * per_h;
        it.pair = rem / nseg;
        it.seg = rem - it.pair * nseg;
        return it;
    };
    auto item_next = [&](Item &it) {
        if (++it.seg == nseg) {
            it.seg = 0;
            if (++it.pair == npairs) {
                it.pair = 0;
                ++it.h;
            }
        }
    };

    if (w < 4) {
        // =========================== outer role: phases A and C, staging ===========================
        const int ptid = tid;                                     // 0..255
        // chunk j of this thread sits at position cn[j % 2] of the item's slot: group cg[], offset co[] in its row
        int cg[2], co[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int n = (ptid + PT * e) * 8;
            cg[e] = n >> lg_half;
            co[e] = n & ((1 << lg_half) - 1);
        }
        uint4 tab1[2][2], tab1i[2][2], tab2[4][2];
        uint2 twa[4][2][4];
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                tab1[a][p] = cs.tab1[((0 * 2 + a) * 2 + p) * 64 + l];       // K step 0 only (n1 < 16)
                tab1i[a][p] = cs.tab1i[((a * 2 + 0) * 2 + p) * 64 + l];     // row tile 0 only (n1 < 16)
            }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c = 4 * w + i;
#pragma unroll
            for (int p = 0; p < 2; ++p) tab2[i][p] = cs.tab2[(c * 2 + p) * 64 + l];
#pragma unroll
            for (int ct = 0; ct < 2; ++ct)
#pragma unroll
                for (int r = 0; r < 4; ++r) twa[i][ct][r] = cs.twa16[((c * 2 + ct) * 4 + r) * 64 + l];
        }
        // input prefetch: the loads of item s+2 are issued at the start of step s and staged at its end
        uint4 pre[PCH];
        uint4 prew[(GATE & 1) ? PCH : 1], prev[(GATE & 2) ? PCH : 1];
        // it: the item min(t, t1 - 1)
        auto issue_loads = [&](int t, const Item &it) {
            const int h = it.h, pair = it.pair, seg = it.seg;
#pragma unroll
            for (int j = 0; j < PCH; ++j) {
                const int s = j / 2;
                const int n = co[j % 2];
                if constexpr (FULL) {
                    // (nseg == 1) past the end of the range the last item is fetched again (in range, unused)
                    const int hc = it.h, pc = it.pair;
                    const size_t ofs = ((size_t)(2 * (pc * groups + cg[j % 2]) + s) * H + hc) * N + n;
                    pre[j] = *(const uint4 *)(u + ofs);
                    if constexpr (GATE & 1) prew[j] = *(const uint4 *)(wg + ofs);
                } else {
                    const int b = 2 * (pair * groups + cg[j % 2]) + s;
                    uint4 v = make_uint4(0, 0, 0, 0);
                    const int in_ofs = seg == 0 ? 0 : G::M / 2 + (seg - 1) * Lo - P;
                    const uint16_t *row = u + ((size_t)b * H + h) * N + in_ofs;
                    const bool ok = t < t1 && b < B && n < N - in_ofs;
                    if (ok) v = *(const uint4 *)(row + n);
                    pre[j] = v;
                    if constexpr (GATE & 1) {
                        uint4 g = make_uint4(0, 0, 0, 0);
                        if (ok) g = *(const uint4 *)(wg + ((size_t)b * H + h) * N + n);     // nseg == 1: in_ofs == 0
                        prew[j] = g;
                    }
                }
            }
        };
        // output gate of item t (the item stored at the end of this step)
        // it: the item max(t, t0)
        auto issue_loads_v = [&](const Item &it) {
            if constexpr (GATE & 2) {
                const int h = it.h, pair = it.pair;
#pragma unroll
                for (int j = 0; j < PCH; ++j) {
                    const int s = j / 2;
                    const int n = co[j % 2];
                    const int b = 2 * (pair * groups + cg[j % 2]) + s;
                    uint4 g = make_uint4(0, 0, 0, 0);
                    if (FULL || (b < B && n < N)) g = *(const uint4 *)(vg + ((size_t)b * H + h) * N + n);
                    prev[j] = g;
                }
            }
        };
        auto stage_in = [&](uint16_t *UB) {
#pragma unroll
            for (int j = 0; j < PCH; ++j) {
                const int s = j / 2;
                const int n = (ptid + PT * (j % 2)) * 8;
                const int n3 = n % 16, n2 = (n / 16) % 16, n1 = n / 256;
                uint32_t *dst = (uint32_t *)(UB + s * G::SU + n1 * G::PQ1 + n2 * G::PR + n3);
                uint4 v = pre[j];
                if constexpr (GATE & 1) v = TT::mul8(v, prew[j]);
                dst[0] = v.x;
                dst[1] = v.y;
                dst[2] = v.z;
                dst[3] = v.w;
            }
        };
        auto store_out = [&](const Item &it, const uint16_t *YB) {
            const int h = it.h, pair = it.pair, seg = it.seg;
            const int skip = seg == 0 ? 0 : P;                    // outputs before `skip` lack history: dropped
            const int out_ofs = seg == 0 ? 0 : G::M / 2 + (seg - 1) * Lo;
            const int out_len = min(seg == 0 ? G::M / 2 : Lo, N - out_ofs);
#pragma unroll
            for (int j = 0; j < PCH; ++j) {
                const int s = j / 2;
                const int n = (ptid + PT * (j % 2)) * 8;          // position in the item's slot
                const int nr = co[j % 2];                         // ... in its row
                const int b = 2 * (pair * groups + cg[j % 2]) + s;
                const int n3 = n % 16, n2 = (n / 16) % 16, n1 = n / 256;
                const uint32_t *src = (const uint32_t *)(YB + s * G::SU + n1 * G::PQ1 + n2 * G::PR + n3);
                uint4 v = make_uint4(src[0], src[1], src[2], src[3]);
                if constexpr (GATE & 2) v = TT::mul8(v, prev[j]);
                if constexpr (FULL) {
                    *(uint4 *)(y + ((size_t)b * H + h) * N + nr) = v;
                } else {
                    uint16_t *row = y + ((size_t)b * H + h) * N + out_ofs;
                    if (b < B && nr >= skip && nr - skip < out_len) *(uint4 *)(row + (nr - skip)) = v;
                }
            }
        };

        // prologue: item t0 staged; item t0+1 is fetched at the start of the first step
        Item it_st = item_at(t0);                                 // the item stored in this step: max(s - 2, t0)
        Item it_ld = it_st;                                       // the item loaded in this step: min(s + 2, t1 - 1)
        issue_loads(t0, it_ld);
        stage_in(UBb + (t0 & 1) * UBE);
        lds_barrier();
        if (t0 + 1 < t1) item_next(it_ld);                        // the first step (s = t0 - 1) loads item t0 + 1

        for (int s = t0 - 1; s <= t1 + 1; ++s) {
            const bool doC = s - 1 >= t0 && s - 1 < t1;
            const bool doA = s + 1 < t1;
            issue_loads(s + 2, it_ld);
            issue_loads_v(it_st);
            // ---- phase C of item s-1: inverse stage 1, n1 < 16; re -> row b, im -> row b+1 -> YB
            if (doC) {
                const uint32_t *XB = XBb + ((s - 1) & 1) * XBW;
                uint32_t *YB32 = (uint32_t *)(YBb + ((s - 1) & 1) * UBE);
                auto read_c = [&](int i, uint4 (&x)[2]) {
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks) {
                        const uint32_t *src = XB + (4 * w + i) * G::PN3 + (16 * ks + 4 * q) * G::PK1 + c16;
                        x[ks] = make_uint4(src[0], src[G::PK1], src[2 * G::PK1], src[3 * G::PK1]);
                    }
                };
                uint4 xc[2][2][2];                                // [buffer][plane of the pair][K step]
                read_c(0, xc[0][0]);
                read_c(1, xc[0][1]);
#pragma unroll
                for (int ip = 0; ip < 2; ++ip) {
                    if (ip == 0) {
                        read_c(2, xc[1][0]);
                        read_c(3, xc[1][1]);
                    }
                    f32x4 dre[2], dim[2];
#pragma unroll
                    for (int k = 0; k < 2; ++k) {
                        dre[k] = zero4;
                        dim[k] = zero4;
#pragma unroll
                        for (int ks = 0; ks < 2; ++ks) {
                            dre[k] = TT::mfma(tab1i[ks][0], xc[ip][k][ks], dre[k]);
                            dim[k] = TT::mfma(tab1i[ks][1], xc[ip][k][ks], dim[k]);
                        }
                    }
                    // lane: n2 = c16; reg r: n1 = 4q + r; the two planes are adjacent n3 -> one word each
                    const int ce = 4 * w + 2 * ip;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int e = (4 * q + r) * G::PQ1 + c16 * G::PR + ce;
                        YB32[e / 2] = TT::pack(dre[0][r], dre[1][r]);
                        YB32[(G::SU + e) / 2] = TT::pack(dim[0][r], dim[1][r]);
                    }
                }
            }
            // ---- phase A of item s+1: stage 1, twiddle, stage 2 -> XB
            if (doA) {
                uint32_t *XB = XBb + ((s + 1) & 1) * XBW;
                // rows n2 = c16; slots (2r+s) = u_s[n1 = 4q + r]; two adjacent n3 planes per 32-bit word
                const uint32_t *UB32 = (const uint32_t *)(UBb + ((s + 1) & 1) * UBE);
                uint32_t w0[2][4], w1[2][4];
#pragma unroll
                for (int ip = 0; ip < 2; ++ip)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int e = (4 * q + r) * G::PQ1 + c16 * G::PR + 4 * w + 2 * ip;
                        w0[ip][r] = UB32[e / 2];
                        w1[ip][r] = UB32[(G::SU + e) / 2];
                    }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int c = 4 * w + i;
                    const uint32_t sel = (i & 1) ? 0x07060302u : 0x05040100u;
                    const uint4 x1 = make_uint4(__builtin_amdgcn_perm(w1[i / 2][0], w0[i / 2][0], sel),
                                                __builtin_amdgcn_perm(w1[i / 2][1], w0[i / 2][1], sel),
                                                __builtin_amdgcn_perm(w1[i / 2][2], w0[i / 2][2], sel),
                                                __builtin_amdgcn_perm(w1[i / 2][3], w0[i / 2][3], sel));
                    uint4 x2[2];
#pragma unroll
                    for (int ct = 0; ct < 2; ++ct) {
                        const f32x4 dre = TT::mfma(x1, tab1[ct][0], zero4);
                        const f32x4 dim = TT::mfma(x1, tab1[ct][1], zero4);
                        x2[ct] = TT::ctw4(dre, dim, twa[i][ct]);
                    }
#pragma unroll
                    for (int ct = 0; ct < 2; ++ct) {
                        const f32x4 dre = TT::mfma(tab2[i][0], x2[ct], zero4);
                        const f32x4 dim = TT::mfma(tab2[i][1], x2[ct], zero4);
                        // lane: k1 = 16 ct + c16; reg r: k2 = 4q + r
                        uint32_t *dst = XB + c * G::PN3 + (16 * ct + c16) * G::PK1 + 4 * q;
                        *(uint4 *)dst = make_uint4(TT::pack(dre[0], dim[0]), TT::pack(dre[1], dim[1]),
                                                   TT::pack(dre[2], dim[2]), TT::pack(dre[3], dim[3]));
                    }
                }
            }
            // ---- staging: input of item s+2 (its loads were issued at the start of this step) -> UB,
            //      then output of item s-2 -> HBM.  The input goes first: it waits for the loads, and
            //      loads and stores retire through one counter on this target.
            if (s + 2 < t1) stage_in(UBb + ((s + 2) & 1) * UBE);
            if (s - 2 >= t0) {
                store_out(it_st, YBb + ((s - 2) & 1) * UBE);
                item_next(it_st);
            }
            if (s + 3 < t1) item_next(it_ld);
            lds_barrier();
        }
    } else {
        // =========================== inner role: phase B ===========================
        const int wq = w - 4;
        uint4 tab3[2], tab3i[2], tab2i[8][2];
        uint2 twb[8][4], kfr[8][4];
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
            for (int r = 0; r < 4; ++r) twb[i][r] = cs.twb16[(c * 4 + r) * 64 + l];
        }
        lds_barrier();                                          // pairs with the outer role's prologue barrier
        int h_cur = -1;
        Item it_b = item_at(t0);                                  // the item of phase B in this step
        for (int s = t0 - 1; s <= t1 + 1; ++s) {
            if (s >= t0 && s < t1) {
                const int h = it_b.h;
                item_next(it_b);
                if (h != h_cur) {                                 // new channel: its k_f slice for this wave's k1 planes
                    h_cur = h;
#pragma unroll
                    for (int i = 0; i < 8; ++i)
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            kfr[i][r] = kf[(size_t)h * G::KF_PER_H + ((8 * wq + i) * 4 + r) * 64 + l];
                }
                uint32_t *XB = XBb + (s & 1) * XBW;
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
                    if constexpr (SKIP1) {
                        if (!((live_k1 >> c) & 1u)) {             // wave-uniform
                            *(uint4 *)(XB + c16 * G::PN3 + c * G::PK1 + 4 * q) = make_uint4(0, 0, 0, 0);
                            continue;
                        }
                    }
                    const uint4 x3v = xq[i % 3];
                    // stage 3: matrix rows k3, data columns k2
                    f32x4 dre = TT::mfma(tab3[0], x3v, zero4);
                    f32x4 dim = TT::mfma(tab3[1], x3v, zero4);
                    const uint4 x3i = TT::ctw4(dre, dim, kfr[i]);
                    // inverse stage 3: rows k2, contraction over k3
                    dre = TT::mfma(x3i, tab3i[0], zero4);
                    dim = TT::mfma(x3i, tab3i[1], zero4);
                    const uint4 x2i = TT::ctw4(dre, dim, twb[i]);
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
    }
}

}  // namespace

// nseg == 1: plain causal convolution (N <= fft/2).  nseg > 1: overlap-save segments of a partial
// convolution, P samples of history per segment, Lo = fft/2 - P outputs per later segment.
int fused3_ws_launch(const fftconv_plan *p, const void *consts, const void *u, const void *kf, void *y, int64_t B,
                     int nseg, int P, hipStream_t s, const void *wg, const void *vg, uint32_t live_k1)
{
    // plans for fft 512 .. 4096 put 8192 / fft transforms into one work item (their tables say so)
    const int groups = p->M < G::M && consts == p->f3.consts ? (int)(G::M / p->M) : 1;
    int lg_half = 0;
    while ((G::M / 2 / groups) >> (lg_half + 1)) ++lg_half;
    const int64_t npairs = (B + 2 * groups - 1) / (2 * groups);
    const int64_t T = p->H * npairs * nseg;
    const int Lo = G::M / 2 - P;
    if (T >= ((int64_t)1 << 31) - 8) {
        set_error("fftconv_forward: H * ceil(B/2) = %lld work items exceed the fused kernel's limit", (long long)T);
        return FFTCONV_EUNSUPPORTED;
    }
    if ((wg || vg) && nseg != 1) {
        set_error("fused 8192 kernel: gates cannot be combined with overlapping segments");
        return FFTCONV_EUNSUPPORTED;
    }
    if (groups > 1 && nseg != 1) {
        set_error("fused 8192 kernel: grouped short transforms cannot be combined with overlapping segments");
        return FFTCONV_EUNSUPPORTED;
    }
    const bool full = (B % (2 * groups) == 0) && p->N == G::M / 2 / groups && nseg == 1;
    const bool f16 = p->dtype == FFTCONV_F16;
    const int gate = (wg ? 1 : 0) | (vg ? 2 : 0);
    using Kern = void (*)(const uint16_t *, uint16_t *, const uint2 *, Consts, int, int, int, int, int, int,
                          const uint16_t *, const uint16_t *, uint32_t, int, int, LaunchGate);
    static const Kern table[2][2][4] = {
        {{k_fused3_ws<BF16, false, 0>, k_fused3_ws<BF16, false, 1>, k_fused3_ws<BF16, false, 2>, k_fused3_ws<BF16, false, 3>},
         {k_fused3_ws<BF16, true, 0>, k_fused3_ws<BF16, true, 1>, k_fused3_ws<BF16, true, 2>, k_fused3_ws<BF16, true, 3>}},
        {{k_fused3_ws<F16, false, 0>, k_fused3_ws<F16, false, 1>, k_fused3_ws<F16, false, 2>, k_fused3_ws<F16, false, 3>},
         {k_fused3_ws<F16, true, 0>, k_fused3_ws<F16, true, 1>, k_fused3_ws<F16, true, 2>, k_fused3_ws<F16, true, 3>}}};
    // plane skipping: plain (ungated) convolution only
    static const Kern table_skip[2][2] = {{k_fused3_ws<BF16, false, 0, true>, k_fused3_ws<BF16, true, 0, true>},
                                          {k_fused3_ws<F16, false, 0, true>, k_fused3_ws<F16, true, 0, true>}};
    const bool skip = live_k1 != 0xffffffffu && gate == 0;
    const Kern kern = skip ? table_skip[f16 ? 1 : 0][full ? 1 : 0] : table[f16 ? 1 : 0][full ? 1 : 0][gate];
    FC_TRY(raise_dynamic_lds((const void *)kern, (int)WS_LDS_BYTES));
    const int grid = (int)(T < p->f3.num_cu ? T : p->f3.num_cu);
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(NT), WS_LDS_BYTES, s, (const uint16_t *)u, (uint16_t *)y,
                       (const uint2 *)kf, consts_at<16, 16>(consts), (int)B, (int)p->H, (int)p->N, nseg, P, Lo,
                       (const uint16_t *)wg, (const uint16_t *)vg, live_k1, groups, lg_half, launch_gate());
    FC_HIP(hipGetLastError());
    return FFTCONV_OK;
}

}  // namespace f3
}  // namespace fftconv
