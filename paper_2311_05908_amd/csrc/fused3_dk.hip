// Fused filter gradient of the causal FFT convolution, fft_size 8192 = 32*16*16, 16-bit I/O
// (paper Section 3.1 "Kernel Fusion and Recomputation": the backward pass recomputes the
// transforms instead of storing them, and reduces over the batch in frequency space).
//
//     dk_f[h] = sum_b conj(FFT(pad(u[b,h]))) . FFT(pad(dy[b,h])),      dk[h] = Re(iFFT(dk_f[h]))[0:Nk].
//
// Two batch rows share one complex transform here as well: z1 = u[b] + i u[b+1], z2 = dy[b] + i dy[b+1];
// conj(Z1) . Z2 = (wanted sum of the two rows) + i (a cross term), and both parts are spectra of real
// sequences, so the real part of the inverse transform of the accumulated products is dk and the
// cross terms only reach the imaginary part, which is dropped.
//
// The forward half of the wave-specialised 8192-point kernel (fused3_ws.hip: same tables, index maps
// and LDS layouts) runs on a stream of inputs u-pair, dy-pair, u-pair, ...:
//   waves 0-3 ("outer"): stage 1, twiddle, stage 2 of input s+1 -> XB[(s+1)&1]; staging of input s+2;
//   waves 4-7 ("inner"): stage 3 of input s; a u input leaves its spectrum in registers (fp32), the
//                        dy input that follows multiplies it in and adds to the channel's accumulator.
// A workgroup owns whole channels, so the accumulator (fp32, 64 registers per lane) never leaves the
// registers until the channel's last pair, when it is written out in the kernel's k_f order.  The
// inverse transform of the H accumulated spectra runs afterwards, one workgroup per channel in LDS (k_dk_finish).
#include "fused3_common.h"
#include "lds_fft.h"

namespace fftconv {
namespace f3 {

namespace {

using G = Geo<16, 16>;
constexpr int XBW = G::XB_WORDS;
constexpr int UBE = G::UB_ELEMS;
constexpr size_t DK_LDS_BYTES = (size_t)2 * XBW * 4 + (size_t)2 * UBE * 2;
constexpr int PT = 256;                       // threads per role
constexpr int PCH = G::M / 8 / PT;            // 16-byte input chunks per outer-role thread and input (4)

// FULL: B even and N == fft_size/2: every load is in range and unconditional.
// groups > 1: plans for fft 256 .. 4096, whose tables put `groups` transforms of length 8192 / groups into one
// input (fused3.hip, build_tables): positions [g * half, (g + 1) * half) of an input's 4096-sample slot,
// half = 2^lg_half = fft_size / 2, hold rows 2 (pair * groups + g), + 1.  The accumulator then holds one
// spectrum per group (slots k1 = g * (32 / groups) + k1'), which the unpacking step adds up.
template <typename TT, bool FULL>
__global__ void __launch_bounds__(NT) k_fused3_dk(const uint16_t *__restrict__ u, const uint16_t *__restrict__ dy,
                                                 float2 *__restrict__ dkf, Consts cs, int B, int H, int N, int groups,
                                                 int lg_half)
{
    extern __shared__ uint32_t smem[];
    uint32_t *const XBb = smem;                                   // [2][XBW]
    uint16_t *const UBb = (uint16_t *)(smem + 2 * XBW);           // [2][UBE]

    const int tid = threadIdx.x, l = tid & 63, q = l >> 4, c16 = l & 15;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    // channels of this workgroup: h = blockIdx.x + j * gridDim.x; its input stream: index
    // s = (j * npairs + pair) * 2 + which, which = 0 for the u rows of the pair, 1 for the dy rows
    const int npairs = (B + 2 * groups - 1) / (2 * groups);
    const int nch = (H - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x;
    const int S = nch * npairs * 2;
    if (S <= 0) return;
    const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};

    if (w < 4) {
        // =========================== outer role: stage 1, twiddle, stage 2, staging ===========================
        const int ptid = tid;
        uint4 tab1[2][2], tab2[4][2];
        uint2 twa[4][2][4];
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int p = 0; p < 2; ++p) tab1[a][p] = cs.tab1[((0 * 2 + a) * 2 + p) * 64 + l];   // K step 0 only (n1 < 16)
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
        uint4 pre[PCH];
        auto issue_loads = [&](int s) {
            const int sc = s < S ? s : S - 1;                     // past the end: the last input again (unused)
            const int which = sc & 1, item = sc >> 1;
            const int j = item / npairs, pair = item - j * npairs;
            const int h = (int)blockIdx.x + j * (int)gridDim.x;
            const uint16_t *src = which ? dy : u;
#pragma unroll
            for (int c = 0; c < PCH; ++c) {
                const int row = c / 2;
                const int np = (ptid + PT * (c % 2)) * 8;             // position in the input's slot
                const int n = np & ((1 << lg_half) - 1);             // ... in its row
                const int b = 2 * (pair * groups + (np >> lg_half)) + row;
                if constexpr (FULL) {
                    pre[c] = *(const uint4 *)(src + ((size_t)b * H + h) * N + n);
                } else {
                    uint4 v = make_uint4(0, 0, 0, 0);
                    if (b < B && n < N) v = *(const uint4 *)(src + ((size_t)b * H + h) * N + n);
                    pre[c] = v;
                }
            }
        };
        auto stage_in = [&](uint16_t *UB) {
#pragma unroll
            for (int c = 0; c < PCH; ++c) {
                const int row = c / 2;
                const int n = (ptid + PT * (c % 2)) * 8;
                const int n3 = n % 16, n2 = (n / 16) % 16, n1 = n / 256;
                uint32_t *dst = (uint32_t *)(UB + row * G::SU + n1 * G::PQ1 + n2 * G::PR + n3);
                dst[0] = pre[c].x;
                dst[1] = pre[c].y;
                dst[2] = pre[c].z;
                dst[3] = pre[c].w;
            }
        };

        // prologue: input 0 staged; input 1 is fetched at the start of the first step
        issue_loads(0);
        stage_in(UBb);
        lds_barrier();

        // One step; all but the last two have both parts and run as a loop of their own with constant flags, so that
        // a step is straight-line code: with the parts behind conditions the compiler moves the loads from the top
        // of the step down into the conditional block that consumes them, where they are waited for at once.
        auto step = [&](const int s, const bool doA, const bool doIn) __attribute__((always_inline)) {
            issue_loads(s + 2);
            // ---- stage 1, twiddle, stage 2 of input s+1 -> XB
            if (doA) {
                uint32_t *XB = XBb + ((s + 1) & 1) * XBW;
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
            if (doIn) stage_in(UBb + ((s + 2) & 1) * UBE);
            lds_barrier();
        };
        int s = -1;
        for (; s + 2 < S; ++s) step(s, true, true);
        for (; s < S; ++s) step(s, s + 1 < S, false);
    } else {
        // =========================== inner role: stage 3, product, accumulation ===========================
        const int wq = w - 4;
        uint4 tab3[2];
#pragma unroll
        for (int p = 0; p < 2; ++p) tab3[p] = cs.tab3[p * 64 + l];
        f32x4 z1re[8], z1im[8], accre[8], accim[8];               // per k1 plane of this wave
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            z1re[i] = zero4;
            z1im[i] = zero4;
            accre[i] = zero4;
            accim[i] = zero4;
        }
        lds_barrier();                                            // pairs with the outer role's prologue barrier
        lds_barrier();                                            // step -1: nothing to do yet
        for (int s = 0; s < S; ++s) {
            {
                const int which = s & 1, item = s >> 1;
                const uint32_t *XB = XBb + (s & 1) * XBW;
                // operand of stage 3 for plane k1: columns k2 = c16, slots = (re, im) of n3 = 4q + r
                auto read_plane = [&](int i) {
                    const uint32_t *src = XB + (4 * q) * G::PN3 + (8 * wq + i) * G::PK1 + c16;
                    return make_uint4(src[0], src[G::PN3], src[2 * G::PN3], src[3 * G::PN3]);
                };
                uint4 xq[3];
#pragma unroll
                for (int i = 0; i < 2; ++i) xq[i] = read_plane(i);
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    if (i + 2 < 8) xq[(i + 2) % 3] = read_plane(i + 2);
                    // stage 3: matrix rows k3, data columns k2; lane: k2 = c16, reg r: k3 slot 4q + r
                    const f32x4 dre = TT::mfma(tab3[0], xq[i % 3], zero4);
                    const f32x4 dim = TT::mfma(tab3[1], xq[i % 3], zero4);
                    if (which == 0) {
                        z1re[i] = dre;
                        z1im[i] = dim;
                    } else {
#pragma unroll
                        for (int r = 0; r < 4; ++r) {             // acc += conj(Z1) * Z2
                            accre[i][r] += z1re[i][r] * dre[r] + z1im[i][r] * dim[r];
                            accim[i][r] += z1re[i][r] * dim[r] - z1im[i][r] * dre[r];
                        }
                    }
                }
                // last pair of a channel: write the accumulator out ([h][k1][r][lane], the k_f order) and clear it
                const int j = item / npairs, pair = item - j * npairs;
                if (which == 1 && pair == npairs - 1) {
                    const int h = (int)blockIdx.x + j * (int)gridDim.x;
#pragma unroll
                    for (int i = 0; i < 8; ++i)
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            dkf[(size_t)h * G::KF_PER_H + ((8 * wq + i) * 4 + r) * 64 + l] =
                                make_float2(accre[i][r], accim[i][r]);
                            accre[i][r] = 0.f;
                            accim[i][r] = 0.f;
                        }
                }
            }
            lds_barrier();
        }
    }
}

// dk_f in the kernel's order (slot (k1 * 4 + r) * 64 + lane as in the fused k_f layout) -> dk, one workgroup
// per channel: the 8192 slots are read in order and scattered to their positions in LDS, the unnormalised
// inverse transform of length Ms = 8192 / groups runs there (lds_fft.h), real part times 1/Ms of the first Nk
// samples goes out.  groups > 1: bin k1' + N1s (k2 + 16 k3) of the short transform is the sum over the groups g
// of the slots k1 = g N1s + k1'; the groups are added one after the other (a fixed order).
constexpr int DK_FIN_THREADS = 512;
__global__ void __launch_bounds__(DK_FIN_THREADS) k_dk_finish(const float2 *__restrict__ dkf, float *__restrict__ dk,
                                                             const float2 *__restrict__ w, FacList fl, int64_t Nk, int groups)
{
    extern __shared__ float2 XD[];
    const int Ms = G::M / groups, N1s = N1 / groups;
    const int64_t h = blockIdx.x;
    const int per_group = G::M / groups;                     // slots of one group: k1 in [g N1s, (g + 1) N1s)
    for (int g = 0; g < groups; ++g) {
#pragma unroll 4
        for (int i = threadIdx.x; i < per_group; i += DK_FIN_THREADS) {
            const int d = g * per_group + i;
            const int lane = d % 64, r = (d / 64) % 4, k1 = d / 256;
            const int k2 = lane % 16, k3 = k3_at_index(4 * (lane / 16) + r, 16);
            const int fs = (k1 % N1s) + N1s * (k2 + 16 * k3);
            const int slot = lds_slot(lds_pos(fs, fl, Ms));
            float2 v = dkf[h * G::M + d];
            if (g > 0) {
                const float2 o = XD[slot];
                v.x += o.x;
                v.y += o.y;
            }
            XD[slot] = v;
        }
        __syncthreads();
    }
    lds_inverse(XD, w, fl, Ms, 1);
    const float scale = 1.0f / (float)Ms;
    for (int n = threadIdx.x; n < Nk; n += DK_FIN_THREADS) dk[h * Nk + n] = XD[lds_slot(n)].x * scale;
}

}  // namespace

bool fused3_dk_supported(const fftconv_plan *p) { return p->path == PATH_FUSED3 && p->M <= G::M; }

// dkf: H * 8192 float2 in the kernel's order.
int fused3_dk_accumulate(const fftconv_plan *p, const void *u, const void *dy, void *dkf, int64_t B, hipStream_t s)
{
    if (((uintptr_t)u | (uintptr_t)dy) & 15) {
        set_error("fftconv_backward_filter: u and dy must be 16-byte aligned for this plan");
        return FFTCONV_EINVAL;
    }
    const int groups = (int)(G::M / p->M);
    int lg_half = 0;
    while ((G::M / 2 / groups) >> (lg_half + 1)) ++lg_half;
    const int64_t npairs = (B + 2 * groups - 1) / (2 * groups);
    if (p->H * npairs >= ((int64_t)1 << 29)) {
        set_error("fftconv_backward_filter: H * ceil(B/2) = %lld exceeds the fused kernel's limit",
                  (long long)(p->H * npairs));
        return FFTCONV_EUNSUPPORTED;
    }
    const bool full = (B % (2 * groups) == 0) && p->N == G::M / 2 / groups;
    const bool f16 = p->dtype == FFTCONV_F16;
    void (*kern)(const uint16_t *, const uint16_t *, float2 *, Consts, int, int, int, int, int) =
        f16 ? (full ? k_fused3_dk<F16, true> : k_fused3_dk<F16, false>)
            : (full ? k_fused3_dk<BF16, true> : k_fused3_dk<BF16, false>);
    FC_TRY(raise_dynamic_lds((const void *)kern, (int)DK_LDS_BYTES));
    const int grid = (int)(p->H < p->f3.num_cu ? p->H : p->f3.num_cu);
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(NT), DK_LDS_BYTES, s, (const uint16_t *)u, (const uint16_t *)dy,
                       (float2 *)dkf, consts_at<16, 16>(p->f3.consts), (int)B, (int)p->H, (int)p->N, groups, lg_half);
    FC_HIP(hipGetLastError());
    return FFTCONV_OK;
}

int fused3_dk_finish(const fftconv_plan *p, const void *dkf, float *dk, int64_t Nk, hipStream_t s)
{
    FC_TRY(raise_dynamic_lds((const void *)k_dk_finish, (int)lds_row_bytes(G::M, sizeof(float2))));
    hipLaunchKernelGGL(k_dk_finish, dim3((unsigned)p->H), dim3(DK_FIN_THREADS), lds_row_bytes(p->M, sizeof(float2)), s,
                       (const float2 *)dkf, dk, (const float2 *)p->st.w32, staged_fac_list(p), Nk, (int)(G::M / p->M));
    FC_HIP(hipGetLastError());
    return FFTCONV_OK;
}

}  // namespace f3
}  // namespace fftconv
