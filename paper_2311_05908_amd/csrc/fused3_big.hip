// Fused causal FFT convolution for fft_size 32768 = 32*32*32 and 16384 = 32*16*32, 16-bit I/O (paper Algorithm 3:
// whole sequence on chip, u read once, y written once).  Same arithmetic and index maps as the
// smaller fused kernels (fused3.hip): time n = (n1*N2 + n2)*32 + n3, frequency
// f = k1 + 32*k2 + 32*N2*k3, two batch rows of a channel share one complex transform, the zero half
// of the padded input is never touched.
//
// What this size changes:
//  * The exchange buffer X(k1,k2,n3) of one pair is 128 KiB of 16-bit (re, im) pairs: it is the only
//    thing in LDS.  u and y are staged through it while it is free (between the last read of one
//    pair and the first write of the next), so HBM sees 16-byte chunks in memory order; the input
//    of the next pair waits in registers until then.
//  * The per-plane constant tables (stage-2 matrices with folded twiddles, elementwise twiddles,
//    k_f) do not fit in registers: they are streamed from L2, each one plane ahead of its use.
//    Twiddles and k_f are 16-bit (re, im) constants, 4 bytes per point (fp16: packed arithmetic,
//    op_sel / neg modifiers do the complex product; bf16: dot-product form, the swapped pair is
//    derived in registers).  The load path of a compute unit moves about 64 bytes per clock
//    whether a line comes from L1 or L2, and streaming these tables is the largest single cost
//    of the kernel, so table bytes count for more than a few vector instructions.
//  * The inverse innermost stage reuses the forward stage-3 matrix: the pointwise product writes
//    conj(A3 * k_f), the (symmetric) forward matrix then yields the conjugate of the inverse
//    transform, and the following twiddle product conjugates back.  Both conjugations are free
//    (instruction modifiers), and 32 registers of matrix are saved.
//  * Schedule per pair, 5 workgroup barriers: [phase B] | [phase C into registers] | [y and the next
//    u into the staging areas] | [staging into registers] | [phase A of the next pair, store y].
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "fused3_common.h"
#include "lds_fft.h"

namespace fftconv {
namespace f3 {

namespace {

// fft_size = 32 * N2 * 32 with N2 = 32 (32768) or 16 (16384)
template <int N2> struct BigGeo {
    static constexpr int M = 1024 * N2;
    static constexpr int R2 = N2 / 16;                    // 16-wide tiles of the middle digit
    static constexpr int PK1 = N2 + 4;                    // X(k1,k2,n3) word = n3*PN3 + k1*PK1 + k2
    // 4 words off a multiple of 32; short rather than long for the smaller size (the last k1 row
    // needs no padding), which brings two workgroups' buffers under the 160 KB of a compute unit
    static constexpr int PN3 = 32 * PK1 + (N2 == 16 ? -4 : 4);
    static constexpr int XB_WORDS = 32 * PN3;
    static constexpr size_t LDS_BYTES = (size_t)XB_WORDS * 4;
    static constexpr int NCH = M / 4096;                  // 16-byte chunks of a pair's input per thread
    static constexpr size_t U4 = (size_t)(4 + 4 + 8 + 2 * 32 * R2 * R2 * 2) * 64;   // operand tables, uint4 entries
    // byte offsets of the tables inside the constant block (layouts: see BigConsts)
    static constexpr int OFF_TAB1 = 0, OFF_TAB1I = 4 * 1024, OFF_TAB3 = 8 * 1024, OFF_TAB2 = 16 * 1024;
    static constexpr int PLANE2 = R2 * R2 * 2 * 1024;     // bytes of one plane's stage-2 matrix
    static constexpr int OFF_TAB2I = OFF_TAB2 + 32 * PLANE2;
    static constexpr int OFF_TWA = OFF_TAB2I + 32 * PLANE2;
    static constexpr int PLANEW = R2 * 2 * 4 * 256;       // bytes of one plane's twiddles (and k_f)
    static constexpr int OFF_TWB = OFF_TWA + 32 * PLANEW;
    static constexpr int CONST_BYTES = OFF_TWB + 32 * PLANEW;
    static_assert((size_t)OFF_TWA == U4 * 16 && 32 * PLANEW == M * 4, "table layout");
};

// Order of the innermost digit (n3 in time, k3 in frequency; 32 values) inside phase B: slot
// m = 16 tile + 4 q + r of a stage-3 operand or result holds digit sigma(m).  Tile 0 holds the
// 16 digits nearest zero on the circle ({0..7} and {24..31}), tile 1 the rest.  k3 is the most
// significant digit of the natural frequency, so a filter whose spectrum is confined to low
// |f| (Appendix A.4: sparsity in the first dimension of k_f) leaves tile 1 of k3 empty, and the
// HALF3 kernels skip its matrix products, its k_f and its share of the inverse contraction.
// The same order on both digits keeps the stage-3 matrix symmetric (see the conjugation trick
// above); on the n3 side it only changes which LDS rows a lane addresses.
__host__ __device__ inline int big_sigma(int m)
{
    const int t = m / 16, q = (m % 16) / 4, r = m % 4;
    const int base = t == 0 ? (q < 2 ? 4 * q : 16 + 4 * q) : 8 + 4 * q;
    return base + r;
}
__host__ __device__ inline int big_sigma_inv(int d)
{
    if (d < 8) return d;
    if (d >= 24) return d - 16;
    return 16 + (d - 8);
}
// Order of the middle frequency digit k2: slot m (16 tile + position in the tile) of a stage-2 result, of the
// exchange buffer, of k_f and of the twiddle tables holds digit big_tau<N2>(m).  With 32 values (fft 32768) it is
// the order above, so that the low-pass set of the digit -- the values nearest the two ends of its range, see
// fftconv_filter_fft_sparse_digits -- falls into tile 0 and the HALF2 kernels can leave tile 1 out: its stage-2
// rows, its columns of stage 3 and of the inverse stage 3, its share of the inverse stage-2 contraction, its k_f
// and twiddles (Appendix A.4: sparsity in the second dimension of k_f).  With 16 values there is one tile.
template <int N2> __host__ __device__ inline int big_tau(int m) { return N2 == 32 ? big_sigma(m) : m; }

// The constant block of a plan, one allocation (byte offsets in BigGeo):
//   tab1   [ct][part][lane] uint4                  W_32^{n1 k1}, n1 < 16
//   tab1i  [K step][part][lane]                    conj(W_32^{k1 n1}), n1 < 16
//   tab3   [K step][tile][part][lane]              W_32^{n3 k3}, both digits in the order big_sigma()
//   tab2   [n3][K step][tile][part][lane]          W_N2^{n2 k2} W_{32 N2}^{k2 n3}, k2 in the order big_tau()
//   tab2i  [k1][K step][tile][part][lane]          conj(W_N2^{k2 n2} W_{32 N2}^{k1 n2}), likewise
//   twa    [n3][rt][ct][r][lane] 4-byte constants  W_M^{k1 (32 n2 + n3)}
//   twb    [k1][ct2][ct3][r][lane]                 W_M^{(k1 + 32 k2) n3}, used as conj(z * w)
// The kernel reads it, and k_f, through buffer descriptors: a load is then "descriptor + scalar
// byte offset + lane offset + immediate", and the scalar offset of a plane is one SALU add.  With
// plain pointers every 4 KB piece of a table needed a 64-bit base of its own; the compiler
// computed those bases ahead of the loop and, out of scalar registers, parked them in vector
// lanes, which cost a fifth of the kernel's vector instructions at N2 = 32.

// nothing may be moved across: pins where the streamed table loads are issued
#define SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

// FULL: B even and N == fft_size / 2, every access of a work item is in range.
// SP (frequency-sparse filters, Appendix A.4), a set of bits:
//   1 (HALF3): k_f is zero wherever k3 is in tile 1 of the order big_sigma();
//   2 (HALF2, N2 = 32): k_f is zero wherever k2 is in tile 1 of the order big_tau();
//   4 (SKIP1): bit k1 of live_k1 clear = k_f is zero on the whole plane k1: phase B writes zeros for it and
//      neither loads its tables nor computes (the trip count of the per-plane loop).
// GATED (gated form y = v . ((u . w) * k), Section 3.1 / 4.1): wg multiplies u as its chunks go into the
// staging area, vg multiplies y as its chunks leave it (either may be null); the gates are fetched with the
// next pair's input, right after phase B.  One workgroup per compute unit then (the extra chunks need registers).
template <typename TT, bool FULL, int N2, int SP, bool GATED = false>
__global__ void __launch_bounds__(NT, (N2 == 16 && !GATED) ? 4 : 2) k_fused3_big(const uint16_t *__restrict__ u, uint16_t *__restrict__ y,
                                                  const void *__restrict__ kf, const void *__restrict__ consts,
                                                  uint32_t kf_bytes, int B, int H, int N,
                                                  const uint16_t *__restrict__ wg, const uint16_t *__restrict__ vg,
                                                  uint32_t live_k1, LaunchGate gate)
{
    using CW = typename TT::CW;
    using BG = BigGeo<N2>;
    constexpr int BPK1 = BG::PK1, BPN3 = BG::PN3, R2 = BG::R2, NCH = BG::NCH;
    constexpr bool HALF3 = (SP & 1) != 0, HALF2 = (SP & 2) != 0, SKIP1 = (SP & 4) != 0;
    static_assert(!HALF2 || N2 == 32, "the middle digit has a second tile only at N2 = 32");
    constexpr int T3 = HALF3 ? 1 : 2;                             // live k3 tiles
    constexpr int T2 = HALF2 ? 1 : R2;                            // live k2 tiles
    extern __shared__ uint32_t XB[];
    if (gate_closed(gate)) return;
    const int tid = threadIdx.x, l = tid & 63, q = l >> 4, c16 = l & 15;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    // Persistent workgroup; a work item t = h * npairs + pair.  Workgroups are dealt to the 8
    // accelerator dies (each with its own L2) round-robin, so die x = blockIdx % 8 takes the
    // channels h = x mod 8 and its workgroups walk through them side by side: at any time the
    // workgroups of a die share a few channels, whose k_f then stays in that die's L2.
    const int npairs = (B + 1) / 2;
    const int nx = gridDim.x % 8 == 0 ? 8 : 1;                    // dies the grid is spread over
    const int x = blockIdx.x % nx, nb = gridDim.x / nx, jb = blockIdx.x / nx;
    const int n_local = ((H - x + nx - 1) / nx) * npairs;         // work items of this die
    if (jb >= n_local) return;
    auto item = [&](int v) { return ((v / npairs) * nx + x) * npairs + v % npairs; };
    const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};

    // LDS base addresses of this lane, chosen so that every access below is base + a small constant
    uint32_t *const wrA = XB + 4 * w * BPN3 + c16 * BPK1 + 4 * q;         // + i*BPN3 + 16 ct*BPK1 + 16 ct2
    const uint32_t *const rdC = XB + 4 * w * BPN3 + 4 * q * BPK1 + c16;   // + i*BPN3 + (16 ks + r)*BPK1 + 16 cn2
    // phase B: wave w owns the planes k1 = w + 8 i, i < 4 (interleaved, so that a low-pass set of k1 -- its values
    // nearest zero on the circle -- spreads over all waves when dead planes are skipped); it addresses n3 in the
    // order big_sigma(): slots 4q .. 4q+3 of a tile are adjacent rows
    const uint32_t *const rdB0 = XB + big_sigma(4 * q) * BPN3 + w * BPK1 + c16;       // + r*BPN3 + 8 i*BPK1 + 16 ct2
    const uint32_t *const rdB1 = XB + big_sigma(16 + 4 * q) * BPN3 + w * BPK1 + c16;  // K step 1
    uint32_t *const wrB0 = XB + big_sigma(c16) * BPN3 + w * BPK1 + 4 * q;             // + 8 i*BPK1 + 16 cn2
    uint32_t *const wrB1 = XB + big_sigma(16 + c16) * BPN3 + w * BPK1 + 4 * q;        // n3 tile 1

    uint4 tab1[2][2], tab1i[2][2], tab3[2][2][2];
    // streamed per-plane tables, PD planes in flight (plane i lives in slot i % PD): the smaller transform
    // has short planes and spare registers, so it requests two planes ahead
    constexpr int PD = 1;
    uint4 tabA[PD][R2][R2][2], tabB[PD][R2][R2][2];      // stage-2 / inverse stage-2 matrices
    CW twaR[PD][R2][2][4], twbR[PD][R2][2][4], kfR[PD][R2][2][4];
    uint4 pre[NCH];                               // next pair's input, 16-byte chunks in memory order
    uint4 prew[GATED ? NCH : 1], prev[GATED ? NCH : 1];   // its input gate; the output gate of the current pair
    uint2 x1r[2][R2][4];                          // the same in operand order: [row of the pair][n2 tile][r], 4 n3 planes each

    // The tables are loop invariant but must be re-read for every work item (they do not fit in
    // registers): opaque zeros added to the lane offset and to the scalar offset keep the loads,
    // and the arithmetic of their offsets, inside the loop.
    const __amdgpu_buffer_rsrc_t rc = __builtin_amdgcn_make_buffer_rsrc((void *)consts, 0, BG::CONST_BYTES, 0x00020000);
    const __amdgpu_buffer_rsrc_t rk = __builtin_amdgcn_make_buffer_rsrc((void *)kf, 0, (int)kf_bytes, 0x00020000);
    int vo4 = 4 * l, vo16 = 16 * l, sz = 0;       // lane offsets of 4- and 16-byte entries; scalar zero
    auto opaque = [&]() {
        int z = 0;
        asm volatile("" : "+v"(z));
        vo4 = 4 * l + z;
        vo16 = 16 * l + z;
        asm volatile("s_mov_b32 %0, 0" : "=s"(sz));
    };
    // entry `ofs` (bytes, compile-time) of the piece that starts at scalar byte offset `base`
    auto ld16 = [&](const __amdgpu_buffer_rsrc_t &r, int base, int ofs) {
        typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, vo16 + (ofs & 4095), base + (ofs & ~4095), 0);
        return make_uint4(v.x, v.y, v.z, v.w);
    };
    auto ld4 = [&](const __amdgpu_buffer_rsrc_t &r, int base, int ofs) {
        return (CW)__builtin_amdgcn_raw_buffer_load_b32(r, vo4 + (ofs & 4095), base + (ofs & ~4095), 0);
    };
    auto load_fixed_outer = [&]() {
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                tab1[a][p] = ld16(rc, sz, BG::OFF_TAB1 + (a * 2 + p) * 1024);
                tab1i[a][p] = ld16(rc, sz, BG::OFF_TAB1I + (a * 2 + p) * 1024);
            }
    };
    auto load_tab3 = [&]() {
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int p = 0; p < 2; ++p) tab3[a][b][p] = ld16(rc, sz, BG::OFF_TAB3 + ((a * 2 + b) * 2 + p) * 1024);
    };
    auto load_tabA = [&](int i) {
        const int c = 4 * w + i, sl = i % PD;
        const int base = sz + c * BG::PLANE2;
#pragma unroll
        for (int a = 0; a < R2; ++a)
#pragma unroll
            for (int b = 0; b < T2; ++b) tabA[sl][a][b][0] = ld16(rc, base, BG::OFF_TAB2 + ((a * R2 + b) * 2 + 0) * 1024);
    };
    auto load_twa = [&](int i) {
        const int c = 4 * w + i, sl = i % PD;
        const int base = sz + c * BG::PLANEW;
#pragma unroll
        for (int a = 0; a < R2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 4; ++r) twaR[sl][a][b][r] = ld4(rc, base, BG::OFF_TWA + ((a * 2 + b) * 4 + r) * 256);
    };
    auto load_tabB = [&](int i) {
        const int c = w + 8 * i, sl = i % PD;
        const int base = sz + c * BG::PLANE2;
#pragma unroll
        for (int a = 0; a < T2; ++a)
#pragma unroll
            for (int b = 0; b < R2; ++b) tabB[sl][a][b][0] = ld16(rc, base, BG::OFF_TAB2I + ((a * R2 + b) * 2 + 0) * 1024);
    };
    auto load_twb = [&](int i) {
        const int c = w + 8 * i, sl = i % PD;
        const int base = sz + c * BG::PLANEW;
#pragma unroll
        for (int a = 0; a < T2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 4; ++r) twbR[sl][a][b][r] = ld4(rc, base, BG::OFF_TWB + ((a * 2 + b) * 4 + r) * 256);
    };
    auto load_kf = [&](int i, int h) {
        const int c = w + 8 * i, sl = i % PD;
        const int base = sz + (h * 32 + c) * BG::PLANEW;
#pragma unroll
        for (int a = 0; a < T2; ++a)
#pragma unroll
            for (int b = 0; b < T3; ++b)
#pragma unroll
                for (int r = 0; r < 4; ++r) kfR[sl][a][b][r] = ld4(rk, base, ((a * 2 + b) * 4 + r) * 256);
    };
    // Input and output pass through LDS so that HBM sees whole 16-byte chunks in memory order
    // (8-byte pieces of a 64-byte row written by 8 different waves cost partial-line fills and
    // write-backs).  Between phase C and phase A the exchange buffer is free: its bytes
    // [0, SB_BYTES) stage y of this pair, [SB_BYTES, 2 SB_BYTES) stage u of the next one, both as
    // (row of the pair, n1 < 16, n2) rows of 32 n3 values, 72 bytes apart (conflict-free 8-byte
    // accesses in operand order, 8-byte aligned 16-byte chunks in memory order).
    constexpr int SB_ROW = 72, SB_BYTES = 2 * 16 * N2 * SB_ROW;
    static_assert(2 * SB_BYTES <= (int)BG::LDS_BYTES, "staging areas must fit in the exchange buffer");
    char *const YS = (char *)XB, *const US = (char *)XB + SB_BYTES;
    // chunk j of this thread: row of the pair j / (NCH/2), elements [8 (tid + 512 (j % (NCH/2))), +8)
    auto issue_pre = [&](int t) {
        const int h = t / npairs, pair = t - h * npairs;
#pragma unroll
        for (int j = 0; j < NCH; ++j) {
            const int s = j / (NCH / 2);                      // wave-uniform: NCH/2 chunks per thread and row
            const int n = (tid + NT * (j % (NCH / 2))) * 8;
            const int b = 2 * pair + s;
            const uint16_t *row = u + ((size_t)(FULL ? b : min(b, B - 1)) * H + h) * N;
            const bool ok = FULL || (b < B && n < N);
            if constexpr (FULL) {
                pre[j] = *(const uint4 *)(row + n);
            } else {
                uint4 v = make_uint4(0, 0, 0, 0);
                if (ok) v = *(const uint4 *)(row + n);
                pre[j] = v;
            }
            if constexpr (GATED) {
                // a missing gate is read from u instead and never multiplied in: the load then needs no branch
                // (behind one, every gate chunk was waited for before the next load went out)
                const uint16_t *wsrc = wg ? wg : u;
                if constexpr (FULL) {
                    prew[j] = *(const uint4 *)(wsrc + (row - u) + n);
                } else {
                    uint4 g = make_uint4(0, 0, 0, 0);
                    if (ok) g = *(const uint4 *)(wsrc + (row - u) + n);
                    prew[j] = g;
                }
            }
        }
    };
    // output gate of pair t (the pair whose y is stored at the end of this iteration)
    auto issue_gate_v = [&](int t) {
        if constexpr (GATED) {
            const int h = t / npairs, pair = t - h * npairs;
#pragma unroll
            for (int j = 0; j < NCH; ++j) {
                const int s = j / (NCH / 2);
                const int n = (tid + NT * (j % (NCH / 2))) * 8;
                const int b = 2 * pair + s;
                const uint16_t *vsrc = vg ? vg : u;               // see the input gate
                if constexpr (FULL) {
                    prev[j] = *(const uint4 *)(vsrc + ((size_t)b * H + h) * N + n);
                } else {
                    uint4 g = make_uint4(0, 0, 0, 0);
                    if (b < B && n < N) g = *(const uint4 *)(vsrc + ((size_t)b * H + h) * N + n);
                    prev[j] = g;
                }
            }
        }
    };
    // byte offset of chunk j inside a staging area
    auto chunk_ofs = [&](int j) {
        const int s = j / (NCH / 2);
        const int n = (tid + NT * (j % (NCH / 2))) * 8;       // n = (n1*N2 + n2)*32 + n3, n3 in {0, 8, 16, 24}
        return (s * 16 * N2 + n / 32) * SB_ROW + (n % 32) * 2;
    };
    // byte offset of this lane's operand-order piece: n1 = 4q + r, n2 = 16 tile + c16, n3 = 4w .. 4w+3
    auto piece_ofs = [&](int s, int tile, int r) {
        return ((s * 16 + 4 * q + r) * N2 + 16 * tile + c16) * SB_ROW + 8 * w;
    };
    auto stage_in = [&]() {                                   // pre -> US
#pragma unroll
        for (int j = 0; j < NCH; ++j) {
            uint2 *dst = (uint2 *)(US + chunk_ofs(j));
            uint4 v = pre[j];
            if constexpr (GATED) {
                if (wg) v = TT::mul8(v, prew[j]);
            }
            dst[0] = make_uint2(v.x, v.y);
            dst[1] = make_uint2(v.z, v.w);
        }
    };
    auto read_x1 = [&]() {                                    // US -> operand order
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int rt = 0; rt < R2; ++rt)
#pragma unroll
                for (int r = 0; r < 4; ++r) x1r[s][rt][r] = *(const uint2 *)(US + piece_ofs(s, rt, r));
    };

    // ---- phase A of one pair: stage 1, twiddle, stage 2 -> XB (this wave's 4 n3 planes).
    // On entry tab1, tabA and twaR hold plane 0's tables; the others follow one plane ahead.
    auto phase_A = [&]() {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t sel = (i & 1) ? 0x07060302u : 0x05040100u;
            uint4 x2[2][R2];                              // stage-2 operands [k1 tile][K step = n2 tile]
#pragma unroll
            for (int rt = 0; rt < R2; ++rt) {
                // rows n2 = 16 rt + c16; slots (2r+s) = u_s[n1 = 4q + r]
                uint32_t d[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const uint32_t lo = i < 2 ? x1r[0][rt][r].x : x1r[0][rt][r].y;
                    const uint32_t hi = i < 2 ? x1r[1][rt][r].x : x1r[1][rt][r].y;
                    d[r] = __builtin_amdgcn_perm(hi, lo, sel);
                }
                const uint4 x1 = make_uint4(d[0], d[1], d[2], d[3]);
#pragma unroll
                for (int ct = 0; ct < 2; ++ct) {
                    const f32x4 dre = TT::mfma(x1, tab1[ct][0], zero4);
                    const f32x4 dim = TT::mfma(x1, tab1[ct][1], zero4);
                    // lane: k1 = 16 ct + c16; reg r: n2 = 16 rt + 4q + r
                    x2[ct][rt] = TT::template ctw4<false>(dre, dim, twaR[i % PD][rt][ct]);
                }
            }
            SCHED_FENCE();
            if (i + PD < 4) load_twa(i + PD);
            SCHED_FENCE();
            // Of the streamed per-plane matrices only the operand of the real part is fetched; the operand of the
            // imaginary part holds the same numbers in another arrangement and is made from it here: one or two vector
            // operations per word instead of four more bytes per lane through the load path, which is the kernel's
            // scarcest resource.
#pragma unroll
            for (int ks = 0; ks < R2; ++ks)
#pragma unroll
                for (int ct2 = 0; ct2 < T2; ++ct2) tabA[i % PD][ks][ct2][1] = TT::imag_operand(tabA[i % PD][ks][ct2][0]);
#pragma unroll
            for (int ct = 0; ct < 2; ++ct)
#pragma unroll
                for (int ct2 = 0; ct2 < T2; ++ct2) {      // (a dead k2 tile is neither computed nor written: nobody reads it)
                    f32x4 dre = zero4, dim = zero4;
#pragma unroll
                    for (int ks = 0; ks < R2; ++ks) {     // matrix as the A operand: rows k2, data columns k1
                        dre = TT::mfma(tabA[i % PD][ks][ct2][0], x2[ct][ks], dre);
                        dim = TT::mfma(tabA[i % PD][ks][ct2][1], x2[ct][ks], dim);
                    }
                    // lane: k1 = 16 ct + c16; reg r: k2 = 16 ct2 + 4q + r -> one 16-byte write
                    uint32_t *dst = wrA + i * BPN3 + 16 * ct * BPK1 + 16 * ct2;
                    *(uint4 *)dst = make_uint4(TT::pack(dre[0], dim[0]), TT::pack(dre[1], dim[1]),
                                               TT::pack(dre[2], dim[2]), TT::pack(dre[3], dim[3]));
                }
            SCHED_FENCE();
            if (i + PD < 4) load_tabA(i + PD);
            SCHED_FENCE();
        }
    };

    // ---- phase C of one pair: inverse stage 1 (n1 < 16) on this wave's 4 n3 planes; the results
    // (real part -> row b, imaginary part -> row b+1) are returned packed, 4 planes per 8 bytes.
    uint2 yo[2][R2][4];                                   // [row of the pair][n2 tile][r]
    auto phase_C = [&]() {
        // one n2 tile of one plane: lane: n2 = 16 cn2 + c16; reg r: n1 = 4q + r
        auto tile = [&](int i, int cn2, f32x4 &dre, f32x4 &dim) {
            const uint32_t *src = rdC + i * BPN3 + 16 * cn2;
            dre = zero4;
            dim = zero4;
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const uint32_t *s2 = src + 16 * ks * BPK1;
                const uint4 x = make_uint4(s2[0], s2[BPK1], s2[2 * BPK1], s2[3 * BPK1]);
                dre = TT::mfma(tab1i[ks][0], x, dre);
                dim = TT::mfma(tab1i[ks][1], x, dim);
            }
        };
#pragma unroll
        for (int ip = 0; ip < 2; ++ip)
#pragma unroll
            for (int cn2 = 0; cn2 < R2; ++cn2) {
                f32x4 are, aim, bre, bim;
                SCHED_FENCE();
                tile(2 * ip, cn2, are, aim);
                tile(2 * ip + 1, cn2, bre, bim);
                // the two planes are adjacent n3 -> one word
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const uint32_t wre = TT::pack(are[r], bre[r]);
                    const uint32_t wim = TT::pack(aim[r], bim[r]);
                    if (ip == 0) {
                        yo[0][cn2][r].x = wre;
                        yo[1][cn2][r].x = wim;
                    } else {
                        yo[0][cn2][r].y = wre;
                        yo[1][cn2][r].y = wim;
                    }
                }
                SCHED_FENCE();
            }
    };
    uint4 yc[NCH];                                        // y of this pair, 16-byte chunks in memory order
    auto stage_out = [&]() {                              // yo -> YS
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int cn2 = 0; cn2 < R2; ++cn2)
#pragma unroll
                for (int r = 0; r < 4; ++r) *(uint2 *)(YS + piece_ofs(s, cn2, r)) = yo[s][cn2][r];
    };
    auto read_y = [&]() {                                 // YS -> memory order
#pragma unroll
        for (int j = 0; j < NCH; ++j) {
            const uint2 *src = (const uint2 *)(YS + chunk_ofs(j));
            const uint2 a = src[0], b = src[1];
            yc[j] = make_uint4(a.x, a.y, b.x, b.y);
        }
    };
    auto store_y = [&](int t) {
        const int h = t / npairs, pair = t - h * npairs;
#pragma unroll
        for (int j = 0; j < NCH; ++j) {
            const int s = j / (NCH / 2);
            const int n = (tid + NT * (j % (NCH / 2))) * 8;
            const int b = 2 * pair + s;
            uint16_t *row = y + ((size_t)(FULL ? b : min(b, B - 1)) * H + h) * N;
            uint4 v = yc[j];
            if constexpr (GATED) {
                if (vg) v = TT::mul8(v, prev[j]);
            }
            if (FULL || (b < B && n < N)) *(uint4 *)(row + n) = v;
        }
    };

    // ---- phase B of one pair: per k1 plane (4 per wave: k1 = w + 8 i): stage 3, k_f, inverse 3, twiddle,
    // inverse 2, in place.  On entry tab3 and, if plane 0 is live, kfR, twbR, tabB of plane 0 are loaded.
    auto plane_live = [&](int i) { return !SKIP1 || ((live_k1 >> (w + 8 * i)) & 1u) != 0; };      // wave-uniform
    auto phase_B = [&](int h) {
        auto read_plane = [&](int i, uint4 (&x)[R2][2]) {
#pragma unroll
            for (int ct2 = 0; ct2 < T2; ++ct2)
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) {
                    const uint32_t *src = (ks ? rdB1 : rdB0) + 8 * i * BPK1 + 16 * ct2;
                    x[ct2][ks] = make_uint4(src[0], src[BPN3], src[2 * BPN3], src[3 * BPN3]);
                }
        };
        uint4 x3[R2][2];                                  // [k2 tile][K step = n3 tile]
        if (plane_live(0)) read_plane(0, x3);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const bool next = i + PD < 4 && plane_live(i + PD);
            if (!plane_live(i)) {
                // k_f is zero on this plane: so is the plane's result; the next live plane's tables are requested here
#pragma unroll
                for (int cn3 = 0; cn3 < 2; ++cn3)
#pragma unroll
                    for (int cn2 = 0; cn2 < R2; ++cn2)
                        *(uint4 *)((cn3 ? wrB1 : wrB0) + 8 * i * BPK1 + 16 * cn2) = make_uint4(0, 0, 0, 0);
                if (next) {
                    load_kf(i + PD, h);
                    load_twb(i + PD);
                    load_tabB(i + PD);
                    read_plane(i + 1, x3);
                }
                continue;
            }
            uint4 x3i[R2][2];                             // [k2 tile][K step = k3 tile], holds conj(A3 k_f)
#pragma unroll
            for (int ct2 = 0; ct2 < T2; ++ct2)
#pragma unroll
                for (int ct3 = 0; ct3 < T3; ++ct3) {
                    f32x4 dre = zero4, dim = zero4;
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks) {      // matrix is the A operand: rows k3, data columns k2
                        dre = TT::mfma(tab3[ks][ct3][0], x3[ct2][ks], dre);
                        dim = TT::mfma(tab3[ks][ct3][1], x3[ct2][ks], dim);
                    }
                    // lane: k2 = big_tau(16 ct2 + c16); reg r: k3 = big_sigma(16 ct3 + 4q + r)
                    x3i[ct2][ct3] = TT::template ctw4<true>(dre, dim, kfR[i % PD][ct2][ct3]);
                }
            SCHED_FENCE();
            if (next) load_kf(i + PD, h);
            if (i + 1 < 4 && plane_live(i + 1)) read_plane(i + 1, x3);   // its latency hides behind the rest of this plane
            SCHED_FENCE();
            uint4 x2i[2][R2];                             // [n3 tile][K step = k2 tile]
#pragma unroll
            for (int ct2 = 0; ct2 < T2; ++ct2)
#pragma unroll
                for (int cn3 = 0; cn3 < 2; ++cn3) {
                    f32x4 dre = zero4, dim = zero4;
#pragma unroll
                    for (int ks = 0; ks < T3; ++ks) {     // data rows k2, the forward matrix as the B operand
                        dre = TT::mfma(x3i[ct2][ks], tab3[ks][cn3][0], dre);
                        dim = TT::mfma(x3i[ct2][ks], tab3[ks][cn3][1], dim);
                    }
                    // = conj of the inverse transform.  lane: n3 = big_sigma(16 cn3 + c16); reg r: k2 = big_tau(16 ct2 + 4q + r)
                    x2i[cn3][ct2] = TT::template ctw4<true>(dre, dim, twbR[i % PD][ct2][cn3]);
                }
            SCHED_FENCE();
            if (next) load_twb(i + PD);
            SCHED_FENCE();
#pragma unroll
            for (int ks = 0; ks < T2; ++ks)                // (see phase A)
#pragma unroll
                for (int cn2 = 0; cn2 < R2; ++cn2) tabB[i % PD][ks][cn2][1] = TT::imag_operand(tabB[i % PD][ks][cn2][0]);
#pragma unroll
            for (int cn3 = 0; cn3 < 2; ++cn3)
#pragma unroll
                for (int cn2 = 0; cn2 < R2; ++cn2) {
                    f32x4 dre = zero4, dim = zero4;
#pragma unroll
                    for (int ks = 0; ks < T2; ++ks) {     // matrix as the A operand: rows n2, data columns n3; K = live k2 tiles
                        dre = TT::mfma(tabB[i % PD][ks][cn2][0], x2i[cn3][ks], dre);
                        dim = TT::mfma(tabB[i % PD][ks][cn2][1], x2i[cn3][ks], dim);
                    }
                    // lane: n3 = 16 cn3 + c16; reg r: n2 = 16 cn2 + 4q + r -> one 16-byte write
                    uint32_t *dst = (cn3 ? wrB1 : wrB0) + 8 * i * BPK1 + 16 * cn2;
                    *(uint4 *)dst = make_uint4(TT::pack(dre[0], dim[0]), TT::pack(dre[1], dim[1]),
                                               TT::pack(dre[2], dim[2]), TT::pack(dre[3], dim[3]));
                }
            SCHED_FENCE();
            if (next) load_tabB(i + PD);
            SCHED_FENCE();
        }
    };
    // tables of the first plane of phase B for channel h (nothing if that plane is dead)
    auto load_plane0 = [&](int h) {
#pragma unroll
        for (int i = 0; i < PD; ++i)
            if (plane_live(i)) {
                load_kf(i, h);
                load_twb(i);
                load_tabB(i);
            }
    };

    // The matrices that do not depend on the plane (stage 1, its inverse, stage 3: 64 registers) stay in registers for
    // the whole launch where the kernel has them to spare; otherwise each set is fetched again before the phase
    // that uses it.
    constexpr bool RESIDENT = FULL && !GATED && N2 == 32 && SP == 0;
    // ---- prologue: phase A of the first pair
    opaque();
    issue_pre(item(jb));
    load_fixed_outer();
#pragma unroll
    for (int i = 0; i < PD; ++i) {
        load_tabA(i);
        load_twa(i);
    }
    stage_in();
    lds_barrier();
    read_x1();
    lds_barrier();
    phase_A();
    SCHED_FENCE();
    load_tab3();
    load_plane0(item(jb) / npairs);
    SCHED_FENCE();
    lds_barrier();

    vmem_settled();                                     // nothing of the prologue is still in flight inside the loop
    // Per pair, 5 workgroup barriers:
    //   [B(t)] | [C(t) -> registers] | [y(t), u(t+1) -> staging] | [staging -> registers] | [A(t+1); store y(t)] |
    for (int v = jb; v < n_local; v += nb) {
        opaque();
        // Past the end of the range the last pair is prepared once more (in range, never used):
        // the loop body stays free of branches.
        const int t = item(v), tn = v + nb < n_local ? item(v + nb) : t;
        phase_B(t / npairs);
        SCHED_FENCE();
        // tables of the next phase and the next pair's input: in flight across the barrier and phase C
        if constexpr (!RESIDENT) load_fixed_outer();
#pragma unroll
        for (int i = 0; i < PD; ++i) {
            load_tabA(i);
            load_twa(i);
        }
        issue_pre(tn);
        issue_gate_v(t);
        SCHED_FENCE();
        lds_barrier();
        phase_C();
        lds_barrier();                                  // every wave has read its planes: the buffer is free
        stage_out();
        stage_in();
        lds_barrier();
        read_y();
        read_x1();
        lds_barrier();                                  // staging consumed: phase A may overwrite it
        phase_A();
        SCHED_FENCE();
        if constexpr (!RESIDENT) load_tab3();
        load_plane0(tn / npairs);
        SCHED_FENCE();
        // the stores go last: loads and stores retire through one counter on this target, and
        // nothing issued after them is waited for before the next barrier
        store_y(t);
        lds_barrier();
    }
}

// ---- Filter gradient for fft 16384 and 32768 (Section 3.1 "Kernel Fusion and Recomputation"; see fused3_dk.hip
// for the arithmetic: dk_f[h] = sum over the pairs of conj(FFT(u pair)) . FFT(dy pair), cross terms of the pair
// packing end up in the dropped imaginary part of the inverse transform).  The forward half of the kernel above
// (staging, phase A, stage 3 of phase B; same tables and layouts) runs on the stream u-pair, dy-pair, u-pair, ...
// of the channels a workgroup owns: a u input leaves its spectrum in registers (fp32), the dy input that
// follows multiplies it in and adds to the channel's accumulator (fp32), which is written out in the kernel's
// k_f order after the channel's last pair.  Spectrum and accumulator of a whole transform are 2 x 64 registers
// at N2 = 16 and would be 2 x 128 at N2 = 32, where the kernel therefore walks through a channel's pairs twice,
// each time keeping one k3 tile of the bins (phase A is repeated, stage 3 is not) with the spectrum of u held as
// 16-bit pairs (32 registers; the accumulator stays fp32).  One workgroup per compute unit.
template <typename TT, bool FULL, int N2>
__global__ void __launch_bounds__(NT, 2) k_fused3_big_dk(const uint16_t *__restrict__ u, const uint16_t *__restrict__ dy,
                                                         float2 *__restrict__ dkf, const void *__restrict__ consts, int B,
                                                         int H, int N)
{
    using CW = typename TT::CW;
    using BG = BigGeo<N2>;
    constexpr int BPK1 = BG::PK1, BPN3 = BG::PN3, NCH = BG::NCH, R2 = BG::R2;
    // Passes over a channel and (k2, k3) tiles of a k1 plane kept per pass.  N2 = 16: both k3 tiles of the only k2
    // tile.  N2 = 32: the pass's k3 tile of both k2 tiles, with the spectrum of u held as 16-bit pairs.
    constexpr int NPASS = R2, TPP = 2;
    constexpr bool PACKZ = N2 == 32;
    extern __shared__ uint32_t XB[];
    const int tid = threadIdx.x, l = tid & 63, q = l >> 4, c16 = l & 15;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int npairs = (B + 1) / 2;
    const int nch = (H - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x;      // channels h = blockIdx.x + j gridDim.x
    const int S = nch * NPASS * npairs * 2;                // inputs: ((j * NPASS + pass) * npairs + pair) * 2 + (0 = u, 1 = dy)
    if (S <= 0) return;
    const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};

    uint32_t *const wrA = XB + 4 * w * BPN3 + c16 * BPK1 + 4 * q;
    const uint32_t *const rdB0 = XB + big_sigma(4 * q) * BPN3 + 4 * w * BPK1 + c16;
    const uint32_t *const rdB1 = XB + big_sigma(16 + 4 * q) * BPN3 + 4 * w * BPK1 + c16;
    constexpr int SB_ROW = 72, SB_BYTES = 2 * 16 * N2 * SB_ROW;
    static_assert(2 * SB_BYTES <= (int)BG::LDS_BYTES, "the staging area must fit in the exchange buffer");
    char *const US = (char *)XB + SB_BYTES;

    const __amdgpu_buffer_rsrc_t rc = __builtin_amdgcn_make_buffer_rsrc((void *)consts, 0, BG::CONST_BYTES, 0x00020000);
    int vo4 = 4 * l, vo16 = 16 * l, sz = 0;
    auto opaque = [&]() {
        int z = 0;
        asm volatile("" : "+v"(z));
        vo4 = 4 * l + z;
        vo16 = 16 * l + z;
        asm volatile("s_mov_b32 %0, 0" : "=s"(sz));
    };
    auto ld16 = [&](int base, int ofs) {
        typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rc, vo16 + (ofs & 4095), base + (ofs & ~4095), 0);
        return make_uint4(v.x, v.y, v.z, v.w);
    };
    auto ld4 = [&](int base, int ofs) {
        return (CW)__builtin_amdgcn_raw_buffer_load_b32(rc, vo4 + (ofs & 4095), base + (ofs & ~4095), 0);
    };
    // resident: stage-1 matrix, the stage-3 tiles of the current pass; streamed one plane ahead: stage-2
    // matrix and twiddles of a plane
    constexpr int T3R = PACKZ ? 1 : 2;                    // resident k3 tiles of the stage-3 matrix
    uint4 tab1[2][2], tab3[2][T3R][2], tabA[R2][R2][2];
    CW twaR[R2][2][4];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int p = 0; p < 2; ++p) tab1[a][p] = ld16(0, BG::OFF_TAB1 + (a * 2 + p) * 1024);
    auto load_tab3 = [&](int ct3) {                        // tiles ct3 .. ct3 + T3R - 1
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < T3R; ++b)
#pragma unroll
                for (int p = 0; p < 2; ++p)
                    tab3[a][b][p] = ld16(sz + ct3 * 2048, BG::OFF_TAB3 + ((a * 2 + b) * 2 + p) * 1024);
    };
    auto load_plane = [&](int i) {
        const int c = 4 * w + i;
#pragma unroll
        for (int a = 0; a < R2; ++a)
#pragma unroll
            for (int b = 0; b < R2; ++b)               // the operand of the real part only (see k_fused3_big)
                tabA[a][b][0] = ld16(sz + c * BG::PLANE2, BG::OFF_TAB2 + ((a * R2 + b) * 2 + 0) * 1024);
#pragma unroll
        for (int a = 0; a < R2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 4; ++r) twaR[a][b][r] = ld4(sz + c * BG::PLANEW, BG::OFF_TWA + ((a * 2 + b) * 4 + r) * 256);
    };

    uint4 pre[NCH];
    uint2 x1r[2][R2][4];
    auto issue_pre = [&](int s, int c0, int c1) {         // chunks c0 .. c1 - 1
        const int item = s >> 1, which = s & 1;
        const int jp = item / npairs, pair = item - jp * npairs;
        const int h = (int)blockIdx.x + (jp / NPASS) * (int)gridDim.x;
        const uint16_t *src = which ? dy : u;
#pragma unroll
        for (int c = c0; c < c1; ++c) {
            const int row = c / (NCH / 2);
            const int n = (tid + NT * (c % (NCH / 2))) * 8;
            const int b = 2 * pair + row;
            if constexpr (FULL) {
                pre[c] = *(const uint4 *)(src + ((size_t)b * H + h) * N + n);
            } else {
                uint4 v = make_uint4(0, 0, 0, 0);
                if (b < B && n < N) v = *(const uint4 *)(src + ((size_t)b * H + h) * N + n);
                pre[c] = v;
            }
        }
    };
    auto chunk_ofs = [&](int c) {
        const int row = c / (NCH / 2);
        const int n = (tid + NT * (c % (NCH / 2))) * 8;
        return (row * 16 * N2 + n / 32) * SB_ROW + (n % 32) * 2;
    };
    auto stage_in = [&]() {
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            uint2 *dst = (uint2 *)(US + chunk_ofs(c));
            dst[0] = make_uint2(pre[c].x, pre[c].y);
            dst[1] = make_uint2(pre[c].z, pre[c].w);
        }
    };
    auto read_x1 = [&]() {
#pragma unroll
        for (int row = 0; row < 2; ++row)
#pragma unroll
            for (int rt = 0; rt < R2; ++rt)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    x1r[row][rt][r] = *(const uint2 *)(US + ((row * 16 + 4 * q + r) * N2 + 16 * rt + c16) * SB_ROW + 8 * w);
    };
    auto phase_A = [&]() {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t sel = (i & 1) ? 0x07060302u : 0x05040100u;
            uint4 x2[2][R2];
#pragma unroll
            for (int rt = 0; rt < R2; ++rt) {
                uint32_t d[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const uint32_t lo = i < 2 ? x1r[0][rt][r].x : x1r[0][rt][r].y;
                    const uint32_t hi = i < 2 ? x1r[1][rt][r].x : x1r[1][rt][r].y;
                    d[r] = __builtin_amdgcn_perm(hi, lo, sel);
                }
                const uint4 x1 = make_uint4(d[0], d[1], d[2], d[3]);
#pragma unroll
                for (int ct = 0; ct < 2; ++ct) {
                    const f32x4 dre = TT::mfma(x1, tab1[ct][0], zero4);
                    const f32x4 dim = TT::mfma(x1, tab1[ct][1], zero4);
                    x2[ct][rt] = TT::template ctw4<false>(dre, dim, twaR[rt][ct]);
                }
            }
            uint4 o[2][R2];
#pragma unroll
            for (int ks = 0; ks < R2; ++ks)
#pragma unroll
                for (int ct2 = 0; ct2 < R2; ++ct2) tabA[ks][ct2][1] = TT::imag_operand(tabA[ks][ct2][0]);
#pragma unroll
            for (int ct = 0; ct < 2; ++ct)
#pragma unroll
                for (int ct2 = 0; ct2 < R2; ++ct2) {
                    f32x4 dre = zero4, dim = zero4;
#pragma unroll
                    for (int ks = 0; ks < R2; ++ks) {
                        dre = TT::mfma(tabA[ks][ct2][0], x2[ct][ks], dre);
                        dim = TT::mfma(tabA[ks][ct2][1], x2[ct][ks], dim);
                    }
                    o[ct][ct2] = make_uint4(TT::pack(dre[0], dim[0]), TT::pack(dre[1], dim[1]), TT::pack(dre[2], dim[2]),
                                            TT::pack(dre[3], dim[3]));
                }
            SCHED_FENCE();
            if (i + 1 < 4) load_plane(i + 1);             // this plane's tables have been consumed
            SCHED_FENCE();
#pragma unroll
            for (int ct = 0; ct < 2; ++ct)
#pragma unroll
                for (int ct2 = 0; ct2 < R2; ++ct2) *(uint4 *)(wrA + i * BPN3 + 16 * ct * BPK1 + 16 * ct2) = o[ct][ct2];
        }
    };

    // [k1 plane of the wave][tile of the pass]
    f32x4 z1re[4][2], z1im[4][2], accre[4][2], accim[4][2];
    uint4 z1p[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int t = 0; t < TPP; ++t) {
            accre[i][t] = accim[i][t] = z1re[i][t] = z1im[i][t] = zero4;
            z1p[i][t] = make_uint4(0, 0, 0, 0);
        }

    opaque();
    issue_pre(0, 0, NCH);
    if constexpr (!PACKZ) load_tab3(0);                   // one pass: the stage-3 matrices stay in registers
    for (int s = 0; s < S; ++s) {
        const int item = s >> 1, which = s & 1;
        const int jp = item / npairs, pair = item - jp * npairs;
        const int j = jp / NPASS, pass = jp - j * NPASS;
        stage_in();
        lds_barrier();
        read_x1();
        lds_barrier();                                    // staging consumed: phase A may overwrite it
        opaque();
        load_plane(0);
        // the next input (past the end: the last one again, in range and unused) is requested ahead of
        // phase A where registers allow, after it otherwise
        constexpr int EARLY = PACKZ ? 0 : NCH;
        issue_pre(s + 1 < S ? s + 1 : s, 0, EARLY);
        SCHED_FENCE();
        phase_A();
        SCHED_FENCE();
        // Two passes: the pass's stage-3 matrices take the place of phase A's tables, in every step and ahead of
        // the input loads.  (Loaded only in a pass's first step they sat behind a condition; the compiler then has to
        // take them as possibly in flight in every step, and as they came after the input loads, the wait before
        // stage 3 waited for the whole next input as well.)
        if constexpr (PACKZ) load_tab3(pass);
        SCHED_FENCE();
        issue_pre(s + 1 < S ? s + 1 : s, EARLY, NCH);
        lds_barrier();
        // stage 3 of this wave's 4 k1 planes
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            uint4 x3[2];                                  // the plane's k2 tile: one for both k3 tiles at N2 = 16
#pragma unroll
            for (int t = 0; t < TPP; ++t) {
                const int ct2 = PACKZ ? t : 0;
                if (PACKZ || t == 0) {
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks) {
                        const uint32_t *src = (ks ? rdB1 : rdB0) + i * BPK1 + 16 * ct2;
                        x3[ks] = make_uint4(src[0], src[BPN3], src[2 * BPN3], src[3 * BPN3]);
                    }
                }
                f32x4 dre = zero4, dim = zero4;
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) {
                    dre = TT::mfma(tab3[ks][PACKZ ? 0 : t][0], x3[ks], dre);
                    dim = TT::mfma(tab3[ks][PACKZ ? 0 : t][1], x3[ks], dim);
                }
                if (which == 0) {                         // wave-uniform
                    if constexpr (PACKZ) {
                        z1p[i][t] = make_uint4(TT::pack(dre[0], dim[0]), TT::pack(dre[1], dim[1]), TT::pack(dre[2], dim[2]),
                                               TT::pack(dre[3], dim[3]));
                    } else {
                        z1re[i][t] = dre;
                        z1im[i][t] = dim;
                    }
                } else {                                  // acc += conj(Z1) . Z2
                    f32x4 zr, zi;
                    if constexpr (PACKZ) {
                        const float2 a0 = TT::widen(z1p[i][t].x), a1 = TT::widen(z1p[i][t].y), a2 = TT::widen(z1p[i][t].z),
                                     a3 = TT::widen(z1p[i][t].w);
                        zr = f32x4{a0.x, a1.x, a2.x, a3.x};
                        zi = f32x4{a0.y, a1.y, a2.y, a3.y};
                    } else {
                        zr = z1re[i][t];
                        zi = z1im[i][t];
                    }
                    accre[i][t] += zr * dre + zi * dim;
                    accim[i][t] += zr * dim - zi * dre;
                }
            }
        }
        if (which == 1 && pair == npairs - 1) {           // the pass's last pair: write its accumulator, start anew
            const int h = (int)blockIdx.x + j * (int)gridDim.x;
            float2 *dst = dkf + (size_t)h * BG::M;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int t = 0; t < TPP; ++t) {
                    const int ct2 = PACKZ ? t : 0, ct3 = PACKZ ? pass : t;
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        dst[((((4 * w + i) * R2 + ct2) * 2 + ct3) * 4 + r) * 64 + l] = make_float2(accre[i][t][r], accim[i][t][r]);
                    accre[i][t] = zero4;
                    accim[i][t] = zero4;
                }
        }
        lds_barrier();                                    // every wave has read its planes: the buffer is free
    }
}

// dk_f of the kernel above ([h][k1][k2 tile][k3 tile][r][lane], lane = (k3 slot / 4 % 4) * 16 + k2 % 16, k3 in the
// order big_sigma()) -> dk, in two kernels.  The inverse transform runs the factors of the generic path
// (16, 16, 16, M / 4096) last to first; all but the first act inside contiguous blocks of M / 16 positions, and
// block d0 (the low four bits of k1) is made of the bins of k1 = d0 and d0 + 16: two contiguous runs of dk_f.
// Kernel 1, one workgroup per (channel, block): the two runs -> LDS at their positions, the length-M/16
// inverse there (twiddle table of W_M with stride 16), natural order out to a scratch row.  Kernel 2: the
// remaining factor across the 16 blocks, real part, 1/M, the first Nk samples.
constexpr int DK_BLK_THREADS = 256;
template <int N2>
__global__ void __launch_bounds__(DK_BLK_THREADS) k_big_dk_blocks(const float2 *__restrict__ dkf, float2 *__restrict__ tmp,
                                                                 const float2 *__restrict__ w, FacList fl, FacList fl_tail)
{
    constexpr int BM = BigGeo<N2>::M, BLK = BM / 16, RUN = BLK / 2, R2 = BigGeo<N2>::R2;
    __shared__ float2 XS[BLK + BLK / 16];
    const int d0 = blockIdx.x;
    const int64_t h = blockIdx.y;
#pragma unroll
    for (int i = threadIdx.x; i < BLK; i += DK_BLK_THREADS) {
        const int k1 = d0 + 16 * (i / RUN), j = i % RUN;                       // slot (k1, j) of dk_f[h]
        const int lane = j % 64, r = (j / 64) % 4, t3 = (j / 256) % 2, t2 = (j / 512) % R2;
        const int k2 = big_tau<N2>(16 * t2 + lane % 16), k3 = big_sigma(16 * t3 + 4 * (lane / 16) + r);
        const int f = k1 + 32 * k2 + 32 * N2 * k3;
        XS[lds_slot(lds_pos(f, fl, BM) - d0 * BLK)] = dkf[h * BM + k1 * RUN + j];
    }
    __syncthreads();
    lds_inverse(XS, w, fl_tail, BLK, 16);
    for (int i = threadIdx.x; i < BLK; i += DK_BLK_THREADS) tmp[h * BM + d0 * BLK + i] = XS[lds_slot(i)];
}

template <int N2>
__global__ void k_big_dk_last(const float2 *__restrict__ tmp, float *__restrict__ dk, const float2 *__restrict__ w,
                              int64_t H, int64_t Nk)
{
    constexpr int BM = BigGeo<N2>::M, BLK = BM / 16;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= H * BLK) return;
    const int64_t h = idx / BLK;
    const int r = (int)(idx % BLK);
    if (r >= Nk) return;
    float2 x[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) x[k] = cmul_conj(tmp[h * BM + k * BLK + r], w[k * r]);
    dft_reg<16, true>(x);
#pragma unroll
    for (int n = 0; n < 16; ++n)
        if (n * BLK + r < Nk) dk[h * Nk + n * BLK + r] = x[n].x * (1.0f / (float)BM);
}

// Filter transform, one workgroup per channel and nothing but the taps and k_f in HBM.  The taps are real, so
// the row is transformed as M/2 complex points z[n] = k[2n] + i k[2n+1] in LDS (fp32, the stages of lds_fft.h;
// 16384 complex points are what LDS holds), and the two interleaved half-length spectra are separated on the way
// out: with Z = FFT(z), E = (Z[f] + conj Z[M/2 - f]) / 2 and O = (Z[f] - conj Z[M/2 - f]) / (2i) are the spectra
// of the even and odd taps, K[f] = E + W_M^f O for f < M/2, K[M/2] = Re Z[0] - Im Z[0], K[M - f] = conj K[f].
// k_f in the kernel's per-lane order: [h][k1][k2 tile][k3 tile][r][lane]; the lane holds
// k2 = big_tau(16 tile + lane%16) and k3 = big_sigma(16 tile + 4 (lane/16) + r).  Scaled by 1/M.
// w: W_M^t, t < M.  flh: factors of the half-length transform.  conj_out: the adjoint filter transform.
constexpr int BIG_FILT_THREADS = 1024;
template <typename TT, int N2>
__global__ void __launch_bounds__(BIG_FILT_THREADS) k_filter_big(const float *__restrict__ k, typename TT::CW *__restrict__ kf,
                                                                const float2 *__restrict__ w, FacList flh, int64_t Nk,
                                                                bool conj_out, const uint8_t *__restrict__ keep,
                                                                int64_t n_blocks)
{
    extern __shared__ float2 ZF[];
    constexpr int BM = BigGeo<N2>::M, MH = BM / 2, R2 = BigGeo<N2>::R2;
    const int64_t h = blockIdx.x;
    const float *row = k + h * Nk;
    // all taps of the thread are requested before the first is used (a tap beyond Nk reads tap 0 and is discarded:
    // behind a branch every load would be waited for in turn)
    constexpr int TPT = MH / BIG_FILT_THREADS;
    float ta[TPT], tb[TPT];
#pragma unroll
    for (int j = 0; j < TPT; ++j) {
        const int n = threadIdx.x + j * BIG_FILT_THREADS;
        ta[j] = row[2 * n < Nk ? 2 * n : 0];
        tb[j] = row[2 * n + 1 < Nk ? 2 * n + 1 : 0];
    }
#pragma unroll
    for (int j = 0; j < TPT; ++j) asm volatile("" ::"v"(ta[j]), "v"(tb[j]));
#pragma unroll
    for (int j = 0; j < TPT; ++j) {
        const int n = threadIdx.x + j * BIG_FILT_THREADS;
        ZF[lds_slot(n)] = make_float2(2 * n < Nk ? ta[j] : 0.f, 2 * n + 1 < Nk ? tb[j] : 0.f);
    }
    __syncthreads();
    lds_forward(ZF, w, flh, MH, 2);
    // (straight-line body, four entries per trip: the twiddle gathers of a trip are then in flight together)
#pragma unroll 4
    for (int d = threadIdx.x; d < BM; d += BIG_FILT_THREADS) {
        const int lane = d % 64, r = (d / 64) % 4, t3 = (d / 256) % 2, t2 = (d / 512) % R2, k1 = d / (512 * R2);
        const int k2 = big_tau<N2>(16 * t2 + lane % 16), k3 = big_sigma(16 * t3 + 4 * (lane / 16) + r);
        const int f = k1 + 32 * k2 + 32 * N2 * k3;
        const int fe = f <= MH ? f : BM - f;              // K[f] = conj K[M - f]
        const bool nyq = fe == MH;                        // the bin M/2: Z[0].re - Z[0].im
        const int fa = nyq ? 0 : fe;
        const float2 tw = w[fa];
        const float2 za = ZF[lds_slot(lds_pos(fa, flh, MH))];
        const float2 zc = ZF[lds_slot(lds_pos((MH - fa) % MH, flh, MH))];
        const float2 e = make_float2(0.5f * (za.x + zc.x), 0.5f * (za.y - zc.y));
        const float2 o = make_float2(0.5f * (za.y + zc.y), -0.5f * (za.x - zc.x));      // (za - conj zc) / (2i)
        float2 v = cmul(o, tw);
        v.x += e.x;
        v.y += e.y;
        if (nyq) v = make_float2(za.x - za.y, 0.f);
        if ((f > MH) != conj_out) v.y = -v.y;
        const float sc = lds_mask_weight(keep, n_blocks, f, BM) / (float)BM;
        const uint32_t pr = TT::pack(v.x * sc, v.y * sc);                       // (re, im) 16-bit pair
        kf[h * BM + d] = TT::cconst(pr & 0xffffu, pr >> 16, true);              // the kernel forms conj(A3 * k_f)
    }
}

// ---------------------------------------------------------------- host side

uint16_t h_bf16(double x)
{
    float f = (float)x;
    uint32_t b;
    std::memcpy(&b, &f, 4);
    b += 0x7fffu + ((b >> 16) & 1u);          // round to nearest even (finite inputs only)
    return (uint16_t)(b >> 16);
}
uint16_t h_f16(double x)
{
    _Float16 hv = (_Float16)(float)x;
    uint16_t b;
    std::memcpy(&b, &hv, 2);
    return b;
}
struct Cx { double re, im; };
Cx wp(int64_t M, int64_t e)                   // exp(-2 pi i e / M)
{
    const double two_pi = 6.283185307179586476925286766559;
    e %= M;
    if (e < 0) e += M;
    const double a = two_pi * (double)e / (double)M;
    return {std::cos(a), -std::sin(a)};
}
Cx cm(Cx a, Cx b) { return {a.re * b.re - a.im * b.im, a.re * b.im + a.im * b.re}; }
Cx cj(Cx a) { return {a.re, -a.im}; }

// One MFMA operand (64 lanes x 8 16-bit slots) of the real form of a complex matrix G: lane
// (c16, q), slot 2r+s multiplies data element e_in = 16 t + 4 q + r, part s (0 = re, 1 = im), and
// contributes to output element e_out = 16 ct + c16, part `part`.
template <typename Fn> void fill_op(uint16_t *dst, bool f16, int t, int ct, int part, Fn G)
{
    for (int lane = 0; lane < 64; ++lane) {
        const int c16 = lane % 16, q = lane / 16;
        for (int r = 0; r < 4; ++r) {
            const Cx g = G(16 * t + 4 * q + r, 16 * ct + c16);
            const double v0 = part == 0 ? g.re : g.im;
            const double v1 = part == 0 ? -g.im : g.re;
            dst[lane * 8 + 2 * r + 0] = f16 ? h_f16(v0) : h_bf16(v0);
            dst[lane * 8 + 2 * r + 1] = f16 ? h_f16(v1) : h_bf16(v1);
        }
    }
}

template <typename TT, bool FULL, int N2, int SP, bool GATED = false>
int launch_big(const fftconv_plan *p, const void *u, const void *kf, void *y, int64_t B, hipStream_t s,
               const void *wg = nullptr, const void *vg = nullptr, uint32_t live_k1 = 0xffffffffu)
{
    using BG = BigGeo<N2>;
    auto kern = k_fused3_big<TT, FULL, N2, SP, GATED>;
    FC_TRY(raise_dynamic_lds((const void *)kern, (int)BG::LDS_BYTES));
    const int64_t T = p->H * ((B + 1) / 2);
    const int64_t kf_bytes = p->H * BG::M * 4;
    if (kf_bytes >= ((int64_t)1 << 31)) {
        set_error("fftconv_forward: H * fft_size = %lld exceeds the fused kernel's k_f addressing (2^29 bins)",
                  (long long)(p->H * BG::M));
        return FFTCONV_EUNSUPPORTED;
    }
    if (T >= ((int64_t)1 << 31) - 8) {
        set_error("fftconv_forward: H * ceil(B/2) = %lld work items exceed the fused kernel's limit", (long long)T);
        return FFTCONV_EUNSUPPORTED;
    }
    // persistent workgroups, as many as are resident at once (two per compute unit for the smaller
    // size: 80 KB of LDS and 128 registers each), a multiple of 8 (see the kernel's work split)
    const int64_t resident = (int64_t)p->f3.num_cu * ((N2 == 16 && !GATED) ? 2 : 1);
    int grid = (int)(T < resident ? T : resident);
    if (grid >= 8) grid -= grid % 8;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(NT), BG::LDS_BYTES, s, (const uint16_t *)u, (uint16_t *)y,
                       kf, (const void *)p->f3.consts, (uint32_t)kf_bytes, (int)B, (int)p->H, (int)p->N,
                       (const uint16_t *)wg, (const uint16_t *)vg, live_k1, launch_gate());
    FC_HIP(hipGetLastError());
    return FFTCONV_OK;
}

template <int N2> int big_init_t(fftconv_plan *p)
{
    using BG = BigGeo<N2>;
    constexpr int R2 = BG::R2;
    const bool f16 = p->dtype == FFTCONV_F16;
    const int64_t M = BG::M;
    std::vector<uint16_t> ops(BG::U4 * 8);
    size_t o = 0;
    auto next = [&]() { uint16_t *d = ops.data() + o * 8; o += 64; return d; };
    for (int ct = 0; ct < 2; ++ct)                        // tab1: K step 0 only (n1 < 16)
        for (int part = 0; part < 2; ++part)
            fill_op(next(), f16, 0, ct, part, [&](int n1, int k1) { return wp(32, (int64_t)n1 * k1); });
    for (int ks = 0; ks < 2; ++ks)                        // tab1i: row tile 0 only (n1 < 16)
        for (int part = 0; part < 2; ++part)
            fill_op(next(), f16, ks, 0, part, [&](int k1, int n1) { return cj(wp(32, (int64_t)n1 * k1)); });
    for (int ks = 0; ks < 2; ++ks)                        // tab3 (forward; also serves the inverse, see the kernel)
        for (int ct = 0; ct < 2; ++ct)
            for (int part = 0; part < 2; ++part)
                fill_op(next(), f16, ks, ct, part,
                        [&](int m3, int j3) { return wp(32, (int64_t)big_sigma(m3) * big_sigma(j3)); });   // slots, both digits
    for (int n3 = 0; n3 < 32; ++n3)                       // tab2
        for (int ks = 0; ks < R2; ++ks)
            for (int ct = 0; ct < R2; ++ct)
                for (int part = 0; part < 2; ++part)
                    fill_op(next(), f16, ks, ct, part, [&](int n2, int m2) {       // row slot m2 holds digit k2
                        const int k2 = big_tau<N2>(m2);
                        return cm(wp(N2, (int64_t)n2 * k2), wp(32 * N2, (int64_t)k2 * n3));
                    });
    for (int k1 = 0; k1 < 32; ++k1)                       // tab2i
        for (int ks = 0; ks < R2; ++ks)
            for (int ct = 0; ct < R2; ++ct)
                for (int part = 0; part < 2; ++part)
                    fill_op(next(), f16, ks, ct, part, [&](int m2, int n2) {       // contraction slot m2 holds digit k2
                        const int k2 = big_tau<N2>(m2);
                        return cj(cm(wp(N2, (int64_t)n2 * k2), wp(32 * N2, (int64_t)k1 * n2)));
                    });
    if (o != BG::U4) {
        set_error("fused3 (32 x N2 x 32): operand table size mismatch");
        return FFTCONV_EINVAL;
    }
    // twiddles as 16-bit constants in the form TT::ctw4 expects
    std::vector<uint32_t> tw((size_t)2 * M);
    auto put = [&](size_t idx, Cx v, bool conj) {
        const uint32_t re = f16 ? h_f16(v.re) : h_bf16(v.re), im = f16 ? h_f16(v.im) : h_bf16(v.im);
        tw[idx] = f16 ? H16::cconst(re, im, conj) : B16::cconst(re, im, conj);
    };
    size_t e = 0;
    for (int n3 = 0; n3 < 32; ++n3)                       // twa: k1 = 16 ct + c16, n2 = 16 rt + 4 q + r
        for (int rt = 0; rt < R2; ++rt)
            for (int ct = 0; ct < 2; ++ct)
                for (int r = 0; r < 4; ++r)
                    for (int lane = 0; lane < 64; ++lane) {
                        const int k1 = 16 * ct + lane % 16, n2 = 16 * rt + 4 * (lane / 16) + r;
                        put(e++, wp(M, (int64_t)k1 * (32 * n2 + n3)), false);
                    }
    for (int k1 = 0; k1 < 32; ++k1)                       // twb: n3 = big_sigma(16 ct3 + c16), k2 = 16 ct2 + 4 q + r
        for (int ct2 = 0; ct2 < R2; ++ct2)
            for (int ct3 = 0; ct3 < 2; ++ct3)
                for (int r = 0; r < 4; ++r)
                    for (int lane = 0; lane < 64; ++lane) {
                        const int n3 = big_sigma(16 * ct3 + lane % 16), k2 = big_tau<N2>(16 * ct2 + 4 * (lane / 16) + r);
                        put(e++, wp(M, ((int64_t)k1 + 32 * (int64_t)k2) * n3), true);
                    }
    const size_t bytes = BG::U4 * 16 + tw.size() * 4;
    FC_HIP(hipMalloc(&p->f3.consts, bytes));
    p->f3.consts_bytes += bytes;
    FC_HIP(hipMemcpy(p->f3.consts, ops.data(), BG::U4 * 16, hipMemcpyHostToDevice));
    FC_HIP(hipMemcpy((char *)p->f3.consts + BG::U4 * 16, tw.data(), tw.size() * 4, hipMemcpyHostToDevice));
    return FFTCONV_OK;
}

template <typename TT, int N2>
int big_filter_tt(const fftconv_plan *p, const float *k, int64_t Nk, bool adjoint, const uint8_t *keep_dev, int64_t n_blocks,
                  void *kf, hipStream_t s)
{
    constexpr int64_t MH = BigGeo<N2>::M / 2;
    const size_t bytes = lds_row_bytes(MH, sizeof(float2));
    FC_TRY(raise_dynamic_lds((const void *)k_filter_big<TT, N2>, (int)bytes));
    hipLaunchKernelGGL((k_filter_big<TT, N2>), dim3((unsigned)p->H), dim3(BIG_FILT_THREADS), bytes, s, k,
                       (typename TT::CW *)kf, (const float2 *)p->st.w32, staged_factors_for(MH), Nk, adjoint, keep_dev,
                       n_blocks);
    FC_HIP(hipGetLastError());
    return FFTCONV_OK;
}

template <typename TT, int N2, int SP>
int big_forward_tt(const fftconv_plan *p, const void *u, const void *kf, void *y, int64_t B, uint32_t live_k1, hipStream_t s)
{
    const bool full = (B % 2 == 0) && p->N == BigGeo<N2>::M / 2;
    return full ? launch_big<TT, true, N2, SP>(p, u, kf, y, B, s, nullptr, nullptr, live_k1)
                : launch_big<TT, false, N2, SP>(p, u, kf, y, B, s, nullptr, nullptr, live_k1);
}

// sp: bit 0 = the k3 tile 1 is empty, bit 1 = the k2 tile 1 is empty (N2 = 32), bit 2 = some k1 planes are empty
template <typename TT, int N2>
int big_forward_sp(const fftconv_plan *p, const void *u, const void *kf, void *y, int64_t B, int sp, uint32_t live_k1,
                   hipStream_t s)
{
    switch (sp) {
    case 1: return big_forward_tt<TT, N2, 1>(p, u, kf, y, B, live_k1, s);
    case 4: return big_forward_tt<TT, N2, 4>(p, u, kf, y, B, live_k1, s);
    case 5: return big_forward_tt<TT, N2, 5>(p, u, kf, y, B, live_k1, s);
    default: break;
    }
    if constexpr (N2 == 32) {
        switch (sp) {
        case 2: return big_forward_tt<TT, N2, 2>(p, u, kf, y, B, live_k1, s);
        case 3: return big_forward_tt<TT, N2, 3>(p, u, kf, y, B, live_k1, s);
        case 6: return big_forward_tt<TT, N2, 6>(p, u, kf, y, B, live_k1, s);
        case 7: return big_forward_tt<TT, N2, 7>(p, u, kf, y, B, live_k1, s);
        default: break;
        }
    }
    return big_forward_tt<TT, N2, 0>(p, u, kf, y, B, live_k1, s);
}

}  // namespace

// fft_size 32768 = 32 * 32 * 32 and 16384 = 32 * 16 * 32
int fused3_big_init(fftconv_plan *p) { return p->M == 32768 ? big_init_t<32>(p) : big_init_t<16>(p); }

size_t fused3_big_kf_bytes(const fftconv_plan *p)
{
    return (size_t)(p->H * p->M) * sizeof(uint32_t);
}

int fused3_big_filter(const fftconv_plan *p, const float *k, int64_t Nk, bool adjoint, const uint8_t *keep_dev,
                      int64_t n_blocks, void *kf, hipStream_t s)
{
    const bool f16 = p->dtype == FFTCONV_F16;
    if (p->M == 32768)
        return f16 ? big_filter_tt<H16, 32>(p, k, Nk, adjoint, keep_dev, n_blocks, kf, s)
                   : big_filter_tt<B16, 32>(p, k, Nk, adjoint, keep_dev, n_blocks, kf, s);
    return f16 ? big_filter_tt<H16, 16>(p, k, Nk, adjoint, keep_dev, n_blocks, kf, s)
               : big_filter_tt<B16, 16>(p, k, Nk, adjoint, keep_dev, n_blocks, kf, s);
}

// live_k3, live_k2, live_k1: bit d set when the value d of that digit of the frequency f = k1 + 32 k2 + 32 N2 k3
// may meet a non-zero bin of k_f; all ones for a dense filter.
int fused3_big_forward(const fftconv_plan *p, const void *u, const void *kf, void *y, int64_t B, uint32_t live_k3,
                       hipStream_t s, uint32_t live_k2, uint32_t live_k1)
{
    if (((uintptr_t)u | (uintptr_t)y) & 15) {
        set_error("fftconv_forward: u and y must be 16-byte aligned for this plan");
        return FFTCONV_EINVAL;
    }
    int sp = 3;                                           // no live digit in tile 1 of the kernel's orders
    for (int d = 0; d < 32; ++d) {
        if (((live_k3 >> d) & 1u) && big_sigma_inv(d) >= 16) sp &= ~1;
        if (p->M != 32768 || (((live_k2 >> d) & 1u) && big_sigma_inv(d) >= 16)) sp &= ~2;
    }
    if (live_k1 != 0xffffffffu) sp |= 4;
    const bool f16 = p->dtype == FFTCONV_F16;
    if (p->M == 32768)
        return f16 ? big_forward_sp<H16, 32>(p, u, kf, y, B, sp, live_k1, s) : big_forward_sp<B16, 32>(p, u, kf, y, B, sp, live_k1, s);
    return f16 ? big_forward_sp<H16, 16>(p, u, kf, y, B, sp, live_k1, s) : big_forward_sp<B16, 16>(p, u, kf, y, B, sp, live_k1, s);
}

// Gated form: wg / vg (same shape and dtype as u; either may be null) are applied inside the kernel.
int fused3_big_forward_gated(const fftconv_plan *p, const void *u, const void *wg, const void *vg, const void *kf, void *y,
                             int64_t B, hipStream_t s)
{
    if (((uintptr_t)u | (uintptr_t)y | (uintptr_t)wg | (uintptr_t)vg) & 15) {
        set_error("fftconv_forward_gated: u, w, v and y must be 16-byte aligned for this plan");
        return FFTCONV_EINVAL;
    }
    const bool f16 = p->dtype == FFTCONV_F16;
    if (p->M == 32768) {
        const bool full = (B % 2 == 0) && p->N == BigGeo<32>::M / 2;
        if (f16)
            return full ? launch_big<H16, true, 32, 0, true>(p, u, kf, y, B, s, wg, vg)
                        : launch_big<H16, false, 32, 0, true>(p, u, kf, y, B, s, wg, vg);
        return full ? launch_big<B16, true, 32, 0, true>(p, u, kf, y, B, s, wg, vg)
                    : launch_big<B16, false, 32, 0, true>(p, u, kf, y, B, s, wg, vg);
    }
    const bool full = (B % 2 == 0) && p->N == BigGeo<16>::M / 2;
    if (f16)
        return full ? launch_big<H16, true, 16, 0, true>(p, u, kf, y, B, s, wg, vg)
                    : launch_big<H16, false, 16, 0, true>(p, u, kf, y, B, s, wg, vg);
    return full ? launch_big<B16, true, 16, 0, true>(p, u, kf, y, B, s, wg, vg)
                : launch_big<B16, false, 16, 0, true>(p, u, kf, y, B, s, wg, vg);
}

bool fused3_big_dk_supported(const fftconv_plan *p) { return p->path == PATH_FUSED3 && (p->M == 16384 || p->M == 32768); }

template <int N2>
static int big_dk_accumulate_t(const fftconv_plan *p, const void *u, const void *dy, void *dkf, int64_t B, hipStream_t s)
{
    using BG = BigGeo<N2>;
    const bool full = (B % 2 == 0) && p->N == BG::M / 2;
    const bool f16 = p->dtype == FFTCONV_F16;
    void (*kern)(const uint16_t *, const uint16_t *, float2 *, const void *, int, int, int) =
        f16 ? (full ? k_fused3_big_dk<H16, true, N2> : k_fused3_big_dk<H16, false, N2>)
            : (full ? k_fused3_big_dk<B16, true, N2> : k_fused3_big_dk<B16, false, N2>);
    FC_TRY(raise_dynamic_lds((const void *)kern, (int)BG::LDS_BYTES));
    const int grid = (int)(p->H < p->f3.num_cu ? p->H : p->f3.num_cu);
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(NT), BG::LDS_BYTES, s, (const uint16_t *)u, (const uint16_t *)dy,
                       (float2 *)dkf, (const void *)p->f3.consts, (int)B, (int)p->H, (int)p->N);
    FC_HIP(hipGetLastError());
    return FFTCONV_OK;
}

// dkf: H * fft_size float2 in the kernel's order
int fused3_big_dk_accumulate(const fftconv_plan *p, const void *u, const void *dy, void *dkf, int64_t B, hipStream_t s)
{
    if (((uintptr_t)u | (uintptr_t)dy) & 15) {
        set_error("fftconv_backward_filter: u and dy must be 16-byte aligned for this plan");
        return FFTCONV_EINVAL;
    }
    const int64_t npairs = (B + 1) / 2;
    if (p->H * npairs >= ((int64_t)1 << 27)) {
        set_error("fftconv_backward_filter: H * ceil(B/2) = %lld exceeds the fused kernel's limit",
                  (long long)(p->H * npairs));
        return FFTCONV_EUNSUPPORTED;
    }
    return p->M == 32768 ? big_dk_accumulate_t<32>(p, u, dy, dkf, B, s) : big_dk_accumulate_t<16>(p, u, dy, dkf, B, s);
}

template <int N2>
static int big_dk_finish_t(const fftconv_plan *p, const void *dkf, void *tmp, float *dk, int64_t Nk, hipStream_t s)
{
    constexpr int BLK = BigGeo<N2>::M / 16;
    const FacList fl = staged_fac_list(p);
    if (fl.nf < 2 || fl.fac[0] != 16) {
        set_error("fftconv_backward_filter: unexpected factor list for fft_size=%lld", (long long)p->M);
        return FFTCONV_EUNSUPPORTED;
    }
    FacList tail;
    tail.nf = fl.nf - 1;
    for (int i = 0; i < MAX_FACTORS; ++i) tail.fac[i] = i + 1 < fl.nf ? fl.fac[i + 1] : 0;
    hipLaunchKernelGGL(k_big_dk_blocks<N2>, dim3(16, (unsigned)p->H), dim3(DK_BLK_THREADS), 0, s, (const float2 *)dkf,
                       (float2 *)tmp, (const float2 *)p->st.w32, fl, tail);
    FC_HIP(hipGetLastError());
    const int bs = 256;
    hipLaunchKernelGGL(k_big_dk_last<N2>, dim3((unsigned)((p->H * BLK + bs - 1) / bs)), dim3(bs), 0, s, (const float2 *)tmp,
                       dk, (const float2 *)p->st.w32, p->H, Nk);
    FC_HIP(hipGetLastError());
    return FFTCONV_OK;
}

// dkf: the accumulated spectra of fused3_big_dk_accumulate; tmp: H * fft_size float2 of scratch
int fused3_big_dk_finish(const fftconv_plan *p, const void *dkf, void *tmp, float *dk, int64_t Nk, hipStream_t s)
{
    return p->M == 32768 ? big_dk_finish_t<32>(p, dkf, tmp, dk, Nk, s) : big_dk_finish_t<16>(p, dkf, tmp, dk, Nk, s);
}

}  // namespace f3
}  // namespace fftconv
