// Internal declarations shared by the translation units of libfftconv.so.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "fftconv.h"

namespace fftconv {

void set_error(const char *fmt, ...);

#define FC_HIP(call)                                                                      \
    do {                                                                                  \
        hipError_t e_ = (call);                                                           \
        if (e_ != hipSuccess) {                                                           \
            ::fftconv::set_error("%s failed: %s (%s:%d)", #call, hipGetErrorString(e_),   \
                                 __FILE__, __LINE__);                                     \
            return FFTCONV_EHIP;                                                          \
        }                                                                                 \
    } while (0)

#define FC_TRY(call)                     \
    do {                                 \
        const int rc_ = (call);          \
        if (rc_ != FFTCONV_OK) return rc_; \
    } while (0)

// Raise a kernel's dynamic-LDS limit to `bytes` on the current device, once per (device, kernel);
// safe to call from several threads and before every launch.
int raise_dynamic_lds(const void *kernel, int bytes);

// A launch gate: when tag is not null a kernel starts by reading *tag and returns at once unless
// (*tag == want) == run_if_equal.  fftconv_forward_partial launches both of its routes with opposite gates
// on the tag that the filter transform left behind the short spectrum, so the choice between them is made
// on the device, where the tag lives, without a host synchronisation.  The gate of the calling thread is
// empty except inside that entry point; every forward kernel takes it as its last argument.
struct LaunchGate {
    const long long *tag = nullptr;
    long long want = 0;
    int run_if_equal = 0;
};
LaunchGate &launch_gate();          // of the calling thread
__device__ __forceinline__ bool gate_closed(const LaunchGate &g)
{
    return g.tag != nullptr && ((*g.tag == g.want) != (g.run_if_equal != 0));
}

enum Path { PATH_STAGED = 0, PATH_FUSED3 = 1, PATH_MULTIPASS = 2, PATH_SMALL = 3 };

constexpr int MAX_FACTORS = 8;

// Factor list of the staged transform, passed to kernels by value.
struct FacList {
    int nf;
    int fac[MAX_FACTORS];
};

// Position, in the staged transform's output order, of natural frequency f:
// f = sum_i k_i R_i (k_1 least significant) sits at sum_i k_i S_i (k_1 most significant).
__host__ __device__ inline int64_t freq_to_pos(int64_t f, const FacList &fl, int64_t M)
{
    int64_t p = 0, S = M;
    for (int i = 0; i < fl.nf; ++i) {
        S /= fl.fac[i];
        p += (f % fl.fac[i]) * S;
        f /= fl.fac[i];
    }
    return p;
}

// Generic multi-kernel path: one launch per stage of the order-p decomposition,
// complex intermediates in a caller-provided workspace.  Used for fp32 I/O, for
// sizes without a fused kernel, and (in fp64) for every filter transform.
struct StagedTables {
    int nf = 0;
    int64_t fac[MAX_FACTORS] = {0};   // outermost (first contracted) first
    float2 *w32 = nullptr;            // W_M^t, t in [0,M), fp32 pairs
    double2 *w64 = nullptr;           // same in fp64 (filter transform)
};

// Fused single-kernel path for 16-bit I/O, fft_size = N1*N2*N3 (Algorithm 3).
struct Fused3Tables {
    int N1 = 0, N2 = 0, N3 = 0;
    int num_cu = 0;                   // compute units of the plan's device (persistent grid size)
    void *consts = nullptr;           // operand tables in the kernel's lane order
    size_t consts_bytes = 0;
    // fft 16384 plans also carry the 8192-point tables: a short (partial) filter runs as overlapping
    // 8192-point segments, and k_f then holds a second, 8192-point spectrum after the dense one
    void *consts_short = nullptr;
};

// fp16 plans of the multi-pass path (fft_size = No * 8192): 1 / fft_size itself is already a subnormal
// fp16 number from No = 8, so a filter of small norm (a unit tap: |K| = 1) would lose most of its bits in
// k_f.  Their k_f is therefore scaled by boost / fft_size with boost = min(No, 64), a power of two, and the
// outer inverse pass multiplies by 1 / boost in fp32.  bf16 has the exponent range of fp32: boost = 1.
__host__ __device__ constexpr int multipass_kf_boost(bool f16, int No) { return !f16 ? 1 : No < 64 ? No : 64; }

// Weight of frequency bin f under a block mask (Section 3.3, frequency-sparse filters).  The
// output is defined as Re(IDFT(mask . K . U)) for real u; that equals IDFT(K' . U) with the
// Hermitian part K'[f] = K[f] (mask[f] + mask[M-f]) / 2, and only a Hermitian K' (a real filter)
// lets two real sequences share one complex transform.  So a bin whose mirror is masked
// differently gets weight 1/2.  keep == nullptr means no mask.
__host__ __device__ inline double mask_weight(const uint8_t *keep, int64_t n_blocks, int64_t f, int64_t M)
{
    if (!keep) return 1.0;
    const int64_t per = M / n_blocks;
    const int64_t fm = f == 0 ? 0 : M - f;
    return 0.5 * ((keep[f / per] ? 1.0 : 0.0) + (keep[fm / per] ? 1.0 : 0.0));
}

}  // namespace fftconv

struct fftconv_plan {
    int64_t N = 0, M = 0, H = 0;
    int dtype = 0;
    int device = 0;
    fftconv::Path path = fftconv::PATH_STAGED;
    fftconv::StagedTables st;
    fftconv::Fused3Tables f3;
    // private scratch of the filter transform (two fp64 complex ping-pong buffers)
    double2 *filt_a = nullptr, *filt_b = nullptr;
    int64_t filt_chunk = 0;           // channels per pass through the scratch
    uint8_t *keep_dev = nullptr;      // device copy of a frequency-block mask (sparse filter transform)
    float2 *long_tw = nullptr;        // twiddle tables of the two-kernel long transforms (long_fft.hip)
};

namespace fftconv {

// ---- staged path (staged.hip)
int staged_init(fftconv_plan *p);
void staged_destroy(fftconv_plan *p);
size_t staged_kf_bytes(const fftconv_plan *p);
size_t staged_workspace_bytes(const fftconv_plan *p, int64_t B);
int staged_forward(const fftconv_plan *p, const void *u, const void *kf, void *y, int64_t B,
                   void *workspace, hipStream_t s);
// fp64 transform of zero-padded filters into p->filt_a for channels [h0, h0+nh):
// on return filt_a holds position-ordered spectra (position -> frequency via staged_pos_to_freq).
// adjoint: the spectrum of the circularly time-reversed filter (= the conjugate spectrum)
int staged_filter_transform(const fftconv_plan *p, const float *k, int64_t Nk, int64_t h0, int64_t nh,
                            hipStream_t s, double2 **result, bool adjoint = false);
// scatter of the fp64 spectra into the staged path's own k_f layout
int staged_pack_kf(const fftconv_plan *p, const double2 *spec, int64_t h0, int64_t nh,
                   const uint8_t *keep_dev, int64_t n_blocks, void *kf, hipStream_t s);
FacList staged_fac_list(const fftconv_plan *p);
FacList staged_factors_for(int64_t M);

// ---- fp32 transforms of long rows in two kernels per direction (long_fft.hip)
bool long_fft_supported(const fftconv_plan *p);
int long_fft_init(fftconv_plan *p);
void long_fft_destroy(fftconv_plan *p);
int long_filter_transform(const fftconv_plan *p, const float *k, int64_t Nk, int64_t h0, int64_t nh, bool adjoint,
                          const uint8_t *keep_dev, int64_t n_blocks, float2 *tmp, void *kf, hipStream_t s);
int long_filter_transform_f32(const fftconv_plan *p, const float *k, int64_t Nk, int64_t h0, int64_t nh, bool adjoint,
                          const uint8_t *keep_dev, int64_t n_blocks, float2 *tmp, void *kf, hipStream_t s);
FacList long_fft_factor_list(int64_t M);
size_t long_forward_workspace_bytes(const fftconv_plan *p);
int long_forward(const fftconv_plan *p, const void *u, const void *kf, void *y, int64_t B, void *workspace, hipStream_t s);
size_t long_backward_filter_bytes(const fftconv_plan *p);
int long_backward_filter(const fftconv_plan *p, const void *u, const void *dy, float *dk, int64_t Nk, int64_t B,
                         void *workspace, hipStream_t s);

// ---- fused 3-stage path (fused3.hip)
bool fused3_supported(int64_t N, int64_t M, int dtype);
int fused3_init(fftconv_plan *p);
void fused3_destroy(fftconv_plan *p);
size_t fused3_kf_bytes(const fftconv_plan *p);
int fused3_forward(const fftconv_plan *p, const void *u, const void *kf, void *y, int64_t B, hipStream_t s);
// frequency-sparse forward: live = number of accumulator registers (1..4) that can hold non-zero k_f
int fused3_forward_sparse(const fftconv_plan *p, const void *u, const void *kf, void *y, int64_t B, uint32_t live_k3,
                          hipStream_t s, uint32_t live_k1 = 0xffffffffu, uint32_t live_k2 = 0xffffffffu);
uint32_t fused3_live_k3(const fftconv_plan *p, const uint8_t *block_keep, int64_t n_blocks);
// partial convolution by overlapping short segments; returns FFTCONV_EUNSUPPORTED if this plan / Nk cannot
bool fused3_short_ok(const fftconv_plan *p, int64_t Nk);
int fused3_init_short(fftconv_plan *p);
size_t fused3_short_kf_bytes(const fftconv_plan *p);
int fused3_filter_short(const fftconv_plan *p, const float *k, int64_t Nk, void *kf, hipStream_t s);
// the tag behind the short spectrum: the Nk that spectrum was built for, 0 = none
const long long *fused3_short_tag(const fftconv_plan *p, const void *kf);
int fused3_set_short_tag(const fftconv_plan *p, void *kf, int64_t Nk, hipStream_t s);
// filter transform in one kernel, taps to k_f; adjoint: the conjugate spectrum
int fused3_filter(const fftconv_plan *p, const float *k, int64_t Nk, bool adjoint, const uint8_t *keep_dev,
                  int64_t n_blocks, void *kf, hipStream_t s);
int fused3_forward_short(const fftconv_plan *p, const void *u, const void *kf, void *y, int64_t B, int64_t Nk,
                         hipStream_t s);
// the 8192-point complex-row kernel used as the inner step of the multi-pass path
int fused3_init_inner(fftconv_plan *p);
int fused3_inner_rows(const fftconv_plan *p, void *rows, const void *kf, int64_t rows_per_kf, int64_t kf_rows,
                      hipStream_t s, int ko_n = 0, int ko_lo = 0, int ko_hi = 0, bool quarter_rows = false);
// the same kernel running the whole convolution of an 8192-point plan, u (B, H, N) -> y with N a multiple of 4
int fused3_inner_whole(const fftconv_plan *p, const void *u, const void *kf, void *y, int64_t B, hipStream_t s);
// Order of the innermost frequency digit k3 (N3 values) inside the fused kernels.  Stage 3 leaves
// k3 in an accumulator slot (tile t, lane group q, register r) = index 16 t + 4 q + r.  The digits are
// ranked by closeness to DC (0, N3-1, 1, N3-2, ...: k3 is the most significant digit of the
// natural frequency, so this is low |f| first) and rank j goes to q = j % 4, r = (j % 16) / 4:
// a low-pass frequency mask then leaves whole registers r zero in every lane, which the
// frequency-sparse kernels skip (Appendix A.4: sparsity in the first dimension of k_f).
__host__ __device__ inline int k3_at_index(int idx, int N3)
{
    const int t = idx / 16, i = idx % 16;
    const int j = 16 * t + (i / 4) + 4 * (i % 4);          // rank held by this slot
    return (j & 1) ? N3 - 1 - (j >> 1) : (j >> 1);
}
__host__ __device__ inline int k3_index(int k3, int N3)
{
    const int j = k3 < N3 / 2 ? 2 * k3 : 2 * (N3 - 1 - k3) + 1;
    const int t = j / 16, jj = j % 16;
    return 16 * t + 4 * (jj % 4) + jj / 4;
}

// Place of column r (< 8192) inside a row of the multi-pass workspace.  r = n1*256 + n2*16 + n3 in the inner
// kernel's digits.  Outer lengths up to 64 store a row as four quarter rows, one per group of four n3 planes -- the
// planes of one outer wave of the inner kernel (fused3_wsc.hip), which then reads and writes whole contiguous
// lines instead of a quarter of each:
//   slot = (n3 / 4) * 2048 + n1 * 64 + n2 * 4 + n3 % 4        (columns r and r + 1, r even, stay adjacent).
// A block of the outer passes holds 8192 / No consecutive columns: from 128 columns (No <= 64) up its share of a
// quarter row is still 128 bytes or more and the sweep gains 5-11 %; at No = 128 it makes no difference, and at 256
// (64- and 32-byte pieces) the outer passes lose more than the inner kernel gains (0.21 -> 0.175 ms against
// 0.095 -> 0.11 and 0.115 -> 0.15 ms on config 4).  Longer outer transforms keep the natural order.
constexpr bool multipass_quarter_rows(int No) { return No <= 64; }
__host__ __device__ inline int multipass_row_slot(int r, bool quarter)
{
    return quarter ? ((r & 12) << 9) | ((r >> 8) << 6) | (((r >> 4) & 15) << 2) | (r & 3) : r;
}

// slot of inner frequency fi (< 8192) in the 8192-point kernel's per-lane k_f order
__host__ __device__ inline int fused3_kf_slot_8192(int64_t fi)
{
    const int k1 = (int)(fi % 32), k2 = (int)((fi / 32) % 16), k3 = (int)(fi / 512);
    const int idx = k3_index(k3, 16);
    const int lane = (idx / 4) * 16 + k2, r = idx % 4;
    return (k1 * 4 + r) * 64 + lane;
}

// gated form y = v . ((u . w) * k): true when the plan's kernel applies the gates itself
bool fused3_gates_fused(const fftconv_plan *p);
int fused3_forward_gated(const fftconv_plan *p, const void *u, const void *w, const void *v, const void *kf, void *y,
                         int64_t B, hipStream_t s);
// out[i] = a[i] * b[i] rounded to the I/O dtype (staged.hip); out may alias a
int gate_multiply(int dtype, const void *a, const void *b, void *out, int64_t n, hipStream_t s);

// filter gradient dk[h,t] = sum_b sum_i dy[b,h,i] upad[b,h,(i-t) mod M], t < Nk, through the generic
// one-kernel-per-stage transforms in fp32 (staged.hip); any plan
size_t staged_backward_filter_bytes(const fftconv_plan *p);
int staged_backward_filter(const fftconv_plan *p, const void *u, const void *dy, float *dk, int64_t Nk, int64_t B,
                           void *workspace, hipStream_t s);

int staged_inverse_to_dk(const fftconv_plan *p, float2 *spec, float2 *other, int64_t nrows, float *dk, int64_t Nk,
                         hipStream_t s);
int64_t staged_backward_chunk(const fftconv_plan *p);
// fused filter gradient of the 8192-point plans (fused3_dk.hip)
namespace f3 {
bool fused3_dk_supported(const fftconv_plan *p);
int fused3_dk_accumulate(const fftconv_plan *p, const void *u, const void *dy, void *dkf, int64_t B, hipStream_t s);
int fused3_dk_finish(const fftconv_plan *p, const void *dkf, float *dk, int64_t Nk, hipStream_t s);
// the same for fft 16384 plans (fused3_big.hip); dkf = H * 16384 float2
bool fused3_big_dk_supported(const fftconv_plan *p);
int fused3_big_dk_accumulate(const fftconv_plan *p, const void *u, const void *dy, void *dkf, int64_t B, hipStream_t s);
int fused3_big_dk_finish(const fftconv_plan *p, const void *dkf, void *tmp, float *dk, int64_t Nk, hipStream_t s);
}  // namespace f3

// ---- short transforms, fft_size 256 .. 4096, any dtype (small.hip); radices reported in f3.N1..N3
bool small_supported(int64_t N, int64_t M, int dtype);
FacList small_factor_list(int64_t M);      // its radices, outermost first
int small_init(fftconv_plan *p);
size_t small_kf_bytes(const fftconv_plan *p);
int small_pack_kf(const fftconv_plan *p, const double2 *spec, int64_t h0, int64_t nh, const uint8_t *keep_dev,
                  int64_t n_blocks, void *kf, hipStream_t s);
int small_forward(const fftconv_plan *p, const void *u, const void *kf, void *y, int64_t B, hipStream_t s);

// ---- the per-GPU static workspace of fftconv_forward_static (multipass.hip)
int static_workspace_init(int device);     // once per device, with that device current (plan creation)
void *static_workspace(int device);        // its device address, nullptr before static_workspace_init

// ---- multi-pass path (multipass.hip)
bool multipass_supported(int64_t N, int64_t M, int dtype);
int multipass_init(fftconv_plan *p);
size_t multipass_kf_bytes(const fftconv_plan *p);
size_t multipass_workspace_bytes(const fftconv_plan *p, int64_t B);
// outer pass of the filter transform of a multi-pass plan (multipass.hip), where a kernel for the plan's outer length exists
bool multipass_filter_outer_ok(const fftconv_plan *p);
int multipass_filter_outer(const fftconv_plan *p, const void *rows, int dtype, int64_t Nk, int64_t nh, void *T2, hipStream_t s);
int multipass_dk_outer_inv(const fftconv_plan *p, const void *T2, float *dk, int64_t Nk, int64_t nh, float scale, hipStream_t s);
int multipass_pack_kf(const fftconv_plan *p, const double2 *spec, int64_t h0, int64_t nh,
                      const uint8_t *keep_dev, int64_t n_blocks, void *kf, hipStream_t s);
int multipass_forward(const fftconv_plan *p, const void *u, const void *kf, void *y, int64_t B, void *workspace,
                      hipStream_t s, int ko_lo = 0, int ko_hi = 0, const void *wg = nullptr, const void *vg = nullptr);

}  // namespace fftconv
