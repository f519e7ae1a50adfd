// C ABI of libfftconv.so: argument checking, plan life cycle and dispatch to the
// kernel families.  See include/fftconv.h for the contract of every entry point.
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>

#include <vector>

#include "fftconv_internal.h"

namespace fftconv {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

// (device, kernel) pairs whose limit has been raised; a fixed table, so nothing is allocated here
int raise_dynamic_lds(const void *kernel, int bytes)
{
    struct Entry { int device; const void *kernel; int bytes; };
    static std::mutex mu;
    static Entry done[1024];
    static int n_done = 0;
    int dev = 0;
    FC_HIP(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lock(mu);
    for (int i = 0; i < n_done; ++i)
        if (done[i].device == dev && done[i].kernel == kernel && done[i].bytes >= bytes) return FFTCONV_OK;
    FC_HIP(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
    if (n_done < 1024) done[n_done++] = Entry{dev, kernel, bytes};
    return FFTCONV_OK;
}

LaunchGate &launch_gate()
{
    static thread_local LaunchGate g;
    return g;
}

static bool is_pow2(int64_t v) { return v > 0 && (v & (v - 1)) == 0; }

constexpr int64_t MAX_BLOCKS = 4096;

}  // namespace fftconv

using namespace fftconv;

static int check_plan(const fftconv_plan *p, const char *who)
{
    if (!p) {
        set_error("%s: plan is NULL", who);
        return FFTCONV_EINVAL;
    }
    return FFTCONV_OK;
}

// ---- which kernel family runs a shape (Section 3.2: the order of the decomposition is chosen with the cost
// model).  Every family that has a kernel for the shape is priced with Eq. 2 on its own factorisation and the
// cheapest one wins.  Families differ in what Eq. 2's terms mean for them: "small" computes on the vector
// ALUs (gamma = tau_G whatever the factor), the others on the matrix cores; "multipass" has its outer step
// in kernels of their own (one more trip through HBM, priced as an order-4 decomposition).
static const char *path_name(Path path)
{
    switch (path) {
    case PATH_FUSED3: return "fused3";
    case PATH_MULTIPASS: return "multipass";
    case PATH_SMALL: return "small";
    default: return "staged";
    }
}

static double path_cost(Path path, int64_t M)
{
    fftconv_machine m;
    fftconv_machine_preset(FFTCONV_MACHINE_MI355X, &m);
    int64_t f[4];
    switch (path) {
    case PATH_FUSED3:
        // the 8192-point kernel runs shorter transforms with its outermost matrix block diagonal
        f[0] = 32, f[1] = M >= 32768 ? 32 : 16, f[2] = M >= 16384 ? 32 : 16;
        return fftconv_cost_model(&m, 1, 1, f[0] * f[1] * f[2], 3, f) * (double)M / (double)(f[0] * f[1] * f[2]);
    case PATH_SMALL: {
        m.mu = 1 << 30;                                  // no factor reaches the matrix unit: vector ALUs
        const FacList fl = small_factor_list(M);
        int64_t g[MAX_FACTORS];
        for (int i = 0; i < fl.nf; ++i) g[i] = fl.fac[i];
        return fftconv_cost_model(&m, 1, 1, M, fl.nf, g);
    }
    case PATH_MULTIPASS:
        f[0] = M / 8192, f[1] = 32, f[2] = 16, f[3] = 16;
        return fftconv_cost_model(&m, 1, 1, M, 4, f);
    default: {
        m.mu = 1 << 30;                                  // fp32 on the vector ALUs, one kernel per group of factors
        const FacList fl = staged_factors_for(M);
        int64_t g[MAX_FACTORS];
        for (int i = 0; i < fl.nf; ++i) g[i] = fl.fac[i];
        m.sram_seq = 0;                                  // every step priced at HBM bandwidth
        return fftconv_cost_model(&m, 1, 1, M, fl.nf, g);
    }
    }
}

static bool path_supported(Path path, int64_t N, int64_t M, int dtype)
{
    switch (path) {
    case PATH_FUSED3: return fused3_supported(N, M, dtype);
    case PATH_SMALL: return small_supported(N, M, dtype);
    case PATH_MULTIPASS: return multipass_supported(N, M, dtype);
    default: return dtype == FFTCONV_F32 && M >= 8192 && N <= M;      // the generic path: fp32 I/O from 8192 up
    }
}

// forced: a family's name, or nullptr / "" for the cheapest supported one; false if nothing fits
static bool choose_path(int64_t N, int64_t M, int dtype, const char *forced, Path *out)
{
    const Path all[4] = {PATH_FUSED3, PATH_SMALL, PATH_MULTIPASS, PATH_STAGED};
    bool found = false;
    double best = 0.0;
    for (Path c : all) {
        if (forced && forced[0] && strcmp(forced, path_name(c)) != 0) continue;
        if (!path_supported(c, N, M, dtype)) continue;
        const double cost = path_cost(c, M);
        if (!found || cost < best) {
            found = true;
            best = cost;
            *out = c;
        }
    }
    return found;
}

extern "C" {

int fftconv_plan_create(fftconv_plan **out, int64_t N, int64_t fft_size, int64_t H, int dtype)
{
    return fftconv_plan_create_path(out, N, fft_size, H, dtype, nullptr);
}

int fftconv_plan_create_path(fftconv_plan **out, int64_t N, int64_t fft_size, int64_t H, int dtype, const char *path)
{
    if (!out) {
        set_error("fftconv_plan_create: out is NULL");
        return FFTCONV_EINVAL;
    }
    *out = nullptr;
    if (!is_pow2(fft_size) || fft_size < 256 || fft_size > ((int64_t)1 << 22)) {
        set_error("fftconv_plan_create: fft_size=%lld must be a power of two in [256, 2^22]", (long long)fft_size);
        return FFTCONV_EINVAL;
    }
    if (N < 1 || N > fft_size) {
        set_error("fftconv_plan_create: N=%lld must satisfy 1 <= N <= fft_size=%lld", (long long)N,
                  (long long)fft_size);
        return FFTCONV_EINVAL;
    }
    if (H < 1 || H > ((int64_t)1 << 24)) {
        set_error("fftconv_plan_create: H=%lld out of range", (long long)H);
        return FFTCONV_EINVAL;
    }
    if (dtype != FFTCONV_F32 && dtype != FFTCONV_F16 && dtype != FFTCONV_BF16) {
        set_error("fftconv_plan_create: unknown dtype %d", dtype);
        return FFTCONV_EINVAL;
    }
    Path chosen = PATH_STAGED;
    if (!choose_path(N, fft_size, dtype, path, &chosen)) {
        set_error("fftconv_plan_create: no kernel of family \"%s\" for N=%lld, fft_size=%lld, dtype %d", path ? path : "",
                  (long long)N, (long long)fft_size, dtype);
        return FFTCONV_EUNSUPPORTED;
    }
    int ndev = 0;
    hipError_t e = hipGetDeviceCount(&ndev);
    if (e != hipSuccess || ndev < 1) {
        (void)hipGetLastError();
        set_error("fftconv_plan_create: no usable GPU (%s)", e == hipSuccess ? "device count 0" : hipGetErrorString(e));
        return FFTCONV_ENODEV;
    }
    fftconv_plan *p = new (std::nothrow) fftconv_plan();
    if (!p) {
        set_error("fftconv_plan_create: out of host memory");
        return FFTCONV_ENOMEM;
    }
    p->N = N;
    p->M = fft_size;
    p->H = H;
    p->dtype = dtype;
    int rc = FFTCONV_OK;
    if (hipGetDevice(&p->device) != hipSuccess) rc = FFTCONV_EHIP;
    // the path first: the generic tables depend on it (position order of the fp32 plans' k_f)
    p->path = chosen;
    if (rc == FFTCONV_OK) rc = static_workspace_init(p->device);       // address of this device's static workspace
    if (rc == FFTCONV_OK) rc = staged_init(p);      // twiddle tables, scratch of the filter transform
    if (rc == FFTCONV_OK && long_fft_supported(p)) rc = long_fft_init(p);
    if (rc == FFTCONV_OK && hipMalloc((void **)&p->keep_dev, (size_t)(fft_size > MAX_BLOCKS ? fft_size : MAX_BLOCKS)) != hipSuccess) {
        set_error("fftconv_plan_create: hipMalloc of the block mask failed");
        rc = FFTCONV_ENOMEM;
    }
    if (rc == FFTCONV_OK) {
        if (p->path == PATH_FUSED3) rc = fused3_init(p);
        else if (p->path == PATH_SMALL) rc = small_init(p);
        else if (p->path == PATH_MULTIPASS) rc = multipass_init(p);
    }
    if (rc != FFTCONV_OK) {
        fftconv_plan_destroy(p);
        return rc;
    }
    *out = p;
    return FFTCONV_OK;
}

int fftconv_plan_destroy(fftconv_plan *p)
{
    if (!p) return FFTCONV_OK;
    fused3_destroy(p);
    staged_destroy(p);
    long_fft_destroy(p);
    if (p->keep_dev) (void)hipFree(p->keep_dev);
    delete p;
    return FFTCONV_OK;
}

size_t fftconv_kf_bytes(const fftconv_plan *p)
{
    if (!p) return 0;
    switch (p->path) {
    case PATH_FUSED3: return fused3_kf_bytes(p);
    case PATH_MULTIPASS: return multipass_kf_bytes(p);
    case PATH_SMALL: return small_kf_bytes(p);
    default: return staged_kf_bytes(p);
    }
}

size_t fftconv_workspace_bytes(const fftconv_plan *p, int64_t B)
{
    if (!p || B <= 0) return 0;
    switch (p->path) {
    case PATH_FUSED3: return 0;
    case PATH_SMALL: return 0;
    case PATH_MULTIPASS: return multipass_workspace_bytes(p, B);
    default: return staged_workspace_bytes(p, B);
    }
}

// block_keep with n_blocks == fft_size is a per-bin mask (internal callers only; the device copy of the
// mask has room for it)
static int filter_fft_impl(const fftconv_plan *p, const float *k, int64_t Nk, const uint8_t *block_keep,
                           int64_t n_blocks, void *k_f, void *stream, const char *who, bool adjoint = false,
                           bool per_bin = false)
{
    int rc = check_plan(p, who);
    if (rc) return rc;
    if (!k || !k_f) {
        set_error("%s: k and k_f must not be NULL", who);
        return FFTCONV_EINVAL;
    }
    if (Nk < 1 || Nk > p->M) {
        set_error("%s: Nk=%lld must satisfy 1 <= Nk <= fft_size=%lld", who, (long long)Nk, (long long)p->M);
        return FFTCONV_EINVAL;
    }
    hipStream_t s = (hipStream_t)stream;
    const uint8_t *keep_dev = nullptr;
    if (block_keep) {
        if (!(per_bin && n_blocks == p->M) && (!is_pow2(n_blocks) || n_blocks > MAX_BLOCKS || n_blocks > p->M)) {
            set_error("%s: n_blocks=%lld must be a power of two <= min(%lld, fft_size)", who, (long long)n_blocks,
                      (long long)MAX_BLOCKS);
            return FFTCONV_EINVAL;
        }
        FC_HIP(hipMemcpyAsync(p->keep_dev, block_keep, (size_t)n_blocks, hipMemcpyHostToDevice, s));
        keep_dev = p->keep_dev;
    }
    if (p->path == PATH_FUSED3) {
        rc = fused3_filter(p, k, Nk, adjoint, keep_dev, n_blocks, k_f, s);
        if (rc) return rc;
    }
    const bool long_rows = p->path == PATH_MULTIPASS && long_fft_supported(p);
    // fp32 k_f in the position order of the long transforms (staged plans from fft 32768 up) with a real outer pass
    const bool long_rows_f32 = p->path == PATH_STAGED && p->M >= 32768 && long_fft_supported(p) && multipass_filter_outer_ok(p);
    // fp32 in two kernels per chunk; the scratch buffer is sized for fp64 spectra, so it takes twice the rows, and
    // where only the outer rows ko <= No/2 pass through it (multipass_filter_outer) nearly twice as many again
    int64_t long_chunk = 2 * p->filt_chunk;
    if ((long_rows || long_rows_f32) && multipass_filter_outer_ok(p)) {
        const int64_t No = p->M / 8192;
        long_chunk = long_chunk * No / (No / 2 + 1);
    }
    for (int64_t h0 = 0; long_rows && h0 < p->H; h0 += long_chunk) {
        const int64_t nh = p->H - h0 < long_chunk ? p->H - h0 : long_chunk;
        rc = long_filter_transform(p, k + h0 * Nk, Nk, h0, nh, adjoint, keep_dev, n_blocks, (float2 *)p->filt_a, k_f, s);
        if (rc) return rc;
    }
    for (int64_t h0 = 0; long_rows_f32 && h0 < p->H; h0 += long_chunk) {
        const int64_t nh = p->H - h0 < long_chunk ? p->H - h0 : long_chunk;
        rc = long_filter_transform_f32(p, k + h0 * Nk, Nk, h0, nh, adjoint, keep_dev, n_blocks, (float2 *)p->filt_a, k_f, s);
        if (rc) return rc;
    }
    for (int64_t h0 = 0; p->path != PATH_FUSED3 && !long_rows && !long_rows_f32 && h0 < p->H; h0 += p->filt_chunk) {
        int64_t nh = p->H - h0 < p->filt_chunk ? p->H - h0 : p->filt_chunk;
        double2 *spec = nullptr;
        rc = staged_filter_transform(p, k, Nk, h0, nh, s, &spec, adjoint);
        if (rc) return rc;
        switch (p->path) {
        case PATH_MULTIPASS: rc = multipass_pack_kf(p, spec, h0, nh, keep_dev, n_blocks, k_f, s); break;
        case PATH_SMALL: rc = small_pack_kf(p, spec, h0, nh, keep_dev, n_blocks, k_f, s); break;
        default: rc = staged_pack_kf(p, spec, h0, nh, keep_dev, n_blocks, k_f, s); break;
        }
        if (rc) return rc;
    }
    // a short filter of a plan that can run partial convolutions as short segments: add the
    // short transform's spectrum behind the dense one, and say in the tag behind it which filter length it
    // belongs to (0: none -- masked, adjoint or longer filters leave that region as it was)
    if (p->f3.consts_short) {
        const bool with_short = !block_keep && !adjoint && fused3_short_ok(p, Nk);
        if (with_short) {
            rc = fused3_filter_short(p, k, Nk, k_f, s);
            if (rc) return rc;
        }
        return fused3_set_short_tag(p, k_f, with_short ? Nk : 0, s);
    }
    return FFTCONV_OK;
}

int fftconv_filter_fft(const fftconv_plan *p, const float *k, int64_t Nk, void *k_f, void *stream)
{
    return filter_fft_impl(p, k, Nk, nullptr, 1, k_f, stream, "fftconv_filter_fft");
}

int fftconv_filter_fft_sparse(const fftconv_plan *p, const float *k, int64_t Nk, const uint8_t *block_keep,
                              int64_t n_blocks, void *k_f, void *stream)
{
    if (!block_keep) {
        set_error("fftconv_filter_fft_sparse: block_keep is NULL");
        return FFTCONV_EINVAL;
    }
    return filter_fft_impl(p, k, Nk, block_keep, n_blocks, k_f, stream, "fftconv_filter_fft_sparse");
}

// ---- digit cut-off patterns (Appendix A.4).  The spectrum is viewed as an array over the digits of
// f in the plan's factorisation, f = sum_i d_i w_i with w_0 = 1, w_i = w_{i-1} * factors[i-1] (the
// outermost factor is the least significant digit); digit i keeps digit_keep[i] of its D_i values, chosen so
// that the kept set of bins is as close to mirror symmetric (f -> M - f) as a product set can be: the
// mirror image of a bin has digits (D_0 - d_0) mod D_0 and, unless all lower digits are zero, D_i - 1 - d_i.
//   digit 0:     the values nearest zero on the circle,        d <= keep / 2      or d >= D_0 - (keep - 1) / 2
//   digits i>0:  the values nearest the two ends of the range, d < ceil(keep / 2) or d >= D_i - keep / 2
struct DigitPattern {
    int nd = 0;
    int64_t D[8] = {0}, lo[8] = {0}, hi[8] = {0};       // kept: d < lo or d >= hi
};

static int digit_pattern(const fftconv_plan *p, const int64_t *digit_keep, int ndigits, const char *who,
                         DigitPattern *out)
{
    int64_t fac[8];
    const int nf = fftconv_plan_factors(p, fac, 8);
    if (!digit_keep || ndigits != nf || nf > 8) {
        set_error("%s: digit_keep must hold one entry per factor of the plan (%d)", who, nf);
        return FFTCONV_EINVAL;
    }
    out->nd = nf;
    for (int i = 0; i < nf; ++i) {
        if (digit_keep[i] < 1 || digit_keep[i] > fac[i]) {
            set_error("%s: digit_keep[%d]=%lld must be in [1, %lld]", who, i, (long long)digit_keep[i], (long long)fac[i]);
            return FFTCONV_EINVAL;
        }
        out->D[i] = fac[i];
        out->lo[i] = i == 0 ? digit_keep[i] / 2 + 1 : (digit_keep[i] + 1) / 2;
        out->hi[i] = i == 0 ? fac[i] - (digit_keep[i] - 1) / 2 : fac[i] - digit_keep[i] / 2;
    }
    return FFTCONV_OK;
}

int fftconv_filter_fft_sparse_digits(const fftconv_plan *p, const float *k, int64_t Nk, const int64_t *digit_keep,
                                     int ndigits, void *k_f, void *stream)
{
    const char *who = "fftconv_filter_fft_sparse_digits";
    int rc = check_plan(p, who);
    if (rc) return rc;
    DigitPattern dp;
    rc = digit_pattern(p, digit_keep, ndigits, who, &dp);
    if (rc) return rc;
    std::vector<uint8_t> keep((size_t)p->M);
    for (int64_t f = 0; f < p->M; ++f) {
        int64_t r = f;
        bool kept = true;
        for (int i = 0; i < dp.nd && kept; ++i) {
            const int64_t d = r % dp.D[i];
            r /= dp.D[i];
            kept = d < dp.lo[i] || d >= dp.hi[i];
        }
        keep[(size_t)f] = kept ? 1 : 0;
    }
    // the copy of a pageable host buffer has completed when hipMemcpyAsync returns
    return filter_fft_impl(p, k, Nk, keep.data(), p->M, k_f, stream, who, false, true);
}

static int forward_check(const fftconv_plan *p, const void *u, const void *k_f, void *y, int64_t B, int64_t H,
                         int64_t N, void *workspace, const char *who)
{
    int rc = check_plan(p, who);
    if (rc) return rc;
    if (B < 0) {
        set_error("%s: B=%lld is negative", who, (long long)B);
        return FFTCONV_EINVAL;
    }
    if (H != p->H || N != p->N) {
        set_error("%s: (H=%lld, N=%lld) differ from the plan's (H=%lld, N=%lld)", who, (long long)H, (long long)N,
                  (long long)p->H, (long long)p->N);
        return FFTCONV_EINVAL;
    }
    if (B == 0) return FFTCONV_OK;
    if (!u || !k_f || !y) {
        set_error("%s: u, k_f and y must not be NULL", who);
        return FFTCONV_EINVAL;
    }
    if (u == y) {
        set_error("%s: y must not alias u", who);
        return FFTCONV_EINVAL;
    }
    if (!workspace && fftconv_workspace_bytes(p, B) != 0) {
        set_error("%s: this plan needs %zu bytes of workspace for B=%lld", who, fftconv_workspace_bytes(p, B),
                  (long long)B);
        return FFTCONV_EINVAL;
    }
    return FFTCONV_OK;
}

int fftconv_forward(const fftconv_plan *p, const void *u, const void *k_f, void *y, int64_t B, int64_t H, int64_t N,
                    void *workspace, void *stream)
{
    int rc = forward_check(p, u, k_f, y, B, H, N, workspace, "fftconv_forward");
    if (rc || B == 0) return rc;
    hipStream_t s = (hipStream_t)stream;
    switch (p->path) {
    case PATH_FUSED3:
        return fused3_forward(p, u, k_f, y, B, s);
    case PATH_MULTIPASS:
        return multipass_forward(p, u, k_f, y, B, workspace, s);
    case PATH_SMALL:
        return small_forward(p, u, k_f, y, B, s);
    default:
        return staged_forward(p, u, k_f, y, B, workspace, s);
    }
}

int fftconv_forward_static(const fftconv_plan *p, const void *u, const void *k_f, void *y, int64_t B, int64_t H,
                           int64_t N, void *stream)
{
    int rc = forward_check(p, u, k_f, y, B, H, N, (void *)1, "fftconv_forward_static");
    if (rc || B == 0) return rc;
    const size_t need = fftconv_workspace_bytes(p, B);
    if (need > FFTCONV_STATIC_WORKSPACE_BYTES) {
        set_error("fftconv_forward_static: this plan needs %zu bytes of workspace for B=%lld, the static workspace "
                  "holds %zu; use fftconv_forward with a workspace of the caller's",
                  need, (long long)B, (size_t)FFTCONV_STATIC_WORKSPACE_BYTES);
        return FFTCONV_EINVAL;
    }
    void *ws = static_workspace(p->device);
    if (need > 0 && !ws) {
        set_error("fftconv_forward_static: the static workspace of device %d was never initialised", p->device);
        return FFTCONV_EHIP;
    }
    return fftconv_forward(p, u, k_f, y, B, H, N, need ? ws : nullptr, stream);
}

int fftconv_filter_fft_adjoint(const fftconv_plan *p, const float *k, int64_t Nk, void *k_f, void *stream)
{
    return filter_fft_impl(p, k, Nk, nullptr, 1, k_f, stream, "fftconv_filter_fft_adjoint", true);
}

int fftconv_backward_input(const fftconv_plan *p, const void *dy, const void *k_f_adjoint, void *du, int64_t B,
                           int64_t H, int64_t N, void *workspace, void *stream)
{
    int rc = forward_check(p, dy, k_f_adjoint, du, B, H, N, workspace, "fftconv_backward_input");
    if (rc || B == 0) return rc;
    // the same kernels as the forward pass: du = iFFT(FFT(pad(dy)) . conj(k_f))[0:N]
    return fftconv_forward(p, dy, k_f_adjoint, du, B, H, N, workspace, stream);
}

size_t fftconv_workspace_bytes_backward_filter(const fftconv_plan *p, int64_t B)
{
    if (!p || B <= 0) return 0;
    if (f3::fused3_dk_supported(p))        // accumulated spectra of every channel (8192 slots each, whatever the plan's fft_size)
        return (size_t)(p->H * 8192) * sizeof(float2);
    if (f3::fused3_big_dk_supported(p))
        return (size_t)(2 * p->H * p->M) * sizeof(float2);
    if (long_fft_supported(p)) return long_backward_filter_bytes(p);
    return staged_backward_filter_bytes(p);
}

int fftconv_backward_filter(const fftconv_plan *p, const void *u, const void *dy, float *dk, int64_t Nk, int64_t B,
                            int64_t H, int64_t N, void *workspace, void *stream)
{
    int rc = check_plan(p, "fftconv_backward_filter");
    if (rc) return rc;
    if (B < 0 || H != p->H || N != p->N) {
        set_error("fftconv_backward_filter: B=%lld must be >= 0 and (H=%lld, N=%lld) equal the plan's (H=%lld, N=%lld)",
                  (long long)B, (long long)H, (long long)N, (long long)p->H, (long long)p->N);
        return FFTCONV_EINVAL;
    }
    if (Nk < 1 || Nk > p->M) {
        set_error("fftconv_backward_filter: Nk=%lld must satisfy 1 <= Nk <= fft_size", (long long)Nk);
        return FFTCONV_EINVAL;
    }
    if (!dk || (B > 0 && (!u || !dy || !workspace))) {
        set_error("fftconv_backward_filter: u, dy, dk and workspace must not be NULL");
        return FFTCONV_EINVAL;
    }
    hipStream_t s = (hipStream_t)stream;
    if (B > 0 && f3::fused3_dk_supported(p)) {
        rc = f3::fused3_dk_accumulate(p, u, dy, workspace, B, s);       // 8192 accumulator slots per channel
        if (!rc) rc = f3::fused3_dk_finish(p, workspace, dk, Nk, s);
        return rc;
    }
    if (B > 0 && f3::fused3_big_dk_supported(p)) {
        float2 *dkf = (float2 *)workspace;                          // accumulated spectra, then a scratch row each
        rc = f3::fused3_big_dk_accumulate(p, u, dy, dkf, B, s);
        if (!rc) rc = f3::fused3_big_dk_finish(p, dkf, dkf + p->H * p->M, dk, Nk, s);
        return rc;
    }
    if (long_fft_supported(p)) return long_backward_filter(p, u, dy, dk, Nk, B, workspace, s);
    return staged_backward_filter(p, u, dy, dk, Nk, B, workspace, s);
}

int fftconv_forward_partial(const fftconv_plan *p, const void *u, const void *k_f, void *y, int64_t B, int64_t H,
                            int64_t N, int64_t Nk, void *workspace, void *stream)
{
    int rc = forward_check(p, u, k_f, y, B, H, N, workspace, "fftconv_forward_partial");
    if (rc) return rc;
    if (Nk < 1 || Nk > p->M) {
        set_error("fftconv_forward_partial: Nk=%lld must satisfy 1 <= Nk <= fft_size", (long long)Nk);
        return FFTCONV_EINVAL;
    }
    if (B == 0) return FFTCONV_OK;
    if (!fused3_short_ok(p, Nk)) return fftconv_forward(p, u, k_f, y, B, H, N, workspace, stream);
    // Both routes are launched, gated on the tag the filter transform left in k_f: the overlapping short
    // segments run if k_f carries a short spectrum for exactly this Nk, the plan's dense kernels otherwise
    // (a k_f from another Nk, a masked or an adjoint one); the kernels of the other route return at once.
    struct GateScope {
        LaunchGate saved = launch_gate();
        ~GateScope() { launch_gate() = saved; }
    } scope;
    launch_gate() = LaunchGate{fused3_short_tag(p, k_f), (long long)Nk, 1};
    rc = fused3_forward_short(p, u, k_f, y, B, Nk, (hipStream_t)stream);
    if (rc) return rc;
    launch_gate().run_if_equal = 0;
    return fftconv_forward(p, u, k_f, y, B, H, N, workspace, stream);
}

int fftconv_forward_freq_sparse(const fftconv_plan *p, const void *u, const void *k_f, const uint8_t *block_keep,
                                int64_t n_blocks, void *y, int64_t B, int64_t H, int64_t N, void *workspace,
                                void *stream)
{
    int rc = forward_check(p, u, k_f, y, B, H, N, workspace, "fftconv_forward_freq_sparse");
    if (rc) return rc;
    if (!block_keep || !is_pow2(n_blocks) || n_blocks > MAX_BLOCKS || n_blocks > p->M) {
        set_error("fftconv_forward_freq_sparse: block_keep must be given, n_blocks a power of two <= min(%lld, fft_size)",
                  (long long)MAX_BLOCKS);
        return FFTCONV_EINVAL;
    }
    if (B == 0) return FFTCONV_OK;
    if (p->path == PATH_FUSED3)
        return fused3_forward_sparse(p, u, k_f, y, B, fused3_live_k3(p, block_keep, n_blocks),
                                     (hipStream_t)stream);
    return fftconv_forward(p, u, k_f, y, B, H, N, workspace, stream);
}

int fftconv_forward_freq_sparse_digits(const fftconv_plan *p, const void *u, const void *k_f, const int64_t *digit_keep,
                                       int ndigits, void *y, int64_t B, int64_t H, int64_t N, void *workspace,
                                       void *stream)
{
    const char *who = "fftconv_forward_freq_sparse_digits";
    int rc = forward_check(p, u, k_f, y, B, H, N, workspace, who);
    if (rc) return rc;
    DigitPattern dp;
    rc = digit_pattern(p, digit_keep, ndigits, who, &dp);
    if (rc) return rc;
    if (B == 0) return FFTCONV_OK;
    // values of a digit that can meet a non-zero bin: the kept ones and their images under both forms of the
    // mirror map (d -> (D - d) mod D and d -> D - 1 - d), as a bit mask (digits of at most 32 values)
    auto live_mask = [&](int i) -> uint32_t {
        if (dp.D[i] > 32) return 0xffffffffu;
        uint32_t m = 0;
        for (int64_t d = 0; d < dp.D[i]; ++d)
            if (d < dp.lo[i] || d >= dp.hi[i]) m |= (1u << d) | (1u << ((dp.D[i] - d) % dp.D[i])) | (1u << (dp.D[i] - 1 - d));
        if (dp.D[i] < 32) m |= ~((1u << dp.D[i]) - 1u);
        return m;
    };
    if (p->path == PATH_FUSED3)          // digits (k1, k2, k3)
        return fused3_forward_sparse(p, u, k_f, y, B, live_mask(2), (hipStream_t)stream, live_mask(0), live_mask(1));
    if (p->path == PATH_MULTIPASS) {
        // digit 0 is the outer frequency ko; kept: ko < lo or ko >= hi, whose mirror images (No - ko) mod No
        // are ko <= lo - 1 and ko >= No - (lo - 1)
        if (!workspace && fftconv_workspace_bytes(p, B) > 0) {
            set_error("%s: workspace is NULL", who);
            return FFTCONV_EINVAL;
        }
        const int64_t a = dp.lo[0] - 1;                  // largest kept distance from zero
        const int64_t lo = a + 1, hi = dp.D[0] - a;
        return multipass_forward(p, u, k_f, y, B, workspace, (hipStream_t)stream, (int)lo, (int)hi);
    }
    return fftconv_forward(p, u, k_f, y, B, H, N, workspace, stream);
}

static size_t elem_bytes(const fftconv_plan *p) { return p->dtype == FFTCONV_F32 ? 4 : 2; }
static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

size_t fftconv_workspace_bytes_gated(const fftconv_plan *p, int64_t B)
{
    if (!p || B <= 0) return 0;
    const size_t base = fftconv_workspace_bytes(p, B);
    if (fused3_gates_fused(p) || p->path == PATH_MULTIPASS) return base;       // gates fused into the plan's kernels
    return align256(base) + (size_t)(B * p->H * p->N) * elem_bytes(p);
}

int fftconv_forward_gated(const fftconv_plan *p, const void *u, const void *w, const void *v, const void *k_f, void *y,
                          int64_t B, int64_t H, int64_t N, void *workspace, void *stream)
{
    if (!w && !v) return fftconv_forward(p, u, k_f, y, B, H, N, workspace, stream);
    // the checks of fftconv_forward, against the larger workspace
    int rc = forward_check(p, u, k_f, y, B, H, N, (void *)1, "fftconv_forward_gated");
    if (rc || B == 0) return rc;
    if (v == y) {
        set_error("fftconv_forward_gated: v must not alias y");
        return FFTCONV_EINVAL;
    }
    if (!workspace && fftconv_workspace_bytes_gated(p, B) != 0) {
        set_error("fftconv_forward_gated: this plan needs %zu bytes of workspace for B=%lld",
                  fftconv_workspace_bytes_gated(p, B), (long long)B);
        return FFTCONV_EINVAL;
    }
    hipStream_t s = (hipStream_t)stream;
    if (fused3_gates_fused(p)) return fused3_forward_gated(p, u, w, v, k_f, y, B, s);
    if (p->path == PATH_MULTIPASS)          // the outer passes multiply the gates in as they load u / store y
        return multipass_forward(p, u, k_f, y, B, workspace, s, 0, 0, w, v);
    const int64_t n = B * p->H * p->N;
    const void *src = u;
    if (w) {
        void *prod = (char *)workspace + align256(fftconv_workspace_bytes(p, B));
        rc = gate_multiply(p->dtype, u, w, prod, n, s);
        if (rc) return rc;
        src = prod;
    }
    rc = fftconv_forward(p, src, k_f, y, B, H, N, workspace, stream);
    if (rc || !v) return rc;
    return gate_multiply(p->dtype, y, v, y, n, s);
}

double fftconv_sparsity_fraction(const int64_t *dims, const int64_t *cuts, int ndim)
{
    if (!dims || !cuts || ndim < 1) return -1.0;
    double kept = 1.0;
    for (int i = 0; i < ndim; ++i) {
        if (dims[i] < 1 || cuts[i] < 0 || cuts[i] > dims[i]) return -1.0;
        kept *= (double)(dims[i] - cuts[i]) / (double)dims[i];
    }
    return 1.0 - kept;
}

const char *fftconv_plan_path(const fftconv_plan *p) { return p ? path_name(p->path) : ""; }

int fftconv_plan_factors(const fftconv_plan *p, int64_t *factors, int max_factors)
{
    if (!p || !factors) return 0;
    int n = 0;
    if (p->path == PATH_FUSED3) {
        int64_t f[3] = {p->f3.N1, p->f3.N2, p->f3.N3};
        for (; n < 3 && n < max_factors; ++n) factors[n] = f[n];
        return 3;
    }
    if (p->path == PATH_SMALL) {
        int64_t f[3] = {p->f3.N1, p->f3.N2, p->f3.N3};
        const int nf = p->f3.N3 > 1 ? 3 : 2;
        for (; n < nf && n < max_factors; ++n) factors[n] = f[n];
        return nf;
    }
    if (p->path == PATH_MULTIPASS) {
        int64_t f[4] = {p->M / ((int64_t)p->f3.N1 * p->f3.N2 * p->f3.N3), p->f3.N1, p->f3.N2, p->f3.N3};
        for (; n < 4 && n < max_factors; ++n) factors[n] = f[n];
        return 4;
    }
    for (; n < p->st.nf && n < max_factors; ++n) factors[n] = p->st.fac[n];
    return p->st.nf;
}

const char *fftconv_strerror(int code)
{
    switch (code) {
    case FFTCONV_OK: return "ok";
    case FFTCONV_EINVAL: return "invalid argument";
    case FFTCONV_EUNSUPPORTED: return "unsupported configuration";
    case FFTCONV_EHIP: return "HIP runtime error";
    case FFTCONV_ENOMEM: return "out of memory";
    case FFTCONV_ENODEV: return "no usable GPU";
    default: return "unknown error code";
    }
}

const char *fftconv_last_error(void) { return fftconv::g_err; }

}  // extern "C"
