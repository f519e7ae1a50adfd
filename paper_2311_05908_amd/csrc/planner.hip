// Cost model of an order-p decomposition (paper Section 3.2, Eq. 2) and the choice of p it gives.
// Host-only arithmetic: nothing here touches the GPU.
//
//   C = B H sum_{i=1..p} ( 16 N N_i / gamma(N_i)  +  4 N / omega(i) )
//
// gamma(N_i) is the matrix-unit rate tau_M when the factor is at least as large as the unit (mu), the
// general arithmetic rate tau_G otherwise; omega(i) is the bandwidth of the memory that holds the
// intermediate result of step i.  The paper gives omega only through its kernels' behaviour (Section
// 3.1, Section 3.2's remarks on the figure): the innermost three steps form one fused kernel that keeps a
// whole (sub)sequence on chip if it fits, every step outside that kernel takes a trip through
// HBM, and the first step of the fused kernel reads its input from HBM.  That is the rule coded here:
//   outer steps (i <= p - 3):                         sigma_H
//   first fused step (i = max(1, p - 2)):             sigma_H
//   later fused steps: sigma_S if the subsequence N / (product of the outer factors) fits on chip
//                      (<= sram_seq), sigma_H otherwise (the "bump" of p = 3 past the on-chip limit).
#include <cmath>

#include "fftconv_internal.h"

extern "C" {

void fftconv_machine_preset(int which, fftconv_machine *m)
{
    if (!m) return;
    if (which == FFTCONV_MACHINE_A100_PAPER) {
        // Appendix C, table of measured constants for A100-40GB
        m->sigma_H = 1.35e12;
        m->sigma_S = 9.5e12;
        m->tau_M = 234e12;
        m->tau_G = 17.6e12;
        m->mu = 16;
        m->sram_seq = 32768;      // Section 3.2: p = 3 runs out of on-chip memory between 32K and 64K
    } else {
        // MI355X: what fftconv_measure_machine() (machine.hip; `python bench.py --constants`) returned on
        // one, median of three runs, rounded to two digits:
        //   sigma_H  plain copy of 1 GiB, bytes read + written per second                        4.79e12
        //   sigma_S  slow-down of a chain of matrix products from a trip through LDS per link    53e12
        //   tau_M    v_mfma_f32_16x16x32_bf16 back to back, 16 accumulators, 2 waves per SIMD     2.27e15
        //   tau_G    fp32 twiddle products (6 operations each) applied over and over             74e12
        m->sigma_H = 4.8e12;
        m->sigma_S = 53e12;
        m->tau_M = 2.27e15;
        m->tau_G = 74e12;
        m->mu = 16;               // 16 x 16 MFMA tiles
        m->sram_seq = 32768;      // 160 KB of LDS hold 32768 16-bit (re, im) pairs
    }
}

double fftconv_cost_model(const fftconv_machine *m, int64_t B, int64_t H, int64_t N, int p, const int64_t *factors)
{
    if (!m || !factors || p < 1 || p > 8 || N < 1 || B < 0 || H < 0) return -1.0;
    int64_t prod = 1;
    for (int i = 0; i < p; ++i) {
        if (factors[i] < 1) return -1.0;
        prod *= factors[i];
    }
    if (prod != N) return -1.0;
    const int first_fused = p > 3 ? p - 3 : 0;            // 0-based index of the fused kernel's first step
    int64_t sub = N;
    for (int i = 0; i < first_fused; ++i) sub /= factors[i];
    const bool on_chip = sub <= m->sram_seq;
    double c = 0.0;
    for (int i = 0; i < p; ++i) {
        const double gamma = factors[i] >= m->mu ? m->tau_M : m->tau_G;
        const double omega = (i <= first_fused || !on_chip) ? m->sigma_H : m->sigma_S;
        c += 16.0 * (double)N * (double)factors[i] / gamma + 4.0 * (double)N / omega;
    }
    return (double)B * (double)H * c;
}

// Balanced power-of-two factors of N for order p, larger ones first (the paper's N_1 = ... = N_p
// where log2 N divides evenly).
int fftconv_balanced_factors(int64_t N, int p, int64_t *factors)
{
    if (!factors || p < 1 || p > 8 || N < 1 || (N & (N - 1))) return FFTCONV_EINVAL;
    int lg = 0;
    while (((int64_t)1 << lg) < N) ++lg;
    for (int i = 0; i < p; ++i) {
        const int e = lg / p + (i < lg % p ? 1 : 0);
        factors[i] = (int64_t)1 << e;
    }
    return FFTCONV_OK;
}

int fftconv_plan_order(const fftconv_machine *m, int64_t N, int *p_out, int64_t *factors_out, double *cost_out)
{
    if (!m || N < 4 || (N & (N - 1))) return FFTCONV_EINVAL;
    int best_p = 0;
    double best = 0.0;
    int64_t best_f[4] = {0, 0, 0, 0};
    for (int p = 2; p <= 4; ++p) {
        int64_t f[4];
        if (fftconv_balanced_factors(N, p, f)) continue;
        const double c = fftconv_cost_model(m, 1, 1, N, p, f);
        if (c < 0) continue;
        if (!best_p || c < best) {
            best_p = p;
            best = c;
            for (int i = 0; i < p; ++i) best_f[i] = f[i];
        }
    }
    if (!best_p) return FFTCONV_EINVAL;
    if (p_out) *p_out = best_p;
    if (factors_out)
        for (int i = 0; i < best_p; ++i) factors_out[i] = best_f[i];
    if (cost_out) *cost_out = best;
    return FFTCONV_OK;
}

}  // extern "C"
