// Transforms of whole rows resident in LDS, shared by the filter transform, the fused filter-transform
// kernels and the tail of the filter gradient.
#pragma once

#include <hip/hip_runtime.h>

#include "dft_reg.h"
#include "fftconv_internal.h"

namespace fftconv {

template <typename V> __device__ __forceinline__ V cmul(V a, V b)
{
    V r;
    r.x = a.x * b.x - a.y * b.y;
    r.y = a.x * b.y + a.y * b.x;
    return r;
}
template <typename V> __device__ __forceinline__ V cmul_conj(V a, V b)   // a * conj(b)
{
    V r;
    r.x = a.x * b.x + a.y * b.y;
    r.y = a.y * b.x - a.x * b.y;
    return r;
}


// The stages of the generic path with a whole row resident in LDS (rows of up to 8192 fp64 or 16384 fp32
// complex points): one workgroup per row, every stage in place (a butterfly reads and writes the same R slots),
// one barrier between stages, HBM touched once on the way in and once on the way out instead of once
// per stage.  Slot p of the row lives at word p + p/16, so that the strided accesses of the late stages
// (neighbouring threads 16^j slots apart) spread over the banks.
constexpr int LDS_ROW_THREADS = 512;
__device__ inline int lds_slot(int p) { return p + (p >> 4); }
inline size_t lds_row_bytes(int64_t M, size_t elem) { return (size_t)(M + M / 16) * elem; }

// The R twiddles W^{k e}, k < R, of one butterfly.  A gather from the table costs the vector-memory path one
// cache-line lookup per lane (the lanes' exponents are k e apart), which is what bounded these kernels when all
// R - 1 were gathered; so only the multiples of 4 e come from the table (tw(x) returns W^x) and the rest are
// products with W^e, W^{2e}, W^{3e}: at most three roundings on top of the table's.
template <int R, typename V, typename TW> __device__ __forceinline__ void stage_twiddles(V (&t)[R], const TW &tw, int64_t e)
{
    t[0].x = 1;
    t[0].y = 0;
    t[1] = tw(e);
    if constexpr (R > 2) {
        t[2] = cmul(t[1], t[1]);
        t[3] = cmul(t[2], t[1]);
    }
    if constexpr (R > 4) {
#pragma unroll
        for (int k = 4; k < R; k += 4) {
            t[k] = tw(k * e);
            t[k + 1] = cmul(t[k], t[1]);
            t[k + 2] = cmul(t[k], t[2]);
            t[k + 3] = cmul(t[k], t[3]);
        }
    }
}

template <typename V> struct TwTable {         // W^x = w[x]
    const V *w;
    __device__ __forceinline__ V operator()(int64_t x) const { return w[x]; }
};

template <int R, bool INV, typename V>
__device__ inline void lds_stage(V *X, const V *__restrict__ w, int M, int Sj, int Rj, int tws)
{
    const TwTable<V> tw{w};
    const int lgS = __ffs(Sj) - 1;                 // every length and stride here is a power of two
    if (Sj == 1) {
        // the innermost stage: r = 0, every twiddle is 1 -- no table gathers (each is a trip to L2 that the
        // butterfly would wait for) and no products
#pragma unroll 4
        for (int t = threadIdx.x; t < M / R; t += blockDim.x) {
            const int base = t * R;
            V x[R];
#pragma unroll
            for (int n = 0; n < R; ++n) x[n] = X[lds_slot(base + n)];
            dft_reg<R, INV>(x);
#pragma unroll
            for (int k = 0; k < R; ++k) X[lds_slot(base + k)] = x[k];
        }
        return;
    }
    for (int t = threadIdx.x; t < M / R; t += blockDim.x) {
        const int r = t & (Sj - 1), prefix = t >> lgS;
        const int base = prefix * (R * Sj) + r;
        V x[R], c[R];
        stage_twiddles<R>(c, tw, (int64_t)Rj * r * tws);
#pragma unroll
        for (int n = 0; n < R; ++n) {
            x[n] = X[lds_slot(base + n * Sj)];
            if (INV) x[n] = cmul_conj(x[n], c[n]);
        }
        dft_reg<R, INV>(x);
#pragma unroll
        for (int k = 0; k < R; ++k) X[lds_slot(base + k * Sj)] = INV ? x[k] : cmul(x[k], c[k]);
    }
}

template <bool INV, typename V>
__device__ inline void lds_stage_any(V *X, const V *w, int M, int Nj, int Sj, int Rj, int tws)
{
    switch (Nj) {
    case 2: lds_stage<2, INV>(X, w, M, Sj, Rj, tws); break;
    case 4: lds_stage<4, INV>(X, w, M, Sj, Rj, tws); break;
    case 8: lds_stage<8, INV>(X, w, M, Sj, Rj, tws); break;
    default: lds_stage<16, INV>(X, w, M, Sj, Rj, tws); break;
    }
}


// every factor has an in-register transform here
inline bool lds_factors_ok(const FacList &fl)
{
    for (int i = 0; i < fl.nf; ++i)
        if (fl.fac[i] != 2 && fl.fac[i] != 4 && fl.fac[i] != 8 && fl.fac[i] != 16) return false;
    return true;
}

// freq_to_pos() and mask_weight() for the lengths of these kernels (powers of two that fit in an int): shifts
// instead of 64-bit divisions
__device__ inline int lds_pos(int f, const FacList &fl, int M)
{
    int pos = 0, lg_s = __ffs(M) - 1;
    for (int i = 0; i < fl.nf; ++i) {
        const int lg = __ffs(fl.fac[i]) - 1;
        lg_s -= lg;
        pos += (f & (fl.fac[i] - 1)) << lg_s;
        f >>= lg;
    }
    return pos;
}
// the inverse of lds_pos(): the frequency held at a position
__device__ inline int lds_freq(int pos, const FacList &fl, int M)
{
    int f = 0, lg_s = __ffs(M) - 1, lg_r = 0;
    for (int i = 0; i < fl.nf; ++i) {
        const int lg = __ffs(fl.fac[i]) - 1;
        lg_s -= lg;
        f |= ((pos >> lg_s) & (fl.fac[i] - 1)) << lg_r;
        lg_r += lg;
    }
    return f;
}
__device__ inline float lds_mask_weight(const uint8_t *keep, int64_t n_blocks, int f, int M)
{
    if (!keep) return 1.f;
    const int lg_per = __ffs(M) - __ffs((int)n_blocks);               // log2(bins per mask block)
    const int fm = f == 0 ? 0 : M - f;
    return 0.5f * ((keep[f >> lg_per] ? 1.f : 0.f) + (keep[fm >> lg_per] ? 1.f : 0.f));
}

// forward transform of the row in X (natural order in, position order out, see freq_to_pos); ends with a barrier
template <typename V> __device__ inline void lds_forward(V *X, const V *w, const FacList &fl, int M, int tws)
{
    int S = M, R = 1;
    for (int i = 0; i < fl.nf; ++i) {
        const int Nj = fl.fac[i];
        S /= Nj;
        lds_stage_any<false>(X, w, M, Nj, S, R, tws);
        __syncthreads();
        R *= Nj;
    }
}

// unnormalised inverse transform (position order in, natural order out); ends with a barrier
template <typename V> __device__ inline void lds_inverse(V *X, const V *w, const FacList &fl, int M, int tws)
{
    int S = 1, R = M;
    for (int i = fl.nf - 1; i >= 0; --i) {
        const int Nj = fl.fac[i];
        R /= Nj;
        lds_stage_any<true>(X, w, M, Nj, S, R, tws);
        __syncthreads();
        S *= Nj;
    }
}

}  // namespace fftconv
