// tq_params: parameter design of the truncated quantizer (arXiv 2402.01798, Sec. IV) from
// the per-bucket statistics, in fp64, one workgroup per bucket.
//
//   tail index      gamma = 1 + n_tail / sum ln(|g|/g_min)            (Sec. V, MLE)
//   tail mass       rho   = n_tail / (2 n)                            (one-sided, Sec. IV-A)
//   threshold       alpha = g_min [2 rho s^2 / ((gamma-2) Q(alpha))]^(1/(gamma-1)),
//                   Q = Q_U (Sec. IV-A, boxed) or Q_N (Sec. IV-B, second boxed equation)
//   codebook        uniform: l_k = -alpha + k 2alpha/s; non-uniform: the points where the
//                   integral of lambda_s ~ p^(1/3) (Sec. IV-B, first boxed equation) reaches k
//
// The density p on [-alpha, alpha] is the histogram's (constant inside a bin).  With the
// prefix sums cum[i] = #{|g| below bin i} and H[i] = int_0^{lo_i} p^(1/3), both Q_U(alpha)
// and the integral of p^(1/3) up to alpha cost O(1) per evaluation, so the fixed-point
// iteration is a short scalar loop on lane 0; the per-bin cube roots and logarithms that
// feed the prefix sums are computed by all lanes.
#include "tq_device.h"

namespace tq {

constexpr int kNB = TQ_NBINS;
constexpr double kGammaFloor = 2.02;
constexpr double kAlphaFloor = 5.421010862427522e-20;   // 2^-64
constexpr int kMaxIter = 100;
constexpr double kRelTol = 1e-10;

__device__ __forceinline__ double bin_lo(int i)
{
    if (i <= 0) return 0.0;
    if (i >= kNB - 1) return 65536.0;
    const int j = i - 1;
    return ldexp(1.0 + (double)(j & 15) * 0.0625, (j >> 4) - 40);
}

__device__ __forceinline__ double bin_hi(int i, double absmax)
{
    if (i >= kNB - 1) return absmax > 131072.0 ? absmax : 131072.0;
    return bin_lo(i + 1);
}

// Bin whose [lo, hi) holds x >= 0 (the last bin is closed above).
__device__ __forceinline__ int bin_of(double x)
{
    if (x < 9.094947017729282e-13) return 0;             // 2^-40
    if (x >= 65536.0) return kNB - 1;
    const int ex = ilogb(x);
    const double m = ldexp(x, -ex);                       // in [1, 2), exact
    return (ex + 40) * 16 + (int)((m - 1.0) * 16.0) + 1;
}

struct ParamsLds {
    double hist[kNB];
    double cum[kNB + 1];   // cum[i] = sum of hist below bin i
    double p13[kNB];       // cube root of the two-sided density on the bin
    double H[kNB + 1];     // H[i] = int_0^{lo_i} p^(1/3)
    double tl[kNB];        // hist * ln(bin's geometric mean / g_min) for the binned tail index
    double g_min;
    int tail_bin;
};

struct DensityView {
    const ParamsLds& L;
    double n, absmax;
    __device__ double covered(int j, double x) const
    {
        const double lo = bin_lo(j), w = bin_hi(j, absmax) - lo;
        double c = x - lo;
        c = c < 0.0 ? 0.0 : (c > w ? w : c);
        return c;
    }
    __device__ double Q_U(double a) const
    {
        const int j = bin_of(a);
        const double w = bin_hi(j, absmax) - bin_lo(j);
        return (L.cum[j] + L.hist[j] * (covered(j, a) / w)) / n;
    }
    __device__ double half_int(double x) const            // int_0^x p^(1/3)
    {
        const int j = bin_of(x);
        return L.H[j] + L.p13[j] * covered(j, x);
    }
    __device__ double Q_N(double a) const
    {
        const double t = 2.0 * half_int(a);
        return t * t * t / (4.0 * a * a);
    }
    __device__ double inv_half_int(double t) const        // smallest x with int_0^x p^(1/3) >= t
    {
        int lo = 0, hi = kNB;                              // smallest i with H[i+1] >= t
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (L.H[mid + 1] >= t) hi = mid; else lo = mid + 1;
        }
        if (lo >= kNB) return bin_hi(kNB - 1, absmax);
        return bin_lo(lo) + (t - L.H[lo]) / L.p13[lo];
    }
};

__global__ __launch_bounds__(kBlock) void tq_params_kernel(const tq_stats_t* __restrict__ stats, int bits,
                                                           int grid, float alpha_override,
                                                           tq_params_t* __restrict__ params)
{
    __shared__ ParamsLds L;
    const tq_stats_t* S = stats + blockIdx.x;
    const int tid = threadIdx.x;
    const double absmax = (double)S->absmax;

    for (int i = tid; i < kNB; i += kBlock) L.hist[i] = (double)S->hist[i];
    __syncthreads();

    if (tid == 0) {
        double c = 0.0;
        for (int i = 0; i < kNB; ++i) { L.cum[i] = c; c += L.hist[i]; }
        L.cum[kNB] = c;
        // Without a caller-fixed g_min the tail starts at the lower edge of the bin that
        // holds the 0.9-quantile of |g|.
        int tb = 0;
        double gm = 0.0;
        if (S->g_min > 0.0f) {
            gm = (double)S->g_min;
        } else if (c > 0.0) {
            tb = kNB - 1;
            for (int i = 0; i < kNB; ++i)
                if (10.0 * L.cum[i + 1] >= 9.0 * c) { tb = i; break; }
            gm = bin_lo(tb);                               // 0 when the quantile sits in bin 0
        }
        L.tail_bin = tb;
        L.g_min = gm;
    }
    __syncthreads();

    const double n = L.cum[kNB];
    const bool binned_tail = !(S->g_min > 0.0f) && L.g_min > 0.0;
    for (int i = tid; i < kNB; i += kBlock) {
        const double lo = bin_lo(i), hi = bin_hi(i, absmax);
        const double dens = n > 0.0 ? L.hist[i] / (2.0 * n * (hi - lo)) : 0.0;
        L.p13[i] = cbrt(dens);
        double t = 0.0;
        if (binned_tail && i >= L.tail_bin && L.hist[i] > 0.0) {
            const double rep = i < kNB - 1 ? sqrt(lo * hi) : lo;
            t = L.hist[i] * log(rep / L.g_min);
        }
        L.tl[i] = t;
    }
    __syncthreads();
    if (tid != 0) return;

    double h = 0.0;
    for (int i = 0; i < kNB; ++i) { L.H[i] = h; h += L.p13[i] * (bin_hi(i, absmax) - bin_lo(i)); }
    L.H[kNB] = h;
    const DensityView D{L, n, absmax};

    const int s = (1 << bits) - 1;
    uint32_t flags = 0;
    double g_min = 0.0, gamma = 0.0, rho = 0.0, alpha;
    if (n <= 0.0 || absmax <= 0.0) {
        flags |= TQ_F_DEGENERATE;
        alpha = kAlphaFloor;
    } else {
        double n_tail, sum_log;
        g_min = L.g_min;
        if (S->g_min > 0.0f) {
            n_tail = (double)S->n_tail;
            sum_log = S->sum_log_tail;
        } else {
            n_tail = g_min > 0.0 ? n - L.cum[L.tail_bin] : 0.0;
            sum_log = 0.0;
            for (int i = L.tail_bin; i < kNB; ++i) sum_log += L.tl[i];
            if (!(g_min > 0.0)) sum_log = 0.0;
        }
        const bool tail_ok = g_min > 0.0 && n_tail > 0.0 && sum_log > 0.0 && g_min < absmax;
        if (tail_ok) {
            gamma = 1.0 + n_tail / sum_log;
            rho = n_tail / (2.0 * n);
        }
        if (alpha_override != 0.0f) {
            flags |= TQ_F_ALPHA_OVERRIDE;
            alpha = alpha_override > 0.0f ? (double)alpha_override : absmax;
        } else if (!tail_ok) {
            flags |= TQ_F_DEGENERATE;
            alpha = absmax;
        } else {
            double gu = gamma;
            if (gu < kGammaFloor) { gu = kGammaFloor; flags |= TQ_F_GAMMA_CLAMPED; }
            const double a_min = g_min * (1.0 + 0.0009765625), a_max = absmax;
            const double C = 2.0 * rho * (double)(s * s) / (gu - 2.0);
            const double ex = 1.0 / (gu - 1.0);
            auto clampa = [&](double a) { a = a > a_min ? a : a_min; return a < a_max ? a : a_max; };
            double a = clampa(g_min * pow(C, ex));         // alpha' of Sec. IV-A (Q = 1)
            bool converged = false;
            for (int it = 0; it < kMaxIter; ++it) {
                const double q = grid == TQ_GRID_UNIFORM ? D.Q_U(a) : D.Q_N(a);
                const double an = q > 0.0 ? clampa(g_min * pow(C / q, ex)) : a_max;
                const bool done = fabs(an - a) <= kRelTol * an;
                a = an;
                if (done) { converged = true; break; }
            }
            if (!converged) flags |= TQ_F_NOT_CONVERGED;
            if (a >= a_max) flags |= TQ_F_ALPHA_CLAMPED_MAX;
            else if (a <= a_min) flags |= TQ_F_ALPHA_CLAMPED_MIN;
            alpha = a;
        }
    }

    tq_params_t* P = params + blockIdx.x;
    const float alpha_f = (float)(alpha > kAlphaFloor ? alpha : kAlphaFloor);
    const double af = (double)alpha_f;
    float lv[16];
    for (int k = 0; k < 16; ++k) lv[k] = 0.0f;
    const double half = D.half_int(af);
    if (grid == TQ_GRID_UNIFORM || !(half > 0.0)) {
        for (int k = 0; k <= s; ++k) lv[k] = (float)(-af + (double)k * (2.0 * af / (double)s));
        lv[s] = alpha_f;
    } else {
        lv[0] = -alpha_f;
        lv[s] = alpha_f;
        for (int k = (s + 1) / 2; k < s; ++k) {
            double x = D.inv_half_int(half * (double)(2 * k - s) / (double)s);
            x = x < af ? x : af;
            lv[k] = (float)x;
            lv[s - k] = -(float)x;
        }
    }
    P->alpha = alpha_f;
    P->bits = (uint32_t)bits;
    P->s = (uint32_t)s;
    P->grid = (uint32_t)grid;
    for (int k = 0; k < 16; ++k) {
        P->level[k] = lv[k];
        float iw = 0.0f;
        if (k < s) {
            if (grid == TQ_GRID_UNIFORM) {
                iw = (float)((double)s / (2.0 * af));
            } else {
                const double width = (double)lv[k + 1] - (double)lv[k];
                if (width > 0.0) {
                    const double r = 1.0 / width;
                    iw = r <= 3.4028234663852886e38 ? (float)r : 0.0f;
                }
            }
        }
        P->inv_w[k] = iw;
    }
    P->gamma_hat = (float)gamma;
    P->rho_hat = (float)rho;
    P->g_min = (float)g_min;
    P->flags = flags;
}

}  // namespace tq

// Host side of tq_params after the argument checks of the C entry point.
hipError_t tq_launch_params(const tq_stats_t* stats, uint64_t nb, int bits, int grid, float alpha_override,
                            tq_params_t* params, hipStream_t st)
{
    if (nb == 0 || nb > 0x7FFFFFFFull) return hipErrorInvalidValue;
    hipLaunchKernelGGL(tq::tq_params_kernel, dim3((unsigned)nb), dim3(tq::kBlock), 0, st, stats, bits, grid,
                       alpha_override, params);
    return hipGetLastError();
}
