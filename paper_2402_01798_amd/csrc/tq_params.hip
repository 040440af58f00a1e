// tq_params: parameter design of the truncated quantizer (arXiv 2402.01798, Sec. IV) from
// the per-bucket statistics, in fp64, one workgroup per bucket.
//
//   tail index      gamma = 1 + n_tail / sum ln(|g|/g_min)            (Sec. V, MLE)
//   tail mass       rho   = n_tail / (2 n)                            (one-sided, Sec. IV-A)
//   threshold       alpha = g_min [2 rho s^2 / ((gamma-2) Q(alpha))]^(1/(gamma-1)),
//                   Q = Q_U (Sec. IV-A, boxed) or Q_N (Sec. IV-B, second boxed equation)
//   codebook        uniform: l_k = -alpha + k 2alpha/s; non-uniform: the points where the
//                   integral of lambda_s ~ p^(1/3) (Sec. IV-B, first boxed equation) reaches k
//   BiScaled        (appendix "Truncated BiScaled Quantization") Q = min_k Q_B(alpha, k),
//                   Q_B = [(2 int_{k alpha}^{alpha} p)^(1/3) (1-k)^(2/3) + (2 int_0^{k alpha} p)^(1/3) k^(2/3)]^3,
//                   k over 0 and the bin edges below alpha; s_beta = the odd integer nearest to
//                   s p1^(1/3) k / (p2^(1/3) (1-k) + p1^(1/3) k) uniform cells on [-k alpha, k alpha],
//                   the other s - s_beta on the rest of [-alpha, alpha]
//
// The density p on [-alpha, alpha] is the histogram's (constant inside a bin).  With the
// prefix sums cum[i] = #{|g| below bin i} and H[i] = int_0^{lo_i} p^(1/3), both Q_U(alpha)
// and the integral of p^(1/3) up to alpha cost O(1) per evaluation.  The per-bin cube roots
// and logarithms and the two prefix sums are computed by all lanes (4 bins per lane, a
// wavefront scan, a 4-entry carry through LDS); only the fixed-point iteration itself, a
// chain of dependent scalar steps, runs on lane 0.  For the BiScaled family every step of that
// chain holds a minimum over up to 898 candidate k: there all lanes walk the chain together
// (each computing the same scalars) and share the search, 4 candidates per lane.
#include "tq_device.h"

namespace tq {

constexpr int kNB = TQ_NBINS;
constexpr int kBinsPerLane = 4;                           // 256 lanes x 4 >= 898 bins
constexpr double kGammaFloor = 2.02;
constexpr double kAlphaFloor = 5.421010862427522e-20;     // 2^-64
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
    if (x < 9.094947017729282e-13) return 0;              // 2^-40
    if (x >= 65536.0) return kNB - 1;
    const int ex = ilogb(x);
    const double m = ldexp(x, -ex);                        // in [1, 2), exact
    return (ex + 40) * 16 + (int)((m - 1.0) * 16.0) + 1;
}

struct ParamsLds {
    double hist[kNB];
    double cum[kNB + 1];   // cum[i] = sum of hist below bin i
    double p13[kNB];       // cube root of the two-sided density on the bin
    double H[kNB + 1];     // H[i] = int_0^{lo_i} p^(1/3)
    double carry[4];       // per-wavefront totals of the scan in flight
    double total;
    int tail_bin;
    double best_q[4];      // per-wavefront minimum of the BiScaled search and the bin it belongs to
    int best_j[4];
};

// Exclusive prefix sum over the 1024 (lane, slot) values v[0..3] of all 256 lanes, in bin
// order; returns each lane's offset and leaves the grand total in L.total.
__device__ __forceinline__ double block_exclusive_scan(double local, ParamsLds& L)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    double incl = local;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const double o = __shfl_up(incl, off, 64);
        if (lane >= off) incl += o;
    }
    __syncthreads();                                       // previous use of carry is over
    if (lane == 63) L.carry[wave] = incl;
    __syncthreads();
    double base = 0.0;
    for (int w = 0; w < wave; ++w) base += L.carry[w];
    if (threadIdx.x == kBlock - 1) L.total = base + incl;
    return base + incl - local;
}

struct DensityView {
    const ParamsLds& L;
    double n, inv_n, absmax;
    // Part of bin j below x, as a fraction of the bin (frac) and as a length (len).  The bins
    // between 2^-40 and 2^16 are 2^(octave-44) wide, so their reciprocal width is exact.
    __device__ void covered(int j, double x, double& frac, double& len) const
    {
        const double lo = bin_lo(j);
        double w, rw;
        if (j >= 1 && j < kNB - 1) {
            const int e = ((j - 1) >> 4) - 44;
            w = ldexp(1.0, e);
            rw = ldexp(1.0, -e);
        } else {
            w = bin_hi(j, absmax) - lo;
            rw = 1.0 / w;
        }
        double c = x - lo;
        c = c < 0.0 ? 0.0 : (c > w ? w : c);
        len = c;
        frac = c * rw;
    }
    __device__ double Q_U(double a) const
    {
        const int j = bin_of(a);
        double frac, len;
        covered(j, a, frac, len);
        return (L.cum[j] + L.hist[j] * frac) * inv_n;
    }
    __device__ double half_int(double x) const            // int_0^x p^(1/3)
    {
        const int j = bin_of(x);
        double frac, len;
        covered(j, x, frac, len);
        return L.H[j] + L.p13[j] * len;
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

__global__ __launch_bounds__(kBlock) void tq_params_kernel(const PtrTable stats_tab, uint32_t nb, int bits, int grid,
                                                           float alpha_override, const MutPtrTable params_tab)
{
    __shared__ ParamsLds L;
    // one workgroup per bucket, blockIdx.y = tensor of the batch
    const uint32_t bucket = linear_block();
    if (bucket >= nb) return;
    const tq_stats_t* S = static_cast<const tq_stats_t*>(stats_tab.p[blockIdx.y]) + bucket;
    tq_params_t* params = static_cast<tq_params_t*>(params_tab.p[blockIdx.y]);
    const int tid = threadIdx.x;
    const int i0 = tid * kBinsPerLane;
    const double absmax = (double)S->absmax;
    const bool fixed_gmin = S->g_min > 0.0f;

    // counts and their prefix sums
    double h[kBinsPerLane], local = 0.0;
#pragma unroll
    for (int k = 0; k < kBinsPerLane; ++k) {
        h[k] = (i0 + k < kNB) ? (double)S->hist[i0 + k] : 0.0;
        local += h[k];
    }
    double run = block_exclusive_scan(local, L);
    if (tid == 0) L.tail_bin = kNB;
    __syncthreads();
    const double n = L.total;
#pragma unroll
    for (int k = 0; k < kBinsPerLane; ++k) {
        if (i0 + k < kNB) { L.hist[i0 + k] = h[k]; L.cum[i0 + k] = run; }
        const double before = run;
        run += h[k];
        // Without a caller-fixed g_min the tail starts at the lower edge of the first bin at
        // which the cumulative count reaches the 0.9-quantile of |g|: exactly one bin has the
        // count below the mark before it and at or above the mark with it.
        if (i0 + k < kNB && n > 0.0 && 10.0 * before < 9.0 * n && 10.0 * run >= 9.0 * n) L.tail_bin = i0 + k;
    }
    if (tid == kBlock - 1) L.cum[kNB] = n;
    __syncthreads();

    int tail_bin = L.tail_bin;
    double g_min;
    if (fixed_gmin) { g_min = (double)S->g_min; tail_bin = kNB; }
    else if (tail_bin >= kNB) { g_min = 0.0; }
    else g_min = bin_lo(tail_bin);                         // 0 when the quantile sits in bin 0
    const bool binned_tail = !fixed_gmin && g_min > 0.0;

    // density^(1/3), its integral up to each bin, and the binned log-sum of the tail
    double pw[kBinsPerLane], local_h = 0.0, local_t = 0.0;
#pragma unroll
    for (int k = 0; k < kBinsPerLane; ++k) {
        const int i = i0 + k;
        pw[k] = 0.0;
        if (i < kNB) {
            const double lo = bin_lo(i), hi = bin_hi(i, absmax);
            const double dens = n > 0.0 ? h[k] / (2.0 * n * (hi - lo)) : 0.0;
            const double c = cbrt(dens);
            L.p13[i] = c;
            pw[k] = c * (hi - lo);
            if (binned_tail && i >= tail_bin && h[k] > 0.0) {
                const double rep = i < kNB - 1 ? sqrt(lo * hi) : lo;
                local_t += h[k] * log(rep / g_min);
            }
        }
        local_h += pw[k];
    }
    double runh = block_exclusive_scan(local_h, L);
#pragma unroll
    for (int k = 0; k < kBinsPerLane; ++k) {
        if (i0 + k < kNB) L.H[i0 + k] = runh;
        runh += pw[k];
    }
    __syncthreads();
    if (tid == kBlock - 1) L.H[kNB] = L.total;
    const double excl_t = block_exclusive_scan(local_t, L);
    (void)excl_t;
    __syncthreads();
    const double sum_log_binned = L.total;
    const bool biscaled = grid == TQ_GRID_BISCALED;
    if (!biscaled && tid != 0) return;                    // BiScaled: all lanes stay, in lockstep

    const DensityView D{L, n, n > 0.0 ? 1.0 / n : 0.0, absmax};

    // BiScaled search, collective: the edge lo_j < a (j = 0: beta = 0) that minimises Q_B(a, lo_j / a),
    // the smallest such edge on a tie; returns Q_B and leaves the bin in best_bin.  Each lane keeps,
    // for its 4 bins, the parts that do not depend on a: (mass below the edge)^(1/3), edge^(2/3).
    double cb13[kBinsPerLane], lo23[kBinsPerLane], lo_e[kBinsPerLane], cb[kBinsPerLane];
    if (biscaled) {
#pragma unroll
        for (int k = 0; k < kBinsPerLane; ++k) {
            const int j = i0 + k;
            lo_e[k] = j < kNB ? bin_lo(j) : 0.0;
            cb[k] = j < kNB ? L.cum[j] * D.inv_n : 0.0;
            cb13[k] = cbrt(cb[k]);
            lo23[k] = cbrt(lo_e[k] * lo_e[k]);
        }
    }
    int best_bin = 0;
    auto biscaled_min = [&](double a) -> double {
        const double c_a = D.Q_U(a);
        const double inv_a = 1.0 / a, inv_a23 = 1.0 / cbrt(a * a);
        double q = 1.0e300;
        int jbest = kNB;
#pragma unroll
        for (int k = 0; k < kBinsPerLane; ++k) {
            const int j = i0 + k;
            if (j < kNB && (j == 0 || lo_e[k] < a)) {
                const double kk = lo_e[k] * inv_a;
                double outer = c_a - cb[k];
                outer = outer > 0.0 ? outer : 0.0;
                const double r = 1.0 - kk;
                const double v = cbrt(outer) * cbrt(r * r) + cb13[k] * (lo23[k] * inv_a23);
                if (v < q) { q = v; jbest = j; }          // ascending j: the first minimum stays
            }
        }
        const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const double oq = __shfl_xor(q, off, 64);
            const int oj = __shfl_xor(jbest, off, 64);
            if (oq < q || (oq == q && oj < jbest)) { q = oq; jbest = oj; }
        }
        __syncthreads();                                   // the previous search has been read
        if (lane == 0) { L.best_q[wave] = q; L.best_j[wave] = jbest; }
        __syncthreads();
        q = L.best_q[0];
        jbest = L.best_j[0];
#pragma unroll
        for (int w = 1; w < 4; ++w) {
            const double oq = L.best_q[w];
            const int oj = L.best_j[w];
            if (oq < q || (oq == q && oj < jbest)) { q = oq; jbest = oj; }
        }
        best_bin = jbest;
        return q * q * q;
    };

    const int s = (1 << bits) - 1;
    uint32_t flags = 0;
    double gamma = 0.0, rho = 0.0, alpha;
    if (n <= 0.0 || absmax <= 0.0) {
        // nothing finite and non-zero to design from; a threshold the caller gives is still honoured
        flags |= TQ_F_DEGENERATE;
        alpha = kAlphaFloor;
        if (alpha_override > 0.0f) { flags |= TQ_F_ALPHA_OVERRIDE; alpha = (double)alpha_override; }
        g_min = 0.0;
    } else {
        double n_tail, sum_log;
        if (fixed_gmin) {
            n_tail = (double)S->n_tail;
            sum_log = S->sum_log_tail;
        } else {
            n_tail = g_min > 0.0 ? n - L.cum[tail_bin] : 0.0;
            sum_log = g_min > 0.0 ? sum_log_binned : 0.0;
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
            const double log_c = log(C);
            auto clampa = [&](double a) { a = a > a_min ? a : a_min; return a < a_max ? a : a_max; };
            double a = clampa(g_min * exp(ex * log_c));    // alpha' of Sec. IV-A (Q = 1)
            bool converged = false;
            for (int it = 0; it < kMaxIter; ++it) {
                const double q = grid == TQ_GRID_UNIFORM ? D.Q_U(a) : (biscaled ? biscaled_min(a) : D.Q_N(a));
                // (C/q)^ex evaluated as exp(ex (ln C - ln q))
                const double an = q > 0.0 ? clampa(g_min * exp(ex * (log_c - log(q)))) : a_max;
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

    tq_params_t* P = params + bucket;
    const float alpha_f = (float)(alpha > kAlphaFloor ? alpha : kAlphaFloor);
    const double af = (double)alpha_f;
    const double half = D.half_int(af);
    if (biscaled) {
        if (half > 0.0) (void)biscaled_min(af);            // the split belongs to the rounded threshold
        if (tid != 0) return;
    }
    float lv[16];
    for (int k = 0; k < 16; ++k) lv[k] = 0.0f;
    if (grid == TQ_GRID_UNIFORM || !(half > 0.0) || (biscaled && best_bin == 0)) {
        for (int k = 0; k <= s; ++k) lv[k] = (float)(-af + (double)k * (2.0 * af / (double)s));
        lv[s] = alpha_f;
    } else if (biscaled) {
        const double beta = bin_lo(best_bin), kk = beta / af;
        const double c_b = L.cum[best_bin] * D.inv_n, c_a = D.Q_U(af);
        const double p1 = c_b / (2.0 * beta);
        const double rest = c_a - c_b > 0.0 ? c_a - c_b : 0.0;
        const double p2 = rest / (2.0 * (af - beta));
        const double inner = cbrt(p1) * kk, outer = cbrt(p2) * (1.0 - kk);
        const double x = inner + outer > 0.0 ? (double)s * inner / (inner + outer) : (double)s;
        int s_beta = 2 * (int)floor((x - 1.0) * 0.5 + 0.5) + 1;           // nearest odd integer
        s_beta = s_beta < 1 ? 1 : (s_beta > s - 2 ? s - 2 : s_beta);
        const int h = (s - s_beta) / 2;                                    // cells beyond beta on each side
        for (int j = 0; j <= s_beta; ++j) lv[h + j] = (float)(-beta + (double)j * (2.0 * beta / (double)s_beta));
        lv[h] = (float)(-beta);
        lv[h + s_beta] = (float)beta;
        for (int j = 1; j <= h; ++j) {
            const double xo = beta + (double)j * ((af - beta) / (double)h);
            lv[h + s_beta + j] = (float)xo;
            lv[h - j] = -(float)xo;
        }
        lv[0] = -alpha_f;
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

// Host side of tq_params / tq_params_multi after the argument checks of the C entry points.
hipError_t tq_launch_params(const tq_stats_t* const* stats, int count, uint64_t nb, int bits, int grid,
                            float alpha_override, tq_params_t* const* params, hipStream_t st)
{
    dim3 blocks;
    if (count < 1 || count > tq::kMaxBatch || !tq::fold_grid(nb, tq::kBlock, (unsigned)count, blocks))
        return hipErrorInvalidValue;
    tq::PtrTable stt{};
    tq::MutPtrTable pt{};
    for (int i = 0; i < count; ++i) { stt.p[i] = stats[i]; pt.p[i] = params[i]; }
    hipLaunchKernelGGL(tq::tq_params_kernel, blocks, dim3(tq::kBlock), 0, st, stt, (uint32_t)nb, bits,
                       grid, alpha_override, pt);
    return hipGetLastError();
}
