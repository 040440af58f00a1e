/*
 * tq_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * A slow, scalar, obviously-correct CPU statement of what the truncated
 * quantizer's data-parallel path computes.  Only the tests, the smoke check
 * and the benchmark's cpu_baseline leg may call it; the GPU library never
 * does and shares no source, header, table or helper with this file.
 *
 * Every function walks the elements one by one in the order and notation of
 * the paper (arXiv 2402.01798):
 *   tqo_truncate            Sec. III-A, Eq. (1)   alpha-truncation T_alpha
 *   tqo_quantize_eq2        Sec. III-A, Eq. (2)   stochastic quantizer Q on a
 *                           codebook L = {l_0..l_s}, s = 2^b - 1, step by step:
 *                           cell by comparison with the levels, p_r, the draw
 *   tqo_quantize_one        the code the wire format specifies: Eq. (2) as above on
 *                           every codebook but the uniform one, where the format
 *                           states the same rounding through the position of g in
 *                           units of cells (see below)
 *   tqo_compress            Alg. 1, client step "quantize, send"
 *   tqo_decompress_aggregate Alg. 1, server step  g_bar = sum_i w_i g_hat_i
 *   tqo_decompress_aggregate_update  ... followed by theta <- theta - eta g_bar
 *   tqo_stats               Sec. V (MLE of the tail index), Sec. IV (rho,
 *                           Q_U, integral of p^(1/3)): the raw reductions
 *   tqo_*_segments          the same three steps with one (alpha, codebook) per
 *                           variable-size segment (Sec. V: layers quantized independently)
 * The parameter design of Sec. IV (alpha fixed points, level tables) lives in
 * params.py beside this file, in fp64.
 *
 * Precision: the paper fixes none.  The quantizer's decision "round up or
 * down" yields an integer code, so it is taken in the precision of the
 * kernel under test: IEEE-754 binary32, one rounding per written operation
 * (build with -ffp-contract=off), no division on the per-element path: the
 * quotient of Eq. (2) uses the stored reciprocal of the cell's width.
 * Reductions compared by tolerance (sum of logs) run in binary64.
 *
 * What the paper leaves open and this file fixes (readings, listed in the
 * design document as well):
 *   - "with probability p_r" (Eq. 2): a 16-bit uniform integer r drawn from
 *     the counter-based generator Philox4x32-10 (Salmon, Moraes, Dror, Shaw,
 *     SC'11) gives the uniform variate u = 1 - (r + 1/2) / 2^16 (exact in
 *     binary32), and the upper end of the cell is taken iff u <= p_r: with
 *     probability p_r to within 2^-16, a larger r never lowering the code.
 *   - the uniform codebook (Sec. IV-A, l_k = -alpha + k 2alpha/s): there
 *     Eq. (2) is stochastic rounding of the position t = (g + alpha) s/(2 alpha),
 *     code = floor(t + U), U = (r + 1/2) / 2^16, and that is how the format
 *     states it, with t + U evaluated by two fused multiply-adds (fmaf: one
 *     rounding each).  tqo_quantize_eq2 is the definition it has to agree with:
 *     the tests enumerate all 65,536 draws for inputs on, next to and between
 *     the levels and require the same cell and the same number of upward
 *     draws to within one.
 *   - "encode using b bits": codes are laid into one little-endian bit
 *     stream, element e at bits [e*b, e*b+b), padded with zero bits to a
 *     multiple of 16 bytes.
 *   - a value lying exactly on a level belongs to the cell above it
 *     (frac = 0, deterministic); NaN is encoded as +0, +-Inf as +-alpha.
 *
 * Parity unpinned by the paper: the bit order of the payload, the assignment
 * of generator words to elements, the histogram's bin edges and the momentum
 * recursion of the fused update are this build's own definitions; the tests
 * pin them against independent readers (numpy.unpackbits, numpy.histogram,
 * hand-computed dyadic values), not against anything the paper prints.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#define TQO_NBINS 898 /* 1 underflow + 56 octaves x 16 + 1 overflow */
#define TQO_BIN_BIAS 1391 /* (biased exponent of 2^-40) * 16 - 1 */

enum { TQO_OK = 0, TQO_EINVAL = 1 };
enum { TQO_F32 = 0, TQO_BF16 = 1 };
enum { TQO_GRID_UNIFORM = 0, TQO_GRID_NONUNIFORM = 1 };

/* Same byte layout as the library's interface structs (an interface has to
 * be alike on both sides); declared here independently. */
typedef struct {
    uint32_t hist[TQO_NBINS];
    uint32_t n_nonfinite;
    float absmax;
    uint64_t n;
    float g_min;
    uint32_t reserved;
    uint64_t n_tail;
    double sum_log_tail;
} tqo_stats_t;

typedef struct {
    float alpha;
    uint32_t bits, s, grid;
    float level[16];
    float inv_w[16];
    float gamma_hat, rho_hat, g_min;
    uint32_t flags;
} tqo_params_t;

/* ------------------------------------------------------------------ RNG -- */

/* Philox4x32 with R rounds: the published round function is two 32x32->64
 * multiplications by fixed odd constants whose halves are crossed over and
 * xored with the round key; the key advances by a Weyl constant per round. */
void tqo_philox4x32(const uint32_t ctr[4], const uint32_t key[2], int rounds,
                    uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int r = 0; r < rounds; ++r) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The 16 random bits of element e of one worker's flat gradient in one step.
 * One generator call serves the 8 elements that share e >> 3: counter =
 * (low, high word of e >> 3, worker, step), key = the 64-bit seed; element
 * e & 7 = j takes word j >> 1, low half for even j, high half for odd j. */
uint32_t tqo_rand16(uint64_t seed, uint32_t worker, uint32_t step, uint64_t e)
{
    uint64_t q = e >> 3;
    uint32_t ctr[4] = { (uint32_t)q, (uint32_t)(q >> 32), worker, step };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t w[4];
    tqo_philox4x32(ctr, key, 10, w);
    unsigned j = (unsigned)(e & 7);
    return (w[j >> 1] >> (16 * (j & 1))) & 0xFFFFu;
}

/* ------------------------------------------------------- element helpers -- */

static float load_elem(const void *g, int dtype, uint64_t e)
{
    if (dtype == TQO_F32) return ((const float *)g)[e];
    uint32_t bits = (uint32_t)((const uint16_t *)g)[e] << 16; /* bf16 widens exactly */
    float x;
    memcpy(&x, &bits, 4);
    return x;
}

/* Eq. (1): T_alpha[g] = g for |g| <= alpha, sgn(g) * alpha otherwise. */
float tqo_truncate(float g, float alpha)
{
    if (g > alpha) return alpha;
    if (g < -alpha) return -alpha;
    return g;
}

/* Eq. (2), step by step, on the codebook P->level[0..s] with the 16-bit draw r:
 *   the cell Delta_k = [l_k, l_{k+1}] that holds the truncated value (a value on a
 *   level belongs to the cell above it; the last cell is closed),
 *   p_r = (g - l_k) / |Delta_k|   (the quotient through the stored reciprocal),
 *   the upper end l_{k+1} with probability p_r, else l_k.
 * Returns the index of the level chosen (the b-bit code).  Valid for any codebook. */
uint32_t tqo_quantize_eq2(float g, const tqo_params_t *P, uint32_t r)
{
    const uint32_t s = P->s;
    float x = g;
    if (x != x) x = 0.0f;                       /* NaN carries no information */
    const float xc = tqo_truncate(x, P->alpha); /* Eq. (1) */
    uint32_t k = 0;                             /* l_k <= xc < l_{k+1} */
    for (uint32_t j = 1; j < s; ++j)
        if (xc >= P->level[j]) k = j;
    const float dist = xc - P->level[k];        /* g - l_k */
    const float p_r = dist * P->inv_w[k];       /* ... / |Delta_k| */
    const float half_grain = 1.0f / 131072.0f;
    const float u = (1.0f - half_grain) - (float)r * (1.0f / 65536.0f);  /* 1 - (r + 1/2)/2^16, exact */
    return (u <= p_r) ? k + 1u : k;
}

/* The code the wire format specifies for element value g and draw r. */
uint32_t tqo_quantize_one(float g, const tqo_params_t *P, uint32_t r)
{
    if (P->grid != TQO_GRID_UNIFORM) return tqo_quantize_eq2(g, P, r);
    /* uniform codebook: all cells have width 2 alpha / s, and Eq. (2) is stochastic
     * rounding of the position of g in units of cells, counted from -alpha:
     * floor(t + U), U = (r + 1/2) / 2^16 uniform on (0, 1) */
    const uint32_t s = P->s;
    float x = g;
    if (x != x) x = 0.0f;
    const float xc = tqo_truncate(x, P->alpha);
    const float t_plus_half_grain = fmaf(xc, P->inv_w[0], 0.5f * (float)s + 1.0f / 131072.0f);
    const float v = fmaf((float)r, 1.0f / 65536.0f, t_plus_half_grain);
    uint32_t code = (uint32_t)v;                /* v >= 0: truncation is floor */
    if (code > s) code = s;
    return code;
}

/* How many of the 65,536 draws give each code, for one value g: count[c] for c = 0..s.
 * form 0: tqo_quantize_one, form 1: tqo_quantize_eq2.  For the tests that enumerate
 * Lemma 1 and compare the two statements of the uniform codebook. */
void tqo_enumerate_draws(float g, const tqo_params_t *P, int form, uint32_t count[16])
{
    for (int c = 0; c < 16; ++c) count[c] = 0;
    for (uint32_t r = 0; r < 65536u; ++r) {
        uint32_t code = form ? tqo_quantize_eq2(g, P, r) : tqo_quantize_one(g, P, r);
        count[code & 15u]++;
    }
}

/* --------------------------------------------------------------- layout -- */

static uint64_t bucket_of(uint64_t e, uint64_t bucket_elems)
{
    return bucket_elems ? e / bucket_elems : 0;
}

uint64_t tqo_num_buckets(uint64_t d, uint64_t bucket_elems)
{
    if (bucket_elems == 0 || d == 0) return d ? 1 : 0;
    return (d + bucket_elems - 1) / bucket_elems;
}

uint64_t tqo_payload_bytes(uint64_t d, int bits)
{
    uint64_t nbytes = (d * (uint64_t)bits + 7) / 8;
    return (nbytes + 15) / 16 * 16;
}

static int check_layout(uint64_t d, uint64_t bucket_elems)
{
    if (d == 0) return TQO_EINVAL;
    if (bucket_elems != 0 && bucket_elems % 128 != 0) return TQO_EINVAL;
    return TQO_OK;
}

/* ---------------------------------------------------------------- stats -- */

/* Histogram bin of a finite magnitude a: bin 0 holds [0, 2^-40); bins 1..896
 * split each octave of [2^-40, 2^16) into 16 equal parts (exponent and top
 * four mantissa bits); bin 897 holds [2^16, inf). */
uint32_t tqo_bin(float a)
{
    uint32_t bits;
    memcpy(&bits, &a, 4);
    int32_t idx = (int32_t)((bits & 0x7FFFFFFFu) >> 19) - TQO_BIN_BIAS;
    if (idx < 0) idx = 0;
    if (idx > TQO_NBINS - 1) idx = TQO_NBINS - 1;
    return (uint32_t)idx;
}

/* Per bucket: what the formulas of Sec. IV and the tail-index estimator of
 * Sec. V consume.  The histogram of |g| stands for the empirical density p
 * (Q_U(alpha) is its CDF, the integral of p^(1/3) a sum over bins); n_tail
 * and sum_log_tail are the two terms of gamma = 1 + n / sum_j ln(g_j/g_min)
 * over |g_j| > g_min (computed only when the caller supplies g_min > 0). */
int tqo_stats_buckets(const void *g, int dtype, uint64_t d, uint64_t bucket_elems,
                      float g_min, tqo_stats_t *stats, uint64_t b_begin, uint64_t b_end)
{
    if (check_layout(d, bucket_elems) || (dtype != TQO_F32 && dtype != TQO_BF16))
        return TQO_EINVAL;
    const uint64_t nb = tqo_num_buckets(d, bucket_elems);
    if (b_begin > b_end || b_end > nb) return TQO_EINVAL;
    for (uint64_t b = b_begin; b < b_end; ++b) {
        tqo_stats_t *S = &stats[b];
        memset(S, 0, sizeof *S);
        const uint64_t lo = b * bucket_elems;
        const uint64_t hi = (bucket_elems && lo + bucket_elems < d) ? lo + bucket_elems : d;
        S->n = hi - lo;
        S->g_min = g_min > 0.0f ? g_min : 0.0f;
        double sum_log = 0.0;
        for (uint64_t e = lo; e < hi; ++e) {
            float a = fabsf(load_elem(g, dtype, e));
            if (!(a <= 3.402823466e38f)) { S->n_nonfinite++; continue; } /* NaN or Inf */
            S->hist[tqo_bin(a)]++;
            if (a > S->absmax) S->absmax = a;
            if (g_min > 0.0f && a > g_min) {
                S->n_tail++;
                sum_log += log((double)a / (double)g_min);
            }
        }
        S->sum_log_tail = sum_log;
    }
    return TQO_OK;
}

/* All buckets; tqo_stats_buckets does the buckets [b_begin, b_end) only (disjoint
 * ranges may run on different host threads). */
int tqo_stats(const void *g, int dtype, uint64_t d, uint64_t bucket_elems,
              float g_min, tqo_stats_t *stats)
{
    return tqo_stats_buckets(g, dtype, d, bucket_elems, g_min, stats, 0,
                             tqo_num_buckets(d, bucket_elems));
}

/* ------------------------------------------------------------- compress -- */

/* Alg. 1, client side: g_hat = Q[T_alpha(g)] element by element, each code
 * written into the b-bit little-endian stream.  params[bucket] holds alpha
 * and the codebook of the bucket the element lies in.
 * tqo_compress_range encodes the elements [e_begin, e_end) only, into a payload the
 * caller has cleared; e_begin is a multiple of 8 (8 codes are whole bytes), so that
 * disjoint ranges touch disjoint bytes and may be encoded by different host threads. */
int tqo_compress_range(const void *g, int dtype, uint64_t d, uint64_t bucket_elems,
                       const tqo_params_t *params, uint64_t seed, uint32_t worker,
                       uint32_t step, uint8_t *payload, uint64_t e_begin, uint64_t e_end)
{
    if (check_layout(d, bucket_elems) || (dtype != TQO_F32 && dtype != TQO_BF16))
        return TQO_EINVAL;
    const uint32_t bits = params[0].bits;
    if (bits < 2 || bits > 4) return TQO_EINVAL;
    if (e_begin % 8 != 0 || e_begin > e_end || e_end > d) return TQO_EINVAL;
    for (uint64_t e = e_begin; e < e_end; ++e) {
        const tqo_params_t *P = &params[bucket_of(e, bucket_elems)];
        if (P->bits != bits || P->s != (1u << bits) - 1u) return TQO_EINVAL;
        uint32_t r = tqo_rand16(seed, worker, step, e);
        uint32_t code = tqo_quantize_one(load_elem(g, dtype, e), P, r);
        uint64_t bitpos = e * bits;
        for (uint32_t t = 0; t < bits; ++t, ++bitpos)
            if ((code >> t) & 1u) payload[bitpos >> 3] |= (uint8_t)(1u << (bitpos & 7));
    }
    return TQO_OK;
}

int tqo_compress(const void *g, int dtype, uint64_t d, uint64_t bucket_elems,
                 const tqo_params_t *params, uint64_t seed, uint32_t worker,
                 uint32_t step, uint8_t *payload)
{
    if (check_layout(d, bucket_elems)) return TQO_EINVAL;
    const uint32_t bits = params[0].bits;
    if (bits < 2 || bits > 4) return TQO_EINVAL;
    memset(payload, 0, tqo_payload_bytes(d, (int)bits));
    return tqo_compress_range(g, dtype, d, bucket_elems, params, seed, worker, step, payload, 0, d);
}

static uint32_t read_code(const uint8_t *payload, uint64_t e, uint32_t bits)
{
    uint32_t code = 0;
    uint64_t bitpos = e * bits;
    for (uint32_t t = 0; t < bits; ++t, ++bitpos)
        code |= (uint32_t)((payload[bitpos >> 3] >> (bitpos & 7)) & 1u) << t;
    return code;
}

/* ----------------------------------------------------------- aggregate -- */

/* Alg. 1, server side: g_bar[e] = sum_i w_i * L_i[code_i(e)].
 * weights == NULL is the analysis' w_i = 1/N: levels are added in worker
 * order 0..N-1 in binary32 and the sum is multiplied once by (float)(1/N).
 * With weights, each term is w_i * L_i[c] (one rounding) and the terms are
 * added in worker order.  accumulate != 0 adds the result to out[e]. */
static int aggregate_one(const uint8_t *const *payload,
                         const tqo_params_t *const *params, const float *weights,
                         int N, uint64_t e, uint64_t bucket_elems, int bits,
                         float *g_bar)
{
    const uint64_t b = bucket_of(e, bucket_elems);
    const float w_uniform = 1.0f / (float)N;
    float acc = 0.0f;
    for (int i = 0; i < N; ++i) {
        const tqo_params_t *P = &params[i][b];
        if ((int)P->bits != bits) return TQO_EINVAL;
        float term = P->level[read_code(payload[i], e, (uint32_t)bits)];
        if (weights) term = weights[i] * term;
        acc = (i == 0) ? term : acc + term;
    }
    if (!weights) acc = acc * w_uniform;
    *g_bar = acc;
    return TQO_OK;
}

/* Elements [e_begin, e_end) only (disjoint ranges may run on different host threads). */
int tqo_decompress_aggregate_range(const uint8_t *const *payload,
                                   const tqo_params_t *const *params,
                                   const float *weights, int N, uint64_t d,
                                   uint64_t bucket_elems, int bits, int accumulate,
                                   float *out, uint64_t e_begin, uint64_t e_end)
{
    if (check_layout(d, bucket_elems) || N < 1 || bits < 2 || bits > 4)
        return TQO_EINVAL;
    if (e_begin > e_end || e_end > d) return TQO_EINVAL;
    for (uint64_t e = e_begin; e < e_end; ++e) {
        float acc;
        if (aggregate_one(payload, params, weights, N, e, bucket_elems, bits, &acc))
            return TQO_EINVAL;
        out[e] = accumulate ? out[e] + acc : acc;
    }
    return TQO_OK;
}

int tqo_decompress_aggregate(const uint8_t *const *payload,
                             const tqo_params_t *const *params,
                             const float *weights, int N, uint64_t d,
                             uint64_t bucket_elems, int bits, int accumulate,
                             float *out)
{
    return tqo_decompress_aggregate_range(payload, params, weights, N, d, bucket_elems, bits,
                                          accumulate, out, 0, d);
}

/* Alg. 1, the two server steps together: g_bar = sum_i w_i g_hat_i as above,
 * then theta <- theta - eta * g_bar.  The experiments of Sec. V train with
 * momentum SGD and weight decay; the paper does not write that recursion out,
 * so the common form is taken (a reading):
 *     u     = g_bar + weight_decay * theta     (u = g_bar when weight_decay == 0)
 *     v     = momentum * v + u                 (only when a velocity is kept)
 *     theta = theta - eta * v                  (theta - eta * u without velocity)
 * every product and sum rounded once to binary32, in this order.
 * velocity == NULL means plain SGD, the update Alg. 1 states. */
int tqo_decompress_aggregate_update(const uint8_t *const *payload,
                                    const tqo_params_t *const *params,
                                    const float *weights, int N, uint64_t d,
                                    uint64_t bucket_elems, int bits, float eta,
                                    float momentum, float weight_decay,
                                    float *theta, float *velocity)
{
    if (check_layout(d, bucket_elems) || N < 1 || bits < 2 || bits > 4)
        return TQO_EINVAL;
    for (uint64_t e = 0; e < d; ++e) {
        float g_bar;
        if (aggregate_one(payload, params, weights, N, e, bucket_elems, bits, &g_bar))
            return TQO_EINVAL;
        float u = g_bar;
        if (weight_decay != 0.0f) {
            const float decay = weight_decay * theta[e];
            u = g_bar + decay;
        }
        if (velocity) {
            const float carried = momentum * velocity[e];
            u = carried + u;
            velocity[e] = u;
        }
        const float step = eta * u;
        theta[e] = theta[e] - step;
    }
    return TQO_OK;
}

/* Level values of one worker's stream, element by element (Q[T_alpha(g)] as
 * the server sees it); used by the statistical pins. */
int tqo_dequantize(const uint8_t *payload, const tqo_params_t *params,
                   uint64_t d, uint64_t bucket_elems, int bits, float *out)
{
    if (check_layout(d, bucket_elems) || bits < 2 || bits > 4) return TQO_EINVAL;
    for (uint64_t e = 0; e < d; ++e)
        out[e] = params[bucket_of(e, bucket_elems)].level[read_code(payload, e, (uint32_t)bits)];
    return TQO_OK;
}


/* ---------------------------------------------------- variable-size segments -- */

/* Sec. V quantizes the layers of a network independently ("per layer type"): here the flat
 * gradient is cut at seg_offsets[0] = 0 < seg_offsets[1] < ... < seg_offsets[nseg] = d into
 * nseg segments (interior offsets multiples of 128), each with its own statistics record and
 * its own (alpha, codebook).  Everything else is as in the bucketed functions above: the
 * element index that keys the random draws and the bit position in the payload are those of
 * the flat gradient. */
static int check_segments(uint64_t d, const uint64_t *off, uint64_t nseg)
{
    if (d == 0 || nseg == 0 || off[0] != 0 || off[nseg] != d) return TQO_EINVAL;
    for (uint64_t s = 0; s < nseg; ++s) {
        if (off[s + 1] <= off[s]) return TQO_EINVAL;
        if (s + 1 < nseg && off[s + 1] % 128 != 0) return TQO_EINVAL;
    }
    return TQO_OK;
}

int tqo_stats_segments(const void *g, int dtype, uint64_t d, const uint64_t *seg_offsets,
                       uint64_t nseg, float g_min, tqo_stats_t *stats)
{
    if (check_segments(d, seg_offsets, nseg) || (dtype != TQO_F32 && dtype != TQO_BF16))
        return TQO_EINVAL;
    const size_t esz = dtype == TQO_F32 ? 4 : 2;
    for (uint64_t s = 0; s < nseg; ++s) {
        /* a segment on its own is a tensor with one bucket */
        const uint64_t lo = seg_offsets[s], n = seg_offsets[s + 1] - lo;
        if (tqo_stats((const char *)g + lo * esz, dtype, n, 0, g_min, &stats[s])) return TQO_EINVAL;
    }
    return TQO_OK;
}

int tqo_compress_segments(const void *g, int dtype, uint64_t d, const uint64_t *seg_offsets,
                          uint64_t nseg, const tqo_params_t *params, uint64_t seed,
                          uint32_t worker, uint32_t step, uint8_t *payload)
{
    if (check_segments(d, seg_offsets, nseg) || (dtype != TQO_F32 && dtype != TQO_BF16))
        return TQO_EINVAL;
    const uint32_t bits = params[0].bits;
    if (bits < 2 || bits > 4) return TQO_EINVAL;
    memset(payload, 0, tqo_payload_bytes(d, (int)bits));
    for (uint64_t s = 0; s < nseg; ++s) {
        const tqo_params_t *P = &params[s];
        if (P->bits != bits || P->s != (1u << bits) - 1u) return TQO_EINVAL;
        for (uint64_t e = seg_offsets[s]; e < seg_offsets[s + 1]; ++e) {
            uint32_t r = tqo_rand16(seed, worker, step, e);
            uint32_t code = tqo_quantize_one(load_elem(g, dtype, e), P, r);
            uint64_t bitpos = e * bits;
            for (uint32_t t = 0; t < bits; ++t, ++bitpos)
                if ((code >> t) & 1u) payload[bitpos >> 3] |= (uint8_t)(1u << (bitpos & 7));
        }
    }
    return TQO_OK;
}

int tqo_decompress_aggregate_segments(const uint8_t *const *payload,
                                      const tqo_params_t *const *params, const float *weights,
                                      int N, uint64_t d, const uint64_t *seg_offsets,
                                      uint64_t nseg, int bits, int accumulate, float *out)
{
    if (check_segments(d, seg_offsets, nseg) || N < 1 || bits < 2 || bits > 4) return TQO_EINVAL;
    const float w_uniform = 1.0f / (float)N;
    for (uint64_t s = 0; s < nseg; ++s) {
        for (uint64_t e = seg_offsets[s]; e < seg_offsets[s + 1]; ++e) {
            float acc = 0.0f;
            for (int i = 0; i < N; ++i) {
                const tqo_params_t *P = &params[i][s];
                if ((int)P->bits != bits) return TQO_EINVAL;
                float term = P->level[read_code(payload[i], e, (uint32_t)bits)];
                if (weights) term = weights[i] * term;
                acc = (i == 0) ? term : acc + term;
            }
            if (!weights) acc = acc * w_uniform;
            out[e] = accumulate ? out[e] + acc : acc;
        }
    }
    return TQO_OK;
}

size_t tqo_sizeof_stats(void) { return sizeof(tqo_stats_t); }
size_t tqo_sizeof_params(void) { return sizeof(tqo_params_t); }
