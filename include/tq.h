/*
 * tq.h -- C ABI of the truncated quantizer for heavy-tailed gradients
 *         (arXiv 2402.01798) on AMD MI355X (gfx950).
 *
 * The four calls follow the paper's statement of the problem: a worker designs
 * the two parameters of its quantizer from the statistics of its gradient
 * (Sec. IV), sends Q[T_alpha(g)] in b bits per element (Sec. III-A, Alg. 1
 * client step), and the server averages what the N workers sent (Alg. 1
 * server step).
 *
 * Conventions shared by every call
 *   - Pointers named *_dev are device (HBM) pointers, 16-byte aligned, owned
 *     by the caller; the library never allocates, frees or keeps them.
 *   - Pointers named *_host are host memory, read before the call returns.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Work is enqueued asynchronously; no call synchronises the stream.
 *   - Return value: TQ_OK or an error code; nothing is enqueued on error.
 *     A bad argument is TQ_EINVAL, a misaligned pointer TQ_EALIGN, a size the
 *     kernels do not cover TQ_EUNSUPPORTED, a failed launch TQ_EHIP.
 *   - d = elements in one worker's flat gradient (d >= 1).  bucket_elems = 0
 *     means one bucket spanning the tensor; otherwise consecutive buckets of
 *     bucket_elems elements (a multiple of 128), the last possibly short.
 *     There is one tq_stats_t and one tq_params_t per bucket.
 */
#ifndef TQ_H
#define TQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { TQ_OK = 0, TQ_EINVAL = 1, TQ_EALIGN = 2, TQ_EUNSUPPORTED = 3, TQ_EHIP = 4 };
enum { TQ_F32 = 0, TQ_BF16 = 1 };                      /* gradient dtype */
enum { TQ_GRID_UNIFORM = 0, TQ_GRID_NONUNIFORM = 1, TQ_GRID_BISCALED = 2 };  /* codebook family */

#define TQ_NBINS 898        /* histogram bins of |g|, see tq_stats */
#define TQ_MAX_WORKERS 64   /* largest N of tq_decompress_aggregate */

/* tq_params_t.flags */
#define TQ_F_ALPHA_CLAMPED_MAX 1u  /* fixed point at or beyond max|g|: alpha = max|g| */
#define TQ_F_GAMMA_CLAMPED     2u  /* tail index estimate below 2.02, lifted to it   */
#define TQ_F_NOT_CONVERGED     4u  /* 100 iterations without meeting 1e-10           */
#define TQ_F_DEGENERATE        8u  /* no finite non-zero data (alpha = 2^-64 unless the
                                      caller gave one), or no usable tail (alpha = max|g|) */
#define TQ_F_ALPHA_OVERRIDE   16u  /* alpha given by the caller                       */
#define TQ_F_ALPHA_CLAMPED_MIN 32u /* fixed point at or below g_min, lifted           */

/* Per-bucket statistics of |g| (3632 bytes).  The integer fields are exact. */
typedef struct {
    uint32_t hist[TQ_NBINS]; /* bin 0: [0,2^-40); bins 1..896: sixteenths of the octaves
                                of [2^-40,2^16); bin 897: [2^16,inf).  Finite values only. */
    uint32_t n_nonfinite;    /* NaN and +-Inf seen (left out of every other field)     */
    float    absmax;         /* largest finite |g|                                      */
    uint64_t n;              /* elements in the bucket                                  */
    float    g_min;          /* the g_min given to tq_stats, 0 if none                  */
    uint32_t reserved;
    uint64_t n_tail;         /* #{|g| > g_min}            (g_min > 0 only, else 0)      */
    double   sum_log_tail;   /* sum of ln(|g|/g_min) over them (g_min > 0 only)         */
} tq_stats_t;

/* Per-bucket quantizer parameters (160 bytes): what a worker sends beside its codes. */
typedef struct {
    float    alpha;          /* truncation threshold, > 0                               */
    uint32_t bits, s, grid;  /* b, s = 2^b - 1, TQ_GRID_*                               */
    float    level[16];      /* l_0 = -alpha < ... < l_s = +alpha; rest 0               */
    float    inv_w[16];      /* (float)(1/(l_{k+1}-l_k)), 0 for an empty cell; uniform
                                grid: every entry (float)(s/(2 alpha))                  */
    float    gamma_hat, rho_hat, g_min; /* estimates the design used (0 if none)        */
    uint32_t flags;          /* TQ_F_*                                                  */
} tq_params_t;

/* Number of buckets, and bytes of one worker's packed payload: the b-bit codes
 * form one little-endian bit stream (element e at bits [e*b, e*b+b)), padded
 * with zero bits to a multiple of 16 bytes.  Pure host arithmetic. */
uint64_t tq_num_buckets(uint64_t d, uint64_t bucket_elems);
uint64_t tq_payload_bytes(uint64_t d, int bits);

/*
 * tq_stats -- the reductions the parameter design consumes (Sec. IV-A: tail
 * mass rho and Q_U(alpha); Sec. IV-B: integral of p^(1/3); Sec. V: the two
 * terms of the maximum-likelihood tail index gamma = 1 + n/sum ln(g_j/g_min)).
 *   g_dev      [d] gradient, TQ_F32 (float) or TQ_BF16 (uint16 bit patterns); a bucket
 *              holds fewer than 2^32 elements (32-bit counts), else TQ_EUNSUPPORTED
 *   g_min      > 0: also count and log-sum the elements with |g| > g_min
 *              (must be >= 2^-40); <= 0: leave the tail to tq_params
 *   stats_dev  [tq_num_buckets] written in full; deterministic
 *   workspace_dev, workspace_bytes
 *              caller-owned device scratch of at least
 *              tq_stats_workspace_bytes(d, bucket_elems) bytes (partial
 *              histograms of the workgroups); need not be cleared, contents
 *              undefined afterwards; calls sharing one workspace must be
 *              ordered on one stream
 */
uint64_t tq_stats_workspace_bytes(uint64_t d, uint64_t bucket_elems);
int tq_stats(const void* g_dev, int dtype, uint64_t d, uint64_t bucket_elems,
             float g_min, tq_stats_t* stats_dev, void* workspace_dev,
             uint64_t workspace_bytes, void* stream);

/*
 * tq_stats_static -- tq_stats for callers that cannot allocate device memory (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): the partial
 * histograms go to a scratch array of TQ_STATS_STATIC_SCRATCH_BYTES bytes that the library
 * itself holds on every device it runs on, in place of the caller's workspace.  The call
 * allocates and frees nothing.  Arguments and result as tq_stats; g_dev and stats_dev are
 * still the caller's.
 *   - TQ_EUNSUPPORTED when tq_stats_workspace_bytes(d, bucket_elems) exceeds the scratch
 *     array (more than about 1200 buckets)
 *   - every call on a device shares that device's array: calls that may overlap in time
 *     on one device (different streams, no ordering between them) race and give wrong
 *     statistics; order them, or use tq_stats with separate workspaces.  Nothing has to
 *     be cleared between calls: every row that is read has been written by the same call.
 *   - the device of the call is the current device (hipSetDevice); the first call on a
 *     device looks the array's address up
 */
#define TQ_STATS_STATIC_SCRATCH_BYTES (8u << 20)
int tq_stats_static(const void* g_dev, int dtype, uint64_t d, uint64_t bucket_elems,
                    float g_min, tq_stats_t* stats_dev, void* stream);

/*
 * tq_params -- the two parameters of the quantizer, per bucket (Sec. IV):
 * truncation threshold alpha by the fixed point of the boxed equation of
 * Sec. IV-A (uniform grid, Q_U) or Sec. IV-B (non-uniform grid, Q_N), and the
 * codebook: l_k = -alpha + k 2alpha/s, or the levels at which the integral of
 * lambda_s ~ p^(1/3) (Sec. IV-B, first boxed equation) reaches k.  TQ_GRID_BISCALED is
 * the truncated BiScaled quantizer of the appendix: alpha from the same boxed form with
 * Q_B(alpha, k*), k* = argmin_k Q_B searched over k = 0 and the histogram's bin edges
 * below alpha, s_beta (odd, nearest to the appendix's formula) uniform cells on
 * [-k* alpha, k* alpha] and s - s_beta on the rest; tq_compress and the server calls treat
 * it like any non-uniform codebook.  p inside
 * [-alpha, alpha] is the histogram's density; gamma, rho come from the tail
 * terms of tq_stats or, without g_min, from the bins above the 0.9-quantile.
 *   stats_dev       [nb] from tq_stats
 *   bits            b in {2,3,4}
 *   alpha_override  0: the paper's formula; > 0: use this alpha;
 *                   < 0: alpha = max|g| (quantization without truncation)
 *   params_dev      [nb] written in full
 * All arithmetic is fp64 on the device, one workgroup per bucket.
 */
int tq_params(const tq_stats_t* stats_dev, uint64_t nb, int bits, int grid,
              float alpha_override, tq_params_t* params_dev, void* stream);

/*
 * tq_compress -- Alg. 1 client step: code[e] = Q[T_alpha(g[e])] (Eq. 1, Eq. 2)
 * on the bucket's codebook, packed to b bits.  The rounding of element e uses
 * 16 bits of Philox4x32-10 with counter (e >> 3, worker, step) and key `seed`,
 * so the payload is a pure function of (g, params, seed, worker, step).
 *   g_dev        [d] gradient (dtype as in tq_stats)
 *   params_dev   [tq_num_buckets]; all records must carry the same bits
 *                (read on the device: a mismatch cannot be reported)
 *   bits         b in {2,3,4}, the bits of params_dev
 *   grid         the codebook family of params_dev as it was given to tq_params (TQ_GRID_*).
 *                It chooses the shape of the launch and nothing else: the records live on
 *                the device, and the two families run fastest with different numbers of
 *                tiles per workgroup.  Every bucket is encoded as ITS record says, so the
 *                payload is the same whatever is passed here; a wrong value costs about a
 *                tenth of the speed.
 *   payload_dev  [tq_payload_bytes(d, bits)] written in full, padding included
 */
int tq_compress(const void* g_dev, int dtype, uint64_t d, uint64_t bucket_elems,
                const tq_params_t* params_dev, int bits, int grid, uint64_t seed,
                uint32_t worker, uint32_t step, void* payload_dev, void* stream);

/*
 * Batched forms for `count` tensors of the same shape (d, dtype, bucket_elems, bits) in one
 * launch each: the N simulated workers of one GPU, or several equal-sized tensors of one
 * worker.  The *_host arguments are host arrays of `count` device pointers, each with the
 * meaning of the single-tensor call; tensor i of tq_compress_multi is worker
 * first_worker + i.  tq_stats_multi needs count * tq_stats_workspace_bytes(d, bucket_elems)
 * bytes of workspace.  count = 1 .. TQ_MAX_WORKERS.  Results are identical to `count`
 * single-tensor calls.
 */
int tq_stats_multi(const void* const* g_host, int count, int dtype, uint64_t d,
                   uint64_t bucket_elems, float g_min, tq_stats_t* const* stats_host,
                   void* workspace_dev, uint64_t workspace_bytes, void* stream);
int tq_params_multi(const tq_stats_t* const* stats_host, int count, uint64_t nb, int bits,
                    int grid, float alpha_override, tq_params_t* const* params_host,
                    void* stream);
int tq_compress_multi(const void* const* g_host, int count, int dtype, uint64_t d,
                      uint64_t bucket_elems, const tq_params_t* const* params_host, int bits,
                      int grid, uint64_t seed, uint32_t first_worker, uint32_t step,
                      void* const* payload_host, void* stream);

/*
 * tq_decompress_aggregate -- Alg. 1 server step: out[e] = sum_i w_i L_i[c_i(e)]
 * over the N workers' payloads in one pass, in binary32, in worker order.
 *   payload_host  [N] host array of device pointers to the payloads
 *   params_host   [N] host array of device pointers to each worker's
 *                 [tq_num_buckets] parameter records
 *   weights_host  NULL: w_i = 1/N, applied once to the sum (Lemma 2);
 *                 else [N] floats, each level is scaled before it is added
 *   N             1 .. TQ_MAX_WORKERS
 *   accumulate    0: out = result; 1: out += result
 *   out_dev       [d] floats
 */
int tq_decompress_aggregate(const void* const* payload_host,
                            const tq_params_t* const* params_host,
                            const float* weights_host, int N, uint64_t d,
                            uint64_t bucket_elems, int bits, int accumulate,
                            float* out_dev, void* stream);

/*
 * tq_decompress_aggregate_update -- both server steps of Alg. 1 in one pass: the aggregate
 * g_bar of tq_decompress_aggregate is not written out but applied to the model,
 *     theta <- theta - eta * g_bar                       (Alg. 1, last server step),
 * with the momentum and weight decay of the momentum SGD the experiments of Sec. V train with
 * (the paper does not write that recursion out; the common form is taken):
 *     u = g_bar + weight_decay * theta      (u = g_bar when weight_decay == 0)
 *     v = momentum * v + u                  (only with a velocity buffer)
 *     theta = theta - eta * v               (theta - eta * u without one)
 * each product and sum rounded once to binary32, in this order.
 *   payload_host, params_host, weights_host, N, d, bucket_elems, bits
 *                 as in tq_decompress_aggregate
 *   theta_dev     [d] floats, updated in place
 *   velocity_dev  [d] floats, updated in place, or NULL for plain SGD (momentum is
 *                 then ignored); must not alias theta_dev
 * Saves the 4 + 4 bytes per element of writing g_bar and reading it back.
 */
int tq_decompress_aggregate_update(const void* const* payload_host,
                                   const tq_params_t* const* params_host,
                                   const float* weights_host, int N, uint64_t d,
                                   uint64_t bucket_elems, int bits, float eta,
                                   float momentum, float weight_decay, float* theta_dev,
                                   float* velocity_dev, void* stream);

/*
 * tq_quantize_dequantize -- out[e] = Q[T_alpha(g[e])] (Eq. 1, Eq. 2) as float values: what the
 * server reconstructs from this worker's message, computed without producing the message.
 * Same draws and arithmetic as tq_compress, so the result equals, bit for bit, what
 * tq_decompress_aggregate returns for N = 1 from tq_compress's payload.  For studies of
 * training under quantization (the experiments of Sec. V) that do not need the wire format.
 *   arguments as in tq_compress; accumulate 0: out = value, 1: out += value
 *   out_dev   [d] floats
 */
int tq_quantize_dequantize(const void* g_dev, int dtype, uint64_t d, uint64_t bucket_elems,
                           const tq_params_t* params_dev, int bits, uint64_t seed,
                           uint32_t worker, uint32_t step, int accumulate, float* out_dev,
                           void* stream);

/*
 * Variable-size segments -- Sec. V quantizes the layers of a network independently: the flat
 * gradient is cut into nseg consecutive segments of any sizes, each with its own statistics
 * record and its own (alpha, codebook), in one launch per step instead of one call per layer.
 * tq_params is used as it is, with nb = nseg.  Payload, random draws and aggregate are those of
 * the bucketed calls: only the record an element is encoded with changes.
 *   seg_offsets_dev   [nseg + 1] device array (8-byte aligned): 0 = off[0] < off[1] < ... <
 *                     off[nseg] = d, every interior offset a multiple of 128
 *   seg_offsets_host  the same table in host memory, or NULL.  When given it is checked
 *                     before anything is enqueued (TQ_EINVAL if malformed); keeping the two
 *                     copies equal is the caller's business.  The kernels bound every access
 *                     by d and nseg themselves, so a malformed device table gives wrong
 *                     results, never an access outside the caller's buffers.
 *   stats_dev / params_dev  [nseg] records
 *   workspace_dev     tq_stats_segments_workspace_bytes(d, nseg) bytes, rules as for tq_stats
 * tq_compress_segments takes no `grid`: it has one launch shape.  The segment kernels favour
 * generality over the last tenth of speed (one tile per workgroup, plain level tables).
 * tq_stats_segments needs d < 2^32 (the counts of a record are 32-bit).
 * The *_multi forms take `count` tensors of the same d and dtype that share ONE segment table
 * (the N workers' gradients of one model) in one launch each, as tq_stats_multi and
 * tq_compress_multi do for buckets: host arrays of `count` device pointers, tensor i of
 * tq_compress_segments_multi is worker first_worker + i, the workspace is count *
 * tq_stats_segments_workspace_bytes(d, nseg) bytes, results are identical to `count` single calls.
 */
uint64_t tq_stats_segments_workspace_bytes(uint64_t d, uint64_t nseg);
int tq_stats_segments(const void* g_dev, int dtype, uint64_t d, const uint64_t* seg_offsets_dev,
                      const uint64_t* seg_offsets_host, uint64_t nseg, float g_min,
                      tq_stats_t* stats_dev, void* workspace_dev, uint64_t workspace_bytes,
                      void* stream);
int tq_compress_segments(const void* g_dev, int dtype, uint64_t d, const uint64_t* seg_offsets_dev,
                         const uint64_t* seg_offsets_host, uint64_t nseg,
                         const tq_params_t* params_dev, int bits, uint64_t seed, uint32_t worker,
                         uint32_t step, void* payload_dev, void* stream);
int tq_stats_segments_multi(const void* const* g_host, int count, int dtype, uint64_t d,
                            const uint64_t* seg_offsets_dev, const uint64_t* seg_offsets_host,
                            uint64_t nseg, float g_min, tq_stats_t* const* stats_host,
                            void* workspace_dev, uint64_t workspace_bytes, void* stream);
int tq_compress_segments_multi(const void* const* g_host, int count, int dtype, uint64_t d,
                               const uint64_t* seg_offsets_dev, const uint64_t* seg_offsets_host,
                               uint64_t nseg, const tq_params_t* const* params_host, int bits,
                               uint64_t seed, uint32_t first_worker, uint32_t step,
                               void* const* payload_host, void* stream);
int tq_decompress_aggregate_segments(const void* const* payload_host,
                                     const tq_params_t* const* params_host,
                                     const float* weights_host, int N, uint64_t d,
                                     const uint64_t* seg_offsets_dev,
                                     const uint64_t* seg_offsets_host, uint64_t nseg, int bits,
                                     int accumulate, float* out_dev, void* stream);

/* Text for a return code (static storage). */
const char* tq_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* TQ_H */
