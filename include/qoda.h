/*
 * qoda.h -- C ABI of the MI355X (gfx950) hot path of Quantized Optimistic Dual Averaging with layer-wise
 * unbiased stochastic quantization (arXiv 2505.14371).
 *
 * One context describes one model: L layers (tensors) of d_l fp32 entries, M types of level sequences, K nodes.
 * The K nodes are K sets of buffers on one GPU; "broadcast / receive" (Alg. 1 lines 13-14) is the caller handing
 * the K message buffers back to the library.
 *
 * Conventions
 *   - Pointers named *_dev are DEVICE pointers owned by the caller; arrays of such pointers are HOST arrays
 *     (the library copies them).  Everything else is host memory.  Every fp32 layer pointer must be 16-byte
 *     aligned; message buffers must be 256-byte aligned and hold qoda_message_bytes() bytes.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work is enqueued on it; no call
 *     waits for the device except qoda_get_levels, qoda_read_buffer and qoda_status, which say so.
 *   - Every call returns QODA_OK (0) or a negative error code and then qoda_last_error() describes it.  Nothing
 *     throws across this boundary.  Bad arguments are rejected before anything is launched.
 *   - A context is not thread-safe: use it from one host thread at a time, on one stream at a time.  It belongs to
 *     the device that was current in qoda_create; a call made with another device current returns QODA_EINVAL.
 *   - Host arrays (pointer tables, levels) are consumed before a call returns: they reach the device as kernel
 *     arguments, so no call copies from host memory later or waits for an earlier upload.  The library keeps a few
 *     device copies of every K-wide pointer array it is given and recognises a set it has seen; the calls of a round
 *     enqueue kernels (and, for the statistics-based fit, one device-to-device copy) only.  Such a round can be
 *     captured into a HIP graph; pointers and the round number are then fixed in the captured launches.  The calls
 *     that wait (see above) cannot be captured.
 *   - Non-finite input (a vector -- layer, whole dual vector or bucket, by scope -- whose sum of squares is not a
 *     finite number or whose norm exceeds FLT_MAX) sets a sticky device-side flag reported by qoda_status(); that
 *     vector's output is then unspecified (but in bounds).  A second flag marks a vector whose norm is positive but
 *     below 2^-126 (the smallest normal float): 1/norm is then not a float, the normalised magnitudes fall short of
 *     |v| / norm and the quantizer of that vector is biased -- the one case in which E[Q(v)] = v (Thm 5.1) does not
 *     hold to rounding.
 *
 * Level sequences (Sec. 3.1): type m has S_m grid points 0 = l_0 < l_1 < ... < l_{S_m-1} = 1, i.e. the paper's
 * alpha_m = S_m - 2 interior levels.  A coordinate's code is one sign bit plus a ceil(log2 S_m)-bit level index.
 *
 * Message format (ENCODE / DECODE of Sec. 3.2 and App. C.1, fixed width, no entropy code):
 *   header   for each layer, in order: fp32 norm (the paper's C_q = 32 bits), then its S fp32 level values
 *            (so that a stored previous-round message stays decodable after the levels change); padded to 256 B;
 *   body     for each layer, ceil(d_l/2048) octets of 2048 coordinates, 256*(1+b) bytes each.  A coordinate's
 *            code is sign | index << 1 (1+b bits).  Inside an octet, "lane" i = (e mod 256)/4 owns the 32
 *            coordinates 256*bb + 4*i + j (bb = 0..7, j = 0..3), numbered jj = 4*bb + j; their codes form a
 *            little-endian bit string (code jj at bit (1+b)*jj), i.e. 1+b 32-bit words; word r of lane i is the
 *            32-bit word r*64 + i of the octet.  Padding coordinates carry code 0.
 */
#ifndef QODA_H_
#define QODA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define QODA_OK 0
#define QODA_EINVAL (-1)    /* bad argument (null, misaligned, out of range, levels not increasing, ...) */
#define QODA_ENOMEM (-2)    /* device or host allocation failed */
#define QODA_EHIP (-3)      /* a HIP runtime call failed; see qoda_last_error() */
#define QODA_ENONFINITE (-4) /* returned by qoda_status(): some vector's norm statistic was not a finite number */
#define QODA_ETINYNORM (-5)  /* returned by qoda_status(): some vector's norm was positive but below 2^-126 */

#define QODA_MAX_POINTS 256 /* S_m <= 256: level index fits 8 bits */

/* What one norm covers (Sec. 2.2 normalises "the vector"; Sec. 3 quantizes layer by layer; the experiments of
 * Sec. 7 normalise buckets of 128 entries).
 *   LAYER   one norm per layer (the default of this library);
 *   VECTOR  one norm for the node's whole dual vector: the L layer sums of squares are combined and every layer
 *           uses that norm (each layer's header carries it); message format as under LAYER;
 *   BUCKET  one norm per 128 consecutive coordinates of a layer, computed in the same pass that quantizes (the
 *           gradient is read once).  The 256*(1+b) code bytes of every octet are followed by the octet's 16 bucket
 *           norms (fp32; the bucket of block bb = 0..7, half hf = 0..1 of the octet at position 8*hf + bb), so an
 *           octet takes 256*(1+b) + 64 bytes; the header's norm entry is 0 and unused.  A bucket's sum of squares is
 *           accumulated in single precision inside a lane (relative error below 3e-7); when that result is below 2^-100
 *           or not finite -- squares may have vanished or overflowed -- the bucket is summed again with exact fp64
 *           squares, so buckets of very small or very large entries are normalised as exactly as layers are. */
#define QODA_SCOPE_LAYER 0
#define QODA_SCOPE_VECTOR 1
#define QODA_SCOPE_BUCKET 2

/* The q of the L^q normalisation u_i = |v_i| / ||v||_q (Sec. 2.2; Thm 5.1 holds for every q, with d^(1/min(q,2))):
 *   L2    norm = largest float whose square does not exceed the fp64 sum of squares (the default of the paper's
 *         experiments and of this library's workloads);
 *   L1    norm = the fp64 sum of magnitudes (same fixed summation order) rounded once to fp32;
 *   LINF  norm = the largest magnitude (the limit q -> infinity), exact.
 * A vector weighs ||v||_q^2 in the level fit (eq. (Qada2)).  Under bucket scope the sums run in single precision
 * inside a lane, as for L2.  The step-size terms are Euclidean whatever q is. */
#define QODA_NORM_LINF 0
#define QODA_NORM_L1 1
#define QODA_NORM_L2 2

typedef struct qoda_ctx qoda_ctx;

typedef struct {
  int32_t num_layers;         /* L >= 1 */
  const int64_t *layer_size;  /* d_l >= 0 elements, host array [L], copied; d_l < 2^34, and at most 2^28 tiles of
                                 16384 elements over all layers (each layer rounded up to whole tiles) */
  const int32_t *layer_type;  /* m(l) in [0, M), host array [L], copied */
  int32_t num_types;          /* M >= 1 */
  const int32_t *type_points; /* S_m in [2, 256], host array [M], copied */
  int32_t num_nodes;          /* K >= 1, K <= 65535, and K * 2^(1+b_max) <= 16384 with b_max = ceil(log2 max_m S_m)
                                 (the decode tables of all K nodes are kept in shared memory), else QODA_EINVAL;
                                 qoda_step_alt needs K * 2^(1+b_max) <= 15872 */
  int32_t norm_kind;          /* QODA_NORM_*: the q of the L^q normalisation */
  uint64_t seed;              /* key of the counter-based generator */
  int32_t norm_scope;         /* QODA_SCOPE_*: what one norm covers */
} qoda_config;

/* Create / destroy.  qoda_create allocates all device scratch (a few MB plus 8 bytes per 16384 coordinates per
 * node; the fit's histogram, 8 KB per (node, layer), is allocated on the first qoda_fit_levels, under bucket scope
 * at once).  Levels start
 * uniform: l_j = j/(S-1).  On failure *out is NULL. */
int qoda_create(const qoda_config *cfg, qoda_ctx **out);
int qoda_destroy(qoda_ctx *ctx);

/* Packed bytes of one node's message (header + body, multiple of 256). */
size_t qoda_message_bytes(const qoda_ctx *ctx);
/* Byte offsets of each layer's header entry and body inside a message (host arrays [L], either may be NULL). */
int qoda_message_layout(const qoda_ctx *ctx, int64_t *hdr_off, int64_t *body_off);

/* Set / get the S_m levels of one type (Sec. 3.1).  set: levels_host[0] == 0, levels_host[S-1] == 1, strictly
 * increasing, else QODA_EINVAL; enqueues the upload and the rebuild of the search tables.  get: waits for `stream`. */
int qoda_set_levels(qoda_ctx *ctx, int32_t type, const float *levels_host, void *stream);
int qoda_get_levels(qoda_ctx *ctx, int32_t type, float *levels_host, void *stream);

/* Level fit, Alg. 1 lines 2-7 / eq. (Qada2) with the weights lambda_z: the K nodes' current vectors are the Z
 * samples; every coordinate of (node, layer) weighs ||v_{k,l}||^2; layers of one type pool.  The distribution is
 * estimated by a histogram of every entry on its top 11 magnitude bits and the objective is minimised exactly
 * over level positions on a 257-point grid (3 mantissa bits per octave down to 2^-32).  A type whose vectors are
 * all zero keeps its levels.  grad_dev: host array [K*L], entry k*L+l.  Alg. 1 places the update before the round's
 * vectors exist, so the vectors given here are normally the previous round's; the quantize calls that follow compute
 * their own norms from whatever they are given (see qoda_fit_levels_keep_norms for the other case).
 * Bucket scope: every bucket is a vector of its own (weight = its sum of squares, normalisation = its norm); with
 * grad_dev the fit takes two passes over these vectors (scale of the weights, then the weighted grid histogram).  With grad_dev == NULL (bucket scope only) it reads nothing: it uses the statistics that the last
 * quantize pass of every node gathered while it quantized -- Alg. 1 runs lines 3-5 before the round's vectors exist,
 * so the estimate comes from the previous round's vectors -- and hands the next pass its weight scale (exponent of the
 * largest bucket sum per type; weights are floor(sum * 2^(23 - exponent)) capped at 2^30).  A pass gathers a
 * histogram only once some fit has produced a scale: call the fit with vectors once (or with NULL twice, the first of
 * which only sets the scale), then with NULL at every later update step. */
int qoda_fit_levels(qoda_ctx *ctx, const float *const *grad_dev, uint32_t round, void *stream);

/* Bucket scope only (no effect otherwise): whether the quantize passes that follow gather the histogram for the next
 * statistics-based fit (default: yes).  Gathering costs the quantize pass 11-13 %; a caller who updates the levels
 * every few thousand rounds, as the paper's experiments do, switches it on for the round before an update step only.
 * A pass that does not gather still records the largest bucket sum per (node, layer), from which the next
 * qoda_fit_levels(NULL) derives the weight scale; its pooled histogram is empty then and the levels stay. */
int qoda_gather_statistics(qoda_ctx *ctx, int32_t enable);

/* The same fit for a caller who fits on the round's own vectors (layer and vector scope; under bucket scope identical
 * to qoda_fit_levels).  Calling it DECLARES that grad_dev holds exactly what the qoda_quantize / qoda_quantize_all
 * calls of the same `round` will be given, unchanged: the norms computed here on the way stay in the context, and such
 * a call with the same `round` and the same pointers skips its norm pass (one read of the vectors less per round).
 * A caller who rewrites the buffers in between gets messages scaled by stale norms; the library cannot see that.
 * Anything else -- another round number, other pointers, any other fit call -- drops the kept norms.
 * grad_dev must not be NULL. */
int qoda_fit_levels_keep_norms(qoda_ctx *ctx, const float *const *grad_dev, uint32_t round, void *stream);

/* ENCODE(Q(V_{k,t+1/2})), Alg. 1 line 12 (Sec. 2.2, 3.1, 3.2): per-layer L2 norm, u = min(|v| / ||v||, 1), level
 * search, stochastic rounding with one 16-bit counter-based draw per coordinate (counter = coordinate, layer,
 * round, node), sign + index codes shifted into per-lane records.  Also leaves delta_k = ||Vhat_{k,t+1/2} - Vhat_{k,t-1/2}||^2 in the
 * context for the step size (eq. (general_stepsize)); msg_prev_dev == NULL means Vhat_{k,t-1/2} = 0 (round 1).
 * grad_dev: host array [L] (node k's layers).  msg_dev / msg_prev_dev must not overlap. */
int qoda_quantize(qoda_ctx *ctx, int32_t node, const float *const *grad_dev, uint32_t round, void *msg_dev,
                  const void *msg_prev_dev, void *stream);
/* The same for all K nodes in one set of launches.  grad_dev: host [K*L]; msg_dev: host [K];
 * msg_prev_dev: host [K] or NULL (all previous messages zero). */
int qoda_quantize_all(qoda_ctx *ctx, const float *const *grad_dev, uint32_t round, void *const *msg_dev,
                      const void *const *msg_prev_dev, void *stream);

/* qoda_quantize for callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same message bytes and the same delta_k left in the context as qoda_quantize,
 * but nothing is allocated, uploaded or waited for: the kernels' scratch (one node's per-tile partial sums, per-layer
 * statistics, norms, reciprocals and pointer tables) lives in a static device array of about 2.1 MiB that every GPU
 * the library runs on holds until the process ends, and the pointers travel as kernel arguments.  The norms are always
 * computed from grad_dev (no reuse of a fit's norms), launches are never timed by qoda_profile_enable, and under
 * bucket scope the node's fit statistics still go to the context.  Limits: L <= 4096 layers and at most 131072 tiles
 * of 16384 coordinates per node (2^31 coordinates), else QODA_EINVAL.  All calls on one GPU share the one array, which
 * keeps the last call's contents (every entry a call reads it has written first, so nothing needs clearing): calls
 * whose work overlaps on one GPU -- two streams, two contexts, two threads -- race; order them on one stream. */
int qoda_quantize_noalloc(qoda_ctx *ctx, int32_t node, const float *const *grad_dev, uint32_t round, void *msg_dev,
                          const void *msg_prev_dev, void *stream);

/* DECODE + mean, Alg. 1 lines 15-17 without the update: mean_out[l][e] = (Vhat_0 + ... + Vhat_{K-1}) / K with
 * Vhat_k = +-norm_k * l_h, summed in fp32 in increasing k.  msgs_dev: host [K]; mean_out_dev: host [L]. */
int qoda_dequant_aggregate(qoda_ctx *ctx, const void *const *msgs_dev, float *const *mean_out_dev, void *stream);

/* Solver state of Alg. 1 (all caller-owned device memory): X_1 (read only), Y_t (in/out, Y_1 = 0), the next
 * query point X_{t+3/2} (out), optionally X_{t+1} (out), the step-size accumulator (in/out, starts at 0) and
 * optionally the two step sizes (out: eta_{t+1}, gamma_{t+1}).  Pointer arrays are host arrays [L]. */
typedef struct {
  const float *const *x1_dev;
  float *const *y_dev;
  float *const *x_half_dev;
  float *const *x_next_dev; /* may be NULL */
  double *acc_dev;          /* device double: sum_{s<=t} sum_k delta_{k,s} / K^2 */
  float *eta_dev;           /* device float[2] or NULL */
} qoda_state;

/* One fused pass, Alg. 1 lines 15-18 and line 10 of the next round (eq. (ODA), eq. (general_stepsize)):
 *   acc += (sum_k delta_k) / K^2 with the delta_k left by the K preceding quantize calls;
 *   eta_{t+1} = gamma_{t+1} = (1 + acc)^(-1/2);
 *   mean = (1/K) sum_k DECODE(msgs[k]);  Y <- Y - mean;  X_{t+1} = X_1 + eta_{t+1} Y;
 *   X_{t+3/2} = X_{t+1} - gamma_{t+1} mean.
 * msgs_dev: host [K]. */
int qoda_step(qoda_ctx *ctx, const void *const *msgs_dev, const qoda_state *state, void *stream);

/* The same fused pass with the caller's own schedule: Alg. 1 takes the learning rates {eta_t}, {gamma_t} as inputs
 * (Sec. 4: any non-increasing pair with gamma_t >= eta_t > 0); eq. (general_stepsize) and eq. (Alt) are the paper's
 * two proposals.  rates_dev: device float[2] = {eta_{t+1}, gamma_{t+1}}, read by the kernel when it runs.
 * state->acc_dev and state->eta_dev are not used; nothing is accumulated. */
int qoda_step_rates(qoda_ctx *ctx, const void *const *msgs_dev, const qoda_state *state, const float *rates_dev,
                    void *stream);

/* Solver state under the alternative pair of step sizes, Sec. 6 eq. (Alt) (all caller-owned device memory).
 * sums_dev: device double[2] = {lambda, mu}, both starting at 0:
 *   lambda = sum over finished rounds s of sum_k ||Vhat_{k,s+1/2}||^2 / K^2,  mu = sum_s ||X_s - X_{s+1}||^2.
 * eta_dev: device float[2], required, in/out: on entry [0] holds eta_t, the rate that produced X_t (start: 1); on
 * exit {eta_{t+1}, gamma_{t+1}}.  The other fields are those of qoda_state. */
typedef struct {
  const float *const *x1_dev;
  float *const *y_dev;
  float *const *x_half_dev;
  float *const *x_next_dev; /* may be NULL */
  double *sums_dev;
  float *eta_dev;
} qoda_alt_state;

/* qoda_step with the rates of eq. (Alt), which use sums over the rounds BEFORE this one only (two-round lag):
 *   eta_{t+1} = (1 + lambda + mu)^(-1/2),  gamma_{t+1} = (1 + lambda)^(q_hat - 1/2),  0 < q_hat <= 1/4;
 *   mean, Y, X_{t+1}, X_{t+3/2} as in qoda_step with these two rates;
 *   then lambda += (sum_k delta_k) / K^2 and mu += ||X_t - X_{t+1}||^2, X_t = X_1 + eta_t Y_t rebuilt from the state.
 * delta_k must be ||Vhat_{k,t+1/2}||^2: run this round's quantize calls with msg_prev_dev = NULL.
 * q_hat is used to 32 binary digits; the power is built from square roots (no library pow), so the rates are
 * reproducible bit for bit.  Of the two forms the paper prints for lambda (sum of the K squared norms in the main
 * text and in the appendix's choice of rates; squared norm of the sum in the appendix's lemma notation) the first is
 * taken.  Errors: QODA_EINVAL for q_hat outside (0, 1/4] or below 2^-32, null sums_dev or eta_dev, or
 * K * 2^(1+b_max) > 15872 (this pass keeps a reduction buffer in shared memory beside the decode tables). */
int qoda_step_alt(qoda_ctx *ctx, const void *const *msgs_dev, const qoda_alt_state *state, double q_hat, void *stream);

/* DECODE + mean + one plain step: out[l][e] = x[l][e] - gamma * mean[l][e] (two fp32 operations), mean as in
 * qoda_dequant_aggregate.  This is the leg that an extra-gradient method (the two-call scheme QODA is compared with in
 * Sec. 4: X_{t+1/2} = X_t - gamma * mean of the vectors at X_t, then X_{t+1} = X_t - gamma * mean of the vectors at
 * X_{t+1/2}) runs twice per round, each with its own quantize + exchange; the library offers it so that this baseline
 * runs on the same kernels.  x_dev, out_dev: host [L] (may alias each other layer by layer); gamma_dev: device float. */
int qoda_extrapolate(qoda_ctx *ctx, const void *const *msgs_dev, const float *const *x_dev, float *const *out_dev,
                     const float *gamma_dev, void *stream);

/* Code-length accounting (Thm 5.3 and its proof in App. C.1; Huffman coding, App. C.3).  The library transmits
 * fixed-width codes; these two calls report what an entropy code on top would save.
 * qoda_index_counts: occurrences of every level index among the real coordinates of the K messages, per type:
 *   counts[m*256 + h] (host array of M*256 entries, overwritten); waits for `stream`.  msgs_dev: host [K].
 * qoda_code_length (host arithmetic only): bit counts for the coordinates behind `counts`, gathered from
 *   `num_messages` messages, with p_j = c_j / n_m the empirical occurrence probabilities of type m:
 *     fixed_bits    32 per norm + (1 + ceil(log2 S_m)) per coordinate (this library's format without level tables
 *                   and padding; norms per message: one per non-empty layer, one in all under vector scope, one per
 *                   bucket under bucket scope);
 *     paper_bits    the expression in the proof of Thm 5.3: C_q + sum_m (1 - p_0) n_m + sum_m (H(l^m) + 1) n_m with
 *                   H(l^m) = -sum_{j=1}^{alpha_m} p_j log2 p_j over the interior levels, as printed;
 *     entropy_bits  32 per norm + one sign bit per non-zero entry + sum_m n_m * (-sum_j p_j log2 p_j), all indices;
 *     huffman_bits  32 per norm + one sign bit per non-zero entry + the total length of a Huffman code per type;
 *     nonzeros      entries with index > 0 (lemma on the expected number of non-zeros, App. C.1);
 *     coordinates   sum_m n_m;   message_bits  8 * qoda_message_bytes() * num_messages. */
typedef struct {
  double fixed_bits, paper_bits, entropy_bits, huffman_bits, nonzeros, coordinates, message_bits;
} qoda_code_length_report;
int qoda_index_counts(qoda_ctx *ctx, const void *const *msgs_dev, uint64_t *counts, void *stream);
int qoda_code_length(qoda_ctx *ctx, const uint64_t *counts, uint32_t num_messages, qoda_code_length_report *out);

/* Read an internal device buffer into host memory (waits for `stream`); for tests and diagnostics. */
#define QODA_BUF_SUMSQ 0  /* double[K*L]  per-layer statistic of the last norm pass (sum of squares; L1: sum of
                              magnitudes; LINF: largest magnitude); bucket scope: largest bucket's */
#define QODA_BUF_NORM 1   /* float [K*L]  norms                                                            */
#define QODA_BUF_INV 2    /* float [K*L]  reciprocal norms                                                 */
#define QODA_BUF_DELTA 3  /* double[K]    delta_k of the last quantize of each node                        */
#define QODA_BUF_HIST 4   /* uint32[K*L*2048] histogram of the last fit                                    */
#define QODA_BUF_POOLED 5 /* uint64[M*257] pooled grid weights of the last fit                             */
int qoda_read_buffer(qoda_ctx *ctx, int32_t which, void *dst_host, size_t bytes, void *stream);

/* Waits for `stream`; returns QODA_OK, or QODA_ENONFINITE if a non-finite vector was seen since the last call, or
 * QODA_ETINYNORM if only vectors with a norm below 2^-126 were (both flags are cleared). */
int qoda_status(qoda_ctx *ctx, void *stream);

/* Measurement aids (no part of the method).
 * qoda_profile_enable: launches of the kernel classes whose bit is set in class_mask (bit i = class i, see
 *   qoda_kernel_name; 0 = off, 0xFFFFFFFF = all) are bracketed by two HIP events on the launch stream.  Each timed
 *   launch costs a few microseconds of idle time around it.
 * qoda_profile_read: waits for `stream`, then returns, per kernel class, the summed elapsed milliseconds and the
 *   number of launches since the last read (host arrays of QODA_NUM_KERNELS entries) and resets both.
 * qoda_kernel_name: the kernel's name for a class index (as it appears in a profiler's kernel trace), "" if out
 *   of range.
 * qoda_copy_calibration: a plain 128-bit copy kernel of `bytes` bytes (multiple of 16; 16-byte aligned device
 *   pointers): the known-traffic kernel that hardware byte counters are scaled by.
 * qoda_stream_calibration: streaming with the access type of the big kernels (nontemporal 128-bit loads and stores,
 *   64 KiB tiles): reads `bytes` (multiple of 65536) from src_dev and writes bytes * stores_per_16_loads / 16 to the
 *   head of each tile of dst_dev.  0 stores: the read-only ceiling; 16: a copy; 2 and 8: about the read/write mix of
 *   the quantize pass and of the decode + update pass.  The measured ceilings that bench.py prints beside the nominal
 *   HBM peak come from this kernel. */
#define QODA_NUM_KERNELS 24
int qoda_profile_enable(qoda_ctx *ctx, uint32_t class_mask);
int qoda_profile_read(qoda_ctx *ctx, double *ms, int64_t *launches, void *stream);
const char *qoda_kernel_name(int32_t id);
int qoda_copy_calibration(qoda_ctx *ctx, const void *src_dev, void *dst_dev, size_t bytes, void *stream);
int qoda_stream_calibration(qoda_ctx *ctx, const void *src_dev, void *dst_dev, size_t bytes, int32_t stores_per_16_loads,
                            void *stream);

const char *qoda_last_error(const qoda_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* QODA_H_ */
