// Device-side data layout and launch entry points shared by the kernels and the host API of libqoda.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace qoda {

constexpr int kBlockCoords = 256;    // coordinates per packed block (one wave64 step of 128-bit loads)
constexpr int kChunkCoords = 16384;  // coordinates per workgroup tile (64 blocks) = one reduction chunk
constexpr int kSuperTile = 8;        // tiles per workgroup in the norm pass
constexpr int kTaperWorkgroups = 2048;   // workgroups of 256 threads the device holds at once (256 CUs x 8)
constexpr int kDecodeWaves = 2;       // waves (= octets) per workgroup in the decode pass: 1, 2 or 4
constexpr int kThreads = 256;        // workgroup size everywhere: 4 waves, 256 reduction slots
constexpr int kHistBins = 2048;      // top 11 magnitude bits of an fp32 value
constexpr int kGridBase = 760;       // (127 - 32) << 3
constexpr int kGridPoints = 257;     // normalised grid g_0 = 2^-32 ... g_256 = 1
constexpr int kMaxPoints = 256;
constexpr int kLutSize = 1024;       // level-search table indexed by bits(u) >> 20 (u in [0,1] -> 0..1016)
constexpr int kTypeSkip = 0x7fffffff;
constexpr int kBucketCoords = 128;   // coordinates per bucket when every bucket carries its own norm

// What one norm covers: a layer, the node's whole vector, or a bucket of 128 consecutive coordinates of a layer.
enum NormScope { kScopeLayer = 0, kScopeVector = 1, kScopeBucket = 2 };
// The q of the L^q normalisation (Sec. 2.2): 2, 1, or 0 standing for the limit q -> infinity.  Each kind reduces a
// statistic over its vector (sum of squares, sum of magnitudes, largest magnitude), derives the fp32 norm from it
// (floor root; one rounding; exact) and weighs the vector by ||v||_q^2 in the level fit.
enum NormKind { kNormLinf = 0, kNormL1 = 1, kNormL2 = 2 };

struct LayerMeta {
  long long d;         // elements
  long long body_off;  // byte offset of the layer's blocks inside a message
  long long nblk;      // ceil(d / 256)
  int hdr_off;         // byte offset of {norm, levels[S]} inside a message
  int S;               // grid points of the layer's type
  int planes;          // 1 + ceil(log2 S)
  int type;
  int first_chunk;     // index of the layer's first tile in the per-node tile list
  int nchunks;         // ceil(d / 16384)
};

// Everything a kernel needs; passed by value.
struct Dev {
  const LayerMeta *meta;
  const int2 *tiles;  // per tile: (layer, chunk inside layer)
  const int4 *stiles; // per run of up to kSuperTile tiles of one layer: (layer, first chunk inside layer, chunks, -)
  int L, G, GS, K, M; // GS = number of runs
  int scope;          // NormScope
  int kind;           // NormKind
  const int *type_points;          // [M]
  const int *empty_layers;         // indices of the layers with d = 0
  int n_empty;
  const float *const *grad;        // [K*L] layer pointers
  unsigned char *const *msg;       // [K]
  const unsigned char *const *prev;  // [K] or nullptr
  const unsigned char *const *msgs_in;  // [K] messages to decode
  double *partial;    // [K*G] per-tile statistics (sums of squares, sums of magnitudes or largest magnitudes)
  double *dpartial;   // [K*G] per-tile squared differences
  double *sumsq;      // [K*L] the statistic of (node, layer); bucket scope: its largest bucket statistic
  float *norm;        // [K*L]
  float *inv;         // [K*L]
  double *delta;      // [K]
  float *lev;         // [M*256]
  float *rgap;        // [M*256]
  unsigned char *lut;  // [M*1024] level-search table: tau at the lower edge of the bin bits(u) >> 20
  unsigned int *hist;          // [K*L*2048]
  unsigned long long *pooled;  // [M*257]
  int *type_exp;               // [M]
  short *dp_arg;               // DP back-pointers, type m at dp_arg_off[m]
  const long long *dp_arg_off; // [M]
  unsigned int *status;
  float *eta;                  // [3] eta, gamma, previous eta (the last one only under eq. (Alt))
  // step / aggregate
  const float *const *x1;
  float *const *y;
  float *const *x_half;
  float *const *x_next;  // table pointer may be nullptr
  float *const *mean_out;
  double *acc;
  float *eta_out;  // may be nullptr
  const float *gamma_in;   // extrapolate mode: device scalar
  unsigned long long *index_counts;   // [M*256] occurrences of every level index per type (code-length accounting)
  double *alt_sums;        // eq. (Alt): [2] lambda, mu (caller's)
  unsigned int q_digits;   // eq. (Alt): the exponent's first 32 binary digits
  unsigned long long seed;
  unsigned int round;
  int node0;    // first node handled by this launch
  int nnodes;   // nodes handled by this launch (grid.y)
  int row0;     // the node whose rows come first in grad, msg, prev, partial, dpartial, sumsq, norm and inv (0 when
                // these hold all K nodes; the node itself when they hold one node's rows only).  delta and the fit
                // statistics of bucket scope (hist, sumsq) are always indexed by the node.
  float invK;
  double invK2;
};

// What the decode kernel does after the K-way mean: store it, apply eq. (ODA), apply eq. (ODA) with the two
// rates of eq. (Alt) and accumulate ||X_t - X_{t+1}||^2, or take one plain step out = x - gamma * mean (the leg an
// extra-gradient method repeats twice per round, Sec. 4).
enum DecodeMode { kDecodeMean = 0, kDecodeUpdate = 1, kDecodeUpdateAlt = 2, kDecodeExtrapolate = 3 };

// Kernel classes, for the optional per-kernel event timing of the host API.
enum KernelId {
  kIdZero = 0, kIdSumsq, kIdSumsqHist, kIdNormFinalize, kIdReserved4 /* no kernel: keeps the class numbers of the others stable */, kIdQuantize, kIdDeltaFinalize, kIdStepScalars,
  kIdDecodeMean, kIdDecodeUpdate, kIdFitTypemax, kIdFitPool, kIdFitDp, kIdBuildTables, kIdCopy, kIdAltScalars,
  kIdDecodeAlt, kIdAltFinalize, kIdNormVector, kIdBucketMax, kIdBucketHist, kIdDecodeExtrapolate, kIdIndexHist, kIdStream, kNumKernelIds
};

// Launch wrappers (each checks nothing: the host API validates shapes before calling).
hipError_t launch_zero_u32(unsigned int *p, size_t n, hipStream_t s);
hipError_t launch_sumsq(const Dev &a, bool with_hist, hipStream_t s);
hipError_t launch_norm_finalize(const Dev &a, hipStream_t s);
hipError_t launch_norm_vector(const Dev &a, hipStream_t s);
hipError_t launch_quantize(const Dev &a, unsigned int planes_mask, hipStream_t s);
hipError_t launch_delta_finalize(const Dev &a, hipStream_t s);
hipError_t launch_step_scalars(const Dev &a, hipStream_t s);
hipError_t launch_decode(const Dev &a, int mode, unsigned int planes_mask, hipStream_t s);   // mode: DecodeMode
hipError_t launch_alt_scalars(const Dev &a, hipStream_t s);
hipError_t launch_index_hist(const Dev &a, unsigned int planes_mask, hipStream_t s);   // counts every code of every octet
hipError_t launch_alt_finalize(const Dev &a, hipStream_t s);
hipError_t launch_bucket_max(const Dev &a, hipStream_t s);    // bucket scope: a.sumsq must be zero
hipError_t launch_bucket_hist(const Dev &a, hipStream_t s);   // bucket scope: grid histograms, then pooling
hipError_t launch_fit_pool_b(const Dev &a, hipStream_t s);    // bucket scope: pooling of gathered grid histograms
hipError_t launch_fit_typemax(const Dev &a, hipStream_t s);
hipError_t launch_fit_pool(const Dev &a, hipStream_t s);
hipError_t launch_fit_dp(const Dev &a, hipStream_t s);
hipError_t launch_copy(const void *src, void *dst, size_t bytes, hipStream_t s);
// nontemporal streaming over whole 64 KiB tiles of `bytes`: 16 loads and `stores` (0, 1, 2, 4, 8 or 16) stores per thread
hipError_t launch_stream(const void *src, void *dst, size_t bytes, int stores, void *sink, hipStream_t s);
hipError_t launch_build_tables(const Dev &a, int type, hipStream_t s);
// Copy a small host array (32-bit words; pointers) into device memory through kernel arguments: no staging buffer, no
// copy engine, and the host array may be reused as soon as the call returns.
hipError_t launch_stage_words(void *dst_dev, const void *src_host, size_t nwords, hipStream_t s);
hipError_t launch_stage_pointers(void **dst_dev, const void *const *src_host, size_t n, hipStream_t s);

}  // namespace qoda
